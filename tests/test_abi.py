"""The C-ABI library loads without a GPU, exports what the header declares, and its host-side
argument checks return error codes before any device work.  No GPU."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def b():
    from paper_2209_01188_amd import binding, build
    if not os.path.exists(binding.LIB_PATH):
        build.build(force=False)
    return binding


def test_library_exports_every_declared_symbol(b):
    header = open(os.path.join(ROOT, "include", "petals_span.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(petals_[a-z0-9_]+)\s*\(", header))
    assert len(declared) >= 19
    L = b.lib()
    for name in declared:
        assert hasattr(L, name), name
    assert declared == set(b.EXPORTS)


def test_library_exports_every_symbol_of_the_client_header(b):
    header = open(os.path.join(ROOT, "include", "petals_client.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(petals_[a-z0-9_]+)\s*\(", header))
    assert len(declared) == 6
    L = b.lib()
    for name in declared:
        assert hasattr(L, name), name
    assert declared == set(b.CLIENT_EXPORTS)
    # host-side checks that need no GPU
    cfg = b.ClientConfig(250880, 14336, 1e-5, 4)
    assert b.petals_client_workspace_bytes(cfg) >= 4 * 14336 * 2
    with pytest.raises(b.PetalsError):
        b.petals_client_workspace_bytes(b.ClientConfig(100, 100, 1e-5, 1))     # hidden not a multiple of 64


def test_size_queries_match_the_layout_arithmetic(b):
    cfg = b.make_config(12, 14336, 112, 57344, 1)
    H = 14336
    wb = b.petals_span_weight_bytes(cfg)
    # int8 weights 12 H^2 per block dominate; scales, biases and LayerNorm add < 0.1 %
    assert 12 * 12 * H * H <= wb <= 12 * 12 * H * H * 1.001
    assert b.petals_span_kv_bytes(cfg, 2049) == 12 * 2 * H * 2049 * 2
    assert b.petals_span_workspace_bytes(cfg) > 0


@pytest.mark.parametrize("kw,code", [
    (dict(hidden=100), -3),           # not a multiple of 64
    (dict(n_heads=7), -1),            # hidden % heads
    (dict(hidden=64 * 24, n_heads=2), -3),   # head_dim 768
    (dict(ffn=131072), -3),           # int32 accumulator overflow
    (dict(n_blocks=0), -1),
    (dict(max_rows_per_call=70000), -3),
])
def test_bad_configs_are_rejected(b, kw, code):
    args = dict(n_blocks=2, hidden=64, n_heads=4, ffn=256, max_rows_per_call=8)
    args.update(kw)
    cfg = b.make_config(**args)
    with pytest.raises(b.PetalsError) as e:
        b.petals_span_weight_bytes(cfg)
    assert e.value.code == code and str(e.value)


def test_host_side_checks_need_no_device(b):
    cfg = b.make_config(2, 64, 4, 256, 8)
    fake = C.c_void_p(0x10000)        # aligned, never dereferenced: create enqueues nothing
    L = b.lib()
    span = C.c_void_p()
    assert L.petals_span_create(C.byref(cfg), fake, C.c_void_p(0x10001), C.byref(span)) == -1   # misaligned
    assert L.petals_span_create(C.byref(cfg), fake, fake, C.byref(span)) == 0
    sess = C.c_void_p()
    assert L.petals_session_open(span, fake, 4, C.byref(sess)) == 0
    n = C.c_int32(-1)
    assert L.petals_session_length(sess, C.byref(n)) == 0 and n.value == 0
    arr = (C.c_void_p * 2)(sess.value, sess.value)
    # every check below fails before a kernel would be launched
    assert L.petals_span_prefill(span, arr, 1, 5, fake, C.c_void_p(0x20000), None) == -2      # 5 > capacity 4
    assert L.petals_span_prefill(span, arr, 1, 9, fake, C.c_void_p(0x20000), None) == -2      # 9 > max rows
    assert L.petals_span_prefill(span, arr, 2, 1, fake, C.c_void_p(0x20000), None) == -1      # duplicate
    assert L.petals_span_prefill(span, arr, 1, 1, fake, fake, None) == -1                     # aliasing
    assert L.petals_span_prefill(span, arr, 1, 1, fake, C.c_void_p(0x20000), None) == -4      # blocks not loaded
    assert b"loaded" in L.petals_last_error()
    assert L.petals_session_length(sess, C.byref(n)) == 0 and n.value == 0                    # nothing changed
    assert L.petals_span_destroy(span) == -4                                                  # session still open
    assert L.petals_session_close(sess) == 0
    assert L.petals_span_destroy(span) == 0
    assert L.petals_hidden_quantize(fake, C.c_size_t(10), 100, fake, fake, None) == -1        # block % 64


def test_measurement_aids_reject_bad_arguments_before_any_launch(b):
    L = b.lib()
    fake = C.c_void_p(0x10000)
    ops = C.c_double()
    assert L.petals_bench_mfma(2, 0, 10, 4, fake, C.byref(ops), None) == -1                  # kind
    assert L.petals_bench_mfma(0, 0, 0, 4, fake, C.byref(ops), None) == -1                   # iterations
    assert L.petals_bench_stage(0, 8, 1, 4, fake, C.c_size_t(1 << 20), fake, None) == -1     # no piece selected
    assert L.petals_bench_stage(7, 3, 1, 4, fake, C.c_size_t(1 << 20), fake, None) == -1     # fewer stages than ring slots
    assert L.petals_bench_stage(7, 8, 1, 4, None, C.c_size_t(1 << 20), fake, None) == -1     # null source
    assert L.petals_bench_stage(7, 8, 5, 4, fake, C.c_size_t(1 << 20), fake, None) == -2     # 5 regions x 8 stages x 32 KiB > 1 MiB
    assert b"32 KiB" in L.petals_last_error()


def test_code_table_bits_equal_the_oracle_table(b):
    import numpy as np
    import oracle
    t = np.array(b.petals_hidden_code_table(), np.float32)
    assert np.array_equal(t.view(np.uint32), oracle.codebook().view(np.uint32))


def test_backward_size_queries_and_host_side_checks(b):
    """Sizes of the backward pass's store and weight cache follow the layout arithmetic; argument errors are
    reported before any device work (Section 2.2 entry points)."""
    cfg = b.make_config(12, 14336, 112, 57344, 4096)
    H, F, M, nb = 14336, 57344, 4096, 12
    store = b.petals_span_backward_bytes(cfg, 8, 512)
    kept = nb * (M * H * 2 * 3 + M * H * 4 + M * F * 2 + 112 * M * 4) + 8 * nb * 2 * H * 512 * 2   # x, q, x1; fp32 context; GeLU input; lse; keys/values
    assert kept <= store <= kept * 1.5
    # a small call still holds the transposed fp16 weights of the largest linear (2 * F * H bytes)
    assert 2 * F * H <= b.petals_span_backward_bytes(cfg, 1, 16) <= 2 * F * H * 1.05
    assert b.petals_span_backward_cache_bytes(cfg) == nb * 12 * H * H * 2            # 2 bytes per weight
    for B, T in ((0, 4), (4, 0), (65, 1), (8, 513)):                                  # empty, empty, too many sequences, too many rows
        with pytest.raises(b.PetalsError):
            b.petals_span_backward_bytes(cfg, B, T)
    L = b.lib()
    small = b.make_config(2, 64, 4, 256, 8)
    fake, other, third = C.c_void_p(0x10000), C.c_void_p(0x20000), C.c_void_p(0x30000)
    span = C.c_void_p()
    assert L.petals_span_create(C.byref(small), fake, fake, C.byref(span)) == 0
    assert L.petals_span_backward(span, fake, 1, 4, fake, other, None, fake, None) == -1        # grad_in aliases hidden_in
    assert L.petals_span_backward(span, C.c_void_p(0x10010), 1, 4, fake, other, None, third, None) == -1   # store misaligned
    assert L.petals_span_backward(span, fake, 3, 4, fake, other, None, third, None) == -2       # 12 rows > 8
    assert L.petals_span_backward(span, fake, 1, 4, fake, other, None, third, None) == -4       # blocks not loaded
    assert L.petals_span_backward_attach_cache(span, C.c_void_p(0x10010)) == -1                 # misaligned
    assert L.petals_span_backward_attach_cache(span, other) == 0 and L.petals_span_backward_attach_cache(span, None) == 0
    assert L.petals_span_destroy(span) == 0
