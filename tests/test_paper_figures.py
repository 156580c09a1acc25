"""The figures the paper prints (tests/golden/paper_figures.txt, each with its citation) against the size formulas
of the library and of the synthetic workloads.  No GPU."""
import os

import pytest

from paper_2209_01188_amd import synth

ROOT = os.path.dirname(os.path.abspath(__file__))


def _figures():
    out = {}
    for line in open(os.path.join(ROOT, "golden", "paper_figures.txt")):
        line = line.split("#")[0].strip()
        if line:
            name, rest = line.split("=", 1)
            out[name.strip()] = float(rest.split(";")[0])
    return out


@pytest.fixture(scope="module")
def b():
    from paper_2209_01188_amd import binding, build
    if not os.path.exists(binding.LIB_PATH):
        build.build(force=False)
    return binding


def test_the_papers_own_arithmetic_is_consistent():
    f = _figures()
    assert f["bloom_parameters_billion"] * 2 == f["bloom_fp16_gb"]                       # 2 bytes per parameter
    assert f["bloom_fp16_gb"] / f["server_memory_gb"] == f["nodes_fp16"]
    assert f["nodes_fp16"] / 2 == f["nodes_int8"]                                         # 8-bit weights halve it
    int8_gbit = f["bloom_parameters_billion"] * f["int8_gb_per_billion"] * 8
    assert int8_gbit / f["pcie_gbit_s"] == f["offload_seconds"]
    assert int8_gbit / (f["pcie_gbit_s"] / 2) == f["offload_seconds_shared_switch"]


def test_library_sizes_of_the_bloom_shaped_stack_match_the_papers_figures(b):
    f = _figures()
    c5, c4 = synth.CONFIGS["C5"], synth.CONFIGS["C4"]
    assert (c5.n_blocks, c5.hidden, c5.n_heads, c5.F) == (70, 14336, 112, 57344)
    # all blocks in int8: the model minus the client's embeddings, at 1 GB per billion parameters
    cfg = b.make_config(c5.n_blocks, c5.hidden, c5.n_heads, c5.F, 1)
    gb = b.petals_span_weight_bytes(cfg) / 1e9
    blocks_billion = f["bloom_parameters_billion"] - f["client_embedding_billion"]
    assert abs(gb - blocks_billion * f["int8_gb_per_billion"]) / blocks_billion < 0.005
    # the embedding matrix the client keeps: 250880 x 14336
    assert abs(250880 * c5.hidden / 1e9 - f["client_embedding_billion"]) < 0.01
    # a 12-block span is 12/70 of that; 22 servers of 8 GB hold the 8-bit model
    span_gb = b.petals_span_weight_bytes(b.make_config(c4.n_blocks, c4.hidden, c4.n_heads, c4.F, 1)) / 1e9
    assert abs(span_gb - gb * 12 / 70) < 1e-6 * gb
    assert gb <= f["nodes_int8"] * f["server_memory_gb"]
    assert 2 * gb > (f["nodes_int8"] + 20) * f["server_memory_gb"]                        # in 16 bits it would not fit them


def test_synthetic_outlier_share_is_of_the_papers_order():
    """The recipe plants a handful of outlier feature dimensions per hidden state: a fraction of the order the paper
    quotes for real models (0.1 %), not a dense sprinkling."""
    f = _figures()
    for name in ("C2", "C3", "C4", "C5"):
        cfg = synth.CONFIGS[name]
        share = 100.0 * cfg.n_outlier_dims / cfg.hidden
        assert f["outlier_share_percent"] / 3 <= share <= f["outlier_share_percent"] * 1.5, (name, share)
