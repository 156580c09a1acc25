"""petals_span_decode_step_static (the decode step whose intermediates live in the library's fixed device array)
against petals_span_decode_step, through the C ABI: same bits, two calls in a row with the second one smaller."""
import numpy as np
import pytest
import torch

from paper_2209_01188_amd import binding, synth
from tests.gpu_util import DEV, to_dev

pytestmark = pytest.mark.gpu


def _span(cfg, nb, rows):
    sp = binding.Span(nb, cfg.hidden, cfg.n_heads, cfg.F, rows, 1e-5, 6.0, DEV)
    for b in range(nb):
        sp.load_block(b, synth.block_params(cfg, b))
    return sp


@pytest.mark.parametrize("name,nb,T", [("C1", 2, 8), ("C2", 3, 70)])
def test_static_decode_step_equals_the_workspace_one_on_two_calls_the_second_smaller(name, nb, T):
    cfg = synth.CONFIGS[name]
    B = 5
    sp = _span(cfg, nb, B * T)
    try:
        cap = T + 4
        own = [sp.open_session(cap) for _ in range(B)]       # stepped through the span's workspace
        fix = [sp.open_session(cap) for _ in range(B)]       # stepped through the static array
        X = to_dev(synth.hidden_states(cfg, 0, B, T))
        y0 = sp.prefill(own, X)
        y1 = sp.prefill(fix, X)
        assert torch.equal(y0, y1)
        # poison the span's workspace: the static call must not depend on (or touch) it
        for step, sub in enumerate(([0, 1, 2, 3, 4], [3, 1])):    # 5 rows, then 2 rows
            x = to_dev(synth.hidden_states(cfg, 10 + step, len(sub), 1)[:, 0])
            ref = sp.decode_step([own[i] for i in sub], x)
            torch.cuda.synchronize()
            sp.workspace.fill_(0xA5)
            got = sp.decode_step_static([fix[i] for i in sub], x)
            torch.cuda.synchronize()
            assert (sp.workspace == 0xA5).all(), "the static call wrote into the span's workspace"
            assert np.array_equal(got.cpu().numpy().view(np.uint16), ref.cpu().numpy().view(np.uint16)), \
                "call %d (%d rows)" % (step, len(sub))
        assert [s.length for s in fix] == [s.length for s in own] == [T + 1, T + 2, T + 1, T + 2, T + 1]
        for b in range(nb):
            for a, f in zip(own, fix):
                assert torch.equal(a.export_kv(b), f.export_kv(b))
        # one row (the fused one-row kernels) after the several-row calls, same array
        x = to_dev(synth.hidden_states(cfg, 20, 1, 1)[:, 0])
        ref = sp.decode_step([own[2]], x)
        got = sp.decode_step_static([fix[2]], x)
        assert torch.equal(ref, got)
    finally:
        sp.close()


def test_static_decode_step_rejects_what_does_not_fit_and_leaves_sessions_alone():
    cfg = synth.CONFIGS["C4"]
    sp = binding.Span(1, cfg.hidden, cfg.n_heads, cfg.F, 64, 1e-5, 6.0, DEV)     # nothing loaded: no kernel will run
    try:
        ses = [sp.open_session(4) for _ in range(64)]
        x = torch.zeros((64, cfg.hidden), dtype=torch.float16, device=DEV)
        with pytest.raises(binding.PetalsError) as e:
            sp.decode_step_static(ses, x)
        assert e.value.code == -2 and "static buffer" in str(e.value)
        with pytest.raises(binding.PetalsError) as e:                                # fits, but the block is not loaded
            sp.decode_step_static(ses[:1], x[:1])
        assert e.value.code == -4
        assert all(s.length == 0 for s in ses)
    finally:
        sp.close()
