"""The allocation-free scoring call (scratch in the library's fixed per-GPU array) against the
call that takes a caller's workspace: same kernels, so the candidates' hidden states must be equal
bit for bit, and both within 2e-2 of the fp64 oracle.  Two calls in a row, the second with a
smaller input (the array keeps the first call's contents)."""
import numpy as np
import pytest

import workloads as W
from harness import GpuStack, max_abs, oracle_stack_users, say

pytestmark = pytest.mark.gpu


def score_both(spec):
    import torch
    w = W.make_stack(spec)
    g = GpuStack(w)
    P = g.P
    packed = torch.empty(P.climber_packed_weights_bytes(g.cfg), dtype=torch.uint8, device="cuda:0")
    P.climber_pack_weights(g.cfg, g.layers, packed)
    g.encode(packed=packed)
    y_ws = g.score(packed=packed)
    y = torch.full((g.m_total, spec.d_model), float("nan"), dtype=torch.float32, device="cuda:0")
    P.climber_sumi_score_static(g.cfg, g.layers, g.tau, g.cache, g.x_cand, g.cand_off, g.m_total,
                                g.m_max, g.cscen, g.cbeh, y, packed)
    torch.cuda.synchronize()
    y_st = y.cpu().numpy()
    ref, _ = oracle_stack_users(w, tuple(range(spec.B)))
    e = max_abs(y_st, ref)
    say(f"[case] {spec.name}: static vs workspace call equal={np.array_equal(y_st, y_ws)}, "
        f"vs oracle max-abs {e:.3e}")
    assert np.array_equal(y_st, y_ws)
    assert np.isfinite(y_st).all() and e < 2e-2
    return g, packed


def test_static_scratch_call_matches_workspace_call_twice_and_rejects_oversize():
    import torch
    big = W.StackSpec("static-first", B=3, L=256, sub_len=128, M=0, n_layers=2, d_model=128, H=2, dh=64,
                      d_ffn=256, n_scen=8, n_beh=4, seed=61, hist_lens=(256, 200, 130),
                      cand_counts=(150, 33, 70))
    small = W.StackSpec("static-second-smaller", B=2, L=128, sub_len=128, M=0, n_layers=2, d_model=128,
                        H=2, dh=64, d_ffn=256, n_scen=8, n_beh=4, seed=62, hist_lens=(128, 77),
                        cand_counts=(20, 9))
    score_both(big)
    g, packed = score_both(small)
    P = g.P
    # beyond the array: rejected before anything is launched; unpacked weights: rejected as well
    n = 1
    while P.climber_workspace_bytes(g.cfg, n) - P.climber_packed_weights_bytes(g.cfg) <= P.STATIC_SCRATCH_BYTES:
        n *= 2
    y = torch.empty((1, 128), dtype=torch.float32, device="cuda:0")
    with pytest.raises(P.ClimberError) as ei:
        P.climber_sumi_score_static(g.cfg, g.layers, g.tau, g.cache, g.x_cand, g.cand_off, n, n,
                                    g.cscen, g.cbeh, y, packed)
    assert ei.value.code == -6
    with pytest.raises(P.ClimberError) as ei:
        P.climber_sumi_score_static(g.cfg, g.layers, g.tau, g.cache, g.x_cand, g.cand_off, g.m_total,
                                    g.m_max, g.cscen, g.cbeh, y, None)
    assert ei.value.code == -1
