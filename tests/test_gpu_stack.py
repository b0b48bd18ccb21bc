"""GPU parity of the full layer stack (history encode -> per-layer KV cache -> candidate scoring)
against the fp64 oracle.  bf16 operands, fp32 accumulation and residual stream; tolerance 2e-2
max-abs on the candidates' final hidden states (unit scale)."""
import numpy as np
import pytest

import workloads as W
from harness import GpuStack, max_abs, oracle_stack_users, say

pytestmark = pytest.mark.gpu
TWO_KERNEL, VIA_ROWS = 2, 4   # config flags: history pass route, keys / values through rows


def run(spec, users, flags=0):
    say(f"[case] {spec.name} layers={spec.n_layers} d={spec.d_model} F={spec.d_ffn} B={spec.B} "
        f"L={spec.L} sub={spec.sub_len} M={spec.M} flags={flags} seed={spec.seed}")
    w = W.make_stack(spec)
    g = GpuStack(w, flags=flags)
    g.encode()
    y = g.score()
    assert np.isfinite(y).all()
    ref, _ = oracle_stack_users(w, users)
    got = np.concatenate([y[w["cand_off"][b]:w["cand_off"][b + 1]] for b in users])
    e = max_abs(got, ref)
    say(f"  y_cand max-abs {e:.3e} (|y| rms {np.sqrt((ref ** 2).mean()):.3f})")
    assert e < 2e-2
    return w, g, y


def test_small_stack_all_users():
    spec = W.StackSpec("stack-small", B=2, L=256, sub_len=128, M=70, n_layers=2, d_model=128, H=2,
                       dh=64, d_ffn=256, n_scen=8, n_beh=4, seed=31)
    run(spec, users=(0, 1))


def test_small_stack_ragged_lengths_nan_padding():
    # ragged histories (one shorter than a subsequence, one with a partial last subsequence and a
    # partial last 32-key block), ragged candidate counts (one user without candidates), NaN
    # embeddings in the padding rows: nothing of the padding may reach a valid row or the cache
    spec = W.StackSpec("stack-ragged", B=4, L=384, sub_len=128, M=0, n_layers=3, d_model=128, H=2,
                       dh=64, d_ffn=384, n_scen=8, n_beh=4, seed=33, hist_lens=(384, 77, 300, 129),
                       cand_counts=(37, 5, 0, 130), nan_padding=True)
    run(spec, users=(0, 1, 3))


def test_small_stack_ragged_lengths_padded_to_64():
    # padded lengths that are odd multiples of 64 (a GEMM wave's 128 rows then hold tokens of up to
    # three users), one user with no history at all (its candidates see only themselves), a batch
    # whose row count is not a multiple of the GEMM tile; NaN embeddings in the padding
    spec = W.StackSpec("stack-ragged-64", B=6, L=0, sub_len=128, M=0, n_layers=3, d_model=128, H=2,
                       dh=64, d_ffn=256, n_scen=8, n_beh=4, seed=36, pad_to=64,
                       hist_lens=(40, 0, 64, 200, 130, 33), cand_counts=(20, 7, 3, 40, 0, 11),
                       nan_padding=True)
    run(spec, users=(0, 1, 2, 3, 5))


def test_small_stack_uniform_partial_lengths():
    # all users with the same valid length, which ends inside a 32-key block and inside a subsequence:
    # the path on which the fused projection writes keys and values straight into the cache (slots past
    # the valid length must come out as zeros although their embeddings are NaN)
    spec = W.StackSpec("stack-uniform-partial", B=3, L=256, sub_len=128, M=45, n_layers=3, d_model=128,
                       H=2, dh=64, d_ffn=256, n_scen=8, n_beh=4, seed=35, hist_lens=(203, 203, 203),
                       nan_padding=True)
    run(spec, users=(0, 2))


def test_small_stack_causal_history():
    # weights large enough that attention matters: with these the candidates' outputs of the causal
    # and the full-visible stack differ by 0.6 (oracle), 30 times the tolerance
    spec = W.StackSpec("stack-causal", B=2, L=256, sub_len=128, M=50, n_layers=3, d_model=128, H=2,
                       dh=64, d_ffn=256, n_scen=8, n_beh=4, seed=34, hist_lens=(256, 200), causal=True,
                       w_std=0.05)
    run(spec, users=(0, 1))


def test_small_stack_one_layer_history_output():
    # climber_layer_forward on the history rows: compare the layer output itself
    import torch
    import oracle
    from harness import oracle_stack_config
    spec = W.StackSpec("stack-1layer", B=2, L=128, sub_len=0, M=33, n_layers=1, d_model=128, H=2,
                       dh=64, d_ffn=128, n_scen=8, n_beh=4, seed=32)
    say(f"[case] {spec.name}")
    w = W.make_stack(spec)
    g = GpuStack(w)
    x32 = g.x_hist.float().contiguous()
    out = torch.empty_like(x32)
    g.P.climber_layer_forward(g.cfg, g.layers[0], g.tau[0], 0, g.P.MODE_HISTORY, g.cache, x32, out,
                              g.scen, g.beh, None, 0, 0, g.ws)
    torch.cuda.synchronize()
    cfg = oracle_stack_config(spec)
    _, _, yh = oracle.stack_encode(cfg, w["layers"], w["tau"], w["tok_off"], w["hist_len"],
                                   w["x_hist"], w["scen"], w["beh"])
    e = max_abs(out.cpu().numpy(), yh)
    say(f"  history layer output max-abs {e:.3e}")
    assert e < 2e-2
    # the cache that call filled serves a candidate layer
    xc = g.x_cand.float().contiguous()
    yc = torch.empty_like(xc)
    g.P.climber_layer_forward(g.cfg, g.layers[0], g.tau[0], 0, g.P.MODE_CANDIDATE, g.cache, xc, yc,
                              g.cscen, g.cbeh, g.cand_off, g.m_total, g.m_max, g.ws)
    torch.cuda.synchronize()
    ref, _ = oracle_stack_users(w, (0, 1))
    e = max_abs(yc.cpu().numpy(), ref)
    say(f"  candidate layer output max-abs {e:.3e}")
    assert e < 2e-2


def test_prepacked_weights_give_the_same_bits():
    # weights brought into operand order once (climber_pack_weights) instead of on every call
    import torch
    spec = W.StackSpec("stack-prepacked", B=2, L=256, sub_len=128, M=70, n_layers=2, d_model=128, H=2,
                       dh=64, d_ffn=256, n_scen=8, n_beh=4, seed=37, hist_lens=(256, 130))
    say(f"[case] {spec.name}")
    w = W.make_stack(spec)
    g = GpuStack(w)
    g.encode()
    y0 = g.score()
    torch.cuda.synchronize()
    cache0 = g.buf.clone()
    payload = spec.n_layers * 2 * int(w["tok_off"][-1]) * spec.d_model * 2
    packed = torch.empty(g.P.climber_packed_weights_bytes(g.cfg), dtype=torch.uint8, device="cuda")
    g.P.climber_pack_weights(g.cfg, g.layers, packed)
    g.buf[g.buf.numel() - payload:].zero_()
    g.encode(packed=packed)
    y1 = g.score(packed=packed)
    assert torch.equal(g.buf, cache0)
    assert np.array_equal(y0, y1)
    ref, _ = oracle_stack_users(w, (0, 1))
    assert max_abs(y1, ref) < 2e-2


def test_config4_full_size_every_user_and_cache():
    # full size: every user's candidates against the oracle, and every layer of the cache, decoded
    # from its operand-fragment layout, against the oracle's per-layer history keys / values
    from harness import decode_bf16_cache, oracle_stack_config
    import oracle
    spec = W.CONFIG4
    w, g, y = run(spec, users=tuple(range(spec.B)))
    K, V = decode_bf16_cache(g.buf.cpu().numpy(), spec.B, w["tok_off"], spec.H, spec.n_layers)
    kc, vc, _ = oracle.stack_encode(oracle_stack_config(spec), w["layers"], w["tau"], w["tok_off"],
                                    w["hist_len"], w["x_hist"], w["scen"], w["beh"])
    T = int(w["tok_off"][-1])
    for l in range(spec.n_layers):
        ek = max_abs(K[l].reshape(T, -1), kc[l])
        ev = max_abs(V[l].reshape(T, -1), vc[l])
        say(f"  layer {l}: cache K max-abs {ek:.3e}, V max-abs {ev:.3e} (|k| rms {np.sqrt((kc[l] ** 2).mean()):.3f})")
        assert ek < 2e-2 and ev < 2e-2


def test_small_stack_cache_contents_ragged():
    # ragged batch: the decoded cache equals the oracle's keys / values on the valid rows of every
    # layer and is zero in every padding slot, on both routes of the keys / values into the cache
    from harness import decode_bf16_cache, oracle_stack_config
    import oracle
    spec = W.StackSpec("stack-cache-ragged", B=4, L=384, sub_len=128, M=0, n_layers=3, d_model=128, H=2,
                       dh=64, d_ffn=256, n_scen=8, n_beh=4, seed=38, hist_lens=(384, 77, 300, 129),
                       cand_counts=(9, 5, 0, 13), nan_padding=True)
    w = W.make_stack(spec)
    kc, vc, _ = oracle.stack_encode(oracle_stack_config(spec), w["layers"], w["tau"], w["tok_off"],
                                    w["hist_len"], np.nan_to_num(w["x_hist"]), w["scen"], w["beh"])
    T = int(w["tok_off"][-1])
    ok = np.zeros(T, bool)
    for b in range(spec.B):
        ok[w["tok_off"][b]:w["tok_off"][b] + w["hist_len"][b]] = True
    for flags in (0, VIA_ROWS):
        say(f"[case] {spec.name} flags={flags}")
        g = GpuStack(w, flags=flags)
        g.buf.fill_(0x7f)
        g.cache = g.P.climber_kv_cache_create(g.cfg, [int(x) for x in w["hist_len"]], g.padded, g.buf)
        g.encode()
        g.torch.cuda.synchronize()
        K, V = decode_bf16_cache(g.buf.cpu().numpy(), spec.B, w["tok_off"], spec.H, spec.n_layers)
        for l in range(spec.n_layers):
            ek = max_abs(K[l].reshape(T, -1)[ok], kc[l][ok])
            ev = max_abs(V[l].reshape(T, -1)[ok], vc[l][ok])
            say(f"  layer {l}: cache K max-abs {ek:.3e}, V max-abs {ev:.3e}")
            assert ek < 2e-2 and ev < 2e-2
            assert np.all(K[l][~ok] == 0) and np.all(V[l][~ok] == 0)


def test_projection_through_rows_path():
    # The fused projection writes keys and values straight into the cache; the same cases must hold
    # when they go through rows and the cache writer (or the one-kernel history pass) instead
    for spec, users in (
            (W.StackSpec("stack-small-rows", B=2, L=256, sub_len=128, M=70, n_layers=2, d_model=128, H=2,
                         dh=64, d_ffn=256, n_scen=8, n_beh=4, seed=31), (0, 1)),
            (W.StackSpec("stack-ragged-rows", B=4, L=384, sub_len=128, M=0, n_layers=3, d_model=128, H=2,
                         dh=64, d_ffn=384, n_scen=8, n_beh=4, seed=33, hist_lens=(384, 77, 300, 129),
                         cand_counts=(37, 5, 0, 130), nan_padding=True), (0, 1, 3)),
            (W.StackSpec("stack-uniform-partial-rows", B=3, L=256, sub_len=128, M=45, n_layers=3,
                         d_model=128, H=2, dh=64, d_ffn=256, n_scen=8, n_beh=4, seed=35,
                         hist_lens=(203, 203, 203), nan_padding=True), (0, 2)),
            (W.StackSpec("stack-causal-rows", B=2, L=256, sub_len=128, M=50, n_layers=3, d_model=128, H=2,
                         dh=64, d_ffn=256, n_scen=8, n_beh=4, seed=34, hist_lens=(256, 200), causal=True,
                         w_std=0.05), (0, 1))):
        run(spec, users, flags=VIA_ROWS)
        run(spec, users, flags=VIA_ROWS | TWO_KERNEL)
