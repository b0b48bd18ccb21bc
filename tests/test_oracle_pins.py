"""Pins for the fp64 oracle: every check compares it with something that is NOT the oracle --
a library attention routine, a closed form, an invariant the definitions fix, or brute force.

Citations are to Climber (arXiv 2502.09888): Eq. (3) = the Adaptive Transformer Layer,
Sec. 3.1.2 = multi-scale sequence extraction, Sec. 3.2 = the "single user, multiple items"
mask and the serving flow with cached K/V.
"""
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as F

import oracle
import workloads as W


def rng(seed=0):
    return np.random.default_rng(seed)


def sdpa(q, k, v, mask, scale):
    """Library softmax attention in fp64.  q,k,v: [n,H,dh]; mask [n_q, n_k] bool -> [n_q, H*dh]."""
    tq, tk, tv = (torch.from_numpy(np.ascontiguousarray(a, dtype=np.float64)).permute(1, 0, 2)
                  for a in (q, k, v))
    o = F.scaled_dot_product_attention(tq, tk, tv, attn_mask=torch.from_numpy(mask), scale=scale)
    return o.permute(1, 0, 2).reshape(q.shape[0], -1).numpy()


def small_sumi(seed, B=2, L=24, M=5, H=2, dh=8, n_scen=3, n_beh=2, sub_len=8, ragged=True):
    g = rng(seed)
    hist_len = g.integers(L // 2, L + 1, size=B).astype(np.int32) if ragged else np.full(B, L, np.int32)
    pad = ((hist_len + 3) // 4 * 4).astype(np.int32)
    tok_off = np.concatenate([[0], np.cumsum(pad)]).astype(np.int32)
    ncand = g.integers(1, M + 1, size=B).astype(np.int32) if ragged else np.full(B, M, np.int32)
    cand_off = np.concatenate([[0], np.cumsum(ncand)]).astype(np.int32)
    T, Mt = tok_off[-1], cand_off[-1]
    d = dict(hist_len=hist_len, tok_off=tok_off, cand_off=cand_off, sub_len=sub_len, H=H, dh=dh)
    for n in ("qh", "kh", "vh"):
        d[n] = g.standard_normal((T, H, dh))
    for n in ("qc", "kc", "vc"):
        d[n] = g.standard_normal((Mt, H, dh))
    d["scen"], d["beh"] = g.integers(0, n_scen, T).astype(np.int32), g.integers(0, n_beh, T).astype(np.int32)
    d["cscen"], d["cbeh"] = g.integers(0, n_scen, Mt).astype(np.int32), g.integers(0, n_beh, Mt).astype(np.int32)
    d["tau"] = g.uniform(0.5, 2.0, (n_scen, n_beh))
    return d


def run_sumi(d, qk_scale=0.3, **over):
    a = {**d, **over}
    return oracle.attn_sumi(a["tok_off"], a["hist_len"], a["cand_off"], a["kh"], a["vh"], a["qc"],
                            a["kc"], a["vc"], a["cscen"], a["cbeh"], a["tau"], qk_scale)


def run_hist(d, qk_scale=0.3, causal=False, **over):
    a = {**d, **over}
    return oracle.attn_history(a["tok_off"], a["hist_len"], a["qh"], a["kh"], a["vh"], a["scen"],
                               a["beh"], a["tau"], qk_scale, sub_len=a["sub_len"], causal=causal)


# ---------------------------------------------------------------- softmax rows
def test_softmax_rows_sum_to_one_and_masked_entries_are_zero():
    g = rng(1)
    n, H, dh = 13, 3, 5
    q, k, v = (g.standard_normal((n, H, dh)) for _ in range(3))
    vis = g.random((n, n)) < 0.5
    vis[np.arange(n), np.arange(n)] = True
    tau = g.uniform(0.5, 2.0, n)
    o, a = oracle.masked_attention(q, k, v, tau, vis, 0.7, return_probs=True)
    assert np.all(a >= 0)
    assert np.abs(a.sum(-1) - 1).max() < 1e-12
    assert np.all(a[:, ~vis] == 0)
    # A V by a library contraction
    ref = np.einsum("hij,jhe->ihe", a, v).reshape(n, -1)
    assert np.abs(o - ref).max() < 1e-12


# ------------------------------------------------ tau = 1 -> textbook attention
def test_tau_one_is_library_softmax_attention_on_history_plus_candidate():
    # Eq. (3) with temperature 1 and qk_scale = 1/sqrt(dh) is plain softmax attention.
    d = small_sumi(2, B=1, L=16, M=4, sub_len=0, ragged=False)
    L, M = 16, 4
    tau1 = np.ones_like(d["tau"])
    scale = 1 / math.sqrt(d["dh"])
    got = run_sumi(d, qk_scale=scale, tau=tau1)
    for c in range(M):
        k = np.concatenate([d["kh"], d["kc"][c:c + 1]])
        v = np.concatenate([d["vh"], d["vc"][c:c + 1]])
        ref = sdpa(d["qc"][c:c + 1], k, v, np.ones((1, L + 1), bool), scale)
        assert np.abs(got[c] - ref[0]).max() < 1e-12


def test_general_tau_is_library_attention_with_row_scaled_queries():
    # softmax(R / tau_i) == softmax of (q_i / tau_i) K^T: feed the library row-scaled queries.
    d = small_sumi(3)
    got_s, got_h = run_sumi(d), run_hist(d)
    for b in range(len(d["hist_len"])):
        t0, Lb = d["tok_off"][b], d["hist_len"][b]
        kh, vh = d["kh"][t0:t0 + Lb], d["vh"][t0:t0 + Lb]
        for c in range(d["cand_off"][b], d["cand_off"][b + 1]):
            tau_c = d["tau"][d["cscen"][c], d["cbeh"][c]]
            ref = sdpa(d["qc"][c:c + 1] / tau_c, np.concatenate([kh, d["kc"][c:c + 1]]),
                       np.concatenate([vh, d["vc"][c:c + 1]]), np.ones((1, Lb + 1), bool), 0.3)
            assert np.abs(got_s[c] - ref[0]).max() < 1e-12
        # history: block-diagonal mask over the valid prefix
        idx = np.arange(Lb)
        mask = (idx[:, None] // d["sub_len"]) == (idx[None, :] // d["sub_len"])
        tau_r = d["tau"][d["scen"][t0:t0 + Lb], d["beh"][t0:t0 + Lb]]
        ref = sdpa(d["qh"][t0:t0 + Lb] / tau_r[:, None, None], kh, vh, mask, 0.3)
        assert np.abs(got_h[t0:t0 + Lb] - ref).max() < 1e-12


def test_scaling_identity_q_and_tau():
    d = small_sumi(4)
    alpha = 3.7
    a = run_sumi(d)
    b = run_sumi(d, qc=d["qc"] * alpha, tau=d["tau"] * alpha)
    assert np.abs(a - b).max() < 1e-12
    # and qk_scale is a plain multiplier of QK^T
    c = run_sumi(d, qk_scale=0.3 * alpha, tau=d["tau"] * alpha)
    assert np.abs(a - c).max() < 1e-12


def test_temperature_is_taken_from_the_query_row_not_the_key():
    # different ids on the history keys must not change a candidate's output
    d = small_sumi(5)
    a = run_hist(d)
    # permuting which (scen, beh) the *other* rows carry changes only those rows
    scen2 = d["scen"].copy()
    scen2[0] = (scen2[0] + 1) % d["tau"].shape[0]
    b = run_hist(d, scen=scen2)
    assert np.abs(a[1:] - b[1:]).max() == 0
    assert np.abs(a[0] - b[0]).max() > 1e-6


# ------------------------------------------------------------- closed forms
def test_two_key_closed_form():
    # L = 1, M = 1, dh = 1: o = (e^{q k1/tau} v1 + e^{q kc/tau} vc) / (e^{q k1/tau} + e^{q kc/tau})
    q, k1, kc, v1, vc, tau, s = 0.8, -1.3, 0.4, 2.0, -5.0, 0.75, 1.9
    got = oracle.attn_sumi([0, 1], [1], [0, 1], [[[k1]]], [[[v1]]], [[[q]]], [[[kc]]], [[[vc]]],
                           [0], [0], [[tau]], s)
    e1, e2 = math.exp(s * q * k1 / tau), math.exp(s * q * kc / tau)
    assert abs(got[0, 0] - (e1 * v1 + e2 * vc) / (e1 + e2)) < 1e-14


def test_large_tau_gives_mean_of_visible_values():
    d = small_sumi(6)
    got = run_sumi(d, tau=np.full_like(d["tau"], 1e9))
    goth = run_hist(d, tau=np.full_like(d["tau"], 1e9))
    for b in range(len(d["hist_len"])):
        t0, Lb = d["tok_off"][b], d["hist_len"][b]
        for c in range(d["cand_off"][b], d["cand_off"][b + 1]):
            ref = (d["vh"][t0:t0 + Lb].sum(0) + d["vc"][c]) / (Lb + 1)
            assert np.abs(got[c] - ref.reshape(-1)).max() < 1e-6
        for i in range(Lb):
            lo = i // d["sub_len"] * d["sub_len"]
            hi = min(lo + d["sub_len"], Lb)
            ref = d["vh"][t0 + lo:t0 + hi].mean(0)
            assert np.abs(goth[t0 + i] - ref.reshape(-1)).max() < 1e-6


def test_small_tau_gives_value_of_argmax_logit():
    d = small_sumi(7, H=1)
    got = run_sumi(d, tau=np.full_like(d["tau"], 1e-4))
    for b in range(len(d["hist_len"])):
        t0, Lb = d["tok_off"][b], d["hist_len"][b]
        for c in range(d["cand_off"][b], d["cand_off"][b + 1]):
            keys = np.concatenate([d["kh"][t0:t0 + Lb, 0], d["kc"][c:c + 1, 0]])
            vals = np.concatenate([d["vh"][t0:t0 + Lb, 0], d["vc"][c:c + 1, 0]])
            logits = keys @ d["qc"][c, 0]
            srt = np.sort(logits)
            assert srt[-1] - srt[-2] > 1e-2  # clear margin in this seed
            assert np.abs(got[c] - vals[np.argmax(logits)]).max() < 1e-9


def test_constant_values_are_reproduced_exactly_up_to_rounding():
    d = small_sumi(8)
    row = rng(80).standard_normal((1, d["H"], d["dh"]))
    vh = np.broadcast_to(row, d["vh"].shape)
    vc = np.broadcast_to(row, d["vc"].shape)
    got = run_sumi(d, vh=vh, vc=vc)
    assert np.abs(got - row.reshape(1, -1)).max() < 1e-14
    goth = run_hist(d, vh=vh)
    for b in range(len(d["hist_len"])):
        t0, Lb = d["tok_off"][b], d["hist_len"][b]
        assert np.abs(goth[t0:t0 + Lb] - row.reshape(1, -1)).max() < 1e-14


# ------------------------------------------------------------ SUMI structure
def test_candidate_isolation_add_remove_permute_chunk():
    # Sec. 3.2: candidates never see each other => a candidate's output does not depend on the
    # rest of the candidate set, bit for bit.
    d = small_sumi(9, B=1, M=7, ragged=False)
    full = run_sumi(d)
    perm = rng(90).permutation(7)
    p = run_sumi(d, qc=d["qc"][perm], kc=d["kc"][perm], vc=d["vc"][perm], cscen=d["cscen"][perm],
                 cbeh=d["cbeh"][perm])
    assert np.array_equal(p, full[perm])
    for lo, hi in ((0, 3), (3, 7), (2, 3)):  # chunks / removal of the others
        sl = slice(lo, hi)
        part = run_sumi(d, cand_off=np.array([0, hi - lo], np.int32), qc=d["qc"][sl], kc=d["kc"][sl],
                        vc=d["vc"][sl], cscen=d["cscen"][sl], cbeh=d["cbeh"][sl])
        assert np.array_equal(part, full[sl])


def test_sumi_equals_candidate_appended_alone_to_history():
    # brute force: the [history; candidate] sequence under the full visibility rule, all rows
    # recomputed; the candidate's row must equal the cached-K/V path, the history rows must equal
    # the block-diagonal history attention.
    d = small_sumi(10)
    got, goth = run_sumi(d), run_hist(d)
    S = d["sub_len"]
    for b in range(len(d["hist_len"])):
        t0, Lb = d["tok_off"][b], d["hist_len"][b]
        for c in range(d["cand_off"][b], d["cand_off"][b + 1]):
            n = Lb + 1
            q = np.concatenate([d["qh"][t0:t0 + Lb], d["qc"][c:c + 1]])
            k = np.concatenate([d["kh"][t0:t0 + Lb], d["kc"][c:c + 1]])
            v = np.concatenate([d["vh"][t0:t0 + Lb], d["vc"][c:c + 1]])
            vis = np.zeros((n, n), bool)
            i = np.arange(Lb)
            vis[:Lb, :Lb] = (i[:, None] // S) == (i[None, :] // S)
            vis[Lb, :] = True
            tau_r = np.concatenate([d["tau"][d["scen"][t0:t0 + Lb], d["beh"][t0:t0 + Lb]],
                                    [d["tau"][d["cscen"][c], d["cbeh"][c]]]])
            o = oracle.masked_attention(q, k, v, tau_r, vis, 0.3)
            assert np.abs(o[Lb] - got[c]).max() < 1e-13
            assert np.abs(o[:Lb] - goth[t0:t0 + Lb]).max() < 1e-13
            # and the same sequence through the library routine
            ref = sdpa(q / tau_r[:, None, None], k, v, vis, 0.3)
            assert np.abs(o - ref).max() < 1e-12


# ------------------------------------------------------------ block-diagonal
def test_block_diagonal_equals_independent_runs_per_subsequence():
    # Sec. 3.1.2: each subsequence is processed on its own.
    d = small_sumi(11, B=1, L=24, sub_len=8, ragged=False)
    got = run_hist(d)
    for s in range(3):
        sl = slice(8 * s, 8 * s + 8)
        alone = oracle.attn_history([0, 8], [8], d["qh"][sl], d["kh"][sl], d["vh"][sl],
                                    d["scen"][sl], d["beh"][sl], d["tau"], 0.3, sub_len=0)
        assert np.abs(alone - got[sl]).max() < 1e-14
    # one subsequence == full attention
    one = run_hist(d, sub_len=0)
    tau_r = d["tau"][d["scen"], d["beh"]]
    ref = sdpa(d["qh"] / tau_r[:, None, None], d["kh"], d["vh"], np.ones((24, 24), bool), 0.3)
    assert np.abs(one - ref).max() < 1e-12
    assert np.abs(one - got).max() > 1e-3


def test_partial_last_subsequence_and_causal_flag():
    d = small_sumi(12, B=1, L=21, sub_len=8, ragged=False)
    d["hist_len"][:] = 21
    Lb = 21
    i = np.arange(Lb)
    block = (i[:, None] // 8) == (i[None, :] // 8)
    tau_r = d["tau"][d["scen"][:Lb], d["beh"][:Lb]]
    qs = d["qh"][:Lb] / tau_r[:, None, None]
    got = run_hist(d)[:Lb]
    assert np.abs(got - sdpa(qs, d["kh"][:Lb], d["vh"][:Lb], block, 0.3)).max() < 1e-12
    gotc = run_hist(d, causal=True)[:Lb]
    assert np.abs(gotc - sdpa(qs, d["kh"][:Lb], d["vh"][:Lb], block & (i[None, :] <= i[:, None]),
                              0.3)).max() < 1e-12


def test_permutation_within_a_subsequence():
    # no positional term in scope => permuting tokens inside one subsequence permutes the history
    # outputs and leaves every candidate output unchanged.
    d = small_sumi(13, B=1, L=24, sub_len=8, ragged=False)
    perm = np.arange(24)
    perm[8:16] = 8 + rng(130).permutation(8)
    dp = {n: d[n][perm] for n in ("qh", "kh", "vh", "scen", "beh")}
    assert np.abs(run_hist(d, **dp) - run_hist(d)[perm]).max() < 1e-13
    assert np.abs(run_sumi(d, **dp) - run_sumi(d)).max() < 1e-13


# ------------------------------------------------------------------ padding
def test_padding_slots_are_never_read():
    d = small_sumi(14)
    a_s, a_h = run_sumi(d), run_hist(d)
    dirty = {n: d[n].copy() for n in ("qh", "kh", "vh", "scen", "beh")}
    for b in range(len(d["hist_len"])):
        lo, hi = d["tok_off"][b] + d["hist_len"][b], d["tok_off"][b + 1]
        for n in ("qh", "kh", "vh"):
            dirty[n][lo:hi] = np.nan
        dirty["scen"][lo:hi] = 10 ** 6
        dirty["beh"][lo:hi] = -5
    assert np.array_equal(run_sumi(d, **dirty), a_s)
    assert np.array_equal(run_hist(d, **dirty), a_h)


def test_empty_history_candidate_sees_only_itself():
    d = small_sumi(15, B=1, ragged=False)
    got = run_sumi(d, hist_len=np.array([0], np.int32))
    assert np.abs(got - d["vc"].reshape(got.shape)).max() < 1e-15


# ------------------------------------------------------------ logit range
def test_logit_shift_invariance_and_large_logits():
    d = small_sumi(16)
    base = run_sumi(d)
    # append a feature that adds the same constant to every visible logit of a row
    ones_h = np.ones(d["kh"].shape[:2] + (1,))
    ones_c = np.ones(d["kc"].shape[:2] + (1,))
    shifted = oracle.attn_sumi(d["tok_off"], d["hist_len"], d["cand_off"],
                               np.concatenate([d["kh"], ones_h], -1),
                               np.concatenate([d["vh"], 0 * ones_h], -1),
                               np.concatenate([d["qc"], 40 * ones_c], -1),
                               np.concatenate([d["kc"], ones_c], -1),
                               np.concatenate([d["vc"], 0 * ones_c], -1),
                               d["cscen"], d["cbeh"], d["tau"], 0.3)
    H, dh = d["H"], d["dh"]
    assert np.abs(shifted.reshape(-1, H, dh + 1)[..., :dh].reshape(base.shape) - base).max() < 1e-11
    big = run_sumi(d, qk_scale=60.0)  # |logit / tau| in the hundreds
    assert np.isfinite(big).all()


# ------------------------------------------------------------- error paths
def test_invalid_ids_and_temperatures_are_rejected():
    d = small_sumi(17)
    bad = d["cscen"].copy()
    bad[0] = d["tau"].shape[0]
    with pytest.raises(oracle.OracleError):
        run_sumi(d, cscen=bad)
    t = d["tau"].copy()
    t[:] = 0.0
    with pytest.raises(oracle.OracleError):
        run_sumi(d, tau=t)
    t[:] = np.nan
    with pytest.raises(oracle.OracleError):
        run_hist(d, tau=t)
    with pytest.raises(oracle.OracleError):
        oracle.masked_attention(d["qh"][:3], d["kh"][:3], d["vh"][:3], np.ones(3),
                                np.zeros((3, 3), bool), 1.0)


# -------------------------------------------------------------- layer pieces
def test_layer_pieces_against_library_one_liners():
    g = rng(18)
    x, gain = g.standard_normal((7, 12)), g.standard_normal(12)
    ref = F.rms_norm(torch.from_numpy(x), (12,), torch.from_numpy(gain), eps=1e-6).numpy()
    assert np.abs(oracle.rmsnorm(x, gain, 1e-6) - ref).max() < 1e-13
    Wm = g.standard_normal((12, 5))
    assert np.abs(oracle.linear(x, Wm) - x @ Wm).max() < 1e-13
    ge = oracle.gelu(x)
    ref = np.array([[0.5 * t * (1 + math.erf(t / math.sqrt(2))) for t in r] for r in x])
    assert np.abs(ge - ref).max() < 1e-15
    assert np.abs(ge - F.gelu(torch.from_numpy(x)).numpy()).max() < 1e-14


def tiny_stack(seed, n_layers=2, B=2, L=12, M=3, H=2, dh=4, F_=24, sub_len=4, causal=False):
    spec = W.StackSpec("tiny", B=B, L=L, sub_len=sub_len, M=M, n_layers=n_layers, d_model=H * dh,
                       H=H, dh=dh, d_ffn=F_, n_scen=3, n_beh=2, w_std=0.3, pad_to=4, seed=seed)
    w = W.make_stack(spec)
    cfg = oracle.StackConfig(n_layers, H * dh, H, dh, F_, 3, 2, sub_len=sub_len, qk_scale=0.5,
                             causal=causal)
    return spec, w, cfg


def torch_layer(cfg, lw, x, tau_row, vis):
    """The layer composed from library routines only (rms_norm, matmul, SDPA, erf-GELU)."""
    t = lambda a: torch.from_numpy(np.asarray(a, dtype=np.float64))
    d, H, dh = cfg.d_model, cfg.n_heads, cfg.d_head
    x = t(x)
    qkv = F.rms_norm(x, (d,), t(lw["g1"]), eps=cfg.rms_eps) @ t(lw["Wqkv"])
    q, k, v = (a.reshape(-1, H, dh).permute(1, 0, 2) for a in qkv.split(d, dim=1))
    q = q / t(tau_row)[None, :, None]
    o = F.scaled_dot_product_attention(q, k, v, attn_mask=torch.from_numpy(vis), scale=cfg.qk_scale)
    h = x + o.permute(1, 0, 2).reshape(-1, d) @ t(lw["Wo"])
    y = h + F.gelu(F.rms_norm(h, (d,), t(lw["g2"]), eps=cfg.rms_eps) @ t(lw["W1"])) @ t(lw["W2"])
    return y.numpy(), k.permute(1, 0, 2).reshape(-1, d).numpy(), v.permute(1, 0, 2).reshape(-1, d).numpy()


@pytest.mark.parametrize("causal", [False, True])
def test_stack_cached_path_equals_bruteforce_and_library_composition(causal):
    # Sec. 3.2: encode once + score against cached K/V == every candidate appended alone to the
    # history and recomputed from scratch, all layers; cached K/V == the brute force's history K/V.
    # With the causal flag a history token sees the tokens j <= i of its subsequence only; the two
    # variants must differ (else the flag would be pinned by nothing).
    spec, w, cfg = tiny_stack(19, causal=causal)
    kc, vc, yh = oracle.stack_encode(cfg, w["layers"], w["tau"], w["tok_off"], w["hist_len"],
                                     w["x_hist"], w["scen"], w["beh"])
    y = oracle.stack_score(cfg, w["layers"], w["tau"], w["tok_off"], w["hist_len"], kc, vc,
                           w["cand_off"], w["x_cand"], w["cscen"], w["cbeh"])
    L, S = spec.L, spec.sub_len
    for b in range(spec.B):
        t0 = w["tok_off"][b]
        for c in range(w["cand_off"][b], w["cand_off"][b + 1]):
            bf = oracle.stack_bruteforce(cfg, w["layers"], w["tau"], w["x_hist"][t0:t0 + L],
                                         w["scen"][t0:t0 + L], w["beh"][t0:t0 + L], w["x_cand"][c],
                                         w["cscen"][c], w["cbeh"][c])
            assert np.abs(bf - y[c]).max() < 1e-12
            # library composition of the same L+1 sequence
            n = L + 1
            i = np.arange(L)
            vis = np.zeros((n, n), bool)
            vis[:L, :L] = (i[:, None] // S) == (i[None, :] // S)
            if causal:
                vis[:L, :L] &= i[None, :] <= i[:, None]
            vis[L] = True
            x = np.concatenate([w["x_hist"][t0:t0 + L], w["x_cand"][c:c + 1]]).astype(np.float64)
            for l in range(cfg.n_layers):
                tau_r = np.concatenate([w["tau"][l][w["scen"][t0:t0 + L], w["beh"][t0:t0 + L]],
                                        [w["tau"][l][w["cscen"][c], w["cbeh"][c]]]])
                x, k_l, v_l = torch_layer(cfg, w["layers"][l], x, tau_r, vis)
                assert np.abs(k_l[:L] - kc[l, t0:t0 + L]).max() < 1e-12
                assert np.abs(v_l[:L] - vc[l, t0:t0 + L]).max() < 1e-12
            assert np.abs(x[L] - y[c]).max() < 1e-11
            assert np.abs(x[:L] - yh[t0:t0 + L]).max() < 1e-11
    if causal:
        _, w2, cfg2 = tiny_stack(19, causal=False)
        kc2, _, yh2 = oracle.stack_encode(cfg2, w2["layers"], w2["tau"], w2["tok_off"], w2["hist_len"],
                                          w2["x_hist"], w2["scen"], w2["beh"])
        assert np.abs(yh2 - yh).max() > 1e-3 and np.abs(kc2[1] - kc[1]).max() > 1e-3


def test_layer_masked_matches_library_composition():
    spec, w, cfg = tiny_stack(20, n_layers=1)
    g = rng(200)
    n = 9
    x = g.standard_normal((n, cfg.d_model))
    vis = g.random((n, n)) < 0.6
    vis[np.arange(n), np.arange(n)] = True
    tau_r = g.uniform(0.5, 2, n)
    y, k, v = oracle.layer_masked(cfg, w["layers"][0], x, tau_r, vis)
    yr, kr, vr = torch_layer(cfg, w["layers"][0], x, tau_r, vis)
    assert np.abs(y - yr).max() < 1e-12 and np.abs(k - kr).max() < 1e-12 and np.abs(v - vr).max() < 1e-12


# ---------------------------------------------- the benchmark's small config
def test_config1_oracle_against_library():
    w = W.make_attention(W.CONFIG1)
    s = W.CONFIG1
    got = oracle.attn_sumi(w["tok_off"], w["hist_len"], w["cand_off"], w["kh"], w["vh"], w["qc"],
                           w["kc"], w["vc"], w["cscen"], w["cbeh"], w["tau"], s.qk_scale)
    tau_c = w["tau"].astype(np.float64)[w["cscen"], w["cbeh"]]
    for c in range(s.M):
        ref = sdpa(w["qc"][c:c + 1].astype(np.float64) / tau_c[c],
                   np.concatenate([w["kh"], w["kc"][c:c + 1]]),
                   np.concatenate([w["vh"], w["vc"][c:c + 1]]), np.ones((1, s.L + 1), bool),
                   s.qk_scale)
        assert np.abs(got[c] - ref[0]).max() < 1e-12
    # unit-scale check of the recipe: logits have roughly unit variance
    logits = np.einsum("chd,jhd->chj", w["qc"].astype(np.float64), w["kh"].astype(np.float64))
    assert 0.7 < logits.std() < 1.4


# ------------------------------------------------ relative attention bias (Eq. (3): R = QK^T + f_b)
def bias_case(seed, **kw):
    base = dict(name="bias-tiny", B=2, L=40, L_min=9, sub_len=16, M=6, M_min=2, H=2, dh=8, n_scen=3, n_beh=2,
                pad_to=4, seed=seed, qk_scale=0.3, dtype="f32", std=1.0)
    base.update(kw)
    spec = W.AttnSpec(**base)
    return spec, W.add_bias_inputs(W.make_attention(spec), n_pos=9, n_time=6)


def hist_bias(spec, w, causal=False, **over):
    a = dict(w, **over)
    return oracle.attn_history_bias(a["tok_off"], a["hist_len"], a["qh"], a["kh"], a["vh"], a["scen"], a["beh"],
                                    a["tau"], spec.qk_scale, a["hist_pos"], a["hist_ts"], a["pos_table"],
                                    a["time_table"], sub_len=spec.sub_len, causal=causal)


def sumi_bias(spec, w, **over):
    a = dict(w, **over)
    return oracle.attn_sumi_bias(a["tok_off"], a["hist_len"], a["cand_off"], a["kh"], a["vh"], a["qc"], a["kc"],
                                 a["vc"], a["cscen"], a["cbeh"], a["tau"], spec.qk_scale, a["hist_pos"],
                                 a["hist_ts"], a["cand_pos"], a["cand_ts"], a["pos_table"], a["time_table"])


def test_bias_zero_tables_reproduce_the_bias_free_functions_bitwise():
    spec, w = bias_case(71)
    z = dict(pos_table=np.zeros_like(w["pos_table"]), time_table=np.zeros_like(w["time_table"]))
    for causal in (False, True):
        ref = oracle.attn_history(w["tok_off"], w["hist_len"], w["qh"], w["kh"], w["vh"], w["scen"], w["beh"],
                                  w["tau"], spec.qk_scale, sub_len=spec.sub_len, causal=causal)
        assert np.array_equal(hist_bias(spec, w, causal=causal, **z), ref)
    ref = oracle.attn_sumi(w["tok_off"], w["hist_len"], w["cand_off"], w["kh"], w["vh"], w["qc"], w["kc"],
                           w["vc"], w["cscen"], w["cbeh"], w["tau"], spec.qk_scale)
    assert np.array_equal(sumi_bias(spec, w, **z), ref)
    # and the tables of the case do change the result (else the pins below would pin nothing)
    assert np.abs(sumi_bias(spec, w) - ref).max() > 1e-2


def test_bias_constant_along_a_row_changes_nothing():
    # a bias that does not depend on the key (tables constant over their buckets, but different per
    # (scenario, behaviour, head)) shifts every logit of a row alike: softmax is unchanged
    spec, w = bias_case(72)
    g = rng(720)
    cp = g.standard_normal(w["pos_table"].shape[:3])[..., None] * np.ones(w["pos_table"].shape[3])
    ct = g.standard_normal(w["time_table"].shape[:3])[..., None] * np.ones(w["time_table"].shape[3])
    z = dict(pos_table=np.zeros_like(cp), time_table=np.zeros_like(ct))
    c = dict(pos_table=cp, time_table=ct)
    assert np.abs(hist_bias(spec, w, **c) - hist_bias(spec, w, **z)).max() < 1e-12
    assert np.abs(sumi_bias(spec, w, **c) - sumi_bias(spec, w, **z)).max() < 1e-12


def np_bias_matrix(w, b, h, scen_q, beh_q, pos_q, ts_q, pos_k, ts_k):
    """bias[i, j] from numpy clipping / log2 (an implementation of its own of the bucket rules)."""
    n_pos, n_time = w["pos_table"].shape[3], w["time_table"].shape[3]
    half = (n_pos - 1) // 2
    dp = np.clip(pos_q[:, None].astype(np.int64) - pos_k[None, :], -half, half) + half
    dt = np.abs(ts_q[:, None].astype(np.int64) - ts_k[None, :])
    bt = np.minimum(np.floor(np.log2(np.maximum(dt, 1))).astype(np.int64), n_time - 1)
    P = w["pos_table"].astype(np.float64)[scen_q, beh_q, h]      # [nq, n_pos]
    Tt = w["time_table"].astype(np.float64)[scen_q, beh_q, h]
    return np.take_along_axis(P, dp, 1) + np.take_along_axis(Tt, bt, 1)


def test_bias_is_library_attention_with_an_additive_mask():
    # (qk_scale QK^T + bias) / tau == SDPA on queries divided by tau with the float mask bias / tau
    spec, w = bias_case(73)
    got_h, got_c = hist_bias(spec, w), sumi_bias(spec, w)
    tq = lambda a: torch.from_numpy(np.asarray(a, np.float64))
    for b in range(spec.B):
        t0, Lb = int(w["tok_off"][b]), int(w["hist_len"][b])
        c0, c1 = int(w["cand_off"][b]), int(w["cand_off"][b + 1])
        sl = slice(t0, t0 + Lb)
        tau_h = w["tau"].astype(np.float64)[w["scen"][sl], w["beh"][sl]]
        i = np.arange(Lb)
        vis = (i[:, None] // spec.sub_len) == (i[None, :] // spec.sub_len)
        for h in range(spec.H):
            bm = np_bias_matrix(w, b, h, w["scen"][sl], w["beh"][sl], w["hist_pos"][sl], w["hist_ts"][sl],
                                w["hist_pos"][sl], w["hist_ts"][sl])
            mask = np.where(vis, bm / tau_h[:, None], -np.inf)
            ref = F.scaled_dot_product_attention(tq(w["qh"][sl, h] / tau_h[:, None])[None], tq(w["kh"][sl, h])[None],
                                                 tq(w["vh"][sl, h])[None], attn_mask=tq(mask)[None],
                                                 scale=spec.qk_scale)[0].numpy()
            assert np.abs(got_h[sl, h * spec.dh:(h + 1) * spec.dh] - ref).max() < 1e-12
            for c in range(c0, c1):
                tau_c = float(w["tau"][w["cscen"][c], w["cbeh"][c]])
                pk = np.concatenate([w["hist_pos"][sl], w["cand_pos"][c:c + 1]])
                tk = np.concatenate([w["hist_ts"][sl], w["cand_ts"][c:c + 1]])
                bm = np_bias_matrix(w, b, h, w["cscen"][c:c + 1], w["cbeh"][c:c + 1], w["cand_pos"][c:c + 1],
                                    w["cand_ts"][c:c + 1], pk, tk)
                kk = np.concatenate([w["kh"][sl, h], w["kc"][c:c + 1, h]])
                vv = np.concatenate([w["vh"][sl, h], w["vc"][c:c + 1, h]])
                ref = F.scaled_dot_product_attention(tq(w["qc"][c:c + 1, h].astype(np.float64) / tau_c)[None], tq(kk)[None], tq(vv)[None],
                                                     attn_mask=tq(bm / tau_c)[None], scale=spec.qk_scale)[0].numpy()
                assert np.abs(got_c[c, h * spec.dh:(h + 1) * spec.dh] - ref[0]).max() < 1e-12


def test_bias_brute_force_python_loops_and_bucket_edges():
    # the definition written out with math only, on a tiny case whose distances hit both clip ends of
    # the position buckets and the open-ended last time bucket
    spec, w = bias_case(74, B=1, L=12, L_min=12, sub_len=0, M=2, M_min=2, H=1, dh=4)
    w["hist_ts"][:12] = np.array([5, 5, 6, 8, 9, 13, 40, 41, 300, 301, 70000, 2_000_000_000], np.int32)
    w["cand_ts"][:] = np.array([2_000_000_000, 2_000_000_100], np.int32)
    n_pos, n_time = 9, 6
    P, Tt = w["pos_table"].astype(np.float64), w["time_table"].astype(np.float64)

    def bias(sc, bh, dp, dt):
        bp = max(-4, min(4, dp)) + 4
        a = max(abs(dt), 1)
        bt = min(int(math.floor(math.log2(a))), n_time - 1)
        return P[sc, bh, 0, bp] + Tt[sc, bh, 0, bt]

    def attend(q, keys, vals, biases, tau):
        r = [(spec.qk_scale * sum(float(a) * float(b) for a, b in zip(q, k)) + bb) / tau for k, bb in zip(keys, biases)]
        m = max(r)
        e = [math.exp(x - m) for x in r]
        z = sum(e)
        return [sum(e[j] / z * float(vals[j][d]) for j in range(len(keys))) for d in range(len(q))]

    got_h = hist_bias(spec, w, causal=True)
    for i in range(12):
        sc, bh = int(w["scen"][i]), int(w["beh"][i])
        js = range(i + 1)
        ref = attend(w["qh"][i, 0], [w["kh"][j, 0] for j in js], [w["vh"][j, 0] for j in js],
                     [bias(sc, bh, i - j, int(w["hist_ts"][i]) - int(w["hist_ts"][j])) for j in js],
                     float(w["tau"][sc, bh]))
        assert np.abs(got_h[i] - np.array(ref)).max() < 1e-12
    got_c = sumi_bias(spec, w)
    for c in range(2):
        sc, bh = int(w["cscen"][c]), int(w["cbeh"][c])
        keys = [w["kh"][j, 0] for j in range(12)] + [w["kc"][c, 0]]
        vals = [w["vh"][j, 0] for j in range(12)] + [w["vc"][c, 0]]
        bs = [bias(sc, bh, 12 - j, int(w["cand_ts"][c]) - int(w["hist_ts"][j])) for j in range(12)] + [bias(sc, bh, 0, 0)]
        ref = attend(w["qc"][c, 0], keys, vals, bs, float(w["tau"][sc, bh]))
        assert np.abs(got_c[c] - np.array(ref)).max() < 1e-12


# ---------------------------------------------- training-side packed forward (Sec. 3.2 mask, no cache)
@pytest.mark.parametrize("causal", [False, True])
def test_packed_forward_equals_cached_path_bruteforce_and_library_composition(causal):
    # one packed sequence [history; all candidates] under the SUMI mask == encode + score against the
    # cache == every candidate appended alone; and == the layer composed from library routines with the
    # mask written out here (candidates mutually invisible: an identity block in the mask)
    spec, w, cfg = tiny_stack(23, causal=causal, M=4)
    kc, vc, yh = oracle.stack_encode(cfg, w["layers"], w["tau"], w["tok_off"], w["hist_len"], w["x_hist"],
                                     w["scen"], w["beh"])
    y = oracle.stack_score(cfg, w["layers"], w["tau"], w["tok_off"], w["hist_len"], kc, vc, w["cand_off"],
                           w["x_cand"], w["cscen"], w["cbeh"])
    L, S = spec.L, spec.sub_len
    for b in range(spec.B):
        t0, c0, c1 = w["tok_off"][b], w["cand_off"][b], w["cand_off"][b + 1]
        ph, pc = oracle.stack_packed(cfg, w["layers"], w["tau"], w["x_hist"][t0:t0 + L], w["scen"][t0:t0 + L],
                                     w["beh"][t0:t0 + L], w["x_cand"][c0:c1], w["cscen"][c0:c1], w["cbeh"][c0:c1])
        assert np.abs(pc - y[c0:c1]).max() < 1e-12 and np.abs(ph - yh[t0:t0 + L]).max() < 1e-12
        bf = oracle.stack_bruteforce(cfg, w["layers"], w["tau"], w["x_hist"][t0:t0 + L], w["scen"][t0:t0 + L],
                                     w["beh"][t0:t0 + L], w["x_cand"][c0], w["cscen"][c0], w["cbeh"][c0])
        assert np.abs(bf - pc[0]).max() < 1e-12
        M = c1 - c0
        n = L + M
        i = np.arange(L)
        vis = np.zeros((n, n), bool)
        vis[:L, :L] = (i[:, None] // S) == (i[None, :] // S)
        if causal:
            vis[:L, :L] &= i[None, :] <= i[:, None]
        vis[L:, :L] = True
        vis[L:, L:] = np.eye(M, dtype=bool)
        x = np.concatenate([w["x_hist"][t0:t0 + L], w["x_cand"][c0:c1]]).astype(np.float64)
        for l in range(cfg.n_layers):
            tau_r = np.concatenate([w["tau"][l][w["scen"][t0:t0 + L], w["beh"][t0:t0 + L]],
                                    w["tau"][l][w["cscen"][c0:c1], w["cbeh"][c0:c1]]])
            x, _, _ = torch_layer(cfg, w["layers"][l], x, tau_r, vis)
        assert np.abs(x[L:] - pc).max() < 1e-11 and np.abs(x[:L] - ph).max() < 1e-11


# ------------------------------------------------------------ bit-wise gating fusion, Eq. (4)
def tiny_bgf(seed, nb=3, m=5, dg=6):
    spec = W.StackSpec("tiny-bgf", B=1, L=4, sub_len=0, M=1, n_layers=1, d_model=8, H=2, dh=4, d_ffn=12,
                       n_scen=3, n_beh=2, w_std=0.3, pad_to=4, seed=seed)
    cfg = oracle.StackConfig(1, 8, 2, 4, 12, 3, 2, qk_scale=0.5)
    return spec, cfg, W.make_bgf(spec, nb, dg, m)


def test_bgf_against_library_composition_and_layer_masked():
    spec, cfg, w = tiny_bgf(41)
    g, y, sc = oracle.bgf(cfg, w["atl"], w["tau_scen"], w["w_down"], w["w_up"], w["w_head"], w["b_head"], w["e"],
                          w["scen"])
    nb = w["n_blocks"]
    for i in range(w["e"].shape[0]):
        tau_r = np.full(nb, float(w["tau_scen"][w["scen"][i]]))
        vis = np.ones((nb, nb), bool)
        gl, _, _ = oracle.layer_masked(cfg, w["atl"], w["e"][i], tau_r, vis)
        gt, _, _ = torch_layer(cfg, w["atl"], w["e"][i], tau_r, vis)
        assert np.array_equal(gl, g[i]) and np.abs(gt - g[i]).max() < 1e-12
        G = torch.from_numpy(g[i].reshape(-1))
        gate = torch.sigmoid(torch.relu(G @ torch.from_numpy(w["w_down"].astype(np.float64))) @
                             torch.from_numpy(w["w_up"].astype(np.float64)))
        yr = (G * gate).numpy()
        assert np.abs(yr - y[i].reshape(-1)).max() < 1e-13
        assert abs(float(yr @ w["w_head"].astype(np.float64)) + w["b_head"] - sc[i]) < 1e-12


def test_bgf_closed_forms():
    spec, cfg, w = tiny_bgf(42)
    args = (w["tau_scen"], w["w_down"], w["w_up"], w["w_head"], w["b_head"])
    g, y, sc = oracle.bgf(cfg, w["atl"], *args, w["e"], w["scen"])
    # a zero up-projection: every gate is sigmoid(0) = 1/2
    g0, y0, sc0 = oracle.bgf(cfg, w["atl"], w["tau_scen"], w["w_down"], np.zeros_like(w["w_up"]), w["w_head"],
                             w["b_head"], w["e"], w["scen"])
    assert np.array_equal(g0, g) and np.abs(y0 - 0.5 * g).max() < 1e-15
    assert np.abs(sc0 - (0.5 * g.reshape(len(sc), -1) @ w["w_head"].astype(np.float64) + w["b_head"])).max() < 1e-12
    # the temperature depends on the scenario only, and matters
    other = (w["scen"] + 1) % 3
    assert np.abs(oracle.bgf(cfg, w["atl"], *args, w["e"], other)[0] - g).max() > 1e-4
    # blocks interact through the fusion attention only: with a zero output projection G = FFN-residual of
    # each row on its own, so permuting the blocks of a candidate permutes the rows of G
    atl0 = dict(w["atl"], Wo=np.zeros_like(w["atl"]["Wo"]))
    perm = np.array([2, 0, 1])
    ga = oracle.bgf(cfg, atl0, *args, w["e"], w["scen"])[0]
    gb = oracle.bgf(cfg, atl0, *args, w["e"][:, perm], w["scen"])[0]
    assert np.abs(gb - ga[:, perm]).max() < 1e-13
    # ... and with it, they do interact: the attention of the fusion layer is permutation-equivariant too
    gc = oracle.bgf(cfg, w["atl"], *args, w["e"][:, perm], w["scen"])[0]
    assert np.abs(gc - g[:, perm]).max() < 1e-12 and np.abs(ga - g).max() > 1e-3
    # one block: softmax over a single key is 1, the attention output is the value row itself
    spec1, cfg1, w1 = tiny_bgf(43, nb=1)
    g1 = oracle.bgf(cfg1, w1["atl"], w1["tau_scen"], w1["w_down"], w1["w_up"], w1["w_head"], w1["b_head"], w1["e"],
                    w1["scen"])[0]
    for i in range(len(g1)):
        x = torch.from_numpy(w1["e"][i].astype(np.float64))
        t = lambda a: torch.from_numpy(np.asarray(a, np.float64))
        v = (F.rms_norm(x, (8,), t(w1["atl"]["g1"]), eps=cfg1.rms_eps) @ t(w1["atl"]["Wqkv"]))[:, 16:]
        h = x + v @ t(w1["atl"]["Wo"])
        ref = h + F.gelu(F.rms_norm(h, (8,), t(w1["atl"]["g2"]), eps=cfg1.rms_eps) @ t(w1["atl"]["W1"])) @ t(w1["atl"]["W2"])
        assert np.abs(ref.numpy() - g1[i]).max() < 1e-12
