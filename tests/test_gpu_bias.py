"""GPU parity of the relative attention bias (Eq. (3): R = Q K^T + f_b, divided by the temperature):
the bias entry points of the C ABI against the oracle's *_bias functions on the same seeded inputs.
Bucket decisions are integer arithmetic on both sides, so they agree exactly; tolerances as for the
bias-free attention (1e-4 fp32, 2e-2 bf16)."""
import numpy as np
import pytest

import workloads as W
from harness import GpuAttention, max_abs, oracle, say, valid_rows

pytestmark = pytest.mark.gpu
TOL = {"f32": 1e-4, "bf16": 2e-2}


class GpuBias(GpuAttention):
    def __init__(self, w, causal=False):
        super().__init__(w, causal=causal)
        t = self.torch
        dev = "cuda:0"
        for n in ("hist_pos", "hist_ts", "cand_pos", "cand_ts", "pos_table", "time_table"):
            setattr(self, n, t.from_numpy(w[n]).to(dev).contiguous())
        self.rb = self.P.rel_bias(self.pos_table, self.time_table, self.hist_pos, self.hist_ts, self.cand_pos,
                                  self.cand_ts)

    def history_bias(self):
        t = self.torch
        o = t.full((self.qh.shape[0], self.d), float("nan"), dtype=self.dt, device="cuda:0")
        self.P.climber_attn_history_bias(self.cfg, self.tau, self.qh, self.kh, self.vh, self.scen, self.beh,
                                         self.cache, 0, o, self.rb)
        t.cuda.synchronize()
        return o.float().cpu().numpy()

    def sumi_bias(self):
        t, w = self.torch, self.w
        m_total = int(w["cand_off"][-1])
        m_max = int(np.diff(w["cand_off"]).max()) if m_total else 0
        o = t.full((max(m_total, 1), self.d), float("nan"), dtype=self.dt, device="cuda:0")
        self.P.climber_attn_sumi_bias(self.cfg, self.tau, self.cache, 0, self.qc, self.kc, self.vc, self.cand_off,
                                      m_total, m_max, self.cscen, self.cbeh, o, self.rb)
        t.cuda.synchronize()
        return o[:m_total].float().cpu().numpy()


def oracle_hist_bias(w, causal=False):
    s = w["spec"]
    return oracle.attn_history_bias(w["tok_off"], w["hist_len"], w["qh"], w["kh"], w["vh"], w["scen"], w["beh"],
                                    w["tau"], s.qk_scale, w["hist_pos"], w["hist_ts"], w["pos_table"],
                                    w["time_table"], sub_len=s.sub_len, causal=causal)


def oracle_sumi_bias(w):
    s = w["spec"]
    return oracle.attn_sumi_bias(w["tok_off"], w["hist_len"], w["cand_off"], w["kh"], w["vh"], w["qc"], w["kc"],
                                 w["vc"], w["cscen"], w["cbeh"], w["tau"], s.qk_scale, w["hist_pos"], w["hist_ts"],
                                 w["cand_pos"], w["cand_ts"], w["pos_table"], w["time_table"])


def check_bias(w, causal=False):
    spec = w["spec"]
    say(f"[case] bias {spec.name} dtype={spec.dtype} B={spec.B} L={spec.L} sub={spec.sub_len} M={spec.M} H={spec.H} "
        f"qk_scale={spec.qk_scale} causal={causal} n_pos={w['pos_table'].shape[3]} n_time={w['time_table'].shape[3]}")
    g = GpuBias(w, causal=causal)
    tol = TOL[spec.dtype]
    oh = g.history_bias()
    ok = valid_rows(w)
    e = max_abs(oh[ok], oracle_hist_bias(w, causal=causal)[ok])
    say(f"  history+bias max-abs {e:.3e}")
    assert np.isfinite(oh[ok]).all() and e < tol and np.all(oh[~ok] == 0)
    os_ = g.sumi_bias()
    ref = oracle_sumi_bias(w)
    e = max_abs(os_, ref)
    # the bias must matter in the case: without it the result is far from the reference
    plain = g.sumi()
    say(f"  sumi+bias max-abs {e:.3e} (bias-free kernel output differs from it by {max_abs(plain, ref):.2e})")
    assert np.isfinite(os_).all() and e < tol
    assert max_abs(plain, ref) > 5 * tol
    return g, os_


def test_fp32_bias_both_masks_ragged():
    spec = W.shrink(W.CONFIG1, name="f32-bias", B=3, L=90, L_min=10, M=11, M_min=1, sub_len=32, pad_to=8,
                    nan_padding=True, dh=48, H=3, seed=81)
    w = W.add_bias_inputs(W.make_attention(spec), n_pos=15, n_time=9)
    check_bias(w)
    check_bias(w, causal=True)
    check_bias(W.add_bias_inputs(W.make_attention(W.CONFIG1)))


def test_bf16_bias_multi_tile_ragged_both_masks():
    spec = W.shrink(W.CONFIG5, name="bf16-bias-ragged", B=4, L=700, L_min=1, sub_len=256, M=200, M_min=1, H=2,
                    seed=82)
    w = W.add_bias_inputs(W.make_attention(spec))
    check_bias(w)
    check_bias(w, causal=True)
    spec = W.shrink(W.CONFIG2, name="bf16-bias-onesub", B=2, L=333, L_min=77, sub_len=0, M=70, H=1,
                    nan_padding=True, seed=83)
    check_bias(W.add_bias_inputs(W.make_attention(spec), n_pos=5, n_time=3))


def test_bf16_bias_single_bucket_tables_and_edges():
    # n_pos = n_time = 1: one entry per (scenario, behaviour, head), i.e. a constant along every row,
    # which softmax ignores: the result equals the bias-free one; and timestamps at the int32 ends
    spec = W.shrink(W.CONFIG2, name="bf16-bias-const", B=2, L=256, sub_len=128, M=60, H=2, seed=84)
    w = W.add_bias_inputs(W.make_attention(spec), n_pos=1, n_time=1, table_std=3.0)
    w["hist_ts"][::7] = -2_000_000_000
    w["cand_ts"][::5] = 2_000_000_000
    g = GpuBias(w)
    g.history(want_output=False)
    ref = oracle_sumi_bias(w)
    e = max_abs(g.sumi_bias(), ref)
    say(f"[case] bias {spec.name}: sumi+bias max-abs {e:.3e}; vs bias-free oracle "
        f"{max_abs(ref, oracle.attn_sumi(w['tok_off'], w['hist_len'], w['cand_off'], w['kh'], w['vh'], w['qc'], w['kc'], w['vc'], w['cscen'], w['cbeh'], w['tau'], spec.qk_scale)):.1e}")
    assert e < 2e-2


def test_bias_buckets_at_the_ends_of_the_int32_range():
    # positions and time stamps at and near the ends of int32: differences that overflow 32-bit
    # subtraction, every one of the 32 possible log2 buckets of |ts_i - ts_j| has a table entry of its own
    ends = np.array([-2**31, -2**31 + 1, -2**30, -3, -1, 0, 1, 2, 2**30, 2**31 - 2, 2**31 - 1], dtype=np.int64)
    for dtype, tol_key in (("f32", "f32"), ("bf16", "bf16")):
        base = W.CONFIG1 if dtype == "f32" else W.CONFIG2
        spec = (W.shrink(base, name="f32-bias-ends", B=2, L=192, sub_len=64, M=33, seed=88) if dtype == "f32" else
                W.shrink(base, name="bf16-bias-ends", B=2, L=256, sub_len=128, M=70, H=2, seed=89))
        w = W.add_bias_inputs(W.make_attention(spec), n_pos=7, n_time=34, table_std=1.0)
        rng = np.random.default_rng(5)
        for n in ("hist_pos", "hist_ts", "cand_pos", "cand_ts"):
            pick = rng.random(w[n].shape) < 0.5
            w[n][pick] = rng.choice(ends, size=int(pick.sum())).astype(np.int32)
        check_bias(w)


def test_bf16_bias_large_logits_take_the_running_maximum_pass():
    spec = W.shrink(W.CONFIG2, name="bf16-bias-biglogits", B=2, L=256, sub_len=128, M=100, H=2, qk_scale=12.0,
                    seed=85)
    check_bias(W.add_bias_inputs(W.make_attention(spec), table_std=20.0))


def test_bf16_bias_zero_tables_reproduce_the_bias_free_result():
    # zero tables: the bias variant computes the bias-free attention (it keeps the query exact and
    # scales the logits in fp32 where the plain kernel folds the scale into the query, so the two agree
    # to rounding, not bit for bit); both against the bias-free oracle
    spec = W.shrink(W.CONFIG2, name="bf16-bias-zero", B=2, L=384, sub_len=128, M=100, H=2, seed=86)
    w = W.add_bias_inputs(W.make_attention(spec))
    w["pos_table"][:] = 0
    w["time_table"][:] = 0
    g = GpuBias(w)
    g.history(want_output=False)
    ref = oracle.attn_sumi(w["tok_off"], w["hist_len"], w["cand_off"], w["kh"], w["vh"], w["qc"], w["kc"], w["vc"],
                           w["cscen"], w["cbeh"], w["tau"], spec.qk_scale)
    with_zero, plain = g.sumi_bias(), g.sumi()
    say(f"[case] bias {spec.name}: zero tables vs bias-free kernel {max_abs(with_zero, plain):.3e}, vs bias-free oracle "
        f"{max_abs(with_zero, ref):.3e} (bias-free kernel: {max_abs(plain, ref):.3e})")
    assert max_abs(with_zero, ref) < 2e-2 and max_abs(with_zero, plain) < 2e-2


def test_bias_at_config2_and_config3_shapes():
    for spec in (W.CONFIG2, W.CONFIG3):
        w = W.add_bias_inputs(W.make_attention(spec))
        say(f"[case] bias {spec.name} full size")
        g = GpuBias(w)
        oh = g.history_bias()
        ok = valid_rows(w)
        e = max_abs(oh[ok], oracle_hist_bias(w)[ok])
        say(f"  history+bias max-abs {e:.3e}")
        assert e < 2e-2
        e = max_abs(g.sumi_bias(), oracle_sumi_bias(w))
        say(f"  sumi+bias max-abs over all users {e:.3e}")
        assert e < 2e-2


def test_randomized_shapes_scales_masks_with_bias():
    # seeded sweep: ragged histories and candidate counts, paddings of 64 / 128, any subsequence length the
    # API admits, 1..4 heads, logit scales from the unit-scale benchmark to far beyond, both masks,
    # table sizes from one bucket to more buckets than distances
    rng = np.random.Generator(np.random.Philox(2502098))
    done = 0
    for i in range(60):
        L = int(rng.integers(1, 1400))
        M = int(rng.choice([1, 2, 31, 33, 64, 127, 128, 129, 255, 256, 257, 300, 513]))
        spec = W.shrink(W.CONFIG2, name=f"bias-sweep-{i}", B=int(rng.integers(1, 6)), L=L, L_min=int(rng.integers(1, L + 1)),
                        sub_len=int(rng.choice([0, 128, 256, 384, 512])), M=M, M_min=int(rng.integers(1, M + 1)),
                        H=int(rng.integers(1, 5)), pad_to=int(rng.choice([64, 128])), nan_padding=bool(rng.integers(0, 2)),
                        n_scen=int(rng.integers(1, 9)), n_beh=int(rng.integers(1, 5)),
                        qk_scale=float(rng.choice([0.125, 0.125, 0.3, 0.7, 1.5, 6.0])), seed=7000 + i)
        w = W.add_bias_inputs(W.make_attention(spec), n_pos=int(rng.choice([1, 5, 33])), n_time=int(rng.choice([1, 7, 34])),
                              table_std=float(rng.choice([0.3, 1.0])))
        causal = bool(rng.integers(0, 2))
        g = GpuBias(w, causal=causal)
        oh = g.history_bias()
        ok = valid_rows(w)
        e1 = max_abs(oh[ok], oracle_hist_bias(w, causal=causal)[ok])
        e2 = max_abs(g.sumi_bias(), oracle_sumi_bias(w))
        say(f"[case] {spec.name} B={spec.B} L={spec.L} sub={spec.sub_len} M={spec.M} H={spec.H} qk_scale={spec.qk_scale} "
            f"causal={causal}: history+bias {e1:.3e}, sumi+bias {e2:.3e}")
        assert np.isfinite(oh[ok]).all() and np.all(oh[~ok] == 0) and e1 < 2e-2 and e2 < 2e-2
        done += 1
    assert done == 60
