"""GPU parity: the HIP attention kernels, called through the C ABI, against the fp64 oracle on the
same seeded inputs.  Tolerances: max-abs 1e-4 on the fp32 path, 2e-2 on the bf16 path (outputs at
unit scale), as the target states."""
import numpy as np
import pytest

import workloads as W
from harness import (GpuAttention, max_abs, oracle_history, oracle_sumi, say, valid_rows)

pytestmark = pytest.mark.gpu
TOL = {"f32": 1e-4, "bf16": 2e-2}


def check_all(w, causal=False, hist=True):
    spec = w["spec"]
    say(f"[case] {spec.name} dtype={spec.dtype} B={spec.B} L={spec.L} sub={spec.sub_len} M={spec.M} "
        f"H={spec.H} dh={spec.dh} causal={causal} seed={spec.seed}")
    g = GpuAttention(w, causal=causal)
    tol = TOL[spec.dtype]
    if hist:
        oh = g.history()
        ref = oracle_history(w, causal=causal)
        ok = valid_rows(w)
        e = max_abs(oh[ok], ref[ok])
        say(f"  history max-abs {e:.3e}")
        assert np.isfinite(oh[ok]).all() and e < tol
        assert np.all(oh[~ok] == 0)
    else:
        g.history(want_output=False)
    os_ = g.sumi()
    ref = oracle_sumi(w)
    e = max_abs(os_, ref)
    say(f"  sumi max-abs {e:.3e}")
    assert np.isfinite(os_).all() and e < tol
    return g, os_


def test_config1_fp32():
    check_all(W.make_attention(W.CONFIG1))


def test_fp32_subsequences_causal_ragged():
    spec = W.shrink(W.CONFIG1, name="f32-ragged", B=3, L=90, L_min=10, M=11, M_min=1, sub_len=32,
                    pad_to=8, nan_padding=True, dh=48, H=3, seed=11)
    w = W.make_attention(spec)
    check_all(w)
    check_all(w, causal=True)


def test_bf16_small_multi_tile_ragged_tail():
    # several key tiles, several query tiles, candidate count with a ragged tail
    spec = W.shrink(W.CONFIG2, name="bf16-small", B=3, L=384, sub_len=128, M=200, H=2, seed=21)
    check_all(W.make_attention(spec))


def test_bf16_ragged_lengths_nan_padding():
    spec = W.shrink(W.CONFIG5, name="bf16-ragged-small", B=5, L=700, L_min=1, sub_len=256, M=300,
                    M_min=1, H=2, seed=22)
    w = W.make_attention(spec)
    check_all(w)


def test_bf16_causal_history():
    # history token i sees j <= i of its subsequence.  Subsequences of 128 and 256 (the query tile of
    # 256 rows holds two resp. one of them; under the flag they take the tiled kernel, not the
    # one-kernel pass), one undivided sequence spanning several query tiles, ragged lengths with
    # NaN padding; the candidate pass on the cache that the causal history call wrote.
    for name, kw in (("bf16-causal-sub128", dict(B=3, L=384, sub_len=128, M=40, H=2, seed=41)),
                     ("bf16-causal-sub256", dict(B=2, L=512, sub_len=256, M=40, H=2, seed=42)),
                     ("bf16-causal-whole", dict(B=2, L=640, sub_len=0, M=33, H=2, seed=43))):
        check_all(W.make_attention(W.shrink(W.CONFIG2, name=name, **kw)), causal=True)
    spec = W.shrink(W.CONFIG5, name="bf16-causal-ragged", B=5, L=700, L_min=1, sub_len=256, M=30,
                    M_min=1, H=2, seed=44)
    check_all(W.make_attention(spec), causal=True)


def test_bf16_large_temperature_table():
    # more (scenario, behaviour) pairs than a wavefront has lanes: the one-kernel history pass keeps
    # small tables in a register and reads larger ones from memory
    spec = W.shrink(W.CONFIG2, name="bf16-tau-128", B=2, L=256, sub_len=128, M=40, H=2, n_scen=16,
                    n_beh=8, seed=45)
    check_all(W.make_attention(spec))
    spec = W.shrink(W.CONFIG2, name="bf16-tau-128-sub256", B=2, L=512, sub_len=256, M=40, H=2, n_scen=16,
                    n_beh=8, seed=46)
    check_all(W.make_attention(spec))


def test_bf16_shape_sweep():
    # seeded sweep over shapes the API admits: paddings of 64 and 128, subsequence lengths that are
    # any multiple of 128 (384 takes the tiled kernel with 128-query tiles), 1..3 heads, ragged
    # histories down to no history at all, candidate counts around the 128 / 256 query tiles and
    # down to none, both masks, NaN padding
    rng = np.random.Generator(np.random.Philox(20250209))
    for i in range(12):
        sub = int(rng.choice([0, 128, 256, 384, 512]))
        L = int(rng.integers(1, 900))
        M = int(rng.choice([1, 31, 127, 128, 129, 255, 257, 300]))
        spec = W.shrink(W.CONFIG2, name=f"bf16-sweep-{i}", B=int(rng.integers(1, 5)), L=L,
                        L_min=int(rng.integers(0, L + 1)), sub_len=sub, M=M, M_min=int(rng.integers(0, M + 1)),
                        H=int(rng.integers(1, 4)), pad_to=int(rng.choice([64, 128])), nan_padding=True,
                        n_scen=int(rng.integers(1, 9)), n_beh=int(rng.integers(1, 5)), seed=1000 + i)
        check_all(W.make_attention(spec), causal=bool(rng.integers(0, 2)))


def test_bf16_single_subsequence_and_odd_lengths():
    spec = W.shrink(W.CONFIG2, name="bf16-onesub", B=2, L=333, L_min=77, sub_len=0, M=70, H=1,
                    nan_padding=True, seed=23)
    check_all(W.make_attention(spec))


def test_bf16_empty_history_and_empty_candidate_set():
    spec = W.shrink(W.CONFIG2, name="bf16-empty", B=3, L=128, sub_len=128, M=40, H=2, seed=24)
    w = W.make_attention(spec)
    w["hist_len"][1] = 0            # user 1: no history -> candidates see only themselves
    c = np.diff(w["cand_off"]).copy()
    c[2] = 0                        # user 2: no candidates
    keep = np.concatenate([np.arange(w["cand_off"][b], w["cand_off"][b] + c[b]) for b in range(3)])
    for n in ("qc", "kc", "vc", "cscen", "cbeh"):
        w[n] = np.ascontiguousarray(w[n][keep])
    w["cand_off"] = np.concatenate([[0], np.cumsum(c)]).astype(np.int32)
    g, o = check_all(w)
    lo, hi = w["cand_off"][1], w["cand_off"][2]
    assert max_abs(o[lo:hi], w["vc"][lo:hi].reshape(hi - lo, -1)) == 0.0


def test_bf16_large_logits_do_not_overflow():
    spec = W.shrink(W.CONFIG2, name="bf16-biglogits", B=1, L=256, sub_len=128, M=64, H=2,
                    qk_scale=12.0, seed=25)   # |logit / tau| in the hundreds
    check_all(W.make_attention(spec))


def test_bf16_candidate_isolation_and_chunking_are_bitwise():
    spec = W.shrink(W.CONFIG2, name="bf16-chunks", B=2, L=256, sub_len=128, M=256, H=2, seed=26)
    w = W.make_attention(spec)
    g, full = check_all(w, hist=False)
    off = w["cand_off"]
    for lo, hi in ((0, 128), (128, 256), (5, 6), (100, 231)):
        part = g.sumi(sel=(lo, hi))
        assert np.array_equal(part, full[g.last_idx]), (lo, hi)


def test_config2_full():
    check_all(W.make_attention(W.CONFIG2))


@pytest.mark.parametrize("spec,users", [(W.CONFIG3, (0, 31, 63)), (W.CONFIG5, None)])
def test_full_size_sampled_users(spec, users):
    # full-size launch (the configuration the benchmark times); the oracle is run on a sample of
    # users, each computed on its own
    w = W.make_attention(spec)
    say(f"[case] {spec.name} full size, T={w['tok_off'][-1]} M_tot={w['cand_off'][-1]}")
    g = GpuAttention(w)
    oh = g.history()
    out = g.sumi()
    assert np.isfinite(out).all()
    if users is None:
        order = np.argsort(w["hist_len"])
        users = (int(order[0]), int(order[len(order) // 2]), int(order[-1]))
    for b in users:
        c0, c1 = w["cand_off"][b], w["cand_off"][b + 1]
        e = max_abs(out[c0:c1], oracle_sumi(w, users=[b]))
        say(f"  user {b}: L={w['hist_len'][b]} M={c1 - c0} sumi max-abs {e:.3e}")
        assert e < 2e-2
    # history: one user in full
    b = users[-1]
    t0, t1 = int(w["tok_off"][b]), int(w["tok_off"][b + 1])
    sub = dict(w, tok_off=np.array([0, t1 - t0], np.int32), hist_len=w["hist_len"][b:b + 1],
               qh=w["qh"][t0:t1], kh=w["kh"][t0:t1], vh=w["vh"][t0:t1], scen=w["scen"][t0:t1],
               beh=w["beh"][t0:t1])
    ref = oracle_history(sub)
    Lb = int(w["hist_len"][b])
    e = max_abs(oh[t0:t0 + Lb], ref[:Lb])
    say(f"  user {b}: history max-abs {e:.3e}")
    assert e < 2e-2


def test_two_kernel_history_path():
    # Subsequences of 128 / 256 tokens take the fused cache-write + attention kernel by default; the
    # same cases must also hold on the two-kernel path (cache writer, then ring attention), which
    # the library reads from the environment once per process: run them in a child process.
    import os
    import subprocess
    import sys
    if os.environ.get("CLIMBER_HIST_FUSED") == "0":
        pytest.skip("this is the child process")
    env = dict(os.environ, CLIMBER_HIST_FUSED="0")
    here = os.path.dirname(os.path.abspath(__file__))
    r = subprocess.run([sys.executable, "-u", "-m", "pytest", os.path.join(here, "test_gpu_attention.py"),
                        "-m", "gpu", "-x", "-q", "-k", "ragged or small_multi or large_logits",
                        "--timeout", "120", "--timeout-method", "thread"],
                       env=env, capture_output=True, text=True, timeout=600)
    say(r.stdout[-1500:])
    assert r.returncode == 0, r.stdout[-3000:] + r.stderr[-2000:]
