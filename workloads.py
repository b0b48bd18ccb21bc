"""Seeded synthetic workloads shaped like the paper's serving sessions.

This module only draws random inputs (and rounds them to the storage type);
it holds none of the method's arithmetic and imports neither the oracle nor
the HIP library.  Both sides of every parity test receive the arrays made
here.

The paper's datasets are not available; these sessions take its shapes
(history lengths of a few hundred to a few thousand behaviours split into a
handful of equal subsequences, hundreds of candidates per request, a small
(scenario x behaviour) temperature table per layer) and stand in for them.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Optional

import numpy as np

BASE_SEED = 2502098880


@dataclass(frozen=True)
class AttnSpec:
    """Attention-only session batch (Q/K/V given, one layer)."""
    name: str
    dtype: str            # "f32" | "bf16"
    B: int
    L: int                # history length (max length when ragged)
    sub_len: int          # subsequence length n_k; 0 = one subsequence
    M: int                # candidates per user (max when ragged)
    H: int
    dh: int
    n_scen: int
    n_beh: int
    std: float            # standard deviation of Q/K/V entries
    qk_scale: float
    L_min: Optional[int] = None   # ragged histories: lengths uniform in [L_min, L]
    M_min: Optional[int] = None   # ragged candidate counts uniform in [M_min, M]
    pad_to: int = 128
    nan_padding: bool = False     # fill padded history slots with NaN / wild ids
    seed: int = BASE_SEED


@dataclass(frozen=True)
class StackSpec:
    """Full layer stack session batch."""
    name: str
    B: int
    L: int
    sub_len: int
    M: int
    n_layers: int
    d_model: int
    H: int
    dh: int
    d_ffn: int
    n_scen: int
    n_beh: int
    qk_scale: float = 1.0
    rms_eps: float = 1e-6
    w_std: float = 0.02
    pad_to: int = 128
    seed: int = BASE_SEED
    hist_lens: tuple = ()      # per-user valid history lengths (default: L for every user)
    cand_counts: tuple = ()    # per-user candidate counts (default: M for every user)
    nan_padding: bool = False  # embeddings of the padding rows are NaN: they must never be used
    causal: bool = False       # history token i sees j <= i of its subsequence only


CONFIG1 = AttnSpec("cfg1-tiny-f32", "f32", B=1, L=64, sub_len=0, M=8, H=2, dh=32, n_scen=4,
                   n_beh=3, std=32.0 ** -0.25, qk_scale=1.0, pad_to=1, seed=BASE_SEED + 1)
CONFIG2 = AttnSpec("cfg2-sumi-bf16", "bf16", B=32, L=512, sub_len=128, M=128, H=4, dh=64,
                   n_scen=8, n_beh=4, std=1.0, qk_scale=0.125, seed=BASE_SEED + 2)
CONFIG3 = AttnSpec("cfg3-sumi-kvcache-bf16", "bf16", B=64, L=1024, sub_len=256, M=512, H=8,
                   dh=64, n_scen=8, n_beh=4, std=1.0, qk_scale=0.125, seed=BASE_SEED + 3)
CONFIG4 = StackSpec("cfg4-stack-bf16", B=32, L=1024, sub_len=256, M=256, n_layers=4, d_model=512,
                    H=8, dh=64, d_ffn=2048, n_scen=8, n_beh=4, seed=BASE_SEED + 4)
CONFIG5 = AttnSpec("cfg5-ragged-bf16", "bf16", B=16, L=4096, sub_len=512, M=1024, H=8, dh=64,
                   n_scen=8, n_beh=4, std=1.0, qk_scale=0.125, L_min=512, M_min=256,
                   nan_padding=True, seed=BASE_SEED + 5)


def shrink(spec, **kw):
    """A smaller / altered copy of a spec (parity-test sizes)."""
    return replace(spec, **kw)


def round_bf16(a: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even to bfloat16, returned as float32 (storage rounding only)."""
    import torch
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32))
    return t.to(torch.bfloat16).to(torch.float32).numpy()


def _rng(seed):
    return np.random.Generator(np.random.Philox(seed))


def _round(a, dtype):
    a = a.astype(np.float32)
    return round_bf16(a) if dtype == "bf16" else a


def _lengths(rng, B, lo, hi):
    if lo is None:
        return np.full(B, hi, dtype=np.int32)
    return rng.integers(lo, hi + 1, size=B).astype(np.int32)


def _offsets(lens):
    off = np.zeros(len(lens) + 1, dtype=np.int32)
    off[1:] = np.cumsum(lens)
    return off


def make_attention(spec: AttnSpec) -> dict:
    """Draw one attention-only batch.  All float arrays are float32 holding values exactly
    representable in ``spec.dtype``."""
    rng = _rng(spec.seed)
    hist_len = _lengths(rng, spec.B, spec.L_min, spec.L)
    n_cand = _lengths(rng, spec.B, spec.M_min, spec.M)
    padded = ((hist_len + spec.pad_to - 1) // spec.pad_to * spec.pad_to).astype(np.int32)
    tok_off, cand_off = _offsets(padded), _offsets(n_cand)
    T, Mt = int(tok_off[-1]), int(cand_off[-1])
    H, dh = spec.H, spec.dh

    def normal(n):
        return _round(rng.standard_normal((n, H, dh), dtype=np.float32) * np.float32(spec.std),
                      spec.dtype)

    w = dict(spec=spec, hist_len=hist_len, tok_off=tok_off, cand_off=cand_off)
    for name in ("qh", "kh", "vh"):
        w[name] = normal(T)
    for name in ("qc", "kc", "vc"):
        w[name] = normal(Mt)
    w["scen"] = rng.integers(0, spec.n_scen, size=T).astype(np.int32)
    w["beh"] = rng.integers(0, spec.n_beh, size=T).astype(np.int32)
    w["cscen"] = rng.integers(0, spec.n_scen, size=Mt).astype(np.int32)
    w["cbeh"] = rng.integers(0, spec.n_beh, size=Mt).astype(np.int32)
    w["tau"] = rng.uniform(0.5, 2.0, size=(spec.n_scen, spec.n_beh)).astype(np.float32)
    if spec.nan_padding:
        for b in range(spec.B):
            lo, hi = tok_off[b] + hist_len[b], tok_off[b + 1]
            for name in ("qh", "kh", "vh"):
                w[name][lo:hi] = np.nan
            w["scen"][lo:hi] = 0x7FFFFFF0
            w["beh"][lo:hi] = -12345
    return w


def make_stack(spec: StackSpec) -> dict:
    """Draw one full-stack batch: bf16-representable weights, embeddings, ids, per-layer tau."""
    rng = _rng(spec.seed)
    d, F = spec.d_model, spec.d_ffn
    assert spec.H * spec.dh == d
    hist_len = np.asarray(spec.hist_lens or (spec.L,) * spec.B, dtype=np.int32)
    n_cand = np.asarray(spec.cand_counts or (spec.M,) * spec.B, dtype=np.int32)
    assert len(hist_len) == spec.B and len(n_cand) == spec.B
    padded = ((hist_len + spec.pad_to - 1) // spec.pad_to * spec.pad_to).astype(np.int32)
    tok_off = _offsets(padded)
    cand_off = _offsets(n_cand)
    T, Mt = int(tok_off[-1]), int(cand_off[-1])
    layers = []
    for _ in range(spec.n_layers):
        lw = {}
        for name, shp in (("g1", (d,)), ("Wqkv", (d, 3 * d)), ("Wo", (d, d)), ("g2", (d,)),
                          ("W1", (d, F)), ("W2", (F, d))):
            a = rng.standard_normal(shp, dtype=np.float32) * np.float32(spec.w_std)
            if name in ("g1", "g2"):
                a = a + np.float32(1.0)
            lw[name] = round_bf16(a)
        layers.append(lw)
    w = dict(spec=spec, hist_len=hist_len, tok_off=tok_off, cand_off=cand_off, layers=layers)
    w["x_hist"] = round_bf16(rng.standard_normal((T, d), dtype=np.float32))
    w["x_cand"] = round_bf16(rng.standard_normal((Mt, d), dtype=np.float32))
    w["scen"] = rng.integers(0, spec.n_scen, size=T).astype(np.int32)
    w["beh"] = rng.integers(0, spec.n_beh, size=T).astype(np.int32)
    w["cscen"] = rng.integers(0, spec.n_scen, size=Mt).astype(np.int32)
    w["cbeh"] = rng.integers(0, spec.n_beh, size=Mt).astype(np.int32)
    w["tau"] = rng.uniform(0.5, 2.0, size=(spec.n_layers, spec.n_scen, spec.n_beh)).astype(
        np.float32)
    if spec.nan_padding:
        for b in range(spec.B):
            w["x_hist"][tok_off[b] + hist_len[b]:tok_off[b + 1]] = np.nan
    return w


def add_bias_inputs(w: dict, n_pos: int = 33, n_time: int = 12, table_std: float = 0.5,
                    seed: int = 7) -> dict:
    """Inputs of the relative attention bias for an attention workload (random draws only):
    positions = index of the token in its user's history, candidates at the position after the
    history; timestamps = increasing, with gaps spread over five decades (the log-scale time
    buckets all occur), candidates a little after the user's last behaviour; bias tables
    N(0, table_std^2) per (scenario, behaviour, head, bucket), stored as float32."""
    spec = w["spec"]
    rng = _rng(spec.seed * 1000 + seed)
    T, Mt = int(w["tok_off"][-1]), int(w["cand_off"][-1])
    hist_pos = np.zeros(T, np.int32)
    hist_ts = np.zeros(T, np.int32)
    cand_pos = np.zeros(Mt, np.int32)
    cand_ts = np.zeros(Mt, np.int32)
    for b in range(spec.B):
        t0, t1 = int(w["tok_off"][b]), int(w["tok_off"][b + 1])
        n = t1 - t0
        hist_pos[t0:t1] = np.arange(n)
        gaps = np.exp2(rng.uniform(0.0, 17.0, size=n)).astype(np.int64)
        ts = 1_000_000 + np.cumsum(gaps)
        hist_ts[t0:t1] = np.minimum(ts, 2_000_000_000).astype(np.int32)
        c0, c1 = int(w["cand_off"][b]), int(w["cand_off"][b + 1])
        Lb = int(w["hist_len"][b])
        cand_pos[c0:c1] = Lb
        last = int(hist_ts[t0 + Lb - 1]) if Lb > 0 else 1_000_000
        cand_ts[c0:c1] = last + rng.integers(0, 5000, size=c1 - c0)
    H = spec.H
    w = dict(w)
    w.update(hist_pos=hist_pos, hist_ts=hist_ts, cand_pos=cand_pos, cand_ts=cand_ts,
             pos_table=(rng.standard_normal((spec.n_scen, spec.n_beh, H, n_pos)) * table_std).astype(np.float32),
             time_table=(rng.standard_normal((spec.n_scen, spec.n_beh, H, n_time)) * table_std).astype(np.float32))
    return w


def make_bgf(spec: StackSpec, n_blocks: int, d_gate: int, m: int, seed: int = 11) -> dict:
    """Random inputs of the fusion module (Eq. (4)): block outputs e [m, n_blocks, d] ~ N(0,1) (the
    scale of the stack's hidden states), scenario ids, the fusion layer's weights (drawn like a stack
    layer's), gate and head weights, a scenario-only temperature table.  bf16-representable where
    the library takes bf16."""
    rng = _rng(spec.seed * 977 + seed)
    d, F = spec.d_model, spec.d_ffn
    nd = n_blocks * d
    lw = {}
    for name, shp in (("g1", (d,)), ("Wqkv", (d, 3 * d)), ("Wo", (d, d)), ("g2", (d,)), ("W1", (d, F)),
                      ("W2", (F, d))):
        a = rng.standard_normal(shp, dtype=np.float32) * np.float32(spec.w_std)
        if name in ("g1", "g2"):
            a = a + np.float32(1.0)
        lw[name] = round_bf16(a)
    return dict(spec=spec, n_blocks=n_blocks, d_gate=d_gate, atl=lw,
                e=rng.standard_normal((m, n_blocks, d), dtype=np.float32),
                scen=rng.integers(0, spec.n_scen, size=m).astype(np.int32),
                tau_scen=rng.uniform(0.5, 2.0, size=spec.n_scen).astype(np.float32),
                w_down=round_bf16(rng.standard_normal((nd, d_gate), dtype=np.float32) * np.float32(nd ** -0.5)),
                w_up=round_bf16(rng.standard_normal((d_gate, nd), dtype=np.float32) * np.float32(2.0 * d_gate ** -0.5)),
                w_head=(rng.standard_normal(nd) * nd ** -0.5).astype(np.float32), b_head=0.25)
