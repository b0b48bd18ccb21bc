"""fp64 CPU oracle for the Climber serving hot path -- TEST INFRASTRUCTURE ONLY.

Thin ctypes/numpy marshalling over ``climber_oracle.c`` (plain C, direct loops,
double precision).  Nothing under the product package imports this module; only
``tests/``, the smoke check and the benchmark's ``cpu_baseline`` leg do.  It
shares no code with the HIP path.

Each wrapper names the passage of the paper (Climber, arXiv 2502.09888) its C
function follows; the arithmetic lives in the C file only.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass
from typing import Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "climber_oracle.c")
_LIB = os.path.join(_HERE, "libclimber_oracle.so")

ERRORS = {-1: "id outside the temperature table or bad length",
          -2: "temperature not finite or <= 0",
          -3: "a query row has no visible key",
          -4: "out of memory"}


class OracleError(ValueError):
    pass


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (-O2 -fopenmp).  Returns the library path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-std=c99", "-Wall", "-Wextra", "-shared",
                               "-fPIC", "-o", _LIB, _SRC, "-lm"])
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.oracle_num_threads.restype = C.c_int
    return _lib


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def _f64(a):
    return np.ascontiguousarray(a, dtype=np.float64)


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def _p(a):
    return a.ctypes.data_as(C.c_void_p) if a is not None else None


def _check(rc):
    if rc != 0:
        raise OracleError(ERRORS.get(rc, f"oracle error {rc}"))


def masked_attention(q, k, v, tau_row, visible, qk_scale, return_probs=False):
    """Eq. (3) with an explicit visibility matrix: A = softmax((qk_scale QK^T)/tau_row), A V.

    q, k, v: [n, H, dh]; tau_row: [n]; visible: [n, n] bool.  Returns o [n, H*dh]
    (and A [H, n, n] when return_probs).
    """
    q, k, v, tau_row = _f64(q), _f64(k), _f64(v), _f64(tau_row)
    n, H, dh = q.shape
    vis = np.ascontiguousarray(visible, dtype=np.uint8)
    assert vis.shape == (n, n) and k.shape == q.shape == v.shape and tau_row.shape == (n,)
    o = np.empty((n, H * dh))
    a = np.empty((H, n, n)) if return_probs else None
    _check(_load().oracle_masked_attention(n, H, dh, _p(q), _p(k), _p(v), _p(tau_row), _p(vis),
                                           C.c_double(qk_scale), _p(o), _p(a)))
    return (o, a) if return_probs else o


def attn_history(tok_off, hist_len, q, k, v, scen, beh, tau, qk_scale, sub_len=0, causal=False):
    """Block-diagonal history attention (Sec. 3.1.2 split + Eq. (3)).

    q, k, v: [T_pad, H, dh] packed histories; scen, beh: [T_pad]; tau: [n_scen, n_beh].
    """
    q, k, v, tau = _f64(q), _f64(k), _f64(v), _f64(tau)
    tok_off, hist_len, scen, beh = _i32(tok_off), _i32(hist_len), _i32(scen), _i32(beh)
    T, H, dh = q.shape
    B = len(hist_len)
    assert tok_off.shape == (B + 1,) and tok_off[B] == T and scen.shape == (T,) == beh.shape
    o = np.empty((T, H * dh))
    _check(_load().oracle_attn_history(B, _p(tok_off), _p(hist_len), H, dh, int(sub_len),
                                       int(bool(causal)), _p(q), _p(k), _p(v), _p(scen), _p(beh),
                                       _p(tau), tau.shape[0], tau.shape[1], C.c_double(qk_scale),
                                       _p(o)))
    return o


def attn_sumi(tok_off, hist_len, cand_off, kh, vh, qc, kc, vc, cscen, cbeh, tau, qk_scale):
    """SUMI attention (Sec. 3.2 mask + Eq. (3)): candidates see the history K/V and themselves.

    kh, vh: [T_pad, H, dh]; qc, kc, vc: [M_tot, H, dh]; returns [M_tot, H*dh].
    """
    kh, vh, qc, kc, vc, tau = _f64(kh), _f64(vh), _f64(qc), _f64(kc), _f64(vc), _f64(tau)
    tok_off, hist_len, cand_off = _i32(tok_off), _i32(hist_len), _i32(cand_off)
    cscen, cbeh = _i32(cscen), _i32(cbeh)
    T, H, dh = kh.shape
    M = qc.shape[0]
    B = len(hist_len)
    assert tok_off[B] == T and cand_off[B] == M and qc.shape == (M, H, dh)
    assert cscen.shape == (M,) == cbeh.shape
    o = np.empty((M, H * dh))
    _check(_load().oracle_attn_sumi(B, _p(tok_off), _p(hist_len), _p(cand_off), H, dh, _p(kh),
                                    _p(vh), _p(qc), _p(kc), _p(vc), _p(cscen), _p(cbeh), _p(tau),
                                    tau.shape[0], tau.shape[1], C.c_double(qk_scale), _p(o)))
    return o


def _bias_args(H, n_scen, n_beh, pos_table, time_table):
    pt, tt = _f64(pos_table), _f64(time_table)
    assert pt.shape[:3] == (n_scen, n_beh, H) and tt.shape[:3] == (n_scen, n_beh, H)
    return pt, tt


def attn_history_bias(tok_off, hist_len, q, k, v, scen, beh, tau, qk_scale, hist_pos, hist_ts,
                      pos_table, time_table, sub_len=0, causal=False):
    """attn_history with the relative attention bias of Eq. (3) added to the logits before the
    temperature divide.  pos_table [n_scen, n_beh, H, n_pos] (n_pos odd), time_table
    [n_scen, n_beh, H, n_time]; hist_pos, hist_ts: int32 [T_pad]."""
    q, k, v, tau = _f64(q), _f64(k), _f64(v), _f64(tau)
    tok_off, hist_len, scen, beh = _i32(tok_off), _i32(hist_len), _i32(scen), _i32(beh)
    hist_pos, hist_ts = _i32(hist_pos), _i32(hist_ts)
    T, H, dh = q.shape
    B = len(hist_len)
    pt, tt = _bias_args(H, tau.shape[0], tau.shape[1], pos_table, time_table)
    assert tok_off[B] == T and hist_pos.shape == (T,) == hist_ts.shape
    o = np.empty((T, H * dh))
    _check(_load().oracle_attn_history_bias(B, _p(tok_off), _p(hist_len), H, dh, int(sub_len),
                                            int(bool(causal)), _p(q), _p(k), _p(v), _p(scen), _p(beh),
                                            _p(tau), tau.shape[0], tau.shape[1], C.c_double(qk_scale),
                                            _p(hist_pos), _p(hist_ts), _p(pt), _p(tt), pt.shape[3],
                                            tt.shape[3], _p(o)))
    return o


def attn_sumi_bias(tok_off, hist_len, cand_off, kh, vh, qc, kc, vc, cscen, cbeh, tau, qk_scale,
                   hist_pos, hist_ts, cand_pos, cand_ts, pos_table, time_table):
    """attn_sumi with the relative attention bias (a candidate's own key has zero distance)."""
    kh, vh, qc, kc, vc, tau = _f64(kh), _f64(vh), _f64(qc), _f64(kc), _f64(vc), _f64(tau)
    tok_off, hist_len, cand_off = _i32(tok_off), _i32(hist_len), _i32(cand_off)
    cscen, cbeh = _i32(cscen), _i32(cbeh)
    hist_pos, hist_ts, cand_pos, cand_ts = _i32(hist_pos), _i32(hist_ts), _i32(cand_pos), _i32(cand_ts)
    T, H, dh = kh.shape
    M = qc.shape[0]
    B = len(hist_len)
    pt, tt = _bias_args(H, tau.shape[0], tau.shape[1], pos_table, time_table)
    assert tok_off[B] == T and cand_off[B] == M and cand_pos.shape == (M,) == cand_ts.shape
    o = np.empty((M, H * dh))
    _check(_load().oracle_attn_sumi_bias(B, _p(tok_off), _p(hist_len), _p(cand_off), H, dh, _p(kh),
                                         _p(vh), _p(qc), _p(kc), _p(vc), _p(cscen), _p(cbeh), _p(tau),
                                         tau.shape[0], tau.shape[1], C.c_double(qk_scale),
                                         _p(hist_pos), _p(hist_ts), _p(cand_pos), _p(cand_ts), _p(pt),
                                         _p(tt), pt.shape[3], tt.shape[3], _p(o)))
    return o


def rmsnorm(x, g, eps):
    x, g = _f64(x), _f64(g)
    n, d = x.shape
    y = np.empty_like(x)
    _load().oracle_rmsnorm(n, d, _p(x), _p(g), C.c_double(eps), _p(y))
    return y


def linear(x, W):
    x, W = _f64(x), _f64(W)
    n, din = x.shape
    assert W.shape[0] == din
    y = np.empty((n, W.shape[1]))
    _load().oracle_linear(n, din, W.shape[1], _p(x), _p(W), _p(y))
    return y


def gelu(x):
    x = _f64(x)
    y = np.empty_like(x)
    _load().oracle_gelu(C.c_size_t(x.size), _p(x), _p(y))
    return y


class _Cfg(C.Structure):
    _fields_ = [(n, C.c_int) for n in ("n_layers", "d_model", "n_heads", "d_head", "d_ffn",
                                       "n_scen", "n_beh", "sub_len", "causal")] + \
               [("qk_scale", C.c_double), ("rms_eps", C.c_double)]


class _LayerW(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("g1", "Wqkv", "Wo", "g2", "W1", "W2")]


@dataclass
class StackConfig:
    """Hyper-parameters of the layer stack (f_QKV / f_FFN of Eq. (3) made concrete)."""
    n_layers: int
    d_model: int
    n_heads: int
    d_head: int
    d_ffn: int
    n_scen: int
    n_beh: int
    sub_len: int = 0
    causal: bool = False
    qk_scale: float = 1.0
    rms_eps: float = 1e-6

    def _c(self):
        return _Cfg(self.n_layers, self.d_model, self.n_heads, self.d_head, self.d_ffn,
                    self.n_scen, self.n_beh, self.sub_len, int(self.causal), self.qk_scale,
                    self.rms_eps)


def _weights(cfg: StackConfig, layers: Sequence[dict]):
    """layers: list of dicts with g1, Wqkv, Wo, g2, W1, W2 (any float dtype)."""
    assert len(layers) == cfg.n_layers
    d, F = cfg.d_model, cfg.d_ffn
    shapes = dict(g1=(d,), Wqkv=(d, 3 * d), Wo=(d, d), g2=(d,), W1=(d, F), W2=(F, d))
    keep, arr = [], (_LayerW * cfg.n_layers)()
    for l, lw in enumerate(layers):
        for name, shp in shapes.items():
            a = _f64(lw[name])
            assert a.shape == shp, (name, a.shape, shp)
            keep.append(a)
            setattr(arr[l], name, a.ctypes.data)
    return arr, keep


def layer_masked(cfg: StackConfig, layer: dict, x, tau_row, visible):
    """One layer over an arbitrary sequence with an explicit visibility matrix.

    Returns (y, k, v), each [n, d]."""
    c1 = StackConfig(**{**cfg.__dict__, "n_layers": 1})
    w, keep = _weights(c1, [layer])
    x, tau_row = _f64(x), _f64(tau_row)
    n, d = x.shape
    vis = np.ascontiguousarray(visible, dtype=np.uint8)
    y, k, v = np.empty_like(x), np.empty_like(x), np.empty_like(x)
    cc = c1._c()
    _check(_load().oracle_layer_masked(C.byref(cc), w, n, _p(x), _p(tau_row), _p(vis), _p(y),
                                       _p(k), _p(v)))
    return y, k, v


def stack_bruteforce(cfg: StackConfig, layers, tau, x_hist, scen, beh, x_cand, cscen, cbeh):
    """"Single user, single item": one candidate appended alone to the valid history, the whole
    L+1 sequence recomputed through every layer (Sec. 3.2).  Returns the candidate's final row."""
    w, keep = _weights(cfg, layers)
    tau, x_hist, x_cand = _f64(tau), _f64(x_hist), _f64(x_cand)
    scen, beh = _i32(scen), _i32(beh)
    L, d = x_hist.shape
    assert tau.shape == (cfg.n_layers, cfg.n_scen, cfg.n_beh) and x_cand.shape == (d,)
    y = np.empty(d)
    cc = cfg._c()
    _check(_load().oracle_stack_bruteforce(C.byref(cc), w, _p(tau), L, _p(x_hist), _p(scen),
                                           _p(beh), _p(x_cand), int(cscen), int(cbeh), _p(y)))
    return y


def stack_encode(cfg: StackConfig, layers, tau, tok_off, hist_len, x_hist, scen, beh):
    """History encode: returns (k_cache, v_cache) [n_layers, T_pad, d] and y_hist [T_pad, d]."""
    w, keep = _weights(cfg, layers)
    tau, x_hist = _f64(tau), _f64(x_hist)
    tok_off, hist_len, scen, beh = _i32(tok_off), _i32(hist_len), _i32(scen), _i32(beh)
    T, d = x_hist.shape
    B = len(hist_len)
    assert tok_off[B] == T and tau.shape == (cfg.n_layers, cfg.n_scen, cfg.n_beh)
    kc = np.empty((cfg.n_layers, T, d))
    vc = np.empty((cfg.n_layers, T, d))
    yh = np.empty((T, d))
    cc = cfg._c()
    _check(_load().oracle_stack_encode(C.byref(cc), w, _p(tau), B, _p(tok_off), _p(hist_len),
                                       _p(x_hist), _p(scen), _p(beh), _p(kc), _p(vc), _p(yh)))
    return kc, vc, yh


def stack_score(cfg: StackConfig, layers, tau, tok_off, hist_len, k_cache, v_cache, cand_off,
                x_cand, cscen, cbeh):
    """Candidate scoring against the per-layer cached history K/V.  Returns y_cand [M_tot, d]."""
    w, keep = _weights(cfg, layers)
    tau, k_cache, v_cache, x_cand = _f64(tau), _f64(k_cache), _f64(v_cache), _f64(x_cand)
    tok_off, hist_len, cand_off = _i32(tok_off), _i32(hist_len), _i32(cand_off)
    cscen, cbeh = _i32(cscen), _i32(cbeh)
    B = len(hist_len)
    M, d = x_cand.shape
    assert cand_off[B] == M and k_cache.shape == (cfg.n_layers, tok_off[B], d)
    y = np.empty((M, d))
    cc = cfg._c()
    _check(_load().oracle_stack_score(C.byref(cc), w, _p(tau), B, _p(tok_off), _p(hist_len),
                                      _p(k_cache), _p(v_cache), _p(cand_off), _p(x_cand),
                                      _p(cscen), _p(cbeh), _p(y)))
    return y


def stack_packed(cfg: StackConfig, layers, tau, x_hist, scen, beh, x_cand, cscen, cbeh):
    """Training-side "single user, multiple items" forward of ONE user (Sec. 3.2): the valid history
    rows and all candidates as one packed sequence under the mask of that section, no cache.
    Returns (y_hist [L, d], y_cand [M, d])."""
    w, keep = _weights(cfg, layers)
    tau, x_hist, x_cand = _f64(tau), _f64(x_hist), _f64(x_cand)
    scen, beh, cscen, cbeh = _i32(scen), _i32(beh), _i32(cscen), _i32(cbeh)
    L, d = x_hist.shape
    M = x_cand.shape[0]
    assert tau.shape == (cfg.n_layers, cfg.n_scen, cfg.n_beh) and x_cand.shape == (M, d)
    yh, yc = np.empty((L, d)), np.empty((M, d))
    cc = cfg._c()
    _check(_load().oracle_stack_packed(C.byref(cc), w, _p(tau), L, _p(x_hist), _p(scen), _p(beh), M,
                                       _p(x_cand), _p(cscen), _p(cbeh), _p(yh), _p(yc)))
    return yh, yc


def bgf(cfg: StackConfig, atl_layer: dict, tau_scen, w_down, w_up, w_head, b_head, e, scen):
    """Bit-wise gating fusion (Eq. (4)) + linear head for m candidates.  e: [m, N_b, d] block outputs;
    scen: [m].  Returns (G [m, N_b, d], Y [m, N_b, d], score [m])."""
    c1 = StackConfig(**{**cfg.__dict__, "n_layers": 1})
    w, keep = _weights(c1, [atl_layer])
    tau_scen, w_down, w_up, w_head, e = _f64(tau_scen), _f64(w_down), _f64(w_up), _f64(w_head), _f64(e)
    scen = _i32(scen)
    m, nb, d = e.shape
    dg = w_down.shape[1]
    assert d == cfg.d_model and w_down.shape == (nb * d, dg) and w_up.shape == (dg, nb * d)
    assert w_head.shape == (nb * d,) and scen.shape == (m,)
    g, y, sc = np.empty_like(e), np.empty_like(e), np.empty(m)
    cc = c1._c()
    _check(_load().oracle_bgf(C.byref(cc), w, _p(tau_scen), len(tau_scen), nb, dg, _p(w_down), _p(w_up),
                              _p(w_head), C.c_double(b_head), m, _p(e), _p(scen), _p(g), _p(y), _p(sc)))
    return g, y, sc
