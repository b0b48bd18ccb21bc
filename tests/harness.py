"""Shared plumbing of the GPU parity tests: run a workload through the C-ABI binding, run the same
arrays through the oracle, compare.  No arithmetic of the method lives here."""
from __future__ import annotations

import sys

import numpy as np

import workloads as W


class _Oracle:
    """The oracle package, imported on first use: the device-side helpers of this module are also
    used where the oracle must not be loaded."""

    def __getattr__(self, name):
        import oracle as _o
        return getattr(_o, name)


oracle = _Oracle()


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


def torch_dtype(spec_dtype):
    import torch
    return torch.bfloat16 if spec_dtype == "bf16" else torch.float32


def make_config(spec, n_layers=1, causal=False, flags=0):
    import paper_2502_09888_amd as P
    return P.Config(n_layers=n_layers, n_heads=spec.H, d_head=spec.dh, n_scen=spec.n_scen,
                    n_beh=spec.n_beh, sub_len=spec.sub_len,
                    dtype=P.BF16 if spec.dtype == "bf16" else P.F32,
                    flags=(P.HIST_CAUSAL if causal else 0) | flags, qk_scale=spec.qk_scale)


class GpuAttention:
    """Device copies of one attention workload + a KV cache created for it."""

    def __init__(self, w, causal=False, flags=0):
        import torch
        import paper_2502_09888_amd as P
        self.P, self.torch, self.w = P, torch, w
        spec = w["spec"]
        self.spec = spec
        self.cfg = make_config(spec, causal=causal, flags=flags)
        dt = torch_dtype(spec.dtype)
        dev = "cuda:0"
        self.dt = dt
        for n in ("qh", "kh", "vh", "qc", "kc", "vc"):
            setattr(self, n, torch.from_numpy(w[n]).to(dev).to(dt).contiguous())
        for n in ("scen", "beh", "cscen", "cbeh", "cand_off"):
            setattr(self, n, torch.from_numpy(w[n]).to(dev))
        self.tau = torch.from_numpy(w["tau"]).to(dev)
        self.padded = [int(x) for x in np.diff(w["tok_off"])]
        nbytes = P.climber_kv_cache_bytes(self.cfg, self.padded)
        assert nbytes > 0
        self.buf = torch.empty(nbytes, dtype=torch.uint8, device=dev)
        self.cache = P.climber_kv_cache_create(self.cfg, [int(x) for x in w["hist_len"]],
                                               self.padded, self.buf)
        self.d = spec.H * spec.dh

    def history(self, want_output=True):
        t = self.torch
        o = t.full((self.qh.shape[0], self.d), float("nan"), dtype=self.dt, device="cuda:0") \
            if want_output else None
        self.P.climber_attn_history(self.cfg, self.tau, self.qh, self.kh, self.vh, self.scen,
                                    self.beh, self.cache, 0, o)
        t.cuda.synchronize()
        return None if o is None else o.float().cpu().numpy()

    def sumi(self, sel=None):
        """Score all candidates (sel None) or, per user, the candidate sub-range sel=(lo, hi)."""
        t, w = self.torch, self.w
        if sel is None:
            qc, kc, vc, cs, cb, off = self.qc, self.kc, self.vc, self.cscen, self.cbeh, self.cand_off
            off_h = w["cand_off"]
        else:
            idx, cnt = [], []
            for b in range(self.spec.B):
                c0, c1 = int(w["cand_off"][b]), int(w["cand_off"][b + 1])
                lo, hi = min(c0 + sel[0], c1), min(c0 + sel[1], c1)
                idx.extend(range(lo, hi))
                cnt.append(hi - lo)
            self.last_idx = np.array(idx, dtype=np.int64)
            ii = t.from_numpy(self.last_idx).to("cuda:0")
            qc, kc, vc = (x[ii].contiguous() for x in (self.qc, self.kc, self.vc))
            cs, cb = self.cscen[ii].contiguous(), self.cbeh[ii].contiguous()
            off_h = np.concatenate([[0], np.cumsum(cnt)]).astype(np.int32)
            off = t.from_numpy(off_h).to("cuda:0")
        m_total = int(off_h[-1])
        m_max = int(np.diff(off_h).max()) if m_total else 0
        o = t.full((max(m_total, 1), self.d), float("nan"), dtype=self.dt, device="cuda:0")
        self.P.climber_attn_sumi(self.cfg, self.tau, self.cache, 0, qc, kc, vc, off, m_total, m_max,
                                 cs, cb, o)
        t.cuda.synchronize()
        return o[:m_total].float().cpu().numpy()


def oracle_history(w, causal=False):
    s = w["spec"]
    return oracle.attn_history(w["tok_off"], w["hist_len"], w["qh"], w["kh"], w["vh"], w["scen"],
                               w["beh"], w["tau"], s.qk_scale, sub_len=s.sub_len, causal=causal)


def oracle_sumi(w, users=None):
    """Oracle SUMI output for all users or for a list of users (rows concatenated in that order)."""
    s = w["spec"]
    if users is None:
        return oracle.attn_sumi(w["tok_off"], w["hist_len"], w["cand_off"], w["kh"], w["vh"],
                                w["qc"], w["kc"], w["vc"], w["cscen"], w["cbeh"], w["tau"],
                                s.qk_scale)
    outs = []
    for b in users:
        t0, t1 = int(w["tok_off"][b]), int(w["tok_off"][b + 1])
        c0, c1 = int(w["cand_off"][b]), int(w["cand_off"][b + 1])
        outs.append(oracle.attn_sumi([0, t1 - t0], [w["hist_len"][b]], [0, c1 - c0],
                                     w["kh"][t0:t1], w["vh"][t0:t1], w["qc"][c0:c1], w["kc"][c0:c1],
                                     w["vc"][c0:c1], w["cscen"][c0:c1], w["cbeh"][c0:c1], w["tau"],
                                     s.qk_scale))
    return np.concatenate(outs)


def valid_rows(w):
    m = np.zeros(int(w["tok_off"][-1]), bool)
    for b in range(len(w["hist_len"])):
        m[w["tok_off"][b]:w["tok_off"][b] + w["hist_len"][b]] = True
    return m


def max_abs(a, b):
    return float(np.max(np.abs(np.asarray(a, np.float64) - np.asarray(b, np.float64)))) if a.size else 0.0


def decode_bf16_cache(buf, B, tok_off, H, n_layers=1):
    """Turn the bf16 KV cache (the layout documented with the cache geometry of the library: per
    layer and (user, head), blocks of 32 keys = 4 KiB of K operand fragments + 4 KiB of V^T operand
    fragments with the key order inside a 16-key group permuted) back into K, V arrays
    [n_layers, T_pad, H, 64] (float32).  buf: the cache's device buffer as a numpy uint8 array.
    Index arithmetic only."""
    import torch
    T = int(tok_off[-1])
    header = ((3 * B + 1 + T // 64) * 4 + 255) // 256 * 256
    layer_bytes = 2 * T * H * 64 * 2
    K = np.zeros((n_layers, T, H, 64), np.float32)
    V = np.zeros((n_layers, T, H, 64), np.float32)
    for l in range(n_layers):
        raw = buf[header + l * layer_bytes: header + (l + 1) * layer_bytes]
        vals = torch.from_numpy(raw.copy()).view(torch.bfloat16).float().numpy()
        for b in range(B):
            t0, Lpad = int(tok_off[b]), int(tok_off[b + 1] - tok_off[b])
            for h in range(H):
                base = (t0 * H + h * Lpad) * 128          # in bf16 elements: 256 bytes per key
                blocks = vals[base: base + Lpad * 128].reshape(Lpad // 32, 4096)
                # K chunk (s, lane), element e:  K[32kb + lane%32][16s + 8(lane/32) + e]
                kf = blocks[:, :2048].reshape(-1, 4, 2, 32, 8)          # [kb][s][lane/32][lane%32][e]
                K[l, t0:t0 + Lpad, h] = kf.transpose(0, 3, 1, 2, 4).reshape(Lpad, 64)
                # V chunk (g, db, lane), element e:
                #   V[32kb + 16g + 8(e/4) + 4(lane/32) + e%4][32db + lane%32]
                vf = blocks[:, 2048:].reshape(-1, 2, 2, 2, 32, 2, 4)    # [kb][g][db][lane/32][lane%32][e/4][e%4]
                V[l, t0:t0 + Lpad, h] = vf.transpose(0, 1, 5, 3, 6, 2, 4).reshape(Lpad, 64)
    return K, V


# ------------------------------------------------------------------ layer stack
def stack_config(spec, flags=0):
    import paper_2502_09888_amd as P
    return P.Config(n_layers=spec.n_layers, d_model=spec.d_model, n_heads=spec.H, d_head=spec.dh,
                    d_ffn=spec.d_ffn, n_scen=spec.n_scen, n_beh=spec.n_beh, sub_len=spec.sub_len,
                    dtype=P.BF16, flags=(P.HIST_CAUSAL if spec.causal else 0) | flags,
                    qk_scale=spec.qk_scale, rms_eps=spec.rms_eps)


def oracle_stack_config(spec):
    return oracle.StackConfig(spec.n_layers, spec.d_model, spec.H, spec.dh, spec.d_ffn, spec.n_scen,
                              spec.n_beh, sub_len=spec.sub_len, causal=spec.causal,
                              qk_scale=spec.qk_scale, rms_eps=spec.rms_eps)


class GpuStack:
    """Device copies of one full-stack workload, cache and workspace."""

    def __init__(self, w, flags=0):
        import torch
        import paper_2502_09888_amd as P
        self.P, self.torch, self.w = P, torch, w
        spec = w["spec"]
        self.spec, self.cfg = spec, stack_config(spec, flags)
        dev, bf = "cuda:0", torch.bfloat16
        self.layers = [{n.lower(): torch.from_numpy(lw[n]).to(dev).to(bf).contiguous()
                        for n in ("g1", "Wqkv", "Wo", "g2", "W1", "W2")} for lw in w["layers"]]
        self.x_hist = torch.from_numpy(w["x_hist"]).to(dev).to(bf)
        self.x_cand = torch.from_numpy(w["x_cand"]).to(dev).to(bf)
        for n in ("scen", "beh", "cscen", "cbeh", "cand_off"):
            setattr(self, n, torch.from_numpy(w[n]).to(dev))
        self.tau = torch.from_numpy(w["tau"]).to(dev)
        self.padded = [int(x) for x in np.diff(w["tok_off"])]
        self.buf = torch.empty(P.climber_kv_cache_bytes(self.cfg, self.padded), dtype=torch.uint8,
                               device=dev)
        self.cache = P.climber_kv_cache_create(self.cfg, [int(x) for x in w["hist_len"]],
                                               self.padded, self.buf)
        rows = max(int(w["tok_off"][-1]), int(w["cand_off"][-1]))
        self.ws = torch.empty(P.climber_workspace_bytes(self.cfg, rows), dtype=torch.uint8, device=dev)
        self.m_total = int(w["cand_off"][-1])
        self.m_max = int(np.diff(w["cand_off"]).max())

    def encode(self, packed=None):
        self.P.climber_history_encode(self.cfg, self.layers, self.tau, self.x_hist, self.scen,
                                      self.beh, self.cache, self.ws, packed=packed)

    def score(self, packed=None):
        t = self.torch
        y = t.full((self.m_total, self.spec.d_model), float("nan"), dtype=t.float32, device="cuda:0")
        self.P.climber_sumi_score(self.cfg, self.layers, self.tau, self.cache, self.x_cand,
                                  self.cand_off, self.m_total, self.m_max, self.cscen, self.cbeh, y,
                                  self.ws, packed=packed)
        t.cuda.synchronize()
        return y.cpu().numpy()


def oracle_stack_users(w, users):
    """Oracle encode + score for selected users, each on its own.  Returns (y_cand rows
    concatenated in that order, list of per-user y_hist)."""
    spec = w["spec"]
    cfg = oracle_stack_config(spec)
    ys, yhs = [], []
    for b in users:
        t0, t1 = int(w["tok_off"][b]), int(w["tok_off"][b + 1])
        c0, c1 = int(w["cand_off"][b]), int(w["cand_off"][b + 1])
        kc, vc, yh = oracle.stack_encode(cfg, w["layers"], w["tau"], [0, t1 - t0],
                                         [w["hist_len"][b]], w["x_hist"][t0:t1], w["scen"][t0:t1],
                                         w["beh"][t0:t1])
        ys.append(oracle.stack_score(cfg, w["layers"], w["tau"], [0, t1 - t0], [w["hist_len"][b]],
                                     kc, vc, [0, c1 - c0], w["x_cand"][c0:c1], w["cscen"][c0:c1],
                                     w["cbeh"][c0:c1]))
        yhs.append(yh)
    return np.concatenate(ys), yhs
