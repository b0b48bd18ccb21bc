"""ctypes binding of include/climber.h.  Function names equal the C entry points; tensors are
passed as raw device pointers (``tensor.data_ptr()``), streams as ``torch.cuda.Stream`` or None
(= torch's current stream).  No arithmetic happens here."""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libclimber.so")

F32, BF16 = 0, 1
MODE_HISTORY, MODE_CANDIDATE = 0, 1
HIST_CAUSAL, HIST_TWO_KERNEL, QKV_VIA_ROWS = 1, 2, 4


class ClimberError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where}: error {code}: {climber_strerror(code)}")


class Config(C.Structure):
    """Mirror of ``climber_config``."""
    _fields_ = [(n, C.c_int32) for n in ("n_layers", "d_model", "n_heads", "d_head", "d_ffn",
                                         "n_scen", "n_beh", "sub_len", "dtype", "flags")] + \
               [("qk_scale", C.c_float), ("rms_eps", C.c_float)]

    def __init__(self, n_layers=1, d_model=0, n_heads=1, d_head=64, d_ffn=0, n_scen=1, n_beh=1,
                 sub_len=0, dtype=BF16, flags=0, qk_scale=1.0, rms_eps=1e-6):
        super().__init__(n_layers, d_model or n_heads * d_head, n_heads, d_head, d_ffn, n_scen,
                         n_beh, sub_len, dtype, flags, qk_scale, rms_eps)


class LayerWeights(C.Structure):
    """Mirror of ``climber_layer_weights`` (device pointers)."""
    _fields_ = [(n, C.c_void_p) for n in ("g1", "wqkv", "wo", "g2", "w1", "w2")]


class RelBias(C.Structure):
    """Mirror of ``climber_rel_bias`` (device pointers).  Build with ``rel_bias(...)``."""
    _fields_ = [("pos_table", C.c_void_p), ("time_table", C.c_void_p), ("n_pos", C.c_int32),
                ("n_time", C.c_int32), ("hist_pos", C.c_void_p), ("hist_ts", C.c_void_p),
                ("cand_pos", C.c_void_p), ("cand_ts", C.c_void_p)]


class BgfWeights(C.Structure):
    """Mirror of ``climber_bgf_weights``."""
    _fields_ = [("atl", LayerWeights), ("w_down", C.c_void_p), ("w_up", C.c_void_p), ("w_head", C.c_void_p),
                ("tau_scen", C.c_void_p), ("b_head", C.c_float), ("n_blocks", C.c_int32), ("d_gate", C.c_int32)]


class _Weights(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("layers", C.POINTER(LayerWeights)), ("packed", C.c_void_p)]


_lib = None


def library_path() -> str:
    return _LIB_PATH


def load_library():
    """Load libclimber.so; raises if it has not been built (no fallback exists)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise ImportError(f"{_LIB_PATH} is missing: build it with `python -m paper_2502_09888_amd.build`"
                          " (there is no CPU fallback)")
    lib = C.CDLL(_LIB_PATH)
    vp, i32, i64, sz = C.c_void_p, C.c_int32, C.c_int64, C.c_size_t
    cfgp = C.POINTER(Config)
    lib.climber_strerror.restype = C.c_char_p
    lib.climber_strerror.argtypes = [C.c_int]
    lib.climber_kv_cache_bytes.restype = sz
    lib.climber_kv_cache_bytes.argtypes = [cfgp, i32, C.POINTER(i32)]
    lib.climber_kv_cache_create.restype = C.c_int
    lib.climber_kv_cache_create.argtypes = [cfgp, i32, C.POINTER(i32), C.POINTER(i32), vp, sz,
                                            C.POINTER(vp)]
    lib.climber_kv_cache_destroy.restype = C.c_int
    lib.climber_kv_cache_destroy.argtypes = [vp]
    lib.climber_kv_cache_rows.restype = i64
    lib.climber_kv_cache_rows.argtypes = [vp]
    lib.climber_attn_history.restype = C.c_int
    lib.climber_attn_history.argtypes = [cfgp, vp, vp, vp, vp, vp, vp, vp, i32, vp, vp]
    lib.climber_attn_sumi.restype = C.c_int
    lib.climber_attn_sumi.argtypes = [cfgp, vp, vp, i32, vp, vp, vp, vp, i32, i32, vp, vp, vp, vp]
    lib.climber_attn_history_bias.restype = C.c_int
    lib.climber_attn_history_bias.argtypes = [cfgp, vp, vp, vp, vp, vp, vp, vp, i32, vp, C.POINTER(RelBias), vp]
    lib.climber_attn_sumi_bias.restype = C.c_int
    lib.climber_attn_sumi_bias.argtypes = [cfgp, vp, vp, i32, vp, vp, vp, vp, i32, i32, vp, vp, vp,
                                           C.POINTER(RelBias), vp]
    lib.climber_check_inputs.restype = C.c_int
    lib.climber_check_inputs.argtypes = [cfgp, vp, vp, vp, vp, i32, vp, i32, i32, vp, vp]
    lib.climber_workspace_bytes.restype = sz
    lib.climber_workspace_bytes.argtypes = [cfgp, i64]
    lib.climber_packed_weights_bytes.restype = sz
    lib.climber_packed_weights_bytes.argtypes = [cfgp]
    lib.climber_pack_weights.restype = C.c_int
    lib.climber_pack_weights.argtypes = [cfgp, C.POINTER(_Weights), vp, sz, vp]
    lib.climber_layer_forward.restype = C.c_int
    lib.climber_layer_forward.argtypes = [cfgp, C.POINTER(LayerWeights), vp, i32, i32, vp, vp, vp,
                                          vp, vp, vp, i32, i32, vp, sz, vp]
    lib.climber_history_encode.restype = C.c_int
    lib.climber_history_encode.argtypes = [cfgp, C.POINTER(_Weights), vp, vp, vp, vp, vp, vp, sz,
                                           vp]
    lib.climber_sumi_score.restype = C.c_int
    lib.climber_sumi_score.argtypes = [cfgp, C.POINTER(_Weights), vp, vp, vp, vp, i32, i32, vp,
                                       vp, vp, vp, sz, vp]
    lib.climber_bgf_workspace_bytes.restype = sz
    lib.climber_bgf_workspace_bytes.argtypes = [cfgp, i32, i32, i64]
    lib.climber_bgf_score.restype = C.c_int
    lib.climber_bgf_score.argtypes = [cfgp, C.POINTER(BgfWeights), vp, vp, i32, vp, vp, vp, sz, vp]
    lib.climber_sumi_forward.restype = C.c_int
    lib.climber_sumi_forward.argtypes = [cfgp, C.POINTER(_Weights), vp, vp, vp, vp, vp, vp, i32, i32, vp, vp,
                                         vp, vp, vp, vp, sz, vp]
    lib.climber_sumi_score_static.restype = C.c_int
    lib.climber_sumi_score_static.argtypes = [cfgp, C.POINTER(_Weights), vp, vp, vp, vp, i32, i32, vp,
                                              vp, vp, vp]
    _lib = lib
    return lib


def _ptr(t) -> Optional[int]:
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return t.data_ptr()


def _stream(stream) -> Optional[int]:
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream or None
    if isinstance(stream, int):
        return stream or None
    return stream.cuda_stream or None


def _i32arr(xs: Sequence[int]):
    return (C.c_int32 * len(xs))(*[int(x) for x in xs])


def _ok(code: int, where: str):
    if code != 0:
        raise ClimberError(code, where)


def climber_strerror(code: int) -> str:
    return load_library().climber_strerror(int(code)).decode()


def climber_kv_cache_bytes(cfg: Config, hist_len_padded: Sequence[int]) -> int:
    return int(load_library().climber_kv_cache_bytes(C.byref(cfg), len(hist_len_padded),
                                                     _i32arr(hist_len_padded)))


class KVCache:
    """Owner of a ``climber_kv_cache`` handle (the device buffer stays with the caller)."""

    def __init__(self, handle: int, dev_buf):
        self.handle = handle
        self.dev_buf = dev_buf  # keeps the tensor alive

    def __del__(self):
        try:
            climber_kv_cache_destroy(self)
        except Exception:
            pass


def climber_kv_cache_create(cfg: Config, hist_len: Sequence[int], hist_len_padded: Sequence[int],
                            dev_buf, nbytes: Optional[int] = None) -> KVCache:
    B = len(hist_len)
    if len(hist_len_padded) != B:
        raise ValueError("hist_len and hist_len_padded differ in length")
    if nbytes is None:
        nbytes = dev_buf.numel() * dev_buf.element_size()
    out = C.c_void_p()
    _ok(load_library().climber_kv_cache_create(C.byref(cfg), B, _i32arr(hist_len),
                                               _i32arr(hist_len_padded), _ptr(dev_buf), nbytes,
                                               C.byref(out)), "climber_kv_cache_create")
    return KVCache(out.value, dev_buf)


def climber_kv_cache_destroy(cache: KVCache) -> None:
    if cache.handle:
        load_library().climber_kv_cache_destroy(cache.handle)
        cache.handle = None


def climber_kv_cache_rows(cache: KVCache) -> int:
    return int(load_library().climber_kv_cache_rows(cache.handle))


def climber_attn_history(cfg: Config, tau_layer, q, k, v, scen, beh, cache: KVCache, layer: int,
                         o_hist=None, stream=None) -> None:
    _ok(load_library().climber_attn_history(C.byref(cfg), _ptr(tau_layer), _ptr(q), _ptr(k),
                                            _ptr(v), _ptr(scen), _ptr(beh), cache.handle, layer,
                                            _ptr(o_hist), _stream(stream)), "climber_attn_history")


def climber_attn_sumi(cfg: Config, tau_layer, cache: KVCache, layer: int, q_c, k_c, v_c, cand_off,
                      m_total: int, m_max: int, cand_scen, cand_beh, o_c, stream=None) -> None:
    _ok(load_library().climber_attn_sumi(C.byref(cfg), _ptr(tau_layer), cache.handle, layer,
                                         _ptr(q_c), _ptr(k_c), _ptr(v_c), _ptr(cand_off), m_total,
                                         m_max, _ptr(cand_scen), _ptr(cand_beh), _ptr(o_c),
                                         _stream(stream)), "climber_attn_sumi")


BAD_SCEN, BAD_BEH, BAD_TAU, BAD_OFFSETS, BAD_M_MAX = 1, 2, 4, 8, 16


def climber_check_inputs(cfg: Config, tau_layer, scen, beh, cache: Optional[KVCache], m_total: int,
                         cand_off, B_cand: int, m_max: int, status, stream=None) -> None:
    """Device-side check of ids / offsets / temperatures; ORs BAD_* bits into status (int32 tensor)."""
    _ok(load_library().climber_check_inputs(C.byref(cfg), _ptr(tau_layer), _ptr(scen), _ptr(beh),
                                            cache.handle if cache is not None else None, m_total,
                                            _ptr(cand_off), B_cand, m_max, _ptr(status),
                                            _stream(stream)), "climber_check_inputs")


def climber_workspace_bytes(cfg: Config, max_rows: int) -> int:
    return int(load_library().climber_workspace_bytes(C.byref(cfg), max_rows))


def _layer_struct(lw) -> LayerWeights:
    if isinstance(lw, LayerWeights):
        return lw
    return LayerWeights(*[_ptr(lw[n]) for n in ("g1", "wqkv", "wo", "g2", "w1", "w2")])


def _weights_struct(layers, packed=None):
    arr = (LayerWeights * len(layers))(*[_layer_struct(l) for l in layers])
    return _Weights(len(layers), arr, _ptr(packed)), arr


def climber_packed_weights_bytes(cfg: Config) -> int:
    return int(load_library().climber_packed_weights_bytes(C.byref(cfg)))


def climber_pack_weights(cfg: Config, layers, packed, stream=None) -> None:
    """Bring the weights into the form the projections read, once; pass the buffer as `packed` to
    climber_history_encode / climber_sumi_score."""
    w, keep = _weights_struct(layers)
    _ok(load_library().climber_pack_weights(C.byref(cfg), C.byref(w), _ptr(packed),
                                            packed.numel() * packed.element_size(), _stream(stream)),
        "climber_pack_weights")


def climber_layer_forward(cfg: Config, layer_weights, tau_layer, layer: int, mode: int,
                          cache: KVCache, x_in, x_out, scen, beh, cand_off, m_total: int,
                          m_max: int, workspace, stream=None) -> None:
    lw = _layer_struct(layer_weights)
    _ok(load_library().climber_layer_forward(
        C.byref(cfg), C.byref(lw), _ptr(tau_layer), layer, mode, cache.handle, _ptr(x_in),
        _ptr(x_out), _ptr(scen), _ptr(beh), _ptr(cand_off), m_total, m_max, _ptr(workspace),
        workspace.numel() * workspace.element_size(), _stream(stream)), "climber_layer_forward")


def climber_history_encode(cfg: Config, layers, tau, x_hist, scen, beh, cache: KVCache, workspace,
                           stream=None, packed=None) -> None:
    w, keep = _weights_struct(layers, packed)
    _ok(load_library().climber_history_encode(
        C.byref(cfg), C.byref(w), _ptr(tau), _ptr(x_hist), _ptr(scen), _ptr(beh), cache.handle,
        _ptr(workspace), workspace.numel() * workspace.element_size(), _stream(stream)),
        "climber_history_encode")


def climber_sumi_score(cfg: Config, layers, tau, cache: KVCache, x_cand, cand_off, m_total: int,
                       m_max: int, cand_scen, cand_beh, y_cand, workspace, stream=None, packed=None) -> None:
    w, keep = _weights_struct(layers, packed)
    _ok(load_library().climber_sumi_score(
        C.byref(cfg), C.byref(w), _ptr(tau), cache.handle, _ptr(x_cand), _ptr(cand_off), m_total,
        m_max, _ptr(cand_scen), _ptr(cand_beh), _ptr(y_cand), _ptr(workspace),
        workspace.numel() * workspace.element_size(), _stream(stream)), "climber_sumi_score")


STATIC_SCRATCH_BYTES = 32 << 20


def climber_sumi_score_static(cfg: Config, layers, tau, cache: KVCache, x_cand, cand_off, m_total: int,
                              m_max: int, cand_scen, cand_beh, y_cand, packed, stream=None) -> None:
    """climber_sumi_score with the scratch in the library's fixed per-GPU array (allocates nothing)."""
    w, keep = _weights_struct(layers if layers is not None else [], packed)
    w.n_layers = cfg.n_layers
    _ok(load_library().climber_sumi_score_static(
        C.byref(cfg), C.byref(w), _ptr(tau), cache.handle, _ptr(x_cand), _ptr(cand_off), m_total,
        m_max, _ptr(cand_scen), _ptr(cand_beh), _ptr(y_cand), _stream(stream)),
        "climber_sumi_score_static")


def rel_bias(pos_table, time_table, hist_pos, hist_ts, cand_pos=None, cand_ts=None) -> RelBias:
    """climber_rel_bias from device tensors: tables [n_scen, n_beh, H, n_pos] / [..., n_time] fp32."""
    rb = RelBias(_ptr(pos_table), _ptr(time_table), int(pos_table.shape[-1]), int(time_table.shape[-1]),
                 _ptr(hist_pos), _ptr(hist_ts), _ptr(cand_pos), _ptr(cand_ts))
    rb._keep = (pos_table, time_table, hist_pos, hist_ts, cand_pos, cand_ts)
    return rb


def climber_attn_history_bias(cfg: Config, tau_layer, q, k, v, scen, beh, cache: KVCache, layer: int,
                              o_hist, bias: RelBias, stream=None) -> None:
    _ok(load_library().climber_attn_history_bias(C.byref(cfg), _ptr(tau_layer), _ptr(q), _ptr(k), _ptr(v),
                                                 _ptr(scen), _ptr(beh), cache.handle, layer, _ptr(o_hist),
                                                 C.byref(bias), _stream(stream)), "climber_attn_history_bias")


def climber_attn_sumi_bias(cfg: Config, tau_layer, cache: KVCache, layer: int, q_c, k_c, v_c, cand_off,
                           m_total: int, m_max: int, cand_scen, cand_beh, o_c, bias: RelBias,
                           stream=None) -> None:
    _ok(load_library().climber_attn_sumi_bias(C.byref(cfg), _ptr(tau_layer), cache.handle, layer, _ptr(q_c),
                                              _ptr(k_c), _ptr(v_c), _ptr(cand_off), m_total, m_max,
                                              _ptr(cand_scen), _ptr(cand_beh), _ptr(o_c), C.byref(bias),
                                              _stream(stream)), "climber_attn_sumi_bias")


def climber_sumi_forward(cfg: Config, layers, tau, x_hist, scen, beh, x_cand, cand_off, m_total: int,
                         m_max: int, cand_scen, cand_beh, scratch_cache: KVCache, y_hist, y_cand, workspace,
                         stream=None, packed=None) -> None:
    """Training-side packed forward: histories and candidates together, no cache kept."""
    w, keep = _weights_struct(layers, packed)
    _ok(load_library().climber_sumi_forward(
        C.byref(cfg), C.byref(w), _ptr(tau), _ptr(x_hist), _ptr(scen), _ptr(beh), _ptr(x_cand),
        _ptr(cand_off), m_total, m_max, _ptr(cand_scen), _ptr(cand_beh), scratch_cache.handle,
        _ptr(y_hist), _ptr(y_cand), _ptr(workspace), workspace.numel() * workspace.element_size(),
        _stream(stream)), "climber_sumi_forward")


def climber_bgf_workspace_bytes(cfg: Config, n_blocks: int, d_gate: int, m_total: int) -> int:
    return int(load_library().climber_bgf_workspace_bytes(C.byref(cfg), n_blocks, d_gate, m_total))


def climber_bgf_score(cfg: Config, atl_layer, w_down, w_up, w_head, tau_scen, b_head: float, n_blocks: int,
                      d_gate: int, e, cand_scen, m_total: int, y, score, workspace, stream=None) -> None:
    """Bit-wise gating fusion (Eq. (4)) + linear head over the candidates' block outputs e."""
    w = BgfWeights(_layer_struct(atl_layer), _ptr(w_down), _ptr(w_up), _ptr(w_head), _ptr(tau_scen), b_head,
                   n_blocks, d_gate)
    _ok(load_library().climber_bgf_score(C.byref(cfg), C.byref(w), _ptr(e), _ptr(cand_scen), m_total, _ptr(y),
                                         _ptr(score), _ptr(workspace), workspace.numel() * workspace.element_size(),
                                         _stream(stream)), "climber_bgf_score")
