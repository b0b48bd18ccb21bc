"""Host-side checks that need no GPU: the built library exports every entry point the header
declares, and argument validation rejects bad calls before anything would be launched."""
import ctypes as C
import os
import re

import pytest

import paper_2502_09888_amd as P
from paper_2502_09888_amd import build as hip_build

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE = 0x7F0000000000  # 256-byte aligned, never dereferenced on the host


@pytest.fixture(scope="module", autouse=True)
def _lib():
    if not os.path.exists(P.library_path()):
        hip_build.build()
    return P.load_library()


def declared_functions():
    text = open(os.path.join(ROOT, "include", "climber.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(climber_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(_lib):
    names = declared_functions()
    assert {"climber_history_encode", "climber_sumi_score", "climber_layer_forward",
            "climber_attn_sumi", "climber_attn_history", "climber_kv_cache_create"} <= set(names)
    for n in names:
        assert hasattr(_lib, n), n
    # the Python binding carries the same names
    for n in names:
        assert hasattr(P, n), n


def cfg(**kw):
    base = dict(n_layers=1, n_heads=4, d_head=64, n_scen=8, n_beh=4, sub_len=128, dtype=P.BF16,
                qk_scale=0.125)
    base.update(kw)
    return P.Config(**base)


def create(c, hist_len, padded, buf=FAKE, nbytes=1 << 40):
    out = C.c_void_p()
    arr = lambda xs: (C.c_int32 * len(xs))(*xs)
    rc = P.load_library().climber_kv_cache_create(C.byref(c), len(hist_len), arr(hist_len),
                                                  arr(padded), buf, nbytes, C.byref(out))
    assert rc != 0 and not out.value
    return rc


def test_strerror_names_every_code():
    seen = {P.climber_strerror(c) for c in range(0, -9, -1)}
    assert len(seen) == 9 and "unknown" not in " ".join(seen)
    assert "unknown" in P.climber_strerror(-99)


def test_cache_bytes():
    c = cfg()
    # header (lengths, offsets, order: 3 B + 1 words; the user of every 64 rows: rows / 64 words;
    # rounded up to 256 bytes) + 2 (K,V) * rows * d_model * 2 bytes
    assert P.climber_kv_cache_bytes(c, [512] * 32) == 1536 + 2 * 32 * 512 * 256 * 2
    assert P.climber_kv_cache_bytes(c, [100]) == 0            # bf16 padding rule
    assert P.climber_kv_cache_bytes(cfg(d_head=32), [128]) == 0
    assert P.climber_kv_cache_bytes(cfg(dtype=P.F32, d_head=32, sub_len=7), [100]) > 0


def test_create_rejects_bad_arguments():
    assert create(cfg(qk_scale=0.0), [64], [64]) == -5
    assert create(cfg(qk_scale=float("nan")), [64], [64]) == -5
    assert create(cfg(d_head=32), [64], [64]) == -7           # bf16 path needs d_head 64
    assert create(cfg(flags=8), [64], [64]) == -2             # unknown flag bit
    assert create(cfg(sub_len=96), [64], [64]) == -3
    assert create(cfg(d_model=100), [64], [64]) == -2
    assert create(cfg(n_scen=0), [64], [64]) == -2
    assert create(cfg(), [64], [100]) == -3                   # padding not a multiple of 64
    assert create(cfg(), [65], [64]) == -4                    # valid length beyond padding
    assert create(cfg(), [-1], [64]) == -4
    assert create(cfg(), [64], [64], buf=None) == -1
    assert create(cfg(), [64], [64], buf=FAKE + 8) == -3
    assert create(cfg(), [64], [64], nbytes=1024) == -6
    assert create(cfg(dtype=P.F32, d_head=300, sub_len=0), [64], [64]) == -7
    assert create(cfg(dtype=P.F32, d_head=32, sub_len=0), [20000], [20000]) == -7


def test_compute_calls_reject_missing_cache_and_pointers():
    lib = P.load_library()
    c = cfg()
    assert lib.climber_attn_sumi(C.byref(c), FAKE, None, 0, FAKE, FAKE, FAKE, FAKE, 8, 8, FAKE, FAKE,
                                 FAKE, None) == -1
    assert lib.climber_attn_history(C.byref(c), FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, None, 0, FAKE,
                                    None) == -1
    assert lib.climber_attn_sumi(None, FAKE, None, 0, FAKE, FAKE, FAKE, FAKE, 8, 8, FAKE, FAKE, FAKE,
                                 None) == -1
    # the stack calls that need a cache handle: none given
    from paper_2502_09888_amd.climber import _Weights
    c4 = P.Config(n_layers=4, n_heads=8, d_head=64, d_ffn=2048, n_scen=8, n_beh=4, sub_len=256)
    w = _Weights(4, None, FAKE)
    assert lib.climber_sumi_forward(C.byref(c4), C.byref(w), FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, 8, 8, FAKE, FAKE,
                                    None, None, FAKE, FAKE, 1 << 40, None) == -1
    assert lib.climber_sumi_score_static(C.byref(c4), C.byref(w), FAKE, None, FAKE, FAKE, 8, 8, FAKE, FAKE, FAKE,
                                         None) == -1
    assert lib.climber_history_encode(C.byref(c4), C.byref(w), FAKE, FAKE, FAKE, FAKE, None, FAKE, 1 << 40,
                                      None) == -1


def test_check_inputs_rejects_bad_arguments():
    lib = P.load_library()
    c = cfg()
    f = lambda *a: lib.climber_check_inputs(*a)
    assert f(C.byref(c), None, FAKE, FAKE, None, 8, FAKE, 2, 8, FAKE, None) == -1
    assert f(C.byref(c), FAKE, FAKE, FAKE, None, 8, FAKE, 2, 8, None, None) == -1
    assert f(C.byref(c), FAKE, FAKE, FAKE, None, -1, FAKE, 2, 8, FAKE, None) == -2
    assert f(C.byref(c), FAKE, FAKE, FAKE, None, 8, FAKE, 0, 8, FAKE, None) == -2
    assert f(None, FAKE, FAKE, FAKE, None, 8, FAKE, 2, 8, FAKE, None) == -1


def test_workspace_bytes():
    c4 = P.Config(n_layers=4, n_heads=8, d_head=64, d_ffn=2048, n_scen=8, n_beh=4, sub_len=256)
    n = 32768
    need = n * 512 * (4 + 4 + 2 + 6 + 2) + n * 8 * 4 + n * 2048 * 2 + 4 * 2 * (4 * 512 * 512 + 2 * 512 * 2048)
    got = P.climber_workspace_bytes(c4, n)
    assert need <= got <= need + 8 * 256
    assert P.climber_workspace_bytes(cfg(dtype=P.F32, d_head=32, sub_len=0), 10) == 0
    assert P.climber_workspace_bytes(P.Config(n_heads=8, d_head=64, d_ffn=100), 10) == 0
    assert P.climber_workspace_bytes(P.Config(n_heads=8, d_head=64, d_ffn=256, rms_eps=0.0), 10) == 0


def test_packed_weights_arguments():
    lib = P.load_library()
    c4 = P.Config(n_layers=4, n_heads=8, d_head=64, d_ffn=2048, n_scen=8, n_beh=4, sub_len=256)
    per_layer = 2 * (4 * 512 * 512 + 2 * 512 * 2048)
    assert P.climber_packed_weights_bytes(c4) == 4 * per_layer
    assert P.climber_packed_weights_bytes(cfg(dtype=P.F32, d_head=32, sub_len=0)) == 0
    from paper_2502_09888_amd.climber import LayerWeights, _Weights
    layers = (LayerWeights * 4)(*[LayerWeights(*([FAKE] * 6)) for _ in range(4)])
    w = _Weights(4, layers, None)
    pack = lambda wts, buf, n: lib.climber_pack_weights(C.byref(c4), C.byref(wts) if wts else None, buf, n, None)
    assert pack(None, FAKE, 1 << 40) == -1
    assert pack(w, None, 1 << 40) == -1
    assert pack(_Weights(4, None, None), FAKE, 1 << 40) == -1
    assert pack(_Weights(3, layers, None), FAKE, 1 << 40) == -2
    assert pack(w, FAKE + 16, 1 << 40) == -3
    assert pack(w, FAKE, 4 * per_layer - 1) == -6
    bad = (LayerWeights * 4)(*[LayerWeights(*([FAKE] * 5 + [None])) for _ in range(4)])
    assert pack(_Weights(4, bad, None), FAKE, 1 << 40) == -1
    # a stack call given a misaligned packed buffer is rejected before anything is launched
    assert lib.climber_sumi_score(C.byref(c4), C.byref(_Weights(4, None, FAKE + 16)), FAKE, None, FAKE, FAKE,
                                  8, 8, FAKE, FAKE, FAKE, FAKE, 1 << 40, None) in (-1, -3)


def test_fusion_module_arguments():
    # bit-wise gating fusion: sizes and pointers are checked on the host before anything is launched
    lib = P.load_library()
    from paper_2502_09888_amd.climber import BgfWeights, LayerWeights
    c = P.Config(n_layers=1, n_heads=8, d_head=64, d_ffn=2048, n_scen=8, n_beh=4, sub_len=0)
    assert P.climber_bgf_workspace_bytes(c, 4, 256, 1000) > 0
    assert P.climber_bgf_workspace_bytes(c, 0, 256, 1000) == 0          # no blocks
    assert P.climber_bgf_workspace_bytes(c, 17, 256, 1000) == 0         # more blocks than the kernel holds
    assert P.climber_bgf_workspace_bytes(c, 4, 200, 1000) == 0          # d_gate not a multiple of 128
    assert P.climber_bgf_workspace_bytes(c, 1, 640, 1000) == 0          # d_gate beyond n_blocks * d_model
    assert P.climber_bgf_workspace_bytes(c, 4, 256, -1) == 0
    assert P.climber_bgf_workspace_bytes(cfg(dtype=P.F32, d_head=32, sub_len=0), 4, 256, 10) == 0
    layer = LayerWeights(*([FAKE] * 6))
    def score(w, e=FAKE, scen=FAKE, m=8, y=FAKE, sc=FAKE, ws=FAKE, nbytes=1 << 40):
        return lib.climber_bgf_score(C.byref(c), C.byref(w) if w else None, e, scen, m, y, sc, ws, nbytes, None)
    good = lambda **kw: BgfWeights(**{**dict(atl=layer, w_down=FAKE, w_up=FAKE, w_head=FAKE, tau_scen=FAKE, b_head=0.0,
                                             n_blocks=4, d_gate=256), **kw})
    assert score(None) == -1
    assert score(good(w_head=None)) == -1 and score(good(tau_scen=None)) == -1
    assert score(good(atl=LayerWeights(*([FAKE] * 5 + [None])))) == -1
    assert score(good(), e=None) == -1 and score(good(), sc=None) == -1 and score(good(), ws=None) == -1
    assert score(good(n_blocks=0)) == -2 and score(good(d_gate=200)) == -7
    assert score(good(), m=-1) == -2
    assert score(good(), ws=FAKE + 16) == -3 and score(good(w_head=FAKE + 4)) == -3 and score(good(), y=FAKE + 8) == -3
    assert score(good(), nbytes=1024) == -6


def test_binding_has_no_cpu_fallback(monkeypatch, tmp_path):
    # a missing library must fail loudly, not route anywhere else
    from paper_2502_09888_amd import climber as mod
    monkeypatch.setattr(mod, "_lib", None)
    monkeypatch.setattr(mod, "_LIB_PATH", str(tmp_path / "nope.so"))
    with pytest.raises(ImportError):
        mod.load_library()


def test_bench_refuses_more_than_one_gpu():
    # one GPU per box: the benchmark says so instead of pretending to scale
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=300)
    assert r.returncode != 0 and "ONE GPU" in (r.stderr + r.stdout)
