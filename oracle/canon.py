"""ctypes front end of sharpv_canon.c (the float32 canonical-order checker).

TEST INFRASTRUCTURE ONLY: imported by tests/, the smoke check and the benchmark's CPU
baseline leg; never by the product path.  `build()` compiles the C file with gcc into
oracle/libsharpv_canon.so; `lib()` loads it (building it first if it is missing).
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import Dict, Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "sharpv_canon.c")
_SO = os.path.join(_HERE, "libsharpv_canon.so")
_lib: Optional[C.CDLL] = None


def build(force: bool = True) -> str:
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-ffp-contract=off", "-fopenmp", "-fPIC", "-shared", "-std=c11",
               "-Wall", "-o", _SO, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _SO


def lib() -> C.CDLL:
    global _lib
    if _lib is None:
        build(force=False)
        L = C.CDLL(_SO)
        fp, ip, vp = C.POINTER(C.c_float), C.POINTER(C.c_int32), C.c_void_p
        L.sharpv_canon_threads.restype = C.c_int
        L.sharpv_canon_threads.argtypes = []
        L.sharpv_canon_set_threads.restype = None
        L.sharpv_canon_set_threads.argtypes = [C.c_int]
        L.sharpv_canon_rowdot.restype = C.c_float
        L.sharpv_canon_rowdot.argtypes = [fp, fp, C.c_int]
        L.sharpv_canon_sum32.restype = C.c_float
        L.sharpv_canon_sum32.argtypes = [fp, C.c_int]
        L.sharpv_canon_colmean.restype = None
        L.sharpv_canon_colmean.argtypes = [fp, C.c_int, C.c_int, fp]
        L.sharpv_canon_cos.restype = C.c_float
        L.sharpv_canon_cos.argtypes = [C.c_float] * 3
        L.sharpv_canon_dissim.restype = C.c_float
        L.sharpv_canon_dissim.argtypes = [C.c_float] * 3
        L.sharpv_canon_prune_tokens.restype = C.c_long
        L.sharpv_canon_one_minus_cos.restype = C.c_float
        L.sharpv_canon_one_minus_cos.argtypes = [C.c_float] * 3
        L.sharpv_canon_prune_tokens.argtypes = [vp, C.c_int, ip, C.c_int, C.c_int, C.c_int, C.c_float, C.c_int,
                                                C.c_float, C.c_int, C.c_int, fp, fp, fp, fp, ip, ip, ip, vp]
        L.sharpv_canon_prune_kv.restype = C.c_long
        L.sharpv_canon_prune_kv.argtypes = [vp, vp, vp, vp, C.c_int, ip, ip, ip, C.c_int, C.c_int, C.c_int, C.c_int,
                                            C.c_float, C.c_int, fp, fp, ip, ip, vp, vp]
        L.sharpv_canon_prune_kv_mapped.restype = C.c_long
        L.sharpv_canon_prune_kv_mapped.argtypes = [vp, vp, ip, vp, vp, C.c_int, ip, C.c_int, C.c_int, C.c_int,
                                                   C.c_int, C.c_int, C.c_float, fp, ip, ip, ip, vp, vp]
        L.sharpv_canon_rope_reencode.restype = C.c_int
        L.sharpv_canon_rope_reencode.argtypes = [vp, C.c_int, ip, C.c_long, ip, C.c_int, C.c_int, C.c_int, fp, fp,
                                                 C.c_int, C.c_int]
        _lib = L
    return _lib


def _fp(a: np.ndarray):
    return a.ctypes.data_as(C.POINTER(C.c_float))


def _ip(a: np.ndarray):
    return a.ctypes.data_as(C.POINTER(C.c_int32))


def _vp(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def threads() -> int:
    return int(lib().sharpv_canon_threads())


def set_threads(n: int) -> None:
    lib().sharpv_canon_set_threads(int(n))


def rowdot(x: np.ndarray, y: np.ndarray) -> float:
    x = np.ascontiguousarray(x, np.float32)
    y = np.ascontiguousarray(y, np.float32)
    return float(lib().sharpv_canon_rowdot(_fp(x), _fp(y), x.shape[0]))


def sum32(v: np.ndarray) -> float:
    v = np.ascontiguousarray(v, np.float32)
    return float(lib().sharpv_canon_sum32(_fp(v), v.shape[0]))


def colmean(frame: np.ndarray) -> np.ndarray:
    frame = np.ascontiguousarray(frame, np.float32)
    out = np.empty(frame.shape[1], np.float32)
    lib().sharpv_canon_colmean(_fp(frame), frame.shape[0], frame.shape[1], _fp(out))
    return out


def cos(xy: float, xx: float, yy: float) -> float:
    return float(lib().sharpv_canon_cos(xy, xx, yy))


def dissim(xy: float, xx: float, yy: float) -> float:
    return float(lib().sharpv_canon_dissim(xy, xx, yy))


def _storage(a: np.ndarray, dtype: int) -> np.ndarray:
    return np.ascontiguousarray(a, np.float32 if dtype == 0 else np.uint16)


def prune_tokens(feats: np.ndarray, dtype: int, frame_offsets: np.ndarray, w: float = 1.0, mode: int = 0,
                 K: float = 1.6, min_keep: int = 0, measure: int = 0) -> Dict[str, np.ndarray]:
    feats = _storage(feats, dtype)
    n_total, f, d = feats.shape
    fo = np.ascontiguousarray(frame_offsets, np.int32)
    assert int(fo[-1]) == n_total
    S = np.empty((n_total, f), np.float32)
    T = np.empty_like(S)
    I = np.empty_like(S)
    ratio = np.empty(n_total, np.float32)
    counts = np.empty(n_total, np.int32)
    offsets = np.empty(n_total + 1, np.int32)
    idx = np.empty(n_total * f, np.int32)
    out = np.empty((n_total * f, d), feats.dtype)
    tot = lib().sharpv_canon_prune_tokens(_vp(feats), dtype, _ip(fo), len(fo) - 1, f, d, w, mode, K, min_keep,
                                          measure, _fp(S), _fp(T), _fp(I), _fp(ratio), _ip(counts), _ip(offsets),
                                          _ip(idx), _vp(out))
    if tot < 0:
        raise ValueError("sharpv_canon_prune_tokens: bad argument")
    return {"S": S, "T": T, "I": I, "ratio": ratio, "counts": counts, "offsets": offsets,
            "idx": idx[:tot].copy(), "out_feats": out[:tot].copy()}


def prune_kv(hidden: np.ndarray, orig: np.ndarray, Kc: Optional[np.ndarray], Vc: Optional[np.ndarray], dtype: int,
             seq_offsets: np.ndarray, vis_start: np.ndarray, vis_offsets: np.ndarray, M: float = 0.2,
             kv_mode: int = 0) -> Dict[str, np.ndarray]:
    hidden = _storage(hidden, dtype)
    orig = _storage(orig, dtype)
    so = np.ascontiguousarray(seq_offsets, np.int32)
    vs = np.ascontiguousarray(vis_start, np.int32)
    vo = np.ascontiguousarray(vis_offsets, np.int32)
    B = len(vs)
    S_total, d = hidden.shape
    assert int(so[-1]) == S_total and int(vo[-1]) == orig.shape[0]
    have_kv = Kc is not None and Vc is not None
    H = D = 0
    K_out = V_out = None
    if have_kv:
        Kc = _storage(Kc, dtype)
        Vc = _storage(Vc, dtype)
        H, _, D = Kc.shape
        K_out = np.empty_like(Kc)
        V_out = np.empty_like(Vc)
    cosv = np.empty(orig.shape[0], np.float32)
    mean_cos = np.empty(B, np.float32)
    idx = np.empty(S_total, np.int32)
    cnt = np.empty(B, np.int32)
    tot = lib().sharpv_canon_prune_kv(_vp(hidden), _vp(orig), _vp(Kc), _vp(Vc), dtype, _ip(so), _ip(vs), _ip(vo),
                                      B, d, H, D, M, kv_mode, _fp(cosv), _fp(mean_cos), _ip(idx), _ip(cnt),
                                      _vp(K_out), _vp(V_out))
    if tot < 0:
        raise ValueError("sharpv_canon_prune_kv: bad argument")
    res = {"cos": cosv, "mean_cos": mean_cos, "idx": idx[:tot].copy(), "counts": cnt}
    if have_kv:
        res["K_out"] = K_out.reshape(-1)[:H * tot * D].reshape(H, tot, D).copy()
        res["V_out"] = V_out.reshape(-1)[:H * tot * D].reshape(H, tot, D).copy()
    return res


def rope_reencode(K_kept: np.ndarray, dtype: int, idx: np.ndarray, seq_offsets: np.ndarray,
                  cos_tab: np.ndarray, sin_tab: np.ndarray, layout: int = 0) -> np.ndarray:
    """Float32 rotary re-encoding of the kept K rows [H, S_kept, D]; returns a new storage array."""
    K = _storage(K_kept, dtype).copy()
    H, n_kept, D = K.shape
    ct = np.ascontiguousarray(cos_tab, np.float32)
    st = np.ascontiguousarray(sin_tab, np.float32)
    assert ct.shape == st.shape and ct.shape[1] == D // 2
    so = np.ascontiguousarray(seq_offsets, np.int32)
    ix = np.ascontiguousarray(idx, np.int32)
    assert len(ix) == n_kept
    rc = lib().sharpv_canon_rope_reencode(_vp(K), dtype, _ip(ix), n_kept, _ip(so), len(so) - 1, H, D,
                                          _fp(ct), _fp(st), ct.shape[0], layout)
    if rc != 0:
        raise ValueError("sharpv_canon_rope_reencode: bad argument or table too short")
    return K


def prune_kv_mapped(hidden: np.ndarray, orig: np.ndarray, orig_row: np.ndarray, Kc: np.ndarray, Vc: np.ndarray,
                    dtype: int, seq_offsets: np.ndarray, M: float = 0.2) -> Dict[str, np.ndarray]:
    hidden = _storage(hidden, dtype)
    orig = _storage(orig, dtype)
    Kc = _storage(Kc, dtype)
    Vc = _storage(Vc, dtype)
    so = np.ascontiguousarray(seq_offsets, np.int32)
    rows = np.ascontiguousarray(orig_row, np.int32)
    S_total, d = hidden.shape
    H, _, D = Kc.shape
    assert int(so[-1]) == S_total == len(rows)
    B = len(so) - 1
    cosv = np.full(S_total, np.nan, np.float32)
    idx = np.empty(S_total, np.int32)
    cnt = np.empty(B, np.int32)
    rows_out = np.empty(S_total, np.int32)
    K_out = np.empty_like(Kc)
    V_out = np.empty_like(Vc)
    tot = lib().sharpv_canon_prune_kv_mapped(_vp(hidden), _vp(orig), _ip(rows), _vp(Kc), _vp(Vc), dtype, _ip(so), B,
                                             orig.shape[0], d, H, D, M, _fp(cosv), _ip(idx), _ip(cnt), _ip(rows_out),
                                             _vp(K_out), _vp(V_out))
    if tot < 0:
        raise ValueError("sharpv_canon_prune_kv_mapped: bad argument")
    return {"cos": cosv, "idx": idx[:tot].copy(), "counts": cnt, "orig_row_out": rows_out[:tot].copy(),
            "K_out": K_out.reshape(-1)[:H * tot * D].reshape(H, tot, D).copy(),
            "V_out": V_out.reshape(-1)[:H * tot * D].reshape(H, tot, D).copy()}
