"""CPU oracle for the Slim-DP communication-set path: ctypes front end.

TEST INFRASTRUCTURE ONLY.  The arithmetic lives in ``slimdp_oracle.c`` (plain C,
single thread); this module compiles it with gcc, loads it and marshals NumPy
arrays.  Nothing here imports, links or shares code with the HIP library, and the
HIP library never imports this package.  Only the tests, the smoke check and the
benchmark's ``cpu_baseline`` leg may use it.

Paper sections each function follows are cited in ``slimdp_oracle.c``.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "slimdp_oracle.c")
_LIB = os.path.join(_HERE, "libslimdp_oracle.so")

# No -ffast-math, no contraction: the only fused operations are the explicit fmaf calls.
_CFLAGS = ["-O2", "-std=c11", "-fPIC", "-shared", "-ffp-contract=off", "-fno-fast-math",
           "-Wall", "-Wextra"]


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (a checker being built is not the product using it).
    SLIMDP_ORACLE_SRC / SLIMDP_ORACLE_LIB (both set): build and load another source file instead -- used only by
    the test that plants mistakes in copies of the oracle and expects the pins to fail."""
    src, lib_path = _SRC, _LIB
    if os.environ.get("SLIMDP_ORACLE_SRC") and os.environ.get("SLIMDP_ORACLE_LIB"):
        src, lib_path = os.environ["SLIMDP_ORACLE_SRC"], os.environ["SLIMDP_ORACLE_LIB"]
    if force or not os.path.exists(lib_path) or os.path.getmtime(lib_path) < os.path.getmtime(src):
        tmp = lib_path + ".tmp.%d" % os.getpid()
        subprocess.check_call(["gcc", *_CFLAGS, "-o", tmp, src, "-lm"])
        os.replace(tmp, lib_path)
    return lib_path


_lib = None


def lib() -> C.CDLL:
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _declare(_lib)
    return _lib


_u32p = C.POINTER(C.c_uint32)
_f32p = C.POINTER(C.c_float)
_f64p = C.POINTER(C.c_double)
_u8p = C.POINTER(C.c_uint8)
_u64p = C.POINTER(C.c_uint64)


def _declare(L: C.CDLL) -> None:
    L.oracle_philox4x32_10.argtypes = [_u32p, _u32p, _u32p]
    L.oracle_philox4x32_10.restype = None
    L.oracle_explore_word.argtypes = [C.c_uint64, C.c_uint64, C.c_uint32, C.c_uint32]
    L.oracle_explore_word.restype = C.c_uint32
    L.oracle_explore_words.argtypes = [C.c_uint64, C.c_uint64, C.c_uint32, C.c_uint32, C.c_uint64, _u32p]
    L.oracle_explore_words.restype = None
    L.oracle_score.argtypes = [C.c_uint64, C.c_uint32, _f32p, C.POINTER(_f32p), C.c_float, _f32p]
    L.oracle_score.restype = None
    L.oracle_dense_update_score.argtypes = [C.c_uint64, C.c_uint32, _f32p, C.POINTER(_f32p), C.c_float, C.c_float, _f32p]
    L.oracle_dense_update_score.restype = None
    L.oracle_select_core.argtypes = [_f32p, C.c_uint32, C.c_uint32, C.c_uint32, _u32p]
    L.oracle_select_core.restype = C.c_int
    L.oracle_sample_explore.argtypes = [_u8p, C.c_uint32, C.c_uint32, C.c_uint64, C.c_uint64,
                                        C.c_uint32, C.c_uint32, _u32p]
    L.oracle_sample_explore.restype = C.c_int
    L.oracle_pack.argtypes = [_f32p, _u32p, C.c_uint64, _u32p, C.c_uint64, _f32p, _f32p]
    L.oracle_pack.restype = None
    L.oracle_merge.argtypes = [C.c_uint64, _f32p, C.c_float, C.c_uint32, _u32p, C.c_uint64,
                               C.POINTER(_f32p), C.POINTER(_u32p), C.POINTER(_f32p), _u64p,
                               _f32p, _u8p]
    L.oracle_merge.restype = None
    L.oracle_merge_f64.argtypes = [C.c_uint64, _f32p, _f64p, C.c_double, C.c_uint32, _u32p,
                                   C.c_uint64, C.POINTER(_f32p), C.POINTER(_u32p),
                                   C.POINTER(_f32p), _u64p]
    L.oracle_merge_f64.restype = None
    L.oracle_pull.argtypes = [_f32p, _u32p, C.c_uint64, _u32p, C.c_uint64, _f32p, _f32p, _f32p]
    L.oracle_pull.restype = None
    L.oracle_splitmix64_mix.argtypes = [C.c_uint64]
    L.oracle_splitmix64_mix.restype = C.c_uint64
    L.oracle_core_signature.argtypes = [_u32p, C.c_uint64]
    L.oracle_core_signature.restype = C.c_uint64
    L.oracle_local_step.argtypes = [C.c_uint64, _f32p, _f32p, _f32p, C.c_float, C.c_int]
    L.oracle_local_step.restype = None
    L.oracle_quant_word.argtypes = [C.c_uint64, C.c_uint64, C.c_uint32, C.c_uint32, C.c_uint64]
    L.oracle_quant_word.restype = C.c_uint32
    L.oracle_quantize.argtypes = [_f32p, C.c_uint64, C.c_uint64, C.c_uint64, C.c_uint32, C.c_uint32, _u8p, _f32p]
    L.oracle_quantize.restype = None
    L.oracle_dequantize.argtypes = [_u8p, _f32p, C.c_uint64, _f32p]
    L.oracle_dequantize.restype = None


def _as(a, dtype) -> np.ndarray:
    a = np.ascontiguousarray(a, dtype=dtype)
    return a


def _p(a: np.ndarray, ctype):
    return a.ctypes.data_as(C.POINTER(ctype))


def _table(arrs: Sequence[np.ndarray], ctype):
    T = (C.POINTER(ctype) * max(1, len(arrs)))()
    for j, a in enumerate(arrs):
        T[j] = _p(a, ctype)
    return T


# --------------------------------------------------------------------------------------
# Philox
# --------------------------------------------------------------------------------------
def philox4x32_10(ctr: Sequence[int], key: Sequence[int]) -> np.ndarray:
    c = np.array(ctr, dtype=np.uint32)
    k = np.array(key, dtype=np.uint32)
    out = np.zeros(4, dtype=np.uint32)
    lib().oracle_philox4x32_10(_p(c, C.c_uint32), _p(k, C.c_uint32), _p(out, C.c_uint32))
    return out


def explore_words(seed: int, iteration: int, worker: int, i0: int, count: int) -> np.ndarray:
    out = np.empty(count, dtype=np.uint32)
    lib().oracle_explore_words(seed, iteration, worker, i0, count, _p(out, C.c_uint32))
    return out


# --------------------------------------------------------------------------------------
# Path steps
# --------------------------------------------------------------------------------------
def score(w: np.ndarray, g: Sequence[np.ndarray], c: float) -> np.ndarray:
    w = _as(w, np.float32)
    gs = [_as(x, np.float32) for x in g]
    assert all(x.shape == w.shape for x in gs) and len(gs) >= 1
    S = np.empty_like(w)
    lib().oracle_score(w.size, len(gs), _p(w, C.c_float), _table(gs, C.c_float), C.c_float(c),
                       _p(S, C.c_float))
    return S


def splitmix64_mix(x: int) -> int:
    return int(lib().oracle_splitmix64_mix(C.c_uint64(x & 0xFFFFFFFFFFFFFFFF)))


def core_signature(core_idx: np.ndarray) -> int:
    """Signature of the cached core keys (section 3.5): sum over j of mix(core_idx[j] + 2^32 j) modulo 2^64."""
    ci = _as(core_idx, np.uint32)
    return int(lib().oracle_core_signature(_p(ci, C.c_uint32), ci.size))


def dense_update_score(w: np.ndarray, g: Sequence[np.ndarray], lr: float, c: float):
    """Algorithm 1, the iteration before a reselection: all updates applied, significance of the new model.
    Returns (w_new, S); the input is not modified."""
    w_new = np.array(_as(w, np.float32), copy=True)
    gs = [_as(x, np.float32) for x in g]
    assert all(x.shape == w_new.shape for x in gs) and len(gs) >= 1
    S = np.empty_like(w_new)
    lib().oracle_dense_update_score(w_new.size, len(gs), _p(w_new, C.c_float), _table(gs, C.c_float), C.c_float(lr),
                                    C.c_float(c), _p(S, C.c_float))
    return w_new, S


def _segments(n: int, seg_off: Optional[Sequence[int]]):
    if seg_off is None:
        return [(0, n)]
    so = [int(x) for x in seg_off]
    assert so[0] == 0 and so[-1] == n
    return [(so[s], so[s + 1] - so[s]) for s in range(len(so) - 1)]


def select_core(S: np.ndarray, k_seg, seg_off=None) -> np.ndarray:
    """Top-k_s per segment by (score bits desc, index asc); ascending global indices."""
    S = _as(S, np.float32)
    segs = _segments(S.size, seg_off)
    ks = [int(k_seg)] if np.isscalar(k_seg) else [int(x) for x in k_seg]
    assert len(ks) == len(segs)
    out = np.empty(sum(ks), dtype=np.uint32)
    pos = 0
    dummy = np.zeros(1, np.uint32)
    for (base, ln), k in zip(segs, ks):
        dst = out[pos:pos + k] if k else dummy
        rc = lib().oracle_select_core(_p(S, C.c_float), base, ln, k, _p(dst, C.c_uint32))
        if rc != 0:
            raise ValueError("oracle_select_core: bad arguments")
        pos += k
    return out


def core_mask(n: int, core_idx: np.ndarray) -> np.ndarray:
    mask = np.zeros(n, dtype=np.uint8)
    mask[np.asarray(core_idx, dtype=np.int64)] = 1
    return mask


def core_bits(n: int, core_idx: np.ndarray) -> np.ndarray:
    """Bitmap layout of the library's core_bits: bit (i mod 32) of word (i div 32)."""
    mask = core_mask(n, core_idx)
    pad = (-n) % 32
    if pad:
        mask = np.concatenate([mask, np.zeros(pad, np.uint8)])
    return np.packbits(mask.reshape(-1, 32), axis=1, bitorder="little").view(np.uint32).reshape(-1)


def sample_explore(n: int, core_idx: np.ndarray, seed: int, iteration: int, worker: int,
                   m_seg, seg_off=None) -> np.ndarray:
    mask = core_mask(n, core_idx)
    segs = _segments(n, seg_off)
    ms = [int(m_seg)] if np.isscalar(m_seg) else [int(x) for x in m_seg]
    assert len(ms) == len(segs)
    out = np.empty(sum(ms), dtype=np.uint32)
    pos = 0
    dummy = np.zeros(1, np.uint32)
    for (base, ln), m in zip(segs, ms):
        dst = out[pos:pos + m] if m else dummy
        rc = lib().oracle_sample_explore(_p(mask, C.c_uint8), base, ln, seed, iteration, worker, m,
                                         _p(dst, C.c_uint32))
        if rc != 0:
            raise ValueError("oracle_sample_explore: m exceeds the non-core count")
        pos += m
    return out


def pack(g_k: np.ndarray, core_idx: np.ndarray, expl_idx: np.ndarray):
    g_k = _as(g_k, np.float32)
    ci = _as(core_idx, np.uint32)
    ei = _as(expl_idx, np.uint32)
    cv = np.empty(ci.size, np.float32)
    ev = np.empty(ei.size, np.float32)
    lib().oracle_pack(_p(g_k, C.c_float), _p(ci, C.c_uint32), ci.size, _p(ei, C.c_uint32), ei.size,
                      _p(cv, C.c_float), _p(ev, C.c_float))
    return cv, ev


def merge(w: np.ndarray, lr: float, core_idx: np.ndarray, core_val: Sequence[np.ndarray],
          expl_idx: Sequence[np.ndarray], expl_val: Sequence[np.ndarray]) -> np.ndarray:
    """Returns the updated copy of w (binary32, worker-ordered sum, one fma)."""
    w = np.array(w, dtype=np.float32, copy=True)
    W = len(core_val)
    ci = _as(core_idx, np.uint32)
    cv = [_as(x, np.float32) for x in core_val]
    ei = [_as(x, np.uint32) for x in expl_idx]
    ev = [_as(x, np.float32) for x in expl_val]
    assert len(ei) == W and len(ev) == W and all(x.size == ci.size for x in cv)
    mw = np.array([x.size for x in ei], dtype=np.uint64)
    acc = np.empty(w.size, np.float32)
    hit = np.empty(w.size, np.uint8)
    lib().oracle_merge(w.size, _p(w, C.c_float), C.c_float(lr), W, _p(ci, C.c_uint32), ci.size,
                       _table(cv, C.c_float), _table(ei, C.c_uint32), _table(ev, C.c_float),
                       _p(mw, C.c_uint64), _p(acc, C.c_float), _p(hit, C.c_uint8))
    return w


def merge_f64(w: np.ndarray, lr: float, core_idx: np.ndarray, core_val: Sequence[np.ndarray],
              expl_idx: Sequence[np.ndarray], expl_val: Sequence[np.ndarray]) -> np.ndarray:
    w = _as(w, np.float32)
    W = len(core_val)
    ci = _as(core_idx, np.uint32)
    cv = [_as(x, np.float32) for x in core_val]
    ei = [_as(x, np.uint32) for x in expl_idx]
    ev = [_as(x, np.float32) for x in expl_val]
    mw = np.array([x.size for x in ei], dtype=np.uint64)
    out = np.empty(w.size, np.float64)
    lib().oracle_merge_f64(w.size, _p(w, C.c_float), _p(out, C.c_double), C.c_double(lr), W,
                           _p(ci, C.c_uint32), ci.size, _table(cv, C.c_float),
                           _table(ei, C.c_uint32), _table(ev, C.c_float), _p(mw, C.c_uint64))
    return out


def pull(w: np.ndarray, core_idx: np.ndarray, expl_idx: np.ndarray,
         w_local: Optional[np.ndarray] = None):
    w = _as(w, np.float32)
    ci = _as(core_idx, np.uint32)
    ei = _as(expl_idx, np.uint32)
    co = np.empty(ci.size, np.float32)
    eo = np.empty(ei.size, np.float32)
    wl = None
    if w_local is not None:
        wl = np.array(w_local, dtype=np.float32, copy=True)
    lib().oracle_pull(_p(w, C.c_float), _p(ci, C.c_uint32), ci.size, _p(ei, C.c_uint32), ei.size,
                      _p(co, C.c_float), _p(eo, C.c_float),
                      _p(wl, C.c_float) if wl is not None else None)
    return co, eo, wl


# --------------------------------------------------------------------------------------
# Worker side: local training stand-in (section 3.3 step 1)
# --------------------------------------------------------------------------------------
def local_step(w_local: np.ndarray, delta: Optional[np.ndarray], grad: np.ndarray, eta: float):
    """One mini-batch step on a local model and the accumulation of its update; delta None starts a new
    accumulation.  Returns (w_local_new, delta_new); the inputs are not modified."""
    w = np.array(_as(w_local, np.float32), copy=True)
    g = _as(grad, np.float32)
    first = delta is None
    # a new accumulation must not read the old one: it gets a buffer of NaNs
    d = np.full_like(w, np.nan) if first else np.array(_as(delta, np.float32), copy=True)
    assert g.shape == w.shape == d.shape
    lib().oracle_local_step(w.size, _p(w, C.c_float), _p(d, C.c_float), _p(g, C.c_float), C.c_float(eta), int(first))
    return w, d


# --------------------------------------------------------------------------------------
# Quantised wire values (section 2.2 end; section 4.2: 8 bits, buckets of 512)
# --------------------------------------------------------------------------------------
QUANT_BUCKET = 512


def quant_word(seed: int, iteration: int, worker: int, kind: int, j: int) -> int:
    return int(lib().oracle_quant_word(seed, iteration, worker, kind, j))


def quantize(v: np.ndarray, seed: int, iteration: int, worker: int, kind: int):
    """Returns (codes uint8 [count], scales float32 [ceil(count / 512)])."""
    v = _as(v, np.float32)
    code = np.empty(v.size, np.uint8)
    scale = np.empty((v.size + QUANT_BUCKET - 1) // QUANT_BUCKET, np.float32)
    lib().oracle_quantize(_p(v, C.c_float), v.size, seed, iteration, worker, kind, _p(code, C.c_uint8),
                          _p(scale, C.c_float))
    return code, scale


def dequantize(code: np.ndarray, scale: np.ndarray) -> np.ndarray:
    code = _as(code, np.uint8)
    scale = _as(scale, np.float32)
    out = np.empty(code.size, np.float32)
    lib().oracle_dequantize(_p(code, C.c_uint8), _p(scale, C.c_float), code.size, _p(out, C.c_float))
    return out


def wire_bytes(k: int, m: int, quantized: bool) -> int:
    """Bytes one worker sends per push (section 3.5): core values only (keys cached), explorer <key, value> pairs;
    quantised values take one byte each plus one binary32 scale per bucket of 512."""
    if not quantized:
        return 4 * (k + 2 * m)
    nb = lambda c: (c + QUANT_BUCKET - 1) // QUANT_BUCKET
    return k + 4 * nb(k) + m + 4 * nb(m) + 4 * m
