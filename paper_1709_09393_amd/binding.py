"""ctypes binding over ``libslimdp.so`` (the C ABI of ``include/slimdp.h``).

Argument marshalling only: every step of the path runs in the library's HIP kernels.
torch is used for device memory and the stream; there is no CPU fallback -- if the shared
library is missing or no GPU is present the calls raise.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import List, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libslimdp.so")

TILE = 4096
MAX_WORKERS = 32

OK = 0
ERR_INVALID_ARG = -1
ERR_OUT_OF_RANGE = -2
ERR_STALE_CORE = -3
ERR_WORKSPACE = -4
ERR_HIP = -5
ERR_DEVICE_STATUS = -6
SELECT_REUSE_HISTOGRAM = 1
PACK_UPDATES_AS_SCORED = 1
LOCAL_FIRST = 1
QUANT_BUCKET = 512

EXPORTS = [
    "slimdp_create", "slimdp_destroy", "slimdp_workspace_bytes", "slimdp_capture_bytes", "slimdp_num_tiles",
    "slimdp_tile_starts", "slimdp_last_error", "slimdp_synchronize", "slimdp_set_option",
    "slimdp_score", "slimdp_dense_update_score", "slimdp_select_core", "slimdp_sample_explore", "slimdp_explore_hint", "slimdp_tile_offsets",
    "slimdp_pack", "slimdp_merge", "slimdp_pull", "slimdp_core_signature", "slimdp_debug_philox",
    "slimdp_select_core_static", "slimdp_import_core", "slimdp_local_step", "slimdp_local_step_pack", "slimdp_pull_local_step", "slimdp_quantize",
    "slimdp_dequantize",
]


class SlimDPError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"libslimdp error {code}: {msg}")
        self.code = code


_lib = None
_vp = C.c_void_p
_u64p = C.POINTER(C.c_uint64)
_vpp = C.POINTER(C.c_void_p)


def load() -> C.CDLL:
    """Loads the in-tree shared library; raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(
            f"{LIB_PATH} is missing: build it first (python -c 'import __graft_entry__ as g; g.build()')")
    L = C.CDLL(LIB_PATH)
    L.slimdp_create.argtypes = [C.POINTER(_vp), C.c_uint64, C.c_uint32, C.c_uint32, _u64p, C.c_uint64, _vp]
    L.slimdp_create.restype = C.c_int
    L.slimdp_destroy.argtypes = [_vp]
    L.slimdp_destroy.restype = C.c_int
    L.slimdp_workspace_bytes.argtypes = [C.c_uint64, C.c_uint32, C.c_uint32, _u64p]
    L.slimdp_workspace_bytes.restype = C.c_uint64
    L.slimdp_capture_bytes.argtypes = [C.c_uint64, C.c_uint32, C.c_uint32, _u64p]
    L.slimdp_capture_bytes.restype = C.c_uint64
    L.slimdp_num_tiles.argtypes = [C.c_uint64, C.c_uint32, _u64p]
    L.slimdp_num_tiles.restype = C.c_uint64
    L.slimdp_tile_starts.argtypes = [_vp, C.POINTER(C.c_uint32)]
    L.slimdp_tile_starts.restype = C.c_int
    L.slimdp_last_error.argtypes = [_vp]
    L.slimdp_last_error.restype = C.c_char_p
    L.slimdp_synchronize.argtypes = [_vp]
    L.slimdp_synchronize.restype = C.c_int
    L.slimdp_set_option.argtypes = [_vp, C.c_char_p, C.c_int64]
    L.slimdp_set_option.restype = C.c_int
    L.slimdp_score.argtypes = [_vp, _vp, _vpp, C.c_uint32, C.c_float, _vp]
    L.slimdp_score.restype = C.c_int
    L.slimdp_dense_update_score.argtypes = [_vp, _vp, _vpp, C.c_uint32, C.c_float, C.c_float, _vp]
    L.slimdp_dense_update_score.restype = C.c_int
    L.slimdp_core_signature.argtypes = [_vp, _vp, C.c_uint64, _vp]
    L.slimdp_core_signature.restype = C.c_int
    L.slimdp_select_core.argtypes = [_vp, _vp, _u64p, C.c_uint32, _vp, _vp, _vp, _u64p]
    L.slimdp_select_core.restype = C.c_int
    L.slimdp_sample_explore.argtypes = [_vp, _vp, _u64p, C.c_uint32, C.c_uint32, C.c_uint64, _u64p, _vpp, _vpp]
    L.slimdp_sample_explore.restype = C.c_int
    L.slimdp_explore_hint.argtypes = [_vp, _u64p, C.c_uint32, C.c_uint32, C.c_uint64, _u64p]
    L.slimdp_explore_hint.restype = C.c_int
    L.slimdp_tile_offsets.argtypes = [_vp, _vp, C.c_uint64, _vp]
    L.slimdp_tile_offsets.restype = C.c_int
    L.slimdp_pack.argtypes = [_vp, C.c_uint32, _vpp, _vp, _vp, C.c_uint64, _vpp, _vpp, _u64p, _vpp, _vpp, C.c_uint64,
                              C.c_uint32]
    L.slimdp_pack.restype = C.c_int
    L.slimdp_merge.argtypes = [_vp, _vp, C.c_float, C.c_uint64, C.c_uint32, _vp, _vp, C.c_uint64, _vpp, _vpp, _vpp,
                               _vpp, _u64p]
    L.slimdp_merge.restype = C.c_int
    L.slimdp_pull.argtypes = [_vp, _vp, C.c_uint64, C.c_uint32, _vp, _vp, C.c_uint64, _vpp, _vpp, _u64p, _vpp, _vpp,
                              _vpp]
    L.slimdp_pull.restype = C.c_int
    L.slimdp_debug_philox.argtypes = [_vp, C.c_uint64, C.c_uint32, C.c_uint32, C.c_uint64, _vp]
    L.slimdp_debug_philox.restype = C.c_int
    L.slimdp_select_core_static.argtypes = [_vp, C.c_uint64, C.c_uint64, _vp, _vp, _vp, _vp]
    L.slimdp_select_core_static.restype = C.c_int
    L.slimdp_import_core.argtypes = [_vp, _vp, _u64p, _vp, _vp, _u64p]
    L.slimdp_import_core.restype = C.c_int
    L.slimdp_local_step.argtypes = [_vp, C.c_uint32, _vpp, _vpp, _vpp, C.c_float, C.c_uint32]
    L.slimdp_local_step.restype = C.c_int
    L.slimdp_local_step_pack.argtypes = [_vp, C.c_uint32, _vpp, _vpp, _vpp, C.c_float, C.c_uint32, _vp, _vp, C.c_uint64, _vpp,
                                         _vpp, _u64p, _vpp, _vpp, C.c_uint64]
    L.slimdp_local_step_pack.restype = C.c_int
    L.slimdp_pull_local_step.argtypes = [_vp, _vp, C.c_uint64, C.c_uint32, _vp, _vp, C.c_uint64, _vpp, _vpp, _u64p, _vpp, _vpp,
                                         _vpp, C.c_float, C.c_uint32]
    L.slimdp_pull_local_step.restype = C.c_int
    L.slimdp_quantize.argtypes = [_vp, C.c_uint32, C.c_uint32, _vpp, _u64p, C.c_uint32, C.c_uint64, _vpp, _vpp]
    L.slimdp_quantize.restype = C.c_int
    L.slimdp_dequantize.argtypes = [_vp, C.c_uint32, _vpp, _vpp, _u64p, _vpp]
    L.slimdp_dequantize.restype = C.c_int
    _lib = L
    return L


def _u64arr(vals) -> "C.Array":
    vals = [int(v) for v in vals]
    return (C.c_uint64 * max(1, len(vals)))(*vals)


def _seg_off(n: int, seg_off) -> "C.Array":
    if seg_off is None:
        seg_off = [0, n]
    return _u64arr(seg_off)


def num_tiles(n: int, seg_off=None) -> int:
    so = [0, n] if seg_off is None else [int(x) for x in seg_off]
    return int(load().slimdp_num_tiles(n, len(so) - 1, _u64arr(so)))


def workspace_bytes(n: int, max_workers: int, seg_off=None) -> int:
    so = [0, n] if seg_off is None else [int(x) for x in seg_off]
    return int(load().slimdp_workspace_bytes(n, max_workers, len(so) - 1, _u64arr(so)))


def capture_bytes(n: int, max_workers: int, seg_off=None) -> int:
    so = [0, n] if seg_off is None else [int(x) for x in seg_off]
    return int(load().slimdp_capture_bytes(n, max_workers, len(so) - 1, _u64arr(so)))


def _ptr(t) -> Optional[int]:
    """Device address of a torch tensor (None passes NULL)."""
    if t is None:
        return None
    return t.data_ptr() if t.numel() else (t.data_ptr() or None)


def _table(ts: Optional[Sequence]) -> "C.Array":
    if ts is None:
        return None
    arr = (C.c_void_p * max(1, len(ts)))()
    for j, t in enumerate(ts):
        arr[j] = _ptr(t)
    return arr


STATIC_MAX_N = 1 << 20


def select_core_static(score, k: int, core_idx, core_bits, core_off, stream=None) -> None:
    """slimdp_select_core_static: flat selection without a context; every array is the caller's (nothing is allocated)."""
    import torch
    st = stream if stream is not None else torch.cuda.current_stream()
    rc = load().slimdp_select_core_static(_ptr(score), score.numel(), int(k), _ptr(core_idx), _ptr(core_bits),
                                          _ptr(core_off), C.c_void_p(st.cuda_stream))
    if rc != OK:
        raise SlimDPError(rc, load().slimdp_last_error(None).decode())


class SlimDP:
    """One context: n parameters, up to max_workers logical workers, one GPU, one stream."""

    def __init__(self, n: int, max_workers: int, seg_off=None, seed: int = 0, stream=None):
        import torch
        self._torch = torch
        self._L = load()
        if not torch.cuda.is_available():
            raise RuntimeError("libslimdp needs a GPU: torch.cuda.is_available() is False")
        self.n = int(n)
        self.max_workers = int(max_workers)
        self.seg_off = [0, self.n] if seg_off is None else [int(x) for x in seg_off]
        self.n_seg = len(self.seg_off) - 1
        self.stream = stream if stream is not None else torch.cuda.current_stream()
        self._h = C.c_void_p()
        rc = self._L.slimdp_create(C.byref(self._h), self.n, self.max_workers, self.n_seg, _u64arr(self.seg_off),
                                   int(seed), C.c_void_p(self.stream.cuda_stream))
        if rc != OK:
            msg = self._L.slimdp_last_error(None).decode()
            self._h = None
            raise SlimDPError(rc, msg)
        self.T = num_tiles(self.n, self.seg_off)
        self.device = torch.device("cuda", torch.cuda.current_device())

    # -- plumbing ------------------------------------------------------------------------
    def _check(self, rc: int) -> None:
        if rc != OK:
            raise SlimDPError(rc, self._L.slimdp_last_error(self._h).decode())

    def close(self) -> None:
        if getattr(self, "_h", None):
            self._L.slimdp_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def synchronize(self) -> None:
        self._check(self._L.slimdp_synchronize(self._h))

    def set_option(self, name: str, value: int) -> None:
        self._check(self._L.slimdp_set_option(self._h, name.encode(), int(value)))

    def tile_starts(self) -> np.ndarray:
        out = np.zeros(self.T + 1, dtype=np.uint32)
        self._check(self._L.slimdp_tile_starts(self._h, out.ctypes.data_as(C.POINTER(C.c_uint32))))
        return out

    def _empty(self, count: int, dtype):
        return self._torch.empty(int(count), dtype=dtype, device=self.device)

    # -- the path ------------------------------------------------------------------------
    def score(self, w, g: Sequence, c: float, out=None):
        torch = self._torch
        if out is None:
            out = self._empty(self.n, torch.float32)
        self._check(self._L.slimdp_score(self._h, _ptr(w), _table(g), len(g), C.c_float(c), _ptr(out)))
        return out

    def dense_update_score(self, w, g: Sequence, lr: float, c: float, out=None):
        """w <- w - lr * sum of all updates (in place), then the significance of the new model."""
        torch = self._torch
        if out is None:
            out = self._empty(self.n, torch.float32)
        self._check(self._L.slimdp_dense_update_score(self._h, _ptr(w), _table(g), len(g), C.c_float(lr), C.c_float(c),
                                                      _ptr(out)))
        return out

    def select_core(self, score, k_seg, reuse_histogram: bool = False, core_idx=None, core_bits=None, core_off=None):
        torch = self._torch
        ks = [int(k_seg)] if np.isscalar(k_seg) else [int(x) for x in k_seg]
        K = sum(ks)
        if core_idx is None:
            core_idx = self._empty(K, torch.int32)
        if core_bits is None:
            core_bits = self._empty((self.n + 31) // 32, torch.int32)
        if core_off is None:
            core_off = self._empty(self.T + 1, torch.int32)
        epoch = C.c_uint64(0)
        self._check(self._L.slimdp_select_core(self._h, _ptr(score), _u64arr(ks),
                                               SELECT_REUSE_HISTOGRAM if reuse_histogram else 0, _ptr(core_idx),
                                               _ptr(core_bits), _ptr(core_off), C.byref(epoch)))
        return core_idx, core_bits, core_off, int(epoch.value)

    def sample_explore(self, core_bits, k_seg, iteration: int, m_seg, worker0: int = 0, n_workers: int = 1,
                       expl_idx: Optional[List] = None, expl_off: Optional[List] = None):
        torch = self._torch
        ks = [int(k_seg)] if np.isscalar(k_seg) else [int(x) for x in k_seg]
        ms = [int(m_seg)] if np.isscalar(m_seg) else [int(x) for x in m_seg]
        M = sum(ms)
        if expl_idx is None:
            expl_idx = [self._empty(M, torch.int32) for _ in range(n_workers)]
        if expl_off is None:
            expl_off = [self._empty(self.T + 1, torch.int32) for _ in range(n_workers)]
        self._check(self._L.slimdp_sample_explore(self._h, _ptr(core_bits), _u64arr(ks), worker0, n_workers,
                                                  int(iteration), _u64arr(ms), _table(expl_idx), _table(expl_off)))
        return expl_idx, expl_off

    def explore_hint(self, k_seg, iteration: int, m_seg, worker0: int = 0, n_workers: int = 1) -> None:
        ks = [int(k_seg)] if np.isscalar(k_seg) else [int(x) for x in k_seg]
        ms = [int(m_seg)] if np.isscalar(m_seg) else [int(x) for x in m_seg]
        self._check(self._L.slimdp_explore_hint(self._h, _u64arr(ks), worker0, n_workers, int(iteration), _u64arr(ms)))

    def tile_offsets(self, idx, out=None):
        if out is None:
            out = self._empty(self.T + 1, self._torch.int32)
        self._check(self._L.slimdp_tile_offsets(self._h, _ptr(idx), idx.numel(), _ptr(out)))
        return out

    def pack(self, g: Sequence, core_idx, core_off, expl_idx: Sequence, expl_off: Sequence, core_epoch: int,
             core_val: Optional[List] = None, expl_val: Optional[List] = None, updates_as_scored: bool = False):
        """updates_as_scored: g is, unchanged, what the last score() on this context read."""
        torch = self._torch
        nw = len(g)
        k = core_idx.numel()
        if core_val is None:
            core_val = [self._empty(k, torch.float32) for _ in range(nw)]
        if expl_val is None:
            expl_val = [self._empty(expl_idx[q].numel(), torch.float32) for q in range(nw)]
        mw = _u64arr([expl_idx[q].numel() for q in range(nw)])
        self._check(self._L.slimdp_pack(self._h, nw, _table(g), _ptr(core_idx), _ptr(core_off), k, _table(expl_idx),
                                        _table(expl_off), mw, _table(core_val), _table(expl_val), int(core_epoch),
                                        PACK_UPDATES_AS_SCORED if updates_as_scored else 0))
        return core_val, expl_val

    def merge(self, w, lr: float, core_epoch: int, core_idx, core_off, core_val: Sequence, expl_idx: Sequence,
              expl_off: Sequence, expl_val: Sequence) -> None:
        nw = len(core_val)
        mw = _u64arr([expl_idx[q].numel() for q in range(nw)])
        self._check(self._L.slimdp_merge(self._h, _ptr(w), C.c_float(lr), int(core_epoch), nw, _ptr(core_idx),
                                         _ptr(core_off), core_idx.numel(), _table(core_val), _table(expl_idx),
                                         _table(expl_off), _table(expl_val), mw))

    def pull(self, w, core_epoch: int, core_idx, core_off, expl_idx: Sequence, expl_off: Sequence,
             w_local: Optional[Sequence] = None, core_out: Optional[List] = None, expl_out: Optional[List] = None):
        torch = self._torch
        nw = len(expl_idx)
        k = core_idx.numel()
        if core_out is None:
            core_out = [self._empty(k, torch.float32) for _ in range(nw)]
        if expl_out is None:
            expl_out = [self._empty(expl_idx[q].numel(), torch.float32) for q in range(nw)]
        mw = _u64arr([expl_idx[q].numel() for q in range(nw)])
        self._check(self._L.slimdp_pull(self._h, _ptr(w), int(core_epoch), nw, _ptr(core_idx), _ptr(core_off), k,
                                        _table(expl_idx), _table(expl_off), mw, _table(core_out), _table(expl_out),
                                        _table(w_local)))
        return core_out, expl_out

    def core_signature(self, core_idx):
        """Signature of the cached core keys; returns a one-element int64 device tensor (read it after synchronize)."""
        out = self._empty(1, self._torch.int64)
        self._check(self._L.slimdp_core_signature(self._h, _ptr(core_idx), core_idx.numel(), _ptr(out)))
        return out

    def debug_philox(self, iteration: int, worker: int, i0: int, count: int):
        out = self._empty(count, self._torch.int32)
        self._check(self._L.slimdp_debug_philox(self._h, int(iteration), int(worker), int(i0), int(count), _ptr(out)))
        return out

    def import_core(self, core_idx, k_seg, core_bits=None, core_off=None):
        """Adopts core keys saved from another context (resume); returns (core_bits, core_off, epoch)."""
        torch = self._torch
        ks = [int(k_seg)] if np.isscalar(k_seg) else [int(x) for x in k_seg]
        if core_bits is None:
            core_bits = self._empty((self.n + 31) // 32, torch.int32)
        if core_off is None:
            core_off = self._empty(self.T + 1, torch.int32)
        epoch = C.c_uint64(0)
        self._check(self._L.slimdp_import_core(self._h, _ptr(core_idx), _u64arr(ks), _ptr(core_bits), _ptr(core_off),
                                               C.byref(epoch)))
        return core_bits, core_off, int(epoch.value)

    # -- worker side and wire codec ------------------------------------------------------
    def local_step(self, w_local: Sequence, grad: Sequence, delta: Sequence, eta: float, first: bool) -> None:
        """One mini-batch step on every local model; delta accumulates the update (first: starts a new sum)."""
        self._check(self._L.slimdp_local_step(self._h, len(w_local), _table(w_local), _table(grad), _table(delta),
                                              C.c_float(eta), LOCAL_FIRST if first else 0))

    def local_step_pack(self, w_local: Sequence, grad: Sequence, delta: Sequence, eta: float, first: bool, core_idx,
                        core_off, expl_idx: Sequence, expl_off: Sequence, core_epoch: int,
                        core_val: Optional[List] = None, expl_val: Optional[List] = None):
        """local_step() and pack(delta, ...) in one pass over the update vectors."""
        torch = self._torch
        nw = len(w_local)
        k = core_idx.numel()
        if core_val is None:
            core_val = [self._empty(k, torch.float32) for _ in range(nw)]
        if expl_val is None:
            expl_val = [self._empty(expl_idx[q].numel(), torch.float32) for q in range(nw)]
        mw = _u64arr([expl_idx[q].numel() for q in range(nw)])
        self._check(self._L.slimdp_local_step_pack(self._h, nw, _table(w_local), _table(grad), _table(delta), C.c_float(eta),
                                                   LOCAL_FIRST if first else 0, _ptr(core_idx), _ptr(core_off), k,
                                                   _table(expl_idx), _table(expl_off), mw, _table(core_val),
                                                   _table(expl_val), int(core_epoch)))
        return core_val, expl_val

    def pull_local_step(self, w, core_epoch: int, core_idx, core_off, expl_idx: Sequence, expl_off: Sequence,
                        w_local: Sequence, grad: Sequence, delta: Sequence, eta: float, first: bool = True) -> None:
        """pull(..., w_local=w_local) (its value outputs aside) and local_step() in one pass over the local models."""
        nw = len(w_local)
        mw = _u64arr([expl_idx[q].numel() for q in range(nw)])
        self._check(self._L.slimdp_pull_local_step(self._h, _ptr(w), int(core_epoch), nw, _ptr(core_idx), _ptr(core_off),
                                                   core_idx.numel(), _table(expl_idx), _table(expl_off), mw, _table(w_local),
                                                   _table(grad), _table(delta), C.c_float(eta), LOCAL_FIRST if first else 0))

    def quantize(self, val: Sequence, kind: int, iteration: int, worker0: int = 0, code=None, scale=None):
        torch = self._torch
        nw = len(val)
        if code is None:
            code = [self._empty(v.numel(), torch.uint8) for v in val]
        if scale is None:
            scale = [self._empty((v.numel() + QUANT_BUCKET - 1) // QUANT_BUCKET, torch.float32) for v in val]
        cnt = _u64arr([v.numel() for v in val])
        self._check(self._L.slimdp_quantize(self._h, nw, int(worker0), _table(val), cnt, int(kind), int(iteration),
                                            _table(code), _table(scale)))
        return code, scale

    def dequantize(self, code: Sequence, scale: Sequence, out=None):
        torch = self._torch
        nw = len(code)
        if out is None:
            out = [self._empty(c.numel(), torch.float32) for c in code]
        cnt = _u64arr([c.numel() for c in code])
        self._check(self._L.slimdp_dequantize(self._h, nw, _table(code), _table(scale), cnt, _table(out)))
        return out


def wire_bytes(k: int, m: int, quantized: bool) -> int:
    """Bytes one worker pushes (core values + explorer <key, value> pairs), plain or with 8-bit values."""
    if not quantized:
        return 4 * (k + 2 * m)
    nb = lambda c: (c + QUANT_BUCKET - 1) // QUANT_BUCKET
    return k + 4 * nb(k) + 5 * m + 4 * nb(m)
