"""ctypes binding of libaircache.so: same names as the C ABI, argument marshalling only.

Every step of the hot path runs in the HIP library; PyTorch only owns device memory and the
stream.  There is no CPU fallback: a missing library raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import List, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libaircache.so")

AIR_OK = 0
AIR_ERR_INVALID_ARG, AIR_ERR_SHAPE, AIR_ERR_WORKSPACE, AIR_ERR_STATE, AIR_ERR_HIP = 1, 2, 3, 4, 5
AIR_F32, AIR_BF16 = 0, 1
AIR_BUDGET_STRENGTH_SKEW, AIR_BUDGET_UNIFORM, AIR_BUDGET_STRENGTH, AIR_BUDGET_SKEW = 0, 1, 2, 3
AIR_WINDOW_TEXT, AIR_WINDOW_VISUAL = 0, 1
_STATUS_NAMES = {0: "AIR_OK", 1: "AIR_ERR_INVALID_ARG", 2: "AIR_ERR_SHAPE", 3: "AIR_ERR_WORKSPACE",
                 4: "AIR_ERR_STATE", 5: "AIR_ERR_HIP"}


class AirError(RuntimeError):
    def __init__(self, status: int, msg: str):
        super().__init__(f"{_STATUS_NAMES.get(status, status)}: {msg}")
        self.status = status


class air_config(C.Structure):
    _fields_ = [(n, C.c_int32) for n in (
        "n_layers", "n_q_heads", "n_kv_heads", "head_dim", "batch", "max_vis_len", "max_nonvis_len",
        "max_window", "max_decode_steps", "dtype", "budget_mode", "min_keep")] + [
        ("alpha", C.c_double), ("retention", C.c_double), ("window_kind", C.c_int32), ("device_steps", C.c_int32),
        ("cache_in_place", C.c_int32), ("causal_text", C.c_int32)]


class air_seq(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("seq_len", "vis_start", "vis_len", "win_start", "win_len")]


class air_layer(C.Structure):
    _fields_ = [("q_text", C.c_void_p), ("k", C.c_void_p), ("v", C.c_void_p)]


class air_tuning(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("decode_splits", "decode_waves", "decode_tiles", "score_block_mb",
                                         "score_rows_kernel", "select_threads", "select_direct_max", "gather_wgs",
                                         "decode_order", "decode_halves", "budget_in_score")]


class air_strides(C.Structure):
    _fields_ = [(n, C.c_int64) for n in ("q_b", "q_h", "q_t", "kv_b", "kv_h", "kv_t")]


EXPORTS = (
    "air_version", "air_workspace_bytes", "air_create", "air_destroy", "air_reset", "air_set_tuning", "air_score",
    "air_budget", "air_select_compact", "air_decode_attn", "air_decode_attn_static", "air_get_scores", "air_get_elite", "air_get_stats",
    "air_get_budgets", "air_set_budgets", "air_get_indices", "air_set_indices", "air_get_lengths", "air_get_cache",
    "air_last_error",
)

_lib = None


def load_library(path: Optional[str] = None):
    """Load libaircache.so (built in-tree by paper_2503_23956_amd.build).  Raises if it is missing."""
    global _lib
    if _lib is not None and path is None:
        return _lib
    p = path or LIB_PATH
    if not os.path.exists(p):
        raise FileNotFoundError(
            f"{p} not found: build it with `python -m paper_2503_23956_amd.build` (there is no CPU fallback)")
    # PyTorch ships its own HIP runtime (soname libamdhip64.so.7).  Import it first so that this
    # library binds to the same runtime instance that owns the tensors and streams it is handed.
    import torch  # noqa: F401

    lib = C.CDLL(p)
    vp, i32 = C.c_void_p, C.c_int32
    lib.air_version.restype = C.c_char_p
    lib.air_workspace_bytes.restype = C.c_size_t
    lib.air_workspace_bytes.argtypes = [C.POINTER(air_config)]
    lib.air_create.argtypes = [C.POINTER(air_config), vp, C.c_size_t, C.POINTER(vp)]
    lib.air_destroy.argtypes = [vp]
    lib.air_reset.argtypes = [vp]
    lib.air_score.argtypes = [vp, vp, i32, i32, C.POINTER(air_layer), C.POINTER(air_strides), C.POINTER(air_seq)]
    lib.air_budget.argtypes = [vp, vp]
    lib.air_select_compact.argtypes = [vp, vp, i32, i32, C.POINTER(air_layer), C.POINTER(air_strides)]
    lib.air_decode_attn.argtypes = [vp, vp, i32, i32, vp, vp, vp, vp]
    lib.air_decode_attn_static.argtypes = [vp, vp, i32, i32, vp, vp, vp, vp]
    lib.air_set_tuning.argtypes = [vp, C.POINTER(air_tuning)]
    lib.air_get_scores.argtypes = [vp, i32, vp]
    lib.air_get_elite.argtypes = [vp, i32, vp, vp]
    lib.air_get_stats.argtypes = [vp, vp, vp]
    lib.air_get_budgets.argtypes = [vp, vp]
    lib.air_set_budgets.argtypes = [vp, vp]
    lib.air_set_indices.argtypes = [vp, C.c_int32, vp]
    lib.air_get_indices.argtypes = [vp, i32, vp]
    lib.air_get_lengths.argtypes = [vp, vp]
    lib.air_get_cache.argtypes = [vp, i32, i32, i32, vp, vp, i32]
    lib.air_last_error.argtypes = [vp]
    lib.air_last_error.restype = C.c_char_p
    for name in EXPORTS:
        if name not in ("air_version", "air_workspace_bytes", "air_last_error"):
            getattr(lib, name).restype = C.c_int
    if path is None:
        _lib = lib
    return lib


def make_config(*, n_layers, n_q_heads, n_kv_heads, head_dim, batch, max_vis_len, max_nonvis_len, max_window,
                max_decode_steps, dtype, alpha=0.9, retention=0.1, budget_mode=AIR_BUDGET_STRENGTH_SKEW,
                min_keep=1, window_kind=AIR_WINDOW_TEXT, device_steps=0, cache_in_place=0, causal_text=0) -> air_config:
    return air_config(n_layers, n_q_heads, n_kv_heads, head_dim, batch, max_vis_len, max_nonvis_len, max_window,
                      max_decode_steps, dtype, budget_mode, min_keep, alpha, retention, window_kind, device_steps, cache_in_place,
                      causal_text)


def _ptr(t) -> int:
    return 0 if t is None else int(t.data_ptr())


class Prepared:
    """Marshalled arguments of a range of layers: air_layer[] / air_strides / air_seq[] plus the tensors they point to."""

    def __init__(self, layers, strides, seqs, n, keepalive):
        self.layers, self.strides, self.seqs, self.n, self._keepalive = layers, strides, seqs, n, keepalive


class AirCache:
    """One context: thin wrapper that keeps the workspace tensor alive and marshals arguments.

    Methods carry the names of the C entry points they call.
    """

    def __init__(self, cfg: air_config, device="cuda:0"):
        import torch

        self.lib = load_library()
        self.cfg = cfg
        self.torch = torch
        self.device = torch.device(device)
        nbytes = self.lib.air_workspace_bytes(C.byref(cfg))
        if nbytes == 0:
            raise AirError(AIR_ERR_SHAPE, "air_workspace_bytes: invalid configuration")
        self.workspace = torch.empty(nbytes, dtype=torch.uint8, device=self.device)
        self.workspace_bytes = nbytes
        h = C.c_void_p()
        st = self.lib.air_create(C.byref(cfg), self.workspace.data_ptr(), nbytes, C.byref(h))
        if st != AIR_OK:
            raise AirError(st, "air_create failed")
        self.handle = h
        self._seqs = None

    def close(self):
        if getattr(self, "handle", None):
            self.lib.air_destroy(self.handle)
            self.handle = None

    def __del__(self):  # pragma: no cover
        try:
            self.close()
        except Exception:
            pass

    # -- helpers ---------------------------------------------------------------------
    def _check(self, st: int):
        if st != AIR_OK:
            raise AirError(st, self.lib.air_last_error(self.handle).decode())

    def _stream(self) -> int:
        return int(self.torch.cuda.current_stream(self.device).cuda_stream)

    @staticmethod
    def _layers(q_text: Optional[Sequence], k: Sequence, v: Sequence):
        n = len(k)
        arr = (air_layer * n)()
        for i in range(n):
            arr[i].q_text = _ptr(q_text[i]) if q_text is not None else 0
            arr[i].k = _ptr(k[i])
            arr[i].v = _ptr(v[i])
        return arr

    @staticmethod
    def strides_of(q_text, k) -> air_strides:
        """Element strides of [B][H][T][d]-indexed tensors (any memory order with contiguous d)."""
        qs = q_text.stride() if q_text is not None else (0, 0, 0, 1)
        ks = k.stride()
        assert ks[3] == 1 and qs[3] == 1
        return air_strides(qs[0], qs[1], qs[2], ks[0], ks[1], ks[2])

    @staticmethod
    def seq_array(seqs) -> "C.Array":
        arr = (air_seq * len(seqs))()
        for i, s in enumerate(seqs):
            arr[i] = air_seq(s.seq_len, s.vis_start, s.vis_len, s.win_start, s.win_len)
        return arr

    # -- the four stages -------------------------------------------------------------
    def prepare(self, q_text: Optional[Sequence], k: Sequence, v: Sequence, seqs=None) -> "Prepared":
        """Marshal a set of layers once (descriptor arrays, strides, segments) for repeated stage calls."""
        return Prepared(self._layers(q_text, k, v), self.strides_of(q_text[0] if q_text is not None else None, k[0]),
                        self.seq_array(seqs) if seqs is not None else None, len(k), (q_text, k, v))

    def air_score(self, l0: int, l1: int, q_text=None, k=None, v=None, seqs=None, strides=None, prepared=None, stream=None):
        """prepared: result of prepare() for exactly the layers [l0, l1) (skips the per-call marshalling).
        stream (here and in the other stage calls): a raw HIP stream handle taken beforehand; default: torch's current stream."""
        p = prepared or self.prepare(q_text, k, v, seqs)
        st = strides or p.strides
        assert p.n == l1 - l0 and p.seqs is not None
        self._check(self.lib.air_score(self.handle, self._stream() if stream is None else stream, l0, l1, p.layers, C.byref(st),
                                       p.seqs))

    def air_budget(self, stream=None):
        self._check(self.lib.air_budget(self.handle, self._stream() if stream is None else stream))

    def air_reset(self):
        self._check(self.lib.air_reset(self.handle))

    def air_set_tuning(self, *, decode_splits=0, decode_waves=0, decode_tiles=0, score_block_mb=0, score_rows_kernel=0,
                       select_threads=0, select_direct_max=-1, gather_wgs=0, decode_order=0, decode_halves=0, budget_in_score=0):
        tn = air_tuning(decode_splits, decode_waves, decode_tiles, score_block_mb, score_rows_kernel, select_threads,
                        select_direct_max, gather_wgs, decode_order, decode_halves, budget_in_score)
        self._check(self.lib.air_set_tuning(self.handle, C.byref(tn)))

    def air_select_compact(self, l0: int, l1: int, k=None, v=None, strides=None, prepared=None, stream=None):
        p = prepared or self.prepare(None, k, v)
        st = strides or p.strides
        assert p.n == l1 - l0
        self._check(self.lib.air_select_compact(self.handle, self._stream() if stream is None else stream, l0, l1, p.layers,
                                                C.byref(st)))

    def air_decode_attn(self, l0: int, l1: int, q_new, k_new, v_new, out, stream=None):
        """Tensors, or raw device addresses (ints) when the caller has taken them beforehand."""
        if type(q_new) is not int:
            q_new, k_new, v_new, out = _ptr(q_new), _ptr(k_new), _ptr(v_new), _ptr(out)
        st = self.lib.air_decode_attn(self.handle, self._stream() if stream is None else stream, l0, l1, q_new, k_new, v_new, out)
        if st != AIR_OK:
            self._check(st)

    def air_decode_attn_static(self, l0: int, l1: int, q_new, k_new, v_new, out, stream=None):
        if type(q_new) is not int:
            q_new, k_new, v_new, out = _ptr(q_new), _ptr(k_new), _ptr(v_new), _ptr(out)
        st = self.lib.air_decode_attn_static(self.handle, self._stream() if stream is None else stream, l0, l1, q_new, k_new,
                                             v_new, out)
        if st != AIR_OK:
            self._check(st)

    # -- inspection ------------------------------------------------------------------
    def air_get_scores(self, l: int) -> np.ndarray:
        c = self.cfg
        out = np.empty((c.batch, c.n_kv_heads, c.max_vis_len), dtype=np.float32)
        self._check(self.lib.air_get_scores(self.handle, l, out.ctypes.data))
        return out

    def air_get_elite(self, l: int):
        c = self.cfg
        cnt = np.empty((c.batch, c.n_q_heads), dtype=np.int32)
        idx = np.empty((c.batch, c.n_q_heads, c.max_window), dtype=np.int32)
        self._check(self.lib.air_get_elite(self.handle, l, cnt.ctypes.data, idx.ctypes.data))
        return cnt, idx

    def air_get_stats(self):
        c = self.cfg
        s_t = np.empty((c.batch, c.n_layers), dtype=np.float64)
        s_k = np.empty((c.batch, c.n_layers), dtype=np.float64)
        self._check(self.lib.air_get_stats(self.handle, s_t.ctypes.data, s_k.ctypes.data))
        return s_t, s_k

    def air_get_budgets(self) -> np.ndarray:
        c = self.cfg
        out = np.empty((c.batch, c.n_layers), dtype=np.int32)
        self._check(self.lib.air_get_budgets(self.handle, out.ctypes.data))
        return out

    def air_set_budgets(self, budgets: np.ndarray):
        b = np.ascontiguousarray(budgets, dtype=np.int32)
        assert b.shape == (self.cfg.batch, self.cfg.n_layers)
        self._check(self.lib.air_set_budgets(self.handle, b.ctypes.data))

    def air_get_indices(self, l: int) -> np.ndarray:
        c = self.cfg
        out = np.empty((c.batch, c.n_kv_heads, c.max_vis_len), dtype=np.int32)
        self._check(self.lib.air_get_indices(self.handle, l, out.ctypes.data))
        return out

    def air_set_indices(self, l: int, indices: np.ndarray):
        c = self.cfg
        idx = np.ascontiguousarray(indices, dtype=np.int32)
        assert idx.shape == (c.batch, c.n_kv_heads, c.max_vis_len)
        self._check(self.lib.air_set_indices(self.handle, l, idx.ctypes.data))

    def air_get_lengths(self) -> np.ndarray:
        c = self.cfg
        out = np.empty((c.batch, c.n_layers), dtype=np.int32)
        self._check(self.lib.air_get_lengths(self.handle, out.ctypes.data))
        return out

    def air_get_cache(self, l: int, b: int, h: int, max_rows: int):
        """Rows of the compacted cache of (l, b, h) in the storage dtype (fp32 array or bf16 bit patterns)."""
        c = self.cfg
        dt = np.uint16 if c.dtype == AIR_BF16 else np.float32
        kk = np.zeros((max_rows, c.head_dim), dtype=dt)
        vv = np.zeros((max_rows, c.head_dim), dtype=dt)
        self._check(self.lib.air_get_cache(self.handle, l, b, h, kk.ctypes.data, vv.ctypes.data, max_rows))
        return kk, vv
