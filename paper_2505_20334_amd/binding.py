"""ctypes binding of ``liblaq.so`` -- argument marshalling only.

Function names and argument meaning follow ``include/laq.h``.  Tensors are torch
tensors that already live on the GPU (torch supplies device memory and the
stream, nothing else); every step of the path runs in the library's kernels.
"""
from __future__ import annotations

import ctypes
import os
from typing import List, Optional, Sequence, Tuple

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_PKG, "liblaq.so")
_lib: Optional[ctypes.CDLL] = None

LAQ_F32, LAQ_BF16 = 0, 1
LAQ_POOL_MAX, LAQ_POOL_AVG = 0, 1


class LaqError(RuntimeError):
    def __init__(self, code: int, what: str):
        super().__init__("%s failed: %s (code %d)" % (what, laq_strerror(code), code))
        self.code = code


class _Shape(ctypes.Structure):
    _fields_ = [("n_inst", ctypes.c_int32), ("Hq", ctypes.c_int32), ("Hkv", ctypes.c_int32),
                ("d", ctypes.c_int32), ("L", ctypes.c_int32), ("W", ctypes.c_int32),
                ("dtype", ctypes.c_int32), ("scale", ctypes.c_float),
                ("q_pos", ctypes.POINTER(ctypes.c_int32)), ("keep", ctypes.c_int32),
                ("pool_mode", ctypes.c_int32), ("kv_stride_inst", ctypes.c_int64),
                ("kv_stride_head", ctypes.c_int64), ("kv_stride_row", ctypes.c_int64),
                ("block_table", ctypes.c_void_p), ("block_rows", ctypes.c_int32),
                ("kv_stride_block", ctypes.c_int64), ("score_choice", ctypes.c_int32)]


def lib_path() -> str:
    return _LIB_PATH


def load_library() -> ctypes.CDLL:
    """Load the built library (building it first if nothing is built); raises if that is impossible --
    there is no fallback path."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        # nothing built yet: build once (hipcc); there is no other way to run, so a failure is final
        try:
            from . import _build
            _build.build()
        except Exception as exc:
            raise ImportError("liblaq.so is not built and building it failed (%s): run "
                              "`python -c 'import __graft_entry__ as g; g.build()'`" % exc)
    lib = ctypes.CDLL(_LIB_PATH)
    vp, i32, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t
    sp = ctypes.POINTER(_Shape)
    lib.laq_workspace_bytes.argtypes = [sp]
    lib.laq_workspace_bytes.restype = sz
    lib.laq_score.argtypes = [sp, vp, vp, i32, vp, vp, sz, vp]
    lib.laq_score.restype = i32
    lib.laq_select.argtypes = [sp, vp, ctypes.POINTER(ctypes.c_int32), i32, vp, vp]
    lib.laq_select.restype = i32
    lib.laq_select_sink_recent.argtypes = [i32, i32, i32, ctypes.POINTER(ctypes.c_int32), i32, vp, vp]
    lib.laq_select_sink_recent.restype = i32
    bp = ctypes.POINTER(ctypes.c_int32)
    lib.laq_decode_attention.argtypes = [sp, vp, vp, vp, bp, vp, vp, sz, vp]
    lib.laq_decode_attention.restype = i32
    lib.laq_decode_workspace_bytes.argtypes = [sp, bp]
    lib.laq_decode_workspace_bytes.restype = sz
    lib.laq_qcache_store.argtypes = [sp, vp, i32, vp, vp]
    lib.laq_qcache_store.restype = i32
    lib.laq_recall.argtypes = [i32, i32, i32, vp, bp, vp, bp, vp, vp, vp]
    lib.laq_recall.restype = i32
    lib.laq_compact.argtypes = [sp, vp, vp, vp, ctypes.POINTER(ctypes.c_int32), vp, vp, vp]
    lib.laq_compact.restype = i32
    lib.laq_evict.argtypes = [sp, vp, vp, vp, ctypes.POINTER(ctypes.c_int32), i32, vp, vp, vp, vp, vp, sz, vp]
    lib.laq_evict.restype = i32
    lib.laq_strerror.argtypes = [i32]
    lib.laq_strerror.restype = ctypes.c_char_p
    lib.laq_evict_static.argtypes = [sp, vp, vp, vp, ctypes.POINTER(ctypes.c_int32), i32, vp, vp, vp, vp, vp]
    lib.laq_evict_static.restype = i32
    lib.laq_init.argtypes = []
    lib.laq_init.restype = i32
    lib.laq_workspace_status.argtypes = [sp, vp, sz, vp]
    lib.laq_workspace_status.restype = i32
    lib.laq_score_kernel.argtypes = [sp]
    lib.laq_score_kernel.restype = i32
    _lib = lib
    return lib


def laq_strerror(code: int) -> str:
    return load_library().laq_strerror(int(code)).decode()


def laq_init() -> None:
    """One-time set-up of the library for torch's current device (optional; needed before a first call
    that is recorded by a stream capture)."""
    rc = load_library().laq_init()
    if rc != 0:
        raise LaqError(rc, "laq_init")


def laq_workspace_status(ws: torch.Tensor, n_inst: int, Hq: int, Hkv: int, d: int, L: int, W: int,
                         dtype: torch.dtype, stream=None) -> int:
    """0 if the last scoring call on this workspace completed all its waits (synchronises the stream)."""
    code = LAQ_F32 if dtype == torch.float32 else LAQ_BF16
    sh = _shape(n_inst, Hq, Hkv, d, L, W, code, 0.0)
    return int(load_library().laq_workspace_status(ctypes.byref(sh), ws.data_ptr(), ws.numel() * ws.element_size(),
                                                   _stream(stream)))


SCORE_KERNELS = ("vector", "two-pass", "single-read")


def laq_score_kernel(n_inst: int, Hq: int, Hkv: int, d: int, L: int, W: int, dtype: torch.dtype,
                     q_pos: Optional[Sequence[int]] = None, keep: Optional[int] = None,
                     kv_strides: Tuple[int, int, int] = (0, 0, 0), paged=None, choose: str = "auto") -> str:
    """Which kernels laq_score takes for this shape on the current device: "vector", "two-pass"
    (K streamed twice) or "single-read" (K read once)."""
    code = LAQ_F32 if dtype == torch.float32 else LAQ_BF16
    sh = _shape(n_inst, Hq, Hkv, d, L, W, code, 0.0, q_pos, keep, "max", kv_strides, paged, choose)
    rc = int(load_library().laq_score_kernel(ctypes.byref(sh)))
    if rc < 0:
        raise LaqError(rc, "laq_score_kernel")
    return SCORE_KERNELS[rc]


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return LAQ_F32
    if t.dtype == torch.bfloat16:
        return LAQ_BF16
    raise TypeError("LAQ takes fp32 or bf16 tensors, got %s" % t.dtype)


def _dev(t: torch.Tensor, name: str) -> torch.Tensor:
    if t.device.type != "cuda":
        raise ValueError("%s must live on the GPU" % name)
    if not t.is_contiguous():
        raise ValueError("%s must be dense (contiguous)" % name)
    return t


def _kv(t: torch.Tensor, name: str) -> Tuple[int, int, int]:
    """k / v [n, Hkv, L, d] on the GPU with contiguous rows; returns its (instance, head, row) strides in
    elements ((0, 0, 0) for a dense tensor).  A view of a token-major cache, k_tm.permute(0, 2, 1, 3), is fine."""
    if t.device.type != "cuda":
        raise ValueError("%s must live on the GPU" % name)
    if t.dim() != 4 or t.stride(3) != 1:
        raise ValueError("%s must be [n, Hkv, L, d] with contiguous rows" % name)
    if t.is_contiguous():
        return (0, 0, 0)
    return (t.stride(0), t.stride(1), t.stride(2))


def _cache(k: torch.Tensor, name: str, block_table: Optional[torch.Tensor], L: Optional[int]):
    """The cache a call reads: (n, Hkv, L, d, strides, paged).  Without a block table k is
    [n, Hkv, L, d] (strided views allowed).  With one, k is a pool of blocks [n_blocks, Hkv, block_rows, d]
    (or a strided view of that shape, e.g. of token-major blocks), block_table is int32 [n, ceil(L /
    block_rows)] on the same device and L must be given."""
    if block_table is None:
        if L is not None and L != k.shape[2]:
            raise ValueError("L is only given with a block table")
        kvs = _kv(k, name)
        return k.shape[0], k.shape[1], k.shape[2], k.shape[3], kvs, None
    if L is None:
        raise ValueError("a paged cache needs L, the number of key rows per instance")
    if k.device.type != "cuda" or k.dim() != 4 or k.stride(3) != 1:
        raise ValueError("%s must be a pool [n_blocks, Hkv, block_rows, d] on the GPU with contiguous rows" % name)
    if block_table.device != k.device or block_table.dtype != torch.int32 or block_table.dim() != 2 \
            or not block_table.is_contiguous():
        raise ValueError("block_table must be a dense int32 [n, blocks per instance] tensor on %s" % k.device)
    n_blocks, Hkv, block_rows, d = k.shape
    if block_rows % 256 or block_table.shape[1] != -(-int(L) // block_rows):
        raise ValueError("blocks hold a multiple of 256 rows and the table ceil(L / block_rows) entries per instance")
    inner = (0, 0, 0) if (k.stride(1) == block_rows * d and k.stride(2) == d) else (0, k.stride(1), k.stride(2))
    return block_table.shape[0], Hkv, int(L), d, inner, (block_table, block_rows, k.stride(0))


def _out(t: Optional[torch.Tensor], name: str, dtype: torch.dtype, numel: int, like: torch.Tensor) -> None:
    """A caller-supplied output buffer must be what the kernels will write: right dtype and device, dense,
    at least `numel` elements, 16-byte aligned."""
    if t is None:
        return
    if t.device != like.device:
        raise ValueError("%s must live on %s" % (name, like.device))
    if t.dtype != dtype:
        raise TypeError("%s must be %s" % (name, dtype))
    if not t.is_contiguous():
        raise ValueError("%s must be dense (contiguous)" % name)
    if t.numel() < numel:
        raise ValueError("%s needs at least %d elements, has %d" % (name, numel, t.numel()))
    if t.data_ptr() % 16:
        raise ValueError("%s must be 16-byte aligned" % name)


def _aligned(t: torch.Tensor, name: str) -> None:
    if t.data_ptr() % 16:
        raise ValueError("%s must be 16-byte aligned" % name)


def _stream(stream) -> int:
    if stream is None:
        return torch.cuda.current_stream().cuda_stream
    return stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream)


def _shape(n: int, Hq: int, Hkv: int, d: int, L: int, W: int, dtype: int, scale: float,
           q_pos: Optional[Sequence[int]] = None, keep: Optional[int] = None, pool_mode: str = "max",
           kv_strides: Tuple[int, int, int] = (0, 0, 0), paged=None, choose: str = "auto") -> _Shape:
    """q_pos: position of every window query in the key sequence (None: the trailing window);
    keep: trailing keys always retained (None: W); pool_mode "max" or "avg"; paged: None or (block
    table tensor, rows per block, element stride between blocks).  The position array and the table
    stay alive with the struct."""
    if pool_mode not in ("max", "avg"):
        raise ValueError("pool_mode is 'max' or 'avg'")
    sh = _Shape(n, Hq, Hkv, d, L, W, dtype, float(scale), None, -1 if keep is None else int(keep),
                LAQ_POOL_AVG if pool_mode == "avg" else LAQ_POOL_MAX, int(kv_strides[0]), int(kv_strides[1]),
                int(kv_strides[2]), None, 0, 0, ("auto", "two-pass", "single-read").index(choose))
    if paged is not None:
        sh._table_keepalive = paged[0]
        sh.block_table = paged[0].data_ptr()
        sh.block_rows = int(paged[1])
        sh.kv_stride_block = int(paged[2])
    if q_pos is not None:
        if len(q_pos) != W:
            raise ValueError("q_pos needs one entry per window query")
        sh._q_pos_keepalive = (ctypes.c_int32 * W)(*[int(x) for x in q_pos])
        sh.q_pos = ctypes.cast(sh._q_pos_keepalive, ctypes.POINTER(ctypes.c_int32))
    return sh


def _budget_array(budget: Sequence[int], n: int):
    if len(budget) != n:
        raise ValueError("budget needs one entry per instance")
    return (ctypes.c_int32 * n)(*[int(b) for b in budget])


def packed_rows(budget: Sequence[int], Hkv: int, L: int) -> Tuple[int, List[int]]:
    """Total packed rows of idx / k_out / v_out and the first row of each instance."""
    starts, row = [], 0
    for b in budget:
        starts.append(row)
        row += Hkv * min(int(b), L)
    return row, starts


def laq_workspace_bytes(n_inst: int, Hq: int, Hkv: int, d: int, L: int, W: int, dtype: torch.dtype,
                        q_pos: Optional[Sequence[int]] = None, keep: Optional[int] = None) -> int:
    code = LAQ_F32 if dtype == torch.float32 else LAQ_BF16
    sh = _shape(n_inst, Hq, Hkv, d, L, W, code, 0.0, q_pos, keep)
    return int(load_library().laq_workspace_bytes(ctypes.byref(sh)))


def _workspace(q_win, k, ws, q_pos=None, keep=None, Hkv=None, L=None):
    n, Hq, W, d = q_win.shape
    if Hkv is None:
        _, Hkv, L, _ = k.shape
    need = laq_workspace_bytes(n, Hq, Hkv, d, L, W, k.dtype, q_pos, keep)
    if ws is None:
        ws = torch.empty(need, dtype=torch.uint8, device=k.device)
    elif ws.device != k.device or not ws.is_contiguous() or ws.data_ptr() % 256:
        raise ValueError("ws must be a dense, 256-byte aligned tensor on %s" % k.device)
    return ws, ws.numel() * ws.element_size()


def laq_score(q_win: torch.Tensor, k: torch.Tensor, pool_kernel: int = 1, scale: float = 0.0,
              scores: Optional[torch.Tensor] = None, ws: Optional[torch.Tensor] = None,
              stream=None, q_pos: Optional[Sequence[int]] = None, keep: Optional[int] = None,
              pool_mode: str = "max", block_table: Optional[torch.Tensor] = None,
              L: Optional[int] = None, choose: str = "auto") -> torch.Tensor:
    """q_win [n, Hq, W, d], k [n, Hkv, L, d] -> scores [n, Hkv, L] fp32 (pooled if pool_kernel > 1).
    q_pos / keep: the general observation window of laq_shape (None: trailing window); pool_mode:
    "max" or "avg" (laq_pool_mode); block_table / L: k is a paged cache (see _cache); choose: "auto",
    "two-pass" or "single-read" (laq_score_choice)."""
    lib = load_library()
    _dev(q_win, "q_win")
    n, Hq, W, d = q_win.shape
    n2, Hkv, L, d2, kvs, paged = _cache(k, "k", block_table, L)
    if n != n2 or d != d2 or q_win.dtype != k.dtype:
        raise ValueError("q_win / k mismatch")
    _aligned(q_win, "q_win"), _aligned(k, "k")
    _out(scores, "scores", torch.float32, n * Hkv * L, k)
    if scores is None:
        scores = torch.empty(n, Hkv, L, dtype=torch.float32, device=k.device)
    ws, ws_bytes = _workspace(q_win, k, ws, q_pos, keep, Hkv, L)
    sh = _shape(n, Hq, Hkv, d, L, W, _dtype_code(k), scale, q_pos, keep, pool_mode, kvs, paged, choose)
    rc = lib.laq_score(ctypes.byref(sh), q_win.data_ptr(), k.data_ptr(), int(pool_kernel), scores.data_ptr(),
                       ws.data_ptr(), ws_bytes, _stream(stream))
    if rc != 0:
        raise LaqError(rc, "laq_score")
    return scores


def laq_select(scores: torch.Tensor, budget: Sequence[int], pool_kernel: int, keep: int,
               idx: Optional[torch.Tensor] = None, stream=None, pool_mode: str = "max") -> torch.Tensor:
    """scores [n, Hkv, L] fp32 -> packed idx (int32, see packed_rows); keep = trailing keys always
    retained (the window size W in the trailing-window layout); pool_mode as in laq_score."""
    lib = load_library()
    _dev(scores, "scores")
    if scores.dtype != torch.float32:
        raise TypeError("scores must be fp32")
    n, Hkv, L = scores.shape
    total, _ = packed_rows(budget, Hkv, L)
    _out(idx, "idx", torch.int32, total, scores)
    if idx is None:
        idx = torch.empty(total, dtype=torch.int32, device=scores.device)
    sh = _shape(n, Hkv, Hkv, 8, L, 1, LAQ_F32, 0.0, None, keep, pool_mode)
    rc = lib.laq_select(ctypes.byref(sh), scores.data_ptr(), _budget_array(budget, n), int(pool_kernel),
                        idx.data_ptr(), _stream(stream))
    if rc != 0:
        raise LaqError(rc, "laq_select")
    return idx


def laq_select_sink_recent(n_inst: int, Hkv: int, L: int, budget: Sequence[int], n_sink: int,
                           idx: Optional[torch.Tensor] = None, device=None, stream=None) -> torch.Tensor:
    """Score-free stage-1 list: packed idx (as laq_select packs it) holding, per KV head, the first
    n_sink positions and the most recent ones.  `device` places a newly made idx (default cuda:0)."""
    lib = load_library()
    total, _ = packed_rows(budget, Hkv, L)
    if idx is None:
        idx = torch.empty(total, dtype=torch.int32, device=device if device is not None else "cuda:0")
    _dev(idx, "idx")
    if idx.dtype != torch.int32 or idx.numel() < total:
        raise ValueError("idx must be int32 with at least %d entries" % total)
    rc = lib.laq_select_sink_recent(int(n_inst), int(Hkv), int(L), _budget_array(budget, n_inst), int(n_sink),
                                    idx.data_ptr(), _stream(stream))
    if rc != 0:
        raise LaqError(rc, "laq_select_sink_recent")
    return idx


def laq_recall(idx_pred: torch.Tensor, budget_pred: Sequence[int], idx_gold: torch.Tensor,
               budget_gold: Sequence[int], Hkv: int, L: int, stream=None) -> Tuple[torch.Tensor, torch.Tensor]:
    """Two packed index lists (as laq_select writes them) -> (overlap int32 [n, Hkv], recall fp32
    [n, Hkv]) with recall = |pred ∩ gold| / |gold| per KV head."""
    lib = load_library()
    _dev(idx_pred, "idx_pred"), _dev(idx_gold, "idx_gold")
    n = len(budget_pred)
    if len(budget_gold) != n:
        raise ValueError("the two budget arrays need one entry per instance each")
    if idx_pred.dtype != torch.int32 or idx_gold.dtype != torch.int32:
        raise TypeError("index lists are int32")
    if idx_pred.numel() < packed_rows(budget_pred, Hkv, L)[0] or idx_gold.numel() < packed_rows(budget_gold, Hkv, L)[0]:
        raise ValueError("an index list is shorter than its budgets say")
    overlap = torch.empty(n, Hkv, dtype=torch.int32, device=idx_pred.device)
    recall = torch.empty(n, Hkv, dtype=torch.float32, device=idx_pred.device)
    rc = lib.laq_recall(n, int(Hkv), int(L), idx_pred.data_ptr(), _budget_array(budget_pred, n),
                        idx_gold.data_ptr(), _budget_array(budget_gold, n), overlap.data_ptr(), recall.data_ptr(),
                        _stream(stream))
    if rc != 0:
        raise LaqError(rc, "laq_recall")
    return overlap, recall


def laq_qcache_store(q_cache: torch.Tensor, q_step: torch.Tensor, t: int, stream=None) -> torch.Tensor:
    """q_cache [n, Hq, W, d] (updated in place: rows [.., t, :] = q_step [n, Hq, d]); returns q_cache."""
    lib = load_library()
    _dev(q_cache, "q_cache"), _dev(q_step, "q_step")
    n, Hq, W, d = q_cache.shape
    if q_step.shape != (n, Hq, d) or q_step.dtype != q_cache.dtype:
        raise ValueError("q_step is [n, Hq, d] in the cache's dtype")
    sh = _shape(n, Hq, Hq, d, max(W, 1), W, _dtype_code(q_cache), 0.0, None, 0)
    rc = lib.laq_qcache_store(ctypes.byref(sh), q_step.data_ptr(), int(t), q_cache.data_ptr(), _stream(stream))
    if rc != 0:
        raise LaqError(rc, "laq_qcache_store")
    return q_cache


def laq_decode_attention(q: torch.Tensor, k_c: torch.Tensor, v_c: torch.Tensor, budget: Sequence[int],
                         Hkv: int, L: int, scale: float = 0.0, out: Optional[torch.Tensor] = None,
                         stream=None, ws: Optional[torch.Tensor] = None, split: bool = True) -> torch.Tensor:
    """q [n, Hq, d] and the packed k_c, v_c [rows, d] of laq_compact -> out [n, Hq, d] fp32: one new
    token's attention over the retained rows of its KV head.  split: let the library spread long
    caches over several workgroups (a workspace of laq_decode_workspace_bytes is made if ws is None)."""
    lib = load_library()
    _dev(q, "q"), _dev(k_c, "k_c"), _dev(v_c, "v_c")
    n, Hq, d = q.shape
    total, _ = packed_rows(budget, Hkv, L)
    if k_c.shape != (total, d) or v_c.shape != (total, d) or not (q.dtype == k_c.dtype == v_c.dtype):
        raise ValueError("k_c / v_c must be the packed [rows, d] tensors of these budgets, in q's dtype")
    _out(out, "out", torch.float32, n * Hq * d, q)
    if out is None:
        out = torch.empty(n, Hq, d, dtype=torch.float32, device=q.device)
    sh = _shape(n, Hq, Hkv, d, L, 1, _dtype_code(q), scale, None, 0)
    bud = _budget_array(budget, n)
    if split and ws is None:
        need = int(lib.laq_decode_workspace_bytes(ctypes.byref(sh), bud))
        if need:
            ws = torch.empty(need, dtype=torch.uint8, device=q.device)
    if not split:
        ws = None
    rc = lib.laq_decode_attention(ctypes.byref(sh), q.data_ptr(), k_c.data_ptr(), v_c.data_ptr(), bud, out.data_ptr(),
                                  ws.data_ptr() if ws is not None else None,
                                  ws.numel() * ws.element_size() if ws is not None else 0, _stream(stream))
    if rc != 0:
        raise LaqError(rc, "laq_decode_attention")
    return out


def laq_decode_workspace_bytes(n_inst: int, Hq: int, Hkv: int, d: int, L: int, dtype: torch.dtype,
                               budget: Sequence[int]) -> int:
    code = LAQ_F32 if dtype == torch.float32 else LAQ_BF16
    sh = _shape(n_inst, Hq, Hkv, d, L, 1, code, 0.0, None, 0)
    return int(load_library().laq_decode_workspace_bytes(ctypes.byref(sh), _budget_array(budget, n_inst)))


def laq_compact(k: torch.Tensor, v: Optional[torch.Tensor], idx: torch.Tensor, budget: Sequence[int], keep: int,
                k_out: Optional[torch.Tensor] = None, v_out: Optional[torch.Tensor] = None, stream=None,
                block_table: Optional[torch.Tensor] = None, L: Optional[int] = None):
    """k, v [n, Hkv, L, d] + packed idx -> packed k_out, v_out [rows, d]; keep as in laq_select
    (only used to check the budgets); block_table / L: k, v are paged caches (see _cache)."""
    lib = load_library()
    _dev(idx, "idx")
    n, Hkv, L, d, kvs, paged = _cache(k, "k", block_table, L)
    total, _ = packed_rows(budget, Hkv, L)
    if idx.dtype != torch.int32 or idx.numel() < total:
        raise ValueError("idx must be int32 with at least %d entries" % total)
    _aligned(k, "k")
    _out(k_out, "k_out", k.dtype, total * d, k)
    if k_out is None:
        k_out = torch.empty(total, d, dtype=k.dtype, device=k.device)
    if v is not None:
        if v.shape != k.shape or v.dtype != k.dtype or v.stride() != k.stride():
            raise ValueError("k / v mismatch (shape, dtype or strides)")
        _aligned(v, "v")
        _out(v_out, "v_out", k.dtype, total * d, k)
        if v_out is None:
            v_out = torch.empty(total, d, dtype=k.dtype, device=k.device)
    elif v_out is not None:
        raise ValueError("v_out without v")
    sh = _shape(n, Hkv, Hkv, d, L, 1, _dtype_code(k), 0.0, None, keep, "max", kvs, paged)
    rc = lib.laq_compact(ctypes.byref(sh), k.data_ptr(), v.data_ptr() if v is not None else None,
                         idx.data_ptr(), _budget_array(budget, n), k_out.data_ptr(),
                         v_out.data_ptr() if v is not None else None, _stream(stream))
    if rc != 0:
        raise LaqError(rc, "laq_compact")
    return k_out, v_out


def laq_evict(q_win: torch.Tensor, k: torch.Tensor, v: Optional[torch.Tensor], budget: Sequence[int],
              pool_kernel: int, scale: float = 0.0, scores=None, idx=None, k_out=None, v_out=None, ws=None,
              stream=None, q_pos: Optional[Sequence[int]] = None, keep: Optional[int] = None,
              pool_mode: str = "max", want_scores: bool = True, static_scratch: bool = False,
              block_table: Optional[torch.Tensor] = None, L: Optional[int] = None, choose: str = "auto"):
    """Whole path on one stream: returns (scores, idx, k_out, v_out); layouts as in the three calls.
    want_scores=False (and no scores buffer): the library hands the scores over inside the workspace and
    None is returned in their place.  static_scratch=True calls laq_evict_static (the library's own scratch
    array instead of a workspace; every output buffer must then be passed in for the call to allocate nothing)."""
    lib = load_library()
    _dev(q_win, "q_win")
    n, Hq, W, d = q_win.shape
    n2, Hkv, L, d2, kvs, paged = _cache(k, "k", block_table, L)
    if n != n2 or d != d2 or q_win.dtype != k.dtype:
        raise ValueError("q_win / k mismatch")
    total, _ = packed_rows(budget, Hkv, L)
    _aligned(q_win, "q_win"), _aligned(k, "k")
    _out(scores, "scores", torch.float32, n * Hkv * L, k)
    _out(idx, "idx", torch.int32, total, k)
    _out(k_out, "k_out", k.dtype, total * d, k)
    if scores is None and want_scores:
        scores = torch.empty(n, Hkv, L, dtype=torch.float32, device=k.device)
    if idx is None:
        idx = torch.empty(total, dtype=torch.int32, device=k.device)
    if k_out is None:
        k_out = torch.empty(total, d, dtype=k.dtype, device=k.device)
    if v is not None:
        if v.shape != k.shape or v.dtype != k.dtype or v.stride() != k.stride():
            raise ValueError("k / v mismatch (shape, dtype or strides)")
        _aligned(v, "v")
        _out(v_out, "v_out", k.dtype, total * d, k)
        if v_out is None:
            v_out = torch.empty(total, d, dtype=k.dtype, device=k.device)
    elif v_out is not None:
        raise ValueError("v_out without v")
    sh = _shape(n, Hq, Hkv, d, L, W, _dtype_code(k), scale, q_pos, keep, pool_mode, kvs, paged, choose)
    if static_scratch:
        rc = lib.laq_evict_static(ctypes.byref(sh), q_win.data_ptr(), k.data_ptr(),
                                  v.data_ptr() if v is not None else None, _budget_array(budget, n), int(pool_kernel),
                                  scores.data_ptr() if scores is not None else None, idx.data_ptr(), k_out.data_ptr(),
                                  v_out.data_ptr() if v is not None else None, _stream(stream))
        if rc != 0:
            raise LaqError(rc, "laq_evict_static")
        return scores, idx, k_out, v_out
    ws, ws_bytes = _workspace(q_win, k, ws, q_pos, keep, Hkv, L)
    rc = lib.laq_evict(ctypes.byref(sh), q_win.data_ptr(), k.data_ptr(), v.data_ptr() if v is not None else None,
                       _budget_array(budget, n), int(pool_kernel),
                       scores.data_ptr() if scores is not None else None, idx.data_ptr(),
                       k_out.data_ptr(), v_out.data_ptr() if v is not None else None, ws.data_ptr(), ws_bytes,
                       _stream(stream))
    if rc != 0:
        raise LaqError(rc, "laq_evict")
    return scores, idx, k_out, v_out
