"""ctypes front end of the CPU oracle (``laq_oracle.c``) -- TEST INFRASTRUCTURE ONLY.

Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of
``bench.py`` may import this package.  It never imports the HIP package, and
the HIP package never imports it.

The functions mirror the steps of the re-eviction procedure (paper Sec. 4.3,
Eq. 4): ``raw_scores`` (window attention summed over the Q-cache and the GQA
group), ``maxpool``, ``select`` (ArgSort[:B] per KV head with the window
retained) and ``compact`` (row gather).  ``evict`` chains them for one
instance; ``gather_paged`` writes a paged cache out densely first.  Tensors are CPU torch tensors (fp32 or bf16); results are fp64 /
int32 torch tensors.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Sequence, Tuple

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "laq_oracle.c")
_LIB = os.path.join(_HERE, "_build", "liblaq_oracle.so")
_lib: Optional[ctypes.CDLL] = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (plain -O2, no threading, no fast-math)."""
    os.makedirs(os.path.dirname(_LIB), exist_ok=True)
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(["gcc", "-O2", "-std=c99", "-shared", "-fPIC", "-Wall", "-Wextra",
                               "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def _load() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        c_int, c_dbl, c_vp = ctypes.c_int, ctypes.c_double, ctypes.c_void_p
        lib.laq_oracle_raw_scores.argtypes = [c_vp, c_vp, c_int, c_int, c_int, c_int, c_int, c_int,
                                              c_vp, c_dbl, c_vp]
        lib.laq_oracle_raw_scores.restype = c_int
        lib.laq_oracle_maxpool.argtypes = [c_vp, c_int, c_int, c_int, c_int, c_vp]
        lib.laq_oracle_maxpool.restype = c_int
        lib.laq_oracle_avgpool.argtypes = [c_vp, c_int, c_int, c_int, c_int, c_vp]
        lib.laq_oracle_avgpool.restype = c_int
        lib.laq_oracle_sink_recent.argtypes = [c_int, c_int, c_int, c_int, c_vp]
        lib.laq_oracle_sink_recent.restype = c_int
        lib.laq_oracle_overlap.argtypes = [c_vp, c_int, c_vp, c_int, c_int, c_int, c_vp]
        lib.laq_oracle_overlap.restype = c_int
        lib.laq_oracle_decode_attention.argtypes = [c_vp, c_vp, c_vp, c_int, c_int, c_int, c_int, c_int,
                                                    ctypes.c_double, c_vp]
        lib.laq_oracle_decode_attention.restype = c_int
        lib.laq_oracle_qcache_store.argtypes = [c_vp, c_int, c_int, c_int, ctypes.c_size_t, c_int, c_vp]
        lib.laq_oracle_qcache_store.restype = c_int
        lib.laq_oracle_select.argtypes = [c_vp, c_int, c_int, c_int, c_int, c_vp]
        lib.laq_oracle_select.restype = c_int
        lib.laq_oracle_compact.argtypes = [c_vp, c_int, c_int, ctypes.c_size_t, c_vp, c_int, c_vp]
        lib.laq_oracle_compact.restype = c_int
        _lib = lib
    return _lib


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return 0
    if t.dtype == torch.bfloat16:
        return 1
    raise TypeError("oracle takes fp32 or bf16 tensors, got %s" % t.dtype)


def _cpu(t: torch.Tensor) -> torch.Tensor:
    if t.device.type != "cpu":
        raise ValueError("the oracle works on host tensors")
    return t.contiguous()


def raw_scores(q_win: torch.Tensor, k: torch.Tensor, scale: float = 0.0,
               q_pos: Optional[Sequence[int]] = None) -> torch.Tensor:
    """Steps 1-4 for one instance: q_win [Hq, W, d], k [Hkv, L, d] -> raw [Hkv, L] fp64.

    q_pos: position of each of the W window queries in the key sequence (query w sees keys
    j <= q_pos[w]); None = the trailing window, q_pos[w] = L - W + w."""
    q_win, k = _cpu(q_win), _cpu(k)
    Hq, W, d = q_win.shape
    Hkv, L, d2 = k.shape
    if d != d2 or q_win.dtype != k.dtype:
        raise ValueError("q_win / k mismatch")
    raw = torch.empty(Hkv, L, dtype=torch.float64)
    pos = None
    if q_pos is not None:
        if len(q_pos) != W:
            raise ValueError("q_pos needs one entry per window query")
        pos = (ctypes.c_int32 * W)(*[int(x) for x in q_pos])
    rc = _load().laq_oracle_raw_scores(q_win.data_ptr(), k.data_ptr(), _dtype_code(k),
                                       Hq, Hkv, d, L, W, pos, float(scale), raw.data_ptr())
    if rc != 0:
        raise ValueError("laq_oracle_raw_scores rejected its arguments")
    return raw


def maxpool(raw: torch.Tensor, W: int, pool: int) -> torch.Tensor:
    """Step 5: raw [Hkv, L] fp64 -> pooled [Hkv, L] fp64; W = trailing keys always retained
    (prefix [0, L-W) pooled, the rest copied)."""
    raw = _cpu(raw.double())
    Hkv, L = raw.shape
    out = torch.empty_like(raw)
    rc = _load().laq_oracle_maxpool(raw.data_ptr(), Hkv, L, W, pool, out.data_ptr())
    if rc != 0:
        raise ValueError("laq_oracle_maxpool rejected its arguments")
    return out


def avgpool(raw: torch.Tensor, W: int, pool: int) -> torch.Tensor:
    """Step 5, average variant (Sec. 5.1): window mean with zeros outside the prefix [0, L-W);
    the trailing W columns are copied."""
    raw = _cpu(raw.double())
    Hkv, L = raw.shape
    out = torch.empty_like(raw)
    rc = _load().laq_oracle_avgpool(raw.data_ptr(), Hkv, L, W, pool, out.data_ptr())
    if rc != 0:
        raise ValueError("laq_oracle_avgpool rejected its arguments")
    return out


def sink_recent(Hkv: int, L: int, n_sink: int, budget: int) -> torch.Tensor:
    """Score-free stage-1 eviction (Sec. 4.2, StreamingLLM form): idx [Hkv, min(budget, L)] int32 =
    the first n_sink positions and the most recent ones."""
    Bk = min(int(budget), L)
    idx = torch.empty(Hkv, Bk, dtype=torch.int32)
    rc = _load().laq_oracle_sink_recent(Hkv, L, int(n_sink), int(budget), idx.data_ptr())
    if rc != 0:
        raise ValueError("laq_oracle_sink_recent rejected its arguments")
    return idx


def overlap(pred: torch.Tensor, gold: torch.Tensor, L: int) -> torch.Tensor:
    """Numerator of Eq. 3: pred [Hkv, n_pred], gold [Hkv, n_gold] int32 position lists (no repeats
    within a row) -> int32 [Hkv] sizes of the row-wise intersections.  Recall = overlap / n_gold."""
    pred, gold = _cpu(pred), _cpu(gold)
    if pred.dtype != torch.int32 or gold.dtype != torch.int32 or pred.shape[0] != gold.shape[0]:
        raise TypeError("overlap takes two int32 lists with the same number of rows")
    Hkv = pred.shape[0]
    out = torch.empty(Hkv, dtype=torch.int32)
    rc = _load().laq_oracle_overlap(pred.data_ptr() if pred.numel() else out.data_ptr(), pred.shape[1],
                                    gold.data_ptr() if gold.numel() else out.data_ptr(), gold.shape[1],
                                    Hkv, int(L), out.data_ptr())
    if rc != 0:
        raise ValueError("laq_oracle_overlap rejected its arguments")
    return out


def decode_attention(q: torch.Tensor, kc: torch.Tensor, vc: torch.Tensor, scale: float = 0.0) -> torch.Tensor:
    """Single-token attention over a compacted cache (Sec. 4.3): q [Hq, d], kc / vc [Hkv, Bk, d]
    -> out [Hq, d] fp64."""
    q, kc, vc = _cpu(q), _cpu(kc), _cpu(vc)
    if not (q.dtype == kc.dtype == vc.dtype) or kc.shape != vc.shape:
        raise TypeError("q, kc, vc share a dtype and kc, vc a shape")
    Hq, d = q.shape
    Hkv, Bk, _ = kc.shape
    out = torch.empty(Hq, d, dtype=torch.float64)
    rc = _load().laq_oracle_decode_attention(q.data_ptr(), kc.data_ptr(), vc.data_ptr(), _dtype_code(kc),
                                             Hq, Hkv, d, Bk, float(scale), out.data_ptr())
    if rc != 0:
        raise ValueError("laq_oracle_decode_attention rejected its arguments")
    return out


def qcache_store(q_cache: torch.Tensor, q_step: torch.Tensor, t: int) -> torch.Tensor:
    """Q-cache capture (Sec. 4.2): returns a copy of q_cache [Hq, W, d] whose row t holds q_step [Hq, d]."""
    q_step = _cpu(q_step)
    out = _cpu(q_cache).clone()
    Hq, W, d = out.shape
    if q_step.shape != (Hq, d) or q_step.dtype != out.dtype:
        raise TypeError("q_step is [Hq, d] in the cache's dtype")
    rc = _load().laq_oracle_qcache_store(q_step.data_ptr(), Hq, W, d, out.element_size(), int(t), out.data_ptr())
    if rc != 0:
        raise ValueError("laq_oracle_qcache_store rejected its arguments")
    return out


def select(scores_f32: torch.Tensor, W: int, budget: int) -> torch.Tensor:
    """Step 6: scores [Hkv, L] fp32 -> idx [Hkv, min(budget, L)] int32, ascending; W = trailing
    keys always retained."""
    if scores_f32.dtype != torch.float32:
        raise TypeError("selection is decided on fp32 scores")
    s = _cpu(scores_f32)
    Hkv, L = s.shape
    Bk = min(int(budget), L)
    idx = torch.empty(Hkv, Bk, dtype=torch.int32)
    rc = _load().laq_oracle_select(s.data_ptr(), Hkv, L, W, int(budget), idx.data_ptr())
    if rc != 0:
        raise ValueError("laq_oracle_select rejected its arguments")
    return idx


def compact(src: torch.Tensor, idx: torch.Tensor) -> torch.Tensor:
    """Step 7: src [Hkv, L, d], idx [Hkv, Bk] int32 -> [Hkv, Bk, d], bit copies."""
    src, idx = _cpu(src), _cpu(idx)
    Hkv, L, d = src.shape
    Bk = idx.shape[1]
    out = torch.empty(Hkv, Bk, d, dtype=src.dtype)
    rc = _load().laq_oracle_compact(src.data_ptr(), Hkv, L, d * src.element_size(),
                                    idx.data_ptr(), Bk, out.data_ptr())
    if rc != 0:
        raise ValueError("laq_oracle_compact rejected its arguments")
    return out


def gather_paged(pool: torch.Tensor, block_table: torch.Tensor, L: int) -> torch.Tensor:
    """A paged cache written out densely (the layout a serving engine hands to the re-eviction of
    Sec. 4.3): pool [n_blocks, Hkv, block_rows, d], block_table int [n, ceil(L / block_rows)] ->
    [n, Hkv, L, d].  Key row j of instance i is row j % block_rows of block block_table[i][j // block_rows].
    Plain loops over instances and blocks; the other functions then take the dense result."""
    pool, block_table = _cpu(pool), block_table.detach().cpu()
    n_blocks, Hkv, block_rows, d = pool.shape
    n, per = block_table.shape
    if per != -(-L // block_rows):
        raise ValueError("the table needs ceil(L / block_rows) entries per instance")
    out = torch.empty(n, Hkv, L, d, dtype=pool.dtype)
    for i in range(n):
        for b in range(per):
            blk = int(block_table[i, b])
            if not 0 <= blk < n_blocks:
                raise ValueError("block number out of range")
            rows = min(block_rows, L - b * block_rows)
            out[i, :, b * block_rows:b * block_rows + rows] = pool[blk, :, :rows]
    return out


def evict(q_win: torch.Tensor, k: torch.Tensor, v: Optional[torch.Tensor], budget: int,
          pool: int, scale: float = 0.0, q_pos: Optional[Sequence[int]] = None, keep: Optional[int] = None,
          pool_mode: str = "max") -> Tuple[torch.Tensor, torch.Tensor, torch.Tensor, Optional[torch.Tensor]]:
    """Whole path for one instance: returns (pooled fp64 [Hkv, L], idx, k', v').
    keep = trailing keys always retained (None: the number of window queries); pool_mode "max" or
    "avg"."""
    W = q_win.shape[1] if keep is None else int(keep)
    if pool_mode not in ("max", "avg"):
        raise ValueError("pool_mode is 'max' or 'avg'")
    pooled = (maxpool if pool_mode == "max" else avgpool)(raw_scores(q_win, k, scale, q_pos), W, pool)
    idx = select(pooled.float(), W, budget)
    return pooled, idx, compact(k, idx), (compact(v, idx) if v is not None else None)
