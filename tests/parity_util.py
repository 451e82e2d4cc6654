"""Comparison rules for HIP-vs-oracle parity (used by the GPU tests, smoke and bench)."""
from __future__ import annotations

import numpy as np
import torch

RTOL = {torch.float32: 1e-5, torch.bfloat16: 1e-3}
ATOL = 1e-30      # only forgives flushed denormals


def check_scores(got_f32: torch.Tensor, want_f64: torch.Tensor, dtype: torch.dtype, what: str = "") -> float:
    """|got - want| <= rtol * |want| + atol element by element; returns the worst relative error."""
    g = got_f32.detach().cpu().double().numpy()
    o = want_f64.detach().cpu().double().numpy()
    assert g.shape == o.shape, (g.shape, o.shape)
    assert np.isfinite(g).all(), "non-finite score " + what
    err = np.abs(g - o)
    bound = RTOL[dtype] * np.abs(o) + ATOL
    worst = float((err / np.maximum(np.abs(o), 1e-300)).max()) if g.size else 0.0
    bad = err > bound
    assert not bad.any(), "%s: %d / %d scores off, worst rel err %.3e (tol %.1e)" % (
        what, int(bad.sum()), g.size, worst, RTOL[dtype])
    return worst


def check_index_row(got: np.ndarray, oracle_pooled_f32: np.ndarray, W: int, budget: int, rtol: float,
                    what: str = "") -> bool:
    """Index-set rule for one KV head.

    `got` must hold min(budget, L) strictly increasing positions ending with the W window
    positions.  With t the oracle's k-th largest prefix score: everything above t(1+2 rtol)
    must be selected, nothing below t(1-2 rtol) may be.  If no unselected oracle score lies within
    that band of t, the set must equal the oracle's exactly (ties to the lowest position).
    Returns True when the exact comparison applied.
    """
    L = oracle_pooled_f32.shape[0]
    P = L - W
    Bk = min(budget, L)
    ksel = Bk - W
    assert got.shape == (Bk,), what
    assert (np.diff(got) > 0).all(), what + ": indices not strictly increasing"
    assert (got[ksel:] == np.arange(P, L)).all(), what + ": window not retained"
    if ksel == 0:
        return True
    assert got[ksel - 1] < P
    if ksel == P:
        assert (got[:P] == np.arange(P)).all()
        return True
    pref = oracle_pooled_f32[:P].astype(np.float64)
    order = np.lexsort((np.arange(P), -pref))          # score descending, position ascending
    want = np.sort(order[:ksel])
    t = pref[order[ksel - 1]]
    nxt = pref[order[ksel]]                            # best unselected score
    sel = np.zeros(P, dtype=bool)
    sel[got[:ksel]] = True
    must = pref > t * (1 + 2 * rtol)
    may = pref >= t * (1 - 2 * rtol)
    assert (sel[must]).all(), what + ": a clearly-above-threshold key was dropped"
    assert (may[sel]).all(), what + ": a clearly-below-threshold key was selected"
    exact = (nxt < t * (1 - 2 * rtol)) or (nxt == t and _plateau_safe(pref, t, rtol))
    if exact:
        assert (got[:ksel] == want).all(), what + ": index set differs from the oracle's"
    return bool(exact)


def _plateau_safe(pref: np.ndarray, t: float, rtol: float) -> bool:
    """True if the only scores within the tolerance band of t are bit-equal to t."""
    band = (pref >= t * (1 - 2 * rtol)) & (pref <= t * (1 + 2 * rtol))
    return bool((pref[band] == t).all())


def split_packed(flat: torch.Tensor, budgets, Hkv: int, L: int):
    """Packed idx / rows -> list of per-instance tensors [Hkv, Bk, ...]."""
    out, row = [], 0
    for b in budgets:
        bk = min(int(b), L)
        out.append(flat[row:row + Hkv * bk].reshape(Hkv, bk, *flat.shape[1:]))
        row += Hkv * bk
    assert row == flat.shape[0]
    return out
