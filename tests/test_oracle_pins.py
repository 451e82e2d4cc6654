"""Pins for the CPU oracle (no GPU): each test fixes the oracle against something
other than itself -- brute force written independently here, closed forms,
invariants, metamorphic relations, hand-computed fixtures, library routines on
special cases -- so that a dropped term, a wrong sign or index, a transposed
operand or an off-by-one in the mask fails at least one of them.

The paper (Sec. 4.3, Eq. 4) prints no worked numeric example for this path.
"""
import math
import os
from fractions import Fraction

import numpy as np
import pytest
import torch

import oracle
from laq_inputs import CONFIGS, budgets_for, make_instance, pyramid_budget

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ----------------------------------------------------------------------------
# independent brute force: the explicit [Hq, W, L] attention matrix with a
# boolean mask, written with numpy array ops (no shared code with the oracle)
# ----------------------------------------------------------------------------
def brute_raw(q, k, scale=None):
    q = q.double().numpy()
    k = k.double().numpy()
    Hq, W, d = q.shape
    Hkv, L, _ = k.shape
    G = Hq // Hkv
    P = L - W
    scale = 1.0 / math.sqrt(d) if scale is None else scale
    kk = np.repeat(k, G, axis=0)                               # [Hq, L, d]
    S = np.einsum("hwc,hjc->hwj", q, kk) * scale               # [Hq, W, L]
    pos_q = P + np.arange(W)[:, None]                          # query positions
    visible = np.arange(L)[None, :] <= pos_q                   # [W, L]
    S = np.where(visible[None], S, -np.inf)
    S = S - S.max(axis=2, keepdims=True)
    E = np.exp(S)
    A = E / E.sum(axis=2, keepdims=True)                       # attention rows
    return A.reshape(Hkv, G, W, L).sum(axis=(1, 2))            # [Hkv, L]


def brute_pool(raw, W, pool):
    Hkv, L = raw.shape
    P = L - W
    out = raw.copy()
    h = pool // 2
    for g in range(Hkv):
        for j in range(P):
            out[g, j] = max(raw[g, i] for i in range(max(0, j - h), min(P, j + h + 1)))
    return out


def brute_select(scores, W, budget):
    Hkv, L = scores.shape
    P = L - W
    Bk = min(budget, L)
    out = np.zeros((Hkv, Bk), dtype=np.int32)
    for g in range(Hkv):
        order = sorted(range(P), key=lambda j: (-float(scores[g, j]), j))
        out[g] = sorted(order[:Bk - W]) + list(range(P, L))
    return out


def rand_case(seed, Hq, Hkv, d, L, W, dtype=torch.float32, qscale=1.0):
    g = torch.Generator().manual_seed(seed)
    q = (torch.randn(Hq, W, d, generator=g) * qscale).to(dtype)
    k = torch.randn(Hkv, L, d, generator=g).to(dtype)
    v = torch.randn(Hkv, L, d, generator=g).to(dtype)
    return q, k, v


# ----------------------------------------------------------------------------
@pytest.mark.parametrize("Hq,Hkv,d,L,W", [
    (1, 1, 4, 9, 1), (2, 1, 8, 17, 3), (4, 2, 8, 32, 5), (6, 2, 16, 23, 8), (3, 3, 5, 12, 12),
])
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_raw_scores_match_explicit_attention_matrix(Hq, Hkv, d, L, W, dtype):
    q, k, _ = rand_case(7 + L, Hq, Hkv, d, L, W, dtype, qscale=2.0)
    got = oracle.raw_scores(q, k).numpy()
    want = brute_raw(q, k)
    np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-15)


def test_explicit_scale_is_used():
    q, k, _ = rand_case(3, 2, 1, 8, 20, 4)
    got = oracle.raw_scores(q, k, scale=0.37).numpy()
    np.testing.assert_allclose(got, brute_raw(q, k, scale=0.37), rtol=1e-12)
    default = oracle.raw_scores(q, k).numpy()
    np.testing.assert_allclose(default, brute_raw(q, k, scale=1 / math.sqrt(8)), rtol=1e-12)
    assert not np.allclose(got, default)


def test_rows_sum_to_one_and_nonnegative():
    # every one of the Hq*W attention rows sums to 1, so each KV head's raw row sums to G*W
    q, k, _ = rand_case(11, 8, 2, 16, 300, 6, qscale=3.0)
    raw = oracle.raw_scores(q, k).numpy()
    assert (raw >= 0).all()
    np.testing.assert_allclose(raw.sum(axis=1), np.full(2, 4 * 6.0), rtol=1e-12)


def test_causal_mask_window_columns():
    # window key P+w' is visible only to queries w >= w'; the last column gets mass from one
    # query per head only, and a huge logit there must not leak into earlier queries' rows
    Hq, Hkv, d, L, W = 2, 1, 4, 10, 4
    q = torch.ones(Hq, W, d)
    k = torch.zeros(Hkv, L, d)
    k[0, L - 1] = 50.0                        # dominant for the one query that can see it
    raw = oracle.raw_scores(q, k, scale=1.0).numpy()[0]
    P = L - W
    # queries w < W-1 see P+w+1 identical (zero) keys -> uniform
    expect = np.zeros(L)
    for w in range(W - 1):
        expect[:P + w + 1] += Hq / (P + w + 1)
    expect[L - 1] += Hq * 1.0                 # last query: all mass on the heavy key (e^-200 elsewhere)
    np.testing.assert_allclose(raw, expect, rtol=1e-12, atol=1e-60)


def test_identical_keys_closed_form_and_all_ties():
    # all keys equal -> every visible key gets 1/(P+w+1): harmonic closed form, exact fractions
    Hq, Hkv, d, L, W, budget, pool = 6, 2, 8, 40, 5, 17, 7
    G, P = Hq // Hkv, L - W
    g = torch.Generator().manual_seed(5)
    q = torch.randn(Hq, W, d, generator=g)
    k = torch.randn(1, 1, d, generator=g).expand(Hkv, L, d).contiguous()
    raw = oracle.raw_scores(q, k).numpy()
    for j in range(L):
        first_w = max(0, j - P)              # first query that sees column j
        want = G * sum(Fraction(1, P + w + 1) for w in range(first_w, W))
        np.testing.assert_allclose(raw[:, j], float(want), rtol=1e-13)
    pooled = oracle.maxpool(torch.from_numpy(raw), W, pool)
    idx = oracle.select(pooled.float(), W, budget).numpy()
    want_idx = list(range(budget - W)) + list(range(P, L))     # all ties -> lowest indices
    assert (idx == np.array(want_idx, dtype=np.int32)[None]).all()


def test_zero_queries_give_uniform_attention():
    Hq, Hkv, d, L, W = 4, 4, 8, 21, 2
    _, k, _ = rand_case(2, Hq, Hkv, d, L, W)
    raw = oracle.raw_scores(torch.zeros(Hq, W, d), k).numpy()
    P = L - W
    np.testing.assert_allclose(raw[:, :P], 1 / (P + 1) + 1 / (P + 2), rtol=1e-13)


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_reduces_to_argsort_of_qk_for_single_query(seed):
    # Eq. 4 read literally: with one query, one head per KV head and no pooling the softmax is
    # monotone, so the retained prefix set is ArgSort(q K^T)[:k_sel]
    Hq = Hkv = 3
    d, L, W, budget = 16, 200, 1, 31
    q, k, v = rand_case(seed, Hq, Hkv, d, L, W)
    pooled, idx, _, _ = oracle.evict(q, k, v, budget, pool=1)
    dots = torch.einsum("hc,hjc->hj", q[:, 0].double(), k.double())[:, :L - 1]
    for h in range(Hkv):
        top = torch.argsort(dots[h], descending=True)[:budget - 1]
        assert sorted(top.tolist()) == idx[h, :budget - 1].tolist()
        assert idx[h, -1].item() == L - 1


def test_gqa_group_is_sum_of_single_head_runs():
    Hq, Hkv, d, L, W = 6, 2, 8, 50, 3
    q, k, _ = rand_case(9, Hq, Hkv, d, L, W, qscale=2.0)
    G = Hq // Hkv
    whole = oracle.raw_scores(q, k).numpy()
    for g in range(Hkv):
        parts = sum(oracle.raw_scores(q[h:h + 1], k[g:g + 1]).numpy()[0]
                    for h in range(g * G, (g + 1) * G))
        np.testing.assert_allclose(whole[g], parts, rtol=1e-12)
    # and the head -> group map is by consecutive blocks: swapping two heads of different groups matters
    q2 = q.clone()
    q2[[0, G]] = q2[[G, 0]]
    assert not np.allclose(oracle.raw_scores(q2, k).numpy(), whole)


def test_window_sum_is_sum_of_single_query_runs_with_their_own_mask():
    # one head, W queries: equals the sum of W single-query runs on the truncated key prefix
    d, L, W = 8, 30, 4
    q, k, _ = rand_case(21, 1, 1, d, L, W, qscale=2.0)
    whole = oracle.raw_scores(q, k).numpy()[0]
    P = L - W
    acc = np.zeros(L)
    for w in range(W):
        vis = P + w + 1
        acc[:vis] += oracle.raw_scores(q[:, w:w + 1], k[:, :vis]).numpy()[0]
    np.testing.assert_allclose(whole, acc, rtol=1e-12)


def test_shift_of_all_keys_leaves_scores_unchanged():
    # adding one vector to every key shifts each row's logits by a constant
    q, k, _ = rand_case(4, 4, 2, 8, 64, 4)
    k = torch.round(k * 64) / 64                 # on a grid, so that k + u is exact in fp32
    u = torch.round(torch.randn(8, generator=torch.Generator().manual_seed(1)) * 64) / 64
    a = oracle.raw_scores(q, k).numpy()
    b = oracle.raw_scores(q, k + u).numpy()
    np.testing.assert_allclose(a, b, rtol=1e-9)


def test_prefix_permutation_permutes_prefix_scores():
    q, k, _ = rand_case(6, 4, 2, 8, 40, 4)
    P = 36
    perm = torch.randperm(P, generator=torch.Generator().manual_seed(2))
    k2 = k.clone()
    k2[:, :P] = k[:, perm]
    a = oracle.raw_scores(q, k).numpy()
    b = oracle.raw_scores(q, k2).numpy()
    np.testing.assert_allclose(b[:, :P], a[:, perm.numpy()], rtol=1e-11)
    np.testing.assert_allclose(b[:, P:], a[:, P:], rtol=1e-11)


def test_softmax_matches_library_on_unmasked_case():
    # W = 1: a single query after the whole prefix; compare with torch's fp64 softmax
    q, k, _ = rand_case(8, 2, 2, 16, 100, 1, qscale=3.0)
    raw = oracle.raw_scores(q, k)
    logits = torch.einsum("hc,hjc->hj", q[:, 0].double(), k.double()) / 4.0
    np.testing.assert_allclose(raw.numpy(), torch.softmax(logits, dim=1).numpy(), rtol=1e-12)


def test_extreme_logits_do_not_overflow():
    # the max is subtracted before exponentiation: logits of +-1000 still give a valid distribution
    q = torch.full((1, 2, 4), 50.0)
    k = torch.zeros(1, 12, 4)
    k[0, 3] = 20.0
    k[0, 5] = -20.0
    raw = oracle.raw_scores(q, k, scale=1.0).numpy()[0]
    assert np.isfinite(raw).all()
    np.testing.assert_allclose(raw.sum(), 2.0, rtol=1e-12)
    assert raw[3] == pytest.approx(2.0, rel=1e-12)


# ----------------------------------------------------------------------------
def _golden_pool_cases():
    cases = []
    with open(os.path.join(GOLDEN, "maxpool_cases.txt")) as fh:
        for line in fh:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            head, raw, want = [p.strip() for p in line.split("|")]
            W, pool = [int(x) for x in head.split()]
            cases.append((W, pool, [float(x) for x in raw.split()], [float(x) for x in want.split()]))
    return cases


@pytest.mark.parametrize("W,pool,raw,want", _golden_pool_cases())
def test_maxpool_hand_computed(W, pool, raw, want):
    got = oracle.maxpool(torch.tensor([raw], dtype=torch.float64), W, pool).numpy()[0]
    assert got.tolist() == want


@pytest.mark.parametrize("pool", [1, 3, 5, 7, 9])
def test_maxpool_vs_brute_and_library(pool):
    g = torch.Generator().manual_seed(pool)
    raw = torch.rand(3, 57, generator=g, dtype=torch.float64)
    W = 6
    got = oracle.maxpool(raw, W, pool).numpy()
    assert (got == brute_pool(raw.numpy(), W, pool)).all()
    P = 57 - W
    lib = torch.nn.functional.max_pool1d(raw[:, :P].unsqueeze(0), pool, stride=1, padding=pool // 2)[0]
    assert (got[:, :P] == lib.numpy()).all()
    assert (got[:, P:] == raw[:, P:].numpy()).all()
    assert (got[:, :P] >= raw[:, :P].numpy()).all()
    if pool == 1:
        assert (got == raw.numpy()).all()


def test_maxpool_isolated_spike_gives_plateau():
    raw = torch.zeros(1, 40, dtype=torch.float64)
    raw[0, 20] = 1.0
    got = oracle.maxpool(raw, 4, 7).numpy()[0]
    assert got[17:24].tolist() == [1.0] * 7 and got[16] == 0 and got[24] == 0


def test_maxpool_rejects_even_kernel():
    with pytest.raises(ValueError):
        oracle.maxpool(torch.zeros(1, 8, dtype=torch.float64), 1, 4)


# ----------------------------------------------------------------------------
@pytest.mark.parametrize("seed", range(4))
def test_select_vs_exhaustive_sort_with_ties(seed):
    g = torch.Generator().manual_seed(seed)
    Hkv, L, W = 3, 61, 5
    # few distinct values -> many exact ties, including across the k-th boundary
    scores = torch.randint(0, 6, (Hkv, L), generator=g).float() / 4
    for budget in (W, W + 1, 20, L - 1, L, L + 10):
        got = oracle.select(scores, W, budget).numpy()
        assert (got == brute_select(scores.numpy(), W, budget)).all()
        Bk = min(budget, L)
        assert got.shape == (Hkv, Bk)
        assert (np.diff(got, axis=1) > 0).all() if Bk > 1 else True
        assert (got[:, Bk - W:] == np.arange(L - W, L)).all()


def test_select_properties_random():
    g = torch.Generator().manual_seed(3)
    Hkv, L, W, budget = 4, 500, 8, 64
    scores = torch.rand(Hkv, L, generator=g)
    idx = oracle.select(scores, W, budget).numpy()
    P = L - W
    for h in range(Hkv):
        sel = idx[h, :budget - W]
        rest = np.setdiff1d(np.arange(P), sel)
        assert scores[h, sel].min() >= scores[h, rest].max()
        lib = torch.topk(scores[h, :P], budget - W).indices.sort().values
        assert sel.tolist() == lib.tolist()                      # tie-free -> library top-k agrees


def test_select_plateau_takes_lowest_indices():
    s = torch.zeros(1, 30)
    s[0, 10:17] = 2.0           # a 7-wide plateau, as max-pooling produces
    s[0, 20:27] = 2.0
    idx = oracle.select(s, 2, 2 + 10).numpy()[0]
    assert idx.tolist() == [10, 11, 12, 13, 14, 15, 16, 20, 21, 22, 28, 29]


def test_select_budget_below_window_is_rejected():
    with pytest.raises(ValueError):
        oracle.select(torch.zeros(1, 10), 4, 3)


def test_compact_is_plain_indexing():
    q, k, v = rand_case(1, 2, 2, 8, 33, 3, torch.bfloat16)
    idx = torch.tensor([[0, 5, 7, 30, 31, 32], [1, 2, 3, 30, 31, 32]], dtype=torch.int32)
    for src in (k, v, k.float()):
        got = oracle.compact(src, idx)
        want = torch.stack([src[h, idx[h].long()] for h in range(2)])
        assert torch.equal(got.view(torch.uint8), want.view(torch.uint8))


# ----------------------------------------------------------------------------
def test_config1_planted_keys_give_closed_form_set():
    # 8 planted keys x pool 7 = 56 = budget - W: with planted positions >= 8 apart and >= 4 from
    # the prefix edges and a dominant amplitude, the retained prefix set is the union of the
    # planted keys' pooling neighbourhoods
    import dataclasses
    cfg = dataclasses.replace(CONFIGS[1], planted_amp=40.0)
    q, k, v, meta = make_instance(cfg)
    budget = budgets_for(cfg)[0]
    pooled, idx, kc, vc = oracle.evict(q, k, v, budget, cfg.pool)
    for g in range(cfg.Hkv):
        want = sorted(j for p in meta["planted"][g].tolist() for j in range(p - 3, p + 4))
        assert len(want) == budget - cfg.W
        assert idx[g, :budget - cfg.W].tolist() == want
        assert idx[g, budget - cfg.W:].tolist() == list(range(cfg.P, cfg.L))
    assert torch.equal(kc, torch.stack([k[g, idx[g].long()] for g in range(cfg.Hkv)]))
    assert torch.equal(vc, torch.stack([v[g, idx[g].long()] for g in range(cfg.Hkv)]))


def test_config1_as_specified_selects_strong_planted_keys():
    cfg = CONFIGS[1]
    q, k, v, meta = make_instance(cfg)
    pooled, idx, _, _ = oracle.evict(q, k, v, 64, 7)
    raw = oracle.raw_scores(q, k)
    for g in range(cfg.Hkv):
        sel = set(idx[g].tolist())
        # every selected prefix index lies in the pooling neighbourhood of a raw-score peak that
        # ranks among the selected, and the strongest planted key is retained
        pl = meta["planted"][g]
        best = pl[raw[g, pl].argmax()].item()
        assert best in sel
        assert len(sel) == 64 and all(j in sel for j in range(cfg.P, cfg.L))


def test_invariants_on_bf16_config_shape():
    import dataclasses
    cfg = dataclasses.replace(CONFIGS[2], L=700, Hq=8, Hkv=2)
    q, k, v, meta = make_instance(cfg)
    pooled, idx, kc, vc = oracle.evict(q, k, v, 128, 7)
    raw = oracle.raw_scores(q, k)
    np.testing.assert_allclose(raw.sum(dim=1).numpy(), cfg.G * cfg.W, rtol=1e-12)
    assert idx.shape == (2, 128)
    assert (idx[:, 1:] > idx[:, :-1]).all()
    assert (idx[:, -cfg.W:] == torch.arange(cfg.P, cfg.L, dtype=torch.int32)).all()
    assert (pooled[:, :cfg.P] >= raw[:, :cfg.P]).all()


def test_pyramid_budget_schedule_endpoints_and_monotone():
    b = [pyramid_budget(l, 32, 2048, 128) for l in range(32)]
    assert b[0] == 2048 and b[-1] == 128
    assert all(x > y for x, y in zip(b, b[1:]))
    assert budgets_for(CONFIGS[4]) == b
    assert budgets_for(CONFIGS[5]) == [256] * 256


# ----------------------------------------------------------------------------
# general observation window (Sec. 4.3, Eq. 5): explicit query positions and an
# independent count of retained trailing keys
# ----------------------------------------------------------------------------
def brute_raw_pos(q, k, q_pos, scale=None):
    """Explicit attention with per-query last visible key, in pure Python loops."""
    q = q.double().tolist()
    k = k.double().tolist()
    Hq, W, d = len(q), len(q[0]), len(q[0][0])
    Hkv, L = len(k), len(k[0])
    G = Hq // Hkv
    scale = 1.0 / math.sqrt(d) if scale is None else scale
    raw = [[0.0] * L for _ in range(Hkv)]
    for h in range(Hq):
        g = h // G
        for w in range(W):
            last = min(q_pos[w], L - 1)
            s = [scale * sum(a * b for a, b in zip(q[h][w], k[g][j])) for j in range(last + 1)]
            m = max(s)
            e = [math.exp(x - m) for x in s]
            z = sum(e)
            for j in range(last + 1):
                raw[g][j] += e[j] / z
    return np.array(raw)


def test_explicit_positions_equal_to_the_default_give_the_same_bits():
    g = torch.Generator().manual_seed(21)
    q, k = torch.randn(4, 5, 16, generator=g), torch.randn(2, 40, 16, generator=g)
    a = oracle.raw_scores(q, k)
    b = oracle.raw_scores(q, k, q_pos=[35 + w for w in range(5)])
    assert torch.equal(a, b)


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_random_positions_match_python_loops(seed):
    g = torch.Generator().manual_seed(100 + seed)
    Hq, Hkv, d, L, W = 4, 2, 8, 23, 6
    q, k = torch.randn(Hq, W, d, generator=g), torch.randn(Hkv, L, d, generator=g)
    pos = torch.randint(0, L + 5, (W,), generator=g).tolist()       # some beyond L-1, maybe 0
    pos[0] = 0                                                        # a query that sees one key only
    got = oracle.raw_scores(q, k, q_pos=pos).numpy()
    np.testing.assert_allclose(got, brute_raw_pos(q, k, pos), rtol=1e-12, atol=1e-15)
    # a query that sees one key puts its whole mass there; nothing lands beyond the furthest position
    assert got[:, 0].min() >= Hq // Hkv - 1e-12
    far = min(max(pos), L - 1)
    assert (got[:, far + 1:] == 0).all()


def test_lookahead_queries_see_every_key_library_softmax():
    # queries generated after the prompt (pure LAQ): no mask at all -> plain softmax, any position >= L-1
    g = torch.Generator().manual_seed(5)
    Hq, Hkv, d, L, W = 6, 3, 32, 77, 4
    q, k = torch.randn(Hq, W, d, generator=g), torch.randn(Hkv, L, d, generator=g)
    for pos in ([L - 1] * W, [L + 3, L, 10 * L, L - 1]):
        got = oracle.raw_scores(q, k, q_pos=pos)
        kk = k.double().repeat_interleave(Hq // Hkv, dim=0)
        att = torch.softmax(torch.einsum("hwc,hjc->hwj", q.double(), kk) / math.sqrt(d), dim=2)
        want = att.reshape(Hkv, Hq // Hkv, W, L).sum(dim=(1, 2))
        torch.testing.assert_close(got, want, rtol=1e-12, atol=1e-15)
        torch.testing.assert_close(got.sum(dim=1), torch.full((Hkv,), float(Hq // Hkv * W), dtype=torch.float64))


def test_joined_window_is_the_sum_of_its_parts():
    # Eq. 5: local window queries joined with lookahead queries; every row is its own softmax, so
    # the score of the union is the sum of the two runs
    g = torch.Generator().manual_seed(6)
    Hq, Hkv, d, L = 4, 2, 16, 50
    q_loc, q_la = torch.randn(Hq, 3, d, generator=g), torch.randn(Hq, 5, d, generator=g)
    k = torch.randn(Hkv, L, d, generator=g)
    pos_loc, pos_la = [L - 3, L - 2, L - 1], [L + i for i in range(5)]
    both = oracle.raw_scores(torch.cat([q_loc, q_la], dim=1), k, q_pos=pos_loc + pos_la)
    parts = oracle.raw_scores(q_loc, k, q_pos=pos_loc) + oracle.raw_scores(q_la, k, q_pos=pos_la)
    torch.testing.assert_close(both, parts, rtol=1e-13, atol=1e-15)
    # the local part alone is the default layout
    assert torch.equal(oracle.raw_scores(q_loc, k, q_pos=pos_loc), oracle.raw_scores(q_loc, k))


def test_query_order_does_not_matter_when_positions_travel_with_the_queries():
    g = torch.Generator().manual_seed(8)
    q, k = torch.randn(2, 6, 8, generator=g), torch.randn(2, 30, 8, generator=g)
    pos = [3, 29, 11, 40, 0, 17]
    perm = [4, 2, 0, 5, 1, 3]
    a = oracle.raw_scores(q, k, q_pos=pos)
    b = oracle.raw_scores(q[:, perm], k, q_pos=[pos[i] for i in perm])
    torch.testing.assert_close(a, b, rtol=1e-13, atol=1e-15)


def test_negative_position_and_wrong_length_are_rejected():
    q, k = torch.randn(2, 3, 8), torch.randn(1, 10, 8)
    with pytest.raises(ValueError):
        oracle.raw_scores(q, k, q_pos=[1, -1, 2])
    with pytest.raises(ValueError):
        oracle.raw_scores(q, k, q_pos=[1, 2])
    with pytest.raises(ValueError):
        oracle.raw_scores(torch.randn(2, 12, 8), k)          # default layout needs W <= L
    oracle.raw_scores(torch.randn(2, 12, 8), k, q_pos=[9] * 12)   # explicit positions do not


@pytest.mark.parametrize("keep", [0, 1, 4, 12])
def test_keep_count_in_pool_and_select_vs_brute(keep):
    g = torch.Generator().manual_seed(30 + keep)
    raw = torch.rand(2, 12, generator=g, dtype=torch.float64)
    raw[0, 5] = raw[0, 2]                                         # a tie
    pooled = oracle.maxpool(raw, keep, 3)
    np.testing.assert_array_equal(pooled.numpy(), brute_pool(raw.numpy(), keep, 3))
    for budget in (keep, keep + 1, 7, 12, 20):
        if budget < max(keep, 1):
            continue
        got = oracle.select(pooled.float(), keep, budget)
        want = brute_select(pooled.float().numpy(), keep, budget)
        np.testing.assert_array_equal(got.numpy(), want)
        assert got.shape[1] == min(budget, 12)
        if keep:
            assert got[:, -keep:].tolist() == [list(range(12 - keep, 12))] * 2


def test_keep_zero_is_plain_topk_library():
    g = torch.Generator().manual_seed(31)
    s = torch.randn(3, 200, generator=g)                          # distinct values: order is unique
    got = oracle.select(s, 0, 17)
    want = torch.sort(torch.topk(s, 17, dim=1).indices, dim=1).values.int()
    assert torch.equal(got, want)


def test_select_rejects_budget_below_keep_and_keep_above_length():
    s = torch.rand(1, 10)
    with pytest.raises(ValueError):
        oracle.select(s, 4, 3)
    with pytest.raises(ValueError):
        oracle.select(s, 11, 11)
    with pytest.raises(ValueError):
        oracle.maxpool(s.double(), -1, 3)


# ----------------------------------------------------------------------------
# Stage-1 eviction variants (Sec. 4.2; Sec. 5.1 for the average pool): pins
@pytest.mark.parametrize("pool", [1, 3, 5, 7, 9])
def test_avgpool_vs_library_routine_and_exact_fractions(pool):
    g = torch.Generator().manual_seed(100 + pool)
    raw = torch.randint(0, 50, (3, 41), generator=g).double()      # small integers: sums are exact
    got = oracle.avgpool(raw, 0, pool)
    lib = torch.nn.functional.avg_pool1d(raw.unsqueeze(0), pool, stride=1, padding=pool // 2,
                                         count_include_pad=True)[0]
    np.testing.assert_allclose(got.numpy(), lib.numpy(), rtol=1e-15, atol=0)
    half = pool // 2
    for j in (0, 1, 20, 39, 40):                                    # exact rational arithmetic
        lo, hi = max(0, j - half), min(40, j + half)
        want = Fraction(int(raw[1, lo:hi + 1].sum().item()), pool)
        assert Fraction(got[1, j].item()) == Fraction(float(want))
    if pool == 1:
        assert torch.equal(got, raw)


def test_avgpool_hand_cases_and_prefix_domain():
    raw = torch.tensor([[3.0, 0.0, 6.0, 9.0, 0.0, 3.0, 1000.0, 2000.0]], dtype=torch.float64)
    got = oracle.avgpool(raw, 2, 3).numpy()[0]                      # prefix = first 6, last 2 copied
    # zeros stand in beyond both ends of the prefix; the kept columns never leak into it
    assert got.tolist() == [1.0, 3.0, 5.0, 5.0, 4.0, 1.0, 1000.0, 2000.0]
    const = torch.full((1, 20), 7.0, dtype=torch.float64)
    got = oracle.avgpool(const, 0, 7).numpy()[0]
    np.testing.assert_allclose(got[3:17], 7.0, rtol=1e-15)
    np.testing.assert_allclose(got[:3], [7.0 * c / 7 for c in (4, 5, 6)], rtol=1e-15)
    np.testing.assert_allclose(got[17:], [7.0 * c / 7 for c in (6, 5, 4)], rtol=1e-15)


def test_avgpool_column_sum_identity_and_linearity():
    g = torch.Generator().manual_seed(77)
    a = torch.rand(2, 64, generator=g, dtype=torch.float64)
    b = torch.rand(2, 64, generator=g, dtype=torch.float64)
    keep, pool, half = 5, 7, 3
    P = 64 - keep
    pa = oracle.avgpool(a, keep, pool)
    # entry i of the prefix lies in min(i, half) + min(P-1-i, half) + 1 windows
    cover = torch.tensor([min(i, half) + min(P - 1 - i, half) + 1 for i in range(P)], dtype=torch.float64)
    np.testing.assert_allclose(pa[:, :P].sum(1).numpy(), ((a[:, :P] * cover).sum(1) / pool).numpy(), rtol=1e-13)
    pab = oracle.avgpool(2.0 * a + b, keep, pool)
    np.testing.assert_allclose(pab.numpy(), (2.0 * pa + oracle.avgpool(b, keep, pool)).numpy(), rtol=1e-13)
    # an isolated spike spreads into a plateau of height 1/pool
    s = torch.zeros(1, 40, dtype=torch.float64)
    s[0, 20] = 1.0
    sp = oracle.avgpool(s, 4, 7).numpy()[0]
    assert sp[17:24].tolist() == [1.0 / 7] * 7 and sp[16] == 0 and sp[24] == 0
    with pytest.raises(ValueError):
        oracle.avgpool(s, 4, 4)


def test_avgpool_differs_from_maxpool_in_selection_on_a_planted_case():
    # one tall spike next to a broad shoulder: the max pool keeps the spike's neighbourhood,
    # the average keeps the shoulder's centre
    raw = torch.zeros(1, 30, dtype=torch.float64)
    raw[0, 5] = 1.0
    raw[0, 18:23] = 0.5
    top_max = oracle.select(oracle.maxpool(raw, 0, 5).float(), 0, 1)
    top_avg = oracle.select(oracle.avgpool(raw, 0, 5).float(), 0, 1)
    assert top_max.tolist() == [[3]]          # plateau 3..7 of height 1, lowest index wins
    assert top_avg.tolist() == [[20]]         # 5 * 0.5 / 5 = 0.5 > 1 / 5


@pytest.mark.parametrize("L,n_sink,budget", [(10, 2, 5), (10, 0, 4), (10, 4, 4), (10, 6, 4), (10, 3, 10),
                                             (10, 3, 25), (1, 4, 1), (257, 4, 64), (10, 2, 1)])
def test_sink_recent_vs_set_construction(L, n_sink, budget):
    got = oracle.sink_recent(3, L, n_sink, budget)
    Bk = min(budget, L)
    s = min(n_sink, Bk)
    want = sorted(set(range(s)) | set(range(L - (Bk - s), L)))
    assert got.shape == (3, Bk)
    assert got.tolist() == [want] * 3
    assert len(set(want)) == Bk


def test_sink_recent_hand_case_and_rejection():
    assert oracle.sink_recent(1, 10, 2, 5).tolist() == [[0, 1, 7, 8, 9]]
    assert oracle.sink_recent(2, 6, 4, 100).tolist() == [list(range(6))] * 2
    with pytest.raises(ValueError):
        oracle.sink_recent(1, 10, -1, 5)
    with pytest.raises(ValueError):
        oracle.sink_recent(1, 10, 2, 0)


def test_evict_with_average_pool_is_pool_then_select():
    cfg = CONFIGS[1]
    q, k, v, _ = make_instance(cfg, 0, 0)
    pooled, idx, k2, v2 = oracle.evict(q, k, v, 64, 7, pool_mode="avg")
    raw = oracle.raw_scores(q, k)
    assert torch.equal(pooled, oracle.avgpool(raw, cfg.W, 7))
    assert torch.equal(idx, oracle.select(pooled.float(), cfg.W, 64))
    # total prefix mass shrinks only through the zero padding at the two ends
    P = cfg.L - cfg.W
    assert (pooled[:, :P].sum(1) <= raw[:, :P].sum(1) * (1 + 1e-12)).all()
    np.testing.assert_allclose(pooled[:, 3:P - 3].numpy(),
                               torch.nn.functional.avg_pool1d(raw[:, :P].unsqueeze(0), 7, stride=1)[0].numpy(),
                               rtol=1e-13)


# ----------------------------------------------------------------------------
# Recall of a selection (Sec. 3, Eq. 1-3): pins of the overlap count
@pytest.mark.parametrize("seed", range(4))
def test_overlap_vs_python_sets_and_symmetry(seed):
    rng = np.random.default_rng(seed)
    Hkv, L, n_pred, n_gold = 3, 97, 20 + seed, 31
    pred = np.stack([rng.permutation(L)[:n_pred] for _ in range(Hkv)]).astype(np.int32)
    gold = np.stack([rng.permutation(L)[:n_gold] for _ in range(Hkv)]).astype(np.int32)
    got = oracle.overlap(torch.from_numpy(pred), torch.from_numpy(gold), L)
    want = [len(set(pred[g].tolist()) & set(gold[g].tolist())) for g in range(Hkv)]
    assert got.tolist() == want
    assert oracle.overlap(torch.from_numpy(gold), torch.from_numpy(pred), L).tolist() == want


def test_overlap_extremes_and_hand_case():
    a = torch.tensor([[0, 2, 4, 6, 8]], dtype=torch.int32)
    assert oracle.overlap(a, a, 10).tolist() == [5]                                   # recall 1
    assert oracle.overlap(a, torch.tensor([[1, 3, 5, 7, 9]], dtype=torch.int32), 10).tolist() == [0]
    assert oracle.overlap(a, torch.tensor([[8, 7, 2]], dtype=torch.int32), 10).tolist() == [2]
    assert oracle.overlap(a, torch.arange(10, dtype=torch.int32)[None], 10).tolist() == [5]
    with pytest.raises(ValueError):
        oracle.overlap(a, torch.tensor([[10]], dtype=torch.int32), 10)               # position out of range


def test_recall_of_a_window_against_all_queries_behaves_as_eq3_says():
    # M_gold from many queries, M_pred from a subset of them: recall is 1 when the subset is the
    # whole set and, on this planted instance, stays high for the subset because both see the
    # planted keys
    cfg = CONFIGS[1]
    q, k, _, _ = make_instance(cfg, 0, 0)
    L = cfg.L
    see_all = [L] * cfg.W
    gold = oracle.select(oracle.maxpool(oracle.raw_scores(q, k, q_pos=see_all), 0, 7).float(), 0, 64)
    pred_all = oracle.select(oracle.maxpool(oracle.raw_scores(q, k, q_pos=see_all), 0, 7).float(), 0, 64)
    assert oracle.overlap(pred_all, gold, L).tolist() == [64] * cfg.Hkv
    pred_half = oracle.select(oracle.maxpool(oracle.raw_scores(q[:, :4], k, q_pos=see_all[:4]), 0, 7).float(), 0, 64)
    ov = oracle.overlap(pred_half, gold, L)
    assert (ov >= 32).all() and (ov <= 64).all()


# ----------------------------------------------------------------------------
# Decoding on the compacted cache (Sec. 4.3) and Q-cache capture (Sec. 4.2): pins
@pytest.mark.parametrize("Hq,Hkv,d,Bk,dtype", [(4, 2, 16, 9, torch.float32), (8, 2, 64, 130, torch.bfloat16),
                                               (3, 3, 8, 1, torch.float32), (6, 1, 32, 40, torch.bfloat16)])
def test_decode_attention_vs_library_softmax_matmul(Hq, Hkv, d, Bk, dtype):
    g = torch.Generator().manual_seed(Hq * 100 + Bk)
    q = torch.randn(Hq, d, generator=g).to(dtype)
    kc = torch.randn(Hkv, Bk, d, generator=g).to(dtype)
    vc = torch.randn(Hkv, Bk, d, generator=g).to(dtype)
    got = oracle.decode_attention(q, kc, vc)
    G = Hq // Hkv
    kk = kc.double().repeat_interleave(G, dim=0)                 # [Hq, Bk, d]: head h -> KV head h // G
    vv = vc.double().repeat_interleave(G, dim=0)
    p = torch.softmax(torch.einsum("hd,hjd->hj", q.double(), kk) / math.sqrt(d), dim=1)
    want = torch.einsum("hj,hjd->hd", p, vv)
    np.testing.assert_allclose(got.numpy(), want.numpy(), rtol=1e-11, atol=1e-13)
    lib = torch.nn.functional.scaled_dot_product_attention(q.double()[:, None, :], kk, vv)[:, 0]
    np.testing.assert_allclose(got.numpy(), lib.numpy(), rtol=1e-10, atol=1e-12)


def test_decode_attention_closed_forms():
    g = torch.Generator().manual_seed(3)
    q = torch.randn(4, 16, generator=g)
    vc = torch.randn(2, 7, 16, generator=g)
    same = torch.randn(2, 1, 16, generator=g).expand(2, 7, 16).contiguous()
    got = oracle.decode_attention(q, same, vc)                   # identical keys: the mean of V
    np.testing.assert_allclose(got[:2].numpy(), vc[0].double().mean(0).expand(2, 16).numpy(), rtol=1e-12)
    np.testing.assert_allclose(got[2:].numpy(), vc[1].double().mean(0).expand(2, 16).numpy(), rtol=1e-12)
    kc = torch.zeros(2, 7, 16)
    kc[0, 3] = q[0] * 50.0                                       # one dominant key for head 0
    got = oracle.decode_attention(q, kc, vc, scale=1.0)
    np.testing.assert_allclose(got[0].numpy(), vc[0, 3].double().numpy(), rtol=1e-9, atol=1e-12)
    # explicit scale is used: zero keys give uniform weights whatever the scale
    got0 = oracle.decode_attention(q, torch.zeros(2, 7, 16), vc, scale=3.0)
    np.testing.assert_allclose(got0[3].numpy(), vc[1].double().mean(0).numpy(), rtol=1e-12)
    # permuting the retained rows (keys and values together) changes nothing
    perm = torch.randperm(7, generator=g)
    kr = torch.randn(2, 7, 16, generator=g)
    a = oracle.decode_attention(q, kr, vc)
    b = oracle.decode_attention(q, kr[:, perm].contiguous(), vc[:, perm].contiguous())
    np.testing.assert_allclose(a.numpy(), b.numpy(), rtol=1e-12, atol=1e-14)
    # extreme logits stay finite
    big = oracle.decode_attention(q * 1e3, kr * 1e3, vc, scale=1.0)
    assert np.isfinite(big.numpy()).all()


def test_qcache_store_is_tensor_indexing():
    g = torch.Generator().manual_seed(9)
    cache = torch.randn(6, 8, 32, generator=g).bfloat16()
    step = torch.randn(6, 32, generator=g).bfloat16()
    for t in (0, 3, 7):
        want = cache.clone()
        want[:, t] = step
        assert torch.equal(oracle.qcache_store(cache, step, t), want)
    with pytest.raises(ValueError):
        oracle.qcache_store(cache, step, 8)


def test_eight_lookahead_steps_fill_the_qcache_that_scoring_reads():
    # the Q-cache built step by step is the q_win tensor the re-eviction takes
    g = torch.Generator().manual_seed(10)
    steps = [torch.randn(4, 16, generator=g) for _ in range(8)]
    cache = torch.zeros(4, 8, 16)
    for t, s in enumerate(steps):
        cache = oracle.qcache_store(cache, s, t)
    assert torch.equal(cache, torch.stack(steps, dim=1))


def test_sink_recent_writes_exactly_its_rows():
    # more sinks than the budget holds: the list is the first Bk positions and nothing is written
    # beyond the Hkv * Bk entries (checked through the C entry point with a guarded buffer)
    lib = oracle._load()
    Hkv, L, n_sink, budget = 3, 10, 6, 4
    buf = torch.full((Hkv * budget + 8,), -7, dtype=torch.int32)
    assert lib.laq_oracle_sink_recent(Hkv, L, n_sink, budget, buf.data_ptr()) == 0
    assert buf[:Hkv * budget].view(Hkv, budget).tolist() == [[0, 1, 2, 3]] * Hkv
    assert buf[Hkv * budget:].tolist() == [-7] * 8


# ----------------------------------------------------------------------------
# paged caches: the gather that precedes the dense functions
# ----------------------------------------------------------------------------
def _scatter_into_pool(dense, block_rows, n_blocks, gen):
    """Writes a dense cache [n, Hkv, L, d] into a pool through a random block table, with numpy
    fancy indexing on flattened rows (independent of the oracle's loops); unused pool rows hold NaN."""
    n, Hkv, L, d = dense.shape
    per = -(-L // block_rows)
    table = torch.randperm(n_blocks, generator=gen)[: n * per].reshape(n, per).int()
    pool = torch.full((n_blocks, Hkv, block_rows, d), float("nan"), dtype=dense.dtype)
    j = np.arange(L)
    for i in range(n):
        blk = table[i].numpy()[j // block_rows]                  # block of every row
        pool.numpy()[blk, :, j % block_rows] = dense[i].permute(1, 0, 2).numpy()
    return pool, table


@pytest.mark.parametrize("L,block_rows", [(512, 256), (700, 256), (1000, 512), (256, 256), (5, 256)])
def test_gather_paged_inverts_an_independent_scatter(L, block_rows):
    gen = torch.Generator().manual_seed(L)
    dense = torch.randn(3, 2, L, 8, generator=gen)
    pool, table = _scatter_into_pool(dense, block_rows, 3 * (-(-L // block_rows)) + 4, gen)
    back = oracle.gather_paged(pool, table, L)
    assert torch.equal(back, dense)                              # no NaN leaked in: only valid rows were read


def test_gather_paged_shared_blocks_identity_table_and_rejections():
    gen = torch.Generator().manual_seed(1)
    pool = torch.randn(4, 2, 256, 8, generator=gen)
    # the identity table of one instance is a reshape
    one = oracle.gather_paged(pool, torch.arange(4).reshape(1, 4).int(), 1024)
    assert torch.equal(one[0], pool.permute(1, 0, 2, 3).reshape(2, 1024, 8))
    # two instances that share their first block (a common prompt prefix) and differ afterwards
    two = oracle.gather_paged(pool, torch.tensor([[0, 1], [0, 2]]).int(), 300)
    assert torch.equal(two[0, :, :256], two[1, :, :256]) and torch.equal(two[0, :, 256:], pool[1, :, :44])
    assert torch.equal(two[1, :, 256:], pool[2, :, :44])
    with pytest.raises(ValueError):
        oracle.gather_paged(pool, torch.tensor([[0, 4]]).int(), 300)      # no such block
    with pytest.raises(ValueError):
        oracle.gather_paged(pool, torch.tensor([[0, 1, 2]]).int(), 300)   # table longer than L needs


def test_evict_on_a_gathered_paged_cache_equals_evict_on_the_dense_cache():
    cfg = CONFIGS[1]
    q, k, v, _ = make_instance(cfg, 0, 0)
    gen = torch.Generator().manual_seed(9)
    kp, table = _scatter_into_pool(k.unsqueeze(0), 256, 7, gen)
    vp = torch.full_like(kp, float("nan"))
    j = np.arange(cfg.L)
    vp.numpy()[table[0].numpy()[j // 256], :, j % 256] = v.permute(1, 0, 2).numpy()
    a = oracle.evict(q, k, v, 64, cfg.pool)
    b = oracle.evict(q, oracle.gather_paged(kp, table, cfg.L)[0], oracle.gather_paged(vp, table, cfg.L)[0], 64, cfg.pool)
    for x, y in zip(a, b):
        assert torch.equal(x, y)
