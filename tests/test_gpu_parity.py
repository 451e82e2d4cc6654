"""HIP path vs CPU oracle, element by element, through the C ABI (needs an MI355X)."""
import dataclasses

import numpy as np
import pytest
import torch

import oracle
from laq_inputs import CONFIGS, budgets_for, make_batch, make_instance
from parity_util import RTOL, check_index_row, check_scores, split_packed

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


@pytest.fixture(scope="module")
def laq():
    import paper_2505_20334_amd as m
    m.load_library()
    assert torch.cuda.is_available()
    return m


def run_and_check(laq, q, k, v, budgets, pool, what, heads=None, scale=0.0, exact_expected=None):
    """q [n,Hq,W,d], k/v [n,Hkv,L,d] on the GPU.  Runs laq_evict and the three calls, compares with
    the oracle instance by instance (optionally only some KV heads)."""
    n, Hq, W, d = q.shape
    _, Hkv, L, _ = k.shape
    G = Hq // Hkv
    print("case:", what, "n=%d Hq=%d Hkv=%d d=%d L=%d W=%d pool=%d" % (n, Hq, Hkv, d, L, W, pool), flush=True)
    scores, idx, ko, vo = laq.laq_evict(q, k, v, budgets, pool, scale=scale)
    torch.cuda.synchronize()
    # the three-call sequence gives the same bits
    s3 = laq.laq_score(q, k, pool, scale=scale)
    i3 = laq.laq_select(s3, budgets, 1, W)
    k3, v3 = laq.laq_compact(k, v, i3, budgets, W)
    torch.cuda.synchronize()
    assert torch.equal(s3, scores) and torch.equal(i3, idx) and torch.equal(k3, ko)
    if v is not None:
        assert torch.equal(v3, vo)
    # ... and so does pooling inside laq_select instead of inside laq_score
    s_raw = laq.laq_score(q, k, 1, scale=scale)
    i_alt = laq.laq_select(s_raw, budgets, pool, W)
    torch.cuda.synchronize()
    assert torch.equal(i_alt, idx)
    alt_l = split_packed(i_alt.cpu(), budgets, Hkv, L)

    idx_l = split_packed(idx.cpu(), budgets, Hkv, L)
    ko_l = split_packed(ko.cpu(), budgets, Hkv, L)
    vo_l = split_packed(vo.cpu(), budgets, Hkv, L) if v is not None else None
    qc, kc = q.cpu(), k.cpu()
    vc = v.cpu() if v is not None else None
    sc = scores.cpu()
    heads = list(range(Hkv)) if heads is None else heads
    n_exact = 0
    for i in range(n):
        # compaction: bit-exact given the library's own indices
        for g in range(Hkv):
            rows = idx_l[i][g].long()
            assert torch.equal(ko_l[i][g].view(torch.int16 if k.dtype == torch.bfloat16 else torch.int32),
                               kc[i, g, rows].view(torch.int16 if k.dtype == torch.bfloat16 else torch.int32))
            if v is not None:
                assert torch.equal(vo_l[i][g], vc[i, g, rows])
        for g in heads:
            raw = oracle.raw_scores(qc[i, g * G:(g + 1) * G], kc[i, g:g + 1], scale)
            pooled = oracle.maxpool(raw, W, pool)
            check_scores(sc[i, g], pooled[0], k.dtype, "%s inst %d head %d" % (what, i, g))
            check_scores(s_raw[i, g].cpu(), raw[0], k.dtype, "%s raw inst %d head %d" % (what, i, g))
            ex = check_index_row(idx_l[i][g].numpy(), pooled[0].float().numpy(), W, budgets[i],
                                 RTOL[k.dtype], "%s inst %d head %d" % (what, i, g))
            n_exact += int(ex)
            # selection on identical fp32 scores is bit-exact
            o_idx = oracle.select(sc[i, g:g + 1], W, budgets[i])
            assert torch.equal(o_idx[0], idx_l[i][g]), "%s: select differs on identical scores" % what
            # ... also when the pooling is done inside laq_select
            p_alt = oracle.maxpool(s_raw[i, g:g + 1].cpu().double(), W, pool).float()
            assert torch.equal(oracle.select(p_alt, W, budgets[i])[0], alt_l[i][g]), "%s: select+pool" % what
            check_index_row(alt_l[i][g].numpy(), pooled[0].float().numpy(), W, budgets[i],
                            RTOL[k.dtype], "%s alt inst %d head %d" % (what, i, g))
    if exact_expected is not None:
        assert n_exact >= exact_expected
    return scores, idx, ko, vo


def test_config1_tiny_fp32(laq):
    cfg = CONFIGS[1]
    q, k, v, budgets, metas = make_batch(cfg, device=DEV)
    run_and_check(laq, q, k, v, budgets, cfg.pool, "cfg1")


def test_config1_planted_exact_set(laq):
    cfg = dataclasses.replace(CONFIGS[1], planted_amp=40.0)
    q, k, v, budgets, metas = make_batch(cfg, device=DEV)
    scores, idx, _, _ = run_and_check(laq, q, k, v, budgets, cfg.pool, "cfg1-planted")
    got = idx.cpu().reshape(cfg.Hkv, 64)
    for g in range(cfg.Hkv):
        want = sorted(j for p in metas[0]["planted"][g].tolist() for j in range(p - 3, p + 4))
        assert got[g, :56].tolist() == want


def test_config2_llama_4k(laq):
    cfg = CONFIGS[2]
    q, k, v, budgets, _ = make_batch(cfg, device=DEV)
    run_and_check(laq, q, k, v, budgets, cfg.pool, "cfg2")


def test_config3_two_layers_full_length(laq):
    cfg = CONFIGS[3]
    q, k, v, budgets, _ = make_batch(cfg, device=DEV, instances=[0, 31])
    run_and_check(laq, q, k, v, budgets, cfg.pool, "cfg3", heads=[0, 5])


@pytest.mark.parametrize("choose", ["auto", "single-read"])
def test_config4_sampled_full_size(laq, choose):
    # full 32-layer launch shape; the oracle checks sampled (instance, head) pairs.  By itself the
    # library streams K twice here (128 score rows); on request the single-read kernel takes it with
    # teams of 128 workgroups
    cfg = CONFIGS[4]
    q, k, v, budgets, _ = make_batch(cfg, device=DEV)
    n, Hkv, L, W, G = cfg.n_inst, cfg.Hkv, cfg.L, cfg.W, cfg.G
    want = "two-pass" if choose == "auto" else "single-read"
    assert laq.laq_score_kernel(n, cfg.Hq, Hkv, cfg.d, L, W, k.dtype, choose=choose) == want
    scores, idx, ko, vo = laq.laq_evict(q, k, v, budgets, cfg.pool, choose=choose)
    raw = laq.laq_score(q, k, 1, choose=choose)
    torch.cuda.synchronize()
    idx_l = split_packed(idx.cpu(), budgets, Hkv, L)
    ko_l = split_packed(ko.cpu(), budgets, Hkv, L)
    vo_l = split_packed(vo.cpu(), budgets, Hkv, L)
    for (i, g) in [(0, 0), (13, 3), (31, 7)]:
        print("cfg4 sample", i, g, flush=True)
        qc, kc = q[i, g * G:(g + 1) * G].cpu(), k[i, g:g + 1].cpu()
        pooled = oracle.maxpool(oracle.raw_scores(qc, kc), W, cfg.pool)
        check_scores(scores[i, g].cpu(), pooled[0], k.dtype, "cfg4 inst %d head %d" % (i, g))
        check_index_row(idx_l[i][g].numpy(), pooled[0].float().numpy(), W, budgets[i], 1e-3, "cfg4")
        assert torch.equal(oracle.select(scores[i, g:g + 1].cpu(), W, budgets[i])[0], idx_l[i][g])
        rows = idx_l[i][g].long()
        assert torch.equal(ko_l[i][g], k[i, g].cpu()[rows]) and torch.equal(vo_l[i][g], v[i, g].cpu()[rows])
    # properties that hold at any size, on every instance and head
    np.testing.assert_allclose(raw.double().sum(dim=2).cpu().numpy(), cfg.R, rtol=2e-4)     # rows sum to 1
    assert (scores >= raw).all() and (raw >= 0).all()
    for i in range(n):
        assert (idx_l[i][:, 1:] > idx_l[i][:, :-1]).all()
        assert (idx_l[i][:, -W:] == torch.arange(L - W, L, dtype=torch.int32)).all()


def test_config5_sampled(laq):
    # 4 of the 256 instances at full length (heavy-tailed query norms), sampled heads
    cfg = CONFIGS[5]
    inst = [0, 77, 200, 255]
    q, k, v, budgets, _ = make_batch(cfg, device=DEV, instances=inst)
    run_and_check(laq, q, k, v, budgets, cfg.pool, "cfg5", heads=[2])


EDGE = [
    # name, dtype, Hq, Hkv, d, L, W, pool, budget
    ("ragged-L", torch.bfloat16, 8, 2, 128, 1000, 8, 7, 100),
    ("one-chunk", torch.bfloat16, 8, 2, 128, 200, 8, 7, 64),
    ("L-lt-tile", torch.bfloat16, 8, 2, 128, 19, 4, 7, 8),
    ("budget-ge-L", torch.bfloat16, 8, 2, 128, 300, 8, 7, 400),
    ("budget-eq-W", torch.bfloat16, 8, 2, 128, 300, 8, 7, 8),
    ("budget-eq-L-1", torch.bfloat16, 8, 2, 128, 300, 8, 7, 299),
    ("pool1", torch.bfloat16, 8, 2, 128, 777, 8, 1, 64),
    ("pool3", torch.bfloat16, 8, 2, 128, 777, 8, 3, 64),
    ("pool63", torch.bfloat16, 8, 2, 128, 777, 8, 63, 200),
    ("W1-G1-one-score-row", torch.bfloat16, 2, 2, 128, 600, 1, 7, 50),
    ("R48-three-tiles", torch.bfloat16, 12, 2, 128, 900, 8, 7, 64),
    ("R160-two-groups", torch.bfloat16, 10, 1, 128, 700, 16, 7, 64),
    ("R20-padded", torch.bfloat16, 5, 1, 128, 700, 4, 7, 64),
    ("R1200-many-row-groups", torch.bfloat16, 4, 1, 128, 700, 300, 7, 400),
    ("R288-nine-tiles", torch.bfloat16, 4, 1, 64, 1300, 72, 5, 200),
    ("d64-mfma", torch.bfloat16, 8, 2, 64, 1500, 8, 7, 128),
    ("d64-R64", torch.bfloat16, 16, 2, 64, 1500, 8, 7, 128),
    ("d96-generic-bf16", torch.bfloat16, 4, 2, 96, 400, 4, 7, 32),
    ("fp32-d128", torch.float32, 8, 2, 128, 700, 4, 7, 64),
    ("fp32-G1", torch.float32, 3, 3, 32, 300, 5, 5, 40),
    ("window-is-everything", torch.bfloat16, 8, 2, 128, 32, 32, 7, 32),
    ("P-eq-1", torch.bfloat16, 8, 2, 128, 9, 8, 7, 9),
    ("long-window", torch.bfloat16, 8, 2, 128, 900, 300, 7, 400),
    ("window-of-600-queries-beyond-the-position-table", torch.bfloat16, 2, 1, 128, 700, 600, 7, 650),
    # pooling windows that cross the 256-key chunk boundaries of pass 2
    ("prefix-ends-on-chunk-boundary", torch.bfloat16, 8, 2, 128, 520, 8, 7, 64),
    ("prefix-ends-one-past-boundary", torch.bfloat16, 8, 2, 128, 521, 8, 7, 64),
    ("prefix-ends-one-before-boundary", torch.bfloat16, 8, 2, 128, 519, 8, 7, 64),
    ("prefix-ends-inside-boundary-window", torch.bfloat16, 8, 2, 128, 267, 8, 7, 64),
    ("pool63-four-chunks", torch.bfloat16, 8, 2, 128, 1024, 8, 63, 200),
    ("pool63-boundary-window-clipped-by-prefix", torch.bfloat16, 8, 2, 128, 290, 8, 63, 100),
    ("pool5-length-multiple-of-chunk", torch.bfloat16, 16, 2, 64, 768, 8, 5, 90),
    ("pool3-R128", torch.bfloat16, 32, 2, 128, 600, 8, 3, 64),
]


@pytest.mark.parametrize("name,dtype,Hq,Hkv,d,L,W,pool,budget", EDGE, ids=[e[0] for e in EDGE])
def test_edge_cases(laq, name, dtype, Hq, Hkv, d, L, W, pool, budget):
    g = torch.Generator().manual_seed(len(name) * 1000 + L)
    n = 2
    q = (torch.randn(n, Hq, W, d, generator=g) * 1.5).to(dtype).to(DEV)
    k = torch.randn(n, Hkv, L, d, generator=g).to(dtype).to(DEV)
    v = torch.randn(n, Hkv, L, d, generator=g).to(dtype).to(DEV)
    run_and_check(laq, q, k, v, [budget, max(W, budget - 3)], pool, name)


def test_peaks_on_chunk_boundaries_spread_to_both_sides(laq):
    # keys aligned with the window queries right before and after every 256-key boundary: their
    # pooled plateau must reach across the boundary in both directions
    g = torch.Generator().manual_seed(5)
    Hq, Hkv, d, L, W = 8, 2, 128, 1100, 8
    q = torch.randn(1, Hq, W, d, generator=g)
    k = torch.randn(1, Hkv, L, d, generator=g) * 0.5
    for b in (256, 512, 768, 1024):
        k[0, 0, b - 1] = q[0, 0].mean(0) * 3.0
        k[0, 1, b] = q[0, 4].mean(0) * 3.0
    q, k = q.bfloat16().to(DEV), k.bfloat16().to(DEV)
    v = torch.randn(1, Hkv, L, d, generator=g).bfloat16().to(DEV)
    sc = run_and_check(laq, q, k, v, [80], 7, "boundary-peaks")[0].cpu()
    for b in (256, 512, 768, 1024):
        assert (sc[0, 0, b - 4:b + 3] == sc[0, 0, b - 1]).all()       # plateau of key b-1
        assert (sc[0, 1, b - 3:b + 4] == sc[0, 1, b]).all()           # plateau of key b


def test_very_long_sequence(laq):
    # one head of 513 chunks: more units than workgroups, all on one head
    g = torch.Generator().manual_seed(77)
    Hq, Hkv, d, L, W = 4, 1, 128, 131072 + 40, 8
    q = torch.randn(1, Hq, W, d, generator=g).bfloat16().to(DEV)
    k = torch.randn(1, Hkv, L, d, generator=g).bfloat16().to(DEV)
    v = torch.randn(1, Hkv, L, d, generator=g).bfloat16().to(DEV)
    run_and_check(laq, q, k, v, [1024], 7, "L131k")


def test_many_heads_dynamic_runs_and_one_unit_tail(laq):
    # 513 short heads = 8721 units per pass: enough for the streaming kernels to hand out the tail of
    # the work in runs of 4 through their counter, and 8721 - 512*10 = 4*900 + 1 leaves a last run of
    # one unit (on a device that holds 512 workgroups).  Sampled heads against the oracle, invariants
    # on everything, and the same bits on a second call.
    n, Hq, Hkv, d, L, W, pool, budget = 57, 18, 9, 128, 4100, 16, 7, 300
    G = Hq // Hkv
    gen = torch.Generator(device=DEV).manual_seed(2024)
    q = (torch.randn(n, Hq, W, d, generator=gen, device=DEV) * 1.5).bfloat16()
    k = torch.randn(n, Hkv, L, d, generator=gen, device=DEV).bfloat16()
    v = torch.randn(n, Hkv, L, d, generator=gen, device=DEV).bfloat16()
    budgets = [budget] * n
    scores, idx, ko, vo = laq.laq_evict(q, k, v, budgets, pool)
    raw = laq.laq_score(q, k, 1)
    again = laq.laq_evict(q, k, v, budgets, pool)
    torch.cuda.synchronize()
    for x, y in zip((scores, idx, ko, vo), again):
        assert torch.equal(x, y)
    np.testing.assert_allclose(raw.double().sum(dim=2).cpu().numpy(), G * W, rtol=2e-4)
    assert (scores >= raw).all() and (raw >= 0).all()
    idx_l = split_packed(idx.cpu(), budgets, Hkv, L)
    ko_l = split_packed(ko.cpu(), budgets, Hkv, L)
    for (i, g) in [(0, 0), (22, 4), (39, 8), (56, 8)]:       # first, middle (static / claimed runs), very last head
        print("many-heads sample", i, g, flush=True)
        qc, kc = q[i, g * G:(g + 1) * G].cpu(), k[i, g:g + 1].cpu()
        r = oracle.raw_scores(qc, kc)
        pooled = oracle.maxpool(r, W, pool)
        check_scores(raw[i, g].cpu(), r[0], k.dtype, "many-heads raw inst %d head %d" % (i, g))
        check_scores(scores[i, g].cpu(), pooled[0], k.dtype, "many-heads inst %d head %d" % (i, g))
        check_index_row(idx_l[i][g].numpy(), pooled[0].float().numpy(), W, budget, 1e-3, "many-heads")
        assert torch.equal(oracle.select(scores[i, g:g + 1].cpu(), W, budget)[0], idx_l[i][g])
        assert torch.equal(ko_l[i][g], k[i, g].cpu()[idx_l[i][g].long()])


def test_per_instance_budgets_pack_correctly(laq):
    cfg = dataclasses.replace(CONFIGS[4], L=2048, n_layer=5)
    q, k, v, budgets, _ = make_batch(cfg, device=DEV)
    assert len(set(budgets)) == 5
    run_and_check(laq, q, k, v, budgets, cfg.pool, "pyramid-small")


def test_all_keys_identical_all_ties(laq):
    Hq, Hkv, d, L, W, budget = 8, 2, 128, 700, 8, 100
    g = torch.Generator().manual_seed(1)
    q = torch.randn(1, Hq, W, d, generator=g).bfloat16().to(DEV)
    k = torch.randn(1, 1, 1, d, generator=g).bfloat16().expand(1, Hkv, L, d).contiguous().to(DEV)
    scores, idx, _, _ = laq.laq_evict(q, k, None, [budget], 7)
    got = idx.cpu().reshape(Hkv, budget)
    # every prefix score is the same number, so the lowest positions win
    P = L - W
    s = scores.cpu()
    assert (s[0, :, :P] == s[0, :, :1]).all()
    want = torch.tensor(list(range(budget - W)) + list(range(P, L)), dtype=torch.int32)
    assert (got == want).all()
    expect = 4 * sum(1.0 / (P + w + 1) for w in range(W))
    np.testing.assert_allclose(s[0, :, :P].double().numpy(), expect, rtol=1e-5)


def test_extreme_logits(laq):
    # logits of magnitude >> 10 (what the heavy-tailed config stresses): no overflow, rows still sum to 1
    Hq, Hkv, d, L, W = 8, 2, 128, 1024, 8
    g = torch.Generator().manual_seed(2)
    q = (torch.randn(1, Hq, W, d, generator=g) * 40).bfloat16().to(DEV)
    k = torch.randn(1, Hkv, L, d, generator=g).bfloat16().to(DEV)
    v = torch.randn(1, Hkv, L, d, generator=g).bfloat16().to(DEV)
    run_and_check(laq, q, k, v, [64], 7, "extreme")
    raw = laq.laq_score(q, k, 1)
    assert torch.isfinite(raw).all()
    np.testing.assert_allclose(raw.double().sum(dim=2).cpu().numpy(), 32.0, rtol=1e-4)


def test_select_alone_with_ties_and_memory_path(laq):
    # scores with few distinct values (many ties across the boundary); L above the register-resident limit
    g = torch.Generator().manual_seed(4)
    for (Hkv, L, W, budget, pool) in [(3, 5000, 8, 600, 1), (2, 40000, 16, 3000, 1), (2, 40000, 16, 3000, 7),
                                      (2, 2000, 4, 100, 5), (1, 70000, 8, 70000 - 5, 1)]:
        s = (torch.randint(0, 50, (2, Hkv, L), generator=g).float() / 7).to(DEV)
        print("select case", Hkv, L, W, budget, pool, flush=True)
        idx = laq.laq_select(s, [budget, budget + 1], pool, W)
        torch.cuda.synchronize()
        parts = split_packed(idx.cpu(), [budget, budget + 1], Hkv, L)
        for i, b in enumerate([budget, budget + 1]):
            pooled = oracle.maxpool(s[i].cpu().double(), W, pool).float()
            assert torch.equal(parts[i], oracle.select(pooled, W, b))


def test_select_four_scores_per_load_and_its_fallbacks(laq):
    # final scores (pool 1) whose rows start 16-byte aligned are fetched four per load; row lengths
    # that are not a multiple of four and a misaligned score plane take the single loads.  Few
    # distinct values: ties across the boundary in every register class (8 and 32 keys per lane) and
    # in the many-heads instantiation
    g = torch.Generator().manual_seed(14)
    cases = [(2, 32768, 16, 1500, False), (3, 20000, 8, 999, False), (2, 8192 + 8, 8, 4000, False),
             (2, 30001, 8, 700, False), (2, 6002, 4, 300, False), (2, 32768, 16, 1500, True), (2, 6000, 8, 64, True),
             (400, 9000, 8, 240, False)]
    for (Hkv, L, W, budget, misaligned) in cases:
        n = 2
        vals = torch.randint(0, 40, (n, Hkv, L), generator=g).float() / 7
        if misaligned:
            flat = torch.empty(n * Hkv * L + 1, device=DEV)
            s = flat[1:].view(n, Hkv, L)
            s.copy_(vals)
            assert s.data_ptr() % 16 == 4 and s.is_contiguous()
        else:
            s = vals.to(DEV)
        print("select case", Hkv, L, W, budget, misaligned, flush=True)
        idx = laq.laq_select(s, [budget, budget + 3], 1, W)
        torch.cuda.synchronize()
        parts = split_packed(idx.cpu(), [budget, budget + 3], Hkv, L)
        for i, bud in enumerate([budget, budget + 3]):
            assert torch.equal(parts[i], oracle.select(vals[i], W, bud))


def test_deterministic_bits(laq):
    cfg = dataclasses.replace(CONFIGS[3], L=4096, n_layer=3)
    q, k, v, budgets, _ = make_batch(cfg, device=DEV)
    a = laq.laq_evict(q, k, v, budgets, cfg.pool)
    b = laq.laq_evict(q, k, v, budgets, cfg.pool)
    torch.cuda.synchronize()
    for x, y in zip(a, b):
        assert torch.equal(x, y)


def test_explicit_scale(laq):
    g = torch.Generator().manual_seed(9)
    q = torch.randn(1, 8, 8, 128, generator=g).bfloat16().to(DEV)
    k = torch.randn(1, 2, 500, 128, generator=g).bfloat16().to(DEV)
    run_and_check(laq, q, k, None, [64], 7, "scale", scale=0.02)


# ---- general observation window (Eq. 5): explicit query positions, independent keep count ----
def run_general(laq, q, k, v, budgets, pool, q_pos, keep, what, heads=None, pool_mode="max"):
    n, Hq, W, d = q.shape
    _, Hkv, L, _ = k.shape
    G = Hq // Hkv
    print("case:", what, "n=%d Hq=%d Hkv=%d d=%d L=%d W=%d pool=%d(%s) keep=%d" % (
        n, Hq, Hkv, d, L, W, pool, pool_mode, keep), flush=True)
    scores, idx, ko, vo = laq.laq_evict(q, k, v, budgets, pool, q_pos=q_pos, keep=keep, pool_mode=pool_mode)
    s3 = laq.laq_score(q, k, pool, q_pos=q_pos, keep=keep, pool_mode=pool_mode)
    i3 = laq.laq_select(s3, budgets, 1, keep, pool_mode=pool_mode)
    k3, v3 = laq.laq_compact(k, v, i3, budgets, keep)
    raw = laq.laq_score(q, k, 1, q_pos=q_pos, keep=keep, pool_mode=pool_mode)
    i_alt = laq.laq_select(raw, budgets, pool, keep, pool_mode=pool_mode)
    torch.cuda.synchronize()
    assert torch.equal(s3, scores) and torch.equal(i3, idx) and torch.equal(k3, ko) and torch.equal(v3, vo)
    assert torch.equal(i_alt, idx)
    idx_l = split_packed(idx.cpu(), budgets, Hkv, L)
    ko_l = split_packed(ko.cpu(), budgets, Hkv, L)
    vo_l = split_packed(vo.cpu(), budgets, Hkv, L)
    qc, kc, vc, sc, rc = q.cpu(), k.cpu(), v.cpu(), scores.cpu(), raw.cpu()
    for i in range(n):
        for g in (range(Hkv) if heads is None else heads):
            o_raw = oracle.raw_scores(qc[i, g * G:(g + 1) * G], kc[i, g:g + 1], q_pos=q_pos)
            pooled = (oracle.maxpool if pool_mode == "max" else oracle.avgpool)(o_raw, keep, pool)
            check_scores(rc[i, g], o_raw[0], k.dtype, "%s raw inst %d head %d" % (what, i, g))
            check_scores(sc[i, g], pooled[0], k.dtype, "%s inst %d head %d" % (what, i, g))
            check_index_row(idx_l[i][g].numpy(), pooled[0].float().numpy(), keep, budgets[i], RTOL[k.dtype],
                            "%s inst %d head %d" % (what, i, g))
            assert torch.equal(oracle.select(sc[i, g:g + 1], keep, budgets[i])[0], idx_l[i][g])
            rows = idx_l[i][g].long()
            assert torch.equal(ko_l[i][g], kc[i, g, rows]) and torch.equal(vo_l[i][g], vc[i, g, rows])
    return scores, idx


def _qkv(seed, n, Hq, Hkv, d, L, W, dtype=torch.bfloat16):
    g = torch.Generator().manual_seed(seed)
    q = (torch.randn(n, Hq, W, d, generator=g) * 1.5).to(dtype).to(DEV)
    k = torch.randn(n, Hkv, L, d, generator=g).to(dtype).to(DEV)
    v = torch.randn(n, Hkv, L, d, generator=g).to(dtype).to(DEV)
    return q, k, v


GENERAL = [
    # name, dtype, Hq, Hkv, d, L, W, pool, budget, keep, positions (callable of L, W)
    ("lookahead-only", torch.bfloat16, 8, 2, 128, 1000, 8, 7, 100, 0, lambda L, W: [L + i for i in range(W)]),
    ("lookahead-keep-local-8", torch.bfloat16, 8, 2, 128, 1000, 8, 7, 100, 8, lambda L, W: [L - 1] * W),
    ("lookahead-no-ragged-chunk", torch.bfloat16, 8, 2, 128, 1024, 8, 7, 64, 0, lambda L, W: [L + 7] * W),
    ("joined-8-local-8-lookahead", torch.bfloat16, 16, 4, 128, 2000, 16, 7, 128, 8,
     lambda L, W: [L - 8 + i for i in range(8)] + [L + i for i in range(8)]),
    ("scattered-positions-three-tiles", torch.bfloat16, 12, 2, 128, 900, 8, 5, 64, 4,
     lambda L, W: [0, 5, 255, 256, 511, 700, L - 1, 3 * L]),
    ("scattered-fp32-generic", torch.float32, 4, 2, 64, 500, 6, 3, 40, 2, lambda L, W: [499, 0, 17, 300, 1000, 256]),
    ("d64-joined", torch.bfloat16, 8, 2, 64, 1500, 16, 7, 128, 8,
     lambda L, W: [L - 8 + i for i in range(8)] + [L - 1] * 8),
    ("keep-everything", torch.bfloat16, 8, 2, 128, 300, 8, 7, 300, 300, lambda L, W: [L] * W),
    ("many-queries-more-than-keys", torch.bfloat16, 4, 2, 128, 40, 64, 3, 20, 0, lambda L, W: [w % 40 for w in range(W)]),
]


@pytest.mark.parametrize("name,dtype,Hq,Hkv,d,L,W,pool,budget,keep,pos", GENERAL, ids=[e[0] for e in GENERAL])
def test_general_window(laq, name, dtype, Hq, Hkv, d, L, W, pool, budget, keep, pos):
    q, k, v = _qkv(len(name) * 77 + L, 2, Hq, Hkv, d, L, W, dtype)
    run_general(laq, q, k, v, [budget, max(keep, budget - 3, 1)], pool, pos(L, W), keep, name)


def test_explicit_trailing_positions_give_the_default_bits(laq):
    q, k, v = _qkv(5, 2, 8, 2, 128, 1300, 8)
    L, W = 1300, 8
    a = laq.laq_evict(q, k, v, [100, 90], 7)
    b = laq.laq_evict(q, k, v, [100, 90], 7, q_pos=[L - W + w for w in range(W)], keep=W)
    torch.cuda.synchronize()
    for x, y in zip(a, b):
        assert torch.equal(x, y)


def test_joined_window_full_size_sampled(laq):
    # the 32k shape with the paper's main setting of 8 local window queries + 8 lookahead queries
    n, Hq, Hkv, d, L, W, pool, keep = 4, 32, 8, 128, 32768, 16, 7, 8
    gen = torch.Generator(device=DEV).manual_seed(99)
    q = (torch.randn(n, Hq, W, d, generator=gen, device=DEV) * 1.5).bfloat16()
    k = torch.randn(n, Hkv, L, d, generator=gen, device=DEV).bfloat16()
    v = torch.randn(n, Hkv, L, d, generator=gen, device=DEV).bfloat16()
    pos = [L - 8 + i for i in range(8)] + [L + i for i in range(8)]
    run_general(laq, q, k, v, [1024, 512, 256, 128], pool, pos, keep, "joined-32k", heads=[3])


# ---- stage-1 eviction variants (Sec. 4.2; Sec. 5.1 for the average pool) ----
def _trailing(L, W):
    return [L - W + w for w in range(W)]


STAGE1_AVG = [
    # name, dtype, Hq, Hkv, d, L, W, pool, budget
    ("avg7-llama-like", torch.bfloat16, 8, 2, 128, 1000, 8, 7, 100),
    ("avg7-two-row-tiles-d64", torch.bfloat16, 16, 2, 64, 1500, 8, 7, 128),
    ("avg3-fp32-generic", torch.float32, 4, 2, 64, 500, 6, 3, 40),
    ("avg1-is-raw", torch.bfloat16, 8, 2, 128, 700, 8, 1, 64),
    ("avg9-prefix-shorter-than-kernel", torch.float32, 2, 1, 32, 12, 8, 9, 10),
    ("avg63-widest-kernel", torch.bfloat16, 8, 2, 128, 600, 8, 63, 50),
    ("avg5-budget-equals-window", torch.bfloat16, 8, 2, 128, 300, 8, 5, 8),
]


@pytest.mark.parametrize("name,dtype,Hq,Hkv,d,L,W,pool,budget", STAGE1_AVG, ids=[e[0] for e in STAGE1_AVG])
def test_stage_one_average_pool(laq, name, dtype, Hq, Hkv, d, L, W, pool, budget):
    q, k, v = _qkv(len(name) * 31 + L, 2, Hq, Hkv, d, L, W, dtype)
    run_general(laq, q, k, v, [budget, max(W, budget - 3)], pool, _trailing(L, W), W, name, pool_mode="avg")


def test_average_pool_default_layout_matches_explicit_layout_and_differs_from_max(laq):
    q, k, v = _qkv(12, 1, 8, 2, 128, 900, 8)
    a = laq.laq_evict(q, k, v, [64], 7, pool_mode="avg")
    b = laq.laq_evict(q, k, v, [64], 7, q_pos=_trailing(900, 8), keep=8, pool_mode="avg")
    m = laq.laq_evict(q, k, v, [64], 7)
    torch.cuda.synchronize()
    for x, y in zip(a, b):
        assert torch.equal(x, y)
    assert not torch.equal(a[0], m[0])
    # the mean of seven non-negative scores never exceeds their maximum
    assert (a[0][..., :892] <= m[0][..., :892] * (1 + 1e-6)).all()


def test_average_pool_full_size_sampled(laq):
    # stage-1 eviction at the 32k shape: prompt suffix as window, low budget, average pool
    cfg = CONFIGS[4]
    n = 2
    q = torch.empty(n, cfg.Hq, cfg.W, cfg.d, dtype=cfg.torch_dtype, device=DEV)
    k = torch.empty(n, cfg.Hkv, cfg.L, cfg.d, dtype=cfg.torch_dtype, device=DEV)
    v = torch.empty_like(k)
    for i in range(n):
        qi, ki, vi, _ = make_instance(cfg, 0, i, device=DEV)
        q[i].copy_(qi); k[i].copy_(ki); v[i].copy_(vi)
    run_general(laq, q, k, v, [256, 128], cfg.pool, _trailing(cfg.L, cfg.W), cfg.W, "avg-32k", heads=[5],
                pool_mode="avg")


SINKS = [
    # name, Hkv, L, n_sink, budgets
    ("four-sinks", 8, 4096, 4, [256, 128, 64]),
    ("no-sinks", 2, 1000, 0, [100]),
    ("sinks-fill-the-budget", 2, 1000, 16, [16, 8, 17]),
    ("budget-beyond-length", 3, 50, 4, [50, 80, 49]),
    ("single-row", 1, 1, 4, [1]),
    ("long-rows-many-strides", 2, 40000, 4, [30000, 1]),
]


@pytest.mark.parametrize("name,Hkv,L,n_sink,budgets", SINKS, ids=[e[0] for e in SINKS])
def test_sink_recent_list_and_compaction(laq, name, Hkv, L, n_sink, budgets):
    print("case:", name, "Hkv=%d L=%d n_sink=%d budgets=%s" % (Hkv, L, n_sink, budgets), flush=True)
    n = len(budgets)
    idx = laq.laq_select_sink_recent(n, Hkv, L, budgets, n_sink, device=DEV)
    g = torch.Generator().manual_seed(L)
    k = torch.randn(n, Hkv, L, 64, generator=g).bfloat16().to(DEV)
    v = torch.randn(n, Hkv, L, 64, generator=g).bfloat16().to(DEV)
    ko, vo = laq.laq_compact(k, v, idx, budgets, 0)
    torch.cuda.synchronize()
    idx_l = split_packed(idx.cpu(), budgets, Hkv, L)
    ko_l = split_packed(ko.cpu(), budgets, Hkv, L)
    vo_l = split_packed(vo.cpu(), budgets, Hkv, L)
    for i in range(n):
        want = oracle.sink_recent(Hkv, L, n_sink, budgets[i])
        assert torch.equal(idx_l[i], want), "%s inst %d" % (name, i)
        assert torch.equal(ko_l[i], oracle.compact(k[i].cpu(), want))
        assert torch.equal(vo_l[i], oracle.compact(v[i].cpu(), want))


def test_sink_recent_more_instances_than_one_launch_holds(laq):
    n, Hkv, L = 600, 2, 300
    budgets = [1 + (7 * i) % 320 for i in range(n)]
    idx = laq.laq_select_sink_recent(n, Hkv, L, budgets, 3, device=DEV)
    torch.cuda.synchronize()
    for i, rows in enumerate(split_packed(idx.cpu(), budgets, Hkv, L)):
        if i % 37 == 0 or i in (255, 256, 511, 512, 599):
            assert torch.equal(rows, oracle.sink_recent(Hkv, L, 3, budgets[i])), i


# ---- recall of one selection against another (Sec. 3, Eq. 1-3) ----
def _random_lists(seed, n, Hkv, L, budgets):
    rng = np.random.default_rng(seed)
    rows = []
    for b in budgets:
        bk = min(b, L)
        rows.append(np.stack([np.sort(rng.permutation(L)[:bk]) for _ in range(Hkv)]).astype(np.int32))
    return rows


RECALL = [
    # name, Hkv, L, pred budgets, gold budgets
    ("equal-budgets", 4, 1000, [64, 128, 7], [64, 128, 7]),
    ("different-budgets", 2, 500, [50, 500, 1], [80, 20, 499]),
    ("budget-beyond-length", 2, 40, [100, 40], [39, 100]),
    ("long-lists", 2, 40000, [30000, 2048], [2048, 30000]),
    ("single-position", 1, 1, [1], [1]),
]


@pytest.mark.parametrize("name,Hkv,L,bp,bg", RECALL, ids=[e[0] for e in RECALL])
def test_recall_of_random_lists(laq, name, Hkv, L, bp, bg):
    print("case:", name, "Hkv=%d L=%d pred=%s gold=%s" % (Hkv, L, bp, bg), flush=True)
    n = len(bp)
    pred = _random_lists(len(name), n, Hkv, L, bp)
    gold = _random_lists(len(name) + 1000, n, Hkv, L, bg)
    p_dev = torch.from_numpy(np.concatenate([r.reshape(-1) for r in pred])).to(DEV)
    g_dev = torch.from_numpy(np.concatenate([r.reshape(-1) for r in gold])).to(DEV)
    overlap, recall = laq.laq_recall(p_dev, bp, g_dev, bg, Hkv, L)
    same, one = laq.laq_recall(g_dev, bg, g_dev, bg, Hkv, L)
    torch.cuda.synchronize()
    for i in range(n):
        want = oracle.overlap(torch.from_numpy(pred[i]), torch.from_numpy(gold[i]), L)
        assert torch.equal(overlap[i].cpu(), want), "%s inst %d" % (name, i)
        np.testing.assert_array_equal(recall[i].cpu().numpy(),
                                      (want.float() / np.float32(min(bg[i], L))).numpy())
        assert same[i].cpu().tolist() == [min(bg[i], L)] * Hkv and one[i].cpu().tolist() == [1.0] * Hkv


def test_recall_more_instances_than_one_launch_holds(laq):
    n, Hkv, L = 300, 2, 200
    bp = [1 + (11 * i) % 210 for i in range(n)]
    bg = [1 + (7 * i) % 190 for i in range(n)]
    pred, gold = _random_lists(1, n, Hkv, L, bp), _random_lists(2, n, Hkv, L, bg)
    p_dev = torch.from_numpy(np.concatenate([r.reshape(-1) for r in pred])).to(DEV)
    g_dev = torch.from_numpy(np.concatenate([r.reshape(-1) for r in gold])).to(DEV)
    overlap, _ = laq.laq_recall(p_dev, bp, g_dev, bg, Hkv, L)
    torch.cuda.synchronize()
    for i in list(range(0, n, 23)) + [127, 128, 255, 256, 299]:
        assert torch.equal(overlap[i].cpu(), oracle.overlap(torch.from_numpy(pred[i]), torch.from_numpy(gold[i]), L)), i


def test_recall_of_the_window_selection_against_the_selection_by_all_queries(laq):
    # Eq. 1-3 end to end on the library's own selections: M_pred from the first 8 queries, M_gold
    # from all 32 (every query placed after the prompt), 4k keys
    q, k, v = _qkv(21, 2, 32, 8, 128, 4096, 32)
    L, budgets = 4096, [256, 128]
    see_all = [L] * 32
    gold = laq.laq_evict(q, k, v, budgets, 7, q_pos=see_all, keep=0)[1]
    pred = laq.laq_evict(q[:, :, :8].contiguous(), k, v, budgets, 7, q_pos=see_all[:8], keep=0)[1]
    sinks = laq.laq_select_sink_recent(2, 8, L, budgets, 4, device=DEV)
    ov, rec = laq.laq_recall(pred, budgets, gold, budgets, 8, L)
    ov_s, rec_s = laq.laq_recall(sinks, budgets, gold, budgets, 8, L)
    torch.cuda.synchronize()
    pl, gl, sl = (split_packed(x.cpu(), budgets, 8, L) for x in (pred, gold, sinks))
    for i in range(2):
        assert torch.equal(ov[i].cpu(), oracle.overlap(pl[i], gl[i], L))
        assert torch.equal(ov_s[i].cpu(), oracle.overlap(sl[i], gl[i], L))
    assert (rec > 0).all() and (rec <= 1).all()
    # scored selections agree far more with the reference than the score-free list does
    assert rec.mean().item() > rec_s.mean().item()


# ---- the steps around the path: Q-cache capture (Sec. 4.2), decoding on the compacted cache (Sec. 4.3) ----
def check_decode(got_f32, q, kc, vc, dtype, what, scale=0.0):
    """|got - want| <= rtol * sum_j p_j |v_j| element by element (the scale of the sum that the
    rounding errors of the weights act on), want and the bound from the oracle."""
    want = oracle.decode_attention(q, kc, vc, scale)
    bound = oracle.decode_attention(q, kc, vc.abs(), scale) * RTOL[dtype] + 1e-30
    err = (got_f32.double() - want).abs()
    assert torch.isfinite(got_f32).all(), what
    assert (err <= bound).all(), "%s: worst err/bound %.3f" % (what, float((err / bound).max()))


DECODE = [
    # name, dtype, Hq, Hkv, d, L, budgets
    ("mistral-like", torch.bfloat16, 32, 8, 128, 4096, [128, 2048, 5000]),
    ("G1", torch.bfloat16, 4, 4, 128, 600, [77]),
    ("G2", torch.bfloat16, 8, 4, 128, 600, [300, 1]),
    ("G3-masked-head-slot", torch.bfloat16, 6, 2, 128, 500, [100]),
    ("G8-two-head-batches", torch.bfloat16, 16, 2, 128, 700, [256]),
    ("G6-ragged-second-batch", torch.bfloat16, 6, 1, 64, 700, [100]),
    ("d64", torch.bfloat16, 8, 2, 64, 900, [500]),
    ("d96-idle-lanes", torch.bfloat16, 4, 2, 96, 400, [64]),
    ("d256", torch.bfloat16, 4, 2, 256, 300, [300]),
    ("d8", torch.bfloat16, 2, 2, 8, 100, [40]),
    ("fp32", torch.float32, 8, 2, 128, 500, [64, 200]),
    ("fp32-d40", torch.float32, 4, 2, 40, 300, [33]),
    ("fewer-rows-than-lane-groups", torch.bfloat16, 8, 2, 128, 50, [3, 15, 16, 17]),
    ("long-cache", torch.bfloat16, 8, 2, 128, 33000, [33000]),
]


@pytest.mark.parametrize("name,dtype,Hq,Hkv,d,L,budgets", DECODE, ids=[e[0] for e in DECODE])
def test_decode_attention_on_packed_cache(laq, name, dtype, Hq, Hkv, d, L, budgets):
    print("case:", name, "Hq=%d Hkv=%d d=%d L=%d budgets=%s" % (Hq, Hkv, d, L, budgets), flush=True)
    n = len(budgets)
    g = torch.Generator().manual_seed(len(name) * 13 + d)
    total, _ = laq.packed_rows(budgets, Hkv, L)
    q = (torch.randn(n, Hq, d, generator=g) * 1.5).to(dtype)
    kc = torch.randn(total, d, generator=g).to(dtype)
    vc = torch.randn(total, d, generator=g).to(dtype)
    out = laq.laq_decode_attention(q.to(DEV), kc.to(DEV), vc.to(DEV), budgets, Hkv, L)
    again = laq.laq_decode_attention(q.to(DEV), kc.to(DEV), vc.to(DEV), budgets, Hkv, L)
    torch.cuda.synchronize()
    assert torch.equal(out, again)
    k_l, v_l = split_packed(kc, budgets, Hkv, L), split_packed(vc, budgets, Hkv, L)
    for i in range(n):
        check_decode(out[i].cpu(), q[i], k_l[i].contiguous(), v_l[i].contiguous(), dtype, "%s inst %d" % (name, i))


def test_decode_attention_extreme_logits_and_scale(laq):
    g = torch.Generator().manual_seed(8)
    q = (torch.randn(1, 8, 128, generator=g) * 30).bfloat16()
    kc = (torch.randn(2 * 200, 128, generator=g) * 30).bfloat16()
    vc = torch.randn(2 * 200, 128, generator=g).bfloat16()
    for scale in (0.0, 1.0, 0.01):
        out = laq.laq_decode_attention(q.to(DEV), kc.to(DEV), vc.to(DEV), [200], 2, 200, scale=scale)
        torch.cuda.synchronize()
        check_decode(out[0].cpu(), q[0], kc.view(2, 200, 128), vc.view(2, 200, 128), torch.bfloat16,
                     "scale %g" % scale, scale)


def test_evict_then_decode_on_the_compacted_cache(laq):
    cfg = CONFIGS[2]
    q, k, v, budgets, _ = make_batch(cfg, device=DEV)
    _, idx, ko, vo = laq.laq_evict(q, k, v, budgets, cfg.pool)
    gen = torch.Generator(device=DEV).manual_seed(4)
    q_new = torch.randn(q.shape[0], cfg.Hq, cfg.d, generator=gen, device=DEV).to(k.dtype)
    out = laq.laq_decode_attention(q_new, ko, vo, budgets, cfg.Hkv, cfg.L)
    torch.cuda.synchronize()
    k_l = split_packed(ko.cpu(), budgets, cfg.Hkv, cfg.L)
    v_l = split_packed(vo.cpu(), budgets, cfg.Hkv, cfg.L)
    for i in range(q.shape[0]):
        check_decode(out[i].cpu(), q_new[i].cpu(), k_l[i].contiguous(), v_l[i].contiguous(), k.dtype, "inst %d" % i)


def test_qcache_capture_feeds_scoring(laq):
    n, Hq, Hkv, d, L, W = 2, 8, 2, 128, 700, 8
    g = torch.Generator().manual_seed(6)
    steps = [torch.randn(n, Hq, d, generator=g).bfloat16() for _ in range(W)]
    k = torch.randn(n, Hkv, L, d, generator=g).bfloat16().to(DEV)
    cache = torch.full((n, Hq, W, d), 7.0, dtype=torch.bfloat16, device=DEV)
    ref = torch.full((n, Hq, W, d), 7.0, dtype=torch.bfloat16)
    for t in (3, 0, 7, 1, 2, 6, 5, 4):                             # any order; a slot only changes its own rows
        laq.laq_qcache_store(cache, steps[t].to(DEV), t)
        for i in range(n):
            ref[i] = oracle.qcache_store(ref[i], steps[t][i], t)
        torch.cuda.synchronize()
        assert torch.equal(cache.cpu(), ref)
    assert torch.equal(cache.cpu(), torch.stack(steps, dim=2))
    pos = [L + t for t in range(W)]
    a = laq.laq_score(cache, k, 7, q_pos=pos, keep=0)
    b = laq.laq_score(torch.stack(steps, dim=2).to(DEV), k, 7, q_pos=pos, keep=0)
    torch.cuda.synchronize()
    assert torch.equal(a, b)
    cache32 = torch.zeros(1, 3, 4, 40, device=DEV)
    step32 = torch.randn(1, 3, 40, generator=g)
    laq.laq_qcache_store(cache32, step32.to(DEV), 2)
    torch.cuda.synchronize()
    assert torch.equal(cache32[:, :, 2].cpu(), step32) and cache32[:, :, :2].abs().sum() == 0


# ---- the path under stream capture ----
@pytest.mark.parametrize("choose", ["two-pass", "single-read"])
def test_evict_replays_from_a_captured_graph(laq, choose):
    """laq_evict enqueues kernels only (no allocation, no synchronisation, no memset node), so a
    caller may capture it into a graph; every replay must give the eager bits, also after the
    inputs changed in place and with eager work in between.  With either scoring kernel (the
    single-read one is a cooperative launch)."""
    cfg = dataclasses.replace(CONFIGS[2], L=3000)
    q, k, v, budgets, _ = make_batch(cfg, device=DEV)
    n = q.shape[0]
    total, _ = laq.packed_rows(budgets, cfg.Hkv, cfg.L)
    scores = torch.empty(n, cfg.Hkv, cfg.L, dtype=torch.float32, device=DEV)
    idx = torch.empty(total, dtype=torch.int32, device=DEV)
    ko = torch.empty(total, cfg.d, dtype=k.dtype, device=DEV)
    vo = torch.empty_like(ko)
    ws = torch.empty(laq.laq_workspace_bytes(n, cfg.Hq, cfg.Hkv, cfg.d, cfg.L, cfg.W, k.dtype), dtype=torch.uint8,
                     device=DEV)

    def run():
        laq.laq_evict(q, k, v, budgets, cfg.pool, scores=scores, idx=idx, k_out=ko, v_out=vo, ws=ws, choose=choose)

    assert laq.laq_score_kernel(n, cfg.Hq, cfg.Hkv, cfg.d, cfg.L, cfg.W, k.dtype, choose=choose) == choose
    laq.laq_init()                                   # attribute and occupancy queries, which a capture must not contain
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        run()
    gen = torch.Generator(device=DEV).manual_seed(3)
    for rep in range(4):
        if rep:
            k.copy_(torch.randn(k.shape, generator=gen, device=DEV).to(k.dtype))      # new inputs, same buffers
        eager = [t.clone() for t in laq.laq_evict(q, k, v, budgets, cfg.pool, choose=choose)]
        for t in (scores, idx, ko, vo):
            t.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for got, want in zip((scores, idx, ko, vo), eager):
            assert torch.equal(got, want), "replay %d" % rep


def test_more_instances_than_one_select_or_compact_launch_holds(laq):
    # 300 small instances with varying budgets: select, compact and decode walk their per-launch
    # tables of 256 instances twice; the packed offsets must carry over
    n, Hq, Hkv, d, L, W = 300, 4, 2, 128, 300, 4
    g = torch.Generator().manual_seed(44)
    q = (torch.randn(n, Hq, W, d, generator=g) * 1.5).bfloat16().to(DEV)
    k = torch.randn(n, Hkv, L, d, generator=g).bfloat16().to(DEV)
    v = torch.randn(n, Hkv, L, d, generator=g).bfloat16().to(DEV)
    budgets = [W + (13 * i) % 120 for i in range(n)]
    scores, idx, ko, vo = laq.laq_evict(q, k, v, budgets, 7)
    q_new = torch.randn(n, Hq, d, generator=g).bfloat16().to(DEV)
    out = laq.laq_decode_attention(q_new, ko, vo, budgets, Hkv, L)
    torch.cuda.synchronize()
    idx_l = split_packed(idx.cpu(), budgets, Hkv, L)
    ko_l, vo_l = split_packed(ko.cpu(), budgets, Hkv, L), split_packed(vo.cpu(), budgets, Hkv, L)
    sc, kc, vc = scores.cpu(), k.cpu(), v.cpu()
    for i in list(range(0, n, 41)) + [254, 255, 256, 257, 299]:
        want = oracle.select(sc[i], W, budgets[i])
        assert torch.equal(idx_l[i], want), i
        assert torch.equal(ko_l[i], oracle.compact(kc[i], want)) and torch.equal(vo_l[i], oracle.compact(vc[i], want)), i
        check_decode(out[i].cpu(), q_new[i].cpu(), ko_l[i].contiguous(), vo_l[i].contiguous(), torch.bfloat16,
                     "inst %d" % i)
    # scores of a sampled instance against the oracle end to end
    pooled = oracle.evict(q[256].cpu(), kc[256], vc[256], budgets[256], 7)[0]
    check_scores(sc[256], pooled, torch.bfloat16, "inst 256")


# ---- key / value caches that are not dense [n, Hkv, L, d] ----
def _token_major_view(t):
    """The same values stored [n, L, Hkv, d], handed over as a strided [n, Hkv, L, d] view."""
    return t.permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3)


def _padded_rows_view(t, pad=8):
    """Rows stored with `pad` unused elements after each (row stride d + pad)."""
    wide = torch.full(t.shape[:-1] + (t.shape[-1] + pad,), 7.0, dtype=t.dtype, device=t.device)
    wide[..., :t.shape[-1]] = t
    return wide[..., :t.shape[-1]]


STRIDED = [
    # name, dtype, Hq, Hkv, d, L, W, pool, budget
    ("token-major-R32", torch.bfloat16, 8, 2, 128, 1000, 8, 7, 100),
    ("token-major-R64-4k", torch.bfloat16, 16, 4, 128, 4096, 16, 7, 256),
    ("token-major-R128", torch.bfloat16, 32, 8, 128, 1500, 32, 7, 200),
    ("token-major-d64", torch.bfloat16, 8, 2, 64, 1500, 8, 7, 128),
    ("token-major-one-chunk", torch.bfloat16, 8, 2, 128, 200, 8, 5, 64),
    ("token-major-fp32-generic", torch.float32, 4, 2, 64, 500, 6, 3, 40),
    ("token-major-R4", torch.bfloat16, 2, 2, 128, 600, 4, 7, 50),
    ("token-major-d96-generic-bf16", torch.bfloat16, 4, 2, 96, 400, 4, 7, 32),
]


@pytest.mark.parametrize("name,dtype,Hq,Hkv,d,L,W,pool,budget", STRIDED, ids=[e[0] for e in STRIDED])
def test_strided_caches_give_the_dense_bits(laq, name, dtype, Hq, Hkv, d, L, W, pool, budget):
    q, k, v = _qkv(len(name) * 7 + L, 2, Hq, Hkv, d, L, W, dtype)
    budgets = [budget, max(W, budget - 5)]
    dense = laq.laq_evict(q, k, v, budgets, pool)
    for how, view in (("token-major", _token_major_view), ("padded-rows", _padded_rows_view)):
        print("case:", name, how, flush=True)
        kv, vv = view(k), view(v)
        assert not kv.is_contiguous() and torch.equal(kv, k)
        got = laq.laq_evict(q, kv, vv, budgets, pool)
        s3 = laq.laq_score(q, kv, pool)
        k3, v3 = laq.laq_compact(kv, vv, dense[1], budgets, W)
        torch.cuda.synchronize()
        for a, b in zip(got, dense):
            assert torch.equal(a, b), "%s %s" % (name, how)
        assert torch.equal(s3, dense[0]) and torch.equal(k3, dense[2]) and torch.equal(v3, dense[3])


def test_token_major_cache_against_the_oracle(laq):
    q, k, v = _qkv(91, 2, 16, 4, 128, 2100, 16)
    pos = [2100 - 8 + i for i in range(8)] + [2100 + i for i in range(8)]
    run_general(laq, q, _token_major_view(k), _token_major_view(v), [128, 96], 7, pos, 8, "token-major-joined")
    run_general(laq, q, _token_major_view(k), _token_major_view(v), [128, 96], 7, _trailing(2100, 16), 16,
                "token-major-avg", pool_mode="avg")


def test_token_major_full_size_sampled(laq):
    # the 32k shape stored [n, L, Hkv, d]: rows of a head lie 2 KiB apart
    n, Hq, Hkv, d, L, W = 2, 32, 8, 128, 32768, 32
    gen = torch.Generator(device=DEV).manual_seed(17)
    k_tm = torch.randn(n, L, Hkv, d, generator=gen, device=DEV).bfloat16()
    v_tm = torch.randn(n, L, Hkv, d, generator=gen, device=DEV).bfloat16()
    q = (torch.randn(n, Hq, W, d, generator=gen, device=DEV) * 1.5).bfloat16()
    run_and_check(laq, q, k_tm.permute(0, 2, 1, 3), v_tm.permute(0, 2, 1, 3), [1024, 256], 7, "token-major-32k",
                  heads=[6])


def test_decode_with_and_without_splitting_long_caches(laq):
    # 40 caches of up to 2300 rows in a small call: 150 parts, i.e. two launches of the part table;
    # both ways of summing must meet the oracle's bound, and a repeated call gives the same bits
    n, Hq, Hkv, d, L = 40, 8, 2, 128, 2300
    budgets = [300 + 50 * i for i in range(n)]
    g = torch.Generator().manual_seed(12)
    total, _ = laq.packed_rows(budgets, Hkv, L)
    q = (torch.randn(n, Hq, d, generator=g) * 1.5).bfloat16()
    kc = torch.randn(total, d, generator=g).bfloat16()
    vc = torch.randn(total, d, generator=g).bfloat16()
    need = laq.laq_decode_workspace_bytes(n, Hq, Hkv, d, L, torch.bfloat16, budgets)
    assert need > 0
    ws = torch.empty(need, dtype=torch.uint8, device=DEV)
    a = laq.laq_decode_attention(q.to(DEV), kc.to(DEV), vc.to(DEV), budgets, Hkv, L, ws=ws)
    a2 = laq.laq_decode_attention(q.to(DEV), kc.to(DEV), vc.to(DEV), budgets, Hkv, L, ws=ws)
    b = laq.laq_decode_attention(q.to(DEV), kc.to(DEV), vc.to(DEV), budgets, Hkv, L, split=False)
    torch.cuda.synchronize()
    assert torch.equal(a, a2)
    k_l, v_l = split_packed(kc, budgets, Hkv, L), split_packed(vc, budgets, Hkv, L)
    for i in (0, 4, 5, 17, 33, 34, 39):
        for got, how in ((a, "split"), (b, "one workgroup per cache")):
            check_decode(got[i].cpu(), q[i], k_l[i].contiguous(), v_l[i].contiguous(), torch.bfloat16,
                         "%s inst %d" % (how, i))
    # many workgroups already: no splitting, no workspace wanted
    assert laq.laq_decode_workspace_bytes(256, 32, 8, 128, 32768, torch.bfloat16, [2048] * 256) == 0


def test_two_lookahead_steps_full_size_sampled(laq):
    # a Q-cache of two lookahead steps (the paper's low-latency setting) with four query heads per KV
    # head: 8 score rows, a quarter of a 32-row tile, at the 32k shape
    n, Hq, Hkv, d, L, W = 2, 32, 8, 128, 32768, 2
    gen = torch.Generator(device=DEV).manual_seed(23)
    q = (torch.randn(n, Hq, W, d, generator=gen, device=DEV) * 1.5).bfloat16()
    k = torch.randn(n, Hkv, L, d, generator=gen, device=DEV).bfloat16()
    v = torch.randn(n, Hkv, L, d, generator=gen, device=DEV).bfloat16()
    run_general(laq, q, k, v, [512, 128], 7, [L, L + 1], 0, "two-steps-32k", heads=[2])


def _random_case(rng):
    d = int(rng.choice([64, 128, 128, 128, 96, 32]))
    Hkv = int(rng.choice([1, 2, 3]))
    G = int(rng.choice([1, 2, 4, 4, 5]))
    W = int(rng.choice([1, 2, 3, 8, 8, 16, 33]))
    L = int(rng.choice([rng.integers(1, 60), rng.integers(200, 300), rng.integers(500, 1100), rng.integers(1100, 2400)]))
    pool = int(rng.choice([1, 3, 7, 7, 15]))
    dtype = torch.float32 if (d == 32 or rng.random() < 0.15) else torch.bfloat16
    mode = rng.choice(["trailing", "lookahead", "joined", "scattered"])
    if mode == "trailing":
        W = min(W, L)
        pos, keep = [L - W + w for w in range(W)], W
    elif mode == "lookahead":
        pos, keep = [L + w for w in range(W)], int(rng.integers(0, min(L, 9)))
    elif mode == "joined":
        local = min(W // 2, L)
        pos, keep = [L - local + w for w in range(local)] + [L + w for w in range(W - local)], local
    else:
        pos, keep = [int(x) for x in rng.integers(0, 2 * L, size=W)], int(rng.integers(0, min(L, 5) + 1))
    budgets = [int(rng.integers(max(keep, 1), L + 20)), int(rng.integers(max(keep, 1), max(keep, 1) + 1 + L // 4))]
    return dict(d=d, Hkv=Hkv, Hq=Hkv * G, W=W, L=L, pool=pool, dtype=dtype, pos=pos, keep=keep, budgets=budgets,
                pool_mode="avg" if rng.random() < 0.2 else "max", strided=bool(rng.random() < 0.25))


@pytest.mark.parametrize("seed", range(24))
def test_random_shapes_against_the_oracle(laq, seed):
    c = _random_case(np.random.default_rng(1000 + seed))
    q, k, v = _qkv(seed, 2, c["Hq"], c["Hkv"], c["d"], c["L"], c["W"], c["dtype"])
    if c["strided"]:
        k, v = _token_major_view(k), _token_major_view(v)
    name = "random-%d d=%d G=%d mode=%s strided=%s dtype=%s" % (seed, c["d"], c["Hq"] // c["Hkv"], c["pool_mode"],
                                                               c["strided"], c["dtype"])
    run_general(laq, q, k, v, c["budgets"], c["pool"], c["pos"], c["keep"], name, pool_mode=c["pool_mode"])


def test_three_stage_flow_with_synthetic_queries(laq):
    """The calls in the order the method uses them (Sec. 4): stage-1 eviction to a low budget, eight
    lookahead steps that decode on the small cache and leave their queries in the Q-cache, the
    re-eviction of the full prefill cache with local window + Q-cache (Eq. 5), decoding on the
    result.  The model's layers are not here: the queries of every step are synthetic draws.  Each
    stage is checked against the oracle's version of the same step."""
    n, Hq, Hkv, d, L, W_local, steps = 2, 16, 4, 128, 3000, 8, 8
    g = torch.Generator().manual_seed(77)
    k = torch.randn(n, Hkv, L, d, generator=g).bfloat16()
    v = torch.randn(n, Hkv, L, d, generator=g).bfloat16()
    q_local = (torch.randn(n, Hq, W_local, d, generator=g) * 1.5).bfloat16()       # queries of the last prompt tokens
    kd, vd, qd = k.to(DEV), v.to(DEV), q_local.to(DEV)

    # stage 1: observation-window eviction with the prompt suffix as window, low budget
    low = [96, 64]
    _, idx1, k1, v1 = laq.laq_evict(qd, kd, vd, low, 7)
    # lookahead: eight decode steps on the small cache; their queries become the Q-cache
    q_cache = torch.zeros(n, Hq, steps, d, dtype=torch.bfloat16, device=DEV)
    ref_cache = torch.zeros(n, Hq, steps, d, dtype=torch.bfloat16)
    outs = []
    for t in range(steps):
        q_t = (torch.randn(n, Hq, d, generator=g) * 1.5).bfloat16()
        laq.laq_qcache_store(q_cache, q_t.to(DEV), t)
        outs.append((q_t, laq.laq_decode_attention(q_t.to(DEV), k1, v1, low, Hkv, L)))
        for i in range(n):
            ref_cache[i] = oracle.qcache_store(ref_cache[i], q_t[i], t)
    # re-eviction of the full cache: local window joined with the Q-cache, the local window's keys kept
    q_win = torch.cat([qd, q_cache], dim=2)
    pos = [L - W_local + w for w in range(W_local)] + [L + t for t in range(steps)]
    budgets = [256, 128]
    scores, idx2, k2, v2 = laq.laq_evict(q_win, kd, vd, budgets, 7, q_pos=pos, keep=W_local)
    q_next = (torch.randn(n, Hq, d, generator=g) * 1.5).bfloat16()
    out2 = laq.laq_decode_attention(q_next.to(DEV), k2, v2, budgets, Hkv, L)
    _, recall = laq.laq_recall(idx1, low, idx2, budgets, Hkv, L)
    torch.cuda.synchronize()

    assert torch.equal(q_cache.cpu(), ref_cache)
    k1_l, v1_l = split_packed(k1.cpu(), low, Hkv, L), split_packed(v1.cpu(), low, Hkv, L)
    k2_l, v2_l = split_packed(k2.cpu(), budgets, Hkv, L), split_packed(v2.cpu(), budgets, Hkv, L)
    idx1_l, idx2_l = split_packed(idx1.cpu(), low, Hkv, L), split_packed(idx2.cpu(), budgets, Hkv, L)
    q_win_c = torch.cat([q_local, ref_cache], dim=2)
    for i in range(n):
        o_pooled1, o_idx1, o_k1, o_v1 = oracle.evict(q_local[i], k[i], v[i], low[i], 7)
        o_pooled2, o_idx2, o_k2, o_v2 = oracle.evict(q_win_c[i], k[i], v[i], budgets[i], 7, q_pos=pos, keep=W_local)
        check_scores(scores[i].cpu(), o_pooled2, torch.bfloat16, "re-eviction inst %d" % i)
        for gh in range(Hkv):
            check_index_row(idx1_l[i][gh].numpy(), o_pooled1[gh].float().numpy(), W_local, low[i], RTOL[torch.bfloat16],
                            "stage-1 inst %d head %d" % (i, gh))
            check_index_row(idx2_l[i][gh].numpy(), o_pooled2[gh].float().numpy(), W_local, budgets[i],
                            RTOL[torch.bfloat16], "re-eviction inst %d head %d" % (i, gh))
        assert torch.equal(k1_l[i], oracle.compact(k[i], idx1_l[i])) and torch.equal(v2_l[i], oracle.compact(v[i], idx2_l[i]))
        for q_t, o_t in outs[::3]:
            check_decode(o_t[i].cpu(), q_t[i], k1_l[i].contiguous(), v1_l[i].contiguous(), torch.bfloat16,
                         "lookahead decode inst %d" % i)
        check_decode(out2[i].cpu(), q_next[i], k2_l[i].contiguous(), v2_l[i].contiguous(), torch.bfloat16,
                     "decode inst %d" % i)
        assert torch.equal(recall[i].cpu() * min(budgets[i], L),
                           oracle.overlap(idx1_l[i], idx2_l[i], L).float())
