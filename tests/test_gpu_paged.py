"""Paged K/V caches (a pool of blocks + a block table per instance) through the C ABI vs the CPU
oracle on the gathered dense cache (needs an MI355X).

The library reads paged caches in laq_score, laq_compact and laq_evict; the oracle side gathers the
cache into its dense form first (oracle.gather_paged, pinned on the CPU against an independent
scatter).  Cases: a permuted table, a ragged last block, blocks shared between instances, blocks of
several sizes, token-major blocks, fp32 (vector kernels) and bf16 (matrix cores: the two streaming
passes and the single-read kernel), and the dense call on the gathered cache as a bit-exact
cross-check of scores, indices and rows.
"""
import numpy as np
import pytest
import torch

import oracle
from parity_util import RTOL, check_index_row, check_scores, split_packed

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


@pytest.fixture(scope="module")
def laq():
    import paper_2505_20334_amd as m
    m.load_library()
    assert torch.cuda.is_available()
    return m


def make_paged(n, Hkv, L, d, block_rows, dtype, seed, share_first_block=False, spare=5):
    """A pool with more blocks than needed, filled through a permuted table; returns the pools, the
    table and the dense caches they spell out.  Rows of a last block beyond L hold NaN (they must
    never be read), unused blocks too."""
    g = torch.Generator().manual_seed(seed)
    per = -(-L // block_rows)
    n_blocks = n * per + spare
    table = torch.randperm(n_blocks, generator=g)[: n * per].reshape(n, per).int()
    if share_first_block and n > 1:
        table[1:, 0] = table[0, 0]
    kp = torch.full((n_blocks, Hkv, block_rows, d), float("nan"))
    vp = torch.full((n_blocks, Hkv, block_rows, d), float("nan"))
    for i in range(n):
        for b in range(per):
            rows = min(block_rows, L - b * block_rows)
            if share_first_block and b == 0 and i > 0:
                continue
            kp[table[i, b], :, :rows] = torch.randn(Hkv, rows, d, generator=g)
            vp[table[i, b], :, :rows] = torch.randn(Hkv, rows, d, generator=g)
    kp, vp = kp.to(dtype), vp.to(dtype)
    return kp, vp, table, oracle.gather_paged(kp, table, L), oracle.gather_paged(vp, table, L)


def run_paged(laq, n, Hkv, G, L, W, d, block_rows, dtype, pool, budgets, what, token_major=False, share=False,
              choose="auto"):
    print("case:", what, "n=%d Hkv=%d G=%d L=%d W=%d d=%d block=%d %s" % (n, Hkv, G, L, W, d, block_rows, choose),
          flush=True)
    kp, vp, table, k, v = make_paged(n, Hkv, L, d, block_rows, dtype, seed=L + W + n, share_first_block=share, spare=5)
    assert torch.isfinite(k.float()).all() and torch.isfinite(v.float()).all()
    g = torch.Generator().manual_seed(n)
    q = torch.randn(n, Hkv * G, W, d, generator=g).to(dtype)
    kpd, vpd, td = kp.to(DEV), vp.to(DEV), table.to(DEV)
    if token_major:                      # blocks stored [block_rows, Hkv, d], handed over as strided views
        kpd = kpd.permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3)
        vpd = vpd.permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3)
        assert not kpd.is_contiguous()
    scores, idx, ko, vo = laq.laq_evict(q.to(DEV), kpd, vpd, budgets, pool, block_table=td, L=L, choose=choose)
    s3 = laq.laq_score(q.to(DEV), kpd, pool, block_table=td, L=L, choose=choose)
    i3 = laq.laq_select(s3, budgets, 1, W)
    k3, v3 = laq.laq_compact(kpd, vpd, i3, budgets, W, block_table=td, L=L)
    torch.cuda.synchronize()
    assert torch.equal(s3, scores) and torch.equal(i3, idx) and torch.equal(k3, ko) and torch.equal(v3, vo)
    assert torch.isfinite(scores).all()
    idx_l = split_packed(idx.cpu(), budgets, Hkv, L)
    ko_l, vo_l = split_packed(ko.cpu(), budgets, Hkv, L), split_packed(vo.cpu(), budgets, Hkv, L)
    sc = scores.cpu()
    for i in range(n):
        rows = idx_l[i].long().unsqueeze(-1).expand(-1, -1, d)
        assert torch.equal(ko_l[i], torch.gather(k[i], 1, rows)), "%s: K' inst %d" % (what, i)
        assert torch.equal(vo_l[i], torch.gather(v[i], 1, rows)), "%s: V' inst %d" % (what, i)
        for h in sorted({0, Hkv - 1}):
            raw = oracle.raw_scores(q[i, h * G:(h + 1) * G], k[i, h:h + 1])
            pooled = oracle.maxpool(raw, W, pool)
            check_scores(sc[i, h], pooled[0], dtype, "%s inst %d head %d" % (what, i, h))
            check_index_row(idx_l[i][h].numpy(), pooled[0].float().numpy(), W, budgets[i], RTOL[dtype], what)
            assert torch.equal(oracle.select(sc[i, h:h + 1], W, budgets[i])[0], idx_l[i][h])
    return q, k, v, scores, idx, ko, vo


CASES = [
    # name, n, Hkv, G, L, W, d, block_rows, dtype, pool, token_major, share
    ("bf16-permuted-ragged", 3, 2, 4, 1300, 32, 128, 256, torch.bfloat16, 7, False, False),
    ("bf16-whole-blocks", 2, 2, 4, 1024, 32, 128, 256, torch.bfloat16, 7, False, False),
    ("bf16-big-blocks", 2, 3, 4, 2500, 32, 128, 1024, torch.bfloat16, 7, False, False),
    ("bf16-few-rows-single-read-shape", 2, 2, 4, 1500, 8, 128, 256, torch.bfloat16, 7, False, False),
    ("bf16-d64", 2, 2, 2, 900, 16, 64, 512, torch.bfloat16, 5, False, False),
    ("bf16-token-major-blocks", 2, 4, 2, 1100, 32, 128, 256, torch.bfloat16, 7, True, False),
    ("bf16-shared-prefix-block", 3, 2, 4, 700, 32, 128, 256, torch.bfloat16, 1, False, True),
    ("bf16-shorter-than-a-block", 2, 2, 4, 100, 8, 128, 256, torch.bfloat16, 3, False, False),
    ("f32-vector-kernels", 2, 2, 2, 800, 8, 64, 256, torch.float32, 7, False, False),
    ("f32-token-major-blocks", 2, 2, 2, 600, 4, 40, 256, torch.float32, 1, True, False),
]


@pytest.mark.parametrize("name,n,Hkv,G,L,W,d,block_rows,dtype,pool,tm,share", CASES, ids=[c[0] for c in CASES])
def test_paged_cache(laq, name, n, Hkv, G, L, W, d, block_rows, dtype, pool, tm, share):
    budgets = [min(L, 64 + 40 * i) for i in range(n)]
    run_paged(laq, n, Hkv, G, L, W, d, block_rows, dtype, pool, budgets, name, token_major=tm, share=share)


# the single-read kernel on paged caches: one and several workgroups per head (512 keys each at 64
# score rows, 1024 at 32 or fewer), tiles beyond the head's end, a ragged last block, more heads than
# teams of workgroups (a wave then asks for the next head's first tile through that head's table row)
SINGLE = [
    # name, n, Hkv, G, L, W, d, block_rows, pool, token_major, share
    ("one-workgroup", 2, 2, 4, 500, 8, 256, 7, False, False),
    ("ragged-last-block", 3, 2, 4, 1300, 16, 256, 7, False, False),
    ("32-rows-long-workgroups", 2, 2, 4, 3000, 8, 512, 7, False, False),
    ("64-rows-big-blocks", 2, 3, 4, 2500, 16, 1024, 5, False, False),
    ("token-major-blocks", 2, 4, 2, 1100, 32, 256, 7, True, False),
    ("shared-prefix-block", 3, 2, 4, 700, 8, 256, 1, False, True),
    ("shorter-than-a-block", 2, 2, 4, 100, 8, 256, 3, False, False),
    ("many-heads", 40, 8, 4, 4200, 8, 256, 7, False, False),
]


@pytest.mark.parametrize("name,n,Hkv,G,L,W,block_rows,pool,tm,share", SINGLE, ids=[c[0] for c in SINGLE])
def test_paged_cache_single_read(laq, name, n, Hkv, G, L, W, block_rows, pool, tm, share):
    budgets = [min(L, 64 + 3 * i) for i in range(n)]
    kind = laq.laq_score_kernel(n, Hkv * G, Hkv, 128, L, W, torch.bfloat16, choose="single-read",
                                paged=(torch.zeros(n, -(-L // block_rows), dtype=torch.int32, device=DEV), block_rows,
                                       Hkv * block_rows * 128))
    assert kind == "single-read"
    run_paged(laq, n, Hkv, G, L, W, 128, block_rows, torch.bfloat16, pool, budgets, "single-read-" + name,
              token_major=tm, share=share, choose="single-read")


def test_paged_single_read_gives_the_dense_single_read_bits(laq):
    n, Hkv, G, L, W = 3, 2, 4, 2900, 16
    budgets = [200, 333, 64]
    q, k, v, scores, idx, ko, vo = run_paged(laq, n, Hkv, G, L, W, 128, 512, torch.bfloat16, 7, budgets,
                                             "paged-vs-dense-single-read", choose="single-read")
    dense = laq.laq_evict(q.to(DEV), k.to(DEV), v.to(DEV), budgets, 7, choose="single-read")
    torch.cuda.synchronize()
    for a, b in zip(dense, (scores, idx, ko, vo)):
        assert torch.equal(a, b)


def test_paged_equals_dense_bit_for_bit_on_the_two_pass_kernels(laq):
    # 128 score rows: dense and paged both take the two streaming passes, in the same order of sums
    n, Hkv, G, L, W, d = 2, 2, 4, 1800, 32, 128
    budgets = [200, 333]
    q, k, v, scores, idx, ko, vo = run_paged(laq, n, Hkv, G, L, W, d, 512, torch.bfloat16, 7, budgets, "paged-vs-dense")
    dense = laq.laq_evict(q.to(DEV), k.to(DEV), v.to(DEV), budgets, 7)
    torch.cuda.synchronize()
    for a, b in zip(dense, (scores, idx, ko, vo)):
        assert torch.equal(a, b)


def test_paged_arguments_are_checked(laq):
    kp = torch.zeros(4, 2, 256, 128, dtype=torch.bfloat16, device=DEV)
    q = torch.zeros(1, 8, 8, 128, dtype=torch.bfloat16, device=DEV)
    table = torch.zeros(1, 2, dtype=torch.int32, device=DEV)
    with pytest.raises(ValueError):
        laq.laq_score(q, kp, 1, block_table=table)                                   # L missing
    with pytest.raises(ValueError):
        laq.laq_score(q, kp, 1, block_table=table, L=1000)                           # 4 blocks needed, table has 2
    with pytest.raises(ValueError):
        laq.laq_score(q, kp, 1, block_table=table.long(), L=500)                     # int64 table
    with pytest.raises(ValueError):
        laq.laq_score(q, kp[:, :, :128], 1, block_table=table, L=200)                # blocks of 128 rows
    assert laq.laq_score_kernel(1, 8, 2, 128, 500, 8, torch.bfloat16, paged=(table, 256, kp.stride(0)),
                                choose="single-read") == "single-read"
    assert laq.laq_score_kernel(1, 8, 2, 128, 500, 8, torch.bfloat16, paged=(table, 256, kp.stride(0))) == "two-pass"
    s = laq.laq_score(q, kp, 1, block_table=table, L=500)
    np.testing.assert_allclose(s.sum(dim=2).cpu().numpy(), 4 * 8, rtol=1e-5)         # zero keys: uniform rows
