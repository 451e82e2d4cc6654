"""HIP path vs CPU oracle at the launch shapes only the large workloads take (needs an MI355X).

The kernels pick different instantiations by the size of a call: the selection kernel built for
two workgroups per compute unit from 768 (instance, KV head) pairs on, the one-workgroup-per-cache
decode kernel from 1024 workgroups on, the streaming kernels' claimed runs with thousands of units.
These cases reach them at their real sizes: oracle comparison on a spread of (instance, head)
pairs, and on every head the properties that hold at any size.
"""
import dataclasses

import numpy as np
import pytest
import torch

import oracle
from laq_inputs import CONFIGS, make_batch
from parity_util import RTOL, check_index_row, check_scores, split_packed

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


@pytest.fixture(scope="module")
def laq():
    import paper_2505_20334_amd as m
    m.load_library()
    assert torch.cuda.is_available()
    return m


def selection_properties(scores, idx_rows, keep, what):
    """scores [H, L] fp32 and idx_rows [H, Bk] int32 on the GPU, Bk < L: on every row the indices
    increase strictly, end with the `keep` trailing positions, every selected prefix score is >= every
    unselected one, and among the scores equal to the smallest selected one the lowest positions
    were taken."""
    H, L = scores.shape
    Bk = idx_rows.shape[1]
    P, ksel = L - keep, Bk - keep
    idx64 = idx_rows.long()
    assert (idx64[:, 1:] > idx64[:, :-1]).all(), what + ": not strictly increasing"
    assert (idx64[:, ksel:] == torch.arange(P, L, device=scores.device)).all(), what + ": window not retained"
    if ksel == 0:
        return
    assert (idx64[:, :ksel] < P).all() and (idx64 >= 0).all(), what
    pref = scores[:, :P]
    sel = torch.zeros(H, P, dtype=torch.bool, device=scores.device)
    sel.scatter_(1, idx64[:, :ksel], True)
    assert (sel.sum(1) == ksel).all(), what + ": repeated index"
    inf = torch.tensor(float("inf"), device=scores.device)
    t = torch.where(sel, pref, inf).min(1).values                     # smallest selected score
    best_out = torch.where(~sel, pref, -inf).max(1).values
    assert (t >= best_out).all(), what + ": an unselected score exceeds a selected one"
    eq = pref == t.unsqueeze(1)
    skipped_before = (eq & ~sel).cumsum(1) > 0                        # an equal score at a lower position was left out
    assert not (eq & sel & skipped_before).any(), what + ": ties not broken towards the lower position"


SELECT_MANY = [
    # name, n_inst, Hkv, L, W, budget, pool: n_inst * Hkv >= 768 in every case; the prefix lengths
    # fall into the kernel's four key-storage classes (2, 8, 32 keys per lane in registers; memory)
    ("two-keys-per-lane", 128, 8, 1500, 8, 200, 1),
    ("eight-keys-per-lane", 100, 8, 6000, 16, 512, 7),
    ("thirty-two-keys-per-lane", 96, 8, 20000, 16, 700, 1),
    ("batched-stress-shape", 96, 8, 32768, 16, 256, 1),
    ("batched-stress-shape-pooling-in-select", 96, 8, 32768, 16, 256, 7),
    ("keys-from-memory", 97, 8, 40000, 8, 3000, 1),
    ("more-than-one-instance-table", 300, 3, 2500, 4, 300, 5),
]


@pytest.mark.parametrize("name,n,Hkv,L,W,budget,pool", SELECT_MANY, ids=[c[0] for c in SELECT_MANY])
def test_select_with_many_heads_in_one_launch(laq, name, n, Hkv, L, W, budget, pool):
    assert n * Hkv >= 768
    print("case:", name, "n=%d Hkv=%d L=%d W=%d budget=%d pool=%d" % (n, Hkv, L, W, budget, pool), flush=True)
    gen = torch.Generator(device=DEV).manual_seed(L + n)
    # few distinct values on a third of the heads (ties across the boundary), continuous on the others,
    # exact plateaus as a max-pool leaves them on some
    s = torch.rand(n, Hkv, L, generator=gen, device=DEV)
    coarse = (torch.randint(0, 40, (n, Hkv, L), generator=gen, device=DEV).float() / 7)
    s[::3] = coarse[::3]
    s[1::3, :, : L // 2] = torch.repeat_interleave(s[1::3, :, : L // 2][..., ::7], 7, dim=-1)[..., : L // 2]
    budgets = [budget + (i % 3) for i in range(n)]
    idx = laq.laq_select(s, budgets, pool, W)
    again = laq.laq_select(s, budgets, pool, W)
    torch.cuda.synchronize()
    assert torch.equal(idx, again)
    parts = split_packed(idx, budgets, Hkv, L)
    if pool == 1:
        for b in range(3):                                            # instances of equal budget, all heads at once
            rows = torch.stack(parts[b::3]).reshape(-1, budget + b)
            selection_properties(s[b::3].reshape(-1, L), rows, W, "%s budget %d" % (name, budget + b))
    sample = sorted(set([0, 1, 2, n // 2, n - 2, n - 1] + list(range(5, n, max(1, n // 9)))))
    for i in sample:
        pooled = oracle.maxpool(s[i].cpu().double(), W, pool).float()
        assert torch.equal(parts[i].cpu(), oracle.select(pooled, W, budgets[i])), "%s inst %d" % (name, i)


def test_decode_one_workgroup_per_cache_with_many_workgroups(laq):
    # 300 instances x 4 KV heads = 1200 workgroups: the kernel that reads every cache whole, two
    # instance tables; caches from one row to more than the splitting length
    n, Hq, Hkv, d, L = 300, 16, 4, 128, 1200
    budgets = [1 + (37 * i) % 900 for i in range(n)]
    g = torch.Generator().manual_seed(31)
    total, _ = laq.packed_rows(budgets, Hkv, L)
    q = (torch.randn(n, Hq, d, generator=g) * 1.5).bfloat16()
    kc = torch.randn(total, d, generator=g).bfloat16()
    vc = torch.randn(total, d, generator=g).bfloat16()
    assert laq.laq_decode_workspace_bytes(n, Hq, Hkv, d, L, torch.bfloat16, budgets) == 0     # nothing is split
    out = laq.laq_decode_attention(q.to(DEV), kc.to(DEV), vc.to(DEV), budgets, Hkv, L)
    again = laq.laq_decode_attention(q.to(DEV), kc.to(DEV), vc.to(DEV), budgets, Hkv, L)
    torch.cuda.synchronize()
    assert torch.equal(out, again) and torch.isfinite(out).all()
    k_l, v_l = split_packed(kc, budgets, Hkv, L), split_packed(vc, budgets, Hkv, L)
    from test_gpu_parity import check_decode
    for i in sorted(set(list(range(0, n, 17)) + [254, 255, 256, 257, n - 1])):
        check_decode(out[i].cpu(), q[i], k_l[i].contiguous(), v_l[i].contiguous(), torch.bfloat16,
                     "inst %d (%d rows)" % (i, budgets[i]))


def full_config_case(laq, cfg, pairs, what, raw_rtol=2e-4):
    """The whole path at a config's full instance count: oracle comparison on `pairs` of (instance,
    KV head), size-independent properties on every instance and head."""
    q, k, v, budgets, _ = make_batch(cfg, device=DEV)
    n, Hkv, L, W, G = cfg.n_inst, cfg.Hkv, cfg.L, cfg.W, cfg.G
    print("case:", what, "n=%d Hkv=%d L=%d W=%d" % (n, Hkv, L, W), flush=True)
    scores, idx, ko, vo = laq.laq_evict(q, k, v, budgets, cfg.pool)
    raw = laq.laq_score(q, k, 1)
    torch.cuda.synchronize()
    # every probability row sums to one, pooling never lowers a score
    np.testing.assert_allclose(raw.double().sum(dim=2).cpu().numpy(), cfg.R, rtol=raw_rtol)
    assert torch.isfinite(scores).all() and (raw >= 0).all() and (scores >= raw).all()
    idx_l = split_packed(idx, budgets, Hkv, L)
    ko_l, vo_l = split_packed(ko, budgets, Hkv, L), split_packed(vo, budgets, Hkv, L)
    for i in range(n):
        selection_properties(scores[i], idx_l[i], W, "%s inst %d" % (what, i))
        rows = idx_l[i].long().unsqueeze(-1).expand(-1, -1, cfg.d)
        assert torch.equal(ko_l[i], torch.gather(k[i], 1, rows)), "%s: K' inst %d" % (what, i)
        assert torch.equal(vo_l[i], torch.gather(v[i], 1, rows)), "%s: V' inst %d" % (what, i)
    for (i, g) in pairs:
        print(what, "oracle pair", i, g, flush=True)
        qc, kc = q[i, g * G:(g + 1) * G].cpu(), k[i, g:g + 1].cpu()
        o_raw = oracle.raw_scores(qc, kc)
        pooled = oracle.maxpool(o_raw, W, cfg.pool)
        check_scores(raw[i, g].cpu(), o_raw[0], k.dtype, "%s raw inst %d head %d" % (what, i, g))
        check_scores(scores[i, g].cpu(), pooled[0], k.dtype, "%s inst %d head %d" % (what, i, g))
        got = idx_l[i][g].cpu()
        check_index_row(got.numpy(), pooled[0].float().numpy(), W, budgets[i], RTOL[k.dtype], what)
        assert torch.equal(oracle.select(scores[i, g:g + 1].cpu(), W, budgets[i])[0], got)
        assert torch.equal(ko_l[i][g].cpu(), oracle.compact(kc, got.unsqueeze(0))[0])


def test_config3_all_32_layers(laq):
    pairs = [(l, (3 * l + 1) % 8) for l in range(0, 32, 4)] + [(31, 7)]
    full_config_case(laq, CONFIGS[3], pairs, "cfg3-full")


def test_config4_one_head_of_every_layer(laq):
    pairs = [(l, (5 * l + 2) % 8) for l in range(32)]
    full_config_case(laq, CONFIGS[4], pairs, "cfg4-full")


def test_config5_all_256_instances(laq):
    # 8 sequences x 32 layers = 2048 heads, 16 GiB of keys: the batched launch shape itself
    pairs = [(0, 0), (1, 5), (31, 7), (32, 2), (77, 3), (100, 6), (128, 1), (160, 4), (200, 0), (223, 7),
             (254, 3), (255, 7)]
    full_config_case(laq, CONFIGS[5], pairs, "cfg5-full")
