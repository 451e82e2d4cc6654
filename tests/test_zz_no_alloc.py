"""The whole-path call that allocates nothing (laq_evict_static) against laq_evict (needs an MI355X)."""
import pytest
import torch

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


def test_evict_on_the_library_scratch_matches_evict_twice_in_a_row():
    import paper_2505_20334_amd as laq
    laq.load_library()
    assert torch.cuda.is_available()
    g = torch.Generator().manual_seed(123)
    # the second call is smaller than the first: whatever the first left in the shared array must not matter
    for (n, Hq, Hkv, d, L, W, pool, budgets) in [(3, 32, 8, 128, 6000, 16, 7, [512, 300, 128]),
                                                 (2, 8, 2, 128, 1300, 8, 7, [100, 64])]:
        print("case: n=%d Hq=%d Hkv=%d d=%d L=%d W=%d" % (n, Hq, Hkv, d, L, W), flush=True)
        q = (torch.randn(n, Hq, W, d, generator=g) * 1.5).bfloat16().to(DEV)
        k = torch.randn(n, Hkv, L, d, generator=g).bfloat16().to(DEV)
        v = torch.randn(n, Hkv, L, d, generator=g).bfloat16().to(DEV)
        assert laq.laq_workspace_bytes(n, Hq, Hkv, d, L, W, torch.bfloat16) <= (16 << 20)
        want = laq.laq_evict(q, k, v, budgets, pool)
        total, _ = laq.packed_rows(budgets, Hkv, L)
        scores = torch.full((n, Hkv, L), -1.0, dtype=torch.float32, device=DEV)
        idx = torch.full((total,), -1, dtype=torch.int32, device=DEV)
        ko = torch.zeros(total, d, dtype=torch.bfloat16, device=DEV)
        vo = torch.zeros(total, d, dtype=torch.bfloat16, device=DEV)
        torch.cuda.synchronize()
        before = torch.cuda.memory_stats()["allocation.all.allocated"]
        got = laq.laq_evict(q, k, v, budgets, pool, scores=scores, idx=idx, k_out=ko, v_out=vo, static_scratch=True)
        assert torch.cuda.memory_stats()["allocation.all.allocated"] == before      # torch was asked for nothing either
        torch.cuda.synchronize()
        for a, b in zip(got, want):
            assert torch.equal(a, b)
        # without a scores buffer the hand-over plane lies in the array too
        idx2 = torch.full((total,), -1, dtype=torch.int32, device=DEV)
        ko2, vo2 = torch.zeros_like(ko), torch.zeros_like(vo)
        laq.laq_evict(q, k, v, budgets, pool, idx=idx2, k_out=ko2, v_out=vo2, want_scores=False, static_scratch=True)
        torch.cuda.synchronize()
        assert torch.equal(idx2, want[1]) and torch.equal(ko2, want[2]) and torch.equal(vo2, want[3])
    # a shape whose workspace exceeds the array is refused, with nothing enqueued
    q = torch.zeros(32, 32, 32, 128, dtype=torch.bfloat16, device=DEV)
    k = torch.zeros(32, 8, 32768, 128, dtype=torch.bfloat16, device=DEV)
    with pytest.raises(laq.LaqError) as err:
        laq.laq_evict(q, k, None, [64] * 32, 7, static_scratch=True)
    assert err.value.code == -3
