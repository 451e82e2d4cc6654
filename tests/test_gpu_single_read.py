"""The single-read scoring kernel (a head's unnormalised probabilities stay in registers until the
softmax denominators are known) vs the CPU oracle (needs an MI355X).

laq_score takes that kernel for bf16 caches with d = 128 and at most 64 score rows per KV head
(R = G * W), by itself from 128 MiB of keys per call on and below that when the shape asks for it, as
the cases here do; a team of workgroups shares a head, 512 keys each with more than 32 score rows,
1024 otherwise.  The cases walk the team sizes (one workgroup, a ragged last workgroup, a key count
one past a boundary) for both, the row counts, heads fewer and more than the teams the device
holds, strided caches, explicit query positions, and check after every call that all the kernel's
waits completed (status of the workspace).
"""
import numpy as np
import pytest
import torch

import oracle
from parity_util import check_scores

pytestmark = pytest.mark.gpu

DEV = "cuda:0"
D = 128


@pytest.fixture(scope="module")
def laq():
    import paper_2505_20334_amd as m
    m.load_library()
    assert torch.cuda.is_available()
    return m


def draw(n, Hkv, G, L, W, seed, sinks=True):
    g = torch.Generator().manual_seed(seed)
    q = torch.randn(n, Hkv * G, W, D, generator=g)
    k = torch.randn(n, Hkv, L, D, generator=g)
    if sinks:
        # a few keys that every query likes (attention sinks), and one query row with a large norm
        k[:, :, :2] += 0.6 * q.reshape(n, Hkv, G * W, D).mean(2, keepdim=True)
        q[:, 0, 0] *= 4.0
    return q.bfloat16(), k.bfloat16()


def score_and_check(laq, q, k, pool, what, heads, k_dev=None, **kw):
    n, Hq, W, _ = q.shape
    _, Hkv, L, _ = k.shape
    G = Hq // Hkv
    print("case:", what, "n=%d Hkv=%d G=%d L=%d W=%d pool=%d" % (n, Hkv, G, L, W, pool), flush=True)
    qd = q.to(DEV)
    kd = k.to(DEV) if k_dev is None else k_dev
    strides = (0, 0, 0) if kd.is_contiguous() else (kd.stride(0), kd.stride(1), kd.stride(2))
    assert laq.laq_score_kernel(n, Hq, Hkv, D, L, W, torch.bfloat16, kw.get("q_pos"), kw.get("keep"),
                                strides, choose="single-read") == "single-read", what
    kw = dict(kw, choose="single-read")
    nb = laq.laq_workspace_bytes(n, Hq, Hkv, D, L, W, torch.bfloat16)
    ws = torch.zeros(nb, dtype=torch.uint8, device=DEV)
    s = laq.laq_score(qd, kd, pool, ws=ws, **kw)
    again = laq.laq_score(qd, kd, pool, ws=ws, **kw)
    torch.cuda.synchronize()
    assert laq.laq_workspace_status(ws, n, Hq, Hkv, D, L, W, torch.bfloat16) == 0, what + ": a wait was given up"
    assert torch.equal(s, again), what + ": two runs differ"
    assert torch.isfinite(s).all()
    sc = s.cpu()
    okw = {key: kw[key] for key in ("scale", "q_pos") if key in kw}
    keep = kw.get("keep", W)
    for (i, h) in heads:
        raw = oracle.raw_scores(q[i, h * G:(h + 1) * G], k[i, h:h + 1], **okw)
        want = oracle.maxpool(raw, keep, pool)
        check_scores(sc[i, h], want[0], torch.bfloat16, "%s inst %d head %d" % (what, i, h))
    return s


SHAPES = [
    # name, n, Hkv, G, L, W, pool
    ("one-workgroup", 3, 2, 4, 300, 8, 7),
    ("exactly-one-workgroup-32-rows", 2, 2, 4, 1024, 8, 1),
    ("exactly-one-workgroup-64-rows", 2, 2, 4, 512, 16, 1),
    ("one-key-past-a-boundary-32-rows", 2, 2, 4, 1025, 8, 7),
    ("one-key-past-a-boundary-64-rows", 2, 2, 4, 513, 16, 7),
    ("window-straddles-a-boundary-32-rows", 2, 2, 4, 2054, 8, 7),
    ("window-straddles-a-boundary-64-rows", 2, 2, 4, 1030, 16, 7),
    ("pool-window-straddles-boundaries", 2, 2, 4, 1540, 12, 15),
    ("ragged-team-of-ten", 2, 3, 4, 4700, 16, 7),
    ("rows-not-a-multiple-of-32", 2, 2, 4, 2100, 5, 5),
    ("48-rows", 2, 2, 4, 3000, 12, 3),
    ("64-rows-no-group", 2, 4, 1, 2500, 64, 7),
    ("group-of-eight", 2, 2, 8, 2049, 8, 7),
    ("one-query", 2, 2, 4, 1500, 1, 1),
    ("wide-pool", 2, 2, 4, 2600, 8, 31),
    # 65 ... 128 score rows: 256 keys per workgroup
    ("exactly-one-workgroup-128-rows", 2, 2, 4, 256, 32, 1),
    ("one-key-past-a-boundary-128-rows", 2, 2, 4, 257, 32, 7),
    ("window-straddles-a-boundary-128-rows", 2, 2, 4, 530, 32, 7),
    ("128-rows-team-of-eleven", 2, 3, 4, 2700, 32, 7),
    ("96-rows", 2, 2, 4, 1900, 24, 5),
    ("68-rows", 2, 2, 4, 1300, 17, 7),
    ("128-rows-group-of-eight", 2, 2, 8, 1111, 16, 3),
    ("128-rows-one-head-per-query", 1, 2, 1, 900, 128, 7),
]


@pytest.mark.parametrize("name,n,Hkv,G,L,W,pool", SHAPES, ids=[c[0] for c in SHAPES])
def test_shapes(laq, name, n, Hkv, G, L, W, pool):
    q, k = draw(n, Hkv, G, L, W, seed=L + W)
    score_and_check(laq, q, k, pool, name, [(0, 0), (n - 1, Hkv - 1)])


def test_more_heads_than_teams_and_fewer(laq):
    # L = 16384, 64 score rows: 32 workgroups per team, the device holds 16 teams; 40 heads take three
    # rounds with an unequal share, 3 heads leave most of the device idle
    for (n, Hkv) in ((5, 8), (1, 3)):
        q, k = draw(n, Hkv, 4, 16384, 16, seed=n * 100 + Hkv, sinks=False)
        score_and_check(laq, q, k, 7, "heads-%d" % (n * Hkv), [(0, 0), (n - 1, Hkv - 1), (n // 2, 1)])


def test_long_head_small_team_count(laq):
    # L = 70000: 137 workgroups per team with 64 score rows (3 teams on the device), 69 with 32 (7 teams)
    q, k = draw(1, 5, 4, 70000, 16, seed=7, sinks=False)
    score_and_check(laq, q, k, 7, "long-head-64-rows", [(0, 0), (0, 4)])
    q, k = draw(1, 9, 4, 70000, 8, seed=8, sinks=False)
    score_and_check(laq, q, k, 7, "long-head-32-rows", [(0, 0), (0, 8)])


def test_strided_and_token_major_caches(laq):
    n, Hkv, G, L, W = 2, 3, 4, 2300, 16
    q, k = draw(n, Hkv, G, L, W, seed=11)
    dense = score_and_check(laq, q, k, 7, "dense", [(0, 0), (1, 2)])
    # head-padded cache: every head is followed by 40 unused rows
    padded = torch.zeros(n, Hkv, L + 40, D, dtype=torch.bfloat16, device=DEV)
    padded[:, :, :L] = k.to(DEV)
    s_pad = score_and_check(laq, q, k, 7, "head-padded", [(1, 1)], k_dev=padded[:, :, :L])
    # token-major cache [n, L, Hkv, d] viewed as [n, Hkv, L, d]
    tm = k.to(DEV).permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3)
    assert not tm.is_contiguous()
    s_tm = score_and_check(laq, q, k, 7, "token-major", [(0, 2)], k_dev=tm)
    assert torch.equal(dense, s_pad) and torch.equal(dense, s_tm)


def test_explicit_query_positions_and_scale(laq):
    n, Hkv, G, L, W = 2, 2, 4, 1800, 8
    q, k = draw(n, Hkv, G, L, W, seed=5)
    # queries in the middle of the sequence: keys behind a query's position are invisible to it
    q_pos = [700, 701, 900, 1100, 1101, 1102, 1500, 1799]
    score_and_check(laq, q, k, 1, "positions", [(0, 0), (1, 1)], q_pos=q_pos, keep=0)
    score_and_check(laq, q, k, 7, "positions-pooled", [(0, 1)], q_pos=q_pos, keep=0)
    # a sharper softmax (large logits): the probabilities span hundreds of binary orders of magnitude
    score_and_check(laq, q, k, 1, "scale-1.5", [(0, 0), (1, 1)], scale=1.5)


def test_which_kernel(laq):
    bf, f32 = torch.bfloat16, torch.float32
    want = "single-read"
    assert laq.laq_score_kernel(2, 32, 8, 128, 4096, 8, bf) == "two-pass"            # 16 MiB of keys: not worth it
    assert laq.laq_score_kernel(64, 32, 8, 128, 4096, 8, bf) == "single-read"        # 512 MiB
    assert laq.laq_score_kernel(16, 32, 8, 128, 4096, 16, bf) == "single-read"       # 128 MiB, 64 rows
    assert laq.laq_score_kernel(64, 32, 8, 128, 4096, 8, bf, choose="two-pass") == "two-pass"
    assert laq.laq_score_kernel(2, 32, 8, 128, 4096, 8, bf, choose=want) == "single-read"     # 32 rows
    assert laq.laq_score_kernel(2, 32, 8, 128, 4096, 16, bf, choose=want) == "single-read"    # 64 rows
    assert laq.laq_score_kernel(2, 32, 8, 128, 4096, 17, bf, choose=want) == "single-read"    # 68 rows
    assert laq.laq_score_kernel(64, 32, 8, 128, 32768, 32, bf, choose=want) == "single-read"  # 128 rows
    assert laq.laq_score_kernel(64, 32, 8, 128, 32768, 32, bf) == "two-pass"                  # ... but not by itself
    assert laq.laq_score_kernel(2, 32, 8, 128, 4096, 33, bf, choose=want) == "two-pass"       # 132 rows
    assert laq.laq_score_kernel(2, 32, 8, 64, 4096, 8, bf, choose=want) == "two-pass"         # d = 64
    assert laq.laq_score_kernel(2, 32, 8, 128, 4096, 8, f32, choose=want) == "vector"
    assert laq.laq_score_kernel(1, 4, 1, 128, 600000, 8, bf, choose=want) == "two-pass"       # a team longer than the device holds
    with pytest.raises(laq.LaqError):
        laq.laq_score_kernel(2, 32, 8, 128, 4096, 0, bf)


def test_status_is_defined_after_every_kind_of_call(laq):
    # a workspace full of ones: whichever kernels score, the call leaves "all waits completed" behind
    for (W, d, dt, kind) in ((8, 128, torch.bfloat16, "single-read"), (32, 128, torch.bfloat16, "two-pass"),
                             (8, 128, torch.bfloat16, "two-pass"), (8, 64, torch.float32, "vector")):
        n, Hq, Hkv, L = 1, 8, 2, 1200
        assert laq.laq_score_kernel(n, Hq, Hkv, d, L, W, dt, choose=kind if kind != "vector" else "auto") == kind
        g = torch.Generator().manual_seed(W)
        q = torch.randn(n, Hq, W, d, generator=g).to(dt).to(DEV)
        k = torch.randn(n, Hkv, L, d, generator=g).to(dt).to(DEV)
        ws = torch.full((laq.laq_workspace_bytes(n, Hq, Hkv, d, L, W, dt),), 0xFF, dtype=torch.uint8, device=DEV)
        laq.laq_score(q, k, 7, ws=ws, choose=kind if kind != "vector" else "auto")
        assert laq.laq_workspace_status(ws, n, Hq, Hkv, d, L, W, dt) == 0, kind


def test_both_kernels_on_the_same_call(laq):
    # the two designs sum in different orders: equal to within fp32 rounding, not bit for bit
    n, Hkv, G, L, W = 3, 4, 4, 6000, 16
    q, k = draw(n, Hkv, G, L, W, seed=21)
    a = laq.laq_score(q.to(DEV), k.to(DEV), 7, choose="single-read")
    b = laq.laq_score(q.to(DEV), k.to(DEV), 7, choose="two-pass")
    torch.cuda.synchronize()
    np.testing.assert_allclose(a.cpu().numpy(), b.cpu().numpy(), rtol=2e-5, atol=1e-30)
    # and the whole path agrees wherever the ranking is not decided inside that rounding
    budgets = [300, 301, 302]
    ia = laq.laq_evict(q.to(DEV), k.to(DEV), None, budgets, 7, choose="single-read")[1]
    ib = laq.laq_evict(q.to(DEV), k.to(DEV), None, budgets, 7, choose="two-pass")[1]
    assert (ia != ib).float().mean().item() < 0.01


def test_constant_keys_give_uniform_probabilities(laq):
    # all keys equal: every visible key gets probability 1 / (number visible), whatever the team split
    n, Hkv, G, L, W = 1, 2, 4, 1300, 8
    g = torch.Generator().manual_seed(3)
    q = torch.randn(n, Hkv * G, W, D, generator=g).bfloat16()
    k = torch.randn(1, 1, 1, D, generator=g).expand(n, Hkv, L, D).contiguous().bfloat16()
    s = laq.laq_score(q.to(DEV), k.to(DEV), 1, choose="single-read").cpu().double()
    P = L - W
    want = torch.zeros(L, dtype=torch.float64)
    for w in range(W):
        want[: P + w + 1] += G / (P + w + 1)
    np.testing.assert_allclose(s[0, 0].numpy(), want.numpy(), rtol=2e-6)
    np.testing.assert_allclose(s[0, 1].numpy(), want.numpy(), rtol=2e-6)


def test_ordinary_launch_gives_the_same_bits(laq, tmp_path):
    # LAQ_COOPERATIVE_LAUNCH=0 (read once per process, so a child process): the same kernel on the same
    # grid, started without the cooperative guarantee, for profilers that cannot follow cooperative launches
    import os
    import subprocess
    import sys
    n, Hkv, G, L, W = 2, 3, 4, 5000, 16
    q, k = draw(n, Hkv, G, L, W, seed=77)
    want = laq.laq_score(q.to(DEV), k.to(DEV), 7, choose="single-read").cpu()
    torch.save({"q": q, "k": k}, tmp_path / "in.pt")
    code = (
        "import sys, torch\n"
        "sys.path.insert(0, %r)\n"
        "import paper_2505_20334_amd as laq\n"
        "d = torch.load(%r, weights_only=True)\n"
        "s = laq.laq_score(d['q'].to('cuda:0'), d['k'].to('cuda:0'), 7, choose='single-read')\n"
        "torch.cuda.synchronize()\n"
        "torch.save(s.cpu(), %r)\n"
    ) % (os.path.dirname(os.path.dirname(os.path.abspath(__file__))), str(tmp_path / "in.pt"), str(tmp_path / "out.pt"))
    env = dict(os.environ, LAQ_COOPERATIVE_LAUNCH="0")
    res = subprocess.run([sys.executable, "-c", code], env=env, capture_output=True, text=True, timeout=110)
    assert res.returncode == 0, res.stderr[-2000:]
    got = torch.load(tmp_path / "out.pt", weights_only=True)
    assert torch.equal(got, want)
