"""CPU-only checks of the boundary: the library loads, exports what include/laq.h declares, and
rejects bad arguments synchronously (these calls return before anything touches a GPU)."""
import ctypes
import os
import re

import pytest
import torch

import paper_2505_20334_amd as laq
from paper_2505_20334_amd import binding


def declared_functions(repo_root):
    text = open(os.path.join(repo_root, "include", "laq.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(laq_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol(repo_root):
    lib = laq.load_library()
    names = declared_functions(repo_root)
    assert names == ["laq_compact", "laq_decode_attention", "laq_decode_workspace_bytes", "laq_evict", "laq_evict_static", "laq_init",
                     "laq_qcache_store", "laq_recall", "laq_score", "laq_score_kernel", "laq_select",
                     "laq_select_sink_recent", "laq_strerror", "laq_workspace_bytes", "laq_workspace_status"]
    for n in names:
        assert getattr(lib, n) is not None


def test_library_is_in_tree():
    assert os.path.dirname(laq.lib_path()) == os.path.dirname(os.path.abspath(laq.__file__))


def test_strerror():
    assert laq.laq_strerror(0) == "ok"
    assert "invalid" in laq.laq_strerror(-1)
    assert "workspace" in laq.laq_strerror(-3)
    assert "gave up" in laq.laq_strerror(-5)
    assert "unknown" in laq.laq_strerror(-99)


def test_workspace_bytes_grows_with_shape():
    a = laq.laq_workspace_bytes(1, 32, 8, 128, 4096, 8, torch.bfloat16)
    b = laq.laq_workspace_bytes(2, 32, 8, 128, 4096, 8, torch.bfloat16)
    c = laq.laq_workspace_bytes(1, 32, 8, 128, 8192, 8, torch.bfloat16)
    assert 0 < a < b and a < c
    assert laq.laq_workspace_bytes(1, 32, 7, 128, 4096, 8, torch.bfloat16) == 0      # Hq % Hkv != 0
    assert laq.laq_workspace_bytes(1, 32, 8, 128, 4, 8, torch.bfloat16) == 0          # W > L


def _shape(**kw):
    base = dict(n_inst=1, Hq=8, Hkv=2, d=128, L=512, W=8, dtype=1, scale=0.0, q_pos=None, keep=-1, pool_mode=0,
                kv_stride_inst=0, kv_stride_head=0, kv_stride_row=0, block_table=None, block_rows=0, kv_stride_block=0, score_choice=0)
    base.update(kw)
    return binding._Shape(*[base[f] for f, _ in binding._Shape._fields_])


def _positions(values):
    arr = (ctypes.c_int32 * len(values))(*values)
    return ctypes.cast(arr, ctypes.POINTER(ctypes.c_int32)), arr


def test_bad_arguments_are_rejected_without_a_gpu():
    lib = laq.load_library()
    fake = ctypes.c_void_p(0x1000)        # never dereferenced: validation fails first
    bud = (ctypes.c_int32 * 1)(64)
    sh = _shape()
    INVALID, WORKSPACE = -1, -3
    assert lib.laq_score(ctypes.byref(sh), None, fake, 7, fake, fake, 1 << 30, None) == INVALID
    assert lib.laq_score(ctypes.byref(sh), fake, fake, 4, fake, fake, 1 << 30, None) == INVALID     # even pool
    assert lib.laq_score(ctypes.byref(sh), fake, fake, 65, fake, fake, 1 << 30, None) == INVALID    # pool too wide
    assert lib.laq_score(ctypes.byref(sh), fake, fake, 7, fake, fake, 16, None) == WORKSPACE
    assert lib.laq_score(ctypes.byref(sh), fake, fake, 7, fake, None, 1 << 30, None) == WORKSPACE
    for bad in (_shape(W=0), _shape(W=600), _shape(Hq=7), _shape(d=12), _shape(d=512), _shape(dtype=5),
                _shape(n_inst=0), _shape(scale=float("nan"))):
        assert lib.laq_score(ctypes.byref(bad), fake, fake, 7, fake, fake, 1 << 30, None) == INVALID
    small = (ctypes.c_int32 * 1)(7)       # budget < W
    assert lib.laq_select(ctypes.byref(sh), fake, small, 7, fake, None) == INVALID
    assert lib.laq_select(ctypes.byref(sh), fake, None, 7, fake, None) == INVALID
    assert lib.laq_select(ctypes.byref(sh), fake, bud, 2, fake, None) == INVALID
    assert lib.laq_compact(ctypes.byref(sh), fake, fake, fake, bud, fake, None, None) == INVALID   # v without v_out
    assert lib.laq_compact(ctypes.byref(sh), fake, None, fake, small, fake, None, None) == INVALID
    assert lib.laq_evict(ctypes.byref(sh), fake, fake, fake, small, 7, fake, fake, fake, fake, fake, 1 << 30,
                         None) == INVALID
    assert lib.laq_evict(ctypes.byref(sh), fake, fake, fake, bud, 7, fake, fake, fake, fake, fake, 8,
                         None) == WORKSPACE
    # the scores buffer of the whole-path call is optional (accepted up to the workspace check), idx is not
    assert lib.laq_evict(ctypes.byref(sh), fake, fake, fake, bud, 7, None, fake, fake, fake, fake, 8,
                         None) == WORKSPACE
    assert lib.laq_evict(ctypes.byref(sh), fake, fake, fake, bud, 7, None, None, fake, fake, fake, 1 << 30,
                         None) == INVALID
    # the variant on the library's own scratch array: same argument checks, and a shape beyond the array is refused
    assert lib.laq_evict_static(ctypes.byref(sh), fake, fake, fake, small, 7, fake, fake, fake, fake, None) == INVALID
    assert lib.laq_evict_static(ctypes.byref(sh), fake, fake, fake, bud, 7, fake, None, fake, fake, None) == INVALID
    big = _shape(n_inst=32, Hq=32, Hkv=8, L=32768, W=32)
    assert laq.laq_workspace_bytes(32, 32, 8, 128, 32768, 32, torch.bfloat16) > (16 << 20)
    assert lib.laq_evict_static(ctypes.byref(big), fake, fake, fake, (ctypes.c_int32 * 32)(*([64] * 32)), 7, fake, fake,
                                fake, fake, None) == WORKSPACE
    assert lib.laq_workspace_status(ctypes.byref(sh), None, 1 << 30, None) == WORKSPACE
    assert lib.laq_workspace_status(ctypes.byref(sh), fake, 8, None) == WORKSPACE
    assert lib.laq_workspace_status(ctypes.byref(_shape(W=0)), fake, 1 << 30, None) == INVALID


def test_general_window_arguments_are_checked_without_a_gpu():
    lib = laq.load_library()
    fake = ctypes.c_void_p(0x1000)
    INVALID, UNSUPPORTED, WORKSPACE = -1, -2, -3
    bud = (ctypes.c_int32 * 1)(64)
    # explicit positions: any W >= 1, entries >= 0, at most 512 of them
    p_ok, keep1 = _positions([511, 600, 0, 3, 3, 3, 3, 3])
    ok = _shape(q_pos=p_ok, keep=0)
    assert lib.laq_score(ctypes.byref(ok), fake, fake, 7, fake, fake, 16, None) == WORKSPACE      # accepted up to here
    p_neg, keep2 = _positions([5, -1, 0, 3, 3, 3, 3, 3])
    assert lib.laq_score(ctypes.byref(_shape(q_pos=p_neg, keep=0)), fake, fake, 7, fake, fake, 1 << 30,
                         None) == INVALID
    p_many, keep3 = _positions([1] * 600)
    assert lib.laq_score(ctypes.byref(_shape(W=600, q_pos=p_many, keep=8)), fake, fake, 7, fake, fake, 1 << 30,
                         None) == UNSUPPORTED
    assert lib.laq_score(ctypes.byref(_shape(W=600, q_pos=p_many, keep=-1)), fake, fake, 7, fake, fake, 1 << 30,
                         None) == INVALID                                                       # keep defaults to W > L
    assert lib.laq_score(ctypes.byref(_shape(keep=513)), fake, fake, 7, fake, fake, 1 << 30, None) == INVALID
    # budgets are checked against keep (every call below is rejected before anything is launched)
    assert lib.laq_select(ctypes.byref(_shape(keep=100)), fake, bud, 7, fake, None) == INVALID    # 64 < keep
    assert lib.laq_select(ctypes.byref(_shape(keep=0)), fake, (ctypes.c_int32 * 1)(0), 7, fake, None) == INVALID
    assert laq.laq_workspace_bytes(1, 8, 2, 128, 512, 600, torch.bfloat16) == 0
    assert laq.laq_workspace_bytes(1, 8, 2, 128, 512, 600, torch.bfloat16, q_pos=[1] * 600, keep=4) == 0   # > 512 positions
    assert laq.laq_workspace_bytes(1, 8, 2, 128, 512, 300, torch.bfloat16, q_pos=[1] * 300, keep=4) > 0


def test_stage_one_variants_are_checked_without_a_gpu():
    lib = laq.load_library()
    fake = ctypes.c_void_p(0x1000)
    INVALID, UNSUPPORTED, WORKSPACE = -1, -2, -3
    bud = (ctypes.c_int32 * 1)(64)
    # pool mode: 0 (max) and 1 (average) pass the shape check, anything else does not
    assert lib.laq_score(ctypes.byref(_shape(pool_mode=1)), fake, fake, 7, fake, fake, 16, None) == WORKSPACE
    assert lib.laq_score(ctypes.byref(_shape(pool_mode=2)), fake, fake, 7, fake, fake, 1 << 30, None) == INVALID
    assert lib.laq_select(ctypes.byref(_shape(pool_mode=-1)), fake, bud, 7, fake, None) == INVALID
    # sink + recent list: every call below is rejected before anything is launched
    assert lib.laq_select_sink_recent(0, 2, 512, bud, 4, fake, None) == INVALID
    assert lib.laq_select_sink_recent(1, 0, 512, bud, 4, fake, None) == INVALID
    assert lib.laq_select_sink_recent(1, 2, 0, bud, 4, fake, None) == INVALID
    assert lib.laq_select_sink_recent(1, 2, 512, bud, -1, fake, None) == INVALID
    assert lib.laq_select_sink_recent(1, 2, 512, None, 4, fake, None) == INVALID
    assert lib.laq_select_sink_recent(1, 2, 512, bud, 4, None, None) == INVALID
    assert lib.laq_select_sink_recent(1, 2, 512, (ctypes.c_int32 * 1)(0), 4, fake, None) == INVALID
    assert lib.laq_select_sink_recent(1, 70000, 512, bud, 4, fake, None) == UNSUPPORTED
    with pytest.raises(ValueError):
        binding._shape(1, 8, 2, 128, 512, 8, 1, 0.0, pool_mode="median")
    # recall of two lists: rejected before anything is launched
    assert lib.laq_recall(0, 2, 512, fake, bud, fake, bud, fake, None, None) == INVALID
    assert lib.laq_recall(1, 2, 512, None, bud, fake, bud, fake, None, None) == INVALID
    assert lib.laq_recall(1, 2, 512, fake, bud, fake, None, fake, None, None) == INVALID
    assert lib.laq_recall(1, 2, 512, fake, bud, fake, bud, None, None, None) == INVALID
    assert lib.laq_recall(1, 2, 512, fake, (ctypes.c_int32 * 1)(0), fake, bud, fake, None, None) == INVALID
    assert lib.laq_recall(1, 70000, 512, fake, bud, fake, bud, fake, None, None) == UNSUPPORTED


def test_decode_side_calls_are_checked_without_a_gpu():
    lib = laq.load_library()
    fake = ctypes.c_void_p(0x1000)
    INVALID = -1
    bud = (ctypes.c_int32 * 1)(64)
    sh = _shape(keep=0)
    assert lib.laq_decode_attention(ctypes.byref(sh), None, fake, fake, bud, fake, None, 0, None) == INVALID
    assert lib.laq_decode_attention(ctypes.byref(sh), fake, fake, None, bud, fake, None, 0, None) == INVALID
    assert lib.laq_decode_attention(ctypes.byref(sh), fake, fake, fake, None, fake, None, 0, None) == INVALID
    assert lib.laq_decode_attention(ctypes.byref(sh), fake, fake, fake, bud, None, None, 0, None) == INVALID
    assert lib.laq_decode_attention(ctypes.byref(sh), fake, fake, fake, (ctypes.c_int32 * 1)(0), fake, None, 0, None) == INVALID
    assert lib.laq_decode_attention(ctypes.byref(_shape(Hq=7)), fake, fake, fake, bud, fake, None, 0, None) == INVALID
    # a cache of more than 512 rows in a small call wants a workspace; one that is too small is refused
    long_bud = (ctypes.c_int32 * 1)(2048)
    big = _shape(keep=0, L=4096)
    need = lib.laq_decode_workspace_bytes(ctypes.byref(big), long_bud)
    assert need > 0 and lib.laq_decode_workspace_bytes(ctypes.byref(big), bud) == 0
    assert lib.laq_decode_attention(ctypes.byref(big), fake, fake, fake, long_bud, fake, fake, need - 1, None) == -3
    assert lib.laq_qcache_store(ctypes.byref(sh), None, 0, fake, None) == INVALID
    assert lib.laq_qcache_store(ctypes.byref(sh), fake, 0, None, None) == INVALID
    assert lib.laq_qcache_store(ctypes.byref(sh), fake, -1, fake, None) == INVALID
    assert lib.laq_qcache_store(ctypes.byref(sh), fake, 8, fake, None) == INVALID      # W = 8 slots: 0..7
    assert lib.laq_qcache_store(ctypes.byref(_shape(d=12)), fake, 0, fake, None) == INVALID


def test_key_value_strides_are_checked_without_a_gpu():
    lib = laq.load_library()
    fake = ctypes.c_void_p(0x1000)
    INVALID, WORKSPACE = -1, -3
    bud = (ctypes.c_int32 * 1)(64)
    token_major = _shape(kv_stride_inst=512 * 2 * 128, kv_stride_head=128, kv_stride_row=2 * 128)
    assert lib.laq_score(ctypes.byref(token_major), fake, fake, 7, fake, fake, 16, None) == WORKSPACE     # accepted
    for bad in (_shape(kv_stride_row=256),                                        # some strides zero, some not
                _shape(kv_stride_inst=131072, kv_stride_head=128, kv_stride_row=64),     # rows overlap (< d)
                _shape(kv_stride_inst=131072, kv_stride_head=100, kv_stride_row=256),    # not a 16-byte multiple
                _shape(kv_stride_inst=-1, kv_stride_head=128, kv_stride_row=256)):
        assert lib.laq_score(ctypes.byref(bad), fake, fake, 7, fake, fake, 1 << 30, None) == INVALID
        assert lib.laq_compact(ctypes.byref(bad), fake, None, fake, bud, fake, None, None) == INVALID
        assert lib.laq_evict(ctypes.byref(bad), fake, fake, fake, bud, 7, fake, fake, fake, fake, fake, 1 << 30,
                             None) == INVALID
    with pytest.raises(ValueError):
        binding._kv(torch.zeros(1, 2, 8, 16)[..., ::2], "k")                      # host tensor is refused first


def test_paged_cache_fields_are_checked_without_a_gpu():
    lib = laq.load_library()
    fake = ctypes.c_void_p(0x1000)
    INVALID, WORKSPACE = -1, -3
    bud = (ctypes.c_int32 * 1)(64)
    table = 0x2000                       # never read: every call below returns before a launch
    good = _shape(block_table=table, block_rows=256, kv_stride_block=2 * 256 * 128)
    assert lib.laq_score(ctypes.byref(good), fake, fake, 7, fake, fake, 16, None) == WORKSPACE             # accepted
    token_major_blocks = _shape(block_table=table, block_rows=512, kv_stride_block=2 * 512 * 128, kv_stride_head=128,
                                kv_stride_row=2 * 128)
    assert lib.laq_score(ctypes.byref(token_major_blocks), fake, fake, 7, fake, fake, 16, None) == WORKSPACE
    for bad in (_shape(block_table=table, block_rows=128, kv_stride_block=2 * 128 * 128),      # not a multiple of 256 rows
                _shape(block_table=table, block_rows=300, kv_stride_block=2 * 300 * 128),
                _shape(block_table=table, block_rows=256, kv_stride_block=0),                  # blocks on top of each other
                _shape(block_table=table, block_rows=256, kv_stride_block=65540 + 1),          # not a 16-byte multiple
                _shape(block_table=table, block_rows=256, kv_stride_block=65536, kv_stride_row=256),   # half an inner layout
                _shape(block_rows=256), _shape(kv_stride_block=65536)):                        # block fields without a table
        assert lib.laq_score(ctypes.byref(bad), fake, fake, 7, fake, fake, 1 << 30, None) == INVALID
        assert lib.laq_compact(ctypes.byref(bad), fake, None, fake, bud, fake, None, None) == INVALID
        assert lib.laq_evict(ctypes.byref(bad), fake, fake, fake, bud, 7, fake, fake, fake, fake, fake, 1 << 30,
                             None) == INVALID


def test_packed_rows():
    total, starts = laq.packed_rows([2048, 128, 40000], 8, 32768)
    assert starts == [0, 8 * 2048, 8 * (2048 + 128)]
    assert total == 8 * (2048 + 128 + 32768)


def test_binding_checks_caller_supplied_outputs():
    like = torch.zeros(4, dtype=torch.bfloat16)
    binding._out(None, "x", torch.float32, 10, like)
    binding._out(torch.zeros(16), "x", torch.float32, 16, like)
    with pytest.raises(TypeError):
        binding._out(torch.zeros(16, dtype=torch.float64), "x", torch.float32, 16, like)
    with pytest.raises(ValueError):
        binding._out(torch.zeros(15), "x", torch.float32, 16, like)             # too small
    with pytest.raises(ValueError):
        binding._out(torch.zeros(8, 8)[:, ::2], "x", torch.float32, 16, like)   # not dense
    with pytest.raises(ValueError):
        binding._out(torch.zeros(20)[1:17], "x", torch.float32, 16, like)       # not 16-byte aligned
    with pytest.raises(ValueError):
        binding._out(torch.zeros(16, device="meta"), "x", torch.float32, 16, like)    # another device


def test_binding_refuses_host_tensors():
    q = torch.zeros(1, 8, 8, 128, dtype=torch.bfloat16)
    k = torch.zeros(1, 2, 512, 128, dtype=torch.bfloat16)
    with pytest.raises(ValueError):
        laq.laq_score(q, k, 7)


def test_bench_refuses_more_than_one_gpu(repo_root):
    import subprocess
    import sys
    res = subprocess.run([sys.executable, os.path.join(repo_root, "bench.py"), "--gpus", "2"], capture_output=True,
                         text=True, timeout=120)
    assert res.returncode == 2
    assert "single-GPU" in res.stderr and res.stdout.strip() == ""
