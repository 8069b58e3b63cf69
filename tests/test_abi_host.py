"""Host-side checks of the C ABI that need no GPU: the library loads, exports
every symbol the header declares, and rejects bad arguments before any launch."""
import ctypes
import os
import re

import numpy as np
import pytest

from paper_2602_07878_amd import binding
from paper_2602_07878_amd.binding import AttnDesc, SwapDesc

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

ST = dict(OK=0, NULL=1, SHAPE=2, DTYPE=3, ALIGN=4, WORKSPACE=5, INDEX=6, HIP=7)


def header_functions():
    src = "".join(open(os.path.join(ROOT, "include", h)).read() for h in ("pkv.h", "pkv_bench.h"))
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(pkv_[a-z_]+|paged_decode_attention[a-z_]*|paged_prefill_attention[a-z_]*|kv_block_swap|kv_append[a-z_]*|kv_swap_[a-z_]+)\s*\(", src)))


def test_library_exports_every_declared_symbol():
    L = binding.lib()
    names = header_functions()
    assert "paged_decode_attention" in names and "kv_block_swap" in names
    assert sorted(names) == sorted(binding.EXPORTS)
    for n in names:
        assert getattr(L, n) is not None
    assert L.pkv_version() >= 100
    assert binding.status_string(0) == "PKV_OK"
    assert binding.status_string(6) == "PKV_ERR_INDEX"


def good_desc(**kw):
    d = AttnDesc()
    d.batch, d.num_q_heads, d.num_kv_heads, d.head_dim = 4, 32, 8, 128
    d.block_size, d.num_pool_blocks, d.max_blocks_per_seq = 16, 100, 64
    d.max_context_len, d.partition_tokens, d.kv_dtype, d.out_dtype = 1024, 0, 1, 0
    d.k_stride_block = d.v_stride_block = 8 * 16 * 128
    d.k_stride_head = d.v_stride_head = 16 * 128
    d.k_stride_token = d.v_stride_token = 128
    for k, v in kw.items():
        setattr(d, k, v)
    return d


def call_attn(d, q=0x1000, k=0x2000, v=0x3000, bt=0x4000, cl=0x5000, out=0x6000, ws=0x7000,
              ws_bytes=1 << 40, scale=0.1):
    # fake (never dereferenced) pointers: every case below must be rejected on the host
    return binding.lib().paged_decode_attention(ctypes.byref(d), q, k, v, bt, cl, scale, out, ws,
                                                ws_bytes, None)


@pytest.mark.parametrize("kw,expect", [
    (dict(kv_dtype=7), "DTYPE"), (dict(out_dtype=9), "DTYPE"),
    (dict(num_q_heads=30), "SHAPE"), (dict(head_dim=96), "SHAPE"), (dict(block_size=8), "SHAPE"),
    (dict(block_size=24), "SHAPE"), (dict(partition_tokens=100), "SHAPE"),
    (dict(partition_tokens=32), "SHAPE"), (dict(batch=-1), "SHAPE"), (dict(flags=2), "SHAPE"),
    (dict(max_context_len=16 * 64 + 1), "SHAPE"), (dict(k_stride_token=4), "ALIGN"),
    (dict(k_stride_token=64), "SHAPE"), (dict(v_stride_head=-128), "SHAPE"),
    (dict(num_pool_blocks=0), "SHAPE"),
])
def test_attention_rejects_bad_descriptor_on_host(kw, expect):
    assert call_attn(good_desc(**kw)) == ST[expect]


def test_attention_rejects_bad_pointers_and_workspace_on_host():
    d = good_desc()
    assert binding.lib().paged_decode_attention(None, 1, 1, 1, 1, 1, 0.1, 1, 1, 0, None) == ST["NULL"]
    assert call_attn(d, q=0) == ST["NULL"]
    assert call_attn(d, out=0) == ST["NULL"]
    assert call_attn(d, k=0x2008) == ST["ALIGN"]
    assert call_attn(d, bt=0x4002) == ST["ALIGN"]
    assert call_attn(d, scale=float("nan")) == ST["SHAPE"]
    need = binding.attn_workspace_bytes(d)
    assert need > 0
    assert call_attn(d, ws_bytes=need - 1) == ST["WORKSPACE"]
    assert call_attn(d, ws=0) == ST["WORKSPACE"]
    # batch 0 is a successful no-op even with null data pointers
    assert call_attn(good_desc(batch=0), q=0, k=0, v=0, bt=0, cl=0, out=0, ws=0) == ST["OK"]


def test_workspace_size_and_partition_defaults():
    d = good_desc()
    assert binding.lib().pkv_attn_partition_tokens(ctypes.byref(d)) == 512
    # bf16 / D=128 takes the stream kernel: a directory plus at least one partial slot per
    # (sequence, KV head) and per wavefront of the grid
    need = binding.attn_workspace_bytes(d)
    assert need >= (4 * 8 + 1) * 4 * (128 + 2) * 4
    assert binding.attn_workspace_bytes(good_desc(partition_tokens=64)) >= need
    assert binding.attn_workspace_bytes(good_desc(batch=64, max_blocks_per_seq=256,
                                                  max_context_len=4096)) < 64 << 20
    # fp32 takes the grid kernel: no workspace while every context fits one partition
    f32 = dict(kv_dtype=0, head_dim=64, k_stride_token=64, v_stride_token=64,
               k_stride_head=16 * 64, v_stride_head=16 * 64, k_stride_block=8 * 16 * 64,
               v_stride_block=8 * 16 * 64)
    assert binding.attn_workspace_bytes(good_desc(max_context_len=512, **f32)) == 0
    assert binding.attn_workspace_bytes(good_desc(max_context_len=513, **f32)) > 0
    assert binding.attn_workspace_bytes(good_desc(partition_tokens=1024, **f32)) == 0
    assert binding.attn_workspace_bytes(good_desc(head_dim=96)) == 0   # invalid -> 0
    assert binding.attn_workspace_bytes(good_desc(batch=0)) == 0


def swap_desc(**kw):
    d = binding.swap_desc(4, 32768, 100, 50)
    for k, v in kw.items():
        setattr(d, k, v)
    return d


def test_swap_rejects_bad_arguments_on_host():
    L = binding.lib()
    f = lambda d, s=0x1000, t=0x2000, m=0x3000, n=5: L.kv_block_swap(ctypes.byref(d), s, t, m, n, None)
    assert L.kv_block_swap(None, 1, 1, 1, 1, None) == ST["NULL"]
    assert f(swap_desc(num_planes=0)) == ST["SHAPE"]
    assert f(swap_desc(block_bytes=24)) == ST["ALIGN"]
    assert f(swap_desc(src_plane_stride_bytes=99 * 32768)) == ST["SHAPE"]
    assert f(swap_desc(dst_plane_stride_bytes=50 * 32768 + 8)) == ST["ALIGN"]
    assert f(swap_desc(), s=0) == ST["NULL"]
    assert f(swap_desc(), t=0x2004) == ST["ALIGN"]
    assert f(swap_desc(), n=-1) == ST["SHAPE"]
    assert f(swap_desc(), s=0, t=0, m=0, n=0) == ST["OK"]


def test_append_rejects_bad_arguments_on_host():
    L = binding.lib()
    f = lambda d, kn=0x1000, vn=0x2000, kp=0x3000, vp=0x4000, bt=0x5000, cl=0x6000: L.kv_append(
        ctypes.byref(d), kn, vn, kp, vp, bt, cl, None)
    assert L.kv_append(None, 1, 1, 1, 1, 1, 1, None) == ST["NULL"]
    assert f(good_desc(head_dim=96)) == ST["SHAPE"]
    assert f(good_desc(kv_dtype=7)) == ST["DTYPE"]
    assert f(good_desc(), kn=0) == ST["NULL"]
    assert f(good_desc(), vp=0x4008) == ST["ALIGN"]
    assert f(good_desc(), cl=0x6002) == ST["ALIGN"]
    assert f(good_desc(batch=0), kn=0, vn=0, kp=0, vp=0, bt=0, cl=0) == ST["OK"]


def test_prefill_workspace_size_and_host_side_rejections():
    L = binding.lib()
    # one 512-token chunk over 8192 tokens: 64 workgroups unsplit -> 4 ranges (256 CUs assumed
    # without a device); rows x heads x ranges x (D + 2) floats
    d = good_desc(batch=1, max_context_len=8192, max_blocks_per_seq=512, num_pool_blocks=1024)
    need = L.pkv_prefill_workspace_bytes(ctypes.byref(d), 512, 512)
    assert need == 512 * 32 * 4 * (128 + 2) * 4
    assert L.pkv_prefill_workspace_bytes(ctypes.byref(good_desc(batch=64)), 64 * 512, 512) == 0   # enough workgroups
    assert L.pkv_prefill_workspace_bytes(ctypes.byref(good_desc(batch=1, max_context_len=256)), 256, 256) == 0  # short walks
    assert L.pkv_prefill_workspace_bytes(ctypes.byref(d), 0, 512) == 0 and L.pkv_prefill_workspace_bytes(None, 512, 512) == 0
    assert L.pkv_prefill_workspace_bytes(ctypes.byref(good_desc(batch=1, kv_dtype=0)), 512, 512) == 0      # fp32: unsupported
    f = lambda ws, wsb, total=512, q=0x1000: L.paged_prefill_attention_ws(
        ctypes.byref(d), q, 0x2000, 0x3000, 0x4000, 0x5000, 0x6000, 0x7000, 512, total, 0.1, 0x8000, ws, wsb, None)
    # fake (never dereferenced) pointers: every case must be rejected before anything is enqueued
    assert f(0x9000, need - 16) == ST["WORKSPACE"]
    assert f(0x9008, need) == ST["ALIGN"]
    assert f(0x9000, need, total=-1) == ST["SHAPE"]
    assert f(0x9000, need, q=0) == ST["NULL"]
    # 8-bit pools: the call decodes the sequences' blocks into a bf16 copy at the head of the
    # workspace (K and V images of batch x ceil(max context / block) blocks, then their table)
    d8 = good_desc(batch=1, max_context_len=8192, max_blocks_per_seq=512, num_pool_blocks=1024, kv_dtype=2)
    copy = 2 * 512 * (8 * 16 * 128 * 2) + 512 * 4
    assert L.pkv_prefill_workspace_bytes(ctypes.byref(d8), 512, 512) == copy + need
    f8 = lambda ws, wsb: L.paged_prefill_attention_ws(
        ctypes.byref(d8), 0x1000, 0x2000, 0x3000, 0x4000, 0x5000, 0x6000, 0x7000, 512, 512, 0.1, 0x8000, ws, wsb, None)
    assert f8(None, 0) == ST["WORKSPACE"] and f8(0x9000, copy - 16) == ST["WORKSPACE"] and f8(0x9008, copy) == ST["ALIGN"]


def test_swap_host_leg_rejects_bad_arguments_on_host():
    L = binding.lib()
    for fn in (L.kv_swap_out_host, L.kv_swap_in_host):
        f = lambda d, a=0x1000, b=0x2000, m=0x3000, n=5, st=0x4000, sb=1 << 22: fn(
            ctypes.byref(d), a, b, m, n, st, sb, None)
        assert fn(None, 1, 1, 1, 1, 1, 1, None) == ST["NULL"]
        assert f(swap_desc(block_bytes=24)) == ST["ALIGN"]
        assert f(swap_desc(), st=0) == ST["NULL"]
        assert f(swap_desc(), a=0x1008) == ST["ALIGN"]
        assert f(swap_desc(), n=-1) == ST["SHAPE"]
        assert f(swap_desc(), n=0, a=0, b=0, m=0, st=0) == ST["OK"]
        assert f(swap_desc(), sb=4 * 32768 - 16) == ST["WORKSPACE"]       # not even one pair of every plane
        # no staging buffer at all: the kernel would touch the host memory itself, which must be
        # page-locked memory the device can see; an address that is not is refused, nothing runs
        assert f(swap_desc(), st=0, sb=0) == ST["HIP"]
    # the host side needs a slot per pair: 50 slots in the 100 -> 50 descriptor, 100 the other way round
    assert L.kv_swap_out_host(ctypes.byref(swap_desc()), 0x1000, 0x2000, 0x3000, 51, 0x4000, 1 << 22, None) == ST["SHAPE"]
    assert L.kv_swap_in_host(ctypes.byref(swap_desc()), 0x1000, 0x2000, 0x3000, 101, 0x4000, 1 << 22, None) == ST["SHAPE"]


def test_chunk_validator_on_host():
    L = binding.lib()
    L.pkv_validate_chunks_host.restype = ctypes.c_int32
    L.pkv_validate_chunks_host.argtypes = [ctypes.POINTER(AttnDesc), ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                                           ctypes.c_int32, ctypes.c_int64]
    d = good_desc(batch=3)
    def f(cl, ql, cu, maxq=512, total=None):
        a, b, c = (np.asarray(x, np.int32) for x in (cl, ql, cu))
        return L.pkv_validate_chunks_host(ctypes.byref(d), a.ctypes.data, b.ctypes.data, c.ctypes.data, maxq,
                                          int(c[-1]) if total is None else total)
    assert f([100, 7, 512], [100, 0, 512], [0, 100, 100, 612]) == ST["OK"]
    assert f([100, 7, 512], [100, 0, 512], [1, 101, 101, 613]) == ST["INDEX"]        # first row is not 0
    assert f([100, 7, 512], [100, 0, 512], [0, 100, 101, 613]) == ST["INDEX"]        # a row that belongs to nobody
    assert f([100, 7, 512], [100, 0, 512], [0, 100, 100, 612], total=611) == ST["INDEX"]   # more rows than the buffers hold
    assert f([100, 7, 512], [100, -1, 512], [0, 100, 99, 611]) == ST["INDEX"]
    assert f([100, 7, 512], [100, 0, 512], [0, 100, 100, 612], maxq=511) == ST["INDEX"]
    assert f([100, 7, 1025], [100, 0, 512], [0, 100, 100, 612]) == ST["INDEX"]       # context above max_context_len
    assert L.pkv_validate_chunks_host(ctypes.byref(d), None, None, None, 1, 1) == ST["NULL"]


def test_host_validators():
    L = binding.lib()
    d = good_desc(batch=2, max_blocks_per_seq=4, max_context_len=64)
    bt = np.array([[3, 99, -1, -1], [0, 1, 2, 7]], np.int32)
    cl = np.array([17, 64], np.int32)
    v = lambda: L.pkv_validate_tables_host(ctypes.byref(d), bt.ctypes.data, cl.ctypes.data)
    assert v() == ST["OK"]
    cl[0] = 33
    assert v() == ST["INDEX"]           # third block of row 0 is -1 but now needed
    cl[0] = 17
    bt[1, 3] = 100
    assert v() == ST["INDEX"]           # block id == num_pool_blocks
    bt[1, 3] = 7
    cl[1] = 65
    assert v() == ST["INDEX"]           # longer than max_context_len
    cl[1] = -1
    assert v() == ST["INDEX"]
    cl[1] = 0
    assert v() == ST["OK"]

    s = swap_desc()
    m = np.array([[0, 0], [99, 49], [5, 7], [5, 8]], np.int32)
    w = lambda: L.pkv_validate_mapping_host(ctypes.byref(s), m.ctypes.data, len(m))
    assert w() == ST["OK"]              # a source block may repeat
    m[3, 1] = 7
    assert w() == ST["INDEX"]           # destination named twice
    m[3, 1] = 50
    assert w() == ST["INDEX"]
    m[3] = (100, 9)
    assert w() == ST["INDEX"]
    m[3] = (-1, 9)
    assert w() == ST["INDEX"]


def test_binding_fails_loudly_without_library(monkeypatch):
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "LIB_PATH", "/nonexistent/libpkv.so")
    with pytest.raises(FileNotFoundError):
        binding.lib()
