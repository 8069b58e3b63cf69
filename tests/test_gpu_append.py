"""GPU parity of kv_append (through the C ABI) against the oracle: bit-exact pool images."""
import numpy as np
import pytest

from paper_2602_07878_amd import workloads as W
from helpers import run_hip, to_device

pytestmark = pytest.mark.gpu


def new_rows(w, seed):
    rng = np.random.default_rng(seed)
    k = rng.standard_normal((w.B, w.Hkv, w.D)).astype(np.float32)
    v = rng.standard_normal((w.B, w.Hkv, w.D)).astype(np.float32)
    if w.dtype == "bf16":
        return W.f32_to_bf16_bits(k), W.f32_to_bf16_bits(v)
    return k, v


def to_torch(a, w):
    import torch
    if w.dtype == "bf16":
        return torch.from_numpy(a.view(np.int16)).cuda().view(torch.bfloat16)
    return torch.from_numpy(a).cuda()


def to_bits(t):
    import torch
    if t.dtype == torch.bfloat16:
        return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)
    return t.contiguous().cpu().numpy().view(np.uint32)


def bits(a):
    return a if a.dtype == np.uint16 else a.view(np.uint32)


def append_both(w, seed, token_major=False):
    """Append on the GPU and in the oracle; returns (gpu K bits, gpu V bits, oracle pools, device dict)."""
    import oracle
    import torch
    from paper_2602_07878_amd import binding
    kn, vn = new_rows(w, seed)
    dev = to_device(w)
    kp, vp = dev["k_pool"], dev["v_pool"]
    if token_major:   # same values stored [blocks][bs][Hkv][D], seen through strides
        kp = kp.permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3)
        vp = vp.permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3)
        dev["k_pool"], dev["v_pool"] = kp, vp
    desc = binding.attn_desc_for(dev["q"], kp, vp, dev["block_tables"], max_context_len=w.max_context_len)
    binding.kv_append(desc, to_torch(kn, w), to_torch(vn, w), kp, vp, dev["block_tables"], dev["context_lens"])
    torch.cuda.synchronize()
    oracle.kv_append(w.k_pool, w.v_pool, kn, vn, w.block_tables, w.context_lens, block_size=w.block_size)
    return to_bits(kp), to_bits(vp), dev


@pytest.mark.parametrize("mk", [W.config1_tiny,
                                lambda: W.config2_llama8b(B=16),
                                lambda: W.make_attn_workload("edge", 61, dtype="bf16", Hq=8, Hkv=2, D=64, block_size=32,
                                                             context_lens=[1, 32, 33, 0, 64, 17], pool_factor=1.5),
                                lambda: W.make_attn_workload("f32d128", 62, dtype="f32", Hq=8, Hkv=4, D=128, block_size=16,
                                                             context_lens=[16, 5, 0, 100], pool_factor=1.2)])
def test_append_image_is_bit_exact(mk):
    w = mk()
    gk, gv, _ = append_both(w, 7)
    # whole pools, bytewise: the new rows are in place and nothing else moved (NaN poison included)
    assert np.array_equal(gk, bits(w.k_pool)) and np.array_equal(gv, bits(w.v_pool))


def test_append_token_major_layout():
    w = W.make_attn_workload("tm", 63, dtype="bf16", Hq=16, Hkv=4, D=128, block_size=16,
                             context_lens=[300, 17, 1024, 16], pool_factor=1.1)
    gk, gv, _ = append_both(w, 8, token_major=True)
    assert np.array_equal(gk, bits(w.k_pool)) and np.array_equal(gv, bits(w.v_pool))


def test_append_then_attention_matches_oracle_on_the_appended_pools():
    import oracle
    w = W.config2_llama8b(B=8)
    gk, gv, dev = append_both(w, 9)
    ref = oracle.paged_decode_attention(w.q, w.k_pool, w.v_pool, w.block_tables, w.context_lens, w.scale,
                                        block_size=w.block_size)
    got = run_hip(w, dev)
    assert np.abs(got - ref).max() <= 2e-3


def test_append_empty_batch_is_a_no_op():
    import torch
    from paper_2602_07878_amd import binding
    w = W.config1_tiny()
    dev = to_device(w)
    desc = binding.attn_desc_for(dev["q"], dev["k_pool"], dev["v_pool"], dev["block_tables"], max_context_len=256)
    desc.batch = 0
    before = dev["k_pool"].clone()
    empty = torch.empty(0, w.Hkv, w.D, device="cuda")
    binding.kv_append(desc, empty, empty, dev["k_pool"], dev["v_pool"], dev["block_tables"], dev["context_lens"])
    torch.cuda.synchronize()
    assert torch.equal(before.view(torch.int32), dev["k_pool"].view(torch.int32))


# ---- the rows of a prefill chunk --------------------------------------------------------------
@pytest.mark.parametrize("lens,qlens,bs,token_major", [
    ((9, 4, 17, 6), (5, 4, 0, 9), 16, False),            # a tail, a whole prompt, nothing, more than the context
    ((700, 33, 1200, 16, 90), (128, 1, 1200, 16, 0), 16, False),
    ((300, 65), (300, 7), 64, True),
])
def test_chunk_rows_land_at_the_tail_positions_bit_exactly(lens, qlens, bs, token_major):
    import oracle
    import torch
    from paper_2602_07878_amd import binding
    w = W.make_attn_workload("chunk", 95, dtype="bf16", Hq=8, Hkv=2, D=128, block_size=bs,
                             context_lens=list(lens), pool_factor=1.3)
    ql = np.asarray(qlens, np.int32)
    total = int(ql.sum())
    rng = np.random.default_rng(96)
    kn = rng.integers(0, 2**16, (total, w.Hkv, w.D)).astype(np.uint16)
    vn = rng.integers(0, 2**16, (total, w.Hkv, w.D)).astype(np.uint16)
    dev = to_device(w)
    kp, vp = dev["k_pool"], dev["v_pool"]
    if token_major:
        kp = kp.permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3)
        vp = vp.permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3)
    desc = binding.attn_desc_for(dev["q"], kp, vp, dev["block_tables"], max_context_len=w.max_context_len)
    cu = torch.from_numpy(np.concatenate([[0], np.cumsum(ql)]).astype(np.int32)).cuda()
    pad = 3                                                # more rows in the buffers than the packed total: ignored
    dk = torch.from_numpy(np.concatenate([kn, np.full((pad, w.Hkv, w.D), 0x7FC0, np.uint16)]).view(np.int16)).cuda().view(torch.bfloat16)
    dv = torch.from_numpy(np.concatenate([vn, np.full((pad, w.Hkv, w.D), 0x7FC0, np.uint16)]).view(np.int16)).cuda().view(torch.bfloat16)
    binding.kv_append_chunk(desc, dk, dv, kp, vp, dev["block_tables"], dev["context_lens"],
                            torch.from_numpy(ql).cuda(), cu)
    torch.cuda.synchronize()
    oracle.kv_append_chunk(w.k_pool, w.v_pool, kn, vn, w.block_tables, w.context_lens, ql, block_size=bs)
    assert np.array_equal(to_bits(kp), w.k_pool) and np.array_equal(to_bits(vp), w.v_pool)   # whole pool images
