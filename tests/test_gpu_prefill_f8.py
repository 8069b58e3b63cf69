"""GPU parity of paged_prefill_attention over 8-bit (OCP E4M3) K/V pools, through the C ABI,
against the fp64 oracle (one decode-oracle row per query token, the pools' codes decoded exactly).

The library decodes the sequences' blocks into a bf16 copy in the caller's workspace (exact) and
walks the copy with the bf16 kernel, so the tolerance is that kernel's: max abs error
2e-3 * max(1, v_scale)."""
import numpy as np
import pytest

from paper_2602_07878_amd import workloads as W
from helpers import to_device

pytestmark = pytest.mark.gpu

TOL = 2e-3


def mk(seed, lens, Hq=8, Hkv=2, bs=16, k_scale=1.0, v_scale=1.0):
    w = W.make_attn_workload("prefill_f8", seed, dtype="f8", Hq=Hq, Hkv=Hkv, D=128, block_size=bs,
                             context_lens=list(lens), pool_factor=1.2)
    w.k_scale, w.v_scale = k_scale, v_scale
    return w


def run(w, query_lens, seed=7, token_major=False, out_dtype=None, short_workspace=False):
    import oracle
    import torch
    from paper_2602_07878_amd import binding
    ql = np.asarray(query_lens, np.int32)
    total = int(ql.sum())
    rng = np.random.default_rng(seed)
    q = W.f32_to_bf16_bits(rng.standard_normal((total, w.Hq, w.D)).astype(np.float32))
    ref = oracle.paged_prefill_attention(q, w.k_pool, w.v_pool, w.block_tables, w.context_lens, ql, w.scale,
                                         block_size=w.block_size, k_scale=w.k_scale, v_scale=w.v_scale)
    dev = to_device(w)
    kp, vp = dev["k_pool"], dev["v_pool"]
    if token_major:
        kp = kp.permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3)
        vp = vp.permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3)
    dq = torch.from_numpy(q.view(np.int16)).cuda().view(torch.bfloat16)
    cu = torch.from_numpy(np.concatenate([[0], np.cumsum(ql)]).astype(np.int32)).cuda()
    odt = out_dtype or torch.float32
    pad = 256
    buf = torch.full((total * w.Hq * w.D + 2 * pad,), 777.0, dtype=odt, device="cuda")
    out = buf[pad:pad + total * w.Hq * w.D].view(total, w.Hq, w.D)
    desc = binding.attn_desc_for(dq, kp, vp, dev["block_tables"], max_context_len=w.max_context_len, out_dtype=odt,
                                 k_scale=w.k_scale, v_scale=w.v_scale)
    desc.batch = w.B
    need = binding.prefill_workspace_bytes(desc, total, int(ql.max()))
    assert need > 0
    if short_workspace:
        ws = torch.empty(need - 256, dtype=torch.uint8, device="cuda")
        with pytest.raises(binding.PkvError):
            binding.paged_prefill_attention(desc, dq, kp, vp, dev["block_tables"], dev["context_lens"],
                                            torch.from_numpy(ql).cuda(), cu, int(ql.max()), w.scale, out, workspace=ws)
        return None, None
    ws = torch.full((need + 64,), 0xFF, dtype=torch.uint8, device="cuda")    # NaN-filled, canary behind it
    binding.paged_prefill_attention(desc, dq, kp, vp, dev["block_tables"], dev["context_lens"],
                                    torch.from_numpy(ql).cuda(), cu, int(ql.max()), w.scale, out, workspace=ws)
    torch.cuda.synchronize()
    assert bool((ws[need:] == 0xFF).all()), "wrote past the workspace"
    assert torch.all(buf[:pad] == 777.0) and torch.all(buf[pad + total * w.Hq * w.D:] == 777.0)
    got = out.float().cpu().numpy().astype(np.float64)
    assert np.all(np.isfinite(got)), "non-finite output (poison leaked?)"
    absent = np.isnan(ref)
    assert np.all(got[absent] == 777.0)
    err = np.abs(got[~absent] - ref[~absent]).max()
    print(f"{w.name}: Hq={w.Hq} Hkv={w.Hkv} bs={w.block_size} ctx={list(w.context_lens)[:6]} q={list(query_lens)[:6]} "
          f"k_scale={w.k_scale} v_scale={w.v_scale} max_abs_err={err:.3e}", flush=True)
    assert err <= TOL * max(1.0, w.v_scale), err
    return got, ref


def test_whole_prompts_ragged_with_poisoned_pools():
    lens = (1, 15, 16, 17, 129, 700, 33)
    run(mk(601, lens), lens)


@pytest.mark.parametrize("Hq,Hkv", [(8, 2), (4, 4), (32, 8), (6, 2)])
def test_head_shapes_and_chunks_over_a_cached_prefix(Hq, Hkv):
    lens = (900, 260, 64, 2000)
    run(mk(602, lens, Hq=Hq, Hkv=Hkv), (130, 260, 5, 512))


def test_pool_scales_that_are_not_powers_of_two():
    lens = (300, 1000)
    run(mk(603, lens, k_scale=0.37, v_scale=2.9), (300, 77))


@pytest.mark.parametrize("bs", [16, 64, 128])
def test_block_sizes_and_token_major_pools(bs):
    lens = (bs + 3, 3 * bs, 500)
    run(mk(604, lens, bs=bs), (bs + 3, bs, 260), token_major=bs != 16)


def test_split_walks_absent_and_clipped_sequences():
    # one long context and a short chunk: the library cuts the walk into ranges; a sequence
    # without tokens, and one whose query length exceeds its context (clipped)
    lens = (4000, 0, 40)
    run(mk(605, lens), (100, 0, 64))


def test_bf16_output():
    import torch
    lens = (700, 130)
    w = mk(606, lens)
    import oracle  # noqa: F401  (the tolerance adds one bf16 ulp of the result)
    global TOL
    old, TOL = TOL, 2e-3 + 2 ** -8 * 4
    try:
        run(w, (200, 130), out_dtype=torch.bfloat16)
    finally:
        TOL = old


def test_a_short_workspace_is_refused():
    lens = (300, 100)
    run(mk(607, lens), (300, 100), short_workspace=True)


def test_chunk_of_8_bit_rows_appended_then_attended():
    """A step of chunked prefill on a quantised cache: the chunk's K/V codes join the pools
    (kv_append_chunk: bytes), then the chunk attends over prefix and itself; pools bit-identical
    to the oracle's, attention within tolerance."""
    import oracle
    import torch
    from paper_2602_07878_amd import binding
    lens, qlens = (600, 90, 1300), (100, 90, 512)
    w = mk(608, lens, Hq=16, Hkv=4, k_scale=0.8, v_scale=1.5)
    ql = np.asarray(qlens, np.int32)
    total = int(ql.sum())
    rng = np.random.default_rng(609)
    kn = W.f32_to_f8e4m3_bits(rng.standard_normal((total, w.Hkv, w.D)).astype(np.float32))
    vn = W.f32_to_f8e4m3_bits(rng.standard_normal((total, w.Hkv, w.D)).astype(np.float32))
    q = W.f32_to_bf16_bits(rng.standard_normal((total, w.Hq, w.D)).astype(np.float32))
    dev = to_device(w)
    dq = torch.from_numpy(q.view(np.int16)).cuda().view(torch.bfloat16)
    d_ql = torch.from_numpy(ql).cuda()
    cu = torch.from_numpy(np.concatenate([[0], np.cumsum(ql)]).astype(np.int32)).cuda()
    desc = binding.attn_desc_for(dq, dev["k_pool"], dev["v_pool"], dev["block_tables"], max_context_len=w.max_context_len,
                                 k_scale=w.k_scale, v_scale=w.v_scale)
    desc.batch = w.B
    binding.kv_append_chunk(desc, torch.from_numpy(kn).cuda(), torch.from_numpy(vn).cuda(), dev["k_pool"], dev["v_pool"],
                            dev["block_tables"], dev["context_lens"], d_ql, cu)
    out = torch.zeros(total, w.Hq, w.D, device="cuda")
    ws = torch.empty(binding.prefill_workspace_bytes(desc, total, int(ql.max())), dtype=torch.uint8, device="cuda")
    binding.paged_prefill_attention(desc, dq, dev["k_pool"], dev["v_pool"], dev["block_tables"], dev["context_lens"],
                                    d_ql, cu, int(ql.max()), w.scale, out, workspace=ws)
    torch.cuda.synchronize()
    oracle.kv_append_chunk(w.k_pool, w.v_pool, kn, vn, w.block_tables, w.context_lens, ql, block_size=w.block_size)
    assert np.array_equal(dev["k_pool"].cpu().numpy(), w.k_pool) and np.array_equal(dev["v_pool"].cpu().numpy(), w.v_pool)
    ref = oracle.paged_prefill_attention(q, w.k_pool, w.v_pool, w.block_tables, w.context_lens, ql, w.scale,
                                         block_size=w.block_size, k_scale=w.k_scale, v_scale=w.v_scale)
    got = out.cpu().numpy().astype(np.float64)
    assert np.all(np.isfinite(got)) and np.abs(got - ref).max() <= TOL * max(1.0, w.v_scale)
