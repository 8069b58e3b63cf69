"""GPU parity of kv_block_swap (through the C ABI) against the memcpy oracle: bytewise."""
import numpy as np
import pytest

import oracle
from paper_2602_07878_amd import workloads as W

pytestmark = pytest.mark.gpu


def gpu_swap(src_np, dst_np, mapping, **desc_kw):
    import torch
    from paper_2602_07878_amd import binding
    src = torch.from_numpy(src_np).cuda()
    dst = torch.from_numpy(dst_np).cuda()
    m = torch.from_numpy(np.ascontiguousarray(mapping, dtype=np.int32)).cuda()
    d = binding.swap_desc(**desc_kw)
    assert binding.validate_mapping(d, m) == 0
    binding.kv_block_swap(d, src, dst, m)
    torch.cuda.synchronize()
    return dst.cpu().numpy()


@pytest.mark.parametrize("planes,bb,lens", [
    (4, 32768, (100, 700, 16, 33)), (64, 4096, (512, 90)), (1, 16, (1, 17, 300)),
    (3, 48, (5, 33, 16, 70)), (2, 32768 + 16, (64, 65)), (7, 1 << 20, (40,)),
])
def test_gather_scatter_round_trip_bitwise(planes, bb, lens):
    sw = W.make_swap_workload("t", 7, victim_lens=lens, num_planes=planes, block_bytes=bb)
    n, NB = sw.n_blocks, sw.num_pool_blocks
    pool = W.random_bytes((planes * NB * bb + 7) // 8 * 8, 8)[:planes * NB * bb].copy()
    # include NaN / -0 bit patterns: bytes are bytes
    pool[:8] = np.frombuffer(np.array([np.nan, -0.0], np.float32).tobytes(), np.uint8)
    staging0 = np.full(planes * n * bb, 0xAB, np.uint8)
    kw = dict(num_planes=planes, block_bytes=bb)
    got_st = gpu_swap(pool, staging0, sw.gather_mapping, src_num_blocks=NB, dst_num_blocks=n, **kw)
    ref_st = staging0.copy()
    oracle.kv_block_swap(pool, ref_st, sw.gather_mapping, **kw)
    assert np.array_equal(got_st, ref_st)
    pool2_0 = np.full_like(pool, 0xCD)
    got_p2 = gpu_swap(got_st, pool2_0, sw.scatter_mapping, src_num_blocks=n, dst_num_blocks=NB, **kw)
    ref_p2 = pool2_0.copy()
    oracle.kv_block_swap(ref_st, ref_p2, sw.scatter_mapping, **kw)
    assert np.array_equal(got_p2, ref_p2)          # includes every untouched 0xCD byte
    p3 = got_p2.reshape(planes, NB, bb)
    o3 = pool.reshape(planes, NB, bb)
    assert np.array_equal(p3[:, sw.new_blocks], o3[:, sw.src_blocks])


def test_plane_strides_and_fan_out():
    planes, bb, NB = 3, 256, 10
    pstride = NB * bb + 64
    src = W.random_bytes(planes * pstride, 9).copy()
    dst0 = np.full(planes * (4 * bb + 32), 0x11, np.uint8)
    mapping = np.array([[2, 0], [2, 3], [9, 1]], np.int32)      # source block 2 copied twice
    kw = dict(num_planes=planes, block_bytes=bb, src_num_blocks=NB, dst_num_blocks=4,
              src_plane_stride_bytes=pstride, dst_plane_stride_bytes=4 * bb + 32)
    got = gpu_swap(src, dst0, mapping, **kw)
    ref = dst0.copy()
    oracle.kv_block_swap(src, ref, mapping, num_planes=planes, block_bytes=bb,
                         src_plane_stride=pstride, dst_plane_stride=4 * bb + 32,
                         src_num_blocks=NB, dst_num_blocks=4)
    assert np.array_equal(got, ref)


@pytest.mark.parametrize("dtype,eb", [("bf16", 2), ("f8", 1)])
def test_swap_is_transparent_to_attention(dtype, eb):
    """Evict a sequence to staging, bring it back into other blocks, rewrite its table:
    the attention output is bit-identical (Sec. 5.1.2: the victim resumes where it stopped).
    The swap moves bytes, so 8-bit pools are the same call with blocks of half the size."""
    import torch
    from paper_2602_07878_amd import binding
    from helpers import run_hip, to_device
    w = W.make_attn_workload("swapattn", 50, dtype=dtype, Hq=32, Hkv=8, D=128, block_size=16,
                             context_lens=[700, 1300, 90], pool_factor=2.5, poison=False)
    before = run_hip(w)
    victim = 1
    nb = int(W.blocks_needed(w.context_lens, 16)[victim])
    old = w.block_tables[victim, :nb].copy()
    used = set(int(b) for b in w.block_tables[w.block_tables >= 0])
    free = np.array([b for b in range(w.num_pool_blocks) if b not in used], np.int32)
    new = np.random.default_rng(3).permutation(free)[:nb].astype(np.int32)
    bb = 8 * 16 * 128 * eb
    dev = to_device(w)
    pools = torch.stack([dev["k_pool"], dev["v_pool"]])            # 2 planes
    staging = torch.zeros(2 * nb * bb, dtype=torch.uint8, device="cuda:0")
    slots = np.arange(nb, dtype=np.int32)
    g = torch.from_numpy(np.stack([old, slots], 1).astype(np.int32)).cuda()
    s = torch.from_numpy(np.stack([slots, new], 1).astype(np.int32)).cuda()
    binding.kv_block_swap(binding.swap_desc(2, bb, w.num_pool_blocks, nb), pools, staging, g)
    pools[:, torch.from_numpy(old).long().cuda()] = float("nan") if eb == 2 else 0x7F   # the old blocks are gone (NaN)
    binding.kv_block_swap(binding.swap_desc(2, bb, nb, w.num_pool_blocks), staging, pools, s)
    torch.cuda.synchronize()
    w.block_tables[victim, :nb] = new
    dev2 = dict(dev, k_pool=pools[0], v_pool=pools[1],
                block_tables=torch.from_numpy(w.block_tables).cuda())
    after = run_hip(w, dev2)
    assert np.array_equal(before, after)


# ---- host leg (Sec. 5.1.2: the victims' blocks go to CPU host memory and come back) ---------
@pytest.mark.parametrize("staging_pairs,side_stream,junk_slots", [(1, False, False), (7, True, False), (64, True, False),
                                                                  (1000, False, False), (7, False, True), (64, False, True),
                                                                  (0, False, False), (0, True, True)])
def test_swap_out_to_pinned_host_and_back_is_bit_exact(staging_pairs, side_stream, junk_slots):
    """Pieces of 1 and 7 pairs of every plane (strided copies), of 2 and of all 6 whole planes
    (contiguous copies), or (0) no staging buffer: the kernel reads and writes the host memory
    itself; on the current stream or on another one.  junk_slots: the host-slot
    column of the mappings holds arbitrary numbers; the host slot of pair j is j whatever it says,
    so the result is the same and nothing outside the buffers is touched."""
    import oracle
    import torch
    from paper_2602_07878_amd import binding
    planes, bb = 6, 4096
    sw = W.make_swap_workload("hostleg", 71, victim_lens=(700, 33, 1200, 16, 90), num_planes=planes,
                              block_bytes=bb)
    n = sw.n_blocks
    pool = W.random_bytes(sw.pool_bytes, 72)
    d_pool = torch.from_numpy(pool).cuda()
    host = torch.zeros(planes * n * bb + 64, dtype=torch.uint8).pin_memory()
    host[-64:] = 0xA5                                                   # canary behind the slots
    staging = None
    if staging_pairs:
        staging = torch.empty((1 if staging_pairs < 64 else 2) * staging_pairs * planes * bb, dtype=torch.uint8, device="cuda")
    stream = torch.cuda.Stream() if side_stream else torch.cuda.current_stream()
    stream.wait_stream(torch.cuda.current_stream())                     # the uploads above
    out_desc = binding.swap_desc(planes, bb, sw.num_pool_blocks, n)
    gmap, smap = sw.gather_mapping.copy(), sw.scatter_mapping.copy()
    if junk_slots:
        gmap[:, 1] = np.random.default_rng(1).integers(-2**31, 2**31 - 1, n)
        smap[:, 0] = np.random.default_rng(2).integers(-2**31, 2**31 - 1, n)
    gm = torch.from_numpy(gmap).cuda()
    stream.wait_stream(torch.cuda.current_stream())
    binding.kv_swap_out_host(out_desc, d_pool, host, gm, staging, stream=stream)
    stream.synchronize()                                                # that stream alone
    ref = np.zeros(planes * n * bb, np.uint8)
    oracle.kv_block_swap(pool, ref, sw.gather_mapping, num_planes=planes, block_bytes=bb)
    assert np.array_equal(host[:-64].numpy(), ref) and bool((host[-64:] == 0xA5).all())
    # back into fresh blocks of a poisoned pool
    d_new = torch.full_like(d_pool, 0x5A)
    in_desc = binding.swap_desc(planes, bb, n, sw.num_pool_blocks)
    sm = torch.from_numpy(smap).cuda()
    stream.wait_stream(torch.cuda.current_stream())
    binding.kv_swap_in_host(in_desc, host, d_new, sm, staging, stream=stream)
    stream.synchronize()
    ref_pool = np.full(sw.pool_bytes, 0x5A, np.uint8)
    oracle.kv_block_swap(ref, ref_pool, sw.scatter_mapping, num_planes=planes, block_bytes=bb)
    assert np.array_equal(d_new.cpu().numpy(), ref_pool)                # blocks in place, nothing else touched


def test_swap_out_to_host_beside_decode_calls_on_another_stream():
    """The paper's setting: a victim's blocks leave while the other requests keep decoding.  The
    unstaged swap-out runs on one stream, planned decode calls over other pools on a second one;
    the calls share nothing, so both results are what they are alone."""
    import oracle
    import torch
    from helpers import run_oracle, to_device
    from paper_2602_07878_amd import binding
    planes, bb = 8, 32768
    sw = W.make_swap_workload("beside", 91, victim_lens=(3000, 2000, 4000, 1500), num_planes=planes, block_bytes=bb)
    n = sw.n_blocks
    pool = W.random_bytes(sw.pool_bytes, 92)
    d_pool = torch.from_numpy(pool).cuda()
    host = torch.zeros(planes * n * bb, dtype=torch.uint8).pin_memory()
    gm = torch.from_numpy(sw.gather_mapping).cuda()
    out_desc = binding.swap_desc(planes, bb, sw.num_pool_blocks, n)
    w = W.config2_llama8b(B=16)
    dev = to_device(w)
    desc = binding.attn_desc_for(dev["q"], dev["k_pool"], dev["v_pool"], dev["block_tables"],
                                 max_context_len=w.max_context_len)
    plan = binding.attn_plan(desc, dev["block_tables"], dev["context_lens"])
    outs = [torch.zeros(w.B, w.Hq, w.D, device="cuda:0") for _ in range(40)]
    s_swap, s_dec = torch.cuda.Stream(), torch.cuda.Stream()
    torch.cuda.synchronize()
    ws = None
    for i, o in enumerate(outs):
        if i == 3:                                    # the decode stream is busy when the swap arrives
            binding.kv_swap_out_host(out_desc, d_pool, host, gm, stream=s_swap)
        ws = binding.paged_decode_attention_planned(desc, plan, dev["q"], dev["k_pool"], dev["v_pool"],
                                                    dev["block_tables"], dev["context_lens"], w.scale, o,
                                                    workspace=ws, stream=s_dec)
    torch.cuda.synchronize()
    ref_host = np.zeros(planes * n * bb, np.uint8)
    oracle.kv_block_swap(pool, ref_host, sw.gather_mapping, num_planes=planes, block_bytes=bb)
    assert np.array_equal(host.numpy(), ref_host)
    ref = run_oracle(w)
    for o in outs:
        assert torch.equal(o, outs[0])                # the same bits every call
    assert np.abs(outs[0].cpu().numpy().astype(np.float64) - ref).max() <= 2e-3
