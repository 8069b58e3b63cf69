"""Seeded random shapes through every GPU call against the oracle: head groupings, block sizes,
length mixes (empty, one token, ragged, long), partition caps, chunked prefill.  Same tolerances as
the fixed cases: 1e-5 (fp32), 2e-3 (bf16), copies bit-exact."""
import numpy as np
import pytest

from paper_2602_07878_amd import workloads as W
from helpers import run_hip, run_oracle, to_device

pytestmark = pytest.mark.gpu


def random_lens(rng, B, hi):
    kind = rng.integers(0, 4, B)
    lens = np.where(kind == 0, rng.integers(0, 3, B),                    # empty / tiny
           np.where(kind == 1, rng.integers(1, 200, B),                  # short
           np.where(kind == 2, rng.integers(1, hi, B),                   # anything
                    (rng.integers(1, max(2, hi // 16), B)) * 16)))       # exact multiples of a tile
    return [int(x) for x in lens]


@pytest.mark.parametrize("seed", range(16))
def test_decode_random(seed):
    rng = np.random.default_rng(1000 + seed)
    Hkv = int(rng.choice([1, 2, 4, 8]))
    G = int(rng.choice([1, 2, 3, 4, 5, 8, 12, 16]))
    dtype = "bf16" if seed % 4 else "f32"
    D = 128 if dtype == "bf16" and seed % 3 else int(rng.choice([64, 128]))
    bs = int(rng.choice([16, 32, 64, 128]))
    B = int(rng.integers(1, 40))
    lens = random_lens(rng, B, int(rng.choice([300, 1500, 6000])))
    w = W.make_attn_workload(f"rnd{seed}", 2000 + seed, dtype=dtype, Hq=Hkv * G, Hkv=Hkv, D=D, block_size=bs,
                             context_lens=lens, pool_factor=float(rng.choice([1.0, 1.3, 2.0])))
    ref = run_oracle(w)
    dev = to_device(w)
    tol = 2e-3 if dtype == "bf16" else 1e-5
    for pt in (0, int(rng.choice([64, 128, 512, 1024]))):
        got = run_hip(w, dev, partition_tokens=pt)
        assert np.all(np.isfinite(got))
        err = np.abs(got - ref).max() if got.size else 0.0
        print(f"seed {seed}: {dtype} Hq={w.Hq} Hkv={Hkv} D={D} bs={bs} B={B} T={w.total_tokens} pt={pt} err={err:.2e}", flush=True)
        assert err <= tol, (seed, pt, err)
        assert np.all(got[np.asarray(lens) == 0] == 0.0)


@pytest.mark.parametrize("seed", range(10))
def test_prefill_and_append_random(seed):
    import oracle
    import torch
    from paper_2602_07878_amd import binding
    rng = np.random.default_rng(3000 + seed)
    Hkv = int(rng.choice([1, 2, 4, 8]))
    G = int(rng.choice([1, 2, 3, 4, 7, 8]))
    bs = int(rng.choice([16, 32, 64]))
    B = int(rng.integers(1, 12))
    lens = [max(1, x) for x in random_lens(rng, B, int(rng.choice([200, 900, 2500])))]
    w = W.make_attn_workload(f"rndp{seed}", 4000 + seed, dtype="bf16", Hq=Hkv * G, Hkv=Hkv, D=128, block_size=bs,
                             context_lens=lens, pool_factor=1.25)
    dev = to_device(w)
    up = lambda a: torch.from_numpy(a.view(np.int16)).cuda().view(torch.bfloat16)
    # append the last token of every sequence, bit-exact
    kn = W.f32_to_bf16_bits(rng.standard_normal((B, Hkv, 128)).astype(np.float32))
    vn = W.f32_to_bf16_bits(rng.standard_normal((B, Hkv, 128)).astype(np.float32))
    desc = binding.attn_desc_for(dev["q"], dev["k_pool"], dev["v_pool"], dev["block_tables"],
                                 max_context_len=w.max_context_len)
    binding.kv_append(desc, up(kn), up(vn), dev["k_pool"], dev["v_pool"], dev["block_tables"], dev["context_lens"])
    oracle.kv_append(w.k_pool, w.v_pool, kn, vn, w.block_tables, w.context_lens, block_size=bs)
    torch.cuda.synchronize()
    assert np.array_equal(dev["k_pool"].view(torch.int16).cpu().numpy().view(np.uint16), w.k_pool)
    assert np.array_equal(dev["v_pool"].view(torch.int16).cpu().numpy().view(np.uint16), w.v_pool)
    # causal attention of a random tail of every sequence
    ql = np.array([int(rng.integers(0, n + 1)) if rng.random() < 0.7 else n for n in lens], np.int32)
    total = int(ql.sum())
    q = W.f32_to_bf16_bits(rng.standard_normal((total, w.Hq, 128)).astype(np.float32))
    ref = oracle.paged_prefill_attention(q, w.k_pool, w.v_pool, w.block_tables, w.context_lens, ql, w.scale,
                                         block_size=bs)
    if total == 0:
        return
    out = torch.empty(total, w.Hq, 128, dtype=torch.float32, device="cuda")
    cu = torch.from_numpy(np.concatenate([[0], np.cumsum(ql)]).astype(np.int32)).cuda()
    binding.paged_prefill_attention(desc, up(q), dev["k_pool"], dev["v_pool"], dev["block_tables"],
                                    dev["context_lens"], torch.from_numpy(ql).cuda(), cu, int(ql.max()), w.scale, out)
    torch.cuda.synchronize()
    got = out.cpu().numpy().astype(np.float64)
    err = np.abs(got - ref).max()
    print(f"seed {seed}: Hq={w.Hq} Hkv={Hkv} bs={bs} lens={lens[:5]} ql={ql[:5].tolist()} err={err:.2e}", flush=True)
    assert np.all(np.isfinite(got)) and err <= 2e-3


@pytest.mark.parametrize("seed", range(6))
def test_swap_random(seed):
    import oracle
    import torch
    from paper_2602_07878_amd import binding
    rng = np.random.default_rng(5000 + seed)
    planes = int(rng.integers(1, 9))
    bb = int(rng.choice([16, 48, 4096, 32768, 32768 + 16, 1 << 18]))
    lens = [int(x) for x in rng.integers(1, 600, int(rng.integers(1, 6)))]
    sw = W.make_swap_workload("rnds", 6000 + seed, victim_lens=lens, num_planes=planes, block_bytes=bb)
    pool = W.random_bytes(sw.pool_bytes, 7000 + seed)
    st = np.zeros(sw.staging_bytes, np.uint8)
    ref = st.copy()
    oracle.kv_block_swap(pool, ref, sw.gather_mapping, num_planes=planes, block_bytes=bb)
    d_pool, d_st = torch.from_numpy(pool).cuda(), torch.from_numpy(st).cuda()
    binding.kv_block_swap(binding.swap_desc(planes, bb, sw.num_pool_blocks, sw.n_blocks), d_pool, d_st,
                          torch.from_numpy(sw.gather_mapping).cuda())
    torch.cuda.synchronize()
    assert np.array_equal(d_st.cpu().numpy(), ref)
    new_pool = np.full(sw.pool_bytes, 0x3C, np.uint8)
    d_new = torch.from_numpy(new_pool.copy()).cuda()
    oracle.kv_block_swap(ref, new_pool, sw.scatter_mapping, num_planes=planes, block_bytes=bb)
    binding.kv_block_swap(binding.swap_desc(planes, bb, sw.n_blocks, sw.num_pool_blocks), d_st, d_new,
                          torch.from_numpy(sw.scatter_mapping).cuda())
    torch.cuda.synchronize()
    assert np.array_equal(d_new.cpu().numpy(), new_pool)
