"""GPU parity of paged_decode_attention with 8-bit (OCP E4M3) K/V pools and a bfloat16 q, through
the C ABI, against the fp64 oracle.

Tolerance: the stored codes decode exactly to bfloat16 values, so the arithmetic is that of the
bfloat16 call: max abs error 2e-3 * max(1, v_scale) (bf16 inputs, fp32 accumulation; v_scale is a
plain factor on the output)."""
import numpy as np
import pytest

import oracle
from paper_2602_07878_amd import workloads as W
from helpers import run_hip, run_oracle, to_device

pytestmark = pytest.mark.gpu

TOL = 2e-3


def check(w, **kw):
    got = run_hip(w, **kw)
    ref = run_oracle(w)
    assert np.all(np.isfinite(got)), "non-finite output (poison leaked?)"
    err = np.abs(got - ref).max() if got.size else 0.0
    print(f"{w.name}: B={w.B} Hq={w.Hq} Hkv={w.Hkv} D={w.D} T={w.total_tokens} flags={kw.get('flags', 0)} "
          f"pt={kw.get('partition_tokens')} max_abs_err={err:.3e}", flush=True)
    assert err <= TOL * max(1.0, w.v_scale), err
    return got, ref


def mk(name, seed, lens, Hq=32, Hkv=8, D=128, bs=16, **kw):
    return W.make_attn_workload(name, seed, dtype="f8", Hq=Hq, Hkv=Hkv, D=D, block_size=bs, context_lens=lens,
                                pool_factor=1.2, **kw)


@pytest.mark.parametrize("flags", [0, 1])
def test_every_code_decodes_exactly(flags):
    """1-token contexts return their V row: the 254 finite codes spread over the dims of two
    sequences come back as the oracle decodes them, exactly (weight 1, normaliser 1)."""
    w = mk("codes", 401, [1, 1, 1], Hq=8, Hkv=8)
    finite = np.array([c for c in range(256) if c not in (0x7F, 0xFF)], np.uint8)
    for i in range(3):
        blk = w.block_tables[i, 0]
        for g in range(8):
            w.v_pool[blk, g, 0] = np.roll(finite, 17 * (i * 8 + g))[:128]
    got = run_hip(w, flags=flags)
    ref = run_oracle(w)
    assert np.array_equal(got, ref)


@pytest.mark.parametrize("flags", [0, 1])
def test_key_codes_in_the_score_path(flags):
    """Keys that hold every finite code of magnitude <= 8 in turn (the rest normal data)."""
    w = mk("kcodes", 402, [254, 100, 254], Hq=8, Hkv=2)
    finite = np.array([c for c in range(256) if c not in (0x7F, 0xFF)], np.uint8)
    import torch
    vals = torch.from_numpy(finite).view(torch.float8_e4m3fn).float().numpy()
    use = finite[np.abs(vals) <= 8]
    for i in (0, 2):
        for t in range(int(w.context_lens[i])):
            blk = w.block_tables[i, t // 16]
            w.k_pool[blk, :, t % 16, (5 * t) % 128] = use[t % len(use)]
    check(w, flags=flags)


@pytest.mark.parametrize("Hq,Hkv,D", [(32, 8, 128), (64, 8, 128), (8, 8, 128), (16, 8, 128), (24, 8, 128),
                                       (32, 2, 128), (4, 1, 256), (8, 2, 256)])
def test_shapes_ragged_lengths(Hq, Hkv, D):
    lens = [1, 15, 16, 17, 63, 64, 65, 511, 512, 513, 1000, 1025, 0, 2047]
    w = mk(f"ragged_f8_{Hq}_{Hkv}_{D}", 403, lens, Hq=Hq, Hkv=Hkv, D=D)
    for flags in (0, 1):
        got, _ = check(w, flags=flags)
        assert np.all(got[12] == 0.0)


@pytest.mark.parametrize("bs", [16, 32, 64, 128])
def test_block_sizes(bs):
    w = mk(f"f8_bs{bs}", 404, [5, bs - 1, bs, bs + 1, 700, 1300], bs=bs)
    check(w)


@pytest.mark.parametrize("pt", [0, 64, 512, 1024])
def test_partition_lengths_and_reproducibility(pt):
    w = mk("f8_parts", 405, [3000, 777, 4096, 129, 1])
    dev = to_device(w)
    a, _ = check(w, dev=dev, partition_tokens=pt)
    b = run_hip(w, dev, partition_tokens=pt)
    assert np.array_equal(a, b)


@pytest.mark.parametrize("ks,vs", [(0.5, 2.0), (0.37, 1.7), (3.0, 0.01)])
def test_dequantisation_factors(ks, vs):
    w = mk("f8_scales", 406, [700, 64, 1500, 17])
    w.k_scale, w.v_scale = ks, vs
    for flags in (0, 1):
        check(w, flags=flags)


def test_every_tile_count_and_tail_length():
    lens = list(range(1, 133)) + [500 + i for i in range(30)]
    w = mk("f8_tails", 407, lens, Hq=8, Hkv=2)
    check(w)
    check(w, partition_tokens=64)


def test_benchmark_batch_reduced_and_token_major_layout():
    import torch
    from paper_2602_07878_amd import binding
    w = W.config2_llama8b_f8(B=16)
    check(w)
    check(w, flags=1)
    ref = run_oracle(w)
    dev = to_device(w)
    k_tm = dev["k_pool"].permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3)
    v_tm = dev["v_pool"].permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3)
    out = torch.empty(w.B, w.Hq, w.D, dtype=torch.float32, device="cuda:0")
    binding.paged_decode_attention(dev["q"], k_tm, v_tm, dev["block_tables"], dev["context_lens"], w.scale, out,
                                   max_context_len=w.max_context_len)
    torch.cuda.synchronize()
    assert np.abs(out.cpu().numpy().astype(np.float64) - ref).max() <= TOL


def test_bf16_output_option():
    import torch
    w = mk("f8_bf16out", 408, [900, 64, 2000])
    got = run_hip(w, out_dtype=torch.bfloat16)
    ref = run_oracle(w)
    ulp = np.maximum(np.abs(ref), 2.0 ** -126) * 2.0 ** -8
    assert np.all(np.abs(got - ref) <= TOL + ulp)


def test_append_of_8_bit_rows_is_bit_exact_and_seen_by_attention():
    import torch
    from paper_2602_07878_amd import binding
    w = mk("f8_append", 409, [33, 16, 1, 700, 0])
    dev = to_device(w)
    rng = np.random.default_rng(4)
    kn = W.f32_to_f8e4m3_bits(rng.standard_normal((w.B, w.Hkv, w.D)).astype(np.float32))
    vn = W.f32_to_f8e4m3_bits(rng.standard_normal((w.B, w.Hkv, w.D)).astype(np.float32))
    desc = binding.attn_desc_for(dev["q"], dev["k_pool"], dev["v_pool"], dev["block_tables"],
                                 max_context_len=w.max_context_len)
    binding.kv_append(desc, torch.from_numpy(kn).cuda(), torch.from_numpy(vn).cuda(), dev["k_pool"], dev["v_pool"],
                      dev["block_tables"], dev["context_lens"])
    # the oracle's append moves bytes, whatever they encode
    oracle.kv_append(w.k_pool, w.v_pool, kn, vn, w.block_tables, w.context_lens, block_size=w.block_size)
    torch.cuda.synchronize()
    assert np.array_equal(dev["k_pool"].cpu().numpy(), w.k_pool)
    assert np.array_equal(dev["v_pool"].cpu().numpy(), w.v_pool)
    check(w, dev=dev)


def test_unsupported_combinations_are_refused():
    import ctypes
    import torch
    from paper_2602_07878_amd import binding
    w = mk("f8_bad", 410, [40, 17], Hq=8, Hkv=2)
    dev = to_device(w)
    out = torch.zeros(w.B, w.Hq, w.D, device="cuda:0")
    desc = binding.attn_desc_for(dev["q"], dev["k_pool"], dev["v_pool"], dev["block_tables"], max_context_len=64)
    for field, value, status in (("k_scale", -1.0, "PKV_ERR_SHAPE"), ("v_scale", float("inf"), "PKV_ERR_SHAPE"),
                                 ("head_dim", 64, "PKV_ERR_SHAPE")):
        d2 = binding.AttnDesc.from_buffer_copy(desc)
        setattr(d2, field, value)
        st = binding.lib().paged_decode_attention(ctypes.byref(d2), dev["q"].data_ptr(), dev["k_pool"].data_ptr(),
                                                  dev["v_pool"].data_ptr(), dev["block_tables"].data_ptr(),
                                                  dev["context_lens"].data_ptr(), 0.1, out.data_ptr(), None, 0, None)
        assert binding.status_string(st) == status
    # the prefill call over 8-bit pools needs a workspace (for the bf16 copy of the blocks): refused without
    z = torch.zeros(4, dtype=torch.int32, device="cuda:0")
    with pytest.raises(binding.PkvError):
        binding.paged_prefill_attention(desc, dev["q"], dev["k_pool"], dev["v_pool"], dev["block_tables"],
                                        dev["context_lens"], z, z, 4, 0.1, out)
