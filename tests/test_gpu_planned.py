"""GPU parity of paged_decode_attention_planned (a per-step plan from pkv_attn_plan, Sec. 4.2: the
layer calls of a decode step share block tables and lengths) against the fp64 oracle, through the
C ABI.  Tolerance as for the unplanned call (2e-3, bf16 inputs and fp32 accumulation)."""
import numpy as np
import pytest

from paper_2602_07878_amd import workloads as W
from helpers import run_hip, run_oracle, to_device

pytestmark = pytest.mark.gpu

TOL = 2e-3


def check(w, **kw):
    got = run_hip(w, planned=True, **kw)
    ref = run_oracle(w)
    assert np.all(np.isfinite(got)), "non-finite output"
    err = np.abs(got - ref).max() if got.size else 0.0
    print(f"{w.name}: B={w.B} Hq={w.Hq} Hkv={w.Hkv} T={w.total_tokens} pt={kw.get('partition_tokens')} "
          f"max_abs_err={err:.3e}", flush=True)
    assert err <= TOL * max(1.0, w.v_scale), err
    return got


def mk(name, seed, lens, dtype="bf16", Hq=32, Hkv=8, bs=16, **kw):
    return W.make_attn_workload(name, seed, dtype=dtype, Hq=Hq, Hkv=Hkv, D=128, block_size=bs, context_lens=lens,
                                pool_factor=1.2, **kw)


@pytest.mark.parametrize("dtype", ["bf16", "f8"])
@pytest.mark.parametrize("Hq,Hkv", [(32, 8), (64, 8), (8, 8), (16, 8), (24, 8), (32, 2)])
def test_shapes_ragged_lengths(dtype, Hq, Hkv):
    lens = [1, 15, 16, 17, 63, 64, 65, 511, 512, 513, 1000, 1025, 0, 2047]
    w = mk(f"planned_ragged_{dtype}_{Hq}_{Hkv}", 501, lens, dtype=dtype, Hq=Hq, Hkv=Hkv)
    got = check(w)
    assert np.all(got[12] == 0.0)


@pytest.mark.parametrize("dtype", ["bf16", "f8"])
@pytest.mark.parametrize("pt", [0, 64, 512])
def test_same_cut_as_the_unplanned_call_and_same_bits_from_call_to_call(dtype, pt):
    """The plan holds what the unplanned call works out for itself: same cut of the work, same
    partials, same merge order.  With 8-bit pools both calls run the same kernel code and give the
    same bits; with bf16 pools the unplanned call has a kernel of its own and the two agree to
    rounding.  One plan serving several calls gives the same bits every time."""
    rng = np.random.default_rng(502)
    lens = [int(x) for x in rng.integers(600, 1500, 40)]
    w = mk(f"planned_bits_{dtype}", 502, lens, dtype=dtype)
    dev = to_device(w)
    a = check(w, dev=dev, partition_tokens=pt)
    plain = run_hip(w, dev, partition_tokens=pt)
    assert np.array_equal(a, plain) if dtype == "f8" else np.abs(a - plain).max() <= 1e-5
    for calls in (1, 3):
        assert np.array_equal(a, run_hip(w, dev, partition_tokens=pt, planned=True, calls=calls))


@pytest.mark.parametrize("dtype", ["bf16", "f8"])
@pytest.mark.parametrize("bs", [16, 32, 128])
def test_block_sizes(dtype, bs):
    w = mk(f"planned_bs{bs}", 503, [5, bs - 1, bs, bs + 1, 700, 1300], dtype=dtype, bs=bs)
    check(w)


@pytest.mark.parametrize("dtype", ["bf16", "f8"])
def test_every_tile_count_and_tail_length(dtype):
    lens = list(range(1, 133)) + [500 + i for i in range(30)]
    w = mk("planned_tails", 504, lens, dtype=dtype, Hq=8, Hkv=2)
    check(w)
    check(w, partition_tokens=64)


def test_all_contexts_empty_and_single_token():
    w = mk("planned_empty", 505, [0, 0, 0])
    assert np.all(run_hip(w, planned=True) == 0.0)
    w = mk("planned_one", 506, [1])
    check(w)


def test_one_plan_serves_calls_with_other_q_pools_and_output_type():
    """The layers of a step: same tables and lengths, other q and pools."""
    import torch
    from paper_2602_07878_amd import binding
    import copy
    w1 = mk("planned_layers", 507, [700, 64, 1500, 17, 3000])
    w2 = copy.deepcopy(w1)                       # another layer: K and V exchanged, the query heads rotated
    w2.k_pool, w2.v_pool, w2.q = w1.v_pool.copy(), w1.k_pool.copy(), np.roll(w1.q, 3, axis=1).copy()
    d1, d2 = to_device(w1), to_device(w2)
    desc = binding.attn_desc_for(d1["q"], d1["k_pool"], d1["v_pool"], d1["block_tables"],
                                 max_context_len=w1.max_context_len)
    plan = binding.attn_plan(desc, d1["block_tables"], d1["context_lens"])
    ws = None
    for w, d in ((w1, d1), (w2, d2), (w1, d1)):
        out = torch.empty(w.B, w.Hq, w.D, device="cuda:0")
        ws = binding.paged_decode_attention_planned(desc, plan, d["q"], d["k_pool"], d["v_pool"], d1["block_tables"],
                                                    d1["context_lens"], w.scale, out, workspace=ws)
        torch.cuda.synchronize()
        assert np.abs(out.cpu().numpy().astype(np.float64) - run_oracle(w)).max() <= TOL
    desc.out_dtype = binding.PKV_BF16
    outb = torch.empty(w1.B, w1.Hq, w1.D, device="cuda:0", dtype=torch.bfloat16)
    binding.paged_decode_attention_planned(desc, plan, d1["q"], d1["k_pool"], d1["v_pool"], d1["block_tables"],
                                           d1["context_lens"], w1.scale, outb, workspace=ws)
    torch.cuda.synchronize()
    ref = run_oracle(w1)
    assert np.all(np.abs(outb.float().cpu().numpy() - ref) <= TOL + np.abs(ref) * 2.0 ** -8)


def test_a_plan_for_another_geometry_or_too_long_contexts_gives_nan_not_a_fault():
    import torch
    from paper_2602_07878_amd import binding
    w = mk("planned_wrong", 509, [700, 64, 1500, 17])
    d = to_device(w)
    desc = binding.attn_desc_for(d["q"], d["k_pool"], d["v_pool"], d["block_tables"], max_context_len=w.max_context_len)
    plan = binding.attn_plan(desc, d["block_tables"], d["context_lens"])
    other = binding.attn_desc_for(d["q"], d["k_pool"], d["v_pool"], d["block_tables"],
                                  max_context_len=w.max_context_len, partition_tokens=64)
    big = torch.zeros(max(binding.lib().pkv_attn_plan_bytes(other), plan.numel()), dtype=torch.uint8, device="cuda:0")
    big[:plan.numel()] = plan
    out = torch.zeros(w.B, w.Hq, w.D, device="cuda:0")
    binding.paged_decode_attention_planned(other, big, d["q"], d["k_pool"], d["v_pool"], d["block_tables"],
                                           d["context_lens"], w.scale, out)
    torch.cuda.synchronize()
    assert bool(torch.isnan(out).all())
    # lengths beyond what the descriptor allows: the plan says so, nothing is read through it
    short = binding.attn_desc_for(d["q"], d["k_pool"], d["v_pool"], d["block_tables"], max_context_len=256)
    plan2 = binding.attn_plan(short, d["block_tables"], d["context_lens"])
    out2 = torch.zeros(w.B, w.Hq, w.D, device="cuda:0")
    binding.paged_decode_attention_planned(short, plan2, d["q"], d["k_pool"], d["v_pool"], d["block_tables"],
                                           d["context_lens"], w.scale, out2)
    torch.cuda.synchronize()
    assert bool(torch.isnan(out2).all())


def test_calls_that_have_no_use_for_a_plan_run_as_ordinary_calls():
    from paper_2602_07878_amd import binding
    w = W.make_attn_workload("planned_f32", 510, dtype="f32", Hq=8, Hkv=2, D=64, block_size=16,
                             context_lens=[40, 700], pool_factor=1.2)
    d = to_device(w)
    desc = binding.attn_desc_for(d["q"], d["k_pool"], d["v_pool"], d["block_tables"], max_context_len=w.max_context_len)
    assert binding.lib().pkv_attn_plan_bytes(desc) == 0
    got = run_hip(w, planned=True)
    assert np.abs(got - run_oracle(w)).max() <= 1e-4


def test_benchmark_batch_reduced():
    for w in (W.config2_llama8b(B=32), W.config2_llama8b_f8(B=32)):
        check(w)


@pytest.mark.parametrize("dtype", ["bf16", "f8", "f32"])
@pytest.mark.parametrize("Hq,Hkv,bs,tm", [(32, 8, 16, False), (64, 8, 16, False), (8, 8, 32, False), (32, 2, 16, True)])
def test_append_inside_the_planned_call_equals_append_then_attention(dtype, Hq, Hkv, bs, tm):
    """paged_decode_attention_planned_append against kv_append followed by the planned call: the
    pools bit-identical, the outputs bit-identical (bf16 with a plan appends inside the streaming
    kernel, the other cases launch the append themselves), and both against the oracle.  Lengths
    put the new token at the first, a middle and the last slot of a tile and of a block, into
    contexts of a single token and of one tile, next to an empty context; tm: token-major pools."""
    import oracle
    import torch
    from paper_2602_07878_amd import binding
    lens = [1, 2, 16, 17, 31, 32, 33, 48, 49, 640, 641, 1000, 0, 15, 1, 1, 16, 16, 2047]
    D = 128 if dtype != "f32" else 64
    w = W.make_attn_workload(f"fused_append_{dtype}", 511, dtype=dtype, Hq=Hq, Hkv=Hkv, D=D, block_size=bs,
                             context_lens=lens, pool_factor=1.3)
    rng = np.random.default_rng(512)
    rows = [rng.standard_normal((w.B, w.Hkv, w.D)).astype(np.float32) for _ in range(2)]
    conv = {"bf16": W.f32_to_bf16_bits, "f8": W.f32_to_f8e4m3_bits, "f32": lambda a: a}[dtype]
    kn, vn = conv(rows[0]), conv(rows[1])

    def dev_rows(a):
        return (torch.from_numpy(a.view(np.int16)).cuda().view(torch.bfloat16) if a.dtype == np.uint16
                else torch.from_numpy(a).cuda())

    results = []
    for fused in (False, True):
        dev = to_device(w)
        kp, vp = dev["k_pool"], dev["v_pool"]
        if tm:      # [blocks][tokens][heads][D] in memory, seen through the same logical shape
            kp = kp.permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3)
            vp = vp.permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3)
        desc = binding.attn_desc_for(dev["q"], kp, vp, dev["block_tables"], max_context_len=w.max_context_len,
                                     k_scale=w.k_scale, v_scale=w.v_scale)
        plan = binding.attn_plan(desc, dev["block_tables"], dev["context_lens"])
        out = torch.full((w.B, w.Hq, w.D), -7.0, device="cuda:0")
        if fused:
            binding.paged_decode_attention_planned(desc, plan, dev["q"], kp, vp, dev["block_tables"], dev["context_lens"],
                                                   w.scale, out, k_new=dev_rows(kn), v_new=dev_rows(vn))
        else:
            binding.kv_append(desc, dev_rows(kn), dev_rows(vn), kp, vp, dev["block_tables"], dev["context_lens"])
            binding.paged_decode_attention_planned(desc, plan, dev["q"], kp, vp, dev["block_tables"], dev["context_lens"],
                                                   w.scale, out)
        torch.cuda.synchronize()
        as_bits = lambda t: t.contiguous().view(torch.int16 if t.element_size() == 2 else torch.uint8 if t.element_size() == 1 else torch.int32).cpu().numpy()
        results.append((as_bits(kp), as_bits(vp), out.cpu().numpy()))
    assert np.array_equal(results[0][0], results[1][0]) and np.array_equal(results[0][1], results[1][1])
    assert np.array_equal(results[0][2], results[1][2])
    oracle.kv_append(w.k_pool, w.v_pool, kn, vn, w.block_tables, w.context_lens, block_size=w.block_size)
    ref = run_oracle(w)
    tol = 1e-5 if dtype == "f32" else TOL
    assert np.abs(results[1][2].astype(np.float64) - ref).max() <= tol
    assert np.all(results[1][2][12] == 0.0)


def test_append_inside_the_planned_call_on_the_benchmark_batch_from_call_to_call():
    """Several layers' worth of fused calls on one plan (other rows every time), each against the oracle."""
    import oracle
    import torch
    from paper_2602_07878_amd import binding
    w = W.config2_llama8b(B=24)
    dev = to_device(w)
    desc = binding.attn_desc_for(dev["q"], dev["k_pool"], dev["v_pool"], dev["block_tables"],
                                 max_context_len=w.max_context_len)
    plan = binding.attn_plan(desc, dev["block_tables"], dev["context_lens"])
    rng = np.random.default_rng(513)
    out = torch.zeros(w.B, w.Hq, w.D, device="cuda:0")
    ws = None
    up = lambda a: torch.from_numpy(a.view(np.int16)).cuda().view(torch.bfloat16)
    for layer in range(3):
        kn = W.f32_to_bf16_bits(rng.standard_normal((w.B, w.Hkv, w.D)).astype(np.float32))
        vn = W.f32_to_bf16_bits(rng.standard_normal((w.B, w.Hkv, w.D)).astype(np.float32))
        ws = binding.paged_decode_attention_planned(desc, plan, dev["q"], dev["k_pool"], dev["v_pool"], dev["block_tables"],
                                                    dev["context_lens"], w.scale, out, workspace=ws, k_new=up(kn), v_new=up(vn))
        torch.cuda.synchronize()
        oracle.kv_append(w.k_pool, w.v_pool, kn, vn, w.block_tables, w.context_lens, block_size=w.block_size)
        assert np.array_equal(dev["k_pool"].view(torch.int16).cpu().numpy().view(np.uint16), w.k_pool)
        assert np.array_equal(dev["v_pool"].view(torch.int16).cpu().numpy().view(np.uint16), w.v_pool)
        assert np.abs(out.cpu().numpy().astype(np.float64) - run_oracle(w)).max() <= TOL


@pytest.mark.parametrize("dtype", ["bf16", "f8"])
def test_many_short_contexts_with_and_without_the_append(dtype):
    """1 500 sequences of 1..40 tokens: most pairs are a single tile, so segments open and close at
    every tile, the queries and new rows of consecutive tiles cannot all be fetched ahead, and the
    descriptor batches are as short as the chunks."""
    import oracle
    import torch
    from paper_2602_07878_amd import binding
    rng = np.random.default_rng(520)
    lens = [int(x) for x in rng.integers(1, 41, 1500)]
    lens[7] = 0
    w = mk(f"planned_short_{dtype}", 521, lens, dtype=dtype, Hq=16, Hkv=8)
    check(w)
    check(w, partition_tokens=64)
    dev = to_device(w)
    conv = W.f32_to_bf16_bits if dtype == "bf16" else W.f32_to_f8e4m3_bits
    kn = conv(rng.standard_normal((w.B, w.Hkv, w.D)).astype(np.float32))
    vn = conv(rng.standard_normal((w.B, w.Hkv, w.D)).astype(np.float32))
    up = (lambda a: torch.from_numpy(a.view(np.int16)).cuda().view(torch.bfloat16)) if dtype == "bf16" else (lambda a: torch.from_numpy(a).cuda())
    desc = binding.attn_desc_for(dev["q"], dev["k_pool"], dev["v_pool"], dev["block_tables"],
                                 max_context_len=w.max_context_len)
    plan = binding.attn_plan(desc, dev["block_tables"], dev["context_lens"])
    out = torch.zeros(w.B, w.Hq, w.D, device="cuda:0")
    binding.paged_decode_attention_planned(desc, plan, dev["q"], dev["k_pool"], dev["v_pool"], dev["block_tables"],
                                           dev["context_lens"], w.scale, out, k_new=up(kn), v_new=up(vn))
    torch.cuda.synchronize()
    oracle.kv_append(w.k_pool, w.v_pool, kn, vn, w.block_tables, w.context_lens, block_size=w.block_size)
    bits = lambda t: t.view(torch.int16).cpu().numpy().view(np.uint16) if dtype == "bf16" else t.cpu().numpy()
    assert np.array_equal(bits(dev["k_pool"]), w.k_pool) and np.array_equal(bits(dev["v_pool"]), w.v_pool)
    assert np.abs(out.cpu().numpy().astype(np.float64) - run_oracle(w)).max() <= TOL
