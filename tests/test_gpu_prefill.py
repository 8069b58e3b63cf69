"""GPU parity of paged_prefill_attention (through the C ABI) against the fp64 oracle.
Tolerance: max abs error 2e-3 (bf16 inputs, fp32 accumulation), outputs read as fp32."""
import numpy as np
import pytest

from paper_2602_07878_amd import workloads as W
from helpers import to_device

pytestmark = pytest.mark.gpu

TOL = 2e-3


def run_prefill(w, query_lens, seed, out_dtype=None, token_major=False, split=False, q_hook=None):
    """Returns (GPU out as float64 [total, Hq, D], oracle out).  split: bring the workspace
    that lets the library cut the walks into ranges (it must want to for the case).  q_hook maps
    the drawn query bits [total, Hq, D] to the ones both sides get."""
    import oracle
    import torch
    from paper_2602_07878_amd import binding
    ql = np.asarray(query_lens, np.int32)
    total = int(ql.sum())
    rng = np.random.default_rng(seed)
    q = W.f32_to_bf16_bits(rng.standard_normal((total, w.Hq, w.D)).astype(np.float32))
    if q_hook is not None:
        q = q_hook(q)
    ref = oracle.paged_prefill_attention(q, w.k_pool, w.v_pool, w.block_tables, w.context_lens, ql,
                                         w.scale, block_size=w.block_size)
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
    desc = binding.attn_desc_for(dq[:max(total, 1)] if total else torch.empty(1, w.Hq, w.D, dtype=torch.bfloat16, device="cuda"),
                                 kp, vp, dev["block_tables"], max_context_len=w.max_context_len, out_dtype=odt)
    desc.batch = w.B
    ws = None
    if split:
        need = binding.prefill_workspace_bytes(desc, total, int(ql.max()))
        assert need > 0, "this case was meant to be split"
        ws = torch.full((need + 64,), 0xFF, dtype=torch.uint8, device="cuda")   # NaN-filled: unwritten rows must not be read
    binding.paged_prefill_attention(desc, dq, kp, vp, dev["block_tables"], dev["context_lens"],
                                    torch.from_numpy(ql).cuda(), cu, int(ql.max()) if ql.size else 0, w.scale, out,
                                    workspace=ws)
    torch.cuda.synchronize()
    if split:
        assert bool((ws[need:] == 0xFF).all()), "wrote past the workspace"
    assert torch.all(buf[:pad] == 777.0) and torch.all(buf[pad + total * w.Hq * w.D:] == 777.0)
    return out.float().cpu().numpy().astype(np.float64), ref


def check(w, query_lens, seed=5, **kw):
    got, ref = run_prefill(w, query_lens, seed, **kw)
    assert np.all(np.isfinite(got)), "non-finite output (poison leaked?)"
    absent = np.isnan(ref)               # rows beyond a clipped query length: left as they were
    assert np.all(got[absent] == 777.0), "a row that does not exist was written"
    err = np.abs(got[~absent] - ref[~absent]).max() if got[~absent].size else 0.0
    print(f"{w.name}: Hq={w.Hq} Hkv={w.Hkv} bs={w.block_size} ctx={list(w.context_lens)[:6]} q={list(query_lens)[:6]} "
          f"max_abs_err={err:.3e}", flush=True)
    assert err <= TOL, err
    return got, ref


def mk(seed, lens, Hq=8, Hkv=2, bs=16):
    return W.make_attn_workload("prefill", seed, dtype="bf16", Hq=Hq, Hkv=Hkv, D=128, block_size=bs,
                                context_lens=list(lens), pool_factor=1.2)


def test_whole_sequences_small_and_ragged():
    lens = (1, 5, 16, 17, 100, 129, 300)
    check(mk(81, lens), lens)


def test_chunks_tails_single_tokens_and_absent_sequences():
    lens = (400, 64, 33, 257, 90, 16)
    check(mk(82, lens), (128, 1, 0, 257, 17, 16))


@pytest.mark.parametrize("Hq,Hkv", [(4, 4), (4, 2), (6, 2), (16, 2), (32, 8)])
def test_group_sizes(Hq, Hkv):
    lens = (70, 200, 31)
    check(mk(83, lens, Hq=Hq, Hkv=Hkv), (70, 130, 5))


@pytest.mark.parametrize("bs", [16, 32, 64, 128])
def test_block_sizes(bs):
    lens = (bs + 3, 3 * bs, 500)
    check(mk(84, lens, bs=bs), (bs + 3, bs, 260))


def test_long_context_short_chunk_and_chunk_of_512():
    lens = (5000, 2048, 700)
    check(mk(85, lens), (512, 512, 512))


# ---- split walks (few chunks over long contexts: the chunked-prefill case) --------------------
@pytest.mark.parametrize("lens,qlens,Hq,Hkv", [
    ((4000,), (100,), 8, 2),                 # one workgroup per head pair would walk 125 pairs: 15 ranges
    ((3000, 40, 700), (300, 40, 1), 8, 2),   # ragged: the short sequences have fewer pairs than ranges
    ((2000,), (256,), 4, 4),                 # one query head per KV head
    ((1500, 0, 900), (512, 0, 0), 8, 2),     # absent sequences
    ((2049,), (2049,), 8, 2),                # a whole prompt: the first ranges start at position 0
])
def test_split_walks_agree_with_the_oracle(lens, qlens, Hq, Hkv):
    w = mk(88, lens, Hq=Hq, Hkv=Hkv)
    got, ref = check(w, qlens, split=True)
    unsplit, _ = run_prefill(w, qlens, 5)
    assert np.abs(got - unsplit).max() <= 2e-5          # same arithmetic, other order of the sums


@pytest.mark.parametrize("bs", [32, 128])
def test_split_walks_with_larger_blocks_and_token_major_pools(bs):
    w = mk(90, (2500, 300), bs=bs)
    check(w, (260, 7), split=True)
    check(w, (100, 0), split=True, token_major=True)


def test_split_walks_bf16_output_and_small_workspace_is_refused():
    import torch
    from paper_2602_07878_amd import binding
    w = mk(89, (3000,))
    got, ref = run_prefill(w, (200,), 3, out_dtype=torch.bfloat16, split=True)
    ulp = np.maximum(np.abs(ref), 2.0 ** -126) * 2.0 ** -8
    assert np.all(np.abs(got - ref) <= TOL + ulp)
    dev = to_device(w)
    q = torch.zeros(200, w.Hq, w.D, dtype=torch.bfloat16, device="cuda")
    desc = binding.attn_desc_for(q, dev["k_pool"], dev["v_pool"], dev["block_tables"], max_context_len=w.max_context_len)
    desc.batch = 1
    need = binding.prefill_workspace_bytes(desc, 200, 200)
    assert need > 0
    ql = torch.tensor([200], dtype=torch.int32, device="cuda")
    cu = torch.tensor([0, 200], dtype=torch.int32, device="cuda")
    with pytest.raises(binding.PkvError):
        binding.paged_prefill_attention(desc, q, dev["k_pool"], dev["v_pool"], dev["block_tables"], dev["context_lens"],
                                        ql, cu, 200, w.scale, torch.empty(200, w.Hq, w.D, device="cuda"),
                                        workspace=torch.empty(need - 16, dtype=torch.uint8, device="cuda"))
    # enough workgroups anyway: no workspace wanted
    desc.batch = 64
    assert binding.prefill_workspace_bytes(desc, 64 * 200, 200) == 0


def test_query_lens_above_the_context_are_clipped_and_surplus_rows_left_alone():
    """query_lens[i] > context_lens[i]: only the first context_lens[i] rows of the sequence exist
    (row j at position j); the others keep what the output buffer held, with and without split
    walks (whose merge kernel must not touch them either)."""
    lens = (100, 40, 700, 0, 16)
    check(mk(91, lens), (130, 40, 50, 3, 17))
    w = mk(92, (3000, 20, 600))
    check(w, (300, 64, 700), split=True)


def sampled_rows_check(w, q_bits, ql, out, rows):
    """Rows `rows` of the packed output against one oracle decode row each (a query token is the
    decode definition over the positions it may see)."""
    import oracle
    cu = np.concatenate([[0], np.cumsum(ql)])
    seq = np.searchsorted(cu, rows, side="right") - 1
    ctx = (w.context_lens[seq] - ql[seq] + (rows - cu[seq]) + 1).astype(np.int32)
    ref = oracle.paged_decode_attention(q_bits[rows], w.k_pool, w.v_pool, w.block_tables[seq], ctx, w.scale,
                                        block_size=w.block_size)
    got = out[rows].astype(np.float64)
    assert np.all(np.isfinite(got))
    return float(np.abs(got - ref).max())


def test_parity_at_the_benchmarked_reprefill_shape():
    """16 sequences x 4096 tokens, 32/8 heads: 128 K/V streams (16 per XCD), 32 query groups per
    stream, the workgroup numbering at the sizes the benchmark times.  More than 512 query rows
    (all heads of each) are checked: for every sequence the first and last rows, both ends of
    wavefronts and of 128-row query groups in the first, a middle and the last group, and random
    rows."""
    import torch
    from paper_2602_07878_amd import binding
    B, n = 16, 4096
    w = W.make_attn_workload("reprefill_16x4096", 1006, dtype="bf16", Hq=32, Hkv=8, D=128, block_size=16,
                             context_lens=[n] * B, pool_factor=1.0, poison=False)
    q_bits = W.normal_array((B * n, w.Hq, w.D), np.random.SeedSequence(1016), "bf16")
    ql = np.full(B, n, np.int32)
    dev = to_device(w)
    dq = torch.from_numpy(q_bits.view(np.int16)).cuda().view(torch.bfloat16)
    cu = torch.arange(0, (B + 1) * n, n, dtype=torch.int32, device="cuda")
    out = torch.full((B * n, w.Hq, w.D), 777.0, dtype=torch.float32, device="cuda")
    desc = binding.attn_desc_for(dq, dev["k_pool"], dev["v_pool"], dev["block_tables"], max_context_len=n)
    desc.batch = B
    binding.paged_prefill_attention(desc, dq, dev["k_pool"], dev["v_pool"], dev["block_tables"],
                                    dev["context_lens"], dev["context_lens"], cu, n, w.scale, out)
    torch.cuda.synchronize()
    rng = np.random.default_rng(3)
    inside = [0, 1, 31, 32, 63, 64, 127, 128, 129, 2016, 2047, 2048, 2079, 2080, 3968, 3999, 4000, 4064, 4095]
    rows = sorted({i * n + j for i in range(B) for j in inside} | set(rng.integers(0, B * n, 256).tolist()))
    assert len(rows) >= 512
    rows = np.array(rows)
    got = out[torch.from_numpy(rows).cuda()].cpu().numpy()
    err = sampled_rows_check(w, q_bits, ql, _Rows(rows, got), rows)   # only the sampled rows were brought back
    print(f"16 x 4096 re-prefill, 32/8 heads: {len(rows)} rows x 32 heads, max_abs_err={err:.3e}", flush=True)
    assert err <= TOL
    assert not bool((out[::997] == 777.0).all(dim=(1, 2)).any()), "an output row was never written"


class _Rows:
    """out[rows] lookup for rows brought back from the device."""
    def __init__(self, rows, values):
        self.pos = {int(r): k for k, r in enumerate(rows)}
        self.values = values

    def __getitem__(self, rows):
        return self.values[[self.pos[int(r)] for r in rows]]


def test_parity_at_the_benchmarked_chunk_shape_split_and_unsplit():
    """One 512-token chunk over a context of 8192 tokens, 32/8 heads (the chunked-prefill leg of
    the benchmark), every row, with the walks split (16 ranges) and unsplit."""
    w = W.make_attn_workload("chunk_512_over_8192", 1008, dtype="bf16", Hq=32, Hkv=8, D=128, block_size=16,
                             context_lens=[8192], pool_factor=1.0, poison=False)
    for split in (True, False):
        check(w, (512,), seed=1018, split=split)


def test_last_query_token_equals_decode_kernel():
    """Row of the last token of a chunk against the decode call on the same pools."""
    import torch
    from helpers import run_hip
    lens = (333, 48, 1000)
    w = mk(86, lens, Hq=32, Hkv=8)
    got, _ = run_prefill(w, lens, 9)
    last = np.cumsum(lens) - 1
    rng = np.random.default_rng(9)
    q = W.f32_to_bf16_bits(rng.standard_normal((sum(lens), 32, 128)).astype(np.float32))
    w.q = q[last]
    dec = run_hip(w)
    assert np.abs(got[last] - dec).max() <= 1e-5


def test_bf16_output_and_token_major_layout():
    import torch
    lens = (150, 40)
    w = mk(87, lens)
    got, ref = run_prefill(w, (150, 40), 3, out_dtype=torch.bfloat16)
    ulp = np.maximum(np.abs(ref), 2.0 ** -126) * 2.0 ** -8
    assert np.all(np.abs(got - ref) <= TOL + ulp)
    check(w, (100, 40), token_major=True)


def test_rejects_unsupported_shapes():
    import torch
    from paper_2602_07878_amd import binding
    w = W.config1_tiny()                                   # fp32, D = 64
    dev = to_device(w)
    desc = binding.attn_desc_for(dev["q"], dev["k_pool"], dev["v_pool"], dev["block_tables"], max_context_len=256)
    z = torch.zeros(8, dtype=torch.int32, device="cuda")
    with pytest.raises(binding.PkvError):
        binding.paged_prefill_attention(desc, dev["q"], dev["k_pool"], dev["v_pool"], dev["block_tables"],
                                        dev["context_lens"], z, z, 4, 0.1, torch.empty_like(dev["q"]))


def test_chunk_validator_reads_the_device_arrays():
    import torch
    from paper_2602_07878_amd import binding
    w = mk(97, (300, 40, 90))
    dev = to_device(w)
    q = torch.zeros(1, w.Hq, w.D, dtype=torch.bfloat16, device="cuda")
    desc = binding.attn_desc_for(q, dev["k_pool"], dev["v_pool"], dev["block_tables"], max_context_len=w.max_context_len)
    desc.batch = 3
    t = lambda a: torch.tensor(a, dtype=torch.int32, device="cuda")
    assert binding.validate_chunks(desc, dev["context_lens"], t([128, 0, 90]), t([0, 128, 128, 218]), 128, 218) == binding.PKV_OK
    assert binding.validate_chunks(desc, dev["context_lens"], t([128, 0, 90]), t([0, 128, 130, 220]), 128, 220) == 6   # PKV_ERR_INDEX
    assert binding.validate_chunks(desc, dev["context_lens"], t([128, 0, 90]), t([0, 128, 128, 218]), 128, 217) == 6
