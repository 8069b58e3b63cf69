"""GPU parity on inputs that drive the online-softmax rescale of the matrix-core kernels.

Both kernels keep a reference maximum that lags the true one: the decode stream kernel raises it
(and rescales its accumulators) when a score exceeds it by more than 8 log2 units, the prefill
kernel when a pair's weights sum to 2^40.  With q, K ~ N(0,1) and scale 1/sqrt(D) neither happens
after a segment's first tile, so these cases plant structure that makes it happen again and again
with non-zero accumulators: a large scale, keys along the query direction whose length rises,
falls or jumps along the context, one key that takes all the weight at every position of a
chunk, and a constant vector added to every key.  bf16, head_dim 128, through the stream kernel
with both merge kernels and through the prefill kernel unsplit and with split walks.

Tolerance: max abs error 2e-3 against the fp64 oracle (bf16 inputs, fp32 accumulation), all
outputs finite."""
import numpy as np
import pytest

from paper_2602_07878_amd import workloads as W
from helpers import run_hip, run_oracle
from test_gpu_prefill import run_prefill

pytestmark = pytest.mark.gpu

TOL = 2e-3
ALPHA = 8.0   # component of every query along its KV head's planted direction


def bf16(x):
    return W.f32_to_bf16_bits(np.asarray(x, np.float32))


def f32(b):
    return W.bf16_bits_to_f32(b)


def directions(w, seed):
    """One unit vector per KV head."""
    u = np.random.default_rng(seed).standard_normal((w.Hkv, w.D))
    return (u / np.linalg.norm(u, axis=1, keepdims=True)).astype(np.float32)


def lean_queries(q_bits, w, u):
    """Every query gets the component ALPHA along its KV head's direction, so that q.u is positive
    (ALPHA + N(0,1)) for every head and a key beta*u scores about scale*ALPHA*beta."""
    G = w.Hq // w.Hkv
    q = f32(q_bits)
    q += ALPHA * np.repeat(u, G, axis=0)[None]
    return bf16(q)


def set_key(w, i, t, vec):
    """Key of token t of sequence i, all KV heads: vec [Hkv, D] (8-bit pools store vec / k_scale)."""
    blk = w.block_tables[i, t // w.block_size]
    if w.dtype == "f8":
        w.k_pool[blk, :, t % w.block_size, :] = W.f32_to_f8e4m3_bits(np.asarray(vec, np.float32) / np.float32(w.k_scale))
    else:
        w.k_pool[blk, :, t % w.block_size, :] = bf16(vec)


def plant_profile(w, u, kind, step, every=11, first=5):
    """Keys along u at positions first, first+every, ... of every sequence; their lengths rise by
    `step` from one to the next ('up'), fall ('down') or come in a seeded shuffle ('mixed')."""
    rng = np.random.default_rng(7)
    for i, n in enumerate(w.context_lens.tolist()):
        pos = list(range(first, n, every))
        beta = step * (1.0 + np.arange(len(pos)))
        if kind == "down":
            beta = beta[::-1]
        elif kind == "mixed":
            beta = rng.permutation(beta)
        for t, b in zip(pos, beta):
            set_key(w, i, t, b * u)


def decode_case(name, seed, lens, Hq, Hkv):
    return W.make_attn_workload(name, seed, dtype="bf16", Hq=Hq, Hkv=Hkv, D=128, block_size=16,
                                context_lens=lens, pool_factor=1.15)


def check_decode(w, partition_tokens):
    ref = run_oracle(w)
    got = run_hip(w, partition_tokens=partition_tokens)
    assert np.all(np.isfinite(got)), "non-finite output"
    err = np.abs(got - ref).max()
    print(f"{w.name} pt={partition_tokens}: T={w.total_tokens} max_abs_err={err:.3e}", flush=True)
    assert err <= TOL, err
    return got


LENS_SMALL = [700, 1500, 333, 64, 4000, 17, 1, 2049]
# the scale of the planted keys' scores: q.u ~ ALPHA, scale 1/sqrt(128), log2(e) per natural unit
LOG2_PER_BETA = ALPHA / np.sqrt(128.0) * 1.4427


@pytest.mark.parametrize("Hq,Hkv", [(32, 8), (64, 8), (8, 8), (4, 2)])
@pytest.mark.parametrize("pt", [0, 64, 512])
def test_decode_unit_scale_on_normal_data(Hq, Hkv, pt):
    """scale = 1: scores ~ N(0, 128), the maximum keeps rising by many log2 units along a context."""
    w = decode_case(f"scale1_{Hq}_{Hkv}", 301, LENS_SMALL, Hq, Hkv)
    w.scale = 1.0
    check_decode(w, pt)


@pytest.mark.parametrize("kind", ["up", "down", "mixed"])
@pytest.mark.parametrize("gap_log2", [9.0, 45.0, 140.0])
@pytest.mark.parametrize("pt", [0, 64, 512])
def test_decode_planted_keys_along_the_query(kind, gap_log2, pt):
    """Planted keys whose scores differ by more than 8, 40 and 128 log2 units from one to the next."""
    w = decode_case(f"plant_{kind}_{gap_log2:g}", 302, LENS_SMALL, 32, 8)
    u = directions(w, 11)
    w.q = lean_queries(w.q, w, u)
    plant_profile(w, u, kind, gap_log2 / LOG2_PER_BETA * 1.6)   # 1.6: q.u may be as low as ALPHA - 3
    check_decode(w, pt)


@pytest.mark.parametrize("kind", ["up", "mixed"])
@pytest.mark.parametrize("pt", [0, 512])
def test_decode_planted_keys_at_the_benchmark_batch(kind, pt):
    """The same on the 64-sequence batch of the benchmark, where a wavefront's chunk spans tens of
    tiles and several sequences: rescales with long-lived accumulators, in whole-pair segments and
    in partials that the merge kernels then combine."""
    w = W.config2_llama8b()
    u = directions(w, 12)
    w.q = lean_queries(w.q, w, u)
    plant_profile(w, u, kind, 20.0 / LOG2_PER_BETA * 1.6, every=23)
    check_decode(w, pt)


@pytest.mark.parametrize("Hq,Hkv", [(32, 8), (8, 8)])
@pytest.mark.parametrize("pt", [0, 64])
def test_decode_one_key_takes_all_at_every_position(Hq, Hkv, pt):
    """Sequence i of 150-token contexts has its one dominant key at position i: first, middle and
    last token of every tile and chunk, and either side of every chunk boundary.  The output is
    that token's V row (also checked directly, without the oracle)."""
    n = 150
    w = decode_case(f"onehot_{Hq}_{Hkv}", 303, [n] * n, Hq, Hkv)
    u = directions(w, 13)
    w.q = lean_queries(w.q, w, u)
    for i in range(n):
        set_key(w, i, i, 400.0 * u)
    got = check_decode(w, pt)
    G = Hq // Hkv
    for i in range(n):
        v = f32(w.v_pool[w.block_tables[i, i // 16], :, i % 16, :]).astype(np.float64)   # [Hkv, D]
        assert np.abs(got[i] - np.repeat(v, G, axis=0)).max() <= TOL


@pytest.mark.parametrize("scale", [None, 1.0])
@pytest.mark.parametrize("pt", [0, 64])
def test_decode_constant_vector_added_to_every_key(scale, pt):
    """Every key shifted by 40 u: all scores of a head move together by tens (scale 1/sqrt(D)) or
    hundreds (scale 1) of units; only differences may matter."""
    w = decode_case("shift", 304, LENS_SMALL, 32, 8)
    u = directions(w, 14)
    w.q = lean_queries(w.q, w, u)
    for i, n in enumerate(w.context_lens.tolist()):
        for t in range(n):
            blk = w.block_tables[i, t // 16]
            w.k_pool[blk, :, t % 16, :] = bf16(f32(w.k_pool[blk, :, t % 16, :]) + 40.0 * u)
    if scale is not None:
        w.scale = scale
    check_decode(w, pt)


# --------------------------------------------------------------- 8-bit pools (the same kernel family)
def f8_case(name, seed, lens, Hq=32, Hkv=8):
    w = W.make_attn_workload(name, seed, dtype="f8", Hq=Hq, Hkv=Hkv, D=128, block_size=16, context_lens=lens,
                             pool_factor=1.15)
    w.k_scale = 64.0      # planted keys reach lengths of thousands; the stored codes stay below 448
    return w


@pytest.mark.parametrize("kind", ["up", "down", "mixed"])
@pytest.mark.parametrize("gap_log2", [9.0, 45.0])
@pytest.mark.parametrize("pt", [0, 64, 512])
def test_f8_decode_planted_keys_along_the_query(kind, gap_log2, pt):
    w = f8_case(f"f8_plant_{kind}_{gap_log2:g}", 322, [700, 1500, 333, 64, 2500, 17, 1, 2049])
    u = directions(w, 21)
    w.q = lean_queries(w.q, w, u)
    plant_profile(w, u, kind, gap_log2 / LOG2_PER_BETA * 1.6 * 1.2, every=29)   # 1.2: room for the 8-bit rounding of the keys
    check_decode(w, pt)


@pytest.mark.parametrize("pt", [0, 64])
def test_f8_decode_one_key_takes_all_at_every_position(pt):
    n = 150
    w = f8_case("f8_onehot", 323, [n] * n, Hq=8, Hkv=8)
    w.k_scale = 1.0       # (with the other keys 64 times longer the planted one would not always win)
    u = directions(w, 22)
    w.q = lean_queries(w.q, w, u)
    for i in range(n):
        set_key(w, i, i, 400.0 * u)
    got = check_decode(w, pt)
    import torch
    for i in range(n):
        codes = torch.from_numpy(np.ascontiguousarray(w.v_pool[w.block_tables[i, i // 16], :, i % 16, :]))
        v = codes.view(torch.float8_e4m3fn).to(torch.float64).numpy()
        assert np.abs(got[i] - v).max() <= TOL


@pytest.mark.parametrize("pt", [0, 512])
def test_f8_decode_unit_scale_and_benchmark_batch(pt):
    w = W.config2_llama8b_f8()
    w.scale = 1.0
    check_decode(w, pt)


# ------------------------------------------------------------------------------------- prefill
def prefill_case(seed, lens, Hq=8, Hkv=2):
    return W.make_attn_workload("prefill_rescale", seed, dtype="bf16", Hq=Hq, Hkv=Hkv, D=128, block_size=16,
                                context_lens=list(lens), pool_factor=1.2)


def check_prefill(w, query_lens, u=None, seed=5, split=False):
    """Queries are drawn inside run_prefill from `seed`; to lean them along u the same draw is
    repeated here and handed over."""
    hook = None
    if u is not None:
        hook = lambda q_bits: lean_queries(q_bits, w, u)
    got, ref = run_prefill(w, query_lens, seed, split=split, q_hook=hook)
    assert np.all(np.isfinite(got)), "non-finite output"
    err = np.abs(got - ref).max()
    print(f"prefill ctx={list(w.context_lens)} q={list(query_lens)} split={split}: max_abs_err={err:.3e}", flush=True)
    assert err <= TOL, err
    return got, ref


# unsplit: whole prompts and tails; split: one 512-token chunk over a long context (8 ranges)
PREFILL_SHAPES = [
    (False, (700, 300, 129, 33), (700, 300, 129, 33)),
    (False, (1500, 900), (256, 130)),
    (True, (2048,), (512,)),
    (True, (3000, 2500), (200, 256)),
]


@pytest.mark.parametrize("split,lens,qlens", PREFILL_SHAPES)
def test_prefill_unit_scale_on_normal_data(split, lens, qlens):
    w = prefill_case(311, lens)
    w.scale = 1.0
    check_prefill(w, qlens, split=split)


@pytest.mark.parametrize("kind", ["up", "down", "mixed"])
@pytest.mark.parametrize("gap_log2", [9.0, 45.0, 140.0])
@pytest.mark.parametrize("split,lens,qlens", PREFILL_SHAPES)
def test_prefill_planted_keys_along_the_query(kind, gap_log2, split, lens, qlens):
    w = prefill_case(312, lens)
    u = directions(w, 15)
    plant_profile(w, u, kind, gap_log2 / LOG2_PER_BETA * 1.6, every=37)
    check_prefill(w, qlens, u=u, split=split)


@pytest.mark.parametrize("split,lens,qlens", [
    (False, (300,) * 12, (300,) * 12),
    (True, (2048,) * 3, (160,) * 3),
])
def test_prefill_one_key_takes_all(split, lens, qlens):
    """One dominant key per sequence, at the first, a middle and the last token of a tile, of a
    pair of tiles and of a query group; queries before it see ordinary weights, those from it on
    return its V row."""
    w = prefill_case(313, lens)
    u = directions(w, 16)
    if split:
        spots = [2048 - 160, 2048 - 100, 1000]          # first query row, inside the chunk, far before it
    else:
        spots = [0, 15, 16, 31, 32, 33, 127, 128, 129, 255, 256, 299]
    for i, t in enumerate(spots):
        set_key(w, i, t, 400.0 * u)
    got, _ = check_prefill(w, qlens, u=u, split=split)
    G = w.Hq // w.Hkv
    row0 = 0
    for i, t in enumerate(spots):
        v = np.repeat(f32(w.v_pool[w.block_tables[i, t // 16], :, t % 16, :]).astype(np.float64), G, axis=0)
        first_pos = lens[i] - qlens[i]
        for j in range(qlens[i]):
            if first_pos + j >= t:
                assert np.abs(got[row0 + j] - v).max() <= TOL
        row0 += qlens[i]


@pytest.mark.parametrize("scale", [None, 1.0])
@pytest.mark.parametrize("split,lens,qlens", PREFILL_SHAPES[1:3])
def test_prefill_constant_vector_added_to_every_key(scale, split, lens, qlens):
    w = prefill_case(314, lens)
    u = directions(w, 17)
    for i, n in enumerate(w.context_lens.tolist()):
        for t in range(n):
            blk = w.block_tables[i, t // 16]
            w.k_pool[blk, :, t % 16, :] = bf16(f32(w.k_pool[blk, :, t % 16, :]) + 40.0 * u)
    if scale is not None:
        w.scale = scale
    check_prefill(w, qlens, u=u, split=split)
