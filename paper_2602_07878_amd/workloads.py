"""Seeded synthetic inputs for paged decode attention and KV-block swap.

This module is shared by the GPU path's callers and by the CPU oracle's
callers, so it holds no arithmetic of the method itself: it only draws random
numbers, lays them out in a paged pool and builds block tables / swap mappings.
It needs numpy only.

The paper (arXiv 2602.07878) measures on Alpaca / ShareGPT / BurstGPT traffic
(Sec. 6.1) driven into the "Fill" (KV cache nearly exhausted) and "Squeeze"
(repeated preemption) states (Sec. 5).  None of those records are used here;
the generators only mimic shapes, length mixes and pool occupancy:
  * context lengths: uniform, or a lognormal body of short benign requests
    plus a few very long ones (the long-output requests of Sec. 5.2);
  * pool occupancy 90-100 % with fully fragmented (permuted) block placement,
    the saturation band of Sec. 6.2;
  * swap mappings for a set of preemption victims (Sec. 5.1.2).

bfloat16 arrays are ``numpy.uint16`` holding the raw bit patterns.
"""
from __future__ import annotations

import math
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, field
from typing import Optional, Sequence

import numpy as np

_FILL_THREADS = 8
_FILL_CHUNK = 1 << 22  # elements drawn per task


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (nearest, ties to even); returns uint16 bits."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = (u + np.uint32(0x7FFF) + lsb) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Widen bfloat16 bit patterns to float32 (exact)."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32)
            << np.uint32(16)).view(np.float32)


def f32_to_f8e4m3_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to OCP E4M3 (1-4-3 bits, bias 7, no infinities; nearest, ties to even,
    saturating at the largest finite value 448); returns uint8 codes.  NaN becomes 0x7F."""
    a = np.ascontiguousarray(x, dtype=np.float32)
    mag = np.minimum(np.abs(np.nan_to_num(a, nan=0.0)), np.float32(448.0)).astype(np.float64)
    # below the smallest normal (2^-6) the grid is uniform with step 2^-9; above it each binade
    # [2^e, 2^(e+1)) has eight steps of 2^(e-3)
    e = np.floor(np.log2(np.maximum(mag, 2.0 ** -6)))
    step = 2.0 ** (e - 3)
    n = np.rint(mag / step)                       # multiples of the step; rint rounds half to even
    val = n * step                                # may have moved up into the next binade: still on the grid
    e2 = np.floor(np.log2(np.maximum(val, 2.0 ** -6)))
    sub = val < 2.0 ** -6
    mant = np.where(sub, np.rint(val * 2.0 ** 9), np.rint((val / 2.0 ** e2 - 1.0) * 8.0)).astype(np.int64)
    expo = np.where(sub, 0, e2.astype(np.int64) + 7)
    code = ((expo << 3) | mant).astype(np.uint8)
    code |= (np.signbit(a).astype(np.uint8) << np.uint8(7))
    code[np.isnan(a)] = 0x7F
    return code


def _normal_fill(out_flat: np.ndarray, seed_seq: np.random.SeedSequence, bf16: bool):
    """Fill a flat array with N(0,1) draws, chunked over threads, reproducibly."""
    n = out_flat.size
    nchunks = max(1, (n + _FILL_CHUNK - 1) // _FILL_CHUNK)
    children = seed_seq.spawn(nchunks)

    def work(c):
        lo, hi = c * _FILL_CHUNK, min(n, (c + 1) * _FILL_CHUNK)
        g = np.random.Generator(np.random.PCG64(children[c]))
        x = g.standard_normal(hi - lo, dtype=np.float32)
        if out_flat.dtype == np.uint8:
            out_flat[lo:hi] = f32_to_f8e4m3_bits(x)
        else:
            out_flat[lo:hi] = f32_to_bf16_bits(x) if bf16 else x

    if nchunks == 1:
        work(0)
    else:
        with ThreadPoolExecutor(_FILL_THREADS) as ex:
            list(ex.map(work, range(nchunks)))


def normal_array(shape, seed_seq, dtype: str) -> np.ndarray:
    """N(0,1) array; dtype 'f32' -> float32, 'bf16' -> uint16 bit patterns, 'f8' -> uint8 E4M3 codes."""
    bf16 = dtype == "bf16"
    a = np.empty(shape, dtype=np.uint8 if dtype == "f8" else np.uint16 if bf16 else np.float32)
    _normal_fill(a.reshape(-1), seed_seq, bf16)
    return a


def nan_bits(dtype: str):
    if dtype == "f8":
        return np.uint8(0x7F)
    return np.uint16(0x7FC0) if dtype == "bf16" else np.float32(np.nan)


@dataclass
class AttnWorkload:
    """One paged_decode_attention call's inputs (host arrays)."""
    name: str
    seed: int
    dtype: str                 # 'f32' | 'bf16' | 'f8' (bf16 q, 8-bit E4M3 pools)
    B: int
    Hq: int
    Hkv: int
    D: int
    block_size: int
    num_pool_blocks: int
    q: np.ndarray              # [B,Hq,D]
    k_pool: np.ndarray         # [num_pool_blocks,Hkv,bs,D]
    v_pool: np.ndarray
    block_tables: np.ndarray   # [B,max_blocks_per_seq] int32, unused entries -1
    context_lens: np.ndarray   # [B] int32
    scale: float
    partition_tokens: int = 0
    notes: dict = field(default_factory=dict)
    k_scale: float = 1.0       # 'f8' only: K = k_scale * stored value, V = v_scale * stored value
    v_scale: float = 1.0

    @property
    def elem_bytes(self) -> int:
        """Bytes of one cached K or V element."""
        return 1 if self.dtype == "f8" else 2 if self.dtype == "bf16" else 4

    @property
    def total_tokens(self) -> int:
        return int(self.context_lens.astype(np.int64).sum())

    @property
    def kv_bytes(self) -> int:
        """Bytes of K and V the definition reads: 2*Hkv*D*e per context token."""
        return 2 * self.Hkv * self.D * self.elem_bytes * self.total_tokens

    @property
    def max_context_len(self) -> int:
        return int(self.context_lens.max()) if self.B else 0


def blocks_needed(context_lens, block_size: int) -> np.ndarray:
    cl = np.asarray(context_lens, dtype=np.int64)
    return (cl + block_size - 1) // block_size


def make_attn_workload(name: str, seed: int, *, dtype: str, Hq: int, Hkv: int, D: int,
                       block_size: int, context_lens: Sequence[int],
                       num_pool_blocks: Optional[int] = None, pool_factor: float = 1.1,
                       scale: Optional[float] = None, poison: bool = True,
                       partition_tokens: int = 0, rng: Optional[np.random.Generator] = None
                       ) -> AttnWorkload:
    """Build pools, tables and queries for given context lengths.

    Owned blocks are the first `need` entries of a seeded permutation of all
    pool blocks (maximally fragmented placement), dealt to sequences in order.
    With `poison`, every element no defined read touches (free blocks, slots at
    or beyond the context length in a last block) is NaN and unused table
    entries are -1.
    """
    ss = np.random.SeedSequence(seed)
    s_perm, s_q, s_k, s_v = ss.spawn(4)
    cl = np.asarray(context_lens, dtype=np.int32)
    B = int(cl.size)
    nb = blocks_needed(cl, block_size)
    need = int(nb.sum())
    if num_pool_blocks is None:
        num_pool_blocks = max(1, int(math.ceil(pool_factor * need)))
    assert num_pool_blocks >= need, (num_pool_blocks, need)
    perm = np.random.Generator(np.random.PCG64(s_perm)).permutation(num_pool_blocks)
    max_blocks = max(1, int(nb.max()) if B else 1)
    bt = np.full((B, max_blocks), -1, dtype=np.int32)
    pos = 0
    for i in range(B):
        bt[i, :nb[i]] = perm[pos:pos + nb[i]]
        pos += int(nb[i])
    q = normal_array((B, Hq, D), s_q, "bf16" if dtype == "f8" else dtype)
    k_pool = normal_array((num_pool_blocks, Hkv, block_size, D), s_k, dtype)
    v_pool = normal_array((num_pool_blocks, Hkv, block_size, D), s_v, dtype)
    if poison:
        nanv = nan_bits(dtype)
        free = perm[need:]
        k_pool[free] = nanv
        v_pool[free] = nanv
        for i in range(B):
            r = int(cl[i]) % block_size
            if r:
                last = bt[i, nb[i] - 1]
                k_pool[last, :, r:, :] = nanv
                v_pool[last, :, r:, :] = nanv
    if scale is None:
        scale = float(np.float32(1.0 / math.sqrt(D)))
    return AttnWorkload(name=name, seed=seed, dtype=dtype, B=B, Hq=Hq, Hkv=Hkv, D=D,
                        block_size=block_size, num_pool_blocks=num_pool_blocks, q=q,
                        k_pool=k_pool, v_pool=v_pool, block_tables=bt, context_lens=cl,
                        scale=scale, partition_tokens=partition_tokens,
                        notes={"blocks_used": need,
                               "occupancy": need / num_pool_blocks})


# ---------------------------------------------------------------------------
# The five named configurations
# ---------------------------------------------------------------------------

def lens_tiny() -> np.ndarray:
    return np.array([17, 64, 100, 256], dtype=np.int32)


def lens_uniform(seed: int, B: int, lo: int, hi: int) -> np.ndarray:
    g = np.random.default_rng([seed, 7])
    return g.integers(lo, hi + 1, size=B).astype(np.int32)


def lens_fill_state(seed: int, B: int = 256, long_frac: float = 0.10) -> np.ndarray:
    """Short lognormal body (median 512, sigma 0.8, clamp [1,4096]) plus
    ceil(long_frac*B) long contexts uniform in [16384, 32768], shuffled."""
    g = np.random.default_rng([seed, 7])
    n_long = int(math.ceil(long_frac * B))
    n_short = B - n_long
    short = np.rint(g.lognormal(math.log(512.0), 0.8, size=n_short))
    short = np.clip(short, 1, 4096).astype(np.int32)
    long_ = g.integers(16384, 32768 + 1, size=n_long).astype(np.int32)
    allv = np.concatenate([short, long_])
    g.shuffle(allv)
    return allv


def config1_tiny(seed: int = 1001) -> AttnWorkload:
    return make_attn_workload("cfg1_tiny_f32", seed, dtype="f32", Hq=8, Hkv=8, D=64,
                              block_size=16, context_lens=lens_tiny(), num_pool_blocks=64)


def config2_llama8b(seed: int = 1002, B: int = 64, lo: int = 128, hi: int = 4096
                    ) -> AttnWorkload:
    return make_attn_workload("cfg2_llama3_8b_b64_bf16", seed, dtype="bf16", Hq=32, Hkv=8,
                              D=128, block_size=16,
                              context_lens=lens_uniform(seed, B, lo, hi), pool_factor=1.1)


def config2_llama8b_f8(seed: int = 1012, B: int = 64, lo: int = 128, hi: int = 4096) -> AttnWorkload:
    """The 8B-shaped decode batch with an 8-bit KV cache: half the bytes per cached token."""
    return make_attn_workload("cfg2_llama3_8b_b64_kv_f8e4m3", seed, dtype="f8", Hq=32, Hkv=8,
                              D=128, block_size=16,
                              context_lens=lens_uniform(seed, B, lo, hi), pool_factor=1.1)


def config3_fill(seed: int = 1003, B: int = 256) -> AttnWorkload:
    cl = lens_fill_state(seed, B)
    need = int(blocks_needed(cl, 16).sum())
    return make_attn_workload("cfg3_fill_b256_bf16", seed, dtype="bf16", Hq=32, Hkv=8,
                              D=128, block_size=16, context_lens=cl,
                              num_pool_blocks=int(math.ceil(need / 0.95)))


def config5_long70b(seed: int = 1005, B: int = 16, lo: int = 32768, hi: int = 131072
                    ) -> AttnWorkload:
    return make_attn_workload("cfg5_long_70b_b16_bf16", seed, dtype="bf16", Hq=64, Hkv=8,
                              D=128, block_size=16,
                              context_lens=lens_uniform(seed, B, lo, hi), pool_factor=1.1,
                              partition_tokens=512)


@dataclass
class SwapWorkload:
    """Preemption churn: gather victims' blocks to staging, scatter to new blocks."""
    name: str
    seed: int
    num_planes: int
    block_bytes: int
    num_pool_blocks: int
    victim_lens: np.ndarray        # [V] int32 tokens
    src_blocks: np.ndarray         # [n] pool blocks owned by the victims, in logical order
    new_blocks: np.ndarray         # [n] pool blocks they get on resume
    gather_mapping: np.ndarray     # [n,2] (pool block, staging slot)
    scatter_mapping: np.ndarray    # [n,2] (staging slot, new pool block)

    @property
    def n_blocks(self) -> int:
        return int(self.src_blocks.size)

    @property
    def payload_bytes(self) -> int:
        return self.n_blocks * self.num_planes * self.block_bytes

    @property
    def pool_bytes(self) -> int:
        return self.num_planes * self.num_pool_blocks * self.block_bytes

    @property
    def staging_bytes(self) -> int:
        return self.payload_bytes


def make_swap_workload(name: str, seed: int, *, victim_lens: Sequence[int], num_planes: int,
                       block_bytes: int, block_size: int = 16, pool_factor: float = 1.25
                       ) -> SwapWorkload:
    g = np.random.default_rng([seed, 11])
    vl = np.asarray(victim_lens, dtype=np.int32)
    n = int(blocks_needed(vl, block_size).sum())
    num_pool_blocks = max(1, int(math.ceil(pool_factor * n)))
    src = g.permutation(num_pool_blocks)[:n].astype(np.int32)
    new = g.permutation(num_pool_blocks)[:n].astype(np.int32)   # fresh, independent placement
    slots = np.arange(n, dtype=np.int32)
    return SwapWorkload(name=name, seed=seed, num_planes=num_planes, block_bytes=block_bytes,
                        num_pool_blocks=num_pool_blocks, victim_lens=vl, src_blocks=src,
                        new_blocks=new,
                        gather_mapping=np.stack([src, slots], axis=1).astype(np.int32),
                        scatter_mapping=np.stack([slots, new], axis=1).astype(np.int32))


def config4_squeeze(seed: int = 1004, victims: int = 64, lo: int = 512, hi: int = 4096,
                    num_planes: int = 64) -> SwapWorkload:
    """64 victims, int-uniform [512,4096] tokens (realised mean is what it is),
    32 layers x {K,V} planes, 8 KV heads x 128 dims x bf16 x 16 tokens = 32 KiB blocks."""
    return make_swap_workload("cfg4_squeeze_swap64", seed,
                              victim_lens=lens_uniform(seed, victims, lo, hi),
                              num_planes=num_planes, block_bytes=16 * 8 * 128 * 2)


def config4_squeeze_f8(seed: int = 1004, victims: int = 64, lo: int = 512, hi: int = 4096,
                       num_planes: int = 64) -> SwapWorkload:
    """The same victims with 8-bit (E4M3) pools: one byte per element, 16 KiB blocks."""
    return make_swap_workload("cfg4_squeeze_swap64_f8", seed,
                              victim_lens=lens_uniform(seed, victims, lo, hi),
                              num_planes=num_planes, block_bytes=16 * 8 * 128)


def config4_evict_all_256(seed: int = 1003, num_planes: int = 64) -> SwapWorkload:
    """Swap-out of all 256 sequences of the Fill-state length mix (the metric's
    'at batch 256' wording)."""
    return make_swap_workload("cfg4b_evict_all_b256", seed, victim_lens=lens_fill_state(seed),
                              num_planes=num_planes, block_bytes=16 * 8 * 128 * 2,
                              pool_factor=1.0 / 0.95)


def random_bytes(nbytes: int, seed: int) -> np.ndarray:
    """Seeded uniform random bytes (uint8), drawn in threads, reproducible."""
    assert nbytes % 8 == 0
    out = np.empty(nbytes // 8, dtype=np.uint64)
    n = out.size
    chunk = 1 << 24
    nchunks = max(1, (n + chunk - 1) // chunk)
    children = np.random.SeedSequence([seed, 13]).spawn(nchunks)

    def work(c):
        lo, hi = c * chunk, min(n, (c + 1) * chunk)
        gen = np.random.Generator(np.random.PCG64(children[c]))
        out[lo:hi] = gen.integers(0, 2**64 - 1, size=hi - lo, dtype=np.uint64, endpoint=True)

    if nchunks == 1:
        work(0)
    else:
        with ThreadPoolExecutor(_FILL_THREADS) as ex:
            list(ex.map(work, range(nchunks)))
    return out.view(np.uint8)


# --------------------------------------------------------------------------- request streams
def poisson_request_stream(seed: int, steps: int, rate: float, *, prompt_median: int = 256,
                           prompt_sigma: float = 0.8, out_median: int = 128, out_sigma: float = 0.7,
                           max_prompt: int = 2048, max_new: int = 1024):
    """Benign open-loop load for the scheduler model: per engine iteration a Poisson(rate)
    number of requests arrives, with lognormal prompt and output lengths (clamped).  Returns a
    list, one entry per iteration, of lists of (request id, prompt_len, max_new_tokens).
    Stands in for the chat traces the paper replays (Sec. 6.1); no dataset record is used."""
    rng = np.random.default_rng(seed)
    out, rid = [], 0
    for _ in range(steps):
        arrivals = []
        for _ in range(int(rng.poisson(rate))):
            p = int(np.clip(round(float(rng.lognormal(math.log(prompt_median), prompt_sigma))), 1, max_prompt))
            n = int(np.clip(round(float(rng.lognormal(math.log(out_median), out_sigma))), 1, max_new))
            arrivals.append((rid, p, n))
            rid += 1
        out.append(arrivals)
    return out
