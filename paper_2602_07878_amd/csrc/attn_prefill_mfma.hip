// Causal prefill attention of a chunk of query tokens over the paged KV cache, bf16 /
// head_dim 128, for gfx950.
//
// Operation (arXiv 2602.07878, Sec. 2.1: masked self-attention, a token attends to itself
// and to everything before it; Sec. 5.1.2 "Recomputation": a preempted request's prompt and
// generated tokens are prefilled again): for the last query_lens[i] tokens of sequence i,
// out[row] = softmax over positions s <= pos(row) of (scale q_row . K_s) V_s, with K and V
// found through the block table.  The chunk's own K/V are already in the pool.
//
// Unlike decode this is a dense contraction with reuse: a 16-token K/V tile serves every
// query row that may see it, so the matrix cores, not HBM, bound it.
//
// Work split.  A workgroup of 4 wavefronts takes 64 consecutive query tokens of one sequence
// and up to two query heads of one KV head; each wavefront owns 16 of those tokens.  Two such
// workgroups share a CU (8 wavefronts in one workgroup of 128 queries measured the same).  The workgroup walks the K/V tiles 0 .. (its last position)/16 once: the wavefronts
// fetch one tile together with direct-to-LDS loads (a quarter of K and a quarter of V
// each) into a ring of four tiles: the pair in use and the pair in flight, and all of them
// consume it from LDS; one barrier per pair orders the ring.  A wavefront skips the pairs
// that lie entirely in its future.
//
// Per pair of tiles and head (the decode kernel's tile code, with the 16 MFMA columns now
// holding 16 query tokens of one head instead of the heads of one token):
//   S^T[token][query] = K Q^T   2 x 4 x v_mfma_f32_16x16x32_bf16
//   causal mask, lazy-max base-2 softmax in fp32 (no cross-lane traffic unless the
//   reference maximum has to be raised)
//   O[query][dim] += P V        2 x 8 x v_mfma_f32_16x16x32_bf16 over the 32 tokens of the
//   pair, P split into a bf16 head and a bf16 remainder, V through the transposing LDS read.

#include <type_traits>

#include "pkv_internal.h"

namespace pkv {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;
typedef const void __attribute__((address_space(1)))* gptr_t;
typedef void __attribute__((address_space(3)))* lptr_t;

constexpr int D = 128;
#ifndef PKV_PREFILL_THREADS
#define PKV_PREFILL_THREADS 256
#endif
constexpr int kThreads = PKV_PREFILL_THREADS, kWaves = kThreads / kWaveSize;
constexpr int kFetches = 8 / kWaves;       // quarter tiles (1 KiB) a wavefront fetches per tile: K has 4, V has 4
static_assert(kWaves == 4 || kWaves == 8, "the eight quarter tiles are dealt to 4 or 8 wavefronts");
constexpr int kQueryPerWave = 16, kQueryPerGroup = kWaves * kQueryPerWave;
constexpr int kTileBytes = 4096, kStageBytes = 2 * kTileBytes;
constexpr int kStages = 4;                 // K/V ring depth: three tiles in flight behind the one in use
constexpr float kNegBig = -1.0e30f;
constexpr float kSlack = 8.0f;
constexpr int kMaxIdsBytes = 64 * 1024;     // LDS for one sequence's block table row: 16 Ki blocks

#define PKV_PF_WAIT_VMCNT(n) \
  __builtin_amdgcn_s_waitcnt(((n) & 0xF) | (((n) >> 4) << 14) | (0x7 << 4) | (0xF << 8))

__device__ __forceinline__ uint32_t bf16x2_rne(float lo, float hi) {
  auto cv = [](float f) -> uint32_t {
    uint32_t u = __builtin_bit_cast(uint32_t, f);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (u >> 16) | 0x40u;
    u += 0x7FFFu + ((u >> 16) & 1u);
    return u >> 16;
  };
  return cv(lo) | (cv(hi) << 16);
}

// NG = query heads per workgroup (1 or 2).
template <int NG>
__global__ __launch_bounds__(kThreads, 2) void attn_prefill_mfma_d128(const AttnParams p) {
  __shared__ __attribute__((aligned(256))) uint8_t ring[kStages * kStageBytes];
  __shared__ __attribute__((aligned(16))) float xchg_all[kWaves][128];
  extern __shared__ int32_t ids_lds[];   // block table row of this sequence: ceil(max context / block size) entries

  const int tid = threadIdx.x;
  const int lane = tid & (kWaveSize - 1);
  const int wave = __builtin_amdgcn_readfirstlane(tid / kWaveSize);
  const int t16 = lane & 15;   // score layout: query token of the wavefront's 16; V layout: dim
  const int q4 = lane >> 4;    // score layout: K tokens 4*q4..+3 of the tile

  // Workgroups are numbered so that the 128-query groups with the most K/V tiles to walk (the
  // latest queries) are dispatched first, across all sequences and heads, and the short ones
  // fill the gaps at the end; in launch order of (group, head, sequence) triples every round
  // of workgroups would last as long as its longest member.
  const int per_group = p.num_kv_heads * p.group_tiles * p.batch;
  const int qgroup = (int)(gridDim.x / per_group) - 1 - (int)(blockIdx.x / per_group);
  const int rest = blockIdx.x % per_group;
  const int pair = rest % (p.num_kv_heads * p.group_tiles);
  const int seq = rest / (p.num_kv_heads * p.group_tiles);
  const int n = p.context_lens[seq];
  const int ql = min(p.query_lens[seq], n);
  const int q0 = qgroup * kQueryPerGroup;              // first query token of this workgroup
  if (ql <= 0 || q0 >= ql) return;                     // uniform over the workgroup
  const int pos0 = n - ql;                             // position of the chunk's first token
  const int kvh = pair / p.group_tiles, gtile = pair - kvh * p.group_tiles;
  const int h0 = kvh * p.group + gtile * NG;
  const int nheads = min(NG, p.group - gtile * NG);

  const int qw = q0 + kQueryPerWave * wave;            // first query token of this wavefront
  const bool wave_live = qw < ql;
  const int qi = qw + t16;                             // query token of this lane's column
  const bool col_live = qi < ql;
  const int qpos = pos0 + qi;
  const int ntiles = (pos0 + min(ql, q0 + kQueryPerGroup) - 1) / kTileTokens + 1;
  const int wave_last_tile = wave_live ? (pos0 + min(ql, qw + kQueryPerWave) - 1) / kTileTokens : -1;

  // ---- per-lane offsets: same swizzled LDS images as the decode kernel -------------------------
  // fetch: quarter tile f (rows 4f..4f+3) of K for f < 4, of V (rows 4(f-4)..) for f >= 4; the
  // wavefronts share the eight quarters evenly
  uint32_t foff[kFetches], fdst[kFetches];
#pragma unroll
  for (int i = 0; i < kFetches; ++i) {
    const int f = wave * kFetches + i;
    const int frow = 4 * (f & 3) + q4;
    foff[i] = f >= 4 ? (uint32_t)(frow * p.v_stride_token) + (uint32_t)((t16 ^ (2 * (frow & 7))) * 16)
                     : (uint32_t)(frow * p.k_stride_token) + (uint32_t)((t16 ^ frow) * 16);
    fdst[i] = (uint32_t)((f >= 4 ? kTileBytes : 0) + (f & 3) * 1024);
  }
  uint32_t krd[4], vrd[8];
  const uint32_t rbase = (uint32_t)(uintptr_t)(lptr_t)ring;   // LDS byte address of the ring
#pragma unroll
  for (int j = 0; j < 4; ++j) krd[j] = (uint32_t)(t16 * 256 + (((4 * j + q4) ^ t16) * 16)) + rbase;
  {
    const int tv = 4 * q4 + (t16 >> 2);
    const uint32_t vbase = (uint32_t)(tv * 256 + ((tv & 7) << 5) + (t16 & 3) * 8);
#pragma unroll
    for (int nb = 0; nb < 8; ++nb) vrd[nb] = (vbase ^ (uint32_t)(nb << 5)) + rbase;
  }
  float* xchg = xchg_all[wave];
  const uint8_t* kpool = reinterpret_cast<const uint8_t*>(p.k_pool);
  const uint8_t* vpool = reinterpret_cast<const uint8_t*>(p.v_pool);
  const int tile_mask = (1 << p.tpb_shift) - 1;
  const int32_t* table = p.block_tables + (int64_t)seq * p.max_blocks_per_seq;

  // The sequence's block ids go to LDS once (a vector load inside the tile loop would make the
  // compiler wait for every fetch in flight before its value is used).
  {
    const int nblk = ((ntiles - 1) >> p.tpb_shift) + 1;
    for (int i = tid; i < nblk; i += kThreads) ids_lds[i] = table[i];
    __syncthreads();
  }
  const uint32_t ids_base = (uint32_t)(uintptr_t)(lptr_t)ids_lds;

  auto issue = [&](int j) {
    int blk_v;
    asm volatile("ds_read_b32 %0, %1\n\ts_waitcnt lgkmcnt(0)"
                 : "=v"(blk_v) : "v"(ids_base + 4u * (uint32_t)(j >> p.tpb_shift)) : "memory");
    const int64_t blk = __builtin_amdgcn_readfirstlane(blk_v);
    const int slot0 = (j & tile_mask) * kTileTokens;
    const uint8_t* kbase = kpool + blk * p.k_stride_block + kvh * p.k_stride_head + slot0 * p.k_stride_token;
    const uint8_t* vbase = vpool + blk * p.v_stride_block + kvh * p.v_stride_head + slot0 * p.v_stride_token;
    // default cache policy: other workgroups (other query groups, the other head pair) read the
    // same tile again, so unlike in the decode kernel it should stay in L2
#pragma unroll
    for (int i = 0; i < kFetches; ++i) {
      const bool is_v = wave * kFetches + i >= 4;   // wave-uniform
      __builtin_amdgcn_global_load_lds((gptr_t)((is_v ? vbase : kbase) + foff[i]),
                                       (lptr_t)(ring + (j & (kStages - 1)) * kStageBytes + fdst[i]), 16, 0, 0);
    }
  };

  // ---- query rows as B operands: column t16 = query token qi, one fragment set per head -------
  bf16x8 qfrag[NG][4];
  {
    const int64_t qrow = (int64_t)p.cu_query_lens[seq] + (col_live ? qi : q0);
#pragma unroll
    for (int g = 0; g < NG; ++g) {
      const uint8_t* qp = reinterpret_cast<const uint8_t*>(p.q) +
                          (qrow * p.num_q_heads + h0 + min(g, nheads - 1)) * (D * 2) + q4 * 16;
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        u32x4 v = *reinterpret_cast<const u32x4*>(qp + c * 64);
        if (!col_live) v = u32x4{0, 0, 0, 0};
        qfrag[g][c] = __builtin_bit_cast(bf16x8, v);
      }
    }
  }

  float m_ref[NG], l_part[NG];
  f32x4 acc[NG][8];
#pragma unroll
  for (int g = 0; g < NG; ++g) {
    m_ref[g] = kNegBig;
    l_part[g] = 0.f;
#pragma unroll
    for (int nb = 0; nb < 8; ++nb) acc[g][nb] = f32x4{0.f, 0.f, 0.f, 0.f};
  }

  // Two tiles (32 tokens) per step, so that P.V can use the 16x16x32 shape: of the eight
  // k-values a lane feeds, four are its tokens of tile A and four its tokens of tile B, for
  // the weights and for V alike.  have_b is false for the odd tile at the end of the walk.
  auto consume = [&](int j, bool have_b) {
    const uint32_t soff_a = (uint32_t)((j & (kStages - 1)) * kStageBytes);
    const uint32_t soff_b = (uint32_t)(((j + 1) & (kStages - 1)) * kStageBytes);
    const int kpos_a = j * kTileTokens + 4 * q4;         // position of this lane's first token of tile A
    const int kpos_b = kpos_a + kTileTokens;

    // All LDS reads are issued by hand: the compiler would put a wait for every outstanding
    // direct-to-LDS load, i.e. for the tiles in flight, in front of reads it cannot tell apart
    // from the ring.  The data is complete: the barrier before this call covered both tiles.
    auto read_k = [&](uint32_t soff, bf16x8* kf) {
      u32x4 raw[4];
      asm volatile(
          "ds_read_b128 %0, %4\n\t"
          "ds_read_b128 %1, %5\n\t"
          "ds_read_b128 %2, %6\n\t"
          "ds_read_b128 %3, %7\n\t"
          "s_waitcnt lgkmcnt(0)"
          : "=&v"(raw[0]), "=&v"(raw[1]), "=&v"(raw[2]), "=&v"(raw[3])
          : "v"(krd[0] + soff), "v"(krd[1] + soff), "v"(krd[2] + soff), "v"(krd[3] + soff)
          : "memory");
#pragma unroll
      for (int i = 0; i < 4; ++i) kf[i] = __builtin_bit_cast(bf16x8, raw[i]);
    };
    auto read_v = [&](uint32_t soff, u32x2* vt) {
      asm volatile(
          "ds_read_b64_tr_b16 %0, %8 offset:%16\n\t"
          "ds_read_b64_tr_b16 %1, %9 offset:%16\n\t"
          "ds_read_b64_tr_b16 %2, %10 offset:%16\n\t"
          "ds_read_b64_tr_b16 %3, %11 offset:%16\n\t"
          "ds_read_b64_tr_b16 %4, %12 offset:%16\n\t"
          "ds_read_b64_tr_b16 %5, %13 offset:%16\n\t"
          "ds_read_b64_tr_b16 %6, %14 offset:%16\n\t"
          "ds_read_b64_tr_b16 %7, %15 offset:%16\n\t"
          "s_waitcnt lgkmcnt(0)"
          : "=&v"(vt[0]), "=&v"(vt[1]), "=&v"(vt[2]), "=&v"(vt[3]), "=&v"(vt[4]), "=&v"(vt[5]),
            "=&v"(vt[6]), "=&v"(vt[7])
          : "v"(vrd[0] + soff), "v"(vrd[1] + soff), "v"(vrd[2] + soff), "v"(vrd[3] + soff),
            "v"(vrd[4] + soff), "v"(vrd[5] + soff), "v"(vrd[6] + soff), "v"(vrd[7] + soff), "n"(kTileBytes)
          : "memory");
    };

    // scores of both tiles, all heads: cfr[g][0] = tile A, cfr[g][1] = tile B
    f32x4 cfr[NG][2];
    {
      bf16x8 kf[4];
      read_k(soff_a, kf);
#pragma unroll
      for (int g = 0; g < NG; ++g) {
        cfr[g][0] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int jj = 0; jj < 4; ++jj)
          cfr[g][0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[jj], qfrag[g][jj], cfr[g][0], 0, 0, 0);
      }
      if (have_b) {
        read_k(soff_b, kf);
#pragma unroll
        for (int g = 0; g < NG; ++g) {
          cfr[g][1] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
          for (int jj = 0; jj < 4; ++jj)
            cfr[g][1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[jj], qfrag[g][jj], cfr[g][1], 0, 0, 0);
        }
      } else {
#pragma unroll
        for (int g = 0; g < NG; ++g) cfr[g][1] = f32x4{0.f, 0.f, 0.f, 0.f};
      }
    }

    // V of both tiles as one B operand per 16 output dims; rows past the context (they may
    // hold NaN) and the absent tile B are zero
    bf16x8 vop[8];
    {
      u32x2 va[8], vb[8];
      read_v(soff_a, va);
      if (have_b) {
        read_v(soff_b, vb);
      } else {
#pragma unroll
        for (int nb = 0; nb < 8; ++nb) vb[nb] = u32x2{0u, 0u};
      }
      if ((j + 2) * kTileTokens > n) {   // some row of the pair is past the context (wave-uniform)
        const uint32_t a0 = (kpos_a + 0 < n ? 0x0000FFFFu : 0u) | (kpos_a + 1 < n ? 0xFFFF0000u : 0u);
        const uint32_t a1 = (kpos_a + 2 < n ? 0x0000FFFFu : 0u) | (kpos_a + 3 < n ? 0xFFFF0000u : 0u);
        const uint32_t b0 = (kpos_b + 0 < n ? 0x0000FFFFu : 0u) | (kpos_b + 1 < n ? 0xFFFF0000u : 0u);
        const uint32_t b1 = (kpos_b + 2 < n ? 0x0000FFFFu : 0u) | (kpos_b + 3 < n ? 0xFFFF0000u : 0u);
#pragma unroll
        for (int nb = 0; nb < 8; ++nb) { va[nb][0] &= a0; va[nb][1] &= a1; vb[nb][0] &= b0; vb[nb][1] &= b1; }
      }
#pragma unroll
      for (int nb = 0; nb < 8; ++nb)
        vop[nb] = __builtin_bit_cast(bf16x8, u32x4{va[nb][0], va[nb][1], vb[nb][0], vb[nb][1]});
    }

#pragma unroll
    for (int g = 0; g < NG; ++g) {
      if (g < nheads) {
        // d = score - reference in log2 units; causal: a query sees positions <= its own
        float d[8];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          d[r] = fmaf(cfr[g][0][r], p.scale_log2e, -m_ref[g]);
          if (kpos_a + r > qpos) d[r] = -INFINITY;
          d[4 + r] = fmaf(cfr[g][1][r], p.scale_log2e, -m_ref[g]);
          if (kpos_b + r > qpos || !have_b) d[4 + r] = -INFINITY;
        }
        const float dmax = fmaxf(fmaxf(fmaxf(d[0], d[1]), fmaxf(d[2], d[3])), fmaxf(fmaxf(d[4], d[5]), fmaxf(d[6], d[7])));
        if (__builtin_amdgcn_ballot_w64(dmax > kSlack) != 0) {   // wave-uniform, rare after the first tiles
          float s[8];
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            s[r] = cfr[g][0][r] * p.scale_log2e;
            if (kpos_a + r > qpos) s[r] = -INFINITY;
            s[4 + r] = cfr[g][1][r] * p.scale_log2e;
            if (kpos_b + r > qpos || !have_b) s[4 + r] = -INFINITY;
          }
          xchg[q4 * 16 + t16] = fmaxf(fmaxf(fmaxf(s[0], s[1]), fmaxf(s[2], s[3])), fmaxf(fmaxf(s[4], s[5]), fmaxf(s[6], s[7])));
          const float tm = fmaxf(fmaxf(xchg[t16], xchg[16 + t16]), fmaxf(xchg[32 + t16], xchg[48 + t16]));
          const float mn = fmaxf(m_ref[g], tm);
          const float alpha = __builtin_amdgcn_exp2f(m_ref[g] - mn);
          m_ref[g] = mn;
          l_part[g] *= alpha;
#pragma unroll
          for (int r = 0; r < 8; ++r) d[r] = s[r] - mn;
          xchg[64 + t16] = alpha;   // accumulator rows of this lane are queries 4q4..4q4+3
          const f32x4 a = *reinterpret_cast<const f32x4*>(xchg + 64 + 4 * q4);
#pragma unroll
          for (int nb = 0; nb < 8; ++nb)
#pragma unroll
            for (int r = 0; r < 4; ++r) acc[g][nb][r] *= a[r];
        }
        // weights, split into a bf16 head and a rounded bf16 remainder
        uint32_t hi[8], lo[8];
        float psum = 0.f;
#pragma unroll
        for (int r = 0; r < 8; ++r) {
          const float pw = __builtin_amdgcn_exp2f(d[r]);
          psum += pw;
          hi[r] = __builtin_bit_cast(uint32_t, pw);
          const float rest = pw - __builtin_bit_cast(float, hi[r] & 0xFFFF0000u);
          lo[r] = __builtin_bit_cast(uint32_t, rest) + 0x8000u;
        }
        l_part[g] += psum;
        const bf16x8 p_hi = __builtin_bit_cast(bf16x8, u32x4{
            __builtin_amdgcn_perm(hi[1], hi[0], 0x07060302u), __builtin_amdgcn_perm(hi[3], hi[2], 0x07060302u),
            __builtin_amdgcn_perm(hi[5], hi[4], 0x07060302u), __builtin_amdgcn_perm(hi[7], hi[6], 0x07060302u)});
        const bf16x8 p_lo = __builtin_bit_cast(bf16x8, u32x4{
            __builtin_amdgcn_perm(lo[1], lo[0], 0x07060302u), __builtin_amdgcn_perm(lo[3], lo[2], 0x07060302u),
            __builtin_amdgcn_perm(lo[5], lo[4], 0x07060302u), __builtin_amdgcn_perm(lo[7], lo[6], 0x07060302u)});
#pragma unroll
        for (int nb = 0; nb < 8; ++nb)
          acc[g][nb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(p_hi, vop[nb], acc[g][nb], 0, 0, 0);
#pragma unroll
        for (int nb = 0; nb < 8; ++nb)
          acc[g][nb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(p_lo, vop[nb], acc[g][nb], 0, 0, 0);
      }
    }
  };

  // ---- walk the tiles in pairs: the next pair is fetched while this one is consumed --------------
  issue(0);
  if (ntiles > 1) issue(1);
  for (int j = 0; j < ntiles; j += 2) {
    PKV_PF_WAIT_VMCNT(0);   // this wavefront's shares of tiles j and j+1 have landed
    // A bare barrier: what it orders is in LDS and complete by the wait above and by data
    // dependence (the LDS reads of the previous pair fed the matrix cores before this point);
    // __syncthreads() could not be told apart from it here, but says more than is meant.  After
    // it every wavefront's share of the pair is there, and everybody is done with the previous
    // pair, whose two stages are refilled now.
    asm volatile("s_barrier" ::: "memory");
    if (j + 2 < ntiles) issue(j + 2);
    if (j + 3 < ntiles) issue(j + 3);
    if (j <= wave_last_tile) consume(j, j + 1 < ntiles);
  }

  // ---- normalise and store ------------------------------------------------------------------------
  if (!wave_live) return;
#pragma unroll
  for (int g = 0; g < NG; ++g) {
    if (g < nheads) {
      xchg[q4 * 16 + t16] = l_part[g];
      float inv[4];
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int c = 4 * q4 + r;
        inv[r] = 1.0f / ((xchg[c] + xchg[16 + c]) + (xchg[32 + c] + xchg[48 + c]));
      }
      const int64_t row0 = (int64_t)p.cu_query_lens[seq] + qw + 4 * q4;
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        if (qw + 4 * q4 + r < ql) {
          const int64_t o = ((row0 + r) * p.num_q_heads + h0 + g) * D + t16;
#pragma unroll
          for (int nb = 0; nb < 8; ++nb) {
            const float v = acc[g][nb][r] * inv[r];
            if (p.out_is_bf16) reinterpret_cast<uint16_t*>(p.out)[o + nb * 16] = (uint16_t)(bf16x2_rne(v, 0.f) & 0xFFFFu);
            else reinterpret_cast<float*>(p.out)[o + nb * 16] = v;
          }
        }
      }
    }
  }
}

}  // namespace

// bf16, head_dim 128, power-of-two block size / 16, block table row of the longest context in LDS
bool attn_prefill_supported(const pkv_attn_desc& d) {
  const int tpb = d.block_size / kTileTokens;
  const int64_t ids_bytes = ((int64_t)d.max_context_len + d.block_size - 1) / d.block_size * 4 + 16;
  return d.kv_dtype == PKV_BF16 && d.head_dim == 128 && tpb >= 1 && (tpb & (tpb - 1)) == 0 &&
         ids_bytes <= kMaxIdsBytes;
}

hipError_t launch_attn_prefill(AttnParams& p, int max_query_len, int max_context_len, hipStream_t s) {
  p.tpb_shift = 0;
  while ((kTileTokens << p.tpb_shift) < p.block_size) ++p.tpb_shift;
  const int ng = p.group == 1 ? 1 : 2;
  p.group_tiles = (p.group + ng - 1) / ng;
  const int64_t nwg = (int64_t)((max_query_len + kQueryPerGroup - 1) / kQueryPerGroup) * p.num_kv_heads *
                      p.group_tiles * p.batch;
  if (nwg > 0x7FFFFFFF) return hipErrorInvalidValue;
  const dim3 grid((unsigned)nwg);
  const size_t ids_bytes = (size_t)((max_context_len + p.block_size - 1) / p.block_size) * 4 + 16;
  static bool prepared = false;   // static + dynamic LDS may exceed 64 KiB: ask once
  if (!prepared) {
    for (const void* f : {reinterpret_cast<const void*>(&attn_prefill_mfma_d128<1>),
                          reinterpret_cast<const void*>(&attn_prefill_mfma_d128<2>)}) {
      const hipError_t e = hipFuncSetAttribute(f, hipFuncAttributeMaxDynamicSharedMemorySize, kMaxIdsBytes);
      if (e != hipSuccess) return e;
    }
    prepared = true;
  }
  if (ng == 1) hipLaunchKernelGGL((attn_prefill_mfma_d128<1>), grid, dim3(kThreads), ids_bytes, s, p);
  else hipLaunchKernelGGL((attn_prefill_mfma_d128<2>), grid, dim3(kThreads), ids_bytes, s, p);
  return hipGetLastError();
}

}  // namespace pkv
