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
// Work split.  A workgroup of 8 wavefronts takes up to two query heads of one KV head and 128
// consecutive query tokens of one sequence per head (256 when the KV head has a single query
// head): each wavefront owns 32 tokens of one head.  The workgroup walks the K/V tiles
// 0 .. (its last position)/16 once, two tiles (32 tokens) per step: the wavefronts fetch the
// tiles together with direct-to-LDS loads (a quarter of K or of V each) into a ring of four
// tiles, the pair in use and the pair in flight, and all of them consume the pair from LDS; one
// barrier per pair orders the ring.  A wavefront skips the pairs that lie entirely in its
// future.
//
// Per pair of tiles, in the 32x32x16 shape (on this part the 16x16 shapes run at half the
// rate: 1.3 against 2.3 PFLOP/s measured for back-to-back bf16 MFMAs):
//   S^T[token][query] = K Q^T   8 x v_mfma_f32_32x32x16_bf16 (32 tokens x 32 queries x 128 dims)
//   causal mask, lazy-max base-2 softmax in fp32: a lane holds 16 tokens of one query, and that
//   is already the A-operand layout of the second product (k-step u = tile u of the pair), so
//   the weights never move between lanes; cross-lane traffic only when the reference maximum
//   has to be raised
//   O[query][dim] += P V        2 x 2 x 4 x v_mfma_f32_32x32x16_bf16, P split into a bf16 head
//   and a bf16 remainder (exact to 2^-17), V through the transposing LDS read.

#include <atomic>
#include <type_traits>

#include "pkv_internal.h"

namespace pkv {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;
typedef const void __attribute__((address_space(1)))* gptr_t;
typedef void __attribute__((address_space(3)))* lptr_t;

constexpr int D = 128;
constexpr int kThreads = 512, kWaves = kThreads / kWaveSize;   // one quarter tile (1 KiB) of K or V per wavefront
constexpr int kQueryPerWave = 32;
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

// HW = query heads per workgroup (1 or 2): wavefront w works on head (w / (8 / HW)) and on the
// 32 query tokens number (w % (8 / HW)) of the workgroup.
template <int HW>
__global__ __launch_bounds__(kThreads, 2) void attn_prefill_mfma_d128(const AttnParams p) {
  constexpr int kGroupsPerHead = kWaves / HW;                       // 32-query groups per head
  constexpr int kQueryPerGroup = kGroupsPerHead * kQueryPerWave;    // query tokens per workgroup
  __shared__ __attribute__((aligned(256))) uint8_t ring[kStages * kStageBytes];
  __shared__ __attribute__((aligned(16))) float xchg_all[kWaves][128];
  extern __shared__ int32_t ids_lds[];   // block table row of this sequence: ceil(max context / block size) entries

  const int tid = threadIdx.x;
  const int lane = tid & (kWaveSize - 1);
  const int wave = __builtin_amdgcn_readfirstlane(tid / kWaveSize);
  const int c32 = lane & 31;   // score layout: query token of the wavefront's 32; output layout: dim of a 32-block
  const int hl = lane >> 5;    // k-group of the operands; rows 4*hl + ... of the results

  // Workgroup numbering.  (1) The workgroups that walk the same K/V stream (sequence, KV head)
  // sit on one XCD, next to each other in launch order, so that the stream is fetched from HBM
  // about once and re-read from that XCD's L2: workgroups are dealt to the XCDs round-robin,
  // so stream st gets the ids congruent to st mod 8.  (2) Within a stream the query groups with
  // the most tiles to walk (the latest queries) come first and the short ones fill the gaps at
  // the end; in ascending order every round of workgroups lasts as long as its longest member.
  const int nq = (int)(gridDim.x / 8) / (p.group_tiles * p.streams_per_xcd);   // query groups per stream
  const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
  const int gtile = slot % p.group_tiles;
  const int qgroup = nq - 1 - (slot / p.group_tiles) % nq;
  const int stream = (slot / (p.group_tiles * nq)) * 8 + xcd;
  if (stream >= p.batch * p.num_kv_heads) return;      // padding of the last round of streams
  const int seq = stream / p.num_kv_heads, kvh = stream - seq * p.num_kv_heads;
  const int n = p.context_lens[seq];
  const int ql = min(p.query_lens[seq], n);
  const int q0 = qgroup * kQueryPerGroup;              // first query token of this workgroup
  if (ql <= 0 || q0 >= ql) return;                     // uniform over the workgroup
  const int pos0 = n - ql;                             // position of the chunk's first token
  const int hslot = wave / kGroupsPerHead;             // which of the workgroup's heads
  const int head = kvh * p.group + gtile * HW + hslot;
  const bool head_live = gtile * HW + hslot < p.group;

  const int qw = q0 + kQueryPerWave * (wave % kGroupsPerHead);   // first query token of this wavefront
  const bool wave_live = head_live && qw < ql;
  const int qi = qw + c32;                             // query token of this lane's column
  const bool col_live = qi < ql;
  const int qpos = pos0 + qi;
  const int ntiles = (pos0 + min(ql, q0 + kQueryPerGroup) - 1) / kTileTokens + 1;
  const int wave_last_tile = wave_live ? (pos0 + min(ql, qw + kQueryPerWave) - 1) / kTileTokens : -1;

  // ---- per-lane offsets: same swizzled LDS images as the decode kernel -------------------------
  // fetch: wavefront w < 4 brings K rows 4w..4w+3 of a tile, wavefront w >= 4 V rows 4(w-4)..+3;
  // K row t keeps its 16-byte piece c at slot c ^ t, V row t at slot c ^ 2(t mod 8)
  const uint32_t rbase = (uint32_t)(uintptr_t)(lptr_t)ring;   // LDS byte address of the ring
  uint32_t foff, fdst;
  {
    const int q4 = lane >> 4, t16 = lane & 15;
    const int frow = 4 * (wave & 3) + q4;
    foff = wave >= 4 ? (uint32_t)(frow * p.v_stride_token) + (uint32_t)((t16 ^ (2 * (frow & 7))) * 16)
                     : (uint32_t)(frow * p.k_stride_token) + (uint32_t)((t16 ^ frow) * 16);
    fdst = (uint32_t)((wave >= 4 ? kTileBytes : 0) + (wave & 3) * 1024);
  }
  // first product: this lane is token c32 of the pair (tile c32/16, row c32%16) and needs dims
  // 16s + 8hl .. +7 of its K row in step s, i.e. piece 2s + hl
  const int krow = c32 & 15;
  uint32_t krd[8];
#pragma unroll
  for (int s8 = 0; s8 < 8; ++s8) krd[s8] = (uint32_t)(krow * 256 + (((2 * s8 + hl) ^ krow) * 16)) + rbase;
  // second product, output dims 32nb .. 32nb+31: a 16-lane group g reads, for k-group hl = g/2
  // and dim half g%2, the tokens 4hl + s/4 (first read) and 8 + 4hl + s/4 (second read) at dims
  // 32nb + 16(g%2) + 4(s%4)..+3, s = lane within the group; the transposing read then leaves
  // every lane with four tokens of its own dim 32nb + c32 from each read
  uint32_t vrd[2];
  {
    const int g16 = lane >> 4, s16 = lane & 15;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const int tok = 4 * (g16 >> 1) + (s16 >> 2) + 8 * h;
      const int piece = 2 * (g16 & 1) + ((s16 & 3) >> 1);           // of dims 32nb.. for nb = 0
      vrd[h] = (uint32_t)(tok * 256 + ((piece ^ (2 * (tok & 7))) * 16) + (s16 & 1) * 8) + rbase + kTileBytes;
    }
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
    const uint8_t* base = wave >= 4 ? vpool + blk * p.v_stride_block + kvh * p.v_stride_head + slot0 * p.v_stride_token
                                    : kpool + blk * p.k_stride_block + kvh * p.k_stride_head + slot0 * p.k_stride_token;
    // default cache policy: other workgroups (other query groups, other heads) read the same
    // tile again, so unlike in the decode kernel it should stay in L2
    __builtin_amdgcn_global_load_lds((gptr_t)(base + foff),
                                     (lptr_t)(ring + (j & (kStages - 1)) * kStageBytes + fdst), 16, 0, 0);
  };

  // ---- query rows as the B operand: column c32 = query token qi, dims 16s + 8hl .. +7 in step s --
  bf16x8 qfrag[8];
  {
    const int64_t qrow = (int64_t)p.cu_query_lens[seq] + (col_live ? qi : q0);
    const uint8_t* qp = reinterpret_cast<const uint8_t*>(p.q) +
                        (qrow * p.num_q_heads + (head_live ? head : kvh * p.group)) * (D * 2) + hl * 16;
#pragma unroll
    for (int s8 = 0; s8 < 8; ++s8) {
      u32x4 v = *reinterpret_cast<const u32x4*>(qp + s8 * 32);
      if (!col_live) v = u32x4{0, 0, 0, 0};
      qfrag[s8] = __builtin_bit_cast(bf16x8, v);
    }
  }

  // softmax state of query column c32 (same value in the two lanes that share a column), and
  // O[query 8(r/4) + 4hl + r%4][dim 32nb + c32] in acc[nb][r]
  float m_ref = kNegBig, l_part = 0.f;
  f32x16 acc[4];
#pragma unroll
  for (int nb = 0; nb < 4; ++nb)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[nb][r] = 0.f;

  // Tiles j (A) and j+1 (B) of the ring; have_b is false for the odd tile at the end of the walk
  // (its tokens lie past every query of the workgroup, so the causal test masks them).
  auto consume = [&](int j, bool have_b) {
    const uint32_t soff_a = (uint32_t)((j & (kStages - 1)) * kStageBytes);
    const uint32_t soff_b = (uint32_t)(((j + 1) & (kStages - 1)) * kStageBytes);
    const uint32_t soff_k = c32 < 16 ? soff_a : soff_b;        // the tile of this lane's K row

    // All LDS reads are issued by hand: the compiler would put a wait for every outstanding
    // direct-to-LDS load, i.e. for the tiles in flight, in front of reads it cannot tell apart
    // from the ring.  The data is complete: the barrier before this call covered both tiles.
    f32x16 cfr;
#pragma unroll
    for (int r = 0; r < 16; ++r) cfr[r] = 0.f;
#pragma unroll
    for (int half = 0; half < 2; ++half) {
      u32x4 raw[4];
      const uint32_t a0 = krd[4 * half + 0] + soff_k, a1 = krd[4 * half + 1] + soff_k;
      const uint32_t a2 = krd[4 * half + 2] + soff_k, a3 = krd[4 * half + 3] + soff_k;
      asm volatile(
          "ds_read_b128 %0, %4\n\t"
          "ds_read_b128 %1, %5\n\t"
          "ds_read_b128 %2, %6\n\t"
          "ds_read_b128 %3, %7\n\t"
          "s_waitcnt lgkmcnt(0)"
          : "=&v"(raw[0]), "=&v"(raw[1]), "=&v"(raw[2]), "=&v"(raw[3])
          : "v"(a0), "v"(a1), "v"(a2), "v"(a3)
          : "memory");
#pragma unroll
      for (int i = 0; i < 4; ++i)
        cfr = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, raw[i]), qfrag[4 * half + i], cfr, 0, 0, 0);
    }
    // cfr[r] = q(query c32) . k(token tk(r) of the pair), tk(r) = 8(r/4) + 4hl + r%4;
    // d = score - reference in log2 units; causal: a query sees positions <= its own
    const int kpos0 = j * kTileTokens + 4 * hl;
    // (only a pair that reaches past the wavefront's first query needs the test: wave-uniform)
    const bool diagonal = (j + 2) * kTileTokens - 1 > pos0 + qw;
    float d[16];
#pragma unroll
    for (int r = 0; r < 16; ++r) d[r] = fmaf(cfr[r], p.scale_log2e, -m_ref);
    if (diagonal) {
#pragma unroll
      for (int r = 0; r < 16; ++r)
        if (kpos0 + 8 * (r / 4) + (r % 4) > qpos) d[r] = -INFINITY;
    }
    float dmax = d[0];
#pragma unroll
    for (int r = 1; r < 16; ++r) dmax = fmaxf(dmax, d[r]);
    if (__builtin_amdgcn_ballot_w64(dmax > kSlack) != 0) {   // wave-uniform, rare after the first tiles
      float smax = -INFINITY;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        float sv = cfr[r] * p.scale_log2e;
        if (diagonal && kpos0 + 8 * (r / 4) + (r % 4) > qpos) sv = -INFINITY;
        d[r] = sv;
        smax = fmaxf(smax, sv);
      }
      xchg[hl * 32 + c32] = smax;
      const float mn = fmaxf(m_ref, fmaxf(xchg[c32], xchg[32 + c32]));
      const float alpha = __builtin_amdgcn_exp2f(m_ref - mn);
      m_ref = mn;
      l_part *= alpha;
#pragma unroll
      for (int r = 0; r < 16; ++r) d[r] -= mn;
      xchg[64 + c32] = alpha;   // both lanes of a column write the same value
      // the accumulator rows of this lane are queries 8k + 4hl .. +3, k = 0..3
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        const f32x4 a = *reinterpret_cast<const f32x4*>(xchg + 64 + 8 * k + 4 * hl);
#pragma unroll
        for (int nb = 0; nb < 4; ++nb)
#pragma unroll
          for (int e = 0; e < 4; ++e) acc[nb][4 * k + e] *= a[e];
      }
    }
    // weights, split into a bf16 head (round to nearest) and a bf16 remainder, two values per
    // packed conversion; k-step u of the second product takes registers 8u .. 8u+7, which are
    // exactly this lane's tokens of tile u
    uint32_t hi[8], lo[8];   // pairs (2i, 2i+1)
    float psum = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const float p0 = __builtin_amdgcn_exp2f(d[2 * i]), p1 = __builtin_amdgcn_exp2f(d[2 * i + 1]);
      psum += p0 + p1;
      hi[i] = __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2{p0, p1}, bf16x2));
      const float r0 = p0 - __builtin_bit_cast(float, hi[i] << 16);
      const float r1 = p1 - __builtin_bit_cast(float, hi[i] & 0xFFFF0000u);
      lo[i] = __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2{r0, r1}, bf16x2));
    }
    l_part += psum;

#pragma unroll
    for (int u = 0; u < 2; ++u) {
      if (u == 1 && !have_b) break;                       // weights of the absent tile are zero
      const uint32_t soff = u == 0 ? soff_a : soff_b;
      const bf16x8 p_hi = __builtin_bit_cast(bf16x8, u32x4{hi[4 * u], hi[4 * u + 1], hi[4 * u + 2], hi[4 * u + 3]});
      const bf16x8 p_lo = __builtin_bit_cast(bf16x8, u32x4{lo[4 * u], lo[4 * u + 1], lo[4 * u + 2], lo[4 * u + 3]});
      // V of tile u as B operands: four tokens per read, two reads per 32 output dims
      u32x2 vt[8];
      {
        const uint32_t b0 = vrd[0] + soff, b1 = vrd[1] + soff;
        const uint32_t a0 = b0, a1 = b1, a2 = b0 ^ 64u, a3 = b1 ^ 64u, a4 = b0 ^ 128u, a5 = b1 ^ 128u,
                       a6 = b0 ^ 192u, a7 = b1 ^ 192u;
        asm volatile(
            "ds_read_b64_tr_b16 %0, %8\n\t"
            "ds_read_b64_tr_b16 %1, %9\n\t"
            "ds_read_b64_tr_b16 %2, %10\n\t"
            "ds_read_b64_tr_b16 %3, %11\n\t"
            "ds_read_b64_tr_b16 %4, %12\n\t"
            "ds_read_b64_tr_b16 %5, %13\n\t"
            "ds_read_b64_tr_b16 %6, %14\n\t"
            "ds_read_b64_tr_b16 %7, %15\n\t"
            "s_waitcnt lgkmcnt(0)"
            : "=&v"(vt[0]), "=&v"(vt[1]), "=&v"(vt[2]), "=&v"(vt[3]), "=&v"(vt[4]), "=&v"(vt[5]),
              "=&v"(vt[6]), "=&v"(vt[7])
            : "v"(a0), "v"(a1), "v"(a2), "v"(a3), "v"(a4), "v"(a5), "v"(a6), "v"(a7)
            : "memory");
      }
      const int tpos = (j + u) * kTileTokens + 4 * hl;    // position of the first token of read 0
      if ((j + u + 1) * kTileTokens > n) {                // rows past the context may hold NaN: zero them
        const uint32_t f0 = (tpos + 0 < n ? 0x0000FFFFu : 0u) | (tpos + 1 < n ? 0xFFFF0000u : 0u);
        const uint32_t f1 = (tpos + 2 < n ? 0x0000FFFFu : 0u) | (tpos + 3 < n ? 0xFFFF0000u : 0u);
        const uint32_t g0 = (tpos + 8 < n ? 0x0000FFFFu : 0u) | (tpos + 9 < n ? 0xFFFF0000u : 0u);
        const uint32_t g1 = (tpos + 10 < n ? 0x0000FFFFu : 0u) | (tpos + 11 < n ? 0xFFFF0000u : 0u);
#pragma unroll
        for (int nb = 0; nb < 4; ++nb) {
          vt[2 * nb][0] &= f0; vt[2 * nb][1] &= f1;
          vt[2 * nb + 1][0] &= g0; vt[2 * nb + 1][1] &= g1;
        }
      }
#pragma unroll
      for (int nb = 0; nb < 4; ++nb) {
        const bf16x8 vop = __builtin_bit_cast(bf16x8, u32x4{vt[2 * nb][0], vt[2 * nb][1], vt[2 * nb + 1][0], vt[2 * nb + 1][1]});
        acc[nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(p_hi, vop, acc[nb], 0, 0, 0);
        acc[nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(p_lo, vop, acc[nb], 0, 0, 0);
      }
    }
  };

  // ---- walk the tiles in pairs: the next pair is fetched while this one is consumed --------------
  issue(0);
  if (ntiles > 1) issue(1);
  for (int j = 0; j < ntiles; j += 2) {
    PKV_PF_WAIT_VMCNT(0);   // this wavefront's shares of tiles j and j+1 have landed
    // A bare barrier: what it orders is in LDS and complete by the wait above and by data
    // dependence (the LDS reads of the previous pair fed the matrix cores before this point).
    // After it every wavefront's share of the pair is there, and everybody is done with the
    // previous pair, whose two stages are refilled now.
    asm volatile("s_barrier" ::: "memory");
    if (j + 2 < ntiles) issue(j + 2);
    if (j + 3 < ntiles) issue(j + 3);
    if (j <= wave_last_tile) consume(j, j + 1 < ntiles);
  }

  // ---- normalise and store ------------------------------------------------------------------------
  if (!wave_live) return;
  xchg[hl * 32 + c32] = l_part;
  const int64_t row0 = (int64_t)p.cu_query_lens[seq] + qw;
#pragma unroll
  for (int k = 0; k < 4; ++k) {
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const int qq = 8 * k + 4 * hl + e;                 // query of accumulator register 4k + e
      if (qw + qq < ql) {
        const float inv = 1.0f / (xchg[qq] + xchg[32 + qq]);
        const int64_t o = ((row0 + qq) * p.num_q_heads + head) * D + c32;
#pragma unroll
        for (int nb = 0; nb < 4; ++nb) {
          const float v = acc[nb][4 * k + e] * inv;
          if (p.out_is_bf16) reinterpret_cast<uint16_t*>(p.out)[o + nb * 32] = (uint16_t)(bf16x2_rne(v, 0.f) & 0xFFFFu);
          else reinterpret_cast<float*>(p.out)[o + nb * 32] = v;
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
  const int hw = p.group == 1 ? 1 : 2;                       // heads per workgroup
  p.group_tiles = (p.group + hw - 1) / hw;
  const int qpg = kWaves / hw * kQueryPerWave;               // query tokens per workgroup
  p.streams_per_xcd = (p.num_kv_heads * p.batch + 7) / 8;
  const int64_t nwg = (int64_t)((max_query_len + qpg - 1) / qpg) * p.group_tiles * p.streams_per_xcd * 8;
  if (nwg > 0x7FFFFFFF) return hipErrorInvalidValue;
  const dim3 grid((unsigned)nwg);
  const size_t ids_bytes = (size_t)((max_context_len + p.block_size - 1) / p.block_size) * 4 + 16;
  static std::atomic<bool> prepared[kMaxDevices];   // static + dynamic LDS may exceed 64 KiB: ask once per device
  const int slot = current_device_slot();
  if (!prepared[slot].load(std::memory_order_acquire)) {
    for (const void* f : {reinterpret_cast<const void*>(&attn_prefill_mfma_d128<1>),
                          reinterpret_cast<const void*>(&attn_prefill_mfma_d128<2>)}) {
      const hipError_t e = hipFuncSetAttribute(f, hipFuncAttributeMaxDynamicSharedMemorySize, kMaxIdsBytes);
      if (e != hipSuccess) return e;
    }
    prepared[slot].store(true, std::memory_order_release);
  }
  if (hw == 1) hipLaunchKernelGGL((attn_prefill_mfma_d128<1>), grid, dim3(kThreads), ids_bytes, s, p);
  else hipLaunchKernelGGL((attn_prefill_mfma_d128<2>), grid, dim3(kThreads), ids_bytes, s, p);
  return hipGetLastError();
}

}  // namespace pkv
