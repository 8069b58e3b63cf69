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
// 0 .. (its last position)/16 once, two tiles (32 tokens, a "pair") per step: the wavefronts
// fetch the tiles together with direct-to-LDS loads (a quarter of K or of V each) into a ring
// of four pairs, and all of them consume the pairs from LDS; one barrier per pair orders the
// ring.  A wavefront skips the pairs that lie entirely in its future.
//
// Per pair, in the 32x32x16 shape (on this part the 16x16 shapes run at half the rate: 1.3
// against 2.3 PFLOP/s measured for back-to-back bf16 MFMAs):
//   S^T[token][query] = K Q^T   8 x v_mfma_f32_32x32x16_bf16 (32 tokens x 32 queries x 128 dims)
//   causal mask, base-2 softmax in fp32 relative to a lazily raised reference maximum: a lane
//   holds 16 tokens of one query, and that is already the A-operand layout of the second
//   product (k-step u = tile u of the pair), so the weights never move between lanes;
//   cross-lane traffic only when the reference maximum has to be raised
//   O[query][dim] += P V        2 x 2 x 4 x v_mfma_f32_32x32x16_bf16, P split into a bf16 head
//   and a bf16 remainder (exact to 2^-17), V through the transposing LDS read.
//
// Schedule.  Run one after the other, the three steps leave the matrix cores idle during the
// softmax, the vector ALU idle during the products, and both idle while LDS answers.  So the
// walk is software-pipelined inside a wavefront, in two phases per pair i:
//   phase 1: the exponentials and the bf16 split of pair i, two weights per slice, with one
//            MFMA of the first product of pair i+1 issued in front of each slice (its K rows
//            were read from LDS a phase earlier; the V rows of pair i are read meanwhile)
//   phase 2: the second product of pair i, interleaved with the scaling of the new scores
//            (and their causal mask); then the K rows of pair i+2 are read and the addresses
//            of the tiles to fetch next are formed, ahead of the barrier
// and the two wavefronts that share a SIMD run in opposite phases: the workgroup's barrier
// falls before phase 1 in wavefronts 0..3 and before phase 2 in wavefronts 4..7.  The ring
// holds four pairs for this: at barrier k the pairs up to k+2 are complete, pair k+3 is
// requested into the place of pair k-1, and the pairs k .. k+2 are being read.
//
// What bounds it (measured): instruction issue.  A pair costs a wavefront some 200
// instructions (24 MFMAs, 115 vector ALU, 26 LDS, the rest scalar), many in dependent chains,
// and a wavefront alone on its SIMD needs about 2000 cycles for them; the two per SIMD that
// the 225 registers allow overlap to about 2500 cycles for their two pairs, against 1536 of
// MFMA time.  Fetches and barriers cost 5 % on top.  A single-phase schedule (24 slices of
// one MFMA and a few ALU instructions) was no faster for a lone wavefront and, short of
// registers, slower for two.

#include <atomic>
#include <type_traits>

#include "pkv_internal.h"

namespace pkv {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;
typedef const void __attribute__((address_space(1)))* gptr_t;
typedef void __attribute__((address_space(3)))* lptr_t;

constexpr int D = 128;
constexpr int kQueryPerWave = 32;
constexpr int kTileBytes = 4096, kStageBytes = 2 * kTileBytes;
constexpr int kStages = 8;                 // K/V ring depth in tiles: four pairs
constexpr int kRingBytes = kStages * kStageBytes;
constexpr float kNoMaximum = -1.0e30f;     // reference maximum of a query that has seen no token yet
constexpr float kGrowLimit = 0x1p40f;       // a pair's weights relative to a stale reference maximum may sum to this
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
// A tile is fetched in eight quarter-tile shares of 1 KiB (four of K, four of V), one per
// wavefront.  (Workgroups of four wavefronts, two to a CU, each wavefront bringing two shares,
// were measured 8 % slower: the same work per SIMD, twice the fetches.)
constexpr int kWaves = 8, kThreads = kWaves * kWaveSize;
template <int HW>
__global__ __launch_bounds__(kThreads, 2) void attn_prefill_mfma_d128(const AttnParams p) {
  constexpr int NW = kWaves;
  constexpr int kShares = 8 / NW;                                   // quarter tiles per wavefront and tile
  constexpr int kGroupsPerHead = kWaves / HW;                       // 32-query groups per head
  constexpr int kQueryPerGroup = kGroupsPerHead * kQueryPerWave;    // query tokens per workgroup
  __shared__ __attribute__((aligned(16))) float xchg_all[kWaves][128];
  // dynamic LDS: the K/V ring, then the block table row of this sequence (ceil(max context /
  // block size) entries)
  extern __shared__ __attribute__((aligned(256))) uint8_t dyn_lds[];
  uint8_t* const ring = dyn_lds;
  int32_t* const ids_lds = reinterpret_cast<int32_t*>(dyn_lds + kRingBytes);

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
  // (3) With nsplit > 1 (few workgroups, long walks: chunked prefill of a few sequences) the walk
  // of a query group is cut into nsplit ranges of pairs, one workgroup each, side by side in
  // the numbering; they leave partial results that a second kernel merges.
  const int nsplit = p.max_partitions;
  const int nq = (int)(gridDim.x / 8) / (p.group_tiles * p.streams_per_xcd * nsplit);   // query groups per stream
  const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
  const int gtile = slot % p.group_tiles;
  const int qs = (slot / p.group_tiles) % (nq * nsplit);
  const int split = qs % nsplit;
  const int qgroup = nq - 1 - qs / nsplit;
  const int stream = (slot / (p.group_tiles * nq * nsplit)) * 8 + xcd;
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
  const int tiles_all = (pos0 + min(ql, q0 + kQueryPerGroup) - 1) / kTileTokens + 1;   // the group's whole walk
  // this workgroup's range of pairs [pr_lo, pr_hi) of it, and the tiles that end it
  const int pairs_all = (tiles_all + 1) / 2;
  const int pr_lo = (int)((int64_t)split * pairs_all / nsplit), pr_hi = (int)((int64_t)(split + 1) * pairs_all / nsplit);
  const int ntiles = min(tiles_all, 2 * pr_hi);
  const int wave_last_tile = wave_live ? (pos0 + min(ql, qw + kQueryPerWave) - 1) / kTileTokens : -1;

  // ---- per-lane offsets: same swizzled LDS images as the decode kernel -------------------------
  // fetch: share s < 4 is K rows 4s..4s+3 of a tile, share s >= 4 V rows 4(s-4)..+3;
  // K row t keeps its 16-byte piece c at slot c ^ t, V row t at slot c ^ 2(t mod 8)
  const uint32_t rbase = (uint32_t)(uintptr_t)(lptr_t)ring;   // LDS byte address of the ring
  uint32_t foff[kShares], fdst[kShares];
#pragma unroll
  for (int k = 0; k < kShares; ++k) {
    const int share = wave + k * NW;
    const int q4 = lane >> 4, t16 = lane & 15;
    const int frow = 4 * (share & 3) + q4;
    foff[k] = share >= 4 ? (uint32_t)(frow * p.v_stride_token) + (uint32_t)((t16 ^ (2 * (frow & 7))) * 16)
                         : (uint32_t)(frow * p.k_stride_token) + (uint32_t)((t16 ^ frow) * 16);
    fdst[k] = (uint32_t)((share >= 4 ? kTileBytes : 0) + (share & 3) * 1024);
  }
  // first product: this lane is token c32 of the pair (tile c32/16, row c32%16) and needs dims
  // 16s + 8hl .. +7 of its K row in step s, i.e. piece 2s + hl
  const int krow = c32 & 15;
  uint32_t krd[8];
#pragma unroll
  for (int s8 = 0; s8 < 8; ++s8)
    krd[s8] = (uint32_t)(krow * 256 + (((2 * s8 + hl) ^ krow) * 16)) + rbase + (c32 < 16 ? 0u : (uint32_t)kStageBytes);
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

  // A tile's fetch in two steps, so that the first can be done ahead of the barrier that frees
  // the tile's place in the ring: locate() forms the address of this wavefront's quarter
  // from the block id (wave-uniform, in scalar registers), request() starts the load.
  auto locate = [&](int j, int blk_id, int k) -> const uint8_t* {
    const int64_t blk = blk_id;
    const int slot0 = (j & tile_mask) * kTileTokens;
    return wave + k * NW >= 4 ? vpool + blk * p.v_stride_block + kvh * p.v_stride_head + slot0 * p.v_stride_token
                              : kpool + blk * p.k_stride_block + kvh * p.k_stride_head + slot0 * p.k_stride_token;
  };
  auto request = [&](int j, const uint8_t* base, int k) {
    // default cache policy: other workgroups (other query groups, other heads) read the same
    // tile again, so unlike in the decode kernel it should stay in L2
    __builtin_amdgcn_global_load_lds((gptr_t)(base + foff[k]),
                                     (lptr_t)(ring + (j & (kStages - 1)) * kStageBytes + fdst[k]), 16, 0, 0);
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
  float m_ref = 0.f, l_part = 0.f;
  f32x16 acc[4];
#pragma unroll
  for (int nb = 0; nb < 4; ++nb)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[nb][r] = 0.f;

  // All LDS reads are issued by hand.  The compiler would put a wait for every outstanding
  // direct-to-LDS load, i.e. for the pairs in flight, in front of reads it cannot tell apart
  // from the ring; and a read issued here is waited for later, by a counted s_waitcnt that
  // names the registers it completes (as in/out operands), so that nothing that uses them can
  // be moved in front of it.  LDS answers in order, which is what the counts rely on; scalar
  // loads the compiler may have in flight only make a counted wait longer.
#define PKV_PF_READ_K4(k0, k1, k2, k3, a0, a1, a2, a3)                                           \
  asm volatile("ds_read_b128 %0, %4\n\tds_read_b128 %1, %5\n\tds_read_b128 %2, %6\n\tds_read_b128 %3, %7" \
               : "=&v"(k0), "=&v"(k1), "=&v"(k2), "=&v"(k3)                                      \
               : "v"(a0), "v"(a1), "v"(a2), "v"(a3)                                              \
               : "memory")
#define PKV_PF_WAIT_K4(cnt, k0, k1, k2, k3) \
  asm volatile("s_waitcnt lgkmcnt(" #cnt ")" : "+v"(k0), "+v"(k1), "+v"(k2), "+v"(k3) : : "memory")
#define PKV_PF_READ_V8(vt, b0, b1)                                                               \
  do {                                                                                           \
    const uint32_t a0_ = (b0), a1_ = (b1), a2_ = a0_ ^ 64u, a3_ = a1_ ^ 64u, a4_ = a0_ ^ 128u,     \
                   a5_ = a1_ ^ 128u, a6_ = a0_ ^ 192u, a7_ = a1_ ^ 192u;                          \
    asm volatile(                                                                                \
        "ds_read_b64_tr_b16 %0, %8\n\tds_read_b64_tr_b16 %1, %9\n\t"                              \
        "ds_read_b64_tr_b16 %2, %10\n\tds_read_b64_tr_b16 %3, %11\n\t"                            \
        "ds_read_b64_tr_b16 %4, %12\n\tds_read_b64_tr_b16 %5, %13\n\t"                            \
        "ds_read_b64_tr_b16 %6, %14\n\tds_read_b64_tr_b16 %7, %15"                                \
        : "=&v"(vt[0]), "=&v"(vt[1]), "=&v"(vt[2]), "=&v"(vt[3]), "=&v"(vt[4]), "=&v"(vt[5]),     \
          "=&v"(vt[6]), "=&v"(vt[7])                                                             \
        : "v"(a0_), "v"(a1_), "v"(a2_), "v"(a3_), "v"(a4_), "v"(a5_), "v"(a6_), "v"(a7_)          \
        : "memory");                                                                             \
  } while (0)
#define PKV_PF_WAIT_V8(cnt, vt)                                                                  \
  asm volatile("s_waitcnt lgkmcnt(" #cnt ")"                                                     \
               : "+v"(vt[0]), "+v"(vt[1]), "+v"(vt[2]), "+v"(vt[3]), "+v"(vt[4]), "+v"(vt[5]),    \
                 "+v"(vt[6]), "+v"(vt[7])                                                        \
               : : "memory")

  // State carried from one pair to the next: the raw scores of the coming pair (q . k;
  // register r = token 8(r/4) + 4hl + r%4 of the pair, query c32) from phase 1 to phase 2, and
  // from phase 2 to the next phase 1 the same scaled, masked and taken relative to the reference
  // maximum (log2 units).
  f32x16 s_next;
  float d[16];
  uint32_t hi[8], lo[8];   // bf16 pairs (2i, 2i+1) of the weights: head and remainder
  u32x2 vta[8];            // V of the pair's first tile, B operands (read in phase 1, used in phase 2)

  // The first pair, not pipelined: its scores, and the reference maximum set to their true
  // maximum (position 0 is visible to every query, so it is finite).
  auto first_scores = [&]() {
    f32x16 sc;
#pragma unroll
    for (int r = 0; r < 16; ++r) sc[r] = 0.f;
#pragma unroll
    for (int half = 0; half < 2; ++half) {
      u32x4 f0, f1, f2, f3;
      const uint32_t so = (uint32_t)(((2 * pr_lo) & (kStages - 1)) * kStageBytes);
      const uint32_t a0 = krd[4 * half + 0] + so, a1 = krd[4 * half + 1] + so, a2 = krd[4 * half + 2] + so,
                     a3 = krd[4 * half + 3] + so;
      PKV_PF_READ_K4(f0, f1, f2, f3, a0, a1, a2, a3);
      PKV_PF_WAIT_K4(0, f0, f1, f2, f3);
      sc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, f0), qfrag[4 * half + 0], sc, 0, 0, 0);
      sc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, f1), qfrag[4 * half + 1], sc, 0, 0, 0);
      sc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, f2), qfrag[4 * half + 2], sc, 0, 0, 0);
      sc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, f3), qfrag[4 * half + 3], sc, 0, 0, 0);
    }
    // causal: a query sees positions <= its own (this also removes an absent second tile)
    const int kpos0 = 2 * pr_lo * kTileTokens + 4 * hl;
    float smax = -INFINITY;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      d[r] = kpos0 + 8 * (r / 4) + (r % 4) > qpos ? -INFINITY : sc[r] * p.scale_log2e;
      smax = fmaxf(smax, d[r]);
    }
    xchg[hl * 32 + c32] = smax;
    // (in a later range of a split walk a query may see nothing of the first pair, and then
    // nothing of the rest of the range either: the floor keeps its arithmetic finite, its
    // weights are all 0 and its normaliser stays 0, which the merge takes as "no part")
    m_ref = fmaxf(fmaxf(xchg[c32], xchg[32 + c32]), kNoMaximum);
#pragma unroll
    for (int r = 0; r < 16; ++r) d[r] -= m_ref;
  };

  // Phase 1 of pair i: weights of pair i from d[], raw scores of pair i+1 into s_next.  (The
  // scores of a pair that does not exist, or that this wavefront will not use, are computed
  // from whatever the ring holds and never looked at.)
  //
  // The reference maximum is lazy in the extreme: the weights are taken relative to m_ref as
  // it stands, without looking at the scores first, and only if their sum shows that a score
  // lies far above m_ref (or is not a number) is m_ref raised to the true maximum and the
  // pair's weights taken again.  A weight of 2^30 is as exact as one of 1 in fp32 and in
  // the bf16 split, so nothing is lost; with the first pair's true maximum as the start, the
  // second path is taken when a later score exceeds everything before it by some 2^35.
  uint32_t sel0 = 0x0000BF80u, sel1 = 0xBF800000u;       // bf16 pairs (-1, 0) and (0, -1)
  asm volatile("" : "+s"(sel0), "+s"(sel1));             // kept out of the instruction's constant field
  const bf16x2 minus_first = __builtin_bit_cast(bf16x2, sel0), minus_second = __builtin_bit_cast(bf16x2, sel1);
  // two weights p0, p1: bf16 head by a packed round-to-nearest conversion, bf16 remainder
  // p - head, exactly, by a dot product of the packed heads with (-1, 0) or (0, -1) added to p
  // (finite weights only: an infinite neighbour would turn 0 x inf into NaN)
#define PKV_PF_SPLIT(c, p0, p1)                                                                    \
    {                                                                                              \
      psum += (p0) + (p1);                                                                         \
      const bf16x2 h = __builtin_convertvector(f32x2{(p0), (p1)}, bf16x2);                         \
      const float r0 = __builtin_amdgcn_fdot2_f32_bf16(h, minus_first, (p0), false);               \
      const float r1 = __builtin_amdgcn_fdot2_f32_bf16(h, minus_second, (p1), false);              \
      hi[c] = __builtin_bit_cast(uint32_t, h);                                                     \
      lo[c] = __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2{r0, r1}, bf16x2));         \
    }
  // The K rows of pair i+1, as A operands, are read one phase ahead of phase 1 of pair i: at
  // the end of the previous pair's phase 2 (pair i+1 is complete in the ring by then).
  u32x4 k0, k1, k2, k3, k4, k5, k6, k7;
  auto read_next_k = [&](int i) {
    const uint32_t soff_n = (uint32_t)(((2 * i + 2) & (kStages - 1)) * kStageBytes);
    const uint32_t a0 = krd[0] + soff_n, a1 = krd[1] + soff_n, a2 = krd[2] + soff_n, a3 = krd[3] + soff_n;
    PKV_PF_READ_K4(k0, k1, k2, k3, a0, a1, a2, a3);
    const uint32_t a4 = krd[4] + soff_n, a5 = krd[5] + soff_n, a6 = krd[6] + soff_n, a7 = krd[7] + soff_n;
    PKV_PF_READ_K4(k4, k5, k6, k7, a4, a5, a6, a7);
  };
  auto phase1 = [&](int i) {
    const uint32_t soff_a = (uint32_t)(((2 * i) & (kStages - 1)) * kStageBytes);
    PKV_PF_WAIT_K4(4, k0, k1, k2, k3);   // K reads 4..7 may still be under way
    PKV_PF_READ_V8(vta, vrd[0] + soff_a, vrd[1] + soff_a);   // (never more than 15 reads under way: the counter's range)
    __builtin_amdgcn_sched_barrier(0);

#pragma unroll
    for (int r = 0; r < 16; ++r) s_next[r] = 0.f;
    float psum = 0.f;
    // one slice: an MFMA of the next scores, the exponentials of the following slice's two
    // weights and the split of this slice's two (two independent chains for the ALU to
    // alternate between); the scheduling barriers keep the slices apart
    float e0 = __builtin_amdgcn_exp2f(d[0]), e1 = __builtin_amdgcn_exp2f(d[1]);
#define PKV_PF_SLICE(c, kreg)                                                                      \
    {                                                                                              \
      s_next = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, kreg), qfrag[c], s_next, 0, 0, 0); \
      const float n0 = (c) < 7 ? __builtin_amdgcn_exp2f(d[((c) < 7 ? 2 * (c) + 2 : 0)]) : 0.f;      \
      const float n1 = (c) < 7 ? __builtin_amdgcn_exp2f(d[((c) < 7 ? 2 * (c) + 3 : 0)]) : 0.f;      \
      PKV_PF_SPLIT(c, e0, e1)                                                                      \
      e0 = n0; e1 = n1;                                                                            \
    }                                                                                              \
    __builtin_amdgcn_sched_barrier(0)
    PKV_PF_SLICE(0, k0);
    PKV_PF_SLICE(1, k1);
    PKV_PF_SLICE(2, k2);
    PKV_PF_SLICE(3, k3);
    PKV_PF_WAIT_K4(8, k4, k5, k6, k7);   // the eight V reads behind them may still be under way
    PKV_PF_SLICE(4, k4);
    PKV_PF_SLICE(5, k5);
    PKV_PF_SLICE(6, k6);
    PKV_PF_SLICE(7, k7);
#undef PKV_PF_SLICE
    if (__builtin_amdgcn_ballot_w64(!(psum < kGrowLimit)) != 0) {   // wave-uniform, rare after the first pair
      float smax = -INFINITY;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const float sv = d[r] + m_ref;                     // the scaled score again; masked stays -inf
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
      psum = 0.f;
#pragma unroll
      for (int c = 0; c < 8; ++c) {
        const float p0 = __builtin_amdgcn_exp2f(d[2 * c]), p1 = __builtin_amdgcn_exp2f(d[2 * c + 1]);
        PKV_PF_SPLIT(c, p0, p1)
      }
    }
    l_part += psum;
  };
#undef PKV_PF_SPLIT

  // Phase 2 of pair i: O += P V for its one or two tiles, and d[] of pair i+1.
  auto phase2 = [&](int i, bool have_b) {
    const uint32_t soff_b = (uint32_t)(((2 * i + 1) & (kStages - 1)) * kStageBytes);
    u32x2 vtb[8];
    PKV_PF_WAIT_V8(0, vta);
    if (have_b) PKV_PF_READ_V8(vtb, vrd[0] + soff_b, vrd[1] + soff_b);
    // rows past the context may hold NaN: zero them (only in the sequence's last tile)
    auto clear_rows_past_context = [&](u32x2* vt, int tile) {
      const int tpos = tile * kTileTokens + 4 * hl;       // position of the first token of read 0
      if ((tile + 1) * kTileTokens > n) {
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
    };
    clear_rows_past_context(vta, 2 * i);
    __builtin_amdgcn_sched_barrier(0);
    {
      // k-step u of the second product takes weight registers 8u .. 8u+7, which are exactly
      // this lane's tokens of tile u; the scaling of the next scores rides along
      const bf16x8 p_hi = __builtin_bit_cast(bf16x8, u32x4{hi[0], hi[1], hi[2], hi[3]});
      const bf16x8 p_lo = __builtin_bit_cast(bf16x8, u32x4{lo[0], lo[1], lo[2], lo[3]});
#pragma unroll
      for (int nb = 0; nb < 4; ++nb) {
        const bf16x8 vop = __builtin_bit_cast(bf16x8, u32x4{vta[2 * nb][0], vta[2 * nb][1], vta[2 * nb + 1][0], vta[2 * nb + 1][1]});
        acc[nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(p_hi, vop, acc[nb], 0, 0, 0);
#pragma unroll
        for (int r = 4 * nb; r < 4 * nb + 2; ++r) d[r] = fmaf(s_next[r], p.scale_log2e, -m_ref);
        __builtin_amdgcn_sched_barrier(0);
        acc[nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(p_lo, vop, acc[nb], 0, 0, 0);
#pragma unroll
        for (int r = 4 * nb + 2; r < 4 * nb + 4; ++r) d[r] = fmaf(s_next[r], p.scale_log2e, -m_ref);
        __builtin_amdgcn_sched_barrier(0);
      }
    }
    if (have_b) {
      PKV_PF_WAIT_V8(0, vtb);
      clear_rows_past_context(vtb, 2 * i + 1);
      const bf16x8 p_hi = __builtin_bit_cast(bf16x8, u32x4{hi[4], hi[5], hi[6], hi[7]});
      const bf16x8 p_lo = __builtin_bit_cast(bf16x8, u32x4{lo[4], lo[5], lo[6], lo[7]});
#pragma unroll
      for (int nb = 0; nb < 4; ++nb) {
        const bf16x8 vop = __builtin_bit_cast(bf16x8, u32x4{vtb[2 * nb][0], vtb[2 * nb][1], vtb[2 * nb + 1][0], vtb[2 * nb + 1][1]});
        acc[nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(p_hi, vop, acc[nb], 0, 0, 0);
        acc[nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(p_lo, vop, acc[nb], 0, 0, 0);
      }
    }
    // causal mask of the next pair (its scaling was done above)
    const int pr = i + 1;
    const int kpos0 = 2 * pr * kTileTokens + 4 * hl;
    if ((2 * pr + 2) * kTileTokens - 1 > pos0 + qw) {
#pragma unroll
      for (int r = 0; r < 16; ++r)
        if (kpos0 + 8 * (r / 4) + (r % 4) > qpos) d[r] = -INFINITY;
    }
  };

  // ---- walk the pairs ------------------------------------------------------------------------------
  const int npairs = pr_hi;                                     // the walk is pairs pr_lo .. pr_hi - 1
  // pairs this wavefront weighs: up to its own last one, within the workgroup's range
  const int np_wave = wave_live ? min(wave_last_tile / 2 + 1, pr_hi) : 0;
  // Barrier k.  Before it every wavefront waits for its own shares of the pairs requested so
  // far, so after it the pairs up to k+2 are complete; and every wavefront has finished
  // phase 2 of pair k-1, whose place pair k+3 takes: its two tiles were located ahead of the
  // barrier and are requested right behind it.  A bare s_barrier: what it orders is in LDS,
  // complete by the wait above (writes) and by data dependence (reads fed the matrix cores
  // before this point).
  const uint8_t* next_a[kShares];
  const uint8_t* next_b[kShares];
  auto locate_pair = [&](int pr) {
    if (2 * pr >= ntiles) return;
    // the block ids of both tiles with one LDS read: an aligned pair of table entries holds them
    // (tile 2pr is even, so with one tile per block they are entries 2pr and 2pr+1, else one entry)
    const int ia = (2 * pr) >> p.tpb_shift, ib = (2 * pr + 1) >> p.tpb_shift;
    u32x2 two;
    asm volatile("ds_read_b64 %0, %1\n\ts_waitcnt lgkmcnt(0)"
                 : "=v"(two) : "v"(ids_base + 4u * (uint32_t)(ia & ~1)) : "memory");
    const int e0 = __builtin_amdgcn_readfirstlane((int)two[0]), e1 = __builtin_amdgcn_readfirstlane((int)two[1]);
#pragma unroll
    for (int k = 0; k < kShares; ++k) {
      next_a[k] = locate(2 * pr, (ia & 1) ? e1 : e0, k);
      if (2 * pr + 1 < ntiles) next_b[k] = locate(2 * pr + 1, (ib & 1) ? e1 : e0, k);
    }
  };
  auto request_pair = [&](int pr) {
#pragma unroll
    for (int k = 0; k < kShares; ++k) {
      if (2 * pr < ntiles) request(2 * pr, next_a[k], k);
      if (2 * pr + 1 < ntiles) request(2 * pr + 1, next_b[k], k);
    }
  };
  auto barrier_and_fetch = [&](int k) {
    PKV_PF_WAIT_VMCNT(0);
    asm volatile("s_barrier" ::: "memory");
    request_pair(k + 3);
  };
  // the wavefront's phase against the barrier: of the two wavefronts of a SIMD the later runs shifted
  const bool shifted = wave >= kWaves / 2;

  if (pr_lo < pr_hi) {                           // (uniform over the workgroup)
    for (int pr = pr_lo; pr < pr_lo + 3; ++pr) {
      locate_pair(pr);
      request_pair(pr);
    }
    locate_pair(pr_lo + 3);
    PKV_PF_WAIT_VMCNT(0);
    asm volatile("s_barrier" ::: "memory");
  }
  if (np_wave > pr_lo) {
    first_scores();
    read_next_k(pr_lo);
  }
  for (int i = pr_lo; i < npairs; ++i) {
    if (!shifted) barrier_and_fetch(i);
    if (i < np_wave) phase1(i);
    if (shifted) barrier_and_fetch(i);
    if (i < np_wave) phase2(i, 2 * i + 1 < ntiles);
    locate_pair(i + 4);                       // (its wait also ends the reads of a last phase 2)
    if (i + 1 < np_wave) read_next_k(i + 1);
  }
#undef PKV_PF_READ_K4
#undef PKV_PF_WAIT_K4
#undef PKV_PF_READ_V8
#undef PKV_PF_WAIT_V8

  // ---- normalise and store ------------------------------------------------------------------------
  if (!wave_live) return;
  xchg[hl * 32 + c32] = l_part;
  const int64_t row0 = (int64_t)p.cu_query_lens[seq] + qw;
  if (nsplit > 1) {
    // partial result of this range: reference maximum and normaliser per query, and the
    // un-normalised output rows; a wavefront that had nothing in the range leaves normaliser 0
    const bool any = np_wave > pr_lo;
    if (hl == 0 && qw + c32 < ql) {
      float* ml = p.ws_ml + (((row0 + c32) * p.num_q_heads + head) * nsplit + split) * 2;
      ml[0] = any ? m_ref : kNoMaximum;
      ml[1] = any ? xchg[c32] + xchg[32 + c32] : 0.f;
    }
    if (!any) return;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int qq = 8 * k + 4 * hl + e;
        if (qw + qq < ql) {
          float* o = p.ws_o + (((row0 + qq) * p.num_q_heads + head) * nsplit + split) * D + c32;
#pragma unroll
          for (int nb = 0; nb < 4; ++nb) o[nb * 32] = acc[nb][4 * k + e];
        }
      }
    }
    return;
  }
#pragma unroll
  for (int k = 0; k < 4; ++k) {
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const int qq = 8 * k + 4 * hl + e;                 // query of accumulator register 4k + e
      if (qw + qq < ql) {
        const float inv = (1.0f / (xchg[qq] + xchg[32 + qq])) * p.v_scale;   // (the V factor of 8-bit pools, else 1)
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

// Merge of the ranges of a split walk: one wavefront per (query row, head), two output dims
// per lane.  out = sum_s O_s 2^(m_s - M) / sum_s l_s 2^(m_s - M) over the ranges that saw a token.
__global__ __launch_bounds__(256) void attn_prefill_merge(const AttnParams p) {
  const int nsplit = p.max_partitions;
  const int lane = threadIdx.x & (kWaveSize - 1);
  const int64_t item = (int64_t)blockIdx.x * (256 / kWaveSize) + threadIdx.x / kWaveSize;   // row * Hq + head
  const int64_t rows = p.cu_query_lens[p.batch];
  if (item >= rows * p.num_q_heads) return;
  {
    // Rows beyond min(query_lens, context_lens) of their sequence do not exist for the walk (a
    // query length above the context is clipped): nothing was written for them, and as in the
    // unsplit call their output rows are left alone.  The row's sequence is the last one whose
    // first row is not behind it.
    const int row = (int)(item / p.num_q_heads);
    int lo = 0, hi = p.batch;
    while (hi - lo > 1) {
      const int mid = (lo + hi) >> 1;
      if (p.cu_query_lens[mid] <= row) lo = mid; else hi = mid;
    }
    if (row - p.cu_query_lens[lo] >= min(p.query_lens[lo], p.context_lens[lo])) return;   // wave-uniform
  }
  const float* ml = p.ws_ml + item * nsplit * 2;
  float mx = kNoMaximum;
  for (int s = 0; s < nsplit; ++s)
    if (ml[2 * s + 1] > 0.f) mx = fmaxf(mx, ml[2 * s]);
  float l = 0.f, o0 = 0.f, o1 = 0.f;
  for (int s = 0; s < nsplit; ++s) {
    const float ls = ml[2 * s + 1];
    if (!(ls > 0.f)) continue;                       // nothing seen in this range (its rows were not written)
    const float w = __builtin_amdgcn_exp2f(ml[2 * s] - mx);
    const float2 o = *reinterpret_cast<const float2*>(p.ws_o + (item * nsplit + s) * D + 2 * lane);
    l += ls * w;
    o0 += o.x * w;
    o1 += o.y * w;
  }
  const float inv = (1.0f / l) * p.v_scale;
  if (p.out_is_bf16) reinterpret_cast<uint32_t*>(p.out)[item * (D / 2) + lane] = bf16x2_rne(o0 * inv, o1 * inv);
  else *reinterpret_cast<float2*>(reinterpret_cast<float*>(p.out) + item * D + 2 * lane) = float2{o0 * inv, o1 * inv};
}

}  // namespace

// Ranges a walk is cut into: 1 unless the unsplit grid would leave more than half of the CUs
// without a workgroup; then as many as fill them, of at least 8 pairs (256 tokens), at most 16.
int prefill_splits(const pkv_attn_desc& d, int max_query_len) {
  const int group = d.num_q_heads / d.num_kv_heads;
  const int hw = group == 1 ? 1 : 2;
  const int qpg = kWaves / hw * kQueryPerWave;
  const int64_t base = (int64_t)((max_query_len + qpg - 1) / qpg) * ((group + hw - 1) / hw) * d.num_kv_heads * d.batch;
  const int ncu = num_cus();
  if (base <= 0 || 2 * base > ncu) return 1;
  const int64_t max_pairs = ((int64_t)d.max_context_len + 2 * kTileTokens - 1) / (2 * kTileTokens);
  int64_t ns = ncu / base;
  if (ns > max_pairs / 8) ns = max_pairs / 8;
  if (ns > 16) ns = 16;
  return ns < 1 ? 1 : (int)ns;
}

size_t prefill_workspace_bytes(const pkv_attn_desc& d, int64_t total_query_tokens, int max_query_len) {
  const int ns = prefill_splits(d, max_query_len);
  if (ns <= 1 || total_query_tokens <= 0) return 0;
  return (size_t)total_query_tokens * d.num_q_heads * ns * (D + 2) * sizeof(float);
}

// bf16, head_dim 128, power-of-two block size / 16, block table row of the longest context in LDS
bool attn_prefill_supported(const pkv_attn_desc& d) {
  const int tpb = d.block_size / kTileTokens;
  const int64_t ids_bytes = ((int64_t)d.max_context_len + d.block_size - 1) / d.block_size * 4 + 16;
  return d.kv_dtype == PKV_BF16 && d.head_dim == 128 && tpb >= 1 && (tpb & (tpb - 1)) == 0 &&
         ids_bytes <= kMaxIdsBytes;
}

// More than 64 KiB of dynamic LDS: asked for once per device (every time outside the table).
hipError_t prepare_attn_prefill() {
  static std::atomic<bool> prepared[kMaxDevices];
  const int slot = device_slot();
  if (slot >= 0 && prepared[slot].load(std::memory_order_acquire)) return hipSuccess;
  for (const void* f : {reinterpret_cast<const void*>(&attn_prefill_mfma_d128<1>),
                        reinterpret_cast<const void*>(&attn_prefill_mfma_d128<2>)}) {
    const hipError_t e = hipFuncSetAttribute(f, hipFuncAttributeMaxDynamicSharedMemorySize, kRingBytes + kMaxIdsBytes);
    if (e != hipSuccess) return e;
  }
  if (slot >= 0) prepared[slot].store(true, std::memory_order_release);
  return hipSuccess;
}

// p.max_partitions = ranges per walk (1: results go to p.out; else partials to p.ws_ml /
// p.ws_o, [rows][Hq][ranges][2] and [rows][Hq][ranges][D] floats, and the merge follows);
// total_query_tokens bounds the rows (the merge reads the true count from cu_query_lens).
hipError_t launch_attn_prefill(AttnParams& p, int max_query_len, int max_context_len, int64_t total_query_tokens,
                               hipStream_t s) {
  p.tpb_shift = 0;
  while ((kTileTokens << p.tpb_shift) < p.block_size) ++p.tpb_shift;
  const int hw = p.group == 1 ? 1 : 2;                       // heads per workgroup
  p.group_tiles = (p.group + hw - 1) / hw;
  const size_t ids_bytes = (size_t)((max_context_len + p.block_size - 1) / p.block_size) * 4 + 16;
  const size_t lds_bytes = (size_t)kRingBytes + ids_bytes;
  const int qpg = kWaves / hw * kQueryPerWave;               // query tokens per workgroup
  p.streams_per_xcd = (p.num_kv_heads * p.batch + 7) / 8;
  if (p.max_partitions < 1) p.max_partitions = 1;
  const int64_t nwg = (int64_t)((max_query_len + qpg - 1) / qpg) * p.max_partitions * p.group_tiles * p.streams_per_xcd * 8;
  if (nwg > 0x7FFFFFFF) return hipErrorInvalidValue;
  const dim3 grid((unsigned)nwg);
  {
    const hipError_t e = prepare_attn_prefill();
    if (e != hipSuccess) return e;
  }
  if (hw == 1) hipLaunchKernelGGL((attn_prefill_mfma_d128<1>), grid, dim3(kThreads), lds_bytes, s, p);
  else hipLaunchKernelGGL((attn_prefill_mfma_d128<2>), grid, dim3(kThreads), lds_bytes, s, p);
  if (p.max_partitions > 1) {
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const int64_t items = total_query_tokens * p.num_q_heads;
    hipLaunchKernelGGL(attn_prefill_merge, dim3((unsigned)((items + 3) / 4)), dim3(256), 0, s, p);
  }
  return hipGetLastError();
}

}  // namespace pkv
