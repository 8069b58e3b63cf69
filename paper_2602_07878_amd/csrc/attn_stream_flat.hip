// Paged decode attention, head_dim 128: the K/V-streaming kernel with a flat tile loop, for gfx950.
//
// Operation (arXiv 2602.07878, Sec. 2.2 "KV-Cache", Sec. 4.2): out = softmax_t(scale q.K_t) V over
// the tokens found through the block table.  Same decomposition as attn_stream_mfma.hip (all
// 16-token tiles of the call on one axis, cut into workgroup ranges and wavefront chunks; a chunk
// ends its (sequence, pair) segments in finished rows or (m, l, O) partials that the merge
// kernels combine), same per-tile arithmetic on the matrix cores.  Two things are different here.
//
// 1. The tile loop is flat.  A tile descriptor says whether the tile opens or closes a
//    (sequence, pair); descriptors of coming batches sit in a ring of tables in LDS; a consumer
//    cursor, a fetch cursor a few tiles ahead of it and a builder cursor ahead of both walk the
//    same sequence of batches.  Chunk boundaries, batch boundaries and segments need no nested
//    loops, and the lookahead crosses all of them.
//
// 2. What it serves.
//    * 8-bit (OCP E4M3) K/V pools beside a bfloat16 query: half the bytes per cached token (Sec.
//      4.2: the time model charges sizeof(T) per cached element).  Every E4M3 value is a bfloat16
//      value, so a tile is decoded exactly into bf16 LDS images (hardware conversion, two codes
//      per instruction) and from there on the arithmetic is that of the bf16 kernel.  A tile is
//      2 KiB per pool, so four tiles per wavefront are kept in flight, in registers.
//    * Calls that come with a per-step plan (pkv_attn_plan: Sec. 4.2, one attention call per layer
//      and step, all of them over the same block tables and lengths).  The plan holds what every
//      layer call would otherwise recompute (tile count, per-tile descriptors, the directory of
//      partials): no prefix sums, no bisections, no table walk in the call itself.
//      bf16 pools take direct-to-LDS loads into a ring of two stages as in attn_stream_mfma.hip.
//
// Every global load of the tile loop is issued and waited for by hand (the query rows are
// loaded only where a segment opens; waits placed by the compiler for them would also wait, on
// every path, for the tiles in flight).  Loads return in order, so a wait that leaves the n
// youngest outstanding completes everything older.
//
// Registers that data is on its way to for longer than one statement are not the compiler's.  A
// value the compiler manages may be moved to another register at any join of control flow, and
// a register moved while its load is in flight takes along whatever was there before (seen: a
// query fetched ahead, copied, and the abandoned register reused for an address that the
// arriving data then overwrote).  So the kernels are compiled with a register budget that ends
// below v174 (8-bit pools) or v234 (bf16 pools), and the statements here name the registers
// above it themselves: v174..v237 take the tile bytes of the four sets in flight (8-bit pools),
// v234..v237 (bf16 pools) or v170..v173 (8-bit pools with a plan) the new token's rows of a call
// that also appends, v238..v253 the query rows fetched ahead.  Their contents enter the compiler's world only through statements
// that run after the wait that completes them.

#include <atomic>
#include <type_traits>

#include <hip/hip_ext.h>

#include "attn_stream_common.h"

namespace pkv {
namespace {

constexpr int kImageBytes = 2 * kTileBytes;     // a bf16 K image, then a bf16 V image (one ring stage)

template <bool KV8> struct FlatGeom;
template <> struct FlatGeom<true> {             // 8-bit pools: four register sets in flight, one pair of images
  static constexpr int kSets = 4, kBatch = 64, kDataBytes = kImageBytes;
};
template <> struct FlatGeom<false> {            // bf16 pools: a ring of two stages filled by direct-to-LDS loads
  static constexpr int kSets = 2, kBatch = 32, kDataBytes = 2 * kImageBytes;
};
// Descriptor tables per wavefront: the batch being consumed, those the fetch cursor can reach
// (it runs at most kSets tiles ahead, and a batch can be as short as one tile), and one more.
template <bool KV8> constexpr int flat_tables() { return FlatGeom<KV8>::kSets + 2; }
// per wavefront: images, exchange area, descriptor tables, one record of 8 words per table
template <bool KV8>
constexpr int flat_wave_lds() {
  return FlatGeom<KV8>::kDataBytes + kXchgBytes + flat_tables<KV8>() * (FlatGeom<KV8>::kBatch * 16 + 32);
}

// The chunk the builder is in: what the next batch of descriptors is cut from.
struct ChunkCursor {
  int ci;         // local id of the chunk
  int c;          // chunk id on the whole axis: orders the partial slots
  int x0;         // axis position of the chunk's first tile
  int ntc;        // tiles of the chunk
  int b0;         // tiles of the chunk already described
};

// GH = query heads accumulated per lane (1, 2, 4 or 8); KV8: the pools hold E4M3 codes; PLANNED:
// the call brings a plan.
template <int GH, bool KV8, bool PLANNED>
__device__ __forceinline__ void flat_body(const AttnParams& p) {
  // (the one place that tells the compiler about them: the kernel's register allocation must
  // reach up to v253; the compiler remarks that v253 is outside its budget, which is the point)
  asm volatile("" ::: "v253");
  using G = FlatGeom<KV8>;
  constexpr bool APPEND = PLANNED;              // the call may also append (see row_for below)
  constexpr int kSets = G::kSets, BT = G::kBatch, kTables = flat_tables<KV8>();
  constexpr int kWaveBytes = flat_wave_lds<KV8>();
  extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
  __shared__ int wave_total[kNW];
  __shared__ int progress[kNW];   // tiles consumed so far, per wavefront

  const int tid = threadIdx.x;
  const int lane = tid & (kWaveSize - 1);
  const int wave = rfl(tid / kWaveSize);
  const int t16 = lane & 15;   // score layout: token of the tile; V layout: 16-byte piece
  const int q4 = lane >> 4;    // score layout: head slots 4*q4..+3; V layout: row of a load
  const int B = p.batch;
  const int NP = p.num_kv_heads * p.group_tiles;   // (KV head, head sub-group) pairs per sequence

  // ---- set-up -------------------------------------------------------------------------------------
  int* prefix = reinterpret_cast<int*>(lds);       // [B + 1], calls without a plan only
  int T;                                           // tiles of the whole call
  if (tid < kNW) progress[tid] = 0;
  if constexpr (PLANNED) {
    const i32x2 hdr = *reinterpret_cast<const i32x2*>(p.plan_hdr);    // (kPlanT, kPlanKey)
    if (hdr[1] != p.plan_key) return;              // not a plan for this call: the merge kernel reports it
    T = rfl(hdr[0]);
    __syncthreads();                               // progress[] is cleared
  } else {
    // exclusive prefix sums of per-sequence tile counts, in LDS
    const int per = (B + kStreamThreads - 1) / kStreamThreads;
    const int i0 = tid * per, i1 = min(B, i0 + per);
    int sum = 0;
    for (int i = i0; i < i1; ++i) sum += (max(p.context_lens[i], 0) + kTileTokens - 1) / kTileTokens;
    int v = sum;
#pragma unroll
    for (int off = 1; off < kWaveSize; off <<= 1) {
      const int t = __shfl_up(v, off, kWaveSize);
      if (lane >= off) v += t;
    }
    if (lane == kWaveSize - 1) wave_total[wave] = v;
    __syncthreads();
    int run = v - sum;
    for (int w = 0; w < wave; ++w) run += wave_total[w];
    if (tid == 0) prefix[0] = 0;
    for (int i = i0; i < i1; ++i) {
      run += (max(p.context_lens[i], 0) + kTileTokens - 1) / kTileTokens;
      prefix[i + 1] = run;
    }
    __syncthreads();
    T = rfl(prefix[B]) * NP;
  }
  if (T == 0) return;

  const ChunkPlan plan = plan_chunks(T, gridDim.x, p.chunk_tiles_max);
  const int g0 = plan.bound(blockIdx.x);                   // first tile of this workgroup's range
  const int gfull = plan.length(blockIdx.x);
  const int glen = min(gfull, T - g0);                     // its length (<= 0: nothing to do)
  if (glen <= 0) return;

  // ---- per-lane, loop-invariant offsets ---------------------------------------------------------
  uint8_t* wlds = lds + (PLANNED ? 0 : p.prefix_bytes) + wave * kWaveBytes;
  const uint32_t wbase = (uint32_t)(uintptr_t)(lptr_t)wlds;
  // bf16 pools.  Load j of a tile brings token rows 4j..4j+3 straight to LDS slot (j, lane); the
  // piece of row 4j + q4 this lane fetches fixes the swizzles of the bf16 kernel on the global
  // side: K row t keeps 16-byte piece c at slot c ^ t, V row t at slot c ^ 2(t mod 8).
  // 8-bit pools.  Raw fetch: load h of a tile brings token rows 8h..8h+7, 128 bytes each; this
  // lane takes the 16-byte piece p8 (dims 16 p8..+15) of row 8h + r8.  Decoded, that is pieces
  // 2 p8 and 2 p8 + 1 of the 256-byte bf16 row, written by two 16-byte LDS stores.  The LDS
  // serves such a store eight lanes at a time, 128 bytes wide: the eight lanes of a row must
  // hit eight different 16-byte columns modulo 8.  With the bf16 kernel's swizzles they would
  // write the even pieces in one store and the odd ones in the other: columns 0, 2, 4, 6 twice,
  // every store a two-way conflict (36 % of the kernel's LDS cycles, measured).  So these
  // images place piece c at sigma(c) ^ row, with sigma(even c) = c / 2 and sigma(odd c) =
  // 8 + (c / 2 ^ 4): even pieces fill the lower half of a row, odd ones the upper half, each
  // store covers all eight columns, and the reads stay free of conflicts too (sixteen rows of
  // one piece for the scores; for the transposing reads four rows of two pieces, whose columns
  // x ^ m and x ^ m ^ 4, m = 0..3, are all different).
  uint32_t koff[4], voff[4], kwr[2][2], vwr[2][2], krd[4], vrd[8];
  auto sigma = [](int c) { return (c & 1) ? 8 + ((c >> 1) ^ 4) : (c >> 1); };
  if constexpr (KV8) {
    const int r8 = lane >> 3, p8 = lane & 7;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const int tok = 8 * h + r8;
      koff[h] = (uint32_t)(tok * p.k_stride_token) + (uint32_t)(p8 * 16);
      voff[h] = (uint32_t)(tok * p.v_stride_token) + (uint32_t)(p8 * 16);
#pragma unroll
      for (int e = 0; e < 2; ++e) {
        const int c = 2 * p8 + e;
        kwr[h][e] = (uint32_t)(tok * 256 + ((sigma(c) ^ tok) * 16));
        vwr[h][e] = (uint32_t)(kTileBytes + tok * 256 + ((sigma(c) ^ (tok & 7)) * 16));
      }
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) krd[j] = (uint32_t)(t16 * 256 + ((sigma(4 * j + q4) ^ t16) * 16));
    // second product, output dims 16nb..16nb+15: the transposing read hands lane i of a 16-lane
    // group element (i mod 4) of the 8-byte pieces addressed by lanes i/4, 4+i/4, 8+i/4, 12+i/4;
    // this lane points at token tv, dims 16nb + 4(t16 mod 4)..+3: half (t16 mod 2) of piece
    // 2nb + hp, which sits at column nb ^ (tv mod 8), in the upper half with bit 2 flipped if hp
    const int tv = 4 * q4 + (t16 >> 2), hp = (t16 >> 1) & 1;
    const uint32_t vbase = (uint32_t)(tv * 256 + ((hp << 7) | ((((hp ? 4 : 0) ^ (tv & 7))) << 4) | ((t16 & 1) << 3)));
#pragma unroll
    for (int nb = 0; nb < 8; ++nb) vrd[nb] = (vbase ^ (uint32_t)(nb << 4)) + wbase;
  } else {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int tok = 4 * j + q4;
      koff[j] = (uint32_t)(tok * p.k_stride_token) + (uint32_t)((t16 ^ tok) * 16);
      voff[j] = (uint32_t)(tok * p.v_stride_token) + (uint32_t)((t16 ^ (2 * (tok & 7))) * 16);
      krd[j] = (uint32_t)(t16 * 256 + (((4 * j + q4) ^ t16) * 16));
    }
    // (as above, for the bf16 kernel's V image: piece pairs are 32-byte units at nb ^ (tv mod 8))
    const int tv = 4 * q4 + (t16 >> 2);
    const uint32_t vbase = (uint32_t)(tv * 256 + ((tv & 7) << 5) + (t16 & 3) * 8);
#pragma unroll
    for (int nb = 0; nb < 8; ++nb) vrd[nb] = (vbase ^ (uint32_t)(nb << 5)) + wbase;
  }
  float* xchg = reinterpret_cast<float*>(wlds + G::kDataBytes);   // 128 floats
  const uint8_t* kpool = reinterpret_cast<const uint8_t*>(p.k_pool);
  const uint8_t* vpool = reinterpret_cast<const uint8_t*>(p.v_pool);
  const int tile_mask = (1 << p.tpb_shift) - 1;

  int tiles_done = 0;
  float m_ref = kNegBig, l_part = 0.f;
  f32x4 acc[8];          // O[head 4q4+r][dim 16nb+t16] in acc[nb][r]
  bf16x8 qfrag[4];
  // descriptor tables, then the record of the batch each table describes
  u32x4* dtabs = reinterpret_cast<u32x4*>(wlds + G::kDataBytes + kXchgBytes);             // [kTables][BT]
  int* brecs = reinterpret_cast<int*>(wlds + G::kDataBytes + kXchgBytes + kTables * BT * 16);   // [kTables][8]

  // Tile descriptors of `count` (<= BT) tiles from axis position xb, one per lane:
  //   x: byte offset / 16 of the tile's first K row      y: same for V
  //   z: sequence << 8 | pair
  //   w: valid tokens (1..16) | first-of-pair << 5 | last-of-pair << 6 | opens << 7 | closes << 8 |
  //      tiles of the pair << 9
  // (opens / closes: a segment begins / ends with this tile: the pair does, or the chunk does).
  // Without a plan they are worked out here; a plan holds them ready, one per axis position.
  // t0: number of the batch's first tile within its chunk of ntc tiles.
  auto build_desc = [&](int xb, int count, int t0, int ntc, u32x4* tab) {
    const int x = xb + min(lane, count - 1);
    const int xq = x / NP;
    int lo = 0, hi = B;                            // prefix[lo] <= xq < prefix[hi]
    while (hi - lo > 1) {
      const int mid = (lo + hi) >> 1;
      if (prefix[mid] <= xq) lo = mid; else hi = mid;
    }
    const int seq = lo;
    const int pstart = prefix[seq];
    const int tiles = prefix[seq + 1] - pstart;
    const int rem = x - pstart * NP;
    const int pp = rem / tiles;
    const int t = rem - pp * tiles;
    const int kvh = pp / p.group_tiles;
    const int n = p.context_lens[seq];
    const int blk = p.block_tables[(int64_t)seq * p.max_blocks_per_seq + (t >> p.tpb_shift)];
    const int slot0 = (t & tile_mask) * kTileTokens;
    u32x4 d;
    d[0] = (uint32_t)((blk * p.k_stride_block + kvh * p.k_stride_head + slot0 * p.k_stride_token) >> 4);
    d[1] = (uint32_t)((blk * p.v_stride_block + kvh * p.v_stride_head + slot0 * p.v_stride_token) >> 4);
    d[2] = (uint32_t)((seq << 8) | pp);
    const int ntok = min(kTileTokens, n - t * kTileTokens);
    const int tc = t0 + min(lane, count - 1);
    d[3] = (uint32_t)(ntok | ((t == 0) << 5) | ((t == tiles - 1) << 6) | ((t == 0 || tc == 0) << 7) |
                      ((t == tiles - 1 || tc == ntc - 1) << 8) | (tiles << 9));
    if (lane < BT) tab[lane] = d;
  };

  // ---- loads ----------------------------------------------------------------------------------
  // Tile bytes of 8-bit pools land in register set S = v[174 + 16 S .. 189 + 16 S] (K rows in the
  // first two quads, V rows in the last two), the query rows fetched ahead in v[238:253].
  auto fetch = [&](uint32_t sk, uint32_t sv, auto set_tag) {
    constexpr int S = decltype(set_tag)::value;
    const uint8_t* kb = kpool + ((uint64_t)sk << 4);
    const uint8_t* vb = vpool + ((uint64_t)sv << 4);
    if constexpr (KV8) {
      const uint32_t k0 = koff[0], k1 = koff[1], v0 = voff[0], v1 = voff[1];
#define PKV_FETCH_SET(Q0, Q1, Q2, Q3)                                                 \
  asm volatile("global_load_dwordx4 " Q0 ", %0, %4 nt\n\t"                            \
               "global_load_dwordx4 " Q1 ", %1, %4 nt\n\t"                            \
               "global_load_dwordx4 " Q2 ", %2, %5 nt\n\t"                            \
               "global_load_dwordx4 " Q3 ", %3, %5 nt"                                \
               :                                                                      \
               : "v"(k0), "v"(k1), "v"(v0), "v"(v1), "s"(kb), "s"(vb)                 \
               : "memory")
      if constexpr (S == 0) PKV_FETCH_SET("v[174:177]", "v[178:181]", "v[182:185]", "v[186:189]");
      else if constexpr (S == 1) PKV_FETCH_SET("v[190:193]", "v[194:197]", "v[198:201]", "v[202:205]");
      else if constexpr (S == 2) PKV_FETCH_SET("v[206:209]", "v[210:213]", "v[214:217]", "v[218:221]");
      else PKV_FETCH_SET("v[222:225]", "v[226:229]", "v[230:233]", "v[234:237]");
#undef PKV_FETCH_SET
    } else {
      uint8_t* kl = wlds + S * kImageBytes;
#pragma unroll
      for (int jj = 0; jj < 4; ++jj)
        __builtin_amdgcn_global_load_lds((gptr_t)(kb + koff[jj]), (lptr_t)(kl + jj * 1024), 16, 0, 2);
#pragma unroll
      for (int jj = 0; jj < 4; ++jj)
        __builtin_amdgcn_global_load_lds((gptr_t)(vb + voff[jj]), (lptr_t)(kl + kTileBytes + jj * 1024), 16, 0, 2);
    }
  };
  // 16 codes in four registers (one 16-byte piece of a row) to 16 bf16 values in order: every
  // E4M3 value is a bf16 value, and the conversion (two codes per instruction) is exact.
#define PKV_DECODE_QUAD(A, B, C, D, lo, hi)                                           \
  {                                                                                   \
    uint32_t o0, o1, o2, o3, o4, o5, o6, o7;                                          \
    asm volatile("v_cvt_scalef32_pk_bf16_fp8 %0, " A ", 1.0\n\t"                      \
                 "v_cvt_scalef32_pk_bf16_fp8 %1, " A ", 1.0 op_sel:[1,0,0]\n\t"       \
                 "v_cvt_scalef32_pk_bf16_fp8 %2, " B ", 1.0\n\t"                      \
                 "v_cvt_scalef32_pk_bf16_fp8 %3, " B ", 1.0 op_sel:[1,0,0]\n\t"       \
                 "v_cvt_scalef32_pk_bf16_fp8 %4, " C ", 1.0\n\t"                      \
                 "v_cvt_scalef32_pk_bf16_fp8 %5, " C ", 1.0 op_sel:[1,0,0]\n\t"       \
                 "v_cvt_scalef32_pk_bf16_fp8 %6, " D ", 1.0\n\t"                      \
                 "v_cvt_scalef32_pk_bf16_fp8 %7, " D ", 1.0 op_sel:[1,0,0]\n\t"       \
                 "s_nop 0"                                                            \
                 : "=&v"(o0), "=&v"(o1), "=&v"(o2), "=&v"(o3), "=&v"(o4), "=&v"(o5), "=&v"(o6), "=&v"(o7)); \
    lo = u32x4{o0, o1, o2, o3};                                                       \
    hi = u32x4{o4, o5, o6, o7};                                                       \
  }
  // The tile of a set is complete once only the loads of the tiles sent after it are outstanding:
  // `younger` of them (8-bit: up to three sets of four loads; bf16: at most the other stage's
  // eight loads, and query rows that were sent behind it).  Anything else that is on its way
  // (query rows, a plan's descriptors) only makes such a wait stricter.
  auto arrive = [&](auto set_tag, int younger, bool q_behind, bool row_behind) {
    constexpr int S = decltype(set_tag)::value;
    if constexpr (KV8) {
      if (younger >= 3) asm volatile("s_waitcnt vmcnt(12)" ::: "memory");
      else if (younger == 2) asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
      else if (younger == 1) asm volatile("s_waitcnt vmcnt(4)" ::: "memory");
      else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      // decode into the LDS images
      u32x4 a0, b0, a1, b1, a2, b2, a3, b3;
#define PKV_DECODE_SET(K0, K1, K2, K3, K4, K5, K6, K7, V0, V1, V2, V3, V4, V5, V6, V7) \
  PKV_DECODE_QUAD(K0, K1, K2, K3, a0, b0)                                              \
  PKV_DECODE_QUAD(K4, K5, K6, K7, a1, b1)                                              \
  PKV_DECODE_QUAD(V0, V1, V2, V3, a2, b2)                                              \
  PKV_DECODE_QUAD(V4, V5, V6, V7, a3, b3)
      if constexpr (S == 0) {
        PKV_DECODE_SET("v174", "v175", "v176", "v177", "v178", "v179", "v180", "v181",
                       "v182", "v183", "v184", "v185", "v186", "v187", "v188", "v189")
      } else if constexpr (S == 1) {
        PKV_DECODE_SET("v190", "v191", "v192", "v193", "v194", "v195", "v196", "v197",
                       "v198", "v199", "v200", "v201", "v202", "v203", "v204", "v205")
      } else if constexpr (S == 2) {
        PKV_DECODE_SET("v206", "v207", "v208", "v209", "v210", "v211", "v212", "v213",
                       "v214", "v215", "v216", "v217", "v218", "v219", "v220", "v221")
      } else {
        PKV_DECODE_SET("v222", "v223", "v224", "v225", "v226", "v227", "v228", "v229",
                       "v230", "v231", "v232", "v233", "v234", "v235", "v236", "v237")
      }
#undef PKV_DECODE_SET
      *reinterpret_cast<u32x4*>(wlds + kwr[0][0]) = a0;
      *reinterpret_cast<u32x4*>(wlds + kwr[0][1]) = b0;
      *reinterpret_cast<u32x4*>(wlds + kwr[1][0]) = a1;
      *reinterpret_cast<u32x4*>(wlds + kwr[1][1]) = b1;
      *reinterpret_cast<u32x4*>(wlds + vwr[0][0]) = a2;
      *reinterpret_cast<u32x4*>(wlds + vwr[0][1]) = b2;
      *reinterpret_cast<u32x4*>(wlds + vwr[1][0]) = a3;
      *reinterpret_cast<u32x4*>(wlds + vwr[1][1]) = b3;
    } else {
      if (younger == 0) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      else if (q_behind && row_behind) asm volatile("s_waitcnt vmcnt(13)" ::: "memory");
      else if (q_behind) asm volatile("s_waitcnt vmcnt(12)" ::: "memory");
      else if (row_behind) asm volatile("s_waitcnt vmcnt(9)" ::: "memory");
      else asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
    }
  };
#undef PKV_DECODE_QUAD
  static_assert(FlatGeom<true>::kSets == 4 && FlatGeom<false>::kSets == 2, "the waits above count the younger sets");

  // Query rows as the B operand of the first product (column t16 is head min(t16, nheads-1) of
  // the group): four 16-byte loads per lane.
  auto q_address = [&](int sp) {
    const int seq = sp >> 8, pp = sp & 255;
    const int kvh = pp / p.group_tiles, gtile = pp - kvh * p.group_tiles;
    const int h0 = kvh * p.group + gtile * GH;
    const int nheads = min(GH, p.group - gtile * GH);
    const int hs = min(t16, nheads - 1);
    return reinterpret_cast<const uint8_t*>(p.q) + ((int64_t)seq * p.num_q_heads + h0 + hs) * (D * 2) + q4 * 16;
  };
  u32x4 qraw[4];                    // query rows of the open segment (qfrag is their operand view)
  // ahead of their segment: left in flight
  auto load_q_ahead = [&](int sp) {
    const uint8_t* qp = q_address(sp);
    asm volatile(
        "global_load_dwordx4 v[238:241], %0, off\n\t"
        "global_load_dwordx4 v[242:245], %0, off offset:64\n\t"
        "global_load_dwordx4 v[246:249], %0, off offset:128\n\t"
        "global_load_dwordx4 v[250:253], %0, off offset:192"
        :
        : "v"(qp)
        : "memory");
  };
  // ... and taken over when the segment opens (a wait has completed them by then)
  auto take_q = [&]() {
    uint32_t t[16];
    asm volatile(
        "v_mov_b32 %0, v238\n\tv_mov_b32 %1, v239\n\tv_mov_b32 %2, v240\n\tv_mov_b32 %3, v241\n\t"
        "v_mov_b32 %4, v242\n\tv_mov_b32 %5, v243\n\tv_mov_b32 %6, v244\n\tv_mov_b32 %7, v245\n\t"
        "v_mov_b32 %8, v246\n\tv_mov_b32 %9, v247\n\tv_mov_b32 %10, v248\n\tv_mov_b32 %11, v249\n\t"
        "v_mov_b32 %12, v250\n\tv_mov_b32 %13, v251\n\tv_mov_b32 %14, v252\n\tv_mov_b32 %15, v253"
        : "=&v"(t[0]), "=&v"(t[1]), "=&v"(t[2]), "=&v"(t[3]), "=&v"(t[4]), "=&v"(t[5]), "=&v"(t[6]), "=&v"(t[7]),
          "=&v"(t[8]), "=&v"(t[9]), "=&v"(t[10]), "=&v"(t[11]), "=&v"(t[12]), "=&v"(t[13]), "=&v"(t[14]), "=&v"(t[15])
        :
        : "memory");
#pragma unroll
    for (int c = 0; c < 4; ++c) qraw[c] = u32x4{t[4 * c], t[4 * c + 1], t[4 * c + 2], t[4 * c + 3]};
  };
  // at the segment's first tile: loaded and waited for in one statement
  auto load_q_now = [&](int sp) {
    const uint8_t* qp = q_address(sp);
    asm volatile(
        "global_load_dwordx4 %0, %4, off\n\t"
        "global_load_dwordx4 %1, %4, off offset:64\n\t"
        "global_load_dwordx4 %2, %4, off offset:128\n\t"
        "global_load_dwordx4 %3, %4, off offset:192\n\t"
        "s_waitcnt vmcnt(0)"
        : "=&v"(qraw[0]), "=&v"(qraw[1]), "=&v"(qraw[2]), "=&v"(qraw[3])
        : "v"(qp)
        : "memory");
  };

  // ---- the arithmetic of one tile, from the images of stage IMG (as in the bf16 kernel) ---------
  auto consume = [&](int ntok, auto img_tag) {
    constexpr int IMG = decltype(img_tag)::value;
    const bool tail = ntok < kTileTokens;            // wave-uniform
    const uint8_t* kl = wlds + IMG * kImageBytes;
    f32x4 cfr = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int jj = 0; jj < 4; ++jj) {
      const bf16x8 kf = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(kl + krd[jj]));
      cfr = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf, qfrag[jj], cfr, 0, 0, 0);
    }
    // cfr[r] = q_head(t16) . k_token(4q4+r); d = score - reference, in log2 units
    float d[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      d[r] = fmaf(cfr[r], p.scale_log2e, -m_ref);
      if (tail && 4 * q4 + r >= ntok) d[r] = -INFINITY;   // stale slot: may hold NaN bits
    }
    const float dmax = fmaxf(fmaxf(d[0], d[1]), fmaxf(d[2], d[3]));
    if (__builtin_amdgcn_ballot_w64(dmax > kSlack) != 0) {   // wave-uniform, rare after a first tile
      float s[4];
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        s[r] = cfr[r] * p.scale_log2e;
        if (tail && 4 * q4 + r >= ntok) s[r] = -INFINITY;
      }
      xchg[q4 * 16 + t16] = fmaxf(fmaxf(s[0], s[1]), fmaxf(s[2], s[3]));
      const float tm = fmaxf(fmaxf(xchg[t16], xchg[16 + t16]), fmaxf(xchg[32 + t16], xchg[48 + t16]));
      const float mn = fmaxf(m_ref, tm);
      const float alpha = __builtin_amdgcn_exp2f(m_ref - mn);
      m_ref = mn;
      l_part *= alpha;
#pragma unroll
      for (int r = 0; r < 4; ++r) d[r] = s[r] - mn;
      xchg[64 + t16] = alpha;   // the four lanes of a column write the same value
      const f32x4 a = *reinterpret_cast<const f32x4*>(xchg + 64 + 4 * q4);
#pragma unroll
      for (int nb = 0; nb < 8; ++nb)
#pragma unroll
        for (int r = 0; r < 4; ++r) acc[nb][r] *= a[r];
    }
    // weights, and their split into a bf16 head and a rounded bf16 remainder
    uint32_t hi[4], lo[4];
    float psum = 0.f;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const float pw = __builtin_amdgcn_exp2f(d[r]);
      psum += pw;
      hi[r] = __builtin_bit_cast(uint32_t, pw);
      const float rest = pw - __builtin_bit_cast(float, hi[r] & 0xFFFF0000u);   // exact, >= 0
      lo[r] = __builtin_bit_cast(uint32_t, rest) + 0x8000u;
    }
    l_part += psum;
    const s16x4 p_hi = __builtin_bit_cast(s16x4, u32x2{__builtin_amdgcn_perm(hi[1], hi[0], 0x07060302u),
                                                       __builtin_amdgcn_perm(hi[3], hi[2], 0x07060302u)});
    const s16x4 p_lo = __builtin_bit_cast(s16x4, u32x2{__builtin_amdgcn_perm(lo[1], lo[0], 0x07060302u),
                                                       __builtin_amdgcn_perm(lo[3], lo[2], 0x07060302u)});
    u32x2 vt[8];
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
        : "v"(vrd[0]), "v"(vrd[1]), "v"(vrd[2]), "v"(vrd[3]), "v"(vrd[4]), "v"(vrd[5]), "v"(vrd[6]),
          "v"(vrd[7]), "n"(IMG * kImageBytes + kTileBytes)
        : "memory");
    s16x4 vf[8];
    if (tail) {   // V rows past the context: zero, not NaN
      const uint32_t keep0 = (4 * q4 + 0 < ntok ? 0x0000FFFFu : 0u) | (4 * q4 + 1 < ntok ? 0xFFFF0000u : 0u);
      const uint32_t keep1 = (4 * q4 + 2 < ntok ? 0x0000FFFFu : 0u) | (4 * q4 + 3 < ntok ? 0xFFFF0000u : 0u);
#pragma unroll
      for (int nb = 0; nb < 8; ++nb) { vt[nb][0] &= keep0; vt[nb][1] &= keep1; }
    }
#pragma unroll
    for (int nb = 0; nb < 8; ++nb) vf[nb] = __builtin_bit_cast(s16x4, vt[nb]);
#pragma unroll
    for (int nb = 0; nb < 8; ++nb)
      acc[nb] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(p_hi, vf[nb], acc[nb], 0, 0, 0);
#pragma unroll
    for (int nb = 0; nb < 8; ++nb)
      acc[nb] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(p_lo, vf[nb], acc[nb], 0, 0, 0);
    // The two wavefronts that share a SIMD (w and w+4) do not get equal issue slots: whoever is
    // behind raises its priority until it catches up.
    ++tiles_done;
    if (lane == 0) progress[wave] = tiles_done;
    if (progress[wave ^ (kNW / 2)] > tiles_done) __builtin_amdgcn_s_setprio(2);
    else __builtin_amdgcn_s_setprio(0);
  };

  // ---- the sequence of batches of this wavefront ----------------------------------------------
  // A batch is up to BT consecutive tiles of one chunk; a wavefront takes the chunks with local
  // ids wave, wave + 8, ... of its workgroup's range.  Three cursors walk the sequence of batches: the builder, which starts the
  // description of a batch (by then the batch has a number, a table, and a record in LDS:
  // chunk id, axis position, tiles); the fetch cursor, which sends tiles on their way; the consumer.
  auto chunk_first = [&](int ci) { return plan.chunk_start(gfull, ci); };
  auto chunk_valid = [&](int ci) { return ci < plan.ns && chunk_first(ci) < glen; };
  auto static_chunk = [&](ChunkCursor& b, int ci) {
    b.ci = ci;
    b.c = blockIdx.x * plan.ns + ci;
    b.x0 = g0 + chunk_first(ci);
    b.ntc = min(glen, chunk_first(ci + 1)) - chunk_first(ci);
    b.b0 = 0;
  };
  int k = 0, fk = 0;              // tiles consumed / sent on their way so far
  int cn = 0, fn = 0;             // number of the batch being consumed / at the fetch cursor
  int started = 0, built = 0;     // batches whose description was started / is complete (started - built <= 1)
  int described = 0;              // tiles of the batches started
  ChunkCursor lb;                 // the chunk of the last batch started, b0 past that batch
  lb.ci = 0; lb.c = 0; lb.x0 = 0; lb.ntc = 0; lb.b0 = 0;
  bool more = true;               // batches after that one may exist
  // With a plan, a description is a direct-to-LDS load of the plan's descriptors; it is left in
  // flight while the tile loop goes on, and is known to be complete kSets tiles later: by then
  // the loop's own wait has let at most the loads of the tiles issued behind it stay outstanding,
  // and loads complete in the order issued.
  bool pending = false;           // a description is in flight
  int pending_k = 0;              // the tile count when it was sent

  // describe the next min(BT, rest) tiles of lb's chunk
  auto start = [&]() {
    const int tab = started % kTables;
    const int nt = min(BT, lb.ntc - lb.b0);
    const int x = lb.x0 + lb.b0;
    if (lane == 0) {
      int* r = brecs + tab * 8;
      r[0] = lb.c; r[1] = x; r[2] = nt;
    }
    if constexpr (PLANNED) {
      // lane i brings the descriptor of tile i of the batch to entry i of the table
      const uint32_t voff = (uint32_t)(x + min(lane, nt - 1)) * 16u;
      const uint32_t dst = (uint32_t)rfl((int)(wbase + G::kDataBytes + kXchgBytes + tab * BT * 16));
      // (M0 carries the LDS address of a direct-to-LDS load; the compiler keeps its own value
      // there, which is put back; a write to M0 needs a wait state before it is used)
      uint32_t m0_save;
      if (lane < BT)
        asm volatile(
            "s_mov_b32 %0, m0\n\t"
            "s_mov_b32 m0, %1\n\t"
            "s_nop 0\n\t"
            "global_load_lds_dwordx4 %2, %3\n\t"
            "s_mov_b32 m0, %0\n\t"
            "s_nop 0"
            : "=&s"(m0_save)
            : "s"(dst), "v"(voff), "s"(p.plan_desc)
            : "memory");
      pending = true;
      pending_k = k;
    } else {
      build_desc(x, nt, lb.b0, lb.ntc, dtabs + tab * BT);
      ++built;
    }
    lb.b0 += nt;
    ++started;
    described += nt;
  };
  // One step of the builder.  wait: whatever is in flight is waited for here, and nothing is
  // put off for later.  Returns whether calling again can get further.
  auto advance = [&](bool wait) -> bool {
    if (pending) {
      if (wait) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      else if (k - pending_k < kSets) return false;
      ++built;
      pending = false;
      return true;
    }
    if (!more || started - cn >= kTables) return false;
    if (!wait && described - k >= BT + kSets) return false;
    if (lb.b0 < lb.ntc) {                              // the chunk goes on
      start();
      return true;
    }
    const int nci = started == 0 ? wave : lb.ci + kNW;
    if (chunk_valid(nci)) {                            // the wavefront's next chunk
      static_chunk(lb, nci);
      start();
      return true;
    }
    more = false;
    return false;
  };
  // batch `number` is needed now
  auto need = [&](int number) {
    while (built <= number && advance(true)) {
    }
    return built > number;
  };
  auto ensure_ahead = [&]() {
    while (advance(false)) {
    }
  };
  auto rec = [&](int number, int field) { return rfl(brecs[(number % kTables) * 8 + field]); };

  int cc, cx, cnt, fnt;           // chunk id, axis position and tiles of the consumer's batch; tiles of the fetch cursor's
  int j = 0, fj = 0;              // tile within those batches
  bool fvalid = true;             // the fetch cursor has not run off the end of the work
  int q_for = -1;                 // the tile whose segment's query waits in qnext
  bool q_late = false;            // (bf16 pools) the last fetch put query rows in flight behind its tile
  // Calls that also append (with a plan): the new token's K and V rows of a (sequence, KV head)
  // are what the pair's last tile lacks.  The wavefront that streams that tile fetches the two
  // rows with it (one 16-byte piece per lane: 2 x 16 lanes into v[234:237] for bf16 pools,
  // 2 x 8 lanes into v[170:173] for 8-bit pools), puts them into the tile's LDS images once it
  // has arrived, and writes them to the pools; nobody else reads those pool rows in this call,
  // so no wavefront waits for another.
  constexpr int kRowLanes = KV8 ? 8 : 16;   // lanes per new row
  int row_for = -1;               // the tile whose new rows are in (or on their way to) those registers
  bool row_late = false;          // the last fetch put such rows in flight behind its tile
  int seg_sp = 0, seg_info0 = 0, seg_x = 0;

  if (!need(0)) return;
  cc = rec(0, 0); cx = rec(0, 1); cnt = rec(0, 2);
  fnt = cnt;

  using set0 = std::integral_constant<int, 0>;
  using set1 = std::integral_constant<int, 1>;
  using set2 = std::integral_constant<int, 2>;
  using set3 = std::integral_constant<int, 3>;

  // The tile at the fetch cursor goes in flight (nothing, once the cursor has run off the end of
  // the wavefront's work).  If that tile opens a segment, its query rows go in flight with it,
  // unless v[238:253] still hold the query of a segment not yet opened: in front of the tile for
  // 8-bit pools, behind it for bf16 pools (where the wait for the tile before it must not have
  // to wait for them).
  auto new_row_source = [&](int sp) {
    const int seq = sp >> 8, pp = sp & 255;
    const int kvh = pp / p.group_tiles;
    // lanes 0..15: the K row, lanes 16..31: the V row (offsets, not a choice between two
    // pointers: the compiler turns that into a table in scratch memory)
    const int64_t v_from_k = reinterpret_cast<const uint8_t*>(p.v_new) - reinterpret_cast<const uint8_t*>(p.k_new);
    return reinterpret_cast<const uint8_t*>(p.k_new) + (lane < kRowLanes ? (int64_t)0 : v_from_k) +
           ((int64_t)seq * p.num_kv_heads + kvh) * (kRowLanes * 16) + (lane & (kRowLanes - 1)) * 16;
  };
  auto fetch_ahead = [&](auto set_tag, int opened) {   // opened: last tile whose segment has its query
    q_late = false;
    row_late = false;
    if (!fvalid) return;
    const u32x4 d2 = dtabs[(fn % kTables) * BT + fj];
    const bool opens2 = ((int)d2[3] >> 7) & 1;
    const bool with_q = opens2 && q_for <= opened;
    // (the registers of a new row are free once the tile they were fetched for has taken them)
    const bool with_row = APPEND && p.k_new != nullptr && (((int)d2[3] >> 6) & 1) && row_for <= opened;
    if constexpr (KV8) {
      if (with_row) {
        const uint8_t* src = new_row_source(rfl((int)d2[2]));
        if (lane < 2 * kRowLanes) asm volatile("global_load_dwordx4 v[170:173], %0, off" : : "v"(src) : "memory");
        row_for = fk;
      }
    }
    if (KV8 && with_q) load_q_ahead(rfl((int)d2[2]));
    fetch((uint32_t)rfl((int)d2[0]), (uint32_t)rfl((int)d2[1]), set_tag);
    if (!KV8 && with_q) load_q_ahead(rfl((int)d2[2]));
    if (with_q) q_for = fk;
    q_late = !KV8 && with_q;
    if constexpr (!KV8) {
      if (with_row) {
        const uint8_t* src = new_row_source(rfl((int)d2[2]));
        if (lane < 2 * kRowLanes) asm volatile("global_load_dwordx4 v[234:237], %0, off" : : "v"(src) : "memory");
        row_for = fk;
        row_late = true;
      }
    }
    ++fk;
    if (++fj == fnt) {               // on to the next batch, which may have to be described first
      if (need(fn + 1)) {
        ++fn;
        fnt = rec(fn, 2);
        fj = 0;
      } else {
        fvalid = false;
      }
    }
  };

  auto tile = [&](auto set_tag) -> bool {
    constexpr int S = decltype(set_tag)::value;
    using img = std::integral_constant<int, KV8 ? 0 : S>;
    const u32x4 dsc = dtabs[(cn % kTables) * BT + j];   // the same entry for every lane
    const int sp = rfl((int)dsc[2]), info = rfl((int)dsc[3]);
    if constexpr (!KV8) fetch_ahead(std::integral_constant<int, 1 - (S & 1)>{}, k - 1);
    arrive(set_tag, fk - 1 - k, q_late, row_late);
    if constexpr (APPEND) {
      if (p.k_new != nullptr && ((info >> 6) & 1)) {       // the pair's last tile: the new token's rows go in
        if (row_for != k) {   // (not fetched ahead: the last tiles of short pairs close together)
          const uint8_t* src = new_row_source(sp);
          if (lane < 2 * kRowLanes) {
            if constexpr (KV8) asm volatile("global_load_dwordx4 v[170:173], %0, off\n\ts_waitcnt vmcnt(0)" : : "v"(src) : "memory");
            else asm volatile("global_load_dwordx4 v[234:237], %0, off\n\ts_waitcnt vmcnt(0)" : : "v"(src) : "memory");
          }
          row_for = k;
        }
        const int r = (info & 31) - 1, lr = lane & (kRowLanes - 1);   // the new token's row in the tile, this lane's piece
        const bool is_k = lane < kRowLanes;
        const int64_t in_k = (int64_t)((uint64_t)dsc[0] << 4) + (int64_t)r * p.k_stride_token;
        const int64_t in_v = (vpool - kpool) + (int64_t)((uint64_t)dsc[1] << 4) + (int64_t)r * p.v_stride_token;
        uint8_t* pool = const_cast<uint8_t*>(kpool) + (is_k ? in_k : in_v) + lr * 16;
        if constexpr (KV8) {
          // 16 codes of this lane: to the pool as they are, decoded into two pieces of the images
          if (lane < 2 * kRowLanes) {
            uint32_t o0, o1, o2, o3, o4, o5, o6, o7;
            asm volatile(
                "global_store_dwordx4 %8, v[170:173], off\n\t"
                "v_cvt_scalef32_pk_bf16_fp8 %0, v170, 1.0\n\t"
                "v_cvt_scalef32_pk_bf16_fp8 %1, v170, 1.0 op_sel:[1,0,0]\n\t"
                "v_cvt_scalef32_pk_bf16_fp8 %2, v171, 1.0\n\t"
                "v_cvt_scalef32_pk_bf16_fp8 %3, v171, 1.0 op_sel:[1,0,0]\n\t"
                "v_cvt_scalef32_pk_bf16_fp8 %4, v172, 1.0\n\t"
                "v_cvt_scalef32_pk_bf16_fp8 %5, v172, 1.0 op_sel:[1,0,0]\n\t"
                "v_cvt_scalef32_pk_bf16_fp8 %6, v173, 1.0\n\t"
                "v_cvt_scalef32_pk_bf16_fp8 %7, v173, 1.0 op_sel:[1,0,0]\n\t"
                "s_nop 0"
                : "=&v"(o0), "=&v"(o1), "=&v"(o2), "=&v"(o3), "=&v"(o4), "=&v"(o5), "=&v"(o6), "=&v"(o7)
                : "v"(pool)
                : "memory");
            const int rs = is_k ? r : (r & 7);
            uint8_t* row = wlds + (is_k ? 0 : kTileBytes) + r * 256;
            *reinterpret_cast<u32x4*>(row + ((sigma(2 * lr) ^ rs) * 16)) = u32x4{o0, o1, o2, o3};
            *reinterpret_cast<u32x4*>(row + ((sigma(2 * lr + 1) ^ rs) * 16)) = u32x4{o4, o5, o6, o7};
          }
        } else {
          const uint32_t image = wbase + (uint32_t)(img::value * kImageBytes + r * 256) +
                                 (uint32_t)(is_k ? ((lr ^ r) & 15) * 16 : kTileBytes + ((lr ^ (2 * (r & 7))) & 15) * 16);
          if (lane < 2 * kRowLanes)
            asm volatile(
                "ds_write_b128 %0, v[234:237]\n\t"
                "global_store_dwordx4 %1, v[234:237], off\n\t"
                "s_waitcnt lgkmcnt(0)"
                :
                : "v"(image), "v"(pool)
                : "memory");
        }
      }
    }
    if ((info >> 7) & 1) {                                 // the tile opens a segment
      seg_sp = sp;
      seg_info0 = info;
      seg_x = cx + j;
      m_ref = kNegBig;
      l_part = 0.f;
#pragma unroll
      for (int nb = 0; nb < 8; ++nb) acc[nb] = f32x4{0.f, 0.f, 0.f, 0.f};
      if (q_for == k) take_q();   // sent with this tile's bytes or before: complete since the wait above
      else load_q_now(sp);        // (the first tiles of a wavefront, and segments of a single tile in a row)
#pragma unroll
      for (int cidx = 0; cidx < 4; ++cidx) qfrag[cidx] = __builtin_bit_cast(bf16x8, qraw[cidx]);
    }
    if constexpr (KV8) fetch_ahead(set_tag, k);

    consume(info & 31, img{});

    const bool last = (info >> 6) & 1;
    if ((info >> 8) & 1) {
      // ---- flush the open segment: the finished rows if it is the whole (sequence, pair), else
      // a partial.  O goes through LDS to turn the accumulator layout (lane = one dim of four
      // heads) into whole rows: through the images just consumed, which the next decode or load
      // overwrites only after these reads ----
      const int c = cc;
      const int seq = seg_sp >> 8, pp = seg_sp & 255;
      const int kvh = pp / p.group_tiles, gtile = pp - kvh * p.group_tiles;
      const int h0 = kvh * p.group + gtile * GH;
      const int nheads = min(GH, p.group - gtile * GH);
      const bool first = (seg_info0 >> 5) & 1;
      const int prank = seq * NP + pp;
      xchg[q4 * 16 + t16] = l_part;
      xchg[64 + t16] = m_ref;
      float* st = reinterpret_cast<float*>(wlds + img::value * kImageBytes);
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        if (4 * q4 + r < GH) {
#pragma unroll
          for (int nb = 0; nb < 8; ++nb) st[(4 * q4 + r) * kStageRow + nb * 16 + t16] = acc[nb][r];
        }
      }
      const int64_t slot = (int64_t)prank + c;   // unique: both terms grow along the axis
      const int hh = lane >> 5, piece = lane & 31;   // two head rows per pass, 32 x 16 bytes each
#pragma unroll
      for (int g2 = 0; g2 < GH; g2 += 2) {
        const int g = g2 + hh;
        if (g < nheads) {
          const f32x4 o4 = *reinterpret_cast<const f32x4*>(st + g * kStageRow + piece * 4);
          const float lsum = (xchg[g] + xchg[16 + g]) + (xchg[32 + g] + xchg[48 + g]);
          if (first && last) {
            const float inv = (1.0f / lsum) * p.v_scale;
            const int64_t o = ((int64_t)seq * p.num_q_heads + h0 + g) * D + piece * 4;
            if (p.out_is_bf16) {
              i32x2 w;
              w[0] = (int)pack_bf16x2_rne(o4[0] * inv, o4[1] * inv);
              w[1] = (int)pack_bf16x2_rne(o4[2] * inv, o4[3] * inv);
              *reinterpret_cast<i32x2*>(reinterpret_cast<uint16_t*>(p.out) + o) = w;
            } else {
              *reinterpret_cast<f32x4*>(reinterpret_cast<float*>(p.out) + o) =
                  f32x4{o4[0] * inv, o4[1] * inv, o4[2] * inv, o4[3] * inv};
            }
          } else {
            f32x4* const row = reinterpret_cast<f32x4*>(p.ws_o + (slot * GH + g) * D + piece * 4);
            if (p.partials_streaming) {
              asm volatile("" ::: "memory");
              __builtin_nontemporal_store(o4, row);
              asm volatile("" ::: "memory");
            } else {
              *row = o4;
            }
            if (piece == 0)
              *reinterpret_cast<f32x2*>(p.ws_ml + (slot * GH + g) * 2) = f32x2{xchg[64 + g], lsum};
          }
        }
      }
      if (!PLANNED && lane == 0) {       // (a plan brings the directory ready)
        if (first && last) {
          *reinterpret_cast<i32x2*>(p.ws_dir + 2 * (int64_t)prank) = i32x2{0, 1};
        } else if (first) {
          const int tiles = seg_info0 >> 9;
          const int c_last = plan.chunk_of(seg_x + tiles - 1);
          *reinterpret_cast<i32x2*>(p.ws_dir + 2 * (int64_t)prank) = i32x2{(int)slot, c_last - c + 1};
        }
      }
    }
    ++k;
    if (++j == cnt) {              // on to the next batch
      if (!need(cn + 1)) return false;
      ++cn;
      cc = rec(cn, 0); cx = rec(cn, 1); cnt = rec(cn, 2);
      j = 0;
    }
    ensure_ahead();
    return true;
  };

  // the first tiles go in flight together; the tables further ahead are built behind the first
  if constexpr (KV8) {
    fetch_ahead(set0{}, -1);
    ensure_ahead();
    fetch_ahead(set1{}, -1);
    fetch_ahead(set2{}, -1);
    fetch_ahead(set3{}, -1);
    while (tile(set0{}) && tile(set1{}) && tile(set2{}) && tile(set3{})) {
    }
  } else {
    fetch_ahead(set0{}, -1);
    ensure_ahead();
    while (tile(set0{}) && tile(set1{})) {
    }
  }
}

// The register budgets: on this target the attribute counts in units of two registers, so 87
// leaves the compiler v0..v173, 85 leaves it v0..v169 and 117 leaves it v0..v233.
template <int GH>
__global__ __launch_bounds__(kStreamThreads) __attribute__((amdgpu_num_vgpr(87)))
void attn_stream_flat_f8_d128(const AttnParams p) {
  flat_body<GH, true, false>(p);
}
template <int GH>
__global__ __launch_bounds__(kStreamThreads) __attribute__((amdgpu_num_vgpr(85)))
void attn_stream_flat_f8_planned_d128(const AttnParams p) {
  flat_body<GH, true, true>(p);
}
template <int GH>
__global__ __launch_bounds__(kStreamThreads) __attribute__((amdgpu_num_vgpr(117)))
void attn_stream_flat_bf16_d128(const AttnParams p) {
  flat_body<GH, false, true>(p);
}

// ---- the per-step plan ------------------------------------------------------------------------------
// One launch per decode step: the tile count, every tile's descriptor (with the chunk boundaries
// of the streaming kernel's cut marked), and for every (sequence, pair) where its partials will sit.
// Lengths that need more descriptors than the plan has room for leave the plan marked invalid.
__global__ __launch_bounds__(kStreamThreads) void attn_plan_build(const AttnParams p, int32_t* hdr, int nwg) {
  extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
  __shared__ int wave_total[kNW];
  const int tid = threadIdx.x;
  const int lane = tid & (kWaveSize - 1);
  const int wave = tid / kWaveSize;
  const int B = p.batch;
  const int NP = p.num_kv_heads * p.group_tiles;
  int* prefix = reinterpret_cast<int*>(lds);       // [B + 1]
  {
    const int per = (B + kStreamThreads - 1) / kStreamThreads;
    const int i0 = tid * per, i1 = min(B, i0 + per);
    int sum = 0;
    for (int i = i0; i < i1; ++i) sum += (max(p.context_lens[i], 0) + kTileTokens - 1) / kTileTokens;
    int v = sum;
#pragma unroll
    for (int off = 1; off < kWaveSize; off <<= 1) {
      const int t = __shfl_up(v, off, kWaveSize);
      if (lane >= off) v += t;
    }
    if (lane == kWaveSize - 1) wave_total[wave] = v;
    __syncthreads();
    int run = v - sum;
    for (int w = 0; w < wave; ++w) run += wave_total[w];
    if (tid == 0) prefix[0] = 0;
    for (int i = i0; i < i1; ++i) {
      run += (max(p.context_lens[i], 0) + kTileTokens - 1) / kTileTokens;
      prefix[i + 1] = run;
    }
    __syncthreads();
  }
  const int64_t T64 = (int64_t)prefix[B] * NP;
  const bool fits = T64 <= p.plan_tiles_cap;
  const int T = fits ? (int)T64 : 0;
  const ChunkPlan plan = plan_chunks(T, nwg, p.chunk_tiles_max);
  if (blockIdx.x == 0 && tid == 0) {
    hdr[kPlanT] = T;
    hdr[kPlanKey] = fits ? p.plan_key : 0;
  }
  const int tile_mask = (1 << p.tpb_shift) - 1;
  const int64_t stride = (int64_t)gridDim.x * kStreamThreads;
  auto chunk_of = [&](int x) { return plan.chunk_of(x); };
  // tile descriptors, one per axis position (the fields the streaming kernel builds for itself
  // when it has no plan)
  for (int64_t x64 = (int64_t)blockIdx.x * kStreamThreads + tid; x64 < T; x64 += stride) {
    const int x = (int)x64;
    const int xq = x / NP;
    int lo = 0, hi = B;
    while (hi - lo > 1) {
      const int mid = (lo + hi) >> 1;
      if (prefix[mid] <= xq) lo = mid; else hi = mid;
    }
    const int seq = lo;
    const int pstart = prefix[seq];
    const int tiles = prefix[seq + 1] - pstart;
    const int rem = x - pstart * NP;
    const int pp = rem / tiles;
    const int t = rem - pp * tiles;
    const int kvh = pp / p.group_tiles;
    const int n = p.context_lens[seq];
    const int blk = p.block_tables[(int64_t)seq * p.max_blocks_per_seq + (t >> p.tpb_shift)];
    const int slot0 = (t & tile_mask) * kTileTokens;
    u32x4 d;
    d[0] = (uint32_t)((blk * p.k_stride_block + kvh * p.k_stride_head + slot0 * p.k_stride_token) >> 4);
    d[1] = (uint32_t)((blk * p.v_stride_block + kvh * p.v_stride_head + slot0 * p.v_stride_token) >> 4);
    d[2] = (uint32_t)((seq << 8) | pp);
    const int ntok = min(kTileTokens, n - t * kTileTokens);
    const int cx = chunk_of(x);
    const bool copens = x == 0 || chunk_of(x - 1) != cx, ccloses = x == T - 1 || chunk_of(x + 1) != cx;
    d[3] = (uint32_t)(ntok | ((t == 0) << 5) | ((t == tiles - 1) << 6) | ((t == 0 || copens) << 7) |
                      ((t == tiles - 1 || ccloses) << 8) | (tiles << 9));
    reinterpret_cast<u32x4*>(const_cast<void*>(p.plan_desc))[x] = d;
  }
  // directory: the partials of a (sequence, pair) sit in consecutive slots, one per chunk that
  // holds some of its tiles
  const int64_t pairs = (int64_t)B * NP;
  for (int64_t pr = (int64_t)blockIdx.x * kStreamThreads + tid; pr < pairs; pr += stride) {
    const int seq = (int)(pr / NP), pp = (int)(pr - (int64_t)seq * NP);
    const int tiles = prefix[seq + 1] - prefix[seq];
    i32x2 e = i32x2{0, 0};
    if (tiles > 0 && fits) {
      const int xs = prefix[seq] * NP + pp * tiles;
      const int c_first = chunk_of(xs), c_last = chunk_of(xs + tiles - 1);
      e = c_first == c_last ? i32x2{0, 1} : i32x2{(int)(pr + c_first), c_last - c_first + 1};
    }
    *reinterpret_cast<i32x2*>(p.ws_dir + 2 * pr) = e;
  }
}

template <typename K>
hipError_t launch_flat_kernel(K kernel, size_t lds, const AttnParams& p, hipStream_t s) {
  // with events: attached to the dispatch itself, so they carry the kernel's own begin and end
  if (p.ev_begin || p.ev_end)
    hipExtLaunchKernelGGL(kernel, dim3(num_cus()), dim3(kStreamThreads), lds, s, p.ev_begin, p.ev_end, 0, p);
  else
    hipLaunchKernelGGL(kernel, dim3(num_cus()), dim3(kStreamThreads), lds, s, p);
  return hipGetLastError();
}

template <int GH>
hipError_t launch_flat_gh(const AttnParams& p, hipStream_t s) {
  const bool planned = p.plan_hdr != nullptr;
  const size_t lds8 = (size_t)(planned ? 0 : p.prefix_bytes) + (size_t)kNW * flat_wave_lds<true>();
  if (p.kv_is_f8)
    return planned ? launch_flat_kernel(attn_stream_flat_f8_planned_d128<GH>, lds8, p, s)
                   : launch_flat_kernel(attn_stream_flat_f8_d128<GH>, lds8, p, s);
  return launch_flat_kernel(attn_stream_flat_bf16_d128<GH>, (size_t)kNW * flat_wave_lds<false>(), p, s);
}

constexpr int kFlatLdsMax = kStreamMaxPrefixBytes + kNW * (flat_wave_lds<true>() > flat_wave_lds<false>() ? flat_wave_lds<true>()
                                                                                                           : flat_wave_lds<false>());
static_assert(kFlatLdsMax + 2 * kNW * 4 <= 160 * 1024, "one workgroup per CU has 160 KiB of LDS");

template <int GH>
hipError_t prepare_gh() {
  for (const void* f : {reinterpret_cast<const void*>(&attn_stream_flat_f8_d128<GH>),
                        reinterpret_cast<const void*>(&attn_stream_flat_f8_planned_d128<GH>),
                        reinterpret_cast<const void*>(&attn_stream_flat_bf16_d128<GH>)}) {
    const hipError_t e = hipFuncSetAttribute(f, hipFuncAttributeMaxDynamicSharedMemorySize, kFlatLdsMax);
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

}  // namespace

// More than 64 KiB of dynamic LDS: asked for once per device (every time outside the table).
hipError_t prepare_attn_flat() {
  static std::atomic<bool> prepared[kMaxDevices];
  const int slot = device_slot();
  if (slot >= 0 && prepared[slot].load(std::memory_order_acquire)) return hipSuccess;
  hipError_t e = prepare_gh<1>();
  if (e == hipSuccess) e = prepare_gh<2>();
  if (e == hipSuccess) e = prepare_gh<4>();
  if (e == hipSuccess) e = prepare_gh<8>();
  if (e != hipSuccess) return e;
  if (slot >= 0) prepared[slot].store(true, std::memory_order_release);
  return hipSuccess;
}

// The streaming kernel of the flat family for p (8-bit pools and/or a plan); the caller puts
// the merge kernel behind it.
hipError_t launch_attn_flat(const AttnParams& p, int gh, hipStream_t s) {
  const hipError_t e = prepare_attn_flat();
  if (e != hipSuccess) return e;
  switch (gh) {
    case 1: return launch_flat_gh<1>(p, s);
    case 2: return launch_flat_gh<2>(p, s);
    case 4: return launch_flat_gh<4>(p, s);
    default: return launch_flat_gh<8>(p, s);
  }
}

// Plan buffer of a call: header, directory, one descriptor per tile the lengths allow.
PlanLayout plan_layout(const pkv_attn_desc& d) {
  PlanLayout l;
  const int G = d.num_q_heads / d.num_kv_heads;
  const int gh = stream_heads_per_lane(G);
  const int64_t np = (int64_t)d.num_kv_heads * ((G + gh - 1) / gh);
  const int64_t pairs = (int64_t)d.batch * np;
  const int64_t tiles_ub = ((int64_t)d.max_context_len + kTileTokens - 1) / kTileTokens * pairs;
  auto up = [](int64_t b) { return (b + 255) / 256 * 256; };
  l.hdr_bytes = kPlanWords * 4;
  l.dir_bytes = up(pairs * 2 * 4);
  l.desc_bytes = up(tiles_ub * 16);
  l.tiles_cap = tiles_ub;
  return l;
}

// p as for the attention call, with the plan's pointers in plan_hdr, ws_dir and plan_desc.
hipError_t launch_attn_plan(AttnParams& p, int32_t* plan_hdr, hipStream_t s) {
  stream_geometry(p);
  const int nwg = num_cus();
  hipLaunchKernelGGL(attn_plan_build, dim3(nwg), dim3(kStreamThreads), (size_t)p.prefix_bytes, s, p, plan_hdr, nwg);
  return hipGetLastError();
}

}  // namespace pkv
