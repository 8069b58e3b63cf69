// Paged decode attention, bf16 / head_dim 128 fast path for gfx950.
//
// Operation (arXiv 2602.07878, Sec. 2.2 "KV-Cache" for the paged pool, Sec. 4.2 for
// the per-step streaming of the whole KV history): out = softmax_t(scale q.K_t) V over
// the tokens found through the block table.
//
// Work split ("stream" decomposition).  All 16-token tiles of the call form one axis:
// sequence-major, then (KV head, head sub-group) pair, then tile.  The axis is cut into
// equal contiguous chunks, one wavefront per chunk, sized on the device from the actual
// context lengths, so every wavefront of a persistent grid streams the same number of
// bytes whatever the length mix, and no workgroup is launched for work that does not
// exist.  A chunk may cover parts of several (sequence, pair)s: each part is a segment
// and ends in a flush -- the finished output row if the segment is the whole pair, else
// an (m, l, O) partial that the merge kernel combines by log-sum-exp.  Wavefronts never
// wait for each other after the set-up; the two wavefronts that share a SIMD only trade
// issue priority so that neither falls behind (the older one would otherwise win every
// arbitration tie and finish a third earlier, leaving the CU half empty at the end).
//
// Per tile:
//  * K goes HBM -> LDS with direct-to-LDS 16-byte loads (no VGPR staging) into a 2-deep
//    ring per wavefront.  The LDS image is XOR-swizzled by choosing which 16-byte piece
//    of its token row each lane fetches, so the row-per-lane reads that feed the matrix
//    cores are bank-conflict free while every wave-wide global load still covers whole
//    contiguous 256-byte rows.
//  * scores S[head slot][token] = Q_g K^T come from v_mfma_f32_16x16x32_bf16 (both
//    operands exact bf16; the query group is replicated to the 16 rows of the tile).
//  * softmax weights stay fp32 and move from the score layout (lane = token) to the V
//    layout (lane = 16-byte piece of a V row) through a 1 KiB LDS tile; P.V is fp32 FMA
//    on V rows loaded straight into registers with coalesced 16-byte loads.
//  * the running maximum is only a reference point for exp2(): it is raised (and the
//    accumulators rescaled) only when a score exceeds it by more than kSlack.
// The loads of tile j+1 are in flight while tile j is consumed; the first tile of the
// next segment is issued before the current segment is flushed.

#include <type_traits>

#include "pkv_internal.h"

namespace pkv {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) int32_t i32x2;

constexpr float kNegBig = -1.0e30f;
constexpr float kSlack = 8.0f;             // log2 units the reference may lag the true max
constexpr int kStreamThreads = 512;        // one workgroup of 8 wavefronts per CU
constexpr int kNW = kStreamThreads / kWaveSize;
constexpr int kTileBytes = 4096;           // 16 tokens x 256-byte rows
constexpr int kStages = 2;
constexpr int kDescBatch = 128;            // tile descriptors per table
constexpr int kWaveLds = kStages * kTileBytes + 1024 + 2 * kDescBatch * 16;   // K ring + P tile + 2 descriptor tables
constexpr int kMinGroupTiles = 32;         // tiles per workgroup range below which fewer workgroups work
constexpr int D = 128;

#define PKV_WAIT_VMCNT(n) \
  __builtin_amdgcn_s_waitcnt(((n) & 0xF) | (((n) >> 4) << 14) | (0x7 << 4) | (0xF << 8))

template <int CTRL>
__device__ __forceinline__ float dpp(float v) {
  return __builtin_bit_cast(
      float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xF, 0xF, true));
}
__device__ __forceinline__ float row16_max(float v) {
  v = fmaxf(v, dpp<0xB1>(v)); v = fmaxf(v, dpp<0x4E>(v));
  v = fmaxf(v, dpp<0x141>(v)); v = fmaxf(v, dpp<0x140>(v));
  return v;
}
__device__ __forceinline__ float row16_sum(float v) {
  v += dpp<0xB1>(v); v += dpp<0x4E>(v); v += dpp<0x141>(v); v += dpp<0x140>(v);
  return v;
}

__device__ __forceinline__ uint32_t pack_bf16x2_rne(float lo, float hi) {
  auto cv = [](float f) -> uint32_t {
    uint32_t u = __builtin_bit_cast(uint32_t, f);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (u >> 16) | 0x40u;
    u += 0x7FFFu + ((u >> 16) & 1u);
    return u >> 16;
  };
  return cv(lo) | (cv(hi) << 16);
}

__device__ __forceinline__ int rfl(int v) { return __builtin_amdgcn_readfirstlane(v); }

typedef const void __attribute__((address_space(1)))* gptr_t;
typedef void __attribute__((address_space(3)))* lptr_t;

// Chunk schedule.  The tile axis is cut into equal contiguous ranges, one per workgroup,
// and each range into `ns` chunks of `rs` tiles: one per wavefront, or more and shorter ones
// when the caller caps the tokens per partial (wavefront w then takes chunks w, w+8, ...).
// Chunk ids grow along the axis: id = workgroup * ns + local id.
struct ChunkPlan {
  int lg, rs, ns;
  __device__ __forceinline__ int chunk_of(int x) const {
    const int g = x / lg;
    return g * ns + (x - g * lg) / rs;
  }
};

__device__ __forceinline__ ChunkPlan plan_chunks(int T, int nwg, int cap) {
  ChunkPlan pl;
  pl.lg = max(kMinGroupTiles, (T + nwg - 1) / nwg);
  pl.rs = (pl.lg + kNW - 1) / kNW;
  if (cap > 0) pl.rs = min(pl.rs, cap);
  pl.ns = (pl.lg + pl.rs - 1) / pl.rs;
  return pl;
}

// GH = query heads accumulated per lane (1, 2, 4 or 8).
template <int GH>
__global__ __launch_bounds__(kStreamThreads, 2) void attn_stream_mfma_d128(const AttnParams p) {
  constexpr int HS = GH >= 8 ? 8 : 4;   // distinct head slots among the 16 MFMA rows

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

  // ---- set-up: exclusive prefix sums of per-sequence tile counts, in LDS ------------------
  int* prefix = reinterpret_cast<int*>(lds);       // [B + 1]
  {
    if (tid < kNW) progress[tid] = 0;
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
  const int T = rfl(prefix[B]) * NP;               // tiles of the whole call
  if (T == 0) return;

  const ChunkPlan plan = plan_chunks(T, gridDim.x, p.chunk_tiles_max);
  const int g0 = blockIdx.x * plan.lg;                     // first tile of this workgroup's range
  const int glen = min(plan.lg, T - g0);                   // its length (<= 0: nothing to do)
  const int rs = plan.rs;                                  // tiles per chunk
  if (glen <= 0) return;
  // ---- per-lane, loop-invariant offsets -------------------------------------------------------
  uint32_t koff[4], voff[4], krd[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int tok = 4 * j + q4;                        // token row this lane fetches in load j
    koff[j] = (uint32_t)(tok * p.k_stride_token) + (uint32_t)((t16 ^ tok) * 16);
    voff[j] = (uint32_t)(tok * p.v_stride_token) + (uint32_t)(t16 * 16);
    // MFMA step j: this lane (token t16) needs piece 4j+q4 of its row, stored at slot piece^t16
    krd[j] = (uint32_t)((t16 >> 2) * 1024 + (t16 & 3) * 256 + (((4 * j + q4) ^ t16) * 16));
  }
  uint8_t* wlds = lds + p.prefix_bytes + wave * kWaveLds;
  float* pbuf = reinterpret_cast<float*>(wlds + kStages * kTileBytes);   // [16 tokens][16 slots]
  const uint8_t* kpool = reinterpret_cast<const uint8_t*>(p.k_pool);
  const uint8_t* vpool = reinterpret_cast<const uint8_t*>(p.v_pool);
  const int tile_mask = (1 << p.tpb_shift) - 1;

  int tiles_done = 0;
  float m[4], l[4];
  float acc[GH][8];
  bf16x8 qfrag[4];
  u32x4 vreg[kStages][4];

  // two descriptor tables per wavefront: the one in use and the one filled ahead for the next chunk
  u32x4* dtabs = reinterpret_cast<u32x4*>(wlds + kStages * kTileBytes + 1024);   // [2][kDescBatch]

  // Tile descriptors of `count` (<= kDescBatch) tiles from axis position xb, built by the lanes:
  //   x: byte offset / 16 of the tile's first K row      y: same for V
  //   z: sequence << 8 | pair
  //   w: valid tokens (1..16) | first-of-pair << 5 | last-of-pair << 6 | tiles of the pair << 8
  auto build_desc = [&](int xb, int count, u32x4* tab) {
#pragma unroll 1
    for (int pass = 0; pass * kWaveSize < count; ++pass) {
    const int idx = pass * kWaveSize + lane;
    const int x = xb + min(idx, count - 1);
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
    d[3] = (uint32_t)(ntok | ((t == 0) << 5) | ((t == tiles - 1) << 6) | (tiles << 8));
    tab[idx] = d;
    }
  };

  int d_k = 0, d_v = 0, d_sp = 0, d_info = 0;   // descriptors of the current group, one tile per lane

  auto issue_at = [&](uint32_t sk, uint32_t sv, int stage) {
    const uint8_t* kb = kpool + ((uint64_t)sk << 4);
    const uint8_t* vb = vpool + ((uint64_t)sv << 4);
    uint8_t* kl = wlds + stage * kTileBytes;
#pragma unroll
    for (int jj = 0; jj < 4; ++jj)
      __builtin_amdgcn_global_load_lds((gptr_t)(kb + koff[jj]), (lptr_t)(kl + jj * 1024), 16, 0, 0);
#pragma unroll
    for (int jj = 0; jj < 4; ++jj)
      vreg[stage][jj] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(vb + voff[jj]));
  };
  auto issue = [&](int j, int stage) {
    issue_at((uint32_t)__builtin_amdgcn_readlane(d_k, j), (uint32_t)__builtin_amdgcn_readlane(d_v, j), stage);
  };

  auto load_q = [&](int sp) {
    const int seq = sp >> 8, pp = sp & 255;
    const int kvh = pp / p.group_tiles, gtile = pp - kvh * p.group_tiles;
    const int h0 = kvh * p.group + gtile * GH;
    const int nheads = min(GH, p.group - gtile * GH);
    const int hs = min(t16 % HS, nheads - 1);
    const uint8_t* qp = reinterpret_cast<const uint8_t*>(p.q) +
                        ((int64_t)seq * p.num_q_heads + h0 + hs) * (D * 2) + q4 * 16;
#pragma unroll
    for (int cidx = 0; cidx < 4; ++cidx)
      qfrag[cidx] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(qp + cidx * 64));
  };

  // TAIL: the tile may hold fewer than 16 valid tokens (only the last tile of a pair can)
  auto consume = [&](int j, int stage, auto tail_tag) {
    constexpr bool TAIL = decltype(tail_tag)::value;
    const int ntok = TAIL ? (__builtin_amdgcn_readlane(d_info, j) & 31) : kTileTokens;
    const uint8_t* kl = wlds + stage * kTileBytes;
    f32x4 cfr = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int jj = 0; jj < 4; ++jj) {
      const bf16x8 kf = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(kl + krd[jj]));
      cfr = __builtin_amdgcn_mfma_f32_16x16x32_bf16(qfrag[jj], kf, cfr, 0, 0, 0);
    }
    const bool dead = TAIL && (t16 >= ntok);
    float s[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) s[r] = dead ? -INFINITY : cfr[r] * p.scale_log2e;

    bool grow = false;
#pragma unroll
    for (int r = 0; r < 4; ++r) grow |= s[r] > m[r] + kSlack;
    if (__builtin_amdgcn_ballot_w64(grow) != 0) {      // wave-uniform, rare after a first tile
      f32x4 alpha;
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const float mn = fmaxf(m[r], row16_max(s[r]));
        alpha[r] = __builtin_amdgcn_exp2f(m[r] - mn);
        m[r] = mn;
        l[r] *= alpha[r];
      }
      // the rescale factors of all head slots are needed by every lane's accumulators
      *reinterpret_cast<f32x4*>(pbuf + 4 * q4) = alpha;
      float a[GH];
#pragma unroll
      for (int g = 0; g < GH; ++g) a[g] = pbuf[g];
#pragma unroll
      for (int g = 0; g < GH; ++g)
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[g][e] *= a[g];
    }

    f32x4 pw;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      pw[r] = __builtin_amdgcn_exp2f(s[r] - m[r]);
      l[r] += pw[r];
    }
    *reinterpret_cast<f32x4*>(pbuf + t16 * 16 + 4 * q4) = pw;

#pragma unroll
    for (int jj = 0; jj < 4; ++jj) {
      const int tok = 4 * jj + q4;                      // V row held by this lane for load jj
      float pv[GH];
      if constexpr (GH >= 4) {
#pragma unroll
        for (int g4 = 0; g4 < GH / 4; ++g4) {
          const f32x4 t = *reinterpret_cast<const f32x4*>(pbuf + tok * 16 + 4 * g4);
          pv[4 * g4] = t[0]; pv[4 * g4 + 1] = t[1]; pv[4 * g4 + 2] = t[2]; pv[4 * g4 + 3] = t[3];
        }
      } else if constexpr (GH == 2) {
        const f32x2 t = *reinterpret_cast<const f32x2*>(pbuf + tok * 16);
        pv[0] = t[0]; pv[1] = t[1];
      } else {
        pv[0] = pbuf[tok * 16];
      }
      u32x4 vv = vreg[stage][jj];
      if (TAIL && tok >= ntok) vv = u32x4{0, 0, 0, 0};   // stale slot: may hold NaN bits
      float vf[8];
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        vf[2 * e] = __builtin_bit_cast(float, vv[e] << 16);
        vf[2 * e + 1] = __builtin_bit_cast(float, vv[e] & 0xFFFF0000u);
      }
#pragma unroll
      for (int g = 0; g < GH; ++g)
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[g][e] = fmaf(pv[g], vf[e], acc[g][e]);
    }
    // The two wavefronts that share a SIMD (w and w+4) do not get equal issue slots: the
    // older one wins every tie.  Whoever is behind raises its priority until it catches up.
    ++tiles_done;
    if (lane == 0) progress[wave] = tiles_done;
    if (progress[wave ^ (kNW / 2)] > tiles_done) __builtin_amdgcn_s_setprio(2);
    else __builtin_amdgcn_s_setprio(0);
  };


  // state of the segment being accumulated (may span groups of one chunk) and of the pipeline
  bool open = false;        // a segment is being accumulated
  bool inflight = false;    // the first tile of the coming group is already issued, its query loaded
  int seg_sp = 0, seg_info0 = 0, seg_x = 0, sp = 0, tab = 0;

  auto chunk_valid = [&](int ci) { return ci < plan.ns && ci * rs < glen; };
  auto chunk_tiles = [&](int ci) { return min(glen, (ci + 1) * rs) - ci * rs; };

  if (chunk_valid(wave)) build_desc(g0 + wave * rs, min(kDescBatch, chunk_tiles(wave)), dtabs);
  for (int ci = wave; chunk_valid(ci); ci += kNW) {   // local chunk id
    const int c = blockIdx.x * plan.ns + ci;         // chunk id on the whole axis
    const int x0 = g0 + ci * rs;
    const int ntc = chunk_tiles(ci);                 // tiles of this chunk
    const bool has_next = chunk_valid(ci + kNW);

    for (int b0 = 0; b0 < ntc; b0 += kDescBatch) {
      const int ntb = min(kDescBatch, ntc - b0);
      u32x4* dtab = dtabs + tab * kDescBatch;
      if (b0 > 0) build_desc(x0 + b0, ntb, dtab);   // a chunk's first batch was built ahead
      const bool last_batch = b0 + ntb == ntc;

      for (int r0 = 0; r0 < ntb; r0 += kWaveSize) {
        const int nt = min(kWaveSize, ntb - r0);    // tiles of this group, one descriptor per lane
        {
          const u32x4 dreg = dtab[r0 + min(lane, nt - 1)];
          d_k = (int)dreg[0]; d_v = (int)dreg[1]; d_sp = (int)dreg[2]; d_info = (int)dreg[3];
        }
        const bool chunk_ends_here = b0 + r0 + nt == ntc;

        int j0 = 0;
        if (!inflight) {
          // tile first, query second: the compiler drains the load queue before a
          // direct-to-LDS load, so anything issued ahead of it would be waited for in full
          sp = __builtin_amdgcn_readlane(d_sp, 0);
          issue(0, 0);
          if (!open) load_q(sp);                    // an open segment continues with its query
        }
        inflight = false;
        // with this chunk's last stretch under way, describe the next chunk: its index loads ride
        // along with the tile that is in flight
        if (r0 == 0 && last_batch && has_next)
          build_desc(g0 + (ci + kNW) * rs, min(kDescBatch, chunk_tiles(ci + kNW)),
                     dtabs + (tab ^ 1) * kDescBatch);

        while (j0 < nt) {
          // tiles j0 .. j1-1 belong to (sequence, pair) sp; the first one is already in flight
          const uint64_t same = __builtin_amdgcn_ballot_w64(d_sp == sp && lane >= j0 && lane < nt);
          const int j1 = j0 + __builtin_popcountll(same);
          const int info1 = __builtin_amdgcn_readlane(d_info, j1 - 1);

        if (!open) {
          open = true;
          seg_sp = sp;
          seg_info0 = __builtin_amdgcn_readlane(d_info, j0);
          seg_x = x0 + b0 + r0 + j0;
#pragma unroll
          for (int r = 0; r < 4; ++r) { m[r] = kNegBig; l[r] = 0.f; }
#pragma unroll
          for (int g = 0; g < GH; ++g)
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[g][e] = 0.f;
        }

        {
          using std::false_type;
          using std::true_type;
          int j = j0;
          while (j + 2 < j1) {
            issue(j + 1, 1); PKV_WAIT_VMCNT(8); consume(j, 0, false_type{});
            issue(j + 2, 0); PKV_WAIT_VMCNT(8); consume(j + 1, 1, false_type{});
            j += 2;
          }
          if (j + 2 == j1) {
            issue(j + 1, 1); PKV_WAIT_VMCNT(8); consume(j, 0, false_type{});
            PKV_WAIT_VMCNT(0); consume(j + 1, 1, true_type{});
          } else {
            PKV_WAIT_VMCNT(0); consume(j, 0, true_type{});
          }
        }

          const bool last = (info1 >> 6) & 1;
          const bool flush = last || (j1 == nt && chunk_ends_here);
          // the next tile of this wavefront (next segment, next group or next chunk) and, if a
          // new segment starts there, its query go in flight before anything is flushed
          if (j1 < nt) {
            sp = __builtin_amdgcn_readlane(d_sp, j1);
            issue(j1, 0);
            load_q(sp);
          } else {
            const u32x4* nx = nullptr;
            if (r0 + kWaveSize < ntb) nx = dtab + r0 + kWaveSize;
            else if (chunk_ends_here && has_next) nx = dtabs + (tab ^ 1) * kDescBatch;
            if (nx != nullptr) {
              const u32x4 pd = *nx;
              issue_at((uint32_t)rfl((int)pd[0]), (uint32_t)rfl((int)pd[1]), 0);
              if (flush) {
                sp = rfl((int)pd[2]);
                load_q(sp);
              }
              inflight = true;
            }
          }

          if (flush) {
          // ---- flush the open segment ----------------------------------------------------------
          const int seq = seg_sp >> 8, pp = seg_sp & 255;
          const int kvh = pp / p.group_tiles, gtile = pp - kvh * p.group_tiles;
          const int h0 = kvh * p.group + gtile * GH;
          const int nheads = min(GH, p.group - gtile * GH);
          const bool first = (seg_info0 >> 5) & 1;
          const int prank = seq * NP + pp;

#pragma unroll
          for (int r = 0; r < 4; ++r) l[r] = row16_sum(l[r]);
          // (m, l) of every head slot to every lane
          *reinterpret_cast<f32x4*>(pbuf + 4 * q4) = f32x4{m[0], m[1], m[2], m[3]};
          *reinterpret_cast<f32x4*>(pbuf + 16 + 4 * q4) = f32x4{l[0], l[1], l[2], l[3]};
          float mg[GH], lg[GH];
#pragma unroll
          for (int g = 0; g < GH; ++g) { mg[g] = pbuf[g]; lg[g] = pbuf[16 + g]; }
          // Sum the accumulators of the four row groups.  Row group q only writes heads g with
          // g % 4 == q, so this is a reduce-scatter: every lane parks its 8 values of head g in
          // LDS (K ring stage 1 is idle during a flush: the tile in flight goes to stage 0) and
          // the lanes of row group g % 4 add the other three groups' values, in fixed order.
          {
            float* red = reinterpret_cast<float*>(wlds + kTileBytes);   // 2 x 2 KiB, alternating
#pragma unroll
            for (int g = 0; g < GH; ++g) {
              float* mine = red + (g & 1) * 512 + (q4 * 16 + t16) * 8;
              *reinterpret_cast<f32x4*>(mine) = f32x4{acc[g][0], acc[g][1], acc[g][2], acc[g][3]};
              *reinterpret_cast<f32x4*>(mine + 4) = f32x4{acc[g][4], acc[g][5], acc[g][6], acc[g][7]};
              if ((g & 3) == q4) {
#pragma unroll
                for (int r = 1; r < 4; ++r) {
                  const float* theirs = red + (g & 1) * 512 + (((q4 + r) & 3) * 16 + t16) * 8;
                  const f32x4 a = *reinterpret_cast<const f32x4*>(theirs);
                  const f32x4 b = *reinterpret_cast<const f32x4*>(theirs + 4);
                  acc[g][0] += a[0]; acc[g][1] += a[1]; acc[g][2] += a[2]; acc[g][3] += a[3];
                  acc[g][4] += b[0]; acc[g][5] += b[1]; acc[g][6] += b[2]; acc[g][7] += b[3];
                }
              }
            }
          }

          if (first && last) {
            // the whole (sequence, pair) was in this segment: finished rows
#pragma unroll
            for (int g = 0; g < GH; ++g) {
              if ((g & 3) == q4 && g < nheads) {
                const float inv = 1.0f / lg[g];
                const int64_t o = ((int64_t)seq * p.num_q_heads + h0 + g) * D + t16 * 8;
                if (p.out_is_bf16) {
                  u32x4 w;
#pragma unroll
                  for (int e = 0; e < 4; ++e)
                    w[e] = pack_bf16x2_rne(acc[g][2 * e] * inv, acc[g][2 * e + 1] * inv);
                  *reinterpret_cast<u32x4*>(reinterpret_cast<uint16_t*>(p.out) + o) = w;
                } else {
                  float* op = reinterpret_cast<float*>(p.out) + o;
                  *reinterpret_cast<f32x4*>(op) =
                      f32x4{acc[g][0] * inv, acc[g][1] * inv, acc[g][2] * inv, acc[g][3] * inv};
                  *reinterpret_cast<f32x4*>(op + 4) =
                      f32x4{acc[g][4] * inv, acc[g][5] * inv, acc[g][6] * inv, acc[g][7] * inv};
                }
              }
            }
            if (lane == 0) *reinterpret_cast<i32x2*>(p.ws_dir + 2 * (int64_t)prank) = i32x2{0, 1};
          } else {
            const int64_t slot = (int64_t)prank + c;   // unique: both terms grow along the axis
#pragma unroll
            for (int g = 0; g < GH; ++g) {
              if ((g & 3) == q4 && g < nheads) {
                float* op = p.ws_o + (slot * GH + g) * D + t16 * 8;
                *reinterpret_cast<f32x4*>(op) = f32x4{acc[g][0], acc[g][1], acc[g][2], acc[g][3]};
                *reinterpret_cast<f32x4*>(op + 4) = f32x4{acc[g][4], acc[g][5], acc[g][6], acc[g][7]};
                if (t16 == 0)
                  *reinterpret_cast<f32x2*>(p.ws_ml + (slot * GH + g) * 2) = f32x2{mg[g], lg[g]};
              }
            }
            if (first && lane == 0) {
              // directory entry of the pair: its partials sit in consecutive slots
              const int tiles = seg_info0 >> 8;
              const int c_last = plan.chunk_of(seg_x + tiles - 1);
              *reinterpret_cast<i32x2*>(p.ws_dir + 2 * (int64_t)prank) = i32x2{(int)slot, c_last - c + 1};
            }
          }
          open = false;
          }
          j0 = j1;
        }
      }
    }
    tab ^= 1;
  }
}

constexpr int kMergeThreads = 256, kMW = kMergeThreads / kWaveSize;

template <int GH>
__global__ __launch_bounds__(kMergeThreads) void attn_stream_merge(const AttnParams p) {
  __shared__ float sM[kMW], sL[kMW];
  __shared__ __attribute__((aligned(16))) float sO[kMW][D];
  const int h = blockIdx.x, seq = blockIdx.y, tid = threadIdx.x;
  const int lane = tid & (kWaveSize - 1), wave = tid / kWaveSize;
  const int kvh = h / p.group, gi = h - kvh * p.group;
  const int gtile = gi / GH, g = gi - gtile * GH;
  const int64_t prank = ((int64_t)seq * p.num_kv_heads + kvh) * p.group_tiles + gtile;
  const int n = p.context_lens[seq];
  const int64_t o = ((int64_t)seq * p.num_q_heads + h) * D;
  if (n <= 0) {                          // block-uniform
    if (tid < D) {
      if (p.out_is_bf16) reinterpret_cast<uint16_t*>(p.out)[o + tid] = 0;
      else reinterpret_cast<float*>(p.out)[o + tid] = 0.f;
    }
    return;
  }
  const i32x2 de = *reinterpret_cast<const i32x2*>(p.ws_dir + 2 * prank);
  const int count = de[1];
  if (count <= 1) return;                // finished by the stream kernel (block-uniform)
  const int64_t s0 = de[0];
  const float* ml = p.ws_ml + (s0 * GH + g) * 2;            // partial q at ml[q*GH*2]
  const float* ov = p.ws_o + (s0 * GH + g) * D + 2 * lane;  // partial q at ov[q*GH*D]

  // reference maximum over all partials
  float M = kNegBig;
  for (int q = tid; q < count; q += kMergeThreads) M = fmaxf(M, ml[(int64_t)q * GH * 2]);
#pragma unroll
  for (int off = 1; off < kWaveSize; off <<= 1) M = fmaxf(M, __shfl_xor(M, off, kWaveSize));
  if (lane == 0) sM[wave] = M;
  __syncthreads();
  M = fmaxf(fmaxf(sM[0], sM[1]), fmaxf(sM[2], sM[3]));

  // wave w sums partials w, w+4, ... (ascending); lane covers output dims 2*lane, 2*lane+1
  float L = 0.f, O0 = 0.f, O1 = 0.f;
#pragma unroll 4
  for (int q = wave; q < count; q += kMW) {
    const f32x2 mlq = *reinterpret_cast<const f32x2*>(ml + (int64_t)q * GH * 2);
    const f32x2 oq = *reinterpret_cast<const f32x2*>(ov + (int64_t)q * GH * D);
    const float f = __builtin_amdgcn_exp2f(mlq[0] - M);
    L = fmaf(mlq[1], f, L);
    O0 = fmaf(oq[0], f, O0);
    O1 = fmaf(oq[1], f, O1);
  }
  sO[wave][2 * lane] = O0;
  sO[wave][2 * lane + 1] = O1;
  if (lane == 0) sL[wave] = L;
  __syncthreads();
  if (tid < D) {
    const float Lt = (sL[0] + sL[1]) + (sL[2] + sL[3]);
    const float r = ((sO[0][tid] + sO[1][tid]) + (sO[2][tid] + sO[3][tid])) / Lt;
    if (p.out_is_bf16) reinterpret_cast<uint16_t*>(p.out)[o + tid] = (uint16_t)(pack_bf16x2_rne(r, 0.f) & 0xFFFFu);
    else reinterpret_cast<float*>(p.out)[o + tid] = r;
  }
}

int num_cus() {
  static int cached = 0;
  if (cached == 0) {
    int dev = 0, v = 0;
    if (hipGetDevice(&dev) == hipSuccess &&
        hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && v > 0)
      cached = v;
    else
      cached = 256;
  }
  return cached;
}

template <int GH>
hipError_t launch(const AttnParams& p, hipStream_t s) {
  const size_t lds = (size_t)p.prefix_bytes + (size_t)kNW * kWaveLds;
  static bool prepared = false;   // more than 64 KiB of dynamic LDS has to be asked for once
  if (!prepared) {
    const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&attn_stream_mfma_d128<GH>),
                                             hipFuncAttributeMaxDynamicSharedMemorySize,
                                             kStreamMaxPrefixBytes + kNW * kWaveLds);
    if (e != hipSuccess) return e;
    prepared = true;
  }
  if (p.ev_begin && hipEventRecord(p.ev_begin, s) != hipSuccess) return hipErrorInvalidValue;
  hipLaunchKernelGGL((attn_stream_mfma_d128<GH>), dim3(num_cus()), dim3(kStreamThreads), lds, s, p);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  if (p.ev_end && hipEventRecord(p.ev_end, s) != hipSuccess) return hipErrorInvalidValue;
  hipLaunchKernelGGL((attn_stream_merge<GH>), dim3(p.num_q_heads, p.batch), dim3(kMergeThreads), 0, s, p);
  return hipGetLastError();
}

}  // namespace

int stream_heads_per_lane(int group) { return group == 1 ? 1 : group == 2 ? 2 : group <= 4 ? 4 : 8; }

// bf16, head_dim 128, power-of-two block size, pools addressable with 32-bit 16-byte units,
// batch small enough for the prefix table in LDS.
bool attn_stream_supported(const pkv_attn_desc& d) {
  const int tpb = d.block_size / kTileTokens;
  const int G = d.num_q_heads / d.num_kv_heads;
  const int gh = stream_heads_per_lane(G);
  const int64_t np = (int64_t)d.num_kv_heads * ((G + gh - 1) / gh);
  const int64_t tiles_ub = ((int64_t)d.max_context_len + kTileTokens - 1) / kTileTokens * d.batch * np;
  auto span = [&](int64_t sb, int64_t sh, int64_t st) {
    return ((int64_t)d.num_pool_blocks * sb + (int64_t)d.num_kv_heads * sh + (int64_t)d.block_size * st) * 2;
  };
  return d.kv_dtype == PKV_BF16 && d.head_dim == 128 && tpb >= 1 && (tpb & (tpb - 1)) == 0 &&
         !(d.flags & PKV_ATTN_FLAG_VECTOR_ALU) && np <= 256 && d.batch < (1 << 23) &&
         (int64_t)(d.batch + 1) * 4 <= kStreamMaxPrefixBytes && tiles_ub < (1ll << 30) &&
         d.k_stride_token * 2 * 16 < (1 << 30) && d.v_stride_token * 2 * 16 < (1 << 30) &&
         span(d.k_stride_block, d.k_stride_head, d.k_stride_token) < (1ll << 36) &&
         span(d.v_stride_block, d.v_stride_head, d.v_stride_token) < (1ll << 36);
}

// Workspace: directory [pairs][2] int32, then (m, l) [slots][GH][2], then rows [slots][GH][D].
StreamWorkspace stream_workspace(const pkv_attn_desc& d) {
  StreamWorkspace w;
  const int G = d.num_q_heads / d.num_kv_heads;
  const int gh = stream_heads_per_lane(G);
  const int64_t np = (int64_t)d.num_kv_heads * ((G + gh - 1) / gh);
  const int64_t pairs = (int64_t)d.batch * np;
  const int64_t tiles_ub = ((int64_t)d.max_context_len + kTileTokens - 1) / kTileTokens * pairs;
  const int pt = d.partition_tokens == 0 ? kDefaultPartition : d.partition_tokens;
  // partition_tokens 0: no cap on what one wavefront accumulates before it writes a partial
  w.chunk_tiles_max = d.partition_tokens == 0 ? 0 : pt / kTileTokens;
  // chunk ids stay below workgroups * chunks-per-workgroup, see plan_chunks()
  const int64_t ncu = num_cus();
  const int64_t cap = w.chunk_tiles_max;
  w.slots = pairs + (cap ? (tiles_ub + kMinGroupTiles * ncu) / cap + ncu : 0) + ncu * (kNW + 1) + 2;
  auto up = [](int64_t b) { return (b + 255) / 256 * 256; };
  w.dir_bytes = up(pairs * 2 * 4);
  w.ml_bytes = up(w.slots * gh * 2 * 4);
  w.o_bytes = up(w.slots * gh * D * 4);
  return w;
}

hipError_t launch_attn_stream(AttnParams& p, hipStream_t s) {
  p.tpb_shift = 0;
  while ((kTileTokens << p.tpb_shift) < p.block_size) ++p.tpb_shift;
  p.prefix_bytes = ((p.batch + 1) * 4 + 15) / 16 * 16;
  const int gh = stream_heads_per_lane(p.group);
  p.group_tiles = (p.group + gh - 1) / gh;
  switch (gh) {
    case 1: return launch<1>(p, s);
    case 2: return launch<2>(p, s);
    case 4: return launch<4>(p, s);
    default: return launch<8>(p, s);
  }
}

}  // namespace pkv
