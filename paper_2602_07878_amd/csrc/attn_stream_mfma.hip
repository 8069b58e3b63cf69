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
// Per tile (the vector ALU, not HBM, limits this kernel as soon as the per-token work is
// done with ordinary FMAs, so everything that is a contraction runs on the matrix cores):
//  * K and V go HBM -> LDS with direct-to-LDS 16-byte loads (no VGPR staging) into a
//    2-deep ring per wavefront.  Both LDS images are XOR-swizzled by choosing which
//    16-byte piece of its token row each lane fetches, so the reads that feed the matrix
//    cores are bank-conflict free while every wave-wide global load still covers whole
//    contiguous 256-byte rows.
//  * scores S^T[token][head] = K Q_g^T come from v_mfma_f32_16x16x32_bf16 (both operands
//    exact bf16; column c of the tile is query head c of the group).  In the result a lane
//    holds four tokens of one head: exactly the A-operand layout of the second product.
//  * the running maximum is only a reference point for exp2(): it is raised (and the
//    accumulators rescaled) only when a score exceeds it by more than kSlack, so the
//    common tile needs no cross-lane reduction at all; row sums stay per lane until the
//    flush.
//  * the fp32 weights are split into a bf16 head and a bf16 remainder (relative error
//    2^-17) and O[head][dim] += P V runs as two v_mfma_f32_16x16x16_bf16 per 16 output
//    dims; the B operand (four tokens of one dim per lane) comes out of the row-major V
//    tile with the transposing LDS read ds_read_b64_tr_b16.
// The loads of tile j+1 are in flight while tile j is consumed; the first tile of the
// next segment is issued before the current segment is flushed.

#include <atomic>
#include <type_traits>

#include <hip/hip_ext.h>

#include "attn_stream_common.h"

namespace pkv {
namespace {

// GH = query heads accumulated per lane (1, 2, 4 or 8).
template <int GH>
__global__ __launch_bounds__(kStreamThreads, 2) void attn_stream_mfma_d128(const AttnParams p) {
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
  const int g0 = plan.bound(blockIdx.x);                   // first tile of this workgroup's range
  const int gfull = plan.length(blockIdx.x);
  const int glen = min(gfull, T - g0);                     // its length (<= 0: nothing to do)
  if (glen <= 0) return;
  // ---- per-lane, loop-invariant offsets -------------------------------------------------------
  // Load j of a tile brings token rows 4j..4j+3; this lane fetches one 16-byte piece of row
  // 4j+q4 and the hardware puts it at LDS slot (j, lane).  Which piece it fetches fixes the swizzle:
  // K row t keeps piece c at slot c ^ t, V row t keeps piece c at slot c ^ 2(t mod 8).
  uint32_t koff[4], voff[4], krd[4], vrd[8];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int tok = 4 * j + q4;
    koff[j] = (uint32_t)(tok * p.k_stride_token) + (uint32_t)((t16 ^ tok) * 16);
    voff[j] = (uint32_t)(tok * p.v_stride_token) + (uint32_t)((t16 ^ (2 * (tok & 7))) * 16);
    // first product, step j: this lane (token t16) needs dims 32j+8q4..+7 of its K row
    krd[j] = (uint32_t)(t16 * 256 + (((4 * j + q4) ^ t16) * 16));
  }
  {
    // second product, output dims 16nb..16nb+15: the transposing read hands lane i of a 16-lane
    // group element (i mod 4) of the 8-byte pieces addressed by lanes i/4, 4+i/4, 8+i/4, 12+i/4.
    // Lane s of group q4 therefore points at token 4q4 + s/4, dims 16nb + 4(s mod 4)..+3, and
    // every lane receives tokens 4q4..4q4+3 of dim 16nb + t16: the B operand.
    const int tv = 4 * q4 + (t16 >> 2);
    const uint32_t vbase = (uint32_t)(tv * 256 + ((tv & 7) << 5) + (t16 & 3) * 8);
#pragma unroll
    for (int nb = 0; nb < 8; ++nb) vrd[nb] = vbase ^ (uint32_t)(nb << 5);
  }
  uint8_t* wlds = lds + p.prefix_bytes + wave * kWaveLds;
  {
    // as LDS byte addresses (a common shift of all addresses leaves the bank pattern conflict free)
    const uint32_t wbase = (uint32_t)(uintptr_t)(lptr_t)wlds;
#pragma unroll
    for (int nb = 0; nb < 8; ++nb) vrd[nb] += wbase;
  }
  float* xchg = reinterpret_cast<float*>(wlds + kStages * kStageBytes);   // 128 floats
  const uint8_t* kpool = reinterpret_cast<const uint8_t*>(p.k_pool);
  const uint8_t* vpool = reinterpret_cast<const uint8_t*>(p.v_pool);
  const int tile_mask = (1 << p.tpb_shift) - 1;

  int tiles_done = 0;
  // Softmax state of head column t16 (the same value in the four lanes that share a column):
  // reference maximum, and this lane's share of the row sum (tokens 4q4..4q4+3 of every tile).
  float m_ref = kNegBig, l_part = 0.f;
  f32x4 acc[8];          // O[head 4q4+r][dim 16nb+t16] in acc[nb][r]
  bf16x8 qfrag[4];

  // two descriptor tables per wavefront: the one in use and the one filled ahead for the next batch
  u32x4* dtabs = reinterpret_cast<u32x4*>(wlds + kStages * kStageBytes + kXchgBytes);   // [2][kDescBatch]

  // Tile descriptors of `count` (<= kDescBatch) tiles from axis position xb, one per lane:
  //   x: byte offset / 16 of the tile's first K row      y: same for V
  //   z: sequence << 8 | pair
  //   w: valid tokens (1..16) | first-of-pair << 5 | last-of-pair << 6 | tiles of the pair << 8
  auto build_desc = [&](int xb, int count, u32x4* tab) {
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
    d[3] = (uint32_t)(ntok | ((t == 0) << 5) | ((t == tiles - 1) << 6) | (tiles << 8));
    tab[lane] = d;
  };

  int d_k = 0, d_v = 0, d_sp = 0, d_info = 0;   // descriptors of the current batch, one tile per lane

  auto issue_at = [&](uint32_t sk, uint32_t sv, int stage) {
    const uint8_t* kb = kpool + ((uint64_t)sk << 4);
    const uint8_t* vb = vpool + ((uint64_t)sv << 4);
    uint8_t* kl = wlds + stage * kStageBytes;
#pragma unroll
    for (int jj = 0; jj < 4; ++jj)
      __builtin_amdgcn_global_load_lds((gptr_t)(kb + koff[jj]), (lptr_t)(kl + jj * 1024), 16, 0, 2);
#pragma unroll
    for (int jj = 0; jj < 4; ++jj)
      __builtin_amdgcn_global_load_lds((gptr_t)(vb + voff[jj]), (lptr_t)(kl + kTileBytes + jj * 1024), 16, 0, 2);
  };
  auto issue = [&](int j, int stage) {
    issue_at((uint32_t)__builtin_amdgcn_readlane(d_k, j), (uint32_t)__builtin_amdgcn_readlane(d_v, j), stage);
  };

  // Query rows as the B operand of the first product: column t16 is head min(t16, nheads-1)
  // of the group (columns past the group repeat its last head and are never written out).
  auto load_q = [&](int sp) {
    const int seq = sp >> 8, pp = sp & 255;
    const int kvh = pp / p.group_tiles, gtile = pp - kvh * p.group_tiles;
    const int h0 = kvh * p.group + gtile * GH;
    const int nheads = min(GH, p.group - gtile * GH);
    const int hs = min(t16, nheads - 1);
    const uint8_t* qp = reinterpret_cast<const uint8_t*>(p.q) +
                        ((int64_t)seq * p.num_q_heads + h0 + hs) * (D * 2) + q4 * 16;
#pragma unroll
    for (int cidx = 0; cidx < 4; ++cidx)
      qfrag[cidx] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(qp + cidx * 64));
  };

  // TAIL: the tile may hold fewer than 16 valid tokens (only the last tile of a pair can)
  auto consume = [&](int j, auto stage_tag, auto tail_tag) {
    constexpr int STAGE = decltype(stage_tag)::value;
    constexpr bool TAIL = decltype(tail_tag)::value;
    const int ntok = TAIL ? (__builtin_amdgcn_readlane(d_info, j) & 31) : kTileTokens;
    const uint8_t* kl = wlds + STAGE * kStageBytes;
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
      if (TAIL && 4 * q4 + r >= ntok) d[r] = -INFINITY;   // stale slot: may hold NaN bits
    }
    const float dmax = fmaxf(fmaxf(d[0], d[1]), fmaxf(d[2], d[3]));
    if (__builtin_amdgcn_ballot_w64(dmax > kSlack) != 0) {   // wave-uniform, rare after a first tile
      float s[4];
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        s[r] = cfr[r] * p.scale_log2e;
        if (TAIL && 4 * q4 + r >= ntok) s[r] = -INFINITY;
      }
      xchg[q4 * 16 + t16] = fmaxf(fmaxf(s[0], s[1]), fmaxf(s[2], s[3]));
      const float tm = fmaxf(fmaxf(xchg[t16], xchg[16 + t16]), fmaxf(xchg[32 + t16], xchg[48 + t16]));
      const float mn = fmaxf(m_ref, tm);
      const float alpha = __builtin_amdgcn_exp2f(m_ref - mn);
      m_ref = mn;
      l_part *= alpha;
#pragma unroll
      for (int r = 0; r < 4; ++r) d[r] = s[r] - mn;
      // the accumulators of this lane belong to heads 4q4..4q4+3
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

    uint32_t keep0 = 0xFFFFFFFFu, keep1 = 0xFFFFFFFFu;   // V rows past the context: zero, not NaN
    if (TAIL) {
      keep0 = (4 * q4 + 0 < ntok ? 0x0000FFFFu : 0u) | (4 * q4 + 1 < ntok ? 0xFFFF0000u : 0u);
      keep1 = (4 * q4 + 2 < ntok ? 0x0000FFFFu : 0u) | (4 * q4 + 3 < ntok ? 0xFFFF0000u : 0u);
    }
    // The transposing reads are written out by hand: through the compiler's builtin each of
    // them would be preceded by a wait for every outstanding direct-to-LDS load, i.e. for the
    // whole next tile, which would undo the prefetch.  The data they read is complete (the
    // wait before this call covered the tile's eight loads).
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
          "v"(vrd[7]), "n"(STAGE * kStageBytes + kTileBytes)
        : "memory");
    s16x4 vf[8];
#pragma unroll
    for (int nb = 0; nb < 8; ++nb) {
      if (TAIL) { vt[nb][0] &= keep0; vt[nb][1] &= keep1; }
      vf[nb] = __builtin_bit_cast(s16x4, vt[nb]);
    }
#pragma unroll
    for (int nb = 0; nb < 8; ++nb)
      acc[nb] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(p_hi, vf[nb], acc[nb], 0, 0, 0);
#pragma unroll
    for (int nb = 0; nb < 8; ++nb)
      acc[nb] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(p_lo, vf[nb], acc[nb], 0, 0, 0);

    // The two wavefronts that share a SIMD (w and w+4) do not get equal issue slots: the
    // older one wins every tie.  Whoever is behind raises its priority until it catches up.
    ++tiles_done;
    if (lane == 0) progress[wave] = tiles_done;
    if (progress[wave ^ (kNW / 2)] > tiles_done) __builtin_amdgcn_s_setprio(2);
    else __builtin_amdgcn_s_setprio(0);
  };

  // state of the segment being accumulated (may span batches of one chunk) and of the pipeline
  bool open = false;        // a segment is being accumulated
  bool inflight = false;    // the first tile of the coming batch is already issued, its query loaded
  int seg_sp = 0, seg_info0 = 0, seg_x = 0, sp = 0, tab = 0;

  auto chunk_first = [&](int ci) { return plan.chunk_start(gfull, ci); };
  auto chunk_valid = [&](int ci) { return ci < plan.ns && chunk_first(ci) < glen; };
  auto chunk_tiles = [&](int ci) { return min(glen, chunk_first(ci + 1)) - chunk_first(ci); };

  // A wavefront's work is a sequence of batches of up to kDescBatch tiles: the batches of its
  // first chunk, then those of its next chunk (local ids wave, wave+8, ...), and so on.
  int ci = wave, b0 = 0;
  bool have = chunk_valid(ci);
  if (have) build_desc(g0 + chunk_first(ci), min(kDescBatch, chunk_tiles(ci)), dtabs);
  while (have) {
    const int c = blockIdx.x * plan.ns + ci;         // chunk id on the whole axis
    const int x0 = g0 + chunk_first(ci);
    const int ntc = chunk_tiles(ci);                 // tiles of this chunk
    const int nt = min(kDescBatch, ntc - b0);        // tiles of this batch, one descriptor per lane
    const bool chunk_ends_here = b0 + nt == ntc;
    int nci = ci, nb0 = b0 + kDescBatch;             // the batch after this one
    bool has_next = true;
    if (chunk_ends_here) { nci = ci + kNW; nb0 = 0; has_next = chunk_valid(nci); }
    const u32x4* dtab = dtabs + tab * kDescBatch;
    u32x4* dnext = dtabs + (tab ^ 1) * kDescBatch;
    {
      const u32x4 dreg = dtab[min(lane, nt - 1)];
      d_k = (int)dreg[0]; d_v = (int)dreg[1]; d_sp = (int)dreg[2]; d_info = (int)dreg[3];
    }

    int j0 = 0;
    if (!inflight) {
      sp = __builtin_amdgcn_readlane(d_sp, 0);
      issue(0, 0);
      if (!open) load_q(sp);                    // an open segment continues with its query
    }
    inflight = false;
    // describe the next batch now: its index loads ride along with the tile that is in flight
    if (has_next) build_desc(g0 + chunk_first(nci) + nb0, min(kDescBatch, chunk_tiles(nci) - nb0), dnext);

    while (j0 < nt) {
      // tiles j0 .. j1-1 belong to (sequence, pair) sp; the first one is already in flight
      const uint64_t same = __builtin_amdgcn_ballot_w64(d_sp == sp && lane >= j0 && lane < nt);
      const int j1 = j0 + __builtin_popcountll(same);
      const int info1 = __builtin_amdgcn_readlane(d_info, j1 - 1);

      if (!open) {
        open = true;
        seg_sp = sp;
        seg_info0 = __builtin_amdgcn_readlane(d_info, j0);
        seg_x = x0 + b0 + j0;
        m_ref = kNegBig;
        l_part = 0.f;
#pragma unroll
        for (int nb = 0; nb < 8; ++nb) acc[nb] = f32x4{0.f, 0.f, 0.f, 0.f};
      }

      {
        using std::false_type;
        using std::true_type;
        using stage0 = std::integral_constant<int, 0>;
        using stage1 = std::integral_constant<int, 1>;
        int j = j0;
        while (j + 2 < j1) {
          issue(j + 1, 1); PKV_WAIT_VMCNT(8); consume(j, stage0{}, false_type{});
          issue(j + 2, 0); PKV_WAIT_VMCNT(8); consume(j + 1, stage1{}, false_type{});
          j += 2;
        }
        if (j + 2 == j1) {
          issue(j + 1, 1); PKV_WAIT_VMCNT(8); consume(j, stage0{}, false_type{});
          PKV_WAIT_VMCNT(0); consume(j + 1, stage1{}, true_type{});
        } else {
          PKV_WAIT_VMCNT(0); consume(j, stage0{}, true_type{});
        }
      }

      const bool last = (info1 >> 6) & 1;
      const bool flush = last || (j1 == nt && chunk_ends_here);
      // the next tile of this wavefront (next segment, next batch or next chunk) and, if a
      // new segment starts there, its query go in flight before anything is flushed
      if (j1 < nt) {
        sp = __builtin_amdgcn_readlane(d_sp, j1);
        issue(j1, 0);
        load_q(sp);
      } else if (has_next) {
        const u32x4 pd = dnext[0];
        issue_at((uint32_t)rfl((int)pd[0]), (uint32_t)rfl((int)pd[1]), 0);
        if (flush) {
          sp = rfl((int)pd[2]);
          load_q(sp);
        }
        inflight = true;
      }

      if (flush) {
        // ---- flush the open segment ------------------------------------------------------------
        const int seq = seg_sp >> 8, pp = seg_sp & 255;
        const int kvh = pp / p.group_tiles, gtile = pp - kvh * p.group_tiles;
        const int h0 = kvh * p.group + gtile * GH;
        const int nheads = min(GH, p.group - gtile * GH);
        const bool first = (seg_info0 >> 5) & 1;
        const int prank = seq * NP + pp;

        // row-sum shares and reference maxima of all head columns, for every lane to read
        xchg[q4 * 16 + t16] = l_part;
        xchg[64 + t16] = m_ref;
        // O goes through LDS to turn the accumulator layout (lane = one dim of four heads) into
        // whole rows: stage 1 of the ring is idle during a flush, the tile in flight uses stage 0
        float* st = reinterpret_cast<float*>(wlds + kStageBytes);
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
              // the whole (sequence, pair) was in this segment: finished rows
              const float inv = 1.0f / lsum;
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
                // (the empty statements keep the compiler from merging the two stores into a plain one)
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
        if (lane == 0) {
          if (first && last) {
            *reinterpret_cast<i32x2*>(p.ws_dir + 2 * (int64_t)prank) = i32x2{0, 1};
          } else if (first) {
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
    tab ^= 1;
    ci = nci;
    b0 = nb0;
    have = has_next;
  }
}


constexpr int kMergeThreads = 256, kMW = kMergeThreads / kWaveSize;

// Calls with a per-step plan: whether the plan is one for this call (else the output is filled
// with NaN).
__device__ __forceinline__ bool plan_ok(const AttnParams& p) {
  return !p.plan_hdr || p.plan_hdr[kPlanKey] == p.plan_key;
}

template <int GH>
__global__ __launch_bounds__(kMergeThreads) void attn_stream_merge(const AttnParams p) {
  __shared__ float sM[kMW], sL[2 * kMW];
  __shared__ __attribute__((aligned(16))) float sO[2 * kMW][D];
  const int h = blockIdx.x, seq = blockIdx.y, tid = threadIdx.x;
  const int lane = tid & (kWaveSize - 1), wave = tid / kWaveSize;
  const int kvh = h / p.group, gi = h - kvh * p.group;
  const int gtile = gi / GH, g = gi - gtile * GH;
  const int64_t prank = ((int64_t)seq * p.num_kv_heads + kvh) * p.group_tiles + gtile;
  const int n = p.context_lens[seq];
  const i32x2 de = *reinterpret_cast<const i32x2*>(p.ws_dir + 2 * prank);   // (requested with the length, not behind it)
  const int64_t o = ((int64_t)seq * p.num_q_heads + h) * D;
  if (!plan_ok(p)) {                     // block-uniform
    if (tid < D) {
      if (p.out_is_bf16) reinterpret_cast<uint16_t*>(p.out)[o + tid] = 0x7FC0;
      else reinterpret_cast<float*>(p.out)[o + tid] = __builtin_nanf("");
    }
    return;
  }
  if (n <= 0) {                          // block-uniform
    if (tid < D) {
      if (p.out_is_bf16) reinterpret_cast<uint16_t*>(p.out)[o + tid] = 0;
      else reinterpret_cast<float*>(p.out)[o + tid] = 0.f;
    }
    return;
  }
  const int count = de[1];
  if (count <= 1) return;                // finished by the stream kernel (block-uniform)
  const int64_t s0 = de[0];
  const float* ml = p.ws_ml + (s0 * GH + g) * 2;            // partial q at ml[q*GH*2]
  // a partial's row is 32 pieces of 16 bytes: each half of a wavefront takes one partial per step
  const int half = lane >> 5, l32 = lane & 31;
  const float* ov = p.ws_o + (s0 * GH + g) * D + 4 * l32;   // partial q at ov[q*GH*D]

  // reference maximum over all partials
  float M = kNegBig;
  for (int q = tid; q < count; q += kMergeThreads) M = fmaxf(M, ml[(int64_t)q * GH * 2]);
#pragma unroll
  for (int off = 1; off < kWaveSize; off <<= 1) M = fmaxf(M, __shfl_xor(M, off, kWaveSize));
  if (lane == 0) sM[wave] = M;
  __syncthreads();
  M = fmaxf(fmaxf(sM[0], sM[1]), fmaxf(sM[2], sM[3]));

  // half-wavefront u = 2 * wave + half sums partials u, u+8, ... (ascending), eight rows in
  // flight each; a lane covers output dims 4*l32 .. 4*l32+3
  float L = 0.f;
  f32x4 O = {0.f, 0.f, 0.f, 0.f};
#pragma unroll 8
  for (int q = 2 * wave + half; q < count; q += 2 * kMW) {
    const f32x2 mlq = *reinterpret_cast<const f32x2*>(ml + (int64_t)q * GH * 2);
    const f32x4 oq = *reinterpret_cast<const f32x4*>(ov + (int64_t)q * GH * D);
    const float f = __builtin_amdgcn_exp2f(mlq[0] - M);
    L = fmaf(mlq[1], f, L);
#pragma unroll
    for (int i = 0; i < 4; ++i) O[i] = fmaf(oq[i], f, O[i]);
  }
  *reinterpret_cast<f32x4*>(&sO[2 * wave + half][4 * l32]) = O;
  if (l32 == 0) sL[2 * wave + half] = L;
  __syncthreads();
  if (tid < D) {
    const float Lt = ((sL[0] + sL[1]) + (sL[2] + sL[3])) + ((sL[4] + sL[5]) + (sL[6] + sL[7]));
    const float r = (((sO[0][tid] + sO[1][tid]) + (sO[2][tid] + sO[3][tid])) +
                     ((sO[4][tid] + sO[5][tid]) + (sO[6][tid] + sO[7][tid]))) / Lt * p.v_scale;
    if (p.out_is_bf16) reinterpret_cast<uint16_t*>(p.out)[o + tid] = (uint16_t)(pack_bf16x2_rne(r, 0.f) & 0xFFFFu);
    else reinterpret_cast<float*>(p.out)[o + tid] = r;
  }
}

// Merge for the library's own split, where a pair has a handful of partials: one workgroup per
// (sequence, pair), one wavefront per query head, no LDS and no barrier.  A wavefront walks its
// head's partials in ascending order, eight loads in flight, rescaling the running sums when
// the reference maximum rises; lane covers output dims 2*lane and 2*lane+1.
template <int GH>
__global__ __launch_bounds__(GH * kWaveSize) void attn_stream_merge_lean(const AttnParams p) {
  const int NP = p.num_kv_heads * p.group_tiles;
  const int prank = blockIdx.x;
  const int seq = prank / NP, pp = prank - seq * NP;
  const int kvh = pp / p.group_tiles, gtile = pp - kvh * p.group_tiles;
  const int lane = threadIdx.x & (kWaveSize - 1), g = threadIdx.x / kWaveSize;
  // everything the decisions below depend on is requested at once (the kernel is a chain of
  // dependent loads; the directory entry exists for every pair, also for empty contexts)
  const int n = p.context_lens[seq];
  const i32x2 de = *reinterpret_cast<const i32x2*>(p.ws_dir + 2 * (int64_t)prank);
  const bool ok = plan_ok(p);
  if (gtile * GH + g >= p.group) return;               // wave-uniform
  const int h = kvh * p.group + gtile * GH + g;
  const int64_t o = ((int64_t)seq * p.num_q_heads + h) * D + 2 * lane;
  auto store = [&](float a, float b) {
    if (p.out_is_bf16) reinterpret_cast<uint32_t*>(p.out)[o / 2] = pack_bf16x2_rne(a, b);
    else *reinterpret_cast<f32x2*>(reinterpret_cast<float*>(p.out) + o) = f32x2{a, b};
  };
  if (!ok) { store(__builtin_nanf(""), __builtin_nanf("")); return; }
  if (n <= 0) { store(0.f, 0.f); return; }
  const int count = de[1];
  if (count <= 1) return;                               // finished by the stream kernel
  const int64_t s0 = de[0];
  const float* ml = p.ws_ml + (s0 * GH + g) * 2;            // partial q at ml[q*GH*2]
  const float* ov = p.ws_o + (s0 * GH + g) * D + 2 * lane;  // partial q at ov[q*GH*D]
  float M = kNegBig, L = 0.f, O0 = 0.f, O1 = 0.f;
  for (int q0 = 0; q0 < count; q0 += 8) {
    f32x2 mlq[8], oq[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const bool live = q0 + i < count;
      const int64_t q = live ? q0 + i : q0;
      mlq[i] = *reinterpret_cast<const f32x2*>(ml + q * GH * 2);
      oq[i] = *reinterpret_cast<const f32x2*>(ov + q * GH * D);
      if (!live) { mlq[i] = f32x2{kNegBig, 0.f}; oq[i] = f32x2{0.f, 0.f}; }
    }
    float Mb = M;
#pragma unroll
    for (int i = 0; i < 8; ++i) Mb = fmaxf(Mb, mlq[i][0]);
    const float fo = __builtin_amdgcn_exp2f(M - Mb);
    L *= fo; O0 *= fo; O1 *= fo;
    M = Mb;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const float f = __builtin_amdgcn_exp2f(mlq[i][0] - M);
      L = fmaf(mlq[i][1], f, L);
      O0 = fmaf(oq[i][0], f, O0);
      O1 = fmaf(oq[i][1], f, O1);
    }
  }
  const float inv = (1.0f / L) * p.v_scale;
  store(O0 * inv, O1 * inv);
}

template <int GH>
hipError_t launch(const AttnParams& p, hipStream_t s) {
  hipError_t e;
  if (p.kv_is_f8 || p.plan_hdr) {
    e = launch_attn_flat(p, GH, s);
  } else {
    const size_t lds = (size_t)p.prefix_bytes + (size_t)kNW * kWaveLds;
    if ((e = prepare_attn_stream()) != hipSuccess) return e;
    // with events: attached to the dispatch itself, so they carry the kernel's own begin and end
    if (p.ev_begin || p.ev_end)
      hipExtLaunchKernelGGL((attn_stream_mfma_d128<GH>), dim3(num_cus()), dim3(kStreamThreads), lds, s,
                            p.ev_begin, p.ev_end, 0, p);
    else
      hipLaunchKernelGGL((attn_stream_mfma_d128<GH>), dim3(num_cus()), dim3(kStreamThreads), lds, s, p);
    e = hipGetLastError();
  }
  if (e != hipSuccess) return e;
  if (p.chunk_tiles_max == 0)   // the library's own split: few partials per pair
    hipLaunchKernelGGL((attn_stream_merge_lean<GH>), dim3(p.batch * p.num_kv_heads * p.group_tiles),
                       dim3(GH * kWaveSize), 0, s, p);
  else
    hipLaunchKernelGGL((attn_stream_merge<GH>), dim3(p.num_q_heads, p.batch), dim3(kMergeThreads), 0, s, p);
  return hipGetLastError();
}

}  // namespace

// The stream kernels use more than 64 KiB of dynamic LDS, which has to be asked for once per
// device (devices outside the table are asked every time).
hipError_t prepare_attn_stream() {
  static std::atomic<bool> prepared[kMaxDevices];
  const int slot = device_slot();
  if (slot >= 0 && prepared[slot].load(std::memory_order_acquire)) return hipSuccess;
  for (const void* f : {reinterpret_cast<const void*>(&attn_stream_mfma_d128<1>),
                        reinterpret_cast<const void*>(&attn_stream_mfma_d128<2>),
                        reinterpret_cast<const void*>(&attn_stream_mfma_d128<4>),
                        reinterpret_cast<const void*>(&attn_stream_mfma_d128<8>)}) {
    const hipError_t e = hipFuncSetAttribute(f, hipFuncAttributeMaxDynamicSharedMemorySize,
                                             kStreamMaxPrefixBytes + kNW * kWaveLds);
    if (e != hipSuccess) return e;
  }
  {
    const hipError_t e = prepare_attn_flat();
    if (e != hipSuccess) return e;
  }
  if (slot >= 0) prepared[slot].store(true, std::memory_order_release);
  return hipSuccess;
}

// CUs of the current device (cached per device).
int num_cus() {
  static std::atomic<int> cached[kMaxDevices];   // zero-initialised: not asked yet
  const int slot = device_slot();
  int v = slot >= 0 ? cached[slot].load(std::memory_order_relaxed) : 0;
  if (v == 0) {
    int dev = 0;
    if (!(hipGetDevice(&dev) == hipSuccess &&
          hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && v > 0))
      v = 256;   // no device (sizing a workspace on a host without one): the MI355X count
    if (slot >= 0) cached[slot].store(v, std::memory_order_relaxed);
  }
  return v;
}

int stream_heads_per_lane(int group) { return group == 1 ? 1 : group == 2 ? 2 : group <= 4 ? 4 : 8; }

// bf16 or 8-bit pools, head_dim 128, power-of-two block size, pools addressable with 32-bit
// 16-byte units, batch small enough for the prefix table in LDS.
bool attn_stream_supported(const pkv_attn_desc& d) {
  const int eb = d.kv_dtype == PKV_F8_E4M3 ? 1 : 2;
  const int tpb = d.block_size / kTileTokens;
  const int G = d.num_q_heads / d.num_kv_heads;
  const int gh = stream_heads_per_lane(G);
  const int64_t np = (int64_t)d.num_kv_heads * ((G + gh - 1) / gh);
  const int64_t tiles_ub = ((int64_t)d.max_context_len + kTileTokens - 1) / kTileTokens * d.batch * np;
  auto span = [&](int64_t sb, int64_t sh, int64_t st) {
    return ((int64_t)d.num_pool_blocks * sb + (int64_t)d.num_kv_heads * sh + (int64_t)d.block_size * st) * eb;
  };
  return (d.kv_dtype == PKV_BF16 || d.kv_dtype == PKV_F8_E4M3) && d.head_dim == 128 && tpb >= 1 && (tpb & (tpb - 1)) == 0 &&
         !(d.flags & PKV_ATTN_FLAG_VECTOR_ALU) && np <= 256 && d.batch < (1 << 23) &&
         (int64_t)(d.batch + 1) * 4 <= kStreamMaxPrefixBytes && tiles_ub < (1ll << 30) &&
         d.k_stride_token * eb * 16 < (1 << 30) && d.v_stride_token * eb * 16 < (1 << 30) &&
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
  // ns = 8k with k < longest range / (8 cap) + 1, the longest range at most 9/8 of a fair share
  w.slots = pairs + (cap ? (tiles_ub + kMinGroupTiles * ncu) * 9 / 8 / cap + 2 * ncu : 0) + ncu * (kNW + 1) + 2;
  auto up = [](int64_t b) { return (b + 255) / 256 * 256; };
  w.dir_bytes = up(pairs * 2 * 4);
  w.ml_bytes = up(w.slots * gh * 2 * 4);
  w.o_bytes = up(w.slots * gh * D * 4);
  return w;
}

int stream_geometry(AttnParams& p) {
  p.tpb_shift = 0;
  while ((kTileTokens << p.tpb_shift) < p.block_size) ++p.tpb_shift;
  p.prefix_bytes = ((p.batch + 1) * 4 + 15) / 16 * 16;
  const int gh = stream_heads_per_lane(p.group);
  p.group_tiles = (p.group + gh - 1) / gh;
  return gh;
}

hipError_t launch_attn_stream(AttnParams& p, hipStream_t s) {
  switch (stream_geometry(p)) {
    case 1: return launch<1>(p, s);
    case 2: return launch<2>(p, s);
    case 4: return launch<4>(p, s);
    default: return launch<8>(p, s);
  }
}

}  // namespace pkv
