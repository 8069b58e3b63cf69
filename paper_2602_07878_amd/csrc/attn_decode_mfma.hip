// Paged decode attention, bf16 / head_dim 128 fast path for gfx950.
//
// Same operation and same work split as the vector-ALU kernel (one workgroup
// per (partition, KV head [x head sub-group], sequence); four wavefronts, each
// with its own stream of 16-token tiles and its own softmax state), but:
//
//  * K goes HBM -> LDS with direct-to-LDS 16-byte loads (no VGPR staging), in
//    a 2-deep ring per wavefront, so the next tile is in flight while one is
//    consumed.  The LDS image is XOR-swizzled by choosing which 16-byte piece
//    of its token row each lane fetches, so the row-per-lane reads that feed
//    the matrix cores are bank-conflict free while every wave-wide global load
//    still covers whole contiguous 256-byte rows.
//  * scores S[head slot][token] = Q_g K^T come from v_mfma_f32_16x16x32_bf16
//    (both operands are exact bf16; the query group is padded/replicated to the
//    16 rows of the tile).
//  * softmax weights stay fp32.  They cross from the score layout (lane =
//    token) to the V layout (lane = 16-byte piece of a V row) through a 1 KiB
//    LDS tile per wavefront; P.V is fp32 FMA on V rows that are loaded straight
//    into registers with fully coalesced 16-byte loads.
//  * the running maximum is only a reference point for exp2(): it is raised
//    (and the accumulators rescaled) only when a score exceeds it by more than
//    kSlack, which after the first tile practically never happens.

#include <type_traits>

#include "pkv_internal.h"

namespace pkv {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

constexpr float kNegBig = -1.0e30f;
constexpr float kSlack = 8.0f;             // log2 units the reference may lag the true max
constexpr int kNW = kAttnThreads / kWaveSize;
constexpr int kTileBytes = 4096;           // 16 tokens x 256-byte rows
constexpr int kStages = 2;
constexpr int kWaveLds = kStages * kTileBytes + 1024;   // K ring + P tile

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

__device__ __forceinline__ uint16_t to_bf16_rne(float f) {
  uint32_t u = __builtin_bit_cast(uint32_t, f);
  if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (uint16_t)((u >> 16) | 0x40);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

typedef const void __attribute__((address_space(1)))* gptr_t;
typedef void __attribute__((address_space(3)))* lptr_t;

// GH = query heads accumulated per lane (1, 2, 4 or 8).
template <int GH>
__global__ __launch_bounds__(kAttnThreads) void attn_partial_mfma_d128(const AttnParams p) {
  constexpr int D = 128;
  constexpr int HS = GH >= 8 ? 8 : 4;   // distinct head slots among the 16 MFMA rows

  extern __shared__ __attribute__((aligned(16))) uint8_t lds[];

  const int part = blockIdx.x;
  const int kvh = blockIdx.y / p.group_tiles;
  const int gtile = blockIdx.y % p.group_tiles;
  const int seq = blockIdx.z;
  const int lane = threadIdx.x & (kWaveSize - 1);
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWaveSize);
  const int t16 = lane & 15;   // score layout: token of the tile; V layout: 16-byte piece
  const int q4 = lane >> 4;    // score layout: head slots 4*q4..+3; V layout: row of a load

  const int n = p.context_lens[seq];
  const int PT = p.partition_tokens;
  const int nparts = n > 0 ? (n + PT - 1) / PT : 1;
  if (part >= nparts) return;

  const int h0 = kvh * p.group + gtile * GH;
  const int nheads = min(GH, p.group - gtile * GH);

  if (n <= 0) {
    for (int idx = threadIdx.x; idx < nheads * D; idx += kAttnThreads) {
      const int64_t o = ((int64_t)seq * p.num_q_heads + h0 + idx / D) * D + idx % D;
      if (p.out_is_bf16) reinterpret_cast<uint16_t*>(p.out)[o] = 0;
      else reinterpret_cast<float*>(p.out)[o] = 0.f;
    }
    return;
  }

  // ---- query operand: row i of the 16x32 A tile is head slot i % HS ----------
  bf16x8 qfrag[4];
  {
    const int hs = min(t16 % HS, nheads - 1);
    const uint8_t* qp = reinterpret_cast<const uint8_t*>(p.q) +
                        ((int64_t)seq * p.num_q_heads + h0 + hs) * (D * 2) + q4 * 16;
#pragma unroll
    for (int c = 0; c < 4; ++c)
      qfrag[c] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(qp + c * 64));
  }

  // ---- per-lane, loop-invariant offsets ------------------------------------------
  uint32_t koff[4], voff[4], krd[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int tok = 4 * j + q4;                        // token row this lane fetches in load j
    koff[j] = (uint32_t)(tok * p.k_stride_token) + (uint32_t)((t16 ^ tok) * 16);
    voff[j] = (uint32_t)(tok * p.v_stride_token) + (uint32_t)(t16 * 16);
    // MFMA step j: this lane (token t16) needs piece 4j+q4 of its row, stored at slot piece^t16
    krd[j] = (uint32_t)((t16 >> 2) * 1024 + (t16 & 3) * 256 + (((4 * j + q4) ^ t16) * 16));
  }

  uint8_t* wlds = lds + wave * kWaveLds;
  float* pbuf = reinterpret_cast<float*>(wlds + kStages * kTileBytes);   // [16 tokens][16 slots]

  // ---- this wave's tiles: w, w+4, ... of the partition ---------------------------
  const int tok_begin = part * PT;
  const int tok_end = min(n, tok_begin + PT);
  const int ntiles = (tok_end - tok_begin + kTileTokens - 1) / kTileTokens;
  const int ntw = ntiles > wave ? (ntiles - wave + kNW - 1) / kNW : 0;
  const int tile_base = tok_begin / kTileTokens + wave;
  const int32_t* table = p.block_tables + (int64_t)seq * p.max_blocks_per_seq;

  const uint8_t* kpool = reinterpret_cast<const uint8_t*>(p.k_pool) + kvh * p.k_stride_head;
  const uint8_t* vpool = reinterpret_cast<const uint8_t*>(p.v_pool) + kvh * p.v_stride_head;

  float m[4], l[4];
#pragma unroll
  for (int r = 0; r < 4; ++r) { m[r] = kNegBig; l[r] = 0.f; }
  float acc[GH][8];
#pragma unroll
  for (int g = 0; g < GH; ++g)
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[g][e] = 0.f;

  u32x4 vreg[kStages][4];

  // block ids of this wave's (at most 64) tiles live one per lane
  const int i_lane = lane < ntw ? lane : 0;
  const int ids = ntw > 0 ? table[(tile_base + kNW * i_lane) >> p.tpb_shift] : 0;

  auto issue = [&](int i, int stage) {
    const int gt = tile_base + kNW * i;                 // global tile index in the sequence
    const int blk = __builtin_amdgcn_readlane(ids, i);
    const int slot0 = (gt & ((1 << p.tpb_shift) - 1)) * kTileTokens;
    const uint8_t* kb = kpool + blk * p.k_stride_block + slot0 * p.k_stride_token;
    const uint8_t* vb = vpool + blk * p.v_stride_block + slot0 * p.v_stride_token;
    uint8_t* kl = wlds + stage * kTileBytes;
#pragma unroll
    for (int j = 0; j < 4; ++j)
      __builtin_amdgcn_global_load_lds((gptr_t)(kb + koff[j]), (lptr_t)(kl + j * 1024), 16, 0, 0);
#pragma unroll
    for (int j = 0; j < 4; ++j)
      vreg[stage][j] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(vb + voff[j]));
  };

  // TAIL: the tile may reach past the end of the context (only a wave's last tile can)
  auto consume = [&](int i, int stage, auto tail_tag) {
    constexpr bool TAIL = decltype(tail_tag)::value;
    const int tok0 = (tile_base + kNW * i) * kTileTokens;
    const uint8_t* kl = wlds + stage * kTileBytes;
    f32x4 c = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const bf16x8 kf = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(kl + krd[j]));
      c = __builtin_amdgcn_mfma_f32_16x16x32_bf16(qfrag[j], kf, c, 0, 0, 0);
    }
    const bool dead = TAIL && (tok0 + t16 >= tok_end);
    float s[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) s[r] = dead ? -INFINITY : c[r] * p.scale_log2e;

    bool grow = false;
#pragma unroll
    for (int r = 0; r < 4; ++r) grow |= s[r] > m[r] + kSlack;
    if (__builtin_amdgcn_ballot_w64(grow) != 0) {      // wave-uniform, rare after the first tile
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
    for (int j = 0; j < 4; ++j) {
      const int tok = 4 * j + q4;                       // V row held by this lane for load j
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
      u32x4 vv = vreg[stage][j];
      if (TAIL && tok0 + tok >= tok_end) vv = u32x4{0, 0, 0, 0};   // stale slot: may hold NaN bits
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
  };

  // ---- software pipeline: tile i+1 in flight while tile i is consumed ------------
  // The steady-state loop is branch-free between an issue and the matching wait, so the
  // number of younger loads outstanding at each wait is exactly one stage (8 loads).
  if (ntw > 0) {
    using std::false_type;
    using std::true_type;
    issue(0, 0);
    int i = 0;
    while (i + 2 < ntw) {
      issue(i + 1, 1); PKV_WAIT_VMCNT(8); consume(i, 0, false_type{});
      issue(i + 2, 0); PKV_WAIT_VMCNT(8); consume(i + 1, 1, false_type{});
      i += 2;
    }
    if (i + 2 == ntw) {
      issue(i + 1, 1); PKV_WAIT_VMCNT(8); consume(i, 0, false_type{});
      PKV_WAIT_VMCNT(0); consume(i + 1, 1, true_type{});
    } else {
      PKV_WAIT_VMCNT(0); consume(i, 0, true_type{});
    }
  }

  // ---- per-wave totals ----------------------------------------------------------------
#pragma unroll
  for (int r = 0; r < 4; ++r) l[r] = row16_sum(l[r]);
#pragma unroll
  for (int g = 0; g < GH; ++g)
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      float v = acc[g][e];
      v += __shfl_xor(v, 16, kWaveSize);
      v += __shfl_xor(v, 32, kWaveSize);
      acc[g][e] = v;
    }

  // ---- merge the waves through LDS (the K ring is dead by now) -----------------------
  __syncthreads();
  float* smem = reinterpret_cast<float*>(lds);      // [kNW][GH][D + 2]
  constexpr int rowf = D + 2;
  if (q4 == 0) {
#pragma unroll
    for (int g = 0; g < GH; ++g) {
      float* row = smem + (wave * GH + g) * rowf + t16 * 8;
#pragma unroll
      for (int e = 0; e < 8; ++e) row[e] = acc[g][e];
    }
  }
  if (t16 == 0) {
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int slot = 4 * q4 + r;
      if (slot < HS && slot < GH) {
        float* row = smem + (wave * GH + slot) * rowf;
        row[D] = m[r];
        row[D + 1] = l[r];
      }
    }
  }
  __syncthreads();

  const bool single = nparts == 1;
  for (int idx = threadIdx.x; idx < nheads * D; idx += kAttnThreads) {
    const int g = idx / D, d = idx % D;
    float M = kNegBig;
#pragma unroll
    for (int w = 0; w < kNW; ++w) M = fmaxf(M, smem[(w * GH + g) * rowf + D]);
    float L = 0.f, O = 0.f;
#pragma unroll
    for (int w = 0; w < kNW; ++w) {
      const float* row = smem + (w * GH + g) * rowf;
      const float f = __builtin_amdgcn_exp2f(row[D] - M);
      L = fmaf(row[D + 1], f, L);
      O = fmaf(row[d], f, O);
    }
    const int h = h0 + g;
    if (single) {
      const float r = O / L;
      const int64_t o = ((int64_t)seq * p.num_q_heads + h) * D + d;
      if (p.out_is_bf16) reinterpret_cast<uint16_t*>(p.out)[o] = to_bf16_rne(r);
      else reinterpret_cast<float*>(p.out)[o] = r;
    } else {
      const int64_t pr = ((int64_t)seq * p.num_q_heads + h) * p.max_partitions + part;
      p.ws_o[pr * D + d] = O;
      if (d == 0) { p.ws_ml[pr * 2] = M; p.ws_ml[pr * 2 + 1] = L; }
    }
  }
}

template <int GH>
hipError_t launch(const AttnParams& p, hipStream_t s) {
  dim3 grid(p.max_partitions, p.num_kv_heads * p.group_tiles, p.batch);
  size_t lds = (size_t)kNW * kWaveLds;
  const size_t merge = sizeof(float) * kNW * GH * (128 + 2);
  if (merge > lds) lds = merge;
  hipLaunchKernelGGL((attn_partial_mfma_d128<GH>), grid, dim3(kAttnThreads), lds, s, p);
  return hipGetLastError();
}

}  // namespace

// bf16, head_dim 128, token rows within a block at most 64 KiB apart.
bool attn_mfma_supported(const AttnParams& p, int dtype) {
  const int tpb = p.block_size / kTileTokens;
  return dtype == PKV_BF16 && p.head_dim == 128 && (tpb & (tpb - 1)) == 0 &&
         p.partition_tokens <= kNW * kWaveSize * kTileTokens &&   // <= 64 tiles per wave
         p.k_stride_token * 16 < (1 << 30) && p.v_stride_token * 16 < (1 << 30);
}

hipError_t launch_attn_partial_mfma(AttnParams& p, hipStream_t s) {
  const int G = p.group;
  p.tpb_shift = 0;
  while ((kTileTokens << p.tpb_shift) < p.block_size) ++p.tpb_shift;
  if (G == 1) { p.group_tiles = 1; return launch<1>(p, s); }
  if (G == 2) { p.group_tiles = 1; return launch<2>(p, s); }
  if (G <= 4) { p.group_tiles = 1; return launch<4>(p, s); }
  p.group_tiles = (G + 7) / 8;
  return launch<8>(p, s);
}

}  // namespace pkv
