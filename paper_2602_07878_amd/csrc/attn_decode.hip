// Paged decode attention for gfx950: split-K partial kernel + log-sum-exp merge.
//
// Operation (arXiv 2602.07878, Sec. 2.2 "KV-Cache" for the paged pool, Sec. 4.2
// for the per-step streaming of the whole KV history): for sequence i and query
// head h, out = softmax_t(scale * q . K_t) V over the n_i tokens found through
// the block table.  The context is cut into partitions of PT tokens; one
// workgroup handles one (partition, KV head [x head sub-group], sequence) and
// produces (m, l, O) partials that the merge kernel combines; a sequence with a
// single partition is finished by the partial kernel itself.
//
// Vector-ALU kernel (all dtypes/shapes).  Layout inside a wavefront: a token
// row of D*e bytes is covered by LPR = D*e/16 consecutive lanes, 16 bytes each,
// so one wave-wide load moves TPL = 64/LPR whole rows and every 64-lane load is
// one contiguous stretch when rows are adjacent.  Lane (r, c) = (lane / LPR,
// lane % LPR) keeps, for each of the GT query heads it serves, its own online
// softmax state over the tokens of row group r: no cross-lane traffic in the
// main loop except the LPR-lane sum that finishes each dot product.

#include <hip/hip_ext.h>

#include "pkv_internal.h"

namespace pkv {
namespace {

constexpr float kNegBig = -1.0e30f;  // finite stand-in for -inf in running maxima

struct alignas(16) U4 { uint32_t x, y, z, w; };

__device__ __forceinline__ U4 load16(const uint8_t* p) {
  return *reinterpret_cast<const U4*>(p);
}
// K/V bytes that no other workgroup reads again: marked as such, they do not push the tables and
// query rows out of L2
__device__ __forceinline__ U4 load16_once(const uint8_t* p) {
  typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
  const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));
  return U4{v[0], v[1], v[2], v[3]};
}

// ---- 16-lane (and narrower) all-reduce sums through DPP -------------------
template <int CTRL>
__device__ __forceinline__ float dpp_f(float v) {
  return __builtin_bit_cast(
      float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xF, 0xF, true));
}
// Sum over the LPR consecutive lanes that share a token row; every one of
// those lanes ends up with the total.
template <int LPR>
__device__ __forceinline__ float row_sum(float v) {
  v += dpp_f<0xB1>(v);                        // quad_perm [1,0,3,2]
  v += dpp_f<0x4E>(v);                        // quad_perm [2,3,0,1]
  if constexpr (LPR >= 8) v += dpp_f<0x141>(v);   // row_half_mirror
  if constexpr (LPR >= 16) v += dpp_f<0x140>(v);  // row_mirror
  if constexpr (LPR >= 32) v += __shfl_xor(v, 16, kWaveSize);
  return v;
}

// ---- element unpacking ------------------------------------------------------
template <int EB> struct Unpack;
template <> struct Unpack<4> {  // fp32: 4 elements per 16 bytes
  static constexpr int N = 4;
  __device__ static __forceinline__ void run(const U4& u, float* f) {
    f[0] = __builtin_bit_cast(float, u.x); f[1] = __builtin_bit_cast(float, u.y);
    f[2] = __builtin_bit_cast(float, u.z); f[3] = __builtin_bit_cast(float, u.w);
  }
};
template <> struct Unpack<2> {  // bf16: 8 elements per 16 bytes, widening is a shift
  static constexpr int N = 8;
  __device__ static __forceinline__ void run(const U4& u, float* f) {
    const uint32_t w[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      f[2 * i] = __builtin_bit_cast(float, w[i] << 16);
      f[2 * i + 1] = __builtin_bit_cast(float, w[i] & 0xFFFF0000u);
    }
  }
};

template <> struct Unpack<1> {  // OCP E4M3: 16 elements per 16 bytes, decoded by the hardware conversion
  static constexpr int N = 16;
  __device__ static __forceinline__ void run(const U4& u, float* f) {
    typedef float f32x2 __attribute__((ext_vector_type(2)));
    const uint32_t w[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const f32x2 lo = __builtin_amdgcn_cvt_pk_f32_fp8((int)w[i], false);   // bytes 0, 1
      const f32x2 hi = __builtin_amdgcn_cvt_pk_f32_fp8((int)w[i], true);    // bytes 2, 3
      f[4 * i] = lo[0]; f[4 * i + 1] = lo[1]; f[4 * i + 2] = hi[0]; f[4 * i + 3] = hi[1];
    }
  }
};

__device__ __forceinline__ uint16_t f32_to_bf16_rne(float f) {
  uint32_t u = __builtin_bit_cast(uint32_t, f);
  if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (uint16_t)((u >> 16) | 0x40);  // NaN
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

// One 16-token tile of K and V held in registers by a wavefront.
template <int NJ>
struct Tile {
  U4 k[NJ];
  U4 v[NJ];
};

// EB = bytes of a K/V element, QEB = bytes of a q element (equal, except bf16 q beside 8-bit pools)
template <int EB, int QEB, int LPR, int GT>
__global__ __launch_bounds__(kAttnThreads) void attn_partial_valu(const AttnParams p) {
  constexpr int EPL = Unpack<EB>::N;       // elements per lane per row
  constexpr int TPL = kWaveSize / LPR;     // token rows per wave-wide load
  constexpr int NJ = kTileTokens / TPL;    // wave-wide loads per 16-token tile
  constexpr int NW = kAttnThreads / kWaveSize;

  const int part = blockIdx.x;
  const int kvh = blockIdx.y / p.group_tiles;
  const int gtile = blockIdx.y % p.group_tiles;
  const int seq = blockIdx.z;
  const int lane = threadIdx.x & (kWaveSize - 1);
  const int wave = threadIdx.x / kWaveSize;
  const int rg = lane / LPR;   // row group: which of the TPL rows of a load
  const int ck = lane % LPR;   // 16-byte chunk inside the row

  const int n = p.context_lens[seq];
  const int D = p.head_dim;
  const int PT = p.partition_tokens;
  const int nparts = n > 0 ? (n + PT - 1) / PT : 1;
  if (part >= nparts) return;

  const int h0 = kvh * p.group + gtile * GT;           // first query head served
  const int nheads = min(GT, p.group - gtile * GT);    // real heads in this sub-group

  if (n <= 0) {  // empty context: defined as a zero row (partition 0 only gets here)
    for (int idx = threadIdx.x; idx < nheads * D; idx += kAttnThreads) {
      const int64_t o = ((int64_t)seq * p.num_q_heads + h0 + idx / D) * D + idx % D;
      if (p.out_is_bf16) reinterpret_cast<uint16_t*>(p.out)[o] = 0;
      else reinterpret_cast<float*>(p.out)[o] = 0.f;
    }
    return;
  }

  // query fragment of this lane, pre-multiplied by scale*log2(e)
  float qf[GT][EPL];
#pragma unroll
  for (int g = 0; g < GT; ++g) {
    const int h = h0 + (g < nheads ? g : 0);
    // the lane's EPL dims of the query row: EPL * QEB bytes, in 16-byte pieces
    const uint8_t* qp = reinterpret_cast<const uint8_t*>(p.q) +
                        (((int64_t)seq * p.num_q_heads + h) * D + ck * EPL) * QEB;
    constexpr int QN = Unpack<QEB>::N;
    float t[EPL];
#pragma unroll
    for (int c = 0; c < EPL / QN; ++c) Unpack<QEB>::run(load16(qp + c * 16), t + c * QN);
#pragma unroll
    for (int e = 0; e < EPL; ++e) qf[g][e] = t[e] * p.scale_log2e;
  }

  float m[GT], l[GT], acc[GT][EPL];
#pragma unroll
  for (int g = 0; g < GT; ++g) {
    m[g] = kNegBig; l[g] = 0.f;
#pragma unroll
    for (int e = 0; e < EPL; ++e) acc[g][e] = 0.f;
  }

  const int tok_begin = part * PT;
  const int tok_end = min(n, tok_begin + PT);
  const int ntiles = (tok_end - tok_begin + kTileTokens - 1) / kTileTokens;
  const int32_t* table = p.block_tables + (int64_t)seq * p.max_blocks_per_seq;
  const uint8_t* kp = reinterpret_cast<const uint8_t*>(p.k_pool) + kvh * p.k_stride_head +
                      ck * 16;
  const uint8_t* vp = reinterpret_cast<const uint8_t*>(p.v_pool) + kvh * p.v_stride_head +
                      ck * 16;

  auto load_tile = [&](int tile, Tile<NJ>& t) {
    const int tok0 = tok_begin + tile * kTileTokens;
    const int blk = table[tok0 / p.block_size];
    const int slot0 = tok0 % p.block_size;
    const uint8_t* kb = kp + blk * p.k_stride_block;
    const uint8_t* vb = vp + blk * p.v_stride_block;
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
      const int slot = slot0 + j * TPL + rg;   // < block_size: tiles never straddle blocks
      // (with one or two heads per workgroup the loads bound the kernel and the hint pays: 16/8
      // heads of 256 dims 52 -> 55 % of the HBM peak; with four or more the vector ALU does, and
      // it cost 2 %: those keep the plain load)
      if constexpr (GT <= 2) {
        t.k[j] = load16_once(kb + slot * p.k_stride_token);
        t.v[j] = load16_once(vb + slot * p.v_stride_token);
      } else {
        t.k[j] = load16(kb + slot * p.k_stride_token);
        t.v[j] = load16(vb + slot * p.v_stride_token);
      }
    }
  };

  auto consume = [&](int tile, const Tile<NJ>& t) {
    const int tok0 = tok_begin + tile * kTileTokens;
    const bool tail = tok0 + kTileTokens > tok_end;
    float s[NJ][GT];
    float vf[NJ][EPL];
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
      float kf[EPL];
      Unpack<EB>::run(t.k[j], kf);
      Unpack<EB>::run(t.v[j], vf[j]);
#pragma unroll
      for (int g = 0; g < GT; ++g) {
        float d = 0.f;
#pragma unroll
        for (int e = 0; e < EPL; ++e) d = fmaf(qf[g][e], kf[e], d);
        s[j][g] = row_sum<LPR>(d);
      }
    }
    if (tail) {  // slots at or beyond the context end hold arbitrary bits (NaN included)
#pragma unroll
      for (int j = 0; j < NJ; ++j) {
        const bool dead = tok0 + j * TPL + rg >= tok_end;
#pragma unroll
        for (int g = 0; g < GT; ++g) s[j][g] = dead ? -INFINITY : s[j][g];
#pragma unroll
        for (int e = 0; e < EPL; ++e) vf[j][e] = dead ? 0.f : vf[j][e];
      }
    }
#pragma unroll
    for (int g = 0; g < GT; ++g) {
      float mt = s[0][g];
#pragma unroll
      for (int j = 1; j < NJ; ++j) mt = fmaxf(mt, s[j][g]);
      const float mn = fmaxf(m[g], mt);
      const float alpha = __builtin_amdgcn_exp2f(m[g] - mn);
      m[g] = mn;
      l[g] *= alpha;
#pragma unroll
      for (int e = 0; e < EPL; ++e) acc[g][e] *= alpha;
#pragma unroll
      for (int j = 0; j < NJ; ++j) {
        const float pj = __builtin_amdgcn_exp2f(s[j][g] - mn);
        l[g] += pj;
#pragma unroll
        for (int e = 0; e < EPL; ++e) acc[g][e] = fmaf(pj, vf[j][e], acc[g][e]);
      }
    }
  };

  // wave w takes tiles w, w+NW, ...; the next tile is in flight while one is consumed
  {
    Tile<NJ> cur, nxt;
    int tile = wave;
    if (tile < ntiles) load_tile(tile, cur);
    while (tile < ntiles) {
      const int tn = tile + NW;
      if (tn < ntiles) load_tile(tn, nxt);
      consume(tile, cur);
      cur = nxt;
      tile = tn;
    }
  }

  // ---- merge the TPL row groups of this wave (lanes with equal ck) ----------
#pragma unroll
  for (int g = 0; g < GT; ++g) {
    float M = m[g];
#pragma unroll
    for (int off = LPR; off < kWaveSize; off <<= 1) M = fmaxf(M, __shfl_xor(M, off, kWaveSize));
    const float f = __builtin_amdgcn_exp2f(m[g] - M);
    m[g] = M;
    l[g] *= f;
#pragma unroll
    for (int e = 0; e < EPL; ++e) acc[g][e] *= f;
#pragma unroll
    for (int off = LPR; off < kWaveSize; off <<= 1) {
      l[g] += __shfl_xor(l[g], off, kWaveSize);
#pragma unroll
      for (int e = 0; e < EPL; ++e) acc[g][e] += __shfl_xor(acc[g][e], off, kWaveSize);
    }
  }

  // ---- merge the NW waves through LDS -----------------------------------------
  extern __shared__ float smem[];            // [NW][GT][D + 2]
  const int rowf = D + 2;
  if (rg == 0) {
#pragma unroll
    for (int g = 0; g < GT; ++g) {
      float* row = smem + (wave * GT + g) * rowf;
#pragma unroll
      for (int e = 0; e < EPL; ++e) row[ck * EPL + e] = acc[g][e];
      if (ck == 0) { row[D] = m[g]; row[D + 1] = l[g]; }
    }
  }
  __syncthreads();

  const bool single = nparts == 1;
  for (int idx = threadIdx.x; idx < nheads * D; idx += kAttnThreads) {
    const int g = idx / D, d = idx % D;
    float M = kNegBig;
#pragma unroll
    for (int w = 0; w < NW; ++w) M = fmaxf(M, smem[(w * GT + g) * rowf + D]);
    float L = 0.f, O = 0.f;
#pragma unroll
    for (int w = 0; w < NW; ++w) {
      const float* row = smem + (w * GT + g) * rowf;
      const float f = __builtin_amdgcn_exp2f(row[D] - M);
      L = fmaf(row[D + 1], f, L);
      O = fmaf(row[d], f, O);
    }
    const int h = h0 + g;
    if (single) {
      const float r = O / L * p.v_scale;
      const int64_t o = ((int64_t)seq * p.num_q_heads + h) * D + d;
      if (p.out_is_bf16) reinterpret_cast<uint16_t*>(p.out)[o] = f32_to_bf16_rne(r);
      else reinterpret_cast<float*>(p.out)[o] = r;
    } else {
      const int64_t pr = ((int64_t)seq * p.num_q_heads + h) * p.max_partitions + part;
      p.ws_o[pr * D + d] = O;
      if (d == 0) { p.ws_ml[pr * 2] = M; p.ws_ml[pr * 2 + 1] = L; }
    }
  }
}

// Merge of the split-K partials: M = max_p m_p, L = sum_p l_p 2^(m_p - M),
// out = sum_p O_p 2^(m_p - M) / L, partitions taken in ascending order.
__global__ __launch_bounds__(256) void attn_merge(const AttnParams p) {
  const int h = blockIdx.x, seq = blockIdx.y;
  const int n = p.context_lens[seq];
  const int PT = p.partition_tokens;
  const int nparts = n > 0 ? (n + PT - 1) / PT : 1;
  if (nparts <= 1) return;  // already finished by the partial kernel
  const int D = p.head_dim;
  const int64_t pr0 = ((int64_t)seq * p.num_q_heads + h) * p.max_partitions;
  float M = kNegBig;
  for (int q = 0; q < nparts; ++q) M = fmaxf(M, p.ws_ml[(pr0 + q) * 2]);
  for (int d = threadIdx.x; d < D; d += blockDim.x) {
    float L = 0.f, O = 0.f;
    for (int q = 0; q < nparts; ++q) {
      const float f = __builtin_amdgcn_exp2f(p.ws_ml[(pr0 + q) * 2] - M);
      L = fmaf(p.ws_ml[(pr0 + q) * 2 + 1], f, L);
      O = fmaf(p.ws_o[(pr0 + q) * D + d], f, O);
    }
    const float r = O / L * p.v_scale;
    const int64_t o = ((int64_t)seq * p.num_q_heads + h) * D + d;
    if (p.out_is_bf16) reinterpret_cast<uint16_t*>(p.out)[o] = f32_to_bf16_rne(r);
    else reinterpret_cast<float*>(p.out)[o] = r;
  }
}

template <int EB, int QEB, int LPR, int GT>
hipError_t launch_valu(const AttnParams& p, hipStream_t s) {
  dim3 grid(p.max_partitions, p.num_kv_heads * p.group_tiles, p.batch);
  const size_t lds = sizeof(float) * (kAttnThreads / kWaveSize) * GT * (p.head_dim + 2);
  if (p.ev_begin || p.ev_end)
    hipExtLaunchKernelGGL((attn_partial_valu<EB, QEB, LPR, GT>), grid, dim3(kAttnThreads), lds, s,
                          p.ev_begin, p.ev_end, 0, p);
  else
    hipLaunchKernelGGL((attn_partial_valu<EB, QEB, LPR, GT>), grid, dim3(kAttnThreads), lds, s, p);
  const hipError_t e = hipGetLastError();
  return e;
}

template <int EB, int QEB, int LPR>
hipError_t launch_valu_g(AttnParams& p, hipStream_t s) {
  const int G = p.group;
  if (G == 1) { p.group_tiles = 1; return launch_valu<EB, QEB, LPR, 1>(p, s); }
  if (G == 2) { p.group_tiles = 1; return launch_valu<EB, QEB, LPR, 2>(p, s); }
  // 16 elements per lane with 8-bit pools: four heads per lane fill the registers
  if (G <= 4 || EB == 1) { p.group_tiles = (G + 3) / 4; return launch_valu<EB, QEB, LPR, 4>(p, s); }
  if constexpr (EB != 1) {
    p.group_tiles = (G + 7) / 8;
    return launch_valu<EB, QEB, LPR, 8>(p, s);
  }
  return hipErrorInvalidValue;
}

}  // namespace

hipError_t launch_attn_decode(const AttnParams& pin, int dtype, hipStream_t s) {
  AttnParams p = pin;
  const int eb = dtype == PKV_BF16 ? 2 : dtype == PKV_F8_E4M3 ? 1 : 4;
  const int row_bytes = p.head_dim * eb;
  hipError_t e = hipErrorInvalidValue;
  if (eb == 2) {
    if (row_bytes == 128) e = launch_valu_g<2, 2, 8>(p, s);
    else if (row_bytes == 256) e = launch_valu_g<2, 2, 16>(p, s);
    else if (row_bytes == 512) e = launch_valu_g<2, 2, 32>(p, s);
  } else if (eb == 1) {   // 8-bit pools, bf16 q
    if (row_bytes == 128) e = launch_valu_g<1, 2, 8>(p, s);
    else if (row_bytes == 256) e = launch_valu_g<1, 2, 16>(p, s);
    else if (row_bytes == 512) e = launch_valu_g<1, 2, 32>(p, s);
  } else {
    if (row_bytes == 128) e = launch_valu_g<4, 4, 8>(p, s);
    else if (row_bytes == 256) e = launch_valu_g<4, 4, 16>(p, s);
    else if (row_bytes == 512) e = launch_valu_g<4, 4, 32>(p, s);
  }
  if (e != hipSuccess) return e;
  if (p.max_partitions > 1) {
    hipLaunchKernelGGL(attn_merge, dim3(p.num_q_heads, p.batch), dim3(p.head_dim >= 256 ? 256 : 128),
                       0, s, p);
    e = hipGetLastError();
  }
  return e;
}

}  // namespace pkv
