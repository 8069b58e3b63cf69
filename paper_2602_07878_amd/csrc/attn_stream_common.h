// Definitions shared by the K/V-streaming decode kernels (attn_stream_mfma.hip: bf16 pools with
// direct-to-LDS loads; attn_stream_flat.hip: the flat tile loop for 8-bit pools and for calls that
// come with a per-step plan): vector types, LDS geometry, and the cut of the tile axis into
// workgroup ranges and wavefront chunks that the kernels and the host-side sizing agree on.
#pragma once
#include "pkv_internal.h"

namespace pkv {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((address_space(3))) s16x4* lds_s16x4_ptr;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;
typedef __attribute__((ext_vector_type(2))) int32_t i32x2;

constexpr float kNegBig = -1.0e30f;
constexpr float kSlack = 8.0f;             // log2 units the reference may lag the true max
constexpr int kStreamThreads = 512;        // one workgroup of 8 wavefronts per CU
constexpr int kNW = kStreamThreads / kWaveSize;
constexpr int kTileBytes = 4096;           // 16 tokens x 256-byte rows
constexpr int kStages = 2;
constexpr int kDescBatch = 64;             // tile descriptors per table
constexpr int kStageBytes = 2 * kTileBytes; // K tile, then V tile
constexpr int kXchgBytes = 512;            // per-head values passed between lanes
// per wavefront: ring of (K, V) stages, exchange area, two descriptor tables
constexpr int kWaveLds = kStages * kStageBytes + kXchgBytes + 2 * kDescBatch * 16;
constexpr int kStageRow = 132;             // floats per head row when a flush stages O in LDS
constexpr int kMinGroupTiles = 32;         // tiles per workgroup range below which fewer workgroups work
constexpr int D = 128;

#define PKV_WAIT_VMCNT(n) \
  __builtin_amdgcn_s_waitcnt(((n) & 0xF) | (((n) >> 4) << 14) | (0x7 << 4) | (0xF << 8))

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

// Chunk schedule.  The tile axis is cut into contiguous ranges, one per workgroup, and each
// range into ns = 8k chunks whose lengths differ by at most one tile: one chunk per wavefront,
// or k per wavefront when the caller caps the tokens per partial (wavefront w then takes
// chunks w, w+8, ...).  Chunk ids grow along the axis without gaps: id = workgroup * ns + local
// id, every workgroup owning exactly ns of them.
//
// Workgroups are dealt to the eight XCDs round-robin, and on this part the odd XCDs finish an
// equal range 6-7 % later than their even neighbours (seen on every machine tried; which pair
// of XCDs is ahead varies, that does not).  Of every two consecutive workgroups the even one
// therefore takes kEvenShare/256 of a fair share and the odd one the rest (measured optimum
// 268-272 on two machines, +2 % throughput; 276 and more overshoots).
constexpr int kEvenShare = 268;
static_assert(kEvenShare >= 224 && kEvenShare <= 288, "the workspace bound allows ranges up to 9/8 of a fair share");

struct ChunkPlan {
  int lg;      // fair share of a workgroup, in tiles
  int ns;      // chunks (and chunk ids) per workgroup
  int first;   // tiles of the even workgroup of a pair
  bool skew;
  __device__ __forceinline__ int bound(int g) const {   // first tile of workgroup g's range
    return skew ? (g >> 1) * 2 * lg + ((g & 1) ? first : 0) : g * lg;
  }
  __device__ __forceinline__ int length(int g) const {  // nominal length of that range
    return skew ? ((g & 1) ? 2 * lg - first : first) : lg;
  }
  // first tile (relative to the range) of chunk i of a range of `len` tiles
  __device__ __forceinline__ int chunk_start(int len, int i) const { return (int)((int64_t)i * len / ns); }
  __device__ __forceinline__ int chunk_of(int x) const {
    int g;
    if (skew) {
      const int pr = x / (2 * lg);
      g = 2 * pr + (x - pr * 2 * lg >= first ? 1 : 0);
    } else {
      g = x / lg;
    }
    const int u = x - bound(g);
    return g * ns + (int)((((int64_t)u + 1) * ns - 1) / length(g));   // inverse of chunk_start
  }
};

__device__ __forceinline__ ChunkPlan plan_chunks(int T, int nwg, int cap) {
  ChunkPlan pl;
  pl.lg = max(kMinGroupTiles, (T + nwg - 1) / nwg);
  pl.skew = kEvenShare != 256 && (nwg & 1) == 0;
  pl.first = pl.skew ? (kEvenShare * pl.lg) >> 8 : pl.lg;
  const int longest = pl.skew ? max(pl.first, 2 * pl.lg - pl.first) : pl.lg;
  const int k = cap > 0 ? (longest + kNW * cap - 1) / (kNW * cap) : 1;
  pl.ns = kNW * k;
  return pl;
}

// A per-step plan (calls that bring one): header words, then the directory, then the tile
// descriptors.  Header: the tile count, then the number that names the call geometry the plan
// was made for (0: the plan is not valid).
enum { kPlanT = 0, kPlanKey = 1, kPlanWords = 64 };

}  // namespace
}  // namespace pkv
