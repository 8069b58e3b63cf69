// KV append (arXiv 2602.07878, Sec. 2.2 "KV-Cache"): the new token's K and V rows of every
// sequence are written to token position n_i - 1 of the paged pools, and the rows of a prefill
// chunk to the tail positions of their sequences, for gfx950.
//
// Pure data movement, a few hundred KiB per call: one lane moves 16 bytes; the
// lanes of a row (D * e / 16 of them) are adjacent so that every row is written with
// contiguous 16-byte stores.  The call is bound by launch latency, not by HBM.

#include "pkv_internal.h"

namespace pkv {
namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

__global__ __launch_bounds__(256) void kv_append_rows(const AttnParams p, const u32x4* __restrict__ k_new,
                                                      const u32x4* __restrict__ v_new, int pieces_per_row) {
  // thread -> (K or V, sequence, KV head, 16-byte piece of the row)
  const int64_t rows = (int64_t)p.batch * p.num_kv_heads;
  const int64_t per_pool = rows * pieces_per_row;
  int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (t >= 2 * per_pool) return;
  const bool is_v = t >= per_pool;
  if (is_v) t -= per_pool;
  const int piece = (int)(t % pieces_per_row);
  const int64_t row = t / pieces_per_row;
  const int g = (int)(row % p.num_kv_heads);
  const int i = (int)(row / p.num_kv_heads);
  const int n = p.context_lens[i];
  if (n <= 0) return;
  const int pos = n - 1;
  const int64_t blk = p.block_tables[(int64_t)i * p.max_blocks_per_seq + pos / p.block_size];
  const int slot = pos % p.block_size;
  const u32x4 val = (is_v ? v_new : k_new)[t];
  uint8_t* base = reinterpret_cast<uint8_t*>(const_cast<void*>(is_v ? p.v_pool : p.k_pool));
  const int64_t off = is_v ? blk * p.v_stride_block + g * p.v_stride_head + slot * p.v_stride_token
                           : blk * p.k_stride_block + g * p.k_stride_head + slot * p.k_stride_token;
  *reinterpret_cast<u32x4*>(base + off + piece * 16) = val;
}

// The rows of a prefill chunk (Sec. 2.1 prefill; Sec. 2.2 "KV-Cache"): packed row r belongs to
// the sequence i with cu_query_lens[i] <= r < cu_query_lens[i + 1] (found by bisection: the
// table is a few hundred entries in L2) and goes to position n_i - q_i + (r - cu_query_lens[i]).
__global__ __launch_bounds__(256) void kv_append_chunk_rows(const AttnParams p, const u32x4* __restrict__ k_new,
                                                            const u32x4* __restrict__ v_new, int pieces_per_row,
                                                            int64_t total_rows) {
  const int64_t per_pool = total_rows * p.num_kv_heads * pieces_per_row;
  int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (t >= 2 * per_pool) return;
  const bool is_v = t >= per_pool;
  if (is_v) t -= per_pool;
  const int piece = (int)(t % pieces_per_row);
  const int64_t rg = t / pieces_per_row;
  const int g = (int)(rg % p.num_kv_heads);
  const int64_t r = rg / p.num_kv_heads;
  if (r >= p.cu_query_lens[p.batch]) return;          // rows beyond the packed total
  int lo = 0, hi = p.batch;                             // invariant: cu[lo] <= r < cu[hi]
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (p.cu_query_lens[mid] <= r) lo = mid; else hi = mid;
  }
  const int i = lo;
  const int n = p.context_lens[i];
  const int ql = min(p.query_lens[i], n);
  const int j = (int)(r - p.cu_query_lens[i]);
  if (j >= ql) return;                                  // rows of a clipped chunk
  const int pos = n - ql + j;
  const int64_t blk = p.block_tables[(int64_t)i * p.max_blocks_per_seq + pos / p.block_size];
  const int slot = pos % p.block_size;
  const u32x4 val = (is_v ? v_new : k_new)[t];
  uint8_t* base = reinterpret_cast<uint8_t*>(const_cast<void*>(is_v ? p.v_pool : p.k_pool));
  const int64_t off = is_v ? blk * p.v_stride_block + g * p.v_stride_head + slot * p.v_stride_token
                           : blk * p.k_stride_block + g * p.k_stride_head + slot * p.k_stride_token;
  *reinterpret_cast<u32x4*>(base + off + piece * 16) = val;
}

}  // namespace

hipError_t launch_kv_append_chunk(const AttnParams& p, const void* k_new, const void* v_new, int elem_bytes,
                                  int64_t total_rows, hipStream_t s) {
  const int pieces = p.head_dim * elem_bytes / 16;
  const int64_t total = 2 * total_rows * p.num_kv_heads * pieces;
  if (total <= 0) return hipSuccess;
  if ((total + 255) / 256 > 0x7FFFFFFF) return hipErrorInvalidValue;
  hipLaunchKernelGGL(kv_append_chunk_rows, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, p,
                     reinterpret_cast<const u32x4*>(k_new), reinterpret_cast<const u32x4*>(v_new), pieces, total_rows);
  return hipGetLastError();
}

hipError_t launch_kv_append(const AttnParams& p, const void* k_new, const void* v_new, int elem_bytes,
                            hipStream_t s) {
  const int pieces = p.head_dim * elem_bytes / 16;
  const int64_t total = 2 * (int64_t)p.batch * p.num_kv_heads * pieces;
  const unsigned grid = (unsigned)((total + 255) / 256);
  hipLaunchKernelGGL(kv_append_rows, dim3(grid), dim3(256), 0, s, p,
                     reinterpret_cast<const u32x4*>(k_new), reinterpret_cast<const u32x4*>(v_new), pieces);
  return hipGetLastError();
}

}  // namespace pkv
