// 8-bit (E4M3) KV pools under the prefill call: the blocks the chunk's sequences own are decoded
// into a bf16 copy, and the bf16 prefill kernel walks the copy.
//
// Operation (arXiv 2602.07878, Sec. 2.1 / Sec. 5.1.2 "Recomputation" for the prefill; a
// quantised KV cache halves the bytes per cached token that Sec. 4.2's time model charges): the
// prefill is bound by the matrix cores, not by HBM, so decoding the cache once per call into
// the format the matrix-core kernel reads costs little (one read of the 8-bit blocks, one write
// and one read of their bf16 images) and keeps one prefill kernel.  E4M3 -> bf16 is exact
// (3 mantissa bits into 7, exponent range inside bf16's), so the pool scales stay where the
// decode call has them: k_scale in the softmax scale, v_scale on the output.
//
// Logical block j of sequence i goes to block i * blocks_per_seq + j of the copy, head-major
// [block][KV head][token][dim]; the copy's block table is that identity, written here too.
// One workgroup per (j, i); it ends at once where the sequence has no such block.

#include "pkv_internal.h"

namespace pkv {
namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kThreads = 256;

// 16 codes -> 16 bf16: the hardware conversion of two codes of a word (its lower or its upper
// half) into a packed pair, with a scale of 1; exact
__device__ __forceinline__ void decode16(const u32x4 c, u32x4& lo, u32x4& hi) {
  uint32_t w[8];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const uint32_t word = c[i];
    asm("v_cvt_scalef32_pk_bf16_fp8 %0, %1, 1.0" : "=v"(w[2 * i]) : "v"(word));
    asm("v_cvt_scalef32_pk_bf16_fp8 %0, %1, 1.0 op_sel:[1,0,0]" : "=v"(w[2 * i + 1]) : "v"(word));
  }
  lo = u32x4{w[0], w[1], w[2], w[3]};
  hi = u32x4{w[4], w[5], w[6], w[7]};
}

__global__ __launch_bounds__(kThreads) void f8_blocks_to_bf16(const AttnParams p, uint8_t* k_copy, uint8_t* v_copy,
                                                              int32_t* copy_table, int blocks_per_seq) {
  const int j = blockIdx.x, seq = blockIdx.y;
  const int n = p.context_lens[seq];
  if (n <= 0 || j >= (n + p.block_size - 1) / p.block_size) return;
  const int64_t blk = p.block_tables[(int64_t)seq * p.max_blocks_per_seq + j];
  const int64_t cb = (int64_t)seq * blocks_per_seq + j;
  if (threadIdx.x == 0) copy_table[cb] = (int32_t)cb;
  const int pieces_per_row = p.head_dim / 16;                      // 16 codes each
  const int rows = p.num_kv_heads * p.block_size;
  const int64_t copy_block_bytes = (int64_t)rows * p.head_dim * 2;
  for (int x = threadIdx.x; x < rows * pieces_per_row; x += kThreads) {
    const int row = x / pieces_per_row, c = x - row * pieces_per_row;
    const int kvh = row / p.block_size, tok = row - kvh * p.block_size;
    const uint8_t* ks = reinterpret_cast<const uint8_t*>(p.k_pool) + blk * p.k_stride_block + kvh * p.k_stride_head +
                        tok * p.k_stride_token + c * 16;
    const uint8_t* vs = reinterpret_cast<const uint8_t*>(p.v_pool) + blk * p.v_stride_block + kvh * p.v_stride_head +
                        tok * p.v_stride_token + c * 16;
    const u32x4 kc = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(ks));
    const u32x4 vc = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(vs));
    u32x4 lo, hi;
    const int64_t o = cb * copy_block_bytes + ((int64_t)row * p.head_dim + c * 16) * 2;
    decode16(kc, lo, hi);
    *reinterpret_cast<u32x4*>(k_copy + o) = lo;
    *reinterpret_cast<u32x4*>(k_copy + o + 16) = hi;
    decode16(vc, lo, hi);
    *reinterpret_cast<u32x4*>(v_copy + o) = lo;
    *reinterpret_cast<u32x4*>(v_copy + o + 16) = hi;
  }
}

}  // namespace

// Bytes of the bf16 copy and its table for a call described by d (a bound from the host-known
// maximum context: every sequence gets room for that many blocks).
F8PrefillCopy f8_prefill_copy_layout(const pkv_attn_desc& d) {
  F8PrefillCopy c;
  c.blocks_per_seq = (int32_t)(((int64_t)d.max_context_len + d.block_size - 1) / d.block_size);
  if (c.blocks_per_seq < 1) c.blocks_per_seq = 1;
  const size_t blocks = (size_t)d.batch * c.blocks_per_seq;
  c.pool_bytes = blocks * d.num_kv_heads * d.block_size * d.head_dim * 2;
  c.table_bytes = (blocks * sizeof(int32_t) + 255) / 256 * 256;
  return c;
}

// p describes the 8-bit pools (strides in bytes); k_copy, v_copy and copy_table lie in the
// caller's workspace
hipError_t launch_f8_blocks_to_bf16(const AttnParams& p, uint8_t* k_copy, uint8_t* v_copy, int32_t* copy_table,
                                    int blocks_per_seq, hipStream_t s) {
  hipLaunchKernelGGL(f8_blocks_to_bf16, dim3((unsigned)blocks_per_seq, (unsigned)p.batch), dim3(kThreads), 0, s, p,
                     k_copy, v_copy, copy_table, blocks_per_seq);
  return hipGetLastError();
}

}  // namespace pkv
