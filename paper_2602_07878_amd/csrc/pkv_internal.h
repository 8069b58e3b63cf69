// Internal declarations shared by the translation units of libpkv (gfx950).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "pkv.h"

namespace pkv {

constexpr int kWaveSize = 64;
constexpr int kTileTokens = 16;          // tokens handled per inner tile
constexpr int kDefaultPartition = 512;   // split-K partition length in tokens
constexpr int kAttnThreads = 256;        // 4 wavefronts per workgroup
constexpr int kStreamMaxPrefixBytes = 8192;   // LDS for per-sequence tile prefix sums

// Per-device bookkeeping (kernel attributes set, CU counts, the address of the static scratch
// array) is kept in small tables indexed by the HIP device id; for ids outside the table (-1)
// nothing is remembered and the question is asked again at every call.
constexpr int kMaxDevices = 16;
inline int device_slot() {
  int d = 0;
  if (hipGetDevice(&d) != hipSuccess || d < 0 || d >= kMaxDevices) return -1;
  return d;
}

// once-per-device set-up of the kernels that need it; also run by pkv_init()
hipError_t prepare_attn_stream();    // attn_stream_mfma.hip
hipError_t prepare_attn_flat();      // attn_stream_flat.hip
hipError_t prepare_attn_prefill();   // attn_prefill_mfma.hip
hipError_t prepare_static_scratch(); // attn_static.hip

int num_cus();   // CUs of the current device (256 when there is none), attn_stream_mfma.hip

// Launch geometry and pointers of one attention call, passed by value.
struct AttnParams {
  const void* q;
  const void* k_pool;
  const void* v_pool;
  const int32_t* block_tables;
  const int32_t* context_lens;
  const int32_t* query_lens;      // prefill only: query tokens per sequence
  const int32_t* cu_query_lens;   // prefill only: [B+1] first packed query row of each sequence
  void* out;
  float* ws_ml;   // [B][Hq][P][2]  (running max in log2 units, normaliser)
  float* ws_o;    // [B][Hq][P][D]  un-normalised partial output rows
  int32_t* ws_dir;          // stream kernel: [pairs][2] (first slot, partial count)
  const int32_t* plan_hdr;  // stream kernel, calls with a per-step plan: its header words, else null
  const void* plan_desc;    // ... and its tile descriptors, 16 bytes per tile of the axis
  const void* k_new;        // stream kernel with a plan, bf16 pools: the new token's rows [B][Hkv][D] to append, else null
  const void* v_new;
  int32_t plan_key;         // ... and the number that names the call geometry a plan is made for
  int32_t plan_tiles_cap;   // ... and how many descriptors the plan has room for
  int64_t k_stride_block, k_stride_head, k_stride_token;  // BYTES
  int64_t v_stride_block, v_stride_head, v_stride_token;  // BYTES
  int32_t batch, num_q_heads, num_kv_heads, head_dim;
  int32_t block_size, max_blocks_per_seq;
  int32_t group;            // G = Hq / Hkv
  int32_t group_tiles;      // ceil(G / GT): workgroups per KV head
  int32_t partition_tokens; // PT
  int32_t max_partitions;   // P
  int32_t out_is_bf16;
  int32_t no_mfma;          // force the vector-ALU kernel
  int32_t kv_is_f8;         // the pools hold 8-bit E4M3 codes (q is bf16)
  int32_t tpb_shift;        // log2(block_size / 16) (matrix-core kernel only)
  int32_t chunk_tiles_max;  // stream kernel: most tiles one wavefront takes per chunk (<= 64)
  int32_t prefix_bytes;     // stream kernel: LDS bytes of the tile prefix table
  int32_t streams_per_xcd;  // prefill kernel: (sequence, KV head) streams dealt to one XCD
  int32_t partials_streaming;  // stream kernel: partial rows are stored past the caches (there are more of them than L2 holds)
  float scale_log2e;        // scale * log2(e) (times the K dequantisation factor of 8-bit pools)
  float v_scale;            // factor on the output: the V dequantisation factor of 8-bit pools, else 1
  // host side only: optional events recorded right before / after the partial kernel
  hipEvent_t ev_begin, ev_end;
};

struct SwapParams {
  const uint8_t* src;
  uint8_t* dst;
  const int32_t* mapping;  // [n_pairs][2]
  int64_t block_bytes, src_plane_stride, dst_plane_stride;
  int32_t num_planes, n_pairs;
  // The host leg moves a swap in pieces through a buffer that holds only the piece: on that side
  // pair j of the (windowed) mapping uses slot j of the buffer, whatever the mapping's column says.
  int32_t src_slot_is_pair, dst_slot_is_pair;
};

// api.hip: checks and launch of the decode-attention call (every entry point that offers it ends
// here).  static_scratch: the partials go to the library's static device array (attn_static.hip)
// and `workspace` is ignored.  plan: a buffer written by pkv_attn_plan for this descriptor, tables
// and lengths, or null.  k_new, v_new: the new token's rows, appended to the pools ahead of (or
// inside) the attention, or null.
int32_t attention_call(const pkv_attn_desc* desc, const void* q, const void* k_pool, const void* v_pool,
                       const int32_t* block_tables, const int32_t* context_lens, float scale, void* out,
                       void* workspace, size_t workspace_bytes, void* hip_stream, void* ev_begin, void* ev_end,
                       bool static_scratch, const void* plan, size_t plan_bytes, const void* k_new, const void* v_new);
// attn_static.hip: size of the static scratch array, and its device address on the current device
size_t static_scratch_bytes();
hipError_t static_scratch_address(void** ptr);
// attn_decode.hip
hipError_t launch_attn_decode(const AttnParams& p, int dtype, hipStream_t s);
// attn_stream_mfma.hip
struct StreamWorkspace {
  int64_t slots, dir_bytes, ml_bytes, o_bytes;
  int32_t chunk_tiles_max;
  int64_t total() const { return dir_bytes + ml_bytes + o_bytes; }
};
bool attn_stream_supported(const pkv_attn_desc& d);
StreamWorkspace stream_workspace(const pkv_attn_desc& d);
int stream_heads_per_lane(int group);
int stream_geometry(AttnParams& p);   // fills tpb_shift, prefix_bytes and group_tiles; returns the heads per lane
hipError_t launch_attn_stream(AttnParams& p, hipStream_t s);
// attn_stream_flat.hip: the streaming kernel for 8-bit pools and for calls with a per-step plan
// (launch_attn_stream puts the merge kernel behind it), and the kernel that writes a plan.
// Plan layout: header words, directory [pairs][2] int32, one 16-byte descriptor per tile.
struct PlanLayout {
  int64_t hdr_bytes, dir_bytes, desc_bytes;
  int64_t tiles_cap;         // descriptors the buffer has room for
  int64_t total() const { return hdr_bytes + dir_bytes + desc_bytes; }
};
PlanLayout plan_layout(const pkv_attn_desc& d);
hipError_t launch_attn_flat(const AttnParams& p, int gh, hipStream_t s);
hipError_t launch_attn_plan(AttnParams& p, int32_t* plan_hdr, hipStream_t s);
// swap.hip
// max_workgroups > 0 caps the grid (a copy that a slower link bounds needs few)
hipError_t launch_swap(const SwapParams& p, hipStream_t s, int max_workgroups = 0);
// attn_prefill_mfma.hip
bool attn_prefill_supported(const pkv_attn_desc& d);
hipError_t launch_attn_prefill(AttnParams& p, int max_query_len, int max_context_len, int64_t total_query_tokens,
                               hipStream_t s);
int prefill_splits(const pkv_attn_desc& d, int max_query_len);
size_t prefill_workspace_bytes(const pkv_attn_desc& d, int64_t total_query_tokens, int max_query_len);

// dequant.hip: the bf16 copy of the blocks a prefill call over 8-bit pools reads
struct F8PrefillCopy {
  int32_t blocks_per_seq;   // rows of the copy's block table
  size_t pool_bytes;        // of the K copy, and of the V copy
  size_t table_bytes;
  size_t total() const { return 2 * pool_bytes + table_bytes; }
};
F8PrefillCopy f8_prefill_copy_layout(const pkv_attn_desc& d);
hipError_t launch_f8_blocks_to_bf16(const AttnParams& p, uint8_t* k_copy, uint8_t* v_copy, int32_t* copy_table,
                                    int blocks_per_seq, hipStream_t s);
// append.hip (uses the pointers, strides and shapes of AttnParams; q/out unused)
hipError_t launch_kv_append(const AttnParams& p, const void* k_new, const void* v_new, int elem_bytes,
                            hipStream_t s);
hipError_t launch_kv_append_chunk(const AttnParams& p, const void* k_new, const void* v_new, int elem_bytes,
                                  int64_t total_rows, hipStream_t s);
// swap_host.hip
hipError_t swap_out_host(const pkv_swap_desc& d, const uint8_t* pool, uint8_t* host_dst, const int32_t* mapping,
                         int32_t n_pairs, uint8_t* staging, size_t staging_bytes, hipStream_t stream,
                         bool* too_small);
hipError_t swap_in_host(const pkv_swap_desc& d, const uint8_t* host_src, uint8_t* pool, const int32_t* mapping,
                        int32_t n_pairs, uint8_t* staging, size_t staging_bytes, hipStream_t stream,
                        bool* too_small);
// the same without a staging buffer: the copy kernel reads or writes the page-locked host memory
// itself (out: pool -> host slots; else host slots -> pool)
hipError_t swap_host_direct(bool out, const pkv_swap_desc& d, const uint8_t* src, uint8_t* dst,
                            const int32_t* mapping, int32_t n_pairs, hipStream_t stream);
hipError_t launch_probe_copy(const void* src, void* dst, size_t bytes, hipStream_t s);
hipError_t launch_probe_read(const void* src, void* sink, size_t bytes, hipStream_t s);

}  // namespace pkv
