// extern "C" entry points of libpkv: host-side validation and launch set-up.
// Everything that can be checked without touching device memory is checked
// here, before any kernel is enqueued.

#include <cmath>
#include <cstring>
#include <vector>

#include "pkv_bench.h"
#include "pkv_internal.h"

namespace {

using namespace pkv;

// Runtime error behind the most recent PKV_ERR_HIP of this thread (diagnostics only).
thread_local hipError_t g_last_hip_error = hipSuccess;

inline int32_t hip_status(hipError_t e) {
  if (e == hipSuccess) return PKV_OK;
  g_last_hip_error = e;
  return PKV_ERR_HIP;
}

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

inline int elem_bytes(int dtype) { return dtype == PKV_BF16 ? 2 : dtype == PKV_F32 ? 4 : dtype == PKV_F8_E4M3 ? 1 : 0; }

// dequantisation factor of an 8-bit pool as given in the descriptor (0 stands for 1)
inline float pool_scale(const pkv_attn_desc* d, float s) { return d->kv_dtype == PKV_F8_E4M3 && s != 0.f ? s : 1.0f; }

// The library's own choice for the vector-ALU kernel (the streaming kernels cut the work
// themselves): 512 tokens, which keeps every CU busy on small batches; 2048 when the batch alone
// brings two (sequence, KV head) streams per CU or more, where the shorter partitions only add
// workgroup set-up, partials and merge work (measured on 64 sequences of 128..4096 tokens: 16/8
// heads of 256 dims 47.9 -> 52.3 % of the HBM peak, 32/8 heads of 64 dims 31.3 -> 34.3 %).
int default_partition(const pkv_attn_desc* d) {
  const int64_t group = d->num_kv_heads > 0 ? d->num_q_heads / d->num_kv_heads : 1;
  const int64_t streams = (int64_t)d->batch * d->num_kv_heads * ((group + 7) / 8);
  return streams >= 512 ? 4 * kDefaultPartition : kDefaultPartition;
}

int32_t partition_tokens_of(const pkv_attn_desc* d) {
  if (!d) return 0;
  const int pt = d->partition_tokens == 0 ? default_partition(d) : d->partition_tokens;
  if (pt < 64 || pt % 64 != 0) return 0;
  return pt;
}

int32_t max_partitions_of(const pkv_attn_desc* d) {
  const int pt = partition_tokens_of(d);
  if (pt == 0) return 0;
  const int64_t mc = d->max_context_len;
  return mc <= 0 ? 1 : (int32_t)((mc + pt - 1) / pt);
}

// Static checks of an attention descriptor (no pointers).
int32_t check_attn_desc(const pkv_attn_desc* d) {
  if (!d) return PKV_ERR_NULL;
  const int eb = elem_bytes(d->kv_dtype);
  if (eb == 0) return PKV_ERR_DTYPE;
  if (d->out_dtype != PKV_F32 && d->out_dtype != PKV_BF16) return PKV_ERR_DTYPE;
  if (d->batch < 0 || d->num_q_heads <= 0 || d->num_kv_heads <= 0 || d->head_dim <= 0 ||
      d->block_size <= 0 || d->num_pool_blocks <= 0 || d->max_blocks_per_seq <= 0 ||
      d->max_context_len < 0 || d->partition_tokens < 0 ||
      (d->flags & ~(int32_t)PKV_ATTN_FLAG_VECTOR_ALU) != 0)
    return PKV_ERR_SHAPE;
  if (d->num_q_heads % d->num_kv_heads != 0) return PKV_ERR_SHAPE;
  if (d->block_size % kTileTokens != 0) return PKV_ERR_SHAPE;
  const int row_bytes = d->head_dim * eb;
  if (row_bytes != 128 && row_bytes != 256 && row_bytes != 512) return PKV_ERR_SHAPE;
  if (partition_tokens_of(d) == 0) return PKV_ERR_SHAPE;
  if (d->kv_dtype == PKV_F8_E4M3 &&
      (!std::isfinite(d->k_scale) || !std::isfinite(d->v_scale) || d->k_scale < 0.f || d->v_scale < 0.f))
    return PKV_ERR_SHAPE;
  if ((int64_t)d->max_blocks_per_seq * d->block_size < d->max_context_len) return PKV_ERR_SHAPE;
  const int64_t st[6] = {d->k_stride_block, d->k_stride_head, d->k_stride_token,
                         d->v_stride_block, d->v_stride_head, d->v_stride_token};
  for (int i = 0; i < 6; ++i) {
    if (st[i] < 0) return PKV_ERR_SHAPE;
    if ((st[i] * eb) % 16 != 0) return PKV_ERR_ALIGN;
  }
  if (d->k_stride_token < d->head_dim || d->v_stride_token < d->head_dim) return PKV_ERR_SHAPE;
  return PKV_OK;
}

int32_t check_swap_desc(const pkv_swap_desc* d) {
  if (!d) return PKV_ERR_NULL;
  if (d->num_planes <= 0 || d->src_num_blocks <= 0 || d->dst_num_blocks <= 0 ||
      d->block_bytes <= 0 || d->reserved != 0)
    return PKV_ERR_SHAPE;
  if (d->block_bytes % 16 != 0 || d->src_plane_stride_bytes % 16 != 0 ||
      d->dst_plane_stride_bytes % 16 != 0)
    return PKV_ERR_ALIGN;
  if (d->src_plane_stride_bytes < (int64_t)d->src_num_blocks * d->block_bytes ||
      d->dst_plane_stride_bytes < (int64_t)d->dst_num_blocks * d->block_bytes)
    return PKV_ERR_SHAPE;
  return PKV_OK;
}

}  // namespace

extern "C" {

int32_t pkv_version(void) { return 300; }

int32_t pkv_init(void) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return hip_status(e);
  (void)num_cus();
  if ((e = prepare_attn_stream()) != hipSuccess) return hip_status(e);
  if ((e = prepare_attn_prefill()) != hipSuccess) return hip_status(e);
  if ((e = prepare_static_scratch()) != hipSuccess) return hip_status(e);
  return PKV_OK;
}

const char* pkv_status_string(int32_t status) {
  switch (status) {
    case PKV_OK: return "PKV_OK";
    case PKV_ERR_NULL: return "PKV_ERR_NULL";
    case PKV_ERR_SHAPE: return "PKV_ERR_SHAPE";
    case PKV_ERR_DTYPE: return "PKV_ERR_DTYPE";
    case PKV_ERR_ALIGN: return "PKV_ERR_ALIGN";
    case PKV_ERR_WORKSPACE: return "PKV_ERR_WORKSPACE";
    case PKV_ERR_INDEX: return "PKV_ERR_INDEX";
    case PKV_ERR_HIP: return "PKV_ERR_HIP";
    default: return "PKV_ERR_UNKNOWN";
  }
}

const char* pkv_last_hip_error_string(void) { return hipGetErrorString(g_last_hip_error); }

int32_t pkv_attn_partition_tokens(const pkv_attn_desc* desc) { return partition_tokens_of(desc); }

size_t pkv_attn_workspace_bytes(const pkv_attn_desc* desc) {
  if (check_attn_desc(desc) != PKV_OK) return 0;
  if (desc->batch == 0) return 0;
  if (attn_stream_supported(*desc)) return (size_t)stream_workspace(*desc).total();
  const int64_t P = max_partitions_of(desc);
  if (P <= 1) return 0;
  const int64_t rows = (int64_t)desc->batch * desc->num_q_heads * P;
  const int64_t ml = (rows * 2 * (int64_t)sizeof(float) + 255) / 256 * 256;
  const int64_t o = rows * desc->head_dim * (int64_t)sizeof(float);
  return (size_t)(ml + (o + 255) / 256 * 256);
}

size_t pkv_attn_plan_bytes(const pkv_attn_desc* desc) {
  if (check_attn_desc(desc) != PKV_OK || desc->batch == 0 || !attn_stream_supported(*desc)) return 0;
  return (size_t)plan_layout(*desc).total();
}

}  // extern "C"

namespace {

// What of a descriptor a plan depends on, folded into one positive number.
int32_t plan_key_of(const pkv_attn_desc* d) {
  const int64_t f[] = {d->batch, d->num_q_heads, d->num_kv_heads, d->head_dim, d->block_size, d->num_pool_blocks,
                       d->max_blocks_per_seq, d->max_context_len, d->partition_tokens, d->kv_dtype,
                       d->k_stride_block, d->k_stride_head, d->k_stride_token,
                       d->v_stride_block, d->v_stride_head, d->v_stride_token, num_cus()};
  uint64_t h = 0x9E3779B97F4A7C15ull;
  for (int64_t v : f) {
    h ^= (uint64_t)v + 0x9E3779B97F4A7C15ull + (h << 6) + (h >> 2);
    h *= 0xFF51AFD7ED558CCDull;
  }
  return (int32_t)((h >> 33) | 1u);
}

// geometry fields of the launch parameters that the attention call and the plan share
void fill_geometry(AttnParams& p, const pkv_attn_desc* desc) {
  const int eb = elem_bytes(desc->kv_dtype);
  p.k_stride_block = desc->k_stride_block * eb;
  p.k_stride_head = desc->k_stride_head * eb;
  p.k_stride_token = desc->k_stride_token * eb;
  p.v_stride_block = desc->v_stride_block * eb;
  p.v_stride_head = desc->v_stride_head * eb;
  p.v_stride_token = desc->v_stride_token * eb;
  p.batch = desc->batch; p.num_q_heads = desc->num_q_heads; p.num_kv_heads = desc->num_kv_heads;
  p.head_dim = desc->head_dim; p.block_size = desc->block_size;
  p.max_blocks_per_seq = desc->max_blocks_per_seq;
  p.group = desc->num_q_heads / desc->num_kv_heads;
  p.group_tiles = 1;
  p.partition_tokens = partition_tokens_of(desc);
  p.max_partitions = max_partitions_of(desc);
  p.kv_is_f8 = desc->kv_dtype == PKV_F8_E4M3;
}

// the plan buffer's parts as launch parameters
void fill_plan(AttnParams& p, const pkv_attn_desc* desc, const void* plan) {
  const PlanLayout l = plan_layout(*desc);
  // (the directory is written by the plan kernel only: the attention call, which has the
  // plan as read-only memory, reads it through the same field)
  uint8_t* base = const_cast<uint8_t*>(reinterpret_cast<const uint8_t*>(plan));
  p.plan_hdr = reinterpret_cast<const int32_t*>(base);
  p.ws_dir = reinterpret_cast<int32_t*>(base + l.hdr_bytes);
  p.plan_desc = base + l.hdr_bytes + l.dir_bytes;
  p.plan_key = plan_key_of(desc);
  p.plan_tiles_cap = (int32_t)l.tiles_cap;
}

}  // namespace

extern "C" int32_t pkv_attn_plan(const pkv_attn_desc* desc, const int32_t* block_tables, const int32_t* context_lens,
                                 void* plan, size_t plan_bytes, void* hip_stream) {
  const int32_t st = check_attn_desc(desc);
  if (st != PKV_OK) return st;
  const size_t need = pkv_attn_plan_bytes(desc);
  if (need == 0) return PKV_OK;                 // a call that has no use for a plan
  if (!block_tables || !context_lens || !plan) return PKV_ERR_NULL;
  if (!aligned16(plan) || (reinterpret_cast<uintptr_t>(block_tables) & 3u) ||
      (reinterpret_cast<uintptr_t>(context_lens) & 3u))
    return PKV_ERR_ALIGN;
  if (plan_bytes < need) return PKV_ERR_WORKSPACE;
  AttnParams p;
  std::memset(&p, 0, sizeof p);
  p.block_tables = block_tables; p.context_lens = context_lens;
  fill_geometry(p, desc);
  fill_plan(p, desc, plan);
  p.chunk_tiles_max = stream_workspace(*desc).chunk_tiles_max;
  return hip_status(launch_attn_plan(p, static_cast<int32_t*>(plan), static_cast<hipStream_t>(hip_stream)));
}

// The decode-attention call behind every entry point that has it: checks, then launches.
int32_t pkv::attention_call(const pkv_attn_desc* desc, const void* q, const void* k_pool,
                            const void* v_pool, const int32_t* block_tables,
                            const int32_t* context_lens, float scale, void* out, void* workspace,
                            size_t workspace_bytes, void* hip_stream, void* ev_begin, void* ev_end,
                            bool static_scratch, const void* plan, size_t plan_bytes, const void* k_new,
                            const void* v_new) {
  const int32_t st = check_attn_desc(desc);
  if (st != PKV_OK) return st;
  if (desc->batch == 0) return PKV_OK;
  if (!q || !k_pool || !v_pool || !block_tables || !context_lens || !out) return PKV_ERR_NULL;
  if ((k_new == nullptr) != (v_new == nullptr)) return PKV_ERR_NULL;
  if (!aligned16(k_new) || !aligned16(v_new)) return PKV_ERR_ALIGN;
  if (!aligned16(q) || !aligned16(k_pool) || !aligned16(v_pool) || !aligned16(out) ||
      !aligned16(workspace) || (reinterpret_cast<uintptr_t>(block_tables) & 3u) ||
      (reinterpret_cast<uintptr_t>(context_lens) & 3u))
    return PKV_ERR_ALIGN;
  if (!std::isfinite(scale)) return PKV_ERR_SHAPE;
  if (plan && pkv_attn_plan_bytes(desc) == 0) plan = nullptr;     // a call that has no use for a plan
  if (plan && (!aligned16(plan) || plan_bytes < pkv_attn_plan_bytes(desc))) return aligned16(plan) ? PKV_ERR_WORKSPACE : PKV_ERR_ALIGN;
  const size_t need = pkv_attn_workspace_bytes(desc);
  if (static_scratch) {
    // the library's own array takes the place of the caller's workspace; its device address is
    // asked for only now, after every check that needs no device
    if (need > static_scratch_bytes()) return PKV_ERR_WORKSPACE;
    if (need > 0) {
      const hipError_t e = static_scratch_address(&workspace);
      if (e != hipSuccess) return hip_status(e);
    }
  } else if (need > 0 && (!workspace || workspace_bytes < need)) {
    return PKV_ERR_WORKSPACE;
  }

  AttnParams p;
  std::memset(&p, 0, sizeof p);
  p.q = q; p.k_pool = k_pool; p.v_pool = v_pool;
  p.block_tables = block_tables; p.context_lens = context_lens; p.out = out;
  fill_geometry(p, desc);
  if (k_new) {
    // the streaming kernels that take a plan append by themselves; everywhere else the append
    // is a launch of its own in front of the attention
    if (plan) {
      p.k_new = k_new;
      p.v_new = v_new;
    } else {
      const hipError_t e = launch_kv_append(p, k_new, v_new, elem_bytes(desc->kv_dtype),
                                            static_cast<hipStream_t>(hip_stream));
      if (e != hipSuccess) return hip_status(e);
    }
  }
  p.out_is_bf16 = desc->out_dtype == PKV_BF16;
  p.no_mfma = (desc->flags & PKV_ATTN_FLAG_VECTOR_ALU) != 0;
  p.scale_log2e = scale * pool_scale(desc, desc->k_scale) * 1.4426950408889634f;
  p.v_scale = pool_scale(desc, desc->v_scale);
  p.ev_begin = static_cast<hipEvent_t>(ev_begin);
  p.ev_end = static_cast<hipEvent_t>(ev_end);
  if (attn_stream_supported(*desc)) {
    const StreamWorkspace w = stream_workspace(*desc);
    uint8_t* base = reinterpret_cast<uint8_t*>(workspace);
    p.ws_dir = reinterpret_cast<int32_t*>(base);
    if (plan) fill_plan(p, desc, plan);      // (the directory is the plan's)
    p.ws_ml = reinterpret_cast<float*>(base + w.dir_bytes);
    p.ws_o = reinterpret_cast<float*>(base + w.dir_bytes + w.ml_bytes);
    p.chunk_tiles_max = w.chunk_tiles_max;
    // With a cap on the chunk there can be more partial rows than the 32 MiB of L2 hold: stored
    // the ordinary way they trickle out to HBM between the reads of the K/V stream, which cost
    // 16 % on the long-context configuration; nontemporal stores cost 12 % there (988 -> 953 us).
    // Few partials are better left in L2 for the merge kernel (90 against 92 us on the B=64 batch).
    p.partials_streaming = w.chunk_tiles_max > 0 && w.o_bytes > (32 << 20);
    const hipError_t e = launch_attn_stream(p, static_cast<hipStream_t>(hip_stream));
    return hip_status(e);
  }
  if (need > 0) {
    const int64_t rows = (int64_t)desc->batch * desc->num_q_heads * p.max_partitions;
    const int64_t ml = (rows * 2 * (int64_t)sizeof(float) + 255) / 256 * 256;
    p.ws_ml = reinterpret_cast<float*>(workspace);
    p.ws_o = reinterpret_cast<float*>(reinterpret_cast<uint8_t*>(workspace) + ml);
  }
  const hipError_t e = launch_attn_decode(p, desc->kv_dtype, static_cast<hipStream_t>(hip_stream));
  return hip_status(e);
}

extern "C" {

int32_t paged_decode_attention(const pkv_attn_desc* desc, const void* q, const void* k_pool,
                               const void* v_pool, const int32_t* block_tables,
                               const int32_t* context_lens, float scale, void* out,
                               void* workspace, size_t workspace_bytes, void* hip_stream) {
  return attention_call(desc, q, k_pool, v_pool, block_tables, context_lens, scale, out, workspace,
                        workspace_bytes, hip_stream, nullptr, nullptr, false, nullptr, 0, nullptr, nullptr);
}

int32_t paged_decode_attention_planned(const pkv_attn_desc* desc, const void* plan, size_t plan_bytes, const void* q,
                                       const void* k_pool, const void* v_pool, const int32_t* block_tables,
                                       const int32_t* context_lens, float scale, void* out, void* workspace,
                                       size_t workspace_bytes, void* hip_stream) {
  return attention_call(desc, q, k_pool, v_pool, block_tables, context_lens, scale, out, workspace,
                        workspace_bytes, hip_stream, nullptr, nullptr, false, plan, plan_bytes, nullptr, nullptr);
}

int32_t paged_decode_attention_planned_append(const pkv_attn_desc* desc, const void* plan, size_t plan_bytes,
                                              const void* q, const void* k_new, const void* v_new, void* k_pool,
                                              void* v_pool, const int32_t* block_tables, const int32_t* context_lens,
                                              float scale, void* out, void* workspace, size_t workspace_bytes,
                                              void* hip_stream) {
  if (!k_new || !v_new) return PKV_ERR_NULL;
  return attention_call(desc, q, k_pool, v_pool, block_tables, context_lens, scale, out, workspace,
                        workspace_bytes, hip_stream, nullptr, nullptr, false, plan, plan_bytes, k_new, v_new);
}

int32_t paged_decode_attention_timed(const pkv_attn_desc* desc, const void* q, const void* k_pool,
                                     const void* v_pool, const int32_t* block_tables,
                                     const int32_t* context_lens, float scale, void* out,
                                     void* workspace, size_t workspace_bytes, void* hip_stream,
                                     void* ev_kernel_begin, void* ev_kernel_end) {
  return attention_call(desc, q, k_pool, v_pool, block_tables, context_lens, scale, out, workspace,
                        workspace_bytes, hip_stream, ev_kernel_begin, ev_kernel_end, false, nullptr, 0, nullptr, nullptr);
}

int32_t paged_decode_attention_planned_timed(const pkv_attn_desc* desc, const void* plan, size_t plan_bytes, const void* q,
                                             const void* k_pool, const void* v_pool, const int32_t* block_tables,
                                             const int32_t* context_lens, float scale, void* out, void* workspace,
                                             size_t workspace_bytes, void* hip_stream, void* ev_kernel_begin,
                                             void* ev_kernel_end) {
  return attention_call(desc, q, k_pool, v_pool, block_tables, context_lens, scale, out, workspace,
                        workspace_bytes, hip_stream, ev_kernel_begin, ev_kernel_end, false, plan, plan_bytes, nullptr, nullptr);
}

size_t pkv_prefill_workspace_bytes(const pkv_attn_desc* desc, int64_t total_query_tokens,
                                   int32_t max_query_len) {
  if (check_attn_desc(desc) != PKV_OK || max_query_len <= 0 || total_query_tokens <= 0) return 0;
  pkv_attn_desc b = *desc;                     // the kernel's own view: bf16 pools (8-bit ones are copied)
  if (desc->kv_dtype == PKV_F8_E4M3) b.kv_dtype = PKV_BF16;
  if (b.kv_dtype != PKV_BF16 || !attn_prefill_supported(b)) return 0;
  const size_t split = prefill_workspace_bytes(b, total_query_tokens, max_query_len);
  return desc->kv_dtype == PKV_F8_E4M3 ? f8_prefill_copy_layout(*desc).total() + split : split;
}

int32_t paged_prefill_attention(const pkv_attn_desc* desc, const void* q, const void* k_pool,
                                const void* v_pool, const int32_t* block_tables,
                                const int32_t* context_lens, const int32_t* query_lens,
                                const int32_t* cu_query_lens, int32_t max_query_len, float scale,
                                void* out, void* hip_stream) {
  return paged_prefill_attention_ws(desc, q, k_pool, v_pool, block_tables, context_lens, query_lens,
                                    cu_query_lens, max_query_len, 0, scale, out, nullptr, 0, hip_stream);
}

int32_t paged_prefill_attention_ws(const pkv_attn_desc* desc, const void* q, const void* k_pool,
                                   const void* v_pool, const int32_t* block_tables,
                                   const int32_t* context_lens, const int32_t* query_lens,
                                   const int32_t* cu_query_lens, int32_t max_query_len,
                                   int64_t total_query_tokens, float scale, void* out,
                                   void* workspace, size_t workspace_bytes, void* hip_stream) {
  const int32_t st = check_attn_desc(desc);
  if (st != PKV_OK) return st;
  if (max_query_len < 0 || total_query_tokens < 0) return PKV_ERR_SHAPE;
  if (desc->batch == 0 || max_query_len == 0) return PKV_OK;
  const bool f8 = desc->kv_dtype == PKV_F8_E4M3;
  if (desc->kv_dtype != PKV_BF16 && !f8) return PKV_ERR_DTYPE;
  pkv_attn_desc bdesc = *desc;                 // what the kernel walks: bf16 pools
  bdesc.kv_dtype = PKV_BF16;
  if (!attn_prefill_supported(bdesc)) return PKV_ERR_SHAPE;
  if (!q || !k_pool || !v_pool || !block_tables || !context_lens || !query_lens || !cu_query_lens || !out)
    return PKV_ERR_NULL;
  if (!aligned16(q) || !aligned16(k_pool) || !aligned16(v_pool) || !aligned16(out) ||
      (reinterpret_cast<uintptr_t>(block_tables) & 3u) || (reinterpret_cast<uintptr_t>(context_lens) & 3u) ||
      (reinterpret_cast<uintptr_t>(query_lens) & 3u) || (reinterpret_cast<uintptr_t>(cu_query_lens) & 3u))
    return PKV_ERR_ALIGN;
  if (!std::isfinite(scale)) return PKV_ERR_SHAPE;
  AttnParams p;
  std::memset(&p, 0, sizeof p);
  p.q = q; p.k_pool = k_pool; p.v_pool = v_pool;
  p.block_tables = block_tables; p.context_lens = context_lens;
  p.query_lens = query_lens; p.cu_query_lens = cu_query_lens; p.out = out;
  p.k_stride_block = desc->k_stride_block * 2;
  p.k_stride_head = desc->k_stride_head * 2;
  p.k_stride_token = desc->k_stride_token * 2;
  p.v_stride_block = desc->v_stride_block * 2;
  p.v_stride_head = desc->v_stride_head * 2;
  p.v_stride_token = desc->v_stride_token * 2;
  p.batch = desc->batch; p.num_q_heads = desc->num_q_heads; p.num_kv_heads = desc->num_kv_heads;
  p.head_dim = desc->head_dim; p.block_size = desc->block_size;
  p.max_blocks_per_seq = desc->max_blocks_per_seq;
  p.group = desc->num_q_heads / desc->num_kv_heads;
  p.out_is_bf16 = desc->out_dtype == PKV_BF16;
  p.scale_log2e = scale * pool_scale(desc, desc->k_scale) * 1.4426950408889634f;
  p.v_scale = pool_scale(desc, desc->v_scale);
  if (!std::isfinite(p.scale_log2e) || !std::isfinite(p.v_scale)) return PKV_ERR_SHAPE;
  uint8_t* ws = static_cast<uint8_t*>(workspace);
  size_t ws_left = workspace ? workspace_bytes : 0;
  if (f8) {
    // 8-bit pools: the blocks of the call's sequences are decoded into a bf16 copy at the head
    // of the workspace, and the kernel walks the copy through the copy's own block table
    const F8PrefillCopy c = f8_prefill_copy_layout(*desc);
    if (!workspace || ws_left < c.total()) return PKV_ERR_WORKSPACE;
    if (!aligned16(workspace)) return PKV_ERR_ALIGN;
    AttnParams src = p;                        // the 8-bit pools: one byte per element
    src.k_stride_block = desc->k_stride_block; src.k_stride_head = desc->k_stride_head;
    src.k_stride_token = desc->k_stride_token;
    src.v_stride_block = desc->v_stride_block; src.v_stride_head = desc->v_stride_head;
    src.v_stride_token = desc->v_stride_token;
    uint8_t* k_copy = ws;
    uint8_t* v_copy = ws + c.pool_bytes;
    int32_t* table = reinterpret_cast<int32_t*>(ws + 2 * c.pool_bytes);
    const hipError_t e = launch_f8_blocks_to_bf16(src, k_copy, v_copy, table, c.blocks_per_seq,
                                                  static_cast<hipStream_t>(hip_stream));
    if (e != hipSuccess) return hip_status(e);
    p.k_pool = k_copy; p.v_pool = v_copy; p.block_tables = table;
    p.max_blocks_per_seq = c.blocks_per_seq;
    p.k_stride_token = p.v_stride_token = (int64_t)desc->head_dim * 2;
    p.k_stride_head = p.v_stride_head = p.k_stride_token * desc->block_size;
    p.k_stride_block = p.v_stride_block = p.k_stride_head * desc->num_kv_heads;
    ws += c.total();
    ws_left -= c.total();
  }
  // the walks are split only if the caller brought the workspace for it
  p.max_partitions = 1;
  if (ws_left > 0 && total_query_tokens > 0) {
    const int ns = prefill_splits(bdesc, max_query_len);
    const size_t need = prefill_workspace_bytes(bdesc, total_query_tokens, max_query_len);
    if (ns > 1) {
      if (ws_left < need) return PKV_ERR_WORKSPACE;
      if (!aligned16(ws)) return PKV_ERR_ALIGN;
      p.max_partitions = ns;
      p.ws_ml = reinterpret_cast<float*>(ws);
      p.ws_o = p.ws_ml + (size_t)total_query_tokens * desc->num_q_heads * ns * 2;
    }
  }
  return hip_status(launch_attn_prefill(p, max_query_len, desc->max_context_len, total_query_tokens,
                                        static_cast<hipStream_t>(hip_stream)));
}

int32_t kv_append(const pkv_attn_desc* desc, const void* k_new, const void* v_new, void* k_pool,
                  void* v_pool, const int32_t* block_tables, const int32_t* context_lens,
                  void* hip_stream) {
  const int32_t st = check_attn_desc(desc);
  if (st != PKV_OK) return st;
  if (desc->batch == 0) return PKV_OK;
  if (!k_new || !v_new || !k_pool || !v_pool || !block_tables || !context_lens) return PKV_ERR_NULL;
  if (!aligned16(k_new) || !aligned16(v_new) || !aligned16(k_pool) || !aligned16(v_pool) ||
      (reinterpret_cast<uintptr_t>(block_tables) & 3u) ||
      (reinterpret_cast<uintptr_t>(context_lens) & 3u))
    return PKV_ERR_ALIGN;
  const int eb = elem_bytes(desc->kv_dtype);
  AttnParams p;
  std::memset(&p, 0, sizeof p);
  p.k_pool = k_pool; p.v_pool = v_pool;
  p.block_tables = block_tables; p.context_lens = context_lens;
  p.k_stride_block = desc->k_stride_block * eb;
  p.k_stride_head = desc->k_stride_head * eb;
  p.k_stride_token = desc->k_stride_token * eb;
  p.v_stride_block = desc->v_stride_block * eb;
  p.v_stride_head = desc->v_stride_head * eb;
  p.v_stride_token = desc->v_stride_token * eb;
  p.batch = desc->batch; p.num_kv_heads = desc->num_kv_heads;
  p.head_dim = desc->head_dim; p.block_size = desc->block_size;
  p.max_blocks_per_seq = desc->max_blocks_per_seq;
  const hipError_t e = launch_kv_append(p, k_new, v_new, eb, static_cast<hipStream_t>(hip_stream));
  return hip_status(e);
}

int32_t kv_append_chunk(const pkv_attn_desc* desc, const void* k_new, const void* v_new, void* k_pool,
                        void* v_pool, const int32_t* block_tables, const int32_t* context_lens,
                        const int32_t* query_lens, const int32_t* cu_query_lens,
                        int64_t total_query_tokens, void* hip_stream) {
  const int32_t st = check_attn_desc(desc);
  if (st != PKV_OK) return st;
  if (total_query_tokens < 0) return PKV_ERR_SHAPE;
  if (desc->batch == 0 || total_query_tokens == 0) return PKV_OK;
  if (!k_new || !v_new || !k_pool || !v_pool || !block_tables || !context_lens || !query_lens || !cu_query_lens)
    return PKV_ERR_NULL;
  if (!aligned16(k_new) || !aligned16(v_new) || !aligned16(k_pool) || !aligned16(v_pool) ||
      (reinterpret_cast<uintptr_t>(block_tables) & 3u) || (reinterpret_cast<uintptr_t>(context_lens) & 3u) ||
      (reinterpret_cast<uintptr_t>(query_lens) & 3u) || (reinterpret_cast<uintptr_t>(cu_query_lens) & 3u))
    return PKV_ERR_ALIGN;
  const int eb = elem_bytes(desc->kv_dtype);
  AttnParams p;
  std::memset(&p, 0, sizeof p);
  p.k_pool = k_pool; p.v_pool = v_pool;
  p.block_tables = block_tables; p.context_lens = context_lens;
  p.query_lens = query_lens; p.cu_query_lens = cu_query_lens;
  p.k_stride_block = desc->k_stride_block * eb;
  p.k_stride_head = desc->k_stride_head * eb;
  p.k_stride_token = desc->k_stride_token * eb;
  p.v_stride_block = desc->v_stride_block * eb;
  p.v_stride_head = desc->v_stride_head * eb;
  p.v_stride_token = desc->v_stride_token * eb;
  p.batch = desc->batch; p.num_kv_heads = desc->num_kv_heads;
  p.head_dim = desc->head_dim; p.block_size = desc->block_size;
  p.max_blocks_per_seq = desc->max_blocks_per_seq;
  const hipError_t e = launch_kv_append_chunk(p, k_new, v_new, eb, total_query_tokens,
                                              static_cast<hipStream_t>(hip_stream));
  return hip_status(e);
}

int32_t kv_block_swap(const pkv_swap_desc* desc, const void* src_pool, void* dst,
                      const int32_t* block_mapping, int32_t n_pairs, void* hip_stream) {
  const int32_t st = check_swap_desc(desc);
  if (st != PKV_OK) return st;
  if (n_pairs < 0) return PKV_ERR_SHAPE;
  if (n_pairs == 0) return PKV_OK;
  if (!src_pool || !dst || !block_mapping) return PKV_ERR_NULL;
  if (!aligned16(src_pool) || !aligned16(dst) || (reinterpret_cast<uintptr_t>(block_mapping) & 3u))
    return PKV_ERR_ALIGN;
  SwapParams p;
  p.src = static_cast<const uint8_t*>(src_pool);
  p.dst = static_cast<uint8_t*>(dst);
  p.mapping = block_mapping;
  p.block_bytes = desc->block_bytes;
  p.src_plane_stride = desc->src_plane_stride_bytes;
  p.dst_plane_stride = desc->dst_plane_stride_bytes;
  p.num_planes = desc->num_planes;
  p.n_pairs = n_pairs;
  p.src_slot_is_pair = 0;
  p.dst_slot_is_pair = 0;
  const hipError_t e = launch_swap(p, static_cast<hipStream_t>(hip_stream));
  return hip_status(e);
}

static int32_t swap_host_impl(bool out, const pkv_swap_desc* desc, const void* src, void* dst,
                              const int32_t* block_mapping, int32_t n_pairs, void* staging,
                              size_t staging_bytes, void* hip_stream) {
  const int32_t st = check_swap_desc(desc);
  if (st != PKV_OK) return st;
  if (n_pairs < 0) return PKV_ERR_SHAPE;
  if (n_pairs == 0) return PKV_OK;
  const bool direct = !staging && staging_bytes == 0;   // no staging buffer: the kernel touches the host memory itself
  if (!src || !dst || !block_mapping || (!staging && !direct)) return PKV_ERR_NULL;
  if (!aligned16(src) || !aligned16(dst) || !aligned16(staging) ||
      (reinterpret_cast<uintptr_t>(block_mapping) & 3u))
    return PKV_ERR_ALIGN;
  // the host side holds one slot per pair
  if ((out ? desc->dst_num_blocks : desc->src_num_blocks) < n_pairs) return PKV_ERR_SHAPE;
  if (direct)
    return hip_status(swap_host_direct(out, *desc, static_cast<const uint8_t*>(src), static_cast<uint8_t*>(dst),
                                       block_mapping, n_pairs, static_cast<hipStream_t>(hip_stream)));
  bool too_small = false;
  const hipError_t e =
      out ? swap_out_host(*desc, static_cast<const uint8_t*>(src), static_cast<uint8_t*>(dst),
                          block_mapping, n_pairs, static_cast<uint8_t*>(staging), staging_bytes,
                          static_cast<hipStream_t>(hip_stream), &too_small)
          : swap_in_host(*desc, static_cast<const uint8_t*>(src), static_cast<uint8_t*>(dst),
                         block_mapping, n_pairs, static_cast<uint8_t*>(staging), staging_bytes,
                         static_cast<hipStream_t>(hip_stream), &too_small);
  if (too_small) return PKV_ERR_WORKSPACE;
  return hip_status(e);
}

int32_t kv_swap_out_host(const pkv_swap_desc* desc, const void* src_pool, void* host_dst,
                         const int32_t* block_mapping, int32_t n_pairs, void* staging,
                         size_t staging_bytes, void* hip_stream) {
  return swap_host_impl(true, desc, src_pool, host_dst, block_mapping, n_pairs, staging,
                        staging_bytes, hip_stream);
}

int32_t kv_swap_in_host(const pkv_swap_desc* desc, const void* host_src, void* dst_pool,
                        const int32_t* block_mapping, int32_t n_pairs, void* staging,
                        size_t staging_bytes, void* hip_stream) {
  return swap_host_impl(false, desc, host_src, dst_pool, block_mapping, n_pairs, staging,
                        staging_bytes, hip_stream);
}

int32_t pkv_validate_tables_host(const pkv_attn_desc* desc, const int32_t* block_tables_host,
                                 const int32_t* context_lens_host) {
  const int32_t st = check_attn_desc(desc);
  if (st != PKV_OK) return st;
  if (desc->batch == 0) return PKV_OK;
  if (!block_tables_host || !context_lens_host) return PKV_ERR_NULL;
  for (int i = 0; i < desc->batch; ++i) {
    const int64_t n = context_lens_host[i];
    if (n < 0 || n > desc->max_context_len) return PKV_ERR_INDEX;
    const int64_t nb = (n + desc->block_size - 1) / desc->block_size;
    if (nb > desc->max_blocks_per_seq) return PKV_ERR_INDEX;
    const int32_t* row = block_tables_host + (int64_t)i * desc->max_blocks_per_seq;
    for (int64_t b = 0; b < nb; ++b)
      if (row[b] < 0 || row[b] >= desc->num_pool_blocks) return PKV_ERR_INDEX;
  }
  return PKV_OK;
}

int32_t pkv_validate_mapping_host(const pkv_swap_desc* desc, const int32_t* block_mapping_host,
                                  int32_t n_pairs) {
  const int32_t st = check_swap_desc(desc);
  if (st != PKV_OK) return st;
  if (n_pairs < 0) return PKV_ERR_SHAPE;
  if (n_pairs == 0) return PKV_OK;
  if (!block_mapping_host) return PKV_ERR_NULL;
  std::vector<uint8_t> seen((size_t)desc->dst_num_blocks, 0);
  for (int j = 0; j < n_pairs; ++j) {
    const int32_t s = block_mapping_host[2 * j], d = block_mapping_host[2 * j + 1];
    if (s < 0 || s >= desc->src_num_blocks || d < 0 || d >= desc->dst_num_blocks)
      return PKV_ERR_INDEX;
    if (seen[d]) return PKV_ERR_INDEX;  // two writers of one destination block
    seen[d] = 1;
  }
  return PKV_OK;
}

int32_t pkv_validate_chunks_host(const pkv_attn_desc* desc, const int32_t* context_lens_host,
                                 const int32_t* query_lens_host, const int32_t* cu_query_lens_host,
                                 int32_t max_query_len, int64_t total_query_tokens) {
  const int32_t st = check_attn_desc(desc);
  if (st != PKV_OK) return st;
  if (max_query_len < 0 || total_query_tokens < 0) return PKV_ERR_SHAPE;
  if (desc->batch == 0) return PKV_OK;
  if (!context_lens_host || !query_lens_host || !cu_query_lens_host) return PKV_ERR_NULL;
  if (cu_query_lens_host[0] != 0) return PKV_ERR_INDEX;
  for (int i = 0; i < desc->batch; ++i) {
    const int64_t q = query_lens_host[i], n = context_lens_host[i];
    if (q < 0 || q > max_query_len || n < 0 || n > desc->max_context_len) return PKV_ERR_INDEX;
    // the rows of sequence i are exactly its query_lens[i] rows, back to back
    if ((int64_t)cu_query_lens_host[i + 1] - cu_query_lens_host[i] != q) return PKV_ERR_INDEX;
  }
  if (cu_query_lens_host[desc->batch] > total_query_tokens) return PKV_ERR_INDEX;
  return PKV_OK;
}

int32_t pkv_validate_chunks(const pkv_attn_desc* desc, const int32_t* context_lens,
                            const int32_t* query_lens, const int32_t* cu_query_lens,
                            int32_t max_query_len, int64_t total_query_tokens, void* hip_stream) {
  const int32_t st = check_attn_desc(desc);
  if (st != PKV_OK) return st;
  if (desc->batch == 0) return PKV_OK;
  if (!context_lens || !query_lens || !cu_query_lens) return PKV_ERR_NULL;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  const size_t B = (size_t)desc->batch;
  std::vector<int32_t> cl(B), ql(B), cu(B + 1);
  if (hipMemcpyAsync(cl.data(), context_lens, B * 4, hipMemcpyDeviceToHost, s) != hipSuccess ||
      hipMemcpyAsync(ql.data(), query_lens, B * 4, hipMemcpyDeviceToHost, s) != hipSuccess ||
      hipMemcpyAsync(cu.data(), cu_query_lens, (B + 1) * 4, hipMemcpyDeviceToHost, s) != hipSuccess ||
      hipStreamSynchronize(s) != hipSuccess)
    return PKV_ERR_HIP;
  return pkv_validate_chunks_host(desc, cl.data(), ql.data(), cu.data(), max_query_len, total_query_tokens);
}

int32_t pkv_validate_tables(const pkv_attn_desc* desc, const int32_t* block_tables,
                            const int32_t* context_lens, void* hip_stream) {
  const int32_t st = check_attn_desc(desc);
  if (st != PKV_OK) return st;
  if (desc->batch == 0) return PKV_OK;
  if (!block_tables || !context_lens) return PKV_ERR_NULL;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  std::vector<int32_t> lens((size_t)desc->batch);
  std::vector<int32_t> tab((size_t)desc->batch * desc->max_blocks_per_seq);
  if (hipMemcpyAsync(lens.data(), context_lens, lens.size() * 4, hipMemcpyDeviceToHost, s) !=
          hipSuccess ||
      hipMemcpyAsync(tab.data(), block_tables, tab.size() * 4, hipMemcpyDeviceToHost, s) !=
          hipSuccess ||
      hipStreamSynchronize(s) != hipSuccess)
    return PKV_ERR_HIP;
  return pkv_validate_tables_host(desc, tab.data(), lens.data());
}

int32_t pkv_validate_mapping(const pkv_swap_desc* desc, const int32_t* block_mapping,
                             int32_t n_pairs, void* hip_stream) {
  const int32_t st = check_swap_desc(desc);
  if (st != PKV_OK) return st;
  if (n_pairs < 0) return PKV_ERR_SHAPE;
  if (n_pairs == 0) return PKV_OK;
  if (!block_mapping) return PKV_ERR_NULL;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  std::vector<int32_t> m((size_t)n_pairs * 2);
  if (hipMemcpyAsync(m.data(), block_mapping, m.size() * 4, hipMemcpyDeviceToHost, s) !=
          hipSuccess ||
      hipStreamSynchronize(s) != hipSuccess)
    return PKV_ERR_HIP;
  return pkv_validate_mapping_host(desc, m.data(), n_pairs);
}

int32_t pkv_probe_copy(const void* src, void* dst, size_t bytes, void* hip_stream) {
  if (!src || !dst) return PKV_ERR_NULL;
  if (!aligned16(src) || !aligned16(dst) || bytes % 16 != 0) return PKV_ERR_ALIGN;
  if (bytes == 0) return PKV_OK;
  return hip_status(launch_probe_copy(src, dst, bytes, static_cast<hipStream_t>(hip_stream)));
}

int32_t pkv_probe_read(const void* src, void* sink, size_t bytes, void* hip_stream) {
  if (!src || !sink) return PKV_ERR_NULL;
  if (!aligned16(src) || !aligned16(sink) || bytes % 16 != 0) return PKV_ERR_ALIGN;
  if (bytes == 0) return PKV_OK;
  return hip_status(launch_probe_read(src, sink, bytes, static_cast<hipStream_t>(hip_stream)));
}

}  // extern "C"
