/*
 * pkv.h -- C ABI of the paged-KV decode-attention / KV-block-swap library for
 * AMD CDNA4 (gfx950).
 *
 * The paper (arXiv 2602.07878) studies a serving stack whose decode step
 * streams the whole KV history of every running request from HBM (Sec. 4.2,
 * the un-numbered execution-time model T_exec ~ N_ctx * d * sizeof(T) / BW_HBM)
 * out of a cache that is partitioned into fixed-size, physically
 * non-contiguous blocks (Sec. 2.2, "KV-Cache"), and whose scheduler, on
 * preemption, moves a victim's KV blocks out of the pool and back (Sec. 5.1.2,
 * "Swapping").  This library implements those two data-parallel operations.
 *
 * General conventions
 *  - Every data pointer is a DEVICE pointer owned by the caller unless the
 *    parameter name ends in `_host`.  The library allocates no device memory
 *    and never synchronises: all work is enqueued on `hip_stream` (a
 *    hipStream_t passed as void*; NULL = default stream).
 *  - State the library keeps, all of it per process: for each HIP device id
 *    below 16, whether the kernels that need more than 64 KiB of LDS have been
 *    given that attribute, the device's compute-unit count, and the device
 *    address of the static scratch array of paged_decode_attention_static; per
 *    thread, the last HIP runtime error.  It is set up by pkv_init(), or by the
 *    first call that needs it on a device.  That set-up makes HIP runtime calls
 *    that may not run inside a stream capture: call pkv_init() (or any one
 *    eager call of the entry point) on a device before capturing there.
 *    pkv_attn_workspace_bytes and pkv_prefill_workspace_bytes depend on the
 *    CURRENT device's compute-unit count: size a workspace with the device
 *    current on which the call will run.
 *  - Inputs are only read; `out`, `workspace` and `dst` are overwritten.
 *  - Every base pointer must be 16-byte aligned and every stride must keep
 *    16-byte alignment of a token row (PKV_ERR_ALIGN otherwise).
 *  - Anything checkable on the host is checked before any kernel is enqueued;
 *    on a non-zero status nothing was enqueued.  Values that live in device
 *    memory (block ids, context lengths, mapping entries) are NOT checked on
 *    the fast path; out-of-range values there are undefined behaviour.  The
 *    pkv_validate_* calls copy them to the host (synchronising) and check them.
 */
#ifndef PKV_H
#define PKV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum pkv_status {
  PKV_OK = 0,
  PKV_ERR_NULL = 1,      /* a required pointer is NULL                          */
  PKV_ERR_SHAPE = 2,     /* a size is non-positive, inconsistent or unsupported */
  PKV_ERR_DTYPE = 3,     /* unknown / unsupported element type                  */
  PKV_ERR_ALIGN = 4,     /* pointer or stride breaks the 16-byte rule           */
  PKV_ERR_WORKSPACE = 5, /* workspace smaller than pkv_attn_workspace_bytes()   */
  PKV_ERR_INDEX = 6,     /* (validators only) an index is out of range          */
  PKV_ERR_HIP = 7        /* the HIP runtime reported an error on launch         */
} pkv_status;

/* PKV_F8_E4M3: the 8-bit float E4M3 of the OCP 8-bit floating point specification (1 sign,
 * 4 exponent bits with bias 7, 3 mantissa bits, subnormals, no infinities, NaN =
 * S.1111.111, largest finite value 448).  Allowed for the K/V pools only. */
typedef enum pkv_dtype { PKV_F32 = 0, PKV_BF16 = 1, PKV_F8_E4M3 = 2 } pkv_dtype;

/* Use the vector-ALU kernel even where the matrix-core kernel applies (a
 * second, independent code path: tests run both against the oracle). */
#define PKV_ATTN_FLAG_VECTOR_ALU 1

/*
 * Geometry of one paged_decode_attention call (one layer, one decode step).
 *
 * Notation: B sequences, Hq query heads, Hkv KV heads, G = Hq/Hkv (query heads
 * g*G .. g*G+G-1 share KV head g), D head dim, bs tokens per block, n_i the
 * context length of sequence i INCLUDING the token being decoded (its K/V are
 * already in the pool; this call never writes KV).
 *
 * Pool layout: element (block b, kv head g, token slot s, dim d) of K lives at
 *   k_pool[b*k_stride_block + g*k_stride_head + s*k_stride_token + d]
 * (strides in ELEMENTS, d is unit stride); likewise V.  The recommended layout
 * is head-major [num_pool_blocks][Hkv][bs][D] (a 4 KiB contiguous tile per
 * (block, head) for bf16, D = 128, bs = 16).
 */
typedef struct pkv_attn_desc {
  int32_t batch;              /* B  >= 0 (0 enqueues nothing)                    */
  int32_t num_q_heads;        /* Hq, a multiple of num_kv_heads                  */
  int32_t num_kv_heads;       /* Hkv                                             */
  int32_t head_dim;           /* D; row bytes D*sizeof(elem) must be 128/256/512 */
  int32_t block_size;         /* bs, a multiple of 16                            */
  int32_t num_pool_blocks;    /* blocks in k_pool / v_pool (validators only)     */
  int32_t max_blocks_per_seq; /* row stride (entries) of block_tables            */
  int32_t max_context_len;    /* host-known upper bound of all n_i; sizes grid   */
  int32_t partition_tokens;   /* most tokens per split-K partial, multiple of 64;
                                 0 = chosen by the library                       */
  int32_t kv_dtype;           /* pkv_dtype of k_pool and v_pool; q has the same
                                 type, except that q is PKV_BF16 beside
                                 PKV_F8_E4M3 pools (a quantised KV cache: half
                                 the bytes per cached token that Sec. 4.2's time
                                 model charges)                                  */
  int32_t out_dtype;          /* pkv_dtype of out: PKV_F32 or PKV_BF16           */
  int32_t flags;              /* 0, or PKV_ATTN_FLAG_* bits                      */
  int64_t k_stride_block, k_stride_head, k_stride_token;
  int64_t v_stride_block, v_stride_head, v_stride_token;
  /* PKV_F8_E4M3 pools only (ignored otherwise): K = k_scale * stored value,
   * V = v_scale * stored value; finite and positive, 0 is read as 1. */
  float k_scale, v_scale;
} pkv_attn_desc;

/*
 * Geometry of one kv_block_swap call.  The pool is seen as `num_planes` planes
 * (layers x {K,V}); plane p of the source starts at src + p*src_plane_stride
 * bytes and holds src_num_blocks chunks of block_bytes bytes each, back to
 * back; the same for dst.
 */
typedef struct pkv_swap_desc {
  int32_t num_planes;             /* >= 1                                        */
  int32_t src_num_blocks;         /* chunks per source plane                     */
  int32_t dst_num_blocks;         /* chunks per destination plane                */
  int32_t reserved;               /* must be 0                                   */
  int64_t block_bytes;            /* bytes per (plane, block) chunk; mult. of 16 */
  int64_t src_plane_stride_bytes; /* >= src_num_blocks*block_bytes, mult. of 16  */
  int64_t dst_plane_stride_bytes; /* >= dst_num_blocks*block_bytes, mult. of 16  */
} pkv_swap_desc;

/* Library version as major*10000 + minor*100 + patch. */
int32_t pkv_version(void);

/*
 * Once-per-device set-up for the CURRENT HIP device, done here instead of
 * inside the first call of each entry point: the LDS attribute of the
 * attention kernels, the compute-unit count, the address of the static
 * scratch array.  Idempotent and thread-safe; PKV_OK or PKV_ERR_HIP.  Callers
 * that capture the calls into a HIP graph run it before the capture.
 */
int32_t pkv_init(void);

/* Static, NUL-terminated name of a status code ("PKV_OK", ...). */
const char* pkv_status_string(int32_t status);

/*
 * Text of the HIP runtime error behind the most recent PKV_ERR_HIP returned to
 * the calling thread ("no error" if there was none).  Diagnostics only.
 */
const char* pkv_last_hip_error_string(void);

/*
 * Split-K partition length in tokens the library will use for `desc`
 * (desc->partition_tokens, or the default when that is 0).  Returns 0 if
 * desc is NULL or the value is unsupported.
 */
int32_t pkv_attn_partition_tokens(const pkv_attn_desc* desc);

/*
 * Bytes of device scratch paged_decode_attention needs for `desc`: fp32
 * partial results (running max, normaliser, un-normalised output row) per
 * (sequence, query head, partition) of the flash-decoding split of the context
 * named by the paper's kernel profile ("splitkv", Sec. 4.2 / App. "System
 * Profile").  Returns 0 when no workspace is needed (every context fits one
 * partition) and also when desc is invalid (the attention call reports why).
 */
size_t pkv_attn_workspace_bytes(const pkv_attn_desc* desc);

/*
 * Decode attention over a paged KV pool (Sec. 2.2 "KV-Cache": fixed-size
 * non-contiguous blocks; Sec. 4.2: every step streams the whole KV history).
 * For each sequence i and query head h (KV head g = h / G), with
 * K_t, V_t the rows of logical token t = 0..n_i-1 found at block
 * block_tables[i*max_blocks_per_seq + t/bs], slot t%bs:
 *     s_t = scale * <q[i,h,:], K_t>,   w = softmax_t(s),
 *     out[i,h,:] = sum_t w_t * V_t.
 * n_i = 0 gives a zero row.  Slots >= n_i of the last block, blocks not named
 * by the first ceil(n_i/bs) table entries, and table entries beyond those are
 * never read.
 *
 *  q            [B][Hq][D]   kv_dtype, contiguous
 *  k_pool/v_pool             kv_dtype, layout per desc strides
 *  block_tables [B][max_blocks_per_seq] int32 physical block ids
 *  context_lens [B] int32, 0 <= n_i <= max_context_len
 *  scale        softmax scale (callers normally pass 1/sqrt(D))
 *  out          [B][Hq][D]   out_dtype, contiguous
 *  workspace    >= pkv_attn_workspace_bytes(desc) bytes, 16-byte aligned; may
 *               be NULL when that size is 0.  Contents on return are
 *               unspecified; one buffer may serve calls with different
 *               descriptors, but not two calls at the same time.
 * Accumulation is fp32.  The result does not depend on where blocks sit in
 * the pool; for a fixed partition length it is bit-reproducible run to run.
 * With PKV_F8_E4M3 pools (head_dim 128 or 256; strides then count bytes) the
 * stored codes are decoded exactly (every E4M3 value is a bfloat16 value) and
 * the arithmetic is that of the bfloat16 call on k_scale * K, v_scale * V.
 */
int32_t paged_decode_attention(const pkv_attn_desc* desc, const void* q,
                               const void* k_pool, const void* v_pool,
                               const int32_t* block_tables,
                               const int32_t* context_lens, float scale,
                               void* out, void* workspace,
                               size_t workspace_bytes, void* hip_stream);

/*
 * paged_decode_attention for callers that cannot allocate device memory: code
 * under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  The same operation, arguments, kernels and results (bit for
 * bit), but the scratch for the split-K partials is not brought by the caller:
 * it is a device array inside the library's code object, of
 * pkv_static_scratch_bytes() = 16 MiB, which every GPU the library runs on
 * holds until the process ends.  Returns PKV_ERR_WORKSPACE, enqueueing
 * nothing, when pkv_attn_workspace_bytes(desc) exceeds that (the five
 * benchmark shapes need 6-10 MiB with partition_tokens = 0; a caller-set
 * partition_tokens on a very long batch can need more).  The call allocates
 * nothing and frees nothing.  All calls on one GPU share the array: calls that
 * overlap in time on one GPU (different streams or threads) race, and the
 * array keeps the previous call's contents (the kernels write everything they
 * later read, nothing needs clearing).  The first call on a device resolves
 * the array's device address (pkv_init does the same ahead of time).
 */
size_t pkv_static_scratch_bytes(void);
int32_t paged_decode_attention_static(const pkv_attn_desc* desc, const void* q,
                                      const void* k_pool, const void* v_pool,
                                      const int32_t* block_tables,
                                      const int32_t* context_lens, float scale,
                                      void* out, void* hip_stream);

/*
 * A per-step plan for paged_decode_attention (Sec. 4.2: a decode step makes
 * one attention call per layer, and all of them walk the same block tables
 * with the same context lengths; only q and the layer's pools differ).  What
 * every one of those calls would work out again from block_tables and
 * context_lens -- the tile counts per sequence, the cut of the work into
 * per-wavefront ranges, the pool offset of every 16-token tile, where each
 * sequence's split-K partials go -- is written once into `plan` (device memory)
 * by pkv_attn_plan, and paged_decode_attention_planned reads it instead.  The
 * cut of the work is the same as without a plan, so are the partials and
 * their order; the result is bit-reproducible from call to call, bit-identical
 * to paged_decode_attention's with 8-bit pools, and equal to it up to fp32
 * rounding with bf16 pools (where the unplanned call has a kernel of its own).
 *
 *  pkv_attn_plan_bytes(desc)  size of the plan buffer; 0 when the call for
 *      `desc` has no use for a plan (not bf16 / 8-bit pools with head_dim 128,
 *      PKV_ATTN_FLAG_VECTOR_ALU, batch 0, invalid desc): pkv_attn_plan then
 *      enqueues nothing and the planned call is the ordinary call.
 *  pkv_attn_plan  enqueues one kernel on hip_stream that reads block_tables and
 *      context_lens (device) and writes `plan` (>= pkv_attn_plan_bytes bytes,
 *      16-byte aligned, else PKV_ERR_WORKSPACE / PKV_ERR_ALIGN).  Context
 *      lengths beyond desc->max_context_len leave the plan marked invalid.
 *  paged_decode_attention_planned  arguments as paged_decode_attention (same
 *      workspace size), plus the plan, which it only reads.  desc,
 *      block_tables and context_lens must be those the plan was made with (and
 *      the device the same); k_scale, v_scale, out_dtype, q, the pools, scale
 *      and out may differ from call to call.  A plan made for another geometry,
 *      or an invalid one, is detected on the device: out is then filled with
 *      NaN.  Changed table or length contents are not detected.
 */
size_t pkv_attn_plan_bytes(const pkv_attn_desc* desc);
int32_t pkv_attn_plan(const pkv_attn_desc* desc, const int32_t* block_tables,
                      const int32_t* context_lens, void* plan, size_t plan_bytes,
                      void* hip_stream);
int32_t paged_decode_attention_planned(const pkv_attn_desc* desc, const void* plan, size_t plan_bytes,
                                       const void* q, const void* k_pool, const void* v_pool,
                                       const int32_t* block_tables, const int32_t* context_lens,
                                       float scale, void* out, void* workspace,
                                       size_t workspace_bytes, void* hip_stream);

/*
 * kv_append and paged_decode_attention_planned in one call (Sec. 2.2: every
 * step appends the new token's K/V to the cache, then attends over it).  The
 * result, in `out` and in the pools, is that of kv_append(desc, k_new, v_new,
 * ...) followed by paged_decode_attention_planned(...) on the same stream.
 * Where the call has use for a plan (pkv_attn_plan_bytes > 0: bf16 or 8-bit
 * pools, head_dim 128) no second kernel is launched: the wavefront that streams
 * the last tile of a (sequence, KV head) takes the new rows from k_new / v_new,
 * puts them into its on-chip copy of the tile and writes them to the pools.  In
 * every other case the call launches the append ahead of the attention itself.  Arguments as for the two calls; k_new / v_new must not be NULL.
 */
int32_t paged_decode_attention_planned_append(const pkv_attn_desc* desc, const void* plan,
                                              size_t plan_bytes, const void* q,
                                              const void* k_new, const void* v_new,
                                              void* k_pool, void* v_pool,
                                              const int32_t* block_tables,
                                              const int32_t* context_lens, float scale,
                                              void* out, void* workspace,
                                              size_t workspace_bytes, void* hip_stream);

/*
 * Causal prefill attention of a chunk over the paged cache (Sec. 2.1: masked
 * self-attention, a token attends to itself and to what precedes it; this is
 * the prefill phase and, after a preemption, the re-prefill of Sec. 5.1.2
 * "Recomputation").  Sequence i contributes its LAST query_lens[i] tokens as
 * queries; context_lens[i] counts all its cached tokens including those, whose
 * K/V are already in the pool.  q and out are packed [total_query_tokens][Hq][D]
 * in sequence order, cu_query_lens [batch+1] holds the first packed row of every
 * sequence (device, int32).  Query token j of sequence i has position
 * context_lens[i] - query_lens[i] + j and sees positions 0..that:
 *   out[row,h,:] = softmax_{s <= pos}(scale * q[row,h,:] . K_s) V_s.
 * desc as for paged_decode_attention (partition_tokens and flags are not
 * used; max_context_len bounds every context_lens[i] and sizes an on-chip copy
 * of a block table row: at most 16 Ki blocks per sequence); max_query_len is a
 * host-known upper bound of all query_lens (it sizes the grid).  Supported: bf16 K/V/q, head_dim 128,
 * block_size a power-of-two multiple of 16 (PKV_ERR_SHAPE / PKV_ERR_DTYPE
 * otherwise); out is fp32 or bf16 per desc->out_dtype.  No workspace (8-bit
 * pools need one: paged_prefill_attention_ws below, PKV_ERR_WORKSPACE here).  Rows of
 * sequences with query_lens[i] = 0 do not exist; query_lens[i] > context_lens[i]
 * is clipped.  batch = 0 or max_query_len = 0 enqueues nothing.
 */
int32_t paged_prefill_attention(const pkv_attn_desc* desc, const void* q, const void* k_pool,
                                const void* v_pool, const int32_t* block_tables,
                                const int32_t* context_lens, const int32_t* query_lens,
                                const int32_t* cu_query_lens, int32_t max_query_len,
                                float scale, void* out, void* hip_stream);

/*
 * The same operation for the case that chunked prefill makes the common one
 * ("Effects of Chunked Prefill": a budget of e.g. 512 tokens per iteration): a
 * few chunks over long contexts.  One workgroup per (128 query tokens, head
 * pair) would then leave most of the GPU idle while each walks a whole context,
 * so the walks are cut into ranges that run side by side and leave fp32
 * partial results (reference maximum, normaliser, un-normalised output row per
 * query row, head and range) in `workspace`; a second kernel merges them as the
 * decode call merges its partitions.
 *
 * pkv_prefill_workspace_bytes: device bytes the call needs for `desc`,
 * total_query_tokens (the number of rows of q, host-known) and max_query_len;
 * 0 when the walks will not be split (enough workgroups anyway, short
 * contexts, unsupported or invalid desc).  The split depends on desc->batch,
 * the head counts, max_query_len, desc->max_context_len and the device's CU
 * count only.
 * paged_prefill_attention_ws: as paged_prefill_attention; workspace >= that many
 * bytes, 16-byte aligned (PKV_ERR_WORKSPACE / PKV_ERR_ALIGN otherwise); NULL
 * workspace, or total_query_tokens = 0, runs the walks unsplit.
 * total_query_tokens must not be smaller than cu_query_lens[batch].  Contents
 * of the workspace on return are unspecified; one buffer must not serve two
 * calls at the same time.  Results agree with the unsplit call to rounding.
 *
 * 8-bit pools (desc->kv_dtype = PKV_F8_E4M3 beside a bf16 q; K = k_scale times
 * the stored value, V = v_scale times, as in paged_decode_attention): the call
 * first decodes the blocks of the call's sequences into a bf16 copy at the head
 * of the workspace (exactly; block j of sequence i becomes block
 * i * ceil(max_context_len / block_size) + j of the copy) and walks the copy;
 * the scales act on the softmax scale and on the output.  The workspace is
 * then required, also for an unsplit walk, and pkv_prefill_workspace_bytes
 * counts the copy: 2 * batch * ceil(max_context_len / block_size) blocks of
 * num_kv_heads * block_size * head_dim bf16 values, their table, then what
 * the split needs.
 */
size_t pkv_prefill_workspace_bytes(const pkv_attn_desc* desc, int64_t total_query_tokens,
                                   int32_t max_query_len);
int32_t paged_prefill_attention_ws(const pkv_attn_desc* desc, const void* q, const void* k_pool,
                                   const void* v_pool, const int32_t* block_tables,
                                   const int32_t* context_lens, const int32_t* query_lens,
                                   const int32_t* cu_query_lens, int32_t max_query_len,
                                   int64_t total_query_tokens, float scale, void* out,
                                   void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * KV append (Sec. 2.2 "KV-Cache": the K and V vectors of the token generated
 * in a step join the request's cache before the step's attention reads it).
 * desc is the descriptor of the attention call that follows; context_lens
 * already counts the new token.  For every sequence i with
 * n_i = context_lens[i] >= 1 and every KV head g, the rows k_new[i][g][:] and
 * v_new[i][g][:] (device, [batch][num_kv_heads][head_dim] contiguous, dtype
 * desc->kv_dtype) are copied bit-exactly to token position n_i - 1 of the
 * pools: block block_tables[i][(n_i-1)/block_size], slot (n_i-1)%block_size,
 * at the strides of desc.  Sequences with n_i = 0 are skipped; nothing else
 * in the pools is touched.  Two sequences whose last token maps to the same
 * (block, slot) race (undefined).  Table entries are trusted as in the
 * attention call (pkv_validate_tables checks them).  Enqueued on hip_stream
 * ahead of the attention call that reads the pools; batch = 0 enqueues
 * nothing.  Errors as for paged_decode_attention (no workspace is used).
 */
int32_t kv_append(const pkv_attn_desc* desc, const void* k_new, const void* v_new,
                  void* k_pool, void* v_pool, const int32_t* block_tables,
                  const int32_t* context_lens, void* hip_stream);

/*
 * The same for the tokens of a prefill chunk (Sec. 2.1: the prefill computes the
 * K/V of all prompt tokens; Sec. 2.2: they are kept in the paged cache; with
 * chunked prefill a chunk at a time).  k_new / v_new are packed
 * [total_query_tokens][num_kv_heads][head_dim] in sequence order, as q is for
 * paged_prefill_attention, with the same query_lens / cu_query_lens: row j of
 * sequence i's query_lens[i] rows is copied bit-exactly to token position
 * context_lens[i] - query_lens[i] + j (the chunk is the tail of the context;
 * query_lens[i] above context_lens[i] is clipped and the surplus rows are
 * skipped, as are rows at or beyond cu_query_lens[batch]).  total_query_tokens
 * is a host-known upper bound of the number of rows (it sizes the grid).
 * Enqueued ahead of the paged_prefill_attention call that reads the pools.
 * Trust and errors as for kv_append.
 */
int32_t kv_append_chunk(const pkv_attn_desc* desc, const void* k_new, const void* v_new,
                        void* k_pool, void* v_pool, const int32_t* block_tables,
                        const int32_t* context_lens, const int32_t* query_lens,
                        const int32_t* cu_query_lens, int64_t total_query_tokens,
                        void* hip_stream);

/*
 * Block gather/scatter of the preemption swap path (Sec. 5.1.2 "Swapping":
 * the victim's KV blocks leave the pool and are later migrated back, in
 * general to different physical blocks).  For every plane p and every pair
 * j < n_pairs with (s, d) = (block_mapping[2j], block_mapping[2j+1]):
 *   copy block_bytes bytes from src_pool + p*src_plane_stride_bytes + s*block_bytes
 *                            to dst      + p*dst_plane_stride_bytes + d*block_bytes.
 * Gather (pool -> contiguous staging) and scatter (staging -> fresh blocks)
 * are this same call with the roles of pool and staging exchanged.  The copy
 * is bytewise exact.  src and dst must not overlap; a destination block named
 * twice is a data race (undefined); a source block may repeat.  n_pairs = 0
 * enqueues nothing.  The order of the pairs does not change the result; pairs
 * listed by ascending destination block copy fastest (sequential writes).
 * src_pool or dst may also be page-locked host memory that the device can
 * address (a swap area in CPU memory whose slots the caller's block manager
 * hands out): the kernel then moves those bytes over the link, which bounds
 * it; kv_swap_out_host / kv_swap_in_host below are that case with the host
 * slots in swap order and a smaller grid.
 */
int32_t kv_block_swap(const pkv_swap_desc* desc, const void* src_pool,
                      void* dst, const int32_t* block_mapping,
                      int32_t n_pairs, void* hip_stream);

/*
 * Host leg of the swap path (Sec. 5.1.2 "Swapping": a victim's KV blocks are
 * offloaded from GPU memory to CPU host memory, and recovery migrates them
 * back over PCIe).
 *
 * kv_swap_out_host: for every plane p and pair j < n_pairs, pool block
 * s_j = block_mapping[2j] goes to host slot j:
 *   host_dst + p*desc->dst_plane_stride_bytes + j*block_bytes
 * (the victims' blocks are stored back to back in swap order: the host slot of
 * pair j is j by definition; block_mapping[2j+1], where callers normally write
 * j, is NOT read, so no value there can send a block outside the host buffer;
 * desc->src_* describe the pool, desc->dst_* the host buffer,
 * dst_num_blocks >= n_pairs).
 * kv_swap_in_host: the reverse: host slot j of host_src goes to pool block
 * block_mapping[2j+1]; block_mapping[2j] is not read (desc->src_* describe the
 * host buffer, desc->dst_* the pool).
 *
 * host_dst / host_src is page-locked HOST memory, everything else is device
 * memory.  The swap moves in pieces through `staging`, a device buffer of
 * staging_bytes >= num_planes*block_bytes (PKV_ERR_WORKSPACE otherwise; bigger
 * pieces make longer PCIe transfers): the kv_block_swap kernel gathers a piece
 * into it, the piece crosses PCIe as one copy, and the next piece follows, all
 * on hip_stream (for swap-in the copy comes first and the kernel scatters).
 * A piece is a group of whole planes, one contiguous copy, when
 * 2*n_pairs*block_bytes fits into `staging` and n_pairs*block_bytes equals the
 * host plane stride; else a range of pairs of every plane, one strided copy.
 * With staging = NULL and staging_bytes = 0 nothing is staged: the copy kernel
 * itself reads or writes the host buffer, which the device sees because it is
 * page-locked (one launch of a few workgroups, bounded by the link like the
 * staged form and measured as fast; an address the device cannot see gives
 * PKV_ERR_HIP and nothing runs).
 * Both calls only enqueue work and keep no state.  After kv_swap_out_host,
 * completion of hip_stream implies that all of host_dst is written; after
 * kv_swap_in_host, that the pool blocks are.  The bytes arrive exactly; same
 * mapping rules as kv_block_swap.
 */
int32_t kv_swap_out_host(const pkv_swap_desc* desc, const void* src_pool, void* host_dst,
                         const int32_t* block_mapping, int32_t n_pairs, void* staging,
                         size_t staging_bytes, void* hip_stream);
int32_t kv_swap_in_host(const pkv_swap_desc* desc, const void* host_src, void* dst_pool,
                        const int32_t* block_mapping, int32_t n_pairs, void* staging,
                        size_t staging_bytes, void* hip_stream);

/*
 * Host-side range checks of the index arrays the fast path trusts.
 * *_host variants take HOST pointers and touch no GPU; the others take device
 * pointers, copy them to the host on `hip_stream` and wait for that copy.
 * Return PKV_ERR_INDEX for: n_i < 0 or > max_context_len or needing more than
 * max_blocks_per_seq blocks; a used table entry outside [0, num_pool_blocks);
 * a mapping entry outside its plane; a destination block named twice.
 */
/*
 * The same for the chunk arrays of paged_prefill_attention[_ws] and
 * kv_append_chunk, which those calls trust: PKV_ERR_INDEX unless
 * cu_query_lens[0] = 0, cu_query_lens[i+1] - cu_query_lens[i] = query_lens[i],
 * 0 <= query_lens[i] <= max_query_len, 0 <= context_lens[i] <= max_context_len
 * and cu_query_lens[batch] <= total_query_tokens (the rows the caller's q, out,
 * k_new, v_new buffers hold).
 */
int32_t pkv_validate_chunks_host(const pkv_attn_desc* desc, const int32_t* context_lens_host,
                                 const int32_t* query_lens_host,
                                 const int32_t* cu_query_lens_host, int32_t max_query_len,
                                 int64_t total_query_tokens);
int32_t pkv_validate_chunks(const pkv_attn_desc* desc, const int32_t* context_lens,
                            const int32_t* query_lens, const int32_t* cu_query_lens,
                            int32_t max_query_len, int64_t total_query_tokens,
                            void* hip_stream);
int32_t pkv_validate_tables_host(const pkv_attn_desc* desc,
                                 const int32_t* block_tables_host,
                                 const int32_t* context_lens_host);
int32_t pkv_validate_mapping_host(const pkv_swap_desc* desc,
                                  const int32_t* block_mapping_host,
                                  int32_t n_pairs);
int32_t pkv_validate_tables(const pkv_attn_desc* desc,
                            const int32_t* block_tables,
                            const int32_t* context_lens, void* hip_stream);
int32_t pkv_validate_mapping(const pkv_swap_desc* desc,
                             const int32_t* block_mapping, int32_t n_pairs,
                             void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* PKV_H */
