/*
 * pkv_bench.h -- measurement scaffolding of libpkv: not part of the product
 * interface.  The benchmark uses these calls to time the K/V-streaming kernel
 * by itself and to measure the machine's plain streaming ceilings.
 */
#ifndef PKV_BENCH_H
#define PKV_BENCH_H

#include "pkv.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * paged_decode_attention with two optional hipEvent_t handles (passed as void*, either
 * may be NULL) that are attached to the launch of the kernel that streams K and
 * V (Sec. 4.2: the part of the step whose time grows with the KV volume) and
 * receive that kernel's own begin and end on hip_stream, i.e. excluding the
 * small kernel that merges the split-K partials.  For profiling: the elapsed
 * time between the two events is that kernel's duration.  The events are the
 * caller's and must have been created with timing enabled; nothing waits on
 * them.
 */
int32_t paged_decode_attention_timed(const pkv_attn_desc* desc, const void* q,
                                     const void* k_pool, const void* v_pool,
                                     const int32_t* block_tables,
                                     const int32_t* context_lens, float scale,
                                     void* out, void* workspace,
                                     size_t workspace_bytes, void* hip_stream,
                                     void* ev_kernel_begin, void* ev_kernel_end);

/* The same for paged_decode_attention_planned. */
int32_t paged_decode_attention_planned_timed(const pkv_attn_desc* desc, const void* plan, size_t plan_bytes,
                                             const void* q, const void* k_pool, const void* v_pool,
                                             const int32_t* block_tables, const int32_t* context_lens,
                                             float scale, void* out, void* workspace,
                                             size_t workspace_bytes, void* hip_stream,
                                             void* ev_kernel_begin, void* ev_kernel_end);

/*
 * Bandwidth probes used by the benchmark to measure this machine's streaming
 * ceilings with the same access idiom as the product kernels (16 bytes per
 * lane): pkv_probe_copy copies `bytes` (multiple of 16) from src to dst;
 * pkv_probe_read reads `bytes` from src and writes one 16-byte checksum per
 * workgroup to `sink` (>= 64 KiB).
 */
int32_t pkv_probe_copy(const void* src, void* dst, size_t bytes, void* hip_stream);
int32_t pkv_probe_read(const void* src, void* sink, size_t bytes, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* PKV_BENCH_H */
