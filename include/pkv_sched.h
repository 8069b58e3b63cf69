/*
 * pkv_sched.h -- C ABI of the host-side scheduler / block-manager model that
 * produces the inputs of the GPU calls of pkv.h over time.
 *
 * What it models (arXiv 2602.07878, Sec. 5.1 "Revisiting vLLM Scheduler"):
 *   - a pool of fixed-size physical KV blocks handed out from a FIFO
 *     free-block queue; running requests grow by one token per engine
 *     iteration and keep their blocks until they finish (Sec. 5.1.1
 *     "KV-Cache Saturation");
 *   - strict first-come-first-served admission from the WAITING queue: the
 *     request at the head must fit (can-allocate check); if it does not,
 *     admission stops for this iteration even if later, smaller requests
 *     would fit ("memory-based head-of-line blocking", Sec. 5.1.1);
 *   - preemption when the running requests outgrow the pool: the most
 *     recently scheduled request is evicted (last in, first out) and put at
 *     the FRONT of the waiting queue; recovery is either by swapping (its
 *     blocks go to host blocks and come back later, in general to other
 *     physical blocks) or by recomputation (its cache is dropped and the
 *     prompt plus everything generated so far is prefilled again)
 *     (Sec. 5.1.2 "Preemption and Recovery Penalties").
 * The attack controller of the paper is NOT part of this library.
 *
 * Time is counted in engine iterations.  One call of pkv_sched_step():
 *   1. every running request, in scheduling order, reserves the slot of its
 *      next token (a new block when its cached tokens fill its blocks
 *      exactly); while the free queue cannot serve it, the LAST running
 *      request is preempted (possibly the request itself);
 *   2. if nothing was preempted in this iteration, waiting requests are
 *      admitted from the head of the queue while they fit: a swapped request
 *      needs as many blocks as it holds on the host (swap-in), any other one
 *      ceil(tokens/block_size) blocks for the tokens it has to prefill
 *      (prompt, plus generated-1 after a recomputation), within the token
 *      budget and the limit on running requests, and leaving
 *      watermark_blocks free; the first one that does not fit ends admission.
 *      Without chunked prefill a prefill is atomic (the paper's section
 *      "Effects of Chunked Prefill"): a recomputation that has outgrown the
 *      budget of a whole iteration is neither split nor dropped, it is
 *      admitted as the only prefill of an iteration (else it would block the
 *      head of the queue for ever);
 *   3. every request that was running before step 2 decodes one token: its
 *      cached length grows by one (that is the context length of the
 *      attention call, which counts the token being decoded) and it finishes
 *      when it has generated max_new_tokens; finished requests return their
 *      blocks to the back of the free queue.  Requests admitted in step 2
 *      join the running list behind them (so they are the next victims) and
 *      decode from the next iteration on; a prefill yields the first token.
 *
 * With chunked_prefill = 1 (the paper's section "Effects of Chunked Prefill":
 * a fixed budget of tokens per iteration, prefill chunks interleaved with the
 * decoding steps of the other requests, the KV-cache use rising chunk by
 * chunk) the token budget of an iteration pays first for one decode token of
 * every running request that decodes, then for prefill chunks:
 *   1'. a running request that is still prefilling reserves, in its turn, the
 *       blocks of its next chunk = min(tokens left to prefill, budget left)
 *       (possibly 0 tokens), with the same last-in-first-out preemption when
 *       the free queue cannot serve it;
 *   2'. an admission takes min(tokens to prefill, budget left) tokens as its
 *       first chunk and the blocks of that chunk only; a chunk of 0 tokens
 *       ends admission like a request that does not fit;
 *   3'. a request that is prefilling does not decode; the chunk that completes
 *       its prefill yields the first token, and it decodes from the next
 *       iteration on.
 * A partial prefill is preempted like any running request: swapped out it
 * keeps its progress, recomputed it starts over.  Prompts may then exceed the
 * budget; max_num_batched_tokens must be >= max_num_seqs.
 *
 * All memory here is host memory.  The handle owns its state; the arrays the
 * getters fill are the caller's.  Functions that report a status return a
 * pkv_status code of pkv.h; getters return a count, or minus such a code.
 * A handle must not be used from two threads at once.
 */
#ifndef PKV_SCHED_H_
#define PKV_SCHED_H_

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct pkv_sched pkv_sched; /* opaque */

enum { PKV_PREEMPT_SWAP = 0, PKV_PREEMPT_RECOMPUTE = 1 };

typedef struct pkv_sched_config {
  int32_t num_gpu_blocks;         /* physical KV blocks of the pool, >= 1           */
  int32_t num_cpu_blocks;         /* host blocks for swapped-out requests, >= 0     */
  int32_t block_size;             /* tokens per block, >= 1                         */
  int32_t max_num_seqs;           /* most requests running at once, >= 1            */
  int32_t max_num_batched_tokens; /* prefill tokens admitted per iteration, >= 1    */
  int32_t max_blocks_per_seq;     /* row length of the block tables handed out      */
  int32_t watermark_blocks;       /* blocks an admission must leave free, >= 0      */
  int32_t preemption_mode;        /* PKV_PREEMPT_SWAP or PKV_PREEMPT_RECOMPUTE; a
                                     swap that finds no host space falls back to
                                     recomputation                                 */
  int32_t chunked_prefill;        /* 0: a prefill is one piece within the budget;
                                     1: prefills proceed in chunks (see above)     */
} pkv_sched_config;

/* What one iteration did (counts) and the state it left. */
typedef struct pkv_sched_step_info {
  int32_t num_decode;          /* rows of the decode batch                         */
  int32_t num_prefill;         /* prefill records: requests prefilled (new or
                                  recomputed), or chunks with chunked prefill      */
  int32_t num_prefill_tokens;
  int32_t num_preempted;       /* evictions in this iteration                      */
  int32_t num_swap_out_blocks; /* pairs in the swap-out mapping                    */
  int32_t num_swap_in_blocks;  /* pairs in the swap-in mapping                     */
  int32_t num_finished;
  int32_t free_blocks, running, waiting, swapped; /* after the iteration; swapped
                                                     requests also count as waiting */
  int32_t head_blocked;        /* 1 if the head of the waiting queue did not fit   */
} pkv_sched_step_info;

/* NULL if cfg is NULL or invalid. */
pkv_sched* pkv_sched_create(const pkv_sched_config* cfg);
void pkv_sched_destroy(pkv_sched* s);

/*
 * Append a request to the back of the waiting queue.  PKV_ERR_SHAPE if
 * prompt_len < 1, max_new_tokens < 1, the prompt exceeds the token budget
 * (without chunked prefill), or the request at full length
 * (prompt_len + max_new_tokens - 1 tokens) would not fit max_blocks_per_seq,
 * or its blocks plus watermark_blocks would not fit the pool (evicted at that
 * length it could never be admitted again and would block the queue for
 * ever); PKV_ERR_INDEX if request_id is already known.
 */
int32_t pkv_sched_add_request(pkv_sched* s, int64_t request_id, int32_t prompt_len,
                              int32_t max_new_tokens);

/* Run one iteration; *info (may be NULL) receives the counts. */
int32_t pkv_sched_step(pkv_sched* s, pkv_sched_step_info* info);

/*
 * Decode batch of the last iteration, in running order: request ids,
 * context_lens (cached tokens including the one being decoded) and block
 * tables [capacity_rows][max_blocks_per_seq] (unused entries -1): exactly the
 * block_tables / context_lens arguments of paged_decode_attention and
 * kv_append.  Any pointer may be NULL.  Returns the number of rows, or
 * -PKV_ERR_SHAPE if capacity_rows is too small.
 */
int32_t pkv_sched_decode_batch(const pkv_sched* s, int64_t* request_ids, int32_t* context_lens,
                               int32_t* block_tables, int32_t capacity_rows);

/*
 * Swap mappings of the last iteration as [n][2] int32 pairs, the
 * block_mapping argument of kv_block_swap: swap-out pairs are (pool block,
 * host block) in eviction order, swap-in pairs (host block, pool block) by
 * ascending pool block (sequential writes for the scatter).  Returns n, or
 * -PKV_ERR_SHAPE if capacity_pairs is too small.
 */
int32_t pkv_sched_swap_out(const pkv_sched* s, int32_t* mapping, int32_t capacity_pairs);
int32_t pkv_sched_swap_in(const pkv_sched* s, int32_t* mapping, int32_t capacity_pairs);

/*
 * Prefills of the last iteration: ids and token counts (with chunked prefill:
 * one record per chunk, the chunks of requests already running first, in
 * running order, then the admissions).  Returns the count.
 * pkv_sched_prefill_contexts: for the same records, the tokens the request has
 * cached after this prefill (= tokens unless it is a later chunk): query_lens =
 * tokens and context_lens = these are the arguments of paged_prefill_attention,
 * the block table rows come from pkv_sched_request_blocks.
 */
int32_t pkv_sched_prefills(const pkv_sched* s, int64_t* request_ids, int32_t* tokens, int32_t capacity);
int32_t pkv_sched_prefill_contexts(const pkv_sched* s, int32_t* context_lens, int32_t capacity);
/* Requests that finished in the last iteration.  Returns the count. */
int32_t pkv_sched_finished(const pkv_sched* s, int64_t* request_ids, int32_t capacity);

/*
 * Pool blocks a live request holds right now, in logical order (what a prefill
 * writes its K/V into before the request's first decode).  Returns their
 * number (0 for a request that is waiting or swapped out), -PKV_ERR_INDEX for
 * an unknown or finished request, -PKV_ERR_SHAPE if capacity is too small.
 */
int32_t pkv_sched_request_blocks(const pkv_sched* s, int64_t request_id, int32_t* blocks,
                                 int32_t capacity);

/* Totals since creation: [0] iterations, [1] preemptions, [2] swapped-out blocks,
 * [3] swapped-in blocks, [4] recomputed tokens, [5] finished requests,
 * [6] iterations in which the head of the waiting queue was blocked,
 * [7] decoded tokens. */
int32_t pkv_sched_totals(const pkv_sched* s, int64_t totals[8]);

#ifdef __cplusplus
}
#endif
#endif /* PKV_SCHED_H_ */
