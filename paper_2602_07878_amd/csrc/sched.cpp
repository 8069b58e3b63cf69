// Host-side scheduler / block-manager model (arXiv 2602.07878, Sec. 5.1): FIFO free-block
// queue, first-come-first-served admission with head-of-line blocking, last-in-first-out
// preemption with swap or recompute recovery, optionally chunked prefill (the paper's section
// "Effects of Chunked Prefill").  It produces, iteration by iteration, the
// block tables, context lengths and swap mappings that the GPU calls of this library take.
// Plain C++ on the host; see pkv_sched.h for the iteration it implements.

#include <algorithm>
#include <cstdint>
#include <deque>
#include <memory>
#include <unordered_map>
#include <utility>
#include <vector>

#include "pkv.h"
#include "pkv_sched.h"

namespace {

struct Request {
  int64_t id;
  int32_t prompt, max_new;
  int32_t generated = 0;   // output tokens produced so far
  int32_t computed = 0;    // tokens whose K/V sit in pool blocks
  bool swapped = false;
  // chunked prefill: part of the tokens to prefill is still to come
  bool prefilling = false;
  int32_t target = 0;      // ... tokens to have cached before decoding starts
  int32_t chunk = 0;       // ... tokens of the chunk of the current iteration
  std::vector<int32_t> blocks;      // pool blocks in logical order
  std::vector<int32_t> cpu_blocks;  // host blocks while swapped out
};

}  // namespace

struct pkv_sched {
  pkv_sched_config cfg;
  std::deque<int32_t> free_gpu, free_cpu;   // taken from the front, returned to the back
  std::deque<Request*> waiting;
  std::vector<Request*> running;            // in scheduling order; back() is the next victim
  std::unordered_map<int64_t, std::unique_ptr<Request>> requests;
  int64_t totals[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  // results of the last iteration
  std::vector<int64_t> dec_ids, prefill_ids, finished_ids;
  std::vector<int32_t> dec_lens, dec_tables, prefill_tokens, prefill_contexts, swap_out, swap_in;
  int32_t preempted_now = 0;

  int32_t take_block() {
    const int32_t b = free_gpu.front();
    free_gpu.pop_front();
    return b;
  }

  void preempt(Request* r) {
    ++totals[1];
    ++preempted_now;
    if (cfg.preemption_mode == PKV_PREEMPT_SWAP && free_cpu.size() >= r->blocks.size()) {
      for (int32_t b : r->blocks) {
        const int32_t c = free_cpu.front();
        free_cpu.pop_front();
        swap_out.push_back(b);
        swap_out.push_back(c);
        r->cpu_blocks.push_back(c);
        free_gpu.push_back(b);
      }
      totals[2] += (int64_t)r->blocks.size();
      r->swapped = true;
    } else {   // recomputation: the cache is dropped
      for (int32_t b : r->blocks) free_gpu.push_back(b);
      r->computed = 0;
      r->prefilling = false;   // it starts over when it is admitted again
    }
    r->blocks.clear();
    waiting.push_front(r);
  }

  void finish(Request* r) {
    for (int32_t b : r->blocks) free_gpu.push_back(b);
    finished_ids.push_back(r->id);
    ++totals[5];
    requests.erase(r->id);   // r is gone after this
  }

  void step(pkv_sched_step_info* info) {
    dec_ids.clear(); dec_lens.clear(); dec_tables.clear();
    prefill_ids.clear(); prefill_tokens.clear(); prefill_contexts.clear(); finished_ids.clear();
    swap_out.clear(); swap_in.clear();
    preempted_now = 0;
    ++totals[0];
    const int32_t bs = cfg.block_size;
    const bool chunked = cfg.chunked_prefill != 0;

    // The token budget of the iteration.  Without chunked prefill it pays for the prefills of
    // the admissions only; with it, first for one decode token of every decoding request,
    // then for the prefill chunks of running requests and admissions.
    int32_t budget = cfg.max_num_batched_tokens;
    if (chunked)
      for (const Request* r : running) budget -= r->prefilling ? 0 : 1;

    // 1. in scheduling order, every running request reserves what it needs in this iteration:
    //    the slot of its next token, or (a request still prefilling) the blocks of its next
    //    chunk, which is as much of the rest as the budget still allows
    for (size_t i = 0; i < running.size();) {
      Request* r = running[i];
      size_t need;
      if (r->prefilling) {
        r->chunk = std::min(r->target - r->computed, budget);
        need = (size_t)((r->computed + r->chunk + bs - 1) / bs) - r->blocks.size();
      } else {
        need = r->computed % bs == 0 ? 1 : 0;
      }
      bool evicted_self = false;
      while (free_gpu.size() < need) {
        Request* victim = running.back();
        running.pop_back();
        preempt(victim);
        if (victim == r) { evicted_self = true; break; }
      }
      if (evicted_self) break;
      for (size_t k = 0; k < need; ++k) r->blocks.push_back(take_block());
      if (r->prefilling) budget -= r->chunk;
      ++i;
    }

    // 2. first-come-first-served admission, unless this iteration had to preempt
    std::vector<Request*> admitted;
    bool head_blocked = false;
    int32_t n_prefill_tokens = 0;
    std::vector<int64_t> adm_ids;                 // prefill records of the admissions
    std::vector<int32_t> adm_tokens;
    if (preempted_now == 0) {
      while (!waiting.empty() && (int32_t)(running.size() + admitted.size()) < cfg.max_num_seqs) {
        Request* r = waiting.front();
        if (r->swapped) {
          const size_t nb = r->cpu_blocks.size();
          if (free_gpu.size() < nb + (size_t)cfg.watermark_blocks) { head_blocked = true; break; }
          for (int32_t c : r->cpu_blocks) {
            const int32_t g = take_block();
            swap_in.push_back(c);
            swap_in.push_back(g);
            r->blocks.push_back(g);
            free_cpu.push_back(c);
          }
          totals[3] += (int64_t)nb;
          r->cpu_blocks.clear();
          r->swapped = false;
          r->chunk = 0;
          waiting.pop_front();
          admitted.push_back(r);
          continue;
        }
        const int32_t total = r->generated == 0 ? r->prompt : r->prompt + r->generated - 1;
        // all of it or nothing without chunked prefill; else what the budget allows
        const int32_t tokens = chunked ? std::min(total, budget) : total;
        const size_t nb = (size_t)((tokens + bs - 1) / bs);
        // An unchunked prefill is atomic: it is neither split nor dropped.  A recomputation that
        // has outgrown the whole budget (prompt + generated - 1 tokens) therefore runs as the
        // only prefill of an iteration; everything else has to fit what the budget has left.
        const bool alone = !chunked && r->generated > 0 && tokens > cfg.max_num_batched_tokens &&
                           budget == cfg.max_num_batched_tokens;
        if ((tokens > budget && !alone) || tokens == 0 || free_gpu.size() < nb + (size_t)cfg.watermark_blocks) {
          head_blocked = true;
          break;
        }
        for (size_t k = 0; k < nb; ++k) r->blocks.push_back(take_block());
        r->target = total;
        r->computed = tokens;
        r->chunk = 0;
        r->prefilling = tokens < total;
        budget = alone ? 0 : budget - tokens;
        n_prefill_tokens += tokens;
        if (r->generated > 0) totals[4] += tokens;
        else if (!r->prefilling) r->generated = 1;   // the (last chunk of the) prefill yields the first token
        adm_ids.push_back(r->id);
        adm_tokens.push_back(tokens);
        waiting.pop_front();
        if (!r->prefilling && r->generated >= r->max_new) finish(r);
        else admitted.push_back(r);
      }
    }
    if (head_blocked) ++totals[6];
    // the order of the pairs is free; ascending pool blocks make the scatter's writes sequential
    {
      std::vector<std::pair<int32_t, int32_t>> pairs;   // (pool block, host block)
      for (size_t k = 0; k + 1 < swap_in.size(); k += 2) pairs.emplace_back(swap_in[k + 1], swap_in[k]);
      std::sort(pairs.begin(), pairs.end());
      for (size_t k = 0; k < pairs.size(); ++k) {
        swap_in[2 * k] = pairs[k].second;
        swap_in[2 * k + 1] = pairs[k].first;
      }
    }

    // 3. one decode token for everything that was running before the admissions
    std::vector<Request*> still;
    still.reserve(running.size() + admitted.size());
    const int32_t mb = cfg.max_blocks_per_seq;
    for (Request* r : running) {
      if (r->prefilling) {           // its chunk of this iteration, if the budget gave it one
        if (r->chunk > 0) {
          r->computed += r->chunk;
          n_prefill_tokens += r->chunk;
          if (r->generated > 0) totals[4] += r->chunk;
          prefill_ids.push_back(r->id);
          prefill_tokens.push_back(r->chunk);
          prefill_contexts.push_back(r->computed);
          if (r->computed == r->target) {
            r->prefilling = false;
            if (r->generated == 0) r->generated = 1;
          }
        }
        if (!r->prefilling && r->generated >= r->max_new) finish(r);
        else still.push_back(r);
        continue;
      }
      r->computed += 1;
      dec_ids.push_back(r->id);
      dec_lens.push_back(r->computed);
      const size_t row = dec_tables.size();
      dec_tables.resize(row + (size_t)mb, -1);
      for (size_t k = 0; k < r->blocks.size(); ++k) dec_tables[row + k] = r->blocks[k];
      r->generated += 1;
      ++totals[7];
      if (r->generated >= r->max_new) finish(r);
      else still.push_back(r);
    }
    for (Request* r : admitted) still.push_back(r);
    running.swap(still);
    // prefill records: the chunks of running requests first, then the admissions (whose
    // cached length is the chunk itself)
    for (size_t k = 0; k < adm_ids.size(); ++k) {
      prefill_ids.push_back(adm_ids[k]);
      prefill_tokens.push_back(adm_tokens[k]);
      prefill_contexts.push_back(adm_tokens[k]);
    }

    if (info) {
      info->num_decode = (int32_t)dec_ids.size();
      info->num_prefill = (int32_t)prefill_ids.size();
      info->num_prefill_tokens = n_prefill_tokens;
      info->num_preempted = preempted_now;
      info->num_swap_out_blocks = (int32_t)(swap_out.size() / 2);
      info->num_swap_in_blocks = (int32_t)(swap_in.size() / 2);
      info->num_finished = (int32_t)finished_ids.size();
      info->free_blocks = (int32_t)free_gpu.size();
      info->running = (int32_t)running.size();
      info->waiting = (int32_t)waiting.size();
      int32_t sw = 0;
      for (const Request* r : waiting) sw += r->swapped ? 1 : 0;
      info->swapped = sw;
      info->head_blocked = head_blocked ? 1 : 0;
    }
  }
};

namespace {

template <typename T>
int32_t copy_out(const std::vector<T>& v, T* dst, int32_t capacity, int32_t per_item = 1) {
  const int32_t n = (int32_t)(v.size() / (size_t)per_item);
  if (n > capacity) return -PKV_ERR_SHAPE;
  if (dst)
    for (size_t i = 0; i < v.size(); ++i) dst[i] = v[i];
  return n;
}

}  // namespace

extern "C" {

pkv_sched* pkv_sched_create(const pkv_sched_config* cfg) {
  if (!cfg || cfg->num_gpu_blocks < 1 || cfg->num_cpu_blocks < 0 || cfg->block_size < 1 ||
      cfg->max_num_seqs < 1 || cfg->max_num_batched_tokens < 1 || cfg->max_blocks_per_seq < 1 ||
      cfg->watermark_blocks < 0 ||
      (cfg->preemption_mode != PKV_PREEMPT_SWAP && cfg->preemption_mode != PKV_PREEMPT_RECOMPUTE) ||
      (cfg->chunked_prefill != 0 && cfg->chunked_prefill != 1) ||
      (cfg->chunked_prefill == 1 && cfg->max_num_batched_tokens < cfg->max_num_seqs))
    return nullptr;
  pkv_sched* s = new pkv_sched;
  s->cfg = *cfg;
  for (int32_t b = 0; b < cfg->num_gpu_blocks; ++b) s->free_gpu.push_back(b);
  for (int32_t b = 0; b < cfg->num_cpu_blocks; ++b) s->free_cpu.push_back(b);
  return s;
}

void pkv_sched_destroy(pkv_sched* s) { delete s; }

int32_t pkv_sched_add_request(pkv_sched* s, int64_t request_id, int32_t prompt_len,
                              int32_t max_new_tokens) {
  if (!s) return PKV_ERR_NULL;
  if (prompt_len < 1 || max_new_tokens < 1 ||
      (prompt_len > s->cfg.max_num_batched_tokens && !s->cfg.chunked_prefill))
    return PKV_ERR_SHAPE;
  const int64_t full = ((int64_t)prompt_len + max_new_tokens - 1 + s->cfg.block_size - 1) / s->cfg.block_size;
  // a victim evicted at full length must be able to return: its blocks plus the watermark
  if (full > s->cfg.max_blocks_per_seq || full + s->cfg.watermark_blocks > s->cfg.num_gpu_blocks)
    return PKV_ERR_SHAPE;
  if (s->requests.count(request_id)) return PKV_ERR_INDEX;
  auto r = std::make_unique<Request>();
  r->id = request_id;
  r->prompt = prompt_len;
  r->max_new = max_new_tokens;
  s->waiting.push_back(r.get());
  s->requests.emplace(request_id, std::move(r));
  return PKV_OK;
}

int32_t pkv_sched_step(pkv_sched* s, pkv_sched_step_info* info) {
  if (!s) return PKV_ERR_NULL;
  s->step(info);
  return PKV_OK;
}

int32_t pkv_sched_decode_batch(const pkv_sched* s, int64_t* request_ids, int32_t* context_lens,
                               int32_t* block_tables, int32_t capacity_rows) {
  if (!s) return -PKV_ERR_NULL;
  const int32_t n = copy_out(s->dec_ids, request_ids, capacity_rows);
  if (n < 0) return n;
  copy_out(s->dec_lens, context_lens, capacity_rows);
  copy_out(s->dec_tables, block_tables, capacity_rows, s->cfg.max_blocks_per_seq);
  return n;
}

int32_t pkv_sched_swap_out(const pkv_sched* s, int32_t* mapping, int32_t capacity_pairs) {
  return s ? copy_out(s->swap_out, mapping, capacity_pairs, 2) : -PKV_ERR_NULL;
}

int32_t pkv_sched_swap_in(const pkv_sched* s, int32_t* mapping, int32_t capacity_pairs) {
  return s ? copy_out(s->swap_in, mapping, capacity_pairs, 2) : -PKV_ERR_NULL;
}

int32_t pkv_sched_prefills(const pkv_sched* s, int64_t* request_ids, int32_t* tokens, int32_t capacity) {
  if (!s) return -PKV_ERR_NULL;
  const int32_t n = copy_out(s->prefill_ids, request_ids, capacity);
  if (n < 0) return n;
  copy_out(s->prefill_tokens, tokens, capacity);
  return n;
}

int32_t pkv_sched_prefill_contexts(const pkv_sched* s, int32_t* context_lens, int32_t capacity) {
  return s ? copy_out(s->prefill_contexts, context_lens, capacity) : -PKV_ERR_NULL;
}

int32_t pkv_sched_finished(const pkv_sched* s, int64_t* request_ids, int32_t capacity) {
  return s ? copy_out(s->finished_ids, request_ids, capacity) : -PKV_ERR_NULL;
}

int32_t pkv_sched_request_blocks(const pkv_sched* s, int64_t request_id, int32_t* blocks,
                                 int32_t capacity) {
  if (!s) return -PKV_ERR_NULL;
  const auto it = s->requests.find(request_id);
  if (it == s->requests.end()) return -PKV_ERR_INDEX;
  return copy_out(it->second->blocks, blocks, capacity);
}

int32_t pkv_sched_totals(const pkv_sched* s, int64_t totals[8]) {
  if (!s || !totals) return PKV_ERR_NULL;
  for (int i = 0; i < 8; ++i) totals[i] = s->totals[i];
  return PKV_OK;
}

}  // extern "C"
