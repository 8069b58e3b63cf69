// Host-sanitizer leg of the scheduler model: replays a request stream from a text file through
// the C ABI of csrc/sched.cpp (built together with this file under -fsanitize=address,undefined
// by tests/test_sanitizers.py) and prints one canonical line per iteration, which the test
// compares with the same line made from the Python reference.  Getter buffers are sized exactly.
//
// Input: "gpu cpu bs seqs budget maxblk watermark mode chunked steps", then per iteration
// "k id prompt max_new ..." (k arrivals).
#include <cinttypes>
#include <cstdio>
#include <vector>

#include "pkv_sched.h"

int main(int argc, char** argv) {
  if (argc != 2) return 2;
  FILE* f = std::fopen(argv[1], "r");
  if (!f) return 2;
  pkv_sched_config c;
  int steps = 0;
  if (std::fscanf(f, "%d %d %d %d %d %d %d %d %d %d", &c.num_gpu_blocks, &c.num_cpu_blocks, &c.block_size,
                  &c.max_num_seqs, &c.max_num_batched_tokens, &c.max_blocks_per_seq, &c.watermark_blocks,
                  &c.preemption_mode, &c.chunked_prefill, &steps) != 10)
    return 2;
  pkv_sched* s = pkv_sched_create(&c);
  if (!s) return 3;
  for (int it = 0; it < steps; ++it) {
    int k = 0;
    if (std::fscanf(f, "%d", &k) != 1) return 2;
    for (int a = 0; a < k; ++a) {
      long long id;
      int p, n;
      if (std::fscanf(f, "%lld %d %d", &id, &p, &n) != 3) return 2;
      std::printf("A%d ", pkv_sched_add_request(s, id, p, n));
    }
    pkv_sched_step_info info;
    if (pkv_sched_step(s, &info) != 0) return 4;
    std::vector<int64_t> ids((size_t)info.num_decode);
    std::vector<int32_t> lens((size_t)info.num_decode), tabs((size_t)info.num_decode * c.max_blocks_per_seq);
    pkv_sched_decode_batch(s, ids.data(), lens.data(), tabs.data(), info.num_decode);
    std::printf("D");
    for (int i = 0; i < info.num_decode; ++i) {
      std::printf(" %" PRId64 ":%d:", ids[i], lens[i]);
      for (int b = 0; b < c.max_blocks_per_seq && tabs[(size_t)i * c.max_blocks_per_seq + b] >= 0; ++b)
        std::printf("%s%d", b ? "," : "", tabs[(size_t)i * c.max_blocks_per_seq + b]);
    }
    std::vector<int32_t> so((size_t)info.num_swap_out_blocks * 2), si((size_t)info.num_swap_in_blocks * 2);
    pkv_sched_swap_out(s, so.data(), info.num_swap_out_blocks);
    pkv_sched_swap_in(s, si.data(), info.num_swap_in_blocks);
    std::printf(" O");
    for (size_t i = 0; i + 1 < so.size(); i += 2) std::printf(" %d>%d", so[i], so[i + 1]);
    std::printf(" I");
    for (size_t i = 0; i + 1 < si.size(); i += 2) std::printf(" %d>%d", si[i], si[i + 1]);
    std::vector<int64_t> pid((size_t)info.num_prefill), fin((size_t)info.num_finished);
    std::vector<int32_t> ptok((size_t)info.num_prefill), pctx((size_t)info.num_prefill);
    pkv_sched_prefills(s, pid.data(), ptok.data(), info.num_prefill);
    pkv_sched_prefill_contexts(s, pctx.data(), info.num_prefill);
    pkv_sched_finished(s, fin.data(), info.num_finished);
    std::printf(" P");
    for (int i = 0; i < info.num_prefill; ++i) std::printf(" %" PRId64 ":%d:%d", pid[i], ptok[i], pctx[i]);
    std::printf(" F");
    for (int i = 0; i < info.num_finished; ++i) std::printf(" %" PRId64, fin[i]);
    std::printf(" S %d %d %d %d %d %d\n", info.free_blocks, info.running, info.waiting, info.swapped,
                info.head_blocked, info.num_preempted);
  }
  int64_t t[8];
  pkv_sched_totals(s, t);
  std::printf("T");
  for (int i = 0; i < 8; ++i) std::printf(" %" PRId64, t[i]);
  std::printf("\n");
  pkv_sched_destroy(s);
  std::fclose(f);
  return 0;
}
