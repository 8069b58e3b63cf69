// Host-sanitizer leg of the library's host-side checks: the validators and the descriptor checks
// of csrc/api.hip run here in a build whose host code is instrumented with
// -fsanitize=address,undefined (tests/test_sanitizers.py builds it with hipcc), on heap arrays of
// exactly the sizes the descriptors state.  No GPU is touched: every call either takes host
// arrays or is refused before a launch.  Prints one status per line; the test compares them with
// the statuses the regular library returns for the same arguments.
#include <cstdint>
#include <cstdio>
#include <cstring>
#include <vector>

#include "pkv.h"

static pkv_attn_desc desc(int B, int maxb, int nblk, int maxctx) {
  pkv_attn_desc d;
  std::memset(&d, 0, sizeof d);
  d.batch = B; d.num_q_heads = 32; d.num_kv_heads = 8; d.head_dim = 128; d.block_size = 16;
  d.num_pool_blocks = nblk; d.max_blocks_per_seq = maxb; d.max_context_len = maxctx;
  d.kv_dtype = PKV_BF16; d.out_dtype = PKV_F32;
  d.k_stride_block = d.v_stride_block = 8 * 16 * 128;
  d.k_stride_head = d.v_stride_head = 16 * 128;
  d.k_stride_token = d.v_stride_token = 128;
  return d;
}

int main() {
  // tables: rows used up to ceil(n/16) entries, the rest of a row poisoned
  {
    const int B = 5, maxb = 7, nblk = 40;
    pkv_attn_desc d = desc(B, maxb, nblk, maxb * 16);
    std::vector<int32_t> lens = {0, 1, 16, 17, 112};
    std::vector<int32_t> tab((size_t)B * maxb, -7);
    for (int i = 0; i < B; ++i)
      for (int b = 0; b < (lens[i] + 15) / 16; ++b) tab[(size_t)i * maxb + b] = (i * 7 + b) % nblk;
    std::printf("%d\n", pkv_validate_tables_host(&d, tab.data(), lens.data()));
    tab[4 * maxb + 6] = nblk;   // last used entry of the last row out of range
    std::printf("%d\n", pkv_validate_tables_host(&d, tab.data(), lens.data()));
    tab[4 * maxb + 6] = 3;
    lens[2] = maxb * 16 + 1;
    std::printf("%d\n", pkv_validate_tables_host(&d, tab.data(), lens.data()));
    lens[2] = -1;
    std::printf("%d\n", pkv_validate_tables_host(&d, tab.data(), lens.data()));
    std::printf("%zu\n", pkv_attn_workspace_bytes(&d) > 0 ? (size_t)1 : (size_t)0);
    d.head_dim = 96;
    std::printf("%d\n", pkv_validate_tables_host(&d, tab.data(), lens.data()));
  }
  // mappings
  {
    pkv_swap_desc s;
    std::memset(&s, 0, sizeof s);
    s.num_planes = 4; s.src_num_blocks = 10; s.dst_num_blocks = 6; s.block_bytes = 4096;
    s.src_plane_stride_bytes = 10 * 4096; s.dst_plane_stride_bytes = 6 * 4096;
    std::vector<int32_t> m = {9, 0, 0, 5, 3, 2, 3, 1};
    std::printf("%d\n", pkv_validate_mapping_host(&s, m.data(), 4));
    m[7] = 2;   // destination 2 twice
    std::printf("%d\n", pkv_validate_mapping_host(&s, m.data(), 4));
    m[7] = 6;   // past the destination plane
    std::printf("%d\n", pkv_validate_mapping_host(&s, m.data(), 4));
    m[7] = 1; m[0] = 10;
    std::printf("%d\n", pkv_validate_mapping_host(&s, m.data(), 4));
    std::printf("%d\n", pkv_validate_mapping_host(&s, m.data(), 0));
    s.block_bytes = 100;
    std::printf("%d\n", pkv_validate_mapping_host(&s, m.data(), 4));
  }
  // chunk arrays
  {
    const int B = 4;
    pkv_attn_desc d = desc(B, 64, 100, 1024);
    std::vector<int32_t> cl = {100, 5, 1024, 0}, ql = {30, 5, 512, 0}, cu = {0, 30, 35, 547, 547};
    std::printf("%d\n", pkv_validate_chunks_host(&d, cl.data(), ql.data(), cu.data(), 512, 547));
    std::printf("%d\n", pkv_validate_chunks_host(&d, cl.data(), ql.data(), cu.data(), 511, 547));
    std::printf("%d\n", pkv_validate_chunks_host(&d, cl.data(), ql.data(), cu.data(), 512, 546));
    cu[2] = 36;
    std::printf("%d\n", pkv_validate_chunks_host(&d, cl.data(), ql.data(), cu.data(), 512, 547));
  }
  // calls refused on the host before any launch (never dereferenced pointers)
  {
    pkv_attn_desc d = desc(2, 8, 16, 128);
    void* fake = reinterpret_cast<void*>(0x1000);
    const int32_t* fi = reinterpret_cast<const int32_t*>(0x2000);
    std::printf("%d\n", paged_decode_attention(&d, fake, fake, fake, fi, fi, 0.1f, fake, nullptr, 0, nullptr));
    std::printf("%d\n", paged_decode_attention(&d, nullptr, fake, fake, fi, fi, 0.1f, fake, fake, 1u << 30, nullptr));
    std::printf("%d\n", paged_decode_attention_static(&d, fake, fake, reinterpret_cast<void*>(0x1004), fi, fi, 0.1f, fake, nullptr));
    d.partition_tokens = 64; d.max_context_len = 1 << 20; d.max_blocks_per_seq = 1 << 16; d.batch = 64;
    std::printf("%d\n", paged_decode_attention_static(&d, fake, fake, fake, fi, fi, 0.1f, fake, nullptr));
    std::printf("%s\n", pkv_status_string(6));
  }
  return 0;
}
