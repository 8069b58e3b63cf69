// paged_decode_attention for callers that cannot allocate device memory (code under HIP graph
// capture, tight serving loops, harnesses that forbid hipMalloc): the split-K partials of the
// call live in a device array that is part of the library's code object instead of a
// caller-provided workspace.
//
// Every GPU the library runs on holds its own copy of the array, at its own address, until the
// process ends.  The array's name is only a host-side handle: the device address is asked for
// once per device (hipGetSymbolAddress, with that device current) and from then on only that
// address is handed to the kernels, exactly as the caller's workspace pointer is in
// paged_decode_attention.  Nothing in the array has to start at zero: the kernels write every
// directory entry and partial they later read.  All calls on one GPU share the array, so calls
// that overlap in time on one GPU (two streams, two threads) race.

#include <atomic>

#include "pkv_internal.h"

namespace {

constexpr size_t kScratchBytes = (size_t)16 << 20;   // 16 MiB per GPU

__attribute__((used)) static __device__ __align__(256) unsigned char scratch[kScratchBytes];

// device address of `scratch` on each device, asked for once
std::atomic<void*> g_scratch_ptr[pkv::kMaxDevices];

hipError_t scratch_on_current_device(void** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  const bool in_table = dev >= 0 && dev < pkv::kMaxDevices;
  void* ptr = in_table ? g_scratch_ptr[dev].load(std::memory_order_acquire) : nullptr;
  if (!ptr) {
    e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!ptr) return hipErrorInvalidSymbol;
    if (in_table) g_scratch_ptr[dev].store(ptr, std::memory_order_release);
  }
  *out = ptr;
  return hipSuccess;
}

}  // namespace

namespace pkv {
hipError_t prepare_static_scratch() {
  void* ptr = nullptr;
  return scratch_on_current_device(&ptr);
}
size_t static_scratch_bytes() { return kScratchBytes; }
hipError_t static_scratch_address(void** ptr) { return scratch_on_current_device(ptr); }
}  // namespace pkv

extern "C" {

size_t pkv_static_scratch_bytes(void) { return kScratchBytes; }

int32_t paged_decode_attention_static(const pkv_attn_desc* desc, const void* q, const void* k_pool,
                                      const void* v_pool, const int32_t* block_tables,
                                      const int32_t* context_lens, float scale, void* out,
                                      void* hip_stream) {
  return pkv::attention_call(desc, q, k_pool, v_pool, block_tables, context_lens, scale, out, nullptr, 0,
                             hip_stream, nullptr, nullptr, /*static_scratch=*/true, nullptr, 0, nullptr, nullptr);
}

}  // extern "C"
