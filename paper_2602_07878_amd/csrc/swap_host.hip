// Host leg of the swap path (arXiv 2602.07878, Sec. 5.1.2 "Swapping": a victim's KV blocks
// are offloaded from GPU memory to CPU host memory and migrated back over PCIe on recovery).
//
// The swap moves in pieces through a device staging buffer of two halves: while piece c
// crosses PCIe as one strided copy (hipMemcpy2DAsync, one row per plane) on the copy stream,
// the gather kernel already fills the other half with piece c+1 on the compute stream (and
// the other way round for swap-in).  Four events order the two streams; a fifth makes the
// copy stream start behind whatever the caller had already enqueued on the compute stream.

#include <mutex>

#include "pkv_internal.h"

namespace pkv {
namespace {

struct DeviceEvents {
  hipEvent_t kernel_done[2], copy_done[2], start;
  bool ready = false;
};

// Events are created once per device and reused by every call (creating them costs far more
// than a piece of the swap).  Calls on one device must therefore not be issued concurrently
// from several host threads.
hipError_t events_for_current_device(DeviceEvents** out) {
  static DeviceEvents table[kMaxDevices];
  static std::mutex mu;
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(mu);
  DeviceEvents& ev = table[dev];
  if (!ev.ready) {
    hipEvent_t* all[5] = {&ev.kernel_done[0], &ev.kernel_done[1], &ev.copy_done[0], &ev.copy_done[1],
                          &ev.start};
    for (hipEvent_t* p : all) {
      e = hipEventCreateWithFlags(p, hipEventDisableTiming);
      if (e != hipSuccess) return e;
    }
    ev.ready = true;
  }
  *out = &ev;
  return hipSuccess;
}

#define PKV_TRY(x) do { const hipError_t e_ = (x); if (e_ != hipSuccess) return e_; } while (0)

struct Pieces {
  int64_t pairs_per_piece, half_bytes;
};

// two halves, each holding `pairs_per_piece` chunks of every plane back to back
bool plan_pieces(const pkv_swap_desc& d, int32_t n_pairs, size_t staging_bytes, Pieces* pc) {
  const int64_t per_pair = (int64_t)d.num_planes * d.block_bytes;
  int64_t cp = (int64_t)(staging_bytes / 2) / per_pair;
  if (cp < 1) return false;
  if (cp > n_pairs) cp = n_pairs;
  pc->pairs_per_piece = cp;
  pc->half_bytes = cp * per_pair;
  return true;
}

}  // namespace

hipError_t swap_out_host(const pkv_swap_desc& d, const uint8_t* pool, uint8_t* host_dst, const int32_t* mapping,
                         int32_t n_pairs, uint8_t* staging, size_t staging_bytes, hipStream_t compute,
                         hipStream_t copy, bool* too_small) {
  Pieces pc;
  if (!plan_pieces(d, n_pairs, staging_bytes, &pc)) { *too_small = true; return hipSuccess; }
  DeviceEvents* ev = nullptr;
  PKV_TRY(events_for_current_device(&ev));
  const int64_t cp = pc.pairs_per_piece;
  const int64_t pieces = (n_pairs + cp - 1) / cp;
  for (int64_t c = 0; c < pieces; ++c) {
    const int h = (int)(c & 1);
    const int32_t np = (int32_t)((c + 1) * cp <= n_pairs ? cp : n_pairs - c * cp);
    if (c >= 2) PKV_TRY(hipStreamWaitEvent(compute, ev->copy_done[h], 0));   // half h has left
    SwapParams p;
    p.src = pool;
    p.dst = staging + h * pc.half_bytes;
    p.mapping = mapping + 2 * c * cp;
    p.block_bytes = d.block_bytes;
    p.src_plane_stride = d.src_plane_stride_bytes;
    p.dst_plane_stride = cp * d.block_bytes;
    p.num_planes = d.num_planes;
    p.n_pairs = np;
    p.src_index_offset = 0;
    p.dst_index_offset = (int32_t)(c * cp);   // host slot j sits at j - c*cp of this piece
    PKV_TRY(launch_swap(p, compute));
    PKV_TRY(hipEventRecord(ev->kernel_done[h], compute));
    PKV_TRY(hipStreamWaitEvent(copy, ev->kernel_done[h], 0));
    PKV_TRY(hipMemcpy2DAsync(host_dst + c * cp * d.block_bytes, (size_t)d.dst_plane_stride_bytes,
                             staging + h * pc.half_bytes, (size_t)(cp * d.block_bytes),
                             (size_t)np * d.block_bytes, (size_t)d.num_planes, hipMemcpyDeviceToHost, copy));
    PKV_TRY(hipEventRecord(ev->copy_done[h], copy));
  }
  // the compute stream is complete only when the last copies are
  PKV_TRY(hipStreamWaitEvent(compute, ev->copy_done[(pieces - 1) & 1], 0));
  if (pieces >= 2) PKV_TRY(hipStreamWaitEvent(compute, ev->copy_done[pieces & 1], 0));
  return hipSuccess;
}

hipError_t swap_in_host(const pkv_swap_desc& d, const uint8_t* host_src, uint8_t* pool, const int32_t* mapping,
                        int32_t n_pairs, uint8_t* staging, size_t staging_bytes, hipStream_t compute,
                        hipStream_t copy, bool* too_small) {
  Pieces pc;
  if (!plan_pieces(d, n_pairs, staging_bytes, &pc)) { *too_small = true; return hipSuccess; }
  DeviceEvents* ev = nullptr;
  PKV_TRY(events_for_current_device(&ev));
  const int64_t cp = pc.pairs_per_piece;
  const int64_t pieces = (n_pairs + cp - 1) / cp;
  // staging may still be read by work the caller enqueued on the compute stream
  PKV_TRY(hipEventRecord(ev->start, compute));
  PKV_TRY(hipStreamWaitEvent(copy, ev->start, 0));
  for (int64_t c = 0; c < pieces; ++c) {
    const int h = (int)(c & 1);
    const int32_t np = (int32_t)((c + 1) * cp <= n_pairs ? cp : n_pairs - c * cp);
    if (c >= 2) PKV_TRY(hipStreamWaitEvent(copy, ev->kernel_done[h], 0));   // half h was scattered
    PKV_TRY(hipMemcpy2DAsync(staging + h * pc.half_bytes, (size_t)(cp * d.block_bytes),
                             host_src + c * cp * d.block_bytes, (size_t)d.src_plane_stride_bytes,
                             (size_t)np * d.block_bytes, (size_t)d.num_planes, hipMemcpyHostToDevice, copy));
    PKV_TRY(hipEventRecord(ev->copy_done[h], copy));
    PKV_TRY(hipStreamWaitEvent(compute, ev->copy_done[h], 0));
    SwapParams p;
    p.src = staging + h * pc.half_bytes;
    p.dst = pool;
    p.mapping = mapping + 2 * c * cp;
    p.block_bytes = d.block_bytes;
    p.src_plane_stride = cp * d.block_bytes;
    p.dst_plane_stride = d.dst_plane_stride_bytes;
    p.num_planes = d.num_planes;
    p.n_pairs = np;
    p.src_index_offset = (int32_t)(c * cp);
    p.dst_index_offset = 0;
    PKV_TRY(launch_swap(p, compute));
    PKV_TRY(hipEventRecord(ev->kernel_done[h], compute));
  }
  return hipSuccess;
}

}  // namespace pkv
