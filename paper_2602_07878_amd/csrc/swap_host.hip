// Host leg of the swap path (arXiv 2602.07878, Sec. 5.1.2 "Swapping": a victim's KV blocks
// are offloaded from GPU memory to CPU host memory and migrated back over PCIe on recovery).
//
// The swap moves in pieces through a device staging buffer of two halves: while piece c
// crosses PCIe on the copy stream, the gather kernel already fills the other half with piece
// c+1 on the compute stream (and the other way round for swap-in).  Four events order the
// two streams; a fifth makes the copy stream start behind whatever the caller had already
// enqueued on the compute stream.
//
// A piece is a group of whole planes when two or more planes' slots (n_pairs blocks each) fit
// into half the staging buffer: the planes lie back to back on the host side too, so the
// piece crosses as one plain contiguous copy (56 GB/s both ways, the rate of a plain copy).  Otherwise a piece is a range of pairs of every plane, one
// strided copy (hipMemcpy2DAsync, one row per plane): device-to-host that form was measured
// at 42-47 GB/s where the plain copy reaches 55-57.

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
  int32_t planes_per_piece;   // > 0: pieces are groups of whole planes (all pairs each)
};

// two halves, each holding `pairs_per_piece` chunks of every plane back to back
bool plan_pieces(const pkv_swap_desc& d, int32_t n_pairs, size_t staging_bytes, int64_t host_plane_stride,
                 Pieces* pc) {
  const int64_t per_pair = (int64_t)d.num_planes * d.block_bytes;
  const int64_t plane_bytes = (int64_t)n_pairs * d.block_bytes;
  pc->planes_per_piece = 0;
  // (groups of at least two planes: with single planes of 57 MB device-to-host fell to 27-34 GB/s)
  if (2 * plane_bytes <= (int64_t)(staging_bytes / 2) && d.num_planes >= 2 && host_plane_stride == plane_bytes) {
    int64_t pp = (int64_t)(staging_bytes / 2) / plane_bytes;
    if (pp > d.num_planes) pp = d.num_planes;
    pc->planes_per_piece = (int32_t)pp;
    pc->pairs_per_piece = n_pairs;
    pc->half_bytes = pp * plane_bytes;
    return true;
  }
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
  if (!plan_pieces(d, n_pairs, staging_bytes, d.dst_plane_stride_bytes, &pc)) { *too_small = true; return hipSuccess; }
  DeviceEvents* ev = nullptr;
  PKV_TRY(events_for_current_device(&ev));
  if (pc.planes_per_piece > 0) {
    const int64_t pp = pc.planes_per_piece, plane_bytes = (int64_t)n_pairs * d.block_bytes;
    const int64_t pieces = (d.num_planes + pp - 1) / pp;
    for (int64_t c = 0; c < pieces; ++c) {
      const int h = (int)(c & 1);
      const int32_t npl = (int32_t)((c + 1) * pp <= d.num_planes ? pp : d.num_planes - c * pp);
      if (c >= 2) PKV_TRY(hipStreamWaitEvent(compute, ev->copy_done[h], 0));   // half h has left
      SwapParams p;
      p.src = pool + c * pp * d.src_plane_stride_bytes;
      p.dst = staging + h * pc.half_bytes;
      p.mapping = mapping;
      p.block_bytes = d.block_bytes;
      p.src_plane_stride = d.src_plane_stride_bytes;
      p.dst_plane_stride = plane_bytes;
      p.num_planes = npl;
      p.n_pairs = n_pairs;
      p.src_index_offset = 0;
      p.dst_index_offset = 0;
      PKV_TRY(launch_swap(p, compute));
      PKV_TRY(hipEventRecord(ev->kernel_done[h], compute));
      PKV_TRY(hipStreamWaitEvent(copy, ev->kernel_done[h], 0));
      PKV_TRY(hipMemcpyAsync(host_dst + c * pp * plane_bytes, staging + h * pc.half_bytes, (size_t)npl * plane_bytes,
                             hipMemcpyDeviceToHost, copy));
      PKV_TRY(hipEventRecord(ev->copy_done[h], copy));
    }
    PKV_TRY(hipStreamWaitEvent(compute, ev->copy_done[(pieces - 1) & 1], 0));
    if (pieces >= 2) PKV_TRY(hipStreamWaitEvent(compute, ev->copy_done[pieces & 1], 0));
    return hipSuccess;
  }
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
  if (!plan_pieces(d, n_pairs, staging_bytes, d.src_plane_stride_bytes, &pc)) { *too_small = true; return hipSuccess; }
  DeviceEvents* ev = nullptr;
  PKV_TRY(events_for_current_device(&ev));
  // staging may still be read by work the caller enqueued on the compute stream
  PKV_TRY(hipEventRecord(ev->start, compute));
  PKV_TRY(hipStreamWaitEvent(copy, ev->start, 0));
  if (pc.planes_per_piece > 0) {
    const int64_t pp = pc.planes_per_piece, plane_bytes = (int64_t)n_pairs * d.block_bytes;
    const int64_t pieces = (d.num_planes + pp - 1) / pp;
    for (int64_t c = 0; c < pieces; ++c) {
      const int h = (int)(c & 1);
      const int32_t npl = (int32_t)((c + 1) * pp <= d.num_planes ? pp : d.num_planes - c * pp);
      if (c >= 2) PKV_TRY(hipStreamWaitEvent(copy, ev->kernel_done[h], 0));   // half h was scattered
      PKV_TRY(hipMemcpyAsync(staging + h * pc.half_bytes, host_src + c * pp * plane_bytes, (size_t)npl * plane_bytes,
                             hipMemcpyHostToDevice, copy));
      PKV_TRY(hipEventRecord(ev->copy_done[h], copy));
      PKV_TRY(hipStreamWaitEvent(compute, ev->copy_done[h], 0));
      SwapParams p;
      p.src = staging + h * pc.half_bytes;
      p.dst = pool + c * pp * d.dst_plane_stride_bytes;
      p.mapping = mapping;
      p.block_bytes = d.block_bytes;
      p.src_plane_stride = plane_bytes;
      p.dst_plane_stride = d.dst_plane_stride_bytes;
      p.num_planes = npl;
      p.n_pairs = n_pairs;
      p.src_index_offset = 0;
      p.dst_index_offset = 0;
      PKV_TRY(launch_swap(p, compute));
      PKV_TRY(hipEventRecord(ev->kernel_done[h], compute));
    }
    return hipSuccess;
  }
  const int64_t cp = pc.pairs_per_piece;
  const int64_t pieces = (n_pairs + cp - 1) / cp;
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
