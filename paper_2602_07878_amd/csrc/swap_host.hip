// Host leg of the swap path (arXiv 2602.07878, Sec. 5.1.2 "Swapping": a victim's KV blocks
// are offloaded from GPU memory to CPU host memory and migrated back over PCIe on recovery).
//
// The swap moves in pieces through a device staging buffer: the gather kernel fills the buffer
// with a piece, the piece crosses PCIe as one copy, and the next piece follows on the same
// stream (the other way round for swap-in).  Nothing is overlapped on purpose: the kernel moves
// a piece at some 6 TB/s and the link at 57 GB/s, so hiding the kernel behind the copy on a
// second stream gains 1 % at best (56.3 against 55.5 GB/s measured), while the cross-stream
// event waits it needs halved the rate (30 GB/s) whenever the process had freed device memory
// since its last long kernel.  One stream also needs no events, so the calls keep no state.
//
// A piece is a group of whole planes when two or more planes' slots (n_pairs blocks each) fit
// into the staging buffer: the planes lie back to back on the host side too, so the piece
// crosses as one plain contiguous copy.  Otherwise a piece is a range of pairs of every plane,
// one strided copy (hipMemcpy2DAsync, one row per plane).

#include "pkv_internal.h"

namespace pkv {
namespace {

#define PKV_TRY(x) do { const hipError_t e_ = (x); if (e_ != hipSuccess) return e_; } while (0)

struct Pieces {
  int64_t pairs_per_piece;
  int32_t planes_per_piece;   // > 0: pieces are groups of whole planes (all pairs each)
};

// a piece fills the staging buffer with `pairs_per_piece` chunks of every plane back to back,
// or with whole planes
bool plan_pieces(const pkv_swap_desc& d, int32_t n_pairs, size_t staging_bytes, int64_t host_plane_stride,
                 Pieces* pc) {
  const int64_t per_pair = (int64_t)d.num_planes * d.block_bytes;
  const int64_t plane_bytes = (int64_t)n_pairs * d.block_bytes;
  pc->planes_per_piece = 0;
  if (2 * plane_bytes <= (int64_t)staging_bytes && d.num_planes >= 2 && host_plane_stride == plane_bytes) {
    int64_t pp = (int64_t)staging_bytes / plane_bytes;
    if (pp > d.num_planes) pp = d.num_planes;
    pc->planes_per_piece = (int32_t)pp;
    pc->pairs_per_piece = n_pairs;
    return true;
  }
  int64_t cp = (int64_t)staging_bytes / per_pair;
  if (cp < 1) return false;
  if (cp > n_pairs) cp = n_pairs;
  pc->pairs_per_piece = cp;
  return true;
}

}  // namespace

hipError_t swap_out_host(const pkv_swap_desc& d, const uint8_t* pool, uint8_t* host_dst, const int32_t* mapping,
                         int32_t n_pairs, uint8_t* staging, size_t staging_bytes, hipStream_t stream,
                         bool* too_small) {
  Pieces pc;
  if (!plan_pieces(d, n_pairs, staging_bytes, d.dst_plane_stride_bytes, &pc)) { *too_small = true; return hipSuccess; }
  SwapParams p;
  p.src_plane_stride = d.src_plane_stride_bytes;
  p.block_bytes = d.block_bytes;
  p.dst = staging;
  // the host slot of pair j is j (the mapping's second column is not read); in the staging
  // buffer, which holds one piece, that is the pair's index within the piece
  p.src_slot_is_pair = 0;
  p.dst_slot_is_pair = 1;
  if (pc.planes_per_piece > 0) {
    const int64_t pp = pc.planes_per_piece, plane_bytes = (int64_t)n_pairs * d.block_bytes;
    for (int64_t first = 0; first < d.num_planes; first += pp) {
      const int32_t npl = (int32_t)(first + pp <= d.num_planes ? pp : d.num_planes - first);
      p.src = pool + first * d.src_plane_stride_bytes;
      p.mapping = mapping;
      p.dst_plane_stride = plane_bytes;
      p.num_planes = npl;
      p.n_pairs = n_pairs;
      PKV_TRY(launch_swap(p, stream));
      PKV_TRY(hipMemcpyAsync(host_dst + first * plane_bytes, staging, (size_t)npl * plane_bytes, hipMemcpyDeviceToHost,
                             stream));
    }
    return hipSuccess;
  }
  const int64_t cp = pc.pairs_per_piece;
  for (int64_t first = 0; first < n_pairs; first += cp) {
    const int32_t np = (int32_t)(first + cp <= n_pairs ? cp : n_pairs - first);
    p.src = pool;
    p.mapping = mapping + 2 * first;
    p.dst_plane_stride = cp * d.block_bytes;
    p.num_planes = d.num_planes;
    p.n_pairs = np;
    PKV_TRY(launch_swap(p, stream));
    PKV_TRY(hipMemcpy2DAsync(host_dst + first * d.block_bytes, (size_t)d.dst_plane_stride_bytes, staging,
                             (size_t)(cp * d.block_bytes), (size_t)np * d.block_bytes, (size_t)d.num_planes,
                             hipMemcpyDeviceToHost, stream));
  }
  return hipSuccess;
}

hipError_t swap_in_host(const pkv_swap_desc& d, const uint8_t* host_src, uint8_t* pool, const int32_t* mapping,
                        int32_t n_pairs, uint8_t* staging, size_t staging_bytes, hipStream_t stream,
                        bool* too_small) {
  Pieces pc;
  if (!plan_pieces(d, n_pairs, staging_bytes, d.src_plane_stride_bytes, &pc)) { *too_small = true; return hipSuccess; }
  SwapParams p;
  p.dst_plane_stride = d.dst_plane_stride_bytes;
  p.block_bytes = d.block_bytes;
  p.src = staging;
  p.src_slot_is_pair = 1;   // host slot of pair j is j: the mapping's first column is not read
  p.dst_slot_is_pair = 0;
  if (pc.planes_per_piece > 0) {
    const int64_t pp = pc.planes_per_piece, plane_bytes = (int64_t)n_pairs * d.block_bytes;
    for (int64_t first = 0; first < d.num_planes; first += pp) {
      const int32_t npl = (int32_t)(first + pp <= d.num_planes ? pp : d.num_planes - first);
      PKV_TRY(hipMemcpyAsync(staging, host_src + first * plane_bytes, (size_t)npl * plane_bytes, hipMemcpyHostToDevice,
                             stream));
      p.dst = pool + first * d.dst_plane_stride_bytes;
      p.mapping = mapping;
      p.src_plane_stride = plane_bytes;
      p.num_planes = npl;
      p.n_pairs = n_pairs;
      PKV_TRY(launch_swap(p, stream));
    }
    return hipSuccess;
  }
  const int64_t cp = pc.pairs_per_piece;
  for (int64_t first = 0; first < n_pairs; first += cp) {
    const int32_t np = (int32_t)(first + cp <= n_pairs ? cp : n_pairs - first);
    PKV_TRY(hipMemcpy2DAsync(staging, (size_t)(cp * d.block_bytes), host_src + first * d.block_bytes,
                             (size_t)d.src_plane_stride_bytes, (size_t)np * d.block_bytes, (size_t)d.num_planes,
                             hipMemcpyHostToDevice, stream));
    p.dst = pool;
    p.mapping = mapping + 2 * first;
    p.src_plane_stride = cp * d.block_bytes;
    p.num_planes = d.num_planes;
    p.n_pairs = np;
    PKV_TRY(launch_swap(p, stream));
  }
  return hipSuccess;
}

// Without a staging buffer.  Page-locked host memory is mapped into the device's address space,
// so the copy kernel can take the host buffer as its source or destination: one launch, every
// chunk crosses the link once, nothing is staged.  The link (some 57 GB/s) bounds it, not the
// CUs, so the grid is a few workgroups: the rest of the device stays free for the requests that
// keep decoding while a victim is swapped.  Kernel completion makes the host writes visible to
// the host like any other result of a kernel.
constexpr int kDirectWorkgroups = 32;

hipError_t swap_host_direct(bool out, const pkv_swap_desc& d, const uint8_t* src, uint8_t* dst,
                            const int32_t* mapping, int32_t n_pairs, hipStream_t stream) {
  // the device's view of the host buffer (an error if the memory is not page-locked and mapped)
  void* view = nullptr;
  void* host = out ? static_cast<void*>(dst) : const_cast<uint8_t*>(src);
  PKV_TRY(hipHostGetDevicePointer(&view, host, 0));
  if (!view) return hipErrorInvalidValue;
  SwapParams p;
  p.src = out ? src : static_cast<const uint8_t*>(view);
  p.dst = out ? static_cast<uint8_t*>(view) : dst;
  p.mapping = mapping;
  p.block_bytes = d.block_bytes;
  p.src_plane_stride = d.src_plane_stride_bytes;
  p.dst_plane_stride = d.dst_plane_stride_bytes;
  p.num_planes = d.num_planes;
  p.n_pairs = n_pairs;
  p.src_slot_is_pair = out ? 0 : 1;   // the host slot of pair j is j
  p.dst_slot_is_pair = out ? 1 : 0;
  return launch_swap(p, stream, kDirectWorkgroups);
}

}  // namespace pkv
