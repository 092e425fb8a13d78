// KV linking kernel of libmpic (gfx950).
//
// Fig. 7 step 2 / Sec. 4.1: rows of the recompute set are replaced by the fresh
// K/V, every other context row is taken from the stored cache of its image chunk
// (Sec. 3.1 item 5).  Stored keys are moved from chunk-local to global positions by
// a rotary shift of the chunk's offset; values are copied.  One launch covers a
// range of batch-flattened context positions: gather, rotation and scatter are fused
// and every destination row has exactly one source, so there is no ordering hazard.
//
// The kernel is bandwidth bound (3 flops per key element); the work of one thread is
// link::link_item (link_rows.h).
#include <algorithm>

#include "common.h"
#include "link_rows.h"

namespace mpic {
namespace {

template <typename T, bool kInterleaved>
__global__ __launch_bounds__(256) void assemble_kernel(AssembleArgs a, AssembleSrcTable tab) {
  const link::Shape sh = link::shape_of<T>(a);
  // one work item (a pair of 16-byte units of one context row) per thread; launches that
  // are held to a small grid (sources read over the bus, see launch_assemble) stride on
  const int64_t n_items = (a.pos_end - a.pos_begin) * sh.pairs_per_row;
  const int64_t stride = static_cast<int64_t>(gridDim.x) * blockDim.x;
  for (int64_t w = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x; w < n_items; w += stride)
    link::link_item<T, kInterleaved>(a, tab, sh, w);
}

}  // namespace
hipError_t launch_assemble(int dtype, const AssembleArgs& a, const AssembleSrcTable& t,
                           hipStream_t stream) {
  const int64_t n_pos = a.pos_end - a.pos_begin;
  if (n_pos <= 0) return hipSuccess;
  const int elems = dtype == MPIC_F32 ? 4 : 8;
  const int64_t pairs_per_row = static_cast<int64_t>(a.n_kv_heads) * (a.head_dim / 2 / elems);
  const int64_t threads = n_pos * pairs_per_row;
  const dim3 block(256);
  // Sources in mapped host memory: the launch lasts as long as the transfer over the bus.  A
  // grid of one item per thread would fill every wave slot of the chip for that long and keep
  // a concurrent kernel (the attention of the previous layer) from being scheduled; a few
  // waves per compute unit are plenty to keep the bus busy, so those launches stride.
  int64_t blocks = (threads + 255) / 256;
  if (a.grid_limit > 0) blocks = std::min<int64_t>(blocks, a.grid_limit);
  const dim3 grid(static_cast<unsigned>(blocks));
  if (dtype == MPIC_F32) {
    if (a.interleaved)
      hipLaunchKernelGGL((assemble_kernel<float, true>), grid, block, 0, stream, a, t);
    else
      hipLaunchKernelGGL((assemble_kernel<float, false>), grid, block, 0, stream, a, t);
  } else {
    if (a.interleaved)
      hipLaunchKernelGGL((assemble_kernel<__bf16, true>), grid, block, 0, stream, a, t);
    else
      hipLaunchKernelGGL((assemble_kernel<__bf16, false>), grid, block, 0, stream, a, t);
  }
  return hipGetLastError();
}

}  // namespace mpic
