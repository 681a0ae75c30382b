// Value chunk gather: V_sparse = Gather(V_store, I) (decoding algorithm, "gather value
// cache" line).  The store may live in pinned host memory that the GPU reads over PCIe,
// so the kernel is a zero-copy reader: every chunk is c*d*(2 or 1) contiguous bytes, lanes take
// 16 bytes each, and each thread keeps four independent loads in flight before it
// stores, which is what keeps a high-latency link busy.  The same kernel serves an HBM
// store when staging is requested.
#include "kernels.hpp"

namespace skv {

constexpr int kGatherUnroll = 4;

__global__ __launch_bounds__(256) void gather_values_kernel(const uint4* __restrict__ store,
                                                            const int32_t* __restrict__ sel_ids,
                                                            uint4* __restrict__ v_sparse, int k, int vec_per_chunk,
                                                            size_t vec_per_unit_store, int last_chunk) {
  const int unit = blockIdx.y;
  const int32_t* ids = sel_ids + (size_t)unit * k;
  const uint4* src_u = store + (size_t)unit * vec_per_unit_store;
  uint4* dst_u = v_sparse + (size_t)unit * k * vec_per_chunk;
  const int total = k * vec_per_chunk;  // 16-byte vectors this unit moves
  const int stride = gridDim.x * 256;
  for (int v0 = blockIdx.x * 256 + threadIdx.x; v0 < total; v0 += stride * kGatherUnroll) {
    uint4 buf[kGatherUnroll];
#pragma unroll
    for (int u = 0; u < kGatherUnroll; ++u) {
      const int v = v0 + u * stride;
      if (v < total) {
        const int ch = v / vec_per_chunk, off = v - ch * vec_per_chunk;
        buf[u] = src_u[(size_t)min(max(ids[ch], 0), last_chunk) * vec_per_chunk + off];
      }
    }
#pragma unroll
    for (int u = 0; u < kGatherUnroll; ++u) {
      const int v = v0 + u * stride;
      if (v < total) dst_u[v] = buf[u];
    }
  }
}

hipError_t launch_gather_values(const void* store, const int32_t* sel_ids, void* v_sparse, int kv_bytes, int units,
                                int d, int s, int s_cap, int c, int k, hipStream_t st) {
  const int vec_per_chunk = c * d * kv_bytes / 16;
  const int total = k * vec_per_chunk;
  int gx = (total + 256 * kGatherUnroll - 1) / (256 * kGatherUnroll);
  if (gx < 1) gx = 1;
  dim3 grid(gx, units), block(256);
  hipLaunchKernelGGL(gather_values_kernel, grid, block, 0, st, reinterpret_cast<const uint4*>(store), sel_ids,
                     reinterpret_cast<uint4*>(v_sparse), k, vec_per_chunk, (size_t)s_cap * d * kv_bytes / 16, s / c - 1);
  return hipGetLastError();
}

// Workgroups of a gather that shares a launch with the key phase: at most one per compute unit, so that the
// key phase finds the other half of every unit's slots free; whole workgroups per unit when there are few units.
void plan_gather(GatherArgs* g) {
  constexpr int kMaxBlocks = 256;
  const long per_unit = (long)g->k * g->vec_per_chunk;
  if (g->units <= kMaxBlocks) {
    long bpu = kMaxBlocks / g->units;
    const long useful = (per_unit + 256 * kGatherUnroll - 1) / (256 * kGatherUnroll);
    if (bpu > useful) bpu = useful;
    if (bpu < 1) bpu = 1;
    g->blocks_per_unit = (int)bpu;
    g->n_blocks = (int)bpu * g->units;
    g->unit_step = g->units;
  } else {
    g->blocks_per_unit = 1;
    g->n_blocks = kMaxBlocks;
    g->unit_step = kMaxBlocks;
  }
}

}  // namespace skv
