// Chunk cache of the offloaded values (section "High-throughput Decoding": the chunks selected by
// adjacent decode steps repeat to a large part, so an index scan finds the missing ones and only
// those are fetched -- the (1 - alpha) term of the equivalent-bandwidth formula).
//
// A (batch, KV head) unit has k slots of one chunk each.  Policy: after a step the slots hold
// exactly that step's selection; a chunk selected again keeps its slot; the new chunks, in
// ascending chunk id, take the slots whose chunk fell out, in ascending slot index.
//   cache_update_kernel    index scan + slot assignment, one workgroup per unit;
//   gather_missing_kernel  copies only the missing chunks from the store (pinned host memory read
//                          over PCIe, or HBM) into their slots.
// Attention is order-invariant over its key/value set, so the step then simply runs over the
// slots in slot order: selected ids := slot ids, staged values := the cache.
#include "kernels.hpp"

namespace skv {

constexpr int kCacheNT = 256;

__global__ __launch_bounds__(kCacheNT) void cache_update_kernel(const int32_t* __restrict__ sel_ids,
                                                                int32_t* __restrict__ cache_ids,
                                                                int32_t* __restrict__ miss_slots,
                                                                int32_t* __restrict__ n_miss,
                                                                int32_t* __restrict__ n_miss_copy, int k) {
  extern __shared__ int32_t cache_sm[];
  int32_t* sel = cache_sm;           // [k] this step's selection, ascending
  int32_t* miss_id = cache_sm + k;   // [k] the new chunks by rank
  uint8_t* hit = reinterpret_cast<uint8_t*>(cache_sm + 2 * k);  // [k] selection entry found in a slot
  uint8_t* keep = hit + k;                                      // [k] slot keeps its chunk
  __shared__ uint32_t wave_tot[kCacheNT / kWave];
  const int unit = blockIdx.x, tid = threadIdx.x;
  const int lane = tid & (kWave - 1), wave = tid / kWave;
  int32_t* slots = cache_ids + (size_t)unit * k;

  for (int i = tid; i < k; i += kCacheNT) { sel[i] = sel_ids[(size_t)unit * k + i]; hit[i] = 0; }
  __syncthreads();
  // index scan: every slot looks its chunk up in the sorted selection
  for (int s = tid; s < k; s += kCacheNT) {
    const int id = slots[s];
    int lo = 0, hi = k;
    while (lo < hi) {
      const int mid = (lo + hi) >> 1;
      if (sel[mid] < id) lo = mid + 1; else hi = mid;
    }
    const bool found = id >= 0 && lo < k && sel[lo] == id;
    keep[s] = found ? 1 : 0;
    if (found) hit[lo] = 1;
  }
  __syncthreads();
  // ranks of the new chunks and of the freed slots: every thread owns a contiguous run
  const int per = (k + kCacheNT - 1) / kCacheNT;
  const int i0 = min(k, tid * per), i1 = min(k, i0 + per);
  uint32_t cm = 0, cf = 0;
  for (int i = i0; i < i1; ++i) { cm += hit[i] ? 0u : 1u; cf += keep[i] ? 0u : 1u; }
  uint32_t incl = (cm << 16) | cf;  // k <= 8192: both running sums fit 16 bits
#pragma unroll
  for (int off = 1; off < kWave; off <<= 1) {
    const uint32_t t = (uint32_t)__shfl_up((int)incl, off, kWave);
    if (lane >= off) incl += t;
  }
  if (lane == kWave - 1) wave_tot[wave] = incl;
  __syncthreads();
  uint32_t base = 0, total = 0;
#pragma unroll
  for (int w = 0; w < kCacheNT / kWave; ++w) {
    if (w < wave) base += wave_tot[w];
    total += wave_tot[w];
  }
  const uint32_t excl = base + incl - ((cm << 16) | cf);
  const int n_new = (int)(total >> 16), n_free = (int)(total & 0xffffu);
  const int n_fill = min(n_new, n_free);  // equal whenever the slots held distinct chunks
  int rm = (int)(excl >> 16), rf = (int)(excl & 0xffffu);
  for (int i = i0; i < i1; ++i)
    if (!hit[i]) miss_id[rm++] = sel[i];
  __syncthreads();
  for (int i = i0; i < i1; ++i)
    if (!keep[i]) {
      if (rf < n_fill) {
        slots[i] = miss_id[rf];
        miss_slots[(size_t)unit * k + rf] = i;
      }
      ++rf;
    }
  if (tid == 0) {
    n_miss[unit] = n_fill;
    if (n_miss_copy) n_miss_copy[unit] = n_fill;
  }
}

constexpr int kMissUnroll = 4;

__global__ __launch_bounds__(256) void gather_missing_kernel(const uint4* __restrict__ store,
                                                             const int32_t* __restrict__ cache_ids,
                                                             const int32_t* __restrict__ miss_slots,
                                                             const int32_t* __restrict__ n_miss,
                                                             uint4* __restrict__ v_cache, int k, int vec_per_chunk,
                                                             size_t vec_per_unit_store, int last_chunk) {
  const int unit = blockIdx.y;
  const int total = min(max(n_miss[unit], 0), k) * vec_per_chunk;  // 16-byte vectors this unit fetches
  const int32_t* slots = cache_ids + (size_t)unit * k;
  const int32_t* ms = miss_slots + (size_t)unit * k;
  const uint4* src_u = store + (size_t)unit * vec_per_unit_store;
  uint4* dst_u = v_cache + (size_t)unit * k * vec_per_chunk;
  const int stride = gridDim.x * 256;
  for (int v0 = blockIdx.x * 256 + threadIdx.x; v0 < total; v0 += stride * kMissUnroll) {
    uint4 buf[kMissUnroll];
    int at[kMissUnroll];
#pragma unroll
    for (int u = 0; u < kMissUnroll; ++u) {
      const int v = v0 + u * stride;
      at[u] = -1;
      if (v < total) {
        const int mi = v / vec_per_chunk, off = v - mi * vec_per_chunk;
        const int slot = min(max(ms[mi], 0), k - 1);
        buf[u] = src_u[(size_t)min(max(slots[slot], 0), last_chunk) * vec_per_chunk + off];
        at[u] = slot * vec_per_chunk + off;
      }
    }
#pragma unroll
    for (int u = 0; u < kMissUnroll; ++u)
      if (at[u] >= 0) dst_u[at[u]] = buf[u];
  }
}

__global__ __launch_bounds__(256) void fill_i32_kernel(int32_t* __restrict__ p, size_t n, int32_t value) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i < n) p[i] = value;
}

size_t cache_update_lds_bytes(int k) { return (size_t)2 * k * sizeof(int32_t) + (size_t)2 * k; }

hipError_t launch_cache_update(const int32_t* sel_ids, int32_t* cache_ids, int32_t* miss_slots, int32_t* n_miss,
                               int32_t* n_miss_copy, int units, int k, hipStream_t st) {
  const size_t lds = cache_update_lds_bytes(k);
  if (lds > 48 * 1024) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&cache_update_kernel),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
  }
  hipLaunchKernelGGL(cache_update_kernel, dim3(units), dim3(kCacheNT), lds, st, sel_ids, cache_ids, miss_slots, n_miss,
                     n_miss_copy, k);
  return hipGetLastError();
}

hipError_t launch_gather_missing(const bf16_t* store, const int32_t* cache_ids, const int32_t* miss_slots,
                                 const int32_t* n_miss, bf16_t* v_cache, int units, int d, int s, int s_cap, int c,
                                 int k, hipStream_t st) {
  const int vec_per_chunk = c * d * 2 / 16;
  const int total = k * vec_per_chunk;
  int gx = (total + 256 * kMissUnroll - 1) / (256 * kMissUnroll);
  if (gx < 1) gx = 1;
  hipLaunchKernelGGL(gather_missing_kernel, dim3(gx, units), dim3(256), 0, st, reinterpret_cast<const uint4*>(store),
                     cache_ids, miss_slots, n_miss, reinterpret_cast<uint4*>(v_cache), k, vec_per_chunk,
                     (size_t)s_cap * d * 2 / 16, s / c - 1);
  return hipGetLastError();
}

hipError_t launch_fill_i32(int32_t* p, size_t n, int32_t value, hipStream_t st) {
  if (n == 0) return hipSuccess;
  hipLaunchKernelGGL(fill_i32_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, p, n, value);
  return hipGetLastError();
}

}  // namespace skv
