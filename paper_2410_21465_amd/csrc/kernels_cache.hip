// Chunk cache of the offloaded values (section "High-throughput Decoding": the chunks selected by
// adjacent decode steps repeat to a large part, so an index scan finds the missing ones and only
// those are fetched -- the (1 - alpha) term of the equivalent-bandwidth formula).
//
// A (batch, KV head) unit has S >= k slots of one chunk each, replaced least-recently-used: every
// step advances the unit's clock; a selected chunk found in a slot stays there and is stamped with
// the clock; the n_miss chunks found nowhere take the n_miss slots that were not hit and carry the
// oldest stamps (empty slots first; equal stamps: lower slot first), missing chunks in ascending
// chunk id to those slots in ascending index.  With S == k the slots hold exactly the last selection.
//   cache_update_kernel    index scan, victim selection, slot assignment; one workgroup per unit;
//   gather_missing_kernel  copies only the missing chunks from the store (pinned host memory read
//                          over PCIe, or HBM) into their slots.
// The attention kernel then reads each selected chunk's values from its slot.
#include "kernels.hpp"
#include "select.hpp"

namespace skv {

constexpr int kCacheNT = 256;

// Thread t owns slots t*E .. t*E + E - 1.
template <int E>
__global__ __launch_bounds__(kCacheNT) void cache_update_kernel(const int32_t* __restrict__ sel_ids,
                                                                int32_t* __restrict__ cache_ids,
                                                                int32_t* __restrict__ stamps,
                                                                int32_t* __restrict__ sel_slots,
                                                                int32_t* __restrict__ miss_slots,
                                                                int32_t* __restrict__ n_miss,
                                                                int32_t* __restrict__ n_miss_copy, int k, int S) {
  extern __shared__ int32_t cache_sm[];
  int32_t* sel = cache_sm;          // [k] this step's selection, ascending
  int32_t* slot_of = cache_sm + k;  // [k] slot of each selected chunk, -1 while unknown
  int32_t* miss_pos = slot_of + k;  // [k] position in `sel` of the new chunks, by rank
  __shared__ SelectSmem<kCacheNT> sm;
  __shared__ uint32_t wave_tot[kCacheNT / kWave];
  const int unit = blockIdx.x, tid = threadIdx.x;
  const int lane = tid & (kWave - 1), wave = tid / kWave;
  int32_t* ids = cache_ids + (size_t)unit * S;
  int32_t* st = stamps + (size_t)unit * (S + 1);
  const int32_t clock = st[S] + 1;

  for (int i = tid; i < k; i += kCacheNT) { sel[i] = sel_ids[(size_t)unit * k + i]; slot_of[i] = -1; }
  __syncthreads();
  // index scan: every slot looks its chunk up in the sorted selection.  A slot that is not hit gets a
  // key that grows with its age (empty: oldest) and, at equal age, with a lower slot index.
  uint64_t key[E];
#pragma unroll
  for (int e = 0; e < E; ++e) {
    const int slot = tid * E + e;
    key[e] = 0ull;
    if (slot < S) {
      const int id = ids[slot];
      int lo = 0, hi = k;
      while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        if (sel[mid] < id) lo = mid + 1; else hi = mid;
      }
      if (id >= 0 && lo < k && sel[lo] == id) {
        slot_of[lo] = slot;
        st[slot] = clock;
      } else {
        const uint32_t age = id < 0 ? 0x7fffffffu : (uint32_t)max(clock - st[slot], 1);
        key[e] = ((uint64_t)age << 32) | (uint32_t)(S - slot);
      }
    }
  }
  __syncthreads();
  // ranks of the new chunks (ascending chunk id): every thread owns a contiguous run of the selection
  const int per = (k + kCacheNT - 1) / kCacheNT;
  const int i0 = min(k, tid * per), i1 = min(k, i0 + per);
  uint32_t cm = 0;
  for (int i = i0; i < i1; ++i) cm += slot_of[i] < 0 ? 1u : 0u;
  uint32_t incl = cm;
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
  int rm = (int)(base + incl - cm);
  const int n_new = (int)total;
  for (int i = i0; i < i1; ++i)
    if (slot_of[i] < 0) miss_pos[rm++] = i;
  __syncthreads();
  // the n_new least recently used of the slots that were not hit; `pos` = how many of them precede
  // this thread's in slot order, which is the order the new chunks are handed out in
  uint32_t victim;
  int pos;
  block_select_topk<kCacheNT, E>(key, n_new, sm, victim, pos);
#pragma unroll
  for (int e = 0; e < E; ++e)
    if ((victim & (1u << e)) && pos < n_new) {
      const int slot = tid * E + e, j = miss_pos[pos];
      ids[slot] = sel[j];
      st[slot] = clock;
      slot_of[j] = slot;
      miss_slots[(size_t)unit * k + pos] = slot;
      ++pos;
    }
  __syncthreads();
  for (int i = tid; i < k; i += kCacheNT) sel_slots[(size_t)unit * k + i] = max(slot_of[i], 0);
  if (tid == 0) {
    st[S] = clock;
    n_miss[unit] = n_new;
    if (n_miss_copy) n_miss_copy[unit] = n_new;
  }
}

constexpr int kMissUnroll = 4;

__global__ __launch_bounds__(256) void gather_missing_kernel(const uint4* __restrict__ store,
                                                             const int32_t* __restrict__ cache_ids,
                                                             const int32_t* __restrict__ miss_slots,
                                                             const int32_t* __restrict__ n_miss,
                                                             uint4* __restrict__ v_cache, int k, int S, int vec_per_chunk,
                                                             size_t vec_per_unit_store, int last_chunk) {
  const int unit = blockIdx.y;
  const int total = min(max(n_miss[unit], 0), k) * vec_per_chunk;  // 16-byte vectors this unit fetches
  const int32_t* slots = cache_ids + (size_t)unit * S;
  const int32_t* ms = miss_slots + (size_t)unit * k;
  const uint4* src_u = store + (size_t)unit * vec_per_unit_store;
  uint4* dst_u = v_cache + (size_t)unit * S * vec_per_chunk;
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
        const int slot = min(max(ms[mi], 0), S - 1);
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

template <int E>
static hipError_t launch_cache_update_e(const int32_t* sel_ids, int32_t* cache_ids, int32_t* stamps, int32_t* sel_slots,
                                        int32_t* miss_slots, int32_t* n_miss, int32_t* n_miss_copy, int units, int k, int S,
                                        hipStream_t st) {
  const size_t lds = (size_t)3 * k * sizeof(int32_t);
  if (lds > 40 * 1024) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&cache_update_kernel<E>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
  }
  hipLaunchKernelGGL((cache_update_kernel<E>), dim3(units), dim3(kCacheNT), lds, st, sel_ids, cache_ids, stamps,
                     sel_slots, miss_slots, n_miss, n_miss_copy, k, S);
  return hipGetLastError();
}

hipError_t launch_cache_update(const int32_t* sel_ids, int32_t* cache_ids, int32_t* stamps, int32_t* sel_slots,
                               int32_t* miss_slots, int32_t* n_miss, int32_t* n_miss_copy, int units, int k, int S,
                               hipStream_t st) {
  int e = 1;
  while (kCacheNT * e < S) e *= 2;
#define SKV_CU(E_) return launch_cache_update_e<E_>(sel_ids, cache_ids, stamps, sel_slots, miss_slots, n_miss, n_miss_copy, units, k, S, st)
  switch (e) {
    case 1: SKV_CU(1);
    case 2: SKV_CU(2);
    case 4: SKV_CU(4);
    case 8: SKV_CU(8);
    case 16: SKV_CU(16);
    case 32: SKV_CU(32);
    default: return hipErrorInvalidValue;
  }
#undef SKV_CU
}

hipError_t launch_gather_missing(const void* store, const int32_t* cache_ids, const int32_t* miss_slots,
                                 const int32_t* n_miss, void* v_cache, int kv_bytes, int units, int d, int s, int s_cap,
                                 int c, int k, int S, hipStream_t st) {
  const int vec_per_chunk = c * d * kv_bytes / 16;
  const int total = k * vec_per_chunk;
  int gx = (total + 256 * kMissUnroll - 1) / (256 * kMissUnroll);
  if (gx < 1) gx = 1;
  hipLaunchKernelGGL(gather_missing_kernel, dim3(gx, units), dim3(256), 0, st, reinterpret_cast<const uint4*>(store),
                     cache_ids, miss_slots, n_miss, reinterpret_cast<uint4*>(v_cache), k, S, vec_per_chunk,
                     (size_t)s_cap * d * kv_bytes / 16, s / c - 1);
  return hipGetLastError();
}

hipError_t launch_fill_i32(int32_t* p, size_t n, int32_t value, hipStream_t st) {
  if (n == 0) return hipSuccess;
  hipLaunchKernelGGL(fill_i32_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, p, n, value);
  return hipGetLastError();
}

}  // namespace skv
