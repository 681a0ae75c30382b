// One more chunk of context from generated tokens (last paragraph of section "High-throughput
// Decoding" and its footnote): new pre-RoPE keys K' are kept as the low-rank states K' Psi, where
// Psi is the right singular matrix of the context keys -- here Psi^T = B over the full key width,
// Psi[(h, x), rho] = B[b, h, rho, x].  The c tokens become chunk n_ch = s / c of the context exactly
// as if the pre-filling algorithm had seen them: c rows of A, one landmark (mean of the chunk's
// post-RoPE keys, fp64, rounded once), its chunk id, and the chunk's values in the store (a plain
// copy; the store may be pinned host memory written over PCIe).  Tiny, latency-bound kernels.
#include "kernels.hpp"

namespace skv {

// grid (c, batch), 256 threads: 16 lanes share one rank index, 16 rank indices per pass.
// EB: bytes per stored element (2 = bf16, 1 = FP8 E5M2), inputs and outputs alike.
template <int EB>
__global__ __launch_bounds__(256) void append_project_kernel(const void* __restrict__ k_pre,
                                                             const void* __restrict__ B, void* __restrict__ A,
                                                             int hkv, int d, int s, int s_cap, int c, int r) {
  const int t = blockIdx.x, b = blockIdx.y;
  const int sub = threadIdx.x & 15, grp = threadIdx.x >> 4;
  const size_t kp = ((size_t)b * c + t) * hkv * d;
  for (int rho0 = 0; rho0 < r; rho0 += 16) {
    const int rho = rho0 + grp;
    double acc = 0.0;
    if (rho < r)
      for (int h = 0; h < hkv; ++h) {
        const size_t brow = (((size_t)b * hkv + h) * r + rho) * d;
        for (int x = sub; x < d; x += 16)
          acc = fma((double)kv_elem<EB>(k_pre, kp + h * d + x), (double)kv_elem<EB>(B, brow + x), acc);
      }
    acc = sum16_f64(acc);
    if (rho < r && sub == 0) kv_store_elem<EB>(A, ((size_t)b * s_cap + s + t) * r + rho, acc);
  }
}

// grid (units), 256 threads: landmark row, its chunk id, and the copy of the chunk's values.
template <int EB>
__global__ __launch_bounds__(256) void append_landmark_kernel(const void* __restrict__ k_rope,
                                                              const uint4* __restrict__ v, void* __restrict__ landmarks,
                                                              int32_t* __restrict__ landmark_chunk_ids,
                                                              uint4* __restrict__ value_store, int d, int s, int s_cap,
                                                              int c, int o) {
  const int unit = blockIdx.x;
  const int n_ch = s / c, n_c = n_ch - o, nc_stride = s_cap / c - o;
  for (int x = threadIdx.x; x < d; x += 256) {
    double acc = 0.0;
    for (int t = 0; t < c; ++t) acc += (double)kv_elem<EB>(k_rope, ((size_t)unit * c + t) * d + x);
    kv_store_elem<EB>(landmarks, ((size_t)unit * nc_stride + n_c) * d + x, acc / (double)c);
  }
  if (threadIdx.x == 0) landmark_chunk_ids[(size_t)unit * nc_stride + n_c] = n_ch;
  const int vec = c * d * EB / 16;
  uint4* dst = value_store + ((size_t)unit * s_cap + s) * d * EB / 16;
  for (int i = threadIdx.x; i < vec; i += 256) dst[i] = v[(size_t)unit * vec + i];
}

template <int EB>
static hipError_t launch_append_eb(const void* k_pre, const void* k_rope, const void* v, const void* B, void* A,
                                   void* landmarks, int32_t* landmark_chunk_ids, void* value_store, int batch, int hkv,
                                   int d, int s, int s_cap, int c, int r, int o, hipStream_t st) {
  hipLaunchKernelGGL(append_project_kernel<EB>, dim3(c, batch), dim3(256), 0, st, k_pre, B, A, hkv, d, s, s_cap, c, r);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(append_landmark_kernel<EB>, dim3(batch * hkv), dim3(256), 0, st, k_rope,
                     reinterpret_cast<const uint4*>(v), landmarks, landmark_chunk_ids,
                     reinterpret_cast<uint4*>(value_store), d, s, s_cap, c, o);
  return hipGetLastError();
}

hipError_t launch_append_chunk(const void* k_pre, const void* k_rope, const void* v, const void* B, void* A,
                               void* landmarks, int32_t* landmark_chunk_ids, void* value_store, int kv_bytes, int batch,
                               int hkv, int d, int s, int s_cap, int c, int r, int o, hipStream_t st) {
  return kv_bytes == 1 ? launch_append_eb<1>(k_pre, k_rope, v, B, A, landmarks, landmark_chunk_ids, value_store, batch,
                                             hkv, d, s, s_cap, c, r, o, st)
                       : launch_append_eb<2>(k_pre, k_rope, v, B, A, landmarks, landmark_chunk_ids, value_store, batch,
                                             hkv, d, s, s_cap, c, r, o, st);
}

}  // namespace skv
