// Key reconstruction fused with RoPE: K_sparse = RoPE(Gather(A, I) * B) (decoding
// algorithm, "reconstruct key cache from low-rank projection" lines).  This is the one
// dense contraction of the path, [k*c x r] * [r x d] per (batch, KV head), on bf16 MFMA
// (v_mfma_f32_16x16x32_bf16, fp32 accumulate).
//
// A workgroup owns 256 selected tokens (4 waves x 4 row tiles of 16) and all d columns.
// B of the head is staged once per workgroup in LDS, transposed to [d][r] so that a lane's
// 8 consecutive k-values are one 16-byte LDS read; the A rows are gathered straight from
// HBM into MFMA operand layout (row = lane % 16, 8 consecutive ranks per lane).  With
// 16-wide column blocks the RoPE partner (i, i + d/2) of an accumulator sits in the same
// lane, d/32 blocks away, for d = 128, 96 and 64 alike, so the rotation is applied in
// registers before the single store.  Angles: position * frequency in fp64 revolutions,
// reduced to [-0.5, 0.5), then an fp32 sincospi -- accurate at positions beyond 2^20.
#include "kernels.hpp"

namespace skv {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;

constexpr int kReconRows = 256;  // selected tokens per workgroup
constexpr int kReconMT = 4;      // 16-row tiles per wave

template <int D>
__global__ __launch_bounds__(256) void recon_rope_kernel(const bf16_t* __restrict__ A, const bf16_t* __restrict__ B,
                                                         const int32_t* __restrict__ sel_ids,
                                                         const int32_t* __restrict__ pos_offset,
                                                         float* __restrict__ k_sparse, RopeFreqs freqs,
                                                         const float* __restrict__ inv_freq_dev, int hkv, int s,
                                                         int r, int c, int k, int r32, int rp) {
  const int last_chunk = s / c - 1;  // ids are clamped so that a bad id can never address outside A
  extern __shared__ __align__(16) bf16_t Bt[];  // [D][rp], element (n, kk) = B[kk][n]
  constexpr int NB = D / 16;
  const int unit = blockIdx.y, b = unit / hkv;
  const int rows_total = k * c;
  const int wg_row0 = blockIdx.x * kReconRows;
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  const int m = lane & 15, kq = lane >> 4;

  // ---- stage B^T (zero beyond rank r) ----
  {
    const bf16_t* Bu = B + (size_t)unit * r * D;
    for (int idx = threadIdx.x; idx < r32 * (D / 8); idx += 256) {
      const int kk = idx % r32, n8 = idx / r32;
      uint4 wv = make_uint4(0u, 0u, 0u, 0u);
      if (kk < r) wv = *reinterpret_cast<const uint4*>(Bu + (size_t)kk * D + n8 * 8);
      const uint32_t w4[4] = {wv.x, wv.y, wv.z, wv.w};
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        Bt[(n8 * 8 + 2 * i) * rp + kk] = (bf16_t)(w4[i] & 0xffffu);
        Bt[(n8 * 8 + 2 * i + 1) * rp + kk] = (bf16_t)(w4[i] >> 16);
      }
    }
  }
  __syncthreads();

  // ---- A rows of this lane's four row tiles ----
  const bf16_t* arow[kReconMT];
  bool valid[kReconMT];
  const int32_t* ids = sel_ids + (size_t)unit * k;
#pragma unroll
  for (int mt = 0; mt < kReconMT; ++mt) {
    const int i = wg_row0 + wave * 64 + mt * 16 + m;
    valid[mt] = i < rows_total;
    const int ch = valid[mt] ? i / c : 0;
    const int t = valid[mt] ? i - ch * c : 0;
    const size_t n = (size_t)min(max(ids[ch], 0), last_chunk) * c + t;
    arow[mt] = A + ((size_t)b * s + n) * r;
  }

  f32x4 acc[kReconMT][NB];
#pragma unroll
  for (int mt = 0; mt < kReconMT; ++mt)
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) acc[mt][nb] = f32x4{0.f, 0.f, 0.f, 0.f};

  const int ksteps = r32 / 32;
  for (int ks = 0; ks < ksteps; ++ks) {
    const int koff = ks * 32 + kq * 8;
    bf16x8 af[kReconMT];
#pragma unroll
    for (int mt = 0; mt < kReconMT; ++mt) {
      uint4 wv = make_uint4(0u, 0u, 0u, 0u);
      if (valid[mt] && koff < r) wv = *reinterpret_cast<const uint4*>(arow[mt] + koff);
      af[mt] = *reinterpret_cast<bf16x8*>(&wv);
    }
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
      const bf16x8 bfrag = *reinterpret_cast<const bf16x8*>(&Bt[(nb * 16 + m) * rp + koff]);
#pragma unroll
      for (int mt = 0; mt < kReconMT; ++mt)
        acc[mt][nb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(af[mt], bfrag, acc[mt][nb], 0, 0, 0);
    }
  }

  // ---- RoPE in registers and store.  Accumulator j of a lane is row 4*(lane/16)+j,
  //      column lane%16 of its 16x16 block. ----
  const double pos0 = pos_offset ? (double)pos_offset[b] : 0.0;
  double frev[NB / 2];
#pragma unroll
  for (int nb = 0; nb < NB / 2; ++nb) {
    const int f = nb * 16 + m;
    frev[nb] = inv_freq_dev ? (double)inv_freq_dev[f] * 0.15915494309189533577 : freqs.rev[f];
  }
  float* outu = k_sparse + (size_t)unit * rows_total * D;
#pragma unroll
  for (int mt = 0; mt < kReconMT; ++mt) {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int i = wg_row0 + wave * 64 + mt * 16 + kq * 4 + j;
      if (i >= rows_total) continue;
      const int ch = i / c, t = i - ch * c;
      const double pos = pos0 + (double)((size_t)min(max(ids[ch], 0), last_chunk) * c + t);
      float* orow = outu + (size_t)i * D;
#pragma unroll
      for (int nb = 0; nb < NB / 2; ++nb) {
        double rev = pos * frev[nb];
        rev -= rint(rev);
        float sn, cs;
        sincospif((float)(2.0 * rev), &sn, &cs);
        const float x0 = acc[mt][nb][j], x1 = acc[mt][nb + NB / 2][j];
        orow[nb * 16 + m] = x0 * cs - x1 * sn;
        orow[nb * 16 + m + D / 2] = x1 * cs + x0 * sn;
      }
    }
  }
}

hipError_t launch_recon(const bf16_t* A, const bf16_t* B, const int32_t* sel_ids, const int32_t* pos_offset,
                        float* k_sparse, const RopeFreqs& freqs, const float* inv_freq_dev, int batch, int hkv,
                        int d, int s, int r, int c, int k, hipStream_t st) {
  const int r32 = (r + 31) / 32 * 32;
  const int rp = r32 + 8;  // row pitch: 16-byte multiple, spreads 8-lane groups over all LDS banks
  const size_t lds = (size_t)d * rp * sizeof(bf16_t);
  dim3 grid((k * c + kReconRows - 1) / kReconRows, batch * hkv), block(256);
#define SKV_RECON(D_)                                                                                         \
  do {                                                                                                        \
    if (lds > 48 * 1024) {                                                                                    \
      hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&recon_rope_kernel<D_>),               \
                                         hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);               \
      if (e != hipSuccess) return e;                                                                          \
    }                                                                                                         \
    hipLaunchKernelGGL((recon_rope_kernel<D_>), grid, block, lds, st, A, B, sel_ids, pos_offset, k_sparse,    \
                       freqs, inv_freq_dev, hkv, s, r, c, k, r32, rp);                                        \
  } while (0)
  switch (d) {
    case 64: SKV_RECON(64); break;
    case 96: SKV_RECON(96); break;
    case 128: SKV_RECON(128); break;
    default: return hipErrorInvalidValue;
  }
#undef SKV_RECON
  return hipGetLastError();
}

}  // namespace skv
