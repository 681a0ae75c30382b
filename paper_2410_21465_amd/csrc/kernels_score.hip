// Landmark scoring: P = Q L^T * scale for every landmark slot (first line of the
// decoding algorithm), streamed once from HBM for the heads of a KV group (up to four here, up to 16 per pass in
// score_kernel_g16 further down).
//
// The scores decide an index set that has to match an fp64 reference: the logit is the
// plain dot product of the bf16 inputs, so the inputs are widened to fp64 and contracted on
// the fp64 matrix pipe (v_mfma_f64_4x4x4f64: four independent 4x4x4 blocks per wave, 256 FMAs
// per issue, no cross-lane reduction needed); the products are exact and the fp64 sum does
// not depend on the order of summation beyond its last bit.  The per-tile softmax statistics
// are formed from the fp64 logits.  What is stored for the selection is the logit rounded once
// to fp32 (half the bytes): the selection searches on those and settles its boundary on logits
// it forms again in fp64, so the rounding never decides a rank.  The vector ALU only unpacks
// and converts, which leaves the kernel bound by the HBM read of L.
//
// Operand layout of the instruction, as measured on gfx950: input lane
// = 16*k + 4*block + (i for A | j for B), result lane = 16*i + 4*block + j.
// Here i = query head (4), j = landmark row inside the block (4 blocks = 16 rows),
// k = which 16-byte piece of each 64-byte row segment the lane loads.  A wave covers
// 64 rows (four 16-row tiles, all loads issued before the first MFMA), a workgroup 256.
// Result lane 16*i + r holds the logit of head i, row r of the tile: it stores it
// (16 consecutive floats per head) and folds the fp64 value into its running (max, sum exp),
// from which the selection kernel forms each head's log-sum-exp.
#include "kernels.hpp"

namespace skv {

// exp(x) for x <= 0 through the fp32 exp2 unit.  It only feeds the softmax normaliser (a sum of
// such terms kept in fp64): its ~1e-7 relative error moves a head's log-sum-exp by ~1e-7, an
// order below the 1e-6 at which two scores count as tied; the logits themselves stay fp64.
__device__ __forceinline__ double exp_neg(double x) {
  return (double)__builtin_amdgcn_exp2f((float)(x * 1.4426950408889634074));
}

// (m, s) <- (m, s) (+) (m2, s2) for s = sum exp(p - m)
__device__ __forceinline__ void lse_merge(double& m, double& s, double m2, double s2) {
  if (m2 == -INFINITY) return;
  if (m == -INFINITY) { m = m2; s = s2; return; }
  const double e = exp_neg(-fabs(m - m2));
  if (m2 > m) { s = s * e + s2; m = m2; } else { s += s2 * e; }
}

// EB = bytes per landmark element: 2 (bf16) or 1 (FP8 E5M2 storage; a row is then d bytes and a lane's
// piece holds twice as many elements, or the same number in 8 bytes when d is not a multiple of 64).
// HG = groups of four heads per landmark element: 1, or 2 for 5 to 8 query heads per KV head.  With HG = 2 every
// widened landmark element feeds two instructions (heads 0-3, heads 4-7; two accumulators per tile), so the
// landmarks are read and converted once for all eight heads.  The queries live in LDS as fp64.
template <int D, int EB, int HG>
__global__ __launch_bounds__(256) void score_kernel(const bf16_t* __restrict__ q, const uint8_t* __restrict__ L,
                                                    float* __restrict__ logits, double2* __restrict__ partials,
                                                    int hq, int hkv, int G, int n_c, int ld, int nc_stride, int n_tiles,
                                                    double scale) {
  constexpr int PB = (EB == 2 || D % 64 == 0) ? 16 : 8;  // bytes per piece
  constexpr int PE = PB / EB;                             // elements per piece
  constexpr int NI = D / (4 * PE);                        // pieces per lane per row
  constexpr int PW = PB / 4;                              // 32-bit words per piece
  __shared__ double2 wred[4][4 * HG];
  // q of the workgroup's heads as fp64; rows padded so that the four heads a block column reads at once fall
  // into different banks
  __shared__ double qs[4 * HG][D + 2];
  const int unit = blockIdx.y, tile = blockIdx.x, g0 = blockIdx.z * 4 * HG;
  const int b = unit / hkv, h = unit % hkv;
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  const int kq = lane >> 4, blk = (lane >> 2) & 3, ij = lane & 3;
  const size_t head0 = (size_t)b * hq + (size_t)h * G + g0;

  const uint8_t* Lu = L + (size_t)unit * nc_stride * D * EB;  // the landmark array may have room to grow
  const int row0 = tile * kScoreTile + wave * kWave;
  uint32_t w[4][NI][PW];  // requested before q: the landmark rows are the long-latency loads
#pragma unroll
  for (int t = 0; t < 4; ++t) {
    const int r = row0 + t * 16 + blk * 4 + ij;
#pragma unroll
    for (int i = 0; i < NI; ++i) {
#pragma unroll
      for (int x = 0; x < PW; ++x) w[t][i][x] = 0u;
      if (r < n_c) {
        const uint8_t* src = Lu + (size_t)r * D * EB + (size_t)(4 * PE * i + PE * kq) * EB;
        if constexpr (PW == 4) {
          const uint4 v = *reinterpret_cast<const uint4*>(src);
          w[t][i][0] = v.x; w[t][i][1] = v.y; w[t][i][2] = v.z; w[t][i][3] = v.w;
        } else {
          const uint2 v = *reinterpret_cast<const uint2*>(src);
          w[t][i][0] = v.x; w[t][i][1] = v.y;
        }
      }
    }
  }

  // A operand: q of the workgroup's heads as fp64, in LDS (registers are better spent on landmark rows in
  // flight); a lane reads head 4 hg + ij, the elements its k-slot meets
  for (int idx = threadIdx.x; idx < 4 * HG * D; idx += 256) {
    const int hh = idx / D, e = idx - hh * D;
    qs[hh][e] = g0 + hh < G ? (double)bf16_to_f32(q[(head0 + hh) * D + e]) : 0.0;
  }
  __syncthreads();

  double m[HG], s[HG];   // heads g0 + 4 hg + lane / 16
#pragma unroll
  for (int hg = 0; hg < HG; ++hg) { m[hg] = -INFINITY; s[hg] = 0.0; }
#pragma unroll
  for (int t = 0; t < 4; ++t) {
    double acc[HG];
#pragma unroll
    for (int hg = 0; hg < HG; ++hg) acc[hg] = 0.0;
    // one widened landmark element against the matching q element of each head group
    auto step = [&](int i, int el, double lv) {
      const int col = 4 * PE * i + PE * kq + el;
#pragma unroll
      for (int hg = 0; hg < HG; ++hg)
        acc[hg] = __builtin_amdgcn_mfma_f64_4x4x4f64(qs[4 * hg + ij][col], lv, acc[hg], 0, 0, 0);
    };
#pragma unroll
    for (int i = 0; i < NI; ++i) {
#pragma unroll
      for (int x = 0; x < PW; ++x) {
        if constexpr (EB == 2) {
          step(i, 2 * x, (double)bf16_lo(w[t][i][x]));
          step(i, 2 * x + 1, (double)bf16_hi(w[t][i][x]));
        } else {
          float f[4];
          e5m2x4_to_f32(w[t][i][x], f);
#pragma unroll
          for (int e = 0; e < 4; ++e) step(i, 4 * x + e, (double)f[e]);
        }
      }
    }
    const int r = row0 + t * 16 + (lane & 15);
#pragma unroll
    for (int hg = 0; hg < HG; ++hg) {
      const int hl = 4 * hg + (lane >> 4);   // head of this lane's result, inside the workgroup's heads
      if (r < n_c && g0 + hl < G) {
        const double p = acc[hg] * scale;   // the logit: exact products, fp64 sum
        logits[(head0 + hl) * ld + r] = (float)p;
        lse_merge(m[hg], s[hg], p, 1.0);
      }
    }
  }

  // (max, sum) of each head over the workgroup's 256 rows
#pragma unroll
  for (int hg = 0; hg < HG; ++hg) {
#pragma unroll
    for (int x = 8; x >= 1; x >>= 1) lse_merge(m[hg], s[hg], shfl_xor_f64(m[hg], x), shfl_xor_f64(s[hg], x));
    if ((lane & 15) == 0) wred[wave][4 * hg + (lane >> 4)] = make_double2(m[hg], s[hg]);
  }
  __syncthreads();
  if (threadIdx.x < 4 * HG && g0 + (int)threadIdx.x < G) {
    const int g = threadIdx.x;
    double M = -INFINITY, S = 0.0;
#pragma unroll
    for (int wv = 0; wv < 4; ++wv) lse_merge(M, S, wred[wv][g].x, wred[wv][g].y);
    partials[(head0 + g) * n_tiles + tile] = make_double2(M, S);
  }
}

// Groups of more than 4 query heads per KV head: the 16x16x4 form of the fp64 matrix instruction takes up to
// 16 heads at once (A lane l = (head l % 16, k-slot l / 16), B lane l = (row l % 16, k-slot l / 16), result register j
// of lane l = (head 4 j + l / 16, row l % 16); measured on gfx950), so every landmark element is loaded and widened
// once instead of once per four heads.  Same tiles, same logits (exact products, fp64 sum) and partials as above.
typedef double f64x4_t __attribute__((ext_vector_type(4)));
template <int D, int EB>
__global__ __launch_bounds__(256) void score_kernel_g16(const bf16_t* __restrict__ q, const uint8_t* __restrict__ L,
                                                        float* __restrict__ logits, double2* __restrict__ partials,
                                                        int hq, int hkv, int G, int n_c, int ld, int nc_stride,
                                                        int n_tiles, double scale) {
  constexpr int PB = (EB == 2 || D % 64 == 0) ? 16 : 8;
  constexpr int PE = PB / EB, NI = D / (4 * PE), PW = PB / 4;
  __shared__ double2 wred[4][16];
  const int unit = blockIdx.y, tile = blockIdx.x, g0 = blockIdx.z * 16;
  const int b = unit / hkv, h = unit % hkv;
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  const int kq = lane >> 4, rl = lane & 15;
  const size_t head0 = (size_t)b * hq + (size_t)h * G + g0;
  const uint8_t* Lu = L + (size_t)unit * nc_stride * D * EB;
  const int row0 = tile * kScoreTile + wave * kWave;
  uint32_t w[4][NI][PW];
#pragma unroll
  for (int t = 0; t < 4; ++t) {
    const int r = row0 + t * 16 + rl;
#pragma unroll
    for (int i = 0; i < NI; ++i) {
#pragma unroll
      for (int x = 0; x < PW; ++x) w[t][i][x] = 0u;
      if (r < n_c) {
        const uint8_t* src = Lu + (size_t)r * D * EB + (size_t)(4 * PE * i + PE * kq) * EB;
        if constexpr (PW == 4) {
          const uint4 v = *reinterpret_cast<const uint4*>(src);
          w[t][i][0] = v.x; w[t][i][1] = v.y; w[t][i][2] = v.z; w[t][i][3] = v.w;
        } else {
          const uint2 v = *reinterpret_cast<const uint2*>(src);
          w[t][i][0] = v.x; w[t][i][1] = v.y;
        }
      }
    }
  }
  double qa[NI][PE];  // head g0 + rl, the elements this lane's k-slot meets (zero for heads past the group)
  const bool hv = g0 + rl < G;
  {
    const bf16_t* qp = q + (head0 + (hv ? rl : 0)) * D + PE * kq;
#pragma unroll
    for (int i = 0; i < NI; ++i)
#pragma unroll
      for (int e8 = 0; e8 < PE / 8; ++e8) {
        float x[8];
        load_bf16_row<8>(qp + 4 * PE * i + 8 * e8, x);
#pragma unroll
        for (int e = 0; e < 8; ++e) qa[i][8 * e8 + e] = hv ? (double)x[e] : 0.0;
      }
  }
  double m[4], s[4];   // heads g0 + 4 j + kq
#pragma unroll
  for (int j = 0; j < 4; ++j) { m[j] = -INFINITY; s[j] = 0.0; }
  // the four 16-row tiles of the wave take turns on the matrix pipe: consecutive instructions are independent,
  // a tile's own chain comes round every fourth one
  f64x4_t acc[4];
#pragma unroll
  for (int t = 0; t < 4; ++t) acc[t] = f64x4_t{0.0, 0.0, 0.0, 0.0};
#pragma unroll
  for (int i = 0; i < NI; ++i)
#pragma unroll
    for (int x = 0; x < PW; ++x) {
      if constexpr (EB == 2) {
#pragma unroll
        for (int t = 0; t < 4; ++t)
          acc[t] = __builtin_amdgcn_mfma_f64_16x16x4f64(qa[i][2 * x], (double)bf16_lo(w[t][i][x]), acc[t], 0, 0, 0);
#pragma unroll
        for (int t = 0; t < 4; ++t)
          acc[t] = __builtin_amdgcn_mfma_f64_16x16x4f64(qa[i][2 * x + 1], (double)bf16_hi(w[t][i][x]), acc[t], 0, 0, 0);
      } else {
        float f[4][4];
#pragma unroll
        for (int t = 0; t < 4; ++t) e5m2x4_to_f32(w[t][i][x], f[t]);
#pragma unroll
        for (int e = 0; e < 4; ++e)
#pragma unroll
          for (int t = 0; t < 4; ++t)
            acc[t] = __builtin_amdgcn_mfma_f64_16x16x4f64(qa[i][4 * x + e], (double)f[t][e], acc[t], 0, 0, 0);
      }
    }
#pragma unroll
  for (int t = 0; t < 4; ++t) {
    const int r = row0 + t * 16 + rl;
    if (r < n_c) {
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        if (g0 + 4 * j + kq < G) {
          const double p = acc[t][j] * scale;   // the logit: exact products, fp64 sum
          logits[(head0 + 4 * j + kq) * ld + r] = (float)p;
          lse_merge(m[j], s[j], p, 1.0);
        }
      }
    }
  }
#pragma unroll
  for (int j = 0; j < 4; ++j) {
#pragma unroll
    for (int x = 8; x >= 1; x >>= 1) lse_merge(m[j], s[j], shfl_xor_f64(m[j], x), shfl_xor_f64(s[j], x));
    if (rl == 0) wred[wave][4 * j + kq] = make_double2(m[j], s[j]);
  }
  __syncthreads();
  if (threadIdx.x < 16 && g0 + (int)threadIdx.x < G) {
    const int g = threadIdx.x;
    double M = -INFINITY, S = 0.0;
#pragma unroll
    for (int wv = 0; wv < 4; ++wv) lse_merge(M, S, wred[wv][g].x, wred[wv][g].y);
    partials[(head0 + g) * n_tiles + tile] = make_double2(M, S);
  }
}

hipError_t launch_score(const bf16_t* q, const void* landmarks, int kv_bytes, float* logits, int ld, double2* partials,
                        int batch, int hq, int hkv, int d, int n_c, int nc_stride, double scale, hipStream_t st) {
  const int G = hq / hkv;
  const int n_tiles = (n_c + kScoreTile - 1) / kScoreTile;
  // up to four heads per KV head: score_kernel<.., 1>; five to eight: score_kernel<.., 2>; more: one pass per 16
  // heads on the 16x16x4 instruction (heads past the group are zero rows of its operand)
  const bool g16 = G > 8;
  dim3 grid(n_tiles, batch * hkv, g16 ? (G + 15) / 16 : 1), block(256);
  const uint8_t* L = static_cast<const uint8_t*>(landmarks);
#define SKV_SCORE(D_, EB_)                                                                                            \
  do {                                                                                                                \
    if (g16) hipLaunchKernelGGL((score_kernel_g16<D_, EB_>), grid, block, 0, st, q, L, logits, partials, hq, hkv, G,   \
                                n_c, ld, nc_stride, n_tiles, scale);                                                  \
    else if (G > 4) hipLaunchKernelGGL((score_kernel<D_, EB_, 2>), grid, block, 0, st, q, L, logits, partials, hq,     \
                                       hkv, G, n_c, ld, nc_stride, n_tiles, scale);                                  \
    else hipLaunchKernelGGL((score_kernel<D_, EB_, 1>), grid, block, 0, st, q, L, logits, partials, hq, hkv, G, n_c,   \
                            ld, nc_stride, n_tiles, scale);                                                           \
  } while (0)
  switch (d * 4 + kv_bytes) {
    case 64 * 4 + 2: SKV_SCORE(64, 2); break;
    case 96 * 4 + 2: SKV_SCORE(96, 2); break;
    case 128 * 4 + 2: SKV_SCORE(128, 2); break;
    case 64 * 4 + 1: SKV_SCORE(64, 1); break;
    case 96 * 4 + 1: SKV_SCORE(96, 1); break;
    case 128 * 4 + 1: SKV_SCORE(128, 1); break;
    default: return hipErrorInvalidValue;
  }
#undef SKV_SCORE
  return hipGetLastError();
}

}  // namespace skv
