// First line of the pre-filling algorithm: A, B <- SVD(K) of the pre-RoPE keys K [s, D = h_kv*d]
// of every sequence, truncated to rank r: B = Psi^T (the r leading right singular vectors), A = K Psi
// (section "High-throughput Decoding", footnote: keys are stored as K Psi and projected back with Psi^T).
//
// On the GPU the right singular vectors are the leading eigenvectors of the Gram matrix G = K^T K:
//   1. gram_kernel: G in fp64 on the fp64 matrix pipe (v_mfma_f64_16x16x4f64; the products of stored
//      elements are exact, the sum is fp64) -- the dense contraction, 2 s D^2 flops, K streamed once per
//      column-block pair; only blocks on and above the diagonal are formed, gram_finish sums the token
//      splits and mirrors;
//   2. subspace iteration on m = r + oversample vectors (X <- orth(G X), modified Gram-Schmidt in groups), then one
//      Rayleigh-Ritz step: T = X^T G X, eigenvectors of the small T by one-sided Jacobi rotations, the r
//      largest kept -- all fp64, small, one launch per dependent step;
//   3. sign convention (largest-magnitude component positive), B written, and project_kernel: A = K Psi on
//      the same matrix instruction.
// Operand layout of v_mfma_f64_16x16x4f64 as measured on gfx950: A lane l holds (m = l % 16, k = l / 16),
// B lane l holds (n = l % 16, k = l / 16), result register j of lane l is (m = 4 j + l / 16, n = l % 16).
#include <algorithm>
#include <cstdlib>
#include <type_traits>

#include "kernels.hpp"

namespace skv {

typedef double f64x4 __attribute__((ext_vector_type(4)));

// four consecutive stored elements starting at element index `at` of `base` (zero when !ok), kept as stored and
// widened to fp64 when they are used: what a prefetch holds
template <int EB>
struct Raw4 {
  uint32_t w[EB == 2 ? 2 : 1];
  __device__ __forceinline__ void load(const void* base, size_t at, bool ok) {
    if constexpr (EB == 2) {
      uint2 v = make_uint2(0u, 0u);
      if (ok) v = *reinterpret_cast<const uint2*>(static_cast<const bf16_t*>(base) + at);
      w[0] = v.x; w[1] = v.y;
    } else {
      w[0] = ok ? *reinterpret_cast<const uint32_t*>(static_cast<const uint8_t*>(base) + at) : 0u;
    }
  }
  __device__ __forceinline__ void widen(double (&x)[4]) const {
    float f[4];
    if constexpr (EB == 2) { f[0] = bf16_lo(w[0]); f[1] = bf16_hi(w[0]); f[2] = bf16_lo(w[1]); f[3] = bf16_hi(w[1]); }
    else e5m2x4_to_f32(w[0], f);
#pragma unroll
    for (int e = 0; e < 4; ++e) x[e] = (double)f[e];
  }
};

// sixteen consecutive stored elements (32 or 16 bytes), widened four at a time
template <int EB>
struct Raw16 {
  uint32_t w[EB == 2 ? 8 : 4];
  __device__ __forceinline__ void load(const void* base, size_t at, bool ok) {
    uint4 lo = make_uint4(0u, 0u, 0u, 0u), hi = lo;
    if (ok) {
      if constexpr (EB == 2) {
        const uint4* p = reinterpret_cast<const uint4*>(static_cast<const bf16_t*>(base) + at);
        lo = p[0]; hi = p[1];
      } else {
        lo = *reinterpret_cast<const uint4*>(static_cast<const uint8_t*>(base) + at);
      }
    }
    w[0] = lo.x; w[1] = lo.y; w[2] = lo.z; w[3] = lo.w;
    if constexpr (EB == 2) { w[4] = hi.x; w[5] = hi.y; w[6] = hi.z; w[7] = hi.w; }
  }
  template <int U>
  __device__ __forceinline__ void widen4(double (&x)[4]) const {
    float f[4];
    if constexpr (EB == 2) { f[0] = bf16_lo(w[2 * U]); f[1] = bf16_hi(w[2 * U]); f[2] = bf16_lo(w[2 * U + 1]); f[3] = bf16_hi(w[2 * U + 1]); }
    else e5m2x4_to_f32(w[U], f);
#pragma unroll
    for (int e = 0; e < 4; ++e) x[e] = (double)f[e];
  }
};

// ---- 1. Gram matrix ---------------------------------------------------------------------------------
// One wave per (pair of 64-column blocks bi <= bj, token split, sequence).  Tile (mt, nt) of the 64 x 64
// block holds columns i0 + 4 m + mt against j0 + 4 n + nt, so that a lane's four consecutive columns feed
// four tiles and every load is 8 (or 4) contiguous bytes.  part [split][b][D][D] fp64, blocks bi <= bj only.
template <int EB>
__global__ __launch_bounds__(64) void gram_kernel(const void* __restrict__ K, double* __restrict__ part, int s, int D,
                                                  int nb, int tokens_per_split, int batch) {
  const int lane = threadIdx.x, mrow = lane & 15, kq = lane >> 4;
  // pair index -> (bi, bj), bi <= bj, row by row of the upper triangle
  int p = blockIdx.x, bi = 0;
  while (p >= nb - bi) { p -= nb - bi; ++bi; }
  const int bj = bi + p;
  const int split = blockIdx.y, b = blockIdx.z;
  const int t_begin = split * tokens_per_split, t_end = min(s, t_begin + tokens_per_split);
  const int ci = bi * 64 + 4 * mrow, cj = bj * 64 + 4 * mrow;
  const bool oki = ci < D, okj = cj < D;
  const size_t base = (size_t)b * s * D;

  f64x4 acc[4][4];
#pragma unroll
  for (int mt = 0; mt < 4; ++mt)
#pragma unroll
    for (int nt = 0; nt < 4; ++nt) acc[mt][nt] = f64x4{0.0, 0.0, 0.0, 0.0};

  // 16 tokens (four matrix steps) per iteration; the next iteration's rows are requested before this one's 64
  // matrix instructions, which is about the latency of a load
  constexpr int PF = 4;
  Raw4<EB> an[PF], bn[PF];
  auto request = [&](int t0) {
#pragma unroll
    for (int u = 0; u < PF; ++u) {
      const int t = t0 + 4 * u + kq;
      const size_t row = base + (size_t)min(t, s - 1) * D;
      an[u].load(K, row + ci, oki && t < t_end);
      bn[u].load(K, row + cj, okj && t < t_end);
    }
  };
  request(t_begin);
  for (int t0 = t_begin; t0 < t_end; t0 += 4 * PF) {
    Raw4<EB> ac[PF], bc[PF];
#pragma unroll
    for (int u = 0; u < PF; ++u) { ac[u] = an[u]; bc[u] = bn[u]; }
    request(t0 + 4 * PF);
#pragma unroll
    for (int u = 0; u < PF; ++u) {
      double a[4], bb[4];
      ac[u].widen(a);
      bc[u].widen(bb);
#pragma unroll
      for (int mt = 0; mt < 4; ++mt)
#pragma unroll
        for (int nt = 0; nt < 4; ++nt)
          acc[mt][nt] = __builtin_amdgcn_mfma_f64_16x16x4f64(a[mt], bb[nt], acc[mt][nt], 0, 0, 0);
    }
  }
  double* out = part + ((size_t)split * batch + b) * D * D;
#pragma unroll
  for (int mt = 0; mt < 4; ++mt)
#pragma unroll
    for (int nt = 0; nt < 4; ++nt)
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int gi = bi * 64 + 4 * (4 * j + kq) + mt, gj = bj * 64 + 4 * mrow + nt;
        if (gi < D && gj < D) out[(size_t)gi * D + gj] = acc[mt][nt][j];
      }
}

// G[b][i][j] = sum over the splits of the block that holds (i, j) or, below the diagonal blocks, (j, i)
__global__ __launch_bounds__(256) void gram_finish_kernel(const double* __restrict__ part, double* __restrict__ G, int D,
                                                          int n_splits, int batch) {
  const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
  const int b = blockIdx.y;
  if (idx >= (size_t)D * D) return;
  const int i = (int)(idx / D), j = (int)(idx % D);
  const bool upper = i / 64 <= j / 64;
  const size_t src = upper ? (size_t)i * D + j : (size_t)j * D + i;
  double sum = 0.0;
  for (int sp = 0; sp < n_splits; ++sp) sum += part[((size_t)sp * batch + b) * D * D + src];
  G[(size_t)b * D * D + idx] = sum;
}

// ---- 2. small fp64 linear algebra --------------------------------------------------------------------
// C[i][j] = sum_k A(i, k) B(k, j), all fp64, element (i, k) of A at A[i * sai + k * sak] (likewise B), C row-major
// with leading dimension ldc; batched by strides.  64 x 64 x 16 tiles through LDS, 4 x 4 results per thread.
__global__ __launch_bounds__(256) void dgemm_kernel(const double* __restrict__ A, const double* __restrict__ B,
                                                    double* __restrict__ C, int M, int N, int Kd, long sai, long sak,
                                                    long sbk, long sbj, int ldc, long strideA, long strideB,
                                                    long strideC) {
  __shared__ double As[16][65], Bs[16][65];
  const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
  const int i0 = blockIdx.y * 64, j0 = blockIdx.x * 64;
  A += (size_t)blockIdx.z * strideA; B += (size_t)blockIdx.z * strideB; C += (size_t)blockIdx.z * strideC;
  double acc[4][4];
#pragma unroll
  for (int x = 0; x < 4; ++x)
#pragma unroll
    for (int y = 0; y < 4; ++y) acc[x][y] = 0.0;
  for (int k0 = 0; k0 < Kd; k0 += 16) {
    for (int e = threadIdx.x; e < 16 * 64; e += 256) {
      // the index that is contiguous in memory runs fastest over the threads
      int kk, ii;
      if (sak == 1) { kk = e & 15; ii = e >> 4; } else { ii = e & 63; kk = e >> 6; }
      const int gi = i0 + ii, gk = k0 + kk;
      As[kk][ii] = (gi < M && gk < Kd) ? A[(size_t)gi * sai + (size_t)gk * sak] : 0.0;
      int kb, jj;
      if (sbk == 1) { kb = e & 15; jj = e >> 4; } else { jj = e & 63; kb = e >> 6; }
      const int gj = j0 + jj, gk2 = k0 + kb;
      Bs[kb][jj] = (gj < N && gk2 < Kd) ? B[(size_t)gk2 * sbk + (size_t)gj * sbj] : 0.0;
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < 16; ++kk) {
      double a[4], bq[4];
#pragma unroll
      for (int x = 0; x < 4; ++x) { a[x] = As[kk][ty + 16 * x]; bq[x] = Bs[kk][tx + 16 * x]; }
#pragma unroll
      for (int x = 0; x < 4; ++x)
#pragma unroll
        for (int y = 0; y < 4; ++y) acc[x][y] = fma(a[x], bq[y], acc[x][y]);
    }
    __syncthreads();
  }
#pragma unroll
  for (int x = 0; x < 4; ++x)
#pragma unroll
    for (int y = 0; y < 4; ++y) {
      const int gi = i0 + ty + 16 * x, gj = j0 + tx + 16 * y;
      if (gi < M && gj < N) C[(size_t)gi * ldc + gj] = acc[x][y];
    }
}

__device__ __forceinline__ double block_sum_256(double v, double* sm) {
  v = wave_sum_f64(v);
  const int wave = threadIdx.x >> 6;
  __syncthreads();
  if ((threadIdx.x & 63) == 0) sm[wave] = v;
  __syncthreads();
  return sm[0] + sm[1] + sm[2] + sm[3];
}

// start vectors: Xt[b][i][x] uniform in (-1, 1) from a counter-based hash (same numbers on every run)
__global__ __launch_bounds__(256) void subspace_init_kernel(double* __restrict__ Xt, size_t n) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= n) return;
  uint64_t z = (i + 1) * 0x9E3779B97F4A7C15ull;
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  z ^= z >> 31;
  Xt[i] = (double)(int64_t)(z >> 11) * (1.0 / 4503599627370496.0) - 1.0;  // 53 bits -> [-1, 1)
}

// sums of NV values per thread over the 256 threads of the workgroup (result in every thread)
template <int NV>
__device__ __forceinline__ void block_sum_multi(double (&v)[NV], double (*sm)[NV]) {
  const int wave = threadIdx.x >> 6;
#pragma unroll
  for (int i = 0; i < NV; ++i) v[i] = wave_sum_f64(v[i]);
  __syncthreads();
  if ((threadIdx.x & 63) == 0)
#pragma unroll
    for (int i = 0; i < NV; ++i) sm[wave][i] = v[i];
  __syncthreads();
#pragma unroll
  for (int i = 0; i < NV; ++i) v[i] = sm[0][i] + sm[1][i] + sm[2][i] + sm[3][i];
}

// Modified Gram-Schmidt in groups of Q vectors (vectors are not normalised until the end), two launches per group
// instead of one per vector.  First the Q pivots j .. j+q-1 are made orthogonal among themselves by one workgroup
// per sequence that keeps them in registers (EPT elements per thread and vector) ...
template <int Q, int EPT>
__global__ __launch_bounds__(256) void mgs_pivots_kernel(double* __restrict__ Xt, int D, int m, int j, int q) {
  __shared__ double sm[4][Q];
  double* X0 = Xt + ((size_t)blockIdx.x * m + j) * D;
  double p[Q][EPT];
#pragma unroll
  for (int a = 0; a < Q; ++a)
#pragma unroll
    for (int e = 0; e < EPT; ++e) {
      const int x = threadIdx.x + 256 * e;
      p[a][e] = (a < q && x < D) ? X0[(size_t)a * D + x] : 0.0;
    }
#pragma unroll
  for (int a = 0; a + 1 < Q; ++a) {
    double v[Q];  // v[a] = |p_a|^2, v[b] = p_a . p_b for b > a
#pragma unroll
    for (int bb = 0; bb < Q; ++bb) {
      v[bb] = 0.0;
      if (bb >= a)
#pragma unroll
        for (int e = 0; e < EPT; ++e) v[bb] = fma(p[a][e], p[bb][e], v[bb]);
    }
    block_sum_multi<Q>(v, sm);
    if (v[a] > 0.0) {
#pragma unroll
      for (int bb = a + 1; bb < Q; ++bb) {
        const double f = v[bb] / v[a];
#pragma unroll
        for (int e = 0; e < EPT; ++e) p[bb][e] = fma(-f, p[a][e], p[bb][e]);
      }
    }
  }
#pragma unroll
  for (int a = 1; a < Q; ++a)
#pragma unroll
    for (int e = 0; e < EPT; ++e) {
      const int x = threadIdx.x + 256 * e;
      if (a < q && x < D) X0[(size_t)a * D + x] = p[a][e];
    }
}
// ... then every later vector k loses its components along the q pivots, one after the other
template <int Q, int EPT>
__global__ __launch_bounds__(256) void mgs_project_kernel(double* __restrict__ Xt, int D, int m, int j, int q) {
  __shared__ double sm[4][2];
  const int k = j + q + blockIdx.x, b = blockIdx.y;
  const double* P0 = Xt + ((size_t)b * m + j) * D;
  double* xk = Xt + ((size_t)b * m + k) * D;
  double x[EPT];
#pragma unroll
  for (int e = 0; e < EPT; ++e) {
    const int c = threadIdx.x + 256 * e;
    x[e] = c < D ? xk[c] : 0.0;
  }
#pragma unroll
  for (int a = 0; a < Q; ++a) {
    if (a >= q) break;
    double pa[EPT], v[2] = {0.0, 0.0};
#pragma unroll
    for (int e = 0; e < EPT; ++e) {
      const int c = threadIdx.x + 256 * e;
      pa[e] = c < D ? P0[(size_t)a * D + c] : 0.0;
      v[0] = fma(pa[e], pa[e], v[0]);
      v[1] = fma(pa[e], x[e], v[1]);
    }
    block_sum_multi<2>(v, sm);
    if (v[0] > 0.0) {
      const double f = v[1] / v[0];
#pragma unroll
      for (int e = 0; e < EPT; ++e) x[e] = fma(-f, pa[e], x[e]);
    }
  }
#pragma unroll
  for (int e = 0; e < EPT; ++e) {
    const int c = threadIdx.x + 256 * e;
    if (c < D) xk[c] = x[e];
  }
}
// key widths beyond what the grouped kernels hold in registers: one launch per vector
__global__ __launch_bounds__(256) void mgs_step_kernel(double* __restrict__ Xt, int D, int m, int j) {
  __shared__ double sm[4];
  const int k = j + 1 + blockIdx.x, b = blockIdx.y;
  double* xj = Xt + ((size_t)b * m + j) * D;
  double* xk = Xt + ((size_t)b * m + k) * D;
  double njj = 0.0, d = 0.0;
  for (int x = threadIdx.x; x < D; x += 256) { const double a = xj[x]; njj = fma(a, a, njj); d = fma(a, xk[x], d); }
  njj = block_sum_256(njj, sm);
  d = block_sum_256(d, sm);
  if (!(njj > 0.0)) return;
  const double f = d / njj;
  for (int x = threadIdx.x; x < D; x += 256) xk[x] = fma(-f, xj[x], xk[x]);
}
__global__ __launch_bounds__(256) void normalize_rows_kernel(double* __restrict__ Xt, int D) {
  __shared__ double sm[4];
  double* x = Xt + (size_t)blockIdx.x * D;
  double n = 0.0;
  for (int i = threadIdx.x; i < D; i += 256) n = fma(x[i], x[i], n);
  n = block_sum_256(n, sm);
  if (!(n > 0.0)) return;
  const double inv = 1.0 / sqrt(n);
  for (int i = threadIdx.x; i < D; i += 256) x[i] *= inv;
}

// V <- identity (mp x mp per sequence); W is filled by the product X^T G X before
__global__ __launch_bounds__(256) void identity_kernel(double* __restrict__ V, int mp) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= (size_t)mp * mp) return;
  V[(size_t)blockIdx.y * mp * mp + i] = (i / mp == i % mp) ? 1.0 : 0.0;
}

// One step of a one-sided Jacobi sweep on the columns of W (initially T = X^T G X, symmetric; column p is
// W[p*mp ...]) with the rotations accumulated in V: after convergence the columns of W are orthogonal, their
// norms are the eigenvalues of T and the columns of V its eigenvectors.  Pairs of step `st` by the circle
// method over mp (even) players: (mp-1, st), ((st+i) mod (mp-1), (st-i) mod (mp-1)).  One wave per pair.
__global__ __launch_bounds__(64) void jacobi_step_kernel(double* __restrict__ W, double* __restrict__ V, int mp, int st) {
  const int i = blockIdx.x, b = blockIdx.y, lane = threadIdx.x;
  int p, q;
  if (i == 0) { p = mp - 1; q = st; }
  else { p = (st + i) % (mp - 1); q = (st - i + (mp - 1)) % (mp - 1); }
  double* wp = W + ((size_t)b * mp + p) * mp;
  double* wq = W + ((size_t)b * mp + q) * mp;
  double al = 0.0, be = 0.0, ga = 0.0;
  for (int x = lane; x < mp; x += 64) { const double a = wp[x], c = wq[x]; al = fma(a, a, al); be = fma(c, c, be); ga = fma(a, c, ga); }
  al = wave_sum_f64(al); be = wave_sum_f64(be); ga = wave_sum_f64(ga);
  if (!(fabs(ga) > 1e-300) || fabs(ga) <= 1e-17 * sqrt(al) * sqrt(be)) return;
  const double zeta = (be - al) / (2.0 * ga);
  const double t = (zeta >= 0.0 ? 1.0 : -1.0) / (fabs(zeta) + sqrt(1.0 + zeta * zeta));
  const double c = 1.0 / sqrt(1.0 + t * t), sn = c * t;
  double* vp = V + ((size_t)b * mp + p) * mp;
  double* vq = V + ((size_t)b * mp + q) * mp;
  for (int x = lane; x < mp; x += 64) {
    const double a = wp[x], d = wq[x];
    wp[x] = c * a - sn * d; wq[x] = sn * a + c * d;
    const double e = vp[x], f = vq[x];
    vp[x] = c * e - sn * f; vq[x] = sn * e + c * f;
  }
}

// the r columns of W with the largest norms (ties: lower index), strongest first: their eigenvectors (columns
// of V, restricted to the first m entries) become the rows of Wsel [r][m]
__global__ __launch_bounds__(256) void ritz_select_kernel(const double* __restrict__ W, const double* __restrict__ V,
                                                          double* __restrict__ Wsel, double* __restrict__ sigma_out,
                                                          int mp, int m, int r) {
  extern __shared__ double nrm[];  // [mp]
  const int b = blockIdx.x;
  for (int p = threadIdx.x; p < mp; p += 256) {
    const double* w = W + ((size_t)b * mp + p) * mp;
    double n = 0.0;
    for (int x = 0; x < mp; ++x) n = fma(w[x], w[x], n);
    nrm[p] = p < m ? n : -1.0;   // padding columns never win
  }
  __syncthreads();
  for (int p = threadIdx.x; p < m; p += 256) {
    int rank = 0;
    for (int o = 0; o < m; ++o) rank += (nrm[o] > nrm[p]) || (nrm[o] == nrm[p] && o < p);
    if (rank < r) {
      const double* v = V + ((size_t)b * mp + p) * mp;
      double* dst = Wsel + ((size_t)b * r + rank) * m;
      for (int x = 0; x < m; ++x) dst[x] = v[x];
      if (sigma_out) sigma_out[(size_t)b * r + rank] = sqrt(sqrt(nrm[p]));  // |column| = eigenvalue of G = sigma^2
    }
  }
}

// sign convention and B: the component of largest magnitude of every right singular vector is made positive
// (ties: lowest index); Psi_t [b][r][D] is updated in place, B [b][h_kv][r][d] is its rounding to storage
template <int EB>
__global__ __launch_bounds__(256) void emit_b_kernel(double* __restrict__ Psi_t, void* __restrict__ Bout, int D, int r,
                                                     int hkv, int d) {
  __shared__ double sv[4];
  __shared__ int si[4];
  const int rho = blockIdx.x, b = blockIdx.y;
  double* v = Psi_t + ((size_t)b * r + rho) * D;
  double best = -1.0;
  int at = 0;
  for (int x = threadIdx.x; x < D; x += 256) { const double a = fabs(v[x]); if (a > best) { best = a; at = x; } }
#pragma unroll
  for (int msk = 32; msk >= 1; msk >>= 1) {
    const double ob = shfl_xor_f64(best, msk);
    const int oa = __shfl_xor(at, msk, kWave);
    if (ob > best || (ob == best && oa < at)) { best = ob; at = oa; }
  }
  if ((threadIdx.x & 63) == 0) { sv[threadIdx.x >> 6] = best; si[threadIdx.x >> 6] = at; }
  __syncthreads();
  best = sv[0]; at = si[0];
  for (int w = 1; w < 4; ++w) if (sv[w] > best || (sv[w] == best && si[w] < at)) { best = sv[w]; at = si[w]; }
  const double sign = v[at] < 0.0 ? -1.0 : 1.0;
  __syncthreads();
  for (int x = threadIdx.x; x < D; x += 256) {
    const double val = sign * v[x];
    v[x] = val;
    const int h = x / d, xx = x - h * d;
    kv_store_elem<EB>(Bout, (((size_t)b * hkv + h) * r + rho) * d + xx, val);
  }
}

// ---- 3. A = K Psi -----------------------------------------------------------------------------------------
// One wave per (48 tokens, up to 80 rank columns, sequence): M = tokens (three 16-row tiles), N = rank index,
// contraction over the key columns (a lane's four consecutive stored elements are four contraction steps).  Every fragment of Psi read from L2 serves the three token tiles (120 accumulator registers: a fourth
// tile makes the compiler move accumulators in and out of the matrix register file every step).
template <int EB>
__global__ __launch_bounds__(64) void project_kernel(const void* __restrict__ K, const double* __restrict__ Psi_t,
                                                     void* __restrict__ Aout, int s, int s_cap, int D, int r) {
  constexpr int NT = 5, MT = 3;
  const int lane = threadIdx.x, mrow = lane & 15, kq = lane >> 4;
  const int tok0 = blockIdx.x * (16 * MT), n0 = blockIdx.y * (16 * NT), b = blockIdx.z;
  size_t krow[MT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) krow[mt] = ((size_t)b * s + min(tok0 + 16 * mt + mrow, s - 1)) * D;
  f64x4 acc[MT][NT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) acc[mt][nt] = f64x4{0.0, 0.0, 0.0, 0.0};
  const double* prow[NT];
  bool okn[NT];
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) {
    const int rho = n0 + 16 * nt + mrow;
    okn[nt] = rho < r;
    prow[nt] = Psi_t + ((size_t)b * r + min(rho, r - 1)) * D;
  }
  // The contraction runs over 64 key columns per outer step: lane group kq owns columns c0 + 16 kq .. + 15 (one
  // 32-byte piece of each of its token rows, requested a whole outer step ahead: it comes from HBM) and takes them
  // four at a time; the Psi fragments of the next inner step (from L2) are requested before the matrix
  // instructions of the current one.
  Raw16<EB> kn[MT];
  double pn[NT][4];
  auto request_k = [&](int c0) {
    const int col = c0 + 16 * kq;
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) kn[mt].load(K, krow[mt] + col, col < D);
  };
  auto request_psi = [&](int col) {   // col = first of this lane group's four columns
    const bool ok = col < D;
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
      double2 lo = make_double2(0.0, 0.0), hi = make_double2(0.0, 0.0);
      if (okn[nt] && ok) {
        lo = *reinterpret_cast<const double2*>(prow[nt] + col);
        hi = *reinterpret_cast<const double2*>(prow[nt] + col + 2);
      }
      pn[nt][0] = lo.x; pn[nt][1] = lo.y; pn[nt][2] = hi.x; pn[nt][3] = hi.y;
    }
  };
  request_k(0);
  request_psi(16 * kq);
#pragma unroll 1
  for (int c0 = 0; c0 < D; c0 += 64) {
    Raw16<EB> kc[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) kc[mt] = kn[mt];
    request_k(c0 + 64);
    auto inner = [&](auto u_tag, int next_col) {
      constexpr int U = decltype(u_tag)::value;
      double a[MT][4], pb[NT][4];
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) kc[mt].template widen4<U>(a[mt]);
#pragma unroll
      for (int nt = 0; nt < NT; ++nt)
#pragma unroll
        for (int e = 0; e < 4; ++e) pb[nt][e] = pn[nt][e];
      request_psi(next_col);
#pragma unroll
      for (int nt = 0; nt < NT; ++nt)
#pragma unroll
        for (int e = 0; e < 4; ++e)
#pragma unroll
          for (int mt = 0; mt < MT; ++mt)
            acc[mt][nt] = __builtin_amdgcn_mfma_f64_16x16x4f64(a[mt][e], pb[nt][e], acc[mt][nt], 0, 0, 0);
    };
    const int cb = c0 + 16 * kq;
    inner(std::integral_constant<int, 0>{}, cb + 4);
    inner(std::integral_constant<int, 1>{}, cb + 8);
    inner(std::integral_constant<int, 2>{}, cb + 12);
    inner(std::integral_constant<int, 3>{}, cb + 64);
  }
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int t = tok0 + 16 * mt + 4 * j + kq, rho = n0 + 16 * nt + mrow;
        if (t < s && rho < r) kv_store_elem<EB>(Aout, ((size_t)b * s_cap + t) * r + rho, acc[mt][nt][j]);
      }
}

// ---- launch sequence ----------------------------------------------------------------------------------------
static hipError_t dgemm(const double* A, const double* B, double* C, int M, int N, int Kd, long sai, long sak, long sbk,
                        long sbj, int ldc, long strideA, long strideB, long strideC, int batch, hipStream_t st) {
  dim3 grid((N + 63) / 64, (M + 63) / 64, batch);
  hipLaunchKernelGGL(dgemm_kernel, grid, dim3(256), 0, st, A, B, C, M, N, Kd, sai, sak, sbk, sbj, ldc, strideA, strideB,
                     strideC);
  return hipGetLastError();
}

FactorizePlan plan_factorize(int batch, int s, int D, int r, int oversample) {
  FactorizePlan p{};
  p.m = std::min(D, r + oversample);
  p.mp = (p.m + 1) & ~1;
  p.nb = (D + 63) / 64;
  const long pairs = (long)p.nb * (p.nb + 1) / 2;
  // enough waves to fill the chip: split the tokens when there are few column-block pairs
  // tuning override: waves aimed at (default 8192; 16384 gains 5 % at the price of twice the partial sums)
  static const long target = [] { const char* e = getenv("SHADOWKV_GRAM_WAVES"); return e ? atol(e) : 8192l; }();
  long splits = (target + pairs * batch - 1) / (pairs * batch);
  const long max_splits = (s + 1023) / 1024;
  if (splits > max_splits) splits = max_splits;
  if (splits < 1) splits = 1;
  p.tokens_per_split = (int)(((s + splits - 1) / splits + 15) / 16 * 16);
  p.n_splits = (s + p.tokens_per_split - 1) / p.tokens_per_split;
  size_t off = 0;
  auto up = [](size_t x) { return (x + 255) / 256 * 256; };
  const size_t DD = (size_t)D * D;
  p.part = off; off += up((size_t)p.n_splits * batch * DD * 8);
  p.G = off; off += up((size_t)batch * DD * 8);
  p.Xt = off; off += up((size_t)batch * p.m * D * 8);
  p.Yt = off; off += up((size_t)batch * p.m * D * 8);
  p.W = off; off += up((size_t)batch * p.mp * p.mp * 8);
  p.V = off; off += up((size_t)batch * p.mp * p.mp * 8);
  p.Wsel = off; off += up((size_t)batch * r * p.m * 8);
  p.Psi_t = off; off += up((size_t)batch * r * D * 8);
  p.total = off;
  return p;
}

hipError_t launch_factorize(const void* k_pre, int kv_bytes, void* A, void* B, double* psi_out, double* sigma_out,
                            char* ws, const FactorizePlan& pl, int batch, int hkv, int d, int s, int s_cap, int r,
                            int n_iter, int n_sweeps, hipStream_t st) {
  const int D = hkv * d, m = pl.m, mp = pl.mp;
  double* part = reinterpret_cast<double*>(ws + pl.part);
  double* G = reinterpret_cast<double*>(ws + pl.G);
  double* Xt = reinterpret_cast<double*>(ws + pl.Xt);
  double* Yt = reinterpret_cast<double*>(ws + pl.Yt);
  double* W = reinterpret_cast<double*>(ws + pl.W);
  double* V = reinterpret_cast<double*>(ws + pl.V);
  double* Wsel = reinterpret_cast<double*>(ws + pl.Wsel);
  double* Psi_t = psi_out ? psi_out : reinterpret_cast<double*>(ws + pl.Psi_t);
  hipError_t e;
#define SKV_CHECK() do { e = hipGetLastError(); if (e != hipSuccess) return e; } while (0)
  // 1. G = K^T K
  {
    dim3 grid(pl.nb * (pl.nb + 1) / 2, pl.n_splits, batch);
    if (kv_bytes == 1) hipLaunchKernelGGL(gram_kernel<1>, grid, dim3(64), 0, st, k_pre, part, s, D, pl.nb, pl.tokens_per_split, batch);
    else hipLaunchKernelGGL(gram_kernel<2>, grid, dim3(64), 0, st, k_pre, part, s, D, pl.nb, pl.tokens_per_split, batch);
    SKV_CHECK();
    hipLaunchKernelGGL(gram_finish_kernel, dim3((unsigned)(((size_t)D * D + 255) / 256), batch), dim3(256), 0, st, part, G, D,
                       pl.n_splits, batch);
    SKV_CHECK();
  }
  // 2. subspace iteration: X <- orth(G X); rows of Xt are the vectors
  const size_t nx = (size_t)batch * m * D;
  hipLaunchKernelGGL(subspace_init_kernel, dim3((unsigned)((nx + 255) / 256)), dim3(256), 0, st, Xt, nx);
  SKV_CHECK();
  auto orthonormalise = [&](double* X) -> hipError_t {
    hipError_t err = hipSuccess;
    if (D <= 1024) {          // groups of 8 vectors, 4 elements per thread
      for (int j = 0; j < m && err == hipSuccess; j += 8) {
        const int q = std::min(8, m - j);
        hipLaunchKernelGGL((mgs_pivots_kernel<8, 4>), dim3(batch), dim3(256), 0, st, X, D, m, j, q);
        if (j + q < m) hipLaunchKernelGGL((mgs_project_kernel<8, 4>), dim3(m - j - q, batch), dim3(256), 0, st, X, D, m, j, q);
        err = hipGetLastError();
      }
    } else if (D <= 3072) {   // groups of 4 vectors, 12 elements per thread
      for (int j = 0; j < m && err == hipSuccess; j += 4) {
        const int q = std::min(4, m - j);
        hipLaunchKernelGGL((mgs_pivots_kernel<4, 12>), dim3(batch), dim3(256), 0, st, X, D, m, j, q);
        if (j + q < m) hipLaunchKernelGGL((mgs_project_kernel<4, 12>), dim3(m - j - q, batch), dim3(256), 0, st, X, D, m, j, q);
        err = hipGetLastError();
      }
    } else {
      for (int j = 0; j + 1 < m && err == hipSuccess; ++j) {
        hipLaunchKernelGGL(mgs_step_kernel, dim3(m - 1 - j, batch), dim3(256), 0, st, X, D, m, j);
        err = hipGetLastError();
      }
    }
    if (err != hipSuccess) return err;
    hipLaunchKernelGGL(normalize_rows_kernel, dim3(batch * m), dim3(256), 0, st, X, D);
    return hipGetLastError();
  };
  if ((e = orthonormalise(Xt)) != hipSuccess) return e;
  for (int it = 0; it < n_iter; ++it) {
    // Yt [m x D] = Xt [m x D] G [D x D]   (G is symmetric)
    if ((e = dgemm(Xt, G, Yt, m, D, D, D, 1, D, 1, D, (long)m * D, (long)D * D, (long)m * D, batch, st)) != hipSuccess) return e;
    // every second product only: two products square the condition number of the basis (~1e8 at most for the
    // spectra this is meant for), which modified Gram-Schmidt still handles; the last basis is done twice
    if (((it & 1) || it + 1 == n_iter) && (e = orthonormalise(Yt)) != hipSuccess) return e;
    if (it + 1 == n_iter && (e = orthonormalise(Yt)) != hipSuccess) return e;  // once more before the Ritz step
    double* tmp = Xt; Xt = Yt; Yt = tmp;
  }
  // Rayleigh-Ritz: T = X^T G X = Xt (Xt G)^T
  if ((e = dgemm(Xt, G, Yt, m, D, D, D, 1, D, 1, D, (long)m * D, (long)D * D, (long)m * D, batch, st)) != hipSuccess) return e;
  {
    // W [mp x mp] = 0 outside the leading m x m block
    const size_t nw = (size_t)batch * mp * mp;
    e = launch_fill_i32(reinterpret_cast<int32_t*>(W), nw * 2, 0, st);
    if (e != hipSuccess) return e;
    // T(i, j) = sum_x Xt[i][x] Yt[j][x]
    if ((e = dgemm(Xt, Yt, W, m, m, D, D, 1, 1, D, mp, (long)m * D, (long)m * D, (long)mp * mp, batch, st)) != hipSuccess) return e;
    hipLaunchKernelGGL(identity_kernel, dim3((unsigned)(((size_t)mp * mp + 255) / 256), batch), dim3(256), 0, st, V, mp);
    SKV_CHECK();
    for (int sw = 0; sw < n_sweeps; ++sw)
      for (int stp = 0; stp < mp - 1; ++stp) {
        hipLaunchKernelGGL(jacobi_step_kernel, dim3(mp / 2, batch), dim3(64), 0, st, W, V, mp, stp);
        SKV_CHECK();
      }
    hipLaunchKernelGGL(ritz_select_kernel, dim3(batch), dim3(256), (size_t)mp * sizeof(double), st, W, V, Wsel, sigma_out, mp,
                       m, r);
    SKV_CHECK();
  }
  // Psi_t [r x D] = Wsel [r x m] Xt [m x D]
  if ((e = dgemm(Wsel, Xt, Psi_t, r, D, m, m, 1, D, 1, D, (long)r * m, (long)m * D, (long)r * D, batch, st)) != hipSuccess) return e;
  // 3. sign convention, B, A = K Psi
  if (kv_bytes == 1) hipLaunchKernelGGL(emit_b_kernel<1>, dim3(r, batch), dim3(256), 0, st, Psi_t, B, D, r, hkv, d);
  else hipLaunchKernelGGL(emit_b_kernel<2>, dim3(r, batch), dim3(256), 0, st, Psi_t, B, D, r, hkv, d);
  SKV_CHECK();
  {
    dim3 grid((s + 47) / 48, (r + 79) / 80, batch);
    if (kv_bytes == 1) hipLaunchKernelGGL(project_kernel<1>, grid, dim3(64), 0, st, k_pre, Psi_t, A, s, s_cap, D, r);
    else hipLaunchKernelGGL(project_kernel<2>, grid, dim3(64), 0, st, k_pre, Psi_t, A, s, s_cap, D, r);
    SKV_CHECK();
  }
#undef SKV_CHECK
  return hipSuccess;
}

}  // namespace skv
