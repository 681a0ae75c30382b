/*
 * ShadowKV CPU oracle -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.
 *
 * A plain, slow, obviously-correct implementation of the operations the GPU
 * library exports: landmark/outlier construction (pre-filling algorithm,
 * Alg. 1 of the paper, every step after the SVD), one sparse decode step
 * (decoding algorithm, Alg. 2, followed by the standard attention over the
 * selected set described in the "Theoretical Equivalent Bandwidth" section),
 * the bookkeeping of the chunk cache of offloaded values and the append of a
 * chunk of generated tokens (both from section "High-throughput Decoding").
 *
 * Rules this file keeps:
 *   - it shares nothing with the HIP path (no header, no helper, no table);
 *   - inputs are the same bit patterns the GPU gets (bf16, or FP8 E5M2 bytes for
 *     the KV-cache tensors in the FP8 storage mode), widened exactly to
 *     fp64; every sum, norm, exponential and angle is fp64; nothing is rounded
 *     on the way to the bf16 outputs (round-to-nearest-even from fp64);
 *   - the steps run in the paper's order with its notation, no blocking and
 *     no fusion, so it can be checked against the paper by eye;
 *   - only tests, the smoke check and the benchmark's cpu_baseline leg may
 *     build or call it.
 *
 * Pins (tests/test_oracle_*.py): brute-force re-implementation on tiny
 * shapes, dense softmax attention when the budget covers every chunk, exact
 * reconstruction at full rank, RoPE group identities, chunk-size-1 reduction
 * to token top-k, closed forms for the cosine criterion; for the cache model
 * hand-worked cases, an independent simulation and its invariants; for the
 * append exact projection inside the subspace and "append == longer
 * prefill"; for the FP8 storage mode the format's definition in exact fractions,
 * a brute-force nearest-code search, a library's own E5M2 type, and bit equality
 * with the bf16 mode on widened inputs; planted mistakes (mutants) must fail
 * these pins.  What is NOT pinned
 * anywhere ("parity unpinned"): how well the method approximates dense
 * attention on a trained model -- that needs weights and evaluation suites.
 *
 * Notation (paper): b batch, h_q / h_kv query / key-value heads, G = h_q/h_kv,
 * d head dim, s chunked context length, c chunk size, n_ch = s/c, o outlier
 * chunks, n_c = n_ch - o landmarks, k selected chunks, w resident recent
 * tokens, r rank.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef struct oracle_params {
  int32_t batch, n_q_heads, n_kv_heads, head_dim;
  int32_t ctx_len, chunk_size, rank;
  int32_t n_outlier_chunks, topk_chunks, local_len;
  double rope_theta;      /* base of the rotary frequencies */
  const float *inv_freq;  /* optional [d/2]; replaces theta^(-2i/d) */
  double softmax_scale;   /* 0 => 1/sqrt(d) */
  int32_t ctx_capacity;   /* tokens the context arrays are laid out for (0 => ctx_len); see below */
  int32_t kv_dtype;       /* storage type of the KV-cache tensors: 0 = bf16, 1 = FP8 E5M2; see below */
} oracle_params;

/* Room to grow (generated tokens are appended chunk by chunk, oracle_append_chunk): the arrays that
 * have a token or landmark axis are laid out for `cap` = ctx_capacity tokens --
 * A [b, cap, r], value_store [b, h_kv, cap, d], landmarks [b, h_kv, cap/c - o, d],
 * landmark_chunk_ids [b, h_kv, cap/c - o] -- and only the first ctx_len tokens (n_c landmarks)
 * of each are valid. */
static int64_t capacity_of(const oracle_params *p) {
  return p->ctx_capacity > 0 ? p->ctx_capacity : p->ctx_len;
}

int oracle_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

/* ---- bf16 <-> fp64 ------------------------------------------------------ */

static double bf16_to_f64(uint16_t h) {
  uint32_t u = (uint32_t)h << 16;
  float f;
  memcpy(&f, &u, sizeof f);
  return (double)f;
}

/* Round an fp64 value to the nearest bf16 (ties to even) in ONE rounding. */
uint16_t oracle_f64_to_bf16(double x) {
  if (isnan(x)) return 0x7fc0;
  uint16_t sign = signbit(x) ? 0x8000 : 0;
  double a = fabs(x);
  if (a == 0.0) return sign;
  if (isinf(a)) return sign | 0x7f80;
  int e;
  (void)frexp(a, &e); /* a = m * 2^e, m in [0.5, 1) => floor(log2 a) = e-1 */
  int E = e - 1;
  if (E < -126) E = -126;              /* subnormal range: fixed spacing */
  double ulp = ldexp(1.0, E - 7);      /* bf16 keeps 7 fraction bits */
  double q = nearbyint(a / ulp);       /* default mode: ties to even */
  double r = q * ulp;                  /* exactly representable in fp32 */
  float f = (float)r;
  if (isinf(f)) return sign | 0x7f80;
  uint32_t u;
  memcpy(&u, &f, sizeof u);
  return sign | (uint16_t)(u >> 16);
}

/* ---- FP8 (E5M2) storage of the KV cache ----------------------------------
 * Section "Precision Sensitivity": besides bf16 the paper runs the method with the
 * KV cache held in FP8, the E5M2 format: one byte per element -- sign, 5 exponent
 * bits (bias 15), 2 fraction bits, with subnormals, infinities and NaNs as in
 * IEEE 754.  The reading taken: with kv_dtype = 1 every tensor that is KV-cache
 * state (A, B, landmarks, outlier and recent K,V, the value store, and the keys and
 * values handed to the pre-filling step and to the append) holds such bytes; the
 * query and the attention output are activations and stay bf16.  The arithmetic
 * does not change: stored elements are widened exactly to fp64, and what the
 * method stores itself (landmarks, low-rank states of generated tokens) is rounded
 * once, to nearest-even, from the fp64 value; beyond the largest finite value
 * (57344) that rounding gives infinity, as IEEE 754 does.                      */
double oracle_e5m2_to_f64(uint8_t v) {
  const int sign = v >> 7, e = (v >> 2) & 31, m = v & 3;
  double a;
  if (e == 31) a = m ? NAN : INFINITY;
  else if (e == 0) a = ldexp((double)m, -16);            /* subnormal: m/4 * 2^-14 */
  else a = ldexp(1.0 + (double)m / 4.0, e - 15);
  return sign ? -a : a;
}

uint8_t oracle_f64_to_e5m2(double x) {
  if (isnan(x)) return 0x7f;
  const uint8_t sign = signbit(x) ? 0x80 : 0;
  const double a = fabs(x);
  if (a == 0.0) return sign;
  if (isinf(a)) return sign | 0x7c;
  int e;
  (void)frexp(a, &e);
  int E = e - 1;                       /* floor(log2 a) */
  if (E < -14) E = -14;                /* subnormal range: fixed spacing 2^-16 */
  const double ulp = ldexp(1.0, E - 2);  /* 2 fraction bits */
  const double r = nearbyint(a / ulp) * ulp; /* ties to even; may carry into the next binade */
  if (r > 57344.0) return sign | 0x7c;
  if (r < ldexp(1.0, -14)) return sign | (uint8_t)(r / ldexp(1.0, -16));
  int er;
  const double fr = frexp(r, &er);     /* r = fr * 2^er, fr in [0.5, 1) */
  const int m = (int)((fr * 2.0 - 1.0) * 4.0);
  return sign | (uint8_t)(((er - 1 + 15) << 2) | m);
}

/* element i of a KV-cache tensor, widened exactly; bytes per element; store with one rounding */
static double kv_get(const oracle_params *p, const void *base, int64_t i) {
  return p->kv_dtype == 1 ? oracle_e5m2_to_f64(((const uint8_t *)base)[i]) : bf16_to_f64(((const uint16_t *)base)[i]);
}
static size_t kv_size(const oracle_params *p) { return p->kv_dtype == 1 ? 1 : 2; }
static void kv_put(const oracle_params *p, void *base, int64_t i, double x) {
  if (p->kv_dtype == 1) ((uint8_t *)base)[i] = oracle_f64_to_e5m2(x);
  else ((uint16_t *)base)[i] = oracle_f64_to_bf16(x);
}
static void kv_copy(const oracle_params *p, void *dst, int64_t di, const void *src, int64_t si, int64_t n) {
  memcpy((char *)dst + di * kv_size(p), (const char *)src + si * kv_size(p), (size_t)n * kv_size(p));
}

/* ---- rotary position embedding ------------------------------------------
 * Rotate-half pairing over the full head dimension: coordinate i < d/2 is
 * paired with i + d/2, frequency theta^(-2i/d), angle = position * frequency
 * (the RoPE the decoding algorithm applies to the rebuilt keys).            */
static double rope_freq(const oracle_params *p, int i) {
  if (p->inv_freq) return (double)p->inv_freq[i];
  return pow(p->rope_theta, -2.0 * (double)i / (double)p->head_dim);
}

static void rope_inplace(const oracle_params *p, double *x, double pos) {
  int half = p->head_dim / 2;
  for (int i = 0; i < half; ++i) {
    double phi = pos * rope_freq(p, i);
    double cs = cos(phi), sn = sin(phi);
    double x0 = x[i], x1 = x[i + half];
    x[i] = x0 * cs - x1 * sn;
    x[i + half] = x1 * cs + x0 * sn;
  }
}

/* Exposed for the identity tests: y[n,:] = RoPE(x[n,:], pos[n]). */
void oracle_rope(const oracle_params *p, const double *x, const double *pos,
                 int64_t n_rows, double *y) {
  int d = p->head_dim;
  for (int64_t n = 0; n < n_rows; ++n) {
    memcpy(y + n * d, x + n * d, sizeof(double) * d);
    rope_inplace(p, y + n * d, pos[n]);
  }
}

/* ---- ArgTopK with the lower-index-wins tie rule ------------------------- */
typedef struct { double key; int32_t idx; } keyed;

static int cmp_desc(const void *a, const void *b) {
  const keyed *x = a, *y = b;
  if (x->key > y->key) return -1;
  if (x->key < y->key) return 1;
  return (x->idx > y->idx) - (x->idx < y->idx);
}

/* ---- Alg. 1 (after the SVD line): landmarks and outliers ----------------
 * k_rope [b, h_kv, s, d] bf16 (the prefill keys, dense); v = the value store
 * [b, h_kv, cap, d].  Outputs per (b, h_kv):
 *   landmarks [n_c, d] bf16, landmark_chunk_ids [n_c] ascending,
 *   outlier_chunk_ids [o] most-outlying first, k_outlier/v_outlier [o*c, d].
 * Optional fp64 diagnostics: chunk_min_cos [b,h_kv,n_ch], chunk_mean
 * [b,h_kv,n_ch,d] (pass NULL to skip).  v / v_outlier may be NULL.         */
int oracle_build_landmarks(const oracle_params *p, const void *k_rope,
                           const void *v, void *landmarks,
                           int32_t *landmark_chunk_ids,
                           int32_t *outlier_chunk_ids, void *k_outlier,
                           void *v_outlier, double *chunk_min_cos,
                           double *chunk_mean) {
  const int d = p->head_dim, c = p->chunk_size, o = p->n_outlier_chunks;
  const int64_t s = p->ctx_len;
  if (d <= 0 || c <= 0 || s % c) return -1;
  const int64_t n_ch = s / c, n_c = n_ch - o;
  if (o < 0 || n_c < 0) return -1;
  const int64_t cap = capacity_of(p);
  if (cap < s || cap % c) return -1;
  const int64_t nc_cap = cap / c - o; /* landmark rows the arrays are laid out for */
  const int64_t units = (int64_t)p->batch * p->n_kv_heads;
  const double eps = 1e-8;
  int fail = 0;

#pragma omp parallel for schedule(dynamic, 1)
  for (int64_t u = 0; u < units; ++u) {
    const int64_t K0 = u * s * d;  /* first element of this unit's keys */
    double *C = malloc(sizeof(double) * n_ch * d);      /* chunk means */
    keyed *m = malloc(sizeof(keyed) * (n_ch ? n_ch : 1)); /* -min cos   */
    char *is_out = calloc(n_ch ? n_ch : 1, 1);
    if (!C || !m || !is_out) {
      fail = 1; free(C); free(m); free(is_out); continue;
    }
    /* C <- Reduce(K^RoPE): mean over the c tokens of each chunk */
    for (int64_t j = 0; j < n_ch; ++j)
      for (int x = 0; x < d; ++x) {
        double acc = 0.0;
        for (int t = 0; t < c; ++t) acc += kv_get(p, k_rope, K0 + (j * c + t) * d + x);
        C[j * d + x] = acc / (double)c;
      }
    /* S <- CosineSimilarity(C, K^RoPE); Min over the chunk's tokens */
    for (int64_t j = 0; j < n_ch; ++j) {
      double cn = 0.0;
      for (int x = 0; x < d; ++x) cn += C[j * d + x] * C[j * d + x];
      cn = sqrt(cn);
      double mn = INFINITY;
      for (int t = 0; t < c; ++t) {
        double dot = 0.0, kn = 0.0;
        for (int x = 0; x < d; ++x) {
          double kv = kv_get(p, k_rope, K0 + (j * c + t) * d + x);
          dot += C[j * d + x] * kv;
          kn += kv * kv;
        }
        kn = sqrt(kn);
        double cs = dot / (fmax(cn, eps) * fmax(kn, eps));
        if (cs < mn) mn = cs;
      }
      m[j].key = -mn; /* ArgTopK(-Min(S), o) */
      m[j].idx = (int32_t)j;
      if (chunk_min_cos) chunk_min_cos[u * n_ch + j] = mn;
    }
    if (chunk_mean) memcpy(chunk_mean + u * n_ch * d, C, sizeof(double) * n_ch * d);
    qsort(m, n_ch, sizeof(keyed), cmp_desc);
    /* Gather the outlier chunks' exact keys and values */
    for (int i = 0; i < o; ++i) {
      int64_t j = m[i].idx;
      is_out[j] = 1;
      outlier_chunk_ids[u * o + i] = (int32_t)j;
      kv_copy(p, k_outlier, (u * o + i) * c * d, k_rope, K0 + j * c * d, (int64_t)c * d);
      if (v && v_outlier)
        kv_copy(p, v_outlier, (u * o + i) * c * d, v, (u * cap + j * c) * d, (int64_t)c * d);
    }
    /* L <- C without the outlier rows, in ascending chunk order */
    int64_t slot = 0;
    for (int64_t j = 0; j < n_ch; ++j) {
      if (is_out[j]) continue;
      landmark_chunk_ids[u * nc_cap + slot] = (int32_t)j;
      for (int x = 0; x < d; ++x)
        kv_put(p, landmarks, (u * nc_cap + slot) * d + x, C[j * d + x]);
      ++slot;
    }
    free(C); free(m); free(is_out);
  }
  return fail ? -2 : 0;
}

/* ---- Alg. 2 + sparse attention: one decode step -------------------------
 * q [b,h_q,d]; A [b,cap,r]; B [b,h_kv,r,d]; landmarks [b,h_kv,cap/c-o,d];
 * landmark_chunk_ids [b,h_kv,cap/c-o]; k_outlier/v_outlier [b,h_kv,o*c,d];
 * k_local/v_local [b,h_kv,w,d]; value_store [b,h_kv,cap,d]; pos_offset [b] or
 * NULL.  All bf16 except ids.  Outputs: out_bf16 [b,h_q,d]; optional:
 * out_f64 [b,h_q,d], chunk_ids [b,h_kv,k] (true chunk ids, best first),
 * z2 [b,h_kv,n_c] (log-domain group score per landmark slot),
 * k_sparse [b,h_kv,k*c,d] fp64 (rebuilt, rotated keys in chunk_ids order).   */
int oracle_decode_step(const oracle_params *p, const uint16_t *q,
                       const void *A, const void *B,
                       const void *landmarks,
                       const int32_t *landmark_chunk_ids,
                       const void *k_outlier, const void *v_outlier,
                       const void *k_local, const void *v_local,
                       const void *value_store, const int32_t *pos_offset,
                       uint16_t *out_bf16, double *out_f64, int32_t *chunk_ids,
                       double *z2_out, double *k_sparse_out) {
  const int d = p->head_dim, c = p->chunk_size, r = p->rank;
  const int o = p->n_outlier_chunks, k = p->topk_chunks, w = p->local_len;
  const int hq = p->n_q_heads, hkv = p->n_kv_heads;
  const int64_t s = p->ctx_len;
  if (d <= 0 || (d & 1) || c <= 0 || s % c || hkv <= 0 || hq % hkv) return -1;
  const int G = hq / hkv;
  const int64_t n_ch = s / c, n_c = n_ch - o;
  if (k < 0 || k > n_c) return -1;
  const int64_t cap = capacity_of(p);
  if (cap < s || cap % c) return -1;
  const int64_t nc_cap = cap / c - o;
  const int64_t T = (int64_t)o * c + (int64_t)k * c + w;
  const double scale = p->softmax_scale != 0.0 ? p->softmax_scale : 1.0 / sqrt((double)d);
  const int64_t units = (int64_t)p->batch * hkv;
  int fail = 0;

#pragma omp parallel for schedule(dynamic, 1)
  for (int64_t u = 0; u < units; ++u) {
    const int64_t bi = u / hkv, h = u % hkv;
    const int64_t L0 = u * nc_cap * d; /* first element of this unit's landmarks */
    const int32_t *Lid = landmark_chunk_ids + u * nc_cap;
    double *P = malloc(sizeof(double) * (size_t)G * (n_c ? n_c : 1));
    keyed *z2 = malloc(sizeof(keyed) * (n_c ? n_c : 1));
    double *Kt = malloc(sizeof(double) * (T ? T : 1) * d); /* attended keys   */
    double *Vt = malloc(sizeof(double) * (T ? T : 1) * d); /* attended values */
    double *a = malloc(sizeof(double) * (T ? T : 1));
    if (!P || !z2 || !Kt || !Vt || !a) {
      fail = 1; free(P); free(z2); free(Kt); free(Vt); free(a); continue;
    }
    /* P <- Q L^T, scaled by 1/sqrt(d); S <- Softmax over the landmarks.
     * Kept in the log domain: log S = P - logsumexp(P) per query head.
     * (The sum over the s_q query positions is the identity for s_q = 1.) */
    for (int g = 0; g < G; ++g) {
      const uint16_t *qg = q + (bi * hq + h * G + g) * d;
      double mx = -INFINITY;
      for (int64_t j = 0; j < n_c; ++j) {
        double dot = 0.0;
        for (int x = 0; x < d; ++x) dot += bf16_to_f64(qg[x]) * kv_get(p, landmarks, L0 + j * d + x);
        P[g * n_c + j] = dot * scale;
        if (P[g * n_c + j] > mx) mx = P[g * n_c + j];
      }
      double se = 0.0;
      for (int64_t j = 0; j < n_c; ++j) se += exp(P[g * n_c + j] - mx);
      double lse = mx + log(se);
      for (int64_t j = 0; j < n_c; ++j) P[g * n_c + j] -= lse;
    }
    /* S2 <- max over the query heads of the KV group */
    for (int64_t j = 0; j < n_c; ++j) {
      double best = -INFINITY;
      for (int g = 0; g < G; ++g)
        if (P[g * n_c + j] > best) best = P[g * n_c + j];
      z2[j].key = best;
      z2[j].idx = (int32_t)j;
      if (z2_out) z2_out[u * n_c + j] = best;
    }
    /* I <- ArgTopK(S2, k): landmark slots; ties go to the lower slot */
    qsort(z2, n_c, sizeof(keyed), cmp_desc);

    /* K <- [K_outlier ; RoPE(Gather(A, I) B) ; K_new],
     * V <- [V_outlier ; Gather(V_store, I) ; V_new]                       */
    int64_t row = 0;
    for (int64_t i = 0; i < (int64_t)o * c; ++i, ++row)
      for (int x = 0; x < d; ++x) {
        Kt[row * d + x] = kv_get(p, k_outlier, (u * o * c + i) * d + x);
        Vt[row * d + x] = kv_get(p, v_outlier, (u * o * c + i) * d + x);
      }
    const double pos0 = pos_offset ? (double)pos_offset[bi] : 0.0;
    for (int i = 0; i < k; ++i) {
      const int64_t ch = Lid[z2[i].idx];
      if (chunk_ids) chunk_ids[u * k + i] = (int32_t)ch;
      for (int t = 0; t < c; ++t, ++row) {
        const int64_t n = ch * c + t; /* token index inside the context */
        const int64_t Arow = (bi * cap + n) * r; /* first element of the token's row of A */
        for (int x = 0; x < d; ++x) {
          double acc = 0.0;
          for (int rho = 0; rho < r; ++rho)
            acc += kv_get(p, A, Arow + rho) * kv_get(p, B, ((u * r) + rho) * d + x);
          Kt[row * d + x] = acc;
        }
        rope_inplace(p, Kt + row * d, pos0 + (double)n);
        if (k_sparse_out)
          memcpy(k_sparse_out + ((u * k + i) * c + t) * d, Kt + row * d, sizeof(double) * d);
        for (int x = 0; x < d; ++x)
          Vt[row * d + x] = kv_get(p, value_store, (u * cap + n) * d + x);
      }
    }
    for (int64_t i = 0; i < w; ++i, ++row)
      for (int x = 0; x < d; ++x) {
        Kt[row * d + x] = kv_get(p, k_local, (u * w + i) * d + x);
        Vt[row * d + x] = kv_get(p, v_local, (u * w + i) * d + x);
      }

    /* standard softmax attention of each query head of the group over K, V */
    for (int g = 0; g < G; ++g) {
      const uint16_t *qg = q + (bi * hq + h * G + g) * d;
      double mx = -INFINITY;
      for (int64_t i = 0; i < T; ++i) {
        double dot = 0.0;
        for (int x = 0; x < d; ++x) dot += bf16_to_f64(qg[x]) * Kt[i * d + x];
        a[i] = dot * scale;
        if (a[i] > mx) mx = a[i];
      }
      double se = 0.0;
      for (int64_t i = 0; i < T; ++i) { a[i] = exp(a[i] - mx); se += a[i]; }
      for (int x = 0; x < d; ++x) {
        double acc = 0.0;
        for (int64_t i = 0; i < T; ++i) acc += a[i] * Vt[i * d + x];
        double ov = T ? acc / se : 0.0;
        int64_t oi = (bi * hq + h * G + g) * d + x;
        if (out_f64) out_f64[oi] = ov;
        out_bf16[oi] = oracle_f64_to_bf16(ov);
      }
    }
    free(P); free(z2); free(Kt); free(Vt); free(a);
  }
  return fail ? -2 : 0;
}

/* ---- chunk cache of the offloaded values -------------------------------------
 * Section "High-throughput Decoding": the chunks selected by adjacent decode steps
 * repeat to a large part, so fetched values are kept, an index scan finds the
 * chunks that are missing, and only those are fetched (the (1 - alpha) term of the
 * equivalent-bandwidth formula).  The paper names "a cache policy" without fixing
 * one; the reading taken is least-recently-used over S >= k slots of one chunk
 * each per (batch, KV head) unit:
 *   - every step advances the unit's clock by one;
 *   - a selected chunk found in a slot is a hit: it stays there, stamped with the
 *     clock;
 *   - the n_miss selected chunks that are in no slot take the n_miss slots that
 *     were not hit and have the oldest stamps (empty slots are older than anything;
 *     equal stamps: lower slot first).  Among those slots the assignment is by
 *     order: missing chunks in ascending chunk id to slots in ascending index.
 * With S == k this keeps exactly the last step's selection.
 *
 * sel_ids    [units, k]  this step's selection, ascending, distinct
 * cache_ids  [units, S]  in/out: chunk id per slot, -1 = empty
 * stamps     [units, S+1] in/out: clock value of each slot's last use (0 = never),
 *                         entry S is the unit's clock
 * sel_slots  [units, k]  out: slot of every selected chunk after the step
 * miss_slots [units, k]  out: the slots that have to be filled, ascending (first n_miss[u]), rest -1
 * n_miss     [units]     out
 * The attention output does not depend on the cache at all: a cached step equals
 * oracle_decode_step. */
int oracle_cache_update(int64_t units, int k, int S, const int32_t *sel_ids,
                        int32_t *cache_ids, int32_t *stamps, int32_t *sel_slots,
                        int32_t *miss_slots, int32_t *n_miss) {
  if (units < 0 || k < 0 || S < k || !sel_ids || !cache_ids || !stamps || !sel_slots || !miss_slots || !n_miss)
    return -1;
  char *hit = (char *)malloc((size_t)k + 1), *keep = (char *)malloc((size_t)S + 1);
  char *victim = (char *)malloc((size_t)S + 1);
  if (!hit || !keep || !victim) { free(hit); free(keep); free(victim); return -2; }
  for (int64_t u = 0; u < units; ++u) {
    const int32_t *sel = sel_ids + u * k;
    int32_t *cache = cache_ids + u * S, *stamp = stamps + u * (S + 1);
    int32_t *ss = sel_slots + u * k, *ms = miss_slots + u * k;
    const int32_t clock = ++stamp[S];
    memset(hit, 0, (size_t)k);
    memset(keep, 0, (size_t)S);
    memset(victim, 0, (size_t)S);
    int n = k;
    for (int slot = 0; slot < S; ++slot)          /* the index scan */
      for (int j = 0; j < k; ++j)
        if (cache[slot] >= 0 && cache[slot] == sel[j] && !hit[j]) {
          hit[j] = 1; keep[slot] = 1; ss[j] = slot; stamp[slot] = clock; --n; break;
        }
    for (int i = 0; i < n; ++i) {                 /* the n least recently used of the other slots */
      int best = -1;
      for (int slot = 0; slot < S; ++slot) {
        if (keep[slot] || victim[slot]) continue;
        const int32_t a = cache[slot] < 0 ? -1 : stamp[slot];   /* empty: older than anything */
        const int32_t b = best < 0 ? 0 : (cache[best] < 0 ? -1 : stamp[best]);
        if (best < 0 || a < b) best = slot;
      }
      victim[best] = 1;
    }
    int slot = 0, m = 0;
    for (int j = 0; j < k; ++j) {
      if (hit[j]) continue;
      while (!victim[slot]) ++slot;
      cache[slot] = sel[j]; stamp[slot] = clock; ss[j] = slot;
      ms[m++] = slot++;
    }
    for (int j = m; j < k; ++j) ms[j] = -1;
    n_miss[u] = m;
  }
  free(hit); free(keep); free(victim);
  return 0;
}

/* ---- generated tokens: one more chunk of context --------------------------
 * Section "High-throughput Decoding", last paragraph and its footnote: new
 * pre-RoPE keys K' are stored as the low-rank states K' Psi, with Psi the right
 * singular matrix of the context keys, and projected back with Psi^T when needed.
 * Here Psi^T is B: Psi[(h, x), rho] = B[b, h, rho, x] over the full key width
 * h_kv * d.  When c tokens have left the recent-token window they become chunk
 * number n_ch = s / c of the context, exactly as if the pre-filling algorithm had
 * seen them: rows of A, one landmark (mean of the chunk's post-RoPE keys), the
 * chunk's values in the store.  The chunk is never an outlier (the outlier set
 * is fixed at pre-filling).
 *
 * k_pre  [b, c, h_kv*d]   pre-RoPE keys of the c tokens, heads side by side
 * k_rope [b, h_kv, c, d]  the same keys after RoPE at their positions
 * v      [b, h_kv, c, d]
 * in/out (laid out for cap tokens, valid up to s before / s + c after):
 * A, landmarks, landmark_chunk_ids, value_store.  Needs s + c <= cap.
 * The caller then continues with ctx_len = s + c.                          */
int oracle_append_chunk(const oracle_params *p, const void *k_pre,
                        const void *k_rope, const void *v,
                        const void *B, void *A, void *landmarks,
                        int32_t *landmark_chunk_ids, void *value_store) {
  const int d = p->head_dim, c = p->chunk_size, r = p->rank, o = p->n_outlier_chunks;
  const int hkv = p->n_kv_heads;
  const int64_t s = p->ctx_len, cap = capacity_of(p);
  if (d <= 0 || c <= 0 || s % c || cap % c || s + c > cap) return -1;
  const int64_t n_ch = s / c, n_c = n_ch - o, nc_cap = cap / c - o;
  if (n_c < 0) return -1;
  for (int64_t bi = 0; bi < p->batch; ++bi)
    for (int t = 0; t < c; ++t)
      for (int rho = 0; rho < r; ++rho) {       /* A' = K' Psi */
        double acc = 0.0;
        for (int h = 0; h < hkv; ++h)
          for (int x = 0; x < d; ++x)
            acc += kv_get(p, k_pre, ((bi * c + t) * hkv + h) * d + x) *
                   kv_get(p, B, (((bi * hkv + h) * r) + rho) * d + x);
        kv_put(p, A, (bi * cap + s + t) * r + rho, acc);
      }
  for (int64_t u = 0; u < (int64_t)p->batch * hkv; ++u) {
    for (int x = 0; x < d; ++x) {                /* landmark = mean of the chunk */
      double acc = 0.0;
      for (int t = 0; t < c; ++t) acc += kv_get(p, k_rope, (u * c + t) * d + x);
      kv_put(p, landmarks, (u * nc_cap + n_c) * d + x, acc / (double)c);
    }
    landmark_chunk_ids[u * nc_cap + n_c] = (int32_t)n_ch;
    kv_copy(p, value_store, (u * cap + s) * d, v, u * c * d, (int64_t)c * d);
  }
  return 0;
}
