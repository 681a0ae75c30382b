/*
 * libshadowkv -- ShadowKV decode hot path on one MI355X (gfx950), C ABI.
 *
 * Two main operations, both enqueue-only on caller-owned HIP streams (further down: the decode step
 * with a chunk cache of an offloaded value store, the append of generated tokens to the context, the
 * SVD line of the pre-filling algorithm, and the ArgTopK primitive on its own):
 *
 *   shadowkv_build_landmarks  pre-filling algorithm (Alg. 1) after its SVD
 *                             line: chunk means of the post-RoPE keys,
 *                             per-chunk minimum cosine between mean and keys,
 *                             the o lowest chunks become resident outliers,
 *                             the other chunk means become landmarks.
 *   shadowkv_decode_step      decoding algorithm (Alg. 2) plus the attention
 *                             over the selected set ("Theoretical Equivalent
 *                             Bandwidth" section): landmark scores, per-head
 *                             softmax, max over the GQA group, top-k chunks;
 *                             values of those chunks gathered, their keys
 *                             rebuilt from the rank-r factors and rotated at
 *                             their true positions; softmax attention over
 *                             [outliers ; selected chunks ; recent tokens].
 *
 * Notation (paper): b batch, h_q / h_kv query / KV heads, G = h_q / h_kv,
 * d head dim, s chunked context length, c chunk size, n_ch = s / c, o outlier
 * chunks, n_c = n_ch - o landmarks, k selected chunks, w recent tokens, r rank.
 *
 * Conventions for every pointer argument:
 *   - "dev"  = device (HBM) memory, "dev|pinned" = HBM or device-readable
 *     pinned host memory.  All tensors are dense, row-major in the layout
 *     written next to them, 16-byte aligned.  bf16 = raw 16-bit patterns;
 *     where a tensor is marked bf16 below and belongs to the KV cache it is
 *     E5M2 bytes instead when params->kv_dtype says so (see shadowkv_kv).
 *   - The caller owns every buffer (workspace included) and both streams.
 *     The library allocates no device memory; it keeps two HIP events per
 *     device for the side-stream fork/join, released by shadowkv_shutdown().
 *   - Calls return after enqueuing; outputs are valid once `stream` has been
 *     synchronised.  Work put on `side_stream` is joined back into `stream`
 *     before the call returns.
 *   - Return value: SHADOWKV_OK or a negative code.  Arguments are validated
 *     on the host before anything is enqueued, so a rejected call has no
 *     effect on the GPU (and can be exercised on a machine without one).
 */
#ifndef SHADOWKV_H
#define SHADOWKV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SHADOWKV_OK 0
#define SHADOWKV_EINVAL (-1)     /* bad shape, null pointer, unsupported size */
#define SHADOWKV_EWORKSPACE (-2) /* workspace missing, misaligned or too small */
#define SHADOWKV_EHIP (-3)       /* HIP runtime / launch error (see last_error) */

#define SHADOWKV_VALUES_DEVICE 0 /* value store in HBM: attention reads it in place */
#define SHADOWKV_VALUES_HOST 1   /* pinned host store: staged by a gather kernel   */

/* flags */
#define SHADOWKV_FLAG_STAGE_VALUES 1u      /* run the chunk gather even for an HBM store            */
#define SHADOWKV_FLAG_KEEP_REBUILT_KEYS 2u /* also write RoPE(Gather(A,I) B) to the workspace (tests) */

typedef uint16_t shadowkv_bf16;
/* Element of a KV-cache tensor (A, B, landmarks, outlier / recent K,V, value store, value cache, and the keys
 * and values handed to build_landmarks / append_chunk): bf16 (2 bytes) or FP8 E5M2 (1 byte), chosen for all of
 * them at once by params->kv_dtype.  Written "kv" next to the arguments below.  The query and the attention
 * output are activations and are always bf16. */
typedef void shadowkv_kv;

#define SHADOWKV_KV_BF16 0
#define SHADOWKV_KV_FP8_E5M2 1   /* section "Precision Sensitivity": sign, 5 exponent bits (bias 15), 2 fraction bits,
                                    subnormals / infinities / NaNs as in IEEE 754 (the upper byte of a half).  Stored
                                    elements are widened exactly; the arithmetic is the bf16 mode's; what the library
                                    stores itself (landmarks, low-rank states of appended tokens) is rounded once, to
                                    nearest-even, from the fp64 value, overflow to infinity. */

typedef struct shadowkv_params {
  int32_t batch;            /* b  >= 1 */
  int32_t n_q_heads;        /* h_q, multiple of n_kv_heads, G <= 64 */
  int32_t n_kv_heads;       /* h_kv >= 1 */
  int32_t head_dim;         /* d in {64, 96, 128} */
  int32_t ctx_len;          /* s: tokens covered by A / landmarks / value store; multiple of chunk_size */
  int32_t chunk_size;       /* c in [1, 64] */
  int32_t rank;             /* r: multiple of 8, 8 <= r <= 256 */
  int32_t n_outlier_chunks; /* o >= 0, o <= 1024 */
  int32_t topk_chunks;      /* k: 1 <= k <= n_c = s/c - o */
  int32_t local_len;        /* w >= 0 resident recent tokens (the current token included) */
  int32_t value_location;   /* SHADOWKV_VALUES_DEVICE | SHADOWKV_VALUES_HOST */
  uint32_t flags;           /* SHADOWKV_FLAG_* */
  double rope_theta;        /* RoPE base; frequency i is theta^(-2i/d), i < d/2, pairs (i, i + d/2) */
  double softmax_scale;     /* 0 => 1/sqrt(d); used for landmark scores and for attention */
  const float *inv_freq;    /* optional dev [d/2]: replaces theta^(-2i/d) (scaled-RoPE models) */
  int32_t ctx_capacity;     /* cap: tokens the context arrays are laid out for; 0 => ctx_len.  Multiple of
                               chunk_size, >= ctx_len.  Room for shadowkv_append_chunk to grow the context. */
  int32_t kv_dtype;         /* SHADOWKV_KV_BF16 | SHADOWKV_KV_FP8_E5M2: storage type of every "kv" tensor */
} shadowkv_params;

/*
 * Layout with room to grow.  The arrays that have a token or a landmark axis are laid out for
 * cap = ctx_capacity tokens (nc_cap = cap/c - o landmark rows), and only the first s = ctx_len tokens
 * (n_c landmark rows) of each unit are valid:
 *   A [b, cap, r]   value_store [b, h_kv, cap, d]   landmarks [b, h_kv, nc_cap, d]
 *   landmark_chunk_ids [b, h_kv, nc_cap]
 * With ctx_capacity == 0 these are the dense shapes written next to each argument below (s for cap,
 * n_c for nc_cap).  Everything else (k_rope of the prefill, outliers, recent tokens, outputs) is dense.
 */

/*
 * Alg. 1, every line after the SVD.  Per (batch, KV head):
 *   C_j   = mean of the c post-RoPE keys of chunk j            (fp64 accumulate)
 *   m_j   = min over the chunk's tokens of cos(C_j, key), each norm clamped at 1e-8
 *   outliers = the o chunks with the smallest m_j (ties: lower chunk id)
 *   landmarks = bf16(C_j) of the other chunks in ascending chunk order.
 *
 *   k_rope              dev        [b, h_kv, s, d] bf16   post-RoPE keys
 *   v                   dev|pinned [b, h_kv, s, d] bf16   the value store (laid out for cap tokens, see above);
 *                                                          may be NULL (then v_outlier is untouched)
 *   landmarks           dev  out   [b, h_kv, n_c, d] bf16
 *   landmark_chunk_ids  dev  out   [b, h_kv, n_c] int32   true chunk id of each landmark slot, ascending
 *   outlier_chunk_ids   dev  out   [b, h_kv, o] int32     ascending chunk id
 *   k_outlier,v_outlier dev  out   [b, h_kv, o*c, d] bf16 exact copies, chunk order as outlier_chunk_ids
 *   workspace           dev        >= shadowkv_build_workspace_bytes(), 256-byte aligned
 * The fields rank, topk_chunks, local_len of params are ignored here.
 */
int shadowkv_build_landmarks(const shadowkv_params *params, const shadowkv_kv *k_rope,
                             const shadowkv_kv *v, shadowkv_kv *landmarks,
                             int32_t *landmark_chunk_ids, int32_t *outlier_chunk_ids,
                             shadowkv_kv *k_outlier, shadowkv_kv *v_outlier, void *workspace,
                             size_t workspace_bytes, void *stream);

/*
 * Alg. 2 followed by softmax attention over the selected set, for one new token per sequence.
 *
 *   q                   dev        [b, h_q, d] bf16       post-RoPE query; head g uses KV head g / G
 *   A                   dev        [b, s, r] bf16         left low-rank factor of the pre-RoPE keys (no head axis)
 *   B                   dev        [b, h_kv, r, d] bf16   right factor, per KV head
 *   landmarks, landmark_chunk_ids  as produced by shadowkv_build_landmarks
 *   k_outlier,v_outlier dev        [b, h_kv, o*c, d] bf16 (may be NULL when o == 0)
 *   k_local, v_local    dev        [b, h_kv, w, d] bf16   post-RoPE keys / values of the w most recent tokens
 *                                                          (may be NULL when w == 0)
 *   value_store         dev|pinned [b, h_kv, s, d] bf16   per params->value_location
 *   pos_offset          dev        [b] int32 or NULL      position of context token 0 (NULL => 0)
 *   out                 dev  out   [b, h_q, d] bf16
 *   out_chunk_ids       dev  out   [b, h_kv, k] int32 or NULL: the selected true chunk ids, ascending
 *   workspace           dev        >= shadowkv_decode_workspace_bytes(), 256-byte aligned
 *   stream              HIP stream all work is ordered on
 *   side_stream         NULL (recommended): a value gather, where one is needed, is done by the first
 *                       workgroups of the launch that rebuilds the keys, so the two overlap inside one
 *                       launch and the whole step is ordered on `stream` alone (it can be captured into a
 *                       HIP graph as it is).  Non-NULL and different from `stream`: the gather is a launch
 *                       of its own on that stream, forked from and joined back into `stream` with events
 *                       (the two-stream arrangement the paper describes; slower here by the cost of the
 *                       events).  Ignored when no gather is needed.
 *
 * Scores are ranked in the log domain: score(slot) = max over the group's heads of
 * (logit_g(slot) - logsumexp_g), which orders slots exactly like softmax-then-max.  The logit is
 * scale * <q_g, L_slot> in fp64 (exact bf16 products, fp64 sum); the normaliser is formed from the fp64
 * logits; the ranking is the one of the fp64 scores (the search runs on fp32 copies of the logits and
 * settles its boundary on fp64 scores formed again from q and the landmarks); ties go to the lower slot.
 */
int shadowkv_decode_step(const shadowkv_params *params, const shadowkv_bf16 *q,
                         const shadowkv_kv *A, const shadowkv_kv *B,
                         const shadowkv_kv *landmarks, const int32_t *landmark_chunk_ids,
                         const shadowkv_kv *k_outlier, const shadowkv_kv *v_outlier,
                         const shadowkv_kv *k_local, const shadowkv_kv *v_local,
                         const shadowkv_kv *value_store, const int32_t *pos_offset,
                         shadowkv_bf16 *out, int32_t *out_chunk_ids, void *workspace,
                         size_t workspace_bytes, void *stream, void *side_stream);

/*
 * shadowkv_decode_step for callers that cannot allocate device memory or hand over a workspace: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments and
 * same results (bit for bit) as shadowkv_decode_step without `workspace`, `workspace_bytes` and
 * `side_stream`: the intermediates live in a scratch array inside the library's device image,
 * shadowkv_static_scratch_bytes() bytes (96 MiB) per GPU the library is loaded on, held until the process
 * ends.  A shape whose shadowkv_decode_workspace_bytes() exceeds that is rejected with SHADOWKV_EWORKSPACE
 * before anything is enqueued (all five benchmark shapes fit).  The call allocates nothing (no hipMalloc,
 * no events); its first use on a device looks up the array's address there.  Nothing in the scratch has to
 * start at zero and nothing is cleared; it keeps the last call's intermediates.  All calls on one GPU share
 * the one array: calls whose work overlaps on that GPU (different streams, or another thread) race -- order
 * them on one stream.  A value gather, where the shape needs one, runs inside the key-phase launch.
 */
int shadowkv_decode_step_static(const shadowkv_params *params, const shadowkv_bf16 *q,
                                const shadowkv_kv *A, const shadowkv_kv *B,
                                const shadowkv_kv *landmarks, const int32_t *landmark_chunk_ids,
                                const shadowkv_kv *k_outlier, const shadowkv_kv *v_outlier,
                                const shadowkv_kv *k_local, const shadowkv_kv *v_local,
                                const shadowkv_kv *value_store, const int32_t *pos_offset,
                                shadowkv_bf16 *out, int32_t *out_chunk_ids, void *stream);
size_t shadowkv_static_scratch_bytes(void);

/*
 * The same decode step with a chunk cache of the value store (section "High-throughput Decoding":
 * the chunks selected by adjacent steps repeat to a large part; an index scan finds the missing ones
 * and only those are fetched -- the (1 - alpha) term of the equivalent-bandwidth formula in section
 * "Theoretical Equivalent Bandwidth").  Meant for a store in pinned host memory; legal for HBM too.
 *
 * Arguments as shadowkv_decode_step, plus
 *   cache_slots      S: slots of one chunk each per (batch, KV head); topk_chunks <= S <= 8192
 *   value_cache      dev in/out [b, h_kv, S*c, d] bf16  shadowkv_value_cache_bytes() bytes, 16-byte aligned
 *   cache_chunk_ids  dev in/out [b, h_kv, S] int32      true chunk id held by each slot, -1 = empty
 *   cache_stamps     dev in/out [b, h_kv, S+1] int32    clock value of each slot's last use, then the
 *                                                       unit's clock (one tick per step)
 *   out_miss_count   dev out    [b, h_kv] int32 or NULL number of chunks fetched for this step
 * The three cache arrays must be what the previous cached step (same params, same store) left there,
 * or freshly reset.
 *
 * Policy (the paper names "a cache policy" without fixing one): least recently used.  A selected
 * chunk found in a slot stays there.  The selected chunks found nowhere take the slots that were not
 * hit in this step and have the oldest stamps (empty slots first; equal stamps: lower slot first);
 * among those slots, missing chunks in ascending chunk id go to slots in ascending index.  With
 * S == topk_chunks the slots hold exactly the last step's selection.  Attention reads each selected
 * chunk's values from its slot in the usual (ascending chunk id) order, so `out` and out_chunk_ids
 * are bit-identical to shadowkv_decode_step with SHADOWKV_FLAG_STAGE_VALUES.  Ownership: the caller
 * owns the buffers and keeps them between steps; the library keeps no pointer to them.
 */
int shadowkv_decode_step_cached(const shadowkv_params *params, const shadowkv_bf16 *q,
                                const shadowkv_kv *A, const shadowkv_kv *B,
                                const shadowkv_kv *landmarks, const int32_t *landmark_chunk_ids,
                                const shadowkv_kv *k_outlier, const shadowkv_kv *v_outlier,
                                const shadowkv_kv *k_local, const shadowkv_kv *v_local,
                                const shadowkv_kv *value_store, const int32_t *pos_offset,
                                int32_t cache_slots, shadowkv_kv *value_cache,
                                int32_t *cache_chunk_ids, int32_t *cache_stamps,
                                int32_t *out_miss_count, shadowkv_bf16 *out, int32_t *out_chunk_ids,
                                void *workspace, size_t workspace_bytes, void *stream,
                                void *side_stream);

/*
 * One more chunk of context from generated tokens (last paragraph of section "High-throughput
 * Decoding" and its footnote): the pre-RoPE keys K' of c tokens that have left the recent-token window
 * are stored as the low-rank states K' Psi, Psi = right singular matrix of the context keys, which here
 * is B transposed over the full key width: Psi[(h, x), rho] = B[b, h, rho, x].  The tokens become chunk
 * number s/c exactly as if the pre-filling algorithm had seen them (never an outlier: the outlier set
 * is fixed at pre-filling).
 *
 *   k_pre   dev [b, c, h_kv*d] bf16   pre-RoPE keys of the c tokens, heads side by side
 *   k_rope  dev [b, h_kv, c, d] bf16  the same keys after RoPE at their positions
 *   v       dev [b, h_kv, c, d] bf16  their values
 *   B       dev [b, h_kv, r, d] bf16
 *   in/out, laid out for ctx_capacity tokens: A (rows s .. s+c-1 written, fp64 accumulate, rounded once),
 *   landmarks (row n_c: mean of the chunk's post-RoPE keys), landmark_chunk_ids (entry n_c = s/c),
 *   value_store (dev|pinned; tokens s .. s+c-1).
 * Needs ctx_len + chunk_size <= ctx_capacity (else SHADOWKV_EINVAL).  params->ctx_len is the length
 * BEFORE the call; the caller continues with ctx_len + chunk_size.  The fields topk_chunks and local_len
 * are ignored.  A value cache (shadowkv_decode_step_cached) stays valid: existing chunks do not change.
 */
int shadowkv_append_chunk(const shadowkv_params *params, const shadowkv_kv *k_pre,
                          const shadowkv_kv *k_rope, const shadowkv_kv *v, const shadowkv_kv *B,
                          shadowkv_kv *A, shadowkv_kv *landmarks, int32_t *landmark_chunk_ids,
                          shadowkv_kv *value_store, void *stream);

/*
 * Alg. 1, first line: A, B <- SVD(K), the rank-r factors of the pre-RoPE keys of every sequence.  With
 * K = Phi Sigma Psi^T the thin SVD of the [s, D = h_kv*d] key matrix of one sequence, truncated to the r largest
 * singular values: B = Psi^T (reshaped [h_kv, r, d]: B[h, rho, x] = Psi[h*d + x, rho]) and A = K Psi = Phi Sigma
 * (the low-rank states of section "High-throughput Decoding": keys are kept as K Psi and projected back with Psi^T).
 * Singular vectors are defined up to sign; the convention here makes the component of largest magnitude of every
 * right singular vector positive (ties: lowest index).  Computed from the Gram matrix K^T K (fp64) by subspace
 * iteration with `n_iter` steps (0 => 16) on r + 32 vectors and a Rayleigh-Ritz step; accurate when sigma_r and
 * sigma_(r+33) are apart (the convergence factor per step is (sigma_(r+33) / sigma_r)^2).
 *
 *   k_pre      dev      [b, s, h_kv*d] kv   pre-RoPE keys, heads side by side
 *   A          dev out  [b, cap, r] kv      rows 0 .. s-1 written (fp64 accumulate, rounded once)
 *   B          dev out  [b, h_kv, r, d] kv
 *   psi_out    dev out  [b, r, h_kv*d] fp64 optional (NULL): the right singular vectors before rounding, as rows
 *   sigma_out  dev out  [b, r] fp64         optional (NULL): singular values, largest first
 *   workspace  dev      >= shadowkv_factorize_workspace_bytes(), 256-byte aligned
 * Needs rank <= h_kv*d.  topk_chunks, local_len, n_outlier_chunks are ignored.  Enqueues several thousand small
 * launches (one per dependent step of the orthogonalisation and of the Jacobi sweeps).
 */
int shadowkv_factorize_keys(const shadowkv_params *params, const shadowkv_kv *k_pre, shadowkv_kv *A,
                            shadowkv_kv *B, double *psi_out, double *sigma_out, int32_t n_iter,
                            void *workspace, size_t workspace_bytes, void *stream);
size_t shadowkv_factorize_workspace_bytes(const shadowkv_params *params);

/* Bytes of `value_cache` for the given shape and slot count (0 if either is invalid). */
size_t shadowkv_value_cache_bytes(const shadowkv_params *params, int32_t cache_slots);

/* Empties the cache: every slot of cache_chunk_ids -1, every stamp and the clocks 0; enqueued on `stream`. */
int shadowkv_value_cache_reset(const shadowkv_params *params, int32_t cache_slots,
                               int32_t *cache_chunk_ids, int32_t *cache_stamps, void *stream);

/*
 * ArgTopK as both algorithms of the paper use it (outlier chunks in Alg. 1, selected chunks in Alg. 2),
 * on its own: for each of `units` rows of `n` fp64 scores, the indices of the k largest values
 * (largest = sign * score, sign = +1 or -1), ties to the lower index, written in ascending index order.
 * NaN scores are not allowed.  Exact for any fp64 input (the internal search runs on a coarser monotone
 * key first and settles coarse ties on the exact values).
 *   scores    dev [units, n] fp64     out_ids  dev out [units, k] int32
 *   workspace dev, >= shadowkv_argtopk_workspace_bytes(units, n, k), 256-byte aligned
 * 1 <= k <= n, units <= 65535; SHADOWKV_EINVAL if the sizes exceed what the selection kernels hold.
 */
int shadowkv_argtopk(const double *scores, int32_t units, int32_t n, int32_t k, double sign,
                     int32_t *out_ids, void *workspace, size_t workspace_bytes, void *stream);
size_t shadowkv_argtopk_workspace_bytes(int32_t units, int32_t n, int32_t k);

/* Workspace sizes in bytes for the given shape (0 if params are invalid). */
size_t shadowkv_build_workspace_bytes(const shadowkv_params *params);
size_t shadowkv_decode_workspace_bytes(const shadowkv_params *params);

/* Host-only check of a parameter block: SHADOWKV_OK or SHADOWKV_EINVAL (reason via last_error). */
int shadowkv_validate_params(const shadowkv_params *params, int for_decode);

/*
 * Intermediates of the last decode step inside `workspace` (for tests and profiling).
 * which: 0 = rebuilt rotated keys RoPE(Gather(A, I) B), fp32 [b, h_kv, k*c, d], rows in out_chunk_ids order
 *            (only with SHADOWKV_FLAG_KEEP_REBUILT_KEYS; the keys normally live in registers only);
 *        1 = staged values Gather(V_store, I), bf16 [b, h_kv, k*c, d] (NULL when the gather did not run);
 *        2 = selected true chunk ids, int32 [b, h_kv, k];
 *        3 = scaled landmark logits P / sqrt(d) as stored for the search, fp32 [b, h_q, ld], ld = n_c rounded up
 *            to a multiple of 4 (the first n_c of a row are valid);
 *        4 = slots filled by the last cached step, int32 [b, h_kv, k] (first out_miss_count entries per unit);
 *        5 = slot of every selected chunk after the last cached step, int32 [b, h_kv, k].
 * Returns a pointer into `workspace`, or NULL.
 */
void *shadowkv_decode_workspace_view(const shadowkv_params *params, void *workspace, int which);

/*
 * How a plain shadowkv_decode_step (no value cache) of this shape is laid out on the GPU (measurement aid: lets
 * a benchmark say which launch the bytes of a stage belong to).  Writes 8 values to `plan` (host):
 *   [0] splits of the selected rows per (sequence, KV head); [1] rows per split;
 *   [2] 1 if the rows resident in HBM (outliers, recent tokens) are attended over by extra workgroups of the
 *       selection launch, 0 if by the attention launch;
 *   [3] 1 if the attention launch is the kernel with key waves and value waves, 0 the single-role kernel;
 *   [4] threads and [5] candidates per thread of the selection's first launch; [6] its launches (1 or 2, 3 with
 *       a middle level); [7] floats per row of the stored logits.
 * Returns SHADOWKV_OK or SHADOWKV_EINVAL (bad params / plan NULL).
 */
int shadowkv_decode_plan(const shadowkv_params *params, int32_t *plan);

/*
 * Per-stage timing of decode steps with HIP events recorded on the caller's stream at the
 * stage boundaries (measurement aid, not part of the method).  Between begin and end every
 * decode step (up to max_steps) records 5 events; end synchronises, writes the summed
 * milliseconds of the 4 stages -- landmark scoring | selection | staged value gather (zero when
 * values are read in place) | attention with key rebuild -- to stage_ms[4] and the number of recorded steps to n_steps.
 */
int shadowkv_profile_begin(int max_steps);
int shadowkv_profile_end(double *stage_ms, int *n_steps);

const char *shadowkv_status_string(int status); /* static string for a return code            */
const char *shadowkv_last_error(void);          /* thread-local detail of the last failure     */
int shadowkv_version(void);                     /* major*10000 + minor*100 + patch             */
void shadowkv_shutdown(void);                   /* destroy cached events; safe to call twice   */

#ifdef __cplusplus
}
#endif
#endif /* SHADOWKV_H */
