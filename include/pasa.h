/*
 * pasa.h -- C ABI of the MI355X (gfx950) implementation of the PASA sparse self-attention forward
 * ("Ride the Wave: Precision-Allocated Sparse Attention for Smooth Video Generation").
 *
 * The forward runs in stages, each an entry point of its own so that a caller (and a checker) can see
 * every intermediate:
 *
 *   pasa_block_score      block-pooled Q/K routing logits             (Eq.8 without its row softmax)
 *   pasa_block_score_with_stats  the same, with the block-mean keys taken from pasa_kv_stats' workspace
 *   pasa_key_prior        optional covariance prior of the routing logits (Eq.8, second term)
 *   pasa_route            seeded stochastic top-k block selection     (Eq.2 + Sec. "Stochastic Routing")
 *   pasa_route_gumbel     the same selection with a Gumbel-distributed bias (a variant)
 *   pasa_kv_stats         key/value block statistics, the query-independent part (Eq.4, Eq.5, Eq.12)
 *   pasa_sparse_attn_fwd  exact attention over the selected blocks + grouped Taylor approximation
 *                         of the unselected ones under one normaliser (Eq.7, Eq.4, Eq.5, Eq.12, Eq.14)
 *   pasa_attn_dense_ref   dense attention with the same tile machinery (Eq.1)
 *   pasa_forward          statistics, scores, routing and piecewise attention in one call
 *
 * Conventions
 *   - Every pointer is a DEVICE pointer unless marked "host".  The caller owns every buffer; the
 *     library never allocates, frees or synchronises.  All work is enqueued on `stream`
 *     (a hipStream_t passed as void*; NULL = the default stream) and is asynchronous.
 *   - Q, K, V, O are bf16 (uint16 storage), logical shape [B, H, n, d], innermost dimension
 *     contiguous, the others addressed by the element strides of pasa_shape_t.  d in {64, 128};
 *     block in {64, 128}.  n need not be a multiple of block: the last block is short, no token
 *     >= n is ever read or written.  N_B = ceil(n / block) for queries and keys alike.
 *   - bh = batch * H + head indexes every per-head array.
 *   - Return value: PASA_OK (0) or a negative pasa_status.  Arguments are validated on the host
 *     before anything is launched; on error nothing has been enqueued.  A launch failure is
 *     reported as PASA_EHIP (hipGetLastError after the launch; never a device synchronise).
 *   - Outputs must not alias inputs.  Base pointers must be 16-byte aligned and strides multiples of
 *     8 elements (PASA_EALIGN otherwise).
 *   - Size limits (PASA_EUNSUPPORTED beyond them): B * H <= 65535; n * stride_n * 2 < 2^32 (byte offsets inside one
 *     head are 32-bit, i.e. 4 GiB per head and tensor); B * H * ceil(n / 128) < 2^31; at most 262,144 key blocks
 *     and 65,535 first-order groups per head in pasa_sparse_attn_fwd; at most 4096 key blocks in pasa_route.
 *   - Device: written for gfx950 (MI355X: 256 compute units in 8 XCDs with an L2 each).  The workgroup-to-tile
 *     mapping assumes that consecutive workgroup ids go round-robin to 8 XCDs; on a device that deals them out
 *     differently the results are the same and only cache locality suffers.  Key-range slicing (kv_slices > 1)
 *     launches two workgroups per compute unit of the current device, as many as can be resident.
 *   - Results are deterministic: no floating-point atomics, fixed reduction order; the same inputs
 *     give the same bits on every call (also with key-range slicing, whose work queue only decides
 *     which workgroup computes an item, not what it computes).
 */
#ifndef PASA_H_
#define PASA_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define PASA_API __attribute__((visibility("default")))

typedef enum {
  PASA_OK = 0,
  PASA_EINVAL = -1,       /* null pointer, non-positive size, ratio outside (0,1], k outside [1,N_B] */
  PASA_EUNSUPPORTED = -2, /* d, block, group or slicing not supported; a size limit exceeded                  */
  PASA_EWORKSPACE = -3,   /* workspace smaller than pasa_*_workspace_bytes says                        */
  PASA_EALIGN = -4,       /* pointer not 16-byte aligned / stride not a multiple of 8 elements         */
  PASA_EHIP = -5,         /* the HIP runtime refused a launch                                          */
  PASA_ESCRATCH = -6      /* pasa_sparse_attn_fwd_static: the shape needs more than PASA_STATIC_SCRATCH_BYTES  */
} pasa_status;

typedef struct {
  int32_t B, H; /* batch, heads                                                                   */
  int32_t n;    /* tokens (queries = keys: self-attention)                                        */
  int32_t d;    /* head dimension, 64 or 128                                                      */
  int32_t block; /* tokens per block, 64 or 128 (Sec. "Taylor Expansion Approximation")           */
  int32_t group; /* key blocks per first-order group (Sec. "Grouped First-Order Approximation":
                    32).  >= N_B: one global matrix (Eq.6).  0: approximation off, unselected blocks
                    are dropped.  Otherwise a multiple of 32 or a power of two below 32.
                    Ignored by pasa_block_score and pasa_attn_dense_ref.                          */
  int64_t stride_b, stride_h, stride_n; /* element strides of Q, K, V and O; d is contiguous     */
  float scale; /* logit scale; 0 means 1/sqrt(d) (Eq.1)                                          */
  int32_t kv_slices; /* tuning knob of pasa_sparse_attn_fwd: the key range is cut into this many
                    contiguous slices, slice s is walked by workgroups of XCD s % 8 only (so that a
                    slice of K and V stays resident in that XCD's L2) and the per-slice partial results
                    are merged by a second kernel.  0 = the library chooses (today: no slicing, which is
                    faster at every shape measured); 1 = no slicing; otherwise a multiple of 8 not above
                    ceil(N_B / 32).  Results do not depend on it beyond
                    floating-point summation order.                                               */
} pasa_shape_t;

/* host-only. */
PASA_API const char* pasa_strerror(int status);

/* host-only.  k = clamp(floor(keep_ratio * n_blocks + 0.5), 1, n_blocks): the number of key blocks
 * computed exactly per query block for a "top-k density" keep_ratio (Sec. "Curvature-Aware Dynamic
 * Budgeting"; the rounding rule is this library's).  Returns PASA_EINVAL (negative) if n_blocks < 1
 * or keep_ratio is not in (0, 1]. */
PASA_API int32_t pasa_topk_count(int32_t n_blocks, double keep_ratio);

/* host-only.  N_B of a shape, or a negative status if the shape is invalid. */
PASA_API int32_t pasa_num_blocks(const pasa_shape_t* shape);

/* host-only.  Number of uint32 words of one row of the selection bitmap: ceil(N_B / 32). */
PASA_API int32_t pasa_mask_words(int32_t n_blocks);

/* host-only.  Bytes of scratch pasa_block_score needs (block means of Q and K, 4 bytes per element); 0 on a bad shape. */
PASA_API size_t pasa_score_workspace_bytes(const pasa_shape_t* shape);

/* host-only.  Bytes of scratch pasa_kv_stats, pasa_sparse_attn_fwd and pasa_attn_dense_ref need (key/value block
 * statistics, group matrices and unit sums, block-mean keys for pasa_block_score_with_stats, room for a selection
 * bitmap: 0.20 GB at 40 heads of 75,600 tokens; with kv_slices > 1 also the per-slice partial results:
 * B*H*kv_slices*n*(d+2)*4 bytes, 12.6 GB at 40 heads of 75,600 tokens with 8 slices); 0 on a bad shape. */
PASA_API size_t pasa_attn_workspace_bytes(const pasa_shape_t* shape);

/*
 * Stage 1 -- block-pooled scoring (Sec. "Taylor Expansion Approximation", Eq.8).
 *   scores[bh, i, j] = mean(Q block i) . mean(K block j) * scale + key_bias[bh, j]
 * Means are over the valid tokens of a block.  Eq.8's softmax over j is monotone per row and is
 * not applied: routing works on the logits.
 *   q, k      bf16 [B,H,n,d] (shape strides)
 *   key_bias  fp32 [B*H, N_B] or NULL (the covariance prior of Eq.8 enters here)
 *   scores    fp32 [B*H, N_B, N_B] contiguous (out)
 *   ws        scratch of pasa_score_workspace_bytes(shape) bytes, 256-byte aligned
 */
PASA_API int pasa_block_score(const void* q, const void* k, const pasa_shape_t* shape, const float* key_bias,
                     float* scores, void* ws, size_t ws_bytes, void* stream);

/*
 * Stage 1 for callers that run pasa_kv_stats first (the statistics do not depend on the queries): the block-mean keys
 * are taken from the statistics workspace instead of being pooled from K again, which saves one pass over K.
 * Same scores as pasa_block_score up to the summation order of the key means (a few units in the last place).
 *   stats_ws  the workspace pasa_kv_stats filled for the same k and shape (shape->group > 0: PASA_EUNSUPPORTED
 *             otherwise), stats_ws_bytes its size; ws as for pasa_block_score (only the query half is used)
 */
PASA_API int pasa_block_score_with_stats(const void* q, const pasa_shape_t* shape, const float* key_bias, float* scores,
                                         void* ws, size_t ws_bytes, const void* stats_ws, size_t stats_ws_bytes,
                                         void* stream);

/*
 * Stage 2 -- top-k routing with a seeded stochastic selection bias (Eq.2; Sec. "Stochastic Routing").
 *   r[bh,i,j] = fmaf(noise_amp, w, scores[bh,i,j]) in binary32 (one rounding), where w in [-1,1) is
 *   ((int32)u >> 8) * 2^-23 and u is word (j & 3) of Philox4x32-10(counter = (j >> 2, i, bh, 0),
 *   key = (seed & 0xffffffff, seed >> 32)).  Row (bh, i) selects the k_sel largest r under the strict
 *   order "larger value first (-0 == +0), then smaller j first".  NaN scores are a caller error.
 *   A fresh seed per layer and denoising step gives the independent re-sampling the paper describes.
 *   scores  fp32 [BH, N_B, N_B]
 *   idx     int32 [BH, N_B, k_sel] (out): selected key blocks of each query block, ascending
 *   mask    uint32 [BH, N_B, ceil(N_B/32)] (out, may be NULL): bit (j & 31) of word (j >> 5) is set
 *           iff key block j is selected; bits >= N_B are zero
 * The output is a pure function of (score bits, k_sel, seed, noise_amp).
 */
PASA_API int pasa_route(const float* scores, int32_t BH, int32_t n_blocks, int32_t k_sel, uint64_t seed,
               float noise_amp, int32_t* idx, uint32_t* mask, void* stream);

/*
 * Stage 2, variant -- the same routing with a Gumbel-distributed selection bias (Sec. "Stochastic Routing" asks
 * for a random bias on the block scores and fixes no distribution; with Gumbel noise the top-k_sel of the
 * perturbed logits is a sample without replacement from softmax(scores / temperature), the Gumbel-top-k trick).
 *   r[bh,i,j] = fmaf(temperature, g, scores[bh,i,j]),  g = -log(-log(u)),  u = ((x >> 9) + 0.5) * 2^-23,
 *   x the same Philox word as in pasa_route.  Order, outputs, limits and errors as in pasa_route.
 * The two logarithms are rounded differently by different math libraries: the selection is reproducible
 * bit for bit on this library only; against another implementation it can differ for blocks whose r lies
 * within rounding distance of the k_sel-th largest.
 */
PASA_API int pasa_route_gumbel(const float* scores, int32_t BH, int32_t n_blocks, int32_t k_sel, uint64_t seed,
                      float temperature, int32_t* idx, uint32_t* mask, void* stream);

/*
 * Key/value block statistics (Eq.4's inner sum, Eq.5, Eq.12) -- the query-independent part of
 * stages 3 and 4, exported on its own so that it can be timed and reused:
 *   Kbar_j = mean_n K_{j,n},  VS_j = sum_n V_{j,n},
 *   Hg_g   = mean over the blocks j of group g of  H_j = sum_n (K_{j,n} - Kbar_j)^T V_{j,n}
 * written into `ws` in the library's internal layout (bf16; Hg pre-multiplied by the logit scale).
 *   k, v  bf16 [B,H,n,d] (shape strides);  ws scratch of pasa_attn_workspace_bytes(shape) bytes,
 *   256-byte aligned.  shape->group == 0 is accepted and does nothing.
 */
PASA_API int pasa_kv_stats(const void* k, const void* v, const pasa_shape_t* shape, void* ws, size_t ws_bytes,
                           void* stream);

/*
 * Covariance-aware routing prior (Eq.8's second term): for every key block
 *   beta[bh, j] = log( || H_j - Hg_{g(j)} ||_F + eps ),
 * H_j the first-order statistic of the block (Eq.5), Hg_{g(j)} the mean over the blocks of its group
 * (Eq.12; Eq.6 when the group is the whole sequence), || ||_F the Frobenius norm (the norm of the paper's
 * error analysis), both without the logit scale.  Feed the result to pasa_block_score as key_bias to
 * obtain the full routing logit of Eq.8.  Requires that `ws` was filled by pasa_kv_stats for the same
 * k, v and shape (it reads the group sums left there) and shape->group > 0 (PASA_EUNSUPPORTED otherwise).
 *   k, v   bf16 [B,H,n,d] (shape strides);  eps >= 0;  beta fp32 [B*H, N_B] contiguous (out)
 */
PASA_API int pasa_key_prior(const void* k, const void* v, const pasa_shape_t* shape, float eps, float* beta,
                            void* ws, size_t ws_bytes, void* stream);

/*
 * Stages 3 and 4 -- piecewise attention (Eq.7 with the grouped first-order term of Eq.14).
 * For query token t of query block i, q~ = Q_t * scale, S = idx[bh, i, :], U = the other blocks:
 *   Num = sum_{j in S} sum_{n < b_j} exp(q~ K_{j,n}) V_{j,n}
 *       + sum_{j in U} a_j VS_j,            a_j = exp(q~ Kbar_j), VS_j = sum_n V_{j,n}     (Eq.4)
 *       + sum_g (sum_{j in U and in group g} a_j) (q~ Hg_g)                                  (Eq.14)
 *   Den = sum_{j in S} sum_{n < b_j} exp(q~ K_{j,n}) + sum_{j in U} b_j a_j
 *   O_t = Num / Den   (one online-softmax normaliser; b_j = valid tokens of block j)
 * pasa_sparse_attn_fwd recomputes the key/value statistics on every call (pasa_kv_stats, then the
 * attention kernel).  pasa_sparse_attn_fwd_prepared runs the attention kernel alone and requires
 * that `ws` was filled by pasa_kv_stats for the same k, v and shape and not touched since.
 *   idx    int32 [BH, N_B, k_sel], each row strictly ascending, values in [0, N_B), or NULL if mask is given
 *   mask   uint32 [BH, N_B, ceil(N_B/32)], the bitmap of the same selection (as pasa_route writes it), or NULL if
 *          idx is given.  The kernels walk a bitmap: with mask == NULL one is first built from idx in the workspace
 *          (a caller with index lists of its own needs nothing else); with both given the bitmap is used and idx
 *          is not read.  Neither is validated here -- entries outside [0, N_B) are ignored when the bitmap is
 *          built, set bits at or beyond N_B are a caller error -- pasa_check_selection checks a selection,
 *          including that list and bitmap agree.
 *   out    bf16 [B,H,n,d] (shape strides)
 *   lse    fp32 [BH, n] or NULL: log(Den) including the subtracted maximum
 *   ws     scratch of pasa_attn_workspace_bytes(shape) bytes, 256-byte aligned
 */
PASA_API int pasa_sparse_attn_fwd(const void* q, const void* k, const void* v, const pasa_shape_t* shape,
                                  const int32_t* idx, const uint32_t* mask, int32_t k_sel, void* out,
                                  float* lse, void* ws, size_t ws_bytes, void* stream);
PASA_API int pasa_sparse_attn_fwd_prepared(const void* q, const void* k, const void* v, const pasa_shape_t* shape,
                                           const int32_t* idx, const uint32_t* mask, int32_t k_sel, void* out,
                                           float* lse, void* ws, size_t ws_bytes, void* stream);

/*
 * The whole forward in one call: statistics, scores (routing logit without the covariance prior), routing with the
 * uniform selection bias, piecewise attention -- exactly the sequence pasa_kv_stats, pasa_block_score_with_stats,
 * pasa_route(k_sel = pasa_topk_count(N_B, keep_ratio)), pasa_sparse_attn_fwd_prepared, with every intermediate
 * (scores, index lists, bitmap, both scratch areas) carved out of one workspace.  Callers that want the
 * intermediates, the prior, the Gumbel bias or their own selection use the stage entry points instead.
 *   keep_ratio in (0, 1]; seed, noise_amp as in pasa_route; out, lse as in pasa_sparse_attn_fwd
 *   ws  pasa_forward_workspace_bytes(shape, keep_ratio) bytes (host-only helper; 0 on invalid arguments), 256-byte aligned
 * N_B <= 4096 (the limit of pasa_route).
 */
PASA_API size_t pasa_forward_workspace_bytes(const pasa_shape_t* shape, double keep_ratio);
PASA_API int pasa_forward(const void* q, const void* k, const void* v, const pasa_shape_t* shape, double keep_ratio,
                          uint64_t seed, float noise_amp, void* out, float* lse, void* ws, size_t ws_bytes, void* stream);

/*
 * Validation of a selection before it is handed to pasa_sparse_attn_fwd (debugging aid for callers that build
 * their own lists or bitmaps).  A row (bh, i) is bad if an index lies outside [0, N_B), its list is not strictly
 * ascending, its bitmap row has a bit set at or beyond N_B or does not have exactly k_sel bits set, or a listed
 * block's bit is not set (list and bitmap name different blocks).  Either of idx and mask may be NULL; then only
 * the other is checked.
 *   idx int32 [BH, N_B, k_sel];  mask uint32 [BH, N_B, ceil(N_B/32)];  n_bad DEVICE int32 (out): number of bad rows.
 * Two small kernels on `stream`; the count is an integer sum, hence deterministic.
 */
PASA_API int pasa_check_selection(const int32_t* idx, const uint32_t* mask, int32_t BH, int32_t n_blocks, int32_t k_sel,
                                  int32_t* n_bad, void* stream);

/*
 * pasa_sparse_attn_fwd for callers that cannot allocate device memory or hand over a workspace: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, results and errors as
 * pasa_sparse_attn_fwd without `ws`: the key/value statistics go to a buffer of PASA_STATIC_SCRATCH_BYTES that is
 * part of the library's device image (one copy per GPU, held until the process ends).  The call allocates and frees
 * nothing and calls no allocating routine; its first call on a device looks the buffer's address up once (make
 * that call outside a graph capture).  shape->kv_slices is ignored (no slicing).
 *   PASA_ESCRATCH if pasa_attn_workspace_bytes(shape with kv_slices = 1) > PASA_STATIC_SCRATCH_BYTES
 *   (e.g. the Wan-1.3B 480p shape, 12 heads of 32,760 tokens, needs 61 MiB; 40 heads of 75,600 tokens do not fit).
 * All calls on one GPU share the buffer: two calls that overlap in time on one GPU (different streams, or
 * different host threads) race and give wrong results.  Nothing in it has to be cleared between calls (every
 * part is rewritten before it is read).
 */
#define PASA_STATIC_SCRATCH_BYTES (64u << 20)
PASA_API int pasa_sparse_attn_fwd_static(const void* q, const void* k, const void* v, const pasa_shape_t* shape,
                                         const int32_t* idx, const uint32_t* mask, int32_t k_sel, void* out,
                                         float* lse, void* stream);

/*
 * Dense attention, Eq.1: O = softmax(Q K^T * scale) V, same kernels with every block selected.
 *   out bf16 [B,H,n,d]; lse fp32 [BH, n] or NULL; ws as for pasa_sparse_attn_fwd.
 */
PASA_API int pasa_attn_dense_ref(const void* q, const void* k, const void* v, const pasa_shape_t* shape,
                        void* out, float* lse, void* ws, size_t ws_bytes, void* stream);

/*
 * Curvature-aware dynamic budget (Sec. "Curvature-Aware Dynamic Budgeting").
 *
 * pasa_l1_distance: the calibration signal -- mean absolute difference of two tensors of n elements (the
 * velocity fields of two consecutive denoising steps), out[0] = sum_i |a_i - b_i| / n.  a, b: DEVICE, 16-byte
 * aligned, dtype PASA_DTYPE_BF16 or PASA_DTYPE_F32; out: DEVICE fp32 scalar; ws: DEVICE scratch of
 * pasa_l1_workspace_bytes() bytes.  Two kernels on `stream`, fixed summation order (deterministic).
 *
 * pasa_budget_schedule: host-only, Eq.9-11.  l1 [n_prompts, n_steps] (host): entry (p, t) is the signal of
 * calibration prompt p at step t (distance between the velocity fields of steps t-1 and t); rho in (0, 1] the
 * baseline density; the first floor(dense_fraction * n_steps + 0.5) steps keep full attention (the paper: 20 %)
 * and get rho_t = 1.  On the other steps  l_t = mean over prompts,  lbar = mean of l_t over those steps (Eq.9),
 * alpha_t = l_t / lbar (Eq.10),  rho_t = min(1, rho * alpha_t) (Eq.11; the cap at 1 is this library's: a density
 * cannot exceed "every block").  rho_t [n_steps] (host, out) feeds pasa_topk_count step by step.  Without the cap
 * the rho_t of the sparse steps sum to rho times their number, the paper's "same total budget".
 * PASA_EINVAL for negative or non-finite signals or an all-zero signal.
 */
enum { PASA_DTYPE_BF16 = 0, PASA_DTYPE_F32 = 1 };
PASA_API size_t pasa_l1_workspace_bytes(void);
PASA_API int pasa_l1_distance(const void* a, const void* b, int64_t n, int32_t dtype, float* out, void* ws,
                              size_t ws_bytes, void* stream);
PASA_API int pasa_budget_schedule(const double* l1, int32_t n_prompts, int32_t n_steps, double rho,
                                  double dense_fraction, double* rho_t);

/*
 * Measurement aid (not part of the forward, cites nothing): launches `workgroups` workgroups of 256 threads that
 * each run `iterations` rounds of 8 independent 32x32x16 bf16 MFMAs on register operands, and returns in
 * *flops (host) the floating-point operations of the launch.  Timed by the caller, it gives the matrix-core rate
 * the device sustains, which bench.py reports beside the published peak.
 *   random_operands  0: all chains share one operand pair of a few distinct small values (least power: the device
 *                    holds close to its nominal clock); nonzero: every chain has its own operands filled with
 *                    N(0,1)-like values, as activations are (the clock, and the rate, the matrix cores sustain on data)
 *   sink   device buffer of at least workgroups * 256 floats (never written in practice)
 */
PASA_API int pasa_mfma_probe(int32_t workgroups, int32_t iterations, int32_t random_operands, float* sink, double* flops,
                             void* stream);

#ifdef __cplusplus
}
#endif
#endif /* PASA_H_ */
