/*
 * pasa_oracle.c -- plain, slow, fp64 CPU reference of the PASA sparse-attention forward.
 *
 * THIS FILE IS TEST INFRASTRUCTURE.  It defines what "correct" means for the GPU library and is
 * used only by the test-suite, by the smoke check and by the benchmark's cpu_baseline leg.  It shares
 * no code, header, table or helper with the GPU path and must never be reachable from the product.
 *
 * What is computed (all floating point in fp64, except the routing-noise step which the method
 * defines in binary32 so that two implementations can agree bit for bit):
 *
 *   Eq.1  (Sec. "Self-Attention in Video Diffusion Transformers")  dense softmax(QK^T/sqrt(D))V
 *   Sec. "Taylor Expansion Approximation for Sparse Attention":
 *         block partition, block-mean keys, alpha_{t,j}, Eq.4 (zeroth order), Eq.5 (H_j),
 *         Eq.6 (global mean of H_j), Eq.7 (piecewise numerator), Eq.8 (routing logit)
 *   Eq.2  top-k selection
 *   Sec. "Stochastic Routing": a random bias on the block scores (the paper gives no formula; the
 *         reading used here: additive uniform noise in [-amp, amp) on the routing logit, drawn from
 *         the counter-based Philox4x32-10 generator keyed by (seed; head, query block, key block))
 *   Sec. "Grouped First-Order Approximation" and Appendix "Error Analysis": Eq.12 (group mean of
 *         H_j), Eq.14 (grouped first-order numerator), Lemma 1 and Proposition 1 quantities.
 *
 * Readings taken where the paper is silent (each is listed in the design document as well):
 *   - the 1/sqrt(D) scale of Eq.1 applies to every logit, i.e. q~ = q*scale replaces Q_t in
 *     alpha_{t,j}, in Eq.7 and in q~ H;
 *   - the normaliser that goes with Eq.7 is  sum_S sum_n exp(q~ K_{j,n}) + sum_U b_j alpha_{t,j}
 *     (the first-order term sums to zero inside a block, so it adds nothing to the normaliser);
 *   - routing is per query BLOCK with mean-pooled queries; k = clamp(floor(keep*N_B + 0.5), 1, N_B);
 *   - a group is G consecutive key blocks; the group mean is over all blocks of the group;
 *   - a ragged last block uses its valid tokens only (mean over b_j tokens, weight b_j).
 *
 * Pin status: every function here is pinned by tests that do not call it to produce their own
 * expected values (closed forms, invariants, a library routine, published known-answer vectors),
 * with one exception stated where it applies: the accuracy of PASA against dense attention on
 * general inputs has no figure in the paper -- "parity unpinned" for that quantity only.
 *
 * Layout: tensors are contiguous [BH][n][d] double, BH = batch*heads flattened.
 * Build:  gcc -O2 -fopenmp -shared -fPIC -o libpasa_oracle.so pasa_oracle.c -lm
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORACLE_API __attribute__((visibility("default")))

ORACLE_API int32_t oracle_num_threads(void) {
#ifdef _OPENMP
  return (int32_t)omp_get_max_threads();
#else
  return 1;
#endif
}

/* ---------------------------------------------------------------------------------------------
 * Block partition (Sec. "Taylor Expansion Approximation", first paragraph): consecutive tokens,
 * block j = [j*b, min((j+1)*b, n)).
 * ------------------------------------------------------------------------------------------- */
static int64_t n_blocks_of(int64_t n, int64_t b) { return (n + b - 1) / b; }
static int64_t block_len(int64_t j, int64_t n, int64_t b) {
  int64_t lo = j * b, hi = lo + b;
  if (hi > n) hi = n;
  return hi - lo;
}

/* k from the keep ratio: "top-k density rho (fraction of blocks computed exactly)"; the rounding
 * rule is this build's reading: nearest integer, at least one block, at most all of them. */
ORACLE_API int32_t oracle_topk_count(int32_t n_blocks, double keep_ratio) {
  double x = floor(keep_ratio * (double)n_blocks + 0.5);
  if (x < 1.0) x = 1.0;
  if (x > (double)n_blocks) x = (double)n_blocks;
  return (int32_t)x;
}

/* ---------------------------------------------------------------------------------------------
 * Philox4x32 with 10 rounds (Salmon, Moraes, Dror, Shaw: "Parallel random numbers: as easy as
 * 1, 2, 3", SC'11).  One round: two 32x32->64 multiplies of counter words 0 and 2, a word
 * permutation with the key xor-ed in, then the key is advanced by the Weyl constants.
 * ------------------------------------------------------------------------------------------- */
ORACLE_API void oracle_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]) {
  uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
  uint32_t k0 = key[0], k1 = key[1];
  for (int round = 0; round < 10; ++round) {
    uint64_t p0 = (uint64_t)0xD2511F53u * (uint64_t)c0;
    uint64_t p1 = (uint64_t)0xCD9E8D57u * (uint64_t)c2;
    uint32_t hi0 = (uint32_t)(p0 >> 32), lo0 = (uint32_t)p0;
    uint32_t hi1 = (uint32_t)(p1 >> 32), lo1 = (uint32_t)p1;
    uint32_t n0 = hi1 ^ c1 ^ k0;
    uint32_t n1 = lo1;
    uint32_t n2 = hi0 ^ c3 ^ k1;
    uint32_t n3 = lo0;
    c0 = n0; c1 = n1; c2 = n2; c3 = n3;
    k0 += 0x9E3779B9u;
    k1 += 0xBB67AE85u;
  }
  out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* The unit noise w in [-1, 1) for the (head bh, query block i, key block j) cell:
 * counter = (j >> 2, i, bh, 0), key = (seed low word, seed high word), word j & 3 of the output,
 * top 24 bits taken as a signed integer and scaled by 2^-23 (exact in binary32). */
ORACLE_API float oracle_noise_unit(uint64_t seed, uint32_t bh, uint32_t i, uint32_t j) {
  uint32_t ctr[4] = {j >> 2, i, bh, 0u};
  uint32_t key[2] = {(uint32_t)(seed & 0xFFFFFFFFu), (uint32_t)(seed >> 32)};
  uint32_t x[4];
  oracle_philox4x32_10(ctr, key, x);
  uint32_t u = x[j & 3u];
  int32_t s = (int32_t)u >> 8; /* arithmetic shift: a signed 24-bit integer */
  return (float)s * 0x1p-23f;
}

/* ---------------------------------------------------------------------------------------------
 * Block means ("mean key vector of block j"; queries are pooled the same way).
 * X [BH][n][d] -> out [BH][N_B][d]
 * ------------------------------------------------------------------------------------------- */
ORACLE_API void oracle_block_mean(const double* X, int64_t BH, int64_t n, int64_t d, int64_t b,
                                  double* out) {
  int64_t NB = n_blocks_of(n, b);
  for (int64_t h = 0; h < BH; ++h)
    for (int64_t j = 0; j < NB; ++j) {
      int64_t len = block_len(j, n, b);
      double* o = out + (h * NB + j) * d;
      for (int64_t c = 0; c < d; ++c) o[c] = 0.0;
      for (int64_t t = 0; t < len; ++t) {
        const double* x = X + (h * n + j * b + t) * d;
        for (int64_t c = 0; c < d; ++c) o[c] += x[c];
      }
      for (int64_t c = 0; c < d; ++c) o[c] /= (double)len;
    }
}

/* Routing logit of Eq.8 without its (monotone) row softmax:
 * s_ij = mean(Q block i) . mean(K block j) * scale + key_bias_j.     scores [BH][N_B][N_B] */
ORACLE_API void oracle_block_scores(const double* Q, const double* K, int64_t BH, int64_t n,
                                    int64_t d, int64_t b, double scale, const double* key_bias,
                                    double* scores) {
  int64_t NB = n_blocks_of(n, b);
  double* qm = (double*)malloc(sizeof(double) * (size_t)(BH * NB * d));
  double* km = (double*)malloc(sizeof(double) * (size_t)(BH * NB * d));
  oracle_block_mean(Q, BH, n, d, b, qm);
  oracle_block_mean(K, BH, n, d, b, km);
  for (int64_t h = 0; h < BH; ++h)
    for (int64_t i = 0; i < NB; ++i)
      for (int64_t j = 0; j < NB; ++j) {
        double acc = 0.0;
        for (int64_t c = 0; c < d; ++c) acc += qm[(h * NB + i) * d + c] * km[(h * NB + j) * d + c];
        acc *= scale;
        if (key_bias) acc += key_bias[h * NB + j];
        scores[(h * NB + i) * NB + j] = acc;
      }
  free(qm);
  free(km);
}

/* ---------------------------------------------------------------------------------------------
 * Routing (Eq.2 with the stochastic bias).  r_ij = fmaf(amp, w_ij, s_ij) in binary32, then the k
 * largest under the strict total order (r descending, j ascending), written in ascending j.
 * The float comparison is done on an order-preserving integer image of the bits, with -0 mapped to
 * +0 first, so "equal" means equal as real numbers and ties go to the smaller index.  NaN scores
 * are a caller error.
 * scores [BH][NB][NB] float; bh_ids (nullable) gives the global head id of each of the BH slices;
 * idx [BH][NB][k] int32; noisy (nullable) [BH][NB][NB] float receives r.
 * ------------------------------------------------------------------------------------------- */
static uint32_t ordered_bits(float x) {
  uint32_t u;
  memcpy(&u, &x, 4);
  if (u == 0x80000000u) u = 0u; /* -0 and +0 are the same value */
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

typedef struct { uint32_t key; int32_t j; } cell_t;

static int cell_before(const void* a, const void* b) {
  const cell_t* x = (const cell_t*)a;
  const cell_t* y = (const cell_t*)b;
  if (x->key != y->key) return (x->key > y->key) ? -1 : 1; /* larger value first */
  return (x->j < y->j) ? -1 : (x->j > y->j); /* then smaller index first */
}

static int int_ascending(const void* a, const void* b) {
  int32_t x = *(const int32_t*)a, y = *(const int32_t*)b;
  return (x < y) ? -1 : (x > y);
}

ORACLE_API void oracle_route(const float* scores, int64_t BH, int64_t NB, int64_t k, uint64_t seed,
                             float amp, const int32_t* bh_ids, int32_t* idx, float* noisy) {
#pragma omp parallel
  {
    cell_t* cells = (cell_t*)malloc(sizeof(cell_t) * (size_t)NB);
#pragma omp for collapse(2) schedule(static)
    for (int64_t h = 0; h < BH; ++h)
      for (int64_t i = 0; i < NB; ++i) {
        uint32_t bh = bh_ids ? (uint32_t)bh_ids[h] : (uint32_t)h;
        for (int64_t j = 0; j < NB; ++j) {
          float s = scores[(h * NB + i) * NB + j];
          float w = oracle_noise_unit(seed, bh, (uint32_t)i, (uint32_t)j);
          float r = fmaf(amp, w, s);
          if (noisy) noisy[(h * NB + i) * NB + j] = r;
          cells[j].key = ordered_bits(r);
          cells[j].j = (int32_t)j;
        }
        qsort(cells, (size_t)NB, sizeof(cell_t), cell_before);
        int32_t* out = idx + (h * NB + i) * k;
        for (int64_t s = 0; s < k; ++s) out[s] = cells[s].j;
        qsort(out, (size_t)k, sizeof(int32_t), int_ascending);
      }
    free(cells);
  }
}

/* ---------------------------------------------------------------------------------------------
 * Key/value statistics.
 *   Kbar_j = mean_n K_{j,n}                       [BH][NB][d]
 *   VS_j   = sum_n  V_{j,n}                       [BH][NB][d]         (inner sum of Eq.4)
 *   H_j    = sum_n (K_{j,n} - Kbar_j)^T V_{j,n}   [BH][NB][d][d]      (Eq.5; nullable output)
 *   Hg_g   = mean_{j in group g} H_j              [BH][NG][d][d]      (Eq.12; G>=NB gives Eq.6)
 * Groups are G consecutive blocks, the last one possibly short.  G <= 0: Hg is not written.
 * ------------------------------------------------------------------------------------------- */
ORACLE_API void oracle_kv_stats(const double* K, const double* V, int64_t BH, int64_t n, int64_t d,
                                int64_t b, int64_t G, double* Kbar, double* VS, double* Hj,
                                double* Hg) {
  int64_t NB = n_blocks_of(n, b);
  int64_t NG = (G > 0) ? (NB + G - 1) / G : 0;
  oracle_block_mean(K, BH, n, d, b, Kbar);
#pragma omp parallel
  {
    double* H = (double*)malloc(sizeof(double) * (size_t)(d * d));
#pragma omp for schedule(dynamic)
    for (int64_t h = 0; h < BH; ++h) {
      if (Hg && NG > 0) memset(Hg + h * NG * d * d, 0, sizeof(double) * (size_t)(NG * d * d));
      for (int64_t j = 0; j < NB; ++j) {
        int64_t len = block_len(j, n, b);
        const double* kb = Kbar + (h * NB + j) * d;
        double* vs = VS + (h * NB + j) * d;
        for (int64_t c = 0; c < d; ++c) vs[c] = 0.0;
        for (int64_t a = 0; a < d * d; ++a) H[a] = 0.0;
        for (int64_t t = 0; t < len; ++t) {
          const double* kr = K + (h * n + j * b + t) * d;
          const double* vr = V + (h * n + j * b + t) * d;
          for (int64_t c = 0; c < d; ++c) vs[c] += vr[c];
          for (int64_t a = 0; a < d; ++a) {
            double dk = kr[a] - kb[a];
            for (int64_t c = 0; c < d; ++c) H[a * d + c] += dk * vr[c];
          }
        }
        if (Hj) memcpy(Hj + (h * NB + j) * d * d, H, sizeof(double) * (size_t)(d * d));
        if (Hg && NG > 0) {
          double* g = Hg + (h * NG + j / G) * d * d;
          for (int64_t a = 0; a < d * d; ++a) g[a] += H[a];
        }
      }
      if (Hg && NG > 0)
        for (int64_t g = 0; g < NG; ++g) {
          int64_t lo = g * G, hi = lo + G;
          if (hi > NB) hi = NB;
          double inv = 1.0 / (double)(hi - lo);
          double* m = Hg + (h * NG + g) * d * d;
          for (int64_t a = 0; a < d * d; ++a) m[a] *= inv;
        }
    }
    free(H);
  }
}

/* ---------------------------------------------------------------------------------------------
 * Dense attention, Eq.1, row by row: logits, their maximum, exponentials, normalise.
 * q_rows (nullable): the n_rows query rows to evaluate (same rows for every head); null = all n.
 * O [BH][n_rows][d], lse (nullable) [BH][n_rows] = log sum_n exp(logit).
 * ------------------------------------------------------------------------------------------- */
ORACLE_API void oracle_dense_attention(const double* Q, const double* K, const double* V, int64_t BH,
                                       int64_t n, int64_t d, double scale, const int32_t* q_rows,
                                       int64_t n_rows, double* O, double* lse) {
  if (!q_rows) n_rows = n;
#pragma omp parallel
  {
    double* p = (double*)malloc(sizeof(double) * (size_t)n);
#pragma omp for collapse(2) schedule(dynamic, 8)
    for (int64_t h = 0; h < BH; ++h)
      for (int64_t r = 0; r < n_rows; ++r) {
        int64_t t = q_rows ? q_rows[r] : r;
        const double* q = Q + (h * n + t) * d;
        double m = -INFINITY;
        for (int64_t s = 0; s < n; ++s) {
          const double* kr = K + (h * n + s) * d;
          double acc = 0.0;
#pragma omp simd reduction(+ : acc)
          for (int64_t c = 0; c < d; ++c) acc += q[c] * kr[c];
          p[s] = acc * scale;
          if (p[s] > m) m = p[s];
        }
        double den = 0.0;
        for (int64_t s = 0; s < n; ++s) {
          p[s] = exp(p[s] - m);
          den += p[s];
        }
        double* o = O + (h * n_rows + r) * d;
        for (int64_t c = 0; c < d; ++c) o[c] = 0.0;
        for (int64_t s = 0; s < n; ++s) {
          const double* vr = V + (h * n + s) * d;
          for (int64_t c = 0; c < d; ++c) o[c] += p[s] * vr[c];
        }
        for (int64_t c = 0; c < d; ++c) o[c] /= den;
        if (lse) lse[h * n_rows + r] = m + log(den);
      }
    free(p);
  }
}

/* ---------------------------------------------------------------------------------------------
 * PASA piecewise attention for one routing decision.
 *
 * For query token t in query block i, q~ = Q_t * scale, S = selected key blocks of block i
 * (idx, k per row, any order), U = the other blocks:
 *
 *   Num = sum_{j in S} sum_{n<b_j} exp(q~ K_{j,n}) V_{j,n}                    (Eq.7 first term)
 *       + sum_{j in U} alpha_j VS_j ,           alpha_j = exp(q~ Kbar_j)      (Eq.4)
 *       + sum_g ( sum_{j in U, j in group g} alpha_j ) (q~ Hg_g)              (Eq.14)
 *   Den = sum_{j in S} sum_{n<b_j} exp(q~ K_{j,n}) + sum_{j in U} b_j alpha_j
 *   O_t = Num / Den,  evaluated with the largest logit subtracted from every exponent.
 *
 * G: blocks per group (G >= N_B reproduces the single global matrix of Eq.6/Eq.7; G = 1 uses every
 *    block's own H_j, the exact first-order numerator of Eq.13); G <= 0 switches the whole
 *    approximation off (unselected blocks are dropped from numerator and normaliser).
 * terms: bit 0 = zeroth-order term (and its b_j alpha_j share of Den), bit 1 = first-order term.
 * q_blocks (nullable): the n_qblocks query blocks to evaluate; null = all.  Rows of other blocks
 *    are left untouched in every output.
 * Outputs: O [BH][n][d]; lse (nullable) [BH][n] = log Den (with the subtracted maximum added back);
 *    parts (nullable) [BH][n][3][d] = the three numerator terms each divided by Den;
 *    wsum (nullable) [BH][n][2] = (sum of exact weights)/Den and (sum_U b_j alpha_j)/Den.
 * ------------------------------------------------------------------------------------------- */
ORACLE_API void oracle_pasa_attention(const double* Q, const double* K, const double* V, int64_t BH,
                                      int64_t n, int64_t d, int64_t b, int64_t G, double scale,
                                      const int32_t* idx, int64_t k, int32_t terms,
                                      const int32_t* q_blocks, int64_t n_qblocks, double* O,
                                      double* lse, double* parts, double* wsum) {
  int64_t NB = n_blocks_of(n, b);
  int64_t NG = (G > 0) ? (NB + G - 1) / G : 0;
  int use0 = (G > 0) && (terms & 1);
  int use1 = (G > 0) && (terms & 2);
  double* Kbar = (double*)malloc(sizeof(double) * (size_t)(BH * NB * d));
  double* VS = (double*)malloc(sizeof(double) * (size_t)(BH * NB * d));
  double* Hg = NG ? (double*)malloc(sizeof(double) * (size_t)(BH * NG * d * d)) : NULL;
  if (NG) {
    oracle_kv_stats(K, V, BH, n, d, b, G, Kbar, VS, NULL, Hg);
  } else {
    oracle_block_mean(K, BH, n, d, b, Kbar);
    memset(VS, 0, sizeof(double) * (size_t)(BH * NB * d));
  }
  if (!q_blocks) n_qblocks = NB;

#pragma omp parallel
  {
    double* e = (double*)malloc(sizeof(double) * (size_t)(k * b)); /* exact logits, then weights */
    double* z = (double*)malloc(sizeof(double) * (size_t)NB);      /* centroid logits / alpha    */
    char* sel = (char*)malloc((size_t)NB);
    double* ag = (double*)malloc(sizeof(double) * (size_t)(NG ? NG : 1));
    double* n0 = (double*)malloc(sizeof(double) * (size_t)d);
    double* n1 = (double*)malloc(sizeof(double) * (size_t)d);
    double* n2 = (double*)malloc(sizeof(double) * (size_t)d);
    double* qt = (double*)malloc(sizeof(double) * (size_t)d);
#pragma omp for collapse(2) schedule(dynamic)
    for (int64_t h = 0; h < BH; ++h)
      for (int64_t bi = 0; bi < n_qblocks; ++bi) {
        int64_t i = q_blocks ? q_blocks[bi] : bi;
        const int32_t* row = idx + (h * NB + i) * k;
        memset(sel, 0, (size_t)NB);
        for (int64_t s = 0; s < k; ++s) sel[row[s]] = 1;
        int64_t qlen = block_len(i, n, b);
        for (int64_t tq = 0; tq < qlen; ++tq) {
          int64_t t = i * b + tq;
          const double* q = Q + (h * n + t) * d;
          for (int64_t c = 0; c < d; ++c) qt[c] = q[c] * scale;
          double m = -INFINITY;
          /* exact logits over the selected blocks */
          for (int64_t s = 0; s < k; ++s) {
            int64_t j = row[s], len = block_len(j, n, b);
            for (int64_t u = 0; u < len; ++u) {
              const double* kr = K + (h * n + j * b + u) * d;
              double acc = 0.0;
#pragma omp simd reduction(+ : acc)
              for (int64_t c = 0; c < d; ++c) acc += qt[c] * kr[c];
              e[s * b + u] = acc;
              if (acc > m) m = acc;
            }
          }
          /* centroid logits over the unselected blocks */
          if (use0 || use1)
            for (int64_t j = 0; j < NB; ++j) {
              if (sel[j]) continue;
              const double* kb = Kbar + (h * NB + j) * d;
              double acc = 0.0;
#pragma omp simd reduction(+ : acc)
              for (int64_t c = 0; c < d; ++c) acc += qt[c] * kb[c];
              z[j] = acc;
              if (acc > m) m = acc;
            }
          /* first term of Eq.7 */
          double den_exact = 0.0, den_approx = 0.0;
          for (int64_t c = 0; c < d; ++c) n0[c] = n1[c] = n2[c] = 0.0;
          for (int64_t s = 0; s < k; ++s) {
            int64_t j = row[s], len = block_len(j, n, b);
            for (int64_t u = 0; u < len; ++u) {
              double p = exp(e[s * b + u] - m);
              den_exact += p;
              const double* vr = V + (h * n + j * b + u) * d;
              for (int64_t c = 0; c < d; ++c) n0[c] += p * vr[c];
            }
          }
          /* Eq.4 and the matching share of the normaliser; group sums of alpha for Eq.14 */
          if (use0 || use1) {
            for (int64_t g = 0; g < NG; ++g) ag[g] = 0.0;
            for (int64_t j = 0; j < NB; ++j) {
              if (sel[j]) continue;
              double a = exp(z[j] - m);
              ag[j / G] += a;
              if (use0) {
                den_approx += (double)block_len(j, n, b) * a;
                const double* vs = VS + (h * NB + j) * d;
                for (int64_t c = 0; c < d; ++c) n1[c] += a * vs[c];
              }
            }
          }
          /* Eq.14: (sum of alpha in the group) * (q~ Hg) */
          if (use1)
            for (int64_t g = 0; g < NG; ++g) {
              if (ag[g] == 0.0) continue;
              const double* Hm = Hg + (h * NG + g) * d * d;
              for (int64_t c = 0; c < d; ++c) {
                double acc = 0.0;
                for (int64_t a = 0; a < d; ++a) acc += qt[a] * Hm[a * d + c];
                n2[c] += ag[g] * acc;
              }
            }
          double den = den_exact + den_approx;
          double* o = O + (h * n + t) * d;
          for (int64_t c = 0; c < d; ++c) o[c] = (n0[c] + n1[c] + n2[c]) / den;
          if (lse) lse[h * n + t] = m + log(den);
          if (parts) {
            double* pp = parts + (h * n + t) * 3 * d;
            for (int64_t c = 0; c < d; ++c) {
              pp[c] = n0[c] / den;
              pp[d + c] = n1[c] / den;
              pp[2 * d + c] = n2[c] / den;
            }
          }
          if (wsum) {
            wsum[(h * n + t) * 2] = den_exact / den;
            wsum[(h * n + t) * 2 + 1] = den_approx / den;
          }
        }
      }
    free(e); free(z); free(sel); free(ag); free(n0); free(n1); free(n2); free(qt);
  }
  free(Kbar);
  free(VS);
  free(Hg);
}

/* ---------------------------------------------------------------------------------------------
 * Appendix "Error Analysis" quantities for one query token t of head slice h and one routing row.
 *   R   = sum_{j in U} alpha_j (H_j - Hg_{g(j)})            (Lemma 1 residual; alpha_j rescaled by
 *                                                             exp(-max_j z_j) on both sides)
 *   out[0] = ||R||_F
 *   out[1] = max_{j in U} ||H_j - Hg_{g(j)}||_F * sum_{j in U} alpha_j   (the Lemma 1 bound)
 * Hj [NB][d][d] and Hg [NG][d][d] are the statistics of that head; q is the scaled query (length d).
 * ------------------------------------------------------------------------------------------- */
ORACLE_API void oracle_lemma1(const double* q_scaled, const double* Kbar, const double* Hj,
                              const double* Hg, int64_t NB, int64_t d, int64_t G,
                              const int32_t* sel_idx, int64_t k, double* out) {
  char* sel = (char*)calloc((size_t)NB, 1);
  for (int64_t s = 0; s < k; ++s) sel[sel_idx[s]] = 1;
  double* z = (double*)malloc(sizeof(double) * (size_t)NB);
  double m = -INFINITY;
  for (int64_t j = 0; j < NB; ++j) {
    if (sel[j]) continue;
    double acc = 0.0;
    for (int64_t c = 0; c < d; ++c) acc += q_scaled[c] * Kbar[j * d + c];
    z[j] = acc;
    if (acc > m) m = acc;
  }
  double* R = (double*)calloc((size_t)(d * d), sizeof(double));
  double asum = 0.0, dmax = 0.0;
  for (int64_t j = 0; j < NB; ++j) {
    if (sel[j]) continue;
    double a = exp(z[j] - m);
    asum += a;
    const double* H = Hj + j * d * d;
    const double* M = Hg + (j / G) * d * d;
    double dev = 0.0;
    for (int64_t x = 0; x < d * d; ++x) {
      double df = H[x] - M[x];
      R[x] += a * df;
      dev += df * df;
    }
    dev = sqrt(dev);
    if (dev > dmax) dmax = dev;
  }
  double rn = 0.0;
  for (int64_t x = 0; x < d * d; ++x) rn += R[x] * R[x];
  out[0] = sqrt(rn);
  out[1] = dmax * asum;
  free(R); free(z); free(sel);
}
