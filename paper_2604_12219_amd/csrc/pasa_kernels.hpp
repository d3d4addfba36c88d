// Host-side launch interface between the C ABI (pasa_api.hip) and the kernel files.
// Every launcher validates nothing: shapes have been checked by the caller.  Each returns
// hipGetLastError() after its last launch and never synchronises.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

struct AttnParams {
  const uint16_t* q;
  const uint16_t* k;
  const uint16_t* v;
  uint16_t* o;
  float* lse;  // nullable
  int64_t stride_b, stride_h, stride_n;
  int32_t bh, H, n, nb, block, tail;  // tail = valid tokens of the last block
  float scale, c;                     // c = scale * log2(e), filled in by the launcher
  int32_t q_tiles, q_tiles_per_xcd;   // filled in by the launcher
  // sparse path only
  const int32_t* idx;    // not read by the attention kernel (it walks the bitmap; a caller without one has it built from idx)
  const uint32_t* mask;  // [BH][nb][mask_words]: bit j of a row = key block j is selected
  int32_t k_sel, mask_words;
  const uint16_t* st;    // bf16 [BH][n_chunks][64][d]: rows 0..31 block-mean keys, rows 32..63 block value
                         // sums of key blocks 32c..32c+31 (zero rows for blocks that do not exist)
  const uint16_t* hg;    // bf16 [BH][n_groups][d][d]: (scale * Hg)^T, row = value column, col = key column
  int32_t group, n_groups, n_chunks;
  // key-range slicing (sparse path): slice s covers chunks [s*n_chunks/n_slices, (s+1)*n_chunks/n_slices)
  int32_t n_slices;      // 1 = off (the attention kernel writes the output itself)
  float* part_o;         // fp32 [BH][n_slices][n][d]: unnormalised partial numerators
  float* part_ml;        // fp32 [BH][n_slices][n][2]: running maximum (log2 units) and partial normaliser
  uint32_t* queue;       // [8] work-item counters, one per XCD (reset by the launcher)
  int32_t items_per_xcd; // filled in by the launcher
};

// dense (sparse = false) or piecewise sparse attention; d in {64,128}, block in {64,128}
hipError_t pasa_launch_attn(AttnParams p, bool sparse, int d, hipStream_t stream);

struct StatsParams {
  const uint16_t* k;
  const uint16_t* v;
  int64_t stride_b, stride_h, stride_n;
  int32_t bh, H, n, nb, block, tail, d;
  int32_t group;     // > 0
  int32_t n_groups;  // ceil(nb / group)
  int32_t unit;      // blocks summed by one workgroup: a power of two that divides the group, at most 32
  int32_t n_units;   // units per head
  float scale;
  int32_t n_chunks;  // ceil(nb / 32)
  uint16_t* st;      // out bf16 [BH][n_chunks][64][d] (see AttnParams::st)
  float* partial;    // scratch fp32 [BH][n_units][d][d]: sum over the unit's blocks of H_j
  uint16_t* hg;      // out bf16 [BH][n_groups][d][d] (see AttnParams::hg)
  uint16_t* kbar_split;  // out [BH][nb][d] x 4 bytes: block-mean keys as split bf16 pairs in the score kernel's layout
                         // (per 32 elements 32 x hi then 32 x lo), so that scoring need not read K again
};
hipError_t pasa_launch_kv_stats(const StatsParams& p, hipStream_t stream);
// beta [BH][nb] fp32 = log(||H_j - Hg_{g(j)}||_F + eps); needs p.partial as pasa_launch_kv_stats left it
hipError_t pasa_launch_key_prior(const StatsParams& p, float eps, float* beta, hipStream_t stream);

struct ScoreParams {
  const uint16_t* q;
  const uint16_t* k;
  int64_t stride_b, stride_h, stride_n;
  int32_t bh, H, n, nb, block, d;
  float scale;
  const float* key_bias;  // nullable [BH][nb]
  float* qbar;            // scratch [BH][nb][d] x 4 bytes: block means as split bf16 pairs, per 32 elements 32 x hi then 32 x lo
  float* kbar;            // the same for the keys
  float* scores;          // out fp32 [BH][nb][nb]
  int32_t pool_k;         // 1: pool the keys here; 0: kbar already holds the split block-mean keys (left by the statistics kernel)
};
hipError_t pasa_launch_block_score(const ScoreParams& p, hipStream_t stream);

struct RouteParams {
  const float* scores;
  int32_t bh, nb, k_sel, mask_words;
  uint32_t seed_lo, seed_hi;
  float amp;
  int32_t gumbel;  // 0: uniform bias in [-amp, amp); 1: Gumbel(0, amp) bias
  int32_t* idx;
  uint32_t* mask;  // nullable
};
constexpr int kRouteMaxBlocks = 4096;  // keys of 4 rows are staged in 64 KB of LDS
hipError_t pasa_launch_route(const RouteParams& p, hipStream_t stream);
// n_bad[0] = number of rows (of `rows` = BH * nb) whose index list / bitmap row is not a valid selection of k_sel blocks
hipError_t pasa_launch_check_selection(const int32_t* idx, const uint32_t* mask, int64_t rows, int nb, int k_sel,
                                       int32_t* n_bad, hipStream_t stream);
// mask [rows][ceil(nb/32)] from idx [rows][k_sel]
hipError_t pasa_launch_mask_from_idx(const int32_t* idx, int64_t rows, int nb, int k_sel, uint32_t* mask, hipStream_t stream);
