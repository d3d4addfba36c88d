// Key/value block statistics of the PASA forward (Eq.4's inner sum, Eq.5, Eq.12) for gfx950.
//
//   Kbar_j = mean_n K_{j,n}   -> bf16, row (j & 31)      of tile [BH][j >> 5][64][d]
//   VS_j   = sum_n  V_{j,n}   -> bf16, row 32 + (j & 31) of the same tile (one tile = one chunk of 32
//                                 blocks, laid out so the attention kernel streams it like a K tile)
//   Hg_g   = mean_{j in group g} H_j,  H_j = sum_n (K_{j,n} - Kbar_j)^T V_{j,n} = K_j^T V_j - Kbar_j^T VS_j
//
// H_j is never written to memory.  A workgroup owns a "unit" of consecutive blocks (a whole group
// when the group has at most 32 blocks, else 32 blocks of it), accumulates sum_j K_j^T V_j on the
// matrix cores with fp32 accumulators (both operands are fetched from the row-major LDS tiles with
// transposing LDS reads, the contraction runs over tokens), subtracts the rank-one term of every
// block in fp32, and writes the unit's sum.  A second small kernel averages the units of a group,
// applies the logit scale and stores the transposed matrix as bf16, row-major [value column][key
// column], which the attention kernel streams through LDS exactly like a K tile.
#include "pasa_device.hpp"
#include "pasa_kernels.hpp"

namespace {

typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));

// The sweep both kernels below share.  A workgroup of four waves owns a unit of consecutive key blocks [j_lo, j_hi)
// of one head and streams their 64-row K and V tiles through LDS (the next tile's global loads are in flight
// during the MFMAs of the current one).  Wave w accumulates the (d_in, d_out) quarter (w >> 1, w & 1) of
// sum K^T V in acc[TI][TI] (32x32 tiles, both operands by transposing LDS reads, the contraction runs over tokens).
// The column sums the rank-one term needs come from the matrix cores as well, as products with an all-ones
// operand: ksum[a][r] = sum over the block's tokens of K[:, 32 (tin0 + a) + mfma_row(r, h)] (what a lane needs to
// correct its rows of the accumulator) and vsum[b][*] = sum of V[:, 32 (tout0 + b) + (lane & 31)] (every register
// the same value).  After the last tile of block j, done(j, len, acc, ksum, vsum) runs with len = valid tokens of
// the block; the sums restart at zero afterwards, acc is the callback's to reset or keep.  Rows beyond the last
// token are staged as zeros, so they add nothing anywhere.
template <int D, typename BlockDone>
PASA_DEVICE void sweep_unit(const StatsParams& p, int bh, int j_lo, int j_hi, char* k_lds, char* v_lds,
                            f32x16 (&acc)[D / 64][D / 64], BlockDone&& done) {
  constexpr int T = 256;
  constexpr int TI = D / 64;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int64_t head_off = (int64_t)(bh / p.H) * p.stride_b + (int64_t)(bh % p.H) * p.stride_h;
  const uint16_t* const kb = p.k + head_off;
  const uint16_t* const vb = p.v + head_off;
  const int tiles_per_block = p.block / 64;
  const int tin0 = (wave >> 1) * TI, tout0 = (wave & 1) * TI;
  bf16x8 ones;
#pragma unroll
  for (int e = 0; e < 8; ++e) ones[e] = (__bf16)1.0f;
  f32x16 ksum[TI], vsum[TI];
#pragma unroll
  for (int a = 0; a < TI; ++a) ksum[a] = vsum[a] = f32x16{0};

  TileStage<D, T> sk, sv;
  const int n_tiles = (j_hi - j_lo) * tiles_per_block;
  auto tile_row0 = [&](int t) { return (j_lo + t / tiles_per_block) * p.block + (t % tiles_per_block) * 64; };
  sk.load(kb, p.stride_n, tile_row0(0), 64, p.n, tid);
  sv.load(vb, p.stride_n, tile_row0(0), 64, p.n, tid);
  for (int t = 0; t < n_tiles; ++t) {
    sk.store(k_lds, 64, tid);
    sv.store(v_lds, 64, tid);
    __syncthreads();
    if (t + 1 < n_tiles) {
      sk.load(kb, p.stride_n, tile_row0(t + 1), 64, p.n, tid);
      sv.load(vb, p.stride_n, tile_row0(t + 1), 64, p.n, tid);
    }
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      bf16x8 af[TI], bf[TI];
#pragma unroll
      for (int a = 0; a < TI; ++a) af[a] = col_frag<D>(k_lds, 16 * ks, 32 * (tin0 + a), lane);
#pragma unroll
      for (int b = 0; b < TI; ++b) bf[b] = col_frag<D>(v_lds, 16 * ks, 32 * (tout0 + b), lane);
#pragma unroll
      for (int a = 0; a < TI; ++a) {
        ksum[a] = mfma32(af[a], ones, ksum[a]);
#pragma unroll
        for (int b = 0; b < TI; ++b) acc[a][b] = mfma32(af[a], bf[b], acc[a][b]);
      }
#pragma unroll
      for (int b = 0; b < TI; ++b) vsum[b] = mfma32(ones, bf[b], vsum[b]);
    }
    if ((t % tiles_per_block) == tiles_per_block - 1) {
      const int j = j_lo + t / tiles_per_block;
      done(j, (j == p.nb - 1) ? p.tail : p.block, acc, ksum, vsum);
#pragma unroll
      for (int a = 0; a < TI; ++a) ksum[a] = vsum[a] = f32x16{0};
    }
    __syncthreads();  // tiles consumed
  }
}

// (two workgroups per CU: the accumulators of the matrix and of the column sums take 128 + 64 registers at d = 128)
template <int D>
__global__ void __launch_bounds__(256, 2) kv_stats_kernel(StatsParams p) {
  constexpr int TI = D / 64;  // 32x32 result tiles per wave along each of d_in, d_out
  constexpr int TILE_BYTES = 64 * 2 * D;
  __shared__ __attribute__((aligned(16))) char smem[2 * TILE_BYTES];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, h = lane >> 5;
  const int u = blockIdx.x, bh = blockIdx.y;
  const int j_lo = u * p.unit, j_hi = min(j_lo + p.unit, p.nb);
  const int tin0 = (wave >> 1) * TI, tout0 = (wave & 1) * TI;

  f32x16 acc[TI][TI];
#pragma unroll
  for (int a = 0; a < TI; ++a)
#pragma unroll
    for (int b = 0; b < TI; ++b) acc[a][b] = f32x16{0};

  sweep_unit<D>(p, bh, j_lo, j_hi, smem, smem + TILE_BYTES, acc,
                [&](int j, int len, f32x16 (&acc)[TI][TI], const f32x16 (&ksum)[TI], const f32x16 (&vsum)[TI]) {
    const float inv_len = 1.0f / (float)len;
    uint16_t* const strow = p.st + (((int64_t)bh * p.n_chunks + (j >> 5)) * 64 + (j & 31)) * D;
#pragma unroll
    for (int a = 0; a < TI; ++a) {
      // H_j = K_j^T V_j - Kbar_j^T VS_j: the rank-one term leaves the running sum in fp32, before any rounding
#pragma unroll
      for (int b = 0; b < TI; ++b)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[a][b][r] -= ksum[a][r] * inv_len * vsum[b][0];
      // block-mean key: the waves of the first d_out half hold every d_in row between them; lanes 0 and 32 write
      // their 4 x 4 consecutive rows
      if ((wave & 1) == 0 && (lane & 31) == 0) {
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          bf16x4 m4;
#pragma unroll
          for (int r = 0; r < 4; ++r) m4[r] = (__bf16)(ksum[a][4 * g + r] * inv_len);
          *reinterpret_cast<bf16x4*>(strow + 32 * (tin0 + a) + 8 * g + 4 * h) = m4;
          // the same means as split bf16 pairs (hi + lo, 16 significant bits) for the score kernel
          bf16x4 lo4;
#pragma unroll
          for (int r = 0; r < 4; ++r) lo4[r] = (__bf16)(ksum[a][4 * g + r] * inv_len - (float)m4[r]);
          uint16_t* const krow = p.kbar_split + ((int64_t)bh * p.nb + j) * (2 * D) + 64 * (tin0 + a) + 8 * g + 4 * h;
          *reinterpret_cast<bf16x4*>(krow) = m4;
          *reinterpret_cast<bf16x4*>(krow + 32) = lo4;
        }
      }
    }
    // block value sum: the waves of the first d_in half, one value column per lane
    if ((wave >> 1) == 0 && h == 0) {
#pragma unroll
      for (int b = 0; b < TI; ++b) strow[32 * D + 32 * (tout0 + b) + lane] = __builtin_bit_cast(uint16_t, (__bf16)vsum[b][0]);
    }
  });

  const bool is_col = tid < 2 * D;
  if (j_hi == p.nb && is_col) {  // rows of blocks that do not exist read as zero
    const int col = tid % D;
    for (int j = p.nb; j < 32 * p.n_chunks; ++j)
      p.st[(((int64_t)bh * p.n_chunks + (j >> 5)) * 64 + (tid >= D ? 32 : 0) + (j & 31)) * D + col] = 0;
  }

  float* out = p.partial + ((int64_t)bh * p.n_units + u) * D * D;
#pragma unroll
  for (int a = 0; a < TI; ++a)
#pragma unroll
    for (int b = 0; b < TI; ++b)
#pragma unroll
      for (int r = 0; r < 16; ++r)
        out[(32 * (tin0 + a) + mfma_row(r, h)) * D + 32 * (tout0 + b) + (lane & 31)] = acc[a][b][r];

  // A group that is one unit: its matrix is finished here, (scale * Hg)^T as bf16, row = value
  // column (hg_finish_kernel does the same for groups of several units).  Registers 4g .. 4g + 3 of a lane are four
  // consecutive key columns of its value column.
  if (p.unit == p.group) {
    const float f = p.scale / (float)(j_hi - j_lo);
    uint16_t* hg = p.hg + ((int64_t)bh * p.n_groups + u) * D * D;
#pragma unroll
    for (int a = 0; a < TI; ++a)
#pragma unroll
      for (int b = 0; b < TI; ++b)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          bf16x4 v4;
#pragma unroll
          for (int r = 0; r < 4; ++r) v4[r] = (__bf16)(acc[a][b][4 * g + r] * f);
          *reinterpret_cast<bf16x4*>(hg + (int64_t)(32 * (tout0 + b) + (lane & 31)) * D + 32 * (tin0 + a) + 8 * g + 4 * h) = v4;
        }
  }
}

// partial [BH][n_units][d_in][d_out] fp32 -> hg [BH][n_groups][d_out][d_in] bf16 = (scale * Hg)^T
template <int D>
__global__ void __launch_bounds__(256) hg_finish_kernel(StatsParams p) {
  const int g = blockIdx.x, bh = blockIdx.y;
  const int upg = (p.group >= p.nb) ? p.n_units : p.group / p.unit;  // units per group
  const int u_lo = g * upg, u_hi = min(u_lo + upg, p.n_units);
  const int blocks_in_group = min((g + 1) * p.group, p.nb) - g * p.group;
  const float f = p.scale / (float)blocks_in_group;
  const float* part = p.partial + (int64_t)bh * p.n_units * D * D;
  uint16_t* out = p.hg + ((int64_t)bh * p.n_groups + g) * D * D;
  // 8 consecutive key columns of one value column per thread; the grid's z dimension covers the matrix
  for (int x = threadIdx.x + 256 * blockIdx.z; x < D * D / 8; x += 256 * gridDim.z) {
    const int d_out = x % D, d_in0 = (x / D) * 8;
    bf16x8 v;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      float sum = 0.f;
      for (int u = u_lo; u < u_hi; ++u) sum += part[((int64_t)u * D + d_in0 + i) * D + d_out];
      v[i] = (__bf16)(sum * f);
    }
    *reinterpret_cast<bf16x8*>(out + (int64_t)d_out * D + d_in0) = v;
  }
}

// Covariance-aware routing prior (Eq.8): beta_j = log(|| H_j - Hg_{g(j)} ||_F + eps) for every key block.
// The same sweep as kv_stats_kernel, but H_j is formed per block and compared, element by element in fp32, with the
// group mean, which the workgroup first sums up from the unit sums that kv_stats_kernel left (`partial`).
// Nothing but beta is written.
template <int D>
__global__ void __launch_bounds__(256) key_prior_kernel(StatsParams p, float eps, float* beta) {
  constexpr int TI = D / 64;
  constexpr int TILE_BYTES = 64 * 2 * D;
  __shared__ __attribute__((aligned(16))) char smem[2 * TILE_BYTES];
  __shared__ float red_s[2][4];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, h = lane >> 5;
  const int u = blockIdx.x, bh = blockIdx.y;
  const int j_lo = u * p.unit, j_hi = min(j_lo + p.unit, p.nb);
  const int tin0 = (wave >> 1) * TI, tout0 = (wave & 1) * TI;

  // the group this unit belongs to, and its mean: sum of the group's unit sums / blocks in the group
  const int g = j_lo / p.group;
  const int upg = (p.group >= p.nb) ? p.n_units : p.group / p.unit;  // units per group
  const int u_lo = g * upg, u_hi = min(u_lo + upg, p.n_units);
  const float inv_blocks = 1.0f / (float)(min((g + 1) * p.group, p.nb) - g * p.group);
  f32x16 mean[TI][TI];
#pragma unroll
  for (int a = 0; a < TI; ++a)
#pragma unroll
    for (int b = 0; b < TI; ++b) {
      mean[a][b] = f32x16{0};
      for (int uu = u_lo; uu < u_hi; ++uu) {
        const float* part = p.partial + ((int64_t)bh * p.n_units + uu) * D * D;
#pragma unroll
        for (int r = 0; r < 16; ++r)
          mean[a][b][r] += part[(32 * (tin0 + a) + mfma_row(r, h)) * D + 32 * (tout0 + b) + (lane & 31)];
      }
#pragma unroll
      for (int r = 0; r < 16; ++r) mean[a][b][r] *= inv_blocks;
    }

  f32x16 acc[TI][TI];
#pragma unroll
  for (int a = 0; a < TI; ++a)
#pragma unroll
    for (int b = 0; b < TI; ++b) acc[a][b] = f32x16{0};

  int parity = 0;  // red_s is double-buffered: one barrier per block is enough
  sweep_unit<D>(p, bh, j_lo, j_hi, smem, smem + TILE_BYTES, acc,
                [&](int j, int len, f32x16 (&acc)[TI][TI], const f32x16 (&ksum)[TI], const f32x16 (&vsum)[TI]) {
    const float inv_len = 1.0f / (float)len;
    float ss = 0.f;
#pragma unroll
    for (int a = 0; a < TI; ++a)
#pragma unroll
      for (int b = 0; b < TI; ++b) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const float hj = acc[a][b][r] - ksum[a][r] * inv_len * vsum[b][0];
          const float dlt = hj - mean[a][b][r];
          ss = fmaf(dlt, dlt, ss);
        }
        acc[a][b] = f32x16{0};
      }
#pragma unroll
    for (int sh = 32; sh >= 1; sh >>= 1) ss += __shfl_xor(ss, sh);
    if (lane == 0) red_s[parity][wave] = ss;
    __syncthreads();
    if (tid == 0)
      beta[(int64_t)bh * p.nb + j] = logf(sqrtf(red_s[parity][0] + red_s[parity][1] + red_s[parity][2] + red_s[parity][3]) + eps);
    parity ^= 1;  // the other half is next written after the sweep's own barrier and this one
  });
}

}  // namespace

hipError_t pasa_launch_kv_stats(const StatsParams& p, hipStream_t stream) {
  // few groups (long groups, or one global matrix): spread each matrix over several workgroups
  const int split = (int64_t)p.n_groups * p.bh < 2048 ? p.d * p.d / 8 / 256 : 1;
  dim3 g1(p.n_units, p.bh), g2(p.n_groups, p.bh, split);
  const bool finish = p.unit != p.group;  // otherwise a unit is a whole group and kv_stats_kernel writes the matrices itself
  if (p.d == 128) {
    hipLaunchKernelGGL(kv_stats_kernel<128>, g1, dim3(256), 0, stream, p);
    if (finish) hipLaunchKernelGGL(hg_finish_kernel<128>, g2, dim3(256), 0, stream, p);
  } else {
    hipLaunchKernelGGL(kv_stats_kernel<64>, g1, dim3(256), 0, stream, p);
    if (finish) hipLaunchKernelGGL(hg_finish_kernel<64>, g2, dim3(256), 0, stream, p);
  }
  return hipGetLastError();
}

hipError_t pasa_launch_key_prior(const StatsParams& p, float eps, float* beta, hipStream_t stream) {
  dim3 g1(p.n_units, p.bh);
  if (p.d == 128) hipLaunchKernelGGL(key_prior_kernel<128>, g1, dim3(256), 0, stream, p, eps, beta);
  else hipLaunchKernelGGL(key_prior_kernel<64>, g1, dim3(256), 0, stream, p, eps, beta);
  return hipGetLastError();
}
