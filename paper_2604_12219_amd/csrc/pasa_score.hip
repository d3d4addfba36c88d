// Stage 1 of the PASA forward on gfx950: block-pooled routing logits (Eq.8 without its softmax).
//   qbar_i = mean of the valid rows of query block i, kbar_j likewise          (HBM-bound reads)
//   scores[bh,i,j] = scale * qbar_i . kbar_j + key_bias[bh,j]                  (fp32 throughout)
#include "pasa_kernels.hpp"

namespace {

// One workgroup per (block, head, tensor): 16-byte loads along d, partial sums over rows in
// registers, a 16-way (or 32-way) reduction through LDS.
template <int D>
__global__ void __launch_bounds__(256) pool_mean_kernel(ScoreParams p) {
  constexpr int CPR = D / 8, RPP = 256 / CPR;  // 16-byte chunks per row, rows per pass
  __shared__ float part[RPP][D];
  const int j = blockIdx.x, bh = blockIdx.y, which = blockIdx.z;
  const int tid = threadIdx.x, c = tid % CPR, r = tid / CPR;
  const int64_t head_off = (int64_t)(bh / p.H) * p.stride_b + (int64_t)(bh % p.H) * p.stride_h;
  const uint16_t* src = (which ? p.k : p.q) + head_off;
  const int row0 = j * p.block, len = min(p.block, p.n - row0);
  float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  for (int row = r; row < len; row += RPP) {
    const uint4 raw = *reinterpret_cast<const uint4*>(src + (int64_t)(row0 + row) * p.stride_n + c * 8);
    const uint32_t wds[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      acc[2 * e] += __uint_as_float(wds[e] << 16);
      acc[2 * e + 1] += __uint_as_float(wds[e] & 0xffff0000u);
    }
  }
#pragma unroll
  for (int e = 0; e < 8; ++e) part[r][c * 8 + e] = acc[e];
  __syncthreads();
  if (tid < D) {
    float s = 0.f;
#pragma unroll
    for (int rr = 0; rr < RPP; ++rr) s += part[rr][tid];
    float* dst = (which ? p.kbar : p.qbar) + ((int64_t)bh * p.nb + j) * D;
    dst[tid] = s / (float)len;
  }
}

// scores: one wave per 32x32 tile, fp32 MFMA (32x32x2: A is 32 rows x 2, B is 2 x 32 columns, one float of
// each per lane).  The contraction order is free as long as both operands agree, so lane (x = lane & 31,
// h = lane >> 5) keeps d/2 consecutive floats of row i0 + x of the pooled queries and of row j0 + x of the
// pooled keys, elements [h*d/2, (h+1)*d/2), straight from global memory (the pooled means of a head are a
// few hundred KB: L2 traffic), and step s multiplies element s of both.  The four waves of a workgroup
// take four neighbouring column tiles of the same row tile.
typedef float f32x16 __attribute__((ext_vector_type(16)));
template <int D>
__global__ void __launch_bounds__(256) score_gemm_kernel(ScoreParams p) {
  constexpr int HALF = D / 2;
  const int bh = blockIdx.z, i0 = blockIdx.y * 32, j0 = (blockIdx.x * 4 + (threadIdx.x >> 6)) * 32;
  if (j0 >= p.nb) return;
  const int lane = threadIdx.x & 63, x = lane & 31, h = lane >> 5;
  const float* qa = p.qbar + ((int64_t)bh * p.nb + min(i0 + x, p.nb - 1)) * D + h * HALF;  // rows past the end: clamped, never stored
  const float* kb = p.kbar + ((int64_t)bh * p.nb + min(j0 + x, p.nb - 1)) * D + h * HALF;
  float4 a[HALF / 4], b[HALF / 4];
#pragma unroll
  for (int c = 0; c < HALF / 4; ++c) {
    a[c] = reinterpret_cast<const float4*>(qa)[c];
    b[c] = reinterpret_cast<const float4*>(kb)[c];
  }
  f32x16 acc = {0};
#pragma unroll
  for (int c = 0; c < HALF / 4; ++c) {
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a[c].x, b[c].x, acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a[c].y, b[c].y, acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a[c].z, b[c].z, acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a[c].w, b[c].w, acc, 0, 0, 0);
  }
  // result register 4g + r of lane (x, h) is row 8g + 4h + r, column x of the tile
  const int j = j0 + x;
  if (j >= p.nb) return;
  const float bias = p.key_bias ? p.key_bias[(int64_t)bh * p.nb + j] : 0.f;
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    const int i = i0 + 8 * (r >> 2) + 4 * h + (r & 3);
    if (i < p.nb) p.scores[((int64_t)bh * p.nb + i) * p.nb + j] = fmaf(acc[r], p.scale, bias);
  }
}

}  // namespace

hipError_t pasa_launch_block_score(const ScoreParams& p, hipStream_t stream) {
  const dim3 gp(p.nb, p.bh, 2);
  const int tiles = (p.nb + 31) / 32;
  const dim3 gg((tiles + 3) / 4, tiles, p.bh);
  if (p.d == 128) {
    hipLaunchKernelGGL(pool_mean_kernel<128>, gp, dim3(256), 0, stream, p);
    hipLaunchKernelGGL(score_gemm_kernel<128>, gg, dim3(256), 0, stream, p);
  } else {
    hipLaunchKernelGGL(pool_mean_kernel<64>, gp, dim3(256), 0, stream, p);
    hipLaunchKernelGGL(score_gemm_kernel<64>, gg, dim3(256), 0, stream, p);
  }
  return hipGetLastError();
}
