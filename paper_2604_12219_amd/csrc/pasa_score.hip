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

// scores tile of 64x64 per workgroup; operands staged transposed in LDS ([d][row]) so that a thread
// reads its 4 rows / 4 columns with one 16-byte LDS read per d.
template <int D>
__global__ void __launch_bounds__(256) score_gemm_kernel(ScoreParams p) {
  constexpr int LD = 68;  // padded leading dimension (floats), keeps 16-byte alignment
  __shared__ __attribute__((aligned(16))) float a_s[D][LD];
  __shared__ __attribute__((aligned(16))) float b_s[D][LD];
  const int bh = blockIdx.z, i0 = blockIdx.y * 64, j0 = blockIdx.x * 64;
  const int tid = threadIdx.x;
  const float* qa = p.qbar + (int64_t)bh * p.nb * D;
  const float* kb = p.kbar + (int64_t)bh * p.nb * D;
  for (int x = tid; x < 64 * D; x += 256) {
    const int row = x / D, dd = x % D;
    a_s[dd][row] = (i0 + row < p.nb) ? qa[(int64_t)(i0 + row) * D + dd] : 0.f;
    b_s[dd][row] = (j0 + row < p.nb) ? kb[(int64_t)(j0 + row) * D + dd] : 0.f;
  }
  __syncthreads();
  const int ty = tid / 16, tx = tid % 16;
  float acc[4][4] = {};
#pragma unroll 4
  for (int dd = 0; dd < D; ++dd) {
    const float4 a = *reinterpret_cast<const float4*>(&a_s[dd][ty * 4]);
    const float4 b = *reinterpret_cast<const float4*>(&b_s[dd][tx * 4]);
    const float av[4] = {a.x, a.y, a.z, a.w}, bv[4] = {b.x, b.y, b.z, b.w};
#pragma unroll
    for (int y = 0; y < 4; ++y)
#pragma unroll
      for (int x = 0; x < 4; ++x) acc[y][x] = fmaf(av[y], bv[x], acc[y][x]);
  }
#pragma unroll
  for (int y = 0; y < 4; ++y) {
    const int i = i0 + ty * 4 + y;
    if (i >= p.nb) continue;
#pragma unroll
    for (int x = 0; x < 4; ++x) {
      const int j = j0 + tx * 4 + x;
      if (j >= p.nb) continue;
      float s = acc[y][x] * p.scale;
      if (p.key_bias) s += p.key_bias[(int64_t)bh * p.nb + j];
      p.scores[((int64_t)bh * p.nb + i) * p.nb + j] = s;
    }
  }
}

}  // namespace

hipError_t pasa_launch_block_score(const ScoreParams& p, hipStream_t stream) {
  const dim3 gp(p.nb, p.bh, 2);
  const int tiles = (p.nb + 63) / 64;
  const dim3 gg(tiles, tiles, p.bh);
  if (p.d == 128) {
    hipLaunchKernelGGL(pool_mean_kernel<128>, gp, dim3(256), 0, stream, p);
    hipLaunchKernelGGL(score_gemm_kernel<128>, gg, dim3(256), 0, stream, p);
  } else {
    hipLaunchKernelGGL(pool_mean_kernel<64>, gp, dim3(256), 0, stream, p);
    hipLaunchKernelGGL(score_gemm_kernel<64>, gg, dim3(256), 0, stream, p);
  }
  return hipGetLastError();
}
