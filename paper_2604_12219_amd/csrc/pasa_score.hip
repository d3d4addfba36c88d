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

// scores: a workgroup of four waves computes a 64x64 tile, each wave a 32x32 quarter of it, with the fp32
// MFMA (32x32x2: A is 32 rows x 2, B is 2 x 32 columns, one float of each per lane).  The pooled means are
// row-major, and an MFMA operand wants one ROW per lane, which as a global load would touch 64 cache lines
// per instruction.  So the contraction runs in quarters of 32 floats: a quarter of a row is exactly one
// 128-byte line, the workgroup fetches the quarters of its 64 + 64 rows with fully coalesced 16-byte loads
// (eight lanes per line), parks them in LDS (rows padded to 144 bytes: conflict-free 16-byte reads down a
// column of rows), and every lane reads its operands from there.  Two LDS buffers: the loads of the next
// quarter are in flight during the MFMAs of the current one.  The contraction order is free as long as both
// operands agree: in a quarter, lane (x, h) holds floats [16h, 16h + 16) of its row, and step s multiplies
// float s of the h = 0 lanes and float 16 + s of the h = 1 lanes.
typedef float f32x16 __attribute__((ext_vector_type(16)));
template <int D>
__global__ void __launch_bounds__(256) score_gemm_kernel(ScoreParams p) {
  constexpr int QF = 32;               // floats per quarter-row
  constexpr int NQ = D / QF;           // quarters
  constexpr int PITCH = QF * 4 + 16;   // bytes per LDS row
  __shared__ __attribute__((aligned(16))) char lds[2][128 * PITCH];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, x = lane & 31, h = lane >> 5;
  const int bh = blockIdx.z, i0 = blockIdx.y * 64, j0 = blockIdx.x * 64;
  const float* const qbar = p.qbar + (int64_t)bh * p.nb * D;
  const float* const kbar = p.kbar + (int64_t)bh * p.nb * D;
  // loader role: thread t fetches 16-byte chunk (t & 7) of tile rows (t >> 3) + 32 i, i = 0..3 (rows 0..63 are
  // pooled queries, 64..127 pooled keys); rows past the end are clamped: their products are never stored
  const float* src[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int r = (tid >> 3) + 32 * i;
    const float* base = r < 64 ? qbar + (int64_t)min(i0 + r, p.nb - 1) * D : kbar + (int64_t)min(j0 + r - 64, p.nb - 1) * D;
    src[i] = base + (tid & 7) * 4;
  }
  float4 stage[4];
  auto fetch = [&](int qtr) {
#pragma unroll
    for (int i = 0; i < 4; ++i) stage[i] = *reinterpret_cast<const float4*>(src[i] + qtr * QF);
  };
  auto park = [&](int buf) {
#pragma unroll
    for (int i = 0; i < 4; ++i)
      *reinterpret_cast<float4*>(&lds[buf][((tid >> 3) + 32 * i) * PITCH + (tid & 7) * 16]) = stage[i];
  };
  // consumer role: wave (wi, wj) multiplies query rows 32 wi + x with key rows 32 wj + x
  const int a_off = (32 * (wave >> 1) + x) * PITCH + h * 64, b_off = (64 + 32 * (wave & 1) + x) * PITCH + h * 64;
  f32x16 acc = {0};
  fetch(0);
  park(0);
  __syncthreads();
#pragma unroll
  for (int qtr = 0; qtr < NQ; ++qtr) {
    if (qtr + 1 < NQ) fetch(qtr + 1);
    const char* buf = lds[qtr & 1];
    float4 a[4], b[4];
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      a[c] = *reinterpret_cast<const float4*>(buf + a_off + 16 * c);
      b[c] = *reinterpret_cast<const float4*>(buf + b_off + 16 * c);
    }
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a[c].x, b[c].x, acc, 0, 0, 0);
      acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a[c].y, b[c].y, acc, 0, 0, 0);
      acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a[c].z, b[c].z, acc, 0, 0, 0);
      acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a[c].w, b[c].w, acc, 0, 0, 0);
    }
    if (qtr + 1 < NQ) {
      park((qtr + 1) & 1);  // the other buffer: its readers finished before the previous barrier
      __syncthreads();
    }
  }
  // result register 4g + r of lane (x, h) is row 8g + 4h + r, column x of the wave's quarter
  const int j = j0 + 32 * (wave & 1) + x;
  if (j >= p.nb) return;
  const float bias = p.key_bias ? p.key_bias[(int64_t)bh * p.nb + j] : 0.f;
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    const int i = i0 + 32 * (wave >> 1) + 8 * (r >> 2) + 4 * h + (r & 3);
    if (i < p.nb) p.scores[((int64_t)bh * p.nb + i) * p.nb + j] = fmaf(acc[r], p.scale, bias);
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
