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
    // The mean leaves as two bf16 numbers, hi = bf16(mean) and lo = bf16(mean - hi) (together 16 significant bits),
    // so that the score kernel can multiply on the bf16 matrix cores.  Row layout: per quarter of 32 elements one
    // 128-byte line, 32 x hi then 32 x lo.
    const float mean = s / (float)len;
    const __bf16 hi = (__bf16)mean;
    const __bf16 lo = (__bf16)(mean - (float)hi);
    uint16_t* dst = reinterpret_cast<uint16_t*>((which ? p.kbar : p.qbar) + ((int64_t)bh * p.nb + j) * D);
    dst[(tid >> 5) * 64 + (tid & 31)] = __builtin_bit_cast(uint16_t, hi);
    dst[(tid >> 5) * 64 + 32 + (tid & 31)] = __builtin_bit_cast(uint16_t, lo);
  }
}

// scores: a workgroup of four waves computes 64x64 tiles, each wave a 32x32 quarter of a tile, on the bf16 matrix
// cores: with q = qh + ql and k = kh + kl (the split pooled means), q.k = qh.kh + qh.kl + ql.kh up to 2^-16 relative,
// accumulated in fp32 -- three bf16 MFMAs (32x32x16) instead of eight fp32 ones (32x32x2) per 16 elements of the
// contraction, five times less matrix time.  The pooled means are row-major, and an MFMA operand wants one ROW per
// lane, which as a global load would touch 64 cache lines per instruction.  So the contraction runs in quarters of
// 32 elements: a quarter of a row (hi and lo) is exactly one 128-byte line, the workgroup fetches the quarters of
// its 64 + 64 rows with fully coalesced 16-byte loads (eight lanes per line), parks them in LDS (rows padded to 144
// bytes: conflict-free 16-byte reads down a column of rows), and every lane reads its operands from there.  Two LDS
// buffers: the loads of the next quarter are in flight during the MFMAs of the current one.  In a quarter, lane
// (x, h) holds elements [8h + 16m, 8h + 16m + 8) of its row for the MFMAs m = 0, 1.
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
template <int D>
__global__ void __launch_bounds__(256) score_gemm_kernel(ScoreParams p, int runs) {
  constexpr int QF = 32;               // elements per quarter-row (stored as 32 bf16 hi + 32 bf16 lo = 32 floats' worth of bytes)
  constexpr int NQ = D / QF;           // quarters
  constexpr int PITCH = QF * 4 + 16;   // bytes per LDS row
  __shared__ __attribute__((aligned(16))) char lds[2][128 * PITCH];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, x = lane & 31, h = lane >> 5;
  // Workgroup ids are decoded so that all workgroups of a head run on one XCD (the hardware deals consecutive ids
  // round-robin to the 8 XCDs): the head's pooled means are then fetched into one L2 instead of eight.
  const int n_tiles = (p.nb + 63) / 64;
  const int per_head = runs * n_tiles;
  // (with fewer than 16 heads that would leave XCDs idle: then ids simply run head by head)
  const bool by_xcd = p.bh >= 16;
  const int slot = by_xcd ? blockIdx.x >> 3 : blockIdx.x;
  const int bh = by_xcd ? (slot / per_head) * 8 + (blockIdx.x & 7) : slot / per_head;
  if (bh >= p.bh) return;  // padding workgroup: leaves before any barrier
  const int within = slot % per_head;
  const int run_id = within % runs, i0 = (within / runs) * 64;
  // A workgroup owns a strip of 64 score rows and walks a run of 64-column tiles along it: the 256-byte row
  // segments of consecutive tiles are then written by the same compute unit one after the other, and the cache
  // lines that straddle two tiles (rows are not a multiple of a line long) are completed in its L2 instead of going
  // to memory as two partial lines from two different L2s (3x the bytes of the scores themselves when every tile
  // was a workgroup of its own).
  const int run = (n_tiles + runs - 1) / runs;
  const int jt0 = run_id * run, jt1 = min(jt0 + run, n_tiles);
  const float* const qbar = p.qbar + (int64_t)bh * p.nb * D;
  const float* const kbar = p.kbar + (int64_t)bh * p.nb * D;
  // loader role: thread t fetches 16-byte chunk (t & 7) of tile rows (t >> 3) + 32 i, i = 0..3 (rows 0..63 are
  // pooled queries, 64..127 pooled keys); rows past the end are clamped: their products are never stored
  // (the staging registers are four named variables and the two roles are macros: with an array captured by a
  // lambda the compiler kept a copy of the staged values in scratch memory, four times the bytes of the scores)
  const int ld_row = tid >> 3, ld_col = (tid & 7) * 4;
  const float* const src0 = qbar + (int64_t)min(i0 + ld_row, p.nb - 1) * D + ld_col;
  const float* const src1 = qbar + (int64_t)min(i0 + ld_row + 32, p.nb - 1) * D + ld_col;
  const float* src2 = nullptr;
  const float* src3 = nullptr;
  float4 st0, st1, st2, st3;
#define PASA_SCORE_FETCH(qtr)                                        \
  do {                                                               \
    st0 = *reinterpret_cast<const float4*>(src0 + (qtr) * QF);       \
    st1 = *reinterpret_cast<const float4*>(src1 + (qtr) * QF);       \
    st2 = *reinterpret_cast<const float4*>(src2 + (qtr) * QF);       \
    st3 = *reinterpret_cast<const float4*>(src3 + (qtr) * QF);       \
  } while (0)
#define PASA_SCORE_PARK(buf)                                                                       \
  do {                                                                                             \
    *reinterpret_cast<float4*>(&lds[buf][(ld_row) * PITCH + (tid & 7) * 16]) = st0;                \
    *reinterpret_cast<float4*>(&lds[buf][(ld_row + 32) * PITCH + (tid & 7) * 16]) = st1;           \
    *reinterpret_cast<float4*>(&lds[buf][(ld_row + 64) * PITCH + (tid & 7) * 16]) = st2;           \
    *reinterpret_cast<float4*>(&lds[buf][(ld_row + 96) * PITCH + (tid & 7) * 16]) = st3;           \
  } while (0)
  // consumer role: wave (wi, wj) multiplies query rows 32 wi + x with key rows 32 wj + x
  const int a_off = (32 * (wave >> 1) + x) * PITCH + h * 16, b_off = (64 + 32 * (wave & 1) + x) * PITCH + h * 16;
#pragma unroll 1
  for (int jt = jt0; jt < jt1; ++jt) {
    const int j0 = jt * 64;
    src2 = kbar + (int64_t)min(j0 + ld_row, p.nb - 1) * D + ld_col;
    src3 = kbar + (int64_t)min(j0 + ld_row + 32, p.nb - 1) * D + ld_col;
    f32x16 acc = {0};
    PASA_SCORE_FETCH(0);
    PASA_SCORE_PARK(0);  // buffer 0 was last read two barriers ago
    __syncthreads();
#pragma unroll
    for (int qtr = 0; qtr < NQ; ++qtr) {
      if (qtr + 1 < NQ) PASA_SCORE_FETCH(qtr + 1);
      const char* buf = lds[qtr & 1];
      // operand fragments of 8 bf16: [m] hi, [2 + m] lo of elements 8h + 16m .. + 8
      bf16x8 a[4], b[4];
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        a[c] = *reinterpret_cast<const bf16x8*>(buf + a_off + 64 * (c >> 1) + 32 * (c & 1));
        b[c] = *reinterpret_cast<const bf16x8*>(buf + b_off + 64 * (c >> 1) + 32 * (c & 1));
      }
#pragma unroll
      for (int m = 0; m < 2; ++m) {
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[2 + m], b[m], acc, 0, 0, 0);  // ql kh  (small terms first)
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[m], b[2 + m], acc, 0, 0, 0);  // qh kl
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[m], b[m], acc, 0, 0, 0);      // qh kh
      }
      if (qtr + 1 < NQ) {
        PASA_SCORE_PARK((qtr + 1) & 1);  // the other buffer: its readers finished before the previous barrier
        __syncthreads();
      }
    }
    // result register 4g + r of lane (x, h) is row 8g + 4h + r, column x of the wave's quarter
    const int j = j0 + 32 * (wave & 1) + x;
    if (j < p.nb) {
      const float bias = p.key_bias ? p.key_bias[(int64_t)bh * p.nb + j] : 0.f;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int i = i0 + 32 * (wave >> 1) + 8 * (r >> 2) + 4 * h + (r & 3);
        if (i < p.nb) p.scores[((int64_t)bh * p.nb + i) * p.nb + j] = fmaf(acc[r], p.scale, bias);
      }
    }
  }
#undef PASA_SCORE_FETCH
#undef PASA_SCORE_PARK
}

}  // namespace

hipError_t pasa_launch_block_score(const ScoreParams& p, hipStream_t stream) {
  const dim3 gp(p.nb, p.bh, p.pool_k ? 2 : 1);  // z = 0 pools the queries, z = 1 the keys
  const int tiles = (p.nb + 63) / 64;
  // strips of 64 rows; a strip is cut into runs of column tiles only as far as it takes to fill the device
  const int64_t strips = (int64_t)tiles * p.bh;
  int runs = (int)((2048 + strips - 1) / strips);
  runs = runs < 1 ? 1 : runs > tiles ? tiles : runs;
  const dim3 gg((unsigned)((p.bh >= 16 ? 8 * ((p.bh + 7) / 8) : p.bh) * runs * tiles));
  if (p.d == 128) {
    hipLaunchKernelGGL(pool_mean_kernel<128>, gp, dim3(256), 0, stream, p);
    hipLaunchKernelGGL(score_gemm_kernel<128>, gg, dim3(256), 0, stream, p, runs);
  } else {
    hipLaunchKernelGGL(pool_mean_kernel<64>, gp, dim3(256), 0, stream, p);
    hipLaunchKernelGGL(score_gemm_kernel<64>, gg, dim3(256), 0, stream, p, runs);
  }
  return hipGetLastError();
}
