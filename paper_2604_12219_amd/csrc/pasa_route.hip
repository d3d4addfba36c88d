// Stage 2 of the PASA forward on gfx950: per-row top-k block selection with a seeded stochastic
// bias (Eq.2; Sec. "Stochastic Routing").  One wavefront per (head, query block) row:
//   1. r_j = fmaf(amp, w_j, s_j) with w_j from Philox4x32-10 (one call serves 4 consecutive j),
//      mapped to an order-preserving uint32 key (-0 folded onto +0) and kept in LDS;
//   2. the k-th largest key is found by a 32-step bitwise search, each step a ballot count;
//   3. keys above the threshold are selected, ties at the threshold are taken in ascending j until
//      k are chosen; the ascending index list and the selection bitmap are emitted with
//      ballot + prefix popcount, so the output order needs no sort.
// Integer work throughout except the single fused multiply-add, hence bit-reproducible on a CPU.
// (The Gumbel variant of the bias takes two logarithms and is reproducible only up to their rounding.)
#include "pasa_kernels.hpp"

namespace {

__device__ __forceinline__ void philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3, uint32_t k0,
                                              uint32_t k1, uint32_t (&out)[4]) {
#pragma unroll
  for (int round = 0; round < 10; ++round) {
    const uint32_t hi0 = __umulhi(0xD2511F53u, c0), lo0 = 0xD2511F53u * c0;
    const uint32_t hi1 = __umulhi(0xCD9E8D57u, c2), lo1 = 0xCD9E8D57u * c2;
    c0 = hi1 ^ c1 ^ k0;
    c1 = lo1;
    c2 = hi0 ^ c3 ^ k1;
    c3 = lo0;
    k0 += 0x9E3779B9u;
    k1 += 0xBB67AE85u;
  }
  out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

__device__ __forceinline__ uint32_t ordered_key(float r) {
  uint32_t u = __float_as_uint(r);
  if (u == 0x80000000u) u = 0u;
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

constexpr int kWavesPerGroup = 4;

__global__ void __launch_bounds__(64 * kWavesPerGroup) route_kernel(RouteParams p) {
  extern __shared__ uint32_t keys_all[];  // [kWavesPerGroup][nb_pad]
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int64_t row = (int64_t)blockIdx.x * kWavesPerGroup + wave;
  if (row >= (int64_t)p.bh * p.nb) return;  // whole wave leaves; no workgroup barrier is used below
  const int nb = p.nb, nb_pad = (nb + 63) & ~63;
  uint32_t* keys = keys_all + wave * nb_pad;
  const uint32_t bh = (uint32_t)(row / nb), i = (uint32_t)(row % nb);
  const float* srow = p.scores + row * nb;

  // 1. noisy keys; lane handles key blocks 4*(lane + 64*t) .. +3
  for (int q4 = lane; q4 * 4 < nb_pad; q4 += 64) {
    uint32_t x[4];
    philox4x32_10((uint32_t)q4, i, bh, 0u, p.seed_lo, p.seed_hi, x);
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const int j = 4 * q4 + e;
      uint32_t key = 0u;  // padding ranks below every real key (real keys are never 0: see ordered_key)
      if (j < nb) {
        float w;
        if (p.gumbel) {  // u in (0,1) on a 2^-23 grid, exact in binary32; standard Gumbel variate -log(-log u)
          const float u = ((float)(x[e] >> 9) + 0.5f) * 0x1p-23f;
          w = -logf(-logf(u));
        } else {
          w = (float)((int32_t)x[e] >> 8) * 0x1p-23f;
        }
        key = ordered_key(__fmaf_rn(p.amp, w, srow[j]));
      }
      keys[j] = key;
    }
  }
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

  // 2. largest T with #{key >= T} >= k
  const int k = p.k_sel;
  uint32_t T = 0u;
  for (int bit = 31; bit >= 0; --bit) {
    const uint32_t cand = T | (1u << bit);
    int cnt = 0;
    for (int j = lane; j < nb_pad; j += 64) cnt += __popcll(__ballot(keys[j] >= cand));
    if (cnt >= k) T = cand;
  }
  int above = 0;
  for (int j = lane; j < nb_pad; j += 64) above += __popcll(__ballot(keys[j] > T));
  int ties_left = k - above;  // how many keys equal to T are still to be taken, in ascending j

  // 3. emit
  int32_t* out = p.idx + row * k;
  uint32_t* mrow = p.mask ? p.mask + row * p.mask_words : nullptr;
  const uint64_t lt = (1ull << lane) - 1ull;
  int written = 0;
  for (int j0 = 0; j0 < nb_pad; j0 += 64) {
    const uint32_t key = keys[j0 + lane];
    const uint64_t tie_b = __ballot(key == T);
    const int tie_rank = __popcll(tie_b & lt);
    const bool sel = (key > T) || (key == T && tie_rank < ties_left);
    const uint64_t sel_b = __ballot(sel);
    if (sel) out[written + __popcll(sel_b & lt)] = j0 + lane;
    written += __popcll(sel_b);
    ties_left -= min(ties_left, (int)__popcll(tie_b));
    if (mrow && lane < 2) {
      const int word = (j0 >> 5) + lane;
      if (word < p.mask_words) mrow[word] = (uint32_t)(sel_b >> (32 * lane));
    }
  }
}

}  // namespace

hipError_t pasa_launch_route(const RouteParams& p, hipStream_t stream) {
  const int64_t rows = (int64_t)p.bh * p.nb;
  const int nb_pad = (p.nb + 63) & ~63;
  const size_t lds = (size_t)kWavesPerGroup * nb_pad * sizeof(uint32_t);
  const unsigned grid = (unsigned)((rows + kWavesPerGroup - 1) / kWavesPerGroup);
  hipLaunchKernelGGL(route_kernel, dim3(grid), dim3(64 * kWavesPerGroup), lds, stream, p);
  return hipGetLastError();
}
