// Stage 2 of the PASA forward on gfx950: per-row top-k block selection with a seeded stochastic
// bias (Eq.2; Sec. "Stochastic Routing").  One wavefront per (head, query block) row:
//   1. r_j = fmaf(amp, w_j, s_j) with w_j from Philox4x32-10 (one call serves 4 consecutive j),
//      mapped to an order-preserving uint32 key (-0 folded onto +0); the keys pass through LDS once
//      and then stay in registers, key block lane + 64 t in register t;
//   2. the k-th largest key is found by a bitwise search from the top bit down; a step counts the keys
//      that reach the candidate (per-lane counts, summed by one ballot per bit of the count) and the
//      search stops as soon as exactly k keys do;
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

// KPL = keys per lane: the row is padded to 64 * KPL keys.
template <int KPL>
__global__ void __launch_bounds__(64 * kWavesPerGroup) route_kernel(RouteParams p) {
  extern __shared__ __attribute__((aligned(16))) uint32_t keys_all[];  // [kWavesPerGroup][64 * KPL]
  static_assert(KPL % 4 == 0, "a lane writes whole quads of keys");
  constexpr int NB_PAD = 64 * KPL;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int64_t row = (int64_t)blockIdx.x * kWavesPerGroup + wave;
  if (row >= (int64_t)p.bh * p.nb) return;  // whole wave leaves; no workgroup barrier is used below
  const int nb = p.nb;
  uint32_t* keys = keys_all + wave * NB_PAD;
  const uint32_t bh = (uint32_t)(row / nb), i = (uint32_t)(row % nb);
  const float* srow = p.scores + row * nb;

  // 1. noisy keys; one Philox call serves key blocks 4 q4 .. 4 q4 + 3, so lane handles those of q4 = lane + 64 t.
  //    They pass through LDS once, to regroup them as j = lane + 64 t for what follows.
#pragma unroll
  for (int t = 0; t < (KPL + 3) / 4; ++t) {
    const int q4 = lane + 64 * t;  // 4 q4 + 3 < 64 KPL: KPL is a multiple of 4
    uint32_t x[4] = {0u, 0u, 0u, 0u};
    if (4 * q4 < nb) philox4x32_10((uint32_t)q4, i, bh, 0u, p.seed_lo, p.seed_hi, x);
    uint4 kq;
    uint32_t* ke = reinterpret_cast<uint32_t*>(&kq);
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
      ke[e] = key;
    }
    *reinterpret_cast<uint4*>(keys + 4 * q4) = kq;
  }
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
  uint32_t key[KPL];  // key[t] belongs to key block lane + 64 t
#pragma unroll
  for (int t = 0; t < KPL; ++t) key[t] = keys[lane + 64 * t];

  // wave-wide number of keys that satisfy a predicate: one compare per key on the vector unit, its lane mask counted
  // and summed on the scalar unit (which runs beside the vector unit)
  auto wave_count = [&](auto pred) -> int {
    int total = 0;
#pragma unroll
    for (int t = 0; t < KPL; ++t) total += (int)__popcll(__ballot(pred(key[t])));
    return total;
  };

  // 2. largest T with #{key >= T} >= k, bit by bit from the top.  As soon as exactly k keys reach a candidate,
  //    the selection is settled (those k keys) and the remaining bits do not matter.
  const int k = p.k_sel;
  uint32_t T = 0u;
  for (int bit = 31; bit >= 0; --bit) {
    const uint32_t cand = T | (1u << bit);
    const int cnt = wave_count([&](uint32_t x) { return x >= cand; });
    if (cnt >= k) T = cand;
    if (cnt == k) break;
  }
  const int above = wave_count([&](uint32_t x) { return x > T; });
  int ties_left = k - above;  // how many keys equal to T are still to be taken, in ascending j

  // 3. emit
  int32_t* out = p.idx + row * k;
  uint32_t* mrow = p.mask ? p.mask + row * p.mask_words : nullptr;
  const uint64_t lt = (1ull << lane) - 1ull;
  int written = 0;
#pragma unroll
  for (int t = 0; t < KPL; ++t) {
    const int j0 = 64 * t;
    if (j0 >= ((nb + 63) & ~63)) break;
    const uint64_t tie_b = __ballot(key[t] == T);
    const int tie_rank = __popcll(tie_b & lt);
    const bool sel = (key[t] > T) || (key[t] == T && tie_rank < ties_left);
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

// ---- selections handed in by a caller -----------------------------------------------------------------
// One wavefront per row (head, query block).  A row is bad if an index lies outside [0, nb), the list is not
// strictly ascending, the bitmap has a bit set at or beyond nb, its population count is not k_sel, or list and
// bitmap name different blocks.  Either of idx and mask may be null (then only the other is checked).
__global__ void __launch_bounds__(256) check_selection_kernel(const int32_t* idx, const uint32_t* mask, int64_t rows, int nb,
                                                              int k_sel, int mask_words, int32_t* n_bad) {
  const int lane = threadIdx.x & 63;
  const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= rows) return;
  bool bad = false;
  const uint32_t* mrow = mask ? mask + row * mask_words : nullptr;
  if (idx) {
    const int32_t* irow = idx + row * k_sel;
    for (int e = lane; e < k_sel; e += 64) {
      const int32_t j = irow[e];
      if (j < 0 || j >= nb) { bad = true; continue; }
      if (e > 0 && irow[e - 1] >= j) bad = true;
      if (mrow && !((mrow[j >> 5] >> (j & 31)) & 1u)) bad = true;
    }
  }
  if (mrow) {
    int count = 0;
    for (int wd = lane; wd < mask_words; wd += 64) {
      const uint32_t x = mrow[wd];
      count += __popc(x);
      const int valid = nb - 32 * wd;  // bits of this word that name existing blocks
      if (valid < 32 && (x >> max(valid, 0)) != 0u) bad = true;
    }
#pragma unroll
    for (int sh = 32; sh >= 1; sh >>= 1) count += __shfl_xor(count, sh);
    if (count != k_sel) bad = true;  // with the list inside the bitmap and k_sel distinct entries, the two sets are equal
  }
  if (__ballot(bad) != 0ull && lane == 0) atomicAdd(n_bad, 1);
}

__global__ void zero_i32_kernel(int32_t* x) { *x = 0; }

// bitmap rows from ascending index lists: one wavefront per row clears the row's words, then sets its bits
// (integer atomic OR inside the row: the result does not depend on the order)
__global__ void __launch_bounds__(256) mask_from_idx_kernel(const int32_t* idx, int64_t rows, int nb, int k_sel, int mask_words,
                                                            uint32_t* mask) {
  const int lane = threadIdx.x & 63;
  const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= rows) return;
  uint32_t* mrow = mask + row * mask_words;
  for (int wd = lane; wd < mask_words; wd += 64) mrow[wd] = 0u;
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
  const int32_t* irow = idx + row * k_sel;
  for (int e = lane; e < k_sel; e += 64) {
    const int32_t j = irow[e];
    if (j >= 0 && j < nb) atomicOr(mrow + (j >> 5), 1u << (j & 31));  // out-of-range entries are a caller error; never written
  }
}

template <int KPL>
hipError_t launch_route(const RouteParams& p, hipStream_t stream) {
  const int64_t rows = (int64_t)p.bh * p.nb;
  const size_t lds = (size_t)kWavesPerGroup * 64 * KPL * sizeof(uint32_t);
  const unsigned grid = (unsigned)((rows + kWavesPerGroup - 1) / kWavesPerGroup);
  hipLaunchKernelGGL(route_kernel<KPL>, dim3(grid), dim3(64 * kWavesPerGroup), lds, stream, p);
  return hipGetLastError();
}

}  // namespace

hipError_t pasa_launch_check_selection(const int32_t* idx, const uint32_t* mask, int64_t rows, int nb, int k_sel,
                                       int32_t* n_bad, hipStream_t stream) {
  hipLaunchKernelGGL(zero_i32_kernel, dim3(1), dim3(1), 0, stream, n_bad);
  hipLaunchKernelGGL(check_selection_kernel, dim3((unsigned)((rows + 3) / 4)), dim3(256), 0, stream, idx, mask, rows, nb, k_sel,
                     (nb + 31) / 32, n_bad);
  return hipGetLastError();
}

hipError_t pasa_launch_mask_from_idx(const int32_t* idx, int64_t rows, int nb, int k_sel, uint32_t* mask, hipStream_t stream) {
  hipLaunchKernelGGL(mask_from_idx_kernel, dim3((unsigned)((rows + 3) / 4)), dim3(256), 0, stream, idx, rows, nb, k_sel,
                     (nb + 31) / 32, mask);
  return hipGetLastError();
}

hipError_t pasa_launch_route(const RouteParams& p, hipStream_t stream) {
  const int kpl = (p.nb + 63) / 64;  // at most kRouteMaxBlocks / 64
  if (kpl <= 4) return launch_route<4>(p, stream);
  if (kpl <= 8) return launch_route<8>(p, stream);
  if (kpl <= 12) return launch_route<12>(p, stream);
  if (kpl <= 16) return launch_route<16>(p, stream);
  if (kpl <= 20) return launch_route<20>(p, stream);
  if (kpl <= 24) return launch_route<24>(p, stream);
  if (kpl <= 32) return launch_route<32>(p, stream);
  if (kpl <= 48) return launch_route<48>(p, stream);
  return launch_route<64>(p, stream);
}
