// Curvature-aware dynamic budget (Sec. "Curvature-Aware Dynamic Budgeting", Eq.9-11): the host-side
// schedule calculator and the device reduction that produces its input signal, the mean L1 distance
// between the velocity fields of two consecutive denoising steps.
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>

#include "pasa.h"

namespace {

constexpr int kL1Threads = 256;
constexpr int kL1MaxGroups = 2048;  // partial sums; also the size of the scratch the entry point asks for

__device__ __forceinline__ float bf16_to_float(uint16_t x) { return __uint_as_float((uint32_t)x << 16); }

// stage 1: grid-stride partial sums of |a - b|, 8 elements (bf16) or 4 elements (fp32) per load, fp32
// accumulation per thread (each thread sees at most n / (groups * 256) elements), fixed-order tree in LDS
template <bool BF16>
__global__ void __launch_bounds__(kL1Threads) l1_partial_kernel(const void* a, const void* b, int64_t n, float* partial) {
  __shared__ float red[kL1Threads];
  constexpr int VEC = BF16 ? 8 : 4;
  const int64_t n_vec = n / VEC;
  float acc = 0.f;
  for (int64_t i = (int64_t)blockIdx.x * kL1Threads + threadIdx.x; i < n_vec; i += (int64_t)gridDim.x * kL1Threads) {
    const uint4 x = reinterpret_cast<const uint4*>(a)[i], y = reinterpret_cast<const uint4*>(b)[i];
    const uint32_t xs[4] = {x.x, x.y, x.z, x.w}, ys[4] = {y.x, y.y, y.z, y.w};
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      if constexpr (BF16) {
        acc += fabsf(bf16_to_float((uint16_t)(xs[e] & 0xffffu)) - bf16_to_float((uint16_t)(ys[e] & 0xffffu)));
        acc += fabsf(bf16_to_float((uint16_t)(xs[e] >> 16)) - bf16_to_float((uint16_t)(ys[e] >> 16)));
      } else {
        acc += fabsf(__uint_as_float(xs[e]) - __uint_as_float(ys[e]));
      }
    }
  }
  if (blockIdx.x == 0 && threadIdx.x < (int)(n - n_vec * VEC)) {  // the few elements after the last whole vector
    const int64_t i = n_vec * VEC + threadIdx.x;
    if constexpr (BF16) acc += fabsf(bf16_to_float(static_cast<const uint16_t*>(a)[i]) - bf16_to_float(static_cast<const uint16_t*>(b)[i]));
    else acc += fabsf(static_cast<const float*>(a)[i] - static_cast<const float*>(b)[i]);
  }
  red[threadIdx.x] = acc;
  __syncthreads();
  for (int s = kL1Threads / 2; s > 0; s >>= 1) {
    if ((int)threadIdx.x < s) red[threadIdx.x] += red[threadIdx.x + s];
    __syncthreads();
  }
  if (threadIdx.x == 0) partial[blockIdx.x] = red[0];
}

// stage 2: one workgroup adds the partial sums in double precision, in a fixed order, and divides by n
__global__ void __launch_bounds__(kL1Threads) l1_final_kernel(const float* partial, int groups, int64_t n, float* out) {
  __shared__ double red[kL1Threads];
  double acc = 0.0;
  for (int i = threadIdx.x; i < groups; i += kL1Threads) acc += (double)partial[i];
  red[threadIdx.x] = acc;
  __syncthreads();
  for (int s = kL1Threads / 2; s > 0; s >>= 1) {
    if ((int)threadIdx.x < s) red[threadIdx.x] += red[threadIdx.x + s];
    __syncthreads();
  }
  if (threadIdx.x == 0) out[0] = (float)(red[0] / (double)n);
}

}  // namespace

extern "C" {

size_t pasa_l1_workspace_bytes(void) { return (size_t)kL1MaxGroups * sizeof(float); }

int pasa_l1_distance(const void* a, const void* b, int64_t n, int32_t dtype, float* out, void* ws, size_t ws_bytes,
                     void* stream) {
  if (!a || !b || !out || !ws || n < 1 || (dtype != PASA_DTYPE_BF16 && dtype != PASA_DTYPE_F32)) return PASA_EINVAL;
  if (((uintptr_t)a | (uintptr_t)b) & 15u) return PASA_EALIGN;
  if (((uintptr_t)ws & 15u) || ((uintptr_t)out & 3u)) return PASA_EALIGN;
  if (ws_bytes < pasa_l1_workspace_bytes()) return PASA_EWORKSPACE;
  const int vec = dtype == PASA_DTYPE_BF16 ? 8 : 4;
  int64_t groups = (n / vec + kL1Threads * 4 - 1) / (kL1Threads * 4);  // at least 4 vectors per thread
  if (groups < 1) groups = 1;
  if (groups > kL1MaxGroups) groups = kL1MaxGroups;
  hipStream_t s = static_cast<hipStream_t>(stream);
  float* partial = static_cast<float*>(ws);
  if (dtype == PASA_DTYPE_BF16) hipLaunchKernelGGL(l1_partial_kernel<true>, dim3((unsigned)groups), dim3(kL1Threads), 0, s, a, b, n, partial);
  else hipLaunchKernelGGL(l1_partial_kernel<false>, dim3((unsigned)groups), dim3(kL1Threads), 0, s, a, b, n, partial);
  hipLaunchKernelGGL(l1_final_kernel, dim3(1), dim3(kL1Threads), 0, s, partial, (int)groups, n, out);
  return hipGetLastError() == hipSuccess ? PASA_OK : PASA_EHIP;
}

int pasa_budget_schedule(const double* l1, int32_t n_prompts, int32_t n_steps, double rho, double dense_fraction,
                         double* rho_t) {
  if (!l1 || !rho_t || n_prompts < 1 || n_steps < 1 || !(rho > 0.0) || rho > 1.0 || !(dense_fraction >= 0.0) ||
      dense_fraction > 1.0)
    return PASA_EINVAL;
  int32_t n_dense = (int32_t)floor(dense_fraction * (double)n_steps + 0.5);
  if (n_dense > n_steps) n_dense = n_steps;
  for (int32_t t = 0; t < n_dense; ++t) rho_t[t] = 1.0;
  if (n_dense == n_steps) return PASA_OK;
  // prompt-averaged signal on the sparse segment, its mean (Eq.9), unit-mean factors (Eq.10), densities (Eq.11)
  double mean = 0.0;
  for (int32_t t = n_dense; t < n_steps; ++t) {
    double lt = 0.0;
    for (int32_t p = 0; p < n_prompts; ++p) {
      const double x = l1[(int64_t)p * n_steps + t];
      if (!(x >= 0.0) || isinf(x)) return PASA_EINVAL;
      lt += x;
    }
    rho_t[t] = lt / (double)n_prompts;
    mean += rho_t[t];
  }
  mean /= (double)(n_steps - n_dense);
  if (!(mean > 0.0)) return PASA_EINVAL;  // a flat zero signal carries no information
  for (int32_t t = n_dense; t < n_steps; ++t) {
    const double r = rho * (rho_t[t] / mean);
    rho_t[t] = r > 1.0 ? 1.0 : r;
  }
  return PASA_OK;
}

}  // extern "C"
