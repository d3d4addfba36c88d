// Measurement aid, not part of the forward: a loop of nothing but bf16 MFMAs on register operands, to read off
// the matrix-core rate (and with it the sustained clock) of the device the benchmark runs on.
#include "pasa.h"
#include "pasa_device.hpp"

namespace {

constexpr int kChains = 8;  // independent accumulators per wave: the MFMAs of a wave never wait for each other

__device__ __forceinline__ uint32_t mix32(uint32_t x) {
  x ^= x >> 16; x *= 0x7feb352du; x ^= x >> 15; x *= 0x846ca68bu; x ^= x >> 16;
  return x;
}

// roughly N(0,1): a scaled sum of four uniforms from an integer hash (any bell-shaped bit pattern will do here)
__device__ __forceinline__ float bell(uint32_t s) {
  float a = 0.f;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    s = mix32(s + (uint32_t)i);
    a += (float)(s >> 8) * 0x1p-24f - 0.5f;
  }
  return a * 1.7320508f;
}

// RANDOM: every chain multiplies its own pair of operand fragments filled with N(0,1)-like values, so that the
// multiplier inputs toggle the way they do on activations; otherwise all chains share one fragment pair of a few
// distinct small values.  The two differ only in the power the matrix cores draw, i.e. in the clock they sustain.
template <bool RANDOM>
__global__ void __launch_bounds__(256) mfma_probe_kernel(int iterations, float* sink) {
  constexpr int NF = RANDOM ? kChains : 1;
  bf16x8 a[NF], b[NF];
#pragma unroll
  for (int c = 0; c < NF; ++c)
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      if constexpr (RANDOM) {
        const uint32_t s = (uint32_t)c * 7919u + threadIdx.x * 131u + (uint32_t)e * 17u + blockIdx.x * 1000003u;
        a[c][e] = (__bf16)bell(s);
        b[c][e] = (__bf16)bell(s ^ 0x9e3779b9u);
      } else {
        a[c][e] = (__bf16)(1.0f + (float)((threadIdx.x + e) & 3) * 0x1p-8f);
        b[c][e] = (__bf16)(0x1p-12f * (float)((threadIdx.x >> 2) & 3));
      }
    }
  f32x16 acc[kChains];
#pragma unroll
  for (int c = 0; c < kChains; ++c) acc[c] = f32x16{0};
  for (int i = 0; i < iterations; ++i) {
#pragma unroll
    for (int c = 0; c < kChains; ++c) acc[c] = mfma32(a[c % NF], b[c % NF], acc[c]);
  }
  float s = 0.f;
#pragma unroll
  for (int c = 0; c < kChains; ++c) s += acc[c][0] + acc[c][15];
  if (s == -1.2345f) sink[blockIdx.x * 256 + threadIdx.x] = s;  // never true: keeps the loop alive without a store
}

}  // namespace

extern "C" int pasa_mfma_probe(int32_t workgroups, int32_t iterations, int32_t random_operands, float* sink, double* flops,
                               void* stream) {
  if (workgroups < 1 || iterations < 1 || !sink || !flops) return PASA_EINVAL;
  if (random_operands) {
    hipLaunchKernelGGL(mfma_probe_kernel<true>, dim3((unsigned)workgroups), dim3(256), 0, static_cast<hipStream_t>(stream), iterations, sink);
  } else {
    hipLaunchKernelGGL(mfma_probe_kernel<false>, dim3((unsigned)workgroups), dim3(256), 0, static_cast<hipStream_t>(stream), iterations, sink);
  }
  *flops = (double)workgroups * 4.0 * (double)iterations * kChains * (2.0 * 32 * 32 * 16);
  return hipGetLastError() == hipSuccess ? PASA_OK : PASA_EHIP;
}
