// Measurement aid, not part of the forward: a loop of nothing but bf16 MFMAs on register operands, to read off
// the matrix-core rate (and with it the sustained clock) of the device the benchmark runs on.
#include "pasa.h"
#include "pasa_device.hpp"

namespace {

constexpr int kChains = 8;  // independent accumulators per wave: the MFMAs of a wave never wait for each other

__global__ void __launch_bounds__(256) mfma_probe_kernel(int iterations, float* sink) {
  bf16x8 a, b;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    a[e] = (__bf16)(1.0f + (float)((threadIdx.x + e) & 3) * 0x1p-8f);
    b[e] = (__bf16)(0x1p-12f * (float)((threadIdx.x >> 2) & 3));
  }
  f32x16 acc[kChains];
#pragma unroll
  for (int c = 0; c < kChains; ++c) acc[c] = f32x16{0};
  for (int i = 0; i < iterations; ++i) {
#pragma unroll
    for (int c = 0; c < kChains; ++c) acc[c] = mfma32(a, b, acc[c]);
  }
  float s = 0.f;
#pragma unroll
  for (int c = 0; c < kChains; ++c) s += acc[c][0] + acc[c][15];
  if (s == -1.0f) sink[blockIdx.x * 256 + threadIdx.x] = s;  // never true: keeps the loop alive without a store
}

}  // namespace

extern "C" int pasa_mfma_probe(int32_t workgroups, int32_t iterations, float* sink, double* flops, void* stream) {
  if (workgroups < 1 || iterations < 1 || !sink || !flops) return PASA_EINVAL;
  hipLaunchKernelGGL(mfma_probe_kernel, dim3((unsigned)workgroups), dim3(256), 0, static_cast<hipStream_t>(stream), iterations, sink);
  *flops = (double)workgroups * 4.0 * (double)iterations * kChains * (2.0 * 32 * 32 * 16);
  return hipGetLastError() == hipSuccess ? PASA_OK : PASA_EHIP;
}
