// Measurement aid: a register-resident bf16 MFMA loop, the practical ceiling of the matrix cores
// that the attention kernels' achieved rates are also quoted against (next to the published
// peak).  No memory traffic inside the loop: operands and accumulators stay in registers.
#include "bsa_common.h"
#include "bsa_mfma.h"

namespace bsa {

constexpr int kProbeAcc = 4;  // independent accumulators per wavefront (hides the MFMA latency)

__global__ __launch_bounds__(256) void mfma_probe_kernel(int iters, float* sink) {
  const int lane = threadIdx.x & 63;
  bf16x8 a, b;
#pragma unroll
  for (int t = 0; t < 8; ++t) {  // small exact values: no overflow however long the loop
    a[t] = (__bf16)(((lane + t) & 3) * 0.25f);
    b[t] = (__bf16)(((lane ^ t) & 1) ? 0.0f : 1.0f / 1024.0f);
  }
  f32x16 acc[kProbeAcc];
#pragma unroll
  for (int k = 0; k < kProbeAcc; ++k)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[k][r] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int k = 0; k < kProbeAcc; ++k) acc[k] = mfma32(a, b, acc[k]);
  }
  float s = 0.f;
#pragma unroll
  for (int k = 0; k < kProbeAcc; ++k)
#pragma unroll
    for (int r = 0; r < 16; ++r) s += acc[k][r];
  sink[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = s;
}

}  // namespace bsa

extern "C" int64_t bsa_mfma_probe(int workgroups, int iters, float* sink, void* stream) {
  if (!sink) return BSA_ERR_NULL;
  if (workgroups <= 0 || iters <= 0) return BSA_ERR_RANGE;
  hipLaunchKernelGGL(bsa::mfma_probe_kernel, dim3(workgroups), dim3(256), 0, static_cast<hipStream_t>(stream), iters, sink);
  if (bsa::check_launch() != BSA_OK) return BSA_ERR_LAUNCH;
  // 4 wavefronts per workgroup, kProbeAcc products of 32 x 32 x 16 per iteration, 2 flops per multiply-add
  return (int64_t)workgroups * 4 * iters * bsa::kProbeAcc * (2LL * 32 * 32 * 16);
}
