// Ceiling probes: three tiny kernels that do nothing but saturate one unit each, so that the roofs the
// benchmark prices kernels against can be measured on the box at hand and printed beside the published
// peaks: the bf16 matrix cores (the instruction the attention and feed-forward kernels use), the
// vector ALU's fused multiply-add, and its exponential.  (HBM is probed with the row-copy kernel.)
// The host times `iters` rounds between two events; work per launch is stated by the launcher.
#include "common.h"
#include "mfma_util.h"

namespace mb {
namespace {

constexpr int kProbeBlocks = 256 * 8;   // 8 workgroups of 4 waves per compute unit
constexpr int kProbeThreads = 256;

// 8 independent accumulator tiles per wave: back-to-back issue without dependency stalls.
__global__ __launch_bounds__(256) void probe_mfma_kernel(int iters, float* __restrict__ out) {
  bf16x8 a, b;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    a[i] = (__bf16)(0.001f * (float)((threadIdx.x + i) & 7));
    b[i] = (__bf16)(0.002f * (float)((threadIdx.x * 3 + i) & 7));
  }
  f32x16 acc[8];
#pragma unroll
  for (int t = 0; t < 8; ++t)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[t][v] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int t = 0; t < 8; ++t) acc[t] = mfma32(a, b, acc[t]);
  }
  float s = 0.f;
#pragma unroll
  for (int t = 0; t < 8; ++t)
#pragma unroll
    for (int v = 0; v < 16; ++v) s += acc[t][v];
  if (s == 12345.678f) out[0] = s;        // never true: keeps the loop alive without a store per thread
}

// 16 independent dependency chains per lane.
__global__ __launch_bounds__(256) void probe_fma_kernel(int iters, float* __restrict__ out) {
  float x[16];
#pragma unroll
  for (int i = 0; i < 16; ++i) x[i] = 0.001f * (float)(threadIdx.x + i);
  const float m = 0.999f, c = 0.0005f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < 16; ++i) x[i] = fmaf(x[i], m, c);
  }
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 16; ++i) s += x[i];
  if (s == 12345.678f) out[0] = s;
}

__global__ __launch_bounds__(256) void probe_exp_kernel(int iters, float* __restrict__ out) {
  float x[16];
#pragma unroll
  for (int i = 0; i < 16; ++i) x[i] = -0.001f * (float)(threadIdx.x + i);
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < 16; ++i) x[i] = __builtin_amdgcn_exp2f(x[i]) - 1.0f;   // one v_exp_f32 + one add per value
  }
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 16; ++i) s += x[i];
  if (s == 12345.678f) out[0] = s;
}

}  // namespace

mb_status launch_probe(int kind, int iters, float* out, double* work_per_launch, hipStream_t stream) {
  const double lanes = (double)kProbeBlocks * kProbeThreads;
  switch (kind) {
    case 0:   // flops: 8 instructions of 2*32*32*16 per wave and round
      probe_mfma_kernel<<<dim3(kProbeBlocks), dim3(kProbeThreads), 0, stream>>>(iters, out);
      *work_per_launch = (double)kProbeBlocks * (kProbeThreads / 64) * 8.0 * 32768.0 * iters;
      break;
    case 1:   // flops: 16 fused multiply-adds (2 flops) per lane and round
      probe_fma_kernel<<<dim3(kProbeBlocks), dim3(kProbeThreads), 0, stream>>>(iters, out);
      *work_per_launch = lanes * 16.0 * 2.0 * iters;
      break;
    case 2:   // exponentials: 16 per lane and round
      probe_exp_kernel<<<dim3(kProbeBlocks), dim3(kProbeThreads), 0, stream>>>(iters, out);
      *work_per_launch = lanes * 16.0 * iters;
      break;
    default:
      return fail(MB_ERR_INVALID_ARG, "unknown probe kind %d", kind);
  }
  return check_launch("probe kernel");
}

}  // namespace mb
