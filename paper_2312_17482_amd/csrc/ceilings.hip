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

// The memory traffic of the single-tile backward attention with its arithmetic taken out: per (sequence, head)
// unit one workgroup reads five tiles of n rows x 128 bytes (Q, K, V rows of a fused [T, 3, H, 64] buffer, dO and
// O rows of [T, H, 64] buffers), passes them once through LDS with one barrier, and writes three tiles (the rows
// of a fused [T, 3, H, 64] gradient buffer).  What this reaches is the ceiling of that access pattern on the
// machine: eight concurrent row streams, 5 in and 3 out, which is below what a plain two-stream copy reaches.
__global__ __launch_bounds__(256) void probe_bwd_traffic_kernel(const uint16_t* __restrict__ qkv,
                                                                const uint16_t* __restrict__ dout,
                                                                const uint16_t* __restrict__ o,
                                                                uint16_t* __restrict__ dqkv,
                                                                const int32_t* __restrict__ cu, int H) {
  __shared__ u32x4 stage[3 * 4 * 256];   // 48 KB: three workgroups per compute unit
  const int h = blockIdx.x, b = blockIdx.y, tid = threadIdx.x;
  const int start = cu[b], n = min(cu[b + 1] - start, 128);
  const int st_row = tid >> 3, st_col = (tid & 7) * 8;
  const int64_t s3 = 3 * (int64_t)H * 64, s1 = (int64_t)H * 64;
  u32x4 t[5][4];
#pragma unroll
  for (int it = 0; it < 4; ++it) {
#pragma unroll
    for (int x = 0; x < 5; ++x) t[x][it] = u32x4{0u, 0u, 0u, 0u};
    const int r = 32 * it + st_row;
    if (r < n) {
      const int64_t row = start + r;
#pragma unroll
      for (int x = 0; x < 3; ++x)
        t[x][it] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(qkv + row * s3 + (x * H + h) * 64 + st_col));
      t[3][it] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(dout + row * s1 + h * 64 + st_col));
      t[4][it] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(o + row * s1 + h * 64 + st_col));
    }
  }
#pragma unroll
  for (int it = 0; it < 4; ++it) {
    stage[(0 * 4 + it) * 256 + tid] = t[0][it] ^ t[3][it];
    stage[(1 * 4 + it) * 256 + tid] = t[1][it] ^ t[4][it];
    stage[(2 * 4 + it) * 256 + tid] = t[2][it] + t[3][it];
  }
  __syncthreads();
#pragma unroll
  for (int it = 0; it < 4; ++it) {
    const int r = 32 * it + st_row;
    if (r < n) {
      const int64_t row = start + r;
#pragma unroll
      for (int x = 0; x < 3; ++x)
        *reinterpret_cast<u32x4*>(dqkv + row * s3 + (x * H + h) * 64 + st_col) = stage[(x * 4 + it) * 256 + (tid ^ 8)];
    }
  }
}

}  // namespace

mb_status launch_probe_bwd_traffic(const void* qkv, const void* dout, const void* o, void* dqkv, const int32_t* cu,
                                   int B, int H, hipStream_t stream) {
  hipLaunchKernelGGL(probe_bwd_traffic_kernel, dim3(H, B), dim3(256), 0, stream, (const uint16_t*)qkv,
                     (const uint16_t*)dout, (const uint16_t*)o, (uint16_t*)dqkv, cu, H);
  return check_launch("probe_bwd_traffic_kernel");
}

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
