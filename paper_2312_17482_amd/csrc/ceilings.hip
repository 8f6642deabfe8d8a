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

// 16-byte LDS reads, the access the GEMM fragments use (rows of 144 bytes, one row per lane of a half-wave):
// 8 independent reads per round and wave.  One workgroup of 4 waves per compute unit slot.
__global__ __launch_bounds__(256) void probe_lds_kernel(int iters, float* __restrict__ out) {
  __shared__ __attribute__((aligned(16))) uint16_t tile[256 * 72];
  for (int i = threadIdx.x; i < 256 * 72; i += 256) tile[i] = (uint16_t)i;
  __syncthreads();
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const uint16_t* base = &tile[((wave & 1) * 128 + (lane & 31)) * 72 + (lane >> 5) * 8];
  u32x4 acc = {0u, 0u, 0u, 0u};
  int off = 0;
  for (int it = 0; it < iters; ++it) {
    asm volatile("" : "+v"(off));     // opaque: the reads cannot be hoisted out of the loop
#pragma unroll
    for (int r = 0; r < 8; ++r) {
      const u32x4 v = *reinterpret_cast<const u32x4*>(base + off + (r & 3) * 32 * 72 + (r >> 2) * 16);
      acc[0] += v[0]; acc[1] += v[1]; acc[2] += v[2]; acc[3] += v[3];
    }
  }
  if ((acc[0] ^ acc[1] ^ acc[2] ^ acc[3]) == 0x12345678u) out[0] = 1.f;
}

// The inner loop of the GEMM kernels without their memory traffic: one workgroup of 4 waves per compute
// unit (the LDS allocation sees to that), each wave 16 accumulator tiles, per k sub-step 8 fragment reads
// of 16 bytes (double-buffered) and 16 matrix instructions, in the same fenced issue order; no global
// loads, no LDS writes; `with_barrier` adds the GEMM's one workgroup barrier per 4 sub-steps.
template <bool kBarrier, bool kWrites, bool kLoads>
__global__ __launch_bounds__(256, 1) void probe_gemm_loop_kernel(int iters, float* __restrict__ out,
                                                                 const uint16_t* __restrict__ src) {
  __shared__ __attribute__((aligned(16))) uint16_t tile[2 * 512 * 72];
  for (int i = threadIdx.x; i < 2 * 512 * 72; i += 256) tile[i] = (uint16_t)(0x3c00 + (i & 63));
  __syncthreads();
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int c = lane & 31, g = lane >> 5, wm = wave >> 1, wn = wave & 1;
  const uint16_t* xb = &tile[(wm * 128 + c) * 72 + g * 8];
  const uint16_t* wb = &tile[(256 + wn * 128 + c) * 72 + g * 8];
  f32x16 acc[4][4];
#pragma unroll
  for (int a = 0; a < 4; ++a)
#pragma unroll
    for (int b = 0; b < 4; ++b)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.f;
  bf16x8 wf[2][4], xf[2][4];
  int off = 0;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    xf[0][i] = lds_read8(xb + i * 32 * 72);
    wf[0][i] = lds_read8(wb + i * 32 * 72);
  }
  // staging registers of a k step (16 x 16 bytes per thread), written to the other LDS stage / loaded from a
  // 64 KB region per workgroup that stays in L2
  u32x4 st[16];
#pragma unroll
  for (int i = 0; i < 16; ++i) st[i] = u32x4{0x3c003c00u, 0x3c003c00u, 0x3c003c00u, 0x3c003c00u};
  const int lrow = threadIdx.x >> 3, lchunk = (threadIdx.x & 7) * 8;
  uint16_t* dep = &tile[512 * 72 + lrow * 72 + lchunk];
  const uint16_t* gsrc = src + (size_t)(blockIdx.x & 255) * 32768 + lrow * 64 + lchunk;
  for (int it = 0; it < iters; ++it) {
    asm volatile("" : "+v"(off));
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      if (kBarrier && kk == 3) __syncthreads();
#pragma unroll
      for (int q = 0; q < 4; ++q) {
#pragma unroll
        for (int mb = 0; mb < 4; ++mb) {
          const int slot = 4 * q + mb;
          if (slot < 8) {
            const int nk = (kk + 1) & 3;
            if (slot < 4) xf[(kk + 1) & 1][slot] = lds_read8(xb + off + slot * 32 * 72 + nk * 16);
            else wf[(kk + 1) & 1][slot - 4] = lds_read8(wb + off + (slot - 4) * 32 * 72 + nk * 16);
          }
          if (kWrites && kk == 0) *reinterpret_cast<u32x4*>(dep + off + slot * 32 * 72) = st[slot];
          if (kLoads && kk == 1)
            st[slot] = *reinterpret_cast<const u32x4*>(gsrc + off + slot * 2048);
          __builtin_amdgcn_sched_barrier(0);
          acc[q][mb] = mfma32(wf[kk & 1][q], xf[kk & 1][mb], acc[q][mb]);
          __builtin_amdgcn_sched_barrier(0);
        }
      }
    }
  }
  float sum = 0.f;
#pragma unroll
  for (int a = 0; a < 4; ++a)
#pragma unroll
    for (int b = 0; b < 4; ++b)
#pragma unroll
      for (int v = 0; v < 16; ++v) sum += acc[a][b][v];
  if (sum == 12345.678f) out[0] = sum;
}

// Do the matrix cores and the vector ALU of a SIMD work at the same time?  One round = 4 matrix instructions
// (independent accumulators) and / or 48 independent fused multiply-adds, written interleaved; the three
// variants run the same number of rounds, so  t(both)  against  t(matrix) + t(vector)  and  max of the two
// answers the question for the instruction mix of the attention kernels.
// kSmall: the same flops as 8 instructions of the 16x16x32 shape (4 accumulator registers each instead of 16).
typedef float f32x4v __attribute__((ext_vector_type(4)));
template <bool kFma>
__global__ __launch_bounds__(256) void probe_mix16_kernel(int iters, float* __restrict__ out) {
  bf16x8 a, b;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    a[i] = (__bf16)(0.001f * (float)((threadIdx.x + i) & 7));
    b[i] = (__bf16)(0.002f * (float)((threadIdx.x * 3 + i) & 7));
  }
  f32x4v acc[8];
#pragma unroll
  for (int t = 0; t < 8; ++t)
#pragma unroll
    for (int v = 0; v < 4; ++v) acc[t][v] = 0.f;
  float x[16];
#pragma unroll
  for (int i = 0; i < 16; ++i) x[i] = 0.001f * (float)(threadIdx.x + i);
  const float m = 0.999f, c = 0.0005f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int t = 0; t < 8; ++t) {
      acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, acc[t], 0, 0, 0);
      if (kFma) {
#pragma unroll
        for (int i = 0; i < 6; ++i) x[(2 * t + i) & 15] = fmaf(x[(2 * t + i) & 15], m, c);
      }
    }
  }
  float s = 0.f;
#pragma unroll
  for (int t = 0; t < 8; ++t)
#pragma unroll
    for (int v = 0; v < 4; ++v) s += acc[t][v];
#pragma unroll
  for (int i = 0; i < 16; ++i) s += x[i];
  if (s == 12345.678f) out[0] = s;
}

template <bool kMfma, bool kFma>
__global__ __launch_bounds__(256) void probe_mix_kernel(int iters, float* __restrict__ out) {
  bf16x8 a, b;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    a[i] = (__bf16)(0.001f * (float)((threadIdx.x + i) & 7));
    b[i] = (__bf16)(0.002f * (float)((threadIdx.x * 3 + i) & 7));
  }
  f32x16 acc[4];
#pragma unroll
  for (int t = 0; t < 4; ++t)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[t][v] = 0.f;
  float x[16];
#pragma unroll
  for (int i = 0; i < 16; ++i) x[i] = 0.001f * (float)(threadIdx.x + i);
  const float m = 0.999f, c = 0.0005f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      if (kMfma) acc[t] = mfma32(a, b, acc[t]);
      if (kFma) {
#pragma unroll
        for (int i = 0; i < 12; ++i) x[(4 * t + i) & 15] = fmaf(x[(4 * t + i) & 15], m, c);
      }
    }
  }
  float s = 0.f;
#pragma unroll
  for (int t = 0; t < 4; ++t)
#pragma unroll
    for (int v = 0; v < 16; ++v) s += acc[t][v];
#pragma unroll
  for (int i = 0; i < 16; ++i) s += x[i];
  if (s == 12345.678f) out[0] = s;
}

}  // namespace

mb_status launch_probe(int kind, int iters, float* out, double* work_per_launch, hipStream_t stream) {
  // kind 7 reads a 16 MiB source that starts 4 floats into `out` (the caller sizes `out` accordingly)
  const uint16_t* src = reinterpret_cast<const uint16_t*>(out + 4);
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
    case 3:   // bytes read from LDS: 8 reads of 16 bytes per lane and round
      probe_lds_kernel<<<dim3(kProbeBlocks), dim3(kProbeThreads), 0, stream>>>(iters, out);
      *work_per_launch = lanes * 8.0 * 16.0 * iters;
      break;
    case 4:   // flops of the GEMM inner loop fed from LDS, no barrier: 64 instructions per wave and round
    case 5:   // the same with one workgroup barrier per round
    case 6:   // the same plus the 16 LDS writes per thread and k step
    case 7:   // the same plus the 16 global loads per thread and k step (from a region that stays in L2)
      if (kind == 4) probe_gemm_loop_kernel<false, false, false><<<dim3(256 * 4), dim3(256), 0, stream>>>(iters, out, src);
      else if (kind == 5) probe_gemm_loop_kernel<true, false, false><<<dim3(256 * 4), dim3(256), 0, stream>>>(iters, out, src);
      else if (kind == 6) probe_gemm_loop_kernel<true, true, false><<<dim3(256 * 4), dim3(256), 0, stream>>>(iters, out, src);
      else probe_gemm_loop_kernel<true, true, true><<<dim3(256 * 4), dim3(256), 0, stream>>>(iters, out, src);
      *work_per_launch = 256.0 * 4 * 4 * 64.0 * 32768.0 * iters;
      break;
    case 8: case 9: case 10:     // rounds of (4 matrix instructions, 48 multiply-adds, both): 8 waves per SIMD
    case 11: case 12: case 13: { // the same with one wave per SIMD
      const int blocks = kind < 11 ? kProbeBlocks : 256;
      const int v = (kind - 8) % 3;
      if (v == 0) probe_mix_kernel<true, false><<<dim3(blocks), dim3(256), 0, stream>>>(iters, out);
      else if (v == 1) probe_mix_kernel<false, true><<<dim3(blocks), dim3(256), 0, stream>>>(iters, out);
      else probe_mix_kernel<true, true><<<dim3(blocks), dim3(256), 0, stream>>>(iters, out);
      *work_per_launch = (double)blocks * 4.0 * iters;   // rounds, over all waves
      break;
    }
    case 14: case 15:   // kinds 8 and 10 with the 16x16x32 shape (8 instructions per round), 8 waves per SIMD
      if (kind == 14) probe_mix16_kernel<false><<<dim3(kProbeBlocks), dim3(256), 0, stream>>>(iters, out);
      else probe_mix16_kernel<true><<<dim3(kProbeBlocks), dim3(256), 0, stream>>>(iters, out);
      *work_per_launch = (double)kProbeBlocks * 4.0 * iters;
      break;
    default:
      return fail(MB_ERR_INVALID_ARG, "unknown probe kind %d", kind);
  }
  return check_launch("probe kernel");
}

}  // namespace mb
