// Add & LayerNorm over packed token rows with bf16 (or fp32) storage: the "Low Precision LayerNorm" of the
// paper (LayerNorm reads and writes 2-byte elements because it is bandwidth-bound) together with the
// residual add in front of it ("Add & Norm" in Figure 1A).  Statistics and normalisation are fp32.
//
//   forward :  s = x + r (stored, rounded once),  y = (s - mean) * rstd * gamma + beta
//   backward:  xhat = (s - mean) rstd, g = dy * gamma,
//              ds = rstd * (g - mean(g) - xhat * mean(g * xhat)),  dgamma = sum_t dy * xhat,  dbeta = sum_t dy
//
// One wave per row, 16-byte pieces, every tensor crosses HBM once.  The column sums of the backward are
// reduced in a fixed order (per-workgroup partials in the workspace, then one pass over them): no atomics.
#include "common.h"

namespace mb {
namespace {

// 16-byte pieces per lane: 2 for rows up to 2 KB (fewer registers, four waves per SIMD), else 4 (up to 4 KB)
constexpr int kLnThreads = 256;
constexpr int kLnWaves = kLnThreads / 64;

__device__ __forceinline__ float wsum(float x) {
  for (int off = 32; off > 0; off >>= 1) x += __shfl_xor(x, off, 64);
  return x;
}

template <typename E> struct Piece;      // one 16-byte piece of a row <-> floats
template <> struct Piece<uint16_t> {
  static constexpr int kN = 8;
  static __device__ __forceinline__ void load(const uint16_t* p, float* f) {
    const uint4 u = *reinterpret_cast<const uint4*>(p);
    const uint32_t w[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      f[2 * i] = __uint_as_float(w[i] << 16);
      f[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
    }
  }
  static __device__ __forceinline__ uint32_t rne(float x) {   // float -> bf16 bits, nearest even; NaN stays NaN
    const uint32_t u = __float_as_uint(x);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;
    return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
  }
  static __device__ __forceinline__ void store(uint16_t* p, const float* f) {
    uint4 u;
    u.x = rne(f[0]) | (rne(f[1]) << 16);
    u.y = rne(f[2]) | (rne(f[3]) << 16);
    u.z = rne(f[4]) | (rne(f[5]) << 16);
    u.w = rne(f[6]) | (rne(f[7]) << 16);
    *reinterpret_cast<uint4*>(p) = u;
  }
  static __device__ __forceinline__ float round(float x) { return __uint_as_float(rne(x) << 16); }
};
// 8-byte pieces of a bf16 row: for rows whose number of 16-byte pieces is not a multiple of 64 while twice as many
// 8-byte pieces is (768 columns: 192 = 3 x 64), every lane then carries the same share and no register sits idle.
// Used by the forward (31.9 -> 30.9 us at 26963 x 768); the backward measured slower with them (37.3 against 35.0 us:
// more load instructions per row than the extra wave per SIMD buys) and keeps 16-byte pieces.
struct HalfPiece {
  static constexpr int kN = 4;
  static __device__ __forceinline__ void load(const uint16_t* p, float* f) {
    const uint2 u = *reinterpret_cast<const uint2*>(p);
    f[0] = __uint_as_float(u.x << 16); f[1] = __uint_as_float(u.x & 0xffff0000u);
    f[2] = __uint_as_float(u.y << 16); f[3] = __uint_as_float(u.y & 0xffff0000u);
  }
  static __device__ __forceinline__ void store(uint16_t* p, const float* f) {
    uint2 u;
    u.x = Piece<uint16_t>::rne(f[0]) | (Piece<uint16_t>::rne(f[1]) << 16);
    u.y = Piece<uint16_t>::rne(f[2]) | (Piece<uint16_t>::rne(f[3]) << 16);
    *reinterpret_cast<uint2*>(p) = u;
  }
  static __device__ __forceinline__ float round(float x) { return Piece<uint16_t>::round(x); }
};
template <> struct Piece<float> {
  static constexpr int kN = 4;
  static __device__ __forceinline__ void load(const float* p, float* f) {
    const float4 u = *reinterpret_cast<const float4*>(p);
    f[0] = u.x; f[1] = u.y; f[2] = u.z; f[3] = u.w;
  }
  static __device__ __forceinline__ void store(float* p, const float* f) {
    *reinterpret_cast<float4*>(p) = make_float4(f[0], f[1], f[2], f[3]);
  }
  static __device__ __forceinline__ float round(float x) { return x; }
};

template <typename E, int kMaxPieces, typename PT = Piece<E>>
__global__ __launch_bounds__(kLnThreads) void add_layernorm_fwd_kernel(
    const E* __restrict__ x, const E* __restrict__ r, const E* __restrict__ gamma, const E* __restrict__ beta,
    int T_cap, const int32_t* __restrict__ meta, int W, float eps, E* __restrict__ y, E* __restrict__ s,
    float* __restrict__ mean, float* __restrict__ rstd, const int32_t* __restrict__ y_rows) {
  constexpr int N = PT::kN;
  const int T = meta ? min(meta[0], T_cap) : T_cap;
  const int row = blockIdx.x * kLnWaves + (threadIdx.x >> 6);
  if (row >= T) return;
  const int lane = threadIdx.x & 63;
  const int pieces = W / N;
  const E* xr = x + (size_t)row * W;
  E* yr = y + (size_t)tok_row(y_rows, row) * W;   // packed row, or the token's row in the padded batch
  float v[kMaxPieces][N];
  float sum = 0.f;
#pragma unroll
  for (int c = 0; c < kMaxPieces; ++c) {
    const int pc = lane + 64 * c;
    if (pc < pieces) {
      PT::load(xr + pc * N, v[c]);
      if (r) {
        float t[N];
        PT::load(r + (size_t)row * W + pc * N, t);
#pragma unroll
        for (int i = 0; i < N; ++i) v[c][i] = PT::round(v[c][i] + t[i]);   // the stored sum is what is normalised
        PT::store(s + (size_t)row * W + pc * N, v[c]);
      }
#pragma unroll
      for (int i = 0; i < N; ++i) sum += v[c][i];
    }
  }
  const float mu = wsum(sum) / (float)W;
  float sq = 0.f;
#pragma unroll
  for (int c = 0; c < kMaxPieces; ++c) {
    if (lane + 64 * c < pieces) {
#pragma unroll
      for (int i = 0; i < N; ++i) { const float d = v[c][i] - mu; sq = fmaf(d, d, sq); }
    }
  }
  const float rs = rsqrtf(wsum(sq) / (float)W + eps);
#pragma unroll
  for (int c = 0; c < kMaxPieces; ++c) {
    const int pc = lane + 64 * c;
    if (pc < pieces) {
      float g[N], b[N], out[N];
      PT::load(gamma + pc * N, g);
      PT::load(beta + pc * N, b);
#pragma unroll
      for (int i = 0; i < N; ++i) out[i] = fmaf((v[c][i] - mu) * rs, g[i], b[i]);
      PT::store(yr + pc * N, out);
    }
  }
  if (lane == 0) { mean[row] = mu; rstd[row] = rs; }
}

// Each wave walks rows  blockIdx*4 + wave, + 4*gridDim, ...: writes ds and keeps per-lane partial column
// sums; the four waves of a block are then added in a fixed order and written to part[block][2][W].
template <typename E, int kMaxPieces, typename PT = Piece<E>>
__global__ __launch_bounds__(kLnThreads) void add_layernorm_bwd_kernel(
    const E* __restrict__ dy, const E* __restrict__ s, const E* __restrict__ gamma, const float* __restrict__ mean,
    const float* __restrict__ rstd, int T_cap, const int32_t* __restrict__ meta, int W, E* __restrict__ ds,
    float* __restrict__ part, const int32_t* __restrict__ dy_rows) {
  constexpr int N = PT::kN;
  extern __shared__ float lds[];   // [kLnWaves][2][W]
  const int T = meta ? min(meta[0], T_cap) : T_cap;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int pieces = W / N;
  float g[kMaxPieces][N], ag[kMaxPieces][N], ab[kMaxPieces][N];
#pragma unroll
  for (int c = 0; c < kMaxPieces; ++c) {
#pragma unroll
    for (int i = 0; i < N; ++i) { g[c][i] = 0.f; ag[c][i] = 0.f; ab[c][i] = 0.f; }
    if (lane + 64 * c < pieces) PT::load(gamma + (lane + 64 * c) * N, g[c]);
  }
  for (int row = blockIdx.x * kLnWaves + wave; row < T; row += gridDim.x * kLnWaves) {
    const float mu = mean[row], rs = rstd[row];
    const E* dyr = dy + (size_t)tok_row(dy_rows, row) * W;   // packed row, or the token's row in the padded batch
    float xh[kMaxPieces][N], gy[kMaxPieces][N];
    float c1 = 0.f, c2 = 0.f;
#pragma unroll
    for (int c = 0; c < kMaxPieces; ++c) {
      const int pc = lane + 64 * c;
      if (pc < pieces) {
        float d[N];
        PT::load(s + (size_t)row * W + pc * N, xh[c]);
        PT::load(dyr + pc * N, d);
#pragma unroll
        for (int i = 0; i < N; ++i) {
          xh[c][i] = (xh[c][i] - mu) * rs;
          ag[c][i] = fmaf(d[i], xh[c][i], ag[c][i]);
          ab[c][i] += d[i];
          gy[c][i] = d[i] * g[c][i];
          c1 += gy[c][i];
          c2 = fmaf(gy[c][i], xh[c][i], c2);
        }
      }
    }
    c1 = wsum(c1) / (float)W;
    c2 = wsum(c2) / (float)W;
#pragma unroll
    for (int c = 0; c < kMaxPieces; ++c) {
      const int pc = lane + 64 * c;
      if (pc < pieces) {
        float out[N];
#pragma unroll
        for (int i = 0; i < N; ++i) out[i] = rs * (gy[c][i] - c1 - xh[c][i] * c2);
        PT::store(ds + (size_t)row * W + pc * N, out);
      }
    }
  }
#pragma unroll
  for (int c = 0; c < kMaxPieces; ++c) {
    const int pc = lane + 64 * c;
    if (pc < pieces) {
#pragma unroll
      for (int i = 0; i < N; ++i) {
        lds[(wave * 2 + 0) * W + pc * N + i] = ag[c][i];
        lds[(wave * 2 + 1) * W + pc * N + i] = ab[c][i];
      }
    }
  }
  __syncthreads();
  for (int idx = threadIdx.x; idx < 2 * W; idx += kLnThreads) {
    float t = 0.f;
#pragma unroll
    for (int w = 0; w < kLnWaves; ++w) t += lds[w * 2 * W + idx];
    part[(size_t)blockIdx.x * 2 * W + idx] = t;
  }
}

// dgamma[w], dbeta[w] = sum over the `nparts` partial rows.  64 columns per block; the partial rows are
// dealt to 16 waves x 16 independent accumulators (so that many loads are in flight: the kernel is a chain of
// memory round trips, nothing else) and combined in a fixed order.
constexpr int kColsumSlices = 16;
__global__ __launch_bounds__(64 * kColsumSlices) void add_layernorm_colsum_kernel(const float* __restrict__ part,
                                                                                int nparts, int W,
                                                                                float* __restrict__ dgamma,
                                                                                float* __restrict__ dbeta) {
  __shared__ float red[kColsumSlices][64];
  const int l = threadIdx.x & 63;
  const int idx = blockIdx.x * 64 + l;
  const int slice = threadIdx.x >> 6;
  constexpr int kAcc = 16;
  float acc[kAcc];
#pragma unroll
  for (int u = 0; u < kAcc; ++u) acc[u] = 0.f;
  if (idx < 2 * W) {
    int p = slice;
    for (; p + (kAcc - 1) * kColsumSlices < nparts; p += kAcc * kColsumSlices) {
      float x[kAcc];
#pragma unroll
      for (int u = 0; u < kAcc; ++u) x[u] = part[(size_t)(p + kColsumSlices * u) * 2 * W + idx];
#pragma unroll
      for (int u = 0; u < kAcc; ++u) acc[u] += x[u];
    }
    for (; p < nparts; p += kColsumSlices) acc[0] += part[(size_t)p * 2 * W + idx];
  }
#pragma unroll
  for (int w = kAcc / 2; w > 0; w >>= 1)
#pragma unroll
    for (int u = 0; u < w; ++u) acc[u] += acc[u + w];
  red[slice][l] = acc[0];
  __syncthreads();
  if (slice == 0 && idx < 2 * W) {
    float t = 0.f;
#pragma unroll
    for (int sl = 0; sl < kColsumSlices; ++sl) t += red[sl][l];
    if (idx < W) dgamma[idx] = t; else dbeta[idx - W] = t;
  }
}

// bf16 rows that split evenly over the 64 lanes in 8-byte pieces but not in 16-byte pieces: 256 or 768 columns
// (one or three pieces per lane)
bool use_half_pieces(mb_dtype dt, int W) { return dt == MB_BF16 && (W == 256 || W == 768); }

int bwd_blocks(int T_cap) { return max(1, min((T_cap + kLnWaves - 1) / kLnWaves, kLayerNormMaxParts)); }

}  // namespace

mb_status launch_add_layernorm_fwd(mb_dtype dt, const void* x, const void* r, const void* gamma, const void* beta,
                                   int T_cap, const int32_t* meta, int W, float eps, void* y, void* s, float* mean,
                                   float* rstd, const int32_t* y_rows, hipStream_t stream) {
  const int blocks = (T_cap + kLnWaves - 1) / kLnWaves;
  const bool small = (size_t)W * elem_size(dt) <= 2048;
#define MB_LN_FWD(E, P)                                                                                           \
  hipLaunchKernelGGL((add_layernorm_fwd_kernel<E, P>), dim3(blocks), dim3(kLnThreads), 0, stream, (const E*)x,    \
                     (const E*)r, (const E*)gamma, (const E*)beta, T_cap, meta, W, eps, (E*)y, (E*)s, mean, rstd,  \
                     y_rows)
  if (use_half_pieces(dt, W)) {
    const int per_lane = W / 4 / 64;
#define MB_LN_FWD_H(P)                                                                                            \
  hipLaunchKernelGGL((add_layernorm_fwd_kernel<uint16_t, P, HalfPiece>), dim3(blocks), dim3(kLnThreads), 0, stream, \
                     (const uint16_t*)x, (const uint16_t*)r, (const uint16_t*)gamma, (const uint16_t*)beta, T_cap, \
                     meta, W, eps, (uint16_t*)y, (uint16_t*)s, mean, rstd, y_rows)
    if (per_lane == 1) MB_LN_FWD_H(1);   // (an even count per lane would also split evenly in 16-byte pieces)
    else MB_LN_FWD_H(3);
#undef MB_LN_FWD_H
  } else if (dt == MB_BF16) { if (small) MB_LN_FWD(uint16_t, 2); else MB_LN_FWD(uint16_t, 4); }
  else { if (small) MB_LN_FWD(float, 2); else MB_LN_FWD(float, 4); }
#undef MB_LN_FWD
  return check_launch("add_layernorm_fwd_kernel");
}

mb_status launch_add_layernorm_bwd(mb_dtype dt, const void* dy, const void* s, const void* gamma, const float* mean,
                                   const float* rstd, int T_cap, const int32_t* meta, int W, void* ds, float* dgamma,
                                   float* dbeta, float* part, const int32_t* dy_rows, hipStream_t stream) {
  if (T_cap == 0) {
    // no rows (dy, s, gamma, ... may be NULL): nothing to read, the column sums are zeros
    hipLaunchKernelGGL(add_layernorm_colsum_kernel, dim3((2 * W + 63) / 64), dim3(64 * kColsumSlices), 0, stream, part, 0, W,
                       dgamma, dbeta);
    return check_launch("add_layernorm_colsum_kernel");
  }
  const int blocks = bwd_blocks(T_cap);
  const size_t smem = sizeof(float) * kLnWaves * 2 * (size_t)W;
  const bool small = (size_t)W * elem_size(dt) <= 2048;
#define MB_LN_BWD(E, P)                                                                                          \
  hipLaunchKernelGGL((add_layernorm_bwd_kernel<E, P>), dim3(blocks), dim3(kLnThreads), smem, stream,             \
                     (const E*)dy, (const E*)s, (const E*)gamma, mean, rstd, T_cap, meta, W, (E*)ds, part, dy_rows)
  if (dt == MB_BF16) { if (small) MB_LN_BWD(uint16_t, 2); else MB_LN_BWD(uint16_t, 4); }
  else { if (small) MB_LN_BWD(float, 2); else MB_LN_BWD(float, 4); }
#undef MB_LN_BWD
  mb_status st = check_launch("add_layernorm_bwd_kernel");
  if (st != MB_OK) return st;
  hipLaunchKernelGGL(add_layernorm_colsum_kernel, dim3((2 * W + 63) / 64), dim3(64 * kColsumSlices), 0, stream, part, blocks, W,
                     dgamma, dbeta);
  return check_launch("add_layernorm_colsum_kernel");
}

}  // namespace mb
