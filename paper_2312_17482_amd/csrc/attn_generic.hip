// Generic attention kernels: plain fp32 ALU arithmetic, any head_dim <= 128, fp32 or bf16 storage.
// They serve the fp32 validation workload and head sizes without a matrix-core kernel.  One wave per
// (token, head); the bias of the paper's Eq. 1, -m_h*|i-j|, is evaluated on the fly.
#include "common.h"

namespace mb {
namespace {

__device__ __forceinline__ float to_f32(float x) { return x; }
__device__ __forceinline__ float to_f32(uint16_t x) { return __uint_as_float((uint32_t)x << 16); }
__device__ __forceinline__ void from_f32(float* p, float x) { *p = x; }
__device__ __forceinline__ void from_f32(uint16_t* p, float x) {
  uint32_t u = __float_as_uint(x);
  if ((u & 0x7fffffffu) > 0x7f800000u) { *p = (uint16_t)((u >> 16) | 0x40u); return; }  // NaN stays NaN
  u += 0x7fffu + ((u >> 16) & 1u);                                                      // nearest even
  *p = (uint16_t)(u >> 16);
}

__device__ __forceinline__ float wave_sum(float x) {
  for (int off = 32; off > 0; off >>= 1) x += __shfl_xor(x, off, 64);
  return x;
}
__device__ __forceinline__ float wave_max(float x) {
  for (int off = 32; off > 0; off >>= 1) x = fmaxf(x, __shfl_xor(x, off, 64));
  return x;
}

// Sequence that owns packed token t: the b with cu[b] <= t < cu[b+1] (empty sequences are skipped).
__device__ __forceinline__ int find_seq(const int32_t* __restrict__ cu, int B, int t) {
  int lo = 0, hi = B;  // invariant: cu[lo] <= t < cu[hi]
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (cu[mid] <= t) lo = mid; else hi = mid;
  }
  return lo;
}

// Forward for token t, head h.  Dynamic LDS: D floats (query row) + max_seqlen floats (scores).
template <typename E>
__global__ __launch_bounds__(64) void fwd_generic_kernel(const E* __restrict__ q, const E* __restrict__ k,
                                                         const E* __restrict__ v, int64_t qs, int64_t ks, int64_t vs,
                                                         const int32_t* __restrict__ cu, int B, int T, int H, int D,
                                                         const float* __restrict__ slopes, float scale,
                                                         E* __restrict__ o, int64_t os, float* __restrict__ lse,
                                                         const int32_t* __restrict__ rows, int max_seqlen,
                                                         int32_t* __restrict__ misuse) {
  extern __shared__ float smem[];
  float* sq = smem;
  float* ss = smem + D;
  const int t = blockIdx.x, h = blockIdx.y, lane = threadIdx.x;
  if (t >= cu[B]) return;   // T may be a capacity: rows past the last real token are not touched
  const int b = find_seq(cu, B, t);
  const int start = cu[b], n = cu[b + 1] - start, i = t - start;
  if (n > max_seqlen) {   // longer than the caller promised (the score row in LDS holds max_seqlen entries): skipped
    raise_misuse(misuse);
    if (lane == 0) lse[(int64_t)h * T + t] = __builtin_nanf("");
    return;
  }
  const float slope = slopes[h];
  for (int d = lane; d < D; d += 64) sq[d] = to_f32(q[tok_row(rows, t) * qs + h * D + d]);
  __syncthreads();
  float m = -INFINITY;
  for (int j = lane; j < n; j += 64) {
    const E* kr = k + tok_row(rows, start + j) * ks + h * D;
    float dot = 0.f;
    for (int d = 0; d < D; ++d) dot = fmaf(sq[d], to_f32(kr[d]), dot);
    const float s = scale * dot - slope * fabsf((float)(i - j));
    ss[j] = s;
    m = fmaxf(m, s);
  }
  m = wave_max(m);
  float z = 0.f;
  for (int j = lane; j < n; j += 64) {
    const float e = expf(ss[j] - m);
    ss[j] = e;
    z += e;
  }
  z = wave_sum(z);
  __syncthreads();
  const float inv = 1.f / z;
  for (int d = lane; d < D; d += 64) {
    float acc = 0.f;
    for (int j = 0; j < n; ++j) acc = fmaf(ss[j], to_f32(v[tok_row(rows, start + j) * vs + h * D + d]), acc);
    from_f32(&o[tok_row(rows, t) * os + h * D + d], acc * inv);
  }
  if (lane == 0) lse[(int64_t)h * T + t] = m + logf(z);
}

// Backward, query side, for token i = t, head h: Delta_i, then dS_ij for all j, then dQ_i.
// Dynamic LDS: 2*D floats (q_i, dO_i) + max_seqlen floats (dS row).
template <typename E>
__global__ __launch_bounds__(64) void bwd_generic_row_kernel(
    const E* __restrict__ dout, const E* __restrict__ q, const E* __restrict__ k, const E* __restrict__ v,
    const E* __restrict__ o, const float* __restrict__ lse, int64_t dos, int64_t qs, int64_t ks, int64_t vs,
    int64_t os, const int32_t* __restrict__ cu, int B, int T, int H, int D, const float* __restrict__ slopes,
    float scale, E* __restrict__ dq, int64_t dqs, float* __restrict__ delta, const int32_t* __restrict__ rows,
    int max_seqlen, int32_t* __restrict__ misuse) {
  extern __shared__ float smem[];
  float* sq = smem;
  float* sg = smem + D;
  float* sds = smem + 2 * D;
  const int t = blockIdx.x, h = blockIdx.y, lane = threadIdx.x;
  if (t >= cu[B]) return;   // T may be a capacity: rows past the last real token are not touched
  const int b = find_seq(cu, B, t);
  const int start = cu[b], n = cu[b + 1] - start, i = t - start;
  if (n > max_seqlen) {
    raise_misuse(misuse);
    return;
  }
  const float slope = slopes[h];
  float part = 0.f;
  for (int d = lane; d < D; d += 64) {
    const float g = to_f32(dout[tok_row(rows, t) * dos + h * D + d]);
    sq[d] = to_f32(q[tok_row(rows, t) * qs + h * D + d]);
    sg[d] = g;
    part = fmaf(g, to_f32(o[tok_row(rows, t) * os + h * D + d]), part);
  }
  const float dlt = wave_sum(part);
  if (lane == 0) delta[(int64_t)h * T + t] = dlt;
  __syncthreads();
  const float l = lse[(int64_t)h * T + t];
  for (int j = lane; j < n; j += 64) {
    const E* kr = k + tok_row(rows, start + j) * ks + h * D;
    const E* vr = v + tok_row(rows, start + j) * vs + h * D;
    float dot = 0.f, dp = 0.f;
    for (int d = 0; d < D; ++d) {
      dot = fmaf(sq[d], to_f32(kr[d]), dot);
      dp = fmaf(sg[d], to_f32(vr[d]), dp);
    }
    const float p = expf(scale * dot - slope * fabsf((float)(i - j)) - l);
    sds[j] = p * (dp - dlt);
  }
  __syncthreads();
  for (int d = lane; d < D; d += 64) {
    float acc = 0.f;
    for (int j = 0; j < n; ++j) acc = fmaf(sds[j], to_f32(k[tok_row(rows, start + j) * ks + h * D + d]), acc);
    from_f32(&dq[tok_row(rows, t) * dqs + h * D + d], scale * acc);
  }
}

// Backward, key side, for token j = t, head h: P_ij and dS_ij for all i, then dV_j and dK_j.
// Dynamic LDS: 2*D floats (k_j, v_j) + 2*max_seqlen floats (P column, dS column).
template <typename E>
__global__ __launch_bounds__(64) void bwd_generic_col_kernel(
    const E* __restrict__ dout, const E* __restrict__ q, const E* __restrict__ k, const E* __restrict__ v,
    const float* __restrict__ lse, const float* __restrict__ delta, int64_t dos, int64_t qs, int64_t ks,
    int64_t vs, const int32_t* __restrict__ cu, int B, int T, int H, int D, int max_seqlen,
    const float* __restrict__ slopes, float scale, E* __restrict__ dk, E* __restrict__ dv, int64_t dks,
    int64_t dvs, const int32_t* __restrict__ rows, int32_t* __restrict__ misuse) {
  extern __shared__ float smem[];
  float* sk = smem;
  float* sv = smem + D;
  float* sp = smem + 2 * D;
  float* sds = sp + max_seqlen;
  const int t = blockIdx.x, h = blockIdx.y, lane = threadIdx.x;
  if (t >= cu[B]) return;   // T may be a capacity: rows past the last real token are not touched
  const int b = find_seq(cu, B, t);
  const int start = cu[b], n = cu[b + 1] - start, j = t - start;
  if (n > max_seqlen) {
    raise_misuse(misuse);
    return;
  }
  const float slope = slopes[h];
  for (int d = lane; d < D; d += 64) {
    sk[d] = to_f32(k[tok_row(rows, t) * ks + h * D + d]);
    sv[d] = to_f32(v[tok_row(rows, t) * vs + h * D + d]);
  }
  __syncthreads();
  for (int i = lane; i < n; i += 64) {
    const E* qr = q + tok_row(rows, start + i) * qs + h * D;
    const E* gr = dout + tok_row(rows, start + i) * dos + h * D;
    float dot = 0.f, dp = 0.f;
    for (int d = 0; d < D; ++d) {
      dot = fmaf(to_f32(qr[d]), sk[d], dot);
      dp = fmaf(to_f32(gr[d]), sv[d], dp);
    }
    const float p = expf(scale * dot - slope * fabsf((float)(i - j)) - lse[(int64_t)h * T + start + i]);
    sp[i] = p;
    sds[i] = p * (dp - delta[(int64_t)h * T + start + i]);
  }
  __syncthreads();
  for (int d = lane; d < D; d += 64) {
    float av = 0.f, ak = 0.f;
    for (int i = 0; i < n; ++i) {
      av = fmaf(sp[i], to_f32(dout[tok_row(rows, start + i) * dos + h * D + d]), av);
      ak = fmaf(sds[i], to_f32(q[tok_row(rows, start + i) * qs + h * D + d]), ak);
    }
    from_f32(&dv[tok_row(rows, t) * dvs + h * D + d], av);
    from_f32(&dk[tok_row(rows, t) * dks + h * D + d], scale * ak);
  }
}

template <typename E>
mb_status fwd_t(const AttnShape& s, const void* q, const void* k, const void* v, int64_t qs, int64_t ks, int64_t vs,
                void* o, int64_t os, float* lse, hipStream_t stream) {
  const size_t smem = sizeof(float) * ((size_t)s.D + s.max_seqlen);
  hipLaunchKernelGGL(fwd_generic_kernel<E>, dim3(s.T, s.H), dim3(64), smem, stream, (const E*)q, (const E*)k,
                     (const E*)v, qs, ks, vs, s.cu_seqlens, s.B, s.T, s.H, s.D, s.slopes, s.scale, (E*)o, os, lse, s.token_rows,
                     s.max_seqlen, s.misuse);
  return check_launch("fwd_generic_kernel");
}

template <typename E>
mb_status bwd_t(const AttnShape& s, const void* dout, const void* q, const void* k, const void* v, const void* o,
                const float* lse, int64_t dos, int64_t qs, int64_t ks, int64_t vs, int64_t os, void* dq, void* dk,
                void* dv, int64_t dqs, int64_t dks, int64_t dvs, float* delta, hipStream_t stream) {
  const size_t smem_row = sizeof(float) * (2 * (size_t)s.D + s.max_seqlen);
  hipLaunchKernelGGL(bwd_generic_row_kernel<E>, dim3(s.T, s.H), dim3(64), smem_row, stream, (const E*)dout,
                     (const E*)q, (const E*)k, (const E*)v, (const E*)o, lse, dos, qs, ks, vs, os, s.cu_seqlens, s.B,
                     s.T, s.H, s.D, s.slopes, s.scale, (E*)dq, dqs, delta, s.token_rows, s.max_seqlen, s.misuse);
  mb_status st = check_launch("bwd_generic_row_kernel");
  if (st != MB_OK) return st;
  const size_t smem_col = sizeof(float) * (2 * (size_t)s.D + 2 * (size_t)s.max_seqlen);
  hipLaunchKernelGGL(bwd_generic_col_kernel<E>, dim3(s.T, s.H), dim3(64), smem_col, stream, (const E*)dout,
                     (const E*)q, (const E*)k, (const E*)v, lse, delta, dos, qs, ks, vs, s.cu_seqlens, s.B, s.T, s.H,
                     s.D, s.max_seqlen, s.slopes, s.scale, (E*)dk, (E*)dv, dks, dvs, s.token_rows, s.misuse);
  return check_launch("bwd_generic_col_kernel");
}

}  // namespace

mb_status launch_attn_fwd_generic(const AttnShape& s, mb_dtype dt, const void* q, const void* k, const void* v,
                                  int64_t qs, int64_t ks, int64_t vs, void* o, int64_t os, float* lse,
                                  hipStream_t stream) {
  return dt == MB_F32 ? fwd_t<float>(s, q, k, v, qs, ks, vs, o, os, lse, stream)
                      : fwd_t<uint16_t>(s, q, k, v, qs, ks, vs, o, os, lse, stream);
}

mb_status launch_attn_bwd_generic(const AttnShape& s, mb_dtype dt, const void* dout, const void* q, const void* k,
                                  const void* v, const void* o, const float* lse, int64_t dos, int64_t qs,
                                  int64_t ks, int64_t vs, int64_t os, void* dq, void* dk, void* dv, int64_t dqs,
                                  int64_t dks, int64_t dvs, float* delta_ws, hipStream_t stream) {
  return dt == MB_F32 ? bwd_t<float>(s, dout, q, k, v, o, lse, dos, qs, ks, vs, os, dq, dk, dv, dqs, dks, dvs,
                                     delta_ws, stream)
                      : bwd_t<uint16_t>(s, dout, q, k, v, o, lse, dos, qs, ks, vs, os, dq, dk, dv, dqs, dks, dvs,
                                        delta_ws, stream);
}

}  // namespace mb
