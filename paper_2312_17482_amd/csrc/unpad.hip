// Padding removal and restoration ("Unpadding" paragraph of the paper): index maps by wave ballot +
// prefix scan, and the two row-copy kernels.  All integer work; results are unique, so they must
// match a plain double loop bit for bit.
#include "common.h"

namespace mb {
namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / 64;

__device__ __forceinline__ int wave_sum(int x) {
  for (int off = 32; off > 0; off >>= 1) x += __shfl_down(x, off, 64);
  return __shfl(x, 0, 64);
}
__device__ __forceinline__ int wave_max(int x) {
  for (int off = 32; off > 0; off >>= 1) x = max(x, __shfl_down(x, off, 64));
  return __shfl(x, 0, 64);
}
// Sum (or max) of one int per thread over the block; every thread gets the result.
template <bool kMax>
__device__ __forceinline__ int block_reduce(int x, int* lds /*[kWaves]*/) {
  x = kMax ? wave_max(x) : wave_sum(x);
  __syncthreads();  // protect lds from the previous use
  if ((threadIdx.x & 63) == 0) lds[threadIdx.x >> 6] = x;
  __syncthreads();
  int r = lds[0];
  for (int w = 1; w < kWaves; ++w) r = kMax ? max(r, lds[w]) : r + lds[w];
  return r;
}

// seqlens[b] = number of nonzero mask entries of row b.  One block per row.
__global__ __launch_bounds__(kThreads) void seqlens_kernel(const int32_t* __restrict__ mask, int L,
                                                           int32_t* __restrict__ seqlens) {
  __shared__ int lds[kWaves];
  const int b = blockIdx.x;
  const int32_t* row = mask + (size_t)b * L;
  int n = 0;
  for (int l = threadIdx.x; l < L; l += kThreads) n += (row[l] != 0);
  n = block_reduce<false>(n, lds);
  if (threadIdx.x == 0) seqlens[b] = n;
}

// One block per row b: cu_seqlens[b] = sum of seqlens before b, then stream compaction of the row
// (ballot + popcount rank inside a wave, running offsets across waves and chunks).  Block 0 also
// writes max_seqlen, the last block writes cu_seqlens[B] and T.  With B == 0 a single block writes
// the empty result.
__global__ __launch_bounds__(kThreads) void compact_kernel(const int32_t* __restrict__ mask, int B, int L,
                                                           const int32_t* __restrict__ seqlens,
                                                           int32_t* __restrict__ cu_seqlens,
                                                           int32_t* __restrict__ indices,
                                                           int32_t* __restrict__ meta) {
  __shared__ int lds[kWaves];
  __shared__ int wave_count[kWaves];
  const int b = blockIdx.x;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  if (B == 0) {
    if (tid == 0) { cu_seqlens[0] = 0; meta[0] = 0; meta[1] = 0; }
    return;
  }
  int part = 0;
  for (int r = tid; r < b; r += kThreads) part += seqlens[r];
  const int prefix = block_reduce<false>(part, lds);
  if (b == 0) {
    int m = 0;
    for (int r = tid; r < B; r += kThreads) m = max(m, seqlens[r]);
    m = block_reduce<true>(m, lds);
    if (tid == 0) meta[1] = m;
  }
  if (tid == 0) {
    cu_seqlens[b] = prefix;
    if (b == B - 1) {
      const int total = prefix + seqlens[b];
      cu_seqlens[B] = total;
      meta[0] = total;
    }
  }
  const int32_t* row = mask + (size_t)b * L;
  int running = prefix;
  for (int base = 0; base < L; base += kThreads) {
    const int l = base + tid;
    const bool keep = (l < L) && (row[l] != 0);
    const unsigned long long vote = __ballot(keep);
    const int rank = __popcll(vote & ((1ull << lane) - 1ull));
    __syncthreads();  // wave_count free again
    if (lane == 0) wave_count[wave] = __popcll(vote);
    __syncthreads();
    int before = 0, total = 0;
    for (int w = 0; w < kWaves; ++w) {
      const int c = wave_count[w];
      before += (w < wave) ? c : 0;
      total += c;
    }
    if (keep) indices[running + before + rank] = b * L + l;
    running += total;
  }
}

// ---- row copies.  A row is `units` 16-byte pieces; 32 lanes walk one row, 8 rows per block. ----
constexpr int kRowsPerBlock = 8;
constexpr int kLanesPerRow = kThreads / kRowsPerBlock;  // 32

// Cache policy: a row that is read here for the last time (the padded input of a gather, the packed
// input of a scatter) is loaded non-temporally, and the padded output of a scatter is stored
// non-temporally, so that these one-pass streams do not push the packed activations, which the attention
// kernels are about to read, out of the L2 and the memory-side cache.  A gather's packed output is stored
// normally for the same reason.
typedef unsigned int nt_u32x4 __attribute__((ext_vector_type(4)));
template <bool kNtLoad, bool kNtStore>
__device__ __forceinline__ void copy_row(const uint4* __restrict__ src, uint4* __restrict__ dst, int units, int c) {
  const nt_u32x4* s = reinterpret_cast<const nt_u32x4*>(src);
  nt_u32x4* d = reinterpret_cast<nt_u32x4*>(dst);
  auto ld = [&](int u) { return kNtLoad ? __builtin_nontemporal_load(s + u) : s[u]; };
  auto st = [&](int u, nt_u32x4 v) { if (kNtStore) __builtin_nontemporal_store(v, d + u); else d[u] = v; };
  int u = c;
  for (; u + 3 * kLanesPerRow < units; u += 4 * kLanesPerRow) {
    const nt_u32x4 a0 = ld(u), a1 = ld(u + kLanesPerRow), a2 = ld(u + 2 * kLanesPerRow), a3 = ld(u + 3 * kLanesPerRow);
    st(u, a0); st(u + kLanesPerRow, a1); st(u + 2 * kLanesPerRow, a2); st(u + 3 * kLanesPerRow, a3);
  }
  for (; u < units; u += kLanesPerRow) st(u, ld(u));
}

__global__ __launch_bounds__(kThreads) void gather_rows_kernel(const uint4* __restrict__ padded,
                                                               const int32_t* __restrict__ indices, int T_cap,
                                                               const int32_t* __restrict__ meta, int units,
                                                               uint4* __restrict__ packed) {
  const int T = meta ? min(meta[0], T_cap) : T_cap;
  const int t = blockIdx.x * kRowsPerBlock + (threadIdx.x / kLanesPerRow);
  if (t >= T) return;
  const int p = indices[t];
  copy_row<true, false>(padded + (size_t)p * units, packed + (size_t)t * units, units, threadIdx.x % kLanesPerRow);
}

// Block = 8 consecutive padded rows p0..p0+7.  Wave 0 finds t0 = first t with indices[t] >= p0 by a
// 64-ary search (indices ascending); the rows of the block that are kept then sit at t0, t0+1, ...
__global__ __launch_bounds__(kThreads) void scatter_rows_kernel(const uint4* __restrict__ packed,
                                                                const int32_t* __restrict__ indices, int T_cap,
                                                                const int32_t* __restrict__ meta, int rows_padded,
                                                                int units, uint4* __restrict__ padded) {
  __shared__ int s_t0, s_off;
  __shared__ int s_v[128];
  const int T = meta ? min(meta[0], T_cap) : T_cap;
  const int p0 = blockIdx.x * kRowsPerBlock;
  if (threadIdx.x < 64) {
    const int lane = threadIdx.x;
    int lo = 0, hi = T;  // answer in [lo, hi]; elements at positions >= hi are known to be >= p0 (or the end)
    while (hi - lo > 64) {
      const int step = (hi - lo + 63) / 64;
      const long long pos = (long long)lo + (long long)(lane + 1) * step - 1;
      const bool less = (pos < hi) && (indices[pos] < p0);
      const int c = __popcll(__ballot(less));  // monotone: the first c probes are < p0
      const long long nlo = (long long)lo + (long long)c * step;
      const long long nhi = nlo + step - 1;
      lo = (int)nlo;
      hi = (int)(nhi < hi ? nhi : hi);
    }
    // last probe: two entries per lane (the end of the list counts as +infinity), so that the entries from t0 on,
    // which say where the block's rows come from, are already here and cost no further round trip
    const int v0 = lo + lane < T ? indices[lo + lane] : 0x7fffffff;
    const int v1 = lo + 64 + lane < T ? indices[lo + 64 + lane] : 0x7fffffff;
    const int t0 = lo + __popcll(__ballot(v0 < p0));   // entries at and beyond hi are >= p0: t0 <= hi <= lo + 64
    s_v[lane] = v0;
    s_v[64 + lane] = v1;
    if (lane == 0) { s_t0 = t0; s_off = t0 - lo; }
  }
  __syncthreads();
  const int t0 = s_t0;
  const int r = threadIdx.x / kLanesPerRow;
  const int p = p0 + r;
  if (p >= rows_padded) return;
  int c = 0;  // kept rows of this block before row p
  bool kept = false;
  for (int x = 0; x < kRowsPerBlock; ++x) {
    const int v = s_v[s_off + x];   // indices[t0 + x], +infinity past the end (s_off + x <= 71)
    c += v < p ? 1 : 0;
    kept = kept || v == p;
  }
  uint4* dst = padded + (size_t)p * units;
  const int lane = threadIdx.x % kLanesPerRow;
  if (kept) {
    copy_row<true, true>(packed + (size_t)(t0 + c) * units, dst, units, lane);
  } else {
    const nt_u32x4 z = {0u, 0u, 0u, 0u};
    for (int u = lane; u < units; u += kLanesPerRow) __builtin_nontemporal_store(z, reinterpret_cast<nt_u32x4*>(dst) + u);
  }
}

// Zero the rows that `indices` does not list.  Block = 64 consecutive padded rows p0..p0+63: wave 0 finds
// t0 = first t with indices[t] >= p0 (64-ary search) and marks the listed rows of the block, which are
// indices[t0], indices[t0+1], ... below p0+64; everything unmarked is padding and is zero-filled.
constexpr int kZeroRows = 64;
__global__ __launch_bounds__(kThreads) void zero_padding_kernel(const int32_t* __restrict__ indices, int T_cap,
                                                                const int32_t* __restrict__ meta, int rows_padded,
                                                                int units, uint4* __restrict__ padded) {
  __shared__ int s_listed[kZeroRows];
  const int T = meta ? min(meta[0], T_cap) : T_cap;
  const int p0 = blockIdx.x * kZeroRows;
  if (threadIdx.x < kZeroRows) s_listed[threadIdx.x] = 0;
  __syncthreads();
  if (threadIdx.x < 64) {
    const int lane = threadIdx.x;
    int lo = 0, hi = T;
    while (hi - lo > 64) {
      const int step = (hi - lo + 63) / 64;
      const long long pos = (long long)lo + (long long)(lane + 1) * step - 1;
      const bool less = (pos < hi) && (indices[pos] < p0);
      const int c = __popcll(__ballot(less));
      const long long nlo = (long long)lo + (long long)c * step;
      const long long nhi = nlo + step - 1;
      lo = (int)nlo;
      hi = (int)(nhi < hi ? nhi : hi);
    }
    const bool less = (lo + lane < hi) && (indices[lo + lane] < p0);
    const int t0 = lo + __popcll(__ballot(less));
    if (t0 + lane < T) {
      const int v = indices[t0 + lane];   // ascending: the listed rows of this block come first
      if (v < p0 + kZeroRows) s_listed[v - p0] = 1;
    }
  }
  __syncthreads();
  const int lane = threadIdx.x % kLanesPerRow;
  const nt_u32x4 z = {0u, 0u, 0u, 0u};
  for (int r = threadIdx.x / kLanesPerRow; r < kZeroRows; r += kRowsPerBlock) {
    const int p = p0 + r;
    if (p < rows_padded && !s_listed[r]) {
      nt_u32x4* dst = reinterpret_cast<nt_u32x4*>(padded + (size_t)p * units);
      for (int u = lane; u < units; u += kLanesPerRow) __builtin_nontemporal_store(z, dst + u);
    }
  }
}

}  // namespace

mb_status launch_unpad_index(const int32_t* mask, int B, int L, int32_t* seqlens, int32_t* cu_seqlens,
                             int32_t* indices, int32_t* meta, hipStream_t stream) {
  if (B > 0) {
    hipLaunchKernelGGL(seqlens_kernel, dim3(B), dim3(kThreads), 0, stream, mask, L, seqlens);
    mb_status st = check_launch("seqlens_kernel");
    if (st != MB_OK) return st;
  }
  hipLaunchKernelGGL(compact_kernel, dim3(B > 0 ? B : 1), dim3(kThreads), 0, stream, mask, B, L, seqlens,
                     cu_seqlens, indices, meta);
  return check_launch("compact_kernel");
}

mb_status launch_gather_rows(const void* padded, const int32_t* indices, int T_cap, const int32_t* meta,
                             int row_bytes, void* packed, hipStream_t stream) {
  const int blocks = (T_cap + kRowsPerBlock - 1) / kRowsPerBlock;
  hipLaunchKernelGGL(gather_rows_kernel, dim3(blocks), dim3(kThreads), 0, stream, (const uint4*)padded, indices,
                     T_cap, meta, row_bytes / 16, (uint4*)packed);
  return check_launch("gather_rows_kernel");
}

mb_status launch_scatter_rows(const void* packed, const int32_t* indices, int T_cap, const int32_t* meta,
                              int rows_padded, int row_bytes, void* padded, hipStream_t stream) {
  const int blocks = (rows_padded + kRowsPerBlock - 1) / kRowsPerBlock;
  hipLaunchKernelGGL(scatter_rows_kernel, dim3(blocks), dim3(kThreads), 0, stream, (const uint4*)packed,
                     indices, T_cap, meta, rows_padded, row_bytes / 16, (uint4*)padded);
  return check_launch("scatter_rows_kernel");
}

mb_status launch_zero_padding(const int32_t* indices, int T_cap, const int32_t* meta, int rows_padded,
                              int row_bytes, void* padded, hipStream_t stream) {
  const int blocks = (rows_padded + kZeroRows - 1) / kZeroRows;
  hipLaunchKernelGGL(zero_padding_kernel, dim3(blocks), dim3(kThreads), 0, stream, indices, T_cap, meta,
                     rows_padded, row_bytes / 16, (uint4*)padded);
  return check_launch("zero_padding_kernel");
}

}  // namespace mb
