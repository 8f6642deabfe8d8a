// Internal declarations shared by the translation units of libmosaicattn (not part of the ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "mosaic_attn.h"

namespace mb {

// Records a message for mb_last_error() and returns `code`.
mb_status fail(mb_status code, const char* fmt, ...) __attribute__((format(printf, 2, 3)));
void clear_error();
// Maps the HIP launch status to MB_OK / MB_ERR_HIP.
mb_status check_launch(const char* what);

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline size_t elem_size(mb_dtype dt) { return dt == MB_F32 ? 4 : 2; }
inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

struct AttnShape {
  int B, T, max_seqlen, H, D;
  const int32_t* cu_seqlens;
  const float* slopes;
  float scale;
  const int32_t* token_rows;   // NULL, or [T]: row of token t inside the activation buffers
};

// Row of packed token t inside the activation buffers: t itself, or token_rows[t] when the call reads
// and writes a padded batch directly.
__device__ __forceinline__ int64_t tok_row(const int32_t* __restrict__ rows, int t) {
  return rows ? (int64_t)rows[t] : (int64_t)t;
}

// How the any-length attention kernels find the buffer rows of a sequence's tokens (template parameter):
//   kRowsPerLane          every row's address is formed per lane (token_rows looked up when given); no limit
//                         on strides.
//   kRowsIdentity         no token_rows: token t sits at row t, so a sequence's rows are consecutive.
//   kRowsMaybeContiguous  token_rows given: a sequence whose rows are listed in ascending order with first
//                         and last n - 1 apart (the usual case: padding behind each sequence) is handled
//                         like kRowsIdentity from its first row, any other like kRowsPerLane.
// The last two require that a sequence's rows span fewer than 2^31 bytes.
enum { kRowsPerLane = 0, kRowsIdentity = 1, kRowsMaybeContiguous = 2 };

// Longest-sequence-first work order for kernels whose workgroups run for a time that grows with the
// sequence length: finds the sequence whose length has rank `rank` (0 = longest; ties by index), so
// that the heaviest workgroups are dispatched first and short ones fill the tail, and returns its index
// with its first token in *start and its length in *len.  Every thread of the block must call it (it
// contains barriers); `lds` is kSortLdsWords words of LDS that nothing else writes.
// Each sequence gets the key (length, reversed index) packed in one word; keys and sequence starts are
// staged in LDS once (the only global loads), and a thread ranks its candidate by counting the larger
// keys, sixteen per round of LDS reads (with few sequences, two or four threads share a candidate).  For
// B > kSortMaxB the order is left as it is (many sequences balance by themselves).
static constexpr int kSortMaxB = 512;
static constexpr int kSortLdsWords = 2 * kSortMaxB + 24;
__device__ __forceinline__ int seq_by_length_rank(const int32_t* __restrict__ cu, int B, int rank, uint32_t* lds,
                                                  int* start, int* len) {
  if (B > kSortMaxB) {
    const int s0 = __builtin_amdgcn_readfirstlane(cu[rank]);
    *start = s0;
    *len = __builtin_amdgcn_readfirstlane(cu[rank + 1]) - s0;
    return rank;
  }
  uint32_t* keys = lds;                                        // [kSortMaxB + 16]
  int* starts = reinterpret_cast<int*>(lds) + kSortMaxB + 16;  // [kSortMaxB + 1]
  int* slot = starts + kSortMaxB + 1;                          // [1]
  const int Bp = (B + 15) & ~15;                               // keys are scanned 16 at a time
  for (int i = threadIdx.x; i < Bp; i += blockDim.x) {
    const int s0 = cu[min(i, B)], s1 = cu[min(i + 1, B)];      // both loads in flight together
    if (i < B) starts[i] = s0;
    // padding keys are 0: never larger than a real key
    keys[i] = i < B ? ((uint32_t)min(s1 - s0, (1 << 22)) << 9) | (uint32_t)(kSortMaxB - 1 - i) : 0u;
  }
  if (threadIdx.x == 0) starts[B] = cu[B];
  __syncthreads();
  // `split` neighbouring lanes share a candidate, each scanning every split-th group of 16 keys
  const int split = B <= 64 ? 4 : (B <= 128 ? 2 : 1);
  const int part = threadIdx.x & (split - 1);
  for (int cand = threadIdx.x / split; cand < B; cand += blockDim.x / split) {
    const uint32_t mine = keys[cand];
    int r = 0;
    for (int other = 16 * part; other < Bp; other += 16 * split) {
      uint4 k4[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) k4[u] = *reinterpret_cast<const uint4*>(&keys[other + 4 * u]);
#pragma unroll
      for (int u = 0; u < 4; ++u)
        r += (k4[u].x > mine ? 1 : 0) + (k4[u].y > mine ? 1 : 0) + (k4[u].z > mine ? 1 : 0) + (k4[u].w > mine ? 1 : 0);
    }
    if (split > 1) r += __shfl_xor(r, 1, 64);
    if (split > 2) r += __shfl_xor(r, 2, 64);
    if (r == rank) *slot = cand;
  }
  __syncthreads();
  // (values read from LDS: readfirstlane tells the compiler that they are wave-uniform)
  const int b = __builtin_amdgcn_readfirstlane(*slot);
  const int s0 = __builtin_amdgcn_readfirstlane(starts[b]);
  *start = s0;
  *len = __builtin_amdgcn_readfirstlane(starts[b + 1]) - s0;
  return b;
}

// Workspace of the backward attention: Delta [H, T] float, then the sequence order [B] int32.
__host__ __device__ inline size_t attn_bwd_delta_bytes(int H, int T) {
  return ((size_t)H * (size_t)T * sizeof(float) + 255) / 256 * 256;
}
__host__ __device__ inline size_t attn_bwd_workspace_bytes(int B, int H, int T) {
  return attn_bwd_delta_bytes(H, T) + ((size_t)B * sizeof(int32_t) + 255) / 256 * 256;
}

// ---- launchers (each enqueues on `stream`, returns MB_OK or MB_ERR_HIP) ----
mb_status launch_unpad_index(const int32_t* mask, int B, int L, int32_t* seqlens, int32_t* cu_seqlens,
                             int32_t* indices, int32_t* meta, hipStream_t stream);
mb_status launch_gather_rows(const void* padded, const int32_t* indices, int T_cap, const int32_t* meta,
                             int row_bytes, void* packed, hipStream_t stream);
mb_status launch_scatter_rows(const void* packed, const int32_t* indices, int T_cap, const int32_t* meta,
                              int rows_padded, int row_bytes, void* padded, hipStream_t stream);

mb_status launch_zero_padding(const int32_t* indices, int T_cap, const int32_t* meta, int rows_padded,
                              int row_bytes, void* padded, hipStream_t stream);

// Add & LayerNorm.  The backward writes one partial row of column sums per workgroup, at most this many.
static constexpr int kLayerNormMaxParts = 1024;
// Ceiling probes (kind 0: bf16 matrix cores, 1: vector fused multiply-add, 2: vector exponential).
mb_status launch_probe(int kind, int iters, float* out, double* work_per_launch, hipStream_t stream);

// GeGLU feed-forward, forward (bf16; hidden a multiple of 256, inter a multiple of 128).
mb_status launch_geglu_fwd(const void* x, const void* w1v, const void* w2, int T_cap, const int32_t* meta,
                           int hidden, int inter, void* act, void* y, hipStream_t stream);
// Backward of the feed-forward (hidden and inter multiples of 256): data gradient dx (bf16) and the fp32
// gradients of the stored (transposed) weight matrices; `workspace` holds geglu_bwd_workspace_bytes bytes.
size_t geglu_bwd_workspace_bytes(int T_cap, int hidden, int inter);
mb_status launch_geglu_bwd(const void* dy, const void* x, const void* w1v, const void* w2, const void* act,
                           const void* hg_saved, int T_cap, const int32_t* meta, int hidden, int inter, void* dx,
                           float* dw1v, float* dw2, void* workspace, hipStream_t stream);
// The pieces of the unfused arrangements: a bias-free projection y = x wt^T (n_in a multiple of 128, n_out a
// multiple of 256 or of 192) and the activation pass act = GeLU(h) (*) gate over rows of stride ld.
mb_status launch_linear_fwd(const void* x, const void* wt, int T_cap, const int32_t* meta, int n_in, int n_out,
                            void* y, hipStream_t stream);
mb_status launch_gelu_gate(const void* h, const void* gate, int64_t ld, int T_cap, const int32_t* meta, int inter,
                           void* act, hipStream_t stream);

mb_status launch_add_layernorm_fwd(mb_dtype dt, const void* x, const void* r, const void* gamma, const void* beta,
                                   int T_cap, const int32_t* meta, int W, float eps, void* y, void* s, float* mean,
                                   float* rstd, const int32_t* y_rows, hipStream_t stream);
mb_status launch_add_layernorm_bwd(mb_dtype dt, const void* dy, const void* s, const void* gamma, const float* mean,
                                   const float* rstd, int T_cap, const int32_t* meta, int W, void* ds, float* dgamma,
                                   float* dbeta, float* part, const int32_t* dy_rows, hipStream_t stream);

// Generic ALU kernels: any D <= 128, fp32 or bf16 storage, fp32 arithmetic.
// Their backward keeps two score rows of max_seqlen floats plus two head vectors in LDS and must stay
// within the 64 KB a kernel may use without opting in to more.
static constexpr int kGenericMaxSeqlen = 8000;
mb_status launch_attn_fwd_generic(const AttnShape& s, mb_dtype dt, const void* q, const void* k, const void* v,
                                  int64_t qs, int64_t ks, int64_t vs, void* o, int64_t os, float* lse,
                                  hipStream_t stream);
mb_status launch_attn_bwd_generic(const AttnShape& s, mb_dtype dt, const void* dout, const void* q, const void* k,
                                  const void* v, const void* o, const float* lse, int64_t dos, int64_t qs,
                                  int64_t ks, int64_t vs, int64_t os, void* dq, void* dk, void* dv, int64_t dqs,
                                  int64_t dks, int64_t dvs, float* delta_ws, hipStream_t stream);

// bf16, D = 64 matrix-core kernels.
mb_status launch_attn_fwd_mfma(const AttnShape& s, const void* q, const void* k, const void* v, int64_t qs,
                               int64_t ks, int64_t vs, void* o, int64_t os, float* lse, hipStream_t stream);
mb_status launch_attn_bwd_mfma(const AttnShape& s, const void* dout, const void* q, const void* k, const void* v,
                               const void* o, const float* lse, int64_t dos, int64_t qs, int64_t ks, int64_t vs,
                               int64_t os, void* dq, void* dk, void* dv, int64_t dqs, int64_t dks, int64_t dvs,
                               float* delta_ws, hipStream_t stream);

}  // namespace mb
