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
  const int32_t* key_lens;     // NULL, or [B]: only the first key_lens[b] tokens of sequence b act as keys
  const int32_t* token_rows;   // NULL, or [T]: row of token t inside the activation buffers
  const int32_t* plan;         // NULL, or a work plan the caller built with mb_attn_plan for these very arguments
  int32_t* misuse;             // this device's sticky flag: set by a kernel that meets a sequence longer than max_seqlen
};

// Device word that the attention kernels set when a sequence is longer than the max_seqlen their launch was
// sized for (such a sequence is skipped, never truncated); read and cleared by mb_device_status.  One copy per
// device; returns its device address for the current device in *flag.
mb_status misuse_flag_address(int32_t** flag);

// What a kernel does on meeting such a sequence: raise the flag (every thread stores the same word).
__device__ __forceinline__ void raise_misuse(int32_t* flag) { *flag = 1; }

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

// Workspace of the backward attention: Delta [H, T] float, then (matrix-core kernels, max_seqlen > 128) the
// work plan; the forward's workspace is the work plan alone (nothing for max_seqlen <= 128).
__host__ __device__ inline size_t attn_bwd_delta_bytes(int H, int T) {
  return ((size_t)H * (size_t)T * sizeof(float) + 255) / 256 * 256;
}
size_t attn_fwd_mfma_workspace_bytes(int B, int max_seqlen, int H);
size_t attn_bwd_mfma_workspace_bytes(int B, int T, int max_seqlen, int H);
// The work plan of the any-length kernels (see attn_plan.h): its size, and the launch that builds it.  `lse` non-NULL:
// the log-sum-exp rows ([H, T]) of sequences the plan skips as longer than max_seqlen are set to NaN.
size_t attn_plan_workspace_bytes(int B, int max_seqlen, int H);
mb_status launch_attn_plan(const AttnShape& s, int32_t* plan, float* lse, hipStream_t stream);

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
mb_status launch_probe_bwd_traffic(const void* qkv, const void* dout, const void* o, void* dqkv, const int32_t* cu,
                                   int B, int H, hipStream_t stream);

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
                               int64_t ks, int64_t vs, void* o, int64_t os, float* lse, void* workspace,
                               hipStream_t stream);
mb_status launch_attn_bwd_mfma(const AttnShape& s, const void* dout, const void* q, const void* k, const void* v,
                               const void* o, const float* lse, int64_t dos, int64_t qs, int64_t ks, int64_t vs,
                               int64_t os, void* dq, void* dk, void* dv, int64_t dqs, int64_t dks, int64_t dvs,
                               float* delta_ws, hipStream_t stream);

}  // namespace mb
