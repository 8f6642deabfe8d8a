// C ABI of libmosaicattn: argument validation on the host (before any launch, so every error path is
// testable without a GPU), then dispatch to the kernel launchers.
#include <atomic>
#include <cmath>
#include <cstdarg>
#include <cstdio>

#include "common.h"

// Device-resident state of the library (one copy per GPU, held until the process ends):
//   g_misuse   sticky word set by an attention kernel that met a sequence longer than max_seqlen;
//   scratch    the workspace of mb_alibi_attn_bwd_static, for callers that cannot allocate.
// Host code never passes these names to a kernel (on the host they are stand-ins, not device addresses): it
// asks the runtime for their device addresses once per device and uses those.
__device__ int32_t g_misuse = 0;
static constexpr size_t kStaticScratchBytes = MB_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace mb {
namespace {
thread_local char g_error[512] = "";

constexpr int kMaxDevices = 64;
std::atomic<int32_t*> g_misuse_ptr[kMaxDevices];
std::atomic<unsigned char*> g_scratch_ptr[kMaxDevices];
}

mb_status fail(mb_status code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_error, sizeof(g_error), fmt, ap);
  va_end(ap);
  return code;
}
void clear_error() { g_error[0] = '\0'; }

static mb_status current_device(int* dev) {
  const hipError_t e = hipGetDevice(dev);
  if (e != hipSuccess) return fail(MB_ERR_HIP, "hipGetDevice: %s", hipGetErrorString(e));
  if (*dev < 0 || *dev >= kMaxDevices) return fail(MB_ERR_UNSUPPORTED, "device ordinal %d is beyond %d", *dev, kMaxDevices);
  return MB_OK;
}

mb_status misuse_flag_address(int32_t** flag) {
  int dev = 0;
  const mb_status st = current_device(&dev);
  if (st != MB_OK) return st;
  int32_t* p = g_misuse_ptr[dev].load(std::memory_order_acquire);
  if (p == nullptr) {   // first call on this device (two racing threads get the same answer)
    const hipError_t e = hipGetSymbolAddress(reinterpret_cast<void**>(&p), HIP_SYMBOL(g_misuse));
    if (e != hipSuccess || p == nullptr) return fail(MB_ERR_HIP, "hipGetSymbolAddress(g_misuse): %s", hipGetErrorString(e));
    g_misuse_ptr[dev].store(p, std::memory_order_release);
  }
  *flag = p;
  return MB_OK;
}

// Device address of this GPU's copy of the static scratch array.
static mb_status static_scratch_address(unsigned char** ptr) {
  int dev = 0;
  const mb_status st = current_device(&dev);
  if (st != MB_OK) return st;
  unsigned char* p = g_scratch_ptr[dev].load(std::memory_order_acquire);
  if (p == nullptr) {
    const hipError_t e = hipGetSymbolAddress(reinterpret_cast<void**>(&p), HIP_SYMBOL(scratch));
    if (e != hipSuccess || p == nullptr) return fail(MB_ERR_HIP, "hipGetSymbolAddress(scratch): %s", hipGetErrorString(e));
    g_scratch_ptr[dev].store(p, std::memory_order_release);
  }
  *ptr = p;
  return MB_OK;
}

mb_status check_launch(const char* what) {
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(MB_ERR_HIP, "%s: %s", what, hipGetErrorString(e));
  return MB_OK;
}

namespace {

#define MB_REQUIRE(cond, code, ...) \
  do {                              \
    if (!(cond)) return fail(code, __VA_ARGS__); \
  } while (0)

mb_status check_ptr(const void* p, const char* name) {
  MB_REQUIRE(p != nullptr, MB_ERR_INVALID_ARG, "%s is NULL", name);
  MB_REQUIRE(aligned16(p), MB_ERR_INVALID_ARG, "%s is not 16-byte aligned", name);
  return MB_OK;
}
#define MB_CHECK_PTR(p)                              \
  do {                                               \
    const mb_status st_ = check_ptr((p), #p);        \
    if (st_ != MB_OK) return st_;                    \
  } while (0)

mb_status check_dtype(mb_dtype dt) {
  MB_REQUIRE(dt == MB_F32 || dt == MB_BF16, MB_ERR_INVALID_ARG, "unknown dtype %d", (int)dt);
  return MB_OK;
}

mb_status check_stride(int64_t stride, int H, int D, mb_dtype dt, const char* name) {
  MB_REQUIRE(stride >= (int64_t)H * D, MB_ERR_INVALID_ARG, "%s=%lld is smaller than H*D=%lld", name,
             (long long)stride, (long long)H * D);
  MB_REQUIRE((stride * (int64_t)elem_size(dt)) % 16 == 0, MB_ERR_INVALID_ARG,
             "%s=%lld elements is not a multiple of 16 bytes", name, (long long)stride);
  // kernels form offsets of up to 128 rows inside a sequence in 32 bits
  MB_REQUIRE(stride < ((int64_t)1 << 24), MB_ERR_UNSUPPORTED, "%s=%lld elements exceeds 2^24", name, (long long)stride);
  return MB_OK;
}
#define MB_CHECK_STRIDE(s, H, D)                               \
  do {                                                         \
    const mb_status st_ = check_stride((s), (H), (D), dt, #s); \
    if (st_ != MB_OK) return st_;                         \
  } while (0)

mb_status check_attn_dims(int B, int T, int max_seqlen, int H, int D, mb_dtype dt) {
  mb_status st = check_dtype(dt);
  if (st != MB_OK) return st;
  MB_REQUIRE(B >= 0 && T >= 0 && max_seqlen >= 0, MB_ERR_INVALID_ARG, "negative size (B=%d T=%d max_seqlen=%d)", B,
             T, max_seqlen);
  MB_REQUIRE(H > 0 && D > 0, MB_ERR_INVALID_ARG, "H=%d and D=%d must be positive", H, D);
  MB_REQUIRE(H <= 65535, MB_ERR_UNSUPPORTED, "H=%d exceeds 65535", H);
  MB_REQUIRE(D <= 128, MB_ERR_UNSUPPORTED, "head_dim %d > 128 has no kernel", D);
  MB_REQUIRE(D % 8 == 0 || dt == MB_F32, MB_ERR_UNSUPPORTED, "bf16 head_dim %d is not a multiple of 8", D);
  MB_REQUIRE(dt != MB_F32 || D % 4 == 0, MB_ERR_UNSUPPORTED, "fp32 head_dim %d is not a multiple of 4", D);
  MB_REQUIRE((int64_t)T * H < ((int64_t)1 << 31), MB_ERR_UNSUPPORTED, "T*H=%lld exceeds 2^31", (long long)T * H);
  MB_REQUIRE((int64_t)B * H < ((int64_t)1 << 30), MB_ERR_UNSUPPORTED, "B*H=%lld exceeds 2^30", (long long)B * H);
  MB_REQUIRE(max_seqlen < (1 << 22), MB_ERR_UNSUPPORTED, "max_seqlen=%d exceeds 2^22", max_seqlen);
  return MB_OK;
}

// The matrix-core kernels fold the scale into the exponent (exp2(acc*c - max*c)), which needs c > 0;
// any other finite scale goes through the generic kernels.
bool use_mfma(mb_dtype dt, int D, float scale) { return dt == MB_BF16 && D == 64 && scale > 0.f; }

}  // namespace
}  // namespace mb

using namespace mb;

extern "C" {

const char* mb_last_error(void) { return g_error; }

int mb_version(void) { return 100; }

mb_status mb_alibi_slopes(int H, float* slopes_host) {
  clear_error();
  MB_REQUIRE(H > 0, MB_ERR_INVALID_ARG, "H=%d must be positive", H);
  MB_REQUIRE(slopes_host != nullptr, MB_ERR_INVALID_ARG, "slopes_host is NULL");
  for (int h = 1; h <= H; ++h) slopes_host[h - 1] = (float)std::exp2(-8.0 * (double)h / (double)H);
  return MB_OK;
}

mb_status mb_unpad_index(const int32_t* mask, int B, int L, int32_t* seqlens, int32_t* cu_seqlens,
                         int32_t* indices, int32_t* meta_dev, void* stream) {
  clear_error();
  MB_REQUIRE(B >= 0 && L >= 0, MB_ERR_INVALID_ARG, "negative size (B=%d L=%d)", B, L);
  MB_REQUIRE((int64_t)B * L < ((int64_t)1 << 31), MB_ERR_UNSUPPORTED, "B*L=%lld does not fit int32",
             (long long)B * L);
  MB_CHECK_PTR(cu_seqlens);
  MB_CHECK_PTR(meta_dev);
  if (B > 0) {
    MB_CHECK_PTR(seqlens);
    if (L > 0) {
      MB_CHECK_PTR(mask);
      MB_CHECK_PTR(indices);
    }
  }
  return launch_unpad_index(mask, B, L, seqlens, cu_seqlens, indices, meta_dev, (hipStream_t)stream);
}

mb_status mb_read_meta(const int32_t* meta_dev, int32_t* meta_host, void* stream) {
  clear_error();
  MB_REQUIRE(meta_dev != nullptr && meta_host != nullptr, MB_ERR_INVALID_ARG, "meta pointer is NULL");
  hipError_t e = hipMemcpyAsync(meta_host, meta_dev, 2 * sizeof(int32_t), hipMemcpyDeviceToHost, (hipStream_t)stream);
  if (e == hipSuccess) e = hipStreamSynchronize((hipStream_t)stream);
  if (e != hipSuccess) return fail(MB_ERR_HIP, "mb_read_meta: %s", hipGetErrorString(e));
  return MB_OK;
}

static mb_status check_rows(int T_cap, int W, mb_dtype dt) {
  mb_status st = check_dtype(dt);
  if (st != MB_OK) return st;
  MB_REQUIRE(T_cap >= 0, MB_ERR_INVALID_ARG, "T_cap=%d is negative", T_cap);
  MB_REQUIRE(W > 0, MB_ERR_INVALID_ARG, "W=%d must be positive", W);
  MB_REQUIRE(((int64_t)W * (int64_t)elem_size(dt)) % 16 == 0, MB_ERR_INVALID_ARG,
             "row of %d elements is not a multiple of 16 bytes", W);
  MB_REQUIRE((int64_t)W * (int64_t)elem_size(dt) < ((int64_t)1 << 31), MB_ERR_UNSUPPORTED, "row too wide");
  return MB_OK;
}

mb_status mb_unpad(const void* padded, const int32_t* indices, int T_cap, const int32_t* meta_dev, int W,
                   mb_dtype dt, void* packed, void* stream) {
  clear_error();
  mb_status st = check_rows(T_cap, W, dt);
  if (st != MB_OK) return st;
  if (T_cap == 0) return MB_OK;
  MB_CHECK_PTR(padded);
  MB_CHECK_PTR(indices);
  MB_CHECK_PTR(packed);
  return launch_gather_rows(padded, indices, T_cap, meta_dev, (int)(W * elem_size(dt)), packed,
                            (hipStream_t)stream);
}

mb_status mb_pad(const void* packed, const int32_t* indices, int T_cap, const int32_t* meta_dev, int B, int L,
                 int W, mb_dtype dt, void* padded, void* stream) {
  clear_error();
  mb_status st = check_rows(T_cap, W, dt);
  if (st != MB_OK) return st;
  MB_REQUIRE(B >= 0 && L >= 0, MB_ERR_INVALID_ARG, "negative size (B=%d L=%d)", B, L);
  MB_REQUIRE((int64_t)B * L < ((int64_t)1 << 31), MB_ERR_UNSUPPORTED, "B*L=%lld does not fit int32",
             (long long)B * L);
  MB_REQUIRE((int64_t)T_cap <= (int64_t)B * L, MB_ERR_INVALID_ARG, "T_cap=%d exceeds B*L=%lld", T_cap,
             (long long)B * L);
  if ((int64_t)B * L == 0) return MB_OK;
  MB_CHECK_PTR(padded);
  if (T_cap > 0) {
    MB_CHECK_PTR(packed);
    MB_CHECK_PTR(indices);
  }
  return launch_scatter_rows(packed, indices, T_cap, meta_dev, B * L, (int)(W * elem_size(dt)), padded,
                             (hipStream_t)stream);
}

mb_status mb_zero_padding(const int32_t* indices, int T_cap, const int32_t* meta_dev, int B, int L, int W,
                          mb_dtype dt, void* padded, void* stream) {
  clear_error();
  mb_status st = check_rows(T_cap, W, dt);
  if (st != MB_OK) return st;
  MB_REQUIRE(B >= 0 && L >= 0, MB_ERR_INVALID_ARG, "negative size (B=%d L=%d)", B, L);
  MB_REQUIRE((int64_t)B * L < ((int64_t)1 << 31), MB_ERR_UNSUPPORTED, "B*L=%lld does not fit int32",
             (long long)B * L);
  MB_REQUIRE((int64_t)T_cap <= (int64_t)B * L, MB_ERR_INVALID_ARG, "T_cap=%d exceeds B*L=%lld", T_cap,
             (long long)B * L);
  if ((int64_t)B * L == 0) return MB_OK;
  MB_CHECK_PTR(padded);
  if (T_cap > 0) MB_CHECK_PTR(indices);
  return launch_zero_padding(indices, T_cap, meta_dev, B * L, (int)(W * elem_size(dt)), padded,
                             (hipStream_t)stream);
}

static mb_status check_ln(int T_cap, int W, mb_dtype dt) {
  mb_status st = check_rows(T_cap, W, dt);
  if (st != MB_OK) return st;
  MB_REQUIRE((int64_t)W * (int64_t)elem_size(dt) <= 4096, MB_ERR_UNSUPPORTED, "rows of %d elements exceed 4096 bytes",
             W);
  return MB_OK;
}

mb_status mb_add_layernorm_fwd(const void* x, const void* r, const void* gamma, const void* beta, int T_cap,
                               const int32_t* meta_dev, int W, float eps, mb_dtype dt, void* y, void* s, float* mean,
                               float* rstd, const int32_t* y_rows, void* stream) {
  clear_error();
  mb_status st = check_ln(T_cap, W, dt);
  if (st != MB_OK) return st;
  MB_REQUIRE(std::isfinite(eps) && eps >= 0.f, MB_ERR_INVALID_ARG, "eps must be finite and non-negative");
  if (T_cap == 0) return MB_OK;
  MB_CHECK_PTR(x);
  MB_CHECK_PTR(gamma);
  MB_CHECK_PTR(beta);
  MB_CHECK_PTR(y);
  MB_CHECK_PTR(mean);
  MB_CHECK_PTR(rstd);
  if (r != nullptr) {
    MB_REQUIRE(aligned16(r), MB_ERR_INVALID_ARG, "r is not 16-byte aligned");
    MB_CHECK_PTR(s);
  }
  MB_REQUIRE((reinterpret_cast<uintptr_t>(y_rows) & 3u) == 0, MB_ERR_INVALID_ARG, "y_rows is not 4-byte aligned");
  return launch_add_layernorm_fwd(dt, x, r, gamma, beta, T_cap, meta_dev, W, eps, y, s, mean, rstd, y_rows,
                                  (hipStream_t)stream);
}

size_t mb_add_layernorm_bwd_workspace_bytes(int W) {
  if (W <= 0) return 0;
  return (size_t)kLayerNormMaxParts * 2 * (size_t)W * sizeof(float);
}

mb_status mb_add_layernorm_bwd(const void* dy, const void* s, const void* gamma, const float* mean, const float* rstd,
                               int T_cap, const int32_t* meta_dev, int W, mb_dtype dt, void* ds, float* dgamma,
                               float* dbeta, void* workspace, size_t workspace_bytes, const int32_t* dy_rows,
                               void* stream) {
  clear_error();
  mb_status st = check_ln(T_cap, W, dt);
  if (st != MB_OK) return st;
  MB_CHECK_PTR(dgamma);
  MB_CHECK_PTR(dbeta);
  const size_t need = mb_add_layernorm_bwd_workspace_bytes(W);
  MB_REQUIRE(workspace != nullptr && workspace_bytes >= need, MB_ERR_WORKSPACE,
             "workspace of %zu bytes given, %zu needed", workspace ? workspace_bytes : (size_t)0, need);
  MB_REQUIRE(aligned16(workspace), MB_ERR_INVALID_ARG, "workspace is not 16-byte aligned");
  if (T_cap > 0) {
    MB_CHECK_PTR(dy);
    MB_CHECK_PTR(s);
    MB_CHECK_PTR(gamma);
    MB_CHECK_PTR(mean);
    MB_CHECK_PTR(rstd);
    MB_CHECK_PTR(ds);
  }
  MB_REQUIRE((reinterpret_cast<uintptr_t>(dy_rows) & 3u) == 0, MB_ERR_INVALID_ARG, "dy_rows is not 4-byte aligned");
  // with T_cap == 0 only the column-sum pass runs, over zero partial rows: dgamma and dbeta become zeros
  return launch_add_layernorm_bwd(dt, dy, s, gamma, mean, rstd, T_cap, meta_dev, W, ds, dgamma, dbeta,
                                  (float*)workspace, dy_rows, (hipStream_t)stream);
}

size_t mb_attn_plan_bytes(int B, int max_seqlen, int H) {
  if (B < 0 || max_seqlen < 0 || H <= 0 || H > 65535 || (int64_t)B * H >= ((int64_t)1 << 30) || max_seqlen >= (1 << 22)) return 0;
  return attn_plan_workspace_bytes(B, max_seqlen, H);
}

mb_status mb_attn_plan(const int32_t* cu_seqlens, const int32_t* key_lens, int B, int max_seqlen, int H, void* plan,
                       size_t plan_bytes, void* stream) {
  clear_error();
  MB_REQUIRE(B >= 0 && max_seqlen >= 0, MB_ERR_INVALID_ARG, "negative size (B=%d max_seqlen=%d)", B, max_seqlen);
  MB_REQUIRE(H > 0, MB_ERR_INVALID_ARG, "H=%d must be positive", H);
  MB_REQUIRE(H <= 65535 && B <= 65535, MB_ERR_UNSUPPORTED, "B=%d or H=%d exceeds 65535", B, H);
  MB_REQUIRE((int64_t)B * H < ((int64_t)1 << 30), MB_ERR_UNSUPPORTED, "B*H=%lld exceeds 2^30", (long long)B * H);
  MB_REQUIRE(max_seqlen < (1 << 22), MB_ERR_UNSUPPORTED, "max_seqlen=%d exceeds 2^22", max_seqlen);
  const size_t need = attn_plan_workspace_bytes(B, max_seqlen, H);
  MB_REQUIRE(plan != nullptr && plan_bytes >= need, MB_ERR_WORKSPACE, "plan of %zu bytes given, %zu needed",
             plan ? plan_bytes : (size_t)0, need);
  MB_REQUIRE(aligned16(plan), MB_ERR_INVALID_ARG, "plan is not 16-byte aligned");
  MB_CHECK_PTR(cu_seqlens);
  MB_REQUIRE((reinterpret_cast<uintptr_t>(key_lens) & 3u) == 0, MB_ERR_INVALID_ARG, "key_lens is not 4-byte aligned");
  int32_t* misuse = nullptr;
  const mb_status st = misuse_flag_address(&misuse);
  if (st != MB_OK) return st;
  const AttnShape s{B, 0, max_seqlen, H, 64, cu_seqlens, nullptr, 0.f, key_lens, nullptr, nullptr, misuse};
  return launch_attn_plan(s, static_cast<int32_t*>(plan), nullptr, (hipStream_t)stream);
}

mb_status mb_alibi_attn_fwd(const void* q, const void* k, const void* v, int64_t q_row_stride,
                            int64_t k_row_stride, int64_t v_row_stride, const int32_t* cu_seqlens, int B, int T,
                            int max_seqlen, int H, int D, const float* slopes, float softmax_scale, mb_dtype dt,
                            void* o, int64_t o_row_stride, float* lse, void* workspace, size_t workspace_bytes,
                            const int32_t* key_lens, const int32_t* token_rows, const void* plan, void* stream) {
  clear_error();
  mb_status st = check_attn_dims(B, T, max_seqlen, H, D, dt);
  if (st != MB_OK) return st;
  MB_CHECK_STRIDE(q_row_stride, H, D);
  MB_CHECK_STRIDE(k_row_stride, H, D);
  MB_CHECK_STRIDE(v_row_stride, H, D);
  MB_CHECK_STRIDE(o_row_stride, H, D);
  MB_REQUIRE(std::isfinite(softmax_scale), MB_ERR_INVALID_ARG, "softmax_scale is not finite");
  if (B == 0 || T == 0) return MB_OK;
  MB_REQUIRE(max_seqlen > 0, MB_ERR_INVALID_ARG, "max_seqlen=0 with T=%d tokens", T);
  MB_CHECK_PTR(q);
  MB_CHECK_PTR(k);
  MB_CHECK_PTR(v);
  MB_CHECK_PTR(cu_seqlens);
  MB_CHECK_PTR(slopes);
  MB_CHECK_PTR(o);
  MB_CHECK_PTR(lse);
  MB_REQUIRE(token_rows == nullptr || aligned16(token_rows), MB_ERR_INVALID_ARG,
             "token_rows is not 16-byte aligned");
  const bool mfma = use_mfma(dt, D, softmax_scale);
  MB_REQUIRE(mfma || max_seqlen <= kGenericMaxSeqlen, MB_ERR_UNSUPPORTED,
             "max_seqlen=%d exceeds %d for this dtype/head_dim", max_seqlen, kGenericMaxSeqlen);
  MB_REQUIRE(key_lens == nullptr || mfma, MB_ERR_UNSUPPORTED,
             "key_lens is served by the matrix-core kernels only (bf16, head_dim 64, softmax_scale > 0)");
  MB_REQUIRE((reinterpret_cast<uintptr_t>(key_lens) & 3u) == 0, MB_ERR_INVALID_ARG, "key_lens is not 4-byte aligned");
  MB_REQUIRE(plan == nullptr || aligned16(plan), MB_ERR_INVALID_ARG, "plan is not 16-byte aligned");
  const size_t need = (mfma && plan == nullptr) ? attn_fwd_mfma_workspace_bytes(B, max_seqlen, H) : 0;
  MB_REQUIRE(need == 0 || (workspace != nullptr && workspace_bytes >= need), MB_ERR_WORKSPACE,
             "workspace of %zu bytes given, %zu needed", workspace ? workspace_bytes : (size_t)0, need);
  MB_REQUIRE(need == 0 || aligned16(workspace), MB_ERR_INVALID_ARG, "workspace is not 16-byte aligned");
  int32_t* misuse = nullptr;   // (first thing that touches the GPU: everything above is testable without one)
  st = misuse_flag_address(&misuse);
  if (st != MB_OK) return st;
  const AttnShape s{B, T, max_seqlen, H, D, cu_seqlens, slopes, softmax_scale, key_lens, token_rows,
                    static_cast<const int32_t*>(plan), misuse};
  if (mfma)
    return launch_attn_fwd_mfma(s, q, k, v, q_row_stride, k_row_stride, v_row_stride, o, o_row_stride, lse,
                                workspace, (hipStream_t)stream);
  return launch_attn_fwd_generic(s, dt, q, k, v, q_row_stride, k_row_stride, v_row_stride, o, o_row_stride, lse,
                                 (hipStream_t)stream);
}

size_t mb_alibi_attn_fwd_workspace_bytes(int B, int T, int max_seqlen, int H, int D, mb_dtype dt) {
  if (B < 0 || T < 0 || max_seqlen < 0 || H <= 0 || D <= 0 || D > 128) return 0;
  if (dt != MB_BF16 || D != 64) return 0;                    // the generic kernels need none
  return attn_fwd_mfma_workspace_bytes(B, max_seqlen, H);   // the work plan (nothing for max_seqlen <= 128)
}

size_t mb_alibi_attn_bwd_workspace_bytes(int B, int T, int max_seqlen, int H, int D, mb_dtype dt) {
  if (B < 0 || T < 0 || max_seqlen < 0 || H <= 0 || D <= 0 || D > 128) return 0;
  if (dt != MB_F32 && dt != MB_BF16) return 0;
  if (dt != MB_BF16 || D != 64) return attn_bwd_delta_bytes(H, T);   // Delta [H, T] float
  return attn_bwd_mfma_workspace_bytes(B, T, max_seqlen, H);          // Delta, then the work plan
}

// Shared by mb_alibi_attn_bwd (caller's workspace) and mb_alibi_attn_bwd_static (the library's static array):
// everything but the workspace checks.
static mb_status attn_bwd_checked(const void* dout, const void* q, const void* k, const void* v, const void* o,
                                  const float* lse, int64_t do_row_stride, int64_t q_row_stride, int64_t k_row_stride,
                                  int64_t v_row_stride, int64_t o_row_stride, const int32_t* cu_seqlens, int B, int T,
                                  int max_seqlen, int H, int D, const float* slopes, float softmax_scale, mb_dtype dt,
                                  void* dq, void* dk, void* dv, int64_t dq_row_stride, int64_t dk_row_stride,
                                  int64_t dv_row_stride, void* workspace, const int32_t* key_lens,
                                  const int32_t* token_rows, const void* plan, void* stream) {
  const bool mfma = use_mfma(dt, D, softmax_scale);
  MB_REQUIRE(mfma || max_seqlen <= kGenericMaxSeqlen, MB_ERR_UNSUPPORTED,
             "max_seqlen=%d exceeds %d for this dtype/head_dim", max_seqlen, kGenericMaxSeqlen);
  MB_REQUIRE(key_lens == nullptr || mfma, MB_ERR_UNSUPPORTED,
             "key_lens is served by the matrix-core kernels only (bf16, head_dim 64, softmax_scale > 0)");
  MB_REQUIRE((reinterpret_cast<uintptr_t>(key_lens) & 3u) == 0, MB_ERR_INVALID_ARG, "key_lens is not 4-byte aligned");
  int32_t* misuse = nullptr;   // (first thing that touches the GPU: everything above is testable without one)
  const mb_status st = misuse_flag_address(&misuse);
  if (st != MB_OK) return st;
  const AttnShape s{B, T, max_seqlen, H, D, cu_seqlens, slopes, softmax_scale, key_lens, token_rows,
                    static_cast<const int32_t*>(plan), misuse};
  if (mfma)
    return launch_attn_bwd_mfma(s, dout, q, k, v, o, lse, do_row_stride, q_row_stride, k_row_stride, v_row_stride,
                                o_row_stride, dq, dk, dv, dq_row_stride, dk_row_stride, dv_row_stride,
                                (float*)workspace, (hipStream_t)stream);
  return launch_attn_bwd_generic(s, dt, dout, q, k, v, o, lse, do_row_stride, q_row_stride, k_row_stride,
                                 v_row_stride, o_row_stride, dq, dk, dv, dq_row_stride, dk_row_stride,
                                 dv_row_stride, (float*)workspace, (hipStream_t)stream);
}

// Host-side validation common to both backward entry points; *empty is set when there is nothing to do.
static mb_status attn_bwd_validate(const void* dout, const void* q, const void* k, const void* v, const void* o,
                                   const float* lse, int64_t do_row_stride, int64_t q_row_stride, int64_t k_row_stride,
                                   int64_t v_row_stride, int64_t o_row_stride, const int32_t* cu_seqlens, int B, int T,
                                   int max_seqlen, int H, int D, const float* slopes, float softmax_scale, mb_dtype dt,
                                   void* dq, void* dk, void* dv, int64_t dq_row_stride, int64_t dk_row_stride,
                                   int64_t dv_row_stride, const int32_t* token_rows, bool* empty) {
  *empty = false;
  mb_status st = check_attn_dims(B, T, max_seqlen, H, D, dt);
  if (st != MB_OK) return st;
  MB_CHECK_STRIDE(do_row_stride, H, D);
  MB_CHECK_STRIDE(q_row_stride, H, D);
  MB_CHECK_STRIDE(k_row_stride, H, D);
  MB_CHECK_STRIDE(v_row_stride, H, D);
  MB_CHECK_STRIDE(o_row_stride, H, D);
  MB_CHECK_STRIDE(dq_row_stride, H, D);
  MB_CHECK_STRIDE(dk_row_stride, H, D);
  MB_CHECK_STRIDE(dv_row_stride, H, D);
  MB_REQUIRE(std::isfinite(softmax_scale), MB_ERR_INVALID_ARG, "softmax_scale is not finite");
  if (B == 0 || T == 0) {
    *empty = true;
    return MB_OK;
  }
  MB_REQUIRE(max_seqlen > 0, MB_ERR_INVALID_ARG, "max_seqlen=0 with T=%d tokens", T);
  MB_CHECK_PTR(dout);
  MB_CHECK_PTR(q);
  MB_CHECK_PTR(k);
  MB_CHECK_PTR(v);
  MB_CHECK_PTR(o);
  MB_CHECK_PTR(lse);
  MB_CHECK_PTR(cu_seqlens);
  MB_CHECK_PTR(slopes);
  MB_CHECK_PTR(dq);
  MB_CHECK_PTR(dk);
  MB_CHECK_PTR(dv);
  MB_REQUIRE(token_rows == nullptr || aligned16(token_rows), MB_ERR_INVALID_ARG,
             "token_rows is not 16-byte aligned");
  return MB_OK;
}

mb_status mb_alibi_attn_bwd(const void* dout, const void* q, const void* k, const void* v, const void* o,
                            const float* lse, int64_t do_row_stride, int64_t q_row_stride, int64_t k_row_stride,
                            int64_t v_row_stride, int64_t o_row_stride, const int32_t* cu_seqlens, int B, int T,
                            int max_seqlen, int H, int D, const float* slopes, float softmax_scale, mb_dtype dt,
                            void* dq, void* dk, void* dv, int64_t dq_row_stride, int64_t dk_row_stride,
                            int64_t dv_row_stride, void* workspace, size_t workspace_bytes,
                            const int32_t* key_lens, const int32_t* token_rows, const void* plan, void* stream) {
  clear_error();
  bool empty = false;
  const mb_status st = attn_bwd_validate(dout, q, k, v, o, lse, do_row_stride, q_row_stride, k_row_stride, v_row_stride,
                                         o_row_stride, cu_seqlens, B, T, max_seqlen, H, D, slopes, softmax_scale, dt, dq,
                                         dk, dv, dq_row_stride, dk_row_stride, dv_row_stride, token_rows, &empty);
  if (st != MB_OK || empty) return st;
  MB_REQUIRE(plan == nullptr || aligned16(plan), MB_ERR_INVALID_ARG, "plan is not 16-byte aligned");
  // with a plan of the caller's only Delta needs room
  const size_t need = plan ? attn_bwd_delta_bytes(H, T) : mb_alibi_attn_bwd_workspace_bytes(B, T, max_seqlen, H, D, dt);
  MB_REQUIRE(workspace != nullptr && workspace_bytes >= need, MB_ERR_WORKSPACE,
             "workspace of %zu bytes given, %zu needed", workspace ? workspace_bytes : (size_t)0, need);
  MB_REQUIRE(aligned16(workspace), MB_ERR_INVALID_ARG, "workspace is not 16-byte aligned");
  return attn_bwd_checked(dout, q, k, v, o, lse, do_row_stride, q_row_stride, k_row_stride, v_row_stride, o_row_stride,
                          cu_seqlens, B, T, max_seqlen, H, D, slopes, softmax_scale, dt, dq, dk, dv, dq_row_stride,
                          dk_row_stride, dv_row_stride, workspace, key_lens, token_rows, plan, stream);
}

mb_status mb_alibi_attn_bwd_static(const void* dout, const void* q, const void* k, const void* v, const void* o,
                                   const float* lse, int64_t do_row_stride, int64_t q_row_stride,
                                   int64_t k_row_stride, int64_t v_row_stride, int64_t o_row_stride,
                                   const int32_t* cu_seqlens, int B, int T, int max_seqlen, int H, int D,
                                   const float* slopes, float softmax_scale, mb_dtype dt, void* dq, void* dk, void* dv,
                                   int64_t dq_row_stride, int64_t dk_row_stride, int64_t dv_row_stride,
                                   const int32_t* key_lens, const int32_t* token_rows, const void* plan, void* stream) {
  clear_error();
  bool empty = false;
  mb_status st = attn_bwd_validate(dout, q, k, v, o, lse, do_row_stride, q_row_stride, k_row_stride, v_row_stride,
                                   o_row_stride, cu_seqlens, B, T, max_seqlen, H, D, slopes, softmax_scale, dt, dq, dk,
                                   dv, dq_row_stride, dk_row_stride, dv_row_stride, token_rows, &empty);
  if (st != MB_OK || empty) return st;
  MB_REQUIRE(plan == nullptr || aligned16(plan), MB_ERR_INVALID_ARG, "plan is not 16-byte aligned");
  const size_t need = plan ? attn_bwd_delta_bytes(H, T) : mb_alibi_attn_bwd_workspace_bytes(B, T, max_seqlen, H, D, dt);
  MB_REQUIRE(need <= kStaticScratchBytes, MB_ERR_WORKSPACE,
             "these sizes need %zu bytes of scratch, the static array holds %zu: use mb_alibi_attn_bwd with a "
             "workspace of the caller's", need, kStaticScratchBytes);
  unsigned char* ws = nullptr;   // this GPU's copy of the array (never the array's name)
  st = static_scratch_address(&ws);
  if (st != MB_OK) return st;
  // Nothing in the array has to start at zero: every word a kernel of this call reads (Delta of the real
  // tokens, the sequence order) is written earlier in the same call.
  return attn_bwd_checked(dout, q, k, v, o, lse, do_row_stride, q_row_stride, k_row_stride, v_row_stride, o_row_stride,
                          cu_seqlens, B, T, max_seqlen, H, D, slopes, softmax_scale, dt, dq, dk, dv, dq_row_stride,
                          dk_row_stride, dv_row_stride, ws, key_lens, token_rows, plan, stream);
}

mb_status mb_device_status(void* stream) {
  clear_error();
  int32_t* flag = nullptr;
  mb_status st = misuse_flag_address(&flag);
  if (st != MB_OK) return st;
  int32_t seen = 0;
  hipError_t e = hipMemcpyAsync(&seen, flag, sizeof(seen), hipMemcpyDeviceToHost, (hipStream_t)stream);
  if (e == hipSuccess) e = hipStreamSynchronize((hipStream_t)stream);
  if (e != hipSuccess) return fail(MB_ERR_HIP, "mb_device_status: %s", hipGetErrorString(e));
  if (seen == 0) return MB_OK;
  const int32_t zero = 0;
  e = hipMemcpyAsync(flag, &zero, sizeof(zero), hipMemcpyHostToDevice, (hipStream_t)stream);
  if (e == hipSuccess) e = hipStreamSynchronize((hipStream_t)stream);
  if (e != hipSuccess) return fail(MB_ERR_HIP, "mb_device_status: %s", hipGetErrorString(e));
  return fail(MB_ERR_INVALID_ARG,
              "an attention call since the last check met a sequence longer than its max_seqlen; that sequence was "
              "skipped (forward: its log-sum-exp rows are NaN; backward: its gradient rows were left untouched)");
}

mb_status mb_geglu_fwd(const void* x, const void* w1v, const void* w2, int T_cap, const int32_t* meta_dev, int hidden,
                       int inter, mb_dtype dt, void* act, void* y, void* stream) {
  clear_error();
  MB_REQUIRE(dt == MB_F32 || dt == MB_BF16, MB_ERR_INVALID_ARG, "unknown dtype %d", (int)dt);
  MB_REQUIRE(T_cap >= 0, MB_ERR_INVALID_ARG, "T_cap must be >= 0 (got %d)", T_cap);
  MB_REQUIRE(hidden > 0 && inter > 0, MB_ERR_INVALID_ARG, "hidden and inter must be positive (got %d, %d)", hidden,
             inter);
  MB_REQUIRE(dt == MB_BF16, MB_ERR_UNSUPPORTED, "the feed-forward kernels are bf16 only");
  MB_REQUIRE(hidden % 256 == 0 && inter % 128 == 0, MB_ERR_UNSUPPORTED,
             "hidden must be a multiple of 256 and inter a multiple of 128 (got %d, %d)", hidden, inter);
  MB_REQUIRE((int64_t)T_cap * (int64_t)(inter > hidden ? inter : hidden) < ((int64_t)1 << 31) &&
                 2 * (int64_t)inter * (int64_t)hidden < ((int64_t)1 << 31),
             MB_ERR_UNSUPPORTED, "tensor of 2^31 elements or more (T_cap=%d hidden=%d inter=%d)", T_cap, hidden, inter);
  if (T_cap == 0) return MB_OK;
  MB_CHECK_PTR(x);
  MB_CHECK_PTR(w1v);
  MB_CHECK_PTR(w2);
  MB_CHECK_PTR(act);
  MB_CHECK_PTR(y);
  return launch_geglu_fwd(x, w1v, w2, T_cap, meta_dev, hidden, inter, act, y, (hipStream_t)stream);
}

mb_status mb_linear_fwd(const void* x, const void* wt, int T_cap, const int32_t* meta_dev, int n_in, int n_out,
                        mb_dtype dt, void* y, void* stream) {
  clear_error();
  MB_REQUIRE(dt == MB_F32 || dt == MB_BF16, MB_ERR_INVALID_ARG, "unknown dtype %d", (int)dt);
  MB_REQUIRE(T_cap >= 0, MB_ERR_INVALID_ARG, "T_cap must be >= 0 (got %d)", T_cap);
  MB_REQUIRE(n_in > 0 && n_out > 0, MB_ERR_INVALID_ARG, "n_in and n_out must be positive (got %d, %d)", n_in, n_out);
  MB_REQUIRE(dt == MB_BF16, MB_ERR_UNSUPPORTED, "the feed-forward kernels are bf16 only");
  MB_REQUIRE(n_in % 128 == 0 && (n_out % 256 == 0 || n_out % 192 == 0), MB_ERR_UNSUPPORTED,
             "n_in must be a multiple of 128 and n_out a multiple of 256 or 192 (got %d, %d)", n_in, n_out);
  MB_REQUIRE((int64_t)T_cap * (int64_t)(n_in > n_out ? n_in : n_out) < ((int64_t)1 << 31) &&
                 (int64_t)n_in * (int64_t)n_out < ((int64_t)1 << 31),
             MB_ERR_UNSUPPORTED, "tensor of 2^31 elements or more (T_cap=%d n_in=%d n_out=%d)", T_cap, n_in, n_out);
  if (T_cap == 0) return MB_OK;
  MB_CHECK_PTR(x);
  MB_CHECK_PTR(wt);
  MB_CHECK_PTR(y);
  return launch_linear_fwd(x, wt, T_cap, meta_dev, n_in, n_out, y, (hipStream_t)stream);
}

mb_status mb_gelu_gate(const void* h, const void* gate, int64_t row_stride, int T_cap, const int32_t* meta_dev,
                       int inter, mb_dtype dt, void* act, void* stream) {
  clear_error();
  MB_REQUIRE(dt == MB_F32 || dt == MB_BF16, MB_ERR_INVALID_ARG, "unknown dtype %d", (int)dt);
  MB_REQUIRE(T_cap >= 0, MB_ERR_INVALID_ARG, "T_cap must be >= 0 (got %d)", T_cap);
  MB_REQUIRE(inter > 0, MB_ERR_INVALID_ARG, "inter must be positive (got %d)", inter);
  MB_REQUIRE(dt == MB_BF16, MB_ERR_UNSUPPORTED, "the feed-forward kernels are bf16 only");
  MB_REQUIRE(inter % 8 == 0 && row_stride % 8 == 0 && row_stride >= inter, MB_ERR_INVALID_ARG,
             "inter and row_stride must be multiples of 8 with row_stride >= inter (got %d, %lld)", inter,
             (long long)row_stride);
  if (T_cap == 0) return MB_OK;
  MB_CHECK_PTR(h);
  MB_CHECK_PTR(gate);
  MB_CHECK_PTR(act);
  return launch_gelu_gate(h, gate, row_stride, T_cap, meta_dev, inter, act, (hipStream_t)stream);
}

mb_status mb_probe_ceiling(int kind, int iters, float* out, double* work_per_launch, void* stream) {
  clear_error();
  MB_REQUIRE(kind >= 0 && kind <= 2, MB_ERR_INVALID_ARG, "unknown probe kind %d", kind);
  MB_REQUIRE(iters > 0 && iters <= (1 << 24), MB_ERR_INVALID_ARG, "iters must be in [1, 2^24] (got %d)", iters);
  MB_REQUIRE(work_per_launch != nullptr, MB_ERR_INVALID_ARG, "work_per_launch is NULL");
  MB_CHECK_PTR(out);
  return launch_probe(kind, iters, out, work_per_launch, (hipStream_t)stream);
}

mb_status mb_probe_bwd_traffic(const void* qkv, const void* dout, const void* o, void* dqkv, const int32_t* cu_seqlens,
                               int B, int H, void* stream) {
  clear_error();
  MB_REQUIRE(B >= 0 && B <= 65535, MB_ERR_INVALID_ARG, "B=%d must be in [0, 65535]", B);
  MB_REQUIRE(H > 0 && H <= 65535, MB_ERR_INVALID_ARG, "H=%d must be in [1, 65535]", H);
  if (B == 0) return MB_OK;
  MB_CHECK_PTR(qkv);
  MB_CHECK_PTR(dout);
  MB_CHECK_PTR(o);
  MB_CHECK_PTR(dqkv);
  MB_CHECK_PTR(cu_seqlens);
  return launch_probe_bwd_traffic(qkv, dout, o, dqkv, cu_seqlens, B, H, (hipStream_t)stream);
}

static mb_status check_geglu_bwd(int T_cap, int hidden, int inter, mb_dtype dt) {
  MB_REQUIRE(dt == MB_F32 || dt == MB_BF16, MB_ERR_INVALID_ARG, "unknown dtype %d", (int)dt);
  MB_REQUIRE(T_cap >= 0, MB_ERR_INVALID_ARG, "T_cap must be >= 0 (got %d)", T_cap);
  MB_REQUIRE(hidden > 0 && inter > 0, MB_ERR_INVALID_ARG, "hidden and inter must be positive (got %d, %d)", hidden,
             inter);
  MB_REQUIRE(dt == MB_BF16, MB_ERR_UNSUPPORTED, "the feed-forward kernels are bf16 only");
  MB_REQUIRE(hidden % 256 == 0 && inter % 256 == 0, MB_ERR_UNSUPPORTED,
             "hidden and inter must be multiples of 256 (got %d, %d)", hidden, inter);
  MB_REQUIRE((int64_t)T_cap * 2 * (int64_t)inter < ((int64_t)1 << 31) &&
                 2 * (int64_t)inter * (int64_t)hidden < ((int64_t)1 << 31) &&
                 (int64_t)T_cap * (int64_t)hidden < ((int64_t)1 << 31),
             MB_ERR_UNSUPPORTED, "tensor of 2^31 elements or more (T_cap=%d hidden=%d inter=%d)", T_cap, hidden, inter);
  return MB_OK;
}

size_t mb_geglu_bwd_workspace_bytes(int T_cap, int hidden, int inter, mb_dtype dt) {
  if (check_geglu_bwd(T_cap, hidden, inter, dt) != MB_OK) return 0;
  return geglu_bwd_workspace_bytes(T_cap, hidden, inter);
}

mb_status mb_geglu_bwd(const void* dy, const void* x, const void* w1v, const void* w2, const void* act,
                       const void* hg, int T_cap, const int32_t* meta_dev, int hidden, int inter, mb_dtype dt, void* dx, float* dw1v, float* dw2,
                       void* workspace, size_t workspace_bytes, void* stream) {
  clear_error();
  mb_status st = check_geglu_bwd(T_cap, hidden, inter, dt);
  if (st != MB_OK) return st;
  MB_CHECK_PTR(w1v);
  MB_CHECK_PTR(w2);
  MB_CHECK_PTR(dw1v);
  MB_CHECK_PTR(dw2);
  const size_t need = geglu_bwd_workspace_bytes(T_cap, hidden, inter);
  MB_REQUIRE(workspace != nullptr && workspace_bytes >= need, MB_ERR_WORKSPACE,
             "workspace of %zu bytes given, %zu needed", workspace ? workspace_bytes : (size_t)0, need);
  MB_REQUIRE((reinterpret_cast<uintptr_t>(workspace) & 255u) == 0, MB_ERR_INVALID_ARG,
             "workspace is not 256-byte aligned");
  if (T_cap > 0) {
    MB_CHECK_PTR(dy);
    MB_CHECK_PTR(x);
    MB_CHECK_PTR(act);
    MB_CHECK_PTR(dx);
    if (hg != nullptr) MB_REQUIRE(aligned16(hg), MB_ERR_INVALID_ARG, "hg is not 16-byte aligned");
  }
  return launch_geglu_bwd(dy, x, w1v, w2, act, hg, T_cap, meta_dev, hidden, inter, dx, dw1v, dw2, workspace,
                          (hipStream_t)stream);
}

}  // extern "C"
