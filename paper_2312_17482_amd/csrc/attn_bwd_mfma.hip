// temporary: routes bf16 D=64 backward to the generic kernels until the matrix-core kernel lands
#include "common.h"
namespace mb {
mb_status launch_attn_bwd_mfma(const AttnShape& s, const void* dout, const void* q, const void* k, const void* v,
                               const void* o, const float* lse, int64_t dos, int64_t qs, int64_t ks, int64_t vs,
                               int64_t os, void* dq, void* dk, void* dv, int64_t dqs, int64_t dks, int64_t dvs,
                               float* delta_ws, hipStream_t stream) {
  return launch_attn_bwd_generic(s, MB_BF16, dout, q, k, v, o, lse, dos, qs, ks, vs, os, dq, dk, dv, dqs, dks, dvs,
                                 delta_ws, stream);
}
}  // namespace mb
