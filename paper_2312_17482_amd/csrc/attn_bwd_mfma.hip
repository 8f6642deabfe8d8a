// Backward ALiBi attention on the matrix cores: bf16, head_dim 64, variable-length packed sequences.
//
// Gradient of sum(O * dO) for the attention of the paper's Eq. 1 (the paper prints no backward; this is
// the standard derivative, with P recomputed from Q, K and the saved row log-sum-exp instead of being
// stored -- the same trade the "FlashAttention" paragraph describes for the forward):
//   Delta_i = dO_i . O_i,  P_ij = exp(S_ij - lse_i),  dV_j = sum_i P_ij dO_i,  dP_ij = dO_i . v_j,
//   dS_ij = P_ij (dP_ij - Delta_i),  dQ_i = scale sum_j dS_ij k_j,  dK_j = scale sum_i dS_ij q_i.
//
// Two kernels for any length, no atomics (results are bitwise reproducible):
//   dq    : one workgroup per (sequence, head, 128 queries); wave w owns 32 queries and streams all keys.
//           Transposed scores S^T = K Q^T (as in the forward) so that dS^T is directly the B operand
//           of dQ^T += K^T dS^T, and lse_i / Delta_i are per-lane scalars.  It runs first and also
//           computes Delta = rowsum(dO * O) of its queries (it holds their dO rows anyway) into [H, T] floats.
//   dkv   : one workgroup per (sequence, head, 128 keys); wave w owns 32 keys and streams all queries.
//           Scores in natural orientation S = Q K^T (queries along accumulator rows, keys along
//           lanes) so that P and dS, rounded to bf16, are directly the B operands of
//           dV^T += dO^T P and dK^T += Q^T dS.  Reads the Delta the first kernel left.
// Masking costs nothing: rows beyond the sequence end are staged as zeros and their lse as +inf
// (P = 0); zero K/V rows make the products with out-of-range keys vanish.
#include "attn_plan.h"
#include "common.h"
#include "mfma_util.h"

namespace mb {
namespace {

constexpr int kD = 64;
constexpr int kTile = 128;
constexpr int kPitch = 72;   // LDS row pitch in bf16 (144 B)

// ------------------------------------------------------------------------------------------------ any length
// Both kernels below stream their second operand in tiles of 64 rows through two LDS buffers: while
// one tile is consumed the next travels HBM -> registers -> the other buffer (one barrier per tile).
// Global memory is touched only as full 128-byte rows of one head; fragments and output rows pass
// through LDS.  Which workgroup does what is read from the work plan (attn_plan.h).
constexpr int kTileS = 64;                          // rows of a streamed tile
constexpr int kHalf = kTileS * kPitch;              // elements of one streamed operand tile (4608)
constexpr int kBuf = 2 * kHalf;                     // one buffer: two operand tiles (= 128 rows of pitch 72)

// ------------------------------------------------------------------------------------------------ dK, dV
// One workgroup per (sequence, head, 128 keys); wave w owns keys 32w.. and streams all queries.
//
// kMode (both kernels; see kRowsIdentity .. in common.h): for a sequence whose tokens sit in consecutive
// rows of the activation buffers, spanning fewer than 2^31 bytes, the rows of a streamed tile are fetched
// with buffer loads whose descriptor starts at the tile's first row and ends at the sequence's last one:
// the address is scalar arithmetic plus one constant per-lane offset, and rows past the end read as
// zeros without a compare.  Otherwise every row's address is formed per lane (row index looked up in
// token_rows when given).
constexpr int kRsrcFlags = 0x00020000;   // raw buffer, 32-bit data format (gfx9 family)

template <int kMode>
__global__ __launch_bounds__(256, 2) void attn_bwd_dkv_kernel(
    const uint16_t* __restrict__ dout, const uint16_t* __restrict__ q, const uint16_t* __restrict__ k,
    const uint16_t* __restrict__ v, const float* __restrict__ lse, const float* __restrict__ delta, int64_t dos,
    int64_t qs, int64_t ks, int64_t vs, const float* __restrict__ slopes,
    float scale, uint16_t* __restrict__ dk, uint16_t* __restrict__ dv, int64_t dks, int64_t dvs, int T,
    const int32_t* __restrict__ token_rows, const int32_t* __restrict__ plan, int64_t plan_cap) {
  const int32_t* rows = kMode == kRowsIdentity ? nullptr : token_rows;
  __shared__ __attribute__((aligned(16))) uint16_t smem[2 * kBuf];   // per buffer: Q tile, dO tile
  __shared__ __attribute__((aligned(16))) float sL[2][kTileS];       // -lse in base-2 units (-inf past the end)
  __shared__ __attribute__((aligned(16))) float sD[2][kTileS];       // -Delta

  int start, n, nk, ktile, h;   // nk <= n: the sequence's first nk tokens are its keys
  if (!plan_fetch(plan, plan_cap, &start, &n, &nk, &ktile, &h)) return;   // this XCD's list is shorter
  const int kv0 = ktile * kTile;   // < n by construction of the plan
  if (kv0 >= nk) {   // a tile of tokens that are no keys (only when the call limits the keys): zero gradient rows
    const u32x4 zero = {0u, 0u, 0u, 0u};
    for (int j = kv0 + (int)(threadIdx.x >> 3); j < min(kv0 + kTile, n); j += 32) {
      const int64_t gr = tok_row(rows, start + j);
      *reinterpret_cast<u32x4*>(dk + gr * dks + h * kD + (threadIdx.x & 7) * 8) = zero;
      *reinterpret_cast<u32x4*>(dv + gr * dvs + h * kD + (threadIdx.x & 7) * 8) = zero;
    }
    return;
  }
  // first buffer row of the sequence, and whether its tokens sit in consecutive rows
  const int row0 = kMode == kRowsMaybeContiguous ? __builtin_amdgcn_readfirstlane(rows[start]) : start;
  const bool contig =
      kMode == kRowsIdentity ||
      (kMode == kRowsMaybeContiguous && __builtin_amdgcn_readfirstlane(rows[start + n - 1]) - row0 == n - 1);

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform: keeps per-wave branches scalar
  const int c = lane & 31, g = lane >> 5;
  const int kw = kv0 + 32 * wave;
  const bool wave_active = kw < nk;           // tokens at and beyond nk are no keys: their dK, dV are zero
  const int kj = kw + c;                      // this lane's key
  const int kblk = (kv0 >> 5) + wave;         // index of this wave's block of 32 keys
  const int ntiles = (n + kTileS - 1) / kTileS;
  const int st_row = tid >> 3, st_col = (tid & 7) * 8;
  const float cs = scale * kLog2e;
  const float k1 = slopes[h] / scale;

  // ---- K, V rows of this workgroup's 128 keys (coalesced) -> LDS -> K^T, V^T fragments
  bf16x8 bk[4], bv[4];
  {
    u32x4 tk[4], tv[4];
#pragma unroll
    for (int it = 0; it < 4; ++it) {
      tk[it] = tv[it] = u32x4{0u, 0u, 0u, 0u};
      const int j = kv0 + 32 * it + st_row;
      if (j < nk) {
        const int64_t gr = tok_row(rows, start + j);
        tk[it] = *reinterpret_cast<const u32x4*>(k + gr * ks + h * kD + st_col);
        tv[it] = *reinterpret_cast<const u32x4*>(v + gr * vs + h * kD + st_col);
      }
    }
#pragma unroll
    for (int it = 0; it < 4; ++it) {
      *reinterpret_cast<u32x4*>(&smem[(32 * it + st_row) * kPitch + st_col]) = tk[it];
      *reinterpret_cast<u32x4*>(&smem[kBuf + (32 * it + st_row) * kPitch + st_col]) = tv[it];
    }
    __syncthreads();
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      bk[s] = lds_read8(&smem[(32 * wave + c) * kPitch + 16 * s + 8 * g]);
      bv[s] = lds_read8(&smem[kBuf + (32 * wave + c) * kPitch + 16 * s + 8 * g]);
    }
    __syncthreads();
  }

  // ---- streamed Q / dO tiles
  const uint16_t* qh = q + h * kD + st_col;
  const uint16_t* gh = dout + h * kD + st_col;
  u32x4 tq[2], tg[2];
  float tl = 0.f, td = 0.f;
  const uint32_t qoff = ((uint32_t)st_row * (uint32_t)qs + (uint32_t)(h * kD + st_col)) * 2u;
  const uint32_t goff = ((uint32_t)st_row * (uint32_t)dos + (uint32_t)(h * kD + st_col)) * 2u;
  auto issue_tile = [&](int i0) {
    if (contig) {
      const int left = n - i0;      // > 0: rows i0 .. n-1 exist
      const __amdgpu_buffer_rsrc_t qr = __builtin_amdgcn_make_buffer_rsrc(
          const_cast<uint16_t*>(q) + (int64_t)(row0 + i0) * qs, 0, left * (int)qs * 2, kRsrcFlags);
      const __amdgpu_buffer_rsrc_t gr = __builtin_amdgcn_make_buffer_rsrc(
          const_cast<uint16_t*>(dout) + (int64_t)(row0 + i0) * dos, 0, left * (int)dos * 2, kRsrcFlags);
#pragma unroll
      for (int it = 0; it < 2; ++it) {
        tq[it] = __builtin_amdgcn_raw_buffer_load_b128(qr, qoff + (uint32_t)it * 64u * (uint32_t)qs, 0, 0);
        tg[it] = __builtin_amdgcn_raw_buffer_load_b128(gr, goff + (uint32_t)it * 64u * (uint32_t)dos, 0, 0);
      }
    } else {
#pragma unroll
      for (int it = 0; it < 2; ++it) {
        tq[it] = tg[it] = u32x4{0u, 0u, 0u, 0u};
        const int i = i0 + 32 * it + st_row;
        if (i < n) {
          const int64_t gr = tok_row(rows, start + i);
          tq[it] = *reinterpret_cast<const u32x4*>(qh + gr * qs);
          tg[it] = *reinterpret_cast<const u32x4*>(gh + gr * dos);
        }
      }
    }
    if (tid < kTileS) {
      const bool ok = i0 + tid < n;
      tl = ok ? -lse[(int64_t)h * T + start + i0 + tid] * kLog2e : -INFINITY;
      td = ok ? -delta[(int64_t)h * T + start + i0 + tid] : 0.f;
    }
  };
  auto store_tile = [&](int buf) {
    uint16_t* bq_ = smem + buf * kBuf;
#pragma unroll
    for (int it = 0; it < 2; ++it) {
      *reinterpret_cast<u32x4*>(&bq_[(32 * it + st_row) * kPitch + st_col]) = tq[it];
      *reinterpret_cast<u32x4*>(&bq_[kHalf + (32 * it + st_row) * kPitch + st_col]) = tg[it];
    }
    if (tid < kTileS) { sL[buf][tid] = tl; sD[buf][tid] = td; }
  };

  f32x16 dkacc[2], dvacc[2];   // dK^T, dV^T: d along accumulator rows (two blocks of 32), keys along lanes
#pragma unroll
  for (int i = 0; i < 16; ++i) { dkacc[0][i] = dkacc[1][i] = dvacc[0][i] = dvacc[1][i] = 0.f; }
  const int tr_i = lane & 15, tr_q = lane >> 4;
  const int tr_row = (tr_i >> 2) + 4 * (tr_q >> 1);
  const int tr_col = 16 * (tr_q & 1) + 4 * (tr_i & 3);
  float fj = (float)(kj - 4 * g);   // i - j = ci - fj with ci = i0 + 32ib + 8*(v/4) + v%4
  asm volatile("" : "+v"(fj));

  // The two blocks of 32 queries of a staged tile (rows 32ib..) against this wave's keys.  The S accumulator
  // is pre-loaded with bias/scale and the dP accumulator with -Delta_i, so that after the products
  // P = exp2(acc_S * c - lse2_i) and dS = P * acc_dP.  Rows past the sequence end are staged as zeros
  // with lse = +inf, which makes their P and dS exact zeros: no branch around the accumulating code.
  // Only the bias pre-load has variants (diagonal block or not); everything after it is one straight
  // run of instructions for both blocks, so that the exponentials of one block can be issued between
  // the matrix instructions of the other.
  auto qtile = [&](const uint16_t* sQ, const uint16_t* sG, const float* pl, const float* pd, int i0) {
    f32x16 sacc[2], pacc[2];
#pragma unroll
    for (int ib = 0; ib < 2; ++ib) {
      const float d0 = (float)(i0 + 32 * ib) - fj;
      const int qb = (i0 >> 5) + ib;
      if (qb == kblk) {   // block with the diagonal
#pragma unroll
        for (int i = 0; i < 16; ++i) sacc[ib][i] = -k1 * fabsf(d0 + (float)(8 * (i >> 2) + (i & 3)));
      } else {            // |i-j| = +-(ci - fj) on the whole block
        const float sk = qb < kblk ? k1 : -k1;
        const float a = sk * d0;
#pragma unroll
        for (int i = 0; i < 16; ++i) sacc[ib][i] = fmaf((float)(8 * (i >> 2) + (i & 3)), sk, a);
      }
    }
#pragma unroll
    for (int ib = 0; ib < 2; ++ib) {
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const float4 d4 = *reinterpret_cast<const float4*>(&pd[32 * ib + 8 * r + 4 * g]);
        pacc[ib][4 * r + 0] = d4.x; pacc[ib][4 * r + 1] = d4.y; pacc[ib][4 * r + 2] = d4.z; pacc[ib][4 * r + 3] = d4.w;
      }
      const uint16_t* qrow = &sQ[(32 * ib + c) * kPitch + 8 * g];
      const uint16_t* grow = &sG[(32 * ib + c) * kPitch + 8 * g];
#pragma unroll
      for (int s = 0; s < 4; ++s) {
        sacc[ib] = mfma32(lds_read8(qrow + 16 * s), bk[s], sacc[ib]);
        pacc[ib] = mfma32(lds_read8(grow + 16 * s), bv[s], pacc[ib]);
      }
    }
#pragma unroll
    for (int ib = 0; ib < 2; ++ib) {
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const float4 l4 = *reinterpret_cast<const float4*>(&pl[32 * ib + 8 * r + 4 * g]);
        const float nl[4] = {l4.x, l4.y, l4.z, l4.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const float p = fast_exp2(fmaf(sacc[ib][4 * r + e], cs, nl[e]));
          sacc[ib][4 * r + e] = p;
          pacc[ib][4 * r + e] = p * pacc[ib][4 * r + e];
        }
      }
#pragma unroll
      for (int kk = 0; kk < 2; ++kk) {
        const bf16x8 bp = pack8(sacc[ib][8 * kk + 0], sacc[ib][8 * kk + 1], sacc[ib][8 * kk + 2], sacc[ib][8 * kk + 3],
                                sacc[ib][8 * kk + 4], sacc[ib][8 * kk + 5], sacc[ib][8 * kk + 6], sacc[ib][8 * kk + 7]);
        const bf16x8 bs = pack8(pacc[ib][8 * kk + 0], pacc[ib][8 * kk + 1], pacc[ib][8 * kk + 2], pacc[ib][8 * kk + 3],
                                pacc[ib][8 * kk + 4], pacc[ib][8 * kk + 5], pacc[ib][8 * kk + 6], pacc[ib][8 * kk + 7]);
        const int roff = (32 * ib + 16 * kk + tr_row) * kPitch + tr_col;
#pragma unroll
        for (int db = 0; db < 2; ++db) {
          const bf16x8 ag = join_tr(lds_read_tr4(&sG[roff + 32 * db]), lds_read_tr4(&sG[roff + 32 * db + 8 * kPitch]));
          dvacc[db] = mfma32(ag, bp, dvacc[db]);
          const bf16x8 aq = join_tr(lds_read_tr4(&sQ[roff + 32 * db]), lds_read_tr4(&sQ[roff + 32 * db + 8 * kPitch]));
          dkacc[db] = mfma32(aq, bs, dkacc[db]);
        }
      }
    }
  };

  issue_tile(0);
  store_tile(0);
#pragma unroll 1
  for (int it = 0; it < ntiles; ++it) {
    const int i0 = it * kTileS;
    __syncthreads();   // tile `it` is complete in its buffer; the other buffer is no longer being read
    if (it + 1 < ntiles) issue_tile(i0 + kTileS);
    if (wave_active) {
      const uint16_t* sQ = smem + (it & 1) * kBuf;
      const uint16_t* sG = sQ + kHalf;
      const float* pl = sL[it & 1];
      const float* pd = sD[it & 1];
      qtile(sQ, sG, pl, pd, i0);
    }
    if (it + 1 < ntiles) store_tile((it + 1) & 1);
  }
  __syncthreads();   // the buffers are free: they now carry the output rows
  const int orow = lane >> 3, ocol = (lane & 7) * 8;
  if (!wave_active) {   // tokens that are no keys (only when the call limits the keys): zero gradient rows
    const u32x4 zero = {0u, 0u, 0u, 0u};
#pragma unroll
    for (int it = 0; it < 4; ++it) {
      const int row = 8 * it + orow;
      if (kw + row < n) {
        const int64_t gr = tok_row(rows, start + kw + row);
        *reinterpret_cast<u32x4*>(dk + gr * dks + h * kD + ocol) = zero;
        *reinterpret_cast<u32x4*>(dv + gr * dvs + h * kD + ocol) = zero;
      }
    }
    return;
  }

  uint16_t* slab = &smem[(32 * wave) * kPitch];   // 32 rows private to this wave
  auto store_rows = [&](const f32x16(&acc)[2], float mul, uint16_t* __restrict__ out, int64_t stride) {
#pragma unroll
    for (int db = 0; db < 2; ++db) {
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        u32x2 w;
        w[0] = pack_bf16(acc[db][4 * r + 0] * mul, acc[db][4 * r + 1] * mul);
        w[1] = pack_bf16(acc[db][4 * r + 2] * mul, acc[db][4 * r + 3] * mul);
        *reinterpret_cast<u32x2*>(&slab[c * kPitch + 32 * db + 8 * r + 4 * g]) = w;
      }
    }
#pragma unroll
    for (int it = 0; it < 4; ++it) {
      const int row = 8 * it + orow;
      u32x4 w = *reinterpret_cast<const u32x4*>(&slab[row * kPitch + ocol]);
      if (kw + row >= nk) w = u32x4{0u, 0u, 0u, 0u};   // a token that is no key
      if (kw + row < n) *reinterpret_cast<u32x4*>(out + tok_row(rows, start + kw + row) * stride + h * kD + ocol) = w;
    }
  };
  store_rows(dkacc, scale, dk, dks);
  store_rows(dvacc, 1.f, dv, dvs);
}

// ------------------------------------------------------------------------------------------------ dQ
// One workgroup per (sequence, head, 128 queries); wave w owns queries 32w.. and streams all keys.
// (at most 168 registers, so that three workgroups share a compute unit)
template <int kMode>
__global__ __launch_bounds__(256, 3) void attn_bwd_dq_kernel(
    const uint16_t* __restrict__ dout, const uint16_t* __restrict__ q, const uint16_t* __restrict__ k,
    const uint16_t* __restrict__ v, const uint16_t* __restrict__ o, const float* __restrict__ lse,
    float* __restrict__ delta, int64_t dos, int64_t qs, int64_t ks, int64_t vs, int64_t os,
    const float* __restrict__ slopes, float scale, uint16_t* __restrict__ dq, int64_t dqs, int T,
    const int32_t* __restrict__ token_rows, const int32_t* __restrict__ plan, int64_t plan_cap) {
  const int32_t* rows = kMode == kRowsIdentity ? nullptr : token_rows;
  __shared__ __attribute__((aligned(16))) uint16_t smem[2 * kBuf];   // per buffer: K tile, V tile
  __shared__ __attribute__((aligned(16))) float sDelta[kTile];       // -Delta of this workgroup's queries

  int start, n, nk, qtile, h;   // nk <= n: the sequence's first nk tokens are its keys
  if (!plan_fetch(plan, plan_cap, &start, &n, &nk, &qtile, &h)) return;
  const int q0 = qtile * kTile;
  const int row0 = kMode == kRowsMaybeContiguous ? __builtin_amdgcn_readfirstlane(rows[start]) : start;
  const bool contig =
      kMode == kRowsIdentity ||
      (kMode == kRowsMaybeContiguous && __builtin_amdgcn_readfirstlane(rows[start + n - 1]) - row0 == n - 1);

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int c = lane & 31, g = lane >> 5;
  const int qw = q0 + 32 * wave;
  const bool wave_active = qw < n;
  const int qi = qw + c;
  const bool q_ok = wave_active && qi < n;
  const int qblk = (q0 >> 5) + wave;
  const int ntiles = (nk + kTileS - 1) / kTileS;
  const int st_row = tid >> 3, st_col = (tid & 7) * 8;
  const float cs = scale * kLog2e;
  const float k1 = slopes[h] / scale;

  // ---- Q, dO rows of this workgroup's 128 queries (coalesced) -> LDS -> Q^T, dO^T fragments; the O rows
  //      only serve Delta_i = dO_i . O_i (8 lanes per row, 8 elements each), kept in LDS for this kernel and
  //      written to [H, T] for the dK/dV kernel
  bf16x8 bq[4], bg[4];
  {
    u32x4 tq[4], tg[4], to[4];
#pragma unroll
    for (int it = 0; it < 4; ++it) {
      tq[it] = tg[it] = to[it] = u32x4{0u, 0u, 0u, 0u};
      const int i = q0 + 32 * it + st_row;
      if (i < n) {
        const int64_t gr = tok_row(rows, start + i);
        tq[it] = *reinterpret_cast<const u32x4*>(q + gr * qs + h * kD + st_col);
        tg[it] = *reinterpret_cast<const u32x4*>(dout + gr * dos + h * kD + st_col);
        to[it] = *reinterpret_cast<const u32x4*>(o + gr * os + h * kD + st_col);
      }
    }
#pragma unroll
    for (int it = 0; it < 4; ++it) {
      *reinterpret_cast<u32x4*>(&smem[(32 * it + st_row) * kPitch + st_col]) = tq[it];
      *reinterpret_cast<u32x4*>(&smem[kBuf + (32 * it + st_row) * kPitch + st_col]) = tg[it];
      float acc = 0.f;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        acc = fmaf(__uint_as_float(tg[it][e] << 16), __uint_as_float(to[it][e] << 16), acc);
        acc = fmaf(__uint_as_float(tg[it][e] & 0xffff0000u), __uint_as_float(to[it][e] & 0xffff0000u), acc);
      }
      acc += __shfl_xor(acc, 1, 64);
      acc += __shfl_xor(acc, 2, 64);
      acc += __shfl_xor(acc, 4, 64);
      const int i = q0 + 32 * it + st_row;
      if ((tid & 7) == 0) {
        sDelta[32 * it + st_row] = -acc;
        if (i < n) delta[(int64_t)h * T + start + i] = acc;
      }
    }
    __syncthreads();
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      bq[s] = lds_read8(&smem[(32 * wave + c) * kPitch + 16 * s + 8 * g]);
      bg[s] = lds_read8(&smem[kBuf + (32 * wave + c) * kPitch + 16 * s + 8 * g]);
    }
    __syncthreads();
  }
  const float nlse2 = q_ok ? -lse[(int64_t)h * T + start + qi] * kLog2e : -INFINITY;   // -inf: P = 0
  const float ndlt = q_ok ? sDelta[32 * wave + c] : 0.f;

  // ---- streamed K / V tiles
  const uint16_t* kh = k + h * kD + st_col;
  const uint16_t* vh = v + h * kD + st_col;
  u32x4 tk[2], tv[2];
  const uint32_t koff = ((uint32_t)st_row * (uint32_t)ks + (uint32_t)(h * kD + st_col)) * 2u;
  const uint32_t voff = ((uint32_t)st_row * (uint32_t)vs + (uint32_t)(h * kD + st_col)) * 2u;
  auto issue_tile = [&](int j0) {
    if (contig) {
      const int left = nk - j0;     // > 0: key rows j0 .. nk-1 exist
      const __amdgpu_buffer_rsrc_t kr = __builtin_amdgcn_make_buffer_rsrc(
          const_cast<uint16_t*>(k) + (int64_t)(row0 + j0) * ks, 0, left * (int)ks * 2, kRsrcFlags);
      const __amdgpu_buffer_rsrc_t vr = __builtin_amdgcn_make_buffer_rsrc(
          const_cast<uint16_t*>(v) + (int64_t)(row0 + j0) * vs, 0, left * (int)vs * 2, kRsrcFlags);
#pragma unroll
      for (int it = 0; it < 2; ++it) {
        tk[it] = __builtin_amdgcn_raw_buffer_load_b128(kr, koff + (uint32_t)it * 64u * (uint32_t)ks, 0, 0);
        tv[it] = __builtin_amdgcn_raw_buffer_load_b128(vr, voff + (uint32_t)it * 64u * (uint32_t)vs, 0, 0);
      }
      return;
    }
#pragma unroll
    for (int it = 0; it < 2; ++it) {
      tk[it] = tv[it] = u32x4{0u, 0u, 0u, 0u};
      const int j = j0 + 32 * it + st_row;
      if (j < nk) {
        const int64_t gr = tok_row(rows, start + j);
        tk[it] = *reinterpret_cast<const u32x4*>(kh + gr * ks);
        tv[it] = *reinterpret_cast<const u32x4*>(vh + gr * vs);
      }
    }
  };
  auto store_tile = [&](int buf) {
    uint16_t* bk_ = smem + buf * kBuf;
#pragma unroll
    for (int it = 0; it < 2; ++it) {
      *reinterpret_cast<u32x4*>(&bk_[(32 * it + st_row) * kPitch + st_col]) = tk[it];
      *reinterpret_cast<u32x4*>(&bk_[kHalf + (32 * it + st_row) * kPitch + st_col]) = tv[it];
    }
  };

  f32x16 dqacc[2];   // dQ^T: d along accumulator rows, queries along lanes
#pragma unroll
  for (int i = 0; i < 16; ++i) { dqacc[0][i] = 0.f; dqacc[1][i] = 0.f; }
  const int tr_i = lane & 15, tr_q = lane >> 4;
  const int tr_row = (tr_i >> 2) + 4 * (tr_q >> 1);
  const int tr_col = 16 * (tr_q & 1) + 4 * (tr_i & 3);

  // One block of 32 keys (rows 32jb.. of the staged tile) against this wave's queries, transposed
  // orientation: S^T = K Q^T (+ bias/scale pre-loaded), dP^T = V dO^T (- Delta pre-loaded).  The code
  // that accumulates dQ exists once with no branch around it; a ragged last tile only zeroes the dS of
  // the keys that do not exist.
  auto kblock = [&](const uint16_t* sK, const uint16_t* sV, int j0, int jb, int rem) {
    float fi = (float)(qi - j0 - 4 * g);   // i - j = fi - cj with cj = 32jb + 8*(v/4) + v%4
    asm volatile("" : "+v"(fi));
    f32x16 sacc, pacc;
    const int kb = (j0 >> 5) + jb;
    if (kb == qblk) {
#pragma unroll
      for (int i = 0; i < 16; ++i) sacc[i] = -k1 * fabsf(fi - (float)(jb * 32 + 8 * (i >> 2) + (i & 3)));
    } else {
      const float sk = kb < qblk ? k1 : -k1;
      const float a = -sk * fi;
#pragma unroll
      for (int i = 0; i < 16; ++i) sacc[i] = fmaf((float)(jb * 32 + 8 * (i >> 2) + (i & 3)), sk, a);
    }
#pragma unroll
    for (int i = 0; i < 16; ++i) pacc[i] = ndlt;
    const uint16_t* krow = &sK[(32 * jb + c) * kPitch + 8 * g];
    const uint16_t* vrow = &sV[(32 * jb + c) * kPitch + 8 * g];
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      sacc = mfma32(lds_read8(krow + 16 * s), bq[s], sacc);
      pacc = mfma32(lds_read8(vrow + 16 * s), bg[s], pacc);
    }
#pragma unroll
    for (int i = 0; i < 16; ++i) pacc[i] = fast_exp2(fmaf(sacc[i], cs, nlse2)) * pacc[i];
    if (rem < kTileS) {
      // a key past the sequence end has a zero K row, but its p may overflow (its score was never part
      // of lse): force the product with that zero row to be 0, not inf * 0
      const int lim = rem - 4 * g;
#pragma unroll
      for (int i = 0; i < 16; ++i) pacc[i] = (32 * jb + 8 * (i >> 2) + (i & 3)) >= lim ? 0.f : pacc[i];
    }
#pragma unroll
    for (int kk = 0; kk < 2; ++kk) {
      const bf16x8 bs = pack8(pacc[8 * kk + 0], pacc[8 * kk + 1], pacc[8 * kk + 2], pacc[8 * kk + 3],
                              pacc[8 * kk + 4], pacc[8 * kk + 5], pacc[8 * kk + 6], pacc[8 * kk + 7]);
      const int roff = (32 * jb + 16 * kk + tr_row) * kPitch + tr_col;
#pragma unroll
      for (int db = 0; db < 2; ++db) {
        const bf16x8 ak = join_tr(lds_read_tr4(&sK[roff + 32 * db]), lds_read_tr4(&sK[roff + 32 * db + 8 * kPitch]));
        dqacc[db] = mfma32(ak, bs, dqacc[db]);
      }
    }
  };

  issue_tile(0);
  store_tile(0);
#pragma unroll 1
  for (int jt = 0; jt < ntiles; ++jt) {
    const int j0 = jt * kTileS;
    __syncthreads();
    if (jt + 1 < ntiles) issue_tile(j0 + kTileS);
    if (wave_active) {
      const uint16_t* sK = smem + (jt & 1) * kBuf;
      const uint16_t* sV = sK + kHalf;
      const int rem = nk - j0;
      kblock(sK, sV, j0, 0, rem);
      kblock(sK, sV, j0, 1, rem);
    }
    if (jt + 1 < ntiles) store_tile((jt + 1) & 1);
  }
  __syncthreads();
  if (!wave_active) return;

  uint16_t* slab = &smem[(32 * wave) * kPitch];
#pragma unroll
  for (int db = 0; db < 2; ++db) {
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      u32x2 w;
      w[0] = pack_bf16(dqacc[db][4 * r + 0] * scale, dqacc[db][4 * r + 1] * scale);
      w[1] = pack_bf16(dqacc[db][4 * r + 2] * scale, dqacc[db][4 * r + 3] * scale);
      *reinterpret_cast<u32x2*>(&slab[c * kPitch + 32 * db + 8 * r + 4 * g]) = w;
    }
  }
  const int orow = lane >> 3, ocol = (lane & 7) * 8;
#pragma unroll
  for (int it = 0; it < 4; ++it) {
    const int row = 8 * it + orow;
    const u32x4 w = *reinterpret_cast<const u32x4*>(&slab[row * kPitch + ocol]);
    if (qw + row < n) *reinterpret_cast<u32x4*>(dq + tok_row(rows, start + qw + row) * dqs + h * kD + ocol) = w;
  }
}

// ------------------------------------------------------------------------------------------------ fused, n <= 128
// Whole backward of one (sequence, head) with at most 128 tokens in one workgroup: every input is read
// from HBM once and every output written once, always as full 128-byte rows shared by 8 lanes; the
// fragment layouts of the matrix cores are produced by passing through LDS.
//   phase 0  K, V, Q, dO rows -> LDS (K and V into the dS buffer, which is idle until phase 1), Delta = rowsum(dO * O)
//            and -lse -> LDS; one barrier; each wave takes the K^T, V^T fragments of its own 32 keys into registers.
//   phase 1  wave w owns keys 32w..: for every block of 32 queries, S = Q K^T, dP = dO V^T, P, dS in
//            registers; dV^T += dO^T P, dK^T += Q^T dS; dS (bf16) is also written to LDS as [key][query].
//   phase 2  dK, dV leave through the (now free) dO tile; the K registers go back to LDS over the Q
//            tile; wave w then owns queries 32w.. and accumulates dQ^T += K^T dS^T, both operands read
//            with transposing LDS reads.
// The kernel is bound by memory latency, not arithmetic: with 73 KB of LDS and about 170 registers only two
// workgroups fit a compute unit, and a workgroup spends half its life waiting for its first rows (measured with
// timestamps: 6.2 of 12.9 us at n = 128), while a traffic-only kernel with the same access pattern runs 1.4x as
// fast in the same place.  With kUnits = 2 a workgroup handles two consecutive (sequence, head) units and requests
// the second unit's rows in phase 2 of the first, when the dK / dV accumulators and the K fragments
// have left their registers: the rows travel while dQ is computed and stored.  (Requesting them earlier, during
// phase 1, needs more registers than there are: the compiler then spills, and a spill reload waits for every
// load in flight, which undoes the overlap.  Measured inside the benchmark step: 76 -> 70 us.)  With packed tokens
// the 40 loads of a thread are not issued in one burst, during which the wave can do nothing else (timestamps: 2.5 us
// for the burst), but five at a time between the four steps of the dQ loop (another 1.1 us off).
constexpr int kDsPitch = 136;   // LDS row pitch of dS in bf16 (272 B)

// kMode (see kRowsIdentity .. in common.h): a unit whose tokens sit in consecutive buffer rows moves all its rows with
// buffer instructions: one descriptor per tensor and unit that starts at the unit's first row and ends with its last
// (built with scalar arithmetic) and one per-lane byte offset per tensor that is the same for every unit, to which
// the step from one group of rows to the next is added (the whole offset must be the vector operand: the scalar
// offset of a buffer instruction takes no part in its range check).  Rows past the unit's end then read as zeros and
// are dropped on a store without a compare, and forming an address is one 32-bit add.  (With per-lane 64-bit
// addresses every row access costs a 64-bit multiply, three quarter-rate vector instructions: a fifth of all vector
// instructions of this kernel were address arithmetic.)
// kUnits: (sequence, head) units per workgroup, 1 or 2.
template <int kMode, int kUnits>
__global__ __launch_bounds__(256, 2) void attn_bwd_fused128_kernel(
    const uint16_t* __restrict__ dout, const uint16_t* __restrict__ q, const uint16_t* __restrict__ k,
    const uint16_t* __restrict__ v, const uint16_t* __restrict__ o, const float* __restrict__ lse, int64_t dos,
    int64_t qs, int64_t ks, int64_t vs, int64_t os, const int32_t* __restrict__ cu,
    const float* __restrict__ slopes, float scale, uint16_t* __restrict__ dq, uint16_t* __restrict__ dk,
    uint16_t* __restrict__ dv, int64_t dqs, int64_t dks, int64_t dvs, int T, const int32_t* __restrict__ rows,
    int32_t* __restrict__ misuse, const int32_t* __restrict__ key_lens, int H, int n_units) {
  constexpr bool kRows = kMode != kRowsIdentity;   // token t may sit at another row than t
  if (kMode == kRowsIdentity) rows = nullptr;
  __shared__ __attribute__((aligned(16))) uint16_t sA[kTile * kPitch];      // Q, then K
  __shared__ __attribute__((aligned(16))) uint16_t sB[kTile * kPitch];      // dO, then output rows
  __shared__ __attribute__((aligned(16))) uint16_t sDs[kTile * kDsPitch];   // K and V rows on their way in, then dS as [key][query]
  __shared__ __attribute__((aligned(16))) float sLse[kTile];                // -lse, base-2 units
  __shared__ __attribute__((aligned(16))) float sDelta[kTile];              // -Delta

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int c = lane & 31, g = lane >> 5;
  const int kw = 32 * wave;
  const int kj = kw + c;
  const float cs = scale * kLog2e;
  const int st_row = tid >> 3, st_col = (tid & 7) * 8;
  const int tr_i = lane & 15, tr_q = lane >> 4;
  const int tr_row = (tr_i >> 2) + 4 * (tr_q >> 1);
  const int tr_col = 16 * (tr_q & 1) + 4 * (tr_i & 3);
  const int orow = lane >> 3, ocol = (lane & 7) * 8;

  // A unit: head h of the sequence that starts at packed token `start` and has n tokens, the first nk of which
  // are keys (n = 0: nothing to do).  Token r of the sequence sits at buffer row row_of(r).  With token_rows, rows listed in ascending
  // order whose first and last differ by n - 1 are consecutive (the usual case: padding is a suffix of each
  // batch row); then no per-token index load is needed.
  struct Unit {
    int h, start, n, nk;
    int64_t row0;
    bool contig;
  };
  auto find_unit = [&](int u) -> Unit {
    Unit U{0, 0, 0, 0, 0, kMode != kRowsPerLane};
    if (u >= n_units) return U;
    const int b = u / H;
    U.h = u - b * H;
    U.start = __builtin_amdgcn_readfirstlane(cu[b]);
    U.n = __builtin_amdgcn_readfirstlane(cu[b + 1]) - U.start;
    if (U.n > kTile) {   // the caller promised max_seqlen <= 128: skipped, never truncated
      raise_misuse(misuse);
      U.n = 0;
    }
    U.nk = key_lens ? min(__builtin_amdgcn_readfirstlane(key_lens[b]), U.n) : U.n;
    if (U.n <= 0 || U.nk <= 0) {   // empty, or no keys: skipped
      U.n = 0;
      return U;
    }
    U.row0 = U.start;
    if (kMode == kRowsMaybeContiguous) {
      const int r0 = __builtin_amdgcn_readfirstlane(rows[U.start]);
      U.row0 = r0;
      U.contig = __builtin_amdgcn_readfirstlane(rows[U.start + U.n - 1]) - r0 == U.n - 1;
    }
    return U;
  };
  // (only for units that are not moved with buffer instructions)
  auto row_of = [&](const Unit& U, int r) -> int64_t { return tok_row(rows, U.start + r); };
  // descriptor of head h of rows row0 .. row0 + cnt - 1 of a tensor with `stride` elements per row (cnt <= 0: of nothing)
  auto unit_rsrc = [&](const uint16_t* base, int64_t stride, const Unit& U, int cnt) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(base) + (U.row0 * stride + U.h * kD), 0,
                                             cnt > 0 ? ((cnt - 1) * (int)stride + kD) * 2 : 0, kRsrcFlags);
  };
  constexpr int kNt = 2;   // cache policy of a buffer instruction: non-temporal

  // ---- coalesced row loads; thread (st_row, st_col) moves 16 bytes of rows st_row, +32, +64, +96.
  // The backward is the last reader of the forward's activations: non-temporal loads keep this one-pass
  // stream from evicting what other kernels of the step still need from L2 / the memory-side cache.
  u32x4 tk[4], tv[4], tq[4], tg[4], to[4];
  auto issue_kv = [&](const Unit& U) {
    if (kMode != kRowsPerLane && U.contig) {
      const __amdgpu_buffer_rsrc_t kr = unit_rsrc(k, ks, U, U.nk), vr = unit_rsrc(v, vs, U, U.nk);
      const uint32_t ko = ((uint32_t)st_row * (uint32_t)ks + (uint32_t)st_col) * 2u;
      const uint32_t vo = ((uint32_t)st_row * (uint32_t)vs + (uint32_t)st_col) * 2u;
#pragma unroll
      for (int it = 0; it < 4; ++it) {
        tk[it] = __builtin_amdgcn_raw_buffer_load_b128(kr, ko + (uint32_t)(it * 64) * (uint32_t)ks, 0, kNt);
        tv[it] = __builtin_amdgcn_raw_buffer_load_b128(vr, vo + (uint32_t)(it * 64) * (uint32_t)vs, 0, kNt);
      }
      return;
    }
#pragma unroll
    for (int it = 0; it < 4; ++it) {
      tk[it] = tv[it] = u32x4{0u, 0u, 0u, 0u};
      if (32 * it + st_row < U.nk) {
        const int64_t gr = row_of(U, 32 * it + st_row);
        tk[it] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(k + gr * ks + U.h * kD + st_col));
        tv[it] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(v + gr * vs + U.h * kD + st_col));
      }
    }
  };
  auto issue_qgo = [&](const Unit& U) {
    if (kMode != kRowsPerLane && U.contig) {
      const __amdgpu_buffer_rsrc_t qr = unit_rsrc(q, qs, U, U.n), gr = unit_rsrc(dout, dos, U, U.n),
                                   orr = unit_rsrc(o, os, U, U.n);
      const uint32_t qo = ((uint32_t)st_row * (uint32_t)qs + (uint32_t)st_col) * 2u;
      const uint32_t go = ((uint32_t)st_row * (uint32_t)dos + (uint32_t)st_col) * 2u;
      const uint32_t oo = ((uint32_t)st_row * (uint32_t)os + (uint32_t)st_col) * 2u;
#pragma unroll
      for (int it = 0; it < 4; ++it) {
        tq[it] = __builtin_amdgcn_raw_buffer_load_b128(qr, qo + (uint32_t)(it * 64) * (uint32_t)qs, 0, kNt);
        tg[it] = __builtin_amdgcn_raw_buffer_load_b128(gr, go + (uint32_t)(it * 64) * (uint32_t)dos, 0, kNt);
        to[it] = __builtin_amdgcn_raw_buffer_load_b128(orr, oo + (uint32_t)(it * 64) * (uint32_t)os, 0, kNt);
      }
      return;
    }
#pragma unroll
    for (int it = 0; it < 4; ++it) {
      tq[it] = tg[it] = to[it] = u32x4{0u, 0u, 0u, 0u};
      if (32 * it + st_row < U.n) {
        const int64_t gr = row_of(U, 32 * it + st_row);
        tq[it] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(q + gr * qs + U.h * kD + st_col));
        tg[it] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(dout + gr * dos + U.h * kD + st_col));
        to[it] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(o + gr * os + U.h * kD + st_col));
      }
    }
  };

  // rows 32 it + st_row of all five tensors of a unit that is moved with buffer instructions
  auto issue_group = [&](const Unit& U, int it) {
    const __amdgpu_buffer_rsrc_t kr = unit_rsrc(k, ks, U, U.nk), vr = unit_rsrc(v, vs, U, U.nk);
    const __amdgpu_buffer_rsrc_t qr = unit_rsrc(q, qs, U, U.n), gr = unit_rsrc(dout, dos, U, U.n),
                                 orr = unit_rsrc(o, os, U, U.n);
    const uint32_t r = (uint32_t)(32 * it + st_row);
    const uint32_t c2 = (uint32_t)st_col * 2u;
    tk[it] = __builtin_amdgcn_raw_buffer_load_b128(kr, r * (uint32_t)ks * 2u + c2, 0, kNt);
    tv[it] = __builtin_amdgcn_raw_buffer_load_b128(vr, r * (uint32_t)vs * 2u + c2, 0, kNt);
    tq[it] = __builtin_amdgcn_raw_buffer_load_b128(qr, r * (uint32_t)qs * 2u + c2, 0, kNt);
    tg[it] = __builtin_amdgcn_raw_buffer_load_b128(gr, r * (uint32_t)dos * 2u + c2, 0, kNt);
    to[it] = __builtin_amdgcn_raw_buffer_load_b128(orr, r * (uint32_t)os * 2u + c2, 0, kNt);
  };

  Unit nxt = find_unit(kUnits * blockIdx.x);
  issue_kv(nxt);
  issue_qgo(nxt);

#pragma unroll
  for (int iu = 0; iu < kUnits; ++iu) {
    const Unit U = nxt;
    const bool more = iu + 1 < kUnits;
    if (more) nxt = find_unit(kUnits * blockIdx.x + iu + 1);
    // n, h and nblk are uniform over the workgroup: every thread takes the same branches around the barriers
    const int n = U.n, nk = U.nk, h = U.h;
    const int nblk = (n + 31) >> 5;        // blocks of 32 queries
    const int nblk_k = (nk + 31) >> 5;     // blocks of 32 keys
    const bool wave_active = wave < nblk;  // this wave's tokens exist: phase 2 (queries) and the gradient rows
    const bool wave_keys = wave < nblk_k;  // ... and are keys: phase 1
    bf16x8 bk[4], bv[4];   // K^T, V^T fragments (B operands): lane = key column, 8 consecutive d per k-step

    if (n > 0) {
      // ---- phase 0
      // stored negated: -lse in base-2 units (-inf past the end, which makes P = 0 there)
      if (tid < kTile) sLse[tid] = tid < n ? -lse[(int64_t)h * T + U.start + tid] * kLog2e : -INFINITY;
      // K and V rows are staged in the dS buffer, which is free until phase 1: the 32 rows of K and of V that wave
      // `it` will own go into the very part of it that this wave later fills with dS (rows of 128 bytes, the 16-byte
      // pieces of a row rotated by the row number so that a wave's fragment reads spread over the banks).  A wave thus
      // overwrites only K/V rows it has already taken into registers, and one barrier serves all four tiles.
#pragma unroll
      for (int it = 0; it < 4; ++it) {
        const int row = 32 * it + st_row;
        if (it < nblk) {   // rows n..32*nblk-1 are zeros; rows >= 32*nblk are never read
          uint16_t* part = &sDs[it * 32 * kDsPitch];
          const int piece = ((st_col >> 3) ^ (st_row & 7)) * 8;
          *reinterpret_cast<u32x4*>(&part[st_row * 64 + piece]) = tk[it];
          *reinterpret_cast<u32x4*>(&part[2048 + st_row * 64 + piece]) = tv[it];
          *reinterpret_cast<u32x4*>(&sA[row * kPitch + st_col]) = tq[it];
          *reinterpret_cast<u32x4*>(&sB[row * kPitch + st_col]) = tg[it];
        }
        float acc = 0.f;   // Delta = rowsum(dO * O): 8 lanes per row, 8 elements each
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          acc = fmaf(__uint_as_float(tg[it][i] << 16), __uint_as_float(to[it][i] << 16), acc);
          acc = fmaf(__uint_as_float(tg[it][i] & 0xffff0000u), __uint_as_float(to[it][i] & 0xffff0000u), acc);
        }
        acc += __shfl_xor(acc, 1, 64);
        acc += __shfl_xor(acc, 2, 64);
        acc += __shfl_xor(acc, 4, 64);
        if ((tid & 7) == 0) sDelta[row] = -acc;
      }
      __syncthreads();
      {
        const uint16_t* part = &sDs[wave * 32 * kDsPitch];
#pragma unroll
        for (int s = 0; s < 4; ++s) {
          const int piece = ((2 * s + g) ^ (c & 7)) * 8;
          bk[s] = lds_read8(&part[c * 64 + piece]);
          bv[s] = lds_read8(&part[2048 + c * 64 + piece]);
        }
      }
    }
    if (n <= 0) {
      if (more) {
        issue_kv(nxt);
        issue_qgo(nxt);
      }
      continue;
    }

    // ---- phase 1
    f32x16 dkacc[2], dvacc[2];   // dK^T, dV^T: d along accumulator rows, this wave's keys along lanes
#pragma unroll
    for (int i = 0; i < 16; ++i) { dkacc[0][i] = dkacc[1][i] = dvacc[0][i] = dvacc[1][i] = 0.f; }
    if (wave_keys) {
      // The S accumulator is pre-loaded with bias/scale = -(m_h/scale)|i-j| and the dP accumulator with
      // -Delta_i, so that after the matrix products  P = exp2(acc_S * c - lse2_i)  and  dS = P * acc_dP.
      const float k1 = slopes[h] / scale;
      float fj = (float)(kj - 4 * g);   // i - j = ci - fj with ci = 32ib + 8*(v/4) + v%4
      asm volatile("" : "+v"(fj));
#pragma unroll 1
      for (int ib = 0; ib < nblk; ++ib) {
        f32x16 sacc, pacc;
        const float d0 = (float)(32 * ib) - fj;
        if (ib == wave) {   // block with the diagonal
#pragma unroll
          for (int i = 0; i < 16; ++i) sacc[i] = -k1 * fabsf(d0 + (float)(8 * (i >> 2) + (i & 3)));
        } else {            // |i-j| = +-(ci - fj) on the whole block
          const float sk = ib < wave ? k1 : -k1;
          const float a = sk * d0;
#pragma unroll
          for (int i = 0; i < 16; ++i) sacc[i] = fmaf((float)(8 * (i >> 2) + (i & 3)), sk, a);
        }
        float nl[16];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const float4 l4 = *reinterpret_cast<const float4*>(&sLse[32 * ib + 8 * r + 4 * g]);
          const float4 d4 = *reinterpret_cast<const float4*>(&sDelta[32 * ib + 8 * r + 4 * g]);
          nl[4 * r + 0] = l4.x; nl[4 * r + 1] = l4.y; nl[4 * r + 2] = l4.z; nl[4 * r + 3] = l4.w;
          pacc[4 * r + 0] = d4.x; pacc[4 * r + 1] = d4.y; pacc[4 * r + 2] = d4.z; pacc[4 * r + 3] = d4.w;
        }
        const uint16_t* qrow = &sA[(32 * ib + c) * kPitch + 8 * g];
        const uint16_t* grow = &sB[(32 * ib + c) * kPitch + 8 * g];
#pragma unroll
        for (int s = 0; s < 4; ++s) {
          sacc = mfma32(lds_read8(qrow + 16 * s), bk[s], sacc);
          pacc = mfma32(lds_read8(grow + 16 * s), bv[s], pacc);
        }
#pragma unroll
        for (int r = 0; r < 4; ++r) {
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const int i = 4 * r + e;
            const float p = fast_exp2(fmaf(sacc[i], cs, nl[i]));
            sacc[i] = p;
            pacc[i] = p * pacc[i];
          }
          // dS of queries 32ib + 8r + 4g + 0..3 for this lane's key.  A key past the sequence end may hold
          // inf/NaN here (its score never entered lse) and phase 2 multiplies it with a zero K row, so it
          // must be an exact zero in LDS.
          u32x2 w;
          w[0] = kj < nk ? pack_bf16(pacc[4 * r + 0], pacc[4 * r + 1]) : 0u;
          w[1] = kj < nk ? pack_bf16(pacc[4 * r + 2], pacc[4 * r + 3]) : 0u;
          *reinterpret_cast<u32x2*>(&sDs[kj * kDsPitch + 32 * ib + 8 * r + 4 * g]) = w;
        }
#pragma unroll
        for (int kk = 0; kk < 2; ++kk) {
          const bf16x8 bp = pack8(sacc[8 * kk + 0], sacc[8 * kk + 1], sacc[8 * kk + 2], sacc[8 * kk + 3],
                                  sacc[8 * kk + 4], sacc[8 * kk + 5], sacc[8 * kk + 6], sacc[8 * kk + 7]);
          const bf16x8 bs = pack8(pacc[8 * kk + 0], pacc[8 * kk + 1], pacc[8 * kk + 2], pacc[8 * kk + 3],
                                  pacc[8 * kk + 4], pacc[8 * kk + 5], pacc[8 * kk + 6], pacc[8 * kk + 7]);
          const int roff = (32 * ib + 16 * kk + tr_row) * kPitch + tr_col;
#pragma unroll
          for (int db = 0; db < 2; ++db) {
            const bf16x8 ag = join_tr(lds_read_tr4(&sB[roff + 32 * db]), lds_read_tr4(&sB[roff + 32 * db + 8 * kPitch]));
            dvacc[db] = mfma32(ag, bp, dvacc[db]);
            const bf16x8 aq = join_tr(lds_read_tr4(&sA[roff + 32 * db]), lds_read_tr4(&sA[roff + 32 * db + 8 * kPitch]));
            dkacc[db] = mfma32(aq, bs, dkacc[db]);
          }
        }
      }
    }
    __syncthreads();   // Q and dO have been read by everyone, all of dS is written

    // Accumulators (lane = token, 4 consecutive d per register group) -> this wave's 32 rows of sB ->
    // full rows of 128 bytes to global memory.  The slab is private to the wave, and the LDS operations
    // of one wave complete in order, so no barrier is needed between its uses.
    uint16_t* slab = &sB[kw * kPitch];
    // (rows at and beyond `live` are written as zeros: tokens that are no keys have zero dK and dV)
    auto store_rows = [&](const f32x16(&acc)[2], float mul, uint16_t* __restrict__ out, int64_t stride, int live) {
#pragma unroll
      for (int db = 0; db < 2; ++db) {
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          u32x2 w;
          w[0] = pack_bf16(acc[db][4 * r + 0] * mul, acc[db][4 * r + 1] * mul);
          w[1] = pack_bf16(acc[db][4 * r + 2] * mul, acc[db][4 * r + 3] * mul);
          *reinterpret_cast<u32x2*>(&slab[c * kPitch + 32 * db + 8 * r + 4 * g]) = w;
        }
      }
      if (kMode != kRowsPerLane && U.contig) {
        const __amdgpu_buffer_rsrc_t wr = unit_rsrc(out, stride, U, n);   // rows at and beyond n are dropped
        const uint32_t wo = ((uint32_t)(kw + orow) * (uint32_t)stride + (uint32_t)ocol) * 2u;
#pragma unroll
        for (int it = 0; it < 4; ++it) {
          const int row = 8 * it + orow;
          u32x4 w = *reinterpret_cast<const u32x4*>(&slab[row * kPitch + ocol]);
          if (kw + row >= live) w = u32x4{0u, 0u, 0u, 0u};
          __builtin_amdgcn_raw_buffer_store_b128(w, wr, wo + (uint32_t)(it * 16) * (uint32_t)stride, 0, kRows ? kNt : 0);
        }
        return;
      }
      uint16_t* oh = out + h * kD + ocol;
#pragma unroll
      for (int it = 0; it < 4; ++it) {
        const int row = 8 * it + orow;
        u32x4 w = *reinterpret_cast<const u32x4*>(&slab[row * kPitch + ocol]);
        if (kw + row >= live) w = u32x4{0u, 0u, 0u, 0u};
        if (kw + row < n) {
          // written into the padded layout these rows are final results of the step: stream them out
          if (rows) __builtin_nontemporal_store(w, reinterpret_cast<u32x4*>(oh + row_of(U, kw + row) * stride));
          else *reinterpret_cast<u32x4*>(oh + row_of(U, kw + row) * stride) = w;
        }
      }
    };

    // ---- phase 2
    if (wave_active) {
      store_rows(dkacc, scale, dk, dks, nk);
      store_rows(dvacc, 1.f, dv, dvs, nk);
    }
    if (wave_keys) {
      // K registers -> LDS over Q; rows of keys >= nk are zeros because they were staged as zeros
#pragma unroll
      for (int s = 0; s < 4; ++s)
        *reinterpret_cast<u32x4*>(&sA[kj * kPitch + 16 * s + 8 * g]) = __builtin_bit_cast(u32x4, bk[s]);
    }
    // dK, dV and the K fragments have left their registers: room for the next unit's rows, which travel while
    // dQ is computed and stored (the fences keep the compiler from moving the loads further up, where the
    // registers are still taken)
    // packed tokens: the next unit's loads go out in four groups between the steps of the dQ loop (with token_rows
    // the compiler runs out of registers for that: there they go out in one burst, before the loop)
    const bool spread = more && kMode == kRowsIdentity;
    __builtin_amdgcn_sched_barrier(0);
    if (more && !spread) {
      issue_kv(nxt);
      issue_qgo(nxt);
    }
    __builtin_amdgcn_sched_barrier(0);
    __syncthreads();
    {
      f32x16 dqacc[2];
#pragma unroll
      for (int i = 0; i < 16; ++i) { dqacc[0][i] = 0.f; dqacc[1][i] = 0.f; }
#pragma unroll
      for (int jb = 0; jb < 4; ++jb) {
        if (spread) issue_group(nxt, jb);
        __builtin_amdgcn_sched_barrier(0);
        if (wave_active && jb < nblk_k)
#pragma unroll
        for (int kk = 0; kk < 2; ++kk) {
          const int krow = 32 * jb + 16 * kk + tr_row;
          const bf16x8 bs = join_tr(lds_read_tr4(&sDs[krow * kDsPitch + kw + tr_col]),
                                    lds_read_tr4(&sDs[(krow + 8) * kDsPitch + kw + tr_col]));
#pragma unroll
          for (int db = 0; db < 2; ++db) {
            const bf16x8 ak = join_tr(lds_read_tr4(&sA[krow * kPitch + tr_col + 32 * db]),
                                      lds_read_tr4(&sA[(krow + 8) * kPitch + tr_col + 32 * db]));
            dqacc[db] = mfma32(ak, bs, dqacc[db]);
          }
        }
        __builtin_amdgcn_sched_barrier(0);
      }
      if (wave_active) store_rows(dqacc, scale, dq, dqs, n);
    }
    if (more) __syncthreads();   // the next unit's phase 0 overwrites sA, sB, sLse and sDelta
  }
}

}  // namespace

mb_status launch_attn_bwd_mfma(const AttnShape& s, const void* dout, const void* q, const void* k, const void* v,
                               const void* o, const float* lse, int64_t dos, int64_t qs, int64_t ks, int64_t vs,
                               int64_t os, void* dq, void* dk, void* dv, int64_t dqs, int64_t dks, int64_t dvs,
                               float* delta_ws, hipStream_t stream) {
  if (s.B > 65535) return fail(MB_ERR_UNSUPPORTED, "B=%d exceeds 65535 sequences per call", s.B);
  if (s.max_seqlen <= kTile) {
    const int64_t units = (int64_t)s.B * s.H;   // (sequence, head) pairs, head fastest; < 2^30 (checked by the caller)
#define MB_LAUNCH_FUSED(R, U)                                                                                        \
  hipLaunchKernelGGL((attn_bwd_fused128_kernel<R, U>), dim3((unsigned)((units + U - 1) / U)), dim3(256), 0,       \
                     stream, (const uint16_t*)dout, (const uint16_t*)q, (const uint16_t*)k, (const uint16_t*)v,    \
                     (const uint16_t*)o, lse, dos, qs, ks, vs, os, s.cu_seqlens, s.slopes, s.scale, (uint16_t*)dq, \
                     (uint16_t*)dk, (uint16_t*)dv, dqs, dks, dvs, s.T, s.token_rows, s.misuse, s.key_lens, s.H,    \
                     (int)units)
    // buffer instructions: the 128 rows a unit can have must lie within 2^31 bytes in every tensor
    int64_t widest = 0;
    for (const int64_t st : {dos, qs, ks, vs, os, dqs, dks, dvs}) widest = st > widest ? st : widest;
    const bool narrow = (int64_t)kTile * widest * 2 < ((int64_t)1 << 31);
    if (!narrow) MB_LAUNCH_FUSED(kRowsPerLane, 2);
    else if (s.token_rows) MB_LAUNCH_FUSED(kRowsMaybeContiguous, 2);
    else MB_LAUNCH_FUSED(kRowsIdentity, 2);
#undef MB_LAUNCH_FUSED
    return check_launch("attn_bwd_fused128_kernel");
  }
  // the work plan: the caller's, or built behind Delta in the workspace
  const int64_t cap = attn_plan_cap(s.B, s.max_seqlen, s.H);
  if (cap * kPlanXcds >= ((int64_t)1 << 31)) return fail(MB_ERR_UNSUPPORTED, "B * H * max_seqlen is too large for one launch");
  const int32_t* plan = s.plan;
  mb_status st = MB_OK;
  if (plan == nullptr) {
    int32_t* own = reinterpret_cast<int32_t*>(reinterpret_cast<char*>(delta_ws) + attn_bwd_delta_bytes(s.H, s.T));
    st = launch_attn_plan(s, own, nullptr, stream);
    if (st != MB_OK) return st;
    plan = own;
  }
  // buffer-load path: a sequence's rows within 2^31 bytes of its first
  int64_t widest = qs > ks ? qs : ks;
  widest = widest > vs ? widest : vs;
  widest = widest > dos ? widest : dos;
  const bool narrow = (int64_t)s.max_seqlen * widest * 2 < ((int64_t)1 << 31);
  const dim3 grid((unsigned)(cap * kPlanXcds));
  // dQ first: it also leaves Delta for the dK/dV kernel
#define MB_LAUNCH_DQ(R)                                                                                            \
  hipLaunchKernelGGL(attn_bwd_dq_kernel<R>, grid, dim3(256), 0, stream, (const uint16_t*)dout, (const uint16_t*)q,  \
                     (const uint16_t*)k, (const uint16_t*)v, (const uint16_t*)o, lse, delta_ws, dos, qs, ks, vs,    \
                     os, s.slopes, s.scale, (uint16_t*)dq, dqs, s.T, s.token_rows, plan, cap)
  if (!narrow) MB_LAUNCH_DQ(kRowsPerLane);
  else if (s.token_rows) MB_LAUNCH_DQ(kRowsMaybeContiguous);
  else MB_LAUNCH_DQ(kRowsIdentity);
#undef MB_LAUNCH_DQ
  st = check_launch("attn_bwd_dq_kernel");
  if (st != MB_OK) return st;
#define MB_LAUNCH_DKV(R)                                                                                           \
  hipLaunchKernelGGL(attn_bwd_dkv_kernel<R>, grid, dim3(256), 0, stream, (const uint16_t*)dout, (const uint16_t*)q, \
                     (const uint16_t*)k, (const uint16_t*)v, lse, delta_ws, dos, qs, ks, vs, s.slopes, s.scale,     \
                     (uint16_t*)dk, (uint16_t*)dv, dks, dvs, s.T, s.token_rows, plan, cap)
  if (!narrow) MB_LAUNCH_DKV(kRowsPerLane);
  else if (s.token_rows) MB_LAUNCH_DKV(kRowsMaybeContiguous);
  else MB_LAUNCH_DKV(kRowsIdentity);
#undef MB_LAUNCH_DKV
  return check_launch("attn_bwd_dkv_kernel");
}

size_t attn_bwd_mfma_workspace_bytes(int B, int T, int max_seqlen, int H) {
  return attn_bwd_delta_bytes(H, T) + (max_seqlen <= kTile ? 0 : attn_plan_bytes(B, max_seqlen, H));
}

}  // namespace mb
