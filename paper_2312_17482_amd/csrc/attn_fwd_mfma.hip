// Forward ALiBi attention on the matrix cores: bf16, head_dim 64, variable-length packed sequences.
//
// Computes the attention weights of the paper's Eq. 1, softmax_j(scale * q_i.k_j - m_h*|i-j|), and
// O = P V tile by tile with a running (online) softmax, so the score matrix never leaves the chip
// ("FlashAttention" paragraph).  The bias is evaluated in registers from the token distance.
//
// Work split: one workgroup (4 waves) per (sequence, head, tile of 128 queries); wave w owns queries
// 32w..32w+31 of the tile.  K and V tiles of 128 keys are staged in LDS and shared by the 4 waves.
// Global memory is always touched as full 128-byte rows of one head (8 lanes x 16 bytes).
// Scores are produced TRANSPOSED, S^T = K Q^T (keys along accumulator rows, queries along lanes), so
//   * a query's row statistics (max, sum) are reductions over a lane's own registers plus one
//     exchange with the partner lane l^32, and
//   * the accumulator tile, rounded to bf16, is already the B operand of O^T += V^T P^T.
#include "attn_plan.h"
#include "common.h"
#include "mfma_util.h"

namespace mb {
namespace {

constexpr int kBlockQ = 128;   // queries per workgroup
constexpr int kBlockK = 128;   // keys per LDS tile
constexpr int kD = 64;
constexpr int kKStride = 72;   // LDS row pitch of K in bf16 (144 B): 16-byte row reads spread over banks
constexpr int kVStride = 80;   // LDS row pitch of V in bf16 (160 B): 4-row transposing reads spread over banks

// Any sequence length: tiles of 64 keys with a running (online) softmax.  LDS holds two K/V tiles: while
// one is consumed, the next travels HBM -> registers -> the other buffer, so a workgroup waits for memory
// only on its first tile and there is one barrier per tile.  Registers are kept <= 128 so that four
// workgroups share a compute unit.  Same arithmetic as the single-tile kernel below (bias pre-loaded
// into the accumulator, scale folded into the exponent); the running output is rescaled only when some
// query's maximum actually moved.
constexpr int kTileK = 64;                                        // keys per LDS tile
constexpr int kBufElems = kTileK * kKStride + kTileK * kVStride;  // one K tile + one V tile

// A sequence longer than the max_seqlen the launch was sized for: the sticky flag is raised and the
// sequence's log-sum-exp rows (n of them, from `row`) become NaN, so the misuse shows in the result too.
__device__ __forceinline__ void poison_lse(float* __restrict__ row, int n, int32_t* __restrict__ misuse) {
  raise_misuse(misuse);
  for (int i = threadIdx.x; i < n; i += blockDim.x) row[i] = __builtin_nanf("");
}

// The forward's own plan launch: workgroup c builds list c (see attn_plan.h); workgroup 0 then marks the
// sequences the plan skipped (longer than max_seqlen) by setting their log-sum-exp rows to NaN.
__global__ __launch_bounds__(kPlanThreads) void attn_plan_kernel(const int32_t* __restrict__ cu,
                                                                 const int32_t* __restrict__ key_lens, int B, int H,
                                                                 int max_seqlen, int64_t cap, int32_t* __restrict__ plan,
                                                                 int32_t* __restrict__ misuse, float* __restrict__ lse,
                                                                 int T) {
  __shared__ __attribute__((aligned(16))) PlanLds lds;
  build_plan_list(cu, key_lens, B, H, max_seqlen, cap, plan, blockIdx.x, misuse, lds);
  if (blockIdx.x != 0 || lse == nullptr) return;
  for (int b = 0; b < B; ++b) {
    const int s0 = cu[b], len = cu[b + 1] - s0;
    if (len > max_seqlen)
      for (int h = 0; h < H; ++h) poison_lse(lse + (int64_t)h * T + s0, len, misuse);
  }
}

// kMode (see kRowsIdentity .. in common.h): for a sequence whose tokens sit in consecutive rows of the
// activation buffers, spanning fewer than 2^31 bytes, the K/V rows of a tile are fetched with buffer loads
// whose descriptor starts at the tile's first row and ends at the sequence's last one: the address is
// scalar arithmetic plus one constant per-lane offset, and rows past the end read as zeros without a
// compare.  Otherwise every row's address is formed per lane (row index looked up in token_rows when given).
template <int kMode>
__global__ __launch_bounds__(256, 3) void attn_fwd_tiled_kernel(
    const uint16_t* __restrict__ q, const uint16_t* __restrict__ k, const uint16_t* __restrict__ v, int64_t qs,
    int64_t ks, int64_t vs, const float* __restrict__ slopes, float scale, uint16_t* __restrict__ o, int64_t os,
    float* __restrict__ lse, int T, const int32_t* __restrict__ token_rows, const int32_t* __restrict__ plan,
    int64_t plan_cap) {
  const int32_t* rows = kMode == kRowsIdentity ? nullptr : token_rows;
  __shared__ __attribute__((aligned(16))) uint16_t smem[2 * kBufElems];   // 38 KB; also stages Q and O rows

  int start, n, nk, qtile, h;   // nk <= n: the sequence's first nk tokens are its keys
  if (!plan_fetch(plan, plan_cap, &start, &n, &nk, &qtile, &h)) return;   // this XCD's list is shorter
  const int q0 = qtile * kBlockQ;   // < n by construction of the plan
  // first buffer row of the sequence, and whether its tokens sit in consecutive rows
  const int row0 = kMode == kRowsMaybeContiguous ? __builtin_amdgcn_readfirstlane(rows[start]) : start;
  const bool contig =
      kMode == kRowsIdentity ||
      (kMode == kRowsMaybeContiguous && __builtin_amdgcn_readfirstlane(rows[start + n - 1]) - row0 == n - 1);

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform: keeps per-wave branches scalar
  const int c = lane & 31, g = lane >> 5;
  const int qw = q0 + 32 * wave;          // first query of this wave
  const bool wave_active = qw < n;
  const int qi = qw + c;                  // this lane's query (position inside the sequence)
  const int qblk = (q0 >> 5) + wave;      // index of this wave's block of 32 queries
  const int ntiles = (nk + kTileK - 1) / kTileK;
  const int st_row = tid >> 3, st_col = (tid & 7) * 8;
  const uint16_t* kh = k + h * kD + st_col;
  const uint16_t* vh = v + h * kD + st_col;

  u32x4 tk[2], tv[2];
  constexpr int kRsrcFlags = 0x00020000;   // raw buffer, 32-bit data format (gfx9 family)
  const uint32_t koff = ((uint32_t)st_row * (uint32_t)ks + (uint32_t)(h * kD + st_col)) * 2u;
  const uint32_t voff = ((uint32_t)st_row * (uint32_t)vs + (uint32_t)(h * kD + st_col)) * 2u;
  auto issue_tile = [&](int j0) {   // rows j0 + 32it + st_row of K and V -> registers (zeros past the end)
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
    uint16_t* bk_ = smem + buf * kBufElems;
    uint16_t* bv_ = bk_ + kTileK * kKStride;
#pragma unroll
    for (int it = 0; it < 2; ++it) {
      *reinterpret_cast<u32x4*>(&bk_[(32 * it + st_row) * kKStride + st_col]) = tk[it];
      *reinterpret_cast<u32x4*>(&bv_[(32 * it + st_row) * kVStride + st_col]) = tv[it];
    }
  };

  // ---- Q rows (coalesced) -> LDS -> Q^T fragments; the first K/V tile is already on its way
  {
    u32x4 tq[4];
#pragma unroll
    for (int it = 0; it < 4; ++it) {
      tq[it] = u32x4{0u, 0u, 0u, 0u};
      const int i = q0 + 32 * it + st_row;
      if (i < n) tq[it] = *reinterpret_cast<const u32x4*>(q + tok_row(rows, start + i) * qs + h * kD + st_col);
    }
    issue_tile(0);
#pragma unroll
    for (int it = 0; it < 4; ++it)
      *reinterpret_cast<u32x4*>(&smem[(32 * it + st_row) * kKStride + st_col]) = tq[it];
  }
  __syncthreads();
  bf16x8 bq[4];
#pragma unroll
  for (int s = 0; s < 4; ++s) bq[s] = lds_read8(&smem[(32 * wave + c) * kKStride + 16 * s + 8 * g]);
  __syncthreads();
  store_tile(0);

  const float cs = scale * kLog2e;
  const float k1 = slopes[h] / scale;
  const int tr_i = lane & 15, tr_q = lane >> 4;
  const int tr_row = (tr_i >> 2) + 4 * (tr_q >> 1);
  const int tr_col = 16 * (tr_q & 1) + 4 * (tr_i & 3);

  f32x16 oacc[2];
#pragma unroll
  for (int i = 0; i < 16; ++i) { oacc[0][i] = 0.f; oacc[1][i] = 0.f; }
  float m_run = -INFINITY;   // running maximum of the raw accumulator (dot product + bias/scale)
  float l_run = 0.f;         // running row sum, this half-wave's share

  // One tile of 64 keys.  The code that touches the running output exists once, with no branch
  // around it: a ragged last tile is handled by pre-loading -inf for the keys that do not exist (their
  // K rows are staged as zeros), so that only the accumulator pre-load has variants.
  auto tile = [&](int j0, int jt) {
    const uint16_t* bufK = smem + (jt & 1) * kBufElems;
    const uint16_t* bufV = bufK + kTileK * kKStride;
    const int rem = nk - j0;
    float fi = (float)(qi - j0 - 4 * g);   // i - j = fi - cj with cj = 32jb + 8*(v/4) + v%4
    asm volatile("" : "+v"(fi));
    f32x16 sacc[2];
#pragma unroll
    for (int jb = 0; jb < 2; ++jb) {
      const int kblk = 2 * jt + jb;
      if (kblk == qblk) {   // the block that holds the diagonal
#pragma unroll
        for (int i = 0; i < 16; ++i) sacc[jb][i] = -k1 * fabsf(fi - (float)(jb * 32 + 8 * (i >> 2) + (i & 3)));
      } else {              // |i-j| = +-(fi - cj) on the whole block
        const float sk = kblk < qblk ? k1 : -k1;
        const float a = -sk * fi;
#pragma unroll
        for (int i = 0; i < 16; ++i) sacc[jb][i] = fmaf((float)(jb * 32 + 8 * (i >> 2) + (i & 3)), sk, a);
      }
    }
    if (rem < kTileK) {   // ragged end: keys that do not exist (or are masked out) get -inf
      const int lim = rem - 4 * g;
#pragma unroll
      for (int jb = 0; jb < 2; ++jb)
#pragma unroll
        for (int i = 0; i < 16; ++i)
          sacc[jb][i] = (jb * 32 + 8 * (i >> 2) + (i & 3)) >= lim ? -INFINITY : sacc[jb][i];
    }
    const uint16_t* krow = &bufK[c * kKStride + 8 * g];
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      sacc[0] = mfma32(lds_read8(krow + 16 * s), bq[s], sacc[0]);
      sacc[1] = mfma32(lds_read8(krow + 32 * kKStride + 16 * s), bq[s], sacc[1]);
    }
    float mt = -INFINITY;
#pragma unroll
    for (int jb = 0; jb < 2; ++jb)
#pragma unroll
      for (int i = 0; i < 16; ++i) mt = fmaxf(mt, sacc[jb][i]);
    mt = max_both_halves(mt);
    const float m_new = fmaxf(m_run, mt);
    if (jt > 0 && __any(m_new > m_run)) {   // some query's maximum moved: rescale the running sums
      const float alpha = fast_exp2((m_run - m_new) * cs);
      l_run *= alpha;
#pragma unroll
      for (int i = 0; i < 16; ++i) { oacc[0][i] *= alpha; oacc[1][i] *= alpha; }
    }
    m_run = m_new;
    const float mc = m_new * cs;
    float lsum[4] = {0.f, 0.f, 0.f, 0.f};   // four short chains of additions instead of one long one
#pragma unroll
    for (int jb = 0; jb < 2; ++jb) {
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const float p = fast_exp2(fmaf(sacc[jb][i], cs, -mc));
        sacc[jb][i] = p;
        lsum[i & 3] += p;
      }
#pragma unroll
      for (int kk = 0; kk < 2; ++kk) {
        const bf16x8 bp = pack8(sacc[jb][8 * kk + 0], sacc[jb][8 * kk + 1], sacc[jb][8 * kk + 2],
                                sacc[jb][8 * kk + 3], sacc[jb][8 * kk + 4], sacc[jb][8 * kk + 5],
                                sacc[jb][8 * kk + 6], sacc[jb][8 * kk + 7]);
        const uint16_t* vb = &bufV[(jb * 32 + 16 * kk + tr_row) * kVStride + tr_col];
#pragma unroll
        for (int db = 0; db < 2; ++db) {
          const s16x4 lo = lds_read_tr4(vb + 32 * db);
          const s16x4 hi = lds_read_tr4(vb + 32 * db + 8 * kVStride);
          oacc[db] = mfma32(join_tr(lo, hi), bp, oacc[db]);
        }
      }
    }
    l_run += (lsum[0] + lsum[1]) + (lsum[2] + lsum[3]);
  };

#pragma unroll 1
  for (int jt = 0; jt < ntiles; ++jt) {
    const int j0 = jt * kTileK;
    __syncthreads();   // tile jt is complete in its buffer; the other buffer is no longer being read
    if (jt + 1 < ntiles) issue_tile(j0 + kTileK);

    if (wave_active) tile(j0, jt);
    if (jt + 1 < ntiles) store_tile((jt + 1) & 1);
  }
  __syncthreads();   // everyone is done with the K/V buffers: they now carry the output rows
  if (!wave_active) return;

  const float l = sum_both_halves(l_run);
  const float inv = 1.f / l;
  if (g == 0 && qi < n) lse[(int64_t)h * T + start + qi] = (m_run * cs + __log2f(l)) * kLn2;
  // O^T accumulators -> 32 LDS rows private to this wave -> full 128-byte rows
  uint16_t* slab = &smem[(32 * wave) * kKStride];
#pragma unroll
  for (int db = 0; db < 2; ++db) {
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      u32x2 w;
      w[0] = pack_bf16(oacc[db][4 * r + 0] * inv, oacc[db][4 * r + 1] * inv);
      w[1] = pack_bf16(oacc[db][4 * r + 2] * inv, oacc[db][4 * r + 3] * inv);
      *reinterpret_cast<u32x2*>(&slab[c * kKStride + 32 * db + 8 * r + 4 * g]) = w;
    }
  }
  const int orow = lane >> 3, ocol = (lane & 7) * 8;
#pragma unroll
  for (int it = 0; it < 4; ++it) {
    const int row = 8 * it + orow;
    const u32x4 w = *reinterpret_cast<const u32x4*>(&slab[row * kKStride + ocol]);
    if (qw + row < n) *reinterpret_cast<u32x4*>(o + tok_row(rows, start + qw + row) * os + h * kD + ocol) = w;
  }
}

// ------------------------------------------------------------------------------------------------ n <= 128
// Sequences of at most 128 tokens (the pretraining length of the paper): one K/V tile per
// (sequence, head), so the softmax is a single pass with no running rescale.  Such a unit is tiny
// (48 KB in, 16 KB out), so the kernel is built for occupancy: one workgroup per (sequence, head),
// <= 128 registers and 39 KB of LDS, i.e. four workgroups per compute unit whose load, compute and
// store phases overlap each other.
//
// Arithmetic per score is kept to a handful of vector instructions:
//   * the accumulator of S^T = K Q^T is not zeroed but pre-loaded with bias/scale = -(m_h/scale)|i-j|,
//     so the matrix core adds the bias; off the diagonal block |i-j| is linear in i and j, which makes
//     the pre-load one fused multiply-add per score;
//   * the row maximum is taken on the raw accumulator and the scale is folded into the exponent:
//     p = exp2(acc * c - max * c), c = scale * log2(e)   (requires scale > 0).
// kRows: the activation buffers are a padded batch and token t sits at row rows[t] (the gather and the
// scatter of the unpadding step happen in this kernel's own row loads and stores).
template <bool kRows>
__global__ __launch_bounds__(256, 4) void attn_fwd_short_kernel(
    const uint16_t* __restrict__ q, const uint16_t* __restrict__ k, const uint16_t* __restrict__ v, int64_t qs,
    int64_t ks, int64_t vs, const int32_t* __restrict__ cu, const float* __restrict__ slopes, float scale,
    uint16_t* __restrict__ o, int64_t os, float* __restrict__ lse, int T, const int32_t* __restrict__ rows,
    int32_t* __restrict__ misuse, const int32_t* __restrict__ key_lens) {
  // Every global access is a full 128-byte row of one head shared by 8 lanes (16 bytes each); the
  // fragment layouts the matrix cores need are produced by passing through LDS:
  //   sV first carries the Q tile (rows -> Q^T fragments), then V;  after the S phase each wave reuses
  //   its own 32 rows of sK to turn its O^T accumulators back into rows.
  __shared__ __attribute__((aligned(16))) uint16_t sK[kBlockK * kKStride];
  __shared__ __attribute__((aligned(16))) uint16_t sV[kBlockK * kVStride];

  const int h = blockIdx.x, b = blockIdx.y;
  const int start = cu[b];
  const int n = cu[b + 1] - start;
  if (n <= 0) return;
  if (n > kBlockK) {   // the caller promised max_seqlen <= 128: skipped, never truncated
    poison_lse(lse + (int64_t)h * T + start, n, misuse);
    return;
  }
  const int nk = key_lens ? min(key_lens[b], n) : n;   // the sequence's first nk tokens are its keys
  if (nk <= 0) return;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int c = lane & 31, g = lane >> 5;
  const int qi = 32 * wave + c;
  const int nblk = (n + 31) >> 5;       // blocks of 32 queries
  const int nblk_k = (nk + 31) >> 5;    // blocks of 32 keys
  const bool wave_active = wave < nblk;

  // ---- coalesced row loads: thread (st_row, st_col) moves 16 bytes of rows st_row, +32, +64, +96
  const int st_row = tid >> 3, st_col = (tid & 7) * 8;
  u32x4 tq[4], tk[4], tv[4];
  // Rows listed in ascending order whose first and last differ by n - 1 are consecutive (the usual
  // case: padding is a suffix of each batch row); then no per-token index load is needed.
  int row0 = 0;
  bool contig = true;
  if (kRows) {
    row0 = rows[start];
    contig = rows[start + n - 1] - row0 == n - 1;
  }
  auto row_of = [&](int r) -> int64_t { return contig ? (int64_t)(row0 + r) : (int64_t)rows[start + r]; };
  if (kRows) {
    int64_t gr[4];
#pragma unroll
    for (int it = 0; it < 4; ++it) gr[it] = 32 * it + st_row < n ? row_of(32 * it + st_row) : 0;
#pragma unroll
    for (int it = 0; it < 4; ++it) {
      tq[it] = tk[it] = tv[it] = u32x4{0u, 0u, 0u, 0u};
      if (32 * it + st_row < n) tq[it] = *reinterpret_cast<const u32x4*>(q + gr[it] * qs + h * kD + st_col);
      if (32 * it + st_row < nk) {
        tk[it] = *reinterpret_cast<const u32x4*>(k + gr[it] * ks + h * kD + st_col);
        tv[it] = *reinterpret_cast<const u32x4*>(v + gr[it] * vs + h * kD + st_col);
      }
    }
  } else {
    const uint16_t* qh = q + (int64_t)start * qs + h * kD;
    const uint16_t* kh = k + (int64_t)start * ks + h * kD;
    const uint16_t* vh = v + (int64_t)start * vs + h * kD;
    const uint32_t qoff = (uint32_t)st_row * (uint32_t)qs + st_col;
    const uint32_t koff = (uint32_t)st_row * (uint32_t)ks + st_col;
    const uint32_t voff = (uint32_t)st_row * (uint32_t)vs + st_col;
#pragma unroll
    for (int it = 0; it < 4; ++it) {
      tq[it] = tk[it] = tv[it] = u32x4{0u, 0u, 0u, 0u};
      if (32 * it + st_row < n) tq[it] = *reinterpret_cast<const u32x4*>(qh + qoff + (uint32_t)(32 * it) * (uint32_t)qs);
      if (32 * it + st_row < nk) {
        tk[it] = *reinterpret_cast<const u32x4*>(kh + koff + (uint32_t)(32 * it) * (uint32_t)ks);
        tv[it] = *reinterpret_cast<const u32x4*>(vh + voff + (uint32_t)(32 * it) * (uint32_t)vs);
      }
    }
  }
  // rows n..32*nblk-1 are staged as zeros; rows >= 32*nblk are never read
#pragma unroll
  for (int it = 0; it < 4; ++it) {
    if (it < nblk) {
      *reinterpret_cast<u32x4*>(&sV[(32 * it + st_row) * kKStride + st_col]) = tq[it];   // Q, pitch kKStride
      *reinterpret_cast<u32x4*>(&sK[(32 * it + st_row) * kKStride + st_col]) = tk[it];
    }
  }
  __syncthreads();
  bf16x8 bq[4];   // Q^T fragments: lane = query column, 8 consecutive d per k-step
#pragma unroll
  for (int s = 0; s < 4; ++s) bq[s] = lds_read8(&sV[qi * kKStride + 16 * s + 8 * g]);
  __syncthreads();   // Q has been read by everyone: sV may now take V
#pragma unroll
  for (int it = 0; it < 4; ++it) {
    if (it < nblk) *reinterpret_cast<u32x4*>(&sV[(32 * it + st_row) * kVStride + st_col]) = tv[it];
  }

  const float cs = scale * kLog2e;
  const float k1 = slopes[h] / scale;   // bias in units of the raw dot product
  float fi = (float)(qi - 4 * g);       // i - j = fi - cj with cj = 32jb + 8*(v/4) + v%4
  asm volatile("" : "+v"(fi));          // keep the distance arithmetic in floating point
  const int lim = nk - 4 * g;           // key of (jb, v) is real iff cj < lim

  // ---- accumulators pre-loaded with the bias, then S^T = K Q^T on top
  f32x16 sacc[4];
  float m = -INFINITY;
  if (wave_active) {
#pragma unroll
    for (int jb = 0; jb < 4; ++jb) {
      if (jb < nblk_k) {
        if (jb == wave) {   // the block that holds the diagonal
#pragma unroll
          for (int i = 0; i < 16; ++i) {
            const float cj = (float)(jb * 32 + 8 * (i >> 2) + (i & 3));
            sacc[jb][i] = -k1 * fabsf(fi - cj);
          }
        } else {            // entirely left (j < i) or right (j > i) of the diagonal: |i-j| = +-(fi - cj)
          const float sk = jb < wave ? k1 : -k1;
          const float a = -sk * fi;
#pragma unroll
          for (int i = 0; i < 16; ++i) {
            const float cj = (float)(jb * 32 + 8 * (i >> 2) + (i & 3));
            sacc[jb][i] = fmaf(cj, sk, a);
          }
        }
        if (jb == nblk_k - 1 && (nk & 31)) {   // ragged end: keys >= nk get -inf
#pragma unroll
          for (int i = 0; i < 16; ++i) {
            const int cj = jb * 32 + 8 * (i >> 2) + (i & 3);
            sacc[jb][i] = cj >= lim ? -INFINITY : sacc[jb][i];
          }
        }
        const uint16_t* krow = &sK[(jb * 32 + c) * kKStride + 8 * g];
#pragma unroll
        for (int s = 0; s < 4; ++s) sacc[jb] = mfma32(lds_read8(krow + 16 * s), bq[s], sacc[jb]);
      }
    }
    // ---- row maximum of the raw accumulators
#pragma unroll
    for (int jb = 0; jb < 4; ++jb) {
      if (jb < nblk_k) {
#pragma unroll
        for (int i = 0; i < 16; ++i) m = fmaxf(m, sacc[jb][i]);
      }
    }
    m = max_both_halves(m);
  }
  __syncthreads();   // V is in LDS; nobody reads sK any more
  if (!wave_active) return;
  const float mc = m * cs;

  // ---- P^T = exp2(acc*cs - m*cs), row sum, O^T = V^T P^T
  const int tr_i = lane & 15, tr_q = lane >> 4;
  const int tr_row = (tr_i >> 2) + 4 * (tr_q >> 1);
  const int tr_col = 16 * (tr_q & 1) + 4 * (tr_i & 3);
  f32x16 oacc[2];
  float l = 0.f;
#pragma unroll
  for (int jb = 0; jb < 4; ++jb) {
    if (jb < nblk_k) {
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const float p = fast_exp2(fmaf(sacc[jb][i], cs, -mc));
        sacc[jb][i] = p;
        l += p;
      }
#pragma unroll
      for (int kk = 0; kk < 2; ++kk) {
        const bf16x8 bp = pack8(sacc[jb][8 * kk + 0], sacc[jb][8 * kk + 1], sacc[jb][8 * kk + 2],
                                sacc[jb][8 * kk + 3], sacc[jb][8 * kk + 4], sacc[jb][8 * kk + 5],
                                sacc[jb][8 * kk + 6], sacc[jb][8 * kk + 7]);
        const uint16_t* vb = &sV[(jb * 32 + 16 * kk + tr_row) * kVStride + tr_col];
#pragma unroll
        for (int db = 0; db < 2; ++db) {
          const s16x4 lo = lds_read_tr4(vb + 32 * db);
          const s16x4 hi = lds_read_tr4(vb + 32 * db + 8 * kVStride);
          if (jb == 0 && kk == 0) {
            const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
            oacc[db] = mfma32(join_tr(lo, hi), bp, zero);
          } else {
            oacc[db] = mfma32(join_tr(lo, hi), bp, oacc[db]);
          }
        }
      }
    }
  }
  l = sum_both_halves(l);
  const float inv = 1.f / l;
  if (g == 0 && qi < n) lse[(int64_t)h * T + start + qi] = (mc + __log2f(l)) * kLn2;

  // ---- O^T accumulators (lane = query, 4 consecutive d per register group) -> this wave's 32 rows of
  //      sK -> full rows of 128 bytes, 8 lanes each
  uint16_t* slab = &sK[(32 * wave) * kKStride];
#pragma unroll
  for (int db = 0; db < 2; ++db) {
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      u32x2 w;
      w[0] = pack_bf16(oacc[db][4 * r + 0] * inv, oacc[db][4 * r + 1] * inv);
      w[1] = pack_bf16(oacc[db][4 * r + 2] * inv, oacc[db][4 * r + 3] * inv);
      *reinterpret_cast<u32x2*>(&slab[c * kKStride + 32 * db + 8 * r + 4 * g]) = w;
    }
  }
  // (same wave wrote and reads the slab: LDS operations of one wave complete in order)
  uint16_t* oh = o + (kRows ? (int64_t)0 : (int64_t)(start + 32 * wave) * os) + h * kD;
  const int orow = lane >> 3, ocol = (lane & 7) * 8;
#pragma unroll
  for (int it = 0; it < 4; ++it) {
    const int row = 8 * it + orow;
    const u32x4 w = *reinterpret_cast<const u32x4*>(&slab[row * kKStride + ocol]);
    if (32 * wave + row < n) {
      if (kRows) *reinterpret_cast<u32x4*>(oh + row_of(32 * wave + row) * os + ocol) = w;
      else *reinterpret_cast<u32x4*>(oh + (uint32_t)row * (uint32_t)os + ocol) = w;
    }
  }
}

}  // namespace

mb_status launch_attn_fwd_mfma(const AttnShape& s, const void* q, const void* k, const void* v, int64_t qs,
                               int64_t ks, int64_t vs, void* o, int64_t os, float* lse, void* workspace,
                               hipStream_t stream) {
  if (s.B > 65535) return fail(MB_ERR_UNSUPPORTED, "B=%d exceeds 65535 sequences per call", s.B);
  if (s.max_seqlen <= kBlockK) {
    if (s.token_rows)
      hipLaunchKernelGGL(attn_fwd_short_kernel<true>, dim3(s.H, s.B), dim3(256), 0, stream, (const uint16_t*)q,
                         (const uint16_t*)k, (const uint16_t*)v, qs, ks, vs, s.cu_seqlens, s.slopes, s.scale,
                         (uint16_t*)o, os, lse, s.T, s.token_rows, s.misuse, s.key_lens);
    else
      hipLaunchKernelGGL(attn_fwd_short_kernel<false>, dim3(s.H, s.B), dim3(256), 0, stream, (const uint16_t*)q,
                         (const uint16_t*)k, (const uint16_t*)v, qs, ks, vs, s.cu_seqlens, s.slopes, s.scale,
                         (uint16_t*)o, os, lse, s.T, s.token_rows, s.misuse, s.key_lens);
    return check_launch("attn_fwd_short_kernel");
  }
  // any length: plan (8 small workgroups), then one workgroup per plan slot
  const int64_t cap = attn_plan_cap(s.B, s.max_seqlen, s.H);
  if (cap * kPlanXcds >= ((int64_t)1 << 31)) return fail(MB_ERR_UNSUPPORTED, "B * H * max_seqlen is too large for one launch");
  const int32_t* plan = s.plan;
  if (plan == nullptr) {   // no plan of the caller's: build one in the workspace
    const mb_status st = launch_attn_plan(s, static_cast<int32_t*>(workspace), lse, stream);
    if (st != MB_OK) return st;
    plan = static_cast<const int32_t*>(workspace);
  }
  // buffer-load path: a sequence's K / V rows within 2^31 bytes of its first
  const int64_t span = (int64_t)s.max_seqlen * (ks > vs ? ks : vs) * 2;
#define MB_LAUNCH_TILED(M)                                                                                         \
  hipLaunchKernelGGL(attn_fwd_tiled_kernel<M>, dim3((unsigned)(cap * kPlanXcds)), dim3(256), 0, stream,            \
                     (const uint16_t*)q, (const uint16_t*)k, (const uint16_t*)v, qs, ks, vs, s.slopes, s.scale,    \
                     (uint16_t*)o, os, lse, s.T, s.token_rows, plan, cap)
  if (span >= ((int64_t)1 << 31)) MB_LAUNCH_TILED(kRowsPerLane);
  else if (s.token_rows) MB_LAUNCH_TILED(kRowsMaybeContiguous);
  else MB_LAUNCH_TILED(kRowsIdentity);
#undef MB_LAUNCH_TILED
  return check_launch("attn_fwd_tiled_kernel");
}

size_t attn_fwd_mfma_workspace_bytes(int B, int max_seqlen, int H) {
  return max_seqlen <= kBlockK ? 0 : attn_plan_bytes(B, max_seqlen, H);
}

size_t attn_plan_workspace_bytes(int B, int max_seqlen, int H) { return attn_plan_bytes(B, max_seqlen, H); }

mb_status launch_attn_plan(const AttnShape& s, int32_t* plan, float* lse, hipStream_t stream) {
  hipLaunchKernelGGL(attn_plan_kernel, dim3(kPlanXcds), dim3(kPlanThreads), 0, stream, s.cu_seqlens, s.key_lens, s.B, s.H,
                     s.max_seqlen, attn_plan_cap(s.B, s.max_seqlen, s.H), plan, s.misuse, lse, s.T);
  return check_launch("attn_plan_kernel");
}

}  // namespace mb
