// GeGLU feed-forward of the encoder block (Eq. 2 of the paper):  y = (GeLU(x W1) (*) x V) W2,
// forward, bf16 storage, fp32 accumulation on the matrix cores.
//
// Two launches of one tiled GEMM kernel, both of the form  out[t, n] = sum_k X[t, k] * Wt[n, k]
// (token rows and weight rows are both contiguous along k, the storage of a linear layer):
//   1. gated:  the weight is the fused [2*inter, hidden] matrix of the appendix on GLU implementations
//      (rows 0..inter-1 = W1^T, rows inter.. = V^T).  A workgroup computes, for 256 tokens, 128 columns
//      of x W1 and THE SAME 128 columns of x V, so the slice and the product GeLU(.) (*) (.) happen on
//      the accumulators: neither projection is ever written to memory.
//   2. plain:  y = a W2 with the [hidden, inter] matrix W2^T.
//
// Tiling: 256 tokens x 256 (or 192) weight rows per workgroup of 4 waves (2 x 2, each 128 x 128 or
// 128 x 96 = 16 or 12 accumulator tiles of v_mfma_f32_32x32x16_bf16), k in steps of 64 through two LDS
// stages (next stage is written while the current one is consumed: one barrier per step), the two steps
// after that in flight in registers.  The narrower tile exists for the second projection, whose few
// column tiles otherwise leave the last round of workgroups mostly empty.
// The products are formed transposed (weight rows along accumulator rows, tokens along lanes), so a
// lane owns runs of 4 consecutive output columns of one token; the tile is turned into full 128-byte
// row segments through a wave-private LDS slab before it is stored.
#include "common.h"
#include "mfma_util.h"




namespace mb {
namespace {

constexpr int kBM = 256;                              // tokens per workgroup
constexpr int kBK = 64;                               // k per stage
constexpr int kPitch = 72;                            // LDS row pitch, elements (144 B: conflict-free 16-byte reads)
constexpr int kGroupM = 4;                            // token panels walked together (L2 reuse of the weight tiles)

// GeLU(h) = h * Phi(h), the exact (error-function) form, with Phi evaluated by the classic five-term
// rational approximation of erfc (Abramowitz & Stegun 7.1.26, absolute error below 1.5e-7):
//   x = |h| / sqrt 2,  t = 1 / (1 + p x),  u = (1/2) (a1 t + ... + a5 t^5) exp(-x^2) = Phi(-|h|),
//   Phi(h) = u for h < 0 and 1 - u otherwise,  hence  h Phi(h) = max(h, 0) - |h| u  for either sign.
// 12 vector instructions and two transcendentals per value; the result is rounded to bf16 (relative
// 2^-9) right after, so the approximation error is invisible.
__device__ __forceinline__ float gelu_exact(float h) {
  const float ah = fabsf(h);
  const float t = __builtin_amdgcn_rcpf(fmaf(0.3275911f * 0.70710678118654752f, ah, 1.0f));
  float poly = fmaf(0.5f * 1.061405429f, t, 0.5f * -1.453152027f);
  poly = fmaf(poly, t, 0.5f * 1.421413741f);
  poly = fmaf(poly, t, 0.5f * -0.284496736f);
  poly = fmaf(poly, t, 0.5f * 0.254829592f);
  const float e = __builtin_amdgcn_exp2f(h * h * (-0.5f * kLog2e));
  const float u = poly * t * e;                       // Phi(-|h|), in (0, 1/2]
  return fmaf(-ah, u, fmaxf(h, 0.0f));
}

// GeLU and its derivative Phi(h) + h phi(h) from the same intermediates (phi = the normal density).
__device__ __forceinline__ void gelu_and_grad(float h, float& val, float& grad) {
  const float ah = fabsf(h);
  const float t = __builtin_amdgcn_rcpf(fmaf(0.3275911f * 0.70710678118654752f, ah, 1.0f));
  float poly = fmaf(0.5f * 1.061405429f, t, 0.5f * -1.453152027f);
  poly = fmaf(poly, t, 0.5f * 1.421413741f);
  poly = fmaf(poly, t, 0.5f * -0.284496736f);
  poly = fmaf(poly, t, 0.5f * 0.254829592f);
  const float e = __builtin_amdgcn_exp2f(h * h * (-0.5f * kLog2e));   // exp(-h^2 / 2)
  const float u = poly * t * e;                                      // Phi(-|h|)
  val = fmaf(-ah, u, fmaxf(h, 0.0f));
  const float phi_cdf = h < 0.f ? u : 1.0f - u;
  grad = fmaf(h * 0.3989422804014327f, e, phi_cdf);
}

// Epilogues of the GEMM kernel.
constexpr int kPlain = 0;      // out = product
constexpr int kGatedFwd = 1;   // out = GeLU(x W1) (*) x V on the accumulators (weight = W1^T over V^T)
constexpr int kGateBwd = 2;    // the product is dA; with h | g read from `aux`: out = dA g GeLU'(h) | dA GeLU(h)

template <int kMode, int kNB>   // kNB: 32-row weight blocks per wave (4 or 3); workgroup = 64 * kNB weight rows
__global__ __launch_bounds__(256, 1) void ffn_gemm_kernel(const uint16_t* __restrict__ X, int ldx,
                                                          const uint16_t* __restrict__ W, int ldw, int K,
                                                          int n_tiles, int gate_row, int w_rows, int T_cap,
                                                          const int32_t* __restrict__ meta,
                                                          uint16_t* __restrict__ out, int ldo,
                                                          const uint16_t* __restrict__ aux, int gate_col) {
  constexpr bool kGated = kMode == kGatedFwd;
  static_assert(!kGated || kNB == 4, "the gated epilogue pairs weight blocks 0,1 with 2,3");
  static_assert(kMode != kGateBwd || kNB == 4, "the gate-backward epilogue is written for 64-column passes");
  constexpr int kBN = 64 * kNB;                     // weight rows per workgroup
  constexpr int kStage = (kBM + kBN) * kPitch;      // elements per LDS stage
  constexpr int kLoads = 8 + 2 * kNB;               // 16-byte loads per thread and k step (32 rows per load)
  constexpr int kSlots = 4 * kNB;                   // matrix instructions per sub-step
  constexpr int kFrags = 4 + kNB;                   // fragments per sub-step
  __shared__ __attribute__((aligned(16))) uint16_t smem[2 * kStage];

  // (readfirstlane: tells the compiler the value is wave-uniform, so descriptors built from it stay scalar)
  const int T = __builtin_amdgcn_readfirstlane(meta ? min(meta[0], T_cap) : T_cap);
  // (the grid is sized for T_cap rows; the tile map uses the token panels that hold tokens, so that the
  // idle workgroups are the last ones and not the share of one XCD)
  const int m_tiles = (T + kBM - 1) / kBM;
  if ((int)blockIdx.x >= m_tiles * n_tiles) return;

  // Workgroup -> tile.  Consecutive workgroup ids go round-robin to the 8 XCDs; give every XCD a
  // contiguous run of tiles, walked kGroupM token panels at a time, so that the tiles resident on one
  // XCD share their token panels and weight tiles in that XCD's L2.
  const int total = m_tiles * n_tiles, per = total >> 3;
  int lin = blockIdx.x;
  if (lin < (per << 3)) lin = (lin & 7) * per + (lin >> 3);
  const int group = lin / (kGroupM * n_tiles);
  const int first_m = group * kGroupM;
  const int gsize = min(m_tiles - first_m, kGroupM);
  const int rem = lin - group * (kGroupM * n_tiles);
  // (the divisions run on the vector unit; readfirstlane moves the wave-uniform results back to scalars)
  const int tile_m = __builtin_amdgcn_readfirstlane(first_m + rem % gsize);
  const int tile_n = __builtin_amdgcn_readfirstlane(rem / gsize);
  const int m0 = tile_m * kBM;
  if (m0 >= T) return;
  constexpr int kOutCols = kGated ? kBN / 2 : kBN;    // output columns per workgroup
  const int n0 = tile_n * kOutCols;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int c = lane & 31, g = lane >> 5;
  const int wm = wave >> 1, wn = wave & 1;

  // Global -> LDS staging: a row of a stage is 128 bytes = 8 lanes x 16 bytes; 32 rows per load.
  const int lrow = tid >> 3, lchunk = (tid & 7) * 8;
  // Buffer loads: address = descriptor base + scalar offset + one per-lane offset, so the loads of a
  // step need no vector address arithmetic.  Token rows get one descriptor per load whose extent ends at
  // row T: rows at or beyond T read as zero instead of touching memory that may not exist.  (Byte
  // offsets fit 32 bits: the host checks rows * row length < 2^31 elements.)
  constexpr int kRsrcFlags = 0x00020000;        // raw buffer, 32-bit data format (gfx9 family)
  const uint32_t xlane = ((uint32_t)lrow * (uint32_t)ldx + lchunk) * 2u;
  const uint32_t wlane = ((uint32_t)lrow * (uint32_t)ldw + lchunk) * 2u;
  const __amdgpu_buffer_rsrc_t wrs =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(W), 0, w_rows * ldw * 2, kRsrcFlags);
  // Load i of a step: i < 8 token rows 32 i .., else weight rows 32 (i - 8) .. of the tile (stage row 32 i).
  // (descriptor and offsets are scalar arithmetic on wave-uniform values)
  auto fetch_one = [&](u32x4 (&st)[kLoads], int i, int k0) {
    if (i < 8) {
      const int first = m0 + 32 * i;
      const int rows = __builtin_amdgcn_readfirstlane(max(min(T - first, 32), 0));   // (the clamp is a vector op)
      const __amdgpu_buffer_rsrc_t xrs = __builtin_amdgcn_make_buffer_rsrc(
          const_cast<uint16_t*>(X) + (int64_t)first * ldx, 0, rows * ldx * 2, kRsrcFlags);
      st[i] = __builtin_amdgcn_raw_buffer_load_b128(xrs, xlane, k0 * 2, 0);
    } else {
      const int p = i - 8;
      const int wr = kGated ? (p < 4 ? n0 + 32 * p : gate_row + n0 + 32 * (p - 4)) : n0 + 32 * p;
      st[i] = __builtin_amdgcn_raw_buffer_load_b128(wrs, wlane, (wr * ldw + k0) * 2, 0);
    }
  };
  auto deposit_one = [&](const u32x4 (&st)[kLoads], int i, uint16_t* buf) {
    *reinterpret_cast<u32x4*>(&buf[(32 * i + lrow) * kPitch + lchunk]) = st[i];
  };
  // Two register sets: while one k step is computed, the next one goes from registers to LDS and the two
  // after it are in flight from memory (a load has two whole steps to arrive).
  u32x4 st0[kLoads], st1[kLoads];

  // Fragment rows of this wave inside a stage: tokens at rows 0..255, weight rows from 256 on.
  // Gated: accumulator rows nb = 0,1 are columns of x W1, nb = 2,3 the same columns of x V.
  int xoff[4], woff[kNB];
#pragma unroll
  for (int i = 0; i < 4; ++i) xoff[i] = (wm * 128 + i * 32 + c) * kPitch + g * 8;
#pragma unroll
  for (int i = 0; i < kNB; ++i) {
    const int wr = kGated ? (i >> 1) * 128 + wn * 64 + (i & 1) * 32 : wn * (32 * kNB) + i * 32;
    woff[i] = (kBM + wr + c) * kPitch + g * 8;
  }

  f32x16 acc[kNB][4];
#pragma unroll
  for (int nb = 0; nb < kNB; ++nb)
#pragma unroll
    for (int mb = 0; mb < 4; ++mb)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[nb][mb][v] = 0.f;

  const int nk = K / kBK;                       // even (the host checks K % 128 == 0)
  // (the first two k steps are requested together, so that only one memory latency is exposed)
#pragma unroll
  for (int i = 0; i < kLoads; ++i) fetch_one(st0, i, 0);
#pragma unroll
  for (int i = 0; i < kLoads; ++i) fetch_one(st1, i, kBK);
#pragma unroll
  for (int i = 0; i < kLoads; ++i) deposit_one(st0, i, smem);
#pragma unroll
  for (int i = 0; i < kLoads; ++i) fetch_one(st0, i, min(2, nk - 1) * kBK);
  __syncthreads();

  // One k step = 4 sub-steps of 4 kNB matrix instructions (k = 16 each) on stage `cur`.  Issue order is
  // written out by hand and fenced (with one wave per SIMD nothing but the order hides latencies): in
  // front of every matrix instruction go at most three memory instructions, so that their issue hides
  // under the previous matrix instruction: one LDS read of the NEXT sub-step's fragments
  // (double-buffered) in each of the first slots; in sub-step 0 the LDS writes that move register set
  // `st` (tile kt + 1) to stage `nxt`; in sub-step 1 the global loads that refill `st` with tile
  // kt + 3.  The workgroup barrier sits before sub-step 3: by then this wave has read all of `cur` and
  // written its share of `nxt`, so sub-step 3 already reads the first fragments of `nxt`, and the next
  // step may overwrite `cur`.  No branches: the last steps fetch a clamped, redundant tile and deposit
  // it where nobody reads.
  bf16x8 wf[2][kNB], xf[2][4];
  // Fragment i of sub-step kk: i = 0..3 token fragments, then the weight fragments.
  auto read_frag = [&](const uint16_t* stage_ptr, int kk, int buf, int i) {
    if (i < 4) xf[buf][i] = lds_read8(stage_ptr + xoff[i] + kk * 16);
    else wf[buf][i - 4] = lds_read8(stage_ptr + woff[i - 4] + kk * 16);
  };
#pragma unroll
  for (int i = 0; i < kFrags; ++i) read_frag(smem, 0, 0, i);
  auto step = [&](const uint16_t* cur, uint16_t* nxt, u32x4 (&st)[kLoads], int k_fetch) {
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      if (kk == 3) __syncthreads();
#pragma unroll
      for (int q = 0; q < kNB; ++q) {
#pragma unroll
        for (int mb = 0; mb < 4; ++mb) {
          const int slot = 4 * q + mb;
          if (slot < kFrags) {
            if (kk < 3) read_frag(cur, kk + 1, (kk + 1) & 1, slot);
            else read_frag(nxt, 0, 0, slot);
          }
#pragma unroll
          for (int i = slot; i < kLoads; i += kSlots) {
            if (kk == 0) deposit_one(st, i, nxt);
            if (kk == 1) fetch_one(st, i, k_fetch);
          }
          __builtin_amdgcn_sched_barrier(0);
          acc[q][mb] = mfma32(wf[kk & 1][q], xf[kk & 1][mb], acc[q][mb]);
          __builtin_amdgcn_sched_barrier(0);
        }
      }
    }
  };
  for (int kt = 0; kt < nk; kt += 2) {
    step(smem, smem + kStage, st1, min(kt + 3, nk - 1) * kBK);
    step(smem + kStage, smem, st0, min(kt + 4, nk - 1) * kBK);
  }
  __syncthreads();

  // Epilogue: through a wave-private slab of 128 tokens x 64 columns (both stages are free now), two
  // 32-column accumulator blocks at a time (the last pass of an odd kNB has one).
  uint16_t* slab = smem + wave * (128 * kPitch);
  const int row_base = m0 + wm * 128;
  constexpr int kOutBlocks = kGated ? 2 : kNB;      // 32-column output blocks per wave
#pragma unroll
  for (int b0 = 0; b0 < kOutBlocks; b0 += 2) {
    constexpr int kTwo = 2;
    const int nblk = (kOutBlocks - b0) < kTwo ? (kOutBlocks - b0) : kTwo;
    // Gate backward: the h and g values this lane will combine with dA are requested before the
    // accumulators go through the slab, so that they arrive meanwhile (the staging registers of the k
    // loop are free now).
    u32x4 hpre[kMode == kGateBwd ? 16 : 1], gpre[kMode == kGateBwd ? 16 : 1];
    if (kMode == kGateBwd) {
      const int orow = lane >> 3, ocol = (lane & 7) * 8;
      const int colp = n0 + wn * (32 * kOutBlocks) + b0 * 32 + ocol;
#pragma unroll
      for (int it = 0; it < 16; ++it) {
        const int row = row_base + 8 * it + orow;
        hpre[it] = gpre[it] = u32x4{0u, 0u, 0u, 0u};
        if (row < T) {
          const int64_t at = (int64_t)row * ldo + colp;
          hpre[it] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(aux + at));
          gpre[it] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(aux + at + gate_col));
        }
      }
    }
#pragma unroll
    for (int nb = 0; nb < 2; ++nb) {
      if (nb < nblk) {
#pragma unroll
        for (int mb = 0; mb < 4; ++mb) {
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            float r[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
              if (kGated) r[i] = gelu_exact(acc[nb][mb][4 * j + i]) * acc[nb + 2][mb][4 * j + i];
              else r[i] = acc[b0 + nb][mb][4 * j + i];
            }
            u32x2 w;
            w[0] = pack_bf16(r[0], r[1]);
            w[1] = pack_bf16(r[2], r[3]);
            *reinterpret_cast<u32x2*>(&slab[(mb * 32 + c) * kPitch + nb * 32 + 8 * j + 4 * g]) = w;
          }
        }
      }
    }
    // (same wave wrote and reads the slab: LDS operations of one wave complete in order)
    const int col0 = n0 + wn * (32 * kOutBlocks) + b0 * 32;
    if (nblk == 2) {                // rows of 64 columns = 128 bytes = 8 lanes
      const int orow = lane >> 3, ocol = (lane & 7) * 8;
#pragma unroll
      for (int it = 0; it < 16; ++it) {
        const int row = 8 * it + orow;
        const u32x4 w = *reinterpret_cast<const u32x4*>(&slab[row * kPitch + ocol]);
        if (row_base + row < T) {
          const int64_t at = (int64_t)(row_base + row) * ldo + col0 + ocol;
          if (kMode == kGateBwd) {
            // w holds 8 values of dA; h and g of the same positions came from aux (columns col and
            // gate_col + col of a row); dh and dg go to the same two places of out
            const u32x4 hv = hpre[kMode == kGateBwd ? it : 0], gv = gpre[kMode == kGateBwd ? it : 0];
            u32x4 dh, dg;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
              float v0, d0, v1, d1;
              gelu_and_grad(__uint_as_float(hv[i] << 16), v0, d0);
              gelu_and_grad(__uint_as_float(hv[i] & 0xffff0000u), v1, d1);
              const float a0 = __uint_as_float(w[i] << 16), a1 = __uint_as_float(w[i] & 0xffff0000u);
              const float g0 = __uint_as_float(gv[i] << 16), g1 = __uint_as_float(gv[i] & 0xffff0000u);
              dh[i] = pack_bf16(a0 * g0 * d0, a1 * g1 * d1);
              dg[i] = pack_bf16(a0 * v0, a1 * v1);
            }
            *reinterpret_cast<u32x4*>(out + at) = dh;
            *reinterpret_cast<u32x4*>(out + at + gate_col) = dg;
          } else {
            *reinterpret_cast<u32x4*>(out + at) = w;
          }
        }
      }
    } else {                        // rows of 32 columns = 64 bytes = 4 lanes
      const int orow = lane >> 2, ocol = (lane & 3) * 8;
#pragma unroll
      for (int it = 0; it < 8; ++it) {
        const int row = 16 * it + orow;
        const u32x4 w = *reinterpret_cast<const u32x4*>(&slab[row * kPitch + ocol]);
        if (row_base + row < T) *reinterpret_cast<u32x4*>(out + (int64_t)(row_base + row) * ldo + col0 + ocol) = w;
      }
    }
  }
}

// a = GeLU(h) (*) g, elementwise over [T, inter]: the separate activation pass of the unfused arrangements
// (the fused path above never runs it).  One 16-byte piece of h and of g per thread; HBM-bound.
__global__ __launch_bounds__(256) void gelu_gate_kernel(const uint16_t* __restrict__ h,
                                                        const uint16_t* __restrict__ gate, int64_t ld, int T_cap,
                                                        const int32_t* __restrict__ meta, int inter,
                                                        uint16_t* __restrict__ act) {
  const int T = meta ? min(meta[0], T_cap) : T_cap;
  const int pieces = inter >> 3;
  const int64_t total = (int64_t)T * pieces;
  for (int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; idx < total;
       idx += (int64_t)gridDim.x * blockDim.x) {
    const int64_t row = idx / pieces;
    const int col = (int)(idx - row * pieces) * 8;
    const u32x4 hv = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(h + row * ld + col));
    const u32x4 gv = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(gate + row * ld + col));
    u32x4 r;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const float h0 = __uint_as_float(hv[i] << 16), h1 = __uint_as_float(hv[i] & 0xffff0000u);
      const float g0 = __uint_as_float(gv[i] << 16), g1 = __uint_as_float(gv[i] & 0xffff0000u);
      r[i] = pack_bf16(gelu_exact(h0) * g0, gelu_exact(h1) * g1);
    }
    *reinterpret_cast<u32x4*>(act + row * (int64_t)inter + col) = r;
  }
}

// ------------------------------------------------------------------------------------------------ weight gradients
// partial[split][m, n] = sum over the split's tokens t of P[t, m] * Q[t, n]: both operands are stored
// token-major, so the contraction runs over ROWS.  Rows of 256 columns go to LDS as they are and the
// matrix-core operands (8 consecutive tokens of one column per lane) come out of transposing LDS reads
// (ds_read_b64_tr_b16).  The accumulator has m along registers and n along lanes, so a store instruction
// writes 128 contiguous bytes of two output rows: fp32 partial tiles need no staging.  Tokens are split
// over `splits` workgroups per tile (there are only M/256 x N/256 tiles); a second kernel adds the
// partial tiles in a fixed order, so the result is deterministic.
constexpr int kWgPitch = 272;                       // LDS row pitch of a 256-column token row, elements (544 B)
constexpr int kWgRows = 64;                         // tokens per k step
constexpr int kWgStage = 2 * kWgRows * kWgPitch;    // P rows + Q rows

__global__ __launch_bounds__(256, 1) void ffn_wgrad_kernel(const uint16_t* __restrict__ P, int ldp,
                                                           const uint16_t* __restrict__ Q, int ldq, int n_tiles,
                                                           int tiles, int splits, int T_cap,
                                                           const int32_t* __restrict__ meta,
                                                           float* __restrict__ partial, int M, int N) {
  __shared__ __attribute__((aligned(16))) uint16_t smem[2 * kWgStage];
  const int T = __builtin_amdgcn_readfirstlane(meta ? min(meta[0], T_cap) : T_cap);
  const int tile = blockIdx.x % tiles, split = blockIdx.x / tiles;
  const int m0 = __builtin_amdgcn_readfirstlane(tile / n_tiles) * 256;
  const int n0 = __builtin_amdgcn_readfirstlane(tile % n_tiles) * 256;
  // k steps of this split: the same even number for every split (the k loop alternates two register
  // sets); steps past the last token read zeros and add nothing
  const int steps_total = (T + kWgRows - 1) / kWgRows;
  const int per = (((steps_total + splits - 1) / splits) + 1) & ~1;
  const int s_begin = split * per;
  const int nsteps = s_begin < steps_total ? per : 0;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int c = lane & 31, g = lane >> 5;
  const int wm = wave >> 1, wn = wave & 1;
  const int lrow = tid >> 5, lchunk = (tid & 31) * 8;   // a row of 256 columns = 32 lanes x 16 bytes; 8 rows per pass
  constexpr int kRsrcFlags = 0x00020000;
  const uint32_t plane = ((uint32_t)lrow * (uint32_t)ldp + lchunk) * 2u;
  const uint32_t qlane = ((uint32_t)lrow * (uint32_t)ldq + lchunk) * 2u;
  // Load i of a step (i < 8: rows 8 i .. of P, else of Q).  The descriptor ends with the last token row,
  // so the rows past T read as zeros and add nothing.
  auto fetch_one = [&](u32x4 (&st)[16], int i, int t0) {
    const int p = i & 7;
    const int first = t0 + 8 * p;
    const int rows = __builtin_amdgcn_readfirstlane(max(min(T - first, 8), 0));
    if (i < 8) {
      const __amdgpu_buffer_rsrc_t r = __builtin_amdgcn_make_buffer_rsrc(
          const_cast<uint16_t*>(P) + (int64_t)first * ldp + m0, 0, rows > 0 ? ((rows - 1) * ldp + 256) * 2 : 0,
          kRsrcFlags);
      st[i] = __builtin_amdgcn_raw_buffer_load_b128(r, plane, 0, 0);
    } else {
      const __amdgpu_buffer_rsrc_t r = __builtin_amdgcn_make_buffer_rsrc(
          const_cast<uint16_t*>(Q) + (int64_t)first * ldq + n0, 0, rows > 0 ? ((rows - 1) * ldq + 256) * 2 : 0,
          kRsrcFlags);
      st[i] = __builtin_amdgcn_raw_buffer_load_b128(r, qlane, 0, 0);
    }
  };
  uint16_t* const dep[2] = {smem + lrow * kWgPitch + lchunk, smem + kWgStage + lrow * kWgPitch + lchunk};
  auto deposit_one = [&](const u32x4 (&st)[16], int i, int stage) {
    *reinterpret_cast<u32x4*>(dep[stage] + ((i < 8 ? 0 : kWgRows) + 8 * (i & 7)) * kWgPitch) = st[i];
  };
  u32x4 st0[16], st1[16];

  f32x16 acc[4][4];   // [m block][n block]
#pragma unroll
  for (int a = 0; a < 4; ++a)
#pragma unroll
    for (int b = 0; b < 4; ++b)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.f;

  const int tr_i = lane & 15, tr_q = lane >> 4;
  const int tr_row = (tr_i >> 2) + 4 * (tr_q >> 1);
  const int tr_col = 16 * (tr_q & 1) + 4 * (tr_i & 3);
  const int poff = tr_row * kWgPitch + wm * 128 + tr_col;
  const int qoff = (kWgRows + tr_row) * kWgPitch + wn * 128 + tr_col;

  if (nsteps > 0) {
    const int t_first = s_begin * kWgRows;
#pragma unroll
    for (int i = 0; i < 16; ++i) fetch_one(st0, i, t_first);
#pragma unroll
    for (int i = 0; i < 16; ++i) fetch_one(st1, i, t_first + kWgRows);
#pragma unroll
    for (int i = 0; i < 16; ++i) deposit_one(st0, i, 0);
#pragma unroll
    for (int i = 0; i < 16; ++i) fetch_one(st0, i, t_first + 2 * kWgRows);
    __syncthreads();

    // Same hand-ordered k step as the projection kernel: per sub-step 16 matrix instructions, each
    // preceded by at most two memory instructions (fragment reads of the next sub-step, double-buffered;
    // LDS writes of the next step in sub-step 0; global loads of the step after next in sub-step 1), the
    // barrier before sub-step 3.
    bf16x8 pf[2][4], qf[2][4];
    auto read_frag = [&](const uint16_t* stage_ptr, int kk, int buf, int i) {   // i = 0..3 P blocks, 4..7 Q blocks
      const uint16_t* p = stage_ptr + (i < 4 ? poff : qoff) + 16 * kk * kWgPitch + 32 * (i & 3);
      const bf16x8 f = join_tr(lds_read_tr4(p), lds_read_tr4(p + 8 * kWgPitch));
      if (i < 4) pf[buf][i] = f;
      else qf[buf][i - 4] = f;
    };
#pragma unroll
    for (int i = 0; i < 8; ++i) read_frag(smem, 0, 0, i);
    auto step = [&](int cur_stage, u32x4 (&st)[16], int t_fetch) {
      const uint16_t* cur = smem + cur_stage * kWgStage;
      const uint16_t* nxt = smem + (cur_stage ^ 1) * kWgStage;
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) {
        if (kk == 3) __syncthreads();
#pragma unroll
        for (int a = 0; a < 4; ++a) {
#pragma unroll
          for (int b = 0; b < 4; ++b) {
            const int slot = 4 * a + b;
            if (slot < 8) {
              if (kk < 3) read_frag(cur, kk + 1, (kk + 1) & 1, slot);
              else read_frag(nxt, 0, 0, slot);
            }
            if (kk == 0) deposit_one(st, slot, cur_stage ^ 1);
            if (kk == 1) fetch_one(st, slot, t_fetch);
            __builtin_amdgcn_sched_barrier(0);
            acc[a][b] = mfma32(pf[kk & 1][a], qf[kk & 1][b], acc[a][b]);
            __builtin_amdgcn_sched_barrier(0);
          }
        }
      }
    };
    for (int kt = 0; kt < nsteps; kt += 2) {
      step(0, st1, t_first + (kt + 3) * kWgRows);
      step(1, st0, t_first + (kt + 4) * kWgRows);
    }
  }
  // fp32 partial tile: register v of block (a, b) is row 8 (v / 4) + 4 g + v % 4, lane c is the column
  float* dst = partial + (int64_t)split * M * N + (int64_t)(m0 + wm * 128) * N + n0 + wn * 128 + c;
#pragma unroll
  for (int a = 0; a < 4; ++a)
#pragma unroll
    for (int b = 0; b < 4; ++b)
#pragma unroll
      for (int v = 0; v < 16; ++v)
        dst[(int64_t)(a * 32 + 8 * (v >> 2) + 4 * g + (v & 3)) * N + b * 32] = acc[a][b][v];
}

// out[i] = sum over splits of partial[s][i], in order.
__global__ __launch_bounds__(256) void ffn_wgrad_reduce_kernel(const float* __restrict__ partial, int splits,
                                                               int64_t count4, float* __restrict__ out) {
  const float4* src = reinterpret_cast<const float4*>(partial);
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < count4; i += (int64_t)gridDim.x * blockDim.x) {
    float4 a = src[i];
    for (int s = 1; s < splits; ++s) {
      const float4 b = src[(int64_t)s * count4 + i];
      a.x += b.x; a.y += b.y; a.z += b.z; a.w += b.w;
    }
    reinterpret_cast<float4*>(out)[i] = a;
  }
}

// out[c][r] = in[r][c] for a [R, C] bf16 matrix (R, C multiples of 64): 64 x 64 tiles through LDS.
__global__ __launch_bounds__(256) void transpose_kernel(const uint16_t* __restrict__ in, int R, int C,
                                                        uint16_t* __restrict__ out) {
  __shared__ uint16_t tile[64][66];
  const int r0 = blockIdx.y * 64, c0 = blockIdx.x * 64;
  const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
#pragma unroll
  for (int i = 0; i < 16; ++i) tile[4 * i + ty][tx] = in[(int64_t)(r0 + 4 * i + ty) * C + c0 + tx];
  __syncthreads();
#pragma unroll
  for (int i = 0; i < 16; ++i) out[(int64_t)(c0 + 4 * i + ty) * R + r0 + tx] = tile[tx][4 * i + ty];
}

}  // namespace

// out[t, n] = sum_k x[t, k] * wt[n, k] with the plain epilogue; the tile width (256 or 192 weight rows) is the
// one that wastes less of the last round of workgroups on the 256 compute units.
static void launch_plain(const void* x, const void* wt, int T_cap, const int32_t* meta, int n_in, int n_out, void* y,
                         hipStream_t stream) {
  const int m_tiles = (T_cap + kBM - 1) / kBM;
  const auto cost = [&](int bn) {
    const int tiles = m_tiles * (n_out / bn);
    return (double)((tiles + 255) / 256) * bn;
  };
  const bool narrow = n_out % 192 == 0 && (n_out % 256 != 0 || cost(192) < cost(256));
  if (narrow) {
    const int n_tiles = n_out / 192;
    ffn_gemm_kernel<kPlain, 3><<<dim3(m_tiles * n_tiles), dim3(256), 0, stream>>>(
        static_cast<const uint16_t*>(x), n_in, static_cast<const uint16_t*>(wt), n_in, n_in, n_tiles, 0, n_out, T_cap,
        meta, static_cast<uint16_t*>(y), n_out, nullptr, 0);
  } else {
    const int n_tiles = n_out / 256;
    ffn_gemm_kernel<kPlain, 4><<<dim3(m_tiles * n_tiles), dim3(256), 0, stream>>>(
        static_cast<const uint16_t*>(x), n_in, static_cast<const uint16_t*>(wt), n_in, n_in, n_tiles, 0, n_out, T_cap,
        meta, static_cast<uint16_t*>(y), n_out, nullptr, 0);
  }
}

mb_status launch_geglu_fwd(const void* x, const void* w1v, const void* w2, int T_cap, const int32_t* meta,
                           int hidden, int inter, void* act, void* y, hipStream_t stream) {
  if (T_cap == 0) return MB_OK;
  const int m_tiles = (T_cap + kBM - 1) / kBM;
  const int n_tiles = inter / 128;
  ffn_gemm_kernel<kGatedFwd, 4><<<dim3(m_tiles * n_tiles), dim3(256), 0, stream>>>(
      static_cast<const uint16_t*>(x), hidden, static_cast<const uint16_t*>(w1v), hidden, hidden, n_tiles, inter,
      2 * inter, T_cap, meta, static_cast<uint16_t*>(act), inter, nullptr, 0);
  launch_plain(act, w2, T_cap, meta, inter, hidden, y, stream);
  return check_launch("ffn_gemm_kernel");
}

mb_status launch_linear_fwd(const void* x, const void* wt, int T_cap, const int32_t* meta, int n_in, int n_out,
                            void* y, hipStream_t stream) {
  if (T_cap == 0) return MB_OK;
  launch_plain(x, wt, T_cap, meta, n_in, n_out, y, stream);
  return check_launch("ffn_gemm_kernel");
}

mb_status launch_gelu_gate(const void* h, const void* gate, int64_t ld, int T_cap, const int32_t* meta, int inter,
                           void* act, hipStream_t stream) {
  if (T_cap == 0) return MB_OK;
  const int64_t pieces = (int64_t)T_cap * (inter >> 3);
  const int blocks = (int)((pieces + 255) / 256 < 8192 ? (pieces + 255) / 256 : 8192);
  gelu_gate_kernel<<<dim3(blocks), dim3(256), 0, stream>>>(static_cast<const uint16_t*>(h),
                                                           static_cast<const uint16_t*>(gate), ld, T_cap, meta, inter,
                                                           static_cast<uint16_t*>(act));
  return check_launch("gelu_gate_kernel");
}

// Workspace of the backward: h|g recomputed, dh|dg, the two transposed weight matrices, the partial
// weight-gradient tiles.
static constexpr int kWgradSplits = 7;
static size_t bwd_ws_layout(int T_cap, int hidden, int inter, size_t off[5]) {
  size_t at = 0;
  const size_t rows = (size_t)T_cap * 2 * inter * 2;
  off[0] = at; at += align_up(rows, 256);                                   // hg   [T_cap, 2 inter] bf16
  off[1] = at; at += align_up(rows, 256);                                   // dhg  [T_cap, 2 inter] bf16
  off[2] = at; at += align_up((size_t)inter * hidden * 2, 256);             // w2 transposed [inter, hidden]
  off[3] = at; at += align_up((size_t)2 * inter * hidden * 2, 256);         // w1v transposed [hidden, 2 inter]
  off[4] = at; at += align_up((size_t)kWgradSplits * 2 * inter * hidden * 4, 256);   // partial tiles, fp32
  return at;
}

size_t geglu_bwd_workspace_bytes(int T_cap, int hidden, int inter) {
  size_t off[5];
  return bwd_ws_layout(T_cap, hidden, inter, off);
}

static void launch_wgrad(const void* p, int ldp, const void* q, int ldq, int M, int N, int T_cap, const int32_t* meta,
                         float* partial, float* out, hipStream_t stream) {
  const int n_tiles = N / 256, tiles = (M / 256) * n_tiles;
  ffn_wgrad_kernel<<<dim3(tiles * kWgradSplits), dim3(256), 0, stream>>>(
      static_cast<const uint16_t*>(p), ldp, static_cast<const uint16_t*>(q), ldq, n_tiles, tiles, kWgradSplits, T_cap,
      meta, partial, M, N);
  const int64_t count4 = (int64_t)M * N / 4;
  ffn_wgrad_reduce_kernel<<<dim3(1024), dim3(256), 0, stream>>>(partial, kWgradSplits, count4, out);
}

mb_status launch_geglu_bwd(const void* dy, const void* x, const void* w1v, const void* w2, const void* act,
                           const void* hg_saved, int T_cap, const int32_t* meta, int hidden, int inter, void* dx,
                           float* dw1v, float* dw2, void* workspace, hipStream_t stream) {
  size_t off[5];
  bwd_ws_layout(T_cap, hidden, inter, off);
  char* ws = static_cast<char*>(workspace);
  const uint16_t* hg = hg_saved ? static_cast<const uint16_t*>(hg_saved) : reinterpret_cast<uint16_t*>(ws + off[0]);
  uint16_t* dhg = reinterpret_cast<uint16_t*>(ws + off[1]);
  uint16_t* w2t = reinterpret_cast<uint16_t*>(ws + off[2]);
  uint16_t* w1vt = reinterpret_cast<uint16_t*>(ws + off[3]);
  float* partial = reinterpret_cast<float*>(ws + off[4]);
  // the weight matrices the data gradients contract over their OTHER index
  transpose_kernel<<<dim3(inter / 64, hidden / 64), dim3(256), 0, stream>>>(static_cast<const uint16_t*>(w2), hidden,
                                                                           inter, w2t);
  transpose_kernel<<<dim3(hidden / 64, 2 * inter / 64), dim3(256), 0, stream>>>(static_cast<const uint16_t*>(w1v),
                                                                               2 * inter, hidden, w1vt);
  if (T_cap > 0) {
    const int m_tiles = (T_cap + kBM - 1) / kBM;
    // h | g = x (W1 | V): handed over by a caller that stored it, else computed again
    if (!hg_saved) launch_plain(x, w1v, T_cap, meta, hidden, 2 * inter, ws + off[0], stream);
    // dA = dy W2^T, and on its way out  dh = dA g GeLU'(h),  dg = dA GeLU(h)
    ffn_gemm_kernel<kGateBwd, 4><<<dim3(m_tiles * (inter / 256)), dim3(256), 0, stream>>>(
        static_cast<const uint16_t*>(dy), hidden, w2t, hidden, hidden, inter / 256, 0, inter, T_cap, meta, dhg,
        2 * inter, hg, inter);
    // dx = dh W1^T + dg V^T = (dh | dg) (W1 | V)^T
    launch_plain(dhg, w1vt, T_cap, meta, 2 * inter, hidden, dx, stream);
  }
  // dW2^T[c, j] = sum_t dy[t, c] act[t, j];   d(W1|V)^T[j, c] = sum_t (dh|dg)[t, j] x[t, c]
  launch_wgrad(dy, hidden, act, inter, hidden, inter, T_cap, meta, partial, dw2, stream);
  launch_wgrad(dhg, 2 * inter, x, hidden, 2 * inter, hidden, T_cap, meta, partial, dw1v, stream);
  return check_launch("geglu backward");
}

}  // namespace mb
