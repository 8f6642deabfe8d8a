// Work plan of the any-length attention kernels (forward, dK/dV, dQ): which workgroup does which
// (sequence, head, tile of 128 tokens), decided on the device from cu_seqlens, with no host round trip.
//
// Why a plan.  The chip has 8 XCDs (32 compute units and one L2 each) and hands the workgroups of a launch to
// them round robin: workgroup i runs on XCD i % 8 (measured with per-workgroup timestamps), and each XCD works
// through its share in launch order.  A grid laid out as (tile, head, sequence) therefore ties the XCD to the tile
// index: on ragged batches some XCDs receive mostly tiles that do not exist and finish in half the time of the
// others, and the tiles of one (sequence, head), which all stream the same K and V rows, land on different L2s.
// The plan deals the work explicitly:
//   * units are (sequence, head) pairs, sequences ranked longest first (ties by index; B <= kSortMaxB, else in
//     the order given); pair p = rank * H + head goes to XCD s(p % 16), s = 0..7,7..0 (boustrophedon, so that no
//     XCD always receives the longer neighbour);
//   * XCD c owns the list plan.items[c][0 .. count[c]): its pairs in that order, each followed by all its tiles,
//     so that an XCD starts its heaviest work first, short work fills the tail, and the tiles that share K / V
//     rows run on one L2 at about the same time;
//   * the launch is one-dimensional with 8 * cap workgroups; workgroup i reads item (i / 8) of list (i % 8) and
//     leaves at once if the list is shorter.
// The plan depends on cu_seqlens, H and max_seqlen only: the same plan serves all three kernels, and results do
// not depend on it (every output element is produced by exactly one workgroup, in a fixed order of operations).
#pragma once
#include "common.h"

namespace mb {

static constexpr int kPlanTile = 128;       // tokens per work item (queries of the forward and of dQ, keys of dK/dV)
static constexpr int kPlanXcds = 8;
static constexpr int kPlanThreads = 256;    // workgroup size of the code that builds a plan
static constexpr int kSortMaxB = 512;       // sequences ranked by length (also the ranks handled per pass)

// One work item, 16 bytes: first packed token and length of the sequence, tile index and head, and how many of
// the sequence's tokens act as keys (the length itself unless the call limits the keys).
struct __attribute__((aligned(16))) PlanItem {
  int32_t start, n, tile_head /* tile | head << 16 */, nk;
};

// Number of pairs p in [0, n) dealt to XCD c:  p % 16 == c  or  p % 16 == 15 - c.
__host__ __device__ inline int64_t plan_pairs_before(int64_t n, int c) {
  const int r = (int)(n & 15);
  return 2 * (n >> 4) + (r > c ? 1 : 0) + (r > 15 - c ? 1 : 0);
}

// Items each XCD's list can hold: the pairs one XCD can receive, every one with the most tiles a sequence may have.
__host__ inline int64_t attn_plan_cap(int B, int max_seqlen, int H) {
  const int64_t pairs = (int64_t)B * H;
  const int64_t tiles = ((int64_t)max_seqlen + kPlanTile - 1) / kPlanTile;
  return 2 * ((pairs + 15) / 16) * tiles;
}
// Bytes of a plan: 8 counts (32 bytes), then 8 lists of `cap` items.
__host__ inline size_t attn_plan_bytes(int B, int max_seqlen, int H) {
  return align_up(32 + (size_t)kPlanXcds * (size_t)attn_plan_cap(B, max_seqlen, H) * sizeof(PlanItem), 256);
}

struct PlanLds {
  uint32_t keys[kSortMaxB + 16];
  int32_t start[kSortMaxB];
  int32_t len[kSortMaxB];
  int32_t klen[kSortMaxB];
  int32_t off[kSortMaxB];
  int32_t wave_sum[kPlanThreads / 64];
  int32_t carry;
};

// Builds list `c` of the plan.  Called by all kPlanThreads threads of one workgroup (contains barriers).
// A sequence longer than max_seqlen gets no items (it is skipped as a whole) and raises the misuse flag; a
// sequence without keys (key_lens[b] <= 0) gets none either.
__device__ inline void build_plan_list(const int32_t* __restrict__ cu, const int32_t* __restrict__ key_lens, int B, int H,
                                       int max_seqlen, int64_t cap, int32_t* __restrict__ plan, int c,
                                       int32_t* __restrict__ misuse, PlanLds& L) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  PlanItem* __restrict__ items = reinterpret_cast<PlanItem*>(plan + 8) + (int64_t)c * cap;
  if (tid == 0) L.carry = 0;
  for (int r0 = 0; r0 < B; r0 += kSortMaxB) {
    const int nb = min(kSortMaxB, B - r0);
    __syncthreads();   // previous pass is done with the staging arrays; L.carry is visible
    if (B <= kSortMaxB) {
      // rank by (length, reversed index): longest first, ties by index.  Global memory is read once (all loads of
      // a thread in flight together); the ranking then works from LDS and registers.
      const int Bp = (B + 15) & ~15;
      int my_s0[kSortMaxB / kPlanThreads], my_len[kSortMaxB / kPlanThreads], my_kl[kSortMaxB / kPlanThreads];
#pragma unroll
      for (int u = 0; u < kSortMaxB / kPlanThreads; ++u) {
        const int i = tid + u * kPlanThreads;
        my_s0[u] = my_len[u] = my_kl[u] = 0;
        if (i < Bp) {
          const int s0 = cu[min(i, B)], s1 = cu[min(i + 1, B)];
          const int kl = (key_lens && i < B) ? key_lens[i] : (1 << 30);
          my_s0[u] = s0;
          my_len[u] = s1 - s0;
          my_kl[u] = min(kl, s1 - s0);
          L.keys[i] = i < B ? ((uint32_t)min(s1 - s0, (1 << 22)) << 9) | (uint32_t)(kSortMaxB - 1 - i) : 0u;
        }
      }
      __syncthreads();
#pragma unroll
      for (int u = 0; u < kSortMaxB / kPlanThreads; ++u) {
        const int cand = tid + u * kPlanThreads;
        if (cand < B) {
          const uint32_t mine = L.keys[cand];
          int r = 0;
          for (int other = 0; other < Bp; other += 4) {
            const uint4 k4 = *reinterpret_cast<const uint4*>(&L.keys[other]);
            r += (k4.x > mine ? 1 : 0) + (k4.y > mine ? 1 : 0) + (k4.z > mine ? 1 : 0) + (k4.w > mine ? 1 : 0);
          }
          L.start[r] = my_s0[u];
          L.len[r] = my_kl[u] > 0 ? my_len[u] : 0;   // no keys: nothing to compute
          L.klen[r] = my_kl[u];
        }
      }
    } else {
      for (int i = tid; i < nb; i += kPlanThreads) {
        const int s0 = cu[r0 + i];
        const int len = cu[r0 + i + 1] - s0;
        const int kl = key_lens ? min(key_lens[r0 + i], len) : len;
        L.start[i] = s0;
        L.len[i] = kl > 0 ? len : 0;
        L.klen[i] = kl;
      }
    }
    __syncthreads();
    // tiles of every rank that land on this XCD, and their exclusive prefix sum (two ranks per thread)
    int w[2];
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      const int i = 2 * tid + u;
      w[u] = 0;
      if (i < nb) {
        const int len = L.len[i];
        if (len > max_seqlen) raise_misuse(misuse);
        const int tiles = len > max_seqlen ? 0 : (len + kPlanTile - 1) / kPlanTile;
        const int64_t p0 = (int64_t)(r0 + i) * H;
        w[u] = tiles * (int)(plan_pairs_before(p0 + H, c) - plan_pairs_before(p0, c));
      }
    }
    int incl = w[0] + w[1];
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
      const int up = __shfl_up(incl, d, 64);
      if (lane >= d) incl += up;
    }
    if (lane == 63) L.wave_sum[wave] = incl;
    __syncthreads();
    int base = L.carry;
    for (int v = 0; v < wave; ++v) base += L.wave_sum[v];
    const int excl = base + incl - (w[0] + w[1]);
    if (2 * tid < nb) L.off[2 * tid] = excl;
    if (2 * tid + 1 < nb) L.off[2 * tid + 1] = excl + w[0];
    __syncthreads();
    if (tid == kPlanThreads - 1) L.carry = base + incl;   // read by everyone after the next barrier
    // the pairs of these ranks that are dealt to this XCD, one thread each
    const int64_t i_end = plan_pairs_before((int64_t)(r0 + nb) * H, c);
    for (int64_t i = plan_pairs_before((int64_t)r0 * H, c) + tid; i < i_end; i += kPlanThreads) {
      const int64_t p = 16 * (i >> 1) + ((i & 1) ? 15 - c : c);
      const int r = (int)(p / H), h = (int)(p - (int64_t)r * H);
      const int len = L.len[r - r0];
      if (len <= 0 || len > max_seqlen) continue;
      const int tiles = (len + kPlanTile - 1) / kPlanTile;
      const int at = L.off[r - r0] + tiles * (int)(i - plan_pairs_before((int64_t)r * H, c));
      PlanItem it;
      it.start = L.start[r - r0];
      it.n = len;
      it.nk = L.klen[r - r0];
      for (int x = 0; x < tiles; ++x) {
        it.tile_head = x | (h << 16);
        items[at + x] = it;
      }
    }
  }
  __syncthreads();
  if (tid == 0) plan[c] = L.carry;
}

// What a kernel's workgroup reads: its item, or nothing.  i = workgroup index of a launch of 8 * cap workgroups.
__device__ __forceinline__ bool plan_fetch(const int32_t* __restrict__ plan, int64_t cap, int* start, int* n, int* nk,
                                           int* tile, int* head) {
  const int c = blockIdx.x & (kPlanXcds - 1);
  const int j = blockIdx.x >> 3;
  const int count = plan[c];
  const int4 it = *(reinterpret_cast<const int4*>(plan + 8) + (int64_t)c * cap + j);   // j < cap always: in bounds
  if (j >= count) return false;
  *start = __builtin_amdgcn_readfirstlane(it.x);
  *n = __builtin_amdgcn_readfirstlane(it.y);
  *nk = __builtin_amdgcn_readfirstlane(it.w);
  *tile = __builtin_amdgcn_readfirstlane(it.z) & 0xffff;
  *head = (int)((uint32_t)__builtin_amdgcn_readfirstlane(it.z) >> 16);
  return true;
}

}  // namespace mb
