// Device code of a2a_sssp_loads: the single-path "SSSP" baseline of Sec. 5.2 (a heuristic that
// computes shortest paths iteration by iteration through a graph whose link weights reflect the
// congestion the earlier iterations caused).  Included once, by a2a_topo.hip, after a2a_kernels.h.
//
// One iteration = one group of batches (64 sources each): the BFS of a2a_kernels.h gives the level
// masks L_l[v]; then, level by level, every (source, node) pair picks the in-link of least
// cost(s,u) + W[link] among the links from the level before (ties: lowest link id), W being the
// link loads when the iteration started; then, deepest level first, every pair hands the number of
// paths that end in or pass through it (1 + what its successors handed it) to the link it picked.
// All integers: the order of additions does not matter, loads are exact.
//
// Layout per batch: dense 64-wide rows, lane j = source j of the batch, row v = node v:
// cost int64[Npad][64], pick int32[Npad][64] (id of the chosen link into v), sub int32[Npad][64].
// Only the lanes in L_l[v] of a row are ever written or read.
#pragma once

#include "a2a_kernels.h"

namespace a2a_dev {

struct SsspView {
  long long* cost;              // [G][Npad][64]
  int* pick;                    // [G][Npad][64]
  int* sub;                     // [G][Npad][64]
  unsigned long long* iload;    // [Epad] paths routed over each link so far (this call)
};

__device__ __forceinline__ uint64_t level_mask(const GroupView& gv, int g, int level, int v) {
  return gv.bm[bm_at(gv, g / kSub, level, v, g % kSub)];
}

// cost and chosen in-link of the pairs on `level` (>= 1).  A wave takes 64 consecutive nodes of one
// batch and visits those that have sources on the level; in-links in list order = ascending link id,
// so the strict comparison keeps the lowest id among equals.
__global__ void __launch_bounds__(kBlock)
k_sssp_fwd(const int32_t* __restrict__ in_ptr, const int32_t* __restrict__ in_col,
           const int32_t* __restrict__ in_link, GroupView gv, SsspView sv, int level, int npw) {
  int g, nblk;
  if (!map_block(gv.G, gv.bpb * (kWave / npw), gv.inflight, g, nblk)) return;
  if (gv.ltot[(size_t)g * gv.Lcap + level] == 0) return;
  const int lane = lane_id();
  // a wave takes npw consecutive nodes (64, or fewer when an iteration has too few batches to fill the chip)
  const int v0 = __builtin_amdgcn_readfirstlane((nblk * kWavesPerBlock + (int)(threadIdx.x / kWave)) * npw);
  if (v0 >= gv.N) return;
  const size_t rows = (size_t)g * gv.Npad * 64;
  const uint64_t mine = (lane < npw && v0 + lane < gv.N) ? level_mask(gv, g, level, v0 + lane) : 0ull;
  uint64_t todo = __ballot(mine != 0);
  while (todo) {
    const int i = __builtin_ctzll(todo);
    todo &= todo - 1;
    const int v = v0 + i;
    const uint64_t mv = readlane64(mine, i);
    long long best = 0x7fffffffffffffffll;
    int via = -1;
    const int p1 = in_ptr[v + 1];
    for (int p = in_ptr[v]; p < p1; p += 8) {  // eight in-links at a time, all requests issued before any is used
      int u[8], a[8];
      uint64_t m[8];
      long long w[8], c[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        u[j] = p + j < p1 ? in_col[p + j] : -1;
        a[j] = p + j < p1 ? in_link[p + j] : 0;
      }
#pragma unroll
      for (int j = 0; j < 8; ++j) m[j] = u[j] >= 0 ? mv & level_mask(gv, g, level - 1, u[j]) : 0ull;
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        w[j] = m[j] != 0 ? (long long)sv.iload[a[j]] : 0ll;
        // the level before level 1 holds the sources themselves: cost 0, no row
        c[j] = (level > 1 && ((m[j] >> lane) & 1ull)) ? sv.cost[rows + (size_t)u[j] * 64 + lane] : 0ll;
      }
#pragma unroll
      for (int j = 0; j < 8; ++j) {  // ascending link id: the strict comparison keeps the lowest among equals
        if ((m[j] >> lane) & 1ull) {
          const long long t = c[j] + w[j];
          if (t < best) {
            best = t;
            via = a[j];
          }
        }
      }
    }
    if ((mv >> lane) & 1ull) {
      sv.cost[rows + (size_t)v * 64 + lane] = best;
      sv.pick[rows + (size_t)v * 64 + lane] = via;
    }
  }
}

// Paths through the pairs on `level` (deepest .. 0), and the loads of the links chosen by the pairs one
// level deeper.  The additions go straight to iload: the cost recursion of this iteration is over, the
// next one starts after this kernel's last launch.
__global__ void __launch_bounds__(kBlock)
k_sssp_bwd(const int32_t* __restrict__ out_ptr, const int32_t* __restrict__ out_col, GroupView gv, SsspView sv,
           int level, int npw) {
  int g, nblk;
  if (!map_block(gv.G, gv.bpb * (kWave / npw), gv.inflight, g, nblk)) return;
  const long long* __restrict__ lt = gv.ltot + (size_t)g * gv.Lcap;
  if (lt[level] == 0) return;
  const bool deeper = level + 1 < gv.Lcap && lt[level + 1] != 0;
  const int lane = lane_id();
  const int u0 = __builtin_amdgcn_readfirstlane((nblk * kWavesPerBlock + (int)(threadIdx.x / kWave)) * npw);
  if (u0 >= gv.N) return;
  const size_t rows = (size_t)g * gv.Npad * 64;
  const uint64_t mine = (lane < npw && u0 + lane < gv.N) ? level_mask(gv, g, level, u0 + lane) : 0ull;
  uint64_t todo = __ballot(mine != 0);
  while (todo) {
    const int i = __builtin_ctzll(todo);
    todo &= todo - 1;
    const int u = u0 + i;
    const uint64_t mu = readlane64(mine, i);
    int through = 1;  // the pair's own commodity (not counted at the source itself, level 0: never read)
    if (deeper) {
      const int q1 = out_ptr[u + 1];
      for (int q = out_ptr[u]; q < q1; q += 8) {  // eight out-links at a time
        int w[8], pk[8], x[8];
        uint64_t m[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) w[j] = q + j < q1 ? out_col[q + j] : -1;
#pragma unroll
        for (int j = 0; j < 8; ++j) m[j] = w[j] >= 0 ? mu & level_mask(gv, g, level + 1, w[j]) : 0ull;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          const bool on = (m[j] >> lane) & 1ull;
          pk[j] = on ? sv.pick[rows + (size_t)w[j] * 64 + lane] : -1;
          x[j] = on ? sv.sub[rows + (size_t)w[j] * 64 + lane] : 0;
        }
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          if (pk[j] != q + j) x[j] = 0;
          through += x[j];
        }
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) {
#pragma unroll
          for (int j = 0; j < 8; ++j) x[j] += __shfl_xor(x[j], o, kWave);
        }
        // lane j adds the total of link q + j
        int mine = 0;
#pragma unroll
        for (int j = 0; j < 8; ++j)
          if (lane == j) mine = x[j];
        if (lane < 8 && mine != 0) atomicAdd(&sv.iload[q + lane], (unsigned long long)mine);
      }
    }
    if (level > 0 && ((mu >> lane) & 1ull)) sv.sub[rows + (size_t)u * 64 + lane] = through;
  }
}

// load[a] = iload[a] as a double (exact below 2^53).
__global__ void __launch_bounds__(kBlock)
k_sssp_output(const unsigned long long* __restrict__ iload, long long E, double* __restrict__ load) {
  const long long a = (long long)blockIdx.x * kBlock + threadIdx.x;
  if (a < E) load[a] = (double)iload[a];
}

}  // namespace a2a_dev
