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
// Layout per batch: dense 64-wide rows, entry j = source j of the batch, row v = node v:
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

// Eight sums over the 64 lanes at once, for ints: on return every lane l holds the sum over all lanes
// of x[l & 7] (as wave_sum8_lds).  buf: 8 x (kWave + 1) ints of LDS of this wave's own.
constexpr int kSum8IntRow = kWave + 1;
__device__ __forceinline__ int wave_sum8_int_lds(const int (&x)[8], int lane, int* buf) {
#pragma unroll
  for (int j = 0; j < 8; ++j) buf[j * kSum8IntRow + lane] = x[j];
  __builtin_amdgcn_wave_barrier();
  const int* row = buf + (lane & 7) * kSum8IntRow + (lane & ~7);
  int w = row[0];
#pragma unroll
  for (int r = 1; r < 8; ++r) w += row[r];
  __builtin_amdgcn_wave_barrier();
  w += __shfl_xor(w, 8, kWave);
  w += __shfl_xor(w, 16, kWave);
  w += __shfl_xor(w, 32, kWave);
  return w;
}

// Both kernels work on tiles of eight nodes, as the EwSP kernels do: lane 8i+j first looks at link j of
// node i (neighbour, link id, the neighbour's level mask, the link's weight: one request each for 64
// links at a time), then the nodes are taken one after the other with lane = source, the eight row
// requests of a node in flight together.  Nodes with more than eight links take further rounds.

// cost and chosen in-link of the pairs on `level` (>= 1).  A wave takes npw (a multiple of 8) consecutive
// nodes of one batch.  In-links in list order = ascending link id, so the strict comparison keeps the
// lowest id among equals.
__global__ void __launch_bounds__(kBlock)
k_sssp_fwd(const int32_t* __restrict__ in_ptr, const int32_t* __restrict__ in_col,
           const int32_t* __restrict__ in_link, GroupView gv, SsspView sv, int level, int npw) {
  int g, nblk;
  if (!map_block(gv.G, gv.bpb * (kWave / npw), gv.inflight, g, nblk)) return;
  if (gv.ltot[(size_t)g * gv.Lcap + level] == 0) return;
  const int lane = lane_id();
  const int v0 = __builtin_amdgcn_readfirstlane((nblk * kWavesPerBlock + (int)(threadIdx.x / kWave)) * npw);
  if (v0 >= gv.N) return;
  const size_t rows = (size_t)g * gv.Npad * 64;
  for (int c = 0; c < npw; c += 8) {
    const int v = v0 + c + (lane >> 3);
    uint64_t mv = 0;  // the same in the eight lanes of a node
    int p0 = 0, p1 = 0;
    if (v < gv.N) mv = level_mask(gv, g, level, v);
    if (mv != 0) {
      p0 = in_ptr[v];
      p1 = in_ptr[v + 1];
    }
    if (__ballot(mv != 0) == 0) continue;
    long long best[8];
    int via[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      best[i] = 0x7fffffffffffffffll;
      via[i] = -1;
    }
    for (int base = 0; __ballot(p0 + base < p1) != 0; base += 8) {
      const int q = p0 + base + (lane & 7);
      int u = 0, a = 0;
      uint64_t m = 0;
      if (q < p1) {
        u = in_col[q];
        a = in_link[q];
        m = mv & level_mask(gv, g, level - 1, u);
      }
      long long w = 0;  // what the link has carried before this iteration
      if (m != 0) w = (long long)sv.iload[a];
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        uint64_t mj[8];
        uint64_t any = 0;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          mj[j] = readlane64(m, 8 * i + j);
          any |= mj[j];
        }
        if (any == 0) continue;  // the same in all lanes
        long long cst[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          cst[j] = 0;  // the level before level 1 holds the sources themselves: cost 0, no row
          if (level > 1 && mj[j] != 0 && lane_in(mj[j]))
            cst[j] = sv.cost[rows + (size_t)__builtin_amdgcn_readlane(u, 8 * i + j) * 64 + lane];
        }
#pragma unroll
        for (int j = 0; j < 8; ++j) {  // ascending link id
          if (mj[j] != 0 && lane_in(mj[j])) {
            const long long t = cst[j] + (long long)readlane64((uint64_t)w, 8 * i + j);
            if (t < best[i]) {
              best[i] = t;
              via[i] = __builtin_amdgcn_readlane(a, 8 * i + j);
            }
          }
        }
      }
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const uint64_t mvi = readlane64(mv, 8 * i);
      if (mvi != 0 && lane_in(mvi)) {
        sv.cost[rows + (size_t)(v0 + c + i) * 64 + lane] = best[i];
        sv.pick[rows + (size_t)(v0 + c + i) * 64 + lane] = via[i];
      }
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
  __shared__ int s_sum[kWavesPerBlock][8 * kSum8IntRow];
  int* const buf = s_sum[threadIdx.x / kWave];
  const size_t rows = (size_t)g * gv.Npad * 64;
  for (int c = 0; c < npw; c += 8) {
    const int un = u0 + c + (lane >> 3);
    uint64_t mu = 0;
    int p0 = 0, p1 = 0;
    if (un < gv.N) mu = level_mask(gv, g, level, un);
    if (mu != 0 && deeper) {
      p0 = out_ptr[un];
      p1 = out_ptr[un + 1];
    }
    if (__ballot(mu != 0) == 0) continue;
    int through[8];  // the pair's own commodity (not counted at the source itself, level 0: never read)
#pragma unroll
    for (int i = 0; i < 8; ++i) through[i] = 1;
    for (int base = 0; __ballot(p0 + base < p1) != 0; base += 8) {
      const int q = p0 + base + (lane & 7);
      int w = 0;
      uint64_t m = 0;
      if (q < p1) {
        w = out_col[q];
        m = mu & level_mask(gv, g, level + 1, w);
      }
      int tot_l = 0;  // lane 8i+j: paths that this iteration routes over link j of node i
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        uint64_t mj[8];
        uint64_t any = 0;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          mj[j] = readlane64(m, 8 * i + j);
          any |= mj[j];
        }
        if (any == 0) continue;
        int pk[8], x[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          pk[j] = -1;
          x[j] = 0;
          if (mj[j] != 0 && lane_in(mj[j])) {
            const size_t e = rows + (size_t)__builtin_amdgcn_readlane(w, 8 * i + j) * 64 + lane;
            pk[j] = sv.pick[e];
            x[j] = sv.sub[e];
          }
        }
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          if (pk[j] != __builtin_amdgcn_readlane(q, 8 * i + j)) x[j] = 0;  // the pair came over another link
          through[i] += x[j];
        }
        const int tot = wave_sum8_int_lds(x, lane, buf);
        if ((lane >> 3) == i) tot_l = tot;
      }
      if (q < p1 && tot_l != 0) atomicAdd(&sv.iload[q], (unsigned long long)tot_l);
    }
    if (level > 0) {
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const uint64_t mui = readlane64(mu, 8 * i);
        if (mui != 0 && lane_in(mui)) sv.sub[rows + (size_t)(u0 + c + i) * 64 + lane] = through[i];
      }
    }
  }
}

// load[a] = iload[a] as a double (exact below 2^53).
__global__ void __launch_bounds__(kBlock)
k_sssp_output(const unsigned long long* __restrict__ iload, long long E, double* __restrict__ load) {
  const long long a = (long long)blockIdx.x * kBlock + threadIdx.x;
  if (a < E) load[a] = (double)iload[a];
}

}  // namespace a2a_dev
