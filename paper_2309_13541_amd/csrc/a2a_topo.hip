// a2a_topo: all-pairs hop distances, shortest-path counts and EwSP link loads of a
// direct-connect topology (Sec. 2.2, 5.2, 5.3, 5.4 of the paper) on one MI355X (gfx950).
//
// Sources are handled 64 at a time ("batch"): bit j of a 64-bit mask = source j of the batch,
// and lane j of a wavefront carries that source's floating-point state.  A "group" of G
// batches advances level by level together, one kernel launch per level and pass:
//   bfs    L_l[v] = (OR over in-neighbours u of L_{l-1}[u]) & ~seen[v]           (pull)
//   fwd    sigma[v] = sum over in-links (u,v) with u one level up of sigma[u]
//   bwd    coef[u] = 1/sigma[u] + sum over out-links (u,w) with w one level down of coef[w]
//          load(u,w) += sum over sources of sigma[u]*coef[w]
// where coef = (1 + delta)/sigma is the dependency recursion of the EwSP split written so
// that one value per (source,node) is gathered per link.  Per-batch link loads are then added
// in ascending batch order.
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstdlib>
#include <cstring>
#include <new>
#include <vector>

#include "a2a_topo.h"

namespace {

constexpr int kWave = 64;
constexpr int kBlock = 256;                    // threads per workgroup
constexpr int kWavesPerBlock = kBlock / kWave;
constexpr int kXcd = 8;                        // workgroups are dealt round-robin to 8 XCDs
constexpr double kTwo53 = 9007199254740992.0;

// per-batch integer counters kept in the workspace control block
enum { CNT_DSUM = 0, CNT_REACHED = 1, CNT_DAG = 2, CNT_STRIDE = 4 };

struct Layout {
  int G = 0;          // batches per group
  int Lcap = 0;       // level slots per batch (levels 0 .. Lcap-1)
  int Npad = 0;       // N rounded up to a multiple of 64
  bool sigma = false, loads = false;
  size_t off_level_new = 0;  // int32 [Lcap]
  size_t off_misc = 0;       // int64: 0 sigma-inexact flag, 1 dist_sum total, 2 reached total, 3 DAG links
  size_t off_cnt = 0;        // int64 [G][CNT_STRIDE]
  size_t off_lvl = 0;        // uint64 [G][Lcap][Npad]
  size_t off_seen = 0;       // uint64 [G][Npad]
  size_t off_sig = 0;        // double [G][Npad][64]
  size_t off_part = 0;       // double [G][Epad]
  size_t Epad = 0;
  size_t total = 0;
};

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

}  // namespace

struct a2a_topo {
  int32_t N = 0;
  int64_t E = 0;
  int32_t dmax = 0;
  int32_t level_bound = 0;
  int32_t* d_out_ptr = nullptr;
  int32_t* d_out_col = nullptr;
  int32_t* d_in_ptr = nullptr;
  int32_t* d_in_col = nullptr;
  int64_t* h_pinned = nullptr;  // 16 x int64 pinned host words for read-backs
  int64_t* d_small = nullptr;   // 16 x int64 device words (schedule_bound result, profile counters)
  // optional per-kernel timing (a2a_profile_enable); events are created per launch while it is on
  struct ProfRec {
    int cls;
    hipEvent_t beg, end;
  };
  mutable bool prof_on = false;
  mutable std::vector<ProfRec> prof_recs;
  mutable int64_t prof_calls = 0;
  mutable int32_t prof_depth = 0;
  mutable int32_t prof_groups = 0;
};

namespace {

Layout make_layout(const a2a_topo* t, int32_t src_count, int flags, size_t ws_bytes, bool minimal,
                   bool recommend) {
  Layout L;
  L.sigma = (flags & (A2A_WS_SIGMA | A2A_WS_LOADS)) != 0;
  L.loads = (flags & A2A_WS_LOADS) != 0;
  L.Npad = (int)align_up((size_t)t->N, 64);
  L.Lcap = t->level_bound + 2;
  L.Epad = align_up((size_t)(t->E > 0 ? t->E : 1), 32);
  const int nb = (src_count + 63) / 64;
  const size_t per_batch = (size_t)L.Npad * 8 * L.Lcap + (size_t)L.Npad * 8 +
                           (L.sigma ? (size_t)L.Npad * 64 * 8 : 0) + (L.loads ? L.Epad * 8 : 0) +
                           CNT_STRIDE * 8;
  const size_t fixed = align_up((size_t)L.Lcap * 4, 256) + 256;
  int G;
  if (recommend) {
    G = minimal ? 1 : nb;
  } else {
    if (ws_bytes < fixed + per_batch + 256) {
      L.G = 0;
      return L;
    }
    size_t g = (ws_bytes - fixed - 256) / per_batch;
    G = (int)(g < (size_t)nb ? g : (size_t)nb);
  }
  if (G < 1) G = 1;
  L.G = G;
  size_t off = 0;
  L.off_level_new = off;
  off += align_up((size_t)L.Lcap * 4, 256);
  L.off_misc = off;
  off += 256;
  L.off_cnt = off;
  off += align_up((size_t)G * CNT_STRIDE * 8, 256);
  L.off_lvl = off;
  off += (size_t)G * L.Lcap * L.Npad * 8;
  L.off_seen = off;
  off += (size_t)G * L.Npad * 8;
  if (L.sigma) {
    L.off_sig = off;
    off += (size_t)G * L.Npad * 64 * 8;
  }
  if (L.loads) {
    L.off_part = off;
    off += (size_t)G * L.Epad * 8;
  }
  L.total = off;
  return L;
}

// ---------------------------------------------------------------------------------------
// device helpers
// ---------------------------------------------------------------------------------------

__device__ __forceinline__ uint64_t readlane64(uint64_t x, int k) {
  uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)x, k);
  uint32_t hi = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(x >> 32), k);
  return ((uint64_t)hi << 32) | lo;
}

__device__ __forceinline__ int lane_id() { return (int)(threadIdx.x & (kWave - 1)); }

// Sum over the 64 lanes in a fixed butterfly order; every lane gets the total.
__device__ __forceinline__ double wave_sum(double x) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) x += __shfl_xor(x, o, kWave);
  return x;
}

__device__ __forceinline__ long long wave_sum_i64(long long x) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) x += __shfl_xor(x, o, kWave);
  return x;
}

// Workgroups go round-robin to the 8 XCDs, each with its own L2.  `inflight` consecutive
// workgroups belong to `inflight` different batches; with inflight = 8 all workgroups of one
// batch run on one XCD, so that the rows its waves gather stay in that XCD's L2.
__device__ __forceinline__ bool map_block(int G, int blocks_per_batch, int inflight, int& g, int& nblk) {
  const unsigned blk = blockIdx.x;
  const unsigned x = blk % (unsigned)inflight;
  const unsigned i = blk / (unsigned)inflight;
  g = (int)((i / (unsigned)blocks_per_batch) * inflight + x);
  nblk = (int)(i % (unsigned)blocks_per_batch);
  return g < G;
}

__device__ __forceinline__ uint64_t valid_mask(int src_count, int batch) {
  const int cnt = src_count - batch * 64;
  return cnt >= 64 ? ~0ull : ((1ull << cnt) - 1ull);
}

// ---------------------------------------------------------------------------------------
// kernels
// ---------------------------------------------------------------------------------------

// Level 0: bit j of L_0[s_j] and seen[s_j] for the batch's sources s_j; sigma(s_j,s_j) = 1.
__global__ void __launch_bounds__(kBlock)
k_init_group(uint64_t* __restrict__ lvl, uint64_t* __restrict__ seen, double* __restrict__ sig,
             int N, int Npad, int Lcap, int G, int bpb, int src_begin, int src_count, int batch0) {
  int g, nblk;
  if (!map_block(G, bpb, kXcd, g, nblk)) return;
  const int v = nblk * kBlock + (int)threadIdx.x;
  if (v >= Npad) return;
  const int s0 = src_begin + (batch0 + g) * 64;
  const int cnt = min(64, src_begin + src_count - s0);
  const int j = v - s0;
  const bool is_src = (v < N) && j >= 0 && j < cnt;
  const uint64_t bit = is_src ? (1ull << j) : 0ull;
  lvl[((size_t)g * Lcap) * Npad + v] = bit;
  seen[(size_t)g * Npad + v] = bit;
  if (sig != nullptr && is_src) sig[((size_t)g * Npad + v) * 64 + j] = 1.0;
}

// One BFS level for every batch of the group, one thread per (batch, node).
__global__ void __launch_bounds__(kBlock)
k_bfs_level(const int32_t* __restrict__ in_ptr, const int32_t* __restrict__ in_col,
            uint64_t* __restrict__ lvl, uint64_t* __restrict__ seen, int N, int Npad, int Lcap,
            int G, int bpb, int level, int src_count, int batch0, int* __restrict__ level_new,
            long long* __restrict__ cnt) {
  int g, nblk;
  if (!map_block(G, bpb, kXcd, g, nblk)) return;
  const int v = nblk * kBlock + (int)threadIdx.x;
  uint64_t nw = 0;
  if (v < Npad) {
    if (v < N) {
      const uint64_t sn = seen[(size_t)g * Npad + v];
      if (sn != valid_mask(src_count, batch0 + g)) {
        const uint64_t* __restrict__ prev = lvl + ((size_t)g * Lcap + (level - 1)) * Npad;
        uint64_t acc = 0;
        const int p1 = in_ptr[v + 1];
        for (int p = in_ptr[v]; p < p1; ++p) acc |= prev[in_col[p]];
        nw = acc & ~sn;
        if (nw) seen[(size_t)g * Npad + v] = sn | nw;
      }
    }
    lvl[((size_t)g * Lcap + level) * Npad + v] = nw;
  }
  // block-wide count of newly reached (source,node) pairs
  __shared__ int s_cnt[kWavesPerBlock];
  int pc = __popcll(nw);
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) pc += __shfl_xor(pc, o, kWave);
  if (lane_id() == 0) s_cnt[threadIdx.x / kWave] = pc;
  __syncthreads();
  if (threadIdx.x == 0) {
    int tot = 0;
#pragma unroll
    for (int w = 0; w < kWavesPerBlock; ++w) tot += s_cnt[w];
    if (tot > 0) {
      atomicAdd((unsigned long long*)&cnt[g * CNT_STRIDE + CNT_DSUM],
                (unsigned long long)((long long)tot * level));
      atomicAdd((unsigned long long*)&cnt[g * CNT_STRIDE + CNT_REACHED], (unsigned long long)tot);
      level_new[level] = 1;
    }
  }
}

// Lane exchange with lane ^ kMask, for the 64-bit reductions below.
template <int kMask>
__device__ __forceinline__ double xor_lanes(double x) {
  union {
    double d;
    int i[2];
  } a, b;
  a.d = x;
  if constexpr (kMask == 1) {  // DPP quad_perm [1,0,3,2]
    b.i[0] = __builtin_amdgcn_mov_dpp(a.i[0], 0xB1, 0xF, 0xF, true);
    b.i[1] = __builtin_amdgcn_mov_dpp(a.i[1], 0xB1, 0xF, 0xF, true);
  } else if constexpr (kMask == 2) {  // DPP quad_perm [2,3,0,1]
    b.i[0] = __builtin_amdgcn_mov_dpp(a.i[0], 0x4E, 0xF, 0xF, true);
    b.i[1] = __builtin_amdgcn_mov_dpp(a.i[1], 0x4E, 0xF, 0xF, true);
  } else if constexpr (kMask < 32) {  // ds_swizzle, bit mode: and 0x1f, or 0, xor kMask
    b.i[0] = __builtin_amdgcn_ds_swizzle(a.i[0], 0x1F | (kMask << 10));
    b.i[1] = __builtin_amdgcn_ds_swizzle(a.i[1], 0x1F | (kMask << 10));
  } else {
    return __shfl_xor(x, kMask, kWave);
  }
  return b.d;
}

// Eight 64-lane sums at once.  x[i] is lane-local; on return every lane l holds the sum over
// all 64 lanes of x[l & 7].  Halving the value set at each of the first three exchange steps
// costs 4+2+1+3 exchanges instead of 8*6, in a fixed order.
__device__ __forceinline__ double wave_sum8(const double (&x)[8], int lane) {
  const bool b0 = lane & 1, b1 = lane & 2, b2 = lane & 4;
  double y[4], z[2];
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    const double keep = b0 ? x[2 * k + 1] : x[2 * k];
    const double send = b0 ? x[2 * k] : x[2 * k + 1];
    y[k] = keep + xor_lanes<1>(send);
  }
#pragma unroll
  for (int k = 0; k < 2; ++k) {
    const double keep = b1 ? y[2 * k + 1] : y[2 * k];
    const double send = b1 ? y[2 * k] : y[2 * k + 1];
    z[k] = keep + xor_lanes<2>(send);
  }
  const double keep = b2 ? z[1] : z[0];
  const double send = b2 ? z[0] : z[1];
  double w = keep + xor_lanes<4>(send);
  w += xor_lanes<8>(w);
  w += xor_lanes<16>(w);
  w += xor_lanes<32>(w);
  return w;
}

// Forward path counts for one level: each wave takes 64 consecutive nodes of one batch and
// visits those with a non-empty L_level mask.  Lane j = source j.  In-links are taken eight at
// a time so that eight row gathers are in flight per wave.
template <bool kCountDag>
__global__ void __launch_bounds__(kBlock)
k_fwd_level(const int32_t* __restrict__ in_ptr, const int32_t* __restrict__ in_col,
            const uint64_t* __restrict__ lvl, double* __restrict__ sig, int N, int Npad, int Lcap,
            int G, int bpb, int inflight, int level, long long* __restrict__ misc,
            long long* __restrict__ cnt) {
  int g, nblk;
  if (!map_block(G, bpb, inflight, g, nblk)) return;
  const int lane = lane_id();
  const int v0 = __builtin_amdgcn_readfirstlane((nblk * kWavesPerBlock + (int)(threadIdx.x / kWave)) * kWave);
  if (v0 >= N) return;
  const uint64_t* __restrict__ cur = lvl + ((size_t)g * Lcap + level) * Npad;
  const uint64_t* __restrict__ prev = lvl + ((size_t)g * Lcap + (level - 1)) * Npad;
  double* __restrict__ sg = sig + (size_t)g * Npad * 64;
  const uint64_t my_new = cur[v0 + lane];  // Npad is a multiple of 64: in bounds, 0 beyond N
  uint64_t todo = __ballot(my_new != 0);
  bool inexact = false;
  long long dag = 0;  // (source, link) pairs on shortest paths seen by this wave
  while (todo) {
    const int k = __builtin_ctzll(todo);
    todo &= todo - 1;
    const int v = v0 + k;
    const uint64_t newv = readlane64(my_new, k);
    const int p0 = in_ptr[v], p1 = in_ptr[v + 1];
    double acc = 0.0;
    for (int p = p0; p < p1; p += kWave) {
      const int q = p + lane;
      const int u_l = q < p1 ? in_col[q] : 0;
      const uint64_t m_l = q < p1 ? (prev[u_l] & newv) : 0ull;
      uint64_t act = __ballot(m_l != 0);
      while (act) {
        const int c = __builtin_ctzll(act) & ~7;  // first lane position of the next octet of links
        act &= ~(0xffull << c);
        double x[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          const int u = __builtin_amdgcn_readlane(u_l, c + i);
          const uint64_t m = readlane64(m_l, c + i);
          if (kCountDag) dag += __popcll(m);
          x[i] = ((m >> lane) & 1ull) ? sg[(size_t)u * 64 + lane] : 0.0;
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) acc += x[i];
      }
    }
    if ((newv >> lane) & 1ull) {
      sg[(size_t)v * 64 + lane] = acc;
      inexact |= acc >= kTwo53;
    }
  }
  if (inexact) misc[0] = 1;
  if (kCountDag && dag != 0 && lane == 0)
    atomicAdd((unsigned long long*)&cnt[g * CNT_STRIDE + CNT_DAG], (unsigned long long)dag);
}

// Backward dependency pass for one level.  On entry sig holds sigma for levels <= level and
// coef for deeper levels; on exit the nodes of this level hold coef.  part[a] accumulates the
// batch's load of link a.  Out-links are taken eight at a time: eight row gathers in flight,
// then one eight-way wave reduction of sigma[u]*coef[w] per link.
__global__ void __launch_bounds__(kBlock)
k_bwd_level(const int32_t* __restrict__ out_ptr, const int32_t* __restrict__ out_col,
            const uint64_t* __restrict__ lvl, double* __restrict__ sig, double* __restrict__ part,
            size_t Epad, int N, int Npad, int Lcap, int G, int bpb, int inflight, int level) {
  int g, nblk;
  if (!map_block(G, bpb, inflight, g, nblk)) return;
  const int lane = lane_id();
  const int u0 = __builtin_amdgcn_readfirstlane((nblk * kWavesPerBlock + (int)(threadIdx.x / kWave)) * kWave);
  if (u0 >= N) return;
  const uint64_t* __restrict__ cur = lvl + ((size_t)g * Lcap + level) * Npad;
  const uint64_t* __restrict__ next = lvl + ((size_t)g * Lcap + (level + 1)) * Npad;
  double* __restrict__ sg = sig + (size_t)g * Npad * 64;
  double* __restrict__ pt = part + (size_t)g * Epad;
  const uint64_t my_cur = cur[u0 + lane];
  uint64_t todo = __ballot(my_cur != 0);
  while (todo) {
    const int k = __builtin_ctzll(todo);
    todo &= todo - 1;
    const int u = u0 + k;
    const uint64_t mu = readlane64(my_cur, k);
    const bool mine = (mu >> lane) & 1ull;
    const double s_u = mine ? sg[(size_t)u * 64 + lane] : 1.0;
    const int p0 = out_ptr[u], p1 = out_ptr[u + 1];
    double acc = 0.0;
    for (int p = p0; p < p1; p += kWave) {
      const int q = p + lane;
      const int w_l = q < p1 ? out_col[q] : 0;
      const uint64_t m_l = q < p1 ? (next[w_l] & mu) : 0ull;
      uint64_t act = __ballot(m_l != 0);
      while (act) {
        const int c = __builtin_ctzll(act) & ~7;
        act &= ~(0xffull << c);
        double x[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          const int w = __builtin_amdgcn_readlane(w_l, c + i);
          const uint64_t m = readlane64(m_l, c + i);
          x[i] = ((m >> lane) & 1ull) ? sg[(size_t)w * 64 + lane] : 0.0;
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          acc += x[i];
          x[i] *= s_u;
        }
        const double tot = wave_sum8(x, lane);  // lane l: load of link p + c + (l & 7)
        if ((lane & ~7) == c && m_l != 0) pt[q] += tot;
      }
    }
    if (mine) sg[(size_t)u * 64 + lane] = 1.0 / s_u + acc;
  }
}

// load[a] = (first group ? 0 : load[a]) + part[0][a] + part[1][a] + ... in that order.
__global__ void __launch_bounds__(kBlock)
k_reduce_part(const double* __restrict__ part, size_t Epad, int G, long long E, int first,
              double* __restrict__ load) {
  const long long a = (long long)blockIdx.x * kBlock + threadIdx.x;
  if (a >= E) return;
  double s = first ? 0.0 : load[a];
  for (int g = 0; g < G; ++g) s += part[(size_t)g * Epad + a];
  load[a] = s;
}

// dist[s][v] from the level masks, through a 64 x 64 LDS tile so that rows of dist are written
// with consecutive lanes on consecutive nodes.  One wave per (batch, 64-node tile).
__global__ void __launch_bounds__(kWave)
k_extract_dist(const uint64_t* __restrict__ lvl, int N, int Npad, int Lcap, int G, int tiles,
               int depth, int src_count, int batch0, int32_t* __restrict__ dist,
               long long* __restrict__ dist_sum) {
  int g, tile;
  if (!map_block(G, tiles, kXcd, g, tile)) return;
  __shared__ int32_t t_d[kWave][kWave + 1];
  const int t = (int)threadIdx.x;
  const int v = tile * kWave + t;
  for (int j = 0; j < kWave; ++j) t_d[j][t] = -1;
  for (int l = 0; l <= depth; ++l) {
    uint64_t m = lvl[((size_t)g * Lcap + l) * Npad + v];
    while (m) {
      const int j = __builtin_ctzll(m);
      m &= m - 1;
      t_d[j][t] = l;
    }
  }
  __syncthreads();
  const int row0 = (batch0 + g) * 64;
  const int cnt = min(64, src_count - row0);
  if (dist != nullptr && v < N) {
    for (int j = 0; j < cnt; ++j) dist[(size_t)(row0 + j) * N + v] = t_d[j][t];
  }
  if (dist_sum != nullptr && t < cnt) {
    long long s = 0;
    const int lim = min(kWave, N - tile * kWave);
    for (int i = 0; i < lim; ++i) {
      const int d = t_d[t][i];
      s += d > 0 ? d : 0;
    }
    if (s) atomicAdd((unsigned long long*)&dist_sum[row0 + t], (unsigned long long)s);
  }
}

// sigma[s][v] from the lane-major rows, transposed through LDS.  One wave per tile.
__global__ void __launch_bounds__(kWave)
k_extract_sigma(const uint64_t* __restrict__ seen, const double* __restrict__ sig, int N, int Npad,
                int G, int tiles, int src_count, int batch0, double* __restrict__ sigma_out) {
  int g, tile;
  if (!map_block(G, tiles, kXcd, g, tile)) return;
  __shared__ double t_s[kWave][kWave + 1];
  const int t = (int)threadIdx.x;
  const int v0 = tile * kWave;
  const uint64_t my_seen = seen[(size_t)g * Npad + v0 + t];
  for (int i = 0; i < kWave; ++i) {
    const uint64_t sn = readlane64(my_seen, i);
    double x = 0.0;
    if ((sn >> t) & 1ull) x = sig[((size_t)g * Npad + v0 + i) * 64 + t];
    t_s[t][i] = x;
  }
  __syncthreads();
  const int row0 = (batch0 + g) * 64;
  const int cnt = min(64, src_count - row0);
  if (v0 + t < N) {
    for (int j = 0; j < cnt; ++j) sigma_out[(size_t)(row0 + j) * N + v0 + t] = t_s[j][t];
  }
}

// Folds the per-batch counters of a group into the running totals.
__global__ void k_fold_counters(const long long* __restrict__ cnt, int G, long long* __restrict__ misc) {
  if (threadIdx.x == 0 && blockIdx.x == 0) {
    long long ds = 0, rc = 0, dg = 0;
    for (int g = 0; g < G; ++g) {
      ds += cnt[g * CNT_STRIDE + CNT_DSUM];
      rc += cnt[g * CNT_STRIDE + CNT_REACHED];
      dg += cnt[g * CNT_STRIDE + CNT_DAG];
    }
    misc[1] += ds;
    misc[2] += rc;
    misc[3] += dg;
  }
}

// Final outputs of a call: totals and flag bits.
__global__ void k_finish(const long long* __restrict__ misc, long long pairs,
                         long long* __restrict__ dist_sum_total, long long* __restrict__ unreachable,
                         long long* __restrict__ flags, long long* __restrict__ prof_out) {
  if (threadIdx.x == 0 && blockIdx.x == 0) {
    const long long unr = pairs - misc[2];
    if (prof_out) prof_out[8] += misc[3];
    if (dist_sum_total) *dist_sum_total = misc[1];
    if (unreachable) *unreachable = unr;
    if (flags) *flags = (misc[0] ? A2A_FLAG_SIGMA_INEXACT : 0) | (unr ? A2A_FLAG_UNREACHABLE : 0);
  }
}

// max (lowest link id on ties) and min of load[0..E): one workgroup.
__global__ void __launch_bounds__(1024)
k_load_extrema(const double* __restrict__ load, long long E, long long* __restrict__ out) {
  __shared__ double s_max[1024], s_min[1024];
  __shared__ long long s_arg[1024];
  const int t = (int)threadIdx.x;
  double mx = -1.0, mn = 1.0e308 * 10.0;
  long long arg = -1;
  for (long long a = t; a < E; a += 1024) {
    const double x = load[a];
    if (x > mx) {
      mx = x;
      arg = a;
    }
    if (x < mn) mn = x;
  }
  s_max[t] = mx;
  s_min[t] = mn;
  s_arg[t] = arg;
  __syncthreads();
  for (int o = 512; o > 0; o >>= 1) {
    if (t < o) {
      const double om = s_max[t + o];
      const long long oa = s_arg[t + o];
      if (oa >= 0 && (s_arg[t] < 0 || om > s_max[t] || (om == s_max[t] && oa < s_arg[t]))) {
        s_max[t] = om;
        s_arg[t] = oa;
      }
      if (s_min[t + o] < s_min[t]) s_min[t] = s_min[t + o];
    }
    __syncthreads();
  }
  if (t == 0) {
    out[0] = __double_as_longlong(s_max[0]);
    out[1] = s_arg[0];
    out[2] = __double_as_longlong(s_min[0]);
  }
}

// ---------------------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------------------

#define HIP_TRY(expr)                     \
  do {                                    \
    if ((expr) != hipSuccess) {           \
      (void)hipGetLastError();            \
      return A2A_ERR_HIP;                 \
    }                                     \
  } while (0)

// Brackets one kernel launch with two events while profiling is on.
struct ProfScope {
  const a2a_topo* t;
  hipStream_t st;
  a2a_topo::ProfRec rec{};
  bool live = false;
  ProfScope(const a2a_topo* t_, int cls, hipStream_t st_) : t(t_), st(st_) {
    if (!t->prof_on) return;
    rec.cls = cls;
    if (hipEventCreate(&rec.beg) != hipSuccess) return;
    if (hipEventCreate(&rec.end) != hipSuccess) {
      (void)hipEventDestroy(rec.beg);
      return;
    }
    live = hipEventRecord(rec.beg, st) == hipSuccess;
  }
  ~ProfScope() {
    if (!live) return;
    (void)hipEventRecord(rec.end, st);
    t->prof_recs.push_back(rec);
  }
};

enum { PROF_INIT = 0, PROF_BFS, PROF_FWD, PROF_BWD, PROF_REDUCE, PROF_EXTRACT, PROF_CLASSES };

inline int grid_for(int G, int blocks_per_batch, int inflight = kXcd) {
  return (G + inflight - 1) / inflight * inflight * blocks_per_batch;
}

inline int env_inflight() {
  const char* e = std::getenv("A2A_INFLIGHT");
  const int v = e ? std::atoi(e) : kXcd;
  return v >= 1 && v <= 64 ? v : kXcd;
}

// Eccentricity of node 0 over the given CSR by queue BFS; -1 if some node is not reached.
int host_ecc0(int32_t N, const int32_t* ptr, const int32_t* col) {
  std::vector<int32_t> d((size_t)N, -1), q((size_t)N);
  int head = 0, tail = 0, ecc = 0;
  d[0] = 0;
  q[tail++] = 0;
  while (head < tail) {
    const int u = q[head++];
    for (int p = ptr[u]; p < ptr[u + 1]; ++p) {
      const int w = col[p];
      if (d[w] < 0) {
        d[w] = d[u] + 1;
        ecc = d[w];
        q[tail++] = w;
      }
    }
  }
  return tail == N ? ecc : -1;
}

struct Run {
  const a2a_topo* t;
  Layout L;
  char* ws;
  hipStream_t st;
  int src_begin, src_count;
  int inflight = env_inflight();
  int* level_new() const { return (int*)(ws + L.off_level_new); }
  long long* misc() const { return (long long*)(ws + L.off_misc); }
  long long* cnt() const { return (long long*)(ws + L.off_cnt); }
  uint64_t* lvl() const { return (uint64_t*)(ws + L.off_lvl); }
  uint64_t* seen() const { return (uint64_t*)(ws + L.off_seen); }
  double* sig() const { return L.sigma ? (double*)(ws + L.off_sig) : nullptr; }
  double* part() const { return L.loads ? (double*)(ws + L.off_part) : nullptr; }
};

// BFS of one group; returns the depth (deepest non-empty level) through *depth.
int run_bfs(const Run& r, int batch0, int G, int* depth) {
  const a2a_topo* t = r.t;
  const Layout& L = r.L;
  const int bpb = (L.Npad + kBlock - 1) / kBlock;
  HIP_TRY(hipMemsetAsync(r.level_new(), 0, (size_t)L.Lcap * 4, r.st));
  HIP_TRY(hipMemsetAsync(r.cnt(), 0, (size_t)G * CNT_STRIDE * 8, r.st));
  {
    ProfScope ps(t, PROF_INIT, r.st);
    k_init_group<<<grid_for(G, bpb), kBlock, 0, r.st>>>(r.lvl(), r.seen(), r.sig(), t->N, L.Npad, L.Lcap,
                                                        G, bpb, r.src_begin, r.src_count, batch0);
  }
  int d = 0;
  int l = 1;
  for (; l < L.Lcap; ++l) {
    {
      ProfScope ps(t, PROF_BFS, r.st);
      k_bfs_level<<<grid_for(G, bpb), kBlock, 0, r.st>>>(t->d_in_ptr, t->d_in_col, r.lvl(), r.seen(), t->N,
                                                         L.Npad, L.Lcap, G, bpb, l, r.src_count, batch0,
                                                         r.level_new(), r.cnt());
    }
    HIP_TRY(hipMemcpyAsync(t->h_pinned, r.level_new() + l, 4, hipMemcpyDeviceToHost, r.st));
    HIP_TRY(hipStreamSynchronize(r.st));
    if (*(volatile int*)t->h_pinned == 0) break;
    d = l;
  }
  if (l == L.Lcap) return A2A_ERR_LEVEL_OVERFLOW;
  HIP_TRY(hipGetLastError());
  *depth = d;
  if (d > t->prof_depth) t->prof_depth = d;
  t->prof_groups++;
  return A2A_OK;
}

int run_fwd(const Run& r, int G, int depth) {
  const a2a_topo* t = r.t;
  const Layout& L = r.L;
  const int bpb = (L.Npad + kBlock - 1) / kBlock;
  for (int l = 1; l <= depth; ++l) {
    ProfScope ps(t, PROF_FWD, r.st);
    if (t->prof_on)
      k_fwd_level<true><<<grid_for(G, bpb, r.inflight), kBlock, 0, r.st>>>(t->d_in_ptr, t->d_in_col, r.lvl(), r.sig(),
                                                               t->N, L.Npad, L.Lcap, G, bpb, r.inflight, l, r.misc(),
                                                               r.cnt());
    else
      k_fwd_level<false><<<grid_for(G, bpb, r.inflight), kBlock, 0, r.st>>>(t->d_in_ptr, t->d_in_col, r.lvl(), r.sig(),
                                                                t->N, L.Npad, L.Lcap, G, bpb, r.inflight, l, r.misc(),
                                                                r.cnt());
  }
  HIP_TRY(hipGetLastError());
  return A2A_OK;
}

// Per-batch counters of the finished group go into the call's running totals.
int run_fold(const Run& r, int G) {
  k_fold_counters<<<1, 64, 0, r.st>>>(r.cnt(), G, r.misc());
  HIP_TRY(hipGetLastError());
  return A2A_OK;
}

int check_common(const a2a_topo* t, int32_t src_begin, int32_t src_count, void* ws) {
  if (!t || src_begin < 0 || src_count < 0 || (int64_t)src_begin + src_count > t->N) return A2A_ERR_INVALID_ARG;
  if (src_count > 0 && (!ws || ((uintptr_t)ws & 255u))) return A2A_ERR_INVALID_ARG;
  return A2A_OK;
}

}  // namespace

extern "C" {

const char* a2a_status_string(int status) {
  switch (status) {
    case A2A_OK: return "ok";
    case A2A_ERR_INVALID_ARG: return "invalid argument";
    case A2A_ERR_SELF_LOOP: return "self-loop in topology";
    case A2A_ERR_WORKSPACE_TOO_SMALL: return "workspace too small";
    case A2A_ERR_HIP: return "HIP runtime error";
    case A2A_ERR_NOT_IMPLEMENTED: return "not implemented";
    case A2A_ERR_DISCONNECTED: return "topology is not strongly connected";
    case A2A_ERR_NO_MEMORY: return "out of host memory";
    case A2A_ERR_LEVEL_OVERFLOW: return "BFS exceeded the level bound";
    default: return "unknown status";
  }
}

int a2a_topo_create(int32_t N, const int32_t* row_ptr, const int32_t* col_idx, a2a_topo** out) {
  if (!out) return A2A_ERR_INVALID_ARG;
  *out = nullptr;
  if (N <= 0 || !row_ptr || row_ptr[0] != 0) return A2A_ERR_INVALID_ARG;
  int32_t dmax = 0;
  for (int32_t u = 0; u < N; ++u) {
    if (row_ptr[u + 1] < row_ptr[u]) return A2A_ERR_INVALID_ARG;
    if (row_ptr[u + 1] - row_ptr[u] > dmax) dmax = row_ptr[u + 1] - row_ptr[u];
  }
  const int64_t E = row_ptr[N];
  if (E > 0 && !col_idx) return A2A_ERR_INVALID_ARG;
  for (int32_t u = 0; u < N; ++u)
    for (int32_t p = row_ptr[u]; p < row_ptr[u + 1]; ++p) {
      if (col_idx[p] < 0 || col_idx[p] >= N) return A2A_ERR_INVALID_ARG;
      if (col_idx[p] == u) return A2A_ERR_SELF_LOOP;
    }
  a2a_topo* t = new (std::nothrow) a2a_topo();
  if (!t) return A2A_ERR_NO_MEMORY;
  std::vector<int32_t> in_ptr, in_col;
  try {
    in_ptr.assign((size_t)N + 1, 0);
    in_col.resize((size_t)(E > 0 ? E : 1));
    for (int64_t p = 0; p < E; ++p) in_ptr[(size_t)col_idx[p] + 1]++;
    for (int32_t v = 0; v < N; ++v) in_ptr[(size_t)v + 1] += in_ptr[v];
    std::vector<int32_t> fill(in_ptr.begin(), in_ptr.end() - 1);
    for (int32_t u = 0; u < N; ++u)  // ascending link id => in-lists are stable in link order
      for (int32_t p = row_ptr[u]; p < row_ptr[u + 1]; ++p) in_col[(size_t)fill[col_idx[p]]++] = u;
    const int e_out = host_ecc0(N, row_ptr, col_idx);
    const int e_in = host_ecc0(N, in_ptr.data(), in_col.data());
    t->level_bound = (e_out >= 0 && e_in >= 0) ? e_out + e_in : N - 1;
    if (t->level_bound > N - 1) t->level_bound = N - 1;
  } catch (const std::bad_alloc&) {
    delete t;
    return A2A_ERR_NO_MEMORY;
  }
  t->N = N;
  t->E = E;
  t->dmax = dmax;
  const size_t pb = ((size_t)N + 1) * sizeof(int32_t);
  const size_t cb = (size_t)(E > 0 ? E : 1) * sizeof(int32_t);
  bool ok = hipMalloc((void**)&t->d_out_ptr, pb) == hipSuccess &&
            hipMalloc((void**)&t->d_out_col, cb) == hipSuccess &&
            hipMalloc((void**)&t->d_in_ptr, pb) == hipSuccess &&
            hipMalloc((void**)&t->d_in_col, cb) == hipSuccess &&
            hipMalloc((void**)&t->d_small, 16 * sizeof(int64_t)) == hipSuccess &&
            hipHostMalloc((void**)&t->h_pinned, 16 * sizeof(int64_t), hipHostMallocDefault) == hipSuccess;
  ok = ok && hipMemcpy(t->d_out_ptr, row_ptr, pb, hipMemcpyHostToDevice) == hipSuccess &&
       hipMemcpy(t->d_in_ptr, in_ptr.data(), pb, hipMemcpyHostToDevice) == hipSuccess;
  if (ok && E > 0)
    ok = hipMemcpy(t->d_out_col, col_idx, (size_t)E * 4, hipMemcpyHostToDevice) == hipSuccess &&
         hipMemcpy(t->d_in_col, in_col.data(), (size_t)E * 4, hipMemcpyHostToDevice) == hipSuccess;
  if (!ok) {
    (void)hipGetLastError();
    a2a_topo_destroy(t);
    return A2A_ERR_HIP;
  }
  *out = t;
  return A2A_OK;
}

void a2a_topo_destroy(a2a_topo* t) {
  if (!t) return;
  if (t->d_out_ptr) (void)hipFree(t->d_out_ptr);
  if (t->d_out_col) (void)hipFree(t->d_out_col);
  if (t->d_in_ptr) (void)hipFree(t->d_in_ptr);
  if (t->d_in_col) (void)hipFree(t->d_in_col);
  if (t->d_small) (void)hipFree(t->d_small);
  if (t->h_pinned) (void)hipHostFree(t->h_pinned);
  delete t;
}

int a2a_topo_info(const a2a_topo* t, int32_t* N, int64_t* E, int32_t* dmax, int32_t* level_bound) {
  if (!t) return A2A_ERR_INVALID_ARG;
  if (N) *N = t->N;
  if (E) *E = t->E;
  if (dmax) *dmax = t->dmax;
  if (level_bound) *level_bound = t->level_bound;
  return A2A_OK;
}

size_t a2a_workspace_bytes(const a2a_topo* t, int32_t src_count, int flags) {
  if (!t || src_count < 0 || src_count > t->N) return 0;
  if (src_count == 0) return 256;
  const Layout L = make_layout(t, src_count, flags & 0xff, 0, (flags & A2A_WS_MINIMAL) != 0, true);
  return L.total + 256;
}

int a2a_distances(const a2a_topo* t, int32_t src_begin, int32_t src_count, int32_t* dist, double* sigma,
                  int64_t* dist_sum, int64_t* unreachable, int64_t* flags, void* workspace,
                  size_t workspace_bytes, void* hip_stream) {
  int rc = check_common(t, src_begin, src_count, workspace);
  if (rc != A2A_OK) return rc;
  hipStream_t st = (hipStream_t)hip_stream;
  if (src_count == 0) {
    if (unreachable) HIP_TRY(hipMemsetAsync(unreachable, 0, 8, st));
    if (flags) HIP_TRY(hipMemsetAsync(flags, 0, 8, st));
    return A2A_OK;
  }
  Run r;
  r.t = t;
  r.L = make_layout(t, src_count, sigma ? A2A_WS_SIGMA : A2A_WS_DISTANCES, workspace_bytes, false, false);
  if (r.L.G < 1) return A2A_ERR_WORKSPACE_TOO_SMALL;
  r.ws = (char*)workspace;
  r.st = st;
  r.src_begin = src_begin;
  r.src_count = src_count;
  const Layout& L = r.L;
  HIP_TRY(hipMemsetAsync(r.misc(), 0, 256, st));
  if (dist_sum) HIP_TRY(hipMemsetAsync(dist_sum, 0, (size_t)src_count * 8, st));
  const int nb = (src_count + 63) / 64;
  const int tiles = L.Npad / kWave;
  for (int b0 = 0; b0 < nb; b0 += L.G) {
    const int G = nb - b0 < L.G ? nb - b0 : L.G;
    int depth = 0;
    rc = run_bfs(r, b0, G, &depth);
    if (rc != A2A_OK) return rc;
    if (sigma) {
      rc = run_fwd(r, G, depth);
      if (rc != A2A_OK) return rc;
      ProfScope ps(t, PROF_EXTRACT, st);
      k_extract_sigma<<<grid_for(G, tiles), kWave, 0, st>>>(r.seen(), r.sig(), t->N, L.Npad, G, tiles,
                                                           src_count, b0, sigma);
    }
    if (dist || dist_sum) {
      ProfScope ps(t, PROF_EXTRACT, st);
      k_extract_dist<<<grid_for(G, tiles), kWave, 0, st>>>(r.lvl(), t->N, L.Npad, L.Lcap, G, tiles, depth,
                                                          src_count, b0, dist, (long long*)dist_sum);
    }
    rc = run_fold(r, G);
    if (rc != A2A_OK) return rc;
  }
  k_finish<<<1, 64, 0, st>>>(r.misc(), (long long)src_count * (t->N - 1), nullptr, (long long*)unreachable,
                             (long long*)flags, t->prof_on ? (long long*)t->d_small : nullptr);
  t->prof_calls++;
  HIP_TRY(hipGetLastError());
  return A2A_OK;
}

int a2a_link_loads(const a2a_topo* t, int32_t src_begin, int32_t src_count, double* load,
                   int64_t* dist_sum_total, int64_t* flags, void* workspace, size_t workspace_bytes,
                   void* hip_stream) {
  int rc = check_common(t, src_begin, src_count, workspace);
  if (rc != A2A_OK) return rc;
  if (!load && t->E > 0) return A2A_ERR_INVALID_ARG;
  hipStream_t st = (hipStream_t)hip_stream;
  if (src_count == 0) {
    if (t->E > 0) HIP_TRY(hipMemsetAsync(load, 0, (size_t)t->E * 8, st));
    if (dist_sum_total) HIP_TRY(hipMemsetAsync(dist_sum_total, 0, 8, st));
    if (flags) HIP_TRY(hipMemsetAsync(flags, 0, 8, st));
    return A2A_OK;
  }
  Run r;
  r.t = t;
  r.L = make_layout(t, src_count, A2A_WS_LOADS, workspace_bytes, false, false);
  if (r.L.G < 1) return A2A_ERR_WORKSPACE_TOO_SMALL;
  r.ws = (char*)workspace;
  r.st = st;
  r.src_begin = src_begin;
  r.src_count = src_count;
  const Layout& L = r.L;
  HIP_TRY(hipMemsetAsync(r.misc(), 0, 256, st));
  const int nb = (src_count + 63) / 64;
  const int bpb = (L.Npad + kBlock - 1) / kBlock;
  for (int b0 = 0; b0 < nb; b0 += L.G) {
    const int G = nb - b0 < L.G ? nb - b0 : L.G;
    int depth = 0;
    rc = run_bfs(r, b0, G, &depth);
    if (rc != A2A_OK) return rc;
    rc = run_fwd(r, G, depth);
    if (rc != A2A_OK) return rc;
    if (t->E > 0) {
      HIP_TRY(hipMemsetAsync(r.part(), 0, (size_t)G * L.Epad * 8, st));
      for (int l = depth; l >= 0; --l) {
        ProfScope ps(t, PROF_BWD, st);
        k_bwd_level<<<grid_for(G, bpb, r.inflight), kBlock, 0, st>>>(t->d_out_ptr, t->d_out_col, r.lvl(), r.sig(),
                                                         r.part(), L.Epad, t->N, L.Npad, L.Lcap, G, bpb, r.inflight, l);
      }
      ProfScope ps(t, PROF_REDUCE, st);
      k_reduce_part<<<(unsigned)((t->E + kBlock - 1) / kBlock), kBlock, 0, st>>>(r.part(), L.Epad, G,
                                                                                 (long long)t->E,
                                                                                 b0 == 0 ? 1 : 0, load);
    }
    rc = run_fold(r, G);
    if (rc != A2A_OK) return rc;
  }
  k_finish<<<1, 64, 0, st>>>(r.misc(), (long long)src_count * (t->N - 1), (long long*)dist_sum_total,
                             nullptr, (long long*)flags, t->prof_on ? (long long*)t->d_small : nullptr);
  t->prof_calls++;
  HIP_TRY(hipGetLastError());
  return A2A_OK;
}

int a2a_schedule_bound(const a2a_topo* t, const double* load, int64_t sum_dist, int64_t flags,
                       double m_bytes, double b_bytes_per_s, a2a_bound* out, void* hip_stream) {
  if (!t || !out || !load || t->E <= 0 || !(m_bytes > 0.0) || !(b_bytes_per_s > 0.0) || sum_dist < 0)
    return A2A_ERR_INVALID_ARG;
  hipStream_t st = (hipStream_t)hip_stream;
  k_load_extrema<<<1, 1024, 0, st>>>(load, (long long)t->E, (long long*)t->d_small);
  HIP_TRY(hipGetLastError());
  HIP_TRY(hipMemcpyAsync(t->h_pinned, t->d_small, 3 * sizeof(int64_t), hipMemcpyDeviceToHost, st));
  HIP_TRY(hipStreamSynchronize(st));
  double lmax, lmin;
  std::memcpy(&lmax, &t->h_pinned[0], 8);
  std::memcpy(&lmin, &t->h_pinned[2], 8);
  const double m = m_bytes, b = b_bytes_per_s;
  out->max_load = lmax;
  out->argmax_arc = t->h_pinned[1];
  out->min_load = lmin;
  out->sum_dist = sum_dist;
  out->n_links = t->E;
  out->n_nodes = t->N;
  out->dmax = t->dmax;
  out->t_sched = lmax * m / b;
  out->t_lb_nd = (double)sum_dist * m / ((double)t->N * (double)t->dmax * b);
  out->t_lb_links = (double)sum_dist * m / ((double)t->E * b);
  out->ratio = out->t_sched / out->t_lb_nd;
  out->throughput = (double)(t->N - 1) * m / out->t_sched;
  out->flow_value = 1.0 / lmax;
  out->throughput_upper = (double)(t->N - 1) * out->flow_value * b;
  return (flags & A2A_FLAG_UNREACHABLE) ? A2A_ERR_DISCONNECTED : A2A_OK;
}

int a2a_profile_enable(a2a_topo* t, int on) {
  if (!t) return A2A_ERR_INVALID_ARG;
  for (auto& rec : t->prof_recs) {
    (void)hipEventDestroy(rec.beg);
    (void)hipEventDestroy(rec.end);
  }
  t->prof_recs.clear();
  t->prof_calls = 0;
  t->prof_depth = 0;
  t->prof_groups = 0;
  t->prof_on = on != 0;
  HIP_TRY(hipMemset(t->d_small + 8, 0, 8 * sizeof(int64_t)));
  return A2A_OK;
}

int a2a_profile_read(a2a_topo* t, a2a_profile* out) {
  if (!t || !out) return A2A_ERR_INVALID_ARG;
  std::memset(out, 0, sizeof(*out));
  HIP_TRY(hipDeviceSynchronize());
  for (auto& rec : t->prof_recs) {
    float ms = 0.f;
    if (hipEventElapsedTime(&ms, rec.beg, rec.end) == hipSuccess && rec.cls >= 0 && rec.cls < PROF_CLASSES) {
      out->ms[rec.cls] += ms;
      out->launches[rec.cls] += 1;
    }
  }
  int64_t dag = 0;
  HIP_TRY(hipMemcpy(&dag, t->d_small + 8, sizeof(dag), hipMemcpyDeviceToHost));
  out->dag_links = dag;
  out->calls = t->prof_calls;
  out->depth = t->prof_depth;
  out->groups = t->prof_groups;
  return A2A_OK;
}

}  // extern "C"
