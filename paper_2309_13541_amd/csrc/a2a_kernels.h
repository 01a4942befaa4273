// Device code of a2a_topo (gfx950, wave64).  Included once, by a2a_topo.hip.
//
// Data model.  Sources are handled 64 at a time ("batch"): bit j of a 64-bit mask = source j of
// the batch, and lane j of a wavefront carries that source's floating-point state.  For every
// batch and BFS level l the index array holds, per node v, the mask L_l[v] of sources that
// reach v in exactly l hops (D(s,v) = l, the hop distance of Sec. 5.4) and an offset into the
// batch's value array.  The value array is level-compact: the entries of (l, v) are the
// popcount(L_l[v]) sources of that mask in lane order, rows follow each other in node order,
// levels follow each other.  Every reachable (source, node) pair owns exactly one entry, at the
// same position in two arrays: sigma(s,v) (number of shortest paths, Sec. 5.2), written by the
// forward pass, and coef(s,v) = (1 + delta(s,v)) / sigma(s,v), written by the backward pass,
// where delta is the traffic forwarded through v under the equal split of Sec. 5.2.  A link
// (u,w) is used by the sources in L_l[u] & L_{l+1}[w]; a gather of row (l,u) therefore reads
// popcount(L_l[u]) values instead of a 64-wide row, and a node's row is written once per pass
// instead of once per level.  coef is always double; sigma is kept as floats on the first
// levels, as long as (largest in-degree)^level < 2^24 bounds every path count of the level by a
// whole number that a float holds exactly, and as doubles from then on (GroupView::f32_levels).
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>

namespace a2a_dev {

constexpr int kWave = 64;
constexpr int kBlock = 256;  // threads per workgroup = nodes per node block
constexpr int kWavesPerBlock = kBlock / kWave;
constexpr int kXcd = 8;      // workgroups are dealt round-robin to 8 XCDs
constexpr double kTwo53 = 9007199254740992.0;
// Up to this many (source, link) pairs per node the backward kernel adds the products lane by
// lane; beyond it the eight-way wave reduction is cheaper.
constexpr int kSerialPairs = 6;

// One node of one (batch, level): 16 bytes so that mask and offset arrive in one request.
struct __align__(16) NodeIdx {
  uint64_t mask;  // L_level[v]
  uint32_t off;   // first entry of the row in the batch's value array
  uint32_t pad;
};

// ---------------------------------------------------------------------------------------
// lane helpers
// ---------------------------------------------------------------------------------------

__device__ __forceinline__ int lane_id() { return (int)(threadIdx.x & (kWave - 1)); }

__device__ __forceinline__ uint64_t readlane64(uint64_t x, int k) {
  const uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)x, k);
  const uint32_t hi = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(x >> 32), k);
  return ((uint64_t)hi << 32) | lo;
}

__device__ __forceinline__ uint64_t shfl64(uint64_t x, int src_lane) {
  const uint32_t lo = (uint32_t)__shfl((int)(uint32_t)x, src_lane, kWave);
  const uint32_t hi = (uint32_t)__shfl((int)(uint32_t)(x >> 32), src_lane, kWave);
  return ((uint64_t)hi << 32) | lo;
}

// Number of set bits of m below this lane: the rank of the lane's entry in a compact row.
__device__ __forceinline__ uint32_t rank_in(uint64_t m) {
  return __builtin_amdgcn_mbcnt_hi((uint32_t)(m >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m, 0u));
}

// True in exactly the lanes whose bit is set in the wave-uniform mask m.  Lowers to a copy of
// m into the execution mask: no per-lane compare.
__device__ __forceinline__ bool lane_in(uint64_t m) { return __builtin_amdgcn_inverse_ballot_w64(m); }

// Entry `e` of a batch's value array.  The 32-bit byte offset keeps the address computation to
// one instruction (uniform base + per-lane offset); a batch's array is Npad*64*8 bytes, which
// the host keeps below 4 GiB.
__device__ __forceinline__ double& entry(double* __restrict__ dat, uint32_t e) {
  return *reinterpret_cast<double*>(reinterpret_cast<char*>(dat) + (size_t)(e * 8u));
}
__device__ __forceinline__ const double& entry(const double* __restrict__ dat, uint32_t e) {
  return *reinterpret_cast<const double*>(reinterpret_cast<const char*>(dat) + (size_t)(e * 8u));
}

// The same position in the batch's single-precision copy of sigma.
__device__ __forceinline__ float& entry(float* __restrict__ datf, uint32_t e) {
  return *reinterpret_cast<float*>(reinterpret_cast<char*>(datf) + (size_t)(e * 4u));
}
__device__ __forceinline__ const float& entry(const float* __restrict__ datf, uint32_t e) {
  return *reinterpret_cast<const float*>(reinterpret_cast<const char*>(datf) + (size_t)(e * 4u));
}

// Returns x unchanged, as far as the compiler can tell a new value: a conversion applied to the
// result stays here instead of being moved up to the load that produced x, where it would make
// the wave wait for that load before the next one is issued.
__device__ __forceinline__ float hold(float x) {
  asm volatile("" : "+v"(x));
  return x;
}
__device__ __forceinline__ double hold(double x) { return x; }  // nothing is converted
__device__ __forceinline__ uint32_t hold(uint32_t x) {
  asm volatile("" : "+v"(x));
  return x;
}

// 16-byte piece number q of a batch's value array in one request: two doubles or four floats.
// The words stay as they are until piece_get picks an entry, so that nothing waits for the data
// before it is needed.
template <typename T>
__device__ __forceinline__ uint4 piece(const T* __restrict__ rows, uint32_t q) {
  return *reinterpret_cast<const uint4*>(reinterpret_cast<const char*>(rows) + (size_t)(q * 16u));
}
template <typename T>
__device__ __forceinline__ double piece_get(const uint4& r, int k);
template <>
__device__ __forceinline__ double piece_get<double>(const uint4& r, int k) {
  return k ? __hiloint2double((int)r.w, (int)r.z) : __hiloint2double((int)r.y, (int)r.x);
}
template <>
__device__ __forceinline__ double piece_get<float>(const uint4& r, int k) {
  return (double)__uint_as_float(hold(k == 0 ? r.x : k == 1 ? r.y : k == 2 ? r.z : r.w));
}

// 1/x for x >= 1: hardware estimate plus two Newton steps (relative error about 1e-16).
__device__ __forceinline__ double recip(double x) {
  double r = __builtin_amdgcn_rcp(x);
  r = __builtin_fma(__builtin_fma(-x, r, 1.0), r, r);
  r = __builtin_fma(__builtin_fma(-x, r, 1.0), r, r);
  return r;
}

__device__ __forceinline__ NodeIdx load_idx(const NodeIdx* __restrict__ p) {
  const ulonglong2 r = *reinterpret_cast<const ulonglong2*>(p);
  NodeIdx n;
  n.mask = r.x;
  n.off = (uint32_t)r.y;
  n.pad = 0;
  return n;
}

// Lane exchange with lane ^ kMask for a 64-bit value.
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

// The same for a 32-bit value (masks below 8 only).
template <int kMask>
__device__ __forceinline__ float xor_lanes(float x) {
  static_assert(kMask == 1 || kMask == 2 || kMask == 4, "exchange inside a group of eight lanes");
  const int a = __float_as_int(x);
  int b;
  if constexpr (kMask == 1) {
    b = __builtin_amdgcn_mov_dpp(a, 0xB1, 0xF, 0xF, true);
  } else if constexpr (kMask == 2) {
    b = __builtin_amdgcn_mov_dpp(a, 0x4E, 0xF, 0xF, true);
  } else {
    b = __builtin_amdgcn_ds_swizzle(a, 0x1F | (kMask << 10));
  }
  return __int_as_float(b);
}

// Eight sums over groups of eight lanes at once.  x[i] is lane-local; on return lane l holds the
// sum of x[l & 7] over the eight lanes 8*(l>>3) .. 8*(l>>3)+7.  Halving the value set at each
// exchange step costs 4+2+1 exchanges instead of 8*3, in a fixed order (so results are
// reproducible).
template <typename T>
__device__ __forceinline__ T group_sum8(const T (&x)[8], int lane) {
  const bool b0 = lane & 1, b1 = lane & 2, b2 = lane & 4;
  T y[4], z[2];
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    const T keep = b0 ? x[2 * k + 1] : x[2 * k];
    const T send = b0 ? x[2 * k] : x[2 * k + 1];
    y[k] = keep + xor_lanes<1>(send);
  }
#pragma unroll
  for (int k = 0; k < 2; ++k) {
    const T keep = b1 ? y[2 * k + 1] : y[2 * k];
    const T send = b1 ? y[2 * k] : y[2 * k + 1];
    z[k] = keep + xor_lanes<2>(send);
  }
  const T keep = b2 ? z[1] : z[0];
  const T send = b2 ? z[0] : z[1];
  return keep + xor_lanes<4>(send);  // lane l: sum of x[l & 7] over the eight lanes of its group
}

// Eight 64-lane sums at once through LDS: on return every lane l holds the sum over all 64 lanes
// of x[l & 7].  Each lane stores its eight values (one row of 64 per value, rows
// padded by one to spread the banks), lane l then adds the eight values of x[l & 7] that lanes
// 8*(l>>3) .. 8*(l>>3)+7 stored, and three exchange steps add the eight partial sums.  Seven
// plus three additions on the vector ALU instead of 4+2+1+3 select-and-add rounds; the moves
// go through the LDS pipeline.  `buf` is this wave's kSum8Doubles doubles of LDS.
constexpr int kSum8Row = kWave + 1;
constexpr int kSum8Doubles = 8 * kSum8Row;
// LDS of a wave of the backward kernel: 7.5 KB (30 KB per workgroup: five workgroups per compute unit, which is
// what the registers allow; with 32 KB only four fit).  Rows layout: the eight sums, then the staged coef rows
// of a tile.
constexpr int kBwdDoubles = 15 * kWave;
constexpr int kStageDoubles = kBwdDoubles - kSum8Doubles;
__device__ __forceinline__ double wave_sum8_lds(const double (&x)[8], int lane, double* buf) {
#pragma unroll
  for (int j = 0; j < 8; ++j) buf[j * kSum8Row + lane] = x[j];
  __builtin_amdgcn_wave_barrier();
  const double* row = buf + (lane & 7) * kSum8Row + (lane & ~7);
  double w = row[0];
#pragma unroll
  for (int r = 1; r < 8; ++r) w += row[r];
  __builtin_amdgcn_wave_barrier();
  w += xor_lanes<8>(w);
  w += xor_lanes<16>(w);
  w += xor_lanes<32>(w);
  return w;
}

__device__ __forceinline__ int wave_sum_int(int x) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) x += __shfl_xor(x, o, kWave);
  return x;
}

// Inclusive prefix sum over the lanes of a wave.
__device__ __forceinline__ int wave_scan_incl(int x, int lane) {
#pragma unroll
  for (int o = 1; o < kWave; o <<= 1) {
    const int y = __shfl_up(x, o, kWave);
    if (lane >= o) x += y;
  }
  return x;
}

// Workgroups go round-robin to the 8 XCDs, each with its own L2.  `inflight` consecutive
// workgroups belong to `inflight` different batches (or super-batches); with inflight = 8 all
// workgroups of one batch run on one XCD, so that the small per-level arrays of that batch
// (masks, offsets, the rows of sparsely populated levels) stay in that XCD's L2 while its waves
// gather from them.
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
  return cnt >= 64 ? ~0ull : (cnt <= 0 ? 0ull : ((1ull << cnt) - 1ull));
}

// The BFS works on super-batches of kSub batches: the masks of one node for the kSub batches
// lie next to each other (64 bytes), so that the kSub lanes that look at the same in-neighbour
// share one memory request.
#ifndef A2A_KSUB
#define A2A_KSUB 8
#endif
constexpr int kSub = A2A_KSUB;
constexpr int kBfsNodes = 64;                    // nodes per BFS workgroup
constexpr int kBfsBlock = kBfsNodes * kSub;      // threads: kBfsNodes nodes x kSub batches
constexpr int kBfsWaves = kBfsBlock / kWave;

// Everything a level kernel needs to find its batch's arrays.  G batches; SB = ceil(G/kSub)
// super-batches (batches past G exist only in the BFS arrays and stay empty).
struct GroupView {
  uint64_t* bm;       // [SB][Lcap][Npad][kSub] BFS level masks L_l[v]
  uint64_t* seen;     // [SB][Npad][kSub]
  NodeIdx* idxb;      // [G][Lcap][Npad]  mask + row offset per batch (nullptr: distances only)
  double* dat;        // [G][Npad*64]  level-compact sigma of the levels from f32_levels on (nullptr:
                      //               distances only)
  float* datf;        // the same memory: sigma of the levels below f32_levels, entry e = the e-th float
                      //               of the batch's array.  Levels on which every path count is certain
                      //               to be below 2^24 keep it in single precision only (exact, half the
                      //               bytes); they come first in the array, so their floats end before
                      //               the first double of a later level begins
  double* coef;       // [G][Npad*64]  level-compact coef (link loads only)
  int* bsum;          // [SB*kSub][Lcap][nb64] newly reached pairs per 64-node block and level;
                      //                       after k_scan_blocks: first entry of the block's rows
  long long* ltot;    // [SB*kSub][Lcap]   newly reached pairs per level
  long long* dag;     // [G][Lcap]      (source, link) pairs into each level (profiling mode 2)
  double* part;       // [G][Epad]      per-batch link loads
  size_t Epad;
  int N, Npad, Lcap, G, SB, bpb, nb64, inflight;
  int split;          // waves that share a block of 64 nodes in k_fwd / k_bwd (1, 2, 4 or 8; above 1 the
                      // kShared kernels are launched; 1 with demands and while shortest-path links are counted)
  int src_begin, src_count, batch0;
  int f32_levels;     // >= 1
  // Commodities of unequal demand (nullptr: every pair has demand 1): demand of source
  // src_begin + j to node t at dem[t * dem_ld + j], and per (batch, 64-node block) the sum of
  // demand x distance over the pairs the backward pass has visited.
  const double* dem;
  long long dem_ld;
  double* wpart;      // [G][nb64]
};

// The demands of one batch's sources: row t = node t, entry j = source j of the batch.
__device__ __forceinline__ const double* demand_rows(const GroupView& gv, int g) {
  return gv.dem + (size_t)(gv.batch0 + g) * 64;
}

// Sum over the lanes, the same in every lane and from run to run.
__device__ __forceinline__ double wave_sum_double(double x) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) x += __shfl_xor(x, o, kWave);
  return x;
}

// Adds level x (a wave's sum of the demands it met) to its (batch, block) slot.
__device__ __forceinline__ void add_weighted_dist(const GroupView& gv, int g, int u0, int level, double lane_sum) {
  const double tot = wave_sum_double(lane_sum);
  if (lane_id() == 0 && tot != 0.0) gv.wpart[(size_t)g * gv.nb64 + u0 / kWave] += (double)level * tot;
}


// The batch's sigma array of the given precision.
template <typename T>
__device__ __forceinline__ T* sigma_rows(const GroupView& gv, int g);
template <>
__device__ __forceinline__ double* sigma_rows<double>(const GroupView& gv, int g) {
  return gv.dat + (size_t)g * gv.Npad * 64;
}
template <>
__device__ __forceinline__ float* sigma_rows<float>(const GroupView& gv, int g) {
  return gv.datf + (size_t)g * gv.Npad * 128;  // the batch's array counted in floats
}

__device__ __forceinline__ size_t bm_at(const GroupView& gv, int sb, int level, int v, int k) {
  return ((((size_t)sb * gv.Lcap + level) * gv.Npad) + v) * kSub + k;
}

// ---------------------------------------------------------------------------------------
// BFS
// ---------------------------------------------------------------------------------------

// Level 0: bit j of L_0[s_j] and seen[s_j] for the batch's sources s_j; sigma(s_j,s_j) = 1 is
// entry j of the value array.  One thread per (node, batch of the super-batch).
__global__ void __launch_bounds__(kBfsBlock) k_init_group(GroupView gv) {
  int sb, nblk;
  if (!map_block(gv.SB, gv.nb64, kXcd, sb, nblk)) return;
  const int t = (int)threadIdx.x;
  const int v = nblk * kBfsNodes + t / kSub, k = t % kSub;
  const int g = sb * kSub + k;
  const int s0 = gv.src_begin + (gv.batch0 + g) * 64;
  // batches past the group's last one only pad the super-batch: no sources
  const int cnt = g < gv.G ? max(0, min(64, gv.src_begin + gv.src_count - s0)) : 0;
  const int j = v - s0;
  const bool is_src = (v < gv.N) && j >= 0 && j < cnt;
  const uint64_t bit = is_src ? (1ull << j) : 0ull;
  gv.bm[bm_at(gv, sb, 0, v, k)] = bit;
  gv.seen[((size_t)sb * gv.Npad + v) * kSub + k] = bit;
  if (gv.datf != nullptr && is_src) gv.datf[(size_t)g * gv.Npad * 128 + j] = 1.0f;  // level 0 is always narrow
  if (v == 0) {
    gv.ltot[(size_t)g * gv.Lcap] = cnt;
    if (g < gv.G)
      for (int l = 0; l < gv.Lcap; ++l) gv.dag[(size_t)g * gv.Lcap + l] = 0;
  }
}

// One BFS level for every batch of the group, pull direction:
// L_l[v] = (OR over in-neighbours u of L_{l-1}[u]) & ~seen[v].
// Thread (node, k): the kSub lanes of a node read the same in-link list and adjacent masks.
__global__ void __launch_bounds__(kBfsBlock)
k_bfs_level(const int32_t* __restrict__ in_ptr, const int32_t* __restrict__ in_col, GroupView gv,
            int level) {
  int sb, nblk;
  if (!map_block(gv.SB, gv.nb64, kXcd, sb, nblk)) return;
  const int t = (int)threadIdx.x;
  const int v = nblk * kBfsNodes + t / kSub, k = t % kSub;
  const int g = sb * kSub + k;
  const uint64_t* __restrict__ prev = gv.bm + bm_at(gv, sb, level - 1, 0, k);
  uint64_t nw = 0;
  if (v < gv.N) {
    const size_t si = ((size_t)sb * gv.Npad + v) * kSub + k;
    const uint64_t sn = gv.seen[si];
    const uint64_t valid = g < gv.G ? valid_mask(gv.src_count, gv.batch0 + g) : 0ull;
    if (sn != valid) {
      uint64_t acc = 0;
      const int p1 = in_ptr[v + 1];
      for (int p = in_ptr[v]; p < p1; p += 8) {  // eight in-links at a time, all requests in flight
        int u[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) u[j] = p + j < p1 ? in_col[p + j] : -1;
#pragma unroll
        for (int j = 0; j < 8; ++j)
          if (u[j] >= 0) acc |= prev[(size_t)u[j] * kSub];
      }
      nw = acc & ~sn;
      if (nw) gv.seen[si] = sn | nw;
    }
  }
  gv.bm[bm_at(gv, sb, level, v, k)] = nw;
  // newly reached (source, node) pairs of this 64-node block, per batch
  __shared__ int s_cnt[kSub];
  if (t < kSub) s_cnt[t] = 0;
  __syncthreads();
  int pc = __popcll(nw);
#pragma unroll
  for (int o = kSub; o < kWave; o <<= 1) pc += __shfl_xor(pc, o, kWave);
  if (lane_id() < kSub && pc != 0) atomicAdd(&s_cnt[k], pc);
  __syncthreads();
  if (t < kSub) {
    const int tot = s_cnt[t];
    gv.bsum[((size_t)g * gv.Lcap + level) * gv.nb64 + nblk] = tot;
    if (tot > 0) atomicAdd((unsigned long long*)&gv.ltot[(size_t)g * gv.Lcap + level], (unsigned long long)tot);
  }
}

// bsum[g][l][*] (pairs per 64-node block) -> position of the block's first row in the batch's
// value array: exclusive prefix over blocks, after all rows of the levels above.  One wave per
// (batch, level), levels 1..depth.
__global__ void __launch_bounds__(kWave) k_scan_blocks(GroupView gv, int depth) {
  const int g = (int)blockIdx.x / depth, level = 1 + (int)blockIdx.x % depth;
  const int lane = lane_id();
  const long long* __restrict__ lt = gv.ltot + (size_t)g * gv.Lcap;
  long long carry = 0;
  for (int l = 0; l < level; ++l) carry += lt[l];
  int* __restrict__ bs = gv.bsum + ((size_t)g * gv.Lcap + level) * gv.nb64;
  for (int b0 = 0; b0 < gv.nb64; b0 += kWave) {
    const int b = b0 + lane;
    const int c = b < gv.nb64 ? bs[b] : 0;
    const int incl = wave_scan_incl(c, lane);
    if (b < gv.nb64) bs[b] = (int)(carry + incl - c);
    carry += __shfl(incl, kWave - 1, kWave);
  }
}

// Index array from the BFS masks: idxb[g][l][v] = { L_l[v], first entry of the row }.
// Thread (node, k) as in the BFS; the row offsets are an exclusive prefix over nodes for each
// batch k (three shuffle steps across the 8 nodes of a wave, then across the 8 waves via LDS).
// A workgroup takes `levels` consecutive levels of its 64 nodes (all of them in a large group; one
// each, in as many workgroups, where the group is too small to fill the chip otherwise).
__global__ void __launch_bounds__(kBfsBlock) k_write_offsets(GroupView gv, int depth, int levels) {
  const int chunks = (depth + levels) / levels;  // levels 0 .. depth
  int sb, unit;
  if (!map_block(gv.SB, gv.nb64 * chunks, kXcd, sb, unit)) return;
  const int nblk = unit / chunks, l0 = unit % chunks * levels;
  const int l1 = min(depth, l0 + levels - 1);
  __shared__ int s_w[kBfsWaves][kSub];
  __shared__ NodeIdx s_n[kSub][kBfsNodes + 1];
  const int t = (int)threadIdx.x, lane = lane_id(), wid = t / kWave;
  const int v = nblk * kBfsNodes + t / kSub, k = t % kSub;
  const int g = sb * kSub + k;
  for (int l = l0; l <= l1; ++l) {
    const uint64_t m = gv.bm[bm_at(gv, sb, l, v, k)];
    NodeIdx n;
    n.mask = m;
    n.pad = 0;
    if (l == 0) {
      n.off = m ? (uint32_t)__builtin_ctzll(m) : 0u;  // source j owns entry j
    } else {
      const int c = __popcll(m);
      int x = c;  // inclusive prefix over the wave's nodes, per batch
#pragma unroll
      for (int o = kSub; o < kWave; o <<= 1) {
        const int y = __shfl_up(x, o, kWave);
        if (lane >= o) x += y;
      }
      if (lane >= kWave - kSub) s_w[wid][k] = x;
      __syncthreads();
      int base = g < gv.G ? gv.bsum[((size_t)g * gv.Lcap + l) * gv.nb64 + nblk] : 0;
      for (int w = 0; w < wid; ++w) base += s_w[w][k];
      n.off = (uint32_t)(base + x - c);
      __syncthreads();
    }
    // transpose through LDS: wave w writes the 64 consecutive entries of batch sb*kSub+w
    s_n[k][t / kSub] = n;
    __syncthreads();
    const int gw = sb * kSub + wid;
    if (gw < gv.G) gv.idxb[((size_t)gw * gv.Lcap + l) * gv.Npad + nblk * kBfsNodes + lane] = s_n[wid][lane];
    __syncthreads();
  }
}

// ---------------------------------------------------------------------------------------
// forward: path counts
// ---------------------------------------------------------------------------------------

// --- well-filled levels: one wave per (batch, node) -------------------------------------
//
// A wave owns 64 consecutive nodes of one batch; lane j = source j.  It works through the nodes
// eight at a time ("group"): the 64 lanes first fetch (neighbour, mask, offset) for 8 nodes x 8
// links at once (an "index tile": lane 8i+j looks at link j of node i), then each node's
// sources gather from the compact rows of its links.  Three things keep enough memory requests
// in flight: the neighbour ids of the group after next and the index tile of the next group are
// requested while the current group is worked on, and the eight row gathers of node i+1 are
// issued before the values of node i are used.  Nodes with more than 8 links take further,
// unpipelined, rounds.

struct Tile {
  uint64_t mask;  // L[neighbour] of this lane's link (0: no link)
  uint32_t off;   // its row offset
};

// Which of the (up to) eight tiles of its 64 nodes a wave works on: first, first + step, ...  {0, 1}: all
// of them, the normal case.  Where a topology is too small to fill the chip, `step` waves share a block of
// 64 nodes (tile c of the block belongs to the wave with first = c mod step): the chain of dependent
// memory requests that a wave goes through gets shorter by that factor.
struct TileShare {
  int first, step;
};

// In- or out-link range of the 64 nodes, one node per lane; nothing for nodes not on this level.
struct LinkRange {
  int p0, p1;
};

__device__ __forceinline__ int tile_request_col(const int32_t* __restrict__ col, const LinkRange& lr, int c,
                                                int base, int lane, int& q) {
  const int src = 8 * c + (lane >> 3);
  const int p0 = __shfl(lr.p0, src, kWave), p1 = __shfl(lr.p1, src, kWave);
  q = p0 + base + (lane & 7);
  if (q >= p1) q = -1;
  return q >= 0 ? col[q] : -1;
}

__device__ __forceinline__ Tile tile_request_idx(const NodeIdx* __restrict__ level, int nb) {
  Tile t;
  t.mask = 0;
  t.off = 0;
  if (nb >= 0) {
    const NodeIdx n = load_idx(level + nb);
    t.mask = n.mask;
    t.off = n.off;
  }
  return t;
}

// Sparse levels: most of a wave's 64 nodes have no source on the level, and a tile of eight nodes costs
// the same with one node on it as with eight.  This moves the per-node values of the nodes in `active`
// to the lowest lanes (in node order; the others follow behind them) and returns their number, so that
// the tiles are filled from the front and only ceil(count / 8) of them are visited.  nid: the node's id.
__device__ __forceinline__ int compact_nodes(uint64_t active, int lane, NodeIdx& me, LinkRange& lr, int& nid) {
  const int count = __popcll(active);
  if (count == kWave) return count;
  const int r = (int)rank_in(active);
  const int dst = 4 * (((active >> lane) & 1ull) ? r : count + lane - r);  // a permutation of the lanes
  const uint32_t lo = (uint32_t)__builtin_amdgcn_ds_permute(dst, (int)(uint32_t)me.mask);
  const uint32_t hi = (uint32_t)__builtin_amdgcn_ds_permute(dst, (int)(uint32_t)(me.mask >> 32));
  me.mask = ((uint64_t)hi << 32) | lo;
  me.off = (uint32_t)__builtin_amdgcn_ds_permute(dst, (int)me.off);
  lr.p0 = __builtin_amdgcn_ds_permute(dst, lr.p0);
  lr.p1 = __builtin_amdgcn_ds_permute(dst, lr.p1);
  nid = __builtin_amdgcn_ds_permute(dst, nid);
  return count;
}

// Issues the (up to) eight row gathers of node i of the current tile: lanes in mk & want read
// their entry of the link's row.  Returns the number of (source, link) pairs.
template <typename T>
__device__ __forceinline__ int gather8(const T* __restrict__ rows, const Tile& tile, int i, uint64_t want,
                                       T (&x)[8], uint64_t (&m)[8]) {
  int pairs = 0;
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    const uint64_t mk = readlane64(tile.mask, 8 * i + j);
    m[j] = mk & want;
    x[j] = (T)0;
    if (m[j] != 0) {  // uniform: skip links that carry nothing for this node
      const uint32_t of = (uint32_t)__builtin_amdgcn_readlane((int)tile.off, 8 * i + j);
      pairs += __popcll(m[j]);
      if (lane_in(m[j])) x[j] = entry(rows, of + rank_in(mk));
    }
  }
  return pairs;
}

// The rows of the (up to eight) nodes of a tile are adjacent in a batch's level-compact array:
// entries of0 .. end - 1, of0 = where the first of the tile's nodes that is on the level starts.
struct TileSpan {
  uint32_t of0, end;
};
__device__ __forceinline__ TileSpan tile_span(const NodeIdx& me, uint64_t nodes_active, int c) {
  const uint32_t on = (uint32_t)(nodes_active >> (8 * c)) & 0xffu;  // not 0
  const int first = 8 * c + __builtin_ctz(on), last = 8 * c + 31 - __builtin_clz(on);
  TileSpan t;
  t.of0 = (uint32_t)__builtin_amdgcn_readlane((int)me.off, first);
  t.end = (uint32_t)__builtin_amdgcn_readlane((int)me.off, last) + (uint32_t)__popcll(readlane64(me.mask, last));
  return t;
}

// The span's entries from their copy in LDS (stage[0] = entry of0), 64 at a time; every store but the
// first starts on a 128-byte boundary of the array, so whole lines go out.  The stores are marked
// non-temporal: the rows are read again by a later launch only, and left in the L2 they push out the
// index entries that this launch keeps coming back to.
template <typename T>
__device__ __forceinline__ void store_staged(T* __restrict__ arr, const T* __restrict__ stage, TileSpan t, int lane) {
  constexpr uint32_t kPerLine = 128 / sizeof(T);
  for (int k = lane - (int)(t.of0 & (kPerLine - 1)); (int)t.of0 + k < (int)t.end; k += kWave)
    if (k >= 0) __builtin_nontemporal_store(stage[k], &entry(arr, t.of0 + (uint32_t)k));
}

// One level of sigma(s,v) = sum over in-links (u,v) with D(s,u) = D(s,v) - 1 of sigma(s,u).
// cf (may be null): the deepest level's coef is just 1/sigma, which goes there now.
// The gathered values are widened here, where they are used, so that the requests stay in
// flight until then.  sigma goes to `stage`, the LDS copy of the tile's piece of the sigma array
// (stage[0] = entry of0), which the caller stores when the tile is done.
template <typename TIn, typename TOut>
__device__ __forceinline__ bool fwd_finish(TOut* __restrict__ stage, uint32_t of0, double* __restrict__ cf,
                                           const NodeIdx& me, int node, const TIn (&x)[8]) {
  // A level kept in single precision has all its path counts below 2^24 (the host's bound), so every
  // partial sum of these whole numbers is below 2^24 too: adding them as floats is exact.
  TOut a = (TOut)0;
#pragma unroll
  for (int j = 0; j < 8; ++j) a += (TOut)hold(x[j]);
  const uint64_t newv = readlane64(me.mask, node);
  const uint32_t of = (uint32_t)__builtin_amdgcn_readlane((int)me.off, node);
  bool big = false;
  if (lane_in(newv)) {
    const uint32_t e = of + rank_in(newv);
    stage[e - of0] = a;
    if (cf != nullptr) entry(cf, e) = recip((double)a);
    if constexpr (sizeof(TOut) == 8) big = a >= kTwo53;
  }
  return big;
}

// TIn / TOut: precision in which the level before / this level keeps sigma (the host's choice).
template <bool kCountDag, typename TIn, typename TOut>
__device__ __forceinline__ void
fwd_rows(const int32_t* __restrict__ in_ptr, const int32_t* __restrict__ in_col, const GroupView& gv,
         int level, bool init_coef, long long* __restrict__ misc, int g, int v0, TOut* __restrict__ stage,
         const TileShare& ts, const NodeIdx& me, const LinkRange& lr) {
  const int lane = lane_id();
  const NodeIdx* __restrict__ cur = gv.idxb + ((size_t)g * gv.Lcap + level) * gv.Npad;
  const NodeIdx* __restrict__ prev = cur - gv.Npad;
  const TIn* __restrict__ rows = sigma_rows<TIn>(gv, g);
  TOut* __restrict__ out = sigma_rows<TOut>(gv, g);
  double* __restrict__ cf = init_coef ? gv.coef + (size_t)g * gv.Npad * 64 : nullptr;
  const uint64_t nodes_active = __ballot(me.mask != 0);
  if (nodes_active == 0) return;
  bool inexact = false;
  long long dag = 0;
  int q;
  Tile tile = tile_request_idx(prev, tile_request_col(in_col, lr, ts.first, 0, lane, q));
  int nb_next = ts.first + ts.step < 8 ? tile_request_col(in_col, lr, ts.first + ts.step, 0, lane, q) : -1;
#pragma unroll 1
  for (int c = ts.first; c < 8; c += ts.step) {
    const Tile tile_next = tile_request_idx(prev, c + ts.step < 8 ? nb_next : -1);
    nb_next = c + 2 * ts.step < 8 ? tile_request_col(in_col, lr, c + 2 * ts.step, 0, lane, q) : -1;
    if (((nodes_active >> (8 * c)) & 0xffull) != 0) {
      TIn xa[8], xb[8];
      uint64_t m[8];
      const TileSpan span = tile_span(me, nodes_active, c);
      int pairs = gather8(rows, tile, 0, readlane64(me.mask, 8 * c), xa, m);
#pragma unroll 1
      for (int i = 0; i < 8; i += 2) {  // two nodes per round, the next one's rows always in flight
        pairs += gather8(rows, tile, i + 1, readlane64(me.mask, 8 * c + i + 1), xb, m);
        inexact |= fwd_finish(stage, span.of0, cf, me, 8 * c + i, xa);
        if (i + 2 < 8) pairs += gather8(rows, tile, i + 2, readlane64(me.mask, 8 * c + i + 2), xa, m);
        inexact |= fwd_finish(stage, span.of0, cf, me, 8 * c + i + 1, xb);
      }
      if (kCountDag) dag += pairs;
      // nodes with more than eight in-links: add the rest to the staged entries
      const int p0 = __shfl(lr.p0, 8 * c + (lane >> 3), kWave), p1 = __shfl(lr.p1, 8 * c + (lane >> 3), kWave);
      for (int base = 8; __ballot(p0 + base < p1) != 0; base += 8) {
        const Tile extra = tile_request_idx(prev, tile_request_col(in_col, lr, c, base, lane, q));
#pragma unroll 1
        for (int i = 0; i < 8; ++i) {
          const uint64_t newv = readlane64(me.mask, 8 * c + i);
          const int np = gather8(rows, extra, i, newv, xa, m);
          if (np == 0) continue;
          if (kCountDag) dag += np;
          double a = 0.0;
#pragma unroll
          for (int j = 0; j < 8; ++j) a += (double)hold(xa[j]);
          const uint32_t of = (uint32_t)__builtin_amdgcn_readlane((int)me.off, 8 * c + i);
          if (lane_in(newv)) {
            const uint32_t pos = of + rank_in(newv);
            a += (double)stage[pos - span.of0];  // written by this lane
            stage[pos - span.of0] = (TOut)a;
            if (cf != nullptr) entry(cf, pos) = recip(a);
            inexact |= a >= kTwo53;
          }
        }
      }
      __builtin_amdgcn_wave_barrier();
      store_staged(out, stage, span, lane);
      __builtin_amdgcn_wave_barrier();
    }
    tile = tile_next;
  }
  if (inexact) misc[0] = 1;
  if (kCountDag && dag != 0 && lane == 0)
    atomicAdd((unsigned long long*)&gv.dag[(size_t)g * gv.Lcap + level], (unsigned long long)dag);
}

// ---------------------------------------------------------------------------------------
// backward: dependency recursion and link loads
// ---------------------------------------------------------------------------------------

// One level of coef(s,u) = 1/sigma(s,u) + sum over out-links (u,w) with D(s,w) = D(s,u) + 1 of
// coef(s,w), and load(u,w) += sum over sources of sigma(s,u) * coef(s,w): the share of the unit
// demands that the equal split over shortest paths (Sec. 5.2) routes over the link.  After the
// eight-way wave reduction lane 8i+j holds the load of out-link j of node i, which is the lane
// that fetched that link's id: one coalesced read-modify-write of the batch's link loads per
// group.
__device__ __forceinline__ double link_sums(double (&x)[8], const uint64_t (&m)[8], int pairs, int i, int lane,
                                            double tot_l, double* sum8_buf) {
  if (pairs > kSerialPairs) {
    const double tot = wave_sum8_lds(x, lane, sum8_buf);  // lane l: load of link (l & 7) of node i
    if ((lane >> 3) == i) tot_l = tot;
  } else {
    // few (source, link) pairs: pick the products out lane by lane instead of reducing
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      uint64_t mm = m[j];
      if (mm == 0) continue;
      double sum = 0.0;
      while (mm) {
        const int l = __builtin_ctzll(mm);
        mm &= mm - 1;
        sum += __longlong_as_double((long long)readlane64((uint64_t)__double_as_longlong(x[j]), l));
      }
      if (lane == 8 * i + j) tot_l = sum;
    }
  }
  return tot_l;
}

// Own sigma of a node (1 in lanes that are not on this level), requested together with the rows.
// Demand of the node's sources (a lane each; 1 where the lane is not on this level or all demands are 1).
template <bool kDemand>
__device__ __forceinline__ double own_demand(const double* __restrict__ dem, long long ld, int u0, const NodeIdx& me,
                                             int node, int lane) {
  double d = 1.0;
  if constexpr (kDemand) {
    if (lane_in(readlane64(me.mask, node))) d = dem[(size_t)(u0 + node) * (size_t)ld + lane];
  }
  return d;
}

template <typename TS>
__device__ __forceinline__ TS own_sigma(const TS* __restrict__ dat, const NodeIdx& me, int node) {
  const uint64_t mu = readlane64(me.mask, node);
  const uint32_t of = (uint32_t)__builtin_amdgcn_readlane((int)me.off, node);
  TS s = (TS)1;
  if (lane_in(mu)) s = entry(dat, of + rank_in(mu));
  return s;
}

// coef of a node from its sigma and the gathered coef rows (x, overwritten by the products that
// the link loads are made of); `add`: further round of a node with more than eight links.  The coef
// goes to `stage` (unless null), the LDS copy of the coef rows of the tile's nodes (entry of0 of the
// batch's array onwards), which the caller stores when the tile is done.
template <typename TS>
__device__ __forceinline__ double bwd_finish(double* __restrict__ cf, const NodeIdx& me, int node, int i, TS sigma,
                                             double dem, double (&x)[8], const uint64_t (&m)[8], int pairs, bool add,
                                             int lane, double tot_l, double* sum8_buf, double* __restrict__ stage,
                                             uint32_t of0) {
  const double s = (double)hold(sigma);
  double a = 0.0;
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    a += x[j];
    x[j] *= s;
  }
  const uint64_t mu = readlane64(me.mask, node);
  const uint32_t of = (uint32_t)__builtin_amdgcn_readlane((int)me.off, node);
  if (lane_in(mu)) {
    double& e = stage != nullptr ? stage[of - of0 + rank_in(mu)] : entry(cf, of + rank_in(mu));
    e = add ? e + a : dem * recip(s) + a;
  }
  if (pairs != 0) tot_l = link_sums(x, m, pairs, i, lane, tot_l, sum8_buf);
  return tot_l;
}

// TS: precision in which this level keeps sigma.  kDemand: commodities of unequal demand.
template <typename TS, bool kDemand>
__device__ __forceinline__ void
bwd_rows(const int32_t* __restrict__ out_ptr, const int32_t* __restrict__ out_col, const GroupView& gv,
         int level, int g, int u0, double* __restrict__ sum8_buf, const TileShare& ts, const NodeIdx& me,
         const LinkRange& lr) {
  double* const stage_buf = sum8_buf + kSum8Doubles;  // kStageDoubles doubles
  const int lane = lane_id();
  const NodeIdx* __restrict__ cur = gv.idxb + ((size_t)g * gv.Lcap + level) * gv.Npad;
  const NodeIdx* __restrict__ next = cur + gv.Npad;
  const TS* __restrict__ dat = sigma_rows<TS>(gv, g);
  double* __restrict__ cf = gv.coef + (size_t)g * gv.Npad * 64;
  double* __restrict__ pt = gv.part + (size_t)g * gv.Epad;
  const double* __restrict__ dem = kDemand ? demand_rows(gv, g) : nullptr;
  double wd = 0.0;  // this lane's source: demands met
  const uint64_t nodes_active = __ballot(me.mask != 0);
  if (nodes_active == 0) return;
  int q, q_next, q_nn;
  Tile tile = tile_request_idx(next, tile_request_col(out_col, lr, ts.first, 0, lane, q));
  q_next = -1;
  int nb_next = ts.first + ts.step < 8 ? tile_request_col(out_col, lr, ts.first + ts.step, 0, lane, q_next) : -1;
#pragma unroll 1
  for (int c = ts.first; c < 8; c += ts.step) {
    const Tile tile_next = tile_request_idx(next, c + ts.step < 8 ? nb_next : -1);
    nb_next = -1;
    q_nn = -1;
    if (c + 2 * ts.step < 8) nb_next = tile_request_col(out_col, lr, c + 2 * ts.step, 0, lane, q_nn);
    if (((nodes_active >> (8 * c)) & 0xffull) != 0) {
      double xa[8], xb[8];
      uint64_t ma[8], mb[8];
      double tot_l = 0.0;  // lane 8i+j: load of out-link j of node i
      // The coef rows of the tile's nodes are adjacent in memory: all but the very longest spans are put
      // together in LDS and stored as whole lines (store_staged), the others entry by entry.
      const TileSpan span = tile_span(me, nodes_active, c);
      double* __restrict__ stage = span.end - span.of0 <= (uint32_t)kStageDoubles ? stage_buf : nullptr;
      TS sa = own_sigma(dat, me, 8 * c), sb;
      double da = own_demand<kDemand>(dem, gv.dem_ld, u0, me, 8 * c, lane), db;
      int pa = gather8(cf, tile, 0, readlane64(me.mask, 8 * c), xa, ma), pb;
#pragma unroll 1
      for (int i = 0; i < 8; i += 2) {  // two nodes per round, the next one's rows always in flight
        sb = own_sigma(dat, me, 8 * c + i + 1);
        db = own_demand<kDemand>(dem, gv.dem_ld, u0, me, 8 * c + i + 1, lane);
        pb = gather8(cf, tile, i + 1, readlane64(me.mask, 8 * c + i + 1), xb, mb);
        tot_l = bwd_finish(cf, me, 8 * c + i, i, sa, da, xa, ma, pa, false, lane, tot_l, sum8_buf, stage, span.of0);
        if (kDemand && lane_in(readlane64(me.mask, 8 * c + i))) wd += da;
        if (i + 2 < 8) {
          sa = own_sigma(dat, me, 8 * c + i + 2);
          da = own_demand<kDemand>(dem, gv.dem_ld, u0, me, 8 * c + i + 2, lane);
          pa = gather8(cf, tile, i + 2, readlane64(me.mask, 8 * c + i + 2), xa, ma);
        }
        tot_l = bwd_finish(cf, me, 8 * c + i + 1, i + 1, sb, db, xb, mb, pb, false, lane, tot_l, sum8_buf, stage, span.of0);
        if (kDemand && lane_in(readlane64(me.mask, 8 * c + i + 1))) wd += db;
      }
      const uint64_t mu_lane = shfl64(me.mask, 8 * c + (lane >> 3));
      if (q >= 0 && (tile.mask & mu_lane) != 0) unsafeAtomicAdd(&pt[q], tot_l);
      // nodes with more than eight out-links: add the rest to the stored coef
      const int p0 = __shfl(lr.p0, 8 * c + (lane >> 3), kWave), p1 = __shfl(lr.p1, 8 * c + (lane >> 3), kWave);
      for (int base = 8; __ballot(p0 + base < p1) != 0; base += 8) {
        int qe;
        const Tile extra = tile_request_idx(next, tile_request_col(out_col, lr, c, base, lane, qe));
        tot_l = 0.0;
#pragma unroll 1
        for (int i = 0; i < 8; ++i) {
          pa = gather8(cf, extra, i, readlane64(me.mask, 8 * c + i), xa, ma);
          if (pa == 0) continue;
          sa = own_sigma(dat, me, 8 * c + i);
          tot_l = bwd_finish(cf, me, 8 * c + i, i, sa, 1.0, xa, ma, pa, true, lane, tot_l, sum8_buf, stage, span.of0);
        }
        if (qe >= 0 && (extra.mask & mu_lane) != 0) unsafeAtomicAdd(&pt[qe], tot_l);
      }
      if (stage != nullptr) {
        __builtin_amdgcn_wave_barrier();
        store_staged(cf, stage, span, lane);
        __builtin_amdgcn_wave_barrier();
      }
    }
    tile = tile_next;
    q = q_next;
    q_next = q_nn;
  }
  if (kDemand) add_weighted_dist(gv, g, u0, level, wd);
}

// --- levels with few sources per node: one lane per (node, link) ---------------------------
//
// With a handful of sources per node, a lane per source leaves most of the wave idle and still
// pays the per-link instruction cost.  These kernels keep the index tile's layout for the
// arithmetic as well: lane 8i+j owns link j of node i and walks the node's sources in ascending
// order, the eight lanes of a node in step.  Per source the lane reads its link's entry (if the
// link carries that source), the eight lanes add up in a fixed order, and lane j = 0 writes the
// node's entry; the node's own row is compact, so its k-th source is simply entry k of the row.
// The entries of the next source are requested before the current ones are used.

__device__ __forceinline__ uint32_t below(uint64_t mask, int s) {
  return (uint32_t)__popcll(mask & ((1ull << s) - 1ull));
}

// Value of lane kSrc of this lane's group of eight lanes.
template <int kSrc>
__device__ __forceinline__ double bcast8(double x) {
  union {
    double d;
    int i[2];
  } a, b;
  a.d = x;  // ds_swizzle, bit mode: lane = (lane & 0x18) | kSrc within each half of the wave
  b.i[0] = __builtin_amdgcn_ds_swizzle(a.i[0], 0x18 | (kSrc << 5));
  b.i[1] = __builtin_amdgcn_ds_swizzle(a.i[1], 0x18 | (kSrc << 5));
  return b.d;
}

// The next (up to) eight sources of `rest`, lowest first: x[k] = the entry of the k-th of them in
// the link's row (mk, ofk), 0 if the link does not carry it or there is no k-th source.  All
// requests are issued before any value is used.
// mine: the source that this lane's place among its eight lanes stands for (-1: none left).
template <typename T>
__device__ __forceinline__ void few_fetch8(const T* __restrict__ rows, uint64_t mk, uint32_t ofk, uint64_t& rest,
                                           T (&x)[8], int place, int& mine) {
  mine = -1;
#pragma unroll
  for (int k = 0; k < 8; ++k) {
    x[k] = (T)0;
    if (rest != 0) {
      const int s = __builtin_ctzll(rest);
      rest &= rest - 1;
      if (k == place) mine = s;
      if ((mk >> s) & 1ull) x[k] = entry(rows, ofk + below(mk, s));
    }
  }
}

// sigma of the node's sources from one tile of in-links (mu, ofu: the node's own mask and row).
// Lane j of the node ends up with the sum for the node's j-th source and writes that entry.
template <typename TIn, typename TOut>
__device__ __forceinline__ bool few_fwd(const TIn* __restrict__ rows, TOut* __restrict__ out, double* __restrict__ cf,
                                        const Tile& tl, uint64_t mu, uint32_t ofu, bool add, int lane) {
  uint64_t rest = mu;
  uint32_t e = ofu + (uint32_t)(lane & 7);
  int left = __popcll(mu) - (lane & 7);  // > 0: this lane owns a source of the current eight
  bool big = false;
  while (__ballot(rest != 0) != 0) {
    TIn xr[8];
    int mine;
    few_fetch8(rows, tl.mask, tl.off, rest, xr, lane & 7, mine);
    TOut x[8];  // a level kept in single precision is summed in it: whole numbers below 2^24, exact
#pragma unroll
    for (int k = 0; k < 8; ++k) x[k] = (TOut)hold(xr[k]);
    TOut a = group_sum8(x, lane);
    if (left > 0 && !(add && a == (TOut)0)) {
      if (add) a += entry(out, e);
      entry(out, e) = a;
      if (cf != nullptr) entry(cf, e) = recip((double)a);
      if constexpr (sizeof(TOut) == 8) big |= a >= kTwo53;
    }
    e += 8;
    left -= 8;
  }
  return big;
}

// coef of the node's sources and this lane's link load from one tile of out-links.
// dem_row (nullptr: all demands 1): the demands of this lane's node; wd collects the ones met.
template <typename TS>
__device__ __forceinline__ double few_bwd(const TS* __restrict__ dat, double* __restrict__ cf, const Tile& tl,
                                          uint64_t mu, uint32_t ofu, bool add, int lane,
                                          const double* __restrict__ dem_row, double& wd) {
  uint64_t rest = mu;
  uint32_t e = ofu + (uint32_t)(lane & 7);
  int left = __popcll(mu) - (lane & 7);
  double acc = 0.0;
  while (__ballot(rest != 0) != 0) {
    double x[8];
    int mine;
    few_fetch8(cf, tl.mask, tl.off, rest, x, lane & 7, mine);
    TS sg_own = (TS)1;  // lane j: sigma of the node's j-th source of these eight
    double dm = 1.0;
    if (left > 0) {
      sg_own = entry(dat, e);
      if (dem_row != nullptr && !add) dm = dem_row[mine];
    }
    const double sg = (double)hold(sg_own);
    acc = __builtin_fma(bcast8<0>(sg), x[0], acc);
    acc = __builtin_fma(bcast8<1>(sg), x[1], acc);
    acc = __builtin_fma(bcast8<2>(sg), x[2], acc);
    acc = __builtin_fma(bcast8<3>(sg), x[3], acc);
    acc = __builtin_fma(bcast8<4>(sg), x[4], acc);
    acc = __builtin_fma(bcast8<5>(sg), x[5], acc);
    acc = __builtin_fma(bcast8<6>(sg), x[6], acc);
    acc = __builtin_fma(bcast8<7>(sg), x[7], acc);
    double a = group_sum8(x, lane);
    if (left > 0 && !(add && a == 0.0)) {
      a += add ? entry(cf, e) : dm * recip(sg);
      entry(cf, e) = a;
    }
    if (dem_row != nullptr && !add && left > 0) wd += dm;
    e += 8;
    left -= 8;
  }
  return acc;
}

// --- the same levels with a lane per (node, source) ---------------------------------------
//
// Second lane layout for the same tile: lane 8i+k owns the k-th source of node i (eight sources
// per round) and walks the node's links, all lanes on link j at the same time.  The lanes of a
// node then read the same row, so their requests share its memory lines, and the sum over the
// links is lane-local; only the link loads need one exchange per tile.  Costs the same
// whether the node has one source or eight, so it pays from a few sources per node upwards.

template <int kSrc>
__device__ __forceinline__ uint32_t bcast8(uint32_t x) {
  return (uint32_t)__builtin_amdgcn_ds_swizzle((int)x, 0x18 | (kSrc << 5));
}
template <int kSrc>
__device__ __forceinline__ uint64_t bcast8(uint64_t x) {
  return ((uint64_t)bcast8<kSrc>((uint32_t)(x >> 32)) << 32) | bcast8<kSrc>((uint32_t)x);
}

// Removes the next (up to) eight sources from `rest`; returns the k-th of them, -1 if none.
__device__ __forceinline__ int slot_take8(uint64_t& rest, int k) {
  int mine = -1;
#pragma unroll
  for (int t = 0; t < 8; ++t) {
    if (rest != 0) {
      const int s = __builtin_ctzll(rest);
      rest &= rest - 1;
      if (t == k) mine = s;
    }
  }
  return mine;
}

// x[j] = entry of source s in the row of link j of this lane's node (0 if not carried).
template <int kJ, typename T>
__device__ __forceinline__ T slot_fetch(const T* __restrict__ rows, const Tile& tl, int s) {
  const uint64_t mk = bcast8<kJ>(tl.mask);
  const uint32_t ofk = bcast8<kJ>(tl.off);
  T x = (T)0;
  if (s >= 0 && ((mk >> s) & 1ull)) x = entry(rows, ofk + below(mk, s));
  return x;
}
template <typename T>
__device__ __forceinline__ void slot_fetch8(const T* __restrict__ rows, const Tile& tl, int s, T (&x)[8]) {
  x[0] = slot_fetch<0>(rows, tl, s);
  x[1] = slot_fetch<1>(rows, tl, s);
  x[2] = slot_fetch<2>(rows, tl, s);
  x[3] = slot_fetch<3>(rows, tl, s);
  x[4] = slot_fetch<4>(rows, tl, s);
  x[5] = slot_fetch<5>(rows, tl, s);
  x[6] = slot_fetch<6>(rows, tl, s);
  x[7] = slot_fetch<7>(rows, tl, s);
}

template <typename TIn, typename TOut>
__device__ __forceinline__ bool slot_fwd(const TIn* __restrict__ rows, TOut* __restrict__ out, double* __restrict__ cf,
                                         const Tile& tl, uint64_t mu, uint32_t ofu, bool add, int lane) {
  uint64_t rest = mu;
  uint32_t e = ofu + (uint32_t)(lane & 7);
  bool big = false;
  while (__ballot(rest != 0) != 0) {
    const int s = slot_take8(rest, lane & 7);
    TIn x[8];
    slot_fetch8(rows, tl, s, x);
    TOut a = (TOut)0;
#pragma unroll
    for (int j = 0; j < 8; ++j) a += (TOut)hold(x[j]);
    if (s >= 0 && !(add && a == (TOut)0)) {
      if (add) a += entry(out, e);
      entry(out, e) = a;
      if (cf != nullptr) entry(cf, e) = recip((double)a);
      if constexpr (sizeof(TOut) == 8) big |= a >= kTwo53;
    }
    e += 8;
  }
  return big;
}

// Returns, in lane 8i+j, the load of link j of node i from this tile.
template <typename TS>
__device__ __forceinline__ double slot_bwd(const TS* __restrict__ dat, double* __restrict__ cf, const Tile& tl,
                                           uint64_t mu, uint32_t ofu, bool add, int lane,
                                           const double* __restrict__ dem_row, double& wd) {
  uint64_t rest = mu;
  uint32_t e = ofu + (uint32_t)(lane & 7);
  double p[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) p[j] = 0.0;
  while (__ballot(rest != 0) != 0) {
    const int s = slot_take8(rest, lane & 7);
    double x[8];
    slot_fetch8(cf, tl, s, x);
    TS sg_own = (TS)1;
    double dm = 1.0;
    if (s >= 0) {
      sg_own = entry(dat, e);
      if (dem_row != nullptr && !add) dm = dem_row[s];
    }
    const double sg = (double)hold(sg_own);
    double a = 0.0;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      a += x[j];
      p[j] = __builtin_fma(sg, x[j], p[j]);
    }
    if (s >= 0 && !(add && a == 0.0)) {
      a += add ? entry(cf, e) : dm * recip(sg);
      entry(cf, e) = a;
    }
    if (dem_row != nullptr && !add && s >= 0) wd += dm;
    e += 8;
  }
  return group_sum8(p, lane);
}

template <bool kCountDag, bool kSlots, typename TIn, typename TOut>
__device__ __forceinline__ void
fwd_few(const int32_t* __restrict__ in_ptr, const int32_t* __restrict__ in_col, const GroupView& gv, int level,
        bool init_coef, long long* __restrict__ misc, int g, int v0, const TileShare& ts, NodeIdx me, LinkRange lr) {
  const int lane = lane_id();
  const NodeIdx* __restrict__ cur = gv.idxb + ((size_t)g * gv.Lcap + level) * gv.Npad;
  const NodeIdx* __restrict__ prev = cur - gv.Npad;
  const TIn* __restrict__ rows = sigma_rows<TIn>(gv, g);
  TOut* __restrict__ out = sigma_rows<TOut>(gv, g);
  double* __restrict__ cf = init_coef ? gv.coef + (size_t)g * gv.Npad * 64 : nullptr;
  const uint64_t nodes_active = __ballot(me.mask != 0);
  if (nodes_active == 0) return;
  int nid = v0 + lane;
  const int tiles = (compact_nodes(nodes_active, lane, me, lr, nid) + 7) >> 3;
  bool inexact = false;
  int dag = 0;
  int q;
  Tile tile = tile_request_idx(prev, tile_request_col(in_col, lr, ts.first, 0, lane, q));
  int nb_next = ts.first + ts.step < tiles ? tile_request_col(in_col, lr, ts.first + ts.step, 0, lane, q) : -1;
#pragma unroll 1
  for (int c = ts.first; c < tiles; c += ts.step) {
    const Tile tile_next = tile_request_idx(prev, c + ts.step < tiles ? nb_next : -1);
    nb_next = c + 2 * ts.step < tiles ? tile_request_col(in_col, lr, c + 2 * ts.step, 0, lane, q) : -1;
    {
      const int node = 8 * c + (lane >> 3);
      const uint64_t mu = shfl64(me.mask, node);
      const uint32_t ofu = (uint32_t)__shfl((int)me.off, node, kWave);
      inexact |= kSlots ? slot_fwd(rows, out, cf, tile, mu, ofu, false, lane) : few_fwd(rows, out, cf, tile, mu, ofu, false, lane);
      if (kCountDag) dag += __popcll(tile.mask & mu);
      // nodes with more than eight in-links: add the rest to the staged entries
      const int p0 = __shfl(lr.p0, node, kWave), p1 = __shfl(lr.p1, node, kWave);
      for (int base = 8; __ballot(p0 + base < p1) != 0; base += 8) {
        const Tile extra = tile_request_idx(prev, tile_request_col(in_col, lr, c, base, lane, q));
        inexact |= kSlots ? slot_fwd(rows, out, cf, extra, mu, ofu, true, lane) : few_fwd(rows, out, cf, extra, mu, ofu, true, lane);
        if (kCountDag) dag += __popcll(extra.mask & mu);
      }
    }
    tile = tile_next;
  }
  if (inexact) misc[0] = 1;
  if (kCountDag) {
    dag = wave_sum_int(dag);
    if (dag != 0 && lane == 0)
      atomicAdd((unsigned long long*)&gv.dag[(size_t)g * gv.Lcap + level], (unsigned long long)dag);
  }
}

// --- forward level whose in-neighbours' rows are short: lane = (node, link), whole rows --------
//
// Third use of the tile layout, for a level with many sources per node whose in-neighbours have
// few: lane 8i+j reads the row of link j of node i from end to end (its entries are adjacent in
// memory: one or two lines per link, one request per entry and 64 links at a time instead of one
// request per link and node) and adds every entry whose source the node has on this level to the
// node's accumulator for that source in LDS (atomic adds: path counts are whole numbers below
// 2^53, so the order does not matter; beyond, the result is flagged as inexact anyway).  Then the
// node's sources collect their sums, a lane per source, and write the node's row.

// Adds the entries of this lane's link to acc[source] (the accumulators of this lane's node).
// The row is read in aligned 16-byte pieces (two or four entries per request: the requests, one
// per lane and instruction, are what bounds this kernel); a piece at either end of the row may
// hold a neighbouring row's entries, which are skipped (the arrays have room for the last piece).
template <typename T>
__device__ __forceinline__ void spread_link(const T* __restrict__ rows, const Tile& tl, uint64_t mu,
                                            double* __restrict__ acc) {
  constexpr int kPer = 16 / (int)sizeof(T);
  uint64_t rest = tl.mask;  // sources of the link's row, ascending = its entries in order
  int skip = (int)(tl.off & (uint32_t)(kPer - 1));  // entries of the first piece that come before the row
  uint32_t q = tl.off / (uint32_t)kPer;
  while (__ballot(rest != 0) != 0) {  // four pieces per round, all requested first
    const int n = __popcll(rest) + skip;
    uint4 y[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      y[k] = make_uint4(0u, 0u, 0u, 0u);
      if (kPer * k < n) y[k] = piece(rows, q + (uint32_t)k);
    }
#pragma unroll
    for (int k = 0; k < 4 * kPer; ++k) {
      if (k < kPer - 1 && k < skip) continue;
      if (rest != 0) {
        const int s = __builtin_ctzll(rest);
        rest &= rest - 1;
        if ((mu >> s) & 1ull) unsafeAtomicAdd(&acc[s], piece_get<T>(y[k / kPer], k % kPer));
      }
    }
    skip = 0;
    q += 4;
  }
}

template <bool kCountDag, typename TIn, typename TOut>
__device__ __forceinline__ void
fwd_spread(const int32_t* __restrict__ in_ptr, const int32_t* __restrict__ in_col, const GroupView& gv, int level,
           bool init_coef, long long* __restrict__ misc, int g, int v0, double (*__restrict__ acc)[kWave],
           const TileShare& ts, const NodeIdx& me, const LinkRange& lr) {
  const int lane = lane_id();
  const NodeIdx* __restrict__ cur = gv.idxb + ((size_t)g * gv.Lcap + level) * gv.Npad;
  const NodeIdx* __restrict__ prev = cur - gv.Npad;
  const TIn* __restrict__ rows = sigma_rows<TIn>(gv, g);
  TOut* __restrict__ out = sigma_rows<TOut>(gv, g);
  double* __restrict__ cf = init_coef ? gv.coef + (size_t)g * gv.Npad * 64 : nullptr;
  const uint64_t nodes_active = __ballot(me.mask != 0);
  if (nodes_active == 0) return;
  bool inexact = false;
  int dag = 0;
  int q;
  Tile tile = tile_request_idx(prev, tile_request_col(in_col, lr, ts.first, 0, lane, q));
  int nb_next = ts.first + ts.step < 8 ? tile_request_col(in_col, lr, ts.first + ts.step, 0, lane, q) : -1;
#pragma unroll 1
  for (int c = ts.first; c < 8; c += ts.step) {
    const Tile tile_next = tile_request_idx(prev, c + ts.step < 8 ? nb_next : -1);
    nb_next = c + 2 * ts.step < 8 ? tile_request_col(in_col, lr, c + 2 * ts.step, 0, lane, q) : -1;
    if (((nodes_active >> (8 * c)) & 0xffull) != 0) {
#pragma unroll
      for (int i = 0; i < 8; ++i) acc[i][lane] = 0.0;
      __builtin_amdgcn_wave_barrier();
      const int node = 8 * c + (lane >> 3);
      const uint64_t mu = shfl64(me.mask, node);
      spread_link(rows, tile, mu, acc[lane >> 3]);
      if (kCountDag) dag += __popcll(tile.mask & mu);
      // nodes with more than eight in-links: further tiles into the same accumulators
      const int p0 = __shfl(lr.p0, node, kWave), p1 = __shfl(lr.p1, node, kWave);
      for (int base = 8; __ballot(p0 + base < p1) != 0; base += 8) {
        const Tile extra = tile_request_idx(prev, tile_request_col(in_col, lr, c, base, lane, q));
        spread_link(rows, extra, mu, acc[lane >> 3]);
        if (kCountDag) dag += __popcll(extra.mask & mu);
      }
      __builtin_amdgcn_wave_barrier();
      // lane = source: the nodes' sums are put together in LDS, in place of the accumulators (once every
      // lane holds its values), as the tile's piece of the sigma array, and stored as whole lines
      double val[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) val[i] = acc[i][lane];
      __builtin_amdgcn_wave_barrier();
      const TileSpan span = tile_span(me, nodes_active, c);
      TOut* __restrict__ flat = reinterpret_cast<TOut*>(&acc[0][0]);
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const uint64_t newv = readlane64(me.mask, 8 * c + i);
        const uint32_t of = (uint32_t)__builtin_amdgcn_readlane((int)me.off, 8 * c + i);
        if (lane_in(newv)) {
          const uint32_t e = of + rank_in(newv);
          flat[e - span.of0] = (TOut)val[i];
          if (cf != nullptr) entry(cf, e) = recip(val[i]);
          inexact |= val[i] >= kTwo53;
        }
      }
      __builtin_amdgcn_wave_barrier();
      store_staged(out, flat, span, lane);
      __builtin_amdgcn_wave_barrier();
    }
    tile = tile_next;
  }
  if (inexact) misc[0] = 1;
  if (kCountDag) {
    dag = wave_sum_int(dag);
    if (dag != 0 && lane == 0)
      atomicAdd((unsigned long long*)&gv.dag[(size_t)g * gv.Lcap + level], (unsigned long long)dag);
  }
}

// --- backward level whose successors' rows are short: the mirror image ----------------------
//
// A level with many sources per node whose successors have few: the node's sigma goes to LDS (a
// lane per source), then lane 8i+j reads the coef row of link j of node i from end to end, adds
// every entry whose source the node has on this level to the node's accumulator for that source
// and, times the node's sigma, to the link's load (lane-local, in row order); then the
// accumulators go to the node's coef row, a lane per source.  The order of every sum is fixed.
// The accumulators are private to the wave and start at zero, so a source that at most two of the
// node's eight links carry gets the same bits whichever of the two lanes is served first (the
// common case: atomic adds, all links at once).  Sources carried by three or more links of the
// tile, and everything in the further tiles of a node with more than eight links, take the ordered
// path instead: source by source, the eight lanes' values added in a fixed tree, one lane adding
// the result to the accumulator.

template <int kMask>
__device__ __forceinline__ uint64_t xor_lanes_u64(uint64_t x) {
  return (uint64_t)__double_as_longlong(xor_lanes<kMask>(__longlong_as_double((long long)x)));
}

// Bits set in at least three of the eight masks held by the lanes 8i .. 8i+7 (the same result in
// all eight): a carry-save count over the three exchange steps.
__device__ __forceinline__ uint64_t three_or_more8(uint64_t m) {
  const uint64_t b = xor_lanes_u64<1>(m);
  uint64_t ones = m ^ b, twos = m & b;  // pair: count = ones + 2 twos
  const uint64_t o2 = xor_lanes_u64<2>(ones), t2 = xor_lanes_u64<2>(twos);
  const uint64_t c1 = ones & o2;
  ones ^= o2;
  const uint64_t fours = (twos & t2) | (twos & c1) | (t2 & c1);
  twos = twos ^ t2 ^ c1;  // four lanes: count = ones + 2 twos + 4 fours
  const uint64_t o3 = xor_lanes_u64<4>(ones), t3 = xor_lanes_u64<4>(twos), f3 = xor_lanes_u64<4>(fours);
  const uint64_t c2 = ones & o3;
  ones ^= o3;
  const uint64_t c4 = (twos & t3) | (twos & c2) | (t3 & c2);
  twos = twos ^ t3 ^ c2;
  return fours | f3 | c4 | (twos & ones);
}

__device__ __forceinline__ uint64_t or8(uint64_t m) {
  m |= xor_lanes_u64<1>(m);
  m |= xor_lanes_u64<2>(m);
  m |= xor_lanes_u64<4>(m);
  return m;
}

// Fast path: the entries of this lane's link whose source is in `take` (sources of the node that at
// most two links of the tile carry).  Returns tot + this lane's share of the link load.
template <typename TS>
__device__ __forceinline__ double spread_link_bwd(const double* __restrict__ rows, const Tile& tl, uint64_t take,
                                                  double* __restrict__ acc, const TS* __restrict__ sig) {
  // entry by entry: with one or two entries per row, pairs (as in spread_link) only fetch more
  uint64_t rest = tl.mask;
  uint32_t e = tl.off;
  double tot = 0.0;
  while (__ballot(rest != 0) != 0) {  // eight entries per round, all requested first
    const int c = __popcll(rest);
    double x[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) {
      x[k] = 0.0;
      if (k < c) x[k] = entry(rows, e + (uint32_t)k);
    }
#pragma unroll
    for (int k = 0; k < 8; ++k) {
      if (rest != 0) {
        const int s = __builtin_ctzll(rest);
        rest &= rest - 1;
        if ((take >> s) & 1ull) {
          unsafeAtomicAdd(&acc[s], x[k]);
          tot = __builtin_fma((double)sig[s], x[k], tot);
        }
      }
    }
    e += 8;
  }
  return tot;
}

// Ordered path: the sources in `set` (the same in the eight lanes of a node), lowest first.  Each
// lane fetches its link's entry for the source (0 if the link does not carry it), the eight
// values are added in a fixed tree, and the node's first lane adds the sum to the accumulator.
template <typename TS>
__device__ __forceinline__ double spread_ordered_bwd(const double* __restrict__ rows, const Tile& tl, uint64_t set,
                                                     double* __restrict__ acc, const TS* __restrict__ sig,
                                                     double tot, int lane) {
  uint64_t todo = or8(tl.mask & set);
  while (__ballot(todo != 0) != 0) {
    const bool live = todo != 0;
    const int s = live ? __builtin_ctzll(todo) : 0;
    todo &= todo - 1;
    double x = 0.0;
    if (live && ((tl.mask >> s) & 1ull)) x = entry(rows, tl.off + below(tl.mask, s));
    tot = __builtin_fma((double)sig[s], x, tot);
    double y = x + xor_lanes<1>(x);
    y += xor_lanes<2>(y);
    y += xor_lanes<4>(y);
    if (live && (lane & 7) == 0) acc[s] += y;
  }
  return tot;
}

template <typename TS, bool kDemand>
__device__ __forceinline__ void
bwd_spread(const int32_t* __restrict__ out_ptr, const int32_t* __restrict__ out_col, const GroupView& gv, int level,
           int g, int u0, double (*__restrict__ acc)[kWave], TS (*__restrict__ sig)[kWave], const TileShare& ts,
           const NodeIdx& me, const LinkRange& lr) {
  const int lane = lane_id();
  const NodeIdx* __restrict__ cur = gv.idxb + ((size_t)g * gv.Lcap + level) * gv.Npad;
  const NodeIdx* __restrict__ next = cur + gv.Npad;
  const TS* __restrict__ dat = sigma_rows<TS>(gv, g);
  double* __restrict__ cf = gv.coef + (size_t)g * gv.Npad * 64;
  double* __restrict__ pt = gv.part + (size_t)g * gv.Epad;
  const double* __restrict__ dem = kDemand ? demand_rows(gv, g) : nullptr;
  double wd = 0.0;
  const uint64_t nodes_active = __ballot(me.mask != 0);
  if (nodes_active == 0) return;
  int q, q_next, q_nn;
  Tile tile = tile_request_idx(next, tile_request_col(out_col, lr, ts.first, 0, lane, q));
  q_next = -1;
  int nb_next = ts.first + ts.step < 8 ? tile_request_col(out_col, lr, ts.first + ts.step, 0, lane, q_next) : -1;
#pragma unroll 1
  for (int c = ts.first; c < 8; c += ts.step) {
    const Tile tile_next = tile_request_idx(next, c + ts.step < 8 ? nb_next : -1);
    nb_next = -1;
    q_nn = -1;
    if (c + 2 * ts.step < 8) nb_next = tile_request_col(out_col, lr, c + 2 * ts.step, 0, lane, q_nn);
    if (((nodes_active >> (8 * c)) & 0xffull) != 0) {
      TS sg_own[8];  // lane = source: sigma of the nodes' sources, all rows requested first
      double dm[8];  // and their demands
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const uint64_t mu_i = readlane64(me.mask, 8 * c + i);
        const uint32_t of = (uint32_t)__builtin_amdgcn_readlane((int)me.off, 8 * c + i);
        sg_own[i] = (TS)1;
        if (lane_in(mu_i)) sg_own[i] = entry(dat, of + rank_in(mu_i));
        dm[i] = own_demand<kDemand>(dem, gv.dem_ld, u0, me, 8 * c + i, lane);
      }
      double sg[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        sg[i] = (double)hold(sg_own[i]);
        sig[i][lane] = (TS)sg[i];  // exact: it came from a TS
        acc[i][lane] = 0.0;
      }
      __builtin_amdgcn_wave_barrier();
      const int node = 8 * c + (lane >> 3);
      const uint64_t mu = shfl64(me.mask, node);
      const uint64_t many = three_or_more8(tile.mask & mu);
      double tot = spread_link_bwd(cf, tile, mu & ~many, acc[lane >> 3], sig[lane >> 3]);
      __builtin_amdgcn_wave_barrier();
      tot = spread_ordered_bwd(cf, tile, many, acc[lane >> 3], sig[lane >> 3], tot, lane);
      if (q >= 0 && (tile.mask & mu) != 0) unsafeAtomicAdd(&pt[q], tot);
      // nodes with more than eight out-links: further tiles into the same accumulators
      const int p0 = __shfl(lr.p0, node, kWave), p1 = __shfl(lr.p1, node, kWave);
      for (int base = 8; __ballot(p0 + base < p1) != 0; base += 8) {
        int qe;
        const Tile extra = tile_request_idx(next, tile_request_col(out_col, lr, c, base, lane, qe));
        const double te = spread_ordered_bwd(cf, extra, mu, acc[lane >> 3], sig[lane >> 3], 0.0, lane);
        if (qe >= 0 && (extra.mask & mu) != 0) unsafeAtomicAdd(&pt[qe], te);
      }
      __builtin_amdgcn_wave_barrier();
      // The coef rows of the tile's nodes are adjacent in memory: they are put together in LDS (in
      // place of the accumulators, once every lane holds its values) and stored as whole lines.
      double val[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) {  // lane = source
        val[i] = dm[i] * recip(sg[i]) + acc[i][lane];
        if (kDemand && lane_in(readlane64(me.mask, 8 * c + i))) wd += dm[i];
      }
      __builtin_amdgcn_wave_barrier();
      const TileSpan span = tile_span(me, nodes_active, c);
      double* __restrict__ flat = &acc[0][0];
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const uint64_t mu_i = readlane64(me.mask, 8 * c + i);
        const uint32_t of = (uint32_t)__builtin_amdgcn_readlane((int)me.off, 8 * c + i);
        if (lane_in(mu_i)) flat[of - span.of0 + rank_in(mu_i)] = val[i];
      }
      __builtin_amdgcn_wave_barrier();
      store_staged(cf, flat, span, lane);
      __builtin_amdgcn_wave_barrier();
    }
    tile = tile_next;
    q = q_next;
    q_next = q_nn;
  }
  if (kDemand) add_weighted_dist(gv, g, u0, level, wd);
}

template <bool kSlots, typename TS, bool kDemand>
__device__ __forceinline__ void
bwd_few(const int32_t* __restrict__ out_ptr, const int32_t* __restrict__ out_col, const GroupView& gv, int level,
        int g, int u0, const TileShare& ts, NodeIdx me, LinkRange lr) {
  const int lane = lane_id();
  const NodeIdx* __restrict__ cur = gv.idxb + ((size_t)g * gv.Lcap + level) * gv.Npad;
  const NodeIdx* __restrict__ next = cur + gv.Npad;
  const TS* __restrict__ dat = sigma_rows<TS>(gv, g);
  double* __restrict__ cf = gv.coef + (size_t)g * gv.Npad * 64;
  double* __restrict__ pt = gv.part + (size_t)g * gv.Epad;
  const double* __restrict__ dem = kDemand ? demand_rows(gv, g) : nullptr;
  double wd = 0.0;
  const uint64_t nodes_active = __ballot(me.mask != 0);
  if (nodes_active == 0) return;
  int nid = u0 + lane;
  const int tiles = (compact_nodes(nodes_active, lane, me, lr, nid) + 7) >> 3;
  int q, q_next = -1, q_nn;
  Tile tile = tile_request_idx(next, tile_request_col(out_col, lr, ts.first, 0, lane, q));
  int nb_next = ts.first + ts.step < tiles ? tile_request_col(out_col, lr, ts.first + ts.step, 0, lane, q_next) : -1;
#pragma unroll 1
  for (int c = ts.first; c < tiles; c += ts.step) {
    const Tile tile_next = tile_request_idx(next, c + ts.step < tiles ? nb_next : -1);
    nb_next = -1;
    q_nn = -1;
    if (c + 2 * ts.step < tiles) nb_next = tile_request_col(out_col, lr, c + 2 * ts.step, 0, lane, q_nn);
    {
      const int node = 8 * c + (lane >> 3);
      const uint64_t mu = shfl64(me.mask, node);
      const uint32_t ofu = (uint32_t)__shfl((int)me.off, node, kWave);
      const double* __restrict__ dem_row =
          kDemand ? dem + (size_t)__shfl(nid, node, kWave) * (size_t)gv.dem_ld : nullptr;
      const double tot = kSlots ? slot_bwd(dat, cf, tile, mu, ofu, false, lane, dem_row, wd)
                                : few_bwd(dat, cf, tile, mu, ofu, false, lane, dem_row, wd);
      if (q >= 0 && (tile.mask & mu) != 0) unsafeAtomicAdd(&pt[q], tot);
      // nodes with more than eight out-links: add the rest to the stored coef
      const int p0 = __shfl(lr.p0, node, kWave), p1 = __shfl(lr.p1, node, kWave);
      for (int base = 8; __ballot(p0 + base < p1) != 0; base += 8) {
        int qe;
        const Tile extra = tile_request_idx(next, tile_request_col(out_col, lr, c, base, lane, qe));
        const double te = kSlots ? slot_bwd(dat, cf, extra, mu, ofu, true, lane, dem_row, wd)
                                 : few_bwd(dat, cf, extra, mu, ofu, true, lane, dem_row, wd);
        if (qe >= 0 && (extra.mask & mu) != 0) unsafeAtomicAdd(&pt[qe], te);
      }
    }
    tile = tile_next;
    q = q_next;
    q_next = q_nn;
  }
  if (kDemand) add_weighted_dist(gv, g, u0, level, wd);
}

// --- one launch per level and pass; every batch picks its own lane layout --------------------
//
// How full a level is differs from batch to batch (and from topology to topology), and it decides
// which of the lane layouts above is the cheap one.  The choice is made here, per batch, from the
// batch's own pair counts (ltot, complete after the BFS): it does not depend on which batches
// happen to advance together, so neither do the sums' orders nor the results' bits, and the host
// needs no read-back to pick a kernel.  sources per node = pairs / N:
//   >= kRowsLanes                       lane = source, one wave per node          (rows)
//   ... and the level the pass reads from (the one before, forward; the one after, backward)
//       below kRowsLanes                lane = (node, link), whole rows           (spread)
//   kSlotLanes .. kRowsLanes            lane = (node, source)                     (few, slots)
//   below kSlotLanes                    lane = (node, link), source by source     (few)
constexpr long long kRowsLanes = 8;
constexpr long long kSlotLanes = 2;

enum Flavour { kFlavRows = 0, kFlavSpread = 1, kFlavSlots = 2, kFlavFew = 3 };

// Pairs on the level, on the one before and on the one after, for batch g.
struct LevelFill {
  long long before, here, after;
};
__device__ __forceinline__ LevelFill level_fill(const GroupView& gv, int g, int level) {
  const long long* __restrict__ lt = gv.ltot + (size_t)g * gv.Lcap;
  LevelFill f;
  f.before = level > 0 ? lt[level - 1] : 0;
  f.here = lt[level];
  f.after = level + 1 < gv.Lcap ? lt[level + 1] : 0;
  return f;
}
__host__ __device__ __forceinline__ int pick_flavour(long long here, long long other, long long N) {
  if (here >= kRowsLanes * N) return (other > 0 && other < kRowsLanes * N) ? kFlavSpread : kFlavRows;
  return here >= kSlotLanes * N ? kFlavSlots : kFlavFew;
}

// One wave's share of a forward level: sigma of the 64 nodes v0 .. v0+63 (v0 < N) of batch g.  The
// batch's deepest level also gets coef = 1 / sigma (unit demands: there is nothing to add to it).
// acc: kFwdWaveDoubles doubles of LDS of this wave's own (spread: accumulators, [node of the tile]
// [source]; rows: the tile's piece of the sigma array).  f: the batch's pair counts around the level.
constexpr int kFwdWaveDoubles = 8 * kWave;
template <bool kCountDag, typename TIn, typename TOut>
__device__ __forceinline__ void
fwd_wave(const int32_t* __restrict__ in_ptr, const int32_t* __restrict__ in_col, const GroupView& gv, int level,
         const LevelFill& f, long long* __restrict__ misc, int g, int v0, double* __restrict__ acc,
         const TileShare& ts) {
  // The wave's own index entries and in-link ranges are requested before the pair counts are looked at:
  // one round trip to memory less on the critical path of a small launch (always in bounds; what they
  // hold on a level the batch does not have is never used).
  const int lane = lane_id();
  const NodeIdx me = load_idx(gv.idxb + ((size_t)g * gv.Lcap + level) * gv.Npad + v0 + lane);
  LinkRange lr;
  lr.p0 = lr.p1 = 0;
  if (v0 + lane < gv.N) {
    lr.p0 = in_ptr[v0 + lane];
    lr.p1 = in_ptr[v0 + lane + 1];
  }
  if (f.here == 0) return;
  if (me.mask == 0) lr.p0 = lr.p1 = 0;  // nothing for nodes not on this level
  const bool init_coef = gv.coef != nullptr && gv.dem == nullptr && f.after == 0;
  switch (pick_flavour(f.here, f.before, gv.N)) {
    case kFlavRows:
      fwd_rows<kCountDag, TIn, TOut>(in_ptr, in_col, gv, level, init_coef, misc, g, v0, reinterpret_cast<TOut*>(acc), ts, me, lr);
      break;
    case kFlavSpread:
      fwd_spread<kCountDag, TIn, TOut>(in_ptr, in_col, gv, level, init_coef, misc, g, v0,
                                       reinterpret_cast<double(*)[kWave]>(acc), ts, me, lr);
      break;
    case kFlavSlots:
      fwd_few<kCountDag, true, TIn, TOut>(in_ptr, in_col, gv, level, init_coef, misc, g, v0, ts, me, lr);
      break;
    default:
      fwd_few<kCountDag, false, TIn, TOut>(in_ptr, in_col, gv, level, init_coef, misc, g, v0, ts, me, lr);
      break;
  }
}

// sigma of one level (1 .. deepest) for every batch of the group.  kShared: gv.split waves share a
// block of 64 nodes (a kernel of its own, so that the usual one keeps its constant loop bounds).
template <bool kCountDag, typename TIn, typename TOut, bool kShared = false>
__global__ void __launch_bounds__(kBlock)
k_fwd(const int32_t* __restrict__ in_ptr, const int32_t* __restrict__ in_col, GroupView gv, int level,
      long long* __restrict__ misc) {
  const int split = kShared ? gv.split : 1;
  int g, nblk;
  if (!map_block(gv.G, gv.bpb * split, gv.inflight, g, nblk)) return;
  const int w = __builtin_amdgcn_readfirstlane(nblk * kWavesPerBlock + (int)(threadIdx.x / kWave));
  const int v0 = w / split * kWave;
  if (v0 >= gv.N) return;
  const TileShare ts = {w % split, split};
  __shared__ double s_acc[kWavesPerBlock][kFwdWaveDoubles];
  fwd_wave<kCountDag, TIn, TOut>(in_ptr, in_col, gv, level, level_fill(gv, g, level), misc, g, v0,
                                 s_acc[threadIdx.x / kWave], ts);
}

// One wave's share of a backward level: coef of the 64 nodes u0 .. u0+63 (u0 < N) of batch g and the
// loads of their out-links.  With unit demands a batch's deepest level is skipped: the forward pass
// left its coef.  buf: bwd_wave_doubles<TS>() doubles of LDS of this wave's own (rows: the eight
// 64-lane sums of a node; spread: accumulators and sigma, [node of the tile][source]).  f: the batch's
// pair counts around the level.
template <typename TS>
__host__ __device__ constexpr int bwd_wave_doubles() {
  constexpr int kSpreadDoubles = 8 * kWave + 8 * kWave * (int)sizeof(TS) / 8;
  return kSpreadDoubles > kBwdDoubles ? kSpreadDoubles : kBwdDoubles;
}
template <typename TS, bool kDemand>
__device__ __forceinline__ void
bwd_wave(const int32_t* __restrict__ out_ptr, const int32_t* __restrict__ out_col, const GroupView& gv, int level,
         const LevelFill& f, int g, int u0, double* __restrict__ buf, const TileShare& ts) {
  const int lane = lane_id();  // as in fwd_wave: requested before the pair counts are looked at
  const NodeIdx me = load_idx(gv.idxb + ((size_t)g * gv.Lcap + level) * gv.Npad + u0 + lane);
  LinkRange lr;
  lr.p0 = lr.p1 = 0;
  if (u0 + lane < gv.N) {
    lr.p0 = out_ptr[u0 + lane];
    lr.p1 = out_ptr[u0 + lane + 1];
  }
  if (f.here == 0 || (!kDemand && f.after == 0)) return;
  if (me.mask == 0) lr.p0 = lr.p1 = 0;
  switch (pick_flavour(f.here, f.after, gv.N)) {
    case kFlavRows:
      bwd_rows<TS, kDemand>(out_ptr, out_col, gv, level, g, u0, buf, ts, me, lr);
      break;
    case kFlavSpread:
      bwd_spread<TS, kDemand>(out_ptr, out_col, gv, level, g, u0, reinterpret_cast<double(*)[kWave]>(buf),
                              reinterpret_cast<TS(*)[kWave]>(buf + 8 * kWave), ts, me, lr);
      break;
    case kFlavSlots:
      bwd_few<true, TS, kDemand>(out_ptr, out_col, gv, level, g, u0, ts, me, lr);
      break;
    default:
      bwd_few<false, TS, kDemand>(out_ptr, out_col, gv, level, g, u0, ts, me, lr);
      break;
  }
}

// coef and link loads of one level for every batch of the group.  kShared: as in k_fwd.
template <typename TS, bool kDemand, bool kShared = false>
__global__ void __launch_bounds__(kBlock)
k_bwd(const int32_t* __restrict__ out_ptr, const int32_t* __restrict__ out_col, GroupView gv, int level) {
  static_assert(!(kDemand && kShared), "a block's demand x distance slot belongs to one wave");
  const int split = kShared ? gv.split : 1;
  int g, nblk;
  if (!map_block(gv.G, gv.bpb * split, gv.inflight, g, nblk)) return;
  const int w = __builtin_amdgcn_readfirstlane(nblk * kWavesPerBlock + (int)(threadIdx.x / kWave));
  const int u0 = w / split * kWave;
  if (u0 >= gv.N) return;
  const TileShare ts = {w % split, split};
  __shared__ double s_buf[kWavesPerBlock][bwd_wave_doubles<TS>()];
  bwd_wave<TS, kDemand>(out_ptr, out_col, gv, level, level_fill(gv, g, level), g, u0, s_buf[threadIdx.x / kWave], ts);
}

// load[a] = (first group ? 0 : load[a]) + part[0][a] + part[1][a] + ... in that order.
__global__ void __launch_bounds__(kBlock)
k_reduce_part(const double* __restrict__ part, size_t Epad, int G, long long E, int first,
              double* __restrict__ load) {
  const long long a = (long long)blockIdx.x * kBlock + threadIdx.x;
  if (a >= E) return;
  double s = first ? 0.0 : load[a];
  int g = 0;
  for (; g + 16 <= G; g += 16) {  // sixteen requests in flight, added in batch order
    double x[16];
#pragma unroll
    for (int k = 0; k < 16; ++k) x[k] = part[(size_t)(g + k) * Epad + a];
#pragma unroll
    for (int k = 0; k < 16; ++k) s += x[k];
  }
  for (; g < G; ++g) s += part[(size_t)g * Epad + a];
  load[a] = s;
}

// ---------------------------------------------------------------------------------------
// a2a_distances outputs
// ---------------------------------------------------------------------------------------

// dist[s][v] from the level masks, through a 64 x 64 LDS tile so that rows of dist are written
// with consecutive lanes on consecutive nodes.  One wave per (batch, 64-node tile).  Any depth.
__global__ void __launch_bounds__(kWave)
k_extract_dist(GroupView gv, int tiles, int depth, int32_t* __restrict__ dist,
               long long* __restrict__ dist_sum) {
  int g, tile;
  if (!map_block(gv.G, tiles, kXcd, g, tile)) return;
  __shared__ int32_t t_d[kWave][kWave + 1];
  const int t = (int)threadIdx.x;
  const int v = tile * kWave + t;
  for (int j = 0; j < kWave; ++j) t_d[j][t] = -1;
  for (int l = 0; l <= depth; ++l) {
    uint64_t m = gv.bm[bm_at(gv, g / kSub, l, v, g % kSub)];
    while (m) {
      const int j = __builtin_ctzll(m);
      m &= m - 1;
      t_d[j][t] = l;
    }
  }
  __syncthreads();
  const int row0 = (gv.batch0 + g) * 64;
  const int cnt = min(64, gv.src_count - row0);
  if (dist != nullptr && v < gv.N) {
    for (int j = 0; j < cnt; ++j) __builtin_nontemporal_store(t_d[j][t], &dist[(size_t)(row0 + j) * gv.N + v]);
  }
  if (dist_sum != nullptr && t < cnt) {
    long long s = 0;
    const int lim = min(kWave, gv.N - tile * kWave);
    for (int i = 0; i < lim; ++i) {
      const int d = t_d[t][i];
      s += d > 0 ? d : 0;
    }
    if (s) atomicAdd((unsigned long long*)&dist_sum[row0 + t], (unsigned long long)s);
  }
}

// The same for depth < 256 without the LDS tile: a thread per node first folds the level masks into
// bit planes (plane k = OR of the masks of the levels whose bit k is set), so that the distance of
// source j is read off bit j of the planes; the wave then goes through the sources together (j is
// wave-uniform: no divergence), every lane writing its node's entry of row j.  The per-source sums
// come from ballots: bit k of the distances of source j over the wave's nodes is one popcount.
// `planes` = number of bits of `depth`.
__global__ void __launch_bounds__(kBlock)
k_extract_dist_planes(GroupView gv, int depth, int planes, int32_t* __restrict__ dist,
                      long long* __restrict__ dist_sum) {
  // The masks of the kSub batches of a super-batch share memory lines (64 bytes per node): their
  // workgroups for the same node block are neighbours in launch order and run on the same XCD, so
  // that the lines are fetched once and found in that XCD's L2 by the other seven.
  const unsigned i = blockIdx.x / kXcd;  // position in the XCD's own sequence of workgroups
  const int k = (int)(i % kSub);
  const int nblk = (int)((i / kSub) % (unsigned)gv.bpb);
  const int sb = (int)(i / kSub / (unsigned)gv.bpb) * kXcd + (int)(blockIdx.x % kXcd);
  const int g = sb * kSub + k;
  if (g >= gv.G) return;
  const int v = nblk * kBlock + (int)threadIdx.x;  // < Npad: the mask arrays are padded with zeros
  const int lane = lane_id();
  uint64_t B[8], R = 0;
#pragma unroll
  for (int p = 0; p < 8; ++p) B[p] = 0;
  for (int l = 0; l <= depth; ++l) {
    const uint64_t m = gv.bm[bm_at(gv, sb, l, v, k)];
    R |= m;
#pragma unroll
    for (int p = 0; p < 8; ++p)
      if ((l >> p) & 1) B[p] |= m;
  }
  const int row0 = (gv.batch0 + g) * 64;
  const int cnt = min(64, gv.src_count - row0);
  const bool live = v < gv.N;
  long long mine = 0;  // lane j: distance sum of source j over this wave's nodes
  for (int j = 0; j < cnt; ++j) {
    int d = 0;
    long long s = 0;
#pragma unroll
    for (int p = 0; p < 8; ++p) {
      if (p < planes) {
        const int bit = (int)((B[p] >> j) & 1ull);
        d |= bit << p;
        if (dist_sum != nullptr) s += (long long)__popcll(__ballot(bit != 0 && live)) << p;
      }
    }
    if (dist != nullptr && live)
      __builtin_nontemporal_store(((R >> j) & 1ull) ? d : -1, &dist[(size_t)(row0 + j) * gv.N + v]);
    if (lane == j) mine = s;
  }
  if (dist_sum != nullptr && lane < cnt && mine != 0)
    atomicAdd((unsigned long long*)&dist_sum[row0 + lane], (unsigned long long)mine);
}

// The same for depth < 128 with the loop over the sources taken eight at a time: the eight bits of a
// plane that belong to sources j0 .. j0+7 are spread to eight bytes (one shift-or pair, two masks),
// so that three or four instructions per plane build eight distances at once, packed in two words;
// a source the node has not been reached from gets the byte 0xFF, which the sign-extending byte
// extract turns into -1.  kPlanes (compile time: no branches in the loop) >= number of bits of the
// depth; planes beyond it stay empty.  kSum: per-source distance sums as well.
__device__ __forceinline__ uint32_t spread_bits4(uint32_t t, uint32_t pick) {
  // t: a byte repeated four times; pick: 0x08040201 or 0x80402010.  Byte i of the result = bit (i or i+4).
  return (((t & pick) + 0x7F7F7F7Fu) >> 7) & 0x01010101u;
}
template <int kPlanes, bool kSum>
__global__ void __launch_bounds__(kBlock)
k_extract_dist_packed(GroupView gv, int depth, int32_t* __restrict__ dist, long long* __restrict__ dist_sum) {
  static_assert(kPlanes >= 1 && kPlanes <= 7, "a distance and the mark for unreachable share a signed byte");
  const unsigned i = blockIdx.x / kXcd;  // workgroup order as in k_extract_dist_planes
  const int k = (int)(i % kSub);
  const int nblk = (int)((i / kSub) % (unsigned)gv.bpb);
  const int sb = (int)(i / kSub / (unsigned)gv.bpb) * kXcd + (int)(blockIdx.x % kXcd);
  const int g = sb * kSub + k;
  if (g >= gv.G) return;
  const int v = nblk * kBlock + (int)threadIdx.x;  // < Npad: the mask arrays are padded with zeros
  const int lane = lane_id();
  uint64_t B[kPlanes], R = 0;
#pragma unroll
  for (int p = 0; p < kPlanes; ++p) B[p] = 0;
  for (int l = 0; l <= depth; ++l) {
    const uint64_t m = gv.bm[bm_at(gv, sb, l, v, k)];
    R |= m;
#pragma unroll
    for (int p = 0; p < kPlanes; ++p)
      if ((l >> p) & 1) B[p] |= m;
  }
  const int row0 = (gv.batch0 + g) * 64;
  const int cnt = min(64, gv.src_count - row0);
  const bool live = v < gv.N;  // nodes past N: all masks 0, nothing stored, nothing added
  int mine = 0;                // lane j: distance sum of source j over this wave's nodes
#pragma unroll
  for (int j0 = 0; j0 < 64; j0 += 8) {
    if (j0 >= cnt) break;  // the same in all lanes
    uint32_t lo = 0, hi = 0;  // byte i: distance of source j0+i / j0+4+i
#pragma unroll
    for (int p = 0; p < kPlanes; ++p) {
      uint32_t t = (uint32_t)(B[p] >> j0) & 0xFFu;
      t |= t << 8;
      t |= t << 16;
      lo |= spread_bits4(t, 0x08040201u) << p;
      hi |= spread_bits4(t, 0x80402010u) << p;
    }
    if (dist != nullptr) {
      uint32_t t = (uint32_t)(~R >> j0) & 0xFFu;  // not reached
      t |= t << 8;
      t |= t << 16;
      const uint32_t nlo = spread_bits4(t, 0x08040201u), nhi = spread_bits4(t, 0x80402010u);
      const uint32_t wlo = lo | ((nlo << 8) - nlo), whi = hi | ((nhi << 8) - nhi);  // 0x01 -> 0xFF
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        if (j0 + e < cnt) {  // the same in all lanes; false only in a call's last, ragged batch
          int32_t* __restrict__ row = dist + (size_t)(row0 + j0 + e) * (size_t)gv.N;
          const int d = __builtin_amdgcn_sbfe((int)(e < 4 ? wlo : whi), 8 * (e & 3), 8);
          if (live) __builtin_nontemporal_store(d, &row[v]);  // written once, not read here: keep the masks in L2
        }
      }
    }
    if (kSum) {
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        int sum = 0;
#pragma unroll
        for (int p = 0; p < kPlanes; ++p)
          sum += __popcll(__builtin_amdgcn_ballot_w64(((B[p] >> (j0 + e)) & 1ull) != 0)) << p;
        if (lane == j0 + e) mine = sum;
      }
    }
  }
  if (kSum && lane < cnt && mine != 0)
    atomicAdd((unsigned long long*)&dist_sum[row0 + lane], (unsigned long long)mine);
}

// sigma[s][v] from the level-compact rows, transposed through LDS.  One wave per tile.
__global__ void __launch_bounds__(kWave)
k_extract_sigma(GroupView gv, int tiles, int depth, double* __restrict__ sigma_out) {
  int g, tile;
  if (!map_block(gv.G, tiles, kXcd, g, tile)) return;
  __shared__ double t_s[kWave][kWave + 1];
  const int t = (int)threadIdx.x;
  const int v0 = tile * kWave;
  const double* __restrict__ dat = gv.dat + (size_t)g * gv.Npad * 64;
  const float* __restrict__ datf = gv.datf + (size_t)g * gv.Npad * 128;
  for (int i = 0; i < kWave; ++i) t_s[t][i] = 0.0;
  for (int l = 0; l <= depth; ++l) {
    const NodeIdx me = load_idx(gv.idxb + ((size_t)g * gv.Lcap + l) * gv.Npad + v0 + t);
    uint64_t todo = __ballot(me.mask != 0);
    while (todo) {
      const int i = __builtin_ctzll(todo);
      todo &= todo - 1;
      const uint64_t mk = readlane64(me.mask, i);
      const uint32_t of = (uint32_t)__builtin_amdgcn_readlane((int)me.off, i);
      if ((mk >> t) & 1ull) {
        const uint32_t e = of + rank_in(mk);
        t_s[t][i] = l < gv.f32_levels ? (double)datf[e] : dat[e];
      }
    }
  }
  __syncthreads();
  const int row0 = (gv.batch0 + g) * 64;
  const int cnt = min(64, gv.src_count - row0);
  if (v0 + t < gv.N) {
    for (int j = 0; j < cnt; ++j)
      __builtin_nontemporal_store(t_s[j][t], &sigma_out[(size_t)(row0 + j) * gv.N + v0 + t]);
  }
}

// ---------------------------------------------------------------------------------------
// bookkeeping
// ---------------------------------------------------------------------------------------

// p[0..n) = 0, eight bytes per thread and step.  Used instead of the runtime's memset so that a
// call only ever enqueues kernels of this library on the caller's stream.
__global__ void __launch_bounds__(kBlock) k_zero(unsigned long long* __restrict__ p, size_t n) {
  const size_t stride = (size_t)gridDim.x * kBlock;
  for (size_t i = (size_t)blockIdx.x * kBlock + threadIdx.x; i < n; i += stride) p[i] = 0ull;
}

// Folds the per-batch level totals of a finished group into the call's running totals:
// misc[1] += sum of distances, misc[2] += reached pairs.  One workgroup; integer sums, so the
// order does not matter.
__global__ void __launch_bounds__(kBlock)
k_fold_counters(GroupView gv, int depth, long long* __restrict__ misc) {
  __shared__ long long s_r[2][kWavesPerBlock];
  const int t = (int)threadIdx.x;
  long long ds = 0, rc = 0;
  for (int i = t; i < gv.G * depth; i += kBlock) {
    const int g = i / depth, l = 1 + i % depth;
    const long long n = gv.ltot[(size_t)g * gv.Lcap + l];
    ds += n * l;
    rc += n;
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    ds += __shfl_xor(ds, o, kWave);
    rc += __shfl_xor(rc, o, kWave);
  }
  if (lane_id() == 0) {
    s_r[0][t / kWave] = ds;
    s_r[1][t / kWave] = rc;
  }
  __syncthreads();
  if (t == 0) {
    for (int w = 1; w < kWavesPerBlock; ++w) {
      s_r[0][0] += s_r[0][w];
      s_r[1][0] += s_r[1][w];
    }
    misc[1] += s_r[0][0];
    misc[2] += s_r[1][0];
  }
}

// Demand x distance of a call: each batch's blocks are added up in a fixed tree (one workgroup per
// batch; the sum lands in the batch's first slot), then the batches are added to *out one after the
// other in ascending order, so the bits do not depend on which batches share a group.
__global__ void __launch_bounds__(kBlock)
k_fold_weighted_batch(double* __restrict__ wpart, int nb64) {
  __shared__ double s_r[kBlock];
  const int t = (int)threadIdx.x;
  double* __restrict__ w = wpart + (size_t)blockIdx.x * nb64;
  double x = 0.0;
  for (int i = t; i < nb64; i += kBlock) x += w[i];
  s_r[t] = x;
  __syncthreads();
  for (int o = kBlock / 2; o > 0; o >>= 1) {
    if (t < o) s_r[t] += s_r[t + o];
    __syncthreads();
  }
  if (t == 0) w[0] = s_r[0];
}
__global__ void k_fold_weighted(const double* __restrict__ wpart, int G, int nb64, double* __restrict__ out) {
  if (threadIdx.x == 0 && blockIdx.x == 0) {
    double run = out[0];
    for (int g = 0; g < G; ++g) run += wpart[(size_t)g * nb64];
    out[0] = run;
  }
}

// ---------------------------------------------------------------------------------------
// level probe (a2a_topo_create): how deep does the BFS go from any source
// ---------------------------------------------------------------------------------------

// The BFS of k_bfs_level with two mask arrays used in turn instead of one per level, and no
// counting: a2a_topo_create runs it from every node once to learn the largest finite distance,
// which sizes the level slots of every later call.  Arrays: [SB][Npad][kSub].
__global__ void __launch_bounds__(kBfsBlock)
k_probe_init(uint64_t* __restrict__ front, uint64_t* __restrict__ seen, int N, int Npad, int SB, int src0) {
  int sb, nblk;
  if (!map_block(SB, Npad / kBfsNodes, kXcd, sb, nblk)) return;
  const int t = (int)threadIdx.x;
  const int v = nblk * kBfsNodes + t / kSub, k = t % kSub;
  const int s0 = src0 + (sb * kSub + k) * 64;
  const int j = v - s0;
  const uint64_t bit = (v < N && j >= 0 && j < 64) ? (1ull << j) : 0ull;
  const size_t at = ((size_t)sb * Npad + v) * kSub + k;
  front[at] = bit;
  seen[at] = bit;
}
__global__ void __launch_bounds__(kBfsBlock)
k_probe_level(const int32_t* __restrict__ in_ptr, const int32_t* __restrict__ in_col,
              const uint64_t* __restrict__ prev, uint64_t* __restrict__ next, uint64_t* __restrict__ seen, int N,
              int Npad, int SB, int* __restrict__ reached) {
  int sb, nblk;
  if (!map_block(SB, Npad / kBfsNodes, kXcd, sb, nblk)) return;
  const int t = (int)threadIdx.x;
  const int v = nblk * kBfsNodes + t / kSub, k = t % kSub;
  const size_t at = ((size_t)sb * Npad + v) * kSub + k;
  const uint64_t* __restrict__ pv = prev + (size_t)sb * Npad * kSub + k;
  uint64_t nw = 0;
  if (v < N) {
    const uint64_t sn = seen[at];
    uint64_t acc = 0;
    const int p1 = in_ptr[v + 1];
    for (int p = in_ptr[v]; p < p1; p += 8) {
      int u[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) u[j] = p + j < p1 ? in_col[p + j] : -1;
#pragma unroll
      for (int j = 0; j < 8; ++j)
        if (u[j] >= 0) acc |= pv[(size_t)u[j] * kSub];
    }
    nw = acc & ~sn;
    if (nw) seen[at] = sn | nw;
  }
  next[at] = nw;
  if (__ballot(nw != 0) != 0 && lane_id() == 0) *reached = 1;
}

// Final outputs of a call: totals and flag bits (bit 0: sigma reached 2^53, bit 1: some pair
// unreachable).
__global__ void k_finish(const long long* __restrict__ misc, long long pairs,
                         long long* __restrict__ dist_sum_total, long long* __restrict__ unreachable,
                         long long* __restrict__ flags) {
  if (threadIdx.x == 0 && blockIdx.x == 0) {
    const long long unr = pairs - misc[2];
    if (dist_sum_total) *dist_sum_total = misc[1];
    if (unreachable) *unreachable = unr;
    if (flags) *flags = (misc[0] ? 1 : 0) | (unr ? 2 : 0);
  }
}

// max (lowest link id on ties) and min of load[0..E): one workgroup.
__global__ void __launch_bounds__(1024)
k_load_extrema(const double* __restrict__ load, long long E, long long* __restrict__ out) {
  __shared__ double s_max[1024], s_min[1024];
  __shared__ long long s_arg[1024];
  const int t = (int)threadIdx.x;
  double mx = -1.0, mn = __builtin_huge_val();
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

// The same with link capacities (Sec. 3.1.1): utilisation load[a] / cap[a] instead of load[a];
// also the total capacity (sum over links in link order, block by block: a fixed order) and the
// largest total out-capacity of a node.  out[0..2] as k_load_extrema, out[3] = sum of cap,
// out[4] = largest node capacity, out[5] = 1 if some capacity is not a positive finite number.
// One workgroup; thread t takes nodes t, t + 1024, ... with their out-links.
__global__ void __launch_bounds__(1024)
k_util_extrema(const int32_t* __restrict__ out_ptr, const double* __restrict__ load,
               const double* __restrict__ cap, int N, long long* __restrict__ out) {
  __shared__ double s_max[1024], s_min[1024], s_sum[1024], s_cap[1024];
  __shared__ long long s_arg[1024];
  __shared__ int s_bad;
  const int t = (int)threadIdx.x;
  if (t == 0) s_bad = 0;
  __syncthreads();
  double mx = -1.0, mn = __builtin_huge_val(), sum = 0.0, cmax = 0.0;
  long long arg = -1;
  bool bad = false;
  for (int u = t; u < N; u += 1024) {
    double node_cap = 0.0;
    const int p1 = out_ptr[u + 1];
    for (int a = out_ptr[u]; a < p1; ++a) {
      const double c = cap[a];
      if (!(c > 0.0) || c > 1.7976931348623157e308) bad = true;
      const double x = load[a] / c;
      if (x > mx) {
        mx = x;
        arg = a;
      }
      if (x < mn) mn = x;
      node_cap += c;
    }
    sum += node_cap;
    if (node_cap > cmax) cmax = node_cap;
  }
  if (bad) s_bad = 1;
  s_max[t] = mx;
  s_min[t] = mn;
  s_arg[t] = arg;
  s_sum[t] = sum;
  s_cap[t] = cmax;
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
      s_sum[t] += s_sum[t + o];
      if (s_cap[t + o] > s_cap[t]) s_cap[t] = s_cap[t + o];
    }
    __syncthreads();
  }
  if (t == 0) {
    out[0] = __double_as_longlong(s_max[0]);
    out[1] = s_arg[0];
    out[2] = __double_as_longlong(s_min[0]);
    out[3] = __double_as_longlong(s_sum[0]);
    out[4] = __double_as_longlong(s_cap[0]);
    out[5] = s_bad;
  }
}

}  // namespace a2a_dev
