// a2a_topo host side: the C ABI of include/a2a_topo.h.  All-pairs hop distances, shortest-path
// counts and EwSP link loads of a direct-connect topology (Sec. 2.2, 5.2, 5.3, 5.4 of the paper)
// on one MI355X.  The kernels and the data model are in a2a_kernels.h.
//
// A "group" of G source batches (64 sources each) advances level by level together, one kernel
// launch per level and pass, as many batches as the caller's workspace holds:
//   bfs    levels 1 .. deepest (the handle knows the deepest level any source reaches)
//   offs   row offsets of the level-compact value array
//   fwd    levels 1 .. deepest: sigma
//   bwd    levels deepest .. 0: coef and per-batch link loads
//   sum    load += per-batch loads, in ascending batch order
// Nothing in a2a_distances / a2a_link_loads waits for the device or reads anything back: the
// launch sequence is fixed by the handle, and what depends on the data (which levels a batch
// has, how full they are) is decided inside the kernels.
#include <hip/hip_runtime.h>

#include <atomic>
#include <cmath>
#include <cstdint>
#include <cstdlib>
#include <cstring>
#include <new>
#include <vector>

#include "a2a_kernels.h"
#include "a2a_sssp_kernels.h"
#include "a2a_topo.h"

using namespace a2a_dev;

// Workspace of a2a_link_loads_static.  One copy per GPU, held until the process ends; in host
// code this name only stands for the symbol: its address on a device is taken once, in
// a2a_topo_create with that device current, and kept in the handle.
static __device__ __align__(256) unsigned char scratch[A2A_STATIC_WORKSPACE_BYTES];

struct a2a_topo {
  int32_t N = 0;
  int64_t E = 0;
  int32_t dmax = 0;
  int32_t dmax_in = 0;  // largest in-degree
  int32_t level_bound = 0;  // largest finite D(s,t), found by the level probe at create
  int32_t* d_out_ptr = nullptr;
  int32_t* d_out_col = nullptr;
  int32_t* d_in_ptr = nullptr;
  int32_t* d_in_col = nullptr;
  int32_t* d_in_link = nullptr;  // link id (position in the out-CSR) of every in-CSR entry
  // Read-back slots of a2a_schedule_bound / _cap: kSlots x kSlotWords int64 on the device and in
  // pinned host memory; every call takes the next slot, so calls on different streams or threads
  // do not share one.
  static constexpr unsigned kSlots = 64, kSlotWords = 8;
  int64_t* h_pinned = nullptr;
  int64_t* d_small = nullptr;
  mutable std::atomic<unsigned> next_slot{0};
  void* d_scratch = nullptr;    // device address of `scratch` on the handle's GPU
  // optional per-kernel timing (a2a_profile_enable); events are created per launch while it is on
  struct ProfRec {
    int cls, level;
    hipEvent_t beg, end;
  };
  mutable int prof_mode = 0;  // 0 off, 1 events, 2 events + shortest-path link count
  mutable std::vector<ProfRec> prof_recs;
  mutable int64_t prof_pairs_level[A2A_PROF_MAX_LEVELS] = {};
  mutable int64_t prof_dag_level[A2A_PROF_MAX_LEVELS] = {};
  mutable int64_t prof_calls = 0;
  mutable int32_t prof_depth = 0;
  mutable int32_t prof_groups = 0;
  mutable uint64_t prof_narrow = 0;
  mutable uint64_t prof_fwd_flavours = 0, prof_bwd_flavours = 0;
};

namespace {

enum {
  PROF_INIT = A2A_K_INIT, PROF_BFS = A2A_K_BFS, PROF_OFFSETS = A2A_K_OFFSETS, PROF_FWD = A2A_K_FWD_ROWS,
  PROF_FWD_FEW = A2A_K_FWD_FEW, PROF_FWD_SPREAD = A2A_K_FWD_SPREAD, PROF_BWD = A2A_K_BWD_ROWS,
  PROF_BWD_FEW = A2A_K_BWD_FEW, PROF_BWD_SPREAD = A2A_K_BWD_SPREAD, PROF_REDUCE = A2A_K_REDUCE, PROF_EXTRACT = A2A_K_EXTRACT,
  PROF_CLASSES = A2A_K_COUNT
};

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// Workspace layout for G batches.  All arrays are 256-byte aligned.
struct Layout {
  int G = 0;     // batches per group
  int Lcap = 0;  // level slots per batch (levels 0 .. Lcap-1)
  int Npad = 0;  // N rounded up to a multiple of 256
  int bpb = 0;   // 256-node blocks per batch
  int nb64 = 0;  // 64-node blocks per batch
  int SB = 0;    // super-batches of kSub batches (BFS arrays)
  bool values = false, loads = false, sssp = false;
  size_t Epad = 0;
  size_t off_misc = 0;       // int64 [8]: 0 sigma-inexact flag, 1 dist_sum, 2 reached pairs, 3 DAG links
  size_t off_ltot = 0;       // int64 [G][Lcap]
  size_t off_dag = 0;        // int64 [G][Lcap]
  size_t off_bsum = 0;       // int32 [SB*kSub][Lcap][nb64]
  size_t off_seen = 0;       // uint64 [SB][Npad][kSub]
  size_t off_bm = 0;         // uint64 [SB][Lcap][Npad][kSub]
  size_t off_idxb = 0;       // NodeIdx [G][Lcap][Npad]        (with sigma / loads)
  size_t off_dat = 0;        // [G][Npad*64] x 8 bytes: sigma.  Entry e of a level kept in double precision is
                             // the e-th double, that of a level kept in single precision the e-th float of
                             // the same array: the single-precision levels come first, so the two never meet
  size_t off_coef = 0;       // double [G][Npad*64]  coef (link loads only)
  size_t off_part = 0;       // double [G][Epad]
  size_t off_wpart = 0;      // double [G][nb64]  demand x distance per (batch, 64-node block)
  size_t off_cost = 0;       // int64 [G][Npad][64]   single-path baseline: cost, chosen link, paths through
  size_t off_pick = 0;       // int32 [G][Npad][64]
  size_t off_sub = 0;        // int32 [G][Npad][64]
  size_t off_iload = 0;      // uint64 [Epad]
  size_t total = 0;
};

// recommend: size for all batches (or one, if minimal); otherwise fit as many batches as
// ws_bytes holds (G = 0: not even one).
Layout make_layout(const a2a_topo* t, int32_t src_count, int flags, size_t ws_bytes, bool recommend,
                   bool minimal) {
  Layout L;
  L.values = (flags & (A2A_WS_SIGMA | A2A_WS_LOADS)) != 0;
  L.loads = (flags & A2A_WS_LOADS) != 0;
  L.sssp = (flags & A2A_WS_SSSP) != 0;
  L.Npad = (int)align_up((size_t)t->N, kBlock);
  L.bpb = L.Npad / kBlock;
  L.nb64 = L.Npad / kBfsNodes;
  L.Lcap = t->level_bound + 2;
  L.Epad = align_up((size_t)(t->E > 0 ? t->E : 1), 32);
  const int nb = (src_count + 63) / 64;
  auto total_for = [&](int G, Layout* out) {
    size_t off = 0;
    auto take = [&](size_t bytes) {
      const size_t at = off;
      off += align_up(bytes, 256);
      return at;
    };
    const size_t o_misc = take(64);
    const size_t SB = (size_t)(G + kSub - 1) / kSub;
    const size_t o_ltot = take(SB * kSub * L.Lcap * 8);
    const size_t o_dag = take((size_t)G * L.Lcap * 8);
    const size_t o_bsum = take(SB * kSub * L.Lcap * L.nb64 * 4);
    const size_t o_seen = take(SB * L.Npad * kSub * 8);
    const size_t o_bm = take(SB * L.Lcap * L.Npad * kSub * 8);
    const size_t o_idxb = L.values ? take((size_t)G * L.Lcap * L.Npad * sizeof(NodeIdx)) : 0;
    // + 256: rows are read in aligned 16-byte pairs, the last of which may reach one entry past the end
    const size_t o_dat = L.values ? take((size_t)G * L.Npad * 64 * 8 + 256) : 0;
    const size_t o_coef = L.loads ? take((size_t)G * L.Npad * 64 * 8 + 256) : 0;
    const size_t o_part = L.loads ? take((size_t)G * L.Epad * 8) : 0;
    const size_t o_wpart = L.loads ? take((size_t)G * L.nb64 * 8) : 0;
    const size_t o_cost = L.sssp ? take((size_t)G * L.Npad * 64 * 8) : 0;
    const size_t o_pick = L.sssp ? take((size_t)G * L.Npad * 64 * 4) : 0;
    const size_t o_sub = L.sssp ? take((size_t)G * L.Npad * 64 * 4) : 0;
    const size_t o_iload = L.sssp ? take(L.Epad * 8) : 0;
    if (out) {
      out->off_misc = o_misc;
      out->off_ltot = o_ltot;
      out->off_dag = o_dag;
      out->off_bsum = o_bsum;
      out->off_seen = o_seen;
      out->off_bm = o_bm;
      out->SB = (int)SB;
      out->off_idxb = o_idxb;
      out->off_dat = o_dat;
      out->off_coef = o_coef;
      out->off_part = o_part;
      out->off_wpart = o_wpart;
      out->off_cost = o_cost;
      out->off_pick = o_pick;
      out->off_sub = o_sub;
      out->off_iload = o_iload;
      out->total = off;
      out->G = G;
    }
    return off;
  };
  int G;
  if (recommend) {
    G = minimal ? 1 : nb;
  } else {
    if (total_for(1, nullptr) > ws_bytes) return L;  // G = 0
    int lo = 1, hi = nb;  // largest G that fits
    while (lo < hi) {
      const int mid = lo + (hi - lo + 1) / 2;
      if (total_for(mid, nullptr) <= ws_bytes)
        lo = mid;
      else
        hi = mid - 1;
    }
    G = lo;
  }
  total_for(G, &L);
  return L;
}

#define HIP_TRY(expr)           \
  do {                          \
    if ((expr) != hipSuccess) { \
      (void)hipGetLastError();  \
      return A2A_ERR_HIP;       \
    }                           \
  } while (0)

// Zeroes `bytes` bytes (rounded up to a multiple of 8; every array it is used on has that room) at
// the 8-byte aligned device address p with a kernel on the stream.
inline hipError_t zero_async(void* p, size_t bytes, hipStream_t st) {
  const size_t n = (bytes + 7) / 8;
  if (n == 0) return hipSuccess;
  const size_t blocks = (n + kBlock - 1) / kBlock;
  k_zero<<<(unsigned)(blocks < 16384 ? blocks : 16384), kBlock, 0, st>>>((unsigned long long*)p, n);
  return hipGetLastError();
}

// Brackets one kernel launch with two events while profiling is on.
struct ProfScope {
  const a2a_topo* t;
  hipStream_t st;
  a2a_topo::ProfRec rec{};
  bool live = false;
  ProfScope(const a2a_topo* t_, int cls, hipStream_t st_, int level = 0) : t(t_), st(st_) {
    if (t->prof_mode == 0) return;
    rec.cls = cls;
    rec.level = level;
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

inline unsigned grid_for(int G, int blocks_per_batch, int inflight = kXcd) {
  return (unsigned)((G + inflight - 1) / inflight * inflight * blocks_per_batch);
}

// Largest topology: a batch's value array (N * 64 entries of 8 bytes) is addressed with 32-bit
// byte offsets.
constexpr int32_t kMaxNodes = 4 * 1024 * 1024;

// Nominal lane layout of a level for the profile's kernel classes (the kernels pick per batch,
// from the same rule applied to the batch's own counts).
constexpr double kNominalRows = 8.0;

struct Run {
  const a2a_topo* t;
  Layout L;
  char* ws;
  hipStream_t st;
  int src_begin, src_count;
  const double* demand = nullptr;  // [N][src_count] by target, or nullptr: every pair has demand 1
  int inflight = kXcd;  // batches in flight = XCDs: one batch's node blocks per XCD at a time
  int split = 1;        // waves per block of 64 nodes in the forward / backward kernels (pick_split)
  mutable std::vector<double> lanes_per_node;  // profiling only: per level of the current group, pairs / (G*N)
  bool few(int level) const {
    return level >= 0 && level < (int)lanes_per_node.size() && lanes_per_node[level] > 0.0 &&
           lanes_per_node[level] < kNominalRows;
  }
  // Path counts on `level` are at most (largest in-degree)^level: while that is below 2^24 the level
  // keeps sigma in single precision (exact: whole numbers a float holds), which halves what the
  // forward pass writes and gathers and what the backward pass reads of it.  If a level is narrow,
  // so are all before it.
  bool narrow(int level) const { return (double)level * std::log2((double)std::max(t->dmax_in, 2)) < 24.0; }
  int f32_levels() const {
    int n = 1;
    while (n < L.Lcap && narrow(n)) ++n;
    return n;
  }
  long long* misc() const { return (long long*)(ws + L.off_misc); }
  GroupView view(int batch0, int G) const {
    GroupView gv;
    gv.bm = (uint64_t*)(ws + L.off_bm);
    gv.idxb = L.values ? (NodeIdx*)(ws + L.off_idxb) : nullptr;
    gv.seen = (uint64_t*)(ws + L.off_seen);
    gv.dat = L.values ? (double*)(ws + L.off_dat) : nullptr;
    gv.datf = L.values ? (float*)(ws + L.off_dat) : nullptr;
    gv.coef = L.loads ? (double*)(ws + L.off_coef) : nullptr;
    gv.bsum = (int*)(ws + L.off_bsum);
    gv.ltot = (long long*)(ws + L.off_ltot);
    gv.dag = (long long*)(ws + L.off_dag);
    gv.part = L.loads ? (double*)(ws + L.off_part) : nullptr;
    gv.Epad = L.Epad;
    gv.N = t->N;
    gv.Npad = L.Npad;
    gv.Lcap = L.Lcap;
    gv.G = G;
    gv.SB = (G + kSub - 1) / kSub;
    gv.bpb = L.bpb;
    gv.nb64 = L.nb64;
    gv.inflight = inflight;
    gv.split = split;
    gv.src_begin = src_begin;
    gv.src_count = src_count;
    gv.batch0 = batch0;
    gv.f32_levels = f32_levels();
    gv.dem = demand;
    gv.dem_ld = src_count;
    gv.wpart = L.loads ? (double*)(ws + L.off_wpart) : nullptr;
    return gv;
  }
};

// A group that cannot fill the chip with one wave per 64 nodes lets 2, 4 or 8 waves share each block of
// 64 nodes (a tile of eight nodes is the unit): a wave's chain of dependent memory requests, which
// is what a launch of a small group costs, gets that much shorter.  Not with demands, not while
// shortest-path links are counted (see GroupView).
constexpr int kSplitWaves = 8192;
int pick_split(const a2a_topo* t, int G, int nb64, bool demand) {
  if (demand || t->prof_mode == 2) return 1;
  int split = 1;
  while (split < 8 && (long long)G * nb64 * split * 2 <= kSplitWaves) split *= 2;
  return split;
}

// BFS of one group: levels 1 .. top (the handle's deepest level, one more when the backward pass
// will look at the empty level after a batch's last one).
int run_bfs(const Run& r, const GroupView& gv, int top) {
  const a2a_topo* t = r.t;
  const Layout& L = r.L;
  HIP_TRY(zero_async(gv.ltot, (size_t)gv.SB * kSub * L.Lcap * 8, r.st));
  {
    ProfScope ps(t, PROF_INIT, r.st);
    k_init_group<<<grid_for(gv.SB, L.nb64), kBfsBlock, 0, r.st>>>(gv);
  }
  for (int l = 1; l <= top; ++l) {
    ProfScope ps(t, PROF_BFS, r.st, l);
    k_bfs_level<<<grid_for(gv.SB, L.nb64), kBfsBlock, 0, r.st>>>(t->d_in_ptr, t->d_in_col, gv, l);
  }
  HIP_TRY(hipGetLastError());
  r.lanes_per_node.clear();
  if (t->prof_mode) {  // profiling only: how full each level is (this is the one place that waits)
    try {
      std::vector<long long> lt((size_t)gv.G * L.Lcap);
      HIP_TRY(hipMemcpyAsync(lt.data(), gv.ltot, lt.size() * 8, hipMemcpyDeviceToHost, r.st));
      HIP_TRY(hipStreamSynchronize(r.st));
      r.lanes_per_node.assign((size_t)L.Lcap, 0.0);
      int d = 0;
      for (int g = 0; g < gv.G; ++g)
        for (int k = 0; k < L.Lcap; ++k) {
          const long long n = lt[(size_t)g * L.Lcap + k];
          r.lanes_per_node[k] += (double)n;
          if (n > 0 && k > d) d = k;
        }
      for (int k = 0; k <= d; ++k)
        t->prof_pairs_level[k < A2A_PROF_MAX_LEVELS ? k : A2A_PROF_MAX_LEVELS - 1] += (int64_t)r.lanes_per_node[k];
      // which lane layout and precision each batch's kernels pick on each level (the kernels' own rule)
      for (int g = 0; g < gv.G; ++g)
        for (int k = 0; k + 1 < L.Lcap; ++k) {
          const long long* row = &lt[(size_t)g * L.Lcap];
          const long long here = row[k], after = row[k + 1], before = k > 0 ? row[k - 1] : 0;
          if (here == 0) continue;
          if (k >= 1 && L.values)
            t->prof_fwd_flavours |= 1ull << (3 * pick_flavour(here, before, t->N) + (r.narrow(k) ? 0 : (r.narrow(k - 1) ? 1 : 2)));
          if (L.loads && (r.demand != nullptr || after > 0))
            t->prof_bwd_flavours |= 1ull << (2 * pick_flavour(here, after, t->N) + (r.narrow(k) ? 0 : 1));
        }
      for (auto& x : r.lanes_per_node) x /= (double)gv.G * (double)t->N;
      if (d > t->prof_depth) t->prof_depth = d;
      t->prof_groups++;
    } catch (const std::bad_alloc&) {
      return A2A_ERR_NO_MEMORY;
    }
  }
  return A2A_OK;
}

// Row offsets, then sigma for levels 1 .. depth.
int run_fwd(const Run& r, const GroupView& gv, int depth) {
  const a2a_topo* t = r.t;
  const Layout& L = r.L;
  {
    // With demands the backward pass also visits a batch's deepest level and looks at the (empty)
    // level after it, which the BFS has computed: its index entries are written too.
    const int idx_depth = gv.dem != nullptr ? depth + 1 : depth;
    ProfScope ps(t, PROF_OFFSETS, r.st);
    if (idx_depth >= 1) k_scan_blocks<<<(unsigned)(gv.G * idx_depth), kWave, 0, r.st>>>(gv, idx_depth);
    // one workgroup per (super-batch, 64 nodes) works through all levels, unless that leaves most of the chip idle
    const int levels = (long long)gv.SB * L.nb64 >= 2048 ? idx_depth + 1 : 1;
    const int chunks = (idx_depth + levels) / levels;
    k_write_offsets<<<grid_for(gv.SB, L.nb64 * chunks), kBfsBlock, 0, r.st>>>(gv, idx_depth, levels);
  }
  const unsigned grid = grid_for(gv.G, L.bpb * gv.split, r.inflight);
  for (int l = 1; l <= depth; ++l) {
    const int cls = r.few(l) ? PROF_FWD_FEW : (r.few(l - 1) ? PROF_FWD_SPREAD : PROF_FWD);
    ProfScope ps(t, cls, r.st, l);
    const bool count = t->prof_mode == 2;
    auto launch = [&](auto kernel) {
      kernel<<<grid, kBlock, 0, r.st>>>(t->d_in_ptr, t->d_in_col, gv, l, r.misc());
    };
    // precision of the level gathered from and of the one written; waves sharing blocks of nodes or not
    const bool shared = gv.split > 1;  // never while counting
    if (r.narrow(l))
      count    ? launch(k_fwd<true, float, float>)
      : shared ? launch(k_fwd<false, float, float, true>)
               : launch(k_fwd<false, float, float>);
    else if (r.narrow(l - 1))
      count    ? launch(k_fwd<true, float, double>)
      : shared ? launch(k_fwd<false, float, double, true>)
               : launch(k_fwd<false, float, double>);
    else
      count    ? launch(k_fwd<true, double, double>)
      : shared ? launch(k_fwd<false, double, double, true>)
               : launch(k_fwd<false, double, double>);
    if (t->prof_mode != 0 && l < 64 && r.narrow(l - 1)) t->prof_narrow |= 1ull << l;
  }
  HIP_TRY(hipGetLastError());
  if (t->prof_mode == 2) {  // shortest-path links into each level, for the roofline accounting
    try {
      std::vector<long long> dg((size_t)gv.G * L.Lcap);
      HIP_TRY(hipMemcpyAsync(dg.data(), gv.dag, dg.size() * 8, hipMemcpyDeviceToHost, r.st));
      HIP_TRY(hipStreamSynchronize(r.st));
      for (int g = 0; g < gv.G; ++g)
        for (int l = 0; l <= depth; ++l)
          t->prof_dag_level[l < A2A_PROF_MAX_LEVELS ? l : A2A_PROF_MAX_LEVELS - 1] += dg[(size_t)g * L.Lcap + l];
    } catch (const std::bad_alloc&) {
      return A2A_ERR_NO_MEMORY;
    }
  }
  return A2A_OK;
}

// Level totals of the finished group go into the call's running totals.
int run_fold(const Run& r, const GroupView& gv, int depth) {
  k_fold_counters<<<1, kBlock, 0, r.st>>>(gv, depth, r.misc());
  HIP_TRY(hipGetLastError());
  return A2A_OK;
}

// Largest finite hop distance of the topology: the BFS from every node, 64 sources per mask, as
// many super-batches at a time as about 1 GiB of temporary device memory holds.  Runs on the
// default stream and waits (this is a2a_topo_create).
int probe_depth(const a2a_topo* t, int32_t* depth_out) {
  const int N = t->N;
  const int Npad = (int)align_up((size_t)N, kBlock);
  const int nb64 = Npad / kBfsNodes;
  const int sb_all = ((N + 63) / 64 + kSub - 1) / kSub;
  const size_t per_sb = (size_t)Npad * kSub * 8;  // one mask array of one super-batch
  const int sb_grp = (int)std::max<size_t>(1, std::min<size_t>((size_t)sb_all, ((size_t)1 << 30) / (3 * per_sb)));
  constexpr int kChunk = 16;  // levels between two looks at the "anything new" flags
  uint64_t* buf = nullptr;
  int* d_flags = nullptr;
  int h_flags[kChunk];
  int rc = A2A_OK, deepest = 0;
  if (hipMalloc((void**)&buf, 3 * per_sb * sb_grp) != hipSuccess ||
      hipMalloc((void**)&d_flags, kChunk * sizeof(int)) != hipSuccess) {
    (void)hipGetLastError();
    if (buf) (void)hipFree(buf);
    return A2A_ERR_HIP;
  }
  uint64_t* ring[2] = {buf, buf + per_sb / 8 * sb_grp};
  uint64_t* seen = buf + 2 * (per_sb / 8) * sb_grp;
  for (int sb0 = 0; sb0 < sb_all && rc == A2A_OK; sb0 += sb_grp) {
    const int SB = std::min(sb_grp, sb_all - sb0);
    k_probe_init<<<grid_for(SB, nb64), kBfsBlock, 0, nullptr>>>(ring[0], seen, N, Npad, SB, sb0 * kSub * 64);
    int level = 1;
    bool done = false;
    while (!done && rc == A2A_OK) {
      rc = zero_async(d_flags, sizeof(h_flags), nullptr) == hipSuccess ? A2A_OK : A2A_ERR_HIP;
      for (int k = 0; k < kChunk && rc == A2A_OK; ++k)
        k_probe_level<<<grid_for(SB, nb64), kBfsBlock, 0, nullptr>>>(t->d_in_ptr, t->d_in_col, ring[(level + k + 1) & 1],
                                                                   ring[(level + k) & 1], seen, N, Npad, SB, d_flags + k);
      if (rc == A2A_OK && (hipGetLastError() != hipSuccess ||
                           hipMemcpy(h_flags, d_flags, sizeof(h_flags), hipMemcpyDeviceToHost) != hipSuccess))
        rc = A2A_ERR_HIP;
      for (int k = 0; k < kChunk && rc == A2A_OK && !done; ++k) {
        if (h_flags[k] == 0)
          done = true;  // level + k reached nothing new: every later level is empty too
        else
          deepest = std::max(deepest, level + k);
      }
      level += kChunk;
      if (level > N) done = true;  // a shortest path has at most N - 1 links
    }
  }
  (void)hipFree(buf);
  (void)hipFree(d_flags);
  if (rc != A2A_OK) (void)hipGetLastError();
  *depth_out = deepest;
  return rc;
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
  if (N > kMaxNodes) return A2A_ERR_NOT_IMPLEMENTED;
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
  std::vector<int32_t> in_ptr, in_col, in_link;
  try {
    in_ptr.assign((size_t)N + 1, 0);
    in_col.resize((size_t)(E > 0 ? E : 1));
    in_link.resize((size_t)(E > 0 ? E : 1));
    for (int64_t p = 0; p < E; ++p) in_ptr[(size_t)col_idx[p] + 1]++;
    for (int32_t v = 0; v < N; ++v) in_ptr[(size_t)v + 1] += in_ptr[v];
    std::vector<int32_t> fill(in_ptr.begin(), in_ptr.end() - 1);
    for (int32_t u = 0; u < N; ++u)  // ascending link id => in-lists are stable in link order
      for (int32_t p = row_ptr[u]; p < row_ptr[u + 1]; ++p) {
        const size_t at = (size_t)fill[col_idx[p]]++;
        in_col[at] = u;
        in_link[at] = p;
      }
    for (int32_t v = 0; v < N; ++v) t->dmax_in = std::max(t->dmax_in, in_ptr[(size_t)v + 1] - in_ptr[v]);
  } catch (const std::bad_alloc&) {
    delete t;
    return A2A_ERR_NO_MEMORY;
  }
  t->N = N;
  t->E = E;
  t->dmax = dmax;
  const size_t pb = ((size_t)N + 1) * sizeof(int32_t);
  const size_t cb = (size_t)(E > 0 ? E : 1) * sizeof(int32_t);
  const size_t slot_bytes = (size_t)a2a_topo::kSlots * a2a_topo::kSlotWords * sizeof(int64_t);
  bool ok = hipMalloc((void**)&t->d_out_ptr, pb) == hipSuccess &&
            hipMalloc((void**)&t->d_out_col, cb) == hipSuccess &&
            hipMalloc((void**)&t->d_in_ptr, pb) == hipSuccess &&
            hipMalloc((void**)&t->d_in_col, cb) == hipSuccess &&
            hipMalloc((void**)&t->d_in_link, cb) == hipSuccess &&
            hipMalloc((void**)&t->d_small, slot_bytes) == hipSuccess &&
            hipHostMalloc((void**)&t->h_pinned, slot_bytes, hipHostMallocDefault) == hipSuccess;
  ok = ok && hipGetSymbolAddress(&t->d_scratch, HIP_SYMBOL(scratch)) == hipSuccess && t->d_scratch != nullptr;
  ok = ok && hipMemset(t->d_small, 0, slot_bytes) == hipSuccess &&
       hipMemcpy(t->d_out_ptr, row_ptr, pb, hipMemcpyHostToDevice) == hipSuccess &&
       hipMemcpy(t->d_in_ptr, in_ptr.data(), pb, hipMemcpyHostToDevice) == hipSuccess;
  if (ok && E > 0)
    ok = hipMemcpy(t->d_out_col, col_idx, (size_t)E * 4, hipMemcpyHostToDevice) == hipSuccess &&
         hipMemcpy(t->d_in_col, in_col.data(), (size_t)E * 4, hipMemcpyHostToDevice) == hipSuccess &&
         hipMemcpy(t->d_in_link, in_link.data(), (size_t)E * 4, hipMemcpyHostToDevice) == hipSuccess;
  if (ok && E > 0) ok = probe_depth(t, &t->level_bound) == A2A_OK;
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
  for (auto& rec : t->prof_recs) {
    (void)hipEventDestroy(rec.beg);
    (void)hipEventDestroy(rec.end);
  }
  if (t->d_out_ptr) (void)hipFree(t->d_out_ptr);
  if (t->d_out_col) (void)hipFree(t->d_out_col);
  if (t->d_in_ptr) (void)hipFree(t->d_in_ptr);
  if (t->d_in_col) (void)hipFree(t->d_in_col);
  if (t->d_in_link) (void)hipFree(t->d_in_link);
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
  if (!t || src_count < 0 || (size_t)src_count > align_up((size_t)t->N, 64)) return 0;
  if (src_count == 0) return 256;
  const Layout L = make_layout(t, src_count, flags & 0xff, 0, true, (flags & A2A_WS_MINIMAL) != 0);
  return L.total;
}

int a2a_distances(const a2a_topo* t, int32_t src_begin, int32_t src_count, int32_t* dist, double* sigma,
                  int64_t* dist_sum, int64_t* unreachable, int64_t* flags, void* workspace,
                  size_t workspace_bytes, void* hip_stream) {
  int rc = check_common(t, src_begin, src_count, workspace);
  if (rc != A2A_OK) return rc;
  hipStream_t st = (hipStream_t)hip_stream;
  if (src_count == 0) {
    if (unreachable) HIP_TRY(zero_async(unreachable, 8, st));
    if (flags) HIP_TRY(zero_async(flags, 8, st));
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
  HIP_TRY(zero_async(r.misc(), 64, st));
  if (dist_sum) HIP_TRY(zero_async(dist_sum, (size_t)src_count * 8, st));
  const int nb = (src_count + 63) / 64;
  const int tiles = L.Npad / kWave;
  for (int b0 = 0; b0 < nb; b0 += L.G) {
    r.split = pick_split(t, nb - b0 < L.G ? nb - b0 : L.G, L.nb64, false);
    const GroupView gv = r.view(b0, nb - b0 < L.G ? nb - b0 : L.G);
    const int depth = t->level_bound;
    rc = run_bfs(r, gv, depth);
    if (rc != A2A_OK) return rc;
    if (sigma) {
      rc = run_fwd(r, gv, depth);
      if (rc != A2A_OK) return rc;
      ProfScope ps(t, PROF_EXTRACT, st);
      k_extract_sigma<<<grid_for(gv.G, tiles), kWave, 0, st>>>(gv, tiles, depth, sigma);
    }
    if (dist || dist_sum) {
      ProfScope ps(t, PROF_EXTRACT, st);
      if (depth < 128) {  // eight sources at a time, the number of bit planes fixed at compile time
        const unsigned grid = grid_for(gv.SB, L.bpb * kSub);
        auto launch = [&](auto kernel) { kernel<<<grid, kBlock, 0, st>>>(gv, depth, dist, (long long*)dist_sum); };
        if (depth < 8)
          dist_sum ? launch(k_extract_dist_packed<3, true>) : launch(k_extract_dist_packed<3, false>);
        else if (depth < 32)
          dist_sum ? launch(k_extract_dist_packed<5, true>) : launch(k_extract_dist_packed<5, false>);
        else
          dist_sum ? launch(k_extract_dist_packed<7, true>) : launch(k_extract_dist_packed<7, false>);
      } else if (depth < 256) {
        int planes = 0;
        while ((depth >> planes) != 0) ++planes;
        k_extract_dist_planes<<<grid_for(gv.SB, L.bpb * kSub), kBlock, 0, st>>>(gv, depth, planes, dist,
                                                                                (long long*)dist_sum);
      } else {
        k_extract_dist<<<grid_for(gv.G, tiles), kWave, 0, st>>>(gv, tiles, depth, dist, (long long*)dist_sum);
      }
    }
    rc = run_fold(r, gv, depth);
    if (rc != A2A_OK) return rc;
  }
  k_finish<<<1, 64, 0, st>>>(r.misc(), (long long)src_count * (t->N - 1), nullptr, (long long*)unreachable,
                             (long long*)flags);
  HIP_TRY(hipGetLastError());
  if (t->prof_mode) t->prof_calls++;
  return A2A_OK;
}

namespace {

// a2a_link_loads (demand == nullptr) and a2a_link_loads_demand.
int link_loads(const a2a_topo* t, int32_t src_begin, int32_t src_count, const double* demand, double* load,
               double* weighted_dist, int64_t* dist_sum_total, int64_t* flags, void* workspace,
               size_t workspace_bytes, void* hip_stream) {
  int rc = check_common(t, src_begin, src_count, workspace);
  if (rc != A2A_OK) return rc;
  if (!load && t->E > 0) return A2A_ERR_INVALID_ARG;
  hipStream_t st = (hipStream_t)hip_stream;
  if (weighted_dist) HIP_TRY(zero_async(weighted_dist, 8, st));
  if (src_count == 0) {
    if (t->E > 0) HIP_TRY(zero_async(load, (size_t)t->E * 8, st));
    if (dist_sum_total) HIP_TRY(zero_async(dist_sum_total, 8, st));
    if (flags) HIP_TRY(zero_async(flags, 8, st));
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
  r.demand = demand;
  const Layout& L = r.L;
  HIP_TRY(zero_async(r.misc(), 64, st));
  const int nb = (src_count + 63) / 64;
  for (int b0 = 0; b0 < nb; b0 += L.G) {
    r.split = pick_split(t, nb - b0 < L.G ? nb - b0 : L.G, L.nb64, demand != nullptr);
    const GroupView gv = r.view(b0, nb - b0 < L.G ? nb - b0 : L.G);
    const int depth = t->level_bound;
    rc = run_bfs(r, gv, demand ? depth + 1 : depth);
    if (rc != A2A_OK) return rc;
    rc = run_fwd(r, gv, depth);
    if (rc != A2A_OK) return rc;
    if (t->E > 0) {
      HIP_TRY(zero_async(gv.part, (size_t)gv.G * L.Epad * 8, st));
      if (demand) HIP_TRY(zero_async(gv.wpart, (size_t)gv.G * L.nb64 * 8, st));
      const unsigned grid = grid_for(gv.G, L.bpb * gv.split, r.inflight);
      // Unit demands: a batch's deepest level has no successors and its coef = 1/sigma was left by
      // the forward pass, nothing to add (the kernel skips it).  With demands it is visited like the others.
      for (int l = demand ? depth : depth - 1; l >= 0; --l) {
        const int cls = r.few(l) ? PROF_BWD_FEW : (r.few(l + 1) ? PROF_BWD_SPREAD : PROF_BWD);
        ProfScope ps(t, cls, st, l);
        auto launch = [&](auto kernel) { kernel<<<grid, kBlock, 0, st>>>(t->d_out_ptr, t->d_out_col, gv, l); };
        if (demand)  // precision of this level's sigma
          r.narrow(l) ? launch(k_bwd<float, true>) : launch(k_bwd<double, true>);
        else if (gv.split > 1)
          r.narrow(l) ? launch(k_bwd<float, false, true>) : launch(k_bwd<double, false, true>);
        else
          r.narrow(l) ? launch(k_bwd<float, false>) : launch(k_bwd<double, false>);
      }
      if (demand && weighted_dist) {
        k_fold_weighted_batch<<<(unsigned)gv.G, kBlock, 0, st>>>(gv.wpart, L.nb64);
        k_fold_weighted<<<1, 64, 0, st>>>(gv.wpart, gv.G, L.nb64, weighted_dist);
      }
      ProfScope ps(t, PROF_REDUCE, st);
      k_reduce_part<<<(unsigned)((t->E + kBlock - 1) / kBlock), kBlock, 0, st>>>(
          gv.part, L.Epad, gv.G, (long long)t->E, b0 == 0 ? 1 : 0, load);
    }
    rc = run_fold(r, gv, depth);
    if (rc != A2A_OK) return rc;
  }
  k_finish<<<1, 64, 0, st>>>(r.misc(), (long long)src_count * (t->N - 1), (long long*)dist_sum_total,
                             nullptr, (long long*)flags);
  HIP_TRY(hipGetLastError());
  if (t->prof_mode) t->prof_calls++;
  return A2A_OK;
}

}  // namespace

int a2a_link_loads(const a2a_topo* t, int32_t src_begin, int32_t src_count, double* load,
                   int64_t* dist_sum_total, int64_t* flags, void* workspace, size_t workspace_bytes,
                   void* hip_stream) {
  return link_loads(t, src_begin, src_count, nullptr, load, nullptr, dist_sum_total, flags, workspace,
                    workspace_bytes, hip_stream);
}

int a2a_link_loads_static(const a2a_topo* t, int32_t src_begin, int32_t src_count, double* load,
                          int64_t* dist_sum_total, int64_t* flags, void* hip_stream) {
  if (!t) return A2A_ERR_INVALID_ARG;
  if (src_count > 0 && src_count <= t->N) {
    // refuse before anything is enqueued: the array must hold at least one batch of this topology
    const Layout L = make_layout(t, src_count, A2A_WS_LOADS, A2A_STATIC_WORKSPACE_BYTES, false, false);
    if (L.G < 1) return A2A_ERR_WORKSPACE_TOO_SMALL;
  }
  return link_loads(t, src_begin, src_count, nullptr, load, nullptr, dist_sum_total, flags, t->d_scratch,
                    A2A_STATIC_WORKSPACE_BYTES, hip_stream);
}

int a2a_link_loads_demand(const a2a_topo* t, int32_t src_begin, int32_t src_count, const double* demand,
                          double* load, double* weighted_dist, int64_t* dist_sum_total, int64_t* flags,
                          void* workspace, size_t workspace_bytes, void* hip_stream) {
  if (!demand) return A2A_ERR_INVALID_ARG;
  return link_loads(t, src_begin, src_count, demand, load, weighted_dist, dist_sum_total, flags, workspace,
                    workspace_bytes, hip_stream);
}

int a2a_sssp_loads(const a2a_topo* t, int32_t src_begin, int32_t src_count, int32_t iter_sources, double* load,
                   int64_t* dist_sum_total, int64_t* flags, void* workspace, size_t workspace_bytes,
                   void* hip_stream) {
  int rc = check_common(t, src_begin, src_count, workspace);
  if (rc != A2A_OK) return rc;
  if (!load && t->E > 0) return A2A_ERR_INVALID_ARG;
  if (iter_sources <= 0 || iter_sources % 64 != 0) return A2A_ERR_INVALID_ARG;
  hipStream_t st = (hipStream_t)hip_stream;
  if (src_count == 0) {
    if (t->E > 0) HIP_TRY(zero_async(load, (size_t)t->E * 8, st));
    if (dist_sum_total) HIP_TRY(zero_async(dist_sum_total, 8, st));
    if (flags) HIP_TRY(zero_async(flags, 8, st));
    return A2A_OK;
  }
  // one iteration = one group: the workspace has to hold all its batches
  const int nb = (src_count + 63) / 64;
  const int per_iter = std::min(iter_sources / 64, nb);
  Run r;
  r.t = t;
  r.L = make_layout(t, per_iter * 64, A2A_WS_SSSP, workspace_bytes, false, false);
  if (r.L.G < per_iter) return A2A_ERR_WORKSPACE_TOO_SMALL;
  r.ws = (char*)workspace;
  r.st = st;
  r.src_begin = src_begin;
  r.src_count = src_count;
  const Layout& L = r.L;
  SsspView sv;
  sv.cost = (long long*)(r.ws + L.off_cost);
  sv.pick = (int*)(r.ws + L.off_pick);
  sv.sub = (int*)(r.ws + L.off_sub);
  sv.iload = (unsigned long long*)(r.ws + L.off_iload);
  HIP_TRY(zero_async(r.misc(), 64, st));
  HIP_TRY(zero_async(sv.iload, L.Epad * 8, st));
  const int depth = t->level_bound;
  for (int b0 = 0; b0 < nb; b0 += per_iter) {
    const GroupView gv = r.view(b0, nb - b0 < per_iter ? nb - b0 : per_iter);
    rc = run_bfs(r, gv, depth);
    if (rc != A2A_OK) return rc;
    // nodes per wave: 64, or 8 when the iteration has too few batches to give every SIMD a wave otherwise
    const int npw = (long long)gv.G * L.Npad >= 64ll * 4096 ? 64 : 8;
    const unsigned grid = grid_for(gv.G, L.bpb * (kWave / npw), r.inflight);
    for (int l = 1; l <= depth; ++l)
      k_sssp_fwd<<<grid, kBlock, 0, st>>>(t->d_in_ptr, t->d_in_col, t->d_in_link, gv, sv, l, npw);
    for (int l = depth; l >= 0; --l)
      k_sssp_bwd<<<grid, kBlock, 0, st>>>(t->d_out_ptr, t->d_out_col, gv, sv, l, npw);
    rc = run_fold(r, gv, depth);
    if (rc != A2A_OK) return rc;
  }
  if (t->E > 0)
    k_sssp_output<<<(unsigned)((t->E + kBlock - 1) / kBlock), kBlock, 0, st>>>(sv.iload, (long long)t->E, load);
  k_finish<<<1, 64, 0, st>>>(r.misc(), (long long)src_count * (t->N - 1), (long long*)dist_sum_total,
                             nullptr, (long long*)flags);
  HIP_TRY(hipGetLastError());
  return A2A_OK;
}

int a2a_schedule_bound(const a2a_topo* t, const double* load, int64_t sum_dist, int64_t flags,
                       double m_bytes, double b_bytes_per_s, a2a_bound* out, void* hip_stream) {
  if (!t || !out || !load || t->E <= 0 || !(m_bytes > 0.0) || !(b_bytes_per_s > 0.0) || sum_dist < 0)
    return A2A_ERR_INVALID_ARG;
  hipStream_t st = (hipStream_t)hip_stream;
  const size_t slot = (size_t)(t->next_slot.fetch_add(1) % a2a_topo::kSlots) * a2a_topo::kSlotWords;
  int64_t* d_res = t->d_small + slot;
  const int64_t* h_res = t->h_pinned + slot;
  k_load_extrema<<<1, 1024, 0, st>>>(load, (long long)t->E, (long long*)d_res);
  HIP_TRY(hipGetLastError());
  HIP_TRY(hipMemcpyAsync((void*)h_res, d_res, 3 * sizeof(int64_t), hipMemcpyDeviceToHost, st));
  HIP_TRY(hipStreamSynchronize(st));
  double lmax, lmin;
  std::memcpy(&lmax, &h_res[0], 8);
  std::memcpy(&lmin, &h_res[2], 8);
  const double m = m_bytes, b = b_bytes_per_s;
  out->max_load = lmax;
  out->argmax_arc = h_res[1];
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

int a2a_schedule_bound_cap(const a2a_topo* t, const double* load, const double* cap, int64_t sum_dist,
                           int64_t flags, double m_bytes, double b_bytes_per_s, a2a_bound_cap* out,
                           void* hip_stream) {
  if (!t || !out || !load || !cap || t->E <= 0 || !(m_bytes > 0.0) || !(b_bytes_per_s > 0.0) || sum_dist < 0)
    return A2A_ERR_INVALID_ARG;
  hipStream_t st = (hipStream_t)hip_stream;
  const size_t slot = (size_t)(t->next_slot.fetch_add(1) % a2a_topo::kSlots) * a2a_topo::kSlotWords;
  int64_t* d_res = t->d_small + slot;
  const int64_t* h_res = t->h_pinned + slot;
  k_util_extrema<<<1, 1024, 0, st>>>(t->d_out_ptr, load, cap, t->N, (long long*)d_res);
  HIP_TRY(hipGetLastError());
  HIP_TRY(hipMemcpyAsync((void*)h_res, d_res, 6 * sizeof(int64_t), hipMemcpyDeviceToHost, st));
  HIP_TRY(hipStreamSynchronize(st));
  if (h_res[5] != 0) return A2A_ERR_INVALID_ARG;  // a capacity that is not positive and finite
  double umax, umin, total, cmax;
  std::memcpy(&umax, &h_res[0], 8);
  std::memcpy(&umin, &h_res[2], 8);
  std::memcpy(&total, &h_res[3], 8);
  std::memcpy(&cmax, &h_res[4], 8);
  const double m = m_bytes, b = b_bytes_per_s;
  out->max_util = umax;
  out->argmax_arc = h_res[1];
  out->min_util = umin;
  out->sum_dist = sum_dist;
  out->n_links = t->E;
  out->n_nodes = t->N;
  out->total_capacity = total;
  out->max_node_capacity = cmax;
  out->t_sched = umax * m / b;
  out->t_lb_nd = (double)sum_dist * m / ((double)t->N * cmax * b);
  out->t_lb_links = (double)sum_dist * m / (total * b);
  out->ratio = out->t_sched / out->t_lb_nd;
  out->throughput = (double)(t->N - 1) * m / out->t_sched;
  out->flow_value = 1.0 / umax;
  out->throughput_upper = (double)(t->N - 1) * out->flow_value * b;
  return (flags & A2A_FLAG_UNREACHABLE) ? A2A_ERR_DISCONNECTED : A2A_OK;
}

int a2a_tree_lower_bound(int32_t N, int32_t d, double m_bytes, double b_bytes_per_s, a2a_tree_bound* out) {
  if (!out || N < 1 || d < 1 || !(m_bytes > 0.0) || !(b_bytes_per_s > 0.0)) return A2A_ERR_INVALID_ARG;
  int64_t left = (int64_t)N - 1, width = 1, sum = 0;
  int32_t level = 0;
  bool full = true;
  while (left > 0) {
    ++level;
    // d^level hosts fit on this level; stop multiplying once it exceeds what is left
    width = width > left / d ? left + 1 : width * d;
    const int64_t take = width < left ? width : left;
    full = take == width;
    sum += take * level;
    left -= take;
  }
  out->s_min = sum;
  out->height = level;
  out->full = full ? 1 : 0;
  out->t_lb = (double)sum * m_bytes / ((double)d * b_bytes_per_s);
  out->throughput_ub = N > 1 ? (double)(N - 1) * m_bytes / out->t_lb : 0.0;
  return A2A_OK;
}

int a2a_profile_enable(a2a_topo* t, int mode) {
  if (!t || mode < 0 || mode > 2) return A2A_ERR_INVALID_ARG;
  for (auto& rec : t->prof_recs) {
    (void)hipEventDestroy(rec.beg);
    (void)hipEventDestroy(rec.end);
  }
  t->prof_recs.clear();
  t->prof_calls = 0;
  t->prof_depth = 0;
  t->prof_groups = 0;
  t->prof_narrow = 0;
  t->prof_fwd_flavours = t->prof_bwd_flavours = 0;
  t->prof_mode = mode;
  std::memset(t->prof_pairs_level, 0, sizeof(t->prof_pairs_level));
  std::memset(t->prof_dag_level, 0, sizeof(t->prof_dag_level));
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
      const int l = rec.level < A2A_PROF_MAX_LEVELS ? rec.level : A2A_PROF_MAX_LEVELS - 1;
      out->ms_level[rec.cls][l] += ms;
    }
  }
  int64_t dag = 0;
  for (int l = 0; l < A2A_PROF_MAX_LEVELS; ++l) {
    out->pairs_level[l] = t->prof_pairs_level[l];
    out->dag_level[l] = t->prof_dag_level[l];
    dag += t->prof_dag_level[l];
  }
  out->dag_links = dag;
  out->calls = t->prof_calls;
  out->depth = t->prof_depth;
  out->groups = t->prof_groups;
  out->narrow_levels = t->prof_narrow;
  out->fwd_flavours = t->prof_fwd_flavours;
  out->bwd_flavours = t->prof_bwd_flavours;
  return A2A_OK;
}

}  // extern "C"
