// mlproj: bi-level / tri-level / multi-level projection onto the l_{1,q} ball for gfx950 (MI355X).
// Method: Perez & Barlaud, "Multi-level projection with exponential parallel speedup",
// arXiv 2405.02086 -- Sec. 3 (Eq. 5-9, Alg. 1), Sec. 4 (Alg. 2-4), Sec. 5 (Alg. 5-6) and the
// iterative forms in the appendix.  The paper describes CPU code only; the kernels below are
// an independent design for a 256-CU, 64-lane-wavefront, HBM-bound machine.
//
// One bi-level call is a chain of kernels on the caller's stream; nothing returns to the host:
//   colagg    Y -> per-(column tile, row group) partial aggregates        (reads Y once)
//   reduce    partials -> v_j = ||y_j||_q                                  (tiny)
//   search    v -> tau, the l1-ball threshold; run redundantly at the head of colmap (of the
//             seeding kernel for l1,1) when there are at most 16384 groups, a kernel of its
//             own otherwise                                                     (tiny)
//   [init, sweep, filter/update ..., finish]  l1,1 only: per-column inner thresholds, one
//             read of Y per lock-step sweep (typically two), stragglers column by column
//   colmap    Y, v, tau -> X                                  (reads Y again, writes X once)
// Workgroups never wait for one another inside a kernel: on this GPU a device-scope fence
// costs an L2 write-back, so cross-workgroup results travel across kernel boundaries only
// (the one exception, the search over more than 32768 groups, exchanges a few words per round
// through device-scope atomics alone).  The tri-level form uses the same chain with groups that are
// contiguous slabs; the generic multi-level form works on contiguous fibres, level by level;
// a batch of matrices shares the three launches of the chain; a matrix of at most 128 KiB takes
// one kernel in which every workgroup holds all of Y (tiny.h).
//
// This file is the one translation unit: the kernels live in the headers it includes (one per
// pass), the host code below checks arguments, plans the launch geometry and enqueues.
#include <atomic>
#include <mutex>
#include <tuple>
#include <utility>

#include "common.h"
#include "reduce.h"
#include "aggregate.h"
#include "search.h"
#include "map.h"
#include "l11.h"
#include "l11grid.h"
#include "l11held.h"
#include "slab.h"
#include "fibre.h"
#include "tiny.h"
#include "held.h"
#include "batch.h"

namespace mlproj {

// ------------------------------------------------------------------ host: checks + launches
constexpr long long MAX_ELEMS = 1LL << 40;       // 4 TiB of fp32: far beyond one GPU
constexpr long long MAX_GROUPS = (1LL << 31) - 1;
constexpr long long MAX_GRID = (1LL << 31) - 1;
constexpr int STAGE_AGGREGATE = 1, STAGE_APPLY = 2, STAGE_ALL = 3;

static int check_dims(long long a, long long b, long long c) {
  if (a <= 0 || b <= 0 || c <= 0) return MLPROJ_ERR_BAD_DIMENSION;
  if (a > MAX_ELEMS || b > MAX_ELEMS || c > MAX_ELEMS) return MLPROJ_ERR_TOO_LARGE;
  if (a > MAX_ELEMS / b || a * b > MAX_ELEMS / c) return MLPROJ_ERR_TOO_LARGE;
  return MLPROJ_OK;
}

static bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

// Elements per lane and access: 16 bytes when the rows allow it, one element otherwise.
static int pick_vec(const void* Y, long long row_len, int elem_bytes = 4) {
  const int wide = 16 / elem_bytes;
  return (row_len % wide == 0 && aligned(Y, 16)) ? wide : 1;
}

static int workspace_bytes_impl(int variant, long long d0, long long d1, long long d2,
                                size_t* out) {
  if (!out) return MLPROJ_ERR_NULL_POINTER;
  if (variant < MLPROJ_L1INF || variant > MLPROJ_L1INFINF) return MLPROJ_ERR_BAD_VARIANT;
  if (variant != MLPROJ_L1INFINF && d2 != 1) return MLPROJ_ERR_BAD_DIMENSION;
  const int st = check_dims(d0, d1, d2);
  if (st != MLPROJ_OK) return st;
  size_t best = 0;
  for (int vec : {8, 4, 1}) {   // bi-level: 4 (fp32) or 8 (16-bit storage) columns per lane
    Geometry g;
    long long ngroups;
    if (variant != MLPROJ_L1INFINF && vec == 1) continue;
    if (variant == MLPROJ_L1INFINF) {
      if (d0 > MAX_GROUPS) return MLPROJ_ERR_TOO_LARGE;
      g = plan_slabs(d0, d1 * d2, vec);
      ngroups = d0;
    } else {
      if (d1 > MAX_GROUPS) return MLPROJ_ERR_TOO_LARGE;
      g = plan_columns(d0, d1, vec, variant);
      ngroups = d1;
    }
    if (g.tiles * g.groups > MAX_GRID) return MLPROJ_ERR_TOO_LARGE;
    const Layout L = layout_for(g, ngroups, variant);
    if (L.bytes > best) best = L.bytes;
  }
  *out = best;
  return MLPROJ_OK;
}

static int check_radius(float eta) {
  if (!(eta >= 0.0f) || std::isinf(eta)) return MLPROJ_ERR_BAD_RADIUS;
  return MLPROJ_OK;
}

// Every kernel goes out through hipLaunchKernel, whose return value is the status of that launch
// alone: the process-wide "last error" of the HIP runtime, which an unrelated earlier call of the
// application may have set, is neither read nor cleared.  A refused launch is remembered for the
// calling thread until the entry point returns (launch_status), which also stops what the call
// had still to enqueue from going out behind it.
static thread_local bool g_launch_refused = false;

template <typename... KArgs, typename... Args>
static inline void launch(void (*kernel)(KArgs...), dim3 grid, dim3 block, hipStream_t stream, Args&&... args) {
  static_assert(sizeof...(KArgs) == sizeof...(Args), "one argument per kernel parameter");
  if (g_launch_refused) return;
  std::tuple<std::decay_t<KArgs>...> held(static_cast<std::decay_t<KArgs>>(args)...);
  const hipError_t e = std::apply(
      [&](auto&... a) {
        void* ptrs[] = {static_cast<void*>(&a)...};
        return hipLaunchKernel(reinterpret_cast<const void*>(kernel), grid, block, ptrs, 0, stream);
      },
      held);
  if (e != hipSuccess) g_launch_refused = true;
}

static int launch_status() {
  const bool refused = g_launch_refused;
  g_launch_refused = false;
  return refused ? MLPROJ_ERR_LAUNCH : MLPROJ_OK;
}

// Compute units of the current device (0 when there is none to ask).  A device's count never
// changes, so it is asked for once per device and remembered.
static int compute_units() {
  constexpr int MAX_DEVICES = 64;
  static std::atomic<int> known[MAX_DEVICES];   // 0: not asked yet
  int dev = -1, cus = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0) return 0;
  if (dev < MAX_DEVICES && (cus = known[dev].load(std::memory_order_relaxed)) > 0) return cus;
  if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0) return 0;
  if (dev < MAX_DEVICES) known[dev].store(cus, std::memory_order_relaxed);
  return cus;
}

// Optional per-kernel timing: while a trace is open on the calling thread, an event is
// recorded on the stream before every kernel of a call and after its last one.
struct Trace {
  hipEvent_t* events = nullptr;
  int capacity = 0;
  int count = 0;
};
static thread_local Trace g_trace;

static inline void mark(hipStream_t stream) {
  if (g_trace.events && g_trace.count < g_trace.capacity)
    (void)hipEventRecord(g_trace.events[g_trace.count++], stream);
}

// Polls a lane of the grid-wide search may spend waiting for another workgroup's post before the
// search gives up and the one-workgroup kernel behind it takes over (0: give up at once).
// (a test hook, see mlproj_set_search_spin_limit; atomic, so a thread that enqueues while another
// sets it reads one value or the other)
static std::atomic<unsigned> g_spin_limit{SPIN_LIMIT};

// The stand-alone search: up to 16384 groups one workgroup running the search of the map
// kernels' prologue (so a split call returns the whole call's bits), one workgroup of 1024
// threads with 32 values each up to 32768, the several-workgroup form beyond that, followed by
// a one-workgroup kernel as a fallback that returns at once unless that form gave up.
// tile_stats / nstats: what the aggregate pass left for the grid-wide form (see search_wide_kernel), if anything.
static void launch_search(const Ws& ws, long long ngroups, double eta, int mode, int outer,
                          double* norm_out, hipStream_t stream, const double* tile_stats = nullptr,
                          long long nstats = 0) {
  if (ngroups <= FUSED_SEARCH_MAX) {
    launch((search_kernel<WG, SEARCH_CACHE>), dim3(1), dim3(WG), stream, ws, ngroups, eta, mode, outer,
                       norm_out, 0, (double*)nullptr, (float*)nullptr);
    return;
  }
  if (ngroups <= FUSED_SEARCH_MAX_BIG) {
    launch((search_kernel<WG, SEARCH_CACHE_BIG>), dim3(1), dim3(WG), stream, ws, ngroups, eta, mode, outer,
                       norm_out, 0, (double*)nullptr, (float*)nullptr);
    return;
  }
  int only_as_fallback = 0;
  // (the l2 and l_inf outer projections need no iteration: one workgroup reads v once)
  const bool iterates = outer == MLPROJ_OUTER_L1 || mode == MODE_NORM;
  if (ngroups <= (long long)SWG * SEARCH_CACHE_ONE_WG && iterates) {
    launch((search_kernel<SWG, SEARCH_CACHE_ONE_WG>), dim3(1), dim3(SWG), stream, ws, ngroups, eta, mode,
                       outer, norm_out, 0, (double*)nullptr, (float*)nullptr);
    return;
  }
  if (iterates) {
    long long nwg = cdiv(ngroups, (long long)COOP_THREADS * COOP_VALUES);
    if (nwg > COOP_MAX_WGS) nwg = COOP_MAX_WGS;
    launch((search_wide_kernel<false, COOP_THREADS, COOP_VALUES>), dim3((unsigned)nwg), dim3(COOP_THREADS), stream, ws, ngroups, eta, mode, norm_out, g_spin_limit.load(std::memory_order_relaxed), tile_stats, nstats);
    only_as_fallback = 1;
  }
  launch((search_kernel<SWG, SEARCH_CACHE>), dim3(1), dim3(SWG), stream, ws, ngroups, eta, mode, outer, norm_out,
                     only_as_fallback, (double*)nullptr, (float*)nullptr);
}

// The search for a weighted l1 ball as outer norm (ws.wts set).  One workgroup re-reads what its
// registers do not hold in every round: beyond 32768 groups the grid-wide form goes first, with
// the one-workgroup kernel as its fallback.
static void launch_weighted_search(const Ws& ws, long long m, double eta, hipStream_t stream,
                                   double* radii = nullptr, float* u_out = nullptr) {
  int only_as_fallback = 0;
  if (m > 32768) {
    long long nwg = cdiv(m, (long long)COOP_THREADS * COOP_VALUES);
    if (nwg > COOP_MAX_WGS) nwg = COOP_MAX_WGS;
    launch((search_wide_kernel<true, COOP_THREADS, COOP_VALUES>), dim3((unsigned)nwg), dim3(COOP_THREADS), stream, ws, m,
                       eta, (int)MODE_PROJECT, (double*)nullptr, g_spin_limit.load(std::memory_order_relaxed), (const double*)nullptr, 0LL);
    only_as_fallback = 1;
  }
  if (m <= 4096)
    launch((search_weighted_kernel<256, 16>), dim3(1), dim3(256), stream, ws, m, eta, only_as_fallback, radii, u_out);
  else if (m <= 16384)
    launch((search_weighted_kernel<256, 64>), dim3(1), dim3(256), stream, ws, m, eta, only_as_fallback, radii, u_out);
  else
    launch((search_weighted_kernel<SWG, 16>), dim3(1), dim3(SWG), stream, ws, m, eta, only_as_fallback, radii, u_out);
}

// l1,1: how many lock-step sweeps to enqueue before the finishing pass, and the number of
// open columns at which the remaining sweeps hand over to it (see l11.h).  Measured on an
// MI355X: a sweep that finds nothing to do costs two launches (3.6 us); one iteration of the
// finishing pass costs about n/512 us for up to 512 groups of 16 columns, and it needs about
// four from the bounds the sweeps leave; two sweeps close every column on Gaussian data,
// heavy tails take up to ten.  So short matrices get few sweeps (finishing is cheap; up to
// 1024 rows it holds the columns in registers and needs no sweep at all), tall ones more, and where a sweep is dearer than finishing a few hundred stragglers the sweeps
// stop as soon as no more than that are open.
static std::atomic<int> g_l11_sweeps{0};  // 0 = automatic (a tuning and test hook, see mlproj_set_l11_sweeps)
static void plan_l11(long long n, long long m, int elem_bytes, int* sweeps, unsigned* handoff) {
  const double sweep_us = (double)n * (double)m * elem_bytes / 4e6 + 6.0;
  const double finish_us = 4.0 * (double)n / 512.0;
  *handoff = sweep_us > finish_us ? 512u : 0u;
  const int forced = g_l11_sweeps.load(std::memory_order_relaxed);
  if (forced > 0) { *sweeps = forced; return; }
  // (up to 4096 rows and 4M elements the finishing pass alone is also faster than the six or more
  // launches of the sweeps: 42 against 54 us at 2048 x 2048, 50 against 58 at 4096 x 1024; at
  // 1536 x 4096 the two are level, beyond that the sweeps win: 92 against 121 us at 4096 x 4096)
  if (n <= 4096 && n * m <= (4ll << 20)) { *sweeps = 0; return; }
  *sweeps = n <= 1024 ? 0 : n <= 2048 ? 2 : n <= 4096 ? 3 : n <= 8192 ? 4 : n <= 32768 ? 6
          : n <= 131072 ? 8 : 12;
}

// l1,1 in fp32 on 4097 to 8192 rows: the columns-in-registers kernel on stripes of 8 columns, as
// long as every stripe has a CU to itself.  (Measured against the lock-step sweeps, Gaussian /
// Cauchy entries: 8192 x 512 53 / 53 against 73 / 129 us, 8192 x 2048 116 / 119 against 101 / 201;
// with more stripes than CUs the 32-byte runs lose: 8192 x 4096 300 against 144.)
static bool l11_narrow_stripes_fit(long long n, long long m) {
  return lh_narrow_fits(n) && cdiv(m, LH_COLS_NARROW) <= compute_units();
}

// STAGE_AGGREGATE = aggregate + threshold search (+ inner searches for l1,1);
// STAGE_APPLY = the per-column map.
template <int Q, typename T = float>
static int run_bilevel(const T* Y, T* X, long long n, long long m, float eta,
                       void* workspace, size_t workspace_bytes, float* v_out, float* u_out,
                       void* stream_, int mode, double* norm_out, int stages, int outer,
                       unsigned char* mask_out = nullptr, bool check_only = false,
                       const float* weights = nullptr) {
  constexpr int WIDE = 16 / (int)sizeof(T);
  if (outer < MLPROJ_OUTER_L1 || outer > MLPROJ_OUTER_LINF) return MLPROJ_ERR_BAD_VARIANT;
  if (weights && (outer != MLPROJ_OUTER_L1 || mode != MODE_PROJECT || stages != STAGE_ALL)) return MLPROJ_ERR_BAD_VARIANT;
  const bool need_x = mode == MODE_PROJECT && (stages & STAGE_APPLY);
  if (!Y || !workspace || (need_x && !X)) return MLPROJ_ERR_NULL_POINTER;
  int st = check_dims(n, m, 1);
  if (st != MLPROJ_OK) return st;
  if (m > MAX_GROUPS) return MLPROJ_ERR_TOO_LARGE;
  if (mode == MODE_PROJECT && (stages & STAGE_AGGREGATE) && (st = check_radius(eta)) != MLPROJ_OK)
    return st;
  if (!aligned(Y, sizeof(T)) || (X && !aligned(X, sizeof(T)))) return MLPROJ_ERR_ALIGNMENT;
  if (!aligned(workspace, 256)) return MLPROJ_ERR_WORKSPACE;
  // Every lane owns WIDE columns; rows that are not 16-byte aligned are read element-wise
  // (the strided form of LaneCols), and a misaligned X alone only narrows the stores.  The
  // geometry depends on n and m only, so the two stages of a split call agree on it.
  const bool wide = pick_vec(Y, m, (int)sizeof(T)) == WIDE;
  const bool x_vec = !X || aligned(X, 16);
  const Geometry g = plan_columns(n, m, WIDE, Q);
  if (g.tiles * g.groups > MAX_GRID) return MLPROJ_ERR_TOO_LARGE;
  const Layout L = layout_for(g, m, Q);
  if (workspace_bytes < L.bytes) return MLPROJ_ERR_WORKSPACE;
  if (check_only) return MLPROJ_OK;
  Ws ws = bind(workspace, L);
  ws.wts = weights;
  hipStream_t stream = static_cast<hipStream_t>(stream_);
  const dim3 grid_dim((unsigned)(g.tiles * g.groups)), block(WG);
  const dim3 mgrid((unsigned)(g.tiles * g.map_groups));
  const int rthreads = fold_threads(g.groups);
  const int parts = reduce_parts(g.groups, rthreads);
  const dim3 rgrid((unsigned)cdiv(m, rthreads / parts)), rblock(rthreads);
  // A whole call on few enough groups lets every map workgroup find tau by itself, which
  // takes the one-workgroup search kernel off the critical path (16 values of v per thread
  // up to 4096 groups, 64 per thread up to 16384).
  // (A weighted outer ball has its own search kernel: nothing is fused and no one-kernel form.)
  const bool fuse = mode == MODE_PROJECT && stages == STAGE_ALL && Q != Q1 && m <= FUSED_SEARCH_MAX_BIG && !weights;
  const bool fuse_big = fuse && m > FUSED_SEARCH_MAX;
  const double fused_eta = fuse ? (double)eta : -1.0;

  if constexpr (tiny_built<Q, T>()) {
    // a matrix of at most 128 KiB: one kernel does it all (up to 16 workgroups when X lies apart
    // from Y, a single one when they overlap)
    TinyPlan tp;
    const bool apart = X && (X + n * m <= Y || Y + n * m <= X);
    if (mode == MODE_PROJECT && stages == STAGE_ALL && wide && x_vec && !weights && tiny_plan(n, m, WIDE, &tp)) {
      mark(stream);
      launch((tiny_kernel<Q, T, WIDE>), dim3(apart ? (unsigned)tp.slots : 1u), dim3(TINY_WG), stream, Y, X, n, m,
                         (double)eta, outer, tp.cw, ws, v_out, u_out, mask_out, apart ? 0 : 1);
      mark(stream);
      return launch_status();
    }
  }
  // l1,1 on at most 4096 rows (16-byte aligned rows, the whole call at once): after the aggregate
  // pass one kernel holds 16 whole columns per workgroup in registers, runs the inner searches
  // there, and maps and stores from the same registers (l11held.h)
  int held_values = 0;
  int held_cols = LH_COLS;
  if constexpr (Q == Q1) {
    // (measured: ahead of the lock-step sweeps up to 64M elements, 57 against 97 us at 4096 x 4096,
    // 108 against 146 at 4096 x 8192, 219 against 227 at 4096 x 16384, and far ahead where most
    // columns are dropped, whose stripes are not even read; behind at 128M.  A forced sweep count,
    // the test hook, keeps the sweeps.)
    if (mode == MODE_PROJECT && stages == STAGE_ALL && wide && x_vec &&
        n * m <= lh_max_elems<T>() && g_l11_sweeps.load(std::memory_order_relaxed) == 0)
      held_values = lh_values_for<T>(n);
    // (fp32 up to 8192 rows: stripes of 8 columns)
    if constexpr (sizeof(T) == 4) {
      if (held_values == 0 && mode == MODE_PROJECT && stages == STAGE_ALL && wide && x_vec && n * m <= lh_max_elems<T>() &&
          g_l11_sweeps.load(std::memory_order_relaxed) == 0 && l11_narrow_stripes_fit(n, m)) {
        held_values = 128;
        held_cols = LH_COLS_NARROW;
      }
    }
  }
  // l1,1 with lock-step sweeps planned: the aggregate pass also evaluates the columns on a grid
  // of thresholds, which stands in for the probing sweep (l11grid.h)
  bool grid = false;
  if constexpr (Q == Q1 && sizeof(T) == 4) {
    int sweeps;
    unsigned handoff;
    plan_l11(n, m, (int)sizeof(T), &sweeps, &handoff);
    // (worth it from 128 MiB on, where the probing pass costs more than the scale kernel, the grid
    // arithmetic and the longer seeding; not on 16-bit storage, where the aggregate pass has twice
    // the elements per byte and the grid arithmetic would double its time)
    grid = mode == MODE_PROJECT && sweeps >= 1 && n * m >= (32LL << 20) && held_values == 0;
  }
  if (stages & STAGE_AGGREGATE) {
    mark(stream);
    if constexpr (Q == Q1 && sizeof(T) == 4) {
      if (grid) {
        launch((l11_scale_kernel<T>), dim3((unsigned)cdiv(m, WG)), block, stream, Y, n, m, ws.scale);
        if (wide)
          launch((colagg_grid_kernel<T, WIDE, false>), grid_dim, block, stream, Y, n, m, g, ws, (const float*)ws.scale, ws.gpart);
        else
          launch((colagg_grid_kernel<T, WIDE, true>), grid_dim, block, stream, Y, n, m, g, ws, (const float*)ws.scale, ws.gpart);
      }
    }
    if (grid) {
      mark(stream);
      if (rthreads == 256)
        launch((reduce_kernel<Q, 256>), rgrid, rblock, stream, ws.partial, m, g, parts, ws.v, v_out, ws.flags);
      else
        launch((reduce_kernel<Q>), rgrid, rblock, stream, ws.partial, m, g, parts, ws.v, v_out, ws.flags);
    } else if (g.groups == 1) {
      // one row group per tile: the aggregate pass writes v itself, there is nothing to fold
      if (wide)
        launch((colagg_direct_kernel<Q, T, WIDE, false>), grid_dim, block, stream, Y, n, m, g, ws.partial, ws.v, v_out, ws.flags);
      else
        launch((colagg_direct_kernel<Q, T, WIDE, true>), grid_dim, block, stream, Y, n, m, g, ws.partial, ws.v, v_out, ws.flags);
      mark(stream);   // (the same number of intervals as the longer chain: the fold's is empty)
    } else {
      if (wide)
        launch((colagg_kernel<Q, T, WIDE, false>), grid_dim, block, stream, Y, n, m, g, ws.partial);
      else
        launch((colagg_kernel<Q, T, WIDE, true>), grid_dim, block, stream, Y, n, m, g, ws.partial);
      mark(stream);
      if (rthreads == 256)
        launch((reduce_kernel<Q, 256>), rgrid, rblock, stream, ws.partial, m, g, parts, ws.v, v_out, ws.flags);
      else
        launch((reduce_kernel<Q>), rgrid, rblock, stream, ws.partial, m, g, parts, ws.v, v_out, ws.flags);
    }
    if constexpr (Q == Q1) {
      if (held_values > 0) {
        const dim3 hgrid((unsigned)cdiv(m, held_cols)), hblock(LH_WG);
        // (a weighted outer ball has a search kernel of its own; the kernel reads its record)
        const bool seeded = !weights && m <= (long long)LH_WG * LH_SEARCH_CACHE;
        mark(stream);
        if (weights) launch_weighted_search(ws, m, (double)eta, stream);
        else if (!seeded) launch_search(ws, m, (double)eta, mode, outer, norm_out, stream);
        mark(stream);   // (the same number of intervals as the longer chain: the sweeps' is empty)
        mark(stream);
        const double seed_eta = seeded ? (double)eta : -1.0;
        // (64 values per thread: two workgroups per CU when there are more stripes than CUs)
        const bool packed = held_values == 64 && cdiv(m, LH_COLS) > compute_units();
        bool narrow_done = false;
        if constexpr (sizeof(T) == 4) {
          if (held_cols == LH_COLS_NARROW) {
            if (seeded) launch((l11_held_kernel<T, 128, LH_SEARCH_CACHE, false, LH_COLS_NARROW>), hgrid, hblock, stream, Y, X, n, m, ws, u_out, mask_out, seed_eta, outer);
            else launch((l11_held_kernel<T, 128, 0, false, LH_COLS_NARROW>), hgrid, hblock, stream, Y, X, n, m, ws, u_out, mask_out, seed_eta, outer);
            narrow_done = true;
          }
        }
        if (narrow_done) {
        } else if (seeded) {
          if (held_values == 32) launch((l11_held_kernel<T, 32, LH_SEARCH_CACHE>), hgrid, hblock, stream, Y, X, n, m, ws, u_out, mask_out, seed_eta, outer);
          else if (packed) launch((l11_held_kernel<T, 64, LH_SEARCH_CACHE, true>), hgrid, hblock, stream, Y, X, n, m, ws, u_out, mask_out, seed_eta, outer);
          else if (held_values == 64) launch((l11_held_kernel<T, 64, LH_SEARCH_CACHE>), hgrid, hblock, stream, Y, X, n, m, ws, u_out, mask_out, seed_eta, outer);
          else launch((l11_held_kernel<T, 128, LH_SEARCH_CACHE>), hgrid, hblock, stream, Y, X, n, m, ws, u_out, mask_out, seed_eta, outer);
        } else {
          if (held_values == 32) launch((l11_held_kernel<T, 32, 0>), hgrid, hblock, stream, Y, X, n, m, ws, u_out, mask_out, seed_eta, outer);
          else if (packed) launch((l11_held_kernel<T, 64, 0, true>), hgrid, hblock, stream, Y, X, n, m, ws, u_out, mask_out, seed_eta, outer);
          else if (held_values == 64) launch((l11_held_kernel<T, 64, 0>), hgrid, hblock, stream, Y, X, n, m, ws, u_out, mask_out, seed_eta, outer);
          else launch((l11_held_kernel<T, 128, 0>), hgrid, hblock, stream, Y, X, n, m, ws, u_out, mask_out, seed_eta, outer);
        }
        mark(stream);
        return launch_status();
      }
    }
    // (l1,1: the kernel that seeds the inner searches runs the outer search the same way)
    const bool fuse_l11 = Q == Q1 && mode == MODE_PROJECT && m <= FUSED_SEARCH_MAX_BIG && !weights;
    if (weights) {
      mark(stream);
      launch_weighted_search(ws, m, (double)eta, stream);
    } else if (!fuse && !fuse_l11) {
      mark(stream);
      if (g.groups == 1 && !grid)   // (the direct aggregate pass ran and left its per-tile triples)
        launch_search(ws, m, (double)eta, mode, outer, norm_out, stream, static_cast<const double*>(ws.partial), g.tiles);
      else
        launch_search(ws, m, (double)eta, mode, outer, norm_out, stream);
    }
    if (mode == MODE_NORM) { mark(stream); return launch_status(); }
    if constexpr (Q == Q1) {
      int sweeps;
      unsigned handoff;
      plan_l11(n, m, (int)sizeof(T), &sweeps, &handoff);
      const dim3 fgrid((unsigned)cdiv(m, FIN_COLS)), fblock(FIN_WG);
      mark(stream);
      if (sweeps == 0 && fuse_l11 && finish_held(n) && m <= FUSED_SEARCH_MAX) {
        // a short matrix of few columns: the finishing pass seeds itself and runs the outer
        // search too (with more columns the search repeated in every workgroup costs more than
        // the seeding kernel it saves: 61 against 56 us at 1000 x 10000)
        launch((l11_finish_seeded_kernel<T, FIN_SEARCH_CACHE>), fgrid, fblock, stream, Y, n, m, ws, (double)eta, outer);
        mark(stream);   // (the same number of intervals as the longer chain: this one is empty)
      } else {
        const dim3 igrid((unsigned)cdiv(m, WG));
        if (grid) {
          const float* sc = ws.scale;
          const float* gp = ws.gpart;
          if (!fuse_l11)
            launch((l11_init_grid_kernel<SEARCH_CACHE>), igrid, block, stream, n, m, g, ws, -1.0, outer, sc, gp);
          else if (m > FUSED_SEARCH_MAX)
            launch((l11_init_grid_kernel<SEARCH_CACHE_BIG>), igrid, block, stream, n, m, g, ws, (double)eta, outer, sc, gp);
          else
            launch((l11_init_grid_kernel<SEARCH_CACHE>), igrid, block, stream, n, m, g, ws, (double)eta, outer, sc, gp);
        } else if (!fuse_l11)
          launch((l11_init_kernel<SEARCH_CACHE>), igrid, block, stream, n, m, ws, -1.0, outer);
        else if (m > FUSED_SEARCH_MAX)
          launch((l11_init_kernel<SEARCH_CACHE_BIG>), igrid, block, stream, n, m, ws, (double)eta, outer);
        else
          launch((l11_init_kernel<SEARCH_CACHE>), igrid, block, stream, n, m, ws, (double)eta, outer);
        if (fuse_l11) mark(stream);   // (keeps one interval for search + seeding, one for the sweeps)
        // (with the grid the seeding kernel has already done what sweep 0 and its update do)
        for (int s = grid ? 1 : 0; s < sweeps; ++s) {
          if (s == 0) {
            if (wide) launch((l11_sweep_kernel<T, WIDE, false>), grid_dim, block, stream, Y, n, m, g, ws);
            else launch((l11_sweep_kernel<T, WIDE, true>), grid_dim, block, stream, Y, n, m, g, ws);
          } else {
            if (wide) launch((l11_filter_kernel<T, WIDE, false>), grid_dim, block, stream, Y, n, m, g, ws, s, handoff);
            else launch((l11_filter_kernel<T, WIDE, true>), grid_dim, block, stream, Y, n, m, g, ws, s, handoff);
          }
          launch(l11_update_kernel, dim3((unsigned)cdiv(m, UPD_COLS)), block, stream, n, m, g, ws, s, handoff);
        }
        if (finish_held(n))
          launch((l11_finish_kernel<T, true>), fgrid, fblock, stream, Y, n, m, ws, sweeps, handoff);
        else
          launch((l11_finish_kernel<T, false>), fgrid, fblock, stream, Y, n, m, ws, sweeps, handoff);
      }
    }
  }
  if (stages & STAGE_APPLY) {
    mark(stream);
    if (fuse_big && wide && x_vec)
      launch((colmap_kernel<Q, T, WIDE, false, true, SEARCH_CACHE_BIG>), mgrid, block, stream, Y, X, n, m, g, ws, u_out, mask_out, fused_eta, outer);
    else if (fuse_big && wide)
      launch((colmap_kernel<Q, T, WIDE, false, false, SEARCH_CACHE_BIG>), mgrid, block, stream, Y, X, n, m, g, ws, u_out, mask_out, fused_eta, outer);
    else if (fuse_big)
      launch((colmap_kernel<Q, T, WIDE, true, false, SEARCH_CACHE_BIG>), mgrid, block, stream, Y, X, n, m, g, ws, u_out, mask_out, fused_eta, outer);
    else if (wide && x_vec)
      launch((colmap_kernel<Q, T, WIDE, false, true>), mgrid, block, stream, Y, X, n, m, g, ws, u_out, mask_out, fused_eta, outer);
    else if (wide)
      launch((colmap_kernel<Q, T, WIDE, false, false>), mgrid, block, stream, Y, X, n, m, g, ws, u_out, mask_out, fused_eta, outer);
    else
      launch((colmap_kernel<Q, T, WIDE, true, false>), mgrid, block, stream, Y, X, n, m, g, ws, u_out, mask_out, fused_eta, outer);
  }
  mark(stream);
  return launch_status();
}

template <typename... A>
static int dispatch_q(int variant, A... a) {
  switch (variant) {
    case MLPROJ_L1INF: return run_bilevel<QINF>(a...);
    case MLPROJ_L11: return run_bilevel<Q1>(a...);
    case MLPROJ_L12: return run_bilevel<Q2>(a...);
    default: return MLPROJ_ERR_BAD_VARIANT;
  }
}

template <typename T>
static int dispatch_stored(int outer, int variant, const void* Y, void* X, long long n, long long m,
                           float eta, void* workspace, size_t workspace_bytes, float* v_out,
                           float* u_out, unsigned char* mask_out, void* stream) {
  return dispatch_q(variant, static_cast<const T*>(Y), static_cast<T*>(X), n, m, eta, workspace,
                    workspace_bytes, v_out, u_out, stream, MODE_PROJECT, (double*)nullptr, STAGE_ALL,
                    outer, mask_out);
}

// ------------------------------------------------------------------ host: tri-level
template <typename T>
static int run_trilevel(const T* Y, T* X, long long d0, long long d1, long long d2, float eta,
                        void* workspace, size_t workspace_bytes, float* v_out, float* u_out,
                        unsigned char* mask_out, void* stream_) {
  constexpr int WIDE = 16 / (int)sizeof(T);
  if (!Y || !X || !workspace) return MLPROJ_ERR_NULL_POINTER;
  int st = check_dims(d0, d1, d2);
  if (st != MLPROJ_OK) return st;
  if (d0 > MAX_GROUPS) return MLPROJ_ERR_TOO_LARGE;
  if ((st = check_radius(eta)) != MLPROJ_OK) return st;
  if (!aligned(Y, sizeof(T)) || !aligned(X, sizeof(T))) return MLPROJ_ERR_ALIGNMENT;
  if (!aligned(workspace, 256)) return MLPROJ_ERR_WORKSPACE;
  const long long len = d1 * d2;
  const int vec = pick_vec(Y, len, (int)sizeof(T));
  const bool x_vec = aligned(X, 16);
  const Geometry g = plan_slabs(d0, len, vec);
  if (g.tiles * g.groups > MAX_GRID) return MLPROJ_ERR_TOO_LARGE;
  const Layout L = layout_for(g, d0, MLPROJ_L1INFINF);
  if (workspace_bytes < L.bytes) return MLPROJ_ERR_WORKSPACE;
  const Ws ws = bind(workspace, L);
  hipStream_t stream = static_cast<hipStream_t>(stream_);
  // A tensor that the register files hold (at most 256 slabs and 256 KiB per CU, 16-byte aligned
  // slabs): one pass over memory, see held.h.  It is ahead of the chain at every size (10 against
  // 12 us at 1 MiB, 34 against 49 us at 64 MiB).  The plan needs the number of CUs.
  if (vec == WIDE) {
    HeldPlan hp;
    if (held_plan_slabs(d0, len, (int)sizeof(T), compute_units(), &hp)) {
      const unsigned limit = g_spin_limit.load(std::memory_order_relaxed);
      const unsigned patience = limit < HELD_PATIENCE ? limit : HELD_PATIENCE;
      mark(stream);
      launch(held_clear_kernel, dim3(1), dim3(WG), stream, ws.posts);
      mark(stream);
      if (x_vec)
        launch((held_slab_kernel<T, true>), dim3((unsigned)hp.nwg), dim3(HELD_WG), stream, Y, X, d0, len, hp, (double)eta, ws, ws.posts, v_out, u_out, mask_out, patience);
      else
        launch((held_slab_kernel<T, false>), dim3((unsigned)hp.nwg), dim3(HELD_WG), stream, Y, X, d0, len, hp, (double)eta, ws, ws.posts, v_out, u_out, mask_out, patience);
      mark(stream);
      return launch_status();
    }
  }
  const dim3 grid((unsigned)(g.tiles * g.groups)), block(WG);
  const int parts = reduce_parts(g.groups);
  const dim3 rgrid((unsigned)cdiv(d0, SWG / parts)), rblock(SWG);
  float* partial = static_cast<float*>(ws.partial);
  mark(stream);
  if (vec == WIDE) launch((slabagg_kernel<T, WIDE>), grid, block, stream, Y, len, g, partial);
  else launch((slabagg_kernel<T, 1>), grid, block, stream, Y, len, g, partial);
  mark(stream);
  launch((reduce_kernel<QINF>), rgrid, rblock, stream, ws.partial, d0, g, parts, ws.v, v_out, ws.flags);
  const bool fuse = d0 <= FUSED_SEARCH_MAX;
  const double fused_eta = fuse ? (double)eta : -1.0;
  if (!fuse) {
    mark(stream);
    launch_search(ws, d0, (double)eta, MODE_PROJECT, MLPROJ_OUTER_L1, nullptr, stream);
  }
  mark(stream);
  if (vec == WIDE && x_vec)
    launch((slabmap_kernel<T, WIDE, true>), grid, block, stream, Y, X, d0, len, g, ws, u_out, mask_out, fused_eta);
  else if (vec == WIDE)
    launch((slabmap_kernel<T, WIDE, false>), grid, block, stream, Y, X, d0, len, g, ws, u_out, mask_out, fused_eta);
  else
    launch((slabmap_kernel<T, 1, false>), grid, block, stream, Y, X, d0, len, g, ws, u_out, mask_out, fused_eta);
  mark(stream);
  return launch_status();
}


// ------------------------------------------------------------------ host: batches
// Every problem is checked first (nothing is enqueued if one fails).  Problems of at most
// 16384 columns (a workgroup can search tau itself) go through the batch kernels, BATCH_MAX
// at a time; wider ones are enqueued one by one behind them.
template <int Q, typename T>
static int run_batch(int outer, int count, const mlproj_problem* pr, void* stream_) {
  constexpr int WIDE = 16 / (int)sizeof(T);
  for (int i = 0; i < count; ++i) {
    const int st = run_bilevel<Q, T>(static_cast<const T*>(pr[i].Y), static_cast<T*>(pr[i].X), pr[i].n, pr[i].m,
                                     pr[i].eta, pr[i].workspace, pr[i].workspace_bytes, pr[i].v_out,
                                     pr[i].u_out, stream_, MODE_PROJECT, nullptr, STAGE_ALL, outer,
                                     pr[i].mask_out, true);
    if (st != MLPROJ_OK) return st;
  }
  hipStream_t stream = static_cast<hipStream_t>(stream_);
  // matrices of at most 128 KiB: one kernel for all
  auto apart = [&](int i) {
    const mlproj_problem& p = pr[i];
    const T* Yp = static_cast<const T*>(p.Y);
    const T* Xp = static_cast<const T*>(p.X);
    return Xp + p.n * p.m <= Yp || Yp + p.n * p.m <= Xp;
  };
  auto tinyable = [&](int i) {
    if (!tiny_built<Q, T>()) return false;
    const mlproj_problem& p = pr[i];
    TinyPlan tp;
    return pick_vec(p.Y, p.m, (int)sizeof(T)) == WIDE && aligned(p.X, 16) && tiny_plan(p.n, p.m, WIDE, &tp);
  };
  // l1,1 problems that a single call sends through the columns-in-registers kernel (see
  // run_bilevel) take the same kernel here, so that a batch gives the bits of its single calls:
  // the values per thread such a problem needs, 0 for the others.  Those of them with more than
  // 4096 columns need a search kernel of their own ahead and are enqueued one by one.
  auto held_values = [&](int i) {
    if constexpr (Q != Q1) return 0;
    const mlproj_problem& p = pr[i];
    if (pick_vec(p.Y, p.m, (int)sizeof(T)) != WIDE || !aligned(p.X, 16) || p.n * p.m > lh_max_elems<T>() ||
        g_l11_sweeps.load(std::memory_order_relaxed) != 0)
      return 0;
    const int wide_stripes = lh_values_for<T>(p.n);
    if (wide_stripes == 0 && sizeof(T) == 4 && l11_narrow_stripes_fit(p.n, p.m)) return -1;   // the narrow stripes: single calls only
    return wide_stripes;
  };
  auto held_batchable = [&](int i) { return held_values(i) > 0 && pr[i].m <= (long long)LH_WG * LH_SEARCH_CACHE; };
  auto batchable = [&](int i) { return pr[i].m <= FUSED_SEARCH_MAX_BIG && !tinyable(i) && held_values(i) == 0; };
  if constexpr (tiny_built<Q, T>()) {
    int k = 0;
    while (k < count) {
      BatchItems it;
      BatchGrid tg;
      it.count = 0;
      unsigned wgs = 0;
      for (; k < count && it.count < BATCH_MAX; ++k) {
        if (!tinyable(k)) continue;
        const mlproj_problem& p = pr[k];
        BatchItem& b = it.item[it.count];
        b.Y = p.Y; b.X = p.X; b.ws = p.workspace;
        b.v_out = p.v_out; b.u_out = p.u_out; b.mask_out = p.mask_out;
        b.n = p.n; b.m = p.m; b.eta = (double)p.eta;
        b.wide = 1; b.x_vec = 1;
        b.whole = apart(k) ? 0 : 1;
        TinyPlan tp;
        tiny_plan(p.n, p.m, WIDE, &tp);
        tg.first[it.count] = wgs; wgs += b.whole ? 1u : (unsigned)tp.slots;
        ++it.count;
      }
      if (it.count == 0) break;
      tg.first[it.count] = wgs;
      mark(stream);
      launch((tiny_batch_kernel<Q, T>), dim3(wgs), dim3(TINY_WG), stream, it, tg, outer);
      mark(stream);
    }
  }
  if constexpr (Q == Q1) {
    int k = 0;
    while (k < count) {
      BatchItems it;
      BatchGrid agg, red, hel;
      it.count = 0;
      unsigned a = 0, r = 0, h = 0;
      int values = 0;
      for (; k < count && it.count < BATCH_MAX; ++k) {
        if (!held_batchable(k)) continue;
        const mlproj_problem& p = pr[k];
        BatchItem& b = it.item[it.count];
        b.Y = p.Y; b.X = p.X; b.ws = p.workspace;
        b.v_out = p.v_out; b.u_out = p.u_out; b.mask_out = p.mask_out;
        b.n = p.n; b.m = p.m; b.eta = (double)p.eta;
        b.wide = 1; b.x_vec = 1; b.whole = 0;
        const Geometry g = plan_columns(p.n, p.m, WIDE, Q);
        agg.first[it.count] = a; a += (unsigned)(g.tiles * g.groups);
        red.first[it.count] = r; r += (unsigned)cdiv(p.m, SWG / reduce_parts(g.groups, fold_threads(g.groups)));
        hel.first[it.count] = h; h += (unsigned)cdiv(p.m, LH_COLS);
        if (held_values(k) > values) values = held_values(k);
        ++it.count;
      }
      if (it.count == 0) break;
      agg.first[it.count] = a; red.first[it.count] = r; hel.first[it.count] = h;
      mark(stream);
      launch((colagg_batch_kernel<Q, T>), dim3(a), dim3(WG), stream, it, agg);
      mark(stream);
      launch((reduce_batch_kernel<Q, T>), dim3(r), dim3(SWG), stream, it, red);
      mark(stream);
      // (a problem's threads hold the rows they would hold in its single call, whatever the
      // largest problem of the launch needs: slots past its last row stay empty)
      if (values == 32) launch((l11_held_batch_kernel<T, 32>), dim3(h), dim3(LH_WG), stream, it, hel, outer);
      else if (values == 64 && (long long)h > compute_units()) launch((l11_held_batch_kernel<T, 64, true>), dim3(h), dim3(LH_WG), stream, it, hel, outer);
      else if (values == 64) launch((l11_held_batch_kernel<T, 64>), dim3(h), dim3(LH_WG), stream, it, hel, outer);
      else launch((l11_held_batch_kernel<T, 128>), dim3(h), dim3(LH_WG), stream, it, hel, outer);
      mark(stream);
    }
  }
  int i = 0;
  while (i < count) {
    BatchItems it;
    BatchGrid agg, red, map, ini, upd;
    BatchL11Plan plan;
    it.count = 0;
    bool big = false;
    unsigned a = 0, r = 0, mp = 0, in = 0, up = 0;
    int max_sweeps = 0;
    for (; i < count && it.count < BATCH_MAX; ++i) {
      if (!batchable(i)) continue;
      const mlproj_problem& p = pr[i];
      BatchItem& b = it.item[it.count];
      b.Y = p.Y; b.X = p.X; b.ws = p.workspace;
      b.v_out = p.v_out; b.u_out = p.u_out; b.mask_out = p.mask_out;
      b.n = p.n; b.m = p.m; b.eta = (double)p.eta;
      b.wide = pick_vec(p.Y, p.m, (int)sizeof(T)) == WIDE ? 1 : 0;
      b.x_vec = aligned(p.X, 16) ? 1 : 0;
      b.whole = 0;
      const Geometry g = plan_columns(p.n, p.m, WIDE, Q);
      agg.first[it.count] = a; a += (unsigned)(g.tiles * g.groups);
      red.first[it.count] = r; r += (unsigned)cdiv(p.m, SWG / reduce_parts(g.groups, fold_threads(g.groups)));
      map.first[it.count] = mp; mp += (unsigned)(g.tiles * g.map_groups);
      ini.first[it.count] = in; in += (unsigned)cdiv(p.m, WG);
      upd.first[it.count] = up; up += (unsigned)cdiv(p.m, UPD_COLS);
      plan_l11(p.n, p.m, (int)sizeof(T), &plan.sweeps[it.count], &plan.handoff[it.count]);
      if (plan.sweeps[it.count] > max_sweeps) max_sweeps = plan.sweeps[it.count];
      big = big || p.m > FUSED_SEARCH_MAX;
      ++it.count;
    }
    if (it.count == 0) break;
    agg.first[it.count] = a; red.first[it.count] = r; map.first[it.count] = mp;
    ini.first[it.count] = in; upd.first[it.count] = up;
    mark(stream);
    launch((colagg_batch_kernel<Q, T>), dim3(a), dim3(WG), stream, it, agg);
    mark(stream);
    launch((reduce_batch_kernel<Q, T>), dim3(r), dim3(SWG), stream, it, red);
    if constexpr (Q == Q1) {
      // the inner searches: every kernel of the single-matrix chain once for the whole batch
      mark(stream);
      if (big) launch((l11_init_batch_kernel<T, SEARCH_CACHE_BIG>), dim3(in), dim3(WG), stream, it, ini, outer);
      else launch((l11_init_batch_kernel<T, SEARCH_CACHE>), dim3(in), dim3(WG), stream, it, ini, outer);
      mark(stream);
      for (int s = 0; s < max_sweeps; ++s) {
        if (s == 0) launch((l11_sweep_batch_kernel<T>), dim3(a), dim3(WG), stream, it, agg, plan);
        else launch((l11_filter_batch_kernel<T>), dim3(a), dim3(WG), stream, it, agg, plan, s);
        launch((l11_update_batch_kernel<T>), dim3(up), dim3(WG), stream, it, upd, plan, s);
      }
      launch((l11_finish_batch_kernel<T>), dim3(up), dim3(FIN_WG), stream, it, upd, plan);
    }
    mark(stream);
    if (big) launch((colmap_batch_kernel<Q, T, SEARCH_CACHE_BIG>), dim3(mp), dim3(WG), stream, it, map, outer);
    else launch((colmap_batch_kernel<Q, T, SEARCH_CACHE>), dim3(mp), dim3(WG), stream, it, map, outer);
    mark(stream);
  }
  int st = launch_status();
  for (int k = 0; k < count && st == MLPROJ_OK; ++k) {
    if (batchable(k) || tinyable(k) || held_batchable(k)) continue;
    st = run_bilevel<Q, T>(static_cast<const T*>(pr[k].Y), static_cast<T*>(pr[k].X), pr[k].n, pr[k].m, pr[k].eta,
                           pr[k].workspace, pr[k].workspace_bytes, pr[k].v_out, pr[k].u_out, stream_,
                           MODE_PROJECT, nullptr, STAGE_ALL, outer, pr[k].mask_out);
  }
  return st;
}

template <typename T>
static int dispatch_batch(int outer, int variant, int count, const mlproj_problem* pr, void* stream) {
  switch (variant) {
    case MLPROJ_L1INF: return run_batch<QINF, T>(outer, count, pr, stream);
    case MLPROJ_L11: return run_batch<Q1, T>(outer, count, pr, stream);
    case MLPROJ_L12: return run_batch<Q2, T>(outer, count, pr, stream);
    default: return MLPROJ_ERR_BAD_VARIANT;
  }
}

// ------------------------------------------------------------------ host: multi-level driver
constexpr int ML_MAX_DIMS = 8;
constexpr long long ML_TARGET_WGS = 1024;
constexpr long long ML_AGG_SHORT_WGS = 512;  // pipelined aggregate: 2 workgroups per CU

struct MlPlan {
  int ndim;
  long long size[ML_MAX_DIMS];   // size[k] = elements of level k = prod dims[0 .. ndim-1-k]
  long long len[ML_MAX_DIMS];    // len[k]  = fibre length aggregated to make level k (k >= 1)
  size_t off_V[ML_MAX_DIMS], off_R[ML_MAX_DIMS];  // fp64 arrays of level k (k = 1 .. ndim-1)
  Layout base;
  size_t bytes;
};

static int ml_plan(int ndim, const long long* dims, const int* norms, MlPlan* P) {
  if (!dims || !norms) return MLPROJ_ERR_NULL_POINTER;
  if (ndim < 2 || ndim > ML_MAX_DIMS) return MLPROJ_ERR_BAD_DIMENSION;
  long long total = 1;
  for (int i = 0; i < ndim; ++i) {
    if (dims[i] <= 0) return MLPROJ_ERR_BAD_DIMENSION;
    if (dims[i] > MAX_ELEMS || total > MAX_ELEMS / dims[i]) return MLPROJ_ERR_TOO_LARGE;
    total *= dims[i];
  }
  if (dims[0] > MAX_GROUPS) return MLPROJ_ERR_TOO_LARGE;
  for (int k = 0; k < ndim - 1; ++k)
    if (norms[k] != MLPROJ_NORM_INF && norms[k] != MLPROJ_NORM_L1 && norms[k] != MLPROJ_NORM_L2)
      return MLPROJ_ERR_BAD_VARIANT;
  P->ndim = ndim;
  long long sz = total;
  for (int k = 0; k < ndim; ++k) {
    P->size[k] = sz;
    P->len[k] = k == 0 ? 0 : dims[ndim - k];
    if (k + 1 < ndim) sz /= dims[ndim - 1 - k];
  }
  Geometry g{};  // no column partials: only the record, the search scratch and v[d0] are used
  g.tiles = 1; g.groups = 1; g.tile_w = 1; g.vec = 1;
  P->base = layout_for(g, dims[0], MLPROJ_L1INF);
  size_t o = P->base.bytes;
  for (int k = 1; k < ndim; ++k) {
    P->off_V[k] = o; o = align_up(o + (size_t)P->size[k] * 8, 256);
    P->off_R[k] = o; o = align_up(o + (size_t)P->size[k] * 8, 256);
  }
  P->bytes = o;
  return MLPROJ_OK;
}

// lanes per fibre: few enough that every lane has up to four chunks to itself
static int seg_for(long long nvec) { return nvec <= 16 ? 4 : (nvec <= 64 ? 16 : 64); }

static unsigned fibre_grid(long long nf, int seg, int unroll) {
  const long long per_wg = (long long)WAVES * (WAVE / seg) * unroll;
  long long wgs = cdiv(nf, per_wg);
  if (wgs > ML_TARGET_WGS) wgs = ML_TARGET_WGS;
  return (unsigned)(wgs < 1 ? 1 : wgs);
}

template <int Q, typename TIN, int VEC>
static void launch_fibre_agg(const TIN* A, long long nf, long long len, double* V, float* v_out,
                             hipStream_t stream) {
  const long long nvec = len / VEC;
  const int seg = seg_for(nvec);
  if (nvec <= (long long)seg * AGG_CHUNKS) {
    // one batch of loads covers a fibre: the pipelined kernel, few enough workgroups that
    // every wavefront has several batches to overlap
    const long long per_wg = (long long)WAVES * (WAVE / seg) * AGG_FIBRES;
    long long wgs = cdiv(nf, per_wg);
    if (wgs > ML_AGG_SHORT_WGS) wgs = ML_AGG_SHORT_WGS;
    const dim3 grid((unsigned)wgs), block(WG);
    if (seg == 4) launch((fibre_agg_short_kernel<Q, TIN, 4, VEC>), grid, block, stream, A, nf, len, V, v_out);
    else if (seg == 16) launch((fibre_agg_short_kernel<Q, TIN, 16, VEC>), grid, block, stream, A, nf, len, V, v_out);
    else launch((fibre_agg_short_kernel<Q, TIN, 64, VEC>), grid, block, stream, A, nf, len, V, v_out);
    return;
  }
  const dim3 grid(fibre_grid(nf, seg, FIB_UNROLL)), block(WG);
  if (seg == 4) launch((fibre_agg_kernel<Q, TIN, 4, VEC>), grid, block, stream, A, nf, len, V, v_out);
  else if (seg == 16) launch((fibre_agg_kernel<Q, TIN, 16, VEC>), grid, block, stream, A, nf, len, V, v_out);
  else launch((fibre_agg_kernel<Q, TIN, 64, VEC>), grid, block, stream, A, nf, len, V, v_out);
}

template <int Q, typename TIN, typename TOUT, int VEC, bool TOP = false>
static void launch_fibre_map(const TIN* A, long long nf, long long len, const double* R,
                             const double* Vn, TOUT* out, hipStream_t stream,
                             const TopFuse& tf = TopFuse{}) {
  const long long nvec = len / VEC;
  const int seg = seg_for(nvec);
  if (nvec <= (long long)seg * 4) {
    // the fibre fits the registers of its segment
    const dim3 cgrid(fibre_grid(nf, seg, FIB_MAP_UNROLL)), cblock(WG);
    const int kreg = nvec <= seg ? 1 : (nvec <= 2LL * seg ? 2 : 4);
#define MLPROJ_LAUNCH_CACHED(SEG_, K_)                                                              \
  launch((fibre_map_cached_kernel<Q, TIN, TOUT, SEG_, VEC, K_, TOP>), cgrid, cblock, stream, \
                     A, nf, len, R, Vn, out, tf)
    if (seg == 4) { if (kreg == 1) MLPROJ_LAUNCH_CACHED(4, 1); else if (kreg == 2) MLPROJ_LAUNCH_CACHED(4, 2); else MLPROJ_LAUNCH_CACHED(4, 4); }
    else if (seg == 16) { if (kreg == 1) MLPROJ_LAUNCH_CACHED(16, 1); else if (kreg == 2) MLPROJ_LAUNCH_CACHED(16, 2); else MLPROJ_LAUNCH_CACHED(16, 4); }
    else { if (kreg == 1) MLPROJ_LAUNCH_CACHED(64, 1); else if (kreg == 2) MLPROJ_LAUNCH_CACHED(64, 2); else MLPROJ_LAUNCH_CACHED(64, 4); }
#undef MLPROJ_LAUNCH_CACHED
    return;
  }
  const dim3 grid(fibre_grid(nf, seg, 1)), block(WG);
  if (seg == 4) launch((fibre_map_kernel<Q, TIN, TOUT, 4, VEC, TOP>), grid, block, stream, A, nf, len, R, Vn, out, tf);
  else if (seg == 16) launch((fibre_map_kernel<Q, TIN, TOUT, 16, VEC, TOP>), grid, block, stream, A, nf, len, R, Vn, out, tf);
  else launch((fibre_map_kernel<Q, TIN, TOUT, 64, VEC, TOP>), grid, block, stream, A, nf, len, R, Vn, out, tf);
}

template <typename F>
static void by_norm(int norm, F&& f) {
  if (norm == MLPROJ_NORM_INF) f(std::integral_constant<int, QINF>{});
  else if (norm == MLPROJ_NORM_L1) f(std::integral_constant<int, Q1>{});
  else f(std::integral_constant<int, Q2>{});
}

// The workspace of a multi-level call: what the level arrays of the unmerged plan need, and
// what the slab kernels need when every inner norm is l_inf (see run_multilevel).
static int ml_workspace_bytes(int ndim, const long long* dims, size_t* out) {
  int norms[ML_MAX_DIMS] = {0};
  MlPlan P;
  int st = ml_plan(ndim, dims, norms, &P);
  if (st != MLPROJ_OK) return st;
  size_t tri = 0;
  st = workspace_bytes_impl(MLPROJ_L1INFINF, dims[0], P.size[0] / dims[0], 1, &tri);
  if (st != MLPROJ_OK) return st;
  *out = P.bytes > tri ? P.bytes : tri;
  return MLPROJ_OK;
}

template <typename T>
static int run_multilevel(int outer, const T* Y, T* X, int ndim, const long long* dims_in,
                          const int* norms_in, float eta, void* workspace, size_t workspace_bytes,
                          float* v_out, float* u_out, void* stream_, const float* weights = nullptr) {
  constexpr int WIDE = 16 / (int)sizeof(T);
  if (!Y || !X || !workspace) return MLPROJ_ERR_NULL_POINTER;
  if (outer < MLPROJ_OUTER_L1 || outer > MLPROJ_OUTER_LINF) return MLPROJ_ERR_BAD_VARIANT;
  if (weights && outer != MLPROJ_OUTER_L1) return MLPROJ_ERR_BAD_VARIANT;
  MlPlan P;
  int st = ml_plan(ndim, dims_in, norms_in, &P);   // checks the arguments as given
  if (st != MLPROJ_OK) return st;
  size_t need = 0;
  if ((st = ml_workspace_bytes(ndim, dims_in, &need)) != MLPROJ_OK) return st;
  if (!aligned(workspace, 256) || workspace_bytes < need) return MLPROJ_ERR_WORKSPACE;
  // Two neighbouring l_inf levels are one: the max of maxima is the max over both axes, and
  // clipping a fibre to min(its own max, the radius above) clips it to the radius above.  So
  // neighbouring l_inf axes are merged (the tensor is C-order: they are contiguous), and a
  // projection whose inner norms are all l_inf is the slab form of the tri-level projection.
  long long dims[ML_MAX_DIMS];
  int norms[ML_MAX_DIMS];
  int nd = 1;
  dims[0] = dims_in[0];
  // level k = 1..ndim-1 aggregates axis ndim-k with norms_in[k-1]; walk the axes from the outside in
  for (int axis = 1; axis < ndim; ++axis) {
    const int nrm = norms_in[ndim - 1 - axis];
    if (nd > 1 && nrm == MLPROJ_NORM_INF && norms[nd - 1] == MLPROJ_NORM_INF) {
      dims[nd - 1] *= dims_in[axis];
    } else {
      dims[nd] = dims_in[axis];
      norms[nd] = nrm;
      ++nd;
    }
  }
  // norms[] above is indexed by axis (1..nd-1); ml_plan wants it innermost first
  int norms_inner_first[ML_MAX_DIMS];
  for (int axis = 1; axis < nd; ++axis) norms_inner_first[nd - 1 - axis] = norms[axis];
  if (nd == 2 && norms_inner_first[0] == MLPROJ_NORM_INF && outer == MLPROJ_OUTER_L1 && !weights)
    return run_trilevel<T>(Y, X, dims[0], dims[1], 1, eta, workspace, workspace_bytes, v_out, u_out,
                           nullptr, stream_);
  ndim = nd;
  const int* norms_use = norms_inner_first;
  st = ml_plan(ndim, dims, norms_use, &P);
  if (st != MLPROJ_OK) return st;
  if ((st = check_radius(eta)) != MLPROJ_OK) return st;
  if (!aligned(Y, sizeof(T)) || !aligned(X, sizeof(T))) return MLPROJ_ERR_ALIGNMENT;
  if (workspace_bytes < P.bytes) return MLPROJ_ERR_WORKSPACE;
  Ws ws = bind(workspace, P.base);
  ws.wts = weights;   // (a weighted l1 ball as outer norm: its own search kernel, nothing fused)
  char* base = static_cast<char*>(workspace);
  double* V[ML_MAX_DIMS];
  double* R[ML_MAX_DIMS];
  for (int k = 1; k < ndim; ++k) {
    V[k] = reinterpret_cast<double*>(base + P.off_V[k]);
    R[k] = reinterpret_cast<double*>(base + P.off_R[k]);
  }
  V[ndim - 1] = ws.v;  // the top aggregate is the vector the search reads
  hipStream_t stream = static_cast<hipStream_t>(stream_);
  const long long len1 = P.len[1];
  const bool wide = len1 % WIDE == 0 && aligned(Y, 16) && aligned(X, 16);

  // up: aggregate level by level
  mark(stream);
  by_norm(norms_use[0], [&](auto q) {
    float* vo = ndim == 2 ? v_out : nullptr;
    if (wide) launch_fibre_agg<decltype(q)::value, T, WIDE>(Y, P.size[1], len1, V[1], vo, stream);
    else launch_fibre_agg<decltype(q)::value, T, 1>(Y, P.size[1], len1, V[1], vo, stream);
  });
  for (int k = 2; k < ndim; ++k) {
    by_norm(norms_use[k - 1], [&](auto q) {
      launch_fibre_agg<decltype(q)::value, double, 1>(V[k - 1], P.size[k], P.len[k], V[k],
                                                      k == ndim - 1 ? v_out : nullptr, stream);
    });
  }
  // top: threshold of the l1-ball projection of the length-d0 vector, then its radii.  With
  // three or more axes and at most 4096 groups the map of the top level does this itself.
  const bool fuse_top = ndim >= 3 && dims[0] <= FUSED_SEARCH_MAX && !weights;
  if (!fuse_top) mark(stream);
  if (fuse_top) {
    // nothing here: see the first map below
  } else if (weights && dims[0] <= 32768) {
    // (one workgroup: it writes the radii too, and nothing has to be cleared for it)
    launch_weighted_search(ws, dims[0], (double)eta, stream, R[ndim - 1], u_out);
  } else if (weights) {
    launch(clear_flags_kernel, dim3(1), dim3(WG), stream, ws);
    launch_weighted_search(ws, dims[0], (double)eta, stream);
    launch(top_radii_kernel, dim3((unsigned)cdiv(dims[0], WG)), dim3(WG), stream, ws,
                       dims[0], R[ndim - 1], u_out);
  } else if (dims[0] <= (long long)SWG * SEARCH_CACHE || outer != MLPROJ_OUTER_L1) {
    launch((search_kernel<SWG, SEARCH_CACHE>), dim3(1), dim3(SWG), stream, ws, dims[0], (double)eta, MODE_PROJECT,
                       outer, (double*)nullptr, 0, R[ndim - 1], u_out);
  } else {
    launch(clear_flags_kernel, dim3(1), dim3(WG), stream, ws);
    launch_search(ws, dims[0], (double)eta, MODE_PROJECT, outer, nullptr, stream);
    launch(top_radii_kernel, dim3((unsigned)cdiv(dims[0], WG)), dim3(WG), stream, ws,
                       dims[0], R[ndim - 1], u_out);
  }
  // down: project the fibres of every level onto the balls of the level above
  mark(stream);
  for (int k = ndim - 1; k >= 2; --k) {
    by_norm(norms_use[k - 1], [&](auto q) {
      if (fuse_top && k == ndim - 1)
        launch_fibre_map<decltype(q)::value, double, double, 1, true>(V[k - 1], P.size[k], P.len[k], R[k], V[k],
                                                                      R[k - 1], stream,
                                                                      TopFuse{ws, (double)eta, outer, u_out});
      else
        launch_fibre_map<decltype(q)::value, double, double, 1>(V[k - 1], P.size[k], P.len[k], R[k], V[k],
                                                                R[k - 1], stream);
    });
  }
  by_norm(norms_use[0], [&](auto q) {
    if (wide) launch_fibre_map<decltype(q)::value, T, T, WIDE>(Y, P.size[1], len1, R[1], V[1], X, stream);
    else launch_fibre_map<decltype(q)::value, T, T, 1>(Y, P.size[1], len1, R[1], V[1], X, stream);
  });
  mark(stream);
  return launch_status();
}

// ------------------------------------------------------------------ host: the built-in scratch
// For callers that cannot allocate (see bilevel_proj_l1inf_no_alloc): the workspace of such a
// call is this array in the library's own device image.  Every GPU the library runs on holds a
// copy of it, at its own address, until the process ends.  In host code the array's name is only
// a handle for hipGetSymbolAddress: the address a kernel can use is asked for once per device,
// with that device current, and kept; from then on only that pointer is used.
constexpr size_t NO_ALLOC_SCRATCH_BYTES = (size_t)MLPROJ_NO_ALLOC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[NO_ALLOC_SCRATCH_BYTES];

constexpr int NO_ALLOC_MAX_DEVICES = 64;
static std::mutex g_scratch_mutex;
static void* g_scratch_ptr[NO_ALLOC_MAX_DEVICES];   // per device: where its copy of `scratch` lives

static int scratch_of_current_device(void** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= NO_ALLOC_MAX_DEVICES) return MLPROJ_ERR_LAUNCH;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return MLPROJ_ERR_LAUNCH;
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return MLPROJ_OK;
}

}  // namespace mlproj

// ------------------------------------------------------------------ C ABI
using namespace mlproj;

extern "C" {

int mlproj_version(void) { return 386; }

const char* mlproj_status_string(int status) {
  switch (status) {
    case MLPROJ_OK: return "ok";
    case MLPROJ_ERR_NULL_POINTER: return "a required pointer is NULL";
    case MLPROJ_ERR_BAD_DIMENSION: return "a dimension is not positive";
    case MLPROJ_ERR_TOO_LARGE: return "input exceeds the supported size";
    case MLPROJ_ERR_BAD_RADIUS: return "eta must be finite and >= 0";
    case MLPROJ_ERR_WORKSPACE: return "workspace too small or not 256-byte aligned";
    case MLPROJ_ERR_BAD_VARIANT: return "unknown variant";
    case MLPROJ_ERR_ALIGNMENT: return "Y and X must be aligned to their element size";
    case MLPROJ_ERR_LAUNCH: return "HIP refused a kernel launch";
    case MLPROJ_ERR_NO_ALLOC_LIMIT: return "input needs more scratch memory than the built-in buffer of the no-allocation entry point holds";
    default: return "unknown status";
  }
}

int mlproj_trace_begin(void** events, int capacity) {
  if (!events) return MLPROJ_ERR_NULL_POINTER;
  if (capacity <= 0) return MLPROJ_ERR_BAD_DIMENSION;
  g_trace.events = reinterpret_cast<hipEvent_t*>(events);
  g_trace.capacity = capacity;
  g_trace.count = 0;
  return MLPROJ_OK;
}

int mlproj_trace_end(void) {
  const int n = g_trace.count;
  g_trace = Trace{};
  return n;
}

int mlproj_set_l11_sweeps(int sweeps) {
  if (sweeps < 0 || sweeps > MAX_INNER_SWEEPS) return MLPROJ_ERR_BAD_DIMENSION;
  return g_l11_sweeps.exchange(sweeps, std::memory_order_relaxed);
}

int mlproj_stripe_of_workgroup(long long workgroup, long long stripes) {
  if (stripes <= 0 || stripes > 0x7fffffffLL || workgroup < 0 || workgroup >= stripes) return -1;
  return (int)stripe_of_workgroup(workgroup, stripes);
}

int mlproj_set_search_spin_limit(int polls) {
  if (polls < 0 || polls > (int)SPIN_LIMIT_MAX) return MLPROJ_ERR_BAD_DIMENSION;
  return (int)g_spin_limit.exchange((unsigned)polls, std::memory_order_relaxed);
}

int mlproj_workspace_bytes(int variant, long long d0, long long d1, long long d2, size_t* bytes_out) {
  return workspace_bytes_impl(variant, d0, d1, d2, bytes_out);
}

int mlproj_norm_l1q(const float* Y, long long n, long long m, int q_variant, void* workspace,
                    size_t workspace_bytes, double* norm_out, float* v_out, void* stream) {
  return dispatch_q(q_variant, Y, (float*)nullptr, n, m, 0.f, workspace, workspace_bytes, v_out,
                    (float*)nullptr, stream, MODE_NORM, norm_out, STAGE_AGGREGATE, (int)MLPROJ_OUTER_L1);
}

int bilevel_proj_l1inf(const float* Y, float* X, long long n, long long m, float eta,
                       void* workspace, size_t workspace_bytes, float* v_out, float* u_out,
                       void* stream) {
  return run_bilevel<QINF>(Y, X, n, m, eta, workspace, workspace_bytes, v_out, u_out, stream,
                           MODE_PROJECT, nullptr, STAGE_ALL, (int)MLPROJ_OUTER_L1);
}

int bilevel_proj_l1inf_no_alloc(const float* Y, float* X, long long n, long long m, float eta,
                                float* v_out, float* u_out, void* stream) {
  // every check that needs no GPU first, so that a refused call has touched nothing
  if (!Y || !X) return MLPROJ_ERR_NULL_POINTER;
  size_t need = 0;
  int st = workspace_bytes_impl(MLPROJ_L1INF, n, m, 1, &need);
  if (st != MLPROJ_OK) return st;
  if ((st = check_radius(eta)) != MLPROJ_OK) return st;
  if (need > NO_ALLOC_SCRATCH_BYTES) return MLPROJ_ERR_NO_ALLOC_LIMIT;
  void* ws = nullptr;
  if ((st = scratch_of_current_device(&ws)) != MLPROJ_OK) return st;
  // (the chain initialises what it needs in the workspace itself: nothing to clear between calls)
  return run_bilevel<QINF>(Y, X, n, m, eta, ws, NO_ALLOC_SCRATCH_BYTES, v_out, u_out, stream,
                           MODE_PROJECT, nullptr, STAGE_ALL, (int)MLPROJ_OUTER_L1);
}

int bilevel_proj_l11(const float* Y, float* X, long long n, long long m, float eta,
                     void* workspace, size_t workspace_bytes, float* v_out, float* u_out,
                     void* stream) {
  return run_bilevel<Q1>(Y, X, n, m, eta, workspace, workspace_bytes, v_out, u_out, stream,
                         MODE_PROJECT, nullptr, STAGE_ALL, (int)MLPROJ_OUTER_L1);
}

int bilevel_proj_l12(const float* Y, float* X, long long n, long long m, float eta,
                     void* workspace, size_t workspace_bytes, float* v_out, float* u_out,
                     void* stream) {
  return run_bilevel<Q2>(Y, X, n, m, eta, workspace, workspace_bytes, v_out, u_out, stream,
                         MODE_PROJECT, nullptr, STAGE_ALL, (int)MLPROJ_OUTER_L1);
}

int bilevel_radii(int variant, const float* Y, long long n, long long m, float eta,
                  void* workspace, size_t workspace_bytes, float* v_out, void* stream) {
  return dispatch_q(variant, Y, (float*)nullptr, n, m, eta, workspace, workspace_bytes, v_out,
                    (float*)nullptr, stream, MODE_PROJECT, (double*)nullptr, STAGE_AGGREGATE, (int)MLPROJ_OUTER_L1);
}

int bilevel_apply(int variant, const float* Y, float* X, long long n, long long m,
                  void* workspace, size_t workspace_bytes, float* u_out, void* stream) {
  return dispatch_q(variant, Y, X, n, m, 0.f, workspace, workspace_bytes, (float*)nullptr, u_out,
                    stream, MODE_PROJECT, (double*)nullptr, STAGE_APPLY, (int)MLPROJ_OUTER_L1);
}

int mlproj_multilevel_workspace_bytes(int ndim, const long long* dims, size_t* bytes_out) {
  if (!bytes_out) return MLPROJ_ERR_NULL_POINTER;
  return ml_workspace_bytes(ndim, dims, bytes_out);
}

int multilevel_proj(const float* Y, float* X, int ndim, const long long* dims, const int* norms,
                    float eta, void* workspace, size_t workspace_bytes, float* v_out, float* u_out,
                    void* stream) {
  return run_multilevel(MLPROJ_OUTER_L1, Y, X, ndim, dims, norms, eta, workspace, workspace_bytes, v_out, u_out, stream);
}

int multilevel_proj_p(int outer_norm, const float* Y, float* X, int ndim, const long long* dims,
                      const int* norms, float eta, void* workspace, size_t workspace_bytes,
                      float* v_out, float* u_out, void* stream) {
  return run_multilevel(outer_norm, Y, X, ndim, dims, norms, eta, workspace, workspace_bytes, v_out, u_out, stream);
}

int bilevel_proj_pq(int outer_norm, int variant, const float* Y, float* X, long long n, long long m,
                    float eta, void* workspace, size_t workspace_bytes, float* v_out, float* u_out,
                    void* stream) {
  return dispatch_q(variant, Y, X, n, m, eta, workspace, workspace_bytes, v_out, u_out, stream,
                    MODE_PROJECT, (double*)nullptr, STAGE_ALL, outer_norm);
}

int bilevel_proj_stored(int storage, int outer_norm, int variant, const void* Y, void* X,
                        long long n, long long m, float eta, void* workspace,
                        size_t workspace_bytes, float* v_out, float* u_out,
                        unsigned char* mask_out, void* stream) {
  switch (storage) {
    case MLPROJ_STORE_F32:
      return dispatch_stored<float>(outer_norm, variant, Y, X, n, m, eta, workspace, workspace_bytes, v_out, u_out, mask_out, stream);
    case MLPROJ_STORE_BF16:
      return dispatch_stored<bf16_t>(outer_norm, variant, Y, X, n, m, eta, workspace, workspace_bytes, v_out, u_out, mask_out, stream);
    case MLPROJ_STORE_F16:
      return dispatch_stored<f16_t>(outer_norm, variant, Y, X, n, m, eta, workspace, workspace_bytes, v_out, u_out, mask_out, stream);
    default: return MLPROJ_ERR_BAD_VARIANT;
  }
}

int bilevel_proj_weighted(int storage, int variant, const void* Y, void* X, long long n, long long m,
                          float eta, const float* weights, void* workspace, size_t workspace_bytes,
                          float* v_out, float* u_out, unsigned char* mask_out, void* stream) {
  if (!weights) return MLPROJ_ERR_NULL_POINTER;
  if (!aligned(weights, sizeof(float))) return MLPROJ_ERR_ALIGNMENT;
  auto go = [&](auto tag) {
    using T = decltype(tag);
    return dispatch_q(variant, static_cast<const T*>(Y), static_cast<T*>(X), n, m, eta, workspace,
                      workspace_bytes, v_out, u_out, stream, MODE_PROJECT, (double*)nullptr, STAGE_ALL,
                      (int)MLPROJ_OUTER_L1, mask_out, false, weights);
  };
  switch (storage) {
    case MLPROJ_STORE_F32: return go(float{});
    case MLPROJ_STORE_BF16: return go(bf16_t{});
    case MLPROJ_STORE_F16: return go(f16_t{});
    default: return MLPROJ_ERR_BAD_VARIANT;
  }
}

int multilevel_proj_weighted(int storage, const void* Y, void* X, int ndim, const long long* dims,
                             const int* norms, float eta, const float* weights, void* workspace,
                             size_t workspace_bytes, float* v_out, float* u_out, void* stream) {
  if (!weights) return MLPROJ_ERR_NULL_POINTER;
  if (!aligned(weights, sizeof(float))) return MLPROJ_ERR_ALIGNMENT;
  const int outer = (int)MLPROJ_OUTER_L1;
  switch (storage) {
    case MLPROJ_STORE_F32:
      return run_multilevel<float>(outer, static_cast<const float*>(Y), static_cast<float*>(X), ndim, dims, norms, eta, workspace, workspace_bytes, v_out, u_out, stream, weights);
    case MLPROJ_STORE_BF16:
      return run_multilevel<bf16_t>(outer, static_cast<const bf16_t*>(Y), static_cast<bf16_t*>(X), ndim, dims, norms, eta, workspace, workspace_bytes, v_out, u_out, stream, weights);
    case MLPROJ_STORE_F16:
      return run_multilevel<f16_t>(outer, static_cast<const f16_t*>(Y), static_cast<f16_t*>(X), ndim, dims, norms, eta, workspace, workspace_bytes, v_out, u_out, stream, weights);
    default: return MLPROJ_ERR_BAD_VARIANT;
  }
}

int bilevel_proj_batch(int storage, int outer_norm, int variant, int count,
                       const mlproj_problem* problems, void* stream) {
  if (!problems) return MLPROJ_ERR_NULL_POINTER;
  if (count <= 0) return MLPROJ_ERR_BAD_DIMENSION;
  switch (storage) {
    case MLPROJ_STORE_F32: return dispatch_batch<float>(outer_norm, variant, count, problems, stream);
    case MLPROJ_STORE_BF16: return dispatch_batch<bf16_t>(outer_norm, variant, count, problems, stream);
    case MLPROJ_STORE_F16: return dispatch_batch<f16_t>(outer_norm, variant, count, problems, stream);
    default: return MLPROJ_ERR_BAD_VARIANT;
  }
}

int trilevel_proj_l1infinf(const float* Y, float* X, long long d0, long long d1, long long d2,
                           float eta, void* workspace, size_t workspace_bytes, float* v_out,
                           float* u_out, void* stream) {
  return run_trilevel<float>(Y, X, d0, d1, d2, eta, workspace, workspace_bytes, v_out, u_out, nullptr, stream);
}

int trilevel_proj_stored(int storage, const void* Y, void* X, long long d0, long long d1, long long d2,
                         float eta, void* workspace, size_t workspace_bytes, float* v_out,
                         float* u_out, unsigned char* mask_out, void* stream) {
  switch (storage) {
    case MLPROJ_STORE_F32:
      return run_trilevel<float>(static_cast<const float*>(Y), static_cast<float*>(X), d0, d1, d2, eta, workspace, workspace_bytes, v_out, u_out, mask_out, stream);
    case MLPROJ_STORE_BF16:
      return run_trilevel<bf16_t>(static_cast<const bf16_t*>(Y), static_cast<bf16_t*>(X), d0, d1, d2, eta, workspace, workspace_bytes, v_out, u_out, mask_out, stream);
    case MLPROJ_STORE_F16:
      return run_trilevel<f16_t>(static_cast<const f16_t*>(Y), static_cast<f16_t*>(X), d0, d1, d2, eta, workspace, workspace_bytes, v_out, u_out, mask_out, stream);
    default: return MLPROJ_ERR_BAD_VARIANT;
  }
}

int multilevel_proj_stored(int storage, int outer_norm, const void* Y, void* X, int ndim,
                           const long long* dims, const int* norms, float eta, void* workspace,
                           size_t workspace_bytes, float* v_out, float* u_out, void* stream) {
  switch (storage) {
    case MLPROJ_STORE_F32:
      return run_multilevel<float>(outer_norm, static_cast<const float*>(Y), static_cast<float*>(X), ndim, dims, norms, eta, workspace, workspace_bytes, v_out, u_out, stream);
    case MLPROJ_STORE_BF16:
      return run_multilevel<bf16_t>(outer_norm, static_cast<const bf16_t*>(Y), static_cast<bf16_t*>(X), ndim, dims, norms, eta, workspace, workspace_bytes, v_out, u_out, stream);
    case MLPROJ_STORE_F16:
      return run_multilevel<f16_t>(outer_norm, static_cast<const f16_t*>(Y), static_cast<f16_t*>(X), ndim, dims, norms, eta, workspace, workspace_bytes, v_out, u_out, stream);
    default: return MLPROJ_ERR_BAD_VARIANT;
  }
}

}  // extern "C"
