// mlproj: several independent bi-level projections in one chain of launches.
#ifndef MLPROJ_BATCH_H
#define MLPROJ_BATCH_H

#include "aggregate.h"
#include "common.h"
#include "l11.h"
#include "l11held.h"
#include "map.h"
#include "tiny.h"

namespace mlproj {

// A training loop projects many weight matrices after every step (the use Sec. 6.3 makes of
// the projection), most of them small enough that the three launches of a call are what it
// costs.  Up to BATCH_MAX matrices share one aggregate, one fold and one map launch (and,
// for l1,1, one launch per kernel of the inner searches): the
// problems travel in the kernel arguments, a workgroup finds the problem its number falls
// into and then runs exactly the code of the single-matrix kernels on it, with the geometry
// and workspace layout recomputed on the device from (n, m).
constexpr int BATCH_MAX = 16;

struct BatchItem {
  const void* Y;
  void* X;
  void* ws;
  float* v_out;
  float* u_out;
  unsigned char* mask_out;
  long long n, m;
  double eta;
  int wide;   // rows are 16-byte aligned: the wide form of LaneCols
  int x_vec;  // ... and so is X: 16-byte stores
  int whole;  // one-kernel form: X overlaps Y, one workgroup does the whole matrix
};

struct BatchItems {
  int count;
  BatchItem item[BATCH_MAX];
};

struct BatchGrid {
  unsigned first[BATCH_MAX + 1];  // first workgroup of every problem in this launch, then the total
};

// The problem a workgroup belongs to, and its number within that problem.
__device__ __forceinline__ int batch_find(const BatchGrid& gr, int count, long long& bid) {
  int p = 0;
  while (p + 1 < count && blockIdx.x >= gr.first[p + 1]) ++p;
  bid = (long long)blockIdx.x - (long long)gr.first[p];
  return p;
}

template <int Q, typename T>
__global__ __launch_bounds__(WG) void colagg_batch_kernel(BatchItems it, BatchGrid gr) {
  constexpr int WIDE = 16 / (int)sizeof(T);
  long long bid;
  const BatchItem& b = it.item[batch_find(gr, it.count, bid)];
  const Geometry g = plan_columns(b.n, b.m, WIDE, Q);
  const Ws ws = bind(b.ws, layout_for(g, b.m, Q));
  const T* Y = static_cast<const T*>(b.Y);
  if (b.wide) colagg_body<Q, T, WIDE, false>(Y, b.n, b.m, g, ws.partial, bid);
  else colagg_body<Q, T, WIDE, true>(Y, b.n, b.m, g, ws.partial, bid);
}

template <int Q, typename T>
__global__ __launch_bounds__(SWG) void reduce_batch_kernel(BatchItems it, BatchGrid gr) {
  constexpr int WIDE = 16 / (int)sizeof(T);
  long long bid;
  const BatchItem& b = it.item[batch_find(gr, it.count, bid)];
  const Geometry g = plan_columns(b.n, b.m, WIDE, Q);
  const Ws ws = bind(b.ws, layout_for(g, b.m, Q));
  reduce_body<Q>(ws.partial, b.m, g, reduce_parts(g.groups, fold_threads(g.groups)), ws.v, b.v_out, ws.flags, bid);
}

template <int Q, typename T, int SC>
__global__ __launch_bounds__(WG) void colmap_batch_kernel(BatchItems it, BatchGrid gr, int outer) {
  constexpr int WIDE = 16 / (int)sizeof(T);
  long long bid;
  const BatchItem& b = it.item[batch_find(gr, it.count, bid)];
  const Geometry g = plan_columns(b.n, b.m, WIDE, Q);
  const Ws ws = bind(b.ws, layout_for(g, b.m, Q));
  const T* Y = static_cast<const T*>(b.Y);
  T* X = static_cast<T*>(b.X);
  const double eta = Q == Q1 ? -1.0 : b.eta;   // l1,1: tau comes from the record, not from a search here
  if (b.wide && b.x_vec)
    colmap_body<Q, T, WIDE, false, true, SC>(Y, X, b.n, b.m, g, ws, b.u_out, b.mask_out, eta, outer, bid);
  else if (b.wide)
    colmap_body<Q, T, WIDE, false, false, SC>(Y, X, b.n, b.m, g, ws, b.u_out, b.mask_out, eta, outer, bid);
  else
    colmap_body<Q, T, WIDE, true, false, SC>(Y, X, b.n, b.m, g, ws, b.u_out, b.mask_out, eta, outer, bid);
}

// Matrices of at most 128 KiB each: the one-kernel form of tiny.h for all of them in one launch
// (up to 16 workgroups for a matrix whose X lies apart from Y, one for a matrix projected in place).
template <int Q, typename T>
__global__ __launch_bounds__(TINY_WG) void tiny_batch_kernel(BatchItems it, BatchGrid gr, int outer) {
  constexpr int WIDE = 16 / (int)sizeof(T);
  long long bid;
  const BatchItem& b = it.item[batch_find(gr, it.count, bid)];
  TinyPlan tp;
  if (!tiny_plan(b.n, b.m, WIDE, &tp)) return;   // (the host only sends matrices that fit)
  const Geometry g = plan_columns(b.n, b.m, WIDE, Q);
  const Ws ws = bind(b.ws, layout_for(g, b.m, Q));
  tiny_body<Q, T, WIDE>(static_cast<const T*>(b.Y), static_cast<T*>(b.X), b.n, b.m, b.eta, outer, tp.cw, ws,
                           b.v_out, b.u_out, b.mask_out, bid, b.whole != 0);
}

// ------------------------------------------------------------------ l1,1: the inner searches
// The same for the kernels of the per-column threshold searches (l11.h).  Every problem has
// its own number of lock-step sweeps and hand-over count; a sweep kernel of the batch leaves
// the problems alone that planned fewer sweeps.
struct BatchL11Plan {
  int sweeps[BATCH_MAX];
  unsigned handoff[BATCH_MAX];
};

template <typename T, int SC>
__global__ __launch_bounds__(WG) void l11_init_batch_kernel(BatchItems it, BatchGrid gr, int outer) {
  constexpr int WIDE = 16 / (int)sizeof(T);
  long long bid;
  const BatchItem& b = it.item[batch_find(gr, it.count, bid)];
  const Geometry g = plan_columns(b.n, b.m, WIDE, Q1);
  const Ws ws = bind(b.ws, layout_for(g, b.m, Q1));
  l11_init_body<SC>(b.n, b.m, ws, b.eta, outer, bid);
}

template <typename T>
__global__ __launch_bounds__(WG) void l11_sweep_batch_kernel(BatchItems it, BatchGrid gr,
                                                             BatchL11Plan plan) {
  constexpr int WIDE = 16 / (int)sizeof(T);
  __shared__ SweepLds<WAVE * WIDE> lds;
  long long bid;
  const int p = batch_find(gr, it.count, bid);
  if (plan.sweeps[p] < 1) return;
  const BatchItem& b = it.item[p];
  const Geometry g = plan_columns(b.n, b.m, WIDE, Q1);
  const Ws ws = bind(b.ws, layout_for(g, b.m, Q1));
  const T* Y = static_cast<const T*>(b.Y);
  if (b.wide) l11_sweep_body<T, WIDE, false>(Y, b.n, b.m, g, ws, bid, lds);
  else l11_sweep_body<T, WIDE, true>(Y, b.n, b.m, g, ws, bid, lds);
}

template <typename T>
__global__ __launch_bounds__(WG) void l11_filter_batch_kernel(BatchItems it, BatchGrid gr,
                                                              BatchL11Plan plan, int sweep) {
  constexpr int WIDE = 16 / (int)sizeof(T);
  __shared__ FilterLds<WAVE * WIDE> lds;
  long long bid;
  const int p = batch_find(gr, it.count, bid);
  if (sweep >= plan.sweeps[p]) return;
  const BatchItem& b = it.item[p];
  const Geometry g = plan_columns(b.n, b.m, WIDE, Q1);
  const Ws ws = bind(b.ws, layout_for(g, b.m, Q1));
  const T* Y = static_cast<const T*>(b.Y);
  if (b.wide) l11_filter_body<T, WIDE, false>(Y, b.n, b.m, g, ws, sweep, plan.handoff[p], bid, lds);
  else l11_filter_body<T, WIDE, true>(Y, b.n, b.m, g, ws, sweep, plan.handoff[p], bid, lds);
}

template <typename T>
__global__ __launch_bounds__(WG) void l11_update_batch_kernel(BatchItems it, BatchGrid gr,
                                                              BatchL11Plan plan, int sweep) {
  constexpr int WIDE = 16 / (int)sizeof(T);
  long long bid;
  const int p = batch_find(gr, it.count, bid);
  if (sweep >= plan.sweeps[p]) return;
  const BatchItem& b = it.item[p];
  const Geometry g = plan_columns(b.n, b.m, WIDE, Q1);
  const Ws ws = bind(b.ws, layout_for(g, b.m, Q1));
  l11_update_body(b.n, b.m, g, ws, sweep, plan.handoff[p], bid);
}

template <typename T>
__global__ __launch_bounds__(FIN_WG) void l11_finish_batch_kernel(BatchItems it, BatchGrid gr,
                                                               BatchL11Plan plan) {
  constexpr int WIDE = 16 / (int)sizeof(T);
  long long bid;
  const int p = batch_find(gr, it.count, bid);
  const BatchItem& b = it.item[p];
  const Geometry g = plan_columns(b.n, b.m, WIDE, Q1);
  const Ws ws = bind(b.ws, layout_for(g, b.m, Q1));
  if (b.n <= (long long)FIN_ROWS * FIN_HELD)
    l11_finish_body<T, true>(static_cast<const T*>(b.Y), b.n, b.m, ws, plan.sweeps[p], plan.handoff[p], bid);
  else
    l11_finish_body<T, false>(static_cast<const T*>(b.Y), b.n, b.m, ws, plan.sweeps[p], plan.handoff[p], bid);
}

// l1,1 problems of at most 4096 rows after their aggregate pass: the columns-in-registers kernel
// of l11held.h, every workgroup running the outer search of its own problem.  NV: the values per
// thread the tallest problem of the launch needs.
template <typename T, int NV, bool PACKED = false>
__global__ __launch_bounds__(LH_WG, lh_min_waves(NV, PACKED)) void l11_held_batch_kernel(BatchItems it, BatchGrid gr,
                                                                                        int outer) {
  constexpr int WIDE = 16 / (int)sizeof(T);
  long long bid;
  const int p = batch_find(gr, it.count, bid);
  const BatchItem& b = it.item[p];
  const Geometry g = plan_columns(b.n, b.m, WIDE, Q1);
  const Ws ws = bind(b.ws, layout_for(g, b.m, Q1));
  const long long stripes = (long long)(gr.first[p + 1] - gr.first[p]);
  l11_held_body<T, NV, LH_SEARCH_CACHE>(static_cast<const T*>(b.Y), static_cast<T*>(b.X), b.n, b.m, ws, b.u_out,
                                        b.mask_out, b.eta, outer, stripe_of_workgroup(bid, stripes));
}

}  // namespace mlproj

#endif
