// mlproj: several independent bi-level projections in one chain of launches.
#ifndef MLPROJ_BATCH_H
#define MLPROJ_BATCH_H

#include "aggregate.h"
#include "common.h"
#include "map.h"

namespace mlproj {

// A training loop projects many weight matrices after every step (the use Sec. 6.3 makes of
// the projection), most of them small enough that the three launches of a call are what it
// costs.  Up to BATCH_MAX matrices share one aggregate, one fold and one map launch: the
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
  reduce_body<Q>(ws.partial, b.m, g, reduce_parts(g.groups), ws.v, b.v_out, ws.flags, bid);
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
  if (b.wide && b.x_vec)
    colmap_body<Q, T, WIDE, false, true, SC>(Y, X, b.n, b.m, g, ws, b.u_out, b.mask_out, b.eta, outer, bid);
  else if (b.wide)
    colmap_body<Q, T, WIDE, false, false, SC>(Y, X, b.n, b.m, g, ws, b.u_out, b.mask_out, b.eta, outer, bid);
  else
    colmap_body<Q, T, WIDE, true, false, SC>(Y, X, b.n, b.m, g, ws, b.u_out, b.mask_out, b.eta, outer, bid);
}

}  // namespace mlproj

#endif
