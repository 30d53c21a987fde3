// mlproj: tri-level l1,inf,inf kernels on contiguous slabs (Sec. 5.1).
#ifndef MLPROJ_SLAB_H
#define MLPROJ_SLAB_H

#include "common.h"
#include "reduce.h"
#include "search.h"

namespace mlproj {

// ------------------------------------------------------------------ tri-level: slab kernels
// Groups are the d0 contiguous slabs of len = d1*d2 elements.  w_a = max over the slab equals
// the two nested maxima of Alg. 5 (max over the fibre, then over the fibres of the slab).
template <typename T, int VEC>
__global__ __launch_bounds__(WG) void slabagg_kernel(const T* __restrict__ Y, long long len,
                                                     Geometry g, float* __restrict__ partial) {
  __shared__ BlockScratch<WAVES> bs;
  const long long a = blockIdx.x / g.groups;
  const long long c = blockIdx.x % g.groups;
  const long long lo = c * g.span;
  const long long hi = (lo + g.span < len) ? lo + g.span : len;
  const T* p = Y + a * len;
  float mx = 0.0f;
  long long i = lo + (long long)threadIdx.x * VEC;
  constexpr long long STEP = (long long)WG * VEC;
  for (; i + 3 * STEP < hi; i += 4 * STEP) {
    float x[4][VEC];
#pragma unroll
    for (int r = 0; r < 4; ++r) load_row<VEC>(p + i + r * STEP, x[r]);
#pragma unroll
    for (int r = 0; r < 4; ++r)
#pragma unroll
      for (int k = 0; k < VEC; ++k) mx = fmaxf(mx, fabsf(x[r][k]));
  }
  for (; i < hi; i += STEP) {
    float x[VEC];
    load_row<VEC>(p + i, x);
#pragma unroll
    for (int k = 0; k < VEC; ++k) mx = fmaxf(mx, fabsf(x[k]));
  }
  const double bmax = block_max((double)mx, bs);
  if (threadIdx.x == 0) partial[(size_t)a * g.groups + c] = (float)bmax;
}

// X_abc = sign(Y_abc) min(|Y_abc|, u_a).  The appendix form clips each fibre to
// U2_ab = min(V_ab, u_a); since |Y_abc| <= V_ab the two clips give the same value.
template <typename T, int VEC, bool XVEC>
__global__ __launch_bounds__(WG) void slabmap_kernel(const T* Y, T* X, long long d0,
                                                     long long len, Geometry g, Ws ws,
                                                     float* __restrict__ u_out,
                                                     unsigned char* __restrict__ mask_out,
                                                     double fused_eta) {
  __shared__ PairScratch<WAVES> bs;
  const long long a = d0 - 1 - blockIdx.x / g.groups;
  const long long c = blockIdx.x % g.groups;
  const long long lo = c * g.span;
  const long long hi = (lo + g.span < len) ? lo + g.span : len;
  Top top;
  if (fused_eta >= 0.0) {
    const SearchOut o = search_block<WG>(ws.v, d0, fused_eta, MODE_PROJECT, MLPROJ_OUTER_L1, bs);
    top = top_of(o);
    if (blockIdx.x == 0 && threadIdx.x == 0) write_result(ws, o, nullptr);
  } else {
    top = top_of(ws.res);
  }
  const double ud = radius(ws.v[a], top);
  const float u = (float)ud;
  if (c == 0 && threadIdx.x == 0) {
    if (u_out) u_out[a] = u;
    if (mask_out) mask_out[a] = ud > 0.0 ? 1 : 0;
  }
  const T* p = Y + a * len;
  T* q = X + a * len;
  long long i = lo + (long long)threadIdx.x * VEC;
  constexpr long long STEP = (long long)WG * VEC;
  for (; i + 3 * STEP < hi; i += 4 * STEP) {
    float x[4][VEC];
#pragma unroll
    for (int r = 0; r < 4; ++r) load_row<VEC>(p + i + r * STEP, x[r]);
#pragma unroll
    for (int r = 0; r < 4; ++r) {
#pragma unroll
      for (int k = 0; k < VEC; ++k) x[r][k] = copysignf(fminf(fabsf(x[r][k]), u), x[r][k]);
      store_row_nt<VEC, XVEC>(q + i + r * STEP, x[r]);
    }
  }
  for (; i < hi; i += STEP) {
    float x[VEC];
    load_row<VEC>(p + i, x);
#pragma unroll
    for (int k = 0; k < VEC; ++k) x[k] = copysignf(fminf(fabsf(x[k]), u), x[k]);
    store_row_nt<VEC, XVEC>(q + i, x);
  }
}

}  // namespace mlproj

#endif
