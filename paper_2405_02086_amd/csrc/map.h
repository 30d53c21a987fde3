// mlproj: the map pass over columns (x_j = P^q_{u_j}(y_j), Eq. 8-9).
#ifndef MLPROJ_MAP_H
#define MLPROJ_MAP_H

#include "common.h"
#include "reduce.h"
#include "search.h"

namespace mlproj {

// ------------------------------------------------------------------ per-column map
// x_j = P^q_{u_j}(y_j) (Eq. 8-9) with u_j = max(v_j - tau, 0) (tau w_j for a weighted l1 ball):
//   q = inf : X = sign(Y) min(|Y|, u_j)          (the symmetric clip; Sec. 4.1)
//   q = 2   : X = Y * u_j / v_j
//   q = 1   : X = sign(Y) max(|Y| - tau_j, 0)    with tau_j from the inner searches
// Row blocks are visited from the bottom up, the reverse of the aggregate pass, so the rows
// read last there (the ones most likely still cached) are read first here.
// With fused_eta >= 0 every workgroup first runs the threshold search itself (see
// search_block) and workgroup 0 files the result record; otherwise tau is read from it.
// `bid` is the workgroup's number within its own problem (blockIdx.x for a single matrix).
template <int Q, typename T, int VEC, bool STRIDED, bool XVEC, int SC>
__device__ __forceinline__ void colmap_body(const T* Y, T* X, long long n, long long m,
                                            const Geometry& g, const Ws& ws,
                                            float* __restrict__ u_out,
                                            unsigned char* __restrict__ mask_out,
                                            double fused_eta, int outer, long long bid) {
  constexpr int TILE_W = WAVE * VEC;
  constexpr int U = MAP_UNROLL;
  __shared__ PairScratch<WAVES> bs;
  const int lane = threadIdx.x & (WAVE - 1);
  const int wave = threadIdx.x / WAVE;
  const long long t = bid % g.tiles;
  const long long grp = bid / g.tiles;
  const LaneCols<T, VEC, STRIDED> lc(t * TILE_W, lane, m);
  const bool col_ok = lc.any();

  // Row blocks of MAP_RBLK rows, bottom block first; the last block may be ragged.
  const long long nblk = (n + MAP_RBLK - 1) / MAP_RBLK;
  long long b = nblk - 1 - grp;
  // The two buffers hold the elements as stored: widening them here would put a use of the
  // loaded values, and with it the wait for them, ahead of the stores of the current block.
  Pack<T, VEC> x[U], y[U];
  auto load_block = [&](long long blk, Pack<T, VEC> (&dst)[U]) {
#pragma unroll
    for (int r = 0; r < U; ++r) {
      const long long row = blk * MAP_RBLK + wave + (long long)r * WAVES;
      if (row < n) lc.load(Y + row * m, dst[r]);
    }
  };
  // The first block is requested before tau is known, so its latency hides the search.
  if (col_ok && b >= 0) load_block(b, x);

  Top top;
  bool inside;
  if (fused_eta >= 0.0) {
    const SearchOut o = search_block<WG, SC>(ws.v, m, fused_eta, MODE_PROJECT, outer, bs);
    top = top_of(o);
    inside = o.inside != 0u;
    if (bid == 0 && threadIdx.x == 0) write_result(ws, o, nullptr);
  } else {
    top = top_of(ws.res);
    inside = ws.res->inside_ball != 0u;
  }
  if constexpr (Q == Q1) {
    // A tile whose columns are all dropped (with sparse results most tiles are) is zeroed
    // without reading the rest of it.
    if (!inside) {
      bool kept = false;
#pragma unroll
      for (int k = 0; k < VEC; ++k)
        if (lc.ok[k]) kept = kept || radius_of(ws, lc.col(k), ws.v[lc.col(k)], top) > 0.0;
      if (!__syncthreads_or(kept ? 1 : 0)) {
        if (grp == 0 && wave == 0) {
#pragma unroll
          for (int k = 0; k < VEC; ++k) {
            if (lc.ok[k] && u_out) u_out[lc.col(k)] = 0.0f;
            if (lc.ok[k] && mask_out) mask_out[lc.col(k)] = 0;
          }
        }
        if (col_ok) {
          float zero[VEC];
#pragma unroll
          for (int k = 0; k < VEC; ++k) zero[k] = 0.0f;
          for (; b >= 0; b -= g.map_groups) {
#pragma unroll
            for (int r = 0; r < U; ++r) {
              const long long row = b * MAP_RBLK + wave + (long long)r * WAVES;
              if (row < n) lc.template store_nt<XVEC>(X + row * m, zero);
            }
          }
        }
        return;
      }
    }
  }
  if (!col_ok) return;

  float uf[VEC];
  double par[VEC];  // q = 2: scale u_j / v_j;  q = 1: inner threshold tau_j
#pragma unroll
  for (int k = 0; k < VEC; ++k) {
    const double vj = lc.ok[k] ? ws.v[lc.col(k)] : 0.0;
    const double uj = lc.ok[k] ? radius_of(ws, lc.col(k), vj, top) : 0.0;
    uf[k] = (float)uj;
    if constexpr (Q == Q2) par[k] = vj > 0.0 ? uj / vj : 0.0;
    else if constexpr (Q == Q1) par[k] = inside ? 0.0 : ((uj > 0.0 && lc.ok[k]) ? ws.tauj[lc.col(k)] : HUGE_VAL);
    else par[k] = 0.0;
  }
  // q = 1: tau_j as an unevaluated fp32 pair, tau_j = th + tl to 2^-48 relative.  |y| - th is
  // exact while |y| <= 2 th (the only place cancellation can occur) and carries one fp32
  // rounding beyond that, so (|y| - th) - tl stays within two fp32 units of the fp64 result.
  float th[VEC], tl[VEC];
#pragma unroll
  for (int k = 0; k < VEC; ++k) {
    th[k] = (float)par[k];
    tl[k] = (Q == Q1 && par[k] < HUGE_VAL) ? (float)(par[k] - (double)th[k]) : 0.0f;
  }
  if (grp == 0 && wave == 0) {
    if (u_out) {
#pragma unroll
      for (int k = 0; k < VEC; ++k)
        if (lc.ok[k]) u_out[lc.col(k)] = uf[k];
    }
    if (mask_out) {  // the kept columns, decided where the radius is: in fp64
#pragma unroll
      for (int k = 0; k < VEC; ++k)
        if (lc.ok[k]) mask_out[lc.col(k)] = radius_of(ws, lc.col(k), ws.v[lc.col(k)], top) > 0.0 ? 1 : 0;
    }
  }

  auto apply = [&](float yv, int k) -> float {
    if constexpr (Q == QINF) return copysignf(fminf(fabsf(yv), uf[k]), yv);
    else if constexpr (Q == Q2) return (float)((double)yv * par[k]);
    else return copysignf(fmaxf((fabsf(yv) - th[k]) - tl[k], 0.0f), yv);
  };

  // Software pipeline: the next block's loads are issued first, then this block is mapped
  // and stored, and only then does the wavefront wait.  On gfx9 loads and stores share one
  // counter, so any wait for a load also waits for every store issued before it: the wait
  // must come after both have been issued, or the two never overlap.
  // A thread reads and writes the same elements only, so X may alias Y.
  for (; b >= 0; b -= g.map_groups) {
    const long long nb = b - g.map_groups;
    if (nb >= 0) load_block(nb, y);
#pragma unroll
    for (int r = 0; r < U; ++r) {
      const long long row = b * MAP_RBLK + wave + (long long)r * WAVES;
      if (row < n) {
        float f[VEC];
#pragma unroll
        for (int k = 0; k < VEC; ++k) f[k] = apply((float)x[r].e[k], k);
        lc.template store_nt<XVEC>(X + row * m, f);
      }
    }
#pragma unroll
    for (int r = 0; r < U; ++r) x[r] = y[r];
  }
}

template <int Q, typename T, int VEC, bool STRIDED, bool XVEC, int SC = SEARCH_CACHE>
__global__ __launch_bounds__(WG) void colmap_kernel(const T* Y, T* X, long long n,
                                                    long long m, Geometry g, Ws ws,
                                                    float* __restrict__ u_out,
                                                    unsigned char* __restrict__ mask_out,
                                                    double fused_eta, int outer) {
  colmap_body<Q, T, VEC, STRIDED, XVEC, SC>(Y, X, n, m, g, ws, u_out, mask_out, fused_eta, outer,
                                            blockIdx.x);
}

}  // namespace mlproj

#endif
