// mlproj: the aggregate pass over columns (v_j = ||y_j||_q, Sec. 3) and the fold of its partials.
#ifndef MLPROJ_AGGREGATE_H
#define MLPROJ_AGGREGATE_H

#include "common.h"
#include "reduce.h"

namespace mlproj {

template <int Q> struct AccOf { using type = double; };
template <> struct AccOf<QINF> { using type = float; };

template <int Q>
__device__ __forceinline__ void accumulate(typename AccOf<Q>::type& a, float y) {
  if constexpr (Q == QINF) a = fmaxf(a, fabsf(y));
  else if constexpr (Q == Q1) a += (double)fabsf(y);
  else a = fma((double)y, (double)y, a);
}
template <int Q>
__device__ __forceinline__ typename AccOf<Q>::type combine(typename AccOf<Q>::type a,
                                                           typename AccOf<Q>::type b) {
  if constexpr (Q == QINF) return fmaxf(a, b);
  else return a + b;
}

// ------------------------------------------------------------------ column aggregate
// Partial column aggregates of v_j = ||y_j||_q (Sec. 3): max |.| (exact), sum |.| or sum of
// squares (both in fp64).  Every lane owns VEC columns of the tile (see LaneCols); the four
// wavefronts of a workgroup take rows r, r+1, r+2, r+3 (mod 4) of each row block.
// `bid` is the workgroup's number within its own problem (blockIdx.x for a single matrix).
// DIRECT (only with one row group per tile, so that a workgroup's partial is the whole column):
// the workgroup writes v_j (and v_out) itself and workgroup 0 clears the meeting area of the
// grid-wide search, which is all the fold kernel would have done; the host then skips that launch.
// The partial array, which has nothing else to hold then, gets three numbers per tile: the sum,
// the sum of squares and the maximum of the tile's v_j.
template <int Q, typename T, int VEC, bool STRIDED, bool DIRECT = false>
__device__ __forceinline__ void colagg_body(const T* __restrict__ Y, long long n, long long m,
                                            const Geometry& g, void* __restrict__ partial_,
                                            long long bid, double* __restrict__ v = nullptr,
                                            float* __restrict__ v_out = nullptr,
                                            unsigned* __restrict__ flags = nullptr) {
  using Acc = typename AccOf<Q>::type;
  constexpr int TILE_W = WAVE * VEC;
  __shared__ Acc sm[WAVES][TILE_W];

  const int lane = threadIdx.x & (WAVE - 1);
  const int wave = threadIdx.x / WAVE;
  const long long t = bid % g.tiles;
  const long long grp = bid / g.tiles;
  const LaneCols<T, VEC, STRIDED> lc(t * TILE_W, lane, m);

  Acc acc[VEC];
#pragma unroll
  for (int k = 0; k < VEC; ++k) acc[k] = (Acc)0;

  if (lc.any()) {
    long long r0 = grp * RBLK;
    for (; r0 + RBLK <= n; r0 += g.groups * RBLK) {
      Pack<T, VEC> x[UNROLL];
#pragma unroll
      for (int r = 0; r < UNROLL; ++r) lc.load(Y + (r0 + wave + (long long)r * WAVES) * m, x[r]);
#pragma unroll
      for (int r = 0; r < UNROLL; ++r)
#pragma unroll
        for (int k = 0; k < VEC; ++k) accumulate<Q>(acc[k], (float)x[r].e[k]);
    }
    for (long long i = r0 + wave; i < n; i += WAVES) {  // the one ragged block at the bottom
      Pack<T, VEC> x;
      lc.load(Y + i * m, x);
#pragma unroll
      for (int k = 0; k < VEC; ++k) accumulate<Q>(acc[k], (float)x.e[k]);
    }
  }
#pragma unroll
  for (int k = 0; k < VEC; ++k) sm[wave][lc.slot(lane, k)] = acc[k];
  __syncthreads();
  double st_sum = 0.0, st_sq = 0.0, st_max = 0.0;   // DIRECT: sum, sum of squares and maximum of the tile's v_j
  for (int c = threadIdx.x; c < TILE_W; c += WG) {
    Acc a = sm[0][c];
#pragma unroll
    for (int w = 1; w < WAVES; ++w) a = combine<Q>(a, sm[w][c]);
    if constexpr (DIRECT) {
      const long long j = t * TILE_W + c;
      if (j < m) {
        const double vj = (Q == Q2) ? sqrt((double)a) : (double)a;
        v[j] = vj;
        if (v_out) v_out[j] = (float)vj;
        st_sum += vj;
        st_sq = fma(vj, vj, st_sq);
        st_max = fmax(st_max, vj);
      }
    } else {
      static_cast<Acc*>(partial_)[((size_t)t * g.groups + grp) * TILE_W + c] = a;
    }
  }
  if constexpr (DIRECT) {
    if (bid == 0) clear_meeting_area(flags);
    // The tile's share of sum v, sum v^2 and max v, folded in a fixed order: with them the search
    // over very many columns knows the totals (and a starting guess) before its first exchange.
    __shared__ PairScratch<WAVES> st;
    block_sum_max(st_sum, st_max, st);
    double none = 0.0;
    block_sum_max(st_sq, none, st);
    if (threadIdx.x == 0) {
      double* out = static_cast<double*>(partial_) + 3 * (size_t)t;
      out[0] = st_sum;
      out[1] = st_sq;
      out[2] = st_max;
    }
  }
}

template <int Q, typename T, int VEC, bool STRIDED>
__global__ __launch_bounds__(WG) void colagg_kernel(const T* __restrict__ Y, long long n,
                                                    long long m, Geometry g,
                                                    void* __restrict__ partial_) {
  colagg_body<Q, T, VEC, STRIDED>(Y, n, m, g, partial_, blockIdx.x);
}

// One row group per tile (a wide or very short matrix): the aggregate pass finishes v itself.
template <int Q, typename T, int VEC, bool STRIDED>
__global__ __launch_bounds__(WG) void colagg_direct_kernel(const T* __restrict__ Y, long long n,
                                                           long long m, Geometry g,
                                                           void* __restrict__ tile_stats,
                                                           double* __restrict__ v,
                                                           float* __restrict__ v_out,
                                                           unsigned* __restrict__ flags) {
  colagg_body<Q, T, VEC, STRIDED, true>(Y, n, m, g, tile_stats, blockIdx.x, v, v_out, flags);
}

// v_j from the partials of its tile, folded in a fixed order.  A workgroup of NT threads
// covers NT/parts groups with `parts` threads each (parts = 1..NT/64, a power of two chosen on
// the host from the number of partials per group); every thread keeps 8 loads in flight.
// Serves columns (tile_w = 64*vec) and slabs (tile_w = 1) alike.
// NT = 1024 or 256.  The kernel is a launch, one load latency and a fold, so for 16 to 64
// partials per group four wavefronts with a few loads each are in and out sooner than sixteen
// (4096 x 4096: 37.2 -> 36.7 us per projection, 25.1 -> 24.3 on bf16 storage); with hundreds of
// partials per group (a tall matrix) the sixteen shorter chains win (130 against 133 us).
template <int Q, int NT = SWG>
__device__ __forceinline__ void reduce_body(const void* __restrict__ partial_, long long ngroups,
                                            const Geometry& g, int parts, double* __restrict__ v,
                                            float* __restrict__ v_out,
                                            unsigned* __restrict__ flags, long long bid) {
  using Acc = typename AccOf<Q>::type;
  __shared__ Acc sm[NT];
  if (bid == 0) clear_meeting_area(flags);  // for the grid-wide search
  const int cols = NT / parts;
  const int c_local = threadIdx.x % cols;
  const int part = threadIdx.x / cols;
  const long long j = bid * cols + c_local;
  Acc a = (Acc)0;
  if (j < ngroups) {
    const long long t = j / g.tile_w, c = j % g.tile_w;
    const Acc* q = static_cast<const Acc*>(partial_) + (size_t)t * g.groups * g.tile_w + c;
    const size_t stride = (size_t)g.tile_w;
    long long b0 = part;
    for (; b0 + 7LL * parts < g.groups; b0 += 8LL * parts) {
      Acc x[8];
#pragma unroll
      for (int r = 0; r < 8; ++r) x[r] = q[(size_t)(b0 + (long long)r * parts) * stride];
#pragma unroll
      for (int r = 0; r < 8; ++r) a = combine<Q>(a, x[r]);
    }
    for (; b0 < g.groups; b0 += parts) a = combine<Q>(a, q[(size_t)b0 * stride]);
  }
  sm[threadIdx.x] = a;
  __syncthreads();
  if (part == 0 && j < ngroups) {
    for (int w = 1; w < parts; ++w) a = combine<Q>(a, sm[w * cols + c_local]);
    const double vj = (Q == Q2) ? sqrt((double)a) : (double)a;
    v[j] = vj;
    if (v_out) v_out[j] = (float)vj;
  }
}

template <int Q, int NT = SWG>
__global__ __launch_bounds__(NT) void reduce_kernel(const void* __restrict__ partial_,
                                                     long long ngroups, Geometry g, int parts,
                                                     double* __restrict__ v,
                                                     float* __restrict__ v_out,
                                                     unsigned* __restrict__ flags) {
  reduce_body<Q, NT>(partial_, ngroups, g, parts, v, v_out, flags, blockIdx.x);
}

}  // namespace mlproj

#endif
