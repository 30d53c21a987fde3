// mlproj: l1,1 without the probing pass: the aggregate pass also evaluates every column on a small
// grid of thresholds, from which the inner searches (Alg. 3) get their first windows.
#ifndef MLPROJ_L11GRID_H
#define MLPROJ_L11GRID_H

#include "aggregate.h"
#include "common.h"
#include "l11.h"
#include "reduce.h"
#include "search.h"

namespace mlproj {

// ------------------------------------------------------------------ l1,1: the grid
// The lock-step inner searches of l11.h open with a pass that evaluates f_j at a guess, only to
// learn where to put the first window.  That pass (a full read of Y) is not needed when the
// aggregate pass, which reads Y anyway, also returns f_j and its slope at a few fixed points:
//   scale     s_j = mean |Y_ij| over the first GRID_SAMPLE_ROWS rows (a tiny kernel; 128 rows put a
//             Gaussian column's estimate within 7 % at one standard deviation);
//   grid      T_ji = s_j * GRID_MULT[i], the same floats for every workgroup of the column;
//   aggregate besides sum_i |Y_ij|: S_ji = sum of the entries above T_ji and their number K_ji,
//             so f_j(T_ji) = S_ji - K_ji T_ji and f_j'(T_ji) = -K_ji, exactly (up to the fp32
//             rounding of the partial sums, which only the model sees);
//   seeding   once u_j is known: the bracket [T_ji, T_j,i+1] with f_j(T_ji) >= u_j >= f_j(T_j,i+1),
//             the root of the cubic through both values with both slopes (off by a handful of
//             entries on smooth data), and a window around it a few dozen entries wide.
// A column whose root lies beyond an end of the grid (tiny or huge radii, heavy tails) gets its
// window from a quadratic model at that end; its first listing pass is then also its probe.  Everything after the seeding is l11.h unchanged: every
// threshold is still closed exactly, whatever the grid said.
constexpr int GRID_PTS = 4;
constexpr int GRID_SAMPLE_ROWS = 128;
__device__ __forceinline__ float grid_mult(int i) {
  // in units of the column's mean magnitude: for Gaussian entries z = 0.48, 1.0, 1.6, 2.4
  return i == 0 ? 0.6f : i == 1 ? 1.25f : i == 2 ? 2.0f : 3.0f;
}
__device__ __forceinline__ float grid_point(float scale, int i) { return scale * grid_mult(i); }

template <typename T>
__global__ __launch_bounds__(WG) void l11_scale_kernel(const T* __restrict__ Y, long long n, long long m,
                                                       float* __restrict__ scale) {
  const long long j = (long long)blockIdx.x * WG + threadIdx.x;
  if (j >= m) return;
  const long long rows = n < GRID_SAMPLE_ROWS ? n : GRID_SAMPLE_ROWS;
  // (the loads of a batch are unconditional, so that all of them are in flight together)
  constexpr int BATCH = 32;
  float s = 0.0f;
  for (int i0 = 0; i0 < GRID_SAMPLE_ROWS && i0 < rows; i0 += BATCH) {
    T x[BATCH];
#pragma unroll
    for (int i = 0; i < BATCH; ++i) x[i] = Y[(i0 + i < rows ? i0 + i : rows - 1) * m + j];
#pragma unroll
    for (int i = 0; i < BATCH; ++i) s += i0 + i < rows ? fabsf((float)x[i]) : 0.0f;
  }
  scale[j] = s / (float)rows;
}

// The aggregate pass of aggregate.h for q = 1 with the grid beside it.  gpart:
// [tile][row group][2 * GRID_PTS][TILE_W] floats (S_0 .. S_3, K_0 .. K_3 of the workgroup's rows).
// Workgroup 0 also clears the sweep counters (the seeding kernel adds to them).
template <typename T, int VEC, bool STRIDED>
__global__ __launch_bounds__(WG) void colagg_grid_kernel(const T* __restrict__ Y, long long n, long long m,
                                                         Geometry g, Ws ws, const float* __restrict__ scale,
                                                         float* __restrict__ gpart) {
  constexpr int TILE_W = WAVE * VEC;
  __shared__ double sm[WAVES][TILE_W];
  __shared__ float smf[WAVES][TILE_W];
  const int lane = threadIdx.x & (WAVE - 1);
  const int wave = threadIdx.x / WAVE;
  const long long t = blockIdx.x % g.tiles;
  const long long grp = blockIdx.x / g.tiles;
  const LaneCols<T, VEC, STRIDED> lc(t * TILE_W, lane, m);
  if (blockIdx.x == 0 && threadIdx.x <= MAX_INNER_SWEEPS) ws.pending[threadIdx.x] = 0u;

  double acc[VEC];
  float S[VEC][GRID_PTS], P[VEC][GRID_PTS];
  unsigned K[VEC][GRID_PTS];
#pragma unroll
  for (int k = 0; k < VEC; ++k) {
    acc[k] = 0.0;
    const float sc = lc.ok[k] ? scale[lc.col(k)] : 0.0f;
#pragma unroll
    for (int i = 0; i < GRID_PTS; ++i) { S[k][i] = 0.0f; K[k][i] = 0u; P[k][i] = grid_point(sc, i); }
  }
  auto visit = [&](float y, int k) {
    const float a = fabsf(y);
    acc[k] += (double)a;
#pragma unroll
    for (int i = 0; i < GRID_PTS; ++i) {
      const bool in = a > P[k][i];
      S[k][i] += in ? a : 0.0f;
      K[k][i] += in ? 1u : 0u;
    }
  };
  if (lc.any()) {
    long long r0 = grp * RBLK;
    for (; r0 + RBLK <= n; r0 += g.groups * RBLK) {
      Pack<T, VEC> x[UNROLL];
#pragma unroll
      for (int r = 0; r < UNROLL; ++r) lc.load(Y + (r0 + wave + (long long)r * WAVES) * m, x[r]);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int r = 0; r < UNROLL; ++r)
#pragma unroll
        for (int k = 0; k < VEC; ++k) visit((float)x[r].e[k], k);
    }
    for (long long i = r0 + wave; i < n; i += WAVES) {  // the one ragged block at the bottom
      Pack<T, VEC> x;
      lc.load(Y + i * m, x);
#pragma unroll
      for (int k = 0; k < VEC; ++k) visit((float)x.e[k], k);
    }
  }
  // the column sums, folded over the four wavefronts exactly as colagg_body does
#pragma unroll
  for (int k = 0; k < VEC; ++k) sm[wave][lc.slot(lane, k)] = acc[k];
  __syncthreads();
  const size_t cell0 = ((size_t)t * g.groups + grp) * TILE_W;
  for (int c = threadIdx.x; c < TILE_W; c += WG) {
    double a = sm[0][c];
#pragma unroll
    for (int w = 1; w < WAVES; ++w) a += sm[w][c];
    static_cast<double*>(ws.partial)[cell0 + c] = a;
  }
  // the grid values, one at a time through one small LDS array
  float* out = gpart + cell0 * (2 * GRID_PTS);
#pragma unroll
  for (int q = 0; q < 2 * GRID_PTS; ++q) {
    __syncthreads();
#pragma unroll
    for (int k = 0; k < VEC; ++k)
      smf[wave][lc.slot(lane, k)] = q < GRID_PTS ? S[k][q] : (float)K[k][q - GRID_PTS];
    __syncthreads();
    for (int c = threadIdx.x; c < TILE_W; c += WG) {
      float a = smf[0][c];
#pragma unroll
      for (int w = 1; w < WAVES; ++w) a += smf[w][c];
      out[(size_t)q * TILE_W + c] = a;
    }
  }
}

// Root in [0, 1] of the cubic with values fa >= 0 >= fb and slopes da, db (per unit of s) at the
// ends: bisection (the cubic need not be monotone when the data are rough; any root will do).
__device__ __forceinline__ double hermite_root(double fa, double fb, double da, double db) {
  double lo = 0.0, hi = 1.0;
  for (int it = 0; it < 32; ++it) {
    const double s = 0.5 * (lo + hi);
    const double s2 = s * s, s3 = s2 * s;
    const double p = (2.0 * s3 - 3.0 * s2 + 1.0) * fa + (s3 - 2.0 * s2 + s) * da + (-2.0 * s3 + 3.0 * s2) * fb + (s3 - s2) * db;
    if (p > 0.0) lo = s; else hi = s;
  }
  return 0.5 * (lo + hi);
}

// The seeding kernel of l11.h (l11_init_body) for a call whose aggregate pass filled the grid:
// the outer search as there, then for every kept column the first window from the grid.  The
// sweep counters were cleared by the aggregate pass; the open columns are counted into
// pending[1], as the update kernel of the probing pass would have done.
template <int SC>
__global__ __launch_bounds__(WG) void l11_init_grid_kernel(long long n, long long m, Geometry g, Ws ws,
                                                           double fused_eta, int outer,
                                                           const float* __restrict__ scale,
                                                           const float* __restrict__ gpart) {
  __shared__ PairScratch<WAVES> bs;
  __shared__ BlockScratch<WAVES> cs;
  Top top;
  bool nothing_to_do;
  if (fused_eta >= 0.0) {
    const SearchOut o = search_block<WG, SC>(ws.v, m, fused_eta, MODE_PROJECT, outer, bs);
    top = top_of(o);
    nothing_to_do = o.inside != 0u || o.active == 0u;
    if (blockIdx.x == 0 && threadIdx.x == 0) write_result(ws, o, nullptr);
  } else {
    const mlproj_result* res = ws.res;
    top = top_of(res);
    nothing_to_do = res->inside_ball != 0u || res->n_active == 0u;
  }
  if (nothing_to_do) return;
  const long long j = (long long)blockIdx.x * WG + threadIdx.x;
  unsigned open = 0u;
  if (j < m) {
    const double vj = ws.v[j];
    const double uj = radius_of(ws, j, vj, top);
    double lo = HUGE_VAL, hi = HUGE_VAL, floor_t = HUGE_VAL;
    if (uj > 0.0) {
      open = 1u;
      const double guess = l11_guess(vj, uj, n, floor_t);
      lo = hi = guess;
      // fold the column's grid partials (fp64: the counts are exact)
      const long long tl = j / g.tile_w, c = j % g.tile_w;
      const float* p = gpart + (size_t)tl * g.groups * g.tile_w * (2 * GRID_PTS) + c;
      double S[GRID_PTS], K[GRID_PTS];
#pragma unroll
      for (int i = 0; i < GRID_PTS; ++i) { S[i] = 0.0; K[i] = 0.0; }
      // (four row groups' worth of loads in flight at a time)
      const size_t step = (size_t)g.tile_w * (2 * GRID_PTS);
      long long b = 0;
      for (; b + 4 <= g.groups; b += 4) {
        float x[4][2 * GRID_PTS];
#pragma unroll
        for (int r = 0; r < 4; ++r)
#pragma unroll
          for (int i = 0; i < 2 * GRID_PTS; ++i) x[r][i] = p[(size_t)(b + r) * step + (size_t)i * g.tile_w];
#pragma unroll
        for (int r = 0; r < 4; ++r)
#pragma unroll
          for (int i = 0; i < GRID_PTS; ++i) { S[i] += (double)x[r][i]; K[i] += (double)x[r][GRID_PTS + i]; }
      }
      for (; b < g.groups; ++b) {
#pragma unroll
        for (int i = 0; i < GRID_PTS; ++i) {
          S[i] += (double)p[(size_t)b * step + (size_t)i * g.tile_w];
          K[i] += (double)p[(size_t)b * step + (size_t)(GRID_PTS + i) * g.tile_w];
        }
      }
      const float sc = scale[j];
      double Tp[GRID_PTS], F[GRID_PTS];
      int last = -1;   // the last grid point with f_j >= u_j
#pragma unroll
      for (int i = 0; i < GRID_PTS; ++i) {
        Tp[i] = (double)grid_point(sc, i);
        F[i] = (S[i] - K[i] * Tp[i]) - uj;
        if (F[i] >= 0.0 && last == i - 1) last = i;
      }
      if (sc > 0.0f && last >= 0 && last < GRID_PTS - 1) {
        // (selected without indexing the arrays by a variable, which would send them to scratch memory)
        double a = 0.0, b = 0.0, fa = 0.0, fb = 0.0, ka = 0.0, kb = 0.0;
#pragma unroll
        for (int i = 0; i < GRID_PTS - 1; ++i)
          if (i == last) { a = Tp[i]; b = Tp[i + 1]; fa = F[i]; fb = F[i + 1]; ka = K[i]; kb = K[i + 1]; }
        const double width = b - a;
        const double inside = ka - kb;          // entries in the bracket
        if (width > 0.0 && fb <= 0.0 && inside >= 1.0) {
          const double that = a + width * hermite_root(fa, fb, -ka * width, -kb * width);
          const double rho = inside / width;
          const double delta = (12.0 + 0.35 * sqrt(inside)) / rho;
          lo = fmax(fmax(that - delta, a), floor_t);
          hi = fmin(that + delta, b);
        }
      } else if (sc > 0.0f) {
        // The root lies beyond an end of the grid (the scale estimate was off, or the radius is
        // very small or very large).  To the right the entries above the last point are a tail:
        // with K of them and mean excess e = f_j(T) / K an exponential tail has
        // f_j(T + d) = K e exp(-d / e), so d = e ln(f_j(T) / u_j) and the density at the root is
        // u_j / e^2 (exact for Laplace entries, a slight overshoot for Gaussian ones, which the
        // error bar covers).  To the left value, slope and the first bracket's density give a
        // quadratic model, as the probing pass would have had at its guess.
        const bool right = last == GRID_PTS - 1;
        double that = 0.0, delta = 0.0, rho = 0.0, d = 0.0;
        if (right) {
          const double kb = K[GRID_PTS - 1];
          const double f_raw = F[GRID_PTS - 1] + uj;      // f_j at the last point
          if (kb > 0.0 && f_raw > uj) {
            const double e = f_raw / kb;
            d = e * log(f_raw / uj);
            rho = uj / (e * e);
          }
        } else {
          const double kb = K[0];
          const double near_w = Tp[1] - Tp[0], near_n = K[0] - K[1];
          if (kb > 0.0 && near_w > 0.0 && near_n >= 1.0) {
            rho = near_n / near_w;
            d = model_step(F[0], kb, rho);
          }
        }
        if (rho > 0.0) {
          const double base = right ? Tp[GRID_PTS - 1] : Tp[0];
          that = base + d;
          delta = 0.25 * fabs(d) + (12.0 + 0.35 * sqrt(rho * fabs(d))) / rho;
          lo = fmax(fmax(that - delta, right ? base : 0.0), floor_t);
          hi = right ? that + delta : fmin(that + delta, base);
        }
      }
      hi = fmax(hi, lo);
      hi = fmin(hi, 2.0 * lo);   // (a window stays within a factor 2: see l11.h)
      if (!(lo > 0.0) || !(hi < HUGE_VAL)) lo = hi = guess;
    }
    ws.tauj[j] = hi;
    ws.tlo[j] = lo;
    ws.lb[j] = floor_t;
    ws.ub[j] = HUGE_VAL;
    ws.kprev[j] = NO_COUNT;
    ws.done[j] = uj > 0.0 ? 0u : 1u;
    ws.gcnt[j] = 0u;
  }
  const unsigned wg_open = block_sum_u(open, cs);
  if (threadIdx.x == 0) {
    if (wg_open) atomicAdd(&ws.pending[1], wg_open);
    if (blockIdx.x == 0) ws.res->inner_sweeps = 1u;
  }
}

}  // namespace mlproj

#endif
