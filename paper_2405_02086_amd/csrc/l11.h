// mlproj: per-column threshold searches of the bi-level l1,1 projection (Alg. 3).
#ifndef MLPROJ_L11_H
#define MLPROJ_L11_H

#include "common.h"
#include "reduce.h"
#include "search.h"

namespace mlproj {

// ------------------------------------------------------------------ l1,1: inner searches
// Alg. 3 needs, for every kept column, the threshold tau_j with
// f_j(tau_j) = sum_i max(|Y_ij| - tau_j, 0) = u_j.  f_j is convex, decreasing and piecewise
// linear.  One pass over Y gives every column the sum S and count K of its entries above a
// point t, i.e. f_j(t) = S - K t and its slope -K; the Newton step N(t) = (S - u_j)/K lands at
// or left of the root from ANY t (the tangent of a convex function lies below it).
// All columns step in lock step, a pass over Y and then a small update kernel per sweep:
//   sweep 0  evaluates a guess g (l11_init_kernel) and counts the entries in (g, g(1+1/16)]:
//            value, slope and density give a quadratic model of f_j, whose root t is the
//            estimate, with an error bar delta from the size of the move and the density;
//   sweep s  evaluates hi = t + delta and LISTS the entries in the window (lo, hi],
//            lo = t - delta (l11_filter_kernel).  With the few listed entries f_j is known on
//            the whole window: if f_j(lo) >= u_j >= f_j(hi) the root is found among them
//            exactly, in fp64, as in the outer search.  Otherwise the evaluated points tighten
//            the certified bounds lb <= tau_j <= ub (Newton steps from below, points with
//            f_j <= u_j from above) and the model gives the next window.
// A column is also closed when the count at a Newton point N(p) equals the count at p (no
// entry between them: f_j is linear there and N(p) is the root), or when the bounds meet.
// On Gaussian data two sweeps close every column; heavy tails take a few more.
// pending[s] is the number of columns still open before sweep s; the kernels of a sweep
// return at once when it is zero, or at most `handoff`: the host sets that to a few hundred
// when a sweep costs more than finishing that many stragglers column by column.  Only a few
// sweeps are enqueued (see plan_l11 on the host side); columns still open after them go to
// the finishing pass (l11_finish_kernel).
//
// A window is kept within a factor 2 (hi <= 2 lo), so its entries differ by at most one
// binary exponent and any fp64 sum of them is exact: the order in which workgroups append
// to a column's list does not reach the result, which stays bit-reproducible.

// The smallest float strictly above t: a float a satisfies a > t exactly when a >= above(t).
__device__ __forceinline__ float above(double t) {
  float f = (float)t;
  if ((double)f <= t) f = nextafterf(f, INFINITY);
  return f;
}

// True for every thread of the workgroup when at least one column of its tile is still open.  A
// tile whose columns are all closed (dropped columns are closed from the start: with sparse
// results most tiles are) needs nothing from a sweep: the update kernel reads the partial sums
// of open columns only.
template <typename LC, int VEC>
__device__ __forceinline__ bool tile_has_open_column(const LC& lc, const Ws& ws) {
  bool any = false;
#pragma unroll
  for (int k = 0; k < VEC; ++k)
    if (lc.ok[k]) any = any || ws.done[lc.col(k)] == 0u;
  return __syncthreads_or(any ? 1 : 0) != 0;
}

// Sweep 0: sum and count of the entries above t = tauj, count above t*(1 + L11_WINDOW).
// (`bid` is the workgroup's number within its own problem: blockIdx.x for a single matrix.
// The LDS arrays belong to the kernel, so that a kernel which holds both access forms of a
// body pays for them once.)
template <int TILE_W>
struct SweepLds {
  double sum[WAVES][TILE_W];
  unsigned cnt[WAVES][TILE_W];
  unsigned cnt2[WAVES][TILE_W];
};

template <typename T, int VEC, bool STRIDED>
__device__ __forceinline__ void l11_sweep_body(const T* __restrict__ Y, long long n, long long m,
                                               const Geometry& g, const Ws& ws, long long bid,
                                               SweepLds<WAVE * VEC>& lds) {
  constexpr int TILE_W = WAVE * VEC;
  auto& sm_sum = lds.sum;
  auto& sm_cnt = lds.cnt;
  auto& sm_cnt2 = lds.cnt2;

  const mlproj_result* res = ws.res;
  if (res->inside_ball != 0u || res->n_active == 0u) return;

  const int lane = threadIdx.x & (WAVE - 1);
  const int wave = threadIdx.x / WAVE;
  const long long t = bid % g.tiles;
  const long long grp = bid / g.tiles;
  const LaneCols<T, VEC, STRIDED> lc(t * TILE_W, lane, m);
  if (!tile_has_open_column<LaneCols<T, VEC, STRIDED>, VEC>(lc, ws)) return;

  double sum[VEC];
  unsigned cnt[VEC], cnt2[VEC];
#pragma unroll
  for (int k = 0; k < VEC; ++k) { sum[k] = 0.0; cnt[k] = 0u; cnt2[k] = 0u; }

  if (lc.any()) {
    // The entries are fp32 (or narrower), so "a > t" with t in fp64 is "a >= above(t)" in fp32.
    float cj[VEC], cw[VEC];
#pragma unroll
    for (int k = 0; k < VEC; ++k) {
      const double tj = lc.ok[k] ? ws.tauj[lc.col(k)] : HUGE_VAL;
      cj[k] = above(tj);
      cw[k] = above(tj * (1.0 + L11_WINDOW));
    }
    auto visit = [&](float y, int k) {
      const float a = fabsf(y);
      const bool in = a >= cj[k];
      sum[k] += (double)(in ? a : 0.0f);
      cnt[k] += in ? 1u : 0u;
      cnt2[k] += a >= cw[k] ? 1u : 0u;
    };
    long long r0 = grp * RBLK;
    for (; r0 + RBLK <= n; r0 += g.groups * RBLK) {
      Pack<T, VEC> x[UNROLL];
#pragma unroll
      for (int r = 0; r < UNROLL; ++r) lc.load(Y + (r0 + wave + (long long)r * WAVES) * m, x[r]);
      __builtin_amdgcn_sched_barrier(0);  // every load of the block is in flight before the first use
#pragma unroll
      for (int r = 0; r < UNROLL; ++r)
#pragma unroll
        for (int k = 0; k < VEC; ++k) visit((float)x[r].e[k], k);
    }
    for (long long i = r0 + wave; i < n; i += WAVES) {
      Pack<T, VEC> x;
      lc.load(Y + i * m, x);
#pragma unroll
      for (int k = 0; k < VEC; ++k) visit((float)x.e[k], k);
    }
  }
#pragma unroll
  for (int k = 0; k < VEC; ++k) {
    sm_sum[wave][lc.slot(lane, k)] = sum[k];
    sm_cnt[wave][lc.slot(lane, k)] = cnt[k];
    sm_cnt2[wave][lc.slot(lane, k)] = cnt2[k];
  }
  __syncthreads();
  for (int col = threadIdx.x; col < TILE_W; col += WG) {
    double a = sm_sum[0][col];
    unsigned c = sm_cnt[0][col], c2 = sm_cnt2[0][col];
#pragma unroll
    for (int w = 1; w < WAVES; ++w) {
      a += sm_sum[w][col];
      c += sm_cnt[w][col];
      c2 += sm_cnt2[w][col];
    }
    const size_t cell = ((size_t)t * g.groups + grp) * TILE_W + col;
    static_cast<double*>(ws.partial)[cell] = a;
    ws.partial_cnt[cell] = c;
    ws.partial_cnt2[cell] = c2;
  }
}

template <typename T, int VEC, bool STRIDED>
__global__ __launch_bounds__(WG) void l11_sweep_kernel(const T* __restrict__ Y, long long n,
                                                       long long m, Geometry g, Ws ws) {
  __shared__ SweepLds<WAVE * VEC> lds;
  l11_sweep_body<T, VEC, STRIDED>(Y, n, m, g, ws, blockIdx.x, lds);
}

// Sweeps 1, 2, ...: sum and count of the entries above hi = tauj, and the entries in
// (tlo, hi] themselves.  A workgroup stages the window entries of its tile's columns in LDS
// (FILTER_LDS_SLOTS / TILE_W slots per column), then reserves room in each column's list with
// one atomic add per column and copies them out; an entry that finds the staging area full goes
// to the column's list directly.  gcnt ends as the true number of window entries of the column
// whether or not they all fitted the list.
template <int TILE_W>
struct FilterLds {
  double sum[WAVES][TILE_W];
  unsigned cnt[WAVES][TILE_W];
  float staged[FILTER_LDS_SLOTS / TILE_W][TILE_W];   // slot-major: the lanes of a wavefront hit different banks
  unsigned staged_cnt[TILE_W];
};

template <typename T, int VEC, bool STRIDED>
__device__ __forceinline__ void l11_filter_body(const T* __restrict__ Y, long long n, long long m,
                                                const Geometry& g, const Ws& ws, int sweep,
                                                unsigned handoff, long long bid,
                                                FilterLds<WAVE * VEC>& lds) {
  constexpr int TILE_W = WAVE * VEC;
  constexpr int CAPW = FILTER_LDS_SLOTS / TILE_W;
  auto& sm_sum = lds.sum;
  auto& sm_cnt = lds.cnt;
  auto& staged = lds.staged;
  auto& staged_cnt = lds.staged_cnt;

  const mlproj_result* res = ws.res;
  if (res->inside_ball != 0u || res->n_active == 0u) return;
  if (ws.pending[sweep] <= handoff) return;

  const int lane = threadIdx.x & (WAVE - 1);
  const int wave = threadIdx.x / WAVE;
  const long long t = bid % g.tiles;
  const long long grp = bid / g.tiles;
  const LaneCols<T, VEC, STRIDED> lc(t * TILE_W, lane, m);
  if (!tile_has_open_column<LaneCols<T, VEC, STRIDED>, VEC>(lc, ws)) return;

  for (int c = threadIdx.x; c < TILE_W; c += WG) staged_cnt[c] = 0u;
  __syncthreads();

  double sum[VEC];
  unsigned cnt[VEC];
#pragma unroll
  for (int k = 0; k < VEC; ++k) { sum[k] = 0.0; cnt[k] = 0u; }

  if (lc.any()) {
    float chi[VEC], clo[VEC];
#pragma unroll
    for (int k = 0; k < VEC; ++k) {
      chi[k] = lc.ok[k] ? above(ws.tauj[lc.col(k)]) : INFINITY;
      clo[k] = lc.ok[k] ? above(ws.tlo[lc.col(k)]) : INFINITY;
    }
    // One row of the lane's columns.  Window entries are rare, so the row is tested as a
    // whole and the staging code runs only for rows that have one.
    auto visit_row = [&](const float (&y)[VEC]) {
      bool any = false;
#pragma unroll
      for (int k = 0; k < VEC; ++k) {
        const float a = fabsf(y[k]);
        const bool in = a >= chi[k];
        sum[k] += (double)(in ? a : 0.0f);
        cnt[k] += in ? 1u : 0u;
        any |= (a >= clo[k]) != in;   // clo <= chi: "above lo but not above hi"
      }
      if (any) {
#pragma unroll
        for (int k = 0; k < VEC; ++k) {
          const float a = fabsf(y[k]);
          if (a >= clo[k] && !(a >= chi[k])) {
            const int c = lc.slot(lane, k);
            const unsigned slot = atomicAdd(&staged_cnt[c], 1u);
            if (slot < (unsigned)CAPW) {
              staged[slot][c] = a;
            } else {
              // no room left in the workgroup's staging area: straight into the column's list
              // (rare; one global atomic per entry instead of one per column)
              const unsigned off = atomicAdd(&ws.gcnt[lc.col(k)], 1u);
              if (off < (unsigned)ws.list_cap) ws.cand[(size_t)off * (size_t)m + (size_t)lc.col(k)] = a;
            }
          }
        }
      }
    };
    long long r0 = grp * RBLK;
    for (; r0 + RBLK <= n; r0 += g.groups * RBLK) {
      Pack<T, VEC> x[UNROLL];
#pragma unroll
      for (int r = 0; r < UNROLL; ++r) lc.load(Y + (r0 + wave + (long long)r * WAVES) * m, x[r]);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int r = 0; r < UNROLL; ++r) {
        float y[VEC];
#pragma unroll
        for (int k = 0; k < VEC; ++k) y[k] = (float)x[r].e[k];
        visit_row(y);
      }
    }
    for (long long i = r0 + wave; i < n; i += WAVES) {
      Pack<T, VEC> x;
      lc.load(Y + i * m, x);
      float y[VEC];
#pragma unroll
      for (int k = 0; k < VEC; ++k) y[k] = (float)x.e[k];
      visit_row(y);
    }
  }
#pragma unroll
  for (int k = 0; k < VEC; ++k) {
    sm_sum[wave][lc.slot(lane, k)] = sum[k];
    sm_cnt[wave][lc.slot(lane, k)] = cnt[k];
  }
  __syncthreads();
  for (int c = threadIdx.x; c < TILE_W; c += WG) {
    double a = sm_sum[0][c];
    unsigned k = sm_cnt[0][c];
#pragma unroll
    for (int w = 1; w < WAVES; ++w) {
      a += sm_sum[w][c];
      k += sm_cnt[w][c];
    }
    const size_t cell = ((size_t)t * g.groups + grp) * TILE_W + c;
    static_cast<double*>(ws.partial)[cell] = a;
    ws.partial_cnt[cell] = k;
    const long long col = t * TILE_W + c;
    const unsigned seen = staged_cnt[c];
    const unsigned r = seen < (unsigned)CAPW ? seen : (unsigned)CAPW;   // (the rest went to the list directly)
    if (col < m && r > 0u) {
      const unsigned off = atomicAdd(&ws.gcnt[col], r);
      for (unsigned s = 0; s < r && off + s < (unsigned)ws.list_cap; ++s)
        ws.cand[(size_t)(off + s) * (size_t)m + (size_t)col] = staged[s][c];
    }
  }
}

template <typename T, int VEC, bool STRIDED>
__global__ __launch_bounds__(WG) void l11_filter_kernel(const T* __restrict__ Y, long long n,
                                                        long long m, Geometry g, Ws ws,
                                                        int sweep, unsigned handoff) {
  __shared__ FilterLds<WAVE * VEC> lds;
  l11_filter_body<T, VEC, STRIDED>(Y, n, m, g, ws, sweep, handoff, blockIdx.x, lds);
}

// Starting points of the inner searches.  Dropped columns get +inf (every entry maps to 0).
// For a kept column the guess assumes its entries are Gaussian with the scale its l1 norm
// implies: E|y| = sigma*sqrt(2/pi) = v_j/n and E max(|y| - t, 0) = sigma*h(t/sigma) with
// h(z) = 2*phi(z) - z*erfc(z/sqrt 2), so z solves h(z) = (u_j/v_j)*sqrt(2/pi) (a few Newton
// steps on the convex h) and the guess is sigma*z.  Only the speed depends on the guess.
// The first certified bounds: every entry active gives the lower bound (v_j - u_j)/n.
// With fused_eta >= 0 every workgroup first runs the outer threshold search itself (see
// search_block) and workgroup 0 files the result record and clears the sweep counters, which
// takes the one-workgroup search kernel off the critical path; otherwise the record is read.
// The guess for a kept column (see above) and the all-active lower bound.
__device__ __forceinline__ double l11_guess(double vj, double uj, long long n, double& floor_t) {
  // (fp32 is plenty here: the guess is a statistical estimate, off by percents)
  const float c = (float)(uj / vj) * 0.79788456f;  // sqrt(2/pi)
  float z = 0.0f;
  for (int it = 0; it < 8; ++it) {
    const float tail = erfcf(z * 0.70710678f);                  // 2*(1 - Phi(z))
    const float h = 0.79788456f * expf(-0.5f * z * z) - z * tail;
    if (!(tail > 1e-30f)) break;
    z += (h - c) / tail;
  }
  const double sigma = (vj / (double)n) * 1.2533141373155001;   // sqrt(pi/2)
  floor_t = fmax((vj - uj) / (double)n, 0.0);
  return fmax(sigma * (double)z, floor_t);  // never below the all-active bound
}

template <int SC>
__device__ __forceinline__ void l11_init_body(long long n, long long m, const Ws& ws,
                                              double fused_eta, int outer, long long bid) {
  __shared__ PairScratch<WAVES> bs;
  Top top;
  bool nothing_to_do;
  if (fused_eta >= 0.0) {
    const SearchOut o = search_block<WG, SC>(ws.v, m, fused_eta, MODE_PROJECT, outer, bs);
    top = top_of(o);
    nothing_to_do = o.inside != 0u || o.active == 0u;
    if (bid == 0) {
      if (threadIdx.x <= MAX_INNER_SWEEPS) ws.pending[threadIdx.x] = 0u;
      if (threadIdx.x == 0) write_result(ws, o, nullptr);
    }
  } else {
    const mlproj_result* res = ws.res;
    top = top_of(res);
    nothing_to_do = res->inside_ball != 0u || res->n_active == 0u;
  }
  if (nothing_to_do) return;
  const long long j = bid * WG + threadIdx.x;
  if (j >= m) return;
  const double vj = ws.v[j];
  const double uj = radius_of(ws, j, vj, top);
  double tj = HUGE_VAL, floor_t = HUGE_VAL;
  if (uj > 0.0) tj = l11_guess(vj, uj, n, floor_t);
  ws.tauj[j] = tj;
  ws.tlo[j] = tj;
  ws.lb[j] = floor_t;
  ws.ub[j] = HUGE_VAL;
  ws.kprev[j] = NO_COUNT;
  ws.done[j] = uj > 0.0 ? 0u : 1u;
  ws.gcnt[j] = 0u;
}

template <int SC>
__global__ __launch_bounds__(WG) void l11_init_kernel(long long n, long long m, Ws ws,
                                                      double fused_eta, int outer) {
  l11_init_body<SC>(n, m, ws, fused_eta, outer, blockIdx.x);
}

// Root of the local model of f_j - u_j: value fb, slope -kb, entry density rho at the base
// point, fb - kb d + rho d^2 / 2 = 0 for the move d (the root next to the base point, in the
// form that does not cancel); the tangent alone when no density is known.
__device__ __forceinline__ double model_step(double fb, double kb, double rho) {
  const double disc = kb * kb - 2.0 * rho * fb;
  if (rho > 0.0 && disc > 0.0) {
    const double den = kb + sqrt(disc);
    if (den > 0.0) return 2.0 * fb / den;
  }
  return kb > 0.0 ? fb / kb : 0.0;
}

struct Window {
  double lo, hi;
  unsigned kp;  // count at the point whose Newton step is lo, or NO_COUNT
};

// The next window: the model's root +- an error bar (a quarter of the move plus six entries'
// worth of spacing, at most an eighth of the list's capacity), cut to the certified bounds
// [lb, ub] and to a factor 2.  `stuck`: nothing was seen at or below the point: step from lb.
__device__ __forceinline__ Window next_window(double base, double fb, double kb, double rho,
                                              double lb, unsigned k_lb, double ub, bool stuck,
                                              int list_cap) {
  Window w;
  w.kp = NO_COUNT;
  if (stuck) {
    w.lo = w.hi = lb;
    return w;
  }
  const double d = model_step(fb, kb, rho);
  const double t = base + d;
  double delta = 0.25 * fabs(d);
  if (rho > 0.0) delta = fmin(delta + 6.0 / rho, 0.125 * (double)list_cap / rho);
  double lo = t - delta, hi = t + delta;
  if (!(lo > lb)) {
    lo = lb;
    w.kp = k_lb;
  }
  hi = fmax(hi, lo);
  hi = fmin(hi, fmax(ub, lo));
  hi = fmin(hi, 2.0 * lo);
  w.lo = lo;
  w.hi = hi;
  return w;
}

// One segment of UPD_SEG = 16 lanes per column: the lanes split the column's partials and its
// listed window entries (in registers), reduce on the DPP crossbar, and every lane takes the
// same decisions from the same numbers, so the kernel needs no LDS and no barrier.
constexpr int UPD_SEG = 16;
constexpr int UPD_COLS = WG / UPD_SEG;   // columns per workgroup
static_assert(UPD_SEG == LIST_LANES, "the list capacity is planned for this many lanes per column");

__device__ __forceinline__ void l11_update_body(long long n, long long m, const Geometry& g,
                                                const Ws& ws, int sweep, unsigned handoff,
                                                long long bid) {
  __shared__ BlockScratch<WAVES> bs;
  const mlproj_result* res = ws.res;
  if (res->inside_ball != 0u || res->n_active == 0u) return;
  if (sweep > 0 && ws.pending[sweep] <= handoff) return;

  const int part = threadIdx.x % UPD_SEG;
  const int seg_base = (threadIdx.x & (WAVE - 1)) & ~(UPD_SEG - 1);   // first lane of the segment
  const long long j = bid * UPD_COLS + threadIdx.x / UPD_SEG;
  const bool mine = j < m && ws.done[j] == 0u;

  // fold the partial sums and counts of the sweep
  double S = 0.0;
  unsigned K = 0u, K2 = 0u;
  if (mine) {
    const long long t = j / g.tile_w, c = j % g.tile_w;
    const size_t base = (size_t)t * g.groups * g.tile_w + c;
    const double* ps = static_cast<const double*>(ws.partial);
    for (long long b = part; b < g.groups; b += UPD_SEG) {
      S += ps[base + (size_t)b * g.tile_w];
      K += ws.partial_cnt[base + (size_t)b * g.tile_w];
      if (sweep == 0) K2 += ws.partial_cnt2[base + (size_t)b * g.tile_w];
    }
  }
  S = __shfl(seg_sum<UPD_SEG>(S), seg_base);   // one lane's sum for all: the lanes must agree
  K = seg_sum_u<UPD_SEG>(K);
  K2 = seg_sum_u<UPD_SEG>(K2);

  // the listed window entries, split over the lanes
  unsigned r = 0u;
  bool complete = false;
  float mylist[LIST_PER_THREAD];
#pragma unroll
  for (int i = 0; i < LIST_PER_THREAD; ++i) mylist[i] = 0.0f;
  double sc = 0.0;
  if (sweep > 0 && mine) {
    r = ws.gcnt[j];
    complete = r <= (unsigned)ws.list_cap;
    if (complete && r > 0u) {
      // every load is unconditional (a slot past the end re-reads the last entry and is then
      // blanked), so they are all in flight together
#pragma unroll
      for (int i = 0; i < LIST_PER_THREAD; ++i) {
        const unsigned s = (unsigned)part + (unsigned)i * (unsigned)UPD_SEG;
        mylist[i] = ws.cand[(size_t)(s < r ? s : r - 1u) * (size_t)m + (size_t)j];
      }
#pragma unroll
      for (int i = 0; i < LIST_PER_THREAD; ++i) {
        const unsigned s = (unsigned)part + (unsigned)i * (unsigned)UPD_SEG;
        if (s >= r) mylist[i] = 0.0f;
        sc += (double)mylist[i];
      }
    }
  }
  sc = seg_sum<UPD_SEG>(sc);   // exact (see the note on windows above): the same in every lane

  bool closed = false, solving = false;
  double tau = 0.0, uj = 0.0, lo = 0.0, lb = 0.0, ub = 0.0;
  Window w{0.0, 0.0, NO_COUNT};
  if (mine) {
    uj = radius_of(ws, j, ws.v[j], top_of(res));
    const double hi = ws.tauj[j];
    lo = ws.tlo[j];
    lb = ws.lb[j];
    ub = ws.ub[j];
    unsigned k_lb = NO_COUNT;  // count at the point whose Newton step is lb, when lb moved now
    tau = hi;
    w = Window{hi, hi, NO_COUNT};
    const double f_hi = (S - (double)K * hi) - uj;
    const double n_hi = K > 0u ? (S - uj) / (double)K : -HUGE_VAL;
    if (sweep == 0) {
      // evaluated at the guess hi = lo, density from the entries in (hi, hi(1 + 1/16)]
      if (n_hi > lb) { lb = n_hi; k_lb = K; }
      if (f_hi <= 0.0) ub = fmin(ub, hi);
      const double rho = (double)(K - K2) / (hi * L11_WINDOW);
      if (ub <= lb * (1.0 + 1e-12)) { closed = true; tau = lb; }
      else w = next_window(hi, f_hi, (double)K, rho, lb, k_lb, ub, K == 0u, ws.list_cap);
    } else {
      const unsigned k_lo = K + r;  // entries above lo
      double f_lo = 0.0, n_lo = -HUGE_VAL;
      if (complete) {
        const double s_lo = S + sc;
        f_lo = (s_lo - (double)k_lo * lo) - uj;
        if (k_lo > 0u) n_lo = (s_lo - uj) / (double)k_lo;
      }
      if (ws.kprev[j] != NO_COUNT && k_lo == ws.kprev[j]) {
        closed = true;  // lo is the Newton step of a point with the same active set
        tau = lo;
      } else if (K > 0u && fabs(f_hi) <= 1e-13 * (S + uj)) {
        closed = true;  // the Newton step from hi does not move: hi is the root, to rounding
        tau = n_hi;
      } else if (complete && f_lo >= 0.0 && f_hi <= 0.0) {
        closed = true;  // the root is inside the window and every entry of the window is known
        solving = true;
        tau = lo;
      } else {
        if (n_hi > lb) { lb = n_hi; k_lb = K; }
        if (complete && n_lo > lb) { lb = n_lo; k_lb = k_lo; }
        if (f_hi <= 0.0) ub = fmin(ub, hi);
        if (complete && f_lo <= 0.0) ub = fmin(ub, lo);
        if (ub <= lb * (1.0 + 1e-12)) { closed = true; tau = lb; }
        else {
          const double rho = (hi > lo && r > 0u) ? (double)r / (hi - lo) : 0.0;
          const bool from_lo = complete && fabs(f_lo) < fabs(f_hi);
          w = next_window(from_lo ? lo : hi, from_lo ? f_lo : f_hi, (double)(from_lo ? k_lo : K),
                          rho, lb, k_lb, ub, K == 0u && r == 0u, ws.list_cap);
        }
      }
    }
  }

  // The root inside a window whose entries are all listed: the fixed point of the outer
  // search on "entries above hi" (S, K) plus the listed ones, started at lo where f_j >= u_j.
  // The lanes of a wavefront loop together until the last of its columns is done.
  unsigned kp = NO_COUNT;
  for (unsigned round = 0; __any(solving) && round < (unsigned)FILTER_MAX_LIST + 2u; ++round) {
    double sa = 0.0;
    unsigned ka = 0u;
#pragma unroll
    for (int i = 0; i < LIST_PER_THREAD; ++i)
      if ((double)mylist[i] > tau) { sa += (double)mylist[i]; ++ka; }
    sa = seg_sum<UPD_SEG>(sa);   // exact, the same in every lane
    ka = seg_sum_u<UPD_SEG>(ka) + K;
    if (solving) {
      const double tn = ka > 0u ? ((S + sa) - uj) / (double)ka : tau;
      if (ka == kp || ka == 0u) {
        tau = tn;
        solving = false;
      } else {
        kp = ka;
        tau = fmax(tau, tn);
      }
    }
  }

  unsigned open = 0u;
  if (part == 0 && j < m) {
    if (mine) {
      ws.tauj[j] = closed ? tau : w.hi;
      ws.tlo[j] = closed ? tau : w.lo;
      ws.kprev[j] = w.kp;
      ws.lb[j] = lb;
      ws.ub[j] = ub;
      ws.done[j] = closed ? 1u : 0u;
      open = closed ? 0u : 1u;
    }
    ws.gcnt[j] = 0u;
  }
  const unsigned wg_open = block_sum_u(open, bs);
  if (threadIdx.x == 0) {
    if (wg_open) atomicAdd(&ws.pending[sweep + 1], wg_open);
    if (bid == 0) ws.res->inner_sweeps = (unsigned)sweep + 1u;
  }
}

__global__ __launch_bounds__(WG) void l11_update_kernel(long long n, long long m, Geometry g,
                                                        Ws ws, int sweep, unsigned handoff) {
  l11_update_body(n, m, g, ws, sweep, handoff, blockIdx.x);
}

// The finishing pass: whatever the lock-step sweeps left open is closed here, column by
// column, with the plain fixed point of the outer search, tau <- (sum_{|y| > tau} |y| - u_j) /
// #{|y| > tau}, started at the certified lower bound the sweeps reached.  From below the
// iteration rises monotonically and the active count only shrinks, so it ends after at most n
// steps (in practice a handful: the bound is already tight) at the exact root, in fp64.
// A workgroup owns FIN_COLS = 16 neighbouring columns (one 64-byte run of every row) and
// leaves at once when none of them is open; thread (r, c) reads rows r, r + 32, ... of column
// c, the four lanes of a wavefront that share a column add up on the crossbar, the eight
// wavefronts through LDS in a fixed order.  The columns are strided in memory, so this pass
// moves 64 bytes for every 4 it needs from a lone open column: good for stragglers, and no
// worse than a sweep when many neighbouring columns are open.  It replaces a long tail of
// lock-step launches that found nothing to do.
constexpr int FIN_COLS = 16;
constexpr int FIN_WG = 512;                // threads: four workgroups fit a CU, so 1024 are resident at once
constexpr int FIN_WAVES = FIN_WG / WAVE;
constexpr int FIN_ROWS = FIN_WG / FIN_COLS;  // rows one trip of the workgroup covers
constexpr int FIN_UNROLL = 16;             // loads in flight per thread
constexpr int FIN_HELD = 32;               // rows per thread a short matrix keeps in registers
static_assert(FIN_HELD % FIN_UNROLL == 0, "the held rows are loaded in batches of FIN_UNROLL");

static_assert(FIN_COLS == UPD_COLS, "a batch launches both kernels on the same grid");

// HELD: the short-matrix form (n <= FIN_ROWS * FIN_HELD), which keeps its rows in registers.
// When no sweep ran (sweeps == 0) the pass can also stand in for the seeding kernel: with
// seed_eta >= 0 every workgroup runs the outer threshold search itself (SC values of v per
// thread in registers), workgroup 0 files the result record, and the columns' guesses and
// bounds are computed here instead of read: one launch less.
template <typename T, bool HELD, int SC = 1>
__device__ __forceinline__ void l11_finish_body(const T* __restrict__ Y, long long n, long long m,
                                                const Ws& ws, int sweeps, unsigned handoff,
                                                long long bid, double seed_eta = -1.0,
                                                int outer = MLPROJ_OUTER_L1) {
  __shared__ double sm_s[FIN_WAVES][FIN_COLS];
  __shared__ unsigned sm_k[FIN_WAVES][FIN_COLS];
  __shared__ PairScratch<FIN_WAVES> bs;
  mlproj_result* res = ws.res;
  const int c = threadIdx.x % FIN_COLS;
  const int r = threadIdx.x / FIN_COLS;
  const int lane = threadIdx.x & (WAVE - 1);
  const int wave = threadIdx.x / WAVE;
  const long long j = bid * FIN_COLS + c;
  const long long jj = j < m ? j : m - 1;   // a column past the end shadows the last one
  const bool seeded = seed_eta >= 0.0;
  Top top;
  bool mine;
  if (seeded) {
    const SearchOut o = search_block<FIN_WG, SC>(ws.v, m, seed_eta, MODE_PROJECT, outer, bs);
    top = top_of(o);
    if (bid == 0 && threadIdx.x == 0) {
      write_result(ws, o, nullptr);
      res->inner_finished = (o.inside != 0u) ? 0u : o.active;
    }
    if (o.inside != 0u || o.active == 0u) return;
    mine = j < m && radius_of(ws, jj, ws.v[jj], top) > 0.0;
  } else {
    if (res->inside_ball != 0u || res->n_active == 0u) return;
    // (no sweep at all, as planned for short matrices: every kept column is open, with the
    // all-active bound of the seeding kernel to start from)
    int stop = 1;   // the sweep at which the lock-step kernels stopped (see `handoff` there)
    while (stop < sweeps && ws.pending[stop] > handoff) ++stop;
    const unsigned left = sweeps > 0 ? ws.pending[stop] : res->n_active;
    if (bid == 0 && threadIdx.x == 0) res->inner_finished = left;
    if (left == 0u) return;
    top = top_of(res);
    mine = j < m && ws.done[jj] == 0u;
  }
  bool open = mine;
  if (!__syncthreads_or(open ? 1 : 0)) return;

  const double uj = radius_of(ws, jj, ws.v[jj], top);
  // Start: the certified lower bound the sweeps reached.  Without any sweep the first point is
  // the seeding guess instead: the fixed-point step from ANY point lands at or left of the
  // root (see the note at the top), so one evaluation there gives a far better lower bound
  // than the all-active one, and the iteration is monotone from then on.
  double lb, t;
  bool first = sweeps == 0;
  if (seeded) {
    lb = 0.0;
    t = mine ? l11_guess(ws.v[jj], uj, n, lb) : 0.0;
  } else {
    lb = ws.lb[jj];
    t = first ? ws.tauj[jj] : lb;
  }
  unsigned kprev = NO_COUNT;
  const T* col = Y + jj;
  // A short matrix (at most FIN_HELD rows per thread) is read once and iterated in registers.
  constexpr bool in_regs = HELD;
  float held[HELD ? FIN_HELD : 1];
  if constexpr (in_regs) {
    // (in batches of FIN_UNROLL loads: every load needs its own address registers)
#pragma unroll
    for (int u0 = 0; u0 < FIN_HELD; u0 += FIN_UNROLL) {
      T x[FIN_UNROLL];
#pragma unroll
      for (int u = 0; u < FIN_UNROLL; ++u) {
        const long long row = r + (long long)(u0 + u) * FIN_ROWS;
        x[u] = col[(row < n ? row : n - 1) * m];
      }
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int u = 0; u < FIN_UNROLL; ++u)
        held[u0 + u] = r + (long long)(u0 + u) * FIN_ROWS < n ? fabsf((float)x[u]) : 0.0f;   // 0 is never above a threshold
      __builtin_amdgcn_sched_barrier(0);
    }
    // With the rows at hand the column's largest entry costs one fold, and it gives a second
    // certified bound: the largest entry alone already sums to a_max - t, so the root is at
    // least a_max - u_j.  Where the radius is small beside the entries (the sparse results the
    // projection is used for) that bound is next to the root, while the climb from the
    // all-active bound takes a dozen rounds (and the Gaussian guess may lie beyond a_max).
    float hm = 0.0f;
#pragma unroll
    for (int u = 0; u < FIN_HELD; ++u) hm = fmaxf(hm, held[u]);
    hm = fmaxf(hm, __shfl_xor(hm, 16));
    hm = fmaxf(hm, __shfl_xor(hm, 32));
    if (lane < FIN_COLS) sm_s[wave][c] = (double)hm;
    __syncthreads();
    double amax = sm_s[0][c];
#pragma unroll
    for (int w = 1; w < FIN_WAVES; ++w) amax = fmax(amax, sm_s[w][c]);
    __syncthreads();   // (the rows of sm_s are written again in the first round)
    if (amax - uj > lb) lb = amax - uj;
    if (first ? (t <= lb || t >= amax) : true) {
      t = lb;          // the guess is no better than the bound (or beyond every entry): start from the bound
      first = false;
    }
  }
  for (;;) {
    const float ct = above(t);
    double s = 0.0;
    unsigned k = 0u;
    auto visit = [&](T x) {
      const float a = fabsf((float)x);
      const bool in = a >= ct;
      s += (double)(in ? a : 0.0f);
      k += in ? 1u : 0u;
    };
    if constexpr (in_regs) {
#pragma unroll
      for (int u = 0; u < FIN_HELD; ++u) {
        float h = held[u];
        asm volatile("" : "+v"(h));   // keeps the widening to fp64 in the loop: hoisted, it doubles the registers
        const bool in = h >= ct;
        s += (double)(in ? h : 0.0f);
        k += in ? 1u : 0u;
      }
    } else {
      long long i = r;
      for (; i + (long long)(FIN_UNROLL - 1) * FIN_ROWS < n; i += (long long)FIN_UNROLL * FIN_ROWS) {
        T x[FIN_UNROLL];
#pragma unroll
        for (int u = 0; u < FIN_UNROLL; ++u) x[u] = col[(i + (long long)u * FIN_ROWS) * m];
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int u = 0; u < FIN_UNROLL; ++u) visit(x[u]);
      }
      for (; i < n; i += FIN_ROWS) visit(col[i * m]);
    }
    // lanes c, c + 16, c + 32, c + 48 of a wavefront share the column
    s += __shfl_xor(s, 16);
    s += __shfl_xor(s, 32);
    k += __shfl_xor(k, 16);
    k += __shfl_xor(k, 32);
    if (lane < FIN_COLS) {
      sm_s[wave][c] = s;
      sm_k[wave][c] = k;
    }
    __syncthreads();
    double S = sm_s[0][c];
    unsigned K = sm_k[0][c];
#pragma unroll
    for (int w = 1; w < FIN_WAVES; ++w) {
      S += sm_s[w][c];
      K += sm_k[w][c];
    }
    if (open) {
      if (first) {
        // from the guess: step to its fixed-point image, or back to the bound if it overshot
        // every entry.  An equal count at the next point still means an equal active set.
        kprev = K > 0u ? K : NO_COUNT;
        t = K > 0u ? fmax((S - uj) / (double)K, lb) : lb;
      } else if (K == 0u || K == kprev) {
        open = false;   // t came from this very active set: it is the root
      } else {
        kprev = K;
        const double tn = (S - uj) / (double)K;
        if (tn > t) t = tn;
        else open = false;   // no move left: t is the root, to rounding
      }
    }
    first = false;
    if (!__syncthreads_or(open ? 1 : 0)) break;   // (also keeps the LDS rows until all have read them)
  }
  if (r == 0 && mine) {
    ws.tauj[j] = t;
    ws.done[j] = 1u;
  }
}

// Which stripe a workgroup takes.  Workgroups go to the chip's 8 XCDs in turn (workgroup b to XCD
// b % 8) and every XCD has an L2 of its own with 128-byte lines, so a line of Y that two
// neighbouring stripes share would cross the fabric twice if the two landed on different XCDs.
// Runs of STRIPE_XCD_RUN neighbouring stripes therefore go to workgroups 8 apart: the same XCD, one
// after the other in dispatch order.  (A permutation of the full runs; the ragged rest keeps
// its numbers.)
constexpr int STRIPE_XCD_RUN = 4;
constexpr int XCDS = 8;
__host__ __device__ __forceinline__ long long stripe_of_workgroup(long long b, long long nstripes) {
  const long long full = nstripes / (XCDS * STRIPE_XCD_RUN) * (XCDS * STRIPE_XCD_RUN);
  if (b >= full) return b;
  const long long xcd = b % XCDS, k = b / XCDS;
  return ((k / STRIPE_XCD_RUN) * XCDS + xcd) * STRIPE_XCD_RUN + k % STRIPE_XCD_RUN;
}

static inline bool finish_held(long long n) { return n <= (long long)FIN_ROWS * FIN_HELD; }

template <typename T, bool HELD>
__global__ __launch_bounds__(FIN_WG, HELD ? 4 : 8) void l11_finish_kernel(const T* __restrict__ Y, long long n,
                                                            long long m, Ws ws, int sweeps,
                                                            unsigned handoff) {
  l11_finish_body<T, HELD>(Y, n, m, ws, sweeps, handoff, stripe_of_workgroup(blockIdx.x, gridDim.x));
}

// The seeded form (no sweep, no seeding kernel before it): short matrices of at most 4096
// columns only.
constexpr int FIN_SEARCH_CACHE = (int)(FUSED_SEARCH_MAX / FIN_WG);   // up to 4096 columns in registers

template <typename T, int SC>
__global__ __launch_bounds__(FIN_WG, 4) void l11_finish_seeded_kernel(const T* __restrict__ Y, long long n,
                                                                      long long m, Ws ws, double eta,
                                                                      int outer) {
  l11_finish_body<T, true, SC>(Y, n, m, ws, 0, 0u, stripe_of_workgroup(blockIdx.x, gridDim.x), eta, outer);
}

}  // namespace mlproj

#endif
