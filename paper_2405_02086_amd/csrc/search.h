// mlproj: the l1-ball threshold search (Eq. 6-7) and the other outer projections.
#ifndef MLPROJ_SEARCH_H
#define MLPROJ_SEARCH_H

#include "common.h"
#include "reduce.h"

namespace mlproj {

// ------------------------------------------------------------------ threshold search
// Euclidean projection of v >= 0 onto the l1 ball of radius eta (Eq. 6-7): tau = 0 when
// sum(v) <= eta, otherwise the root of sum_j max(v_j - tau, 0) = eta.  The root is reached
// by the fixed point tau <- (sum_{v_j > tau} v_j - eta) / #{v_j > tau}, started from a lower
// bound; tau rises monotonically, the active set only shrinks, and when it stops shrinking
// tau is exactly (sum over the final active set - eta) / K, in fp64.
// Run by one whole workgroup of NT threads; every thread returns the same record.  Because
// the arithmetic and its order are fixed, any number of workgroups that run it on the same v
// get the same bits, which lets the map kernels run it redundantly instead of waiting for a
// separate one-workgroup kernel.
struct SearchOut {
  double tau, scale, cap;   // u_j = min(cap, scale * max(v_j - tau, 0))
  double total, vmax, norm; // sum v, max v, ||v||_p
  unsigned active, iters, inside;
};

// How the outer projection u = P^p_eta(v) acts on one aggregate (Eq. 6-7; Sec. 3 names the
// l1, l2 and l_inf balls as available outer projections): shrink by tau (p = 1), rescale
// (p = 2) or cap at eta (p = inf).  For p = 1 scale is 1 and cap is +inf, which leaves
// max(v - tau, 0) bit for bit.
struct Top {
  double tau, scale, cap;
};
__device__ __forceinline__ double radius(double v, const Top& t) {
  return fmin(t.cap, t.scale * fmax(v - t.tau, 0.0));
}
// The weighted l1 ball {u : sum_j w_j |u_j| <= eta} (the l_w1 norm Sec. 3 lists beside them)
// shrinks group j by tau * w_j instead (scale is 1 there, except 0 with eta = 0: tau = max v_j / w_j
// is a rounded quotient, and v_j - tau w_j could otherwise come out a rounding error above 0).
// Without weights this is radius() above, bit for bit.
__device__ __forceinline__ double radius_of(const Ws& ws, long long j, double v, const Top& t) {
  return ws.wts ? t.scale * fmax(v - t.tau * (double)ws.wts[j], 0.0) : radius(v, t);
}
__device__ __forceinline__ Top top_of(const SearchOut& o) { return Top{o.tau, o.scale, o.cap}; }
__device__ __forceinline__ Top top_of(const mlproj_result* r) { return Top{r->tau, r->scale, r->cap}; }

// NTHREADS > NT: a larger workgroup runs the search of an NT-thread one; the threads beyond
// NT hold nothing and add zeros, so the result has the bits the NT-thread workgroup gets.
// VT: the type v is stored in where the search reads it (fp64 in the workspace; fp32 for exact
// l_inf aggregates staged in LDS); every value is widened exactly before it is used.
// after_loads: called once the loads of v are issued and before anything waits for them; a
// caller that has loads of its own to issue (data the search does not depend on) issues them
// there, so that the search runs while they are in flight (loads return in order: issued ahead
// of v's, they would hold up the search's first wait).
struct NothingAfterLoads { __device__ __forceinline__ void operator()() const {} };
template <int NT, int CACHE = SEARCH_CACHE, int NTHREADS = NT, typename VT = double, typename AfterLoads = NothingAfterLoads>
__device__ __forceinline__ SearchOut search_block(const VT* __restrict__ v, long long ngroups,
                                                  double eta, int mode, int outer,
                                                  PairScratch<NTHREADS / WAVE>& s,
                                                  AfterLoads after_loads = AfterLoads()) {
  static_assert(NTHREADS >= NT && NTHREADS % WAVE == 0, "whole wavefronts, at least NT threads");
  // (a thread beyond NT starts past the end of v: every bound check below leaves it idle)
  const long long tid = (NTHREADS == NT || threadIdx.x < NT) ? (long long)threadIdx.x : ngroups;
  double vr[CACHE];
  double a = 0.0, mx = 0.0;
#pragma unroll
  for (int k = 0; k < CACHE; ++k) {
    const long long i = tid + (long long)k * NT;
    vr[k] = i < ngroups ? (double)v[i] : 0.0;  // 0 is never active: tau >= 0 and the test is strict
  }
  after_loads();
#pragma unroll
  for (int k = 0; k < CACHE; ++k) {
    a += vr[k];
    mx = fmax(mx, vr[k]);
  }
  for (long long i = tid + (long long)CACHE * NT; i < ngroups; i += NT) {
    const double x = (double)v[i];
    a += x;
    mx = fmax(mx, x);
  }
  SearchOut o;
  block_sum_max(a, mx, s);
  o.total = a;
  o.vmax = mx;
  o.norm = a;
  o.tau = 0.0;
  o.scale = 1.0;
  o.cap = HUGE_VAL;
  o.active = 0;
  o.iters = 0;
  o.inside = 0;
  if (mode == MODE_NORM) {
    // norm only: nothing to search
  } else if (outer != MLPROJ_OUTER_L1) {
    // l2 ball: rescale by eta / ||v||_2; l_inf ball: cap at eta.  No iteration.
    double sq = 0.0, dummy = 0.0;
    unsigned c = 0;
#pragma unroll
    for (int k = 0; k < CACHE; ++k) { sq = fma(vr[k], vr[k], sq); c += vr[k] > 0.0 ? 1u : 0u; }
    for (long long i = tid + (long long)CACHE * NT; i < ngroups; i += NT) {
      const double x = (double)v[i];
      sq = fma(x, x, sq);
      c += x > 0.0 ? 1u : 0u;
    }
    block_sum_count(sq, c, s);
    (void)dummy;
    if (outer == MLPROJ_OUTER_L2) {
      o.norm = sqrt(sq);
      o.inside = o.norm <= eta ? 1u : 0u;
      if (!o.inside) o.scale = eta / o.norm;
    } else {
      o.norm = o.vmax;
      o.inside = o.vmax <= eta ? 1u : 0u;
      if (!o.inside) o.cap = eta;
    }
    o.active = eta == 0.0 ? 0u : c;
  } else if (eta == 0.0) {
    o.tau = o.vmax;  // nothing exceeds vmax: every u_j is 0
  } else if (o.total <= eta) {
    o.inside = 1;  // already in the ball: tau = 0, u = v
    unsigned c = 0;
#pragma unroll
    for (int k = 0; k < CACHE; ++k) c += vr[k] > 0.0 ? 1u : 0u;
    for (long long i = tid + (long long)CACHE * NT; i < ngroups; i += NT)
      c += (double)v[i] > 0.0 ? 1u : 0u;
    double zero = 0.0;
    block_sum_count(zero, c, s);
    o.active = c;
  } else {
    // two lower bounds on the root: all groups active, and only the largest active
    double tau = fmax((o.total - eta) / (double)ngroups, o.vmax - eta);
    unsigned kprev = 0xffffffffu;
    for (;;) {
      double sum = 0.0;
      unsigned cnt = 0;
#pragma unroll
      for (int k = 0; k < CACHE; ++k) {
        if (vr[k] > tau) { sum += vr[k]; ++cnt; }
      }
      for (long long i = tid + (long long)CACHE * NT; i < ngroups; i += NT) {
        const double x = (double)v[i];
        if (x > tau) { sum += x; ++cnt; }
      }
      block_sum_count(sum, cnt, s);
      const double S = sum;
      const unsigned K = cnt;
      o.active = K;
      if (K == 0u || K == kprev) break;  // K == 0: eta below the resolution of vmax
      kprev = K;
      const double t = (S - eta) / (double)K;
      if (t > tau) tau = t;
      ++o.iters;
    }
    o.tau = tau;
  }
  return o;
}

__device__ __forceinline__ void write_result(const Ws& ws, const SearchOut& o,
                                             double* __restrict__ norm_out) {
  mlproj_result* r = ws.res;
  r->tau = o.tau;
  r->scale = o.scale;
  r->cap = o.cap;
  r->norm = o.norm;
  r->vmax = o.vmax;
  r->n_active = o.active;
  r->inside_ball = o.inside;
  r->search_iters = o.iters;
  r->inner_sweeps = 0;
  r->inner_pending = 0;
  r->inner_finished = 0;
  if (norm_out) *norm_out = o.total;
}

// radii / u_out (optional): also write u_j = max(v_j - tau, 0) for every group.
// NT threads with CACHE values of v per thread in registers.  Up to 16384 groups the host
// launches the very search the map kernels run in their prologue (256 threads, 16 or 64
// values), so that a split call (radii first, map later) finds tau with the bits of the whole
// call; 1024 threads with 32 values serve 16385-32768 groups (64 would not fit the 128
// registers a 1024-thread workgroup leaves each thread), 1024 x 16 stands behind the
// several-workgroup search.
template <int NT, int CACHE>
__global__ __launch_bounds__(NT) void search_kernel(Ws ws, long long ngroups, double eta,
                                                    int mode, int outer,
                                                    double* __restrict__ norm_out,
                                                    int only_as_fallback,
                                                    double* __restrict__ radii,
                                                    float* __restrict__ u_out) {
  __shared__ PairScratch<NT / WAVE> s;
  if (only_as_fallback && ws.flags[1] == 0u) return;
  const SearchOut o = search_block<NT, CACHE>(ws.v, ngroups, eta, mode, outer, s);
  if (threadIdx.x <= MAX_INNER_SWEEPS) ws.pending[threadIdx.x] = 0u;
  if (threadIdx.x == 0) write_result(ws, o, norm_out);
  if (radii) {
    const Top top = top_of(o);
    for (long long i = threadIdx.x; i < ngroups; i += NT) {
      const double u = radius(ws.v[i], top);
      radii[i] = u;
      if (u_out) u_out[i] = (float)u;
    }
  }
}

// ------------------------------------------------------------------ weighted threshold search
// Euclidean projection of v >= 0 onto the weighted l1 ball {u : sum_j w_j u_j <= eta}, w > 0:
// u_j = max(v_j - tau w_j, 0), with tau = 0 when sum w_j v_j <= eta and otherwise the root of
// g(tau) = sum_j w_j max(v_j - tau w_j, 0) = eta.  g is convex, decreasing and piecewise linear,
// and the fixed point tau <- (sum_A w_j v_j - eta) / sum_A w_j^2 over A = {v_j > tau w_j} is
// Newton's step on it: started from the all-active value (a lower bound on the root) tau rises
// monotonically, A only shrinks, and when it stops shrinking tau is exact for the final A.
// One workgroup of NT threads; CACHE pairs (v_j, w_j) per thread stay in registers, longer
// vectors are re-read from memory (the L2) in every round; beyond 32768 groups the host
// enqueues the grid-wide form below first and this one as its fallback.  A round costs what the
// workgroup issues, every wavefront repeating the last fold: 256 threads (one wavefront per
// SIMD) take a third of the time of 1024 per round, so the host picks few threads with many
// pairs each: 256 x 16 up to 4096 groups, 256 x 64 up to 16384 (6 and 14 us on an MI355X for
// four rounds), 1024 x 16 beyond (512 x 64 spills).
// The record gets norm = sum w_j v_j and vmax = max v_j; with eta = 0, tau = max v_j / w_j.
template <int NT, int CACHE>
__global__ __launch_bounds__(NT) void search_weighted_kernel(Ws ws, long long ngroups, double eta,
                                                              int only_as_fallback,
                                                              double* __restrict__ radii,
                                                              float* __restrict__ u_out) {
  __shared__ PairScratch<NT / WAVE> s;
  if (only_as_fallback && ws.flags[1] == 0u) return;
  const long long tid = threadIdx.x;
  const float* __restrict__ wts = ws.wts;
  const double* __restrict__ v = ws.v;
  double vr[CACHE];
  float wr[CACHE];   // (as stored: widened where used, which keeps the pairs within the registers)
  // every load is unconditional (a slot past the end re-reads the last pair and is then blanked),
  // so all of them are in flight together
#pragma unroll
  for (int k = 0; k < CACHE; ++k) {
    const long long i = tid + (long long)k * NT;
    const long long ii = i < ngroups ? i : ngroups - 1;
    vr[k] = v[ii];
    wr[k] = wts[ii];
  }
  __builtin_amdgcn_sched_barrier(0);
  double num = 0.0, den = 0.0, vmax = 0.0;
#pragma unroll
  for (int k = 0; k < CACHE; ++k) {
    const bool ok = tid + (long long)k * NT < ngroups;
    if (!ok) { vr[k] = 0.0; wr[k] = 1.0f; }   // 0 is never active: tau >= 0, w > 0 and the test is strict
    const double w = (double)wr[k];
    num = fma(w, vr[k], num);
    den = ok ? fma(w, w, den) : den;
    vmax = fmax(vmax, vr[k]);
  }
  for (long long i = tid + (long long)CACHE * NT; i < ngroups; i += NT) {
    const double x = v[i], w = (double)wts[i];
    num = fma(w, x, num);
    den = fma(w, w, den);
    vmax = fmax(vmax, x);
  }
  block_sum_max<NT / WAVE, 4>(num, vmax, s);
  double none = 0.0;
  block_sum_max<NT / WAVE, 4>(den, none, s);
  SearchOut o;
  o.total = num;
  o.norm = num;
  o.vmax = vmax;
  o.tau = 0.0;
  o.scale = 1.0;
  o.cap = HUGE_VAL;
  o.active = 0;
  o.iters = 0;
  o.inside = 0;
  if (eta == 0.0) {
    double rmax = 0.0, zero = 0.0;   // tau = max v_j / w_j: v_j - tau w_j <= 0 for every j
    for (long long i = tid; i < ngroups; i += NT) rmax = fmax(rmax, v[i] / (double)wts[i]);
    block_sum_max<NT / WAVE, 4>(zero, rmax, s);
    o.tau = rmax;
    o.scale = 0.0;   // (see radius_of)
  } else {
    const bool inside = num <= eta;
    double tau = inside ? 0.0 : (num - eta) / den;
    unsigned kprev = 0xffffffffu;
    for (;;) {
      double sn = 0.0, sd = 0.0;
      unsigned cnt = 0;
#pragma unroll
      for (int k = 0; k < CACHE; ++k) {
        float wf = wr[k];
        asm volatile("" : "+v"(wf));   // (keeps the widening inside the loop: hoisted, the doubles spill)
        const double w = (double)wf;
        if (vr[k] > tau * w) { sn = fma(w, vr[k], sn); sd = fma(w, w, sd); ++cnt; }
      }
      for (long long i = tid + (long long)CACHE * NT; i < ngroups; i += NT) {
        const double x = v[i], w = (double)wts[i];
        if (x > tau * w) { sn = fma(w, x, sn); sd = fma(w, w, sd); ++cnt; }
      }
      block_sum2_count(sn, sd, cnt, s);
      o.active = cnt;
      if (inside || cnt == 0u || cnt == kprev) break;  // inside: one round, just to count
      kprev = cnt;
      const double t = (sn - eta) / sd;
      if (t > tau) tau = t;
      ++o.iters;
    }
    o.tau = tau;
    o.inside = inside ? 1u : 0u;
  }
  if (threadIdx.x <= MAX_INNER_SWEEPS) ws.pending[threadIdx.x] = 0u;
  if (threadIdx.x == 0) write_result(ws, o, nullptr);
  if (radii) {   // (optional) also the radii u_j = max(v_j - tau w_j, 0) of every group
    const Top top = top_of(o);
    for (long long i = tid; i < ngroups; i += NT) {
      const double u = radius_of(ws, i, v[i], top);
      radii[i] = u;
      if (u_out) u_out[i] = (float)u;
    }
  }
}

// The same search for very long v (more groups than one workgroup holds in registers): up to
// 64 workgroups of NT threads, each keeping its slice of v in registers (VALUES per thread).
// As in the one-workgroup kernels a round costs what a workgroup issues, so the host launches
// 256 threads with 32 values each rather than 1024 with 8.
// Every round each workgroup posts the sum and count of its slice above tau, every workgroup
// collects all the posts and adds them up in the same fixed order, so all of them step tau
// identically and leave the loop together.
//
// The exchange is built for this GPU, where a device-scope fence means an L2 write-back
// (microseconds, and it serialises).  A post is a handful of 64-bit words, each carrying the
// round number in its upper half and 32 bits of payload in its lower half, written with
// device-scope atomic exchanges (performed at the memory side) and never waited for; lane g of
// the first wavefront polls workgroup g's words with device-scope atomic loads (which bypass
// the per-XCD L2) until every one carries the current round number.  A word is complete or
// absent, so neither an arrival counter nor an ordering between the words is needed, and a
// round costs one write and one read latency.  Slots alternate by round parity: a workgroup can
// post round r + 2 only after it has collected round r + 1, which every workgroup posts only
// after collecting round r, so nobody overwrites what another still reads.  The slots start
// cleared (clear_meeting_area, in a kernel that precedes this one in every call).
// The grid is far smaller than the chip, so all workgroups become resident; a lane that
// nevertheless polls SPIN_LIMIT times raises flags[1], every poller sees that and everybody
// leaves: the kernel always ends, and the one-workgroup kernel queued behind it then does the
// work instead.
__device__ __forceinline__ void post_word(unsigned long long* q, unsigned round, unsigned payload) {
  __hip_atomic_exchange(q, ((unsigned long long)round << 32) | payload, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ unsigned lo32(double x) { return (unsigned)(unsigned long long)__double_as_longlong(x); }
__device__ __forceinline__ unsigned hi32(double x) { return (unsigned)((unsigned long long)__double_as_longlong(x) >> 32); }
__device__ __forceinline__ double from32(unsigned lo, unsigned hi) {
  return __longlong_as_double((long long)(((unsigned long long)hi << 32) | lo));
}

// A non-negative double as a float, rounded towards zero.
__device__ __forceinline__ float float_at_or_below(double x) {
  float f = (float)x;
  if ((double)f > x) f = __uint_as_float(__float_as_uint(f) - 1u);   // (f > x >= 0: f is positive, also when it is inf)
  return f;
}

// Collect W words of every workgroup's post of this round into pay[] of lane g (zeros in the
// other lanes).  False, for every thread of the workgroup alike, when the search gives up.
// spin_limit: polls a lane may spend waiting (checked every 64th); 0 = give up without polling,
// which the host uses to exercise the fallback.
template <int W>
__device__ __forceinline__ bool collect(const unsigned long long* q, unsigned* flags, unsigned round,
                                        int nwg, unsigned spin_limit, unsigned (&pay)[W], unsigned* lds_ok) {
  if (threadIdx.x == 0) *lds_ok = 1u;
  __syncthreads();
#pragma unroll
  for (int w = 0; w < W; ++w) pay[w] = 0u;
  if ((int)threadIdx.x < nwg) {
    unsigned spins = 0;
    bool ok = spin_limit != 0u;
    while (ok) {
      bool all = true;
#pragma unroll
      for (int w = 0; w < W; ++w) {
        const unsigned long long x = __hip_atomic_load(&q[w * COOP_MAX_WGS + threadIdx.x], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        all = all && (unsigned)(x >> 32) == round;
        pay[w] = (unsigned)x;
      }
      if (all) break;
      if ((++spins & 63u) == 0u &&
          (spins > spin_limit || __hip_atomic_load(&flags[1], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0u)) {
        ok = false;
        break;
      }
      __builtin_amdgcn_s_sleep(1);
    }
    if (!ok) {
      __hip_atomic_exchange(&flags[1], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      *lds_ok = 0u;
    }
  }
  __syncthreads();
  const bool ok = *lds_ok != 0u;
  __syncthreads();
  return ok;
}

// WEIGHTED: the weighted l1 ball (see search_weighted_kernel): slices hold (v_j, w_j) pairs and
// post a third number per round, the sum of w_j^2 over their active entries.
// tile_stats (plain l1 ball only; null: not available): nstats triples (sum, sum of squares,
// maximum) of disjoint parts of v, left by the aggregate pass.  Every workgroup folds them in
// the same order, so the totals are known without the first exchange, and with the variance
// comes a starting guess: the root if v were Gaussian with that mean and variance.  The guess
// is evaluated first; its fixed-point image is a lower bound on the root whichever side of the
// root the guess lies on (the tangent of a convex function lies below it), and from there the
// iteration goes on as ever, so only the number of rounds depends on the guess.  A round also
// posts the smallest entry above its point (plain ball), which tells whether the point's image is
// already the root: the round that only confirmed an unchanged count is not needed.  Three
// exchanges instead of seven on 262144 column maxima of Laplace entries.
template <bool WEIGHTED, int NT, int VALUES>
__global__ __launch_bounds__(NT) void search_wide_kernel(Ws ws, long long ngroups, double eta,
                                                          int mode, double* __restrict__ norm_out,
                                                          unsigned spin_limit,
                                                          const double* __restrict__ tile_stats,
                                                          long long nstats) {
  static_assert(NT >= COOP_MAX_WGS, "one lane per workgroup collects its post");
  __shared__ PairScratch<NT / WAVE> s;
  __shared__ RoundScratch<NT / WAVE> rs;
  __shared__ unsigned lds_ok;
  const int tid = threadIdx.x;
  const int nwg = (int)gridDim.x, wg = (int)blockIdx.x;
  const long long chunk = (ngroups + nwg - 1) / nwg;
  const long long lo = (long long)wg * chunk;
  const long long hi = (lo + chunk < ngroups) ? lo + chunk : ngroups;
  const double* __restrict__ v = ws.v;
  const float* __restrict__ wts = ws.wts;
  // word w of workgroup g in the slots of parity p
  auto slot = [&](unsigned p, int w, int g) { return ws.coop_q + ((size_t)p * COOP_WORDS + w) * COOP_MAX_WGS + g; };

  double vr[VALUES];
  float wr[WEIGHTED ? VALUES : 1];
  double a = 0.0, mx = 0.0, den = 0.0;   // a: sum of v, weighted: of w v
  // every load is unconditional (a slot past the slice re-reads its last entry, or entry 0 for
  // an empty slice, and is then blanked), so all of them are in flight together
  const long long last = hi > lo ? hi - 1 : 0;
#pragma unroll
  for (int k = 0; k < VALUES; ++k) {
    const long long i = lo + tid + (long long)k * NT;
    const long long ii = i < hi ? i : last;
    vr[k] = v[ii];
    if constexpr (WEIGHTED) wr[k] = wts[ii];
  }
  // (the first STAT_SLOTS triples per thread of the aggregate pass's statistics travel with them)
  constexpr int STAT_SLOTS = 4;
  const bool have_stats = !WEIGHTED && tile_stats != nullptr;
  double st[STAT_SLOTS][3];
#pragma unroll
  for (int k = 0; k < STAT_SLOTS; ++k) {
    const long long i = tid + (long long)k * NT;
    const long long ii = have_stats ? (i < nstats ? i : nstats - 1) : 0;
    const double* p = have_stats ? tile_stats + 3 * ii : v;
#pragma unroll
    for (int c = 0; c < 3; ++c) st[k][c] = p[have_stats ? c : 0];
  }
  __builtin_amdgcn_sched_barrier(0);
#pragma unroll
  for (int k = 0; k < VALUES; ++k) {
    const bool ok = lo + tid + (long long)k * NT < hi;
    if (!ok) vr[k] = 0.0;
    if constexpr (WEIGHTED) {
      if (!ok) wr[k] = 1.0f;
      const double w = (double)wr[k];
      a = fma(w, vr[k], a);
      den = ok ? fma(w, w, den) : den;
    } else {
      a += vr[k];
    }
    mx = fmax(mx, vr[k]);
  }
  for (long long i = lo + tid + (long long)VALUES * NT; i < hi; i += NT) {
    const double x = v[i];
    if constexpr (WEIGHTED) {
      const double w = (double)wts[i];
      a = fma(w, x, a);
      den = fma(w, w, den);
    } else {
      a += x;
    }
    mx = fmax(mx, x);
  }
  if (!have_stats) block_sum_max(a, mx, s);   // (with the statistics the totals come from them)
  double third = 0.0;   // weighted: the slice's sum of w^2, or with eta = 0 its maximum of v/w
  if constexpr (WEIGHTED) {
    double rmax = 0.0;
    if (eta == 0.0) {   // then tau = max v_j / w_j, and the sum of w^2 is not needed
      // (read again rather than taken from the registers: unrolled, the divisions spill)
      for (long long i = lo + tid; i < hi; i += NT) rmax = fmax(rmax, v[i] / (double)wts[i]);
    }
    block_sum_max<NT / WAVE, 4>(den, rmax, s);
    third = eta == 0.0 ? rmax : den;
  }
  unsigned round = 1;  // the first round carries the totals
  SearchOut o;
  double den_all = 0.0, rmax_all = 0.0;
  double guess = -1.0;
  if (have_stats) {
    double sa = 0.0, sq = 0.0, sm = 0.0, none = 0.0;
#pragma unroll
    for (int k = 0; k < STAT_SLOTS; ++k) {
      if (tid + (long long)k * NT < nstats) {
        sa += st[k][0];
        sq += st[k][1];
        sm = fmax(sm, st[k][2]);
      }
    }
    for (long long i = tid + (long long)STAT_SLOTS * NT; i < nstats; i += NT) {
      sa += tile_stats[3 * i];
      sq += tile_stats[3 * i + 1];
      sm = fmax(sm, tile_stats[3 * i + 2]);
    }
    block_sum_max(sa, sm, s);
    block_sum_max(sq, none, s);
    o.total = sa;
    o.vmax = sm;
    // E max(V - tau, 0) = sd h(z) for V ~ N(mean, sd^2), z = (tau - mean) / sd, with
    // h(z) = phi(z) - z Q(z), h' = -Q (Q the upper tail): solve sd h(z) = eta / m by Newton on
    // the convex h (it lands left of the root after the first step and rises from there)
    const double mean = sa / (double)ngroups;
    const double var = sq / (double)ngroups - mean * mean;
    if (mode == MODE_PROJECT && eta > 0.0 && sa > eta && var > 0.0) {
      // (fp32 is plenty: the guess is a statistical estimate, and only the speed depends on it)
      const double sd = sqrt(var);
      const float want = (float)(eta / ((double)ngroups * sd));
      float z = 0.0f;
      for (int it = 0; it < 8; ++it) {
        const float tail = 0.5f * erfcf(z * 0.70710678f);
        if (!(tail > 1e-30f)) break;
        const float h = 0.39894228f * expf(-0.5f * z * z) - z * tail;
        z += (h - want) / tail;
      }
      guess = mean + sd * (double)z;
    }
  } else {
    if (tid == 0) {
      post_word(slot(1u, 0, wg), round, lo32(a));
      post_word(slot(1u, 1, wg), round, hi32(a));
      post_word(slot(1u, 2, wg), round, lo32(mx));
      post_word(slot(1u, 3, wg), round, hi32(mx));
      if constexpr (WEIGHTED) {
        post_word(slot(1u, 4, wg), round, lo32(third));
        post_word(slot(1u, 5, wg), round, hi32(third));
      }
    }
    unsigned pay[WEIGHTED ? 6 : 4];
    if (!collect(slot(1u, 0, 0), ws.flags, round, nwg, spin_limit, pay, &lds_ok)) return;
    o.total = from32(pay[0], pay[1]);
    o.vmax = from32(pay[2], pay[3]);
    block_sum_max(o.total, o.vmax, s);
    if constexpr (WEIGHTED) {
      den_all = from32(pay[4], pay[5]);
      rmax_all = den_all;
      block_sum_max<NT / WAVE, 4>(den_all, rmax_all, s);
    }
  }
  o.norm = o.total;
  o.tau = 0.0;
  o.scale = 1.0;
  o.cap = HUGE_VAL;
  o.active = 0;
  o.iters = 0;
  o.inside = 0;
  if (mode == MODE_NORM) {
  } else if (eta == 0.0) {
    o.tau = WEIGHTED ? rmax_all : o.vmax;
    if (WEIGHTED) o.scale = 0.0;   // (see radius_of)
  } else {
    const bool inside = o.total <= eta;
    double tau = inside ? 0.0
               : WEIGHTED ? (o.total - eta) / den_all
                          : fmax((o.total - eta) / (double)ngroups, o.vmax - eta);
    unsigned kprev = 0xffffffffu;
    // (a guess at or below the lower bound, or beyond every entry, says nothing the bound does not)
    bool guessing = !inside && guess > tau && guess < o.vmax;
    for (;;) {
      const double at = guessing ? guess : tau;
      double sum = 0.0, sd = 0.0;
      unsigned cnt = 0;
      double nxt = HUGE_VAL;   // (plain ball) the smallest entry above the point, +inf when there is none
#pragma unroll
      for (int k = 0; k < VALUES; ++k) {
        if constexpr (WEIGHTED) {
          float wf = wr[k];
          asm volatile("" : "+v"(wf));   // (keeps the widening inside the loop)
          const double w = (double)wf;
          if (vr[k] > at * w) { sum = fma(w, vr[k], sum); sd = fma(w, w, sd); ++cnt; }
        } else {
          if (vr[k] > at) { sum += vr[k]; ++cnt; nxt = fmin(nxt, vr[k]); }
        }
      }
      for (long long i = lo + tid + (long long)VALUES * NT; i < hi; i += NT) {
        const double x = v[i];
        if constexpr (WEIGHTED) {
          const double w = (double)wts[i];
          if (x > at * w) { sum = fma(w, x, sum); sd = fma(w, w, sd); ++cnt; }
        } else {
          if (x > at) { sum += x; ++cnt; nxt = fmin(nxt, x); }
        }
      }
      // as a float, rounded down: a test against it can only err on the side of one more round
      float nxt_f = float_at_or_below(nxt);
      if constexpr (WEIGHTED) block_sum2_count(sum, sd, cnt, s);
      else block_sum_count_min(sum, cnt, nxt_f, rs);
      ++round;
      const unsigned par = round & 1u;
      if (tid == 0) {
        post_word(slot(par, 0, wg), round, lo32(sum));
        post_word(slot(par, 1, wg), round, hi32(sum));
        post_word(slot(par, 2, wg), round, cnt);
        if constexpr (WEIGHTED) {
          post_word(slot(par, 3, wg), round, lo32(sd));
          post_word(slot(par, 4, wg), round, hi32(sd));
        } else {
          post_word(slot(par, 3, wg), round, __float_as_uint(nxt_f));
        }
      }
      unsigned pay[WEIGHTED ? 5 : 4];
      if (!collect(slot(par, 0, 0), ws.flags, round, nwg, spin_limit, pay, &lds_ok)) return;
      double S = from32(pay[0], pay[1]), D = 0.0;
      unsigned K = pay[2];
      float above_pt = INFINITY;
      if constexpr (WEIGHTED) {
        D = from32(pay[3], pay[4]);
        block_sum2_count(S, D, K, s);
      } else {
        if (tid < nwg) above_pt = __uint_as_float(pay[3]);
        block_sum_count_min(S, K, above_pt, rs);
      }
      if (guessing) {
        // The image of the guess.  If it beats the bound it becomes the point, and the count at
        // the guess stands for "the point it came from": an equal count at the image means no
        // entry lies between the two, so the image is the root of that linear piece.
        guessing = false;
        ++o.iters;
        if (K > 0u) {
          const double t = (S - eta) / (double)K;
          if (t > tau) { tau = t; kprev = K; }
        }
        continue;
      }
      o.active = K;
      if (inside || K == 0u || K == kprev) break;  // inside: one round, just to count
      kprev = K;
      const double t = WEIGHTED ? (S - eta) / D : (S - eta) / (double)K;
      if (t > tau) tau = t;
      ++o.iters;
      // From below the image t of the point p lies at or right of p, and f is linear up to the
      // smallest entry above p: if t stays left of that entry it is the root, and the K entries
      // above p are the ones above t.  The posted neighbour decides it without another round.
      if (!WEIGHTED && t < (double)above_pt) break;
    }
    o.tau = tau;
    o.inside = inside ? 1u : 0u;
  }
  if (wg == 0) {
    if (tid <= MAX_INNER_SWEEPS) ws.pending[tid] = 0u;
    if (tid == 0) write_result(ws, o, norm_out);
  }
}

}  // namespace mlproj

#endif
