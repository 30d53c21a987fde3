// mlproj: generic multi-level kernels on contiguous fibres (Sec. 5.2).
#ifndef MLPROJ_FIBRE_H
#define MLPROJ_FIBRE_H

#include "common.h"
#include "reduce.h"
#include "search.h"

namespace mlproj {

// ------------------------------------------------------------------ multi-level: fibre kernels
// The generic multi-level projection MP^nu (Sec. 5.2, Def. 5.2, Alg. 6 and its iterative form
// in the appendix) on a C-order tensor with the groups on axis 0: every level aggregates the
// contiguous last-axis fibres of the level below (fibre_agg), the top vector is projected
// onto the l1 ball (the search above), and on the way back every fibre is projected onto the
// ball whose radius is the matching entry of the level above (fibre_map).
// SEG lanes (4, 16 or 64) cooperate on one fibre, so a wavefront holds 64/SEG fibres (see the
// segment reductions above).
// Every load below is unconditional: a fibre or chunk index past the end is clamped to an
// existing one and what such a slot computes is masked afterwards.  (A load under a branch
// brings its wait with it, which leaves one load in flight per wavefront.)  The loaded chunks
// stay as stored until every load of the trip is issued (sched_barrier), then they are widened.
template <typename T, int VEC>
__device__ __forceinline__ Pack<T, VEC> load_chunk(const T* p) {
  return *reinterpret_cast<const Pack<T, VEC>*>(p);
}

template <int Q>
__device__ __forceinline__ void accumulate_d(double& a, double y) {
  if constexpr (Q == QINF) a = fmax(a, fabs(y));
  else if constexpr (Q == Q1) a += fabs(y);
  else a = fma(y, y, a);
}

constexpr int FIB_UNROLL = 4;  // fibres a segment works on at once (x2 chunks each: loads in flight)

// V[f] = || fibre f ||_q for nf contiguous fibres of len elements (len = nvec * VEC).
template <int Q, typename TIN, int SEG, int VEC>
__global__ __launch_bounds__(WG) void fibre_agg_kernel(const TIN* __restrict__ A, long long nf,
                                                       long long len, double* __restrict__ V,
                                                       float* __restrict__ v_out) {
  constexpr int PER_WAVE = WAVE / SEG;
  const int lane = threadIdx.x & (WAVE - 1);
  const int sl = lane % SEG;
  const long long nvec = len / VEC;
  const long long wave_id = (long long)blockIdx.x * WAVES + threadIdx.x / WAVE;
  const long long nwaves = (long long)gridDim.x * WAVES;
  const long long step = nwaves * PER_WAVE;
  for (long long f0 = wave_id * PER_WAVE + lane / SEG; f0 - lane / SEG < nf; f0 += step * FIB_UNROLL) {
    double acc[FIB_UNROLL];
    const TIN* base[FIB_UNROLL];
#pragma unroll
    for (int u = 0; u < FIB_UNROLL; ++u) {
      acc[u] = 0.0;
      const long long f = f0 + (long long)u * step;
      base[u] = A + (f < nf ? f : nf - 1) * len;
    }
    // two chunks per lane and fibre per trip
    for (long long i = sl; i < nvec; i += 2 * SEG) {
      const bool second = i + SEG < nvec;
      const long long i2 = second ? i + SEG : i;
      Pack<TIN, VEC> x[FIB_UNROLL], y[FIB_UNROLL];
#pragma unroll
      for (int u = 0; u < FIB_UNROLL; ++u) {
        x[u] = load_chunk<TIN, VEC>(base[u] + i * VEC);
        y[u] = load_chunk<TIN, VEC>(base[u] + i2 * VEC);
      }
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int u = 0; u < FIB_UNROLL; ++u)
#pragma unroll
        for (int k = 0; k < VEC; ++k) {
          accumulate_d<Q>(acc[u], (double)x[u].e[k]);
          accumulate_d<Q>(acc[u], second ? (double)y[u].e[k] : 0.0);
        }
    }
#pragma unroll
    for (int u = 0; u < FIB_UNROLL; ++u) {
      const double tot = (Q == QINF) ? seg_max<SEG>(acc[u]) : seg_sum<SEG>(acc[u]);
      const long long f = f0 + (long long)u * step;
      if (sl == 0 && f < nf) {
        const double vf = (Q == Q2) ? sqrt(tot) : tot;
        V[f] = vf;
        if (v_out) v_out[f] = (float)vf;
      }
    }
  }
}

// The same aggregate for fibres that one batch of loads covers (at most AGG_CHUNKS chunks per
// lane): a segment works through its fibres with the next batch already in flight while it
// folds the current one, so the reductions and stores hide behind the memory latency instead
// of adding to it (measured on a 64 MiB tensor of 256-element fibres: 19.5 -> 12 us).
constexpr int AGG_CHUNKS = 4;
constexpr int AGG_FIBRES = 2;  // fibres per segment and batch

template <int Q, typename TIN, int SEG, int VEC>
__global__ __launch_bounds__(WG) void fibre_agg_short_kernel(const TIN* __restrict__ A, long long nf,
                                                             long long len, double* __restrict__ V,
                                                             float* __restrict__ v_out) {
  constexpr int PER_WAVE = WAVE / SEG;
  constexpr int U = AGG_FIBRES, CH = AGG_CHUNKS;
  const int lane = threadIdx.x & (WAVE - 1);
  const int sl = lane % SEG;
  const int sub = lane / SEG;
  const long long nvec = len / VEC;   // <= CH * SEG
  const long long wave_id = (long long)blockIdx.x * WAVES + threadIdx.x / WAVE;
  const long long nwaves = (long long)gridDim.x * WAVES;
  const long long step = nwaves * PER_WAVE;
  bool ok[CH];
  long long at[CH];   // element offset of the lane's chunk k inside a fibre (chunk 0 when it has none)
#pragma unroll
  for (int k = 0; k < CH; ++k) {
    const long long i = sl + (long long)k * SEG;
    ok[k] = i < nvec;
    at[k] = (ok[k] ? i : 0) * VEC;
  }
  auto load_batch = [&](long long f0, Pack<TIN, VEC> (&dst)[U][CH]) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const long long f = f0 + (long long)u * step;
      const TIN* base = A + (f < nf ? f : nf - 1) * len;
#pragma unroll
      for (int k = 0; k < CH; ++k) dst[u][k] = load_chunk<TIN, VEC>(base + at[k]);
    }
  };
  long long f0 = wave_id * PER_WAVE + sub;   // f0 - sub is the same in every lane of the wavefront
  Pack<TIN, VEC> x[U][CH], y[U][CH];
  if (f0 - sub < nf) load_batch(f0, x);
  while (f0 - sub < nf) {
    const long long f1 = f0 + step * U;
    const bool more = f1 - sub < nf;
    if (more) load_batch(f1, y);
#pragma unroll
    for (int u = 0; u < U; ++u) {
      double acc = 0.0;
#pragma unroll
      for (int k = 0; k < CH; ++k)
#pragma unroll
        for (int e = 0; e < VEC; ++e) accumulate_d<Q>(acc, ok[k] ? (double)x[u][k].e[e] : 0.0);
      const double tot = (Q == QINF) ? seg_max<SEG>(acc) : seg_sum<SEG>(acc);
      const long long f = f0 + (long long)u * step;
      if (sl == 0 && f < nf) {
        const double vf = (Q == Q2) ? sqrt(tot) : tot;
        V[f] = vf;
        if (v_out) v_out[f] = (float)vf;
      }
    }
    if (more) {
#pragma unroll
      for (int u = 0; u < U; ++u)
#pragma unroll
        for (int k = 0; k < CH; ++k) x[u][k] = y[u][k];
    }
    f0 = f1;
  }
}

__global__ void clear_flags_kernel(Ws ws) { clear_meeting_area(ws.flags); }

// Radii of the top level from the threshold: R[a] = max(w[a] - tau, 0) (tau * weight[a] for a
// weighted l1 ball).
__global__ __launch_bounds__(WG) void top_radii_kernel(Ws ws, long long d0, double* __restrict__ R,
                                                       float* __restrict__ u_out) {
  const long long a = (long long)blockIdx.x * WG + threadIdx.x;
  if (a >= d0) return;
  const double u = radius_of(ws, a, ws.v[a], top_of(ws.res));
  R[a] = u;
  if (u_out) u_out[a] = (float)u;
}

// Output in the tensor's own element type is X itself, written once and not read again by the
// call: rounded through fp32 and streamed past the caches like the bi-level map pass does
// (dirty lines left behind would be written back under the next kernel's reads).  fp64 output
// is a level of radii the next kernel reads.
template <typename TOUT, int VEC>
__device__ __forceinline__ void store_chunk(TOUT* q, const double (&z)[VEC]) {
  if constexpr (std::is_same<TOUT, double>::value) {
#pragma unroll
    for (int k = 0; k < VEC; ++k) q[k] = z[k];
  } else {
    float f[VEC];
#pragma unroll
    for (int k = 0; k < VEC; ++k) f[k] = (float)z[k];
    store_row_nt<VEC>(q, f);
  }
}

template <int Q>
__device__ __forceinline__ double map_one(double x, double r, double par) {
  if constexpr (Q == QINF) return copysign(fmin(fabs(x), r), x);
  else if constexpr (Q == Q2) return x * par;
  else return copysign(fmax(fabs(x) - par, 0.0), x);
}

// The map of the top level can find the outer threshold itself: with TOP every workgroup runs
// the search over the nf aggregates redundantly (see search_block; same bits everywhere),
// takes its fibres' radii from it instead of from R, and workgroup 0 files the result record
// and the radii u.  That takes the one-workgroup search kernel and its launch off the path.
struct TopFuse {
  Ws ws;          // ws.v = the top aggregate (the same array as Vn)
  double eta;
  int outer;
  float* u_out;   // may be NULL
};

template <bool TOP>
__device__ __forceinline__ Top top_prologue(const TopFuse& tf, long long nf) {
  Top top{0.0, 1.0, HUGE_VAL};
  if constexpr (TOP) {
    __shared__ PairScratch<WAVES> bs;
    const SearchOut o = search_block<WG, SEARCH_CACHE>(tf.ws.v, nf, tf.eta, MODE_PROJECT, tf.outer, bs);
    top = top_of(o);
    if (blockIdx.x == 0 && threadIdx.x == 0) write_result(tf.ws, o, nullptr);
    if (tf.u_out)
      for (long long a = (long long)blockIdx.x * WG + threadIdx.x; a < nf; a += (long long)gridDim.x * WG)
        tf.u_out[a] = (float)radius(tf.ws.v[a], top);
  }
  return top;
}

// out fibre f = P^q_{R[f]}(fibre f of A), where Vn[f] is that fibre's own q-norm (known from
// the aggregation): clip (q = inf), rescale by R/Vn (q = 2), or shrink by the fibre's own
// threshold (q = 1), which the segment finds with the same Newton iteration as everywhere
// else, re-reading its fibre from cache on every step.  MAP_CHUNKS chunks per lane and trip.
constexpr int MAP_CHUNKS = 4;

template <int Q, typename TIN, typename TOUT, int SEG, int VEC, bool TOP = false>
__global__ __launch_bounds__(WG) void fibre_map_kernel(const TIN* A, long long nf, long long len,
                                                       const double* __restrict__ R,
                                                       const double* __restrict__ Vn, TOUT* out,
                                                       TopFuse tf) {
  constexpr int PER_WAVE = WAVE / SEG;
  const Top top = top_prologue<TOP>(tf, nf);
  const int lane = threadIdx.x & (WAVE - 1);
  const int sl = lane % SEG;
  const long long nvec = len / VEC;
  const long long wave_id = (long long)blockIdx.x * WAVES + threadIdx.x / WAVE;
  const long long nwaves = (long long)gridDim.x * WAVES;
  const long long step = nwaves * PER_WAVE;
  for (long long f0 = wave_id * PER_WAVE + lane / SEG; f0 - lane / SEG < nf; f0 += step) {
    const bool live = f0 < nf;
    const long long f = live ? f0 : nf - 1;  // idle segments shadow the last fibre, stores off
    const double nv = Vn[f];
    const double r = TOP ? radius(nv, top) : R[f];
    const TIN* p = A + f * len;
    TOUT* q = out + f * len;
    double par = 0.0;  // q = 2: scale; q = 1: threshold
    if constexpr (Q == Q2) par = nv > r ? r / nv : 1.0;
    if constexpr (Q == Q1) {
      // all lanes of the wavefront stay in the loop until every segment is done
      // (radius 0: the fibre goes to zero whatever its entries, no search)
      bool open = nv > r && r > 0.0;
      double t = open ? (nv - r) / (double)len   // every entry active: a lower bound
               : (nv > r ? HUGE_VAL : 0.0);
      unsigned kprev = 0xffffffffu;
      while (__any(open)) {
        double s = 0.0;
        unsigned c = 0;
        for (long long i = sl; i < nvec; i += (long long)MAP_CHUNKS * SEG) {
          Pack<TIN, VEC> x[MAP_CHUNKS];
#pragma unroll
          for (int k = 0; k < MAP_CHUNKS; ++k) {
            const long long ik = i + (long long)k * SEG;
            x[k] = load_chunk<TIN, VEC>(p + (ik < nvec ? ik : i) * VEC);
          }
          __builtin_amdgcn_sched_barrier(0);
#pragma unroll
          for (int k = 0; k < MAP_CHUNKS; ++k) {
            const bool ok = i + (long long)k * SEG < nvec;
#pragma unroll
            for (int e = 0; e < VEC; ++e) {
              const double a = fabs((double)x[k].e[e]);
              if (ok && a > t) { s += a; ++c; }
            }
          }
        }
        s = seg_sum<SEG>(s);
        c = seg_sum_u<SEG>(c);
        if (open) {
          if (c == 0u || c == kprev) open = false;
          else {
            kprev = c;
            const double tn = (s - r) / (double)c;
            if (tn > t) t = tn;
          }
        }
      }
      par = t;
    }
    for (long long i = sl; i < nvec; i += (long long)MAP_CHUNKS * SEG) {
      Pack<TIN, VEC> x[MAP_CHUNKS];
#pragma unroll
      for (int k = 0; k < MAP_CHUNKS; ++k) {
        const long long ik = i + (long long)k * SEG;
        x[k] = load_chunk<TIN, VEC>(p + (ik < nvec ? ik : i) * VEC);
      }
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int k = 0; k < MAP_CHUNKS; ++k) {
        const long long ik = i + (long long)k * SEG;
        double z[VEC];
#pragma unroll
        for (int e = 0; e < VEC; ++e) z[e] = map_one<Q>((double)x[k].e[e], r, par);
        if (live && ik < nvec) store_chunk<TOUT, VEC>(q + ik * VEC, z);
      }
    }
  }
}

// The same map for fibres short enough to sit in registers (at most KREG chunks of VEC elements
// per lane): each segment loads FIB_MAP_UNROLL fibres once, searches in registers, and stores.
constexpr int FIB_MAP_UNROLL = 2;

template <int Q, typename TIN, typename TOUT, int SEG, int VEC, int KREG, bool TOP = false>
__global__ __launch_bounds__(WG) void fibre_map_cached_kernel(const TIN* A, long long nf,
                                                              long long len,
                                                              const double* __restrict__ R,
                                                              const double* __restrict__ Vn,
                                                              TOUT* out, TopFuse tf) {
  constexpr int PER_WAVE = WAVE / SEG;
  const Top top = top_prologue<TOP>(tf, nf);
  constexpr int UF = FIB_MAP_UNROLL;
  const int lane = threadIdx.x & (WAVE - 1);
  const int sl = lane % SEG;
  const long long nvec = len / VEC;
  const long long wave_id = (long long)blockIdx.x * WAVES + threadIdx.x / WAVE;
  const long long nwaves = (long long)gridDim.x * WAVES;
  const long long step = nwaves * PER_WAVE;
  for (long long f0 = wave_id * PER_WAVE + lane / SEG; f0 - lane / SEG < nf; f0 += step * UF) {
    Pack<TIN, VEC> raw[UF][KREG];
    double r[UF], nv[UF];
    bool live[UF];
    long long f[UF];
#pragma unroll
    for (int u = 0; u < UF; ++u) {
      const long long fu = f0 + (long long)u * step;
      live[u] = fu < nf;
      f[u] = live[u] ? fu : nf - 1;  // idle segments shadow the last fibre, stores off
#pragma unroll
      for (int k = 0; k < KREG; ++k) {
        const long long i = sl + (long long)k * SEG;
        raw[u][k] = load_chunk<TIN, VEC>(A + f[u] * len + (i < nvec ? i : nvec - 1) * VEC);
      }
      nv[u] = Vn[f[u]];
      r[u] = TOP ? radius(nv[u], top) : R[f[u]];
    }
    __builtin_amdgcn_sched_barrier(0);
    double x[UF][KREG][VEC];
#pragma unroll
    for (int u = 0; u < UF; ++u)
#pragma unroll
      for (int k = 0; k < KREG; ++k) {
        const bool ok = sl + (long long)k * SEG < nvec;
#pragma unroll
        for (int c = 0; c < VEC; ++c) x[u][k][c] = ok ? (double)raw[u][k].e[c] : 0.0;  // 0 never counts: thresholds are > 0
      }
    double par[UF];
#pragma unroll
    for (int u = 0; u < UF; ++u) par[u] = (Q == Q2) ? (nv[u] > r[u] ? r[u] / nv[u] : 1.0) : 0.0;
    if constexpr (Q == Q1) {
      // The fixed point of the outer search, per fibre, in registers.  The first point is a
      // guess, the threshold an exponential tail of the fibre's mean magnitude would have,
      // shortened a little: the step from any point lands at or left of the root, so its image
      // (or the all-active bound, if larger) is a lower bound far closer than that bound alone,
      // and the iteration is monotone from there.  It saves about three rounds in eight.
      bool open[UF], first[UF];
      unsigned kprev[UF];
      double floor_t[UF];
      bool any_open = false;
#pragma unroll
      for (int u = 0; u < UF; ++u) {
        open[u] = nv[u] > r[u] && r[u] > 0.0;   // (radius 0: everything goes to zero, no search)
        floor_t[u] = open[u] ? (nv[u] - r[u]) / (double)len : 0.0;
        const float guess = open[u]
            ? -0.75f * (float)(nv[u] / (double)len) * __logf((float)(r[u] / nv[u])) : 0.0f;
        first[u] = (double)guess > floor_t[u];
        par[u] = first[u] ? (double)guess : floor_t[u];
        if (nv[u] > r[u] && !(r[u] > 0.0)) par[u] = HUGE_VAL;
        kprev[u] = 0xffffffffu;
        any_open = any_open || open[u];
      }
      while (__any(any_open)) {
        any_open = false;
#pragma unroll
        for (int u = 0; u < UF; ++u) {
          double s = 0.0;
          unsigned c = 0;
#pragma unroll
          for (int k = 0; k < KREG; ++k)
#pragma unroll
            for (int e = 0; e < VEC; ++e) {
              const double a = fabs(x[u][k][e]);
              if (a > par[u]) { s += a; ++c; }
            }
          s = seg_sum<SEG>(s);
          c = seg_sum_u<SEG>(c);
          if (open[u]) {
            if (first[u]) {
              kprev[u] = c > 0u ? c : 0xffffffffu;
              par[u] = c > 0u ? fmax((s - r[u]) / (double)c, floor_t[u]) : floor_t[u];
            } else if (c == 0u || c == kprev[u]) {
              open[u] = false;
            } else {
              kprev[u] = c;
              const double tn = (s - r[u]) / (double)c;
              if (tn > par[u]) par[u] = tn;
            }
          }
          first[u] = false;
          any_open = any_open || open[u];
        }
      }
    }
#pragma unroll
    for (int u = 0; u < UF; ++u) {
#pragma unroll
      for (int k = 0; k < KREG; ++k) {
        const long long i = sl + (long long)k * SEG;
        double z[VEC];
#pragma unroll
        for (int e = 0; e < VEC; ++e) z[e] = map_one<Q>(x[u][k][e], r[u], par[u]);
        if (live[u] && i < nvec) store_chunk<TOUT, VEC>(out + f[u] * len + i * VEC, z);
      }
    }
  }
}

}  // namespace mlproj

#endif
