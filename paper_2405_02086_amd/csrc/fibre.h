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
template <typename T, int VEC>
__device__ __forceinline__ void load_elems(const T* p, double (&x)[VEC]) {
  if constexpr (VEC == 4) {
    const float4 t = *reinterpret_cast<const float4*>(p);
    x[0] = t.x; x[1] = t.y; x[2] = t.z; x[3] = t.w;
  } else {
    x[0] = (double)*p;
  }
}

template <int Q>
__device__ __forceinline__ void accumulate_d(double& a, double y) {
  if constexpr (Q == QINF) a = fmax(a, fabs(y));
  else if constexpr (Q == Q1) a += fabs(y);
  else a = fma(y, y, a);
}

constexpr int FIB_UNROLL = 4;  // fibres a segment works on at once (loads in flight)

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
#pragma unroll
    for (int u = 0; u < FIB_UNROLL; ++u) acc[u] = 0.0;
    for (long long i = sl; i < nvec; i += SEG) {
      double x[FIB_UNROLL][VEC];
#pragma unroll
      for (int u = 0; u < FIB_UNROLL; ++u) {
        const long long f = f0 + (long long)u * step;
        if (f < nf) load_elems<TIN, VEC>(A + f * len + i * VEC, x[u]);
        else {
#pragma unroll
          for (int k = 0; k < VEC; ++k) x[u][k] = 0.0;
        }
      }
#pragma unroll
      for (int u = 0; u < FIB_UNROLL; ++u)
#pragma unroll
        for (int k = 0; k < VEC; ++k) accumulate_d<Q>(acc[u], x[u][k]);
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

__global__ void clear_flags_kernel(Ws ws) {
  if (threadIdx.x < 2) ws.flags[threadIdx.x] = 0u;
}

// Radii of the top level from the threshold: R[a] = max(w[a] - tau, 0).
__global__ __launch_bounds__(WG) void top_radii_kernel(Ws ws, long long d0, double* __restrict__ R,
                                                       float* __restrict__ u_out) {
  const long long a = (long long)blockIdx.x * WG + threadIdx.x;
  if (a >= d0) return;
  const double u = radius(ws.v[a], top_of(ws.res));
  R[a] = u;
  if (u_out) u_out[a] = (float)u;
}

// out fibre f = P^q_{R[f]}(fibre f of A), where Vn[f] is that fibre's own q-norm (known from
// the aggregation): clip (q = inf), rescale by R/Vn (q = 2), or shrink by the fibre's own
// threshold (q = 1), which the segment finds with the same Newton iteration as everywhere
// else, re-reading its fibre from cache on every step.
template <int Q, typename TIN, typename TOUT, int SEG, int VEC>
__global__ __launch_bounds__(WG) void fibre_map_kernel(const TIN* A, long long nf, long long len,
                                                       const double* __restrict__ R,
                                                       const double* __restrict__ Vn, TOUT* out) {
  constexpr int PER_WAVE = WAVE / SEG;
  const int lane = threadIdx.x & (WAVE - 1);
  const int sl = lane % SEG;
  const long long nvec = len / VEC;
  const long long wave_id = (long long)blockIdx.x * WAVES + threadIdx.x / WAVE;
  const long long nwaves = (long long)gridDim.x * WAVES;
  const long long step = nwaves * PER_WAVE;
  for (long long f0 = wave_id * PER_WAVE + lane / SEG; f0 - lane / SEG < nf; f0 += step) {
    const bool live = f0 < nf;
    const long long f = live ? f0 : nf - 1;  // idle segments shadow the last fibre, stores off
    const double r = R[f];
    const double nv = Vn[f];
    const TIN* p = A + f * len;
    TOUT* q = out + f * len;
    double par = 0.0;  // q = 2: scale; q = 1: threshold
    if constexpr (Q == Q2) par = nv > r ? r / nv : 1.0;
    if constexpr (Q == Q1) {
      // all lanes of the wavefront stay in the loop until every segment is done
      bool open = nv > r;
      double t = open ? (nv - r) / (double)len : 0.0;  // every entry active: a lower bound
      unsigned kprev = 0xffffffffu;
      while (__any(open)) {
        double s = 0.0;
        unsigned c = 0;
        for (long long i = sl; i < nvec; i += SEG) {
          double x[VEC];
          load_elems<TIN, VEC>(p + i * VEC, x);
#pragma unroll
          for (int k = 0; k < VEC; ++k) {
            const double a = fabs(x[k]);
            if (a > t) { s += a; ++c; }
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
    for (long long i = sl; i < nvec; i += SEG) {
      double x[VEC];
      load_elems<TIN, VEC>(p + i * VEC, x);
      TOUT y[VEC];
#pragma unroll
      for (int k = 0; k < VEC; ++k) {
        double z;
        if constexpr (Q == QINF) z = copysign(fmin(fabs(x[k]), r), x[k]);
        else if constexpr (Q == Q2) z = x[k] * par;
        else z = copysign(fmax(fabs(x[k]) - par, 0.0), x[k]);
        y[k] = (TOUT)z;
      }
      if (live) {
        if constexpr (VEC == 4) {
          *reinterpret_cast<float4*>(q + i * VEC) = make_float4(y[0], y[1], y[2], y[3]);
        } else {
          q[i] = y[0];
        }
      }
    }
  }
}

// The same map for fibres short enough to sit in registers (at most KREG chunks of VEC elements
// per lane): each segment loads FIB_MAP_UNROLL fibres once, searches in registers, and stores.
constexpr int FIB_MAP_UNROLL = 2;

template <int Q, typename TIN, typename TOUT, int SEG, int VEC, int KREG>
__global__ __launch_bounds__(WG) void fibre_map_cached_kernel(const TIN* A, long long nf,
                                                              long long len,
                                                              const double* __restrict__ R,
                                                              const double* __restrict__ Vn,
                                                              TOUT* out) {
  constexpr int PER_WAVE = WAVE / SEG;
  constexpr int UF = FIB_MAP_UNROLL;
  const int lane = threadIdx.x & (WAVE - 1);
  const int sl = lane % SEG;
  const long long nvec = len / VEC;
  const long long wave_id = (long long)blockIdx.x * WAVES + threadIdx.x / WAVE;
  const long long nwaves = (long long)gridDim.x * WAVES;
  const long long step = nwaves * PER_WAVE;
  for (long long f0 = wave_id * PER_WAVE + lane / SEG; f0 - lane / SEG < nf; f0 += step * UF) {
    double x[UF][KREG][VEC];
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
        if (i < nvec) load_elems<TIN, VEC>(A + f[u] * len + i * VEC, x[u][k]);
        else {
#pragma unroll
          for (int c = 0; c < VEC; ++c) x[u][k][c] = 0.0;  // 0 never counts: thresholds are > 0
        }
      }
      r[u] = R[f[u]];
      nv[u] = Vn[f[u]];
    }
    double par[UF];
#pragma unroll
    for (int u = 0; u < UF; ++u) par[u] = (Q == Q2) ? (nv[u] > r[u] ? r[u] / nv[u] : 1.0) : 0.0;
    if constexpr (Q == Q1) {
      bool open[UF];
      unsigned kprev[UF];
      bool any_open = false;
#pragma unroll
      for (int u = 0; u < UF; ++u) {
        open[u] = nv[u] > r[u];
        par[u] = open[u] ? (nv[u] - r[u]) / (double)len : 0.0;
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
            if (c == 0u || c == kprev[u]) open[u] = false;
            else {
              kprev[u] = c;
              const double tn = (s - r[u]) / (double)c;
              if (tn > par[u]) par[u] = tn;
            }
          }
          any_open = any_open || open[u];
        }
      }
    }
#pragma unroll
    for (int u = 0; u < UF; ++u) {
#pragma unroll
      for (int k = 0; k < KREG; ++k) {
        const long long i = sl + (long long)k * SEG;
        TOUT y[VEC];
#pragma unroll
        for (int e = 0; e < VEC; ++e) {
          double z;
          if constexpr (Q == QINF) z = copysign(fmin(fabs(x[u][k][e]), r[u]), x[u][k][e]);
          else if constexpr (Q == Q2) z = x[u][k][e] * par[u];
          else z = copysign(fmax(fabs(x[u][k][e]) - par[u], 0.0), x[u][k][e]);
          y[e] = (TOUT)z;
        }
        if (live[u] && i < nvec) {
          TOUT* q = out + f[u] * len + i * VEC;
          if constexpr (VEC == 4) *reinterpret_cast<float4*>(q) = make_float4(y[0], y[1], y[2], y[3]);
          else q[0] = y[0];
        }
      }
    }
  }
}

}  // namespace mlproj

#endif
