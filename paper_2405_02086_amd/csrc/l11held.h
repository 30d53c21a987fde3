// mlproj: bi-level l1,1 (Alg. 3) for matrices of at most 4096 rows, columns kept in registers.
#ifndef MLPROJ_L11HELD_H
#define MLPROJ_L11HELD_H

#include "common.h"
#include "l11.h"
#include "reduce.h"
#include "search.h"

namespace mlproj {

// ------------------------------------------------------------------ l1,1 from registers
// Alg. 3 after the column sums: the outer threshold, then for every kept column the threshold
// tau_j with sum_i max(|Y_ij| - tau_j, 0) = u_j, then X = sign(Y) max(|Y| - tau_j, 0).  The
// lock-step sweeps of l11.h read the whole matrix once per step because a column is strided in
// memory.  A matrix of at most 4096 rows lets one workgroup hold 16 whole columns instead (one
// 64-byte run of every row, as the finishing pass does): 512 threads x up to 128 elements.  The
// workgroup reads its stripe once, runs the fixed point of the finishing pass on registers
// (no memory traffic per step), and maps and stores from the same registers: after the
// aggregate pass Y is read once and X written once, whatever the number of steps.
//
// A lane owns VEC = 16 bytes' worth of neighbouring columns (one vector access per row), CW
// lanes span the stripe, and the thread of row lane r holds rows r, r + RL, r + 2 RL, ...  The
// partial sums and counts of a column are folded over the row lanes of a 16-lane row on the
// DPP crossbar (rotations by CW, 2 CW, ... 8), then over the 4 rows of each of the 8
// wavefronts through LDS by the first wavefront (four lanes per column), always in the same
// order: the result repeats bit for bit.  The column's owner thread steps its threshold and
// publishes it.
constexpr int LH_WG = 512;
constexpr int LH_COLS = 16;
constexpr int LH_COLS_NARROW = 8;   // fp32, 4097 to 8192 rows: stripes of 8 columns (32-byte runs), 128 values per thread
constexpr int LH_WAVES = LH_WG / WAVE;
constexpr int LH_FOLD_ROWS = LH_WAVES * (WAVE / 16);   // partial rows per column in LDS
// The host sends larger matrices through the sweeps: 64M elements of fp32, 32M of a 16-bit type
// (whose 16-column stripes are 32-byte runs: 1024 x 65536 bf16 takes 0.34 ms here against 0.21).
template <typename T>
constexpr long long lh_max_elems() { return sizeof(T) == 4 ? (64LL << 20) : (32LL << 20); }
constexpr int DPP_ROR2 = 0x122;
constexpr int LH_SEARCH_CACHE = 8;   // values of v per thread when the kernel runs the outer search itself: up to 4096 columns

template <typename T, int COLS = LH_COLS>
struct LhShape {
  static constexpr int VEC = 16 / (int)sizeof(T);
  static constexpr int CW = COLS / VEC;
  static constexpr int RL = LH_WG / CW;
  static_assert(CW == 2 || CW == 4, "the crossbar fold is written for 2 or 4 lanes per run");
  static_assert(COLS <= LH_COLS, "the LDS arrays hold LH_COLS columns");
};

// values per thread a matrix of n rows needs (32, 64 or 128), 0 when it has too many rows
template <typename T>
static inline int lh_values_for(long long n) {
  const long long rows = (n + LhShape<T>::RL - 1) / LhShape<T>::RL * LhShape<T>::VEC;
  return rows <= 32 ? 32 : rows <= 64 ? 64 : rows <= 128 ? 128 : 0;
}
// ... and whether the narrow stripes (fp32 only) reach a matrix too tall for the wide ones
static inline bool lh_narrow_fits(long long n) {
  return (n + LhShape<float, LH_COLS_NARROW>::RL - 1) / LhShape<float, LH_COLS_NARROW>::RL * 4 <= 128;
}

struct LhLds {
  double s[LH_FOLD_ROWS][LH_COLS];
  unsigned k[LH_FOLD_ROWS][LH_COLS];
  float ct[LH_COLS];      // the columns' current thresholds as published by their owners: the smallest float above each
  float th[LH_COLS];      // ... and the final ones as fp32 pairs (see colmap_body)
  float tl[LH_COLS];
};

// Sum over the lanes of a 16-lane row that own the same columns (the same lane % CW).
template <int CW>
__device__ __forceinline__ double lh_row_sum(double x) {
  if constexpr (CW <= 2) x += dpp_f64<DPP_ROR2>(x);
  x += dpp_f64<DPP_ROR4>(x);
  x += dpp_f64<DPP_ROR8>(x);
  return x;
}
template <int CW>
__device__ __forceinline__ unsigned lh_row_sum_u(unsigned x) {
  if constexpr (CW <= 2) x += dpp_u32<DPP_ROR2>(x);
  x += dpp_u32<DPP_ROR4>(x);
  x += dpp_u32<DPP_ROR8>(x);
  return x;
}
template <int CW>
__device__ __forceinline__ float lh_row_max(float x) {
  if constexpr (CW <= 2) x = fmaxf(x, __uint_as_float(dpp_u32<DPP_ROR2>(__float_as_uint(x))));
  x = fmaxf(x, __uint_as_float(dpp_u32<DPP_ROR4>(__float_as_uint(x))));
  x = fmaxf(x, __uint_as_float(dpp_u32<DPP_ROR8>(__float_as_uint(x))));
  return x;
}

// NV: values per thread (rows per thread x VEC).  SC > 0: every workgroup runs the outer search
// itself (SC values of v per thread), workgroup 0 files the result record; SC = 0: a search
// kernel ran before and the record is read.  X may alias Y (a thread reads and writes the same
// elements only).
template <typename T, int NV, int SC, int COLS = LH_COLS>
__device__ __forceinline__ void l11_held_body(const T* Y, T* X, long long n, long long m, const Ws& ws,
                                              float* __restrict__ u_out, unsigned char* __restrict__ mask_out,
                                              double seed_eta, int outer, long long bid) {
  using Sh = LhShape<T, COLS>;
  constexpr int VEC = Sh::VEC, CW = Sh::CW, RL = Sh::RL;
  constexpr int ROWS = NV / VEC;
  __shared__ LhLds lds;
  __shared__ PairScratch<LH_WAVES> bs;
  const int tid = threadIdx.x;
  const int lane = tid & (WAVE - 1);
  const int wave = tid / WAVE;
  const int cw = tid % CW;            // which 16-byte piece of the stripe's run
  const int rl = tid / CW;            // row lane
  const long long col0 = bid * COLS + (long long)cw * VEC;
  const bool lane_ok = col0 < m;      // (m is a multiple of VEC: a lane's columns exist together)
  const long long col0c = lane_ok ? col0 : m - VEC;   // a lane past the end shadows the last columns
  // Byte offsets of the thread's elements from the start of the matrix, in 32 bits (the host
  // sends at most lh_max_elems<T>() elements here): one address register per access instead of two.
  const unsigned off0 = (unsigned)(((long long)rl * m + col0c) * (long long)sizeof(T));
  const unsigned step = (unsigned)((long long)RL * m * (long long)sizeof(T));
  const unsigned off_last = (unsigned)(((n - 1) * m + col0c) * (long long)sizeof(T));
  const char* const ybytes = reinterpret_cast<const char*>(Y);

  // the stripe, as stored, every load in flight at once (a row past the end re-reads the last one)
  Pack<T, VEC> raw[ROWS];
  auto request_rows = [&](auto first, auto last) {   // (compile-time bounds: raw[] must stay in registers)
#pragma unroll
    for (int u = decltype(first)::value; u < decltype(last)::value; ++u) {
      const unsigned off = rl + u * RL < n ? off0 + (unsigned)u * step : off_last;
      raw[u] = *reinterpret_cast<const Pack<T, VEC>*>(ybytes + off);
    }
    __builtin_amdgcn_sched_barrier(0);
  };
  // (with the search ahead: the first quarter of the rows is requested at once, the rest when
  // the stripe is known to be needed)
  constexpr int EARLY = ROWS >= 4 ? ROWS / 4 : 1;
  using R0 = std::integral_constant<int, 0>;
  using RE = std::integral_constant<int, EARLY>;
  using RN = std::integral_constant<int, ROWS>;
  auto request_stripe = [&]() { request_rows(R0(), RN()); };

  // The owner of column c of the stripe: thread c.
  const bool owner = tid < COLS;
  const long long j = bid * COLS + tid;
  const long long jj = (owner && j < m) ? j : 0;
  double vj = 0.0;

  Top top;
  bool inside, nothing;
  if constexpr (SC > 0) {
    // (the stripe is requested right behind the search's own loads: the search runs under it)
    const SearchOut o = search_block<LH_WG, SC, LH_WG, double>(ws.v, m, seed_eta, MODE_PROJECT, outer, bs, request_stripe);
    top = top_of(o);
    inside = o.inside != 0u;
    nothing = inside || o.active == 0u;
    if (bid == 0 && tid == 0) {
      write_result(ws, o, nullptr);
      ws.res->inner_finished = nothing ? 0u : o.active;
    }
  } else {
    // (the record and the column sums are requested ahead of the rows: loads return in order)
    mlproj_result* res = ws.res;
    top = top_of(res);
    inside = res->inside_ball != 0u;
    const unsigned n_active = res->n_active;
    if (owner) vj = ws.v[jj];
    __builtin_amdgcn_sched_barrier(0);
    request_rows(R0(), RE());
    nothing = inside || n_active == 0u;
    if (bid == 0 && tid == 0) res->inner_finished = nothing ? 0u : n_active;
  }

  // The owner's column: its radius, bounds and state.
  double uj = 0.0, lb = 0.0, t = 0.0;
  bool mine = false, open = false, first = true;
  unsigned kprev = NO_COUNT;
  if (owner) {
    if constexpr (SC > 0) vj = ws.v[jj];
    uj = j < m ? radius_of(ws, jj, vj, top) : 0.0;
    mine = j < m && !inside && uj > 0.0;
    open = mine;
    if (j < m) {
      if (u_out) u_out[j] = (float)uj;
      if (mask_out) mask_out[j] = uj > 0.0 ? 1 : 0;
    }
  }
  if constexpr (SC == 0) {
    // The search ran ahead, so the radii are known early: a stripe whose columns are all dropped
    // (the sparse results the projection is used for) is zeroed, and three quarters of it are
    // never read (the first quarter was requested with the radii, so that a stripe that is
    // needed does not wait twice).
    const bool need = inside || __syncthreads_or((owner && j < m && uj > 0.0) ? 1 : 0) != 0;
    if (!need) {
      if (lane_ok) {
        float zero[VEC];
#pragma unroll
        for (int k = 0; k < VEC; ++k) zero[k] = 0.0f;
#pragma unroll
        for (int u = 0; u < ROWS; ++u)
          if (rl + u * RL < n) store_row_nt<VEC, true>(reinterpret_cast<T*>(reinterpret_cast<char*>(X) + (off0 + (unsigned)u * step)), zero);
      }
      return;
    }
    request_rows(RE(), RN());
  }
  // (the starting guess only now: with the search ahead, the rest of the stripe is on its way)
  // a dropped column maps to zero: threshold +inf; inside the ball nothing moves: threshold 0
  if (owner) t = mine ? l11_guess(vj, uj, n, lb) : (inside ? 0.0 : HUGE_VAL);

  float held[ROWS][VEC];
#pragma unroll
  for (int u = 0; u < ROWS; ++u) {
    const bool row_ok = rl + (long long)u * RL < n;
#pragma unroll
    for (int k = 0; k < VEC; ++k) held[u][k] = row_ok ? (float)raw[u].e[k] : 0.0f;   // |0| is never above a threshold
  }

  if (!nothing) {
    // The columns' largest entries: a_max - u_j is a second certified lower bound (the largest
    // entry alone sums to a_max - t), next to the root where the radius is small.
    {
      float hm[VEC];
#pragma unroll
      for (int k = 0; k < VEC; ++k) hm[k] = 0.0f;
#pragma unroll
      for (int u = 0; u < ROWS; ++u)
#pragma unroll
        for (int k = 0; k < VEC; ++k) hm[k] = fmaxf(hm[k], fabsf(held[u][k]));
#pragma unroll
      for (int k = 0; k < VEC; ++k) hm[k] = lh_row_max<CW>(hm[k]);
      if ((lane & 15) < CW) {
#pragma unroll
        for (int k = 0; k < VEC; ++k) lds.s[wave * 4 + lane / 16][cw * VEC + k] = (double)hm[k];
      }
      __syncthreads();
      // (the fold over the partial rows: the 64 lanes of the first wavefront take a quarter of the
      // rows of one column each, lane = column + 16 * quarter, and meet on the crossbar)
      double amax = 0.0;
      if (wave == 0) {
#pragma unroll
        for (int w = 0; w < LH_FOLD_ROWS / 4; ++w) amax = fmax(amax, lds.s[(lane >> 4) * (LH_FOLD_ROWS / 4) + w][lane & 15]);
        amax = fmax(amax, __shfl_xor(amax, 16));
        amax = fmax(amax, __shfl_xor(amax, 32));
      }
      if (owner) {
        if (mine) {
          if (amax - uj > lb) lb = amax - uj;
          if (t <= lb || t >= amax) {   // the guess is no better than the bound, or beyond every entry
            t = lb;
            first = false;
          }
        }
        lds.ct[tid] = above(t);
      }
      __syncthreads();
    }
    for (;;) {
      float ct[VEC];
#pragma unroll
      for (int k = 0; k < VEC; ++k) ct[k] = lds.ct[cw * VEC + k];
      double s[VEC];
      unsigned cnt[VEC];
#pragma unroll
      for (int k = 0; k < VEC; ++k) { s[k] = 0.0; cnt[k] = 0u; }
#pragma unroll
      for (int u = 0; u < ROWS; ++u) {
#pragma unroll
        for (int k = 0; k < VEC; ++k) {
          asm volatile("" : "+v"(held[u][k]));   // keeps the widening to fp64 in the loop: hoisted, it doubles the registers
          const float h = fabsf(held[u][k]);
          const bool in = h >= ct[k];
          s[k] += (double)(in ? h : 0.0f);
          cnt[k] += in ? 1u : 0u;
        }
      }
#pragma unroll
      for (int k = 0; k < VEC; ++k) {
        s[k] = lh_row_sum<CW>(s[k]);
        cnt[k] = lh_row_sum_u<CW>(cnt[k]);
      }
      if ((lane & 15) < CW) {
#pragma unroll
        for (int k = 0; k < VEC; ++k) {
          lds.s[wave * 4 + lane / 16][cw * VEC + k] = s[k];
          lds.k[wave * 4 + lane / 16][cw * VEC + k] = cnt[k];
        }
      }
      __syncthreads();
      double S = 0.0;
      unsigned K = 0u;
      if (wave == 0) {   // (as for the maxima above; always in this order, so the sums repeat bit for bit)
#pragma unroll
        for (int w = 0; w < LH_FOLD_ROWS / 4; ++w) {
          S += lds.s[(lane >> 4) * (LH_FOLD_ROWS / 4) + w][lane & 15];
          K += lds.k[(lane >> 4) * (LH_FOLD_ROWS / 4) + w][lane & 15];
        }
        S += __shfl_xor(S, 16);
        K += __shfl_xor(K, 16);
        S += __shfl_xor(S, 32);
        K += __shfl_xor(K, 32);
      }
      if (owner && open) {
        if (first) {
          // from the guess: step to its fixed-point image (a lower bound from any point), or
          // back to the bound if it overshot every entry
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
        first = false;
        lds.ct[tid] = above(t);
      }
      if (!__syncthreads_or((owner && open) ? 1 : 0)) break;
    }
  }
  if (owner) {
    const float th = (float)t;
    lds.th[tid] = th;
    lds.tl[tid] = t < HUGE_VAL ? (float)(t - (double)th) : 0.0f;
    if (mine) {
      ws.tauj[j] = t;
      ws.done[j] = 1u;
    }
  }
  __syncthreads();
  if (!lane_ok) return;
  float th[VEC], tl[VEC];
#pragma unroll
  for (int k = 0; k < VEC; ++k) {
    th[k] = lds.th[cw * VEC + k];
    tl[k] = lds.tl[cw * VEC + k];
  }
  char* const xbytes = reinterpret_cast<char*>(X);
#pragma unroll
  for (int u = 0; u < ROWS; ++u) {
    if (rl + u * RL < n) {
      float f[VEC];
#pragma unroll
      for (int k = 0; k < VEC; ++k)
        f[k] = copysignf(fmaxf((fabsf(held[u][k]) - th[k]) - tl[k], 0.0f), held[u][k]);
      store_row_nt<VEC, true>(reinterpret_cast<T*>(xbytes + (off0 + (unsigned)u * step)), f);
    }
  }
}

// Registers: 32 values per thread leave room for two workgroups per CU, 128 for one.  64 fit two
// only with some twenty registers spilled, which pays when there are more stripes than CUs (the
// second workgroup's loads and stores run under the first one's arithmetic: 42 against 52 us at
// 2048 x 8192) and costs when every stripe has a CU to itself (27 against 23 us at 2048 x 2048):
// PACKED picks the two-per-CU build.
constexpr int lh_min_waves(int nv, bool packed) { return nv <= 32 ? 4 : nv <= 64 ? (packed ? 4 : 2) : 2; }

template <typename T, int NV, int SC, bool PACKED = false, int COLS = LH_COLS>
__global__ __launch_bounds__(LH_WG, lh_min_waves(NV, PACKED)) void l11_held_kernel(
    const T* Y, T* X, long long n, long long m, Ws ws, float* __restrict__ u_out,
    unsigned char* __restrict__ mask_out, double seed_eta, int outer) {
  l11_held_body<T, NV, SC, COLS>(Y, X, n, m, ws, u_out, mask_out, seed_eta, outer,
                                 stripe_of_workgroup(blockIdx.x, gridDim.x));
}

}  // namespace mlproj

#endif
