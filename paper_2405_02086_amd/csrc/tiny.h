// mlproj: a whole bi-level projection in one kernel, for matrices of at most 128 KiB.
#ifndef MLPROJ_TINY_H
#define MLPROJ_TINY_H

#include "aggregate.h"
#include "common.h"
#include "reduce.h"
#include "search.h"

namespace mlproj {

// ------------------------------------------------------------------ tiny matrices
// A matrix this small costs three kernel launches and nothing else (13 us for 256 x 128).
// Here every workgroup reads ALL of Y into registers (16 chunks of 16 bytes per thread, 512
// threads: 128 KiB), folds the column aggregates through LDS in a fixed order, runs the
// threshold search (Eq. 6-7) itself, and then maps and stores its own share of the rows: the
// three steps of Alg. 1 with no hand-over between workgroups, so one launch.  All workgroups
// compute the same v and tau, bit for bit.  Reading Y sixteen times is served by the L2.
// For q = inf the aggregate is exact and the result has the bits of the three-kernel chain; for
// q = 2 the fp64 sums are folded in another order than there, which can show in the last bit of
// an output (a batch sends the same matrices here as single calls do, so it still returns
// their bits).
//
// Threads form TINY_WG / cw row lanes of cw column lanes (cw = the chunks of a row, rounded up
// to a power of two); a thread holds rows tr, tr + rl, tr + 2 rl, ... of its chunk column, and
// workgroup b stores the rows of slot b.  That needs X apart from Y: a workgroup still reading Y
// would see rows another has already written.  When X overlaps Y (a projection in place, the
// usual call of a training loop) ONE workgroup does the whole matrix (`whole`): it has read all
// of Y into its registers before its first store, so any overlap is harmless, and the 128 KiB
// it then stores alone cost little beside the launches saved.
// Which forms are built: q = inf and q = 2.  (A q = 1 form, with the per-column searches of
// Alg. 3 run on the held registers, was built and dropped: on fp32 storage it took 43 us for a
// 256 x 128 matrix against 23 us for the general path, whose finishing pass spreads the columns
// over many workgroups instead of repeating every search in each; on 16-bit storage it needed 82 KB
// of LDS, all 256 registers and scratch memory, and its one run ended in a memory aperture fault.)
template <int Q, typename T>
constexpr bool tiny_built() { return Q != Q1; }

constexpr int TINY_WG = 512;
constexpr int TINY_WAVES = TINY_WG / WAVE;
constexpr int TINY_SLOTS = 16;            // rows per thread

struct TinyPlan {
  int cw;     // column lanes
  int rl;     // row lanes
  int slots;  // rows per thread in use = workgroups
};

// Whether an n x m matrix with `vec` elements per 16-byte chunk fits, and how.
__host__ __device__ static inline bool tiny_plan(long long n, long long m, int vec, TinyPlan* p) {
  if (m % vec != 0 || m > FUSED_SEARCH_MAX) return false;
  const long long cpr = m / vec;
  if (cpr > TINY_WG) return false;
  int cw = 1;
  while (cw < cpr) cw *= 2;
  const int rl = TINY_WG / cw;
  const long long slots = cdiv(n, rl);
  if (slots > TINY_SLOTS) return false;
  p->cw = cw;
  p->rl = rl;
  p->slots = (int)slots;
  return true;
}

// (`bid` is the workgroup's number within its own problem: blockIdx.x for a single matrix.)
template <int Q, typename T, int VEC>
__device__ __forceinline__ void tiny_body(const T* Y, T* X, long long n,
                                          long long m, double eta, int outer, int cw, const Ws& ws,
                                          float* __restrict__ v_out, float* __restrict__ u_out,
                                          unsigned char* __restrict__ mask_out, long long bid,
                                          bool whole) {
  using Acc = typename AccOf<Q>::type;
  __shared__ Acc sm_part[TINY_WG * VEC];   // [row lane][column]
  __shared__ PairScratch<TINY_WAVES> bs;
  // v (zero beyond column m) takes the place of row lane 0 of the partials, in their type (fp32
  // maxima are exact, sums stay fp64): column c of that row is read by the one thread that then
  // writes v_c, and the other rows lie behind it.  So the body's LDS is at most 32 KiB.
  Acc* const sm_v = sm_part;
  static_assert(sizeof(Acc) * TINY_WG * VEC + sizeof(PairScratch<TINY_WAVES>) <= 49152,
                "tiny_body: the partial aggregates of this (q, storage type) need more LDS than planned");
  const int rl = TINY_WG / cw;
  const int tc = threadIdx.x % cw;
  const int tr = threadIdx.x / cw;
  const long long cpr = m / VEC;
  const bool col_ok = tc < cpr;
  const long long at = (col_ok ? tc : cpr - 1) * VEC;   // a lane without a chunk shadows the last one
  const int width = cw * VEC;

  Pack<T, VEC> raw[TINY_SLOTS];
#pragma unroll
  for (int k = 0; k < TINY_SLOTS; ++k) {
    const long long row = tr + (long long)k * rl;
    raw[k] = *reinterpret_cast<const Pack<T, VEC>*>(Y + (row < n ? row : n - 1) * m + at);
  }
  __builtin_amdgcn_sched_barrier(0);
  Acc acc[VEC];
#pragma unroll
  for (int e = 0; e < VEC; ++e) acc[e] = (Acc)0;
#pragma unroll
  for (int k = 0; k < TINY_SLOTS; ++k) {
    if (tr + (long long)k * rl < n) {
#pragma unroll
      for (int e = 0; e < VEC; ++e) accumulate<Q>(acc[e], (float)raw[k].e[e]);
    }
  }
#pragma unroll
  for (int e = 0; e < VEC; ++e) sm_part[tr * width + tc * VEC + e] = acc[e];
  __syncthreads();
  for (int c = threadIdx.x; c < width; c += TINY_WG) {
    Acc a = sm_part[c];
    for (int r = 1; r < rl; ++r) a = combine<Q>(a, sm_part[r * width + c]);
    const double vj = (Q == Q2) ? sqrt((double)a) : (double)a;
    sm_v[c] = c < m ? (Acc)vj : (Acc)0;
  }
  __syncthreads();

  // (the search of the map kernel's 256-thread workgroups, so that tau has the same bits here
  // as in the three-kernel chain and in a batch)
  const SearchOut o = search_block<WG, SEARCH_CACHE, TINY_WG, Acc>(sm_v, m, eta, MODE_PROJECT, outer, bs);
  const Top top = top_of(o);
  if (bid == 0) {
    if (threadIdx.x == 0) write_result(ws, o, nullptr);
    for (long long c = threadIdx.x; c < m; c += TINY_WG) {
      const double uj = radius((double)sm_v[c], top);
      if (v_out) v_out[c] = (float)sm_v[c];
      if (u_out) u_out[c] = (float)uj;
      if (mask_out) mask_out[c] = uj > 0.0 ? 1 : 0;
    }
  }
  float uf[VEC];
  double par[VEC];   // q = 2: scale u_j / v_j
#pragma unroll
  for (int e = 0; e < VEC; ++e) {
    const double vj = (double)sm_v[tc * VEC + e];
    const double uj = radius(vj, top);
    uf[e] = (float)uj;
    par[e] = (Q == Q2 && vj > 0.0) ? uj / vj : 0.0;
  }
  if (!col_ok) return;
  // this workgroup's rows: slot `bid` of every thread (every slot when it works alone)
#pragma unroll
  for (int k = 0; k < TINY_SLOTS; ++k) {
    if (whole || k == (int)bid) {
      const long long row = tr + (long long)k * rl;
      if (row < n) {
        float f[VEC];
#pragma unroll
        for (int e = 0; e < VEC; ++e) {
          const float y = (float)raw[k].e[e];
          if constexpr (Q == QINF) f[e] = copysignf(fminf(fabsf(y), uf[e]), y);
          else f[e] = (float)((double)y * par[e]);
        }
        store_row_nt<VEC>(X + row * m + at, f);
      }
    }
  }
}

template <int Q, typename T, int VEC>
__global__ __launch_bounds__(TINY_WG) void tiny_kernel(const T* Y, T* X,
                                                       long long n, long long m, double eta,
                                                       int outer, int cw, Ws ws,
                                                       float* __restrict__ v_out,
                                                       float* __restrict__ u_out,
                                                       unsigned char* __restrict__ mask_out,
                                                       int whole) {
  tiny_body<Q, T, VEC>(Y, X, n, m, eta, outer, cw, ws, v_out, u_out, mask_out, blockIdx.x, whole != 0);
}

}  // namespace mlproj

#endif
