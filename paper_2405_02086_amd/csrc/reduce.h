// mlproj: wavefront, workgroup and segment reductions on the DPP crossbar.
#ifndef MLPROJ_REDUCE_H
#define MLPROJ_REDUCE_H

#include "common.h"

namespace mlproj {

// Wavefront reductions on the DPP crossbar (no LDS round trips).  Each step adds the value of
// another lane: swap within pairs, swap pairs within quads, shift the 16-lane row by 4 and by
// 8, then carry row totals across the four rows; lanes with no source lane add 0, which is
// neutral for sums and for maxima of non-negative values.  Lane 63 ends with the total and is
// broadcast.  The order of operations is fixed, so results repeat bit for bit.
template <int CTRL>
__device__ __forceinline__ unsigned dpp_u32(unsigned x) {
  return (unsigned)__builtin_amdgcn_update_dpp(0, (int)x, CTRL, 0xf, 0xf, false);
}
template <int CTRL>
__device__ __forceinline__ double dpp_f64(double x) {
  const unsigned long long b = (unsigned long long)__double_as_longlong(x);
  const unsigned lo = dpp_u32<CTRL>((unsigned)b), hi = dpp_u32<CTRL>((unsigned)(b >> 32));
  return __longlong_as_double((long long)(((unsigned long long)hi << 32) | lo));
}
constexpr int DPP_SWAP1 = 0xb1, DPP_SWAP2 = 0x4e, DPP_SHR4 = 0x114, DPP_SHR8 = 0x118,
              DPP_BCAST15 = 0x142, DPP_BCAST31 = 0x143;

__device__ __forceinline__ unsigned bcast63_u32(unsigned x) {
  return (unsigned)__builtin_amdgcn_readlane((int)x, 63);
}
__device__ __forceinline__ double bcast63_f64(double x) {
  const unsigned long long b = (unsigned long long)__double_as_longlong(x);
  const unsigned lo = bcast63_u32((unsigned)b), hi = bcast63_u32((unsigned)(b >> 32));
  return __longlong_as_double((long long)(((unsigned long long)hi << 32) | lo));
}
__device__ __forceinline__ double wave_sum(double x) {
  x += dpp_f64<DPP_SWAP1>(x);
  x += dpp_f64<DPP_SWAP2>(x);
  x += dpp_f64<DPP_SHR4>(x);
  x += dpp_f64<DPP_SHR8>(x);
  x += dpp_f64<DPP_BCAST15>(x);
  x += dpp_f64<DPP_BCAST31>(x);
  return bcast63_f64(x);
}
// maximum of non-negative values
__device__ __forceinline__ double wave_max(double x) {
  x = fmax(x, dpp_f64<DPP_SWAP1>(x));
  x = fmax(x, dpp_f64<DPP_SWAP2>(x));
  x = fmax(x, dpp_f64<DPP_SHR4>(x));
  x = fmax(x, dpp_f64<DPP_SHR8>(x));
  x = fmax(x, dpp_f64<DPP_BCAST15>(x));
  x = fmax(x, dpp_f64<DPP_BCAST31>(x));
  return bcast63_f64(x);
}
__device__ __forceinline__ unsigned wave_sum_u(unsigned x) {
  x += dpp_u32<DPP_SWAP1>(x);
  x += dpp_u32<DPP_SWAP2>(x);
  x += dpp_u32<DPP_SHR4>(x);
  x += dpp_u32<DPP_SHR8>(x);
  x += dpp_u32<DPP_BCAST15>(x);
  x += dpp_u32<DPP_BCAST31>(x);
  return bcast63_u32(x);
}

// Workgroup-wide reductions for NW wavefronts; every thread gets the result.  The order of
// the additions is fixed, so results repeat bit for bit from run to run.
template <int NW>
struct BlockScratch {
  double d[NW];
  unsigned u[NW];
};

template <int NW>
__device__ __forceinline__ double block_sum(double x, BlockScratch<NW>& s) {
  x = wave_sum(x);
  if ((threadIdx.x & (WAVE - 1)) == 0) s.d[threadIdx.x / WAVE] = x;
  __syncthreads();
  double r = 0.0;
#pragma unroll
  for (int w = 0; w < NW; ++w) r += s.d[w];
  __syncthreads();
  return r;
}
template <int NW>
__device__ __forceinline__ double block_max(double x, BlockScratch<NW>& s) {
  x = wave_max(x);
  if ((threadIdx.x & (WAVE - 1)) == 0) s.d[threadIdx.x / WAVE] = x;
  __syncthreads();
  double r = s.d[0];
#pragma unroll
  for (int w = 1; w < NW; ++w) r = fmax(r, s.d[w]);
  __syncthreads();
  return r;
}
template <int NW>
__device__ __forceinline__ unsigned block_sum_u(unsigned x, BlockScratch<NW>& s) {
  x = wave_sum_u(x);
  if ((threadIdx.x & (WAVE - 1)) == 0) s.u[threadIdx.x / WAVE] = x;
  __syncthreads();
  unsigned r = 0;
#pragma unroll
  for (int w = 0; w < NW; ++w) r += s.u[w];
  __syncthreads();
  return r;
}

// Two reductions for the price of one barrier pair: (sum, max) and (sum, count).
template <int NW>
struct PairScratch {
  double a[NW];
  double b[NW];
  unsigned u[NW];
};
// (AT_ONCE: how many waves' pairs are fetched together; fewer where registers are short)
template <int NW, int AT_ONCE = NW>
__device__ __forceinline__ void block_sum_max(double& sum, double& mx, PairScratch<NW>& s) {
  sum = wave_sum(sum);
  mx = wave_max(mx);
  if ((threadIdx.x & (WAVE - 1)) == 0) { s.a[threadIdx.x / WAVE] = sum; s.b[threadIdx.x / WAVE] = mx; }
  __syncthreads();
  double r = 0.0, q = 0.0;
#pragma unroll AT_ONCE
  for (int w = 0; w < NW; ++w) { r += s.a[w]; q = fmax(q, s.b[w]); }
  __syncthreads();
  sum = r;
  mx = q;
}
template <int NW>
__device__ __forceinline__ void block_sum_count(double& sum, unsigned& cnt, PairScratch<NW>& s) {
  sum = wave_sum(sum);
  cnt = wave_sum_u(cnt);
  if ((threadIdx.x & (WAVE - 1)) == 0) { s.a[threadIdx.x / WAVE] = sum; s.u[threadIdx.x / WAVE] = cnt; }
  __syncthreads();
  double r = 0.0;
  unsigned c = 0;
#pragma unroll
  for (int w = 0; w < NW; ++w) { r += s.a[w]; c += s.u[w]; }
  __syncthreads();
  sum = r;
  cnt = c;
}

// ... and (sum, count, minimum) with a float minimum (+inf = no candidate).
template <int NW>
struct RoundScratch {
  double a[NW];
  unsigned u[NW];
  float lo[NW];
};
__device__ __forceinline__ float wave_min_f(float x) {
  x = fminf(x, __uint_as_float(dpp_u32<DPP_SWAP1>(__float_as_uint(x))));
  x = fminf(x, __uint_as_float(dpp_u32<DPP_SWAP2>(__float_as_uint(x))));
  x = fminf(x, __uint_as_float(dpp_u32<DPP_SHR4>(__float_as_uint(x))));
  x = fminf(x, __uint_as_float(dpp_u32<DPP_SHR8>(__float_as_uint(x))));
  x = fminf(x, __uint_as_float(dpp_u32<DPP_BCAST15>(__float_as_uint(x))));
  x = fminf(x, __uint_as_float(dpp_u32<DPP_BCAST31>(__float_as_uint(x))));
  return __uint_as_float(bcast63_u32(__float_as_uint(x)));
}
template <int NW>
__device__ __forceinline__ void block_sum_count_min(double& sum, unsigned& cnt, float& mn, RoundScratch<NW>& s) {
  sum = wave_sum(sum);
  cnt = wave_sum_u(cnt);
  mn = wave_min_f(mn);
  if ((threadIdx.x & (WAVE - 1)) == 0) {
    const int w = threadIdx.x / WAVE;
    s.a[w] = sum; s.u[w] = cnt; s.lo[w] = mn;
  }
  __syncthreads();
  double r = 0.0;
  unsigned c = 0;
  float l = INFINITY;
#pragma unroll
  for (int w = 0; w < NW; ++w) { r += s.a[w]; c += s.u[w]; l = fminf(l, s.lo[w]); }
  __syncthreads();
  sum = r;
  cnt = c;
  mn = l;
}

// ... and (sum, sum, count), for the weighted threshold search.
template <int NW>
__device__ __forceinline__ void block_sum2_count(double& sum, double& sum2, unsigned& cnt, PairScratch<NW>& s) {
  sum = wave_sum(sum);
  sum2 = wave_sum(sum2);
  cnt = wave_sum_u(cnt);
  if ((threadIdx.x & (WAVE - 1)) == 0) {
    s.a[threadIdx.x / WAVE] = sum; s.b[threadIdx.x / WAVE] = sum2; s.u[threadIdx.x / WAVE] = cnt;
  }
  __syncthreads();
  double r = 0.0, q = 0.0;
  unsigned c = 0;
#pragma unroll 4   // (all 16 triples at once would take 80 registers)
  for (int w = 0; w < NW; ++w) { r += s.a[w]; q += s.b[w]; c += s.u[w]; }
  __syncthreads();
  sum = r;
  sum2 = q;
  cnt = c;
}

// Segment reductions: SEG lanes (4, 16 or 64) of a wavefront that cooperate on one item
// (a fibre of a tensor, a column's partials) reduce on the DPP crossbar with rotations, which
// leave a result in every lane of the segment (for floating-point sums the lanes may differ
// in the last bit: take one lane's value where that matters).
constexpr int DPP_ROR4 = 0x124, DPP_ROR8 = 0x128;

template <int SEG>
__device__ __forceinline__ double seg_sum(double x) {
  x += dpp_f64<DPP_SWAP1>(x);
  x += dpp_f64<DPP_SWAP2>(x);
  if constexpr (SEG >= 16) {
    x += dpp_f64<DPP_ROR4>(x);
    x += dpp_f64<DPP_ROR8>(x);
  }
  if constexpr (SEG == 64) {
    const unsigned long long b = (unsigned long long)__double_as_longlong(x);
    double r = 0.0;
#pragma unroll
    for (int row = 0; row < 4; ++row) {
      const unsigned lo = (unsigned)__builtin_amdgcn_readlane((int)(unsigned)b, row * 16);
      const unsigned hi = (unsigned)__builtin_amdgcn_readlane((int)(unsigned)(b >> 32), row * 16);
      r += __longlong_as_double((long long)(((unsigned long long)hi << 32) | lo));
    }
    x = r;
  }
  return x;
}
template <int SEG>
__device__ __forceinline__ double seg_max(double x) {  // non-negative values
  x = fmax(x, dpp_f64<DPP_SWAP1>(x));
  x = fmax(x, dpp_f64<DPP_SWAP2>(x));
  if constexpr (SEG >= 16) {
    x = fmax(x, dpp_f64<DPP_ROR4>(x));
    x = fmax(x, dpp_f64<DPP_ROR8>(x));
  }
  if constexpr (SEG == 64) {
    const unsigned long long b = (unsigned long long)__double_as_longlong(x);
    double r = 0.0;
#pragma unroll
    for (int row = 0; row < 4; ++row) {
      const unsigned lo = (unsigned)__builtin_amdgcn_readlane((int)(unsigned)b, row * 16);
      const unsigned hi = (unsigned)__builtin_amdgcn_readlane((int)(unsigned)(b >> 32), row * 16);
      r = fmax(r, __longlong_as_double((long long)(((unsigned long long)hi << 32) | lo)));
    }
    x = r;
  }
  return x;
}
template <int SEG>
__device__ __forceinline__ unsigned seg_sum_u(unsigned x) {
  x += dpp_u32<DPP_SWAP1>(x);
  x += dpp_u32<DPP_SWAP2>(x);
  if constexpr (SEG >= 16) {
    x += dpp_u32<DPP_ROR4>(x);
    x += dpp_u32<DPP_ROR8>(x);
  }
  if constexpr (SEG == 64) {
    unsigned r = 0;
#pragma unroll
    for (int row = 0; row < 4; ++row) r += (unsigned)__builtin_amdgcn_readlane((int)x, row * 16);
    x = r;
  }
  return x;
}

}  // namespace mlproj

#endif
