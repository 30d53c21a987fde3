// mlproj: the tri-level l1,inf,inf projection in one pass over memory, for tensors the register
// files hold.
#ifndef MLPROJ_HELD_H
#define MLPROJ_HELD_H

#include "common.h"
#include "reduce.h"
#include "search.h"

namespace mlproj {

// ------------------------------------------------------------------ held slabs
// The tri-level projection (Sec. 5.1, Alg. 5; its two nested maxima are one maximum over the
// slab) reads Y twice in the three-kernel chain: once for the aggregate, once for the clip.  A
// tensor of at most 64 MiB fits the vector registers of the chip (256 CUs x 512 KiB), so here
// every workgroup loads its share of Y ONCE, keeps it in registers (32 chunks of 16 bytes per
// thread, 512 threads: 256 KiB), and clips and stores it from there once tau is known: 8 bytes
// of traffic per fp32 element instead of 12, and two launches instead of three.
//
// Shares.  The tensor is its d0 slabs (the groups) times `parts` contiguous pieces of a slab; a
// workgroup owns one piece, so its aggregate is ONE number, the piece's maximum.
//
// Meeting.  tau needs every piece's maximum, so the workgroups exchange them inside the kernel.
// On this GPU a device-scope fence means an L2 write-back, so nothing is fenced: a piece POSTS
// its maximum as one 32-bit word (the fp32 bit pattern; a cleared word is all ones, which no
// maximum of finite data has) with a device-scope atomic exchange that is performed at the
// memory side and never waited for, and lane g of every workgroup polls piece g's word with
// device-scope atomic loads, which bypass the per-XCD L2.  A word is complete or absent, so no
// counter and no ordering between words is needed.  The words are cleared by a small kernel
// ahead of this one.
//
// Progress without co-residency.  The grid is at most one workgroup per CU, and on an idle GPU
// all of them run at once.  Nothing relies on that: a workgroup that has polled `patience` times
// for a piece's word computes that piece's maximum ITSELF (a streaming read; a maximum is exact,
// so whoever computes it gets the same bits) and posts it on the owner's behalf.  Every wait is
// bounded and everything a workgroup waits for it can produce alone, so every workgroup ends
// whatever the others do, and no second kernel stands behind this one.
//
// In place (X = Y).  Only a piece's owner writes that piece of X, and only after it has seen
// every word, its own included.  A helper reads the piece, THEN looks at the piece's word, and
// posts only if the word is still absent: an absent word after its reads means the owner had not
// seen its own post when they completed, so it had not started to write and the reads saw Y
// itself.  If the word is there the helper's number is dropped.
//
// Measured on an MI355X, 256 x 256 x 256 fp32, cold: 31 us against 39 us for the chain.  The same
// scheme for a MATRIX (column stripes of 16 to 64 columns times row parts, so that column maxima
// stay workgroup-local) was built and measured too and is not here: 38 to 47 us at 4096 x 4096
// against 36 to 37 us for the chain (reads and writes in runs of 64 to 256 bytes, thousands of
// words to post and fetch, and every workgroup waits for the slowest one's loads).
constexpr int HELD_WG = 512;
constexpr int HELD_WAVES = HELD_WG / WAVE;
constexpr int HELD_SLOTS = 32;                       // 16-byte chunks a thread holds
constexpr long long HELD_WG_BYTES = (long long)HELD_WG * HELD_SLOTS * 16;   // 256 KiB per workgroup
constexpr int HELD_MAX_WGS = 256;                    // pieces (= posted words): one per CU, one per polling lane
constexpr unsigned HELD_ABSENT = 0xffffffffu;
constexpr unsigned HELD_PATIENCE = 64;               // polls (1-2 us each) before a workgroup starts helping
constexpr int HELD_MAX_ROUNDS = 16;                  // wait-then-help rounds (two suffice: see held_slab_kernel)

struct HeldPlan {
  int parts;            // pieces per slab
  int slabs;            // d0
  int nwg;              // slabs * parts
  long long per_part;   // elements per piece (a multiple of the elements in 16 bytes)
};

// A tensor of d0 slabs of len elements of elem_bytes each (slabs 16-byte aligned: len a multiple
// of the elements in 16 bytes), on a GPU with max_wgs compute units.
__host__ __device__ static inline bool held_plan_slabs(long long d0, long long len, int elem_bytes, int max_wgs,
                                                       HeldPlan* hp) {
  const int vec = 16 / elem_bytes;
  if (d0 <= 0 || len <= 0 || len % vec != 0) return false;
  if (max_wgs > HELD_MAX_WGS) max_wgs = HELD_MAX_WGS;
  if (d0 > max_wgs) return false;
  const long long cap = HELD_WG_BYTES / elem_bytes;    // elements a workgroup holds
  const long long parts_min = cdiv(len, cap);
  if (parts_min > max_wgs || d0 * parts_min > max_wgs) return false;
  // as many pieces as the grid allows (more workgroups, up to one per CU), none shorter than 16 KiB
  long long parts = max_wgs / d0;
  const long long parts_most = cdiv(len * elem_bytes, 16384);
  if (parts > parts_most) parts = parts_most;
  if (parts < parts_min) parts = parts_min;
  const long long per_part = cdiv(cdiv(len, parts), vec) * vec;
  parts = cdiv(len, per_part);
  hp->parts = (int)parts;
  hp->slabs = (int)d0;
  hp->nwg = (int)(d0 * parts);
  hp->per_part = per_part;
  return true;
}

__device__ __forceinline__ void held_post(unsigned* w, unsigned bits) {
  __hip_atomic_exchange(w, bits, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ unsigned held_peek(const unsigned* w) {
  return __hip_atomic_load(w, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Piece `piece` = (slab, part): where it lies and which chunks its threads hold.  Slot k of a
// thread is the 16-byte chunk k * HELD_WG + thread of the piece when k < nk; a slot that does
// not exist reads the thread's first chunk again and its values are ignored (so that no load is
// conditional).  A slot's address is one add: nothing per slot is kept in registers between the
// loads and the stores.
template <typename T>
struct HeldPiece {
  static constexpr int VEC = 16 / (int)sizeof(T);
  long long first;      // element offset of the thread's first chunk (of the piece's first chunk if it has none)
  int nk;               // slots of this thread that exist (0 .. HELD_SLOTS)
  int slab, part;
  __device__ __forceinline__ HeldPiece(int piece, const HeldPlan& hp, long long len) {
    slab = piece / hp.parts;
    part = piece % hp.parts;
    const long long start = (long long)part * hp.per_part;
    const long long left = len - start;
    const long long count = left < hp.per_part ? left : hp.per_part;    // elements in the piece
    const long long mine = (long long)threadIdx.x * VEC;
    constexpr long long PITCH = (long long)HELD_WG * VEC;
    first = (long long)slab * len + start + (mine < count ? mine : 0);
    const long long cnt = mine < count ? (count - mine + PITCH - 1) / PITCH : 0;
    nk = (int)(cnt < HELD_SLOTS ? cnt : HELD_SLOTS);
  }
  __device__ __forceinline__ bool ok(int k) const { return k < nk; }
  __device__ __forceinline__ const Pack<T, VEC>* at(const T* origin, int k) const {
    return reinterpret_cast<const Pack<T, VEC>*>(reinterpret_cast<const char*>(origin + first) +
                                                 (k < nk ? (unsigned)k * (unsigned)(HELD_WG * 16) : 0u));
  }
  __device__ __forceinline__ T* at(T* origin, int k) const {
    return reinterpret_cast<T*>(reinterpret_cast<char*>(origin + first) +
                                (k < nk ? (unsigned)k * (unsigned)(HELD_WG * 16) : 0u));
  }
  // (between the loads and the stores: makes the compiler form the slot addresses again rather
  // than keep 32 of them alive beside the held data)
  __device__ __forceinline__ void forget() { asm volatile("" : "+v"(nk), "+v"(first)); }
};

template <typename T, int VEC>
__device__ __forceinline__ float held_chunk_max(const Pack<T, VEC>& c, float mx) {
#pragma unroll
  for (int e = 0; e < VEC; ++e) mx = fmaxf(mx, fabsf((float)c.e[e]));
  return mx;
}

// The piece's maximum from what every thread found in its own chunks, posted as word `piece`.
// only_absent: a helper's post.
__device__ __forceinline__ void held_fold_and_post(int piece, float mx, unsigned* posts, bool only_absent,
                                                   float (&sm_w)[HELD_WAVES]) {
  for (int o = 32; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o));
  if ((threadIdx.x & (WAVE - 1)) == 0) sm_w[threadIdx.x / WAVE] = mx;
  __syncthreads();
  if (threadIdx.x == 0) {
    float a = sm_w[0];
#pragma unroll
    for (int w = 1; w < HELD_WAVES; ++w) a = fmaxf(a, sm_w[w]);
    unsigned* w = posts + piece;
    if (!only_absent || held_peek(w) == HELD_ABSENT) held_post(w, __float_as_uint(a));
  }
  __syncthreads();
}

// A piece's maximum by a workgroup that does not own it: a streaming read with the owner's
// thread layout, eight chunks in flight per thread.
template <typename T>
__device__ __forceinline__ void held_help(int piece, const T* __restrict__ Y, const HeldPlan& hp, long long len,
                                          unsigned* posts, float (&sm_w)[HELD_WAVES]) {
  constexpr int VEC = 16 / (int)sizeof(T);
  const HeldPiece<T> hb(piece, hp, len);
  float mx = 0.0f;
  for (int k0 = 0; k0 < HELD_SLOTS; k0 += 8) {
    Pack<T, VEC> t[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) t[k] = *hb.at(Y, k0 + k);
#pragma unroll
    for (int k = 0; k < 8; ++k)
      if (hb.ok(k0 + k)) mx = held_chunk_max<T, VEC>(t[k], mx);
  }
  // (the fold's barrier stands between every thread's reads above and the look at the word)
  held_fold_and_post(piece, mx, posts, true, sm_w);
}

__global__ __launch_bounds__(WG) void held_clear_kernel(unsigned* __restrict__ posts) {
  posts[threadIdx.x] = HELD_ABSENT;    // (HELD_MAX_WGS = WG words)
}

// posts: HELD_MAX_WGS words, cleared to HELD_ABSENT.  d0 slabs of len elements; the plan's grid.
template <typename T, bool XVEC>
__global__ __launch_bounds__(HELD_WG) void held_slab_kernel(const T* Y, T* X, long long d0, long long len,
                                                            HeldPlan hp, double eta, Ws ws, unsigned* posts,
                                                            float* __restrict__ v_out, float* __restrict__ u_out,
                                                            unsigned char* __restrict__ mask_out,
                                                            unsigned patience) {
  constexpr int VEC = 16 / (int)sizeof(T);
  static_assert(HELD_MAX_WGS <= HELD_WG && HELD_MAX_WGS == WG && HELD_MAX_WGS == HELD_POST_WORDS,
                "one polling lane, one cleared word and one workspace word per piece");
  __shared__ float sm_v[HELD_MAX_WGS];       // the aggregate w_a of every slab (exact in fp32)
  __shared__ float sm_w[HELD_WAVES];
  __shared__ PairScratch<HELD_WAVES> bs;
  __shared__ unsigned char sm_missing[HELD_MAX_WGS];
  __shared__ unsigned sm_any;

  const int piece = blockIdx.x;
  HeldPiece<T> hb(piece, hp, len);

  // 1. the piece, into registers (as stored)
  Pack<T, VEC> d[HELD_SLOTS];
#pragma unroll
  for (int k = 0; k < HELD_SLOTS; ++k) d[k] = *hb.at(Y, k);
  __builtin_amdgcn_sched_barrier(0);

  // 2. its maximum, posted
  {
    float mx = 0.0f;
#pragma unroll
    for (int k = 0; k < HELD_SLOTS; ++k)
      if (hb.ok(k)) mx = held_chunk_max<T, VEC>(d[k], mx);
    held_fold_and_post(piece, mx, posts, false, sm_w);
  }

  // 3. w from everybody's words: lane g polls piece g's word and, once it is there, folds it into
  // its slab's maximum in LDS.  When patience is over the pieces still missing are computed here,
  // and the wait starts again for the words just posted.
  for (int a = threadIdx.x; a < HELD_MAX_WGS; a += HELD_WG) sm_v[a] = 0.0f;
  bool complete = false;
  bool taken = false;      // this lane's word is already folded into sm_v
  for (int round = 0; round < HELD_MAX_ROUNDS && !complete; ++round) {
    if (threadIdx.x == 0) sm_any = 0u;
    __syncthreads();
    if ((int)threadIdx.x < HELD_MAX_WGS) {      // (whole wavefronts: HELD_MAX_WGS is a multiple of 64)
      const bool watch = (int)threadIdx.x < hp.nwg;
      bool here = !watch || taken;
      unsigned word = HELD_ABSENT;
      for (unsigned spins = 0;; ++spins) {
        if (!here) {
          word = held_peek(posts + threadIdx.x);
          here = word != HELD_ABSENT;
        }
        if (__all(here) || spins >= patience) break;
        __builtin_amdgcn_s_sleep(8);
      }
      if (watch && here && !taken) {
        // (non-negative floats order as their bit patterns)
        atomicMax(reinterpret_cast<unsigned*>(&sm_v[threadIdx.x / hp.parts]), word);
        taken = true;
      }
      sm_missing[threadIdx.x] = here ? 0 : 1;
      if (!here) sm_any = 1u;
    }
    __syncthreads();
    complete = sm_any == 0u;
    if (!complete) {
      for (int i = 1; i < hp.nwg; ++i) {
        const int g = (piece + i) % hp.nwg;
        if (sm_missing[g]) held_help<T>(g, Y, hp, len, posts, sm_w);   // (uniform: an LDS flag)
      }
    }
    __syncthreads();
  }

  // 4. tau, by every workgroup for itself (the search of the three-kernel chain: same bits)
  SearchOut o = search_block<WG, 4, HELD_WG, float>(sm_v, d0, eta, MODE_PROJECT, MLPROJ_OUTER_L1, bs);
  if (!complete) o.tau = __longlong_as_double(0x7ff8000000000000LL);   // never reached (see above): make it loud
  const Top top = top_of(o);
  if (piece == 0) {
    if (threadIdx.x == 0) write_result(ws, o, nullptr);
    for (int a = threadIdx.x; a < (int)d0; a += HELD_WG) {
      const double va = (double)sm_v[a];
      const double ua = radius(va, top);
      ws.v[a] = va;
      if (v_out) v_out[a] = sm_v[a];
      if (u_out) u_out[a] = (float)ua;
      if (mask_out) mask_out[a] = ua > 0.0 ? 1 : 0;
    }
  }

  // 5. clip from the registers, streamed past the caches
  const float u = (float)radius((double)sm_v[hb.slab], top);
  hb.forget();
#pragma unroll
  for (int k = 0; k < HELD_SLOTS; ++k) {
    if (hb.ok(k)) {
      float f[VEC];
#pragma unroll
      for (int e = 0; e < VEC; ++e) {
        const float y = (float)d[k].e[e];
        f[e] = copysignf(fminf(fabsf(y), u), y);
      }
      store_row_nt<VEC, XVEC>(hb.at(X, k), f);
    }
  }
}

}  // namespace mlproj

#endif
