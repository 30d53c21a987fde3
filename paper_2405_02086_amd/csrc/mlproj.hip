// mlproj: bi-level / tri-level / multi-level projection onto the l_{1,q} ball for gfx950 (MI355X).
// Method: Perez & Barlaud, "Multi-level projection with exponential parallel speedup",
// arXiv 2405.02086 -- Sec. 3 (Eq. 5-9, Alg. 1), Sec. 4 (Alg. 2-4), Sec. 5 (Alg. 5-6) and the
// iterative forms in the appendix.  The paper describes CPU code only; the kernels below are
// an independent design for a 256-CU, 64-lane-wavefront, HBM-bound machine.
//
// One bi-level call is a chain of kernels on the caller's stream; nothing returns to the host:
//   colagg    Y -> per-(column tile, row group) partial aggregates        (reads Y once)
//   reduce    partials -> v_j = ||y_j||_q                                  (tiny)
//   search    v -> tau, the l1-ball threshold; run redundantly at the head of colmap when
//             there are at most 4096 groups, a kernel of its own otherwise      (tiny)
//   [sweep/update]  l1,1 only: per-column inner thresholds, one read of Y per iteration
//   colmap    Y, v, tau -> X                                  (reads Y again, writes X once)
// Workgroups never wait for one another inside a kernel: on this GPU a device-scope fence
// costs an L2 write-back, so cross-workgroup results travel across kernel boundaries only
// (the one exception, the search over more than 16384 groups, meets at a barrier made of
// device-scope atomics alone).  The tri-level form uses the same chain with groups that are
// contiguous slabs; the generic multi-level form works on contiguous fibres, level by level.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdint>
#include <type_traits>

#include "../../include/mlproj.h"

namespace mlproj {

constexpr int WAVE = 64;                 // gfx950 wavefront
constexpr int WG = 256;                  // threads per streaming workgroup
constexpr int WAVES = WG / WAVE;
constexpr int UNROLL = 8;                // rows in flight per wavefront
constexpr int RBLK = WAVES * UNROLL;     // rows one workgroup consumes per trip
constexpr int SWG = 1024;                // threads of the search / reduce workgroups
constexpr int SWAVES = SWG / WAVE;
constexpr int SEARCH_CACHE = 16;         // values of v per search thread kept in registers
constexpr int MAX_INNER_SWEEPS = 12;     // l1,1: passes over Y allowed to the inner searches
constexpr double L11_WINDOW = 1.0 / 16;  // l1,1: relative width of the window that samples the density
constexpr int FILTER_LDS_SLOTS = 8192;   // l1,1: entries a workgroup can stage for its tile (32 KiB of LDS)
constexpr int FILTER_MAX_LIST = 256;     // l1,1: entries kept per column
constexpr unsigned NO_COUNT = 0xffffffffu;
constexpr int QINF = MLPROJ_L1INF, Q1 = MLPROJ_L11, Q2 = MLPROJ_L12;
constexpr int MODE_PROJECT = 0, MODE_NORM = 1;
constexpr int MAP_UNROLL = 4;            // rows in flight per wavefront in the map pass (x2: pipelined)
constexpr int MAP_RBLK = WAVES * MAP_UNROLL;
constexpr long long TARGET_WGS = 512;    // workgroups of a read-only pass on 256 CUs (2 per CU)
constexpr long long TARGET_WGS_MAP = 256;  // workgroups of the read+write pass (1 per CU)
constexpr int COOP_MAX_WGS = 64;         // workgroups of the grid-wide search (far fewer than CUs)
constexpr int COOP_VALUES = 8;           // values of v per thread there
constexpr unsigned SPIN_LIMIT = 1u << 22; // polls before a waiting workgroup gives up (~0.1 s)
constexpr long long FUSED_SEARCH_MAX = (long long)WG * SEARCH_CACHE;  // groups a map workgroup can search in registers
constexpr int SEARCH_CACHE_BIG = 64;     // ... the same with four times the registers, for up to 16384 groups
constexpr long long FUSED_SEARCH_MAX_BIG = (long long)WG * SEARCH_CACHE_BIG;

// ------------------------------------------------------------------ host-side geometry
// A matrix is cut into column tiles of 64*vec columns; each tile is shared by `groups` row
// groups, and row group g takes the row blocks g, g+groups, g+2*groups, ... of RBLK rows, so
// that at any moment the running workgroups sweep a narrow band of rows.  A tensor seen as d0
// contiguous slabs uses tiles = slabs and `groups` chunks of `span` elements per slab.
struct Geometry {
  long long tiles;
  long long groups;
  long long map_groups;  // columns only: row groups of the map pass (its own workgroup count)
  long long span;   // slabs only: elements per chunk
  int vec;          // floats per lane per access: 4 or 1
  int tile_w;       // partial results per (tile, group): 64*vec for columns, 1 for slabs
};

struct Ws {
  mlproj_result* res;
  unsigned* pending;       // [MAX_INNER_SWEEPS + 1] l1,1: columns still searching before sweep s
  double* coop_d;          // [2][COOP_MAX_WGS] grid-wide search: per-workgroup sums, by parity
  double* coop_m;          // [COOP_MAX_WGS]    per-workgroup maxima
  unsigned* coop_u;        // [2][COOP_MAX_WGS] per-workgroup counts, by parity
  unsigned* flags;         // [0] arrivals at the grid-wide search's barrier, [1] that search gave up
  double* v;               // [groups] aggregate, fp64 (exact for q = inf)
  double* tauj;            // [m] l1,1 inner thresholds: the point the next sweep evaluates, then the result
  double* tlo;             // [m] l1,1: lower end of the window whose entries the next sweep lists
  double* lb;              // [m] l1,1: certified lower bound on the threshold
  double* ub;              // [m] l1,1: certified upper bound
  unsigned* kprev;         // [m] l1,1: active count at the point whose Newton step is tlo, or NO_COUNT
  unsigned* done;          // [m] l1,1: 1 once tauj is final
  unsigned* gcnt;          // [m] l1,1: entries in the window, all workgroups
  unsigned* gflag;         // [m] l1,1: some workgroup could not stage all of its window entries
  float* cand;             // [list_cap][m] l1,1: the window entries, slot-major
  int list_cap;            // slots per column in cand
  void* partial;           // [tiles][groups][tile_w] float (q = inf) or double
  unsigned* partial_cnt;   // [tiles][groups][tile_w] l1,1: entries above t
  unsigned* partial_cnt2;  // [tiles][groups][tile_w] l1,1: entries above t*(1 + L11_WINDOW)
};

struct Layout {
  size_t off_pending, off_coop_d, off_coop_m, off_coop_u, off_flags, off_v, off_tauj, off_kprev, off_partial, off_partial_cnt, off_partial_cnt2, bytes;
  size_t off_tlo, off_lb, off_ub, off_done, off_gcnt, off_gflag, off_cand;
  int list_cap;
};

static inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }
static inline long long cdiv(long long a, long long b) { return (a + b - 1) / b; }

// Both passes were tuned on an MI355X: a read-only pass is fastest with about two workgroups
// per CU, the read+write pass with one per CU and fewer rows in flight (a narrower band of
// DRAM pages open at a time).
static Geometry plan_columns(long long n, long long m, int vec, int variant) {
  Geometry g;
  g.vec = vec;
  g.tile_w = WAVE * vec;
  g.tiles = cdiv(m, g.tile_w);
  // Row groups per tile: as many as keep the whole grid within the target, so that every
  // workgroup is resident at once.  One workgroup too many runs alone after all the others
  // and a pass takes twice as long (what an odd number of tiles used to cost).
  long long grp = TARGET_WGS / g.tiles;
  const long long max_grp = cdiv(n, RBLK);
  if (grp > max_grp) grp = max_grp;
  if (grp < 1) grp = 1;
  g.groups = grp;
  (void)variant;
  long long mg = TARGET_WGS_MAP / g.tiles;
  const long long max_mg = cdiv(n, MAP_RBLK);
  if (mg > max_mg) mg = max_mg;
  if (mg < 1) mg = 1;
  g.map_groups = mg;
  g.span = 0;
  return g;
}

static Geometry plan_slabs(long long d0, long long len, int vec) {
  Geometry g;
  g.vec = vec;
  g.tile_w = 1;
  g.tiles = d0;
  g.map_groups = 0;
  long long chunks = cdiv(TARGET_WGS, d0);
  const long long quantum = (long long)WG * vec * 4;  // one unrolled trip of the workgroup
  long long span = cdiv(cdiv(len, chunks), quantum) * quantum;
  g.span = span;
  g.groups = cdiv(len, span);
  return g;
}

// Threads per group in the kernels that fold per-(tile, row group) partials: a power of two,
// at most 16, chosen from the number of partials per group.
static int reduce_parts(long long partials_per_group) {
  int parts = 1;
  while (parts < SWAVES && parts < partials_per_group) parts *= 2;
  return parts;
}

constexpr int LIST_PER_THREAD = 16;      // l1,1: listed entries one lane of the update kernel holds in registers
constexpr int LIST_LANES = 16;           // ... and the lanes that share a column there

static Layout layout_for(const Geometry& g, long long ngroups, int variant) {
  Layout L{};
  size_t o = align_up(sizeof(mlproj_result), 256);
  L.off_pending = o;       o = align_up(o + (MAX_INNER_SWEEPS + 1) * 4, 256);
  L.off_coop_d = o;        o = align_up(o + 2 * COOP_MAX_WGS * 8, 256);
  L.off_coop_m = o;        o = align_up(o + COOP_MAX_WGS * 8, 256);
  L.off_coop_u = o;        o = align_up(o + 2 * COOP_MAX_WGS * 4, 256);
  L.off_flags = o;         o += 256;
  L.off_v = o;             o = align_up(o + (size_t)ngroups * 8, 256);
  L.off_tauj = o;          o = align_up(o + (variant == Q1 ? (size_t)ngroups * 8 : 0), 256);
  L.off_kprev = o;         o = align_up(o + (variant == Q1 ? (size_t)ngroups * 4 : 0), 256);
  const size_t cells = (size_t)g.tiles * (size_t)g.groups * (size_t)g.tile_w;
  L.off_partial = o;       o = align_up(o + cells * 8, 256);
  L.off_partial_cnt = o;   o = align_up(o + (variant == Q1 ? cells * 4 : 0), 256);
  L.off_partial_cnt2 = o;  o = align_up(o + (variant == Q1 ? cells * 4 : 0), 256);
  // l1,1: a column's list takes what its row groups can stage together, up to FILTER_MAX_LIST
  // and what the update kernel's lanes of that column can hold in registers
  long long staged = g.groups * (FILTER_LDS_SLOTS / (g.tile_w > 0 ? g.tile_w : 1));
  if (staged > FILTER_MAX_LIST) staged = FILTER_MAX_LIST;
  if (staged > (long long)LIST_PER_THREAD * LIST_LANES) staged = (long long)LIST_PER_THREAD * LIST_LANES;
  L.list_cap = (int)staged;
  const size_t per_col8 = variant == Q1 ? (size_t)ngroups * 8 : 0, per_col4 = variant == Q1 ? (size_t)ngroups * 4 : 0;
  L.off_tlo = o;           o = align_up(o + per_col8, 256);
  L.off_lb = o;            o = align_up(o + per_col8, 256);
  L.off_ub = o;            o = align_up(o + per_col8, 256);
  L.off_done = o;          o = align_up(o + per_col4, 256);
  L.off_gcnt = o;          o = align_up(o + per_col4, 256);
  L.off_gflag = o;         o = align_up(o + per_col4, 256);
  L.off_cand = o;          o = align_up(o + per_col4 * (size_t)L.list_cap, 256);
  L.bytes = o;
  return L;
}

static Ws bind(void* workspace, const Layout& L) {
  char* b = static_cast<char*>(workspace);
  Ws w;
  w.res = reinterpret_cast<mlproj_result*>(b);
  w.pending = reinterpret_cast<unsigned*>(b + L.off_pending);
  w.coop_d = reinterpret_cast<double*>(b + L.off_coop_d);
  w.coop_m = reinterpret_cast<double*>(b + L.off_coop_m);
  w.coop_u = reinterpret_cast<unsigned*>(b + L.off_coop_u);
  w.flags = reinterpret_cast<unsigned*>(b + L.off_flags);
  w.v = reinterpret_cast<double*>(b + L.off_v);
  w.tauj = reinterpret_cast<double*>(b + L.off_tauj);
  w.kprev = reinterpret_cast<unsigned*>(b + L.off_kprev);
  w.partial = b + L.off_partial;
  w.partial_cnt = reinterpret_cast<unsigned*>(b + L.off_partial_cnt);
  w.partial_cnt2 = reinterpret_cast<unsigned*>(b + L.off_partial_cnt2);
  w.tlo = reinterpret_cast<double*>(b + L.off_tlo);
  w.lb = reinterpret_cast<double*>(b + L.off_lb);
  w.ub = reinterpret_cast<double*>(b + L.off_ub);
  w.done = reinterpret_cast<unsigned*>(b + L.off_done);
  w.gcnt = reinterpret_cast<unsigned*>(b + L.off_gcnt);
  w.gflag = reinterpret_cast<unsigned*>(b + L.off_gflag);
  w.cand = reinterpret_cast<float*>(b + L.off_cand);
  w.list_cap = L.list_cap;
  return w;
}

// ------------------------------------------------------------------ device helpers
// Storage types of Y and X: fp32, or a 16-bit format widened to fp32 on load and rounded to
// nearest-even on store (the arithmetic is the same fp32 / fp64 in every case).
using bf16_t = __bf16;
using f16_t = _Float16;

// One lane's share of a row: VEC consecutive elements, 16 bytes when VEC > 1.
template <typename T, int VEC>
struct alignas(sizeof(T) * VEC) Pack {
  static_assert(VEC == 1 || sizeof(T) * VEC == 16, "a vector access is 16 bytes");
  T e[VEC];
};

template <int VEC, typename T>
__device__ __forceinline__ void load_row(const T* p, float (&x)[VEC]) {
  const Pack<T, VEC> t = *reinterpret_cast<const Pack<T, VEC>*>(p);
#pragma unroll
  for (int k = 0; k < VEC; ++k) x[k] = (float)t.e[k];
}

template <typename T>
__device__ __forceinline__ void store_one_nt(T* p, float x) {
  if constexpr (sizeof(T) == 4) {
    __builtin_nontemporal_store(x, p);
  } else {
    const T t = (T)x;
    unsigned short bits;
    __builtin_memcpy(&bits, &t, 2);
    __builtin_nontemporal_store(bits, reinterpret_cast<unsigned short*>(p));
  }
}

// X is written once and never read again by this call: a non-temporal store keeps it from
// displacing Y in the caches between the two passes over Y.  WIDE = one 16-byte store
// (X 16-byte aligned), otherwise element by element.
template <int VEC, bool WIDE = (VEC > 1), typename T>
__device__ __forceinline__ void store_row_nt(T* p, const float (&x)[VEC]) {
  if constexpr (VEC > 1 && WIDE) {
    typedef unsigned vu4 __attribute__((ext_vector_type(4)));
    Pack<T, VEC> t;
#pragma unroll
    for (int k = 0; k < VEC; ++k) t.e[k] = (T)x[k];
    vu4 w;
    __builtin_memcpy(&w, &t, 16);
    __builtin_nontemporal_store(w, reinterpret_cast<vu4*>(p));
  } else {
#pragma unroll
    for (int k = 0; k < VEC; ++k) store_one_nt(p + k, x[k]);
  }
}

// The columns of a tile that one lane owns, and how it reaches them in a row.
//   wide    : VEC consecutive columns, one 16-byte access per row; needs 16-byte aligned
//             rows (base aligned, row length a multiple of VEC);
//   strided : columns lane, lane + 64, lane + 128, ... of the tile, one element per access,
//             for any alignment and row length.  A wavefront's access is still one coalesced
//             run of 64 elements and a lane has the same bytes in flight as in the wide form.
template <typename T, int VEC, bool STRIDED>
struct LaneCols {
  long long first;      // the first owned column
  bool ok[VEC];         // which owned columns exist (column < m)
  long long from[VEC];  // strided: the column to read for slot k (an existing one, see load)
  __device__ __forceinline__ LaneCols(long long tile0, int lane, long long m) {
    first = STRIDED ? tile0 + lane : tile0 + (long long)lane * VEC;
#pragma unroll
    for (int k = 0; k < VEC; ++k) {
      ok[k] = col(k) < m;
      from[k] = ok[k] ? col(k) : first;
    }
  }
  __device__ __forceinline__ long long col(int k) const {
    return STRIDED ? first + (long long)k * WAVE : first + k;
  }
  // position of owned column k inside the tile
  static __device__ __forceinline__ int slot(int lane, int k) {
    return STRIDED ? lane + k * WAVE : lane * VEC + k;
  }
  __device__ __forceinline__ bool any() const { return ok[0]; }  // owned columns ascend with k
  // The lane's elements of the row that starts at `row`, as stored.  Call only when any().
  // Strided: a slot whose column does not exist reads the lane's first column instead, so
  // that no load is conditional (a conditional load brings its wait with it); what such a slot
  // computes is never stored or read.
  __device__ __forceinline__ void load(const T* row, Pack<T, VEC>& dst) const {
    if constexpr (STRIDED) {
#pragma unroll
      for (int k = 0; k < VEC; ++k) dst.e[k] = row[from[k]];
    } else {
      dst = *reinterpret_cast<const Pack<T, VEC>*>(row + first);
    }
  }
  // XWIDE: one 16-byte store (wide form and X 16-byte aligned), else element by element
  template <bool XWIDE>
  __device__ __forceinline__ void store_nt(T* row, const float (&x)[VEC]) const {
    if constexpr (STRIDED) {
#pragma unroll
      for (int k = 0; k < VEC; ++k)
        if (ok[k]) store_one_nt(row + col(k), x[k]);
    } else {
      store_row_nt<VEC, XWIDE>(row + first, x);
    }
  }
};

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
template <int NW>
__device__ __forceinline__ void block_sum_max(double& sum, double& mx, PairScratch<NW>& s) {
  sum = wave_sum(sum);
  mx = wave_max(mx);
  if ((threadIdx.x & (WAVE - 1)) == 0) { s.a[threadIdx.x / WAVE] = sum; s.b[threadIdx.x / WAVE] = mx; }
  __syncthreads();
  double r = 0.0, q = 0.0;
#pragma unroll
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
template <int Q, typename T, int VEC, bool STRIDED>
__global__ __launch_bounds__(WG) void colagg_kernel(const T* __restrict__ Y, long long n,
                                                    long long m, Geometry g,
                                                    void* __restrict__ partial_) {
  using Acc = typename AccOf<Q>::type;
  constexpr int TILE_W = WAVE * VEC;
  __shared__ Acc sm[WAVES][TILE_W];

  const int lane = threadIdx.x & (WAVE - 1);
  const int wave = threadIdx.x / WAVE;
  const long long t = blockIdx.x % g.tiles;
  const long long grp = blockIdx.x / g.tiles;
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
  for (int c = threadIdx.x; c < TILE_W; c += WG) {
    Acc a = sm[0][c];
#pragma unroll
    for (int w = 1; w < WAVES; ++w) a = combine<Q>(a, sm[w][c]);
    static_cast<Acc*>(partial_)[((size_t)t * g.groups + grp) * TILE_W + c] = a;
  }
}

// v_j from the partials of its tile, folded in a fixed order.  A workgroup of 1024 threads
// covers 1024/parts groups with `parts` threads each (parts = 1..16, a power of two chosen on
// the host from the number of partials per group); every thread keeps 8 loads in flight.
// Serves columns (tile_w = 64*vec) and slabs (tile_w = 1) alike.
template <int Q>
__global__ __launch_bounds__(SWG) void reduce_kernel(const void* __restrict__ partial_,
                                                     long long ngroups, Geometry g, int parts,
                                                     double* __restrict__ v,
                                                     float* __restrict__ v_out,
                                                     unsigned* __restrict__ flags) {
  using Acc = typename AccOf<Q>::type;
  __shared__ Acc sm[SWG];
  if (blockIdx.x == 0 && threadIdx.x < 2) flags[threadIdx.x] = 0u;  // for the grid-wide search
  const int cols = SWG / parts;
  const int c_local = threadIdx.x % cols;
  const int part = threadIdx.x / cols;
  const long long j = (long long)blockIdx.x * cols + c_local;
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
__device__ __forceinline__ Top top_of(const SearchOut& o) { return Top{o.tau, o.scale, o.cap}; }
__device__ __forceinline__ Top top_of(const mlproj_result* r) { return Top{r->tau, r->scale, r->cap}; }

template <int NT, int CACHE = SEARCH_CACHE>
__device__ __forceinline__ SearchOut search_block(const double* __restrict__ v, long long ngroups,
                                                  double eta, int mode, int outer,
                                                  PairScratch<NT / WAVE>& s) {
  const int tid = threadIdx.x;
  double vr[CACHE];
  double a = 0.0, mx = 0.0;
#pragma unroll
  for (int k = 0; k < CACHE; ++k) {
    const long long i = tid + (long long)k * NT;
    vr[k] = i < ngroups ? v[i] : 0.0;  // 0 is never active: tau >= 0 and the test is strict
    a += vr[k];
    mx = fmax(mx, vr[k]);
  }
  for (long long i = tid + (long long)CACHE * NT; i < ngroups; i += NT) {
    const double x = v[i];
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
      const double x = v[i];
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
      c += v[i] > 0.0 ? 1u : 0u;
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
        const double x = v[i];
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
  if (norm_out) *norm_out = o.total;
}

// radii / u_out (optional): also write u_j = max(v_j - tau, 0) for every group.
__global__ __launch_bounds__(SWG) void search_kernel(Ws ws, long long ngroups, double eta,
                                                     int mode, int outer,
                                                     double* __restrict__ norm_out,
                                                     int only_as_fallback,
                                                     double* __restrict__ radii,
                                                     float* __restrict__ u_out) {
  __shared__ PairScratch<SWAVES> s;
  if (only_as_fallback && ws.flags[1] == 0u) return;
  const SearchOut o = search_block<SWG>(ws.v, ngroups, eta, mode, outer, s);
  if (threadIdx.x <= MAX_INNER_SWEEPS) ws.pending[threadIdx.x] = 0u;
  if (threadIdx.x == 0) write_result(ws, o, norm_out);
  if (radii) {
    const Top top = top_of(o);
    for (long long i = threadIdx.x; i < ngroups; i += SWG) {
      const double u = radius(ws.v[i], top);
      radii[i] = u;
      if (u_out) u_out[i] = (float)u;
    }
  }
}

// The same search for very long v (more groups than one workgroup holds in registers): up to
// 64 workgroups, each keeping its slice of v in registers.  Every round each workgroup files
// the sum and count of its slice above tau, all wait at a barrier, and every workgroup adds up
// all slices in the same fixed order, so all of them step tau identically and leave the loop
// together.  Slots alternate by round parity so that a fast workgroup never overwrites what a
// slow one is still reading.
//
// The barrier is built for this GPU, where a device-scope fence means an L2 write-back
// (microseconds, and it serialises): everything the workgroups exchange -- the slots and the
// arrival counter -- is written with device-scope atomic read-modify-writes, which are
// performed at the memory side, and read with device-scope atomic loads, which bypass the
// per-XCD L2; "s_waitcnt vmcnt(0)" makes a wavefront's slot writes complete before its
// arrival is counted.  No ordinary load or store takes part, so no cache has to be flushed.
// The grid is far smaller than the chip, so all workgroups become resident; a workgroup that
// nevertheless waits SPIN_LIMIT polls raises flags[1] and everybody leaves: the kernel always
// ends, and the one-workgroup search_kernel queued behind it then does the work instead.
__device__ __forceinline__ bool wide_barrier(unsigned* flags, unsigned target, unsigned* lds_ok) {
  if (threadIdx.x == 0) {
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __hip_atomic_fetch_add(&flags[0], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    unsigned spins = 0, ok = 1;
    while (__hip_atomic_load(&flags[0], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < target) {
      if (__hip_atomic_load(&flags[1], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0u || ++spins > SPIN_LIMIT) {
        ok = 0;
        break;
      }
      __builtin_amdgcn_s_sleep(1);
    }
    if (!ok) __hip_atomic_exchange(&flags[1], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    *lds_ok = ok;
  }
  __syncthreads();
  const bool ok = *lds_ok != 0u;
  __syncthreads();
  return ok;
}
__device__ __forceinline__ void put_f64(double* p, double x) {
  __hip_atomic_exchange(reinterpret_cast<unsigned long long*>(p),
                        (unsigned long long)__double_as_longlong(x), __ATOMIC_RELAXED,
                        __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ double get_f64(const double* p) {
  return __longlong_as_double((long long)__hip_atomic_load(
      reinterpret_cast<const unsigned long long*>(p), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
}

__global__ __launch_bounds__(SWG) void search_wide_kernel(Ws ws, long long ngroups, double eta,
                                                          int mode, double* __restrict__ norm_out) {
  __shared__ PairScratch<SWAVES> s;
  __shared__ unsigned lds_ok;
  const int tid = threadIdx.x;
  const int nwg = (int)gridDim.x, wg = (int)blockIdx.x;
  const long long chunk = (ngroups + nwg - 1) / nwg;
  const long long lo = (long long)wg * chunk;
  const long long hi = (lo + chunk < ngroups) ? lo + chunk : ngroups;

  double vr[COOP_VALUES];
  double a = 0.0, mx = 0.0;
#pragma unroll
  for (int k = 0; k < COOP_VALUES; ++k) {
    const long long i = lo + tid + (long long)k * SWG;
    vr[k] = i < hi ? ws.v[i] : 0.0;
    a += vr[k];
    mx = fmax(mx, vr[k]);
  }
  for (long long i = lo + tid + (long long)COOP_VALUES * SWG; i < hi; i += SWG) {
    const double x = ws.v[i];
    a += x;
    mx = fmax(mx, x);
  }
  block_sum_max(a, mx, s);
  if (tid == 0) { put_f64(&ws.coop_d[wg], a); put_f64(&ws.coop_m[wg], mx); }
  unsigned round = 1;  // barrier rounds so far; parity 0 carries the totals
  if (!wide_barrier(ws.flags, round * (unsigned)nwg, &lds_ok)) return;
  SearchOut o;
  o.total = tid < nwg ? get_f64(&ws.coop_d[tid]) : 0.0;
  o.vmax = tid < nwg ? get_f64(&ws.coop_m[tid]) : 0.0;
  block_sum_max(o.total, o.vmax, s);
  o.norm = o.total;
  o.tau = 0.0;
  o.scale = 1.0;
  o.cap = HUGE_VAL;
  o.active = 0;
  o.iters = 0;
  o.inside = 0;
  if (mode == MODE_NORM) {
  } else if (eta == 0.0) {
    o.tau = o.vmax;
  } else {
    const bool inside = o.total <= eta;
    double tau = inside ? 0.0 : fmax((o.total - eta) / (double)ngroups, o.vmax - eta);
    unsigned kprev = 0xffffffffu;
    for (;;) {
      double sum = 0.0;
      unsigned cnt = 0;
#pragma unroll
      for (int k = 0; k < COOP_VALUES; ++k) {
        if (vr[k] > tau) { sum += vr[k]; ++cnt; }
      }
      for (long long i = lo + tid + (long long)COOP_VALUES * SWG; i < hi; i += SWG) {
        const double x = ws.v[i];
        if (x > tau) { sum += x; ++cnt; }
      }
      block_sum_count(sum, cnt, s);
      const unsigned par = round & 1u;
      if (tid == 0) {
        put_f64(&ws.coop_d[par * COOP_MAX_WGS + wg], sum);
        __hip_atomic_exchange(&ws.coop_u[par * COOP_MAX_WGS + wg], cnt, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
      ++round;
      if (!wide_barrier(ws.flags, round * (unsigned)nwg, &lds_ok)) return;
      double S = tid < nwg ? get_f64(&ws.coop_d[par * COOP_MAX_WGS + tid]) : 0.0;
      unsigned K = tid < nwg ? __hip_atomic_load(&ws.coop_u[par * COOP_MAX_WGS + tid], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : 0u;
      block_sum_count(S, K, s);
      o.active = K;
      if (inside || K == 0u || K == kprev) break;  // inside: one round, just to count
      kprev = K;
      const double t = (S - eta) / (double)K;
      if (t > tau) tau = t;
      ++o.iters;
    }
    o.tau = tau;
    o.inside = inside ? 1u : 0u;
  }
  if (wg == 0) {
    if (tid <= MAX_INNER_SWEEPS) ws.pending[tid] = 0u;
    if (tid == 0) write_result(ws, o, norm_out);
  }
}

// ------------------------------------------------------------------ per-column map
// x_j = P^q_{u_j}(y_j) (Eq. 8-9) with u_j = max(v_j - tau, 0):
//   q = inf : X = sign(Y) min(|Y|, u_j)          (the symmetric clip; Sec. 4.1)
//   q = 2   : X = Y * u_j / v_j
//   q = 1   : X = sign(Y) max(|Y| - tau_j, 0)    with tau_j from the inner searches
// Row blocks are visited from the bottom up, the reverse of the aggregate pass, so the rows
// read last there (the ones most likely still cached) are read first here.
// With fused_eta >= 0 every workgroup first runs the threshold search itself (see
// search_block) and workgroup 0 files the result record; otherwise tau is read from it.
template <int Q, typename T, int VEC, bool STRIDED, bool XVEC, int SC = SEARCH_CACHE>
__global__ __launch_bounds__(WG) void colmap_kernel(const T* Y, T* X, long long n,
                                                    long long m, Geometry g, Ws ws,
                                                    float* __restrict__ u_out,
                                                    unsigned char* __restrict__ mask_out,
                                                    double fused_eta, int outer) {
  constexpr int TILE_W = WAVE * VEC;
  constexpr int U = MAP_UNROLL;
  __shared__ PairScratch<WAVES> bs;
  const int lane = threadIdx.x & (WAVE - 1);
  const int wave = threadIdx.x / WAVE;
  const long long t = blockIdx.x % g.tiles;
  const long long grp = blockIdx.x / g.tiles;
  const LaneCols<T, VEC, STRIDED> lc(t * TILE_W, lane, m);
  const bool col_ok = lc.any();

  // Row blocks of MAP_RBLK rows, bottom block first; the last block may be ragged.
  const long long nblk = (n + MAP_RBLK - 1) / MAP_RBLK;
  long long b = nblk - 1 - grp;
  // The two buffers hold the elements as stored: widening them here would put a use of the
  // loaded values, and with it the wait for them, ahead of the stores of the current block.
  Pack<T, VEC> x[U], y[U];
  auto load_block = [&](long long blk, Pack<T, VEC> (&dst)[U]) {
#pragma unroll
    for (int r = 0; r < U; ++r) {
      const long long row = blk * MAP_RBLK + wave + (long long)r * WAVES;
      if (row < n) lc.load(Y + row * m, dst[r]);
    }
  };
  // The first block is requested before tau is known, so its latency hides the search.
  if (col_ok && b >= 0) load_block(b, x);

  Top top;
  bool inside;
  if (fused_eta >= 0.0) {
    const SearchOut o = search_block<WG, SC>(ws.v, m, fused_eta, MODE_PROJECT, outer, bs);
    top = top_of(o);
    inside = o.inside != 0u;
    if (blockIdx.x == 0 && threadIdx.x == 0) write_result(ws, o, nullptr);
  } else {
    top = top_of(ws.res);
    inside = ws.res->inside_ball != 0u;
    if constexpr (Q == Q1) {
      // how many columns the inner searches left open (0 = every threshold is exact)
      if (blockIdx.x == 0 && threadIdx.x == 0) {
        const unsigned s = ws.res->inner_sweeps;
        ws.res->inner_pending = (s >= (unsigned)MAX_INNER_SWEEPS) ? ws.pending[MAX_INNER_SWEEPS] : 0u;
      }
    }
  }
  if (!col_ok) return;

  float uf[VEC];
  double par[VEC];  // q = 2: scale u_j / v_j;  q = 1: inner threshold tau_j
#pragma unroll
  for (int k = 0; k < VEC; ++k) {
    const double vj = lc.ok[k] ? ws.v[lc.col(k)] : 0.0;
    const double uj = radius(vj, top);
    uf[k] = (float)uj;
    if constexpr (Q == Q2) par[k] = vj > 0.0 ? uj / vj : 0.0;
    else if constexpr (Q == Q1) par[k] = inside ? 0.0 : ((uj > 0.0 && lc.ok[k]) ? ws.tauj[lc.col(k)] : HUGE_VAL);
    else par[k] = 0.0;
  }
  // q = 1: tau_j as an unevaluated fp32 pair, tau_j = th + tl to 2^-48 relative.  |y| - th is
  // exact while |y| <= 2 th (the only place cancellation can occur) and carries one fp32
  // rounding beyond that, so (|y| - th) - tl stays within two fp32 units of the fp64 result.
  float th[VEC], tl[VEC];
#pragma unroll
  for (int k = 0; k < VEC; ++k) {
    th[k] = (float)par[k];
    tl[k] = (Q == Q1 && par[k] < HUGE_VAL) ? (float)(par[k] - (double)th[k]) : 0.0f;
  }
  if (grp == 0 && wave == 0) {
    if (u_out) {
#pragma unroll
      for (int k = 0; k < VEC; ++k)
        if (lc.ok[k]) u_out[lc.col(k)] = uf[k];
    }
    if (mask_out) {  // the kept columns, decided where the radius is: in fp64
#pragma unroll
      for (int k = 0; k < VEC; ++k)
        if (lc.ok[k]) mask_out[lc.col(k)] = radius(ws.v[lc.col(k)], top) > 0.0 ? 1 : 0;
    }
  }

  auto apply = [&](float yv, int k) -> float {
    if constexpr (Q == QINF) return copysignf(fminf(fabsf(yv), uf[k]), yv);
    else if constexpr (Q == Q2) return (float)((double)yv * par[k]);
    else return copysignf(fmaxf((fabsf(yv) - th[k]) - tl[k], 0.0f), yv);
  };

  // Software pipeline: the next block's loads are issued first, then this block is mapped
  // and stored, and only then does the wavefront wait.  On gfx9 loads and stores share one
  // counter, so any wait for a load also waits for every store issued before it: the wait
  // must come after both have been issued, or the two never overlap.
  // A thread reads and writes the same elements only, so X may alias Y.
  for (; b >= 0; b -= g.map_groups) {
    const long long nb = b - g.map_groups;
    if (nb >= 0) load_block(nb, y);
#pragma unroll
    for (int r = 0; r < U; ++r) {
      const long long row = b * MAP_RBLK + wave + (long long)r * WAVES;
      if (row < n) {
        float f[VEC];
#pragma unroll
        for (int k = 0; k < VEC; ++k) f[k] = apply((float)x[r].e[k], k);
        lc.template store_nt<XVEC>(X + row * m, f);
      }
    }
#pragma unroll
    for (int r = 0; r < U; ++r) x[r] = y[r];
  }
}

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
// return at once when it is zero.
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

// Sweep 0: sum and count of the entries above t = tauj, count above t*(1 + L11_WINDOW).
template <typename T, int VEC, bool STRIDED>
__global__ __launch_bounds__(WG) void l11_sweep_kernel(const T* __restrict__ Y, long long n,
                                                       long long m, Geometry g, Ws ws) {
  constexpr int TILE_W = WAVE * VEC;
  __shared__ double sm_sum[WAVES][TILE_W];
  __shared__ unsigned sm_cnt[WAVES][TILE_W];
  __shared__ unsigned sm_cnt2[WAVES][TILE_W];

  const mlproj_result* res = ws.res;
  if (res->inside_ball != 0u || res->n_active == 0u) return;

  const int lane = threadIdx.x & (WAVE - 1);
  const int wave = threadIdx.x / WAVE;
  const long long t = blockIdx.x % g.tiles;
  const long long grp = blockIdx.x / g.tiles;
  const LaneCols<T, VEC, STRIDED> lc(t * TILE_W, lane, m);

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

// Sweeps 1, 2, ...: sum and count of the entries above hi = tauj, and the entries in
// (tlo, hi] themselves.  A workgroup stages the window entries of its tile's columns in LDS
// (FILTER_LDS_SLOTS / TILE_W slots per column), then reserves room in each column's list with
// one atomic add per column and copies them out.  gcnt ends as the true number of window
// entries of the column whether or not they all fitted; gflag marks a column some workgroup
// could not stage completely.
template <typename T, int VEC, bool STRIDED>
__global__ __launch_bounds__(WG) void l11_filter_kernel(const T* __restrict__ Y, long long n,
                                                        long long m, Geometry g, Ws ws,
                                                        int sweep) {
  constexpr int TILE_W = WAVE * VEC;
  constexpr int CAPW = FILTER_LDS_SLOTS / TILE_W;
  __shared__ double sm_sum[WAVES][TILE_W];
  __shared__ unsigned sm_cnt[WAVES][TILE_W];
  __shared__ float staged[CAPW][TILE_W];   // slot-major: the lanes of a wavefront hit different banks
  __shared__ unsigned staged_cnt[TILE_W];

  const mlproj_result* res = ws.res;
  if (res->inside_ball != 0u || res->n_active == 0u) return;
  if (ws.pending[sweep] == 0u) return;

  const int lane = threadIdx.x & (WAVE - 1);
  const int wave = threadIdx.x / WAVE;
  const long long t = blockIdx.x % g.tiles;
  const long long grp = blockIdx.x / g.tiles;
  const LaneCols<T, VEC, STRIDED> lc(t * TILE_W, lane, m);

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
            if (slot < (unsigned)CAPW) staged[slot][c] = a;
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
    const unsigned r = staged_cnt[c];
    if (col < m && r > 0u) {
      if (r > (unsigned)CAPW) {
        ws.gflag[col] = 1u;
        atomicAdd(&ws.gcnt[col], r);
      } else {
        const unsigned off = atomicAdd(&ws.gcnt[col], r);
        for (unsigned s = 0; s < r && off + s < (unsigned)ws.list_cap; ++s)
          ws.cand[(size_t)(off + s) * (size_t)m + (size_t)col] = staged[s][c];
      }
    }
  }
}

// Starting points of the inner searches.  Dropped columns get +inf (every entry maps to 0).
// For a kept column the guess assumes its entries are Gaussian with the scale its l1 norm
// implies: E|y| = sigma*sqrt(2/pi) = v_j/n and E max(|y| - t, 0) = sigma*h(t/sigma) with
// h(z) = 2*phi(z) - z*erfc(z/sqrt 2), so z solves h(z) = (u_j/v_j)*sqrt(2/pi) (a few Newton
// steps on the convex h) and the guess is sigma*z.  Only the speed depends on the guess.
// The first certified bounds: every entry active gives the lower bound (v_j - u_j)/n.
__global__ __launch_bounds__(WG) void l11_init_kernel(long long n, long long m, Ws ws) {
  const mlproj_result* res = ws.res;
  if (res->inside_ball != 0u || res->n_active == 0u) return;
  const long long j = (long long)blockIdx.x * WG + threadIdx.x;
  if (j >= m) return;
  const double vj = ws.v[j];
  const double uj = radius(vj, top_of(res));
  double tj = HUGE_VAL, floor_t = HUGE_VAL;
  if (uj > 0.0) {
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
    tj = fmax(sigma * (double)z, floor_t);  // never below the all-active bound
  }
  ws.tauj[j] = tj;
  ws.tlo[j] = tj;
  ws.lb[j] = floor_t;
  ws.ub[j] = HUGE_VAL;
  ws.kprev[j] = NO_COUNT;
  ws.done[j] = uj > 0.0 ? 0u : 1u;
  ws.gcnt[j] = 0u;
  ws.gflag[j] = 0u;
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

__global__ __launch_bounds__(WG) void l11_update_kernel(long long n, long long m, Geometry g,
                                                        Ws ws, int sweep) {
  __shared__ BlockScratch<WAVES> bs;
  const mlproj_result* res = ws.res;
  if (res->inside_ball != 0u || res->n_active == 0u) return;
  if (sweep > 0 && ws.pending[sweep] == 0u) return;

  const int part = threadIdx.x % UPD_SEG;
  const int seg_base = (threadIdx.x & (WAVE - 1)) & ~(UPD_SEG - 1);   // first lane of the segment
  const long long j = (long long)blockIdx.x * UPD_COLS + threadIdx.x / UPD_SEG;
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
    complete = ws.gflag[j] == 0u && r <= (unsigned)ws.list_cap;
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
    uj = radius(ws.v[j], top_of(res));
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
    ws.gflag[j] = 0u;
  }
  const unsigned wg_open = block_sum_u(open, bs);
  if (threadIdx.x == 0) {
    if (wg_open) atomicAdd(&ws.pending[sweep + 1], wg_open);
    if (blockIdx.x == 0) ws.res->inner_sweeps = (unsigned)sweep + 1u;
  }
}

// After the last sweep: how many columns were still open (0 = every inner search is exact).
// (Only for a call that stops before the map pass, which otherwise does this itself.)
__global__ void l11_close_kernel(Ws ws) {
  if (threadIdx.x == 0) {
    const unsigned s = ws.res->inner_sweeps;
    ws.res->inner_pending = (s >= (unsigned)MAX_INNER_SWEEPS) ? ws.pending[MAX_INNER_SWEEPS] : 0u;
  }
}

// ------------------------------------------------------------------ tri-level: slab kernels
// Groups are the d0 contiguous slabs of len = d1*d2 elements.  w_a = max over the slab equals
// the two nested maxima of Alg. 5 (max over the fibre, then over the fibres of the slab).
template <int VEC>
__global__ __launch_bounds__(WG) void slabagg_kernel(const float* __restrict__ Y, long long len,
                                                     Geometry g, float* __restrict__ partial) {
  __shared__ BlockScratch<WAVES> bs;
  const long long a = blockIdx.x / g.groups;
  const long long c = blockIdx.x % g.groups;
  const long long lo = c * g.span;
  const long long hi = (lo + g.span < len) ? lo + g.span : len;
  const float* p = Y + a * len;
  float mx = 0.0f;
  long long i = lo + (long long)threadIdx.x * VEC;
  constexpr long long STEP = (long long)WG * VEC;
  for (; i + 3 * STEP < hi; i += 4 * STEP) {
    float x[4][VEC];
#pragma unroll
    for (int r = 0; r < 4; ++r) load_row<VEC>(p + i + r * STEP, x[r]);
#pragma unroll
    for (int r = 0; r < 4; ++r)
#pragma unroll
      for (int k = 0; k < VEC; ++k) mx = fmaxf(mx, fabsf(x[r][k]));
  }
  for (; i < hi; i += STEP) {
    float x[VEC];
    load_row<VEC>(p + i, x);
#pragma unroll
    for (int k = 0; k < VEC; ++k) mx = fmaxf(mx, fabsf(x[k]));
  }
  const double bmax = block_max((double)mx, bs);
  if (threadIdx.x == 0) partial[(size_t)a * g.groups + c] = (float)bmax;
}

// X_abc = sign(Y_abc) min(|Y_abc|, u_a).  The appendix form clips each fibre to
// U2_ab = min(V_ab, u_a); since |Y_abc| <= V_ab the two clips give the same value.
template <int VEC, bool XVEC>
__global__ __launch_bounds__(WG) void slabmap_kernel(const float* Y, float* X, long long d0,
                                                     long long len, Geometry g, Ws ws,
                                                     float* __restrict__ u_out, double fused_eta) {
  __shared__ PairScratch<WAVES> bs;
  const long long a = d0 - 1 - blockIdx.x / g.groups;
  const long long c = blockIdx.x % g.groups;
  const long long lo = c * g.span;
  const long long hi = (lo + g.span < len) ? lo + g.span : len;
  Top top;
  if (fused_eta >= 0.0) {
    const SearchOut o = search_block<WG>(ws.v, d0, fused_eta, MODE_PROJECT, MLPROJ_OUTER_L1, bs);
    top = top_of(o);
    if (blockIdx.x == 0 && threadIdx.x == 0) write_result(ws, o, nullptr);
  } else {
    top = top_of(ws.res);
  }
  const float u = (float)radius(ws.v[a], top);
  if (u_out && c == 0 && threadIdx.x == 0) u_out[a] = u;
  const float* p = Y + a * len;
  float* q = X + a * len;
  long long i = lo + (long long)threadIdx.x * VEC;
  constexpr long long STEP = (long long)WG * VEC;
  for (; i + 3 * STEP < hi; i += 4 * STEP) {
    float x[4][VEC];
#pragma unroll
    for (int r = 0; r < 4; ++r) load_row<VEC>(p + i + r * STEP, x[r]);
#pragma unroll
    for (int r = 0; r < 4; ++r) {
#pragma unroll
      for (int k = 0; k < VEC; ++k) x[r][k] = copysignf(fminf(fabsf(x[r][k]), u), x[r][k]);
      store_row_nt<VEC, XVEC>(q + i + r * STEP, x[r]);
    }
  }
  for (; i < hi; i += STEP) {
    float x[VEC];
    load_row<VEC>(p + i, x);
#pragma unroll
    for (int k = 0; k < VEC; ++k) x[k] = copysignf(fminf(fabsf(x[k]), u), x[k]);
    store_row_nt<VEC, XVEC>(q + i, x);
  }
}

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

// ------------------------------------------------------------------ host: checks + launches
constexpr long long MAX_ELEMS = 1LL << 40;       // 4 TiB of fp32: far beyond one GPU
constexpr long long MAX_GROUPS = (1LL << 31) - 1;
constexpr long long MAX_GRID = (1LL << 31) - 1;
constexpr int STAGE_AGGREGATE = 1, STAGE_APPLY = 2, STAGE_ALL = 3;

static int check_dims(long long a, long long b, long long c) {
  if (a <= 0 || b <= 0 || c <= 0) return MLPROJ_ERR_BAD_DIMENSION;
  if (a > MAX_ELEMS || b > MAX_ELEMS || c > MAX_ELEMS) return MLPROJ_ERR_TOO_LARGE;
  if (a > MAX_ELEMS / b || a * b > MAX_ELEMS / c) return MLPROJ_ERR_TOO_LARGE;
  return MLPROJ_OK;
}

static bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

// Elements per lane and access: 16 bytes when the rows allow it, one element otherwise.
static int pick_vec(const void* Y, long long row_len, int elem_bytes = 4) {
  const int wide = 16 / elem_bytes;
  return (row_len % wide == 0 && aligned(Y, 16)) ? wide : 1;
}

static int workspace_bytes_impl(int variant, long long d0, long long d1, long long d2,
                                size_t* out) {
  if (!out) return MLPROJ_ERR_NULL_POINTER;
  if (variant < MLPROJ_L1INF || variant > MLPROJ_L1INFINF) return MLPROJ_ERR_BAD_VARIANT;
  if (variant != MLPROJ_L1INFINF && d2 != 1) return MLPROJ_ERR_BAD_DIMENSION;
  const int st = check_dims(d0, d1, d2);
  if (st != MLPROJ_OK) return st;
  size_t best = 0;
  for (int vec : {8, 4, 1}) {   // bi-level: 4 (fp32) or 8 (16-bit storage) columns per lane
    Geometry g;
    long long ngroups;
    if (variant != MLPROJ_L1INFINF && vec == 1) continue;
    if (variant == MLPROJ_L1INFINF) {
      if (vec == 8) continue;
      if (d0 > MAX_GROUPS) return MLPROJ_ERR_TOO_LARGE;
      g = plan_slabs(d0, d1 * d2, vec);
      ngroups = d0;
    } else {
      if (d1 > MAX_GROUPS) return MLPROJ_ERR_TOO_LARGE;
      g = plan_columns(d0, d1, vec, variant);
      ngroups = d1;
    }
    if (g.tiles * g.groups > MAX_GRID) return MLPROJ_ERR_TOO_LARGE;
    const Layout L = layout_for(g, ngroups, variant);
    if (L.bytes > best) best = L.bytes;
  }
  *out = best;
  return MLPROJ_OK;
}

static int check_radius(float eta) {
  if (!(eta >= 0.0f) || std::isinf(eta)) return MLPROJ_ERR_BAD_RADIUS;
  return MLPROJ_OK;
}

static int launch_status() { return hipGetLastError() == hipSuccess ? MLPROJ_OK : MLPROJ_ERR_LAUNCH; }

// Optional per-kernel timing: while a trace is open on the calling thread, an event is
// recorded on the stream before every kernel of a call and after its last one.
struct Trace {
  hipEvent_t* events = nullptr;
  int capacity = 0;
  int count = 0;
};
static thread_local Trace g_trace;

static inline void mark(hipStream_t stream) {
  if (g_trace.events && g_trace.count < g_trace.capacity)
    (void)hipEventRecord(g_trace.events[g_trace.count++], stream);
}

// The stand-alone search: one workgroup when v fits its registers, the grid-wide form beyond
// that, followed by the one-workgroup kernel as a fallback that returns at once unless the
// grid-wide one gave up.
static void launch_search(const Ws& ws, long long ngroups, double eta, int mode, int outer,
                          double* norm_out, hipStream_t stream) {
  int only_as_fallback = 0;
  // (the l2 and l_inf outer projections need no iteration: one workgroup reads v once)
  if (ngroups > (long long)SWG * SEARCH_CACHE && (outer == MLPROJ_OUTER_L1 || mode == MODE_NORM)) {
    long long nwg = cdiv(ngroups, (long long)SWG * COOP_VALUES);
    if (nwg > COOP_MAX_WGS) nwg = COOP_MAX_WGS;
    hipLaunchKernelGGL(search_wide_kernel, dim3((unsigned)nwg), dim3(SWG), 0, stream, ws, ngroups, eta, mode, norm_out);
    only_as_fallback = 1;
  }
  hipLaunchKernelGGL(search_kernel, dim3(1), dim3(SWG), 0, stream, ws, ngroups, eta, mode, outer, norm_out,
                     only_as_fallback, (double*)nullptr, (float*)nullptr);
}

// STAGE_AGGREGATE = aggregate + threshold search (+ inner searches for l1,1);
// STAGE_APPLY = the per-column map.
template <int Q, typename T = float>
static int run_bilevel(const T* Y, T* X, long long n, long long m, float eta,
                       void* workspace, size_t workspace_bytes, float* v_out, float* u_out,
                       void* stream_, int mode, double* norm_out, int stages, int outer,
                       unsigned char* mask_out = nullptr) {
  constexpr int WIDE = 16 / (int)sizeof(T);
  if (outer < MLPROJ_OUTER_L1 || outer > MLPROJ_OUTER_LINF) return MLPROJ_ERR_BAD_VARIANT;
  const bool need_x = mode == MODE_PROJECT && (stages & STAGE_APPLY);
  if (!Y || !workspace || (need_x && !X)) return MLPROJ_ERR_NULL_POINTER;
  int st = check_dims(n, m, 1);
  if (st != MLPROJ_OK) return st;
  if (m > MAX_GROUPS) return MLPROJ_ERR_TOO_LARGE;
  if (mode == MODE_PROJECT && (stages & STAGE_AGGREGATE) && (st = check_radius(eta)) != MLPROJ_OK)
    return st;
  if (!aligned(Y, sizeof(T)) || (X && !aligned(X, sizeof(T)))) return MLPROJ_ERR_ALIGNMENT;
  if (!aligned(workspace, 256)) return MLPROJ_ERR_WORKSPACE;
  // Every lane owns WIDE columns; rows that are not 16-byte aligned are read element-wise
  // (the strided form of LaneCols), and a misaligned X alone only narrows the stores.  The
  // geometry depends on n and m only, so the two stages of a split call agree on it.
  const bool wide = pick_vec(Y, m, (int)sizeof(T)) == WIDE;
  const bool x_vec = !X || aligned(X, 16);
  const Geometry g = plan_columns(n, m, WIDE, Q);
  if (g.tiles * g.groups > MAX_GRID) return MLPROJ_ERR_TOO_LARGE;
  const Layout L = layout_for(g, m, Q);
  if (workspace_bytes < L.bytes) return MLPROJ_ERR_WORKSPACE;
  const Ws ws = bind(workspace, L);
  hipStream_t stream = static_cast<hipStream_t>(stream_);
  const dim3 grid((unsigned)(g.tiles * g.groups)), block(WG);
  const dim3 mgrid((unsigned)(g.tiles * g.map_groups));
  const int parts = reduce_parts(g.groups);
  const dim3 rgrid((unsigned)cdiv(m, SWG / parts)), rblock(SWG);
  // A whole call on few enough groups lets every map workgroup find tau by itself, which
  // takes the one-workgroup search kernel off the critical path (16 values of v per thread
  // up to 4096 groups, 64 per thread up to 16384).
  const bool fuse = mode == MODE_PROJECT && stages == STAGE_ALL && Q != Q1 && m <= FUSED_SEARCH_MAX_BIG;
  const bool fuse_big = fuse && m > FUSED_SEARCH_MAX;
  const double fused_eta = fuse ? (double)eta : -1.0;

  if (stages & STAGE_AGGREGATE) {
    mark(stream);
    if (wide)
      hipLaunchKernelGGL((colagg_kernel<Q, T, WIDE, false>), grid, block, 0, stream, Y, n, m, g, ws.partial);
    else
      hipLaunchKernelGGL((colagg_kernel<Q, T, WIDE, true>), grid, block, 0, stream, Y, n, m, g, ws.partial);
    mark(stream);
    hipLaunchKernelGGL((reduce_kernel<Q>), rgrid, rblock, 0, stream, ws.partial, m, g, parts, ws.v, v_out, ws.flags);
    if (!fuse) {
      mark(stream);
      launch_search(ws, m, (double)eta, mode, outer, norm_out, stream);
    }
    if (mode == MODE_NORM) { mark(stream); return launch_status(); }
    if constexpr (Q == Q1) {
      mark(stream);
      hipLaunchKernelGGL(l11_init_kernel, dim3((unsigned)cdiv(m, WG)), block, 0, stream, n, m, ws);
      for (int s = 0; s < MAX_INNER_SWEEPS; ++s) {
        if (s == 0) {
          if (wide) hipLaunchKernelGGL((l11_sweep_kernel<T, WIDE, false>), grid, block, 0, stream, Y, n, m, g, ws);
          else hipLaunchKernelGGL((l11_sweep_kernel<T, WIDE, true>), grid, block, 0, stream, Y, n, m, g, ws);
        } else {
          if (wide) hipLaunchKernelGGL((l11_filter_kernel<T, WIDE, false>), grid, block, 0, stream, Y, n, m, g, ws, s);
          else hipLaunchKernelGGL((l11_filter_kernel<T, WIDE, true>), grid, block, 0, stream, Y, n, m, g, ws, s);
        }
        hipLaunchKernelGGL(l11_update_kernel, dim3((unsigned)cdiv(m, UPD_COLS)), block, 0, stream, n, m, g, ws, s);
      }
      if (!(stages & STAGE_APPLY)) hipLaunchKernelGGL(l11_close_kernel, dim3(1), dim3(WAVE), 0, stream, ws);
    }
  }
  if (stages & STAGE_APPLY) {
    mark(stream);
    if (fuse_big && wide && x_vec)
      hipLaunchKernelGGL((colmap_kernel<Q, T, WIDE, false, true, SEARCH_CACHE_BIG>), mgrid, block, 0, stream, Y, X, n, m, g, ws, u_out, mask_out, fused_eta, outer);
    else if (fuse_big && wide)
      hipLaunchKernelGGL((colmap_kernel<Q, T, WIDE, false, false, SEARCH_CACHE_BIG>), mgrid, block, 0, stream, Y, X, n, m, g, ws, u_out, mask_out, fused_eta, outer);
    else if (fuse_big)
      hipLaunchKernelGGL((colmap_kernel<Q, T, WIDE, true, false, SEARCH_CACHE_BIG>), mgrid, block, 0, stream, Y, X, n, m, g, ws, u_out, mask_out, fused_eta, outer);
    else if (wide && x_vec)
      hipLaunchKernelGGL((colmap_kernel<Q, T, WIDE, false, true>), mgrid, block, 0, stream, Y, X, n, m, g, ws, u_out, mask_out, fused_eta, outer);
    else if (wide)
      hipLaunchKernelGGL((colmap_kernel<Q, T, WIDE, false, false>), mgrid, block, 0, stream, Y, X, n, m, g, ws, u_out, mask_out, fused_eta, outer);
    else
      hipLaunchKernelGGL((colmap_kernel<Q, T, WIDE, true, false>), mgrid, block, 0, stream, Y, X, n, m, g, ws, u_out, mask_out, fused_eta, outer);
  }
  mark(stream);
  return launch_status();
}

template <typename... A>
static int dispatch_q(int variant, A... a) {
  switch (variant) {
    case MLPROJ_L1INF: return run_bilevel<QINF>(a...);
    case MLPROJ_L11: return run_bilevel<Q1>(a...);
    case MLPROJ_L12: return run_bilevel<Q2>(a...);
    default: return MLPROJ_ERR_BAD_VARIANT;
  }
}

template <typename T>
static int dispatch_stored(int outer, int variant, const void* Y, void* X, long long n, long long m,
                           float eta, void* workspace, size_t workspace_bytes, float* v_out,
                           float* u_out, unsigned char* mask_out, void* stream) {
  return dispatch_q(variant, static_cast<const T*>(Y), static_cast<T*>(X), n, m, eta, workspace,
                    workspace_bytes, v_out, u_out, stream, MODE_PROJECT, (double*)nullptr, STAGE_ALL,
                    outer, mask_out);
}

// ------------------------------------------------------------------ host: multi-level driver
constexpr int ML_MAX_DIMS = 8;
constexpr long long ML_TARGET_WGS = 1024;

struct MlPlan {
  int ndim;
  long long size[ML_MAX_DIMS];   // size[k] = elements of level k = prod dims[0 .. ndim-1-k]
  long long len[ML_MAX_DIMS];    // len[k]  = fibre length aggregated to make level k (k >= 1)
  size_t off_V[ML_MAX_DIMS], off_R[ML_MAX_DIMS];  // fp64 arrays of level k (k = 1 .. ndim-1)
  Layout base;
  size_t bytes;
};

static int ml_plan(int ndim, const long long* dims, const int* norms, MlPlan* P) {
  if (!dims || !norms) return MLPROJ_ERR_NULL_POINTER;
  if (ndim < 2 || ndim > ML_MAX_DIMS) return MLPROJ_ERR_BAD_DIMENSION;
  long long total = 1;
  for (int i = 0; i < ndim; ++i) {
    if (dims[i] <= 0) return MLPROJ_ERR_BAD_DIMENSION;
    if (dims[i] > MAX_ELEMS || total > MAX_ELEMS / dims[i]) return MLPROJ_ERR_TOO_LARGE;
    total *= dims[i];
  }
  if (dims[0] > MAX_GROUPS) return MLPROJ_ERR_TOO_LARGE;
  for (int k = 0; k < ndim - 1; ++k)
    if (norms[k] != MLPROJ_NORM_INF && norms[k] != MLPROJ_NORM_L1 && norms[k] != MLPROJ_NORM_L2)
      return MLPROJ_ERR_BAD_VARIANT;
  P->ndim = ndim;
  long long sz = total;
  for (int k = 0; k < ndim; ++k) {
    P->size[k] = sz;
    P->len[k] = k == 0 ? 0 : dims[ndim - k];
    if (k + 1 < ndim) sz /= dims[ndim - 1 - k];
  }
  Geometry g{};  // no column partials: only the record, the search scratch and v[d0] are used
  g.tiles = 1; g.groups = 1; g.tile_w = 1; g.vec = 1;
  P->base = layout_for(g, dims[0], MLPROJ_L1INF);
  size_t o = P->base.bytes;
  for (int k = 1; k < ndim; ++k) {
    P->off_V[k] = o; o = align_up(o + (size_t)P->size[k] * 8, 256);
    P->off_R[k] = o; o = align_up(o + (size_t)P->size[k] * 8, 256);
  }
  P->bytes = o;
  return MLPROJ_OK;
}

// lanes per fibre: few enough that every lane has up to four chunks to itself
static int seg_for(long long nvec) { return nvec <= 16 ? 4 : (nvec <= 64 ? 16 : 64); }

static unsigned fibre_grid(long long nf, int seg, int unroll) {
  const long long per_wg = (long long)WAVES * (WAVE / seg) * unroll;
  long long wgs = cdiv(nf, per_wg);
  if (wgs > ML_TARGET_WGS) wgs = ML_TARGET_WGS;
  return (unsigned)(wgs < 1 ? 1 : wgs);
}

template <int Q, typename TIN, int VEC>
static void launch_fibre_agg(const TIN* A, long long nf, long long len, double* V, float* v_out,
                             hipStream_t stream) {
  const int seg = seg_for(len / VEC);
  const dim3 grid(fibre_grid(nf, seg, FIB_UNROLL)), block(WG);
  if (seg == 4) hipLaunchKernelGGL((fibre_agg_kernel<Q, TIN, 4, VEC>), grid, block, 0, stream, A, nf, len, V, v_out);
  else if (seg == 16) hipLaunchKernelGGL((fibre_agg_kernel<Q, TIN, 16, VEC>), grid, block, 0, stream, A, nf, len, V, v_out);
  else hipLaunchKernelGGL((fibre_agg_kernel<Q, TIN, 64, VEC>), grid, block, 0, stream, A, nf, len, V, v_out);
}

template <int Q, typename TIN, typename TOUT, int VEC>
static void launch_fibre_map(const TIN* A, long long nf, long long len, const double* R,
                             const double* Vn, TOUT* out, hipStream_t stream) {
  const long long nvec = len / VEC;
  const int seg = seg_for(nvec);
  if (nvec <= (long long)seg * 4) {
    // the fibre fits the registers of its segment
    const dim3 cgrid(fibre_grid(nf, seg, FIB_MAP_UNROLL)), cblock(WG);
    const int kreg = nvec <= seg ? 1 : (nvec <= 2LL * seg ? 2 : 4);
#define MLPROJ_LAUNCH_CACHED(SEG_, K_)                                                              \
  hipLaunchKernelGGL((fibre_map_cached_kernel<Q, TIN, TOUT, SEG_, VEC, K_>), cgrid, cblock, 0, stream, \
                     A, nf, len, R, Vn, out)
    if (seg == 4) { if (kreg == 1) MLPROJ_LAUNCH_CACHED(4, 1); else if (kreg == 2) MLPROJ_LAUNCH_CACHED(4, 2); else MLPROJ_LAUNCH_CACHED(4, 4); }
    else if (seg == 16) { if (kreg == 1) MLPROJ_LAUNCH_CACHED(16, 1); else if (kreg == 2) MLPROJ_LAUNCH_CACHED(16, 2); else MLPROJ_LAUNCH_CACHED(16, 4); }
    else { if (kreg == 1) MLPROJ_LAUNCH_CACHED(64, 1); else if (kreg == 2) MLPROJ_LAUNCH_CACHED(64, 2); else MLPROJ_LAUNCH_CACHED(64, 4); }
#undef MLPROJ_LAUNCH_CACHED
    return;
  }
  const dim3 grid(fibre_grid(nf, seg, 1)), block(WG);
  if (seg == 4) hipLaunchKernelGGL((fibre_map_kernel<Q, TIN, TOUT, 4, VEC>), grid, block, 0, stream, A, nf, len, R, Vn, out);
  else if (seg == 16) hipLaunchKernelGGL((fibre_map_kernel<Q, TIN, TOUT, 16, VEC>), grid, block, 0, stream, A, nf, len, R, Vn, out);
  else hipLaunchKernelGGL((fibre_map_kernel<Q, TIN, TOUT, 64, VEC>), grid, block, 0, stream, A, nf, len, R, Vn, out);
}

template <typename F>
static void by_norm(int norm, F&& f) {
  if (norm == MLPROJ_NORM_INF) f(std::integral_constant<int, QINF>{});
  else if (norm == MLPROJ_NORM_L1) f(std::integral_constant<int, Q1>{});
  else f(std::integral_constant<int, Q2>{});
}

static int run_multilevel(int outer, const float* Y, float* X, int ndim, const long long* dims,
                          const int* norms, float eta, void* workspace, size_t workspace_bytes,
                          float* v_out, float* u_out, void* stream_) {
  if (!Y || !X || !workspace) return MLPROJ_ERR_NULL_POINTER;
  if (outer < MLPROJ_OUTER_L1 || outer > MLPROJ_OUTER_LINF) return MLPROJ_ERR_BAD_VARIANT;
  MlPlan P;
  int st = ml_plan(ndim, dims, norms, &P);
  if (st != MLPROJ_OK) return st;
  if ((st = check_radius(eta)) != MLPROJ_OK) return st;
  if (!aligned(Y, 4) || !aligned(X, 4)) return MLPROJ_ERR_ALIGNMENT;
  if (!aligned(workspace, 256) || workspace_bytes < P.bytes) return MLPROJ_ERR_WORKSPACE;
  const Ws ws = bind(workspace, P.base);
  char* base = static_cast<char*>(workspace);
  double* V[ML_MAX_DIMS];
  double* R[ML_MAX_DIMS];
  for (int k = 1; k < ndim; ++k) {
    V[k] = reinterpret_cast<double*>(base + P.off_V[k]);
    R[k] = reinterpret_cast<double*>(base + P.off_R[k]);
  }
  V[ndim - 1] = ws.v;  // the top aggregate is the vector the search reads
  hipStream_t stream = static_cast<hipStream_t>(stream_);
  const long long len1 = P.len[1];
  const bool vec4 = len1 % 4 == 0 && aligned(Y, 16) && aligned(X, 16);

  // up: aggregate level by level
  mark(stream);
  by_norm(norms[0], [&](auto q) {
    float* vo = ndim == 2 ? v_out : nullptr;
    if (vec4) launch_fibre_agg<decltype(q)::value, float, 4>(Y, P.size[1], len1, V[1], vo, stream);
    else launch_fibre_agg<decltype(q)::value, float, 1>(Y, P.size[1], len1, V[1], vo, stream);
  });
  for (int k = 2; k < ndim; ++k) {
    by_norm(norms[k - 1], [&](auto q) {
      launch_fibre_agg<decltype(q)::value, double, 1>(V[k - 1], P.size[k], P.len[k], V[k],
                                                      k == ndim - 1 ? v_out : nullptr, stream);
    });
  }
  // top: threshold of the l1-ball projection of the length-d0 vector, then its radii
  mark(stream);
  if (dims[0] <= (long long)SWG * SEARCH_CACHE || outer != MLPROJ_OUTER_L1) {
    hipLaunchKernelGGL(search_kernel, dim3(1), dim3(SWG), 0, stream, ws, dims[0], (double)eta, MODE_PROJECT,
                       outer, (double*)nullptr, 0, R[ndim - 1], u_out);
  } else {
    hipLaunchKernelGGL(clear_flags_kernel, dim3(1), dim3(WAVE), 0, stream, ws);
    launch_search(ws, dims[0], (double)eta, MODE_PROJECT, outer, nullptr, stream);
    hipLaunchKernelGGL(top_radii_kernel, dim3((unsigned)cdiv(dims[0], WG)), dim3(WG), 0, stream, ws,
                       dims[0], R[ndim - 1], u_out);
  }
  // down: project the fibres of every level onto the balls of the level above
  mark(stream);
  for (int k = ndim - 1; k >= 2; --k) {
    by_norm(norms[k - 1], [&](auto q) {
      launch_fibre_map<decltype(q)::value, double, double, 1>(V[k - 1], P.size[k], P.len[k], R[k], V[k],
                                                              R[k - 1], stream);
    });
  }
  by_norm(norms[0], [&](auto q) {
    if (vec4) launch_fibre_map<decltype(q)::value, float, float, 4>(Y, P.size[1], len1, R[1], V[1], X, stream);
    else launch_fibre_map<decltype(q)::value, float, float, 1>(Y, P.size[1], len1, R[1], V[1], X, stream);
  });
  mark(stream);
  return launch_status();
}

}  // namespace mlproj

// ------------------------------------------------------------------ C ABI
using namespace mlproj;

extern "C" {

int mlproj_version(void) { return 330; }

const char* mlproj_status_string(int status) {
  switch (status) {
    case MLPROJ_OK: return "ok";
    case MLPROJ_ERR_NULL_POINTER: return "a required pointer is NULL";
    case MLPROJ_ERR_BAD_DIMENSION: return "a dimension is not positive";
    case MLPROJ_ERR_TOO_LARGE: return "input exceeds the supported size";
    case MLPROJ_ERR_BAD_RADIUS: return "eta must be finite and >= 0";
    case MLPROJ_ERR_WORKSPACE: return "workspace too small or not 256-byte aligned";
    case MLPROJ_ERR_BAD_VARIANT: return "unknown variant";
    case MLPROJ_ERR_ALIGNMENT: return "Y and X must be aligned to their element size";
    case MLPROJ_ERR_LAUNCH: return "HIP refused a kernel launch";
    default: return "unknown status";
  }
}

int mlproj_trace_begin(void** events, int capacity) {
  if (!events) return MLPROJ_ERR_NULL_POINTER;
  if (capacity <= 0) return MLPROJ_ERR_BAD_DIMENSION;
  g_trace.events = reinterpret_cast<hipEvent_t*>(events);
  g_trace.capacity = capacity;
  g_trace.count = 0;
  return MLPROJ_OK;
}

int mlproj_trace_end(void) {
  const int n = g_trace.count;
  g_trace = Trace{};
  return n;
}

int mlproj_workspace_bytes(int variant, long long d0, long long d1, long long d2, size_t* bytes_out) {
  return workspace_bytes_impl(variant, d0, d1, d2, bytes_out);
}

int mlproj_norm_l1q(const float* Y, long long n, long long m, int q_variant, void* workspace,
                    size_t workspace_bytes, double* norm_out, float* v_out, void* stream) {
  return dispatch_q(q_variant, Y, (float*)nullptr, n, m, 0.f, workspace, workspace_bytes, v_out,
                    (float*)nullptr, stream, MODE_NORM, norm_out, STAGE_AGGREGATE, (int)MLPROJ_OUTER_L1);
}

int bilevel_proj_l1inf(const float* Y, float* X, long long n, long long m, float eta,
                       void* workspace, size_t workspace_bytes, float* v_out, float* u_out,
                       void* stream) {
  return run_bilevel<QINF>(Y, X, n, m, eta, workspace, workspace_bytes, v_out, u_out, stream,
                           MODE_PROJECT, nullptr, STAGE_ALL, (int)MLPROJ_OUTER_L1);
}

int bilevel_proj_l11(const float* Y, float* X, long long n, long long m, float eta,
                     void* workspace, size_t workspace_bytes, float* v_out, float* u_out,
                     void* stream) {
  return run_bilevel<Q1>(Y, X, n, m, eta, workspace, workspace_bytes, v_out, u_out, stream,
                         MODE_PROJECT, nullptr, STAGE_ALL, (int)MLPROJ_OUTER_L1);
}

int bilevel_proj_l12(const float* Y, float* X, long long n, long long m, float eta,
                     void* workspace, size_t workspace_bytes, float* v_out, float* u_out,
                     void* stream) {
  return run_bilevel<Q2>(Y, X, n, m, eta, workspace, workspace_bytes, v_out, u_out, stream,
                         MODE_PROJECT, nullptr, STAGE_ALL, (int)MLPROJ_OUTER_L1);
}

int bilevel_radii(int variant, const float* Y, long long n, long long m, float eta,
                  void* workspace, size_t workspace_bytes, float* v_out, void* stream) {
  return dispatch_q(variant, Y, (float*)nullptr, n, m, eta, workspace, workspace_bytes, v_out,
                    (float*)nullptr, stream, MODE_PROJECT, (double*)nullptr, STAGE_AGGREGATE, (int)MLPROJ_OUTER_L1);
}

int bilevel_apply(int variant, const float* Y, float* X, long long n, long long m,
                  void* workspace, size_t workspace_bytes, float* u_out, void* stream) {
  return dispatch_q(variant, Y, X, n, m, 0.f, workspace, workspace_bytes, (float*)nullptr, u_out,
                    stream, MODE_PROJECT, (double*)nullptr, STAGE_APPLY, (int)MLPROJ_OUTER_L1);
}

int mlproj_multilevel_workspace_bytes(int ndim, const long long* dims, size_t* bytes_out) {
  if (!bytes_out) return MLPROJ_ERR_NULL_POINTER;
  int norms[ML_MAX_DIMS] = {0};
  MlPlan P;
  const int st = ml_plan(ndim, dims, norms, &P);
  if (st != MLPROJ_OK) return st;
  *bytes_out = P.bytes;
  return MLPROJ_OK;
}

int multilevel_proj(const float* Y, float* X, int ndim, const long long* dims, const int* norms,
                    float eta, void* workspace, size_t workspace_bytes, float* v_out, float* u_out,
                    void* stream) {
  return run_multilevel(MLPROJ_OUTER_L1, Y, X, ndim, dims, norms, eta, workspace, workspace_bytes, v_out, u_out, stream);
}

int multilevel_proj_p(int outer_norm, const float* Y, float* X, int ndim, const long long* dims,
                      const int* norms, float eta, void* workspace, size_t workspace_bytes,
                      float* v_out, float* u_out, void* stream) {
  return run_multilevel(outer_norm, Y, X, ndim, dims, norms, eta, workspace, workspace_bytes, v_out, u_out, stream);
}

int bilevel_proj_pq(int outer_norm, int variant, const float* Y, float* X, long long n, long long m,
                    float eta, void* workspace, size_t workspace_bytes, float* v_out, float* u_out,
                    void* stream) {
  return dispatch_q(variant, Y, X, n, m, eta, workspace, workspace_bytes, v_out, u_out, stream,
                    MODE_PROJECT, (double*)nullptr, STAGE_ALL, outer_norm);
}

int bilevel_proj_stored(int storage, int outer_norm, int variant, const void* Y, void* X,
                        long long n, long long m, float eta, void* workspace,
                        size_t workspace_bytes, float* v_out, float* u_out,
                        unsigned char* mask_out, void* stream) {
  switch (storage) {
    case MLPROJ_STORE_F32:
      return dispatch_stored<float>(outer_norm, variant, Y, X, n, m, eta, workspace, workspace_bytes, v_out, u_out, mask_out, stream);
    case MLPROJ_STORE_BF16:
      return dispatch_stored<bf16_t>(outer_norm, variant, Y, X, n, m, eta, workspace, workspace_bytes, v_out, u_out, mask_out, stream);
    case MLPROJ_STORE_F16:
      return dispatch_stored<f16_t>(outer_norm, variant, Y, X, n, m, eta, workspace, workspace_bytes, v_out, u_out, mask_out, stream);
    default: return MLPROJ_ERR_BAD_VARIANT;
  }
}

int trilevel_proj_l1infinf(const float* Y, float* X, long long d0, long long d1, long long d2,
                           float eta, void* workspace, size_t workspace_bytes, float* v_out,
                           float* u_out, void* stream_) {
  if (!Y || !X || !workspace) return MLPROJ_ERR_NULL_POINTER;
  int st = check_dims(d0, d1, d2);
  if (st != MLPROJ_OK) return st;
  if (d0 > MAX_GROUPS) return MLPROJ_ERR_TOO_LARGE;
  if ((st = check_radius(eta)) != MLPROJ_OK) return st;
  if (!aligned(Y, 4) || !aligned(X, 4)) return MLPROJ_ERR_ALIGNMENT;
  if (!aligned(workspace, 256)) return MLPROJ_ERR_WORKSPACE;
  const long long len = d1 * d2;
  const int vec = pick_vec(Y, len);
  const bool x_vec = aligned(X, 16);
  const Geometry g = plan_slabs(d0, len, vec);
  if (g.tiles * g.groups > MAX_GRID) return MLPROJ_ERR_TOO_LARGE;
  const Layout L = layout_for(g, d0, MLPROJ_L1INFINF);
  if (workspace_bytes < L.bytes) return MLPROJ_ERR_WORKSPACE;
  const Ws ws = bind(workspace, L);
  hipStream_t stream = static_cast<hipStream_t>(stream_);
  const dim3 grid((unsigned)(g.tiles * g.groups)), block(WG);
  const int parts = reduce_parts(g.groups);
  const dim3 rgrid((unsigned)cdiv(d0, SWG / parts)), rblock(SWG);
  float* partial = static_cast<float*>(ws.partial);
  mark(stream);
  if (vec == 4) hipLaunchKernelGGL((slabagg_kernel<4>), grid, block, 0, stream, Y, len, g, partial);
  else hipLaunchKernelGGL((slabagg_kernel<1>), grid, block, 0, stream, Y, len, g, partial);
  mark(stream);
  hipLaunchKernelGGL((reduce_kernel<QINF>), rgrid, rblock, 0, stream, ws.partial, d0, g, parts, ws.v, v_out, ws.flags);
  const bool fuse = d0 <= FUSED_SEARCH_MAX;
  const double fused_eta = fuse ? (double)eta : -1.0;
  if (!fuse) {
    mark(stream);
    launch_search(ws, d0, (double)eta, MODE_PROJECT, MLPROJ_OUTER_L1, nullptr, stream);
  }
  mark(stream);
  if (vec == 4 && x_vec)
    hipLaunchKernelGGL((slabmap_kernel<4, true>), grid, block, 0, stream, Y, X, d0, len, g, ws, u_out, fused_eta);
  else if (vec == 4)
    hipLaunchKernelGGL((slabmap_kernel<4, false>), grid, block, 0, stream, Y, X, d0, len, g, ws, u_out, fused_eta);
  else
    hipLaunchKernelGGL((slabmap_kernel<1, false>), grid, block, 0, stream, Y, X, d0, len, g, ws, u_out, fused_eta);
  mark(stream);
  return launch_status();
}

}  // extern "C"
