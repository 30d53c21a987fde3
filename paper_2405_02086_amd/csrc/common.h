// mlproj: constants, workspace layout, launch geometry and the element access helpers.
#ifndef MLPROJ_COMMON_H
#define MLPROJ_COMMON_H

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
constexpr int SEARCH_CACHE_ONE_WG = 32;  // ... in the stand-alone one-workgroup search of 16385..32768 groups
constexpr int MAX_INNER_SWEEPS = 16;     // l1,1: most lock-step passes over Y a call may plan for the inner searches
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
constexpr int COOP_THREADS = 256;        // threads of each of them
constexpr int COOP_VALUES = 32;          // values of v per thread there
// Polls a lane of the grid-wide search spends on another workgroup's post before the search gives
// up and the one-workgroup kernel behind it takes over.  A poll is one round trip to the memory
// side (1-2 us) and every workgroup posts within microseconds of starting, so the default is a
// fraction of a millisecond: on a GPU that other work keeps full (not every workgroup resident)
// the call pays that once, never seconds.
constexpr unsigned SPIN_LIMIT = 256;
constexpr unsigned SPIN_LIMIT_MAX = 1u << 22;   // the most the test hook accepts
constexpr int COOP_WORDS = 6;            // 64-bit words a workgroup posts per round there (tag and 32 bits of payload each)
constexpr int COOP_SLOT_WORDS = 2 * COOP_WORDS * COOP_MAX_WGS;
constexpr int COOP_FLAG_BYTES = 256;
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
  unsigned* flags;         // [1] the grid-wide search gave up ([0] spare); 256 bytes, and right behind them:
  unsigned long long* coop_q;  // [2][COOP_WORDS][COOP_MAX_WGS] grid-wide search: what the workgroups post per round, by parity
  double* v;               // [groups] aggregate, fp64 (exact for q = inf)
  double* tauj;            // [m] l1,1 inner thresholds: the point the next sweep evaluates, then the result
  double* tlo;             // [m] l1,1: lower end of the window whose entries the next sweep lists
  double* lb;              // [m] l1,1: certified lower bound on the threshold
  double* ub;              // [m] l1,1: certified upper bound
  unsigned* kprev;         // [m] l1,1: active count at the point whose Newton step is tlo, or NO_COUNT
  unsigned* done;          // [m] l1,1: 1 once tauj is final
  unsigned* gcnt;          // [m] l1,1: entries in the window, all workgroups
  float* cand;             // [list_cap][m] l1,1: the window entries, slot-major
  int list_cap;            // slots per column in cand
  void* partial;           // [tiles][groups][tile_w] float (q = inf) or double
  unsigned* partial_cnt;   // [tiles][groups][tile_w] l1,1: entries above t
  unsigned* partial_cnt2;  // [tiles][groups][tile_w] l1,1: entries above t*(1 + L11_WINDOW)
  const float* wts;        // [groups] weights of a weighted l1 ball as outer norm; null: the plain norms
  unsigned* posts;         // [HELD_POST_WORDS] one-pass tri-level kernel: what its workgroups post to one another
  float* scale;            // [m] l1,1: the columns' scale estimates that anchor the grid (l11grid.h)
  float* gpart;            // [tiles][groups][8][tile_w] l1,1: grid partials of the aggregate pass
};

struct Layout {
  size_t off_pending, off_flags, off_coop_q, off_v, off_tauj, off_kprev, off_partial, off_partial_cnt, off_partial_cnt2, bytes;
  size_t off_tlo, off_lb, off_ub, off_done, off_gcnt, off_cand, off_posts, off_scale, off_gpart;
  int list_cap;
};

__host__ __device__ static inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }
__host__ __device__ static inline long long cdiv(long long a, long long b) { return (a + b - 1) / b; }

// Both passes were tuned on an MI355X: a read-only pass is fastest with about two workgroups
// per CU, the read+write pass with one per CU and fewer rows in flight (a narrower band of
// DRAM pages open at a time).
__host__ __device__ static inline Geometry plan_columns(long long n, long long m, int vec, int variant) {
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
// The fold kernel's workgroup size for a matrix with `groups` partials per group (see
// reduce_body).  A batch folds with 1024 threads throughout but with the `parts` this size
// gives, so that its sums associate as in the single call and return its bits.
__host__ __device__ static inline int fold_threads(long long groups) {
  return (groups >= 16 && groups <= 64) ? 256 : SWG;
}
// (`threads`: the fold kernel's workgroup size, 1024 or 256.)
__host__ __device__ static inline int reduce_parts(long long partials_per_group, int threads = SWG) {
  int parts = 1;
  while (parts < threads / WAVE && parts < partials_per_group) parts *= 2;
  return parts;
}

constexpr int HELD_POST_WORDS = 256;     // one-pass tri-level kernel: one posted word per workgroup

constexpr int LIST_PER_THREAD = 16;      // l1,1: listed entries one lane of the update kernel holds in registers
constexpr int LIST_LANES = 16;           // ... and the lanes that share a column there

__host__ __device__ static inline Layout layout_for(const Geometry& g, long long ngroups, int variant) {
  Layout L{};
  size_t o = align_up(sizeof(mlproj_result), 256);
  L.off_pending = o;       o = align_up(o + (MAX_INNER_SWEEPS + 1) * 4, 256);
  L.off_flags = o;         o += COOP_FLAG_BYTES;
  L.off_coop_q = o;        o = align_up(o + (size_t)COOP_SLOT_WORDS * 8, 256);   // (must follow the flags: see clear_meeting_area)
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
  L.off_cand = o;          o = align_up(o + per_col4 * (size_t)L.list_cap, 256);
  L.off_posts = o;         o = align_up(o + (variant == MLPROJ_L1INFINF ? (size_t)HELD_POST_WORDS * 4 : 0), 256);
  L.off_scale = o;         o = align_up(o + per_col4, 256);
  L.off_gpart = o;         o = align_up(o + (variant == Q1 ? cells * 32 : 0), 256);
  L.bytes = o;
  return L;
}

__host__ __device__ static inline Ws bind(void* workspace, const Layout& L) {
  char* b = static_cast<char*>(workspace);
  Ws w;
  w.res = reinterpret_cast<mlproj_result*>(b);
  w.pending = reinterpret_cast<unsigned*>(b + L.off_pending);
  w.coop_q = reinterpret_cast<unsigned long long*>(b + L.off_coop_q);
  w.flags = reinterpret_cast<unsigned*>(b + L.off_flags);
  w.v = reinterpret_cast<double*>(b + L.off_v);
  w.tauj = reinterpret_cast<double*>(b + L.off_tauj);
  w.kprev = reinterpret_cast<unsigned*>(b + L.off_kprev);
  w.partial = b + L.off_partial;
  w.partial_cnt = reinterpret_cast<unsigned*>(b + L.off_partial_cnt);
  w.partial_cnt2 = reinterpret_cast<unsigned*>(b + L.off_partial_cnt2);
  w.wts = nullptr;
  w.tlo = reinterpret_cast<double*>(b + L.off_tlo);
  w.lb = reinterpret_cast<double*>(b + L.off_lb);
  w.ub = reinterpret_cast<double*>(b + L.off_ub);
  w.done = reinterpret_cast<unsigned*>(b + L.off_done);
  w.gcnt = reinterpret_cast<unsigned*>(b + L.off_gcnt);
  w.cand = reinterpret_cast<float*>(b + L.off_cand);
  w.list_cap = L.list_cap;
  w.posts = reinterpret_cast<unsigned*>(b + L.off_posts);
  w.scale = reinterpret_cast<float*>(b + L.off_scale);
  w.gpart = reinterpret_cast<float*>(b + L.off_gpart);
  return w;
}

// The grid-wide search's meeting area: the flags, and behind them the slots its workgroups post
// into.  Cleared by one whole workgroup of a kernel that runs before the search in every call
// (a stale tag from an earlier call would pass for a posted word).
__device__ __forceinline__ void clear_meeting_area(unsigned* flags) {
  if (threadIdx.x < 2) flags[threadIdx.x] = 0u;
  unsigned long long* q = reinterpret_cast<unsigned long long*>(reinterpret_cast<char*>(flags) + COOP_FLAG_BYTES);
  for (int i = threadIdx.x; i < COOP_SLOT_WORDS; i += blockDim.x) q[i] = 0ull;
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

}  // namespace mlproj

#endif
