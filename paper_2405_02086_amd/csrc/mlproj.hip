// mlproj: bi-level / tri-level projection onto the l_{1,q} ball for gfx950 (MI355X).
// Method: Perez & Barlaud, "Multi-level projection with exponential parallel speedup",
// arXiv 2405.02086 -- Sec. 3 (Eq. 5-9, Alg. 1), Sec. 4 (Alg. 2-4), Sec. 5.1 (Alg. 5) and the
// iterative forms in the appendix.  The paper describes CPU code only; the kernels below are
// an independent design for a 256-CU, 64-lane-wavefront, HBM-bound machine.
//
// Pipeline of one bi-level call (all on the caller's stream, nothing returns to the host):
//   colagg  : every workgroup reduces a (row block) x (column tile) patch of Y to per-column
//             partials; the last workgroup of a tile folds that tile's partials into v, the
//             last tile runs the l1-ball threshold search for tau (step 2 of Alg. 1).
//   [sweep] : l1,1 only -- per-column inner threshold searches, one pass over Y per iteration.
//   colmap  : X = per-column map of Y with u_j = max(v_j - tau, 0) (clip / rescale / shrink).
// The tri-level form uses the same tail with groups that are contiguous slabs.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdint>
#include <type_traits>

#include "../../include/mlproj.h"

namespace mlproj {

constexpr int WG = 256;          // threads per workgroup
constexpr int WAVE = 64;         // gfx950 wavefront
constexpr int WAVES = WG / WAVE; // wavefronts per workgroup
constexpr int QINF = MLPROJ_L1INF, Q1 = MLPROJ_L11, Q2 = MLPROJ_L12;
constexpr int MODE_PROJECT = 0, MODE_NORM = 1;
constexpr int SEARCH_CACHE = 16; // values of v each thread of the search keeps in registers
constexpr int MAX_INNER_SWEEPS = 40;

// ------------------------------------------------------------------ host-side geometry
// How a matrix (or a tensor seen as d0 contiguous slabs) is cut into workgroup patches.
struct Geometry {
  long long tiles;        // column tiles (bi-level) or slabs (tri-level)
  long long blocks;       // row blocks per tile / chunks per slab
  long long span;         // rows per row block / elements per chunk
  int vec;                // floats per lane per access: 4 or 1
};

// Device view of the workspace.  Everything below `res` is scratch; the ticket words are
// zero between calls (mlproj_workspace_init, then every kernel puts them back).
struct Ws {
  mlproj_result* res;
  unsigned* ticket;        // [1]  tiles that have finished
  unsigned* pending;       // [2]  l1,1: columns still searching, ping-pong by sweep parity
  unsigned* tile_ticket;   // [tiles]
  unsigned* tile_pending;  // [tiles] l1,1
  double* tile_sum;        // [tiles]
  double* tile_max;        // [tiles]
  double* v;               // [groups] aggregate, fp64 (exact for q = inf)
  double* tauj;            // [groups] l1,1 inner thresholds
  unsigned* kprev;         // [groups] l1,1 previous active counts
  void* partial;           // [tiles][blocks][tile_w] float or double
  unsigned* partial_cnt;   // [tiles][blocks][tile_w] l1,1
};

struct Layout {
  size_t off_ticket, off_pending, off_tile_ticket, off_tile_pending, off_tile_sum, off_tile_max,
      off_v, off_tauj, off_kprev, off_partial, off_partial_cnt, bytes;
};

static inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }
static inline long long cdiv(long long a, long long b) { return (a + b - 1) / b; }

static Geometry plan_columns(long long n, long long m, int vec) {
  Geometry g;
  g.vec = vec;
  const long long tile_w = (long long)WAVE * vec;
  g.tiles = cdiv(m, tile_w);
  const long long target_wgs = 2048;  // ~8 workgroups per CU
  long long rb = target_wgs / g.tiles;
  if (rb < 1) rb = 1;
  long long span = cdiv(n, rb);
  span = cdiv(span, 8 * WAVES) * (8 * WAVES);  // whole unrolled trips per wavefront
  g.span = span;
  g.blocks = cdiv(n, span);
  return g;
}

static Geometry plan_slabs(long long d0, long long len, int vec) {
  Geometry g;
  g.vec = vec;
  g.tiles = d0;
  const long long target_wgs = 2048;
  long long chunks = target_wgs / d0;
  if (chunks < 1) chunks = 1;
  const long long quantum = (long long)WG * vec * 4;  // one unrolled trip of the workgroup
  long long span = cdiv(len, chunks);
  span = cdiv(span, quantum) * quantum;
  g.span = span;
  g.blocks = cdiv(len, span);
  return g;
}

static Layout layout_for(const Geometry& g, long long groups, int variant) {
  Layout L{};
  size_t o = align_up(sizeof(mlproj_result), 256);
  L.off_ticket = o;            o += 256;
  L.off_pending = o;           o += 256;
  L.off_tile_ticket = o;       o = align_up(o + (size_t)g.tiles * 4, 256);
  L.off_tile_pending = o;      o = align_up(o + (size_t)g.tiles * 4, 256);
  L.off_tile_sum = o;          o = align_up(o + (size_t)g.tiles * 8, 256);
  L.off_tile_max = o;          o = align_up(o + (size_t)g.tiles * 8, 256);
  L.off_v = o;                 o = align_up(o + (size_t)groups * 8, 256);
  L.off_tauj = o;              o = align_up(o + (variant == Q1 ? (size_t)groups * 8 : 0), 256);
  L.off_kprev = o;             o = align_up(o + (variant == Q1 ? (size_t)groups * 4 : 0), 256);
  const size_t tile_w = variant == MLPROJ_L1INFINF ? 1 : (size_t)WAVE * g.vec;
  const size_t cells = (size_t)g.tiles * (size_t)g.blocks * tile_w;
  L.off_partial = o;           o = align_up(o + cells * 8, 256);
  L.off_partial_cnt = o;       o = align_up(o + (variant == Q1 ? cells * 4 : 0), 256);
  L.bytes = o;
  return L;
}

static Ws bind(void* workspace, const Layout& L) {
  char* b = static_cast<char*>(workspace);
  Ws w;
  w.res = reinterpret_cast<mlproj_result*>(b);
  w.ticket = reinterpret_cast<unsigned*>(b + L.off_ticket);
  w.pending = reinterpret_cast<unsigned*>(b + L.off_pending);
  w.tile_ticket = reinterpret_cast<unsigned*>(b + L.off_tile_ticket);
  w.tile_pending = reinterpret_cast<unsigned*>(b + L.off_tile_pending);
  w.tile_sum = reinterpret_cast<double*>(b + L.off_tile_sum);
  w.tile_max = reinterpret_cast<double*>(b + L.off_tile_max);
  w.v = reinterpret_cast<double*>(b + L.off_v);
  w.tauj = reinterpret_cast<double*>(b + L.off_tauj);
  w.kprev = reinterpret_cast<unsigned*>(b + L.off_kprev);
  w.partial = b + L.off_partial;
  w.partial_cnt = reinterpret_cast<unsigned*>(b + L.off_partial_cnt);
  return w;
}

// ------------------------------------------------------------------ device helpers
template <int VEC> struct Pack;
template <> struct Pack<4> { using type = float4; };
template <> struct Pack<1> { using type = float; };

template <int VEC>
__device__ __forceinline__ void load_row(const float* p, float (&x)[VEC]) {
  if constexpr (VEC == 4) {
    const float4 t = *reinterpret_cast<const float4*>(p);
    x[0] = t.x; x[1] = t.y; x[2] = t.z; x[3] = t.w;
  } else {
    x[0] = *p;
  }
}

// X is written once and never read again by this call: a non-temporal store keeps it from
// displacing Y in the caches between the two passes over Y.
template <int VEC>
__device__ __forceinline__ void store_row_nt(float* p, const float (&x)[VEC]) {
  if constexpr (VEC == 4) {
    typedef float vf4 __attribute__((ext_vector_type(4)));
    vf4 t = {x[0], x[1], x[2], x[3]};
    __builtin_nontemporal_store(t, reinterpret_cast<vf4*>(p));
  } else {
    __builtin_nontemporal_store(x[0], p);
  }
}

__device__ __forceinline__ double wave_sum(double x) {
#pragma unroll
  for (int o = WAVE / 2; o > 0; o >>= 1) x += __shfl_down(x, o, WAVE);
  return x;
}
__device__ __forceinline__ double wave_max(double x) {
#pragma unroll
  for (int o = WAVE / 2; o > 0; o >>= 1) x = fmax(x, __shfl_down(x, o, WAVE));
  return x;
}
__device__ __forceinline__ unsigned wave_sum_u(unsigned x) {
#pragma unroll
  for (int o = WAVE / 2; o > 0; o >>= 1) x += __shfl_down(x, o, WAVE);
  return x;
}
__device__ __forceinline__ float wave_max_f(float x) {
#pragma unroll
  for (int o = WAVE / 2; o > 0; o >>= 1) x = fmaxf(x, __shfl_down(x, o, WAVE));
  return x;
}

// Workgroup-wide reductions; every thread gets the result.  Fixed order => deterministic.
struct BlockScratch {
  double d[WAVES];
  unsigned u[WAVES];
  unsigned flag;
};

__device__ __forceinline__ double block_sum(double x, BlockScratch& s) {
  x = wave_sum(x);
  if ((threadIdx.x & (WAVE - 1)) == 0) s.d[threadIdx.x / WAVE] = x;
  __syncthreads();
  double r = 0.0;
#pragma unroll
  for (int w = 0; w < WAVES; ++w) r += s.d[w];
  __syncthreads();
  return r;
}
__device__ __forceinline__ double block_max(double x, BlockScratch& s) {
  x = wave_max(x);
  if ((threadIdx.x & (WAVE - 1)) == 0) s.d[threadIdx.x / WAVE] = x;
  __syncthreads();
  double r = s.d[0];
#pragma unroll
  for (int w = 1; w < WAVES; ++w) r = fmax(r, s.d[w]);
  __syncthreads();
  return r;
}
__device__ __forceinline__ unsigned block_sum_u(unsigned x, BlockScratch& s) {
  x = wave_sum_u(x);
  if ((threadIdx.x & (WAVE - 1)) == 0) s.u[threadIdx.x / WAVE] = x;
  __syncthreads();
  unsigned r = 0;
#pragma unroll
  for (int w = 0; w < WAVES; ++w) r += s.u[w];
  __syncthreads();
  return r;
}

// "Last one out" ticket: every workgroup that shares `counter` calls this once after writing
// its results; exactly one of them (the last to arrive) gets true, and it may then read what
// all the others wrote.  Release fence before the atomic, acquire fence after.
__device__ __forceinline__ bool take_ticket(unsigned* counter, unsigned total, BlockScratch& s) {
  __threadfence();
  __syncthreads();
  if (threadIdx.x == 0) {
    const unsigned old = atomicAdd(counter, 1u);
    s.flag = (old + 1u == total) ? 1u : 0u;
  }
  __syncthreads();
  const bool last = s.flag != 0u;
  if (last) __threadfence();
  return last;
}

// ------------------------------------------------------------------ step 2: threshold search
// Euclidean projection of v >= 0 onto the l1 ball of radius eta (Eq. 6-7): tau = 0 when
// sum(v) <= eta, otherwise the root of sum_j max(v_j - tau, 0) = eta.  The root is reached
// by the fixed point tau <- (sum_{v_j > tau} v_j - eta) / #{v_j > tau}, started from a lower
// bound; tau rises monotonically, the active set only shrinks, and when it stops shrinking
// tau is exactly (sum over the final active set - eta) / K, in fp64.  Run by ONE workgroup.
__device__ void finish_search(const Ws& ws, long long groups, long long tiles, double eta,
                              int mode, double* norm_out, BlockScratch& s) {
  const int tid = threadIdx.x;
  double a = 0.0, mx = 0.0;
  for (long long i = tid; i < tiles; i += WG) {
    a += ws.tile_sum[i];
    mx = fmax(mx, ws.tile_max[i]);
  }
  const double total = block_sum(a, s);
  const double vmax = block_max(mx, s);
  if (mode == MODE_NORM) {
    if (tid == 0) {
      ws.res->norm = total;
      ws.res->vmax = vmax;
      if (norm_out) *norm_out = total;
    }
    return;
  }
  double tau = 0.0;
  unsigned active = 0, iters = 0, inside = 0;
  if (eta == 0.0) {
    tau = vmax;  // nothing exceeds vmax: every u_j is 0
  } else if (total <= eta) {
    inside = 1;  // already in the ball: tau = 0, u = v
    unsigned c = 0;
    for (long long i = tid; i < groups; i += WG) c += ws.v[i] > 0.0 ? 1u : 0u;
    active = block_sum_u(c, s);
  } else {
    double vr[SEARCH_CACHE];
#pragma unroll
    for (int k = 0; k < SEARCH_CACHE; ++k) {
      const long long i = tid + (long long)k * WG;
      vr[k] = i < groups ? ws.v[i] : 0.0;
    }
    // two lower bounds on the root: all groups active, and only the largest active
    tau = fmax((total - eta) / (double)groups, vmax - eta);
    unsigned kprev = 0xffffffffu;
    for (;;) {
      double sum = 0.0;
      unsigned cnt = 0;
#pragma unroll
      for (int k = 0; k < SEARCH_CACHE; ++k) {
        if (vr[k] > tau) { sum += vr[k]; ++cnt; }
      }
      for (long long i = tid + (long long)SEARCH_CACHE * WG; i < groups; i += WG) {
        const double x = ws.v[i];
        if (x > tau) { sum += x; ++cnt; }
      }
      const double S = block_sum(sum, s);
      const unsigned K = block_sum_u(cnt, s);
      active = K;
      if (K == 0u || K == kprev) break;  // K == 0: eta below the resolution of vmax
      kprev = K;
      const double t = (S - eta) / (double)K;
      if (t > tau) tau = t;
      ++iters;
    }
  }
  if (tid == 0) {
    mlproj_result* r = ws.res;
    r->tau = tau;
    r->norm = total;
    r->vmax = vmax;
    r->n_active = active;
    r->inside_ball = inside;
    r->search_iters = iters;
    r->inner_sweeps = 0;
    r->inner_pending = 0;
    if (norm_out) *norm_out = total;
  }
}

// ------------------------------------------------------------------ step 1: column aggregate
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

// v_j = ||y_j||_q for all columns (Sec. 3; max, sum of |.| or root of sum of squares), then
// the threshold search.  Grid: tiles * blocks workgroups, tile index fastest so neighbouring
// workgroups read neighbouring addresses.  Lane l of every wavefront owns VEC consecutive
// columns; the four wavefronts of a workgroup take rows r, r+1, r+2, r+3 (mod 4).
template <int Q, int VEC>
__global__ __launch_bounds__(WG) void colagg_kernel(const float* __restrict__ Y, long long n,
                                                    long long m, Geometry g, Ws ws, double eta,
                                                    int mode, float* __restrict__ v_out,
                                                    double* __restrict__ norm_out) {
  using Acc = typename AccOf<Q>::type;
  constexpr int TILE_W = WAVE * VEC;
  __shared__ Acc sm[WAVES][TILE_W];
  __shared__ BlockScratch bs;

  const int lane = threadIdx.x & (WAVE - 1);
  const int wave = threadIdx.x / WAVE;
  const long long t = blockIdx.x % g.tiles;
  const long long rb = blockIdx.x / g.tiles;
  const long long col0 = t * TILE_W + (long long)lane * VEC;
  const long long r0 = rb * g.span;
  const long long r1 = (r0 + g.span < n) ? r0 + g.span : n;

  Acc acc[VEC];
#pragma unroll
  for (int k = 0; k < VEC; ++k) acc[k] = (Acc)0;

  if (col0 < m) {
    const float* p = Y + col0;
    long long i = r0 + wave;
    for (; i + 7 * WAVES < r1; i += 8 * WAVES) {
      float x[8][VEC];
#pragma unroll
      for (int r = 0; r < 8; ++r) load_row<VEC>(p + (i + (long long)r * WAVES) * m, x[r]);
#pragma unroll
      for (int r = 0; r < 8; ++r)
#pragma unroll
        for (int k = 0; k < VEC; ++k) accumulate<Q>(acc[k], x[r][k]);
    }
    for (; i < r1; i += WAVES) {
      float x[VEC];
      load_row<VEC>(p + i * m, x);
#pragma unroll
      for (int k = 0; k < VEC; ++k) accumulate<Q>(acc[k], x[k]);
    }
  }
#pragma unroll
  for (int k = 0; k < VEC; ++k) sm[wave][lane * VEC + k] = acc[k];
  __syncthreads();

  Acc* partial = static_cast<Acc*>(ws.partial);
  if (threadIdx.x < TILE_W) {
    Acc a = sm[0][threadIdx.x];
#pragma unroll
    for (int w = 1; w < WAVES; ++w) a = combine<Q>(a, sm[w][threadIdx.x]);
    partial[((size_t)t * g.blocks + rb) * TILE_W + threadIdx.x] = a;
  }
  if (!take_ticket(&ws.tile_ticket[t], (unsigned)g.blocks, bs)) return;

  // last workgroup of this column tile: fold the row-block partials, in a fixed order
  double vj = 0.0;
  const long long col = t * TILE_W + threadIdx.x;
  if (threadIdx.x < TILE_W && col < m) {
    Acc a = (Acc)0;
    const Acc* q = partial + (size_t)t * g.blocks * TILE_W + threadIdx.x;
    for (long long b = 0; b < g.blocks; ++b) a = combine<Q>(a, q[(size_t)b * TILE_W]);
    vj = (Q == Q2) ? sqrt((double)a) : (double)a;
    ws.v[col] = vj;
    if (v_out) v_out[col] = (float)vj;
  }
  const double tsum = block_sum(vj, bs);
  const double tmax = block_max(vj, bs);
  if (threadIdx.x == 0) {
    ws.tile_sum[t] = tsum;
    ws.tile_max[t] = tmax;
    ws.tile_ticket[t] = 0u;
  }
  if (!take_ticket(ws.ticket, (unsigned)g.tiles, bs)) return;

  // last tile of the matrix: every v_j is known
  finish_search(ws, m, g.tiles, eta, mode, norm_out, bs);
  if (threadIdx.x == 0) ws.ticket[0] = 0u;
}

// ------------------------------------------------------------------ step 3: per-column map
// x_j = P^q_{u_j}(y_j) (Eq. 8-9) with u_j = max(v_j - tau, 0):
//   q = inf : X = sign(Y) min(|Y|, u_j)          (the symmetric clip; Sec. 4.1)
//   q = 2   : X = Y * u_j / v_j
//   q = 1   : X = sign(Y) max(|Y| - tau_j, 0)    with tau_j from the inner searches
// Row blocks are visited in the reverse order of the aggregate pass, so the rows read last
// there (the ones most likely still cached) are read first here.
template <int Q, int VEC>
__global__ __launch_bounds__(WG) void colmap_kernel(const float* Y, float* X, long long n,
                                                    long long m, Geometry g, Ws ws,
                                                    float* __restrict__ u_out) {
  constexpr int TILE_W = WAVE * VEC;
  const int lane = threadIdx.x & (WAVE - 1);
  const int wave = threadIdx.x / WAVE;
  const long long t = blockIdx.x % g.tiles;
  const long long rb = g.blocks - 1 - blockIdx.x / g.tiles;
  const long long col0 = t * TILE_W + (long long)lane * VEC;
  if (col0 >= m) return;
  const long long r0 = rb * g.span;
  const long long r1 = (r0 + g.span < n) ? r0 + g.span : n;

  const double tau = ws.res->tau;
  const bool inside = ws.res->inside_ball != 0u;
  float uf[VEC];
  double par[VEC];  // q = 2: scale u_j / v_j;  q = 1: inner threshold tau_j
#pragma unroll
  for (int k = 0; k < VEC; ++k) {
    const double vj = ws.v[col0 + k];
    const double uj = fmax(vj - tau, 0.0);
    uf[k] = (float)uj;
    if constexpr (Q == Q2) par[k] = vj > 0.0 ? uj / vj : 0.0;
    else if constexpr (Q == Q1) par[k] = inside ? 0.0 : (uj > 0.0 ? ws.tauj[col0 + k] : HUGE_VAL);
    else par[k] = 0.0;
  }
  if (u_out && rb == 0 && wave == 0) {
#pragma unroll
    for (int k = 0; k < VEC; ++k) u_out[col0 + k] = uf[k];
  }

  auto apply = [&](float y, int k) -> float {
    if constexpr (Q == QINF) return copysignf(fminf(fabsf(y), uf[k]), y);
    else if constexpr (Q == Q2) return (float)((double)y * par[k]);
    else return copysignf((float)fmax((double)fabsf(y) - par[k], 0.0), y);
  };

  const float* p = Y + col0;
  float* q = X + col0;
  long long i = r0 + wave;
  for (; i + 7 * WAVES < r1; i += 8 * WAVES) {
    float x[8][VEC];
#pragma unroll
    for (int r = 0; r < 8; ++r) load_row<VEC>(p + (i + (long long)r * WAVES) * m, x[r]);
#pragma unroll
    for (int r = 0; r < 8; ++r) {
#pragma unroll
      for (int k = 0; k < VEC; ++k) x[r][k] = apply(x[r][k], k);
      store_row_nt<VEC>(q + (i + (long long)r * WAVES) * m, x[r]);
    }
  }
  for (; i < r1; i += WAVES) {
    float x[VEC];
    load_row<VEC>(p + i * m, x);
#pragma unroll
    for (int k = 0; k < VEC; ++k) x[k] = apply(x[k], k);
    store_row_nt<VEC>(q + i * m, x);
  }
}

// ------------------------------------------------------------------ l1,1: inner searches
// Step 3 of Alg. 3 needs, for every kept column, the threshold tau_j with
// sum_i max(|Y_ij| - tau_j, 0) = u_j.  All columns run the same monotone fixed point as
// step 2, in lock step: one launch = one pass over Y that gives every column the sum and
// count of its entries above the current tau_j; the last workgroup of a tile updates tau_j.
// A column is finished when its count repeats.  Launch k reads pending[k & 1] (written by
// launch k-1) and returns at once when no column is left.
template <int VEC, bool FIRST>
__global__ __launch_bounds__(WG) void l11_sweep_kernel(const float* __restrict__ Y, long long n,
                                                       long long m, Geometry g, Ws ws,
                                                       int sweep) {
  constexpr int TILE_W = WAVE * VEC;
  __shared__ double sm_sum[WAVES][TILE_W];
  __shared__ unsigned sm_cnt[WAVES][TILE_W];
  __shared__ BlockScratch bs;

  const mlproj_result* res = ws.res;
  if (res->inside_ball != 0u || res->n_active == 0u) return;
  if (!FIRST && ws.pending[sweep & 1] == 0u) return;

  const int lane = threadIdx.x & (WAVE - 1);
  const int wave = threadIdx.x / WAVE;
  const long long t = blockIdx.x % g.tiles;
  const long long rb = blockIdx.x / g.tiles;
  const long long col0 = t * TILE_W + (long long)lane * VEC;
  const long long r0 = rb * g.span;
  const long long r1 = (r0 + g.span < n) ? r0 + g.span : n;
  const double tau = res->tau;
  const bool tile_live = FIRST || ws.tile_pending[t] != 0u;

  double sum[VEC];
  unsigned cnt[VEC];
#pragma unroll
  for (int k = 0; k < VEC; ++k) { sum[k] = 0.0; cnt[k] = 0u; }

  if (tile_live && col0 < m) {
    double tj[VEC];
#pragma unroll
    for (int k = 0; k < VEC; ++k) {
      if constexpr (FIRST) {
        // lower bound for the inner root: all n entries active gives (v_j - u_j)/n = tau/n
        tj[k] = (ws.v[col0 + k] > tau) ? tau / (double)n : HUGE_VAL;
      } else {
        tj[k] = ws.tauj[col0 + k];
      }
    }
    const float* p = Y + col0;
    long long i = r0 + wave;
    for (; i + 7 * WAVES < r1; i += 8 * WAVES) {
      float x[8][VEC];
#pragma unroll
      for (int r = 0; r < 8; ++r) load_row<VEC>(p + (i + (long long)r * WAVES) * m, x[r]);
#pragma unroll
      for (int r = 0; r < 8; ++r)
#pragma unroll
        for (int k = 0; k < VEC; ++k) {
          const double a = (double)fabsf(x[r][k]);
          if (a > tj[k]) { sum[k] += a; ++cnt[k]; }
        }
    }
    for (; i < r1; i += WAVES) {
      float x[VEC];
      load_row<VEC>(p + i * m, x);
#pragma unroll
      for (int k = 0; k < VEC; ++k) {
        const double a = (double)fabsf(x[k]);
        if (a > tj[k]) { sum[k] += a; ++cnt[k]; }
      }
    }
  }
#pragma unroll
  for (int k = 0; k < VEC; ++k) {
    sm_sum[wave][lane * VEC + k] = sum[k];
    sm_cnt[wave][lane * VEC + k] = cnt[k];
  }
  __syncthreads();
  double* psum = static_cast<double*>(ws.partial);
  unsigned* pcnt = ws.partial_cnt;
  if (threadIdx.x < TILE_W) {
    double a = sm_sum[0][threadIdx.x];
    unsigned c = sm_cnt[0][threadIdx.x];
#pragma unroll
    for (int w = 1; w < WAVES; ++w) { a += sm_sum[w][threadIdx.x]; c += sm_cnt[w][threadIdx.x]; }
    const size_t cell = ((size_t)t * g.blocks + rb) * TILE_W + threadIdx.x;
    psum[cell] = a;
    pcnt[cell] = c;
  }
  if (!take_ticket(&ws.tile_ticket[t], (unsigned)g.blocks, bs)) return;

  unsigned open = 0u;
  const long long col = t * TILE_W + threadIdx.x;
  if (tile_live && threadIdx.x < TILE_W && col < m) {
    double S = 0.0;
    unsigned K = 0u;
    const size_t base = (size_t)t * g.blocks * TILE_W + threadIdx.x;
    for (long long b = 0; b < g.blocks; ++b) {
      S += psum[base + (size_t)b * TILE_W];
      K += pcnt[base + (size_t)b * TILE_W];
    }
    const double vj = ws.v[col];
    const double uj = fmax(vj - tau, 0.0);
    double tj;
    if constexpr (FIRST) tj = (vj > tau) ? tau / (double)n : HUGE_VAL;
    else tj = ws.tauj[col];
    const unsigned kp = FIRST ? 0xffffffffu : ws.kprev[col];
    if (uj > 0.0 && K > 0u) {
      const double tn = (S - uj) / (double)K;
      if (tn > tj) tj = tn;
      open = (K != kp) ? 1u : 0u;
    }
    ws.tauj[col] = tj;
    ws.kprev[col] = K;
  }
  const unsigned tile_open = block_sum_u(open, bs);
  if (threadIdx.x == 0) {
    ws.tile_pending[t] = tile_open;
    if (tile_open) atomicAdd(&ws.pending[(sweep + 1) & 1], tile_open);
    ws.tile_ticket[t] = 0u;
  }
  if (!take_ticket(ws.ticket, (unsigned)g.tiles, bs)) return;
  if (threadIdx.x == 0) {
    const unsigned left = ws.pending[(sweep + 1) & 1];
    ws.pending[sweep & 1] = 0u;
    ws.res->inner_sweeps = (unsigned)sweep + 1u;
    ws.res->inner_pending = left;
    ws.ticket[0] = 0u;
  }
}

// ------------------------------------------------------------------ tri-level: slab kernels
// Groups are the d0 contiguous slabs of len = d1*d2 elements.  w_a = max over the slab equals
// the two nested maxima of Alg. 5 (max over the fibre, then over the fibres of the slab).
template <int VEC>
__global__ __launch_bounds__(WG) void slabagg_kernel(const float* __restrict__ Y, long long d0,
                                                     long long len, Geometry g, Ws ws,
                                                     double eta, float* __restrict__ v_out) {
  __shared__ BlockScratch bs;
  const long long a = blockIdx.x / g.blocks;
  const long long c = blockIdx.x % g.blocks;
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
  double* partial = static_cast<double*>(ws.partial);
  if (threadIdx.x == 0) partial[(size_t)a * g.blocks + c] = bmax;
  if (!take_ticket(&ws.tile_ticket[a], (unsigned)g.blocks, bs)) return;

  double w = 0.0;
  for (long long b = threadIdx.x; b < g.blocks; b += WG)
    w = fmax(w, partial[(size_t)a * g.blocks + b]);
  w = block_max(w, bs);
  if (threadIdx.x == 0) {
    ws.v[a] = w;
    if (v_out) v_out[a] = (float)w;
    ws.tile_sum[a] = w;
    ws.tile_max[a] = w;
    ws.tile_ticket[a] = 0u;
  }
  if (!take_ticket(ws.ticket, (unsigned)g.tiles, bs)) return;
  finish_search(ws, d0, g.tiles, eta, MODE_PROJECT, nullptr, bs);
  if (threadIdx.x == 0) ws.ticket[0] = 0u;
}

// X_abc = sign(Y_abc) min(|Y_abc|, u_a).  The appendix form clips each fibre to
// U2_ab = min(V_ab, u_a); since |Y_abc| <= V_ab the two clips give the same value.
template <int VEC>
__global__ __launch_bounds__(WG) void slabmap_kernel(const float* Y, float* X, long long d0,
                                                     long long len, Geometry g, Ws ws,
                                                     float* __restrict__ u_out) {
  const long long a = d0 - 1 - blockIdx.x / g.blocks;
  const long long c = blockIdx.x % g.blocks;
  const long long lo = c * g.span;
  const long long hi = (lo + g.span < len) ? lo + g.span : len;
  const float u = (float)fmax(ws.v[a] - ws.res->tau, 0.0);
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
      store_row_nt<VEC>(q + i + r * STEP, x[r]);
    }
  }
  for (; i < hi; i += STEP) {
    float x[VEC];
    load_row<VEC>(p + i, x);
#pragma unroll
    for (int k = 0; k < VEC; ++k) x[k] = copysignf(fminf(fabsf(x[k]), u), x[k]);
    store_row_nt<VEC>(q + i, x);
  }
}

__global__ __launch_bounds__(WG) void fill_zero_kernel(uint32_t* p, size_t words) {
  for (size_t i = (size_t)blockIdx.x * WG + threadIdx.x; i < words; i += (size_t)gridDim.x * WG)
    p[i] = 0u;
}

// ------------------------------------------------------------------ host: checks + launches
constexpr long long MAX_ELEMS = 1LL << 40;       // 4 TiB of fp32: far beyond one GPU
constexpr long long MAX_GROUPS = (1LL << 31) - 1;
constexpr long long MAX_GRID = (1LL << 31) - 1;

static int check_dims(long long a, long long b, long long c) {
  if (a <= 0 || b <= 0 || c <= 0) return MLPROJ_ERR_BAD_DIMENSION;
  if (a > MAX_ELEMS || b > MAX_ELEMS || c > MAX_ELEMS) return MLPROJ_ERR_TOO_LARGE;
  if (a > MAX_ELEMS / b || a * b > MAX_ELEMS / c) return MLPROJ_ERR_TOO_LARGE;
  return MLPROJ_OK;
}

static bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

static int pick_vec(const void* Y, const void* X, long long row_len) {
  return (row_len % 4 == 0 && aligned(Y, 16) && (X == nullptr || aligned(X, 16))) ? 4 : 1;
}

static int workspace_bytes_impl(int variant, long long d0, long long d1, long long d2,
                                size_t* out) {
  if (!out) return MLPROJ_ERR_NULL_POINTER;
  if (variant < MLPROJ_L1INF || variant > MLPROJ_L1INFINF) return MLPROJ_ERR_BAD_VARIANT;
  if (variant != MLPROJ_L1INFINF && d2 != 1) return MLPROJ_ERR_BAD_DIMENSION;
  const int st = check_dims(d0, d1, d2);
  if (st != MLPROJ_OK) return st;
  size_t best = 0;
  for (int vec : {4, 1}) {
    Geometry g;
    long long groups;
    if (variant == MLPROJ_L1INFINF) {
      if (d0 > MAX_GROUPS) return MLPROJ_ERR_TOO_LARGE;
      g = plan_slabs(d0, d1 * d2, vec);
      groups = d0;
    } else {
      if (d1 > MAX_GROUPS) return MLPROJ_ERR_TOO_LARGE;
      g = plan_columns(d0, d1, vec);
      groups = d1;
    }
    if (g.tiles * g.blocks > MAX_GRID) return MLPROJ_ERR_TOO_LARGE;
    const Layout L = layout_for(g, groups, variant);
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

template <int Q>
static int run_bilevel(const float* Y, float* X, long long n, long long m, float eta,
                       void* workspace, size_t workspace_bytes, float* v_out, float* u_out,
                       void* stream_, int mode, double* norm_out) {
  if (!Y || !workspace || (mode == MODE_PROJECT && !X)) return MLPROJ_ERR_NULL_POINTER;
  int st = check_dims(n, m, 1);
  if (st != MLPROJ_OK) return st;
  if (m > MAX_GROUPS) return MLPROJ_ERR_TOO_LARGE;
  if (mode == MODE_PROJECT && (st = check_radius(eta)) != MLPROJ_OK) return st;
  if (!aligned(Y, 4) || (X && !aligned(X, 4))) return MLPROJ_ERR_ALIGNMENT;
  if (!aligned(workspace, 256)) return MLPROJ_ERR_WORKSPACE;
  const int vec = pick_vec(Y, X, m);
  const Geometry g = plan_columns(n, m, vec);
  if (g.tiles * g.blocks > MAX_GRID) return MLPROJ_ERR_TOO_LARGE;
  const Layout L = layout_for(g, m, Q);
  if (workspace_bytes < L.bytes) return MLPROJ_ERR_WORKSPACE;
  const Ws ws = bind(workspace, L);
  hipStream_t stream = static_cast<hipStream_t>(stream_);
  const dim3 grid((unsigned)(g.tiles * g.blocks)), block(WG);
  const double eta_d = (double)eta;

  if (vec == 4)
    hipLaunchKernelGGL((colagg_kernel<Q, 4>), grid, block, 0, stream, Y, n, m, g, ws, eta_d, mode, v_out, norm_out);
  else
    hipLaunchKernelGGL((colagg_kernel<Q, 1>), grid, block, 0, stream, Y, n, m, g, ws, eta_d, mode, v_out, norm_out);
  if (mode == MODE_NORM) return launch_status();

  if constexpr (Q == Q1) {
    for (int s = 0; s < MAX_INNER_SWEEPS; ++s) {
      if (vec == 4) {
        if (s == 0) hipLaunchKernelGGL((l11_sweep_kernel<4, true>), grid, block, 0, stream, Y, n, m, g, ws, s);
        else hipLaunchKernelGGL((l11_sweep_kernel<4, false>), grid, block, 0, stream, Y, n, m, g, ws, s);
      } else {
        if (s == 0) hipLaunchKernelGGL((l11_sweep_kernel<1, true>), grid, block, 0, stream, Y, n, m, g, ws, s);
        else hipLaunchKernelGGL((l11_sweep_kernel<1, false>), grid, block, 0, stream, Y, n, m, g, ws, s);
      }
    }
  }
  if (vec == 4)
    hipLaunchKernelGGL((colmap_kernel<Q, 4>), grid, block, 0, stream, Y, X, n, m, g, ws, u_out);
  else
    hipLaunchKernelGGL((colmap_kernel<Q, 1>), grid, block, 0, stream, Y, X, n, m, g, ws, u_out);
  return launch_status();
}

}  // namespace mlproj

// ------------------------------------------------------------------ C ABI
using namespace mlproj;

extern "C" {

int mlproj_version(void) { return 100; }

const char* mlproj_status_string(int status) {
  switch (status) {
    case MLPROJ_OK: return "ok";
    case MLPROJ_ERR_NULL_POINTER: return "a required pointer is NULL";
    case MLPROJ_ERR_BAD_DIMENSION: return "a dimension is not positive";
    case MLPROJ_ERR_TOO_LARGE: return "input exceeds the supported size";
    case MLPROJ_ERR_BAD_RADIUS: return "eta must be finite and >= 0";
    case MLPROJ_ERR_WORKSPACE: return "workspace too small or not 256-byte aligned";
    case MLPROJ_ERR_BAD_VARIANT: return "unknown variant";
    case MLPROJ_ERR_ALIGNMENT: return "Y and X must be 4-byte aligned";
    case MLPROJ_ERR_LAUNCH: return "HIP refused a kernel launch";
    default: return "unknown status";
  }
}

int mlproj_workspace_bytes(int variant, long long d0, long long d1, long long d2, size_t* bytes_out) {
  return workspace_bytes_impl(variant, d0, d1, d2, bytes_out);
}

int mlproj_workspace_init(void* workspace, size_t workspace_bytes, void* stream) {
  if (!workspace) return MLPROJ_ERR_NULL_POINTER;
  if (!aligned(workspace, 256) || workspace_bytes < 1024 || workspace_bytes % 4 != 0)
    return MLPROJ_ERR_WORKSPACE;
  const size_t words = workspace_bytes / 4;
  size_t blocks = (words + WG - 1) / WG;
  if (blocks > 4096) blocks = 4096;
  hipLaunchKernelGGL(fill_zero_kernel, dim3((unsigned)blocks), dim3(WG), 0,
                     static_cast<hipStream_t>(stream), static_cast<uint32_t*>(workspace), words);
  return launch_status();
}

int mlproj_norm_l1q(const float* Y, long long n, long long m, int q_variant, void* workspace,
                    size_t workspace_bytes, double* norm_out, float* v_out, void* stream) {
  switch (q_variant) {
    case MLPROJ_L1INF: return run_bilevel<QINF>(Y, nullptr, n, m, 0.f, workspace, workspace_bytes, v_out, nullptr, stream, MODE_NORM, norm_out);
    case MLPROJ_L11: return run_bilevel<Q1>(Y, nullptr, n, m, 0.f, workspace, workspace_bytes, v_out, nullptr, stream, MODE_NORM, norm_out);
    case MLPROJ_L12: return run_bilevel<Q2>(Y, nullptr, n, m, 0.f, workspace, workspace_bytes, v_out, nullptr, stream, MODE_NORM, norm_out);
    default: return MLPROJ_ERR_BAD_VARIANT;
  }
}

int bilevel_proj_l1inf(const float* Y, float* X, long long n, long long m, float eta,
                       void* workspace, size_t workspace_bytes, float* v_out, float* u_out,
                       void* stream) {
  return run_bilevel<QINF>(Y, X, n, m, eta, workspace, workspace_bytes, v_out, u_out, stream, MODE_PROJECT, nullptr);
}

int bilevel_proj_l11(const float* Y, float* X, long long n, long long m, float eta,
                     void* workspace, size_t workspace_bytes, float* v_out, float* u_out,
                     void* stream) {
  return run_bilevel<Q1>(Y, X, n, m, eta, workspace, workspace_bytes, v_out, u_out, stream, MODE_PROJECT, nullptr);
}

int bilevel_proj_l12(const float* Y, float* X, long long n, long long m, float eta,
                     void* workspace, size_t workspace_bytes, float* v_out, float* u_out,
                     void* stream) {
  return run_bilevel<Q2>(Y, X, n, m, eta, workspace, workspace_bytes, v_out, u_out, stream, MODE_PROJECT, nullptr);
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
  const int vec = pick_vec(Y, X, len);
  const Geometry g = plan_slabs(d0, len, vec);
  if (g.tiles * g.blocks > MAX_GRID) return MLPROJ_ERR_TOO_LARGE;
  const Layout L = layout_for(g, d0, MLPROJ_L1INFINF);
  if (workspace_bytes < L.bytes) return MLPROJ_ERR_WORKSPACE;
  const Ws ws = bind(workspace, L);
  hipStream_t stream = static_cast<hipStream_t>(stream_);
  const dim3 grid((unsigned)(g.tiles * g.blocks)), block(WG);
  if (vec == 4) {
    hipLaunchKernelGGL((slabagg_kernel<4>), grid, block, 0, stream, Y, d0, len, g, ws, (double)eta, v_out);
    hipLaunchKernelGGL((slabmap_kernel<4>), grid, block, 0, stream, Y, X, d0, len, g, ws, u_out);
  } else {
    hipLaunchKernelGGL((slabagg_kernel<1>), grid, block, 0, stream, Y, d0, len, g, ws, (double)eta, v_out);
    hipLaunchKernelGGL((slabmap_kernel<1>), grid, block, 0, stream, Y, X, d0, len, g, ws, u_out);
  }
  return launch_status();
}

}  // extern "C"
