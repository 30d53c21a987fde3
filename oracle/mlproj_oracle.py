"""CPU oracle for the bi-level / tri-level l1,q projections (Perez & Barlaud,
"Multi-level projection with exponential parallel speedup", arXiv 2405.02086).

THIS IS TEST INFRASTRUCTURE.  It is slow, plain and written to be checked
against the paper by eye.  Only tests, the smoke check and the benchmark's
CPU-baseline leg may import it; the GPU library never does, and this file
imports nothing from the GPU package.

Conventions
-----------
* A matrix Y has shape (n, m); column j (Y[:, j]) is group j (Sec. 2, Eq. 1-2).
* Storage is fp32.  Every sum, the l1-ball threshold and every division are
  taken in fp64.  max / min / abs / copysign are exact in fp32 and done there.
* Where fp64 meets fp32 (the radii u_j that bound fp32 data) the radius is
  rounded to fp32 first, then compared -- the same decision rule the fp32
  storage format forces on any implementation.
* A group is kept iff v_j > tau (strict); v_j == tau gives u_j = 0.

Every function is pinned by tests/test_oracle_pins.py against optimality
certificates of the Euclidean projection (Eq. 4), brute force, closed forms and
hand-worked examples; nothing here is "parity unpinned".
"""
import numpy as np

__all__ = [
    "column_norms", "norm_l1q", "project_l1_ball_nonneg", "project_l1_ball",
    "project_linf_ball", "project_l2_ball", "bilevel_l1inf", "bilevel_l11",
    "bilevel_l12", "trilevel_l1infinf", "bilevel", "multilevel", "project_outer",
    "round_to_storage", "bilevel_stored", "bilevel_batch", "trilevel_stored",
]


# --------------------------------------------------------------------------
# Sec. 2, Eq. 1-2: column norms and the l_{1,q} matrix norm
# --------------------------------------------------------------------------
def column_norms(Y, q):
    """v_q = (||y_1||_q, ..., ||y_m||_q), the aggregate vector of Sec. 3.

    q = "inf": exact fp32 maxima (returned as float32).
    q = 1, 2 : fp64 accumulation (returned as float64).
    """
    Y = np.asarray(Y)
    assert Y.ndim == 2 and Y.dtype == np.float32
    n, m = Y.shape
    if q == "inf":
        v = np.zeros(m, dtype=np.float32)
        for i in range(n):                       # plain loop over rows
            v = np.maximum(v, np.abs(Y[i, :]))
        return v
    if q == 1:
        v = np.zeros(m, dtype=np.float64)
        for i in range(n):
            v += np.abs(Y[i, :].astype(np.float64))
        return v
    if q == 2:
        s = np.zeros(m, dtype=np.float64)
        for i in range(n):
            r = Y[i, :].astype(np.float64)
            s += r * r
        return np.sqrt(s)
    raise ValueError("q must be 'inf', 1 or 2")


def norm_l1q(Y, q):
    """||Y||_{1,q} = sum_j ||y_j||_q  (Eq. 1 with p = 1; Eq. 10 for q = inf)."""
    return float(np.sum(column_norms(Y, q).astype(np.float64)))


# --------------------------------------------------------------------------
# Eq. 4 with p = 1: Euclidean projection onto the l1 ball (sort-based)
# --------------------------------------------------------------------------
def project_l1_ball_nonneg(v, eta):
    """P^1_eta(v) for v >= 0, in fp64.  Returns (u, tau).

    The minimiser of ||u - v||_2 over {u : ||u||_1 <= eta} is
    u_j = max(v_j - tau, 0) with tau = 0 if sum(v) <= eta, and otherwise the
    unique tau > 0 with sum_j max(v_j - tau, 0) = eta.  tau is found from the
    values sorted in decreasing order mu_1 >= ... >= mu_m and their prefix sums
    c_k: K = max{k : mu_k > (c_k - eta)/k}, tau = (c_K - eta)/K.
    """
    v = np.asarray(v, dtype=np.float64)
    assert v.ndim == 1 and np.all(v >= 0.0)
    eta = float(eta)
    assert eta >= 0.0
    if v.size == 0:
        return v.copy(), 0.0
    if eta == 0.0:
        return np.zeros_like(v), float(np.max(v))
    if float(np.sum(v)) <= eta:
        return v.copy(), 0.0
    mu = np.sort(v)[::-1]
    c = np.cumsum(mu)
    k = np.arange(1, v.size + 1, dtype=np.float64)
    cand = (c - eta) / k
    K = int(np.nonzero(mu > cand)[0][-1]) + 1     # largest k with mu_k > cand_k
    tau = float(cand[K - 1])
    u = np.maximum(v - tau, 0.0)
    return u, tau


def project_weighted_l1_ball_nonneg(v, w, eta):
    """Euclidean projection of v >= 0 onto the weighted l1 ball {u : sum_j w_j |u_j| <= eta},
    w_j > 0 (the l_w1 ball Sec. 3 names beside l1, l2 and l_inf), in fp64.  Returns (u, tau).

    The Lagrangian of min ||u - v||^2 / 2 s.t. sum w_j u_j <= eta, u >= 0 gives
    u_j = max(v_j - tau w_j, 0) with tau = 0 if sum w_j v_j <= eta, and otherwise the unique
    tau > 0 with sum_j w_j max(v_j - tau w_j, 0) = eta.  With the ratios rho_j = v_j / w_j sorted
    in decreasing order the active set is a prefix: K = max{k : rho_(k) > tau_k},
    tau_k = (sum_{i<=k} w_i v_i - eta) / sum_{i<=k} w_i^2, tau = tau_K.
    """
    v = np.asarray(v, dtype=np.float64)
    w = np.asarray(w, dtype=np.float64)
    assert v.ndim == 1 and v.shape == w.shape and np.all(v >= 0.0) and np.all(w > 0.0)
    eta = float(eta)
    assert eta >= 0.0
    if v.size == 0:
        return v.copy(), 0.0
    rho = v / w
    if eta == 0.0:
        return np.zeros_like(v), float(np.max(rho))
    if float(np.sum(w * v)) <= eta:
        return v.copy(), 0.0
    order = np.argsort(-rho, kind="stable")
    num = np.cumsum((w * v)[order]) - eta
    den = np.cumsum((w * w)[order])
    cand = num / den
    K = int(np.nonzero(rho[order] > cand)[0][-1]) + 1
    tau = float(cand[K - 1])
    u = np.maximum(v - tau * w, 0.0)
    return u, tau


def project_l1_ball(y, r):
    """P^1_r(y) for a signed vector: sign(y) * P^1_r(|y|).  Returns (x, tau)."""
    y = np.asarray(y, dtype=np.float64)
    a, tau = project_l1_ball_nonneg(np.abs(y), r)
    return np.copysign(a, y), tau


# --------------------------------------------------------------------------
# Per-group maps of Eq. 9: projections onto the l_inf and l2 balls
# --------------------------------------------------------------------------
def project_linf_ball(y, r):
    """P^inf_r(y) = sign(y) * min(|y|, r), elementwise; r broadcasts.

    Sec. 4.1 prints this map without the sign; the Euclidean projection onto
    {x : max|x_i| <= r} is the symmetric clip written here.
    fp32 in, fp32 out, exact.
    """
    y = np.asarray(y, dtype=np.float32)
    r = np.asarray(r, dtype=np.float32)
    return np.copysign(np.minimum(np.abs(y), r), y).astype(np.float32)


def project_l2_ball(y, r, norm=None):
    """P^2_r(y) = y * min(1, r / ||y||_2) in fp64 (0 if y = 0)."""
    y = np.asarray(y, dtype=np.float64)
    nrm = float(np.sqrt(np.sum(y * y))) if norm is None else float(norm)
    if nrm <= r:
        return y.copy()
    return y * r / nrm


def project_outer(v, eta, p=1):
    """u = P^p_eta(v) for the non-negative aggregate vector v (Eq. 6-7), p in {1, 2, "inf"} or
    ("w1", weights): the l1-ball projection above, the rescale onto the l2 ball, the clip to
    [0, eta], or the projection onto the weighted l1 ball.
    Returns (u, tau); tau is the (weighted) l1 threshold and 0 for the other two norms."""
    v = np.asarray(v, dtype=np.float64)
    if isinstance(p, tuple) and p[0] == "w1":
        return project_weighted_l1_ball_nonneg(v, np.asarray(p[1], dtype=np.float64), eta)
    if p == 1:
        return project_l1_ball_nonneg(v, eta)
    if p == 2:
        return project_l2_ball(v, eta), 0.0
    if p == "inf":
        return np.minimum(v, eta), 0.0
    raise ValueError("outer norm must be 1, 2 or 'inf'")


# --------------------------------------------------------------------------
# Alg. 1 with p in {1, 2, inf}; Alg. 2 / 3 / 4: bi-level projections BP^{p,q}_eta
# --------------------------------------------------------------------------
def _out_and_columns(Y, columns):
    """Output buffer and the list of columns the per-column map visits.  With `columns`
    given (a sample of a huge input) the unvisited columns stay NaN."""
    if columns is None:
        return np.empty_like(Y), range(Y.shape[1])
    return np.full_like(Y, np.nan), list(columns)


def bilevel_l1inf(Y, eta, columns=None, p=1):
    """BP^{p,inf}_eta(Y); p = 1 is Eq. 13 / Alg. 2.  Returns dict(X, v, u, tau)."""
    Y = np.asarray(Y)
    assert Y.dtype == np.float32 and Y.ndim == 2
    v = column_norms(Y, "inf")                         # aggregate
    u64, tau = project_outer(v, eta, p)                # u = P^p_eta(v)
    u = u64.astype(np.float32)
    X, cols = _out_and_columns(Y, columns)
    for j in cols:                                     # x_j = P^inf_{u_j}(y_j), column by column
        X[:, j] = project_linf_ball(Y[:, j], u[j])
    return {"X": X, "v": v, "u": u, "tau": tau}


def bilevel_l12(Y, eta, columns=None, p=1):
    """BP^{p,2}_eta(Y); p = 1 is Eq. 15 / Alg. 4.  Returns dict(X, v, u, tau) (v, u fp64)."""
    Y = np.asarray(Y)
    assert Y.dtype == np.float32 and Y.ndim == 2
    v = column_norms(Y, 2)
    u, tau = project_outer(v, eta, p)
    X, cols = _out_and_columns(Y, columns)
    for j in cols:
        X[:, j] = project_l2_ball(Y[:, j], u[j], norm=v[j]).astype(np.float32)
    return {"X": X, "v": v, "u": u, "tau": tau}


def bilevel_l11(Y, eta, columns=None, p=1):
    """BP^{p,1}_eta(Y); p = 1 is Eq. 14 / Alg. 3.

    Returns dict(X, v, u, tau, tau_col); tau_col[j] is the inner threshold of
    column j.  `columns` (optional index list) restricts the per-column map to those
    columns; the others are left as NaN in X (used to sample huge inputs).
    """
    Y = np.asarray(Y)
    assert Y.dtype == np.float32 and Y.ndim == 2
    v = column_norms(Y, 1)
    u, tau = project_outer(v, eta, p)
    X, cols = _out_and_columns(Y, columns)
    tau_col = np.full(Y.shape[1], np.nan)
    for j in cols:
        x, tj = project_l1_ball(Y[:, j], u[j])
        X[:, j] = x.astype(np.float32)
        tau_col[j] = tj
    return {"X": X, "v": v, "u": u, "tau": tau, "tau_col": tau_col}


def bilevel(Y, eta, q, columns=None, p=1):
    """BP^{p,q}_eta(Y), Alg. 1, for p, q in {1, 2, "inf"}."""
    return {"inf": bilevel_l1inf, 1: bilevel_l11, 2: bilevel_l12}[q](Y, eta, columns, p)


# --------------------------------------------------------------------------
# 16-bit storage (an extension for training loops; the paper fixes no storage format)
# --------------------------------------------------------------------------
def round_to_storage(x, storage):
    """Round fp32 values to the storage format, to nearest with ties to even, and return them
    as fp32 again.  storage: "f32" (identity), "f16" (IEEE binary16: 10 fraction bits,
    subnormals, overflow to infinity) or "bf16" (the upper 16 bits of binary32: 7 fraction bits).
    """
    x = np.ascontiguousarray(x, dtype=np.float32)
    if storage == "f32":
        return x.copy()
    if storage == "f16":
        with np.errstate(over="ignore"):              # beyond 65504 the format has only infinity
            return x.astype(np.float16).astype(np.float32)
    if storage == "bf16":
        b = x.view(np.uint32).astype(np.uint64)
        kept_lsb = (b >> 16) & 1                      # ties go to the even 16-bit pattern
        r = ((b + 0x7FFF + kept_lsb) >> 16) << 16
        out = (r & 0xFFFFFFFF).astype(np.uint32).view(np.float32).reshape(x.shape)
        return np.where(np.isnan(x), x, out)
    raise ValueError("storage must be 'f32', 'f16' or 'bf16'")


def bilevel_stored(Y, eta, q, storage, columns=None, p=1):
    """BP^{p,q}_eta (Alg. 1) on a matrix kept in a 16-bit format.

    Y is an fp32 array whose values are all representable in `storage` (the caller's 16-bit
    data widened exactly).  The projection is the fp32-storage one, unchanged; only its
    result X is rounded to the storage format (returned widened to fp32).  The aggregate v,
    the radii u and tau are not rounded.  Also returns mask (u_j > 0: the kept columns) and
    X32, the result before rounding.
    """
    Y = np.asarray(Y)
    assert Y.dtype == np.float32
    assert np.array_equal(round_to_storage(Y, storage), Y), "Y must be representable in the storage format"
    out = dict(bilevel(Y, eta, q, columns, p))
    out["X32"] = out["X"]
    out["X"] = round_to_storage(out["X32"], storage)
    out["mask"] = np.asarray(out["u"], dtype=np.float64) > 0
    return out


def bilevel_batch(Ys, etas, q, storage="f32", p=1):
    """A batch is nothing but independent projections: one bilevel_stored per matrix."""
    assert len(Ys) == len(etas)
    return [bilevel_stored(Y, eta, q, storage, p=p) for Y, eta in zip(Ys, etas)]


# --------------------------------------------------------------------------
# Def. 5.1, Alg. 5 and its iterative form (appendix Alg. 7): tri-level
# --------------------------------------------------------------------------
def trilevel_l1infinf(Y, eta):
    """TP^{1,inf,inf}_eta of a C-order tensor Y[a, b, c].

    Axis convention: groups live on axis 0; the innermost aggregate runs over
    axis 2, the second over axis 1.  This is the paper's R^{c,n,m} tensor with
    the axis names reversed (the paper aggregates its first axis, then its
    second, and keeps groups on its last).

    Follows the iterative form step by step and keeps the intermediate radius
    matrix U2, so that "the element clip only needs u_a" is something tests
    can check rather than something assumed here.
    Returns dict(X, V, w, u, U2, tau).
    """
    Y = np.asarray(Y)
    assert Y.dtype == np.float32 and Y.ndim == 3
    d0, d1, d2 = Y.shape
    V = np.zeros((d0, d1), dtype=np.float32)           # V_inf: fibre maxima
    for c in range(d2):
        V = np.maximum(V, np.abs(Y[:, :, c]))
    w = np.zeros(d0, dtype=np.float32)                 # v_{inf,inf}
    for b in range(d1):
        w = np.maximum(w, V[:, b])
    u64, tau = project_l1_ball_nonneg(w, eta)          # u^3
    u = u64.astype(np.float32)
    U2 = np.empty_like(V)
    for a in range(d0):                                # first loop: U^2_t
        U2[a, :] = project_linf_ball(V[a, :], u[a])
    X = np.empty_like(Y)
    for a in range(d0):                                # second loop: U^1_t
        for b in range(d1):
            X[a, b, :] = project_linf_ball(Y[a, b, :], U2[a, b])
    return {"X": X, "V": V, "w": w, "u": u, "U2": U2, "tau": tau}


def trilevel_stored(Y, eta, storage):
    """TP^{1,inf,inf}_eta (Alg. 5) on a tensor kept in a 16-bit format: the fp32-storage result,
    with X rounded to the storage format; mask = kept slabs (u_a > 0)."""
    Y = np.asarray(Y)
    assert Y.dtype == np.float32
    assert np.array_equal(round_to_storage(Y, storage), Y), "Y must be representable in the storage format"
    out = dict(trilevel_l1infinf(Y, eta))
    out["X32"] = out["X"]
    out["X"] = round_to_storage(out["X32"], storage)
    out["mask"] = np.asarray(out["u"], dtype=np.float64) > 0
    return out


# --------------------------------------------------------------------------
# Def. 5.2, Alg. 6 and its iterative form (appendix Alg. 8): multi-level
# --------------------------------------------------------------------------
def _fibre_norms(A, q):
    """q-norm of every last-axis fibre of A, in fp64 (the aggregation V_nu of Sec. 5.2)."""
    A = np.asarray(A, dtype=np.float64)
    if q == "inf":
        return np.max(np.abs(A), axis=-1)
    if q == 1:
        return np.sum(np.abs(A), axis=-1)
    if q == 2:
        return np.sqrt(np.sum(A * A, axis=-1))
    raise ValueError("norm must be 'inf', 1 or 2")


def _project_fibre(y, r, q):
    """P^q_r of one fibre (fp64), by the single-vector projections defined above."""
    y = np.asarray(y, dtype=np.float64)
    if q == "inf":
        return np.copysign(np.minimum(np.abs(y), r), y)
    if q == 2:
        return project_l2_ball(y, r)
    return project_l1_ball(y, r)[0]


def multilevel(Y, norms, eta, p=1):
    """MP^nu_eta of a C-order tensor with single-axis norms, outermost norm p (l1 by default).

    `norms` lists the inner norms innermost first: norms[0] aggregates the LAST axis, norms[1]
    the one before, ... down to axis 1; axis 0 carries the groups whose aggregate vector is
    projected onto the l1 ball of radius eta.  In the paper's notation (which keeps the groups
    on the last axis and aggregates the first axes first) this is nu = ((norms[0]), ...,
    (norms[-1]), (1)) on the tensor with its axes reversed.

    Follows the iterative form: aggregate level by level up to the vector, project it, then
    for each level going back down project every fibre of that level's aggregate onto the
    ball whose radius is the corresponding entry of the level above.
    All intermediate levels in fp64; the result is rounded to fp32 once.
    Returns dict(X, w, u, tau, V (list of aggregates), U (list of projected aggregates)).
    """
    Y = np.asarray(Y)
    assert Y.dtype == np.float32 and Y.ndim >= 2 and len(norms) == Y.ndim - 1
    V = [Y.astype(np.float64)]
    for q in norms:                                   # aggregation, innermost axis first
        V.append(_fibre_norms(V[-1], q))
    w = V[-1]
    u, tau = project_outer(w, eta, p)
    U = [None] * len(V)
    U[-1] = u
    for k in range(len(norms), 0, -1):                # back down: level k radii -> level k-1
        q = norms[k - 1]
        src, rad = V[k - 1], U[k]
        out = np.empty_like(src)
        for idx in np.ndindex(rad.shape):
            out[idx] = _project_fibre(src[idx], rad[idx], q)
        U[k - 1] = out
    return {"X": U[0].astype(np.float32), "w": w, "u": u, "tau": tau, "V": V, "U": U}


def multilevel_stored(Y, norms, eta, storage, p=1):
    """MP^nu_eta (Def. 5.2, Alg. 6) on a tensor kept in a 16-bit format: the fp32-storage result,
    with X rounded to the storage format (X32 is the result before that rounding)."""
    Y = np.asarray(Y)
    assert Y.dtype == np.float32
    assert np.array_equal(round_to_storage(Y, storage), Y), "Y must be representable in the storage format"
    out = dict(multilevel(Y, norms, eta, p=p))
    out["X32"] = out["X"]
    out["X"] = round_to_storage(out["X32"], storage)
    return out

