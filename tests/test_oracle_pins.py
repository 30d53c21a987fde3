"""Pins for the CPU oracle: every stage is checked against something other than
itself -- optimality certificates of the Euclidean projection (Eq. 4), brute
force over all active-set sizes, numpy's own norm routine, closed forms,
invariants the paper states, and hand-worked fixtures."""
import itertools

import numpy as np
import pytest

from oracle import mlproj_oracle as orc
from paper_2405_02086_amd import workloads

RNG = np.random.default_rng(20240502)
QS = ["inf", 1, 2]


def rand_matrix(n, m, rng=RNG, dist="normal"):
    if dist == "normal":
        return rng.standard_normal((n, m)).astype(np.float32)
    return rng.laplace(size=(n, m)).astype(np.float32)


def lq(x, q, axis=None):
    x = np.asarray(x, dtype=np.float64)
    if q == "inf":
        return np.max(np.abs(x), axis=axis)
    if q == 1:
        return np.sum(np.abs(x), axis=axis)
    return np.sqrt(np.sum(x * x, axis=axis))


def dual(q):
    return {"inf": 1, 1: "inf", 2: 2}[q]


def assert_is_projection(y, x, r, q, tol=1e-9):
    """x = argmin_{||z||_q <= r} ||z - y||_2  (Eq. 4)  iff  x is feasible and
    <y - x, z - x> <= 0 for every feasible z.  The supremum of <y - x, z> over
    the ball is r * ||y - x||_{q*} (dual norm), so the whole family of
    inequalities collapses to one: r * ||y - x||_{q*} <= <y - x, x>."""
    y = np.asarray(y, dtype=np.float64)
    x = np.asarray(x, dtype=np.float64)
    scale = max(1.0, float(np.sum(np.abs(y))))
    assert lq(x, q) <= r + tol * scale
    g = y - x
    assert r * lq(g, dual(q)) <= float(np.dot(g, x)) + tol * scale * max(1.0, r)


# ---------------------------------------------------------------- stage pins
@pytest.mark.parametrize("q", QS)
def test_column_norms_match_numpy_norm(q):
    Y = rand_matrix(37, 53)
    ord_ = {"inf": np.inf, 1: 1, 2: 2}[q]
    ref = np.linalg.norm(Y.astype(np.float64), ord=ord_, axis=0)
    got = orc.column_norms(Y, q)
    if q == "inf":
        assert got.dtype == np.float32
        assert np.array_equal(got.astype(np.float64), ref)
    else:
        np.testing.assert_allclose(got, ref, rtol=1e-13)
    assert orc.norm_l1q(Y, q) == pytest.approx(ref.sum(), rel=1e-13)


def test_column_norms_are_per_column_not_per_row():
    Y = np.array([[1, -7], [2, 3], [-4, 5]], dtype=np.float32)
    assert orc.column_norms(Y, "inf").tolist() == [4.0, 7.0]
    assert orc.column_norms(Y, 1).tolist() == [7.0, 15.0]
    np.testing.assert_allclose(orc.column_norms(Y, 2), [21 ** 0.5, 83 ** 0.5], rtol=1e-15)


@pytest.mark.parametrize("m", [1, 2, 3, 7, 12, 40, 301])
@pytest.mark.parametrize("frac", [1e-3, 0.05, 0.3, 0.9, 0.999, 1.0, 1.7])
def test_l1_ball_projection_certificate(m, frac):
    v = np.abs(RNG.standard_normal(m)) * np.power(10.0, RNG.uniform(-2, 0, m))
    eta = frac * v.sum()
    u, tau = orc.project_l1_ball_nonneg(v, eta)
    assert_is_projection(v, u, eta, 1)
    assert np.all(u >= 0) and np.all(u <= v)
    if frac >= 1.0:
        assert tau == 0.0 and np.array_equal(u, v)
    else:
        assert tau > 0 and u.sum() == pytest.approx(eta, rel=1e-12)
        assert np.array_equal(u > 0, v > tau)


@pytest.mark.parametrize("m", [1, 2, 5, 9, 12])
def test_l1_ball_bruteforce_over_active_sets(m):
    """Enumerate every active-set size k: tau_k = (c_k - eta)/k is consistent
    iff mu_k > tau_k >= mu_{k+1}; exactly one k is, and it is the oracle's."""
    for trial in range(25):
        v = np.round(np.abs(RNG.standard_normal(m)) * 8) / 4      # ties likely
        if v.sum() == 0:
            continue
        eta = float(RNG.uniform(0.05, 0.95) * v.sum())
        mu = np.sort(v)[::-1]
        ext = np.append(mu, 0.0)
        ok = []
        for k in range(1, m + 1):
            tk = (mu[:k].sum() - eta) / k
            if mu[k - 1] > tk >= ext[k]:
                ok.append((k, tk))
        assert len(ok) == 1
        u, tau = orc.project_l1_ball_nonneg(v, eta)
        assert tau == pytest.approx(ok[0][1], abs=1e-12)
        assert int((u > 0).sum()) == ok[0][0]
        # root of the monotone function tau -> sum max(v - tau, 0) - eta by bisection
        lo, hi = 0.0, float(v.max())
        for _ in range(200):
            mid = 0.5 * (lo + hi)
            if np.maximum(v - mid, 0).sum() > eta:
                lo = mid
            else:
                hi = mid
        assert tau == pytest.approx(0.5 * (lo + hi), abs=1e-12)


def test_l1_ball_projection_beats_random_feasible_points():
    v = np.abs(RNG.standard_normal(6)) + 0.1
    eta = 0.4 * v.sum()
    u, _ = orc.project_l1_ball_nonneg(v, eta)
    d0 = np.linalg.norm(u - v)
    for _ in range(2000):
        z = RNG.standard_normal(6)
        z *= RNG.uniform(0, 1) * eta / np.abs(z).sum()
        assert np.linalg.norm(z - v) >= d0 - 1e-12


def test_l1_ball_signed_vector_certificate():
    for m in (1, 4, 33):
        y = RNG.standard_normal(m) * 3
        r = 0.3 * np.abs(y).sum()
        x, tau = orc.project_l1_ball(y, r)
        assert_is_projection(y, x, r, 1)
        assert np.all(np.sign(x) * np.sign(y) >= 0)


def test_l1_ball_edge_cases():
    u, tau = orc.project_l1_ball_nonneg(np.array([2.0, 2.0, 2.0, 2.0]), 2.0)
    assert tau == pytest.approx(1.5) and np.allclose(u, 0.5)          # equal entries: tau = c - eta/m
    u, tau = orc.project_l1_ball_nonneg(np.array([1.0, 4.0, 0.0]), 0.0)
    assert np.array_equal(u, np.zeros(3)) and tau == 4.0               # eta = 0
    u, tau = orc.project_l1_ball_nonneg(np.array([1.0, 4.0, 0.0]), 5.0)
    assert np.array_equal(u, [1.0, 4.0, 0.0]) and tau == 0.0           # boundary of the ball
    u, tau = orc.project_l1_ball_nonneg(np.zeros(4), 1.0)
    assert np.array_equal(u, np.zeros(4)) and tau == 0.0


def test_linf_and_l2_ball_projection_certificates():
    for n in (1, 5, 64):
        y = (RNG.standard_normal(n) * 2).astype(np.float32)
        for r in (0.0, float(np.float32(0.3)), 1.0, 10.0):
            x = orc.project_linf_ball(y, np.float32(r))
            assert x.dtype == np.float32
            assert_is_projection(y, x, r, "inf")
            x2 = orc.project_l2_ball(y, r)
            assert_is_projection(y, x2, r, 2)
    # the sign survives the clip: a negative entry is clipped to -r, not left alone
    assert orc.project_linf_ball(np.float32([-3.0, 3.0, -0.5]), np.float32(1.0)).tolist() == [-1.0, 1.0, -0.5]


# ---------------------------------------------------------- bi-level as a whole
@pytest.mark.parametrize("q", QS)
@pytest.mark.parametrize("shape", [(1, 1), (1, 9), (9, 1), (7, 5), (33, 20)])
@pytest.mark.parametrize("frac", [0.02, 0.4, 0.95])
def test_bilevel_is_the_composition_of_two_projections(q, shape, frac):
    """Eq. 5: u is the projection of v_q onto the l1 ball of radius eta, and each
    column x_j is the projection of y_j onto the l_q ball of radius u_j."""
    Y = rand_matrix(*shape)
    eta = frac * orc.norm_l1q(Y, q)
    out = orc.bilevel(Y, eta, q)
    v = lq(Y, q, axis=0)
    np.testing.assert_allclose(out["v"], v, rtol=1e-12)
    # for q = inf the oracle reports u rounded to fp32 (the radius the fp32 clip uses)
    assert_is_projection(v, out["u"], eta, 1, tol=3e-7 if q == "inf" else 1e-9)
    for j in range(shape[1]):
        assert_is_projection(Y[:, j], out["X"][:, j], float(out["u"][j]), q, tol=3e-7)
    assert orc.norm_l1q(out["X"], q) == pytest.approx(eta, rel=1e-5)


@pytest.mark.parametrize("q", QS)
def test_golden_worked_2x2(golden, q):
    g = golden("bilevel_worked_2x2.txt")
    Y = np.array(g["Y"], dtype=np.float32)
    cases = [c for c in g["cases"] if c["q"] == q]
    assert cases
    for c in cases:
        out = orc.bilevel(Y, c["eta"], q)
        np.testing.assert_allclose(out["v"], c["v"], rtol=1e-15)
        assert out["tau"] == pytest.approx(c["tau"], rel=1e-15)
        np.testing.assert_allclose(out["u"], c["u"], rtol=1e-7, atol=1e-15)
        np.testing.assert_allclose(out["X"], np.array(c["X"]), rtol=1e-7, atol=0)


@pytest.mark.parametrize("q", QS)
def test_inside_the_ball_is_returned_bit_exactly_and_eta_zero_gives_zero(q):
    Y = rand_matrix(19, 11)
    nrm = orc.norm_l1q(Y, q)
    for eta in (nrm, 1.5 * nrm):
        out = orc.bilevel(Y, eta, q)
        assert np.array_equal(out["X"], Y)
        assert out["tau"] == 0.0
    out = orc.bilevel(Y, 0.0, q)
    assert not out["X"].any() and not np.asarray(out["u"]).any()


def test_single_column_is_plain_linf_ball_projection():
    Y = rand_matrix(50, 1)
    eta = 0.7
    out = orc.bilevel_l1inf(Y, eta)
    np.testing.assert_array_equal(out["X"], np.clip(Y, -np.float32(eta), np.float32(eta)))


@pytest.mark.parametrize("q", QS)
def test_single_row_is_plain_l1_ball_projection(q):
    Y = rand_matrix(1, 40)
    eta = 0.25 * np.abs(Y).sum()
    out = orc.bilevel(Y, eta, q)
    assert_is_projection(Y[0], out["X"][0], eta, 1, tol=3e-7)


@pytest.mark.parametrize("q", QS)
def test_invariants_idempotence_homogeneity_equivariance(q):
    Y = rand_matrix(24, 17, dist="laplace")
    eta = np.float32(0.2 * orc.norm_l1q(Y, q))
    X = orc.bilevel(Y, float(eta), q)["X"]
    # the paper's one-iteration claim (Sec. 4.1): projecting again changes nothing
    X2 = orc.bilevel(X, float(eta), q)["X"]
    np.testing.assert_allclose(X2, X, rtol=1e-5, atol=1e-6)
    assert np.all(np.abs(X) <= np.abs(Y)) and np.all(X * Y >= 0)
    # positive homogeneity, exact for a power of two
    X4 = orc.bilevel(4 * Y, 4 * float(eta), q)["X"]
    np.testing.assert_allclose(X4, 4 * X, rtol=1e-6 if q != "inf" else 0, atol=0)
    # equivariance: column permutation, row permutation, entrywise sign flips
    pc, pr = RNG.permutation(17), RNG.permutation(24)
    S = RNG.choice(np.float32([-1, 1]), size=Y.shape)
    tol = dict(rtol=1e-6, atol=1e-7) if q != "inf" else dict(rtol=0, atol=0)
    np.testing.assert_allclose(orc.bilevel(Y[:, pc], float(eta), q)["X"], X[:, pc], **tol)
    np.testing.assert_allclose(orc.bilevel(Y[pr, :], float(eta), q)["X"], X[pr, :], **tol)
    np.testing.assert_allclose(orc.bilevel(Y * S, float(eta), q)["X"], X * S, **tol)


def test_l1inf_entries_are_copied_or_clipped_to_the_radius():
    Y = rand_matrix(64, 48)
    out = orc.bilevel_l1inf(Y, 0.3 * orc.norm_l1q(Y, "inf"))
    X, u = out["X"], out["u"]
    assert np.all((X == Y) | (np.abs(X) == u[None, :]))
    assert np.array_equal(np.abs(X).max(axis=0), u)
    assert np.array_equal(u == 0, out["v"].astype(np.float64) <= out["tau"])


def test_l11_inner_thresholds_share_the_outer_threshold():
    """For a surviving column, sum_i min(|Y_ij|, tau_j) = v_j - u_j = tau."""
    Y = rand_matrix(40, 12)
    out = orc.bilevel_l11(Y, 0.3 * orc.norm_l1q(Y, 1))
    keep = out["u"] > 0
    assert keep.any()
    s = np.minimum(np.abs(Y.astype(np.float64)), out["tau_col"][None, :]).sum(axis=0)
    np.testing.assert_allclose(s[keep], out["tau"], rtol=1e-12)


def test_column_sampling_agrees_with_full_run():
    Y = rand_matrix(30, 10)
    for q in QS:
        eta = 0.5 * orc.norm_l1q(Y, q)
        full = orc.bilevel(Y, eta, q)["X"]
        part = orc.bilevel(Y, eta, q, columns=[2, 7])["X"]
        assert np.array_equal(part[:, [2, 7]], full[:, [2, 7]])
        assert np.isnan(part[:, 0]).all()


# ------------------------------------------------------------------ tri-level
def test_golden_trilevel_worked(golden):
    g = golden("trilevel_worked_2x2x2.txt")
    out = orc.trilevel_l1infinf(np.array(g["Y"], dtype=np.float32), g["eta"])
    for key in ("V", "w", "u", "U2", "X"):
        np.testing.assert_array_equal(out[key], np.array(g[key], dtype=np.float32))
    assert out["tau"] == g["tau"]


@pytest.mark.parametrize("shape", [(3, 4, 5), (1, 6, 2), (6, 1, 1), (5, 2, 9)])
def test_trilevel_is_bilevel_of_the_fibre_maxima_then_fibre_clips(shape):
    """Def. 5.1: U-hat = BP^{1,inf}_eta(V_inf), then each fibre is projected onto the
    l_inf ball of its own radius.  Groups on axis 0 means V_inf is used as a matrix
    whose columns are indexed by axis 0, i.e. transposed to (d1, d0)."""
    Y = RNG.standard_normal(shape).astype(np.float32)
    V = np.abs(Y).max(axis=2)
    eta = 0.35 * float(V.max(axis=1).astype(np.float64).sum())
    out = orc.trilevel_l1infinf(Y, eta)
    bi = orc.bilevel_l1inf(np.ascontiguousarray(V.T), eta)
    assert np.array_equal(out["U2"], bi["X"].T)
    for a, b in itertools.product(range(shape[0]), range(shape[1])):
        assert_is_projection(Y[a, b], out["X"][a, b], float(out["U2"][a, b]), "inf")
    # collapse: the element clip only ever needs u_a, and the whole operator equals the
    # bi-level projection of the (d1*d2) x d0 matrix whose columns are the axis-0 slabs
    assert np.array_equal(out["X"], orc.project_linf_ball(Y, out["u"][:, None, None]))
    flat = np.ascontiguousarray(Y.reshape(shape[0], -1).T)
    assert np.array_equal(orc.bilevel_l1inf(flat, eta)["X"].T.reshape(shape), out["X"])


# ----------------------------------------------------- seeded workload generators
def test_generators_are_seeded_and_shaped():
    w, Y = workloads.make("small_256x128")
    assert Y.shape == (256, 128) and Y.dtype == np.float32 and Y.flags.c_contiguous
    _, Y2 = workloads.make("small_256x128")
    assert np.array_equal(Y, Y2)
    Z = workloads.generate((64, 32), "normal_colscale", 5)
    s = np.abs(Z).max(axis=0)
    assert s.max() / s.min() > 5          # column maxima really vary
    L = workloads.generate((400, 50), "laplace", 6)
    assert abs(np.abs(L).mean() - 1.0) < 0.05
    U = workloads.generate((100, 100), "uniform", 7)
    assert U.min() >= 0 and U.max() < 1


def test_small_workload_through_the_oracle():
    w, Y = workloads.make("small_256x128")
    eta = float(np.float32(w.eta_frac * orc.norm_l1q(Y, "inf")))
    out = orc.bilevel_l1inf(Y, eta)
    assert orc.norm_l1q(out["X"], "inf") == pytest.approx(eta, rel=1e-5)
    zeroed = int((out["u"] == 0).sum())
    assert 0 < zeroed < 128


# ---------------------------------------------------------------- multi-level
def test_golden_multilevel_l111_worked(golden):
    g = golden("multilevel_worked_2x2x2.txt")
    out = orc.multilevel(np.array(g["Y"], dtype=np.float32), g["norms"], g["eta"])
    np.testing.assert_allclose(out["w"], g["w"], rtol=1e-15)
    assert out["tau"] == pytest.approx(g["tau"], rel=1e-15)
    np.testing.assert_allclose(out["u"], g["u"], rtol=1e-15)
    np.testing.assert_allclose(out["U"][1], np.array(g["U1"]), rtol=1e-15, atol=1e-15)
    np.testing.assert_allclose(out["X"], np.array(g["X"]), rtol=1e-7, atol=0)


@pytest.mark.parametrize("q", QS)
def test_multilevel_with_one_inner_norm_is_the_bilevel_projection(q):
    """nu = ((q),(1)) is the bi-level l1,q projection (Sec. 5.2); with groups on axis 0 the
    matrix is the transpose of the column-group layout."""
    Y = rand_matrix(13, 21)                      # 21 column groups
    eta = 0.3 * orc.norm_l1q(Y, q)
    bi = orc.bilevel(Y, eta, q)
    ml = orc.multilevel(np.ascontiguousarray(Y.T), [q], eta)
    np.testing.assert_allclose(ml["X"].T, bi["X"], rtol=1e-6, atol=1e-7)
    assert ml["tau"] == pytest.approx(bi["tau"], rel=1e-12)


def test_multilevel_inf_inf_is_the_trilevel_projection():
    Y = RNG.standard_normal((5, 4, 7)).astype(np.float32)
    eta = 0.4 * float(np.abs(Y).reshape(5, -1).max(axis=1).astype(np.float64).sum())
    tri = orc.trilevel_l1infinf(Y, eta)
    ml = orc.multilevel(Y, ["inf", "inf"], eta)
    assert np.array_equal(ml["X"], tri["X"])
    assert np.array_equal(ml["U"][1].astype(np.float32), tri["U2"])


@pytest.mark.parametrize("norms", [[1, 1], [2, 2], ["inf", 1], [1, "inf"], [2, "inf"], [1, 2], ["inf", 2, 1], [1, 1, 1]])
@pytest.mark.parametrize("frac", [0.05, 0.6, 1.5])
def test_multilevel_every_level_is_a_projection(norms, frac):
    """Def. 5.2: the top vector is projected onto the l1 ball, and at every level each fibre
    of that level's aggregate is the projection onto the ball of the radius from above."""
    shape = (4, 3, 5) if len(norms) == 2 else (3, 2, 3, 4)
    Y = RNG.standard_normal(shape).astype(np.float32)
    nrm = Y.astype(np.float64)
    for q in norms:
        nrm = lq(nrm, q, axis=-1)
    eta = frac * float(nrm.sum())
    out = orc.multilevel(Y, norms, eta)
    np.testing.assert_allclose(out["w"], nrm, rtol=1e-13)
    assert_is_projection(out["w"], out["u"], eta, 1)
    for k in range(len(norms), 0, -1):
        q = norms[k - 1]
        for idx in np.ndindex(out["U"][k].shape):
            assert_is_projection(out["V"][k - 1][idx], out["U"][k - 1][idx], float(out["U"][k][idx]), q)
    # the result is feasible for the nested norm, and on the boundary when Y was outside
    got = out["X"].astype(np.float64)
    for q in norms:
        got = lq(got, q, axis=-1)
    assert got.sum() <= eta * (1 + 1e-5)
    if frac < 1:
        assert got.sum() == pytest.approx(eta, rel=1e-5)
    else:
        assert np.array_equal(out["X"], Y)


# ---------------------------------------------------------------- other outer norms (Alg. 1, general p)
@pytest.mark.parametrize("p", [2, "inf"])
@pytest.mark.parametrize("q", QS)
@pytest.mark.parametrize("frac", [0.05, 0.5, 1.2])
def test_bilevel_pq_is_the_composition_of_two_projections(p, q, frac):
    """Alg. 1 for a general outer norm: u = P^p_eta(v_q), then x_j = P^q_{u_j}(y_j)."""
    Y = rand_matrix(23, 14)
    v = lq(Y, q, axis=0)
    eta = frac * float(lq(v, p))
    out = orc.bilevel(Y, eta, q, p=p)
    assert_is_projection(v, out["u"], eta, p, tol=3e-7 if q == "inf" else 1e-9)
    for j in range(Y.shape[1]):
        assert_is_projection(Y[:, j], out["X"][:, j], float(out["u"][j]), q, tol=3e-7)
    got = lq(lq(out["X"], q, axis=0), p)
    if frac < 1:
        assert got == pytest.approx(eta, rel=1e-5)
    else:
        assert np.array_equal(out["X"], Y)


def test_outer_projection_closed_forms():
    v = np.array([3.0, 4.0, 0.0])
    u, tau = orc.project_outer(v, 2.5, 2)
    np.testing.assert_allclose(u, [1.5, 2.0, 0.0], rtol=1e-15)        # ||v||_2 = 5 -> scale 1/2
    u, tau = orc.project_outer(v, 3.5, "inf")
    assert u.tolist() == [3.0, 3.5, 0.0] and tau == 0.0
    u, _ = orc.project_outer(v, 6.0, 2)
    assert np.array_equal(u, v)


@pytest.mark.parametrize("p", [2, "inf"])
def test_multilevel_outer_norm(p):
    Y = RNG.standard_normal((6, 3, 5)).astype(np.float32)
    norms = [1, "inf"]
    w = lq(lq(Y, 1, axis=-1), "inf", axis=-1)
    eta = 0.4 * float(lq(w, p))
    out = orc.multilevel(Y, norms, eta, p=p)
    assert_is_projection(w, out["u"], eta, p)
    got = lq(lq(lq(out["X"], 1, axis=-1), "inf", axis=-1), p)
    assert got == pytest.approx(eta, rel=1e-5)


# ------------------------------------------------------------------ 16-bit storage
def test_storage_rounding_hand_cases():
    """Ties go to the even pattern; values written as exact binary fractions."""
    bf = lambda x: float(orc.round_to_storage(np.float32([x]), "bf16")[0])
    assert bf(1.0 + 2.0 ** -8) == 1.0                        # halfway between 1 and 1+2^-7: even is 1
    assert bf(1.0 + 3 * 2.0 ** -8) == 1.0 + 2.0 ** -6        # halfway between 1+2^-7 and 1+2^-6: even is up
    assert bf(1.0 + 2.0 ** -8 + 2.0 ** -20) == 1.0 + 2.0 ** -7
    assert bf(-(1.0 + 2.0 ** -8 - 2.0 ** -20)) == -1.0
    assert bf(3.3895313892515355e38) == 3.3895313892515355e38          # the largest finite bf16 value
    assert bf(0.0) == 0.0 and np.signbit(orc.round_to_storage(np.float32([-0.0]), "bf16")[0])
    h = lambda x: float(orc.round_to_storage(np.float32([x]), "f16")[0])
    assert h(1.0 + 2.0 ** -11) == 1.0 and h(1.0 + 3 * 2.0 ** -11) == 1.0 + 2.0 ** -9
    assert h(65504.0) == 65504.0 and h(65519.0) == 65504.0 and np.isinf(h(65520.0))
    assert h(2.0 ** -24) == 2.0 ** -24 and h(2.0 ** -25) == 0.0 and h(1.5 * 2.0 ** -24) == 2.0 ** -23
    x = np.float32([0.1, -2.5, 7.0])
    assert np.array_equal(orc.round_to_storage(x, "f32"), x)


@pytest.mark.parametrize("storage", ["bf16", "f16"])
def test_storage_rounding_matches_a_library_conversion_and_is_monotone(storage):
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(5)
    x = np.concatenate([rng.standard_normal(200000) * 10.0 ** rng.uniform(-6, 4, 200000),
                        np.float32([0.0, -0.0, 1e-40, -1e-40, 6.0e-8, 65504.0])]).astype(np.float32)
    ties = (np.arange(1 << 16, dtype=np.uint32) << 16 | 0x8000).view(np.float32)   # every bf16 midpoint
    ties = ties[np.isfinite(ties)]
    x = np.concatenate([x, ties])
    if storage == "f16":
        x = x[np.abs(x) < 65000]
    want = torch.from_numpy(x).to({"bf16": torch.bfloat16, "f16": torch.float16}[storage]).float().numpy()
    got = orc.round_to_storage(x, storage)
    assert np.array_equal(got.view(np.uint32), want.view(np.uint32))
    assert np.array_equal(orc.round_to_storage(got, storage), got)        # idempotent
    xs = np.sort(x)
    assert np.all(np.diff(orc.round_to_storage(xs, storage)) >= 0)        # monotone
    rel = np.abs(got.astype(np.float64) - x) / np.maximum(np.abs(x), 1e-30)
    normal = (np.abs(x) > (1e-37 if storage == "bf16" else 6.2e-5)) & np.isfinite(got)
    assert rel[normal].max() <= 2.0 ** (-8 if storage == "bf16" else -11)   # half a unit in the last place


@pytest.mark.parametrize("storage", ["bf16", "f16"])
@pytest.mark.parametrize("q", QS)
def test_bilevel_stored_is_the_fp32_result_rounded(storage, q):
    Y = orc.round_to_storage(rand_matrix(40, 30), storage)
    eta = 0.3 * orc.norm_l1q(Y, q)
    out = orc.bilevel_stored(Y, eta, q, storage)
    ref = orc.bilevel(Y, eta, q)
    assert np.array_equal(out["X32"], ref["X"]) and out["tau"] == ref["tau"]
    assert np.array_equal(out["X"], orc.round_to_storage(ref["X"], storage))
    assert np.array_equal(out["mask"], np.abs(ref["X"]).max(axis=0) > 0)
    # rounding moves every entry by at most half a unit in the last place of the format
    half_ulp = 2.0 ** (-8 if storage == "bf16" else -11)
    assert np.all(np.abs(out["X"].astype(np.float64) - ref["X"]) <= half_ulp * np.abs(ref["X"]) + 1e-7)
    assert lq(lq(out["X"], q, axis=0), 1) <= eta * (1 + 2 * half_ulp)
    if q == "inf":   # entries under the radius are untouched, the others sit on the rounded radius
        ur = orc.round_to_storage(np.asarray(ref["u"], dtype=np.float32), storage)
        inside = np.abs(Y) <= np.asarray(ref["u"], dtype=np.float32)[None, :]
        assert np.array_equal(out["X"][inside], Y[inside])
        assert np.array_equal(np.abs(out["X"])[~inside], np.broadcast_to(ur, Y.shape)[~inside])
    with pytest.raises(AssertionError):
        orc.bilevel_stored(Y + np.float32(1e-3), eta, q, storage)


def test_batch_is_independent_projections():
    """Each member of a batch satisfies the single-matrix certificates on its own."""
    shapes = [(5, 7), (40, 3), (1, 9)]
    Ys = [rand_matrix(*sh) for sh in shapes]
    etas = [0.3 * orc.norm_l1q(Y, "inf") for Y in Ys]
    outs = orc.bilevel_batch(Ys, etas, "inf")
    assert len(outs) == 3
    for Y, eta, out in zip(Ys, etas, outs):
        v = lq(Y, "inf", axis=0)
        assert_is_projection(v, out["u"], eta, 1, tol=3e-7)
        for j in range(Y.shape[1]):
            assert_is_projection(Y[:, j], out["X"][:, j], float(out["u"][j]), "inf", tol=3e-7)


@pytest.mark.parametrize("storage", ["bf16", "f16"])
def test_trilevel_stored_is_the_fp32_result_rounded(storage):
    Y = orc.round_to_storage(RNG.standard_normal((6, 5, 9)).astype(np.float32), storage)
    w = np.abs(Y).reshape(6, -1).max(axis=1)
    eta = 0.4 * float(w.sum())
    out = orc.trilevel_stored(Y, eta, storage)
    ref = orc.trilevel_l1infinf(Y, eta)
    assert np.array_equal(out["X32"], ref["X"]) and np.array_equal(out["X"], orc.round_to_storage(ref["X"], storage))
    assert np.array_equal(out["mask"], np.abs(ref["X"]).reshape(6, -1).max(axis=1) > 0)
    ur = orc.round_to_storage(np.asarray(ref["u"], dtype=np.float32), storage)
    inside = np.abs(Y) <= np.asarray(ref["u"], dtype=np.float32)[:, None, None]
    assert np.array_equal(out["X"][inside], Y[inside])
    assert np.array_equal(np.abs(out["X"])[~inside], np.broadcast_to(ur[:, None, None], Y.shape)[~inside])


@pytest.mark.parametrize("storage", ["bf16", "f16"])
@pytest.mark.parametrize("norms", [[1, 1], [2, "inf"], ["inf", 1], [2]])
def test_multilevel_stored_is_the_fp32_result_rounded(storage, norms):
    """Storage only: the stored result is the fp32 result rounded once; entries the projection
    leaves alone come back exactly, and so does everything when the radius covers the norm."""
    shape = (5, 4, 8)[: len(norms) + 1]
    Y = orc.round_to_storage(RNG.standard_normal(shape).astype(np.float32), storage)
    ref_in = orc.multilevel(Y, norms, 1e9)
    assert np.array_equal(orc.multilevel_stored(Y, norms, 1e9, storage)["X"], Y) and ref_in["tau"] == 0.0
    eta = 0.3 * float(np.sum(ref_in["w"]))
    out = orc.multilevel_stored(Y, norms, eta, storage)
    ref = orc.multilevel(Y, norms, eta)
    assert np.array_equal(out["X32"], ref["X"])
    assert np.array_equal(out["X"], orc.round_to_storage(ref["X"], storage))
    assert np.all(np.abs(out["X"]) <= np.abs(Y)) and np.all(out["X"] * Y >= 0)   # rounding is monotone and odd


# --------------------------------------------------------------------------
# weighted l1 ball (the l_w1 outer norm Sec. 3 names)
# --------------------------------------------------------------------------
def test_weighted_l1_with_unit_weights_is_the_plain_l1_projection():
    v = np.abs(RNG.standard_normal(200))
    for eta in (0.0, 0.5, 10.0, 1e6):
        u, tau = orc.project_weighted_l1_ball_nonneg(v, np.ones_like(v), eta)
        u0, tau0 = orc.project_l1_ball_nonneg(v, eta)
        assert np.allclose(u, u0, rtol=0, atol=1e-14) and tau == pytest.approx(tau0, abs=1e-14)


def test_weighted_l1_optimality_certificate():
    """KKT: u_j > 0 => (v_j - u_j) / w_j = tau; u_j = 0 => v_j / w_j <= tau; sum w_j u_j = eta."""
    for seed in range(20):
        rng = np.random.default_rng([seed, 5150])
        m = int(rng.integers(1, 300))
        v = np.abs(rng.standard_normal(m)) * rng.choice([0.0, 1.0, 5.0], m)
        w = np.exp(rng.uniform(-2, 2, m))
        total = float(np.sum(w * v))
        if total == 0.0:
            continue
        eta = total * float(rng.uniform(0.01, 0.99))
        u, tau = orc.project_weighted_l1_ball_nonneg(v, w, eta)
        assert tau > 0 and np.all(u >= 0) and np.sum(w * u) == pytest.approx(eta, rel=1e-12)
        act = u > 0
        assert np.allclose((v[act] - u[act]) / w[act], tau, rtol=1e-12, atol=0)
        assert np.all(v[~act] / w[~act] <= tau * (1 + 1e-12))
        # inside the ball nothing moves
        u_in, tau_in = orc.project_weighted_l1_ball_nonneg(v, w, total * 1.01)
        assert np.array_equal(u_in, v) and tau_in == 0.0


def test_weighted_l1_against_a_constrained_minimiser_and_brute_force():
    """scipy's SLSQP on min ||u - v||^2 s.t. sum w u <= eta, u >= 0 (small sizes), and brute
    force over all active sets (tiny sizes): two routes that share nothing with the sort."""
    from itertools import combinations
    from scipy.optimize import minimize
    for seed in range(6):
        rng = np.random.default_rng([seed, 909])
        m = 6
        v = np.abs(rng.standard_normal(m)) + 0.1
        w = np.exp(rng.uniform(-1, 1, m))
        eta = 0.4 * float(np.sum(w * v))
        u, tau = orc.project_weighted_l1_ball_nonneg(v, w, eta)
        res = minimize(lambda x: 0.5 * np.sum((x - v) ** 2), np.zeros(m), jac=lambda x: x - v, method="SLSQP",
                       bounds=[(0, None)] * m, constraints=[{"type": "ineq", "fun": lambda x: eta - np.dot(w, x),
                                                             "jac": lambda x: -w}], options={"ftol": 1e-14, "maxiter": 500})
        assert res.success and np.allclose(res.x, u, atol=1e-6)
        best, best_d = None, np.inf
        for k in range(1, m + 1):
            for A in combinations(range(m), k):
                A = list(A)
                t = (np.dot(w[A], v[A]) - eta) / np.dot(w[A], w[A])
                cand = np.zeros(m)
                cand[A] = v[A] - t * w[A]
                if t >= 0 and np.all(cand >= 0) and np.dot(w, cand) <= eta * (1 + 1e-12):
                    d = np.sum((cand - v) ** 2)
                    if d < best_d:
                        best, best_d = cand, d
        assert np.allclose(best, u, atol=1e-12)


def test_bilevel_with_weighted_outer_norm():
    """Alg. 1 with the weighted l1 ball as outer norm: the radii come from the weighted projection of
    the aggregate, every column lands on (or inside) its own ball, the weighted norm of the result is eta."""
    Y = RNG.standard_normal((30, 12)).astype(np.float32)
    w = np.exp(RNG.uniform(-1, 1, 12))
    for q in ("inf", 1, 2):
        v = orc.column_norms(Y, q).astype(np.float64)
        eta = 0.3 * float(np.sum(w * v))
        out = orc.bilevel(Y, eta, q, p=("w1", w))
        u, tau = orc.project_weighted_l1_ball_nonneg(v, w, eta)
        assert np.allclose(np.asarray(out["u"], dtype=np.float64), u, rtol=1e-6) and out["tau"] == tau
        vx = orc.column_norms(out["X"], q).astype(np.float64)
        assert np.allclose(vx, u, rtol=1e-5, atol=1e-6)
        assert np.dot(w, vx) == pytest.approx(eta, rel=1e-5)

