"""The entry point that allocates nothing (bilevel_proj_l1inf_no_alloc) against the entry point
it is a variant of, through the C ABI: same kernels on the library's built-in scratch buffer, so
every output must have the same bits.  Two calls in a row share that buffer and the second is the
smaller one, so whatever the first left behind must not reach the second."""
import numpy as np
import pytest

from oracle import mlproj_oracle as orc

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def mp():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2405_02086_amd import binding
    binding.lib()            # raises if the HIP library is not built: no fallback
    return binding


def both_ways(mp, Y, eta):
    dev = torch.device("cuda:0")
    n, m = Y.shape
    Yd = torch.from_numpy(Y).to(dev)
    out = []
    for no_alloc in (False, True):
        X = torch.full_like(Yd, float("nan"))
        v = torch.full((m,), -1.0, dtype=torch.float32, device=dev)
        u = torch.full((m,), -1.0, dtype=torch.float32, device=dev)
        if no_alloc:
            mp.bilevel_proj_l1inf_no_alloc(Yd, eta, X, v_out=v, u_out=u)
        else:
            mp.bilevel_proj_l1inf(Yd, eta, X=X, workspace=mp.Workspace.for_call("l1inf", n, m, device=dev), v_out=v, u_out=u)
        torch.cuda.synchronize()
        out.append((X.cpu().numpy(), v.cpu().numpy(), u.cpu().numpy()))
    return out


# (the first of each pair is the larger input; between them they take the several-workgroup search,
# the one-workgroup search, the search fused into the map pass and the one-kernel path)
@pytest.mark.parametrize("shapes", [((8, 262144), (300, 1000)), ((2048, 3000), (256, 128)), ((64, 20000), (7, 5))])
def test_two_calls_in_a_row_match_the_workspace_entry_point(mp, shapes):
    rng = np.random.default_rng([shapes[0][0], shapes[0][1]])
    for shape in shapes:
        Y = rng.standard_normal(shape).astype(np.float32)
        Y *= np.power(10.0, rng.uniform(-1.0, 0.0, shape[1])).astype(np.float32)[None, :]
        eta = float(np.float32(0.2 * orc.norm_l1q(Y, "inf")))
        (X0, v0, u0), (X1, v1, u1) = both_ways(mp, Y, eta)
        assert np.array_equal(v0, v1) and np.array_equal(u0, u1)
        assert np.array_equal(X0.view(np.uint32), X1.view(np.uint32))
        # ... and the oracle, to the bar of the other parity tests
        ref = orc.bilevel_l1inf(Y, eta)
        assert np.array_equal(v1, ref["v"])
        np.testing.assert_allclose(u1, ref["u"], rtol=1e-5, atol=1e-6)
        assert np.array_equal(u1 == 0, ref["u"] == 0)
        np.testing.assert_allclose(X1, ref["X"], rtol=1e-5, atol=1e-6)


def test_in_place_and_inside_the_ball(mp):
    rng = np.random.default_rng(7)
    dev = torch.device("cuda:0")
    Y = rng.standard_normal((500, 700)).astype(np.float32)
    eta = float(np.float32(0.3 * orc.norm_l1q(Y, "inf")))
    Z = torch.from_numpy(Y).to(dev)
    mp.bilevel_proj_l1inf_no_alloc(Z, eta, Z)                      # X = Y
    torch.cuda.synchronize()
    np.testing.assert_allclose(Z.cpu().numpy(), orc.bilevel_l1inf(Y, eta)["X"], rtol=1e-5, atol=1e-6)
    Yd = torch.from_numpy(Y).to(dev)
    X = torch.empty_like(Yd)
    mp.bilevel_proj_l1inf_no_alloc(Yd, float(np.float32(2.0 * orc.norm_l1q(Y, "inf"))), X)
    torch.cuda.synchronize()
    assert torch.equal(X, Yd)                                      # inside the ball: X = Y bit for bit


def test_inputs_beyond_the_built_in_buffer_are_refused(mp):
    dev = torch.device("cuda:0")
    Y = torch.zeros((1, 1 << 20), dtype=torch.float32, device=dev)   # a million columns: 16 MiB of workspace
    X = torch.full_like(Y, 5.0)
    with pytest.raises(mp.MlprojError) as err:
        mp.bilevel_proj_l1inf_no_alloc(Y, 1.0, X)
    assert err.value.status == -9
    torch.cuda.synchronize()
    assert bool((X == 5.0).all())                                    # nothing was enqueued
