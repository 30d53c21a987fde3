"""Host-side checks that need no GPU: the shared library loads, exports every function the
header declares, sizes workspaces sanely, and rejects bad arguments before enqueuing."""
import ctypes
import os
import re

import pytest

from paper_2405_02086_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE = ctypes.c_void_p(1 << 20)       # non-null, 256-aligned; never dereferenced on these paths
F = ctypes.c_float


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(binding.LIB_PATH):
        binding.build()
    return binding.lib()


def declared_functions():
    text = open(os.path.join(ROOT, "include", "mlproj.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"^\s*(?:const\s+char\s*\*|int)\s+(\w+)\s*\(", text, flags=re.M)))


def test_every_declared_function_is_exported(lib):
    names = declared_functions()
    assert set(names) == set(binding.EXPORTS)
    for n in names:
        assert getattr(lib, n) is not None


def test_version_and_status_strings(lib):
    assert lib.mlproj_version() >= 200
    seen = {lib.mlproj_status_string(s) for s in range(0, -10, -1)}
    assert len(seen) == 10 and b"unknown status" not in seen
    assert lib.mlproj_status_string(-99) == b"unknown status"


def test_workspace_sizes(lib):
    small = binding.workspace_bytes("l1inf", 1, 1)
    assert 0 < small <= 1 << 16
    for variant, dims in [("l1inf", (4096, 4096, 1)), ("l1inf", (262144, 256, 1)), ("l1inf", (256, 262144, 1)),
                          ("l11", (16384, 16384, 1)), ("l12", (16384, 16384, 1)), ("tri", (256, 256, 256))]:
        b = binding.workspace_bytes(variant, *dims)
        assert b % 256 == 0 and small <= b < 64 << 20, (variant, dims, b)
    out = ctypes.c_size_t(0)
    assert lib.mlproj_workspace_bytes(0, 0, 4, 1, ctypes.byref(out)) == -2
    assert lib.mlproj_workspace_bytes(0, 4, -1, 1, ctypes.byref(out)) == -2
    assert lib.mlproj_workspace_bytes(0, 4, 4, 2, ctypes.byref(out)) == -2     # bi-level takes d2 = 1
    assert lib.mlproj_workspace_bytes(9, 4, 4, 1, ctypes.byref(out)) == -6
    assert lib.mlproj_workspace_bytes(0, 1 << 30, 1 << 30, 1, ctypes.byref(out)) == -3
    assert lib.mlproj_workspace_bytes(0, 4, 1 << 32, 1, ctypes.byref(out)) == -3
    assert lib.mlproj_workspace_bytes(0, 4, 4, 1, None) == -1


@pytest.mark.parametrize("name", ["bilevel_proj_l1inf", "bilevel_proj_l11", "bilevel_proj_l12"])
def test_bilevel_argument_checks_happen_before_any_launch(lib, name):
    fn = getattr(lib, name)
    big = 1 << 30
    assert fn(None, FAKE, 4, 4, F(1), FAKE, big, None, None, None) == -1
    assert fn(FAKE, None, 4, 4, F(1), FAKE, big, None, None, None) == -1
    assert fn(FAKE, FAKE, 4, 4, F(1), None, big, None, None, None) == -1
    assert fn(FAKE, FAKE, 0, 4, F(1), FAKE, big, None, None, None) == -2
    assert fn(FAKE, FAKE, 4, -3, F(1), FAKE, big, None, None, None) == -2
    assert fn(FAKE, FAKE, 1 << 21, 1 << 21, F(1), FAKE, big, None, None, None) == -3
    assert fn(FAKE, FAKE, 4, 4, F(-1e-9), FAKE, big, None, None, None) == -4
    assert fn(FAKE, FAKE, 4, 4, F(float("nan")), FAKE, big, None, None, None) == -4
    assert fn(FAKE, FAKE, 4, 4, F(float("inf")), FAKE, big, None, None, None) == -4
    assert fn(FAKE, FAKE, 4, 4, F(1), FAKE, 512, None, None, None) == -5            # too small
    assert fn(FAKE, FAKE, 4, 4, F(1), ctypes.c_void_p((1 << 20) + 64), big, None, None, None) == -5
    assert fn(ctypes.c_void_p((1 << 20) + 2), FAKE, 4, 4, F(1), FAKE, big, None, None, None) == -7


def test_trilevel_and_norm_argument_checks(lib):
    big = 1 << 30
    tri = lib.trilevel_proj_l1infinf
    assert tri(None, FAKE, 2, 2, 2, F(1), FAKE, big, None, None, None) == -1
    assert tri(FAKE, FAKE, 2, 0, 2, F(1), FAKE, big, None, None, None) == -2
    assert tri(FAKE, FAKE, 2, 2, 2, F(-1), FAKE, big, None, None, None) == -4
    assert tri(FAKE, FAKE, 2, 2, 2, F(1), FAKE, 16, None, None, None) == -5
    assert tri(FAKE, FAKE, 1 << 14, 1 << 14, 1 << 14, F(1), FAKE, big, None, None, None) == -3
    nrm = lib.mlproj_norm_l1q
    assert nrm(None, 4, 4, 0, FAKE, big, None, None, None) == -1
    assert nrm(FAKE, 4, 4, 7, FAKE, big, None, None, None) == -6
    assert nrm(FAKE, 4, 0, 0, FAKE, big, None, None, None) == -2
    assert lib.mlproj_trace_begin(None, 4) == -1
    assert lib.mlproj_trace_end() == 0
    assert lib.bilevel_radii(0, None, 4, 4, F(1), FAKE, big, None, None) == -1
    assert lib.bilevel_radii(5, FAKE, 4, 4, F(1), FAKE, big, None, None) == -6
    assert lib.bilevel_radii(1, FAKE, 4, 4, F(-2), FAKE, big, None, None) == -4
    assert lib.bilevel_apply(0, FAKE, None, 4, 4, FAKE, big, None, None) == -1
    assert lib.bilevel_apply(2, FAKE, FAKE, 4, 4, FAKE, 64, None, None) == -5


def test_missing_library_fails_loudly(monkeypatch, tmp_path):
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "LIB_PATH", str(tmp_path / "nope.so"))
    with pytest.raises(RuntimeError, match="no CPU fallback"):
        binding.lib()


def test_multilevel_argument_checks(lib):
    big = 1 << 30
    LL, I = ctypes.c_longlong, ctypes.c_int
    dims = (LL * 3)(4, 5, 6)
    norms = (I * 2)(0, 1)
    out = ctypes.c_size_t(0)
    assert lib.mlproj_multilevel_workspace_bytes(3, dims, ctypes.byref(out)) == 0 and out.value % 256 == 0
    assert lib.mlproj_multilevel_workspace_bytes(1, dims, ctypes.byref(out)) == -2
    assert lib.mlproj_multilevel_workspace_bytes(9, dims, ctypes.byref(out)) == -2
    assert lib.mlproj_multilevel_workspace_bytes(3, None, ctypes.byref(out)) == -1
    assert lib.mlproj_multilevel_workspace_bytes(3, dims, None) == -1
    assert lib.mlproj_multilevel_workspace_bytes(3, (LL * 3)(4, 0, 6), ctypes.byref(out)) == -2
    assert lib.mlproj_multilevel_workspace_bytes(3, (LL * 3)(1 << 20, 1 << 20, 1 << 20), ctypes.byref(out)) == -3
    ml = lib.multilevel_proj
    assert ml(None, FAKE, 3, dims, norms, F(1), FAKE, big, None, None, None) == -1
    assert ml(FAKE, FAKE, 3, dims, None, F(1), FAKE, big, None, None, None) == -1
    assert ml(FAKE, FAKE, 3, dims, (I * 2)(0, 7), F(1), FAKE, big, None, None, None) == -6
    assert ml(FAKE, FAKE, 3, dims, norms, F(-1), FAKE, big, None, None, None) == -4
    assert ml(FAKE, FAKE, 3, dims, norms, F(1), FAKE, 64, None, None, None) == -5


def test_general_outer_norm_argument_checks(lib):
    big = 1 << 30
    pq = lib.bilevel_proj_pq
    assert pq(0, 0, None, FAKE, 4, 4, F(1), FAKE, big, None, None, None) == -1
    assert pq(3, 0, FAKE, FAKE, 4, 4, F(1), FAKE, big, None, None, None) == -6      # unknown outer norm
    assert pq(-1, 0, FAKE, FAKE, 4, 4, F(1), FAKE, big, None, None, None) == -6
    assert pq(1, 9, FAKE, FAKE, 4, 4, F(1), FAKE, big, None, None, None) == -6      # unknown q
    assert pq(2, 1, FAKE, FAKE, 4, 4, F(-1), FAKE, big, None, None, None) == -4
    LL, I = ctypes.c_longlong, ctypes.c_int
    dims, norms = (LL * 3)(4, 5, 6), (I * 2)(0, 1)
    assert lib.multilevel_proj_p(5, FAKE, FAKE, 3, dims, norms, F(1), FAKE, big, None, None, None) == -6
    assert lib.multilevel_proj_p(1, FAKE, FAKE, 3, dims, norms, F(1), FAKE, 64, None, None, None) == -5


def test_stored_entry_point_argument_checks(lib):
    big = 1 << 30
    st = lib.bilevel_proj_stored
    odd2 = ctypes.c_void_p((1 << 20) + 2)      # 2-byte aligned only
    odd1 = ctypes.c_void_p((1 << 20) + 1)
    assert st(3, 0, 0, FAKE, FAKE, 4, 4, F(1), FAKE, big, None, None, None, None) == -6     # unknown storage
    assert st(-1, 0, 0, FAKE, FAKE, 4, 4, F(1), FAKE, big, None, None, None, None) == -6
    for storage in (0, 1, 2):
        assert st(storage, 0, 0, None, FAKE, 4, 4, F(1), FAKE, big, None, None, None, None) == -1
        assert st(storage, 0, 0, FAKE, None, 4, 4, F(1), FAKE, big, None, None, None, None) == -1
        assert st(storage, 4, 0, FAKE, FAKE, 4, 4, F(1), FAKE, big, None, None, None, None) == -6
        assert st(storage, 0, 3, FAKE, FAKE, 4, 4, F(1), FAKE, big, None, None, None, None) == -6
        assert st(storage, 0, 0, FAKE, FAKE, 4, 0, F(1), FAKE, big, None, None, None, None) == -2
        assert st(storage, 0, 0, FAKE, FAKE, 4, 4, F(-1), FAKE, big, None, None, None, None) == -4
        assert st(storage, 0, 0, FAKE, FAKE, 4, 4, F(1), FAKE, 64, None, None, None, None) == -5
        assert st(storage, 0, 0, odd1, FAKE, 4, 4, F(1), FAKE, big, None, None, None, None) == -7
    assert st(0, 0, 0, odd2, FAKE, 4, 4, F(1), FAKE, big, None, None, None, None) == -7      # fp32 wants 4 bytes


def test_weighted_entry_point_argument_checks(lib):
    big = 1 << 30
    wt = lib.bilevel_proj_weighted
    odd2 = ctypes.c_void_p((1 << 20) + 2)
    assert wt(0, 0, FAKE, FAKE, 4, 4, F(1), None, FAKE, big, None, None, None, None) == -1     # no weights
    assert wt(0, 0, FAKE, FAKE, 4, 4, F(1), odd2, FAKE, big, None, None, None, None) == -7
    assert wt(5, 0, FAKE, FAKE, 4, 4, F(1), FAKE, FAKE, big, None, None, None, None) == -6     # unknown storage
    for storage in (0, 1, 2):
        assert wt(storage, 0, None, FAKE, 4, 4, F(1), FAKE, FAKE, big, None, None, None, None) == -1
        assert wt(storage, 0, FAKE, None, 4, 4, F(1), FAKE, FAKE, big, None, None, None, None) == -1
        assert wt(storage, 3, FAKE, FAKE, 4, 4, F(1), FAKE, FAKE, big, None, None, None, None) == -6
        assert wt(storage, 0, FAKE, FAKE, 0, 4, F(1), FAKE, FAKE, big, None, None, None, None) == -2
        assert wt(storage, 1, FAKE, FAKE, 4, 4, F(float("nan")), FAKE, FAKE, big, None, None, None, None) == -4
        assert wt(storage, 2, FAKE, FAKE, 4, 4, F(1), FAKE, FAKE, 64, None, None, None, None) == -5


def test_no_alloc_entry_point_checks_before_touching_the_gpu(lib):
    """Everything that can be refused is refused on the host, the size limit of the built-in
    scratch buffer included (this container has no GPU: a call that got past the checks would
    come back with the launch status instead)."""
    na = lib.bilevel_proj_l1inf_no_alloc
    assert na(None, FAKE, 4, 4, F(1), None, None, None) == -1
    assert na(FAKE, None, 4, 4, F(1), None, None, None) == -1
    assert na(FAKE, FAKE, 0, 4, F(1), None, None, None) == -2
    assert na(FAKE, FAKE, 4, -1, F(1), None, None, None) == -2
    assert na(FAKE, FAKE, 1 << 41, 4, F(1), None, None, None) == -3
    assert na(FAKE, FAKE, 4, 4, F(-1), None, None, None) == -4
    assert na(FAKE, FAKE, 4, 4, F(float("nan")), None, None, None) == -4
    # the limit: the workspace of the call must fit the 6 MiB buffer
    limit = 6 << 20
    assert binding.workspace_bytes("l1inf", 100000, 262144) <= limit
    assert binding.workspace_bytes("l1inf", 16384, 16384) <= limit
    assert binding.workspace_bytes("l1inf", 4, 1 << 20) > limit
    assert na(FAKE, FAKE, 4, 1 << 20, F(1), None, None, None) == -9
    assert b"scratch" in lib.mlproj_status_string(-9)


def test_search_spin_limit_knob(lib):
    default = lib.mlproj_set_search_spin_limit(0)
    assert default == 256      # a fraction of a millisecond of polling, not seconds
    assert lib.mlproj_set_search_spin_limit(64) == 0
    assert lib.mlproj_set_search_spin_limit(-1) == -2 and lib.mlproj_set_search_spin_limit((1 << 22) + 1) == -2
    assert lib.mlproj_set_search_spin_limit(default) == 64
    assert lib.mlproj_set_search_spin_limit(default) == default


def test_stripes_are_dealt_to_workgroups_by_a_permutation_that_keeps_neighbours_on_one_xcd(lib):
    """The column-stripe kernels of l1,1 take stripe f(b) in workgroup b.  f must be a permutation
    of 0..n-1 for every n (a hole would leave columns unprojected), and runs of 4 neighbouring
    stripes must sit in workgroups 8 apart, i.e. on the same XCD and consecutive in its queue."""
    f = lib.mlproj_stripe_of_workgroup
    for n in list(range(1, 300)) + [511, 512, 513, 625, 1000, 4096, 16384, 16385]:
        image = [f(b, n) for b in range(n)]
        assert sorted(image) == list(range(n)), n
        where = {s: b for b, s in enumerate(image)}
        full = n // 32 * 32
        for s0 in range(0, full, 4):
            bs = [where[s0 + i] for i in range(4)]
            assert len({b % 8 for b in bs}) == 1 and [b // 8 for b in bs] == list(range(bs[0] // 8, bs[0] // 8 + 4)), (n, s0)
        assert image[full:] == list(range(full, n))      # the ragged rest keeps its numbers
    assert f(0, 0) == -1 and f(-1, 5) == -1 and f(5, 5) == -1


def test_weighted_multilevel_argument_checks(lib):
    big = 1 << 30
    LL, I = ctypes.c_longlong, ctypes.c_int
    dims, norms = (LL * 3)(4, 5, 6), (I * 2)(0, 1)
    mw = lib.multilevel_proj_weighted
    assert mw(0, FAKE, FAKE, 3, dims, norms, F(1), None, FAKE, big, None, None, None) == -1       # no weights
    assert mw(0, FAKE, FAKE, 3, dims, norms, F(1), ctypes.c_void_p((1 << 20) + 2), FAKE, big, None, None, None) == -7
    assert mw(4, FAKE, FAKE, 3, dims, norms, F(1), FAKE, FAKE, big, None, None, None) == -6       # unknown storage
    for storage in (0, 1, 2):
        assert mw(storage, None, FAKE, 3, dims, norms, F(1), FAKE, FAKE, big, None, None, None) == -1
        assert mw(storage, FAKE, FAKE, 3, dims, None, F(1), FAKE, FAKE, big, None, None, None) == -1
        assert mw(storage, FAKE, FAKE, 3, dims, (I * 2)(0, 9), F(1), FAKE, FAKE, big, None, None, None) == -6
        assert mw(storage, FAKE, FAKE, 3, dims, norms, F(-1), FAKE, FAKE, big, None, None, None) == -4
        assert mw(storage, FAKE, FAKE, 3, dims, norms, F(1), FAKE, FAKE, 64, None, None, None) == -5


def test_batch_argument_checks(lib):
    big = 1 << 30
    bt = lib.bilevel_proj_batch
    P = binding.Problem

    def problems(*specs):
        arr = (P * len(specs))()
        for pr, (Y, X, n, m, eta, ws, nbytes) in zip(arr, specs):
            pr.Y, pr.X, pr.n, pr.m, pr.eta, pr.workspace, pr.workspace_bytes = Y, X, n, m, eta, ws, nbytes
        return arr

    good = (FAKE.value, FAKE.value, 4, 4, 1.0, FAKE.value, big)
    assert bt(0, 0, 0, 1, None, None) == -1
    assert bt(0, 0, 0, 0, problems(good), None) == -2
    assert bt(7, 0, 0, 1, problems(good), None) == -6                       # unknown storage
    assert bt(0, 0, 5, 1, problems(good), None) == -6                       # unknown variant
    assert bt(0, 9, 0, 1, problems(good), None) == -6                       # unknown outer norm
    # one bad problem anywhere rejects the whole batch before anything is enqueued
    assert bt(0, 0, 0, 3, problems(good, (None, FAKE.value, 4, 4, 1.0, FAKE.value, big), good), None) == -1
    assert bt(1, 0, 2, 2, problems(good, (FAKE.value, FAKE.value, 4, 0, 1.0, FAKE.value, big)), None) == -2
    assert bt(0, 0, 0, 2, problems(good, (FAKE.value, FAKE.value, 4, 4, -1.0, FAKE.value, big)), None) == -4
    assert bt(2, 0, 1, 2, problems(good, (FAKE.value, FAKE.value, 4, 4, 1.0, FAKE.value, 64)), None) == -5
    assert bt(0, 0, 0, 2, problems(good, (FAKE.value + 2, FAKE.value, 4, 4, 1.0, FAKE.value, big)), None) == -7
    assert ctypes.sizeof(P) == 80


def _imports(path):
    import ast
    names = set()
    for node in ast.walk(ast.parse(open(path).read())):
        if isinstance(node, ast.Import):
            names.update(a.name.split(".")[0] for a in node.names)
        elif isinstance(node, ast.ImportFrom) and node.module:
            names.add(node.module.split(".")[0])
    return names


def test_product_and_oracle_do_not_import_each_other():
    """The package (binding, workloads) never touches the oracle, the oracle never touches the
    binding, and no C++/HIP source mentions the oracle: parity claims rest on that."""
    pkg = os.path.join(ROOT, "paper_2405_02086_amd")
    for name in os.listdir(pkg):
        if name.endswith(".py"):
            assert "oracle" not in _imports(os.path.join(pkg, name)), name
    for name in os.listdir(os.path.join(ROOT, "oracle")):
        if name.endswith(".py"):
            assert "paper_2405_02086_amd" not in _imports(os.path.join(ROOT, "oracle", name)), name
    for name in os.listdir(os.path.join(pkg, "csrc")):
        assert "oracle" not in open(os.path.join(pkg, "csrc", name)).read().lower(), name
    assert "oracle" not in open(os.path.join(ROOT, "include", "mlproj.h")).read().lower()


def test_stored_trilevel_argument_checks(lib):
    big = 1 << 30
    tri = lib.trilevel_proj_stored
    assert tri(5, FAKE, FAKE, 2, 2, 2, F(1), FAKE, big, None, None, None, None) == -6
    for storage in (0, 1, 2):
        assert tri(storage, None, FAKE, 2, 2, 2, F(1), FAKE, big, None, None, None, None) == -1
        assert tri(storage, FAKE, FAKE, 2, 0, 2, F(1), FAKE, big, None, None, None, None) == -2
        assert tri(storage, FAKE, FAKE, 2, 2, 2, F(-1), FAKE, big, None, None, None, None) == -4
        assert tri(storage, FAKE, FAKE, 2, 2, 2, F(1), FAKE, 16, None, None, None, None) == -5
        assert tri(storage, ctypes.c_void_p((1 << 20) + 1), FAKE, 2, 2, 2, F(1), FAKE, big, None, None, None, None) == -7


def test_stored_multilevel_argument_checks(lib):
    big = 1 << 30
    ml = lib.multilevel_proj_stored
    dims = (ctypes.c_longlong * 3)(4, 5, 6)
    bad_dims = (ctypes.c_longlong * 3)(4, 0, 6)
    norms = (ctypes.c_int * 2)(0, 1)
    bad_norms = (ctypes.c_int * 2)(0, 7)
    assert ml(5, 0, FAKE, FAKE, 3, dims, norms, F(1), FAKE, big, None, None, None) == -6
    for storage in (0, 1, 2):
        assert ml(storage, 9, FAKE, FAKE, 3, dims, norms, F(1), FAKE, big, None, None, None) == -6
        assert ml(storage, 0, None, FAKE, 3, dims, norms, F(1), FAKE, big, None, None, None) == -1
        assert ml(storage, 0, FAKE, FAKE, 3, bad_dims, norms, F(1), FAKE, big, None, None, None) == -2
        assert ml(storage, 0, FAKE, FAKE, 3, dims, bad_norms, F(1), FAKE, big, None, None, None) == -6
        assert ml(storage, 0, FAKE, FAKE, 3, dims, norms, F(-1), FAKE, big, None, None, None) == -4
        assert ml(storage, 0, FAKE, FAKE, 3, dims, norms, F(1), FAKE, 16, None, None, None) == -5
        assert ml(storage, 0, ctypes.c_void_p((1 << 20) + 1), FAKE, 3, dims, norms, F(1), FAKE, big, None, None, None) == -7


def test_l11_sweep_knob(lib):
    """A plain process-wide integer: 0..16 accepted, the old value comes back, nothing else changes it."""
    assert lib.mlproj_set_l11_sweeps(3) == 0
    assert lib.mlproj_set_l11_sweeps(16) == 3
    assert lib.mlproj_set_l11_sweeps(17) == -2 and lib.mlproj_set_l11_sweeps(-1) == -2
    assert lib.mlproj_set_l11_sweeps(0) == 16
    assert lib.mlproj_set_l11_sweeps(0) == 0


def test_result_record_layout():
    """The record is 72 bytes with inner_finished behind inner_pending (read from the header by a C compiler)."""
    import shutil
    import subprocess
    import tempfile
    if shutil.which("gcc") is None:
        pytest.skip("gcc not installed")
    src = ('#include <stdio.h>\n#include <stddef.h>\n#include "mlproj.h"\n'
           'int main(void) { printf("%zu %zu %zu %zu\\n", sizeof(mlproj_result), offsetof(mlproj_result, inner_sweeps),'
           ' offsetof(mlproj_result, inner_pending), offsetof(mlproj_result, inner_finished)); return 0; }\n')
    with tempfile.TemporaryDirectory() as d:
        open(os.path.join(d, "t.c"), "w").write(src)
        subprocess.run(["gcc", "-I", os.path.join(ROOT, "include"), os.path.join(d, "t.c"), "-o", os.path.join(d, "t")],
                       check=True)
        out = subprocess.run([os.path.join(d, "t")], capture_output=True, text=True, check=True).stdout.split()
    assert [int(x) for x in out] == [72, 52, 56, 60]


def test_header_is_plain_c():
    """include/mlproj.h stands on its own as C99 and as C++11 (no HIP or torch types in it)."""
    import shutil
    import subprocess
    header = os.path.join(ROOT, "include", "mlproj.h")
    for cc, flags in (("gcc", ["-std=c99", "-x", "c"]), ("g++", ["-std=c++11", "-x", "c++"])):
        if shutil.which(cc) is None:
            pytest.skip(cc + " not installed")
        proc = subprocess.run([cc, "-Wall", "-Wextra", "-pedantic", "-Werror", "-fsyntax-only"] + flags + [header],
                              capture_output=True, text=True)
        assert proc.returncode == 0, proc.stderr
    text = open(header).read()
    assert "hip" not in re.sub(r"/\*.*?\*/", "", text, flags=re.S).lower() and "torch" not in text.lower()


def test_bench_refuses_more_than_one_gpu():
    """bench.py measures one GPU; asked for more it says so and exits before touching any device."""
    import subprocess
    import sys
    proc = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert proc.returncode != 0
    assert "one GPU" in (proc.stdout + proc.stderr)
