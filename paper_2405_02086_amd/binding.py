"""ctypes binding for libmlproj.so (declared in include/mlproj.h).

Argument marshalling only: every step of the projection runs in the HIP kernels.
PyTorch is used for device memory and streams.  There is no CPU fallback: if the
shared library has not been built, every entry point raises.
"""
import ctypes
import os
import struct
import subprocess

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmlproj.so")
SRC_PATH = os.path.join(_HERE, "csrc", "mlproj.hip")

L1INF, L11, L12, L1INFINF = 0, 1, 2, 3
_VARIANTS = {"l1inf": L1INF, "l11": L11, "l12": L12, "tri": L1INFINF}

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-shared", "-fPIC",
    # keep the compiler from forming packed-fp32 VALU ops
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
]


class MlprojError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        msg = lib().mlproj_status_string(status).decode() if _lib is not None else "?"
        super().__init__(f"{where}: {msg} (status {status})")


def build(verbose=False):
    """Compile csrc/mlproj.hip (one translation unit that includes csrc/*.h) for gfx950 into
    libmlproj.so next to this file."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc] + HIPCC_FLAGS + ["-o", LIB_PATH, SRC_PATH]
    proc = subprocess.run(cmd, capture_output=True, text=True)
    if verbose or proc.returncode != 0:
        print(" ".join(cmd))
        print(proc.stdout + proc.stderr)
    if proc.returncode != 0:
        raise RuntimeError("hipcc failed building libmlproj.so")
    global _lib
    _lib = None
    return LIB_PATH


_lib = None


def lib():
    """The loaded C library; raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(
            f"{LIB_PATH} is missing: build it first (python -c 'import __graft_entry__ as g; g.build()'). "
            "There is no CPU fallback.")
    L = ctypes.CDLL(LIB_PATH)
    c_ll, c_sz, c_vp, c_f, c_i = ctypes.c_longlong, ctypes.c_size_t, ctypes.c_void_p, ctypes.c_float, ctypes.c_int
    L.mlproj_version.restype = c_i
    L.mlproj_version.argtypes = []
    L.mlproj_status_string.restype = ctypes.c_char_p
    L.mlproj_status_string.argtypes = [c_i]
    L.mlproj_workspace_bytes.restype = c_i
    L.mlproj_workspace_bytes.argtypes = [c_i, c_ll, c_ll, c_ll, ctypes.POINTER(c_sz)]
    L.mlproj_trace_begin.restype = c_i
    L.mlproj_trace_begin.argtypes = [ctypes.POINTER(c_vp), c_i]
    L.mlproj_trace_end.restype = c_i
    L.mlproj_trace_end.argtypes = []
    L.mlproj_set_l11_sweeps.restype = c_i
    L.mlproj_set_l11_sweeps.argtypes = [c_i]
    L.mlproj_set_search_spin_limit.restype = c_i
    L.mlproj_set_search_spin_limit.argtypes = [c_i]
    L.mlproj_stripe_of_workgroup.restype = c_i
    L.mlproj_stripe_of_workgroup.argtypes = [c_ll, c_ll]
    L.mlproj_norm_l1q.restype = c_i
    L.mlproj_norm_l1q.argtypes = [c_vp, c_ll, c_ll, c_i, c_vp, c_sz, c_vp, c_vp, c_vp]
    for name in ("bilevel_proj_l1inf", "bilevel_proj_l11", "bilevel_proj_l12"):
        fn = getattr(L, name)
        fn.restype = c_i
        fn.argtypes = [c_vp, c_vp, c_ll, c_ll, c_f, c_vp, c_sz, c_vp, c_vp, c_vp]
    L.bilevel_proj_l1inf_no_alloc.restype = c_i
    L.bilevel_proj_l1inf_no_alloc.argtypes = [c_vp, c_vp, c_ll, c_ll, c_f, c_vp, c_vp, c_vp]
    L.bilevel_radii.restype = c_i
    L.bilevel_radii.argtypes = [c_i, c_vp, c_ll, c_ll, c_f, c_vp, c_sz, c_vp, c_vp]
    L.bilevel_apply.restype = c_i
    L.bilevel_apply.argtypes = [c_i, c_vp, c_vp, c_ll, c_ll, c_vp, c_sz, c_vp, c_vp]
    L.mlproj_multilevel_workspace_bytes.restype = c_i
    L.mlproj_multilevel_workspace_bytes.argtypes = [c_i, ctypes.POINTER(c_ll), ctypes.POINTER(c_sz)]
    L.multilevel_proj.restype = c_i
    L.multilevel_proj.argtypes = [c_vp, c_vp, c_i, ctypes.POINTER(c_ll), ctypes.POINTER(c_i), c_f, c_vp, c_sz,
                                  c_vp, c_vp, c_vp]
    L.multilevel_proj_p.restype = c_i
    L.multilevel_proj_p.argtypes = [c_i, c_vp, c_vp, c_i, ctypes.POINTER(c_ll), ctypes.POINTER(c_i), c_f, c_vp,
                                    c_sz, c_vp, c_vp, c_vp]
    L.multilevel_proj_stored.restype = c_i
    L.multilevel_proj_stored.argtypes = [c_i, c_i, c_vp, c_vp, c_i, ctypes.POINTER(c_ll), ctypes.POINTER(c_i), c_f,
                                         c_vp, c_sz, c_vp, c_vp, c_vp]
    L.bilevel_proj_pq.restype = c_i
    L.bilevel_proj_pq.argtypes = [c_i, c_i, c_vp, c_vp, c_ll, c_ll, c_f, c_vp, c_sz, c_vp, c_vp, c_vp]
    L.bilevel_proj_stored.restype = c_i
    L.bilevel_proj_stored.argtypes = [c_i, c_i, c_i, c_vp, c_vp, c_ll, c_ll, c_f, c_vp, c_sz, c_vp, c_vp, c_vp, c_vp]
    L.bilevel_proj_batch.restype = c_i
    L.bilevel_proj_batch.argtypes = [c_i, c_i, c_i, c_i, ctypes.POINTER(Problem), c_vp]
    L.multilevel_proj_weighted.restype = c_i
    L.multilevel_proj_weighted.argtypes = [c_i, c_vp, c_vp, c_i, ctypes.POINTER(c_ll), ctypes.POINTER(c_i), c_f, c_vp,
                                           c_vp, c_sz, c_vp, c_vp, c_vp]
    L.bilevel_proj_weighted.restype = c_i
    L.bilevel_proj_weighted.argtypes = [c_i, c_i, c_vp, c_vp, c_ll, c_ll, c_f, c_vp, c_vp, c_sz, c_vp, c_vp, c_vp, c_vp]
    L.trilevel_proj_stored.restype = c_i
    L.trilevel_proj_stored.argtypes = [c_i, c_vp, c_vp, c_ll, c_ll, c_ll, c_f, c_vp, c_sz, c_vp, c_vp, c_vp, c_vp]
    L.trilevel_proj_l1infinf.restype = c_i
    L.trilevel_proj_l1infinf.argtypes = [c_vp, c_vp, c_ll, c_ll, c_ll, c_f, c_vp, c_sz, c_vp, c_vp, c_vp]
    _lib = L
    return L


class Problem(ctypes.Structure):
    """mlproj_problem of include/mlproj.h."""
    _fields_ = [("Y", ctypes.c_void_p), ("X", ctypes.c_void_p), ("n", ctypes.c_longlong), ("m", ctypes.c_longlong),
                ("eta", ctypes.c_float), ("workspace", ctypes.c_void_p), ("workspace_bytes", ctypes.c_size_t),
                ("v_out", ctypes.c_void_p), ("u_out", ctypes.c_void_p), ("mask_out", ctypes.c_void_p)]


EXPORTS = (
    "mlproj_version", "mlproj_status_string", "mlproj_workspace_bytes", "mlproj_trace_begin", "mlproj_trace_end",
    "mlproj_norm_l1q", "bilevel_proj_l1inf", "bilevel_proj_l11", "bilevel_proj_l12",
    "trilevel_proj_l1infinf", "bilevel_radii", "bilevel_apply",
    "mlproj_multilevel_workspace_bytes", "multilevel_proj", "multilevel_proj_p", "bilevel_proj_pq",
    "bilevel_proj_stored", "bilevel_proj_batch", "trilevel_proj_stored", "mlproj_set_l11_sweeps",
    "multilevel_proj_stored", "bilevel_proj_weighted", "multilevel_proj_weighted", "mlproj_set_search_spin_limit",
    "bilevel_proj_l1inf_no_alloc", "mlproj_stripe_of_workgroup",
)


def _check(status, where):
    if status != 0:
        raise MlprojError(status, where)


def set_search_spin_limit(polls):
    """Polls after which the several-workgroup search gives up (0 = at once); returns the old value."""
    before = lib().mlproj_set_search_spin_limit(int(polls))
    if before < 0:
        raise MlprojError(int(before), "mlproj_set_search_spin_limit")
    return int(before)


def set_l11_sweeps(sweeps):
    """Lock-step passes an l1,1 call enqueues before its finishing pass (0 = default); returns the old value."""
    before = lib().mlproj_set_l11_sweeps(int(sweeps))
    if before < 0:
        raise MlprojError(before, "mlproj_set_l11_sweeps")
    return before


def workspace_bytes(variant, d0, d1, d2=1):
    out = ctypes.c_size_t(0)
    v = _VARIANTS.get(variant, variant)
    _check(lib().mlproj_workspace_bytes(v, d0, d1, d2, ctypes.byref(out)), "mlproj_workspace_bytes")
    return out.value


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream(stream):
    import torch
    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


class Workspace:
    """Device scratch for one call at a time; needs no initialisation."""

    def __init__(self, nbytes, device="cuda", stream=None):
        import torch
        nbytes = (int(nbytes) + 255) // 256 * 256
        self.buf = torch.empty(nbytes, dtype=torch.uint8, device=device)
        assert self.buf.data_ptr() % 256 == 0
        self.nbytes = nbytes

    @classmethod
    def for_call(cls, variant, d0, d1, d2=1, **kw):
        return cls(workspace_bytes(variant, d0, d1, d2), **kw)

    def result(self):
        """Synchronise and decode the mlproj_result record at the head of the workspace."""
        raw = bytes(self.buf[:64].cpu().numpy().tobytes())
        tau, norm, vmax, scale, cap, n_active, inside, iters, sweeps, pending, finished = struct.unpack_from("<dddddIIIIII", raw)
        return {"tau": tau, "norm": norm, "vmax": vmax, "scale": scale, "cap": cap, "n_active": n_active,
                "inside_ball": bool(inside), "search_iters": iters,
                "inner_sweeps": sweeps, "inner_pending": pending, "inner_finished": finished}


def _prep(Y, X):
    import torch
    assert Y.is_cuda and Y.dtype == torch.float32 and Y.is_contiguous(), "Y: contiguous fp32 device tensor"
    if X is None:
        X = torch.empty_like(Y)
    assert X.is_cuda and X.dtype == torch.float32 and X.is_contiguous() and X.shape == Y.shape
    return X


def _bilevel(name, variant, Y, eta, X, workspace, v_out, u_out, stream):
    assert Y.dim() == 2
    n, m = Y.shape
    X = _prep(Y, X)
    if workspace is None:
        workspace = Workspace.for_call(variant, n, m, device=Y.device, stream=stream)
    st = getattr(lib(), name)(_ptr(Y), _ptr(X), n, m, ctypes.c_float(eta), _ptr(workspace.buf),
                              workspace.nbytes, _ptr(v_out), _ptr(u_out), _stream(stream))
    _check(st, name)
    return X


def bilevel_proj_l1inf(Y, eta, X=None, workspace=None, v_out=None, u_out=None, stream=None):
    return _bilevel("bilevel_proj_l1inf", L1INF, Y, eta, X, workspace, v_out, u_out, stream)


def bilevel_proj_l1inf_no_alloc(Y, eta, X, v_out=None, u_out=None, stream=None):
    """bilevel_proj_l1inf on the library's built-in scratch buffer: the call allocates nothing,
    so X is the caller's (and there is no workspace to pass)."""
    assert Y.dim() == 2 and X is not None
    n, m = Y.shape
    assert _prep(Y, X) is X
    st = lib().bilevel_proj_l1inf_no_alloc(_ptr(Y), _ptr(X), n, m, ctypes.c_float(eta), _ptr(v_out), _ptr(u_out),
                                           _stream(stream))
    _check(st, "bilevel_proj_l1inf_no_alloc")
    return X


def bilevel_proj_l11(Y, eta, X=None, workspace=None, v_out=None, u_out=None, stream=None):
    return _bilevel("bilevel_proj_l11", L11, Y, eta, X, workspace, v_out, u_out, stream)


def bilevel_proj_l12(Y, eta, X=None, workspace=None, v_out=None, u_out=None, stream=None):
    return _bilevel("bilevel_proj_l12", L12, Y, eta, X, workspace, v_out, u_out, stream)


def bilevel_radii(variant, Y, eta, workspace, v_out=None, stream=None):
    n, m = Y.shape
    v = _VARIANTS.get(variant, variant)
    _check(lib().bilevel_radii(v, _ptr(Y), n, m, ctypes.c_float(eta), _ptr(workspace.buf), workspace.nbytes,
                               _ptr(v_out), _stream(stream)), "bilevel_radii")


def bilevel_apply(variant, Y, X, workspace, u_out=None, stream=None):
    n, m = Y.shape
    v = _VARIANTS.get(variant, variant)
    _check(lib().bilevel_apply(v, _ptr(Y), _ptr(X), n, m, _ptr(workspace.buf), workspace.nbytes,
                               _ptr(u_out), _stream(stream)), "bilevel_apply")
    return X


def trilevel_proj_l1infinf(Y, eta, X=None, workspace=None, v_out=None, u_out=None, stream=None):
    assert Y.dim() == 3
    d0, d1, d2 = Y.shape
    X = _prep(Y, X)
    if workspace is None:
        workspace = Workspace.for_call(L1INFINF, d0, d1, d2, device=Y.device, stream=stream)
    st = lib().trilevel_proj_l1infinf(_ptr(Y), _ptr(X), d0, d1, d2, ctypes.c_float(eta),
                                      _ptr(workspace.buf), workspace.nbytes, _ptr(v_out), _ptr(u_out),
                                      _stream(stream))
    _check(st, "trilevel_proj_l1infinf")
    return X


OUTER_L1, OUTER_L2, OUTER_LINF = 0, 1, 2
_OUTERS = {1: OUTER_L1, 2: OUTER_L2, "inf": OUTER_LINF}


def bilevel_proj_pq(p, q, Y, eta, X=None, workspace=None, v_out=None, u_out=None, stream=None):
    """BP^{p,q}: p in {1, 2, "inf"} (outer), q in {"inf", 1, 2} (per column)."""
    assert Y.dim() == 2
    n, m = Y.shape
    X = _prep(Y, X)
    variant = {"inf": L1INF, 1: L11, 2: L12}[q]
    if workspace is None:
        workspace = Workspace.for_call(variant, n, m, device=Y.device, stream=stream)
    st = lib().bilevel_proj_pq(_OUTERS[p], variant, _ptr(Y), _ptr(X), n, m, ctypes.c_float(eta),
                               _ptr(workspace.buf), workspace.nbytes, _ptr(v_out), _ptr(u_out), _stream(stream))
    _check(st, "bilevel_proj_pq")
    return X


STORE_F32, STORE_BF16, STORE_F16 = 0, 1, 2


def bilevel_proj_stored(Y, eta, q, p=1, X=None, workspace=None, v_out=None, u_out=None, mask_out=None,
                        stream=None):
    """BP^{p,q} on a contiguous fp32, bf16 or fp16 device matrix (X has Y's dtype); mask_out is an
    optional uint8 tensor of m entries that receives 1 for every kept column."""
    import torch
    storages = {torch.float32: STORE_F32, torch.bfloat16: STORE_BF16, torch.float16: STORE_F16}
    assert Y.is_cuda and Y.dim() == 2 and Y.is_contiguous() and Y.dtype in storages
    n, m = Y.shape
    if X is None:
        X = torch.empty_like(Y)
    assert X.is_cuda and X.dtype == Y.dtype and X.is_contiguous() and X.shape == Y.shape
    assert mask_out is None or (mask_out.dtype == torch.uint8 and mask_out.numel() >= m)
    variant = {"inf": L1INF, 1: L11, 2: L12}[q]
    if workspace is None:
        workspace = Workspace.for_call(variant, n, m, device=Y.device, stream=stream)
    st = lib().bilevel_proj_stored(storages[Y.dtype], _OUTERS[p], variant, _ptr(Y), _ptr(X), n, m,
                                   ctypes.c_float(eta), _ptr(workspace.buf), workspace.nbytes, _ptr(v_out),
                                   _ptr(u_out), _ptr(mask_out), _stream(stream))
    _check(st, "bilevel_proj_stored")
    return X


def bilevel_proj_weighted(Y, eta, q, weights, X=None, workspace=None, v_out=None, u_out=None, mask_out=None,
                          stream=None):
    """BP^{p,q} with the weighted l1 ball {u : sum_j w_j |u_j| <= eta} as outer norm, on a contiguous
    fp32, bf16 or fp16 device matrix; weights is an fp32 device tensor of m positive entries."""
    import torch
    storages = {torch.float32: STORE_F32, torch.bfloat16: STORE_BF16, torch.float16: STORE_F16}
    assert Y.is_cuda and Y.dim() == 2 and Y.is_contiguous() and Y.dtype in storages
    n, m = Y.shape
    assert weights.is_cuda and weights.dtype == torch.float32 and weights.is_contiguous() and weights.numel() == m
    if X is None:
        X = torch.empty_like(Y)
    assert X.is_cuda and X.dtype == Y.dtype and X.is_contiguous() and X.shape == Y.shape
    assert mask_out is None or (mask_out.dtype == torch.uint8 and mask_out.numel() >= m)
    variant = {"inf": L1INF, 1: L11, 2: L12}[q]
    if workspace is None:
        workspace = Workspace.for_call(variant, n, m, device=Y.device, stream=stream)
    st = lib().bilevel_proj_weighted(storages[Y.dtype], variant, _ptr(Y), _ptr(X), n, m, ctypes.c_float(eta),
                                     _ptr(weights), _ptr(workspace.buf), workspace.nbytes, _ptr(v_out),
                                     _ptr(u_out), _ptr(mask_out), _stream(stream))
    _check(st, "bilevel_proj_weighted")
    return X


def trilevel_proj_stored(Y, eta, X=None, workspace=None, v_out=None, u_out=None, mask_out=None, stream=None):
    """TP^{1,inf,inf} on a contiguous fp32, bf16 or fp16 device tensor of three axes."""
    import torch
    storages = {torch.float32: STORE_F32, torch.bfloat16: STORE_BF16, torch.float16: STORE_F16}
    assert Y.is_cuda and Y.dim() == 3 and Y.is_contiguous() and Y.dtype in storages
    d0, d1, d2 = Y.shape
    if X is None:
        X = torch.empty_like(Y)
    assert X.is_cuda and X.dtype == Y.dtype and X.is_contiguous() and X.shape == Y.shape
    if workspace is None:
        workspace = Workspace.for_call("tri", d0, d1, d2, device=Y.device, stream=stream)
    st = lib().trilevel_proj_stored(storages[Y.dtype], _ptr(Y), _ptr(X), d0, d1, d2, ctypes.c_float(eta),
                                    _ptr(workspace.buf), workspace.nbytes, _ptr(v_out), _ptr(u_out),
                                    _ptr(mask_out), _stream(stream))
    _check(st, "trilevel_proj_stored")
    return X


class PreparedBatch:
    """The argument block of a bilevel_proj_batch call, marshalled once: a training loop projects
    the same buffers after every step, and filling the block costs more host time than the
    call.  Calling the object enqueues the batch; `.X` lists the output tensors.  It keeps every
    tensor it points to alive."""

    def __init__(self, Ys, etas, q, p=1, Xs=None, workspaces=None, v_outs=None, u_outs=None, mask_outs=None):
        import torch
        storages = {torch.float32: STORE_F32, torch.bfloat16: STORE_BF16, torch.float16: STORE_F16}
        count = len(Ys)
        assert count > 0 and len(etas) == count
        self.variant = {"inf": L1INF, 1: L11, 2: L12}[q]
        self.outer = _OUTERS[p]
        self.count = count
        pick = lambda lst, i: None if lst is None else lst[i]
        self.problems = (Problem * count)()
        self.X = []
        self.keep = [Ys, v_outs, u_outs, mask_outs]   # every buffer the block points to
        for i, Y in enumerate(Ys):
            assert Y.is_cuda and Y.dim() == 2 and Y.is_contiguous() and Y.dtype == Ys[0].dtype and Y.dtype in storages
            n, m = Y.shape
            X = pick(Xs, i)
            if X is None:
                X = torch.empty_like(Y)
            assert X.is_cuda and X.dtype == Y.dtype and X.is_contiguous() and X.shape == Y.shape
            # every problem needs a workspace of its own
            ws = pick(workspaces, i) or Workspace.for_call(self.variant, n, m, device=Y.device)
            self.keep.append(ws)
            self.X.append(X)
            pr = self.problems[i]
            pr.Y, pr.X, pr.n, pr.m, pr.eta = Y.data_ptr(), X.data_ptr(), n, m, float(etas[i])
            pr.workspace, pr.workspace_bytes = ws.buf.data_ptr(), ws.nbytes
            for field, lst in (("v_out", v_outs), ("u_out", u_outs), ("mask_out", mask_outs)):
                t = pick(lst, i)
                setattr(pr, field, None if t is None else t.data_ptr())
        self.storage = storages[Ys[0].dtype]

    def __call__(self, stream=None):
        st = lib().bilevel_proj_batch(self.storage, self.outer, self.variant, self.count, self.problems,
                                      _stream(stream))
        _check(st, "bilevel_proj_batch")
        return self.X


def bilevel_proj_batch(Ys, etas, q, p=1, Xs=None, workspaces=None, v_outs=None, u_outs=None, mask_outs=None,
                       stream=None):
    """Independent BP^{p,q} projections of the matrices in Ys (same dtype, any shapes) with radii
    etas, through bilevel_proj_batch; returns the list of X tensors.  Optional lists give the
    per-problem X, workspace, v_out, u_out and mask_out."""
    return PreparedBatch(Ys, etas, q, p=p, Xs=Xs, workspaces=workspaces, v_outs=v_outs, u_outs=u_outs,
                         mask_outs=mask_outs)(stream)


NORM_INF, NORM_L1, NORM_L2 = 0, 1, 2
_NORMS = {"inf": NORM_INF, 1: NORM_L1, 2: NORM_L2}


def multilevel_workspace_bytes(shape):
    dims = (ctypes.c_longlong * len(shape))(*shape)
    out = ctypes.c_size_t(0)
    _check(lib().mlproj_multilevel_workspace_bytes(len(shape), dims, ctypes.byref(out)),
           "mlproj_multilevel_workspace_bytes")
    return out.value


def multilevel_proj(Y, norms, eta, X=None, workspace=None, v_out=None, u_out=None, stream=None, p=1):
    """norms: inner norms, innermost (last axis) first, each "inf", 1 or 2; groups on axis 0;
    p: outermost norm (1, 2 or "inf")."""
    X = _prep(Y, X)
    shape = tuple(Y.shape)
    assert len(norms) == len(shape) - 1
    if workspace is None:
        workspace = Workspace(multilevel_workspace_bytes(shape), device=Y.device)
    dims = (ctypes.c_longlong * len(shape))(*shape)
    nrm = (ctypes.c_int * len(norms))(*[_NORMS[q] for q in norms])
    if p == 1:
        st = lib().multilevel_proj(_ptr(Y), _ptr(X), len(shape), dims, nrm, ctypes.c_float(eta),
                                   _ptr(workspace.buf), workspace.nbytes, _ptr(v_out), _ptr(u_out), _stream(stream))
    else:
        st = lib().multilevel_proj_p(_OUTERS[p], _ptr(Y), _ptr(X), len(shape), dims, nrm, ctypes.c_float(eta),
                                     _ptr(workspace.buf), workspace.nbytes, _ptr(v_out), _ptr(u_out), _stream(stream))
    _check(st, "multilevel_proj")
    return X


def multilevel_proj_stored(Y, norms, eta, p=1, X=None, workspace=None, v_out=None, u_out=None, stream=None):
    """multilevel_proj on a contiguous fp32, bf16 or fp16 device tensor (X has Y's dtype)."""
    import torch
    storages = {torch.float32: STORE_F32, torch.bfloat16: STORE_BF16, torch.float16: STORE_F16}
    assert Y.is_cuda and Y.is_contiguous() and Y.dtype in storages
    if X is None:
        X = torch.empty_like(Y)
    assert X.is_cuda and X.dtype == Y.dtype and X.is_contiguous() and X.shape == Y.shape
    shape = tuple(Y.shape)
    assert len(norms) == len(shape) - 1
    if workspace is None:
        workspace = Workspace(multilevel_workspace_bytes(shape), device=Y.device)
    dims = (ctypes.c_longlong * len(shape))(*shape)
    nrm = (ctypes.c_int * len(norms))(*[_NORMS[q] for q in norms])
    st = lib().multilevel_proj_stored(storages[Y.dtype], _OUTERS[p], _ptr(Y), _ptr(X), len(shape), dims, nrm,
                                      ctypes.c_float(eta), _ptr(workspace.buf), workspace.nbytes, _ptr(v_out),
                                      _ptr(u_out), _stream(stream))
    _check(st, "multilevel_proj_stored")
    return X


def multilevel_proj_weighted(Y, norms, eta, weights, X=None, workspace=None, v_out=None, u_out=None, stream=None):
    """multilevel_proj_stored with the weighted l1 ball {u : sum_a w_a |u_a| <= eta} as outermost norm;
    weights is an fp32 device tensor with one positive entry per group of axis 0."""
    import torch
    storages = {torch.float32: STORE_F32, torch.bfloat16: STORE_BF16, torch.float16: STORE_F16}
    assert Y.is_cuda and Y.is_contiguous() and Y.dtype in storages
    shape = tuple(Y.shape)
    assert weights.is_cuda and weights.dtype == torch.float32 and weights.is_contiguous() and weights.numel() == shape[0]
    if X is None:
        X = torch.empty_like(Y)
    assert X.is_cuda and X.dtype == Y.dtype and X.is_contiguous() and X.shape == Y.shape
    assert len(norms) == len(shape) - 1
    if workspace is None:
        workspace = Workspace(multilevel_workspace_bytes(shape), device=Y.device)
    dims = (ctypes.c_longlong * len(shape))(*shape)
    nrm = (ctypes.c_int * len(norms))(*[_NORMS[q] for q in norms])
    st = lib().multilevel_proj_weighted(storages[Y.dtype], _ptr(Y), _ptr(X), len(shape), dims, nrm,
                                        ctypes.c_float(eta), _ptr(weights), _ptr(workspace.buf), workspace.nbytes,
                                        _ptr(v_out), _ptr(u_out), _stream(stream))
    _check(st, "multilevel_proj_weighted")
    return X


def norm_l1q(Y, variant, workspace=None, v_out=None, stream=None):
    """||Y||_{1,q} computed on the device; returns a python float (synchronises)."""
    import torch
    assert Y.dim() == 2 and Y.is_cuda and Y.dtype == torch.float32 and Y.is_contiguous()
    n, m = Y.shape
    v = _VARIANTS.get(variant, variant)
    if workspace is None:
        workspace = Workspace.for_call(v, n, m, device=Y.device, stream=stream)
    out = torch.empty(1, dtype=torch.float64, device=Y.device)
    st = lib().mlproj_norm_l1q(_ptr(Y), n, m, v, _ptr(workspace.buf), workspace.nbytes, _ptr(out),
                               _ptr(v_out), _stream(stream))
    _check(st, "mlproj_norm_l1q")
    return float(out.item())


class KernelTrace:
    """Times the kernels inside library calls with HIP events (mlproj_trace_begin / _end).

    with KernelTrace(capacity) as tr: ...calls...; tr.durations_ms() then gives the time
    between consecutive events, i.e. one entry per kernel launched, in launch order.
    """

    def __init__(self, capacity):
        self.hip = ctypes.CDLL("libamdhip64.so")
        self.capacity = capacity
        self.events = (ctypes.c_void_p * capacity)()
        for i in range(capacity):
            ev = ctypes.c_void_p()
            assert self.hip.hipEventCreate(ctypes.byref(ev)) == 0
            self.events[i] = ev
        self.count = 0

    def __enter__(self):
        _check(lib().mlproj_trace_begin(self.events, self.capacity), "mlproj_trace_begin")
        return self

    def __exit__(self, *exc):
        self.count = lib().mlproj_trace_end()
        return False

    def durations_ms(self):
        import torch
        torch.cuda.synchronize()
        out = []
        for i in range(self.count - 1):
            ms = ctypes.c_float()
            assert self.hip.hipEventElapsedTime(ctypes.byref(ms), ctypes.c_void_p(self.events[i]),
                                                ctypes.c_void_p(self.events[i + 1])) == 0
            out.append(ms.value)
        return out

    def close(self):
        for i in range(self.capacity):
            self.hip.hipEventDestroy(ctypes.c_void_p(self.events[i]))
