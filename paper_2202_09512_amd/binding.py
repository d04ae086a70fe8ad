"""ctypes marshalling for libnnrescal.so.  No arithmetic of the method lives here."""
import ctypes as C
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB = None

EXPORTED_SYMBOLS = [
    "nnrescal_init", "nnrescal_mu_step", "nnrescal_fit", "nnrescal_fit_until", "nnrescal_start_nndsvd", "nnrescal_objective", "nnrescal_get_factors",
    "nnrescal_set_factors", "nnrescal_products", "nnrescal_perturb", "nnrescal_cluster", "nnrescal_select_k", "nnrescal_destroy",
    "nnrescal_last_error", "nnrescal_profile", "nnrescal_mu_step_static", "nnrescal_gather_form",
]
PROF_CLASSES = 6
PROF_NAMES = ["gram_mul", "matrix_mul", "matrix_mul_sparse", "elementwise", "matrix_mul_tail", "a_rule"]


class NNRescalError(RuntimeError):
    def __init__(self, status, msg):
        super().__init__(f"nnrescal status {status}: {msg}")
        self.status = status


class _Tensor(C.Structure):
    _fields_ = [("format", C.c_int32), ("n", C.c_int64), ("m", C.c_int32), ("dense", C.c_void_p),
                ("csr_rowptr", C.c_void_p), ("csr_col", C.c_void_p), ("csr_val", C.c_void_p),
                ("csr_slice_off", C.POINTER(C.c_int64)), ("csc_colptr", C.c_void_p), ("csc_row", C.c_void_p),
                ("csc_val", C.c_void_p), ("csc_slice_off", C.POINTER(C.c_int64))]


_ALLOC_FN = C.CFUNCTYPE(C.c_void_p, C.c_size_t, C.c_void_p)
_DEALLOC_FN = C.CFUNCTYPE(None, C.c_void_p, C.c_void_p)


class _Params(C.Structure):
    _fields_ = [("k", C.c_int32), ("q", C.c_int32), ("delta", C.c_float), ("eps_div", C.c_float),
                ("seed", C.c_uint64), ("stream", C.c_void_p), ("alloc", _ALLOC_FN), ("dealloc", _DEALLOC_FN),
                ("alloc_ctx", C.c_void_p), ("A0", C.c_void_p), ("R0", C.c_void_p), ("start", C.c_int32),
                ("start_svd_iters", C.c_int32), ("start_r_iters", C.c_int32), ("start_floor_rel", C.c_float),
                ("no_fused_small", C.c_int32), ("no_csc_build", C.c_int32),
                ("no_rank_packing", C.c_int32), ("check_input", C.c_int32), ("deterministic", C.c_int32), ("handover_spin_limit", C.c_int32),
                ("gather_form", C.c_int32)]


def lib_path():
    return os.path.join(_HERE, "libnnrescal.so")


def load():
    """Load the shared library; raises if it has not been built (python -m paper_2202_09512_amd.build)."""
    global _LIB
    if _LIB is not None:
        return _LIB
    path = lib_path()
    if not os.path.exists(path):
        raise ImportError(f"{path} is missing: build it with `python -m paper_2202_09512_amd.build`")
    lib = C.CDLL(path)
    P = C.POINTER
    lib.nnrescal_init.argtypes = [P(C.c_void_p), P(_Tensor), P(_Params)]
    lib.nnrescal_mu_step.argtypes = [C.c_void_p]
    lib.nnrescal_fit.argtypes = [C.c_void_p, C.c_int32, P(C.c_double)]
    lib.nnrescal_fit_until.argtypes = [C.c_void_p, C.c_int32, C.c_double, C.c_int32, P(C.c_int32), P(C.c_double)]
    lib.nnrescal_start_nndsvd.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_float, P(C.c_float)]
    lib.nnrescal_mu_step_static.argtypes = [P(_Tensor), P(_Params), C.c_void_p, C.c_void_p, C.c_void_p]
    lib.nnrescal_objective.argtypes = [C.c_void_p, P(C.c_double), P(C.c_double)]
    lib.nnrescal_get_factors.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32]
    lib.nnrescal_set_factors.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p]
    lib.nnrescal_products.argtypes = [C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p]
    lib.nnrescal_perturb.argtypes = [P(_Tensor), C.c_int32, C.c_float, C.c_uint64, C.c_int32, C.c_void_p, C.c_void_p]
    lib.nnrescal_cluster.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_int32, C.c_int32, C.c_int32, P(_Params),
                                     P(C.c_int32), C.c_void_p, C.c_void_p, P(C.c_float), P(C.c_float), P(C.c_int32)]
    lib.nnrescal_select_k.argtypes = [P(_Tensor), P(_Params), C.c_int32, C.c_int32, C.c_int32, C.c_int32,
                                      P(C.c_float), P(C.c_float), P(C.c_float), P(C.c_int32), C.c_void_p, C.c_void_p]
    lib.nnrescal_destroy.argtypes = [C.c_void_p]
    lib.nnrescal_gather_form.argtypes = [C.c_void_p]
    lib.nnrescal_gather_form.restype = C.c_int32
    lib.nnrescal_destroy.restype = None
    lib.nnrescal_last_error.argtypes = [C.c_void_p]
    lib.nnrescal_last_error.restype = C.c_char_p
    lib.nnrescal_profile.argtypes = [C.c_void_p, C.c_int32, P(C.c_double), P(C.c_int64)]
    for name in EXPORTED_SYMBOLS:
        if name not in ("nnrescal_destroy", "nnrescal_last_error", "nnrescal_gather_form"):
            getattr(lib, name).restype = C.c_int
    _LIB = lib
    return lib


# ------------------------------------------------------------------------------- device memory from torch
class _TorchAllocator:
    """alloc/dealloc callbacks backed by torch's caching allocator (uint8 tensors kept alive by pointer)."""

    def __init__(self, device):
        import torch
        self._torch = torch
        self.device = device
        self.live = {}
        self.fail_after = None          # tests: make the n-th next allocation return NULL
        self.alloc_cb = _ALLOC_FN(self._alloc)
        self.dealloc_cb = _DEALLOC_FN(self._dealloc)

    def _alloc(self, nbytes, _ctx):
        if self.fail_after is not None:
            if self.fail_after == 0:
                return None
            self.fail_after -= 1
        try:
            t = self._torch.empty(int(nbytes), dtype=self._torch.uint8, device=self.device)
        except Exception:
            return None
        self.live[t.data_ptr()] = t
        return t.data_ptr()

    def _dealloc(self, ptr, _ctx):
        self.live.pop(ptr, None)


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def _dev_f32(t, what):
    """The library reads plain row-major arrays: hand it a contiguous float32 device tensor (copying if needed)."""
    import torch
    if t is None:
        return None
    if not t.is_cuda or t.dtype != torch.float32:
        raise TypeError(f"{what} must be a float32 tensor on the GPU")
    return t if t.is_contiguous() else t.contiguous()


class DenseX:
    """Dense tensor X[m][n][n], float32, on the GPU (borrowed by the library)."""

    def __init__(self, X):
        import torch
        assert X.is_cuda and X.dtype == torch.float32 and X.dim() == 3 and X.shape[1] == X.shape[2] and X.is_contiguous()
        self.X = X
        self.m, self.n = int(X.shape[0]), int(X.shape[1])
        self.device = X.device
        self.c = _Tensor(format=0, n=self.n, m=self.m, dense=X.data_ptr())


class SparseX:
    """CSR (+ optional CSC) tensor; device arrays as torch tensors, slice offsets as host int64 lists.  csr_val (and
    csc_val) None: a binary tensor, every stored entry is 1."""

    def __init__(self, n, m, csr_rowptr, csr_col, csr_val, csr_slice_off, csc_colptr=None, csc_row=None,
                 csc_val=None, csc_slice_off=None):
        self.n, self.m = int(n), int(m)
        self.keep = [csr_rowptr, csr_col, csr_val, csc_colptr, csc_row, csc_val]
        self.device = csr_col.device
        self._off1 = (C.c_int64 * (m + 1))(*[int(v) for v in csr_slice_off])
        has_csc = csc_colptr is not None
        self._off2 = (C.c_int64 * (m + 1))(*[int(v) for v in (csc_slice_off if has_csc else csr_slice_off)])
        self.c = _Tensor(format=2 if has_csc else 1, n=self.n, m=self.m, dense=None,
                         csr_rowptr=csr_rowptr.data_ptr(), csr_col=csr_col.data_ptr(),
                         csr_val=None if csr_val is None else csr_val.data_ptr(),
                         csr_slice_off=C.cast(self._off1, C.POINTER(C.c_int64)),
                         csc_colptr=csc_colptr.data_ptr() if has_csc else None,
                         csc_row=csc_row.data_ptr() if has_csc else None,
                         csc_val=csc_val.data_ptr() if has_csc and csc_val is not None else None,
                         csc_slice_off=C.cast(self._off2, C.POINTER(C.c_int64)) if has_csc else None)
        self.nnz = int(csr_slice_off[-1])

    @staticmethod
    def from_device(S, with_csc=True):
        """S: synth.device_generators.DeviceSparseTensor (torch arrays already on the GPU)."""
        v = (lambda a: None) if getattr(S, "binary", False) else (lambda a: a)     # binary: no value arrays
        if with_csc:
            return SparseX(S.n, S.m, S.csr_rowptr, S.csr_col, v(S.csr_val), S.csr_slice_off,
                           S.csc_colptr, S.csc_row, v(S.csc_val), S.csc_slice_off)
        return SparseX(S.n, S.m, S.csr_rowptr, S.csr_col, v(S.csr_val), S.csr_slice_off)

    @staticmethod
    def from_host(S, device, with_csc=True):
        """S: synth.generators.SparseTensor (host numpy arrays); a binary one is handed over without value arrays."""
        import torch
        up = lambda a: torch.from_numpy(a).to(device)
        v = (lambda a: None) if getattr(S, "binary", False) else up
        if with_csc:
            return SparseX(S.n, S.m, up(S.csr_rowptr), up(S.csr_col), v(S.csr_val), S.csr_slice_off,
                           up(S.csc_colptr), up(S.csc_row), v(S.csc_val), S.csc_slice_off)
        return SparseX(S.n, S.m, up(S.csr_rowptr), up(S.csr_col), v(S.csr_val), S.csr_slice_off)


def _make_params(X, k, q, delta, eps_div, seed, stream, allocator, A0=None, R0=None, start=None, fused_small=True,
                 rank_packing=True, csc_build=True, handover_spin_limit=0, check_input=False, deterministic=False,
                 gather_form=0):
    """start: None (random start or A0/R0) or (svd_iters, r_iters, floor_rel) for the SVD-based start."""
    import torch
    if stream is None:
        stream = torch.cuda.current_stream(X.device)
    p = _Params(k=k, q=q, delta=delta, eps_div=eps_div, seed=seed, stream=stream.cuda_stream,
                alloc=allocator.alloc_cb, dealloc=allocator.dealloc_cb, alloc_ctx=None,
                A0=None if A0 is None else A0.data_ptr(), R0=None if R0 is None else R0.data_ptr())
    if start is not None:
        p.start, p.start_svd_iters, p.start_r_iters, p.start_floor_rel = 1, start[0], start[1], start[2]
    p.no_fused_small = 0 if fused_small else 1
    p.no_rank_packing = 0 if rank_packing else 1
    p.no_csc_build = 0 if csc_build else 1
    p.handover_spin_limit = handover_spin_limit
    p.check_input = 1 if check_input else 0
    p.deterministic = 1 if deterministic else 0
    p.gather_form = gather_form
    return p, stream


def _check(status, handle=None):
    if status != 0:
        msg = load().nnrescal_last_error(handle).decode()
        raise NNRescalError(status, msg)


class Handle:
    def __init__(self, ptr, X, params, allocator, stream, k, q):
        self.ptr, self.X, self.params, self.allocator, self.stream = ptr, X, params, allocator, stream
        self.k, self.q = k, q


# ------------------------------------------------------------------------------- the C ABI, same names
def nnrescal_init(X, k, q, delta=0.03, eps_div=1e-16, seed=0, stream=None, A0=None, R0=None, allocator=None,
                  start=None, fused_small=True, csc_build=True, handover_spin_limit=0, check_input=False,
                  deterministic=False, gather_form=0):
    lib = load()
    allocator = allocator or _TorchAllocator(X.device)
    A0, R0 = _dev_f32(A0, "A0"), _dev_f32(R0, "R0")
    p, stream = _make_params(X, k, q, delta, eps_div, seed, stream, allocator, A0, R0, start, fused_small,
                             csc_build=csc_build, handover_spin_limit=handover_spin_limit, check_input=check_input,
                             deterministic=deterministic, gather_form=gather_form)
    out = C.c_void_p()
    _check(lib.nnrescal_init(C.byref(out), C.byref(X.c), C.byref(p)))
    return Handle(out, X, p, allocator, stream, k, q)


def nnrescal_gather_form(h):
    """1 rows, 2 lines (the NNRESCAL_GATHER_ constants); 0: no batched sparse products on this handle."""
    return int(load().nnrescal_gather_form(h.ptr))


def nnrescal_mu_step(h):
    _check(load().nnrescal_mu_step(h.ptr), h.ptr)


def nnrescal_mu_step_static(X, A, R, delta=0.03, eps_div=1e-16, seed=0, stream=None, status=None):
    """One iteration on the caller's factors A [q][n][k], R [q][m][k][k] (float32, contiguous, on the GPU; updated in
    place) with every workspace in the library's static device array: the call allocates nothing.  status: optional
    int32 device tensor of one element that a kernel sets to 1 if a bounded wait ran out."""
    import torch
    for t, what in ((A, "A"), (R, "R")):
        if not (t.is_cuda and t.dtype == torch.float32 and t.is_contiguous()):
            raise TypeError(f"{what} must be a contiguous float32 tensor on the GPU")
    q, _, k = (int(v) for v in A.shape)
    if stream is None:
        stream = torch.cuda.current_stream(X.device)
    p = _Params(k=k, q=q, delta=delta, eps_div=eps_div, seed=seed, stream=stream.cuda_stream)
    _check(load().nnrescal_mu_step_static(C.byref(X.c), C.byref(p), _ptr(A), _ptr(R), _ptr(status)))


def nnrescal_fit(h, iters, objective=False):
    if objective:
        obj = (C.c_double * h.q)()
        _check(load().nnrescal_fit(h.ptr, iters, obj), h.ptr)
        return list(obj)
    _check(load().nnrescal_fit(h.ptr, iters, None), h.ptr)
    return None


def nnrescal_fit_until(h, max_iters, tau, check_every=1):
    """Returns (iterations done, trace) with trace[c][r] the objective of member r at check c."""
    done = C.c_int32(0)
    rows = max_iters // check_every if check_every >= 1 else 0
    trace = (C.c_double * max(rows * h.q, 1))()
    _check(load().nnrescal_fit_until(h.ptr, max_iters, C.c_double(tau), check_every, C.byref(done), trace), h.ptr)
    made = done.value // check_every
    return done.value, [[trace[c * h.q + r] for r in range(h.q)] for c in range(made)]


def nnrescal_start_nndsvd(h, svd_iters=30, r_iters=10, floor_rel=0.01):
    """Replaces the handle's factors by the SVD-based start; returns the singular values found, [q][k]."""
    sig = (C.c_float * (h.q * h.k))()
    _check(load().nnrescal_start_nndsvd(h.ptr, svd_iters, r_iters, C.c_float(floor_rel), sig), h.ptr)
    return [[sig[r * h.k + j] for j in range(h.k)] for r in range(h.q)]


def nnrescal_objective(h):
    obj, xn = (C.c_double * h.q)(), (C.c_double * h.q)()
    _check(load().nnrescal_objective(h.ptr, obj, xn), h.ptr)
    return list(obj), list(xn)


def nnrescal_get_factors(h, normalised=False):
    import torch
    A = torch.empty((h.q, h.X.n, h.k), dtype=torch.float32, device=h.X.device)
    R = torch.empty((h.q, h.X.m, h.k, h.k), dtype=torch.float32, device=h.X.device)
    with torch.cuda.stream(h.stream):
        _check(load().nnrescal_get_factors(h.ptr, _ptr(A), _ptr(R), 1 if normalised else 0), h.ptr)
    return A, R


def nnrescal_products(h, t):
    """(P, Q) of slice t for the current factors, torch [q][n][k] each."""
    import torch
    P = torch.empty((h.q, h.X.n, h.k), dtype=torch.float32, device=h.X.device)
    Q = torch.empty_like(P)
    with torch.cuda.stream(h.stream):
        _check(load().nnrescal_products(h.ptr, t, _ptr(P), _ptr(Q)), h.ptr)
    return P, Q


def nnrescal_set_factors(h, A, R):
    A, R = _dev_f32(A, "A"), _dev_f32(R, "R")
    _check(load().nnrescal_set_factors(h.ptr, _ptr(A), _ptr(R)), h.ptr)


def nnrescal_perturb(X, member, delta, seed, from_csc=False, stream=None):
    import torch
    stream = stream or torch.cuda.current_stream(X.device)
    if isinstance(X, DenseX):
        out = torch.empty_like(X.X)
    else:
        out = torch.empty(X.nnz, dtype=torch.float32, device=X.device)
    _check(load().nnrescal_perturb(C.byref(X.c), member, delta, seed, 1 if from_csc else 0, stream.cuda_stream,
                                   _ptr(out)))
    return out


def nnrescal_cluster(A_ens, R_ens=None, stream=None):
    """A_ens: torch [q][n][k] (cuda), R_ens: [q][m][k][k] or None -> dict."""
    import torch
    A_ens, R_ens = _dev_f32(A_ens, "A_ens"), _dev_f32(R_ens, "R_ens")
    q, n, k = (int(v) for v in A_ens.shape)
    m = int(R_ens.shape[1]) if R_ens is not None else 0
    allocator = _TorchAllocator(A_ens.device)

    class _X:
        device = A_ens.device
    p, stream = _make_params(_X, k, q, 0.0, 0.0, 0, stream, allocator)
    perm = (C.c_int32 * (q * k))()
    A_med = torch.empty((n, k), dtype=torch.float32, device=A_ens.device)
    R_med = torch.empty((m, k, k), dtype=torch.float32, device=A_ens.device) if R_ens is not None else None
    s_min, s_avg, rounds = C.c_float(), C.c_float(), C.c_int32()
    _check(load().nnrescal_cluster(_ptr(A_ens), _ptr(R_ens), n, m, k, q, C.byref(p), perm, _ptr(A_med), _ptr(R_med),
                                   C.byref(s_min), C.byref(s_avg), C.byref(rounds)))
    return {"perm": [[perm[r * k + s] for s in range(k)] for r in range(q)], "A_med": A_med, "R_med": R_med,
            "s_min": s_min.value, "s_avg": s_avg.value, "rounds": rounds.value}


def nnrescal_select_k(X, k_lo, k_hi, q, delta, iters, seed=0, eps_div=1e-16, regress_iters=1000, stream=None,
                      start=None, fused_small=True, rank_packing=True, csc_build=True, check_input=False,
                      deterministic=False, gather_form=0):
    import torch
    allocator = _TorchAllocator(X.device)
    p, stream = _make_params(X, 0, q, delta, eps_div, seed, stream, allocator, start=start, fused_small=fused_small,
                             rank_packing=rank_packing, csc_build=csc_build, check_input=check_input,
                             deterministic=deterministic, gather_form=gather_form)
    nk = k_hi - k_lo + 1
    s_min, s_avg, err = (C.c_float * nk)(), (C.c_float * nk)(), (C.c_float * nk)()
    k_opt = C.c_int32()
    A_med = torch.zeros((X.n * k_hi,), dtype=torch.float32, device=X.device)
    R_reg = torch.zeros((X.m * k_hi * k_hi,), dtype=torch.float32, device=X.device)
    _check(load().nnrescal_select_k(C.byref(X.c), C.byref(p), k_lo, k_hi, iters, regress_iters, s_min, s_avg, err,
                                    C.byref(k_opt), _ptr(A_med), _ptr(R_reg)))
    ko = k_opt.value
    return {"ks": list(range(k_lo, k_hi + 1)), "s_min": list(s_min), "s_avg": list(s_avg), "err": list(err),
            "k_opt": ko, "A_med": A_med[: X.n * ko].view(X.n, ko), "R_reg": R_reg[: X.m * ko * ko].view(X.m, ko, ko)}


def nnrescal_destroy(h):
    if h is not None and h.ptr:
        load().nnrescal_destroy(h.ptr)
        h.ptr = None


def nnrescal_last_error(h=None):
    return load().nnrescal_last_error(h.ptr if h is not None else None).decode()


def nnrescal_profile(h, enable):
    """enable: False/0 off, True/1 every kernel class, 2 only the passes over X."""
    ms, n = (C.c_double * PROF_CLASSES)(), (C.c_int64 * PROF_CLASSES)()
    _check(load().nnrescal_profile(h.ptr, int(enable), ms, n), h.ptr)
    return {PROF_NAMES[c]: (ms[c], n[c]) for c in range(PROF_CLASSES)}
