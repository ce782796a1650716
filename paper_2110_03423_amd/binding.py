"""ctypes binding of the C ABI in include/rsvd.h (argument marshalling only)."""
import ctypes as C
import os

F32, F64 = 0, 1
DEVICE_NONE = -1        # rsvd_create: planning context, no HIP call
ERR_NO_DEVICE = 5
JOB_S, JOB_SV, JOB_SUV = 0, 1, 2

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB = None


class RsvdError(RuntimeError):
    def __init__(self, code, text):
        super().__init__(f"rsvd error {code}: {text}")
        self.code = code


class _Info(C.Structure):
    _fields_ = [("status", C.c_int32), ("jacobi_sweeps", C.c_int32),
                ("refilled_columns", C.c_int32), ("skipped_reorth", C.c_int32), ("raised_pivots", C.c_int32)]


def library_path():
    return os.path.join(_HERE, "librsvd_gfx950.so")


_I64, _INT, _U64, _U32, _VP, _SZ = C.c_int64, C.c_int, C.c_uint64, C.c_uint32, C.c_void_p, C.c_size_t

# name -> argument types; mirrors include/rsvd.h
PROTOTYPES = {
    "rsvd_create": [C.POINTER(_VP), _INT],
    "rsvd_destroy": [_VP],
    "rsvd_status_string": [_INT],
    "rsvd_last_hip_error": [_VP],
    "rsvd_profile_enable": [_VP, _INT],
    "rsvd_profile_read": [_VP, _INT, C.POINTER(C.c_double), C.POINTER(_INT)],
    "rsvd_profile_kind_name": [_INT],
    "rsvd_workspace_bytes": [_VP, _INT, _I64, _I64, _INT, _INT, _INT, _INT, C.POINTER(_SZ)],
    "rsvd_run": [_VP, _VP, _INT, _INT, _I64, _I64, _VP, _I64, _INT, _INT, _INT, _U64,
                 _VP, _VP, _I64, _VP, _I64, _VP, _SZ, C.POINTER(_Info)],
    "rsvd_run_static": [_VP, _VP, _INT, _INT, _I64, _I64, _VP, _I64, _INT, _INT, _INT, _U64,
                        _VP, _VP, _I64, _VP, _I64, C.POINTER(_Info)],
    "rsvd_static_scratch_bytes": [],
    "rsvd_run_centered": [_VP, _VP, _INT, _INT, _I64, _I64, _VP, _I64, _INT, _INT, _INT, _U64,
                          _VP, _VP, _I64, _VP, _I64, _VP, _SZ, C.POINTER(_Info), _VP],
    "rsvd_workspace_bytes_batched": [_VP, _INT, _INT, _I64, _I64, _INT, _INT, _INT, _INT, C.POINTER(_SZ)],
    "rsvd_run_batched": [_VP, _VP, _INT, _INT, _INT, _I64, _I64, _VP, _I64, _I64, _INT, _INT, _INT, _U64,
                         _VP, _I64, _VP, _I64, _I64, _VP, _I64, _I64, _VP, _SZ, C.POINTER(_Info)],
    "rsvd_stage_workspace_bytes": [_VP, _INT, _I64, _I64, C.POINTER(_SZ)],
    "rsvd_stage_sketch": [_VP, _VP, _INT, _U64, _U32, _I64, _I64, _VP, _I64],
    "rsvd_stage_philox_raw": [_VP, _VP, _U64, _U32, _U64, _I64, _VP],
    "rsvd_stage_gemm_an": [_VP, _VP, _INT, _I64, _I64, _I64, _VP, _I64, _VP, _I64, _VP, _I64, _VP, _SZ],
    "rsvd_stage_gemm_atn": [_VP, _VP, _INT, _I64, _I64, _I64, _VP, _I64, _VP, _I64, _VP, _I64, _VP, _SZ],
    "rsvd_stage_orth": [_VP, _VP, _INT, _I64, _I64, _VP, _I64, _VP, _U64, _U32, _VP, _SZ, C.POINTER(_Info)],
    "rsvd_stage_small_svd": [_VP, _VP, _INT, _I64, _I64, _VP, _I64, _VP, _VP, _VP, _I64, _U64, _VP, _SZ,
                             C.POINTER(_Info)],
    "rsvd_stage_jacobi": [_VP, _VP, _INT, _I64, _VP, _VP, _VP, _VP, _VP, _SZ, C.POINTER(_Info)],
    "rsvd_stage_lift": [_VP, _VP, _INT, _I64, _I64, _I64, _VP, _I64, _VP, _I64, _VP, _I64, _INT, _VP, _SZ],
}


def load_library():
    """Load librsvd_gfx950.so; raises if it has not been built (no fallback path exists)."""
    global _LIB
    if _LIB is None:
        # torch first: it brings its own HIP runtime, and the library must bind to that one
        # (loading the library first pulls in another copy and torch then sees no GPU)
        import torch  # noqa: F401
        path = library_path()
        if not os.path.exists(path):
            raise RsvdError(-1, f"{path} is missing: build it with `python -m paper_2110_03423_amd.build`")
        lib = C.CDLL(path)
        for name, argtypes in PROTOTYPES.items():
            fn = getattr(lib, name)
            fn.argtypes = argtypes
            if name in ("rsvd_status_string", "rsvd_last_hip_error", "rsvd_profile_kind_name"):
                fn.restype = C.c_char_p
            elif name == "rsvd_static_scratch_bytes":
                fn.restype = C.c_size_t
            else:
                fn.restype = C.c_int
        _LIB = lib
    return _LIB


def _dtype_code(t):
    import torch
    if t.dtype == torch.float32:
        return F32
    if t.dtype == torch.float64:
        return F64
    raise TypeError("fp32 or fp64 tensors only")


def _ptr(t):
    return C.c_void_p(t.data_ptr()) if t is not None else C.c_void_p(0)


class Rsvd:
    """One context per device.  Methods mirror the C entry points by name."""

    def __init__(self, device=0):
        """device=None gives a planning context (RSVD_DEVICE_NONE): workspace sizes and argument checks only,
        no GPU and no torch needed."""
        self.lib = load_library()
        self._ws = None
        h = C.c_void_p()
        if device is None:
            self.torch = None
            self.device = None
            rc = self.lib.rsvd_create(C.byref(h), DEVICE_NONE)
        else:
            import torch
            self.torch = torch
            self.device = torch.device("cuda", device)
            rc = self.lib.rsvd_create(C.byref(h), device)
        if rc != 0:
            raise RsvdError(rc, "rsvd_create failed (no such device?)")
        self.h = h

    def close(self):
        if getattr(self, "h", None):
            self.lib.rsvd_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # ---- helpers
    def _check(self, rc):
        if rc != 0:
            text = self.lib.rsvd_status_string(rc).decode()
            if rc == 3 and getattr(self, "h", None):
                text += " (" + self.lib.rsvd_last_hip_error(self.h).decode() + ")"
            raise RsvdError(rc, text)

    def _stream(self):
        return C.c_void_p(self.torch.cuda.current_stream(self.device).cuda_stream)

    def rsvd_profile_enable(self, on):
        self._check(self.lib.rsvd_profile_enable(self.h, int(on)))

    def rsvd_profile_read(self):
        """{kernel class name: (total ms, launches)} since the last read."""
        n = 12
        ms = (C.c_double * n)()
        cnt = (C.c_int * n)()
        self._check(self.lib.rsvd_profile_read(self.h, n, ms, cnt))
        return {self.lib.rsvd_profile_kind_name(i).decode(): (ms[i], cnt[i]) for i in range(n) if cnt[i] > 0}

    def workspace_bytes(self, dtype, m, n, k, p, q=0, job=JOB_SUV):
        out = C.c_size_t()
        self._check(self.lib.rsvd_workspace_bytes(self.h, dtype, m, n, k, p, q, job, C.byref(out)))
        return out.value

    def workspace(self, dtype, m, n, k, p):
        """A cached uint8 tensor large enough for the problem (grown on demand).  The cache is one buffer per
        context: calls that rely on it must stay on one stream (a call on another stream could still be using
        the buffer that a growing request replaces); pass `workspace=` to own the buffer yourself."""
        return self._grow(self.workspace_bytes(dtype, m, n, k, p))

    def _grow(self, need):
        if self._ws is None or self._ws.numel() < need:
            self._ws = None
            self._ws = self.torch.empty(need, dtype=self.torch.uint8, device=self.device)
        return self._ws

    def stage_workspace(self, dtype, rows, l):
        """Cached workspace for the stage calls on one rows x l panel (orth, small_svd, jacobi)."""
        out = C.c_size_t()
        self._check(self.lib.rsvd_stage_workspace_bytes(self.h, dtype, rows, l, C.byref(out)))
        return self._grow(out.value)

    def _empty(self, shape, like):
        return self.torch.empty(shape, dtype=like.dtype, device=self.device)

    # ---- Algorithm 1
    def rsvd_run_centered(self, A, k, p, q, seed=0, job=JOB_SUV, workspace=None, want_info=True, out=None):
        """PCA front end: decomposition of A minus its column means.  Returns (S, U, Vt, info, mean)."""
        mean = self._empty((A.shape[1],), A)
        S, U, Vt, info = self.rsvd_run(A, k, p, q, seed, job, workspace, want_info, out, _mean=mean)
        return S, U, Vt, info, mean

    def rsvd_run(self, A, k, p, q, seed=0, job=JOB_SUV, workspace=None, want_info=True, out=None, _mean=None):
        """Returns (S, U, Vt, info).  A: row-major (m, n) device tensor, stride(1) == 1."""
        assert A.is_cuda and A.dim() == 2 and A.stride(1) == 1
        m, n = A.shape
        dt = _dtype_code(A)
        ws = workspace if workspace is not None else self.workspace(dt, m, n, k, p)
        if out is None:
            S = self._empty((k,), A)
            U = self._empty((m, k), A) if job == JOB_SUV else None
            Vt = self._empty((k, n), A) if job >= JOB_SV else None
        else:
            S, U, Vt = out
        info = _Info()
        args = (self.h, self._stream(), dt, job, m, n, _ptr(A), A.stride(0), k, p, q, seed,
                _ptr(S), _ptr(U), U.stride(0) if U is not None else 0,
                _ptr(Vt), Vt.stride(0) if Vt is not None else 0,
                _ptr(ws), ws.numel(), C.byref(info) if want_info else None)
        if _mean is None:
            rc = self.lib.rsvd_run(*args)
        else:
            rc = self.lib.rsvd_run_centered(*args, _ptr(_mean))
        self._check(rc)
        return S, U, Vt, (info if want_info else None)

    def rsvd_run_static(self, A, k, p, q, seed=0, job=JOB_SUV, want_info=True, out=None):
        """rsvd_run on the library's own static scratch buffer (no workspace argument).  `out` = (S, U, Vt)
        tensors of the caller; without it they are allocated here, by torch, before the call."""
        assert A.is_cuda and A.dim() == 2 and A.stride(1) == 1
        m, n = A.shape
        dt = _dtype_code(A)
        if out is None:
            S = self._empty((k,), A)
            U = self._empty((m, k), A) if job == JOB_SUV else None
            Vt = self._empty((k, n), A) if job >= JOB_SV else None
        else:
            S, U, Vt = out
        info = _Info()
        self._check(self.lib.rsvd_run_static(
            self.h, self._stream(), dt, job, m, n, _ptr(A), A.stride(0), k, p, q, seed,
            _ptr(S), _ptr(U), U.stride(0) if U is not None else 0,
            _ptr(Vt), Vt.stride(0) if Vt is not None else 0, C.byref(info) if want_info else None))
        return S, U, Vt, (info if want_info else None)

    def rsvd_run_batched(self, A, k, p, q, seed=0, job=JOB_SUV, workspace=None, want_info=True, out=None):
        """A: (batch, m, n) device tensor, each matrix row-major.  Returns (S (batch, k), U (batch, m, k),
        Vt (batch, k, n), info of the whole batch).  Problem b uses seed + b."""
        assert A.is_cuda and A.dim() == 3 and A.stride(2) == 1
        batch, m, n = A.shape
        dt = _dtype_code(A)
        if workspace is None:
            need = C.c_size_t()
            self._check(self.lib.rsvd_workspace_bytes_batched(self.h, dt, batch, m, n, k, p, q, job, C.byref(need)))
            if self._ws is None or self._ws.numel() < need.value:
                self._ws = None
                self._ws = self.torch.empty(need.value, dtype=self.torch.uint8, device=self.device)
            workspace = self._ws
        if out is None:
            S = self._empty((batch, k), A)
            U = self._empty((batch, m, k), A) if job == JOB_SUV else None
            Vt = self._empty((batch, k, n), A) if job >= JOB_SV else None
        else:
            S, U, Vt = out
        info = _Info()
        self._check(self.lib.rsvd_run_batched(
            self.h, self._stream(), dt, job, batch, m, n, _ptr(A), A.stride(1), A.stride(0), k, p, q, seed,
            _ptr(S), S.stride(0), _ptr(U), U.stride(1) if U is not None else 0, U.stride(0) if U is not None else 0,
            _ptr(Vt), Vt.stride(1) if Vt is not None else 0, Vt.stride(0) if Vt is not None else 0,
            _ptr(workspace), workspace.numel(), C.byref(info) if want_info else None))
        return S, U, Vt, (info if want_info else None)

    # ---- stages
    def rsvd_stage_sketch(self, seed, rows, cols, dtype, stream_id=0, out=None):
        t = self.torch
        if out is None:
            out = t.empty((rows, cols), dtype=t.float32 if dtype == F32 else t.float64, device=self.device)
        self._check(self.lib.rsvd_stage_sketch(self.h, self._stream(), dtype, seed, stream_id, rows, cols,
                                               _ptr(out), out.stride(0) if rows > 0 and cols > 0 else cols))
        return out

    def rsvd_stage_philox_raw(self, seed, first_group, n_groups, stream_id=0):
        t = self.torch
        out = t.empty((n_groups, 4), dtype=t.int32, device=self.device)
        self._check(self.lib.rsvd_stage_philox_raw(self.h, self._stream(), seed, stream_id, first_group, n_groups,
                                                   _ptr(out)))
        return out

    def _stage_gemm(self, fn, A, X, out_rows):
        m, n = A.shape
        l = X.shape[1]
        dt = _dtype_code(A)
        ws = self.workspace(dt, m, n, l, 0)
        Y = self._empty((out_rows, l), A)
        self._check(fn(self.h, self._stream(), dt, m, n, l, _ptr(A), A.stride(0), _ptr(X), X.stride(0),
                       _ptr(Y), Y.stride(0), _ptr(ws), ws.numel()))
        return Y

    def rsvd_stage_gemm_an(self, A, X):
        return self._stage_gemm(self.lib.rsvd_stage_gemm_an, A, X, A.shape[0])

    def rsvd_stage_gemm_atn(self, A, X):
        return self._stage_gemm(self.lib.rsvd_stage_gemm_atn, A, X, A.shape[1])

    def rsvd_stage_orth(self, Y, seed=0, refill_stream=16, want_r=False):
        """In place on Y.  Returns (Y, R or None, info)."""
        rows, l = Y.shape
        dt = _dtype_code(Y)
        ws = self.stage_workspace(dt, rows, l)
        R = self.torch.empty((l, l), dtype=self.torch.float64, device=self.device) if want_r else None
        info = _Info()
        self._check(self.lib.rsvd_stage_orth(self.h, self._stream(), dt, rows, l, _ptr(Y), Y.stride(0), _ptr(R),
                                             seed, refill_stream, _ptr(ws), ws.numel(), C.byref(info)))
        return Y, R, info

    def rsvd_stage_small_svd(self, Bt, seed=0):
        """Bt (n, l) is overwritten.  Returns (sigma, Ub, V, info)."""
        n, l = Bt.shape
        dt = _dtype_code(Bt)
        ws = self.stage_workspace(dt, n, l)
        sigma = self._empty((l,), Bt)
        Ub = self._empty((l, l), Bt)
        V = self._empty((n, l), Bt)
        info = _Info()
        self._check(self.lib.rsvd_stage_small_svd(self.h, self._stream(), dt, n, l, _ptr(Bt), Bt.stride(0),
                                                  _ptr(sigma), _ptr(Ub), _ptr(V), V.stride(0), seed,
                                                  _ptr(ws), ws.numel(), C.byref(info)))
        return sigma, Ub, V, info

    def rsvd_stage_jacobi(self, M):
        """M (l, l) is overwritten.  Returns (sigma, X, W, info)."""
        l = M.shape[0]
        dt = _dtype_code(M)
        ws = self.stage_workspace(dt, l, l)
        sigma = self._empty((l,), M)
        X = self._empty((l, l), M)
        W = self._empty((l, l), M)
        info = _Info()
        self._check(self.lib.rsvd_stage_jacobi(self.h, self._stream(), dt, l, _ptr(M), _ptr(sigma), _ptr(X),
                                               _ptr(W), _ptr(ws), ws.numel(), C.byref(info)))
        return sigma, X, W, info

    def rsvd_stage_lift(self, Q, W, k, transpose_out=False):
        m, l = Q.shape
        dt = _dtype_code(Q)
        U = self._empty((k, m) if transpose_out else (m, k), Q)
        self._check(self.lib.rsvd_stage_lift(self.h, self._stream(), dt, m, l, k, _ptr(Q), Q.stride(0),
                                             _ptr(W), W.stride(0), _ptr(U), U.stride(0), int(transpose_out),
                                             None, 0))
        return U
