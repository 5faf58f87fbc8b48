"""ctypes binding over libexat.so (C ABI in include/exat.h).

Argument marshalling only: every step of the compression runs in the HIP kernels.  PyTorch is
used for device memory (torch tensors own the buffers) and for the stream handle.  There is no
CPU fallback: if the library is missing, loading fails loudly.
"""
import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libexat.so")

EXAT_F32, EXAT_BF16, EXAT_F32_SPLIT = 0, 1, 2
OK, ERR_NULL, ERR_SHAPE, ERR_DTYPE, ERR_STATE, ERR_ALLOC, ERR_HIP = 0, -1, -2, -3, -4, -5, -6

EXPORTS = ["exat_plan_create", "exat_plan_destroy", "exat_set_factors", "exat_compress",
           "exat_compress_block", "exat_compress_blocks", "exat_finalize", "exat_compress_host", "exat_compress_gen", "exat_gen_block",
           "exat_plan_set_timing", "exat_plan_last_timing", "exat_plan_timing_of",
           "exat_stage1_create", "exat_stage1_destroy", "exat_stage1_dims", "exat_stage1_apply", "exat_stage1_apply_host",
           "exat_stage1_set_timing", "exat_stage1_last_timing", "exat_cpals_workspace_floats", "exat_cpals",
           "exat_cpals_checked", "exat_cpals_noalloc",
           "exat_ls_workspace_floats", "exat_ls", "exat_probe_mfma", "exat_strerror"]


class Desc(ctypes.Structure):
    _fields_ = [("I", ctypes.c_int64), ("J", ctypes.c_int64), ("K", ctypes.c_int64),
                ("L", ctypes.c_int32), ("M", ctypes.c_int32), ("N", ctypes.c_int32), ("P", ctypes.c_int32),
                ("dI", ctypes.c_int32), ("dJ", ctypes.c_int32), ("dK", ctypes.c_int32),
                ("in_dtype", ctypes.c_int32)]


class Gen(ctypes.Structure):
    _fields_ = [("A", ctypes.c_void_p), ("B", ctypes.c_void_p), ("C", ctypes.c_void_p),
                ("R", ctypes.c_int32), ("seed", ctypes.c_uint64), ("sigma", ctypes.c_float)]


class Box(ctypes.Structure):
    _fields_ = [("i0", ctypes.c_int64), ("i1", ctypes.c_int64), ("j0", ctypes.c_int64),
                ("j1", ctypes.c_int64), ("k0", ctypes.c_int64), ("k1", ctypes.c_int64)]


class Csr(ctypes.Structure):
    _fields_ = [("rows", ctypes.c_int32), ("cols", ctypes.c_int64), ("rowptr", ctypes.c_void_p),
                ("colidx", ctypes.c_void_p), ("val", ctypes.c_void_p)]


class ExatError(RuntimeError):
    def __init__(self, status, msg):
        super().__init__("exat: %s (status %d)" % (msg, status))
        self.status = status


_lib = None


def lib():
    """Loads libexat.so; raises if it has not been built (python -m paper_2311_13693_amd.build)."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            # nothing built yet: build the HIP library now (needs hipcc); there is no CPU fallback
            try:
                from . import build as _b
                _b.build(force=True)
            except Exception as e:
                raise ImportError("libexat.so is not built and building it failed (%s): run "
                                  "`python paper_2311_13693_amd/build.py`; there is no CPU fallback" % e)
        L = ctypes.CDLL(_LIB_PATH)
        vp, i32, i64 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64
        L.exat_plan_create.argtypes = [ctypes.POINTER(vp), ctypes.POINTER(Desc)]
        L.exat_plan_destroy.argtypes = [vp]
        L.exat_set_factors.argtypes = [vp, vp, i64, vp, i64, vp, i64, vp]
        L.exat_compress.argtypes = [vp, vp, vp, vp]
        L.exat_compress_block.argtypes = [vp, vp, i32, i32, i32, vp]
        L.exat_compress_blocks.argtypes = [vp, ctypes.POINTER(vp), i32, i32, i32, i32, vp]
        L.exat_finalize.argtypes = [vp, vp, vp]
        L.exat_compress_host.argtypes = [vp, vp, vp, vp]
        L.exat_compress_gen.argtypes = [vp, ctypes.POINTER(Gen), ctypes.POINTER(Box), vp, vp]
        L.exat_gen_block.argtypes = [ctypes.POINTER(Desc), ctypes.POINTER(Gen), i32, i32, i32, vp, vp]
        L.exat_plan_set_timing.argtypes = [vp, ctypes.c_int]
        L.exat_plan_last_timing.argtypes = [vp, ctypes.POINTER(ctypes.c_float), ctypes.POINTER(ctypes.c_float)]
        L.exat_plan_timing_of.argtypes = [vp, i32, ctypes.POINTER(ctypes.c_float), ctypes.POINTER(ctypes.c_float)]
        L.exat_stage1_create.argtypes = [ctypes.POINTER(vp), i64, i64, i64, ctypes.POINTER(Csr), ctypes.POINTER(Csr),
                                         ctypes.POINTER(Csr)]
        L.exat_stage1_destroy.argtypes = [vp]
        L.exat_stage1_dims.argtypes = [vp, ctypes.POINTER(i32), ctypes.POINTER(i32), ctypes.POINTER(i32)]
        L.exat_stage1_apply.argtypes = [vp, vp, vp, vp]
        L.exat_stage1_apply_host.argtypes = [vp, vp, vp, vp]
        L.exat_stage1_set_timing.argtypes = [vp, ctypes.c_int]
        L.exat_stage1_last_timing.argtypes = [vp, ctypes.POINTER(ctypes.c_float), ctypes.POINTER(ctypes.c_float)]
        L.exat_cpals_workspace_floats.argtypes = [i32, i32, i32, i32]
        L.exat_cpals.argtypes = [vp, i32, i32, i32, i32, i32, i32, vp, vp, vp, vp, vp]
        L.exat_cpals_checked.argtypes = [vp, i32, i32, i32, i32, i32, i32, vp, vp, vp, vp, vp, vp]
        L.exat_cpals_noalloc.argtypes = [vp, i32, i32, i32, i32, i32, i32, vp, vp, vp, vp]
        L.exat_ls_workspace_floats.argtypes = [i32, i32, i32, i32]
        L.exat_ls.argtypes = [vp, i64, i32, i32, i32, vp, i32, i32, ctypes.c_float, vp, vp, vp, vp]
        L.exat_probe_mfma.argtypes = [i32, i32, i32, i32, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_double)]
        L.exat_strerror.argtypes = [ctypes.c_int]
        L.exat_strerror.restype = ctypes.c_char_p
        for name in EXPORTS[:-1]:
            getattr(L, name).restype = ctypes.c_int
        L.exat_cpals_workspace_floats.restype = ctypes.c_int64
        L.exat_ls_workspace_floats.restype = ctypes.c_int64
        _lib = L
    return _lib


def probe_mfma(kind, random_operands, iters, workgroups=256):
    """MFMA-only rate (TFLOP/s) and core clock (GHz) of this GPU; kind 0 = bf16 32x32x16, 1 = fp32 32x32x2."""
    tf, ghz = ctypes.c_double(0.0), ctypes.c_double(0.0)
    _check(lib().exat_probe_mfma(kind, 1 if random_operands else 0, iters, workgroups, ctypes.byref(tf), ctypes.byref(ghz)))
    return tf.value, ghz.value


def strerror(status):
    return lib().exat_strerror(int(status)).decode()


def _check(status):
    if status != OK:
        raise ExatError(status, strerror(status))


def _stream_handle(stream):
    import torch
    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


def _ptr(t):
    return ctypes.c_void_p(t.data_ptr())


def make_desc(I, J, K, L, M, N, P, dI, dJ, dK, in_dtype=EXAT_F32):
    return Desc(I, J, K, L, M, N, P, dI, dJ, dK, in_dtype)


def make_gen(A, B, C, seed, sigma):
    """A, B, C: float32 CUDA tensors holding the column-major I x R, J x R, K x R factor matrices,
    i.e. torch tensors of shape (R, I) etc. that are contiguous (element (i, r) at r*I + i)."""
    import torch
    for t in (A, B, C):
        assert t.is_cuda and t.dtype == torch.float32 and t.is_contiguous() and t.dim() == 2
    g = Gen(A.data_ptr(), B.data_ptr(), C.data_ptr(), A.shape[0], seed & 0xFFFFFFFFFFFFFFFF, float(sigma))
    g._keep = (A, B, C)
    return g


def gen_block(desc, gen, bi, bj, bk, out, stream=None):
    """Writes block (bi,bj,bk) of the synthetic tensor into `out` (CUDA tensor of dI*dJ*dK elements,
    float32 or bfloat16 according to desc.in_dtype, column-major on the block)."""
    _check(lib().exat_gen_block(ctypes.byref(desc), ctypes.byref(gen), bi, bj, bk, _ptr(out), _stream_handle(stream)))
    return out


class Plan:
    """Owns an exat_plan_t.  Tensors passed in must be CUDA tensors on the current device."""

    def __init__(self, desc):
        self.desc = desc
        self._h = ctypes.c_void_p()
        _check(lib().exat_plan_create(ctypes.byref(self._h), ctypes.byref(desc)))
        self.ysize = desc.P * desc.L * desc.M * desc.N

    def close(self):
        if self._h:
            import torch
            torch.cuda.synchronize()
            lib().exat_plan_destroy(self._h)
            self._h = ctypes.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def set_factors(self, U, V, W, stream=None):
        """U (P*L, I), V (P*M, J), W (P*N, K): float32 CUDA tensors, last dimension contiguous."""
        import torch
        for t in (U, V, W):
            assert t.is_cuda and t.dtype == torch.float32 and t.dim() == 2 and t.stride(1) == 1
        _check(lib().exat_set_factors(self._h, _ptr(U), U.stride(0), _ptr(V), V.stride(0), _ptr(W), W.stride(0),
                                      _stream_handle(stream)))

    def set_timing(self, enable=True):
        _check(lib().exat_plan_set_timing(self._h, 1 if enable else 0))

    def last_timing(self):
        """(ms of the fused mode-1/2 kernel, ms of the mode-3 kernel) of the most recent compress call."""
        a, b = ctypes.c_float(), ctypes.c_float()
        _check(lib().exat_plan_last_timing(self._h, ctypes.byref(a), ctypes.byref(b)))
        return a.value, b.value

    def timing_of(self, age):
        """The same for the compress call `age` calls back (0 = the most recent, at most 127)."""
        a, b = ctypes.c_float(), ctypes.c_float()
        _check(lib().exat_plan_timing_of(self._h, int(age), ctypes.byref(a), ctypes.byref(b)))
        return a.value, b.value

    def new_y(self):
        import torch
        return torch.empty(self.ysize, dtype=torch.float32, device="cuda")

    def compress(self, X, Y=None, stream=None):
        """X: CUDA tensor holding the column-major I x J x K tensor (float32 or bfloat16)."""
        Y = self.new_y() if Y is None else Y
        _check(lib().exat_compress(self._h, _ptr(X), _ptr(Y), _stream_handle(stream)))
        return Y

    def compress_block(self, Xblk, bi, bj, bk, stream=None):
        _check(lib().exat_compress_block(self._h, _ptr(Xblk), bi, bj, bk, _stream_handle(stream)))

    def compress_blocks(self, blocks, bj0, bj1, bk0, bk1, stream=None):
        """blocks: device tensors of the slab's blocks, bi fastest, then bj, then bk (whole block columns along i)."""
        arr = (ctypes.c_void_p * len(blocks))(*[b.data_ptr() for b in blocks])
        _check(lib().exat_compress_blocks(self._h, arr, bj0, bj1, bk0, bk1, _stream_handle(stream)))

    def finalize(self, Y=None, stream=None):
        Y = self.new_y() if Y is None else Y
        _check(lib().exat_finalize(self._h, _ptr(Y), _stream_handle(stream)))
        return Y

    def compress_host(self, Xhost, Y=None, stream=None):
        """Xhost: CPU tensor (ideally pinned) holding the column-major I x J x K tensor; streamed block by block."""
        assert not Xhost.is_cuda and Xhost.is_contiguous()
        Y = self.new_y() if Y is None else Y
        _check(lib().exat_compress_host(self._h, _ptr(Xhost), _ptr(Y), _stream_handle(stream)))
        return Y

    def compress_gen(self, gen, box=None, Y=None, stream=None):
        Y = self.new_y() if Y is None else Y
        b = None if box is None else ctypes.byref(Box(*box))
        _check(lib().exat_compress_gen(self._h, ctypes.byref(gen), b, _ptr(Y), _stream_handle(stream)))
        return Y


def make_csr(rowptr, colidx, val, cols):
    """Host CSR arrays (numpy) -> exat_csr_t; the arrays are converted to int64 / int32 / float32 and kept alive."""
    import numpy as np
    rp = np.ascontiguousarray(rowptr, dtype=np.int64)
    ci = np.ascontiguousarray(colidx, dtype=np.int32)
    v = np.ascontiguousarray(val, dtype=np.float32)
    c = Csr(len(rp) - 1, cols, rp.ctypes.data, ci.ctypes.data, v.ctypes.data)
    c._keep = (rp, ci, v)
    return c


class Stage1:
    """Owns an exat_stage1_t: the sparse first stage X1 = X x1 U x2 V x3 W of the two-stage compression.
    U, V, W are (rowptr, colidx, val) CSR triples in host memory."""

    def __init__(self, I, J, K, U, V, W):
        self._h = ctypes.c_void_p()
        cu, cv, cw = make_csr(*U, I), make_csr(*V, J), make_csr(*W, K)
        _check(lib().exat_stage1_create(ctypes.byref(self._h), I, J, K, ctypes.byref(cu), ctypes.byref(cv),
                                        ctypes.byref(cw)))
        a, b, c = ctypes.c_int32(), ctypes.c_int32(), ctypes.c_int32()
        _check(lib().exat_stage1_dims(self._h, ctypes.byref(a), ctypes.byref(b), ctypes.byref(c)))
        self.dims = (a.value, b.value, c.value)

    def close(self):
        if self._h:
            import torch
            torch.cuda.synchronize()
            lib().exat_stage1_destroy(self._h)
            self._h = ctypes.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def set_timing(self, enable=True):
        _check(lib().exat_stage1_set_timing(self._h, 1 if enable else 0))

    def last_timing(self):
        a, b = ctypes.c_float(), ctypes.c_float()
        _check(lib().exat_stage1_last_timing(self._h, ctypes.byref(a), ctypes.byref(b)))
        return a.value, b.value

    def apply(self, X, X1=None, stream=None):
        """X: float32 CUDA tensor holding the column-major I x J x K tensor; returns the flat column-major
        A1 x B1 x C1 result."""
        import torch
        assert X.is_cuda and X.dtype == torch.float32 and X.is_contiguous()
        if X1 is None:
            X1 = torch.empty(self.dims[0] * self.dims[1] * self.dims[2], dtype=torch.float32, device="cuda")
        _check(lib().exat_stage1_apply(self._h, _ptr(X), _ptr(X1), _stream_handle(stream)))
        return X1

    def apply_host(self, Xhost, X1=None, stream=None):
        """Xhost: float32 CPU tensor (ideally pinned) holding the column-major tensor; streamed slab by slab."""
        import torch
        assert (not Xhost.is_cuda) and Xhost.dtype == torch.float32 and Xhost.is_contiguous()
        if X1 is None:
            X1 = torch.empty(self.dims[0] * self.dims[1] * self.dims[2], dtype=torch.float32, device="cuda")
        _check(lib().exat_stage1_apply_host(self._h, _ptr(Xhost), _ptr(X1), _stream_handle(stream)))
        return X1


def cpals(Y, L, M, N, P, R, sweeps, A, B, C, work=None, stream=None):
    """Batched CP-ALS (Alg. 1) on the P proxy tensors in Y (the flat output of Plan.compress).  A, B, C: float32 CUDA
    tensors of P*L*R, P*M*R, P*N*R elements (per replica column-major), start values in, results out (in place)."""
    import torch
    for t in (Y, A, B, C):
        assert t.is_cuda and t.dtype == torch.float32 and t.is_contiguous()
    if work is None:
        work = torch.empty(lib().exat_cpals_workspace_floats(L, M, N, P), dtype=torch.float32, device="cuda")
    _check(lib().exat_cpals(_ptr(Y), L, M, N, P, R, sweeps, _ptr(A), _ptr(B), _ptr(C), _ptr(work), _stream_handle(stream)))
    return A, B, C


def cpals_checked(Y, L, M, N, P, R, sweeps, A, B, C, work=None, status=None, stream=None):
    """cpals that also reports, per replica, how many factor updates met a normal matrix that was not positive definite
    (int32 CUDA tensor of P entries, all zero in a healthy run).  Returns (A, B, C, status)."""
    import torch
    if work is None:
        work = torch.empty(lib().exat_cpals_workspace_floats(L, M, N, P), dtype=torch.float32, device="cuda")
    if status is None:
        status = torch.empty(P, dtype=torch.int32, device="cuda")
    _check(lib().exat_cpals_checked(_ptr(Y), L, M, N, P, R, sweeps, _ptr(A), _ptr(B), _ptr(C), _ptr(work), _ptr(status),
                                    _stream_handle(stream)))
    return A, B, C, status


def cpals_noalloc(Y, L, M, N, P, R, sweeps, A, B, C, stream=None):
    """cpals on the library's static workspace: allocates nothing (no torch tensor is created here either)."""
    _check(lib().exat_cpals_noalloc(_ptr(Y), L, M, N, P, R, sweeps, _ptr(A), _ptr(B), _ptr(C), _stream_handle(stream)))
    return A, B, C


def ls(U, P, L, I, Astack, R, iters, tol=1e-6, X=None, relres=None, work=None, stream=None):
    """Stacked least squares of Eq. 4 (CGLS, at most `iters` iterations from zero, columns frozen at relative
    normal-equation residual `tol`).  U: float32 CUDA tensor holding the
    stacked (P*L, I) matrix row-major (its stride(0) is the leading dimension); Astack: P*L*R floats in the layout
    cpals writes.  Returns (X, relres): X as I*R floats column-major, relres R floats."""
    import torch
    assert U.is_cuda and U.dtype == torch.float32 and U.dim() == 2 and U.stride(1) == 1 and tuple(U.shape) == (P * L, I)
    assert Astack.is_cuda and Astack.dtype == torch.float32 and Astack.is_contiguous() and Astack.numel() == P * L * R
    if X is None:
        X = torch.empty(I * R, dtype=torch.float32, device="cuda")
    if relres is None:
        relres = torch.empty(R, dtype=torch.float32, device="cuda")
    if work is None:
        work = torch.empty(lib().exat_ls_workspace_floats(P, L, I, R), dtype=torch.float32, device="cuda")
    _check(lib().exat_ls(_ptr(U), ctypes.c_int64(U.stride(0)), P, L, I, _ptr(Astack), R, iters, ctypes.c_float(tol), _ptr(X), _ptr(relres),
                         _ptr(work), _stream_handle(stream)))
    return X, relres
