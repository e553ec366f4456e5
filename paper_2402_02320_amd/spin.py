"""ctypes binding of libspin.so (include/spin.h).  Argument marshalling only:
every step of the protocol runs in the library's kernels.

Ring tensors are torch.int64 CUDA tensors (the bit pattern of a uint64 ring
element), party-major ([n, ...]).  Calls are enqueued on torch's current
stream.  The library must have been built (python -m paper_2402_02320_amd.build);
there is no fallback: a missing library raises.
"""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libspin.so")

LIMB_MFMA, VALU = 0, 1
MAX_PARTIES = 8

_lib = None


class SpinError(RuntimeError):
    pass


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise SpinError("%s not found: build it with `python -m paper_2402_02320_amd.build`" % LIB_PATH)
        L = ctypes.CDLL(LIB_PATH)
        u64, sz, i32, p = ctypes.c_uint64, ctypes.c_size_t, ctypes.c_int, ctypes.c_void_p
        L.spin_random.argtypes = [p, sz, u64, u64, u64, u64, p]
        L.spin_share.argtypes = [p, sz, i32, u64, u64, p, p]
        L.spin_open.argtypes = [p, p, sz, i32, p, p]
        L.spin_beaver_matmul.argtypes = [i32] * 5 + [p] * 6 + [i32, p, sz, p]
        L.spin_beaver_matmul_nt.argtypes = L.spin_beaver_matmul.argtypes
        L.spin_beaver_matmul_nt.restype = i32
        L.spin_beaver_matmul_static.argtypes = [i32] * 5 + [p] * 6 + [i32, p]
        L.spin_beaver_matmul_static.restype = i32
        L.spin_beaver_matmul_grouped.argtypes = [i32, i32, p, i32, p, sz, p]
        L.spin_beaver_matmul_grouped.restype = i32
        L.spin_beaver_matmul_grouped_workspace_bytes.argtypes = [i32, i32, p, i32]
        L.spin_beaver_matmul_grouped_workspace_bytes.restype = sz
        L.spin_beaver_matmul_workspace_bytes.argtypes = [i32] * 5 + [i32]
        L.spin_beaver_matmul_workspace_bytes.restype = sz
        L.spin_beaver_mul.argtypes = [i32, sz] + [p] * 6 + [p]
        L.spin_beaver_mul_trunc.argtypes = [i32, sz, i32] + [p] * 9 + [p]
        L.spin_beaver_mul_trunc.restype = i32
        L.spin_beaver_mul_bcast.argtypes = [i32, sz, sz, sz, i32] + [p] * 6 + [p]
        L.spin_beaver_mul_bcast.restype = i32
        L.spin_trunc.argtypes = [i32, sz, i32] + [p] * 5 + [p]
        L.spin_lincomb_trunc.argtypes = [i32, sz, i32, p, p, u64, i32, p, p, p, p, p]
        L.spin_lincomb_trunc.restype = i32
        L.spin_bshare.argtypes = [p, sz, i32, u64, u64, p, p]
        L.spin_bopen.argtypes = [p, p, sz, i32, p, p]
        L.spin_beaver_and.argtypes = [i32, sz] + [p] * 6 + [p]
        for name in ("spin_bshare", "spin_bopen", "spin_beaver_and"):
            getattr(L, name).restype = i32
        for name in ("spin_random", "spin_share", "spin_open", "spin_beaver_matmul", "spin_beaver_mul", "spin_trunc"):
            getattr(L, name).restype = i32
        L.spin_profile_enable.argtypes = [i32]
        L.spin_profile_enable.restype = None
        L.spin_profile_reset.restype = None
        L.spin_profile_read.argtypes = [i32, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_uint)]
        L.spin_profile_read.restype = i32
        L.spin128_share.argtypes = L.spin_share.argtypes
        L.spin128_open.argtypes = L.spin_open.argtypes
        L.spin128_beaver_matmul.argtypes = L.spin_beaver_matmul.argtypes
        L.spin128_beaver_matmul_workspace_bytes.argtypes = L.spin_beaver_matmul_workspace_bytes.argtypes
        L.spin128_beaver_matmul_workspace_bytes.restype = sz
        L.spin128_beaver_mul.argtypes = L.spin_beaver_mul.argtypes
        L.spin128_trunc.argtypes = L.spin_trunc.argtypes
        for name in ("spin128_share", "spin128_open", "spin128_beaver_matmul", "spin128_beaver_mul", "spin128_trunc"):
            getattr(L, name).restype = i32
        L.spin32_share.argtypes = L.spin_share.argtypes
        L.spin32_open.argtypes = L.spin_open.argtypes
        L.spin32_beaver_matmul.argtypes = L.spin_beaver_matmul.argtypes
        L.spin32_beaver_matmul_workspace_bytes.argtypes = L.spin_beaver_matmul_workspace_bytes.argtypes
        L.spin32_beaver_matmul_workspace_bytes.restype = sz
        L.spin32_beaver_mul.argtypes = L.spin_beaver_mul.argtypes
        L.spin32_trunc.argtypes = L.spin_trunc.argtypes
        L.spin_cast_64_to_32.argtypes = [p, sz, p, p]
        for name in ("spin32_share", "spin32_open", "spin32_beaver_matmul", "spin32_beaver_mul", "spin32_trunc",
                     "spin_cast_64_to_32"):
            getattr(L, name).restype = i32
        L.spin_probe_mfma.argtypes = [p, i32, i32, p, p]
        L.spin_probe_mfma.restype = i32
        L.spin_status_string.argtypes = [i32]
        L.spin_status_string.restype = ctypes.c_char_p
        L.spin_last_hip_error.restype = ctypes.c_char_p
        _lib = L
    return _lib


def _check(status):
    if status != 0:
        L = lib()
        msg = L.spin_status_string(status).decode()
        if status == 4:
            msg += ": " + L.spin_last_hip_error().decode()
        raise SpinError(msg)


def _dev(t, name):
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.dtype == torch.int64 and t.is_contiguous()):
        raise SpinError("%s must be a contiguous torch.int64 CUDA tensor" % name)
    return t.data_ptr()


def _stream():
    return torch.cuda.current_stream().cuda_stream


def random(count, seed, stream_id, party, first_idx=0, device="cuda"):
    out = torch.empty(count, dtype=torch.int64, device=device)
    _check(lib().spin_random(_dev(out, "out"), count, seed, stream_id, party, first_idx, _stream()))
    return out


def share(x, n, seed, stream_id, out=None):
    if out is None:
        out = torch.empty((n,) + tuple(x.shape), dtype=torch.int64, device=x.device)
    _check(lib().spin_share(_dev(x, "x"), x.numel(), n, seed, stream_id, _dev(out, "shares"), _stream()))
    return out


def open(shares, mask=None, out=None):  # noqa: A001 - named after the C entry point
    n = shares.shape[0]
    if out is None:
        out = torch.empty(tuple(shares.shape[1:]), dtype=torch.int64, device=shares.device)
    if mask is not None and mask.shape != shares.shape:
        raise SpinError("mask must have the shape of shares")
    _check(lib().spin_open(_dev(shares, "shares"), None if mask is None else _dev(mask, "mask"),
                           out.numel(), n, _dev(out, "out"), _stream()))
    return out


def beaver_matmul_workspace_bytes(n, batch, M, N, K, path=LIMB_MFMA):
    return int(lib().spin_beaver_matmul_workspace_bytes(n, batch, M, N, K, path))


def beaver_matmul(X, Y, A, B, C, path=LIMB_MFMA, out=None, workspace=None, y_transposed=False):
    """X, A: [n,batch,M,K]; Y, B: [n,batch,K,N] (or [n,batch,N,K] with y_transposed, for X . Y^T);
    C: [n,batch,M,N] -> Z [n,batch,M,N]."""
    n, batch, M, K = X.shape
    N = Y.shape[2] if y_transposed else Y.shape[3]
    yshape = (n, batch, N, K) if y_transposed else (n, batch, K, N)
    if tuple(Y.shape) != yshape or A.shape != X.shape or B.shape != Y.shape or tuple(C.shape) != (n, batch, M, N):
        raise SpinError("inconsistent operand shapes")
    if out is None:
        out = torch.empty_like(C)
    need = beaver_matmul_workspace_bytes(n, batch, M, N, K, path)
    if need == 0:
        raise SpinError("invalid matmul dimensions")
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=X.device)
    if not (workspace.is_cuda and workspace.is_contiguous()):
        raise SpinError("workspace must be a contiguous CUDA tensor")
    call = lib().spin_beaver_matmul_nt if y_transposed else lib().spin_beaver_matmul
    _check(call(n, batch, M, N, K, _dev(X, "X"), _dev(Y, "Y"), _dev(A, "A"), _dev(B, "B"), _dev(C, "C"),
                _dev(out, "Z"), path, workspace.data_ptr(), workspace.numel() * workspace.element_size(), _stream()))
    return out


STATIC_WORKSPACE_BYTES = 64 << 20


def beaver_matmul_static(X, Y, A, B, C, out, path=LIMB_MFMA):
    """spin_beaver_matmul_static: the Beaver matmul on the library's built-in workspace.  The entry point
    allocates nothing, so the binding does not either: the caller passes `out`."""
    n, batch, M, K = X.shape
    N = Y.shape[3]
    if tuple(Y.shape) != (n, batch, K, N) or A.shape != X.shape or B.shape != Y.shape \
            or tuple(C.shape) != (n, batch, M, N) or out.shape != C.shape:
        raise SpinError("inconsistent operand shapes")
    _check(lib().spin_beaver_matmul_static(n, batch, M, N, K, _dev(X, "X"), _dev(Y, "Y"), _dev(A, "A"), _dev(B, "B"),
                                           _dev(C, "C"), _dev(out, "Z"), path, _stream()))
    return out


class _MatmulGroup(ctypes.Structure):
    _fields_ = [("batch", ctypes.c_int), ("M", ctypes.c_int), ("N", ctypes.c_int), ("K", ctypes.c_int),
                ("X", ctypes.c_void_p), ("Y", ctypes.c_void_p), ("A", ctypes.c_void_p), ("B", ctypes.c_void_p),
                ("C", ctypes.c_void_p), ("Z", ctypes.c_void_p), ("y_transposed", ctypes.c_int)]


def beaver_matmul_grouped(groups, path=LIMB_MFMA, workspace=None):
    """groups: list of dicts with X, Y, A, B, C (as for beaver_matmul), optional out and y_transposed; shapes may
    differ between groups, the party count may not.  Returns the list of Z tensors."""
    n = groups[0]["X"].shape[0]
    desc = (_MatmulGroup * len(groups))()
    outs = []
    for d, g in zip(desc, groups):
        X, Y, A, B, C = g["X"], g["Y"], g["A"], g["B"], g["C"]
        yt = bool(g.get("y_transposed", False))
        nn, batch, M, K = X.shape
        N = Y.shape[2] if yt else Y.shape[3]
        yshape = (n, batch, N, K) if yt else (n, batch, K, N)
        if nn != n or tuple(Y.shape) != yshape or A.shape != X.shape or B.shape != Y.shape \
                or tuple(C.shape) != (n, batch, M, N):
            raise SpinError("inconsistent operand shapes")
        out = g.get("out")
        if out is None:
            out = torch.empty_like(C)
        outs.append(out)
        d.batch, d.M, d.N, d.K = batch, M, N, K
        d.X, d.Y, d.A, d.B, d.C, d.Z = (_dev(t, k) for t, k in ((X, "X"), (Y, "Y"), (A, "A"), (B, "B"), (C, "C"), (out, "Z")))
        d.y_transposed = 1 if yt else 0
    L = lib()
    need = int(L.spin_beaver_matmul_grouped_workspace_bytes(n, len(groups), desc, path))
    if need == 0:
        raise SpinError("invalid matmul dimensions")
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=outs[0].device)
    _check(L.spin_beaver_matmul_grouped(n, len(groups), desc, path, workspace.data_ptr(),
                                        workspace.numel() * workspace.element_size(), _stream()))
    return outs


def beaver_mul(x, y, a, b, c, out=None):
    n = x.shape[0]
    for t in (y, a, b, c):
        if t.shape != x.shape:
            raise SpinError("inconsistent operand shapes")
    if out is None:
        out = torch.empty_like(x)
    _check(lib().spin_beaver_mul(n, x[0].numel(), _dev(x, "x"), _dev(y, "y"), _dev(a, "a"), _dev(b, "b"),
                                 _dev(c, "c"), _dev(out, "z"), _stream()))
    return out


def beaver_mul_trunc(x, y, a, b, c, r, r_top, r_msb, f, out=None):
    """Mul then Truncate by f bits in one pass; all operands [n, count]."""
    n = x.shape[0]
    for t in (y, a, b, c, r, r_top, r_msb):
        if t.shape != x.shape:
            raise SpinError("inconsistent operand shapes")
    if out is None:
        out = torch.empty_like(x)
    _check(lib().spin_beaver_mul_trunc(n, x[0].numel(), f, _dev(x, "x"), _dev(y, "y"), _dev(a, "a"), _dev(b, "b"),
                                       _dev(c, "c"), _dev(r, "r"), _dev(r_top, "r_top"), _dev(r_msb, "r_msb"),
                                       _dev(out, "out"), _stream()))
    return out


def beaver_mul_bcast(x, y, a, b, c, over_inner, out=None):
    """Batch multiplication with the small factor tiled (Section 7.3).  y, b, c: [n, outer, mid, inner];
    x, a: [n, outer, mid] (over_inner, one factor per row) or [n, outer, inner] (one per column)."""
    n, outer, mid, inner = y.shape
    small = (n, outer, mid) if over_inner else (n, outer, inner)
    if tuple(x.shape) != small or a.shape != x.shape or b.shape != y.shape or c.shape != y.shape:
        raise SpinError("inconsistent operand shapes")
    if out is None:
        out = torch.empty_like(y)
    _check(lib().spin_beaver_mul_bcast(n, outer, mid, inner, 1 if over_inner else 0, _dev(x, "x"), _dev(y, "y"),
                                       _dev(a, "a"), _dev(b, "b"), _dev(c, "c"), _dev(out, "z"), _stream()))
    return out


def trunc(x, r, r_top, r_msb, f, out=None):
    n = x.shape[0]
    for t in (r, r_top, r_msb):
        if t.shape != x.shape:
            raise SpinError("inconsistent operand shapes")
    if out is None:
        out = torch.empty_like(x)
    _check(lib().spin_trunc(n, x[0].numel(), f, _dev(x, "x"), _dev(r, "r"), _dev(r_top, "r_top"),
                            _dev(r_msb, "r_msb"), _dev(out, "out"), _stream()))
    return out


def bshare(x, n, seed, stream_id, out=None):
    if out is None:
        out = torch.empty((n,) + tuple(x.shape), dtype=torch.int64, device=x.device)
    _check(lib().spin_bshare(_dev(x, "x"), x.numel(), n, seed, stream_id, _dev(out, "shares"), _stream()))
    return out


def bopen(shares, mask=None, out=None):
    n = shares.shape[0]
    if out is None:
        out = torch.empty(tuple(shares.shape[1:]), dtype=torch.int64, device=shares.device)
    if mask is not None and mask.shape != shares.shape:
        raise SpinError("mask must have the shape of shares")
    _check(lib().spin_bopen(_dev(shares, "shares"), None if mask is None else _dev(mask, "mask"),
                            out.numel(), n, _dev(out, "out"), _stream()))
    return out


def beaver_and(x, y, a, b, c, out=None):
    n = x.shape[0]
    for t in (y, a, b, c):
        if t.shape != x.shape:
            raise SpinError("inconsistent operand shapes")
    if out is None:
        out = torch.empty_like(x)
    _check(lib().spin_beaver_and(n, x[0].numel(), _dev(x, "x"), _dev(y, "y"), _dev(a, "a"), _dev(b, "b"),
                                 _dev(c, "c"), _dev(out, "z"), _stream()))
    return out


def lincomb_trunc(terms, coefs, constant=0, f=0, tuple_=None, out=None):
    """out = Truncate(sum_j coefs[j] * terms[j] + constant, f); f = 0 leaves the sum untruncated."""
    n = terms[0].shape[0]
    for t in terms:
        if t.shape != terms[0].shape:
            raise SpinError("inconsistent operand shapes")
    if out is None:
        out = torch.empty_like(terms[0])
    ptrs = (ctypes.c_void_p * len(terms))(*[_dev(t, "term") for t in terms])
    cf = (ctypes.c_uint64 * len(terms))(*[int(c) % (1 << 64) for c in coefs])
    r = rt = rm = None
    if f > 0:
        r, rt, rm = (_dev(t, "tuple") for t in tuple_)
        for t in tuple_:
            if t.numel() != terms[0].numel():
                raise SpinError("truncation tuple must have the shape of the terms")
    _check(lib().spin_lincomb_trunc(n, terms[0][0].numel(), len(terms), ptrs, cf, int(constant) % (1 << 64), f,
                                    r, rt, rm, _dev(out, "out"), _stream()))
    return out


class ring128:
    """The same calls over Z_2^128.  A ring tensor of shape S is a torch.int64 tensor of shape S + (2,):
    two 64-bit words per element, low word first."""

    @staticmethod
    def _elems(t):
        if t.shape[-1] != 2:
            raise SpinError("128-bit ring tensors carry a trailing axis of 2 words")
        return t.numel() // 2

    @staticmethod
    def share(x, n, seed, stream_id, out=None):
        if out is None:
            out = torch.empty((n,) + tuple(x.shape), dtype=torch.int64, device=x.device)
        _check(lib().spin128_share(_dev(x, "x"), ring128._elems(x), n, seed, stream_id, _dev(out, "shares"), _stream()))
        return out

    @staticmethod
    def open(shares, mask=None, out=None):  # noqa: A003
        n = shares.shape[0]
        if out is None:
            out = torch.empty(tuple(shares.shape[1:]), dtype=torch.int64, device=shares.device)
        _check(lib().spin128_open(_dev(shares, "shares"), None if mask is None else _dev(mask, "mask"),
                                  ring128._elems(out), n, _dev(out, "out"), _stream()))
        return out

    @staticmethod
    def beaver_matmul_workspace_bytes(n, batch, M, N, K, path=LIMB_MFMA):
        return int(lib().spin128_beaver_matmul_workspace_bytes(n, batch, M, N, K, path))

    @staticmethod
    def beaver_matmul(X, Y, A, B, C, path=LIMB_MFMA, out=None, workspace=None):
        n, batch, M, K, _ = X.shape
        N = Y.shape[3]
        if tuple(Y.shape) != (n, batch, K, N, 2) or A.shape != X.shape or B.shape != Y.shape \
                or tuple(C.shape) != (n, batch, M, N, 2):
            raise SpinError("inconsistent operand shapes")
        if out is None:
            out = torch.empty_like(C)
        need = ring128.beaver_matmul_workspace_bytes(n, batch, M, N, K, path)
        if need == 0:
            raise SpinError("invalid matmul dimensions")
        if workspace is None:
            workspace = torch.empty(need, dtype=torch.uint8, device=X.device)
        _check(lib().spin128_beaver_matmul(n, batch, M, N, K, _dev(X, "X"), _dev(Y, "Y"), _dev(A, "A"), _dev(B, "B"),
                                           _dev(C, "C"), _dev(out, "Z"), path, workspace.data_ptr(),
                                           workspace.numel() * workspace.element_size(), _stream()))
        return out

    @staticmethod
    def beaver_mul(x, y, a, b, c, out=None):
        n = x.shape[0]
        if out is None:
            out = torch.empty_like(x)
        _check(lib().spin128_beaver_mul(n, ring128._elems(x[0]), _dev(x, "x"), _dev(y, "y"), _dev(a, "a"),
                                        _dev(b, "b"), _dev(c, "c"), _dev(out, "z"), _stream()))
        return out

    @staticmethod
    def trunc(x, r, r_top, r_msb, f, out=None):
        n = x.shape[0]
        if out is None:
            out = torch.empty_like(x)
        _check(lib().spin128_trunc(n, ring128._elems(x[0]), f, _dev(x, "x"), _dev(r, "r"), _dev(r_top, "r_top"),
                                   _dev(r_msb, "r_msb"), _dev(out, "out"), _stream()))
        return out


def _dev32(t, name):
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.dtype == torch.int32 and t.is_contiguous()):
        raise SpinError("%s must be a contiguous torch.int32 CUDA tensor" % name)
    return t.data_ptr()


class ring32:
    """The same calls over Z_2^32 (the Fixed32 representation of Section 7.1).  Ring tensors are
    torch.int32 CUDA tensors (the bit pattern of a uint32 ring element), party-major."""

    @staticmethod
    def cast_from_64(shares, out=None):
        """Local Fixed64 -> Fixed32 cast: every party keeps the low half of its own share."""
        if out is None:
            out = torch.empty(tuple(shares.shape), dtype=torch.int32, device=shares.device)
        _check(lib().spin_cast_64_to_32(_dev(shares, "shares"), shares.numel(), _dev32(out, "out"), _stream()))
        return out

    @staticmethod
    def share(x, n, seed, stream_id, out=None):
        if out is None:
            out = torch.empty((n,) + tuple(x.shape), dtype=torch.int32, device=x.device)
        _check(lib().spin32_share(_dev32(x, "x"), x.numel(), n, seed, stream_id, _dev32(out, "shares"), _stream()))
        return out

    @staticmethod
    def open(shares, mask=None, out=None):  # noqa: A003
        n = shares.shape[0]
        if out is None:
            out = torch.empty(tuple(shares.shape[1:]), dtype=torch.int32, device=shares.device)
        if mask is not None and mask.shape != shares.shape:
            raise SpinError("mask must have the shape of shares")
        _check(lib().spin32_open(_dev32(shares, "shares"), None if mask is None else _dev32(mask, "mask"),
                                 out.numel(), n, _dev32(out, "out"), _stream()))
        return out

    @staticmethod
    def beaver_matmul_workspace_bytes(n, batch, M, N, K, path=LIMB_MFMA):
        return int(lib().spin32_beaver_matmul_workspace_bytes(n, batch, M, N, K, path))

    @staticmethod
    def beaver_matmul(X, Y, A, B, C, path=LIMB_MFMA, out=None, workspace=None):
        n, batch, M, K = X.shape
        N = Y.shape[3]
        if tuple(Y.shape) != (n, batch, K, N) or A.shape != X.shape or B.shape != Y.shape \
                or tuple(C.shape) != (n, batch, M, N):
            raise SpinError("inconsistent operand shapes")
        if out is None:
            out = torch.empty_like(C)
        need = ring32.beaver_matmul_workspace_bytes(n, batch, M, N, K, path)
        if need == 0:
            raise SpinError("invalid matmul dimensions")
        if workspace is None:
            workspace = torch.empty(need, dtype=torch.uint8, device=X.device)
        _check(lib().spin32_beaver_matmul(n, batch, M, N, K, _dev32(X, "X"), _dev32(Y, "Y"), _dev32(A, "A"),
                                          _dev32(B, "B"), _dev32(C, "C"), _dev32(out, "Z"), path,
                                          workspace.data_ptr(), workspace.numel() * workspace.element_size(),
                                          _stream()))
        return out

    @staticmethod
    def beaver_mul(x, y, a, b, c, out=None):
        n = x.shape[0]
        if out is None:
            out = torch.empty_like(x)
        _check(lib().spin32_beaver_mul(n, x[0].numel(), _dev32(x, "x"), _dev32(y, "y"), _dev32(a, "a"),
                                       _dev32(b, "b"), _dev32(c, "c"), _dev32(out, "z"), _stream()))
        return out

    @staticmethod
    def trunc(x, r, r_top, r_msb, f, out=None):
        n = x.shape[0]
        if out is None:
            out = torch.empty_like(x)
        _check(lib().spin32_trunc(n, x[0].numel(), f, _dev32(x, "x"), _dev32(r, "r"), _dev32(r_top, "r_top"),
                                  _dev32(r_msb, "r_msb"), _dev32(out, "out"), _stream()))
        return out


KERNELS = {"random": 0, "share": 1, "open": 2, "beaver_mul": 3, "trunc": 4, "pack": 5, "gemm_limb": 6,
           "gemm_valu": 7, "lincomb": 8, "binary": 9, "cast": 10, "probe": 11, "beaver_mul_trunc": 12}


def probe_mfma(operands, blocks, iters, sink=None):
    """Register-only int8 MFMA loop on the 24 operand fragments in `operands` ([24*128] int64); returns sink."""
    if operands.numel() != 24 * 128:
        raise SpinError("operands must hold 24 fragments of 128 words")
    if sink is None:
        sink = torch.empty(blocks * 256, dtype=torch.int64, device=operands.device)
    _check(lib().spin_probe_mfma(_dev(operands, "operands"), blocks, iters, _dev(sink, "sink"), _stream()))
    return sink


PROBE_OPS_PER_WAVE_ITERATION = 72 * 65536      # 72 MFMAs of 32x32x32 multiply-adds, two operations each


def profile_enable(on=True):
    lib().spin_profile_enable(1 if on else 0)


def profile_reset():
    lib().spin_profile_reset()


def profile_read(kernel):
    """(total milliseconds, launches) of one kernel class since the last reset; waits for the events."""
    ms, cnt = ctypes.c_double(0.0), ctypes.c_uint(0)
    _check(lib().spin_profile_read(KERNELS[kernel], ctypes.byref(ms), ctypes.byref(cnt)))
    return ms.value, cnt.value


# Fixed-point encoding of Section 4.1 (host-side convenience for the harness; not part of the C ABI).
def encode(x, f):
    """float64 tensor -> ring tensor holding floor(x * 2^f)."""
    return torch.floor(torch.ldexp(x.to(torch.float64), torch.tensor(f))).to(torch.int64)


def decode(u, f):
    return torch.ldexp(u.to(torch.float64), torch.tensor(-f))
