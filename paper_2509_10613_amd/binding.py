"""Thin ctypes binding of libsigkernel.so (the C ABI declared in include/sigkernel.h).

Argument marshalling only: every step of the method runs in the HIP kernels.  PyTorch is used for device
memory and streams.  There is no CPU fallback: if the library is missing, loading raises.
"""
import ctypes as C
import os

import torch

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libsigkernel.so")

SK_F32, SK_F64 = 0, 1
SK_FLAG_TIME_AUG = 1
SK_FLAG_BWD_REPLAY = 2
SK_FLAG_SHORT_WAITS = 4
SK_FLAG_LEAD_LAG = 8
SK_FLAG_KEEP_FORWARD = 16
SK_FLAG_HAVE_FORWARD = 32
SK_OP_FWD, SK_OP_BWD, SK_OP_GRAM, SK_OP_GRAM_BWD = 0, 1, 2, 3


def SK_SIG_BLOCK(s):
    """Diagnostic flag of the signature entry points: forces the letter block of a lane."""
    return s << 12


SK_SIG_ONE_PATH_PER_WAVE = 0x200000   # diagnostic flag of signature_fwd: a wave never holds more than one path


def SK_SIG_PIECES(q):
    """Diagnostic flag of signature_fwd: cut every path into 2^q pieces (q = 0: never)."""
    return (q + 1) << 16


def SK_SIG_DEPTH(m):
    """Diagnostic flag of signature_fwd: forces the depth of the register-resident subtree of a lane."""
    return (m + 1) << 8


EXPORTS = ["sigkernel_workspace_bytes", "sigkernel_fwd", "sigkernel_bwd", "sigkernel_bwd_static", "sigkernel_gram",
           "sigkernel_describe",
           "sigkernel_mmd2", "sigkernel_mmd2_workspace_bytes",
           "sigkernel_event_timing", "sigkernel_event_timing_read", "sigkernel_event_timing_read_tag", "sigkernel_last_error", "sigkernel_version",
           "signature_length", "signature_workspace_bytes", "signature_fwd", "signature_describe",
           "signature_bwd_workspace_bytes", "signature_bwd", "signature_bwd_describe"]

_lib = None


class SigKernelError(RuntimeError):
    pass


def load():
    """Load the built library (build it first with ``python -m paper_2509_10613_amd.build`` or
    ``__graft_entry__.build()``); raises if it is not there."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise SigKernelError("%s not found: build the HIP library first (python paper_2509_10613_amd/build.py)"
                             % LIB_PATH)
    lib = C.CDLL(LIB_PATH)
    i64, vp, ci = C.c_int64, C.c_void_p, C.c_int
    lib.sigkernel_workspace_bytes.restype = C.c_size_t
    lib.sigkernel_workspace_bytes.argtypes = [ci, i64, i64, i64, i64, i64, ci, ci, ci, ci]
    lib.sigkernel_describe.restype = ci
    lib.sigkernel_describe.argtypes = [ci, i64, i64, i64, i64, i64, ci, ci, ci, ci, C.c_char_p, C.c_size_t]
    lib.sigkernel_fwd.restype = ci
    lib.sigkernel_fwd.argtypes = [vp, vp, vp, i64, i64, i64, i64, ci, ci, ci, ci, vp, C.c_size_t, vp]
    lib.sigkernel_bwd.restype = ci
    lib.sigkernel_bwd.argtypes = [vp, vp, vp, vp, vp, vp, i64, i64, i64, i64, ci, ci, ci, ci, vp, C.c_size_t, vp]
    lib.sigkernel_bwd_static.restype = ci
    lib.sigkernel_bwd_static.argtypes = [vp, vp, vp, vp, vp, vp, i64, i64, i64, i64, ci, ci, ci, ci, vp]
    lib.sigkernel_gram.restype = ci
    lib.sigkernel_gram.argtypes = [vp, vp, vp, vp, vp, vp, i64, i64, i64, i64, i64, ci, ci, ci, ci, vp, C.c_size_t,
                                   vp]
    lib.sigkernel_mmd2_workspace_bytes.restype = C.c_size_t
    lib.sigkernel_mmd2_workspace_bytes.argtypes = [i64, i64, i64, i64, i64, ci, ci, ci, ci, ci]
    lib.sigkernel_mmd2.restype = ci
    lib.sigkernel_mmd2.argtypes = [vp, vp, vp, vp, vp, i64, i64, i64, i64, i64, ci, ci, ci, ci, vp, C.c_size_t, vp]
    lib.sigkernel_event_timing.restype = ci
    lib.sigkernel_event_timing.argtypes = [ci]
    lib.sigkernel_event_timing_read.restype = ci
    lib.sigkernel_event_timing_read.argtypes = [C.POINTER(C.c_double), C.POINTER(ci), C.POINTER(C.c_double),
                                                C.POINTER(ci)]
    lib.sigkernel_event_timing_read_tag.restype = ci
    lib.sigkernel_event_timing_read_tag.argtypes = [ci, C.POINTER(C.c_double), C.POINTER(ci), C.POINTER(C.c_double),
                                                    C.POINTER(ci)]
    lib.signature_length.restype = i64
    lib.signature_length.argtypes = [i64, ci, ci]
    lib.signature_workspace_bytes.restype = C.c_size_t
    lib.signature_workspace_bytes.argtypes = [i64, i64, i64, ci, ci, ci]
    lib.signature_fwd.restype = ci
    lib.signature_fwd.argtypes = [vp, vp, i64, i64, i64, ci, ci, ci, vp, C.c_size_t, vp]
    lib.signature_describe.restype = ci
    lib.signature_describe.argtypes = [i64, i64, i64, ci, ci, ci, C.c_char_p, C.c_size_t]
    lib.signature_bwd_describe.restype = ci
    lib.signature_bwd_describe.argtypes = [i64, i64, i64, ci, ci, ci, C.c_char_p, C.c_size_t]
    lib.signature_bwd_workspace_bytes.restype = C.c_size_t
    lib.signature_bwd_workspace_bytes.argtypes = [i64, i64, i64, ci, ci, ci, ci]
    lib.signature_bwd.restype = ci
    lib.signature_bwd.argtypes = [vp, vp, vp, vp, i64, i64, i64, ci, ci, ci, vp, C.c_size_t, vp]
    lib.sigkernel_last_error.restype = C.c_char_p
    lib.sigkernel_version.restype = C.c_char_p
    _lib = lib
    return lib


def _dt(t):
    if t.dtype == torch.float64:
        return SK_F64
    if t.dtype == torch.float32:
        return SK_F32
    raise TypeError("float32 or float64 tensors expected, got %s" % t.dtype)


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def _check(rc):
    if rc != 0:
        raise SigKernelError("sigkernel error %d: %s" % (rc, load().sigkernel_last_error().decode()))


def _dev(t, name):
    if not (t.is_cuda and t.is_contiguous()):
        raise ValueError("%s must be a contiguous device tensor" % name)
    return t


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def sigkernel_workspace_bytes(op, B_or_N, M, L1, L2, d, lam1, lam2, flags, dt):
    return int(load().sigkernel_workspace_bytes(op, B_or_N, M, L1, L2, d, lam1, lam2, flags, dt))


def sigkernel_describe(op, B_or_N, M, L1, L2, d, lam1, lam2, flags, dt):
    """The launch the library would make for this operation and shape, as 'key=value' text (no GPU call)."""
    buf = C.create_string_buffer(512)
    _check(load().sigkernel_describe(op, B_or_N, M, L1, L2, d, lam1, lam2, flags, dt, buf, len(buf)))
    return buf.value.decode()


def sigkernel_event_timing(enable):
    """False / 0: off; True or a positive tag: on, launches are recorded under that tag."""
    _check(load().sigkernel_event_timing(int(enable)))


def sigkernel_event_timing_read(tag=0):
    """Returns (fwd_ms, fwd_launches, bwd_ms, bwd_launches) summed since the last read (tag > 0: of the launches
    recorded under that tag only)."""
    f, b = C.c_double(0), C.c_double(0)
    nf, nb = C.c_int(0), C.c_int(0)
    _check(load().sigkernel_event_timing_read_tag(int(tag), C.byref(f), C.byref(nf), C.byref(b), C.byref(nb)))
    return f.value, nf.value, b.value, nb.value


_ws_cache = {}


def workspace(nbytes, device):
    """A cached, 256-byte aligned scratch tensor of at least nbytes on `device` for calls on the current stream
    (grown on demand; one per device and stream: calls that share a workspace must be ordered)."""
    key = (str(device), torch.cuda.current_stream(device).cuda_stream)
    t = _ws_cache.get(key)
    if t is None or t.numel() < nbytes:
        t = torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)
        _ws_cache[key] = t
    return t


def keeps_forward(B, L1, L2, d, lam1, lam2, flags, dt, gram_M=None):
    """Whether sigkernel_fwd (gram_M = M: sigkernel_gram on B x M paths) with SK_FLAG_KEEP_FORWARD leaves a sweep that
    the backward call with SK_FLAG_HAVE_FORWARD takes over for this shape (the launch plan names the first half of the
    backward pass), or ignores the flag."""
    if B < 1 or L1 < 2 or L2 < 2 or (gram_M is not None and gram_M < 1):
        return False
    if gram_M is None:
        desc = sigkernel_describe(SK_OP_FWD, B, 0, L1, L2, d, lam1, lam2, flags | SK_FLAG_KEEP_FORWARD, dt)
    else:
        desc = sigkernel_describe(SK_OP_GRAM, B, gram_M, L1, L2, d, lam1, lam2, flags | SK_FLAG_KEEP_FORWARD, dt)
    return " kept_sweep_half=1 " in desc


def sigkernel_fwd(x, y, lam1=0, lam2=0, flags=0, k=None, ws=None):
    """x[B,L1,d], y[B,L2,d] -> k[B] (device tensors)."""
    _dev(x, "x"); _dev(y, "y")
    B, L1, d = x.shape
    L2 = y.shape[1]
    assert y.shape[0] == B and y.shape[2] == d and y.dtype == x.dtype
    dt = _dt(x)
    if k is None:
        k = torch.empty((B,), dtype=x.dtype, device=x.device)
    need = sigkernel_workspace_bytes(SK_OP_FWD, B, 0, L1, L2, d, lam1, lam2, flags, dt)
    if ws is None:
        ws = workspace(need, x.device)
    _check(load().sigkernel_fwd(_ptr(x), _ptr(y), _ptr(k), B, L1, L2, d, lam1, lam2, flags, dt, _ptr(ws),
                                ws.numel(), _stream()))
    return k


def sigkernel_bwd(x, y, grad_k, lam1=0, lam2=0, flags=0, grad_x=None, grad_y=None, k_out=None, ws=None,
                  want_x=True, want_y=True):
    """Returns (k[B], grad_x[B,L1,d], grad_y[B,L2,d]) for upstream gradients grad_k[B]."""
    _dev(x, "x"); _dev(y, "y"); _dev(grad_k, "grad_k")
    B, L1, d = x.shape
    L2 = y.shape[1]
    assert y.shape[0] == B and y.shape[2] == d and y.dtype == x.dtype and grad_k.dtype == x.dtype
    dt = _dt(x)
    if grad_x is None and want_x:
        grad_x = torch.empty_like(x)
    if grad_y is None and want_y:
        grad_y = torch.empty_like(y)
    if k_out is None:
        k_out = torch.empty((B,), dtype=x.dtype, device=x.device)
    need = sigkernel_workspace_bytes(SK_OP_BWD, B, 0, L1, L2, d, lam1, lam2, flags, dt)
    if ws is None:
        ws = workspace(need, x.device)
    _check(load().sigkernel_bwd(_ptr(x), _ptr(y), _ptr(grad_k), _ptr(grad_x), _ptr(grad_y), _ptr(k_out), B, L1, L2,
                                d, lam1, lam2, flags, dt, _ptr(ws), ws.numel(), _stream()))
    return k_out, grad_x, grad_y


SK_STATIC_SCRATCH_BYTES = 64 << 20


def sigkernel_bwd_static(x, y, grad_k, grad_x, grad_y, k_out, lam1=0, lam2=0, flags=0):
    """sigkernel_bwd with the library's own per-device scratch: the caller passes every output, nothing is allocated."""
    _dev(x, "x"); _dev(y, "y"); _dev(grad_k, "grad_k")
    B, L1, d = x.shape
    L2 = y.shape[1]
    assert y.shape[0] == B and y.shape[2] == d and y.dtype == x.dtype and grad_k.dtype == x.dtype
    _check(load().sigkernel_bwd_static(_ptr(x), _ptr(y), _ptr(grad_k), _ptr(grad_x), _ptr(grad_y), _ptr(k_out), B, L1,
                                       L2, d, lam1, lam2, flags, _dt(x), _stream()))
    return k_out, grad_x, grad_y


def sigkernel_gram(X, Y, grad_K=None, lam1=0, lam2=0, flags=0, K=None, grad_X=None, grad_Y=None, ws=None):
    """K[N,M] = k(X[n], Y[m]); with grad_K also (grad_X, grad_Y).  Passing the same tensor for X and Y
    selects the symmetric case (grad_X is the total derivative, grad_Y is None)."""
    _dev(X, "X"); _dev(Y, "Y")
    N, L1, d = X.shape
    M, L2, d2 = Y.shape
    assert d2 == d and Y.dtype == X.dtype
    sym = Y.data_ptr() == X.data_ptr()
    dt = _dt(X)
    if K is None:
        K = torch.empty((N, M), dtype=X.dtype, device=X.device)
    backward = grad_K is not None
    if backward:
        _dev(grad_K, "grad_K")
        assert grad_K.shape == (N, M) and grad_K.dtype == X.dtype
        if grad_X is None:
            grad_X = torch.empty_like(X)
        if grad_Y is None and not sym:
            grad_Y = torch.empty_like(Y)
    need = sigkernel_workspace_bytes(SK_OP_GRAM_BWD if backward else SK_OP_GRAM, N, M, L1, L2, d, lam1, lam2, flags,
                                     dt)
    if ws is None:
        ws = workspace(need, X.device)
    _check(load().sigkernel_gram(_ptr(X), _ptr(Y), _ptr(K), _ptr(grad_K), _ptr(grad_X), _ptr(grad_Y), N, M, L1, L2,
                                 d, lam1, lam2, flags, dt, _ptr(ws), ws.numel(), _stream()))
    if backward:
        return K, grad_X, grad_Y
    return K


def sigkernel_mmd2(X, Y, lam1=0, lam2=0, flags=0, want_x=True, want_y=True, ws=None):
    """Squared MMD between the path sets X[N,L1,d] and Y[M,L2,d] under the signature kernel.
    Returns (loss[1], grad_X or None, grad_Y or None)."""
    _dev(X, "X"); _dev(Y, "Y")
    N, L1, d = X.shape
    M, L2, d2 = Y.shape
    assert d2 == d and Y.dtype == X.dtype
    dt = _dt(X)
    loss = torch.empty((1,), dtype=X.dtype, device=X.device)
    gX = torch.empty_like(X) if want_x else None
    gY = torch.empty_like(Y) if want_y else None
    need = int(load().sigkernel_mmd2_workspace_bytes(N, M, L1, L2, d, lam1, lam2, flags, dt, 1 if (want_x or want_y) else 0))
    if ws is None:
        ws = workspace(need, X.device)
    _check(load().sigkernel_mmd2(_ptr(X), _ptr(Y), _ptr(loss), _ptr(gX), _ptr(gY), N, M, L1, L2, d, lam1, lam2, flags,
                                 dt, _ptr(ws), ws.numel(), _stream()))
    return loss, gX, gY


# ---------------------------------------------------------------- truncated signatures (include/signature.h)
def signature_length(d, N, flags=0):
    return int(load().signature_length(d, N, flags))


def signature_workspace_bytes(B, L, d, N, flags, dt):
    return int(load().signature_workspace_bytes(B, L, d, N, flags, dt))


def signature_describe(B, L, d, N, flags, dt):
    buf = C.create_string_buffer(512)
    _check(load().signature_describe(B, L, d, N, flags, dt, buf, len(buf)))
    return buf.value.decode()


def signature_fwd(x, N, flags=0, ws=None, out=None):
    """x[B,L,d] (device) -> out[B, signature_length(d, N, flags)]: truncated signatures, levels 0..N flattened."""
    _dev(x, "x")
    B, L, d = x.shape
    dt = _dt(x)
    n = signature_length(d, N, flags)
    if out is None:
        out = torch.empty((B, n), dtype=x.dtype, device=x.device)
    need = signature_workspace_bytes(B, L, d, N, flags, dt)
    if ws is None:
        ws = workspace(need, x.device)
    _check(load().signature_fwd(_ptr(x), _ptr(out), B, L, d, N, flags, dt, _ptr(ws), ws.numel(), _stream()))
    return out


def signature_bwd_describe(B, L, d, N, flags, dt):
    buf = C.create_string_buffer(512)
    _check(load().signature_bwd_describe(B, L, d, N, flags, dt, buf, len(buf)))
    return buf.value.decode()


def signature_bwd(x, grad_out, N, flags=0, sig=None, ws=None, grad_x=None):
    """dF/dx [B,L,d] for upstream gradients grad_out[B, signature_length(d, N, flags)]; sig = signature_fwd(x, N, flags)
    if the caller has it, else it is recomputed inside."""
    _dev(x, "x"); _dev(grad_out, "grad_out")
    B, L, d = x.shape
    dt = _dt(x)
    n = signature_length(d, N, flags)
    if n == 0:
        signature_bwd_describe(B, L, d, N, flags, dt)   # raises with the library's message for these arguments
    assert grad_out.shape == (B, n) and grad_out.dtype == x.dtype
    if sig is not None:
        _dev(sig, "sig")
        assert sig.shape == (B, n) and sig.dtype == x.dtype
    if grad_x is None:
        grad_x = torch.empty_like(x)
    need = int(load().signature_bwd_workspace_bytes(B, L, d, N, flags, dt, 0 if sig is None else 1))
    if ws is None:
        ws = workspace(need, x.device)
    _check(load().signature_bwd(_ptr(x), _ptr(sig), _ptr(grad_out), _ptr(grad_x), B, L, d, N, flags, dt, _ptr(ws),
                                ws.numel(), _stream()))
    return grad_x
