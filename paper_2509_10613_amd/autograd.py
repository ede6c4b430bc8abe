"""PyTorch autograd over the C ABI (Section 1 states that the paper's library takes part in PyTorch's automatic
differentiation): thin ``torch.autograd.Function`` wrappers whose forward is ``sigkernel_fwd`` /
``sigkernel_gram`` and whose backward is ``sigkernel_bwd`` / ``sigkernel_gram`` with the upstream gradient
(Section 3.4: exact gradients of the discrete scheme).  Argument marshalling only; no arithmetic of the
method happens here.

    k = sig_kernel(x, y, lam1, lam2, flags)          # x[B,L1,d], y[B,L2,d] -> k[B]
    K = sig_kernel_gram(X, Y, lam1, lam2, flags)     # X[N,L1,d], Y[M,L2,d] -> K[N,M]
    K = sig_kernel_gram(X, None, lam1, lam2, flags)  # symmetric case K(X, X)
    loss = sig_mmd2(X, Y, lam1, lam2, flags)         # squared MMD between two sets of paths, one library call
    S = signature(x, N, flags)                       # x[B,L,d] -> truncated signatures [B, entries] (Section 2)

A time grid of the caller's own (Section 4 defines the time-augmented path as (x_{t_i}, t_i) and fixes no grid; the
library's flag takes t_i = i/(L-1)) is an ordinary channel: ``with_times(x, t)`` appends it, and the wrappers below take
``times=`` / ``times_x=, times_y=`` and do that for the caller.

The gradients are first-order only (the backward pass is not itself differentiable).
"""
import torch

from . import binding as sk


_KEEP_LIMIT = 1 << 30   # bytes of workspace a forward call may hold on to for its backward call


class _PairKernel(torch.autograd.Function):
    @staticmethod
    def forward(ctx, x, y, lam1, lam2, flags):
        x = x.contiguous()
        y = y.contiguous()
        ctx.save_for_backward(x, y)
        ctx.args = (lam1, lam2, flags)
        ctx.ws = None
        # Where the launch mode can hand its forward sweep to the backward call, this call keeps it in a workspace of
        # its own, which lives until the graph is freed (the grid the paper's backward pass takes over from its
        # forward pass, here as checkpoints).
        B, L1, d = x.shape
        if (ctx.needs_input_grad[0] or ctx.needs_input_grad[1]) and sk.keeps_forward(B, L1, y.shape[1], d, lam1, lam2,
                                                                                     flags, sk._dt(x)):
            need = sk.sigkernel_workspace_bytes(sk.SK_OP_FWD, B, 0, L1, y.shape[1], d, lam1, lam2,
                                                flags | sk.SK_FLAG_KEEP_FORWARD, sk._dt(x))
            if need <= _KEEP_LIMIT:    # large batches of pairs would pin gigabytes per live graph: they sweep twice
                ctx.ws = torch.empty(max(int(need), 256), dtype=torch.uint8, device=x.device)
                return sk.sigkernel_fwd(x, y, lam1, lam2, flags | sk.SK_FLAG_KEEP_FORWARD, ws=ctx.ws)
        return sk.sigkernel_fwd(x, y, lam1, lam2, flags)

    @staticmethod
    def backward(ctx, grad_k):
        x, y = ctx.saved_tensors
        lam1, lam2, flags = ctx.args
        want_x, want_y = ctx.needs_input_grad[0], ctx.needs_input_grad[1]
        if not (want_x or want_y):
            return None, None, None, None, None
        if ctx.ws is not None:
            _, gx, gy = sk.sigkernel_bwd(x, y, grad_k.contiguous(), lam1, lam2, flags | sk.SK_FLAG_HAVE_FORWARD,
                                         want_x=want_x, want_y=want_y, ws=ctx.ws)
        else:
            _, gx, gy = sk.sigkernel_bwd(x, y, grad_k.contiguous(), lam1, lam2, flags, want_x=want_x, want_y=want_y)
        return gx, gy, None, None, None


def _gram_keep_workspace(ctx, X, Y, lam1, lam2, flags):
    """A workspace of this call's own if it wants gradients, the launch mode can keep the forward sweep of a Gram matrix
    for its backward call, and that costs no more than _KEEP_LIMIT bytes; else None."""
    if not any(ctx.needs_input_grad[:2]):
        return None
    N, L1, d = X.shape
    M, L2 = Y.shape[0], Y.shape[1]
    if not sk.keeps_forward(N, L1, L2, d, lam1, lam2, flags, sk._dt(X), gram_M=M):
        return None
    need = sk.sigkernel_workspace_bytes(sk.SK_OP_GRAM, N, M, L1, L2, d, lam1, lam2, flags | sk.SK_FLAG_KEEP_FORWARD,
                                        sk._dt(X))
    if need > _KEEP_LIMIT:
        return None
    return torch.empty(max(int(need), 256), dtype=torch.uint8, device=X.device)


class _GramKernel(torch.autograd.Function):
    @staticmethod
    def forward(ctx, X, Y, lam1, lam2, flags):
        X = X.contiguous()
        Y = Y.contiguous()
        ctx.save_for_backward(X, Y)
        ctx.args = (lam1, lam2, flags)
        ctx.ws = _gram_keep_workspace(ctx, X, Y, lam1, lam2, flags)
        if ctx.ws is not None:
            return sk.sigkernel_gram(X, Y, None, lam1, lam2, flags | sk.SK_FLAG_KEEP_FORWARD, ws=ctx.ws)
        return sk.sigkernel_gram(X, Y, None, lam1, lam2, flags)

    @staticmethod
    def backward(ctx, grad_K):
        X, Y = ctx.saved_tensors
        lam1, lam2, flags = ctx.args
        if ctx.ws is not None:
            _, gX, gY = sk.sigkernel_gram(X, Y, grad_K.contiguous(), lam1, lam2, flags | sk.SK_FLAG_HAVE_FORWARD, ws=ctx.ws)
        else:
            _, gX, gY = sk.sigkernel_gram(X, Y, grad_K.contiguous(), lam1, lam2, flags)
        return (gX if ctx.needs_input_grad[0] else None), (gY if ctx.needs_input_grad[1] else None), None, None, None


class _GramKernelSym(torch.autograd.Function):
    @staticmethod
    def forward(ctx, X, lam1, lam2, flags):
        X = X.contiguous()
        ctx.save_for_backward(X)
        ctx.args = (lam1, lam2, flags)
        ctx.ws = _gram_keep_workspace(ctx, X, X, lam1, lam2, flags)
        if ctx.ws is not None:
            return sk.sigkernel_gram(X, X, None, lam1, lam2, flags | sk.SK_FLAG_KEEP_FORWARD, ws=ctx.ws)
        return sk.sigkernel_gram(X, X, None, lam1, lam2, flags)

    @staticmethod
    def backward(ctx, grad_K):
        (X,) = ctx.saved_tensors
        lam1, lam2, flags = ctx.args
        keep = sk.SK_FLAG_HAVE_FORWARD if ctx.ws is not None else 0
        _, gX, _ = sk.sigkernel_gram(X, X, grad_K.contiguous(), lam1, lam2, flags | keep, ws=ctx.ws)   # total derivative
        return gX, None, None, None


class _Mmd2(torch.autograd.Function):
    @staticmethod
    def forward(ctx, X, Y, lam1, lam2, flags):
        X = X.contiguous()
        Y = Y.contiguous()
        want_x, want_y = ctx.needs_input_grad[0], ctx.needs_input_grad[1]
        loss, gX, gY = sk.sigkernel_mmd2(X, Y, lam1, lam2, flags, want_x=want_x, want_y=want_y)
        ctx.save_for_backward(*[g for g in (gX, gY) if g is not None])
        ctx.have = (gX is not None, gY is not None)
        return loss[0]

    @staticmethod
    def backward(ctx, grad_loss):
        saved = list(ctx.saved_tensors)
        gX = saved.pop(0) if ctx.have[0] else None
        gY = saved.pop(0) if ctx.have[1] else None
        return (None if gX is None else gX * grad_loss), (None if gY is None else gY * grad_loss), None, None, None


class _Signature(torch.autograd.Function):
    @staticmethod
    def forward(ctx, x, N, flags):
        x = x.contiguous()
        out = sk.signature_fwd(x, N, flags)
        ctx.save_for_backward(x, out)
        ctx.args = (N, flags)
        return out

    @staticmethod
    def backward(ctx, grad_out):
        x, out = ctx.saved_tensors
        N, flags = ctx.args
        return sk.signature_bwd(x, grad_out.contiguous(), N, flags, sig=out), None, None


def signature(x, N, flags=0, times=None):
    """Truncated signatures of device paths x[B,L,d] up to level N, levels 0..N flattened (signature_fwd);
    differentiable in x (signature_bwd, handed the signatures of the forward call).  times: a time grid of the
    caller's own, appended as the last channel."""
    if times is not None:
        x = with_times(x, times)
    return _Signature.apply(x, N, flags)


def with_times(x, t):
    """x[..., L, d] with the channel t appended: t[L] (one grid for every path) or t[..., L]."""
    t = torch.as_tensor(t, dtype=x.dtype, device=x.device)
    t = t.expand(x.shape[:-1]) if t.dim() == 1 else t
    return torch.cat([x, t.unsqueeze(-1)], dim=-1)


def sig_mmd2(X, Y, lam1=0, lam2=0, flags=0):
    """mean K(X,X) - 2 mean K(X,Y) + mean K(Y,Y) for device tensors X[N,L1,d], Y[M,L2,d] (sigkernel_mmd2: value and
    gradients in one call, the upstream weights never leave the GPU); differentiable in X and Y."""
    return _Mmd2.apply(X, Y, lam1, lam2, flags)


def sig_kernel(x, y, lam1=0, lam2=0, flags=0, times_x=None, times_y=None):
    """k[b] = k(x[b], y[b]) for device tensors x[B,L1,d], y[B,L2,d]; differentiable in x and y.  times_x, times_y: time
    grids of the caller's own (both or neither), appended as the last channel of each side."""
    if (times_x is None) != (times_y is None):
        raise ValueError("give time grids for both sides or for neither")
    if times_x is not None:
        x, y = with_times(x, times_x), with_times(y, times_y)
    return _PairKernel.apply(x, y, lam1, lam2, flags)


def sig_kernel_gram(X, Y=None, lam1=0, lam2=0, flags=0, times_x=None, times_y=None):
    """K[n,m] = k(X[n], Y[m]); Y = None is the symmetric case K(X, X); differentiable in X and Y.  times_x (and times_y
    when Y is given): time grids of the caller's own, appended as the last channel."""
    if times_x is not None:
        X = with_times(X, times_x)
        if Y is not None:
            if times_y is None:
                raise ValueError("give time grids for both sides or for neither")
            Y = with_times(Y, times_y)
    elif times_y is not None:
        raise ValueError("give time grids for both sides or for neither")
    if Y is None:
        return _GramKernelSym.apply(X, lam1, lam2, flags)
    return _GramKernel.apply(X, Y, lam1, lam2, flags)
