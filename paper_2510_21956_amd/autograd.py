"""torch.autograd wrapper over the C ABI (the paper's plug-and-play module, Sec. 6).

Plumbing only: it allocates the outputs, the workspaces and the hand-over buffer with
torch, keeps the set {Q, K, V, O, g} of Sec. 3.2 (plus the forward pass's running sums at
the segment boundaries) for the backward pass, and calls la_forward_save /
la_backward_saved.  Every arithmetic step runs in the HIP library; there is no fallback.
Gradients are with respect to the Q, K, V handed in; with ``normalize_qk`` the rows of Q and
K are scaled to unit length inside the kernels (Sec. 3.3) and the gradients are those for the
raw rows.  a and b are constants.
"""
import torch

from . import binding as _b


def _code(t):
    return _b.LA_F32 if t.dtype == torch.float32 else _b.LA_BF16


def _bytes(n, device):
    return torch.empty(max(int(n), 256), dtype=torch.uint8, device=device)


class LinearAttentionFunction(torch.autograd.Function):
    """O = LA(Q, K, V) with kernel f(x) = a + b x; Q, K, V: [B, H, N, D] device tensors."""

    @staticmethod
    def forward(ctx, Q, K, V, a, b, causal, normalize_qk=False):
        Q, K, V = Q.contiguous(), K.contiguous(), V.contiguous()
        B, H, N, D = Q.shape
        dt = _code(Q)
        O = torch.empty_like(Q)
        G = torch.empty((B, H, N), dtype=torch.float32, device=Q.device)
        ws = _bytes(_b.la_workspace_bytes(B, H, N, D, dt, causal, 0), Q.device)
        ns = _b.la_saved_state_bytes(B, H, N, D, dt, causal)
        saved = _bytes(ns, Q.device) if ns else None
        fwd = _b.la_forward_qknorm_save if normalize_qk else _b.la_forward_save
        fwd(Q, K, V, O, G, a, b, causal, ws, saved)
        ctx.save_for_backward(Q, K, V, O, G)
        ctx.la_saved = saved
        ctx.la_args = (float(a), float(b), bool(causal), bool(normalize_qk))
        return O

    @staticmethod
    def backward(ctx, dO):
        Q, K, V, O, G = ctx.saved_tensors
        a, b, causal, normalize_qk = ctx.la_args
        B, H, N, D = Q.shape
        dO = dO.contiguous()
        dQ, dK, dV = torch.empty_like(Q), torch.empty_like(Q), torch.empty_like(Q)
        ws = _bytes(_b.la_workspace_bytes(B, H, N, D, _code(Q), causal, 1), Q.device)
        bwd = _b.la_backward_qknorm_saved if normalize_qk else _b.la_backward_saved
        bwd(Q, K, V, O, G, dO, dQ, dK, dV, a, b, causal, ws, ctx.la_saved)
        return dQ, dK, dV, None, None, None, None


def linear_attention(Q, K, V, a=1.0, b=0.5, causal=True, normalize_qk=False):
    """Differentiable linear attention on [B, H, N, D] float32 or bfloat16 device tensors;
    ``normalize_qk`` scales the rows of Q and K to unit length inside the kernels (D <= 128)."""
    return LinearAttentionFunction.apply(Q, K, V, a, b, causal, normalize_qk)
