"""Helpers for the GPU parity tests: upload seeded inputs, call the C ABI through
the Python binding, compare against the fp64 oracle."""
import numpy as np
import torch

import la_workloads as wl

TOL = {"f32": 1e-4, "bf16": 2e-2}


def to_device(bits, dtype):
    """numpy input bits (float32 array or uint16 bf16 patterns) -> device tensor."""
    if dtype == "f32":
        return torch.from_numpy(np.ascontiguousarray(bits)).cuda()
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).cuda().view(torch.bfloat16)


def to_f64(t):
    return t.detach().to(torch.float64).cpu().numpy()


def torch_dtype(dtype):
    return torch.float32 if dtype == "f32" else torch.bfloat16


def excess(x_gpu, x_ref, tol, floor=0.0):
    """max over elements of |gpu - ref| / (tol * (|ref| + rms(ref)) + floor); passes if <= 1.

    Element-wise relative error is unbounded where the reference crosses zero,
    so each element is allowed tol times (its own magnitude + the tensor's rms).
    ``floor`` is an absolute allowance for the one degenerate case whose exact
    result is identically zero (N = 1: dQ = dK = 0), where the reference has no
    scale of its own."""
    x_ref = np.asarray(x_ref, dtype=np.float64)
    x_gpu = np.asarray(x_gpu, dtype=np.float64)
    if x_ref.size == 0:
        return 0.0
    if not np.all(np.isfinite(x_gpu)):
        return float("inf")
    rms = float(np.sqrt(np.mean(x_ref * x_ref)))
    bound = tol * (np.abs(x_ref) + rms) + floor
    bound = np.maximum(bound, 1e-300)
    return float(np.max(np.abs(x_gpu - x_ref) / bound))


def _dt(la, Q):
    return la.LA_F32 if Q.dtype == torch.float32 else la.LA_BF16


def scratch(nbytes, device):
    """A workspace / hand-over buffer filled with 0xFF (NaN patterns), so that a kernel
    that reads a part of it nobody wrote shows up in the results."""
    return torch.full((max(int(nbytes), 256),), 0xFF, dtype=torch.uint8, device=device)


def gpu_forward(la, dev, a, b, causal):
    """dev: dict of device tensors Q, K, V [B,H,N,D].  Returns O, G (poisoned first,
    so that rows the kernels fail to write are caught)."""
    Q, K, V = dev["Q"], dev["K"], dev["V"]
    B, H, N, D = Q.shape
    O = torch.full_like(Q, float("nan"))
    G = torch.full((B, H, N), float("nan"), dtype=torch.float32, device=Q.device)
    wf = scratch(la.la_workspace_bytes(B, H, N, D, _dt(la, Q), causal, 0), Q.device)
    la.la_forward(Q, K, V, O, G, a, b, causal, wf)
    torch.cuda.synchronize()
    return O, G


def gpu_backward(la, dev, O, G, a, b, causal):
    """Returns dQ, dK, dV for the saved set (Q, K, V, O, G) and upstream gradient dO."""
    Q, K, V, dO = dev["Q"], dev["K"], dev["V"], dev["dO"]
    B, H, N, D = Q.shape
    dQ, dK, dV = (torch.full_like(Q, float("nan")) for _ in range(3))
    wb = scratch(la.la_workspace_bytes(B, H, N, D, _dt(la, Q), causal, 1), Q.device)
    la.la_backward(Q, K, V, O, G, dO, dQ, dK, dV, a, b, causal, wb)
    torch.cuda.synchronize()
    return dQ, dK, dV


def gpu_forward_save(la, dev, a, b, causal):
    """la_forward_save: O, G and the hand-over buffer for la_backward_saved (None when the
    library uses none for this problem).  The buffer is poisoned first."""
    Q, K, V = dev["Q"], dev["K"], dev["V"]
    B, H, N, D = Q.shape
    O = torch.full_like(Q, float("nan"))
    G = torch.full((B, H, N), float("nan"), dtype=torch.float32, device=Q.device)
    wf = scratch(la.la_workspace_bytes(B, H, N, D, _dt(la, Q), causal, 0), Q.device)
    nb = la.la_saved_state_bytes(B, H, N, D, _dt(la, Q), causal)
    saved = scratch(nb, Q.device) if nb else None
    la.la_forward_save(Q, K, V, O, G, a, b, causal, wf, saved)
    torch.cuda.synchronize()
    return O, G, saved


def gpu_backward_saved(la, dev, O, G, saved, a, b, causal):
    """la_backward_saved with the buffer of gpu_forward_save."""
    Q, K, V, dO = dev["Q"], dev["K"], dev["V"], dev["dO"]
    B, H, N, D = Q.shape
    dQ, dK, dV = (torch.full_like(Q, float("nan")) for _ in range(3))
    wb = scratch(la.la_workspace_bytes(B, H, N, D, _dt(la, Q), causal, 1), Q.device)
    la.la_backward_saved(Q, K, V, O, G, dO, dQ, dK, dV, a, b, causal, wb, saved)
    torch.cuda.synchronize()
    return dQ, dK, dV


def run_gpu(la, dev, a, b, causal):
    """Forward then backward on the forward's own outputs: O, G, dQ, dK, dV."""
    O, G = gpu_forward(la, dev, a, b, causal)
    dQ, dK, dV = gpu_backward(la, dev, O, G, a, b, causal)
    return O, G, dQ, dK, dV


def saved_set(O_ref, G_ref, dtype):
    """The stored set of the forward pass as the backward pass receives it: O
    rounded to the I/O type, g in float32.  Returns (O_bits, O_64, G_32, G_64)."""
    O_bits, O_64 = wl.round_to_dtype(O_ref, dtype)
    G_32 = np.ascontiguousarray(G_ref, dtype=np.float32)
    return O_bits, O_64, G_32, G_32.astype(np.float64)


def upload_case(B, H, N, D, dtype, seed, keep_slices, normalise=True, only_kept=False):
    """Draw the inputs slice by slice, upload all of them, and keep float64 copies
    of the slices in ``keep_slices`` (flat b*H+h indices) for the oracle.

    ``only_kept``: for the largest shapes only the kept slices follow the seeded
    recipe; the others (never compared) are drawn on the device from the same
    distributions, which saves minutes of host-side drawing."""
    td = torch_dtype(dtype)
    dev = {n: torch.empty((B * H, N, D), dtype=td, device="cuda") for n in ("Q", "K", "V", "dO")}
    kept = {n: [] for n in ("Q", "K", "V", "dO")}
    keep = set(keep_slices)
    if only_kept:
        gen = torch.Generator(device="cuda")
        gen.manual_seed(seed)
        for n in dev:
            for s in range(B * H):
                x = torch.randn((N, D), device="cuda", dtype=torch.float32, generator=gen)
                if normalise and n in ("Q", "K"):
                    x = x / x.norm(dim=-1, keepdim=True)
                dev[n][s].copy_(x.to(td))
    for s in (sorted(keep) if only_kept else range(B * H)):
        sl = wl.make_slice(N, D, dtype, seed, s, normalise)
        for n in dev:
            dev[n][s].copy_(to_device(sl[n][0], dtype))
            if s in keep:
                kept[n].append(sl[n][1])
    dev = {n: t.view(B, H, N, D) for n, t in dev.items()}
    ref = {n: np.stack(v) if v else np.zeros((0, N, D)) for n, v in kept.items()}
    return dev, ref
