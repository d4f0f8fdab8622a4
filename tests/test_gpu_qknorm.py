"""GPU parity of la_forward_qknorm / la_backward_qknorm and of the pair with the hand-over
(row normalisation of Q and K inside the call, Sec. 3.3) against the oracle: normalisation, running-sum passes, backward of the
normalisation, all in fp64.  Inputs are raw Gaussian rows of widely different lengths."""
import numpy as np
import pytest
import torch

import la_workloads as wl
from la_testlib import TOL, excess, saved_set, scratch, to_device, to_f64, torch_dtype

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def la():
    import paper_2510_21956_amd as la_mod
    la_mod.load_library()
    assert torch.cuda.is_available()
    return la_mod


def draw_raw(BH, N, D, dtype, seed):
    """Q, K: Gaussian rows times a per-row scale between 0.05 and 20 (not normalised);
    V, dO standard Gaussian.  Rounded to the I/O type."""
    dev, ref = {}, {}
    rng = np.random.Generator(np.random.PCG64([seed, 0]))
    for n in ("Q", "K", "V", "dO"):
        x = rng.standard_normal((BH, N, D))
        if n in ("Q", "K"):
            x *= np.exp(rng.uniform(np.log(0.05), np.log(20.0), size=(BH, N, 1)))
        bits, vals = wl.round_to_dtype(x, dtype)
        dev[n], ref[n] = to_device(bits, dtype), vals
    return dev, ref


CASES = [(1, 2, 203, 16, 64), (1, 2, 203, 32, 64), (2, 2, 333, 64, 64), (1, 3, 300, 128, 128),
         (2, 4, 1500, 64, 0), (1, 4, 1100, 128, 0)]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("causal", [True, False])
@pytest.mark.parametrize("case", CASES)
def test_qknorm(oracle_mod, la, case, causal, dtype):
    B, H, N, D, seg = case
    BH = B * H
    a, b = 1.0, 0.5
    tol = TOL[dtype]
    td = torch_dtype(dtype)
    dt = la.LA_F32 if dtype == "f32" else la.LA_BF16
    tag = "qknorm B%d H%d N%d D%d seg=%d %s causal=%d" % (B, H, N, D, seg, dtype, causal)
    print("case", tag, flush=True)
    try:
        la.la_debug_override(seg, 0)
        dev, ref = draw_raw(BH, N, D, dtype, 7000 + N + D)
        dev = {n: t.reshape(B, H, N, D).contiguous() for n, t in dev.items()}
        O_ref, G_ref = oracle_mod.forward_qknorm(ref["Q"], ref["K"], ref["V"], a, b, causal)
        O_bits, O_64, G_32, G_64 = saved_set(O_ref, G_ref, dtype)
        grads_ref = oracle_mod.backward_qknorm(ref["Q"], ref["K"], ref["V"], O_64, G_64, ref["dO"],
                                               a, b, causal)
        O = torch.full((B, H, N, D), float("nan"), dtype=td, device="cuda")
        G = torch.full((B, H, N), float("nan"), dtype=torch.float32, device="cuda")
        la.la_forward_qknorm(dev["Q"], dev["K"], dev["V"], O, G, a, b, causal,
                             scratch(la.la_workspace_bytes(B, H, N, D, dt, causal, 0), "cuda"))
        # backward on the oracle's stored set (O rounded to the I/O type, g in float32)
        O_in = to_device(O_bits, dtype).reshape(B, H, N, D).contiguous()
        G_in = torch.from_numpy(G_32).cuda().reshape(B, H, N).contiguous()
        g = [torch.full((B, H, N, D), float("nan"), dtype=td, device="cuda") for _ in range(3)]
        la.la_backward_qknorm(dev["Q"], dev["K"], dev["V"], O_in, G_in, dev["dO"], g[0], g[1], g[2],
                              a, b, causal,
                              scratch(la.la_workspace_bytes(B, H, N, D, dt, causal, 1), "cuda"))
        # and with O, G recomputed inside the call (also normalised there)
        g2 = [torch.full((B, H, N, D), float("nan"), dtype=td, device="cuda") for _ in range(3)]
        la.la_backward_qknorm(dev["Q"], dev["K"], dev["V"], None, None, dev["dO"], g2[0], g2[1],
                              g2[2], a, b, causal,
                              scratch(la.la_workspace_bytes(B, H, N, D, dt, causal, 2), "cuda"))
        # the pair with the hand-over: same forward outputs bit for bit, gradients from the
        # sums the forward pass handed over
        O3 = torch.full((B, H, N, D), float("nan"), dtype=td, device="cuda")
        G3 = torch.full((B, H, N), float("nan"), dtype=torch.float32, device="cuda")
        nsv = la.la_saved_state_bytes(B, H, N, D, dt, causal)
        saved = scratch(nsv, "cuda") if nsv else None
        la.la_forward_qknorm_save(dev["Q"], dev["K"], dev["V"], O3, G3, a, b, causal,
                                  scratch(la.la_workspace_bytes(B, H, N, D, dt, causal, 0), "cuda"),
                                  saved)
        g3 = [torch.full((B, H, N, D), float("nan"), dtype=td, device="cuda") for _ in range(3)]
        la.la_backward_qknorm_saved(dev["Q"], dev["K"], dev["V"], O_in, G_in, dev["dO"], g3[0],
                                    g3[1], g3[2], a, b, causal,
                                    scratch(la.la_workspace_bytes(B, H, N, D, dt, causal, 1),
                                            "cuda"), saved)
        torch.cuda.synchronize()
        assert torch.equal(O3, O) and torch.equal(G3, G), "%s hand-over forward differs" % tag
        worst = {"O": excess(to_f64(O.reshape(BH, N, D)), O_ref, tol),
                 "G": excess(to_f64(G.reshape(BH, N)), G_ref, TOL["f32"])}
        for nm, x, y, z, want in zip(("dQ", "dK", "dV"), g, g2, g3, grads_ref):
            worst[nm] = excess(to_f64(x.reshape(BH, N, D)), want, tol)
            worst[nm + "_recomputed"] = excess(to_f64(y.reshape(BH, N, D)), want, tol)
            worst[nm + "_saved"] = excess(to_f64(z.reshape(BH, N, D)), want, tol)
        print(tag, {k: round(v, 4) for k, v in worst.items()}, flush=True)
        for nm, e in worst.items():
            assert e <= 1.0, "%s %s exceeds tolerance by factor %.3g" % (tag, nm, e)
    finally:
        la.la_debug_override(0, 0)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_autograd_wrapper_normalised(oracle_mod, la, dtype):
    """linear_attention(..., normalize_qk=True): gradients through torch's backward() for the raw
    rows against the oracle's.  The wrapper's backward consumes its own stored O and g; the
    oracle's backward is given its O rounded to the I/O type and its g in float32, the same
    stored set up to the rare element the two forward passes round differently."""
    B, H, N, D = 2, 2, 500, 64
    BH = B * H
    a, b, causal = 1.0, 0.5, True
    dev, ref = draw_raw(BH, N, D, dtype, 7900)
    dev = {n: t.reshape(B, H, N, D).contiguous() for n, t in dev.items()}
    O_ref, G_ref = oracle_mod.forward_qknorm(ref["Q"], ref["K"], ref["V"], a, b, causal)
    _, O_64, _, G_64 = saved_set(O_ref, G_ref, dtype)
    grads_ref = oracle_mod.backward_qknorm(ref["Q"], ref["K"], ref["V"], O_64, G_64, ref["dO"], a,
                                           b, causal)
    Q, K, V = (dev[n].clone().requires_grad_(True) for n in ("Q", "K", "V"))
    O = la.linear_attention(Q, K, V, a, b, causal, normalize_qk=True)
    (O.float() * dev["dO"].float()).sum().backward()
    torch.cuda.synchronize()
    got = {"O": O.detach(), "dQ": Q.grad, "dK": K.grad, "dV": V.grad}
    want = {"O": O_ref, "dQ": grads_ref[0], "dK": grads_ref[1], "dV": grads_ref[2]}
    for name in got:
        e = excess(to_f64(got[name].reshape(BH, N, D)), want[name], TOL[dtype])
        print("autograd normalised", dtype, name, round(e, 4), flush=True)
        assert e <= 1.0, "%s exceeds tolerance by factor %.3g" % (name, e)
