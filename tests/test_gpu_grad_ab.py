"""GPU parity of la_backward_ab (gradients with respect to the kernel's coefficients a, b)
against the oracle's pairwise definition, which the CPU tests pin with finite differences
and library autograd."""
import numpy as np
import pytest
import torch

from la_testlib import TOL, gpu_forward, scratch, upload_case

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def la():
    import paper_2510_21956_amd as la_mod
    la_mod.load_library()
    assert torch.cuda.is_available()
    return la_mod


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("D", [16, 32, 64, 128, 256])
def test_grad_ab(oracle_mod, la, D, dtype):
    """Short forced segments (several segments, ragged tail); b = 0 included: the sweep runs
    with unit b, so the gradient with respect to b exists there as well.

    The results are two scalars, sums over slices of terms of both signs; each is allowed
    tol * (|ref| + sqrt(BH) * rms of the per-slice references), the scalar counterpart of
    the per-element allowance used for tensors."""
    B, H, N = 2, 2, 203
    BH = B * H
    tol = TOL[dtype]
    slices = list(range(BH))
    dt = la.LA_F32 if dtype == "f32" else la.LA_BF16
    try:
        la.la_debug_override(64, 0)
        dev, ref = upload_case(B, H, N, D, dtype, 1300 + D, slices)
        for a, b in ((1.0, 0.5), (2.0, -0.7), (1.5, 0.0)):
            for causal in (True, False):
                O, G = gpu_forward(la, dev, a, b, causal)
                dab = torch.full((2,), float("nan"), dtype=torch.float32, device="cuda")
                ws = scratch(la.la_workspace_bytes(B, H, N, D, dt, causal, 3), "cuda")
                la.la_backward_ab(dev["Q"], dev["K"], dev["V"], O, G, dev["dO"], dab, a, b, causal,
                                  ws)
                torch.cuda.synchronize()
                per = np.array([oracle_mod.grad_ab_def(ref["Q"][s], ref["K"][s], ref["V"][s],
                                                       ref["dO"][s], a, b, causal)
                                for s in range(BH)])
                want = per.sum(axis=0)
                got = dab.cpu().numpy().astype(np.float64)
                allow = tol * (np.abs(want) + np.sqrt(BH) * np.sqrt(np.mean(per ** 2, axis=0)))
                err = np.abs(got - want) / np.maximum(allow, 1e-300)
                print("grad_ab D=%d %s a=%g b=%g causal=%d" % (D, dtype, a, b, causal),
                      "got", got, "want", want, "excess", np.round(err, 4), flush=True)
                if b == 0.0:
                    assert got[0] == 0.0  # dL/da = -(b / a) dL/db
                    err = err[1:]
                assert np.all(err <= 1.0)
    finally:
        la.la_debug_override(0, 0)


def test_grad_ab_errors(la):
    B, H, N, D = 1, 1, 64, 64
    Q = torch.zeros((B, H, N, D), device="cuda")
    G = torch.ones((B, H, N), device="cuda")
    dab = torch.zeros(2, device="cuda")
    ws = scratch(la.la_workspace_bytes(B, H, N, D, la.LA_F32, 1, 3), "cuda")
    with pytest.raises(la.LaError) as e:   # a = 0: the ratio form has no gradient for a
        la.la_backward_ab(Q, Q.clone(), Q.clone(), Q.clone(), G, Q.clone(), dab, 0.0, 1.0, True, ws)
    assert e.value.code == 3
    with pytest.raises(la.LaError) as e:
        la.la_backward_ab(Q, Q.clone(), Q.clone(), Q.clone(), G, Q.clone(), dab, 1.0, 0.5, True,
                          ws[:4096])
    assert e.value.code == 5
