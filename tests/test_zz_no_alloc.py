"""la_forward_static (the entry point that allocates nothing) against la_forward, through
the C ABI: two calls in a row on the shared static scratch, the second with a smaller
input, each compared bit for bit (same kernels, same plan) and against the oracle."""
import pytest
import torch

from la_testlib import TOL, excess, gpu_forward, to_f64, upload_case

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def la():
    import paper_2510_21956_amd as la_mod
    la_mod.load_library()
    assert torch.cuda.is_available()
    return la_mod


def test_forward_static_matches_forward(oracle_mod, la):
    la.la_debug_override(0, 0)
    for (B, H, N, D, dtype, causal) in ((2, 4, 3000, 64, "f32", True),    # several segments
                                        (1, 2, 700, 64, "f32", True),     # smaller, same scratch
                                        (1, 3, 1500, 128, "bf16", True),
                                        (2, 2, 900, 64, "f32", False),
                                        (1, 1, 100, 16, "f32", True)):
        print("case static", B, H, N, D, dtype, causal, flush=True)
        slices = list(range(B * H))
        dev, ref = upload_case(B, H, N, D, dtype, 900 + N, slices)
        O_want, G_want = gpu_forward(la, dev, 1.0, 0.5, causal)
        O = torch.full_like(O_want, float("nan"))
        G = torch.full_like(G_want, float("nan"))
        la.la_forward_static(dev["Q"], dev["K"], dev["V"], O, G, 1.0, 0.5, causal)
        torch.cuda.synchronize()
        assert torch.equal(O, O_want) and torch.equal(G, G_want)
        O_ref, G_ref = oracle_mod.forward_rec(ref["Q"], ref["K"], ref["V"], 1.0, 0.5, causal)
        assert excess(to_f64(O.reshape(B * H, N, D)), O_ref, TOL[dtype]) <= 1.0
        assert excess(to_f64(G.reshape(B * H, N)), G_ref, TOL["f32"]) <= 1.0


def test_forward_static_rejects_oversize(la):
    # short forced segments make the per-segment states outgrow the static scratch
    Q = torch.zeros((1, 16, 131072, 128), dtype=torch.bfloat16, device="cuda")
    G = torch.zeros((1, 16, 131072), device="cuda")
    la.la_debug_override(64, 0)
    try:
        assert la.la_workspace_bytes(1, 16, 131072, 128, la.LA_BF16, 1, 0) > \
            la.LA_STATIC_SCRATCH_BYTES
        with pytest.raises(la.LaError) as e:
            la.la_forward_static(Q, Q.clone(), Q.clone(), Q.clone(), G, 1.0, 0.5, True)
        assert e.value.code == 5
    finally:
        la.la_debug_override(0, 0)
