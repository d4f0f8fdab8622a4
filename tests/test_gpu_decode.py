"""GPU parity of the incremental (decode) entry points against the oracle's incremental form
(App. B.1), which the CPU tests pin to the definition."""
import numpy as np
import pytest
import torch

import la_workloads as wl
from la_testlib import TOL, excess, scratch, to_device, to_f64, torch_dtype

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def la():
    import paper_2510_21956_amd as la_mod
    la_mod.load_library()
    assert torch.cuda.is_available()
    la_mod.la_debug_override(0, 0)
    return la_mod


def draw(BH, N, D, dtype, seed):
    bits = {n: [] for n in ("Q", "K", "V")}
    vals = {n: [] for n in ("Q", "K", "V")}
    for s in range(BH):
        sl = wl.make_slice(N, D, dtype, seed, s)
        for n in bits:
            bits[n].append(sl[n][0])
            vals[n].append(sl[n][1])
    dev = {n: to_device(np.stack(bits[n]), dtype) for n in bits}
    ref = {n: np.stack(vals[n]) for n in vals}
    return dev, ref


def canonical_state(state, BH, D):
    """[S | z | p | count] of every slice from the library's padded state."""
    return to_f64(state.view(BH, -1)[:, :D * D + 2 * D + 1])


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("D", [16, 32, 64, 128, 256])
def test_decode_steps(oracle_mod, la, D, dtype):
    """A sequence fed in pieces of 1, 5, 1, 2, ... rows with the state carried over: every
    output row and the final state against the oracle; a = 1, b = 0.5 and a = 2, b = -0.7."""
    B, H = 2, 3
    BH = B * H
    steps = [1, 5, 1, 2, 16, 1, 7]
    N = sum(steps)
    tol = TOL[dtype]
    td = torch_dtype(dtype)
    dev, ref = draw(BH, N, D, dtype, 600 + D)
    for a, b in ((1.0, 0.5), (2.0, -0.7)):
        print("case decode D=%d %s a=%g b=%g" % (D, dtype, a, b), flush=True)
        state = torch.zeros(la.la_decode_state_bytes(B, H, D) // 4, dtype=torch.float32,
                            device="cuda")
        st_ref = np.zeros((BH, oracle_mod.decode_state_floats(D)))
        at = 0
        for T in steps:
            q, k, v = (dev[n][:, at:at + T].reshape(B, H, T, D).contiguous() for n in "QKV")
            o = torch.full((B, H, T, D), float("nan"), dtype=td, device="cuda")
            g = torch.full((B, H, T), float("nan"), dtype=torch.float32, device="cuda")
            la.la_decode_step(q, k, v, o, g, state, a, b)
            torch.cuda.synchronize()
            o_ref, g_ref = oracle_mod.decode(ref["Q"][:, at:at + T], ref["K"][:, at:at + T],
                                             ref["V"][:, at:at + T], st_ref, a, b)
            eo = excess(to_f64(o.reshape(BH, T, D)), o_ref, tol)
            eg = excess(to_f64(g.reshape(BH, T)), g_ref, TOL["f32"])
            assert eo <= 1.0 and eg <= 1.0, (at, T, eo, eg)
            at += T
        # the state is float32 whatever the I/O type
        es = excess(canonical_state(state, BH, D), st_ref, TOL["f32"])
        print("  final state excess", round(es, 4), flush=True)
        assert es <= 1.0


@pytest.mark.parametrize("dtype,D,N0", [("f32", 64, 700), ("bf16", 128, 1000), ("f32", 32, 300),
                                        ("f32", 256, 700), ("bf16", 256, 400)])
def test_prefill_then_decode(oracle_mod, la, dtype, D, N0):
    """la_decode_prefill over a prompt (in two parts, the second accumulated), then single
    decode steps: outputs must equal the rows of the causal forward pass over the whole
    sequence (oracle: running sums), and la_forward's own rows on the GPU within tolerance."""
    B, H, extra = 1, 4, 6
    BH, N = B * H, N0 + extra
    tol = TOL[dtype]
    td = torch_dtype(dtype)
    dev, ref = draw(BH, N, D, dtype, 900 + D)
    a, b = 1.0, 0.5
    dt = la.LA_F32 if dtype == "f32" else la.LA_BF16
    state = torch.full((la.la_decode_state_bytes(B, H, D) // 4,), float("nan"),
                       dtype=torch.float32, device="cuda")
    cut = 192  # first part: overwrite; second part: accumulate
    for lo, hi, acc in ((0, cut, 0), (cut, N0, 1)):
        K = dev["K"][:, lo:hi].reshape(B, H, hi - lo, D).contiguous()
        V = dev["V"][:, lo:hi].reshape(B, H, hi - lo, D).contiguous()
        ws = scratch(la.la_workspace_bytes(B, H, hi - lo, D, dt, 0, 0), "cuda")
        la.la_decode_prefill(K, V, state, acc, ws)
    O_ref, G_ref = oracle_mod.forward_rec(ref["Q"], ref["K"], ref["V"], a, b, True)
    for t in range(N0, N):
        q, k, v = (dev[n][:, t:t + 1].reshape(B, H, 1, D).contiguous() for n in "QKV")
        o = torch.full((B, H, 1, D), float("nan"), dtype=td, device="cuda")
        g = torch.full((B, H, 1), float("nan"), dtype=torch.float32, device="cuda")
        la.la_decode_step(q, k, v, o, g, state, a, b)
        torch.cuda.synchronize()
        eo = excess(to_f64(o.reshape(BH, D)), O_ref[:, t], tol)
        eg = excess(to_f64(g.reshape(BH)), G_ref[:, t], TOL["f32"])
        print("prefill+decode", dtype, D, "row", t, round(eo, 4), round(eg, 4), flush=True)
        assert eo <= 1.0 and eg <= 1.0


def test_decode_argument_errors(la):
    B, H, T, D = 1, 2, 1, 64
    q = torch.zeros((B, H, T, D), device="cuda")
    st = torch.zeros(la.la_decode_state_bytes(B, H, D) // 4, device="cuda")
    with pytest.raises(la.LaError) as e:
        la.la_decode_step(q, q.clone(), q.clone(), q.clone(), None, st[:64], 1.0, 0.5)
    assert e.value.code == 5
    with pytest.raises(la.LaError) as e:
        la.la_decode_step(q, q.clone(), q.clone(), q, None, st, 1.0, 0.5)
    assert e.value.code == 7
    q48 = torch.zeros((B, H, T, 48), device="cuda")
    with pytest.raises(la.LaError) as e:
        la.la_decode_step(q48, q48.clone(), q48.clone(), q48.clone(), None, st, 1.0, 0.5)
    assert e.value.code == 3
    assert la.la_decode_state_bytes(1, 1, 48) == 0
