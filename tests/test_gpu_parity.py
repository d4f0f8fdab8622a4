"""GPU parity: the HIP path, called through the C ABI binding, against the fp64
oracle on the same seeded inputs.

Tolerance (stated by the benchmark spec: max relative error 1e-4 for fp32 I/O, 2e-2 for
bf16 I/O with fp32 accumulation), applied per element as
|gpu - ref| <= tol * (|ref| + rms(ref)) for each output tensor."""
import numpy as np
import pytest
import torch

import la_workloads as wl
from la_testlib import gpu_backward_saved, gpu_forward_save
from la_testlib import (TOL, excess, gpu_backward, gpu_forward, run_gpu, saved_set, to_device,
                        to_f64, upload_case)

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def la():
    import paper_2510_21956_amd as la_mod
    la_mod.load_library()
    assert torch.cuda.is_available()
    return la_mod


@pytest.fixture
def knobs(la):
    """la_debug_override for the duration of one test: knobs(seg_len, force_generic)."""
    yield la.la_debug_override
    la.la_debug_override(0, 0)


def check_against_oracle(oracle_mod, la, dev, ref, slices, dtype, a, b, causal, tag):
    """Forward: O, G against the oracle.  Backward: la_backward is given the stored
    set {Q, K, V, O, g} (Sec. 3.2) as the oracle's forward produces it -- O rounded
    to the I/O type, g in float32 -- and the oracle's backward consumes exactly the
    same stored values, so that the quantisation of the stored O is an input, not
    an error of the kernel.  The chained run (backward on the GPU forward's own
    outputs) is compared with the same reference, and so is the pair la_forward_save /
    la_backward_saved, whose forward outputs must equal la_forward's bit for bit."""
    B, H, N, D = dev["Q"].shape
    tol = TOL[dtype]
    slices = list(slices)
    O_ref, G_ref = oracle_mod.forward_rec(ref["Q"], ref["K"], ref["V"], a, b, causal)
    O_bits, O_64, G_32, G_64 = saved_set(O_ref, G_ref, dtype)
    grads_ref = oracle_mod.backward_rec(ref["Q"], ref["K"], ref["V"], O_64, G_64, ref["dO"],
                                        a, b, causal)

    O, G = gpu_forward(la, dev, a, b, causal)
    dQc, dKc, dVc = gpu_backward(la, dev, O, G, a, b, causal)            # chained
    O_in, G_in = O.clone(), G.clone()
    O_in.view(B * H, N, D)[slices] = to_device(O_bits, dtype)
    G_in.view(B * H, N)[slices] = torch.from_numpy(G_32).cuda()
    dQ, dK, dV = gpu_backward(la, dev, O_in, G_in, a, b, causal)         # oracle's stored set
    O2, G2, saved = gpu_forward_save(la, dev, a, b, causal)
    assert torch.equal(O2, O) and torch.equal(G2, G), "%s la_forward_save outputs differ" % tag
    dQs, dKs, dVs = gpu_backward_saved(la, dev, O_in, G_in, saved, a, b, causal)

    got = {"O": O, "G": G, "dQ": dQ, "dK": dK, "dV": dV, "dQ_chained": dQc, "dK_chained": dKc,
           "dV_chained": dVc, "dQ_saved": dQs, "dK_saved": dKs, "dV_saved": dVs}
    want = {"O": O_ref, "G": G_ref, "dQ": grads_ref[0], "dK": grads_ref[1], "dV": grads_ref[2],
            "dQ_chained": grads_ref[0], "dK_chained": grads_ref[1], "dV_chained": grads_ref[2],
            "dQ_saved": grads_ref[0], "dK_saved": grads_ref[1], "dV_saved": grads_ref[2]}
    # every output element must have been written
    for name, t in got.items():
        assert bool(torch.isfinite(t.float()).all()), "%s %s has non-finite values" % (tag, name)
    worst = {}
    for name in got:
        flat = got[name].reshape((B * H,) + tuple(got[name].shape[2:]))
        x = to_f64(flat[slices])
        # N = 1: dQ = dK = 0 exactly; allow rounding noise at the scale of V, dO ~ 1
        floor = tol if (N == 1 and name[:2] in ("dQ", "dK")) else 0.0
        # G is stored in fp32 whatever the I/O type
        worst[name] = excess(x, want[name], TOL["f32"] if name == "G" else tol, floor)
    print(tag, {k: round(v, 4) for k, v in worst.items()}, flush=True)
    for name, e in worst.items():
        assert e <= 1.0, "%s %s exceeds tolerance by factor %.3g" % (tag, name, e)


SMALL = [
    # B, H, N, D
    (1, 1, 1, 16), (1, 2, 5, 16), (2, 1, 16, 16), (1, 1, 17, 32), (1, 3, 100, 32),
    (1, 1, 256, 16), (2, 2, 300, 64), (1, 2, 129, 128), (1, 1, 700, 64), (1, 1, 520, 128),
    # matrix-core path at its edges: a single row, one short chunk, one row past a chunk,
    # exactly one chunk, one row past a 64-row segment boundary
    (1, 1, 1, 64), (1, 1, 31, 64), (1, 2, 33, 128), (1, 1, 64, 64), (3, 1, 65, 64), (1, 1, 1, 128),
    # head size 256 (four passes of the D = 128 kernels over column blocks)
    (1, 1, 1, 256), (1, 2, 70, 256), (2, 1, 300, 256),
]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("causal", [True, False])
@pytest.mark.parametrize("shape", SMALL)
def test_small_shapes(oracle_mod, la, knobs, shape, causal, dtype):
    """Sizes the oracle finishes in well under a second; several chunks, ragged
    tails, single rows; segments forced short so that several segments and a
    ragged last segment occur."""
    B, H, N, D = shape
    a, b = 1.0, 0.5
    for seg in ("64", "192", None):
        knobs(int(seg) if seg else 0, 0)
        tag = "small B%d H%d N%d D%d %s %s seg=%s" % (B, H, N, D, dtype,
                                                      "causal" if causal else "full", seg)
        print("case", tag, flush=True)
        slices = list(range(B * H))
        dev, ref = upload_case(B, H, N, D, dtype, 1234 + N + D, slices)
        check_against_oracle(oracle_mod, la, dev, ref, slices, dtype, a, b, causal, tag)


# General coefficients on every path.  With a = 1 every factor `a` in the kernels is
# invisible, so: a != 1 with b < 0, b = 0 (the linear term vanishes), b close to a (small
# denominators), and a = b = 1, the kernel the paper's own implementation fixes (Sec. 4).
# 64-row segments and N = 203 give four segments with a ragged tail in the last chunk.
COEFS = [(2.0, -0.7), (0.5, 0.0), (1.0, 0.9), (1.0, 1.0)]


@pytest.mark.parametrize("ab", COEFS)
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("D", [32, 64, 128, 256])
def test_other_coefficients(oracle_mod, la, knobs, D, dtype, ab):
    knobs(64, 0)
    a, b = ab
    for causal in (True, False):
        slices = [0, 1]
        tag = "coef D=%d %s a=%g b=%g causal=%d" % (D, dtype, a, b, causal)
        print("case", tag, flush=True)
        dev, ref = upload_case(1, 2, 203, D, dtype, 77 + D, slices)
        check_against_oracle(oracle_mod, la, dev, ref, slices, dtype, a, b, causal, tag)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("D", [32, 64, 128, 256])
def test_plain_alu_path_at_large_heads(oracle_mod, la, knobs, D, dtype):
    """The plain-ALU kernels are compiled for every head size (token-serial ones at D = 256);
    force them where the matrix-core kernels would normally run."""
    knobs(128, 1)
    for causal in (True, False):
        slices = [0, 1, 2]
        tag = "plain-ALU D=%d %s causal=%d" % (D, dtype, causal)
        print("case", tag, flush=True)
        dev, ref = upload_case(1, 3, 300, D, dtype, 501 + D, slices)
        check_against_oracle(oracle_mod, la, dev, ref, slices, dtype, 1.5, 0.6, causal, tag)


def test_optional_saved_set(la, knobs):
    """G = NULL in la_forward; O and/or G = NULL in la_backward (recomputed inside the call).
    The recomputation runs the same kernels on the same plan, so gradients must equal the
    chained run's bit for bit."""
    for (B, H, N, D, dtype, seg) in ((2, 2, 700, 64, "f32", 0), (1, 2, 333, 128, "bf16", 64),
                                     (1, 2, 100, 32, "f32", 0), (1, 2, 200, 256, "f32", 64),
                                     (1, 1, 130, 256, "bf16", 0)):
        knobs(seg, 0)
        for causal in (True, False):
            print("case optional", B, H, N, D, dtype, seg, causal, flush=True)
            dev, _ = upload_case(B, H, N, D, dtype, 31 + D, [])
            O, G, dQ, dK, dV = run_gpu(la, dev, 1.0, 0.5, causal)
            dt = la.LA_F32 if dtype == "f32" else la.LA_BF16
            from la_testlib import scratch
            O2 = torch.full_like(O, float("nan"))
            la.la_forward(dev["Q"], dev["K"], dev["V"], O2, None, 1.0, 0.5, causal,
                          scratch(la.la_workspace_bytes(B, H, N, D, dt, causal, 0), "cuda"))
            assert torch.equal(O2, O)
            for Oin, Gin in ((None, None), (O, None), (None, G)):
                g = [torch.full_like(O, float("nan")) for _ in range(3)]
                wb = scratch(la.la_workspace_bytes(B, H, N, D, dt, causal, 2), "cuda")
                la.la_backward(dev["Q"], dev["K"], dev["V"], Oin, Gin, dev["dO"], g[0], g[1], g[2],
                               1.0, 0.5, causal, wb)
                torch.cuda.synchronize()
                assert torch.equal(g[0], dQ) and torch.equal(g[1], dK) and torch.equal(g[2], dV)
            # the plain workspace size is not enough for the recomputation
            with pytest.raises(la.LaError) as e:
                wb = scratch(la.la_workspace_bytes(B, H, N, D, dt, causal, 1), "cuda")
                la.la_backward(dev["Q"], dev["K"], dev["V"], None, None, dev["dO"], g[0], g[1],
                               g[2], 1.0, 0.5, causal, wb)
            assert e.value.code == 5


# Full-size configurations, in the launch configuration the benchmark times.  The
# oracle evaluates whole slices (all rows of a few (batch, head) pairs) with the
# running-sum form, which the CPU tests pin to the definition.
FULL = [(0, [0]), (1, [0, 37, 63]), (2, [0, 41]), (3, [0, 127]), (4, [5])]


@pytest.mark.parametrize("index,slices", FULL)
def test_full_configs(oracle_mod, la, knobs, index, slices):
    knobs(0, 0)
    c = wl.CONFIGS[index]
    print("case", c.name, "slices", slices, flush=True)
    dev, ref = upload_case(c.B, c.H, c.N, c.D, c.dtype, wl.SEED_BASE + index, slices)
    check_against_oracle(oracle_mod, la, dev, ref, slices, c.dtype, c.a, c.b, c.causal, c.name)


@pytest.mark.parametrize("shape", [(1, 16, 5000, 128), (2, 16, 3333, 64)])
def test_cost_balanced_segments(oracle_mod, la, knobs, shape):
    """bf16 with the mask: the library cuts a sequence into segments of equal cost rather than
    equal length (the first rows cost more).  Mid-sized shapes where that plan has many
    segments, a sequence length that is no multiple of any tile, and the boundary between
    the two kinds of rows inside a segment."""
    knobs(0, 0)
    B, H, N, D = shape
    slices = [0, 7, B * H - 1]
    tag = "balanced B%d H%d N%d D%d bf16" % shape
    print("case", tag, flush=True)
    dev, ref = upload_case(B, H, N, D, "bf16", 4100 + N, slices)
    check_against_oracle(oracle_mod, la, dev, ref, slices, "bf16", 1.0, 0.5, True, tag)


@pytest.mark.parametrize("causal", [True, False])
def test_head_size_256_bf16(oracle_mod, la, knobs, causal):
    """bf16 at D = 256 in the plan the library picks for a mid-sized shape: every output is
    built up over passes on column blocks and rounded to bf16 in between; N is no multiple of
    a tile, and with the mask the first rows (second planes on chip) share a segment with
    later ones."""
    knobs(0, 0)
    B, H, N, D = 2, 8, 4100, 256
    slices = [0, 9, B * H - 1]
    tag = "D256 bf16 B%d H%d N%d causal=%d" % (B, H, N, causal)
    print("case", tag, flush=True)
    dev, ref = upload_case(B, H, N, D, "bf16", 2560 + causal, slices)
    check_against_oracle(oracle_mod, la, dev, ref, slices, "bf16", 1.0, 0.5, causal, tag)


UNUSUAL = [(64, 32, 3, 64, "f32", True), (64, 32, 3, 32, "bf16", True), (1, 1, 70000, 32, "f32", True),
           (2, 300, 100, 128, "bf16", True), (1, 2, 5, 256, "f32", False), (1, 600, 64, 32, "f32", True),
           (1, 1, 20000, 256, "bf16", True), (1, 1, 2, 32, "f32", True)]


@pytest.mark.parametrize("case", UNUSUAL)
def test_unusual_shapes(oracle_mod, la, knobs, case):
    """Shapes far from the benchmark's, in the plan the library picks: thousands of slices of a
    few rows, hundreds of heads, one long slice, two rows; three sampled slices each."""
    knobs(0, 0)
    B, H, N, D, dtype, causal = case
    BH = B * H
    slices = sorted(set([0, BH // 2, BH - 1]))
    tag = "unusual B%d H%d N%d D%d %s causal=%d" % (B, H, N, D, dtype, causal)
    print("case", tag, flush=True)
    dev, ref = upload_case(B, H, N, D, dtype, 9100 + N + D, slices)
    check_against_oracle(oracle_mod, la, dev, ref, slices, dtype, 1.0, 0.5, causal, tag)


# The paper's own benchmark shapes (Sec. 5.1), the ones the oracle finishes in seconds on a
# few sampled slices: the two shorter lengths of the D = 128 sweep (N = 10000 is not a
# multiple of any tile size) and the three head sizes at N = 4096.
PAPER = [("paper_causal_f32_B4_H16_N1000_D128", [0, 21, 63]),
         ("paper_causal_f32_B4_H16_N10000_D128", [0, 40]),
         ("paper_causal_f32_B4_H16_N4096_D32", [0, 50]),
         ("paper_causal_f32_B4_H16_N4096_D64", [7]),
         ("paper_causal_f32_B4_H16_N4096_D128", [63]),
         ("paper_causal_f32_B4_H16_N4096_D256", [17])]


@pytest.mark.parametrize("name,slices", PAPER)
def test_paper_shapes(oracle_mod, la, knobs, name, slices):
    knobs(0, 0)
    c = wl.find_workload(name)
    print("case", c.name, "slices", slices, flush=True)
    dev, ref = upload_case(c.B, c.H, c.N, c.D, c.dtype, wl.workload_seed(c), slices)
    check_against_oracle(oracle_mod, la, dev, ref, slices, c.dtype, c.a, c.b, c.causal, c.name)


@pytest.mark.parametrize("name,with_backward", [("paper_causal_f32_B4_H16_N100000_D128", True),
                                                ("paper_causal_f32_B4_H16_N300000_D128", False)])
def test_paper_long_shapes(oracle_mod, la, knobs, name, with_backward):
    """The two long rows of the paper's length sweep (Sec. 5.1) in the launch configuration
    the benchmark times: sampled rows of O, g recomputed one by one from the O(N^2 D)
    definition, and (N = 10^5) every row of one slice's gradients against the running-sum
    oracle fed the stored set."""
    knobs(0, 0)
    c = wl.find_workload(name)
    s = 29
    print("case", c.name, "slice", s, flush=True)
    dev, ref = upload_case(c.B, c.H, c.N, c.D, c.dtype, wl.workload_seed(c), [s], only_kept=True)
    O, G = gpu_forward(la, dev, c.a, c.b, c.causal)
    rng = np.random.default_rng(6)
    rows = np.unique(np.concatenate([[0, 1, 31, 32, c.N - 1], rng.integers(0, c.N, 120)]))
    o_ref, g_ref = oracle_mod.forward_def_rows(ref["Q"][0], ref["K"][0], ref["V"][0], rows,
                                               c.a, c.b, c.causal)
    o_gpu = to_f64(O.reshape(c.B * c.H, c.N, c.D)[s][rows])
    g_gpu = to_f64(G.reshape(c.B * c.H, c.N)[s][rows])
    eo, eg = excess(o_gpu, o_ref, TOL[c.dtype]), excess(g_gpu, g_ref, TOL["f32"])
    print(c.name, "rows: O", round(eo, 4), "G", round(eg, 4), flush=True)
    assert eo <= 1.0 and eg <= 1.0
    if not with_backward:
        return
    O_ref, G_ref = oracle_mod.forward_rec(ref["Q"], ref["K"], ref["V"], c.a, c.b, c.causal)
    O_bits, O_64, G_32, G_64 = saved_set(O_ref, G_ref, c.dtype)
    grads_ref = oracle_mod.backward_rec(ref["Q"], ref["K"], ref["V"], O_64, G_64, ref["dO"],
                                        c.a, c.b, c.causal)
    assert excess(to_f64(O.reshape(c.B * c.H, c.N, c.D)[s]), O_ref[0], TOL[c.dtype]) <= 1.0
    O.view(c.B * c.H, c.N, c.D)[s] = to_device(O_bits, c.dtype)[0]
    G.view(c.B * c.H, c.N)[s] = torch.from_numpy(G_32).cuda()[0]
    dQ, dK, dV = gpu_backward(la, dev, O, G, c.a, c.b, c.causal)
    for nm, got, want in (("dQ", dQ, grads_ref[0]), ("dK", dK, grads_ref[1]),
                          ("dV", dV, grads_ref[2])):
        e = excess(to_f64(got.reshape(c.B * c.H, c.N, c.D)[s]), want[0], TOL[c.dtype])
        print(c.name, nm, round(e, 4), flush=True)
        assert e <= 1.0, "%s exceeds tolerance by factor %.3g" % (nm, e)


def test_definition_rows_on_long_config(oracle_mod, la, knobs):
    """Long-sequence configuration: sampled rows recomputed one by one from the
    O(N^2 D) definition (not the running sums)."""
    knobs(0, 0)
    index = 4
    c = wl.CONFIGS[index]
    s = 11
    dev, ref = upload_case(c.B, c.H, c.N, c.D, c.dtype, wl.SEED_BASE + index, [s])
    O, G, _, _, _ = run_gpu(la, dev, c.a, c.b, c.causal)
    rng = np.random.default_rng(5)
    rows = np.unique(np.concatenate([[0, 1, c.N - 1], rng.integers(0, c.N, 200)]))
    o_ref, g_ref = oracle_mod.forward_def_rows(ref["Q"][0], ref["K"][0], ref["V"][0], rows,
                                               c.a, c.b, c.causal)
    o_gpu = to_f64(O.reshape(c.B * c.H, c.N, c.D)[s][rows])
    g_gpu = to_f64(G.reshape(c.B * c.H, c.N)[s][rows])
    # rms of the whole slice is not available here; use the sampled rows' own rms
    assert excess(o_gpu, o_ref, TOL[c.dtype]) <= 1.0
    assert excess(g_gpu, g_ref, TOL["f32"]) <= 1.0


@pytest.mark.parametrize("dtype,causal", [("f32", True), ("bf16", True), ("f32", False)])
def test_autograd_wrapper(oracle_mod, la, knobs, dtype, causal):
    """The torch.autograd wrapper: gradients of sum(O * dO) obtained through
    torch's backward() against the oracle's (chained: the wrapper's backward consumes the
    wrapper's own O and g)."""
    knobs(0, 0)
    B, H, N, D = 2, 3, 700, 64
    a, b = 1.0, 0.5
    slices = list(range(B * H))
    dev, ref = upload_case(B, H, N, D, dtype, 4242, slices)
    O_ref, G_ref = oracle_mod.forward_rec(ref["Q"], ref["K"], ref["V"], a, b, causal)
    grads_ref = oracle_mod.backward_rec(ref["Q"], ref["K"], ref["V"], O_ref, G_ref, ref["dO"], a, b,
                                        causal)
    Q, K, V = (dev[n].clone().requires_grad_(True) for n in ("Q", "K", "V"))
    O = la.linear_attention(Q, K, V, a, b, causal)
    (O.float() * dev["dO"].float()).sum().backward()
    torch.cuda.synchronize()
    tol = TOL[dtype]
    got = {"O": O.detach(), "dQ": Q.grad, "dK": K.grad, "dV": V.grad}
    want = {"O": O_ref, "dQ": grads_ref[0], "dK": grads_ref[1], "dV": grads_ref[2]}
    for name in got:
        e = excess(to_f64(got[name].reshape(B * H, N, D)), want[name], tol)
        print("autograd", dtype, causal, name, round(e, 4), flush=True)
        assert e <= 1.0, "%s exceeds tolerance by factor %.3g" % (name, e)


def test_run_to_run_determinism(la, knobs):
    knobs(0, 0)
    dev, _ = upload_case(2, 4, 1500, 64, "f32", 99, [])
    r1 = run_gpu(la, dev, 1.0, 0.5, True)
    r2 = run_gpu(la, dev, 1.0, 0.5, True)
    for x, y in zip(r1, r2):
        assert torch.equal(x, y)


def test_argument_errors(la):
    B, H, N, D = 1, 1, 64, 16
    Q = torch.zeros((B, H, N, D), device="cuda")
    G = torch.zeros((B, H, N), device="cuda")
    ws = torch.zeros(1 << 16, dtype=torch.uint8, device="cuda")
    tiny = torch.zeros(256, dtype=torch.uint8, device="cuda")
    with pytest.raises(la.LaError) as e:
        la.la_forward(Q, Q.clone(), Q.clone(), Q.clone(), G, 1.0, 0.5, True, tiny[:16])
    assert e.value.code == 5
    Q24 = torch.zeros((1, 1, 64, 24), device="cuda")
    with pytest.raises(la.LaError) as e:
        la.la_forward(Q24, Q24.clone(), Q24.clone(), Q24.clone(), G, 1.0, 0.5, True, ws)
    assert e.value.code == 3
    mis = torch.zeros(N * D + 1, device="cuda")[1:].view(B, H, N, D)
    with pytest.raises(la.LaError) as e:
        la.la_forward(mis, Q.clone(), Q.clone(), Q.clone(), G, 1.0, 0.5, True, ws)
    assert e.value.code == 4
    # an output that overlaps an input, and two outputs that overlap each other
    with pytest.raises(la.LaError) as e:
        la.la_forward(Q, Q.clone(), Q.clone(), Q, G, 1.0, 0.5, True, ws)
    assert e.value.code == 7
    with pytest.raises(la.LaError) as e:
        dq = Q.clone()
        la.la_backward(Q, Q.clone(), Q.clone(), Q.clone(), G, Q.clone(), dq, dq, Q.clone(), 1.0,
                       0.5, True, ws)
    assert e.value.code == 7
    # hand-over buffer: none is used for D = 16, one is required for D = 64
    assert la.la_saved_state_bytes(1, 1, 64, 16, la.LA_F32, 1) == 0
    la.la_forward_save(Q, Q.clone(), Q.clone(), Q.clone(), G, 1.0, 0.5, True, ws, None)
    need = la.la_saved_state_bytes(1, 2, 300, 64, la.LA_F32, 1)
    assert need > 0
    Q64 = torch.zeros((1, 2, 300, 64), device="cuda")
    G64 = torch.zeros((1, 2, 300), device="cuda")
    big = torch.zeros(1 << 22, dtype=torch.uint8, device="cuda")
    for bad in (None, tiny):
        with pytest.raises(la.LaError) as e:
            la.la_forward_save(Q64, Q64.clone(), Q64.clone(), Q64.clone(), G64, 1.0, 0.5, True,
                               big, bad)
        assert e.value.code == 5
        with pytest.raises(la.LaError) as e:
            la.la_backward_saved(Q64, Q64.clone(), Q64.clone(), Q64.clone(), G64, Q64.clone(),
                                 Q64.clone(), Q64.clone(), Q64.clone(), 1.0, 0.5, True, big, bad)
        assert e.value.code == 5
