"""Pins for the fp64 CPU oracle (no GPU).

The paper prints no worked numeric example, so the oracle is pinned by:
  * a hand-evaluated example with exact fractions (tests/golden/),
  * definition == running-sum factorisation (an exact identity, Sec. 3.1/3.2),
  * central finite differences of L = sum(O * dO) (pins the corrected gradient
    formulas of Sec. 3.2),
  * closed forms (b = 0, N = 1, first causal row),
  * invariants (weights sum to one, scale invariances, column sums of dV),
  * the augmented-vector dense form evaluated with library matrix products,
    and PyTorch fp64 autograd through that dense form,
  * a = 0: normalised linear attention with the identity feature map
    (App. B.1), evaluated with library cumulative sums.
"""
import os
from fractions import Fraction

import numpy as np
import pytest
import torch

import la_workloads as wl

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "tiny_hand_example.txt")


def rand_inputs(BH, N, D, seed, normalise=True):
    x = wl.make_inputs(1, BH, N, D, "f32", seed, normalise)
    return tuple(x[n][1][0] for n in ("Q", "K", "V", "dO"))


def relerr(x, y):
    return float(np.max(np.abs(x - y)) / (np.max(np.abs(y)) + 1e-300))


# --------------------------------------------------------------------------
# hand example
# --------------------------------------------------------------------------
def _golden():
    out = {}
    for line in open(GOLDEN):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        mode, name, *vals = line.split()
        out[(mode, name)] = np.array([float(Fraction(v)) for v in vals])
    return out


@pytest.mark.parametrize("mode", ["causal", "noncausal"])
def test_hand_example(oracle_mod, mode):
    gold = _golden()
    causal = mode == "causal"
    q = np.array([[1.0], [2.0]]); k = np.array([[3.0], [4.0]])
    v = np.array([[5.0], [6.0]]); do = np.array([[1.0], [1.0]])
    for fwd in (oracle_mod.forward_def, oracle_mod.forward_rec):
        O, G = fwd(q, k, v, 1.0, 0.5, causal)
        np.testing.assert_allclose(O[:, 0], gold[(mode, "O")], rtol=1e-14)
        np.testing.assert_allclose(G, gold[(mode, "G")], rtol=1e-14)
    O, G = oracle_mod.forward_def(q, k, v, 1.0, 0.5, causal)
    grads = [oracle_mod.backward_def(q, k, v, do, 1.0, 0.5, causal),
             oracle_mod.backward_rec(q, k, v, O, G, do, 1.0, 0.5, causal)]
    for dq, dk, dv in grads:
        np.testing.assert_allclose(dq[:, 0], gold[(mode, "dQ")], rtol=1e-13, atol=1e-16)
        np.testing.assert_allclose(dk[:, 0], gold[(mode, "dK")], rtol=1e-13, atol=1e-16)
        np.testing.assert_allclose(dv[:, 0], gold[(mode, "dV")], rtol=1e-13, atol=1e-16)


# --------------------------------------------------------------------------
# definition == factorisation
# --------------------------------------------------------------------------
@pytest.mark.parametrize("causal", [True, False])
@pytest.mark.parametrize("BH,N,D", [(1, 1, 1), (2, 7, 3), (3, 65, 16), (1, 256, 16), (2, 300, 64)])
def test_def_equals_rec(oracle_mod, causal, BH, N, D):
    Q, K, V, dO = rand_inputs(BH, N, D, seed=11 + N)
    for a, b in ((1.0, 0.5), (2.0, -0.7), (1.0, 0.9)):
        O1, G1 = oracle_mod.forward_def(Q, K, V, a, b, causal)
        O2, G2 = oracle_mod.forward_rec(Q, K, V, a, b, causal)
        assert relerr(O2, O1) < 1e-11 and relerr(G2, G1) < 1e-12
        g1 = oracle_mod.backward_def(Q, K, V, dO, a, b, causal)
        g2 = oracle_mod.backward_rec(Q, K, V, O1, G1, dO, a, b, causal)
        for x, y in zip(g2, g1):
            assert relerr(x, y) < 1e-10


def test_def_rows_matches_full(oracle_mod):
    Q, K, V, _ = rand_inputs(1, 97, 8, seed=5)
    rows = np.array([0, 1, 50, 96])
    for causal in (True, False):
        O, G = oracle_mod.forward_def(Q, K, V, 1.0, 0.5, causal)
        o, g = oracle_mod.forward_def_rows(Q[0], K[0], V[0], rows, 1.0, 0.5, causal)
        np.testing.assert_allclose(o, O[0][rows], rtol=1e-14)
        np.testing.assert_allclose(g, G[0][rows], rtol=1e-14)


# --------------------------------------------------------------------------
# finite differences
# --------------------------------------------------------------------------
@pytest.mark.parametrize("causal", [True, False])
@pytest.mark.parametrize("N,D", [(1, 1), (5, 2), (8, 4)])
def test_finite_differences(oracle_mod, causal, N, D):
    a, b = 1.0, 0.5
    Q, K, V, dO = rand_inputs(1, N, D, seed=3)
    O, G = oracle_mod.forward_def(Q, K, V, a, b, causal)
    g_def = oracle_mod.backward_def(Q, K, V, dO, a, b, causal)
    g_rec = oracle_mod.backward_rec(Q, K, V, O, G, dO, a, b, causal)

    def loss(q, k, v):
        o, _ = oracle_mod.forward_def(q, k, v, a, b, causal)
        return float(np.sum(o * dO))

    h = 1e-6
    args = [Q, K, V]
    for t in range(3):
        fd = np.zeros_like(args[t])
        it = np.nditer(args[t], flags=["multi_index"])
        for _ in it:
            idx = it.multi_index
            plus = [x.copy() for x in args]
            minus = [x.copy() for x in args]
            plus[t][idx] += h
            minus[t][idx] -= h
            fd[idx] = (loss(*plus) - loss(*minus)) / (2 * h)
        scale = np.max(np.abs(fd)) + 1e-12
        assert np.max(np.abs(g_def[t] - fd)) / scale < 1e-6, ("def", t)
        assert np.max(np.abs(g_rec[t] - fd)) / scale < 1e-6, ("rec", t)


# --------------------------------------------------------------------------
# closed forms
# --------------------------------------------------------------------------
@pytest.mark.parametrize("causal", [True, False])
def test_b_zero_is_mean_of_v(oracle_mod, causal):
    BH, N, D, a = 2, 33, 5, 1.7
    Q, K, V, dO = rand_inputs(BH, N, D, seed=9)
    cnt = np.arange(1, N + 1, dtype=np.float64) if causal else np.full(N, float(N))
    if causal:
        mean = np.cumsum(V, axis=1) / cnt[None, :, None]
    else:
        mean = np.broadcast_to(V.mean(axis=1, keepdims=True), V.shape)
    # dv_p = sum over rows i that attend to p of dO_i / n_i   (w = a, g = a n)
    sc = dO / cnt[None, :, None]
    if causal:
        dv_ref = np.flip(np.cumsum(np.flip(sc, axis=1), axis=1), axis=1)
    else:
        dv_ref = np.broadcast_to(sc.sum(axis=1, keepdims=True), sc.shape)
    for fwd in (oracle_mod.forward_def, oracle_mod.forward_rec):
        O, G = fwd(Q, K, V, a, 0.0, causal)
        np.testing.assert_allclose(O, mean, rtol=1e-12, atol=1e-14)
        np.testing.assert_allclose(G, np.broadcast_to(a * cnt, G.shape), rtol=1e-14)
    O, G = oracle_mod.forward_def(Q, K, V, a, 0.0, causal)
    for dq, dk, dv in (oracle_mod.backward_def(Q, K, V, dO, a, 0.0, causal),
                       oracle_mod.backward_rec(Q, K, V, O, G, dO, a, 0.0, causal)):
        assert np.all(dq == 0) and np.all(dk == 0)
        np.testing.assert_allclose(dv, dv_ref, rtol=1e-12, atol=1e-14)


@pytest.mark.parametrize("causal", [True, False])
def test_single_row(oracle_mod, causal):
    Q, K, V, dO = rand_inputs(3, 1, 6, seed=2)
    O, G = oracle_mod.forward_rec(Q, K, V, 1.0, 0.5, causal)
    np.testing.assert_allclose(O, V, rtol=1e-14)
    for dq, dk, dv in (oracle_mod.backward_def(Q, K, V, dO, 1.0, 0.5, causal),
                       oracle_mod.backward_rec(Q, K, V, O, G, dO, 1.0, 0.5, causal)):
        np.testing.assert_allclose(dv, dO, rtol=1e-13)
        assert np.max(np.abs(dq)) < 1e-14 and np.max(np.abs(dk)) < 1e-14


def test_first_causal_row(oracle_mod):
    Q, K, V, dO = rand_inputs(2, 9, 4, seed=4)
    O, G = oracle_mod.forward_rec(Q, K, V, 1.0, 0.5, True)
    np.testing.assert_allclose(O[:, 0], V[:, 0], rtol=1e-14)
    dq, _, _ = oracle_mod.backward_rec(Q, K, V, O, G, dO, 1.0, 0.5, True)
    assert np.max(np.abs(dq[:, 0])) < 1e-14


# --------------------------------------------------------------------------
# invariants
# --------------------------------------------------------------------------
@pytest.mark.parametrize("causal", [True, False])
def test_invariants(oracle_mod, causal):
    BH, N, D, a, b = 2, 40, 6, 1.0, 0.5
    Q, K, V, dO = rand_inputs(BH, N, D, seed=21)
    O, G = oracle_mod.forward_rec(Q, K, V, a, b, causal)
    dq, dk, dv = oracle_mod.backward_rec(Q, K, V, O, G, dO, a, b, causal)

    # attention weights sum to one: constant V rows give the same constant rows
    c = np.linspace(-1, 2, D)
    Vc = np.broadcast_to(c, V.shape).copy()
    Oc, _ = oracle_mod.forward_rec(Q, K, Vc, a, b, causal)
    np.testing.assert_allclose(Oc, Vc, rtol=1e-12)

    # (a, b) -> (lambda a, lambda b) changes nothing but G
    lam = 3.25
    O2, G2 = oracle_mod.forward_rec(Q, K, V, lam * a, lam * b, causal)
    np.testing.assert_allclose(O2, O, rtol=1e-12)
    np.testing.assert_allclose(G2, lam * G, rtol=1e-12)
    g2 = oracle_mod.backward_rec(Q, K, V, O2, G2, dO, lam * a, lam * b, causal)
    for x, y in zip(g2, (dq, dk, dv)):
        np.testing.assert_allclose(x, y, rtol=1e-10, atol=1e-14)

    # b can be folded into Q
    O3, G3 = oracle_mod.forward_rec(b * Q, K, V, a, 1.0, causal)
    np.testing.assert_allclose(O3, O, rtol=1e-12)
    np.testing.assert_allclose(G3, G, rtol=1e-12)

    # shifting every v by a constant shifts every o by it: column sums of dV
    np.testing.assert_allclose(dv.sum(axis=1), dO.sum(axis=1), rtol=1e-11)

    # sum_n c_in w_in = 0 per row, hence q_i . dq_i = -a sum_n c_in
    oh = dO / G[..., None]
    delta = np.sum(O * oh, axis=-1)
    cmat = np.einsum("bij,bnj->bin", oh, V) - delta[..., None]
    if causal:
        cmat = np.tril(cmat)
    np.testing.assert_allclose(np.sum(Q * dq, axis=-1), -a * cmat.sum(axis=-1),
                               rtol=1e-9, atol=1e-13)


# --------------------------------------------------------------------------
# dense augmented form with library matrix products; autograd through it
# --------------------------------------------------------------------------
def dense_augmented(Q, K, V, a, b, causal):
    """q' = [b q, a], k' = [k, 1], v' = [v, 1]:  F = mask(Q'K'^T) V',
    O = F[:, :D] / F[:, D], G = F[:, D]."""
    ones = torch.ones_like(Q[..., :1])
    Qa = torch.cat([b * Q, a * ones], dim=-1)
    Ka = torch.cat([K, ones], dim=-1)
    Va = torch.cat([V, ones], dim=-1)
    W = Qa @ Ka.transpose(-1, -2)
    if causal:
        W = torch.tril(W)
    F = W @ Va
    return F[..., :-1] / F[..., -1:], F[..., -1]


@pytest.mark.parametrize("causal", [True, False])
@pytest.mark.parametrize("BH,N,D", [(2, 19, 4), (1, 130, 16)])
def test_dense_form_and_autograd(oracle_mod, causal, BH, N, D):
    a, b = 1.0, 0.5
    Q, K, V, dO = rand_inputs(BH, N, D, seed=31)
    tq, tk, tv = (torch.tensor(x, dtype=torch.float64, requires_grad=True) for x in (Q, K, V))
    O_t, G_t = dense_augmented(tq, tk, tv, a, b, causal)
    (O_t * torch.tensor(dO)).sum().backward()
    O, G = oracle_mod.forward_rec(Q, K, V, a, b, causal)
    np.testing.assert_allclose(O, O_t.detach().numpy(), rtol=1e-11, atol=1e-14)
    np.testing.assert_allclose(G, G_t.detach().numpy(), rtol=1e-12)
    for grads in (oracle_mod.backward_def(Q, K, V, dO, a, b, causal),
                  oracle_mod.backward_rec(Q, K, V, O, G, dO, a, b, causal)):
        for x, t in zip(grads, (tq, tk, tv)):
            np.testing.assert_allclose(x, t.grad.numpy(), rtol=1e-9, atol=1e-13)


# --------------------------------------------------------------------------
# a = 0: identity-feature-map normalised linear attention via cumulative sums
# --------------------------------------------------------------------------
def test_a_zero_matches_cumsum_rnn_form(oracle_mod):
    BH, N, D = 2, 50, 5
    Q, K, V, _ = rand_inputs(BH, N, D, seed=41, normalise=False)
    Q, K = np.abs(Q) + 0.1, np.abs(K) + 0.1      # keep q.z > 0
    S = np.cumsum(np.einsum("bnm,bnj->bnmj", K, V), axis=1)
    z = np.cumsum(K, axis=1)
    ref = np.einsum("bnm,bnmj->bnj", Q, S) / np.einsum("bnm,bnm->bn", Q, z)[..., None]
    for fwd in (oracle_mod.forward_def, oracle_mod.forward_rec):
        O, _ = fwd(Q, K, V, 0.0, 1.0, True)
        np.testing.assert_allclose(O, ref, rtol=1e-11)


# --------------------------------------------------------------------------
# incremental (decode) form with a carried state (App. B.1)
# --------------------------------------------------------------------------
def test_decode_hand_example(oracle_mod):
    """The hand-evaluated causal example, one row per call with the state carried over."""
    gold = _golden()
    q = np.array([[1.0], [2.0]]); k = np.array([[3.0], [4.0]]); v = np.array([[5.0], [6.0]])
    state = np.zeros(oracle_mod.decode_state_floats(1))
    for t in range(2):
        o, g = oracle_mod.decode(q[t:t + 1], k[t:t + 1], v[t:t + 1], state, 1.0, 0.5)
        np.testing.assert_allclose(o[0, 0], gold[("causal", "O")][t], rtol=1e-14)
        np.testing.assert_allclose(g[0], gold[("causal", "G")][t], rtol=1e-14)
    # the state is [S | z | p | count] = [3*5 + 4*6 | 3 + 4 | 5 + 6 | 2]
    np.testing.assert_allclose(state, [39.0, 7.0, 11.0, 2.0], rtol=1e-15)


@pytest.mark.parametrize("steps", [[1] * 9, [4, 1, 3, 1], [9], [2, 7]])
def test_decode_matches_definition_and_composes(oracle_mod, steps):
    """Fed a sequence in pieces of any sizes, the incremental form reproduces the causal
    definition row by row, and its final state is the plain sums over all rows."""
    BH, D = 3, 5
    N = sum(steps)
    Q, K, V, _ = rand_inputs(BH, N, D, seed=71)
    for a, b in ((1.0, 0.5), (2.0, -0.7)):
        O_def, G_def = oracle_mod.forward_def(Q, K, V, a, b, True)
        state = np.zeros((BH, oracle_mod.decode_state_floats(D)))
        at = 0
        for T in steps:
            o, g = oracle_mod.decode(Q[:, at:at + T], K[:, at:at + T], V[:, at:at + T], state, a, b)
            np.testing.assert_allclose(o, O_def[:, at:at + T], rtol=1e-11, atol=1e-14)
            np.testing.assert_allclose(g, G_def[:, at:at + T], rtol=1e-12)
            at += T
        S = np.einsum("bnm,bnj->bmj", K, V).reshape(BH, D * D)
        want = np.concatenate([S, K.sum(axis=1), V.sum(axis=1), np.full((BH, 1), float(N))], axis=1)
        np.testing.assert_allclose(state, want, rtol=1e-12, atol=1e-14)


# --------------------------------------------------------------------------
# gradients with respect to the kernel's coefficients a, b
# --------------------------------------------------------------------------
@pytest.mark.parametrize("causal", [True, False])
def test_grad_ab(oracle_mod, causal):
    BH, N, D = 2, 23, 6
    Q, K, V, dO = rand_inputs(BH, N, D, seed=83)
    for a, b in ((1.0, 0.5), (2.0, -0.7), (1.5, 0.0)):
        da, db = oracle_mod.grad_ab_def(Q, K, V, dO, a, b, causal)

        def loss(a_, b_):
            o, _ = oracle_mod.forward_def(Q, K, V, a_, b_, causal)
            return float(np.sum(o * dO))

        # central finite differences
        h = 1e-6
        np.testing.assert_allclose(da, (loss(a + h, b) - loss(a - h, b)) / (2 * h),
                                   rtol=1e-6, atol=1e-8)
        np.testing.assert_allclose(db, (loss(a, b + h) - loss(a, b - h)) / (2 * h),
                                   rtol=1e-6, atol=1e-8)
        # library autograd through the dense form
        ta = torch.tensor(a, dtype=torch.float64, requires_grad=True)
        tb = torch.tensor(b, dtype=torch.float64, requires_grad=True)
        O_t, _ = dense_augmented(torch.tensor(Q), torch.tensor(K), torch.tensor(V), ta, tb, causal)
        (O_t * torch.tensor(dO)).sum().backward()
        np.testing.assert_allclose(da, ta.grad.item(), rtol=1e-9, atol=1e-12)
        np.testing.assert_allclose(db, tb.grad.item(), rtol=1e-9, atol=1e-12)
        # O depends on (a, b) only through their ratio: a dL/da + b dL/db = 0, and the
        # gradient of Q carries the same number: sum q.dq = b dL/db
        assert abs(a * da + b * db) < 1e-9 * (abs(a * da) + abs(b * db)) + 1e-11
        dq, _, _ = oracle_mod.backward_def(Q, K, V, dO, a, b, causal)
        np.testing.assert_allclose(np.sum(Q * dq), b * db, rtol=1e-9, atol=1e-12)


# --------------------------------------------------------------------------
# row normalisation of Q and K (Sec. 3.3) and its backward
# --------------------------------------------------------------------------
def test_normalise_rows(oracle_mod):
    rng = np.random.default_rng(17)
    X = rng.standard_normal((3, 11, 7)) * 3.0
    Xh = oracle_mod.normalise_rows(X)
    np.testing.assert_allclose(np.linalg.norm(Xh, axis=-1), 1.0, rtol=1e-14)
    np.testing.assert_allclose(Xh, X / np.linalg.norm(X, axis=-1, keepdims=True), rtol=1e-14)
    np.testing.assert_allclose(oracle_mod.normalise_rows(5.0 * X), Xh, rtol=1e-14)  # scale-free
    dXh = rng.standard_normal(X.shape)
    dX = oracle_mod.normalise_rows_backward(X, dXh)
    # library autograd through torch's own normalisation
    tx = torch.tensor(X, requires_grad=True)
    (torch.nn.functional.normalize(tx, dim=-1) * torch.tensor(dXh)).sum().backward()
    np.testing.assert_allclose(dX, tx.grad.numpy(), rtol=1e-11, atol=1e-14)
    # xhat depends on the direction of x only: the gradient is orthogonal to x
    np.testing.assert_allclose(np.sum(dX * X, axis=-1), 0.0, atol=1e-13)
    # hand case: x = (3, 4), dxhat = (1, 0): dx = ((1, 0) - (0.6, 0.8) 0.6) / 5
    np.testing.assert_allclose(
        oracle_mod.normalise_rows_backward(np.array([[3.0, 4.0]]), np.array([[1.0, 0.0]])),
        [[0.128, -0.096]], rtol=1e-14)


@pytest.mark.parametrize("causal", [True, False])
def test_qknorm_composition(oracle_mod, causal):
    """Attention on normalised rows with gradients for the raw rows: finite differences and
    library autograd through normalisation + dense form."""
    BH, N, D = 2, 9, 4
    a, b = 1.0, 0.5
    Q, K, V, dO = rand_inputs(BH, N, D, seed=91, normalise=False)
    O, G = oracle_mod.forward_qknorm(Q, K, V, a, b, causal)
    dQ, dK, dV = oracle_mod.backward_qknorm(Q, K, V, O, G, dO, a, b, causal)
    tq, tk, tv = (torch.tensor(x, dtype=torch.float64, requires_grad=True) for x in (Q, K, V))
    nq = torch.nn.functional.normalize(tq, dim=-1)
    nk = torch.nn.functional.normalize(tk, dim=-1)
    O_t, G_t = dense_augmented(nq, nk, tv, a, b, causal)
    (O_t * torch.tensor(dO)).sum().backward()
    np.testing.assert_allclose(O, O_t.detach().numpy(), rtol=1e-11, atol=1e-14)
    for x, t in ((dQ, tq), (dK, tk), (dV, tv)):
        np.testing.assert_allclose(x, t.grad.numpy(), rtol=1e-9, atol=1e-13)

    def loss(q, k, v):
        o, _ = oracle_mod.forward_qknorm(q, k, v, a, b, causal)
        return float(np.sum(o * dO))

    h = 1e-6
    rng = np.random.default_rng(3)
    for t, grad in enumerate((dQ, dK)):
        for _ in range(6):
            idx = tuple(rng.integers(0, s) for s in Q.shape)
            args_p, args_m = [Q.copy(), K.copy(), V], [Q.copy(), K.copy(), V]
            args_p[t][idx] += h
            args_m[t][idx] -= h
            fd = (loss(*args_p) - loss(*args_m)) / (2 * h)
            np.testing.assert_allclose(grad[idx], fd, rtol=1e-5, atol=1e-8)
