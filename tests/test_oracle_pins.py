"""Pins for the fp64 CPU oracle: it is checked against what the paper and the
mathematics fix, never against itself alone.

  - hand-worked rational cases (tests/golden/rational_case_*.json);
  - the defining quadratic forms (eq. 3, eq. 8) against the linear-time forms
    (eq. 5-6, eq. 10-12) and against the step-by-step recurrence (eq. 16-20);
  - torch's own elu, matmul, tril and autograd in fp64 as independent library routines;
  - central finite differences of L = sum(G * O);
  - closed forms: Q = K = 0 (running mean), constant V, N = 1, ones column, weights
    non-negative with unit row sums (eq. 3's requirement that sim be non-negative).
"""
import json
import math
import os
from fractions import Fraction

import numpy as np
import pytest
import torch

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _frac(s):
    """'a/b', 'a', or a sum/difference of such terms -> float via exact Fractions."""
    s = s.replace("-", "+-")
    total = Fraction(0)
    for term in s.split("+"):
        term = term.strip()
        if term:
            total += Fraction(term)
    return float(total)


def _fr(a):
    return np.array([[_frac(x) for x in row] if isinstance(row, list) else _frac(row) for row in a],
                    dtype=np.float64)


def _rand(seed, B, H, N, D, M):
    rng = np.random.default_rng(seed)
    return (rng.standard_normal((B, H, N, D)), rng.standard_normal((B, H, N, D)),
            rng.standard_normal((B, H, N, M)), rng.standard_normal((B, H, N, M)))


# ------------------------------------------------------------------ feature map (eq. 7)

def test_phi_values_and_library(oracle):
    x = np.array([-745.0, -30.0, -1.0, -1e-9, 0.0, 1e-9, 0.5, 3.0, 1e6])
    got = oracle.phi(x)
    assert got[4] == 1.0                       # phi(0) = exp(0) = 1
    assert np.all(got[5:] == x[5:] + 1.0)      # x > 0: exactly x + 1
    assert got[2] == math.exp(-1.0)
    assert np.all(got > 0.0) or got[0] == 0.0  # positive (may underflow far left)
    lib = torch.nn.functional.elu(torch.tensor(x, dtype=torch.float64)).numpy() + 1.0
    # torch forms elu(x) + 1 = expm1(x) + 1, which rounds at 2^-53 absolute for x << 0
    np.testing.assert_allclose(got, lib, rtol=1e-15, atol=3e-16)


def test_dphi_is_derivative_of_phi(oracle):
    x = np.array([-5.0, -1.0, -0.1, 0.3, 2.0])
    h = 1e-6
    fd = (oracle.phi(x + h) - oracle.phi(x - h)) / (2 * h)
    np.testing.assert_allclose(oracle.dphi(x), fd, rtol=1e-8)
    assert oracle.dphi(np.array([0.0]))[0] == 1.0


# ------------------------------------------------------------------ hand-worked cases

def test_rational_case_a(oracle):
    g = json.load(open(os.path.join(GOLD, "rational_case_a.json")))
    Q, K, V, G = (np.array(g[k], dtype=np.float64) for k in "QKVG")
    eps = g["eps"]
    for fwd in (oracle.causal_fwd_quadratic, oracle.causal_fwd_prefix):
        O, den = fwd(Q, K, V, eps, return_den=True)
        np.testing.assert_allclose(O, _fr(g["O_causal"]), rtol=1e-14, atol=1e-15)
        np.testing.assert_allclose(den, _fr(g["den_causal"]), rtol=1e-14)
    for gf in (oracle.global_fwd_quadratic, oracle.global_fwd_linear):
        np.testing.assert_allclose(gf(Q, K, V, eps), _fr(g["O_global"]), rtol=1e-14, atol=1e-15)
    for bwd in (oracle.causal_bwd_quadratic, oracle.causal_bwd_linear):
        dQ, dK, dV = bwd(Q, K, V, G, eps)
        np.testing.assert_allclose(dV, _fr(g["dV"]), rtol=1e-13, atol=1e-15)
        np.testing.assert_allclose(dQ, _fr(g["dQ"]), rtol=1e-13, atol=1e-15)
        np.testing.assert_allclose(dK, _fr(g["dK"]), rtol=1e-13, atol=1e-15)


def test_rational_case_b_exp_branch(oracle):
    g = json.load(open(os.path.join(GOLD, "rational_case_b.json")))
    sym = {"-ln2": -math.log(2.0), "-ln4": -math.log(4.0), "1": 1.0, "0": 0.0}
    Q = np.array([[sym[s]] for s in g["Q_expr"]])
    K = np.array([[sym[s]] for s in g["K_expr"]])
    V = np.array(g["V"], dtype=np.float64)
    G = np.array(g["G"], dtype=np.float64)
    for fwd in (oracle.causal_fwd_quadratic, oracle.causal_fwd_prefix):
        O, den = fwd(Q, K, V, 0.0, return_den=True)
        np.testing.assert_allclose(O, _fr(g["O_causal"]), rtol=1e-14)
        np.testing.assert_allclose(den, _fr(g["den_causal"]), rtol=1e-14)
    for bwd in (oracle.causal_bwd_quadratic, oracle.causal_bwd_linear):
        dQ, dK, dV = bwd(Q, K, V, G, 0.0)
        np.testing.assert_allclose(dV, _fr(g["dV"]), rtol=1e-13)
        np.testing.assert_allclose(dK, _fr(g["dK"]), rtol=1e-13)
        np.testing.assert_allclose(dQ, 0.0, atol=1e-14)


# ------------------------------------------------------------------ causal forward

def _torch_causal(Q, K, V, eps):
    """eq. 8 with torch library routines (elu, matmul, tril) in fp64."""
    Q, K, V = (torch.as_tensor(a, dtype=torch.float64) for a in (Q, K, V))
    fq = torch.nn.functional.elu(Q) + 1
    fk = torch.nn.functional.elu(K) + 1
    A = torch.tril(fq @ fk.transpose(-1, -2))
    den = A.sum(-1, keepdim=True) + eps
    return (A @ V) / den, den.squeeze(-1)


@pytest.mark.parametrize("shape", [(1, 1, 1, 3, 2), (2, 3, 37, 8, 5), (1, 2, 130, 32, 32),
                                   (1, 1, 64, 64, 64)])
def test_causal_prefix_equals_quadratic_and_library(oracle, shape):
    B, H, N, D, M = shape
    Q, K, V, _ = _rand(11 + N, B, H, N, D, M)
    for eps in (0.0, 1e-6, 0.5):
        Oq, dq = oracle.causal_fwd_quadratic(Q, K, V, eps, return_den=True)
        Op, dp = oracle.causal_fwd_prefix(Q, K, V, eps, return_den=True)
        Ot, dt = _torch_causal(Q, K, V, eps)
        np.testing.assert_allclose(Op, Oq, rtol=1e-12, atol=1e-13)
        np.testing.assert_allclose(dp, dq, rtol=1e-13)
        np.testing.assert_allclose(Oq, Ot.numpy(), rtol=1e-11, atol=1e-12)
        np.testing.assert_allclose(dq, dt.numpy(), rtol=1e-12)


def test_recurrent_steps_reproduce_prefix_bit_for_bit(oracle):
    B, H, N, D, M = 2, 2, 50, 16, 8
    Q, K, V, _ = _rand(5, B, H, N, D, M)
    Op, dp = oracle.causal_fwd_prefix(Q, K, V, 1e-6, return_den=True)
    S = np.zeros((B, H, D, M))           # eq. 16
    z = np.zeros((B, H, D))              # eq. 17
    for i in range(N):
        out, den = oracle.recurrent_step(Q[:, :, i], K[:, :, i], V[:, :, i], S, z, 1e-6,
                                         return_den=True)
        assert np.array_equal(out, Op[:, :, i])
        assert np.array_equal(den, dp[:, :, i])
    # the final state is the full sum of eq. 10 / eq. 11
    fk = oracle.phi(K)
    np.testing.assert_allclose(S, np.einsum("bhnd,bhnm->bhdm", fk, V), rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(z, fk.sum(2), rtol=1e-13)


def test_recurrent_split_and_resume(oracle):
    B, H, N, D, M = 1, 3, 40, 8, 8
    Q, K, V, _ = _rand(6, B, H, N, D, M)
    S = np.zeros((B, H, D, M)); z = np.zeros((B, H, D))
    outs = [oracle.recurrent_step(Q[:, :, i], K[:, :, i], V[:, :, i], S, z) for i in range(N)]
    S2 = np.zeros((B, H, D, M)); z2 = np.zeros((B, H, D))
    for i in range(N // 2):
        oracle.recurrent_step(Q[:, :, i], K[:, :, i], V[:, :, i], S2, z2)
    S3, z3 = S2.copy(), z2.copy()        # "checkpoint"
    for i in range(N // 2, N):
        o = oracle.recurrent_step(Q[:, :, i], K[:, :, i], V[:, :, i], S3, z3)
        assert np.array_equal(o, outs[i])
    assert np.array_equal(S3, S) and np.array_equal(z3, z)


def test_closed_form_zero_qk_is_running_mean(oracle):
    B, H, N, D, M = 1, 2, 33, 4, 3
    _, _, V, _ = _rand(7, B, H, N, D, M)
    Zq = np.zeros((B, H, N, D))
    eps = 1e-6
    i = np.arange(1, N + 1, dtype=np.float64)[None, None, :, None]
    expect = D * np.cumsum(V, axis=2) / (D * i + eps)
    np.testing.assert_allclose(oracle.causal_fwd_prefix(Zq, Zq, V, eps), expect, rtol=1e-13, atol=1e-14)
    np.testing.assert_allclose(oracle.causal_fwd_quadratic(Zq, Zq, V, eps), expect, rtol=1e-13, atol=1e-14)
    gexp = D * V.sum(2, keepdims=True) / (D * N + eps) * np.ones_like(V)
    np.testing.assert_allclose(oracle.global_fwd_linear(Zq, Zq, V, eps), gexp, rtol=1e-13, atol=1e-14)
    np.testing.assert_allclose(oracle.global_fwd_quadratic(Zq, Zq, V, eps), gexp, rtol=1e-13, atol=1e-14)


def test_constant_v_gives_constant_output(oracle):
    B, H, N, D, M = 1, 2, 45, 8, 4
    Q, K, _, _ = _rand(8, B, H, N, D, M)
    c = np.array([1.5, -2.0, 0.25, 7.0])
    V = np.broadcast_to(c, (B, H, N, M)).copy()
    eps = 1e-6
    for fwd in (oracle.causal_fwd_prefix, oracle.causal_fwd_quadratic):
        O, den = fwd(Q, K, V, eps, return_den=True)
        np.testing.assert_allclose(O, c * (1.0 - eps / den[..., None]), rtol=1e-12)
    O0 = oracle.causal_fwd_prefix(Q, K, V, 0.0)
    np.testing.assert_allclose(O0, V, rtol=1e-13)
    np.testing.assert_allclose(oracle.global_fwd_linear(Q, K, V, 0.0), V, rtol=1e-13)


def test_single_token(oracle):
    rng = np.random.default_rng(9)
    Q = rng.standard_normal((1, 1, 1, 6)); K = rng.standard_normal((1, 1, 1, 6))
    V = rng.standard_normal((1, 1, 1, 3)); eps = 0.25
    a = float((oracle.phi(Q) * oracle.phi(K)).sum())
    for fwd in (oracle.causal_fwd_prefix, oracle.causal_fwd_quadratic, oracle.global_fwd_linear,
                oracle.global_fwd_quadratic):
        np.testing.assert_allclose(fwd(Q, K, V, eps), V * a / (a + eps), rtol=1e-14)
    G = rng.standard_normal((1, 1, 1, 3))
    for bwd in (oracle.causal_bwd_linear, oracle.causal_bwd_quadratic):
        _, _, dV = bwd(Q, K, V, G, eps)
        np.testing.assert_allclose(dV, G * a / (a + eps), rtol=1e-14)   # the reverse sum starts at j = i


def test_weights_nonnegative_rows_sum_to_one(oracle):
    """Config 1 of the benchmark set: N = 256, D = 32."""
    rng = np.random.default_rng(1001)
    Q = rng.standard_normal((256, 32)); K = rng.standard_normal((256, 32))
    V = rng.standard_normal((256, 32))
    eps = 1e-6
    W = oracle.causal_weights(Q, K, eps)
    O, den = oracle.causal_fwd_prefix(Q, K, V, eps, return_den=True)
    assert np.all(W >= 0.0)
    assert np.all(np.triu(W, 1) == 0.0)
    np.testing.assert_allclose(W.sum(1), 1.0 - eps / den, rtol=1e-13)
    np.testing.assert_allclose(W @ V, O, rtol=1e-11, atol=1e-13)
    # with eps > 0 the weights sum to slightly less than 1: a convex combination of the
    # rows of V seen so far and of the zero vector
    assert np.all(O <= np.maximum(np.maximum.accumulate(V, axis=0), 0.0) + 1e-12)
    assert np.all(O >= np.minimum(np.minimum.accumulate(V, axis=0), 0.0) - 1e-12)


def test_ones_column_reads_back_the_row_sum(oracle):
    B, H, N, D, M = 1, 1, 30, 8, 3
    Q, K, V, _ = _rand(10, B, H, N, D, M)
    V[..., 1] = 1.0
    eps = 1e-3
    O, den = oracle.causal_fwd_prefix(Q, K, V, eps, return_den=True)
    np.testing.assert_allclose(O[..., 1], 1.0 - eps / den, rtol=1e-13)


def test_causality_and_slab_independence(oracle):
    B, H, N, D, M = 2, 2, 40, 8, 8
    Q, K, V, _ = _rand(12, B, H, N, D, M)
    O = oracle.causal_fwd_prefix(Q, K, V)
    t = 17
    Q2, K2, V2 = Q.copy(), K.copy(), V.copy()
    Q2[:, :, t:] += 3.0; K2[:, :, t:] -= 1.0; V2[:, :, t:] *= -2.0
    O2 = oracle.causal_fwd_prefix(Q2, K2, V2)
    assert np.array_equal(O2[:, :, :t], O[:, :, :t])
    assert not np.allclose(O2[:, :, t:], O[:, :, t:])
    # prefix property: the first n rows of an N-run equal an n-run
    assert np.array_equal(oracle.causal_fwd_prefix(Q[:, :, :t], K[:, :, :t], V[:, :, :t]), O[:, :, :t])
    # slabs are independent problems
    perm = [1, 0]
    assert np.array_equal(oracle.causal_fwd_prefix(Q[perm], K[perm], V[perm]), O[perm])


def test_underflowed_features_give_zero_output(oracle):
    N, D, M = 6, 4, 2
    rng = np.random.default_rng(13)
    Q = rng.standard_normal((1, 1, N, D)); V = rng.standard_normal((1, 1, N, M))
    K = np.full((1, 1, N, D), -800.0)          # exp underflows to exactly 0 in fp64
    K[0, 0, 3:] = rng.standard_normal((N - 3, D))
    O = oracle.causal_fwd_prefix(Q, K, V, 1e-6)
    assert np.all(O[0, 0, :3] == 0.0)
    assert np.all(np.isfinite(O))


# ------------------------------------------------------------------ global forward

def test_global_linear_equals_quadratic_and_last_causal_row(oracle):
    B, H, N, D, M = 2, 2, 61, 16, 8
    Q, K, V, _ = _rand(14, B, H, N, D, M)
    for eps in (0.0, 1e-6):
        Ol = oracle.global_fwd_linear(Q, K, V, eps)
        Oq = oracle.global_fwd_quadratic(Q, K, V, eps)
        np.testing.assert_allclose(Ol, Oq, rtol=1e-12, atol=1e-13)
        Oc = oracle.causal_fwd_prefix(Q, K, V, eps)
        np.testing.assert_allclose(Oc[:, :, -1], Ol[:, :, -1], rtol=1e-12, atol=1e-13)
    fq = torch.nn.functional.elu(torch.tensor(Q)) + 1
    fk = torch.nn.functional.elu(torch.tensor(K)) + 1
    A = fq @ fk.transpose(-1, -2)
    Ot = (A @ torch.tensor(V)) / (A.sum(-1, keepdim=True) + 1e-6)
    np.testing.assert_allclose(Ol, Ot.numpy(), rtol=1e-11, atol=1e-12)


# ------------------------------------------------------------------ Algorithm 1 (numerator)

def test_algorithm1_numerator_against_autograd(oracle):
    """eq. 13-15: gradients of the numerator alone, against torch autograd of tril(QK^T)V."""
    B, H, N, C, M = 1, 2, 29, 6, 5
    rng = np.random.default_rng(15)
    fQ = rng.random((B, H, N, C)) + 0.1
    fK = rng.random((B, H, N, C)) + 0.1
    V = rng.standard_normal((B, H, N, M)); G = rng.standard_normal((B, H, N, M))
    tq, tk, tv = (torch.tensor(a, requires_grad=True) for a in (fQ, fK, V))
    vbar = torch.tril(tq @ tk.transpose(-1, -2)) @ tv
    vbar.backward(torch.tensor(G))
    np.testing.assert_allclose(oracle.causal_numerator_fwd(fQ, fK, V), vbar.detach().numpy(),
                               rtol=1e-12, atol=1e-12)
    gQ, gK, gV = oracle.causal_numerator_bwd(fQ, fK, V, G)
    np.testing.assert_allclose(gQ, tq.grad.numpy(), rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(gK, tk.grad.numpy(), rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(gV, tv.grad.numpy(), rtol=1e-11, atol=1e-12)


# ------------------------------------------------------------------ full backward

@pytest.mark.parametrize("shape", [(1, 1, 1, 3, 2), (2, 2, 23, 8, 5), (1, 1, 100, 32, 32)])
def test_bwd_linear_equals_quadratic_and_autograd(oracle, shape):
    B, H, N, D, M = shape
    Q, K, V, G = _rand(16 + N, B, H, N, D, M)
    for eps in (0.0, 1e-6, 0.3):
        lin = oracle.causal_bwd_linear(Q, K, V, G, eps)
        qua = oracle.causal_bwd_quadratic(Q, K, V, G, eps)
        tq, tk, tv = (torch.tensor(a, requires_grad=True) for a in (Q, K, V))
        O, _ = _torch_causal(tq, tk, tv, eps)
        O.backward(torch.tensor(G))
        # one common scale: for N = 1 and eps = 0 the exact dQ and dK are zero
        scale = max(np.abs(b).max() for b in qua)
        for a, b, c in zip(lin, qua, (tq.grad, tk.grad, tv.grad)):
            assert np.abs(a - b).max() / scale < 1e-12
            assert np.abs(b - c.numpy()).max() / scale < 1e-11


def test_bwd_against_central_finite_differences(oracle):
    B, H, N, D, M = 1, 1, 7, 3, 2
    Q, K, V, G = _rand(17, B, H, N, D, M)
    eps = 1e-3
    dQ, dK, dV = oracle.causal_bwd_linear(Q, K, V, G, eps)

    def loss(q, k, v):
        return float((G * oracle.causal_fwd_quadratic(q, k, v, eps)).sum())

    h = 1e-6
    for X, dX, which in ((Q, dQ, 0), (K, dK, 1), (V, dV, 2)):
        fd = np.zeros_like(X)
        for idx in np.ndindex(X.shape):
            args = [Q.copy(), K.copy(), V.copy()]
            args[which][idx] += h
            up = loss(*args)
            args[which][idx] -= 2 * h
            fd[idx] = (up - loss(*args)) / (2 * h)
        np.testing.assert_allclose(dX, fd, rtol=2e-6, atol=1e-8)


def test_bwd_closed_forms(oracle):
    B, H, N, D, M = 1, 2, 31, 4, 3
    Q, K, V, G = _rand(18, B, H, N, D, M)
    eps = 1e-4
    _, den = oracle.causal_fwd_prefix(Q, K, V, eps, return_den=True)
    _, _, dV = oracle.causal_bwd_linear(Q, K, V, G, eps)
    # columns of the weight matrix: sum_j dV_j = sum_i G_i * (row sum of weights)
    np.testing.assert_allclose(dV.sum(2), (G * (1.0 - eps / den[..., None])).sum(2), rtol=1e-12)
    # constant V and eps = 0: the output does not depend on Q, K at all
    Vc = np.broadcast_to(np.array([0.5, -1.0, 2.0]), V.shape).copy()
    dQ, dK, _ = oracle.causal_bwd_linear(Q, K, Vc, G, 0.0)
    assert np.abs(dQ).max() < 1e-13 and np.abs(dK).max() < 1e-13
    # Q = K = 0: weights are 1/i, so dV_j = sum_{i>=j} G_i * D / (D i + eps)
    Zq = np.zeros_like(Q)
    _, _, dV0 = oracle.causal_bwd_linear(Zq, Zq, V, G, eps)
    i = np.arange(1, N + 1, dtype=np.float64)[None, None, :, None]
    w = G * D / (D * i + eps)
    expect = np.flip(np.cumsum(np.flip(w, 2), 2), 2)
    np.testing.assert_allclose(dV0, expect, rtol=1e-12, atol=1e-14)


# ------------------------------------------------------------------ global backward

@pytest.mark.parametrize("shape", [(1, 1, 1, 3, 2), (2, 2, 23, 8, 5), (1, 1, 70, 32, 16)])
def test_global_bwd_linear_equals_quadratic_and_autograd(oracle, shape):
    B, H, N, D, M = shape
    Q, K, V, G = _rand(40 + N, B, H, N, D, M)
    for eps in (0.0, 1e-6, 0.3):
        lin = oracle.global_bwd_linear(Q, K, V, G, eps)
        qua = oracle.global_bwd_quadratic(Q, K, V, G, eps)
        tq, tk, tv = (torch.tensor(a, requires_grad=True) for a in (Q, K, V))
        fq = torch.nn.functional.elu(tq) + 1
        fk = torch.nn.functional.elu(tk) + 1
        A = fq @ fk.transpose(-1, -2)
        O = (A @ tv) / (A.sum(-1, keepdim=True) + eps)
        O.backward(torch.tensor(G))
        scale = max(np.abs(b).max() for b in qua)
        for a, b, c in zip(lin, qua, (tq.grad, tk.grad, tv.grad)):
            assert np.abs(a - b).max() / scale < 1e-12
            assert np.abs(b - c.numpy()).max() / scale < 1e-11


def test_global_bwd_finite_differences_and_closed_forms(oracle):
    B, H, N, D, M = 1, 1, 6, 3, 2
    Q, K, V, G = _rand(41, B, H, N, D, M)
    eps = 1e-3
    dQ, dK, dV = oracle.global_bwd_linear(Q, K, V, G, eps)

    def loss(q, k, v):
        return float((G * oracle.global_fwd_quadratic(q, k, v, eps)).sum())

    h = 1e-6
    for X, dX, which in ((Q, dQ, 0), (K, dK, 1), (V, dV, 2)):
        fd = np.zeros_like(X)
        for idx in np.ndindex(X.shape):
            args = [Q.copy(), K.copy(), V.copy()]
            args[which][idx] += h
            up = loss(*args)
            args[which][idx] -= 2 * h
            fd[idx] = (up - loss(*args)) / (2 * h)
        np.testing.assert_allclose(dX, fd, rtol=2e-6, atol=1e-8)
    # Q = K = 0: every weight is D/(D N + eps), so dV_j is the same for all j
    Zq = np.zeros_like(Q)
    _, _, dV0 = oracle.global_bwd_linear(Zq, Zq, V, G, eps)
    expect = np.broadcast_to(G.sum(2, keepdims=True) * D / (D * N + eps), V.shape)
    np.testing.assert_allclose(dV0, expect, rtol=1e-12)
    # constant V, eps = 0: the output does not depend on Q, K
    Vc = np.broadcast_to(np.array([0.5, -1.0]), V.shape).copy()
    dQc, dKc, _ = oracle.global_bwd_linear(Q, K, Vc, G, 0.0)
    assert np.abs(dQc).max() < 1e-13 and np.abs(dKc).max() < 1e-13


# ------------------------------------------------------------------ state handed in and out

def _elu1(x):
    return torch.nn.functional.elu(torch.tensor(x, dtype=torch.float64)).numpy() + 1.0


def test_state_functions_with_zero_state_are_the_plain_ones(oracle):
    Q, K, V, G = _rand(50, 2, 2, 19, 8, 5)
    O, den, S1, Z1 = oracle.causal_fwd_state(Q, K, V, None, None, 1e-6)
    ref, dref = oracle.causal_fwd_quadratic(Q, K, V, 1e-6, return_den=True)
    np.testing.assert_allclose(O, ref, rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(den, dref, rtol=1e-13)
    # the final state is the pair of sums of eq. 5-6 over the whole sequence (library einsum)
    np.testing.assert_allclose(S1, np.einsum("bhnd,bhnm->bhdm", _elu1(K), V), rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(Z1, _elu1(K).sum(2), rtol=1e-13)
    got = oracle.causal_bwd_state(Q, K, V, G, eps=1e-6)
    want = oracle.causal_bwd_quadratic(Q, K, V, G, 1e-6)
    scale = max(np.abs(b).max() for b in want)
    for a, b in zip(got[:3], want):
        assert np.abs(a - b).max() / scale < 1e-12


def test_state_equals_a_real_prefix(oracle):
    """A state built from P real tokens stands for those tokens: outputs and gradients of the
    remaining tokens equal those of the uncut sequence (brute force, eq. 8), and the gradient
    that leaves through the state reproduces the prefix tokens' dK, dV."""
    B, H, N, D, M, P = 1, 2, 17, 6, 4, 7
    Q, K, V, G = _rand(51, B, H, N, D, M)
    G[:, :, :P] = 0.0                               # the loss sees the tail only
    eps = 1e-4
    fk = _elu1(K[:, :, :P])
    S0 = np.einsum("bhnd,bhnm->bhdm", fk, V[:, :, :P])
    Z0 = fk.sum(2)
    tail = [x[:, :, P:] for x in (Q, K, V, G)]
    O, den, S1, Z1 = oracle.causal_fwd_state(*tail[:3], S0, Z0, eps)
    ref = oracle.causal_fwd_quadratic(Q, K, V, eps)
    np.testing.assert_allclose(O, ref[:, :, P:], rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(S1, np.einsum("bhnd,bhnm->bhdm", _elu1(K), V), rtol=1e-12, atol=1e-13)
    dQ, dK, dV, dS0, dZ0 = oracle.causal_bwd_state(*tail, S0, Z0, None, None, eps)
    wq, wk, wv = oracle.causal_bwd_quadratic(Q, K, V, G, eps)
    scale = max(np.abs(b).max() for b in (wq, wk, wv))
    for a, b in ((dQ, wq), (dK, wk), (dV, wv)):
        assert np.abs(a - b[:, :, P:]).max() / scale < 1e-12
    # prefix token p entered the state as phi(K_p) V_p^T and phi(K_p)
    dphi = np.where(K[:, :, :P] > 0, 1.0, np.exp(np.minimum(K[:, :, :P], 0.0)))
    dK_prefix = (np.einsum("bhdm,bhnm->bhnd", dS0, V[:, :, :P]) + dZ0[:, :, None, :]) * dphi
    dV_prefix = np.einsum("bhdm,bhnd->bhnm", dS0, fk)
    assert np.abs(dK_prefix - wk[:, :, :P]).max() / scale < 1e-12
    assert np.abs(dV_prefix - wv[:, :, :P]).max() / scale < 1e-12


def test_two_chained_pieces_equal_the_uncut_sequence(oracle):
    B, H, N, D, M, cut = 2, 1, 29, 5, 7, 11
    Q, K, V, G = _rand(52, B, H, N, D, M)
    eps = 1e-6
    a = [x[:, :, :cut] for x in (Q, K, V, G)]
    b = [x[:, :, cut:] for x in (Q, K, V, G)]
    Oa, _, Sa, Za = oracle.causal_fwd_state(*a[:3], None, None, eps)
    Ob, _, _, _ = oracle.causal_fwd_state(*b[:3], Sa, Za, eps)
    ref = oracle.causal_fwd_quadratic(Q, K, V, eps)
    np.testing.assert_allclose(np.concatenate([Oa, Ob], 2), ref, rtol=1e-12, atol=1e-14)
    gb = oracle.causal_bwd_state(*b, Sa, Za, None, None, eps)
    ga = oracle.causal_bwd_state(*a, None, None, gb[3], gb[4], eps)
    want = oracle.causal_bwd_quadratic(Q, K, V, G, eps)
    scale = max(np.abs(w).max() for w in want)
    for xa, xb, w in zip(ga[:3], gb[:3], want):
        assert np.abs(np.concatenate([xa, xb], 2) - w).max() / scale < 1e-12


def test_state_gradients_against_central_finite_differences(oracle):
    B, H, N, D, M = 1, 1, 5, 3, 2
    Q, K, V, G = _rand(53, B, H, N, D, M)
    rng = np.random.default_rng(54)
    S0 = rng.standard_normal((B, H, D, M))
    Z0 = rng.uniform(0.5, 2.0, (B, H, D))
    W = rng.standard_normal((B, H, D, M))           # dL/dS_N
    w = rng.standard_normal((B, H, D))              # dL/dZ_N
    eps = 1e-3

    def loss(q, k, v, s0, z0):
        O, _, S1, Z1 = oracle.causal_fwd_state(q, k, v, s0, z0, eps)
        return float((G * O).sum() + (W * S1).sum() + (w * Z1).sum())

    grads = oracle.causal_bwd_state(Q, K, V, G, S0, Z0, W, w, eps)
    args = [Q, K, V, S0, Z0]
    h = 1e-6
    for which, dX in enumerate(grads):
        fd = np.zeros_like(args[which])
        for idx in np.ndindex(fd.shape):
            up = [x.copy() for x in args]
            dn = [x.copy() for x in args]
            up[which][idx] += h
            dn[which][idx] -= h
            fd[idx] = (loss(*up) - loss(*dn)) / (2 * h)
        np.testing.assert_allclose(dX, fd, rtol=3e-6, atol=1e-8)


# ------------------------------------------------------------------ caller-supplied features

@pytest.fixture
def features_given(oracle):
    oracle.set_feature_map(1)
    yield oracle
    oracle.set_feature_map(0)


def test_identity_feature_map_against_torch(features_given):
    """With the identity map the oracle is attention with sim(q, k) = q . k on non-negative
    features (section 3.2): checked against torch's matmul / tril / autograd in fp64, causal
    and non-causal, and against Algorithm 1's numerator functions."""
    o = features_given
    rng = np.random.default_rng(60)
    B, H, N, C, M = 2, 2, 21, 6, 5
    FQ, FK = rng.uniform(0.05, 3.0, (2, B, H, N, C))
    V, G = rng.standard_normal((2, B, H, N, M))
    eps = 1e-4
    for causal in (True, False):
        tq, tk, tv = (torch.tensor(a, requires_grad=True) for a in (FQ, FK, V))
        A = tq @ tk.transpose(-1, -2)
        if causal:
            A = torch.tril(A)
        O = (A @ tv) / (A.sum(-1, keepdim=True) + eps)
        O.backward(torch.tensor(G))
        got = o.causal_fwd_prefix(FQ, FK, V, eps) if causal else o.global_fwd_linear(FQ, FK, V, eps)
        np.testing.assert_allclose(got, O.detach().numpy(), rtol=1e-12, atol=1e-14)
        grads = (o.causal_bwd_linear if causal else o.global_bwd_linear)(FQ, FK, V, G, eps)
        for a, b in zip(grads, (tq.grad, tk.grad, tv.grad)):
            np.testing.assert_allclose(a, b.numpy(), rtol=1e-10, atol=1e-12)
    # numerator of the causal form == Algorithm 1 forward on the same features
    num = o.causal_numerator_fwd(FQ, FK, V)
    O, den = o.causal_fwd_prefix(FQ, FK, V, eps, return_den=True)
    np.testing.assert_allclose(O * den[..., None], num, rtol=1e-12)


def test_identity_map_equals_elu_map_on_shifted_positive_inputs(oracle):
    """elu(x) + 1 = x + 1 with slope 1 for x > 0: features F = x + 1 through the identity map
    give the same outputs and gradients as raw x through eq. 7."""
    rng = np.random.default_rng(61)
    B, H, N, D, M = 1, 2, 17, 4, 3
    X = rng.uniform(0.01, 2.0, (2, B, H, N, D))
    V, G = rng.standard_normal((2, B, H, N, M))
    ref = oracle.causal_bwd_linear(X[0], X[1], V, G, 1e-6)
    oref = oracle.causal_fwd_prefix(X[0], X[1], V, 1e-6)
    oracle.set_feature_map(1)
    try:
        got = oracle.causal_bwd_linear(X[0] + 1.0, X[1] + 1.0, V, G, 1e-6)
        ogot = oracle.causal_fwd_prefix(X[0] + 1.0, X[1] + 1.0, V, 1e-6)
    finally:
        oracle.set_feature_map(0)
    np.testing.assert_allclose(ogot, oref, rtol=1e-13)
    for a, b in zip(got, ref):
        np.testing.assert_allclose(a, b, rtol=1e-12, atol=1e-15)


# ---- degree-2 polynomial kernel (section 3.2): the written-out (q . k)^2 attention ----------------

def _poly2_attention_torch(Q, K, V, eps, causal):
    """The definition with the kernel itself, no feature map: sim(q, k) = (q . k)^2 (torch fp64)."""
    A = (Q @ K.transpose(-1, -2)) ** 2
    if causal:
        A = torch.tril(A)
    return (A @ V) / (A.sum(-1, keepdim=True) + eps)


@pytest.mark.parametrize("causal", [True, False])
def test_poly2_map_is_the_squared_dot_product_kernel(oracle, causal):
    rng = np.random.default_rng(77)
    B, H, N, d, M = 2, 2, 37, 8, 5
    Q, K = rng.standard_normal((B, H, N, d)), rng.standard_normal((B, H, N, d))
    V, G = rng.standard_normal((B, H, N, M)), rng.standard_normal((B, H, N, M))
    eps = 1e-3
    # the feature map reproduces the kernel: phi(q) . phi(k) = (q . k)^2
    fq, fk = oracle.poly2_features(Q), oracle.poly2_features(K)
    assert fq.shape == (B, H, N, d * d)
    np.testing.assert_allclose(np.einsum("bhic,bhjc->bhij", fq, fk), np.einsum("bhid,bhjd->bhij", Q, K) ** 2,
                               rtol=1e-12, atol=1e-12)
    assert fq[0, 0, 3, 8 * 2 + 5] == Q[0, 0, 3, 2] * Q[0, 0, 3, 5]          # feature d*i + j = x_i x_j
    tq, tk, tv = (torch.tensor(x, dtype=torch.float64, requires_grad=True) for x in (Q, K, V))
    ref = _poly2_attention_torch(tq, tk, tv, eps, causal)
    ref.backward(torch.tensor(G))
    if causal:
        O = oracle.causal_fwd_poly2(Q, K, V, eps)
        dQ, dK, dV = oracle.causal_bwd_poly2(Q, K, V, G, eps)
    else:
        O = oracle.global_fwd_poly2(Q, K, V, eps)
        dQ, dK, dV = oracle.global_bwd_poly2(Q, K, V, G, eps)
    np.testing.assert_allclose(O, ref.detach().numpy(), rtol=1e-9, atol=1e-11)
    for got, t in ((dQ, tq), (dK, tk), (dV, tv)):
        np.testing.assert_allclose(got, t.grad.numpy(), rtol=1e-8, atol=1e-10)
    # the switch is put back: the default map is elu + 1 again
    assert oracle.phi(-1.0) == pytest.approx(np.exp(-1.0))


def test_poly2_gradients_against_finite_differences_and_recurrence(oracle):
    rng = np.random.default_rng(78)
    N, d, M = 9, 8, 3
    Q, K = rng.standard_normal((1, 1, N, d)), rng.standard_normal((1, 1, N, d))
    V, G = rng.standard_normal((1, 1, N, M)), rng.standard_normal((1, 1, N, M))
    eps = 1e-2
    dQ, dK, dV = oracle.causal_bwd_poly2(Q, K, V, G, eps)
    loss = lambda q, k, v: float((oracle.causal_fwd_poly2(q, k, v, eps) * G).sum())
    h = 1e-6
    for X, dX, which in ((Q, dQ, 0), (K, dK, 1), (V, dV, 2)):
        for idx in [(0, 0, 0, 0), (0, 0, 4, min(2, X.shape[-1] - 1)), (0, 0, N - 1, X.shape[-1] - 1)]:
            args = [Q.copy(), K.copy(), V.copy()]
            args[which][idx] += h
            up = loss(*args)
            args[which][idx] -= 2 * h
            fd = (up - loss(*args)) / (2 * h)
            assert fd == pytest.approx(dX[idx], rel=1e-5, abs=1e-8)
    # stepping the recurrence (eq. 16-20 on the mapped vectors) reproduces the parallel form
    S, z = np.zeros((1, 1, d * d, M)), np.zeros((1, 1, d * d))
    O = oracle.causal_fwd_poly2(Q, K, V, eps)
    for i in range(N):
        out = oracle.recurrent_step_poly2(Q[:, :, i], K[:, :, i], V[:, :, i], S, z, eps)
        np.testing.assert_allclose(out, O[:, :, i], rtol=1e-12, atol=1e-14)
    # the chain rule helper alone: d/dx of sum(W * vec(x x^T)) = (W + W^T) x
    x, W = rng.standard_normal(d), rng.standard_normal((d, d))
    np.testing.assert_allclose(oracle.poly2_chain(x, W.reshape(-1)), (W + W.T) @ x, rtol=1e-12)
