"""Pins for the oracle of the flow step's neighbours (Actnorm, 1 x 1 convolution) and of the step composed
with the inverse convolution: every check compares the oracle with something that is not itself - library
routines (torch conv2d and autograd, numpy slogdet), dense Jacobians built explicitly, finite differences in
float64, and a hand-worked example."""
import os

import numpy as np
import pytest
import torch
import torch.nn.functional as F

import oracle
from paper_2410_14634_amd import inputs
from tests import dense_ref as dr

HERE = os.path.dirname(os.path.abspath(__file__))
SHAPES = [(2, 1, 3, 4), (1, 2, 2, 3), (2, 3, 4, 3), (1, 4, 2, 2), (2, 5, 1, 3)]   # (B, C, H, W)


def params(C, seed):
    p = inputs.make_flow_params(C, seed)
    return p["s"].astype(np.float64), p["b"].astype(np.float64), p["Q"].astype(np.float64)


def rand(shape, seed):
    return np.random.default_rng([7, seed]).normal(size=shape)


def test_hand_worked_example():
    rows = {}
    for line in open(os.path.join(HERE, "golden", "flowstep_worked_1px.txt")):
        if line.strip() and not line.startswith("#"):
            name, *vals = line.split()
            rows[name] = np.array([float(v) for v in vals])
    x, gz = rows["x"].reshape(1, 2, 1, 1), rows["gz"].reshape(1, 2, 1, 1)
    s, b, Q = rows["s"], rows["b"], rows["Q"].reshape(2, 2)
    a = oracle.actnorm_fwd(x, s, b)
    np.testing.assert_allclose(a.ravel(), rows["a"], rtol=0, atol=1e-15)
    np.testing.assert_allclose(oracle.conv1x1_fwd(a, Q).ravel(), rows["z"], rtol=0, atol=1e-15)
    ga, gQ = oracle.conv1x1_bwd(a, Q, gz)
    np.testing.assert_allclose(ga.ravel(), rows["ga"], rtol=0, atol=1e-15)
    np.testing.assert_allclose(gQ.ravel(), rows["gQ"], rtol=0, atol=1e-15)
    gx, gs, gb = oracle.actnorm_bwd(x, s, ga)
    np.testing.assert_allclose(gx.ravel(), rows["gx"], rtol=0, atol=1e-15)
    np.testing.assert_allclose(gs, rows["gs"], rtol=0, atol=1e-15)
    np.testing.assert_allclose(gb, rows["gb"], rtol=0, atol=1e-15)
    assert oracle.actnorm_logdet(s, 1, 1) == pytest.approx(np.log(6.0), abs=1e-15)
    assert oracle.conv1x1_logdet(Q, 1, 1) == pytest.approx(np.log(2.0), abs=1e-15)


@pytest.mark.parametrize("shape", SHAPES)
def test_actnorm_and_conv1x1_match_torch_and_autograd(shape):
    B, C, H, W = shape
    s, b, Q = params(C, 3)
    x, gz = rand(shape, 1), rand(shape, 2)
    xt = torch.tensor(x, requires_grad=True)
    st, bt, Qt = (torch.tensor(t, requires_grad=True) for t in (s, b, Q))
    at = xt * st.view(1, C, 1, 1) + bt.view(1, C, 1, 1)
    zt = F.conv2d(at, Qt.view(C, C, 1, 1))              # library definition of the 1 x 1 convolution
    a = oracle.actnorm_fwd(x, s, b)
    z = oracle.conv1x1_fwd(a, Q)
    np.testing.assert_allclose(a, at.detach().numpy(), rtol=0, atol=1e-13)
    np.testing.assert_allclose(z, zt.detach().numpy(), rtol=0, atol=1e-13)
    (zt * torch.tensor(gz)).sum().backward()
    ga, gQ = oracle.conv1x1_bwd(a, Q, gz)
    gx, gs, gb = oracle.actnorm_bwd(x, s, ga)
    np.testing.assert_allclose(gx, xt.grad.numpy(), rtol=0, atol=1e-12)
    np.testing.assert_allclose(gs, st.grad.numpy(), rtol=0, atol=1e-12)
    np.testing.assert_allclose(gb, bt.grad.numpy(), rtol=0, atol=1e-12)
    np.testing.assert_allclose(gQ, Qt.grad.numpy(), rtol=0, atol=1e-12)


@pytest.mark.parametrize("shape", SHAPES)
def test_logdets_match_slogdet_of_dense_jacobians(shape):
    B, C, H, W = shape
    s, b, Q = params(C, 5)
    n = C * H * W
    # Jacobians built column by column from the forward maps (they are affine / linear, so this is exact)
    Ja, Jq = np.zeros((n, n)), np.zeros((n, n))
    zero = np.zeros((1, C, H, W))
    a0 = oracle.actnorm_fwd(zero, s, b)
    for j in range(n):
        e = zero.copy().reshape(-1)
        e[j] = 1.0
        e = e.reshape(1, C, H, W)
        Ja[:, j] = (oracle.actnorm_fwd(e, s, b) - a0).reshape(-1)
        Jq[:, j] = oracle.conv1x1_fwd(e, Q).reshape(-1)
    assert oracle.actnorm_logdet(s, H, W) == pytest.approx(np.linalg.slogdet(Ja)[1], abs=1e-11)
    assert oracle.conv1x1_logdet(Q, H, W) == pytest.approx(np.linalg.slogdet(Jq)[1], abs=1e-11)
    assert oracle.conv1x1_logdet(Q, H, W) == pytest.approx(H * W * np.linalg.slogdet(Q)[1], abs=1e-11)


def test_conv1x1_logdet_special_cases():
    assert oracle.conv1x1_logdet(np.eye(4), 5, 7) == 0.0
    P = np.eye(3)[[2, 0, 1]]                                   # a permutation: |det| = 1, needs pivoting
    assert oracle.conv1x1_logdet(P, 3, 3) == pytest.approx(0.0, abs=1e-15)
    assert oracle.conv1x1_logdet(np.diag([2.0, -0.5, 4.0]), 2, 3) == pytest.approx(6 * np.log(4.0), abs=1e-13)
    assert oracle.conv1x1_logdet(np.ones((2, 2)), 2, 2) == -np.inf


STEP_SHAPES = [(2, 1, 4, 4, 2), (1, 2, 3, 4, 3), (2, 3, 4, 3, 3), (1, 3, 2, 2, 4)]   # (B, C, H, W, k)


def step_case(shape, seed):
    B, C, H, W, k = shape
    cs = inputs.make_case(B, C, H, W, k, seed=seed, tap_std=0.3)
    s, b, Q = params(C, seed + 1)
    return cs["y"].astype(np.float64), cs["w"][0].astype(np.float64), s, b, Q, cs["g"].astype(np.float64)


@pytest.mark.parametrize("shape", STEP_SHAPES)
def test_flowstep_forward_is_the_dense_composition(shape):
    B, C, H, W, k = shape
    y, w, s, b, Q, _ = step_case(shape, 11)
    x, z = oracle.flowstep_fwd(y, w, s, b, Q)
    M = dr.dense_M(w, H, W)                                   # pixel-major, channel innermost
    A = np.kron(np.eye(H * W), Q @ np.diag(s))                # per-pixel channel map in the same ordering
    d = np.tile(Q @ b, H * W)
    for n in range(B):
        xv = np.linalg.solve(M, dr.to_vec(y[n]))
        np.testing.assert_allclose(dr.to_vec(x[n]), xv, rtol=0, atol=1e-11)
        np.testing.assert_allclose(dr.to_vec(z[n]), A @ xv + d, rtol=0, atol=1e-11)
    # log-determinant of the whole step = slogdet of its dense Jacobian A M^-1
    J = A @ np.linalg.inv(M)
    assert oracle.flowstep_logdet(w, s, Q, H, W) == pytest.approx(np.linalg.slogdet(J)[1], abs=1e-9)


@pytest.mark.parametrize("shape", STEP_SHAPES)
def test_flowstep_backward_matches_finite_differences(shape):
    B, C, H, W, k = shape
    y, w, s, b, Q, gz = step_case(shape, 21)
    x, z = oracle.flowstep_fwd(y, w, s, b, Q)
    grads = oracle.flowstep_bwd(x, w, s, b, Q, gz)

    def loss(y_=y, w_=w, s_=s, b_=b, Q_=Q):
        return float(np.sum(gz * oracle.flowstep_fwd(y_, w_, s_, b_, Q_)[1]))

    rng = np.random.default_rng(5)
    eps = 1e-6
    mask = np.ones_like(w)
    mask[:, :, k - 1, k - 1] = np.tril(np.ones((C, C)))       # masked entries have no effect and zero gradient
    for name, base, grad in (("y", y, grads["dy"]), ("w", w, grads["dw"]), ("s", s, grads["ds"]),
                             ("b", b, grads["db"]), ("Q", Q, grads["dQ"])):
        for trial in range(3):
            d = rng.normal(size=base.shape)
            if name == "w":
                d = d * mask
            kw = {name + "_": base + eps * d}
            kw2 = {name + "_": base - eps * d}
            fd = (loss(**kw) - loss(**kw2)) / (2 * eps)
            assert fd == pytest.approx(float(np.sum(grad * d)), rel=2e-6, abs=1e-7), name
    assert np.all(grads["dw"][:, :, k - 1, k - 1][np.triu_indices(C, 1)] == 0.0)


@pytest.mark.parametrize("shape", STEP_SHAPES)
def test_flowstep_backward_is_autograd_through_the_neighbours_then_the_inverse_convolution(shape):
    B, C, H, W, k = shape
    y, w, s, b, Q, gz = step_case(shape, 31)
    x, z = oracle.flowstep_fwd(y, w, s, b, Q)
    xt = torch.tensor(x, requires_grad=True)
    st, bt, Qt = (torch.tensor(t, requires_grad=True) for t in (s, b, Q))
    zt = F.conv2d(xt * st.view(1, C, 1, 1) + bt.view(1, C, 1, 1), Qt.view(C, C, 1, 1))
    np.testing.assert_allclose(z, zt.detach().numpy(), rtol=0, atol=1e-12)
    (zt * torch.tensor(gz)).sum().backward()
    grads = oracle.flowstep_bwd(x, w, s, b, Q, gz)
    np.testing.assert_allclose(grads["ds"], st.grad.numpy(), rtol=0, atol=1e-11)
    np.testing.assert_allclose(grads["db"], bt.grad.numpy(), rtol=0, atol=1e-11)
    np.testing.assert_allclose(grads["dQ"], Qt.grad.numpy(), rtol=0, atol=1e-11)
    # dL/dx from autograd, carried through the transposed dense solve (Theorem 1) and Theorem 2's sum
    M = dr.dense_M(w, H, W)
    for n in range(B):
        v = np.linalg.solve(M.T, dr.to_vec(xt.grad.numpy()[n]))
        np.testing.assert_allclose(dr.to_vec(grads["dy"][n]), v, rtol=0, atol=1e-10)


@pytest.mark.parametrize("shape", STEP_SHAPES)
def test_flowstep_logdet_gradients_match_finite_differences(shape):
    B, C, H, W, k = shape
    _, w, s, b, Q, _ = step_case(shape, 41)
    gw, gs, gQ = oracle.flowstep_logdet_grads(w, s, Q, H, W)
    eps = 1e-6
    rng = np.random.default_rng(9)
    for name, base, grad in (("w", w, gw), ("s", s, gs), ("Q", Q, gQ)):
        d = rng.normal(size=base.shape)
        if name == "w":
            m = np.ones_like(w)
            m[:, :, k - 1, k - 1] = np.tril(np.ones((C, C)))
            d = d * m
        args = dict(w=w, s=s, Q=Q)
        hi, lo = dict(args), dict(args)
        hi[name], lo[name] = base + eps * d, base - eps * d
        fd = (oracle.flowstep_logdet(hi["w"], hi["s"], hi["Q"], H, W) -
              oracle.flowstep_logdet(lo["w"], lo["s"], lo["Q"], H, W)) / (2 * eps)
        assert fd == pytest.approx(float(np.sum(grad * d)), rel=1e-6, abs=1e-6), name


def test_identity_neighbours_reduce_the_step_to_the_inverse_convolution():
    shape = (2, 3, 5, 4, 3)
    y, w, _, _, _, gz = step_case(shape, 51)
    C = 3
    x, z = oracle.flowstep_fwd(y, w, np.ones(C), np.zeros(C), np.eye(C))
    np.testing.assert_array_equal(x, z)
    grads = oracle.flowstep_bwd(x, w, np.ones(C), np.zeros(C), np.eye(C), gz)
    v, dw = oracle.invconv_bwd(x, w, gz)
    np.testing.assert_array_equal(grads["dy"], v)
    np.testing.assert_array_equal(grads["dw"], dw)
