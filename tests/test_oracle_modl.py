"""Pins of the oracle's MoDL module (MoDL section, Eq. 6-8) against things other than itself: a dense solve of
the normal equations, the Krylov-subspace optimality that defines the k-th CG iterate, a closed form where
A^H A = I, and torch autograd through torch.linalg.solve for the module gradient."""
import numpy as np
import torch

from oracle import gleam_oracle as og
from paper_2207_08393_amd import synth
from tests.test_oracle_prox import torch_prox

RNG = np.random.default_rng(77)


def dense_q(c, b, mu):
    """Q = A^H A + mu I of batch sample b as an explicit n x n matrix, one unit vector at a time."""
    shp = c.geom.image_shape[1:]
    n = int(np.prod(shp))
    Q = np.zeros((n, n), np.complex128)
    for i in range(n):
        e = np.zeros((1,) + shp, np.complex128)
        e.reshape(-1)[i] = 1.0
        Q[:, i] = og.sense_normal(e, c.S[b:b + 1], c.M[b:b + 1], c.geom.ndim_fft).reshape(-1)
    return Q + mu * np.eye(n)


def small_case(seed=4, B=2):
    geom = synth.Geom(2, B, 3, 1, 1, 4, 6)
    return synth.make_custom(seed, geom, synth.resblock_prox(3, 1), accel=2.0, centre=2, bias_std=0.1)


def test_cg_reaches_the_dense_solution_and_is_per_sample():
    c = small_case()
    mu, nd = 0.3, c.geom.ndim_fft
    b = RNG.standard_normal(c.geom.image_shape) + 1j * RNG.standard_normal(c.geom.image_shape)
    b[1] *= 50.0                                      # very different scales: shared step sizes would show
    x = og.cg_solve(b.shape, c.S, c.M, mu, b, 30, nd)
    for s in range(2):
        ref = np.linalg.solve(dense_q(c, s, mu), b[s].reshape(-1)).reshape(b.shape[1:])
        assert np.allclose(x[s], ref, rtol=1e-9, atol=1e-10 * np.abs(ref).max())
        # a truncated solve of the batch equals the truncated solve of each sample alone
        alone = og.cg_solve(b[s:s + 1].shape, c.S[s:s + 1], c.M[s:s + 1], mu, b[s:s + 1], 3, nd)
        both = og.cg_solve(b.shape, c.S, c.M, mu, b, 3, nd)
        assert np.allclose(both[s], alone[0], rtol=1e-12, atol=1e-13)


def test_truncated_cg_iterate_is_the_krylov_energy_minimiser():
    """The k-th CG iterate from zero minimises the Q-norm of the error over span{b, Qb, .., Q^(k-1) b}: solving
    that small least-squares problem directly must give the same vector."""
    c = small_case(seed=6, B=1)
    mu, nd = 0.05, c.geom.ndim_fft
    b = RNG.standard_normal(c.geom.image_shape) + 1j * RNG.standard_normal(c.geom.image_shape)
    Q = dense_q(c, 0, mu)
    bv = b.reshape(-1)
    for k in (1, 2, 4):
        V = np.stack([np.linalg.matrix_power(Q, j) @ bv for j in range(k)], axis=1)
        V, _ = np.linalg.qr(V)
        coef = np.linalg.solve(V.conj().T @ Q @ V, V.conj().T @ bv)
        x = og.cg_solve(b.shape, c.S, c.M, mu, b, k, nd)
        assert np.allclose(x.reshape(-1), V @ coef, rtol=1e-9, atol=1e-11)
        # and it is not yet the full solution, so the test can tell k from k + 1
        assert np.linalg.norm(V @ coef - np.linalg.solve(Q, bv)) > 1e-3 * np.linalg.norm(bv)


def test_cg_closed_form_when_the_normal_operator_is_the_identity():
    """One coil of unit magnitude, full sampling: A^H A = I, so x = b / (1 + mu) after the first step, and the
    zero residual that follows must not produce NaNs."""
    geom = synth.Geom(2, 2, 1, 1, 1, 4, 6)
    S = np.exp(1j * RNG.standard_normal((2, 1, 1, 4, 6)))
    M = np.ones(geom.image_shape, np.uint8)
    b = RNG.standard_normal(geom.image_shape) + 1j * RNG.standard_normal(geom.image_shape)
    b[1] = 0.0                                        # an all-zero right-hand side stays at zero
    for n in (1, 5):
        x = og.cg_solve(b.shape, S, M, 0.5, b, n, 2)
        assert np.all(np.isfinite(x)) and np.allclose(x, b / 1.5, rtol=1e-12, atol=1e-14)


def test_modl_module_forward_and_gradient_vs_torch_dense_solve():
    for loss_kind in (0, 1):
        c = small_case(seed=8 + loss_kind)
        c.prox.loss_kind = loss_kind
        mu, n_cg, nd = 0.4, 40, c.geom.ndim_fft      # 24 unknowns per sample: 40 steps are a converged solve
        aty = og.sense_adjoint(c.y.astype(np.complex128), c.S, c.M, nd)
        theta = c.theta.astype(np.float64)
        f = og.modl_module_fwd(c.geom, c.prox, c.x_in, c.S, c.M, aty, mu, n_cg, theta, c.x_true)
        g = og.modl_module_bwd(c.geom, c.prox, c.S, c.M, mu, n_cg, theta, f)

        p = torch.tensor(theta.copy(), requires_grad=True)
        x_in = torch.from_numpy(c.x_in.astype(np.complex128))
        z = torch.view_as_complex(torch_prox(c.prox.layers, p, torch.view_as_real(x_in), c.geom.image_shape).contiguous())
        outs = []
        for s in range(c.geom.B):
            Q = torch.from_numpy(dense_q(c, s, mu))
            rhs = torch.from_numpy(aty[s].reshape(-1)) + mu * z[s].reshape(-1)
            outs.append(torch.linalg.solve(Q, rhs).reshape(z.shape[1:]))
        x_out = torch.stack(outs)
        d = x_out - torch.from_numpy(c.x_true.astype(np.complex128))
        loss = (d.abs() ** 2).mean() if loss_kind == 0 else d.abs().mean()
        loss.backward()
        assert np.allclose(f["x_out"], x_out.detach().numpy(), rtol=1e-9, atol=1e-11)
        assert np.isclose(f["loss"], loss.item(), rtol=1e-10)
        gt = p.grad.numpy()
        assert np.linalg.norm(g - gt) <= 1e-8 * np.linalg.norm(gt)


def test_modl_gradient_uses_the_same_truncated_solve_and_scales_with_mu():
    """With few CG steps the backward pass is by definition mu * CG_k(dL/dx) pushed through the prox: the
    input gradient of the prox sweep must equal that vector, built here from the Krylov minimiser."""
    c = small_case(seed=10, B=1)
    mu, k, nd = 0.7, 2, c.geom.ndim_fft
    aty = og.sense_adjoint(c.y.astype(np.complex128), c.S, c.M, nd)
    theta = c.theta.astype(np.float64)
    f = og.modl_module_fwd(c.geom, c.prox, c.x_in, c.S, c.M, aty, mu, k, theta, c.x_true)
    Q = dense_q(c, 0, mu)
    gx = og.channels_to_complex(f["g_x"]).reshape(-1)
    V, _ = np.linalg.qr(np.stack([gx, Q @ gx], axis=1))
    gz = mu * (V @ np.linalg.solve(V.conj().T @ Q @ V, V.conj().T @ gx)).reshape(c.geom.image_shape)
    expect = og.prox_bwd(c.prox.layers, theta, f["t"], f["conv_in"], f["act"], og.complex_to_channels(gz))
    got = og.modl_module_bwd(c.geom, c.prox, c.S, c.M, mu, k, theta, f)
    assert np.linalg.norm(got - expect) <= 1e-10 * np.linalg.norm(expect)
