"""Pins of the oracle's greedy training iteration (Alg. 1) and Adam update against things that are not the
oracle: torch.optim.Adam, the closed form of the first Adam step, and an independent two-module torch
model (torch.fft + conv3d + autograd + torch.optim.Adam) whose hand-off between modules is detached."""
import numpy as np
import torch

from oracle import gleam_oracle as og
from paper_2207_08393_amd import synth
from tests.test_oracle_prox import torch_prox

RNG = np.random.default_rng(77)


def test_adam_matches_torch_optim_over_several_steps():
    theta = RNG.standard_normal(50)
    m = np.zeros(50)
    v = np.zeros(50)
    p = torch.tensor(theta.copy(), requires_grad=True)
    opt = torch.optim.Adam([p], lr=3e-3, betas=(0.9, 0.999), eps=1e-8)
    for t in range(1, 8):
        g = RNG.standard_normal(50) * (0.1 if t % 2 else 10.0)
        theta, m, v = og.adam_step(theta, g, m, v, t, 3e-3)
        p.grad = torch.tensor(g)
        opt.step()
        assert np.allclose(theta, p.detach().numpy(), rtol=1e-12, atol=1e-15), t


def test_adam_first_step_closed_form_and_zero_gradient():
    theta = RNG.standard_normal(20)
    g = RNG.standard_normal(20)
    t1, m1, v1 = og.adam_step(theta, g, np.zeros(20), np.zeros(20), 1, 1e-2, eps=1e-8)
    # bias correction makes m_hat = g and v_hat = g^2 at t = 1
    assert np.allclose(t1, theta - 1e-2 * g / (np.abs(g) + 1e-8), rtol=1e-12)
    assert np.allclose(m1, 0.1 * g) and np.allclose(v1, 0.001 * g * g)
    t0, m0, v0 = og.adam_step(theta, np.zeros(20), np.zeros(20), np.zeros(20), 1, 1e-2)
    assert np.array_equal(t0, theta) and not m0.any() and not v0.any()


def torch_dc(x, S, M, y, alpha, nd):
    """u = x - alpha A^H (A x - y) with torch.fft (orthonormal, uncentred), complex128."""
    dims = tuple(range(-nd, 0))
    k = torch.fft.fftn(S[:, :, None] * x[:, None], dim=dims, norm="ortho")
    r = torch.where(M[:, None] != 0, k - y, torch.zeros_like(k))
    g = (torch.conj(S)[:, :, None] * torch.fft.ifftn(r, dim=dims, norm="ortho")).sum(1)
    return x - alpha * g


def test_greedy_iteration_vs_two_module_torch_model_with_detached_handoff():
    geom = synth.Geom(2, 2, 3, 1, 1, 6, 8)
    prox = synth.resblock_prox(3, 1)
    c = synth.make_custom(12, geom, prox, accel=2.0, centre=2, bias_std=0.1)
    n = c.theta.size
    thetas = [c.theta.astype(np.float64), (c.theta + 0.05 * RNG.standard_normal(n)).astype(np.float64)]
    ms = [0.01 * RNG.standard_normal(n) for _ in thetas]
    vs = [1e-4 * RNG.random(n) for _ in thetas]
    t, lr, alpha = 3, 2e-3, 0.7
    x_fin, losses, th2, m2, v2 = og.greedy_iteration(c.geom, c.prox, c.x_in, c.S, c.M, c.y, alpha, thetas, ms, vs, t, lr, c.x_true)

    S = torch.from_numpy(c.S.astype(np.complex128))
    M = torch.from_numpy(c.M)
    y = torch.from_numpy(c.y.astype(np.complex128))
    ref = torch.from_numpy(og.complex_to_channels(c.x_true.astype(np.complex128)))
    x = torch.from_numpy(c.x_in.astype(np.complex128))
    for i in range(2):
        p = torch.tensor(thetas[i].copy(), requires_grad=True)
        opt = torch.optim.Adam([p], lr=lr, betas=(0.9, 0.999), eps=1e-8)
        # continue an optimizer that has already taken t - 1 steps with these moments
        opt.state[p] = {"step": torch.tensor(float(t - 1)), "exp_avg": torch.tensor(ms[i].copy()),
                        "exp_avg_sq": torch.tensor(vs[i].copy())}
        u = torch_dc(x.detach(), S, M, y, alpha, 2)
        z = torch_prox(c.prox.layers, p, torch.view_as_real(u), c.geom.image_shape)
        loss = ((z - ref) ** 2).sum(-1).mean()
        loss.backward()
        opt.step()
        assert np.isclose(losses[i], loss.item(), rtol=1e-11)
        assert np.allclose(th2[i], p.detach().numpy(), rtol=1e-9, atol=1e-12)
        assert np.allclose(m2[i], opt.state[p]["exp_avg"].numpy(), rtol=1e-9, atol=1e-15)
        assert np.allclose(v2[i], opt.state[p]["exp_avg_sq"].numpy(), rtol=1e-9, atol=1e-18)
        x = torch.view_as_complex(z.detach().contiguous())   # constant input of the next module
    assert np.allclose(x_fin, x.numpy(), atol=1e-12)


def test_greedy_iteration_is_local_and_inference_reuses_modules():
    geom = synth.Geom(2, 1, 2, 1, 1, 6, 6)
    prox = synth.chain_prox([2, 3, 2], [(1, 1, 3, 3)] * 2)
    c = synth.make_custom(3, geom, prox, accel=2.0, centre=2)
    n = c.theta.size
    thetas = [c.theta + 0.02 * k * RNG.standard_normal(n) for k in range(3)]
    zeros = [np.zeros(n) for _ in thetas]
    base = og.greedy_iteration(c.geom, c.prox, c.x_in, c.S, c.M, c.y, 1.0, thetas, zeros, zeros, 1, 1e-3, c.x_true)
    # a later module's parameters do not influence an earlier module's loss or update (no backprop across modules)
    pert = [thetas[0], thetas[1], thetas[2] + 1.0]
    other = og.greedy_iteration(c.geom, c.prox, c.x_in, c.S, c.M, c.y, 1.0, pert, zeros, zeros, 1, 1e-3, c.x_true)
    assert base[1][:2] == other[1][:2]
    assert np.array_equal(base[2][0], other[2][0]) and np.array_equal(base[2][1], other[2][1])
    # the output handed on was computed with the parameters BEFORE the update
    assert np.allclose(base[0], og.unrolled_inference(c.geom, c.prox, c.x_in, c.S, c.M, c.y, 1.0, thetas), atol=1e-14)
    # early exit: the first N_inf modules alone are a valid shallower network
    x2 = og.unrolled_inference(c.geom, c.prox, c.x_in, c.S, c.M, c.y, 1.0, thetas[:2])
    f = og.module_fwd(c.geom, c.prox, x2, c.S, c.M, c.y, 1.0, thetas[2])
    assert np.allclose(f["x_out"], base[0], atol=1e-14)


def test_deep_module_gradients_vs_torch_autograd_through_dc_and_finite_differences():
    """A module of K = 3 unrolled iterations: torch differentiates through torch.fft's DC and the convs."""
    geom = synth.Geom(2, 2, 3, 1, 1, 6, 8)
    for prox in (synth.resblock_prox(3, 1), synth.chain_prox([2, 4, 2], [(1, 1, 3, 3)] * 2)):
        for loss_kind in (0, 1):
            prox.loss_kind = loss_kind
            c = synth.make_custom(14, geom, prox, accel=2.0, centre=2, bias_std=0.1)
            n = c.theta.size
            thetas = [(c.theta + 0.05 * k * RNG.standard_normal(n)).astype(np.float64) for k in range(3)]
            alpha = 0.6
            fwd = og.deep_module_fwd(c.geom, c.prox, c.x_in, c.S, c.M, c.y, alpha, thetas, c.x_true)
            grads = og.deep_module_bwd(c.geom, c.prox, c.S, c.M, alpha, thetas, fwd)
            S = torch.from_numpy(c.S.astype(np.complex128))
            M = torch.from_numpy(c.M)
            y = torch.from_numpy(c.y.astype(np.complex128))
            ref = torch.from_numpy(og.complex_to_channels(c.x_true.astype(np.complex128)))
            ps = [torch.tensor(t.copy(), requires_grad=True) for t in thetas]
            x = torch.from_numpy(c.x_in.astype(np.complex128))
            for p in ps:
                u = torch_dc(x, S, M, y, alpha, 2)
                z = torch_prox(c.prox.layers, p, torch.view_as_real(u), c.geom.image_shape)
                x = torch.view_as_complex(z.contiguous())
            d2 = ((z - ref) ** 2).sum(-1)
            loss = d2.mean() if loss_kind == 0 else torch.sqrt(d2).mean()
            loss.backward()
            assert np.isclose(fwd["loss"], loss.item(), rtol=1e-11)
            assert np.allclose(fwd["x_out"], x.detach().numpy(), atol=1e-12)
            for g, p in zip(grads, ps):
                assert np.allclose(g, p.grad.numpy(), rtol=1e-8, atol=1e-13)
    # central differences on the first iteration's parameters (their gradient crosses two DC steps)
    eps = 1e-6
    d = RNG.standard_normal(n)

    def loss_at(t0):
        return og.deep_module_fwd(c.geom, c.prox, c.x_in, c.S, c.M, c.y, alpha, [t0] + thetas[1:], c.x_true)["loss"]

    num = (loss_at(thetas[0] + eps * d) - loss_at(thetas[0] - eps * d)) / (2 * eps)
    assert np.isclose(num, grads[0] @ d, rtol=1e-5)


def test_deep_module_of_one_iteration_is_the_plain_module():
    geom = synth.Geom(2, 1, 2, 1, 1, 6, 6)
    prox = synth.chain_prox([2, 3, 2], [(1, 1, 3, 3)] * 2)
    c = synth.make_custom(4, geom, prox, accel=2.0, centre=2)
    th = c.theta.astype(np.float64)
    f1 = og.module_fwd(c.geom, c.prox, c.x_in, c.S, c.M, c.y, 0.9, th, c.x_true)
    fd = og.deep_module_fwd(c.geom, c.prox, c.x_in, c.S, c.M, c.y, 0.9, [th], c.x_true)
    assert np.array_equal(f1["x_out"], fd["x_out"]) and f1["loss"] == fd["loss"]
    assert np.array_equal(og.module_bwd(c.prox, th, f1), og.deep_module_bwd(c.geom, c.prox, c.S, c.M, 0.9, [th], fd)[0])


def test_dc_gradient_operator_is_conditioned_by_one_over_one_minus_alpha():
    """With maps normalised to sum_c |S_c|^2 = 1 and the orthonormal DFT, A^H A has its spectrum in [0, 1]; so
    I - alpha A^H A (the backward of the data-consistency step) maps any g to a norm in [(1-alpha)|g|, |g|].
    The bf16 tolerance of modules of several iterations rests on this bound."""
    c = synth.make_custom(9, synth.Geom(2, 1, 4, 1, 1, 10, 12), synth.resblock_prox(4, 1), accel=3.0, centre=2)
    rng = np.random.default_rng(2)
    alpha, nd = 0.7, c.geom.ndim_fft
    lo, hi = np.inf, 0.0
    for k in range(20):
        g = rng.standard_normal(c.geom.image_shape) + 1j * rng.standard_normal(c.geom.image_shape)
        if k % 2:                                   # half of the probes live in the sampled subspace
            g = og.sense_normal(g, c.S, c.M, nd)
        r = np.linalg.norm(g - alpha * og.sense_normal(g, c.S, c.M, nd)) / np.linalg.norm(g)
        lo, hi = min(lo, r), max(hi, r)
    assert 1 - alpha - 1e-12 <= lo and hi <= 1 + 1e-12
    assert lo < 0.6                                 # the contraction is real: sampled components do shrink


def test_step_size_gradient_vs_torch_autograd_and_finite_differences():
    """dL/dalpha of the local loss, with alpha a differentiable scalar of the torch model (torch.fft DC step,
    conv3d prox) and by central differences of the oracle's own forward pass."""
    for loss_kind, prox in ((0, synth.resblock_prox(3, 1)), (1, synth.chain_prox([2, 4, 2], [(1, 1, 3, 3)] * 2))):
        prox.loss_kind = loss_kind
        c = synth.make_custom(21 + loss_kind, synth.Geom(2, 2, 3, 1, 1, 6, 8), prox, accel=2.0, centre=2, bias_std=0.1)
        alpha = 0.6
        theta = c.theta.astype(np.float64)
        f = og.module_fwd(c.geom, c.prox, c.x_in, c.S, c.M, c.y, alpha, theta, c.x_true)
        g_theta, g_alpha = og.module_bwd_alpha(c.geom, c.prox, c.x_in, c.S, c.M, c.y, theta, f)
        assert np.allclose(g_theta, og.module_bwd(c.prox, theta, f), rtol=0, atol=0)      # same parameter gradient

        S = torch.from_numpy(c.S.astype(np.complex128)); M = torch.from_numpy(c.M)
        y = torch.from_numpy(c.y.astype(np.complex128)); x = torch.from_numpy(c.x_in.astype(np.complex128))
        a_t = torch.tensor(alpha, dtype=torch.float64, requires_grad=True)
        p = torch.tensor(theta.copy(), requires_grad=True)
        u = torch_dc(x, S, M, y, a_t, 2)
        z = torch_prox(c.prox.layers, p, torch.view_as_real(u), c.geom.image_shape)
        d = torch.view_as_complex(z.contiguous()) - torch.from_numpy(c.x_true.astype(np.complex128))
        loss = (d.abs() ** 2).mean() if loss_kind == 0 else d.abs().mean()
        loss.backward()
        assert np.isclose(g_alpha, a_t.grad.item(), rtol=1e-9)
        assert np.allclose(g_theta, p.grad.numpy(), rtol=1e-8, atol=1e-12)

        h = 1e-5
        lp = og.module_fwd(c.geom, c.prox, c.x_in, c.S, c.M, c.y, alpha + h, theta, c.x_true)["loss"]
        lm = og.module_fwd(c.geom, c.prox, c.x_in, c.S, c.M, c.y, alpha - h, theta, c.x_true)["loss"]
        assert np.isclose(g_alpha, (lp - lm) / (2 * h), rtol=1e-5)
