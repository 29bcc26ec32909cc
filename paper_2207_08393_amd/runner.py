"""Device-resident buffers for one module step: uploads a case with torch, allocates the workspace and
saved-activation buffers the library asks for, and forwards to the binding.  No arithmetic here."""
from __future__ import annotations

import numpy as np
import torch

from . import binding as gb


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def cplx(a):
    """complex64 numpy -> device tensor [..., 2] float32 (interleaved re, im)."""
    a = np.ascontiguousarray(np.asarray(a, np.complex64))
    return torch.from_numpy(a.view(np.float32).reshape(a.shape + (2,))).cuda()


def to_complex(t):
    return t.cpu().numpy().view(np.complex64).reshape(t.shape[:-1])


def byte_buffer(n):
    return torch.empty(max(int(n), 256), dtype=torch.uint8, device="cuda")


class SenseRunner:
    """gleam_sense_normal on device-resident x, S, M."""

    def __init__(self, geom, x, S, M):
        self.geom = gb.make_geom(geom)
        ws_bytes, _ = gb.gleam_workspace_bytes(self.geom, None)
        self.ws = byte_buffer(ws_bytes)
        self.x, self.S, self.M = cplx(x), cplx(S), dev(M)
        self.out = torch.full_like(self.x, float("nan"))

    def run(self):
        gb.gleam_sense_normal(self.geom, self.x, self.S, self.M, self.out, self.ws)

    def result(self):
        torch.cuda.synchronize()
        return to_complex(self.out)


def reduce_if_separable(geom, M_host, y_dev):
    """When the mask does not depend on the outermost transformed axis, that transform cancels in A^H A: takes the
    device k-space `y_dev` to hybrid space in place (gleam_kspace_to_hybrid) and returns the geometry with one
    transformed axis less; otherwise returns `geom` unchanged.  geom: a binding.gleam_geom."""
    if geom.ndim_fft < 2 or not gb.gleam_mask_constant_along_outer_axis(geom, M_host):
        return geom
    gb.gleam_kspace_to_hybrid(geom, y_dev, y_dev)
    return gb.gleam_geom(geom.ndim_fft - 1, geom.centred, geom.B, geom.C, geom.T, geom.D, geom.H, geom.W)


class ModuleRunner:
    """Device-resident copy of a case; `step()` = one gleam_module_fwd + one gleam_module_bwd.
    separable: use the reduced problem (one transformed axis less, k-space in hybrid space) when the mask allows."""

    def __init__(self, case, theta=None, alpha=None, x_in=None, separable=False):
        self.case = case
        self.geom = gb.make_geom(case.geom)
        self.prox = gb.make_prox(case.prox)
        self.S, self.M, self.y = cplx(case.S), dev(case.M), cplx(case.y)
        if separable:
            self.geom = reduce_if_separable(self.geom, case.M, self.y)
        self.ws_bytes, self.saved_bytes = gb.gleam_workspace_bytes(self.geom, self.prox)
        self.ws = byte_buffer(self.ws_bytes)
        self.saved = byte_buffer(self.saved_bytes)
        self.x_in = cplx(case.x_in if x_in is None else x_in)
        self.x_ref = cplx(case.x_true)
        self.theta = dev(np.asarray(case.theta if theta is None else theta, np.float32))
        self.alpha = float(case.alpha if alpha is None else alpha)
        self.x_out = torch.full_like(self.x_in, float("nan"))
        self.loss = torch.full((1,), float("nan"), device="cuda")
        self.grad = torch.full_like(self.theta, float("nan"))

    def fwd(self, with_ref=True):
        gb.gleam_module_fwd(self.geom, self.prox, self.x_in, self.S, self.M, self.y, self.alpha, self.theta,
                            self.x_ref if with_ref else None, self.x_out, self.loss if with_ref else None,
                            self.saved if with_ref else None, self.ws)

    def bwd(self):
        gb.gleam_module_bwd(self.geom, self.prox, self.theta, self.saved, self.grad, self.ws)

    def bwd_alpha(self):
        """Backward pass that also forms dL/dalpha (returned as a float after a synchronisation)."""
        g_alpha = torch.full((1,), float("nan"), device="cuda")
        gb.gleam_module_bwd_alpha(self.geom, self.prox, self.x_in, self.S, self.M, self.y, self.theta, self.saved, self.grad,
                                  g_alpha, self.ws)
        torch.cuda.synchronize()
        return float(g_alpha.item())

    def step(self):
        self.fwd()
        self.bwd()

    def results(self):
        torch.cuda.synchronize()
        return to_complex(self.x_out), float(self.loss.item()), self.grad.cpu().numpy()


class GreedyRunner:
    """Device-resident state of greedy training (Alg. 1): per-module parameters and Adam moments;
    `iteration()` = one gleam_greedy_iteration over the case's mini-batch."""

    def __init__(self, case, thetas, lr, alpha=None, beta1=0.9, beta2=0.999, eps=1e-8, adam_m=None, adam_v=None):
        self.case = case
        self.geom = gb.make_geom(case.geom)
        self.prox = gb.make_prox(case.prox)
        self.n_modules = len(thetas)
        self.ws_bytes, self.saved_bytes = gb.gleam_workspace_bytes(self.geom, self.prox)
        self.ws = byte_buffer(self.ws_bytes)
        self.saved = byte_buffer(self.saved_bytes)
        self.x0 = cplx(case.x_in)
        self.S, self.M, self.y = cplx(case.S), dev(case.M), cplx(case.y)
        self.x_ref = cplx(case.x_true)
        self.theta = dev(np.stack([np.asarray(t, np.float32) for t in thetas]))
        zeros = np.zeros(self.theta.shape, np.float32)
        self.m = dev(zeros if adam_m is None else np.stack([np.asarray(a, np.float32) for a in adam_m]))
        self.v = dev(zeros if adam_v is None else np.stack([np.asarray(a, np.float32) for a in adam_v]))
        self.hyper = gb.make_adam(lr, beta1, beta2, eps)
        self.alpha = float(case.alpha if alpha is None else alpha)
        self.x_out = torch.full_like(self.x0, float("nan"))
        self.x_tmp = torch.full_like(self.x0, float("nan"))
        self.losses = torch.full((self.n_modules,), float("nan"), device="cuda")
        self.grad = torch.empty(self.theta.shape[1], device="cuda")

    def iteration(self, t):
        gb.gleam_greedy_iteration(self.geom, self.prox, self.n_modules, self.x0, self.S, self.M, self.y, self.alpha,
                                  self.theta, self.m, self.v, self.hyper, t, self.x_ref, self.x_out, self.x_tmp,
                                  self.losses, self.grad, self.saved, self.ws)

    def infer(self, n_modules=None):
        gb.gleam_unrolled_infer(self.geom, self.prox, self.n_modules if n_modules is None else n_modules, self.x0,
                                self.S, self.M, self.y, self.alpha, self.theta, self.x_out, self.x_tmp, self.ws)
        torch.cuda.synchronize()
        return to_complex(self.x_out)

    def results(self):
        torch.cuda.synchronize()
        return (to_complex(self.x_out), self.losses.cpu().numpy(), self.theta.cpu().numpy(), self.m.cpu().numpy(),
                self.v.cpu().numpy())


class DeepModuleRunner:
    """A module of n_iter unrolled iterations (own parameters each): `step()` = gleam_deep_module_fwd + _bwd."""

    def __init__(self, case, thetas, alpha=None):
        self.case = case
        self.geom = gb.make_geom(case.geom)
        self.prox = gb.make_prox(case.prox)
        self.n_iter = len(thetas)
        self.ws_bytes, self.saved_bytes = gb.gleam_deep_workspace_bytes(self.geom, self.prox, self.n_iter)
        self.ws = byte_buffer(self.ws_bytes)
        self.saved = byte_buffer(self.saved_bytes)
        self.x_in = cplx(case.x_in)
        self.S, self.M, self.y = cplx(case.S), dev(case.M), cplx(case.y)
        self.x_ref = cplx(case.x_true)
        self.theta = dev(np.stack([np.asarray(t, np.float32) for t in thetas]))
        self.alpha = float(case.alpha if alpha is None else alpha)
        self.x_out = torch.full_like(self.x_in, float("nan"))
        self.x_tmp = torch.full_like(self.x_in, float("nan"))
        self.loss = torch.full((1,), float("nan"), device="cuda")
        self.grad = torch.full_like(self.theta, float("nan"))

    def step(self):
        gb.gleam_deep_module_fwd(self.geom, self.prox, self.n_iter, self.x_in, self.S, self.M, self.y, self.alpha,
                                 self.theta, self.x_ref, self.x_out, self.x_tmp, self.loss, self.saved, self.ws)
        gb.gleam_deep_module_bwd(self.geom, self.prox, self.n_iter, self.S, self.M, self.alpha, self.theta, self.saved,
                                 self.grad, self.ws)

    def results(self):
        torch.cuda.synchronize()
        return to_complex(self.x_out), float(self.loss.item()), self.grad.cpu().numpy()


class ModlRunner:
    """One MoDL module (prox, then n_cg conjugate-gradient steps on A^H A + mu I): `step()` = fwd + bwd.
    A^H y is formed once at construction with gleam_sense_adjoint."""

    def __init__(self, case, mu, n_cg, theta=None):
        self.case = case
        self.geom = gb.make_geom(case.geom)
        self.prox = gb.make_prox(case.prox)
        self.mu, self.n_cg = float(mu), int(n_cg)
        self.ws_bytes, self.saved_bytes = gb.gleam_modl_workspace_bytes(self.geom, self.prox)
        self.ws = byte_buffer(self.ws_bytes)
        self.saved = byte_buffer(self.saved_bytes)
        self.x_in = cplx(case.x_in)
        self.S, self.M, self.y = cplx(case.S), dev(case.M), cplx(case.y)
        self.x_ref = cplx(case.x_true)
        self.theta = dev(np.asarray(case.theta if theta is None else theta, np.float32))
        self.aty = torch.full_like(self.x_in, float("nan"))
        gb.gleam_sense_adjoint(self.geom, self.S, self.M, self.y, self.aty, self.ws)
        self.x_out = torch.full_like(self.x_in, float("nan"))
        self.loss = torch.full((1,), float("nan"), device="cuda")
        self.grad = torch.full_like(self.theta, float("nan"))

    def step(self):
        gb.gleam_modl_module_fwd(self.geom, self.prox, self.x_in, self.S, self.M, self.aty, self.mu, self.n_cg, self.theta,
                                 self.x_ref, self.x_out, self.loss, self.saved, self.ws)
        gb.gleam_modl_module_bwd(self.geom, self.prox, self.S, self.M, self.mu, self.n_cg, self.theta, self.saved, self.grad,
                                 self.ws)

    def results(self):
        torch.cuda.synchronize()
        return to_complex(self.x_out), float(self.loss.item()), self.grad.cpu().numpy(), to_complex(self.aty)
