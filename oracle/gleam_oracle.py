"""CPU oracle for one GLEAM module step of an unrolled PGD network.  TEST INFRASTRUCTURE ONLY.

Only the tests, the smoke check and the benchmark's CPU-baseline leg may import this file; the
product (the HIP library and its binding) never does, and this file imports nothing of the
product.  Everything is float64 / complex128 numpy, written as the plain definitions:

  * F        : orthonormal DFT applied as an explicit n x n matrix product per axis (direct O(n^2) definition; `F`
               of the sensing model, Eq. 1), uncentred by default (zero frequency at index 0) or, for a geometry
               with `centred` set, with frequency and spatial origin in the middle of every transformed axis
  * A        : A = Omega F S and its Hermitian transpose A^H = S^H F^H Omega (Eq. 1, Eq. 2, PGD section)
  * DC       : u = x - alpha A^H (A x - y), alpha = 2t   (data-consistency step of PGD, Eq. 3, read with
               the same iterate on both sides)
  * prox     : learned proximal CNN f_theta (Eq. 4-5): cross-correlation, zero "same" padding,
               stride 1, ReLU, residual skips; one tap at a time with a matmul over input channels
  * loss     : local greedy objective L(f_theta(DC(x_in)), x_ref) (Eq. 10), mean squared or mean
               absolute complex error
  * backward : analytic reverse sweep for dL/dtheta of this module only (Alg. 1, gradient step);
               nothing is propagated to x_in, S or y (decoupled modules).

  * alpha    : gradient of the local loss with respect to the step size of the data-consistency step
  * deep     : a module of K = N/M unrolled iterations (GLEAM section): backpropagation inside the module,
               through its prox networks and data-consistency steps, none beyond its input
  * MoDL     : the half-quadratic-splitting module (MoDL section, Eq. 6-8): z = f_theta(x), then
               x+ = (A^H A + mu I)^-1 (A^H y + mu z) by a fixed number of conjugate-gradient steps from zero,
               one system per batch sample; the backward pass applies the same truncated solve to the loss
               gradient (the inverse is Hermitian) and stops at the module input
  * greedy   : Alg. 1 for one mini-batch: modules in order, each with its own parameters, local loss,
               local gradient and Adam update (beta1 = 0.9, beta2 = 0.999, Implementation Details); the
               detached output of module m is the input of module m + 1
  * Adam     : Kingma & Ba's update with bias correction (the optimizer the paper names)

  * bf16     : the same prox with the library's bfloat16 rounding points (the paper does not state a precision;
               this is the reading the bf16 configuration is built to): the stored activations t_1..t_{L-1} and the
               stored gradients G_1..G_{L-1} are rounded to bfloat16 (nearest even), and so are a layer's weights
               wherever they multiply such a tensor (forward pass of every layer but the first, data gradient of
               every layer but the last); everything else stays exact.  The ReLU masks are then decided from the rounded activations, as on the device, so
               that the two sides take that 0/1 decision in the same precision.  Off by default.

Pins (tests/test_oracle_*.py): numpy.fft and closed forms for the DFT, the adjoint identity, the
full-sampling identity A^H A = I, circular-convolution form of a single-coil 1D mask, scipy
correlate and torch CPU convolutions for the prox, central finite differences and torch autograd
for the gradient; torch.optim.Adam, the closed-form first step and a two-module torch autograd model
with a detached hand-off for the greedy iteration; a dense solve, the Krylov-subspace optimality of the
truncated iterate and torch autograd through torch.linalg.solve for the MoDL module.  No function here is unpinned.

Array layouts: image [B,T,D,H,W], coils [B,C,D,H,W], mask [B,T,D,H,W], k-space [B,C,T,D,H,W],
activations [B,T,D,H,W,channels] (an image is its own 2-channel activation: re, im).
"""
from __future__ import annotations

import numpy as np


# ----------------------------------------------------------------------------- Fourier
def dft_matrix(n: int, inverse: bool = False, centred: bool = False) -> np.ndarray:
    """F[q, j] = n^(-1/2) exp(-+ 2 pi i ((j - c)(q - c) mod n) / n), with c = 0 (zero frequency and the spatial origin
    at index 0) or, centred, c = floor(n/2) (both in the middle of the array: the transform that the MRI literature
    writes as fftshift . F . ifftshift).  The paper leaves the convention of `F` in Eq. 1 open; uncentred is the
    default reading here and the centred one a variant."""
    c = n // 2 if centred else 0
    j = np.arange(n, dtype=np.int64) - c
    jq = np.outer(j, j) % n
    sign = 1.0 if inverse else -1.0
    return np.exp(sign * 2j * np.pi * jq / n) / np.sqrt(n)


def dft_axis(a: np.ndarray, axis: int, inverse: bool = False, centred: bool = False) -> np.ndarray:
    """X[..., q, ...] = sum_j F[q, j] a[..., j, ...] along one axis."""
    F = dft_matrix(a.shape[axis], inverse, centred)
    moved = np.moveaxis(np.asarray(a, np.complex128), axis, -1)
    return np.moveaxis(moved @ F.T, -1, axis)


def dft_nd(a: np.ndarray, ndim_fft: int, inverse: bool = False, centred: bool = False) -> np.ndarray:
    """Separable DFT over the last `ndim_fft` axes."""
    out = np.asarray(a, np.complex128)
    for ax in range(a.ndim - ndim_fft, a.ndim):
        out = dft_axis(out, ax, inverse, centred)
    return out


def _centred(geom) -> bool:
    return bool(getattr(geom, "centred", 0))


# ----------------------------------------------------------------------------- SENSE operator
def sense_forward(x, S, M, ndim_fft, centred=False):
    """A x = Omega F S x  ->  k-space [B,C,T,D,H,W]."""
    x = np.asarray(x, np.complex128)
    S = np.asarray(S, np.complex128)
    c = S[:, :, None] * x[:, None]
    k = dft_nd(c, ndim_fft, centred=centred)
    return np.where((np.asarray(M) != 0)[:, None], k, 0.0)


def sense_adjoint(k, S, M, ndim_fft, centred=False):
    """A^H k = S^H F^H Omega k  ->  image [B,T,D,H,W]."""
    S = np.asarray(S, np.complex128)
    r = np.where((np.asarray(M) != 0)[:, None], np.asarray(k, np.complex128), 0.0)
    rt = dft_nd(r, ndim_fft, inverse=True, centred=centred)
    return (np.conj(S)[:, :, None] * rt).sum(axis=1)


def sense_normal(x, S, M, ndim_fft, centred=False):
    """A^H A x."""
    return sense_adjoint(sense_forward(x, S, M, ndim_fft, centred), S, M, ndim_fft, centred)


def masked_residual(x, S, M, y, ndim_fft, centred=False):
    """r = Omega (F S x - y): exactly zero off the mask, whatever y holds there."""
    x = np.asarray(x, np.complex128)
    S = np.asarray(S, np.complex128)
    k = dft_nd(S[:, :, None] * x[:, None], ndim_fft, centred=centred)
    return np.where((np.asarray(M) != 0)[:, None], k - np.asarray(y, np.complex128), 0.0)


def dc_step(x, S, M, y, alpha, ndim_fft, centred=False):
    """u = x - alpha A^H (A x - y)."""
    r = masked_residual(x, S, M, y, ndim_fft, centred)
    g = sense_adjoint(r, S, np.ones_like(np.asarray(M)), ndim_fft, centred)
    return np.asarray(x, np.complex128) - alpha * g


# ----------------------------------------------------------------------------- convolutions
def _pad(a, k):
    """Zero 'same' padding of [B,T,D,H,W,ch] for odd kernel extents k = (kt,kd,kh,kw)."""
    pads = [(0, 0)] + [(e // 2, e // 2) for e in k] + [(0, 0)]
    return np.pad(a, pads)


def conv_fwd(a, w, b=None):
    """out[.., p, co] = b[co] + sum_{tap, ci} w[co, tap, ci] a[.., p + tap - floor(k/2), ci],
    zero outside the grid.  a [B,T,D,H,W,cin], w [cout,kt,kd,kh,kw,cin]."""
    a = np.asarray(a, np.float64)
    w = np.asarray(w, np.float64)
    B, T, D, H, W, _ = a.shape
    k = w.shape[1:5]
    ap = _pad(a, k)
    out = np.zeros((B, T, D, H, W, w.shape[0]))
    for it in range(k[0]):
        for i_d in range(k[1]):
            for ih in range(k[2]):
                for iw in range(k[3]):
                    out += ap[:, it:it + T, i_d:i_d + D, ih:ih + H, iw:iw + W, :] @ w[:, it, i_d, ih, iw, :].T
    if b is not None:
        out += np.asarray(b, np.float64)
    return out


def conv_dgrad(g, w):
    """g_in[.., p, ci] = sum_{tap, co} w[co, tap, ci] g[.., p - (tap - floor(k/2)), co]
    (transpose of conv_fwd with respect to its input)."""
    g = np.asarray(g, np.float64)
    w = np.asarray(w, np.float64)
    B, T, D, H, W, _ = g.shape
    k = w.shape[1:5]
    gp = _pad(g, k)
    out = np.zeros((B, T, D, H, W, w.shape[5]))
    for it in range(k[0]):
        for i_d in range(k[1]):
            for ih in range(k[2]):
                for iw in range(k[3]):
                    st, sd, sh, sw = k[0] - 1 - it, k[1] - 1 - i_d, k[2] - 1 - ih, k[3] - 1 - iw
                    out += gp[:, st:st + T, sd:sd + D, sh:sh + H, sw:sw + W, :] @ w[:, it, i_d, ih, iw, :]
    return out


def conv_wgrad(g, a, k):
    """dw[co, tap, ci] = sum_{b, p} g[b, p, co] a[b, p + tap - floor(k/2), ci];  db[co] = sum g."""
    g = np.asarray(g, np.float64)
    a = np.asarray(a, np.float64)
    B, T, D, H, W, cout = g.shape
    cin = a.shape[-1]
    ap = _pad(a, k)
    dw = np.zeros((cout,) + tuple(k) + (cin,))
    g2 = g.reshape(-1, cout)
    for it in range(k[0]):
        for i_d in range(k[1]):
            for ih in range(k[2]):
                for iw in range(k[3]):
                    sl = ap[:, it:it + T, i_d:i_d + D, ih:ih + H, iw:iw + W, :].reshape(-1, cin)
                    dw[:, it, i_d, ih, iw, :] = g2.T @ sl
    return dw, g2.sum(axis=0)


# ----------------------------------------------------------------------------- prox network
def round_bf16(a):
    """Nearest-even rounding of float32(a) to bfloat16 (8 bits of significand), returned as float64."""
    x = np.ascontiguousarray(np.asarray(a, np.float64).astype(np.float32))
    bits = x.view(np.uint32).astype(np.uint64)
    bits = (bits + 0x7FFF + ((bits >> 16) & 1)) & 0xFFFF0000
    return bits.astype(np.uint32).view(np.float32).reshape(x.shape).astype(np.float64)


def split_theta(layers, theta):
    """Views (w, b) per layer out of the flat parameter vector: per layer
    w[cout][kt][kd][kh][kw][cin] then b[cout] when the layer has a bias."""
    theta = np.asarray(theta, np.float64)
    out, o = [], 0
    for l in layers:
        nw = l.cout * l.kt * l.kd * l.kh * l.kw * l.cin
        w = theta[o:o + nw].reshape(l.cout, l.kt, l.kd, l.kh, l.kw, l.cin)
        o += nw
        b = None
        if l.has_bias:
            b = theta[o:o + l.cout]
            o += l.cout
        out.append((w, b))
    assert o == theta.size, "theta length does not match the prox description"
    return out


def complex_to_channels(x):
    x = np.asarray(x, np.complex128)
    return np.stack([x.real, x.imag], axis=-1)


def channels_to_complex(a):
    return a[..., 0] + 1j * a[..., 1]


def _weights_bf16(params, keep_exact):
    """Weights rounded to bfloat16 wherever they multiply a bfloat16 tensor: every layer but `keep_exact`, whose other
    operand is float32 (the first layer's input u going forward, the last layer's incoming gradient going back)."""
    return [(w if i == keep_exact else round_bf16(w), b) for i, (w, b) in enumerate(params)]


def prox_fwd(layers, theta, u, bf16_points=False):
    """Tensors t_0 = u (2 channels) ... t_L = z, and per layer the conv input and the value
    before the skip add (needed for the ReLU derivatives).  With bf16_points the weights of every layer but the first
    and every stored interior tensor t_1..t_{L-1} (after bias, ReLU and skip add) are rounded to bfloat16."""
    params = split_theta(layers, theta)
    if bf16_points:
        params = _weights_bf16(params, keep_exact=0)
    L = len(layers)
    t = [complex_to_channels(u)]
    conv_in, act = [], []
    for i, (l, (w, b)) in enumerate(zip(layers, params)):
        a = t[-1]
        if l.relu_in:
            a = np.maximum(a, 0.0)
        v = conv_fwd(a, w, b)
        if l.relu_out:
            v = np.maximum(v, 0.0)
        out = v + t[l.skip_src] if l.skip_src >= 0 else v
        if bf16_points and i < L - 1:
            out = round_bf16(out)
            if l.skip_src < 0:
                v = out              # the ReLU mask of this layer is read off the stored value
        conv_in.append(a)
        act.append(v)
        t.append(out)
    return t, conv_in, act


def loss_and_grad(z, x_ref, loss_kind):
    """L and dL/dz (as 2 real channels).  kind 0: mean |z-x|^2;  kind 1: mean |z-x| with the
    complex magnitude, sub-gradient 0 where z == x."""
    d = np.asarray(z, np.complex128) - np.asarray(x_ref, np.complex128)
    n = d.size
    if loss_kind == 0:
        return float((np.abs(d) ** 2).sum() / n), complex_to_channels(2.0 * d / n)
    mag = np.abs(d)
    safe = np.where(mag > 0, mag, 1.0)
    return float(mag.sum() / n), complex_to_channels(np.where(mag > 0, d / safe, 0.0) / n)


def prox_bwd(layers, theta, t, conv_in, act, g_z, want_input_grad=False, bf16_points=False):
    """dL/dtheta (flat, same layout as theta) from dL/dz.  The gradient reaching t_0 = u is dropped (modules
    are decoupled) unless want_input_grad, which returns (dL/dtheta, dL/du as 2 real channels): a module
    that holds several unrolled iterations backpropagates through its own iterations.  With bf16_points (t, conv_in
    and act then come from prox_fwd with the same flag) the weights of every layer but the last, as the data gradient
    uses them, and every stored interior gradient G_1..G_{L-1} (complete: data gradient plus skip gradient) are
    rounded to bfloat16."""
    params = split_theta(layers, theta)
    if bf16_points:
        params = _weights_bf16(params, keep_exact=len(layers) - 1)
    L = len(layers)
    G = [None] * (L + 1)
    G[L] = g_z
    grads = [None] * L
    for i in range(L - 1, -1, -1):
        l = layers[i]
        w, b = params[i]
        g = G[i + 1]
        if g is None:
            g = np.zeros_like(act[i])
        elif bf16_points and i + 1 < L:
            g = round_bf16(g)        # every contribution has arrived by now: one rounding of the stored tensor
        if l.skip_src >= 0:
            s = l.skip_src
            G[s] = g if G[s] is None else G[s] + g
        gc = g * (act[i] > 0) if l.relu_out else g
        dw, db = conv_wgrad(gc, conv_in[i], (l.kt, l.kd, l.kh, l.kw))
        grads[i] = (dw, db if l.has_bias else None)
        if i >= 1 or want_input_grad:
            gin = conv_dgrad(gc, w)
            if l.relu_in:
                gin = gin * (t[i] > 0)
            G[i] = gin if G[i] is None else G[i] + gin
    flat = []
    for dw, db in grads:
        flat.append(dw.ravel())
        if db is not None:
            flat.append(db.ravel())
    if want_input_grad:
        return np.concatenate(flat), G[0]
    return np.concatenate(flat)


# ----------------------------------------------------------------------------- module
def module_fwd(geom, prox, x_in, S, M, y, alpha, theta, x_ref=None, bf16_points=False):
    """x_out = f_theta(DC(x_in)); loss against x_ref when given.  Returns a dict holding
    everything module_bwd needs."""
    u = dc_step(x_in, S, M, y, alpha, geom.ndim_fft, _centred(geom))
    t, conv_in, act = prox_fwd(prox.layers, theta, u, bf16_points)
    z = channels_to_complex(t[-1])
    out = {"u": u, "x_out": z, "t": t, "conv_in": conv_in, "act": act, "loss": None, "g_z": None,
           "bf16_points": bf16_points}
    if x_ref is not None:
        out["loss"], out["g_z"] = loss_and_grad(z, x_ref, prox.loss_kind)
    return out


def module_bwd(prox, theta, fwd):
    """dL/dtheta_m of the local objective; stops at the module input."""
    return prox_bwd(prox.layers, theta, fwd["t"], fwd["conv_in"], fwd["act"], fwd["g_z"],
                    bf16_points=fwd.get("bf16_points", False))


def module_bwd_alpha(geom, prox, x_in, S, M, y, theta, fwd):
    """Gradients of the local loss with respect to theta and to the step size alpha = 2t of the module's
    data-consistency step (Eq. 3), for a learnable step size.  u = x - alpha r with r = A^H (A x - y), so
    dL/dalpha = -<dL/du, r> over the real and imaginary parts; still nothing goes to x_in."""
    g_theta, g_u = prox_bwd(prox.layers, theta, fwd["t"], fwd["conv_in"], fwd["act"], fwd["g_z"], want_input_grad=True)
    r = sense_adjoint(masked_residual(x_in, S, M, y, geom.ndim_fft, _centred(geom)), S, M, geom.ndim_fft, _centred(geom))
    return g_theta, float(-(g_u * complex_to_channels(r)).sum())


# ----------------------------------------------------------------------------- module of several iterations
def deep_module_fwd(geom, prox, x_in, S, M, y, alpha, thetas, x_ref=None, bf16_points=False):
    """A module that holds K = N/M unrolled iterations (GLEAM section, N > M): x_j = f_theta_j(DC(x_{j-1})),
    j = 1..K, with the local loss on x_K only.  Returns the per-iteration forward records."""
    x = np.asarray(x_in, np.complex128)
    recs = []
    for j, th in enumerate(thetas):
        last = j == len(thetas) - 1
        recs.append(module_fwd(geom, prox, x, S, M, y, alpha, th, x_ref if last else None, bf16_points))
        x = recs[-1]["x_out"]
    return {"x_out": x, "loss": recs[-1]["loss"], "iters": recs}


def deep_module_bwd(geom, prox, S, M, alpha, thetas, fwd):
    """Gradients of the module's loss with respect to theta_1..theta_K (list): backpropagation inside the
    module, through every prox and every data-consistency step.  DC is affine in x with the Hermitian
    linear part I - alpha A^H A, so dL/dx_{j-1} = g_u - alpha A^H A g_u with g_u = dL/du_j (complex view of
    the two real channels).  Nothing is propagated to the module's input."""
    K = len(thetas)
    grads = [None] * K
    g_out = fwd["iters"][-1]["g_z"]
    bf = fwd["iters"][-1].get("bf16_points", False)   # the hand-off between iterations stays exact either way
    for j in range(K - 1, -1, -1):
        r = fwd["iters"][j]
        if j == 0:
            grads[j] = prox_bwd(prox.layers, thetas[j], r["t"], r["conv_in"], r["act"], g_out, bf16_points=bf)
        else:
            grads[j], g_u = prox_bwd(prox.layers, thetas[j], r["t"], r["conv_in"], r["act"], g_out, want_input_grad=True,
                                     bf16_points=bf)
            gc = channels_to_complex(g_u)
            g_out = complex_to_channels(gc - alpha * sense_normal(gc, S, M, geom.ndim_fft, _centred(geom)))
    return grads


# ----------------------------------------------------------------------------- MoDL module (Eq. 6-8)
def cg_solve(x_shape, S, M, mu, b, n_cg, ndim_fft, centred=False):
    """n_cg conjugate-gradient steps from x = 0 on (A^H A + mu I) x = b, one system per batch sample
    (leading axis): the textbook recurrence
        a = <r,r> / <p, Q p> ; x += a p ; r -= a Q p ; beta = <r,r>_new / <r,r>_old ; p = r + beta p.
    A sample whose residual is exactly zero stops moving (a = beta = 0) instead of dividing by zero."""
    b = np.asarray(b, np.complex128)
    x = np.zeros(x_shape, np.complex128)
    r = b.copy()
    p = b.copy()
    B = b.shape[0]
    axes = tuple(range(1, b.ndim))
    bc = (slice(None),) + (None,) * (b.ndim - 1)
    rr = np.sum(np.abs(r) ** 2, axis=axes)
    for _ in range(n_cg):
        Qp = sense_normal(p, S, M, ndim_fft, centred) + mu * p
        pQp = np.sum((np.conj(p) * Qp).real, axis=axes)
        a = np.where(pQp > 0, rr / np.where(pQp > 0, pQp, 1.0), 0.0)
        x = x + a[bc] * p
        r = r - a[bc] * Qp
        rr_new = np.sum(np.abs(r) ** 2, axis=axes)
        beta = np.where(rr > 0, rr_new / np.where(rr > 0, rr, 1.0), 0.0)
        p = r + beta[bc] * p
        rr = rr_new
    assert x.shape[0] == B
    return x


def modl_module_fwd(geom, prox, x_in, S, M, aty, mu, n_cg, theta, x_ref=None):
    """One MoDL module: z = f_theta(x_in) (Eq. 8), x_out = (A^H A + mu I)^-1 (A^H y + mu z) by n_cg CG steps
    (Eq. 7); aty is A^H y.  Loss against x_ref when given."""
    t, conv_in, act = prox_fwd(prox.layers, theta, np.asarray(x_in, np.complex128))
    z = channels_to_complex(t[-1])
    x_out = cg_solve(z.shape, S, M, mu, np.asarray(aty, np.complex128) + mu * z, n_cg, geom.ndim_fft, _centred(geom))
    out = {"z": z, "x_out": x_out, "t": t, "conv_in": conv_in, "act": act, "loss": None, "g_x": None}
    if x_ref is not None:
        out["loss"], out["g_x"] = loss_and_grad(x_out, x_ref, prox.loss_kind)
    return out


def modl_module_bwd(geom, prox, S, M, mu, n_cg, theta, fwd):
    """dL/dtheta of the MoDL module.  x_out = Q^-1 (A^H y + mu z) with Q = A^H A + mu I Hermitian, so
    dL/dz = mu Q^-1 dL/dx_out; the inverse is again applied by n_cg CG steps (the same truncated solve as
    the forward pass), then the prox is swept backwards.  Nothing goes to the module input."""
    gx = channels_to_complex(fwd["g_x"])
    g_z = complex_to_channels(mu * cg_solve(gx.shape, S, M, mu, gx, n_cg, geom.ndim_fft, _centred(geom)))
    return prox_bwd(prox.layers, theta, fwd["t"], fwd["conv_in"], fwd["act"], g_z)


# ----------------------------------------------------------------------------- greedy training (Alg. 1)
def adam_step(theta, grad, m, v, t, lr, beta1=0.9, beta2=0.999, eps=1e-8):
    """One Adam update (the optimizer named in Implementation Details), step count t >= 1:
        m <- beta1 m + (1 - beta1) g ;  v <- beta2 v + (1 - beta2) g^2
        theta <- theta - lr * (m / (1 - beta1^t)) / (sqrt(v / (1 - beta2^t)) + eps)
    Returns (theta, m, v) as new float64 arrays."""
    theta = np.asarray(theta, np.float64)
    g = np.asarray(grad, np.float64)
    m = beta1 * np.asarray(m, np.float64) + (1.0 - beta1) * g
    v = beta2 * np.asarray(v, np.float64) + (1.0 - beta2) * g * g
    m_hat = m / (1.0 - beta1 ** t)
    v_hat = v / (1.0 - beta2 ** t)
    return theta - lr * m_hat / (np.sqrt(v_hat) + eps), m, v


def greedy_iteration(geom, prox, x0, S, M, y, alpha, thetas, ms, vs, t, lr, x_ref, beta1=0.9, beta2=0.999, eps=1e-8):
    """Alg. 1 for one mini-batch: for module i = 1..len(thetas): forward x_i = f_theta_i(DC(x_{i-1})), local
    loss against x_ref, gradient of that loss with respect to theta_i only, Adam update of theta_i; the
    activations of the module are dropped and x_i is handed on as a constant.
    Returns (x_final, losses, thetas, ms, vs) with the updated per-module lists."""
    x = np.asarray(x0, np.complex128)
    losses, new_t, new_m, new_v = [], [], [], []
    for th, m, v in zip(thetas, ms, vs):
        f = module_fwd(geom, prox, x, S, M, y, alpha, th, x_ref)
        g = module_bwd(prox, th, f)
        th2, m2, v2 = adam_step(th, g, m, v, t, lr, beta1, beta2, eps)
        losses.append(f["loss"])
        new_t.append(th2); new_m.append(m2); new_v.append(v2)
        x = f["x_out"]          # computed with the parameters before the update; detached hand-off
    return x, losses, new_t, new_m, new_v


def unrolled_inference(geom, prox, x0, S, M, y, alpha, thetas):
    """x_i = f_theta_i(DC(x_{i-1})) through the given modules (all of them, or the first N_inf: Alg. 1's
    modules can be evaluated up to any depth)."""
    x = np.asarray(x0, np.complex128)
    for th in thetas:
        x = module_fwd(geom, prox, x, S, M, y, alpha, th)["x_out"]
    return x
