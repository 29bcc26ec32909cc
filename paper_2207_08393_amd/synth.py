"""Seeded synthetic inputs shaped like the paper's workloads (Datasets section).

This module only *draws inputs*: phantoms, coil-sensitivity maps, sampling masks,
noise, prox weights and the measured k-space of the sensing model (Eq. 1,
y = Omega F S x + eps), the latter synthesised with numpy's library FFT.  It holds
no part of the module computation (no data-consistency step, no prox, no loss, no
gradient); the CPU oracle and the HIP library both receive what it returns as
plain input arrays and neither imports the other.

Layouts (row-major, last dimension contiguous):
  image   x  [B][T][D][H][W]        complex64
  coils   S  [B][C][D][H][W]        complex64   (time-invariant, broadcast over T)
  mask    M  [B][T][D][H][W]        uint8       (non-zero = sampled; no coil dimension)
  k-space y  [B][C][T][D][H][W]     complex64
  theta      flat float32: per layer W[cout][kt][kd][kh][kw][cin], then b[cout] if has_bias
The Fourier transform is orthonormal over the last `ndim_fft` dimensions, uncentred (zero
frequency at index 0) unless the geometry says `centred`.
"""
from __future__ import annotations

import dataclasses
from typing import List, Optional, Sequence, Tuple

import numpy as np

BASE_SEED = 20220708


# --------------------------------------------------------------------------- descriptors
@dataclasses.dataclass
class Geom:
    ndim_fft: int
    B: int
    C: int
    T: int
    D: int
    H: int
    W: int
    centred: int = 0   # 1: frequency and spatial origin in the middle of every transformed axis (fftshift convention)

    @property
    def image_shape(self):
        return (self.B, self.T, self.D, self.H, self.W)

    @property
    def coil_shape(self):
        return (self.B, self.C, self.D, self.H, self.W)

    @property
    def kspace_shape(self):
        return (self.B, self.C, self.T, self.D, self.H, self.W)

    @property
    def P(self):
        return self.T * self.D * self.H * self.W

    @property
    def E(self):
        return self.B * self.C * self.P

    @property
    def fft_axes_image(self):
        return tuple(range(5 - self.ndim_fft, 5))


@dataclasses.dataclass
class ConvLayer:
    cin: int
    cout: int
    kt: int = 1
    kd: int = 1
    kh: int = 1
    kw: int = 1
    relu_in: int = 0
    relu_out: int = 0
    has_bias: int = 1
    skip_src: int = -1  # -1: none; s >= 0: tensor t_s is added to this layer's output (t_0 = u)

    @property
    def taps(self):
        return self.kt * self.kd * self.kh * self.kw

    @property
    def n_weight(self):
        return self.cout * self.taps * self.cin

    @property
    def n_param(self):
        return self.n_weight + (self.cout if self.has_bias else 0)


@dataclasses.dataclass
class ProxDesc:
    layers: List[ConvLayer]
    dtype: int = 0      # 0: fp32 convs; 1: bf16 operands with fp32 accumulation
    loss_kind: int = 0  # 0: mean |z-x|^2 ; 1: mean |z-x| (complex magnitude)

    @property
    def n_theta(self):
        return sum(l.n_param for l in self.layers)


def chain_prox(channels: Sequence[int], kernels: Sequence[Tuple[int, int, int, int]],
               has_bias: int = 1, dtype: int = 0, loss_kind: int = 0) -> ProxDesc:
    """z = u + conv_L(ReLU(... ReLU(conv_1(u)))) : ReLU after every layer but the last,
    one outer skip from the prox input (residual CNN of the MoDL/3D set-ups)."""
    L = len(channels) - 1
    layers = []
    for l in range(L):
        kt, kd, kh, kw = kernels[l]
        layers.append(ConvLayer(channels[l], channels[l + 1], kt, kd, kh, kw,
                                relu_in=0, relu_out=int(l < L - 1), has_bias=has_bias,
                                skip_src=(0 if l == L - 1 else -1)))
    return ProxDesc(layers, dtype, loss_kind)


def resblock_prox(nf: int, n_blocks: int, k=(1, 1, 3, 3), has_bias: int = 1,
                  dtype: int = 0, loss_kind: int = 0) -> ProxDesc:
    """conv_in, n_blocks pre-activation residual blocks (ReLU-conv-ReLU-conv + identity),
    ReLU, conv_out (2D PGD prox of the Implementation Details)."""
    kt, kd, kh, kw = k
    layers = [ConvLayer(2, nf, kt, kd, kh, kw, 0, 0, has_bias, -1)]
    for _ in range(n_blocks):
        src = len(layers)  # index of the tensor entering the block
        layers.append(ConvLayer(nf, nf, kt, kd, kh, kw, 1, 0, has_bias, -1))
        layers.append(ConvLayer(nf, nf, kt, kd, kh, kw, 1, 0, has_bias, src))
    layers.append(ConvLayer(nf, 2, kt, kd, kh, kw, 1, 0, has_bias, -1))
    return ProxDesc(layers, dtype, loss_kind)


def init_theta(rng: np.random.Generator, prox: ProxDesc, bias_std: float = 0.0) -> np.ndarray:
    """He-normal weights N(0, 2/(cin*taps)); biases 0 (or N(0, bias_std^2) for tests)."""
    parts = []
    for l in prox.layers:
        std = np.sqrt(2.0 / (l.cin * l.taps))
        parts.append((rng.standard_normal(l.n_weight) * std).astype(np.float32))
        if l.has_bias:
            parts.append((rng.standard_normal(l.cout) * bias_std).astype(np.float32))
    return np.concatenate(parts)


# --------------------------------------------------------------------------- pieces
def _freq(n: int) -> np.ndarray:
    """Signed frequency of each uncentred DFT index."""
    i = np.arange(n)
    return np.where(i < (n + 1) // 2, i, i - n)


def lowest_freq_indices(n: int, count: int) -> np.ndarray:
    order = np.argsort(np.abs(_freq(n)), kind="stable")
    return np.sort(order[:count])


def _grid(shape: Sequence[int]):
    axes = [np.linspace(-1.0, 1.0, n) if n > 1 else np.zeros(1) for n in shape]
    return np.meshgrid(*axes, indexing="ij")


def smooth_coils(rng, B: int, C: int, spatial: Tuple[int, int, int], degree: int) -> np.ndarray:
    """C complex polynomial maps of total degree <= `degree` over the (D,H,W) grid,
    constant term offset by +2, normalised so that sum_c |S_c|^2 = 1 at every pixel."""
    D, H, W = spatial
    g = _grid((D, H, W))
    monos = []
    for a in range(degree + 1):
        for b in range(degree + 1 - a):
            for c in range(degree + 1 - a - b):
                if D == 1 and a > 0:
                    continue
                monos.append((g[0] ** a) * (g[1] ** b) * (g[2] ** c))
    monos = np.stack(monos, 0)  # [K, D, H, W]
    S = np.empty((B, C, D, H, W), np.complex128)
    for b in range(B):
        coef = rng.standard_normal((C, monos.shape[0])) + 1j * rng.standard_normal((C, monos.shape[0]))
        coef[:, 0] += 2.0
        S[b] = np.tensordot(coef, monos, axes=(1, 0))
    S /= np.sqrt((np.abs(S) ** 2).sum(1, keepdims=True))
    return S.astype(np.complex64)


def _smooth_phase(rng, spatial) -> np.ndarray:
    g = _grid(spatial)
    ph = np.zeros(spatial)
    for a in range(3):
        for b in range(3 - a):
            for c in range(3 - a - b):
                if spatial[0] == 1 and a > 0:
                    continue
                ph += rng.standard_normal() * (g[0] ** a) * (g[1] ** b) * (g[2] ** c)
    ph *= (np.pi / 2) / max(np.abs(ph).max(), 1e-12)
    return ph


def ellipse_phantom(rng, spatial: Tuple[int, int, int], n_shapes: int, radius_scale=None) -> np.ndarray:
    """Sum of random ellipses (2D, D == 1) or ellipsoids (3D) with smooth random phase.
    `radius_scale` (n_shapes,) optionally scales each shape's semi-axes (used for cine)."""
    D, H, W = spatial
    g = _grid(spatial)
    img = np.zeros(spatial)
    for s in range(n_shapes):
        ctr = rng.uniform(-0.6, 0.6, 3)
        ax = rng.uniform(0.05, 0.4, 3)
        ang = rng.uniform(0, np.pi)
        amp = rng.uniform(0.2, 1.0)
        if radius_scale is not None:
            ax = ax * radius_scale[s]
        ch, sh = np.cos(ang), np.sin(ang)
        yy = (g[1] - ctr[1]) * ch + (g[2] - ctr[2]) * sh
        xx = -(g[1] - ctr[1]) * sh + (g[2] - ctr[2]) * ch
        q = (yy / ax[1]) ** 2 + (xx / ax[2]) ** 2
        if D > 1:
            q = q + ((g[0] - ctr[0]) / ax[0]) ** 2
        img += amp * (q <= 1.0)
    return img


def gaussian_blur_last2(a: np.ndarray, sigma: float) -> np.ndarray:
    """Separable Gaussian blur over the last two axes, zero padding, truncated at 4 sigma."""
    r = int(np.ceil(4 * sigma))
    t = np.arange(-r, r + 1)
    k = np.exp(-0.5 * (t / sigma) ** 2)
    k /= k.sum()
    out = a
    for axis in (-2, -1):
        out = np.apply_along_axis(lambda v: np.convolve(v, k, mode="same"), axis, out)
    return out


def _lines_to_mask(lines_per_bt, geom: Geom) -> np.ndarray:
    """lines_per_bt[b][t] = sampled W indices; the mask is constant along D and H."""
    M = np.zeros(geom.image_shape, np.uint8)
    for b in range(geom.B):
        for t in range(geom.T):
            M[b, t, :, :, lines_per_bt[b][t]] = 1
    return M


def _draw_lines(rng, n: int, total: int, centre: int, kind: str) -> np.ndarray:
    """`total` distinct phase-encode indices out of n: `centre` lowest-|freq| ones plus
    others drawn without replacement: uniformly ('uniform'), with pdf ~ (1-|k|/kmax)^2
    ('vd'), or equispaced with a random offset topped up uniformly ('equi')."""
    cen = lowest_freq_indices(n, centre)
    rest = np.setdiff1d(np.arange(n), cen)
    need = total - centre
    if kind == "uniform":
        extra = rng.choice(rest, need, replace=False)
    elif kind == "vd":
        f = np.abs(_freq(n))[rest].astype(np.float64)
        pdf = (1.0 - f / (f.max() + 1.0)) ** 2
        extra = rng.choice(rest, need, replace=False, p=pdf / pdf.sum())
    elif kind == "equi":
        step = int(np.ceil(n / max(need, 1)))
        off = int(rng.integers(0, step))
        eq = np.setdiff1d(np.arange(off, n, step), cen)[:need]
        left = np.setdiff1d(rest, eq)
        extra = np.concatenate([eq, rng.choice(left, need - len(eq), replace=False)])
    else:
        raise ValueError(kind)
    return np.sort(np.concatenate([cen, extra])).astype(np.int64)


def poisson_disc_plane(rng, H: int, W: int, total: int, calib: int) -> np.ndarray:
    """Variable-density Poisson-disc pattern on an uncentred H x W phase-encode plane:
    a calib x calib block of lowest frequencies plus dart-thrown points whose minimum
    distance grows linearly with |k|; trimmed / topped up to exactly `total` points."""
    fh, fw = np.meshgrid(_freq(H), _freq(W), indexing="ij")
    rad = np.sqrt((fh / (H / 2.0)) ** 2 + (fw / (W / 2.0)) ** 2)
    m = np.zeros((H, W), bool)
    ch, cw = lowest_freq_indices(H, calib), lowest_freq_indices(W, calib)
    m[np.ix_(ch, cw)] = True
    order = rng.permutation(H * W)

    def throw(slope):
        acc = m.copy()
        for idx in order:
            h, w = divmod(int(idx), W)
            if acc[h, w]:
                continue
            r = 1.0 + slope * rad[h, w]
            ri = int(np.ceil(r))
            hs = (np.arange(h - ri, h + ri + 1)) % H
            ws = (np.arange(w - ri, w + ri + 1)) % W
            dh = np.arange(-ri, ri + 1)[:, None]
            dw = np.arange(-ri, ri + 1)[None, :]
            near = acc[np.ix_(hs, ws)] & (dh * dh + dw * dw < r * r)
            if not near.any():
                acc[h, w] = True
        return acc

    lo, hi = 0.0, 12.0
    best = None
    for _ in range(7):
        mid = 0.5 * (lo + hi)
        acc = throw(mid)
        best = acc
        if acc.sum() > total:
            lo = mid
        else:
            hi = mid
    acc = best
    extra = np.flatnonzero(acc & ~m)
    free = np.flatnonzero(~acc)
    n_extra = total - int(m.sum())
    if len(extra) > n_extra:
        keep = rng.choice(extra, n_extra, replace=False)
    else:
        keep = np.concatenate([extra, rng.choice(free, n_extra - len(extra), replace=False)])
    out = m.copy().ravel()
    out[keep] = True
    return out.reshape(H, W)


def measure(x_true, S, M, geom: Geom, rng, sigma: float, sigma_rel: bool):
    """Eq. 1 with numpy's FFT: y = M * FFT_ortho(S * x) + noise (noise masked too).
    Returns (y, x0) with x0 = sum_c conj(S_c) IFFT_ortho(y_c), the zero-filled SENSE image
    the Training paragraph names as the network input."""
    axes = tuple(range(6 - geom.ndim_fft, 6))
    c = S[:, :, None].astype(np.complex128) * x_true[:, None].astype(np.complex128)
    if geom.centred:
        fwd = lambda a: np.fft.fftshift(np.fft.fftn(np.fft.ifftshift(a, axes=axes), axes=axes, norm="ortho"), axes=axes)
        inv = lambda a: np.fft.fftshift(np.fft.ifftn(np.fft.ifftshift(a, axes=axes), axes=axes, norm="ortho"), axes=axes)
    else:
        fwd = lambda a: np.fft.fftn(a, axes=axes, norm="ortho")
        inv = lambda a: np.fft.ifftn(a, axes=axes, norm="ortho")
    k = fwd(c)
    m = (M != 0)[:, None]
    k = k * m
    scale = sigma * (np.abs(k).max() if sigma_rel else 1.0)
    noise = rng.standard_normal(k.shape) + 1j * rng.standard_normal(k.shape)
    y = ((k + scale * noise) * m).astype(np.complex64)
    x0 = (np.conj(S[:, :, None]) * inv(y.astype(np.complex128))).sum(1)
    return y, x0.astype(np.complex64)


# --------------------------------------------------------------------------- cases
@dataclasses.dataclass
class Case:
    name: str
    geom: Geom
    prox: ProxDesc
    alpha: float
    x_true: np.ndarray
    S: np.ndarray
    M: np.ndarray
    y: np.ndarray
    x_in: np.ndarray
    theta: np.ndarray
    n_modules: int = 1


def make_custom(seed: int, geom: Geom, prox: ProxDesc, accel: float = 4.0, centre: int = 4,
                mask_kind: str = "uniform", sigma: float = 1e-3, coil_degree: int = 2,
                bias_std: float = 0.05, n_shapes: int = 0, alpha: float = 1.0,
                name: str = "custom") -> Case:
    """Small free-form case for tests. mask_kind: 'uniform' | 'vd' | 'equi' (1D lines along W),
    'random2d' (independent points on the (H,W) plane, constant along D), 'full'."""
    rng = np.random.default_rng(seed)
    sp = (geom.D, geom.H, geom.W)
    if n_shapes > 0:
        x = np.stack([np.stack([ellipse_phantom(rng, sp, n_shapes) * np.exp(1j * _smooth_phase(rng, sp))
                                for _ in range(geom.T)]) for _ in range(geom.B)])
    else:
        x = rng.standard_normal(geom.image_shape) + 1j * rng.standard_normal(geom.image_shape)
    x = x.astype(np.complex64)
    S = smooth_coils(rng, geom.B, geom.C, sp, coil_degree)
    if mask_kind == "full":
        M = np.ones(geom.image_shape, np.uint8)
    elif mask_kind == "random2d":
        keep = rng.random((geom.B, geom.T, 1, geom.H, geom.W)) < 1.0 / accel
        M = np.broadcast_to(keep, geom.image_shape).astype(np.uint8).copy()
        M[..., 0, 0] = 1
    else:
        total = max(int(round(geom.W / accel)), min(centre, geom.W))
        cen = min(centre, total)
        lines = [[_draw_lines(rng, geom.W, total, cen, mask_kind) for _ in range(geom.T)]
                 for _ in range(geom.B)]
        M = _lines_to_mask(lines, geom)
    if geom.centred:   # the generators put the low frequencies at index 0: move them to the middle of the array
        M = np.ascontiguousarray(np.fft.fftshift(M, axes=tuple(range(5 - geom.ndim_fft, 5))))
    y, x0 = measure(x, S, M, geom, rng, sigma, False)
    theta = init_theta(rng, prox, bias_std)
    return Case(name, geom, prox, alpha, x, S, M, y, x0, theta, 1)


def make_case(cfg: int, seed: Optional[int] = None) -> Case:
    """The five benchmark-shaped workloads (index = position in the configs list):
    0 tiny 2D, 1 knee-shaped 2D, 2 brain-shaped 2D with bf16 convs, 3 3D volume, 4 2D+t cine."""
    seed = BASE_SEED + cfg if seed is None else seed
    rng = np.random.default_rng(seed)
    k2, k3 = (1, 1, 3, 3), (1, 3, 3, 3)
    if cfg == 0:
        geom = Geom(2, 1, 4, 1, 1, 64, 64)
        x = rng.standard_normal(geom.image_shape) + 1j * rng.standard_normal(geom.image_shape)
        x = gaussian_blur_last2(x.real, 2.0) + 1j * gaussian_blur_last2(x.imag, 2.0)
        S = smooth_coils(rng, 1, 4, (1, 64, 64), 2)
        lines = [[_draw_lines(rng, 64, 16, 8, "uniform")]]
        M = _lines_to_mask(lines, geom)
        prox = chain_prox([2, 16, 16, 2], [k2] * 3)
        sigma, rel, nmod, name = 1e-3, False, 1, "tiny2d_64x64_c4_b1"
    elif cfg == 1:
        geom = Geom(2, 2, 15, 1, 1, 640, 368)
        x = np.stack([ellipse_phantom(rng, (1, 640, 368), 12) * np.exp(1j * _smooth_phase(rng, (1, 640, 368)))
                      for _ in range(2)])[:, None]
        S = smooth_coils(rng, 2, 15, (1, 640, 368), 3)
        lines = [[_draw_lines(rng, 368, 46, 15, "vd")] for _ in range(2)]
        M = _lines_to_mask(lines, geom)
        prox = resblock_prox(64, 2)
        sigma, rel, nmod, name = 0.01, True, 5, "knee2d_640x368_c15_b2"
    elif cfg == 2:
        geom = Geom(2, 4, 16, 1, 1, 640, 320)
        x = np.stack([ellipse_phantom(rng, (1, 640, 320), 12) * np.exp(1j * _smooth_phase(rng, (1, 640, 320)))
                      for _ in range(4)])[:, None]
        S = smooth_coils(rng, 4, 16, (1, 640, 320), 3)
        lines = [[_draw_lines(rng, 320, 80, 26, "equi")] for _ in range(4)]
        M = _lines_to_mask(lines, geom)
        prox = chain_prox([2, 128, 128, 128, 128, 2], [k2] * 5, dtype=1)
        sigma, rel, nmod, name = 0.01, True, 8, "brain2d_640x320_c16_b4_bf16"
    elif cfg == 3:
        geom = Geom(3, 1, 8, 1, 256, 160, 160)
        sp = (256, 160, 160)
        x = (ellipse_phantom(rng, sp, 10) * np.exp(1j * _smooth_phase(rng, sp)))[None, None]
        S = smooth_coils(rng, 1, 8, sp, 2)
        plane = poisson_disc_plane(rng, 160, 160, 3200, 24)
        M = np.broadcast_to(plane[None, None, None], geom.image_shape).astype(np.uint8).copy()
        prox = chain_prox([2, 32, 32, 32, 2], [k3] * 4)
        sigma, rel, nmod, name = 0.01, True, 4, "vol3d_256x160x160_c8_b1"
    elif cfg == 4:
        geom = Geom(2, 1, 8, 20, 1, 192, 160)
        sp = (1, 192, 160)
        static = ellipse_phantom(rng, sp, 8)
        phi = rng.uniform(0, 2 * np.pi, 3)
        dyn_seed = int(rng.integers(1 << 31))
        frames = []
        for t in range(20):
            sub = np.random.default_rng(dyn_seed)  # the same three shapes in every frame
            frames.append(static + ellipse_phantom(sub, sp, 3, 1.0 + 0.2 * np.sin(2 * np.pi * t / 20 + phi)))
        x =(np.stack(frames) * np.exp(1j * _smooth_phase(rng, sp)))[None]
        S = smooth_coils(rng, 1, 8, sp, 2)
        lines = [[_draw_lines(rng, 160, 13, 8, "vd") for _ in range(20)]]
        M = _lines_to_mask(lines, geom)
        ks, kt = (1, 1, 3, 3), (3, 1, 1, 1)
        prox = chain_prox([2, 64, 64, 64, 2], [ks, kt, ks, kt])
        sigma, rel, nmod, name = 0.01, True, 10, "cine2dt_20x192x160_c8_b1"
    else:
        raise ValueError("cfg must be 0..4")
    x = np.ascontiguousarray(x.reshape(geom.image_shape)).astype(np.complex64)
    y, x0 = measure(x, S, M, geom, rng, sigma, rel)
    theta = init_theta(rng, prox, 0.0)
    return Case(name, geom, prox, 1.0, x, S, M, y, x0, theta, nmod)
