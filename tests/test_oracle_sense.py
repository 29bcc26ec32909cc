"""Pins for the oracle's Fourier / SENSE / data-consistency parts (CPU only).

Every check compares the oracle with something that is not the oracle: a closed form, an
identity the sensing model implies (Eq. 1, PGD section: A = Omega F S and its Hermitian
transpose), numpy's FFT library, or a brute-force circular convolution.
"""
import numpy as np
import pytest

from oracle import gleam_oracle as og
from paper_2207_08393_amd import synth

RNG = np.random.default_rng(7)


def crandn(*shape):
    return RNG.standard_normal(shape) + 1j * RNG.standard_normal(shape)


# ----------------------------------------------------------------------------- DFT
def test_dft_closed_forms_n1_n2_n4():
    assert np.allclose(og.dft_axis(np.array([3 - 2j]), 0), [3 - 2j])
    a, b = 1.5 + 0.5j, -2 + 1j
    assert np.allclose(og.dft_axis(np.array([a, b]), 0), np.array([a + b, a - b]) / np.sqrt(2))
    v = np.array([1, 2j, -3, 4 + 1j])
    expect = np.array([v[0] + v[1] + v[2] + v[3],
                       v[0] - 1j * v[1] - v[2] + 1j * v[3],
                       v[0] - v[1] + v[2] - v[3],
                       v[0] + 1j * v[1] - v[2] - 1j * v[3]]) / 2.0
    assert np.allclose(og.dft_axis(v, 0), expect, atol=1e-14)


@pytest.mark.parametrize("n", [1, 2, 3, 4, 5, 8, 12, 23, 46, 64, 160, 368])
def test_dft_matches_numpy_fft_and_unitary(n):
    v = crandn(3, n)
    X = og.dft_axis(v, 1)
    assert np.allclose(X, np.fft.fft(v, axis=1, norm="ortho"), atol=1e-11)
    assert np.allclose(og.dft_axis(X, 1, inverse=True), v, atol=1e-11)          # F^H F = I
    assert np.allclose(np.linalg.norm(X), np.linalg.norm(v), rtol=1e-12)          # Parseval
    F = og.dft_matrix(n)
    assert np.allclose(F.conj().T @ F, np.eye(n), atol=1e-12)
    assert np.allclose(og.dft_matrix(n, inverse=True), F.conj().T, atol=1e-15)


@pytest.mark.parametrize("n", [5, 16, 23, 40])
def test_dft_delta_constant_exponential_shift(n):
    d = np.zeros(n, complex)
    d[0] = 1
    assert np.allclose(og.dft_axis(d, 0), np.full(n, n ** -0.5))
    assert np.allclose(og.dft_axis(np.ones(n), 0), np.sqrt(n) * d, atol=1e-12)
    f0 = 3 % n
    e = np.exp(2j * np.pi * f0 * np.arange(n) / n)
    E = og.dft_axis(e, 0)
    expect = np.zeros(n, complex)
    expect[f0] = np.sqrt(n)
    assert np.allclose(E, expect, atol=1e-11)            # sign of the exponent is -
    v = crandn(n)
    s = 2
    shifted = np.roll(v, s)
    assert np.allclose(og.dft_axis(shifted, 0),
                       og.dft_axis(v, 0) * np.exp(-2j * np.pi * s * np.arange(n) / n), atol=1e-11)


def test_dft_nd_axis_order_and_numpy():
    v = crandn(2, 3, 6, 5, 4)
    a = og.dft_nd(v, 3)
    assert np.allclose(a, np.fft.fftn(v, axes=(2, 3, 4), norm="ortho"), atol=1e-11)
    b = og.dft_axis(og.dft_axis(og.dft_axis(v, 2), 4), 3)
    assert np.allclose(a, b, atol=1e-12)
    a2 = og.dft_nd(v, 2)
    assert np.allclose(a2, np.fft.fftn(v, axes=(3, 4), norm="ortho"), atol=1e-11)
    assert np.allclose(og.dft_nd(a2, 2, inverse=True), v, atol=1e-11)


# ----------------------------------------------------------------------------- operator
def small_case(ndim_fft=2, B=2, C=3, T=2, D=1, H=6, W=10, mask_kind="uniform", seed=3):
    geom = synth.Geom(ndim_fft, B, C, T, D, H, W)
    prox = synth.chain_prox([2, 4, 2], [(1, 1, 3, 3)] * 2)
    return synth.make_custom(seed, geom, prox, accel=2.5, centre=2, mask_kind=mask_kind)


@pytest.mark.parametrize("nd,D,kind", [(2, 1, "uniform"), (2, 3, "vd"), (3, 4, "random2d")])
def test_adjoint_identity_and_psd(nd, D, kind):
    c = small_case(nd, D=D, mask_kind=kind)
    g = c.geom
    x = crandn(*g.image_shape)
    z = crandn(*g.kspace_shape)
    Ax = og.sense_forward(x, c.S, c.M, nd)
    AHz = og.sense_adjoint(z, c.S, c.M, nd)
    lhs, rhs = np.vdot(z, Ax), np.vdot(AHz, x)     # <Ax, z> = <x, A^H z>
    assert abs(lhs - rhs) <= 1e-12 * abs(lhs)
    n = og.sense_normal(x, c.S, c.M, nd)
    q = np.vdot(x, n)
    assert abs(q.imag) <= 1e-12 * abs(q) and q.real >= 0
    assert np.isclose(q.real, np.linalg.norm(Ax) ** 2, rtol=1e-12)
    assert np.linalg.norm(n) <= np.linalg.norm(x) * (1 + 1e-12)   # ||A|| <= 1 when sum|S|^2 = 1


def test_mask_bit_exact_zero_and_idempotent():
    c = small_case(2, mask_kind="uniform")
    x = crandn(*c.geom.image_shape)
    k = og.sense_forward(x, c.S, c.M, 2)
    off = np.broadcast_to((c.M == 0)[:, None], k.shape)
    assert np.all(k[off] == 0) and not np.signbit(k[off].real).any() and not np.signbit(k[off].imag).any()
    again = np.where((c.M != 0)[:, None], k, 0.0)
    assert np.array_equal(again, k)                      # M o M = M
    junk = crandn(*c.geom.kspace_shape)                  # y is ignored off the mask
    r1 = og.masked_residual(x, c.S, c.M, c.y, 2)
    r2 = og.masked_residual(x, c.S, c.M, np.where(off, junk, c.y), 2)
    assert np.array_equal(r1, r2) and np.all(r1[off] == 0)


def test_mask_selects_expected_index_set():
    c = small_case(2, B=1, C=1, T=1, H=4, W=8)
    ramp = np.arange(c.geom.E, dtype=np.float64).reshape(c.geom.kspace_shape) + 1.0
    S1 = np.ones(c.geom.coil_shape)
    img = og.sense_adjoint(ramp, S1, c.M, 2)
    back = og.dft_nd(img[:, None], 2)
    lines = np.flatnonzero(c.M[0, 0, 0, 0])
    expect = np.zeros_like(ramp)
    expect[..., lines] = ramp[..., lines]
    assert np.allclose(back, expect, atol=1e-10)


@pytest.mark.parametrize("nd,D", [(2, 1), (3, 3)])
def test_full_sampling_is_identity_and_dc_recovers_truth(nd, D):
    c = small_case(nd, D=D, mask_kind="full")
    x = crandn(*c.geom.image_shape)
    assert np.allclose(og.sense_normal(x, c.S, c.M, nd), x, atol=1e-6)   # float32 coil normalisation
    S = c.S.astype(np.complex128)
    S /= np.sqrt((np.abs(S) ** 2).sum(1, keepdims=True))
    assert np.allclose(og.sense_normal(x, S, c.M, nd), x, atol=1e-12)
    y = og.sense_forward(c.x_true, S, c.M, nd)
    u = og.dc_step(x, S, c.M, y, 1.0, nd)
    assert np.allclose(u, c.x_true, atol=1e-11)


def test_single_coil_1d_mask_is_circular_convolution():
    H, W = 5, 12
    geom = synth.Geom(2, 1, 1, 1, 1, H, W)
    m = np.zeros(W)
    m[[0, 1, 4, 7, 11]] = 1
    M = np.broadcast_to(m, geom.image_shape).astype(np.uint8)
    S = np.ones(geom.coil_shape)
    x = crandn(*geom.image_shape)
    got = og.sense_normal(x, S, M, 2)
    # A^H A = F^H diag(m) F along W: circular convolution with h = W^-1 sum_q m[q] e^{+2 pi i q j / W}
    q = np.arange(W)
    h = np.array([(m * np.exp(2j * np.pi * q * j / W)).sum() / W for j in range(W)])
    expect = np.zeros_like(x)
    for j in range(W):
        for l in range(W):
            expect[..., j] += h[(j - l) % W] * x[..., l]
    assert np.allclose(got, expect, atol=1e-12)


def test_dc_step_formula_pieces():
    c = small_case(2)
    x = crandn(*c.geom.image_shape)
    alpha = 0.7
    u = og.dc_step(x, c.S, c.M, c.y, alpha, 2)
    ym = np.where((c.M != 0)[:, None], c.y, 0)
    expect = x - alpha * (og.sense_normal(x, c.S, c.M, 2) - og.sense_adjoint(ym, c.S, c.M, 2))
    assert np.allclose(u, expect, atol=1e-12)
    # gradient of ||Ax - y||^2 is 2 A^H(Ax - y): a step of 2t reduces the data misfit (t = 0.25 here)
    f = lambda v: np.linalg.norm(og.sense_forward(v, c.S, c.M, 2) - ym) ** 2
    assert f(og.dc_step(x, c.S, c.M, c.y, 0.5, 2)) < f(x)
    eps = 1e-6
    d = crandn(*c.geom.image_shape)
    num = (f(x + eps * d) - f(x - eps * d)) / (2 * eps)
    ana = 2 * np.real(np.vdot(d, (x - og.dc_step(x, c.S, c.M, c.y, 1.0, 2))))
    assert np.isclose(num, ana, rtol=1e-6)


def test_time_frames_and_batch_are_independent():
    c = small_case(2, B=2, T=3)
    x = crandn(*c.geom.image_shape)
    full = og.dc_step(x, c.S, c.M, c.y, 1.0, 2)
    for b in range(2):
        for t in range(3):
            one = og.dc_step(x[b:b + 1, t:t + 1], c.S[b:b + 1], c.M[b:b + 1, t:t + 1],
                             c.y[b:b + 1, :, t:t + 1], 1.0, 2)
            assert np.allclose(full[b, t], one[0, 0], atol=1e-12)


# ----------------------------------------------------------------------------- generator
@pytest.mark.parametrize("cfg", [0])
def test_generator_invariants_cfg0(cfg):
    c = synth.make_case(cfg)
    assert np.allclose((np.abs(c.S) ** 2).sum(1), 1.0, atol=1e-6)
    assert c.M.dtype == np.uint8 and int(c.M[0, 0, 0, 0].sum()) == 16
    assert np.all(c.M[0, 0, 0] == c.M[0, 0, 0, 0])
    low = synth.lowest_freq_indices(64, 8)
    assert np.all(c.M[0, 0, 0, 0, low] == 1) and set(int(v) for v in low) == {0, 1, 2, 3, 4, 61, 62, 63}
    off = np.broadcast_to((c.M == 0)[:, None], c.y.shape)
    assert np.all(c.y[off] == 0)
    # the generator's library-FFT measurement agrees with the oracle's operator (noise level 1e-3)
    k = og.sense_forward(c.x_true, c.S, c.M, 2)
    assert np.abs(k - c.y).max() < 1e-2
    assert np.allclose(og.sense_adjoint(c.y, c.S, c.M, 2), c.x_in, atol=1e-5)
    assert c.theta.size == c.prox.n_theta == 2 * 9 * 16 + 16 + 16 * 9 * 16 + 16 + 16 * 9 * 2 + 2


@pytest.mark.parametrize("nd,kind", [(1, "uniform"), (1, "random2d"), (2, "uniform"), (2, "vd"), (2, "equi"),
                                     (2, "random2d"), (2, "full"), (3, "random2d"), (3, "uniform"), (3, "full")])
def test_generator_measurement_is_the_oracles_operator_for_every_mask_kind_and_dimension(nd, kind):
    """synth.measure draws y and x_in for BOTH sides with numpy's FFT; here it is held to the oracle's explicit-DFT
    operators on every mask kind and transform dimension, with several samples, frames and depth slices (per-sample
    and per-frame masks), so that a wrong axis, normalisation, broadcast or conjugate in it cannot go unnoticed."""
    geom = synth.Geom(nd, 2, 3, 2, 4, 6, 8)
    prox = synth.chain_prox([2, 4, 2], [(1, 1, 3, 3)] * 2)
    c = synth.make_custom(900 + nd, geom, prox, accel=2.0, centre=2, mask_kind=kind, sigma=0.0)
    if kind not in ("full",):
        assert 0 < c.M.sum() < c.M.size
        assert not np.array_equal(c.M[0], c.M[1]) or kind == "full"          # per-sample masks
    k = og.sense_forward(c.x_true, c.S, c.M, nd)
    assert np.abs(k - c.y).max() <= 1e-5 * np.abs(k).max()                   # complex64 storage of y
    x0 = og.sense_adjoint(c.y, c.S, c.M, nd)
    assert np.abs(x0 - c.x_in).max() <= 1e-5 * np.abs(x0).max()
    # with noise: y is whatever was drawn, but still exactly zero off the mask, and x_in is still A^H y
    cn = synth.make_custom(900 + nd, geom, prox, accel=2.0, centre=2, mask_kind=kind, sigma=0.05)
    off = np.broadcast_to((cn.M == 0)[:, None], cn.y.shape)
    assert np.all(cn.y[off] == 0) and np.abs(cn.y - c.y).max() > 1e-3
    x0n = og.sense_adjoint(cn.y, cn.S, cn.M, nd)
    assert np.abs(x0n - cn.x_in).max() <= 1e-5 * np.abs(x0n).max()


def test_generator_measurement_of_the_cine_shaped_case_matches_the_oracle():
    """The 2D+t benchmark case (per-frame masks, coils shared by the frames), shrunk: relative noise level."""
    geom = synth.Geom(2, 1, 3, 5, 1, 12, 10)
    rng = np.random.default_rng(3)
    x = (rng.standard_normal(geom.image_shape) + 1j * rng.standard_normal(geom.image_shape)).astype(np.complex64)
    S = synth.smooth_coils(rng, 1, 3, (1, 12, 10), 2)
    lines = [[synth._draw_lines(rng, 10, 4, 2, "vd") for _ in range(5)]]
    M = synth._lines_to_mask(lines, geom)
    assert len({tuple(l) for l in lines[0]}) > 1                              # the frames do differ
    y, x0 = synth.measure(x, S, M, geom, rng, 0.0, True)
    k = og.sense_forward(x, S, M, 2)
    assert np.abs(k - y).max() <= 1e-5 * np.abs(k).max()
    assert np.abs(og.sense_adjoint(y, S, M, 2) - x0).max() <= 1e-5 * np.abs(x0).max()


# ----------------------------------------------------------------------------- centred transform (variant of F)
@pytest.mark.parametrize("n", [1, 2, 3, 4, 5, 6, 8, 10, 23, 46, 160])
def test_centred_dft_is_fftshift_fft_ifftshift(n):
    """The centred matrix against the library composition fftshift . fft . ifftshift (odd lengths included, where the
    two shifts differ), forward and inverse, and the closed forms that fix what "centred" means: a delta at the
    spatial centre transforms to a constant, a constant to a delta at the frequency centre."""
    r = np.random.default_rng(n)
    x = r.standard_normal((3, n)) + 1j * r.standard_normal((3, n))
    ref = np.fft.fftshift(np.fft.fft(np.fft.ifftshift(x, axes=-1), axis=-1, norm="ortho"), axes=-1)
    got = og.dft_axis(x, 1, centred=True)
    assert np.allclose(got, ref, atol=1e-12)
    refi = np.fft.fftshift(np.fft.ifft(np.fft.ifftshift(x, axes=-1), axis=-1, norm="ortho"), axes=-1)
    assert np.allclose(og.dft_axis(x, 1, inverse=True, centred=True), refi, atol=1e-12)
    assert np.allclose(og.dft_axis(got, 1, inverse=True, centred=True), x, atol=1e-12)          # unitary
    d = np.zeros((1, n), complex)
    d[0, n // 2] = 1.0
    assert np.allclose(og.dft_axis(d, 1, centred=True), 1.0 / np.sqrt(n), atol=1e-12)
    assert np.allclose(og.dft_axis(np.ones((1, n)), 1, centred=True), np.sqrt(n) * d, atol=1e-12)
    if n > 2:
        assert not np.allclose(got, og.dft_axis(x, 1), atol=1e-6)                              # and it is a different transform


def test_centred_dft_for_even_lengths_is_sign_flips_around_the_uncentred_one():
    """For even n: F_c = (-1)^(n/2) D F D with D = diag((-1)^index): the identity the device path uses to run the
    centred variant on its uncentred transform (sign of the inputs and outputs, nothing else)."""
    for n in (2, 4, 6, 10, 46, 160):
        r = np.random.default_rng(n)
        x = r.standard_normal(n) + 1j * r.standard_normal(n)
        D = (-1.0) ** np.arange(n)
        s = (-1.0) ** (n // 2)
        assert np.allclose(og.dft_axis(x[None], 1, centred=True)[0], s * D * og.dft_axis((D * x)[None], 1)[0], atol=1e-12)


@pytest.mark.parametrize("nd", [1, 2, 3])
def test_centred_operator_adjoint_identity_full_sampling_and_sign_flip_form(nd):
    geom = synth.Geom(nd, 2, 3, 2, 4, 6, 8, centred=1)
    prox = synth.chain_prox([2, 4, 2], [(1, 1, 3, 3)] * 2)
    c = synth.make_custom(40 + nd, geom, prox, accel=2.0, centre=2, mask_kind="random2d" if nd > 1 else "uniform", sigma=0.0)
    r = np.random.default_rng(nd)
    x = r.standard_normal(geom.image_shape) + 1j * r.standard_normal(geom.image_shape)
    z = r.standard_normal(geom.kspace_shape) + 1j * r.standard_normal(geom.kspace_shape)
    Ax = og.sense_forward(x, c.S, c.M, nd, centred=True)
    AHz = og.sense_adjoint(z, c.S, c.M, nd, centred=True)
    assert np.isclose(np.vdot(z, Ax), np.vdot(AHz, x), rtol=1e-12)                            # <Ax, z> = <x, A^H z>
    ones = np.ones_like(c.M)
    assert np.allclose(og.sense_normal(x, c.S, ones, nd, centred=True), x, atol=1e-12)          # full sampling: identity
    # the generator's measurement (library FFT with shifts) is the centred operator, and x_in its adjoint on y
    assert np.allclose(og.sense_forward(c.x_true, c.S, c.M, nd, centred=True), c.y, atol=1e-5)
    assert np.allclose(og.sense_adjoint(c.y, c.S, c.M, nd, centred=True), c.x_in, atol=1e-5)
    # sign-flip form of the whole data-consistency step: u = D dc_uncentred(D x, s D y) with the mask array as stored
    axes = geom.image_shape[5 - nd:]
    idx = np.indices(axes).sum(0)
    D = (-1.0) ** idx
    s = np.prod([(-1.0) ** (n // 2) for n in axes])
    u_c = og.dc_step(x, c.S, c.M, c.y, 0.8, nd, centred=True)
    u_u = D * og.dc_step(D * x, c.S, c.M, s * D * c.y, 0.8, nd)
    assert np.allclose(u_c, u_u, atol=1e-10)
    # and the mask of a centred case keeps its low frequencies in the middle of the array
    mid = tuple(n // 2 for n in axes)
    assert np.all(c.M[(slice(None),) * (5 - nd) + mid] == 1) or nd == 1


def test_generator_mask_counts_all_configs():
    g = synth
    rng = np.random.default_rng(1)
    assert len(g._draw_lines(rng, 368, 46, 15, "vd")) == 46
    l3 = g._draw_lines(rng, 320, 80, 26, "equi")
    assert len(l3) == 80 and len(set(l3)) == 80
    assert len(g._draw_lines(rng, 160, 13, 8, "vd")) == 13
    plane = g.poisson_disc_plane(rng, 40, 40, 200, 6)
    assert plane.sum() == 200 and plane[np.ix_(g.lowest_freq_indices(40, 6), g.lowest_freq_indices(40, 6))].all()


def test_mask_constant_along_an_axis_reduces_the_transform_dimension():
    """A mask that does not depend on H commutes with the transform along H, so the 2D operator on (x, y) equals
    the 1D operator (W only, H as a batch axis) on y inverse-transformed along H: the identity behind
    ndim_fft = 1 (and behind decoupling a fully sampled read-out)."""
    from paper_2207_08393_amd import synth
    c = synth.make_custom(5, synth.Geom(2, 2, 3, 1, 1, 6, 8), synth.resblock_prox(2, 1), accel=2.0, centre=2)
    assert np.all(c.M == c.M[..., :1, :])                         # 1D line mask: constant along H
    x = c.x_in.astype(np.complex128)
    y = c.y.astype(np.complex128)
    y_hyb = og.dft_axis(y, axis=y.ndim - 2, inverse=True)         # k-space -> (h, kw) hybrid space
    assert np.allclose(og.sense_normal(x, c.S, c.M, 2), og.sense_normal(x, c.S, c.M, 1), atol=1e-12)
    assert np.allclose(og.dc_step(x, c.S, c.M, y, 0.7, 2), og.dc_step(x, c.S, c.M, y_hyb, 0.7, 1), atol=1e-12)
    # and a mask that does depend on H breaks it
    M2 = c.M.copy()
    M2[..., 0, :] = 1 - M2[..., 0, :]
    assert not np.allclose(og.sense_normal(x, c.S, M2, 2), og.sense_normal(x, c.S, M2, 1), atol=1e-6)
