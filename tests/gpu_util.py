"""Helpers for the GPU parity tests."""
import numpy as np

from paper_2207_08393_amd.runner import ModuleRunner, SenseRunner  # noqa: F401


def rel_l2(a, b):
    a = np.asarray(a).astype(np.complex128 if np.iscomplexobj(a) else np.float64)
    b = np.asarray(b).astype(a.dtype)
    return float(np.linalg.norm((a - b).ravel()) / max(np.linalg.norm(b.ravel()), 1e-300))


def run_sense_normal(geom, x, S, M):
    r = SenseRunner(geom, x, S, M)
    r.run()
    return r.result()


def elementwise_factor(n):
    """An error field that meets a relative-L2 tolerance `tol` with independent rounding errors has a per-element
    standard deviation of at most tol * rms(ref) <= tol * max|ref|, and the largest of n such errors stays below
    sqrt(2 ln 2n) standard deviations (3.9 for n = 1000, 5.0 for n = 150 000).  A single wrong value of the size of
    the data is 1 / tol of that scale and cannot pass."""
    return max(1.0, float(np.sqrt(2.0 * np.log(2.0 * max(int(n), 1)))))


def assert_close(got, ref, tol, what, sup=None):
    """Relative L2 <= tol (the stated tolerance), and every element within elementwise_factor(n) * tol * max|ref| of
    its reference, so that a wrong value cannot hide behind the norm of the rest (`sup`, when given, replaces that
    element-wise bound, as a fraction of max|ref|).  A reference that is exactly zero must be matched exactly."""
    got = np.asarray(got)
    ref = np.asarray(ref)
    assert got.shape == ref.shape, (what, got.shape, ref.shape)
    assert np.all(np.isfinite(got)), what
    scale = float(np.abs(ref).max()) if ref.size else 0.0
    if scale == 0.0:
        assert not np.any(got), what
        return 0.0
    err = rel_l2(got, ref)
    worst = float(np.abs(got.astype(ref.dtype if np.iscomplexobj(ref) else np.float64) - ref).max()) / scale
    assert err <= tol, (what, "rel-L2", err, "tol", tol)
    bound = elementwise_factor(ref.size) * tol if sup is None else sup
    assert worst <= bound, (what, "max |d| / max |ref|", worst, "bound", bound)
    return err


def theta_slices(prox):
    """(layer index, 'W' or 'b', slice into the flat parameter vector) in the library's layout."""
    out, off = [], 0
    for i, l in enumerate(prox.layers):
        out.append((i + 1, "W", slice(off, off + l.n_weight)))
        off += l.n_weight
        if l.has_bias:
            out.append((i + 1, "b", slice(off, off + l.cout)))
            off += l.cout
    return out


def assert_grad_close(prox, got, ref, tol, what="grad_theta", exact=None, share=0.15):
    """Weights and bias of every layer separately: relative L2 and the element-wise bound of assert_close.
    With `exact` (the exact oracle's gradient, `ref` being the oracle run with the bfloat16 rounding points) a
    layer's tolerance is max(tol, share * relative distance between ref and exact in that layer): what separates
    the library from the rounding-point oracle is float32 against float64 accumulation, which moves a stored
    bfloat16 value by one spacing in about 6e-4 of the elements, i.e. by about a tenth (1.2e-4 against 2^-9 / sqrt 3
    = 1.1e-3) of what the rounding itself moves it; a layer whose gradient the rounding moves a lot (the first
    layer's, which sums over all later ReLU masks) is moved proportionally more by that difference too.  Both
    terms come from the oracle alone."""
    got = np.asarray(got)
    ref = np.asarray(ref)
    assert got.shape == ref.shape == (prox.n_theta,), (got.shape, ref.shape, prox.n_theta)
    errs = {}
    for layer, kind, sl in theta_slices(prox):
        t = tol
        if exact is not None and np.any(ref[sl]):
            t = max(tol, share * rel_l2(np.asarray(exact)[sl], ref[sl]))
        errs[f"{kind}{layer}"] = assert_close(got[sl], ref[sl], t, f"{what} layer {layer} {kind}")
    return errs


def assert_image_close(got, ref, tol, what="x_out", sup=None):
    """Per batch sample (axis 0)."""
    return [assert_close(got[b], ref[b], tol, f"{what} sample {b}", sup) for b in range(ref.shape[0])]
