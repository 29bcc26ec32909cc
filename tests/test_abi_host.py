"""Host-only checks of the C ABI: the library loads, exports every symbol the header declares, and
rejects bad arguments on the host before anything could be launched (no GPU needed)."""
import ctypes as C
import os
import re

import pytest

from paper_2207_08393_amd import binding as gb
from paper_2207_08393_amd import synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "gleam.h")).read()
    declared = set(re.findall(r"\b(gleam_[a-z_0-9]+)\s*\(", header))
    assert {"gleam_sense_normal", "gleam_module_fwd", "gleam_module_bwd"} <= declared
    lib = gb.lib()
    for name in declared:
        assert hasattr(lib, name), name
    assert declared == set(gb.EXPORTS)


def test_strerror_and_counts():
    assert gb.strerror(0) == "ok"
    for code in range(-6, 0):
        assert gb.strerror(code) and "unknown" not in gb.strerror(code)
    assert "unknown" in gb.strerror(-99)
    c = synth.make_case(0)
    prox = gb.make_prox(c.prox)
    assert gb.gleam_theta_count(prox) == c.theta.size == c.prox.n_theta
    ws, saved = gb.gleam_workspace_bytes(gb.make_geom(c.geom), prox)
    Q = 64 * 64
    assert saved >= Q * 4 * (2 + 16 + 16 + 2) and ws >= 8 * c.geom.E and ws % 256 == 0 and saved % 256 == 0
    ws0, saved0 = gb.gleam_workspace_bytes(gb.make_geom(c.geom), None)
    assert saved0 == 0 and ws0 >= 8 * c.geom.E
    for n in (64, 640, 368, 320, 256, 160, 192):
        assert gb.gleam_fft_size_supported(n)
    assert not gb.gleam_fft_size_supported(7) and not gb.gleam_fft_size_supported(0)


def _status(fn, *a):
    with pytest.raises(gb.GleamError) as e:
        fn(*a)
    return e.value.status


def test_bad_geometry_and_sizes_are_rejected():
    good = synth.Geom(2, 1, 2, 1, 1, 8, 8)
    for field, val, code in (("ndim_fft", 0, gb.GLEAM_E_DIMS), ("ndim_fft", 4, gb.GLEAM_E_DIMS),
                             ("B", 0, gb.GLEAM_E_DIMS), ("C", -1, gb.GLEAM_E_DIMS),
                             ("W", 7, gb.GLEAM_E_UNSUPPORTED_SIZE), ("H", 9, gb.GLEAM_E_UNSUPPORTED_SIZE)):
        g = synth.Geom(**{**good.__dict__, field: val})
        assert _status(gb.gleam_workspace_bytes, gb.make_geom(g), None) == code
    g3 = synth.Geom(3, 1, 2, 1, 7, 8, 8)
    assert _status(gb.gleam_workspace_bytes, gb.make_geom(g3), None) == gb.GLEAM_E_UNSUPPORTED_SIZE
    g2 = synth.Geom(2, 1, 2, 1, 7, 8, 8)     # D is only batched for ndim_fft = 2
    gb.gleam_workspace_bytes(gb.make_geom(g2), None)


def test_bad_prox_descriptions_are_rejected():
    geom = gb.make_geom(synth.Geom(2, 1, 2, 1, 1, 8, 8))
    k = (1, 1, 3, 3)
    ok = synth.chain_prox([2, 4, 2], [k, k])
    gb.gleam_workspace_bytes(geom, gb.make_prox(ok))

    def bad(mut):
        p = synth.chain_prox([2, 4, 2], [k, k])
        mut(p)
        return _status(gb.gleam_workspace_bytes, geom, gb.make_prox(p))

    assert bad(lambda p: setattr(p.layers[0], "cin", 3)) == gb.GLEAM_E_DESC
    assert bad(lambda p: setattr(p.layers[1], "cout", 3)) == gb.GLEAM_E_DESC
    assert bad(lambda p: setattr(p.layers[1], "cin", 5)) == gb.GLEAM_E_DESC
    assert bad(lambda p: setattr(p.layers[0], "kh", 2)) == gb.GLEAM_E_DESC
    assert bad(lambda p: setattr(p.layers[0], "kw", 9)) == gb.GLEAM_E_DESC
    assert bad(lambda p: setattr(p.layers[1], "skip_src", 1)) == gb.GLEAM_E_DESC   # 4 channels into 2
    assert bad(lambda p: setattr(p.layers[1], "skip_src", 5)) == gb.GLEAM_E_DESC
    assert bad(lambda p: setattr(p.layers[1], "relu_out", 1)) == gb.GLEAM_E_DESC   # relu_out with a skip
    assert bad(lambda p: setattr(p, "dtype", 7)) == gb.GLEAM_E_DESC
    assert bad(lambda p: setattr(p, "loss_kind", 2)) == gb.GLEAM_E_DESC
    empty = synth.ProxDesc([])
    assert _status(gb.gleam_workspace_bytes, geom, gb.make_prox(empty)) == gb.GLEAM_E_DESC


def test_null_pointers_and_short_workspace_are_rejected_before_launch():
    c = synth.make_case(0)
    geom, prox = gb.make_geom(c.geom), gb.make_prox(c.prox)
    ws, saved = gb.gleam_workspace_bytes(geom, prox)
    fake = 0x1000  # 256-byte aligned, never dereferenced: validation fails first
    L = gb.lib()
    assert L.gleam_sense_normal(C.byref(geom), None, fake, fake, fake, fake, ws, None) == gb.GLEAM_E_NULL
    assert L.gleam_sense_normal(C.byref(geom), fake, fake, fake, None, fake, ws, None) == gb.GLEAM_E_NULL
    assert L.gleam_sense_normal(C.byref(geom), fake, fake, fake, fake, fake, 16, None) == gb.GLEAM_E_WORKSPACE
    assert L.gleam_sense_normal(C.byref(geom), fake, fake, fake, fake, fake + 8, ws, None) == gb.GLEAM_E_WORKSPACE
    assert L.gleam_sense_normal(None, fake, fake, fake, fake, fake, ws, None) == gb.GLEAM_E_NULL
    args = [C.byref(geom), C.byref(prox), fake, fake, fake, fake, C.c_float(1.0), fake, fake, fake, fake,
            fake, saved, fake, ws, None]
    for i in (2, 3, 4, 5, 7, 9, 10, 11, 13):
        a = list(args)
        a[i] = None
        assert L.gleam_module_fwd(*a) == gb.GLEAM_E_NULL, i
    a = list(args); a[12] = saved - 256
    assert L.gleam_module_fwd(*a) == gb.GLEAM_E_WORKSPACE
    a = list(args); a[14] = ws - 256
    assert L.gleam_module_fwd(*a) == gb.GLEAM_E_WORKSPACE
    bargs = [C.byref(geom), C.byref(prox), fake, fake, saved, fake, fake, ws, None]
    for i in (2, 3, 5, 6):
        a = list(bargs)
        a[i] = None
        assert L.gleam_module_bwd(*a) == gb.GLEAM_E_NULL, i
    a = list(bargs); a[4] = 0
    assert L.gleam_module_bwd(*a) == gb.GLEAM_E_WORKSPACE
    assert L.gleam_theta_count(C.byref(prox), None) == gb.GLEAM_E_NULL


def test_greedy_entry_points_reject_bad_arguments_before_launch():
    c = synth.make_case(0)
    geom, prox = gb.make_geom(c.geom), gb.make_prox(c.prox)
    ws, saved = gb.gleam_workspace_bytes(geom, prox)
    fake = 0x1000
    L = gb.lib()
    h = gb.make_adam(1e-3)
    assert L.gleam_adam_step(None, 1, 4, fake, fake, fake, fake, None) == gb.GLEAM_E_NULL
    assert L.gleam_adam_step(C.byref(h), 1, 4, fake, None, fake, fake, None) == gb.GLEAM_E_NULL
    assert L.gleam_adam_step(C.byref(h), 0, 4, fake, fake, fake, fake, None) == gb.GLEAM_E_DESC     # t starts at 1
    bad = gb.make_adam(1e-3, beta1=1.0)
    assert L.gleam_adam_step(C.byref(bad), 1, 4, fake, fake, fake, fake, None) == gb.GLEAM_E_DESC
    assert L.gleam_adam_step(C.byref(h), 1, 0, fake, fake, fake, fake, None) == gb.GLEAM_OK          # nothing to do
    x0, xo, xt = 0x1000, 0x2000, 0x3000
    args = [C.byref(geom), C.byref(prox), 2, x0, fake, fake, fake, C.c_float(1.0), fake, fake, fake, C.byref(h), 1,
            fake, xo, xt, fake, fake, fake, saved, fake, ws, None]
    a = list(args); a[2] = 0
    assert L.gleam_greedy_iteration(*a) == gb.GLEAM_E_DIMS
    for i in (3, 8, 9, 10, 13, 14, 15, 16, 17):
        a = list(args); a[i] = None
        assert L.gleam_greedy_iteration(*a) == gb.GLEAM_E_NULL, i
    a = list(args); a[14] = x0          # output aliases the input image
    assert L.gleam_greedy_iteration(*a) == gb.GLEAM_E_DIMS
    a = list(args); a[15] = xo          # scratch image aliases the output
    assert L.gleam_greedy_iteration(*a) == gb.GLEAM_E_DIMS
    a = list(args); a[21] = ws - 256    # short workspace: refused before any launch
    assert L.gleam_greedy_iteration(*a) == gb.GLEAM_E_WORKSPACE
    a = list(args); a[19] = saved - 256
    assert L.gleam_greedy_iteration(*a) == gb.GLEAM_E_WORKSPACE
    # what the Adam update of module 1 would refuse is refused up front too, not after module 1 has run
    a = list(args); a[12] = 0
    assert L.gleam_greedy_iteration(*a) == gb.GLEAM_E_DESC
    a = list(args); a[11] = C.byref(bad)
    assert L.gleam_greedy_iteration(*a) == gb.GLEAM_E_DESC
    for i in (4, 5, 6):
        a = list(args); a[i] = None
        assert L.gleam_greedy_iteration(*a) == gb.GLEAM_E_NULL, i
    iargs = [C.byref(geom), C.byref(prox), 2, x0, fake, fake, fake, C.c_float(1.0), fake, xo, xt, fake, ws, None]
    a = list(iargs); a[2] = -1
    assert L.gleam_unrolled_infer(*a) == gb.GLEAM_E_DIMS
    a = list(iargs); a[8] = None
    assert L.gleam_unrolled_infer(*a) == gb.GLEAM_E_NULL
    a = list(iargs); a[9] = x0
    assert L.gleam_unrolled_infer(*a) == gb.GLEAM_E_DIMS
    a = list(iargs); a[12] = ws - 256
    assert L.gleam_unrolled_infer(*a) == gb.GLEAM_E_WORKSPACE
    a = list(iargs); a[5] = None
    assert L.gleam_unrolled_infer(*a) == gb.GLEAM_E_NULL


def test_deep_module_entry_points_reject_bad_arguments_before_launch():
    c = synth.make_case(0)
    geom, prox = gb.make_geom(c.geom), gb.make_prox(c.prox)
    ws1, saved1 = gb.gleam_workspace_bytes(geom, prox)
    ws, saved = gb.gleam_deep_workspace_bytes(geom, prox, 3)
    assert ws == ws1 and saved >= 3 * saved1 and saved % 256 == 0
    assert gb.gleam_deep_workspace_bytes(geom, prox, 1) == (ws1, (saved1 + 255) // 256 * 256)
    L = gb.lib()
    w, s = C.c_size_t(0), C.c_size_t(0)
    assert L.gleam_deep_workspace_bytes(C.byref(geom), C.byref(prox), 0, C.byref(w), C.byref(s)) == gb.GLEAM_E_DIMS
    # several iterations need the gradient with respect to the prox input: no ReLU on the input, one skip from it at most
    relu_first = synth.chain_prox([2, 8, 2], [(1, 1, 3, 3)] * 2)
    relu_first.layers[0].relu_in = 1
    p = gb.make_prox(relu_first)
    assert L.gleam_deep_workspace_bytes(C.byref(geom), C.byref(p), 2, C.byref(w), C.byref(s)) == gb.GLEAM_E_DESC
    assert L.gleam_deep_workspace_bytes(C.byref(geom), C.byref(p), 1, C.byref(w), C.byref(s)) == gb.GLEAM_OK
    two_skips = synth.chain_prox([2, 2, 2], [(1, 1, 3, 3)] * 2)
    two_skips.layers[0].skip_src = 0
    two_skips.layers[1].skip_src = 0
    p = gb.make_prox(two_skips)
    assert L.gleam_deep_workspace_bytes(C.byref(geom), C.byref(p), 2, C.byref(w), C.byref(s)) == gb.GLEAM_E_DESC
    ws, saved = gb.gleam_deep_workspace_bytes(geom, prox, 2)
    fake, x0, xo, xt = 0x1000, 0x1000, 0x2000, 0x3000
    fargs = [C.byref(geom), C.byref(prox), 2, x0, fake, fake, fake, C.c_float(1.0), fake, fake, xo, xt, fake, fake, saved,
             fake, ws, None]
    for i in (3, 8, 9, 10, 11, 12, 13):
        a = list(fargs); a[i] = None
        assert L.gleam_deep_module_fwd(*a) == gb.GLEAM_E_NULL, i
    a = list(fargs); a[10] = x0
    assert L.gleam_deep_module_fwd(*a) == gb.GLEAM_E_DIMS
    a = list(fargs); a[11] = xo
    assert L.gleam_deep_module_fwd(*a) == gb.GLEAM_E_DIMS
    a = list(fargs); a[14] = saved - 256
    assert L.gleam_deep_module_fwd(*a) == gb.GLEAM_E_WORKSPACE
    a = list(fargs); a[16] = ws - 256
    assert L.gleam_deep_module_fwd(*a) == gb.GLEAM_E_WORKSPACE
    for i in (4, 5, 6, 15):
        a = list(fargs); a[i] = None
        assert L.gleam_deep_module_fwd(*a) == gb.GLEAM_E_NULL, i
    bargs = [C.byref(geom), C.byref(prox), 2, fake, fake, C.c_float(1.0), fake, fake, saved, fake, fake, ws, None]
    for i in (3, 4, 6, 7, 9, 10):
        a = list(bargs); a[i] = None
        assert L.gleam_deep_module_bwd(*a) == gb.GLEAM_E_NULL, i
    a = list(bargs); a[8] = saved - 256
    assert L.gleam_deep_module_bwd(*a) == gb.GLEAM_E_WORKSPACE
    a = list(bargs); a[11] = ws - 256
    assert L.gleam_deep_module_bwd(*a) == gb.GLEAM_E_WORKSPACE
    a = list(bargs); a[2] = 0
    assert L.gleam_deep_module_bwd(*a) == gb.GLEAM_E_DIMS


def test_modl_entry_points_reject_bad_arguments_before_launch():
    c = synth.make_case(0)
    geom, prox = gb.make_geom(c.geom), gb.make_prox(c.prox)
    ws1, saved1 = gb.gleam_workspace_bytes(geom, prox)
    ws, saved = gb.gleam_modl_workspace_bytes(geom, prox)
    n_img = c.geom.B * c.geom.T * c.geom.D * c.geom.H * c.geom.W * 8
    assert saved == saved1 and ws >= ws1 + 3 * n_img      # residual, direction and operator output
    L = gb.lib()
    fake, x0, xo, aty = 0x1000, 0x2000, 0x3000, 0x4000
    mu = C.c_float(0.5)
    fargs = [C.byref(geom), C.byref(prox), x0, fake, fake, aty, mu, 10, fake, fake, xo, fake, fake, saved, fake, ws, None]
    for i in (2, 3, 4, 5, 8, 10, 11, 12, 14):
        a = list(fargs); a[i] = None
        assert L.gleam_modl_module_fwd(*a) == gb.GLEAM_E_NULL, i
    a = list(fargs); a[10] = x0
    assert L.gleam_modl_module_fwd(*a) == gb.GLEAM_E_DIMS
    a = list(fargs); a[10] = aty
    assert L.gleam_modl_module_fwd(*a) == gb.GLEAM_E_DIMS
    a = list(fargs); a[7] = 0
    assert L.gleam_modl_module_fwd(*a) == gb.GLEAM_E_DIMS
    a = list(fargs); a[6] = C.c_float(-1.0)
    assert L.gleam_modl_module_fwd(*a) == gb.GLEAM_E_DIMS
    a = list(fargs); a[6] = C.c_float(float("nan"))
    assert L.gleam_modl_module_fwd(*a) == gb.GLEAM_E_DIMS
    a = list(fargs); a[15] = ws1                          # a plain module workspace is too small for the solver
    assert L.gleam_modl_module_fwd(*a) == gb.GLEAM_E_WORKSPACE
    a = list(fargs); a[13] = saved - 256
    assert L.gleam_modl_module_fwd(*a) == gb.GLEAM_E_WORKSPACE
    bargs = [C.byref(geom), C.byref(prox), fake, fake, mu, 10, fake, fake, saved, fake, fake, ws, None]
    for i in (2, 3, 6, 7, 9, 10):
        a = list(bargs); a[i] = None
        assert L.gleam_modl_module_bwd(*a) == gb.GLEAM_E_NULL, i
    a = list(bargs); a[5] = -3
    assert L.gleam_modl_module_bwd(*a) == gb.GLEAM_E_DIMS
    a = list(bargs); a[11] = ws - 256
    assert L.gleam_modl_module_bwd(*a) == gb.GLEAM_E_WORKSPACE
    # a prox that ends in a ReLU would need the mask of z behind the solve: not supported
    relu_last = synth.chain_prox([2, 8, 2], [(1, 1, 3, 3)] * 2)
    relu_last.layers[-1].relu_out = 1
    p = gb.make_prox(relu_last)
    w, s = C.c_size_t(0), C.c_size_t(0)
    assert L.gleam_modl_workspace_bytes(C.byref(geom), C.byref(p), C.byref(w), C.byref(s)) == gb.GLEAM_E_DESC
    # adjoint
    aargs = [C.byref(geom), fake, fake, x0, xo, fake, ws, None]
    for i in (1, 2, 3, 4, 5):
        a = list(aargs); a[i] = None
        assert L.gleam_sense_adjoint(*a) == gb.GLEAM_E_NULL, i
    a = list(aargs); a[4] = x0
    assert L.gleam_sense_adjoint(*a) == gb.GLEAM_E_DIMS
    a = list(aargs); a[6] = 1024
    assert L.gleam_sense_adjoint(*a) == gb.GLEAM_E_WORKSPACE


def test_step_size_gradient_entry_point_rejects_bad_arguments_before_launch():
    c = synth.make_case(0)
    geom, prox = gb.make_geom(c.geom), gb.make_prox(c.prox)
    ws, saved = gb.gleam_workspace_bytes(geom, prox)
    L = gb.lib()
    fake = 0x1000
    args = [C.byref(geom), C.byref(prox), fake, fake, fake, fake, fake, fake, saved, fake, fake, fake, ws, None]
    for i in (2, 3, 4, 5, 6, 7, 9, 10, 11):
        a = list(args); a[i] = None
        assert L.gleam_module_bwd_alpha(*a) == gb.GLEAM_E_NULL, i
    a = list(args); a[8] = saved - 256
    assert L.gleam_module_bwd_alpha(*a) == gb.GLEAM_E_WORKSPACE
    a = list(args); a[12] = ws - 256
    assert L.gleam_module_bwd_alpha(*a) == gb.GLEAM_E_WORKSPACE
    relu_first = synth.chain_prox([2, 8, 2], [(1, 1, 3, 3)] * 2)
    relu_first.layers[0].relu_in = 1
    p = gb.make_prox(relu_first)
    a = list(args); a[1] = C.byref(p)
    assert L.gleam_module_bwd_alpha(*a) == gb.GLEAM_E_DESC


def test_single_axis_geometry_is_accepted_and_needs_only_w_to_have_a_transform():
    prox = gb.make_prox(synth.resblock_prox(4, 1))
    g = gb.make_geom(synth.Geom(1, 1, 2, 1, 3, 7, 64))            # H = 7 has no transform kernel, and needs none
    ws, saved = gb.gleam_workspace_bytes(g, prox)
    assert ws > 0 and saved > 0
    w, s_ = C.c_size_t(0), C.c_size_t(0)
    bad = gb.make_geom(synth.Geom(1, 1, 2, 1, 1, 8, 7))
    assert gb.lib().gleam_workspace_bytes(C.byref(bad), C.byref(prox), C.byref(w), C.byref(s_)) == gb.GLEAM_E_UNSUPPORTED_SIZE
    bad = gb.make_geom(synth.Geom(0, 1, 2, 1, 1, 8, 8))
    assert gb.lib().gleam_workspace_bytes(C.byref(bad), C.byref(prox), C.byref(w), C.byref(s_)) == gb.GLEAM_E_DIMS


def test_kernel_policy_is_an_explicit_process_wide_word_and_not_the_environment():
    assert gb.gleam_get_kernel_policy() == 0                       # default: the fastest kernels
    try:
        gb.gleam_set_kernel_policy(gb.POLICY_NO_WINOGRAD | gb.POLICY_NO_THIN_MFMA)
        assert gb.gleam_get_kernel_policy() == 5
        assert _status(gb.gleam_set_kernel_policy, 32) == gb.GLEAM_E_DESC      # unknown bit
        assert gb.gleam_get_kernel_policy() == 5                               # and nothing changed
    finally:
        gb.gleam_set_kernel_policy(0)
    src = os.path.join(ROOT, "paper_2207_08393_amd", "csrc")
    for name in os.listdir(src):
        assert "getenv" not in open(os.path.join(src, name)).read(), name


def test_static_scratch_entry_point_checks_on_the_host_first():
    L = gb.lib()
    fake = 0x1000
    too_big = gb.make_geom(synth.Geom(2, 3, 15, 1, 1, 640, 368))               # 84.8 MB of k-space > 64 MiB
    assert L.gleam_sense_normal_static(C.byref(too_big), fake, fake, fake, fake, None) == gb.GLEAM_E_WORKSPACE
    assert L.gleam_sense_normal_static(C.byref(too_big), fake, None, fake, fake, None) == gb.GLEAM_E_NULL
    bad = gb.make_geom(synth.Geom(2, 1, 2, 1, 1, 8, 7))
    assert L.gleam_sense_normal_static(C.byref(bad), fake, fake, fake, fake, None) == gb.GLEAM_E_UNSUPPORTED_SIZE


def test_centred_flag_and_hybrid_space_entry_points_check_on_the_host():
    import numpy as np
    L = gb.lib()
    fake = 0x1000
    w, s_ = C.c_size_t(0), C.c_size_t(0)
    bad = gb.make_geom(synth.Geom(2, 1, 2, 1, 1, 8, 8, centred=2))
    assert L.gleam_workspace_bytes(C.byref(bad), None, C.byref(w), C.byref(s_)) == gb.GLEAM_E_DIMS
    ok = gb.make_geom(synth.Geom(2, 1, 2, 1, 1, 8, 8, centred=1))
    assert L.gleam_workspace_bytes(C.byref(ok), None, C.byref(w), C.byref(s_)) == gb.GLEAM_OK
    assert L.gleam_kspace_to_hybrid(C.byref(ok), None, fake, None) == gb.GLEAM_E_NULL
    assert L.gleam_kspace_to_hybrid(C.byref(ok), fake, None, None) == gb.GLEAM_E_NULL
    one_axis = gb.make_geom(synth.Geom(1, 1, 2, 1, 1, 8, 8))
    assert L.gleam_kspace_to_hybrid(C.byref(one_axis), fake, fake, None) == gb.GLEAM_E_DIMS       # no axis to remove
    # mask check: nonzero-ness, per outer index, along H (two transformed axes) or D (three)
    g2 = synth.Geom(2, 2, 1, 2, 3, 4, 6)
    M = np.zeros(g2.image_shape, np.uint8)
    M[..., [0, 3]] = 1                                  # lines along W, the same for every H: constant along H
    M[1, 1, 2, :, 5] = 7                                # another line in one slice, any non-zero byte counts
    assert gb.gleam_mask_constant_along_outer_axis(gb.make_geom(g2), M)
    M2 = M.copy(); M2[1, 0, 1, 2, 4] = 1                # one extra point: H matters now
    assert not gb.gleam_mask_constant_along_outer_axis(gb.make_geom(g2), M2)
    g3 = synth.Geom(3, 1, 1, 2, 4, 4, 6)
    P = (np.random.default_rng(0).random((1, 2, 1, 4, 6)) < 0.4).astype(np.uint8)
    M3 = np.broadcast_to(P, g3.image_shape).copy()      # a pattern on the (H, W) plane, the same for every D
    assert gb.gleam_mask_constant_along_outer_axis(gb.make_geom(g3), M3)
    M3[0, 1, 2, 0, 0] ^= 1
    assert not gb.gleam_mask_constant_along_outer_axis(gb.make_geom(g3), M3)
    out = C.c_int(0)
    assert L.gleam_mask_constant_along_outer_axis(C.byref(one_axis), fake, C.byref(out)) == gb.GLEAM_E_DIMS
    assert L.gleam_mask_constant_along_outer_axis(C.byref(ok), None, C.byref(out)) == gb.GLEAM_E_NULL
