"""gleam_sense_normal_static (the entry point for callers that cannot allocate: its coil k-space buffer is a
file-scope device array) against gleam_sense_normal through the C ABI: two calls in a row, the second on a
smaller problem, so that whatever the first call left in the shared array must not leak into the second."""
import ctypes as C

import numpy as np
import pytest
import torch

from oracle import gleam_oracle as og
from paper_2207_08393_amd import binding as gb
from paper_2207_08393_amd import synth
from paper_2207_08393_amd.runner import byte_buffer, cplx, dev, to_complex
from tests.gpu_util import rel_l2

pytestmark = pytest.mark.gpu
K2 = (1, 1, 3, 3)


def _both(geom_s, c):
    """(static entry point, workspace entry point) results for one case, called through the raw C ABI."""
    L = gb.lib()
    geom = gb.make_geom(geom_s)
    x, S, M = cplx(c.x_true), cplx(c.S), dev(c.M)
    out_s = torch.full_like(x, float("nan"))
    out_w = torch.full_like(x, float("nan"))
    ws_bytes, _ = gb.gleam_workspace_bytes(geom, None)
    ws = byte_buffer(ws_bytes)
    st = torch.cuda.current_stream().cuda_stream or None
    rc = L.gleam_sense_normal_static(C.byref(geom), x.data_ptr(), S.data_ptr(), M.data_ptr(), out_s.data_ptr(), st)
    assert rc == gb.GLEAM_OK, gb.strerror(rc)
    rc = L.gleam_sense_normal(C.byref(geom), x.data_ptr(), S.data_ptr(), M.data_ptr(), out_w.data_ptr(), ws.data_ptr(),
                              ws_bytes, st)
    assert rc == gb.GLEAM_OK, gb.strerror(rc)
    torch.cuda.synchronize()
    return to_complex(out_s), to_complex(out_w)


def test_static_scratch_entry_point_matches_the_workspace_one_twice_in_a_row():
    prox = synth.chain_prox([2, 4, 2], [K2] * 2)
    big = synth.Geom(2, 2, 3, 2, 1, 96, 64)            # 73 728 coil-pixels, several tiles per sweep
    small = synth.Geom(3, 1, 2, 1, 8, 12, 10)          # smaller, another transform dimension: stale k-space around it
    knee = synth.Geom(2, 2, 15, 1, 1, 640, 368)        # 56.5 MB of k-space: close to the 64 MiB limit
    for seed, g in ((6, knee), (7, big), (8, small)):
        c = synth.make_custom(seed, g, prox, accel=3.0, centre=2, mask_kind="random2d")
        print("case static scratch", g, flush=True)
        got, ref = _both(g, c)
        assert np.array_equal(got.view(np.uint32), ref.view(np.uint32))      # same kernels: bit-identical
        assert rel_l2(got, og.sense_normal(c.x_true, c.S, c.M, g.ndim_fft)) <= 1e-4


def test_static_scratch_entry_point_rejects_what_does_not_fit():
    L = gb.lib()
    # 640 x 368 x 15 coils x batch 3 = 84.8 MB of k-space: beyond the 64 MiB array
    geom = gb.make_geom(synth.Geom(2, 3, 15, 1, 1, 640, 368))
    assert 3 * 15 * 640 * 368 * 8 > gb.STATIC_SCRATCH_BYTES
    one = torch.zeros(256, dtype=torch.uint8, device="cuda")     # never touched: the size check comes first
    rc = L.gleam_sense_normal_static(C.byref(geom), one.data_ptr(), one.data_ptr(), one.data_ptr(), one.data_ptr(), None)
    assert rc == gb.GLEAM_E_WORKSPACE
    rc = L.gleam_sense_normal_static(C.byref(geom), None, one.data_ptr(), one.data_ptr(), one.data_ptr(), None)
    assert rc == gb.GLEAM_E_NULL
