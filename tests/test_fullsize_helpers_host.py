"""The checks used on task sizes the serial checker cannot recompute whole, tried on the CPU on
sizes it can: each must accept the checker's own full result and refuse a planted mistake."""
import numpy as np
import pytest

import oracle
import workloads as W
from helpers import (FREIVALDS_TOL, band_samples, cnn_patch_for, freivalds_ratio, jacobi_cone_check,
                     jacobi_cone_points)


def test_freivalds_accepts_a_rounded_product_and_refuses_a_wrong_block():
    a, b = W.gemm_operands_f32(3, 384, 512, 256)
    c = oracle.gemm_f32(a, b).astype(np.float32)                    # the exact product, rounded once
    assert freivalds_ratio(a, b, c, 1) < 1e-7
    # fp32 accumulation in some other order stays far below the tolerance as well
    assert freivalds_ratio(a, b, (a[:, :128] @ b[:128]) + (a[:, 128:] @ b[128:]), 2) <= FREIVALDS_TOL / 4
    bad = c.copy()
    bad[64:128, 192:256] = c[128:192, 192:256]                      # one 64 x 64 block from the wrong rows
    assert freivalds_ratio(a, b, bad, 1) > 50 * FREIVALDS_TOL
    bad = c.copy()
    bad[200, 300] += 8.0                                            # one entry off by about its own size
    assert freivalds_ratio(a, b, bad, 1) > FREIVALDS_TOL
    assert freivalds_ratio(a, b, c.T.copy() if c.shape[0] == c.shape[1] else np.zeros_like(c), 1) > 1e-2


def test_band_samples_reach_every_block():
    rows, cols = band_samples(1000, 700, 64, 5)
    assert len(rows) == 16 and len(cols) == 11
    assert all(64 * i <= r < min(1000, 64 * (i + 1)) for i, r in enumerate(rows))
    assert all(64 * i <= c < min(700, 64 * (i + 1)) for i, c in enumerate(cols))


def test_cone_check_equals_the_full_sweep_and_sees_a_wrong_cell():
    n, it = 300, 23
    u = W.jacobi_field(9, n)
    full = oracle.jacobi_f32(u, it)
    pts = jacobi_cone_points(n, it, 4, extra=6)
    jacobi_cone_check(lambda r0, r1, c0, c1: u[r0:r1, c0:c1], lambda r, c: full[r, c], n, it, pts)
    r, c = pts[-1]
    wrong = full.copy()
    wrong[r, c] = np.nextafter(wrong[r, c], np.float32(2.0))        # one unit in the last place
    with pytest.raises(AssertionError):
        jacobi_cone_check(lambda r0, r1, c0, c1: u[r0:r1, c0:c1], lambda rr, cc: wrong[rr, cc], n, it, pts)
    with pytest.raises(AssertionError):                             # one sweep too few
        less = oracle.jacobi_f32(u, it - 1)
        jacobi_cone_check(lambda r0, r1, c0, c1: u[r0:r1, c0:c1], lambda rr, cc: less[rr, cc], n, it, pts)


def test_an_output_pixel_of_the_net_through_its_window_equals_the_whole_image():
    # 160 x 160 = 5 x 5 output pixels: corners, rims and the centre, each recomputed from its window
    h = w = 160
    layers = W.cnn_layers(h, w)
    wts = W.cnn_weights(3, layers)
    x = W.cnn_input(3, 2, h, w)
    strides = [L["stride"] for L in layers]
    full = oracle.cnn_forward(x, wts, strides)
    assert full.shape == (2, 5, 5, 512)
    for b, oy, ox in ((0, 0, 0), (1, 4, 4), (0, 2, 2), (1, 0, 3), (0, 4, 1), (1, 2, 4)):
        y0, y1, x0, x1, ly, lx = cnn_patch_for(oy, ox, h, w)
        assert y0 % 32 == 0 and x0 % 32 == 0 and (y1 == h or y1 % 32 == 0)
        out = oracle.cnn_forward(np.ascontiguousarray(x[b:b + 1, y0:y1, x0:x1, :]), wts, strides)
        assert np.array_equal(out[0, ly, lx], full[b, oy, ox]), (b, oy, ox)
    # a window one stride unit short on one side misses part of the receptive field
    y0, y1, x0, x1, ly, lx = cnn_patch_for(2, 2, h, w, reach=1)
    out = oracle.cnn_forward(np.ascontiguousarray(x[0:1, y0:y1, x0:x1, :]), wts, strides)
    assert not np.array_equal(out[0, ly, lx], full[0, 2, 2])
