"""Pins for the oracle's textual density (Eq. 8, Appendix B)."""
import numpy as np
import pytest

from oracle import rtprune_oracle as orc


def _gray_rgb(g):
    return np.repeat(np.asarray(g, dtype=np.uint8)[..., None], 3, axis=2)


def test_gray_weights_are_bt601_and_sum_to_one():
    assert orc.GRAY_MILLI == (299, 587, 114) and sum(orc.GRAY_MILLI) == 1000
    px = np.array([[[255, 0, 0], [0, 255, 0], [0, 0, 255], [255, 255, 255], [10, 20, 30]]], dtype=np.uint8)
    g = orc.gray_milli(px)[0] / 255000.0
    np.testing.assert_allclose(g[:4], [0.299, 0.587, 0.114, 1.0], atol=1e-15)
    assert abs(g[4] - (0.299 * 10 + 0.587 * 20 + 0.114 * 30) / 255) < 1e-15


def test_sobel_equals_library_sobel_with_nearest_border():
    nd = pytest.importorskip("scipy.ndimage")
    rng = np.random.default_rng(30)
    gray = rng.integers(0, 255001, size=(37, 53)).astype(np.int64)
    gx, gy = orc.sobel_xy(gray)
    np.testing.assert_array_equal(gx, nd.sobel(gray.astype(np.float64), axis=1, mode="nearest"))
    # the printed G_y kernel has its positive row on top: minus the library's orientation
    np.testing.assert_array_equal(gy, -nd.sobel(gray.astype(np.float64), axis=0, mode="nearest"))


def test_sobel_equals_true_2d_convolution_in_the_interior():
    sig = pytest.importorskip("scipy.signal")
    rng = np.random.default_rng(31)
    gray = rng.integers(0, 1000, size=(20, 24)).astype(np.int64)
    kx = np.array([[-1, 0, 1], [-2, 0, 2], [-1, 0, 1]])
    ky = np.array([[1, 2, 1], [0, 0, 0], [-1, -2, -1]])
    gx, gy = orc.sobel_xy(gray)
    cx = sig.convolve2d(gray, kx, mode="valid")       # true convolution flips the kernel
    cy = sig.convolve2d(gray, ky, mode="valid")
    np.testing.assert_array_equal(np.abs(gx[1:-1, 1:-1]), np.abs(cx))
    np.testing.assert_array_equal(np.abs(gy[1:-1, 1:-1]), np.abs(cy))
    np.testing.assert_array_equal(gx[1:-1, 1:-1] ** 2 + gy[1:-1, 1:-1] ** 2, cx ** 2 + cy ** 2)


def test_constant_image_has_no_edges():
    img = _gray_rgb(np.full((64, 64), 200))
    rho, rho_k = orc.text_density(img, 16, 16, 0.2)
    assert rho == 0.0 and (rho_k == 0).all() and rho_k.shape == (16,)


def test_vertical_step_edge_hand_count():
    # left half 0, right half v: G_x = 4 v / 255 on the two columns next to the step, 0 elsewhere
    v = 100
    g = np.zeros((32, 32), dtype=np.uint8)
    g[:, 16:] = v
    e = orc.edge_map(_gray_rgb(g), 0.2)
    assert 4 * v / 255 >= 0.2
    assert e[:, 15].all() and e[:, 16].all() and e.sum() == 2 * 32
    rho, rho_k = orc.text_density(_gray_rgb(g), 16, 16, 0.2)
    assert rho == np.float32(64 / 1024)
    np.testing.assert_array_equal(rho_k.reshape(2, 2), np.float32([[1 / 16, 1 / 16], [1 / 16, 1 / 16]]))
    # a step too small for the threshold: 4 v / 255 < tau
    g[:, 16:] = 12
    assert 4 * 12 / 255 < 0.2 and not orc.edge_map(_gray_rgb(g), 0.2).any()


def test_single_bright_pixel_hand_values():
    # around an isolated pixel of value v the magnitudes are 2v (4-neighbours), sqrt(2) v (diagonals), 0 (centre)
    for v, tau, want in ((255, 0.2, 8), (30, 0.2, 4), (30, 0.17, 4), (30, 0.16, 8), (20, 0.2, 0)):
        g = np.zeros((9, 9), dtype=np.uint8)
        g[4, 4] = v
        e = orc.edge_map(_gray_rgb(g), tau)
        assert e.sum() == want, (v, tau, e.sum())
        assert not e[4, 4]
        if want == 4:
            assert e[3, 4] and e[5, 4] and e[4, 3] and e[4, 5]


def test_threshold_is_inclusive_and_monotone():
    g = np.zeros((8, 8), dtype=np.uint8)
    g[:, 4:] = 255                                 # step of 1.0: G = 4.0 exactly on two columns
    assert orc.edge_map(_gray_rgb(g), 4.0).sum() == 16                      # G >= tau holds with equality
    assert orc.edge_map(_gray_rgb(g), np.nextafter(np.float32(4.0), np.float32(5))).sum() == 0
    rng = np.random.default_rng(32)
    img = rng.integers(0, 256, size=(64, 64, 3)).astype(np.uint8)
    rhos = [float(orc.text_density(img, 8, 8, t)[0]) for t in (0.05, 0.1, 0.2, 0.3, 0.5, 1.0, 3.0)]
    assert all(a >= b for a, b in zip(rhos, rhos[1:])) and rhos[0] > rhos[-1]


def test_density_is_the_average_of_the_patch_densities_and_invariant_to_flips():
    rng = np.random.default_rng(33)
    img = (rng.integers(0, 2, size=(96, 128, 1)) * rng.integers(0, 256, size=(96, 128, 3))).astype(np.uint8)
    rho, rho_k = orc.text_density(img, 32, 32, 0.2)
    assert rho_k.shape == (12,)
    assert abs(float(rho) - float(np.mean(rho_k.astype(np.float64)))) < 1e-7
    rho_f, rho_kf = orc.text_density(img[::-1, ::-1].copy(), 32, 32, 0.2)
    assert rho_f == rho
    np.testing.assert_array_equal(rho_kf.reshape(3, 4), rho_k.reshape(3, 4)[::-1, ::-1])
    # colour only matters through the BT.601 luma: swapping channels of a grey image changes nothing
    grey = _gray_rgb(rng.integers(0, 256, size=(32, 32)))
    assert orc.text_density(grey, 16, 16, 0.2)[0] == orc.text_density(grey[..., ::-1].copy(), 16, 16, 0.2)[0]
