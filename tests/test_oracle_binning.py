"""Pins of the oracle's binning rule 1 (a tile of the support rectangle is kept
only if the splat can reach alpha >= 1/255 on the square of the tile's pixel
centres; Sec. 4.2.1, "intersection operations for each tile").  What fixes it:
the mathematics of the ellipse/square intersection (checked by dense sampling),
and the definition of the image (rule 1 may only drop pairs that can never
contribute, so the image must not change)."""
import math

import numpy as np
import pytest

from oracle import ref
from paper_2503_21364_amd import scenes


def test_tau_bounds_the_contribution_threshold_from_above_and_tightly():
    os_ = np.concatenate([np.linspace(1 / 255, 1.0, 4000), 2.0 ** -np.arange(0, 8.0, 0.125)])
    os_ = os_[(os_ >= 1 / 255) & (os_ <= 1.0)].astype(np.float32)
    for o in os_:
        tau = ref.opacity_tau(o)
        exact = 2 * math.log(255.0 * float(o))
        assert tau >= exact + 0.005, (o, tau, exact)
        assert tau <= exact + 0.26, (o, tau, exact)
    assert ref.opacity_tau(1.0) <= 2 * math.log(255 * 1.125) + 0.011


def _random_conic(rng):
    th = rng.uniform(0, math.pi)
    s1, s2 = np.exp(rng.uniform(math.log(0.6), math.log(60.0), 2))
    R = np.array([[math.cos(th), -math.sin(th)], [math.sin(th), math.cos(th)]])
    S = R @ np.diag([s1 * s1, s2 * s2]) @ R.T
    Ci = np.linalg.inv(S)
    return np.float32(Ci[0, 0]), np.float32(Ci[0, 1]), np.float32(Ci[1, 1])


def test_tile_test_matches_dense_sampling_of_the_square():
    rng = np.random.default_rng(7)
    g = np.linspace(0.5, 15.5, 241)
    xs, ys = np.meshgrid(g, g)
    decided = 0
    for _ in range(3000):
        A, B, Cc = _random_conic(rng)
        o = np.float32(rng.uniform(1 / 255, 1.0))
        u, v = np.float32(rng.uniform(-60, 80)), np.float32(rng.uniform(-60, 80))
        tx, ty = int(rng.integers(0, 3)), int(rng.integers(0, 3))
        dx = float(u) - (xs + 16 * tx); dy = float(v) - (ys + 16 * ty)
        q = float(A) * dx * dx + 2 * float(B) * dx * dy + float(Cc) * dy * dy
        qmin = q.min()
        tau = ref.opacity_tau(o)
        kept = ref.tile_kept(u, v, A, B, Cc, o, tx, ty)
        # grid minimum is an upper bound of the true minimum, and close to it
        slack = 0.02 * max(1.0, qmin)
        if qmin <= tau * (1 - 1e-4):
            assert kept, (u, v, A, B, Cc, o, tx, ty, qmin, tau)
            decided += 1
        elif qmin > tau + slack + 0.3:
            assert not kept, (u, v, A, B, Cc, o, tx, ty, qmin, tau)
            decided += 1
    assert decided > 2500


def test_centre_inside_the_square_is_always_kept():
    for (u, v) in [(8.0, 8.0), (0.6, 15.4), (15.5, 0.5)]:
        assert ref.tile_kept(u, v, 3.3, 0.0, 3.3, 1 / 255, 0, 0)
    # just outside with a tiny splat of threshold opacity: nothing can reach alpha >= 1/255
    assert not ref.tile_kept(-3.0, 8.0, 3.3, 0.0, 3.3, 0.004, 0, 0)


@pytest.mark.parametrize("seed,n,w,h,mul", [(31, 1500, 64, 48, 2.0), (33, 3000, 130, 70, 1.0), (35, 400, 96, 96, 6.0)])
def test_rule1_never_drops_a_contributing_pair_and_leaves_the_image_unchanged(seed, n, w, h, mul):
    sc = scenes.make_scene(0, n=n, seed=seed)
    sc["scale"] *= np.float32(mul)
    cam0 = scenes.make_cameras(0, w, h)[0]
    cam0["bg"] = np.array([0.3, 0.1, 0.2], np.float32)
    cam1 = dict(cam0, binning=1)
    f0, f1 = ref.render_frame(sc, cam0), ref.render_frame(sc, cam1)
    assert f1.binned.D < f0.binned.D
    # identical per-primitive projection; fewer or equal tiles per primitive
    assert np.array_equal(f0.pre.rect[f1.pre.tiles_touched > 0], f1.pre.rect[f1.pre.tiles_touched > 0])
    assert np.all(f1.pre.tiles_touched <= f0.pre.tiles_touched)
    # every tile list of rule 1 is a sub-sequence of rule 0's, in the same order
    T = f0.binned.tiles_x * f0.binned.tiles_y
    for t in range(T):
        l0 = f0.binned.vals[int(f0.binned.tile_offsets[t]):int(f0.binned.tile_offsets[t + 1])]
        l1 = f1.binned.vals[int(f1.binned.tile_offsets[t]):int(f1.binned.tile_offsets[t + 1])]
        keep = np.isin(l0, l1)
        assert np.array_equal(l0[keep], l1) and len(l1) == keep.sum()
    # the image is the same, bit for bit; fewer entries are visited
    assert np.array_equal(f0.img.rgb, f1.img.rgb) and np.array_equal(f0.img.T, f1.img.T)
    assert np.array_equal(f0.img.C, f1.img.C)
    assert f1.img.E.sum() < f0.img.E.sum()
    # direct check of conservativeness: any pair with alpha >= 1/255 at some pixel of a tile is binned there
    pre = f1.pre
    ys, xs = np.mgrid[0:h, 0:w]
    tx_of, ty_of = xs // 16, ys // 16
    for gidx in np.nonzero(f0.pre.tiles_touched > 0)[0][:400]:
        dx = pre.mean2d[0, gidx].astype(np.float64) - (xs + 0.5)
        dy = pre.mean2d[1, gidx].astype(np.float64) - (ys + 0.5)
        A, B, Cc = pre.conic[:, gidx].astype(np.float64)
        alpha = float(pre.opacity[gidx]) * np.exp(-0.5 * (A * dx * dx + 2 * B * dx * dy + Cc * dy * dy))
        hit = alpha >= 1 / 255
        for t in np.unique((ty_of[hit] * f1.binned.tiles_x + tx_of[hit])):
            lst = f1.binned.vals[int(f1.binned.tile_offsets[t]):int(f1.binned.tile_offsets[t + 1])]
            assert gidx in lst


def test_rule1_pipeline_still_equals_brute_force():
    sc = scenes.make_scene(0, n=2000, seed=32)
    sc["scale"] *= np.float32(2.0)
    cam = dict(scenes.make_cameras(0, 50, 37)[0], binning=1)
    fr = ref.render_frame(sc, cam)
    ys, xs = np.mgrid[0:37, 0:50]
    br = ref.render_pixels_brute(fr.pre, cam, xs.ravel(), ys.ravel())
    assert np.array_equal(br.rgb.T.reshape(3, 37, 50), fr.img.rgb)
    assert np.array_equal(br.T.reshape(37, 50), fr.img.T)
    for (tx, ty) in [(0, 0), (2, 1), (3, 2)]:
        t = ty * fr.binned.tiles_x + tx
        sl = fr.binned.vals[int(fr.binned.tile_offsets[t]):int(fr.binned.tile_offsets[t + 1])]
        np.testing.assert_array_equal(sl, ref.tile_list(fr.pre, tx, ty, cam))


def test_rule1_statistics_on_config_shapes():
    # the reduction in pairs the rule buys on the benchmark distributions
    sc = scenes.make_scene(1, n=50_000)
    cam0 = scenes.make_cameras(1)[0]
    pre0 = ref.preprocess(sc, cam0)
    pre1 = ref.preprocess(sc, dict(cam0, binning=1))
    r = pre1.tiles_touched.sum() / pre0.tiles_touched.sum()
    assert 0.6 < r < 0.9


@pytest.mark.parametrize("binning", [0, 1])
def test_band_lists_and_band_render_are_the_frame_cut_into_tile_rows(binning):
    """The band-streaming functions (for frames too large to bin whole) against three other
    routes to the same thing: the whole-frame sort, the per-tile list from the definition, and
    the brute-force image."""
    sc = scenes.make_scene(0, n=4000, seed=61)
    sc["scale"] *= np.float32(2.5)
    W, H = 150, 101                                    # ragged in both directions: 10 x 7 tiles
    cam = dict(scenes.make_cameras(0, W, H)[0], binning=binning)
    fr = ref.render_frame(sc, cam)
    tx, ty = ref.tiles_xy(cam)
    order = ref.depth_order(fr.pre)
    total = 0
    for a, b in [(0, 2), (2, 3), (3, ty)]:
        band = ref.band_lists(fr.pre, cam, a, b, order)
        lo, hi = int(fr.binned.tile_offsets[a * tx]), int(fr.binned.tile_offsets[b * tx])
        np.testing.assert_array_equal(band.vals, fr.binned.vals[lo:hi])
        np.testing.assert_array_equal(band.offsets, fr.binned.tile_offsets[a * tx:b * tx + 1] - np.uint64(lo))
        total += band.vals.size
        # one tile of the band straight from the definition
        t = a * tx + 3
        np.testing.assert_array_equal(band.vals[int(band.offsets[3]):int(band.offsets[4])],
                                      ref.tile_list(fr.pre, 3, a, cam))
        img = ref.render_band(fr.pre, cam, band)
        assert (img.y0, img.y1) == (a * 16, min(b * 16, H))
        ys, xs = np.mgrid[img.y0:img.y1, 0:W]
        br = ref.render_pixels_brute(fr.pre, cam, xs.ravel(), ys.ravel(), order)
        assert np.array_equal(br.rgb.T.reshape(3, img.y1 - img.y0, W), img.rgb)
        assert np.array_equal(br.T.reshape(img.y1 - img.y0, W), img.T)
        assert np.array_equal(img.E, fr.img.E[img.y0:img.y1]) and np.array_equal(img.C, fr.img.C[img.y0:img.y1])
        assert np.array_equal(img.amb, fr.img.amb[img.y0:img.y1])
    assert total == fr.binned.D
