"""Pins of the oracle's gradient through the compositing of Eq. 9-10 (Sec. 2.2: the rasteriser is
differentiable and the primitives' parameters are optimised through it).  What fixes it, other than
itself: central differences of the forward oracle (a separate function with pins of its own), closed
forms for one and two splats, and the partition of unity of the compositing weights."""
import copy
import math

import numpy as np
import pytest

from oracle import ref
from paper_2503_21364_amd import scenes


def _cam(w=64, h=48, bg=(0.1, 0.2, 0.3)):
    cam = scenes.make_cameras(0, w, h)[0]
    cam = dict(cam)
    cam["bg"] = np.array(bg, np.float32)
    return cam


def _frame(n=300, seed=3, w=64, h=48, scale_mul=3.0):
    sc = scenes.make_scene(0, n=n, seed=seed)
    sc["scale"] = sc["scale"] * np.float32(scale_mul)
    cam = _cam(w, h)
    pre = ref.preprocess(sc, cam)
    b = ref.bin_sort(pre, cam)
    return sc, cam, pre, b


def _loss(pre, b, cam, Gc, GT):
    """The loss, and the per-pixel decision counts (a finite difference is only meaningful when the
    two evaluations took the same decisions at every pixel)."""
    img = ref.render(pre, b, cam)
    return float((Gc * img.rgb).sum() + (GT * img.T).sum()), (img.E.copy(), img.C.copy())


def test_forward_walk_of_the_backward_is_the_forward_oracle():
    sc, cam, pre, b = _frame()
    H, W = cam["height"], cam["width"]
    g = ref.render_backward(pre, b, cam, np.zeros((3, H, W)), np.zeros((H, W)))
    img = ref.render(pre, b, cam)
    assert np.array_equal(g.img_rgb, img.rgb) and np.array_equal(g.img_T, img.T)
    for a in (g.mean2d, g.conic, g.opacity, g.rgb):
        assert not a.any()                        # zero loss gradient in, zero out


@pytest.mark.parametrize("seed", [3, 4])
def test_against_central_differences_of_the_forward_oracle(seed):
    sc, cam, pre, b = _frame(seed=seed)
    H, W = cam["height"], cam["width"]
    rng = np.random.default_rng(seed)
    Gc = rng.normal(size=(3, H, W))
    GT = rng.normal(size=(H, W))
    g = ref.render_backward(pre, b, cam, Gc, GT)
    assert g.amb.sum() == 0                       # no decision sits on a threshold in this frame
    # the primitives with the largest gradients, each attribute perturbed by a representable step
    score = np.abs(g.opacity) + np.abs(g.mean2d).sum(0)
    picks = np.argsort(-score)[:6]
    checked = 0
    for i in picks:
        for name, row, analytic, rel_step in (
                ("mean2d", 0, g.mean2d[0, i], None), ("mean2d", 1, g.mean2d[1, i], None),
                ("conic", 0, g.conic[0, i], 2.0 ** -11), ("conic", 1, g.conic[1, i], 2.0 ** -11),
                ("conic", 2, g.conic[2, i], 2.0 ** -11), ("opacity", None, g.opacity[i], 2.0 ** -11),
                ("rgb", 0, g.rgb[0, i], 2.0 ** -6), ("rgb", 2, g.rgb[2, i], 2.0 ** -6)):
            lo, hi = copy.deepcopy(pre), copy.deepcopy(pre)
            arr_lo, arr_hi = getattr(lo, name), getattr(hi, name)
            idx = (i,) if row is None else (row, i)
            x = arr_lo[idx]
            step = type(x)(2.0 ** -11) if rel_step is None else type(x)(max(abs(float(x)), 1e-3) * rel_step)
            arr_lo[idx] = x - step
            arr_hi[idx] = x + step
            den = float(arr_hi[idx]) - float(arr_lo[idx])
            (l_hi, d_hi), (l_lo, d_lo) = _loss(hi, b, cam, Gc, GT), _loss(lo, b, cam, Gc, GT)
            if not (np.array_equal(d_hi[0], d_lo[0]) and np.array_equal(d_hi[1], d_lo[1])):
                continue                          # a threshold was crossed between the two evaluations
            fd = (l_hi - l_lo) / den
            scale = max(abs(fd), abs(analytic), 1e-3)
            assert abs(fd - analytic) <= 1e-4 * scale, (i, name, row, fd, analytic)
            checked += 1
    assert checked >= 40


def _one_splat(o=0.6, c=(0.9, 0.5, 0.2), at=(20.3, 17.8), conic=(0.02, 0.005, 0.03), n_pad=0):
    """A hand-made projected frame: one primitive, its list in every tile."""
    cam = _cam(32, 32)
    n = 1 + n_pad
    pre = ref.preprocess(scenes.make_scene(0, n=n, seed=1), cam)     # shapes and dtypes, then overwritten
    pre.mean2d[:, 0] = at
    pre.conic[:, 0] = conic
    pre.opacity[0] = o
    pre.rgb[:, 0] = c
    vals = np.zeros(4, np.uint32)
    b = type(pre)(D=4, vals=vals, tile_offsets=np.arange(5, dtype=np.uint64))
    return cam, pre, b


def test_single_splat_closed_form():
    o, c, at, conic = 0.6, np.array([0.9, 0.5, 0.2]), (20.3, 17.8), (0.02, 0.005, 0.03)
    cam, pre, b = _one_splat(o, c, at, conic)
    H = W = 32
    # the loss reads one pixel only
    px, py = 23, 15
    Gc = np.zeros((3, H, W)); GT = np.zeros((H, W))
    Gc[:, py, px] = (1.0, -2.0, 0.5); GT[py, px] = 0.7
    g = ref.render_backward(pre, b, cam, Gc, GT)
    o32 = float(np.float32(o))
    A, B, Cc = (float(np.float32(v)) for v in conic)
    dx, dy = float(np.float32(at[0])) - (px + 0.5), float(np.float32(at[1])) - (py + 0.5)
    q = A * dx * dx + 2 * B * dx * dy + Cc * dy * dy
    G = math.exp(-0.5 * q)
    alpha = o32 * G
    bg = cam["bg"].astype(np.float64)
    gc = Gc[:, py, px]
    # C = c alpha + bg (1 - alpha), T_end = 1 - alpha
    dLda = float(gc @ (c - bg)) - GT[py, px]
    np.testing.assert_allclose(g.rgb[:, 0], alpha * gc, rtol=1e-12)
    np.testing.assert_allclose(g.opacity[0], dLda * G, rtol=1e-12)
    dLdq = dLda * (-0.5 * alpha)
    np.testing.assert_allclose(g.conic[:, 0], [dLdq * dx * dx, dLdq * 2 * dx * dy, dLdq * dy * dy], rtol=1e-12)
    np.testing.assert_allclose(g.mean2d[:, 0], [dLdq * 2 * (A * dx + B * dy), dLdq * 2 * (B * dx + Cc * dy)], rtol=1e-12)


def test_clamped_alpha_and_skipped_entries_get_no_shape_gradient():
    # opacity 1 at the centre pixel: alpha is clamped to 0.99 there, so only the colour has a gradient
    cam, pre, b = _one_splat(o=1.0, at=(20.5, 17.5), conic=(1e-4, 0.0, 1e-4))
    H = W = 32
    Gc = np.zeros((3, H, W)); Gc[:, 17, 20] = 1.0
    g = ref.render_backward(pre, b, cam, Gc, None)
    np.testing.assert_allclose(g.rgb[:, 0], 0.99, rtol=1e-6)
    assert g.opacity[0] == 0.0 and not g.conic[:, 0].any() and not g.mean2d[:, 0].any()
    # far away from a small splat alpha < 1/255: nothing at all
    cam, pre, b = _one_splat(o=0.9, at=(4.5, 4.5), conic=(0.5, 0.0, 0.5))
    Gc = np.zeros((3, H, W)); Gc[:, 20, 20] = 1.0
    GT = np.zeros((H, W)); GT[20, 20] = 1.0
    g = ref.render_backward(pre, b, cam, Gc, GT)
    assert not g.rgb.any() and g.opacity[0] == 0.0 and not g.conic.any() and not g.mean2d.any()


def test_weights_and_final_transmittance_sum_to_one():
    """dC/dc_i = w_i and sum_i w_i + T_end = 1 at every pixel: with dL/dC = 1 on one channel the
    colour gradients of that channel add up to (number of pixels) - sum of T_end."""
    sc, cam, pre, b = _frame(n=800, seed=11, scale_mul=4.0)
    H, W = cam["height"], cam["width"]
    Gc = np.zeros((3, H, W)); Gc[1] = 1.0
    g = ref.render_backward(pre, b, cam, Gc, None)
    img = ref.render(pre, b, cam)
    assert abs(g.rgb[1].sum() + img.T.sum() - H * W) < 1e-9 * H * W
    assert not g.rgb[0].any() and not g.rgb[2].any()
    # and T_end alone: d(sum T_end)/d(opacity) is never positive
    g2 = ref.render_backward(pre, b, cam, np.zeros((3, H, W)), np.ones((H, W)))
    assert (g2.opacity <= 1e-15).all() and (g2.opacity < 0).any()


def test_two_splats_order_matters_as_in_the_closed_form():
    """Front splat a, back splat b at one pixel: C = c_a a + c_b b (1 - a) + bg (1 - a)(1 - b)."""
    cam = _cam(16, 16, bg=(0.0, 0.0, 0.0))
    pre = ref.preprocess(scenes.make_scene(0, n=2, seed=1), cam)
    pre.mean2d[:, 0] = (8.5, 8.5); pre.mean2d[:, 1] = (8.5, 8.5)
    pre.conic[:, 0] = (0.01, 0.0, 0.01); pre.conic[:, 1] = (0.01, 0.0, 0.01)
    pre.opacity[:] = (0.5, 0.8)
    pre.rgb[:, 0] = (1.0, 0.0, 0.0); pre.rgb[:, 1] = (0.0, 1.0, 0.0)
    b = type(pre)(D=2, vals=np.array([0, 1], np.uint32), tile_offsets=np.array([0, 2], np.uint64))
    Gc = np.zeros((3, 16, 16)); Gc[:, 8, 8] = (1.0, 1.0, 1.0)
    g = ref.render_backward(pre, b, cam, Gc, None)
    a, bb = 0.5, float(np.float32(0.8))
    # dL/da = c_a - c_b b = 1 - b (summed over channels: 1*1 - 1*b); dL/db = (1 - a)
    np.testing.assert_allclose(g.opacity, [1.0 - bb, 1.0 - a], rtol=1e-12)
    np.testing.assert_allclose(g.rgb[:, 0], [a, a, a], rtol=1e-12)
    np.testing.assert_allclose(g.rgb[:, 1], [bb * (1 - a)] * 3, rtol=1e-12)


def test_magnitude_sums_bound_the_gradients():
    sc, cam, pre, b = _frame(n=500, seed=5)
    H, W = cam["height"], cam["width"]
    rng = np.random.default_rng(5)
    g = ref.render_backward(pre, b, cam, rng.normal(size=(3, H, W)), rng.normal(size=(H, W)))
    signed = np.concatenate([g.mean2d, g.conic, g.opacity[None, :], g.rgb])
    assert signed.shape == g.abs.shape
    assert (np.abs(signed) <= g.abs * (1 + 1e-12) + 1e-300).all()
    assert (g.abs[:, np.abs(signed).sum(0) > 0] > 0).any()


# ---------------------------------------------------------------- the chain through the projection
def _proj_loss(sc, cam, wts, i):
    """sum of weights x (u, v, A, B, C, o, r, g, b) of primitive i, from the forward oracle; None
    when the primitive is not binned."""
    pre = ref.preprocess(sc, cam)
    if pre.stage[i] != ref.VISIBLE:
        return None
    vals = np.array([pre.mean2d[0, i], pre.mean2d[1, i], pre.conic[0, i], pre.conic[1, i], pre.conic[2, i],
                     pre.opacity[i], pre.rgb[0, i], pre.rgb[1, i], pre.rgb[2, i]], dtype=np.float64)
    return float(wts @ vals)


@pytest.mark.parametrize("seed,guard", [(31, False), (32, False), (33, True)])
def test_projection_gradient_against_central_differences(seed, guard):
    """The forward oracle evaluates u, v and the conic in fp32, so a central difference with a
    relative step of 2^-9 carries a noise of about 1e-4 of the values; a wrong or missing term is of
    order one."""
    n = 24
    sc = scenes.make_scene(0, n=n, seed=seed)
    sc["scale"] = sc["scale"] * np.float32(3.0)
    cam = dict(scenes.make_cameras(0, 256, 256)[0])
    if guard:
        # far off to the side, large enough to stay binned: the guard-band clamp of the Jacobian is active
        sc["mean"][0] = np.float32(6.0) + sc["mean"][0]
        sc["scale"] = sc["scale"] * np.float32(40.0)
    pre = ref.preprocess(sc, cam)
    vis = np.flatnonzero(pre.stage == ref.VISIBLE)
    assert len(vis) >= 5
    if guard:
        lim = 1.3 * 0.5 * cam["width"] / cam["fx"]
        V = np.asarray(cam["view"], np.float64).reshape(3, 4)
        pc = V[:, :3] @ sc["mean"].astype(np.float64) + V[:, 3:4]
        assert (np.abs(pc[0, vis] / pc[2, vis]) > lim).any()
    rng = np.random.default_rng(seed)
    W = rng.normal(size=(9, n))
    W[2:5] *= 1e-2                              # conic entries are large for small splats: keep the terms comparable
    g = ref.preprocess_backward(sc, cam, pre, W)
    checked = 0
    for i in vis[:5]:
        for name, rows in (("mean", 3), ("scale", 3), ("rot", 4), ("opacity", 0)):
            for r in range(max(rows, 1)):
                idx = (i,) if rows == 0 else (r, i)
                lo, hi = {k: (v.copy() if isinstance(v, np.ndarray) else v) for k, v in sc.items()}, \
                         {k: (v.copy() if isinstance(v, np.ndarray) else v) for k, v in sc.items()}
                x = sc[name][idx]
                step = np.float32(max(abs(float(x)), 0.05) * 2.0 ** -9)
                lo[name][idx] = x - step; hi[name][idx] = x + step
                den = float(hi[name][idx]) - float(lo[name][idx])
                l_hi, l_lo = _proj_loss(hi, cam, W[:, i], i), _proj_loss(lo, cam, W[:, i], i)
                assert l_hi is not None and l_lo is not None
                fd = (l_hi - l_lo) / den
                analytic = getattr(g, name)[idx]
                scale_ = max(abs(fd), abs(analytic), 1e-6)
                # noise floor of the fp32 forward values under this step
                terms = np.abs(W[:, i] * np.array([pre.mean2d[0, i], pre.mean2d[1, i], pre.conic[0, i], pre.conic[1, i],
                                                   pre.conic[2, i], pre.opacity[i], 0, 0, 0]))
                noise = 4 * 2.0 ** -24 * terms.sum() / den
                assert abs(fd - analytic) <= 2e-3 * scale_ + noise, (i, name, r, fd, analytic, noise)
                checked += 1
    assert checked == 5 * 11
    # SH coefficients: the colour is linear in them (fp64 in the forward oracle)
    i = int(vis[0])
    for k in (0, 3, 8, 15):
        for ch in range(3):
            lo = dict(sc, sh=sc["sh"].copy()); hi = dict(sc, sh=sc["sh"].copy())
            lo["sh"][k, ch, i] -= np.float32(2.0 ** -6); hi["sh"][k, ch, i] += np.float32(2.0 ** -6)
            den = float(hi["sh"][k, ch, i]) - float(lo["sh"][k, ch, i])
            fd = (_proj_loss(hi, cam, W[:, i], i) - _proj_loss(lo, cam, W[:, i], i)) / den
            assert abs(fd - g.sh[k, ch, i]) <= 1e-6 * max(abs(fd), 1e-3), (k, ch, fd, g.sh[k, ch, i])


def test_projection_gradient_special_cases():
    sc = scenes.make_scene(0, n=40, seed=35)
    cam = scenes.make_cameras(0, 128, 128)[0]
    pre = ref.preprocess(sc, cam)
    W = np.random.default_rng(1).normal(size=(9, 40))
    g = ref.preprocess_backward(sc, cam, pre, W)
    hidden = pre.stage != ref.VISIBLE
    # a primitive that was not binned gets nothing
    sc2 = dict(sc, mean=sc["mean"].copy()); sc2["mean"][2, :5] += 100.0
    pre2 = ref.preprocess(sc2, cam)
    g2 = ref.preprocess_backward(sc2, cam, pre2, W)
    assert (pre2.stage[:5] != ref.VISIBLE).all()
    for arr in (g2.mean, g2.scale, g2.rot):
        assert not arr[:, :5].any()
    assert not g2.opacity[:5].any() and not g2.sh[:, :, :5].any()
    assert not g.mean[:, hidden].any()
    # opacity passes straight through; the quaternion gradient is orthogonal to the quaternion
    # (the covariance does not depend on its norm); scaling all three scales by t scales Sigma by t^2
    vis = ~hidden
    np.testing.assert_array_equal(g.opacity[vis], W[5, vis])
    dots = (g.rot * sc["rot"].astype(np.float64)).sum(0)
    assert np.abs(dots[vis]).max() <= 1e-9 * np.abs(g.rot[:, vis]).max()
    # only the DC coefficient: the colour does not depend on the direction, so the mean gets
    # nothing from the colour -- drop the colour weights and the mean gradient must not change
    W0 = W.copy(); W0[6:] = 0.0
    sc3 = dict(sc, sh=sc["sh"].copy()); sc3["sh"][1:] = 0.0
    pre3 = ref.preprocess(sc3, cam)
    g3a = ref.preprocess_backward(sc3, cam, pre3, W)
    g3b = ref.preprocess_backward(sc3, cam, pre3, W0)
    np.testing.assert_allclose(g3a.mean, g3b.mean, rtol=0, atol=1e-12 * np.abs(g3a.mean).max())
