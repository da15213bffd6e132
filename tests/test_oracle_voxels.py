"""Pins of the oracle's voxel reordering and view-frustum filtering of voxels (Sec. 4.2.2,
frustum-based dynamic loading: primitives are reordered offline into a voxel grid and the
voxels, not the primitives, are filtered against the view frustum).  What fixes it: the
definition of the index (checked by a plain Python loop), and the requirement that
filtering is invisible in the result -- a skipped voxel may only hold primitives that the
per-primitive culling would have removed anyway, so images, lists and counts do not change."""
import math

import numpy as np
import pytest

from oracle import ref
from paper_2503_21364_amd import scenes


def _morton(ix, iy, iz):
    k = 0
    for b in range(21):
        k |= ((ix >> b) & 1) << (3 * b) | ((iy >> b) & 1) << (3 * b + 1) | ((iz >> b) & 1) << (3 * b + 2)
    return k


def test_index_is_the_definition_on_a_small_scene():
    sc = scenes.make_scene(2, n=3000, seed=5)
    size = 3.0
    idx = ref.build_voxel_index(sc, size)
    n = sc["n"]
    assert np.array_equal(np.sort(idx.perm), np.arange(n))
    assert idx.first[0] == 0 and idx.first[-1] == n and np.all(np.diff(idx.first.astype(np.int64)) > 0)
    # plain loop: cell, Morton key, expected order = (key, original index)
    cells = [tuple(int(math.floor(np.float32(sc["mean"][a, i]) / np.float32(size))) for a in range(3)) for i in range(n)]
    mins = [min(c[a] for c in cells) for a in range(3)]
    keys = [_morton(c[0] - mins[0], c[1] - mins[1], c[2] - mins[2]) for c in cells]
    expect = sorted(range(n), key=lambda i: (keys[i], i))
    assert expect == idx.perm.tolist()
    # voxels = runs of equal key; boxes and smax are the extremes over the run
    for v in range(idx.num_voxels):
        a, b = int(idx.first[v]), int(idx.first[v + 1])
        members = idx.perm[a:b]
        assert len({keys[i] for i in members}) == 1
        assert v == 0 or keys[idx.perm[a]] > keys[idx.perm[a - 1]]
        m = sc["mean"][:, members]
        np.testing.assert_array_equal(idx.box_lo[v], m.min(axis=1))
        np.testing.assert_array_equal(idx.box_hi[v], m.max(axis=1))
        assert idx.smax[v] == sc["scale"][:, members].max()


def test_reordering_keeps_every_primitive_intact():
    sc = scenes.make_scene(0, n=500, seed=9)
    idx = ref.build_voxel_index(sc, 0.5)
    sc2 = ref.reorder_scene(sc, idx.perm)
    for k in ("mean", "scale", "rot", "sh"):
        np.testing.assert_array_equal(sc2[k][..., 7], sc[k][..., idx.perm[7]])
    np.testing.assert_array_equal(sc2["opacity"], sc["opacity"][idx.perm])


def _cam(w=640, h=360, eye=(0, 0, -10), target=(0, 0, 0), fov=50.0):
    return scenes.make_camera(scenes.look_at(eye, target, (0, -1, 0)), eye, w, h, fov)


def test_visibility_closed_cases():
    cam = _cam()
    box = lambda c, r: (np.array(c, np.float32) - r, np.array(c, np.float32) + r)
    # in front of the camera on the optical axis: visible; mirrored behind it: not
    assert ref.voxel_visible(cam, *box((0, 0, 0), 0.5), 0.05)
    assert not ref.voxel_visible(cam, *box((0, 0, -20), 0.5), 0.05)
    # straddling the near plane counts as visible
    assert ref.voxel_visible(cam, *box((0, 0, -9.9), 0.5), 0.05)
    # far off to one side: the half-frustum at depth 10 is 10 * tan(25 deg) * 16/9 = 8.3 wide
    assert not ref.voxel_visible(cam, *box((40, 0, 0), 0.5), 0.05)
    assert not ref.voxel_visible(cam, *box((-40, 0, 0), 0.5), 0.05)
    assert not ref.voxel_visible(cam, *box((0, 30, 0), 0.5), 0.05)
    assert not ref.voxel_visible(cam, *box((0, -30, 0), 0.5), 0.05)
    # ... unless its splats are large enough to reach into the image: support radius ~ 3.33 * 1.3.. * smax
    assert ref.voxel_visible(cam, *box((40, 0, 0), 0.5), 8.0)
    # a box that spans the frustum although all its corners are outside
    assert ref.voxel_visible(cam, np.array([-50, -50, -1], np.float32), np.array([50, 50, 1], np.float32), 0.01)


def test_single_primitive_sweep_across_every_image_edge():
    """One primitive = one voxel.  Wherever the primitive is binned the voxel must be visible,
    and the filter must not be vacuous: well outside the image it must say no."""
    cam = _cam(320, 200)
    for axis, sign in ((0, 1), (0, -1), (1, 1), (1, -1)):
        seen_invisible = False
        for scale in (0.01, 0.2, 1.5):
            for d in np.linspace(0.0, 40.0, 401):
                pos = np.zeros(3); pos[axis] = sign * d
                sc = scenes.hand_placed_scene(pos[None, :], [(scale, scale * 0.3, scale * 0.6)], opacity=0.9,
                                              sh_dc=np.array([[0.5, 0.5, 0.5]]))
                pre = ref.preprocess(sc, cam)
                idx = ref.build_voxel_index(sc, 1.0)
                vis = bool(ref.voxels_visible(idx, cam)[0])
                if pre.tiles_touched[0] > 0:
                    assert vis, (axis, sign, scale, d)
                seen_invisible |= not vis
        assert seen_invisible


@pytest.mark.parametrize("cfg,n,voxel,mul,view", [
    (2, 60_000, 2.0, 1.0, 4), (2, 60_000, 2.0, 1.0, 5), (2, 60_000, 4.0, 8.0, 7), (2, 60_000, 1.0, 30.0, 6),
    (3, 200_000, 50.0, 1.0, 0), (3, 200_000, 25.0, 10.0, 1), (1, 30_000, 1.0, 3.0, 2), (0, 5_000, 0.25, 20.0, 0),
])
def test_filter_never_hides_a_binned_primitive(cfg, n, voxel, mul, view):
    sc = scenes.make_scene(cfg, n=n, seed=100 + cfg)
    sc["scale"] = sc["scale"] * np.float32(mul)
    idx = ref.build_voxel_index(sc, voxel)
    sc2 = ref.reorder_scene(sc, idx.perm)
    cam = scenes.make_cameras(cfg)[view]
    vis = ref.voxels_visible(idx, cam)
    mask = ref.primitives_in_visible_voxels(idx, vis)
    pre = ref.preprocess(sc2, cam)
    assert not np.any((pre.tiles_touched > 0) & ~mask)
    if cfg in (2, 3) and mul == 1.0:
        assert mask.mean() < 0.7          # and it does remove a good part of the scene


def test_a_planted_mistake_is_caught():
    # without the splat reach (smax = 0) large splats centred outside the frustum get hidden
    sc = scenes.make_scene(2, n=60_000, seed=102)
    sc["scale"] = sc["scale"] * np.float32(30.0)
    idx = ref.build_voxel_index(sc, 1.0)
    sc2 = ref.reorder_scene(sc, idx.perm)
    cam = scenes.make_cameras(2)[6]
    wrong = ref.build_voxel_index(sc, 1.0); wrong.smax[:] = 0
    mask = ref.primitives_in_visible_voxels(wrong, ref.voxels_visible(wrong, cam))
    pre = ref.preprocess(sc2, cam)
    assert np.any((pre.tiles_touched > 0) & ~mask)


def test_removing_the_hidden_voxels_leaves_the_frame_unchanged():
    sc = scenes.make_scene(2, n=40_000, seed=103)
    sc["scale"] = sc["scale"] * np.float32(3.0)
    idx = ref.build_voxel_index(sc, 2.0)
    sc2 = ref.reorder_scene(sc, idx.perm)
    cam = dict(scenes.make_cameras(2, 320, 180)[5], binning=1)
    cam["bg"] = np.array([0.2, 0.3, 0.1], np.float32)
    mask = ref.primitives_in_visible_voxels(idx, ref.voxels_visible(idx, cam))
    assert 0.02 < mask.mean() < 0.6
    kept = np.flatnonzero(mask)
    sub = dict(sc2, n=len(kept), mean=np.ascontiguousarray(sc2["mean"][:, kept]),
               scale=np.ascontiguousarray(sc2["scale"][:, kept]), rot=np.ascontiguousarray(sc2["rot"][:, kept]),
               opacity=np.ascontiguousarray(sc2["opacity"][kept]), sh=np.ascontiguousarray(sc2["sh"][..., kept]))
    full, part = ref.render_frame(sc2, cam), ref.render_frame(sub, cam)
    assert np.array_equal(full.img.rgb, part.img.rgb) and np.array_equal(full.img.T, part.img.T)
    assert full.binned.D == part.binned.D
    np.testing.assert_array_equal(full.binned.keys, part.binned.keys)
    np.testing.assert_array_equal(full.binned.vals, kept[part.binned.vals].astype(np.uint32))
