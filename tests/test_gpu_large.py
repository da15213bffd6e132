"""Config 4 at its full size (2 M primitives, 3840x2160, about 6e9 pairs, ~160 GB
of device buffers): too large for the oracle to bin whole, so the GPU result is
checked on what the oracle can compute piece by piece -- every per-primitive
output, the complete per-tile range table (from a 2-D difference array over the
oracle's rectangles), and, for sampled tiles, the exact sorted list and the
pixels composited from it."""
import numpy as np
import pytest
import torch

from oracle import ref
from paper_2503_21364_amd import binding as B
from paper_2503_21364_amd import scenes

import parity as P

pytestmark = pytest.mark.gpu


def _tile_counts_from_rects(pre, tx, ty):
    """Pairs per tile by definition: +1 over every primitive's rectangle."""
    diff = np.zeros((ty + 1, tx + 1), np.int64)
    r = pre.rect[pre.tiles_touched > 0].astype(np.int64)
    np.add.at(diff, (r[:, 1], r[:, 0]), 1)
    np.add.at(diff, (r[:, 1], r[:, 2]), -1)
    np.add.at(diff, (r[:, 3], r[:, 0]), -1)
    np.add.at(diff, (r[:, 3], r[:, 2]), 1)
    return diff.cumsum(axis=0).cumsum(axis=1)[:ty, :tx]


@pytest.mark.parametrize("binning", [0, 1])
def test_cfg4_full_size_sampled(binning):
    free, _ = torch.cuda.mem_get_info()
    if free < 180 * 2**30:
        pytest.skip(f"needs ~165 GB of free device memory, {free / 2**30:.0f} GB available")
    sc = scenes.make_scene(4)
    cam = dict(scenes.make_cameras(4)[0], binning=binning)
    W, H = int(cam["width"]), int(cam["height"])
    pre = ref.preprocess(sc, cam)
    D = int(pre.tiles_touched.astype(np.uint64).sum())
    assert D > (5_000_000_000 if binning == 0 else 2_000_000_000)
    print(f"[parity] cfg4 full, binning {binning}: D={D}", flush=True)

    dev = B.Scene(sc)
    fr = B.Frame(dev.n, W, H, D + 4096, want_offsets=False)
    B.render_frame(dev, B.make_camera(cam), fr)
    torch.cuda.synchronize()
    Dg, status = B.read_status(fr)
    assert status == B.OK and Dg == D

    P.compare_projected(fr, pre)

    tx, ty = fr.tiles_x, fr.tiles_y
    tile_offsets = P.to_np(fr.tile_offsets).view(np.uint64)
    assert tile_offsets[0] == 0 and tile_offsets[-1] == D
    assert np.all(np.diff(tile_offsets.astype(np.int64)) >= 0)
    if binning == 0:
        counts = _tile_counts_from_rects(pre, tx, ty).reshape(-1)
        expect_offsets = np.concatenate([[0], np.cumsum(counts)]).astype(np.uint64)
        np.testing.assert_array_equal(tile_offsets, expect_offsets)

    rng = np.random.default_rng(44)
    tiles = [(0, 0), (tx - 1, ty - 1), (tx // 2, ty // 2)] + \
            [(int(rng.integers(tx)), int(rng.integers(ty))) for _ in range(5)]
    worst = 0.0
    for (cx, cy) in tiles:
        t = cy * tx + cx
        lst = ref.tile_list(pre, cx, cy, cam)
        a, b = int(tile_offsets[t]), int(tile_offsets[t + 1])
        assert b - a == len(lst)
        np.testing.assert_array_equal(P.to_np(fr.vals[a:b]).view(np.uint32), lst, err_msg=f"tile {cx},{cy} values")
        keys = P.to_np(fr.keys[a:b]).view(np.uint64)
        expect_keys = (np.uint64(t) << np.uint64(32)) | pre.depth[lst].view(np.uint32).astype(np.uint64)
        np.testing.assert_array_equal(keys, expect_keys, err_msg=f"tile {cx},{cy} keys")
        # every pixel of the tile that lies inside the image
        ys, xs = np.mgrid[cy * 16:min(cy * 16 + 16, H), cx * 16:min(cx * 16 + 16, W)]
        o = ref.render_pixels_list(pre, cam, lst, xs.ravel(), ys.ravel())
        g_rgb = P.to_np(fr.out_rgb[:, ys.min():ys.max() + 1, xs.min():xs.max() + 1]).astype(np.float64)
        g_T = P.to_np(fr.out_T[ys.min():ys.max() + 1, xs.min():xs.max() + 1]).astype(np.float64)
        err = np.abs(g_rgb.reshape(3, -1).T - o.rgb).max(axis=1)
        errT = np.abs(g_T.reshape(-1) - o.T)
        plain = o.amb == 0
        assert np.all(err <= np.where(plain, P.IMG_TOL, P.IMG_TOL + o.beta)), f"tile {cx},{cy}: image error {err.max():.3e}"
        assert np.all(errT <= np.where(plain, P.IMG_TOL, P.IMG_TOL + o.beta_T)), f"tile {cx},{cy}: T error {errT.max():.3e}"
        if plain.any():
            worst = max(worst, float(err[plain].max()))
        print(f"[parity] cfg4 full tile ({cx},{cy}): list {len(lst)}, E/pixel {o.E.mean():.0f}, "
              f"C/pixel {o.C.mean():.0f}, max err {err.max():.2e}", flush=True)
    print(f"[parity] cfg4 full: worst unambiguous pixel error {worst:.2e}", flush=True)
    del fr
    torch.cuda.empty_cache()
