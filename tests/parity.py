"""Helpers of the GPU parity tests: run the HIP path through the C ABI, run the
CPU oracle on the same seeded inputs, compare stage by stage.

Bars (written out here, used by every parity test):
  * integer outputs -- tiles_touched, rect, pair count, offsets, keys, values,
    tile ranges -- and the depth bits: bit-exact;
  * key-path floats (u, v, conic, opacity): produced by the same fp32 operation
    sequence on both sides, compared exactly;
  * SH colour (fp32 on the GPU, fp64 in the oracle): 2e-5 absolute + 1e-5 relative;
  * image and transmittance: |gpu - oracle| <= 1e-4 per channel on every pixel in which the
    oracle found no decision (alpha against 1/255, T' against 1e-4) within fp32 rounding of its
    threshold.  A pixel that holds such a decision may take it either way in any fp32 renderer,
    which moves it by that pair's whole contribution (up to 4e-3); there the bar is
    1e-4 + beta(pixel), beta being the oracle's bound on what the flips can move plus the
    first-order fp32 rounding of the walk.  The share of such pixels is bounded (0.5 %), and so
    is the share of the other pixels whose rounding budget alone exceeds a quarter of the bar.
"""
from __future__ import annotations

from types import SimpleNamespace

import numpy as np
import torch

from oracle import ref
from paper_2503_21364_amd import binding as B

IMG_TOL = 1e-4


def to_np(t):
    return t.detach().cpu().numpy()


def gpu_frame(scene_dev: B.Scene, cam: dict, capacity: int, want_offsets=True, index=None) -> B.Frame:
    fr = B.Frame(scene_dev.n, int(cam["width"]), int(cam["height"]), capacity, want_offsets=want_offsets)
    B.render_frame(scene_dev, B.make_camera(cam), fr, index=index)
    torch.cuda.synchronize()
    return fr


def compare_projected(fr: B.Frame, pre) -> dict:
    n = pre.n
    tt = to_np(fr.tiles_touched)[:n].view(np.uint32)
    np.testing.assert_array_equal(tt, pre.tiles_touched, err_msg="tiles_touched")
    vis = pre.tiles_touched > 0
    rect = to_np(fr.rect)[:n].view(np.uint16)
    np.testing.assert_array_equal(rect[vis], pre.rect[vis], err_msg="rect")
    depth = to_np(fr.depth)[:n]
    np.testing.assert_array_equal(depth[vis].view(np.uint32), pre.depth[vis].view(np.uint32), err_msg="depth bits")
    feat = to_np(fr.feat)[:n]
    np.testing.assert_array_equal(feat[vis, 0], pre.mean2d[0, vis], err_msg="u")
    np.testing.assert_array_equal(feat[vis, 1], pre.mean2d[1, vis], err_msg="v")
    for k, name in enumerate("ABC"):
        np.testing.assert_array_equal(feat[vis, 2 + k], pre.conic[k, vis], err_msg=f"conic {name}")
    np.testing.assert_array_equal(feat[vis, 5], pre.opacity[vis], err_msg="opacity")
    rgb_err = np.abs(feat[vis, 6:9].T.astype(np.float64) - pre.rgb[:, vis])
    tol = 2e-5 + 1e-5 * np.abs(pre.rgb[:, vis])
    assert np.all(rgb_err <= tol), f"SH colour off by {rgb_err.max()}"
    return dict(visible=int(vis.sum()), rgb_max_err=float(rgb_err.max()) if vis.any() else 0.0)


def compare_binned(fr: B.Frame, b) -> dict:
    D, status = B.read_status(fr)
    assert status == B.OK, f"status {status}"
    assert D == b.D, f"pair count {D} != {b.D}"
    if fr.offsets is not None:
        np.testing.assert_array_equal(to_np(fr.offsets).view(np.uint64), b.offsets, err_msg="offsets")
    np.testing.assert_array_equal(to_np(fr.tile_offsets).view(np.uint64), b.tile_offsets, err_msg="tile_offsets")
    np.testing.assert_array_equal(to_np(fr.keys[:D]).view(np.uint64), b.keys, err_msg="sorted keys")
    np.testing.assert_array_equal(to_np(fr.vals[:D]).view(np.uint32), b.vals, err_msg="sorted values")
    return dict(D=D)


def image_errors(rgb, T, img):
    """Per-pixel errors, tolerances and the mask of pixels without an ambiguous decision."""
    plain = img.amb == 0
    tol_rgb = np.where(plain, IMG_TOL, IMG_TOL + img.beta)
    tol_T = np.where(plain, IMG_TOL, IMG_TOL + img.beta_T)
    err_rgb = np.abs(rgb - img.rgb).max(axis=0)
    err_T = np.abs(T - img.T)
    return err_rgb, err_T, tol_rgb, tol_T, plain


def compare_image(fr: B.Frame, img, cam: dict, max_ambiguous_share=0.005, max_loose_share=0.25) -> dict:
    rgb = to_np(fr.out_rgb).astype(np.float64)
    T = to_np(fr.out_T).astype(np.float64)
    assert float(np.max(np.abs(cam["bg"]))) <= 1.0
    err_rgb, err_T, tol_rgb, tol_T, plain = image_errors(rgb, T, img)
    share = 1.0 - plain.mean()
    bad = (err_rgb > tol_rgb) | (err_T > tol_T)
    if bad.any():
        ys, xs = np.nonzero(bad)
        raise AssertionError(f"{bad.sum()} pixels beyond tolerance ({(bad & plain).sum()} of them without an "
                             f"ambiguous decision: bar {IMG_TOL}); first (x={xs[0]}, y={ys[0]}): "
                             f"rgb err {err_rgb[ys[0], xs[0]]:.3e}, T err {err_T[ys[0], xs[0]]:.3e}, "
                             f"beta {img.beta[ys[0], xs[0]]:.3e}, amb {img.amb[ys[0], xs[0]]}; "
                             f"worst unambiguous rgb err {err_rgb[plain].max():.3e}")
    assert share <= max_ambiguous_share, f"{share:.4f} of the pixels hold an ambiguous decision"
    # the rounding part of the budget must stay a small fraction of the bar for most pixels
    loose = (img.beta[plain] > 0.25 * IMG_TOL).mean() if plain.any() else 0.0
    assert loose <= max_loose_share, f"rounding budget above a quarter of the bar on {loose:.3f} of the pixels"
    assert np.median(img.beta) <= 0.1 * IMG_TOL, f"median rounding budget {np.median(img.beta):.2e}"
    return dict(max_err_plain=float(err_rgb[plain].max()) if plain.any() else 0.0,
                max_err_T_plain=float(err_T[plain].max()) if plain.any() else 0.0,
                max_err_all=float(err_rgb.max()), ambiguous_share=float(share),
                median_budget=float(np.median(img.beta)), loose_share=float(loose))


def full_compare(scene: dict, cam: dict, capacity: int | None = None, scene_dev: B.Scene | None = None,
                 oracle_frame=None, index=None) -> SimpleNamespace:
    """GPU frame vs oracle frame, every stage, element by element.  With a voxel index the GPU
    runs the voxel filter first; the oracle frame is always the unfiltered definition."""
    ofr = ref.render_frame(scene, cam) if oracle_frame is None else oracle_frame
    if capacity is None:
        capacity = ofr.binned.D + 1000
    if scene_dev is None:
        scene_dev = B.Scene(scene)
    fr = gpu_frame(scene_dev, cam, capacity, index=index)
    stats = {}
    stats.update(compare_projected(fr, ofr.pre))
    stats.update(compare_binned(fr, ofr.binned))
    stats.update(compare_image(fr, ofr.img, cam))
    stats["E"] = int(ofr.img.E.sum()); stats["C"] = int(ofr.img.C.sum())
    return SimpleNamespace(gpu=fr, oracle=ofr, stats=stats)
