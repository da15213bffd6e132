"""GPU parity of the voxel filter in front of the projection (lmk_gs_preprocess_culled):
the per-group flags against the oracle's voxel test, and -- the point of the filter -- every
output identical to the oracle's unfiltered frame of the same reordered scene."""
import numpy as np
import pytest
import torch

from oracle import ref
from paper_2503_21364_amd import binding as B
from paper_2503_21364_amd import scenes

import parity as P

pytestmark = pytest.mark.gpu


def _oracle_block_flags(oidx, cam, n):
    vis = ref.voxels_visible(oidx, cam)
    mask = ref.primitives_in_visible_voxels(oidx, vis)
    nb = (n + B.PRE_BLOCK - 1) // B.PRE_BLOCK
    pad = np.zeros(nb * B.PRE_BLOCK, bool); pad[:n] = mask
    return pad.reshape(nb, B.PRE_BLOCK).any(axis=1).astype(np.uint8), mask


@pytest.mark.parametrize("cfg,n,voxel,mul,view,wh,binning", [
    (2, 300_000, 2.0, 1.0, 4, (960, 540), 1),
    (2, 300_000, 2.0, 1.0, 5, (960, 540), 0),
    (2, 300_000, 3.0, 6.0, 7, (640, 360), 1),      # fat splats: the reach term decides
    (2, 300_000, 2.0, 1.0, 0, (960, 540), 1),      # exterior: nearly everything visible
    (3, 1_000_000, 40.0, 1.0, 0, (1920, 1080), 1),
    (0, 10_000, 0.25, 1.0, 0, (256, 256), 0),
    (1, 999, 1.0, 2.0, 3, (333, 222), 1),          # ragged: last group partial
])
def test_filtered_frame_is_the_unfiltered_frame(cfg, n, voxel, mul, view, wh, binning):
    sc = scenes.make_scene(cfg, n=n, seed=300 + cfg)
    sc["scale"] = sc["scale"] * np.float32(mul)
    vi = B.VoxelIndex(sc, voxel)
    oidx = ref.build_voxel_index(sc, voxel)
    assert np.array_equal(vi.perm, oidx.perm)
    sc2 = vi.reorder(sc)
    cam = dict(scenes.make_cameras(cfg, *wh)[view], binning=binning)
    vi.upload()
    r = P.full_compare(sc2, cam, index=vi)
    # the flags themselves, and what was skipped
    dev = B.Scene(sc2)
    fr = B.Frame(dev.n, wh[0], wh[1], 16)
    nb = (dev.n + B.PRE_BLOCK - 1) // B.PRE_BLOCK
    flags = torch.full((nb,), 7, dtype=torch.uint8, device="cuda")
    fr.tiles_touched.fill_(-1)
    B.preprocess(dev, B.make_camera(cam), fr, index=vi, block_visible=flags)
    torch.cuda.synchronize()
    expect, mask = _oracle_block_flags(oidx, cam, dev.n)
    np.testing.assert_array_equal(flags.cpu().numpy(), expect)
    tt = P.to_np(fr.tiles_touched)[:dev.n].view(np.uint32)
    np.testing.assert_array_equal(tt, r.oracle.pre.tiles_touched)
    print(f"[parity] voxels cfg{cfg} view {view}: {vi.num_voxels} voxels, groups processed "
          f"{expect.mean():.3f}, primitives in visible voxels {mask.mean():.3f}, binned "
          f"{(r.oracle.pre.tiles_touched > 0).mean():.3f}", flush=True)


def test_cfg2_full_size_interior_view_with_the_filter():
    sc = scenes.make_scene(2)
    vi = B.VoxelIndex(sc, 2.0)
    sc2 = vi.reorder(sc)
    vi.upload()
    cam = dict(scenes.make_cameras(2)[5], binning=1)
    r = P.full_compare(sc2, cam, index=vi)
    print("[parity] voxels cfg2 full view 5:", {k: v for k, v in r.stats.items() if k in ("D", "visible")}, flush=True)
    del r
    torch.cuda.empty_cache()


def test_rejects_a_camera_that_is_not_rigid():
    sc = scenes.make_scene(0, n=600, seed=3)
    vi = B.VoxelIndex(sc, 0.5).upload()
    dev = B.Scene(vi.reorder(sc))
    cam = scenes.make_cameras(0)[0]
    cam["view"] = cam["view"].copy(); cam["view"][0] *= 1.05
    fr = B.Frame(dev.n, 256, 256, 16)
    with pytest.raises(B.LmkGsError) as e:
        B.preprocess(dev, B.make_camera(cam), fr, index=vi)
    assert e.value.code == B.ERR_UNSUPPORTED
