"""GPU parity of the parameter cache (Sec. 5.2.2: "inference parameter cache"): the cached
covariances against the oracle's Eq. 8, and frames rendered from the cache against the oracle."""
import numpy as np
import pytest
import torch

from oracle import ref
from paper_2503_21364_amd import binding as B
from paper_2503_21364_amd import scenes

import parity as P

pytestmark = pytest.mark.gpu


def test_cached_covariances_are_the_oracles_bit_for_bit():
    sc = scenes.make_scene(2, n=20_001, seed=77)
    sc["rot"][:, :100] *= np.float32(7.5)          # unnormalised quaternions are allowed
    dev = B.Scene(sc).build_cov3d()
    torch.cuda.synchronize()
    got = dev.cov3d.cpu().numpy()[:, :sc["n"]]
    for i in list(range(0, 300)) + list(range(19_800, 20_001)):
        S = np.asarray(ref.covariance3d(sc["rot"][:, i], sc["scale"][:, i]), np.float32).reshape(3, 3)
        expect = np.array([S[0, 0], S[0, 1], S[0, 2], S[1, 1], S[1, 2], S[2, 2]], np.float32)
        assert np.array_equal(got[:, i].view(np.uint32), expect.view(np.uint32)), i


@pytest.mark.parametrize("cfg,n,view,wh,binning,voxel", [
    (2, 200_000, 0, (960, 540), 1, 0.0),
    (2, 200_000, 5, (960, 540), 0, 2.0),
    (0, 999, 0, (250, 130), 1, 0.0),
])
def test_frames_from_the_cache_match_the_oracle(cfg, n, view, wh, binning, voxel):
    sc = scenes.make_scene(cfg, n=n, seed=78)
    index = None
    if voxel > 0:
        index = B.VoxelIndex(sc, voxel)
        sc = index.reorder(sc)
        index.upload()
    cam = dict(scenes.make_cameras(cfg, *wh)[view], binning=binning)
    dev = B.Scene(sc).build_cov3d()
    # the kernels must not need rotation and scale any more
    dev.c.rot = None
    dev.c.scale = None
    r = P.full_compare(sc, cam, scene_dev=dev, index=index)
    print(f"[parity] cache cfg{cfg} view {view}: D={r.stats['D']}", flush=True)
