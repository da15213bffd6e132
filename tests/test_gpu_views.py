"""Every viewpoint of configurations 1-3 at full size, in the configuration bench.py times: binning
rule 1, the scene reordered into voxels with the view-frustum filter in front (where bench.py uses
one), the covariance cache.  Each frame is compared stage by stage, element by element, with the
oracle's frame of the same (reordered) scene -- which knows nothing of voxels or caches -- to the
bars of tests/parity.py."""
import numpy as np
import pytest
import torch

import bench
from paper_2503_21364_amd import binding as B
from paper_2503_21364_amd import scenes

import parity as P

pytestmark = pytest.mark.gpu

_cache = {}


def _setup(cfg):
    """Scene, voxel index and device copies of one configuration; one configuration is held at a time."""
    if cfg not in _cache:
        _cache.clear()
        torch.cuda.empty_cache()
        sc = scenes.make_scene(cfg)
        voxel = bench.VOXEL_SIZE[cfg]
        index = None
        if voxel > 0.0:
            index = B.VoxelIndex(sc, voxel)
            sc = index.reorder(sc)
            index.upload()
        dev = B.Scene(sc).build_cov3d()
        _cache[cfg] = (sc, index, dev, scenes.make_cameras(cfg))
    return _cache[cfg]


@pytest.mark.parametrize("cfg,view", [(c, v) for c in (1, 2, 3) for v in range(8)])
def test_bench_configuration_every_view(cfg, view):
    sc, index, dev, cams = _setup(cfg)
    cam = dict(cams[view], binning=1)
    print(f"[views] cfg{cfg} view {view}: start", flush=True)
    r = P.full_compare(sc, cam, scene_dev=dev, index=index)
    print(f"[parity] cfg{cfg} view {view} (rule 1, voxel {bench.VOXEL_SIZE[cfg]}, cache): "
          + ", ".join(f"{k}={v:.3e}" if isinstance(v, float) else f"{k}={v}" for k, v in r.stats.items()),
          flush=True)
    del r
    if view == 7:
        _cache.clear()
        torch.cuda.empty_cache()
