"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on
the same seeded inputs (bars in tests/parity.py)."""
import numpy as np
import pytest
import torch

from oracle import ref
from paper_2503_21364_amd import binding as B
from paper_2503_21364_amd import scenes

import parity as P

pytestmark = pytest.mark.gpu


def _report(name, stats):
    print(f"[parity] {name}: " + ", ".join(f"{k}={v:.3e}" if isinstance(v, float) else f"{k}={v}"
                                            for k, v in stats.items()), flush=True)


# ------------------------------------------------------------------ configs
def test_cfg0_full():
    sc = scenes.make_scene(0)
    cam = scenes.make_cameras(0)[0]
    r = P.full_compare(sc, cam)
    _report("cfg0", r.stats)
    assert r.stats["D"] > 30000


@pytest.mark.parametrize("w,h,n,seed,scale_mul", [
    (37, 23, 1000, 71, 1.0),        # partial tiles on both edges
    (200, 120, 4000, 21, 1.0),      # 13 x 8 tiles
    (256, 256, 257, 5, 4.0),        # one primitive past a workgroup boundary, fat splats
    (640, 360, 30011, 6, 2.0),      # several sort tiles with a ragged tail
    (16, 16, 500, 8, 6.0),          # a single tile holding everything
])
def test_small_ragged(w, h, n, seed, scale_mul):
    sc = scenes.make_scene(0, n=n, seed=seed)
    sc["scale"] *= np.float32(scale_mul)
    cam = scenes.make_cameras(0, w, h)[0]
    cam["bg"] = np.array([0.25, 0.5, 0.125], np.float32)
    r = P.full_compare(sc, cam)
    _report(f"ragged {w}x{h} n={n}", r.stats)


@pytest.mark.parametrize("view", [0, 5])
def test_cfg1_full_size(view):
    sc = scenes.make_scene(1)
    cam = scenes.make_cameras(1)[view]
    r = P.full_compare(sc, cam)
    _report(f"cfg1 view {view}", r.stats)
    assert r.stats["D"] > 3_000_000


def test_cfg2_full_size_exterior_and_interior():
    sc = scenes.make_scene(2)
    dev = B.Scene(sc)
    cams = scenes.make_cameras(2)
    for view in (0, 5):
        r = P.full_compare(sc, cams[view], scene_dev=dev)
        _report(f"cfg2 view {view}", r.stats)
        del r
    torch.cuda.empty_cache()


def test_cfg3_full_size_one_view():
    sc = scenes.make_scene(3)
    cam = scenes.make_cameras(3)[0]
    r = P.full_compare(sc, cam)
    _report("cfg3 view 0", r.stats)
    assert r.stats["visible"] < 0.5 * sc["n"]       # most primitives are frustum-culled
    del r
    torch.cuda.empty_cache()


def test_cfg4_distributions_reduced_count():
    # the heavy-overlap distributions at 1/100 of the primitives and 1080p, so
    # that the oracle can bin the whole frame (full size: test_gpu_large.py)
    sc = scenes.make_scene(4, n=20_000)
    cam = scenes.make_cameras(4, 1920, 1080)[0]
    r = P.full_compare(sc, cam)
    _report("cfg4 reduced", r.stats)
    assert r.stats["D"] / r.stats["visible"] > 300   # hundreds of tiles per primitive


@pytest.mark.parametrize("w,h,n,seed,binning,lo,hi", [
    (64, 64, 20_000, 41, 0, 4096, 8192),         # the four central tiles hold lists of two chunks: one merge round, then a copy
    (64, 64, 30_000, 45, 1, 8192, 12288),        # three chunks: a run without a partner in the first round
    (64, 64, 42_000, 46, 0, 12288, 16384),       # four chunks (ragged last one): both merge rounds
    (64, 64, 100_000, 47, 0, 16384, 1 << 30),    # beyond kHuge next to mid-sized lists
    (48, 40, 150_000, 42, 0, 16384, 1 << 30),    # 9 tiles (ragged), lists beyond kHuge: merges inside one workgroup
    (48, 40, 150_000, 43, 1, 16384, 1 << 30),
    (16, 16, 70_001, 44, 0, 16384, 1 << 30),     # everything in one tile: several merge rounds, ragged last run
])
def test_long_lists_in_few_tiles(w, h, n, seed, binning, lo, hi):
    sc = scenes.make_scene(0, n=n, seed=seed)
    cam = dict(scenes.make_cameras(0, w, h)[0], binning=binning)
    r = P.full_compare(sc, cam)
    _report(f"long lists {w}x{h} n={n} binning {binning}", r.stats)
    lens = np.diff(r.oracle.binned.tile_offsets.astype(np.int64))
    assert lo < lens.max() <= hi, lens.max()


def test_large_capacity_takes_the_wide_partition_tiles():
    """Above 64 Mi pairs of capacity the partition works on 4096-pair tiles instead of 2048:
    same result, here with several whole tiles and a ragged last one."""
    sc = scenes.make_scene(0, n=30011, seed=48)
    sc["scale"] *= np.float32(2.0)
    cam = dict(scenes.make_cameras(0, 640, 360)[0], binning=1)
    r = P.full_compare(sc, cam, capacity=(64 << 20) + 5)
    _report("wide partition tiles", r.stats)
    assert r.stats["D"] > 10 * 4096


@pytest.mark.parametrize("binning", [0, 1])
def test_rectangles_of_every_size_class(binning):
    """Rectangle areas from 1 tile to the whole 120 x 68 grid, dense around the sizes at which the
    emit stage switches method (32, 128 and 2048 tiles)."""
    rng = np.random.default_rng(5)
    n = 4000
    sc = scenes.make_scene(0, n=n, seed=55)
    sc["scale"] = sc["scale"] * np.exp(rng.uniform(np.log(0.5), np.log(60.0), n)).astype(np.float32)[None, :]
    cam = dict(scenes.make_cameras(0, 1920, 1080)[0], binning=binning)
    r = P.full_compare(sc, cam)
    rc = r.oracle.pre.rect.astype(int)
    area = ((rc[:, 2] - rc[:, 0]) * (rc[:, 3] - rc[:, 1]))[r.oracle.pre.tiles_touched > 0]
    for lo, hi in ((0, 16), (16, 32), (32, 48), (100, 128), (128, 160), (1800, 2048), (2048, 2400), (8159, 8160)):
        assert ((area > lo) & (area <= hi)).sum() > 20, (lo, hi)
    assert (area == 32).sum() > 0 and (area == 128).sum() > 0
    _report(f"size classes binning {binning}", r.stats)


# ------------------------------------------------------------------ binning rule 1
def _tight(cam):
    return dict(cam, binning=1)


@pytest.mark.parametrize("w,h,n,seed,scale_mul", [
    (37, 23, 1000, 71, 1.0),
    (256, 256, 257, 5, 4.0),        # rectangles of a few dozen tiles: the wavefront-cooperative count
    (640, 360, 30011, 6, 2.0),
    (16, 16, 500, 8, 6.0),
])
def test_binning1_small_ragged(w, h, n, seed, scale_mul):
    sc = scenes.make_scene(0, n=n, seed=seed)
    sc["scale"] *= np.float32(scale_mul)
    cam = _tight(scenes.make_cameras(0, w, h)[0])
    cam["bg"] = np.array([0.25, 0.5, 0.125], np.float32)
    r = P.full_compare(sc, cam)
    _report(f"binning1 ragged {w}x{h} n={n}", r.stats)


def test_binning1_configs_and_image_equal_to_rule0():
    for cfg, view, n, wh in [(0, 0, None, None), (1, 0, None, None), (2, 0, None, None), (2, 5, None, None),
                             (4, 0, 20_000, (1920, 1080))]:
        sc = scenes.make_scene(cfg, n=n)
        cam0 = scenes.make_cameras(cfg, *(wh or (None, None)))[view]
        dev = B.Scene(sc)
        r1 = P.full_compare(sc, _tight(cam0), scene_dev=dev)
        _report(f"binning1 cfg{cfg} view {view}", r1.stats)
        fr0 = P.gpu_frame(dev, cam0, r1.stats["D"] * 3 + 1000)
        D0, _ = B.read_status(fr0)
        assert r1.stats["D"] < D0
        # dropping pairs that cannot contribute leaves every pixel exactly as it was
        assert torch.equal(fr0.out_rgb, r1.gpu.out_rgb) and torch.equal(fr0.out_T, r1.gpu.out_T)
        del r1, fr0, dev
        torch.cuda.empty_cache()


# ------------------------------------------------------------------ degenerate inputs
def test_empty_scene():
    sc = scenes.make_scene(0, n=0)
    cam = scenes.make_cameras(0, 64, 48)[0]
    cam["bg"] = np.array([0.1, 0.2, 0.3], np.float32)
    r = P.full_compare(sc, cam)
    assert r.stats["D"] == 0
    assert torch.all(r.gpu.out_T == 1.0)


def test_everything_culled():
    sc = scenes.make_scene(0, n=5000, seed=9)
    eye = (0.0, 0.0, 4.0)
    cam = scenes.make_camera(scenes.look_at(eye, (0, 0, 8.0), (0, 1, 0)), eye, 100, 60, 60.0, bg=(0.2, 0.4, 0.6))
    r = P.full_compare(sc, cam)
    assert r.stats["D"] == 0 and r.stats["visible"] == 0
    np.testing.assert_array_equal(P.to_np(r.gpu.out_rgb[1]), np.float32(0.4))


@pytest.mark.parametrize("binning", [0, 1])
def test_degenerate_attribute_values(binning):
    # non-finite centres, zero / non-finite / overflowing rotations and scales, opacities at the threshold
    sc, groups = scenes.hostile_scene()
    cam = dict(scenes.make_cameras(0, 300, 200)[0], binning=binning)
    r = P.full_compare(sc, cam)
    assert torch.isfinite(r.gpu.out_rgb).all() and torch.isfinite(r.gpu.out_T).all()
    _report(f"degenerate values binning {binning}", r.stats)


def test_single_primitive_covering_many_tiles():
    sc = scenes.hand_placed_scene([(0.1, -0.2, 0.0)], [(0.8, 0.3, 0.5)], rot=(0.9, 0.1, 0.3, -0.2),
                                  opacity=0.7, sh_dc=(1.0, 0.2, -0.4))
    cam = scenes.make_cameras(0, 320, 200)[0]
    r = P.full_compare(sc, cam)
    assert r.stats["D"] > 100 and r.stats["visible"] == 1


@pytest.mark.parametrize("deg", [0, 1, 2])
def test_lower_sh_degrees(deg):
    sc = scenes.make_scene(0, n=3000, seed=13)
    sc["sh_degree"] = deg
    cam = scenes.make_cameras(0, 128, 128)[0]
    r = P.full_compare(sc, cam)
    _report(f"sh degree {deg}", r.stats)


def test_equal_depths_are_ordered_by_index():
    # many primitives on one plane facing the camera: identical depth bits inside a tile
    rng = np.random.default_rng(3)
    n = 3000
    mean = np.stack([rng.uniform(-1, 1, n), rng.uniform(-1, 1, n), np.zeros(n)], axis=1)
    sc = scenes.hand_placed_scene(mean, [(0.05, 0.05, 0.05)], opacity=0.5,
                                  sh_dc=rng.uniform(-1, 1, (n, 3)))
    cam = scenes.make_cameras(0, 128, 128)[0]
    r = P.full_compare(sc, cam)
    keys = r.oracle.binned.keys
    assert (keys[1:] == keys[:-1]).sum() > 1000


@pytest.mark.parametrize("n,scale_mul,wh,binning", [
    (5000, 1.0, (128, 128), 0),
    (3000, 6.0, (1920, 1080), 0),   # rectangles of hundreds and thousands of tiles: the deferred expansion paths
    (3000, 6.0, (1920, 1080), 1),
])
def test_capacity_overflow_sets_status_and_stays_in_bounds(n, scale_mul, wh, binning):
    sc = scenes.make_scene(0, n=n, seed=17)
    sc["scale"] = sc["scale"] * np.float32(scale_mul)
    cam = dict(scenes.make_cameras(0, *wh)[0], binning=binning)
    ofr = ref.render_frame(sc, cam)
    if scale_mul > 1.0:
        area = (ofr.pre.rect[:, 2].astype(int) - ofr.pre.rect[:, 0]) * (ofr.pre.rect[:, 3].astype(int) - ofr.pre.rect[:, 1])
        assert (area > 2048).sum() > 10 and ((area > 128) & (area <= 2048)).sum() > 100 and (area <= 128).sum() > 10
    cap = ofr.binned.D // 2
    dev = B.Scene(sc)
    fr = B.Frame(dev.n, wh[0], wh[1], cap)
    for t in (fr.keys, fr.vals, fr.keys_alt, fr.vals_alt):
        t.fill_(-3)
    B.render_frame(dev, B.make_camera(cam), fr)
    torch.cuda.synchronize()
    D, status = B.read_status(fr)
    # the true pair count comes back, so that the caller can size a retry
    assert D == ofr.binned.D and status == B.ERR_CAPACITY
    # nothing was emitted: every range is empty, the pair buffers are as they were, the image is the background
    assert not P.to_np(fr.tile_offsets).any()
    assert bool((fr.keys == -3).all()) and bool((fr.vals == -3).all())
    assert bool((fr.out_T == 1.0).all())
    bg = torch.tensor(np.asarray(cam["bg"], np.float32), device="cuda")[:, None, None]
    assert bool((fr.out_rgb == bg).all())
    # and the retry with the capacity the call reported fits exactly
    fr2 = B.Frame(dev.n, wh[0], wh[1], D, want_offsets=True)
    B.render_frame(dev, B.make_camera(cam), fr2)
    torch.cuda.synchronize()
    P.compare_binned(fr2, ofr.binned)


@pytest.mark.parametrize("binning", [0, 1])
def test_bin_sort_again_on_the_same_scratch_after_an_overflow(binning):
    """Stage 2 leaves the scratch ready for another stage 2: after a call that overflowed, a second
    call with enough room -- same scratch, no preprocess in between -- gives the oracle's arrays, and
    a third call gives them again."""
    sc = scenes.make_scene(0, n=20000, seed=23)
    sc["scale"] = sc["scale"] * np.float32(3.0)           # rectangles on all three paths of stage 2
    cam = dict(scenes.make_cameras(0, 640, 360)[0], binning=binning)
    ofr = ref.render_frame(sc, cam)
    dev = B.Scene(sc)
    fr = B.Frame(dev.n, 640, 360, ofr.binned.D + 7, want_offsets=True)
    cc = B.make_camera(cam)
    B.preprocess(dev, cc, fr)
    full = fr.binned.capacity
    fr.binned.capacity = ofr.binned.D // 3               # the scratch was sized for the larger capacity
    B.bin_sort(cc, fr)
    torch.cuda.synchronize()
    D, status = B.read_status(fr)
    assert D == ofr.binned.D and status == B.ERR_CAPACITY
    assert not P.to_np(fr.tile_offsets).any()
    fr.binned.capacity = full
    for _ in range(2):
        B.bin_sort(cc, fr)
        torch.cuda.synchronize()
        D, status = B.read_status(fr)
        assert D == ofr.binned.D and status == B.OK         # the status is that of the latest call
        P.compare_binned(fr, ofr.binned)


# ------------------------------------------------------------------ stage isolation
def _upload_projected(fr, pre):
    n = pre.n
    fr.depth[:n] = torch.from_numpy(pre.depth).cuda()
    fr.tiles_touched[:n] = torch.from_numpy(pre.tiles_touched.view(np.int32)).cuda()
    fr.rect[:n] = torch.from_numpy(pre.rect.view(np.int16)).cuda()
    feat = np.zeros((n, B.FEAT_STRIDE), np.float32)
    feat[:, 0:2] = pre.mean2d.T
    feat[:, 2:5] = pre.conic.T
    feat[:, 5] = pre.opacity
    feat[:, 6:9] = pre.rgb.T.astype(np.float32)
    fr.feat[:n] = torch.from_numpy(feat).cuda()


def test_bin_sort_alone_from_oracle_projection():
    sc = scenes.make_scene(0, n=20000, seed=23)
    sc["scale"] *= np.float32(2.0)
    cam = scenes.make_cameras(0, 300, 200)[0]
    ofr = ref.render_frame(sc, cam)
    dev = B.Scene(sc)
    c = B.make_camera(cam)
    fr = B.Frame(dev.n, 300, 200, ofr.binned.D + 7, want_offsets=True)
    B.preprocess(dev, c, fr)          # fills the workgroup tile counts in scratch
    _upload_projected(fr, ofr.pre)    # then the oracle's arrays replace the GPU's
    B.bin_sort(c, fr)
    torch.cuda.synchronize()
    P.compare_binned(fr, ofr.binned)


def test_render_alone_from_oracle_lists():
    sc = scenes.make_scene(0, n=8000, seed=29)
    sc["scale"] *= np.float32(2.5)
    cam = scenes.make_cameras(0, 200, 136)[0]
    cam["bg"] = np.array([0.5, 0.25, 0.75], np.float32)
    ofr = ref.render_frame(sc, cam)
    fr = B.Frame(sc["n"], 200, 136, ofr.binned.D + 1, tile_order=False)   # bin_sort never runs here
    _upload_projected(fr, ofr.pre)
    D = ofr.binned.D
    fr.vals[:D] = torch.from_numpy(ofr.binned.vals.view(np.int32)).cuda()
    fr.tile_offsets[:] = torch.from_numpy(ofr.binned.tile_offsets.view(np.int64)).cuda()
    B.render(B.make_camera(cam), fr)
    torch.cuda.synchronize()
    st = P.compare_image(fr, ofr.img, cam)
    _report("render alone", st)


def test_tile_order_is_a_permutation_by_descending_length_class():
    sc = scenes.make_scene(0, n=20000, seed=37)
    sc["scale"] *= np.float32(2.0)
    cam = scenes.make_cameras(0, 400, 240)[0]
    fr = P.gpu_frame(B.Scene(sc), cam, 2_000_000)
    order = P.to_np(fr.tile_order).view(np.uint32).astype(np.int64)
    T = fr.tiles_x * fr.tiles_y
    assert np.array_equal(np.sort(order), np.arange(T))
    lens = np.diff(P.to_np(fr.tile_offsets).view(np.uint64).astype(np.int64))[order]
    # classes: bit length of (length - 1), so that 2^k pairs still belong to the class below
    cls = np.where(lens > 1, np.floor(np.log2(np.maximum(lens - 1, 1))).astype(np.int64) + 1, 0)
    assert np.all(np.diff(cls) <= 0)
    # and the image does not depend on the hint
    fr2 = B.Frame(sc["n"], 400, 240, 2_000_000, tile_order=False)
    B.render_frame(B.Scene(sc), B.make_camera(cam), fr2)
    torch.cuda.synchronize()
    assert torch.equal(fr.out_rgb, fr2.out_rgb) and torch.equal(fr.out_T, fr2.out_T)


def test_two_runs_are_bytewise_identical():
    sc = scenes.make_scene(1, n=100_000)
    cam = scenes.make_cameras(1, 960, 540)[3]
    dev = B.Scene(sc)
    outs = []
    for _ in range(2):
        fr = P.gpu_frame(dev, cam, 2_000_000)
        D, status = B.read_status(fr)
        assert status == B.OK
        outs.append((D, fr.keys[:D].clone(), fr.vals[:D].clone(), fr.tile_offsets.clone(),
                     fr.out_rgb.clone(), fr.out_T.clone()))
    assert outs[0][0] == outs[1][0]
    for a, b in zip(outs[0][1:], outs[1][1:]):
        assert torch.equal(a, b)


def test_runs_on_a_side_stream():
    sc = scenes.make_scene(0, n=5000, seed=31)
    cam = scenes.make_cameras(0, 160, 96)[0]
    ofr = ref.render_frame(sc, cam)
    dev = B.Scene(sc)
    s = torch.cuda.Stream()
    torch.cuda.synchronize()
    fr = B.Frame(dev.n, 160, 96, ofr.binned.D + 5)
    torch.cuda.synchronize()
    with torch.cuda.stream(s):
        B.render_frame(dev, B.make_camera(cam), fr, stream=s)
    s.synchronize()
    P.compare_binned(fr, ofr.binned)
    P.compare_image(fr, ofr.img, cam)


@pytest.mark.parametrize("lengths", [
    (4096, 4097, 8192, 8193), (16384, 16385, 512, 513), (2048, 2049, 1, 0), (12288, 12289, 64, 65),
])
def test_list_lengths_on_the_size_class_boundaries(lengths):
    """Four tiles whose lists have exactly the given lengths (tiny splats at the tile centres, at
    random depths): every boundary between the per-tile sort's size classes, from both sides."""
    W, H = 64, 16
    eye = (0.0, 0.0, -10.0)
    cam = scenes.make_camera(scenes.look_at(eye, (0.0, 0.0, 0.0), (0.0, -1.0, 0.0)), eye, W, H, 50.0)
    rng = np.random.default_rng(sum(lengths))
    means = []
    # the camera's axes from its own view matrix: world = eye + R^T (x, y, z)_camera
    V = np.asarray(cam["view"], np.float64).reshape(3, 4)
    R, t = V[:, :3], V[:, 3]
    for tile, L in enumerate(lengths):
        u, v = 16.0 * tile + 8.0, 8.0
        z = 10.0 + rng.uniform(-1.0, 1.0, size=L)
        pc = np.stack([(u - cam["cx"]) / cam["fx"] * z, (v - cam["cy"]) / cam["fy"] * z, z])
        means.append((R.T @ (pc - t[:, None])).T)
    means = np.concatenate(means) if sum(lengths) else np.zeros((0, 3))
    order = rng.permutation(len(means))
    sc = scenes.hand_placed_scene(means[order], (0.002, 0.002, 0.002), opacity=0.5, sh_dc=(0.4, 0.2, 0.1))
    r = P.full_compare(sc, dict(cam, binning=1))
    lens = np.diff(r.oracle.binned.tile_offsets.astype(np.int64))
    assert tuple(lens) == tuple(lengths), lens
    _report(f"class boundaries {lengths}", r.stats)
