"""lmk_gs_bin_sort_static (the entry point that allocates nothing and brings its own scratch)
against lmk_gs_bin_sort on the same per-primitive outputs: pair count, sorted keys and values,
tile ranges and tile order classes bit for bit, on two calls in a row, the second with a smaller
input (the shared array keeps the first call's contents)."""
import numpy as np
import pytest
import torch

from paper_2503_21364_amd import binding as B
from paper_2503_21364_amd import scenes

pytestmark = pytest.mark.gpu


def _np(t):
    return t.detach().cpu().numpy()


def _one(n, w, h, seed, binning, scale_mul, count_status):
    sc = scenes.make_scene(0, n=n, seed=seed)
    sc["scale"] *= np.float32(scale_mul)
    cam = B.make_camera(dict(scenes.make_cameras(0, w, h)[0], binning=binning))
    dev = B.Scene(sc)
    # reference: preprocess + bin_sort on a caller's workspace
    probe = B.Frame(dev.n, w, h, 1, want_offsets=False)
    B.preprocess(dev, cam, probe)
    D = int(probe.tiles_touched[:dev.n].sum().item())
    cap = D + 100
    a = B.Frame(dev.n, w, h, cap, want_offsets=True)
    B.preprocess(dev, cam, a)
    B.bin_sort(cam, a)
    torch.cuda.synchronize()
    Da, status = B.read_status(a)
    assert (Da, status) == (D, B.OK)
    # the variant: same per-primitive outputs (from a preprocess call on another scratch), no workspace
    b = B.Frame(dev.n, w, h, cap, want_offsets=True)
    B.preprocess(dev, cam, b)
    b.scratch.fill_(0xAB)                      # whatever preprocess left there is not what the variant reads
    for t in (b.keys, b.vals, b.tile_offsets, b.tile_order, b.offsets):
        t.fill_(-1)
    count_status.fill_(-7)
    B.bin_sort_static(cam, b, count_status)
    torch.cuda.synchronize()
    cs = _np(count_status)
    assert int(cs[0]) == D and int(cs[1]) == B.OK, cs
    np.testing.assert_array_equal(_np(b.tile_offsets), _np(a.tile_offsets), err_msg="tile_offsets")
    np.testing.assert_array_equal(_np(b.keys[:D]), _np(a.keys[:D]), err_msg="sorted keys")
    np.testing.assert_array_equal(_np(b.vals[:D]), _np(a.vals[:D]), err_msg="sorted values")
    np.testing.assert_array_equal(_np(b.offsets), _np(a.offsets), err_msg="offsets")
    # tile_order is unique up to the order inside a length class: compare the lengths it lists
    lens = np.diff(_np(a.tile_offsets))
    cls = lambda L: np.where(L > 1, np.ceil(np.log2(np.maximum(L, 1))), 0)
    np.testing.assert_array_equal(cls(lens[_np(b.tile_order)]), cls(lens[_np(a.tile_order)]))
    # and the frame renders to the same image
    B.render(cam, a); B.render(cam, b)
    torch.cuda.synchronize()
    assert torch.equal(a.out_rgb, b.out_rgb) and torch.equal(a.out_T, b.out_T)
    return D


@pytest.mark.parametrize("binning", [0, 1])
def test_static_scratch_variant_matches_bin_sort_twice_in_a_row(binning):
    count_status = torch.zeros(2, dtype=torch.int64, device="cuda:0")
    print(f"[no-alloc] binning {binning}: first call, 30011 primitives 640x360", flush=True)
    D1 = _one(30011, 640, 360, 6, binning, 2.0, count_status)
    print(f"[no-alloc] first call ok, D = {D1}; second call, 3000 primitives 200x120", flush=True)
    D2 = _one(3000, 200, 120, 21, binning, 1.0, count_status)
    print(f"[no-alloc] second call ok, D = {D2}", flush=True)
    assert D2 < D1


def test_static_scratch_variant_capacity_overflow_and_limits():
    sc = scenes.make_scene(0, n=2000, seed=3)
    w = h = 128
    cam = B.make_camera(scenes.make_cameras(0, w, h)[0])
    dev = B.Scene(sc)
    probe = B.Frame(dev.n, w, h, 1)
    B.preprocess(dev, cam, probe)
    D = int(probe.tiles_touched[:dev.n].sum().item())
    fr = B.Frame(dev.n, w, h, D // 2)
    B.preprocess(dev, cam, fr)
    cs = torch.zeros(2, dtype=torch.int64, device="cuda:0")
    B.bin_sort_static(cam, fr, cs)
    torch.cuda.synchronize()
    assert int(cs[0].item()) == D and int(cs[1].item()) == B.ERR_CAPACITY
    # sizes beyond the fixed array are refused on the host, nothing is enqueued
    fr.binned.capacity = B.STATIC_MAX_CAPACITY + 1
    with pytest.raises(B.LmkGsError) as ei:
        B.bin_sort_static(cam, fr, cs)
    assert ei.value.code == B.ERR_CAPACITY
    fr.binned.capacity = D // 2
    fr.n = B.STATIC_MAX_N + 1
    with pytest.raises(B.LmkGsError) as ei:
        B.bin_sort_static(cam, fr, cs)
    assert ei.value.code == B.ERR_CAPACITY
