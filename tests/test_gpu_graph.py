"""The calls of a frame are plain kernel launches on the caller's stream (no allocation, no memset
node, no synchronisation), so a caller may record them into a HIP graph once and replay it per
frame.  Recorded here through torch's graph capture: the forward path, the allocation-free stage 2
and the two gradient calls; every replay is compared with the oracle (forward) or with the eager
calls (gradients, which differ from run to run by the order of their float atomics)."""
import numpy as np
import pytest
import torch

from oracle import ref
from paper_2503_21364_amd import binding as B
from paper_2503_21364_amd import scenes

import parity as P

pytestmark = pytest.mark.gpu


def _scene():
    sc = scenes.make_scene(0, n=20000, seed=31)
    sc["scale"] = sc["scale"] * np.float32(2.0)
    return sc


@pytest.mark.parametrize("binning,static_stage2", [(0, False), (1, False), (1, True)])
def test_forward_path_recorded_once_and_replayed(binning, static_stage2):
    sc = _scene()
    cams = [dict(c, binning=binning) for c in scenes.make_cameras(1, 640, 360)[:3]]
    oracle = [ref.render_frame(sc, c) for c in cams]
    dev = B.Scene(sc)
    cap = max(o.binned.D for o in oracle) + 64
    fr = B.Frame(dev.n, 640, 360, cap, want_offsets=True)
    # the camera is an argument passed by value when the launch is recorded: one graph per viewpoint
    graphs, ccams = [], [B.make_camera(c) for c in cams]
    count_status = torch.zeros(2, dtype=torch.int64, device="cuda")
    side = torch.cuda.Stream()
    for cc in ccams:
        B.render_frame(dev, cc, fr)                                     # eager once, before recording
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=side):
            B.preprocess(dev, cc, fr)
            if static_stage2:
                B.bin_sort_static(cc, fr, count_status)
            else:
                B.bin_sort(cc, fr)
            B.render(cc, fr)
        graphs.append(g)
    for rnd in range(3):
        for v, (g, o) in enumerate(zip(graphs, oracle)):
            # the program's own eager work between the replays
            fr.keys.fill_(-1); fr.vals.fill_(-1); fr.out_rgb.fill_(7.0); fr.tile_offsets.fill_(-1)
            torch.cuda.synchronize()
            g.replay()
            torch.cuda.synchronize()
            if static_stage2:
                D, status = (int(x) for x in count_status.cpu())
            else:
                D, status = B.read_status(fr)
            assert D == o.binned.D and status == B.OK, (rnd, v)
            P.compare_binned(fr, o.binned)
            P.compare_image(fr, o.img, cams[v])


def test_gradient_calls_recorded_and_replayed():
    sc = _scene()
    cam = dict(scenes.make_cameras(1, 320, 200)[0], binning=1)
    dev = B.Scene(sc)
    o = ref.render_frame(sc, cam)
    fr = B.Frame(dev.n, 320, 200, o.binned.D + 16)
    cc = B.make_camera(cam)
    B.render_frame(dev, cc, fr)
    gen = torch.Generator(device="cuda"); gen.manual_seed(5)
    g_rgb = torch.randn(3, 200, 320, device="cuda", generator=gen)
    g_T = torch.randn(200, 320, device="cuda", generator=gen)
    g_feat = torch.empty(dev.n, B.FEAT_STRIDE, dtype=torch.float32, device="cuda")
    grads = B.SceneGrads(dev)
    B.render_backward(cc, fr, g_rgb, g_T, g_feat)
    B.preprocess_backward(dev, cc, fr, g_feat, grads)
    torch.cuda.synchronize()
    eager = {k: getattr(grads, k).clone() for k in ("mean", "scale", "rot", "opacity", "sh")}
    eager_feat = g_feat.clone()
    g = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    with torch.cuda.graph(g, stream=side):
        B.render_backward(cc, fr, g_rgb, g_T, g_feat)
        B.preprocess_backward(dev, cc, fr, g_feat, grads)
    for rnd in range(3):
        g_feat.fill_(3.0)
        for k in eager:
            getattr(grads, k).fill_(9.0)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        # the float atomics of the gradient kernel add in no fixed order: equal up to fp32 rounding of the sums
        scale = float(eager_feat.abs().max())
        assert float((g_feat - eager_feat).abs().max()) <= 1e-4 * scale, rnd
        for k, e in eager.items():
            got = getattr(grads, k)
            assert float((got - e).abs().max()) <= 1e-4 * max(float(e.abs().max()), 1e-20), (rnd, k)
