"""GPU parity of lmk_gs_anchor_decode (AnchorDecoder, Sec. 3.1 / Sec. 4.2.1) against the float64
oracle, element by element, within the float32 evaluation error bound the oracle states.

Tolerances (u = 2^-24).  The raw output y of a perceptron carries at most B = oracle bound():
(n1 + n2 + 8) u (|W2|(|W1||x| + |b1|) + |b2|).  The activations are 1-Lipschitz (tanh) or
1/4-Lipschitz (logistic) and are evaluated with the hardware exp and reciprocal (a few u each,
16 u allowed); so opacity <= B + 16u, colour <= B/4 + 16u, and their images under the exact
scalings (x extent, (c - 0.5) / Y_00) scale alike.  The kept/not kept decision must agree wherever
|y| > B; inside that band either answer is valid (the opacity is below B either way).  Centres are
one fused multiply-add: 2u (|position| + |offset x reach|).
"""
import numpy as np
import pytest
import torch

from oracle import anchor_ref as AR
from oracle import ref
from paper_2503_21364_amd import binding as B
from paper_2503_21364_amd import scenes

pytestmark = pytest.mark.gpu

U = 2.0 ** -24


def _run(anchors, mlp, cam_pos, visible=None):
    dev = B.AnchorScene(anchors, mlp)
    v = anchors["a"] if visible is None else len(visible)
    out = B.DecodedScene(v, anchors["k"])
    for t in (out.mean, out.scale, out.rot, out.opacity, out.sh):
        t.fill_(float("nan"))                      # every slot must be written
    vis = None if visible is None else torch.from_numpy(np.asarray(visible, np.int64).astype(np.uint32).view(np.int32)).cuda()
    B.anchor_decode(dev, cam_pos, out, vis)
    torch.cuda.synchronize()
    return out


def _compare(out, anchors, mlp, cam_pos, visible=None, skip_slots=None):
    want = AR.decode(anchors, mlp, cam_pos, visible)
    bnd = AR.bound(anchors, mlp, cam_pos, visible)
    n, k = want.n, want.k
    assert out.n == n
    keep = np.ones(n, bool)
    if skip_slots is not None:
        keep[skip_slots] = False
    got = lambda t: t.cpu().numpy().astype(np.float64)
    idx = np.arange(anchors["a"]) if visible is None else np.asarray(visible)
    worst = {}

    def check(name, g, w, tol):
        g, w, tol = g[..., keep], w[..., keep], tol[..., keep]
        assert np.isfinite(g).all(), name
        ratio = np.abs(g - w) / tol
        worst[name] = float(ratio.max()) if ratio.size else 0.0
        assert (ratio <= 1.0).all(), (name, worst[name], int((ratio > 1).sum()))

    g_op = got(out.opacity)[:n]
    check("opacity", g_op, want.opacity, bnd.opacity + 16 * U)
    decided = keep & (np.abs(want.pre_opacity) > bnd.opacity)
    assert ((g_op > 0) == (want.opacity > 0))[decided].all()
    assert decided.sum() > 0.99 * keep.sum() or n < 1000
    sh = got(out.sh)[:n]
    check("sh", sh[:, :3].T, want.sh_dc, (bnd.colour / 4 + 16 * U) / AR.Y00)
    assert (sh[keep, 3] == 0).all()
    ext = np.repeat(np.asarray(anchors["extent"], np.float64)[:, idx], k, axis=1)
    check("scale", got(out.scale)[:, :n], want.scale, ext[3:6] * (bnd.cov[0:3] / 4 + 16 * U))
    check("rot", got(out.rot)[:, :n], want.rot, bnd.cov[3:7] + 1e-30)
    pos = np.repeat(np.asarray(anchors["position"], np.float64)[:, idx], k, axis=1)
    check("mean", got(out.mean)[:, :n], want.mean, 2 * U * (np.abs(pos) + np.abs(want.mean - pos)) + 1e-30)
    print(f"[anchor parity] n={n} error/tolerance: " + " ".join(f"{a}={b:.3f}" for a, b in worst.items()), flush=True)
    return want


@pytest.mark.parametrize("a,k", [(3000, 10), (257, 10), (64, 10), (1, 10), (1500, 4)])
def test_every_anchor_decoded_matches_the_oracle(a, k):
    anchors = scenes.make_anchor_scene(a, seed=100 + a, k=k)
    mlp = scenes.make_decoder(seed=200 + a, k=k)
    cam = (0.3, -0.2, 4.0)
    out = _run(anchors, mlp, cam)
    _compare(out, anchors, mlp, cam)


def test_larger_weights_still_within_the_bound():
    anchors = scenes.make_anchor_scene(2000, seed=7)
    mlp = scenes.make_decoder(seed=8, scale=3.0)
    cam = (-1.5, 0.4, 2.5)
    out = _run(anchors, mlp, cam)
    _compare(out, anchors, mlp, cam)


def test_a_list_of_anchors_with_repeats_and_a_ragged_length():
    a = 5000
    anchors = scenes.make_anchor_scene(a, seed=31)
    mlp = scenes.make_decoder(seed=32)
    rng = np.random.default_rng(33)
    visible = rng.integers(0, a, size=777)
    visible[5] = visible[4]
    visible[-1] = a - 1
    cam = (0.0, 0.5, 3.0)
    out = _run(anchors, mlp, cam, visible)
    _compare(out, anchors, mlp, cam, visible)


def test_an_index_beyond_the_scene_decodes_to_nothing():
    a, k = 300, 10
    anchors = scenes.make_anchor_scene(a, seed=41)
    mlp = scenes.make_decoder(seed=42)
    visible = np.array([3, a, 7, 2 ** 32 - 1, 299, a + 5, 0], dtype=np.int64)
    cam = (0.0, 0.0, 4.0)
    out = _run(anchors, mlp, cam, visible)
    bad = np.flatnonzero(visible >= a)
    bad_slots = (bad[:, None] * k + np.arange(k)[None, :]).reshape(-1)
    ok = np.where(visible < a, visible, 0)
    _compare(out, anchors, mlp, cam, ok, skip_slots=bad_slots)
    for t in (out.mean, out.scale, out.rot):
        assert (t.cpu().numpy()[:, bad_slots] == 0).all()
    assert (out.opacity.cpu().numpy()[bad_slots] == 0).all()
    assert (out.sh.cpu().numpy()[bad_slots] == 0).all()


def test_an_anchor_at_the_camera_has_no_view_direction():
    anchors = scenes.make_anchor_scene(130, seed=51)
    mlp = scenes.make_decoder(seed=52)
    cam = tuple(float(x) for x in anchors["position"][:, 77])
    out = _run(anchors, mlp, cam)
    _compare(out, anchors, mlp, cam)


def test_saturated_activations_and_large_outputs():
    # weights ten times larger: raw outputs of tens, tanh and the logistic function at their limits
    anchors = scenes.make_anchor_scene(1000, seed=55)
    mlp = scenes.make_decoder(seed=56, scale=10.0)
    cam = (0.1, 0.2, 3.0)
    out = _run(anchors, mlp, cam)
    want = _compare(out, anchors, mlp, cam)
    assert np.abs(want.pre_opacity).max() > 50 and (want.opacity > 0.999999).any()
    assert (want.colour < 1e-6).any() and (want.colour > 1 - 1e-6).any()


def test_non_finite_anchors_stay_confined_and_render():
    """Anchors with NaN / infinite features, extents or centres: what they decode to is not defined,
    but every other anchor's slots are unaffected and the rasteriser takes the result and returns a
    finite image."""
    a, k = 2000, 10
    anchors = scenes.make_anchor_scene(a, seed=57)
    mlp = scenes.make_decoder(seed=58)
    bad = np.array([0, 31, 32, 500, 1023, 1999])
    anchors["feature"][bad[0], 3] = np.nan
    anchors["feature"][bad[1], :] = np.inf
    anchors["feature"][bad[2], 17] = -np.inf
    anchors["extent"][4, bad[3]] = np.nan
    anchors["position"][1, bad[4]] = np.inf
    anchors["offsets"][bad[5], 2, 0] = np.nan
    cam = dict(scenes.make_cameras(0)[0], binning=1)
    out = _run(anchors, mlp, cam["cam_pos"])
    bad_slots = (bad[:, None] * k + np.arange(k)[None, :]).reshape(-1)
    clean = {key: (np.nan_to_num(val, nan=0.0, posinf=0.0, neginf=0.0) if isinstance(val, np.ndarray) else val)
             for key, val in anchors.items()}
    with np.errstate(all="ignore"):
        _compare(out, clean, mlp, cam["cam_pos"], skip_slots=bad_slots)
    scene = out.scene()
    fr = B.Frame(scene.n, cam["width"], cam["height"], 2_000_000)
    B.render_frame(scene, B.make_camera(cam), fr)
    torch.cuda.synchronize()
    d, status = B.read_status(fr)
    assert status == B.OK and d > 1000
    img = fr.out_rgb.cpu().numpy()
    assert np.isfinite(img).all() and np.isfinite(fr.out_T.cpu().numpy()).all()


def test_nothing_listed_is_a_no_op():
    anchors = scenes.make_anchor_scene(10, seed=61)
    mlp = scenes.make_decoder(seed=62)
    dev = B.AnchorScene(anchors, mlp)
    out = B.DecodedScene(0, 10)
    out.opacity.fill_(5.0)
    B.anchor_decode(dev, (0.0, 0.0, 4.0), out, None, v=0)
    torch.cuda.synchronize()
    assert float(out.opacity[0]) == 5.0


def test_calls_on_a_side_stream_and_repeated_are_identical():
    anchors = scenes.make_anchor_scene(4000, seed=71)
    mlp = scenes.make_decoder(seed=72)
    dev = B.AnchorScene(anchors, mlp)
    cam = (0.2, 0.1, 3.5)
    first = B.DecodedScene(4000, 10)
    B.anchor_decode(dev, cam, first)
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    second = B.DecodedScene(4000, 10)
    with torch.cuda.stream(side):
        B.anchor_decode(dev, cam, second, stream=side)
        B.anchor_decode(dev, cam, second, stream=side)
    side.synchronize()
    for name in ("mean", "scale", "rot", "opacity", "sh"):
        assert torch.equal(getattr(first, name), getattr(second, name)), name


def test_decoded_primitives_render_like_the_oracles():
    """Chained: decode -> preprocess -> bin_sort -> render on the GPU against the oracle's decode
    (rounded to float32) through the oracle rasteriser.  The two rasterisers get inputs that differ
    in the last bits, so keys and threshold decisions may differ and the image bound of the
    rasteriser's own parity tests does not apply; this checks that the decoder's output is
    consumed as laid out: mean error tiny, almost every pixel within 1e-4."""
    a, k = 4000, 10
    anchors = scenes.make_anchor_scene(a, seed=81)
    mlp = scenes.make_decoder(seed=82)
    cam = dict(scenes.make_cameras(0)[0], binning=1)
    out = _run(anchors, mlp, cam["cam_pos"])
    scene = out.scene()
    cc = B.make_camera(cam)
    fr = B.Frame(scene.n, cam["width"], cam["height"], 2_000_000)
    B.render_frame(scene, cc, fr)
    torch.cuda.synchronize()
    d, status = B.read_status(fr)
    assert status == B.OK and d > 10_000
    want = ref.render_frame(AR.as_scene(AR.decode(anchors, mlp, cam["cam_pos"])), cam)
    got = fr.out_rgb.cpu().numpy().astype(np.float64)
    err = np.abs(got - want.img.rgb)
    print(f"[anchor chain] D={d} mean |err| {err.mean():.2e} max {err.max():.2e} "
          f"pixels over 1e-4: {(err.max(axis=0) > 1e-4).mean():.2e}", flush=True)
    assert err.mean() < 1e-6
    assert (err.max(axis=0) > 1e-4).mean() < 1e-3
    assert err.max() < 5e-3                        # one flipped 1/255 threshold moves a pixel by up to 4e-3
    assert want.img.rgb.max() > 0.2                     # the image is not empty


def test_full_size_cluster_scene_matches_the_oracle():
    """300 k anchors of the cluster layout (3 M candidate primitives, the size of config 2), every
    slot compared."""
    a = 300_000
    anchors = scenes.make_anchor_scene(a, seed=6000, layout="clusters")
    mlp = scenes.make_decoder(seed=7000)
    cam = scenes.make_cameras(2)[1]["cam_pos"]
    out = _run(anchors, mlp, cam)
    want = _compare(out, anchors, mlp, cam)
    assert 0.3 < (want.opacity > 0).mean() < 0.7


def _culled_run(anchors, mlp, cam):
    dev = B.AnchorScene(anchors, mlp)
    index = B.AnchorIndex(anchors)
    out = B.DecodedScene(anchors["a"], anchors["k"])
    out.opacity.fill_(float("nan"))                 # every slot's opacity must be written
    B.anchor_decode_culled(dev, index, B.make_camera(cam), out)
    torch.cuda.synchronize()
    return dev, index, out


@pytest.mark.parametrize("a,k,view,layout", [(20_000, 10, 4, "clusters"), (20_000, 10, 5, "clusters"),
                                             (20_000, 10, 7, "clusters"), (3001, 4, 5, "clusters"),
                                             (2000, 10, 0, "cube")])
def test_culled_decode_mask_and_slots_match_the_oracle(a, k, view, layout):
    anchors = scenes.make_anchor_scene(a, seed=300 + view, k=k, layout=layout)
    mlp = scenes.make_decoder(seed=301, k=k)
    cam = scenes.make_cameras(2, 480, 270)[view] if layout == "clusters" else scenes.make_cameras(0)[0]
    _, index, out = _culled_run(anchors, mlp, cam)
    vis = AR.anchors_visible(anchors, cam)
    got = index.visible.cpu().numpy()[:a].astype(bool)
    assert np.array_equal(got, vis)                                           # the decision is unique
    if layout == "clusters":
        assert 0.01 < vis.mean() < 0.99
    hidden_slots = np.flatnonzero(np.repeat(~vis, k))
    _compare(out, anchors, mlp, cam["cam_pos"], skip_slots=hidden_slots)      # the anchors in view, as without a mask
    assert (out.opacity.cpu().numpy()[hidden_slots] == 0).all()


def test_culled_decode_with_nothing_in_view():
    anchors = scenes.make_anchor_scene(700, seed=310)
    mlp = scenes.make_decoder(seed=311)
    cam = dict(scenes.make_cameras(0)[0])
    view = np.asarray(cam["view"], np.float32).reshape(3, 4).copy()
    view[2, 3] -= 100.0                                                       # everything far behind the camera
    cam["view"] = view
    _, index, out = _culled_run(anchors, mlp, cam)
    assert not AR.anchors_visible(anchors, cam).any()
    assert (index.visible.cpu().numpy()[:700] == 0).all()
    assert (out.opacity.cpu().numpy() == 0).all()


@pytest.mark.parametrize("view", [4, 7])
def test_culled_pipeline_renders_like_the_oracles(view):
    """Masked decode -> lmk_gs_preprocess_culled over the anchors' boxes -> bin_sort -> render against the
    oracle's masked decode through the oracle rasteriser (same loose image bound as the unmasked chain)."""
    a, k = 30_000, 10
    anchors = scenes.make_anchor_scene(a, seed=320, layout="clusters")
    mlp = scenes.make_decoder(seed=321)
    cam = dict(scenes.make_cameras(2, 480, 270)[view], binning=1)
    _, index, out = _culled_run(anchors, mlp, cam)
    scene = out.scene()
    cc = B.make_camera(cam)
    fr = B.Frame(scene.n, cam["width"], cam["height"], 4_000_000)
    B.preprocess(scene, cc, fr, index=index)
    B.bin_sort(cc, fr)
    B.render(cc, fr)
    torch.cuda.synchronize()
    d, status = B.read_status(fr)
    want = ref.render_frame(AR.as_scene(AR.decode_culled(anchors, mlp, cam)), cam)
    assert status == B.OK and d == want.binned.D and d > 10_000
    # the primitives binned are the same ones
    tt = fr.tiles_touched.cpu().numpy()[:scene.n]
    assert np.array_equal(tt > 0, want.pre.tiles_touched > 0)
    err = np.abs(fr.out_rgb.cpu().numpy().astype(np.float64) - want.img.rgb)
    print(f"[anchor culled chain] view {view}: D={d} mean |err| {err.mean():.2e} max {err.max():.2e}", flush=True)
    assert err.mean() < 1e-6 and (err.max(axis=0) > 1e-4).mean() < 1e-3 and err.max() < 5e-3


def test_full_size_masked_decode_on_every_benchmark_view():
    """The configuration bench.py --anchors 300000 times: 300 k cluster anchors in voxel order (the order
    comes from the oracle's index builder here), the eight views of config 2 at 1080p.  Per view: the mask
    bit for bit, opacity 0 for every slot out of view, and the slots in view against the oracle on the
    two views with the fewest anchors in view (the others decode what the unmasked full-size test covers)."""
    a, k = 300_000, 10
    anchors = scenes.make_anchor_scene(a, seed=6000, layout="clusters")
    perm = ref.build_voxel_index(dict(mean=anchors["position"], scale=anchors["extent"][3:6], n=a), 2.0).perm
    anchors = dict(anchors, position=np.ascontiguousarray(anchors["position"][:, perm]),
                   feature=np.ascontiguousarray(anchors["feature"][perm]),
                   extent=np.ascontiguousarray(anchors["extent"][:, perm]),
                   offsets=np.ascontiguousarray(anchors["offsets"][perm]))
    mlp = scenes.make_decoder(seed=7000)
    dev = B.AnchorScene(anchors, mlp)
    index = B.AnchorIndex(anchors)
    out = B.DecodedScene(a, k)
    fractions = []
    for view, cam in enumerate(scenes.make_cameras(2)):
        out.opacity.fill_(float("nan"))
        B.anchor_decode_culled(dev, index, B.make_camera(cam), out)
        torch.cuda.synchronize()
        vis = AR.anchors_visible(anchors, cam)
        assert np.array_equal(index.visible.cpu().numpy()[:a].astype(bool), vis), view
        hidden = np.flatnonzero(np.repeat(~vis, k))
        op = out.opacity.cpu().numpy()
        assert (op[hidden] == 0).all() and np.isfinite(op).all(), view
        fractions.append(vis.mean())
        if view in (5, 6):
            _compare(out, anchors, mlp, cam["cam_pos"], skip_slots=hidden)
    print("[anchor masks] in view:", " ".join(f"{x:.3f}" for x in fractions), flush=True)
    assert min(fractions) < 0.1 and max(fractions) > 0.9
