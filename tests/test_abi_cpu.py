"""No-GPU checks of the C-ABI library: it loads, exports every symbol the header
declares, and rejects bad arguments on the host before any HIP call."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from paper_2503_21364_amd import binding as B
from paper_2503_21364_amd import scenes

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    names = set()
    inc = os.path.join(ROOT, "include")
    for fn in os.listdir(inc):
        if fn.endswith(".h"):
            text = open(os.path.join(inc, fn)).read()
            text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
            names |= set(re.findall(r"\b(lmk_gs_[a-z_0-9]+)\s*\(", text))
    return names


def test_library_exports_every_declared_symbol():
    lib = B.lib()
    declared = _declared_symbols()
    assert declared == set(B.EXPORTS)
    for name in declared:
        assert getattr(lib, name) is not None
    assert lib.lmk_gs_version() >= 100


def test_struct_layouts_match_the_header():
    # plain 4- and 8-byte fields in declaration order, no padding surprises
    assert C.sizeof(B.Camera) == 4 * (12 + 3 + 4 + 3 + 2 + 3 + 1)
    assert C.sizeof(B.Gaussians) == 5 * 8 + 2 * 4 + 8 and B.Gaussians.cov3d.offset == 48
    assert C.sizeof(B.Projected) == 5 * 8
    assert C.sizeof(B.GaussianGrads) == 5 * 8
    assert C.sizeof(B.Binned) == 7 * 8
    assert B.Binned.capacity.offset == 32 and B.Binned.tile_offsets.offset == 40


def test_strerror_covers_all_codes():
    seen = {B.strerror(c) for c in (0, -1, -2, -3, -4)}
    assert len(seen) == 5 and "ok" in seen
    assert B.strerror(-99) == "unknown error code"


def test_workspace_bytes_grows_with_inputs_and_rejects_bad_sizes():
    a = B.workspace_bytes(1000, 640, 480, 10_000)
    b = B.workspace_bytes(100_000, 640, 480, 10_000)
    c = B.workspace_bytes(100_000, 640, 480, 10_000_000)
    assert 0 < a < b < c and a % 256 == 0
    out = C.c_size_t(0)
    assert B.lib().lmk_gs_workspace_bytes(10, 0, 480, 10, C.byref(out)) == B.ERR_INVALID
    assert B.lib().lmk_gs_workspace_bytes(10, 640, 480, 10, None) == B.ERR_INVALID
    assert B.lib().lmk_gs_workspace_bytes(10, 1 << 20, 480, 10, C.byref(out)) == B.ERR_UNSUPPORTED


def _good_camera():
    return B.make_camera(scenes.make_cameras(0)[0])


def _fake(ptr=0x1000):
    return C.c_void_p(ptr)


def _args():
    """Argument set that passes validation up to the pointer checks; pointers are
    fake non-NULL values, so every test below must fail validation before launch."""
    g = B.Gaussians(0x1000, 0x1000, 0x1000, 0x1000, 0x1000, 10, 3)
    proj = B.Projected(0x1000, 0x1000, 0x1000, 0x1000, None)
    binned = B.Binned(0x1000, 0x1000, 0x1000, 0x1000, 100, 0x1000, None)
    return g, proj, binned


def test_preprocess_rejects_bad_arguments_without_touching_the_gpu():
    lib = B.lib()
    g, proj, _ = _args()
    cam = _good_camera()
    scratch = C.c_void_p(0x10000)
    call = lambda g_, c_, p_, s_=scratch, sb=1 << 20: lib.lmk_gs_preprocess(
        None if g_ is None else C.byref(g_), None if c_ is None else C.byref(c_),
        None if p_ is None else C.byref(p_), s_, sb, None)
    assert call(None, cam, proj) == B.ERR_INVALID
    assert call(g, None, proj) == B.ERR_INVALID
    assert call(g, cam, None) == B.ERR_INVALID
    assert call(g, cam, proj, None) == B.ERR_INVALID
    assert call(g, cam, proj, C.c_void_p(0x10010)) == B.ERR_INVALID        # scratch not 256-aligned
    assert call(g, cam, proj, scratch, 16) == B.ERR_CAPACITY                # scratch too small
    bad = _good_camera(); bad.tile = 8
    assert call(g, bad, proj) == B.ERR_UNSUPPORTED
    bad = _good_camera(); bad.width = 0
    assert call(g, bad, proj) == B.ERR_INVALID
    bad = _good_camera(); bad.fx = float("nan")
    assert call(g, bad, proj) == B.ERR_INVALID
    bad = _good_camera(); bad.view[5] = float("inf")
    assert call(g, bad, proj) == B.ERR_INVALID
    bad = _good_camera(); bad.near_z = 0.0
    assert call(g, bad, proj) == B.ERR_INVALID
    bad = _good_camera(); bad.binning = 2
    assert call(g, bad, proj) == B.ERR_INVALID
    g2, _, _ = _args(); g2.sh_degree = 4
    assert call(g2, cam, proj) == B.ERR_INVALID
    g2, _, _ = _args(); g2.sh = None
    assert call(g2, cam, proj) == B.ERR_INVALID
    p2 = B.Projected(0x1000, 0x1000, 0x1000, None, None)
    assert call(g, cam, p2) == B.ERR_INVALID
    p2 = B.Projected(0x1000, 0x1000, 0x1000, 0x1004, None)                 # feat not 16-byte aligned
    assert call(g, cam, p2) == B.ERR_INVALID


def test_bin_sort_and_render_reject_bad_arguments():
    lib = B.lib()
    _, proj, binned = _args()
    cam = _good_camera()
    scratch = C.c_void_p(0x10000)
    need = B.workspace_bytes(10, cam.width, cam.height, 100)
    bs = lambda p_, c_, b_, s_=scratch, sb=need: lib.lmk_gs_bin_sort(
        None if p_ is None else C.byref(p_), 10, None if c_ is None else C.byref(c_),
        None if b_ is None else C.byref(b_), s_, sb, None)
    assert bs(None, cam, binned) == B.ERR_INVALID
    assert bs(proj, None, binned) == B.ERR_INVALID
    assert bs(proj, cam, None) == B.ERR_INVALID
    assert bs(proj, cam, binned, None) == B.ERR_INVALID
    assert bs(proj, cam, binned, scratch, need - 256) == B.ERR_CAPACITY
    b2 = B.Binned(0x1000, 0x1000, None, 0x1000, 100, 0x1000, None)
    assert bs(proj, cam, b2) == B.ERR_INVALID
    b2 = B.Binned(0x1000, 0x1000, 0x1000, 0x1000, 100, None, None)
    assert bs(proj, cam, b2) == B.ERR_INVALID
    rd = lambda p_, b_, c_, o1=_fake(), o2=_fake(): lib.lmk_gs_render(
        None if p_ is None else C.byref(p_), None if b_ is None else C.byref(b_),
        None if c_ is None else C.byref(c_), o1, o2, None)
    assert rd(None, binned, cam) == B.ERR_INVALID
    assert rd(proj, None, cam) == B.ERR_INVALID
    assert rd(proj, binned, None) == B.ERR_INVALID
    assert rd(proj, binned, cam, None) == B.ERR_INVALID
    assert rd(proj, binned, cam, _fake(), None) == B.ERR_INVALID
    bad = _good_camera(); bad.tile = 32
    assert rd(proj, binned, bad) == B.ERR_UNSUPPORTED
    assert lib.lmk_gs_read_status(None, None, None, None) == B.ERR_INVALID
    # the gradient call checks its arguments the same way, before any HIP call
    rb = lambda p_, b_, c_, g1=_fake(), g2=_fake(), out=_fake(): lib.lmk_gs_render_backward(
        None if p_ is None else C.byref(p_), 100, None if b_ is None else C.byref(b_),
        None if c_ is None else C.byref(c_), g1, g2, out, None)
    assert rb(None, binned, cam) == B.ERR_INVALID
    assert rb(proj, None, cam) == B.ERR_INVALID
    assert rb(proj, binned, None) == B.ERR_INVALID
    assert rb(proj, binned, cam, None) == B.ERR_INVALID          # dL/d rgb is required, dL/dT is not
    assert rb(proj, binned, cam, _fake(), None, None) == B.ERR_INVALID
    assert rb(proj, binned, cam, _fake(), None, 0x1004) == B.ERR_INVALID   # grad_feat must be 16-byte aligned
    assert rb(proj, binned, bad) == B.ERR_UNSUPPORTED


def test_bin_sort_static_rejects_bad_arguments_and_sizes_beyond_its_array():
    lib = B.lib()
    _, proj, binned = _args()
    cam = _good_camera()
    bs = lambda p_, n_, c_, b_, cs=None: lib.lmk_gs_bin_sort_static(
        None if p_ is None else C.byref(p_), n_, None if c_ is None else C.byref(c_),
        None if b_ is None else C.byref(b_), cs, None)
    assert bs(None, 10, cam, binned) == B.ERR_INVALID
    assert bs(proj, 10, None, binned) == B.ERR_INVALID
    assert bs(proj, 10, cam, None) == B.ERR_INVALID
    assert bs(proj, 10, cam, binned, 0x1004) == B.ERR_INVALID          # count_status must be 8-byte aligned
    b2 = B.Binned(0x1000, 0x1000, None, 0x1000, 100, 0x1000, None)
    assert bs(proj, 10, cam, b2) == B.ERR_INVALID
    # beyond the fixed array: refused before anything touches the GPU
    assert bs(proj, B.STATIC_MAX_N + 1, cam, binned) == B.ERR_CAPACITY
    b3 = B.Binned(0x1000, 0x1000, 0x1000, 0x1000, B.STATIC_MAX_CAPACITY + 1, 0x1000, None)
    assert bs(proj, 10, cam, b3) == B.ERR_CAPACITY
    big = _good_camera(); big.width, big.height = 16 * 200, 16 * 100       # 20000 tiles
    assert bs(proj, 10, big, binned) == B.ERR_CAPACITY
    # the limits fit the array: the workspace of the largest accepted call is below 96 MiB
    assert B.workspace_bytes(B.STATIC_MAX_N, 2048, 2048, B.STATIC_MAX_CAPACITY) <= 96 << 20


def test_preprocess_backward_rejects_bad_arguments():
    lib = B.lib()
    g, proj, _ = _args()
    cam = _good_camera()
    grads = B.GaussianGrads(0x1000, 0x2000, 0x3000, 0x4000, 0x5000)
    call = lambda g_, c_, p_, gf=C.c_void_p(0x6000), o_=grads: lib.lmk_gs_preprocess_backward(
        None if g_ is None else C.byref(g_), None if c_ is None else C.byref(c_),
        None if p_ is None else C.byref(p_), gf, None if o_ is None else C.byref(o_), None)
    assert call(None, cam, proj) == B.ERR_INVALID
    assert call(g, None, proj) == B.ERR_INVALID
    assert call(g, cam, None) == B.ERR_INVALID
    assert call(g, cam, proj, None) == B.ERR_INVALID
    assert call(g, cam, proj, C.c_void_p(0x6004)) == B.ERR_INVALID          # grad_feat must be 16-byte aligned
    assert call(g, cam, proj, C.c_void_p(0x6000), None) == B.ERR_INVALID
    assert call(g, cam, proj, C.c_void_p(0x6000), B.GaussianGrads(0x1000, 0x2000, None, 0x4000, 0x5000)) == B.ERR_INVALID
    g2, _, _ = _args(); g2.rot = None                                        # the cache alone is not enough here
    assert call(g2, cam, proj) == B.ERR_INVALID
    bad = _good_camera(); bad.tile = 8
    assert call(g, bad, proj) == B.ERR_UNSUPPORTED


def test_anchor_decode_rejects_bad_arguments():
    lib = B.lib()
    assert C.sizeof(B.Anchors) == 4 * 8 + 2 * 4 and C.sizeof(B.Perceptron) == 4 * 8
    assert C.sizeof(B.AnchorDecoder) == 3 * C.sizeof(B.Perceptron) and C.sizeof(B.Decoded) == 5 * 8
    an = lambda **kw: B.Anchors(**{**dict(position=0x1000, feature=0x2000, extent=0x3000, offsets=0x4000, a=100, k=10), **kw})
    net = lambda **kw: B.Perceptron(**{**dict(w1=0x5000, b1=0x5100, w2t=0x5200, b2=0x5300), **kw})
    dec = lambda **kw: B.AnchorDecoder(**{**dict(opacity=net(), colour=net(), cov=net()), **kw})
    out = lambda **kw: B.Decoded(**{**dict(mean=0x6000, scale=0x7000, rot=0x8000, opacity=0x9000, sh=0xa000), **kw})
    cam = (C.c_float * 3)(0.0, 0.0, 4.0)

    def call(a_=an(), d_=dec(), c_=cam, vis=C.c_void_p(0xb000), v=50, o_=out()):
        return lib.lmk_gs_anchor_decode(None if a_ is None else C.byref(a_), None if d_ is None else C.byref(d_),
                                        c_, vis, C.c_uint32(v), None if o_ is None else C.byref(o_), None)
    assert call(a_=None) == B.ERR_INVALID
    assert call(d_=None) == B.ERR_INVALID
    assert call(c_=None) == B.ERR_INVALID
    assert call(o_=None) == B.ERR_INVALID
    assert call(a_=an(k=7)) == B.ERR_UNSUPPORTED
    assert call(a_=an(feature=None)) == B.ERR_INVALID
    assert call(a_=an(feature=0x2004)) == B.ERR_INVALID                      # records are 16-byte aligned
    assert call(a_=an(offsets=0x4004)) == B.ERR_INVALID
    assert call(d_=dec(colour=net(w2t=None))) == B.ERR_INVALID
    assert call(d_=dec(cov=net(b1=None))) == B.ERR_INVALID
    assert call(o_=out(rot=None)) == B.ERR_INVALID
    assert call(o_=out(sh=0xa008)) == B.ERR_INVALID
    assert call(vis=None, v=101) == B.ERR_INVALID                            # no list: at most all anchors
    assert call(v=(1 << 32) // 10 + 1) == B.ERR_INVALID                      # v * k must fit 32 bits
    assert call(c_=(C.c_float * 3)(0.0, float("nan"), 0.0)) == B.ERR_INVALID
    assert call(v=0) == B.OK                                                 # nothing listed: nothing launched
    assert call(v=0, a_=an(a=0, position=None, feature=None, extent=None, offsets=None)) == B.OK


def test_anchor_index_build_matches_the_oracle_and_rejects_bad_input():
    from oracle import anchor_ref as AR
    lib = B.lib()
    for a, k, layout in ((1000, 10, "clusters"), (77, 4, "cube"), (1, 10, "cube")):
        an = scenes.make_anchor_scene(a, seed=5 + a, k=k, layout=layout)
        nb = (a * k + B.PRE_BLOCK - 1) // B.PRE_BLOCK
        box = np.full((a, 8), np.nan, np.float32)
        rng = np.full((nb, 2), 0xFFFFFFFF, np.uint32)
        rc = lib.lmk_gs_anchor_index_build(an["position"].ctypes.data, an["extent"].ctypes.data,
                                           an["offsets"].ctypes.data, a, k, box.ctypes.data, rng.ctypes.data)
        assert rc == B.OK
        want = AR.anchor_boxes(an)
        assert np.array_equal(box[:, 0:3].view(np.uint32), want.box_lo.view(np.uint32))
        assert np.array_equal(box[:, 3:6].view(np.uint32), want.box_hi.view(np.uint32))
        assert np.array_equal(box[:, 6].view(np.uint32), want.smax.view(np.uint32)) and (box[:, 7] == 0).all()
        slots = np.arange(a * k)
        first = (slots // k)[::B.PRE_BLOCK]
        last = np.minimum(slots[::B.PRE_BLOCK] + B.PRE_BLOCK - 1, a * k - 1) // k
        assert np.array_equal(rng[:, 0], first) and np.array_equal(rng[:, 1], last)
    an = scenes.make_anchor_scene(10, seed=1)
    box = np.zeros((10, 8), np.float32); rng = np.zeros((1, 2), np.uint32)
    args = lambda **kw: [kw.get("p", an["position"].ctypes.data), kw.get("e", an["extent"].ctypes.data),
                         kw.get("o", an["offsets"].ctypes.data), kw.get("a", 10), kw.get("k", 10),
                         kw.get("b", box.ctypes.data), kw.get("r", rng.ctypes.data)]
    assert lib.lmk_gs_anchor_index_build(*args()) == B.OK
    assert lib.lmk_gs_anchor_index_build(*args(p=None)) == B.ERR_INVALID
    assert lib.lmk_gs_anchor_index_build(*args(b=None)) == B.ERR_INVALID
    assert lib.lmk_gs_anchor_index_build(*args(r=None)) == B.ERR_INVALID
    assert lib.lmk_gs_anchor_index_build(*args(k=0)) == B.ERR_INVALID
    assert lib.lmk_gs_anchor_index_build(*args(a=1 << 30, k=10)) == B.ERR_INVALID
    assert lib.lmk_gs_anchor_index_build(*args(a=0, p=None, e=None, o=None, b=None, r=None)) == B.OK


def test_anchor_decode_culled_rejects_bad_arguments():
    lib = B.lib()
    an = B.Anchors(position=0x1000, feature=0x2000, extent=0x3000, offsets=0x4000, a=100, k=10)
    net = B.Perceptron(w1=0x5000, b1=0x5100, w2t=0x5200, b2=0x5300)
    dec = B.AnchorDecoder(opacity=net, colour=net, cov=net)
    out = B.Decoded(mean=0x6000, scale=0x7000, rot=0x8000, opacity=0x9000, sh=0xa000)
    cam = _good_camera()

    def call(a_=an, d_=dec, c_=cam, box=C.c_void_p(0xb000), vis=C.c_void_p(0xc000), o_=out):
        return lib.lmk_gs_anchor_decode_culled(None if a_ is None else C.byref(a_), None if d_ is None else C.byref(d_),
                                               None if c_ is None else C.byref(c_), box, vis,
                                               None if o_ is None else C.byref(o_), None)
    assert call(a_=None) == B.ERR_INVALID
    assert call(d_=None) == B.ERR_INVALID
    assert call(c_=None) == B.ERR_INVALID
    assert call(o_=None) == B.ERR_INVALID
    assert call(box=None) == B.ERR_INVALID
    assert call(box=C.c_void_p(0xb008)) == B.ERR_INVALID                     # boxes are read as 16-byte vectors
    assert call(vis=None) == B.ERR_INVALID
    assert call(a_=B.Anchors(position=0x1000, feature=0x2000, extent=0x3000, offsets=0x4000, a=100, k=7)) == B.ERR_UNSUPPORTED
    assert call(a_=B.Anchors(position=0x1000, feature=None, extent=0x3000, offsets=0x4000, a=100, k=10)) == B.ERR_INVALID
    assert call(o_=B.Decoded(mean=0x6000, scale=0x7000, rot=None, opacity=0x9000, sh=0xa000)) == B.ERR_INVALID
    bad = _good_camera(); bad.tile = 8
    assert call(c_=bad) == B.ERR_UNSUPPORTED
    assert call(a_=B.Anchors(position=None, feature=None, extent=None, offsets=None, a=0, k=10), box=None, vis=None) == B.OK


def test_index_build_matches_the_oracle_and_rejects_bad_input():
    from oracle import ref
    for cfg, n, vs in [(2, 50_000, 2.0), (3, 80_000, 40.0), (0, 1000, 0.3), (1, 777, 1.0), (0, 1, 1.0)]:
        sc = scenes.make_scene(cfg, n=n, seed=11 + cfg)
        vi = B.VoxelIndex(sc, vs)
        oi = ref.build_voxel_index(sc, vs)
        assert vi.num_voxels == oi.num_voxels
        np.testing.assert_array_equal(vi.perm, oi.perm)
        np.testing.assert_array_equal(vi.first, oi.first)
        np.testing.assert_array_equal(vi.box[:, 0:3], oi.box_lo)
        np.testing.assert_array_equal(vi.box[:, 3:6], oi.box_hi)
        np.testing.assert_array_equal(vi.box[:, 6], oi.smax)
        # voxel range of every group of PRE_BLOCK primitives, by definition
        vox_of = np.repeat(np.arange(oi.num_voxels), np.diff(oi.first.astype(np.int64)))
        for b in range(len(vi.block_range)):
            a, e = b * B.PRE_BLOCK, min((b + 1) * B.PRE_BLOCK, n) - 1
            assert tuple(vi.block_range[b]) == (vox_of[a], vox_of[e])
    lib = B.lib()
    nv = C.c_uint32(5)
    m = np.zeros((3, 4), np.float32); sc_ = np.ones((3, 4), np.float32)
    perm = np.zeros(4, np.uint32); first = np.zeros(5, np.uint32); box = np.zeros((4, 8), np.float32)
    br = np.zeros((1, 2), np.uint32)
    call = lambda mean=m, vs=1.0, p=perm: lib.lmk_gs_index_build(
        None if mean is None else mean.ctypes.data, sc_.ctypes.data, 4, vs,
        None if p is None else p.ctypes.data, first.ctypes.data, box.ctypes.data, br.ctypes.data, C.byref(nv))
    assert call() == B.OK and nv.value == 1
    assert call(vs=0.0) == B.ERR_INVALID and call(vs=float("nan")) == B.ERR_INVALID
    assert call(mean=None) == B.ERR_INVALID and call(p=None) == B.ERR_INVALID
    bad = m.copy(); bad[1, 2] = np.inf
    assert call(mean=bad) == B.ERR_INVALID
    wide = m.copy(); wide[0, 0] = 1e9
    assert call(mean=wide, vs=1.0) == B.ERR_UNSUPPORTED
    assert lib.lmk_gs_index_build(None, None, 0, 1.0, None, None, None, None, C.byref(nv)) == B.OK and nv.value == 0


def test_parameter_cache_arguments():
    lib = B.lib()
    g, proj, _ = _args()
    assert lib.lmk_gs_build_cov3d(None, C.c_void_p(0x1000), None) == B.ERR_INVALID
    assert lib.lmk_gs_build_cov3d(C.byref(g), None, None) == B.ERR_INVALID
    g2, _, _ = _args(); g2.rot = None
    assert lib.lmk_gs_build_cov3d(C.byref(g2), C.c_void_p(0x1000), None) == B.ERR_INVALID
    # with a cache, preprocess no longer needs rotation and scale; without one it does
    cam = _good_camera()
    call = lambda g_: lib.lmk_gs_preprocess(C.byref(g_), C.byref(cam), C.byref(proj), C.c_void_p(0x10000), 16, None)
    g3, _, _ = _args(); g3.rot = None; g3.scale = None
    assert call(g3) == B.ERR_INVALID
    g3.cov3d = 0x1000
    assert call(g3) == B.ERR_CAPACITY          # passes the pointer checks, stops at the scratch size


def test_preprocess_culled_rejects_bad_arguments():
    lib = B.lib()
    g, proj, _ = _args()
    cam = _good_camera()
    scratch = C.c_void_p(0x10000)
    idx = B.VoxelIndexC(0x1000, 0x1000, 3, None)
    call = lambda i_, c_=cam: lib.lmk_gs_preprocess_culled(
        C.byref(g), None if i_ is None else C.byref(i_), C.byref(c_), C.byref(proj), None, scratch, 1 << 20, None)
    assert C.sizeof(B.VoxelIndexC) == 32 and B.VoxelIndexC.visible.offset == 24
    assert call(None) == B.ERR_INVALID
    assert call(B.VoxelIndexC(None, 0x1000, 3, None)) == B.ERR_INVALID
    assert call(B.VoxelIndexC(0x1000, None, 3, None)) == B.ERR_INVALID
    assert call(B.VoxelIndexC(0x1000, 0x1000, 0, None)) == B.ERR_INVALID
    assert call(B.VoxelIndexC(0x1000, 0x1000, 11, None)) == B.ERR_INVALID          # more voxels than primitives
    assert call(B.VoxelIndexC(0x1008, 0x1000, 3, None)) == B.ERR_INVALID          # box records not 16-byte aligned
    skew = _good_camera(); skew.view[0] *= 1.1
    assert call(idx, skew) == B.ERR_UNSUPPORTED


def test_binding_refuses_to_run_without_the_library(monkeypatch, tmp_path):
    monkeypatch.setattr(B, "_lib", None)
    monkeypatch.setattr(B, "LIB_PATH", str(tmp_path / "absent.so"))
    with pytest.raises(RuntimeError, match="no CPU fallback"):
        B.lib()


def test_scene_generator_shapes_and_determinism():
    a = scenes.make_scene(2, n=1000)
    b = scenes.make_scene(2, n=1000)
    for k in ("mean", "scale", "rot", "opacity", "sh"):
        assert a[k].dtype == np.float32 and np.array_equal(a[k], b[k])
    assert a["sh"].shape == (16, 3, 1000) and a["rot"].shape == (4, 1000)
    assert np.all(a["scale"] > 0) and np.all((a["opacity"] >= 0) & (a["opacity"] <= 1))
    for cfg in range(5):
        cams = scenes.make_cameras(cfg)
        assert len(cams) == scenes.CONFIGS[cfg]["views"]
        for c in cams:
            R = c["view"].reshape(3, 4)[:, :3].astype(np.float64)
            np.testing.assert_allclose(R @ R.T, np.eye(3), atol=1e-6)
            assert np.linalg.det(R) > 0.999          # right-handed: x right, y down, z forward
            np.testing.assert_allclose(R @ c["cam_pos"].astype(np.float64) + c["view"].reshape(3, 4)[:, 3],
                                       0, atol=1e-3)
