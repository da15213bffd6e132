"""ctypes front end of the CPU oracle (oracle/lmk_ref.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by __graft_entry__.smoke() and by
the cpu_baseline leg of bench.py.  Nothing in the product package imports it,
and it imports nothing from the product package.

All arrays are host numpy arrays.  The C file is compiled with gcc on first
use (plain C11 + OpenMP, -O2 -ffp-contract=off) if the library is absent or
older than its source.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from types import SimpleNamespace

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "lmk_ref.c")
_LIB = os.path.join(_HERE, "liblmk_ref.so")

VISIBLE, CULL_NEAR, CULL_DET, CULL_OPACITY, CULL_OFFSCREEN = range(5)


def build(force: bool = False) -> str:
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + f".tmp{os.getpid()}"
        subprocess.check_call(["gcc", "-std=c11", "-O2", "-ffp-contract=off", "-fopenmp", "-fPIC",
                               "-shared", "-Wall", "-Wextra", "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


class RefCamera(C.Structure):
    _fields_ = [("view", C.c_float * 12), ("cam_pos", C.c_float * 3),
                ("fx", C.c_float), ("fy", C.c_float), ("cx", C.c_float), ("cy", C.c_float),
                ("width", C.c_uint32), ("height", C.c_uint32), ("tile", C.c_uint32),
                ("near_z", C.c_float), ("lowpass", C.c_float), ("bg", C.c_float * 3),
                ("binning", C.c_uint32)]


def _camera(cam: dict) -> RefCamera:
    c = RefCamera()
    c.view[:] = [float(x) for x in np.asarray(cam["view"], dtype=np.float32).reshape(12)]
    c.cam_pos[:] = [float(x) for x in np.asarray(cam["cam_pos"], dtype=np.float32)]
    c.fx, c.fy, c.cx, c.cy = (float(np.float32(cam[k])) for k in ("fx", "fy", "cx", "cy"))
    c.width, c.height, c.tile = int(cam["width"]), int(cam["height"]), int(cam["tile"])
    c.near_z, c.lowpass = float(np.float32(cam["near_z"])), float(np.float32(cam["lowpass"]))
    c.bg[:] = [float(x) for x in np.asarray(cam["bg"], dtype=np.float32)]
    c.binning = int(cam.get("binning", 0))
    return c


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.lmk_ref_scan.restype = C.c_uint64
        _lib.lmk_ref_depth_order.restype = C.c_uint32
        _lib.lmk_ref_tile_list.restype = C.c_uint64
        _lib.lmk_ref_trace_pixel.restype = C.c_uint32
        _lib.lmk_ref_opacity_tau.restype = C.c_float
        _lib.lmk_ref_opacity_tau.argtypes = [C.c_float]
        _lib.lmk_ref_tile_kept.restype = C.c_int
        _lib.lmk_ref_tile_kept.argtypes = [C.c_float] * 6 + [C.c_uint32] * 3
    return _lib


def _p(a):
    return a.ctypes.data_as(C.c_void_p)


def _f32(a):
    a = np.ascontiguousarray(a, dtype=np.float32)
    return a


def tiles_xy(cam):
    t = int(cam["tile"])
    return (int(cam["width"]) + t - 1) // t, (int(cam["height"]) + t - 1) // t


def covariance3d(q, s):
    q = _f32(q); s = _f32(s)
    out = np.empty(9, dtype=np.float32)
    lib().lmk_ref_covariance3d(_p(q), _p(s), _p(out))
    return out.reshape(3, 3)


def sh_basis(d):
    d = np.ascontiguousarray(d, dtype=np.float64)
    out = np.empty(16, dtype=np.float64)
    lib().lmk_ref_sh_basis(_p(d), _p(out))
    return out


def preprocess(scene: dict, cam: dict) -> SimpleNamespace:
    """Steps 1-9: per-primitive projection, culls, rectangle, colour."""
    n = int(scene["n"])
    mean, scale, rot = _f32(scene["mean"]), _f32(scene["scale"]), _f32(scene["rot"])
    opacity, sh = _f32(scene["opacity"]), _f32(scene["sh"])
    deg = int(scene["sh_degree"])
    assert mean.shape == (3, n) and scale.shape == (3, n) and rot.shape == (4, n)
    assert sh.shape[0] >= (deg + 1) ** 2 and sh.shape[1:] == (3, n)
    out = SimpleNamespace(
        n=n, stage=np.empty(n, np.uint8), depth=np.empty(n, np.float32),
        mean2d=np.empty((2, n), np.float32), cov2d=np.empty((3, n), np.float32),
        conic=np.empty((3, n), np.float32), rect=np.empty((n, 4), np.uint16),
        tiles_touched=np.empty(n, np.uint32), rgb=np.empty((3, n), np.float64),
        opacity=opacity)
    cc = _camera(cam)
    lib().lmk_ref_preprocess(C.c_uint32(n), _p(mean), _p(scale), _p(rot), _p(opacity), _p(sh),
                             C.c_uint32(deg), C.byref(cc), _p(out.stage), _p(out.depth),
                             _p(out.mean2d), _p(out.cov2d), _p(out.conic), _p(out.rect),
                             _p(out.tiles_touched), _p(out.rgb))
    return out


def bin_sort(pre: SimpleNamespace, cam: dict, keep_unsorted: bool = False) -> SimpleNamespace:
    """Steps 10-13: offsets, (tile|depth) keys, sorted pairs, per-tile ranges."""
    n = pre.n
    tx, ty = tiles_xy(cam)
    offsets = np.empty(n + 1, np.uint64)
    D = int(lib().lmk_ref_scan(C.c_uint32(n), _p(pre.tiles_touched), _p(offsets)))
    keys = np.empty(max(D, 1), np.uint64)
    vals = np.empty(max(D, 1), np.uint32)
    lib().lmk_ref_emit(C.c_uint32(n), _p(pre.tiles_touched), _p(pre.rect), _p(pre.depth),
                       _p(offsets), C.c_uint32(tx), C.c_uint32(int(cam.get("binning", 0))),
                       C.c_uint32(int(cam["tile"])), _p(pre.mean2d), _p(pre.conic), _p(pre.opacity),
                       _p(keys), _p(vals))
    out = SimpleNamespace(D=D, offsets=offsets, tiles_x=tx, tiles_y=ty)
    if keep_unsorted:
        out.keys_unsorted = keys[:D].copy()
        out.vals_unsorted = vals[:D].copy()
    lib().lmk_ref_sort(C.c_uint64(D), _p(keys), _p(vals))
    tile_offsets = np.empty(tx * ty + 1, np.uint64)
    lib().lmk_ref_ranges(C.c_uint64(D), _p(keys), C.c_uint32(tx * ty), _p(tile_offsets))
    out.keys, out.vals, out.tile_offsets = keys[:D], vals[:D], tile_offsets
    return out


def render(pre: SimpleNamespace, binned: SimpleNamespace, cam: dict) -> SimpleNamespace:
    """Step 14 over the whole image through the tile lists."""
    H, W = int(cam["height"]), int(cam["width"])
    out = SimpleNamespace(rgb=np.empty((3, H, W), np.float64), T=np.empty((H, W), np.float64),
                          E=np.empty((H, W), np.uint32), C=np.empty((H, W), np.uint32),
                          beta=np.empty((H, W), np.float64), beta_T=np.empty((H, W), np.float64),
                          amb=np.empty((H, W), np.uint32))
    cc = _camera(cam)
    vals = binned.vals if binned.D else np.zeros(1, np.uint32)
    lib().lmk_ref_render(C.c_uint32(pre.n), _p(pre.stage), _p(pre.mean2d), _p(pre.conic),
                         _p(pre.opacity), _p(pre.rgb), _p(vals), _p(binned.tile_offsets),
                         C.byref(cc), _p(out.rgb), _p(out.T), _p(out.E), _p(out.C),
                         _p(out.beta), _p(out.beta_T), _p(out.amb))
    return out


def render_backward(pre: SimpleNamespace, binned: SimpleNamespace, cam: dict, grad_rgb, grad_T=None) -> SimpleNamespace:
    """Gradient of a loss through the compositing, with respect to every primitive's 2D mean,
    conic, opacity and colour; grad_rgb [3][H][W], grad_T [H][W] or None (fp64).  `abs` [9][n]
    (rows u, v, A, B, C, o, r, g, b): the sums of the magnitudes of the terms."""
    H, W = int(cam["height"]), int(cam["width"])
    n = pre.n
    grad_rgb = np.ascontiguousarray(grad_rgb, dtype=np.float64)
    assert grad_rgb.shape == (3, H, W)
    gT = None if grad_T is None else np.ascontiguousarray(grad_T, dtype=np.float64)
    out = SimpleNamespace(mean2d=np.empty((2, n), np.float64), conic=np.empty((3, n), np.float64),
                          opacity=np.empty(n, np.float64), rgb=np.empty((3, n), np.float64),
                          img_rgb=np.empty((3, H, W), np.float64), img_T=np.empty((H, W), np.float64),
                          amb=np.empty((H, W), np.uint32), abs=np.empty((9, n), np.float64))
    cc = _camera(cam)
    vals = binned.vals if binned.D else np.zeros(1, np.uint32)
    lib().lmk_ref_render_backward(C.c_uint32(n), _p(pre.mean2d), _p(pre.conic), _p(pre.opacity), _p(pre.rgb),
                                  _p(vals), _p(binned.tile_offsets), C.byref(cc), _p(grad_rgb),
                                  _p(gT) if gT is not None else None,
                                  _p(out.mean2d), _p(out.conic), _p(out.opacity), _p(out.rgb),
                                  _p(out.img_rgb), _p(out.img_T), _p(out.amb), _p(out.abs))
    return out


def preprocess_backward(scene: dict, cam: dict, pre: SimpleNamespace, g_feat) -> SimpleNamespace:
    """Gradient through the per-primitive projection: g_feat [9][n] (planes u, v, A, B, C, o, r, g, b)
    -> gradients with respect to mean [3][n], scale [3][n], rot [4][n], opacity [n], sh [k][3][n]."""
    n = scene["n"]
    g_feat = np.ascontiguousarray(g_feat, dtype=np.float64)
    assert g_feat.shape == (9, n)
    sh = _f32(scene["sh"])
    out = SimpleNamespace(mean=np.empty((3, n), np.float64), scale=np.empty((3, n), np.float64),
                          rot=np.empty((4, n), np.float64), opacity=np.empty(n, np.float64),
                          sh=np.zeros(sh.shape, np.float64))      # coefficients beyond the degree stay 0
    cc = _camera(cam)
    mean, scale, rot = _f32(scene["mean"]), _f32(scene["scale"]), _f32(scene["rot"])
    lib().lmk_ref_preprocess_backward(C.c_uint32(n), _p(mean), _p(scale), _p(rot), _p(sh),
                                      C.c_uint32(int(scene.get("sh_degree", 3))), C.byref(cc), _p(pre.stage),
                                      _p(g_feat), _p(out.mean), _p(out.scale), _p(out.rot), _p(out.opacity),
                                      _p(out.sh))
    return out


def depth_order(pre: SimpleNamespace) -> np.ndarray:
    order = np.empty(max(pre.n, 1), np.uint32)
    m = lib().lmk_ref_depth_order(C.c_uint32(pre.n), _p(pre.stage), _p(pre.depth), _p(order))
    return order[:m].copy()


def render_pixels_brute(pre: SimpleNamespace, cam: dict, xs, ys, order=None) -> SimpleNamespace:
    """The image by definition at chosen pixels: every surviving primitive, depth order."""
    if order is None:
        order = depth_order(pre)
    xs = np.ascontiguousarray(xs, dtype=np.uint32)
    ys = np.ascontiguousarray(ys, dtype=np.uint32)
    k = xs.size
    out = SimpleNamespace(rgb=np.empty((k, 3), np.float64), T=np.empty(k, np.float64),
                          C=np.empty(k, np.uint32), beta=np.empty(k, np.float64),
                          beta_T=np.empty(k, np.float64), amb=np.empty(k, np.uint32))
    cc = _camera(cam)
    o = order if order.size else np.zeros(1, np.uint32)
    lib().lmk_ref_render_pixels_brute(C.c_uint32(pre.n), _p(pre.stage), _p(pre.mean2d), _p(pre.conic),
                                      _p(pre.opacity), _p(pre.rgb), _p(o), C.c_uint32(order.size),
                                      C.byref(cc), C.c_uint32(k), _p(xs), _p(ys),
                                      _p(out.rgb), _p(out.T), _p(out.C), _p(out.beta), _p(out.beta_T), _p(out.amb))
    return out


def opacity_tau(o: float) -> float:
    return float(lib().lmk_ref_opacity_tau(float(np.float32(o))))


def tile_kept(u, v, A, B, Cc, o, tx, ty, ts=16) -> bool:
    f = lambda x: float(np.float32(x))
    return bool(lib().lmk_ref_tile_kept(f(u), f(v), f(A), f(B), f(Cc), f(o), int(tx), int(ty), int(ts)))


def tile_list(pre: SimpleNamespace, tile_x: int, tile_y: int, cam: dict | None = None) -> np.ndarray:
    """Sorted primitive list of one tile, straight from the definition (under the
    camera's binning rule; rule 0 when no camera is given)."""
    binning = int(cam.get("binning", 0)) if cam is not None else 0
    ts = int(cam["tile"]) if cam is not None else 16
    cap = 1 << 16
    while True:
        out = np.empty(cap, np.uint32)
        m = int(lib().lmk_ref_tile_list(C.c_uint32(pre.n), _p(pre.tiles_touched), _p(pre.rect),
                                        _p(pre.depth), C.c_uint32(tile_x), C.c_uint32(tile_y),
                                        C.c_uint32(binning), C.c_uint32(ts), _p(pre.mean2d), _p(pre.conic),
                                        _p(pre.opacity), _p(out), C.c_uint64(cap)))
        if m <= cap:
            return out[:m].copy()
        cap = m


def band_lists(pre: SimpleNamespace, cam: dict, ty0: int, ty1: int, order=None) -> SimpleNamespace:
    """Sorted lists of every tile of the tile rows [ty0, ty1) (frames too large to bin whole):
    offsets [(ty1 - ty0) * tiles_x + 1] into vals, lists in tile order."""
    if order is None:
        order = depth_order(pre)
    tx, _ = tiles_xy(cam)
    nt = (ty1 - ty0) * tx
    offsets = np.empty(nt + 1, np.uint64)
    o = order if order.size else np.zeros(1, np.uint32)
    args = lambda vals, cap: (C.c_uint32(pre.n), _p(pre.tiles_touched), _p(pre.rect), _p(o), C.c_uint32(order.size),
                              C.c_uint32(int(cam.get("binning", 0))), C.c_uint32(int(cam["tile"])), C.c_uint32(tx),
                              C.c_uint32(ty0), C.c_uint32(ty1), _p(pre.mean2d), _p(pre.conic), _p(pre.opacity),
                              _p(offsets), _p(vals), C.c_uint64(cap))
    lib().lmk_ref_band_lists.restype = C.c_uint64
    dummy = np.zeros(1, np.uint32)
    m = int(lib().lmk_ref_band_lists(*args(dummy, 0)))          # sizes only
    vals = np.empty(max(m, 1), np.uint32)
    if m:
        lib().lmk_ref_band_lists(*args(vals, m))
    return SimpleNamespace(offsets=offsets, vals=vals[:m], ty0=ty0, ty1=ty1, tiles_x=tx)


def render_band(pre: SimpleNamespace, cam: dict, band: SimpleNamespace) -> SimpleNamespace:
    """Step 14 for the pixel rows of a band through its lists (outputs cover only those rows)."""
    H, W, ts = int(cam["height"]), int(cam["width"]), int(cam["tile"])
    y0, y1 = band.ty0 * ts, min(band.ty1 * ts, H)
    rows = max(y1 - y0, 0)
    out = SimpleNamespace(rgb=np.empty((3, rows, W), np.float64), T=np.empty((rows, W), np.float64),
                          E=np.empty((rows, W), np.uint32), C=np.empty((rows, W), np.uint32),
                          beta=np.empty((rows, W), np.float64), beta_T=np.empty((rows, W), np.float64),
                          amb=np.empty((rows, W), np.uint32), y0=y0, y1=y1)
    cc = _camera(cam)
    vals = band.vals if band.vals.size else np.zeros(1, np.uint32)
    lib().lmk_ref_render_band(C.c_uint32(pre.n), _p(pre.stage), _p(pre.mean2d), _p(pre.conic), _p(pre.opacity),
                              _p(pre.rgb), _p(vals), _p(band.offsets), C.byref(cc), C.c_uint32(band.ty0),
                              C.c_uint32(band.ty1), _p(out.rgb), _p(out.T), _p(out.E), _p(out.C),
                              _p(out.beta), _p(out.beta_T), _p(out.amb))
    return out


def render_pixels_list(pre: SimpleNamespace, cam: dict, lst: np.ndarray, xs, ys) -> SimpleNamespace:
    xs = np.ascontiguousarray(xs, dtype=np.uint32)
    ys = np.ascontiguousarray(ys, dtype=np.uint32)
    k = xs.size
    out = SimpleNamespace(rgb=np.empty((k, 3), np.float64), T=np.empty(k, np.float64),
                          E=np.empty(k, np.uint32), C=np.empty(k, np.uint32),
                          beta=np.empty(k, np.float64), beta_T=np.empty(k, np.float64),
                          amb=np.empty(k, np.uint32))
    cc = _camera(cam)
    l = np.ascontiguousarray(lst, dtype=np.uint32) if len(lst) else np.zeros(1, np.uint32)
    lib().lmk_ref_render_pixels_list(C.c_uint32(pre.n), _p(pre.stage), _p(pre.mean2d), _p(pre.conic),
                                     _p(pre.opacity), _p(pre.rgb), _p(l), C.c_uint64(len(lst)),
                                     C.byref(cc), C.c_uint32(k), _p(xs), _p(ys),
                                     _p(out.rgb), _p(out.T), _p(out.E), _p(out.C),
                                     _p(out.beta), _p(out.beta_T), _p(out.amb))
    return out


def trace_pixel(pre: SimpleNamespace, lst: np.ndarray, x: int, y: int) -> np.ndarray:
    cap = max(len(lst), 1)
    trace = np.empty(cap, np.float64)
    l = np.ascontiguousarray(lst, dtype=np.uint32) if len(lst) else np.zeros(1, np.uint32)
    m = lib().lmk_ref_trace_pixel(C.c_uint32(pre.n), _p(pre.mean2d), _p(pre.conic), _p(pre.opacity),
                                  _p(pre.rgb), _p(l), C.c_uint64(len(lst)), C.c_uint32(x),
                                  C.c_uint32(y), _p(trace), C.c_uint32(cap))
    return trace[:m].copy()


def build_voxel_index(scene: dict, voxel_size: float) -> SimpleNamespace:
    """Offline reordering of the primitives into a voxel grid (Sec. 4.2.2, frustum-based dynamic loading): cell of a primitive =
    floor(mean / voxel_size) per axis (fp32), cells in Morton order, primitives of a cell in their
    original order.  Returns the permutation, the first primitive of every occupied voxel, the
    bounding box of the means and the largest scale component of every voxel."""
    n = int(scene["n"])
    mean = _f32(scene["mean"]); scale = _f32(scene["scale"])
    cell = np.floor(mean / np.float32(voxel_size)).astype(np.int64)            # (3, n)
    cell -= cell.min(axis=1, keepdims=True) if n else 0
    assert n == 0 or cell.max() < (1 << 21)
    key = np.zeros(n, np.uint64)
    for bit in range(21):
        for ax in range(3):
            key |= ((cell[ax].astype(np.uint64) >> np.uint64(bit)) & np.uint64(1)) << np.uint64(3 * bit + ax)
    perm = np.lexsort((np.arange(n), key)).astype(np.uint32)
    skey = key[perm]
    starts = np.flatnonzero(np.concatenate([[True], skey[1:] != skey[:-1]])) if n else np.zeros(0, np.int64)
    first = np.concatenate([starts, [n]]).astype(np.uint32)
    V = len(starts)
    m = mean[:, perm]; s = scale[:, perm].max(axis=0) if n else np.zeros(0, np.float32)
    lo = np.stack([np.minimum.reduceat(m[a], starts) for a in range(3)], axis=1) if V else np.zeros((0, 3), np.float32)
    hi = np.stack([np.maximum.reduceat(m[a], starts) for a in range(3)], axis=1) if V else np.zeros((0, 3), np.float32)
    smax = np.maximum.reduceat(s, starts) if V else np.zeros(0, np.float32)
    return SimpleNamespace(n=n, perm=perm, first=first, num_voxels=V,
                           box_lo=np.ascontiguousarray(lo, np.float32), box_hi=np.ascontiguousarray(hi, np.float32),
                           smax=np.ascontiguousarray(smax, np.float32))


def reorder_scene(scene: dict, perm: np.ndarray) -> dict:
    """The same primitives in the order perm (new index k holds old primitive perm[k])."""
    out = dict(scene)
    for k in ("mean", "scale", "rot", "sh"):
        out[k] = np.ascontiguousarray(np.asarray(scene[k])[..., perm])
    out["opacity"] = np.ascontiguousarray(np.asarray(scene["opacity"])[perm])
    return out


def voxels_visible(index: SimpleNamespace, cam: dict) -> np.ndarray:
    """Per voxel: 0 only if every primitive in it is certain to be culled for this camera."""
    vis = np.empty(index.num_voxels, np.uint8)
    cc = _camera(cam)
    lib().lmk_ref_voxels_visible(C.byref(cc), C.c_uint32(index.num_voxels), _p(index.box_lo), _p(index.box_hi),
                                 _p(index.smax), _p(vis))
    return vis


def voxel_visible(cam: dict, lo, hi, smax: float) -> bool:
    lo = np.ascontiguousarray(lo, np.float32); hi = np.ascontiguousarray(hi, np.float32)
    lib().lmk_ref_voxel_visible.restype = C.c_int
    return bool(lib().lmk_ref_voxel_visible(C.byref(_camera(cam)), _p(lo), _p(hi), C.c_float(float(np.float32(smax)))))


def primitives_in_visible_voxels(index: SimpleNamespace, vis: np.ndarray) -> np.ndarray:
    """Boolean mask over the (reordered) primitives: the voxel holding it passed the filter."""
    counts = np.diff(index.first.astype(np.int64))
    return np.repeat(vis.astype(bool), counts)


def render_frame(scene: dict, cam: dict) -> SimpleNamespace:
    """Whole path, one frame."""
    pre = preprocess(scene, cam)
    b = bin_sort(pre, cam)
    img = render(pre, b, cam)
    return SimpleNamespace(pre=pre, binned=b, img=img)
