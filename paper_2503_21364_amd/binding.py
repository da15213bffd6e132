"""Thin ctypes binding of liblmk_gs.so (include/lmk_gs.h).

Argument marshalling only: every step of the path runs in the HIP kernels
behind the C ABI.  torch is used for device memory and streams.  There is no
CPU fallback: if the library is missing, import of the symbols fails loudly.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np
import torch  # must be imported before the library so that both share one HIP runtime

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "liblmk_gs.so")

OK, ERR_INVALID, ERR_CAPACITY, ERR_HIP, ERR_UNSUPPORTED = 0, -1, -2, -3, -4
TILE = 16
FEAT_STRIDE = 12

PRE_BLOCK = 256

EXPORTS = ("lmk_gs_workspace_bytes", "lmk_gs_preprocess", "lmk_gs_bin_sort", "lmk_gs_render",
           "lmk_gs_read_status", "lmk_gs_strerror", "lmk_gs_last_hip_error", "lmk_gs_version",
           "lmk_gs_index_build", "lmk_gs_preprocess_culled", "lmk_gs_build_cov3d", "lmk_gs_render_backward",
           "lmk_gs_preprocess_backward", "lmk_gs_anchor_decode", "lmk_gs_anchor_index_build",
           "lmk_gs_anchor_decode_culled", "lmk_gs_bin_sort_static")


class Gaussians(C.Structure):
    _fields_ = [("mean", C.c_void_p), ("scale", C.c_void_p), ("rot", C.c_void_p),
                ("opacity", C.c_void_p), ("sh", C.c_void_p), ("n", C.c_uint32), ("sh_degree", C.c_uint32),
                ("cov3d", C.c_void_p)]


class GaussianGrads(C.Structure):
    _fields_ = [("mean", C.c_void_p), ("scale", C.c_void_p), ("rot", C.c_void_p),
                ("opacity", C.c_void_p), ("sh", C.c_void_p)]


class Anchors(C.Structure):
    _fields_ = [("position", C.c_void_p), ("feature", C.c_void_p), ("extent", C.c_void_p),
                ("offsets", C.c_void_p), ("a", C.c_uint32), ("k", C.c_uint32)]


class Perceptron(C.Structure):
    _fields_ = [("w1", C.c_void_p), ("b1", C.c_void_p), ("w2t", C.c_void_p), ("b2", C.c_void_p)]


class AnchorDecoder(C.Structure):
    _fields_ = [("opacity", Perceptron), ("colour", Perceptron), ("cov", Perceptron)]


class Decoded(C.Structure):
    _fields_ = [("mean", C.c_void_p), ("scale", C.c_void_p), ("rot", C.c_void_p),
                ("opacity", C.c_void_p), ("sh", C.c_void_p)]


class Camera(C.Structure):
    _fields_ = [("view", C.c_float * 12), ("cam_pos", C.c_float * 3),
                ("fx", C.c_float), ("fy", C.c_float), ("cx", C.c_float), ("cy", C.c_float),
                ("width", C.c_uint32), ("height", C.c_uint32), ("tile", C.c_uint32),
                ("near_z", C.c_float), ("lowpass", C.c_float), ("bg", C.c_float * 3),
                ("binning", C.c_uint32)]


class VoxelIndexC(C.Structure):
    _fields_ = [("box", C.c_void_p), ("block_range", C.c_void_p), ("num_voxels", C.c_uint32),
                ("visible", C.c_void_p)]


class Projected(C.Structure):
    _fields_ = [("depth", C.c_void_p), ("tiles_touched", C.c_void_p), ("rect", C.c_void_p),
                ("feat", C.c_void_p), ("offsets", C.c_void_p)]


class Binned(C.Structure):
    _fields_ = [("keys", C.c_void_p), ("vals", C.c_void_p), ("keys_alt", C.c_void_p),
                ("vals_alt", C.c_void_p), ("capacity", C.c_uint64), ("tile_offsets", C.c_void_p),
                ("tile_order", C.c_void_p)]


class LmkGsError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where}: {strerror(code)} ({code})"
                         + (f", hipError {last_hip_error()}" if code == ERR_HIP else ""))


_lib = None


def lib() -> C.CDLL:
    """Loads the HIP library.  Raises if it has not been built: there is no fallback."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2503_21364_amd.build` "
                               "(the renderer has no CPU fallback)")
        l = C.CDLL(LIB_PATH)
        l.lmk_gs_workspace_bytes.argtypes = [C.c_uint32, C.c_uint32, C.c_uint32, C.c_uint64, C.POINTER(C.c_size_t)]
        l.lmk_gs_preprocess.argtypes = [C.POINTER(Gaussians), C.POINTER(Camera), C.POINTER(Projected),
                                        C.c_void_p, C.c_size_t, C.c_void_p]
        l.lmk_gs_bin_sort.argtypes = [C.POINTER(Projected), C.c_uint32, C.POINTER(Camera), C.POINTER(Binned),
                                      C.c_void_p, C.c_size_t, C.c_void_p]
        l.lmk_gs_bin_sort_static.argtypes = [C.POINTER(Projected), C.c_uint32, C.POINTER(Camera), C.POINTER(Binned),
                                             C.c_void_p, C.c_void_p]
        l.lmk_gs_render.argtypes = [C.POINTER(Projected), C.POINTER(Binned), C.POINTER(Camera),
                                    C.c_void_p, C.c_void_p, C.c_void_p]
        l.lmk_gs_index_build.argtypes = [C.c_void_p, C.c_void_p, C.c_uint32, C.c_float, C.c_void_p, C.c_void_p,
                                         C.c_void_p, C.c_void_p, C.POINTER(C.c_uint32)]
        l.lmk_gs_preprocess_culled.argtypes = [C.POINTER(Gaussians), C.POINTER(VoxelIndexC), C.POINTER(Camera),
                                               C.POINTER(Projected), C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
        l.lmk_gs_build_cov3d.argtypes = [C.POINTER(Gaussians), C.c_void_p, C.c_void_p]
        l.lmk_gs_preprocess_backward.argtypes = [C.POINTER(Gaussians), C.POINTER(Camera), C.POINTER(Projected),
                                                 C.c_void_p, C.POINTER(GaussianGrads), C.c_void_p]
        l.lmk_gs_render_backward.argtypes = [C.POINTER(Projected), C.c_uint32, C.POINTER(Binned), C.POINTER(Camera),
                                             C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        l.lmk_gs_anchor_decode.argtypes = [C.POINTER(Anchors), C.POINTER(AnchorDecoder), C.POINTER(C.c_float),
                                           C.c_void_p, C.c_uint32, C.POINTER(Decoded), C.c_void_p]
        l.lmk_gs_anchor_index_build.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_uint32, C.c_uint32,
                                                C.c_void_p, C.c_void_p]
        l.lmk_gs_anchor_decode_culled.argtypes = [C.POINTER(Anchors), C.POINTER(AnchorDecoder), C.POINTER(Camera),
                                                  C.c_void_p, C.c_void_p, C.POINTER(Decoded), C.c_void_p]
        l.lmk_gs_read_status.argtypes = [C.c_void_p, C.POINTER(C.c_uint64), C.POINTER(C.c_int32), C.c_void_p]
        l.lmk_gs_strerror.argtypes = [C.c_int32]
        l.lmk_gs_strerror.restype = C.c_char_p
        for name in ("lmk_gs_workspace_bytes", "lmk_gs_preprocess", "lmk_gs_bin_sort", "lmk_gs_render",
                     "lmk_gs_read_status", "lmk_gs_last_hip_error", "lmk_gs_index_build",
                     "lmk_gs_preprocess_culled", "lmk_gs_build_cov3d", "lmk_gs_render_backward",
                     "lmk_gs_preprocess_backward", "lmk_gs_anchor_decode", "lmk_gs_anchor_index_build",
                     "lmk_gs_anchor_decode_culled", "lmk_gs_bin_sort_static"):
            getattr(l, name).restype = C.c_int32
        l.lmk_gs_version.restype = C.c_uint32
        _lib = l
    return _lib


def strerror(code: int) -> str:
    return lib().lmk_gs_strerror(code).decode()


def last_hip_error() -> int:
    return int(lib().lmk_gs_last_hip_error())


def make_camera(cam: dict) -> Camera:
    c = Camera()
    c.view[:] = [float(x) for x in np.asarray(cam["view"], dtype=np.float32).reshape(12)]
    c.cam_pos[:] = [float(x) for x in np.asarray(cam["cam_pos"], dtype=np.float32)]
    c.fx, c.fy, c.cx, c.cy = (float(np.float32(cam[k])) for k in ("fx", "fy", "cx", "cy"))
    c.width, c.height, c.tile = int(cam["width"]), int(cam["height"]), int(cam["tile"])
    c.near_z, c.lowpass = float(np.float32(cam["near_z"])), float(np.float32(cam["lowpass"]))
    c.bg[:] = [float(x) for x in np.asarray(cam["bg"], dtype=np.float32)]
    c.binning = int(cam.get("binning", 0))
    return c


def workspace_bytes(n: int, width: int, height: int, capacity: int) -> int:
    out = C.c_size_t(0)
    rc = lib().lmk_gs_workspace_bytes(n, width, height, capacity, C.byref(out))
    if rc != OK:
        raise LmkGsError(rc, "lmk_gs_workspace_bytes")
    return int(out.value)


def _ptr(t) -> int | None:
    return None if t is None else t.data_ptr()


def _stream_handle(stream) -> int | None:
    if stream is None:
        stream = torch.cuda.current_stream()
    return stream.cuda_stream or None


def sh_stride(sh_degree: int) -> int:
    """LMK_GS_SH_STRIDE of include/lmk_gs.h."""
    return (3 * (sh_degree + 1) ** 2 + 3) & ~3


class Scene:
    """Device-resident primitives (layouts of include/lmk_gs.h)."""

    def __init__(self, scene: dict, device="cuda:0"):
        self.n = int(scene["n"])
        self.sh_degree = int(scene["sh_degree"])
        f = lambda a: torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(device)
        self.mean, self.scale, self.rot = f(scene["mean"]), f(scene["scale"]), f(scene["rot"])
        self.opacity = f(scene["opacity"])
        # the generator's [coefficient][channel][n] planes become one record per primitive
        ncoef = (self.sh_degree + 1) ** 2
        rec = np.zeros((self.n, sh_stride(self.sh_degree)), np.float32)
        rec[:, :3 * ncoef] = np.asarray(scene["sh"][:ncoef], np.float32).reshape(3 * ncoef, self.n).T
        self.sh = f(rec)
        self.cov3d = None
        self.c = Gaussians(_ptr(self.mean), _ptr(self.scale), _ptr(self.rot), _ptr(self.opacity),
                           _ptr(self.sh), self.n, self.sh_degree, None)

    def build_cov3d(self, stream=None) -> "Scene":
        """Fills the parameter cache (lmk_gs_build_cov3d); later preprocess calls read it."""
        self.cov3d = torch.empty((6, max(self.n, 1)), dtype=torch.float32, device=self.mean.device)
        rc = lib().lmk_gs_build_cov3d(C.byref(self.c), _ptr(self.cov3d), _stream_handle(stream))
        if rc != OK:
            raise LmkGsError(rc, "lmk_gs_build_cov3d")
        self.c.cov3d = _ptr(self.cov3d)
        return self


class VoxelIndex:
    """Offline voxel reordering of a scene (lmk_gs_index_build, host side).  `perm`, `first`, `box`
    and `block_range` are the host arrays the library returned; `reorder` applies the permutation
    to a scene dict; `upload` puts the two arrays the kernels read on the device."""

    def __init__(self, scene: dict, voxel_size: float):
        n = int(scene["n"])
        mean = np.ascontiguousarray(scene["mean"], dtype=np.float32)
        scale = np.ascontiguousarray(scene["scale"], dtype=np.float32)
        nb = (n + PRE_BLOCK - 1) // PRE_BLOCK
        perm = np.empty(max(n, 1), np.uint32)
        first = np.empty(n + 1, np.uint32)
        box = np.empty((max(n, 1), 8), np.float32)
        block_range = np.empty((max(nb, 1), 2), np.uint32)
        nv = C.c_uint32(0)
        rc = lib().lmk_gs_index_build(mean.ctypes.data, scale.ctypes.data, n, float(voxel_size), perm.ctypes.data,
                                      first.ctypes.data, box.ctypes.data, block_range.ctypes.data, C.byref(nv))
        if rc != OK:
            raise LmkGsError(rc, "lmk_gs_index_build")
        self.n, self.num_voxels, self.voxel_size = n, int(nv.value), float(voxel_size)
        self.perm = perm[:n]
        self.first = first[:self.num_voxels + 1].copy()
        self.box = box[:self.num_voxels].copy()
        self.block_range = block_range[:nb]
        self.c = None

    def reorder(self, scene: dict) -> dict:
        out = dict(scene)
        for k in ("mean", "scale", "rot", "sh"):
            out[k] = np.ascontiguousarray(np.asarray(scene[k])[..., self.perm])
        out["opacity"] = np.ascontiguousarray(np.asarray(scene["opacity"])[self.perm])
        return out

    def upload(self, device="cuda:0") -> "VoxelIndex":
        self.box_dev = torch.from_numpy(np.ascontiguousarray(self.box if self.num_voxels else np.zeros((1, 8), np.float32))).to(device)
        self.block_range_dev = torch.from_numpy(np.ascontiguousarray(
            self.block_range if len(self.block_range) else np.zeros((1, 2), np.uint32)).view(np.int32)).to(device)
        self.c = VoxelIndexC(_ptr(self.box_dev), _ptr(self.block_range_dev), self.num_voxels, None)
        return self


class Frame:
    """All device buffers of one frame in flight: per-primitive outputs, pair
    buffers for `capacity` pairs, scratch, and the image."""

    def __init__(self, n: int, width: int, height: int, capacity: int, device="cuda:0",
                 want_offsets: bool = False, tile_order: bool = True):
        self.n, self.width, self.height, self.capacity = n, width, height, int(capacity)
        self.tiles_x = (width + TILE - 1) // TILE
        self.tiles_y = (height + TILE - 1) // TILE
        dev = device
        e = lambda shape, dt: torch.empty(shape, dtype=dt, device=dev)
        self.depth = e((max(n, 1),), torch.float32)
        self.tiles_touched = e((max(n, 1),), torch.int32)
        self.rect = e((max(n, 1), 4), torch.int16)
        self.feat = e((max(n, 1), FEAT_STRIDE), torch.float32)
        self.offsets = e((n + 1,), torch.int64) if want_offsets else None
        cap = max(self.capacity, 1)
        self.keys, self.keys_alt = e((cap,), torch.int64), e((cap,), torch.int64)
        self.vals, self.vals_alt = e((cap,), torch.int32), e((cap,), torch.int32)
        self.tile_offsets = e((self.tiles_x * self.tiles_y + 1,), torch.int64)
        self.tile_order = e((self.tiles_x * self.tiles_y,), torch.int32) if tile_order else None
        self.scratch_bytes = workspace_bytes(n, width, height, self.capacity)
        self.scratch = e((self.scratch_bytes,), torch.uint8)
        self.out_rgb = e((3, height, width), torch.float32)
        self.out_T = e((height, width), torch.float32)
        self.proj = Projected(_ptr(self.depth), _ptr(self.tiles_touched), _ptr(self.rect),
                              _ptr(self.feat), _ptr(self.offsets))
        self.binned = Binned(_ptr(self.keys), _ptr(self.vals), _ptr(self.keys_alt), _ptr(self.vals_alt),
                             self.capacity, _ptr(self.tile_offsets), _ptr(self.tile_order))


def preprocess(scene: Scene, cam: Camera, frame: Frame, stream=None, index: VoxelIndex | None = None,
               block_visible=None) -> None:
    """lmk_gs_preprocess, or lmk_gs_preprocess_culled when a (uploaded) voxel index is given;
    block_visible: optional uint8 device tensor receiving the per-group flags of the filter."""
    if index is None:
        rc = lib().lmk_gs_preprocess(C.byref(scene.c), C.byref(cam), C.byref(frame.proj),
                                     _ptr(frame.scratch), frame.scratch_bytes, _stream_handle(stream))
        where = "lmk_gs_preprocess"
    else:
        rc = lib().lmk_gs_preprocess_culled(C.byref(scene.c), C.byref(index.c), C.byref(cam), C.byref(frame.proj),
                                            _ptr(block_visible), _ptr(frame.scratch), frame.scratch_bytes,
                                            _stream_handle(stream))
        where = "lmk_gs_preprocess_culled"
    if rc != OK:
        raise LmkGsError(rc, where)


def bin_sort(cam: Camera, frame: Frame, stream=None) -> None:
    rc = lib().lmk_gs_bin_sort(C.byref(frame.proj), frame.n, C.byref(cam), C.byref(frame.binned),
                               _ptr(frame.scratch), frame.scratch_bytes, _stream_handle(stream))
    if rc != OK:
        raise LmkGsError(rc, "lmk_gs_bin_sort")


STATIC_MAX_N, STATIC_MAX_CAPACITY, STATIC_MAX_TILES = 4 << 20, 16 << 20, 16384


def bin_sort_static(cam: Camera, frame: Frame, count_status=None, stream=None) -> None:
    """lmk_gs_bin_sort_static: stage 2 on the library's own fixed scratch array (no workspace, no
    allocation); count_status: optional int64 device tensor of two elements receiving {D, status}."""
    rc = lib().lmk_gs_bin_sort_static(C.byref(frame.proj), frame.n, C.byref(cam), C.byref(frame.binned),
                                      _ptr(count_status), _stream_handle(stream))
    if rc != OK:
        raise LmkGsError(rc, "lmk_gs_bin_sort_static")


def render(cam: Camera, frame: Frame, stream=None) -> None:
    rc = lib().lmk_gs_render(C.byref(frame.proj), C.byref(frame.binned), C.byref(cam),
                             _ptr(frame.out_rgb), _ptr(frame.out_T), _stream_handle(stream))
    if rc != OK:
        raise LmkGsError(rc, "lmk_gs_render")


def render_backward(cam: Camera, frame: Frame, grad_rgb, grad_T, grad_feat, stream=None) -> None:
    """lmk_gs_render_backward on a frame that went through preprocess and bin_sort: grad_rgb
    [3][H][W] and grad_T [H][W] (or None) float32 device tensors in, grad_feat [n][FEAT_STRIDE] out."""
    rc = lib().lmk_gs_render_backward(C.byref(frame.proj), C.c_uint32(frame.n), C.byref(frame.binned),
                                      C.byref(cam), _ptr(grad_rgb), _ptr(grad_T), _ptr(grad_feat),
                                      _stream_handle(stream))
    if rc != OK:
        raise LmkGsError(rc, "lmk_gs_render_backward")


class SceneGrads:
    """Device buffers for the output of lmk_gs_preprocess_backward, laid out like the scene."""

    def __init__(self, scene: "Scene", device="cuda:0"):
        n = max(scene.n, 1)
        e = lambda shape: torch.empty(shape, dtype=torch.float32, device=device)
        self.mean, self.scale, self.rot = e((3, n)), e((3, n)), e((4, n))
        self.opacity, self.sh = e((n,)), e((n, sh_stride(scene.sh_degree)))
        self.c = GaussianGrads(_ptr(self.mean), _ptr(self.scale), _ptr(self.rot), _ptr(self.opacity), _ptr(self.sh))


def preprocess_backward(scene: "Scene", cam: Camera, frame: Frame, grad_feat, grads: SceneGrads, stream=None) -> None:
    rc = lib().lmk_gs_preprocess_backward(C.byref(scene.c), C.byref(cam), C.byref(frame.proj), _ptr(grad_feat),
                                          C.byref(grads.c), _stream_handle(stream))
    if rc != OK:
        raise LmkGsError(rc, "lmk_gs_preprocess_backward")


class AnchorScene:
    """Device-resident anchors and decoder weights (layouts of include/lmk_gs.h)."""

    def __init__(self, anchors: dict, mlp: dict, device="cuda:0"):
        self.a, self.k = int(anchors["a"]), int(anchors["k"])
        f = lambda t: torch.from_numpy(np.ascontiguousarray(t, dtype=np.float32)).to(device)
        self.position, self.feature = f(anchors["position"]), f(anchors["feature"])
        self.extent, self.offsets = f(anchors["extent"]), f(anchors["offsets"])
        self.c = Anchors(_ptr(self.position), _ptr(self.feature), _ptr(self.extent), _ptr(self.offsets),
                         self.a, self.k)
        self.weights = {name: {w: f(mlp[name][w]) for w in ("w1", "b1", "w2t", "b2")}
                        for name in ("opacity", "colour", "cov")}
        net = lambda p: Perceptron(_ptr(p["w1"]), _ptr(p["b1"]), _ptr(p["w2t"]), _ptr(p["b2"]))
        self.decoder = AnchorDecoder(net(self.weights["opacity"]), net(self.weights["colour"]),
                                     net(self.weights["cov"]))


def reorder_anchors(anchors: dict, voxel_size: float) -> dict:
    """Offline: the anchors in the voxel order of lmk_gs_index_build applied to their centres, so that
    consecutive anchors are close in space (a tile of the decoder and a group of the rasteriser then
    fall inside or outside a view together)."""
    idx = VoxelIndex(dict(mean=anchors["position"], scale=anchors["extent"][3:6], n=anchors["a"]), voxel_size)
    perm = idx.perm
    return dict(anchors, position=np.ascontiguousarray(anchors["position"][:, perm]),
                feature=np.ascontiguousarray(anchors["feature"][perm]),
                extent=np.ascontiguousarray(anchors["extent"][:, perm]),
                offsets=np.ascontiguousarray(anchors["offsets"][perm]))


class AnchorIndex:
    """Offline part of the anchors' view-frustum mask (lmk_gs_anchor_index_build, host side): per-anchor
    boxes and, for the decoded scene, the anchors spanned by every group of PRE_BLOCK slots.  `c` is the
    lmk_gs_voxel_index over the decoded slots for lmk_gs_preprocess_culled (one "voxel" per anchor)."""

    def __init__(self, anchors: dict, device="cuda:0"):
        a, k = int(anchors["a"]), int(anchors["k"])
        pos = np.ascontiguousarray(anchors["position"], dtype=np.float32)
        ext = np.ascontiguousarray(anchors["extent"], dtype=np.float32)
        off = np.ascontiguousarray(anchors["offsets"], dtype=np.float32)
        nb = (a * k + PRE_BLOCK - 1) // PRE_BLOCK
        self.box = np.zeros((max(a, 1), 8), np.float32)
        self.block_range = np.zeros((max(nb, 1), 2), np.uint32)
        rc = lib().lmk_gs_anchor_index_build(pos.ctypes.data, ext.ctypes.data, off.ctypes.data, a, k,
                                             self.box.ctypes.data, self.block_range.ctypes.data)
        if rc != OK:
            raise LmkGsError(rc, "lmk_gs_anchor_index_build")
        self.a, self.k, self.num_voxels = a, k, a
        self.box_dev = torch.from_numpy(self.box).to(device)
        self.block_range_dev = torch.from_numpy(self.block_range.view(np.int32)).to(device)
        self.visible = torch.zeros(max(a, 1), dtype=torch.uint8, device=device)     # per-frame mask
        # after lmk_gs_anchor_decode_culled of a frame, `visible` holds that frame's mask: preprocess reuses it
        self.c = VoxelIndexC(_ptr(self.box_dev), _ptr(self.block_range_dev), a, _ptr(self.visible))
        self.c_recompute = VoxelIndexC(_ptr(self.box_dev), _ptr(self.block_range_dev), a, None)


class DecodedScene:
    """Output buffers of lmk_gs_anchor_decode for a list of v anchors with k primitives each."""

    def __init__(self, v: int, k: int, device="cuda:0"):
        self.k, self.v, self.n = int(k), int(v), int(v) * int(k)
        n = max(self.n, 1)
        e = lambda shape: torch.empty(shape, dtype=torch.float32, device=device)
        self.mean, self.scale, self.rot = e((3, n)), e((3, n)), e((4, n))
        self.opacity, self.sh = e((n,)), e((n, 4))
        self.c = Decoded(_ptr(self.mean), _ptr(self.scale), _ptr(self.rot), _ptr(self.opacity), _ptr(self.sh))

    def scene(self) -> "Scene":
        """The decoded slots as a Scene object (no copy) for preprocess."""
        sc = Scene.__new__(Scene)
        sc.n, sc.sh_degree = self.n, 0
        sc.mean, sc.scale, sc.rot, sc.opacity, sc.sh = self.mean, self.scale, self.rot, self.opacity, self.sh
        sc.cov3d = None
        sc.c = Gaussians(_ptr(self.mean), _ptr(self.scale), _ptr(self.rot), _ptr(self.opacity), _ptr(self.sh),
                         self.n, 0, None)
        return sc


def anchor_decode(anchors: AnchorScene, cam_pos, out: DecodedScene, visible=None, v: int | None = None,
                  stream=None) -> None:
    """lmk_gs_anchor_decode: `visible` is a uint32/int32 device tensor of anchor indices or None
    (then anchors 0..v-1, v defaulting to all).  `out` must be sized for v anchors."""
    if v is None:
        v = anchors.a if visible is None else int(visible.numel())
    if out.n != v * anchors.k:
        raise ValueError("output buffers are sized for another list length")
    cam = (C.c_float * 3)(*[float(x) for x in cam_pos])
    rc = lib().lmk_gs_anchor_decode(C.byref(anchors.c), C.byref(anchors.decoder), cam, _ptr(visible),
                                    C.c_uint32(v), C.byref(out.c), _stream_handle(stream))
    if rc != OK:
        raise LmkGsError(rc, "lmk_gs_anchor_decode")


def anchor_decode_culled(anchors: AnchorScene, index: AnchorIndex, cam: Camera, out: DecodedScene, stream=None) -> None:
    """lmk_gs_anchor_decode_culled: every anchor in order, those outside the view masked; the mask is
    left in index.visible."""
    if out.n != anchors.a * anchors.k:
        raise ValueError("output buffers are sized for another number of anchors")
    rc = lib().lmk_gs_anchor_decode_culled(C.byref(anchors.c), C.byref(anchors.decoder), C.byref(cam),
                                           _ptr(index.box_dev), _ptr(index.visible), C.byref(out.c),
                                           _stream_handle(stream))
    if rc != OK:
        raise LmkGsError(rc, "lmk_gs_anchor_decode_culled")


def read_status(frame: Frame, stream=None) -> tuple[int, int]:
    """(pair count D, status) of the frame; synchronises the stream."""
    d, s = C.c_uint64(0), C.c_int32(0)
    rc = lib().lmk_gs_read_status(_ptr(frame.scratch), C.byref(d), C.byref(s), _stream_handle(stream))
    if rc != OK:
        raise LmkGsError(rc, "lmk_gs_read_status")
    return int(d.value), int(s.value)


def render_frame(scene: Scene, cam: Camera, frame: Frame, stream=None, index: VoxelIndex | None = None) -> None:
    """The whole hot path for one view: three asynchronous calls on one stream."""
    preprocess(scene, cam, frame, stream, index)
    bin_sort(cam, frame, stream)
    render(cam, frame, stream)
