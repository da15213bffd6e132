"""Seeded synthetic scenes and cameras for the five benchmark configurations.

This module only *draws inputs*: primitive attributes from the stated
distributions and camera poses/intrinsics.  It holds none of the renderer's
arithmetic and is the one module that both the GPU tests and the CPU oracle's
tests import.

The scenes stand in for the workload the report evaluates on (Sec. 5: 1920x1080
renders of a city-scale capture, about 3.7 M primitives for the single-device
vanilla model, Table 1), which is not available offline.

Layout of a scene (all float32, structure of arrays, N contiguous last):
    mean    (3, N)   world-space centres
    scale   (3, N)   linear standard deviations (already exponentiated)
    rot     (4, N)   quaternion (w, x, y, z), unit norm up to rounding
    opacity (N,)     in [0, 1] (already passed through the sigmoid)
    sh      (16, 3, N)  spherical-harmonic coefficients, degree 3
Camera: dict with view (3x4 row-major world->camera, +x right, +y down,
+z forward), cam_pos, fx, fy, cx, cy, width, height, tile, near_z, lowpass, bg,
binning (0: every tile of the support rectangle, 1: only tiles the splat can reach).
"""
from __future__ import annotations

import math

import numpy as np

TILE = 16
LOWPASS = 0.3
NEAR = 0.2

CONFIGS = {
    0: dict(n=10_000, width=256, height=256, fov_deg=60.0, views=1),
    1: dict(n=500_000, width=1920, height=1080, fov_deg=50.0, views=8),
    2: dict(n=3_000_000, width=1920, height=1080, fov_deg=50.0, views=8),
    3: dict(n=20_000_000, width=1920, height=1080, fov_deg=60.0, views=8),
    4: dict(n=2_000_000, width=3840, height=2160, fov_deg=60.0, views=1),
}


def _sigmoid(x):
    return (1.0 / (1.0 + np.exp(-x.astype(np.float64)))).astype(np.float32)


def _normal(rng, shape, mu=0.0, sigma=1.0):
    out = rng.standard_normal(shape, dtype=np.float32)
    if sigma != 1.0:
        out *= np.float32(sigma)
    if mu != 0.0:
        out += np.float32(mu)
    return out


def _common_attrs(rng, n, log_scale_mu, log_scale_sigma, op_mu, op_sigma):
    scale = np.exp(_normal(rng, (3, n), log_scale_mu, log_scale_sigma)).astype(np.float32)
    rot = _normal(rng, (4, n))
    rot /= np.sqrt((rot.astype(np.float64) ** 2).sum(axis=0)).astype(np.float32)
    opacity = _sigmoid(_normal(rng, (n,), op_mu, op_sigma))
    sh = _normal(rng, (16, 3, n), 0.0, 0.3)
    sh[0] = _normal(rng, (3, n), 0.5, 0.2)
    return scale, rot, opacity, sh


def _random_rotations(rng, k):
    q = rng.standard_normal((k, 4))
    q /= np.linalg.norm(q, axis=1, keepdims=True)
    w, x, y, z = q.T
    R = np.empty((k, 3, 3))
    R[:, 0, 0] = 1 - 2 * (y * y + z * z); R[:, 0, 1] = 2 * (x * y - w * z); R[:, 0, 2] = 2 * (x * z + w * y)
    R[:, 1, 0] = 2 * (x * y + w * z); R[:, 1, 1] = 1 - 2 * (x * x + z * z); R[:, 1, 2] = 2 * (y * z - w * x)
    R[:, 2, 0] = 2 * (x * z - w * y); R[:, 2, 1] = 2 * (y * z + w * x); R[:, 2, 2] = 1 - 2 * (x * x + y * y)
    return R


def cluster_layout(seed=2000):
    """Cluster centres / axes of config 2 (also used to place its interior cameras)."""
    rng = np.random.default_rng(seed + 77)
    centres = rng.uniform(-16.0, 16.0, size=(64, 3))
    stds = np.exp(rng.uniform(math.log(0.5), math.log(4.0), size=(64, 3)))
    rots = _random_rotations(rng, 64)
    return centres, stds, rots


def make_scene(cfg: int, n: int | None = None, seed: int | None = None) -> dict:
    """Draw the primitives of configuration `cfg` (optionally with a reduced count n)."""
    spec = CONFIGS[cfg]
    n = spec["n"] if n is None else int(n)
    seed = 1000 * cfg if seed is None else seed
    rng = np.random.default_rng(seed)
    if cfg == 0:
        mean = rng.uniform(-1.0, 1.0, size=(3, n)).astype(np.float32)
        attrs = _common_attrs(rng, n, -3.5, 0.5, 0.0, 1.5)
    elif cfg == 1:
        mean = rng.uniform(-5.0, 5.0, size=(3, n)).astype(np.float32)
        attrs = _common_attrs(rng, n, -3.5, 0.5, 0.0, 1.5)
    elif cfg == 2:
        centres, stds, rots = cluster_layout(1000 * cfg)
        which = rng.integers(0, 64, size=n)
        local = _normal(rng, (n, 3)) * stds[which].astype(np.float32)
        mean = (np.einsum("nij,nj->ni", rots[which].astype(np.float32), local)
                + centres[which].astype(np.float32)).T.astype(np.float32)
        mean = np.ascontiguousarray(mean)
        attrs = _common_attrs(rng, n, -4.0, 0.8, 0.0, 2.0)
    elif cfg == 3:
        mean = np.empty((3, n), dtype=np.float32)
        mean[0] = rng.uniform(-1000.0, 1000.0, size=n).astype(np.float32)
        mean[1] = rng.uniform(-1000.0, 1000.0, size=n).astype(np.float32)
        mean[2] = np.abs(_normal(rng, (n,), 0.0, 15.0))
        attrs = _common_attrs(rng, n, -1.0, 1.0, 0.0, 1.5)
    elif cfg == 4:
        mean = rng.uniform(-1.0, 1.0, size=(3, n)).astype(np.float32)
        attrs = _common_attrs(rng, n, -2.0, 0.7, -1.0, 1.0)
    else:
        raise ValueError(f"unknown config {cfg}")
    scale, rot, opacity, sh = attrs
    return dict(mean=mean, scale=scale, rot=rot, opacity=opacity, sh=sh, sh_degree=3, n=n)


def look_at(eye, target, up):
    """3x4 world->camera matrix with +x right, +y down, +z forward."""
    eye = np.asarray(eye, dtype=np.float64)
    f = np.asarray(target, dtype=np.float64) - eye
    f /= np.linalg.norm(f)
    r = np.cross(f, np.asarray(up, dtype=np.float64))
    r /= np.linalg.norm(r)
    d = np.cross(f, r)
    R = np.stack([r, d, f])
    t = -R @ eye
    return np.concatenate([R, t[:, None]], axis=1)


def make_camera(view34, eye, width, height, fov_deg, bg=(0.0, 0.0, 0.0),
                tile=TILE, near=NEAR, lowpass=LOWPASS, binning=0) -> dict:
    """Pinhole camera; fov is the vertical field of view, square pixels."""
    f = height / (2.0 * math.tan(math.radians(fov_deg) / 2.0))
    return dict(view=np.asarray(view34, dtype=np.float32).reshape(12),
                cam_pos=np.asarray(eye, dtype=np.float32),
                fx=np.float32(f), fy=np.float32(f),
                cx=np.float32(width / 2.0), cy=np.float32(height / 2.0),
                width=int(width), height=int(height), tile=int(tile),
                near_z=np.float32(near), lowpass=np.float32(lowpass),
                bg=np.asarray(bg, dtype=np.float32), binning=int(binning))


def make_cameras(cfg: int, width: int | None = None, height: int | None = None) -> list[dict]:
    """The seeded viewpoints of configuration `cfg`."""
    spec = CONFIGS[cfg]
    W = spec["width"] if width is None else width
    H = spec["height"] if height is None else height
    fov = spec["fov_deg"]
    rng = np.random.default_rng(1000 * cfg + 500)
    cams = []
    if cfg == 0:
        eye = (0.0, 0.0, 4.0)
        cams.append(make_camera(look_at(eye, (0, 0, 0), (0, 1, 0)), eye, W, H, fov))
    elif cfg == 1:
        for k in range(8):
            th = 2 * math.pi * k / 8 + rng.uniform(-0.1, 0.1)
            eye = (12 * math.cos(th), 2.0, 12 * math.sin(th))
            cams.append(make_camera(look_at(eye, (0, 0, 0), (0, 1, 0)), eye, W, H, fov))
    elif cfg == 2:
        centres, _, _ = cluster_layout(1000 * cfg)
        for k in range(4):
            th = 2 * math.pi * k / 4 + rng.uniform(-0.2, 0.2)
            eye = (45 * math.cos(th), 10.0, 45 * math.sin(th))
            cams.append(make_camera(look_at(eye, (0, 0, 0), (0, 1, 0)), eye, W, H, fov))
        for k in range(4):
            a, b = rng.choice(64, size=2, replace=False)
            eye = centres[a] + rng.uniform(-1.0, 1.0, size=3)
            cams.append(make_camera(look_at(eye, centres[b], (0, 1, 0)), eye, W, H, fov))
    elif cfg == 3:
        for k in range(8):
            ex, ey = rng.uniform(-500.0, 500.0, size=2)
            yaw = rng.uniform(0, 2 * math.pi)
            eye = np.array([ex, ey, 300.0])
            c45 = math.cos(math.radians(45.0))
            fwd = np.array([math.cos(yaw) * c45, math.sin(yaw) * c45, -c45])
            cams.append(make_camera(look_at(eye, eye + fwd, (0, 0, 1)), eye, W, H, fov))
    elif cfg == 4:
        eye = (0.0, 0.0, 3.0)
        cams.append(make_camera(look_at(eye, (0, 0, 0), (0, 1, 0)), eye, W, H, fov))
    else:
        raise ValueError(f"unknown config {cfg}")
    return cams


def hand_placed_scene(mean, scale, rot=(1, 0, 0, 0), opacity=1.0, sh_dc=(0.0, 0.0, 0.0)) -> dict:
    """A scene of hand-placed primitives (for closed-form checks).  Arguments may
    be single values or lists of equal length; only the degree-0 SH coefficient
    is set (to the raw value `sh_dc`), all higher ones are zero."""
    mean = np.atleast_2d(np.asarray(mean, dtype=np.float32))
    n = mean.shape[0]
    scale = np.broadcast_to(np.atleast_2d(np.asarray(scale, dtype=np.float32)), (n, 3))
    rot = np.broadcast_to(np.atleast_2d(np.asarray(rot, dtype=np.float32)), (n, 4))
    opacity = np.broadcast_to(np.atleast_1d(np.asarray(opacity, dtype=np.float32)), (n,))
    sh_dc = np.broadcast_to(np.atleast_2d(np.asarray(sh_dc, dtype=np.float32)), (n, 3))
    sh = np.zeros((16, 3, n), dtype=np.float32)
    sh[0] = sh_dc.T
    return dict(mean=np.ascontiguousarray(mean.T), scale=np.ascontiguousarray(scale.T),
                rot=np.ascontiguousarray(rot.T), opacity=np.ascontiguousarray(opacity),
                sh=sh, sh_degree=3, n=n)


HOSTILE_GROUPS = ("mean_nan", "mean_pinf", "mean_ninf", "quat_zero", "scale_nan", "scale_zero", "scale_negative",
                  "scale_huge", "scale_denormal", "opacity_threshold", "opacity_below", "opacity_zero", "opacity_one",
                  "on_near_plane", "quat_tiny", "quat_large")


def hostile_scene(n: int = 3000, seed: int = 91, group_size: int = 40):
    """Config-0 primitives with groups of degenerate attribute values (non-finite centres, zero or
    non-finite rotations and scales, opacities at and around the 1/255 threshold, centres exactly
    on the near plane of config 0's camera).  Returns (scene, {group name: primitive indices})."""
    sc = make_scene(0, n=n, seed=seed)
    idx = np.random.default_rng(seed).permutation(n)
    groups = {name: idx[j * group_size:(j + 1) * group_size] for j, name in enumerate(HOSTILE_GROUPS)}
    g = groups
    sc["mean"][0, g["mean_nan"]] = np.nan
    sc["mean"][2, g["mean_pinf"]] = np.inf
    sc["mean"][1, g["mean_ninf"]] = -np.inf
    sc["rot"][:, g["quat_zero"]] = 0.0
    sc["scale"][1, g["scale_nan"]] = np.nan
    sc["scale"][:, g["scale_zero"]] = 0.0                 # a point: only the low-pass remains
    sc["scale"][0, g["scale_negative"]] *= -1.0           # the sign of a scale does not matter
    sc["scale"][:, g["scale_huge"]] = 1e20                # the covariance overflows
    sc["scale"][2, g["scale_denormal"]] = 1e-30
    sc["opacity"][g["opacity_threshold"]] = np.float32(1.0 / 255.0)
    sc["opacity"][g["opacity_below"]] = np.nextafter(np.float32(1.0 / 255.0), np.float32(0))
    sc["opacity"][g["opacity_zero"]] = 0.0
    sc["opacity"][g["opacity_one"]] = 1.0
    sc["mean"][:, g["on_near_plane"]] = np.array([[0.0], [0.0], [4.0 - NEAR]], np.float32)
    sc["rot"][:, g["quat_tiny"]] *= np.float32(1e-20)
    sc["rot"][:, g["quat_large"]] *= np.float32(1e18)
    return sc, groups


# ---------------------------------------------------------------------------------------------
# Anchor scenes (the input of the AnchorDecoder, Sec. 4.2.1): anchors that carry a feature
# vector, per-axis extents and K learnable offsets, plus the weights of the three two-layer
# perceptrons that turn an anchor and a viewing direction into K Gaussian primitives.
# Layout (float32):
#     position (3, A)        anchor centres
#     feature  (A, F)        F = ANCHOR_FEAT values per anchor, one record per anchor
#     extent   (6, A)        linear, > 0: rows 0-2 scale the offsets, rows 3-5 bound the scales
#     offsets  (A, K, 3)     offsets of the K primitives of an anchor, in units of extent 0-2
#     mlp      {"opacity" | "colour" | "cov": dict(w1 (F, F+3), b1 (F,), w2t (F, outs), b2 (outs,))}
#              first layer as (hidden unit, input), second layer as (hidden unit, output);
#              outs = K, 3K, 7K
ANCHOR_FEAT = 32
ANCHOR_K = 10
ANCHOR_OUTS = {"opacity": 1, "colour": 3, "cov": 7}      # outputs per primitive


def make_decoder(seed: int = 7000, k: int = ANCHOR_K, scale: float = 1.0) -> dict:
    """Random weights of the three perceptrons (fan-in scaled normal draws, small biases)."""
    rng = np.random.default_rng(seed)
    F, D = ANCHOR_FEAT, ANCHOR_FEAT + 3
    mlp = {}
    for name, per in ANCHOR_OUTS.items():
        outs = per * k
        mlp[name] = dict(
            w1=_normal(rng, (F, D), 0.0, scale / math.sqrt(D)),
            b1=_normal(rng, (F,), 0.0, 0.1),
            w2t=_normal(rng, (F, outs), 0.0, scale / math.sqrt(F)),
            b2=_normal(rng, (outs,), 0.0, 0.1))
    return mlp


def make_anchor_scene(a: int, seed: int = 6000, k: int = ANCHOR_K, layout: str = "cube") -> dict:
    """Draw `a` anchors.  layout "cube": centres uniform in [-1,1]^3 (seen by config 0's camera);
    "clusters": the 64 clusters of config 2 (seen by its cameras).  With k = 10, 300 k anchors
    of the cluster layout decode to 3 M candidate primitives, the size of config 2."""
    rng = np.random.default_rng(seed)
    if layout == "cube":
        position = rng.uniform(-1.0, 1.0, size=(3, a)).astype(np.float32)
        reach_mu, bound_mu = -3.0, -3.0
    elif layout == "clusters":
        centres, stds, rots = cluster_layout(2000)
        which = rng.integers(0, 64, size=a)
        local = _normal(rng, (a, 3)) * stds[which].astype(np.float32)
        position = np.ascontiguousarray((np.einsum("nij,nj->ni", rots[which].astype(np.float32), local)
                                         + centres[which].astype(np.float32)).T.astype(np.float32))
        reach_mu, bound_mu = -2.0, -3.3
    else:
        raise ValueError(f"unknown layout {layout}")
    feature = _normal(rng, (a, ANCHOR_FEAT))
    extent = np.empty((6, a), dtype=np.float32)
    extent[:3] = np.exp(_normal(rng, (3, a), reach_mu, 0.4))
    extent[3:] = np.exp(_normal(rng, (3, a), bound_mu, 0.8))
    offsets = _normal(rng, (a, k, 3))
    return dict(position=position, feature=feature, extent=extent, offsets=offsets, a=a, k=k)
