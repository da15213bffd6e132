"""CPU oracle of the AnchorDecoder: anchors + viewing position -> Gaussian primitives.

TEST INFRASTRUCTURE ONLY: imported by tests/, by __graft_entry__.smoke() and by the
cpu_baseline leg of bench.py.  It shares no code with the HIP library and imports nothing
from the product package.  Plain numpy in float64; library matrix products are the steps.

What it follows (LandMarkSystem technical report):
  Sec. 3.1     the AnchorDecoder is the Decoder component of the anchor-based Gaussian
               models (ScaffoldGSEncoding, OctreeGSEncoding): it turns the encoding's anchors
               into the Gaussian primitives that the rasteriser consumes
  Sec. 4.2.1   the steps the decoder is made of, by their timer names: the mask of the
               anchors to decode, the collation of an anchor's local feature with the view
               (without the distance), three dual-layer perceptrons (covariance, colour,
               neural opacity), the combination of their outputs with the anchor's own
               tensors, post-processing

The report names these steps and gives no formula for any of them.  What each computes is
taken from the anchor-based method that the named encodings implement (anchors that carry a
feature, per-axis extents and K offsets; view-dependent perceptrons that emit the attributes
of K primitives per anchor), restated here; every choice is a [reading]:

  1. mask [reading]: the anchors to decode arrive as a list of indices `visible`, computed
     beforehand (the report's pre-computed mask indices); order of the list = order of output.
  2. view [reading]: delta = position - camera position; dir = delta / |delta| (zero when
     |delta| = 0); the distance is not an input.
  3. input [reading]: x = [feature (F values), dir (3)]  (F + 3 values).
  4. perceptrons [reading]: y = W2 relu(W1 x + b1) + b2, one per attribute group, hidden width
     F; outputs of primitive j of the anchor are adjacent: opacity unit j, colour units
     3j..3j+2, covariance units 7j..7j+6 (three scale units, then four quaternion units).
  5. neural opacity [reading]: tanh(y); a primitive is kept only if that is > 0.
  6. colour [reading]: logistic function of its three units, used as the view-independent
     colour of the primitive (degree-0 SH coefficient (colour - 0.5) / Y_00).
  7. covariance [reading]: scale = extent[3:6] * logistic(first three units); rotation = the
     last four units as an unnormalised quaternion (w, x, y, z) (the rasteriser normalises).
  8. combination [reading]: centre = position + offsets[j] * extent[0:3].
  9. post-processing [reading]: the output keeps one slot per (list entry v, primitive j),
     slot v K + j; a primitive that is not kept gets opacity exactly 0 (the rasteriser culls
     every opacity below 1/255), so slots do not depend on rounding.

Precision: float64 from the float32 inputs.  The one decision (kept or not) is the sign of
the opacity perceptron's output; the GPU takes it in float32, so the tests treat slots whose
float64 output is within the float32 error bound of zero as undecided (either way is valid:
such a primitive has an opacity far below 1/255 and never reaches the image).  `bound`
returns that error bound: for a dot product accumulated in float32, |error| <= n u |w|.|x|.

View-frustum mask of the anchors [reading; Sec. 4.2.1 names a mask computation with pre-computed
indices, Sec. 4.2.2 the frustum test of boxes]: offline, every anchor gets the box that holds every
centre its primitives can take, position +- max_j |offset_j| * extent[0:3] per axis (float32, one
rounding per operation), and the largest scale any of them can take, max(extent[3:6]) (the logistic
factor is below 1).  Per frame an anchor is decoded only if that box passes the rasteriser oracle's
conservative box-against-frustum test (lmk_ref_voxel_visible: a box that fails cannot hold a
primitive that is binned); the primitives of an anchor that fails get opacity 0.  The decision is
taken in float32 by the same written formulas on both sides, so it is unique.

Pins (tests/test_oracle_anchor.py): closed forms with a zero second layer, with a
pass-through first layer, with a view-only first layer; the perceptron against
torch.nn.Linear/ReLU modules; translation, offset-scaling and list-permutation invariants;
the colour round trip through the rasteriser oracle's degree-0 SH evaluation.
"""
from __future__ import annotations

from types import SimpleNamespace

import numpy as np

Y00 = 0.5 * np.sqrt(1.0 / np.pi)          # degree-0 real spherical harmonic

GROUPS = (("opacity", 1), ("colour", 3), ("cov", 7))


def _logistic(y):
    return 1.0 / (1.0 + np.exp(-y))


def perceptron(p: dict, x: np.ndarray) -> np.ndarray:
    """Step 4: y = W2 relu(W1 x + b1) + b2 for every row of x.  w1 is (hidden, input), w2t is
    (hidden, output)."""
    w1, b1 = np.asarray(p["w1"], np.float64), np.asarray(p["b1"], np.float64)
    w2t, b2 = np.asarray(p["w2t"], np.float64), np.asarray(p["b2"], np.float64)
    h = np.maximum(x @ w1.T + b1, 0.0)
    return h @ w2t + b2


def view_input(anchors: dict, cam_pos, idx: np.ndarray) -> np.ndarray:
    """Steps 2-3: [feature, unit vector from the camera to the anchor]."""
    pos = np.asarray(anchors["position"], np.float64)[:, idx].T
    delta = pos - np.asarray(cam_pos, np.float64).reshape(1, 3)
    dist = np.sqrt((delta * delta).sum(axis=1, keepdims=True))
    direction = np.divide(delta, dist, out=np.zeros_like(delta), where=dist > 0)
    return np.concatenate([np.asarray(anchors["feature"], np.float64)[idx], direction], axis=1)


def decode(anchors: dict, mlp: dict, cam_pos, visible=None) -> SimpleNamespace:
    """Steps 1-9.  Returns float64 arrays in the rasteriser's layout, n = len(visible) * K:
    mean (3, n), scale (3, n), rot (4, n), opacity (n,), colour (3, n), sh_dc (3, n), and
    pre_opacity (n,) = the opacity perceptron's raw output."""
    a, k = int(anchors["a"]), int(anchors["k"])
    idx = np.arange(a, dtype=np.int64) if visible is None else np.asarray(visible, dtype=np.int64)
    v = len(idx)
    x = view_input(anchors, cam_pos, idx)
    y_op = perceptron(mlp["opacity"], x).reshape(v, k)
    y_col = perceptron(mlp["colour"], x).reshape(v, k, 3)
    y_cov = perceptron(mlp["cov"], x).reshape(v, k, 7)
    extent = np.asarray(anchors["extent"], np.float64)[:, idx].T            # (v, 6)
    pos = np.asarray(anchors["position"], np.float64)[:, idx].T             # (v, 3)
    off = np.asarray(anchors["offsets"], np.float64)[idx]                   # (v, k, 3)

    opacity = np.where(y_op > 0.0, np.tanh(y_op), 0.0)
    colour = _logistic(y_col)
    scale = extent[:, None, 3:6] * _logistic(y_cov[:, :, 0:3])
    rot = y_cov[:, :, 3:7]
    mean = pos[:, None, :] + off * extent[:, None, 0:3]

    n = v * k
    flat = lambda t, c: np.ascontiguousarray(t.reshape(n, c).T)
    colour_f = flat(colour, 3)
    return SimpleNamespace(n=n, k=k, v=v, mean=flat(mean, 3), scale=flat(scale, 3), rot=flat(rot, 4),
                           opacity=opacity.reshape(n), colour=colour_f, sh_dc=(colour_f - 0.5) / Y00,
                           pre_opacity=y_op.reshape(n))


def bound(anchors: dict, mlp: dict, cam_pos, visible=None) -> SimpleNamespace:
    """Float32 evaluation error bound of the three perceptrons' raw outputs, per slot:
    (n_1 + n_2 + 8) u (|W2| (|W1| |x| + |b1|) + |b2|), u = 2^-24, n_1 = F + 4 and n_2 = F + 1
    terms per dot product, 8 u for the rounding of the direction.  Shapes as decode's: opacity
    (n,), colour (3, n), cov (7, n)."""
    a, k = int(anchors["a"]), int(anchors["k"])
    idx = np.arange(a, dtype=np.int64) if visible is None else np.asarray(visible, dtype=np.int64)
    x = np.abs(view_input(anchors, cam_pos, idx))
    n = len(idx) * k
    out = {}
    for name, per in GROUPS:
        p = mlp[name]
        m1 = x @ np.abs(np.asarray(p["w1"], np.float64)).T + np.abs(np.asarray(p["b1"], np.float64))
        m2 = m1 @ np.abs(np.asarray(p["w2t"], np.float64)) + np.abs(np.asarray(p["b2"], np.float64))
        terms = (x.shape[1] + 1) + (m1.shape[1] + 1) + 8
        out[name] = np.ascontiguousarray((terms * 2.0 ** -24 * m2).reshape(n, per).T)
    return SimpleNamespace(opacity=out["opacity"][0], colour=out["colour"], cov=out["cov"])


def anchor_boxes(anchors: dict) -> SimpleNamespace:
    """Offline: per anchor the box of its primitives' possible centres and the bound of their scales,
    in float32 (box_lo, box_hi (a, 3); smax (a,))."""
    f32 = np.float32
    pos = np.asarray(anchors["position"], f32).T                                  # (a, 3)
    ext = np.asarray(anchors["extent"], f32)
    off = np.asarray(anchors["offsets"], f32)                                     # (a, k, 3)
    a = int(anchors["a"])
    if a == 0:
        z = np.zeros((0, 3), f32)
        return SimpleNamespace(num_voxels=0, box_lo=z, box_hi=z.copy(), smax=np.zeros(0, f32))
    reach = (np.abs(off) * ext[0:3].T[:, None, :]).astype(f32).max(axis=1)        # (a, 3)
    return SimpleNamespace(num_voxels=a, box_lo=np.ascontiguousarray(pos - reach, f32),
                           box_hi=np.ascontiguousarray(pos + reach, f32),
                           smax=np.ascontiguousarray(ext[3:6].max(axis=0), f32))


def anchors_visible(anchors: dict, cam: dict) -> np.ndarray:
    """Per anchor: False only if none of its primitives can be binned for this camera."""
    from oracle import ref
    return ref.voxels_visible(anchor_boxes(anchors), cam).astype(bool)


def decode_culled(anchors: dict, mlp: dict, cam: dict) -> SimpleNamespace:
    """decode() of every anchor, with the primitives of anchors that fail the frustum test at opacity 0.
    `.visible` is the per-anchor mask."""
    d = decode(anchors, mlp, cam["cam_pos"])
    d.visible = anchors_visible(anchors, cam)
    d.opacity = np.where(np.repeat(d.visible, d.k), d.opacity, 0.0)
    return d


def as_scene(dec: SimpleNamespace) -> dict:
    """The decoded primitives as a float32 scene of SH degree 0 for the rasteriser oracle."""
    sh = np.zeros((16, 3, dec.n), dtype=np.float32)
    sh[0] = dec.sh_dc.astype(np.float32)
    return dict(mean=dec.mean.astype(np.float32), scale=dec.scale.astype(np.float32),
                rot=dec.rot.astype(np.float32), opacity=dec.opacity.astype(np.float32),
                sh=sh, sh_degree=0, n=dec.n)
