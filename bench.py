#!/usr/bin/env python3
"""Benchmark of the splatting forward path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--cfg 2] [--no-cpu-baseline]

A step is one pass over the configuration's seeded viewpoints (8 for configs 1-3, 1 for configs 0
and 4), each frame being lmk_gs_preprocess_culled (or lmk_gs_preprocess with --voxel 0) +
lmk_gs_bin_sort + lmk_gs_render, all enqueued on one stream with no host synchronisation, so that
every viewpoint weighs the same whatever --steps is.  The scene is reordered into voxels once,
before anything is timed.  Inputs are resident in HBM before the timed region.  Prints ONE JSON
line (metric = frames/s) that also carries Gaussian-pixel blends/s, per-stage times, the roofline
of the dominant kernel and of the HBM-bound stages, and the CPU oracle timed on the same
workload as a baseline.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

# voxel edge per configuration for the offline reordering (a few hundred primitives per voxel);
# 0 = off (configs 0 and 4: one viewpoint that sees everything); the spatial order also lets the
# counting workgroups of stage 2 combine the pairs of neighbouring primitives per tile
VOXEL_SIZE = {0: 0.0, 1: 1.0, 2: 2.0, 3: 40.0, 4: 0.0}

HBM_PEAK_GBS = 8000.0        # MI355X HBM3E
FP32_PEAK_TFLOPS = 157.3     # 256 CU x 128 lanes x 2 flop x 2.4 GHz (vector FP32, packed-FMA rate)
FP32_MFMA_PEAK_TFLOPS = 157.3   # dense fp32 MFMA: 256 CU x 256 flop per cycle x 2.4 GHz


def algorithmic_bytes(n, n_near, n_bin, D, tiles, long_lists, binning=0, n_proc=None, voxels=0, cov_cache=False):
    """HBM bytes the method itself must move in preprocess + bin_sort (per frame), for the
    scheme this library runs.

    preprocess: tiles_touched 4 B for every primitive; mean 12 B for every primitive of a
    group the voxel filter lets through (all of them without the filter; n_near and n_bin count
    only those); scale, rotation, opacity 32 B for those past the near plane (28 B with the
    parameter cache: six covariance entries instead of seven rotation and scale values); SH 192 B +
    outputs 64 B (depth 4, rect 8, feature record 48, reread count 4) for binned ones, plus the
    4 B mask of kept tiles under binning rule 1; the voxel table, 32 B per voxel + 8 B per group.
    bin_sort (pairs are written straight into their tile's slice, no partition passes):
    count: tiles_touched 4 + rect 8 (+ mask 4 under rule 1) for every primitive of a group that
    was projected; scan: 16 B per tile; emit: the same again + depth 4, and the 8-byte composite
    (depth bits, index) of every pair written; per-tile sort: 8 B read + 12 B written per pair;
    a list of 4097 .. 16384 pairs is sorted in chunks and then goes through two merge rounds
    between the pair buffers (the second a copy for a list of two chunks), 24 B per pair each; a
    list longer than 16384 pairs is merged, 24 B per pair and doubling round.  The (tile, run
    start) lists of the counting workgroups and the second reads of the few rectangles above 32
    tiles are not charged.  `long_lists`: the lengths above 4096.
    """
    n_proc = n if n_proc is None else n_proc
    b_pre = 4 * n + 12 * n_proc + (28 if cov_cache else 32) * n_near + (260 if binning else 256) * n_bin + 32 * voxels + (8 * ((n + 255) // 256) if voxels else 0)
    per_prim = 16 if binning else 12
    b_count = per_prim * n_proc + 16 * tiles
    b_emit = (per_prim + 4) * n_proc + 8 * D
    b_tsort = 20 * D
    for L in long_lists:
        if L <= 16384:
            b_tsort += 48 * L
            continue
        rounds = 0
        run = 16384
        while run < L:
            run *= 2
            rounds += 1
        b_tsort += 24 * L * rounds
    # context only: what a single-level LSD radix sort of the 64-bit keys (8-bit digits over the
    # 32 depth bits + the tile bits) with duplication in index order and a range pass would move
    tile_bits = max(1, (tiles - 1).bit_length())
    passes = (32 + tile_bits + 7) // 8
    b_radix = 20 * n_bin + 12 * D + D * (8 + 24 * passes) + 8 * D
    return dict(preprocess=b_pre, count=b_count, emit=b_emit, tile_sort=b_tsort,
                total=b_pre + b_count + b_emit + b_tsort, radix_scheme_bin_sort=b_radix)


def timed_steps(steps):
    """The steps of the timed region that carry event records (for the stage times and the kernel
    durations of the roofline objects): every fourth, the others run as a caller would run them --
    four event records per frame cost about 3 % of the frame rate.  Short runs record every step."""
    every = 4 if steps >= 8 else 1
    return [s for s in range(steps) if s % every == 0], every


def committed_counters(cfg, binning):
    """VALU counters of the blend kernel from the rocprofv3 --pmc summary committed under profiles/
    (lines `cfgN binningB blend_kernel <name> <value>`); {} when there is none for this workload."""
    path = os.path.join(ROOT, "profiles", "blend_counters.txt")
    out = {}
    try:
        with open(path) as f:
            for line in f:
                t = line.split()
                if len(t) == 5 and t[0] == f"cfg{cfg}" and t[1] == f"binning{binning}" and t[2] == "blend_kernel":
                    out[t[3]] = float(t[4])
    except OSError:
        return {}
    return out


def _projection_backward_report(ms, n, stats, nviews):
    """lmk_gs_preprocess_backward: HBM-bound.  Algorithmic bytes per call: 4 B (tile count) for every
    primitive; a binned one reads its 36 B of feature-record gradient, 40 B of mean, scale and rotation
    and 192 B of SH, and every primitive gets 44 B + 192 B of gradient written (zeros when not binned)."""
    byts = [4.0 * n + 268.0 * stats[v]["n_bin"] + 236.0 * n for v in range(nviews)]
    gbs = sum(byts) / (sum(ms) * 1e-3) / 1e9
    return {"entry": "lmk_gs_preprocess_backward", "ms_per_call": sum(ms) / len(ms),
            "per_view_ms": [float(x) for x in ms],
            "roofline": {"kernel": "preprocess_backward_kernel", "bound": "hbm", "achieved": gbs,
                         "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": gbs / HBM_PEAK_GBS, "traffic": None,
                         "bytes_per_call": sum(byts) / len(byts)}}


def committed_traffic(cfg, binning, workload=None):
    """HBM bytes per launch measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (already scaled
    by the copy-kernel calibration), from the summary committed under profiles/.  None when
    there is no measurement for this workload."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic.txt")
    out = {}
    try:
        with open(path) as f:
            for line in f:
                t = line.split()
                if len(t) == 5 and t[0] == (workload or f"cfg{cfg}") and t[1] == f"binning{binning}":
                    out[t[2]] = float(t[3]) + float(t[4])
    except OSError:
        return {}
    return out


def anchor_bench(args):
    """Anchor-model frames: lmk_gs_anchor_decode + preprocess + bin_sort + render per viewpoint.

    Algorithmic work of the decode kernel per listed anchor (k primitives, F = 32 features):
    flops = 2 (3 F (F + 3) + F 11 k) for the two layers of the three perceptrons (13 760 at k = 10;
    the activations are not counted); bytes = 4 (3 + F + 6 + 3 k) read + 4 k (3 + 3 + 4 + 1 + 4) written
    (884 at k = 10).  The perceptrons run on the matrix cores in fp32, so the roofline is the dense
    fp32 MFMA peak; the padding of the matrix tiles (36 inputs, outputs in tiles of 32) is not counted."""
    import numpy as np
    import torch
    from paper_2503_21364_amd import binding as B
    from paper_2503_21364_amd import scenes

    a, k, F = args.anchors, scenes.ANCHOR_K, scenes.ANCHOR_FEAT
    anchors = scenes.make_anchor_scene(a, seed=6000, k=k, layout="clusters")
    mlp = scenes.make_decoder(seed=7000, k=k)
    spec = scenes.CONFIGS[2]
    W, H = spec["width"], spec["height"]
    cams = [dict(c, binning=args.binning) for c in scenes.make_cameras(2)]
    if args.views is not None:
        cams = cams[:max(1, args.views)]
    ccams = [B.make_camera(c) for c in cams]
    nviews = len(cams)
    masked = not args.no_anchor_mask
    if masked:
        # offline, not timed: anchors in voxel order, per-anchor boxes; the oracle leg uses the same order
        anchors = B.reorder_anchors(anchors, 2.0)
        aindex = B.AnchorIndex(anchors)
    dev = B.AnchorScene(anchors, mlp)
    dec = B.DecodedScene(a, k)
    scene = dec.scene()
    n = scene.n

    def decode(c, cc):
        if masked:
            B.anchor_decode_culled(dev, aindex, cc, dec)
        else:
            B.anchor_decode(dev, c["cam_pos"], dec)

    def project(cc, frame_):
        B.preprocess(scene, cc, frame_, index=aindex if masked else None)

    fr = B.Frame(n, W, H, 64_000_000)
    Ds = []
    in_view = []
    for c, cc in zip(cams, ccams):
        decode(c, cc)
        project(cc, fr)
        B.bin_sort(cc, fr)
        B.render(cc, fr)
        D, status = B.read_status(fr)
        assert status == B.OK, f"status {status} in the sizing run"
        Ds.append(D)
        in_view.append(float(aindex.visible[:a].float().mean().item()) if masked else 1.0)
    kept = float((dec.opacity > 0).float().mean().item())
    del fr
    torch.cuda.empty_cache()
    capacity = int(max(Ds) * 1.25) + 4096
    fr = B.Frame(n, W, H, capacity)

    def frame(i, marks=None):
        c, cc = cams[i % nviews], ccams[i % nviews]
        if marks: marks[0].record()
        decode(c, cc)
        if marks: marks[1].record()
        project(cc, fr)
        if marks: marks[2].record()
        B.bin_sort(cc, fr)
        if marks: marks[3].record()
        B.render(cc, fr)
        if marks: marks[4].record()

    if args.pmc_calibration:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")      # 1 GiB
        dst = torch.empty_like(src)
        for _ in range(4):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
        torch.cuda.empty_cache()

    nframes = args.steps * nviews                   # a step = one pass over the viewpoints
    for i in range(args.warmup * nviews):
        frame(i)
    torch.cuda.synchronize()
    ev = lambda: torch.cuda.Event(enable_timing=True)
    recorded_steps, events_every = timed_steps(args.steps)
    recorded = [s * nviews + v for s in recorded_steps for v in range(nviews)]
    marks = {i: [ev() for _ in range(5)] for i in recorded}
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(nframes):
        frame(i, marks.get(i))
    torch.cuda.synchronize()
    total_s = time.perf_counter() - t0
    _, status = B.read_status(fr)
    assert status == B.OK, f"status {status}"
    stage = lambda j: np.array([marks[i][j].elapsed_time(marks[i][j + 1]) for i in recorded])
    t_dec, t_pre, t_sort, t_blend = stage(0), stage(1), stage(2), stage(3)

    # algorithmic work of a launch: anchors in view are decoded (flops, all their bytes); an anchor out of
    # view costs its 32-byte box, its mask byte (written, then read) and the k opacities written
    view_of = np.array(recorded) % nviews
    seen = np.array(in_view)[view_of] * a
    flops = float((2.0 * (3 * F * (F + 3) + F * 11 * k) * seen).mean())
    per_seen = 4.0 * (3 + F + 6 + 3 * k) + 4.0 * k * 15
    byts = float((per_seen * seen + ((34.0 * a + (a - seen) * 4.0 * k) if masked else 0.0)).mean())
    tf = flops / (t_dec.mean() * 1e-3) / 1e12
    # the committed counter measurement is of the default command of this mode
    traffic = committed_traffic(2, args.binning, f"anchors{a}" + ("" if masked else "-nomask")) if args.views is None else {}
    out = {
        "metric": "frames/s, anchor model: decode + 1080p render",
        "value": nframes / total_s, "unit": "frames/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": 1e3 * total_s / args.steps, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"frames_per_step": nviews, "event_records_every_steps": events_every, "workload": f"anchors: {a} anchors (config 2's clusters) x {k} primitives = {n} candidate "
                               f"Gaussians decoded per frame, {W}x{H}, {nviews} seeded viewpoints of config 2",
                   "binning": args.binning, "kept_fraction": kept, "pairs_per_frame_mean": float(np.mean(Ds)),
                   "capacity": capacity, "frustum_mask": masked,
                   "anchors_in_view": [round(x, 4) for x in in_view]},
        "stage_ms": {"anchor_decode": float(t_dec.mean()), "preprocess": float(t_pre.mean()),
                     "bin_sort": float(t_sort.mean()), "render": float(t_blend.mean())},
        "decode_ms_per_view": [float(t_dec[view_of == v].mean()) for v in range(nviews) if (view_of == v).any()],
        "preprocess_ms_per_view": [float(t_pre[view_of == v].mean()) for v in range(nviews) if (view_of == v).any()],
        "roofline": {"kernel": "anchor_decode_kernel", "bound": "mfma", "achieved": tf, "peak": FP32_MFMA_PEAK_TFLOPS,
                     "unit": "TFLOP/s", "frac": tf / FP32_MFMA_PEAK_TFLOPS,
                     "traffic": traffic.get("anchor_decode_kernel"),
                     "avg_launch_ms": float(t_dec.mean()), "flops_per_launch": flops,
                     "hbm_GBs": byts / (t_dec.mean() * 1e-3) / 1e9, "bytes_per_launch": byts,
                     "note": "time of the whole decode call (with the mask: box test kernel + decode kernel), "
                             "work of the anchors in view, both as means over the views"},
    }
    if not args.no_cpu_baseline:
        from oracle import anchor_ref as AR
        from oracle import ref
        c0 = time.perf_counter()
        d = AR.decode_culled(anchors, mlp, cams[0]) if masked else AR.decode(anchors, mlp, cams[0]["cam_pos"])
        c1 = time.perf_counter()
        ofr = ref.render_frame(AR.as_scene(d), dict(cams[0], binning=0))
        c2 = time.perf_counter()
        cores = len(os.sched_getaffinity(0))
        omp = os.environ.get("OMP_NUM_THREADS")
        threads = min(cores, int(omp)) if omp and omp.isdigit() else cores
        out["cpu_baseline"] = dict(value=1.0 / (c2 - c0), unit="frames/s", cores=threads, kind="oracle",
                                   sample=f"viewpoint 0 only: decode of all {a} anchors ({c1 - c0:.1f} s, numpy float64) "
                                          f"and one whole frame of the rasteriser oracle ({c2 - c1:.1f} s)",
                                   decode_anchors_per_s=a / (c1 - c0))
        del ofr
    print(json.dumps(out), flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20,
                    help="timed steps; a step is one pass over the configuration's viewpoints (8 frames for configs 1-3)")
    ap.add_argument("--warmup", type=int, default=2, help="untimed steps before them")
    ap.add_argument("--cfg", type=int, default=2, help="configuration 0-4 (2 is the headline: 3M Gaussians, 1080p)")
    ap.add_argument("--n", type=int, default=None, help="override the primitive count (reported in config)")
    ap.add_argument("--binning", type=int, default=1, choices=(0, 1),
                    help="0: a pair for every tile of a support rectangle; 1 (default): only for tiles the "
                         "splat can reach (same image, fewer pairs)")
    ap.add_argument("--voxel", type=float, default=None,
                    help="edge of the voxels for the offline spatial reordering + per-frame view-frustum filtering "
                         "of voxels (default: a size per configuration; 0 = primitives in the order drawn, "
                         "no filtering)")
    ap.add_argument("--backward", action="store_true",
                    help="also time lmk_gs_render_backward (gradient through the compositing) on every viewpoint "
                         "and add a \"backward\" object to the JSON line; the headline value is unchanged")
    ap.add_argument("--anchors", type=int, default=0, metavar="A",
                    help="anchor-model mode: A anchors of the cluster layout (300000 gives 3 M candidate primitives) "
                         "are decoded by lmk_gs_anchor_decode in every frame and rendered by the three calls; the "
                         "JSON line then reports that pipeline and the roofline of the decode kernel")
    ap.add_argument("--no-anchor-mask", action="store_true",
                    help="anchor-model mode without the view-frustum mask: every anchor is decoded and every slot "
                         "projected in every frame")
    ap.add_argument("--no-cov-cache", action="store_true",
                    help="compute every primitive's 3D covariance from rotation and scale in every frame instead "
                         "of reading the parameter cache built once per scene")
    ap.add_argument("--streams", type=int, default=1,
                    help="frames in flight: with S > 1, frame i runs on stream i mod S with its own buffers, so the "
                         "latency-bound kernels of one frame overlap the bandwidth- and ALU-bound ones of another "
                         "(throughput mode; per-stage times then include the overlap)")
    ap.add_argument("--views", type=int, default=None, help="use only the first K viewpoints of the configuration")
    ap.add_argument("--no-cpu-baseline", action="store_true", help="skip the oracle leg (no blends/s either)")
    ap.add_argument("--pmc-calibration", action="store_true",
                    help="before timing, run four plain device copies of 1 GiB (known traffic, for scaling "
                         "rocprofv3 FETCH_SIZE / WRITE_SIZE readings)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (no collectives, no sharding); "
              "use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2503_21364_amd import binding as B
    from paper_2503_21364_amd import scenes

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    B.lib()   # fails loudly if the HIP library is not built
    if args.anchors > 0:
        return anchor_bench(args)
    spec = scenes.CONFIGS[args.cfg]
    n = spec["n"] if args.n is None else args.n
    W, H = spec["width"], spec["height"]
    scene = scenes.make_scene(args.cfg, n=n)
    cams = scenes.make_cameras(args.cfg)
    if args.views is not None:
        cams = cams[:max(1, args.views)]
    cams = [dict(c, binning=args.binning) for c in cams]
    ccams = [B.make_camera(c) for c in cams]
    if args.voxel is None:
        args.voxel = VOXEL_SIZE[args.cfg]
    index = None
    if args.voxel > 0.0:
        # offline step, not timed: from here on "the scene" is the reordered scene, for the oracle too
        index = B.VoxelIndex(scene, args.voxel)
        scene = index.reorder(scene)
        index.upload()
    dev = B.Scene(scene)
    if not args.no_cov_cache:
        dev.build_cov3d()          # once per scene, not timed
    tiles = ((W + 15) // 16) * ((H + 15) // 16)

    # size the pair buffers from a dry run of every viewpoint (not timed)
    probe_cap = 64_000_000 if args.cfg != 4 else 7_000_000_000
    fr = B.Frame(n, W, H, probe_cap)
    Ds, stats = [], []
    nb = (n + B.PRE_BLOCK - 1) // B.PRE_BLOCK
    flags = torch.ones(max(nb, 1), dtype=torch.uint8, device="cuda")
    for cc in ccams:
        B.preprocess(dev, cc, fr, index=index, block_visible=flags if index is not None else None)
        B.bin_sort(cc, fr)
        D, status = B.read_status(fr)
        assert status == B.OK, f"status {status} in the sizing run"
        tt = fr.tiles_touched[:n]
        n_bin = int((tt > 0).sum().item())
        lens = (fr.tile_offsets[1:] - fr.tile_offsets[:-1])
        Ds.append(D)
        stats.append(dict(D=D, n_bin=n_bin, long_lists=[int(x) for x in lens[lens > 4096].tolist()],
                          processed=flags[:nb].bool().cpu().numpy().copy()))
    del fr
    torch.cuda.empty_cache()
    capacity = int(max(Ds) * 1.25) + 4096
    S = max(1, args.streams)
    frames = [B.Frame(n, W, H, capacity) for _ in range(S)]
    streams = [None] if S == 1 else [torch.cuda.Stream() for _ in range(S)]
    fr = frames[0]

    if args.pmc_calibration:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")      # 1 GiB
        dst = torch.empty_like(src)
        for _ in range(4):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
        torch.cuda.empty_cache()

    nviews = len(ccams)
    nframes = args.steps * nviews                   # a step = one pass over the viewpoints
    ev = lambda: torch.cuda.Event(enable_timing=True)
    for i in range(args.warmup * nviews):
        B.render_frame(dev, ccams[i % nviews], frames[i % S], stream=streams[i % S], index=index)
    torch.cuda.synchronize()
    for f in frames[:min(S, max(args.warmup * nviews, 1))]:
        _, status = B.read_status(f)
        assert status == B.OK, f"status {status}"

    recorded_steps, events_every = timed_steps(args.steps)
    recorded = [s * nviews + v for s in recorded_steps for v in range(nviews)]
    marks = {i: [ev(), ev(), ev(), ev()] for i in recorded}
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(nframes):
        cc = ccams[i % nviews]
        m = marks.get(i)
        f, st = frames[i % S], streams[i % S]
        if m is None:
            B.render_frame(dev, cc, f, stream=st, index=index)
            continue
        m[0].record(st)
        B.preprocess(dev, cc, f, stream=st, index=index)
        m[1].record(st)
        B.bin_sort(cc, f, stream=st)
        m[2].record(st)
        B.render(cc, f, stream=st)
        m[3].record(st)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    total_s = t1 - t0
    ms_per_step = 1e3 * total_s / args.steps
    fps = nframes / total_s
    for f in frames:
        _, status = B.read_status(f)
        assert status == B.OK, f"status {status}"

    ms = [marks[i] for i in recorded]
    t_pre = np.array([m[0].elapsed_time(m[1]) for m in ms])
    t_sort = np.array([m[1].elapsed_time(m[2]) for m in ms])
    t_blend = np.array([m[2].elapsed_time(m[3]) for m in ms])
    t_frame = np.array([m[0].elapsed_time(m[3]) for m in ms])
    view_of = np.array(recorded) % nviews

    # ---- CPU oracle: counts E, C (algorithmic pairs) and the baseline time
    cpu = None
    E = C = None
    bwd_ms = None
    if args.backward:
        # per viewpoint: the forward frame once (not timed), then the gradient call a few times with
        # HIP events around it; random dL/d rgb and dL/dT, resident before the timed region
        gen = torch.Generator(device="cuda"); gen.manual_seed(1)
        g_rgb = torch.randn(3, H, W, device="cuda", generator=gen)
        g_T = torch.randn(H, W, device="cuda", generator=gen)
        g_feat = torch.empty(max(n, 1), B.FEAT_STRIDE, dtype=torch.float32, device="cuda")
        grads = B.SceneGrads(dev)
        reps = 5
        bwd_ms, bwd_pre_ms = [], []
        for v in range(nviews):
            B.render_frame(dev, ccams[v], fr, index=index)
            B.render_backward(ccams[v], fr, g_rgb, g_T, g_feat)          # warm-up
            B.preprocess_backward(dev, ccams[v], fr, g_feat, grads)
            torch.cuda.synchronize()
            e0, e1, e2 = ev(), ev(), ev()
            e0.record()
            for _ in range(reps):
                B.render_backward(ccams[v], fr, g_rgb, g_T, g_feat)
            e1.record()
            for _ in range(reps):
                B.preprocess_backward(dev, ccams[v], fr, g_feat, grads)
            e2.record()
            torch.cuda.synchronize()
            bwd_ms.append(e0.elapsed_time(e1) / reps)
            bwd_pre_ms.append(e1.elapsed_time(e2) / reps)
        del g_rgb, g_T, g_feat, grads

    n_near = None
    estimated = False
    if not args.no_cpu_baseline and args.cfg == 4 and args.n is None:
        # The frame is too large for the oracle to bin whole (6e9 pairs): it is timed on a sample -- all
        # primitives projected, then three bands of three tile rows each (top, middle, bottom of the
        # image) binned and blended -- and the frame time and the pair counts E, C are scaled up from
        # the sampled pixel rows.
        from oracle import ref
        estimated = True
        cam0 = dict(cams[0], binning=0)
        c0 = time.perf_counter()
        pre = ref.preprocess(scene, cam0)
        order = ref.depth_order(pre)
        t_head = time.perf_counter() - c0
        ty = (H + 15) // 16
        rows, t_bands, e_sum, c_sum, px = 0, 0.0, 0, 0, 0
        for frac in (0.1, 0.5, 0.9):
            a = min(max(int(frac * ty) - 1, 0), max(ty - 3, 0))
            c1 = time.perf_counter()
            band = ref.band_lists(pre, cam0, a, min(a + 3, ty), order)
            img = ref.render_band(pre, cam0, band)
            t_bands += time.perf_counter() - c1
            rows += min(a + 3, ty) - a
            e_sum += int(img.E.sum()); c_sum += int(img.C.sum()); px += img.E.size
            del band, img
        scale = (W * H) / px
        E, C = [e_sum * scale], [c_sum * scale]
        t_frame_cpu = t_head + t_bands * ty / rows
        proc = np.repeat(stats[0]["processed"], B.PRE_BLOCK)[:n]
        stats[0]["n_proc"] = int(proc.sum())
        n_near = [int(((pre.stage != ref.CULL_NEAR) & proc).sum())]
        D_ref = int(pre.tiles_touched.astype(np.uint64).sum()) if args.binning == 0 else \
            int(ref.preprocess(scene, cams[0]).tiles_touched.astype(np.uint64).sum())
        assert D_ref == stats[0]["D"], "GPU and oracle disagree on the pair count"
        cores = len(os.sched_getaffinity(0))
        omp = os.environ.get("OMP_NUM_THREADS")
        threads = min(cores, int(omp)) if omp and omp.isdigit() else cores
        cpu = dict(value=1.0 / t_frame_cpu, unit="frames/s", cores=threads, kind="oracle",
                   sample=f"cfg 4: every primitive projected and depth-ordered ({t_head:.1f} s), then {rows} of the "
                          f"{ty} tile rows binned and blended in three bands ({t_bands:.1f} s; binning rule 0); frame "
                          f"time and pair counts scaled up from the sampled rows",
                   blends_per_s=e_sum / t_bands)
        del pre, order
    elif not args.no_cpu_baseline:
        from oracle import ref
        E, C, n_near, cpu_t = [], [], [], []
        sample_views = list(range(nviews))
        for v in sample_views:
            # the timed baseline and the pair counts E, C of the metric use the plain binning
            # rule (a pair for every tile of the support rectangle), whatever rule the GPU ran
            c0 = time.perf_counter()
            ofr = ref.render_frame(scene, dict(cams[v], binning=0))
            cpu_t.append(time.perf_counter() - c0)
            E.append(int(ofr.img.E.sum())); C.append(int(ofr.img.C.sum()))
            proc = np.repeat(stats[v]["processed"], B.PRE_BLOCK)[:n]
            stats[v]["n_proc"] = int(proc.sum())
            n_near.append(int(((ofr.pre.stage != ref.CULL_NEAR) & proc).sum()))
            D_ref = ofr.binned.D if args.binning == 0 else \
                int(ref.preprocess(scene, cams[v]).tiles_touched.astype(np.uint64).sum())
            assert D_ref == stats[v]["D"], "GPU and oracle disagree on the pair count"
            del ofr
        cores = len(os.sched_getaffinity(0))
        omp = os.environ.get("OMP_NUM_THREADS")
        threads = min(cores, int(omp)) if omp and omp.isdigit() else cores
        cpu = dict(value=len(sample_views) / sum(cpu_t), unit="frames/s", cores=threads, kind="oracle",
                   sample=f"cfg {args.cfg}: one whole frame (preprocess, bin+sort, blend; binning rule 0) for each "
                          f"of its {len(sample_views)} viewpoints, {sum(cpu_t):.1f} s of oracle time",
                   blends_per_s=sum(E) / sum(cpu_t))

    out = {
        "metric": "frames/s, 1080p render of 3M Gaussians (whole forward path: preprocess + bin/sort + blend)"
                  if args.cfg == 2 and args.n is None and args.views is None else f"frames/s, config {args.cfg}",
        "value": fps, "unit": "frames/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"frames_per_step": nviews, "event_records_every_steps": events_every,
                   "workload": f"cfg{args.cfg}: {n} Gaussians, {W}x{H}, 16x16 tiles, SH degree 3, "
                               f"{nviews} seeded viewpoints rendered back-to-back",
                   "binning": args.binning, "pairs_per_frame_mean": float(np.mean(Ds)), "capacity": capacity,
                   "frames_in_flight": S, "parameter_cache": not args.no_cov_cache,
                   "voxel_filter": None if index is None else
                   {"voxel_size": args.voxel, "voxels": index.num_voxels,
                    "note": "primitives reordered offline into voxels; voxels filtered against the frustum per frame"}},
        "stage_ms": {"preprocess": float(t_pre.mean()), "bin_sort": float(t_sort.mean()),
                     "render": float(t_blend.mean())},
        "frame_ms": {"mean": float(t_frame.mean()), "median": float(np.median(t_frame)), "min": float(t_frame.min())},
        "per_view": [{"pairs": int(Ds[v]), "binned": stats[v]["n_bin"],
                      "preprocess_ms": float(t_pre[view_of == v].mean()),
                      "bin_sort_ms": float(t_sort[view_of == v].mean()),
                      "render_ms": float(t_blend[view_of == v].mean())} for v in range(nviews)
                     if (view_of == v).any()],
    }
    if E is not None:
        Ev = np.array(E, dtype=np.float64); Cv = np.array(C, dtype=np.float64)
        # blends/s: algorithmic evaluated pairs of each step's view over that step's render time
        blends = Ev[view_of].sum() / (t_blend.sum() * 1e-3)
        flops = (14.0 * Ev + 10.0 * Cv)[view_of].sum()
        tf = flops / (t_blend.sum() * 1e-3) / 1e12
        out["blends_per_s"] = blends
        if estimated:
            out["blends_note"] = "E and C are scaled up from the sampled tile rows of the CPU baseline"
        # the committed measurement is of the default command of each configuration
        traffic = committed_traffic(args.cfg, args.binning) \
            if args.n is None and args.views is None and args.voxel == VOXEL_SIZE[args.cfg] else {}
        out["roofline"] = {"kernel": "blend_kernel", "bound": "alu", "achieved": tf, "peak": FP32_PEAK_TFLOPS,
                           "unit": "TFLOP/s", "frac": tf / FP32_PEAK_TFLOPS, "traffic": traffic.get("blend_kernel"),
                           "avg_launch_ms": float(t_blend.mean()),
                           "flops_per_launch": float(flops / nframes),
                           "note": "algorithmic flops 14 E + 10 C (E, C counted by the oracle under binning rule 0) "
                                   "over the blend kernel's time; the instruction-issue view is in valu_counters"}
        counters = committed_counters(args.cfg, args.binning) \
            if args.n is None and args.views is None and args.voxel == VOXEL_SIZE[args.cfg] else {}
        if counters:
            out["roofline"]["valu_counters"] = counters
        byts, byts_pre, byts_radix = [], [], []
        for v in range(nviews):
            ab = algorithmic_bytes(n, n_near[v], stats[v]["n_bin"], stats[v]["D"], tiles,
                                   stats[v]["long_lists"], args.binning, stats[v]["n_proc"],
                                   0 if index is None else index.num_voxels, not args.no_cov_cache)
            byts.append(ab["total"]); byts_pre.append(ab["preprocess"]); byts_radix.append(ab["radix_scheme_bin_sort"])
        byts = np.array(byts, dtype=np.float64); byts_pre = np.array(byts_pre, dtype=np.float64)
        byts_radix = np.array(byts_radix, dtype=np.float64)
        gbs = byts[view_of].sum() / ((t_pre.sum() + t_sort.sum()) * 1e-3) / 1e9
        gbs_pre = byts_pre[view_of].sum() / (t_pre.sum() * 1e-3) / 1e9
        gbs_sort = (byts - byts_pre)[view_of].sum() / (t_sort.sum() * 1e-3) / 1e9
        gbs_radix = (byts_pre + byts_radix)[view_of].sum() / ((t_pre.sum() + t_sort.sum()) * 1e-3) / 1e9
        out["roofline_hbm_stages"] = {"kernels": "preprocess + block scan + count + tile scan + emit + per-tile sorts",
                                      "bound": "hbm", "achieved": gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                                      "frac": gbs / HBM_PEAK_GBS, "traffic": traffic.get("preprocess+bin_sort"),
                                      "preprocess_GBs": gbs_pre, "bin_sort_GBs": gbs_sort,
                                      "bytes_per_frame": float(byts.mean()),
                                      "radix_scheme_equivalent_GBs": gbs_radix,
                                      "note": "achieved = bytes of the scheme this library runs (no partition passes) over "
                                              "the two stages' time; radix_scheme_equivalent_GBs charges the same time with "
                                              "what a single-level 64-bit LSD radix sort of the same pairs would have to "
                                              "move -- context for comparisons across schemes, not a roofline claim"}
        if bwd_ms is not None:
            # algorithmic flops of the gradient call: both passes evaluate alpha for every visited pair
            # (14 E each, E as counted by the oracle), pass 1 also composites (10 C), pass 2 spends 45 per
            # composited pair (1 / (1 - alpha), T_i, w: 4; dL/dalpha: 14; S and the colour gradient: 9;
            # opacity, conic and mean gradients: 18)
            bflops = 28.0 * Ev + 55.0 * Cv
            btf = bflops.sum() / (sum(bwd_ms) * 1e-3) / 1e12
            out["backward"] = {"entry": "lmk_gs_render_backward", "ms_per_call": float(np.mean(bwd_ms)),
                               "per_view_ms": [float(x) for x in bwd_ms],
                               "pairs_per_s": float(Ev.sum() / (sum(bwd_ms) * 1e-3)),
                               "projection": _projection_backward_report(bwd_pre_ms, n, stats, nviews),
                               "roofline": {"kernel": "blend_backward_kernel", "bound": "alu", "achieved": btf,
                                            "peak": FP32_PEAK_TFLOPS, "unit": "TFLOP/s",
                                            "frac": btf / FP32_PEAK_TFLOPS, "traffic": None,
                                            "flops_per_launch": float(bflops.mean())}}
        out["cpu_baseline"] = cpu
    elif bwd_ms is not None:
        out["backward"] = {"entry": "lmk_gs_render_backward", "ms_per_call": float(np.mean(bwd_ms)),
                           "per_view_ms": [float(x) for x in bwd_ms],
                           "projection": _projection_backward_report(bwd_pre_ms, n, stats, nviews)}
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
