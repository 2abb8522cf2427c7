#!/usr/bin/env python3
"""Benchmark of the fusion hot path on one MI355X.

One step = one pass of the whole path over one synthetic scene already resident in HBM:
aura_fuse_scores (visibility mask and view counts, fusion, scoring) -> aura_property_integrate
(--staged: aura_project_visibility, aura_fuse_features, aura_material_scores, aura_property_integrate).
Prints ONE JSON line: whole-path throughput in fused point-views per second, the roofline figure
of the dominant call (the fusion, HBM bound on writing the fused rows) measured with events on the
launch stream in a run of its own right after the timed steps, and the CPU oracle timed on a bounded sample of the
same workload.
"""
import argparse
import gc
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)
sys.path.insert(0, os.path.join(ROOT, "tests"))

HBM_PEAK_GBPS = 8000.0   # MI355X HBM3E


def fuse_algorithmic_bytes(s):
    """Each input read once, the fused rows and counts written once."""
    elt = 4 if s.feat_dtype == "f32" else 2
    return (12 * s.N + 64 * s.n_views + 4 * s.n_views * s.H * s.W + elt * s.n_views * s.Hf * s.Wf * s.D
            + 4 * s.N * s.D + 4 * s.N)


# HBM bytes per aura_fuse_features call on workload c2 from the rocprofv3 counter runs summarised in
# profiles/whole_path_c2_hbm_traffic.md (FETCH_SIZE and WRITE_SIZE of k_tile_fused, each
# scaled by the reading of the 256 MiB calibration copy in the same run).  Valid only for the kernel source
# the counters were taken with: any change to that file makes the figure null until they are taken again.
TRAFFIC_C2_BYTES = 671120393
TRAFFIC_SOURCE_SHA256 = "63db4f76e914b9c5077bed0f61aa2c7c53b41fa1caaaf60b6282018b9fe2b1ee"


def measured_traffic():
    import hashlib
    src = os.path.join(ROOT, "paper_2511_03126_amd", "csrc", "fuse_tile.hip")
    try:
        digest = hashlib.sha256(open(src, "rb").read()).hexdigest()
    except OSError:
        return None
    return TRAFFIC_C2_BYTES if digest == TRAFFIC_SOURCE_SHA256 else None


def time_densify(torch, d, s, reps, n_sources=150, k=5):
    """The step after the hot path (Sec. 3.4.1 Eq. 5): every point of the scene as a query, its fused row as the
    feature, 150 evenly spaced points as sources with their scores.  HBM bound on reading the query features."""
    import paper_2511_03126_amd as aura
    from paper_2511_03126_amd import binding
    ns = min(n_sources, s.N)
    src = torch.linspace(0, s.N - 1, ns, device=d.dev).long()
    fs, ws = d.fused[src].contiguous(), d.scores[src].contiguous()
    wq, prop = torch.empty_like(d.scores), torch.empty_like(d.prop)
    label = torch.empty_like(d.label)
    work = torch.empty(aura.workspace_bytes(binding.CALL_KNN_DENSIFY, D=s.D, Ns=ns), dtype=torch.uint8, device=d.dev)
    run = lambda: aura.knn_densify(d.fused, fs, ws, k, d.y, d.params, wq, prop, label, None, work)
    for _ in range(2):
        run()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        run()
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / reps
    nbytes = 4 * s.N * s.D + 4 * ns * s.D + 4 * ns * s.K + 4 * s.N * s.K + 4 * s.N * s.P + 4 * s.N
    gbps = nbytes / (ms * 1e-3) / 1e9
    return {"call": "aura_knn_densify", "queries": s.N, "sources": ns, "k": k, "ms": ms, "bound": "hbm",
            "algorithmic_bytes": nbytes, "achieved": gbps, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
            "frac": gbps / HBM_PEAK_GBPS}


def time_thickness(torch, d, s, reps):
    """Sec. 3.4.2, thickness-based integration and centre of mass over the scene's scores (three small launches;
    reads the score rows, the positions and the view counts once)."""
    import paper_2511_03126_amd as aura
    from paper_2511_03126_amd import binding
    from workloads.scenes import material_thickness
    theta = torch.from_numpy(material_thickness(s.K, s.meta["seed"])).to(d.dev)
    total, com = torch.empty(s.B, device=d.dev), torch.empty((s.B, 3), device=d.dev)
    work = torch.empty(aura.workspace_bytes(binding.CALL_THICKNESS_INTEGRATE, N=s.N, B=s.B), dtype=torch.uint8, device=d.dev)
    run = lambda: aura.thickness_integrate(d.scores, d.y, theta, d.xyz, d.params, total, p_index=0, count=d.count_fuse,
                                           pt_offsets=None if d.single else s.pt_offsets, lam=0.6, scale_factor=1.0,
                                           com=com, workspace=work)
    for _ in range(2):
        run()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        run()
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / reps
    nbytes = 4 * s.N * s.K + 2 * 12 * s.N + 4 * s.N       # positions are read by the box pass and by the point pass
    gbps = nbytes / (ms * 1e-3) / 1e9
    return {"call": "aura_thickness_integrate", "ms": ms, "bound": "hbm", "algorithmic_bytes": nbytes, "achieved": gbps,
            "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": gbps / HBM_PEAK_GBPS, "mass": total.cpu().tolist(),
            "centre_of_mass": com.cpu().tolist()[0]}


def time_selection(torch, d, s, reps, k=3):
    """Sec. 3.2.2 / 3.2.3: the k = 3 most important views of every point, then the fusion over the kept views."""
    import paper_2511_03126_amd as aura
    from workloads.scenes import synthetic_normals
    nrm = torch.from_numpy(synthetic_normals(s.xyz, s.pt_offsets, s.meta["seed"])).to(d.dev)
    sel_view = torch.empty((s.N, k), dtype=torch.int32, device=d.dev)
    sel_score = torch.empty((s.N, k), device=d.dev)
    sel_mask = torch.empty((s.N, s.vis_pitch), dtype=torch.uint8, device=d.dev)
    fused = torch.empty_like(d.fused)
    count = torch.empty_like(d.count_fuse)
    select = lambda: aura.select_views(d.views, d.params, d.xyz, nrm, k, sel_view, sel_score, sel_mask, None, d.pt_offsets,
                                       d.view_offsets)
    fuse = lambda: aura.fuse_selected(d.views, d.params, d.xyz, sel_mask, fused, count, d.pt_offsets, d.view_offsets,
                                      d.ws_fuse)
    out = {"k": k}
    for name, fn in (("aura_select_views_ms", select), ("aura_fuse_selected_ms", fuse)):
        for _ in range(2):
            fn()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        out[name] = e0.elapsed_time(e1) / reps
    out["mean_views_kept"] = float(count.float().mean())
    return out


def time_downsample(torch, d, s, reps, n_target=150):
    """Sec. 3.2.1: adaptive voxel down-sampling of the scene's points to about 150 source points per object."""
    import numpy as np
    import paper_2511_03126_amd as aura
    po = s.pt_offsets
    lo = np.stack([s.xyz[po[b]:po[b + 1]].min(0) for b in range(s.B)]).astype(np.float32)
    hi = np.stack([s.xyz[po[b]:po[b + 1]].max(0) for b in range(s.B)]).astype(np.float32)
    cap = 64 * n_target * s.B
    out_xyz = torch.empty((cap, 3), device=d.dev)
    out_offsets = torch.empty(s.B + 1, dtype=torch.int32, device=d.dev)
    vop = torch.empty(s.N, dtype=torch.int32, device=d.dev)
    work = torch.empty(aura.voxel_workspace_bytes(lo, hi, n_target), dtype=torch.uint8, device=d.dev)
    run = lambda: aura.voxel_downsample(d.xyz, lo, hi, n_target, out_xyz, out_offsets, None, vop,
                                        pt_offsets=None if d.single else po, workspace=work)
    for _ in range(2):
        run()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        run()
    e1.record()
    torch.cuda.synchronize()
    return {"call": "aura_voxel_downsample", "n_target": n_target, "ms": e0.elapsed_time(e1) / reps,
            "sampled_points": int(out_offsets[-1].item())}


def time_patches(torch, d, s, reps, M=150, k=3, R=224, half=False):
    """Sec. 3.2.3: the encoder batch of M source points x k views x 3 scales (20, 40, 60 pixels) at R x R.  HBM bound on
    writing the batch."""
    import numpy as np
    import paper_2511_03126_amd as aura
    from workloads.scenes import synthetic_images, synthetic_normals
    images = torch.from_numpy(synthetic_images(s.n_views, s.H, s.W, s.meta["seed"])).to(d.dev)
    idx = np.linspace(0, int(s.pt_offsets[1]) - 1, M).astype(np.int64)
    xyz = d.xyz[torch.from_numpy(idx).to(d.dev)].contiguous()
    nrm = torch.from_numpy(synthetic_normals(s.xyz, s.pt_offsets, s.meta["seed"])[idx]).to(d.dev)
    v1 = int(s.view_offsets[1])
    views = aura.Views(cam=d.views.cam[:v1], depth=d.views.depth[:v1])
    sel = torch.empty((M, k), dtype=torch.int32, device=d.dev)
    aura.select_views(views, d.params, xyz, nrm, k, sel)
    out = torch.empty((M, k, 3, 3, R, R), dtype=torch.float16 if half else torch.float32, device=d.dev)
    run = lambda: aura.patch_batch(views.cam, images[:v1], xyz, sel, [20.0, 40.0, 60.0], out)
    for _ in range(2):
        run()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        run()
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / reps
    nbytes = out.numel() * out.element_size()
    gbps = nbytes / (ms * 1e-3) / 1e9
    return {"call": "aura_patch_batch", "patches": M * k * 3, "resolution": R, "out_dtype": "f16" if half else "f32",
            "ms": ms, "bound": "hbm", "algorithmic_bytes": nbytes, "achieved": gbps, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
            "frac": gbps / HBM_PEAK_GBPS}


def time_normals(torch, d, s, reps, n_target=150, k=30):
    """Sec. 3.2.2: normals of the ~150 sampled points of the first object from their 30 nearest points of its cloud."""
    import numpy as np
    import paper_2511_03126_amd as aura
    p1 = int(s.pt_offsets[1])
    lo, hi = s.xyz[:p1].min(0, keepdims=True), s.xyz[:p1].max(0, keepdims=True)
    cloud = d.xyz[:p1]
    q = torch.empty((64 * n_target, 3), device=d.dev)
    off = torch.empty(2, dtype=torch.int32, device=d.dev)
    work = torch.empty(aura.voxel_workspace_bytes(lo, hi, n_target), dtype=torch.uint8, device=d.dev)
    aura.voxel_downsample(cloud, lo, hi, n_target, q, off, workspace=work)
    q = q[: int(off[1].item())].contiguous()
    centre = s.xyz[:p1].mean(0, keepdims=True).astype(np.float32)
    normals = torch.empty_like(q)
    run = lambda: aura.estimate_normals(cloud, q, centre, k, normals)
    for _ in range(2):
        run()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        run()
    e1.record()
    torch.cuda.synchronize()
    return {"call": "aura_estimate_normals", "queries": int(q.shape[0]), "cloud": p1, "k": k, "ms": e0.elapsed_time(e1) / reps}


def cpu_baseline(scene, seconds_target=15.0):
    """The oracle, as it stands, on a contiguous sample of the scene's first object."""
    import numpy as np
    from oracle import aura_oracle as orc
    s = scene
    p1 = int(s.pt_offsets[1])
    v1 = int(s.view_offsets[1])
    cam, depth, feat = s.cam[:v1], s.depth[:v1], s.feat[:v1]

    stages = {"project_visibility": 0.0, "fuse_features": 0.0, "material_scores": 0.0, "property_integrate": 0.0}

    def run(n):
        xyz = s.xyz[:n]
        t = [time.perf_counter()]
        pv = orc.project_visibility(cam, depth, xyz, tau=s.tau, z_near=s.z_near)
        t.append(time.perf_counter())
        fu = orc.fuse_features(cam, depth, feat, s.feat_dtype, xyz, tau=s.tau, z_near=s.z_near)
        t.append(time.perf_counter())
        sc = orc.material_scores(fu["fused"], s.temb, s.y, T=s.temperature)
        t.append(time.perf_counter())
        orc.property_integrate(sc["prop"], 0, fu["count"], vol_uniform=s.vol_uniform, xyz=xyz,
                               grid_lo=None if s.G == 0 else s.grid_lo[:1], grid_h=None if s.G == 0 else s.grid_h[:1],
                               G=s.G)
        t.append(time.perf_counter())
        del pv
        for name, a, b in zip(stages, t[:-1], t[1:]):
            stages[name] += b - a
        return t[-1] - t[0]

    n = min(p1, 2000)
    t = run(n)                       # also warms the library up
    n = int(min(p1, max(n, n * seconds_target / max(t, 1e-3))))
    n = min(n, 400_000)
    for name in stages:
        stages[name] = 0.0           # the sizing run above does not count
    t = run(n)
    reps = 1
    while t < 0.7 * seconds_target and reps < 64:     # the whole object is quicker than the target: repeat it
        t += run(n)
        reps += 1
    return {"value": reps * n * v1 / t, "unit": "point-views/s", "cores": orc.max_threads(), "kind": "oracle",
            "sample": f"first {n} points of object 0 x {v1} views, whole path, {reps} passes, {t:.1f} s",
            "stage_seconds": {k: round(v, 3) for k, v in stages.items()}}


CAL_BYTES = 256 << 20   # size of the calibration copy (read) and of its destination (write)


def calibrate(torch, reps=10):
    """What the memory system gives the plainest kernels: the library's copy and fill over 256 MiB, timed
    outside the benchmark's timed region.  A profiler run of this file therefore always holds launches of a
    copy kernel of known size (CAL_BYTES read, CAL_BYTES written) to scale its byte counters by."""
    from paper_2511_03126_amd import binding
    src = torch.zeros(CAL_BYTES, dtype=torch.uint8, device="cuda")
    dst = torch.empty(CAL_BYTES, dtype=torch.uint8, device="cuda")
    out = {"bytes": CAL_BYTES}
    for name, fn, moved in (("copy", lambda: binding.calibration_copy(dst, src), 2 * CAL_BYTES),
                            ("fill", lambda: binding.calibration_fill(dst, 0), CAL_BYTES)):
        fn()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        out[name + "_GBps"] = moved / (e0.elapsed_time(e1) * 1e-3 / reps) / 1e9
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=100,
                    help="untimed steps before the timed ones; the GPU needs some tens of milliseconds of load to reach its clocks")
    ap.add_argument("--workload", default="c2", choices=["c1", "c2", "c3", "c4", "c5"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--staged", action="store_true", help="fusion and scoring as two library calls")
    ap.add_argument("--hot-path-only", action="store_true",
                    help="skip the calls beyond the hot path (densification, thickness integration, view selection)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this library runs on exactly one GPU (the path would shard by points, one GPU each); "
                 "use --gpus 1")

    import torch
    import gpu_harness as H
    from workloads.scenes import make_scene
    assert torch.cuda.is_available(), "bench.py needs a GPU"

    s = make_scene(args.workload)
    d = H.DeviceScene(s)
    if args.staged:
        names = ["project_visibility", "fuse_features", "material_scores", "property_integrate"]
        calls = [d.project_visibility, d.fuse_features, d.material_scores, d.property_integrate]
    else:
        names = ["fuse_scores", "property_integrate"]       # the mask and view counts come out of the fusion
        calls = [d.fuse_scores_vis, d.property_integrate]
    # Python's cyclic garbage collector is off during the warm-up and the timed steps: a full collection (it comes
    # after a few hundred steps' worth of allocations and walks every object torch has created) stops the host for
    # about 40 ms, the launch queue runs dry and the figure would be the host's, not the GPU's.
    gc.collect()
    gc.disable()
    for _ in range(max(args.warmup, 0)):
        for call in calls:
            call()
    torch.cuda.synchronize()

    # The timed region: exactly args.steps steps between two synchronisations, nothing else on the stream.
    t0 = time.perf_counter()
    for _ in range(args.steps):
        for call in calls:
            call()
    t_enqueued = time.perf_counter()
    torch.cuda.synchronize()
    t1 = time.perf_counter()

    ms_per_step = (t1 - t0) * 1e3 / args.steps
    # host time to enqueue one step; once the launch queue is full it is the GPU's pace, not the host's cost
    enqueue_ms_per_step = (t_enqueued - t0) * 1e3 / args.steps

    # Time per call, from a short run of its own with an event after every call.
    n_split = min(args.steps, 20)
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(len(calls) + 1)] for _ in range(n_split)]
    for k in range(n_split):
        ev[k][0].record()
        for c, call in enumerate(calls):
            call()
            ev[k][c + 1].record()
    torch.cuda.synchronize()
    call_ms = {n: sum(ev[k][c].elapsed_time(ev[k][c + 1]) for k in range(n_split)) / n_split
               for c, n in enumerate(names)}
    pv = s.point_views
    tile = d.ws_fuse is not None
    gpu = d.results()

    # Roofline of the dominant work: the fusion proper (the matrix-core kernels, or k_fuse_gather), which writes
    # the fused rows.  Inside aura_fuse_scores it cannot be bracketed by events, so it is timed through
    # aura_fuse_features (same inputs, same workspace) right after the timed steps, with events on the launch
    # stream.  Inside aura_fuse_scores the same kernels also serve the scoring (a scoring wave per workgroup, or the
    # k-steps left in memory for the scoring kernel; see calls_ms for the whole call).
    fuse_reps = max(args.steps, 10)
    fuse_warmup = max(3, min(args.warmup, 50))
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    for _ in range(fuse_warmup):
        d.fuse_features()
    e0.record()
    for _ in range(fuse_reps):
        d.fuse_features()
    e1.record()
    torch.cuda.synchronize()
    fuse_ms = e0.elapsed_time(e1) / fuse_reps
    # the same call one at a time (its own pair of events): spread of the launches, and a second figure with the
    # caches flushed by a 512 MiB fill before every call (maps, depth and workspace then come from HBM)
    def one_by_one(flush):
        big = torch.empty(512 << 20, dtype=torch.uint8, device="cuda") if flush else None
        pairs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(fuse_reps)]
        from paper_2511_03126_amd import binding
        for a, b in pairs:
            if flush:
                binding.calibration_fill(big, 1)
            a.record()
            d.fuse_features()
            b.record()
        torch.cuda.synchronize()
        t = sorted(a.elapsed_time(b) for a, b in pairs)
        return {"min_ms": t[0], "median_ms": t[len(t) // 2], "max_ms": t[-1]}
    warm_each, cold_each = one_by_one(False), one_by_one(True)
    calibration = calibrate(torch)   # after the measurements above: its 256 MiB sweeps leave the caches full of its data
    fuse_bytes = fuse_algorithmic_bytes(s)
    achieved = fuse_bytes / (fuse_ms * 1e-3) / 1e9
    kernel = "aura_fuse_features: " + (f"matrix-core fusion <{s.feat_dtype}, {s.D // 256} product waves> (k_tile_fused where the "
                                       "one-kernel form applies, else k_tile_prepare + k_tile_product)" if tile
                                       else "k_fuse_gather")
    traffic = measured_traffic() if (tile and args.workload == "c2") else None
    extras = {}
    if not args.hot_path_only:
        extras = {"densify": time_densify(torch, d, s, max(args.steps // 2, 5)),
                  "thickness_integrate": time_thickness(torch, d, s, max(args.steps // 2, 5)),
                  "view_selection": time_selection(torch, d, s, max(args.steps // 2, 5)),
                  "voxel_downsample": time_downsample(torch, d, s, max(args.steps // 2, 5)),
                  "estimate_normals": time_normals(torch, d, s, max(args.steps // 2, 5)),
                  "patch_batch": time_patches(torch, d, s, max(args.steps // 2, 5)),
                  "patch_batch_f16": time_patches(torch, d, s, max(args.steps // 2, 5), half=True)}
    gc.enable()
    out = {
        "metric": "fused point-views/sec", "value": pv / (ms_per_step * 1e-3), "unit": "point-views/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{args.workload}: N={s.N} points, B={s.B} objects, {s.n_views} views {s.H}x{s.W}, "
                               f"feature grid {s.Hf}x{s.Wf}x{s.D} {s.feat_dtype}, K={s.K} materials, P={s.P}, "
                               f"mass grid G={s.G}", "point_views": pv,
                   "visible_point_views_per_s": float(gpu["vis"].mean()) * pv / (ms_per_step * 1e-3),
                   "visible_fraction": float(gpu["vis"].mean()), "unseen_points": float((gpu["count_fuse"] == 0).mean()),
                   "order": s.meta["order"], "seed": s.meta["seed"]},
        "calls_ms": call_ms, "host_enqueue_ms_per_step": enqueue_ms_per_step,
        "roofline": {"bound": "hbm", "kernel": kernel, "achieved": achieved,
                     "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBPS, "traffic": traffic,
                     "algorithmic_bytes": fuse_bytes, "avg_launch_ms": fuse_ms, "launches": fuse_reps, "warmup_launches": fuse_warmup,
                     "single_launches": warm_each, "single_launches_caches_flushed": cold_each,
                     "frac_caches_flushed": fuse_bytes / (cold_each["median_ms"] * 1e-3) / 1e9 / HBM_PEAK_GBPS,
                     "frac_of_fill_kernel": achieved / calibration["fill_GBps"]},
        **extras,
        "calibration": calibration,
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(s)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
