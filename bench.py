#!/usr/bin/env python3
"""Benchmark of the fusion hot path on one MI355X.

One step = one pass of the whole path over one synthetic scene already resident in HBM:
aura_fuse_scores (visibility mask and view counts, fusion, scoring) -> aura_property_integrate
(--staged: aura_project_visibility, aura_fuse_features, aura_material_scores, aura_property_integrate).
Prints ONE JSON line.  Headline: whole-path throughput in fused point-views per second on the largest configuration
(c5: 64 objects, 6.4 M points, 13.3 GB per fusion launch), with the roofline figure of the dominant kernel - the fusion
kernel inside aura_fuse_scores, HBM bound on writing the fused rows - timed with events that the library records around
that kernel in a second pass over the same steps.  `configs` holds the same measurement for c1-c4, `single_pass` the
whole path as one call that never writes the fused rows (aura_fuse_score_integrate), `stress` the frustum-only and
unsorted-points cases, `beyond_hot_path` the calls around the hot path on c2, and `cpu_baseline` the CPU oracle timed on
a bounded sample of the headline workload.
"""
import argparse
import gc
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0   # MI355X HBM3E


def fuse_algorithmic_bytes(s):
    """Each input read once, the fused rows and counts written once."""
    elt = 4 if s.feat_dtype == "f32" else 2
    return (12 * s.N + 64 * s.n_views + 4 * s.n_views * s.H * s.W + elt * s.n_views * s.Hf * s.Wf * s.D
            + 4 * s.N * s.D + 4 * s.N)


# HBM bytes per launch of the dominant kernel from the rocprofv3 counter runs summarised under profiles/ (FETCH_SIZE and
# WRITE_SIZE, each scaled by the reading of the 256 MiB calibration copy in the same run), per workload.  Valid only for
# the kernel source the counters were taken with: any change to that file makes the figure null until they are taken again.
TRAFFIC_BYTES = {'c5': 13697295716}
TRAFFIC_SOURCE_SHA256 = "2f4d7b709ce57a2d0d6fbca40083399d1a869fcd639011d54007a03e0707784c"


def measured_traffic(workload):
    import hashlib
    src = os.path.join(ROOT, "paper_2511_03126_amd", "csrc", "fuse_tile.hip")
    try:
        digest = hashlib.sha256(open(src, "rb").read()).hexdigest()
    except OSError:
        return None
    return TRAFFIC_BYTES.get(workload) if digest == TRAFFIC_SOURCE_SHA256 else None


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
    clock_ramp(torch, [run], 50.0)   # the GPU has idled while the inputs were put together
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
    clock_ramp(torch, [run], 50.0)
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
    out = {"call": "aura_estimate_normals", "queries": int(q.shape[0]), "cloud": p1, "k": k, "ms": e0.elapsed_time(e1) / reps}
    # the same queries against a cloud of 1.7 M points (the voxel centres of workload c4 are that many): the object's
    # points tiled and shifted by multiples of its extent
    reps_cloud = 8
    big = torch.cat([cloud + float(j) * 10.0 for j in range(reps_cloud)]) if p1 * reps_cloud <= 2_000_000 else cloud
    big[:p1] = cloud
    run_big = lambda: aura.estimate_normals(big, q, centre, k, normals)
    for _ in range(2):
        run_big()
    e0.record()
    for _ in range(reps):
        run_big()
    e1.record()
    torch.cuda.synchronize()
    out["large_cloud"] = {"cloud": int(big.shape[0]), "ms": e0.elapsed_time(e1) / reps}
    return out


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
    while t < 0.7 * seconds_target and reps < 1024:   # the whole object is quicker than the target: repeat it
        t += run(n)
        reps += 1
    return {"value": reps * n * v1 / t, "unit": "point-views/s", "cores": orc.max_threads(), "kind": "oracle",
            "sample": f"first {n} points of object 0 x {v1} views, whole path, {reps} passes, {t:.1f} s",
            "stage_seconds": {k: round(v, 3) for k, v in stages.items()}}


def cpu_single_thread(scene, n=20000):
    """The oracle on one host thread: the first n points of the smallest workload through the whole path."""
    from oracle import aura_oracle as orc
    s = scene
    threads = orc.max_threads()
    orc.set_threads(1)
    try:
        xyz = s.xyz[:n]
        t0 = time.perf_counter()
        fu = orc.fuse_features(s.cam, s.depth, s.feat, s.feat_dtype, xyz, tau=s.tau, z_near=s.z_near)
        sc = orc.material_scores(fu["fused"], s.temb, s.y, T=s.temperature)
        orc.property_integrate(sc["prop"], 0, fu["count"], vol_uniform=s.vol_uniform, xyz=xyz,
                               grid_lo=None if s.G == 0 else s.grid_lo[:1], grid_h=None if s.G == 0 else s.grid_h[:1], G=s.G)
        t = time.perf_counter() - t0
    finally:
        orc.set_threads(threads)
    return {"value": len(xyz) * s.n_views / t, "unit": "point-views/s", "cores": 1,
            "sample": f"first {len(xyz)} points of c1 x {s.n_views} views, fusion + scores + integration, {t:.2f} s"}


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


MFMA_PEAK_TFLOPS = 2500.0   # MI355X dense bf16 / fp16 matrix cores
CLOCK_RAMP_MS = 300.0       # load put on the GPU before the counted warm-up, so that the clocks are up whatever --warmup is
KERNEL_WARMUP = 3           # steps before the per-kernel event pass (its own, not tied to --warmup)


def single_pass_algorithmic_bytes(s):
    """aura_fuse_score_integrate: every input once; scores, properties, labels, view counts and the mask once."""
    elt = 4 if s.feat_dtype == "f32" else 2
    return (12 * s.N + 64 * s.n_views + 4 * s.n_views * s.H * s.W + elt * s.n_views * s.Hf * s.Wf * s.D
            + 4 * s.K * s.D + 4 * s.N * s.K + 4 * s.N * s.P + 4 * s.N + 4 * s.N + s.N * s.vis_pitch)


def timed_steps(torch, calls, steps):
    """Exactly `steps` steps between two synchronisations; returns (ms per step, host enqueue ms per step)."""
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        for call in calls:
            call()
    t_enqueued = time.perf_counter()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    return (t1 - t0) * 1e3 / steps, (t_enqueued - t0) * 1e3 / steps


def clock_ramp(torch, calls, ramp_ms):
    """The same calls as the timed steps for at least ramp_ms of wall time (the GPU reaches its clocks only after some tens
    of milliseconds of load); the host waits every few steps so that the queue does not run far ahead."""
    t0 = time.perf_counter()
    while (time.perf_counter() - t0) * 1e3 < ramp_ms:
        for _ in range(4):
            for call in calls:
                call()
        torch.cuda.synchronize()
    return (time.perf_counter() - t0) * 1e3


def fusion_kernel_ms(torch, calls, steps):
    """Average duration of the fusion kernel inside the step's calls: the library records a pair of events around that
    kernel (aura_time_next_fusion) on the launch stream, one pair per step, over `steps` further steps queued back to back."""
    import paper_2511_03126_amd as aura
    pairs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
    for a, b in pairs:      # a first record creates the handles the library records on
        a.record()
        b.record()
    for _ in range(KERNEL_WARMUP):
        for call in calls:
            call()
    torch.cuda.synchronize()
    for a, b in pairs:
        aura.time_next_fusion(a, b)
        for call in calls:
            call()
    aura.time_next_fusion(None, None)
    torch.cuda.synchronize()
    t = sorted(a.elapsed_time(b) for a, b in pairs)
    return sum(t) / len(t), {"min_ms": t[0], "median_ms": t[len(t) // 2], "max_ms": t[-1]}


def marker_overhead_ms(torch, n=20):
    """What a pair of stream markers adds to the interval they bracket: the same two event records around a 16-byte fill
    (a kernel of a few microseconds), queued back to back like the pairs of fusion_kernel_ms."""
    from paper_2511_03126_amd import binding
    tiny = torch.zeros(16, dtype=torch.uint8, device="cuda")
    pairs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n)]
    binding.calibration_fill(tiny, 0)
    for a, b in pairs:
        a.record()
        binding.calibration_fill(tiny, 0)
        b.record()
    torch.cuda.synchronize()
    t = sorted(a.elapsed_time(b) for a, b in pairs)
    return t[len(t) // 2]


def back_to_back_ms(torch, call, n):
    """n launches of one call between one pair of events: no marker between the launches."""
    for _ in range(KERNEL_WARMUP):
        call()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(n):
        call()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / n


def cold_call_ms(torch, call, n=5, flush_bytes=512 << 20):
    """One call at a time behind a 512 MiB fill that pushes the call's inputs out of the last-level cache; the events
    bracket the call only.  Median of n."""
    from paper_2511_03126_amd import binding
    junk = torch.empty(flush_bytes, dtype=torch.uint8, device="cuda")
    pairs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n)]
    for a, b in pairs:
        binding.calibration_fill(junk, 0)
        a.record()
        call()
        b.record()
    torch.cuda.synchronize()
    del junk
    t = sorted(a.elapsed_time(b) for a, b in pairs)
    return t[len(t) // 2]


def tile_steps(torch, d, s):
    """k-steps (16 feature cells each) per 32-point tile of the matrix-core fusion, read from the tile headers that the
    two-kernel form leaves in the workspace; None where the gather kernel runs."""
    if d.ws_fuse is None:
        return None
    import numpy as np
    d.fuse_features(two_kernels=True)
    torch.cuda.synchronize()
    ntile = int(np.sum((np.diff(s.pt_offsets) + 31) // 32))
    n = d.ws_fuse[:ntile * 144].cpu().numpy().view(np.int32).reshape(ntile, 36)[:, 0]
    return {"tiles": ntile, "mean": float(n[n >= 0].mean()) if (n >= 0).any() else 0.0, "max": int(n.max()),
            "fused_by_gather": int((n < 0).sum()), "total": int(n[n >= 0].sum())}


def measure(torch, s, name, steps, warmup, step="combined", flags=0, want_single_pass=True, extras=True):
    """One workload: the timed steps, the time per call, the fusion kernel's roofline figure, and the single-pass call.
    step: which calls make a step (combined: aura_fuse_scores + aura_property_integrate; staged: one call per stage;
    single_pass: aura_fuse_score_integrate).  extras=False leaves out everything that launches the fusion kernels in
    another way (for profiler runs, where launches are told apart by kernel name only)."""
    from paper_2511_03126_amd.device_scene import DeviceScene
    d = DeviceScene(s, flags=flags)
    staged = step == "staged"
    if staged:
        names = ["project_visibility", "fuse_features", "material_scores", "property_integrate"]
        calls = [d.project_visibility, d.fuse_features, d.material_scores, d.property_integrate]
    elif step == "single_pass":
        names = ["fuse_score_integrate"]
        calls = [d.step_single_pass_call]
        want_single_pass = False
    else:
        names = ["fuse_scores", "property_integrate"]       # the mask and view counts come out of the fusion
        calls = [d.fuse_scores_vis, d.property_integrate]
    ramp_ms = clock_ramp(torch, calls, CLOCK_RAMP_MS)
    for _ in range(max(warmup, 0)):
        for call in calls:
            call()
    ms_per_step, enqueue_ms = timed_steps(torch, calls, steps)

    # time per call, from a short run of its own with an event after every call
    n_split = min(steps, 20)
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(len(calls) + 1)] for _ in range(n_split)]
    for k in range(n_split):
        ev[k][0].record()
        for c, call in enumerate(calls):
            call()
            ev[k][c + 1].record()
    torch.cuda.synchronize()
    call_ms = {n: sum(ev[k][c].elapsed_time(ev[k][c + 1]) for k in range(n_split)) / n_split for c, n in enumerate(names)}

    pv = s.point_views
    tile = d.ws_fuse is not None
    vis_frac = float(d.vis.float().mean())
    unseen = float((d.count_fuse == 0).float().mean())
    kernel_ms, spread = fusion_kernel_ms(torch, calls, max(steps, 10))
    fuse_bytes = single_pass_algorithmic_bytes(s) if step == "single_pass" else fuse_algorithmic_bytes(s)
    achieved = fuse_bytes / (kernel_ms * 1e-3) / 1e9
    fusion_call = names[1] if staged else names[0]
    kernel = (f"matrix-core fusion <{s.feat_dtype}, {s.D // 256} product waves> inside {fusion_call} "
              "(k_tile_fused; k_tile_prepare + k_tile_product where the lists do not fit the one-kernel form)"
              if tile else f"k_fuse_gather inside {names[1] if staged else names[0]}")
    out = {
        "workload": f"{name}: N={s.N} points, B={s.B} objects, {s.n_views} views {s.H}x{s.W}, "
                    f"feature grid {s.Hf}x{s.Wf}x{s.D} {s.feat_dtype}, K={s.K} materials, P={s.P}, mass grid G={s.G}",
        "point_views": pv, "ms_per_step": ms_per_step, "point_views_per_s": pv / (ms_per_step * 1e-3),
        "visible_fraction": vis_frac, "visible_point_views_per_s": vis_frac * pv / (ms_per_step * 1e-3),
        "unseen_points": unseen, "order": s.meta["order"], "seed": s.meta["seed"], "flags": flags,
        "clock_ramp_ms": ramp_ms, "calls_ms": call_ms, "host_enqueue_ms_per_step": enqueue_ms,
        "roofline": {"bound": "hbm", "kernel": kernel, "achieved": achieved, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBPS, "traffic": measured_traffic(name) if (tile and not flags) else None,
                     "algorithmic_bytes": fuse_bytes, "avg_launch_ms": kernel_ms, "launches": max(steps, 10),
                     "launch_spread": spread,
                     # context for short kernels: the interval between the two markers holds the kernel plus the markers'
                     # own cost; the same fusion launched by aura_fuse_features, many calls between one pair of events
                     "marker_pair_overhead_ms": marker_overhead_ms(torch)},
    }
    if not extras:
        return out, d
    out["roofline"]["fuse_features_back_to_back_ms"] = back_to_back_ms(torch, d.fuse_features, max(steps, 10))
    out["roofline"]["fuse_features_cold_ms"] = cold_call_ms(torch, d.fuse_features)   # the markers' cost is in this one
    ks = None if (flags & 4) else tile_steps(torch, d, s)     # (AURA_FUSE_GATHER: no tiles)
    if ks is not None:
        out["tile_k_steps"] = {k: ks[k] for k in ("tiles", "mean", "max", "fused_by_gather")}
    if want_single_pass:
        one = [d.step_single_pass_call]
        clock_ramp(torch, one, 50.0)
        sp_ms, _ = timed_steps(torch, one, steps)
        sp_kernel_ms, sp_spread = fusion_kernel_ms(torch, one, max(steps, 10))
        sp_bytes = single_pass_algorithmic_bytes(s)
        sp = {"call": "aura_fuse_score_integrate", "ms_per_step": sp_ms, "point_views_per_s": pv / (sp_ms * 1e-3),
              "fusion_kernel_ms": sp_kernel_ms, "launch_spread": sp_spread, "algorithmic_bytes": sp_bytes,
              "algorithmic_GBps": sp_bytes / (sp_ms * 1e-3) / 1e9,
              "hbm_frac": sp_bytes / (sp_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS}
        if ks is not None and ks["fused_by_gather"] == 0:
            # Matrix-core work of the fusion kernel: per k-step the 32 x 16 weights (two 16-bit terms) times 16 x D cells;
            # where it scores its tiles itself, three partial products of 32 x 16 by 16 x 32 more.  Not what bounds the
            # kernel (its producer waves are: dependent chains of projection, depth read, cell lists), reported for scale.
            flops = ks["total"] * (2 * 2 * 32 * 16 * s.D)
            sp["roofline"] = {"bound": "mfma", "kernel": "fusion kernel of aura_fuse_score_integrate (no row stores)",
                              "achieved": flops / (sp_kernel_ms * 1e-3) / 1e12, "peak": MFMA_PEAK_TFLOPS, "unit": "TFLOP/s",
                              "frac": flops / (sp_kernel_ms * 1e-3) / 1e12 / MFMA_PEAK_TFLOPS, "traffic": None,
                              "algorithmic_flops": flops}
        out["single_pass"] = sp
    return out, d


def _make(job):
    """Scene generation in a worker process (numpy only; started before this process touches the GPU)."""
    from workloads.scenes import make_scene
    name, order = job[0], job[1]
    return make_scene(name, order=order, overrides=dict(dtype=job[2]) if len(job) > 2 else None)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5,
                    help="untimed steps before the timed ones (after a time-based clock ramp of the same calls)")
    ap.add_argument("--workload", default="c5", choices=["c1", "c2", "c3", "c4", "c5"],
                    help="the headline workload; the others are reported under `configs`")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--staged", action="store_true", help="one library call per stage (same as --step staged)")
    ap.add_argument("--step", default="combined", choices=["combined", "staged", "single_pass"],
                    help="the calls of a step: aura_fuse_scores + aura_property_integrate; one call per stage; or "
                         "aura_fuse_score_integrate alone")
    ap.add_argument("--plain", action="store_true",
                    help="with --only-headline: nothing but the step's own calls (for profiler runs)")
    ap.add_argument("--only-headline", action="store_true",
                    help="skip the other configurations, the stress cases and the calls beyond the hot path")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this library runs on exactly one GPU (the path would shard by points, one GPU each); "
                 "use --gpus 1")

    # every scene is generated up front, in worker processes forked before anything touches the GPU
    from concurrent.futures import ProcessPoolExecutor
    import multiprocessing
    others = [] if args.only_headline else [w for w in ("c1", "c2", "c3", "c4") if w != args.workload]
    jobs = [(args.workload, "morton")] + [(w, "morton") for w in others]
    if not args.only_headline:
        jobs += [("c2", "random"), ("c5", "random"), ("c2", "morton", "f32")]
    try:
        with ProcessPoolExecutor(max_workers=min(len(jobs), 8), mp_context=multiprocessing.get_context("fork")) as pool:
            scenes = dict(zip(jobs, pool.map(_make, jobs)))
    except (OSError, RuntimeError, ImportError):      # no worker processes to be had: one scene after the other
        scenes = {job: _make(job) for job in jobs}

    import torch
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    # Python's cyclic garbage collector is off during the measurements: a full collection (it comes after a few hundred
    # steps' worth of allocations and walks every object torch has created) stops the host for about 40 ms, the launch
    # queue runs dry and the figure would be the host's, not the GPU's.
    gc.collect()
    gc.disable()

    def release(d):
        del d
        gc.collect()
        torch.cuda.empty_cache()

    s = scenes[(args.workload, "morton")]
    step = "staged" if args.staged else args.step
    head, d = measure(torch, s, args.workload, args.steps, args.warmup, step=step, extras=not args.plain)
    release(d)
    out = {
        "metric": "fused point-views/sec", "value": head["point_views_per_s"], "unit": "point-views/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": head["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": s.feat_dtype, "data": "synthetic",
        "clock_ramp_ms": head["clock_ramp_ms"],
        "config": {"workload": head["workload"], "point_views": head["point_views"],
                   "visible_point_views_per_s": head["visible_point_views_per_s"],
                   "visible_fraction": head["visible_fraction"], "unseen_points": head["unseen_points"],
                   "order": head["order"], "seed": head["seed"]},
        "calls_ms": head["calls_ms"], "host_enqueue_ms_per_step": head["host_enqueue_ms_per_step"],
        "roofline": head["roofline"], "single_pass": head.get("single_pass"),
    }
    if "tile_k_steps" in head:
        out["tile_k_steps"] = head["tile_k_steps"]
    if not args.only_headline:
        configs = []
        for w in others:
            r, d = measure(torch, scenes[(w, "morton")], w, args.steps, args.warmup, step=step)
            if w == "c2":
                reps = max(args.steps // 2, 5)
                d.step_combined()      # the calls beyond the hot path take the fused rows and scores as input
                out["beyond_hot_path"] = {"workload": "c2",
                                          "densify": time_densify(torch, d, d.scene, reps),
                                          "thickness_integrate": time_thickness(torch, d, d.scene, reps),
                                          "view_selection": time_selection(torch, d, d.scene, reps),
                                          "voxel_downsample": time_downsample(torch, d, d.scene, reps),
                                          "estimate_normals": time_normals(torch, d, d.scene, reps),
                                          "patch_batch": time_patches(torch, d, d.scene, reps),
                                          "patch_batch_f16": time_patches(torch, d, d.scene, reps, half=True)}
            release(d)
            configs.append(r)
        out["configs"] = configs
        # Stress cases.  c4 with the depth test off: 94 % of its voxels are inside the solid and seen by no view, so only
        # without the test do all its pairs gather.  Points in generation order instead of Morton order: the tiles' cell
        # lists outgrow their storage and the in-kernel gather takes over; AURA_FUSE_GATHER is the kernel meant for that.
        from paper_2511_03126_amd import binding
        stress = {}
        r, d = measure(torch, scenes[("c4", "morton")] if args.workload != "c4" else s, "c4", args.steps, args.warmup,
                       flags=binding.VIS_FRUSTUM_ONLY)
        release(d)
        stress["c4_frustum_only"] = r
        for w in ("c2", "c5"):
            for label, flags in (("matrix_core_path", 0), ("gather_kernel", binding.FUSE_GATHER)):
                r, d = measure(torch, scenes[(w, "random")], w, max(args.steps // 2, 5), 2, flags=flags,
                               want_single_pass=False)
                release(d)
                stress[f"{w}_unsorted_{label}"] = {k: r[k] for k in ("workload", "order", "ms_per_step", "point_views_per_s",
                                                                     "calls_ms", "roofline", "tile_k_steps") if k in r}
        # fp32 feature maps (or a channel count that is not a multiple of 256) take the per-point gather kernel: the
        # matrix-core path needs 16-bit maps
        r, d = measure(torch, scenes[("c2", "morton", "f32")], "c2 with fp32 maps", max(args.steps // 2, 5), 2, want_single_pass=False)
        release(d)
        stress["c2_fp32_maps_gather_kernel"] = {k: r[k] for k in ("workload", "ms_per_step", "point_views_per_s", "calls_ms",
                                                                   "roofline") if k in r}
        out["stress"] = stress
    out["calibration"] = calibrate(torch)
    for r in [out] + out.get("configs", []):   # the same figure against what the plainest kernels reach on this machine
        r["roofline"]["frac_of_copy_kernel"] = r["roofline"]["achieved"] / out["calibration"]["copy_GBps"]
        r["roofline"]["frac_of_fill_kernel"] = r["roofline"]["achieved"] / out["calibration"]["fill_GBps"]
    gc.enable()
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(s)
        if ("c1", "morton") in scenes:
            out["cpu_baseline"]["single_thread_c1"] = cpu_single_thread(scenes[("c1", "morton")])
    print(json.dumps(out))


if __name__ == "__main__":
    main()
