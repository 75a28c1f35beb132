#!/usr/bin/env python3
"""Benchmark of the Flattened Window Attention block on one MI355X.

One "step" = one pass of the whole hot path over one synthetic frame: the sorts of the block
(window keys, radix argsort, grouping; each distinct (axis, shift) pair once) followed by the
layer stack (gather, LayerNorm, QKV, softmax attention, out-proj, FFN, scatter per layer).
Inputs are resident in HBM before the timed region.  Prints ONE JSON line: the headline (mean over the K
timed steps), median / min over a second loop of K steps, the same block replayed from a HIP graph, the
roofline of the layer kernel, per-part timings, what the box reaches on a plain copy and on an MFMA issue
loop (`peaks_measured`), the same kernels on a batch of 128 frames (`saturation`), the oracle on the host.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 2] [--tail mask|drop] [--pos-embed] [--f16]
                    [--no-cpu] [--no-peaks] [--no-saturation] [--sweep]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_HBM_GBS = 8000.0          # MI355X HBM3E
PEAK_BF16_TFLOPS = 2500.0      # dense bf16 MFMA
PEAK_F32_TFLOPS = 157.3        # fp32 vector / MFMA

def measured_layer_traffic(config_id):
    """HBM bytes per launch of the fused layer kernel, read from the committed rocprofv3 summary of this
    workload (profiles/fwa_layer_cfg<N>_hbm_counters.txt, line 'TRAFFIC_BYTES_PER_LAUNCH <bytes>': FETCH_SIZE and
    WRITE_SIZE per dispatch, each scaled by what the same counter reads for a plain copy of known size).  None when
    no summary of that configuration is committed."""
    path = os.path.join(ROOT, "profiles", f"fwa_layer_cfg{config_id}_hbm_counters.txt")
    try:
        for line in open(path):
            if line.startswith("TRAFFIC_BYTES_PER_LAUNCH"):
                return int(line.split()[1])
    except OSError:
        pass
    return None


def layer_flops_per_voxel(C, F, G):
    # QKV 6C^2 + QK^T 2GC + PV 2GC + out-proj 2C^2 + FFN 4CF (multiply-add = 2 flops)
    return 8 * C * C + 4 * G * C + 4 * C * F


def time_region(fn, steps, warmup, stats=False):
    """Mean device time per call (ms) of `steps` calls bracketed by one event pair on the launch stream, and the
    host wall time per call.  With stats: also a dict with the median and minimum over per-call event pairs of a
    second loop of the same length (the latency protocol: warm-up runs, then median and min of the timed ones)."""
    import torch
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    for _ in range(steps):
        fn()
    e1.record()
    torch.cuda.synchronize()
    wall = (time.perf_counter() - t0) * 1e3
    mean = e0.elapsed_time(e1) / steps
    if not stats:
        return mean, wall / steps
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
    ev[0].record()
    for k in range(steps):
        fn()
        ev[k + 1].record()
    torch.cuda.synchronize()
    per = sorted(ev[k].elapsed_time(ev[k + 1]) for k in range(steps))
    return mean, wall / steps, {"mean": mean, "median": per[len(per) // 2], "min": per[0], "runs": steps}


def graph_replay_ms(fn, steps):
    """fn captured once into a HIP graph (it must have run eagerly before), replayed `steps` times back to back:
    device time per replay.  What the kernels cost without the host's issue time between them."""
    import torch
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            fn()
    torch.cuda.current_stream().wait_stream(side)
    for _ in range(3):
        graph.replay()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(steps):
        graph.replay()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / steps


def peaks_measured(torch, dev):
    """What this machine reaches on the two rooflines: a plain streaming copy of 1 GiB (bytes read + written per
    second) and a loop of independent bf16 matrix-core products on every SIMD (csrc/bench/peaks.hip)."""
    import ctypes as C
    lib = C.CDLL(os.path.join(ROOT, "paper_2301_08739_amd", "libffpeaks.so"))
    lib.ffpeak_stream_copy.restype, lib.ffpeak_stream_copy.argtypes = C.c_int, [C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
    lib.ffpeak_mfma_bf16.restype = C.c_int
    lib.ffpeak_mfma_bf16.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_void_p, C.POINTER(C.c_double), C.c_void_p]
    stream = C.c_void_p(torch.cuda.current_stream().cuda_stream)
    nbytes = 1 << 30
    src = torch.empty(nbytes, dtype=torch.uint8, device=dev)
    dst = torch.empty_like(src)
    src.zero_()

    def copy():
        assert lib.ffpeak_stream_copy(C.c_void_p(dst.data_ptr()), C.c_void_p(src.data_ptr()), nbytes, stream) == 0

    ms_copy, _ = time_region(copy, 10, 3)
    del src, dst
    iters = 2000
    res = {"stream_copy_GBps": 2 * nbytes / (ms_copy * 1e-3) / 1e9, "stream_copy_bytes": nbytes,
           "nominal": {"hbm_GBps": PEAK_HBM_GBS, "mfma_bf16_TFLOPs": PEAK_BF16_TFLOPS},
           "note": "copy: 1 GiB read + 1 GiB written per launch; MFMA loops: every wavefront issues 16000 independent "
                   "products; clock_MHz = shader cycles per 100 MHz tick of one wavefront's loop"}
    # all SIMDs busy (8 and 4 wavefronts each), both product shapes; and one workgroup alone, where the chip is
    # not power limited
    for name, blocks, shape in (("mfma_bf16_16x16x32", 256 * 8, 0), ("mfma_bf16_32x32x16", 256 * 4, 1),
                                ("mfma_bf16_16x16x32_one_workgroup", 1, 0)):
        sink = torch.empty(blocks * 256, dtype=torch.float32, device=dev)
        ticks = torch.zeros(2, dtype=torch.int64, device=dev)
        flops = C.c_double(0.0)

        def mfma():
            assert lib.ffpeak_mfma_bf16(C.c_void_p(sink.data_ptr()), blocks, iters, shape, C.c_void_p(ticks.data_ptr()),
                                        C.byref(flops), stream) == 0

        ms_mfma, _ = time_region(mfma, 5, 2)
        cyc, tk = (int(v) for v in ticks.cpu())
        res[name] = {"TFLOPs": flops.value / (ms_mfma * 1e-3) / 1e12, "workgroups": blocks,
                     "clock_MHz": 100.0 * cyc / max(tk, 1), "cycles_per_product_per_wavefront": cyc / (iters * 8.0)}
    res["mfma_bf16_TFLOPs"] = max(res["mfma_bf16_16x16x32"]["TFLOPs"], res["mfma_bf16_32x32x16"]["TFLOPs"])
    return res


def cpu_baseline(c, budget_s=20.0):
    """The oracle as it stands, timed on this host: whole frames of the same workload."""
    import numpy as np
    import oracle
    try:
        from threadpoolctl import threadpool_info
        cores = max([int(t.get("num_threads", 1)) for t in threadpool_info()] + [1])
    except Exception:
        cores = 1
    og = oracle.Geometry(c["B"], c["grid"], c["grid"], c["window"], c["window"])

    def one_frame():
        perms, offs = {}, {}
        for key in dict.fromkeys(c["schedule"]):
            perms[key], offs[key], _ = oracle.flatten(c["coords"], og, key[0], key[1], c["G"])
        oracle.stack(c["feats"], perms, offs, c["layer_params"], c["schedule"])

    t0 = time.perf_counter()
    one_frame()
    first = time.perf_counter() - t0
    reps = int(max(1, min(10, (budget_s - first) // max(first, 1e-3))))
    t0 = time.perf_counter()
    for _ in range(reps):
        one_frame()
    dt = (time.perf_counter() - t0) / reps
    return {"value": c["n"] / dt, "unit": "voxels/s", "cores": cores, "kind": "oracle",
            "sample": f"{reps} whole frame(s) of the same workload after 1 warm-up frame "
                      f"({c['n']} voxels, {len(c['schedule'])} layers, float64 numpy + tuple sort)"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=500)
    ap.add_argument("--warmup", type=int, default=100)
    ap.add_argument("--config", type=int, default=2)
    ap.add_argument("--no-cpu", action="store_true")
    ap.add_argument("--no-peaks", action="store_true", help="skip the stream-copy and MFMA-loop measurements")
    ap.add_argument("--no-saturation", action="store_true", help="skip the 128-frame saturation point")
    ap.add_argument("--sweep", action="store_true",
                    help="also time flatten / gather / scatter / layer on batches of frames (JSON lines on stderr)")
    ap.add_argument("--variant", type=int, default=0, help="wave-to-group mapping of the fused layer kernel (0 = auto)")
    ap.add_argument("--tail", choices=("mask", "drop"), default="mask",
                    help="short last groups attend over their members (mask) or skip the layer (drop, Sec. 4.3)")
    ap.add_argument("--f16", action="store_true",
                    help="IEEE half storage and operands instead of the configuration's bf16 (the paper's precision)")
    ap.add_argument("--pos-embed", action="store_true",
                    help="hand every layer a positional embedding [n, C] (second argument of the attention in Eq. (2))")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also launch one plain 256 MiB device copy (reference for scaling rocprofv3 byte counters)")
    a = ap.parse_args()
    if a.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (run with --gpus 1)", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import ffsynth
    import paper_2301_08739_amd as ff

    ff.load_library()
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    c = ffsynth.make_config(a.config)
    n, C, F, G, L = c["n"], c["C"], c["F"], c["G"], len(c["schedule"])
    dt = ff.FF_F32 if c["dtype"] == "f32" else (ff.FF_F16 if a.f16 else ff.FF_BF16)
    tdt = {ff.FF_F32: torch.float32, ff.FF_BF16: torch.bfloat16, ff.FF_F16: torch.float16}[dt]
    esz = 4 if dt == ff.FF_F32 else 2
    geom = ff.Geometry(c["B"], c["grid"], c["grid"], c["window"], c["window"])
    coords = torch.from_numpy(c["coords"]).to(dev)
    feats = torch.from_numpy(c["feats"]).to(dev).to(tdt)
    layers = [ff.LayerWeights(p, dt, dev) for p in c["layer_params"]]
    out = torch.empty_like(feats)
    ws = torch.empty(ff.ff_fwa_block_workspace_bytes(n, geom, G, layers, dt) + 512, dtype=torch.uint8, device=dev)

    tail = ff.FF_TAIL_DROP if a.tail == "drop" else ff.FF_TAIL_MASK
    pe = (0.5 * torch.randn_like(feats, dtype=torch.float32)).to(tdt) if a.pos_embed else None

    def step():
        ff.ff_fwa_block(coords, geom, G, layers, dt, feats, out=out, workspace=ws, tail=tail, pos_embed=pe)

    ms, wall_ms, step_stats = time_region(step, a.steps, a.warmup, stats=True)
    # how long the host needs to issue a step (the launches are asynchronous: the loop returns before the GPU is
    # done; the GPU time above is only meaningful while this stays below it)
    # (few enough steps that the launch queue never fills and pushes back)
    torch.cuda.synchronize()
    issue_steps = min(a.steps, 40)
    t0 = time.perf_counter()
    for _ in range(issue_steps):
        step()
    host_issue_ms = (time.perf_counter() - t0) * 1e3 / issue_steps
    torch.cuda.synchronize()
    # the same block replayed from a HIP graph: the kernels without the host's issue time between them
    ms_graph = graph_replay_ms(step, a.steps)
    # the same block with the layers' weights re-tiled once beforehand (weights that stay fixed across frames); the
    # headline step above re-tiles them inside every call
    layers_pk = [ff.LayerWeights(p, dt, dev).pack() for p in c["layer_params"]]
    ws_pk = torch.empty(ff.ff_fwa_block_workspace_bytes(n, geom, G, layers_pk, dt) + 512, dtype=torch.uint8, device=dev)
    out_pk = torch.empty_like(out)
    step_pk = lambda: ff.ff_fwa_block(coords, geom, G, layers_pk, dt, feats, out=out_pk, workspace=ws_pk, tail=tail,
                                      pos_embed=pe)
    ms_pk, _ = time_region(step_pk, a.steps, a.warmup)
    torch.cuda.synchronize()
    pk_ok = bool(torch.equal(out_pk, out))

    # ---- the same steps with two frames in flight: blocks issued alternately on two streams, each with
    # its own workspace and output buffer (what a serving loop that overlaps consecutive frames gets;
    # reported beside the headline, which stays one block after the other on one stream) ----
    ref_out = out.clone()
    side = [torch.cuda.Stream(), torch.cuda.Stream()]
    side_ws = [ws, torch.empty_like(ws)]
    side_out = [torch.empty_like(out), torch.empty_like(out)]

    def in_flight(k_steps):
        for k in range(k_steps):
            with torch.cuda.stream(side[k % 2]):
                ff.ff_fwa_block(coords, geom, G, layers, dt, feats, out=side_out[k % 2], workspace=side_ws[k % 2],
                                tail=tail, pos_embed=pe)

    torch.cuda.synchronize()
    in_flight(max(2, a.warmup))
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    in_flight(a.steps)
    torch.cuda.synchronize()
    ms_two = (time.perf_counter() - t0) * 1e3 / a.steps
    two_ok = bool(torch.equal(side_out[0], ref_out) and torch.equal(side_out[1], ref_out))

    # ---- the second input order: cells in row-major order, what a voxeliser's `unique` emits (the timed
    # workload keeps first-occurrence order); the gather's locality differs ----
    order = np.lexsort((c["coords"][:, 2], c["coords"][:, 1], c["coords"][:, 0]))
    coords_rm = torch.from_numpy(np.ascontiguousarray(c["coords"][order])).to(dev)
    assert np.array_equal(coords_rm.cpu().numpy(), ffsynth.row_major_order(c["coords"]))
    feats_rm = feats[torch.from_numpy(order).to(dev)].contiguous()
    ms_rm, _ = time_region(lambda: ff.ff_fwa_block(coords_rm, geom, G, layers, dt, feats_rm, out=out, workspace=ws,
                                                   tail=tail, pos_embed=pe), a.steps, a.warmup)

    # ---- per-part timings, same launch configuration as inside the block ----
    perm, goff, ng, _ = ff.ff_flatten(coords, geom, 0, 0, G, tail=tail)
    torch.cuda.synchronize()
    max_groups = -(-n // G) + c["B"]
    fws = torch.empty(ff.ff_flatten_batch_workspace_bytes(n, geom, 4) + 512, dtype=torch.uint8, device=dev)
    lws = torch.empty(ff.ff_group_attention_workspace_bytes(n, G, layers[0], dt) + 512, dtype=torch.uint8, device=dev)
    gth = torch.empty_like(feats)
    reps = max(a.steps, 20)
    ms_flat, _ = time_region(lambda: ff.ff_flatten(coords, geom, 0, 1, G, tail=tail, workspace=fws), reps, 5)
    # the block's own sorts: every distinct (axis, shift) pair of the schedule in one launch set
    sort_keys = list(dict.fromkeys(c["schedule"]))
    sorts4 = ff.ff_flatten_batch(coords, geom, sort_keys, G, tail=tail, workspace=fws)
    batch = lambda: ff.ff_flatten_batch(coords, geom, sort_keys, G, tail=tail, workspace=fws, out=sorts4)
    ms_sorts, _ = time_region(batch, reps, 5)
    ms_sorts_graph = graph_replay_ms(batch, reps)
    lpk = ff.LayerWeights(c["layer_params"][0], dt, dev).pack()       # exactly one kernel in the timed region
    vflag = ff.FF_FLAG_VARIANT(a.variant) | (ff.FF_FLAG_TAIL_DROP if a.tail == "drop" else 0)
    # The layer kernel as the method runs it: every launch reads the rows the launch before it wrote, grouped
    # by the next sort of the schedule (x, y, shifted x, shifted y), so its input comes from what other
    # XCDs wrote.  (The same launch repeated on a buffer nothing writes finds its rows in the local L2 and
    # is about 2 us faster: reported as ms_warm_input, not used for the roofline.)
    torch.cuda.synchronize()
    ping = [torch.empty_like(feats), torch.empty_like(feats)]
    ping[1].copy_(feats)
    ns = len(sorts4)

    def layer_chain():
        for k in range(4):
            p_, g_, n_ = sorts4[k % ns]
            ff.ff_group_attention(ping[(k + 1) & 1], p_, g_, n_, max_groups, lpk, G, dt, vflag, out=ping[k & 1],
                                  workspace=lws, pos_embed=pe)

    ms_chain, _, chain_stats = time_region(layer_chain, max(reps // 4, 5), 2, stats=True)
    ms_layer = ms_chain / 4
    ms_layer_graph = graph_replay_ms(layer_chain, max(reps // 4, 5)) / 4
    ms_layer_warm, _ = time_region(lambda: ff.ff_group_attention(feats, perm, goff, ng, max_groups, lpk, G, dt, vflag,
                                                                 out=out, workspace=lws, pos_embed=pe), reps, 5)
    ms_gather, _ = time_region(lambda: ff.ff_gather(feats, perm, dt, out=gth), reps, 5)
    ms_scatter, _ = time_region(lambda: ff.ff_scatter(gth, perm, dt, out=out), reps, 5)
    # launched alone, a 4 us copy kernel is timed with its launch gap; from a graph the gaps shrink
    ms_gather_graph = graph_replay_ms(lambda: [ff.ff_gather(feats, perm, dt, out=gth) for _ in range(8)], reps) / 8
    ms_scatter_graph = graph_replay_ms(lambda: [ff.ff_scatter(gth, perm, dt, out=out) for _ in range(8)], reps) / 8

    # the steps either side of the block: points -> pillars, pillars -> dense map
    m_pts, cp = 6 * n, 4
    xy_h, fr_h, pf_h = ffsynth.lidar_points(11, m_pts, c["B"], cp)
    xy_d, fr_d, pf_d = (torch.from_numpy(v).to(dev) for v in (xy_h, fr_h, pf_h))
    half = 0.5 * c["grid"] * 0.32
    vgrid = ff.VoxelGrid(-half, -half, 0.32, 0.32)
    vws = torch.empty(ff.ff_voxelize_workspace_bytes(m_pts, geom) + 512, dtype=torch.uint8, device=dev)
    _, _, npil, _ = ff.ff_voxelize(xy_d, fr_d, pf_d, geom, vgrid, want_map=False, workspace=vws)
    n_vox = int(npil.item())
    ms_vox, _ = time_region(lambda: ff.ff_voxelize(xy_d, fr_d, pf_d, geom, vgrid, want_map=False, workspace=vws), reps, 5)
    bev = torch.empty((c["B"], c["grid"], c["grid"], C), dtype=tdt, device=dev)
    ms_bev, _ = time_region(lambda: ff.ff_bev_scatter(feats, coords, geom, dt, out=bev), reps, 5)

    if a.copy_calibration:
        src = torch.empty(256 << 20, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    flops_layer = layer_flops_per_voxel(C, F, G) * n
    fb = flatten_bytes(n, c["B"], c["grid"], c["window"])
    bytes_rows = (2 * C * esz + 4) * n
    # voxelisation: inputs once, the sort credited like flatten (key = frame, x, y), the pillar rows once
    live_v = _bits(c["B"] + 1) + 2 * _bits(c["grid"])
    bytes_vox = (12 + 4 * cp) * m_pts + (28 + 24 * -(-live_v // 8)) * m_pts + (12 + 4 * cp) * n_vox
    bytes_bev = c["B"] * c["grid"] * c["grid"] * C * esz + (C * esz + 12) * n
    peak_tf = PEAK_F32_TFLOPS if dt == ff.FF_F32 else PEAK_BF16_TFLOPS
    ach_tf = flops_layer / (ms_layer * 1e-3) / 1e12
    default_run = a.variant == 0 and a.tail == "mask" and not a.pos_embed and not a.f16

    def hbm(nbytes, t_ms):
        return {"ms": t_ms, "bytes": nbytes, "GBps": nbytes / (t_ms * 1e-3) / 1e9,
                "frac_hbm": nbytes / (t_ms * 1e-3) / 1e9 / PEAK_HBM_GBS}

    def flat_part(t_ms, sorts):
        d = hbm(sorts * fb["algorithmic"], t_ms)
        d.update({"sorts": sorts, "radix_passes_credited": fb["passes_credited"], "radix_passes_run": fb["passes_run"],
                  "bytes_moved": sorts * fb["moved"], "GBps_moved": sorts * fb["moved"] / (t_ms * 1e-3) / 1e9,
                  "frac_hbm_moved": sorts * fb["moved"] / (t_ms * 1e-3) / 1e9 / PEAK_HBM_GBS})
        return d

    res = {
        "metric": "FWA block voxels/sec at 30k pillars C=128 G=64; %HBM BW sort, %MFMA attn",
        "value": n / (ms * 1e-3), "unit": "voxels/s", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": {ff.FF_F32: "f32", ff.FF_BF16: "bf16", ff.FF_F16: "f16"}[dt], "data": "synthetic",
        "config": {"workload": f"config {a.config} ({c['name']}): {n} pillars on {c['grid']}x{c['grid']}, "
                               f"B={c['B']}, window {c['window']}x{c['window']}, G={G}, C={C}, heads={c['heads']}, "
                               f"F={F}, {L} layers (x, y, shifted x, shifted y ...), "
                               f"{len(sort_keys)} sorts + {L} layers per step"
                               + (", short groups dropped" if a.tail == "drop" else "")
                               + (", with positional embedding" if a.pos_embed else "")},
        "step_stats_ms": step_stats, "graph_replay_ms": ms_graph,
        "prepacked_weights": {"ms_per_step": ms_pk, "voxels_per_s": n / (ms_pk * 1e-3), "same_result": pk_ok},
        "roofline": {"bound": "mfma", "kernel": "group attention layer (ff_group_attention, one launch; mean over launches chained through the four sorts)",
                     "achieved": ach_tf, "peak": peak_tf, "unit": "TFLOP/s", "frac": ach_tf / peak_tf,
                     "traffic": measured_layer_traffic(a.config) if default_run else None,
                     "algorithmic_bytes": bytes_rows, "ms": ms_layer, "ms_warm_input": ms_layer_warm,
                     "ms_graph_replay": ms_layer_graph,
                     "chain_of_4_stats_ms": chain_stats, "flops": flops_layer},
        "parts": {
            "flatten": flat_part(ms_flat, 1),
            "flatten_block_sorts": dict(flat_part(ms_sorts, len(sort_keys)), ms_graph_replay=ms_sorts_graph),
            "gather": dict(hbm(bytes_rows, ms_gather), ms_graph_replay=ms_gather_graph,
                           frac_hbm_graph_replay=bytes_rows / (ms_gather_graph * 1e-3) / 1e9 / PEAK_HBM_GBS),
            "scatter": dict(hbm(bytes_rows, ms_scatter), ms_graph_replay=ms_scatter_graph,
                            frac_hbm_graph_replay=bytes_rows / (ms_scatter_graph * 1e-3) / 1e9 / PEAK_HBM_GBS),
            "voxelize": dict(hbm(bytes_vox, ms_vox), points=m_pts, pillars=n_vox, point_feats=cp,
                             Mpoints_s=m_pts / ms_vox / 1e3),
            "bev_scatter": hbm(bytes_bev, ms_bev),
            "wall_ms_per_step": wall_ms, "host_issue_ms_per_step": host_issue_ms,
            "two_frames_in_flight": {"streams": 2, "ms_per_step": ms_two, "voxels_s": n / (ms_two * 1e-3),
                                     "equals_single_stream": two_ok},
            "row_major_input_order": {"ms_per_step": ms_rm, "voxels_s": n / (ms_rm * 1e-3)},
        },
    }
    del ping, gth, bev, side_out, side_ws
    torch.cuda.empty_cache()
    if not a.no_peaks:
        res["peaks_measured"] = peaks_measured(torch, dev)
    if not a.no_saturation and dt != ff.FF_F32:
        # the same kernels once the problem fills the machine: a batch of 128 frames of this workload
        res["saturation"] = saturation_point(ff, torch, c, dt, dev, 128, (0,))
    if not a.no_cpu:
        res["cpu_baseline"] = cpu_baseline(c)
    print(json.dumps(res), flush=True)
    if a.sweep:
        for B in (1, 8, 32, 128, 512):
            line = saturation_point(ff, torch, c, dt, dev, B, (0,) if dt == ff.FF_F32 else (6, 7, 11, 12))
            print(json.dumps(line), file=sys.stderr, flush=True)


def _bits(v):
    return int(v - 1).bit_length() if v > 1 else 0


def flatten_bytes(n, B, grid, window):
    """Bytes of one sort configuration (shifted geometry, the wider key).  algorithmic: what the method is
    credited with, 28 + 24 P per pillar for P = ceil(live key bits / 8) passes that move key and index as two
    arrays.  moved: what this implementation moves: one 64-bit word per pillar carries key and index, digits are
    up to 10 bits wide: coordinates in (12) and words out (8), 16 per pass but the last, which reads 8 and writes
    the 4-byte permutation; above 131,072 pillars every pass after the first also reads its words once more to
    count its tiles (8)."""
    nw = -(-(grid + window // 2) // window)
    live = _bits(B) + 2 * _bits(nw) + 2 * _bits(window)
    p8, p10 = -(-live // 8), max(1, -(-live // 10))
    moved = 12 + 8 + 16 * (p10 - 1) + 8 + 4 + (8 * (p10 - 1) if n > 131072 else 0)
    return {"algorithmic": (28 + 24 * p8) * n, "moved": moved * n, "passes_credited": p8, "passes_run": p10}


def saturation_point(ff, torch, c, dt, dev, B, variants):
    """flatten / gather / scatter / one layer on a batch of B frames of the configuration's frame (each frame
    cyclically shifted by a random offset of its own, frame id in column 0, rows shuffled), same C / G."""
    import numpy as np
    n1, C, F, G = c["n"], c["C"], c["F"], c["G"]
    esz = 4 if dt == ff.FF_F32 else 2
    tdt = {ff.FF_F32: torch.float32, ff.FF_BF16: torch.bfloat16, ff.FF_F16: torch.float16}[dt]
    lw = ff.LayerWeights(c["layer_params"][0], dt, dev).pack()
    coords = np.tile(c["coords"], (B, 1))
    coords[:, 0] = np.repeat(np.arange(B, dtype=np.int32), n1)
    rng = np.random.default_rng(B)
    # every frame gets its own cyclic offset: identical frames would give every window the same
    # population in every frame, a regularity real batches do not have
    off = rng.integers(0, c["grid"], size=(B, 2))
    off[0] = 0
    coords[:, 1:] = (coords[:, 1:] + np.repeat(off, n1, axis=0)) % c["grid"]
    coords = np.ascontiguousarray(coords[rng.permutation(coords.shape[0])])
    n = coords.shape[0]
    geom = ff.Geometry(B, c["grid"], c["grid"], c["window"], c["window"])
    ct = torch.from_numpy(coords).to(dev)
    feats = torch.randn((n, C), device=dev, dtype=torch.float32).to(tdt)
    out = torch.empty_like(feats)
    gth = torch.empty_like(feats)
    fws = torch.empty(ff.ff_flatten_workspace_bytes(n, geom) + 512, dtype=torch.uint8, device=dev)
    lws = torch.empty(ff.ff_group_attention_workspace_bytes(n, G, lw, dt) + 512, dtype=torch.uint8, device=dev)
    perm, goff, ng, _ = ff.ff_flatten(ct, geom, 0, 1, G, workspace=fws)
    torch.cuda.synchronize()
    mg = -(-n // G) + B
    reps = 20 if B <= 32 else (8 if B <= 128 else 4)
    fb = flatten_bytes(n, B, c["grid"], c["window"])
    rows = (2 * C * esz + 4) * n
    line = {"frames": B, "n": n, "radix_passes_credited": fb["passes_credited"], "radix_passes_run": fb["passes_run"]}
    ms, _ = time_region(lambda: ff.ff_flatten(ct, geom, 0, 1, G, workspace=fws), reps, 3)
    line["flatten"] = {"ms": ms, "GBps": fb["algorithmic"] / ms / 1e6, "frac_hbm": fb["algorithmic"] / ms / 1e6 / PEAK_HBM_GBS,
                       "GBps_moved": fb["moved"] / ms / 1e6, "frac_hbm_moved": fb["moved"] / ms / 1e6 / PEAK_HBM_GBS,
                       "Mvox_s": n / ms / 1e3}
    ms, _ = time_region(lambda: ff.ff_gather(feats, perm, dt, out=gth), reps, 3)
    line["gather"] = {"ms": ms, "GBps": rows / ms / 1e6, "frac_hbm": rows / ms / 1e6 / PEAK_HBM_GBS}
    ms, _ = time_region(lambda: ff.ff_scatter(gth, perm, dt, out=out), reps, 3)
    line["scatter"] = {"ms": ms, "GBps": rows / ms / 1e6, "frac_hbm": rows / ms / 1e6 / PEAK_HBM_GBS}
    flops = layer_flops_per_voxel(C, F, G) * n
    peak_tf = PEAK_F32_TFLOPS if dt == ff.FF_F32 else PEAK_BF16_TFLOPS
    for variant in variants:
        name = "layer" if variant == 0 else f"layer_v{variant}"
        try:
            fl = ff.FF_FLAG_VARIANT(variant)
            ms, _ = time_region(lambda: ff.ff_group_attention(feats, perm, goff, ng, mg, lw, G, dt, fl, out=out,
                                                              workspace=lws), reps, 3)
            line[name] = {"ms": ms, "TFLOPs": flops / ms / 1e9, "frac_mfma": flops / ms / 1e9 / peak_tf,
                          "Mvox_s": n / ms / 1e3}
        except ff.FlatformerError as e:
            line[name] = str(e)
    return line


if __name__ == "__main__":
    main()
