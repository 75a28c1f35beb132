#!/usr/bin/env python3
"""Benchmark of the Flattened Window Attention block on one MI355X.

One "step" = one pass of the whole hot path over one synthetic frame: the sorts of the block
(window keys, radix argsort, grouping; each distinct (axis, shift) pair once) followed by the
layer stack (gather, LayerNorm, QKV, softmax attention, out-proj, FFN, scatter per layer).
Inputs are resident in HBM before the timed region.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 2] [--tail mask|drop] [--pos-embed] [--f16] [--no-cpu] [--sweep]
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

# HBM bytes per launch of the fused layer kernel, from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE scaled by
# a plain copy of known size (profiles/fwa_layer_cfg2_hbm_counters.txt): config id -> bytes.
MEASURED_LAYER_TRAFFIC = {2: 18374656}


def layer_flops_per_voxel(C, F, G):
    # QKV 6C^2 + QK^T 2GC + PV 2GC + out-proj 2C^2 + FFN 4CF (multiply-add = 2 flops)
    return 8 * C * C + 4 * G * C + 4 * C * F


def time_region(fn, steps, warmup):
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
    return e0.elapsed_time(e1) / steps, wall / steps


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
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", type=int, default=2)
    ap.add_argument("--no-cpu", action="store_true")
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

    ms, wall_ms = time_region(step, a.steps, a.warmup)

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

    # ---- per-part timings, same launch configuration as inside the block ----
    perm, goff, ng, _ = ff.ff_flatten(coords, geom, 0, 0, G, tail=tail)
    torch.cuda.synchronize()
    max_groups = -(-n // G) + c["B"]
    fws = torch.empty(ff.ff_flatten_workspace_bytes(n, geom) + 512, dtype=torch.uint8, device=dev)
    lws = torch.empty(ff.ff_group_attention_workspace_bytes(n, G, layers[0], dt) + 512, dtype=torch.uint8, device=dev)
    gth = torch.empty_like(feats)
    reps = max(a.steps, 20)
    ms_flat, _ = time_region(lambda: ff.ff_flatten(coords, geom, 0, 1, G, tail=tail, workspace=fws), reps, 5)
    lpk = ff.LayerWeights(c["layer_params"][0], dt, dev).pack()       # exactly one kernel in the timed region
    vflag = ff.FF_FLAG_VARIANT(a.variant) | (ff.FF_FLAG_TAIL_DROP if a.tail == "drop" else 0)
    # The layer kernel as the method runs it: every launch reads the rows the launch before it wrote, grouped
    # by the next sort of the schedule (x, y, shifted x, shifted y), so its input comes from what other
    # XCDs wrote.  (The same launch repeated on a buffer nothing writes finds its rows in the local L2 and
    # is about 2 us faster: reported as ms_warm_input, not used for the roofline.)
    sorts4 = [ff.ff_flatten(coords, geom, k % 2, (k // 2) % 2, G, tail=tail)[:3] for k in range(4)]
    torch.cuda.synchronize()
    ping = [torch.empty_like(feats), torch.empty_like(feats)]
    ping[1].copy_(feats)

    def layer_chain():
        for k in range(4):
            p_, g_, n_ = sorts4[k]
            ff.ff_group_attention(ping[(k + 1) & 1], p_, g_, n_, max_groups, lpk, G, dt, vflag, out=ping[k & 1],
                                  workspace=lws, pos_embed=pe)

    ms_chain, _ = time_region(layer_chain, max(reps // 4, 5), 2)
    ms_layer = ms_chain / 4
    ms_layer_warm, _ = time_region(lambda: ff.ff_group_attention(feats, perm, goff, ng, max_groups, lpk, G, dt, vflag,
                                                                 out=out, workspace=lws, pos_embed=pe), reps, 5)
    ms_gather, _ = time_region(lambda: ff.ff_gather(feats, perm, dt, out=gth), reps, 5)
    ms_scatter, _ = time_region(lambda: ff.ff_scatter(gth, perm, dt, out=out), reps, 5)

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

    flops_layer = layer_flops_per_voxel(C, F, G) * n
    # live key bits -> radix passes (8 bits each), shifted geometry
    def bits(v):
        return int(v - 1).bit_length() if v > 1 else 0
    s = c["window"] // 2
    nw = -(-(c["grid"] + s) // c["window"])
    live = bits(c["B"]) + 2 * bits(nw) + 2 * bits(c["window"])
    passes = -(-live // 8)
    bytes_flat = (28 + 24 * passes) * n
    bytes_rows = (2 * C * esz + 4) * n
    # voxelisation: inputs once, the sort credited like flatten (key = frame, x, y), the pillar rows once
    live_v = bits(c["B"] + 1) + 2 * bits(c["grid"])
    bytes_vox = (12 + 4 * cp) * m_pts + (28 + 24 * -(-live_v // 8)) * m_pts + (12 + 4 * cp) * n_vox
    bytes_bev = c["B"] * c["grid"] * c["grid"] * C * esz + (C * esz + 12) * n
    peak_tf = PEAK_F32_TFLOPS if dt == ff.FF_F32 else PEAK_BF16_TFLOPS
    ach_tf = flops_layer / (ms_layer * 1e-3) / 1e12

    res = {
        "metric": "FWA block voxels/sec at 30k pillars C=128 G=64; %HBM BW sort, %MFMA attn",
        "value": n / (ms * 1e-3), "unit": "voxels/s", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": {ff.FF_F32: "f32", ff.FF_BF16: "bf16", ff.FF_F16: "f16"}[dt], "data": "synthetic",
        "config": {"workload": f"config {a.config} ({c['name']}): {n} pillars on {c['grid']}x{c['grid']}, "
                               f"B={c['B']}, window {c['window']}x{c['window']}, G={G}, C={C}, heads={c['heads']}, "
                               f"F={F}, {L} layers (x, y, shifted x, shifted y ...), "
                               f"{len(dict.fromkeys(c['schedule']))} sorts + {L} layers per step"
                               + (", short groups dropped" if a.tail == "drop" else "")
                               + (", with positional embedding" if a.pos_embed else "")},
        "roofline": {"bound": "mfma", "kernel": "group attention layer (ff_group_attention, one launch; mean over launches chained through the four sorts)",
                     "achieved": ach_tf, "peak": peak_tf, "unit": "TFLOP/s", "frac": ach_tf / peak_tf,
                     "traffic": MEASURED_LAYER_TRAFFIC.get(a.config) if a.variant == 0 and a.tail == "mask" and not a.pos_embed and not a.f16 else None,
                     "algorithmic_bytes": bytes_rows, "ms": ms_layer, "ms_warm_input": ms_layer_warm,
                     "flops": flops_layer},
        "parts": {
            "flatten": {"ms": ms_flat, "bytes": bytes_flat, "GBps": bytes_flat / (ms_flat * 1e-3) / 1e9,
                        "frac_hbm": bytes_flat / (ms_flat * 1e-3) / 1e9 / PEAK_HBM_GBS, "radix_passes_credited": passes},
            "gather": {"ms": ms_gather, "bytes": bytes_rows, "GBps": bytes_rows / (ms_gather * 1e-3) / 1e9,
                       "frac_hbm": bytes_rows / (ms_gather * 1e-3) / 1e9 / PEAK_HBM_GBS},
            "scatter": {"ms": ms_scatter, "bytes": bytes_rows, "GBps": bytes_rows / (ms_scatter * 1e-3) / 1e9,
                        "frac_hbm": bytes_rows / (ms_scatter * 1e-3) / 1e9 / PEAK_HBM_GBS},
            "voxelize": {"ms": ms_vox, "points": m_pts, "pillars": n_vox, "point_feats": cp,
                         "Mpoints_s": m_pts / ms_vox / 1e3, "bytes": bytes_vox, "GBps": bytes_vox / (ms_vox * 1e-3) / 1e9,
                         "frac_hbm": bytes_vox / (ms_vox * 1e-3) / 1e9 / PEAK_HBM_GBS},
            "bev_scatter": {"ms": ms_bev, "bytes": bytes_bev, "GBps": bytes_bev / (ms_bev * 1e-3) / 1e9,
                            "frac_hbm": bytes_bev / (ms_bev * 1e-3) / 1e9 / PEAK_HBM_GBS},
            "wall_ms_per_step": wall_ms,
            "two_frames_in_flight": {"streams": 2, "ms_per_step": ms_two, "voxels_s": n / (ms_two * 1e-3),
                                     "equals_single_stream": two_ok},
        },
    }
    if not a.no_cpu:
        res["cpu_baseline"] = cpu_baseline(c)
    print(json.dumps(res), flush=True)
    if a.sweep:
        sweep(ff, torch, c, dt, dev)


def sweep(ff, torch, c, dt, dev):
    """Saturation sweep: a batch of B frames (the frame of the configuration, cyclically shifted by a
    random offset per frame; frame id in column 0), same C / G."""
    import numpy as np
    n1, C, F, G = c["n"], c["C"], c["F"], c["G"]
    esz = 4 if dt == ff.FF_F32 else 2
    tdt = {ff.FF_F32: torch.float32, ff.FF_BF16: torch.bfloat16, ff.FF_F16: torch.float16}[dt]
    lw = ff.LayerWeights(c["layer_params"][0], dt, dev).pack()
    for B in (1, 8, 32, 128, 512):
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
        def bits(v):
            return int(v - 1).bit_length() if v > 1 else 0
        nw = -(-(c["grid"] + c["window"] // 2) // c["window"])
        passes = -(-(bits(B) + 2 * bits(nw) + 2 * bits(c["window"])) // 8)
        line = {"sweep_frames": B, "n": n, "radix_passes": passes}
        ms, _ = time_region(lambda: ff.ff_flatten(ct, geom, 0, 1, G, workspace=fws), reps, 3)
        line["flatten"] = {"ms": ms, "GBps": (28 + 24 * passes) * n / ms / 1e6, "Mvox_s": n / ms / 1e3}
        ms, _ = time_region(lambda: ff.ff_gather(feats, perm, dt, out=gth), reps, 3)
        line["gather"] = {"ms": ms, "GBps": (2 * C * esz + 4) * n / ms / 1e6}
        ms, _ = time_region(lambda: ff.ff_scatter(gth, perm, dt, out=out), reps, 3)
        line["scatter"] = {"ms": ms, "GBps": (2 * C * esz + 4) * n / ms / 1e6}
        flops = layer_flops_per_voxel(C, F, G) * n
        for variant in ((0,) if dt == ff.FF_F32 else (6, 7, 11)):
            try:
                fl = ff.FF_FLAG_VARIANT(variant)
                ms, _ = time_region(lambda: ff.ff_group_attention(feats, perm, goff, ng, mg, lw, G, dt, fl, out=out,
                                                                  workspace=lws), reps, 3)
                line[f"layer_v{variant}"] = {"ms": ms, "TFLOPs": flops / ms / 1e9, "Mvox_s": n / ms / 1e3}
            except ff.FlatformerError as e:
                line[f"layer_v{variant}"] = str(e)
        print(json.dumps(line), file=sys.stderr, flush=True)


if __name__ == "__main__":
    main()
