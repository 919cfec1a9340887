#!/usr/bin/env python3
"""Benchmark of the SharpV pruning hot path on one MI355X.

A step is one pass of the whole path over the long-video workload (256 frames x 196 tokens,
d=3584 bf16): `sharpv_prune_tokens` once (score + select + compact), then `sharpv_prune_kv` on
every layer of the 28-layer cache (cosine + decision + K/V gather).  Inputs are synthetic, seeded
and resident in HBM before the timed region starts.

Prints ONE JSON line.  `value` is visual tokens per second through score+select+compact (the
pre-LLM stage, timed inside the steps with events on the launch stream); `kv_prune` carries the
intra-LLM stage's GB/s per layer call against the HBM peak; `roofline` describes the kernel that
takes most of the step (kv_cosine), its duration measured with HIP events around every launch;
`cpu_baseline` is the CPU oracle timed on this machine's host cores.
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

HBM_PEAK_GBPS = 8000.0          # MI355X HBM3E, published peak


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", type=int, default=5, help="workload 1..8 (5 = the 256-frame video; 6, 7 = other model shapes; 8 = tall frames)")
    ap.add_argument("--layers", type=int, default=0, help="KV layers per step (0 = all layers of the config)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cold-mb", type=int, default=768,
                    help="the timed steps rotate over as many copies of the inputs as make this many MB "
                         "(more than the 256 MB Infinity Cache holds); 0 = always the same buffers")
    ap.add_argument("--no-two-streams", dest="two_streams", action="store_false",
                    help="skip the pass that deals the KV layer calls to two streams (its kernels overlap, so "
                         "profiler runs that average kernel durations leave it out)")
    ap.add_argument("--threads", type=int, default=min(16, os.cpu_count() or 1), help="input generator threads")
    return ap.parse_args()


def main() -> int:
    args = parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU; --gpus N with N > 1 is not supported "
              "(the path has no collectives between GPUs)", file=sys.stderr)
        return 2

    import numpy as np
    import torch
    from paper_2511_08003_amd import sharpv, workloads as wl

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    sharpv.load()
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    cfg = wl.config(args.config)
    esz = wl.elem_bytes(cfg.dtype)
    tdt = torch.bfloat16 if cfg.dtype == wl.BF16 else torch.float32

    def to_dev(a):
        if cfg.dtype == wl.BF16:
            return torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).view(torch.bfloat16).to(dev)
        return torch.from_numpy(np.ascontiguousarray(a, np.float32)).to(dev)

    # ------------------------------------------------------------------ inputs (seeded, synthetic)
    t0 = time.time()
    tok = wl.tokens_for(cfg, threads=args.threads)
    lay = wl.kv_layout_for(cfg)
    n, f, d = tok.n_total, cfg.f, cfg.d
    Nv, S = n * f, lay.S
    feats = to_dev(tok.feats)
    orig = feats.view(Nv, d)
    orig32 = wl.storage_to_f32(tok.feats, tok.dtype).reshape(-1, d)
    layers = list(range(cfg.n_layers)) if args.layers <= 0 else list(range(min(args.layers, cfg.n_layers)))
    hidden, Kc, Vc = [], [], []
    host_layer0 = None
    for l in layers:
        kv = wl.kv_layer_for(cfg, tok, l, threads=args.threads, orig32=orig32)
        hidden.append(to_dev(kv["hidden"]))
        Kc.append(to_dev(kv["K"]))
        Vc.append(to_dev(kv["V"]))
        if l == layers[len(layers) // 2]:
            host_layer0 = (l, kv)
    del orig32
    ragged = lay.B > 1
    fo = torch.from_numpy(tok.frame_offsets).to(dev) if tok.B > 1 else None
    so = torch.from_numpy(lay.seq_offsets).to(dev) if ragged else None
    vs = torch.from_numpy(lay.vis_start).to(dev) if ragged else None
    vo = torch.from_numpy(lay.vis_offsets).to(dev) if ragged else None
    gen_s = time.time() - t0

    ptok = sharpv.default_params(cfg.dtype)
    tplan = sharpv.TokensPlan(n, f, d, ptok, device=dev, scores=False, ratio=False)
    kplan = sharpv.KvPlan(lay.B, S, lay.n_vis, d, cfg.H, cfg.D, ptok, device=dev, cos=False, mean_cos=False)
    kept_per_layer = torch.zeros(len(layers), dtype=torch.int64, device=dev)

    # A workload whose inputs fit in the 256 MB Infinity Cache is timed over several copies of them, taken
    # in turn, so that no step finds its inputs cached (the 256-frame workload needs no copy: one step reads
    # 10 GB); the same-buffer figure is reported beside it as the warm one.
    step_input_bytes = feats.nbytes + sum(hidden[i].nbytes + Kc[i].nbytes + Vc[i].nbytes for i in range(len(layers)))
    copies = 1 if args.cold_mb <= 0 else max(1, -(-args.cold_mb * (1 << 20) // step_input_bytes))
    sets = [(feats, hidden, Kc, Vc)]
    for _ in range(copies - 1):
        sets.append((feats.clone(), [h.clone() for h in hidden], [k.clone() for k in Kc], [v.clone() for v in Vc]))

    def stage1(c=0):
        rc = tplan.run(sets[c][0], fo)
        if rc:
            raise RuntimeError(sharpv.status_string(rc))

    def stage2(i, c=0):
        ft, hd, kc, vc = sets[c]
        rc = kplan.run(hd[i], ft.view(Nv, d), kc[i], vc[i], int(lay.vis_start[0]), so, vs, vo, layers[i])
        if rc:
            raise RuntimeError(sharpv.status_string(rc))

    def step(ev=None, c=0):
        if ev:
            ev[0].record()
        stage1(c)
        if ev:
            ev[1].record()
        for i in range(len(layers)):
            stage2(i, c)
        if ev:
            ev[2].record()

    # kept counts (for the algorithmic byte counts), outside the timed region
    stage1()
    torch.cuda.synchronize()
    kept_tokens = int(tplan.out_offsets[-1].item())
    for i in range(len(layers)):
        stage2(i)
        kept_per_layer[i] = kplan.out_count.sum()
    torch.cuda.synchronize()
    kept_kv = kept_per_layer.cpu().numpy().astype(np.int64)

    # ------------------------------------------------------------------ timed region
    def timed_steps(rotate):
        for k in range(args.warmup):
            step(None, k % copies if rotate else 0)
        torch.cuda.synchronize()
        evs = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(args.steps)]
        torch.cuda.synchronize()
        t_start = time.perf_counter()
        for k in range(args.steps):
            step(evs[k], (args.warmup + k) % copies if rotate else 0)
        torch.cuda.synchronize()
        wall = (time.perf_counter() - t_start) * 1e3
        return (wall / args.steps, sum(e[0].elapsed_time(e[1]) for e in evs) / args.steps,
                sum(e[1].elapsed_time(e[2]) for e in evs) / args.steps)

    ms_per_step, ms_stage1, ms_stage2 = timed_steps(True)
    ms_stage2_layer = ms_stage2 / len(layers)
    warm = None
    if copies > 1:
        _, w1, w2 = timed_steps(False)
        warm = {"stage1_ms": round(w1, 4), "visual_tokens_per_s": round(Nv / (w1 * 1e-3), 1),
                "kv_prune_ms_per_layer": round(w2 / len(layers), 4)}

    # ------------------------------------------------------------------ the same step replayed from a captured HIP graph
    # (the entry points only enqueue kernels, so the whole step records into one graph)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    graph.replay()
    torch.cuda.synchronize()
    eg = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    eg[0].record()
    for _ in range(args.steps):
        graph.replay()
    eg[1].record()
    torch.cuda.synchronize()
    ms_graph_step = eg[0].elapsed_time(eg[1]) / args.steps

    # ------------------------------------------------------------------ the KV stage with the layers dealt to two streams
    # (each stream has its own outputs and workspace; one layer's gather then overlaps the next layer's cosines)
    ms_two_streams_layer = None
    kplan_b = sharpv.KvPlan(lay.B, S, lay.n_vis, d, cfg.H, cfg.D, ptok, device=dev, cos=False, mean_cos=False) \
        if args.two_streams else None
    side = [torch.cuda.Stream(device=dev), torch.cuda.Stream(device=dev)] if args.two_streams else []   # default priority
    plans2 = [kplan, kplan_b]

    def stage2_two_streams():
        cur = torch.cuda.current_stream()
        for sst in side:
            sst.wait_stream(cur)
        for i in range(len(layers)):
            with torch.cuda.stream(side[i & 1]):
                rc = plans2[i & 1].run(hidden[i], orig, Kc[i], Vc[i], int(lay.vis_start[0]), so, vs, vo, layers[i])
                if rc:
                    raise RuntimeError(sharpv.status_string(rc))
        for sst in side:
            cur.wait_stream(sst)

    if args.two_streams:
        stage2_two_streams()
        torch.cuda.synchronize()
        e2 = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
        e2[0].record()
        for _ in range(args.steps):
            stage2_two_streams()
        e2[1].record()
        torch.cuda.synchronize()
        ms_two_streams_layer = e2[0].elapsed_time(e2[1]) / (args.steps * len(layers))

    # ------------------------------------------------------------------ the KV stage with rotary re-encoding of the kept K rows
    # (same step, sharpv_prune_kv_rope instead of sharpv_prune_kv; reported beside the headline, not in it)
    theta = 1e6 ** (-2.0 * np.arange(cfg.D // 2) / cfg.D)
    ang = np.arange(S)[:, None] * theta[None, :]
    rope_cos = torch.from_numpy(np.cos(ang).astype(np.float32)).to(dev)
    rope_sin = torch.from_numpy(np.sin(ang).astype(np.float32)).to(dev)

    def stage2_rope(i):
        rc = kplan.run(hidden[i], orig, Kc[i], Vc[i], int(lay.vis_start[0]), so, vs, vo, layers[i], rope_cos, rope_sin)
        if rc:
            raise RuntimeError(sharpv.status_string(rc))

    for i in range(len(layers)):
        stage2_rope(i)
    torch.cuda.synchronize()
    er = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    er[0].record()
    for _ in range(args.steps):
        for i in range(len(layers)):
            stage2_rope(i)
    er[1].record()
    torch.cuda.synchronize()
    ms_rope_layer = er[0].elapsed_time(er[1]) / (args.steps * len(layers))

    # ------------------------------------------------------------------ the KV stage in its layer-to-layer form
    # (sharpv_prune_kv_carried on the full sequence with the block map: same rows, the visual tokens found
    # through the position -> original-row map)
    rows_np = np.full(S, -1, np.int32)
    rows_np[lay.visual_positions()] = np.arange(lay.n_vis, dtype=np.int32)
    rows_dev = torch.from_numpy(rows_np).to(dev)
    cplan = sharpv.KvCarriedPlan(lay.B, S, lay.n_vis, d, cfg.H, cfg.D, ptok, device=dev, cos=False)

    def stage2_carried(i):
        rc = cplan.run(hidden[i], orig, rows_dev, Kc[i], Vc[i], so, layers[i])
        if rc:
            raise RuntimeError(sharpv.status_string(rc))

    for i in range(len(layers)):
        stage2_carried(i)
    torch.cuda.synchronize()
    ec = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    ec[0].record()
    for _ in range(args.steps):
        for i in range(len(layers)):
            stage2_carried(i)
    ec[1].record()
    torch.cuda.synchronize()
    ms_carried_layer = ec[0].elapsed_time(ec[1]) / (args.steps * len(layers))

    # ------------------------------------------------------------------ per-kernel durations (events around every launch)
    launches_per_step = 6 + 5 * len(layers)
    n_ceiling = 6
    sharpv.timing_enable(launches_per_step * args.steps + 6 * n_ceiling + 8)
    for _ in range(args.steps):
        step()
    for i in range(len(layers)):
        stage2_rope(i)
    # practical HBM ceilings of this device: plain read and plain copy of buffers of the same size
    # class (hidden states of different layers, so nothing is served from cache); and the floors of the
    # pre-LLM stage's two memory-bound passes: the features read in the fused kernel's slab pattern with the
    # arithmetic left out, and the kept rows copied with the selection already made
    sink = torch.zeros(4, dtype=torch.int32, device=dev)
    for k in range(n_ceiling):
        sharpv.stream_read(hidden[k % len(hidden)], sink)
    for k in range(n_ceiling):
        sharpv.stream_copy(tplan.out_feats, hidden[k % len(hidden)][:Nv])
    kept_idx = tplan.out_idx[:kept_tokens].clone()
    for k in range(n_ceiling):
        # between two floor measurements a layer's hidden states pass through the caches, as in a step
        sharpv.stream_read(hidden[k % len(hidden)], sink)
        if f <= 208:
            sharpv.stream_read_slabs(sets[k % copies][0], sink)
        sharpv.stream_read(hidden[(k + 1) % len(hidden)], sink)
        if kept_tokens:
            sharpv.stream_gather_rows(tplan.out_feats, sets[k % copies][0].view(Nv, d), kept_idx)
    torch.cuda.synchronize()
    kern = {}
    for name in sharpv.KERNEL_NAMES:
        cnt, ms = sharpv.timing_read(name)
        if cnt:
            kern[name] = {"launches": cnt, "avg_us": round(ms / cnt * 1e3, 3)}
    sharpv.timing_disable()

    # ------------------------------------------------------------------ algorithmic bytes (per launch / per call)
    row = d * esz
    bytes_stage1 = Nv * row + kept_tokens * row + 4 * kept_tokens + 8 * n
    kv_row = cfg.H * cfg.D * esz
    bytes_cos = 2 * lay.n_vis * row                                   # hidden + original rows of the visual tokens
    bytes_gather_avg = float(np.mean(4 * kept_kv * kv_row + 4 * kept_kv))   # read + write kept K and V rows, indices
    bytes_stage2_avg = bytes_cos + bytes_gather_avg
    gbps_stage1 = bytes_stage1 / (ms_stage1 * 1e-3) / 1e9
    gbps_stage2 = bytes_stage2_avg / (ms_stage2_layer * 1e-3) / 1e9
    tokens_per_s = Nv / (ms_stage1 * 1e-3)

    dom = "kv_cosine"
    dom_gbps = bytes_cos / (kern[dom]["avg_us"] * 1e-6) / 1e9
    hid_bytes = hidden[0].numel() * esz
    # re-encoding adds one row of each table (D/2 float32 cos + sin) per kept position
    bytes_gather_rope_avg = bytes_gather_avg + float(np.mean(kept_kv)) * cfg.D * 4
    gbps_rope = (bytes_cos + bytes_gather_rope_avg) / (ms_rope_layer * 1e-3) / 1e9
    for name, b in (("kv_cosine", bytes_cos), ("kv_gather", bytes_gather_avg), ("kv_gather_rope", bytes_gather_rope_avg),
                    ("frame_slab", Nv * row),
                    ("frame_mean", Nv * row), ("token_dots", Nv * row), ("token_gather", 2 * kept_tokens * row),
                    ("stream_read", hid_bytes), ("stream_copy", 2 * Nv * row), ("stream_read_slabs", Nv * row),
                    ("stream_gather_rows", 2 * kept_tokens * row)):
        if name in kern:
            kern[name]["alg_GBps"] = round(b / (kern[name]["avg_us"] * 1e-6) / 1e9, 1)

    # HBM bytes of the dominant kernel come from the committed counter runs (profiles/*_traffic.json), not from
    # this run: they are reported only while the kernel sources are the ones those runs were taken on, with
    # the file named beside them.  The same records carry the profiler's durations of the two plain streaming
    # kernels, which are the ceilings to hold the kernels against (event timing adds 2-4 us to every launch).
    import hashlib
    csrc = os.path.join(ROOT, "paper_2511_08003_amd", "csrc")
    sha = hashlib.sha256(b"".join(open(os.path.join(csrc, fn), "rb").read()
                                  for fn in sorted(os.listdir(csrc)))).hexdigest()

    def committed_record(name):
        rel = os.path.join("profiles", name)
        try:
            rec = json.load(open(os.path.join(ROOT, rel)))
        except Exception:
            return None, None
        if rec.get("sources_sha256") != sha or rec.get("workload") != cfg.name:
            return None, None
        return rec, rel

    rec_cos, src_cos = committed_record("kv_cosine_c5_256f_traffic.json")
    traffic = rec_cos["traffic_bytes_per_launch"] if rec_cos and len(layers) == cfg.n_layers else None
    rec_slab, src_slab = committed_record("frame_slab_c5_256f_traffic.json")
    traffic_slab = rec_slab["traffic_bytes_per_launch"] if rec_slab else None
    prof = (rec_cos or {}).get("profiler_avg_us", {})

    out = {
        "metric": "visual tokens/sec through score+select+compact; KV-prune GB/s vs HBM peak",
        "value": round(tokens_per_s, 1),
        "unit": "visual tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32",                                   # the arithmetic type of every score and decision
        "storage_dtype": "f32" if cfg.dtype == wl.F32 else "bf16",
        "data": "synthetic",
        "config": {"workload": cfg.name, "frames": n, "tokens_per_frame": f, "d": d, "visual_tokens": Nv,
                   "kv_layers_per_step": len(layers), "kv_heads": cfg.H, "head_dim": cfg.D, "seq_len": S,
                   "w": 1.0, "M": 0.2, "kept_tokens": kept_tokens,
                   "kept_kv_positions_mean": round(float(kept_kv.mean()), 1)},
        "input_copies_rotated": copies, "warm_same_buffers": warm,
        "stage1": {"ms": round(ms_stage1, 4), "alg_bytes": int(bytes_stage1), "GBps": round(gbps_stage1, 1),
                   "frac_hbm_peak": round(gbps_stage1 / HBM_PEAK_GBPS, 4)},
        "kv_prune": {"ms_per_layer": round(ms_stage2_layer, 4), "alg_bytes_per_layer": int(bytes_stage2_avg),
                     "GBps": round(gbps_stage2, 1), "frac_hbm_peak": round(gbps_stage2 / HBM_PEAK_GBPS, 4)},
        "kv_prune_rope": {"ms_per_layer": round(ms_rope_layer, 4),
                          "alg_bytes_per_layer": int(bytes_cos + bytes_gather_rope_avg), "GBps": round(gbps_rope, 1),
                          "frac_hbm_peak": round(gbps_rope / HBM_PEAK_GBPS, 4)},
        "kv_prune_carried": {"ms_per_layer": round(ms_carried_layer, 4),
                             "alg_bytes_per_layer": int(bytes_stage2_avg + 4 * S + 4 * float(np.mean(kept_kv))),
                             "GBps": round((bytes_stage2_avg + 4 * S + 4 * float(np.mean(kept_kv)))
                                           / (ms_carried_layer * 1e-3) / 1e9, 1)},
        "kv_prune_two_streams": None if ms_two_streams_layer is None else {
            "ms_per_layer": round(ms_two_streams_layer, 4),
            "GBps": round(bytes_stage2_avg / (ms_two_streams_layer * 1e-3) / 1e9, 1),
            "frac_hbm_peak": round(bytes_stage2_avg / (ms_two_streams_layer * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4)},
        "graph_replay_ms_per_step": round(ms_graph_step, 4),
        "tokens_per_s_whole_step": round(Nv / (ms_per_step * 1e-3), 1),
        "roofline": {"kernel": dom, "bound": "hbm", "achieved": round(dom_gbps, 1), "peak": HBM_PEAK_GBPS,
                     "unit": "GB/s", "frac": round(dom_gbps / HBM_PEAK_GBPS, 4), "traffic": traffic,
                     "traffic_source": src_cos if traffic is not None else None,
                     "alg_bytes_per_launch": int(bytes_cos), "avg_launch_us": kern[dom]["avg_us"],
                     "timing": "HIP events around every launch"},
        "roofline_stage1": None if "frame_slab" not in kern else {
            "kernel": "frame_slab", "bound": "hbm", "achieved": kern["frame_slab"]["alg_GBps"], "peak": HBM_PEAK_GBPS,
            "unit": "GB/s", "frac": round(kern["frame_slab"]["alg_GBps"] / HBM_PEAK_GBPS, 4), "traffic": traffic_slab,
            "traffic_source": src_slab if traffic_slab is not None else None,
            "alg_bytes_per_launch": int(Nv * row), "avg_launch_us": kern["frame_slab"]["avg_us"]},
        "kernels": kern,
        # plain streaming kernels of this library on this device, timed like every kernel above (events around
        # the launch, 2-4 us more than the kernel itself); the profiler's durations of the same two kernels, from
        # the committed record, are what a kernel's own profiler duration is to be compared with
        "hbm_ceiling": {"read_GBps_event_timed": kern.get("stream_read", {}).get("alg_GBps"),
                        "copy_GBps_event_timed": kern.get("stream_copy", {}).get("alg_GBps"),
                        "read_GBps_profiler": None if "stream_read" not in prof else
                        round(hid_bytes / (prof["stream_read"] * 1e-6) / 1e9, 1),
                        "copy_GBps_profiler": None if "stream_copy" not in prof else
                        round(2 * Nv * row / (prof["stream_copy"] * 1e-6) / 1e9, 1),
                        "profiler_source": src_cos if prof else None},
        # the pre-LLM stage's two memory-bound passes with everything but the memory traffic taken out
        "stage1_floors": None if "stream_read_slabs" not in kern or "stream_gather_rows" not in kern else {
            "read_in_slab_order_us": kern["stream_read_slabs"]["avg_us"],
            "copy_kept_rows_us": kern["stream_gather_rows"]["avg_us"],
            "frac_hbm_peak_at_floors": round(bytes_stage1 / ((kern["stream_read_slabs"]["avg_us"]
                                                             + kern["stream_gather_rows"]["avg_us"]) * 1e-6)
                                             / 1e9 / HBM_PEAK_GBPS, 4),
            "timing": "HIP events around every launch, like the kernels they bound"},
        "input_generation_s": round(gen_s, 1),
    }

    # ------------------------------------------------------------------ CPU oracle on this machine's cores
    if not args.no_cpu_baseline:
        from oracle import canon
        canon.lib()
        reps = 5
        canon.prune_tokens(tok.feats, cfg.dtype, tok.frame_offsets)              # page the inputs in
        t0 = time.perf_counter()
        for _ in range(reps):
            canon.prune_tokens(tok.feats, cfg.dtype, tok.frame_offsets)
        cpu_s1 = (time.perf_counter() - t0) / reps
        l0, kv0 = host_layer0
        t0 = time.perf_counter()
        for _ in range(reps):
            ck = canon.prune_kv(kv0["hidden"], tok.feats.reshape(-1, d), kv0["K"], kv0["V"], cfg.dtype,
                                lay.seq_offsets, lay.vis_start, lay.vis_offsets, M=0.2)
        cpu_s2 = (time.perf_counter() - t0) / reps
        b2 = bytes_cos + 4 * len(ck["idx"]) * kv_row + 4 * len(ck["idx"])
        cores = canon.threads()
        # one core: the whole pre-LLM stage of this workload, and the same layer of the intra-LLM stage
        canon.set_threads(1)
        t0 = time.perf_counter()
        canon.prune_tokens(tok.feats, cfg.dtype, tok.frame_offsets)
        cpu_s1_single = time.perf_counter() - t0
        t0 = time.perf_counter()
        canon.prune_kv(kv0["hidden"], tok.feats.reshape(-1, d), kv0["K"], kv0["V"], cfg.dtype,
                       lay.seq_offsets, lay.vis_start, lay.vis_offsets, M=0.2)
        cpu_s2_single = time.perf_counter() - t0
        canon.set_threads(cores)
        # the 32-frame workload (the paper's own clip length, Table 2), both stages, all cores and one core
        c2 = wl.config(2)
        tok2 = wl.tokens_for(c2, threads=args.threads)
        lay2 = wl.kv_layout_for(c2)
        kv2 = wl.kv_layer_for(c2, tok2, c2.kv_layers[0], threads=args.threads)
        o2 = tok2.feats.reshape(-1, c2.d)

        def c2_pass():
            t0 = time.perf_counter()
            canon.prune_tokens(tok2.feats, c2.dtype, tok2.frame_offsets)
            t1 = time.perf_counter()
            canon.prune_kv(kv2["hidden"], o2, kv2["K"], kv2["V"], c2.dtype, lay2.seq_offsets, lay2.vis_start,
                           lay2.vis_offsets, M=0.2)
            return t1 - t0, time.perf_counter() - t1

        c2_pass()
        c2_all = [c2_pass() for _ in range(reps)]
        canon.set_threads(1)
        c2_one = c2_pass()
        canon.set_threads(cores)
        c2_s1 = sum(a for a, _ in c2_all) / reps
        c2_s2 = sum(b for _, b in c2_all) / reps
        core_seconds = reps * (cpu_s1 + cpu_s2) * cores + cpu_s1_single + cpu_s2_single \
            + reps * (c2_s1 + c2_s2) * cores + sum(c2_one)
        out["cpu_baseline"] = {
            "value": round(Nv / cpu_s1, 1), "unit": "visual tokens/s", "cores": cores, "kind": "oracle",
            "sample": f"float32 canonical-order oracle (C, OpenMP over frames / tokens, {cores} threads), mean of {reps} "
                      f"runs: pre-LLM stage on all {n} frames of the workload ({cpu_s1:.3f} s per run); intra-LLM "
                      f"stage on layer {l0} of the same workload ({cpu_s2:.3f} s per run); the same two once on one "
                      f"thread ({cpu_s1_single:.3f} s, {cpu_s2_single:.3f} s); the 32-frame workload {c2.name} likewise; "
                      f"about {core_seconds:.0f} core-seconds in all",
            "kv_prune_GBps": round(b2 / cpu_s2 / 1e9, 3),
            "single_thread_value": round(Nv / cpu_s1_single, 1),
            "single_thread_kv_prune_GBps": round(b2 / cpu_s2_single / 1e9, 3),
            "kv_prune_28_layers_s_single_thread": round(cpu_s2_single * cfg.n_layers, 2),
            "c2_32f": {"value": round(c2.n_vis / c2_s1, 1), "single_thread_value": round(c2.n_vis / c2_one[0], 1),
                       "kv_prune_ms": round(c2_s2 * 1e3, 3), "single_thread_kv_prune_ms": round(c2_one[1] * 1e3, 3)},
        }
    print(json.dumps(out), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
