#!/usr/bin/env python3
"""Benchmark of the tree-verification stage hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload C2] [--no-cpu-baseline]

A step is one pass of the whole hot path over one synthetic batch, for a LLaMA2-7B-shaped 8-layer last
stage (workload C2): the 64-node draft tree is verified in 4 score-ordered segments of 16 tokens (stage
forward + LM head + row argmax each), acceptance is planted on the logits, then greedy accept with the
continuous condition, KV-cache compaction and pruning of one in-flight segment.  All inputs are resident
in HBM before the timed region.  One JSON line is printed: verified draft tokens/s of the stage, the
roofline of the dominant kernel (gate/up projection: HBM weight stream) measured with HIP events, and the
CPU oracle timed on the host cores for one segment of the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0  # MI355X published HBM3E bandwidth
GEMM_SRC = "paper_2507_02620_amd/csrc/gemm.hip"


def source_sha(rel):
    """sha256 (first 16 hex digits) of a source file of the library, the stamp the counter summaries under profiles/ carry."""
    import hashlib
    try:
        return hashlib.sha256(open(os.path.join(ROOT, rel), "rb").read()).hexdigest()[:16]
    except OSError:
        return None


def read_traffic(path, source_rel):
    """(HBM bytes per launch, stale) of the dominant kernel from a committed rocprofv3 --pmc summary: the file holds a line
    'traffic_bytes: N' and a line 'kernel_source_sha256: H' with the stamp of the kernel's source file at the time the counters
    were taken.  stale = the source has changed since (or the file has no stamp): the figure is then context, not evidence.
    Counters cannot be read inside a timed run, so this one number comes from a file; everything else in the line is measured live."""
    traffic, stamp = None, None
    try:
        for line in open(path):
            if line.startswith("traffic_bytes:"):
                traffic = float(line.split(":")[1])
            if line.startswith("kernel_source_sha256:"):
                stamp = line.split(":")[1].strip()
    except OSError:
        return None, None
    return traffic, (stamp is None or stamp != source_sha(source_rel))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="C2", choices=["C1", "C2", "C3", "C4", "C5", "P1", "P2"])
    ap.add_argument("--layers", type=int, default=0, help="override the number of layers (debug only; invalidates the metric)")
    ap.add_argument("--seg-len", type=int, default=0, help="override the segment length l_s (debug only; invalidates the metric)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-head", action="store_true", help="time the stage forward alone (an intermediate stage)")
    ap.add_argument("--weights", default="dense", choices=["dense", "int4"],
                    help="int4: 4-bit group weights with bf16 activations (W4A16, the paper's 13B setting); bf16 workloads only")
    ap.add_argument("--temperature", type=float, default=0.0, help="> 0: stochastic acceptance at that temperature instead of greedy")
    ap.add_argument("--no-extras", action="store_true", help="default run only: skip the two short extra legs (long-context attention, "
                    "1024-row projections) that reuse the stage's weights")
    ap.add_argument("--no-probes", action="store_true", help="skip the achievable-peak probes (pure streaming read, pure MFMA loop) and the "
                    "large-size KV compaction measurement")
    ap.add_argument("--batch", type=int, default=1, metavar="B",
                    help="B > 1: B independent requests (own KV cache, tree and hidden states) served by the stage together through "
                         "fs_tree_verify_batch; tokens/s counts all of them")
    ap.add_argument("--graph", action="store_true", help="capture one whole step into a HIP graph and time its replays")
    ap.add_argument("--calibrate-copy", type=int, default=0, metavar="MiB",
                    help="before the timed region, run one plain device-to-device copy of this many MiB (a kernel of known "
                         "traffic that scales the FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc run)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2507_02620_amd import flowspec as fs
    from paper_2507_02620_amd import synth

    cfg = synth.CONFIGS[args.workload]
    if args.layers:
        cfg = cfg.with_(n_layers=args.layers)
    if args.seg_len:
        cfg = cfg.with_(seg_len=args.seg_len)
    seed = 0
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    tdt = torch.float32 if cfg.dtype == "f32" else torch.bfloat16
    use_head = cfg.vocab > 0 and not args.no_head

    t_setup = time.time()
    B = max(1, args.batch)
    if B > 1 and (args.temperature > 0 or B > fs.FS_MAX_BATCH or B * cfg.seg_len > 1024):
        print("bench.py: --batch needs greedy acceptance, B <= %d and B * segment <= 1024" % fs.FS_MAX_BATCH, file=sys.stderr)
        sys.exit(2)
    w4 = args.weights == "int4"
    up = lambda a: None if a is None else torch.from_numpy(a).to(dev, tdt)
    if w4:
        host_layers = [synth.layer_weights_w4(cfg, l, seed) for l in range(cfg.n_layers)]
        fn, lm, lm_scale = synth.head_weights_w4(cfg, seed) if use_head else (None, None, None)
        codes = lambda a: None if a is None else torch.from_numpy(a).to(dev)
        dev_layers = [{k: (codes(v) if v is not None and v.dtype == np.uint8 else up(v)) for k, v in lw.items()} for lw in host_layers]
        dfn, dlm, dls = up(fn), codes(lm), up(lm_scale)
        stage = fs.stage_from_config(cfg, dev_layers, dfn, dlm, lm_head_scale=dls, weight_format=fs.FS_WFMT_INT4_G128, max_seg=B * cfg.seg_len)
    else:
        host_layers = [synth.layer_weights(cfg, l, seed) for l in range(cfg.n_layers)]
        fn, lm = synth.head_weights(cfg, seed) if use_head else (None, None)
        dev_layers = [{k: up(v) for k, v in lw.items()} for lw in host_layers]
        dfn, dlm, dls = up(fn), up(lm), None
        stage = fs.stage_from_config(cfg, dev_layers, dfn, dlm, max_seg=B * cfg.seg_len)
    torch.cuda.synchronize()
    extras_on = (args.workload == "C2" and B == 1 and not w4 and not args.no_extras and not args.layers and not args.seg_len
                 and args.temperature <= 0 and not args.no_head)
    extra_stages = {}
    if extras_on:
        # the same device weights re-tiled into two more stages (same layer shape): the long-context workload (the one where
        # tree attention carries weight) and the 1024-row chunk (the one where the projections are bound by the matrix units)
        for name in ("C5", "P2"):
            xc = synth.CONFIGS[name]
            extra_stages[name] = fs.stage_from_config(xc, dev_layers, None, None, kv_capacity=xc.l_glo + xc.tree_size + xc.seg_len,
                                                      max_tree=xc.tree_size, max_seg=xc.seg_len)
        torch.cuda.synchronize()
    del dev_layers, dfn, dlm, dls
    torch.cuda.empty_cache()
    kv = stage.new_kv_cache()
    for l in range(cfg.n_layers):
        kv[l].copy_(up(synth.prefix_kv(cfg, l, None, seed)))
    tree = synth.config_tree(cfg, seed)
    T = tree.size
    segs = synth.segments(T, cfg.seg_len)
    hid = up(synth.hidden(cfg, T, 0, seed))
    hid_segs = [hid[o:o + n].contiguous() for o, n in segs]
    out_segs = [torch.empty_like(h) for h in hid_segs]
    token_d = torch.from_numpy(tree.token).to(dev)
    parent_d = torch.from_numpy(tree.parent).to(dev)
    logits = torch.zeros((T, max(cfg.vocab, 1)), dtype=torch.float32, device=dev) if use_head else None
    amax = torch.zeros(T, dtype=torch.int32, device=dev)
    res, retain, work = fs.new_accept_buffers(T, T, dev)
    new_len = torch.zeros(2, dtype=torch.int32, device=dev)
    pr_out = torch.empty_like(hid_segs[-1])
    pr_n = torch.zeros(1, dtype=torch.int32, device=dev)
    plants = synth.resolve_plants(synth.plant_path(tree, T, seed, 0, p_stop=0.0, mean_extra=2.0), tree, max(cfg.vocab, 2))
    plant_rows = torch.tensor([r for r, _ in plants], dtype=torch.long, device=dev)
    plant_toks = torch.tensor([t for _, t in plants], dtype=torch.long, device=dev)
    swork = torch.empty(32 + 12 * T, dtype=torch.uint8, device=dev)
    step_no = [0]
    if B > 1:
        # requests 1 .. B-1: same prefix contents (a copy of request 0's cache), own tree, hidden states and planted path
        reqs = [dict(kv=kv, tree=tree, hid=hid, token=token_d, parent=parent_d, amax=amax, res=res, retain=retain, work=work,
                     plant_rows=plant_rows, plant_toks=plant_toks)]
        for r in range(1, B):
            tr = synth.random_tree(cfg.tree_size, cfg.max_depth, cfg.max_branch, max(cfg.vocab, 2), seed, stream=r, forest=cfg.forest)
            pl = synth.resolve_plants(synth.plant_path(tr, T, seed, r, p_stop=0.0, mean_extra=2.0), tr, max(cfg.vocab, 2))
            rs_, rt_, wk_ = fs.new_accept_buffers(T, T, dev)
            reqs.append(dict(kv=kv.clone(), tree=tr, hid=up(synth.hidden(cfg, T, r, seed)), token=torch.from_numpy(tr.token).to(dev),
                             parent=torch.from_numpy(tr.parent).to(dev), amax=torch.zeros(T, dtype=torch.int32, device=dev),
                             res=rs_, retain=rt_, work=wk_,
                             plant_rows=torch.tensor([a_ for a_, _ in pl], dtype=torch.long, device=dev),
                             plant_toks=torch.tensor([b_ for _, b_ in pl], dtype=torch.int32, device=dev)))
        stack_in = [torch.cat([q["hid"][o:o + n] for q in reqs], dim=0).contiguous() for o, n in segs]
        stack_out = [torch.empty_like(x) for x in stack_in]
        stack_logits = torch.zeros((B * cfg.seg_len, max(cfg.vocab, 1)), dtype=torch.float32, device=dev) if use_head else None
        # argmax rows of a segment arrive stacked [request][row of the segment]; one concatenation per step turns the segments'
        # arrays into [request][node], and one indexed store plants every request's accepted path
        seg_amax = [torch.zeros(B * n, dtype=torch.int32, device=dev) for _, n in segs]
        all_plant_req = torch.cat([torch.full_like(q["plant_rows"], r) for r, q in enumerate(reqs)])
        all_plant_rows = torch.cat([q["plant_rows"] for q in reqs])
        all_plant_toks = torch.cat([q["plant_toks"].to(torch.int32) for q in reqs])
    setup_s = time.time() - t_setup

    def step_batch():
        l_glo = cfg.l_glo
        for i, (off, n) in enumerate(segs):
            items = [(q["kv"], l_glo, l_glo + off, off, n, q["tree"].parent[: off + n]) for q in reqs]
            stage.tree_verify_batch(items, stack_in[i], stack_out[i])
            if use_head:
                stage.tree_logits(stack_out[i], stack_logits[: B * n], seg_amax[i])
        all_amax = torch.cat([a.view(B, -1) for a in seg_amax], dim=1)  # [request][node]
        # planted acceptance, written into the argmax (the logits of a batch stay stacked per segment)
        all_amax[all_plant_req, all_plant_rows] = all_plant_toks
        for r, q in enumerate(reqs):
            fs.tree_accept(None, all_amax[r], q["token"], q["parent"], T, q["res"], q["retain"], q["work"])
            stage.kv_compact(q["kv"], l_glo, l_glo + T, q["retain"], res=q["res"], new_len=new_len)
            fs.seg_prune(q["hid"][segs[-1][0]:], segs[-1][0], q["retain"], res=q["res"], seg_out=pr_out, l_s_out=pr_n)

    def step():
        l_glo = cfg.l_glo
        for i, (off, n) in enumerate(segs):
            stage.tree_verify_stage(kv, l_glo, l_glo + off, hid_segs[i], off, tree.parent[: off + n], out_segs[i])
            if use_head:
                stage.tree_logits(out_segs[i], logits[off:off + n], amax[off:off + n])
        if use_head:
            logits[plant_rows, plant_toks] += 100.0  # planted acceptance (stand-in for a trained draft model's hit rate)
            if args.temperature > 0:
                fs.tree_accept_sample(logits, args.temperature, token_d, parent_d, T, seed, step_no[0], res, retain, swork)
                step_no[0] += 1
            else:
                fs.tree_accept(logits, amax, token_d, parent_d, T, res, retain, work)
        else:
            amax[plant_rows] = plant_toks.to(torch.int32)
            fs.tree_accept(None, amax, token_d, parent_d, T, res, retain, work)
        stage.kv_compact(kv, l_glo, l_glo + T, retain, res=res, new_len=new_len)
        fs.seg_prune(hid_segs[-1], segs[-1][0], retain, res=res, seg_out=pr_out, l_s_out=pr_n)

    if args.calibrate_copy:
        src = torch.ones(args.calibrate_copy << 20, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    run = step_batch if B > 1 else step
    if args.graph:
        # every launch of the step (the library's kernels take the tree as kernel arguments, nothing is allocated or
        # cleared by memset) goes into one graph on a side stream; a replay is one step
        run()
        torch.cuda.synchronize()
        cap_stream = torch.cuda.Stream()
        graph = torch.cuda.CUDAGraph()
        if B > 1:
            with torch.cuda.graph(graph, stream=cap_stream):
                step_batch()  # the binding launches on the current stream, which is the capturing one here
        else:
            with torch.cuda.graph(graph, stream=cap_stream):
                cur = torch.cuda.current_stream().cuda_stream
                l_glo = cfg.l_glo
                for i, (off, n) in enumerate(segs):
                    stage.tree_verify_stage(kv, l_glo, l_glo + off, hid_segs[i], off, tree.parent[: off + n], out_segs[i], stream=cur)
                    if use_head:
                        stage.tree_logits(out_segs[i], logits[off:off + n], amax[off:off + n], stream=cur)
                if use_head:
                    logits[plant_rows, plant_toks] += 100.0
                    fs.tree_accept(logits, amax, token_d, parent_d, T, res, retain, work, stream=cur)
                else:
                    amax[plant_rows] = plant_toks.to(torch.int32)
                    fs.tree_accept(None, amax, token_d, parent_d, T, res, retain, work, stream=cur)
                stage.kv_compact(kv, l_glo, l_glo + T, retain, res=res, new_len=new_len, stream=cur)
                fs.seg_prune(hid_segs[-1], segs[-1][0], retain, res=res, seg_out=pr_out, l_s_out=pr_n, stream=cur)
        run = graph.replay
    for _ in range(args.warmup):
        run()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        run()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt / args.steps * 1e3
    tok_s = B * T * args.steps / dt

    # second pass of the same steps with the per-kernel event timers armed
    stage.profile_begin(args.steps * (len(segs) * (5 + B + 6 * cfg.n_layers) + 4 * B) + 16)
    for _ in range(args.steps):
        (step_batch if B > 1 else step)()
    prof = stage.profile_end()
    out_res, out_ret = fs.accept_result_to_host(res, retain, T)

    elem = 4 if cfg.dtype == "f32" else 2
    welem = (0.5 + 2.0 / 128) if w4 else elem                 # weight bytes per parameter (4-bit code + a bf16 scale per 128)
    gu_bytes = int(2 * cfg.d_ffn * cfg.d_model * welem)       # gate + up weights, streamed once per launch
    gu_ms, gu_n = prof["gateup"]
    gu_avg_ms = gu_ms / max(gu_n, 1)
    achieved = gu_bytes / (gu_avg_ms * 1e-3) / 1e9 if gu_n else 0.0
    kern = {k: {"avg_us": round(v[0] / v[1] * 1e3, 2), "launches": v[1]} for k, v in prof.items() if v[1]}
    stage_weight_bytes = cfg.n_layers * (2 * cfg.n_q_heads * cfg.head_dim * cfg.d_model + 2 * cfg.n_kv_heads * cfg.head_dim * cfg.d_model
                                         + 3 * cfg.d_ffn * cfg.d_model) * welem
    head_bytes = cfg.vocab * cfg.d_model * welem if use_head else 0
    kv_bytes = B * cfg.n_layers * 2 * cfg.n_kv_heads * cfg.head_dim * elem * sum(cfg.l_glo + o + n for o, n in segs)
    step_bytes = int(len(segs) * (stage_weight_bytes + head_bytes) + kv_bytes)

    # the metric's two companions: MFMA utilisation of the projections and HBM rate of the tree attention
    gemm_flops = 2.0 * B * sum(n for _, n in segs) * cfg.n_layers * (2 * cfg.n_q_heads * cfg.head_dim * cfg.d_model
                                                                   + 2 * cfg.n_kv_heads * cfg.head_dim * cfg.d_model + 3 * cfg.d_ffn * cfg.d_model)
    gemm_ms = sum(prof[k][0] for k in ("qkv", "oproj", "gateup", "down")) / args.steps
    mfma_peak = 157.3 if cfg.dtype == "f32" else 2500.0          # TFLOP/s, dense
    at_ms, at_n = prof["attn"]
    attn = None
    if at_n:
        at_bytes = kv_bytes / max(len(segs) * cfg.n_layers, 1)   # K and V of the visible slots, one layer, average segment
        at_avg = at_ms / at_n                                     # one record spans the attention kernel and its split merge
        attn = {"kernel": "tree attention (tree_attn_kernel, or tree_attn_dma_kernel where the split plan picks it) + attn_merge_kernel", "bound": "hbm", "algorithmic_bytes": int(at_bytes),
                "avg_us": round(at_avg * 1e3, 2), "achieved": round(at_bytes / (at_avg * 1e-3) / 1e9, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": round(at_bytes / (at_avg * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)}

    # many-row segments run the MFMA-bound projection kernel: the dominant kernel is then priced against the matrix peak
    rows_per_launch = B * min(cfg.seg_len, T)
    wide = cfg.dtype == "bf16" and not w4 and rows_per_launch >= 128
    if wide:
        gu_flops = 2.0 * rows_per_launch * 2 * cfg.d_ffn * cfg.d_model
        gu_tf = gu_flops / (gu_avg_ms * 1e-3) / 1e12 if gu_n else 0.0
        roofline = {"kernel": "wide_gemm_kernel<EPI_SWIGLU> (RMSNorm + gate/up + SiLU*up, %d rows)" % rows_per_launch, "bound": "mfma",
                    "achieved": round(gu_tf, 1), "peak": mfma_peak, "unit": "TFLOP/s", "frac": round(gu_tf / mfma_peak, 4),
                    "avg_launch_us": round(gu_avg_ms * 1e3, 2), "algorithmic_flops": gu_flops,
                    "traffic": None}
        if B == 1:
            roofline["traffic"], roofline["traffic_stale"] = read_traffic(os.path.join(ROOT, "profiles", "gateup_%s_traffic.txt" % args.workload.lower()), GEMM_SRC)
    else:
        roofline = {"kernel": "skinny_gemm%s_kernel<EPI_SWIGLU> (RMSNorm + gate/up + SiLU*up)" % ("_w4" if w4 else ""), "bound": "hbm",
                    "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
                    "avg_launch_us": round(gu_avg_ms * 1e3, 2), "algorithmic_bytes": gu_bytes,
                    "traffic": None}
        roofline["traffic"], roofline["traffic_stale"] = read_traffic(os.path.join(ROOT, "profiles", "gateup_%s%s_traffic.txt" % (args.workload.lower(), "_w4" if w4 else "")), GEMM_SRC)

    # KV compaction of the step: rows kept in the cache that actually move (retained draft rows), read + written, K and V, all layers
    cp_ms, cp_n = prof["compact"]
    n_keep = max(out_res.n_retain, 0)
    cp_bytes = 2 * 2 * n_keep * cfg.n_kv_heads * cfg.head_dim * elem * cfg.n_layers
    kvc = {"rows_kept": n_keep, "algorithmic_bytes": cp_bytes, "avg_us": round(cp_ms / max(cp_n, 1) * 1e3, 2),
           "achieved_GBs": round(cp_bytes / (cp_ms / max(cp_n, 1) * 1e-3) / 1e9, 1) if cp_n and cp_ms > 0 else None,
           "note": "a few rows per step: launch-latency bound at this size; see kv_compact_large"}
    achievable = None
    if not args.no_probes:
        # (1) what a launch can reach at all on this machine; (2) compaction at the largest size one call takes (1024-node
        # tree, every other node kept): the HBM-bound regime of the same kernel
        big = torch.empty((3 << 30) + 64, dtype=torch.uint8, device=dev)
        achievable = {"hbm_stream_read_GBs": round(fs.probe_stream_read(big, 176 << 20, 20), 1),
                      "hbm_stream_read_small_GBs": round(fs.probe_stream_read(big, 32 << 20, 20), 1),
                      "mfma_bf16_TFLOPs": round(fs.probe_mfma_bf16(big, 5), 1),
                      "note": "one-pass reads of 176 MiB / 32 MiB per launch rotating through 3 GiB; register-resident 16x16x32 bf16 MFMA loop"}
        del big
        torch.cuda.empty_cache()
        big = torch.empty((1 << 28) + 64, dtype=torch.uint8, device=dev)
        achievable["fill_l2_hit_GBs_per_cu"] = round(fs.probe_fill(big, 256, 8, 64, 512, 1, True, 3) / 256, 1)
        achievable["fill_beyond_l2_GBs_per_cu"] = round(fs.probe_fill(big, 256, 8, 512, 512, 1, True, 3) / 256, 1)
        achievable["fill_note"] = ("rate at which one compute unit (all 256 at once) pulls data into LDS with direct-to-LDS loads: from its "
                                   "XCD's L2 / from beyond it (128 MiB re-read cyclically); bounds the many-row projection kernels")
        del big
        torch.cuda.empty_cache()
        Tb = 1024
        # compaction only looks at the cache geometry, so a stage with the workload's layers / KV heads / head dim and
        # token-sized projections stands in (no second copy of the weights)
        cfg_b = cfg.with_(d_model=128, d_ffn=128, vocab=0, tree_size=Tb, seg_len=16)
        lw_b = [{k: up(v) for k, v in synth.layer_weights(cfg_b, l, seed).items()} for l in range(cfg_b.n_layers)]
        stage_b = fs.stage_from_config(cfg_b, lw_b, kv_capacity=cfg.l_glo + Tb + 64, max_tree=Tb, max_seg=16)
        kv_b = stage_b.new_kv_cache()
        # two retain sets of 512 of 1024 nodes: every other node (256-byte rows with 256-byte holes) and an accepted path of 4
        # plus one contiguous run (what a subtree looks like when its nodes were appended together)
        patterns = {"every_other_row": list(range(0, Tb, 2)), "path_plus_contiguous_run": [0, 1, 2, 3] + list(range(300, 808))}
        for pname, keep in patterns.items():
            ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            reps = 10
            for _ in range(2):
                stage_b.kv_compact(kv_b, cfg.l_glo, cfg.l_glo + Tb, keep, n_acc=4)
            ev0.record()
            for _ in range(reps):
                stage_b.kv_compact(kv_b, cfg.l_glo, cfg.l_glo + Tb, keep, n_acc=4)
            ev1.record()
            torch.cuda.synchronize()
            ms_b = ev0.elapsed_time(ev1) / reps
            moved = sum(1 for j, i in enumerate(keep) if i != j)
            bytes_b = 2 * 2 * moved * cfg.n_kv_heads * cfg.head_dim * elem * cfg.n_layers
            entry = {"rows_kept": len(keep), "rows_moved": moved, "of_tree_nodes": Tb, "algorithmic_bytes": bytes_b, "avg_us": round(ms_b * 1e3, 2),
                     "achieved_GBs": round(bytes_b / (ms_b * 1e-3) / 1e9, 1), "peak": HBM_PEAK_GBS,
                     "frac": round(bytes_b / (ms_b * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)}
            if pname == "every_other_row":
                kvc["kv_compact_large"] = entry
            else:
                kvc["kv_compact_large_" + pname] = entry
        del stage_b, kv_b, lw_b

    # the two extra legs of the default run: same weights, other geometry, a few steps each, every launch timed by events
    extras = None
    if extras_on:
        extras = {}
        for name, xst in extra_stages.items():
            xc = synth.CONFIGS[name]
            xkv = xst.new_kv_cache()
            xkv[:, :, :, : xc.l_glo].normal_()   # timing only: any finite prefix will do
            xtree = synth.config_tree(xc, seed)
            xsegs = synth.segments(xtree.size, xc.seg_len)
            xh = [torch.randn((n, xc.d_model), device=dev).to(tdt) for _, n in xsegs]
            xo = [torch.empty_like(h) for h in xh]

            def xstep():
                for i, (off, n) in enumerate(xsegs):
                    xst.tree_verify_stage(xkv, xc.l_glo, xc.l_glo + off, xh[i], off, xtree.parent[: off + n], xo[i])
            xsteps = 5
            for _ in range(2):
                xstep()
            torch.cuda.synchronize()
            t0x = time.perf_counter()
            for _ in range(xsteps):
                xstep()
            torch.cuda.synchronize()
            x_ms = (time.perf_counter() - t0x) / xsteps * 1e3
            xst.profile_begin(xsteps * len(xsegs) * (6 * xc.n_layers + 4) + 16)
            for _ in range(xsteps):
                xstep()
            xp = xst.profile_end()
            rows = min(xc.seg_len, xtree.size)
            ent = {"workload": xc.name, "stage": "intermediate (no head)", "ms_per_step": round(x_ms, 4), "steps": xsteps,
                   "rows_per_s": round(xtree.size / (x_ms * 1e-3), 1),
                   "kernels": {k: {"avg_us": round(v[0] / v[1] * 1e3, 2), "launches": v[1]} for k, v in xp.items() if v[1]}}
            if name == "C5":
                xb = 2 * xc.n_kv_heads * xc.head_dim * elem * sum(xc.l_glo + o + n for o, n in xsegs) / len(xsegs)
                at = xp["attn"][0] / xp["attn"][1]
                ent["tree_attention"] = {"kernel": "tree attention (tree_attn_dma_kernel where the split plan picks it, else tree_attn_kernel) + attn_merge_kernel", "bound": "hbm", "algorithmic_bytes": int(xb),
                                         "avg_us": round(at * 1e3, 2), "achieved": round(xb / (at * 1e-3) / 1e9, 1), "peak": HBM_PEAK_GBS,
                                         "unit": "GB/s", "frac": round(xb / (at * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)}
            else:
                gu = xp["gateup"][0] / xp["gateup"][1]
                fl = 2.0 * rows * 2 * xc.d_ffn * xc.d_model
                allf = 2.0 * rows * (2 * xc.n_q_heads * xc.head_dim * xc.d_model + 2 * xc.n_kv_heads * xc.head_dim * xc.d_model + 3 * xc.d_ffn * xc.d_model)
                allms = sum(xp[k][0] / xp[k][1] for k in ("qkv", "oproj", "gateup", "down"))
                ent["gateup_mfma"] = {"kernel": "gate/up projection, %d rows" % rows, "bound": "mfma", "algorithmic_flops": fl, "avg_us": round(gu * 1e3, 2),
                                      "achieved": round(fl / (gu * 1e-3) / 1e12, 1), "peak": 2500.0, "unit": "TFLOP/s",
                                      "frac": round(fl / (gu * 1e-3) / 1e12 / 2500.0, 4)}
                ent["projections_mfma_frac"] = round(allf / (allms * 1e-3) / 1e12 / 2500.0, 4)
            extras[name] = ent
            del xkv, xh, xo
            xst.close()
        extra_stages.clear()
        torch.cuda.empty_cache()

    result = {
        "metric": "verified draft tokens/sec per stage; MFMA util (GEMMs) + HBM GB/s (tree attn)",
        "value": round(tok_s, 1),
        "unit": "verified draft tokens/s per stage",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": cfg.name + ("-w4a16" if w4 else "") + ("-batch%d" % B if B > 1 else ""), "requests": B, "weights": "int4 codes, bf16 scale per 128 columns" if w4 else cfg.dtype, "stage": "last" if use_head else "intermediate", "n_layers": cfg.n_layers, "d_model": cfg.d_model,
                   "heads": f"{cfg.n_q_heads}q/{cfg.n_kv_heads}kv x {cfg.head_dim}", "d_ffn": cfg.d_ffn, "vocab": cfg.vocab if use_head else 0,
                   "kv_prefix": cfg.l_glo, "tree_nodes": T, "segment": cfg.seg_len, "segments_per_step": len(segs),
                   "step": "verify x%d + lm_head + accept + kv_compact + seg_prune" % len(segs),
                   "acceptance": "greedy" if args.temperature <= 0 else "sampled, temperature %g" % args.temperature},
        "roofline": roofline,
        "whole_step": {"algorithmic_bytes": step_bytes, "achieved_GBs": round(step_bytes / (ms_per_step * 1e-3) / 1e9, 1),
                       "frac_of_hbm_peak": round(step_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)},
        "tree_attention": attn,
        "kv_compact": kvc,
        "achievable": achievable,
        "gemm_mfma": {"flops_per_step": gemm_flops, "ms_per_step": round(gemm_ms, 4),
                      "achieved": round(gemm_flops / (gemm_ms * 1e-3) / 1e12, 2) if gemm_ms else None, "peak": mfma_peak, "unit": "TFLOP/s",
                      "util": round(gemm_flops / (gemm_ms * 1e-3) / 1e12 / mfma_peak, 5) if gemm_ms else None,
                      "note": ("rows per launch = segment length: MFMA-bound projection kernel" if wide else
                               "rows per launch = segment length: the projections are weight-stream bound, see roofline")},
        "kernels": kern,
        "extra_legs": extras,
        "accept": {"n_acc": out_res.n_acc, "continuous": out_res.continuous, "n_retain": out_res.n_retain},
        "setup_s": round(setup_s, 1),
    }

    if not args.no_cpu_baseline:
        from oracle import oracle  # cpu_baseline leg: the oracle as it stands, timed on the host cores
        bits = lambda a: None if a is None else synth.f32_to_bf16_bits(a)
        if w4:  # the oracle runs on the plain matrices the codes stand for
            ost = oracle.Stage(cfg, [oracle.dequant_layer(lw) for lw in host_layers], fn, None if lm is None else oracle.dequant_w4(lm, lm_scale))
        else:
            wl = host_layers if cfg.dtype == "f32" else [{k: bits(v) for k, v in lw.items()} for lw in host_layers]
            ost = oracle.Stage(cfg, wl, fn if cfg.dtype == "f32" else bits(fn), lm if cfg.dtype == "f32" else bits(lm), None,
                               bf16_bits=cfg.dtype != "f32")
        for l in range(cfg.n_layers):
            ost.load_prefix(l, synth.prefix_kv(cfg, l, None, seed))
        hs = synth.hidden(cfg, T, 0, seed)
        # the sample: whole steps of the same workload (every segment of the tree, LM head, accept, compaction), a few times
        times, y0 = [], None
        reps = 5 if cfg.n_layers * cfg.d_model * cfg.d_ffn <= 8 * 4096 * 11008 else 2
        for rep in range(reps):
            t0 = time.perf_counter()
            am_all = np.zeros(T, dtype=np.int32)
            for off, n in segs:
                y = ost.verify(cfg.l_glo, cfg.l_glo + off, hs[off:off + n], off, tree.parent[: off + n])
                if off == 0:
                    y0 = y
                if use_head:
                    am_all[off:off + n] = ost.logits(y)[1]
            o_res, o_ret = oracle.accept(am_all, tree.token, tree.parent, T)
            oracle.kv_compact(ost.kv, cfg.l_glo, cfg.l_glo + T, o_ret, o_res.n_acc)
            times.append(time.perf_counter() - t0)
        cdt = float(np.median(times))
        result["cpu_baseline"] = {"value": round(T / cdt, 3), "unit": "verified draft tokens/s per stage", "cores": oracle.num_threads(),
                                  "kind": "oracle", "sample": "%d whole steps (%d segments of %d tokens through all %d layers%s + accept + "
                                  "kv_compact each), fp64, median %.2f s per step, %.1f s in total" %
                                  (reps, len(segs), cfg.seg_len, cfg.n_layers, " + LM head" if use_head else "", cdt, sum(times))}
        # the GPU's first segment against the oracle's, as a sanity line (the parity tests are the gate)
        g = out_segs[0].float().cpu().numpy()
        result["cpu_baseline"]["gpu_vs_oracle_max_rel_err"] = float(np.abs(g - y0).max() / np.abs(y0).max())
    print(json.dumps(result))


if __name__ == "__main__":
    main()
