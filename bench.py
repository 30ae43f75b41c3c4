#!/usr/bin/env python3
"""Benchmark of the prefill-only adapter-apply hot path on one MI355X.

A "step" is one pass of the whole path over one synthetic batch: the adapter work of one decoder
layer on that batch,

    1 x token-segment scheduler                              (preft_schedule)
    7 x segmented multi-adapter LoRA, rank R, prefill-only   (q, k, v, o, gate, up, down; q,k,v and
                                                              gate,up go out as packed launches)
    1 x segmented multi-adapter DiReFT, rank R, prefill-only (the residual stream)

The default workload is the largest single-GPU configuration, `llama70b_lora` (512 prompts with
lognormal lengths + 3584 decode rows, 512 adapters, unsharded Llama-3.1-70B layer shapes, bf16) at
its heaviest rank, 64.  Every projection has its own activation buffers (about 100 GB in total),
so every launch streams cold data from HBM; adapter weights are warm (steady-state serving).
`value` = active (prompt) rows per second through the step.  Rows are laid out densely (row pitch
= width); `--pitch pow2` pads wide rows to the next power of two, which this chip streams faster.

The same JSON line carries: the HBM roofline of the dominant kernel (timed per launch with HIP
events on the launch stream inside the timed region; median over the steps), the all-token
(conventional PEFT) time of the same batch, the batch's decode rows alone as a decode-only step in
both modes, DiReFT at every layer, a serving-trace replay, the CPU oracle timed on a sample of the
same batch, and -- each measured in a short child process of this same script -- the same step on
the other configurations (`llama8b_lora` rank 16, `llama8b_direft` rank 16, `skewed70b` rank 32),
at the configuration's other ranks and with the power-of-two row pitch.
"""
import argparse
import hashlib
import json
import os
import subprocess
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_HBM_GBPS = 8000.0      # MI355X HBM3E, published
METRIC = "prefill tokens/s through multi-adapter LoRA/DiReFT apply; % of peak HBM GB/s"
DEFAULT_RANK = {"llama70b_lora": 64, "llama8b_lora": 16, "llama8b_direft": 16, "skewed70b": 32, "tiny": 4}
TRAFFIC_PROFILE = os.path.join("profiles", "lora_row_split_kernel_llama70b_rank64_hbm_traffic.txt")


def kernel_sources_sha256():
    """Hash of the kernel sources: a committed counter summary applies to the kernels it was taken from."""
    h = hashlib.sha256()
    csrc = os.path.join(ROOT, "paper_2605_14217_amd", "csrc")
    for name in sorted(os.listdir(csrc)):
        if name.endswith((".hpp", ".hip")):
            h.update(name.encode())
            with open(os.path.join(csrc, name), "rb") as f:
                h.update(f.read())
    return h.hexdigest()


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", default="llama70b_lora")
    ap.add_argument("--rank", type=int, default=0, help="adapter rank (0: the configuration's heaviest)")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--pitch", choices=["dense", "pow2"], default="dense",
                    help="row pitch of the activation buffers: their width (default) or the next power of two "
                         "(28672-wide rows every 32768 elements; measured 5-10 %% faster on MI355X)")
    ap.add_argument("--sub", action="store_true",
                    help="short form used for the child processes: main measurement, all-token and decode-only legs")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true", help="only the timed region (what the rocprofv3 summaries profile)")
    ap.add_argument("--no-children", action="store_true", help="skip the other configurations, ranks and row pitch")
    ap.add_argument("--no-trace", action="store_true", help="skip the serving-trace replay leg")
    ap.add_argument("--no-packed", action="store_true",
                    help="one launch per projection instead of packed q,k,v and gate,up launches")
    ap.add_argument("--no-z", action="store_true",
                    help="workspace without room for z: every LoRA call runs both sweeps in one launch")
    ap.add_argument("--only", default="", help="experiment: comma-separated subset of projections")
    ap.add_argument("--variant", type=int, default=0)
    ap.add_argument("--waves", type=int, default=0)
    ap.add_argument("--rowblocks", type=int, default=0)
    ap.add_argument("--colsplit", type=int, default=0)
    ap.add_argument("--resident", type=int, default=0)
    ap.add_argument("--ldpad", type=int, default=0, help="experiment: extra elements of row stride on every buffer")
    ap.add_argument("--trace-requests", type=int, default=1000)
    ap.add_argument("--trace-batch", type=int, default=32)
    ap.add_argument("--trace-adapters", type=int, default=32)
    ap.add_argument("--trace-mix", default="uniform", choices=["identical", "uniform", "skewed", "distinct"])
    ap.add_argument("--trace-slots", type=int, default=0,
                    help="serve the trace through the adapter slot manager with this many device slots "
                         "(0: every adapter resident); --trace-adapters may then exceed the configuration's pool")
    ap.add_argument("--cpu-rows-per-segment", type=int, default=32,
                    help="random rows per prompt in the sample the CPU oracle is timed on")
    return ap.parse_args()


def experiment_flags(args):
    return bool(args.variant or args.waves or args.rowblocks or args.colsplit or args.resident or args.ldpad or args.only
                or args.no_packed or args.no_z)


def run(args):
    import numpy as np
    import torch

    import paper_2605_14217_amd as preft
    from paper_2605_14217_amd import workloads as wl

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    preft.load_library()
    preft.set_test_flags(preft.test_flags(variant=args.variant, waves=args.waves, rowblocks=args.rowblocks,
                                          colsplit=args.colsplit, resident=args.resident))
    dev = "cuda:0"
    torch.cuda.set_device(0)

    cfg = wl.CONFIGS[args.config]
    r = args.rank or DEFAULT_RANK[args.config]
    N, d_res = cfg["N"], cfg["direft_d"]
    scale = cfg["lora_scale"]
    tab = wl.make_segments(args.config, seed=args.seed)
    T, S = tab.T, tab.S
    T_act = tab.active_rows(False, N)
    n_ad = tab.distinct_active_adapters(False, N)
    ss, sa, sp = (torch.from_numpy(a.copy()).to(dev) for a in (tab.seg_start, tab.seg_adapter, tab.seg_prefill_len))
    # with room for z the LoRA calls at rank 20..64 run their sweeps as two launches where that is faster
    # (preft_workspace_bytes_z)
    ws = preft.new_workspace(T, S, device=dev, z_rank=0 if args.no_z else r, z_proj=3)

    # ---- buffers and pools --------------------------------------------------------------
    projs = []

    def act(T_, d_, seed_):
        pitch = d_ + args.ldpad
        if args.pitch == "pow2":                       # row pitch = next power of two (a caller's layout choice)
            pitch = 1 << (d_ - 1).bit_length()
        if pitch != d_:
            buf = torch.empty((T_, pitch), dtype=torch.bfloat16, device=dev)
            step_rows = max(1, (1 << 28) // pitch)     # filled piecewise: no second full-size temporary
            for lo in range(0, T_, step_rows):
                hi = min(T_, lo + step_rows)
                buf[lo:hi, :d_].copy_(wl.activations(hi - lo, d_, "bf16", device=dev, seed=seed_ * 131 + lo))
            return buf[:, :d_]
        return wl.activations(T_, d_, "bf16", device=dev, seed=seed_)

    for i, (name, (d_in, d_out)) in enumerate(cfg["lora_shapes"].items()):
        if args.only and name not in args.only.split(","):
            continue
        pool = wl.lora_pool(N, r, d_in, d_out, "bf16", device=dev, seed=args.seed + 10 + i)
        A = [pool.A[j] for j in range(N)]
        B = [pool.B[j] for j in range(N)]
        projs.append(dict(name=name, d_in=d_in, d_out=d_out, pool=pool,
                          Ap=preft.pointer_table(A), Bp=preft.pointer_table(B),
                          x=act(T, d_in, args.seed + 100 + i), y=act(T, d_out, args.seed + 200 + i)))
    dpool = wl.direft_pool(N, r, d_res, "bf16", device=dev, seed=args.seed + 50)
    W1 = [dpool.A[j] for j in range(N)]
    W2t = [dpool.B[j].t().contiguous() for j in range(N)]
    bb = [dpool.b[j] for j in range(N)]
    W1p, W2tp, bp = preft.pointer_table(W1), preft.pointer_table(W2t), preft.pointer_table(bb)
    h = act(T, d_res, args.seed + 300)
    direft_scale = 1.0

    # launches of a step: projections that read the same x (q,k,v; gate,up) go out as one packed call
    # (one launch that reads x once for bf16 ranks 1-16 and, widths being multiples of 128, for ranks 17-64;
    # above, the call issues one launch per projection)
    packs = {"q": "qkv", "k": "qkv", "v": "qkv", "gate": "gate_up", "up": "gate_up"}
    packed = not args.no_packed and r <= 64
    groups = []
    for p in projs:
        key = packs.get(p["name"]) if packed else None
        if key is not None and groups and groups[-1]["key"] == key and groups[-1]["members"][0]["d_in"] == p["d_in"]:
            groups[-1]["members"].append(p)
        else:
            groups.append(dict(key=key, members=[p]))
    for g_ in groups:
        g_["name"] = "+".join(m["name"] for m in g_["members"])
    singles = [dict(key=None, members=[p], name=p["name"]) for p in projs]

    def step(mode, tables=(ss, sa, sp), T_=T, events=None, groups=groups, pools=None):
        # pools: {projection: (A table, B table), "direft": (W1, W2t, b tables), "N": slots} from a slot manager
        s0, s1, s2 = tables
        preft.preft_schedule(ws, s0, s1, s2, T_, N if pools is None else pools["N"], mode)
        ready = mode | preft.PREFT_SCHEDULE_READY
        for i, g_ in enumerate(groups):
            m = g_["members"]
            if events is not None:
                events[i][0].record()
            Aps = [q["Ap"] if pools is None else pools[q["name"]][0] for q in m]
            Bps = [q["Bp"] if pools is None else pools[q["name"]][1] for q in m]
            if len(m) == 1:
                preft.preft_lora_apply(m[0]["y"][:T_], m[0]["x"][:T_], s0, s1, s2, Aps[0], Bps[0], r, scale, ready, ws)
            else:
                preft.preft_lora_apply_packed([q["y"][:T_] for q in m], m[0]["x"][:T_], s0, s1, s2, Aps, Bps, r, scale,
                                              ready, ws)
            if events is not None:
                events[i][1].record()
        if events is not None:
            events[len(groups)][0].record()
        d1, d2, d3 = (W1p, W2tp, bp) if pools is None else pools["direft"]
        preft.preft_direft_apply(h[:T_], s0, s1, s2, d1, d2, d3, r, direft_scale, ready, ws)
        if events is not None:
            events[len(groups)][1].record()

    def timed(fn, iters, warm):
        for _ in range(warm):
            fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(iters):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / iters * 1e3

    # ---- timed region: K prefill-only steps ------------------------------------------------
    K, W = args.steps, args.warmup
    ev = [[(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
           for _ in range(len(groups) + 1)] for _ in range(K)]
    for _ in range(W):
        step(preft.PREFT_PREFILL_ONLY)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(K):
        step(preft.PREFT_PREFILL_ONLY, events=ev[k])
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) / K * 1e3
    counts = preft.preft_schedule_counts(ws)

    per_launch_ms = np.array([[a.elapsed_time(b) for (a, b) in evk] for evk in ev])     # [K, launches]
    med_ms = np.median(per_launch_ms, axis=0)             # median over the K timed steps
    breakdown, launch_bytes = {}, {}
    lora_b, lora_t = 0.0, 0.0
    for i, g_ in enumerate(groups):
        m = g_["members"]
        # x once per launch, every output read and written once, every distinct adapter's factors once
        b = wl.lora_algorithmic_bytes(T_act, m[0]["d_in"], [q["d_out"] for q in m], r, n_ad)
        launch_bytes[g_["name"]] = b
        breakdown[g_["name"]] = dict(us=round(med_ms[i] * 1e3, 2), GBps=round(b / med_ms[i] / 1e6, 1),
                                     frac=round(b / med_ms[i] / 1e6 / PEAK_HBM_GBPS, 4))
        lora_b += b
        lora_t += med_ms[i]
    db = wl.direft_algorithmic_bytes(T_act, d_res, r, n_ad)
    launch_bytes["direft"] = db
    breakdown["direft"] = dict(us=round(med_ms[-1] * 1e3, 2), GBps=round(db / med_ms[-1] / 1e6, 1),
                               frac=round(db / med_ms[-1] / 1e6 / PEAK_HBM_GBPS, 4))
    # the dominant kernel: the launch that takes the largest share of the step
    names = [g_["name"] for g_ in groups] + ["direft"]
    dom = names[int(np.argmax(med_ms))]
    achieved = launch_bytes[dom] / (breakdown[dom]["us"] * 1e-6) / 1e9
    roofline = dict(bound="hbm", kernel=f"the {dom} launch" + (" (packed: one read of x)" if "+" in dom else ""),
                    achieved=round(achieved, 1), peak=PEAK_HBM_GBPS, unit="GB/s", frac=round(achieved / PEAK_HBM_GBPS, 4),
                    traffic=None, bytes_per_launch=int(launch_bytes[dom]), us_per_launch=breakdown[dom]["us"],
                    timing="median of the timed steps, HIP events on the launch stream")
    lora_frac = round(lora_b / lora_t / 1e6 / PEAK_HBM_GBPS, 4) if projs else None

    # HBM traffic of the dominant kernel: two rocprofv3 --pmc runs of this same command, summarised under
    # profiles/.  A quoted figure, not one of this run: it is attached only while the kernel sources are
    # the ones the counters were taken from (hash recorded in the summary).
    if args.config == "llama70b_lora" and r == 64 and args.pitch == "dense" and not experiment_flags(args):
        try:
            fields = {}
            with open(os.path.join(ROOT, TRAFFIC_PROFILE)) as f:
                for line in f:
                    key = line.split("=")[0].strip()
                    if "=" in line and key in ("traffic_bytes_per_launch", "kernel_sources_sha256", "launch"):
                        fields[key] = line.split("=", 1)[1].strip()
            if fields.get("kernel_sources_sha256") == kernel_sources_sha256() and fields.get("launch") == dom:
                roofline["traffic"] = int(fields["traffic_bytes_per_launch"])
                roofline["traffic_source"] = (TRAFFIC_PROFILE + ": rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this "
                                              "command on these kernel sources (quoted, not measured in this run)")
            else:
                roofline["traffic_source"] = TRAFFIC_PROFILE + " was taken from other kernel sources: not quoted"
        except (OSError, ValueError, KeyError):
            pass

    out = {
        "metric": METRIC,
        "value": round(T_act / (ms_per_step * 1e-3), 1), "unit": "tokens/s",
        "n_gpus": 1, "steps": K, "warmup": W, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": f"{args.config}: one decoder layer's adapter work = scheduler + {len(projs)} LoRA projections "
                               f"({','.join(p['name'] for p in projs)}; launches: {','.join(g_['name'] for g_ in groups)}) "
                               f"+ DiReFT d={d_res}, rank {r}, prefill-only",
                   "T": T, "S": S, "active_rows": T_act, "decode_rows": int(T - T_act), "adapters": N,
                   "distinct_active_adapters": n_ad, "rank": r, "seed": args.seed,
                   "row_pitch": ("dense (row pitch = width)" if args.pitch == "dense" else
                                 "next power of two (rows of 14336 or 28672 elements start every 16384 or 32768; "
                                 "the padding is never touched)") + (f" + {args.ldpad}" if args.ldpad else ""),
                   "workspace_bytes": int(ws.numel()),
                   "schedule": {"chunks": counts[0], "short_rows": counts[1]}},
        "roofline": roofline,
        "pct_peak_hbm": round(100 * achieved / PEAK_HBM_GBPS, 2),
        "lora_launches_frac": lora_frac,
        "breakdown": breakdown,
    }
    # ---- practical ceiling: a plain device copy (also the known-size dispatch that calibrates the
    # HBM byte counters of the rocprofv3 --pmc runs) ----------------------------------------------
    src = wl.activations(min(T, 65536), 14336, "bf16", device=dev, seed=1)
    dst = torch.empty_like(src)
    ms = timed(lambda: dst.copy_(src), 5 if args.no_extras else 20, 2)
    out["copy_GBps"] = round(2 * src.numel() * 2 / ms / 1e6, 1)
    out["copy_bytes_each_way"] = int(src.numel() * 2)
    del dst, src
    if args.no_extras:
        return out, None

    # ---- conventional baseline and the decode-only step ----------------------------------------
    n_light = max(3, K // 4)
    ms_all = timed(lambda: step(preft.PREFT_ALL_TOKENS), n_light, 2)
    dec = tab.decode_only()
    dt = tuple(torch.from_numpy(a.copy()).to(dev) for a in (dec.seg_start, dec.seg_adapter, dec.seg_prefill_len))

    def graphed(mode):                 # one engine step as a HIP graph: no host launch gaps
        step(mode, dt, dec.T)
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            step(mode, dt, dec.T)
        return g
    g_all, g_pre = graphed(preft.PREFT_ALL_TOKENS), graphed(preft.PREFT_PREFILL_ONLY)
    ms_dec_all = timed(g_all.replay, 50, 5)
    ms_dec_pre = timed(g_pre.replay, 50, 5)
    out["all_token"] = {"ms_per_step": round(ms_all, 4), "speedup_prefill_only": round(ms_all / ms_per_step, 4)}
    if len(groups) != len(singles):
        ms_single = timed(lambda: step(preft.PREFT_PREFILL_ONLY, groups=singles), n_light, 2)
        out["one_launch_per_projection"] = {"ms_per_step": round(ms_single, 4),
                                            "speedup_packed": round(ms_single / ms_per_step, 4)}
    out["decode_only_step"] = {"rows": dec.T, "all_token_ms": round(ms_dec_all, 4),
                               "prefill_only_ms": round(ms_dec_pre, 4),
                               "speedup_prefill_only": round(ms_dec_all / ms_dec_pre, 2)}
    if args.sub:
        return out, None

    # ---- DiReFT at every layer (App. A.2): L residual streams, one call per layer or one call for all ----
    L = int(max(2, min(32, 48e9 // (T * d_res * 2))))
    hs = [h] + [h.clone() for _ in range(L - 1)]
    per_layer = [(W1p, W2tp, bp)]
    keep = []
    for _ in range(L - 1):                      # every layer has factors of its own (distinct memory)
        mats = [[m.clone() for m in group] for group in (W1, W2t, bb)]
        keep.append(mats)
        per_layer.append(tuple(preft.pointer_table(g_) for g_ in mats))
    as_table = lambda ptrs: torch.tensor(ptrs, dtype=torch.int64, device=dev)
    h_tab = preft.pointer_table(hs)
    W1s, W2s, bs = (as_table([pl[i].data_ptr() for pl in per_layer]) for i in range(3))

    def layers_step(mode, fused, tables=(ss, sa, sp), T_=T):
        s0, s1, s2 = tables
        preft.preft_schedule(ws, s0, s1, s2, T_, N, mode)
        ready = mode | preft.PREFT_SCHEDULE_READY
        if fused:
            preft.preft_direft_apply_layers([x[:T_] for x in hs], h_tab, s0, s1, s2, W1s, W2s, bs, N, r,
                                            direft_scale, ready, ws)
        else:
            for x, (a1, a2, a3) in zip(hs, per_layer):
                preft.preft_direft_apply(x[:T_], s0, s1, s2, a1, a2, a3, r, direft_scale, ready, ws)

    it = max(3, K // 10)
    ms_each = timed(lambda: layers_step(preft.PREFT_PREFILL_ONLY, False), it, 2)
    ms_one = timed(lambda: layers_step(preft.PREFT_PREFILL_ONLY, True), it, 2)

    def graphed_layers(fused):
        layers_step(preft.PREFT_ALL_TOKENS, fused, dt, dec.T)
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            layers_step(preft.PREFT_ALL_TOKENS, fused, dt, dec.T)
        return g
    ms_dec_each = timed(graphed_layers(False).replay, 50, 5)
    ms_dec_one = timed(graphed_layers(True).replay, 50, 5)
    out["direft_every_layer"] = {
        "layers": L, "rank": r, "d": d_res,
        "mixed_batch_prefill_only_ms": {"one_call_per_layer": round(ms_each, 4), "one_call": round(ms_one, 4)},
        "frac_of_peak_one_call": round(L * db / ms_one / 1e6 / PEAK_HBM_GBPS, 4),
        "decode_rows_all_token_ms": {"rows": dec.T, "one_call_per_layer": round(ms_dec_each, 4),
                                     "one_call": round(ms_dec_one, 4)}}
    del hs, keep, per_layer, h_tab

    # ---- serving-weighted comparison: first-come-first-served trace of the paper's microbenchmark --
    # (App. E.1, E.3): every engine step's adapter work, in both modes.  Decode-only steps are
    # HIP-graph replays (the paper's engine runs under graph capture too); steps that hold a
    # prompt are launched eagerly.  Only the adapter kernels run: the ratio says how the adapter
    # cost splits over a serving run, it is not an end-to-end throughput ratio.
    if not args.no_trace:
        paged = args.trace_slots > 0
        n_trace_adapters = args.trace_adapters if paged else min(args.trace_adapters, N)
        req = wl.request_stream(args.trace_requests, n_trace_adapters, args.trace_mix, l_max=2048, seed=args.seed)
        epochs = list(wl.fcfs_steps(req, args.trace_batch))
        Bmax = args.trace_batch
        mgr, trace_pools = None, None
        if paged:
            # the paper's paged setting (Sec. 4; App. E.2): the catalogue in pinned host memory, at most
            # --trace-slots adapters in device slots; a step first makes its adapters resident.  One
            # random matrix per part serves every adapter: only the traffic matters here.
            shapes = []
            for p_ in projs:
                shapes += [(r, p_["d_in"]), (p_["d_out"], r)]
            shapes += [(r, d_res), (d_res, r), (r,)]
            host = [torch.randn(sh).to(torch.bfloat16).contiguous() for sh in shapes]
            mgr = preft.preft_slots_create(n_trace_adapters, args.trace_slots, [t.numel() * 2 for t in host])
            for a_ in range(n_trace_adapters):
                for pi, t in enumerate(host):
                    preft.preft_slots_store(mgr, a_, pi, t)
            trace_pools = {p_["name"]: (preft.preft_slots_pool(mgr, 2 * i), preft.preft_slots_pool(mgr, 2 * i + 1))
                           for i, p_ in enumerate(projs)}
            nb = 2 * len(projs)
            trace_pools["direft"] = tuple(preft.preft_slots_pool(mgr, nb + j) for j in range(3))
            trace_pools["N"] = preft.preft_slots_stats(mgr)["n_slots"]
        st = [torch.zeros(Bmax + 1, dtype=torch.int32, device=dev), torch.zeros(Bmax, dtype=torch.int32, device=dev),
              torch.zeros(Bmax, dtype=torch.int32, device=dev)]

        def upload(t_):
            ids = t_.seg_adapter
            if paged:                  # adapter ids -> slot ids; missing adapters are copied in on this stream
                ids = np.asarray(preft.preft_slots_acquire(mgr, ids.tolist()), dtype=np.int32)
            st[0][:t_.S + 1].copy_(torch.from_numpy(t_.seg_start.copy()))
            st[1][:t_.S].copy_(torch.from_numpy(ids.copy()))
            st[2][:t_.S].copy_(torch.from_numpy(t_.seg_prefill_len.copy()))
            return (st[0][:t_.S + 1], st[1][:t_.S], st[2][:t_.S])

        def replay(mode):
            graphs, pairs = {}, []
            for t_, repeat in epochs:
                if t_.T > T:
                    raise RuntimeError("trace step larger than the benchmark buffers")
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                decode_only = not bool(t_.seg_prefill_len.any())
                if decode_only and t_.S not in graphs:
                    views = upload(t_)
                    step(mode, views, t_.T, pools=trace_pools)
                    torch.cuda.synchronize()
                    g = torch.cuda.CUDAGraph()
                    with torch.cuda.graph(g):
                        step(mode, views, t_.T, pools=trace_pools)
                    graphs[t_.S] = g
                e0.record()                      # the bracket holds the table upload and any adapter copies
                views = upload(t_)
                if decode_only:
                    for _ in range(repeat):
                        graphs[t_.S].replay()
                else:
                    step(mode, views, t_.T, pools=trace_pools)
                e1.record()
                pairs.append((decode_only, e0, e1))
            torch.cuda.synchronize()
            ms_dec = sum(a.elapsed_time(b) for d_, a, b in pairs if d_)
            ms_pre = sum(a.elapsed_time(b) for d_, a, b in pairs if not d_)
            return ms_pre, ms_dec

        pre_p, dec_p = replay(preft.PREFT_PREFILL_ONLY)
        pre_a, dec_a = replay(preft.PREFT_ALL_TOKENS)
        n_steps = sum(rep for _, rep in epochs)
        n_dec_steps = sum(rep for t_, rep in epochs if not t_.seg_prefill_len.any())
        out["fcfs_trace"] = {
            "shapes": f"{args.config} layer, rank {r}",
            "requests": len(req.prompt_len), "in_flight": Bmax, "mix": args.trace_mix,
            "adapters": int(n_trace_adapters), "l_max": 2048,
            "engine_steps": int(n_steps), "decode_only_steps": int(n_dec_steps),
            "prompt_rows": int(req.prompt_len.sum()), "decode_rows": int((req.output_len - 1).sum()),
            "prefill_only_ms": {"steps_with_prompts": round(pre_p, 2), "decode_only_steps": round(dec_p, 2)},
            "all_token_ms": {"steps_with_prompts": round(pre_a, 2), "decode_only_steps": round(dec_a, 2)},
            "adapter_time_ratio_all_token_over_prefill_only": round((pre_a + dec_a) / (pre_p + dec_p), 2),
            "same_ratio_if_the_caller_skips_decode_only_steps": round((pre_a + dec_a) / pre_p, 2),
            "us_per_decode_only_step": {"all_token": round(dec_a / max(n_dec_steps, 1) * 1e3, 2),
                                        "prefill_only": round(dec_p / max(n_dec_steps, 1) * 1e3, 2)},
        }
        if paged:
            torch.cuda.synchronize()
            stats = preft.preft_slots_stats(mgr)           # both replays together
            out["fcfs_trace"]["slot_manager"] = {"device_slots": stats["n_slots"], "hits": stats["hits"],
                                                 "misses": stats["misses"], "evictions": stats["evictions"],
                                                 "MB_copied": round(stats["bytes_copied"] / 1e6, 1)}
            preft.preft_slots_destroy(mgr)

    # ---- CPU oracle on a deterministic row sample of the same batch ---------------------------
    # every prompt's first and last row and --cpu-rows-per-segment random rows of it (decode rows are
    # not active in prefill-only mode); the sampled rows go through the whole step on the host cores
    cpu_job = None
    if not args.no_cpu_baseline:
        rows = wl.sample_rows(tab, args.cpu_rows_per_segment, seed=args.seed)
        owner = np.repeat(np.arange(S), tab.seg_len)
        rel = rows - tab.seg_start[owner[rows]]
        rows = rows[(rel < tab.seg_prefill_len[owner[rows]]) & (tab.seg_adapter[owner[rows]] >= 0)]   # active ones
        idx = torch.from_numpy(rows).to(dev)
        used = set(int(a) for a in np.unique(tab.seg_adapter[owner[rows]]))
        pick = lambda mats: [mats[j].cpu() if j in used else None for j in range(N)]
        cpu_job = dict(rows=rows,
                       lora=[(p["x"][idx].cpu(), p["y"][idx].cpu(), pick(p["pool"].A), pick(p["pool"].B)) for p in projs],
                       h=h[idx].cpu(), dA=pick(dpool.A), dB=pick(dpool.B), db=pick(dpool.b))

        cpu_job.update(tab=tab, r=r, scale=scale, direft_scale=direft_scale, T_act=T_act, n_projs=len(projs),
                       per_segment=args.cpu_rows_per_segment)
    return out, cpu_job


def cpu_baseline(job):
    """The fp64 oracle, as it stands, on the sampled rows: the whole step on the host cores."""
    from oracle import preft_oracle as ora
    tab, r = job["tab"], job["r"]
    t0 = time.perf_counter()
    for (x_c, y_c, A_c, B_c) in job["lora"]:
        ora.lora(y_c, x_c, tab.seg_start, tab.seg_adapter, tab.seg_prefill_len, A_c, B_c, r, job["scale"], ora.PROMPT_ONLY,
                 rows=job["rows"], gathered=True)
    ora.direft(job["h"], tab.seg_start, tab.seg_adapter, tab.seg_prefill_len, job["dA"], job["dB"], job["db"], r,
               job["direft_scale"], ora.PROMPT_ONLY, rows=job["rows"], gathered=True)
    dt_cpu = time.perf_counter() - t0
    n_rows = len(job["rows"])
    return {"value": round(n_rows / dt_cpu, 1), "unit": "tokens/s", "cores": ora.threads(), "kind": "oracle",
            "sample": f"sampled: {n_rows} of the {job['T_act']} active rows (first and last row of every prompt + "
                      f"{job['per_segment']} random rows per prompt), full step ({job['n_projs']} LoRA projections + "
                      f"DiReFT, rank {r}), fp64 loops, {dt_cpu:.1f} s wall; value = sampled rows per second"}


def child(argv, timeout=900):
    """The same measurement in a fresh process; returns its JSON line reduced to the figures quoted."""
    cmd = [sys.executable, os.path.abspath(__file__), "--sub", "--no-cpu-baseline"] + argv
    try:
        res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.DEVNULL, text=True, timeout=timeout)
    except subprocess.TimeoutExpired:
        return {"error": "child timed out"}
    lines = [l for l in res.stdout.splitlines() if l.startswith("{")]
    if res.returncode != 0 or not lines:
        return {"error": f"child exited with {res.returncode}"}
    d_ = json.loads(lines[-1])
    rec = {"workload": d_["config"]["workload"].split(":")[0], "rank": d_["config"]["rank"],
           "active_rows": d_["config"]["active_rows"], "row_pitch": d_["config"]["row_pitch"].split(" (")[0],
           "value": d_["value"], "ms_per_step": d_["ms_per_step"], "steps": d_["steps"],
           "dominant_launch": d_["roofline"]["kernel"], "roofline_frac": d_["roofline"]["frac"],
           "lora_launches_frac": d_["lora_launches_frac"],
           "frac_per_launch": {k_: v_["frac"] for k_, v_ in d_["breakdown"].items()},
           "us_per_launch": {k_: v_["us"] for k_, v_ in d_["breakdown"].items()}}
    if "all_token" in d_:
        rec["all_token_ms_per_step"] = d_["all_token"]["ms_per_step"]
        rec["decode_only_step"] = d_["decode_only_step"]
    return rec


def main():
    args = parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build measures one GPU only (the path has no cross-GPU step); run with --gpus 1",
              file=sys.stderr)
        sys.exit(2)
    out, cpu_job = run(args)
    # run() has returned: its buffers are released, the GPU is free for the child processes below
    if cpu_job is not None:
        import gc
        import torch
        gc.collect()
        torch.cuda.empty_cache()
        out["cpu_baseline"] = cpu_baseline(cpu_job)

    # ---- the other configurations, ranks and row pitch: the same measurement in a child process each ----
    if not (args.sub or args.no_extras or args.no_children or experiment_flags(args)):
        from paper_2605_14217_amd import workloads as wl
        K = args.steps
        others = {}
        for cfg_name in ("llama8b_lora", "llama8b_direft", "skewed70b"):
            if cfg_name == args.config:
                continue
            steps = K if cfg_name.startswith("llama8b") else max(5, K // 4)
            others[cfg_name] = child(["--config", cfg_name, "--seed", str(args.seed), "--steps", str(steps), "--warmup", "3",
                                      "--pitch", args.pitch])
        out["other_configurations"] = others
        r_main = args.rank or DEFAULT_RANK[args.config]
        ranks = {}
        for rk in wl.CONFIGS[args.config]["ranks"]:
            if rk != r_main:
                ranks[str(rk)] = child(["--config", args.config, "--rank", str(rk), "--seed", str(args.seed), "--steps",
                                        str(max(5, K // 4)), "--warmup", "2", "--pitch", args.pitch])
        if ranks:
            out["other_ranks"] = ranks
        other_pitch = "pow2" if args.pitch == "dense" else "dense"
        out["pow2_row_pitch" if other_pitch == "pow2" else "dense_rows"] = child(
            ["--config", args.config, "--rank", str(r_main), "--seed", str(args.seed), "--steps", str(max(5, K // 4)),
             "--warmup", "2", "--pitch", other_pitch])
    print(json.dumps(out))


if __name__ == "__main__":
    main()
