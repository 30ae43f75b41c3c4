#!/usr/bin/env python3
"""Benchmark of the prefill-only adapter-apply hot path on one MI355X.

A "step" is one pass of the whole path over one synthetic batch of the Llama-3.1-8B LoRA
configuration (32 prompts of U[256,2048] rows + 224 decode rows, 64 adapters, bf16):

    1 x token-segment scheduler                              (preft_schedule)
    7 x segmented multi-adapter LoRA, rank R, prefill-only   (q, k, v, o, gate, up, down)
    1 x segmented multi-adapter DiReFT, rank R, prefill-only (residual stream d = 4096)

i.e. the adapter work of one decoder layer on that batch.  Every projection has its own
activation buffers (about 6 GB per step in total), so every launch streams cold data from HBM;
adapter weights are warm (steady-state serving).  `value` = active (prefill) rows per second
through the step.

The same JSON line also carries: the HBM roofline of the dominant kernel (the LoRA tile kernel,
timed per launch with HIP events on the launch stream inside the timed region), the all-token
(conventional PEFT) time for the same batch, the batch's decode rows alone as a decode-only
step in both modes, and the CPU oracle timed on a sample of the same batch.
"""
import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_HBM_GBPS = 8000.0      # MI355X HBM3E, published


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--rank", type=int, default=16, help="adapter rank (the configuration lists 1, 8, 16)")
    ap.add_argument("--config", default="llama8b_lora")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true", help="skip the all-token / decode-only legs")
    ap.add_argument("--variant", type=int, default=0)
    ap.add_argument("--waves", type=int, default=0)
    ap.add_argument("--rowblocks", type=int, default=0)
    ap.add_argument("--colsplit", type=int, default=0, help="workgroups per tile on small batches (0: automatic)")
    ap.add_argument("--ldpad", type=int, default=0, help="experiment: extra elements of row stride on every buffer")
    ap.add_argument("--pitch", choices=["dense", "pow2"], default="pow2",
                    help="row pitch of the activation buffers: the next power of two (default: 14336-wide rows "
                         "every 16384 elements, measured 7-10 %% faster on MI355X) or their width")
    ap.add_argument("--only", default="", help="experiment: comma-separated subset of projections")
    ap.add_argument("--no-packed", action="store_true",
                    help="one launch per projection instead of packed q,k,v and gate,up launches")
    ap.add_argument("--no-trace", action="store_true", help="skip the serving-trace replay leg")
    ap.add_argument("--no-other-ranks", action="store_true",
                    help="skip the short runs at the configuration's other ranks")
    ap.add_argument("--trace-requests", type=int, default=1000)
    ap.add_argument("--trace-batch", type=int, default=32)
    ap.add_argument("--trace-adapters", type=int, default=32)
    ap.add_argument("--trace-mix", default="uniform", choices=["identical", "uniform", "skewed", "distinct"])
    ap.add_argument("--trace-slots", type=int, default=0,
                    help="serve the trace through the adapter slot manager with this many device slots "
                         "(0: every adapter resident); --trace-adapters may then exceed the configuration's pool")
    args = ap.parse_args()

    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build measures one GPU only (the path has no cross-GPU step); run with --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import paper_2605_14217_amd as preft
    from paper_2605_14217_amd import workloads as wl

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    preft.load_library()
    preft.set_test_flags(preft.test_flags(variant=args.variant, waves=args.waves, rowblocks=args.rowblocks,
                                          colsplit=args.colsplit))
    dev = "cuda:0"
    torch.cuda.set_device(0)

    cfg = wl.CONFIGS[args.config]
    N, r, d_res = cfg["N"], args.rank, cfg["direft_d"]
    scale = cfg["lora_scale"]
    tab = wl.make_segments(args.config, seed=args.seed)
    T, S = tab.T, tab.S
    T_act = tab.active_rows(False, N)
    n_ad = tab.distinct_active_adapters(False, N)
    ss, sa, sp = (torch.from_numpy(a.copy()).to(dev) for a in (tab.seg_start, tab.seg_adapter, tab.seg_prefill_len))
    ws = preft.new_workspace(T, S, device=dev)

    # ---- buffers and pools --------------------------------------------------------------
    projs = []
    def act(T_, d_, seed_):
        t = wl.activations(T_, d_, "bf16", device=dev, seed=seed_)
        pitch = d_ + args.ldpad
        if args.pitch == "pow2":                       # row pitch = next power of two (a caller's layout choice)
            pitch = 1 << (d_ - 1).bit_length()
        if pitch != d_:
            buf = torch.empty((T_, pitch), dtype=t.dtype, device=dev)
            buf[:, :d_].copy_(t)
            return buf[:, :d_]
        return t

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
    # (the library fuses such a call into one launch for rank 1-4, 8, 12, 16; other ranks stay one
    # call and one launch per projection, accounted per projection)
    packs = {"q": "qkv", "k": "qkv", "v": "qkv", "gate": "gate_up", "up": "gate_up"}
    packed = not args.no_packed and (r <= 3 or (r % 4 == 0 and r <= 16))
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

    per_launch_ms = np.array([[a.elapsed_time(b) for (a, b) in evk] for evk in ev])     # [K, 8]
    mean_ms = per_launch_ms.mean(axis=0)
    breakdown = {}
    lora_b, lora_t = 0.0, 0.0
    for i, g_ in enumerate(groups):
        m = g_["members"]
        # x once per launch, every output read and written once, every distinct adapter's factors once
        b = wl.lora_algorithmic_bytes(T_act, m[0]["d_in"], [q["d_out"] for q in m], r, n_ad)
        breakdown[g_["name"]] = dict(us=round(mean_ms[i] * 1e3, 2), GBps=round(b / mean_ms[i] / 1e6, 1),
                                     frac=round(b / mean_ms[i] / 1e6 / PEAK_HBM_GBPS, 4))
        lora_b += b
        lora_t += mean_ms[i]
    db = wl.direft_algorithmic_bytes(T_act, d_res, r, n_ad)
    breakdown["direft"] = dict(us=round(mean_ms[-1] * 1e3, 2), GBps=round(db / mean_ms[-1] / 1e6, 1),
                               frac=round(db / mean_ms[-1] / 1e6 / PEAK_HBM_GBPS, 4))
    if projs:
        achieved = lora_b / lora_t / 1e6                                                 # GB/s
        roofline = dict(bound="hbm", kernel=f"lora tile kernel ({len(groups)} launches per step: "
                                            + ",".join(g_["name"] for g_ in groups) + ")",
                        achieved=round(achieved, 1), peak=PEAK_HBM_GBPS, unit="GB/s",
                        frac=round(achieved / PEAK_HBM_GBPS, 4), traffic=None,
                        bytes_per_launch=int(lora_b / len(groups)), us_per_launch=round(lora_t / len(groups) * 1e3, 2))
    else:
        achieved = db / mean_ms[-1] / 1e6
        roofline = dict(bound="hbm", kernel="direft tile kernel (1 launch per step)",
                        achieved=round(achieved, 1), peak=PEAK_HBM_GBPS, unit="GB/s",
                        frac=round(achieved / PEAK_HBM_GBPS, 4), traffic=None,
                        bytes_per_launch=int(db), us_per_launch=round(mean_ms[-1] * 1e3, 2))

    # HBM traffic of the dominant kernel comes from two rocprofv3 --pmc runs of this same command;
    # their summary is committed under profiles/ and quoted here when the configuration matches.
    if projs and args.config == "llama8b_lora" and r == 16 and args.pitch == "pow2" and not (
            args.variant or args.waves or args.rowblocks or args.ldpad or args.only or not packed):
        try:
            with open(os.path.join(ROOT, "profiles", "lora_tile_kernel_llama8b_rank16_hbm_traffic.txt")) as f:
                for line in f:
                    if line.startswith("traffic_bytes_per_launch"):
                        roofline["traffic"] = int(line.split("=")[1])
        except OSError:
            pass

    out = {
        "metric": "prefill tokens/s through multi-adapter LoRA/DiReFT apply; % of peak HBM GB/s",
        "value": round(T_act / (ms_per_step * 1e-3), 1), "unit": "tokens/s",
        "n_gpus": 1, "steps": K, "warmup": W, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": f"{args.config}: one decoder layer's adapter work = scheduler + {len(projs)} LoRA projections "
                               f"({','.join(p['name'] for p in projs)}; launches: {','.join(g_['name'] for g_ in groups)}) "
                               f"+ DiReFT d={d_res}, rank {r}, prefill-only",
                   "T": T, "S": S, "active_rows": T_act, "decode_rows": int(T - T_act), "adapters": N,
                   "distinct_active_adapters": n_ad, "rank": r, "seed": args.seed,
                   "row_pitch": ("next power of two (rows of 14336 or 28672 elements start every 16384 or 32768; "
                                 "the padding is never touched)" if args.pitch == "pow2" else "dense")
                                + (f" + {args.ldpad}" if args.ldpad else ""),
                   "schedule": {"chunks": counts[0], "short_rows": counts[1]}},
        "roofline": roofline,
        "pct_peak_hbm": round(100 * achieved / PEAK_HBM_GBPS, 2),
        "breakdown": breakdown,
    }

    # ---- practical ceiling: a plain device copy ------------------------------------------------
    src = wl.activations(T, 14336, "bf16", device=dev, seed=1)
    dst = torch.empty_like(src)
    ms = timed(lambda: dst.copy_(src), 20, 3)
    out["copy_GBps"] = round(2 * src.numel() * 2 / ms / 1e6, 1)
    out["copy_bytes_each_way"] = int(src.numel() * 2)       # known size: calibrates the HBM byte counters
    del dst

    # ---- conventional baseline and the decode-only step ----------------------------------------
    if not args.no_extras:
        ms_all = timed(lambda: step(preft.PREFT_ALL_TOKENS), max(5, K // 4), 3)
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
            ms_single = timed(lambda: step(preft.PREFT_PREFILL_ONLY, groups=singles), max(5, K // 4), 3)
            out["one_launch_per_projection"] = {"ms_per_step": round(ms_single, 4),
                                                "speedup_packed": round(ms_single / ms_per_step, 4)}
        out["decode_only_step"] = {"rows": dec.T, "all_token_ms": round(ms_dec_all, 4),
                                   "prefill_only_ms": round(ms_dec_pre, 4),
                                   "speedup_prefill_only": round(ms_dec_all / ms_dec_pre, 2)}

    # ---- DiReFT at every layer (App. A.2): L residual streams, one call per layer or one call for all ----
    if not args.no_extras:
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
        dec = tab.decode_only()
        dt = tuple(torch.from_numpy(a.copy()).to(dev) for a in (dec.seg_start, dec.seg_adapter, dec.seg_prefill_len))

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
        del hs, keep, per_layer

    # ---- the configuration's other ranks: the same measurement in a child process each ----------
    if not (args.no_extras or args.no_other_ranks or args.variant or args.waves or args.rowblocks or args.colsplit
            or args.ldpad or args.only or args.no_packed):
        import subprocess

        def child(rk, pitch):
            cmd = [sys.executable, os.path.abspath(__file__), "--config", args.config, "--rank", str(rk), "--seed",
                   str(args.seed), "--steps", str(max(5, K // 4)), "--warmup", "3", "--no-extras", "--no-cpu-baseline",
                   "--pitch", pitch]
            res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.DEVNULL, text=True, timeout=600)
            lines = [l for l in res.stdout.splitlines() if l.startswith("{")]
            if res.returncode != 0 or not lines:
                return {"error": f"child exited with {res.returncode}"}
            d_ = json.loads(lines[-1])
            return {"value": d_["value"], "ms_per_step": d_["ms_per_step"], "roofline_frac": d_["roofline"]["frac"],
                    "frac_per_launch": {k_: v_["frac"] for k_, v_ in d_["breakdown"].items()}}

        others = {}
        for rk in cfg["ranks"]:
            if rk == r:
                continue
            others[str(rk)] = child(rk, args.pitch)
        if others:
            out["other_ranks"] = others
        if args.pitch != "dense":          # the same step with every buffer's rows packed densely
            out["dense_rows"] = child(r, "dense")

    # ---- serving-weighted comparison: first-come-first-served trace of the paper's microbenchmark --
    # (App. E.1, E.3): every engine step's adapter work, in both modes.  Decode-only steps are
    # HIP-graph replays (the paper's engine runs under graph capture too); steps that hold a
    # prompt are launched eagerly.  Only the adapter kernels run: the ratio says how the adapter
    # cost splits over a serving run, it is not an end-to-end throughput ratio.
    if not args.no_trace and not args.no_extras:
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

    # ---- CPU oracle on a sample of the same batch ---------------------------------------------
    if not args.no_cpu_baseline:
        from oracle import preft_oracle as ora
        budget_rows = 1 << 30          # the whole batch: a few seconds on the machine's cores
        keep, rows_kept = [], 0
        for s in np.argsort(-tab.seg_prefill_len, kind="stable"):
            if tab.seg_prefill_len[s] == 0 or rows_kept >= budget_rows:
                break
            keep.append(int(s))
            rows_kept += int(tab.seg_len[s])
        keep = sorted(keep)
        sub = wl.from_lengths(tab.seg_len[keep], tab.seg_adapter[keep], tab.seg_prefill_len[keep])
        idx = torch.from_numpy(np.concatenate([np.arange(tab.seg_start[s], tab.seg_start[s + 1]) for s in keep])).to(dev)
        used = set(int(a) for a in sub.seg_adapter)
        cpu_in = []
        for p in projs:
            cpu_in.append((p["x"][idx].cpu(), p["y"][idx].cpu(),
                           [p["pool"].A[j].cpu() if j in used else None for j in range(N)],
                           [p["pool"].B[j].cpu() if j in used else None for j in range(N)]))
        h_cpu = h[idx].cpu()
        dA = [dpool.A[j].cpu() if j in used else None for j in range(N)]
        dB = [dpool.B[j].cpu() if j in used else None for j in range(N)]
        db_ = [dpool.b[j].cpu() if j in used else None for j in range(N)]
        t0 = time.perf_counter()
        for (x_c, y_c, A_c, B_c) in cpu_in:
            ora.lora(y_c, x_c, sub.seg_start, sub.seg_adapter, sub.seg_prefill_len, A_c, B_c, r, scale, ora.PROMPT_ONLY)
        ora.direft(h_cpu, sub.seg_start, sub.seg_adapter, sub.seg_prefill_len, dA, dB, db_, r, direft_scale,
                   ora.PROMPT_ONLY)
        dt_cpu = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": round(sub.T / dt_cpu, 1), "unit": "tokens/s", "cores": ora.threads(),
                               "kind": "oracle",
                               "sample": f"{len(keep)} prompts of the batch ({sub.T} of {T_act} active rows), full step "
                                         f"({len(projs)} LoRA projections + DiReFT), fp64 loops, {dt_cpu:.1f} s wall"}

    print(json.dumps(out))


if __name__ == "__main__":
    main()
