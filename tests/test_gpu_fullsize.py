"""Full-size parity: the named configurations at their real shapes, in the launch configuration
bench.py times (automatic kernel choice), checked on sampled rows the oracle computes one by one
(every segment's first/last row and both sides of its prompt boundary, random rows, decode rows)
plus a bitwise check of *all* inactive rows."""
import gc

import numpy as np
import pytest
import torch

import paper_2605_14217_amd as preft
from paper_2605_14217_amd import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(autouse=True)
def _reset(request):
    print(f"\n[case] {request.node.name}", flush=True)
    preft.set_test_flags(0)
    yield
    gc.collect()
    torch.cuda.empty_cache()


# rows start every next-power-of-two elements (the layout bench.py times) unless the case says "dense"
LORA = [
    ("llama8b_lora", "q", 16, False), ("llama8b_lora", "q", 16, True), ("llama8b_lora", "down", 8, False),
    ("llama8b_lora", "k", 1, False), ("llama8b_lora", "gate", 16, False),
    ("llama70b_lora", "q", 64, False), ("llama70b_lora", "q", 64, True), ("llama70b_lora", "gate", 16, False),
    ("llama70b_lora", "down", 1, False), ("llama70b_lora", "k", 16, True),
    ("skewed70b", "res", 32, False), ("skewed70b", "res", 32, True),
    ("llama8b_lora", "gate", 16, False, "dense"), ("llama8b_lora", "down", 16, False, "dense"),
    ("llama8b_lora", "o", 16, True, "dense"), ("llama8b_lora", "v", 8, False, "dense"),
    ("llama70b_lora", "down", 64, False, "dense"), ("llama70b_lora", "o", 64, False, "dense"),
    ("llama70b_lora", "gate", 64, True, "dense"), ("llama70b_lora", "o", 32, False, "dense"),
    ("skewed70b", "res", 32, False, "dense"),
    # a workspace with room for z: on a batch of this size the call runs its sweeps as two launches
    ("llama8b_lora", "gate", 64, False, "dense", "z"), ("llama8b_lora", "o", 32, True, "dense", "z"),
    ("llama8b_lora", "down", 48, False, "dense", "z"),
    # ... and on the larger batches as one, whatever the workspace
    ("llama70b_lora", "down", 64, False, "dense", "z"),
]


def _pow2_pad(width):
    """Guard columns that bring a row to the next power of two: the row pitch bench.py uses by default."""
    return (1 << (width - 1).bit_length()) - width


@pytest.mark.parametrize("case", LORA, ids=["-".join([c[0], c[1], f"r{c[2]}", "all" if c[3] else "prefill", *c[4:]])
                                            for c in LORA])
def test_fullsize_lora(case):
    from parity_util import run_lora_case
    config, proj, rank, all_tokens = case[:4]
    dense = len(case) > 4
    cfg = wl.CONFIGS[config]
    d_in, d_out = cfg["lora_shapes"][proj]
    tab = wl.make_segments(config, seed=0)
    pool = wl.lora_pool(cfg["N"], rank, d_in, d_out, "bf16", device="cuda", seed=5)
    x = wl.activations(tab.T, d_in, "bf16", device="cuda", seed=51)
    y0 = wl.activations(tab.T, d_out, "bf16", device="cuda", seed=52)
    # the 8B LoRA batch is compared whole (every row); the larger batches on a deterministic row sample
    rows = None if config == "llama8b_lora" else wl.sample_rows(tab, 2, max_rows=1200)
    worst, counts = run_lora_case(tab, pool, x, y0, "bf16", cfg["lora_scale"], all_tokens, rows=rows,
                                  pad_x=0 if dense else _pow2_pad(d_in), pad_y=0 if dense else _pow2_pad(d_out),
                                  z_room=len(case) > 5)
    print(f"  T={tab.T} S={tab.S} rows checked={tab.T if rows is None else len(rows)} worst {worst:.2e} counts {counts}")


# (config, rank, all positions, prefactor: "1" = Eq. 3 as printed, "rsqrt" = 1 / sqrt(rank) of App. C.2)
DIREFT = [("llama8b_direft", 8, False, "1"), ("llama8b_direft", 8, True, "rsqrt"), ("llama8b_direft", 16, False, "1"),
          ("llama8b_direft", 16, True, "rsqrt"), ("llama8b_direft", 16, False, "rsqrt"), ("llama8b_direft", 8, False, "rsqrt"),
          ("skewed70b", 32, False, "rsqrt"), ("skewed70b", 32, True, "1"),
          ("llama70b_lora", 64, False, "rsqrt"), ("llama70b_lora", 16, True, "1"), ("tiny", 4, False, "rsqrt")]


@pytest.mark.parametrize("config,rank,all_tokens,prefactor", DIREFT,
                         ids=[f"{c}-r{r}-{'all' if a else 'prefill'}-s{p}" for c, r, a, p in DIREFT])
def test_fullsize_direft(config, rank, all_tokens, prefactor):
    from parity_util import run_direft_case
    cfg = wl.CONFIGS[config]
    d = cfg["direft_d"]
    dtype = cfg["dtype"]
    tab = wl.make_segments(config, seed=0)
    pool = wl.direft_pool(cfg["N"], rank, d, dtype, device="cuda", seed=6)
    h = wl.activations(tab.T, d, dtype, device="cuda", seed=61)
    # the 8B DiReFT batch at rank 16 in prefill-only mode is compared whole; the others on a row sample
    whole = config in ("tiny",) or (config == "llama8b_direft" and rank == 16 and not all_tokens)
    rows = None if whole else wl.sample_rows(tab, 2, max_rows=1200)
    scale = 1.0 if prefactor == "1" else 1.0 / np.sqrt(rank)
    worst, counts = run_direft_case(tab, pool, h, dtype, scale, all_tokens, rows=rows)
    print(f"  T={tab.T} S={tab.S} rows checked={tab.T if rows is None else len(rows)} scale={scale:.4f} worst {worst:.2e} counts {counts}")


PACKED = [("llama8b_lora", ("q", "k", "v"), 16, False), ("llama8b_lora", ("gate", "up"), 16, False),
          ("llama8b_lora", ("q", "k", "v"), 1, True), ("llama70b_lora", ("q", "k", "v"), 16, True),
          ("llama70b_lora", ("gate", "up"), 1, False),
          # the packed launches of the row-split kernel (rank 32 and 64), on dense rows as bench.py times them
          ("llama70b_lora", ("q", "k", "v"), 64, False, "dense"), ("llama70b_lora", ("gate", "up"), 64, False, "dense"),
          ("llama70b_lora", ("q", "k", "v"), 32, True, "dense"), ("llama70b_lora", ("gate", "up"), 64, True),
          # a workspace with room for z: two launches on a batch of this size
          ("llama8b_lora", ("q", "k", "v"), 64, False, "dense", "z"), ("llama8b_lora", ("gate", "up"), 32, True, "dense", "z")]


@pytest.mark.parametrize("case", PACKED,
                         ids=["-".join([c[0], "+".join(c[1]), f"r{c[2]}", "all" if c[3] else "prefill", *c[4:]]) for c in PACKED])
def test_fullsize_packed_lora(case):
    """The packed launches of the benchmark step (q+k+v, gate+up), at full size, on sampled rows."""
    from oracle import preft_oracle as ora
    from parity_util import compare, dev_tables, lora_pools_to_device
    config, projs, rank, all_tokens = case[:4]
    dense = len(case) > 4
    cfg = wl.CONFIGS[config]
    N = cfg["N"]
    shapes = [cfg["lora_shapes"][p] for p in projs]
    d_in = shapes[0][0]
    assert all(s[0] == d_in for s in shapes)
    tab = wl.make_segments(config, seed=0)
    x = wl.activations(tab.T, d_in, "bf16", device="cuda", seed=71)
    pools = [wl.lora_pool(N, rank, d_in, n, "bf16", device="cuda", seed=72 + i) for i, (_, n) in enumerate(shapes)]
    from parity_util import check_guards, padded
    y0s = [wl.activations(tab.T, n, "bf16", device="cuda", seed=80 + i) for i, (_, n) in enumerate(shapes)]
    bufs = [padded(y, 0 if dense else _pow2_pad(y.shape[1]), 7.0) for y in y0s]   # dense rows, or rows every next power of two
    ys = [b[1] for b in bufs]
    tables = [lora_pools_to_device(pl) for pl in pools]
    ss, sa, sp = dev_tables(tab)
    ws = preft.new_workspace(tab.T, tab.S, z_rank=rank if len(case) > 5 else 0, z_proj=len(projs))
    mode = preft.PREFT_ALL_TOKENS if all_tokens else preft.PREFT_PREFILL_ONLY
    preft.preft_lora_apply_packed(ys, x, ss, sa, sp, [t[0] for t in tables], [t[1] for t in tables], rank,
                                  cfg["lora_scale"], mode, ws)
    torch.cuda.synchronize()
    rows = wl.sample_rows(tab, 2, max_rows=1200)
    idx = torch.from_numpy(np.asarray(rows)).to("cuda")
    pos = ora.ALL_POSITIONS if all_tokens else ora.PROMPT_ONLY
    owner = ora.positions(tab.T, tab.seg_start, tab.seg_adapter, tab.seg_prefill_len, N, pos)
    needed = set(np.unique(owner[rows][owner[rows] >= 0]).tolist())
    x_rows = x[idx].cpu()
    worst = 0.0
    for i, pl in enumerate(pools):
        A = [pl.A[j].cpu() if j in needed else None for j in range(N)]
        B = [pl.B[j].cpu() if j in needed else None for j in range(N)]
        want = ora.lora(y0s[i][idx].cpu(), x_rows, tab.seg_start, tab.seg_adapter, tab.seg_prefill_len, A, B, rank,
                        cfg["lora_scale"], pos, rows=rows, gathered=True)
        worst = max(worst, compare(ys[i], y0s[i], want, owner, "bf16", rows=rows))
        check_guards(bufs[i][0], tab.T, y0s[i].shape[1], 7.0)
    print(f"  T={tab.T} S={tab.S} rows checked={len(rows)} outputs={len(projs)} worst {worst:.2e}")


LAYERS = [("llama8b_direft", 16, 4, False), ("llama8b_lora", 8, 3, True), ("skewed70b", 32, 2, False)]


@pytest.mark.parametrize("config,rank,layers,all_tokens", LAYERS,
                         ids=[f"{c}-r{r}-L{n}-{'all' if a else 'prefill'}" for c, r, n, a in LAYERS])
def test_fullsize_direft_layers(config, rank, layers, all_tokens):
    """DiReFT on several layers' residual streams in one launch, as the benchmark's every-layer leg
    issues it: every layer on sampled rows against the oracle, all inactive rows bit for bit."""
    from oracle import preft_oracle as ora
    from parity_util import compare, dev_tables, direft_pools_to_device
    cfg = wl.CONFIGS[config]
    N, d = cfg["N"], cfg["direft_d"]
    tab = wl.make_segments(config, seed=0)
    pools = [wl.direft_pool(N, rank, d, "bf16", device="cuda", seed=400 + l) for l in range(layers)]
    dev = [direft_pools_to_device(pl) for pl in pools]
    h0s = [wl.activations(tab.T, d, "bf16", device="cuda", seed=410 + l) for l in range(layers)]
    hs = [h.clone() for h in h0s]
    table = lambda ptrs: torch.tensor(ptrs, dtype=torch.int64, device="cuda")
    ss, sa, sp = dev_tables(tab)
    ws = preft.new_workspace(tab.T, tab.S)
    mode = preft.PREFT_ALL_TOKENS if all_tokens else preft.PREFT_PREFILL_ONLY
    scale = 1.0 / np.sqrt(rank)
    preft.preft_direft_apply_layers(hs, preft.pointer_table(hs), ss, sa, sp, table([m[0].data_ptr() for m in dev]),
                                    table([m[1].data_ptr() for m in dev]), table([m[2].data_ptr() for m in dev]),
                                    N, rank, scale, mode, ws)
    torch.cuda.synchronize()
    rows = wl.sample_rows(tab, 2, max_rows=800)
    idx = torch.from_numpy(np.asarray(rows)).to("cuda")
    pos = ora.ALL_POSITIONS if all_tokens else ora.PROMPT_ONLY
    owner = ora.positions(tab.T, tab.seg_start, tab.seg_adapter, tab.seg_prefill_len, N, pos)
    needed = set(np.unique(owner[rows][owner[rows] >= 0]).tolist())
    worst = 0.0
    for l, pl in enumerate(pools):
        pick = lambda mats: [mats[j].cpu() if j in needed else None for j in range(N)]
        want = ora.direft(h0s[l][idx].cpu(), tab.seg_start, tab.seg_adapter, tab.seg_prefill_len, pick(pl.A), pick(pl.B),
                          pick(pl.b), rank, scale, pos, rows=rows, gathered=True)
        worst = max(worst, compare(hs[l], h0s[l], want, owner, "bf16", rows=rows))
    print(f"  T={tab.T} layers={layers} rows checked={len(rows)} worst {worst:.2e}")

