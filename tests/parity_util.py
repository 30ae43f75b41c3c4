"""Shared plumbing of the GPU parity tests: run the HIP path through the C ABI binding, run
the CPU oracle on the very same tensors, compare.

Bar (stated here once, used by every parity test):
  * rows outside the position set: bit-identical to the input (compared on the raw bits);
  * active rows, primary figure: row-wise max-norm relative error  max_t |g_t - o_t|_inf / |o_t|_inf
    <= 1e-2 for bf16 storage with fp32 accumulation, <= 1e-5 for fp32;
  * active rows, secondary figure: elementwise  |g - o| / max(|o|, 1e-3 |o_t|_inf)  (a plain
    elementwise relative error is ill-posed where y + delta cancels to about zero, hence the floor
    at a thousandth of the row's largest element).  Computed and printed by every comparison; for
    bf16 it is asserted <= 1e-2 as well: an element's error is one rounding of the result (<= 2^-9
    of itself) plus fp32 accumulation error of the order 1e-6 of the row scale, i.e. at most about
    1e-3 of the floor.  For fp32 the primary bound implies <= 1e-5 / 1e-3 = 1e-2, which is what is
    asserted;
  * padding beyond the row width (ld > width) and guard rows around the buffer: untouched.
"""
from __future__ import annotations

import numpy as np
import torch

import paper_2605_14217_amd as preft
from oracle import preft_oracle as ora
from paper_2605_14217_amd import workloads as wl

TOL = {"bf16": 1e-2, "f32": 1e-5}
TOL_ELEMENTWISE = {"bf16": 1e-2, "f32": 1e-2}     # secondary figure, see above
FLOOR = 1e-3
GUARD_ROWS = 3
last_secondary = 0.0                               # secondary figure of the latest compare() call


def dev_tables(tab: wl.SegmentTable, device="cuda"):
    return (torch.from_numpy(tab.seg_start.copy()).to(device),
            torch.from_numpy(tab.seg_adapter.copy()).to(device),
            torch.from_numpy(tab.seg_prefill_len.copy()).to(device))


def padded(t: torch.Tensor, pad_cols: int, sentinel: float):
    """Copy of t inside a larger buffer: GUARD_ROWS sentinel rows above and below, pad_cols
    sentinel columns to the right.  Returns (buffer, view)."""
    T, d = t.shape
    buf = torch.full((T + 2 * GUARD_ROWS, d + pad_cols), sentinel, dtype=t.dtype, device=t.device)
    view = buf[GUARD_ROWS:GUARD_ROWS + T, :d]
    view.copy_(t)
    return buf, view


def bits(t: torch.Tensor) -> torch.Tensor:
    return t.contiguous().view(torch.int16 if t.dtype == torch.bfloat16 else torch.int32)


def check_guards(buf: torch.Tensor, T: int, d: int, sentinel: float):
    ref = torch.full_like(buf, sentinel)
    assert torch.equal(bits(buf[:GUARD_ROWS]), bits(ref[:GUARD_ROWS])), "guard rows above were written"
    assert torch.equal(bits(buf[GUARD_ROWS + T:]), bits(ref[GUARD_ROWS + T:])), "guard rows below were written"
    if buf.shape[1] > d:
        assert torch.equal(bits(buf[:, d:]), bits(ref[:, d:])), "row padding was written"


def compare(got: torch.Tensor, before: torch.Tensor, want64: np.ndarray, row_adapter: np.ndarray,
            dtype: str, rows=None, assert_elementwise=True):
    """got/before: device tensors [T,d] (after / before the call); want64: oracle output for
    `rows` (all rows if None).  Checks every inactive row bitwise (on the device) and the
    selected active rows against the oracle; returns the worst row-wise relative error."""
    T = got.shape[0]
    active = row_adapter >= 0
    inactive = torch.from_numpy(~active).to(got.device)
    if bool(inactive.any()):
        assert torch.equal(bits(got)[inactive], bits(before)[inactive]), \
            "a row outside the position set was modified"
    if rows is None:
        rows = np.arange(T)
    rows = np.asarray(rows)
    sel_active = active[rows]
    if not sel_active.any():
        return 0.0
    global last_secondary
    worst, second = 0.0, 0.0
    act_rows = rows[sel_active]
    o_all = want64[sel_active]
    step = max(1, (1 << 27) // max(1, got.shape[1]))          # bounded host memory for large full-size cases
    for lo in range(0, len(act_rows), step):
        g = got[torch.from_numpy(act_rows[lo:lo + step]).to(got.device)].double().cpu().numpy()
        o = o_all[lo:lo + step]
        diff = np.abs(g - o)
        row_max = np.maximum(np.max(np.abs(o), axis=1), 1e-30)
        worst = max(worst, float((np.max(diff, axis=1) / row_max).max()))
        second = max(second, float((diff / np.maximum(np.abs(o), FLOOR * row_max[:, None])).max()))
    last_secondary = second
    print(f"    [parity] rows {len(act_rows)}: row-wise {worst:.2e} (bar {TOL[dtype]:.0e}), "
          f"elementwise with floor {second:.2e} (bar {TOL_ELEMENTWISE[dtype]:.0e})", flush=True)
    assert worst <= TOL[dtype], f"row-wise relative error {worst:.3e} exceeds {TOL[dtype]:.0e}"
    assert not assert_elementwise or second <= TOL_ELEMENTWISE[dtype], f"elementwise relative error (floored) {second:.3e} exceeds {TOL_ELEMENTWISE[dtype]:.0e}"
    return worst


def lora_pools_to_device(pool: wl.LoraPool, perm=None):
    """Pointer tables for the C ABI.  LoRA's A [r,m] and B [n,r] are already in the ABI layout.
    `perm` scatters the slots in memory so that nothing can rely on slot i sitting at base+i*size."""
    N = pool.N
    order = list(range(N)) if perm is None else list(perm)
    A_store = [None] * N
    B_store = [None] * N
    for slot in order:                       # allocate in permuted order
        A_store[slot] = pool.A[slot].clone()
        B_store[slot] = pool.B[slot].clone()
    return preft.pointer_table(A_store), preft.pointer_table(B_store), (A_store, B_store)


def direft_pools_to_device(pool: wl.DireftPool, perm=None, bias=True, null_bias=()):
    """W1 = paper's A [r,d]; W2t = transpose of the paper's B -> [d,r]; b [r].  Adapters listed in
    null_bias get a null entry in the bias table (no bias for them)."""
    N = pool.N
    order = list(range(N)) if perm is None else list(perm)
    W1, W2t, b = [None] * N, [None] * N, [None] * N
    for slot in order:
        W1[slot] = pool.A[slot].clone()
        W2t[slot] = pool.B[slot].t().contiguous()
        b[slot] = pool.b[slot].clone()
    btab = None
    if bias:
        btab = preft.pointer_table(b)
        for i in null_bias:
            btab[i] = 0
    return (preft.pointer_table(W1), preft.pointer_table(W2t), btab, (W1, W2t, b))


def run_lora_case(tab: wl.SegmentTable, pool: wl.LoraPool, x: torch.Tensor, y0: torch.Tensor, dtype: str,
                  scale: float, all_tokens: bool, pad_cols=0, rows=None, perm=None, reuse_schedule=False,
                  pad_x=None, pad_y=None, z_room=False):
    """Tensors live on the GPU; returns (worst error, schedule counts).  pad_cols (or pad_x / pad_y for
    x and y separately): guard columns that widen the row pitch and must come back untouched.
    z_room: a workspace with room for z (the call may then run its sweeps as two launches)."""
    N, r = pool.N, pool.r
    T = tab.T
    mode = preft.PREFT_ALL_TOKENS if all_tokens else preft.PREFT_PREFILL_ONLY
    ss, sa, sp = dev_tables(tab)
    Ap, Bp, keep = lora_pools_to_device(pool, perm)
    ybuf, y = padded(y0, pad_cols if pad_y is None else pad_y, 7.0)
    xbuf, xv = padded(x, pad_cols if pad_x is None else pad_x, -3.0)
    ws = preft.new_workspace(T, tab.S, z_rank=r if z_room else 0)
    if reuse_schedule:
        preft.preft_schedule(ws, ss, sa, sp, T, N, mode)
        preft.preft_lora_apply(y, xv, ss, sa, sp, Ap, Bp, r, scale, mode | preft.PREFT_SCHEDULE_READY, ws)
    else:
        preft.preft_lora_apply(y, xv, ss, sa, sp, Ap, Bp, r, scale, mode, ws)
    torch.cuda.synchronize()
    counts = preft.preft_schedule_counts(ws)
    check_guards(ybuf, T, y0.shape[1], 7.0)
    assert torch.equal(bits(xv), bits(x)), "x was modified"
    pos = ora.ALL_POSITIONS if all_tokens else ora.PROMPT_ONLY
    row_adapter = ora.positions(T, tab.seg_start, tab.seg_adapter, tab.seg_prefill_len, N, pos)
    needed = set(np.unique(row_adapter[row_adapter >= 0] if rows is None else
                           row_adapter[np.asarray(rows)][row_adapter[np.asarray(rows)] >= 0]).tolist())
    A_cpu = [pool.A[i].cpu() if i in needed else None for i in range(N)]
    B_cpu = [pool.B[i].cpu() if i in needed else None for i in range(N)]
    if rows is None:
        want = ora.lora(y0.cpu(), x.cpu(), tab.seg_start, tab.seg_adapter, tab.seg_prefill_len,
                        A_cpu, B_cpu, r, scale, pos)
    else:                                    # large batches: only the sampled rows leave the GPU
        idx = torch.from_numpy(np.asarray(rows)).to(x.device)
        want = ora.lora(y0[idx].cpu(), x[idx].cpu(), tab.seg_start, tab.seg_adapter, tab.seg_prefill_len,
                        A_cpu, B_cpu, r, scale, pos, rows=rows, gathered=True)
    worst = compare(y, y0, want, row_adapter, dtype, rows=rows)
    assert counts[2] == int((row_adapter >= 0).sum()), "scheduler's active-row count differs from the oracle's"
    return worst, counts


def run_direft_case(tab: wl.SegmentTable, pool: wl.DireftPool, h0: torch.Tensor, dtype: str, scale: float,
                    all_tokens: bool, pad_cols=0, rows=None, perm=None, bias=True, reuse_schedule=False,
                    null_bias=()):
    N, r = pool.N, pool.r
    T = tab.T
    mode = preft.PREFT_ALL_TOKENS if all_tokens else preft.PREFT_PREFILL_ONLY
    ss, sa, sp = dev_tables(tab)
    W1p, W2tp, bp, keep = direft_pools_to_device(pool, perm, bias, null_bias)
    hbuf, h = padded(h0, pad_cols, 7.0)
    ws = preft.new_workspace(T, tab.S)
    if reuse_schedule:
        preft.preft_schedule(ws, ss, sa, sp, T, N, mode)
        preft.preft_direft_apply(h, ss, sa, sp, W1p, W2tp, bp, r, scale, mode | preft.PREFT_SCHEDULE_READY, ws)
    else:
        preft.preft_direft_apply(h, ss, sa, sp, W1p, W2tp, bp, r, scale, mode, ws)
    torch.cuda.synchronize()
    counts = preft.preft_schedule_counts(ws)
    check_guards(hbuf, T, h0.shape[1], 7.0)
    pos = ora.ALL_POSITIONS if all_tokens else ora.PROMPT_ONLY
    row_adapter = ora.positions(T, tab.seg_start, tab.seg_adapter, tab.seg_prefill_len, N, pos)
    sel = row_adapter if rows is None else row_adapter[np.asarray(rows)]
    needed = set(np.unique(sel[sel >= 0]).tolist())
    A_cpu = [pool.A[i].cpu() if i in needed else None for i in range(N)]
    B_cpu = [pool.B[i].cpu() if i in needed else None for i in range(N)]
    b_cpu = [pool.b[i].cpu() if (i in needed and i not in null_bias) else None for i in range(N)] if bias else None
    if rows is None:
        want = ora.direft(h0.cpu(), tab.seg_start, tab.seg_adapter, tab.seg_prefill_len,
                          A_cpu, B_cpu, b_cpu, r, scale, pos)
    else:
        idx = torch.from_numpy(np.asarray(rows)).to(h0.device)
        want = ora.direft(h0[idx].cpu(), tab.seg_start, tab.seg_adapter, tab.seg_prefill_len,
                          A_cpu, B_cpu, b_cpu, r, scale, pos, rows=rows, gathered=True)
    worst = compare(h, h0, want, row_adapter, dtype, rows=rows)
    assert counts[2] == int((row_adapter >= 0).sum())
    return worst, counts


def run_direft_layers_case(tab: wl.SegmentTable, pools, h0s, dtype: str, scale: float, all_tokens: bool,
                           bias_layers, pad_cols=0):
    """One many-layer call on len(h0s) residual streams (layer l: pools[l], bias iff bias_layers[l]).
    Every layer is compared with the oracle and, bit for bit, with a one-layer call on a copy."""
    L, N, r, T = len(h0s), pools[0].N, pools[0].r, tab.T
    mode = preft.PREFT_ALL_TOKENS if all_tokens else preft.PREFT_PREFILL_ONLY
    ss, sa, sp = dev_tables(tab)
    dev = [direft_pools_to_device(pools[l], None, bias_layers[l]) for l in range(L)]
    bufs = [padded(h0s[l], pad_cols, 7.0) for l in range(L)]
    hs = [b[1] for b in bufs]
    singles = [padded(h0s[l], pad_cols, 7.0) for l in range(L)]
    table = lambda ptrs: torch.tensor(ptrs, dtype=torch.int64, device="cuda")
    W1s = table([dev[l][0].data_ptr() for l in range(L)])
    W2s = table([dev[l][1].data_ptr() for l in range(L)])
    bs = table([dev[l][2].data_ptr() if bias_layers[l] else 0 for l in range(L)]) if any(bias_layers) else None
    ws = preft.new_workspace(T, tab.S)
    preft.preft_direft_apply_layers(hs, preft.pointer_table(hs) if all(h.is_contiguous() for h in hs) else
                                    table([h.data_ptr() for h in hs]), ss, sa, sp, W1s, W2s, bs, N, r, scale, mode, ws)
    for l in range(L):
        preft.preft_direft_apply(singles[l][1], ss, sa, sp, dev[l][0], dev[l][1], dev[l][2], r, scale,
                                 mode | preft.PREFT_SCHEDULE_READY, ws)
    torch.cuda.synchronize()
    pos = ora.ALL_POSITIONS if all_tokens else ora.PROMPT_ONLY
    row_adapter = ora.positions(T, tab.seg_start, tab.seg_adapter, tab.seg_prefill_len, N, pos)
    needed = set(np.unique(row_adapter[row_adapter >= 0]).tolist())
    worst = 0.0
    for l in range(L):
        check_guards(bufs[l][0], T, h0s[l].shape[1], 7.0)
        assert torch.equal(bits(hs[l]), bits(singles[l][1])), f"layer {l}: differs from the one-layer call"
        pick = lambda mats: [mats[i].cpu() if i in needed else None for i in range(N)]
        want = ora.direft(h0s[l].cpu(), tab.seg_start, tab.seg_adapter, tab.seg_prefill_len, pick(pools[l].A),
                          pick(pools[l].B), pick(pools[l].b) if bias_layers[l] else None, r, scale, pos)
        worst = max(worst, compare(hs[l], h0s[l], want, row_adapter, dtype))
    return worst


def run_loreft_case(tab: wl.SegmentTable, W, R, b, h0: torch.Tensor, dtype: str, scale: float, all_tokens: bool,
                    pad_cols=0):
    """W, R: lists of [r,d] device tensors, b: list of [r] or None.  Derived factors come from
    preft_loreft_prepare; the oracle sees W, R and b themselves."""
    N, r, d = len(W), int(W[0].shape[0]), int(W[0].shape[1])
    T = tab.T
    mode = preft.PREFT_ALL_TOKENS if all_tokens else preft.PREFT_PREFILL_ONLY
    ss, sa, sp = dev_tables(tab)
    D = [torch.full_like(W[i], float("nan")) for i in range(N)]
    Rt = [torch.full((d, r), float("nan"), dtype=W[i].dtype, device=W[i].device) for i in range(N)]
    for i in range(N):
        preft.preft_loreft_prepare(D[i], Rt[i], W[i], R[i])
    hbuf, h = padded(h0, pad_cols, 7.0)
    ws = preft.new_workspace(T, tab.S)
    preft.preft_loreft_apply(h, ss, sa, sp, preft.pointer_table(D), preft.pointer_table(Rt),
                             None if b is None else preft.pointer_table(b), r, scale, mode, ws)
    torch.cuda.synchronize()
    for i in range(N):         # the derived factors themselves: one rounding of the exact difference, exact transpose
        assert torch.equal(bits(D[i]), bits((W[i].double() - R[i].double()).to(W[i].dtype)))
        assert torch.equal(bits(Rt[i]), bits(R[i].t().contiguous()))
    check_guards(hbuf, T, d, 7.0)
    pos = ora.ALL_POSITIONS if all_tokens else ora.PROMPT_ONLY
    row_adapter = ora.positions(T, tab.seg_start, tab.seg_adapter, tab.seg_prefill_len, N, pos)
    want = ora.loreft(h0.cpu(), tab.seg_start, tab.seg_adapter, tab.seg_prefill_len, [w.cpu() for w in W],
                      [q.cpu() for q in R], None if b is None else [v.cpu() for v in b], r, scale, pos)
    # secondary figure reported only: the derived factor D = W - R is itself rounded to the storage type,
    # an error of 2^-9 of each element of D, which reaches an output element scaled by the row, not by
    # that element
    return compare(h, h0, want, row_adapter, dtype, assert_elementwise=False)
