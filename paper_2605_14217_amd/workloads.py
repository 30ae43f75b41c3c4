"""Seeded synthetic inputs for the adapter-apply path: segment tables, activations, pools.

This module holds *no* adapter arithmetic.  It is the only code shared by the CPU-oracle
tests and the GPU tests/benchmark, and it serves both the same arrays.

The batches stand in for the serving workload of the paper's benchmark appendix (App. E:
a flattened continuous batch of prompt chunks and single decode tokens, one adapter per
request drawn from a popularity mix, random untrained adapter weights).  Sizes, length
laws and popularity laws are the five configurations this build is measured on; they are
listed in ``CONFIGS`` below.

Small integer tables come from ``numpy.random.Generator(PCG64(seed))`` on the host.
Activations and weights come from ``torch.randn`` with a seeded generator *on the device
they are requested for* (so the 10^10-element buffers of the large configurations are
never produced on the host); a test always hands the very same tensors to both sides.
"""
from __future__ import annotations

import dataclasses
import math
from typing import Dict, List, Optional

import numpy as np
import torch


# ----------------------------------------------------------------------------------------
# segment tables
# ----------------------------------------------------------------------------------------
@dataclasses.dataclass
class SegmentTable:
    """A flattened token batch: rows seg_start[s]..seg_start[s+1]-1 belong to sequence s."""
    seg_start: np.ndarray        # int32 [S+1], seg_start[0] = 0, seg_start[S] = T
    seg_adapter: np.ndarray      # int32 [S], -1 = no adapter
    seg_prefill_len: np.ndarray  # int32 [S], leading rows that are prompt positions

    @property
    def S(self) -> int:
        return int(len(self.seg_adapter))

    @property
    def T(self) -> int:
        return int(self.seg_start[-1]) if len(self.seg_start) else 0

    @property
    def seg_len(self) -> np.ndarray:
        return np.diff(self.seg_start)

    def active_rows(self, all_tokens: bool, N: int) -> int:
        """Rows the given mode makes active (bookkeeping for throughput figures only)."""
        has = (self.seg_adapter >= 0) & (self.seg_adapter < N)
        n = self.seg_len if all_tokens else np.minimum(self.seg_prefill_len, self.seg_len)
        return int(np.sum(np.where(has, n, 0)))

    def distinct_active_adapters(self, all_tokens: bool, N: int) -> int:
        has = (self.seg_adapter >= 0) & (self.seg_adapter < N)
        n = self.seg_len if all_tokens else np.minimum(self.seg_prefill_len, self.seg_len)
        return int(len(np.unique(self.seg_adapter[has & (n > 0)])))

    def decode_only(self) -> "SegmentTable":
        """The batch's decode segments alone (a decode-only engine step)."""
        keep = self.seg_prefill_len == 0
        lens = self.seg_len[keep]
        return from_lengths(lens, self.seg_adapter[keep], np.zeros_like(lens))


def lora_algorithmic_bytes(T_act: int, d_in: int, d_outs, r: int, n_adapters: int, e: int = 2) -> int:
    """Bytes one LoRA launch has to move, whatever the kernel: every active row of x once, every
    active row of each output once in and once out, and the two factors of every distinct active
    adapter once per output.  d_outs: the outputs computed from the same x (one entry unless packed)."""
    return e * T_act * (d_in + 2 * sum(d_outs)) + e * r * n_adapters * sum(d_in + n for n in d_outs)


def direft_algorithmic_bytes(T_act: int, d: int, r: int, n_adapters: int, e: int = 2) -> int:
    """Bytes one DiReFT launch has to move: every active row of h once in and once out; both
    factors and the bias of every distinct active adapter once."""
    return e * T_act * 2 * d + e * (2 * r * d + r) * n_adapters


def from_lengths(lens, adapters, prefill_lens) -> SegmentTable:
    lens = np.asarray(lens, dtype=np.int64)
    start = np.zeros(len(lens) + 1, dtype=np.int64)
    np.cumsum(lens, out=start[1:])
    assert start[-1] < 2**31
    return SegmentTable(start.astype(np.int32), np.asarray(adapters, dtype=np.int32),
                        np.asarray(prefill_lens, dtype=np.int32))


def _zipf_ids(rng, n, N, alpha):
    p = 1.0 / np.arange(1, N + 1, dtype=np.float64) ** alpha
    return rng.choice(N, size=n, p=p / p.sum()).astype(np.int32)


def _mixed_batch(rng, prefill_lens, prefill_ids, decode_ids, shuffle=True) -> SegmentTable:
    """Prompt chunks (prefill_len == len) plus single decode tokens (len 1, prefill_len 0)."""
    n_p, n_d = len(prefill_lens), len(decode_ids)
    lens = np.concatenate([np.asarray(prefill_lens, dtype=np.int64), np.ones(n_d, dtype=np.int64)])
    ids = np.concatenate([np.asarray(prefill_ids, dtype=np.int32), np.asarray(decode_ids, dtype=np.int32)])
    pre = np.concatenate([np.asarray(prefill_lens, dtype=np.int64), np.zeros(n_d, dtype=np.int64)])
    if shuffle:
        order = rng.permutation(n_p + n_d)
        lens, ids, pre = lens[order], ids[order], pre[order]
    return from_lengths(lens, ids, pre)


CONFIGS: Dict[str, dict] = {
    # hidden 512, one 512->512 projection, 4 adapters, rank 4, fp32, 8 x 64 prompt rows + 8 decode rows
    "tiny": dict(dtype="f32", N=4, ranks=(4,), lora_scale=2.0,
                 lora_shapes={"proj": (512, 512)}, direft_d=512),
    # Llama-3.1-8B projections, 64 LoRA adapters, 32 prompts U[256,2048] + 224 decode rows
    "llama8b_lora": dict(dtype="bf16", N=64, ranks=(1, 8, 16), lora_scale=2.0,
                         lora_shapes={"q": (4096, 4096), "k": (4096, 1024), "v": (4096, 1024),
                                      "o": (4096, 4096), "gate": (4096, 14336),
                                      "up": (4096, 14336), "down": (14336, 4096)},
                         direft_d=4096),
    # Llama-3.1-8B residual stream, 256 DiReFT adapters, 128 prompts U[128,1024] + 896 decode rows
    "llama8b_direft": dict(dtype="bf16", N=256, ranks=(8, 16), direft_d=4096, lora_shapes={},
                           lora_scale=2.0),
    # Llama-3.1-70B single-layer shapes, 512 adapters, 512 prompts lognormal + 3584 decode rows
    "llama70b_lora": dict(dtype="bf16", N=512, ranks=(1, 16, 64), lora_scale=2.0,
                          lora_shapes={"q": (8192, 8192), "k": (8192, 1024), "v": (8192, 1024),
                                       "o": (8192, 8192), "gate": (8192, 28672),
                                       "up": (8192, 28672), "down": (28672, 8192)},
                          direft_d=8192),
    # skewed mixed batch at d=8192: Zipf(1.1) over 1024 adapters, bimodal prompts, 16384 decode rows
    "skewed70b": dict(dtype="bf16", N=1024, ranks=(32,), lora_scale=2.0,
                      lora_shapes={"res": (8192, 8192)}, direft_d=8192),
}


def make_segments(config: str, seed: int = 0, scale_down: int = 1) -> SegmentTable:
    """Segment table of a named configuration.

    ``scale_down`` > 1 divides request counts and lengths (never below 1) so that the CPU
    oracle can finish the same *structure* in seconds; 1 gives the full-size batch.
    """
    rng = np.random.Generator(np.random.PCG64(seed))
    k = max(1, int(scale_down))

    def cnt(n):
        return max(1, n // k)

    def ln(a):
        return np.maximum(1, np.asarray(a) // k)

    if config == "tiny":
        N = 4
        req_ids = rng.integers(0, N, size=8)
        return _mixed_batch(rng, np.full(8, 64), req_ids, rng.integers(0, N, size=8), shuffle=False)
    if config == "llama8b_lora":
        N, n_p, n_d = 64, cnt(32), cnt(224)
        lens = ln(rng.integers(256, 2048 + 1, size=n_p))
        return _mixed_batch(rng, lens, rng.integers(0, N, size=n_p), rng.integers(0, N, size=n_d))
    if config == "llama8b_direft":
        N, n_p, n_d = 256, cnt(128), cnt(896)
        lens = ln(rng.integers(128, 1024 + 1, size=n_p))
        return _mixed_batch(rng, lens, rng.integers(0, N, size=n_p), rng.integers(0, N, size=n_d))
    if config == "llama70b_lora":
        N, n_p, n_d = 512, cnt(512), cnt(3584)
        # median 512, sigma 0.8 (the sigma of the paper's own prompt-length law, App. E.1)
        raw = np.exp(math.log(512.0) + 0.8 * rng.standard_normal(n_p))
        lens = ln(np.clip(np.rint(raw), 32, 8192).astype(np.int64))
        ids = rng.permutation(N)[:n_p]            # every request its own adapter
        return _mixed_batch(rng, lens, ids, rng.integers(0, N, size=n_d))
    if config == "skewed70b":
        N, n_p, n_d = 1024, cnt(256), cnt(16384)
        short = rng.integers(16, 128 + 1, size=n_p)
        long_ = rng.integers(4096, 16384 + 1, size=n_p)
        lens = ln(np.where(rng.random(n_p) < 0.7, short, long_))
        return _mixed_batch(rng, lens, _zipf_ids(rng, n_p, N, 1.1), _zipf_ids(rng, n_d, N, 1.1))
    raise KeyError(config)


def random_segments(rng: np.random.Generator, S: int, N: int, max_len: int,
                    p_none: float = 0.15, p_empty: float = 0.1) -> SegmentTable:
    """Arbitrary table for property tests: empty segments, adapter-less segments, decode
    rows, whole-prompt chunks and sequences whose prompt ends mid-segment."""
    lens = rng.integers(1, max_len + 1, size=S)
    lens[rng.random(S) < p_empty] = 0
    lens[rng.random(S) < 0.3] = 1
    kind = rng.integers(0, 3, size=S)            # 0: decode, 1: whole prompt, 2: prompt ends inside
    pre = np.where(kind == 0, 0, np.where(kind == 1, lens, (lens * rng.random(S)).astype(np.int64)))
    ids = rng.integers(0, max(N, 1), size=S).astype(np.int32)
    ids[rng.random(S) < p_none] = -1
    return from_lengths(lens, ids, pre)


# ----------------------------------------------------------------------------------------
# request stream and first-come-first-served engine steps (paper App. E.1 and E.3)
# ----------------------------------------------------------------------------------------
@dataclasses.dataclass
class RequestStream:
    prompt_len: np.ndarray   # int64 [R]
    output_len: np.ndarray   # int64 [R], >= 2
    adapter: np.ndarray      # int32 [R]


def request_stream(n_requests: int, n_adapters: int, mix: str = "uniform", l_max: int = 2048,
                   seed: int = 0, zipf_alpha: float = 1.0) -> RequestStream:
    """Requests of the paper's serving microbenchmark (App. E.1).

    Prompt length: lognormal with shape 0.8, shift -1 and scale 18 (i.e. -1 + 18 exp(0.8 Z)),
    rounded to an integer (the paper does not say how it is made integral) and clipped to
    [1, l_max - 2]; prompt + output drawn uniformly from [prompt + 2, l_max].  Adapter per
    request from one of the four mixes: identical, uniform, skewed (Zipf), distinct.
    """
    rng = np.random.Generator(np.random.PCG64(seed))
    p = -1.0 + 18.0 * np.exp(0.8 * rng.standard_normal(n_requests))
    p = np.clip(np.rint(p), 1, l_max - 2).astype(np.int64)
    total = rng.integers(p + 2, l_max + 1)               # inclusive upper end
    if mix == "identical":
        ids = np.zeros(n_requests, dtype=np.int32)
    elif mix == "uniform":
        ids = rng.integers(0, n_adapters, size=n_requests).astype(np.int32)
    elif mix == "skewed":
        ids = _zipf_ids(rng, n_requests, n_adapters, zipf_alpha)
    elif mix == "distinct":
        ids = (np.arange(n_requests) % n_adapters).astype(np.int32)
        rng.shuffle(ids)
    else:
        raise ValueError(f"unknown adapter mix {mix!r}")
    return RequestStream(p, total - p, ids)


def fcfs_steps(req: RequestStream, batch: int):
    """Engine steps of a first-come-first-served continuous-batching loop (App. E.3).

    At most ``batch`` requests are in flight; a freed slot is refilled from the stream in
    arrival order.  A request's first step holds its whole prompt as one segment (all rows are
    prompt positions) and yields its first output token; each later step holds one decode
    row for it, until ``output_len`` tokens exist.  Yields ``(table, repeat)``: ``repeat``
    consecutive steps share the table (a run of decode-only steps between two departures).
    """
    R = len(req.prompt_len)
    slots: List[Optional[list]] = [None] * batch      # [request, tokens produced]
    nxt = 0
    while True:
        for i in range(batch):                        # admission, in arrival order
            if slots[i] is None and nxt < R:
                slots[i] = [nxt, 0]
                nxt += 1
        live = [s for s in slots if s is not None]
        if not live:
            return
        lens = [int(req.prompt_len[r]) if done == 0 else 1 for r, done in live]
        pre = [int(req.prompt_len[r]) if done == 0 else 0 for r, done in live]
        ids = [int(req.adapter[r]) for r, _ in live]
        repeat = 1
        if all(done > 0 for _, done in live):         # decode-only: identical until someone leaves
            repeat = min(int(req.output_len[r]) - done for r, done in live)
        yield from_lengths(lens, ids, pre), repeat
        for i in range(batch):
            if slots[i] is None:
                continue
            slots[i][1] += repeat
            if slots[i][1] >= int(req.output_len[slots[i][0]]):
                slots[i] = None


# ----------------------------------------------------------------------------------------
# tensors
# ----------------------------------------------------------------------------------------
_TORCH_DTYPE = {"f32": torch.float32, "bf16": torch.bfloat16, "f64": torch.float64}


def torch_dtype(name: str) -> torch.dtype:
    return _TORCH_DTYPE[name]


def _gen(device, seed):
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def _randn(shape, std, dtype, device, seed):
    """N(0, std^2), drawn in fp32 chunk by chunk and rounded once to ``dtype``."""
    g = _gen(device, seed)
    out = torch.empty(shape, dtype=dtype, device=device)
    flat = out.view(-1)
    step = 1 << 26
    for lo in range(0, flat.numel(), step):
        hi = min(flat.numel(), lo + step)
        flat[lo:hi] = (torch.randn(hi - lo, generator=g, device=device, dtype=torch.float32) * std).to(dtype)
    return out


def activations(T: int, d: int, dtype: str, device="cpu", seed: int = 0) -> torch.Tensor:
    """[T, d] ~ N(0,1) in the activation dtype."""
    return _randn((T, d), 1.0, _TORCH_DTYPE[dtype], device, seed)


@dataclasses.dataclass
class LoraPool:
    """N LoRA adapters in the paper's shapes: A[i]:[r,m] ~ N(0,1/m), B[i]:[n,r] ~ N(0,1/r)."""
    A: torch.Tensor   # [N, r, m]
    B: torch.Tensor   # [N, n, r]

    @property
    def N(self):
        return self.A.shape[0]

    @property
    def r(self):
        return self.A.shape[1]


@dataclasses.dataclass
class DireftPool:
    """N DiReFT adapters in the paper's shapes: A[i],B[i]:[r,d], b[i]:[r].
    A ~ N(0,1/d), B ~ N(0,1/r), b ~ N(0,1)."""
    A: torch.Tensor   # [N, r, d]
    B: torch.Tensor   # [N, r, d]
    b: torch.Tensor   # [N, r]

    @property
    def N(self):
        return self.A.shape[0]

    @property
    def r(self):
        return self.A.shape[1]


def lora_pool(N: int, r: int, m: int, n: int, dtype: str, device="cpu", seed: int = 0) -> LoraPool:
    dt = _TORCH_DTYPE[dtype]
    return LoraPool(A=_randn((N, r, m), 1.0 / math.sqrt(m), dt, device, seed * 7919 + 1),
                    B=_randn((N, n, r), 1.0 / math.sqrt(r), dt, device, seed * 7919 + 2))


def direft_pool(N: int, r: int, d: int, dtype: str, device="cpu", seed: int = 0) -> DireftPool:
    dt = _TORCH_DTYPE[dtype]
    return DireftPool(A=_randn((N, r, d), 1.0 / math.sqrt(d), dt, device, seed * 7919 + 3),
                      B=_randn((N, r, d), 1.0 / math.sqrt(r), dt, device, seed * 7919 + 4),
                      b=_randn((N, r), 1.0, dt, device, seed * 7919 + 5))


# ----------------------------------------------------------------------------------------
# row samples for checking full-size batches against the oracle
# ----------------------------------------------------------------------------------------
def sample_rows(tab: SegmentTable, per_segment: int, seed: int = 0, max_rows: Optional[int] = None) -> np.ndarray:
    """Deterministic rows worth checking one by one: every segment's first and last row, the
    rows either side of its prompt/decode boundary, and ``per_segment`` random rows; all
    single-row (decode) segments are included while ``max_rows`` allows."""
    rng = np.random.Generator(np.random.PCG64(seed + 12345))
    rows: List[int] = []
    for s in range(tab.S):
        lo, hi = int(tab.seg_start[s]), int(tab.seg_start[s + 1])
        if hi <= lo:
            continue
        p = int(min(max(tab.seg_prefill_len[s], 0), hi - lo))
        cand = {lo, hi - 1, lo + p - 1, lo + p}
        if hi - lo > 4 and per_segment > 0:
            cand.update(int(v) for v in rng.integers(lo, hi, size=per_segment))
        rows.extend(t for t in cand if lo <= t < hi)
    out = np.unique(np.asarray(rows, dtype=np.int64))
    if max_rows is not None and len(out) > max_rows:
        out = np.sort(rng.choice(out, size=max_rows, replace=False))
    return out
