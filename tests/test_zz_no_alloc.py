"""The allocation-free DiReFT entry point (preft_direft_apply_static), through the C ABI: same bits
as preft_direft_apply on the same input, on two calls in a row that share the library's static
schedule area -- the second on a smaller batch, so that anything it wrongly kept from the first
(list entries, counters) would show."""
import numpy as np
import pytest
import torch

import paper_2605_14217_amd as preft
from paper_2605_14217_amd import workloads as wl

pytestmark = pytest.mark.gpu


def _batch(seed, n_prompts, max_len, n_decode, N):
    rng = np.random.Generator(np.random.PCG64(seed))
    lens = list(rng.integers(5, max_len + 1, size=n_prompts)) + [129, 3, 0, 64] + [1] * n_decode
    ids = list(rng.integers(0, N, size=n_prompts)) + [0, 1, 0, -1] + list(rng.integers(0, N, size=n_decode))
    pre = list(lens[:n_prompts]) + [100, 2, 0, 64] + [0] * n_decode
    order = rng.permutation(len(lens))
    return wl.from_lengths(np.asarray(lens)[order], np.asarray(ids)[order], np.asarray(pre)[order])


@pytest.mark.parametrize("dtype,rank,d", [("bf16", 16, 1024), ("bf16", 32, 512), ("bf16", 3, 264), ("f32", 4, 132)])
def test_static_entry_point_matches_the_workspace_entry_point(dtype, rank, d):
    from parity_util import bits, dev_tables, direft_pools_to_device, run_direft_case
    print(f"\n[case] static entry {dtype} r={rank} d={d}", flush=True)
    N = 6
    pool = wl.direft_pool(N, rank, d, dtype, device="cuda", seed=5)
    W1p, W2tp, bp, keep = direft_pools_to_device(pool)
    # first a larger batch, then a smaller one, then a decode-only one (empty schedule in prefill-only mode)
    batches = [_batch(1, 9, 400, 40, N), _batch(2, 3, 90, 7, N), wl.from_lengths(np.ones(5), np.arange(5) % N, np.zeros(5))]
    for mode in (preft.PREFT_PREFILL_ONLY, preft.PREFT_ALL_TOKENS):
        for k, tab in enumerate(batches):
            ss, sa, sp = dev_tables(tab)
            h0 = wl.activations(tab.T, d, dtype, device="cuda", seed=50 + k)
            h_static, h_ws = h0.clone(), h0.clone()
            before = torch.cuda.memory_allocated()
            preft.preft_direft_apply_static(h_static, ss, sa, sp, W1p, W2tp, bp, rank, 0.5, mode)
            assert torch.cuda.memory_allocated() == before
            preft.preft_direft_apply(h_ws, ss, sa, sp, W1p, W2tp, bp, rank, 0.5, mode, preft.new_workspace(tab.T, tab.S))
            torch.cuda.synchronize()
            assert torch.equal(bits(h_static), bits(h_ws)), f"batch {k}, mode {mode}: differs from preft_direft_apply"
            if k < 2:
                assert not torch.equal(bits(h_static), bits(h0))
            # the schedule the static call left serves a second call on the same batch
            h_again = h0.clone()
            preft.preft_direft_apply_static(h_again, ss, sa, sp, W1p, W2tp, bp, rank, 0.5, mode | preft.PREFT_SCHEDULE_READY)
            torch.cuda.synchronize()
            assert torch.equal(bits(h_again), bits(h_ws))
    # and the result is the oracle's (the workspace entry point on the same kind of batch)
    worst, _ = run_direft_case(batches[1], pool, wl.activations(batches[1].T, d, dtype, device="cuda", seed=9), dtype,
                               0.5, False)
    print(f"  oracle check of the reference entry point: worst {worst:.2e}")


def test_static_entry_point_refuses_batches_beyond_its_area():
    from parity_util import dev_tables, direft_pools_to_device
    N, rank, d = 2, 4, 64
    pool = wl.direft_pool(N, rank, d, "bf16", device="cuda", seed=1)
    W1p, W2tp, bp, keep = direft_pools_to_device(pool)
    S = 60000                                           # 60 000 decode rows: 4 bytes short of nothing -- too many list entries
    tab = wl.from_lengths(np.ones(S), np.zeros(S), np.zeros(S))
    assert preft.preft_workspace_bytes(tab.T, tab.S) > preft.PREFT_STATIC_SCRATCH_BYTES
    ss, sa, sp = dev_tables(tab)
    h0 = wl.activations(tab.T, d, "bf16", device="cuda", seed=2)
    h = h0.clone()
    with pytest.raises(preft.PreftError) as e:
        preft.preft_direft_apply_static(h, ss, sa, sp, W1p, W2tp, bp, rank, 1.0, preft.PREFT_ALL_TOKENS)
    assert e.value.code == preft.PREFT_ETOOLARGE
    torch.cuda.synchronize()
    assert torch.equal(h, h0)
