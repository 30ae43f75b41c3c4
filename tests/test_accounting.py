"""The numerator of the roofline figure: the algorithmic bytes bench.py divides by the launch time
are checked against a brute-force count of the distinct elements the definition touches (Eq. 1-3),
and the shrink's arithmetic intensity against the paper's closed form (Eq. 5)."""
import numpy as np
import pytest

from oracle import preft_oracle as ora
from paper_2605_14217_amd import workloads as wl


def _touched(tab, N, d_in, d_outs, r, all_positions, direft):
    """Distinct (tensor, index) pairs read and written by the definition, counted one by one."""
    pos = ora.ALL_POSITIONS if all_positions else ora.PROMPT_ONLY
    owner = ora.positions(tab.T, tab.seg_start, tab.seg_adapter, tab.seg_prefill_len, N, pos)
    reads, writes = set(), set()
    for t in range(tab.T):
        i = int(owner[t])
        if i < 0:
            continue
        if direft:
            for j in range(d_in):
                reads.add(("h", t, j))
                writes.add(("h", t, j))
            for k in range(r):
                reads.add(("b", i, k))
                for j in range(d_in):
                    reads.add(("W1", i, k, j))
                    reads.add(("W2", i, k, j))
        else:
            for j in range(d_in):
                reads.add(("x", t, j))
            for p, n_out in enumerate(d_outs):
                for n in range(n_out):
                    reads.add(("y", p, t, n))
                    writes.add(("y", p, t, n))
                for k in range(r):
                    for j in range(d_in):
                        reads.add(("A", p, i, k, j))
                    for n in range(n_out):
                        reads.add(("B", p, i, n, k))
    return len(reads) + len(writes)


@pytest.mark.parametrize("all_positions", [False, True])
@pytest.mark.parametrize("d_outs", [(12,), (8, 4, 4)])
def test_lora_bytes_equal_a_brute_force_count(all_positions, d_outs):
    rng = np.random.Generator(np.random.PCG64(3))
    N, d_in, r = 5, 10, 3
    tab = wl.random_segments(rng, 14, N + 1, 9)
    elements = _touched(tab, N, d_in, d_outs, r, all_positions, direft=False)
    T_act = tab.active_rows(all_positions, N)
    n_ad = tab.distinct_active_adapters(all_positions, N)
    assert T_act > 0 and n_ad > 1
    assert wl.lora_algorithmic_bytes(T_act, d_in, d_outs, r, n_ad, e=2) == 2 * elements
    assert wl.lora_algorithmic_bytes(T_act, d_in, d_outs, r, n_ad, e=4) == 4 * elements


@pytest.mark.parametrize("all_positions", [False, True])
def test_direft_bytes_equal_a_brute_force_count(all_positions):
    rng = np.random.Generator(np.random.PCG64(4))
    N, d, r = 4, 7, 2
    tab = wl.random_segments(rng, 12, N + 1, 8)
    elements = _touched(tab, N, d, (), r, all_positions, direft=True)
    T_act = tab.active_rows(all_positions, N)
    n_ad = tab.distinct_active_adapters(all_positions, N)
    assert wl.direft_algorithmic_bytes(T_act, d, r, n_ad, e=2) == 2 * elements


def test_active_row_counts_agree_with_the_position_sets():
    rng = np.random.Generator(np.random.PCG64(5))
    for _ in range(10):
        N = 6
        tab = wl.random_segments(rng, 30, N + 2, 12)
        for all_positions in (False, True):
            pos = ora.ALL_POSITIONS if all_positions else ora.PROMPT_ONLY
            owner = ora.positions(tab.T, tab.seg_start, tab.seg_adapter, tab.seg_prefill_len, N, pos)
            assert tab.active_rows(all_positions, N) == int((owner >= 0).sum())
            assert tab.distinct_active_adapters(all_positions, N) == len(np.unique(owner[owner >= 0]))


@pytest.mark.parametrize("r,b,d", [(1, 1, 4096), (16, 2048, 4096), (64, 7, 8192), (8, 100000, 512)])
def test_shrink_intensity_is_the_closed_form_of_eq5(r, b, d):
    """Eq. 5: the down projection of b tokens through one rank-r adapter does 2 r b d flops on
    r d + b d + r b elements, i.e. 1 / (1/r + 1/b + 1/d) flops per byte at two bytes per element.
    The byte count of a launch with a single adapter contains exactly those terms for its shrink
    (x and A), so its intensity is bounded by the closed form with the z traffic taken out."""
    flops = 2 * r * b * d
    elements = r * d + b * d + r * b
    closed = 1.0 / (1.0 / r + 1.0 / b + 1.0 / d)
    assert flops / (2 * elements) == pytest.approx(closed, rel=1e-12)
    # fused path: z never leaves the chip, so the shrink's share of a launch is x and A only, and
    # the launch's byte count is that share plus the output's rows (in and out) and B
    n = 3 * d
    launch = wl.lora_algorithmic_bytes(b, d, (n,), r, 1)
    shrink_bytes = 2 * (b * d + r * d)
    assert launch == shrink_bytes + 2 * (2 * b * n + r * n)
    assert flops / shrink_bytes >= closed
    assert closed < r and closed < b + 1e-9                 # memory-bound by rank and by batch (Sec. 3.3)
