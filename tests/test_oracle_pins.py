"""Pins of the fp64 CPU oracle against things other than itself.

Each test checks ``oracle/preft_oracle.c`` against what the paper and the mathematics fix:
a hand-worked example (tests/golden/hand_example.txt), the merged dense operator computed
by a library matmul, a brute-force block operator built in pure Python, the identity and
position-set invariants of Eq. 1/4, algebraic properties of Eq. 2/3, and for LoReFT (App. C.2)
a hand example, its zero-delta initialisation, its reduction to DiReFT and its subspace property.  The last test
shows that plausible mistakes (dropped prefactor, transposed operand, unscaled or missing
bias, off-by-one position set) would fail these pins.
"""
import os

import numpy as np
import pytest
import torch

from oracle import preft_oracle as ora
from paper_2605_14217_amd import workloads as wl

GOLD = os.path.join(os.path.dirname(__file__), "golden", "hand_example.txt")
RNG = lambda s: np.random.Generator(np.random.PCG64(s))


def _one_seg(T, adapter=0, prompt=None):
    return wl.from_lengths([T], [adapter], [T if prompt is None else prompt])


def _read_gold():
    vals = {}
    with open(GOLD) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            k, *v = line.split()
            vals[k] = np.array([float(t) for t in v])
    return vals


# ---------------------------------------------------------------------------------------
# 1. hand-worked example (Eq. 2, Eq. 3 / App. C.2)
# ---------------------------------------------------------------------------------------
def test_hand_worked_example():
    g = _read_gold()
    tab = _one_seg(1)
    out = ora.lora(g["lora_y0"][None], g["lora_x"][None], tab.seg_start, tab.seg_adapter,
                   tab.seg_prefill_len, [g["lora_A"].reshape(2, 3)], [g["lora_B"].reshape(2, 2)],
                   2, float(g["lora_alpha"][0]), ora.PROMPT_ONLY)
    assert np.array_equal(out[0], g["lora_out"])
    out = ora.direft(g["direft_h"][None], tab.seg_start, tab.seg_adapter, tab.seg_prefill_len,
                     [g["direft_A"].reshape(2, 3)], [g["direft_B"].reshape(2, 3)], [g["direft_b"]],
                     2, float(g["direft_s"][0]), ora.PROMPT_ONLY)
    assert np.array_equal(out[0], g["direft_out"])


# ---------------------------------------------------------------------------------------
# 2. a single adapter is the merged dense map (library matmul as the textbook routine)
# ---------------------------------------------------------------------------------------
@pytest.mark.parametrize("m,n,r", [(24, 40, 3), (64, 16, 8), (7, 5, 1)])
def test_lora_equals_merged_dense(m, n, r):
    rng = RNG(1)
    T, alpha = 11, 0.37
    W = rng.standard_normal((n, m))
    A = rng.standard_normal((r, m))
    B = rng.standard_normal((n, r))
    x = rng.standard_normal((T, m))
    y0 = x @ W.T
    tab = _one_seg(T)
    got = ora.lora(y0, x, tab.seg_start, tab.seg_adapter, tab.seg_prefill_len, [A], [B], r, alpha,
                   ora.PROMPT_ONLY)
    want = x @ (W + alpha * (B @ A)).T
    assert np.max(np.abs(got - want)) <= 1e-12 * np.max(np.abs(want))


@pytest.mark.parametrize("d,r", [(32, 4), (9, 2), (48, 16)])
def test_direft_equals_dense_affine_map(d, r):
    rng = RNG(2)
    T, s = 9, 1.0 / np.sqrt(r)
    A = rng.standard_normal((r, d))
    B = rng.standard_normal((r, d))
    b = rng.standard_normal(r)
    h = rng.standard_normal((T, d))
    tab = _one_seg(T)
    got = ora.direft(h, tab.seg_start, tab.seg_adapter, tab.seg_prefill_len, [A], [B], [b], r, s,
                     ora.PROMPT_ONLY)
    M = np.eye(d) + s * (B.T @ A)
    want = h @ M.T + s * (B.T @ b)[None, :]
    assert np.max(np.abs(got - want)) <= 1e-12 * np.max(np.abs(want))


# ---------------------------------------------------------------------------------------
# 3. brute force on tiny inputs: the whole batch as one dense block operator, pure Python
# ---------------------------------------------------------------------------------------
def _brute_force_lora(y0, x, tab, A, B, alpha, all_positions):
    T, m = x.shape
    n = y0.shape[1]
    N = len(A)
    op = [[0.0] * (T * m) for _ in range(T * n)]        # (T n) x (T m), block diagonal
    for s in range(tab.S):
        a = int(tab.seg_adapter[s])
        if a < 0 or a >= N:
            continue
        lo, hi = int(tab.seg_start[s]), int(tab.seg_start[s + 1])
        last = hi if all_positions else lo + min(int(tab.seg_prefill_len[s]), hi - lo)
        for t in range(lo, last):
            for i in range(n):
                for j in range(m):
                    acc = 0.0
                    for k in range(len(A[a])):
                        acc += B[a][i][k] * A[a][k][j]
                    op[t * n + i][t * m + j] = alpha * acc
    xf = [float(v) for v in x.reshape(-1)]
    out = np.array(y0, dtype=np.float64).reshape(-1).copy()
    for row in range(T * n):
        acc = 0.0
        for col in range(T * m):
            acc += op[row][col] * xf[col]
        out[row] += acc
    return out.reshape(T, n)


@pytest.mark.parametrize("all_positions", [False, True])
def test_lora_brute_force_block_operator(all_positions):
    rng = RNG(3)
    N, m, n, r = 3, 6, 5, 2
    tab = wl.from_lengths([3, 1, 0, 4, 1, 2, 3], [0, 1, 2, -1, 2, 7, 1], [3, 0, 0, 4, 1, 1, 0])
    T = tab.T
    A = [rng.integers(-3, 4, size=(r, m)).astype(np.float64) for _ in range(N)]
    B = [rng.integers(-3, 4, size=(n, r)).astype(np.float64) for _ in range(N)]
    x = rng.integers(-4, 5, size=(T, m)).astype(np.float64)
    y0 = rng.integers(-9, 10, size=(T, n)).astype(np.float64)
    got = ora.lora(y0, x, tab.seg_start, tab.seg_adapter, tab.seg_prefill_len, A, B, r, 0.25,
                   ora.ALL_POSITIONS if all_positions else ora.PROMPT_ONLY)
    want = _brute_force_lora(y0, x, tab, [a.tolist() for a in A], [b.tolist() for b in B], 0.25,
                             all_positions)
    assert np.array_equal(got, want)     # small integers and alpha = 1/4: exact in fp64


def test_direft_brute_force_per_row():
    rng = RNG(4)
    N, d, r, s = 3, 7, 2, 0.5
    tab = wl.from_lengths([2, 1, 5, 1, 0, 3], [2, 0, 1, -1, 0, 5], [2, 0, 3, 1, 0, 3])
    T = tab.T
    A = rng.integers(-3, 4, size=(N, r, d)).astype(np.float64)
    B = rng.integers(-3, 4, size=(N, r, d)).astype(np.float64)
    b = rng.integers(-3, 4, size=(N, r)).astype(np.float64)
    h = rng.integers(-4, 5, size=(T, d)).astype(np.float64)
    got = ora.direft(h, tab.seg_start, tab.seg_adapter, tab.seg_prefill_len, list(A), list(B), list(b),
                     r, s, ora.PROMPT_ONLY)
    want = h.copy()
    for sg in range(tab.S):
        a = int(tab.seg_adapter[sg])
        if a < 0 or a >= N:
            continue
        lo, hi = int(tab.seg_start[sg]), int(tab.seg_start[sg + 1])
        for t in range(lo, lo + min(int(tab.seg_prefill_len[sg]), hi - lo)):
            for j in range(d):
                acc = 0.0
                for k in range(r):
                    inner = b[a, k]
                    for jj in range(d):
                        inner += A[a, k, jj] * h[t, jj]
                    acc += B[a, k, j] * inner
                want[t, j] = h[t, j] + s * acc
    assert np.array_equal(got, want)


# ---------------------------------------------------------------------------------------
# 4. identity cases (zero-delta initialisation, App. C.1; no adapter; zero prefactor)
# ---------------------------------------------------------------------------------------
def _rand_lora_case(seed, dtype="f64", N=4, m=32, n=24, r=4, S=12, max_len=9):
    rng = RNG(seed)
    tab = wl.random_segments(rng, S, N, max_len)
    pool = wl.lora_pool(N, r, m, n, dtype, seed=seed)
    x = wl.activations(tab.T, m, dtype, seed=seed + 100)
    y0 = wl.activations(tab.T, n, dtype, seed=seed + 200)
    return tab, pool, x, y0


def _rand_direft_case(seed, dtype="f64", N=4, d=32, r=4, S=12, max_len=9):
    rng = RNG(seed)
    tab = wl.random_segments(rng, S, N, max_len)
    pool = wl.direft_pool(N, r, d, dtype, seed=seed)
    h = wl.activations(tab.T, d, dtype, seed=seed + 100)
    return tab, pool, h


def _lora(tab, pool, x, y0, alpha=2.0, mode=ora.PROMPT_ONLY, rows=None):
    return ora.lora(y0, x, tab.seg_start, tab.seg_adapter, tab.seg_prefill_len,
                    list(pool.A), list(pool.B), pool.r, alpha, mode, rows=rows)


def _direft(tab, pool, h, s=1.0, mode=ora.PROMPT_ONLY, rows=None, bias=True):
    return ora.direft(h, tab.seg_start, tab.seg_adapter, tab.seg_prefill_len,
                      list(pool.A), list(pool.B), list(pool.b) if bias else None, pool.r, s, mode,
                      rows=rows)


def test_identity_cases():
    tab, pool, x, y0 = _rand_lora_case(5)
    y0n = y0.numpy()
    zeroB = wl.LoraPool(pool.A, torch.zeros_like(pool.B))
    assert np.array_equal(_lora(tab, zeroB, x, y0, mode=ora.ALL_POSITIONS), y0n)
    assert np.array_equal(_lora(tab, pool, x, y0, alpha=0.0, mode=ora.ALL_POSITIONS), y0n)
    none = wl.SegmentTable(tab.seg_start, np.full_like(tab.seg_adapter, -1), tab.seg_prefill_len)
    assert np.array_equal(_lora(none, pool, x, y0, mode=ora.ALL_POSITIONS), y0n)
    assert not np.array_equal(_lora(tab, pool, x, y0, mode=ora.ALL_POSITIONS), y0n)

    tab, dp, h = _rand_direft_case(6)
    hn = h.numpy()
    # either factor zero (the paper states the zero-delta initialisation both ways round)
    assert np.array_equal(_direft(tab, wl.DireftPool(dp.A, torch.zeros_like(dp.B), dp.b), h,
                                  mode=ora.ALL_POSITIONS), hn)
    assert np.array_equal(_direft(tab, wl.DireftPool(torch.zeros_like(dp.A), dp.B, torch.zeros_like(dp.b)), h,
                                  mode=ora.ALL_POSITIONS), hn)
    assert not np.array_equal(_direft(tab, dp, h, mode=ora.ALL_POSITIONS), hn)


# ---------------------------------------------------------------------------------------
# 5. position sets (Eq. 1, Eq. 4): which rows change, which stay bit-identical
# ---------------------------------------------------------------------------------------
def test_position_sets_against_python():
    rng = RNG(7)
    for trial in range(20):
        N = 5
        tab = wl.random_segments(rng, 15, N + 2, 7)       # some ids >= N: treated as no adapter
        for mode in (ora.PROMPT_ONLY, ora.ALL_POSITIONS):
            got = ora.positions(tab.T, tab.seg_start, tab.seg_adapter, tab.seg_prefill_len, N, mode)
            want = np.full(tab.T, -1, dtype=np.int32)
            for s in range(tab.S):
                a = tab.seg_adapter[s]
                if not (0 <= a < N):
                    continue
                lo, hi = tab.seg_start[s], tab.seg_start[s + 1]
                for pos in range(1, hi - lo + 1):          # 1-based position within the sequence
                    in_P = pos <= tab.seg_prefill_len[s] if mode == ora.PROMPT_ONLY else True
                    if in_P:
                        want[lo + pos - 1] = a
            assert np.array_equal(got, want)


def test_prompt_boundary_is_inclusive_and_decode_rows_untouched():
    # one sequence of 6 rows whose prompt is 4 long: rows 0..3 change, rows 4,5 do not
    tab = wl.from_lengths([6, 1], [0, 0], [4, 0])
    pool = wl.lora_pool(1, 2, 8, 8, "f64", seed=8)
    x = wl.activations(7, 8, "f64", seed=1)
    y0 = wl.activations(7, 8, "f64", seed=2)
    out = _lora(tab, pool, x, y0)
    changed = np.any(out != y0.numpy(), axis=1)
    assert changed.tolist() == [True, True, True, True, False, False, False]
    out_all = _lora(tab, pool, x, y0, mode=ora.ALL_POSITIONS)
    assert np.all(np.any(out_all != y0.numpy(), axis=1))
    assert np.array_equal(out_all[:4], out[:4])


def test_all_decode_batch_is_identity_in_prompt_only_mode():
    tab = wl.from_lengths([1] * 9, list(range(3)) * 3, [0] * 9)
    dp = wl.direft_pool(3, 4, 16, "f64", seed=9)
    h = wl.activations(9, 16, "f64", seed=3)
    assert np.array_equal(_direft(tab, dp, h), h.numpy())
    assert not np.array_equal(_direft(tab, dp, h, mode=ora.ALL_POSITIONS), h.numpy())


def test_all_positions_equals_prompt_only_with_full_prompt():
    tab, pool, x, y0 = _rand_lora_case(10)
    full = wl.SegmentTable(tab.seg_start, tab.seg_adapter, tab.seg_len.astype(np.int32))
    assert np.array_equal(_lora(tab, pool, x, y0, mode=ora.ALL_POSITIONS), _lora(full, pool, x, y0))
    tab, dp, h = _rand_direft_case(11)
    full = wl.SegmentTable(tab.seg_start, tab.seg_adapter, tab.seg_len.astype(np.int32))
    assert np.array_equal(_direft(tab, dp, h, mode=ora.ALL_POSITIONS), _direft(full, dp, h))


def test_segment_permutation_invariance():
    rng = RNG(12)
    tab, pool, x, y0 = _rand_lora_case(12, S=14)
    out = _lora(tab, pool, x, y0)
    perm = rng.permutation(tab.S)
    lens = tab.seg_len
    row_idx = np.concatenate([np.arange(tab.seg_start[s], tab.seg_start[s + 1]) for s in perm]).astype(np.int64)
    tab2 = wl.from_lengths(lens[perm], tab.seg_adapter[perm], tab.seg_prefill_len[perm])
    out2 = _lora(tab2, pool, x[row_idx], y0[row_idx])
    assert np.array_equal(out2, out[row_idx])


# ---------------------------------------------------------------------------------------
# 6. algebraic properties of Eq. 2 / Eq. 3
# ---------------------------------------------------------------------------------------
def test_direft_without_bias_is_lora_on_the_residual():
    tab, dp, h = _rand_direft_case(13, d=24, r=3)
    lp = wl.LoraPool(A=dp.A, B=dp.B.transpose(1, 2).contiguous())     # LoRA's B is [n,r]
    a = _direft(tab, dp, h, s=0.7, bias=False)
    b = _lora(tab, lp, h, h, alpha=0.7)
    assert np.max(np.abs(a - b)) <= 1e-13 * np.max(np.abs(a))


def test_rank_additivity_and_affine_in_scale():
    tab, pool, x, y0 = _rand_lora_case(14, r=5)
    y0n = y0.numpy()
    full = _lora(tab, pool, x, y0, alpha=1.3) - y0n
    parts = np.zeros_like(full)
    for k in range(pool.r):
        pk = wl.LoraPool(pool.A[:, k:k + 1].contiguous(), pool.B[:, :, k:k + 1].contiguous())
        parts += _lora(tab, pk, x, y0, alpha=1.3) - y0n
    assert np.max(np.abs(full - parts)) <= 1e-12 * np.max(np.abs(full))
    d1 = _lora(tab, pool, x, y0, alpha=1.0) - y0n
    assert np.max(np.abs(full - 1.3 * d1)) <= 1e-12 * np.max(np.abs(full))

    tab, dp, h = _rand_direft_case(15)
    hn = h.numpy()
    e1 = _direft(tab, dp, h, s=1.0) - hn
    e2 = _direft(tab, dp, h, s=-2.5) - hn
    assert np.max(np.abs(e2 + 2.5 * e1)) <= 1e-12 * np.max(np.abs(e2))   # bias is inside the prefactor


def test_orthonormal_rows_make_the_delta_an_isometry():
    # App. C.2: if the rows of B are orthonormal, ||delta|| = s * ||A h + b||
    rng = RNG(16)
    d, r, T, s = 40, 6, 8, 1.0 / np.sqrt(6)
    Q, _ = np.linalg.qr(rng.standard_normal((d, r)))
    B = Q.T.copy()
    A = rng.standard_normal((r, d))
    b = rng.standard_normal(r)
    h = rng.standard_normal((T, d))
    tab = _one_seg(T)
    out = ora.direft(h, tab.seg_start, tab.seg_adapter, tab.seg_prefill_len, [A], [B], [b], r, s,
                     ora.PROMPT_ONLY)
    lhs = np.linalg.norm(out - h, axis=1)
    rhs = s * np.linalg.norm(h @ A.T + b[None], axis=1)
    assert np.allclose(lhs, rhs, rtol=1e-12, atol=0)


# ---------------------------------------------------------------------------------------
# 7. storage types are widened exactly; row selection matches the full run
# ---------------------------------------------------------------------------------------
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_storage_types_are_widened_exactly(dtype):
    tab, pool, x, y0 = _rand_lora_case(17, dtype=dtype)
    wide = wl.LoraPool(pool.A.double(), pool.B.double())
    assert np.array_equal(_lora(tab, pool, x, y0), _lora(tab, wide, x.double(), y0.double()))
    tab, dp, h = _rand_direft_case(18, dtype=dtype)
    wide = wl.DireftPool(dp.A.double(), dp.B.double(), dp.b.double())
    assert np.array_equal(_direft(tab, dp, h), _direft(tab, wide, h.double()))


def test_row_selection_matches_full_run():
    tab, pool, x, y0 = _rand_lora_case(19, S=20)
    full = _lora(tab, pool, x, y0)
    rows = wl.sample_rows(tab, 2)
    assert np.array_equal(_lora(tab, pool, x, y0, rows=rows), full[rows])
    idx = torch.from_numpy(rows)
    got = ora.lora(y0[idx], x[idx], tab.seg_start, tab.seg_adapter, tab.seg_prefill_len, list(pool.A),
                   list(pool.B), pool.r, 2.0, ora.PROMPT_ONLY, rows=rows, gathered=True)
    assert np.array_equal(got, full[rows])
    tab, dp, h = _rand_direft_case(20, S=20)
    full = _direft(tab, dp, h)
    rows = wl.sample_rows(tab, 2)
    assert np.array_equal(_direft(tab, dp, h, rows=rows), full[rows])
    got = ora.direft(h[torch.from_numpy(rows)], tab.seg_start, tab.seg_adapter, tab.seg_prefill_len, list(dp.A),
                     list(dp.B), list(dp.b), dp.r, 1.0, ora.PROMPT_ONLY, rows=rows, gathered=True)
    assert np.array_equal(got, full[rows])


# ---------------------------------------------------------------------------------------
# 7b. LoReFT (App. C.2): hand example, zero-delta initialisation, reduction to DiReFT, and the
#     subspace property that defines it when R has orthonormal rows
# ---------------------------------------------------------------------------------------
def _loreft(tab, W, R, b, h, s=1.0, mode=ora.PROMPT_ONLY, rows=None):
    return ora.loreft(h, tab.seg_start, tab.seg_adapter, tab.seg_prefill_len, list(W), list(R),
                      None if b is None else list(b), W[0].shape[0], s, mode, rows=rows)


def test_loreft_hand_worked_example():
    g = _read_gold()
    tab = _one_seg(1)
    out = _loreft(tab, [g["loreft_W"].reshape(2, 3)], [g["loreft_R"].reshape(2, 3)], [g["loreft_b"]],
                  g["loreft_h"][None], float(g["loreft_s"][0]))
    assert np.array_equal(out[0], g["loreft_out"])


def test_loreft_identity_at_its_initialisation_and_on_rows_outside_the_set():
    tab, pool, h = _rand_direft_case(21)
    R = [m.numpy() for m in pool.B]
    # W = R, b = 0 (the zero-delta initialisation of App. C.1): exact identity
    out = _loreft(tab, R, R, [np.zeros(pool.r)] * pool.N, h, s=0.7, mode=ora.ALL_POSITIONS)
    assert np.array_equal(out, h.numpy())
    # rows outside the position set keep their value whatever the weights
    W = [m.numpy() for m in pool.A]
    out = _loreft(tab, W, R, list(pool.b), h, s=0.7)
    owner = ora.positions(tab.T, tab.seg_start, tab.seg_adapter, tab.seg_prefill_len, pool.N, ora.PROMPT_ONLY)
    assert np.array_equal(out[owner < 0], h.numpy()[owner < 0])
    assert not np.array_equal(out[owner >= 0], h.numpy()[owner >= 0])


def test_loreft_is_direft_with_the_difference_factor():
    # integer-valued factors: W - R is exact, so the two oracles must agree to rounding order
    rng = RNG(22)
    tab = wl.random_segments(rng, 10, 3, 7)
    d, r, N = 12, 3, 3
    W = [rng.integers(-4, 5, size=(r, d)).astype(np.float64) for _ in range(N)]
    R = [rng.integers(-4, 5, size=(r, d)).astype(np.float64) for _ in range(N)]
    b = [rng.integers(-4, 5, size=r).astype(np.float64) for _ in range(N)]
    h = rng.integers(-4, 5, size=(tab.T, d)).astype(np.float64)
    got = _loreft(tab, W, R, b, h, s=0.5, mode=ora.ALL_POSITIONS)
    want = ora.direft(h, tab.seg_start, tab.seg_adapter, tab.seg_prefill_len, [w - q for w, q in zip(W, R)], R, b,
                      r, 0.5, ora.ALL_POSITIONS)
    assert np.array_equal(got, want)             # small integers: every sum is exact in fp64


@pytest.mark.parametrize("s", [1.0, 0.25])
def test_loreft_subspace_property_with_orthonormal_rows(s):
    # R R^T = I: the component of h in the row space of R becomes (1-s) R h + s (W h + b) and the
    # orthogonal complement is untouched; for s = 1 the projection is replaced by W h + b outright
    rng = RNG(23)
    d, r, T = 40, 5, 9
    R = np.linalg.qr(rng.standard_normal((d, r)))[0].T
    W = rng.standard_normal((r, d))
    b = rng.standard_normal(r)
    h = rng.standard_normal((T, d))
    out = _loreft(_one_seg(T), [W], [R], [b], h, s=s)
    np.testing.assert_allclose(out @ R.T, (1 - s) * (h @ R.T) + s * (h @ W.T + b), rtol=1e-12, atol=1e-12)
    P = np.eye(d) - R.T @ R
    np.testing.assert_allclose(out @ P, h @ P, rtol=1e-12, atol=1e-12)


def test_loreft_plausible_mistakes_would_fail_the_pins():
    g = _read_gold()
    W, R = g["loreft_W"].reshape(2, 3), g["loreft_R"].reshape(2, 3)
    b, h, s = g["loreft_b"], g["loreft_h"], float(g["loreft_s"][0])
    want = g["loreft_out"]
    assert np.array_equal(h + s * (R.T @ (W @ h + b - R @ h)), want)
    wrong = {
        "rotation term added": h + s * (R.T @ (W @ h + b + R @ h)),
        "rotation term missing": h + s * (R.T @ (W @ h + b)),
        "W in the write-back": h + s * (W.T @ (W @ h + b - R @ h)),
        "bias outside the prefactor": h + s * (R.T @ (W @ h - R @ h)) + R.T @ b,
        "dropped prefactor": h + R.T @ (W @ h + b - R @ h),
        "W and R swapped": h + s * (W.T @ (R @ h + b - W @ h)),
    }
    for name, w in wrong.items():
        assert not np.allclose(w, want), name


# ---------------------------------------------------------------------------------------
# 8. the pins discriminate: plausible mistakes, planted in numpy restatements, fail them
# ---------------------------------------------------------------------------------------
def test_plausible_mistakes_would_fail_the_pins():
    g = _read_gold()
    A, B = g["lora_A"].reshape(2, 3), g["lora_B"].reshape(2, 2)
    x, y0, al = g["lora_x"], g["lora_y0"], float(g["lora_alpha"][0])
    want = g["lora_out"]
    wrong = {
        "dropped prefactor": y0 + B @ (A @ x),
        "transposed B": y0 + al * (B.T @ (A @ x)),
        "prefactor on y0": al * (y0 + B @ (A @ x)),
        "delta only": al * (B @ (A @ x)),
    }
    for name, w in wrong.items():
        assert not np.allclose(w, want), name
    A, B = g["direft_A"].reshape(2, 3), g["direft_B"].reshape(2, 3)
    b, h, s = g["direft_b"], g["direft_h"], float(g["direft_s"][0])
    want = g["direft_out"]
    wrong = {
        "missing bias": h + s * (B.T @ (A @ h)),
        "bias outside the prefactor": h + s * (B.T @ (A @ h)) + B.T @ b,
        "A and B swapped": h + s * (A.T @ (B @ h + b)),
        "dropped prefactor": h + B.T @ (A @ h + b),
    }
    for name, w in wrong.items():
        assert not np.allclose(w, want), name
