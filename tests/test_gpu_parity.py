"""GPU parity: the HIP path, called through the C ABI, against the fp64 CPU oracle on the same
seeded inputs (see parity_util for the bar).  Sizes are chosen so that the oracle finishes in
seconds while the batch still spans several tiles, ragged tails and every segment kind."""
import sys

import numpy as np
import pytest
import torch

import paper_2605_14217_amd as preft
from paper_2605_14217_amd import workloads as wl

pytestmark = pytest.mark.gpu

VARIANT_AUTO, VARIANT_ROW, VARIANT_VALU, VARIANT_MFMA, VARIANT_WIDE = 0, 1, 2, 3, 4


@pytest.fixture(autouse=True)
def _announce_and_reset(request):
    print(f"\n[case] {request.node.name}", flush=True)
    sys.stdout.flush()
    yield
    preft.set_test_flags(0)


_flags = dict(variant=0, waves=0, rowblocks=0, colsplit=0, resident=0)


def _set(variant=0, waves=0, rowblocks=0, **more):
    """Kernel selection for the calls that follow (test-only bits of the mode argument)."""
    _flags.update(variant=variant, waves=waves, rowblocks=rowblocks, colsplit=0, resident=0)
    _flags.update(more)
    preft.set_test_flags(preft.test_flags(**_flags))


def _set_colsplit(colsplit):
    _flags.update(colsplit=colsplit)
    preft.set_test_flags(preft.test_flags(**_flags))


def _mixed_table(seed, N, n_prompts=6, max_len=300, n_decode=10):
    """Prompt chunks of ragged length (several tiles + tails), decode rows, a sequence whose
    prompt ends inside the segment, an empty segment, an adapter-less prompt, an id >= N."""
    rng = np.random.Generator(np.random.PCG64(seed))
    lens = list(rng.integers(5, max_len + 1, size=n_prompts)) + [129, 128, 17, 4, 3, 0, 200, 64]
    ids = list(rng.integers(0, N, size=n_prompts)) + [0, N - 1, 1, 0, 1, 0, -1, N + 3]
    pre = list(lens[:n_prompts]) + [129, 128, 9, 4, 2, 0, 200, 64]
    lens += [1] * n_decode
    ids += list(rng.integers(0, N, size=n_decode))
    pre += [0] * n_decode
    order = rng.permutation(len(lens))
    return wl.from_lengths(np.asarray(lens)[order], np.asarray(ids)[order], np.asarray(pre)[order])


# ---------------------------------------------------------------------------------------
# Tiny configuration, fp32, exactly as specified (hidden 512, 4 adapters, rank 4, scale 2)
# ---------------------------------------------------------------------------------------
@pytest.mark.parametrize("all_tokens", [False, True])
def test_tiny_fp32_lora_and_direft(all_tokens):
    from parity_util import run_direft_case, run_lora_case
    tab = wl.make_segments("tiny", seed=0)
    assert tab.T == 8 * 64 + 8 and tab.S == 16
    pool = wl.lora_pool(4, 4, 512, 512, "f32", device="cuda", seed=0)
    x = wl.activations(tab.T, 512, "f32", device="cuda", seed=1)
    y0 = wl.activations(tab.T, 512, "f32", device="cuda", seed=2)
    worst, counts = run_lora_case(tab, pool, x, y0, "f32", 2.0, all_tokens)
    print(f"  lora worst rel err {worst:.2e} counts {counts}")
    assert counts[2] == (520 if all_tokens else 512)
    dp = wl.direft_pool(4, 4, 512, "f32", device="cuda", seed=0)
    worst, counts = run_direft_case(tab, dp, x, "f32", 0.5, all_tokens)
    print(f"  direft worst rel err {worst:.2e} counts {counts}")


# ---------------------------------------------------------------------------------------
# bf16: every kernel variant x rank x mode on a mixed batch with ragged tiles
# ---------------------------------------------------------------------------------------
LORA_CASES = [
    # (variant, rank, d_in, d_out, waves, rowblocks)
    (VARIANT_ROW, 1, 256, 128, 0, 0), (VARIANT_ROW, 6, 264, 136, 0, 0), (VARIANT_ROW, 16, 512, 256, 0, 0),
    (VARIANT_ROW, 12, 128, 520, 0, 0), (VARIANT_ROW, 100, 128, 64, 0, 0),
    (VARIANT_VALU, 1, 1024, 512, 0, 0), (VARIANT_VALU, 2, 520, 264, 2, 0), (VARIANT_VALU, 3, 512, 1032, 1, 0),
    (VARIANT_VALU, 4, 1024, 256, 0, 0), (VARIANT_VALU, 5, 136, 128, 0, 0), (VARIANT_VALU, 7, 256, 520, 2, 0),
    (VARIANT_VALU, 8, 1024, 1024, 0, 0),
    (VARIANT_MFMA, 4, 512, 512, 4, 1), (VARIANT_MFMA, 8, 1024, 520, 2, 1), (VARIANT_MFMA, 16, 1024, 1024, 8, 1),
    (VARIANT_MFMA, 16, 520, 264, 4, 2), (VARIANT_MFMA, 32, 512, 1024, 2, 2), (VARIANT_MFMA, 64, 1024, 512, 4, 2),
    (VARIANT_MFMA, 64, 264, 136, 8, 1), (VARIANT_MFMA, 128, 256, 256, 4, 1), (VARIANT_MFMA, 24, 512, 256, 8, 2),
    (VARIANT_MFMA, 20, 136, 72, 2, 2), (VARIANT_MFMA, 128, 128, 136, 2, 2), (VARIANT_MFMA, 16, 40, 24, 4, 1),
    (VARIANT_MFMA, 16, 4096, 1024, 0, 0), (VARIANT_MFMA, 32, 96, 4104, 0, 0),
    # row-split shape, factors shared through LDS (rank > 16, widths multiples of 128)
    (VARIANT_WIDE, 32, 512, 1024, 4, 1), (VARIANT_WIDE, 32, 512, 1024, 4, 2), (VARIANT_WIDE, 64, 1024, 512, 8, 1),
    (VARIANT_WIDE, 64, 256, 384, 4, 2), (VARIANT_WIDE, 128, 256, 256, 4, 1), (VARIANT_WIDE, 128, 128, 256, 0, 0),
    (VARIANT_WIDE, 24, 512, 256, 4, 2), (VARIANT_WIDE, 40, 384, 640, 8, 1), (VARIANT_WIDE, 20, 128, 128, 4, 1),
    (VARIANT_WIDE, 32, 520, 256, 0, 0),
    (VARIANT_AUTO, 1, 2048, 512, 0, 0), (VARIANT_AUTO, 8, 512, 2048, 0, 0), (VARIANT_AUTO, 16, 2048, 2048, 0, 0),
    (VARIANT_AUTO, 9, 256, 256, 0, 0), (VARIANT_AUTO, 64, 1024, 1024, 0, 0),
]


_VNAME = {0: "auto", 1: "rowk", 2: "valu", 3: "mfma", 4: "wide"}


@pytest.mark.parametrize("variant,rank,d_in,d_out,waves,rowblocks", LORA_CASES,
                         ids=[f"{_VNAME[c[0]]}-r{c[1]}-{c[2]}x{c[3]}-w{c[4]}-mb{c[5]}" for c in LORA_CASES])
def test_bf16_lora_variants(variant, rank, d_in, d_out, waves, rowblocks):
    from parity_util import run_lora_case
    N = 5
    tab = _mixed_table(rank * 1000 + d_in, N)
    pool = wl.lora_pool(N, rank, d_in, d_out, "bf16", device="cuda", seed=rank)
    x = wl.activations(tab.T, d_in, "bf16", device="cuda", seed=11)
    y0 = wl.activations(tab.T, d_out, "bf16", device="cuda", seed=12)
    for all_tokens in (False, True):
        _set(variant, waves, rowblocks)
        worst, counts = run_lora_case(tab, pool, x, y0, "bf16", 2.0, all_tokens, pad_cols=8 if rank % 2 else 0,
                                      perm=[3, 0, 4, 1, 2])
        print(f"  all_tokens={all_tokens} worst rel err {worst:.2e} counts {counts}")


DIREFT_CASES = [
    (VARIANT_ROW, 4, 256, 0, 0), (VARIANT_ROW, 7, 136, 0, 0),
    (VARIANT_VALU, 1, 512, 0, 0), (VARIANT_VALU, 4, 1032, 2, 0), (VARIANT_VALU, 8, 512, 1, 0),
    (VARIANT_MFMA, 8, 1024, 4, 1), (VARIANT_MFMA, 16, 520, 2, 2), (VARIANT_MFMA, 32, 2048, 8, 2),
    (VARIANT_MFMA, 64, 256, 4, 1), (VARIANT_AUTO, 16, 4096, 0, 0), (VARIANT_AUTO, 2, 1024, 0, 0),
    # tile held in registers (automatic shape): 16 and 32 steps per wavefront, ragged widths
    (VARIANT_MFMA, 16, 4096, 0, 2), (VARIANT_MFMA, 8, 520, 0, 0), (VARIANT_MFMA, 32, 8192, 0, 0),
    (VARIANT_MFMA, 64, 4104, 0, 0), (VARIANT_MFMA, 16, 8200, 0, 0), (VARIANT_MFMA, 64, 8192, 0, 0),
    (VARIANT_MFMA, 128, 1024, 0, 0), (VARIANT_MFMA, 32, 16384, 0, 0),
    (VARIANT_WIDE, 32, 2048, 4, 2), (VARIANT_WIDE, 64, 1024, 8, 1), (VARIANT_WIDE, 20, 512, 4, 1), (VARIANT_WIDE, 128, 256, 4, 2),
    # vector-ALU kernel with its rows held in registers (automatic shape up to 4096 columns): full
    # and ragged vector counts per lane; one column group past the limit takes the streamed shape
    (VARIANT_AUTO, 2, 4096, 0, 0), (VARIANT_AUTO, 3, 264, 0, 0), (VARIANT_AUTO, 6, 2056, 0, 0), (VARIANT_AUTO, 7, 8, 0, 0),
    (VARIANT_AUTO, 1, 4088, 0, 0), (VARIANT_AUTO, 5, 4104, 0, 0), (VARIANT_VALU, 3, 4096, 4, 0),
]


@pytest.mark.parametrize("variant,rank,d,waves,rowblocks", DIREFT_CASES,
                         ids=[f"{_VNAME[c[0]]}-r{c[1]}-d{c[2]}-w{c[3]}-mb{c[4]}" for c in DIREFT_CASES])
def test_bf16_direft_variants(variant, rank, d, waves, rowblocks):
    from parity_util import run_direft_case
    N = 5
    tab = _mixed_table(rank * 77 + d, N, max_len=(40 if d > 4200 else 200) if d >= 2048 else 300, n_prompts=3 if d > 4200 else 6)
    pool = wl.direft_pool(N, rank, d, "bf16", device="cuda", seed=rank)
    h = wl.activations(tab.T, d, "bf16", device="cuda", seed=13)
    for all_tokens, scale, bias in ((False, 1.0, True), (True, 1.0 / np.sqrt(rank), True), (False, 0.75, False)):
        _set(variant, waves, rowblocks)
        worst, counts = run_direft_case(tab, pool, h, "bf16", scale, all_tokens, pad_cols=8, perm=[2, 4, 0, 3, 1],
                                        bias=bias)
        print(f"  all_tokens={all_tokens} bias={bias} worst rel err {worst:.2e} counts {counts}")


@pytest.mark.parametrize("rank", [5, 6, 7, 9, 10, 11, 13, 14, 15])
def test_ranks_that_are_not_multiples_of_four_on_the_matrix_core_kernel(rank):
    """bf16 ranks 5..15 other than 8 and 12 take the column-split MFMA kernel's any-rank shape (nothing
    padded in memory): LoRA on ragged widths, DiReFT with the tile held in registers (d <= 8192) and
    streamed (d > 8192), with and without bias, both modes, small-batch shape included."""
    from parity_util import run_direft_case, run_lora_case
    N = 5
    shapes = [(512, 1024), (1000, 264), (136, 4096)][rank % 3:][:2]
    for d_in, d_out in shapes:
        for n_prompts, max_len in ((6, 300), (2, 60)):            # a large batch and one of the small-batch shape
            tab = _mixed_table(rank * 13 + d_in + n_prompts, N, n_prompts=n_prompts, max_len=max_len)
            pool = wl.lora_pool(N, rank, d_in, d_out, "bf16", device="cuda", seed=rank)
            x = wl.activations(tab.T, d_in, "bf16", device="cuda", seed=11)
            y0 = wl.activations(tab.T, d_out, "bf16", device="cuda", seed=12)
            for all_tokens in (False, True):
                _set()
                worst, counts = run_lora_case(tab, pool, x, y0, "bf16", 2.0, all_tokens, pad_cols=8, perm=[2, 4, 0, 3, 1])
                print(f"  lora r={rank} {d_in}->{d_out} T={tab.T} all_tokens={all_tokens} worst {worst:.2e}")
    for d in ((4096, 520) if rank % 2 else (8192, 264)) + ((16384 + 8,) if rank in (7, 10) else ()):
        tab = _mixed_table(rank * 17 + d, N, max_len=40 if d > 4200 else 200, n_prompts=3 if d > 4200 else 6)
        pool = wl.direft_pool(N, rank, d, "bf16", device="cuda", seed=rank + 2)
        h = wl.activations(tab.T, d, "bf16", device="cuda", seed=13)
        for all_tokens, scale, bias in ((False, 1.0, True), (True, 1.0 / np.sqrt(rank), False)):
            _set()
            worst, counts = run_direft_case(tab, pool, h, "bf16", scale, all_tokens, pad_cols=8, bias=bias)
            print(f"  direft r={rank} d={d} all_tokens={all_tokens} bias={bias} worst {worst:.2e}")


@pytest.mark.parametrize("rank", [17, 18, 19, 21, 23, 30, 37, 50, 63, 65, 100, 127])
def test_ranks_above_16_that_are_not_multiples_of_four(rank):
    """bf16 ranks above 16 that are not multiples of 4 take the row-split MFMA kernel's any-rank form when
    every width is a multiple of 128 (chunks; the gathered tiles of the all-token mode go to the per-row
    kernel), and the per-row kernels otherwise: LoRA and DiReFT (with and without bias, one call for
    several layers), both modes, small and large batches."""
    from parity_util import run_direft_case, run_direft_layers_case, run_lora_case
    N = 4
    for (d_in, d_out), (n_prompts, max_len) in (((256, 384), (6, 300)), ((128, 128), (2, 50)), ((384, 264), (4, 200))):
        tab = _mixed_table(rank * 11 + d_in, N, n_prompts=n_prompts, max_len=max_len)
        pool = wl.lora_pool(N, rank, d_in, d_out, "bf16", device="cuda", seed=rank)
        x = wl.activations(tab.T, d_in, "bf16", device="cuda", seed=21)
        y0 = wl.activations(tab.T, d_out, "bf16", device="cuda", seed=22)
        for all_tokens in (False, True):
            _set()
            worst, counts = run_lora_case(tab, pool, x, y0, "bf16", 2.0, all_tokens, pad_cols=8)
            print(f"  lora r={rank} {d_in}->{d_out} T={tab.T} all_tokens={all_tokens} worst {worst:.2e}")
    for d in (512, 136):
        tab = _mixed_table(rank * 19 + d, N, max_len=260)
        pool = wl.direft_pool(N, rank, d, "bf16", device="cuda", seed=rank + 3)
        h = wl.activations(tab.T, d, "bf16", device="cuda", seed=23)
        for all_tokens, scale, bias in ((False, 1.0, True), (True, 1.0 / np.sqrt(rank), False)):
            _set()
            worst, counts = run_direft_case(tab, pool, h, "bf16", scale, all_tokens, pad_cols=8, bias=bias)
            print(f"  direft r={rank} d={d} all_tokens={all_tokens} bias={bias} worst {worst:.2e}")
    if rank in (19, 37, 65):
        tab = _mixed_table(rank * 23, N, max_len=150)
        pools = [wl.direft_pool(N, rank, 256, "bf16", device="cuda", seed=300 + l) for l in range(3)]
        h0s = [wl.activations(tab.T, 256, "bf16", device="cuda", seed=310 + l) for l in range(3)]
        _set()
        worst = run_direft_layers_case(tab, pools, h0s, "bf16", 0.5, False, [True, False, True], pad_cols=8)
        print(f"  direft layers r={rank} worst {worst:.2e}")


@pytest.mark.parametrize("resident", [3])
@pytest.mark.parametrize("rank,d", [(32, 8192), (32, 4096), (32, 1160), (20, 8192), (24, 2048), (32, 16384), (28, 520)])
def test_partially_resident_in_place_tiles(resident, rank, d):
    """In place at rank 32..64: a wavefront keeps some of its units in registers between the sweeps and
    streams the others twice (or keeps all of them when the row is narrow enough); ragged widths
    put the 32-column tail steps on top."""
    from parity_util import run_direft_case
    N = 5
    tab = _mixed_table(rank * 31 + d + resident, N, max_len=40 if d > 4200 else 150, n_prompts=3 if d > 4200 else 6)
    pool = wl.direft_pool(N, rank, d, "bf16", device="cuda", seed=rank + 1)
    h = wl.activations(tab.T, d, "bf16", device="cuda", seed=14)
    for all_tokens, scale, bias in ((False, 1.0, True), (True, 1.0 / np.sqrt(rank), False)):
        _set(0, 0, 0, resident=resident)
        worst, counts = run_direft_case(tab, pool, h, "bf16", scale, all_tokens, pad_cols=8, bias=bias)
        print(f"  resident={resident} r={rank} d={d} all_tokens={all_tokens} worst rel err {worst:.2e} counts {counts}")


@pytest.mark.parametrize("rank,d", [(3, 132), (8, 64), (17, 260)])
def test_fp32_generic_path(rank, d):
    from parity_util import run_direft_case, run_lora_case
    N = 4
    tab = _mixed_table(rank + d, N, max_len=150)
    pool = wl.lora_pool(N, rank, d, d + 4, "f32", device="cuda", seed=rank)
    x = wl.activations(tab.T, d, "f32", device="cuda", seed=21)
    y0 = wl.activations(tab.T, d + 4, "f32", device="cuda", seed=22)
    worst, _ = run_lora_case(tab, pool, x, y0, "f32", 2.0, True, pad_cols=4)
    print(f"  lora worst rel err {worst:.2e}")
    dp = wl.direft_pool(N, rank, d, "f32", device="cuda", seed=rank)
    worst, _ = run_direft_case(tab, dp, x, "f32", 1.0, False)
    print(f"  direft worst rel err {worst:.2e}")


# ---------------------------------------------------------------------------------------
# the five batch structures, shrunk so that the oracle finishes in seconds
# ---------------------------------------------------------------------------------------
@pytest.mark.parametrize("config,scale_down,rank,d_in,d_out", [
    ("llama8b_lora", 8, 16, 1024, 1024), ("llama8b_lora", 8, 1, 1024, 256),
    ("llama70b_lora", 16, 64, 1024, 512), ("skewed70b", 32, 32, 512, 512),
])
def test_scaled_down_config_lora(config, scale_down, rank, d_in, d_out):
    from parity_util import run_lora_case
    cfg = wl.CONFIGS[config]
    tab = wl.make_segments(config, seed=0, scale_down=scale_down)
    pool = wl.lora_pool(cfg["N"], rank, d_in, d_out, "bf16", device="cuda", seed=3)
    x = wl.activations(tab.T, d_in, "bf16", device="cuda", seed=31)
    y0 = wl.activations(tab.T, d_out, "bf16", device="cuda", seed=32)
    rows = wl.sample_rows(tab, 3, max_rows=1500)
    for all_tokens in (False, True):
        worst, counts = run_lora_case(tab, pool, x, y0, "bf16", cfg["lora_scale"], all_tokens, rows=rows,
                                      reuse_schedule=all_tokens)
        print(f"  T={tab.T} S={tab.S} all_tokens={all_tokens} worst {worst:.2e} counts {counts}")


@pytest.mark.parametrize("config,scale_down,rank,d", [("llama8b_direft", 8, 8, 1024), ("skewed70b", 32, 32, 1024)])
def test_scaled_down_config_direft(config, scale_down, rank, d):
    from parity_util import run_direft_case
    cfg = wl.CONFIGS[config]
    tab = wl.make_segments(config, seed=0, scale_down=scale_down)
    pool = wl.direft_pool(cfg["N"], rank, d, "bf16", device="cuda", seed=4)
    h = wl.activations(tab.T, d, "bf16", device="cuda", seed=33)
    rows = wl.sample_rows(tab, 3, max_rows=1500)
    for all_tokens in (False, True):
        worst, counts = run_direft_case(tab, pool, h, "bf16", 1.0, all_tokens, rows=rows, reuse_schedule=not all_tokens)
        print(f"  T={tab.T} S={tab.S} all_tokens={all_tokens} worst {worst:.2e} counts {counts}")


# ---------------------------------------------------------------------------------------
# scheduler and degenerate cases
# ---------------------------------------------------------------------------------------
def test_schedule_counts_match_the_tables():
    from parity_util import dev_tables
    rng = np.random.Generator(np.random.PCG64(5))
    for trial in range(8):
        N = 7 if trial % 2 == 0 else 5000          # above 4096 slots the short rows are not sorted
        S = int(rng.integers(1, 3000))
        tab = wl.random_segments(rng, S, N + 2, int(rng.integers(1, 600)))
        if tab.T == 0:
            continue
        ss, sa, sp = dev_tables(tab)
        ws = preft.new_workspace(tab.T, tab.S)
        for mode in (preft.PREFT_PREFILL_ONLY, preft.PREFT_ALL_TOKENS):
            ws.fill_(0xAB)
            preft.preft_schedule(ws, ss, sa, sp, tab.T, N, mode)
            got = preft.preft_schedule_counts(ws)
            has = (tab.seg_adapter >= 0) & (tab.seg_adapter < N)
            n = np.where(has, tab.seg_len if mode else np.minimum(tab.seg_prefill_len, tab.seg_len), 0)
            want = (int(np.sum((n[n > 4] + 127) // 128)), int(np.sum(n[n <= 4])), int(n.sum()))
            assert got == want
            # the lists cover exactly the active rows, each once
            hdr = ws[:64].view(torch.int32).cpu().numpy()
            chunks = ws[64:64 + 16 * hdr[0]].view(torch.int32).view(-1, 4).cpu().numpy()
            cap = (preft.preft_workspace_bytes(tab.T, tab.S) - 64)
            chunk_cap = tab.T // 128 + min(tab.S, tab.T // 5) + 1
            short_cap = min(4 * tab.S, tab.T) + 1
            g0 = 64 + 16 * chunk_cap
            s0 = g0 + 16 * short_cap
            gtiles = ws[g0:g0 + 16 * hdr[4]].view(torch.int32).view(-1, 4).cpu().numpy()
            shorts = ws[s0:s0 + 8 * hdr[1]].view(torch.int32).view(-1, 2).cpu().numpy()
            # gathered tiles partition the short-row list; a tile's rows share its adapter
            seen = np.zeros(len(shorts), dtype=np.int32)
            for a, first, cnt, _ in gtiles:
                assert 1 <= cnt <= 16
                assert np.all(shorts[first:first + cnt, 0] == a)
                seen[first:first + cnt] += 1
            assert np.all(seen == 1)
            # the launch grids are sized from these bounds
            if N <= 4096:
                assert np.all(np.diff(shorts[:, 0]) >= 0)                 # sorted by adapter
                partial = gtiles[gtiles[:, 2] < 16, 0]
                assert len(np.unique(partial)) == len(partial)            # one partial tile per adapter
                assert len(gtiles) <= min(short_cap, N + short_cap // 16 + 1)
            else:
                assert len(gtiles) <= min(short_cap, tab.S)
            covered = np.zeros(tab.T, dtype=np.int32)
            owner = np.full(tab.T, -1, dtype=np.int32)
            for a, row0, nrows, seg in chunks:
                assert 1 <= nrows <= 128
                covered[row0:row0 + nrows] += 1
                owner[row0:row0 + nrows] = a
            for a, row in shorts:
                covered[row] += 1
                owner[row] = a
            from oracle import preft_oracle as ora
            want_owner = ora.positions(tab.T, tab.seg_start, tab.seg_adapter, tab.seg_prefill_len, N,
                                       ora.ALL_POSITIONS if mode else ora.PROMPT_ONLY)
            assert np.array_equal(covered, (want_owner >= 0).astype(np.int32))
            assert np.array_equal(owner, want_owner)
            assert cap > 0


def test_all_decode_batch_is_skipped_in_prefill_only_mode():
    from parity_util import bits, dev_tables, lora_pools_to_device
    N, S, d = 8, 300, 512
    rng = np.random.Generator(np.random.PCG64(6))
    tab = wl.from_lengths(np.ones(S), rng.integers(0, N, size=S), np.zeros(S))
    pool = wl.lora_pool(N, 16, d, d, "bf16", device="cuda", seed=6)
    x = wl.activations(S, d, "bf16", device="cuda", seed=61)
    y0 = wl.activations(S, d, "bf16", device="cuda", seed=62)
    y = y0.clone()
    ss, sa, sp = dev_tables(tab)
    Ap, Bp, keep = lora_pools_to_device(pool)
    ws = preft.new_workspace(tab.T, tab.S)
    preft.preft_lora_apply(y, x, ss, sa, sp, Ap, Bp, 16, 2.0, preft.PREFT_PREFILL_ONLY, ws)
    torch.cuda.synchronize()
    assert preft.preft_schedule_counts(ws) == (0, 0, 0)
    assert torch.equal(bits(y), bits(y0))
    preft.preft_lora_apply(y, x, ss, sa, sp, Ap, Bp, 16, 2.0, preft.PREFT_ALL_TOKENS, ws)
    torch.cuda.synchronize()
    assert preft.preft_schedule_counts(ws) == (0, S, S)
    assert not torch.equal(bits(y), bits(y0))


def test_zero_adapters_and_zero_scale_leave_values_unchanged():
    from parity_util import dev_tables, lora_pools_to_device
    N, d, r = 3, 256, 16
    tab = _mixed_table(9, N)
    pool = wl.lora_pool(N, r, d, d, "bf16", device="cuda", seed=9)
    zero_B = wl.LoraPool(pool.A, torch.zeros_like(pool.B))
    x = wl.activations(tab.T, d, "bf16", device="cuda", seed=91)
    y0 = wl.activations(tab.T, d, "bf16", device="cuda", seed=92)
    ss, sa, sp = dev_tables(tab)
    ws = preft.new_workspace(tab.T, tab.S)
    for p, scale in ((zero_B, 2.0), (pool, 0.0)):
        Ap, Bp, keep = lora_pools_to_device(p)
        y = y0.clone()
        preft.preft_lora_apply(y, x, ss, sa, sp, Ap, Bp, r, scale, preft.PREFT_ALL_TOKENS, ws)
        torch.cuda.synchronize()
        assert torch.equal(y, y0)     # value equality (a zero delta may rewrite -0.0 as itself)


def test_results_are_deterministic_and_schedule_reuse_matches():
    from parity_util import dev_tables, lora_pools_to_device
    N, d, r = 6, 1024, 16
    tab = wl.make_segments("llama8b_lora", seed=1, scale_down=8)
    pool = wl.lora_pool(64, r, d, d, "bf16", device="cuda", seed=10)
    x = wl.activations(tab.T, d, "bf16", device="cuda", seed=101)
    y0 = wl.activations(tab.T, d, "bf16", device="cuda", seed=102)
    ss, sa, sp = dev_tables(tab)
    Ap, Bp, keep = lora_pools_to_device(pool)
    ws = preft.new_workspace(tab.T, tab.S)
    outs = []
    for i in range(3):
        y = y0.clone()
        mode = preft.PREFT_PREFILL_ONLY
        if i == 2:
            mode |= preft.PREFT_SCHEDULE_READY        # schedule left in ws by the previous call
        preft.preft_lora_apply(y, x, ss, sa, sp, Ap, Bp, r, 2.0, mode, ws)
        torch.cuda.synchronize()
        outs.append(y)
    assert torch.equal(outs[0], outs[1]) and torch.equal(outs[0], outs[2])


@pytest.mark.parametrize("variant,dtype,rank,d", [(0, "bf16", 16, 1024), (0, "bf16", 8, 4096), (0, "bf16", 32, 512),
                                                  (0, "bf16", 64, 256), (VARIANT_MFMA, "bf16", 32, 264), (0, "bf16", 3, 520),
                                                  (0, "bf16", 7, 256), (VARIANT_ROW, "bf16", 12, 264), (0, "f32", 4, 132)])
def test_null_entries_of_the_bias_table_mean_no_bias_for_that_adapter(variant, dtype, rank, d):
    """Eq. 3 with b = 0 for single adapters: a null entry in b_pool (the oracle gets no bias for them)."""
    from parity_util import run_direft_case
    N = 5
    _set(variant)
    tab = _mixed_table(1300 + rank, N)
    pool = wl.direft_pool(N, rank, d, dtype, device="cuda", seed=131)
    h = wl.activations(tab.T, d, dtype, device="cuda", seed=132)
    for all_tokens in (False, True):
        worst, _ = run_direft_case(tab, pool, h, dtype, 0.5, all_tokens, pad_cols=8, null_bias=(0, 3))
        print(f"  variant={variant} {dtype} r={rank} d={d} all_tokens={all_tokens} worst {worst:.2e}")
    # the bias matters in this test: with every entry present the result differs on adapter 0's rows
    from parity_util import dev_tables, direft_pools_to_device
    ss, sa, sp = dev_tables(tab)
    outs = []
    for nulls in ((), (0, 3)):
        W1p, W2tp, bp, keep = direft_pools_to_device(pool, None, True, nulls)
        hh = h.clone()
        preft.preft_direft_apply(hh, ss, sa, sp, W1p, W2tp, bp, rank, 0.5, preft.PREFT_ALL_TOKENS,
                                 preft.new_workspace(tab.T, tab.S))
        torch.cuda.synchronize()
        outs.append(hh)
    assert not torch.equal(outs[0], outs[1])


@pytest.mark.parametrize("N", [3, 5000])          # short rows sorted by adapter / listed per segment
def test_overlapping_segments_stay_inside_the_buffers(N):
    """Malformed tables: offsets that go back and forth name the same rows many times, so the lists of
    the schedule would outgrow the capacities computed from T and S.  The result is unspecified, but
    every access must stay inside the buffers: guard rows and row padding come back untouched and
    the schedule's counters stay within their capacities."""
    from parity_util import GUARD_ROWS, check_guards, padded
    d, r = 256, 16
    for T, starts in ((4, [0, 4] * 40 + [0, 4]), (300, [0, 300, 0, 3, 100, 1, 2, 300] * 6 + [300]),
                      (64, list(np.tile([0, 2, 64, 1], 30)) + [64])):
        starts = np.asarray(starts, dtype=np.int32)
        S = len(starts) - 1
        tab = wl.SegmentTable(starts, (np.arange(S) % min(N, 7)).astype(np.int32), np.full(S, 1000, dtype=np.int32))
        ss, sa, sp = (torch.from_numpy(a.copy()).cuda() for a in (tab.seg_start, tab.seg_adapter, tab.seg_prefill_len))
        pool = wl.lora_pool(7, r, d, d, "bf16", device="cuda", seed=3)
        tabA = preft.pointer_table([pool.A[i].contiguous() for i in range(7)])
        tabB = preft.pointer_table([pool.B[i].contiguous() for i in range(7)])
        if N > 7:                                   # a large pool whose used slots are the first seven
            tabA = torch.cat([tabA, torch.zeros(N - 7, dtype=torch.int64, device="cuda")])
            tabB = torch.cat([tabB, torch.zeros(N - 7, dtype=torch.int64, device="cuda")])
        else:
            tabA, tabB = tabA[:N].contiguous(), tabB[:N].contiguous()
            tab.seg_adapter[:] = tab.seg_adapter % N
            sa = torch.from_numpy(tab.seg_adapter.copy()).cuda()
        x = wl.activations(T, d, "bf16", device="cuda", seed=31)
        ws = preft.new_workspace(T, S)
        cap_short = min(4 * S, T) + 1
        for variant in (0, VARIANT_ROW, VARIANT_VALU):
            _set(variant)
            for mode in (preft.PREFT_PREFILL_ONLY, preft.PREFT_ALL_TOKENS):
                ybuf, y = padded(wl.activations(T, d, "bf16", device="cuda", seed=32), 8, 7.0)
                hbuf, h = padded(x, 8, 7.0)
                preft.preft_lora_apply(y, x, ss, sa, sp, tabA, tabB, r, 1.0, mode, ws)
                preft.preft_direft_apply(h, ss, sa, sp, tabA, tabB, None, r, 1.0, mode | preft.PREFT_SCHEDULE_READY, ws)
                torch.cuda.synchronize()
                counts = preft.preft_schedule_counts(ws)
                assert counts[1] <= cap_short, counts
                check_guards(ybuf, T, d, 7.0)
                check_guards(hbuf, T, d, 7.0)
                assert bool(torch.isfinite(y.float()).all())
        print(f"  N={N} T={T} S={S} counts {counts}")


def test_a_schedule_built_for_another_batch_is_refused_not_misread():
    """PREFT_SCHEDULE_READY with a workspace whose schedule was built for another position set, T, S
    or N: the apply call must do nothing, and preft_schedule_counts must say so."""
    from parity_util import bits, dev_tables, direft_pools_to_device, lora_pools_to_device
    N, d, r = 4, 512, 16
    tab = _mixed_table(77, N)
    ss, sa, sp = dev_tables(tab)
    pool = wl.lora_pool(N, r, d, d, "bf16", device="cuda", seed=7)
    dp = wl.direft_pool(N, r, d, "bf16", device="cuda", seed=8)
    Ap, Bp, keep = lora_pools_to_device(pool)
    W1p, W2tp, bp, keep2 = direft_pools_to_device(dp)
    x = wl.activations(tab.T, d, "bf16", device="cuda", seed=71)
    y0 = wl.activations(tab.T, d, "bf16", device="cuda", seed=72)
    ws = preft.new_workspace(tab.T, tab.S)
    ready = preft.PREFT_SCHEDULE_READY
    for variant in (0, VARIANT_ROW, VARIANT_WIDE):
        _set(variant)
        # another position set
        preft.preft_schedule(ws, ss, sa, sp, tab.T, N, preft.PREFT_ALL_TOKENS)
        y, h = y0.clone(), x.clone()
        preft.preft_lora_apply(y, x, ss, sa, sp, Ap, Bp, r, 2.0, preft.PREFT_PREFILL_ONLY | ready, ws)
        preft.preft_direft_apply(h, ss, sa, sp, W1p, W2tp, bp, r, 1.0, preft.PREFT_PREFILL_ONLY | ready, ws)
        torch.cuda.synchronize()
        assert torch.equal(bits(y), bits(y0)) and torch.equal(bits(h), bits(x))
        with pytest.raises(preft.PreftError) as e:
            preft.preft_schedule_counts(ws)
        assert e.value.code == preft.PREFT_ESCHEDULE
        # another pool size (N), another row count (T: one row fewer, the tables still describe tab.T rows)
        preft.preft_schedule(ws, ss, sa, sp, tab.T, N, preft.PREFT_PREFILL_ONLY)
        assert preft.preft_schedule_counts(ws)[2] > 0                      # a fresh schedule clears the mark
        preft.preft_lora_apply(y, x, ss, sa, sp, Ap[:N - 1].contiguous(), Bp[:N - 1].contiguous(), r, 2.0, ready, ws)
        torch.cuda.synchronize()
        assert torch.equal(bits(y), bits(y0))
        with pytest.raises(preft.PreftError):
            preft.preft_schedule_counts(ws)
        preft.preft_schedule(ws, ss, sa, sp, tab.T, N, preft.PREFT_PREFILL_ONLY)
        preft.preft_direft_apply(h[:-1], ss, sa, sp, W1p, W2tp, bp, r, 1.0, ready, ws)
        torch.cuda.synchronize()
        assert torch.equal(bits(h), bits(x))
        with pytest.raises(preft.PreftError):
            preft.preft_schedule_counts(ws)
        # and the matching call still works
        preft.preft_schedule(ws, ss, sa, sp, tab.T, N, preft.PREFT_PREFILL_ONLY)
        preft.preft_lora_apply(y, x, ss, sa, sp, Ap, Bp, r, 2.0, ready, ws)
        torch.cuda.synchronize()
        assert not torch.equal(bits(y), bits(y0))
        preft.preft_schedule_counts(ws)


def test_gpu_side_error_codes():
    N, d = 2, 64
    tab = wl.from_lengths([8], [0], [8])
    from parity_util import dev_tables, lora_pools_to_device
    ss, sa, sp = dev_tables(tab)
    pool = wl.lora_pool(N, 4, d, d, "bf16", device="cuda", seed=1)
    Ap, Bp, keep = lora_pools_to_device(pool)
    x = wl.activations(8, d, "bf16", device="cuda", seed=1)
    y = wl.activations(8, d, "bf16", device="cuda", seed=2)
    ws = preft.new_workspace(8, 1)
    with pytest.raises(preft.PreftError) as e:
        preft.preft_lora_apply(y, y, ss, sa, sp, Ap, Bp, 4, 1.0, 0, ws)          # x aliases y
    assert e.value.code == -1
    with pytest.raises(preft.PreftError) as e:
        preft.preft_lora_apply(y, x, ss, sa, sp, Ap, Bp, 4, 1.0, 0, ws[:32])     # workspace too small
    assert e.value.code == -4
    with pytest.raises(preft.PreftError) as e:
        preft.preft_lora_apply(y[:, 4:], x[:, 4:], ss, sa, sp, Ap, Bp, 4, 1.0, 0, ws)   # misaligned base
    assert e.value.code == -3


def test_calls_are_graph_capturable_and_read_their_tables_on_the_device():
    """The header promises: no allocation, no synchronisation, launch shapes from host-visible sizes
    only.  Capture schedule + LoRA + DiReFT into one HIP graph, then replay it with the segment
    tables rewritten in place between replays (same T and S): every replay must match an eager
    run on the tables of that moment."""
    from parity_util import bits, dev_tables, direft_pools_to_device, lora_pools_to_device
    N, d, r = 6, 512, 16
    rng = np.random.Generator(np.random.PCG64(77))
    lens = np.array([300, 1, 129, 1, 1, 64, 200, 1, 5, 3])
    tabs = []
    for k in range(3):
        ids = rng.integers(-1, N, size=len(lens))
        pre = np.where(rng.random(len(lens)) < 0.5, lens, (lens * rng.random(len(lens))).astype(np.int64))
        tabs.append(wl.from_lengths(lens, ids, pre))
    T, S = tabs[0].T, tabs[0].S
    pool = wl.lora_pool(N, r, d, d, "bf16", device="cuda", seed=7)
    dpool = wl.direft_pool(N, r, d, "bf16", device="cuda", seed=8)
    Ap, Bp, keep1 = lora_pools_to_device(pool)
    W1p, W2tp, bp, keep2 = direft_pools_to_device(dpool)
    x = wl.activations(T, d, "bf16", device="cuda", seed=71)
    y0 = wl.activations(T, d, "bf16", device="cuda", seed=72)
    ss, sa, sp = dev_tables(tabs[0])
    ws = preft.new_workspace(T, S)
    y = y0.clone()
    mode = preft.PREFT_PREFILL_ONLY

    def body():
        y.copy_(y0)
        preft.preft_schedule(ws, ss, sa, sp, T, N, mode)
        preft.preft_lora_apply(y, x, ss, sa, sp, Ap, Bp, r, 2.0, mode | preft.PREFT_SCHEDULE_READY, ws)
        preft.preft_direft_apply(y, ss, sa, sp, W1p, W2tp, bp, r, 0.5, mode | preft.PREFT_SCHEDULE_READY, ws)

    body()                                        # warm-up outside capture
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        body()
    for k in (1, 2, 0, 1):
        sa.copy_(torch.from_numpy(tabs[k].seg_adapter.copy()))      # same buffers, new contents
        sp.copy_(torch.from_numpy(tabs[k].seg_prefill_len.copy()))
        graph.replay()
        torch.cuda.synchronize()
        got = y.clone()
        body()                                    # eager run on the same tables
        torch.cuda.synchronize()
        assert torch.equal(bits(got), bits(y)), f"graph replay differs from the eager run (table {k})"
        assert not torch.equal(bits(got), bits(y0))


def test_packed_and_many_layer_calls_are_graph_capturable():
    """The same promise for the packed LoRA call and the many-layer DiReFT call: a captured graph,
    replayed with the tables rewritten in place, matches the eager run every time."""
    from parity_util import bits, dev_tables, direft_pools_to_device, lora_pools_to_device
    N, d, r, L = 5, 512, 8, 3
    rng = np.random.Generator(np.random.PCG64(78))
    lens = np.array([200, 1, 1, 77, 1, 140, 2, 1, 33])
    tabs = []
    for k in range(3):
        ids = rng.integers(-1, N, size=len(lens))
        pre = np.where(rng.random(len(lens)) < 0.5, lens, (lens * rng.random(len(lens))).astype(np.int64))
        tabs.append(wl.from_lengths(lens, ids, pre))
    T, S = tabs[0].T, tabs[0].S
    pools = [lora_pools_to_device(wl.lora_pool(N, r, d, n, "bf16", device="cuda", seed=80 + i)) for i, n in enumerate((256, 384))]
    dev = [direft_pools_to_device(wl.direft_pool(N, r, d, "bf16", device="cuda", seed=85 + l)) for l in range(L)]
    table = lambda ptrs: torch.tensor(ptrs, dtype=torch.int64, device="cuda")
    W1s, W2s, bs = (table([m[i].data_ptr() for m in dev]) for i in range(3))
    x = wl.activations(T, d, "bf16", device="cuda", seed=86)
    y0 = wl.activations(T, 640, "bf16", device="cuda", seed=87)
    h0s = [wl.activations(T, d, "bf16", device="cuda", seed=88 + l) for l in range(L)]
    y, hs = y0.clone(), [h.clone() for h in h0s]
    h_tab = preft.pointer_table(hs)
    ss, sa, sp = dev_tables(tabs[0])
    ws = preft.new_workspace(T, S)
    mode = preft.PREFT_ALL_TOKENS

    def body():
        y.copy_(y0)
        for h, h0 in zip(hs, h0s):
            h.copy_(h0)
        preft.preft_schedule(ws, ss, sa, sp, T, N, mode)
        ready = mode | preft.PREFT_SCHEDULE_READY
        preft.preft_lora_apply_packed([y[:, :256], y[:, 256:]], x, ss, sa, sp, [p[0] for p in pools],
                                      [p[1] for p in pools], r, 2.0, ready, ws)
        preft.preft_direft_apply_layers(hs, h_tab, ss, sa, sp, W1s, W2s, bs, N, r, 0.5, ready, ws)

    body()
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        body()
    for k in (2, 0, 1, 2):
        sa.copy_(torch.from_numpy(tabs[k].seg_adapter.copy()))
        sp.copy_(torch.from_numpy(tabs[k].seg_prefill_len.copy()))
        graph.replay()
        torch.cuda.synchronize()
        got = [y.clone()] + [h.clone() for h in hs]
        body()
        torch.cuda.synchronize()
        for a, b in zip(got, [y] + hs):
            assert torch.equal(bits(a), bits(b)), f"graph replay differs from the eager run (table {k})"
        assert not torch.equal(bits(got[0]), bits(y0)) and not torch.equal(bits(got[1]), bits(h0s[0]))


def test_fcfs_trace_steps_match_the_oracle():
    """Every engine step of a small first-come-first-served serving trace (App. E.1, E.3), in both
    modes: prompt steps mix whole prompts with decode rows, decode-only steps hold one row per
    request in flight."""
    from parity_util import run_direft_case, run_lora_case
    N, d, r = 3, 256, 8
    req = wl.request_stream(14, N, "uniform", l_max=40, seed=4)
    pool = wl.lora_pool(N, r, d, d, "bf16", device="cuda", seed=41)
    dpool = wl.direft_pool(N, r, d, "bf16", device="cuda", seed=42)
    x_all = wl.activations(4 * 40, d, "bf16", device="cuda", seed=43)
    y_all = wl.activations(4 * 40, d, "bf16", device="cuda", seed=44)
    steps = prompts = 0
    for tab, repeat in wl.fcfs_steps(req, 4):
        steps += repeat
        prompts += int((tab.seg_prefill_len > 0).sum())
        x, y0 = x_all[:tab.T].contiguous(), y_all[:tab.T].contiguous()
        for all_tokens in (False, True):
            _, counts = run_lora_case(tab, pool, x, y0, "bf16", 2.0, all_tokens)
            assert counts[2] == (tab.T if all_tokens else int(tab.seg_prefill_len.sum()))
            run_direft_case(tab, dpool, y0, "bf16", 1.0, all_tokens)
    assert prompts == 14 and steps > 14


# ---------------------------------------------------------------------------------------
# LoReFT (App. C.2) through its derived factors
# ---------------------------------------------------------------------------------------
def _loreft_weights(N, r, d, dtype, seed, spread):
    """R with orthonormal rows (before rounding to the storage type); W = R + spread * noise."""
    g = torch.Generator(device="cuda").manual_seed(seed)
    td = wl.torch_dtype(dtype)
    W, R, b = [], [], []
    for _ in range(N):
        q = torch.linalg.qr(torch.randn(d, r, generator=g, device="cuda", dtype=torch.float32))[0].t().contiguous()
        noise = torch.randn(r, d, generator=g, device="cuda", dtype=torch.float32) / d ** 0.5
        R.append(q.to(td))
        W.append((q + spread * noise).to(td))
        b.append(torch.randn(r, generator=g, device="cuda", dtype=torch.float32).to(td))
    return W, R, b


@pytest.mark.parametrize("dtype,r,d,spread", [("bf16", 4, 512, 1.0), ("bf16", 16, 1000, 1.0), ("bf16", 8, 4096, 0.05),
                                              ("bf16", 3, 264, 1.0), ("f32", 4, 512, 1.0), ("bf16", 64, 1024, 1.0)])
def test_loreft_matches_the_oracle(dtype, r, d, spread):
    from parity_util import run_loreft_case
    N = 5
    rng = np.random.Generator(np.random.PCG64(90 + r))
    tab = wl.random_segments(rng, 40, N + 1, 70)
    W, R, b = _loreft_weights(N, r, d, dtype, seed=91, spread=spread)
    h0 = wl.activations(tab.T, d, dtype, device="cuda", seed=92)
    for all_tokens in (False, True):
        worst = run_loreft_case(tab, W, R, b, h0, dtype, 1.0 / r ** 0.5, all_tokens, pad_cols=8)
        print(f"  loreft {dtype} r={r} d={d} all_tokens={all_tokens} worst {worst:.2e}")


def test_loreft_is_the_identity_at_its_initialisation():
    """W = R, b = 0 (zero-delta initialisation, App. C.1): the derived difference factor is exactly
    zero and every row keeps its bits."""
    from parity_util import bits, dev_tables
    N, r, d = 3, 8, 1024
    W, R, _ = _loreft_weights(N, r, d, "bf16", seed=93, spread=0.0)
    rng = np.random.Generator(np.random.PCG64(94))
    tab = wl.random_segments(rng, 20, N, 50)
    h0 = wl.activations(tab.T, d, "bf16", device="cuda", seed=95)
    h = h0.clone()
    D = [torch.empty_like(w) for w in W]
    Rt = [torch.empty((d, r), dtype=w.dtype, device="cuda") for w in W]
    for i in range(N):
        preft.preft_loreft_prepare(D[i], Rt[i], W[i], R[i])
    ss, sa, sp = dev_tables(tab)
    ws = preft.new_workspace(tab.T, tab.S)
    zero_b = [torch.zeros(r, dtype=torch.bfloat16, device="cuda") for _ in range(N)]
    preft.preft_loreft_apply(h, ss, sa, sp, preft.pointer_table(D), preft.pointer_table(Rt),
                             preft.pointer_table(zero_b), r, 0.7, preft.PREFT_ALL_TOKENS, ws)
    torch.cuda.synchronize()
    assert all(int(torch.count_nonzero(m)) == 0 for m in D)
    assert torch.equal(bits(h), bits(h0))


def test_loreft_prepare_rejects_bad_arguments():
    lib = preft.load_library()
    W = torch.zeros(4, 64, dtype=torch.bfloat16, device="cuda")
    R, D, Rt = torch.zeros_like(W), torch.zeros_like(W), torch.zeros(64, 4, dtype=torch.bfloat16, device="cuda")
    call = lambda D_, Rt_, W_, R_, d, r, dt: lib.preft_loreft_prepare(D_, Rt_, W_, R_, d, r, dt, None)
    assert call(D.data_ptr(), Rt.data_ptr(), W.data_ptr(), R.data_ptr(), 64, 4, preft.PREFT_BF16) == 0
    assert call(None, Rt.data_ptr(), W.data_ptr(), R.data_ptr(), 64, 4, preft.PREFT_BF16) == -1
    assert call(D.data_ptr(), Rt.data_ptr(), W.data_ptr(), R.data_ptr(), 64, 4, 7) == -1
    assert call(D.data_ptr(), Rt.data_ptr(), W.data_ptr(), R.data_ptr(), 64, 129, preft.PREFT_BF16) == -2
    assert call(D.data_ptr() + 2, Rt.data_ptr(), W.data_ptr(), R.data_ptr(), 64, 4, preft.PREFT_BF16) == -3
    assert call(W.data_ptr(), Rt.data_ptr(), W.data_ptr(), R.data_ptr(), 64, 4, preft.PREFT_BF16) == -1   # D aliases W
    torch.cuda.synchronize()


# ---------------------------------------------------------------------------------------
# packed projections: several LoRA outputs from one x
# ---------------------------------------------------------------------------------------
def _packed_case(dtype, r, d_in, d_outs, fused_buffer, seed, all_tokens, S=30, max_len=150, min_rows=0):
    from oracle import preft_oracle as ora
    from parity_util import bits, compare, dev_tables, lora_pools_to_device
    N = 5
    rng = np.random.Generator(np.random.PCG64(seed))
    tab = wl.random_segments(rng, S, N + 1, max_len)
    T = tab.T
    assert T >= min_rows, f"the case needs at least {min_rows} rows, the table has {T}"
    x = wl.activations(T, d_in, dtype, device="cuda", seed=seed + 1)
    pools = [wl.lora_pool(N, r, d_in, n, dtype, device="cuda", seed=seed + 10 + i) for i, n in enumerate(d_outs)]
    if fused_buffer:            # one [T, sum d_out (+ padding)] buffer, outputs are column ranges of it
        width = sum(d_outs) + 8
        buf0 = wl.activations(T, width, dtype, device="cuda", seed=seed + 2)
        buf = buf0.clone()
        offs = np.concatenate([[0], np.cumsum(d_outs)])
        ys = [buf[:, offs[i]:offs[i + 1]] for i in range(len(d_outs))]
        y0s = [buf0[:, offs[i]:offs[i + 1]] for i in range(len(d_outs))]
    else:
        y0s = [wl.activations(T, n, dtype, device="cuda", seed=seed + 20 + i) for i, n in enumerate(d_outs)]
        ys = [y.clone() for y in y0s]
    tables = [lora_pools_to_device(pl) for pl in pools]
    ss, sa, sp = dev_tables(tab)
    ws = preft.new_workspace(T, tab.S)
    mode = preft.PREFT_ALL_TOKENS if all_tokens else preft.PREFT_PREFILL_ONLY
    preft.preft_lora_apply_packed(ys, x, ss, sa, sp, [t[0] for t in tables], [t[1] for t in tables], r, 2.0, mode, ws)
    torch.cuda.synchronize()
    pos = ora.ALL_POSITIONS if all_tokens else ora.PROMPT_ONLY
    owner = ora.positions(T, tab.seg_start, tab.seg_adapter, tab.seg_prefill_len, N, pos)
    worst = 0.0
    for i, pl in enumerate(pools):
        want = ora.lora(y0s[i].contiguous().cpu(), x.cpu(), tab.seg_start, tab.seg_adapter, tab.seg_prefill_len,
                        [a.cpu() for a in pl.A], [b.cpu() for b in pl.B], r, 2.0, pos)
        worst = max(worst, compare(ys[i], y0s[i], want, owner, dtype))
    if fused_buffer:            # the padding columns of the fused buffer are not touched
        assert torch.equal(bits(buf[:, sum(d_outs):].contiguous()), bits(buf0[:, sum(d_outs):].contiguous()))
    assert torch.equal(bits(x), bits(wl.activations(T, d_in, dtype, device="cuda", seed=seed + 1)))
    return worst


@pytest.mark.parametrize("dtype,r,d_in,d_outs,fused_buffer", [
    ("bf16", 16, 512, (512, 128, 128), True),        # q, k, v into one fused output
    ("bf16", 16, 512, (1408, 1408), True),           # gate, up
    ("bf16", 8, 1000, (264, 520), False),            # widths with 32- and 8-column tails, separate buffers
    ("bf16", 4, 256, (256, 256, 256), False),
    ("bf16", 16, 4096, (4096, 1024, 1024), True),    # Llama-3.1-8B q, k, v
    ("bf16", 32, 512, (512, 136), True),             # rank 32 with a width the row-split kernel does not take: one launch each
    ("bf16", 3, 512, (512, 128, 128), False),        # ranks 1..3: fused by the vector-ALU kernel
    ("bf16", 1, 4096, (4096, 1024, 1024), True),
    ("bf16", 2, 520, (1408, 264), False),
    ("bf16", 5, 512, (512, 128), True),              # ranks 5..15 that are not multiples of 4: the any-rank shape
    ("bf16", 7, 1000, (264, 520, 136), False),
    ("bf16", 11, 4096, (4096, 1024, 1024), True),
    ("bf16", 13, 512, (1408, 1408), True),
    ("bf16", 17, 256, (256, 128), False),            # a rank no kernel fuses: one launch each
    ("f32", 4, 256, (256, 64), True),
    ("bf16", 16, 512, (384,), False),                # a single projection is an ordinary apply
])
def test_packed_projections_match_the_oracle(dtype, r, d_in, d_outs, fused_buffer):
    for all_tokens in (False, True):
        worst = _packed_case(dtype, r, d_in, list(d_outs), fused_buffer, 300 + r, all_tokens)
        print(f"  packed {dtype} r={r} {d_in}->{d_outs} fused_buffer={fused_buffer} all_tokens={all_tokens} worst {worst:.2e}")


@pytest.mark.parametrize("r,d_in,d_outs,fused_buffer", [
    (32, 512, (512, 128, 128), True), (64, 1024, (1024, 128, 128), False), (64, 256, (1536, 1536), True),
    (48, 384, (128, 256), False), (20, 128, (256, 128, 384), True), (64, 8192, (1024, 1024), False),
    # ranks that are not multiples of 4: the any-rank form of the same kernel
    (31, 256, (256, 128), True), (50, 128, (384, 128, 256), False), (17, 512, (128, 128), True), (63, 384, (256, 256, 128), True),
])
def test_packed_projections_in_the_row_split_kernel(r, d_in, d_outs, fused_buffer):
    """Rank 20..64 with widths that are multiples of 128 on a batch of more than 1024 rows: one launch
    of the row-split kernel reads x once for all outputs (chunks); decode rows of the all-token mode
    take the column-split kernel per output."""
    for all_tokens in (False, True):
        worst = _packed_case("bf16", r, d_in, list(d_outs), fused_buffer, 500 + r, all_tokens, S=70, max_len=220,
                             min_rows=1025)
        print(f"  packed r={r} {d_in}->{d_outs} fused_buffer={fused_buffer} all_tokens={all_tokens} worst {worst:.2e}")


def test_two_launch_lora_in_a_graph_and_with_a_foreign_schedule():
    """The two-launch form keeps the boundary's promises: captured into a HIP graph and replayed with the
    tables rewritten in place it matches the eager run every time (z is rewritten by every replay), and
    with PREFT_SCHEDULE_READY on a workspace whose schedule belongs to another position set neither of
    its launches touches y, and preft_schedule_counts reports it."""
    from parity_util import bits, dev_tables, lora_pools_to_device
    N, d_in, r = 5, 512, 64
    d_outs = (512, 256)
    rng = np.random.Generator(np.random.PCG64(79))
    lens = np.array([300, 1, 129, 1, 1, 64, 450, 1, 5, 3, 700, 260])
    tabs = []
    for k in range(3):
        ids = rng.integers(-1, N, size=len(lens))
        pre = np.where(rng.random(len(lens)) < 0.6, lens, (lens * rng.random(len(lens))).astype(np.int64))
        tabs.append(wl.from_lengths(lens, ids, pre))
    T, S = tabs[0].T, tabs[0].S
    assert T > 1024
    pools = [lora_pools_to_device(wl.lora_pool(N, r, d_in, n, "bf16", device="cuda", seed=90 + i)) for i, n in enumerate(d_outs)]
    x = wl.activations(T, d_in, "bf16", device="cuda", seed=91)
    y0 = wl.activations(T, sum(d_outs), "bf16", device="cuda", seed=92)
    y1 = y0.clone()
    y2 = wl.activations(T, d_outs[0], "bf16", device="cuda", seed=93)
    y2_0 = y2.clone()
    ss, sa, sp = dev_tables(tabs[0])
    ws = preft.new_workspace(T, S, z_rank=r, z_proj=2)
    mode = preft.PREFT_PREFILL_ONLY
    _set(resident=1)

    def body():
        y1.copy_(y0)
        y2.copy_(y2_0)
        preft.preft_schedule(ws, ss, sa, sp, T, N, mode)
        ready = mode | preft.PREFT_SCHEDULE_READY
        preft.preft_lora_apply_packed([y1[:, :d_outs[0]], y1[:, d_outs[0]:]], x, ss, sa, sp, [p[0] for p in pools],
                                      [p[1] for p in pools], r, 2.0, ready, ws)
        preft.preft_lora_apply(y2, x, ss, sa, sp, pools[0][0], pools[0][1], r, 0.5, ready, ws)

    body()
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        body()
    for k in (1, 2, 0, 1):
        sa.copy_(torch.from_numpy(tabs[k].seg_adapter.copy()))
        sp.copy_(torch.from_numpy(tabs[k].seg_prefill_len.copy()))
        graph.replay()
        torch.cuda.synchronize()
        got = (y1.clone(), y2.clone())
        body()
        torch.cuda.synchronize()
        assert torch.equal(bits(got[0]), bits(y1)) and torch.equal(bits(got[1]), bits(y2)), f"replay differs (table {k})"
        assert not torch.equal(bits(y1), bits(y0)) and not torch.equal(bits(y2), bits(y2_0))
    # a schedule of the other position set in the workspace: both launches of a call must leave y alone
    preft.preft_schedule(ws, ss, sa, sp, T, N, preft.PREFT_ALL_TOKENS)
    y1.copy_(y0)
    y2.copy_(y2_0)
    ready = mode | preft.PREFT_SCHEDULE_READY
    preft.preft_lora_apply_packed([y1[:, :d_outs[0]], y1[:, d_outs[0]:]], x, ss, sa, sp, [p[0] for p in pools],
                                  [p[1] for p in pools], r, 2.0, ready, ws)
    preft.preft_lora_apply(y2, x, ss, sa, sp, pools[0][0], pools[0][1], r, 0.5, ready, ws)
    torch.cuda.synchronize()
    assert torch.equal(bits(y1), bits(y0)) and torch.equal(bits(y2), bits(y2_0))
    with pytest.raises(preft.PreftError) as e:
        preft.preft_schedule_counts(ws)
    assert e.value.code == preft.PREFT_ESCHEDULE
    _set()


TWO_LAUNCH_CASES = [
    # (rank, d_in, d_outs): widths the two-launch form takes (d_in % 128 == 0, every d_out % 256 == 0)
    (64, 512, (512,)), (64, 1024, (1024, 256, 256)), (64, 256, (1792, 1792)), (32, 512, (512, 256, 256)),
    (32, 384, (768,)), (20, 128, (256, 512)), (48, 640, (256,)), (36, 256, (512, 256, 768)),
]


@pytest.mark.parametrize("rank,d_in,d_outs", TWO_LAUNCH_CASES, ids=[f"r{c[0]}-{c[1]}-{'x'.join(map(str, c[2]))}" for c in TWO_LAUNCH_CASES])
def test_two_launch_lora_equals_the_single_launch_and_the_oracle(rank, d_in, d_outs):
    """A workspace with room for z (preft_workspace_bytes_z) lets a LoRA call at rank 20..64 run its
    shrink and its expand as two launches, the expand in 2-D tiles (single and packed calls; by itself on
    batches of 8192 to 131072 rows -- the full-size tests have such cases -- and here, on a smaller batch,
    by test flag).  The result must equal the small workspace's bit for bit (same arithmetic, same
    order), both must match the oracle, in both modes; the guard columns of the buffer and every
    inactive row stay untouched."""
    from oracle import preft_oracle as ora
    from parity_util import bits, compare, dev_tables, lora_pools_to_device
    N, dtype = 5, "bf16"
    tab = _mixed_table(rank * 7 + d_in, N, n_prompts=9, max_len=420, n_decode=40)
    T = tab.T
    assert T > 1024
    ss, sa, sp = dev_tables(tab)
    ws_small = preft.new_workspace(T, tab.S)
    ws_big = preft.new_workspace(T, tab.S, z_rank=rank, z_proj=len(d_outs))
    assert ws_big.numel() == preft.preft_workspace_bytes_z(T, tab.S, rank, len(d_outs)) > ws_small.numel()
    x = wl.activations(T, d_in, dtype, device="cuda", seed=41)
    pools = [wl.lora_pool(N, rank, d_in, n, dtype, device="cuda", seed=50 + i) for i, n in enumerate(d_outs)]
    tables = [lora_pools_to_device(pl) for pl in pools]
    width = sum(d_outs) + 8
    buf0 = wl.activations(T, width, dtype, device="cuda", seed=42)
    offs = np.concatenate([[0], np.cumsum(d_outs)])
    for all_tokens in (False, True):
        mode = preft.PREFT_ALL_TOKENS if all_tokens else preft.PREFT_PREFILL_ONLY
        pos = ora.ALL_POSITIONS if all_tokens else ora.PROMPT_ONLY
        owner = ora.positions(T, tab.seg_start, tab.seg_adapter, tab.seg_prefill_len, N, pos)
        got = {}
        for name, ws in (("one launch", ws_small), ("two launches", ws_big)):
            buf = buf0.clone()
            ys = [buf[:, offs[i]:offs[i + 1]] for i in range(len(d_outs))]
            _set(resident=1)                  # the two-launch form also below the batch size that takes it by itself
            if len(d_outs) == 1:
                preft.preft_lora_apply(ys[0], x, ss, sa, sp, tables[0][0], tables[0][1], rank, 2.0, mode, ws)
            else:
                preft.preft_lora_apply_packed(ys, x, ss, sa, sp, [t[0] for t in tables], [t[1] for t in tables], rank, 2.0, mode, ws)
            torch.cuda.synchronize()
            preft.preft_schedule_counts(ws)
            got[name] = buf
        assert torch.equal(bits(got["one launch"]), bits(got["two launches"]))
        buf = got["two launches"]
        assert torch.equal(bits(buf[:, sum(d_outs):].contiguous()), bits(buf0[:, sum(d_outs):].contiguous()))
        worst = 0.0
        for i, pl in enumerate(pools):
            y0 = buf0[:, offs[i]:offs[i + 1]].contiguous()
            want = ora.lora(y0.cpu(), x.cpu(), tab.seg_start, tab.seg_adapter, tab.seg_prefill_len,
                            [a.cpu() for a in pl.A], [b.cpu() for b in pl.B], rank, 2.0, pos)
            worst = max(worst, compare(buf[:, offs[i]:offs[i + 1]], y0, want, owner, dtype))
        print(f"  two launches r={rank} {d_in}->{d_outs} T={T} all_tokens={all_tokens} worst {worst:.2e}")
    # the forced single-launch variant on the large workspace is the single-launch result too
    _set(5)
    buf = buf0.clone()
    ys = [buf[:, offs[i]:offs[i + 1]] for i in range(len(d_outs))]
    if len(d_outs) == 1:
        preft.preft_lora_apply(ys[0], x, ss, sa, sp, tables[0][0], tables[0][1], rank, 2.0, mode, ws_big)
    else:
        preft.preft_lora_apply_packed(ys, x, ss, sa, sp, [t[0] for t in tables], [t[1] for t in tables], rank, 2.0, mode, ws_big)
    torch.cuda.synchronize()
    assert torch.equal(bits(buf), bits(got["one launch"]))
    _set()


@pytest.mark.parametrize("rank,d_in,d_outs", [(32, 256, (256, 128, 128)), (64, 128, (384, 128)), (64, 384, (128, 128, 256)),
                                              (7, 264, (256, 136, 128)), (13, 128, (392, 128)), (29, 128, (256, 128)),
                                              (61, 256, (128, 128, 128))])
def test_packed_row_split_kernel_gives_the_exactly_rounded_result(rank, d_in, d_outs):
    """Small-integer data (every product and sum exact on both sides): the packed launch must equal
    the oracle's result rounded once to bf16, bit for bit, on every output.  (Rank 32 and 64: the
    row-split kernel; rank 7 and 13: the column-split kernel's any-rank shape; rank 29 and 61: the
    row-split kernel's any-rank form.)"""
    from oracle import preft_oracle as ora
    from parity_util import dev_tables
    N = 4
    gen = torch.Generator(device="cpu").manual_seed(rank * 100 + d_in)
    ints = lambda shape, lo, hi: torch.randint(lo, hi + 1, shape, generator=gen).to(torch.bfloat16).cuda()
    tab = _mixed_table(rank + d_in, N, n_prompts=8, max_len=400, n_decode=30)
    T = tab.T
    assert T > 1024
    ss, sa, sp = dev_tables(tab)
    ws = preft.new_workspace(T, tab.S)
    x = ints((T, d_in), -2, 2)
    A = [[ints((rank, d_in), -1, 1) for _ in range(N)] for _ in d_outs]
    B = [[ints((n, rank), -1, 1) for _ in range(N)] for n in d_outs]
    y0s = [ints((T, n), -3, 3) for n in d_outs]
    for mode, pos in ((preft.PREFT_ALL_TOKENS, ora.ALL_POSITIONS), (preft.PREFT_PREFILL_ONLY, ora.PROMPT_ONLY)):
        row_adapter = ora.positions(T, tab.seg_start, tab.seg_adapter, tab.seg_prefill_len, N, pos)
        ys = [y.clone() for y in y0s]
        preft.preft_lora_apply_packed(ys, x, ss, sa, sp, [preft.pointer_table(a) for a in A],
                                      [preft.pointer_table(b) for b in B], rank, 0.5, mode, ws)
        torch.cuda.synchronize()
        for i in range(len(d_outs)):
            want = ora.lora(y0s[i].cpu(), x.cpu(), tab.seg_start, tab.seg_adapter, tab.seg_prefill_len,
                            [a.cpu() for a in A[i]], [b.cpu() for b in B[i]], rank, 0.5, pos)
            assert np.abs(want).max() < 2 ** 15
            rounded = torch.from_numpy(want).to(torch.float32).to(torch.bfloat16)
            _same_bits(ys[i].cpu(), rounded, want, row_adapter, f"packed row-split output {i}")
            assert (ys[i].cpu() != y0s[i].cpu()).any()


def test_packed_projections_reject_overlapping_outputs():
    from parity_util import dev_tables, lora_pools_to_device
    N, r, d = 3, 16, 256
    tab = wl.from_lengths([20, 1], [0, 1], [20, 0])
    x = wl.activations(tab.T, d, "bf16", device="cuda", seed=1)
    buf = wl.activations(tab.T, 3 * d, "bf16", device="cuda", seed=2)
    before = buf.clone()
    pool = wl.lora_pool(N, r, d, d, "bf16", device="cuda", seed=3)
    Ap, Bp, keep = lora_pools_to_device(pool)
    ss, sa, sp = dev_tables(tab)
    ws = preft.new_workspace(tab.T, tab.S)
    def call(ys, xin=x):
        preft.preft_lora_apply_packed(ys, xin, ss, sa, sp, [Ap] * len(ys), [Bp] * len(ys), r, 1.0,
                                      preft.PREFT_PREFILL_ONLY, ws)
    for ys in ([buf[:, :d], buf[:, :d]],                       # the same range twice
               [buf[:, :d], buf[:, d // 2:d // 2 + d]],        # ranges that share columns
               [buf[:, :d], buf[1:, d:2 * d][:tab.T - 1]]):    # rows/dtype mismatch is caught by the binding
        with pytest.raises((preft.PreftError, ValueError)):
            call(ys)
    with pytest.raises(preft.PreftError):                      # x inside the output buffer
        call([buf[:, :d], buf[:, d:2 * d]], xin=buf[:, 2 * d:])
    with pytest.raises(preft.PreftError):                      # four projections
        call([buf[:, :64], buf[:, 64:128], buf[:, 128:192], buf[:, 192:256]])
    torch.cuda.synchronize()
    assert torch.equal(buf, before)
    call([buf[:, :d], buf[:, d:2 * d], buf[:, 2 * d:]])        # three disjoint ranges of one buffer: fine
    torch.cuda.synchronize()
    assert not torch.equal(buf, before)


# ---------------------------------------------------------------------------------------
# small batches: several workgroups share a tile, each writes its share of the columns
# ---------------------------------------------------------------------------------------
@pytest.mark.parametrize("colsplit", [1, 2, 3, 5, 8, 15])
@pytest.mark.parametrize("r,d_in,d_out", [(16, 512, 1024), (8, 1000, 264), (64, 512, 520), (4, 256, 128)])
def test_column_split_over_workgroups(colsplit, r, d_in, d_out):
    from parity_util import run_lora_case
    N = 5
    _set()
    _set_colsplit(colsplit)
    tab = _mixed_table(700 + r, N, n_prompts=3, max_len=90, n_decode=12)
    pool = wl.lora_pool(N, r, d_in, d_out, "bf16", device="cuda", seed=71)
    x = wl.activations(tab.T, d_in, "bf16", device="cuda", seed=72)
    y0 = wl.activations(tab.T, d_out, "bf16", device="cuda", seed=73)
    for all_tokens in (False, True):
        worst, _ = run_lora_case(tab, pool, x, y0, "bf16", 2.0, all_tokens, pad_cols=8)
        print(f"  colsplit={colsplit} r={r} {d_in}->{d_out} all_tokens={all_tokens} worst {worst:.2e}")


@pytest.mark.parametrize("colsplit", [1, 4, 7])
def test_column_split_with_packed_projections_and_in_place_calls(colsplit):
    """Packed outputs are split per output; DiReFT (in place) never splits a tile over workgroups."""
    from parity_util import run_direft_case
    _set()
    _set_colsplit(colsplit)
    for all_tokens in (False, True):
        for r, d_outs in ((16, [512, 128, 264]), (6, [512, 128, 264]), (15, [264, 512])):
            worst = _packed_case("bf16", r, 512, d_outs, True, 800 + colsplit + r, all_tokens, S=12, max_len=60)
            print(f"  colsplit={colsplit} packed r={r} all_tokens={all_tokens} worst {worst:.2e}")
    N, r, d = 4, 16, 1000
    tab = _mixed_table(810, N, n_prompts=3, max_len=90, n_decode=12)
    pool = wl.direft_pool(N, r, d, "bf16", device="cuda", seed=81)
    h = wl.activations(tab.T, d, "bf16", device="cuda", seed=82)
    run_direft_case(tab, pool, h, "bf16", 0.25, True)


# ---------------------------------------------------------------------------------------
# DiReFT on several layers' residual streams in one launch
# ---------------------------------------------------------------------------------------
LAYER_CASES = [
    # (variant, dtype, rank, d, layers, waves, rowblocks): every kernel family an in-place call can take
    (0, "bf16", 8, 1024, 3, 0, 0), (0, "bf16", 16, 4096, 2, 0, 0), (0, "bf16", 16, 8192, 2, 0, 0),   # resident tiles
    (0, "bf16", 16, 1000, 3, 0, 0), (0, "bf16", 32, 1024, 2, 0, 0), (0, "bf16", 64, 512, 3, 0, 0),   # streamed, row-split
    (0, "bf16", 2, 520, 4, 0, 0), (0, "bf16", 7, 256, 2, 0, 0), (VARIANT_VALU, "bf16", 4, 512, 2, 2, 0),
    (VARIANT_ROW, "bf16", 12, 264, 3, 0, 0), (0, "f32", 4, 132, 5, 0, 0), (0, "bf16", 24, 264, 2, 0, 0),
    (0, "bf16", 5, 4096, 2, 0, 0), (0, "bf16", 11, 8192 + 32, 2, 0, 0), (0, "bf16", 13, 8192 + 264, 2, 0, 0),   # any-rank shapes
]


@pytest.mark.parametrize("variant,dtype,rank,d,layers,waves,rowblocks", LAYER_CASES,
                         ids=[f"v{c[0]}-{c[1]}-r{c[2]}-d{c[3]}-L{c[4]}" for c in LAYER_CASES])
def test_direft_layers_match_the_oracle_and_the_one_layer_call(variant, dtype, rank, d, layers, waves, rowblocks):
    from parity_util import run_direft_layers_case
    N = 4
    tab = _mixed_table(rank * 31 + d, N, max_len=40 if d > 4200 else 150, n_prompts=3 if d > 4200 else 5)
    pools = [wl.direft_pool(N, rank, d, dtype, device="cuda", seed=100 + l) for l in range(layers)]
    h0s = [wl.activations(tab.T, d, dtype, device="cuda", seed=200 + l) for l in range(layers)]
    for all_tokens, bias_layers in ((False, [True] * layers), (True, [l % 2 == 0 for l in range(layers)]),
                                    (False, [False] * layers)):
        _set(variant, waves, rowblocks)
        worst = run_direft_layers_case(tab, pools, h0s, dtype, 1.0 / np.sqrt(rank), all_tokens, bias_layers, pad_cols=8)
        print(f"  layers={layers} all_tokens={all_tokens} bias={bias_layers} worst rel err {worst:.2e}")


def test_direft_layers_leave_other_layers_and_decode_rows_alone():
    """A call on layers 0 and 2 of three buffers leaves buffer 1 bit-identical; in prefill-only mode an
    all-decode batch leaves every buffer bit-identical; zero layers is a no-op."""
    from parity_util import bits, dev_tables, direft_pools_to_device
    N, r, d = 3, 16, 2048
    tab = _mixed_table(5, N)
    hs0 = [wl.activations(tab.T, d, "bf16", device="cuda", seed=300 + l) for l in range(3)]
    hs = [h.clone() for h in hs0]
    dev = [direft_pools_to_device(wl.direft_pool(N, r, d, "bf16", device="cuda", seed=310 + l)) for l in range(2)]
    table = lambda ptrs: torch.tensor(ptrs, dtype=torch.int64, device="cuda")
    ss, sa, sp = dev_tables(tab)
    ws = preft.new_workspace(tab.T, tab.S)
    used = [hs[0], hs[2]]
    args = (table([m[0].data_ptr() for m in dev]), table([m[1].data_ptr() for m in dev]),
            table([m[2].data_ptr() for m in dev]), N, r, 1.0)
    preft.preft_direft_apply_layers(used, preft.pointer_table(used), ss, sa, sp, *args, preft.PREFT_ALL_TOKENS, ws)
    torch.cuda.synchronize()
    assert torch.equal(bits(hs[1]), bits(hs0[1]))
    assert not torch.equal(bits(hs[0]), bits(hs0[0])) and not torch.equal(bits(hs[2]), bits(hs0[2]))
    # all-decode batch, prefill-only: nothing moves
    S = 12
    dec = wl.SegmentTable(np.arange(S + 1, dtype=np.int32), np.arange(S, dtype=np.int32) % N, np.zeros(S, dtype=np.int32))
    ss, sa, sp = dev_tables(dec)
    small0 = [wl.activations(S, d, "bf16", device="cuda", seed=320 + l) for l in range(2)]
    small = [h.clone() for h in small0]
    ws = preft.new_workspace(S, S)
    preft.preft_direft_apply_layers(small, preft.pointer_table(small), ss, sa, sp, *args, preft.PREFT_PREFILL_ONLY, ws)
    torch.cuda.synchronize()
    assert all(torch.equal(bits(a), bits(b)) for a, b in zip(small, small0))
    lib = preft.load_library()
    rc = lib.preft_direft_apply_layers(None, d, 0, S, d, ss.data_ptr(), sa.data_ptr(), sp.data_ptr(), S, None, None, None,
                                       N, r, 1.0, preft.PREFT_BF16, 0, ws.data_ptr(), ws.numel() * ws.element_size(), None)
    assert rc == 0


# ---------------------------------------------------------------------------------------
# exact arithmetic: small-integer data, every product and sum exact on both sides, so the kernel's
# output must be the oracle's fp64 result rounded once to the storage type -- bit for bit
# ---------------------------------------------------------------------------------------
EXACT_CASES = [
    # (dtype, variant, rank, d_in, d_out): one case per kernel family
    ("bf16", VARIANT_AUTO, 16, 256, 384), ("bf16", VARIANT_AUTO, 8, 200, 72), ("bf16", VARIANT_VALU, 2, 136, 264),
    ("bf16", VARIANT_AUTO, 32, 256, 256), ("bf16", VARIANT_AUTO, 64, 128, 384), ("bf16", VARIANT_ROW, 5, 64, 40),
    ("bf16", VARIANT_AUTO, 5, 256, 384), ("bf16", VARIANT_AUTO, 7, 200, 136), ("bf16", VARIANT_AUTO, 11, 128, 264),
    ("bf16", VARIANT_AUTO, 14, 264, 128),
    ("bf16", VARIANT_AUTO, 17, 128, 256), ("bf16", VARIANT_AUTO, 30, 256, 128), ("bf16", VARIANT_AUTO, 63, 128, 128),
    ("bf16", VARIANT_AUTO, 101, 128, 256),
    ("f32", VARIANT_AUTO, 4, 132, 68), ("f32", VARIANT_AUTO, 9, 64, 64),
]


def _same_bits(got, rounded, exact, row_adapter, what):
    from parity_util import bits
    bad = (bits(got) != bits(rounded)).nonzero()
    if len(bad):
        lines = [f"row {int(t)} (adapter {int(row_adapter[t])}) col {int(j)}: got {float(got[t, j])}, "
                 f"exact {float(exact[t, j])} -> {float(rounded[t, j])}" for t, j in bad[:8].tolist()]
        raise AssertionError(f"{what}: {len(bad)} of {got.numel()} elements differ from the exactly rounded "
                             "result\n" + "\n".join(lines))


@pytest.mark.parametrize("dtype,variant,rank,d_in,d_out", EXACT_CASES,
                         ids=[f"{c[0]}-v{c[1]}-r{c[2]}-{c[3]}x{c[4]}" for c in EXACT_CASES])
def test_integer_data_gives_the_exactly_rounded_result(dtype, variant, rank, d_in, d_out):
    from oracle import preft_oracle as ora
    from parity_util import bits, dev_tables
    N = 4
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    gen = torch.Generator(device="cpu").manual_seed(rank * 1000 + d_in)
    ints = lambda shape, lo, hi: torch.randint(lo, hi + 1, shape, generator=gen).to(tdt).cuda()
    tab = _mixed_table(rank + d_in + d_out, N, max_len=90)
    T = tab.T
    ss, sa, sp = dev_tables(tab)
    ws = preft.new_workspace(T, tab.S)
    mode = preft.PREFT_ALL_TOKENS
    row_adapter = ora.positions(T, tab.seg_start, tab.seg_adapter, tab.seg_prefill_len, N, ora.ALL_POSITIONS)
    assert (row_adapter >= 0).sum() > 100

    # LoRA: |x| <= 2, A in {-1,0,1}, B in {-1,0,1}, s = 0.5: |z| <= 2 d_in, halves; |delta| <= rank d_in
    x, y0 = ints((T, d_in), -2, 2), ints((T, d_out), -3, 3)
    A = [ints((rank, d_in), -1, 1) for _ in range(N)]
    B = [ints((d_out, rank), -1, 1) for _ in range(N)]
    y = y0.clone()
    _set(variant)
    preft.preft_lora_apply(y, x, ss, sa, sp, preft.pointer_table(A), preft.pointer_table(B), rank, 0.5, mode, ws)
    torch.cuda.synchronize()
    want = ora.lora(y0.cpu(), x.cpu(), tab.seg_start, tab.seg_adapter, tab.seg_prefill_len,
                    [a.cpu() for a in A], [b.cpu() for b in B], rank, 0.5, ora.ALL_POSITIONS)
    assert np.array_equal(want * 2, np.round(want * 2)), "the reference values should be multiples of 1/2"
    assert np.abs(want).max() < 2 ** 15
    rounded = torch.from_numpy(want).to(torch.float32).to(tdt)       # exact in fp32, then one rounding to nearest even
    _same_bits(y.cpu(), rounded, want, row_adapter, "LoRA")
    assert (y.cpu() != y0.cpu()).any()
    # the same projection as a packed call on two column ranges of one output buffer
    cut = (d_out // 16) * 8
    y2 = y0.clone()
    B_lo, B_hi = [m[:cut].contiguous() for m in B], [m[cut:].contiguous() for m in B]
    Ap = preft.pointer_table(A)
    _set(variant)
    preft.preft_lora_apply_packed([y2[:, :cut], y2[:, cut:]], x, ss, sa, sp, [Ap, Ap],
                                  [preft.pointer_table(B_lo), preft.pointer_table(B_hi)], rank, 0.5, mode, ws)
    torch.cuda.synchronize()
    _same_bits(y2.cpu(), rounded, want, row_adapter, "packed LoRA")

    # DiReFT on the d_in-wide stream: h' = h + s W2^T (W1 h + b)
    h0 = ints((T, d_in), -2, 2)
    W1 = [ints((rank, d_in), -1, 1) for _ in range(N)]
    W2 = [ints((rank, d_in), -1, 1) for _ in range(N)]
    b = [ints((rank,), -4, 4) for _ in range(N)]
    h = h0.clone()
    _set(variant)
    W2t = [w.t().contiguous() for w in W2]                   # kept alive: the pointer table only names them
    preft.preft_direft_apply(h, ss, sa, sp, preft.pointer_table(W1), preft.pointer_table(W2t),
                             preft.pointer_table(b), rank, 0.5, mode, ws)
    torch.cuda.synchronize()
    want = ora.direft(h0.cpu(), tab.seg_start, tab.seg_adapter, tab.seg_prefill_len, [w.cpu() for w in W1],
                      [w.cpu() for w in W2], [v.cpu() for v in b], rank, 0.5, ora.ALL_POSITIONS)
    rounded = torch.from_numpy(want).to(torch.float32).to(tdt)
    _same_bits(h.cpu(), rounded, want, row_adapter, "DiReFT")


@pytest.mark.parametrize("dtype,rank,d", [("bf16", 16, 512), ("bf16", 2, 264), ("bf16", 32, 256), ("bf16", 64, 1024), ("f32", 4, 132)])
def test_segment_permutation_moves_the_rows_and_nothing_else(dtype, rank, d):
    """Batch items are independent (Sec. 1): with the segments in another order -- rows moving with
    them -- every row comes out with the same bits, whatever tile it now shares with other rows."""
    from parity_util import bits, dev_tables, direft_pools_to_device, lora_pools_to_device
    N = 5
    rng = np.random.Generator(np.random.PCG64(rank * 7 + d))
    tab = _mixed_table(rank + d + 3, N, max_len=200)
    lens = tab.seg_len
    order = rng.permutation(tab.S)
    ptab = wl.from_lengths(lens[order], tab.seg_adapter[order], tab.seg_prefill_len[order])
    # row t of the permuted batch is row src[t] of the original
    src = np.concatenate([np.arange(tab.seg_start[s], tab.seg_start[s + 1]) for s in order]).astype(np.int64)
    assert sorted(src.tolist()) == list(range(tab.T))
    idx = torch.from_numpy(src).cuda()
    pool = wl.lora_pool(N, rank, d, d + 8, dtype, device="cuda", seed=3)
    dpool = wl.direft_pool(N, rank, d, dtype, device="cuda", seed=4)
    Ap, Bp, keep1 = lora_pools_to_device(pool)
    W1p, W2tp, bp, keep2 = direft_pools_to_device(dpool)
    x = wl.activations(tab.T, d, dtype, device="cuda", seed=5)
    y0 = wl.activations(tab.T, d + 8, dtype, device="cuda", seed=6)
    for mode in (preft.PREFT_PREFILL_ONLY, preft.PREFT_ALL_TOKENS):
        outs = []
        for t, rows in ((tab, None), (ptab, idx)):
            ss, sa, sp = dev_tables(t)
            ws = preft.new_workspace(t.T, t.S)
            xx, yy = (x, y0.clone()) if rows is None else (x[rows].contiguous(), y0[rows].contiguous())
            hh = xx.clone()
            preft.preft_lora_apply(yy, xx, ss, sa, sp, Ap, Bp, rank, 2.0, mode, ws)
            preft.preft_direft_apply(hh, ss, sa, sp, W1p, W2tp, bp, rank, 0.5, mode, ws)
            torch.cuda.synchronize()
            outs.append((yy, hh))
        (ya, ha), (yb, hb) = outs
        assert torch.equal(bits(ya[idx]), bits(yb)), "LoRA rows changed with the order of the segments"
        assert torch.equal(bits(ha[idx]), bits(hb)), "DiReFT rows changed with the order of the segments"
        assert not torch.equal(bits(ya), bits(y0))


@pytest.mark.parametrize("rank,d,same_bits", [(16, 1024, True), (8, 4096, True), (2, 520, True), (32, 512, False), (64, 256, False),
                                               (16, 8192, False)])    # 8192 columns in registers: another order of the partial sums
def test_direft_without_bias_is_the_lora_entry_on_a_copy_of_the_stream(rank, d, same_bits):
    """Eq. 3 with b = 0 is Eq. 2 with A = W1, B = W2, x = h and y0 = h: the in-place entry and the
    out-of-place entry must agree -- bit for bit where both take the same kernel family (one rounding
    of the same fp32 sums), within two roundings of the output type elsewhere."""
    from parity_util import bits, dev_tables, direft_pools_to_device
    N = 4
    tab = _mixed_table(rank + d, N, max_len=150)
    dpool = wl.direft_pool(N, rank, d, "bf16", device="cuda", seed=12)
    W1p, W2tp, _, keep = direft_pools_to_device(dpool, bias=False)
    h0 = wl.activations(tab.T, d, "bf16", device="cuda", seed=13)
    ss, sa, sp = dev_tables(tab)
    ws = preft.new_workspace(tab.T, tab.S)
    for mode in (preft.PREFT_PREFILL_ONLY, preft.PREFT_ALL_TOKENS):
        h, y = h0.clone(), h0.clone()
        preft.preft_direft_apply(h, ss, sa, sp, W1p, W2tp, None, rank, 0.75, mode, ws)
        preft.preft_lora_apply(y, h0, ss, sa, sp, W1p, W2tp, rank, 0.75, mode, ws)
        torch.cuda.synchronize()
        if same_bits:
            assert torch.equal(bits(h), bits(y))
        else:
            err = (h.float() - y.float()).abs().amax(dim=1)
            ref = y.float().abs().amax(dim=1).clamp_min(1e-6)
            assert float((err / ref).max()) <= 2.0 ** -7
        assert not torch.equal(bits(h), bits(h0))


@pytest.mark.parametrize("dtype,rank,d", [("bf16", 16, 512), ("bf16", 3, 264), ("bf16", 32, 256), ("f32", 5, 68)])
def test_all_positions_is_prompt_only_with_every_row_a_prompt_row(dtype, rank, d):
    """Sec. 3.2: the all-position set is the prompt set of a sequence whose prompt is the whole
    sequence.  Same schedule, same launches, same bits."""
    from parity_util import bits, dev_tables, lora_pools_to_device
    N = 4
    tab = _mixed_table(rank * 3 + d, N, max_len=180)
    full = wl.SegmentTable(tab.seg_start, tab.seg_adapter, tab.seg_len.astype(np.int32))
    pool = wl.lora_pool(N, rank, d, d, dtype, device="cuda", seed=21)
    Ap, Bp, keep = lora_pools_to_device(pool)
    x = wl.activations(tab.T, d, dtype, device="cuda", seed=22)
    y0 = wl.activations(tab.T, d, dtype, device="cuda", seed=23)
    outs, counts = [], []
    for t, mode in ((tab, preft.PREFT_ALL_TOKENS), (full, preft.PREFT_PREFILL_ONLY)):
        ss, sa, sp = dev_tables(t)
        ws = preft.new_workspace(t.T, t.S)
        y = y0.clone()
        preft.preft_lora_apply(y, x, ss, sa, sp, Ap, Bp, rank, 2.0, mode, ws)
        torch.cuda.synchronize()
        outs.append(y)
        counts.append(preft.preft_schedule_counts(ws))
    assert counts[0] == counts[1]
    assert torch.equal(bits(outs[0]), bits(outs[1]))
    assert not torch.equal(bits(outs[0]), bits(y0))


@pytest.mark.parametrize("seed", [11, 12])
def test_randomised_shapes_ranks_pitches_and_modes(seed):
    """A seeded sweep over valid inputs: every rank class, widths with and without tails, row
    pitches with padding, both dtypes and modes, the small-batch shape forced on and off, one-layer
    and many-layer in-place calls -- each case against the oracle with the guards checked."""
    from parity_util import run_direft_case, run_direft_layers_case, run_lora_case
    rng = np.random.Generator(np.random.PCG64(seed))
    ranks = [1, 2, 3, 4, 5, 6, 7, 8, 9, 12, 16, 20, 24, 28, 32, 40, 48, 64, 96, 128]
    widths = [8, 16, 24, 64, 72, 128, 136, 256, 264, 384, 512, 520, 640, 1000, 1024, 1032, 2048, 4096, 4104]
    done = 0
    for case in range(150):
        dtype = "bf16" if rng.random() < 0.8 else "f32"
        r = int(rng.choice(ranks))
        d_in, d_out = int(rng.choice(widths)), int(rng.choice(widths))
        if dtype == "f32":
            d_in, d_out, r = min(d_in, 520), min(d_out, 520), min(r, 24)
        N = int(rng.integers(1, 9))
        tab = wl.random_segments(rng, int(rng.integers(1, 60)), N + 1, int(rng.integers(1, 300)))
        if tab.T == 0 or tab.T * max(d_in, d_out) * r > 4e9:
            continue
        all_tokens = bool(rng.integers(0, 2))
        pad = int(rng.choice([0, 8, 64, 1024]))
        scale = float(rng.choice([1.0, 0.5, 2.0, 0.37]))
        print(f"  case {case}: {dtype} r={r} {d_in}->{d_out} N={N} S={tab.S} T={tab.T} all={all_tokens} pad={pad}", flush=True)
        _set()
        _set_colsplit(int(rng.integers(1, 9)) if rng.random() < 0.3 else 0)
        pool = wl.lora_pool(N, r, d_in, d_out, dtype, device="cuda", seed=case)
        x = wl.activations(tab.T, d_in, dtype, device="cuda", seed=case + 1)
        y0 = wl.activations(tab.T, d_out, dtype, device="cuda", seed=case + 2)
        run_lora_case(tab, pool, x, y0, dtype, scale, all_tokens, pad_cols=pad, reuse_schedule=bool(rng.integers(0, 2)))
        dp = wl.direft_pool(N, r, d_in, dtype, device="cuda", seed=case + 3)
        run_direft_case(tab, dp, x, dtype, scale, all_tokens, pad_cols=pad, bias=bool(rng.integers(0, 2)))
        if rng.random() < 0.3:
            L = int(rng.integers(1, 4))
            pools = [wl.direft_pool(N, r, d_in, dtype, device="cuda", seed=case + 10 + l) for l in range(L)]
            hs = [wl.activations(tab.T, d_in, dtype, device="cuda", seed=case + 20 + l) for l in range(L)]
            run_direft_layers_case(tab, pools, hs, dtype, scale, all_tokens,
                                   [bool(rng.integers(0, 2)) for _ in range(L)], pad_cols=pad)
        done += 1
    _set()
    assert done > 100

