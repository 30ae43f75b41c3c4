// MFMA tile kernel (bf16 storage, fp32 accumulation), rank a multiple of 4 up to 128.
//
// One workgroup of WAVES wavefronts owns a tile of R = 16 * MB consecutive active rows of
// one segment.  The wavefronts split the *columns* in units of 128 (256 bytes per row):
// wavefront w takes units w, w + WAVES, ... of both sweeps, so the workgroup walks the
// same rows side by side and each wavefront has 1/WAVES of the dependent round trips.
//
// Memory side.  Every activation access is one instruction over 4 rows x 256 contiguous
// bytes (lane l': row l'/16, bytes 16 (l'%16) ..), which is what HBM and the texture path
// want: measured on this chip, 64-byte row pieces stream at ~4.8 TB/s at best, 256-byte
// pieces at ~5.4 TB/s.  The matrix cores want the opposite order (lane l: row l%16), so a
// unit is turned through a wavefront-private LDS buffer (4 x ds_write_b128, 4 x
// ds_read_b128 per 16 rows x 128 columns, rows padded by 16 bytes, no barrier: the LDS
// executes one wavefront's operations in order).  The adapter factors come from L2: the
// shrink loads a rank block of the [r, d_in] factor like a unit of activations (4 ranks x
// 256 bytes per instruction, turned through a second LDS buffer); the expand reads its
// operand of the [d_out, r] factor directly, 8 bytes (4 ranks of one column) per lane.
// Only the single 32-column steps of odd widths use 64-byte row pieces and ds_bpermute.
//
// Compute side.
//   shrink (Eq. 2: z = A x;  Eq. 3: z = A h + b), per 32 columns of the row:
//       v_mfma_f32_16x16x32_bf16 with  A-operand = 16 ranks x 32 columns of the adapter's
//       [r, d_in] factor, B-operand = 32 columns x 16 rows of activations.  The accumulator
//       leaves lane (row, g) holding the wavefront's partial z[row][16b + 4g .. + 3] for
//       rank block b.
//   reduce: the WAVES partial sums meet in LDS; every wavefront adds them in the same
//       order, so all hold the same z.
//   expand (Eq. 2: y += s B z;  Eq. 3: h += s B^T z), per 32 columns of the output row:
//       two MFMAs per rank block with  A-operand = 16 output columns x (16 ranks, twice) of
//       the [d_out, r] factor, B-operand = z split into a bf16 head and a bf16 remainder
//       (k index 8g + j: j < 4 the head of rank 16b + 4g + j, j >= 4 the remainder of rank
//       16b + 4g + j - 4), so the fp32 intermediate is not rounded to bf16.  The 16 columns
//       of MFMA e are c0 + 8(m/4) + 4e + m%4, which leaves lane (row, g) holding the 8
//       consecutive outputs y[row][c0 + 8g .. c0 + 8g + 7] -- the same (row, column)
//       ownership as the activation operand of the shrink.
//
// Because of that shared ownership the DiReFT variant (HUNITS > 0) keeps its share of the
// h tile in registers between the two sweeps: h is read from HBM once and written once.
//
// Both sweeps are software-pipelined by hand: the loads of unit u+1 are issued before the
// MFMAs of unit u, and the streamed shapes with one rank block request the first unit of the
// expand before the cross-wavefront sum of z.  Widths that are not a multiple of 128 finish
// with up to four single 32-column steps (64-byte row pieces, ds_bpermute).
#pragma once
#include "common.hpp"

#include <type_traits>

namespace preft {

__device__ __forceinline__ bf16x8_t as_bf16x8(u32x4_t v) { return __builtin_bit_cast(bf16x8_t, v); }
__device__ __forceinline__ u32x4_t as_u32x4(bf16x8_t v) { return __builtin_bit_cast(u32x4_t, v); }

// XCD-aware unit index: workgroup ids are dealt round-robin to the 8 XCDs, so the units
// are cut into 8 contiguous runs and XCD x walks run x in order.  Consecutive units (same
// segment, same adapter) then share one XCD's L2.
__device__ __forceinline__ int xcd_unit(int n_units)
{
    const int per_xcd = (n_units + 7) >> 3;
    const int xcd = blockIdx.x & 7, j = blockIdx.x >> 3;
    if (j >= per_xcd) return -1;
    const int v = xcd * per_xcd + j;
    return v < n_units ? v : -1;
}

constexpr int MFMA_TRS = 17;      // LDS row stride of the turn buffer in 16-byte vectors (256 B + 16 B pad)

// Wavefronts per SIMD the register allocation must leave room for: the register-resident DiReFT
// shapes need two workgroups per compute unit so that one streams in while the other streams out.
constexpr int mfma_min_waves(int NB, int MB, int WAVES, int HUNITS)
{
    return (HUNITS > 0 && WAVES == 8 && NB * MB == 1 && HUNITS <= 4) ? 4 : 1;
}

// SLICES > 1 (LoRA only): packed projections.  The outputs y_0 .. y_{SLICES-1} are all computed
// from the same x (q, k, v of an attention block; gate and up of an MLP), each with its own
// factors of NB rank blocks: one shrink sweep over x feeds SLICES * NB accumulator blocks, then
// one expand sweep per output.  x is read once instead of SLICES times.
//
// COLSPLIT (LoRA only): the small-batch shape, see below.
//
// PARTIAL (in place, HUNITS > 0): the wavefront keeps its first HUNITS units and streams the rest in
// both sweeps -- for tiles too large to hold (32 rows of 8192 elements are the whole register file).
// Without it a HUNITS > 0 shape expects every unit to fit (the host picks it only then).
//
// ODD (rank <= 16): ranks that are not multiples of 4 (5, 6, 7, 9, ...).  Nothing is padded in memory:
// the shrink's rank rows past r alias row r-1 and their z is zeroed; in the expand a column's r
// factors no longer start on an 8-byte boundary, so a wavefront fetches its unit's [128 columns][r]
// block of B -- contiguous in the [d_out, r] layout -- with coalesced 16-byte loads, parks it in its
// private LDS buffer (the shrink's factor buffer, idle by then) and picks its operands from there,
// two bytes at a time, zero for the ranks past r.  ODD is the number of 16-byte pieces of that block a
// lane carries: 2 up to rank 8, 4 up to rank 16.  In place with the tile in registers, the blocks of the
// first two units are requested before the reduction of z and the next ones while a unit is finished.
template <int NB, int MB, int WAVES, int HUNITS, bool DIREFT, int SLICES = 1, bool COLSPLIT = false, bool PARTIAL = false,
          int ODD = 0>
__device__ __forceinline__ void mfma_tile_body(const ApplyArgs &p)
{
    static_assert(!PARTIAL || HUNITS > 0, "a partially resident tile keeps some units");
    static_assert(!ODD || (NB == 1 && !PARTIAL), "the any-rank shape covers rank <= 16");
    static_assert(ODD == 0 || ODD == 2 || ODD == 4, "pieces per lane of a unit's factor block");
    constexpr bool STREAMS = HUNITS == 0 || PARTIAL;         // some units pass through both sweeps
    static_assert(!COLSPLIT || !DIREFT, "a tile of an in-place call belongs to one workgroup");
    // x is read a second time by this workgroup (in place without a resident tile) or by the
    // workgroups that share the tile (small-batch shape): then its loads stay cacheable
    // (in place, the units the wavefront does not keep: HUNITS names how many of its units stay in
    // registers; the others are streamed in both sweeps)
    constexpr bool X_READ_AGAIN = DIREFT || COLSPLIT;
    constexpr int R = 16 * MB;
    constexpr int NBT = NB * SLICES;                          // rank blocks of the shrink sweep
    constexpr bool PREFETCH_A = (NBT * MB <= 3);              // register budget
    static_assert(SLICES == 1 || (!DIREFT && HUNITS == 0), "packed projections are a LoRA feature");
    static_assert(CHUNK_ROWS % R == 0, "tile height must divide the chunk height");
    static_assert(HUNITS == 0 || DIREFT, "only the in-place variant keeps its tile in registers");
    static_assert(WAVES >= 4, "the tail steps are dealt one per wavefront");

    __shared__ float red[WAVES * NBT * MB * 4 * 64];          // cross-wavefront reduction of z
    __shared__ u32x4_t turn[WAVES][MB * 16 * MFMA_TRS];       // wavefront-private turn buffers: activations
    __shared__ u32x4_t turn_a[WAVES][16 * MFMA_TRS];          // ... and one rank block of the factor

    // Small batches (LoRA): col_split workgroups share a tile.  Each runs the whole shrink sweep
    // (the tile's x and the factor come from L2 after the first) and expands its own share of
    // the output columns, so that a step of a few dozen rows is spread over the chip instead
    // of walking every column in one workgroup.  Never in place: another workgroup's writes
    // must not meet this one's reads.
    if (!schedule_matches(p)) return;
    const int csplit = COLSPLIT ? p.col_split : 1;
    int n_chunk_units, cslice = 0;
    const int n_units = tile_units<R>(p, &n_chunk_units);
    int unit;
    if constexpr (COLSPLIT) {
        // the workgroups that share a tile sit side by side on one XCD (workgroup ids are dealt round-robin
        // to the 8 XCDs), so that all but the first of them find the tile's x in that XCD's L2
        const int xcd = blockIdx.x & 7, j = blockIdx.x >> 3;
        const int per_xcd = (n_units + 7) >> 3;
        const int t = j / csplit;
        cslice = j - t * csplit;
        unit = t < per_xcd ? xcd * per_xcd + t : -1;
        if (unit >= n_units) unit = -1;
    } else {
        unit = xcd_unit(n_units);
    }
    if (unit < 0) return;
    TileRows tile;
    if (!tile_rows<R>(p, unit, n_chunk_units, tile)) return;   // uniform over the workgroup
    const int adapter = tile.adapter;
    const int n_rows = tile.n_rows;

    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int rl = lane & 15, g = lane >> 4;                  // MFMA order: row rl, 16-byte group g
    const int q = lane >> 4, c16 = lane & 15;                 // unit load order: row 4i + q, 16-byte chunk c16
    const int ld_row = lane >> 2, ld_chunk = lane & 3;        // step load order: row, 16-byte chunk

    const int r = p.rank;
    const int64_t ldx_b = p.ldx * 2;
    u32x4_t *tr = turn[wave];
    u32x4_t *tra = turn_a[wave];

    // ---- lane permutations for single 32-column steps (factors, tails) ----------------
    const int gather_addr  = (4 * (lane & 15) + (lane >> 4)) << 2;    // MFMA lane <- step-load lane
    const int scatter_addr = ((lane >> 2) + 16 * (lane & 3)) << 2;    // step-store lane <- MFMA lane
    auto step_to_mfma = [&](u32x4_t raw) -> bf16x8_t {
        u32x4_t o;
#pragma unroll
        for (int i = 0; i < 4; ++i) o[i] = (uint32_t)__builtin_amdgcn_ds_bpermute(gather_addr, (int)raw[i]);
        return as_bf16x8(o);
    };
    auto mfma_to_step = [&](u32x4_t v) -> u32x4_t {
        u32x4_t o;
#pragma unroll
        for (int i = 0; i < 4; ++i) o[i] = (uint32_t)__builtin_amdgcn_ds_bpermute(scatter_addr, (int)v[i]);
        return o;
    };

    // ---- row pointers.  Row slots past the end of the tile alias its last row: they load the
    // same bytes, compute the same values and store the same bits, so no access below depends
    // on the row.
    int64_t row_u[MB][4], row_s[MB];   // unit order: instruction i covers rows 4i .. 4i+3; step order
    gcptr_t xu[MB][4];
    gcptr_t xs[MB];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            row_u[mb][i] = tile.row(mb * 16 + 4 * i + q);
            xu[mb][i] = as_global(p.x) + row_u[mb][i] * ldx_b + c16 * 16;
        }
        row_s[mb] = tile.row(mb * 16 + ld_row);
        xs[mb] = as_global(p.x) + row_s[mb] * ldx_b + ld_chunk * 16;
    }
    // factor pointers (ranks past r alias rank r-1; their z entries are zeroed below): a uniform
    // base per rank block's slice plus per-lane byte offsets, in unit order (instruction i covers
    // ranks 4i .. 4i+3 of a block, 256 bytes each) and in step order (the tails)
    gcptr_t abase[SLICES];
    abase[0] = as_global(slice_A<0>(p)[adapter]);
    if constexpr (SLICES > 1) abase[1] = as_global(slice_A<1>(p)[adapter]);
    if constexpr (SLICES > 2) abase[2] = as_global(slice_A<2>(p)[adapter]);
    int32_t aoff_u[NB][4], aoff_s[NB];
#pragma unroll
    for (int b = 0; b < NB; ++b) {
#pragma unroll
        for (int i = 0; i < 4; ++i) aoff_u[b][i] = (min(16 * b + 4 * i + q, r - 1) * p.d_in + c16 * 8) * 2;
        aoff_s[b] = (min(16 * b + ld_row, r - 1) * p.d_in + ld_chunk * 8) * 2;
    }

    // one unit (16 MB rows x 128 columns) from load order to MFMA order, through LDS
    auto unit_to_mfma = [&](const u32x4_t (&raw)[MB][4], u32x4_t (&op)[MB][4]) {
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
#pragma unroll
            for (int i = 0; i < 4; ++i) tr[(mb * 16 + 4 * i + q) * MFMA_TRS + c16] = raw[mb][i];
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
#pragma unroll
            for (int s = 0; s < 4; ++s) op[mb][s] = tr[(mb * 16 + rl) * MFMA_TRS + 4 * s + g];
    };

    // ---------------------------------------------------------------- shrink
    f32x4_t acc[NBT][MB];
#pragma unroll
    for (int b = 0; b < NBT; ++b)
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) acc[b][mb] = f32x4_t{0.f, 0.f, 0.f, 0.f};

    const int k_units = p.d_in >> 7;                          // whole 128-column units
    // which units a wavefront takes: every WAVES-th one (the workgroup then touches 16 rows x 2 KB side by side
    // at any moment), or, with a whole tile of more than 4096 columns held in registers, a contiguous range
    // (in place, d = 8192, rank 8-16: +1.5 to +2.6 points of bandwidth on the 70B-sized and skewed batches; at
    // d = 4096 the same costs 2-5 points and is not done)
    constexpr bool CONTIG = HUNITS > 4 && WAVES == 8 && !PARTIAL;
    const int k_per = (k_units + WAVES - 1) / WAVES;
    const int my_ku = CONTIG ? max(0, min(k_per, k_units - wave * k_per))
                             : (k_units > wave ? (k_units - wave + WAVES - 1) / WAVES : 0);
    auto k_unit = [&](int u) { return CONTIG ? wave * k_per + u : wave + u * WAVES; };
    const int k_steps = (p.d_in + 31) >> 5;                   // 32-column steps, the last may be partial
    const int k_tail_step = k_units * 4 + wave;               // this wavefront's tail step, if < k_steps

    u32x4_t hreg[HUNITS > 0 ? HUNITS : 1][MB][4];             // DiReFT: this wavefront's units, MFMA order
    u32x4_t htail[MB];                                        // DiReFT: its tail step, MFMA order

    auto load_x_unit = [&](u32x4_t (&raw)[MB][4], int u, auto again_tag) {
        constexpr bool AGAIN = decltype(again_tag)::value;    // these bytes are read a second time: keep them cacheable
        const int64_t off = (int64_t)k_unit(u) * 256;
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
#pragma unroll
            for (int i = 0; i < 4; ++i) raw[mb][i] = ld16_first<AGAIN>(xu[mb][i] + off);
    };
    constexpr std::integral_constant<bool, false> read_once{};
    constexpr std::integral_constant<bool, X_READ_AGAIN> read_streamed{};
    auto load_a_unit = [&](u32x4_t (&araw)[NBT][4], int u) {
        const int64_t off = (int64_t)k_unit(u) * 256;
#pragma unroll
        for (int b = 0; b < NBT; ++b)
#pragma unroll
            for (int i = 0; i < 4; ++i) araw[b][i] = ld16(abase[b / NB] + off + aoff_u[b % NB][i]);
    };
    // a rank block of the factor is turned into MFMA order like the activations: lane (rank rl, g)
    // then holds columns 8g .. 8g+7 of step s
    auto mfma_unit = [&](const u32x4_t (&op)[MB][4], const u32x4_t (&araw)[NBT][4]) {
#pragma unroll
        for (int b = 0; b < NBT; ++b) {
#pragma unroll
            for (int i = 0; i < 4; ++i) tra[(4 * i + q) * MFMA_TRS + c16] = araw[b][i];
            u32x4_t aop[4];
#pragma unroll
            for (int s = 0; s < 4; ++s) aop[s] = tra[rl * MFMA_TRS + 4 * s + g];
#pragma unroll
            for (int s = 0; s < 4; ++s)
#pragma unroll
                for (int mb = 0; mb < MB; ++mb)
                    acc[b][mb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(aop[s]), as_bf16x8(op[mb][s]),
                                                                         acc[b][mb], 0, 0, 0);
        }
    };

    if constexpr (HUNITS > 0) {
        // DiReFT: the wavefront's first HUNITS units stay in registers between the sweeps: issue
        // every load of them, then turn and multiply
        u32x4_t raw[HUNITS][MB][4];
#pragma unroll
        for (int u = 0; u < HUNITS; ++u)
            if (u < my_ku) load_x_unit(raw[u], u, read_once);
#pragma unroll
        for (int u = 0; u < HUNITS; ++u)
            if (u < my_ku) {
                u32x4_t araw[NBT][4];
                load_a_unit(araw, u);
                unit_to_mfma(raw[u], hreg[u]);
                mfma_unit(hreg[u], araw);
            }
    }
    // the units that are not kept (all of them unless HUNITS > 0) are streamed, two in flight
    if (STREAMS && my_ku > HUNITS) {
        u32x4_t x0[MB][4], x1[MB][4], a0[NBT][4], a1[NBT][4], op[MB][4];
        auto stage_load = [&](u32x4_t (&xr)[MB][4], u32x4_t (&ar)[NBT][4], int u) {
            load_x_unit(xr, u, read_streamed);
            if constexpr (PREFETCH_A) load_a_unit(ar, u);
        };
        auto stage_compute = [&](const u32x4_t (&xr)[MB][4], u32x4_t (&ar)[NBT][4], int u) {
            if constexpr (!PREFETCH_A) load_a_unit(ar, u);
            unit_to_mfma(xr, op);
            mfma_unit(op, ar);
        };
        int u = HUNITS;
        stage_load(x0, a0, u);
        while (u + 2 < my_ku) {
            stage_load(x1, a1, u + 1);
            stage_compute(x0, a0, u);
            stage_load(x0, a0, u + 2);
            stage_compute(x1, a1, u + 1);
            u += 2;
        }
        if (my_ku - u == 2) {
            stage_load(x1, a1, u + 1);
            stage_compute(x0, a0, u);
            stage_compute(x1, a1, u + 1);
        } else {
            stage_compute(x0, a0, u);
        }
    }
    // tail: at most one 32-column step per wavefront (width not a multiple of 128)
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) htail[mb] = u32x4_t{0u, 0u, 0u, 0u};
    if (k_tail_step < k_steps) {
        const bool col_ok = (k_tail_step * 32 + ld_chunk * 8) < p.d_in;   // step-load lane order
        const u32x4_t zero = {0u, 0u, 0u, 0u};
        const int64_t off = (int64_t)k_tail_step * 64;
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
            htail[mb] = as_u32x4(step_to_mfma(col_ok ? ld16_first<(X_READ_AGAIN && HUNITS == 0)>(xs[mb] + off) : zero));
#pragma unroll
        for (int b = 0; b < NBT; ++b) {
            const bf16x8_t av = step_to_mfma(col_ok ? ld16(abase[b / NB] + off + aoff_s[b % NB]) : zero);
#pragma unroll
            for (int mb = 0; mb < MB; ++mb)
                acc[b][mb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, as_bf16x8(htail[mb]), acc[b][mb], 0, 0, 0);
        }
    }

    // ---------------------------------------------------------------- first unit of the expand
    // Streamed variants with one rank block and one row block: this wavefront's first unit of the
    // first output's y and factor is requested before the reduction of z, so that the sweep over
    // the output starts without a gap.  The addresses are those of the sweep.  (Measured: +1 to +3
    // points of bandwidth with one output, nothing with two, a loss with three.)
    constexpr bool EARLY_UNIT = SLICES <= 2 && HUNITS == 0 && NB == 1 && MB == 1 && !ODD;
    u32x4_t y_early[MB][4];
    u32x2_t w_early[4][2][NB];
    if constexpr (EARLY_UNIT) {
        const int c_units = p.d_out >> 7;
        const int ubase = c_units * cslice / csplit;
        const int n_cu = c_units * (cslice + 1) / csplit - ubase;
        if (n_cu > wave) {
            const int64_t ldy_b = p.ldy * 2;
            const int64_t off = (int64_t)(ubase + wave) * 256;
#pragma unroll
            for (int i = 0; i < 4; ++i)
                y_early[0][i] = ld16_stream(as_global(p.y) + row_u[0][i] * ldy_b + c16 * 16 + off);
            if constexpr (PREFETCH_A) {
                const int col = 8 * (rl >> 2) + (rl & 3);
                const int rank0 = 4 * g;
                gcptr_t w0p = as_global(p.Bt_pool[adapter]) + ((int64_t)col * r + (rank0 < r ? rank0 : 0)) * 2;
                const int64_t w_step = (int64_t)32 * r * 2;
#pragma unroll
                for (int s = 0; s < 4; ++s)
#pragma unroll
                    for (int e = 0; e < 2; ++e)
                        w_early[s][e][0] = ld8(w0p + (int64_t)4 * e * r * 2 + ((ubase + wave) * 4 + s) * w_step);
            }
        }
    }

    // what a wavefront holds of a unit's factors between request and use: its MFMA operands
    // (8-byte pieces straight from memory), or, for ranks that are not multiples of 4, its share
    // of the unit's contiguous [128 columns][r] block (16 r pieces of 16 bytes, ODD per lane)
    using wbuf_t = std::conditional_t<(ODD > 0), u32x4_t[ODD > 0 ? ODD : 1], u32x2_t[4][2][NB]>;
    auto load_w_block = [&](wbuf_t &wb, gcptr_t Bt, int unit_index) {     // any-rank shape only
        if constexpr (ODD > 0) {
            gcptr_t base = Bt + (int64_t)unit_index * 256 * r;
#pragma unroll
            for (int i = 0; i < ODD; ++i)
                if (lane + 64 * i < 16 * r) wb[i] = ld16(base + (lane + 64 * i) * 16);
        }
    };
    // in place, tile in registers: the blocks of two units are in flight
    constexpr int W_AHEAD = (ODD > 0 && HUNITS > 0) ? 2 : 1;
    wbuf_t w_ahead[W_AHEAD];
    if constexpr (ODD > 0 && HUNITS > 0) {
#pragma unroll
        for (int u = 0; u < W_AHEAD; ++u)
            if (u < my_ku) load_w_block(w_ahead[u], as_global(p.Bt_pool[adapter]), k_unit(u));
    }

    // ---------------------------------------------------------------- reduce over wavefronts
    {
        constexpr int PER = NBT * MB * 4;
#pragma unroll
        for (int b = 0; b < NBT; ++b)
#pragma unroll
            for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                for (int v = 0; v < 4; ++v)
                    red[(wave * PER + (b * MB + mb) * 4 + v) * 64 + lane] = acc[b][mb][v];
        __syncthreads();          // also: every read of the tile precedes every write (in-place use)
#pragma unroll
        for (int b = 0; b < NBT; ++b)
#pragma unroll
            for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    float s = 0.f;
#pragma unroll
                    for (int w = 0; w < WAVES; ++w) s += red[(w * PER + (b * MB + mb) * 4 + v) * 64 + lane];
                    acc[b][mb][v] = s;
                }
    }

    // ---------------------------------------------------------------- z -> expand operand
    // lane (row rl, g) holds z[row][16b + 4g + v]; add the bias, apply the prefactor, zero the
    // padding ranks, and split into bf16 head + bf16 remainder.
    bf16x8_t zop[NBT][MB];
#pragma unroll
    for (int b = 0; b < NBT; ++b) {
        const int rank0 = 16 * (b % NB) + 4 * g;              // rank within the block's own slice
        const bool rank_ok = rank0 < r;                       // r % 4 == 0: all four or none; else see v_ok
        float bias[4] = {0.f, 0.f, 0.f, 0.f};
        if (DIREFT && rank_ok) {
            gcptr_t bias_p = bias_of(p, adapter);
            if (bias_p) {
#pragma unroll
                for (int v = 0; v < 4; ++v)
                    if (!ODD || rank0 + v < r) bias[v] = Elem<bf16_tag>::load1(bias_p, rank0 + v);
            }
        }
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) {
            float head_f[4], rem_f[4];
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const bool v_ok = ODD ? rank0 + v < r : rank_ok;
                const float zv = v_ok ? (acc[b][mb][v] + bias[v]) * p.scale : 0.f;
                const uint32_t hb = pack_bf16(zv, 0.f) & 0xffffu;
                head_f[v] = zv;
                rem_f[v] = zv - __uint_as_float(hb << 16);
            }
            u32x4_t packed;
            packed[0] = pack_bf16(head_f[0], head_f[1]);
            packed[1] = pack_bf16(head_f[2], head_f[3]);
            packed[2] = pack_bf16(rem_f[0], rem_f[1]);
            packed[3] = pack_bf16(rem_f[2], rem_f[3]);
            zop[b][mb] = as_bf16x8(packed);
        }
    }

    // ---------------------------------------------------------------- expand (once per output)
    // any-rank shape: where this lane's factors of step 0, column 8(rl/4) + rl%4 start in the parked block
    // (steps and the second MFMA of a step move on by an even number of elements), and which of its
    // four ranks 4g .. 4g+3 exist
    const int odd_at = (8 * (rl >> 2) + (rl & 3)) * r + 4 * g;
    const uint32_t *odd_words = reinterpret_cast<const uint32_t *>(tra) + (odd_at >> 1);
    const uint32_t odd_shift = (odd_at & 1) * 16;
    const int odd_n = r - 4 * g;
    const uint32_t odd_mask01 = odd_n >= 2 ? 0xffffffffu : odd_n == 1 ? 0xffffu : 0u;
    const uint32_t odd_mask23 = odd_n >= 4 ? 0xffffffffu : odd_n == 3 ? 0xffffu : 0u;
    auto take_early_w = [&](wbuf_t &w) {                      // the factors requested before the reduction of z
        if constexpr (EARLY_UNIT && PREFETCH_A) {
#pragma unroll
            for (int s = 0; s < 4; ++s)
#pragma unroll
                for (int e = 0; e < 2; ++e) w[s][e][0] = w_early[s][e][0];
        }
    };
    auto expand_slice = [&](auto sl_tag) {
    constexpr int SL = decltype(sl_tag)::value;
    gcptr_t Bt = as_global(slice_Bt<SL>(p)[adapter]);
    const int d_out = slice_d_out<SL>(p);
    const int64_t ldy_b = slice_ldy<SL>(p) * 2;
    // this workgroup's share of the output: whole units [ubase, ubase + n_cu), and the tail
    // steps of an odd width if it has the last share
    const int c_units = d_out >> 7;
    const int ubase = c_units * cslice / csplit;
    const int n_cu = c_units * (cslice + 1) / csplit - ubase;
    const int c_per = (n_cu + WAVES - 1) / WAVES;
    auto c_unit = [&](int u) { return ubase + (CONTIG ? wave * c_per + u : wave + u * WAVES); };
    gptr_t yu[MB][4];             // unit order
    gptr_t ys[MB];                // step order
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
#pragma unroll
        for (int i = 0; i < 4; ++i) yu[mb][i] = as_global(slice_y<SL>(p)) + row_u[mb][i] * ldy_b + c16 * 16;
        ys[mb] = as_global(slice_y<SL>(p)) + row_s[mb] * ldy_b + ld_chunk * 16;
    }
    // Weight pointer of MFMA e, rank block b: column 8(rl/4) + 4e + rl%4 of the current
    // 32-column step, ranks 16b + 4g .. +3 (padding ranks alias rank 0; their z is zero).
    gcptr_t bp[2][NB];
#pragma unroll
    for (int e = 0; e < 2; ++e)
#pragma unroll
        for (int b = 0; b < NB; ++b) {
            const int col = 8 * (rl >> 2) + 4 * e + (rl & 3);
            const int rank0 = 16 * b + 4 * g;
            bp[e][b] = Bt + ((int64_t)col * r + (rank0 < r ? rank0 : 0)) * 2;
        }
    const int64_t w_step = (int64_t)32 * r * 2;               // bytes per 32 output columns

    // out = y + delta for one 32-column step and one row block; y and the result in MFMA order
    auto expand_step = [&](const u32x4_t yv, const u32x2_t (&wv)[2][NB], int mb) -> u32x4_t {
        float out[8];
#pragma unroll
        for (int e = 0; e < 2; ++e) {
            f32x4_t d = f32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int b = 0; b < NB; ++b) {
                const u32x2_t w = wv[e][b];
                const bf16x8_t wop = as_bf16x8(u32x4_t{w[0], w[1], w[0], w[1]});
                d = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wop, zop[SL * NB + b][mb], d, 0, 0, 0);
            }
            const uint32_t y01 = yv[2 * e], y23 = yv[2 * e + 1];
            out[4 * e + 0] = bf16_lo(y01) + d[0];
            out[4 * e + 1] = bf16_hi(y01) + d[1];
            out[4 * e + 2] = bf16_lo(y23) + d[2];
            out[4 * e + 3] = bf16_hi(y23) + d[3];
        }
        return Elem<bf16_tag>::pack(out);
    };
    auto load_w_unit = [&](wbuf_t &wb, int u) {
        if constexpr (ODD > 0) {
            load_w_block(wb, Bt, c_unit(u));
        } else {
            const int cs0 = c_unit(u) * 4;
#pragma unroll
            for (int s = 0; s < 4; ++s)
#pragma unroll
                for (int e = 0; e < 2; ++e)
#pragma unroll
                    for (int b = 0; b < NB; ++b) wb[s][e][b] = ld8(bp[e][b] + (cs0 + s) * w_step);
        }
    };
    // the MFMA operands of step s of a unit from what load_w_unit fetched (any-rank shape: from the
    // block parked in LDS)
    auto w_operands = [&](const wbuf_t &wb, int s, u32x2_t (&wv)[2][NB]) {
        if constexpr (ODD > 0) {
            // this lane's four factors of a column are two or three consecutive 32-bit words of the
            // block (three when they start on an odd element): shift them into place, mask the ranks past r
#pragma unroll
            for (int e = 0; e < 2; ++e) {
                const uint32_t *w3 = odd_words + (16 * s + 2 * e) * r;
                const uint32_t d0 = w3[0], d1 = w3[1], d2 = w3[2];
                wv[e][0] = u32x2_t{__builtin_amdgcn_alignbit(d1, d0, odd_shift) & odd_mask01,
                                   __builtin_amdgcn_alignbit(d2, d1, odd_shift) & odd_mask23};
            }
        } else {
#pragma unroll
            for (int e = 0; e < 2; ++e)
#pragma unroll
                for (int b = 0; b < NB; ++b) wv[e][b] = wb[s][e][b];
        }
    };
    auto load_y_unit = [&](u32x4_t (&raw)[MB][4], int u) {
        const int64_t off = (int64_t)c_unit(u) * 256;
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
#pragma unroll
            for (int i = 0; i < 4; ++i) raw[mb][i] = ld16_stream(yu[mb][i] + off);
    };
    // a whole unit: y (MFMA order) -> out, turned back to load order through LDS and stored
    auto finish_unit = [&](const u32x4_t (&yop)[MB][4], const wbuf_t &wb, int u) {
        if constexpr (ODD > 0) {
#pragma unroll
            for (int i = 0; i < ODD; ++i)
                if (lane + 64 * i < 16 * r) tra[lane + 64 * i] = wb[i];
        }
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            u32x2_t wv[2][NB];
            w_operands(wb, s, wv);
#pragma unroll
            for (int mb = 0; mb < MB; ++mb) {
                const u32x4_t yv = yop[mb][s];
                tr[(mb * 16 + rl) * MFMA_TRS + 4 * s + g] = expand_step(yv, wv, mb);
            }
        }
        const int64_t off = (int64_t)c_unit(u) * 256;
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
#pragma unroll
            for (int i = 0; i < 4; ++i) st16_stream(yu[mb][i] + off, tr[(mb * 16 + 4 * i + q) * MFMA_TRS + c16]);
    };

    const int my_cu = CONTIG ? max(0, min(c_per, n_cu - wave * c_per)) : (n_cu > wave ? (n_cu - wave + WAVES - 1) / WAVES : 0);
    const int c_steps = cslice == csplit - 1 ? (d_out + 31) >> 5 : 0;
    const int c_tail_step = c_units * 4 + wave;

    // streamed units first (in place these are second reads: the sooner after the first the better),
    // then the units held in registers (d_in == d_out: the units of the expand are the units of hreg)
    if (STREAMS && my_cu > HUNITS) {
        u32x4_t y0[MB][4], y1[MB][4], yop[MB][4];
        wbuf_t w0, w1;
        auto stage_load = [&](u32x4_t (&yr)[MB][4], wbuf_t &wr, int u) {
            load_y_unit(yr, u);
            if constexpr (PREFETCH_A) load_w_unit(wr, u);
        };
        auto stage_compute = [&](const u32x4_t (&yr)[MB][4], wbuf_t &wr, int u) {
            if constexpr (!PREFETCH_A) load_w_unit(wr, u);
            unit_to_mfma(yr, yop);
            finish_unit(yop, wr, u);
        };
        int u = HUNITS;
        if constexpr (EARLY_UNIT && SL == 0) {
#pragma unroll
            for (int i = 0; i < 4; ++i) y0[0][i] = y_early[0][i];
            take_early_w(w0);
        } else {
            stage_load(y0, w0, u);
        }
        while (u + 2 < my_cu) {
            stage_load(y1, w1, u + 1);
            stage_compute(y0, w0, u);
            stage_load(y0, w0, u + 2);
            stage_compute(y1, w1, u + 1);
            u += 2;
        }
        if (my_cu - u == 2) {
            stage_load(y1, w1, u + 1);
            stage_compute(y0, w0, u);
            stage_compute(y1, w1, u + 1);
        } else {
            stage_compute(y0, w0, u);
        }
    }
    if constexpr (HUNITS > 0) {
#pragma unroll
        for (int u = 0; u < HUNITS; ++u)
            if (u < my_cu) {
                if constexpr (ODD > 0) {
                    finish_unit(hreg[u], w_ahead[u % W_AHEAD], u);
                    if (u + W_AHEAD < HUNITS && u + W_AHEAD < my_cu) load_w_unit(w_ahead[u % W_AHEAD], u + W_AHEAD);
                } else {
                    wbuf_t wb;
                    load_w_unit(wb, u);
                    finish_unit(hreg[u], wb, u);
                }
            }
    }
    // tail step of this wavefront (DiReFT: it still holds those activations in htail)
    if (c_tail_step < c_steps) {
        const int c0 = c_tail_step * 32;
        const bool col_ok = (c0 + ld_chunk * 8) < d_out;              // step-load lane order
        const int64_t off = (int64_t)c_tail_step * 64;
        u32x2_t wv[2][NB];
#pragma unroll
        for (int e = 0; e < 2; ++e) {
            // this lane's weight column may lie past d_out: alias the last column (its
            // products land in outputs that are not stored)
            const int col = c0 + 8 * (rl >> 2) + 4 * e + (rl & 3);
            const int64_t back = col < d_out ? 0 : (int64_t)(col - (d_out - 1)) * r * 2;
#pragma unroll
            for (int b = 0; b < NB; ++b) {
                gcptr_t wp = bp[e][b] + c_tail_step * w_step - back;
                if constexpr (ODD > 0) {                      // two bytes at a time, zero past rank r
                    uint32_t f[4];
#pragma unroll
                    for (int v = 0; v < 4; ++v)
                        f[v] = 4 * g + v < r ? (uint32_t) reinterpret_cast<const PREFT_GLOBAL uint16_t *>(wp)[v] : 0u;
                    wv[e][b] = u32x2_t{f[0] | (f[1] << 16), f[2] | (f[3] << 16)};
                } else {
                    wv[e][b] = ld8(wp);
                }
            }
        }
        // every load before the first store: row slots of different blocks may alias one row
        u32x4_t yv[MB];
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) {
            if constexpr (HUNITS > 0) yv[mb] = htail[mb];
            else yv[mb] = as_u32x4(step_to_mfma(col_ok ? ld16_stream(ys[mb] + off) : u32x4_t{0u, 0u, 0u, 0u}));
        }
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) {
            const u32x4_t o = mfma_to_step(expand_step(yv[mb], wv, mb));
            if (col_ok) st16_stream(ys[mb] + off, o);
        }
    }
    };
    expand_slice(std::integral_constant<int, 0>{});
    if constexpr (SLICES > 1) expand_slice(std::integral_constant<int, 1>{});
    if constexpr (SLICES > 2) expand_slice(std::integral_constant<int, 2>{});
}

template <int NB, int MB, int WAVES, int HUNITS, bool DIREFT, int SLICES = 1, bool COLSPLIT = false, bool PARTIAL = false,
          int ODD = 0>
__global__ __launch_bounds__(WAVES * 64, mfma_min_waves(NB, MB, WAVES, HUNITS)) void mfma_tile_kernel(ApplyArgs p)
{
    mfma_tile_body<NB, MB, WAVES, HUNITS, DIREFT, SLICES, COLSPLIT, PARTIAL, ODD>(p);
}

// the same for one of several residual streams (in-place calls): blockIdx.y is the layer
template <int NB, int MB, int WAVES, int HUNITS, bool PARTIAL = false, int ODD = 0>
__global__ __launch_bounds__(WAVES * 64, mfma_min_waves(NB, MB, WAVES, HUNITS)) void mfma_tile_layers_kernel(ApplyArgs p)
{
    select_layer(p);
    mfma_tile_body<NB, MB, WAVES, HUNITS, true, 1, false, PARTIAL, ODD>(p);
}

}  // namespace preft
