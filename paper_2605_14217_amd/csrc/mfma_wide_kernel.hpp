// MFMA tile kernel for larger ranks (bf16, rank % 4 == 0, 32 <= rank <= 128 in practice),
// widths that are multiples of 128 * CW.
//
// From rank 32 up the adapter factors outweigh a 16-row tile's activations (rank r costs
// r/16 factor bytes per activation byte), so here several 16-row blocks share the factors: a
// workgroup of RW x CW wavefronts owns a tile of 16 MB RW rows (up to a whole 128-row chunk);
// wavefront (rb, cg) owns row block rb and, of every group of CW adjacent 128-column units,
// unit cg.  In each step the workgroup loads the CW units of A (r ranks x 256 bytes each) or of
// B (128 columns x r factors each, contiguous in the [d_out, r] layout) once, with fully
// coalesced 16-byte loads, into a double-buffered LDS area, and every wavefront reads its MFMA
// operands from there (padded strides, no bank conflicts).  Factor traffic from L2 drops to
// r / (16 MB RW) of the activation traffic.
//
// Why column groups.  Measured on this chip with a kernel that only moves the bytes (read x,
// read y, write y; 352 814 rows of 8192 bf16, one barrier per step): a workgroup whose wavefronts
// all sit on the same 256-byte column slice of 64 different rows (RW x CW = 4 x 1) sustains 65 % of
// the 8 TB/s peak however many units it keeps in flight and however many workgroups share a
// compute unit; 4 x 2 (512 contiguous bytes per row and step) 73-74 %, 2 x 2 and 4 x 4 77-78 %,
// 8 x 1 60 %.  The memory system wants each row's bytes requested side by side, not 16 KB apart.
//
// With CW = 1 a wavefront walks all columns of its own rows and z never leaves its registers;
// with CW > 1 the CW partial sums of a row block meet in LDS after the sweep (every wavefront adds
// them in the same order, so all hold the same z).  Activations take the same path as in
// mfma_tile_kernel: 4 rows x 256 bytes per instruction, turned through a wavefront-private LDS
// buffer.  One barrier per step publishes the next factor units.  MFMA operand layouts as in
// mfma_tile_kernel, except that MFMA e of the expand takes the columns 2m + e of a 32-column
// step (lane (row, g) then owns outputs 8g + 2v + e), which makes the LDS reads of the B unit
// conflict-free.
//
// SLICES > 1 (LoRA only): packed projections, as in mfma_tile_kernel.  The outputs share x: every
// unit of x is loaded and turned once and then multiplied with the unit of each output's own A
// (one factor step and one barrier per output and unit of x, through the same two LDS buffers),
// which leaves SLICES * NB accumulator blocks; one expand sweep per output follows.
#pragma once
#include "common.hpp"
#include "mfma_kernel.hpp"

namespace preft {

constexpr int wide_fac_bytes(int NB, int CW)                   // one buffer of CW factor units
{
    const int fa = NB * 16 * MFMA_TRS * 16;                   // A unit: NB*16 ranks x 272 B
    const int fb = 128 * (32 * NB + 8);                       // B unit: 128 columns x (2r + 8) B
    return CW * (fa > fb ? fa : fb);
}
constexpr int wide_lds_bytes(int NB, int MB, int RW, int CW)
{
    return RW * CW * MB * 16 * MFMA_TRS * 16 + 2 * wide_fac_bytes(NB, CW);
}

//
// ZOUT (LoRA only): the shrink sweep alone.  z, already in the form the expand's MFMAs take it (scaled,
// split into bf16 head and remainder, in lane order), goes to the z area of the workspace, 1 KB per
// 16-row block and rank block, and mfma_expand_panel_kernel does the expand in a second launch.
//
// ODD: ranks that are not multiples of 4 (17, 18, 19, 21, ...; nothing is padded in memory).  The shrink
// needs nothing new (rank rows past r alias row r-1, their z is zeroed, here per element).  The expand's B
// units go to LDS as they lie in memory, a column's r factors right behind the previous column's, and a
// lane reads its four factors of a column as the three 32-bit words that hold them, shifts them into place
// and masks the ranks past r (as the any-rank shape of mfma_tile_kernel does for rank 5..15).
template <int NB, int MB, int RW, int CW, bool DIREFT, int SLICES = 1, bool ZOUT = false, bool ODD = false>
__device__ __forceinline__ void mfma_wide_body(const ApplyArgs &p)
{
    static_assert(!ODD || (!ZOUT && MB == 1 && CW == 1), "the any-rank form: one launch, the basic shape");
    static_assert(SLICES == 1 || !DIREFT, "packed projections are a LoRA feature");
    static_assert(!ZOUT || (!DIREFT && MB == 1), "the two-launch form: LoRA, 16-row blocks per wavefront");
    constexpr int WAVES = RW * CW;
    constexpr int NBT = NB * SLICES;                          // accumulator blocks of the shrink sweep
    constexpr int R = 16 * MB * RW;
    constexpr int TPC = CHUNK_ROWS / R;
    constexpr int NT = WAVES * 64;
    constexpr int A_UNIT = NB * 16 * MFMA_TRS;                // 16-byte vectors of an A unit in LDS
    constexpr int A_PIECES = NB * 16 * 16 * CW;               // 16-byte pieces of a step's A units (padded ranks included)
    constexpr int A_ITERS = (A_PIECES + NT - 1) / NT;
    constexpr int B_UNIT = 128 * (32 * NB + 8);               // bytes reserved for a B unit in LDS
    constexpr int B_ITERS = (NB * 16 * 16 * CW + NT - 1) / NT;   // upper bound: 16 r CW pieces, r <= 16 NB
    constexpr int FAC = wide_fac_bytes(NB, CW);
    static_assert(CHUNK_ROWS % R == 0, "tile height must divide the chunk height");
    static_assert(CW == 1 || WAVES * NB * MB * 4 * 64 * 4 <= 2 * FAC, "the partial sums of one output must fit the factor area");

    __shared__ __attribute__((aligned(16))) char lds_raw[wide_lds_bytes(NB, MB, RW, CW)];
    u32x4_t *turn_all = reinterpret_cast<u32x4_t *>(lds_raw);
    char *fac = lds_raw + WAVES * MB * 16 * MFMA_TRS * 16;    // factor area (A units, later B units): two buffers of FAC bytes

    if (!schedule_matches(p)) return;
    const int unit_id = xcd_unit(p.header[HDR_CHUNKS] * TPC);
    if (unit_id < 0) return;
    const int4 ch = p.chunks[unit_id / TPC];
    const int tile_row0 = (unit_id % TPC) * R;
    if (tile_row0 >= ch.z) return;                            // uniform over the workgroup
    const int adapter = ch.x;
    const int n_rows = min(R, ch.z - tile_row0);

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int rb = wave / CW, cg = wave % CW;                 // row block, column group
    const int rl = lane & 15, g = lane >> 4;                  // MFMA order
    const int q = lane >> 4, c16 = lane & 15;                 // unit load order
    const int r = p.rank;
    const int64_t ldx_b = p.ldx * 2;
    gcptr_t A[SLICES];
    A[0] = as_global(slice_A<0>(p)[adapter]);
    if constexpr (SLICES > 1) A[1] = as_global(slice_A<1>(p)[adapter]);
    if constexpr (SLICES > 2) A[2] = as_global(slice_A<2>(p)[adapter]);
    u32x4_t *tr = turn_all + wave * (MB * 16 * MFMA_TRS);

    // Row slots past the end of the tile alias its last row for loads; their stores are masked
    // (another wavefront may own that row, and a second read-modify-write would apply the delta twice).
    gcptr_t xu[MB][4];
    int64_t row_u[MB][4];
    bool row_ok[MB][4];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int t = rb * 16 * MB + mb * 16 + 4 * i + q;
            row_ok[mb][i] = t < n_rows;
            row_u[mb][i] = (int64_t)ch.y + tile_row0 + min(t, n_rows - 1);
            xu[mb][i] = as_global(p.x) + row_u[mb][i] * ldx_b + (cg * 16 + c16) * 16;
        }

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

    // a step covers CW adjacent units: this wavefront's unit of step u is u * CW + cg
    const int k_steps = p.d_in / (128 * CW);                  // d_in % (128 CW) == 0 (host-checked)
    auto load_x = [&](u32x4_t (&raw)[MB][4], int u) {
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
#pragma unroll
            for (int i = 0; i < 4; ++i) raw[mb][i] = ld16_first<DIREFT>(xu[mb][i] + (int64_t)u * (256 * CW));
    };
    // this thread's pieces of the step's A units: piece = (rank, 16-byte chunk of the 256 CW bytes of the step)
    auto load_a = [&](u32x4_t (&areg)[A_ITERS], gcptr_t Asl, int u) {
#pragma unroll
        for (int i = 0; i < A_ITERS; ++i) {
            const int piece = tid + i * NT;
            const int rank = min(piece / (16 * CW), r - 1);   // padding ranks alias rank r-1 (their z is zeroed)
            if (A_PIECES % NT == 0 || piece < A_PIECES)
                areg[i] = ld16(Asl + ((int64_t)rank * p.d_in) * 2 + (int64_t)u * (256 * CW) + (piece % (16 * CW)) * 16);
        }
    };
    auto publish_a = [&](const u32x4_t (&areg)[A_ITERS], int buf) {
        u32x4_t *fa = reinterpret_cast<u32x4_t *>(fac + buf * FAC);
#pragma unroll
        for (int i = 0; i < A_ITERS; ++i) {
            const int piece = tid + i * NT;
            const int chunk = piece % (16 * CW);
            if (A_PIECES % NT == 0 || piece < A_PIECES)
                fa[(chunk >> 4) * A_UNIT + (piece / (16 * CW)) * MFMA_TRS + (chunk & 15)] = areg[i];
        }
    };
    auto mfma_a = [&](const u32x4_t (&op)[MB][4], int buf, auto sl_tag) {
        constexpr int SL = decltype(sl_tag)::value;
        const u32x4_t *fa = reinterpret_cast<const u32x4_t *>(fac + buf * FAC) + cg * A_UNIT;
#pragma unroll
        for (int s = 0; s < 4; ++s)
#pragma unroll
            for (int b = 0; b < NB; ++b) {
                const u32x4_t ao = fa[(16 * b + rl) * MFMA_TRS + 4 * s + g];
#pragma unroll
                for (int mb = 0; mb < MB; ++mb) {
                    const u32x4_t xo = op[mb][s];
                    acc[SL * NB + b][mb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(ao), as_bf16x8(xo),
                                                                                  acc[SL * NB + b][mb], 0, 0, 0);
                }
            }
    };
    {
        // Pipeline.  A wavefront keeps two units of x on their way (three register buffers in
        // rotation) while it multiplies a third.  One trip handles a unit of x in SLICES steps, one
        // per output's factor units: step t = u * SLICES + sl multiplies from LDS buffer (t & 1)
        // while the factor units of step t + 1 are published into the other buffer; one barrier per
        // step.  With one output the factor units of step t + 1 are requested at the start of step
        // t; with several outputs a step is only a handful of MFMAs long, so the requests run two
        // steps ahead, the units of output sl always through register set sl.  Requests are issued
        // factor first, activations second: the memory counter retires in order, and the publish at
        // the end of a step must not wait for the activations requested in the same step.  Trips
        // come in threes with compile-time buffer numbers; GUARD = false (steady state) has no
        // conditional load, so that the compiler's wait counts stay exact; the last trips of a sweep
        // check which requests still exist.
        u32x4_t X[3][MB][4], op[MB][4], areg[SLICES][A_ITERS];
        int par = 0;                                          // LDS buffer of the current step
        auto trip = [&](auto xi_tag, int u, auto guard_tag) {
            constexpr int XI = decltype(xi_tag)::value;
            constexpr bool GUARD = decltype(guard_tag)::value;
            const bool has1 = !GUARD || u + 1 < k_steps, has2 = !GUARD || u + 2 < k_steps;
            auto step = [&](auto sl_tag) {
                constexpr int SL = decltype(sl_tag)::value;
                if constexpr (SLICES == 1) {
                    if (has1) load_a(areg[0], A[0], u + 1);
                } else {                                      // step t + 2 is (u, SL + 2) or (u + 1, SL + 2 - SLICES)
                    constexpr int S2 = (SL + 2) % SLICES, DU = (SL + 2) / SLICES;
                    if (DU == 0 || has1) load_a(areg[S2], A[S2], u + DU);
                }
                if constexpr (SL == 0) {
                    if (has2) load_x(X[(XI + 2) % 3], u + 2);
                    unit_to_mfma(X[XI], op);
                }
                mfma_a(op, par, sl_tag);
                if (SL + 1 < SLICES || has1) publish_a(areg[(SL + 1) % SLICES], par ^ 1);   // step t + 1 exists
                __syncthreads();                              // the last one: the factor area is reused below
                par ^= 1;
            };
            step(std::integral_constant<int, 0>{});
            if constexpr (SLICES > 1) step(std::integral_constant<int, 1>{});
            if constexpr (SLICES > 2) step(std::integral_constant<int, 2>{});
        };
        constexpr std::integral_constant<bool, false> steady{};
        constexpr std::integral_constant<bool, true> guarded{};
        constexpr std::integral_constant<int, 0> b0{};
        constexpr std::integral_constant<int, 1> b1{};
        constexpr std::integral_constant<int, 2> b2{};
        load_a(areg[0], A[0], 0);
        if constexpr (SLICES > 1) load_a(areg[1], A[1], 0);
        load_x(X[0], 0);
        if (k_steps > 1) load_x(X[1], 1);
        publish_a(areg[0], 0);
        __syncthreads();
        int u = 0;
        for (; u + 5 <= k_steps; u += 3) {                    // steps u .. u + 4 exist
            trip(b0, u, steady);
            trip(b1, u + 1, steady);
            trip(b2, u + 2, steady);
        }
        for (; u < k_steps; u += 3) {
            trip(b0, u, guarded);
            if (u + 1 < k_steps) trip(b1, u + 1, guarded);
            if (u + 2 < k_steps) trip(b2, u + 2, guarded);
        }
    }

    // ---------------------------------------------------------------- sum over the column groups
    // the CW partial sums of a row block meet in the factor area (free after the sweep's last
    // barrier), one output at a time; every wavefront adds them in the same order
    if constexpr (CW > 1) {
        float *red = reinterpret_cast<float *>(fac);
        constexpr int PER = NB * MB * 4;
#pragma unroll
        for (int sl = 0; sl < SLICES; ++sl) {
#pragma unroll
            for (int b = 0; b < NB; ++b)
#pragma unroll
                for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                    for (int v = 0; v < 4; ++v)
                        red[(wave * PER + (b * MB + mb) * 4 + v) * 64 + lane] = acc[sl * NB + b][mb][v];
            __syncthreads();
#pragma unroll
            for (int b = 0; b < NB; ++b)
#pragma unroll
                for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        float s = 0.f;
#pragma unroll
                        for (int c = 0; c < CW; ++c) s += red[((rb * CW + c) * PER + (b * MB + mb) * 4 + v) * 64 + lane];
                        acc[sl * NB + b][mb][v] = s;
                    }
            __syncthreads();                                  // the area is written again (next output, or B units)
        }
    }

    // ---------------------------------------------------------------- z -> expand operand
    bf16x8_t zop[NBT][MB];
#pragma unroll
    for (int b = 0; b < NBT; ++b) {
        const int rank0 = 16 * (b % NB) + 4 * g;              // rank within the block's own output
        const bool rank_ok = rank0 < r;
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

    if constexpr (ZOUT) {
        if (cg == 0) {                                        // with column groups every one of them holds the same z
            const int64_t blk16 = (int64_t)(unit_id / TPC) * (CHUNK_ROWS / 16) + tile_row0 / 16 + rb;
            u32x4_t *zw = reinterpret_cast<u32x4_t *>(p.zws) + blk16 * (NBT * 64) + lane;
#pragma unroll
            for (int b = 0; b < NBT; ++b) zw[b * 64] = as_u32x4(zop[b][0]);
        }
        return;
    }

    // ---------------------------------------------------------------- expand (once per output)
    // B units in LDS: column c of the step (0 .. 128 CW - 1) at byte c * CS, its r factors contiguous; CS = 2r + 8
    // (any-rank form: CS = 2r, the units as they lie in memory)
    const int cs = ODD ? 2 * r : 2 * r + 8;
    const int b_halves = 32 * r * CW;                         // 8-byte halves of a step's B units (128 CW columns x r factors)
    // where this thread's pieces land in LDS (the same for every step): two 8-byte halves each,
    // a half never straddles a column because r % 4 == 0
    int b_dst[B_ITERS][2];
#pragma unroll
    for (int i = 0; i < B_ITERS; ++i)
#pragma unroll
        for (int hh = 0; hh < 2; ++hh) {
            const int byte = ((tid + i * NT) * 2 + hh) * 8;   // offset in the contiguous units
            const int col = byte / (2 * r);
            b_dst[i][hh] = col * cs + (byte - col * 2 * r);
        }
    // byte offset of this lane's factors inside the step's B units for MFMA e, rank block b, 32-column step 0
    int w_off[2][NB];
#pragma unroll
    for (int e = 0; e < 2; ++e)
#pragma unroll
        for (int b = 0; b < NB; ++b) {
            const int rank0 = 16 * b + 4 * g;
            w_off[e][b] = (cg * 128 + 2 * rl + e) * cs + (rank0 < r ? rank0 : 0) * 2;
        }
    // any-rank form: element offset of this lane's factors (its four ranks may run past r: masked), the
    // shift that brings an odd start into place (columns 2m + e: odd only for e = 1 and odd r), the masks
    int odd_at[2][NB];
    uint32_t odd_m01[NB], odd_m23[NB];
    const uint32_t odd_shift[2] = {0u, (uint32_t)((r & 1) * 16)};
#pragma unroll
    for (int b = 0; b < NB; ++b) {
        const int n = r - (16 * b + 4 * g);
        odd_m01[b] = n >= 2 ? 0xffffffffu : n == 1 ? 0xffffu : 0u;
        odd_m23[b] = n >= 4 ? 0xffffffffu : n == 3 ? 0xffffu : 0u;
#pragma unroll
        for (int e = 0; e < 2; ++e) odd_at[e][b] = (cg * 128 + 2 * rl + e) * r + 16 * b + 4 * g;
    }

    auto expand_slice = [&](auto sl_tag) {
    constexpr int SL = decltype(sl_tag)::value;
    gcptr_t Bt = as_global(slice_Bt<SL>(p)[adapter]);
    const int64_t ldy_b = slice_ldy<SL>(p) * 2;
    gptr_t yu[MB][4];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int i = 0; i < 4; ++i) yu[mb][i] = as_global(slice_y<SL>(p)) + row_u[mb][i] * ldy_b + (cg * 16 + c16) * 16;

    auto load_b = [&](u32x4_t (&breg)[B_ITERS], int u) {
        gcptr_t base = Bt + (int64_t)u * (256 * CW) * r;      // 128 CW columns x r x 2 bytes
#pragma unroll
        for (int i = 0; i < B_ITERS; ++i) {
            const int piece = tid + i * NT;
            if (piece * 2 < b_halves) breg[i] = ld16(base + (int64_t)piece * 16);
        }
    };
    auto publish_b = [&](const u32x4_t (&breg)[B_ITERS], int buf) {
        char *fb = fac + buf * FAC;
#pragma unroll
        for (int i = 0; i < B_ITERS; ++i) {
            const int piece = tid + i * NT;
            if (piece * 2 < b_halves) {
                const u32x4_t v = breg[i];
                *reinterpret_cast<u32x2_t *>(fb + b_dst[i][0]) = u32x2_t{v[0], v[1]};
                *reinterpret_cast<u32x2_t *>(fb + b_dst[i][1]) = u32x2_t{v[2], v[3]};
            }
        }
    };
    auto load_y = [&](u32x4_t (&raw)[MB][4], int u) {
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
#pragma unroll
            for (int i = 0; i < 4; ++i) raw[mb][i] = ld16_stream(yu[mb][i] + (int64_t)u * (256 * CW));
    };
    auto finish_unit = [&](const u32x4_t (&yop)[MB][4], int buf, int u) {
        const char *fb = fac + buf * FAC;
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            f32x4_t d[2][MB];
#pragma unroll
            for (int e = 0; e < 2; ++e) {
#pragma unroll
                for (int mb = 0; mb < MB; ++mb) d[e][mb] = f32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int b = 0; b < NB; ++b) {
                    u32x2_t w;
                    if constexpr (ODD) {
                        const uint32_t *w3 = reinterpret_cast<const uint32_t *>(fb) + s * 16 * r + (odd_at[e][b] >> 1);
                        const uint32_t d0 = w3[0], d1 = w3[1], d2 = w3[2];
                        w = u32x2_t{__builtin_amdgcn_alignbit(d1, d0, odd_shift[e]) & odd_m01[b],
                                    __builtin_amdgcn_alignbit(d2, d1, odd_shift[e]) & odd_m23[b]};
                    } else {
                        w = *reinterpret_cast<const u32x2_t *>(fb + s * 32 * cs + w_off[e][b]);
                    }
                    const bf16x8_t wop = as_bf16x8(u32x4_t{w[0], w[1], w[0], w[1]});
#pragma unroll
                    for (int mb = 0; mb < MB; ++mb)
                        d[e][mb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wop, zop[SL * NB + b][mb], d[e][mb], 0, 0, 0);
                }
            }
#pragma unroll
            for (int mb = 0; mb < MB; ++mb) {
                // lane (row, g) owns columns 8g + 2v + e of the step
                const u32x4_t yv = yop[mb][s];
                float out[8];
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    out[2 * v]     = bf16_lo(yv[v]) + d[0][mb][v];
                    out[2 * v + 1] = bf16_hi(yv[v]) + d[1][mb][v];
                }
                tr[(mb * 16 + rl) * MFMA_TRS + 4 * s + g] = Elem<bf16_tag>::pack(out);
            }
        }
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const u32x4_t o = tr[(mb * 16 + 4 * i + q) * MFMA_TRS + c16];
                if (row_ok[mb][i]) st16_stream(yu[mb][i] + (int64_t)u * (256 * CW), o);
            }
    };

    const int c_steps = slice_d_out<SL>(p) / (128 * CW);      // d_out % (128 CW) == 0 (host-checked)
    {
        // the same pipeline: two units of y on their way while a third is finished and stored
        u32x4_t Y[3][MB][4], yop[MB][4], breg[B_ITERS];
        int par = 0;
        auto trip = [&](auto yi_tag, int u, auto guard_tag) {
            constexpr int YI = decltype(yi_tag)::value;
            constexpr bool GUARD = decltype(guard_tag)::value;
            const bool has1 = !GUARD || u + 1 < c_steps, has2 = !GUARD || u + 2 < c_steps;
            if (has1) load_b(breg, u + 1);
            if (has2) load_y(Y[(YI + 2) % 3], u + 2);
            unit_to_mfma(Y[YI], yop);
            finish_unit(yop, par, u);
            if (has1) publish_b(breg, par ^ 1);
            __syncthreads();
            par ^= 1;
        };
        constexpr std::integral_constant<bool, false> steady{};
        constexpr std::integral_constant<bool, true> guarded{};
        constexpr std::integral_constant<int, 0> b0{};
        constexpr std::integral_constant<int, 1> b1{};
        constexpr std::integral_constant<int, 2> b2{};
        load_b(breg, 0);
        load_y(Y[0], 0);
        if (c_steps > 1) load_y(Y[1], 1);
        if constexpr (SL > 0) __syncthreads();                // the previous output's last step is still being read
        publish_b(breg, 0);
        __syncthreads();
        int u = 0;
        for (; u + 5 <= c_steps; u += 3) {
            trip(b0, u, steady);
            trip(b1, u + 1, steady);
            trip(b2, u + 2, steady);
        }
        for (; u < c_steps; u += 3) {
            trip(b0, u, guarded);
            if (u + 1 < c_steps) trip(b1, u + 1, guarded);
            if (u + 2 < c_steps) trip(b2, u + 2, guarded);
        }
    }
    };
    expand_slice(std::integral_constant<int, 0>{});
    if constexpr (SLICES > 1) expand_slice(std::integral_constant<int, 1>{});
    if constexpr (SLICES > 2) expand_slice(std::integral_constant<int, 2>{});
}

// Wavefronts per SIMD the register allocation must leave room for.  Packed launches carry SLICES * NB
// accumulator blocks: with four wavefronts per workgroup they are held to two workgroups per compute
// unit, which the unpacked shapes reach by themselves.
constexpr int wide_min_waves(int RW, int CW, int SLICES)
{
    return (RW * CW == 4 && SLICES > 1) ? 2 : 1;
}

template <int NB, int MB, int RW, int CW, bool DIREFT, int SLICES = 1, bool ZOUT = false, bool ODD = false>
__global__ __launch_bounds__(RW * CW * 64, wide_min_waves(RW, CW, SLICES)) void mfma_wide_kernel(ApplyArgs p)
{
    mfma_wide_body<NB, MB, RW, CW, DIREFT, SLICES, ZOUT, ODD>(p);
}

// The expand sweep as a launch of its own (LoRA, after a ZOUT launch of the kernel above), in 2-D tiles:
// a workgroup of RW wavefronts takes 16 RW rows x PU units of 128 columns of one output; neighbouring
// workgroups take neighbouring column panels of the same rows.  Why: what the memory system rewards is
// a small set of rows in flight.  Measured with a kernel that only moves the bytes (read and write y,
// 352 814 rows): 64-row tiles that sweep all 8192 columns of their rows sustain 62 % of the 8 TB/s
// peak, the same tiles cut into 32 panels of 256 columns 77 % (16-row tiles of 8 wavefronts: 71 -> 83 %
// with 1024-column panels; on dense 28 672-wide rows 63 -> 68 % and 65 -> 71 %).  A workgroup that
// sweeps only a panel cannot afford the shrink sweep over the whole of x, hence the two launches, with z
// (r values per row) through HBM in between: 4 r bytes per row and output against 2 (d_in + 2 d_out).
// blockIdx.y is the output of a packed call.  Which calls take this form: see the notes at the launch site.
// The panel's factors (PU * 128 columns x r, contiguous in [d_out, r]) go to LDS once per workgroup
// and are shared by its RW row blocks; operand layouts as in the expand of mfma_wide_body.
// 52 KB of LDS at rank 64: three workgroups per compute unit, and the register allocation is held to that.
template <int NB, int RW, int PU>
__global__ __launch_bounds__(RW * 64, 3) void mfma_expand_panel_kernel(ApplyArgs p, int n_slices)
{
    constexpr int R = 16 * RW;
    constexpr int TPC = CHUNK_ROWS / R;
    constexpr int NT = RW * 64;
    constexpr int B_ITERS = (NB * 16 * 16 * PU + NT - 1) / NT;   // upper bound: 16 r PU pieces, r <= 16 NB
    constexpr int B_BYTES = PU * 128 * (32 * NB + 8);            // column c of the panel at byte c * (2r + 8)
    static_assert(CHUNK_ROWS % R == 0, "tile height must divide the chunk height");
    __shared__ __attribute__((aligned(16))) char lds_raw[RW * 16 * MFMA_TRS * 16 + B_BYTES];

    if (!schedule_matches(p)) return;
    const int sl = blockIdx.y;                                // output of a packed call
    void *y = p.y;
    int64_t ldy_b = p.ldy * 2;
    int d_out = p.d_out;
    const void *const *Bt_pool = p.Bt_pool;
    if (sl > 0) {
        y = p.more[sl - 1].y; ldy_b = p.more[sl - 1].ldy * 2; d_out = p.more[sl - 1].d_out; Bt_pool = p.more[sl - 1].Bt_pool;
    }
    const int panels = d_out / (128 * PU);                    // d_out % (128 PU) == 0 (host-checked)
    const int tid = threadIdx.x, rb = tid >> 6, lane = tid & 63;
    const int rl = lane & 15, g = lane >> 4;                  // MFMA order
    const int q = lane >> 4, c16 = lane & 15;                 // unit load order
    const int r = p.rank;
    u32x4_t *tr = reinterpret_cast<u32x4_t *>(lds_raw) + rb * (16 * MFMA_TRS);
    char *fb = lds_raw + RW * 16 * MFMA_TRS * 16;

    // The launch has at most a fixed number of workgroups (a multiple of 8: workgroup ids are dealt round-robin
    // to the 8 XCDs, and XCD x walks its own run of the tile list); a workgroup takes every gridDim.x-th tile
    // of its XCD's run, so that a launch that finds little or no work stays cheap whatever the batch's bounds.
    const int n_tiles = p.header[HDR_CHUNKS] * TPC * panels;
    const int per_xcd = (n_tiles + 7) >> 3;
    const int xcd = blockIdx.x & 7;
    for (int j = blockIdx.x >> 3; j < per_xcd; j += gridDim.x >> 3) {
    const int id = xcd * per_xcd + j;
    if (id >= n_tiles) break;
    const int tile = id / panels, panel = id - tile * panels;
    const int4 ch = p.chunks[tile / TPC];
    const int tile_row0 = (tile % TPC) * R;
    if (tile_row0 >= ch.z) continue;                          // uniform over the workgroup
    const int adapter = ch.x;
    const int n_rows = min(R, ch.z - tile_row0);

    // requests first: the panel's factors, this row block's z, its PU units of y
    gcptr_t Wp = as_global(Bt_pool[adapter]) + (int64_t)panel * (PU * 256) * r;
    const int b_halves = 32 * r * PU;                         // 8-byte halves of the panel's factors
    u32x4_t breg[B_ITERS];
#pragma unroll
    for (int i = 0; i < B_ITERS; ++i) {
        const int piece = tid + i * NT;
        if (piece * 2 < b_halves) breg[i] = ld16(Wp + (int64_t)piece * 16);
    }
    const int64_t blk16 = (int64_t)(tile / TPC) * (CHUNK_ROWS / 16) + tile_row0 / 16 + rb;
    gcptr_t zw = as_global(p.zws) + ((blk16 * n_slices + sl) * NB * 64 + lane) * 16;
    bf16x8_t zop[NB];
#pragma unroll
    for (int b = 0; b < NB; ++b) zop[b] = as_bf16x8(ld16(zw + b * 1024));
    gptr_t yu[4];
    bool row_ok[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int t = rb * 16 + 4 * i + q;
        row_ok[i] = t < n_rows;                               // rows past the tile alias its last row; their stores are masked
        yu[i] = as_global(y) + ((int64_t)ch.y + tile_row0 + min(t, n_rows - 1)) * ldy_b + (int64_t)panel * (PU * 256) + c16 * 16;
    }
    u32x4_t Y[PU][4];
#pragma unroll
    for (int u = 0; u < PU; ++u)
#pragma unroll
        for (int i = 0; i < 4; ++i) Y[u][i] = ld16_stream(yu[i] + u * 256);

    // factors to LDS: two 8-byte halves per piece, a half never straddles a column because r % 4 == 0
    const int cs = 2 * r + 8;
#pragma unroll
    for (int i = 0; i < B_ITERS; ++i) {
        const int piece = tid + i * NT;
        if (piece * 2 < b_halves) {
            const u32x4_t v = breg[i];
#pragma unroll
            for (int hh = 0; hh < 2; ++hh) {
                const int byte = (piece * 2 + hh) * 8;
                const int col = byte / (2 * r);
                *reinterpret_cast<u32x2_t *>(fb + col * cs + (byte - col * 2 * r)) = u32x2_t{v[2 * hh], v[2 * hh + 1]};
            }
        }
    }
    int w_off[2][NB];
#pragma unroll
    for (int e = 0; e < 2; ++e)
#pragma unroll
        for (int b = 0; b < NB; ++b) {
            const int rank0 = 16 * b + 4 * g;
            w_off[e][b] = (2 * rl + e) * cs + (rank0 < r ? rank0 : 0) * 2;
        }
    __syncthreads();

#pragma unroll
    for (int u = 0; u < PU; ++u) {
        u32x4_t yop[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) tr[(4 * i + q) * MFMA_TRS + c16] = Y[u][i];
#pragma unroll
        for (int s = 0; s < 4; ++s) yop[s] = tr[rl * MFMA_TRS + 4 * s + g];
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            f32x4_t d[2];
#pragma unroll
            for (int e = 0; e < 2; ++e) {
                d[e] = f32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int b = 0; b < NB; ++b) {
                    const u32x2_t w = *reinterpret_cast<const u32x2_t *>(fb + (u * 128 + s * 32) * cs + w_off[e][b]);
                    const bf16x8_t wop = as_bf16x8(u32x4_t{w[0], w[1], w[0], w[1]});
                    d[e] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wop, zop[b], d[e], 0, 0, 0);
                }
            }
            const u32x4_t yv = yop[s];                        // lane (row, g) owns columns 8g + 2v + e of the step
            float out[8];
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                out[2 * v]     = bf16_lo(yv[v]) + d[0][v];
                out[2 * v + 1] = bf16_hi(yv[v]) + d[1][v];
            }
            tr[rl * MFMA_TRS + 4 * s + g] = Elem<bf16_tag>::pack(out);
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const u32x4_t o = tr[(4 * i + q) * MFMA_TRS + c16];
            if (row_ok[i]) st16_stream(yu[i] + u * 256, o);
        }
    }
    __syncthreads();                                          // the next tile's factors overwrite this one's
    }
}

// the same for one of several residual streams (in-place calls): blockIdx.y is the layer
template <int NB, int MB, int RW, int CW, bool ODD = false>
__global__ __launch_bounds__(RW * CW * 64) void mfma_wide_layers_kernel(ApplyArgs p)
{
    select_layer(p);
    mfma_wide_body<NB, MB, RW, CW, true, 1, false, ODD>(p);
}

}  // namespace preft
