// MFMA tile kernel for larger ranks (bf16, rank % 4 == 0, 32 <= rank <= 128 in practice),
// widths that are multiples of 128.
//
// From rank 32 up the adapter factors outweigh a 16-row tile's activations (rank r costs
// r/16 factor bytes per activation byte), so here the wavefronts of a workgroup split the
// *rows* -- wavefront w owns rows 16 MB w .. of a tile of 16 MB WAVES rows (up to a whole
// 128-row chunk) -- and share the factors: for every 128-column unit the workgroup loads the
// unit of A (r ranks x 256 bytes) or of B (128 columns x r factors, contiguous in the
// [d_out, r] layout) once, with fully coalesced 16-byte loads, into a double-buffered LDS
// area, and every wavefront reads its MFMA operands from there (padded strides, no bank
// conflicts).  Factor traffic from L2 drops to r / (16 MB WAVES) of the activation traffic.
//
// Each wavefront walks all columns of its own rows, so z needs no cross-wavefront sum and
// stays in registers.  Activations take the same path as in mfma_tile_kernel: 4 rows x 256
// bytes per instruction, turned through a wavefront-private LDS buffer, next unit's loads in
// flight while the current unit is multiplied.  One barrier per unit publishes the next
// factor unit.  MFMA operand layouts as in mfma_tile_kernel, except that MFMA e of the
// expand takes the columns 2m + e of a 32-column step (lane (row, g) then owns outputs
// 8g + 2v + e), which makes the LDS reads of the B unit conflict-free.
//
// SLICES > 1 (LoRA only): packed projections, as in mfma_tile_kernel.  The outputs share x: every
// unit of x is loaded and turned once and then multiplied with the unit of each output's own A
// (one factor unit and one barrier per output and unit of x, through the same two LDS buffers),
// which leaves SLICES * NB accumulator blocks; one expand sweep per output follows.
#pragma once
#include "common.hpp"
#include "mfma_kernel.hpp"

namespace preft {

constexpr int wide_lds_bytes(int NB, int MB, int WAVES)
{
    const int turn = WAVES * MB * 16 * MFMA_TRS * 16;
    const int fa = 2 * NB * 16 * MFMA_TRS * 16;               // A units: NB*16 ranks x 272 B, two buffers
    const int fb = 2 * 128 * (32 * NB + 8);                   // B units: 128 columns x (2r + 8) B, two buffers
    return turn + (fa > fb ? fa : fb);
}

template <int NB, int MB, int WAVES, bool DIREFT, int SLICES = 1>
__device__ __forceinline__ void mfma_wide_body(const ApplyArgs &p)
{
    static_assert(SLICES == 1 || !DIREFT, "packed projections are a LoRA feature");
    constexpr int NBT = NB * SLICES;                          // accumulator blocks of the shrink sweep
    constexpr int R = 16 * MB * WAVES;
    constexpr int TPC = CHUNK_ROWS / R;
    constexpr int NT = WAVES * 64;
    constexpr int A_PIECES = NB * 16 * 16;                    // 16-byte pieces of an A unit (padded ranks included)
    constexpr int A_ITERS = (A_PIECES + NT - 1) / NT;
    constexpr int B_ITERS = (NB * 16 * 16 + NT - 1) / NT;     // upper bound: 16 r pieces, r <= 16 NB
    static_assert(CHUNK_ROWS % R == 0, "tile height must divide the chunk height");

    __shared__ __attribute__((aligned(16))) char lds_raw[wide_lds_bytes(NB, MB, WAVES)];
    u32x4_t *turn_all = reinterpret_cast<u32x4_t *>(lds_raw);
    char *fac = lds_raw + WAVES * MB * 16 * MFMA_TRS * 16;    // factor area (A units, later B units)

    if (!schedule_matches(p)) return;
    const int unit_id = xcd_unit(p.header[HDR_CHUNKS] * TPC);
    if (unit_id < 0) return;
    const int4 ch = p.chunks[unit_id / TPC];
    const int tile_row0 = (unit_id % TPC) * R;
    if (tile_row0 >= ch.z) return;                            // uniform over the workgroup
    const int adapter = ch.x;
    const int n_rows = min(R, ch.z - tile_row0);

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
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
            const int t = wave * 16 * MB + mb * 16 + 4 * i + q;
            row_ok[mb][i] = t < n_rows;
            row_u[mb][i] = (int64_t)ch.y + tile_row0 + min(t, n_rows - 1);
            xu[mb][i] = as_global(p.x) + row_u[mb][i] * ldx_b + c16 * 16;
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

    const int k_units = p.d_in >> 7;                          // d_in % 128 == 0 (host-checked)
    auto load_x = [&](u32x4_t (&raw)[MB][4], int u) {
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
#pragma unroll
            for (int i = 0; i < 4; ++i) raw[mb][i] = ld16_first<DIREFT>(xu[mb][i] + (int64_t)u * 256);
    };
    // this thread's pieces of the A unit: piece t + i NT = rank (piece >> 4), 16-byte chunk (piece & 15)
    auto load_a = [&](u32x4_t (&areg)[A_ITERS], gcptr_t Asl, int u) {
#pragma unroll
        for (int i = 0; i < A_ITERS; ++i) {
            const int piece = tid + i * NT;
            const int rank = min(piece >> 4, r - 1);          // padding ranks alias rank r-1 (their z is zeroed)
            if (A_PIECES % NT == 0 || piece < A_PIECES)
                areg[i] = ld16(Asl + ((int64_t)rank * p.d_in) * 2 + (int64_t)u * 256 + (piece & 15) * 16);
        }
    };
    auto publish_a = [&](const u32x4_t (&areg)[A_ITERS], int buf) {
        u32x4_t *fa = reinterpret_cast<u32x4_t *>(fac) + buf * (NB * 16 * MFMA_TRS);
#pragma unroll
        for (int i = 0; i < A_ITERS; ++i) {
            const int piece = tid + i * NT;
            if (A_PIECES % NT == 0 || piece < A_PIECES) fa[(piece >> 4) * MFMA_TRS + (piece & 15)] = areg[i];
        }
    };
    auto mfma_a = [&](const u32x4_t (&op)[MB][4], int buf, auto sl_tag) {
        constexpr int SL = decltype(sl_tag)::value;
        const u32x4_t *fa = reinterpret_cast<const u32x4_t *>(fac) + buf * (NB * 16 * MFMA_TRS);
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
        // One trip of `unit` handles a unit of x: SLICES steps, one per output's factor unit.  Step
        // number t = u * SLICES + sl multiplies from LDS buffer (t & 1) while the factor unit of step
        // t + 1 is published into the other buffer; one barrier per step.  With one output the factor
        // unit of step t + 1 is requested at the start of step t (before x is turned, so its latency
        // overlaps the wait for x); with several outputs a step is only a handful of MFMAs long, so
        // the requests run two steps ahead, through two register sets.  P0 is the buffer of the trip's
        // first step: the trips come in pairs (the register buffers of x swap without copies) and a
        // pair takes an even number of steps, so P0 is known at compile time.  No conditional loads
        // in the steady state: the prefetches stay in flight across the MFMAs.
        constexpr int DEPTH = SLICES > 1 ? 2 : 1;
        u32x4_t x0[MB][4], x1[MB][4], op[MB][4], areg[DEPTH][A_ITERS];
        auto unit = [&](const u32x4_t (&xc)[MB][4], u32x4_t (&xn)[MB][4], int u, auto next_tag, auto p0_tag) {
            constexpr bool HAS_NEXT = decltype(next_tag)::value;
            constexpr int P0 = decltype(p0_tag)::value;
            if constexpr (HAS_NEXT) load_x(xn, u + 1);
            if constexpr (SLICES == 1 && HAS_NEXT) load_a(areg[0], A[0], u + 1);
            unit_to_mfma(xc, op);
            auto step = [&](auto sl_tag) {
                constexpr int SL = decltype(sl_tag)::value;
                constexpr int BUF = (P0 + SL) & 1;
                constexpr bool PUBLISH = SL + 1 < SLICES || HAS_NEXT;       // step t + 1 exists
                if constexpr (SLICES > 1) {
                    constexpr int S2 = SL + 2;                               // step t + 2: (u, S2) or (u + 1, S2 - SLICES)
                    if constexpr (S2 < SLICES) load_a(areg[BUF], A[S2 % SLICES], u);
                    else if constexpr (HAS_NEXT) load_a(areg[BUF], A[(S2 - SLICES) % SLICES], u + 1);
                }
                mfma_a(op, BUF, sl_tag);
                if constexpr (PUBLISH) publish_a(areg[SLICES > 1 ? (BUF ^ 1) : 0], BUF ^ 1);
                __syncthreads();                              // the last one: the factor area is reused by the expand
            };
            step(std::integral_constant<int, 0>{});
            if constexpr (SLICES > 1) step(std::integral_constant<int, 1>{});
            if constexpr (SLICES > 2) step(std::integral_constant<int, 2>{});
        };
        constexpr std::integral_constant<bool, true> more{};
        constexpr std::integral_constant<bool, false> last{};
        constexpr std::integral_constant<int, 0> even{};
        constexpr std::integral_constant<int, SLICES & 1> second{};
        load_x(x0, 0);
        load_a(areg[0], A[0], 0);
        if constexpr (SLICES > 1) load_a(areg[1], A[1], 0);
        publish_a(areg[0], 0);
        __syncthreads();
        int u = 0;
        while (u + 2 < k_units) {
            unit(x0, x1, u, more, even);
            unit(x1, x0, u + 1, more, second);
            u += 2;
        }
        if (k_units - u == 2) {
            unit(x0, x1, u, more, even);
            unit(x1, x0, u + 1, last, second);
        } else {
            unit(x0, x1, u, last, even);
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
                for (int v = 0; v < 4; ++v) bias[v] = Elem<bf16_tag>::load1(bias_p, rank0 + v);
            }
        }
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) {
            float head_f[4], rem_f[4];
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const float zv = rank_ok ? (acc[b][mb][v] + bias[v]) * p.scale : 0.f;
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
    // B unit in LDS: column c of the unit at byte c * CS, its r factors contiguous; CS = 2r + 8.
    const int cs = 2 * r + 8;
    const int b_halves = 32 * r;                              // 8-byte halves of a B unit (128 columns x r factors)
    // where this thread's pieces land in LDS (the same for every unit): two 8-byte halves each,
    // a half never straddles a column because r % 4 == 0
    int b_dst[B_ITERS][2];
#pragma unroll
    for (int i = 0; i < B_ITERS; ++i)
#pragma unroll
        for (int hh = 0; hh < 2; ++hh) {
            const int byte = ((tid + i * NT) * 2 + hh) * 8;   // offset in the contiguous unit
            const int col = byte / (2 * r);
            b_dst[i][hh] = col * cs + (byte - col * 2 * r);
        }
    // byte offset of this lane's factors inside a B unit for MFMA e, rank block b, step 0
    int w_off[2][NB];
#pragma unroll
    for (int e = 0; e < 2; ++e)
#pragma unroll
        for (int b = 0; b < NB; ++b) {
            const int rank0 = 16 * b + 4 * g;
            w_off[e][b] = (2 * rl + e) * cs + (rank0 < r ? rank0 : 0) * 2;
        }

    auto expand_slice = [&](auto sl_tag) {
    constexpr int SL = decltype(sl_tag)::value;
    gcptr_t Bt = as_global(slice_Bt<SL>(p)[adapter]);
    const int64_t ldy_b = slice_ldy<SL>(p) * 2;
    gptr_t yu[MB][4];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int i = 0; i < 4; ++i) yu[mb][i] = as_global(slice_y<SL>(p)) + row_u[mb][i] * ldy_b + c16 * 16;

    auto load_b = [&](u32x4_t (&breg)[B_ITERS], int u) {
        gcptr_t base = Bt + (int64_t)u * 256 * r;             // 128 columns x r x 2 bytes
#pragma unroll
        for (int i = 0; i < B_ITERS; ++i) {
            const int piece = tid + i * NT;
            if (piece * 2 < b_halves) breg[i] = ld16(base + (int64_t)piece * 16);
        }
    };
    auto publish_b = [&](const u32x4_t (&breg)[B_ITERS], int buf) {
        char *fb = fac + buf * (128 * (32 * NB + 8));
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
            for (int i = 0; i < 4; ++i) raw[mb][i] = ld16_stream(yu[mb][i] + (int64_t)u * 256);
    };
    auto finish_unit = [&](const u32x4_t (&yop)[MB][4], int buf, int u) {
        const char *fb = fac + buf * (128 * (32 * NB + 8));
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            f32x4_t d[2][MB];
#pragma unroll
            for (int e = 0; e < 2; ++e) {
#pragma unroll
                for (int mb = 0; mb < MB; ++mb) d[e][mb] = f32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int b = 0; b < NB; ++b) {
                    const u32x2_t w = *reinterpret_cast<const u32x2_t *>(fb + s * 32 * cs + w_off[e][b]);
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
                if (row_ok[mb][i]) st16_stream(yu[mb][i] + (int64_t)u * 256, o);
            }
    };

    const int c_units = slice_d_out<SL>(p) >> 7;              // d_out % 128 == 0 (host-checked)
    {
        u32x4_t y0[MB][4], y1[MB][4], yop[MB][4], breg[B_ITERS];
        load_y(y0, 0);
        load_b(breg, 0);
        if constexpr (SL > 0) __syncthreads();                // the previous output's last unit is still being read
        publish_b(breg, 0);
        __syncthreads();
        int u = 0;
        while (u + 2 < c_units) {
            load_y(y1, u + 1);
            load_b(breg, u + 1);
            unit_to_mfma(y0, yop);
            finish_unit(yop, u & 1, u);
            publish_b(breg, (u + 1) & 1);
            __syncthreads();
            load_y(y0, u + 2);
            load_b(breg, u + 2);
            unit_to_mfma(y1, yop);
            finish_unit(yop, (u + 1) & 1, u + 1);
            publish_b(breg, u & 1);
            __syncthreads();
            u += 2;
        }
        if (c_units - u == 2) {
            load_y(y1, u + 1);
            load_b(breg, u + 1);
            unit_to_mfma(y0, yop);
            finish_unit(yop, u & 1, u);
            publish_b(breg, (u + 1) & 1);
            __syncthreads();
            unit_to_mfma(y1, yop);
            finish_unit(yop, (u + 1) & 1, u + 1);
        } else {
            unit_to_mfma(y0, yop);
            finish_unit(yop, u & 1, u);
        }
    }
    };
    expand_slice(std::integral_constant<int, 0>{});
    if constexpr (SLICES > 1) expand_slice(std::integral_constant<int, 1>{});
    if constexpr (SLICES > 2) expand_slice(std::integral_constant<int, 2>{});
}

// Packed launches carry SLICES * NB accumulator blocks: the register allocation is held to two
// wavefronts per SIMD (two workgroups of four wavefronts per compute unit), which the unpacked
// shapes reach by themselves.
template <int NB, int MB, int WAVES, bool DIREFT, int SLICES = 1>
__global__ __launch_bounds__(WAVES * 64, (SLICES > 1 && WAVES == 4) ? 2 : 1) void mfma_wide_kernel(ApplyArgs p)
{
    mfma_wide_body<NB, MB, WAVES, DIREFT, SLICES>(p);
}

// the same for one of several residual streams (in-place calls): blockIdx.y is the layer
template <int NB, int MB, int WAVES>
__global__ __launch_bounds__(WAVES * 64) void mfma_wide_layers_kernel(ApplyArgs p)
{
    select_layer(p);
    mfma_wide_body<NB, MB, WAVES, true>(p);
}

}  // namespace preft
