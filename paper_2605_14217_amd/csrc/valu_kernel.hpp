// Vector-ALU tile kernel for small ranks (bf16 storage, fp32 accumulation, rank 1..8).
//
// At rank <= 8 the contraction is too thin for the matrix cores to matter: the pass is a
// pure stream over the activations with r multiply-adds per element.  One wavefront owns
// RB rows at a time and sweeps them with 16-byte loads, 64 lanes side by side:
//
//   shrink (Eq. 2: z = A x;  Eq. 3: z = A h + b): every lane keeps RB x r partial sums over
//           its columns (packed bf16 dot products, fp32 accumulate); one wavefront
//           reduction per (row, rank) finishes z.  The adapter's factor is loaded once per
//           RB rows.
//   expand (Eq. 2: y += s B z;  Eq. 3: h += s B^T z): a lane owns 8 consecutive output
//           columns; their 8 x r factors are contiguous in the [d_out, r] layout and are
//           converted once per RB rows.
//
// A workgroup of WAVES wavefronts owns a tile of RB * WAVES consecutive rows of a chunk;
// wavefronts never exchange data.
//
// HV > 0 (in place only): the wavefront's rows stay in registers between the sweeps, HV 16-byte
// vectors per lane and row, so rows of up to 512 HV elements are read once and written once.
//
// SLICES > 1 (LoRA only): packed projections, as in mfma_tile_kernel: the outputs share x, so
// one shrink sweep feeds SLICES * RANK partial sums per row and one expand sweep per output follows.
#pragma once
#include "common.hpp"
#include "mfma_kernel.hpp"   // xcd_unit

namespace preft {

// acc + a.lo * b.lo + a.hi * b.hi on packed bf16 pairs, fp32 accumulate (v_dot2c_f32_bf16).
// The operands are taken by value: a bit cast applied directly to a vector-element lvalue
// reads element 0 of the vector.
__device__ __forceinline__ float dot2_bf16(uint32_t a, uint32_t b, float acc)
{
    return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, a), __builtin_bit_cast(bf16x2_t, b), acc, false);
}

template <int RANK, int RB, int WAVES, bool DIREFT, int SLICES = 1, int HV = 0>
__device__ __forceinline__ void valu_tile_body(const ApplyArgs &p)
{
    constexpr int R = RB * WAVES;
    static_assert(HV == 0 || DIREFT, "only an in-place call keeps its rows between the sweeps");
    constexpr int RT = RANK * SLICES;                         // partial sums per row in the shrink sweep
    static_assert(SLICES == 1 || !DIREFT, "packed projections are a LoRA feature");
    static_assert(CHUNK_ROWS % R == 0, "tile height must divide the chunk height");

    if (!schedule_matches(p)) return;
    int n_chunk_units;
    const int unit = xcd_unit(tile_units<R>(p, &n_chunk_units));
    if (unit < 0) return;
    TileRows tile;
    if (!tile_rows<R>(p, unit, n_chunk_units, tile)) return;
    const int adapter = tile.adapter;
    const int n_rows = tile.n_rows;

    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int wave_row0 = wave * RB;
    if (wave_row0 >= n_rows) return;

    gcptr_t A[SLICES];
    A[0] = as_global(slice_A<0>(p)[adapter]);
    if constexpr (SLICES > 1) A[1] = as_global(slice_A<1>(p)[adapter]);
    if constexpr (SLICES > 2) A[2] = as_global(slice_A<2>(p)[adapter]);
    const int64_t ldx_b = p.ldx * 2;

    // Row slots past the end of the tile alias its last row (which this wavefront owns): they
    // load the same bytes, compute the same values and store the same bits, so no access in
    // the sweeps below is conditional.
    gcptr_t xp[RB];
    int64_t rows[RB];
#pragma unroll
    for (int i = 0; i < RB; ++i) {
        rows[i] = tile.row(wave_row0 + i);
        xp[i] = as_global(p.x) + rows[i] * ldx_b;
    }

    // ---------------------------------------------------------------- shrink
    float z[RB][RT];
#pragma unroll
    for (int i = 0; i < RB; ++i)
#pragma unroll
        for (int k = 0; k < RT; ++k) z[i][k] = 0.f;

    const int nvec_in = p.d_in >> 3;                          // 16-byte vectors per row
    auto shrink_step = [&](const u32x4_t (&xv)[RB], const u32x4_t (&av)[RT]) {
#pragma unroll
        for (int k = 0; k < RT; ++k)
#pragma unroll
            for (int i = 0; i < RB; ++i)
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    z[i][k] = dot2_bf16(xv[i][q], av[k][q], z[i][k]);
    };
    // HV > 0 (in place, rows of at most 512 HV elements): the wavefront keeps its RB rows in
    // registers between the sweeps -- lane l holds the 16-byte vectors l, l + 64, ... of each row --
    // so h is read once and written once.
    u32x4_t hreg[RB][HV > 0 ? HV : 1];
    int c = lane;
    if constexpr (HV > 0) {
#pragma unroll
        for (int v = 0; v < HV; ++v) {
            const int cv = lane + 64 * v;
            if (cv < nvec_in) {
                u32x4_t xv[RB], av[RT];
#pragma unroll
                for (int i = 0; i < RB; ++i) xv[i] = ld16_stream(xp[i] + (int64_t)cv * 16);
#pragma unroll
                for (int k = 0; k < RT; ++k) av[k] = ld16(A[k / RANK] + ((int64_t)(k % RANK) * p.d_in + (int64_t)cv * 8) * 2);
                shrink_step(xv, av);
#pragma unroll
                for (int i = 0; i < RB; ++i) hreg[i][v] = xv[i];
            }
        }
        c = nvec_in;                                          // nothing left for the streamed loops
    }
    for (; c + 64 < nvec_in; c += 128) {                      // two sweeps in flight
        u32x4_t xv0[RB], xv1[RB], av0[RT], av1[RT];
#pragma unroll
        for (int i = 0; i < RB; ++i) {
            xv0[i] = ld16_first<DIREFT>(xp[i] + (int64_t)c * 16);
            xv1[i] = ld16_first<DIREFT>(xp[i] + (int64_t)(c + 64) * 16);
        }
#pragma unroll
        for (int k = 0; k < RT; ++k) {
            av0[k] = ld16(A[k / RANK] + ((int64_t)(k % RANK) * p.d_in + (int64_t)c * 8) * 2);
            av1[k] = ld16(A[k / RANK] + ((int64_t)(k % RANK) * p.d_in + (int64_t)(c + 64) * 8) * 2);
        }
        shrink_step(xv0, av0);
        shrink_step(xv1, av1);
    }
    for (; c < nvec_in; c += 64) {
        u32x4_t xv[RB], av[RT];
#pragma unroll
        for (int i = 0; i < RB; ++i) xv[i] = ld16_first<DIREFT>(xp[i] + (int64_t)c * 16);
#pragma unroll
        for (int k = 0; k < RT; ++k) av[k] = ld16(A[k / RANK] + ((int64_t)(k % RANK) * p.d_in + (int64_t)c * 8) * 2);
        shrink_step(xv, av);
    }
    gcptr_t bias_p = DIREFT ? bias_of(p, adapter) : nullptr;
#pragma unroll
    for (int k = 0; k < RT; ++k) {
        float bias = 0.f;
        if (DIREFT && bias_p) bias = Elem<bf16_tag>::load1(bias_p, k);
#pragma unroll
        for (int i = 0; i < RB; ++i) z[i][k] = (wave_sum(z[i][k]) + bias) * p.scale;
    }

    // ---------------------------------------------------------------- expand (once per output)
    auto expand_slice = [&](auto sl_tag) {
        constexpr int SL = decltype(sl_tag)::value;
        gcptr_t Bt = as_global(slice_Bt<SL>(p)[adapter]);
        const int64_t ldy_b = slice_ldy<SL>(p) * 2;
        gptr_t yp[RB];
#pragma unroll
        for (int i = 0; i < RB; ++i) yp[i] = as_global(slice_y<SL>(p)) + rows[i] * ldy_b;
        const int nvec_out = slice_d_out<SL>(p) >> 3;
        if constexpr (HV > 0) {
#pragma unroll
            for (int v = 0; v < HV; ++v) {
                const int c = lane + 64 * v;
                if (c < nvec_out) {
                    float w[8 * RANK];
                    gcptr_t wp = Bt + (int64_t)c * 8 * RANK * 2;
#pragma unroll
                    for (int j = 0; j < RANK; ++j) {
                        const u32x4_t raw = ld16(wp + j * 16);
#pragma unroll
                        for (int q = 0; q < 4; ++q) {
                            w[j * 8 + 2 * q] = bf16_lo(raw[q]);
                            w[j * 8 + 2 * q + 1] = bf16_hi(raw[q]);
                        }
                    }
#pragma unroll
                    for (int i = 0; i < RB; ++i) {
                        float out[8];
                        Elem<bf16_tag>::unpack(hreg[i][v], out);
#pragma unroll
                        for (int col = 0; col < 8; ++col) {
                            float d = 0.f;
#pragma unroll
                            for (int k = 0; k < RANK; ++k) d = fmaf(w[col * RANK + k], z[i][SL * RANK + k], d);
                            out[col] += d;
                        }
                        st16_stream(yp[i] + (int64_t)c * 16, Elem<bf16_tag>::pack(out));
                    }
                }
            }
            return;
        }
        for (int c = lane; c < nvec_out; c += 64) {
            // 8 columns x RANK factors, contiguous: RANK 16-byte vectors
            float w[8 * RANK];
            gcptr_t wp = Bt + (int64_t)c * 8 * RANK * 2;
#pragma unroll
            for (int j = 0; j < RANK; ++j) {
                const u32x4_t raw = ld16(wp + j * 16);
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    w[j * 8 + 2 * q] = bf16_lo(raw[q]);
                    w[j * 8 + 2 * q + 1] = bf16_hi(raw[q]);
                }
            }
            u32x4_t yv[RB];
#pragma unroll
            for (int i = 0; i < RB; ++i) yv[i] = ld16_stream(yp[i] + (int64_t)c * 16);
#pragma unroll
            for (int i = 0; i < RB; ++i) {
                float out[8];
                Elem<bf16_tag>::unpack(yv[i], out);
#pragma unroll
                for (int col = 0; col < 8; ++col) {
                    float d = 0.f;
#pragma unroll
                    for (int k = 0; k < RANK; ++k) d = fmaf(w[col * RANK + k], z[i][SL * RANK + k], d);
                    out[col] += d;
                }
                st16_stream(yp[i] + (int64_t)c * 16, Elem<bf16_tag>::pack(out));
            }
        }
    };
    expand_slice(std::integral_constant<int, 0>{});
    if constexpr (SLICES > 1) expand_slice(std::integral_constant<int, 1>{});
    if constexpr (SLICES > 2) expand_slice(std::integral_constant<int, 2>{});
}

template <int RANK, int RB, int WAVES, bool DIREFT, int SLICES = 1, int HV = 0>
__global__ __launch_bounds__(WAVES * 64) void valu_tile_kernel(ApplyArgs p)
{
    valu_tile_body<RANK, RB, WAVES, DIREFT, SLICES, HV>(p);
}

// the same for one of several residual streams (in-place calls): blockIdx.y is the layer
template <int RANK, int RB, int WAVES, int HV = 0>
__global__ __launch_bounds__(WAVES * 64) void valu_tile_layers_kernel(ApplyArgs p)
{
    select_layer(p);
    valu_tile_body<RANK, RB, WAVES, true, 1, HV>(p);
}

}  // namespace preft
