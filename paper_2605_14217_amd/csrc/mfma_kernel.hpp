// MFMA tile kernel (bf16 storage, fp32 accumulation), rank a multiple of 4 up to 128.
//
// One workgroup owns a tile of R = 16 * MB * WAVES consecutive active rows of one segment;
// each wavefront owns 16 * MB of them for the whole pass, so no data crosses wavefronts:
//
//   shrink (Eq. 2: z = A x;  Eq. 3: z = A h + b), per 32 columns of the row:
//       v_mfma_f32_16x16x32_bf16 with  A-operand = 16 ranks x 32 columns of the adapter's
//       [r, d_in] factor, B-operand = 32 columns x 16 rows of activations.  Lane (l%16, l/16)
//       loads 16 contiguous bytes of "its" row for both operands, straight from global
//       memory into the operand registers.  The accumulator leaves lane (row, g) holding
//       z[row][16b + 4g .. 16b + 4g + 3] for rank block b.
//   expand (Eq. 2: y += s B z;  Eq. 3: h += s B^T z), per 32 columns of the output row:
//       two MFMAs per rank block with  A-operand = 16 output columns x (16 ranks, twice) of
//       the [d_out, r] factor, B-operand = z split into a bf16 head and a bf16 remainder
//       (k index 8g + j: j < 4 the head of rank 16b + 4g + j, j >= 4 the remainder of rank
//       16b + 4g + j - 4), so the fp32 intermediate is not rounded to bf16.  The 16 columns
//       of MFMA e are c0 + 8(m/4) + 4e + m%4, which leaves lane (row, g) holding the 8
//       consecutive outputs y[row][c0 + 8g .. c0 + 8g + 7]: one 16-byte load and one 16-byte
//       store per lane, the same ownership as the activation operand of the shrink.
//
// The rank-r intermediate therefore never leaves the register file (the LDS is not needed:
// the accumulator layout of the shrink is already the operand layout of the expand).
#pragma once
#include "common.hpp"

namespace preft {

__device__ __forceinline__ bf16x8_t as_bf16x8(u32x4_t v) { return __builtin_bit_cast(bf16x8_t, v); }

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

template <int NB, int MB, int WAVES, bool DIREFT>
__global__ __launch_bounds__(WAVES * 64) void mfma_tile_kernel(ApplyArgs p)
{
    constexpr int R = 16 * MB * WAVES;
    constexpr int TPC = CHUNK_ROWS / R;
    static_assert(CHUNK_ROWS % R == 0, "tile height must divide the chunk height");
    // 32-column steps whose loads are in flight together (about 4 KB of activations a wave)
    constexpr int US = (NB * MB >= 8) ? 2 : 4;
    constexpr int UE = (NB * MB >= 8) ? 1 : (NB * MB >= 4 ? 2 : 4);

    const int unit = xcd_unit(p.header[0] * TPC);
    if (unit < 0) return;
    const int4 ch = p.chunks[unit / TPC];
    const int tile_row0 = (unit % TPC) * R;
    if (tile_row0 >= ch.z) return;
    const int adapter = ch.x;
    const int n_rows = min(R, ch.z - tile_row0);              // rows of this tile

    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int rl = lane & 15, g = lane >> 4;
    const int wave_row0 = wave * 16 * MB;
    if (wave_row0 >= n_rows) return;                          // whole wavefront idle

    const int r = p.rank;
    const int64_t ldx_b = p.ldx * 2, ldy_b = p.ldy * 2;
    gcptr_t A  = as_global(p.A_pool[adapter]);
    gcptr_t Bt = as_global(p.Bt_pool[adapter]);

    // Row slots past the end of the tile alias its last row (which this wavefront owns): they
    // load the same bytes, compute the same values and store the same bits, so no access in
    // the sweeps below depends on the row.
    gcptr_t xp[MB];
    gptr_t yp[MB];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
        const int t = wave_row0 + mb * 16 + rl;
        const int64_t row = (int64_t)ch.y + tile_row0 + min(t, n_rows - 1);
        xp[mb] = as_global(p.x) + row * ldx_b + g * 16;
        yp[mb] = as_global(p.y) + row * ldy_b + g * 16;
    }

    // ---------------------------------------------------------------- shrink
    f32x4_t acc[NB][MB];
#pragma unroll
    for (int b = 0; b < NB; ++b)
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) acc[b][mb] = f32x4_t{0.f, 0.f, 0.f, 0.f};

    // Ranks past r alias rank r-1; their z entries are zeroed below.
    gcptr_t ap[NB];
#pragma unroll
    for (int b = 0; b < NB; ++b) ap[b] = A + ((int64_t)min(16 * b + rl, r - 1) * p.d_in + g * 8) * 2;

    const int k_full = p.d_in >> 5;                           // whole 32-column steps
    int ks = 0;
    // US steps per trip: all loads of a trip are issued before its first MFMA
    for (; ks + US <= k_full; ks += US) {
        bf16x8_t xv[US][MB], av[US][NB];
#pragma unroll
        for (int u = 0; u < US; ++u) {
#pragma unroll
            for (int mb = 0; mb < MB; ++mb) xv[u][mb] = as_bf16x8(ld16(xp[mb] + (int64_t)(ks + u) * 64));
#pragma unroll
            for (int b = 0; b < NB; ++b) av[u][b] = as_bf16x8(ld16(ap[b] + (int64_t)(ks + u) * 64));
        }
#pragma unroll
        for (int u = 0; u < US; ++u)
#pragma unroll
            for (int b = 0; b < NB; ++b)
#pragma unroll
                for (int mb = 0; mb < MB; ++mb)
                    acc[b][mb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av[u][b], xv[u][mb], acc[b][mb], 0, 0, 0);
    }
    for (; ks < k_full; ++ks) {
        bf16x8_t xv[MB];
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) xv[mb] = as_bf16x8(ld16(xp[mb] + (int64_t)ks * 64));
#pragma unroll
        for (int b = 0; b < NB; ++b) {
            const bf16x8_t av = as_bf16x8(ld16(ap[b] + (int64_t)ks * 64));
#pragma unroll
            for (int mb = 0; mb < MB; ++mb)
                acc[b][mb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, xv[mb], acc[b][mb], 0, 0, 0);
        }
    }
    if (p.d_in & 31) {                                        // last, partial step (d_in % 8 == 0)
        const bool col_ok = (k_full * 32 + g * 8) < p.d_in;
        const u32x4_t zero = {0u, 0u, 0u, 0u};
        bf16x8_t xv[MB];
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
            xv[mb] = as_bf16x8(col_ok ? ld16(xp[mb] + (int64_t)k_full * 64) : zero);
#pragma unroll
        for (int b = 0; b < NB; ++b) {
            const bf16x8_t av = as_bf16x8(col_ok ? ld16(ap[b] + (int64_t)k_full * 64) : zero);
#pragma unroll
            for (int mb = 0; mb < MB; ++mb)
                acc[b][mb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, xv[mb], acc[b][mb], 0, 0, 0);
        }
    }

    // ---------------------------------------------------------------- z -> expand operand
    // lane (row rl, g) holds z[row][16b + 4g + v]; add the bias, apply the prefactor, zero the
    // padding ranks, and split into bf16 head + bf16 remainder.
    bf16x8_t zop[NB][MB];
#pragma unroll
    for (int b = 0; b < NB; ++b) {
        const int rank0 = 16 * b + 4 * g;
        const bool rank_ok = rank0 < r;                       // r % 4 == 0: all four or none
        float bias[4] = {0.f, 0.f, 0.f, 0.f};
        if (DIREFT && p.bias_pool && rank_ok) {
            gcptr_t bp_ = as_global(p.bias_pool[adapter]);
#pragma unroll
            for (int v = 0; v < 4; ++v) bias[v] = Elem<bf16_tag>::load1(bp_, rank0 + v);
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

    // ---------------------------------------------------------------- expand
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

    const int c_full = p.d_out >> 5;
    int cs = 0;
    for (; cs + UE <= c_full; cs += UE) {
        u32x4_t yv[UE][MB];
        u32x2_t wv[UE][2][NB];
#pragma unroll
        for (int u = 0; u < UE; ++u) {
#pragma unroll
            for (int mb = 0; mb < MB; ++mb) yv[u][mb] = ld16(yp[mb] + (int64_t)(cs + u) * 64);
#pragma unroll
            for (int e = 0; e < 2; ++e)
#pragma unroll
                for (int b = 0; b < NB; ++b)
                    wv[u][e][b] = ld8(bp[e][b] + (cs + u) * w_step);
        }
#pragma unroll
        for (int u = 0; u < UE; ++u) {
            float out[MB][8];
#pragma unroll
            for (int e = 0; e < 2; ++e) {
                f32x4_t d[MB];
#pragma unroll
                for (int mb = 0; mb < MB; ++mb) d[mb] = f32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int b = 0; b < NB; ++b) {
                    const u32x2_t w = wv[u][e][b];
                    const bf16x8_t wop = as_bf16x8(u32x4_t{w[0], w[1], w[0], w[1]});
#pragma unroll
                    for (int mb = 0; mb < MB; ++mb)
                        d[mb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wop, zop[b][mb], d[mb], 0, 0, 0);
                }
#pragma unroll
                for (int mb = 0; mb < MB; ++mb) {
                    out[mb][4 * e + 0] = bf16_lo(yv[u][mb][2 * e]) + d[mb][0];
                    out[mb][4 * e + 1] = bf16_hi(yv[u][mb][2 * e]) + d[mb][1];
                    out[mb][4 * e + 2] = bf16_lo(yv[u][mb][2 * e + 1]) + d[mb][2];
                    out[mb][4 * e + 3] = bf16_hi(yv[u][mb][2 * e + 1]) + d[mb][3];
                }
            }
#pragma unroll
            for (int mb = 0; mb < MB; ++mb)
                st16(yp[mb] + (int64_t)(cs + u) * 64, Elem<bf16_tag>::pack(out[mb]));
        }
    }
    for (; cs < c_full; ++cs) {
        u32x4_t yv[MB];
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) yv[mb] = ld16(yp[mb] + (int64_t)cs * 64);
        float out[MB][8];
#pragma unroll
        for (int e = 0; e < 2; ++e) {
            f32x4_t d[MB];
#pragma unroll
            for (int mb = 0; mb < MB; ++mb) d[mb] = f32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int b = 0; b < NB; ++b) {
                const u32x2_t w = ld8(bp[e][b] + cs * w_step);
                const bf16x8_t wop = as_bf16x8(u32x4_t{w[0], w[1], w[0], w[1]});
#pragma unroll
                for (int mb = 0; mb < MB; ++mb)
                    d[mb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wop, zop[b][mb], d[mb], 0, 0, 0);
            }
#pragma unroll
            for (int mb = 0; mb < MB; ++mb) {
                out[mb][4 * e + 0] = bf16_lo(yv[mb][2 * e]) + d[mb][0];
                out[mb][4 * e + 1] = bf16_hi(yv[mb][2 * e]) + d[mb][1];
                out[mb][4 * e + 2] = bf16_lo(yv[mb][2 * e + 1]) + d[mb][2];
                out[mb][4 * e + 3] = bf16_hi(yv[mb][2 * e + 1]) + d[mb][3];
            }
        }
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
            st16(yp[mb] + (int64_t)cs * 64, Elem<bf16_tag>::pack(out[mb]));
    }
    if (p.d_out & 31) {                                       // last, partial step (d_out % 8 == 0)
        const int c0 = c_full * 32;
        const bool col_ok = (c0 + g * 8) < p.d_out;
        u32x4_t yv[MB];
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
            yv[mb] = col_ok ? ld16(yp[mb] + (int64_t)c_full * 64) : u32x4_t{0u, 0u, 0u, 0u};
        float out[MB][8];
#pragma unroll
        for (int e = 0; e < 2; ++e) {
            f32x4_t d[MB];
#pragma unroll
            for (int mb = 0; mb < MB; ++mb) d[mb] = f32x4_t{0.f, 0.f, 0.f, 0.f};
            // this lane's weight column may lie past d_out: alias the last column (its
            // products land in outputs that are not stored)
            const int col = c0 + 8 * (rl >> 2) + 4 * e + (rl & 3);
            const int64_t back = col < p.d_out ? 0 : (int64_t)(col - (p.d_out - 1)) * r * 2;
#pragma unroll
            for (int b = 0; b < NB; ++b) {
                const u32x2_t w = ld8(bp[e][b] + c_full * w_step - back);
                const bf16x8_t wop = as_bf16x8(u32x4_t{w[0], w[1], w[0], w[1]});
#pragma unroll
                for (int mb = 0; mb < MB; ++mb)
                    d[mb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wop, zop[b][mb], d[mb], 0, 0, 0);
            }
#pragma unroll
            for (int mb = 0; mb < MB; ++mb) {
                out[mb][4 * e + 0] = bf16_lo(yv[mb][2 * e]) + d[mb][0];
                out[mb][4 * e + 1] = bf16_hi(yv[mb][2 * e]) + d[mb][1];
                out[mb][4 * e + 2] = bf16_lo(yv[mb][2 * e + 1]) + d[mb][2];
                out[mb][4 * e + 3] = bf16_hi(yv[mb][2 * e + 1]) + d[mb][3];
            }
        }
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
            if (col_ok) st16(yp[mb] + (int64_t)c_full * 64, Elem<bf16_tag>::pack(out[mb]));
    }
}

}  // namespace preft
