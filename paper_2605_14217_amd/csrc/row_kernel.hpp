// Per-row ("batched gather matrix-vector") kernel: one workgroup applies one adapter to a group
// of at most GROUP_ROWS rows that share it.
//
// This is the generic fallback for element types and ranks the tile kernels do not cover (fp32;
// bf16 ranks that are neither <= 8 nor multiples of 4): a chunk is cut into groups of consecutive
// rows, and the short rows (decode tokens of the all-position baseline, segments with at most
// SHORT_ROWS active rows), which the scheduler has sorted by adapter and cut into gathered tiles,
// into groups of rows of one adapter -- an adapter's factors are streamed once per group rather
// than once per row, the per-request gather cost the paper's Sec. 3.2 attributes to decode time.
//
//   shrink  (Eq. 2: A x;  Eq. 3: A h + b):  wavefront w owns ranks w, w+4, ... (two at a time);
//           its 64 lanes sweep the rows with 16-byte loads, every factor vector is used for all
//           rows of the group, one wavefront reduction per (row, rank) finishes z (LDS).
//   expand  (Eq. 2: y + s B z;  Eq. 3: h + s B^T z):  the [d_out, r] factor is read as one
//           contiguous stream of 16-byte vectors; a vector holds part of one column (r >= 8
//           elements per vector: the lanes of a column combine with xor-shuffles) or several
//           whole columns (small r).  Ranks that fit neither pattern take one column per thread.
#pragma once
#include "common.hpp"

namespace preft {

constexpr int ROW_THREADS = 256;
constexpr int ROW_KG = 2;                         // ranks per wavefront pass in the shrink

template <typename E>
__device__ __forceinline__ float dot_vec(u32x4_t a, u32x4_t b, float acc)
{
    if constexpr (Elem<E>::BYTES == 2) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const uint32_t ua = a[q], ub = b[q];
            acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, ua), __builtin_bit_cast(bf16x2_t, ub), acc, false);
        }
    } else {
#pragma unroll
        for (int q = 0; q < 4; ++q) acc = fmaf(__uint_as_float(a[q]), __uint_as_float(b[q]), acc);
    }
    return acc;
}

// One column per thread (any rank): WB = bytes per factor load.
template <typename E, int WB>
__device__ __forceinline__ void expand_by_column(const ApplyArgs &p, gcptr_t Bt, gptr_t yrow, const float *z)
{
    constexpr int BYTES = Elem<E>::BYTES;
    const int row_bytes = p.rank * BYTES;
    for (int n = threadIdx.x; n < p.d_out; n += ROW_THREADS) {
        gcptr_t w = Bt + (int64_t)n * row_bytes;
        float acc = 0.f;
        for (int o = 0; o < row_bytes; o += WB) {
            const int k = o / BYTES;
            if constexpr (WB == 4 && BYTES == 2) {
                const uint32_t raw = ld4(w + o);
                acc = fmaf(bf16_lo(raw), z[k], acc);
                acc = fmaf(bf16_hi(raw), z[k + 1], acc);
            } else {
                acc = fmaf(Elem<E>::load1(w, k), z[k], acc);
            }
        }
        Elem<E>::store1(yrow, n, Elem<E>::load1(yrow, n) + acc);
    }
}

// Small ranks: a 16-byte vector holds all R factors of V / R whole columns.
template <typename E, int R>
__device__ __forceinline__ void expand_whole_columns(const ApplyArgs &p, gcptr_t Bt, gptr_t (&yrow)[GROUP_ROWS], int count,
                                                     const float *z)
{
    constexpr int V = Elem<E>::V;
    constexpr int CPL = V / R;                                  // columns per vector
    static_assert(V % R == 0, "rank must divide the vector length");
    const int n_vec = p.d_out / CPL;                            // d_out % V == 0
    for (int jc = threadIdx.x; jc < n_vec; jc += ROW_THREADS) {
        float wf[V];
        Elem<E>::unpack(ld16(Bt + (int64_t)jc * 16), wf);
        float yv[GROUP_ROWS][CPL];
#pragma unroll
        for (int j = 0; j < GROUP_ROWS; ++j)
#pragma unroll
            for (int cc = 0; cc < CPL; ++cc) yv[j][cc] = j < count ? Elem<E>::load1(yrow[j], jc * CPL + cc) : 0.f;
#pragma unroll
        for (int j = 0; j < GROUP_ROWS; ++j) {
            if (j < count) {
                const float *zj = z + j * PREFT_MAX_RANK_DEV;
#pragma unroll
                for (int cc = 0; cc < CPL; ++cc) {
                    float d = 0.f;
#pragma unroll
                    for (int k = 0; k < R; ++k) d = fmaf(wf[cc * R + k], zj[k], d);
                    Elem<E>::store1(yrow[j], jc * CPL + cc, yv[j][cc] + d);
                }
            }
        }
    }
}

// Applies adapter `adapter` to rows rows[0..count) (count <= GROUP_ROWS, rows distinct).
// z: LDS scratch of GROUP_ROWS * PREFT_MAX_RANK floats.  Must be called by the whole workgroup.
template <typename E, bool DIREFT>
__device__ __forceinline__ void group_apply(const ApplyArgs &p, int adapter, const int (&rows)[GROUP_ROWS], int count,
                                            float *z)
{
    constexpr int V = Elem<E>::V;                 // elements per 16-byte vector
    constexpr int BYTES = Elem<E>::BYTES;
    constexpr int G = GROUP_ROWS;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int r = p.rank;
    gcptr_t A  = as_global(p.A_pool[adapter]);
    gcptr_t Bt = as_global(p.Bt_pool[adapter]);
    gcptr_t bias = DIREFT ? bias_of(p, adapter) : nullptr;        // null: no table, or a null entry
    gcptr_t xrow[G];
    gptr_t yrow[G];
#pragma unroll
    for (int j = 0; j < G; ++j) {
        const int row = j < count ? rows[j] : rows[0];
        xrow[j] = as_global(p.x) + (int64_t)row * p.ldx * BYTES;
        yrow[j] = as_global(p.y) + (int64_t)row * p.ldy * BYTES;
    }

    // ---------------------------------------------------------------- shrink
    const int nvec = p.d_in / V;
    const int64_t a_row = (int64_t)p.d_in * BYTES;
    for (int k0 = wave * ROW_KG; k0 < r; k0 += (ROW_THREADS / 64) * ROW_KG) {
        float acc[G][ROW_KG];
#pragma unroll
        for (int j = 0; j < G; ++j)
#pragma unroll
            for (int kk = 0; kk < ROW_KG; ++kk) acc[j][kk] = 0.f;
        const bool second = (k0 + 1) < r;                       // uniform over the wavefront
        gcptr_t A0 = A + (int64_t)k0 * a_row;
        gcptr_t A1 = A + (int64_t)(second ? k0 + 1 : k0) * a_row;
        constexpr int UC = 4;                                   // vectors in flight per lane and stream
        const u32x4_t zero = {0u, 0u, 0u, 0u};
        for (int c0 = lane; c0 < nvec; c0 += 64 * UC) {
            u32x4_t a0[UC], a1[UC], xv[UC][G];
#pragma unroll
            for (int u = 0; u < UC; ++u) {
                const int c = c0 + 64 * u;
                const bool ok = c < nvec;
                a0[u] = ok ? ld16(A0 + (int64_t)c * 16) : zero;
                a1[u] = ok ? ld16(A1 + (int64_t)c * 16) : zero;
#pragma unroll
                for (int j = 0; j < G; ++j) xv[u][j] = (ok && j < count) ? ld16(xrow[j] + (int64_t)c * 16) : zero;
            }
#pragma unroll
            for (int u = 0; u < UC; ++u)
#pragma unroll
                for (int j = 0; j < G; ++j) {
                    acc[j][0] = dot_vec<E>(xv[u][j], a0[u], acc[j][0]);
                    acc[j][1] = dot_vec<E>(xv[u][j], a1[u], acc[j][1]);
                }
        }
#pragma unroll
        for (int j = 0; j < G; ++j)
#pragma unroll
            for (int kk = 0; kk < ROW_KG; ++kk) {
                const float s = wave_sum(acc[j][kk]);
                if (lane == 0 && k0 + kk < r) {
                    const float b = bias ? Elem<E>::load1(bias, k0 + kk) : 0.f;
                    z[j * PREFT_MAX_RANK_DEV + k0 + kk] = (s + b) * p.scale;
                }
            }
    }
    __syncthreads();          // z complete; for DiReFT also: every read of the rows precedes every write

    // ---------------------------------------------------------------- expand
    const int lpc = r / V;                                      // lanes per column when r % V == 0
    const bool by_lanes = (r % V) == 0 && (lpc & (lpc - 1)) == 0 && lpc <= 64;
    const bool by_cols = r < V && (V % r) == 0;
    if (by_lanes) {
        // vector jc holds elements k0 .. k0+V-1 of column jc / lpc
        const int n_vec = p.d_out * lpc;
        const int lpc_shift = __ffs(lpc) - 1;
        constexpr int UE = 4;
        const bool leader = (threadIdx.x & (lpc - 1)) == 0;
        // a thread meets the same V ranks in every vector it takes (the stride is a multiple of lpc)
        float zr[G][V];
        {
            const int k0 = (threadIdx.x & (lpc - 1)) * V;
#pragma unroll
            for (int j = 0; j < G; ++j)
#pragma unroll
                for (int i = 0; i < V; ++i) zr[j][i] = z[j * PREFT_MAX_RANK_DEV + k0 + i];
        }
        for (int jc0 = threadIdx.x; jc0 < n_vec; jc0 += ROW_THREADS * UE) {
            u32x4_t wraw[UE];
            float yv[UE][G];
#pragma unroll
            for (int u = 0; u < UE; ++u) {
                const int jc = jc0 + ROW_THREADS * u;
                const bool ok = jc < n_vec;                     // uniform over the lanes of a column
                wraw[u] = ok ? ld16(Bt + (int64_t)jc * 16) : u32x4_t{0u, 0u, 0u, 0u};
#pragma unroll
                for (int j = 0; j < G; ++j)
                    yv[u][j] = (ok && leader && j < count) ? Elem<E>::load1(yrow[j], jc >> lpc_shift) : 0.f;
            }
#pragma unroll
            for (int u = 0; u < UE; ++u) {
                const int jc = jc0 + ROW_THREADS * u;
                const bool ok = jc < n_vec;
                float wf[V];
                Elem<E>::unpack(wraw[u], wf);
#pragma unroll
                for (int j = 0; j < G; ++j) {
                    float part = 0.f;
#pragma unroll
                    for (int i = 0; i < V; ++i) part = fmaf(wf[i], zr[j][i], part);
                    for (int o = 1; o < lpc; o <<= 1) part += __shfl_xor(part, o, 64);
                    if (ok && leader && j < count) Elem<E>::store1(yrow[j], jc >> lpc_shift, yv[u][j] + part);
                }
            }
        }
    } else if (by_cols) {
        switch (r) {
        case 1: expand_whole_columns<E, 1>(p, Bt, yrow, count, z); break;
        case 2: expand_whole_columns<E, 2>(p, Bt, yrow, count, z); break;
        default: if constexpr (V == 8) expand_whole_columns<E, 4>(p, Bt, yrow, count, z); break;
        }
    } else {
        for (int j = 0; j < count; ++j) {
            if constexpr (BYTES == 2) {
                if ((r & 1) == 0) expand_by_column<E, 4>(p, Bt, yrow[j], z + j * PREFT_MAX_RANK_DEV);
                else              expand_by_column<E, 2>(p, Bt, yrow[j], z + j * PREFT_MAX_RANK_DEV);
            } else {
                expand_by_column<E, 4>(p, Bt, yrow[j], z + j * PREFT_MAX_RANK_DEV);
            }
        }
    }
    __syncthreads();          // z is reused by the next group
}

// Short rows: the schedule's gathered tiles (rows of one adapter) are cut into groups of at most
// GROUP_ROWS rows, fewer when the batch has few short rows so that a decode-only step still
// fills the chip; grid-stride over the groups.
template <typename E, bool DIREFT>
__device__ __forceinline__ void row_short_body(const ApplyArgs &p)
{
    __shared__ float z[GROUP_ROWS * PREFT_MAX_RANK_DEV];
    if (!schedule_matches(p)) return;
    const int grows = max(1, min(GROUP_ROWS, p.header[HDR_SHORT_ROWS] / 512));
    const int per_tile = (GTILE_ROWS + grows - 1) / grows;
    // tiles are sorted by adapter: deal contiguous runs to the 8 XCDs (workgroup ids go round-robin
    // over them) so that the groups of one adapter meet in one L2
    const int n = p.header[HDR_GTILES] * per_tile;
    const int per_xcd = (n + 7) >> 3;
    const int first = (blockIdx.x & 7) * per_xcd, last = min(first + per_xcd, n);
    for (int e = first + (blockIdx.x >> 3); e < last; e += gridDim.x >> 3) {
        const int4 gt = p.gtiles[e / per_tile];
        const int g0 = (e % per_tile) * grows;
        if (g0 >= gt.z) continue;                              // uniform over the workgroup
        const int count = min(grows, gt.z - g0);
        int rows[GROUP_ROWS];
#pragma unroll
        for (int j = 0; j < GROUP_ROWS; ++j) rows[j] = p.shorts[gt.y + g0 + min(j, count - 1)].y;
        group_apply<E, DIREFT>(p, gt.x, rows, count, z);
    }
}

// Generic fallback for chunks: one workgroup per GROUP_ROWS consecutive rows of a chunk.
template <typename E, bool DIREFT>
__device__ __forceinline__ void row_chunks_body(const ApplyArgs &p)
{
    __shared__ float z[GROUP_ROWS * PREFT_MAX_RANK_DEV];
    constexpr int PER_CHUNK = CHUNK_ROWS / GROUP_ROWS;
    if (!schedule_matches(p)) return;
    const int c = blockIdx.x / PER_CHUNK;
    if (c >= p.header[HDR_CHUNKS]) return;
    const int4 ch = p.chunks[c];
    const int first = (blockIdx.x % PER_CHUNK) * GROUP_ROWS;
    if (first >= ch.z) return;
    const int count = min(GROUP_ROWS, ch.z - first);
    int rows[GROUP_ROWS];
#pragma unroll
    for (int j = 0; j < GROUP_ROWS; ++j) rows[j] = ch.y + first + min(j, count - 1);
    group_apply<E, DIREFT>(p, ch.x, rows, count, z);
}

template <typename E, bool DIREFT>
__global__ __launch_bounds__(ROW_THREADS) void row_kernel_short(ApplyArgs p) { row_short_body<E, DIREFT>(p); }
template <typename E, bool DIREFT>
__global__ __launch_bounds__(ROW_THREADS) void row_kernel_chunks(ApplyArgs p) { row_chunks_body<E, DIREFT>(p); }

// the same for one of several residual streams (in-place calls): blockIdx.y is the layer
template <typename E>
__global__ __launch_bounds__(ROW_THREADS) void row_layers_kernel_short(ApplyArgs p)
{
    select_layer(p);
    row_short_body<E, true>(p);
}
template <typename E>
__global__ __launch_bounds__(ROW_THREADS) void row_layers_kernel_chunks(ApplyArgs p)
{
    select_layer(p);
    row_chunks_body<E, true>(p);
}

}  // namespace preft
