// Per-row ("batched gather matrix-vector") kernel: one workgroup applies one adapter to one row.
//
// This is the path of the conventional all-position baseline for decode tokens -- every row
// gathers its own adapter's factors, which is the memory-bound cost the paper's Sec. 3.2
// attributes to per-request adapters at decode time -- and of any segment with at most
// SHORT_ROWS active rows.  It is also the generic fallback for element types and ranks the
// tile kernels do not cover (fp32, ranks that are neither <= 8 nor multiples of 4).
//
//   shrink  (Eq. 2: A x;  Eq. 3: A h + b):  wave w owns ranks w, w+4, ...; its 64 lanes sweep
//           the row with 16-byte loads and finish each rank with one wavefront reduction.
//   expand  (Eq. 2: y + s B z;  Eq. 3: h + s B^T z):  one output column per thread, the
//           column's r factors are contiguous ([d_out, r] layout) and z sits in LDS.
#pragma once
#include "common.hpp"

namespace preft {

constexpr int ROW_THREADS = 256;

template <typename E, int WB /* bytes per weight load */>
__device__ __forceinline__ void row_expand(const ApplyArgs &p, gcptr_t Bt, gptr_t yrow, const float *z)
{
    constexpr int BYTES = Elem<E>::BYTES;
    constexpr int PER = WB / BYTES;                       // weights per load
    const int r = p.rank;
    const int row_bytes = r * BYTES;
    for (int n = threadIdx.x; n < p.d_out; n += ROW_THREADS) {
        gcptr_t w = Bt + (int64_t)n * row_bytes;
        float acc = 0.f;
        for (int o = 0; o < row_bytes; o += WB) {
            const int k = o / BYTES;
            if constexpr (WB == 16) {
                float f[Elem<E>::V];
                Elem<E>::unpack(ld16(w + o), f);
#pragma unroll
                for (int e = 0; e < PER; ++e) acc = fmaf(f[e], z[k + e], acc);
            } else if constexpr (WB == 8) {
                u32x2_t raw = ld8(w + o);
                if constexpr (BYTES == 2) {
                    acc = fmaf(bf16_lo(raw[0]), z[k], acc);
                    acc = fmaf(bf16_hi(raw[0]), z[k + 1], acc);
                    acc = fmaf(bf16_lo(raw[1]), z[k + 2], acc);
                    acc = fmaf(bf16_hi(raw[1]), z[k + 3], acc);
                } else {
                    acc = fmaf(__uint_as_float(raw[0]), z[k], acc);
                    acc = fmaf(__uint_as_float(raw[1]), z[k + 1], acc);
                }
            } else if constexpr (WB == 4) {
                uint32_t raw = ld4(w + o);
                if constexpr (BYTES == 2) {
                    acc = fmaf(bf16_lo(raw), z[k], acc);
                    acc = fmaf(bf16_hi(raw), z[k + 1], acc);
                } else {
                    acc = fmaf(__uint_as_float(raw), z[k], acc);
                }
            } else {
                acc = fmaf(Elem<E>::load1(w, k), z[k], acc);
            }
        }
        Elem<E>::store1(yrow, n, Elem<E>::load1(yrow, n) + acc);
    }
}

// Applies adapter `adapter` to row `row`.  z: LDS scratch of PREFT_MAX_RANK floats.
// Must be called by all ROW_THREADS threads of the workgroup.
template <typename E, bool DIREFT>
__device__ __forceinline__ void row_apply(const ApplyArgs &p, int adapter, int row, float *z)
{
    constexpr int V = Elem<E>::V;
    constexpr int BYTES = Elem<E>::BYTES;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int r = p.rank;
    gcptr_t A  = as_global(p.A_pool[adapter]);
    gcptr_t Bt = as_global(p.Bt_pool[adapter]);
    gcptr_t bias = (DIREFT && p.bias_pool) ? as_global(p.bias_pool[adapter]) : nullptr;
    gcptr_t xrow = as_global(p.x) + (int64_t)row * p.ldx * BYTES;
    gptr_t yrow = as_global(p.y) + (int64_t)row * p.ldy * BYTES;

    const int nvec = p.d_in / V;
    for (int k = wave; k < r; k += ROW_THREADS / 64) {
        gcptr_t Ak = A + (int64_t)k * p.d_in * BYTES;
        float acc = 0.f;
        for (int c = lane; c < nvec; c += 64) {
            float xv[V], av[V];
            Elem<E>::unpack(ld16(xrow + (int64_t)c * 16), xv);
            Elem<E>::unpack(ld16(Ak + (int64_t)c * 16), av);
#pragma unroll
            for (int i = 0; i < V; ++i) acc = fmaf(xv[i], av[i], acc);
        }
        acc = wave_sum(acc);
        if (lane == 0) {
            if (bias) acc += Elem<E>::load1(bias, k);
            z[k] = acc * p.scale;
        }
    }
    __syncthreads();          // z complete; for DiReFT also: every read of the row precedes every write

    const int row_bytes = r * BYTES;
    if ((row_bytes & 15) == 0)      row_expand<E, 16>(p, Bt, yrow, z);
    else if ((row_bytes & 7) == 0)  row_expand<E, 8>(p, Bt, yrow, z);
    else if ((row_bytes & 3) == 0)  row_expand<E, 4>(p, Bt, yrow, z);
    else                            row_expand<E, BYTES>(p, Bt, yrow, z);
    __syncthreads();          // z is reused by the next row
}

// Short rows: grid-stride over the schedule's row list.
template <typename E, bool DIREFT>
__global__ __launch_bounds__(ROW_THREADS) void row_kernel_short(ApplyArgs p)
{
    __shared__ float z[PREFT_MAX_RANK_DEV];
    const int n = p.header[1];
    for (int e = blockIdx.x; e < n; e += gridDim.x) {
        const int2 s = p.shorts[e];
        row_apply<E, DIREFT>(p, s.x, s.y, z);
    }
}

// Generic fallback for chunks: `split` workgroups share one chunk and take its rows in turn.
template <typename E, bool DIREFT>
__global__ __launch_bounds__(ROW_THREADS) void row_kernel_chunks(ApplyArgs p, int split)
{
    __shared__ float z[PREFT_MAX_RANK_DEV];
    const int c = blockIdx.x / split;
    if (c >= p.header[0]) return;
    const int4 ch = p.chunks[c];
    for (int i = blockIdx.x % split; i < ch.z; i += split) row_apply<E, DIREFT>(p, ch.x, ch.y + i, z);
}

}  // namespace preft
