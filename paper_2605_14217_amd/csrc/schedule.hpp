// Token-segment scheduler: segment tables -> list of work units over active rows only.
//
// Position sets follow the paper's Eq. 1 and Eq. 4: in prefill-only mode the first
// seg_prefill_len[s] rows of segment s are active, in all-token mode every row is; a
// segment without a valid adapter has no active row.  Inactive rows appear in no unit, so
// the apply kernels never touch them.
#pragma once
#include "common.hpp"

namespace preft {

constexpr int SCHED_THREADS = 1024;

struct SegInfo { int32_t adapter, row0, n_act; };

__device__ __forceinline__ SegInfo seg_info(const int32_t *seg_start, const int32_t *seg_adapter,
                                             const int32_t *seg_prefill_len, int32_t s, int32_t T,
                                             int32_t N, bool all_tokens)
{
    SegInfo r;
    int32_t lo = seg_start[s], hi = seg_start[s + 1];
    lo = max(0, min(lo, T));
    hi = max(lo, min(hi, T));
    int32_t len = hi - lo;
    int32_t a = seg_adapter[s];
    int32_t n = all_tokens ? len : max(0, min(seg_prefill_len[s], len));
    if (a < 0 || a >= N) n = 0;
    r.adapter = a;
    r.row0 = lo;
    r.n_act = n;
    return r;
}

// Exclusive scan of one int per thread over the block; returns the block total through *total.
__device__ __forceinline__ int32_t block_exclusive_scan(int32_t v, int32_t *lds /* >= 32 ints */, int32_t *total)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, n_waves = blockDim.x >> 6;
    int32_t incl = v;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        int32_t up = __shfl_up(incl, off, 64);
        if (lane >= off) incl += up;
    }
    __syncthreads();                         // lds may still be read from a previous scan
    if (lane == 63) lds[wave] = incl;
    __syncthreads();
    int32_t base = 0, sum = 0;
    for (int w = 0; w < n_waves; ++w) {
        int32_t t = lds[w];
        if (w < wave) base += t;
        sum += t;
    }
    *total = sum;
    return base + incl - v;
}

// A gathered tile names entries [first, first + n) of the short-row list.  With well-formed
// tables the list never outgrows its capacity (a row belongs to one segment); tables whose
// segments overlap can make it do so, and the entries beyond the capacity are never written:
// a tile is cut back to the entries that exist, so that no kernel indexes past the list.
__device__ __forceinline__ int4 clamped_gtile(int32_t adapter, int32_t first, int32_t n, int32_t short_cap)
{
    if (first >= short_cap) return make_int4(adapter, 0, 0, 0);
    return make_int4(adapter, first, min(n, short_cap - first), 0);
}

// One workgroup.  Thread i owns the contiguous slice of segments [i*per, (i+1)*per), so the
// chunk list keeps segment order (consecutive chunks of one segment share an adapter, which
// the tile kernels exploit for cache locality).  Short rows are counting-sorted by adapter
// (LDS histogram) and cut into gathered tiles of at most GTILE_ROWS rows of one adapter; a
// pool too large for the histogram gets one gathered tile per short segment instead.
__global__ __launch_bounds__(SCHED_THREADS) void schedule_kernel(
    const int32_t *__restrict__ seg_start, const int32_t *__restrict__ seg_adapter,
    const int32_t *__restrict__ seg_prefill_len, int32_t S, int32_t T, int32_t N, int all_tokens,
    ScheduleView out)
{
    __shared__ int32_t lds[32];
    __shared__ int32_t bin_start[SORT_MAX_N + 1];   // first short-row entry of each adapter
    __shared__ int32_t bin_cursor[SORT_MAX_N];      // running insertion point while scattering
    const int tid = threadIdx.x, lane = tid & 63;
    const bool all = all_tokens != 0;
    const bool sorted = N <= SORT_MAX_N;
    const int32_t per = (S + SCHED_THREADS - 1) / SCHED_THREADS;
    const int32_t s0 = (int32_t)min((int64_t)tid * per, (int64_t)S);
    const int32_t s1 = (int32_t)min((int64_t)s0 + per, (int64_t)S);

    if (sorted)
        for (int32_t a = tid; a <= N; a += SCHED_THREADS) bin_start[a] = 0;
    __syncthreads();

    // ---- pass 1: counts
    int32_t my_chunks = 0, my_short = 0, my_short_segs = 0, my_act = 0;
    for (int32_t s = s0; s < s1; ++s) {
        SegInfo g = seg_info(seg_start, seg_adapter, seg_prefill_len, s, T, N, all);
        my_act += g.n_act;
        if (g.n_act == 0) continue;
        if (g.n_act <= SHORT_ROWS) {
            my_short += g.n_act;
            my_short_segs += 1;
            if (sorted) atomicAdd(&bin_start[g.adapter], g.n_act);
        } else {
            my_chunks += (g.n_act + CHUNK_ROWS - 1) / CHUNK_ROWS;
        }
    }
    int32_t tot_chunks, tot_short, tot_short_segs, tot_act;
    int32_t chunk_off = block_exclusive_scan(my_chunks, lds, &tot_chunks);
    int32_t short_off = block_exclusive_scan(my_short, lds, &tot_short);
    int32_t seg_off   = block_exclusive_scan(my_short_segs, lds, &tot_short_segs);
    (void)block_exclusive_scan(my_act, lds, &tot_act);

    // ---- sorted case: histogram -> first entry per adapter, tile counts -> first tile per adapter
    const int32_t bins_per = (N + SCHED_THREADS) / SCHED_THREADS;      // covers bins 0..N-1
    const int32_t b0 = min(tid * bins_per, N), b1 = min(b0 + bins_per, N);
    int32_t tot_gtiles = tot_short_segs;
    int32_t my_gtile_off = 0;
    if (sorted) {
        constexpr int32_t grows = GTILE_ROWS;   // rows per gathered tile
        int32_t rows_here = 0, gtiles_here = 0;
        for (int32_t a = b0; a < b1; ++a) {
            const int32_t c = bin_start[a];
            rows_here += c;
            gtiles_here += (c + grows - 1) / grows;
        }
        int32_t dummy;
        int32_t row_base = block_exclusive_scan(rows_here, lds, &dummy);
        my_gtile_off = block_exclusive_scan(gtiles_here, lds, &tot_gtiles);
        // the scans end with a barrier-protected read of lds, the histogram is final here
        int32_t grp = my_gtile_off;
        for (int32_t a = b0; a < b1; ++a) {
            const int32_t c = bin_start[a];
            bin_start[a] = row_base;
            bin_cursor[a] = row_base;
            for (int32_t i = 0; i * grows < c; ++i, ++grp)
                if (grp < out.short_cap)
                    out.gtiles[grp] = clamped_gtile(a, row_base + i * grows, min(grows, c - i * grows), out.short_cap);
            row_base += c;
        }
        __syncthreads();
    }

    if (tid == 0) {
        out.header[HDR_CHUNKS] = min(tot_chunks, out.chunk_cap);
        out.header[HDR_SHORT_ROWS] = min(tot_short, out.short_cap);
        out.header[HDR_ACTIVE] = tot_act;
        out.header[HDR_ALL] = all ? 1 : 0;
        out.header[HDR_GTILES] = min(tot_gtiles, out.short_cap);
        out.header[HDR_T] = T;
        out.header[HDR_S] = S;
        out.header[HDR_N] = N;
        out.header[HDR_MISMATCH] = 0;
    }

    // ---- pass 2: emission.  All lanes of a wave run the same number of iterations; a segment
    // with many chunks is written by the whole wave.
    for (int32_t i = 0; i < per; ++i) {
        const int32_t s = s0 + i;
        SegInfo g = {-1, 0, 0};
        if (s < s1) g = seg_info(seg_start, seg_adapter, seg_prefill_len, s, T, N, all);
        int32_t n_ch = 0;
        if (g.n_act > 0 && g.n_act <= SHORT_ROWS) {
            int32_t pos;
            if (sorted) {
                pos = atomicAdd(&bin_cursor[g.adapter], g.n_act);
            } else {
                pos = short_off;
                if (seg_off < out.short_cap) out.gtiles[seg_off] = clamped_gtile(g.adapter, pos, g.n_act, out.short_cap);
                short_off += g.n_act;
                seg_off += 1;
            }
            for (int32_t j = 0; j < g.n_act; ++j)
                if (pos + j < out.short_cap) out.shorts[pos + j] = make_int2(g.adapter, g.row0 + j);
        } else if (g.n_act > SHORT_ROWS) {
            n_ch = (g.n_act + CHUNK_ROWS - 1) / CHUNK_ROWS;
        }
        unsigned long long pending = __ballot(n_ch > 0);
        while (pending) {
            const int src = __ffsll((long long)pending) - 1;
            pending &= pending - 1;
            const int32_t b_off = __shfl(chunk_off, src, 64);
            const int32_t b_n   = __shfl(g.n_act, src, 64);
            const int32_t b_row = __shfl(g.row0, src, 64);
            const int32_t b_a   = __shfl(g.adapter, src, 64);
            const int32_t b_s   = __shfl(s, src, 64);
            const int32_t b_ch  = (b_n + CHUNK_ROWS - 1) / CHUNK_ROWS;
            for (int32_t c = lane; c < b_ch; c += 64) {
                if (b_off + c < out.chunk_cap)
                    out.chunks[b_off + c] = make_int4(b_a, b_row + c * CHUNK_ROWS,
                                                      min(CHUNK_ROWS, b_n - c * CHUNK_ROWS), b_s);
            }
        }
        chunk_off += n_ch;
    }
}

}  // namespace preft
