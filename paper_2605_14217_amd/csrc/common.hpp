// Shared device-side definitions of the gfx950 adapter-apply kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace preft {

// ---------------------------------------------------------------------------------------
// Schedule (written by schedule_kernel, read by every apply kernel)
//
//   header   int32[16]   [0] number of chunks  [1] number of short rows  [2] active rows
//                        [3] position set (1: every position)  [4] number of gathered tiles
//                        [5] T  [6] S  [7] N of the batch the schedule was built for
//                        [8] set to 1 by an apply kernel whose call names another batch shape
//                            or position set than [3], [5..7]
//   chunks   int4[]      {adapter, first row, rows (1..CHUNK_ROWS), segment}
//   shorts   int2[]      {adapter, row}, sorted by adapter when the pool has <= SORT_MAX_N slots
//   gtiles   int4[]      {adapter, first entry in shorts, entries (1..GTILE_ROWS), 0}
//
// A chunk is a run of at most CHUNK_ROWS consecutive active rows of one segment; a tile
// kernel of height R (a divisor of CHUNK_ROWS) splits it into CHUNK_ROWS / R tiles.
// Segments with at most SHORT_ROWS active rows (decode tokens, speculative tokens, the
// last token of a chunked prompt) are listed row by row; rows that share an adapter are
// gathered into tiles of at most GTILE_ROWS rows, which the tile kernels process like a tile
// of a chunk except that every row has its own address: an adapter's factors are read once
// per gathered tile, not once per decode token.
// ---------------------------------------------------------------------------------------
constexpr int CHUNK_ROWS  = 128;
constexpr int SHORT_ROWS  = 4;
constexpr int GTILE_ROWS  = 16;     // >= SHORT_ROWS: a short segment always fits one gathered tile
constexpr int GROUP_ROWS  = 4;      // rows the per-row kernel carries through one sweep of the factors
constexpr int SORT_MAX_N  = 4096;   // pools up to this many slots get their short rows sorted by adapter
constexpr int HEADER_INTS = 16;
constexpr int HDR_CHUNKS = 0, HDR_SHORT_ROWS = 1, HDR_ACTIVE = 2, HDR_ALL = 3, HDR_GTILES = 4, HDR_T = 5, HDR_S = 6,
              HDR_N = 7, HDR_MISMATCH = 8;
constexpr int PREFT_MAX_RANK_DEV = 128;   // must equal PREFT_MAX_RANK of the public header

struct ScheduleView {
    int32_t *header;
    int4    *chunks;
    int2    *shorts;
    int4    *gtiles;        // capacity short_cap (a gathered tile holds at least one row)
    int32_t  chunk_cap;
    int32_t  short_cap;
};

// Upper bounds from host-visible sizes only (a long segment has > SHORT_ROWS rows).
__host__ __device__ inline int64_t chunk_capacity(int64_t T, int64_t S)
{
    int64_t long_segs = T / (SHORT_ROWS + 1);
    if (long_segs > S) long_segs = S;
    return T / CHUNK_ROWS + long_segs + 1;
}
__host__ __device__ inline int64_t short_capacity(int64_t T, int64_t S)
{
    int64_t c = (int64_t)SHORT_ROWS * S;
    return (c < T ? c : T) + 1;
}
// Gathered tiles: sorted pools cut every adapter's rows into tiles (at most one partial tile per
// adapter); unsorted pools get one tile per short segment.
__host__ __device__ inline int64_t gtile_capacity(int64_t T, int64_t S, int64_t N)
{
    const int64_t rows = short_capacity(T, S);
    const int64_t c = N <= SORT_MAX_N ? N + rows / GTILE_ROWS + 1 : S;
    return c < rows ? c : rows;
}

// ---------------------------------------------------------------------------------------
// bf16 <-> fp32
// ---------------------------------------------------------------------------------------
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x4_t __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float  f32x2_t  __attribute__((ext_vector_type(2)));
typedef float  f32x4_t  __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));

__device__ __forceinline__ float bf16_lo(uint32_t packed) { return __uint_as_float(packed << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t packed) { return __uint_as_float(packed & 0xffff0000u); }

// two fp32 -> packed bf16x2, round to nearest even (v_cvt_pk_bf16_f32 on gfx950)
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi)
{
    f32x2_t v = {lo, hi};
    bf16x2_t b = __builtin_convertvector(v, bf16x2_t);
    return __builtin_bit_cast(uint32_t, b);
}

__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}

// Pointers read from a pool table are generic; every buffer this library touches lives in
// global memory, so they are cast to the global address space (global_load / global_store
// instead of flat accesses).
#define PREFT_GLOBAL __attribute__((address_space(1)))
typedef const PREFT_GLOBAL char *gcptr_t;
typedef PREFT_GLOBAL char *gptr_t;
__device__ __forceinline__ gcptr_t as_global(const void *p) { return (gcptr_t)p; }
__device__ __forceinline__ gptr_t as_global(void *p) { return (gptr_t)p; }

// 16-, 8- and 4-byte global accesses
__device__ __forceinline__ u32x4_t ld16(gcptr_t p) { return *reinterpret_cast<const PREFT_GLOBAL u32x4_t *>(p); }
__device__ __forceinline__ u32x4_t ld16(gptr_t p) { return *reinterpret_cast<const PREFT_GLOBAL u32x4_t *>(p); }
__device__ __forceinline__ u32x2_t ld8(gcptr_t p) { return *reinterpret_cast<const PREFT_GLOBAL u32x2_t *>(p); }
__device__ __forceinline__ uint32_t ld4(gcptr_t p) { return *reinterpret_cast<const PREFT_GLOBAL uint32_t *>(p); }
__device__ __forceinline__ void st16(gptr_t p, u32x4_t v) { *reinterpret_cast<PREFT_GLOBAL u32x4_t *>(p) = v; }
// Activations are touched once per call: their loads and stores carry the non-temporal hint, so
// that they stream through the caches without displacing the adapter factors, which every tile
// of an adapter reads again.  Measured on the LoRA tile kernel, hint on x loads / y loads /
// y stores: none 59.7 %, all three 64.6 % of peak on the 8B shapes; 61.5 % -> 71.2 % on the 70B shapes
// (each hint alone gives part of it).
#ifndef PREFT_STREAM_HINTS
#define PREFT_STREAM_HINTS 1
#endif
__device__ __forceinline__ u32x4_t ld16_stream(gcptr_t p)
{
    if constexpr (PREFT_STREAM_HINTS != 0) return __builtin_nontemporal_load(reinterpret_cast<const PREFT_GLOBAL u32x4_t *>(p));
    else return ld16(p);
}
__device__ __forceinline__ u32x4_t ld16_stream(gptr_t p) { return ld16_stream((gcptr_t)p); }
// first of two reads of the same bytes (an in-place call that does not keep its tile): cacheable
template <bool AGAIN_LATER>
__device__ __forceinline__ u32x4_t ld16_first(gcptr_t p)
{
    if constexpr (AGAIN_LATER) return ld16(p);
    else return ld16_stream(p);
}
__device__ __forceinline__ void st16_stream(gptr_t p, u32x4_t v)
{
    if constexpr (PREFT_STREAM_HINTS != 0) __builtin_nontemporal_store(v, reinterpret_cast<PREFT_GLOBAL u32x4_t *>(p));
    else st16(p, v);
}

// Element traits: V = elements per 16-byte vector
template <typename T> struct Elem;
template <> struct Elem<float> {
    static constexpr int V = 4;
    static constexpr int BYTES = 4;
    __device__ static __forceinline__ void unpack(u32x4_t raw, float (&f)[4])
    {
#pragma unroll
        for (int i = 0; i < 4; ++i) f[i] = __uint_as_float(raw[i]);
    }
    __device__ static __forceinline__ u32x4_t pack(const float (&f)[4])
    {
        u32x4_t r;
#pragma unroll
        for (int i = 0; i < 4; ++i) r[i] = __float_as_uint(f[i]);
        return r;
    }
    __device__ static __forceinline__ float load1(gcptr_t p, int64_t i) { return reinterpret_cast<const PREFT_GLOBAL float *>(p)[i]; }
    __device__ static __forceinline__ float load1(gptr_t p, int64_t i) { return reinterpret_cast<const PREFT_GLOBAL float *>(p)[i]; }
    __device__ static __forceinline__ void store1(gptr_t p, int64_t i, float v) { reinterpret_cast<PREFT_GLOBAL float *>(p)[i] = v; }
};
struct bf16_tag {};
template <> struct Elem<bf16_tag> {
    static constexpr int V = 8;
    static constexpr int BYTES = 2;
    __device__ static __forceinline__ void unpack(u32x4_t raw, float (&f)[8])
    {
#pragma unroll
        for (int i = 0; i < 4; ++i) { f[2 * i] = bf16_lo(raw[i]); f[2 * i + 1] = bf16_hi(raw[i]); }
    }
    __device__ static __forceinline__ u32x4_t pack(const float (&f)[8])
    {
        u32x4_t r;
#pragma unroll
        for (int i = 0; i < 4; ++i) r[i] = pack_bf16(f[2 * i], f[2 * i + 1]);
        return r;
    }
    __device__ static __forceinline__ float load1(gcptr_t p, int64_t i)
    {
        return __uint_as_float((uint32_t) reinterpret_cast<const PREFT_GLOBAL uint16_t *>(p)[i] << 16);
    }
    __device__ static __forceinline__ float load1(gptr_t p, int64_t i) { return load1((gcptr_t)p, i); }
    __device__ static __forceinline__ void store1(gptr_t p, int64_t i, float v)
    {
        reinterpret_cast<PREFT_GLOBAL uint16_t *>(p)[i] = (uint16_t)(pack_bf16(v, 0.0f) & 0xffffu);
    }
};

// Arguments common to every apply kernel.  For DiReFT x == y == h, d_in == d_out == d,
// A = W1, Bt = W2^T and bias may be non-null.
struct ApplyArgs {
    void               *y;
    const void         *x;
    int64_t             ldy, ldx;        // row strides in elements
    int32_t             T, d_in, d_out;
    const void *const  *A_pool;          // [rank, d_in] each
    const void *const  *Bt_pool;         // [d_out, rank] each
    const void *const  *bias_pool;       // [rank] each, or null
    int32_t             N, rank;
    float               scale;
    int32_t             S, all_tokens;   // with T and N: what the schedule in `header` must have been built for
    int32_t            *header;
    const int4         *chunks;
    const int2         *shorts;
    const int4         *gtiles;
    void               *zws;             // z area of the workspace (two-launch LoRA), or null
    int32_t             gathered_only;   // tile kernels: skip the chunks (another launch covers them)
    int32_t             col_split;       // >= 1: workgroups per tile, each expanding its share of the columns
    // packed projections (LoRA only): further outputs computed from the same x, each with its
    // own factors; slice 0 is (y, ldy, d_out, A_pool, Bt_pool) above
    struct Slice {
        void               *y;
        int64_t             ldy;
        int32_t             d_out;
        const void *const  *A_pool;
        const void *const  *Bt_pool;
    } more[2];
    // several layers in one launch (in-place calls only): blockIdx.y picks the residual stream
    // and the pools of its layer from these device tables; h_layers null: the one layer above
    void *const               *h_layers = nullptr;      // [n_layers]
    const void *const *const  *A_layers = nullptr;      // [n_layers] pointer tables as A_pool
    const void *const *const  *Bt_layers = nullptr;
    const void *const *const  *bias_layers = nullptr;   // null: no bias in any layer
    int32_t                    n_layers = 1;
};

// First thing every apply kernel does: the schedule it is about to walk must be the one of this
// call's batch (same T, S, N and position set).  A caller that passes PREFT_SCHEDULE_READY with a
// workspace built for something else would otherwise skip rows or apply the wrong position set
// without any sign: such a launch does nothing and raises the mismatch flag of the header instead
// (one ordinary vector store; preft_schedule_counts reports it).  Uniform: four scalar loads of
// the cache line the kernel reads anyway.
__device__ __forceinline__ bool schedule_matches(const ApplyArgs &p)
{
    const bool ok = p.header[HDR_T] == p.T && p.header[HDR_S] == p.S && p.header[HDR_N] == p.N &&
                    p.header[HDR_ALL] == p.all_tokens;
    if (!ok && blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x == 0)
        *reinterpret_cast<volatile int32_t *>(p.header + HDR_MISMATCH) = 1;
    return ok;
}

// bias vector of an adapter, or null: no bias table, or a null entry in it (Eq. 3 with b = 0)
__device__ __forceinline__ gcptr_t bias_of(const ApplyArgs &p, int adapter)
{
    return p.bias_pool ? as_global(p.bias_pool[adapter]) : nullptr;
}

// Kernels of a many-layer in-place call: switch to the layer this workgroup belongs to
// (uniform: scalar loads).
__device__ __forceinline__ void select_layer(ApplyArgs &p)
{
    const int l = blockIdx.y;
    p.y = p.h_layers[l];
    p.x = p.y;
    p.A_pool = p.A_layers[l];
    p.Bt_pool = p.Bt_layers[l];
    p.bias_pool = p.bias_layers ? p.bias_layers[l] : nullptr;
}

template <int SL> __device__ __forceinline__ void *slice_y(const ApplyArgs &p) { if constexpr (SL == 0) return p.y; else return p.more[SL - 1].y; }
template <int SL> __device__ __forceinline__ int64_t slice_ldy(const ApplyArgs &p) { if constexpr (SL == 0) return p.ldy; else return p.more[SL - 1].ldy; }
template <int SL> __device__ __forceinline__ int32_t slice_d_out(const ApplyArgs &p) { if constexpr (SL == 0) return p.d_out; else return p.more[SL - 1].d_out; }
template <int SL> __device__ __forceinline__ const void *const *slice_A(const ApplyArgs &p) { if constexpr (SL == 0) return p.A_pool; else return p.more[SL - 1].A_pool; }
template <int SL> __device__ __forceinline__ const void *const *slice_Bt(const ApplyArgs &p) { if constexpr (SL == 0) return p.Bt_pool; else return p.more[SL - 1].Bt_pool; }

// The tile a workgroup of a tile kernel of height R works on: rows of one adapter, either
// consecutive (a tile of a chunk) or listed one by one (a gathered tile).
struct TileRows {
    int32_t      adapter, n_rows;
    int64_t      base;                   // first row, or first entry of the list
    const int2  *list;                   // null: consecutive rows

    // row of slot `slot`; slots past the end alias the last row
    __device__ __forceinline__ int64_t row(int slot) const
    {
        slot = min(slot, n_rows - 1);
        return list ? (int64_t)list[base + slot].y : base + slot;
    }
};

// Maps tile number `unit` of a launch onto its rows.  Units 0 .. chunks * (CHUNK_ROWS / R) - 1
// are the tiles of the chunks, the gathered tiles follow (a gathered tile takes GTILE_ROWS / R
// units when R is smaller).  Returns false when the unit has no rows.
template <int R>
__device__ __forceinline__ bool tile_rows(const ApplyArgs &p, int unit, int n_chunk_units, TileRows &t)
{
    constexpr int TPC = CHUNK_ROWS / R;
    constexpr int UPG = R >= GTILE_ROWS ? 1 : GTILE_ROWS / R;
    if (unit < n_chunk_units) {
        const int4 ch = p.chunks[unit / TPC];
        const int row0 = (unit % TPC) * R;
        t.adapter = ch.x;
        t.n_rows = min(R, ch.z - row0);
        t.base = (int64_t)ch.y + row0;
        t.list = nullptr;
    } else {
        const int u = unit - n_chunk_units;
        const int4 gt = p.gtiles[u / UPG];
        const int first = (u % UPG) * R;
        t.adapter = gt.x;
        t.n_rows = min(R, gt.z - first);
        t.base = (int64_t)gt.y + first;
        t.list = p.shorts;
    }
    return t.n_rows > 0;
}

// Number of units of a tile-kernel launch of height R (see tile_rows).
template <int R>
__device__ __forceinline__ int tile_units(const ApplyArgs &p, int *n_chunk_units)
{
    constexpr int UPG = R >= GTILE_ROWS ? 1 : GTILE_ROWS / R;
    *n_chunk_units = p.gathered_only ? 0 : p.header[HDR_CHUNKS] * (CHUNK_ROWS / R);
    return *n_chunk_units + p.header[HDR_GTILES] * UPG;
}

}  // namespace preft
