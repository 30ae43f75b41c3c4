// C ABI of the adapter-apply library: argument validation, variant choice, launches.
// See include/preft.h for the contract of every entry point.
#include "../../include/preft.h"

#include "common.hpp"
#include "mfma_kernel.hpp"
#include "mfma_wide_kernel.hpp"
#include "row_kernel.hpp"
#include "schedule.hpp"
#include "valu_kernel.hpp"
// most kernel instantiations are compiled in instances/group_*.hip (see gen_instances.py), in parallel
#ifndef PREFT_NO_EXTERN_KERNELS
#include "instances/extern_kernels.inc"
#endif

#include <mutex>

static_assert(preft::PREFT_MAX_RANK_DEV == PREFT_MAX_RANK, "device and public rank limits differ");

// Schedule area of preft_direft_apply_static: device memory that exists without any allocation call.
// Each GPU the library runs on holds its own copy at its own address until the process ends.  In
// host code the name below is only a stand-in for the symbol: the address a kernel can use comes
// from hipGetSymbolAddress (static_scratch_of), once per device.
static __device__ __align__(256) unsigned char scratch[PREFT_STATIC_SCRATCH_BYTES];

namespace {

using namespace preft;

// Kernel selection for tests and benchmarks, carried by the mode argument of the call itself
// (PREFT_TEST_* of the public header): the library keeps no state between calls.
struct Knobs {
    int variant, waves, rowblocks, colsplit, resident;
};
constexpr int MODE_TEST_MASK = 0x7fff0000;
constexpr int MODE_MASK = PREFT_ALL_TOKENS | PREFT_SCHEDULE_READY | MODE_TEST_MASK;

inline Knobs knobs_of(int mode)
{
    Knobs k;
    k.variant   = (mode >> 16) & 7;
    k.waves     = (mode >> 19) & 15;
    k.rowblocks = (mode >> 23) & 3;
    k.colsplit  = (mode >> 25) & 15;
    k.resident  = (mode >> 29) & 3;
    return k;
}
inline bool knobs_valid(const Knobs &k)
{
    if (k.variant > 5) return false;
    if (k.waves != 0 && k.waves != 1 && k.waves != 2 && k.waves != 4 && k.waves != 8) return false;
    if (k.rowblocks > 2) return false;
    return true;
}

inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

size_t workspace_bytes(int64_t T, int64_t S)
{
    return (size_t)HEADER_INTS * 4 + (size_t)chunk_capacity(T, S) * sizeof(int4) +
           (size_t)short_capacity(T, S) * (sizeof(int4) + sizeof(int2));
}

// z area (LoRA calls whose sweeps run as two launches): after the schedule, 1 KB per 16-row block of
// a chunk and rank block of 16
size_t z_offset(int64_t T, int64_t S) { return (workspace_bytes(T, S) + 255) & ~(size_t)255; }
size_t z_bytes(int64_t T, int64_t S, int rank, int n_proj)
{
    return (size_t)chunk_capacity(T, S) * (CHUNK_ROWS / 16) * (size_t)(((rank + 15) / 16) * n_proj) * 1024;
}

ScheduleView view_of(void *workspace, int64_t T, int64_t S)
{
    ScheduleView v;
    char *base = reinterpret_cast<char *>(workspace);
    v.header = reinterpret_cast<int32_t *>(base);
    v.chunks = reinterpret_cast<int4 *>(base + HEADER_INTS * 4);
    v.chunk_cap = (int32_t)chunk_capacity(T, S);
    v.short_cap = (int32_t)short_capacity(T, S);
    char *after_chunks = base + HEADER_INTS * 4 + (size_t)v.chunk_cap * sizeof(int4);
    v.gtiles = reinterpret_cast<int4 *>(after_chunks);                  // 16-byte aligned
    v.shorts = reinterpret_cast<int2 *>(after_chunks + (size_t)v.short_cap * sizeof(int4));
    return v;
}

// Device address of this GPU's copy of `scratch` (looked up on the first call per device, with that
// device current; no allocation).
constexpr int MAX_DEVICES = 64;
std::mutex g_scratch_mutex;
void *g_scratch_ptr[MAX_DEVICES] = {};

int static_scratch_of(void **out)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) return PREFT_EHIP;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return PREFT_EHIP;
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return PREFT_OK;
}

int check_launch()
{
    return hipGetLastError() == hipSuccess ? PREFT_OK : PREFT_EHIP;
}

int check_tables(const void *workspace, size_t bytes, const int32_t *seg_start, const int32_t *seg_adapter,
                 const int32_t *seg_prefill_len, int32_t S, int32_t T, int32_t N, int mode)
{
    if (T < 0 || S < 0 || N < 0) return PREFT_EINVAL;
    if ((mode & ~MODE_MASK) != 0 || !knobs_valid(knobs_of(mode))) return PREFT_EINVAL;
    if (T == 0 || S == 0) return PREFT_OK;
    if (!seg_start || !seg_adapter || !seg_prefill_len) return PREFT_EINVAL;
    if (!workspace || !aligned16(workspace) || bytes < workspace_bytes(T, S)) return PREFT_EWORKSPACE;
    return PREFT_OK;
}

int launch_schedule(void *workspace, const int32_t *seg_start, const int32_t *seg_adapter,
                    const int32_t *seg_prefill_len, int32_t S, int32_t T, int32_t N, int mode,
                    hipStream_t stream)
{
    ScheduleView v = view_of(workspace, T, S);
    hipLaunchKernelGGL(schedule_kernel, dim3(1), dim3(SCHED_THREADS), 0, stream, seg_start, seg_adapter,
                       seg_prefill_len, S, T, N, (mode & PREFT_ALL_TOKENS) ? 1 : 0, v);
    return check_launch();
}

// ------------------------------------------------------------------------------------
// tile-kernel dispatch
// ------------------------------------------------------------------------------------
// Upper bound of the units of a tile-kernel launch of height `rows`, from host-visible sizes,
// rounded to the 8 XCDs.
inline unsigned tile_grid(const ApplyArgs &a, int64_t S, int rows)
{
    const int64_t per_gtile = rows >= GTILE_ROWS ? 1 : GTILE_ROWS / rows;
    int64_t units = gtile_capacity(a.T, S, a.N) * per_gtile;
    if (!a.gathered_only) units += chunk_capacity(a.T, S) * (CHUNK_ROWS / rows);
    return (unsigned)(((units + 7) / 8) * 8 * (a.col_split > 1 ? a.col_split : 1));
}
// Workgroups per tile for the LoRA column-split kernel: a batch of a few hundred rows has too
// few tiles to occupy the chip, and one workgroup per tile would walk every output column alone.
inline int choose_col_split(int32_t T, const Knobs &k)
{
    if (k.colsplit && k.variant != 4) return k.colsplit;      // with variant 4 the knob names the row-split kernel's column groups
    return T <= 1024 ? 4 : 1;
}

// the small-batch shape of the column-split kernel (col_split > 1): one shape per rank class
template <int NB, int SLICES, int PIECES = 0>
void launch_mfma_colsplit(const ApplyArgs &a, int64_t S, hipStream_t stream)
{
    constexpr int WAVES = NB >= 4 ? 4 : 8;                 // register budget
    hipLaunchKernelGGL((mfma_tile_kernel<NB, 1, WAVES, 0, false, SLICES, true, false, PIECES>), dim3(tile_grid(a, S, 16)),
                       dim3(WAVES * 64), 0, stream, a);
}
// the row-split kernel takes whole chunks only
inline unsigned chunk_grid(const ApplyArgs &a, int64_t S, int rows)
{
    const int64_t units = chunk_capacity(a.T, S) * (CHUNK_ROWS / rows);
    return (unsigned)(((units + 7) / 8) * 8);
}

// in place, part of the tile held in registers (HUNITS units of each wavefront), the rest streamed twice
template <int NB, int MB, int WAVES, int HUNITS>
void launch_mfma_partial(const ApplyArgs &a, int64_t S, hipStream_t stream)
{
    void (*kernel)(ApplyArgs) = mfma_tile_kernel<NB, MB, WAVES, HUNITS, true, 1, false, true>;
    if (a.h_layers) kernel = mfma_tile_layers_kernel<NB, MB, WAVES, HUNITS, true>;
    hipLaunchKernelGGL(kernel, dim3(tile_grid(a, S, 16 * MB), a.n_layers), dim3(WAVES * 64), 0, stream, a);
}

template <int NB, int MB, int WAVES, int HUNITS, bool DIREFT>
void launch_mfma(const ApplyArgs &a, int64_t S, hipStream_t stream)
{
    constexpr int R = 16 * MB;
    void (*kernel)(ApplyArgs) = mfma_tile_kernel<NB, MB, WAVES, HUNITS, DIREFT>;
    if constexpr (DIREFT) {
        if (a.h_layers) kernel = mfma_tile_layers_kernel<NB, MB, WAVES, HUNITS>;
    }
    hipLaunchKernelGGL(kernel, dim3(tile_grid(a, S, R), a.n_layers), dim3(WAVES * 64), 0, stream, a);
}

// streaming variant (activations read in both sweeps): LoRA, and DiReFT rows too wide to hold
template <int NB, bool DIREFT>
void launch_mfma_stream(const ApplyArgs &a, int64_t S, int mb, int waves, hipStream_t stream)
{
    if constexpr (NB < 2) {                                // register budget
        if (waves == 8) {
            launch_mfma<NB, 1, 8, 0, DIREFT>(a, S, stream);
            return;
        }
    }
    if constexpr (NB < 8) {
        if (mb == 2) {
            launch_mfma<NB, 2, 4, 0, DIREFT>(a, S, stream);
            return;
        }
    }
    launch_mfma<NB, 1, 4, 0, DIREFT>(a, S, stream);
}

// DiReFT with the tile held in registers between the sweeps (rank <= 16): 8 wavefronts, HUNITS
// units of 128 columns each (register budget: 16 VGPRs per unit).  From rank 32 up the factor
// sweeps of a 16-row tile outweigh its activations and the register file has no room left to
// run them ahead, so those ranks take 32-row tiles (rank 32) or the row-split kernel (rank >= 64).
template <int NB>
bool launch_mfma_resident(const ApplyArgs &a, int64_t S, hipStream_t stream)
{
    if constexpr (NB > 1) {
        return false;
    } else {
        const int units = ((a.d_in >> 7) + 7) / 8;        // whole units per wavefront
        if (units <= 4) {
            launch_mfma<NB, 1, 8, 4, true>(a, S, stream);
            return true;
        }
        if (units <= 8) {
            launch_mfma<NB, 1, 8, 8, true>(a, S, stream);
            return true;
        }
        return false;
    }
}

// row-split kernel with the factors shared through LDS (rank >= 32, widths multiples of 128):
// `rw` row blocks of 16 `mb` rows x `cw` column groups of wavefronts per workgroup
template <int NB, int MB, int RW, int CW, bool DIREFT, bool ODD = false>
void launch_wide_shape(const ApplyArgs &a, int64_t S, hipStream_t stream)
{
    void (*kernel)(ApplyArgs) = mfma_wide_kernel<NB, MB, RW, CW, DIREFT, 1, false, ODD>;
    if constexpr (DIREFT) { if (a.h_layers) kernel = mfma_wide_layers_kernel<NB, MB, RW, CW, ODD>; }   // set on in-place calls only
    hipLaunchKernelGGL(kernel, dim3(chunk_grid(a, S, 16 * MB * RW), a.n_layers), dim3(RW * CW * 64), 0, stream, a);
}

// widths the shape with `cw` column groups takes
inline bool wide_widths_ok(const ApplyArgs &a, int cw)
{
    const int m = 128 * cw;
    return (a.d_in % m) == 0 && (a.d_out % m) == 0;
}

// LoRA at rank 20..64 with a z area in the workspace: the chunks' shrink sweep and expand sweep as two
// launches, the expand in 2-D tiles of 64 rows x 256 columns (see mfma_expand_panel_kernel).  Measured on
// the same buffers, % of peak, one launch -> two:
//   8B-sized batch (38 416 rows): rank 64 q+k+v 37 -> 42, o 42-43 -> 51-53, gate+up 47 -> 59, down 46 -> 51;
//     rank 32 q+k+v 52 -> 53, o 58 -> 62.5, gate+up 58 -> 66.5, down 62 -> 62 (a 64-row tile per workgroup
//     leaves the chip 1.2 rounds of tiles; the expand launch has thousands of small workgroups);
//   70B-sized batch (352 814 rows): rank 64 o and down +2 to +4 on one set of buffers, -2 on another (the
//     one-launch kernel moves between 62 and 68 % with the placement of its buffers, the two launches stay
//     at 62-66 %), packed q+k+v 57.8 -> 52, gate+up 61.8 -> 60.8 (the shrink launch of two or three outputs is
//     bound by LDS reads and MFMA issue once no expand sweep of another workgroup runs beside it: 33 % of peak
//     for q+k+v; 28 672-wide dense rows gain little from the tiling); rank 32 o 73.8 -> 74.2, down 71.9 -> 76.5,
//     packed q+k+v 69 -> 61, gate+up 74 -> 68; skewed batch (836 609 rows), rank 32, 8192 -> 8192: 77.4 -> 73.9.
// Hence: batches of 8192 to 131 072 rows.  PREFT_TEST_RESIDENT(1) takes this form wherever it exists,
// PREFT_TEST_VARIANT(5) never.  Panels of 128 columns: -1 to -3 points; of 512: one workgroup per compute
// unit, -15.
template <int NB, int SLICES>
bool launch_mfma_split(const ApplyArgs &a, int64_t S, const Knobs &k, hipStream_t stream)
{
    constexpr int PU = 2;
    if (!a.zws || k.variant == 5 || k.waves || k.rowblocks || k.colsplit) return false;
    if (k.resident != 1 && (a.T < 8192 || a.T > 131072)) return false;
    if ((a.d_in % 128) != 0 || (a.d_out % (128 * PU)) != 0) return false;
    int max_d_out = a.d_out;
    for (int i = 1; i < SLICES; ++i) {
        if ((a.more[i - 1].d_out % (128 * PU)) != 0) return false;
        if (a.more[i - 1].d_out > max_d_out) max_d_out = a.more[i - 1].d_out;
    }
    void (*shrink)(ApplyArgs) = mfma_wide_kernel<NB, 1, 4, 1, false, SLICES, true>;
    int threads = 256;
    if constexpr (NB <= 2) {
        if ((a.d_in % 256) == 0) { shrink = mfma_wide_kernel<NB, 1, 4, 2, false, SLICES, true>; threads = 512; }
    }
    hipLaunchKernelGGL(shrink, dim3(chunk_grid(a, S, 64)), dim3(threads), 0, stream, a);
    int64_t tiles = chunk_capacity(a.T, S) * (CHUNK_ROWS / 64) * (int64_t)(max_d_out / (128 * PU));
    tiles = ((tiles + 7) / 8) * 8;
    if (tiles > 8192) tiles = 8192;                         // the kernel strides over the rest
    hipLaunchKernelGGL((mfma_expand_panel_kernel<NB, 4, PU>), dim3((unsigned)tiles, SLICES), dim3(256), 0, stream, a, SLICES);
    return true;
}

template <int NB, bool DIREFT>
bool launch_mfma_wide(const ApplyArgs &a, int64_t S, int mb, int waves, int cw, const Knobs &k, hipStream_t stream)
{
    if (NB < 2 && k.variant != 4) return false;               // rank <= 16: only on request
    if (!wide_widths_ok(a, 1)) return false;
    if constexpr (!DIREFT && NB >= 2 && NB <= 4) {
        if (launch_mfma_split<NB, 1>(a, S, k, stream)) return true;
    }
    if (!wide_widths_ok(a, cw)) cw = 1;
    if (mb != 1 && NB <= 4) {                                  // 4 wavefronts x 32 rows
        if constexpr (NB <= 4) launch_wide_shape<NB, 2, 4, 1, DIREFT>(a, S, stream);
        return true;
    }
    if (cw >= 2 && NB <= 4) {                                  // 2 column groups: 8 wavefronts on 64 rows
        if constexpr (NB <= 4) launch_wide_shape<NB, 1, 4, 2, DIREFT>(a, S, stream);
        return true;
    }
    if (waves == 8) launch_wide_shape<NB, 1, 8, 1, DIREFT>(a, S, stream);
    else            launch_wide_shape<NB, 1, 4, 1, DIREFT>(a, S, stream);
    return true;
}

template <int NB, bool DIREFT>
void launch_mfma_nb(const ApplyArgs &a, int64_t S, const Knobs &k, hipStream_t stream)
{
    // rank >= 32: the factors outweigh a 16-row tile's activations, so more rows share them: the
    // row-split kernel.  Up to rank 64 with 4 wavefronts x 16 rows (two or three independent
    // workgroups per compute unit and twice the tiles: measured 3-10 points ahead of 8 wavefronts on
    // the 8B- and 70B-sized batches); above, 8 wavefronts (4 would leave one workgroup per unit)
    const int wide_mb = k.rowblocks ? k.rowblocks : 1;
    const int wide_waves = k.waves ? (k.waves == 8 ? 8 : 4) : (NB <= 4 ? 4 : 8);
    // Column groups (with test variant 4 the column-split knob names them: 1 or 2).  Two of them at
    // rank 32 (measured: 70B q,k,v,o 64 -> 70-76 % of peak, skewed batch 64-75 -> 78 %); at rank 48-64
    // the two factor units per step leave one workgroup per compute unit and that costs more than the
    // access pattern gains (o 62 -> 64.5 %, but gate+up 69 -> 62.5 %, down 64 -> 59 %).
    const int wide_cw = (k.variant == 4 && k.colsplit) ? k.colsplit : (NB <= 2 ? 2 : 1);
    // column-split kernel.  rank <= 16: 8 wavefronts per 16-row tile; rank 32 (widths the
    // row-split kernel does not take): 32-row tiles of 4 wavefronts
    const int mb = k.rowblocks ? k.rowblocks : (NB == 2 ? 2 : 1);
    const int waves = k.waves ? (k.waves == 8 ? 8 : 4) : (NB == 2 ? 4 : 8);
    if constexpr (DIREFT) {
        if (k.waves == 0 && k.variant != 4 && launch_mfma_resident<NB>(a, S, stream)) return;
        // rank 32: 32-row tiles of the column-split kernel (half the factor traffic per row of a
        // 16-row tile, and the tile's second read mostly still finds it in the memory-side cache)
        // measured ahead of the resident and row-split shapes at d = 4096 and d = 8192
        if constexpr (NB == 2) {
            if (k.waves == 0 && (k.variant == 0 || k.variant == 5) && k.rowblocks == 0) {
                // resident == 3 (tests): each wavefront keeps 8 of its units in registers and streams the
                // rest twice.  Measured on the skewed batch (d = 8192): traffic through the fabric falls
                // by a sixth (half of the tile is read once), the time by 4 % (5985 against 6216 us): the
                // 256 + 248 registers leave one workgroup of four wavefronts per compute unit, and what
                // binds is the latency of the factor sweeps, not the bytes.  Not the default.
                if (k.resident == 3) launch_mfma_partial<2, 2, 4, 8>(a, S, stream);
                else                 launch_mfma<2, 2, 4, 0, true>(a, S, stream);
                return;
            }
        }
    }
    if constexpr (!DIREFT) {
        if (a.col_split > 1) {
            launch_mfma_colsplit<NB, 1>(a, S, stream);
            return;
        }
    }
    if (k.variant != 3 && launch_mfma_wide<NB, DIREFT>(a, S, wide_mb, wide_waves, wide_cw, k, stream)) {
        // the row-split kernel shares one adapter's factors among the 128 rows of a chunk;
        // gathered tiles (16 rows of an adapter) go to the column-split kernel
        ApplyArgs g = a;
        g.gathered_only = 1;
        launch_mfma_stream<NB, DIREFT>(g, S, 1, NB >= 2 ? 4 : 8, stream);
        return;
    }
    launch_mfma_stream<NB, DIREFT>(a, S, mb, waves, stream);
}

// packed projections (LoRA, rank <= 16): one shrink sweep over x, one expand sweep per output.
// PIECES > 0: the any-rank shape (ranks that are not multiples of 4)
template <int SLICES, int PIECES = 0>
void launch_mfma_packed(const ApplyArgs &a, int64_t S, const Knobs &k, hipStream_t stream)
{
    if (a.col_split > 1) {
        launch_mfma_colsplit<1, SLICES, PIECES>(a, S, stream);
        return;
    }
    // three outputs: 4 wavefronts per tile leave room for two workgroups per compute unit (measured
    // better on small and large batches); two outputs: as for a single projection
    const int waves = k.waves ? (k.waves == 8 ? 8 : 4) : (SLICES == 2 ? 8 : 4);
    if (waves == 8)
        hipLaunchKernelGGL((mfma_tile_kernel<1, 1, 8, 0, false, SLICES, false, false, PIECES>), dim3(tile_grid(a, S, 16)),
                           dim3(512), 0, stream, a);
    else
        hipLaunchKernelGGL((mfma_tile_kernel<1, 1, 4, 0, false, SLICES, false, false, PIECES>), dim3(tile_grid(a, S, 16)),
                           dim3(256), 0, stream, a);
}

template <typename E, bool DIREFT>
void launch_rows(const ApplyArgs &a, int64_t S, bool chunks_too, hipStream_t stream);

// packed projections at rank 32..64 (widths multiples of 128): the row-split kernel with one sweep
// over x for all outputs.  It takes the chunks; the gathered tiles (all-token mode: decode rows)
// go to one launch of the column-split kernel per output.
template <int NB>
void launch_mfma_wide_packed(const ApplyArgs &a, int n_proj, int64_t S, const Knobs &k, hipStream_t stream)
{
    if (a.rank % 4) {
        // the any-rank form: the basic shape for the chunks, the per-row kernel for the gathered tiles
        void (*odd)(ApplyArgs) = n_proj == 2 ? mfma_wide_kernel<NB, 1, 4, 1, false, 2, false, true>
                                             : mfma_wide_kernel<NB, 1, 4, 1, false, 3, false, true>;
        hipLaunchKernelGGL(odd, dim3(chunk_grid(a, S, 64)), dim3(256), 0, stream, a);
        for (int i = 0; i < n_proj; ++i) {
            ApplyArgs g = a;
            if (i > 0) {
                g.y = a.more[i - 1].y; g.ldy = a.more[i - 1].ldy; g.d_out = a.more[i - 1].d_out;
                g.A_pool = a.more[i - 1].A_pool; g.Bt_pool = a.more[i - 1].Bt_pool;
            }
            launch_rows<bf16_tag, false>(g, S, false, stream);
        }
        return;
    }
    const bool split = n_proj == 2 ? launch_mfma_split<NB, 2>(a, S, k, stream) : launch_mfma_split<NB, 3>(a, S, k, stream);
    // two column groups at rank 32 where every width allows it (see launch_mfma_nb)
    bool cw2 = NB <= 2 && (a.d_in % 256) == 0 && (a.d_out % 256) == 0;
    for (int i = 1; i < n_proj; ++i) cw2 = cw2 && (a.more[i - 1].d_out % 256) == 0;
    void (*kernel)(ApplyArgs) = n_proj == 2 ? mfma_wide_kernel<NB, 1, 4, 1, false, 2> : mfma_wide_kernel<NB, 1, 4, 1, false, 3>;
    if constexpr (NB <= 2) {
        if (cw2) kernel = n_proj == 2 ? mfma_wide_kernel<NB, 1, 4, 2, false, 2> : mfma_wide_kernel<NB, 1, 4, 2, false, 3>;
    }
    if (!split) hipLaunchKernelGGL(kernel, dim3(chunk_grid(a, S, 64)), dim3(cw2 ? 512 : 256), 0, stream, a);
    for (int i = 0; i < n_proj; ++i) {
        ApplyArgs g = a;
        if (i > 0) {
            g.y = a.more[i - 1].y; g.ldy = a.more[i - 1].ldy; g.d_out = a.more[i - 1].d_out;
            g.A_pool = a.more[i - 1].A_pool; g.Bt_pool = a.more[i - 1].Bt_pool;
        }
        g.gathered_only = 1;
        launch_mfma_stream<NB, false>(g, S, 1, 4, stream);
    }
}

// bf16 ranks up to 16 that are not multiples of 4 (5, 6, 7, 9, ...): the column-split kernel's any-rank
// shape, 8 wavefronts per 16-row tile; in place with the tile held in registers where it fits
template <bool DIREFT, int PIECES>
void launch_mfma_odd_pieces(const ApplyArgs &a, int64_t S, hipStream_t stream)
{
    void (*kernel)(ApplyArgs);
    int waves = 8;
    if constexpr (DIREFT) {
        // In place the tile stays in registers where it fits.  Up to 4096 columns: 4 wavefronts of 8
        // units each (the 8-wavefront shape of the other ranks has no registers left for the factor
        // block and spills; measured 58 against 55 % of peak at d = 4096), up to 8192: 8 wavefronts of 8
        const int units = (a.d_in >> 7) + ((a.d_in & 127) ? 1 : 0);
        const bool L = a.h_layers != nullptr;
        if (units <= 32) {
            kernel = L ? mfma_tile_layers_kernel<1, 1, 4, 8, false, PIECES> : mfma_tile_kernel<1, 1, 4, 8, true, 1, false, false, PIECES>;
            waves = 4;
        } else if (units <= 64) {
            kernel = L ? mfma_tile_layers_kernel<1, 1, 8, 8, false, PIECES> : mfma_tile_kernel<1, 1, 8, 8, true, 1, false, false, PIECES>;
        } else {
            kernel = L ? mfma_tile_layers_kernel<1, 1, 8, 0, false, PIECES> : mfma_tile_kernel<1, 1, 8, 0, true, 1, false, false, PIECES>;
        }
    } else {
        kernel = a.col_split > 1 ? mfma_tile_kernel<1, 1, 8, 0, false, 1, true, false, PIECES>
                                 : mfma_tile_kernel<1, 1, 8, 0, false, 1, false, false, PIECES>;
    }
    hipLaunchKernelGGL(kernel, dim3(tile_grid(a, S, 16), a.n_layers), dim3(waves * 64), 0, stream, a);
}

template <bool DIREFT>
void launch_mfma_odd(const ApplyArgs &a, int64_t S, hipStream_t stream)
{
    // a unit's [128 columns][rank] block of the expand factor is 16 * rank pieces of 16 bytes: 2 per lane
    // up to rank 8, 4 up to rank 16
    if (a.rank <= 8) launch_mfma_odd_pieces<DIREFT, 2>(a, S, stream);
    else             launch_mfma_odd_pieces<DIREFT, 4>(a, S, stream);
}

// bf16 ranks above 16 that are not multiples of 4, widths multiples of 128: the row-split kernel's any-rank
// form takes the chunks (its basic shape: 4 wavefronts x 16 rows, above rank 64 8 x 16), the per-row kernel
// the gathered tiles (all-token mode: decode rows)
template <bool DIREFT>
void launch_mfma_odd_wide(const ApplyArgs &a, int64_t S, hipStream_t stream)
{
    const int nb = (a.rank + 15) / 16;
    if (nb <= 2)      launch_wide_shape<2, 1, 4, 1, DIREFT, true>(a, S, stream);
    else if (nb <= 4) launch_wide_shape<4, 1, 4, 1, DIREFT, true>(a, S, stream);
    else              launch_wide_shape<8, 1, 8, 1, DIREFT, true>(a, S, stream);
    launch_rows<bf16_tag, DIREFT>(a, S, false, stream);
}

template <bool DIREFT>
void launch_mfma_rank(const ApplyArgs &a, int64_t S, const Knobs &k, hipStream_t stream)
{
    const int nb = (a.rank + 15) / 16;
    if ((a.rank % 4) && a.rank > 16) { launch_mfma_odd_wide<DIREFT>(a, S, stream); return; }   // widths: choose_path
    if (a.rank % 4) { launch_mfma_odd<DIREFT>(a, S, stream); return; }      // rank <= 16 (choose_path)
    if (nb <= 1)      launch_mfma_nb<1, DIREFT>(a, S, k, stream);
    else if (nb <= 2) launch_mfma_nb<2, DIREFT>(a, S, k, stream);
    else if (nb <= 4) launch_mfma_nb<4, DIREFT>(a, S, k, stream);
    else              launch_mfma_nb<8, DIREFT>(a, S, k, stream);
}

template <int RANK, bool DIREFT>
void launch_valu(const ApplyArgs &a, int64_t S, const Knobs &k, hipStream_t stream)
{
    // in place, rows of at most 4096 elements: 2 rows per wavefront stay in registers between the
    // sweeps, so h is read once (d = 4096: 56-59 -> 62-72 % of peak at rank 1-3).  Wider rows
    // would leave one row per wavefront, and the factors re-read for every row cost more than the
    // second read of h (d = 8192, rank 3: 42 % against 60 %).
    if constexpr (DIREFT) {
        if (k.waves == 0 && k.rowblocks == 0 && a.d_in <= 4096) {
            void (*resident)(ApplyArgs) = valu_tile_kernel<RANK, 2, 4, true, 1, 8>;
            if (a.h_layers) resident = valu_tile_layers_kernel<RANK, 2, 4, 8>;
            hipLaunchKernelGGL(resident, dim3(tile_grid(a, S, 8), a.n_layers), dim3(256), 0, stream, a);
            return;
        }
    }
    constexpr int RB = RANK <= 4 ? 4 : 2;
    int waves = k.waves ? k.waves : 4;
    void (*kernel)(ApplyArgs);
    if (waves == 4) {
        kernel = valu_tile_kernel<RANK, RB, 4, DIREFT>;
        if constexpr (DIREFT) { if (a.h_layers) kernel = valu_tile_layers_kernel<RANK, RB, 4>; }
    } else if (waves == 2) {
        kernel = valu_tile_kernel<RANK, RB, 2, DIREFT>;
        if constexpr (DIREFT) { if (a.h_layers) kernel = valu_tile_layers_kernel<RANK, RB, 2>; }
    } else {
        waves = 1;
        kernel = valu_tile_kernel<RANK, RB, 1, DIREFT>;
        if constexpr (DIREFT) { if (a.h_layers) kernel = valu_tile_layers_kernel<RANK, RB, 1>; }
    }
    hipLaunchKernelGGL(kernel, dim3(tile_grid(a, S, RB * waves), a.n_layers), dim3(64 * waves), 0, stream, a);
}

// packed projections at ranks 1..3 (vector-ALU kernel)
template <int SLICES>
void launch_valu_packed(const ApplyArgs &a, int64_t S, hipStream_t stream)
{
    constexpr int RB = 4;
    switch (a.rank) {
    case 1:  hipLaunchKernelGGL((valu_tile_kernel<1, RB, 4, false, SLICES>), dim3(tile_grid(a, S, RB * 4)), dim3(256), 0, stream, a); break;
    case 2:  hipLaunchKernelGGL((valu_tile_kernel<2, RB, 4, false, SLICES>), dim3(tile_grid(a, S, RB * 4)), dim3(256), 0, stream, a); break;
    default: hipLaunchKernelGGL((valu_tile_kernel<3, RB, 4, false, SLICES>), dim3(tile_grid(a, S, RB * 4)), dim3(256), 0, stream, a); break;
    }
}

template <bool DIREFT>
void launch_valu_rank(const ApplyArgs &a, int64_t S, const Knobs &k, hipStream_t stream)
{
    switch (a.rank) {
    case 1: launch_valu<1, DIREFT>(a, S, k, stream); break;
    case 2: launch_valu<2, DIREFT>(a, S, k, stream); break;
    case 3: launch_valu<3, DIREFT>(a, S, k, stream); break;
    case 4: launch_valu<4, DIREFT>(a, S, k, stream); break;
    case 5: launch_valu<5, DIREFT>(a, S, k, stream); break;
    case 6: launch_valu<6, DIREFT>(a, S, k, stream); break;
    case 7: launch_valu<7, DIREFT>(a, S, k, stream); break;
    default: launch_valu<8, DIREFT>(a, S, k, stream); break;
    }
}

template <typename E, bool DIREFT>
void launch_rows(const ApplyArgs &a, int64_t S, bool chunks_too, hipStream_t stream)
{
    void (*chunks_kernel)(ApplyArgs) = row_kernel_chunks<E, DIREFT>;
    void (*short_kernel)(ApplyArgs) = row_kernel_short<E, DIREFT>;
    if constexpr (DIREFT) {
        if (a.h_layers) {
            chunks_kernel = row_layers_kernel_chunks<E>;
            short_kernel = row_layers_kernel_short<E>;
        }
    }
    if (chunks_too) {
        hipLaunchKernelGGL(chunks_kernel,
                           dim3((unsigned)(chunk_capacity(a.T, S) * (CHUNK_ROWS / GROUP_ROWS)), a.n_layers),
                           dim3(ROW_THREADS), 0, stream, a);
    }
    int64_t g = ((gtile_capacity(a.T, S, a.N) * GTILE_ROWS + 7) / 8) * 8;     // a multiple of 8: one share per XCD
    if (g > 4096) g = 4096;
    hipLaunchKernelGGL(short_kernel, dim3((unsigned)g, a.n_layers), dim3(ROW_THREADS), 0, stream, a);
}

enum class Path { Rows, Valu, Mfma };

Path choose_path(int dtype, int rank, bool widths_128, const Knobs &k)
{
    if (dtype != PREFT_BF16 || k.variant == 1) return Path::Rows;
    // matrix-core kernels: multiples of 4, every rank from 5 to 16 (the any-rank shape of the column-split
    // kernel) and, widths being multiples of 128, every rank above (the any-rank form of the row-split
    // kernel); ranks 1..3 are a vector-ALU matter
    const bool valu_ok = rank <= 8, mfma_ok = (rank % 4) == 0 || (rank > 4 && rank < 16) || (rank > 16 && widths_128);
    if (k.variant == 2 && valu_ok) return Path::Valu;
    if ((k.variant == 3 || k.variant == 4) && mfma_ok) return Path::Mfma;
    if (rank <= 3) return Path::Valu;
    if (mfma_ok) return Path::Mfma;
    return Path::Rows;
}

template <bool DIREFT>
int launch_apply(const ApplyArgs &a, int64_t S, int dtype, const Knobs &k, hipStream_t stream)
{
    switch (choose_path(dtype, a.rank, wide_widths_ok(a, 1), k)) {
    case Path::Mfma: {                     // the tile kernels take chunks and gathered tiles alike
        ApplyArgs b = a;
        if (!DIREFT) b.col_split = choose_col_split(a.T, k);
        launch_mfma_rank<DIREFT>(b, S, k, stream);
        break;
    }
    case Path::Valu:
        launch_valu_rank<DIREFT>(a, S, k, stream);
        break;
    default:
        if (dtype == PREFT_BF16) launch_rows<bf16_tag, DIREFT>(a, S, true, stream);
        else                     launch_rows<float, DIREFT>(a, S, true, stream);
        break;
    }
    return check_launch();
}

// LoReFT derived factors of one adapter (App. C.2): D = W - R in the storage type, Rt = R^T.
template <typename E>
__global__ __launch_bounds__(256) void loreft_prepare_kernel(void *D, void *Rt, const void *W, const void *R,
                                                             int32_t d, int32_t rank)
{
    const int64_t n = (int64_t)d * rank;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) {
        const int64_t k = i / d, j = i - k * d;
        const float w = Elem<E>::load1(as_global(W), i), q = Elem<E>::load1(as_global(R), i);
        Elem<E>::store1(as_global(D), i, w - q);
        Elem<E>::store1(as_global(Rt), j * rank + k, q);
    }
}

// the fields of a launch that name the batch and its schedule
void bind_schedule(ApplyArgs &a, void *workspace, int32_t T, int32_t S, int32_t N, int mode)
{
    const ScheduleView v = view_of(workspace, T, S);
    a.T = T; a.S = S; a.N = N; a.all_tokens = (mode & PREFT_ALL_TOKENS) ? 1 : 0;
    a.header = v.header; a.chunks = v.chunks; a.shorts = v.shorts; a.gtiles = v.gtiles;
    a.gathered_only = 0; a.col_split = 1; a.zws = nullptr;
}

// a workspace with room for z lets the LoRA calls of large batches run their sweeps as two launches
void bind_z(ApplyArgs &a, void *workspace, size_t bytes, int32_t T, int32_t S, int32_t rank, int32_t n_proj)
{
    if (T > 1024 && bytes >= z_offset(T, S) + z_bytes(T, S, rank, n_proj))
        a.zws = reinterpret_cast<char *>(workspace) + z_offset(T, S);
}

int check_matrix(const void *p, int64_t ld, int32_t width, int dtype)
{
    const int per16 = dtype == PREFT_BF16 ? 8 : 4;
    if (!p || width <= 0 || ld < width) return PREFT_EINVAL;
    if (!aligned16(p) || (width % per16) != 0 || (ld % per16) != 0) return PREFT_EALIGN;
    return PREFT_OK;
}

// the in-place launch shared by the one-layer and the many-layer DiReFT entry points; `a` names
// the residual stream(s) and the pools
int direft_launch(ApplyArgs a, int64_t ldh, int32_t T, int32_t d, const int32_t *seg_start,
                  const int32_t *seg_adapter, const int32_t *seg_prefill_len, int32_t S, int32_t N, int32_t rank,
                  float scale, int dtype, int mode, void *workspace, void *stream)
{
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    if (!(mode & PREFT_SCHEDULE_READY)) {
        const int rc = launch_schedule(workspace, seg_start, seg_adapter, seg_prefill_len, S, T, N, mode, st);
        if (rc != PREFT_OK) return rc;
    }
    bind_schedule(a, workspace, T, S, N, mode);
    a.ldy = ldh; a.ldx = ldh; a.d_in = d; a.d_out = d;
    a.rank = rank; a.scale = scale;
    return launch_apply<true>(a, S, dtype, knobs_of(mode), st);
}

}  // namespace

extern "C" {

size_t preft_workspace_bytes(int32_t T, int32_t S)
{
    if (T < 0 || S < 0) return 0;
    return workspace_bytes(T, S);
}

size_t preft_workspace_bytes_z(int32_t T, int32_t S, int32_t rank, int32_t n_proj)
{
    if (T < 0 || S < 0 || rank < 1 || rank > PREFT_MAX_RANK || n_proj < 1 || n_proj > PREFT_MAX_PACKED) return 0;
    return z_offset(T, S) + z_bytes(T, S, rank, n_proj);
}

int preft_schedule(void *workspace, size_t bytes, const int32_t *seg_start, const int32_t *seg_adapter,
                   const int32_t *seg_prefill_len, int32_t S, int32_t T, int32_t N, int mode, void *stream)
{
    if (mode & PREFT_SCHEDULE_READY) return PREFT_EINVAL;
    int rc = check_tables(workspace, bytes, seg_start, seg_adapter, seg_prefill_len, S, T, N, mode);
    if (rc != PREFT_OK || T == 0 || S == 0) return rc;
    return launch_schedule(workspace, seg_start, seg_adapter, seg_prefill_len, S, T, N, mode,
                           reinterpret_cast<hipStream_t>(stream));
}

int preft_lora_apply(void *y, int64_t ldy, const void *x, int64_t ldx, int32_t T, int32_t d_in, int32_t d_out,
                     const int32_t *seg_start, const int32_t *seg_adapter, const int32_t *seg_prefill_len,
                     int32_t S, const void *const *A_pool, const void *const *B_pool, int32_t N, int32_t rank,
                     float scale, int dtype, int mode, void *workspace, size_t bytes, void *stream)
{
    if (dtype != PREFT_F32 && dtype != PREFT_BF16) return PREFT_EINVAL;
    int rc = check_tables(workspace, bytes, seg_start, seg_adapter, seg_prefill_len, S, T, N, mode);
    if (rc != PREFT_OK) return rc;
    if (rank < 1 || rank > PREFT_MAX_RANK) return PREFT_EUNSUPPORTED;
    if (T == 0 || S == 0) return PREFT_OK;
    if ((rc = check_matrix(y, ldy, d_out, dtype)) != PREFT_OK) return rc;
    if ((rc = check_matrix(x, ldx, d_in, dtype)) != PREFT_OK) return rc;
    if (!A_pool || !B_pool) return PREFT_EINVAL;
    {   // x and y must not overlap
        const size_t es = dtype == PREFT_BF16 ? 2 : 4;
        const char *y0 = reinterpret_cast<const char *>(y), *x0 = reinterpret_cast<const char *>(x);
        const char *y1 = y0 + ((size_t)(T - 1) * ldy + d_out) * es, *x1 = x0 + ((size_t)(T - 1) * ldx + d_in) * es;
        if (y0 < x1 && x0 < y1) return PREFT_EINVAL;
    }
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    if (!(mode & PREFT_SCHEDULE_READY)) {
        rc = launch_schedule(workspace, seg_start, seg_adapter, seg_prefill_len, S, T, N, mode, st);
        if (rc != PREFT_OK) return rc;
    }
    ApplyArgs a;
    bind_schedule(a, workspace, T, S, N, mode);
    a.y = y; a.x = x; a.ldy = ldy; a.ldx = ldx; a.d_in = d_in; a.d_out = d_out;
    a.A_pool = A_pool; a.Bt_pool = B_pool; a.bias_pool = nullptr; a.rank = rank; a.scale = scale;
    bind_z(a, workspace, bytes, T, S, rank, 1);
    return launch_apply<false>(a, S, dtype, knobs_of(mode), st);
}

int preft_lora_apply_packed(int32_t n_proj, void *const *y, const int64_t *ldy, const int32_t *d_out, const void *x,
                            int64_t ldx, int32_t T, int32_t d_in, const int32_t *seg_start,
                            const int32_t *seg_adapter, const int32_t *seg_prefill_len, int32_t S,
                            const void *const *const *A_pools, const void *const *const *B_pools, int32_t N,
                            int32_t rank, float scale, int dtype, int mode, void *workspace, size_t bytes,
                            void *stream)
{
    if (n_proj < 1 || n_proj > PREFT_MAX_PACKED || !y || !ldy || !d_out || !A_pools || !B_pools) return PREFT_EINVAL;
    if (dtype != PREFT_F32 && dtype != PREFT_BF16) return PREFT_EINVAL;
    int rc = check_tables(workspace, bytes, seg_start, seg_adapter, seg_prefill_len, S, T, N, mode);
    if (rc != PREFT_OK) return rc;
    if (rank < 1 || rank > PREFT_MAX_RANK) return PREFT_EUNSUPPORTED;
    if (T == 0 || S == 0) return PREFT_OK;
    if ((rc = check_matrix(x, ldx, d_in, dtype)) != PREFT_OK) return rc;
    const size_t es = dtype == PREFT_BF16 ? 2 : 4;
    const char *x0 = reinterpret_cast<const char *>(x), *x1 = x0 + ((size_t)(T - 1) * ldx + d_in) * es;
    for (int32_t i = 0; i < n_proj; ++i) {
        if ((rc = check_matrix(y[i], ldy[i], d_out[i], dtype)) != PREFT_OK) return rc;
        if (!A_pools[i] || !B_pools[i]) return PREFT_EINVAL;
        const char *y0 = reinterpret_cast<const char *>(y[i]), *y1 = y0 + ((size_t)(T - 1) * ldy[i] + d_out[i]) * es;
        if (y0 < x1 && x0 < y1) return PREFT_EINVAL;                       // x and y must not overlap
        // outputs must not share an element: disjoint buffers, or disjoint column ranges of one
        // buffer (same row stride, both inside one row pitch); anything else that overlaps is refused
        for (int32_t j = 0; j < i; ++j) {
            const char *z0 = reinterpret_cast<const char *>(y[j]);
            const char *z1 = z0 + ((size_t)(T - 1) * ldy[j] + d_out[j]) * es;
            if (!(y0 < z1 && z0 < y1)) continue;
            if (ldy[i] != ldy[j]) return PREFT_EINVAL;
            const bool i_low = y0 < z0;
            const size_t w_lo = (size_t)(i_low ? d_out[i] : d_out[j]) * es, w_hi = (size_t)(i_low ? d_out[j] : d_out[i]) * es;
            const size_t delta = (size_t)(i_low ? z0 - y0 : y0 - z0), pitch = (size_t)ldy[i] * es;
            if (delta < w_lo || delta + w_hi > pitch) return PREFT_EINVAL;
        }
    }
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    if (!(mode & PREFT_SCHEDULE_READY)) {
        rc = launch_schedule(workspace, seg_start, seg_adapter, seg_prefill_len, S, T, N, mode, st);
        if (rc != PREFT_OK) return rc;
    }
    const int ready = mode | PREFT_SCHEDULE_READY;
    const Knobs k = knobs_of(mode);
    const bool fused_mfma = n_proj > 1 && dtype == PREFT_BF16 && rank >= 4 && rank <= 16 &&
                            (k.variant == 0 || k.variant == 3 || k.variant == 5);
    const bool fused_valu = n_proj > 1 && dtype == PREFT_BF16 && rank <= 3 && (k.variant == 0 || k.variant == 2) &&
                            (k.waves == 0 || k.waves == 4);
    bool fused_wide = n_proj > 1 && dtype == PREFT_BF16 && rank > 16 && rank <= 64 &&
                      (k.variant == 0 || k.variant == 4 || k.variant == 5) && k.waves == 0 && k.rowblocks == 0 && (d_in % 128) == 0 &&
                      choose_col_split(T, k) == 1;
    for (int32_t i = 0; i < n_proj && fused_wide; ++i) fused_wide = (d_out[i] % 128) == 0;
    const bool fused = fused_mfma || fused_valu || fused_wide;
    if (!fused) {                                  // same result, one launch per projection
        for (int32_t i = 0; i < n_proj; ++i) {
            rc = preft_lora_apply(y[i], ldy[i], x, ldx, T, d_in, d_out[i], seg_start, seg_adapter, seg_prefill_len, S,
                                  A_pools[i], B_pools[i], N, rank, scale, dtype, ready, workspace, bytes, stream);
            if (rc != PREFT_OK) return rc;
        }
        return PREFT_OK;
    }
    ApplyArgs a;
    bind_schedule(a, workspace, T, S, N, mode);
    a.y = y[0]; a.x = x; a.ldy = ldy[0]; a.ldx = ldx; a.d_in = d_in; a.d_out = d_out[0];
    a.A_pool = A_pools[0]; a.Bt_pool = B_pools[0]; a.bias_pool = nullptr; a.rank = rank; a.scale = scale;
    for (int32_t i = 1; i < n_proj; ++i) {
        a.more[i - 1].y = y[i]; a.more[i - 1].ldy = ldy[i]; a.more[i - 1].d_out = d_out[i];
        a.more[i - 1].A_pool = A_pools[i]; a.more[i - 1].Bt_pool = B_pools[i];
    }
    if (fused_wide) {
        bind_z(a, workspace, bytes, T, S, rank, n_proj);
        if (rank <= 32) launch_mfma_wide_packed<2>(a, n_proj, S, k, st);
        else            launch_mfma_wide_packed<4>(a, n_proj, S, k, st);
    } else if (fused_mfma) {
        a.col_split = choose_col_split(T, k);
        const int pieces = (rank % 4) == 0 ? 0 : rank < 8 ? 2 : 4;      // the any-rank shape's block pieces per lane
        if (n_proj == 2) {
            if (pieces == 0)      launch_mfma_packed<2>(a, S, k, st);
            else if (pieces == 2) launch_mfma_packed<2, 2>(a, S, k, st);
            else                  launch_mfma_packed<2, 4>(a, S, k, st);
        } else {
            if (pieces == 0)      launch_mfma_packed<3>(a, S, k, st);
            else if (pieces == 2) launch_mfma_packed<3, 2>(a, S, k, st);
            else                  launch_mfma_packed<3, 4>(a, S, k, st);
        }
    } else {
        if (n_proj == 2) launch_valu_packed<2>(a, S, st);
        else             launch_valu_packed<3>(a, S, st);
    }
    return check_launch();
}

int preft_loreft_prepare(void *D, void *Rt, const void *W, const void *R, int32_t d, int32_t rank, int dtype,
                         void *stream)
{
    if (dtype != PREFT_F32 && dtype != PREFT_BF16) return PREFT_EINVAL;
    if (!D || !Rt || !W || !R || d <= 0) return PREFT_EINVAL;
    if (rank < 1 || rank > PREFT_MAX_RANK) return PREFT_EUNSUPPORTED;
    if (!aligned16(D) || !aligned16(Rt) || !aligned16(W) || !aligned16(R)) return PREFT_EALIGN;
    {   // outputs must not overlap the inputs or each other
        const size_t bytes = (size_t)d * rank * (dtype == PREFT_BF16 ? 2 : 4);
        const char *p[4] = {reinterpret_cast<const char *>(D), reinterpret_cast<const char *>(Rt),
                            reinterpret_cast<const char *>(W), reinterpret_cast<const char *>(R)};
        for (int a = 0; a < 2; ++a)
            for (int b = a + 1; b < 4; ++b)
                if (p[a] < p[b] + bytes && p[b] < p[a] + bytes) return PREFT_EINVAL;
    }
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    const int64_t n = (int64_t)d * rank;
    const unsigned grid = (unsigned)((n + 255) / 256 < 4096 ? (n + 255) / 256 : 4096);
    if (dtype == PREFT_BF16)
        hipLaunchKernelGGL((loreft_prepare_kernel<bf16_tag>), dim3(grid), dim3(256), 0, st, D, Rt, W, R, d, rank);
    else
        hipLaunchKernelGGL((loreft_prepare_kernel<float>), dim3(grid), dim3(256), 0, st, D, Rt, W, R, d, rank);
    return check_launch();
}

int preft_loreft_apply(void *h, int64_t ldh, int32_t T, int32_t d, const int32_t *seg_start,
                       const int32_t *seg_adapter, const int32_t *seg_prefill_len, int32_t S,
                       const void *const *D_pool, const void *const *Rt_pool, const void *const *b_pool,
                       int32_t N, int32_t rank, float scale, int dtype, int mode, void *workspace, size_t bytes,
                       void *stream)
{
    // h += s R^T (W h + b - R h) = s Rt (D h + b): the in-place kernels with the derived factors
    return preft_direft_apply(h, ldh, T, d, seg_start, seg_adapter, seg_prefill_len, S, D_pool, Rt_pool, b_pool, N,
                              rank, scale, dtype, mode, workspace, bytes, stream);
}

int preft_direft_apply(void *h, int64_t ldh, int32_t T, int32_t d, const int32_t *seg_start,
                       const int32_t *seg_adapter, const int32_t *seg_prefill_len, int32_t S,
                       const void *const *W1_pool, const void *const *W2t_pool, const void *const *b_pool,
                       int32_t N, int32_t rank, float scale, int dtype, int mode, void *workspace, size_t bytes,
                       void *stream)
{
    if (dtype != PREFT_F32 && dtype != PREFT_BF16) return PREFT_EINVAL;
    int rc = check_tables(workspace, bytes, seg_start, seg_adapter, seg_prefill_len, S, T, N, mode);
    if (rc != PREFT_OK) return rc;
    if (rank < 1 || rank > PREFT_MAX_RANK) return PREFT_EUNSUPPORTED;
    if (T == 0 || S == 0) return PREFT_OK;
    if ((rc = check_matrix(h, ldh, d, dtype)) != PREFT_OK) return rc;
    if (!W1_pool || !W2t_pool) return PREFT_EINVAL;
    ApplyArgs a;
    a.y = h; a.x = h; a.A_pool = W1_pool; a.Bt_pool = W2t_pool; a.bias_pool = b_pool;
    return direft_launch(a, ldh, T, d, seg_start, seg_adapter, seg_prefill_len, S, N, rank, scale, dtype, mode,
                         workspace, stream);
}

int preft_direft_apply_static(void *h, int64_t ldh, int32_t T, int32_t d, const int32_t *seg_start,
                              const int32_t *seg_adapter, const int32_t *seg_prefill_len, int32_t S,
                              const void *const *W1_pool, const void *const *W2t_pool, const void *const *b_pool,
                              int32_t N, int32_t rank, float scale, int dtype, int mode, void *stream)
{
    // sizes first (host arithmetic only): the schedule of this batch must fit the static area
    if (T < 0 || S < 0) return PREFT_EINVAL;
    if (workspace_bytes(T, S) > (size_t)PREFT_STATIC_SCRATCH_BYTES) return PREFT_ETOOLARGE;
    if (dtype != PREFT_F32 && dtype != PREFT_BF16) return PREFT_EINVAL;
    if (T == 0 || S == 0) {     // nothing to do: same answers as preft_direft_apply, without touching the device
        const int rc = check_tables(nullptr, 0, seg_start, seg_adapter, seg_prefill_len, S, T, N, mode);
        if (rc != PREFT_OK) return rc;
        return (rank < 1 || rank > PREFT_MAX_RANK) ? PREFT_EUNSUPPORTED : PREFT_OK;
    }
    void *area = nullptr;
    const int rc = static_scratch_of(&area);
    if (rc != PREFT_OK) return rc;
    return preft_direft_apply(h, ldh, T, d, seg_start, seg_adapter, seg_prefill_len, S, W1_pool, W2t_pool, b_pool, N,
                              rank, scale, dtype, mode, area, (size_t)PREFT_STATIC_SCRATCH_BYTES, stream);
}

int preft_direft_apply_layers(void *const *h_layers, int64_t ldh, int32_t n_layers, int32_t T, int32_t d,
                              const int32_t *seg_start, const int32_t *seg_adapter,
                              const int32_t *seg_prefill_len, int32_t S, const void *const *const *W1_pools,
                              const void *const *const *W2t_pools, const void *const *const *b_pools, int32_t N,
                              int32_t rank, float scale, int dtype, int mode, void *workspace, size_t bytes,
                              void *stream)
{
    if (dtype != PREFT_F32 && dtype != PREFT_BF16) return PREFT_EINVAL;
    if (n_layers < 0 || n_layers > PREFT_MAX_LAYERS) return PREFT_EINVAL;
    int rc = check_tables(workspace, bytes, seg_start, seg_adapter, seg_prefill_len, S, T, N, mode);
    if (rc != PREFT_OK) return rc;
    if (rank < 1 || rank > PREFT_MAX_RANK) return PREFT_EUNSUPPORTED;
    if (T == 0 || S == 0 || n_layers == 0) return PREFT_OK;
    if (!h_layers || !W1_pools || !W2t_pools) return PREFT_EINVAL;
    // the residual streams themselves are named on the device: only their common shape is checked
    const int per16 = dtype == PREFT_BF16 ? 8 : 4;
    if (d <= 0 || ldh < d) return PREFT_EINVAL;
    if ((d % per16) || (ldh % per16)) return PREFT_EALIGN;
    ApplyArgs a;
    a.y = nullptr; a.x = nullptr; a.A_pool = nullptr; a.Bt_pool = nullptr; a.bias_pool = nullptr;
    a.h_layers = h_layers; a.A_layers = W1_pools; a.Bt_layers = W2t_pools; a.bias_layers = b_pools;
    a.n_layers = n_layers;
    return direft_launch(a, ldh, T, d, seg_start, seg_adapter, seg_prefill_len, S, N, rank, scale, dtype, mode,
                         workspace, stream);
}

int preft_schedule_counts(const void *workspace, int32_t *counts, void *stream)
{
    if (!workspace || !counts) return PREFT_EINVAL;
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    int32_t header[HEADER_INTS];
    if (hipMemcpyAsync(header, workspace, sizeof(header), hipMemcpyDeviceToHost, st) != hipSuccess)
        return PREFT_EHIP;
    if (hipStreamSynchronize(st) != hipSuccess) return PREFT_EHIP;
    counts[0] = header[HDR_CHUNKS]; counts[1] = header[HDR_SHORT_ROWS]; counts[2] = header[HDR_ACTIVE];
    return header[HDR_MISMATCH] ? PREFT_ESCHEDULE : PREFT_OK;
}

const char *preft_strerror(int code)
{
    switch (code) {
    case PREFT_OK:           return "ok";
    case PREFT_EINVAL:       return "invalid argument (null pointer, negative size, bad enum, overlapping x and y, or row stride below the width)";
    case PREFT_EUNSUPPORTED: return "unsupported rank (must be 1..128)";
    case PREFT_EALIGN:       return "pointer, width or row stride not a multiple of 16 bytes";
    case PREFT_EWORKSPACE:   return "workspace missing, misaligned or smaller than preft_workspace_bytes(T, S)";
    case PREFT_EHIP:         return "HIP runtime error (launch, copy or allocation)";
    case PREFT_ECAPACITY:    return "more distinct adapters in one batch than the slot manager has slots";
    case PREFT_ETOOLARGE:    return "batch too large for the static schedule area of preft_direft_apply_static (preft_workspace_bytes(T, S) exceeds PREFT_STATIC_SCRATCH_BYTES)";
    case PREFT_ESCHEDULE:    return "an apply call named another T, S, N or position set than the schedule in its workspace was built for; that call did nothing";
    default:                 return "unknown preft error code";
    }
}

int preft_version(void) { return 200; }

}  // extern "C"
