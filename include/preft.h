/*
 * preft.h -- C ABI of the MI355X (gfx950) prefill-only adapter-apply library.
 *
 * The library applies per-request adapters to a flattened, mixed prefill+decode token
 * batch, in place, on one GPU:
 *
 *   LoRA    (paper Eq. 2):             y_t <- y_t + s * B_i (A_i x_t)
 *   DiReFT  (paper Eq. 3, App. C.2):   h_t <- h_t + s * W2_i^T (W1_i h_t + b_i)
 *   LoReFT  (paper App. C.2):          h_t <- h_t + s * R_i^T (W_i h_t + b_i - R_i h_t)
 *
 * for every row t whose position lies in the adapter's position set (paper Eq. 1):
 * the prompt positions of its sequence only (PREFT_PREFILL_ONLY, paper Eq. 4) or every
 * position (PREFT_ALL_TOKENS, the all-position set of Sec. 3.2).  Every other row -- decode
 * tokens in prefill-only mode, sequences without an adapter -- is neither read nor
 * written: it stays bit-identical.
 *
 * Batch description (App. D.3: the flattened batch and its cumulative sequence offsets;
 * App. D.5/D.6: one adapter and one position schedule per request):
 *   seg_start[S+1]      int32, device.  Rows seg_start[s] .. seg_start[s+1]-1 belong to
 *                       sequence s.  seg_start[0] = 0, seg_start[S] = T, non-decreasing.
 *   seg_adapter[S]      int32, device.  Index into the adapter pools; a value < 0 or >= N
 *                       means "no adapter" (rows untouched).
 *   seg_prefill_len[S]  int32, device.  How many leading rows of the segment are prompt
 *                       positions (clamped to [0, segment length]).  A decode token is a
 *                       segment of length 1 with prefill length 0; a prompt chunk has
 *                       prefill length == length.  Ignored in PREFT_ALL_TOKENS mode.
 * The tables are read on the device only; their contents are not validated on the host
 * (that would need a synchronisation).  Every segment is clamped to [0,T) on the device and
 * every list of the schedule is cut back to its capacity, so a malformed table (offsets that
 * decrease, segments that overlap) cannot cause an out-of-range access; its result is
 * unspecified (a row named by two segments may be updated twice).
 *
 * Adapter pools: device arrays of N device pointers, one matrix per adapter, all of one
 * rank, row-major, in the activation dtype:
 *   A_pool[i]   [rank, d_in]   the paper's A as printed in Eq. 2
 *   B_pool[i]   [d_out, rank]  the paper's B as printed in Eq. 2
 *   W1_pool[i]  [rank, d]      the paper's A of Eq. 3
 *   W2t_pool[i] [d, rank]      the TRANSPOSE of the paper's B of Eq. 3 (rank contiguous)
 *   b_pool[i]   [rank]         the paper's b of Eq. 3; b_pool == NULL, or an entry
 *                              b_pool[i] == NULL, means b = 0 (for that adapter)
 * Every matrix must be 16-byte aligned.  Pool slots are caller-owned and may be overwritten
 * in place between calls.  Only the slots named by active segments are dereferenced.
 *
 * Ownership / execution: every pointer is caller-owned device memory unless marked
 * "host".  The schedule and apply calls allocate nothing and the library keeps no state
 * between calls: whatever selects a kernel travels in the arguments of the call.  Only the
 * optional slot manager at the end of this header owns memory.  Calls only
 * enqueue work on `stream` (a hipStream_t passed as void*, NULL = the default stream) and
 * return; they never synchronise.  All launch shapes depend on host-visible sizes only,
 * so a call may be captured into a HIP graph.
 *
 * Arithmetic: products and sums are accumulated in fp32 (PREFT_BF16 and PREFT_F32); the
 * rank-r intermediate stays in fp32; each output element is rounded once, to nearest
 * even, to the activation dtype.
 *
 * Errors: every entry point returns PREFT_OK (0) or a negative code and leaves the output
 * untouched when it returns an error detected before launch.
 */
#ifndef PREFT_H
#define PREFT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* mode: position set, optionally OR-ed with PREFT_SCHEDULE_READY */
enum {
    PREFT_PREFILL_ONLY   = 0,      /* paper Eq. 4: prompt positions only                 */
    PREFT_ALL_TOKENS     = 1,      /* all positions: the conventional PEFT baseline      */
    PREFT_SCHEDULE_READY = 0x100   /* workspace already holds this batch's schedule      */
};

/*
 * Test-only kernel selection, OR-ed into `mode` (bits 16..30).  A serving call leaves these
 * bits zero and gets the library's own choice; tests and benchmarks use them to reach every
 * kernel family on any input.  They change which kernel runs, never what is computed.  A value
 * a kernel family does not offer selects its nearest shape; an undefined value is PREFT_EINVAL.
 *   PREFT_TEST_VARIANT(v)    0 = automatic
 *                            1 = per-row kernel everywhere
 *                            2 = vector-ALU tile kernel where it applies (bf16, rank <= 8)
 *                            3 = MFMA tile kernel, column-split shape (bf16, rank a multiple
 *                                of 4 or between 5 and 15)
 *                            4 = MFMA tile kernel, row-split shape with the factors shared
 *                                through LDS where it applies (rank a multiple of 4 or above
 *                                16, widths multiples of 128), and no register-resident DiReFT
 *                            5 = automatic, but both sweeps of a LoRA call in one launch even
 *                                if the workspace has room for z (preft_workspace_bytes_z)
 *   PREFT_TEST_WAVES(w)      wavefronts per tile workgroup: 0 = automatic, else 1, 2, 4 or 8
 *                            (any non-zero value also makes DiReFT stream its tile instead
 *                            of holding it in registers)
 *   PREFT_TEST_ROWBLOCKS(b)  MFMA kernels: 16-row blocks per wavefront: 0 = automatic, 1 or 2
 *   PREFT_TEST_COLSPLIT(c)   LoRA, MFMA column-split kernel: workgroups that share a tile, each
 *                            writing its share of the output columns: 0 = automatic (4 for
 *                            batches of up to 1024 rows, else 1), or 1..15.  Together with
 *                            variant 4 it names the column groups of the row-split kernel
 *                            instead: 0 = automatic, 1 or 2
 *   PREFT_TEST_RESIDENT(n)   0 = automatic.  LoRA: 1 = two launches (preft_workspace_bytes_z)
 *                            wherever that form exists, whatever the batch size.  In-place
 *                            MFMA kernel at rank 20..32 (automatic: 32-row tiles streamed in
 *                            both sweeps): 3 = every wavefront keeps 8 of its
 *                            128-column units in registers between the sweeps (half of a
 *                            32-row tile of 8192 columns) and streams the rest twice
 */
#define PREFT_TEST_VARIANT(v)   (((v) & 7) << 16)
#define PREFT_TEST_WAVES(w)     (((w) & 15) << 19)
#define PREFT_TEST_ROWBLOCKS(b) (((b) & 3) << 23)
#define PREFT_TEST_COLSPLIT(c)  (((c) & 15) << 25)
#define PREFT_TEST_RESIDENT(n)  (((n) & 3) << 29)

/* dtype of activations AND adapter weights */
enum { PREFT_F32 = 0, PREFT_BF16 = 1 };

enum {
    PREFT_OK           =  0,
    PREFT_EINVAL       = -1,   /* null pointer, negative size, bad enum, ld < width      */
    PREFT_EUNSUPPORTED = -2,   /* rank outside 1..PREFT_MAX_RANK                         */
    PREFT_EALIGN       = -3,   /* base pointer or row stride not 16-byte aligned, or a   */
                               /* width that is not a multiple of 16 bytes               */
    PREFT_EWORKSPACE   = -4,   /* workspace missing, misaligned or too small             */
    PREFT_EHIP         = -5,   /* the HIP runtime refused a launch, copy or allocation   */
    PREFT_ECAPACITY    = -6,   /* slot manager: more distinct adapters than slots        */
    PREFT_ESCHEDULE    = -7,   /* preft_schedule_counts: an apply call found a schedule  */
                               /* built for another T, S, N or position set, and did nothing */
    PREFT_ETOOLARGE    = -8    /* preft_direft_apply_static: the batch's schedule does   */
                               /* not fit the static area                                */
};

#define PREFT_MAX_RANK 128
#define PREFT_MAX_LAYERS 1024      /* residual streams per preft_direft_apply_layers call */
#define PREFT_MAX_PACKED 3      /* projections one packed call may fuse */
#define PREFT_MAX_PARTS 32      /* matrices per adapter a slot manager may hold */

/*
 * Bytes of device workspace that hold the schedule of a batch of T rows in S segments.
 * The workspace must be 16-byte aligned.  Returns 0 if T or S is negative.
 */
size_t preft_workspace_bytes(int32_t T, int32_t S);

/*
 * Bytes of a workspace that, beyond the schedule, has room for the intermediate z = A_i x of Eq. 2 of
 * every active row: LoRA calls of up to `rank` with up to n_proj outputs per call.  A LoRA call
 * (bf16, rank 20..64 in multiples of 4, d_in a multiple of 128, every d_out a multiple of 256) on a
 * batch of 8192 to 131 072 rows that is handed at least this many bytes runs its two sweeps as two
 * launches -- shrink into z, then the expand in 2-D tiles -- which measured 4 to 12 points of
 * bandwidth faster at that size (a batch of 38 416 rows, rank 32 and 64).  With fewer bytes, or
 * outside those limits, the same call runs as before.  The result is the same bit for bit.  The z area lies behind the schedule and is rewritten by every such call: calls that
 * share a workspace must be ordered on one stream, as they must be for the schedule already.
 * Returns 0 for a negative T or S, a rank outside 1..PREFT_MAX_RANK or n_proj outside
 * 1..PREFT_MAX_PACKED.
 */
size_t preft_workspace_bytes_z(int32_t T, int32_t S, int32_t rank, int32_t n_proj);

/*
 * Token-segment scheduler (paper Eq. 1 and Eq. 4; App. D.3 "position mask", which the
 * paper derives once per forward pass from the sequence offsets and skips for all-decode
 * batches).  Reads the three segment tables on the device and writes into `workspace` the
 * list of work units that cover exactly the active rows -- inactive rows appear in no
 * unit, and a batch without active rows yields an empty list, which makes every apply
 * call that consumes it return after an empty launch.
 *
 * The schedule depends on (tables, S, T, N, position set) only -- not on dtype, rank or
 * widths -- so one schedule serves every projection and layer of an engine step: pass the
 * same workspace with mode | PREFT_SCHEDULE_READY to the apply calls that follow on the
 * same stream, with the same T, S, N and position set.  The schedule records those four values
 * and every apply kernel compares them with its own arguments first: a call that names another
 * batch shape or position set does nothing at all (its launch sizes are bounds computed from
 * T, S and N, so it could only process part of the batch, or the wrong rows) and marks the
 * workspace, which preft_schedule_counts reports as PREFT_ESCHEDULE.
 *
 * mode: PREFT_PREFILL_ONLY or PREFT_ALL_TOKENS.
 */
int preft_schedule(void *workspace, size_t workspace_bytes,
                   const int32_t *seg_start, const int32_t *seg_adapter,
                   const int32_t *seg_prefill_len, int32_t S, int32_t T, int32_t N,
                   int mode, void *stream);

/*
 * Segmented multi-adapter LoRA (paper Eq. 2 under the position set of Eq. 1/4):
 *   y[t, :] += scale * B_i (A_i x[t, :])     for active rows t of segments with adapter i.
 *
 * y  [T, d_out]  in/out, row stride ldy elements.   x  [T, d_in]  in, row stride ldx.
 * x and y must not overlap.  d_in, d_out, ldx, ldy must be multiples of 16 bytes worth of
 * elements (8 for bf16, 4 for fp32) and x, y 16-byte aligned, else PREFT_EALIGN.  That is the
 * rule for correctness; for full speed rows should start on 128-byte boundaries (bases 128-byte
 * aligned, ldx and ldy multiples of 64 bf16 elements): the kernels move rows in 256-byte pieces,
 * and rows that start 16 bytes off a line cost about a fifth of the bandwidth.  Row pitches that
 * are powers of two measured 5-10 % faster on MI355X than the dense pitch of a wide buffer (a
 * 14336-wide bf16 buffer with rows every 16384 elements: 64 -> 71 % of peak bandwidth): a caller
 * that owns the layout of its activations should pad wide rows to the next power of two.
 * rank in 1..PREFT_MAX_RANK.  scale is the paper's alpha (or alpha/r), already evaluated.
 * Every rank is computed as given (rank 1 is not padded to 8 in memory).  Every bf16 rank runs on
 * the library's fast kernels (vector-ALU and matrix-core kernels; ranks that are not multiples of 4
 * a few points below their neighbours), with one exception: a rank above 16 that is not a multiple
 * of 4 needs d_in and d_out to be multiples of 128 for that, and takes the slow per-row kernels
 * otherwise (an adapter of such a rank and such widths is served faster when its factors are
 * zero-padded to the next multiple of 4).  fp32 takes the per-row kernels.
 * Unless mode carries PREFT_SCHEDULE_READY the call first runs the scheduler into
 * `workspace` (>= preft_workspace_bytes(T, S) bytes).
 * T == 0 or S == 0 returns PREFT_OK without launching.
 */
int preft_lora_apply(void *y, int64_t ldy, const void *x, int64_t ldx,
                     int32_t T, int32_t d_in, int32_t d_out,
                     const int32_t *seg_start, const int32_t *seg_adapter,
                     const int32_t *seg_prefill_len, int32_t S,
                     const void *const *A_pool, const void *const *B_pool, int32_t N,
                     int32_t rank, float scale, int dtype, int mode,
                     void *workspace, size_t workspace_bytes, void *stream);

/*
 * Packed projections: n_proj (1..PREFT_MAX_PACKED) LoRA applications that read the SAME x --
 * the q, k and v projections of an attention block, the gate and up projections of an MLP
 * (the paper's LoRA targets, App. A.1) -- as one call:
 *   y_p[t, :] += scale * B_{p,i} (A_{p,i} x[t, :])      p = 0 .. n_proj-1, active rows t.
 * Each projection has its own output y[p] ([T, d_out[p]], row stride ldy[p]) and its own pools
 * A_pools[p] / B_pools[p] (device pointer tables as in preft_lora_apply); y, ldy, d_out, A_pools
 * and B_pools are HOST arrays of n_proj entries.  The outputs may be separate buffers or
 * disjoint column ranges of one buffer (a fused qkv or gate-up output: same row stride, every
 * range inside one row); any other overlap, and any overlap with x, is PREFT_EINVAL.
 * The result is that of n_proj preft_lora_apply calls.  For bf16 and rank 1..16,
 * and for rank 17..64 when every width is a multiple of 128 and the batch has more
 * than 1024 rows, they run as one launch that reads x once; otherwise the call issues one launch per
 * projection.
 */
int preft_lora_apply_packed(int32_t n_proj, void *const *y, const int64_t *ldy, const int32_t *d_out,
                            const void *x, int64_t ldx, int32_t T, int32_t d_in,
                            const int32_t *seg_start, const int32_t *seg_adapter,
                            const int32_t *seg_prefill_len, int32_t S,
                            const void *const *const *A_pools, const void *const *const *B_pools,
                            int32_t N, int32_t rank, float scale, int dtype, int mode,
                            void *workspace, size_t workspace_bytes, void *stream);

/*
 * Segmented multi-adapter DiReFT (paper Eq. 3 with the prefactor of App. C.2, under the
 * position set of Eq. 1/4), in place on the residual stream:
 *   h[t, :] += scale * W2_i^T (W1_i h[t, :] + b_i)     for active rows t.
 * Every read of a row precedes every write of that row.  scale = 1 gives Eq. 3 as
 * printed; scale = 1/sqrt(rank) gives the rank-stable form.  The prefactor multiplies the
 * bias term too.
 *
 * h [T, d] in/out, row stride ldh elements; alignment rules as for preft_lora_apply.
 * b_pool may be NULL (no bias for any adapter), and so may single entries of it (Eq. 3 with
 * b = 0 for that adapter); every other entry named by an active segment must be a valid pointer.
 */
int preft_direft_apply(void *h, int64_t ldh, int32_t T, int32_t d,
                       const int32_t *seg_start, const int32_t *seg_adapter,
                       const int32_t *seg_prefill_len, int32_t S,
                       const void *const *W1_pool, const void *const *W2t_pool,
                       const void *const *b_pool, int32_t N,
                       int32_t rank, float scale, int dtype, int mode,
                       void *workspace, size_t workspace_bytes, void *stream);

/*
 * preft_direft_apply for callers that cannot allocate and have no workspace to hand over: code
 * under HIP-graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same operation,
 * same arguments and same results, bit for bit, as preft_direft_apply -- except that the schedule is
 * kept in a static area of device memory inside the library (PREFT_STATIC_SCRATCH_BYTES bytes,
 * which every GPU the library runs on holds until the process ends) instead of a caller workspace.
 * The call allocates and frees nothing, on the host or the device.
 *
 * Limit: preft_workspace_bytes(T, S) <= PREFT_STATIC_SCRATCH_BYTES (every batch of up to 32 768
 * rows, whatever S; T = 262 144 rows in up to 8192 segments), else PREFT_ETOOLARGE, checked
 * before anything touches the device.
 * All calls on one GPU share that GPU's area, which keeps the previous call's schedule: a call
 * rewrites everything it reads from it (nothing there has to start at zero), and with
 * PREFT_SCHEDULE_READY it reuses the schedule the previous static call on this GPU left, under the
 * same T, S, N and position-set check as any apply call.  Two calls that overlap in time on one GPU
 * (different streams, different threads) race on the area: order them.  The first call on a device
 * looks up the area's address (no allocation); under graph capture make one call before capturing.
 */
#define PREFT_STATIC_SCRATCH_BYTES (1u << 20)
int preft_direft_apply_static(void *h, int64_t ldh, int32_t T, int32_t d,
                              const int32_t *seg_start, const int32_t *seg_adapter,
                              const int32_t *seg_prefill_len, int32_t S,
                              const void *const *W1_pool, const void *const *W2t_pool,
                              const void *const *b_pool, int32_t N,
                              int32_t rank, float scale, int dtype, int mode, void *stream);

/*
 * DiReFT on n_layers residual streams in one launch: the paper intervenes at every layer
 * (App. A.2), each layer with weights of its own, and an engine step of a few dozen rows is
 * bound by launches, not bytes.  Layer l applies
 *   h_layers[l][t, :] += scale * W2_{l,i}^T (W1_{l,i} h_layers[l][t, :] + b_{l,i})
 * to its own buffer, exactly as preft_direft_apply(h_layers[l], ..., W1_pools[l], W2t_pools[l],
 * b_pools[l], ...) would; the layers share T, d, ldh, the segment tables, rank, scale and one
 * schedule.  The caller decides that the buffers may be processed side by side (states kept per
 * layer, independent streams); buffers that overlap give undefined results.
 *
 * h_layers, W1_pools, W2t_pools and b_pools are DEVICE arrays of n_layers device pointers: the
 * residual streams ([T, d], row stride ldh, each 16-byte aligned -- not checkable from the host)
 * and, per layer, pointer tables as in preft_direft_apply.  b_pools may be NULL (no bias in any
 * layer); an entry of it may be NULL (no bias in that layer).
 * n_layers in 0..PREFT_MAX_LAYERS (0: nothing to do); everything else as preft_direft_apply.
 * With the derived pools of preft_loreft_prepare the same call applies LoReFT.
 */
int preft_direft_apply_layers(void *const *h_layers, int64_t ldh, int32_t n_layers, int32_t T, int32_t d,
                              const int32_t *seg_start, const int32_t *seg_adapter,
                              const int32_t *seg_prefill_len, int32_t S,
                              const void *const *const *W1_pools, const void *const *const *W2t_pools,
                              const void *const *const *b_pools, int32_t N,
                              int32_t rank, float scale, int dtype, int mode,
                              void *workspace, size_t workspace_bytes, void *stream);

/*
 * LoReFT (paper App. C.2): h[t, :] += scale * R_i^T (W_i h[t, :] + b_i - R_i h[t, :]), with
 * W_i, R_i in R^{rank x d} (R_i the materialised rotation) and b_i in R^rank.
 *
 * The rotation enters twice, once per layout the kernels stream (rank-major for the
 * projection, column-major for the write-back), and the projection needs only W_i - R_i.  Like
 * the derived tensors the paper caches outside its compiled region (App. D.3), these are
 * computed once per weight update, not per call:
 *
 * preft_loreft_prepare writes, for one adapter,
 *   D  [rank, d]  = W - R, rounded once (to nearest even) to the storage type,
 *   Rt [d, rank]  = R transposed,
 * from W, R [rank, d] (all device pointers, 16-byte aligned, contiguous; D and Rt are
 * caller-owned and must not overlap W or R).  In bf16 the rounding of W - R is exact whenever
 * W and R are within a factor two of each other elementwise (always at the zero-delta
 * initialisation W = R and close to it); in general it perturbs each element of D by at most
 * 2^-9 relative.
 *
 * preft_loreft_apply then computes h[t, :] += scale * Rt_i (D_i h[t, :] + b_i) on the active
 * rows; its arguments, layouts and rules are those of preft_direft_apply with W1_pool = D_pool
 * and W2t_pool = Rt_pool.
 */
int preft_loreft_prepare(void *D, void *Rt, const void *W, const void *R,
                         int32_t d, int32_t rank, int dtype, void *stream);

int preft_loreft_apply(void *h, int64_t ldh, int32_t T, int32_t d,
                       const int32_t *seg_start, const int32_t *seg_adapter,
                       const int32_t *seg_prefill_len, int32_t S,
                       const void *const *D_pool, const void *const *Rt_pool,
                       const void *const *b_pool, int32_t N,
                       int32_t rank, float scale, int dtype, int mode,
                       void *workspace, size_t workspace_bytes, void *stream);

/*
 * Adapter slot manager (paper Sec. 4, paged setting: 512 adapters of which 32 are on the GPU;
 * App. E.2: the active set in GPU memory, the catalogue in host memory; App. D.4: weights at
 * stable addresses are refreshed in place so the next launch or graph replay sees them).
 *
 * A manager owns: a pinned host store with one record per adapter (n_parts <= PREFT_MAX_PARTS
 * matrices of part_bytes[p] bytes each, e.g. {A, B} for LoRA or {W1, W2t, b} for DiReFT), a device slab
 * of n_slots records at addresses that never change, and per part a device table of n_slots
 * pointers (preft_slots_pool) to pass as A_pool / B_pool / ... with N = n_slots.  The apply
 * calls then take SLOT ids in seg_adapter: before a batch, preft_slots_acquire maps the
 * batch's adapter ids to slot ids, bringing missing adapters in (least recently used slot
 * first, never a slot the same call names) with asynchronous host-to-device copies on
 * `stream`.  Work that uses the slots must run on the same stream, or be ordered after it
 * by the caller.  These calls are host-side bookkeeping and copies: no kernel.
 *
 * preft_slots_create    allocates the three areas (the only allocating call of the library;
 *                       n_slots is clamped to n_adapters).  n_parts == 0 makes a manager
 *                       without memory that only does the residency bookkeeping.
 * preft_slots_store     copies part `part` of adapter `adapter` from host memory `src`
 *                       (part_bytes[part] bytes) into the store; if the adapter is resident
 *                       its slot is refreshed in place on `stream`.  The call first waits for
 *                       the latest copy that reads this adapter's record (queued by an
 *                       acquire or an earlier store, on whatever stream, whether or not the
 *                       adapter is still resident), so no copy ever reads a half-written
 *                       record.
 * preft_slots_acquire   adapter_ids[n] (host) -> slot_ids[n] (host); ids outside
 *                       [0, n_adapters) map to -1 ("no adapter").  PREFT_ECAPACITY if the call
 *                       names more distinct adapters than there are slots (the manager stays
 *                       consistent; slot_ids past the failing entry are -1).
 * preft_slots_pool      device array of n_slots device pointers for part `part`, or NULL.
 * preft_slots_resident  slot of an adapter, or -1.
 * preft_slots_stats     stats[5] (host) = {hits, misses, evictions, bytes copied, n_slots};
 *                       a hit or miss is counted once per distinct adapter and acquire call.
 * preft_slots_destroy   frees everything; the caller makes sure no work still uses the slots.
 * Not thread-safe: one thread drives a manager.
 */
typedef struct preft_slots preft_slots_t;

int preft_slots_create(preft_slots_t **out, int32_t n_adapters, int32_t n_slots, int32_t n_parts,
                       const size_t *part_bytes);
int preft_slots_destroy(preft_slots_t *m);
int preft_slots_store(preft_slots_t *m, int32_t adapter, int32_t part, const void *src, void *stream);
int preft_slots_acquire(preft_slots_t *m, const int32_t *adapter_ids, int32_t n, int32_t *slot_ids,
                        void *stream);
const void *const *preft_slots_pool(preft_slots_t *m, int32_t part);
int32_t preft_slots_resident(const preft_slots_t *m, int32_t adapter);
int preft_slots_stats(const preft_slots_t *m, int64_t *stats);

/*
 * Copies the schedule counters of a workspace to the host: counts[0] = multi-row work
 * units (chunks of up to 128 rows of one segment), counts[1] = rows of short segments (at most
 * 4 active rows, e.g. decode tokens), which run as gathered tiles, counts[2] = active rows.
 * `counts` is a host pointer to 3 int32.  Returns PREFT_ESCHEDULE (with the counts filled in) if,
 * since the schedule was written, an apply call with PREFT_SCHEDULE_READY named another T, S, N
 * or position set than the schedule's and therefore did nothing.  This call synchronises
 * `stream`; it is meant for tests, statistics and debugging, never for the serving loop.
 */
int preft_schedule_counts(const void *workspace, int32_t *counts, void *stream);

/* Static, NUL-terminated description of a return code (host pointer, never freed). */
const char *preft_strerror(int code);

/* Library version: major * 10000 + minor * 100 + patch. */
int preft_version(void);

#ifdef __cplusplus
}
#endif
#endif /* PREFT_H */
