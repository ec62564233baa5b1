/*
 * lutq — fused lookup-table dequantise + small-batch matmul for AMD MI355X (gfx950).
 *
 * C ABI of liblutq.so.  Plain pointers and sizes only; every buffer is owned by
 * the caller.  The library never allocates device memory, never synchronises the
 * device and never aborts: arguments are validated on the host and a status code
 * is returned BEFORE anything is launched, so on error no output is touched.
 *
 * Problem (Section 3 of "Fast Matrix Multiplications for Lookup Table-Quantized
 * LLMs", arXiv 2407.10960): an index matrix Q with entries in {0..2^b-1}, a table
 * T = [v_0 .. v_{2^b-1}] of 16-bit floats, dequantised weights W^ = T[Q], and the
 * product Y = X * W^ with a small number of activation rows.  With the group
 * scales of Section 4.1 ("LUT quantization method") / Section 4.2 the weight is
 *
 *        W^[n, k] = round16( T[Q[n, k]] * S[n, k / group_size] )
 *        Y[m, n]  = sum_k X[m, k] * W^[n, k]          (fp32 accumulation)
 *
 * Orientation: the paper writes Q and W as k-by-n; this library stores their
 * transposes, [N, K] row-major (one row per output channel, as a linear layer
 * does).  A group is `group_size` consecutive elements along K inside one row.
 * round16 is one round-to-nearest-even to the 16-bit type `dtype`.
 *
 * Supported domain: bits in {2,3,4}; group_size in {32,64,128,256}; 1 <= M <= 128
 * (a launch works on up to 32 activation rows, at 4 bits on up
 * to 64; more are served in slices of that many rows, one launch each on the caller's stream, so the
 * weights are streamed once per slice; a 33..64-row launch is preceded by a small launch that copies
 * the slice's activations into the workspace in the order the matrix instruction reads them);
 * N a multiple of 16; K a multiple of the K-tile of the bit width (128 for
 * 4-bit, 256 for 2- and 3-bit) and of group_size; device pointers 16-byte aligned.
 *
 * Environment (read once per process, diagnostics only): LUTQ_VERBOSE=1 prints the launch shape
 * of every call and the tuner's finalists to stderr (2: also the tuner's first-pass times);
 * LUTQ_NO_SHARED_X=1 / LUTQ_NO_XM8=1 switch off two activation-load variants for comparisons.
 * They change at most the order of the fp32 summation.
 */
#ifndef LUTQ_H
#define LUTQ_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    LUTQ_OK = 0,
    LUTQ_ERR_NULL = 1,         /* a required pointer is NULL */
    LUTQ_ERR_BITS = 2,         /* bits not in {2,3,4} */
    LUTQ_ERR_GROUP = 3,        /* group_size not in {32,64,128,256} or does not divide K */
    LUTQ_ERR_SHAPE = 4,        /* M, N or K outside the supported domain */
    LUTQ_ERR_ALIGN = 5,        /* a device pointer is not 16-byte aligned */
    LUTQ_ERR_INDEX_RANGE = 6,  /* lutq_pack: an index is >= 2^bits */
    LUTQ_ERR_WORKSPACE = 7,    /* workspace missing or smaller than lutq_workspace_bytes() */
    LUTQ_ERR_DTYPE = 8,        /* dtype not LUTQ_F16 / LUTQ_BF16 */
    LUTQ_ERR_DEVICE = 9,       /* a HIP runtime call failed (launch, device query) */
    LUTQ_ERR_PLAN = 10,        /* lutq_plan fields outside their documented ranges */
    LUTQ_ERR_SCRATCH = 11      /* lutq_matmul_static: the launch needs more than the built-in scratch */
} lutq_status;

typedef enum { LUTQ_F16 = 0, LUTQ_BF16 = 1 } lutq_dtype;

/* Human-readable name of a status code (static storage, never NULL). */
const char* lutq_status_string(lutq_status s);

/* ---------------------------------------------------------------------------
 * Offline restructuring (Section 3.1 "Offline Matrix Restructuring"; first line of
 * Algorithm 1, reorder_and_split).  Host code, run once per weight matrix.
 *
 * The packed form orders indices so that a wavefront's 128-bit loads deliver them
 * already in the operand order of the gfx950 16x16x32 matrix instruction, and
 * splits 3-bit indices into a 2-bit slice and a 1-bit slice so that every load is
 * a power-of-two number of bits.  It does not depend on group_size (the argument is
 * validated and otherwise unused).
 *
 * Packed layout (normative; this library's own -- the paper's is tied to NVIDIA Ampere fragments).
 * Q is [N, K] row-major.  N is cut into row blocks of 16 rows, K into tiles of TK columns (TK = 128
 * for 4-bit, 256 for 2- and 3-bit).  Row blocks are grouped into super-blocks of SB consecutive row
 * blocks: with nb = N / 16, SB = 4 if nb is a multiple of 4, else 2 if nb is even, else 1 -- except
 * SB = 2 for multiples of 4 in 257..512 (a choice tuned for 256 compute units and frozen into the
 * format: it holds on every device; lutq_pack_layout reports SB for a given N, so that it can be
 * recorded next to a packed blob).  Storage order is super-block, then K tile, then row block inside
 * the super-block: tile (rb, kt) starts at byte
 *        (((rb / SB) * (K / TK) + kt) * SB + rb % SB) * TILE_BYTES,
 * so the SB tiles that cover 16*SB rows x TK columns are adjacent.  A tile is what one 64-lane
 * wavefront loads with one 128-bit load per lane (plus one 64-bit load for the 3-bit high slice).
 * v_mfma_f32_16x16x32_{f16,bf16} takes, from lane l = 16*o + i (i = 0..15, o = 0..3), the eight
 * A-matrix elements of row i and columns 8*o .. 8*o+7 of a 16 x 32 block; a tile holds TK/32 such
 * blocks ("steps" t).  Lane l owns, for step t, the indices Q[16*rb + i][TK*kt + 32*t + 8*o + j],
 * j = 0..7, and its bytes sit at offset 16*l of the tile:
 *   4-bit  TILE_BYTES = 1024.  Four little-endian 32-bit words d = 0..3; word d is step d; nibble j
 *          (bits 4j..4j+3) is index j, so byte p of a word is the pair (2p, 2p+1).
 *   2-bit  TILE_BYTES = 1024.  Words d = 0..3; 2-bit field e (bits 2e..2e+1), e = 0..15, of word d is
 *          index j = e % 8 of step t = 2d + e / 8, so byte p holds four consecutive indices.
 *   3-bit  TILE_BYTES = 1536 = 1024 (low slice: index bits 0..1) + 512 (high slice: bit 2).
 *          Low slice, lane l at 16*l, words d = 0..3, byte p = 0..3 of word d:
 *              bits 0..1 low2(index 2p, step 2d)      bits 2..3 low2(index 2p+1, step 2d)
 *              bits 4..5 low2(index 2p, step 2d+1)    bits 6..7 low2(index 2p+1, step 2d+1)
 *          High slice, lane l at 1024 + 8*l, words h = 0..1, byte p of word h, u = 0..3:
 *              bit 2u = bit2(index 2p, step 4h+u)     bit 2u+1 = bit2(index 2p+1, step 4h+u)
 *          so that, for one step, (low word >> 0 or 4) supplies bits 0..3 of each byte and (high word
 *          shifted by 4 - 2u) supplies bits 4..5: four 6-bit pair-table addresses.
 * ------------------------------------------------------------------------- */

/* Geometry of the packed form of an [N, K] matrix at `bits` bits. */
typedef struct {
    int tile_k;                       /* K columns per tile: 128 (4-bit) or 256 */
    int tile_bytes;                   /* 1024, or 1536 at 3 bits */
    int row_blocks_per_super_block;   /* SB: 4, 2 or 1 */
    int64_t row_blocks;               /* N / 16 */
    int64_t k_tiles;                  /* K / tile_k */
} lutq_layout;

/* Fills *out for (N, K, bits).  Errors: NULL, BITS, GROUP, SHAPE. */
lutq_status lutq_pack_layout(int64_t N, int64_t K, int bits, int group_size, lutq_layout* out);

/* Size in bytes of the packed form (N*K*bits/8); 0 if the arguments are unsupported. */
size_t lutq_packed_bytes(int64_t N, int64_t K, int bits, int group_size);

/* indices: host, [N, K] row-major, one index per byte, each < 2^bits.
 * packed_out: host, caller-owned, lutq_packed_bytes() bytes, fully overwritten.
 * Errors: NULL, BITS, GROUP, SHAPE, INDEX_RANGE (packed_out contents then unspecified). */
lutq_status lutq_pack(const uint8_t* indices, int64_t N, int64_t K, int bits, int group_size,
                      void* packed_out);

/* Inverse of lutq_pack (host to host). indices_out: [N, K] row-major, one index per byte. */
lutq_status lutq_unpack(const void* packed, int64_t N, int64_t K, int bits, int group_size,
                        uint8_t* indices_out);

/* ---------------------------------------------------------------------------
 * The fused kernel (Algorithm 1 / Algorithm 2: copy table to on-chip memory, stream
 * packed weights, combine bit-slices, vectorised table lookup + group scale, matrix
 * instruction, Stream-K style partial-sum fix-up through global scratch).
 * ------------------------------------------------------------------------- */

/* Bytes of device scratch lutq_matmul may need for any M with these arguments
 * (the semaphore and partial-sum areas of Algorithm 2).  0 if unsupported. */
size_t lutq_workspace_bytes(int64_t N, int64_t K, int bits, int group_size);

/* Work-decomposition knobs (Section 3.3 Stream-K partitioning; Section 4.1: the kernel instance is
 * chosen per shape).  All fields 0 = let the library choose.  The number of table duplicates, a
 * tuning knob in the paper, is fixed here: one copy per lane (64 copies of a 4-byte entry, 32 of an
 * 8-byte entry), which is conflict-free by construction and makes the entry stride 256 bytes. */
typedef struct {
    int row_blocks_per_wave;  /* R: 16-row blocks each wavefront streams together: 0,1,2,4; must divide N/16 */
    int grid;                 /* number of workgroups: 0 or 1..4096 (grid x row groups per workgroup <= 4096) */
    int waves_per_workgroup;  /* wavefronts that share one table: 0 or 4..16, a multiple of the next-but-one field */
    int tiles_in_flight;      /* K tiles each wavefront keeps in flight (software pipeline depth): 0, 2 or 4 */
    int row_groups_per_workgroup; /* teams: row groups (of R blocks) a workgroup works on side by side, each
                                     by waves_per_workgroup / this many wavefronts that split K: 0 or 1..16;
                                     must divide N / (16 R) */
    int scheduling;           /* how a workgroup's work is dealt to its wavefronts: 0 = library chooses,
                                 LUTQ_SCHED_TEAMS (1) = the static teams described above,
                                 LUTQ_SCHED_QUEUE (2) = a work queue (M <= 4 and K / group_size a multiple of 8
                                 only): a workgroup owns whole row groups over the whole of K, cut into items of
                                 tiles_per_item K tiles that its wavefronts take one after the other from a
                                 counter.  The N / (16 R) row groups are dealt to `grid` workgroups as evenly
                                 as whole row groups allow: row_groups_per_workgroup (1..64) = the whole part of
                                 row groups / grid, the first workgroups one more.  Give grid (then
                                 row_groups_per_workgroup is 0 or that quotient) or row_groups_per_workgroup
                                 (a divisor of the row groups); R is 1 or 2, waves_per_workgroup 4..16 with
                                 no relation to the row groups, tiles_in_flight 2 */
                              /* LUTQ_SCHED_ROWS (3) = activation-stationary (M >= 5): `grid` workgroups own
                                 whole 16-row blocks over the whole of K, dealt as evenly as whole row blocks
                                 allow (row_groups_per_workgroup = the whole part of N / 16 / grid, 0 or that
                                 value; at most 64); the wavefronts (waves_per_workgroup 4..16, as many as the
                                 instance's registers allow) split K, hold a K tile's activations in registers
                                 and stream the weights of row_blocks_per_wave (4 or 8) row blocks past them
                                 side by side, in as many passes as the workgroup's row blocks need;
                                 tiles_in_flight 2.  For M > 32 this scheduling asks for slices of 64 rows
                                 (4 bits; LUTQ_ERR_PLAN where no such
                                 instance exists); that launch has one decomposition (4 row blocks side by
                                 side, one workgroup per compute unit, 8 waves at most), so every other
                                 field is 0 or the value lutq_plan_default reports; any other plan, and
                                 the default where 64-row slices are not faster, means slices of 32 rows.
                                 With tiles_per_item > 0 (launches of up to 32 rows; more rows go in slices
                                 of 32) K is cut into slices of that many K tiles
                                 across workgroups: `grid` (required, a multiple of the number of slices) =
                                 shares x slices, a share being at most row_blocks_per_wave row blocks (one
                                 pass: row_groups_per_workgroup = the whole part of N / 16 / shares), so a
                                 workgroup reads only its slice of the activations; every workgroup leaves
                                 its slice's sums in the scratch and the last of a share to finish adds them
                                 in slice order (shares <= 1024; shares x slices x row_blocks_per_wave x
                                 ceil(M / 16) KiB of scratch) */
    int tiles_per_item;       /* LUTQ_SCHED_QUEUE: K tiles (128 columns at 4 bits, 256 at 2 and 3) per item:
                                 0, or a multiple of tiles_in_flight that divides the K tiles of a row.
                                 LUTQ_SCHED_ROWS: 0 = K is not cut across workgroups, else the K tiles per
                                 slice: the K tiles of a row divided by it, rounded up, is the number of
                                 slices (at least two), which are as even as whole tiles allow */
} lutq_plan;

#define LUTQ_SCHED_TEAMS 1
#define LUTQ_SCHED_QUEUE 2
#define LUTQ_SCHED_ROWS 3

/* Fills *plan with the library's choice for this problem on the current device. */
lutq_status lutq_plan_default(int bits, int group_size, int64_t M, int64_t N, int64_t K,
                              lutq_dtype dtype, lutq_plan* plan);

/* The same choice for a device with `compute_units` compute units (1..4096), without touching any
 * device: host logic only, for planning ahead and for tests.  MI355X has 256. */
lutq_status lutq_plan_default_for(int bits, int group_size, int64_t M, int64_t N, int64_t K,
                                  lutq_dtype dtype, int compute_units, lutq_plan* plan);

/* Whether lutq_matmul_plan would accept `plan` (NULL = the default plan) for this problem on a device
 * with `compute_units` compute units: LUTQ_OK, or the status lutq_matmul_plan would return for the
 * plan and the problem (BITS, GROUP, SHAPE, DTYPE, PLAN).  Host logic only; no device is touched. */
lutq_status lutq_plan_check(int bits, int group_size, int64_t M, int64_t N, int64_t K, lutq_dtype dtype,
                            int compute_units, const lutq_plan* plan);

/* Plans chosen by measurement (lutq_tune; Section 4.1 picks the kernel configuration per shape offline and
 * dispatches on it): a process-wide table that lutq_matmul and lutq_matmul_static consult, when no plan
 * is passed, before their own choice.  An entry applies to calls with its bits, group_size, dtype, N,
 * K and m_min <= M <= m_max (for M > 32 the M of each slice of up to 32 rows counts; slices of 33..64
 * rows have a single decomposition and do not consult the table); the first match wins; an
 * entry whose plan the kernels cannot run for a call is skipped (the library's own choice is used). */
typedef struct {
    int bits, group_size;
    lutq_dtype dtype;
    int64_t m_min, m_max, N, K;
    lutq_plan plan;
} lutq_plan_entry;

/* Replaces the table by a copy of entries[0 .. count-1] (count = 0 clears it).  Host memory only; safe to
 * call from any thread, but calls already in flight may still use the old table.  Errors: NULL, SHAPE
 * (count < 0 or > 4096). */
lutq_status lutq_plan_table_set(const lutq_plan_entry* entries, int count);

/* The plan the table holds for this call: LUTQ_OK and *plan, or LUTQ_ERR_PLAN if no entry matches. */
lutq_status lutq_plan_table_lookup(int bits, int group_size, int64_t M, int64_t N, int64_t K, lutq_dtype dtype,
                                   lutq_plan* plan);

/* Y = X * W^T-dequantised, asynchronous on `stream`.
 *   X       device, [M, K] row-major, dtype
 *   packed  device, bytes produced by lutq_pack for (N, K, bits)
 *   scales  device, [N, K / group_size] row-major, dtype
 *   lut     device, 2^bits entries, dtype (any finite values, any order)
 *   Y       device, [M, N] row-major, dtype; fully overwritten
 *   workspace  device, >= lutq_workspace_bytes(); must be zero-filled once before its
 *              first use.  Its first 64 KiB hold the arrival counters, which every successful
 *              call returns to zero; the rest holds partial sums that the next call simply
 *              overwrites.  The same workspace can therefore be reused by any later call on
 *              the same stream without clearing it.  Calls that may run concurrently
 *              (different streams) need separate workspaces.
 *   stream  a hipStream_t (NULL = the default stream)
 * Errors: NULL, BITS, GROUP, SHAPE, ALIGN, WORKSPACE, DTYPE, DEVICE; Y untouched on error. */
lutq_status lutq_matmul(const void* X, const void* packed, const void* scales, const void* lut,
                        int bits, int group_size, int64_t M, int64_t N, int64_t K,
                        lutq_dtype dtype, void* Y,
                        void* workspace, size_t workspace_bytes, void* stream);

/* Same, with an explicit work decomposition (additionally returns LUTQ_ERR_PLAN).
 * The result does not depend on the plan beyond fp32 summation order. */
lutq_status lutq_matmul_plan(const void* X, const void* packed, const void* scales, const void* lut,
                             int bits, int group_size, int64_t M, int64_t N, int64_t K,
                             lutq_dtype dtype, void* Y,
                             void* workspace, size_t workspace_bytes, void* stream,
                             const lutq_plan* plan);

/* lutq_matmul_plan for callers that cannot allocate device memory or hand over a workspace: code under
 * HIP graph capture, tight serving loops, harnesses that forbid allocation.  The arrival counters and
 * partial sums live in a device array of the library's own, LUTQ_STATIC_SCRATCH_BYTES large (64 KiB of
 * counters + 16 MiB of partial-sum slots), which every GPU the library runs on holds from the first use
 * of the library on it until the process ends.  The call allocates nothing and calls no allocating
 * routine; the first call on a device looks the array's address up once (make that call outside a
 * graph capture).  Every other argument and the result are those of lutq_matmul_plan (plan may be NULL
 * for the default decomposition), bit for bit under the same plan.
 * A launch needs partial-sum slots only when its plan cuts output tiles across workgroups:
 * grid x row groups per workgroup x 2 slots of R x ceil(M/16) x 1 KiB (M capped at 32).  If that exceeds
 * the 16 MiB, a call with a plan returns LUTQ_ERR_SCRATCH before anything is launched (Y untouched), and a
 * call without one takes the library's choice among the decompositions that need little scratch (of the
 * LLaMA-3 8B/70B shapes only 70B gate+up in bf16 beyond sixteen rows does not fit with its first choice).
 * All calls on one GPU share the one array: calls that may overlap on a GPU (different streams) race
 * on it and must use lutq_matmul with separate workspaces instead.  The counters are returned to zero by
 * every launch; the slots keep the last call's partial sums and are overwritten before they are read. */
#define LUTQ_STATIC_SCRATCH_BYTES ((size_t)(64 * 1024 + 16 * 1024 * 1024))
lutq_status lutq_matmul_static(const void* X, const void* packed, const void* scales, const void* lut,
                               int bits, int group_size, int64_t M, int64_t N, int64_t K,
                               lutq_dtype dtype, void* Y, void* stream, const lutq_plan* plan);

/* Finer-grained tables: one table per output row (Section 2.3: lookup tables obtained at the
 * output-channel level; Section 5 names flexible tables as what the kernel is for).
 *        W^[n, k] = round16( T[n][Q[n, k]] * S[n, k / group_size] )
 *   luts    device, [N, 2^bits] row-major, dtype, 16-byte aligned
 *   every other argument as in lutq_matmul (scales of 1.0 give tables without group scales).
 * M <= 4 with K / group_size a multiple of 8: the work-queue kernel with the tables of all of a
 * workgroup's row blocks built once and resident (sixteen copies per row block: the four lanes that
 * work on a row share one).  5 <= M <= 32 with at least two row blocks per compute unit: the row-streaming
 * kernel with the tables of four row blocks at a time.  Otherwise a workgroup holds the tables of one 16-row block at a time and
 * rebuilds its on-chip copies for every row block it works on (one row block per workgroup, K split
 * over its waves and, for few row blocks, over workgroups).  The work decomposition is the library's
 * in both cases.  Errors: those of lutq_matmul. */
lutq_status lutq_matmul_channel(const void* X, const void* packed, const void* scales, const void* luts,
                                int bits, int group_size, int64_t M, int64_t N, int64_t K,
                                lutq_dtype dtype, void* Y,
                                void* workspace, size_t workspace_bytes, void* stream);

/* Vector codebooks (Section 5 names them, beside finer-grained tables, as what a flexible lookup kernel is
 * for): one 8-bit index selects a PAIR of adjacent weights from a codebook of 256 pairs, 4 bits per weight.
 *        W^[n, 2j + c] = round16( C[V[n, j]][c] * S[n, 2j / group_size] ),  c = 0, 1
 *   codebook  device, [256][2] values of dtype (1 KiB), 4-byte aligned
 *   packed    the 4-bit layout of lutq_pack applied to the indices Q[n, 2j] = V[n, j] & 15,
 *             Q[n, 2j + 1] = V[n, j] >> 4 (one byte of the 4-bit layout is one codebook index)
 *   every other argument as in lutq_matmul with bits = 4.
 * The kernels are those of lutq_matmul: their on-chip table at 4 bits already is a table of 256 pairs
 * (built from sixteen scalars there, copied from the codebook here), so the cost is the same.  A codebook
 * with C[e] = (T[e & 15], T[e >> 4]) gives lutq_matmul's result bit for bit.  The work decomposition is the
 * library's.  Errors: those of lutq_matmul; LUTQ_ERR_ALIGN also for a codebook that is not 4-byte aligned.
 *
 * lutq_matmul_quads is the same at 2 bits per weight: one 8-bit index selects FOUR adjacent weights,
 *        W^[n, 4j + c] = round16( C[V[n, j]][c] * S[n, 4j / group_size] ),  c = 0 .. 3
 *   codebook  device, [256][4] values of dtype (2 KiB), 4-byte aligned
 *   packed    the 2-bit layout of lutq_pack applied to Q[n, 4j + c] = (V[n, j] >> 2c) & 3
 * (the 2-bit kernels' on-chip table is a table of 256 quads); a codebook with C[e][c] = T[(e >> 2c) & 3]
 * gives lutq_matmul's 2-bit result bit for bit. */
lutq_status lutq_matmul_pairs(const void* X, const void* packed, const void* scales, const void* codebook,
                              int group_size, int64_t M, int64_t N, int64_t K,
                              lutq_dtype dtype, void* Y,
                              void* workspace, size_t workspace_bytes, void* stream);

lutq_status lutq_matmul_quads(const void* X, const void* packed, const void* scales, const void* codebook,
                              int group_size, int64_t M, int64_t N, int64_t K,
                              lutq_dtype dtype, void* Y,
                              void* workspace, size_t workspace_bytes, void* stream);

/* Instance selection by measurement (Section 4.1: the fastest kernel configuration is picked per
 * shape; Section 3.3: how the K range is cut across workgroups is part of that choice).  Times the
 * default plan and the candidate plans that lutq_tune_candidates lists, first with a few launches
 * each, then the eight fastest and the default in three rounds of `reps` launches (the minimum per
 * plan counts), with events on `stream`, and
 * writes the fastest to *best and, if best_us is not NULL, its microseconds per launch to *best_us.
 *   packed, scales  host arrays of `ring` >= 1 device pointers each: weight sets of the same shape
 *                   (copies of one matrix will do) that successive launches visit in turn, so that
 *                   with a ring larger than the caches every launch streams from HBM as it would
 *                   inside a model; ring = 1 tunes for weights that stay in cache.
 *   the other arguments are those of lutq_matmul.  Y is overwritten by every candidate.
 * Blocks until the measurements on `stream` are done (it creates and destroys two events, nothing
 * else); must not be called while `stream` is being captured.
 * Errors: those of lutq_matmul; SHAPE also for ring < 1 or reps < 1. */
lutq_status lutq_tune(const void* X, const void* const* packed, const void* const* scales, int ring,
                      const void* lut, int bits, int group_size, int64_t M, int64_t N, int64_t K,
                      lutq_dtype dtype, void* Y, void* workspace, size_t workspace_bytes, void* stream,
                      int reps, lutq_plan* best, float* best_us);

/* The plans lutq_tune tries for this problem on the current device, the default plan first.
 * Writes min(*count, capacity) of them to plans (host) and their number to *count; plans may be
 * NULL when capacity is 0.  Some of them have no kernel instance: lutq_matmul_plan answers those
 * with LUTQ_ERR_PLAN, and lutq_tune skips them. */
lutq_status lutq_tune_candidates(int bits, int group_size, int64_t M, int64_t N, int64_t K,
                                 lutq_dtype dtype, lutq_plan* plans, int capacity, int* count);

/* Quantiser on the GPU (Section 3, first equation: each weight is replaced by the index of the
 * nearest table entry; Section 4.1 "LUT quantization method" / Section 4.2: one absmax scale per
 * group, kept in the 16-bit type), fused with the restructuring of Section 3.1: a dense weight
 * matrix already in device memory becomes scales + packed indices in one pass, ready for lutq_matmul.
 *   scale S[n, g] = round16( max |W[n, k]| over the group )
 *   Q[n, k]       = the lowest c that minimises | W[n, k] / S[n, g] - T[c] |   (u = 0 where S = 0)
 * with the division, the difference and the comparison in IEEE fp64 on the exact input values, so
 * the result depends on the inputs only, not on the launch.
 *   W           device, [N, K] row-major; fp32 if w_is_f32 != 0, else `dtype`; 16-byte aligned; finite
 *   lut         device, 2^bits entries, dtype
 *   scales_out  device, [N, K / group_size] row-major, dtype, fully overwritten
 *   packed_out  device, lutq_packed_bytes() bytes, 16-byte aligned, fully overwritten (the bytes
 *               lutq_pack would produce from Q)
 * Asynchronous on `stream`; allocates nothing.  Errors: NULL, BITS, GROUP, SHAPE, DTYPE, ALIGN, DEVICE. */
lutq_status lutq_quantize(const void* W, int w_is_f32, const void* lut, int bits, int group_size,
                          int64_t N, int64_t K, lutq_dtype dtype, void* scales_out, void* packed_out,
                          void* stream);

/* The separate-kernel path of Section 3 (dequantise to memory): writes
 * W_out[n, k] = round16(T[Q[n,k]] * S[n, k/group_size]), device [N, K] row-major, dtype,
 * using the same on-chip lookup + scale routine as lutq_matmul.  Asynchronous on `stream`. */
lutq_status lutq_dequant(const void* packed, const void* scales, const void* lut,
                         int bits, int group_size, int64_t N, int64_t K, lutq_dtype dtype,
                         void* W_out, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* LUTQ_H */
