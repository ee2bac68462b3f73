/* dmm.h -- C ABI of the universal one-sided matmul hot path on one MI355X.
 *
 * The library computes C = A B for three distributed matrices with arbitrary,
 * possibly misaligned partitionings and replication factors ("Slicing Is All
 * You Need", arXiv 2510.08874).  Every virtual rank's tiles live as separate
 * HBM buffers on the one GPU; a one-sided "get" of a remote tile is a direct
 * strided read of that buffer.  The path is
 *
 *   dmm_plan      host, integer only: Stationary-C op generation by slicing
 *                 (Algorithm 1 + the replication rule of Section 4.1), then a
 *                 grouping of the ops by output sub-tile so that every C region
 *                 is accumulated by one workgroup in ascending k, no atomics;
 *   dmm_execute   device: one grouped-GEMM launch over all ranks' ops (the
 *                 "local matrix multiplication" step of Section 4.2), then the
 *                 replica sum when C is replicated;
 *   dmm_reduce_replicas   device: reduce_replicas of Table 1 on its own.
 *
 * Conventions
 *   - All matrices and tiles are row-major.  Index intervals are half-open.
 *   - Host pointers: descriptors, cut arrays, pointer tables, ld tables.
 *     Device pointers: the tile buffers named *inside* the pointer tables.
 *   - Tile tables are indexed  rep * (grid_rows * grid_cols) + ti * grid_cols + tj.
 *   - Every function returns DMM_OK (0) or a negative dmm_status; nothing throws
 *     across the boundary; on failure output arguments are left untouched.
 *   - A plan may be used by one thread at a time.
 */
#ifndef DMM_H
#define DMM_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  DMM_OK = 0,
  DMM_EINVAL = -1, /* null argument, bad cuts (not spanning [0, dim], decreasing), empty grid, bad dtype/flag */
  DMM_ESHAPE = -2, /* shapes do not form C[m,n] = A[m,k] B[k,n] */
  DMM_EREPL = -3,  /* replication factor does not divide nranks (Section 2.1: p/c must be an integer),
                      or the process grid needs more ranks than one replica has */
  DMM_ENOMEM = -4, /* host or device allocation failed */
  DMM_EHIP = -5,   /* a HIP call failed; dmm_last_hip_error() holds its code */
  DMM_ELD = -6,    /* a leading dimension is smaller than the tile's width, or a row pitch (leading
                      dimension times element size) of an A, B or C tile is 2^24 bytes or more */
  DMM_ELIMIT = -7  /* dmm_reduce_replicas_static: the work tables of this call do not fit the library's
                      static device buffer (DMM_STATIC_SCRATCH_BYTES) */
} dmm_status;

/* Element type of the A and B tiles.  All partial sums are fp32, and so are the C tiles unless
 * dmm_execute is given DMM_C_BF16. */
typedef enum { DMM_BF16 = 1, DMM_F32 = 2 } dmm_dtype;

/* dmm_plan flags (bits 0 .. 7): the data movement strategy of Section 4, i.e. which matrix stays
 * in place and so decides which rank performs an op.  0 = Stationary C (Algorithm 1). */
#define DMM_STATIONARY_B 0x1u /* Algorithm 2 */
#define DMM_STATIONARY_A 0x2u /* its mirror image (Section 4.1: "analogous") */
/* Iteration offset of Section 4.2: each rank's ops of stationary tile (i, j) start i + j
 * positions later in their cyclic order.  It changes the order of the raw task list only
 * (what a rank would fetch when); the grouped order and the results do not depend on it. */
#define DMM_ITERATION_OFFSET 0x4u
/* Keep the merged work list (see dmm_plan_merged_items) whenever the plan can have one, also
 * where it saves no macro-tiles. */
#define DMM_MERGE_ALWAYS 0x8u

/* dmm_execute flags (bits 8 .. 15; the two sets share no bit, so a flag handed to the wrong call
 * is rejected with DMM_EINVAL) */
#define DMM_NO_REDUCE 0x100u /* leave every C replica holding its partial sum */
#define DMM_TIMING 0x200u    /* record events around the GEMM launch and around the replica-sum launch
                                on the given stream; read them with dmm_plan_elapsed_ms */
#define DMM_C_BF16 0x400u    /* the C tiles are bf16 buffers (c_ld in bf16 elements): every element receives
                                its fp32 sum rounded to nearest even, once.  Only for a C with one replica
                                (DMM_EINVAL otherwise): the partial sums of a replicated C stay fp32, since one
                                rounding to bf16 already costs a relative error of up to 2^-8 per element */
#define DMM_NO_MERGE 0x800u  /* run the macro-tiles of dmm_plan_items even where the plan has merged ones */
#define DMM_SEPARATE_REDUCE 0x1000u /* replicated C: sum the replicas in a kernel of its own behind the GEMM
                                (the one dmm_reduce_replicas runs).  Without the flag the sum is fused into the
                                GEMM wherever that is possible: the macro-tiles of replicas 1, 2, ... run
                                first, those of replica 0 behind them (in the same launch where each finds
                                its partial sums written by its own workgroup, else in a second launch), and
                                each of these adds the other replicas' partial sums of its region to its own,
                                ((own + C_1) + C_2) ..., before it stores.  Same final contents of every
                                replica, bit for bit, either way: the sum in replica 0, their partial sums in
                                the others.  The separate kernel also runs, flag or not, where the fused form
                                does not apply: merged macro-tiles, macro-tiles cut along K */

/* Distributed matrix descriptor (Section 3): shape, partition object, replication
 * factor.  The partition is a tile grid given by cut points (a uniform tile
 * shape is cuts[i] = min(i * t, dim); uneven cuts are allowed, and so are empty
 * tiles) plus a process grid onto which tiles are dealt block-cyclically, row-
 * major (Section 2.1, ScaLAPACK convention):
 *     owner(ti, tj, rep) = rep * (nranks / replication)
 *                        + (ti % proc_rows) * proc_cols + (tj % proc_cols).
 * The `replication` copies are laid out over consecutive blocks of
 * nranks / replication ranks; rank r belongs to replica r / (nranks/replication).
 * Caller-owned; dmm_plan copies what it needs. */
typedef struct {
  int64_t rows, cols;           /* global shape */
  int32_t grid_rows, grid_cols; /* tile grid: grid_shape() of Table 1 */
  const int64_t *row_cuts;      /* host, grid_rows + 1 entries, [0] = 0, [last] = rows, non-decreasing */
  const int64_t *col_cuts;      /* host, grid_cols + 1 entries */
  int32_t proc_rows, proc_cols; /* process grid inside one replica */
  int32_t replication;          /* c >= 1, must divide nranks */
} dmm_matrix_desc;

/* One local multiply = one op of Algorithm 1: the three tiles and the global box
 * [m0,m1) x [k0,k1) x [n0,n1) whose A slice (rows m, cols k), B slice (rows k,
 * cols n) and C slice (rows m, cols n) are multiplied.  Offsets inside a tile
 * are the global bound minus the tile's lower bound (footnote of Section 4.1). */
typedef struct {
  int32_t rank;             /* virtual rank that owns the stationary tile (of C, B or A) */
  int32_t a_rep, a_ti, a_tj;
  int32_t b_rep, b_ti, b_tj;
  int32_t c_rep, c_ti, c_tj;
  int64_t m0, m1, k0, k1, n0, n1;
} dmm_task;

/* One unit of GPU work: a macro-tile of one group's output sub-tile, i.e. the
 * C region rows [m0, m0 + m_ext) x cols [n0, n0 + n_ext) (global indices) of
 * replica c_rep, which one workgroup accumulates over the group's K-segments in
 * ascending k and writes once.  group = -1 marks a zero-fill item: a C region
 * no op of the plan updates in that replica (a replica with an empty share of the
 * inner dimension; with Stationary B or A, regions other replicas' ranks compute),
 * which therefore holds a partial sum of zero. */
typedef struct {
  int64_t group;            /* index into group_offsets, or -1 */
  int64_t m0, n0;           /* global top-left corner */
  int32_t m_ext, n_ext;     /* extent, each at most the macro-tile edge */
  int32_t c_rep, c_ti, c_tj;/* C tile written */
  int32_t reserved;
} dmm_work_item;

/* A merged macro-tile: the C region rows [m0, m0 + m_ext) x cols [n0, n0 + n_ext) of replica
 * c_rep, cut from the replica as a whole, so that it may cover several output sub-tiles, i.e.
 * meet several tiles of A, B and C.  Its rows fall into row_pieces intervals of the merged row
 * cuts of A and C, its columns into col_pieces intervals of the merged column cuts of B and C;
 * inside the macro-tile a column piece starts at a multiple of 8 columns.  One workgroup
 * accumulates it over the K-segments of the replica's share of k in ascending k, exactly as the
 * macro-tiles of dmm_plan_items do for their group, so both lists give bitwise the same C (except
 * where dmm_execute cuts the last round of one list along K and not of the other: see there). */
typedef struct {
  int64_t m0, n0;
  int32_t m_ext, n_ext;
  int32_t c_rep;
  int32_t row_pieces, col_pieces;
  int32_t reserved;
} dmm_merged_item;

/* A plan may be used by one thread at a time (different plans: any threads).  The device
 * entry points act on the calling thread's current HIP device; a plan stays with the device
 * of its first dmm_execute / dmm_reduce_replicas / dmm_broadcast_replica. */
typedef struct dmm_plan_s dmm_plan_t;

/* Slicing planner (Algorithm 1, or Algorithm 2 / its mirror image when `flags` asks for
 * Stationary B / A; replication rule of Section 4.1; grouping by output sub-tile).
 * A c-fold replicated stationary matrix splits between its replicas the one dimension it
 * does not index, in contiguous ranges [floor(r L / c), floor((r+1) L / c)): K for C
 * (Section 4.1), M for B, N for A.  An op's product goes to the C tile in the performing
 * rank's local replica of C; dmm_execute gives every C replica its partial sum and then
 * adds the replicas up.  Host only: makes no HIP call.  `nranks` is p, the number of
 * virtual ranks.  `flags`: 0, DMM_STATIONARY_B or DMM_STATIONARY_A, each optionally with
 * DMM_ITERATION_OFFSET and DMM_MERGE_ALWAYS (anything else, or both stationary flags:
 * DMM_EINVAL).  On success *out owns the plan.
 * A plan that holds a merged work list (dmm_plan_merged_items) keeps the slicing in factored
 * form, as the three merged cut lists whose cells the ops are, and runs from that; its op list,
 * grouped order and per-group macro-tiles are written out on first use (by the accessors below, or
 * by dmm_execute when it is to run the per-group macro-tiles), not by dmm_plan.  If memory runs
 * out then, the accessors return 0 / NULL and dmm_execute DMM_ENOMEM. */
int dmm_plan(const dmm_matrix_desc *A, const dmm_matrix_desc *B, const dmm_matrix_desc *C,
             int32_t nranks, uint32_t flags, dmm_plan_t **out);

/* Accessors.  Returned pointers are borrowed from the plan and live until
 * dmm_plan_destroy.  A null plan gives 0 / NULL. */
int64_t dmm_plan_num_tasks(const dmm_plan_t *p);
const dmm_task *dmm_plan_tasks(const dmm_plan_t *p);        /* Algorithm-1 order: rank ascending, then loop order */
const int64_t *dmm_plan_order(const dmm_plan_t *p);         /* stable sort of task indices by (c_rep, c_ti, c_tj, m0, n0, k0) */
int64_t dmm_plan_num_groups(const dmm_plan_t *p);
const int64_t *dmm_plan_group_offsets(const dmm_plan_t *p); /* num_groups + 1 offsets into order */
int64_t dmm_plan_num_items(const dmm_plan_t *p);
const dmm_work_item *dmm_plan_items(const dmm_plan_t *p);   /* launch order (workgroup id -> item) */
int32_t dmm_plan_macro_tile(const dmm_plan_t *p);           /* edge of the square macro-tile, elements */
/* The alternative work list of merged macro-tiles, in launch order; 0 / NULL when the plan has
 * none.  A plan has one when (a) it is a Stationary C plan in which all ranks of a C replica read
 * the same replica of A and of B (the replication factor of C is a multiple of those of A and
 * B), or a Stationary B / A plan without any replication, so that the ops of a replica are the
 * cells of one grid, (b) no replica has an empty share
 * of k, and (c) merging saves at least a tenth of the macro-tiles (tile grids much finer than the
 * macro-tile: block-cyclic layouts), or the op list is long against the work list (at least 4096
 * ops and 16 per macro-tile), so that running from the factored form saves the host the time to
 * write the list out.  dmm_execute then runs this list instead of dmm_plan_items. */
int64_t dmm_plan_num_merged_items(const dmm_plan_t *p);
const dmm_merged_item *dmm_plan_merged_items(const dmm_plan_t *p);

/* Run the plan: C = A B (overwrite; C need not be initialised).
 *   dtype                 element type of every A and B tile
 *   a_tiles, b_tiles      host arrays of device pointers, one per (replica, tile) in table order
 *   c_tiles               host array of device pointers to fp32 tiles (bf16 tiles with DMM_C_BF16)
 *   a_ld, b_ld, c_ld      host arrays, leading dimension in elements, >= the tile's width
 *   flags                 0 or any of DMM_NO_REDUCE, DMM_TIMING, DMM_C_BF16, DMM_NO_MERGE, DMM_SEPARATE_REDUCE
 *   hip_stream            hipStream_t, may be null (default stream)
 * Pointers of empty tiles may be null.  Tile buffers are caller-owned and must
 * stay valid until the stream work completes.  Asynchronous: returns after
 * enqueueing.  Every element of every C replica is written exactly once with
 * that replica's partial sum; then, unless DMM_NO_REDUCE, replica 0 receives
 * the sum over replicas (other replicas keep their partials).  When the number
 * of macro-tiles leaves most of the device idle in the last round of workgroups,
 * those macro-tiles are cut along K into runs whose partial sums go through a
 * scratch buffer and are added in ascending k (fixed cut, fixed order: results
 * stay bitwise reproducible on a given device).  The first call on a plan takes
 * the plan's device work table (and, if needed, that scratch buffer) from a
 * process-wide pool, allocating only when the pool has none that fits; later
 * calls with the same arguments allocate nothing and do not synchronise. */
int dmm_execute(dmm_plan_t *p, int dtype,
                const void *const *a_tiles, const int64_t *a_ld,
                const void *const *b_tiles, const int64_t *b_ld,
                void *const *c_tiles, const int64_t *c_ld,
                uint32_t flags, void *hip_stream);

/* reduce_replicas(origin) of Table 1: for every C tile, the origin replica's
 * buffer receives C_0 + C_1 + ... (fp32, ascending replica index); the other
 * replicas are left unchanged.  A no-op when C has one replica. */
int dmm_reduce_replicas(dmm_plan_t *p, void *const *c_tiles, const int64_t *c_ld,
                        int32_t origin_replica, void *hip_stream);

/* broadcast_replica (Table 1): the tiles of every other replica of C become copies of the
 * tiles of replica `origin_replica` (after dmm_execute that replica holds the product, so
 * reduce + broadcast leaves the product in every replica).  Arguments, ownership and error
 * behaviour as for dmm_reduce_replicas; asynchronous on `hip_stream`; a no-op when C is not
 * replicated.  HBM-bound: c * 4 bytes per element of C. */
int dmm_broadcast_replica(dmm_plan_t *p, void *const *c_tiles, const int64_t *c_ld, int32_t origin_replica,
                          void *hip_stream);

/* reduce_replicas for callers that cannot allocate: code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc.  Same arguments, result (bit for bit) and error
 * behaviour as dmm_reduce_replicas, but the call allocates nothing, on the device or on the host:
 * the kernel's work tables (one record per C tile and per block of rows, the replicas' tile
 * pointers and leading dimensions) are assembled in a fixed host buffer inside the library and
 * copied on `hip_stream` into a static device buffer of DMM_STATIC_SCRATCH_BYTES, of which every
 * GPU the library runs on holds one copy for the life of the process.  A call whose tables need
 * more (about 48 bytes per C tile plus 16 per replica of it, and 16 bytes per 4096 elements of C)
 * fails with DMM_ELIMIT and launches nothing.  All calls on one GPU share that buffer: calls on
 * one stream follow each other safely (stream order), calls that overlap on different streams
 * of one GPU race and must be ordered by the caller.  The plan's device state is not touched, so
 * dmm_plan_destroy does not wait for work enqueued here (that work reads nothing the plan owns). */
#define DMM_STATIC_SCRATCH_BYTES (1u << 20)
int dmm_reduce_replicas_static(dmm_plan_t *p, void *const *c_tiles, const int64_t *c_ld,
                               int32_t origin_replica, void *hip_stream);

/* ---- measurement and test aids (not steps of the method) ---------------------------------- */

/* What the last dmm_execute on a plan did.
 *   ran_merged    1: it ran the merged macro-tiles (the plan has such a list, DMM_NO_MERGE was not
 *                 given and the device grants a workgroup the 160 KB of LDS their kernel asks for)
 *   ran_k_split   1: it cut macro-tiles along K (partial tiles through a scratch buffer, added up
 *                 in ascending k by a second kernel: the last round of workgroups would have left
 *                 most of the device idle, or a merged macro-tile had more K-segments than its
 *                 workgroup can hold descriptors for).  Such a run sums in another order than an
 *                 uncut one
 *   ran_fused     how it summed the replicas of C: 0 = not in the GEMM (one replica,
 *                 DMM_NO_REDUCE, DMM_SEPARATE_REDUCE, or the fused form did not apply), 1 = in the
 *                 GEMM, one launch, 2 = in the GEMM, replica 0's macro-tiles in a second launch
 *                 (see DMM_SEPARATE_REDUCE)
 *   table_reused  1: it found the work tables of the call before it in place and launched from
 *                 them (same element type, same flags apart from DMM_TIMING, same device, same
 *                 contents of all six pointer and leading-dimension tables); 0: it assembled and
 *                 uploaded them.  The tables hold addresses, not data: what the tiles contain
 *                 plays no part
 * All zero for a plan that has not been executed, and for a null plan.  DMM_EINVAL if out is null. */
typedef struct {
  int32_t ran_merged, ran_k_split, ran_fused, table_reused;
} dmm_execute_report;
int dmm_plan_last_execute(const dmm_plan_t *p, dmm_execute_report *out);

/* Device time of the kernels of the last dmm_execute(..., DMM_TIMING, ...) on this plan, in
 * milliseconds, excluding the work-table upload: gemm_ms from in front of the first GEMM launch
 * to behind the last (one launch, two with a fused replica sum that needs two, plus the pass
 * that adds up macro-tiles cut along K), reduce_ms the replica-sum kernel.  Blocks until those
 * kernels have finished.  A kernel that was not timed (or did not run) reports -1.  Either
 * output pointer may be null.  (Measurement aid for the roofline figures: Section 5.2
 * reports the best of repeated runs.) */
int dmm_plan_elapsed_ms(dmm_plan_t *p, float *gemm_ms, float *reduce_ms);

/* The two GEMM launches of a fused replica sum that needed two, one by one, for the last
 * dmm_execute that ran with DMM_TIMING: ms[0] and flops[0] are the duration of the launch over the
 * macro-tiles of replicas 1, 2, ... and the 2 m n k of the ops behind it, ms[1] and flops[1] those
 * of the launch over replica 0's macro-tiles, which also adds the other replicas' partial sums.
 * Blocks until that call's launches have finished.  ms = -1 and flops = 0 where there was nothing
 * to report (no timing, no fused sum, a fused sum in one launch).  Errors: DMM_EINVAL (null
 * argument), DMM_EHIP. */
int dmm_plan_gemm_launch_ms(dmm_plan_t *p, float ms[2], double flops[2]);

/* Measurement aid, independent of any plan: the rate the matrix pipes of the current device
 * sustain right now with nothing else going on.  Every SIMD of every CU issues independent
 * v_mfma_f32_32x32x16_bf16 back to back from registers (no LDS, no memory) for about
 * `milliseconds` of device time; operands are pseudo-random bf16 values in (-1, 1) when
 * `random_operands` is non-zero, constants otherwise.  The part lowers its clock under matrix
 * load by an amount that depends on the operand data, so this, not the published peak, is what
 * a kernel on this device can approach at that moment.  Outputs (either may be null): achieved
 * TFLOP/s and the average shader clock in MHz.  Synchronous; launches on the null stream.
 * Errors: DMM_EINVAL (milliseconds <= 0 or > 1000), DMM_EHIP. */
int dmm_measure_mfma_rate(float milliseconds, int random_operands, float *tflops, float *shader_mhz);

/* Frees host and device memory of the plan (waits for the plan's own enqueued
 * work first; device buffers return to a process-wide pool).  Null is allowed. */
void dmm_plan_destroy(dmm_plan_t *p);

const char *dmm_strerror(int status);
int dmm_last_hip_error(void); /* hipError_t of the last failed HIP call on this thread, 0 if none */
int dmm_version(void);         /* 4: the replica sum is fused into the GEMM unless DMM_SEPARATE_REDUCE asks
                                  for the kernel of its own; dmm_plan_last_execute replaces the
                                  dmm_plan_ran_* accessors (3: flag values of dmm_plan and dmm_execute disjoint,
                                  dmm_reduce_replicas_static) */

#ifdef __cplusplus
}
#endif
#endif /* DMM_H */
