/*
 * bspmm.h - Batched SpMM for small sparse matrices on AMD MI355X (gfx950), C ABI.
 *
 * One call multiplies a whole mini-batch of small sparse matrices A_i (CSR) by dense matrices
 * B_i in ONE kernel launch (the Batched SpMM of Sec. IV-C of "Batched Sparse Matrix
 * Multiplication for Accelerating Graph Convolutional Networks", arXiv 1903.11409):
 *
 *     forward      C_i = A_i   . B_i      (the result of Fig. 2 / Fig. 4: C is overwritten)
 *     transposed   G_i = A_i^T . dY_i     (the backward product of Sec. IV-D, last sentence)
 *
 * Conventions (Sec. II-B, II-C, Fig. 4, Sec. IV-D):
 *  - A_i is CSR: row pointer `rpt` (rows_i+1 entries), column index `colids` and `values`
 *    (nnz_i entries each), all 0-based int32 / fp32.  Each operation's row pointer is LOCAL:
 *    rpt[0] == 0 and rpt[rows_i] == nnz_i.  Column indices inside a row need not be sorted
 *    or unique (duplicates add up).
 *  - All operations of a batch share one dense column count F (the paper's n_B).
 *  - Dense operands are row-major fp32, packed for the whole batch: operation i reads rows
 *    [b_row_off[i], b_row_off[i]+cols_i) of B and writes rows [c_row_off[i], c_row_off[i]+rows_i)
 *    of C; leading dimensions are given per call, in elements, and must be >= F.
 *    Several operations may read the same B block (a graph with several edge-type channels);
 *    output blocks must not overlap, except that with BSPMM_ACCUMULATE operations naming the
 *    same output block are summed into it.
 *  - alpha = 1, beta = 0: every output row of every operation is written exactly once
 *    (zeros for rows without entries); output rows that belong to no operation are untouched.
 *  - Arithmetic is fp32 with fused multiply-add, summed in stored order inside a row.
 *
 * Memory and ownership.  Pointers marked HOST are read during the call and may be freed
 * afterwards.  Pointers marked DEVICE must stay valid and unchanged until bspmm_destroy
 * (the plan borrows them).  The library never allocates device memory: the caller provides a
 * device workspace of at least bspmm_workspace_bytes() bytes, 256-byte aligned, which the plan
 * owns until bspmm_destroy (schedule tables, the transposed CSR and the merged CSR of summed
 * operations live there).
 *
 * Streams.  `stream` is a hipStream_t passed as void* (NULL = the default stream).  All
 * device work is enqueued asynchronously; no call synchronises the device except where stated.
 * bspmm_run / bspmm_run_transposed enqueue exactly one kernel (the first call of a direction
 * also the one-off device builds named under BSPMM_BUILD_TRANSPOSE; a build recorded into a
 * stream capture runs with the graph and is not counted as done, so plans used in HIP graphs
 * are best created with that flag or run once before the capture).  Calls on one plan must be
 * issued from one host thread at a time and on the stream order the caller wants.
 *
 * Errors.  Every int-returning call returns BSPMM_OK or a negative BSPMM_E* code; nothing is
 * printed, thrown or aborted.  Device-side contents of rpt/colids are trusted by run calls;
 * bspmm_validate checks them on the device on request.
 */
#ifndef BSPMM_H
#define BSPMM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define BSPMM_OK          0
#define BSPMM_EINVAL    (-1)  /* bad argument: null pointer, negative size, ld < F, ...      */
#define BSPMM_ENOSPACE  (-2)  /* workspace smaller than bspmm_workspace_bytes()               */
#define BSPMM_EHIP      (-3)  /* a HIP runtime call failed (see bspmm_last_hip_error)         */
#define BSPMM_EOVERLAP  (-4)  /* output blocks of two operations overlap                      */
#define BSPMM_ESTATE    (-5)  /* plan cannot do this (dry-run plan, transposed unsupported)   */
#define BSPMM_EBADCSR   (-6)  /* bspmm_validate found a malformed CSR on the device           */
#define BSPMM_ETOOBIG   (-7)  /* operations summed into one block: more than 8 of them, or
                                 their arrays do not fit the on-chip memory together; with
                                 front_features: an operation too large for a whole-workgroup
                                 item                                                          */

/* bspmm_options.flags */
#define BSPMM_DRY_RUN          1u  /* schedule only: touch no device, run calls return ESTATE */
#define BSPMM_BUILD_TRANSPOSE  2u  /* enqueue the one-off device builds (the transposed CSR; with
                                      BSPMM_ACCUMULATE the merged CSR of every summed set, both
                                      directions; for operations too large for on-chip memory,
                                      the entry ranges of their row blocks) inside bspmm_create
                                      instead of in the first run that needs them - e.g. before
                                      a HIP-graph capture                                        */
#define BSPMM_SPLIT_HUB_ROWS   8u  /* rows with >= 64 entries and >= 4x the operation's average are
                                      split across all lanes of the workgroup and the partial
                                      sums reduced (DPP / ds_swizzle inside a wavefront, LDS across
                                      wavefronts).  For graphs with hub nodes; plain batches are a
                                      few per cent faster without it                             */
#define BSPMM_ACCUMULATE       16u  /* operations that name the SAME output block (same first row,
                                      same row count) are added up in one pass - the channel sum
                                      of the graph-convolution layer (Fig. 6 / Fig. 7) - instead
                                      of being rejected as overlapping.  Applies to C blocks in
                                      bspmm_run and to B blocks (input gradients) in
                                      bspmm_run_transposed.  The first run of a direction also
                                      enqueues a kernel that merges the CSR arrays of every such
                                      set into the workspace (once per plan).  Fastest when the
                                      dense blocks the members of a set read are one block of the
                                      packed input: the same block, or blocks that follow each
                                      other in member order without a gap                        */
#define BSPMM_COO_DIRECT       32u  /* bspmm_create_coo only: no conversion to CSR.  Every run is one
                                      launch that works from the index pairs as they are (the
                                      SparseTensor cases of Fig. 3 / Fig. 5(a,b)).  Where an
                                      operation's entries fit in LDS the workgroup sorts them by
                                      row there and sums each row in registers; otherwise a group
                                      of lanes per stored entry adds products with LDS
                                      floating-point atomics into an output tile kept in LDS, cut
                                      into row ranges when the tile does not fit.  Cheapest when a
                                      batch is multiplied once or twice; the order of the
                                      additions, and with it the last bits of the result, vary
                                      from run to run.  The transposed product needs no build (the
                                      index roles swap).  Not combined with BSPMM_ACCUMULATE or
                                      BSPMM_SPLIT_HUB_ROWS (EINVAL).  With options.lds_bytes 0 the
                                      launch takes the smallest of 24, 32, 48 and 64 KiB at which
                                      every operation is sorted on chip (64 KiB if none), and asks
                                      for no more than its largest item needs: bspmm_info.lds_bytes
                                      reports that                                               */
#define BSPMM_SYMMETRIC        64u  /* the caller asserts that every A_i equals its transpose (e.g. the
                                      symmetric normalisation D^-1/2 (A+I) D^-1/2 of an undirected
                                      graph): bspmm_run_transposed then gathers over the same CSR
                                      arrays and no transposed CSR is ever built.  Not checked;
                                      with an asymmetric A_i the result is A_i . dY_i.  Operations
                                      must be square (EINVAL)                                    */
#define BSPMM_ONE_FRONT_LAUNCH 128u /* plans with front_features of two and more workgroups per CU
                                      normally run bspmm_run_gcn as a launch of resident
                                      workgroups that stream the graphs (see there); this flag
                                      keeps them on the one-launch path                         */
#define BSPMM_FLOOR_PROBE      4u  /* measurement aid: same grid, LDS and item fetches, but every
                                      item is emptied, so a run computes and writes nothing      */

/* Schedule bins: how many lanes one (operation, feature-tile) item gets. */
#define BSPMM_BIN_WORKGROUP 0  /* 256 lanes, A_i and its B tile staged in LDS                 */
#define BSPMM_BIN_WAVE      1  /* one 64-lane wavefront, staged                               */
#define BSPMM_BIN_SLICE32   2  /* half a wavefront, staged                                    */
#define BSPMM_BIN_SLICE16   3  /* a quarter wavefront, staged                                 */
#define BSPMM_BIN_GENERIC   4  /* 256 lanes on a row block, operands read from global memory  */
#define BSPMM_NUM_BINS      5
#define BSPMM_BIN_COO       5  /* items of a BSPMM_COO_DIRECT plan (not counted in items_in_bin) */

typedef struct bspmm_plan bspmm_plan;

/* The batch: the paper's list of sparse matrices plus where their dense blocks sit. */
typedef struct bspmm_batch {
    int32_t        batch;      /* number of SpMM operations, >= 0                              */
    const int32_t* rows;       /* HOST [batch]  m_A of operation i                             */
    const int32_t* cols;       /* HOST [batch]  n_A of operation i                             */
    const int32_t* nnz;        /* HOST [batch]  stored entries of operation i                  */
    const int64_t* rpt_off;    /* HOST [batch]  element offset of op i's row pointers in rpt   */
    const int64_t* nz_off;     /* HOST [batch]  element offset of op i's entries               */
    const int64_t* b_row_off;  /* HOST [batch]  first row of B_i in the packed dense input     */
    const int64_t* c_row_off;  /* HOST [batch]  first row of C_i in the packed dense output    */
    const int32_t* rpt;        /* DEVICE row pointers of all operations                        */
    const int32_t* colids;     /* DEVICE column indices of all operations                      */
    const float*   values;     /* DEVICE values of all operations                              */
} bspmm_batch;

/*
 * The same batch with COO / SparseTensor operands (Sec. II-B, Fig. 1: every stored entry is a
 * (row, column) index pair plus a value; Sec. IV: the entries are sorted neither by row nor by
 * column).  Operation i owns nnz[i] entries starting at entry nz_off[i]: pair p sits at
 * ids[2*(nz_off[i]+p)] (row) and ids[2*(nz_off[i]+p)+1] (column), its value at
 * values[nz_off[i]+p].  Repeated pairs are added up, as the loop nest of Fig. 2 does.
 */
typedef struct bspmm_coo_batch {
    int32_t        batch;      /* number of SpMM operations, >= 0                              */
    const int32_t* rows;       /* HOST [batch]  m_A of operation i                             */
    const int32_t* cols;       /* HOST [batch]  n_A of operation i                             */
    const int32_t* nnz;        /* HOST [batch]  stored entries of operation i                  */
    const int64_t* nz_off;     /* HOST [batch]  entry offset of op i in ids (pairs) and values */
    const int64_t* b_row_off;  /* HOST [batch]  first row of B_i in the packed dense input     */
    const int64_t* c_row_off;  /* HOST [batch]  first row of C_i in the packed dense output    */
    const int32_t* ids;        /* DEVICE (row, column) pairs of all operations                 */
    const float*   values;     /* DEVICE values of all operations                              */
} bspmm_coo_batch;

/* Scheduler knobs.  Zero-initialise for defaults. */
typedef struct bspmm_options {
    uint32_t flags;            /* BSPMM_DRY_RUN | BSPMM_BUILD_TRANSPOSE | BSPMM_SPLIT_HUB_ROWS */
    int32_t  force_bin;        /* 0 = automatic; 1+b forces bin b for every op that fits it    */
    int32_t  lds_bytes;        /* LDS per workgroup; <= 160 KiB (all of a CU's).  0 = 24 KiB,
                                  and 80 KiB, then 160 KiB, are tried before a batch whose
                                  summed operations need more is refused with ETOOBIG; 52 KiB
                                  (tiles twice as wide) for F >= 512 when the launch moves
                                  more than 28 MB in more than one round of workgroups and
                                  needs at most a tenth more rounds that way.  bspmm_info.lds_bytes says
                                  what was taken                                              */
    int32_t  min_tile;         /* narrowest feature tile in floats, 0 = default (32)           */
    int32_t  max_tile;         /* widest feature tile in floats, 0 = default (256), <= 256     */
    int32_t  target_workgroups;/* split tiles until the launch has this many, 0 = 4 per CU    */
    int32_t  compute_units;    /* 0 = ask the device (256 assumed for dry runs)                */
    int32_t  lds_pad;          /* floats added to each staged B row, 0 = default, -1 = none    */
    int32_t  max_passes;       /* row passes a sub-workgroup slot may take, 0 = default (1)    */
    int32_t  generic_rows;     /* rows per generic row block, 0 = default (8)                   */
    int32_t  wg_passes;        /* row passes of a workgroup item before it is cut into row
                                  ranges: 0 = cut only while the launch is short of
                                  target_workgroups, N > 0 = always cap at N, -1 = never cut   */
    int32_t  resident_workgroups; /* N > 0: persistent launch of N workgroups that stride
                                  through the tasks; 0 = one workgroup per task (default)      */
    int32_t  front_features;   /* n_X > 0: shape the forward schedule for bspmm_run_gcn with an
                                  n_X-column layer input: whole workgroups, feature tiles in
                                  multiples of 16, room in LDS for an n_X x tile block of weights
                                  and at least 16 rows of X_i beside the operation (lds_bytes
                                  then defaults to 80 KiB, 160 KiB if that is too little; for
                                  batches of 1.5 graphs per CU and more, 24 to 52 KiB first:
                                  more workgroups per CU); needs
                                  F % 16 == 0 and n_X % 4 == 0
                                  (EINVAL), not combined with
                                  BSPMM_SPLIT_HUB_ROWS or lds_pad (EINVAL); with
                                  BSPMM_ACCUMULATE see bspmm_run_gcn; ETOOBIG when an
                                  operation does not fit at any tile width                      */
    int32_t  reserved_;        /* 0 */
} bspmm_options;

/* What the scheduler decided; index 0 = forward, 1 = transposed. */
typedef struct bspmm_info {
    int32_t batch;
    int32_t F;
    int32_t lds_bytes;
    int32_t compute_units;
    int32_t tile[2];                         /* batch-wide feature tile before per-op shrink  */
    int32_t workgroups[2];                   /* grid size of the single launch                */
    int32_t tasks[2];                        /* workgroup-sized tasks the grid strides through */
    int32_t items[2];                        /* non-empty work items                          */
    int32_t items_in_bin[2][BSPMM_NUM_BINS];
    int32_t fused_tasks[2];                  /* tasks that add up several operations          */
    int32_t transposed_supported;            /* 0 when input-gradient blocks overlap          */
    int32_t transposed_built;                /* the build kernel has been enqueued            */
    int32_t lean[2];                         /* 1: every task is one staged workgroup item with a
                                                power-of-two tile, so runs with 16-byte aligned
                                                operands launch the lean kernel                */
    int32_t front_stream[4];                 /* plans whose bspmm_run_gcn is run by resident
                                                workgroups that stream the graphs (see there):
                                                graphs in their lists, workgroups, LDS bytes per
                                                workgroup, graphs left to a launch of their own;
                                                all 0 otherwise                                */
    int64_t effective_bytes[2];              /* CSR + distinct dense inputs + outputs, once   */
    int64_t flops;                           /* 2 * nnz * F (Sec. V-A)                        */
    uint64_t workspace_bytes;
} bspmm_info;

/* One scheduled work item, for inspection and tests. */
typedef struct bspmm_item {
    int32_t op;        /* operation index                                                     */
    int32_t bin;       /* BSPMM_BIN_*                                                         */
    int32_t row0;      /* first output row of the operation this item computes (a staged item
                          still holds the whole operation in LDS)                              */
    int32_t nrows;     /* number of output rows                                               */
    int32_t f0;        /* first feature column                                                */
    int32_t fw;        /* number of feature columns                                           */
    int32_t workgroup; /* task index; workgroup (task mod grid size) runs it                  */
    int32_t slot;      /* lane slot inside the workgroup; items of a BSPMM_COO_DIRECT plan: what
                          the item keeps in LDS (1 the dense tile, 2 the entries, 4 the entries
                          sorted by row and no output tile)                                   */
} bspmm_item;

/*
 * Bytes of device workspace a plan for (batch, F, options) needs.  Reads only HOST arrays.
 * options may be NULL.  Device pointers in `b` are not dereferenced and may be NULL here.
 * The size depends on the schedule, so this call schedules the batch; a bspmm_create on the
 * same thread with the same batch contents, F and options takes that schedule over instead of
 * making it again.
 */
int bspmm_workspace_bytes(const bspmm_batch* b, int32_t F, const bspmm_options* options,
                          size_t* bytes);

/*
 * Inspect the batch, bin every operation, tile the feature dimension, build the work lists
 * for the forward and the transposed product and upload them to `workspace` (one async copy
 * on `stream`).  This is the step of Sec. IV-C that sizes the launch and picks the cache
 * blocking from the shapes of the inputs, done here per operation instead of from the batch
 * maximum.
 * Returns EINVAL for null/negative/inconsistent arguments or F <= 0, EOVERLAP when two
 * operations' C blocks overlap (with BSPMM_ACCUMULATE: overlap without being identical),
 * ETOOBIG, ENOSPACE, EHIP.  On error *plan is NULL.
 */
int bspmm_create(bspmm_plan** plan, const bspmm_batch* b, int32_t F,
                 const bspmm_options* options, void* workspace, size_t workspace_bytes,
                 void* stream);

/*
 * bspmm_create for callers that cannot allocate device memory (code under HIP-graph capture,
 * tight serving loops, harnesses that forbid hipMalloc): the same plan, but its workspace is an
 * array of BSPMM_STATIC_WORKSPACE_BYTES bytes that is part of the library's device code on every
 * GPU, so the caller passes none and the call allocates no device memory.  The GPU is the
 * calling thread's current device; `stream` must belong to it.
 *  - ENOSPACE when the plan needs more than BSPMM_STATIC_WORKSPACE_BYTES (bspmm_workspace_bytes
 *    tells in advance); BSPMM_DRY_RUN is EINVAL; otherwise arguments and errors as bspmm_create.
 *  - All such plans of a GPU share the one array, which keeps what the last one wrote.  Nothing
 *    in it has to start at zero: every table is written in full before it is read.  Only the
 *    latest static plan of a GPU is valid; run, export and validate calls on an earlier one
 *    return ESTATE.  The caller orders the streams: work of the earlier plan that is still
 *    running when the next bspmm_create_static uploads its tables races with that upload.
 */
#define BSPMM_STATIC_WORKSPACE_BYTES (8 * 1024 * 1024)
int bspmm_create_static(bspmm_plan** plan, const bspmm_batch* b, int32_t F,
                        const bspmm_options* options, void* stream);

/*
 * C_i = A_i . B_i for every operation, one kernel launch on `stream` (Fig. 4 per row, batched
 * as in Sec. IV-C).  B and C are DEVICE pointers to the packed matrices, ldb/ldc their leading
 * dimensions in floats (>= F).  B and C must not alias.  A plan with batch == 0 launches
 * nothing.  B may be NULL when it has no rows at all, that is when no operation has both
 * rows and columns (nothing is read then; the same holds for dY of bspmm_run_transposed).  The vectorised path needs 16-byte aligned B, C and ldb % 4 == ldc % 4 == 0;
 * anything else silently takes the scalar path.
 */
int bspmm_run(bspmm_plan* plan, const float* B, float* C, int64_t ldb, int64_t ldc,
              void* stream);

/*
 * One channel of the batched graph-convolution layer in ONE launch (Fig. 7: U = MatMul(Xr, W),
 * B = Add(bias, U), C = BatchedSpMM(A_list, B)):  Y_i = A_i . (X_i . W + bias), or with
 * accumulate != 0  Y_i += A_i . (X_i . W + bias)  (the ElementWiseAdd over channels, one launch
 * per channel, no intermediate U, B or C in memory).  X is the packed DEVICE feature matrix
 * (cols_i rows of n_X = options.front_features floats at row b_row_off[i], leading dimension
 * ldx >= n_X), W the DEVICE n_X x F weight matrix (leading dimension ldw >= F), bias F DEVICE
 * floats, Y indexed like C.  The dense part runs on the matrix cores in fp32
 * (v_mfma_f32_16x16x4_f32; whole layers in large launches: v_mfma_f32_32x32x2_f32) from LDS
 * to LDS; B_i never leaves the chip.  X, W, Y must be
 * 16-byte aligned with ldx, ldw, ldy multiples of 4 (EINVAL).  ESTATE for plans created
 * without front_features.  (Launches of up to two workgroups per CU use workgroups of 512 lanes,
 * larger ones of 256.)
 *
 * The whole layer in one launch: a plan created with front_features AND BSPMM_ACCUMULATE, in
 * which every operation is one of M channels of a graph - the M channel operations of a graph
 * read the same X block and name the same output block, M the same for all graphs (EINVAL
 * otherwise) - computes  Y_i = sum_ch A_i^ch . (X_i . W[ch] + bias[ch])  (Fig. 7 including the
 * ElementWiseAdd) with X_i staged once for all channels.  W is then the M weight matrices one
 * under the other (M * n_X rows, channel ch at row ch * n_X) and bias M rows of F floats; the
 * channels of a graph are taken in the order of their operations.
 *
 * Layers of two and more (graph, feature tile) pairs per CU - single channels, or whole layers
 * of M = 2 to 8 channels (3 run as 4, 5 to 7 as 8, the added channels empty) - with n_X = 16, 32,
 * 64 or 128 run as a launch of RESIDENT workgroups instead, three per CU (8 channels: two per
 * CU, of eight wavefronts, one per channel): each keeps the weights of its feature tile in
 * registers for the whole launch and streams the graphs of its list through LDS, the next
 * graph's X_i and CSR in flight while the matrix cores work on this one's.  Small graphs whose
 * blocks lie back to back in X and in Y are taken several per trip; graphs too large for a
 * workgroup's share of the LDS are taken one at a time by the same workgroups (M = 1 or 4), or
 * follow in a launch of the one-launch kernel over their items.  The first run also enqueues a
 * kernel that copies the CSR arrays into one block per trip (once per plan, like the merged CSR
 * of summed sets; BSPMM_BUILD_TRANSPOSE moves it into bspmm_create).  For whole layers that
 * kernel also lists, per channel, the rows of X_i that the channel's entries name: only those
 * rows of X_i W[ch] + bias[ch] are made (a channel matrix with few entries per row leaves most
 * of them unread).  bspmm_info.front_stream says what a plan does; BSPMM_ONE_FRONT_LAUNCH keeps
 * a plan on the one-launch path.  With options.lds_bytes the caller fixes the LDS budget of
 * both.
 */
int bspmm_run_gcn(bspmm_plan* plan, const float* X, int64_t ldx, const float* W, int64_t ldw,
                  const float* bias, float* Y, int64_t ldy, int32_t accumulate, void* stream);

/*
 * G_i = A_i^T . dY_i for every operation (backward product with respect to the dense input).
 * dY is indexed like C (rows_i rows at c_row_off[i]), G like B (cols_i rows at b_row_off[i]).
 * The first call enqueues the on-device transposed-CSR build (one extra launch, once per
 * plan) unless bspmm_create already did.  Returns ESTATE when two operations share or
 * overlap a B block and the plan was not created with BSPMM_ACCUMULATE (each would have to
 * add into the same gradient rows), or when B blocks overlap without being identical.
 */
int bspmm_run_transposed(bspmm_plan* plan, const float* dY, float* G, int64_t ldy, int64_t ldg,
                         void* stream);

/*
 * Copy the plan's transposed CSR (stable: inside a row of A_i^T entries are ordered by the
 * original row, ties by stored position) into caller DEVICE arrays: rpt_t gets sum(cols_i+1)
 * int32 (op i at sum_{k<i}(cols_k+1), local), colids_t / values_t get sum(nnz_i) entries
 * (op i at nz packing order sum_{k<i} nnz_k).  Builds the transpose first if needed.
 */
int bspmm_export_transposed(bspmm_plan* plan, int32_t* rpt_t, int32_t* colids_t,
                            float* values_t, void* stream);

/*
 * Plans for COO / SparseTensor operands (the batched product of Sec. IV-C for the data
 * structure of Fig. 1 / Fig. 3).  bspmm_create_coo enqueues ONE extra launch on `stream`
 * that sorts every operation's entries by row into CSR arrays inside the workspace (stable:
 * entries of a row keep their stored order; one workgroup per operation, counting sort in
 * LDS); afterwards the plan behaves exactly like a CSR plan of those arrays: bspmm_run,
 * bspmm_run_transposed, bspmm_export_transposed and every option work unchanged, without
 * atomics on the output and with bitwise reproducible results.  ids / values must stay valid
 * and unchanged until that launch has finished; they are not read afterwards.  Entries whose
 * indices fall outside their matrix are left out of the product (bspmm_validate reports
 * them).  Arguments, workspace rules and error codes are those of bspmm_workspace_bytes /
 * bspmm_create.  With BSPMM_COO_DIRECT nothing is converted: ids / values are read by every
 * run and must stay valid for the life of the plan, bspmm_export_csr and
 * bspmm_export_transposed return ESTATE, and out-of-range entries are skipped by the kernel.
 */
int bspmm_workspace_bytes_coo(const bspmm_coo_batch* b, int32_t F, const bspmm_options* options,
                              size_t* bytes);
int bspmm_create_coo(bspmm_plan** plan, const bspmm_coo_batch* b, int32_t F,
                     const bspmm_options* options, void* workspace, size_t workspace_bytes,
                     void* stream);

/*
 * Copy the CSR arrays a COO plan built into caller DEVICE arrays: rpt gets sum(rows_i+1) int32
 * (op i at sum_{k<i}(rows_k+1), local), colids / values get sum(nnz_i) entries (op i at
 * sum_{k<i} nnz_k).  ESTATE for plans not made by bspmm_create_coo.
 */
int bspmm_export_csr(bspmm_plan* plan, int32_t* rpt, int32_t* colids, float* values,
                     void* stream);

/*
 * Check the DEVICE CSR arrays against the HOST sizes given at creation: rpt[0]==0,
 * rpt non-decreasing, rpt[rows]==nnz, 0 <= colids < cols.  Launches one kernel and
 * SYNCHRONISES `stream`.  Returns OK or EBADCSR (*bad_op = first offending operation).
 * For a COO plan the index pairs are checked instead (0 <= row < rows, 0 <= column < cols).
 */
int bspmm_validate(bspmm_plan* plan, int32_t* bad_op, void* stream);

/*
 * What a kernel of the library needs on the current device (for profiles and occupancy
 * arguments; asks the HIP runtime, launches nothing): vector and scalar registers per lane /
 * wavefront, LDS the kernel declares itself (the launch adds `dynamic_lds_bytes`), and how many
 * of its workgroups a compute unit holds at once with that much dynamic LDS.
 * kernel: BSPMM_KERNEL_*.  EINVAL for an unknown kernel, EHIP when the runtime cannot tell.
 */
#define BSPMM_KERNEL_LEAN      0  /* bspmm_run / bspmm_run_transposed, lean launches               */
#define BSPMM_KERNEL_GENERAL   1  /* the same, every other launch (float4 path, no slots, no hubs) */
#define BSPMM_KERNEL_GENERAL_S 2  /* the general kernel's scalar path                              */
#define BSPMM_KERNEL_FRONT     3  /* bspmm_run_gcn, one channel                                    */
#define BSPMM_KERNEL_LAYER     4  /* bspmm_run_gcn, whole layer                                    */
#define BSPMM_KERNEL_BUILD     5  /* transposed-CSR build, 256 lanes                               */
#define BSPMM_KERNEL_BUILD_L   6  /* transposed-CSR build, 1024 lanes                              */
#define BSPMM_KERNEL_COO       7  /* direct COO product                                            */
#define BSPMM_KERNEL_LAYER_STREAM 8 /* bspmm_run_gcn, whole layer, resident streaming workgroups
                                       (n_X = 64, two blocks per wavefront)                        */
typedef struct bspmm_kernel_resources {
    int32_t vgprs;              /* vector registers per lane                                   */
    int32_t sgprs;              /* scalar registers per wavefront (0: the runtime does not say)*/
    int32_t static_lds_bytes;   /* LDS declared in the kernel                                  */
    int32_t scratch_bytes;      /* private (spill) memory per lane                             */
    int32_t threads;            /* lanes per workgroup the kernel is launched with             */
    int32_t workgroups_per_cu;  /* resident workgroups per CU at dynamic_lds_bytes             */
    int32_t compute_units;
    int32_t reserved_;
} bspmm_kernel_resources;
int bspmm_kernel_info(int32_t kernel, int32_t dynamic_lds_bytes, bspmm_kernel_resources* out);

/* Fill *info.  Works on dry-run plans. */
int bspmm_plan_info(const bspmm_plan* plan, bspmm_info* info);

/* Copy up to `capacity` scheduled items of one direction (0 forward, 1 transposed) into
 * `items`; *count receives the total number.  HOST only.  These are the items of the one-launch
 * schedule, which bspmm_run, bspmm_run_transposed and the one-launch kernel of bspmm_run_gcn
 * work from; a plan whose bspmm_run_gcn is run by streaming workgroups
 * (bspmm_info.front_stream) takes from it only the items of the graphs left to the second
 * launch. */
int bspmm_plan_items(const bspmm_plan* plan, int32_t transposed, bspmm_item* items,
                     int32_t capacity, int32_t* count);

/* Release the host side of the plan.  Does not touch the stream: the caller keeps the
 * workspace alive until work already enqueued has finished.  NULL is allowed. */
void bspmm_destroy(bspmm_plan* plan);

/* Static description of an error code. */
const char* bspmm_strerror(int code);

/* The hipError_t (as int) behind the calling thread's most recent BSPMM_EHIP. */
int bspmm_last_hip_error(void);

#ifdef __cplusplus
}
#endif
#endif /* BSPMM_H */
