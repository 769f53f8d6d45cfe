/*
 * seer.h -- C ABI of the MI355X (gfx950) SpMV schedule family, the CSR feature
 * reduction and the decision-tree kernel selector of the Seer case study.
 *
 * Runtime flow (Sec. III-B, "Runtime Inference"): gather the dynamically computed
 * features of the matrix, walk a decision tree over them to obtain a kernel index,
 * run that SpMV kernel.  seer_features, seer_select and seer_spmv are those three steps;
 * seer_spmv_auto and seer_spmv_model run them without the host in between; and for
 * several products with one matrix (Sec. IV-E) seer_spmv_plan selects with the iteration
 * count, runs the chosen kernel's preprocessing once, and seer_spmv_prepared is each
 * product.
 *
 * General rules
 *   - Plain C types only.  Every pointer is marked DEVICE (memory the current HIP
 *     device can access, owned and freed by the caller) or HOST.
 *   - The library never allocates or frees device memory.  Scratch is a caller
 *     buffer handed in as (workspace, workspace_bytes); its contents on entry do
 *     not matter and are undefined on return.  Required sizes come from the
 *     *_workspace_bytes calls.  A workspace must be 16-byte aligned.  What a
 *     preprocessing pass produces lives in a second caller buffer (plan_mem), which
 *     the products then only read.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  All
 *     device work is enqueued on it.  seer_spmv, seer_spmv_auto, seer_spmv_model and
 *     seer_spmv_prepared return without waiting; seer_features, seer_spmv_prepare and
 *     seer_spmv_plan wait for their own result because they return host values.
 *   - Every call returns SEER_OK (0) or a negative seer_status; on error no output
 *     is written.  Nothing throws or aborts.  Matrix contents (monotone row_ptr,
 *     column range) are NOT validated: they are the caller's contract.
 *   - The first seer_features call allocates one 64-byte pinned host buffer per
 *     process (its result mailbox); no other state is kept, on the host or the device.
 *   - Calls that use the same workspace must not overlap in time; seer_features calls
 *     are serialised inside the library (they share the mailbox).
 */
#ifndef SEER_H
#define SEER_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    SEER_OK = 0,
    SEER_EINVAL = -1,     /* null pointer, negative size, misaligned buffer           */
    SEER_EKERNEL = -2,    /* kernel id outside [0, seer_num_kernels())                */
    SEER_ETREE = -3,      /* malformed tree: index out of range, cycle, bad feature   */
    SEER_EWORKSPACE = -4, /* workspace missing, misaligned or too small               */
    SEER_EHIP = -5,       /* a HIP runtime call failed; see seer_last_hip_error()     */
    SEER_ELIMIT = -6      /* seer_spmv_auto_static: the matrix needs more scratch than
                             the library's built-in array holds                         */
} seer_status;

/* Kernel ids: the CSR rows of Table II ("load balancing schedules"), in its order. */
enum {
    SEER_CSR_TM = 0, /* thread mapped: whole rows per lane (one; two from 2^20 short
                        rows on)                                                      */
    SEER_CSR_WM = 1, /* wavefront mapped: one row per group of 2..64 lanes of a wave  */
    SEER_CSR_BM = 2, /* block mapped: a block of consecutive rows per workgroup,
                        nonzeros staged through LDS                                   */
    SEER_CSR_MP = 3, /* merge path: equal shares of rows + nonzeros (Table III's CSR,MP) */
    SEER_CSR_WO = 4, /* work oriented: equal shares of nonzeros (Table III's CSR,WO)   */
    SEER_NUM_DIRECT_KERNELS = 5, /* ids below this need no preprocessing               */
    SEER_CSR_A = 5,  /* adaptive: row blocks of about 2048 nonzeros found in a
                        preprocessing pass over row_ptr, long rows split between
                        blocks (Table II's Adaptive-CSR (A); Sec. IV on its
                        preprocessing and when it is amortised)                        */
    SEER_ELL_TM = 6, /* thread mapped over the ELL format: every row padded to the
                        longest row's length, stored column-major, so that a wave's
                        loads are contiguous (Table II, "TM ... CSR, ELL").  The
                        conversion is its preprocessing; it has no one-call form.      */
    SEER_COO_WM = 7, /* wavefront mapped over the COO format: a wave takes 512 consecutive
                        (row, column, value) triples and reduces them by row (Table II,
                        "WM ... CSR, COO").  Its preprocessing expands row_ptr into one
                        row index per nonzero; columns and values are the CSR arrays.   */
    SEER_CSR_S = 8,  /* column slabbed (this build's addition to the pool, not in Table II): a
                        preprocessing pass stores the matrix a second time, every row cut into
                        one virtual row per slab of 2^w columns (w below) and the entries laid out slab
                        after slab; the product is CSR,WO over the virtual rows that hold
                        entries followed by a sum over each row's pieces, so that the gathers
                        of a long stretch of work stay inside one slab of x.  For large matrices with scattered
                        columns, whose x no longer fits one XCD's L2.  No one-call form.       */
    SEER_NUM_KERNELS = 9
};

/* CSR matrix, fp32 values, int32 indices.  All pointers DEVICE, caller-owned.
 * row_ptr[0] must be 0, row_ptr non-decreasing, row_ptr[rows] == nnz < 2^31;
 * columns may be in any order inside a row and may repeat (repeats are summed). */
typedef struct {
    int32_t rows, cols, nnz;
    const int32_t *row_ptr; /* DEVICE [rows + 1] */
    const int32_t *col_idx; /* DEVICE [nnz]      */
    const float *values;    /* DEVICE [nnz]      */
} seer_csr;

/* Feature vector indices.  0-2 are the "known" features of Sec. IV (rows, columns,
 * nonzeros); 8-11 are the gathered row-density statistics named there (density of
 * a row = its nonzero count / cols, Sec. IV-A); 3-7 are the same statistics on
 * row lengths (Table III: Most, Least, Avg, Var) plus the fraction of empty rows;
 * 12 is the number of products the caller is about to run with this matrix, known
 * to every model at no cost (Sec. IV-E, multiple iteration evaluation).  Every call here
 * that fills a vector writes 1 there; seer_spmv_plan writes the caller's count. */
enum {
    SEER_F_ROWS = 0, SEER_F_COLS, SEER_F_NNZ,
    SEER_F_MEAN_LEN, SEER_F_MAX_LEN, SEER_F_MIN_LEN, SEER_F_VAR_LEN, SEER_F_EMPTY_FRAC,
    SEER_F_MEAN_DENSITY, SEER_F_MAX_DENSITY, SEER_F_MIN_DENSITY, SEER_F_VAR_DENSITY,
    SEER_F_ITERATIONS,
    SEER_NUM_FEATURES = 13
};

/* HOST struct filled by seer_features.  Integer fields are exact.  f[] is derived
 * from them on the host: each entry is computed in fp64 from exact integers
 * (int -> double correctly rounded, one division; densities one further division
 * by cols, the variance by cols*cols) and rounded once to fp32.  Variance is the
 * population variance: (rows * sum_sq_len - nnz^2) / rows^2.  rows == 0 gives all
 * zeros except f[SEER_F_COLS]; cols == 0 gives zero densities. */
typedef struct {
    int64_t rows, cols, nnz;  /* nnz = row_ptr[rows] - row_ptr[0], read on the device */
    int64_t max_len, min_len; /* longest / shortest row (0 when rows == 0)            */
    int64_t empty_rows;
    uint64_t sum_sq_len;      /* sum over rows of len^2                               */
    float f[SEER_NUM_FEATURES];
} seer_features_t;

/* Decision tree as a flat node array, HOST memory.  Node 0 is the root.  A node with
 * feature < 0 is a leaf and yields klass.  Otherwise go to `left` iff
 * (double)f[feature] <= threshold, else to `right` (the CART convention of the
 * library the paper trains with, Sec. III-A). */
typedef struct {
    int32_t feature;
    int32_t left, right;
    int32_t klass;
    double threshold;
} seer_node;

typedef struct {
    int32_t n_nodes;
    int32_t n_features; /* entries of f[] the tree may index; <= SEER_NUM_FEATURES     */
    int32_t n_classes;  /* klass of every leaf must be in [0, n_classes)               */
    const seer_node *nodes; /* HOST [n_nodes] */
} seer_tree;

/* Feature collection (Sec. IV-A: parallel kernels that loop over the CSR offsets).
 * Reads A->row_ptr only (col_idx / values may be NULL).  Enqueues the reduction (one
 * launch up to 8192 rows, two above) on `stream`, waits for its result (the kernel's last act is to write it to
 * pinned host memory; on return the stream may still be retiring that kernel), and
 * fills *out.  workspace: DEVICE, at least
 * seer_features_workspace_bytes(A->rows) bytes (per-workgroup partial results). */
int seer_features(const seer_csr *A, seer_features_t *out,
                  void *workspace, size_t workspace_bytes, void *stream);
size_t seer_features_workspace_bytes(int32_t rows);

/* Recomputes io->f[] from the integer fields of *io by the rule stated at
 * seer_features_t (what seer_features does after its reduction; also the way to
 * finish integer partials that were combined elsewhere).  Rejects negative fields
 * and min_len > max_len.  HOST only. */
int seer_derive_features(seer_features_t *io);

/* Fills out->f[] from rows, cols, nnz alone: the input of a "known features" model
 * (Sec. III-A), which costs nothing at run time.  Besides the three integers it sets
 * the two statistics that follow from them without looking at the matrix,
 * f[SEER_F_MEAN_LEN] = nnz / rows and f[SEER_F_MEAN_DENSITY] = nnz / rows / cols
 * (same rounding rule as seer_features_t); every other gathered entry is 0.
 * HOST only, no GPU work. */
int seer_known_features(int32_t rows, int32_t cols, int32_t nnz, seer_features_t *out);

/* Tree inference (Sec. III-B: nested if/else over the input vector, yielding an
 * integer index).  HOST only.  Validates the tree (SEER_ETREE) before walking. */
int seer_select(const seer_features_t *f, const seer_tree *tree, int *kernel_id);

/* What a tree can still answer once the features that cost nothing are fixed (Sec. III-A:
 * rows, columns and nonzeros come with the dataset; Sec. III-B: collecting the others is
 * only justified where it can change the choice).  `known` is what seer_known_features
 * filled (f[SEER_F_ITERATIONS] may be set by the caller); its other entries are ignored.
 * *class_mask receives one bit per class of a leaf that a walk as in seer_select can end
 * in when every entry other than rows, cols, nnz, mean length, mean density and the
 * iteration count may take any value: at a node that tests a known entry the walk goes
 * where seer_select would, at any other node both children stay possible (tests of one
 * entry along a path are not reconciled, so the set may hold a class no matrix reaches;
 * it never misses one).  One bit set: the answer does not depend on the matrix beyond its
 * sizes.  HOST only.  SEER_ETREE for a malformed tree or more than 32 classes. */
int seer_tree_reachable(const seer_tree *tree, const seer_features_t *known, uint32_t *class_mask);

/* y = A x with the schedule `kernel_id` (Table II).  x: DEVICE [cols], y: DEVICE
 * [rows], overwritten (no alpha/beta); x and y must not overlap (SEER_EINVAL).  Every kernel id is
 * valid for every matrix and gives the same y up to fp32 summation order.
 * rows == 0: nothing is written.  Asynchronous on `stream`.
 * workspace: at least seer_spmv_workspace_bytes(kernel_id, rows, nnz) bytes (0 for
 * ids 0-2, then workspace may be NULL).
 * SEER_CSR_A and SEER_COO_WM in this single call run their preprocessing pass first, every
 * time (what one product with them costs); seer_spmv_prepare / seer_spmv_prepared split the two.
 * SEER_ELL_TM and SEER_CSR_S have no one-call form (SEER_EKERNEL): whether they apply and
 * what their plans take is only known after a look at the matrix. */
int seer_spmv(int kernel_id, const seer_csr *A, const float *x, float *y,
              void *workspace, size_t workspace_bytes, void *stream);
size_t seer_spmv_workspace_bytes(int kernel_id, int32_t rows, int32_t nnz);

/* The three steps above as one asynchronous call: the feature reduction, the tree
 * walk (on the device: the tree travels in the kernel arguments) and the SpMV with
 * the chosen schedule are enqueued on `stream` back to back and the call returns;
 * no device result is waited for, so the sequence can also be captured in a HIP
 * graph.  This is the runtime flow of Sec. III-B with the cost of feature
 * collection (Sec. III-C) cut down to the reduction kernel itself.
 * y is the same as seer_spmv would give with the id seer_select would return for
 * the features seer_features would return (all three bit for bit).
 * Before anything is enqueued the host prunes the tree with what it knows from rows,
 * cols and nnz (seer_tree_reachable): the launches are sized for the schedules that stay
 * reachable, the carry fix-up of CSR,MP / CSR,WO is enqueued only if one of them does,
 * and if a single kernel is left the matrix is not looked at: that kernel is launched and
 * nothing is gathered (Sec. III-B: collection only where it is justified).
 * tree: HOST, at most 127 nodes, no cycles, every leaf a kernel id below
 * SEER_NUM_DIRECT_KERNELS (SEER_ETREE otherwise; validated before anything is
 * enqueued).  f[SEER_F_ITERATIONS] is 1 on this path.
 * workspace: DEVICE, 16-byte aligned, >= seer_spmv_auto_workspace_bytes(rows, nnz);
 * it must stay untouched until the work has run. */
int seer_spmv_auto(const seer_csr *A, const seer_tree *tree, const float *x, float *y,
                   void *workspace, size_t workspace_bytes, void *stream);
size_t seer_spmv_auto_workspace_bytes(int32_t rows, int32_t nnz);

/* seer_spmv_auto for callers that cannot allocate device memory or hand over a workspace:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.
 * Same arguments, checks, launches and results as seer_spmv_auto, but the scratch (feature
 * partials, selection record, tile carry-outs) is an array of SEER_STATIC_SCRATCH_BYTES that
 * the library itself holds in device memory, one copy per GPU, from the moment the library
 * is loaded on that GPU until the process ends.  The call allocates and frees nothing, on the
 * device or the host.
 *   - Limit: SEER_ELIMIT if seer_spmv_auto_workspace_bytes(rows, nnz) exceeds
 *     SEER_STATIC_SCRATCH_BYTES (about 4.6e8 rows + nonzeros); nothing is enqueued then.
 *   - The first call on a device looks the array's address up (hipGetSymbolAddress, with
 *     that device current); make that call before capturing a graph.
 *   - All calls on one GPU share the one array, and it keeps the last call's contents; the
 *     kernels overwrite every word they later read, so nothing needs clearing.  Two calls
 *     on the same GPU must not overlap in time: on different streams without an ordering
 *     between them they race on the array and both results are undefined.
 *   - There is no way to ask what was selected (seer_spmv_auto_result takes a workspace). */
#define SEER_STATIC_SCRATCH_BYTES (2u << 20)
int seer_spmv_auto_static(const seer_csr *A, const seer_tree *tree, const float *x, float *y,
                          void *stream);

/* The three models of Sec. III-A.  `selector` is the classifier-selection model: it
 * sees only the known features (seer_known_features) and answers 0 = "the known
 * model is good enough" or 1 = "gather the features first".  `known` maps the known
 * features to a kernel id, `gathered` maps the full feature vector to a kernel id.
 * selector == NULL means: always gather.  All pointers HOST. */
typedef struct {
    const seer_tree *selector;
    const seer_tree *known;
    const seer_tree *gathered;
} seer_model;

/* model == NULL in seer_spmv_model and seer_spmv_plan selects the models the library was built
 * with: the trained trees of selector_model.json emitted as nested if/else code
 * (selector_model_generated.h, the deployment form of Sec. III-D) and compiled in; they choose
 * exactly as the same trees passed as node arrays would.
 *
 * Runtime inference with the classifier-selection model (Sec. III-B): the selector is
 * evaluated on the host at no GPU cost; on 0 the known model's kernel is launched
 * directly (seer_spmv), on 1 the features are gathered and the gathered model is
 * applied on the device (seer_spmv_auto).  Asynchronous on `stream` either way.
 * *path (may be NULL) receives 0 or 1; *kernel_id (may be NULL) receives the kernel id
 * when the known model was used and -1 otherwise (ask seer_spmv_auto_result then).
 * Both models must answer with ids below SEER_NUM_DIRECT_KERNELS (SEER_ETREE).
 * workspace: >= seer_spmv_auto_workspace_bytes(rows, nnz). */
int seer_spmv_model(const seer_csr *A, const seer_model *model, const float *x, float *y,
                    void *workspace, size_t workspace_bytes, void *stream,
                    int *path, int *kernel_id);

/* Waits for `stream`, then reports what the last seer_spmv_auto that used `workspace`
 * decided: the features it gathered and the kernel id it ran (either may be NULL).
 * If the host could decide alone (see seer_spmv_auto) nothing was gathered: *features
 * then holds what seer_known_features gives, with max_len = min_len = empty_rows = -1
 * as the mark.  The record is whatever that call left at a fixed place in the workspace;
 * other calls that are handed the same workspace may overwrite it.
 * SEER_EINVAL if no selection has been written there. */
int seer_spmv_auto_result(const void *workspace, void *stream, seer_features_t *features,
                          int *kernel_id);

/* Preprocessing split from the product (Sec. IV: a preprocessing step that occurs once
 * over the span of the iterations and is amortised from some iteration count on).
 * A seer_plan is a HOST struct the caller owns; `device` points into the caller's
 * plan_mem.  It belongs to the matrix it was prepared for (same row_ptr contents) and
 * stays valid until plan_mem is reused. */
typedef struct {
    int32_t kernel_id;
    int32_t rows, nnz;    /* of the matrix it was prepared for                          */
    int32_t n_blocks;     /* SEER_CSR_A: row blocks in the plan; SEER_CSR_S: column slabs  */
    int32_t split_rows;   /* SEER_CSR_A: 1 if some row is shared between blocks (the
                             product then needs the carry workspace and a second launch);
                             SEER_CSR_S: the number of virtual rows kept                 */
    int32_t ell_width;    /* SEER_ELL_TM: slots per row = the longest row; SEER_CSR_S: log2
                             of the columns per slab                                     */
    void *device;         /* DEVICE, inside plan_mem; NULL for kernels without a plan   */
    size_t device_bytes;
} seer_plan;

/* Device bytes seer_spmv_prepare needs for `kernel_id` (0 for ids that need none, and for
 * SEER_ELL_TM, whose need depends on the longest row: see seer_ell_plan_bytes). */
size_t seer_plan_bytes(int kernel_id, int32_t rows, int32_t nnz);

/* Device bytes of the ELL form of a matrix with `rows` rows whose longest row has max_len
 * entries: 2 arrays of roundup(rows, 64) * max_len 4-byte words (each padded to 256 bytes).
 * 0 if that is 2^31 words or more: the format is then not applicable. */
size_t seer_ell_plan_bytes(int32_t rows, int32_t max_len);

/* Device bytes of the column-slabbed form of a rows x cols matrix with nnz nonzeros: offsets
 * and piece lists for up to min(nnz, S * rows) kept virtual rows, S = ceil(cols / 2^w), a
 * second copy of col_idx and of values, and the preprocessing's own scratch (8 bytes per
 * virtual row).  0 if the form does not apply by size alone:
 * S < 2 (x is one slab) or S * rows >= 2^31.
 * The slab width: w = 19 (2 MiB of x); w = 20 if that gives at least four slabs and fewer
 * than three entries are to be expected per piece of a row (nnz / rows < 3 * ceil(cols / 2^19));
 * the "slab_shift" tuning knob overrides both.  The plan keeps its w in ell_width. */
size_t seer_slab_plan_bytes(int32_t rows, int32_t cols, int32_t nnz);

/* Runs the preprocessing of `kernel_id` for A on `stream` and fills *plan.  For
 * SEER_CSR_A: one pass over A->row_ptr that writes, for block k = 0 .. n-1 of
 * n = max(1, ceil(nnz / 2048)), the pair {first row, first nonzero}:
 *   block 0 starts at row 0, nonzero 0; block k > 0 starts with the first row that ends
 *   after nonzero 2048 k, at that row's first nonzero, or at nonzero 2048 k if the row
 *   also began block k - 1 (such a block holds nothing but part of that row);
 *   entry n is {rows, nnz}.
 * For SEER_ELL_TM: finds the longest row (the feature reduction, with plan_mem as its
 * workspace, so plan_mem must hold at least seer_features_workspace_bytes(rows)), then
 * writes cols[j * R + i] / vals[j * R + i] = the j-th entry of row i in CSR order, or
 * -1 / 0 where the row is shorter, R = roundup(rows, 64), cols first, vals at half of
 * seer_ell_plan_bytes(rows, longest row).  If plan_mem is too small the call returns
 * SEER_EWORKSPACE and stores the bytes needed in plan->device_bytes, the one output written
 * on an error (the rest of *plan stays as it was): seer_features_workspace_bytes(rows) while
 * plan_mem cannot even hold the reduction's workspace, the size of the ELL form after that,
 * so sizing may take two rounds.  SEER_EINVAL if the format is not applicable.
 * For SEER_COO_WM: writes the row index of every nonzero, in CSR order (int32 [nnz]).
 * For SEER_CSR_S: with S = ceil(cols / 2^w) slabs, virtual row s * rows + i is the entries of
 * row i with column >> w == s, in their CSR order; only the virtual rows that hold entries
 * are kept, numbered in the order of s * rows + i.  With K of them and M = min(nnz, S * rows),
 * plan_mem receives, each array padded to 256 bytes: rp_z (uint32 [M + 1], used [K + 1]: the
 * entries before kept row j; rp_z[K] = nnz), p_idx (uint32 [M + 1], used [K]: the kept rows that
 * are pieces of row 0, then of row 1, ..., in slab order), rp_j (uint32 [rows + 1]: the pieces
 * before row i), then col_idx and values ([nnz + 1] each) in the order of the kept rows;
 * plan->n_blocks = S, plan->split_rows = K.
 * plan_mem must hold seer_slab_plan_bytes(rows, cols, nnz) (SEER_EWORKSPACE otherwise, with
 * the bytes needed in plan->device_bytes, as for SEER_ELL_TM).  SEER_EINVAL if the form does
 * not apply: by size (seer_slab_plan_bytes gives 0), or because some row's columns do not
 * ascend -- a virtual row must be one contiguous piece of its row.
 * HOST-SYNCHRONOUS: returns after the pass has finished (it reads back whether any row
 * is split, or the longest row).  plan_mem: DEVICE, 16-byte aligned, >= seer_plan_bytes();
 * may be NULL for kernels that need no plan (the call then only records the id).  Not
 * capturable. */
int seer_spmv_prepare(int kernel_id, const seer_csr *A, void *plan_mem, size_t plan_bytes,
                      void *stream, seer_plan *plan);

/* y = A x with a prepared plan; same contract as seer_spmv.  For kernels without
 * preprocessing this is seer_spmv(plan->kernel_id, ...).  Asynchronous, capturable.
 * workspace: >= seer_spmv_prepared_workspace_bytes(plan) (0 for SEER_CSR_A when no row
 * is split).  SEER_EINVAL if rows / nnz differ from the matrix the plan was made for. */
int seer_spmv_prepared(const seer_plan *plan, const seer_csr *A, const float *x, float *y,
                       void *workspace, size_t workspace_bytes, void *stream);
size_t seer_spmv_prepared_workspace_bytes(const seer_plan *plan);

/* Selection for `iterations` >= 1 products with the same matrix (Sec. IV-E, multiple
 * iteration evaluation): classifier-selection inference as in seer_spmv_model, with
 * f[SEER_F_ITERATIONS] = iterations in the vector every tree sees, so a model trained on
 * (preprocessing + iterations * run time) can tell when preprocessing is amortised; then
 * seer_spmv_prepare for the chosen kernel.  The features, when the selector asks for
 * them, are gathered with seer_features.  HOST-SYNCHRONOUS.  Any kernel id may be
 * chosen; if it is SEER_ELL_TM or SEER_CSR_S and plan_mem cannot hold the converted matrix
 * (or the form is not applicable) the call prepares SEER_CSR_A instead, the schedule that
 * is safe on every matrix.  *path (may be NULL): 0 known model, 1 gathered model.
 * workspace: >= seer_features_workspace_bytes(rows); plan_mem: >= seer_plan_bytes(
 * SEER_CSR_A, rows, nnz) unless the model cannot answer SEER_CSR_A. */
int seer_spmv_plan(const seer_csr *A, const seer_model *model, int32_t iterations,
                   void *plan_mem, size_t plan_bytes, void *workspace, size_t workspace_bytes,
                   void *stream, seer_plan *plan, int *path);

/* Input check (the kernels consume the CSR offsets and entries as given, Sec. IV-A, and
 * read or write out of bounds on a matrix that is not well formed; no other entry point
 * looks at the contents).  Counts on the device
 *   *bad_row_ptr = [row_ptr[0] != 0] + [row_ptr[rows] != nnz]
 *                  + #{ i in [0, rows) : row_ptr[i+1] < row_ptr[i] }
 *   *bad_col_idx = #{ k in [0, nnz) : col_idx[k] < 0 or col_idx[k] >= cols }
 * Both zero means every schedule may run on A: offsets lie in [0, nnz], rows are
 * contiguous ranges, gathers stay inside x.  Reads row_ptr[0..rows] and col_idx[0..nnz-1]
 * only (A->values may be NULL; with A->col_idx NULL the column count is 0), so the arrays
 * must have those sizes, whatever they hold.  workspace: DEVICE, 16-byte aligned, at least
 * 16 bytes.  Host-synchronous (waits for `stream`; not capturable).  Returns SEER_OK
 * when the check ran, whatever it found; the counts are the verdict. */
int seer_csr_check(const seer_csr *A, int64_t *bad_row_ptr, int64_t *bad_col_idx,
                   void *workspace, size_t workspace_bytes, void *stream);

/* Launch-shape overrides for experiments; the defaults (value < 0) derive every
 * launch shape from rows and nnz alone (the trivially known sizes of Sec. III-A).
 *   "wm_lanes"  lanes per row of CSR,WM: 2, 4, 8, 16, 32 or 64
 *   "bm_rows"   rows per workgroup of CSR,BM: 1..2048 (seer_spmv_auto takes at most 1024)
 *   "bm_chunk"  products staged in LDS per pass of CSR,BM: 2048 or 4096
 *   "mp_ipt"    merge items per lane of CSR,MP: 7 or 15
 *   "xcd_remap" 1: consecutive tiles stay on one XCD (default), 0: round-robin
 *   "nt"        1: the matrix streams are loaded with the non-temporal hint, 0: plain
 *               loads.  Default: 1 in seer_spmv / seer_spmv_auto; in seer_spmv_prepared
 *               (repeated products) 1 only if what the kernel reads and writes exceeds
 *               288 MiB (last-level cache + L2), so that a smaller matrix stays cached
 *               between products
 *   "vec"       0: CSR,BM / CSR,MP / CSR,WO / CSR,A take entries with lane-strided 4-byte
 *               loads instead of 16-byte loads (what matrices whose col_idx / values
 *               are not 16-byte aligned get anyway); default 1
 *   "auto_fused_rows", "auto_fused_grid", "auto_fused_max_rows"  seer_spmv_auto: a matrix of
 *               at most auto_fused_rows rows (default 8192) is gathered, selected and
 *               multiplied in one launch; a larger one gets a first reduction pass and the
 *               selection runs inside the product's launch if that launch has at most
 *               auto_fused_grid workgroups (default 1024) or the matrix at most
 *               auto_fused_max_rows rows (default 2^21); otherwise the selection is a
 *               launch of its own (both 0: always)
 *   "auto_prune" 0: seer_spmv_auto does not prune the tree with the known features (every
 *               schedule counts as reachable, the features are always gathered); default 1
 *   "slab_shift" CSR,S: log2 of the columns per slab, 1..30 (default: 19 or 20, see
 *               seer_slab_plan_bytes); the size functions follow it
 *   "coo_runs"  COO,WM: 1 (default): a lane sums a run of eight consecutive triples,
 *               0: lane <-> triple in rounds of 64
 *   "poll"      0: seer_features waits with hipStreamSynchronize only; otherwise
 *               (default) it first watches its pinned result word for up to 2 ms
 * Unknown name: SEER_EINVAL.  A value outside the listed set selects the default. */
int seer_set_tuning(const char *name, int value);

/* Measurement aid, not part of the method: dst[i] = src[i] for n 4-byte words with
 * 16-byte accesses (dst, src DEVICE, 16-byte aligned, non-overlapping).  A kernel of
 * exactly known traffic (4n bytes read, 4n written) against which hardware byte
 * counters are calibrated and the attainable streaming bandwidth is measured. */
int seer_stream_copy(void *dst, const void *src, size_t n_words, void *stream);

/* Measurement aid: reads n 4-byte words of src (DEVICE, 16-byte aligned) and adds a
 * checksum into out64 (DEVICE, 64 uint32 words, caller-zeroed or not): a read-only
 * stream of exactly 4n bytes, the access pattern an SpMV mostly is. */
int seer_stream_sum(const void *src, size_t n_words, void *out64, void *stream);
/* Measurement aid: sum over k < n (rounded down to a multiple of 4) of val[k] * x[idx[k]],
 * idx and val (DEVICE, 16-byte aligned) streamed, x (DEVICE) gathered; every idx[k] must
 * index x.  With uniformly random idx its rate is the ceiling of a product whose columns
 * are random, for that size of x.  out64: DEVICE, 256 bytes, receives per-wave sums
 * (meaningless).  Asynchronous. */
int seer_gather_sum(const int32_t *idx, const float *val, size_t n, const float *x, void *out64,
                    void *stream);

/* Measurement aid: what the host part of seer_spmv_model costs -- the known features, the
 * walk of the classifier-selection tree and, where it answers 0, of the known model (Sec.
 * III-B: the cost of inference is small but accounted for).  Runs exactly that `reps` times
 * and stores the mean wall-clock nanoseconds per decision in *ns.  HOST only. */
int seer_model_host_ns(const seer_model *model, int32_t rows, int32_t cols, int32_t nnz, int32_t reps,
                       double *ns);

int seer_num_kernels(void);
const char *seer_kernel_name(int kernel_id); /* "CSR,TM" ...; NULL if out of range  */
const char *seer_strerror(int status);
int seer_last_hip_error(void);               /* raw hipError_t of the last SEER_EHIP */

#ifdef __cplusplus
}
#endif
#endif /* SEER_H */
