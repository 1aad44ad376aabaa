/*
 * libfuse -- execution of generated fused operators on MI355X (gfx950).
 *
 * One entry point per fusion template of the paper (Table 1, "CPlan Template
 * Types and their Variants"): Cell, MAgg, Row and Outer.  A fused operator is
 * a template skeleton (data access, parallelisation, aggregation: hand-written
 * HIP) plus a generated body (Sec. 2.2, "Runtime Integration": the skeleton
 * calls `genexec` per cell / row / non-zero).  Here the body is given as a
 * postfix expression descriptor (the analogue of a CPlan, Sec. 2.2 "Code
 * Generation Plans"), turned into HIP source, compiled with hipRTC and kept in
 * a plan cache keyed by the descriptor (Sec. 2.1 "Codegen Architecture": equal
 * CPlans are compiled once).
 *
 * Conventions for every call
 *   - All `data`, `vals`, `colidx`, `rowptr` and `out` pointers are DEVICE
 *     pointers owned by the caller; libfuse never frees or reallocates them and
 *     never copies them to the host.  Descriptor structs (`fuse_expr`,
 *     `fuse_tok`, `fuse_dense`, `fuse_csr`, `fuse_side`) live in HOST memory and
 *     are only read during the call.
 *   - Matrices are fp64 (the paper's precision, Sec. 5.1 "Baselines"),
 *     row-major with a leading dimension `ld` >= cols counted in elements.
 *   - `stream` is a hipStream_t passed as void* (NULL = the null stream).  A call
 *     enqueues its kernel(s) on that stream and returns without synchronising;
 *     results are in `out` once the stream reaches that point.  The first call
 *     with a new descriptor compiles it (hipRTC, host-side, blocking).
 *   - libfuse owns a small per-(device, stream) workspace for block partials;
 *     two calls that overlap on the same stream handle from different host
 *     threads are not supported.  The workspace is allocated (hipMalloc) by the
 *     first call on a stream and grows to the largest request seen there; a call
 *     whose plan is cached and loaded and whose workspace is large enough only
 *     launches kernels (outputs are cleared by a fill kernel, arrival counters
 *     reset themselves), so after one warm-up call on the capturing stream a
 *     sequence of calls can be recorded into a HIP graph and replayed.  A call
 *     that still has to compile or to allocate while its stream is being
 *     captured fails (FUSE_ENOMEM / FUSE_ERUNTIME: the runtime refuses the
 *     allocation) and the capture is lost: warm up first.
 *   - Return value: FUSE_OK (0) or a negative fuse_status; on error nothing is
 *     enqueued and `fuse_last_error()` returns a thread-local message
 *     (including the hipRTC log for FUSE_ECOMPILE).
 *   - The only aggregation function is sum (the one the paper's operators in
 *     Sec. 5.2 use).  Sums are accumulated in fp64 in an unspecified but
 *     run-to-run deterministic order, except where noted.
 */
#ifndef LIBFUSE_FUSE_H
#define LIBFUSE_FUSE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    FUSE_OK = 0,
    FUSE_EINVAL = -1,       /* NULL pointer, negative size, bad enum value            */
    FUSE_ESHAPE = -2,       /* operand shapes do not match                            */
    FUSE_EDESC = -3,        /* malformed expression (stack, kinds, sparse-safety)     */
    FUSE_ECOMPILE = -4,     /* hipRTC rejected the generated source                   */
    FUSE_ERUNTIME = -5,     /* a HIP runtime call failed                              */
    FUSE_ENOMEM = -6,       /* workspace allocation failed                            */
    FUSE_EUNSUPPORTED = -7, /* valid request that this build does not implement       */
    FUSE_ENOTREADY = -8     /* fuse_magg_noalloc: the operator is not compiled and loaded yet */
} fuse_status;

/* Aggregation variants of Table 1.  COL and COL_T produce the same n values
 * (column sums); they differ only in the logical shape (1 x n vs n x 1). */
typedef enum {
    FUSE_AGG_NONE = 0,
    FUSE_AGG_FULL = 1,
    FUSE_AGG_ROW = 2,
    FUSE_AGG_COL = 3,
    FUSE_AGG_COL_T = 4,
    FUSE_AGG_RIGHT_MM = 5,  /* Outer only */
    FUSE_AGG_LEFT_MM = 6    /* Outer only */
} fuse_agg;

/* How a side input is addressed from cell (rix, cix) of the main input
 * (Sec. 2.2, Cell listing: getValue(b[k], n, rix, cix) and getValue(b[k], rix)). */
typedef enum {
    FUSE_SIDE_MATRIX = 0,   /* rows x cols as the main input, value at (rix, cix)     */
    FUSE_SIDE_COLVEC = 1,   /* `rows` values, value at rix  (data[rix * ld])          */
    FUSE_SIDE_ROWVEC = 2,   /* `cols` values, value at cix  (data[cix], contiguous)   */
    FUSE_SIDE_SCALAR = 3,   /* host scalar in `scalar`; passed as a kernel argument   */
    /* Row bodies only (Sec. 2.2 Row listing, vectMatMult / getVector): */
    FUSE_SIDE_RHS = 4,      /* cols(X) x k right-hand side of FUSE_OP_MATMULT, 1 <= k <= 16 */
    FUSE_SIDE_KVEC = 5,     /* rows(X) x k: row rix is a k-vector (data[rix * ld + j])       */
    /* Sparse side input (Table 1: Cell, MAgg and Row bind to sparse / dense side inputs; Sec. 5.2,
     * "Cell Operations": sparse lookups behind getValue()).  Calls over a CSR main input only
     * (fuse_cell_csr, fuse_magg_csr, fuse_row with Xs), bodies without k-vectors: */
    FUSE_SIDE_SPARSE = 6    /* rows x cols as the main input, stored as CSR in `sp`: the value at
                               (rix, cix) is the stored one, or 0 where nothing is stored   */
} fuse_side_kind;

#define FUSE_MAX_K 16

typedef struct {
    const double *data;     /* device pointer                                         */
    int64_t rows, cols;
    int64_t ld;             /* leading dimension in elements, >= cols                 */
} fuse_dense;

/* CSR with sorted, distinct column indices per row.  Every STORED entry is
 * processed, whatever its value (Table 1: the binding is to the stored cells). */
typedef struct fuse_csr_ {
    const double *vals;     /* device, nnz values                                     */
    const int32_t *colidx;  /* device, nnz column indices in [0, cols)                */
    const void *rowptr;     /* device, rows+1 offsets, int32 or int64                 */
    int32_t rowptr_is64;    /* 0: int32 offsets (nnz < 2^31), 1: int64                */
    int64_t rows, cols;
    int64_t nnz;            /* must equal rowptr[rows]                                */
} fuse_csr;

typedef struct {
    int32_t kind;           /* fuse_side_kind                                         */
    fuse_dense m;           /* MATRIX: rows x cols, ld; COLVEC: rows x 1, ld = stride
                               between consecutive rows' values; ROWVEC: 1 x cols     */
    double scalar;          /* SCALAR only                                            */
    const struct fuse_csr_ *sp; /* SPARSE only: the side matrix (host struct, device arrays; sorted, distinct
                               column indices per row, as for a main input); NULL otherwise.  `m` is not read. */
} fuse_side;

/* Postfix expression tokens. */
typedef enum {
    /* leaves */
    FUSE_OP_MAIN = 1,       /* the main input: cell value / row vector / non-zero     */
    FUSE_OP_SIDE = 2,       /* side input number `arg`                                */
    FUSE_OP_CONST = 3,      /* literal `imm` (compiled into the body)                 */
    FUSE_OP_UVDOT = 4,      /* Outer only: U[i,:] . V[j,:] at the non-zero (i, j)     */
    /* element-wise unary */
    FUSE_OP_NEG = 16, FUSE_OP_ABS, FUSE_OP_SQRT, FUSE_OP_EXP, FUSE_OP_LOG,
    FUSE_OP_POW2,           /* x * x                                                  */
    FUSE_OP_SIGN,           /* -1, 0, +1                                              */
    FUSE_OP_NEQ0,           /* x != 0 ? 1 : 0  (Sec. 2.2, Outer listing)              */
    FUSE_OP_SIGMOID,        /* 1 / (1 + exp(-x))                                      */
    /* element-wise binary: pops b, then a; pushes a (op) b */
    FUSE_OP_ADD = 32, FUSE_OP_SUB, FUSE_OP_MUL, FUSE_OP_DIV, FUSE_OP_MIN, FUSE_OP_MAX,
    FUSE_OP_POW,
    FUSE_OP_LT, FUSE_OP_LE, FUSE_OP_GT, FUSE_OP_GE, FUSE_OP_EQ, FUSE_OP_NE, /* 1.0 / 0.0 */
    /* Row template only: row vector -> per-row scalar */
    FUSE_OP_ROWSUM = 48,    /* sum over the columns of a row vector, or over the
                               entries of a k-vector                  (vectSum)        */
    FUSE_OP_DOT = 49,       /* inner product of two row vectors / two k-vectors (dotProduct) */
    /* Row template only (over a CSR main input: the products run over the stored cells) */
    FUSE_OP_MATMULT = 50,   /* pops a RHS side, then a row vector; pushes the k-vector
                               row %*% RHS                             (vectMatMult)    */
    FUSE_OP_OUTERK = 51     /* last token: pops a k-vector, then a row vector; the result is
                               the n x k matrix t(row) %*% kvec of every row, summed over
                               the rows with FUSE_AGG_COL / COL_T  (vectOuterMultAdd)   */
} fuse_op;

typedef struct {
    int32_t op;             /* fuse_op                                                */
    int32_t arg;            /* FUSE_OP_SIDE: index into `sides`; else 0               */
    double imm;             /* FUSE_OP_CONST: the literal; else 0                     */
} fuse_tok;

typedef struct {
    const fuse_tok *toks;   /* host pointer                                           */
    int32_t ntoks;
} fuse_expr;

/* --------------------------------------------------------------------------
 * Cell template (Table 1, row "Cell"; Sec. 2.2 Cell listing; Fig. 1a / Fig. 8a
 * sum(X*Y*Z)).  The body is a scalar expression evaluated at every cell
 * (rix, cix) of the dense main input X; side inputs are read at the same cell.
 *   agg NONE : out[rix * X->cols + cix] = body          (m*n values, dense, ld = cols)
 *   agg ROW  : out[rix] = sum over cix                  (m values)
 *   agg COL / COL_T : out[cix] = sum over rix           (n values)
 *   agg FULL : out[0] = sum over all cells              (1 value)
 * Shape rules: MATRIX sides m x n, COLVEC m, ROWVEC n.  Empty inputs give zero
 * sums.  Row tokens (ROWSUM, DOT) and UVDOT are FUSE_EDESC.
 */
int fuse_cell(const fuse_expr *expr, const fuse_dense *X, const fuse_side *sides, int nsides,
              int agg, double *out, void *stream);

/* MAgg template (Table 1, row "MAgg"; Fig. 1c; Sec. 5.2 "Multi-Aggregate
 * Operations"): k full aggregates over shared inputs in ONE scan of X and the
 * side inputs.  exprs[0..k) are Cell bodies; out_k[j] = sum over all cells of
 * body j (the k x 1 output).  1 <= k <= 16. */
int fuse_magg(const fuse_expr *exprs, int k, const fuse_dense *X, const fuse_side *sides,
              int nsides, double *out_k, void *stream);

/* fuse_magg for callers that cannot allocate device memory: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  Same arguments, result and summation order as
 * fuse_magg (k = 1 is the full aggregate of fuse_cell), but the call never allocates or frees device
 * memory and never compiles or loads code:
 *   - the block partials and the arrival counter live in a file-scope device array of the library
 *     (256 bytes + FUSE_NOALLOC_MAX_PARTIALS doubles, 64.25 KB, held by every GPU the library runs on
 *     until the process ends) instead of the per-stream workspace; a call whose grid needs more
 *     (number of blocks x k; at most 256 x 16 with the default launch shape) is FUSE_EUNSUPPORTED;
 *   - the operator must already be compiled and loaded on the current device, i.e. fuse_magg must have
 *     run once with the same descriptor, side kinds and 16-byte alignment of the pointers;
 *     otherwise FUSE_ENOTREADY and nothing is enqueued;
 *   - only the flat form: X and all matrix sides contiguous (ld = cols), sides MATRIX or SCALAR;
 *     anything else is FUSE_EUNSUPPORTED.
 * Each call enqueues a one-block kernel that clears the arrival counter, then the operator's kernel.
 * All calls on one GPU share the one array: calls of this entry point that overlap on a GPU (different
 * streams or host threads) race; calls on one stream are ordered and independent of each other. */
#define FUSE_NOALLOC_MAX_PARTIALS 8192
int fuse_magg_noalloc(const fuse_expr *exprs, int k, const fuse_dense *X, const fuse_side *sides,
                      int nsides, double *out_k, void *stream);

/* Cell and MAgg over a SPARSE main input (Fig. 8b / 8d; Sec. 5.2: the sparse
 * matrix X is the "sparse driver" that makes the whole operator sparse-safe).
 * The body is evaluated at the stored cells of the CSR matrix X only, with the
 * side inputs read at the same positions (dense sides by address, FUSE_SIDE_SPARSE
 * sides by a search in the side's row: 0 where the side stores nothing); it must be sparse-safe, i.e. be
 * zero wherever X has no stored cell (products with X, zero-preserving unaries,
 * sums of such), otherwise FUSE_EDESC.
 *   fuse_cell_csr: agg NONE -> nnz values on X's pattern; ROW -> rows(X) sums;
 *                  COL / COL_T -> cols(X) sums; FULL -> 1 value.
 *   fuse_magg_csr: k full aggregates in one scan of X; out_k[j] = sum of body j.
 */
int fuse_cell_csr(const fuse_expr *expr, const fuse_csr *X, const fuse_side *sides, int nsides,
                  int agg, double *out, void *stream);
int fuse_magg_csr(const fuse_expr *exprs, int k, const fuse_csr *X, const fuse_side *sides,
                  int nsides, double *out_k, void *stream);

/* Row template (Table 1, row "Row"; Sec. 2.2 Row listing; Fig. 1b / Fig. 8e-f
 * t(X) %*% (X %*% v)).  The body runs once per row of the main input, dense
 * (Xd) or CSR (Xs) -- exactly one of the two is non-NULL.  Values in the body
 * are row vectors (MAIN, MATRIX and ROWVEC sides) or per-row scalars (COLVEC
 * and SCALAR sides, constants, results of ROWSUM / DOT); binary operators
 * broadcast a scalar over a vector.
 *   vector result:  NONE -> out is m x n dense (Xd) or nnz values on X's pattern
 *                   (Xs); ROW -> m row sums; COL / COL_T -> n column sums
 *                   (t(X) %*% q is the body `X_i * q_i` with COL_T); FULL -> 1.
 *   scalar result:  NONE -> m values; FULL -> 1; others FUSE_EDESC.
 *   k-vector result (products with a FUSE_SIDE_RHS, FUSE_SIDE_KVEC sides;
 *                   element-wise operators work per component, scalars broadcast):
 *                   NONE -> m x k; COL / COL_T -> k sums over the rows; FULL -> 1.
 *   OUTERK result:  COL / COL_T -> out is n x k, contiguous: sum over the rows of
 *                   t(row vector) %*% k-vector.  t(X) %*% (X %*% V) is the body
 *                   MAIN, MAIN, SIDE V, MATMULT, OUTERK  (Fig. 8g); the core of multinomial
 *                   logistic regression (Sec. 2.2, second example) is one such body too.
 *                   Limit of this build: ceil(n / 2048) * 2 * k <= 48 (n <= 2048 for k = 16).
 *                   From 2 to 5 classes on, depending on the number of columns (and up to about
 *                   1200 columns), this shape runs on the fp64 matrix units; so does a CSR main
 *                   input that stores at least 15 % of its cells, from 5 classes on.
 * For CSR input the body must be sparse-safe (Sec. 2.2 "Template Types": a
 * sparse-safe template binds only to the non-zeros): every vector that is
 * aggregated, multiplied with a right-hand side or returned must be zero
 * wherever X has no stored cell (products with X, zero-preserving unaries,
 * sums of such); otherwise FUSE_EDESC.  MATMULT / OUTERK then run over the
 * stored cells of a row.
 * With CSR input and COL / COL_T the order in which a block's rows are added
 * to a column sum is not fixed (shared-memory atomics while the sums fit in LDS, about 18000 columns; fp64
 * atomics on the zeroed output beyond); all else is deterministic.
 * Limits of this build: bodies with ROWSUM / DOT need cols <= 32768 for dense
 * input, bodies with k-vectors cols <= 2048 (FUSE_EUNSUPPORTED beyond).
 */
int fuse_row(const fuse_expr *expr, const fuse_dense *Xd, const fuse_csr *Xs,
             const fuse_side *sides, int nsides, int agg, double *out, void *stream);

/* Outer template (Table 1, row "Outer"; Sec. 2.2 Outer listing and the
 * paragraph after it; Fig. 1d / Fig. 8h sum(X * log(U %*% t(V) + eps))).
 * The body is a scalar expression evaluated at every stored cell (i, j) of
 * the CSR matrix X with MAIN = X_ij and UVDOT = U[i,:] . V[j,:]; U is
 * X->rows x r, V is X->cols x r; U %*% t(V) is never formed.  Side inputs are
 * dense and read at (i, j) / i / j.
 *   agg FULL     : out[0] = sum over stored cells of body
 *   agg NONE     : out[p] = body at stored cell p (nnz values on X's pattern)
 *   agg RIGHT_MM : out is rows(X) x r, contiguous: out[i,:] = sum over the stored
 *                  cells (i, j) of row i of body * V[j,:]  (the listing's
 *                  vectMultAdd: "scale V_j by w_ij and add it to the output row")
 *   agg LEFT_MM  : out is cols(X) x r, contiguous: out[j,:] = sum over the stored
 *                  cells (i, j) of column j of body * U[i,:]  (the mirrored variant).
 *                  The library first transposes X into its workspace (a counting sort
 *                  by column, a few small kernels on the same stream; about 28 bytes
 *                  per stored cell) and then walks the columns like
 *                  RIGHT_MM walks the rows; the cells of a column are added in the order
 *                  the sort's atomics left them in, which is not fixed from run to run.
 *                  rows(X) < 2^27 (else a scatter with fp64 atomics on the output).
 * 1 <= r <= 1024.  When V is larger than a few MB, FULL and NONE first build a table of
 * per-row offsets into column panels in the library's workspace (one more kernel on
 * the same stream; (P+1) x rows(X) offsets, P <= 1024 panels) and rely on the
 * ascending column indices the CSR format prescribes; with other column orders the
 * result is undefined (but no access leaves the arrays). */
int fuse_outer(const fuse_expr *expr, const fuse_csr *X, const fuse_dense *U, const fuse_dense *V,
               const fuse_side *sides, int nsides, int agg, double *out, void *stream);

/* Outer LEFT_MM over a pattern prepared once (Sec. 2.2, first example: the ALS-CG update is evaluated in
 * every iteration on the same X while U and V change).  fuse_outer LEFT_MM sorts X by column in every call;
 * here that is done once:
 *   fuse_outer_left_pattern_bytes : device bytes a prepared pattern of X takes (20 bytes per stored cell plus
 *                                   the column offsets; 0 for a NULL / negative X);
 *   fuse_outer_left_prepare       : writes the pattern of X -- its cells ordered by column: their rows, their
 *                                   places in X's arrays and their values -- into `pattern` (device memory of that
 *                                   many bytes, 16-byte aligned, owned by the caller); a few kernels on `stream`,
 *                                   scratch from the library's per-stream workspace;
 *   fuse_outer_left_values        : X has new values on the same structure: brings them into the pattern's order
 *                                   again (one kernel; rowptr and colidx of X are not read);
 *   fuse_outer_left               : fuse_outer LEFT_MM (same arguments, result and errors) over the pattern: MAIN is
 *                                   the value the pattern holds since the last prepare / values call, X gives the
 *                                   shape only.  The cells of a column are added in the pattern's order: calls with
 *                                   one pattern are run-to-run deterministic.
 * rows(X) < 2^27 (FUSE_EUNSUPPORTED beyond).  A pattern that was prepared for another structure than X's gives
 * undefined results (but no access leaves the arrays of a pattern of the right size). */
size_t fuse_outer_left_pattern_bytes(const fuse_csr *X);
int fuse_outer_left_prepare(const fuse_csr *X, void *pattern, void *stream);
int fuse_outer_left_values(const fuse_csr *X, void *pattern, void *stream);
int fuse_outer_left(const fuse_expr *expr, const fuse_csr *X, const void *pattern, const fuse_dense *U,
                    const fuse_dense *V, const fuse_side *sides, int nsides, double *out, void *stream);

/* Validate a request and compile its body into the plan cache without
 * launching anything (no device needed: the target is FUSE_ARCH, default
 * gfx950, when no GPU is present).  Same arguments and errors as the calls
 * above; data pointers may be NULL, only shapes, `ld`, kinds and the
 * expression are used (alignment is assumed to be 16 bytes). */
int fuse_prepare_cell(const fuse_expr *expr, const fuse_dense *X, const fuse_side *sides,
                      int nsides, int agg);
int fuse_prepare_magg(const fuse_expr *exprs, int k, const fuse_dense *X, const fuse_side *sides,
                      int nsides);
int fuse_prepare_cell_csr(const fuse_expr *expr, const fuse_csr *X, const fuse_side *sides,
                          int nsides, int agg);
int fuse_prepare_magg_csr(const fuse_expr *exprs, int k, const fuse_csr *X, const fuse_side *sides,
                          int nsides);
int fuse_prepare_row(const fuse_expr *expr, const fuse_dense *Xd, const fuse_csr *Xs,
                     const fuse_side *sides, int nsides, int agg);
int fuse_prepare_outer(const fuse_expr *expr, const fuse_csr *X, const fuse_dense *U,
                       const fuse_dense *V, const fuse_side *sides, int nsides, int agg);

/* Number of fp64 values that `out` of the fuse_row call with the same arguments must hold (Table 1, row
 * "Row": the shape of the result follows from the kind of the body's result -- row vector, per-row scalar,
 * k-vector, row (x) k-vector -- and the variant).  Validates like fuse_prepare_row (data pointers may be
 * NULL), compiles and launches nothing; same errors.  *count is written only on FUSE_OK. */
int fuse_row_out_count(const fuse_expr *expr, const fuse_dense *Xd, const fuse_csr *Xs,
                       const fuse_side *sides, int nsides, int agg, int64_t *count);

/* Structure check of a CSR matrix, on the device (the template calls themselves trust the
 * format they are given: offsets or column indices that point outside the arrays make them
 * read outside the arrays).  Verifies rowptr[0] == 0, rowptr[rows] == nnz, non-decreasing
 * offsets inside [0, nnz], every column index in [0, cols) and strictly ascending column
 * indices within each row (sorted, no duplicates); no cell is read before its row's offsets
 * have passed.  The values are not looked at.  Enqueues one kernel on `stream` and WAITS for
 * the stream (the only call here that synchronises; it also allocates and frees 32 bytes of
 * device memory).  FUSE_OK, or FUSE_ESHAPE with fuse_last_error() naming the violation and
 * the first row that shows it; FUSE_EINVAL for NULL arrays. */
int fuse_check_csr(const fuse_csr *X, void *stream);

/* Message of the calling thread's last failed call ("" if none).  The pointer
 * stays valid until that thread's next libfuse call. */
const char *fuse_last_error(void);

/* Plan-cache counters since load / last clear: lookups that found a compiled
 * body, lookups that compiled one, and total hipRTC milliseconds.  Any pointer
 * may be NULL. */
int fuse_cache_stats(int64_t *hits, int64_t *misses, double *compile_ms);

/* Compiled code objects can outlive the process: when the environment variable
 * FUSE_CACHE_DIR names an existing directory, every body compiled by hipRTC is
 * also written there (a file per kernel, named by a hash of the generated
 * source, the compiler options and the hipRTC version; written under a
 * temporary name and renamed), and a plan-cache miss first looks there.  A
 * file that fails its length / checksum test is ignored and rewritten; an
 * unwritable directory is not an error.  Returns how many misses since load /
 * last clear were served from the directory (they count as misses above and
 * add nothing to compile_ms). */
int64_t fuse_cache_disk_hits(void);

/* Drop every compiled body and free the workspaces.  The caller must have
 * synchronised all streams that libfuse work was enqueued on. */
void fuse_cache_clear(void);

/* Copy the HIP source generated for the most recent plan-cache miss of the
 * calling thread into buf (NUL-terminated, truncated to buflen); returns the
 * full length.  For inspection and tests. */
size_t fuse_last_source(char *buf, size_t buflen);

/* Name of the kernel that the most recent successful fuse_* / fuse_prepare_*
 * call of the calling thread launched or compiled (as a profiler shows it). */
const char *fuse_last_kernel(void);

/* Measurement helpers (statically compiled kernels, not part of the paper's
 * method): a plain device-to-device copy and a read-only pass over n_doubles
 * fp64 values (n_doubles even, pointers 16-byte aligned), launched with
 * `blocks` blocks of 256 threads on `stream`.  They give the achievable HBM
 * ceiling and calibrate profiler byte counters against a known transfer.
 * `sink` is one device double that is practically never written. */
int fuse_probe_copy(double *dst, const double *src, int64_t n_doubles, int blocks, void *stream);
int fuse_probe_read(const double *src, int64_t n_doubles, int blocks, double *sink, void *stream);
/* A third measurement helper: reads `count` whole rows of a dense table (rows x row_doubles, leading
 * dimension ld, all even, row_doubles <= 128, table 16-byte aligned) in the order idx[0..count) gives
 * (device array; every entry must lie in [0, rows): like the CSR arrays it is trusted, not checked),
 * 8 lanes per row and 4 rows in flight per group -- the V_j fetch of the Outer template without its
 * arithmetic.  With random indices it gives the rate at which the device serves such row gathers from a
 * table of that size, which is the ceiling the Outer template is measured against. */
int fuse_probe_gather(const double *table, int64_t rows, int64_t row_doubles, int64_t ld,
                      const int32_t *idx, int64_t count, int blocks, double *sink, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* LIBFUSE_FUSE_H */
