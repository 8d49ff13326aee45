/*
 * mggcn -- single-GPU hot path of full-batch GCN training (MG-GCN, arXiv 2110.08688)
 * for AMD MI355X (gfx950).  C ABI.
 *
 * Conventions that hold for every entry point
 *   - Returns 0 (MGGCN_OK) or a negative mggcn_status.  mggcn_last_error() gives a
 *     thread-local message for the most recent failure on the calling thread.
 *   - Arguments are checked on the host before any HIP call is made; a call that fails
 *     with MGGCN_E_INVALID_ARG / _BAD_CSR / _OVERFLOW / _WORKSPACE / _UNSUPPORTED has
 *     touched neither the device nor any output.
 *   - "dev" pointers are device (HBM) pointers, "host" pointers are ordinary host memory.
 *     The caller owns every buffer.  The library never allocates device memory: scratch
 *     comes in through (ws, ws_bytes) arguments sized by the matching *_bytes query, and
 *     must stay untouched by the caller until the work enqueued on it has completed.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Work is
 *     enqueued asynchronously and in order on that stream; unless stated otherwise an
 *     entry point does not synchronise, and outputs are valid once the stream has drained.
 *   - Dense matrices are row-major fp32 with an explicit leading dimension in elements
 *     (ld >= number of columns); only the first `cols` entries of a row are written.  Reads stay
 *     inside the first `cols` entries too, with one exception: the gathered operand X of
 *     mggcn_spmm / mggcn_spmm_bf16 on the 16-byte path (16-byte aligned X, ldx a multiple of 4
 *     floats / 8 bfloat16) is read in whole 16-byte vectors, i.e. up to min(ldx, cols rounded up
 *     to 4 floats / 8 bfloat16) entries of every row; what lies beyond `cols` never reaches an
 *     output, but it must be readable memory (it is, inside ldx) and not part of Y.  Sparse matrices are CSR with int32 `rowptr` (n_rows+1 entries, rowptr[0]=0),
 *     int32 `colidx` ascending and duplicate-free inside a row, fp32 `val`; nnz < 2^31.
 *   - Results do not depend on launch order or timing: no floating-point atomics are used,
 *     so repeated calls on the same inputs give bit-identical outputs.
 */
#ifndef MGGCN_H_
#define MGGCN_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  MGGCN_OK = 0,
  MGGCN_E_INVALID_ARG = -1, /* null pointer, negative size, ld < cols, bad enum value ... */
  MGGCN_E_BAD_CSR = -2,     /* rowptr not monotone / index out of range / unsorted row     */
  MGGCN_E_OVERFLOW = -3,    /* a size does not fit the int32 index type                    */
  MGGCN_E_WORKSPACE = -4,   /* workspace missing, too small or misaligned (256 B)          */
  MGGCN_E_HIP = -5,         /* a HIP runtime call failed (message holds hipGetErrorString)  */
  MGGCN_E_UNSUPPORTED = -6, /* valid request this build does not implement                 */
  MGGCN_E_NO_MEMORY = -7    /* host memory for the library's own tables could not be had    */
} mggcn_status;

/* Which normalisation mggcn_csr_normalize applies to the pattern A~ = A united with I. */
typedef enum {
  MGGCN_NORM_SYM_SELFLOOP = 0, /* A^_ij = 1/sqrt(d_i d_j), d = entries per row of A~              */
  MGGCN_NORM_MEAN_IN = 1       /* A^_uv = 1/(entries in column v of A~): Eq. 2 of the paper        */
} mggcn_norm;
/* Eq. 2 normalises the columns of A, and the paper's layer (Eq. 1, 6) multiplies by the TRANSPOSE of
 * that matrix: (A^^T H)_v is the average of H over the in-neighbours of v.  mggcn_spmm's op N and the
 * forward pass of a model multiply by the matrix the graph handle was created with, so to run the
 * paper's mean-aggregation layer on a MEAN_IN matrix, create the handle with the transpose as the
 * matrix and the matrix as its transpose: mggcn_graph_create(.., rowptr_t, colidx_t, val_t, rowptr,
 * colidx, val, ..) with the arrays mggcn_csr_transpose wrote.  (For the symmetric normalisation of an
 * undirected graph the two coincide.) */

typedef enum { MGGCN_OP_N = 0, MGGCN_OP_T = 1 } mggcn_op;

/* Fused element-wise tail of a product. */
typedef enum {
  MGGCN_EPI_NONE = 0,
  MGGCN_EPI_RELU = 1,     /* out = max(out, 0)                                  (Eq. 7)          */
  MGGCN_EPI_RELU_MASK = 2 /* out = out where the value previously stored at the same output
                             element was > 0, else 0 (in-place ReLU', Eq. 8); excludes beta=1   */
} mggcn_epilogue;

/* Order of the two products inside a layer (section "Order of Computation"). */
typedef enum {
  MGGCN_ORDER_AUTO = -1,      /* SpMM first iff d_in < d_out, otherwise GeMM first (tie: GeMM) */
  MGGCN_ORDER_GEMM_FIRST = 0, /* Z = A^ (H W)                                                   */
  MGGCN_ORDER_SPMM_FIRST = 1  /* Z = (A^ H) W                                                   */
} mggcn_order;

const char* mggcn_last_error(void);

/* Library version (major*10000 + minor*100 + patch). */
int mggcn_version(void);

/* ------------------------------------------------------------------------------------------
 * Normalised adjacency  A^ = D^-1/2 (A + I) D^-1/2   (Eq. 1-2; Kipf-style self-loops)
 *
 * Input: a CSR pattern (no values).  The diagonal entry (i,i) is inserted into every row
 * i < n_cols that lacks it (an existing one is kept as a single entry), columns stay
 * ascending.  Two calls:
 *   _count  writes rowptr_out (dev, n_rows+1) and returns the entry count of A~ through
 *           nnz_out (host); it SYNCHRONISES the stream to do so.
 *   normalize  fills colidx_out / val_out (dev, nnz_out entries each) given that rowptr_out.
 * SYM mode on a square matrix takes d_i as the row count of A~ for both factors; on a
 * rectangular block (one GPU's row block of a 1-D partition) the global degrees must be
 * passed in deg_row (n_rows) and deg_col (n_cols), int32 dev arrays.  MEAN_IN uses deg_col
 * if given, else the column counts of A~.  Values are evaluated in fp64 and rounded once
 * to fp32.  validate != 0 additionally checks the input pattern on the device (sorted,
 * in range) and returns MGGCN_E_BAD_CSR after a synchronisation if it is malformed.
 * Workspace: mggcn_csr_normalize_workspace_bytes(n_rows, n_cols).
 * ---------------------------------------------------------------------------------------- */
size_t mggcn_csr_normalize_workspace_bytes(int32_t n_rows, int32_t n_cols);

int mggcn_csr_normalize_count(int32_t n_rows, int32_t n_cols, const int32_t* rowptr_in /*dev*/,
                              const int32_t* colidx_in /*dev*/, int validate,
                              int32_t* rowptr_out /*dev*/, int64_t* nnz_out /*host*/, void* ws,
                              size_t ws_bytes, void* stream);

int mggcn_csr_normalize(int32_t n_rows, int32_t n_cols, const int32_t* rowptr_in /*dev*/,
                        const int32_t* colidx_in /*dev*/, int mode /*mggcn_norm*/,
                        const int32_t* deg_row /*dev or NULL*/, const int32_t* deg_col /*dev or NULL*/,
                        const int32_t* rowptr_out /*dev, from _count*/, int32_t* colidx_out /*dev*/,
                        float* val_out /*dev*/, void* ws, size_t ws_bytes, void* stream);

/* The same two calls with 64-bit row offsets (input and output), for patterns whose entry count
 * with the diagonal reaches 2^31 (up to 2^32 - 1; one row holds fewer than 2^31).  Same
 * workspace size.  The 32-bit calls return MGGCN_E_OVERFLOW for such a pattern. */
int mggcn_csr_normalize_count64(int32_t n_rows, int32_t n_cols, const int64_t* rowptr_in /*dev*/,
                                const int32_t* colidx_in /*dev*/, int validate,
                                int64_t* rowptr_out /*dev*/, int64_t* nnz_out /*host*/, void* ws,
                                size_t ws_bytes, void* stream);

int mggcn_csr_normalize64(int32_t n_rows, int32_t n_cols, const int64_t* rowptr_in /*dev*/,
                          const int32_t* colidx_in /*dev*/, int mode /*mggcn_norm*/,
                          const int32_t* deg_row /*dev or NULL*/, const int32_t* deg_col /*dev or NULL*/,
                          const int64_t* rowptr_out /*dev, from _count64*/, int32_t* colidx_out /*dev*/,
                          float* val_out /*dev*/, void* ws, size_t ws_bytes, void* stream);

/* Explicit transpose of a CSR matrix (the paper keeps A^ and A^^T both, for the backward
 * SpMM of Eq. 9): a counting sort by column -- integer histogram, prefix sum, stable radix sort of the
 * entry positions.  Rows of the result have ascending columns; the result is unique, so it
 * is bit-reproducible.  All arrays dev; rowptr_t has n_cols+1 entries.  The input must be a
 * well-formed CSR (what mggcn_csr_normalize writes): nothing is validated here; a column index
 * outside [0, n_cols) is never followed, but the result is then meaningless.
 * _transpose64 takes and writes 64-bit row offsets (fewer than 2^32 entries); the 32-bit form
 * returns MGGCN_E_OVERFLOW from 2^31 - 1 entries on.  One workspace size serves both. */
size_t mggcn_csr_transpose_workspace_bytes(int32_t n_rows, int32_t n_cols, int64_t nnz);

int mggcn_csr_transpose(int32_t n_rows, int32_t n_cols, int64_t nnz, const int32_t* rowptr,
                        const int32_t* colidx, const float* val, int32_t* rowptr_t,
                        int32_t* colidx_t, float* val_t, void* ws, size_t ws_bytes, void* stream);

int mggcn_csr_transpose64(int32_t n_rows, int32_t n_cols, int64_t nnz, const int64_t* rowptr,
                          const int32_t* colidx, const float* val, int64_t* rowptr_t,
                          int32_t* colidx_t, float* val_t, void* ws, size_t ws_bytes, void* stream);

/* ------------------------------------------------------------------------------------------
 * Graph handle: A^ in CSR, optionally A^^T in CSR, and the one-time load-balancing analysis
 * the SpMM uses (rows cut into segments of bounded length, segments ordered longest first).
 *
 * _create reads rowptr (and rowptr_t) back to the host (validation, and the sizes the workspace query
 * needs), checks on the device that every column index lies in [0, n_cols), and SYNCHRONISES the
 * stream.  rowptr_t == NULL declares A^ symmetric (A^^T = A^, the case for the symmetric
 * normalisation of an undirected graph); op T then runs on A^ itself.
 * The CSR arrays are borrowed, not copied: they must outlive the handle.  _create checks that
 * rowptr starts at 0 and never decreases and that every column index lies in [0, n_cols)
 * (MGGCN_E_BAD_CSR otherwise, so that no product ever gathers outside X); ascending columns
 * inside a row, which the panel forms rely on, are the caller's to guarantee
 * (mggcn_csr_normalize writes them so).
 * seg_len = maximum entries per segment (0 = library default).
 * n_panels = number of column panels the SpMM walks one after the other so that all wavefronts
 * in flight gather from the same slice of X (0 = automatic: forms for 2, 4, 8, ... panels are
 * built as far as the average row length affords, and each product picks the count that brings
 * one panel of its gathered operand down to about 12 MiB (16 MiB for a bfloat16 operand), or
 * none for a small operand;
 * 1 = never; > 1 = always that many).
 * _bind builds the segment tables on the device (count, prefix sums, a stable sort by panel and
 * length, fill -- a few launches per table) in caller memory of _workspace_bytes(g, F_max) bytes, which
 * also holds the partial sums of rows that were cut, for feature widths up to F_max, and the scratch
 * of that construction; it SYNCHRONISES the stream.
 * A handle may be re-bound; it must be bound before mggcn_spmm is called.  Products on one handle
 * share its partial-sum table: enqueue them on one stream (or otherwise keep them from
 * overlapping in time); use one handle per stream for concurrent products.
 * ---------------------------------------------------------------------------------------- */
typedef struct mggcn_graph mggcn_graph;

int mggcn_graph_create(int32_t n_rows, int32_t n_cols, const int32_t* rowptr /*dev*/,
                       const int32_t* colidx /*dev*/, const float* val /*dev*/,
                       const int32_t* rowptr_t /*dev or NULL*/, const int32_t* colidx_t,
                       const float* val_t, int32_t seg_len, int32_t n_panels, void* stream,
                       mggcn_graph** out);
/* The same with 64-bit row offsets, for matrices of 2^31 entries and more (fewer than 2^32: the
 * segment tables hold entry offsets in 32 unsigned bits; a single row holds fewer than 2^29).
 * Everything else about the handle is unchanged. */
int mggcn_graph_create64(int32_t n_rows, int32_t n_cols, const int64_t* rowptr /*dev*/,
                         const int32_t* colidx /*dev*/, const float* val /*dev*/,
                         const int64_t* rowptr_t /*dev or NULL*/, const int32_t* colidx_t,
                         const float* val_t, int32_t seg_len, int32_t n_panels, void* stream,
                         mggcn_graph** out);
size_t mggcn_graph_workspace_bytes(const mggcn_graph* g, int32_t F_max);
int mggcn_graph_bind(mggcn_graph* g, int32_t F_max, void* ws /*dev*/, size_t ws_bytes, void* stream);
int mggcn_graph_destroy(mggcn_graph* g);
/* Tuning knobs of a handle (sweeps and tests; the defaults are what was measured best on MI355X).
 * They change how later products are launched, never their result beyond summation order, and
 * leave the binding valid.
 * panel_mib: size in MiB that one column panel of a product's gathered operand is brought down to
 *   when the panel count is automatic (n_panels = 0 at creation); 0 = leave as it is (default 16:
 *   16 MiB for a bfloat16 operand, three quarters of it for an fp32 one).
 * chunk_lanes: lanes of a wavefront that share one gathered row (a power of two up to 64; fewer
 *   lanes = narrower feature chunks, dealt to workgroups round-robin); 0 = leave as it is,
 *   -1 = back to the default (as many as the row needs). */
int mggcn_graph_tune(mggcn_graph* g, int32_t panel_mib, int32_t chunk_lanes);
/* The segment tables of a bound handle, for tests and tools (read-only; the layout may change with the
 * library version).  form 0 = the single-pass table, 1.. = the column-panel tables in ascending panel
 * count; returns the number of panel tables (>= 0) or a negative status.  Any output pointer may be
 * NULL.  tasks (dev): n_tasks records {int32 row; uint32 first entry; uint32 length | first << 30 |
 * last << 29; int32 slot (< 0: the row's result goes to Y)}, panel-major, inside a panel longest
 * first and in row order among equal lengths; task_begin / fix_begin (host): n_panels + 1 offsets, so
 * give room for 65 entries; fix (dev): n_fix records {int32 row, first slot, slot count; uint32 flags}
 * of the (row, panel) ranges that were cut into several segments. */
int mggcn_graph_tables(const mggcn_graph* g, int op /*mggcn_op*/, int32_t form, int32_t* n_panels,
                       int64_t* n_tasks, const void** tasks /*dev*/, int64_t* task_begin /*host*/,
                       int64_t* n_fix, const void** fix /*dev*/, int64_t* fix_begin /*host*/,
                       int64_t* n_slots);
/* Number of passes over the entries a plain (epilogue NONE or RELU) fp32 SpMM of width F with
 * the given op makes on this graph: column panels x feature slices (1 = single pass), or a
 * negative status. */
int mggcn_graph_panels(const mggcn_graph* g, int op /*mggcn_op*/, int32_t F);

/* SpMM (Eq. 6 forward, Eq. 9 backward):   Y = epilogue( op(A^) X + beta Y )
 * op N: X is n_cols x F, Y is n_rows x F.  op T: X is n_rows x F, Y is n_cols x F.
 * beta is 0 or 1 (1 = accumulate, the stage loop C^i += A^{ij} H^j of the 1-D row scheme).
 * The address ranges of X and Y must not overlap (checked).  F <= the F_max the graph was bound with.  16-byte aligned
 * pointers and leading dimensions that are multiples of 4 take the widest gather path;
 * anything else still works through narrower loads.  A gather costs time per 128-byte line a row
 * of X touches: rows that start at multiples of 64 bytes (ldx a multiple of 16; 32 for the
 * bfloat16 form) never touch more lines than their length requires -- a bfloat16 row of 41 elements
 * at multiples of 32 bytes measured 30 % slower than at multiples of 64. */
int mggcn_spmm(const mggcn_graph* g, int op /*mggcn_op*/, const float* X /*dev*/, int64_t ldx,
               int32_t F, float beta, int epilogue /*mggcn_epilogue*/, float* Y /*dev*/,
               int64_t ldy, void* stream);

/* SpMM with a bfloat16 gathered operand -- an extension beyond the paper, whose operands are all
 * fp32.  The product spends its memory traffic on gathering rows of X; holding X as bfloat16
 * (the upper 16 bits of an fp32: 8 exponent, 7 fraction bits) halves it.  Values of A^ stay fp32,
 * every product and sum is fp32, Y is fp32; given the same bfloat16 X the result meets the same
 * error bound as mggcn_spmm, and against an fp32 X it differs by the rounding of X (relative
 * 2^-8 per element at most).  Same arguments and rules as mggcn_spmm; X is n x F 2-byte elements
 * with leading dimension ldx (elements).  A 16-byte aligned X with ldx a multiple of 8 (and a
 * 16-byte aligned Y with ldy a multiple of 4) takes the wide path, anything else goes element
 * by element. */
int mggcn_spmm_bf16(const mggcn_graph* g, int op /*mggcn_op*/, const uint16_t* X /*dev, bfloat16*/,
                    int64_t ldx, int32_t F, float beta, int epilogue /*mggcn_epilogue*/, float* Y /*dev*/,
                    int64_t ldy, void* stream);

/* fp32 -> bfloat16 copy of a rows x cols matrix, IEEE round to nearest, ties to even (overflow
 * goes to infinity, a NaN stays a NaN).  Columns [cols, ldd) of dst are left untouched. */
int mggcn_f32_to_bf16(int64_t rows, int32_t cols, const float* src /*dev*/, int64_t lds,
                      uint16_t* dst /*dev*/, int64_t ldd, void* stream);

/* ------------------------------------------------------------------------------------------
 * GeMM (Eq. 5, 10, 11):   C = epilogue( op(A) op(B) + beta C ),   C is M x N, inner size K
 *   opA = N: A is M x K;  opA = T: A is K x M.   opB = N: B is K x N;  opB = T: B is N x K.
 * beta is 0 or 1.  fp32 inputs, fp32 MFMA accumulation.  opA = T with a long inner dimension
 * (the weight gradient W_G = H^T HW_G of Eq. 10, inner size = vertex count) is split along K
 * into partial products held in ws and summed in a fixed order.
 * Any alignment and leading dimension is accepted; operands whose rows start on 16-byte boundaries
 * (A and B 16-byte aligned, lda and ldb multiples of 4) with N a multiple of 64 and K >= 64 take the
 * faster of the two kernels (about 1.1x; results agree to rounding, the order of summation differs).
 * Workspace: mggcn_gemm_workspace_bytes (0 for opA = N; one size serves mggcn_gemm and
 * mggcn_gemm_bf16x3).
 * ---------------------------------------------------------------------------------------- */
size_t mggcn_gemm_workspace_bytes(int opA, int opB, int64_t M, int64_t N, int64_t K);

int mggcn_gemm(int opA, int opB, int64_t M, int64_t N, int64_t K, const float* A /*dev*/,
               int64_t lda, const float* B /*dev*/, int64_t ldb, float beta, int epilogue,
               float* C /*dev*/, int64_t ldc, void* ws, size_t ws_bytes, void* stream);

/* The same product, same arguments and workspace, on the bfloat16 matrix instructions (beyond the
 * paper, which multiplies in fp32 on CUDA cores).  Nothing is rounded to bfloat16: every fp32 operand is
 * cut, exactly, into three bfloat16 pieces (its upper 16 bits, the upper 16 bits of the rest, the
 * rest), and the product a b is formed from the six largest of the nine piece products, each of
 * them exact, added in fp32.  What is left out is below 2^-21 |a b| per product (2^-24 |a b| on
 * average, one fp32 rounding of it) and does not grow with K; measured against the fp64 result
 * the error is a third of mggcn_gemm's (2e-7 against 7e-7 of a row's norm at K = 602).  About
 * 1.1-1.45x the speed of mggcn_gemm on the shapes of a GCN layer.  Inner dimensions below 64 run
 * on the fp32 instruction as in mggcn_gemm.  An Inf operand gives NaN where fp32 arithmetic gives
 * Inf; operands below 2^-110 in magnitude lose their lower pieces (absolute error < 2^-126). */
int mggcn_gemm_bf16x3(int opA, int opB, int64_t M, int64_t N, int64_t K, const float* A /*dev*/,
                      int64_t lda, const float* B /*dev*/, int64_t ldb, float beta, int epilogue,
                      float* C /*dev*/, int64_t ldc, void* ws, size_t ws_bytes, void* stream);

/* In-place ReLU' (Eq. 8):  G[i,f] = act[i,f] > 0 ? G[i,f] : 0.  act may be the layer's
 * pre- or post-activation output (same mask). */
int mggcn_relu_bwd(int64_t rows, int32_t cols, const float* act /*dev*/, int64_t lda,
                   float* G /*dev*/, int64_t ldg, void* stream);

/* Softmax cross-entropy, mean over all n rows, and its gradient (the loss the paper trains
 * with):  *loss_dev = (1/n) sum_i [logsumexp(z_i) - z_i[label_i]],
 *         dlogits = (softmax(z) - onehot(label)) / n   (may alias logits: in place).
 * labels: int32 dev array of n entries in [0, C); out-of-range labels are not detected.
 * loss_dev: one fp32 on the device.  Workspace: mggcn_softmax_ce_workspace_bytes(n). */
size_t mggcn_softmax_ce_workspace_bytes(int64_t n);

int mggcn_softmax_ce(int64_t n, int32_t C, const float* logits /*dev*/, int64_t ld,
                     const int32_t* labels /*dev*/, float* loss_dev, float* dlogits /*dev*/,
                     int64_t ldd, void* ws, size_t ws_bytes, void* stream);

/* For callers that cannot allocate or hand over device memory at the point of the call -- code under
 * HIP graph capture, tight serving or training loops, harnesses that forbid hipMalloc: the same loss
 * and gradient as mggcn_softmax_ce (same kernels, same bits), with the loss partials in a 16 KiB
 * buffer that is part of the library's device code instead of a caller workspace.  The call makes no
 * hipMalloc / hipFree and uses no allocating routine; it only enqueues two kernels on `stream`.
 * Limits: n <= MGGCN_SOFTMAX_CE_STATIC_MAX_ROWS (MGGCN_E_UNSUPPORTED beyond; that many rows already
 * fill the buffer's 4096 partials many times over).  Every call on one GPU uses that GPU's one
 * buffer, which keeps the previous call's contents (each call overwrites the partials it then
 * reads): calls that overlap in time on one GPU race -- keep them on one stream or order them with
 * events.  The first call on a GPU looks up the buffer's address (hipGetSymbolAddress, no
 * allocation): make that one outside any stream capture. */
#define MGGCN_SOFTMAX_CE_STATIC_MAX_ROWS ((int64_t)1 << 40)
int mggcn_softmax_ce_static(int64_t n, int32_t C, const float* logits /*dev*/, int64_t ld,
                            const int32_t* labels /*dev*/, float* loss_dev, float* dlogits /*dev*/,
                            int64_t ldd, void* stream);

/* Adam update of one dense parameter array (the optimiser the paper trains with; it states no
 * hyper-parameters, so they are arguments).  step counts from 1.  All arrays dev, `count` fp32
 * elements, updated in place:
 *   m <- beta1 m + (1-beta1) g ;  v <- beta2 v + (1-beta2) g^2
 *   W <- W - lr (m / (1-beta1^step)) / (sqrt(v / (1-beta2^step)) + eps)
 * Not part of mggcn_epoch (the benchmarked epoch is forward + backward). */
int mggcn_adam_step(int64_t count, float* W, const float* G, float* m, float* v, int32_t step, float lr,
                    float beta1, float beta2, float eps, void* stream);

/* ------------------------------------------------------------------------------------------
 * Model handle: L GCN layers H^(l+1) = relu( A^ H^(l) W^(l) ) (no ReLU after the last layer,
 * whose output are the logits), the per-layer order decision and the activation buffer plan
 * (section "Memory Optimizations"): one result buffer per layer plus one temporary shared
 * by all layers, carved from a caller-provided arena.  A layer that runs SpMM first also
 * keeps its A^ H product for the backward pass (one more buffer for that layer).
 *
 * dims: host array of L+1 widths d_0..d_L.  orders: host array of L mggcn_order values or
 * NULL (= AUTO everywhere).  The graph must be square, bound with F_max >= every SpMM
 * width the model needs (mggcn_model_spmm_width_max), and outlive the model.  Calls on one model
 * use its arena (and its graph's tables): keep them on one stream.
 * ---------------------------------------------------------------------------------------- */
typedef struct mggcn_model mggcn_model;

/* Model flags.
 * MGGCN_MODEL_CACHE_INPUT: the input features X do not change between epochs, so A^ X is formed
 * once (mggcn_model_cache_input) and kept in the arena; the first layer then runs as
 * relu((A^ X) W) forward and W_G = (A^ X)^T Z_G backward with no SpMM at all in either pass --
 * the exact form of the paper's "saving one SpMM" (section "Order of Computation and Saving one
 * SpMM").  Costs one n x d_0 buffer.  mggcn_layer_bwd(l = 0) of such a model takes H_G = NULL only
 * (MGGCN_E_INVALID_ARG otherwise): the shared temporary is not sized for the gradient of X.
 * MGGCN_MODEL_GATHER_BF16 (beyond the paper, which is fp32 throughout): every SpMM of the model
 * gathers a bfloat16 copy of its dense operand, made by mggcn_f32_to_bf16 just before the product
 * (see mggcn_spmm_bf16); GeMMs, activations, loss and all accumulation stay fp32.  The backward
 * pass treats the rounding as the identity.  Costs one n x (widest SpMM) 2-byte buffer.
 * MGGCN_MODEL_GEMM_BF16X3 (beyond the paper): every GeMM of the model runs as mggcn_gemm_bf16x3,
 * i.e. on the bfloat16 matrix instructions at fp32 accuracy. */
enum { MGGCN_MODEL_CACHE_INPUT = 1, MGGCN_MODEL_GATHER_BF16 = 2, MGGCN_MODEL_GEMM_BF16X3 = 4 };

int mggcn_model_create(const mggcn_graph* g, int32_t L, const int32_t* dims /*host*/,
                       const int32_t* orders /*host or NULL*/, int32_t flags, mggcn_model** out);
int mggcn_model_destroy(mggcn_model* m);
int32_t mggcn_model_spmm_width_max(const int32_t* dims /*host*/, const int32_t* orders, int32_t L,
                                   int32_t flags);
/* With MGGCN_MODEL_CACHE_INPUT: compute and keep A^ X (one SpMM of width d_0).  Call after
 * mggcn_model_bind and again whenever X changes; mggcn_epoch / mggcn_layer_fwd(l = 0) fail with
 * MGGCN_E_INVALID_ARG until it has been called, and afterwards ignore their X / H_in argument
 * for the first layer. */
int mggcn_model_cache_input(mggcn_model* m, const float* X /*dev*/, int64_t ldx, void* stream);
size_t mggcn_model_arena_bytes(const mggcn_model* m);
int mggcn_model_bind(mggcn_model* m, void* arena /*dev*/, size_t arena_bytes);
/* resolved order of layer l (mggcn_order), or a negative status */
int mggcn_model_order(const mggcn_model* m, int32_t l);
/* device pointer and leading dimension of layer l's result buffer (its output H^(l+1),
 * later overwritten in place by the gradient with respect to it) */
int mggcn_model_activation(const mggcn_model* m, int32_t l, float** ptr_out, int64_t* ld_out);
/* With MGGCN_MODEL_GATHER_BF16: device pointer of the buffer that holds the bfloat16 operand of
 * the most recent SpMM, and the leading dimension it has for an operand `width` columns wide
 * (tests read the operand back between mggcn_layer_fwd / mggcn_layer_bwd calls). */
int mggcn_model_gather_operand(const mggcn_model* m, int32_t width, uint16_t** ptr_out, int64_t* ld_out);

/* One layer forward (Eq. 5-7): H_out = [relu]( A^ H_in W ).  H_in is n x d_l, W is
 * d_l x d_{l+1}, H_out is n x d_{l+1}; relu != 0 applies Eq. 7.  Uses the model's shared
 * temporary (and, SpMM-first, stores A^ H_in in the layer's own buffer).  With
 * MGGCN_MODEL_CACHE_INPUT, l = 0 ignores H_in (may be NULL) and works from the stored A^ X. */
int mggcn_layer_fwd(mggcn_model* m, int32_t l, const float* H_in, int64_t ld_in, const float* W,
                    int64_t ldw, int relu, float* H_out, int64_t ld_out, void* stream);

/* One layer backward (Eq. 8-11).  On entry G (n x d_{l+1}) holds the gradient with respect
 * to the layer output H_out.  If act != NULL, Eq. 8 is applied first: G <- G where act > 0
 * (pass the layer's saved output; NULL means G is already the gradient of the pre-activation).
 * Then  W_G = H_in^T (A^^T G)   (d_l x d_{l+1}, Eq. 9-10)
 *       H_G = (A^^T G) W^T      (n x d_l,      Eq. 11)      unless H_G == NULL.
 * hg_relu_mask != 0: the H_G buffer currently holds the previous layer's output H^(l) and
 * receives H_G masked by (H^(l) > 0) in place, i.e. Eq. 8 of the layer below fused in; H_G
 * may then be the same buffer as H_in.  Must follow mggcn_layer_fwd(m, l, same H_in) when the
 * layer runs SpMM first (it reuses the stored A^ H_in).  G is preserved except for the mask. */
int mggcn_layer_bwd(mggcn_model* m, int32_t l, const float* H_in, int64_t ld_in,
                    const float* act /*or NULL*/, int64_t ld_act, float* G, int64_t ldg,
                    const float* W, int64_t ldw, float* W_G, int64_t ldwg, float* H_G /*or NULL*/,
                    int64_t ldhg, int hg_relu_mask, void* stream);

/* One training epoch without the optimiser step: L x layer_fwd, softmax-CE, L x layer_bwd.
 * Only enqueues kernels on `stream` (no allocation, copy, memset or synchronisation), so the call
 * may be captured in a HIP graph and replayed.
 * X: n x d_0 (ld ldx).  labels: n int32.  W / W_G: host arrays of L device pointers, W[l]
 * and W_G[l] dense d_l x d_{l+1} (ld = d_{l+1}).  loss_dev: one fp32 on the device.  No
 * gradient with respect to X is formed; the first layer's backward SpMM is kept whenever
 * W_G needs it (GeMM-first order) and absent otherwise.  With MGGCN_MODEL_CACHE_INPUT, X is
 * ignored (may be NULL): the first layer works from the stored A^ X. */
int mggcn_epoch(mggcn_model* m, const float* X, int64_t ldx, const int32_t* labels,
                const float* const* W /*host array of dev ptrs*/, float* loss_dev,
                float* const* W_G /*host array of dev ptrs*/, void* stream);

/* ------------------------------------------------------------------------------------------
 * Memory-system probes -- measurement aids, not part of the training path.  The benchmark runs them
 * next to the SpMM (Eq. 6, 9) so that its rate can be quoted against what this GPU delivers for
 * the SpMM's two access patterns, beside the datasheet bandwidth.
 * `sink` (dev) receives one fp32 per workgroup: room for mggcn_probe_sink_floats() entries.
 *   _read:   reads `bytes` (a multiple of 16) from buf (dev, 16-byte aligned) once, contiguously.
 *   _write:  fills `bytes` (a multiple of 16) of buf (dev, 16-byte aligned) with `value`, contiguously.
 *   _gather: for k in [0, n_idx): reads row idx[k] (row_bytes = 64 .. 1024, a power of two) of the
 *            n_rows x row_stride-byte matrix X (dev, 16-byte aligned; row_stride a multiple of 16),
 *            eight rows in flight per lane.  idx: int32 dev; an index outside [0, n_rows) is read
 *            as row n_rows - 1.
 *   _mfma:   512 workgroups issue `iters` x 32 v_mfma_f32_32x32x2_f32 per wavefront on register
 *            operands; returns the number of floating-point operations enqueued (or a negative
 *            status), for the caller to divide by the time it measures.
 * ---------------------------------------------------------------------------------------- */
int32_t mggcn_probe_sink_floats(void);
int mggcn_probe_write(void* buf /*dev*/, int64_t bytes, float value, void* stream);
int64_t mggcn_probe_mfma(int32_t iters, float* sink /*dev*/, void* stream);
int mggcn_probe_read(const void* buf /*dev*/, int64_t bytes, float* sink /*dev*/, void* stream);
int mggcn_probe_gather(const void* X /*dev*/, int64_t n_rows, int32_t row_bytes, int64_t row_stride,
                       const int32_t* idx /*dev*/, int64_t n_idx, float* sink /*dev*/, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* MGGCN_H_ */
