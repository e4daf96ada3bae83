/*
 * blast.h -- C ABI of the MI355X (gfx950) block-sparse MLP library.
 *
 * The library implements the hot path of BLaST (arxiv 2507.03117): block-norm
 * pruning + packing of a weight matrix into a block-compressed format
 * (Sec. 3.2, Sec. 3.4.1), the block-sparse matrix product built on it
 * (Sec. 3.4, Listing 2) and the fused block-sparse SwiGLU MLP (Eq. (1),
 * Sec. 3.4.3).  Around that path it also holds the two-matrix MLP of the
 * GPT-2 family (Sec. 4), the two backward products of a block-sparse weight
 * (Sec. 3.2, Sec. 3.4.1), the mask update of the prune-and-grow step with its sparsity
 * schedule (Sec. 3.2: Listing 1 and Eq. (2)), the pooled top-k mask used for
 * post-training sparsification (Sec. 3.3) and the product on 8-bit E5M2
 * operands (Sec. 5.2).
 *
 * Conventions
 *  - Weights are `out x in`, row-major, like a linear layer's weight: W is
 *    rows x cols and the product is Y = W * X with X: cols x T, Y: rows x T.
 *    The paper writes Y = X W with W `in x out` stored BCSC; BSR of the
 *    `out x in` matrix is the same object (each block transposed), and the
 *    paper notes the two orientations are mirror images (Sec. 3.4.1).
 *  - bf16 values travel as uint16_t bit patterns.
 *  - Unless a parameter says HOST, every pointer is a DEVICE pointer into memory
 *    owned by the caller.  The library never allocates or frees device memory
 *    and only enqueues work on the given stream (`stream` is a hipStream_t
 *    passed as void*; NULL = the default stream).
 *  - State the library keeps for the life of the process: a counter that hands
 *    every single-launch MLP call its own 64-bit token; per-device caches of the
 *    compute-unit count, of which kernels have had their dynamic-LDS limit raised
 *    and of the address of the scratch array below (all atomics: host threads may
 *    race on them); one small pinned host buffer per host thread that has called
 *    blast_bsr_pack (hipHostMalloc, never freed); the last HIP error text per
 *    host thread; and, on every GPU the library is loaded on, the device array of
 *    BLAST_STATIC_SCRATCH_BYTES behind blast_sparse_mlp_static.
 *  - Every call returns 0 (BLAST_OK) or a negative error code.  Argument errors
 *    (INVALID_ARG, SHAPE, UNSUPPORTED_BLOCK, WORKSPACE) are found before anything
 *    is enqueued.  BLAST_ERR_HIP can come from any launch of a call that enqueues
 *    several (the two products of the MLP, the token ranges of a very long
 *    activation, the packer's passes): the launches before it stay enqueued and
 *    the outputs are then undefined.  BLAST_ERR_CAPACITY: see blast_bsr_pack.
 *  - Buffers must stay alive and unmodified until the stream has executed the
 *    enqueued work.  Calls on distinct streams may run concurrently from
 *    different host threads as long as their output/workspace buffers differ.
 */
#ifndef BLAST_H_
#define BLAST_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* ---- error codes ------------------------------------------------------- */
#define BLAST_OK 0
#define BLAST_ERR_INVALID_ARG (-1)       /* null pointer, negative size, ld too small, bad enum, misalignment */
#define BLAST_ERR_SHAPE (-2)             /* rows/cols not a multiple of b; MLP matrices inconsistent */
#define BLAST_ERR_UNSUPPORTED_BLOCK (-3) /* block size outside {16, 32, 64, 128} */
#define BLAST_ERR_CAPACITY (-4)          /* nnz_cap smaller than the number of kept blocks */
#define BLAST_ERR_WORKSPACE (-5)         /* workspace / aux buffer missing or too small */
#define BLAST_ERR_HIP (-6)               /* HIP runtime error; text via blast_strerror */

/* ---- enums -------------------------------------------------------------- */
#define BLAST_PACK_MASK 0           /* keep exactly the blocks flagged in block_mask */
#define BLAST_PACK_TOPK_FROBENIUS 1 /* keep the highest-Frobenius-norm blocks (Sec. 3.2) */

#define BLAST_TOKEN_MAJOR 0   /* element (k, t) at X[t*ld + k]: the [tokens, features] activation tensor */
#define BLAST_FEATURE_MAJOR 1 /* element (k, t) at X[k*ld + t] */
#define BLAST_COLUMN_GROUPS_64 2 /* E5M2 activations only: element (k, t) at X8[((k/64)*T + t)*64 + k%64], written by
                                   blast_quantize_e5m2_groups; ld is ignored */

#define BLAST_F32 0
#define BLAST_BF16 1

#define BLAST_ACT_SILU 0 /* x * sigmoid(x), Eq. (1) */
#define BLAST_ACT_GELU 1 /* x/2 * (1 + erf(x / sqrt 2)) */
#define BLAST_ACT_RELU 2

/*
 * Packed block-sparse matrix (Sec. 3.2: the pruned weight W_new in block
 * compressed form; Sec. 3.4.1).  A plain view: all arrays are caller-owned
 * device memory; the struct itself is host memory and is read at call time.
 */
typedef struct blast_bsr_view {
  int64_t rows, cols;       /* logical size; both multiples of b */
  int32_t b;                /* block edge: 16, 32, 64 or 128 */
  int32_t max_row_blocks;   /* stored blocks of the fullest block row, as reported by blast_bsr_pack;
                               0 = unknown (rows are then never split into chunks) */
  int64_t nnz;              /* number of stored blocks */
  const int32_t* row_ptr;   /* [rows/b + 1], row_ptr[0] = 0, non-decreasing, row_ptr[rows/b] = nnz */
  const int32_t* col_idx;   /* [nnz], block-column of each stored block, strictly ascending inside a block row */
  const uint16_t* vals;     /* [nnz * b * b] bf16, block k occupies vals[k*b*b ..], row-major inside the block;
                               must be 16-byte aligned */
  const int32_t* row_order; /* [rows/b] block rows by stored-block count, descending (schedule); may be NULL */
  const void* aux;          /* chunk plan + column-grouped index written by blast_bsr_pack
                               (blast_bsr_aux_bytes bytes); may be NULL: rows are then never split */
} blast_bsr_view;

/* Human-readable text for an error code.  For BLAST_ERR_HIP the text of the
 * last HIP error seen by the calling thread is appended.  Never NULL. */
const char* blast_strerror(int code);

/* Number of blocks kept for a target sparsity over n_blocks blocks (Sec. 3.2: the
 * lowest-scoring blocks are removed until the zero fraction reaches s): the drop count
 * is ceil(s * n_blocks) with s taken in basis points, s_bp = round(s * 1e4),
 * n_zero = ceil(s_bp * n_blocks / 1e4).  Returns -1 if sparsity is outside [0, 1]
 * or n_blocks < 0.  Pure host arithmetic. */
int64_t blast_n_keep(int64_t n_blocks, double sparsity);

/* Bytes of the `aux` buffer for a matrix with the given block grid and capacity. */
size_t blast_bsr_aux_bytes(int64_t rows, int64_t cols, int32_t b, int64_t nnz_cap);

/*
 * Sizes needed by blast_bsr_pack (all outputs HOST pointers, any may be NULL).
 *   nnz_cap   : TOPK -> exactly blast_n_keep(); MASK -> (rows/b)*(cols/b), the upper bound
 *               (a caller that knows its mask's population may allocate less).
 *   aux_bytes : blast_bsr_aux_bytes() for that nnz_cap.
 *   ws_bytes  : scratch needed during the call.
 * Errors: INVALID_ARG, SHAPE, UNSUPPORTED_BLOCK.
 */
int blast_bsr_pack_bound(int64_t rows, int64_t cols, int32_t b, int32_t mode, double sparsity,
                         int64_t* nnz_cap, size_t* aux_bytes, size_t* ws_bytes);

/*
 * Prune and pack a dense bf16 weight (Sec. 3.2 generate_masks() pruning half +
 * prune_weights(); Sec. 3.4.1 storage format).
 *
 *   W, ldw      dense weight, element (i, j) at W[i*ldw + j]; ldw >= cols, ldw % 8 == 0, W 16-byte aligned.
 *   mode        BLAST_PACK_MASK: block_mask [rows/b][cols/b] uint8 (nonzero = keep) is the structure;
 *               a kept block is stored even when all its values are zero; the value 2 marks a regrown
 *               block (Sec. 3.2), which is stored as zeros whatever W holds there.
 *               BLAST_PACK_TOPK_FROBENIUS: block_mask is ignored (may be NULL).  Each block is scored by
 *               its squared Frobenius norm accumulated in fp64; the blast_n_keep() highest are kept;
 *               equal scores are ordered by linear block index (block_row * (cols/b) + block_col), lower
 *               first.  Weights must be finite.
 *   sparsity    target fraction of dropped blocks in [0, 1] (TOPK only).
 *   row_ptr     out [rows/b + 1]
 *   col_idx     out [nnz_cap]
 *   vals        out [nnz_cap * b * b], 16-byte aligned
 *   row_order   out [rows/b]: stable sort of block rows by stored-block count, descending (empty rows last)
 *   aux         out, aux_bytes >= blast_bsr_aux_bytes(rows, cols, b, nnz_cap), 16-byte aligned; may be NULL
 *               (then neither the chunk plan nor the column-grouped index is produced)
 *   nnz_out     HOST, receives the number of stored blocks (also on BLAST_ERR_CAPACITY)
 *   max_row_blocks_out  HOST, may be NULL: stored blocks of the fullest block row (0 without aux).  Copy it
 *               into blast_bsr_view.max_row_blocks: with `aux`, block rows of more than 16 blocks are cut into
 *               chunks of 16 (and, in a second plan for the many-token kernels, rows of more than 64 blocks
 *               into chunks of 64), and the product schedules chunks instead of rows when that row would
 *               otherwise be the critical path of the launch (the load balance Sec. 3.4.1 asks of the
 *               launch grid).
 *   ws          scratch of at least the ws_bytes reported by blast_bsr_pack_bound, 16-byte aligned
 *
 * The call enqueues all its work and then synchronises `stream` once (to return nnz and max_row_blocks): when
 * it returns, the outputs are complete and ws may be reused.
 * Errors: INVALID_ARG, SHAPE, UNSUPPORTED_BLOCK, WORKSPACE, CAPACITY (row_ptr and row_order are complete,
 * col_idx/vals hold the first nnz_cap blocks, the column-grouped index in aux has not been written), HIP.
 */
int blast_bsr_pack(const uint16_t* W, int64_t ldw, int64_t rows, int64_t cols, int32_t b, int32_t mode,
                   const uint8_t* block_mask, double sparsity, int32_t* row_ptr, int32_t* col_idx, uint16_t* vals,
                   int32_t* row_order, void* aux, size_t aux_bytes, int64_t nnz_cap, int64_t* nnz_out,
                   int32_t* max_row_blocks_out, void* ws, size_t ws_bytes, void* stream);

/*
 * blast_bsr_pack without the synchronisation, for re-packing many matrices in a row (Sec. 3.2: every
 * step_size iterations the masks of all layers are regenerated and all weights are packed again).  Same
 * arguments and outputs, except:
 *   result      out [2] int32, 8-byte aligned, DEVICE: {number of stored blocks, stored blocks of the fullest
 *               block row (0 without aux)}; the caller reads it after synchronising, once for all matrices.
 * Only enqueues kernels (no copies, no memsets): the call can be recorded into a HIP graph and replayed on a
 * weight whose values change.  ws belongs to the call until the stream has passed its work; calls on the same stream may
 * share one ws (the larger of their sizes).  When result[0] > nnz_cap the outputs are as blast_bsr_pack
 * leaves them on BLAST_ERR_CAPACITY.  Errors: INVALID_ARG, SHAPE, UNSUPPORTED_BLOCK, WORKSPACE, HIP.
 */
int blast_bsr_pack_enqueue(const uint16_t* W, int64_t ldw, int64_t rows, int64_t cols, int32_t b, int32_t mode,
                           const uint8_t* block_mask, double sparsity, int32_t* row_ptr, int32_t* col_idx,
                           uint16_t* vals, int32_t* row_order, void* aux, size_t aux_bytes, int64_t nnz_cap,
                           int32_t* result, void* ws, size_t ws_bytes, void* stream);

/*
 * Dense form of a packed matrix: the pruned weight W_new that prune_weights() applies in the training loop of
 * Sec. 3.2 (stored blocks copied to their places, zeros everywhere else; regrown blocks are zeros by
 * construction).  The inverse of blast_bsr_pack on the kept blocks.
 *   W, ldw      out, bf16 [rows][cols], row pitch ldw >= cols, ldw % 8 == 0, 16-byte aligned; fully overwritten
 * Never synchronises.  Errors: INVALID_ARG, SHAPE, UNSUPPORTED_BLOCK, HIP.
 */
int blast_bsr_unpack(const blast_bsr_view* Wp, uint16_t* W, int64_t ldw, void* stream);

/*
 * One mask update of blocked prune-and-grow (Sec. 3.2, the generate_masks() step of the training loop):
 *   S(W) = the blocks of W kept at `sparsity` by block Frobenius norm (same count, ranking and tie rule as
 *          BLAST_PACK_TOPK_FROBENIUS), S(G) = the same selection on the gradient G, D = S(G) \ S(W).
 *   mask_out[block] = 1 for S(W), 2 for D (regrown: kept in the structure, values start at zero), 0 otherwise.
 * Feeding mask_out to blast_bsr_pack in BLAST_PACK_MASK mode packs W_new: blocks with code 2 are stored as
 * zeros, so they do not change the current product.
 *   W, G        bf16 [rows][cols], row pitches ldw / ldg (multiples of 8), 16-byte aligned
 *   mask_out    out, uint8 [rows/b][cols/b]
 *   ws          at least blast_generate_masks_workspace(rows, cols, b) bytes, 16-byte aligned
 * Never synchronises.  Errors: INVALID_ARG, SHAPE, UNSUPPORTED_BLOCK, WORKSPACE, HIP.
 */
int blast_generate_masks(const uint16_t* W, int64_t ldw, const uint16_t* G, int64_t ldg, int64_t rows, int64_t cols,
                         int32_t b, double sparsity, uint8_t* mask_out, void* ws, size_t ws_bytes, void* stream);
size_t blast_generate_masks_workspace(int64_t rows, int64_t cols, int32_t b);

/*
 * Eq. (2): sparsity at training iteration i,  s(i) = s_max + (s_init - s_max) * (1 - i / (m - d))^3,
 * with i held inside [0, m - d] (the paper gives no value past m - d, where the cube would exceed s_max).
 * Host arithmetic only.
 */
double blast_sparsity_schedule(int64_t i, int64_t m, int64_t d, double s_init, double s_max);

/*
 * Block selection from a sensitivity matrix (Sec. 3.3): S holds one fp32 sensitivity per weight; a block's
 * score is the 2D average pooling (mean) of its b x b entries, accumulated in fp64; the blast_n_keep()
 * highest-scoring blocks are kept, equal scores ordered by linear block index, lower first (the rule of
 * BLAST_PACK_TOPK_FROBENIUS).  Sensitivities may have any sign but must be finite.  How S is computed
 * (curvature estimates, gradients) is the caller's business.
 *   S, lds      fp32 [rows][cols], row pitch lds (multiple of 4), 16-byte aligned
 *   mask_out    out, uint8 [rows/b][cols/b], 1 = keep; feed it to blast_bsr_pack in BLAST_PACK_MASK mode
 *   ws          at least blast_pooled_topk_mask_workspace(rows, cols, b) bytes, 16-byte aligned
 * Never synchronises.  Errors: INVALID_ARG, SHAPE, UNSUPPORTED_BLOCK, WORKSPACE, HIP.
 */
int blast_pooled_topk_mask(const float* S, int64_t lds, int64_t rows, int64_t cols, int32_t b, double sparsity,
                           uint8_t* mask_out, void* ws, size_t ws_bytes, void* stream);
size_t blast_pooled_topk_mask_workspace(int64_t rows, int64_t cols, int32_t b);

/*
 * E5M2 (8-bit floating point; Sec. 5.2 reports the kernel in float8_e5m2 next to the 16-bit types).
 * E5M2 = 1 sign, 5 exponent (bias 15), 2 mantissa bits, subnormals / infinities / NaN as in IEEE half
 * precision, of which a code is the upper byte.
 *
 * blast_quantize_e5m2: out[i] = E5M2(in[i]) for bf16 input, round to nearest with ties to the even
 * mantissa, magnitudes of 61440 and above become infinity.  Serves the block values of a packed matrix
 * (W->vals, nnz*b*b values: the structure arrays are shared with the bf16 form) and activations alike.
 * Never synchronises.  Errors: INVALID_ARG, HIP.
 *
 * blast_quantize_e5m2_groups: the same conversion for a token-major bf16 activation X[T][K] (row pitch ldx
 * elements, K a multiple of 64), written in column groups of 64 features: out[((k/64)*T + t)*64 + k%64], T*K bytes,
 * 16-byte aligned.  In this layout a token's share of a 64-wide contraction slice and the next token's are one
 * 128-byte line, which is what the product kernel's copies fetch (token-major E5M2 rows give it half a line per
 * token: an MI355X layout choice, not the paper's).  Never synchronises.  Errors: INVALID_ARG, HIP.
 *
 * blast_bsr_spmm_e5m2: Y = W~ X as in blast_bsr_spmm with both operands in E5M2 and fp32 accumulation.
 *   W          structure of the packed matrix (row_ptr, col_idx, row_order, aux, max_row_blocks, nnz, b;
 *              W->vals is not read).  With fp32 output and few tokens, rows much longer than a chunk are
 *              accumulated with atomic additions, as in blast_bsr_spmm.
 *   vals8      E5M2 block values, [W->nnz][b][b], one byte each, same order as W->vals
 *   X8, ldx    E5M2 activations, [T][cols] (token-major) or [cols][T], row pitch ldx bytes; or
 *              BLAST_COLUMN_GROUPS_64 (b >= 64, X8 16-byte aligned, ldx ignored)
 *   Y, ldy     as in blast_bsr_spmm (fp32 or bf16, same layout as X8; token-major for column groups)
 * The tuned kernel needs b >= 64, token-major operands, 16-byte aligned pointers and ldx % 16 == 0; other
 * cases take a plain kernel.  Never synchronises, allocates nothing.
 * Errors: INVALID_ARG, SHAPE, UNSUPPORTED_BLOCK, HIP.
 */
int blast_quantize_e5m2(const uint16_t* in_bf16, int64_t n, uint8_t* out, void* stream);
int blast_quantize_e5m2_groups(const uint16_t* X_bf16, int64_t ldx, int64_t T, int64_t K, uint8_t* out, void* stream);
int blast_bsr_spmm_e5m2(const blast_bsr_view* W, const uint8_t* vals8, const uint8_t* X8, int64_t ldx, int32_t x_layout,
                        int64_t T, void* Y, int64_t ldy, int32_t y_dtype, void* stream);

/*
 * Fused gated MLP with the three weights stored in E5M2 (Sec. 5.2 reports the kernel in float8_e5m2; at decode
 * token counts the pass is bound by reading the stored blocks once, and one byte per weight halves those
 * bytes).  Activations and the intermediate stay in bf16:
 *   G = W~gate X, U = W~up X with every E5M2 code widened exactly to bf16, fp32 accumulation;
 *   H = bf16(act(G) * U), one rounding; Y = W~down H, fp32 accumulation (Eq. (1)).
 * That is blast_sparse_mlp on the dequantised weights, with half the weight traffic.
 *   Wgate/Wup/Wdown   structure of the packed matrices (row_ptr, col_idx, row_order, aux, max_row_blocks, nnz, b; vals is
 *                     not read);
 *                     b = 64 or 128
 *   gate8/up8/down8   E5M2 block values, [nnz][b][b], one byte each, in the order of the view's vals
 *                     (blast_quantize_e5m2 of it), 16-byte aligned
 *   X, ldx            token-major bf16 activations [T][E], ldx % 8 == 0, 16-byte aligned; T * ldx * 2 and
 *                     T * I * 2 below 2^32 (the call is meant for decode token counts; any such T is correct)
 *   Y, ldy, y_dtype   token-major [T][E], fp32 or bf16
 *   ws                at least blast_sparse_mlp_e5m2w_workspace() bytes (H), 256-byte aligned
 * Two launches, no in-kernel hand-over; with fp32 output a very full row of Wdown (see max_row_blocks) is cut
 * into chunks that add into cleared rows, as in blast_bsr_spmm.  Never synchronises.
 * Errors: INVALID_ARG, SHAPE, UNSUPPORTED_BLOCK (b other than 64 / 128), WORKSPACE, HIP.
 */
int blast_sparse_mlp_e5m2w(const blast_bsr_view* Wgate, const uint8_t* gate8, const blast_bsr_view* Wup,
                           const uint8_t* up8, const blast_bsr_view* Wdown, const uint8_t* down8, const uint16_t* X,
                           int64_t ldx, int64_t T, int32_t act, void* Y, int64_t ldy, int32_t y_dtype, void* ws,
                           size_t ws_bytes, void* stream);
int blast_sparse_mlp_e5m2w_workspace(const blast_bsr_view* Wgate, int64_t T, size_t* ws_bytes /* HOST */);

/*
 * Packed transpose.  Sec. 3.2: the pruned matrix is the one used in forward AND backward propagation;
 * Sec. 3.4 / 3.4.1: which compressed format suits depends on the side the sparse matrix is multiplied
 * from, and the kernel for the other side is the symmetric one.  This call builds, from a packed W~
 * (rows x cols), the packed W~^T (cols x rows): the same stored blocks grouped by block column, every
 * block turned.  The backward product with respect to the activations,
 *     dX = W~^T dY,
 * is then blast_bsr_spmm on the result (dY in the place of X, [T][rows] token-major or [rows][T]).
 *
 *   W                 a packed matrix WITH its aux buffer (the column-grouped index is read from it).
 *   row_ptr_t         out, [cols/b + 1]
 *   col_idx_t         out, [W->nnz]   block-row indices of W, ascending inside each block column
 *   vals_t            out, [W->nnz * b * b], 16-byte aligned; block e = transpose of the e-th block of W in
 *                     column-grouped order
 *   row_order_t       out, [cols/b]   schedule of the transpose (block columns of W by population)
 *   aux_t             out, may be NULL; at least blast_bsr_aux_bytes(cols, rows, b, W->nnz) bytes
 *   max_row_blocks_t_out  HOST, may be NULL: stored blocks of the fullest block column of W (0 without
 *                     aux_t); goes into the view's max_row_blocks.  Asking for it makes the call wait for
 *                     `stream` (one small copy); otherwise the call never synchronises.
 * Errors: INVALID_ARG, SHAPE, UNSUPPORTED_BLOCK, WORKSPACE (W->aux missing, aux_t too small), HIP.
 */
int blast_bsr_transpose(const blast_bsr_view* W, int32_t* row_ptr_t, int32_t* col_idx_t, uint16_t* vals_t,
                        int32_t* row_order_t, void* aux_t, size_t aux_t_bytes, int32_t* max_row_blocks_t_out /* HOST */,
                        void* stream);

/*
 * Gradient of the stored blocks (Sec. 3.2: the backward pass uses the same sparsity pattern; a dropped
 * block holds no weight and receives no gradient).  With Y = W~ X:
 *     dvals[q][i][j] = sum_t dY(r*b + i, t) * X(c*b + j, t)      for the q-th stored block, at (r, c),
 * the entries of dY X^T that fall on kept blocks, in the storage order of W->vals.  bf16 operands, fp32
 * accumulation, fp32 result.  Only the structure of W is read (row_ptr, col_idx, nnz), not its values.
 *
 *   dY, X, layout     BLAST_TOKEN_MAJOR: dY is [T][rows] with row pitch ldy, X is [T][cols] with pitch ldx
 *                     (the tuned path needs b >= 32, both 16-byte aligned with pitches that are multiples
 *                     of 8); BLAST_FEATURE_MAJOR: [rows][T] / [cols][T].  Other cases take a plain kernel.
 *   dvals             out, fp32 [W->nnz][b][b], 16-byte aligned; overwritten.  T = 0 gives zeros.
 * When the matrix has few blocks the tokens are cut into chunks whose partial sums meet through fp32
 * atomic additions: the result is then reproducible only up to the rounding of the summation order.
 * Never synchronises, allocates nothing.  Errors: INVALID_ARG, SHAPE, UNSUPPORTED_BLOCK, HIP.
 */
int blast_bsr_sddmm(const blast_bsr_view* W, const uint16_t* dY, int64_t ldy, const uint16_t* X, int64_t ldx,
                    int32_t layout, int64_t T, float* dvals, void* stream);

/*
 * Schedule for two matrices that are multiplied together row by row (W_gate and W_up of Eq. (1)):
 * row_order[rank] = block rows sorted by the SUM of their stored-block counts, descending, stable.
 * Passing it as Wgate->row_order lets the gated product balance its workgroups on the work they really
 * do (Sec. 3.4.1 derives the launch grid from the stored blocks for the same reason).  A and B must have the
 * same number of rows and the same block size.  row_order: out, [rows/b].  Enqueues one small kernel;
 * never synchronises.  Errors: INVALID_ARG, SHAPE, UNSUPPORTED_BLOCK, HIP.
 */
int blast_bsr_joint_row_order(const blast_bsr_view* A, const blast_bsr_view* B, int32_t* row_order, void* stream);

/*
 * Block-sparse product Y = W * X (Sec. 3.4, Listing 2: for every output tile,
 * loop over the stored blocks of its block row, load the block and the matching
 * slice of X through the index array, accumulate).  bf16 x bf16 products,
 * fp32 accumulation.  Rows of an empty block row are written as zeros.
 *
 *   X, ldx, x_layout   activation, cols x T, layout per BLAST_TOKEN_MAJOR / BLAST_FEATURE_MAJOR.
 *                      The fast path needs TOKEN_MAJOR, ldx % 8 == 0 and X 16-byte aligned; other
 *                      inputs are handled by a slower load path with identical results.
 *   T                  number of tokens (columns of X), >= 0; T == 0 is a no-op.
 *   Y, ldy, y_dtype    output rows x T in the SAME layout as X; fp32 (BLAST_F32) or bf16 (BLAST_BF16,
 *                      rounded to nearest even from the fp32 accumulator).
 *   ws, ws_bytes       scratch of blast_bsr_spmm_workspace() bytes, 16-byte aligned.  Nonzero only for 16 x 16
 *                      blocks from 33 tokens on: there the activations are first regrouped by block column
 *                      ([cols/16][T][16], so that the 16 tokens x 16 features a block multiplies are 512
 *                      consecutive bytes instead of 16 pieces of 32); a call with less (or NULL) reads X as it
 *                      lies, with identical results.
 * When W carries `aux` and a very full block row (see max_row_blocks), that row's chunks add their partial
 * sums into an fp32 Y with atomics in no fixed order: such rows are reproducible up to fp32 rounding of that
 * sum only (bf16 output and the gated product never take that path).
 * Never synchronises.  Errors: INVALID_ARG, SHAPE, UNSUPPORTED_BLOCK, WORKSPACE, HIP.
 */
int blast_bsr_spmm(const blast_bsr_view* W, const uint16_t* X, int64_t ldx, int32_t x_layout, int64_t T, void* Y,
                   int64_t ldy, int32_t y_dtype, void* ws, size_t ws_bytes, void* stream);
int blast_bsr_spmm_workspace(const blast_bsr_view* W, int64_t T, size_t* ws_bytes /* HOST */);

/*
 * Fused block-sparse gated MLP, Eq. (1):  Y = Wdown * ( act(Wgate * X) (.) (Wup * X) ).
 * Wgate, Wup: I x E;  Wdown: E x I;  X: E x T;  Y: E x T;  all three share one block size.
 * G = Wgate*X and U = Wup*X are accumulated in fp32 and never rounded; H = act(G)*U is
 * computed in fp32 and rounded ONCE to bf16 (nearest even) to enter the second product;
 * Y is accumulated in fp32 (Sec. 3.4.3: the nonlinearity is fused into the product kernel).
 * An empty gate or up block row gives a zero row of H; empty Wdown block rows give zero rows of Y.
 *
 *   act                BLAST_ACT_SILU (the paper's Eq. (1)), BLAST_ACT_GELU, BLAST_ACT_RELU.
 *   X / Y layout       as in blast_bsr_spmm.
 *   ws, ws_bytes       at least blast_sparse_mlp_workspace() bytes, 256-byte aligned.  Scratch: its contents
 *                      need no initialisation and mean nothing afterwards; two calls that may overlap in
 *                      time (different streams) need different workspaces.
 * Up to one token tile (T <= 32; 64 for b = 64) with token-major, 16-byte aligned X and at most 32 MB of
 * stored blocks in the three matrices the whole of Eq. (1) runs as one kernel launch: the workgroups of the second
 * product wait inside the kernel until the slices of H they read have been published by the workgroups of the first
 * (a bounded wait; should it ever expire, their output rows are NaN and blast_sparse_mlp_status reports it).  The
 * hand-over state lives in the workspace and sets itself up: the workspace still needs no initialisation.  The call
 * can be recorded into a HIP graph like any other; replays tell themselves apart through an epoch that the kernel
 * advances in the workspace.
 * Beyond 64 tokens, when Wgate or Wup carries `aux` and a block row so full that walking it alone would take
 * several times the average share of a workgroup (the load balance Sec. 3.4.1 asks for), the rows of more than
 * 16 blocks are summed chunk by chunk into fp32 scratch behind H and H's rows of those block rows are written by a
 * launch of their own, which adds a row's chunks in a fixed order (the result is reproducible, but such a row's
 * fp32 sums are rounded differently from a row walked in one piece); blast_sparse_mlp_workspace() includes that
 * scratch exactly when the path applies, and a call handed the smaller workspace of the plain path takes the
 * plain path.
 * With 16 x 16 blocks, from 33 tokens on, blast_sparse_mlp_workspace() also includes room for X regrouped by
 * block column (see blast_bsr_spmm); H is then kept in the same form.  A call handed the smaller workspace reads
 * X as it lies.
 * Never synchronises.  Errors: INVALID_ARG, SHAPE (including inconsistent I/E/b between the three
 * matrices), UNSUPPORTED_BLOCK, WORKSPACE, HIP.
 */
int blast_sparse_mlp(const blast_bsr_view* Wgate, const blast_bsr_view* Wup, const blast_bsr_view* Wdown,
                     const uint16_t* X, int64_t ldx, int32_t x_layout, int64_t T, int32_t act, void* Y, int64_t ldy,
                     int32_t y_dtype, void* ws, size_t ws_bytes, void* stream);
int blast_sparse_mlp_workspace(const blast_bsr_view* Wgate, const blast_bsr_view* Wup, const blast_bsr_view* Wdown,
                               int64_t T, size_t* ws_bytes /* HOST */);

/*
 * Status of the in-kernel hand-over of the single-launch form (see blast_sparse_mlp) for the workspace a call
 * used: *status = 0 when every wait ended normally (or no single-launch call has used the workspace at this
 * shape), 1 when a workgroup of the second product gave up waiting for H (its output rows are NaN), 2 when
 * a wave gave up waiting for the set-up of the control block.  A nonzero status is cleared by the call.
 *   Wgate, T   the first matrix and the token count of the calls in question (they fix where the control
 *              block sits in the workspace)
 *   ws         the workspace those calls used; NULL = the library's own scratch (blast_sparse_mlp_static)
 *   status     HOST, out
 * Waits for `stream`.  Errors: INVALID_ARG, SHAPE, UNSUPPORTED_BLOCK, WORKSPACE, HIP.
 */
int blast_sparse_mlp_status(const blast_bsr_view* Wgate, int64_t T, const void* ws, size_t ws_bytes,
                            int32_t* status /* HOST */, void* stream);

/*
 * Diagnostic form of blast_sparse_mlp for testing the failure handling of the hand-over from the host, with
 * every kernel still exiting normally: `spin_limit` (>= 1) replaces the number of polls after which a wait gives
 * up, and a nonzero `withhold_publication` makes the workgroups of the first product compute H without
 * publishing it, so that every wait of the second product expires.  Outside the single-launch form the two
 * extra arguments have no effect.  Same arguments, results and errors as blast_sparse_mlp otherwise.
 */
int blast_sparse_mlp_handover_test(const blast_bsr_view* Wgate, const blast_bsr_view* Wup,
                                   const blast_bsr_view* Wdown, const uint16_t* X, int64_t ldx, int32_t x_layout,
                                   int64_t T, int32_t act, void* Y, int64_t ldy, int32_t y_dtype, void* ws,
                                   size_t ws_bytes, void* stream, int32_t spin_limit, int32_t withhold_publication);

/*
 * blast_sparse_mlp for callers that cannot allocate device memory or hand over a workspace: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments (without ws),
 * same kernels, same results and errors as blast_sparse_mlp; the scratch (H, hand-over slots, status words)
 * lives in a device array of BLAST_STATIC_SCRATCH_BYTES that the library owns: every GPU the library runs on
 * holds one such array from the moment the library is loaded until the process ends.  The call allocates and
 * frees nothing.
 *   limit   the scratch the call cannot do without - H, the hand-over slots and the status words, about
 *           2 * T * I bytes - must not exceed blast_sparse_mlp_static_limit() (= BLAST_STATIC_SCRATCH_BYTES):
 *           otherwise BLAST_ERR_WORKSPACE and nothing is enqueued.  The optional parts that
 *           blast_sparse_mlp_workspace() adds (sums of long rows, regrouped activations of 16 x 16 blocks) are
 *           used when the array has room for them and left out otherwise, as with a caller's smaller workspace.
 *           The Llama-3.2-1B-shaped layer (I = 8192) fits up to T = 2048.
 *   sharing every call on one GPU uses that GPU's one array: calls that may overlap in time on the same GPU
 *           (different streams, different host threads) race on it and must be serialised by the caller.
 *           Nothing in the array needs clearing between calls and nothing in it outlives a call.
 */
#define BLAST_STATIC_SCRATCH_BYTES ((size_t)36 << 20)
int blast_sparse_mlp_static(const blast_bsr_view* Wgate, const blast_bsr_view* Wup, const blast_bsr_view* Wdown,
                            const uint16_t* X, int64_t ldx, int32_t x_layout, int64_t T, int32_t act, void* Y,
                            int64_t ldy, int32_t y_dtype, void* stream);
size_t blast_sparse_mlp_static_limit(void);

/*
 * Two-matrix MLP (Sec. 2.1: an MLP block has two or three weight matrices; Sec. 3.4.3: two projections
 * with an element-wise nonlinearity between them, fused into the first product):
 *   H = bf16(act(W1 X)),  Y = W2 H.
 * W1 is I x E, W2 is E x I, both packed with the same block size.  Arithmetic, layouts, workspace rules,
 * the single-launch form for one token tile and errors are those of
 * blast_sparse_mlp (with W1 in the place of Wgate and no Wup); an empty block row of W1 gives a zero
 * row of H since act(0) = 0 for all three activations.
 */
int blast_sparse_mlp2(const blast_bsr_view* W1, const blast_bsr_view* W2, const uint16_t* X, int64_t ldx,
                      int32_t x_layout, int64_t T, int32_t act, void* Y, int64_t ldy, int32_t y_dtype, void* ws,
                      size_t ws_bytes, void* stream);
int blast_sparse_mlp2_workspace(const blast_bsr_view* W1, const blast_bsr_view* W2, int64_t T,
                                size_t* ws_bytes /* HOST */);

/*
 * blast_sparse_mlp with three caller-created hipEvent_t recorded on `stream`, so that a caller can
 * time the phases of Eq. (1) inside its own timed region:
 *   events[0] before the first kernel, events[1] after the kernel that finishes H = act(G) (.) U
 *   (Sec. 3.4.3), events[2] after the kernel that finishes Y.  In the single-launch form events[1] is
 *   recorded right after events[0], before the kernel.  `events` is a HOST array of 3 hipEvent_t.
 * Same arguments, results and errors as blast_sparse_mlp otherwise.
 */
int blast_sparse_mlp_events(const blast_bsr_view* Wgate, const blast_bsr_view* Wup, const blast_bsr_view* Wdown,
                            const uint16_t* X, int64_t ldx, int32_t x_layout, int64_t T, int32_t act, void* Y,
                            int64_t ldy, int32_t y_dtype, void* ws, size_t ws_bytes, void* stream,
                            void* const* events);

/*
 * The gated first half of Eq. (1) on its own (Sec. 3.4.3: the nonlinearity that follows the product is
 * fused into the product kernel):  H = act(Wgate * X) (.) (Wup * X), rounded once to bf16.
 * Wgate and Wup have the same shape and block size.  H is rows x T bf16 in the same layout as X.
 * Never synchronises.  Errors as blast_bsr_spmm.
 */
int blast_bsr_gated_spmm(const blast_bsr_view* Wgate, const blast_bsr_view* Wup, const uint16_t* X, int64_t ldx,
                         int32_t x_layout, int64_t T, int32_t act, uint16_t* H, int64_t ldh, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* BLAST_H_ */
