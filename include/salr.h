/*
 * salr.h -- C boundary of the MI355X (gfx950) library for the SALR inference linear layer
 *
 *     Y[M,N] = X[M,K] * decode(bitmap, values)[N,K]^T  +  (X[M,K] * A_cat[K,R]) * B_cat[R,N]
 *
 * (paper Sec. 3.2 for the concatenated adapters, Sec. 3.3 for the bitmap format and the
 * decode/GEMM pipeline).
 *
 * Conventions for every entry point
 *   - bf16 tensors are passed as pointers to their raw 16-bit patterns (uint16_t), row-major.
 *   - Orientation: the frozen pruned weight W-hat is [N = out features, K = in features]; the
 *     bits of one bitmap row run along K, the contraction dimension.  (The paper writes the
 *     transpose, y = xW with W in R^{d_in x d_out}.)
 *   - All data pointers are DEVICE pointers owned by the caller, 16-byte aligned at their base.
 *     The library allocates nothing, frees nothing and never synchronises: every call only
 *     enqueues kernels on `stream` (a hipStream_t passed as void*, NULL = default stream).
 *   - Arguments are validated on the host before anything is enqueued; on a non-zero status no
 *     kernel has been launched and no output has been touched.
 *   - Sizes are int64_t; a dimension of 0 is legal (SALR_OK): a call whose outputs are empty does nothing, and
 *     an empty contraction (K == 0 in the linear layer) gives the empty sum, Y = 0.
 *
 * The sparse format (Sec. 3.3, "Mapping Sparse Weights")
 *   bitmap      [rows, ceil(cols/32)] uint32.  Bit t (least significant first) of word w of a row
 *               is column 32*w + t: 1 iff the entry is nonzero.  Seen as bytes this is the paper's
 *               byte mask, bit t of byte b = column 8*b + t.  Pad bits of a row's last word are 0.
 *   values      [nnz] bf16 patterns: the nonzero entries in row-major order (the paper's v).
 *               As an INPUT the buffer must be readable up to the next multiple of 16 bytes past its
 *               nnz elements (the padding is loaded by vector reads, its contents are never used);
 *               it may be NULL only when nnz == 0.
 *   row_offsets [rows + 1] uint32: row_offsets[n] = number of nonzeros before row n, so
 *               row_offsets[rows] = nnz.  (The paper leaves open how a row's start in v is found;
 *               this array is that.)  nnz must be < 2^32.
 *   "Nonzero" is a value test: +0.0 and -0.0 are zero (and decode to +0.0); NaN and Inf are nonzero
 *   and are carried bit for bit.
 */
#ifndef SALR_H
#define SALR_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    SALR_OK = 0,
    SALR_ERR_INVALID_ARG = 1, /* null pointer where data is required, negative size            */
    SALR_ERR_SHAPE = 2,       /* sizes violate a stated constraint                              */
    SALR_ERR_CAPACITY = 3,    /* values buffer or workspace smaller than required               */
    SALR_ERR_UNSUPPORTED = 4, /* legal request that this build has no kernel for                */
    SALR_ERR_HIP = 5          /* the HIP runtime reported an error while enqueuing              */
} salr_status_t;

/* Static, NUL-terminated description of a status code (host memory, never freed). */
const char* salr_status_string(salr_status_t status);

/* ceil(cols / 32): uint32 words per bitmap row.  Returns -1 for cols < 0. */
int64_t salr_bitmap_words_per_row(int64_t cols);

/*
 * salr_magnitude_mask_rows -- Sec. 2, the static magnitude mask W-hat = W .* [|W| > T_p], with the
 * threshold taken per output row so that every row keeps exactly `keep` entries (its
 * round((1-p) * cols) largest magnitudes; among equal magnitudes the lower column wins).  Kept
 * entries are copied bit for bit, pruned ones become +0.0.  Magnitudes compare as the 15 low bits of
 * the bf16 pattern, so NaN/Inf rank above every finite value.
 *
 *   w      in   [rows, cols] bf16
 *   keep   in   entries to keep per row, 0 <= keep <= cols
 *   w_hat  out  [rows, cols] bf16; must not overlap w
 *
 * Errors: INVALID_ARG (null pointer with rows*cols > 0, negative size, keep outside [0, cols]),
 * SHAPE (rows > 2^31 - 1 or cols > 2^31 - 32), HIP.
 */
salr_status_t salr_magnitude_mask_rows(const uint16_t* w, int64_t rows, int64_t cols, int64_t keep,
                                       uint16_t* w_hat, void* stream);

/*
 * salr_magnitude_mask_nm -- the N:M pattern of the inference-throughput comparison (Sec. 4, 2:4): in
 * every group of m_group consecutive columns of a row the n_keep largest magnitudes survive, ties to
 * the lower column; the rest become +0.0.
 *
 *   w, w_hat  as above; cols % m_group == 0 (else SHAPE); 1 <= m_group <= 64 (else UNSUPPORTED);
 *             0 <= n_keep <= m_group (else INVALID_ARG)
 */
salr_status_t salr_magnitude_mask_nm(const uint16_t* w, int64_t rows, int64_t cols, int64_t n_keep,
                                     int64_t m_group, uint16_t* w_hat, void* stream);

/*
 * salr_encode_bitmap -- Sec. 3.3: B[n][k] = [W-hat[n][k] != 0], v = nonzeros in row-major order.
 *
 *   w_dense          in   [rows, cols] bf16, already pruned (zeros where entries were removed)
 *   bitmap           out  [rows, ceil(cols/32)] uint32
 *   values           out  [values_capacity] bf16; NULL = count only (bitmap and row_offsets are
 *                         still produced, so a caller can size `values` from row_offsets[rows])
 *   values_capacity  in   elements available in `values` (ignored when values == NULL)
 *   row_offsets      out  [rows + 1] uint32; row_offsets[rows] = nnz stays on the device
 *
 * If nnz exceeds values_capacity the kernel never writes past the buffer: entries with index
 * >= values_capacity are dropped, row_offsets still holds the true counts, and it is the caller who
 * compares row_offsets[rows] with the capacity (the library cannot know nnz without a sync).
 * Errors: INVALID_ARG (null w_dense/bitmap/row_offsets, negative size), SHAPE (rows * cols or a
 * dimension beyond 2^31 - 1 rows / 2^31 - 32 cols), HIP.
 */
salr_status_t salr_encode_bitmap(const uint16_t* w_dense, int64_t rows, int64_t cols, uint32_t* bitmap,
                                 uint16_t* values, int64_t values_capacity, uint32_t* row_offsets,
                                 void* stream);

/*
 * salr_decode -- Sec. 3.3, the reconstruction rule: for byte block b of row n with mask m,
 * W-hat[n][8b+t] = (bit t of m) ? segment[popcount(m & (2^t - 1))] : 0, where the block's segment
 * starts at row_offsets[n] + popcount of the row's earlier bits.  (The paper tabulates
 * popcount(m & (2^t - 1)) in a 256 x 8 lookup table; the result is the same.)
 *
 *   bitmap, values, row_offsets  in   the format above
 *   w_dense_out                  out  [rows, cols] bf16; clear bits give +0.0 (0x0000)
 *
 * The format is trusted: offsets that point outside `values` are the caller's error.
 * Errors: INVALID_ARG (null bitmap/row_offsets/w_dense_out with rows*cols > 0), SHAPE, HIP.
 */
salr_status_t salr_decode(const uint32_t* bitmap, const uint16_t* values, const uint32_t* row_offsets,
                          int64_t rows, int64_t cols, uint16_t* w_dense_out, void* stream);

/*
 * Bytes of device workspace salr_sparse_lowrank_linear needs for these sizes (0 is possible).
 * It holds T = X * A_cat and fp32 partial results of contractions that are split over K; for large
 * batches (M > 128, or M > 64 where K is no multiple of 128), where the weight is decoded once per
 * call into a dense scratch matrix that the matrix-core stage then reads, also a transposed copy of
 * A_cat and N * K bf16 elements of decoded weight; for batches of up to 128 tokens with adapters on rows of whole
 * 128-column chunks, a slice table (64 bytes per weight row, see below) that the call builds for itself beside the
 * first adapter product when it is not handed one.  Nothing in it outlives the call.  Returns 0 for invalid sizes.
 */
size_t salr_linear_workspace_bytes(int64_t M, int64_t K, int64_t N, int64_t R);

/*
 * Slice table of a layer: a derived index for small batches (Sec. 3.3 reads the value array sequentially; where a
 * row's values for a given range of columns start is otherwise found by popcounting the bitmap words before them, a
 * round trip to memory that every workgroup of the small-batch kernel pays before it can ask for its first value).
 * For row n and slice w = 0..7 of the row's C = ceil(K / 128) chunks of 128 columns (chunks [C w / 8, C (w + 1) / 8)):
 *     table[(n * 8 + w) * 2 + 0] = row_offsets[n] + nonzeros of row n in the columns before the slice
 *     table[(n * 8 + w) * 2 + 1] = the most nonzeros that any one chunk of the slice holds
 * It follows from bitmap and row_offsets alone (the three arrays above stay the format); build it once per layer.
 *   salr_slice_table_bytes   N * 64 bytes (0 for arguments the builder would refuse)
 *   salr_build_slice_table   slice_table out, [N, 8, 2] uint32, at least that many bytes (else CAPACITY)
 *   salr_sparse_lowrank_linear_prepared   salr_sparse_lowrank_linear with the table as one more input; the result is
 *       the same bit for bit; paths that have no use for the table (larger batches, rows that are not whole chunks)
 *       ignore it.  (The plain call builds the same table in its workspace on calls with adapters, inside the launch
 *       that computes X * A_cat, except for up to 16 tokens on rows of 12288 columns and more; handing it over saves
 *       that pass over the bitmap, 2 to 10 us on the larger layers, and serves calls without adapters and those long
 *       rows too.)  A table that does not belong to the weight gives unspecified values in Y and may read `values`
 *       out of bounds: it is the caller's to keep the two together, as with row_offsets.
 * Errors: INVALID_ARG, SHAPE, CAPACITY, HIP, and those of salr_sparse_lowrank_linear.
 */
size_t salr_slice_table_bytes(int64_t N, int64_t K);
salr_status_t salr_build_slice_table(const uint32_t* bitmap, const uint32_t* row_offsets, int64_t N, int64_t K,
                                     uint32_t* slice_table, size_t slice_table_bytes, void* stream);
salr_status_t salr_sparse_lowrank_linear_prepared(const uint16_t* x, int64_t M, int64_t K, int64_t N, const uint32_t* bitmap,
                                                  const uint16_t* values, const uint32_t* row_offsets,
                                                  const uint32_t* slice_table, const uint16_t* a_cat, const uint16_t* b_cat,
                                                  int64_t R, uint16_t* y, void* workspace, size_t workspace_bytes,
                                                  void* stream);

/*
 * The least workspace salr_sparse_lowrank_linear runs with.  It differs from the size above for large batches only:
 * given at least this much but less than salr_linear_workspace_bytes, the call keeps no decoded copy of the weight
 * and runs the pipeline of Sec. 3.3 inside one kernel instead (bitmap decode of the next weight tile into
 * double-buffered LDS tiles while the matrix cores multiply the current one).  That is slower than decoding once
 * into memory (every 256-row block of X decodes the weight again) but the weight never exists in dense form
 * outside LDS, which is what the format is for when memory is short.  Returns 0 for invalid sizes.
 */
size_t salr_linear_workspace_bytes_min(int64_t M, int64_t K, int64_t N, int64_t R);

/*
 * salr_sparse_lowrank_linear -- the layer of Sec. 3.2 / 3.3:
 *
 *     Y = X * W-hat^T + (X * A_cat) * B_cat
 *
 * with W-hat decoded on the fly from the bitmap format (decode stage feeding the matrix-core
 * stage, Sec. 3.3 "Pipeline Design") and all adapters applied as ONE concatenated pair
 * A_cat = [A_1 ... A_n], B_cat = [B_1; ...; B_n] (Sec. 3.2).  bf16 inputs, fp32 accumulation,
 * T = X * A_cat rounded once to bf16, Y rounded to bf16 (nearest even).  No bias and no LoRA scale:
 * fold alpha/r into B_cat.
 *
 *   x            in   [M, K] bf16
 *   bitmap       in   [N, K/32] uint32      } W-hat, [N, K], in the format above
 *   values       in   [nnz] bf16            }
 *   row_offsets  in   [N + 1] uint32        }
 *   a_cat        in   [K, R] bf16; may be NULL iff R == 0
 *   b_cat        in   [R, N] bf16; may be NULL iff R == 0
 *   y            out  [M, N] bf16, overwritten
 *   workspace    --   salr_linear_workspace_bytes(M, K, N, R) bytes, 256-byte aligned (at least
 *                     salr_linear_workspace_bytes_min: see there for what the smaller size means); may be NULL
 *                     when that size is 0.  Contents before and after are unspecified.
 *
 * Constraints: K % 32 == 0 (else SHAPE); R <= 256 (else UNSUPPORTED); M, N < 2^31.
 * K == 0: x, bitmap, values, a_cat may be NULL; Y is written as zeros (both products are empty sums).
 * Errors: INVALID_ARG, SHAPE, CAPACITY (workspace too small), UNSUPPORTED, HIP.
 * Calls that share a workspace must be ordered by the stream.
 */
salr_status_t salr_sparse_lowrank_linear(const uint16_t* x, int64_t M, int64_t K, int64_t N,
                                         const uint32_t* bitmap, const uint16_t* values,
                                         const uint32_t* row_offsets, const uint16_t* a_cat,
                                         const uint16_t* b_cat, int64_t R, uint16_t* y, void* workspace,
                                         size_t workspace_bytes, void* stream);

/*
 * salr_sparse_lowrank_linear_noalloc -- salr_sparse_lowrank_linear for callers that cannot allocate device memory
 * or carry a workspace around: code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.
 * Arguments, result and rounding are those of salr_sparse_lowrank_linear without `workspace`; the kernels are the
 * same ones.  What they keep in the workspace there (split-K partial sums of T = X * A_cat and of Y) lives here in a
 * fixed array of SALR_NOALLOC_SCRATCH_BYTES bytes of device memory inside the library's code object, which every GPU
 * the library runs on holds from the first use until the process ends.  The call allocates and frees nothing.
 *
 * Limit: sizes for which neither salr_linear_workspace_bytes(M, K, N, R) nor salr_linear_workspace_bytes_min(M, K, N,
 * R) fits SALR_NOALLOC_SCRATCH_BYTES are refused with SALR_ERR_CAPACITY before anything is enqueued.  Decode-sized
 * batches fit; large batches, whose preferred path decodes the weight into a dense scratch matrix, run the
 * fused kernel of salr_linear_workspace_bytes_min instead as long as their adapter intermediates fit.
 * The device that is current when the call is made must be the one `stream` belongs to; the first call on a device
 * looks up that device's copy of the array (no allocation; make it outside a graph capture).
 * All calls on one GPU share that GPU's array: calls that may overlap on one GPU (different streams without
 * ordering between them) race on it and must be ordered by the caller.  Nothing in the array has to survive
 * between calls or start at zero: every call writes what it later reads.
 * Errors: as salr_sparse_lowrank_linear, with CAPACITY as above.
 */
#define SALR_NOALLOC_SCRATCH_BYTES (16u * 1024u * 1024u)
salr_status_t salr_sparse_lowrank_linear_noalloc(const uint16_t* x, int64_t M, int64_t K, int64_t N,
                                                 const uint32_t* bitmap, const uint16_t* values,
                                                 const uint32_t* row_offsets, const uint16_t* a_cat,
                                                 const uint16_t* b_cat, int64_t R, uint16_t* y, void* stream);

/*
 * QSALR -- Sec. 4 ("Coupled with Quantization", the size/accuracy table of 20 % sparsity + NF4): the packed values
 * of the bitmap format stored as 4-bit NormalFloat codes.  The paper names the data type and nothing else; this
 * library's reading is
 *   levels   the 16 NF4 levels of the QLoRA paper that the SALR paper cites (normal quantiles scaled to [-1, 1],
 *            ascending, exact zero at index 7);
 *   scales   [ceil(count / 64)] bf16: one per block of 64 CONSECUTIVE packed values (in the order of `values`,
 *            whatever rows they belong to; the last block may be short), the block's largest magnitude (one of its
 *            own values, so exact in bf16);
 *   codes    [ceil(count / 2)] bytes, two codes per byte, the even-indexed value in the low nibble (the unused high
 *            nibble of an odd count is 0).  A value x gets the code of the level nearest to x / scale, decided
 *            without division: the number of k in 0..14 with x > fp32(mid_k * scale), mid_k =
 *            fp32(0.5 * (level_k + level_{k+1})); a value on a boundary takes the lower code; an all-zero block has
 *            scale 0 and codes 7;
 *   value    bf16_rne(fp32(level[code] * scale)).
 * Size: bitmap 1 bit + (1 - p) * (4 + 16 / 64) bits per weight element = 4.4 bits at p = 0.2, against 16 dense.
 *
 * salr_nf4_quantize_values / salr_nf4_dequantize_values convert between `values` [count] bf16 and (codes, scales);
 * bitmap and row_offsets of the format are untouched.  values_out must be writable up to the next multiple of 8
 * elements.  Errors: INVALID_ARG (null pointer with count > 0, negative count), SHAPE (count >= 2^32), HIP.
 *
 * salr_qsalr_linear is salr_sparse_lowrank_linear on such a weight: Y = X * W-hat'^T + (X * A_cat) * B_cat with
 * W-hat' = decode(bitmap, dequantised values); arguments, rounding and errors otherwise as there.  nnz =
 * row_offsets[N], which the caller knows from encoding (host value).
 *   - Up to 64 tokens on rows of whole 128-column chunks (K % 128 == 0, nnz > 0) one kernel reads bitmap, codes and
 *     scales and dequantises inside its decode stage: the weight crosses the memory system at 1 + 4.25 (1 - p) bits
 *     per element and no bf16 copy of the values exists.  Workspace: the layer's partial sums of X * A_cat and a
 *     slice table built per call (64 bytes per weight row).
 *   As an INPUT to salr_qsalr_linear `codes` must be readable up to the next multiple of 16 bytes (vector reads; the
 *   padding is never used).
 *   - Large batches that take the two-stage path (more than 128 tokens, or more than 64 where the row-tiled kernel
 *     does not apply; K % 64 == 0): its decode stage reads the codes; workspace as for the plain layer.
 *   - Otherwise the values are dequantised once per call into the first part of the workspace (2 * nnz bytes,
 *     rounded up), then the layer runs as usual on them.
 * Both compute the same products; where the plain layer would take its small-batch streaming kernels Y is the same
 * bit for bit (finite scales).
 * Workspace: salr_qsalr_linear_workspace_bytes(M, K, N, R, nnz) bytes, 256-byte aligned.
 */
salr_status_t salr_nf4_quantize_values(const uint16_t* values, int64_t count, uint8_t* codes, uint16_t* scales,
                                       void* stream);
salr_status_t salr_nf4_dequantize_values(const uint8_t* codes, const uint16_t* scales, int64_t count,
                                         uint16_t* values_out, void* stream);
size_t salr_qsalr_linear_workspace_bytes(int64_t M, int64_t K, int64_t N, int64_t R, int64_t nnz);
salr_status_t salr_qsalr_linear(const uint16_t* x, int64_t M, int64_t K, int64_t N, const uint32_t* bitmap,
                                const uint8_t* codes, const uint16_t* scales, const uint32_t* row_offsets,
                                int64_t nnz, const uint16_t* a_cat, const uint16_t* b_cat, int64_t R, uint16_t* y,
                                void* workspace, size_t workspace_bytes, void* stream);

/*
 * The layer on 2:4-masked weights (the N:M protocol of the inference-throughput table, Sec. 4).
 *
 * salr_bitmap_is_2of4 writes 1 to *result (device memory, one uint32) when every aligned group of four
 * columns of the bitmap has exactly two set bits, else 0 (also for an empty bitmap); a layer is checked once,
 * when it is prepared.
 *   bitmap   in   [rows, cols/32] uint32;  cols % 32 == 0 (else SHAPE)
 *   result   out  one uint32 in device memory, written on the stream
 *
 * salr_sparse_lowrank_linear_2of4 computes what salr_sparse_lowrank_linear computes, arguments and
 * rounding as there, for a weight that passes that check.  In the SALR format such a weight already is the
 * operand of the sparse matrix-core instructions (two stored values and two 2-bit positions per group of
 * four), so for M <= 128 and K % 128 == 0 bitmap and packed values are multiplied as they are, without the
 * decode stage; other shapes are passed on to salr_sparse_lowrank_linear.  The precondition is not checked
 * by this call (the flag that salr_bitmap_is_2of4 writes lives in device memory, and reading it here would
 * mean a synchronisation, which no entry point of this library performs: the caller reads it once per layer
 * and picks the entry point): on a weight that fails it the result is unspecified (no memory outside the
 * buffers is read or written).  Workspace: salr_linear_2of4_workspace_bytes(M, K, N, R) bytes.
 * Errors of both: INVALID_ARG, SHAPE, CAPACITY, UNSUPPORTED, HIP as above.
 */
salr_status_t salr_bitmap_is_2of4(const uint32_t* bitmap, int64_t rows, int64_t cols, uint32_t* result,
                                  void* stream);
size_t salr_linear_2of4_workspace_bytes(int64_t M, int64_t K, int64_t N, int64_t R);
salr_status_t salr_sparse_lowrank_linear_2of4(const uint16_t* x, int64_t M, int64_t K, int64_t N,
                                              const uint32_t* bitmap, const uint16_t* values,
                                              const uint32_t* row_offsets, const uint16_t* a_cat,
                                              const uint16_t* b_cat, int64_t R, uint16_t* y, void* workspace,
                                              size_t workspace_bytes, void* stream);

/*
 * salr_sparse_lowrank_linear_backward -- the adjoint of the layer of Sec. 3.2 / 3.3, which fine-tuning (the
 * training-throughput comparison of Sec. 4) runs every step.  The pruned base weight is frozen and gets no
 * gradient; the concatenated adapters do:
 *
 *     dX [M, K] = dY W-hat + (dY B_cat^T) A_cat^T
 *     dA [K, R] = X^T (dY B_cat^T)           (gradient of A_cat: columns in the order of the concatenation)
 *     dB [R, N] = (X A_cat)^T dY
 *
 * bf16 in and out, fp32 sums; as in the forward pass the two [M, R] intermediates are rounded to bf16 once.
 *
 *   x            in   [M, K] bf16, the layer's input (needed for dA / dB only; may be NULL otherwise)
 *   dy           in   [M, N] bf16, the gradient of the layer's output
 *   bitmap, values, row_offsets, a_cat, b_cat, R   as for salr_sparse_lowrank_linear (the weight is needed for dX only)
 *   dx, da, db   out  any of them may be NULL: that gradient is not computed
 *   workspace    --   at least salr_linear_backward_workspace_bytes(M, K, N, R, dx != NULL, da != NULL || db != NULL)
 *                     bytes, 256-byte aligned (for dX it holds the decoded weight and its transpose, 4 N K bytes)
 *
 * Constraints: K % 32 == 0 (SHAPE); N % 64 == 0 for dX, N % 32 == 0 with adapters, M % 32 == 0 for dA / dB,
 * R <= 256 (UNSUPPORTED otherwise).  The workspace query returns 0 for sizes the call would refuse.
 * Errors: INVALID_ARG, SHAPE, UNSUPPORTED, CAPACITY, HIP.
 */
size_t salr_linear_backward_workspace_bytes(int64_t M, int64_t K, int64_t N, int64_t R, int want_dx, int want_dadb);
salr_status_t salr_sparse_lowrank_linear_backward(const uint16_t* x, const uint16_t* dy, int64_t M, int64_t K,
                                                  int64_t N, const uint32_t* bitmap, const uint16_t* values,
                                                  const uint32_t* row_offsets, const uint16_t* a_cat,
                                                  const uint16_t* b_cat, int64_t R, uint16_t* dx, uint16_t* da,
                                                  uint16_t* db, void* workspace, size_t workspace_bytes, void* stream);

/*
 * salr_residual -- Sec. 3.1 ("Sparsity Preservation Pruning"): the residual E = W - W-hat that the pruning
 * leaves behind and whose truncated SVD becomes the residual adapter.
 *
 *   w, w_hat   in   [rows, cols] bf16
 *   e          out  [rows, cols] bf16: bf16(float(w) - float(w_hat)), the subtraction in fp32, rounded to
 *                   nearest even.  When every entry of w_hat is the entry of w or zero (a mask), this is exact:
 *                   the entry of w where it was pruned and +0 where it was kept.  May alias neither input.
 * Errors: INVALID_ARG, SHAPE (rows or cols >= 2^31), HIP.
 */
salr_status_t salr_residual(const uint16_t* w, const uint16_t* w_hat, int64_t rows, int64_t cols, uint16_t* e,
                            void* stream);

/*
 * salr_residual_adapter -- Sec. 3.1: the residual adapter, a low-rank pair whose product is the best rank-r
 * approximation E_r (truncated SVD) of the residual E, in the orientation of the linear layer:
 *
 *     (A_res B_res)^T ~ E_r,   A_res = V_r S_r^{1/2} [K, r],   B_res = S_r^{1/2} U_r^T [r, N]   for E = U S V^T,
 *
 * so that appending (A_res, B_res) to A_cat / B_cat adds x E_r^T to the layer output.  The factors are computed
 * by randomized subspace iteration (the paper names no algorithm): a sketch E Omega with l = r + oversample
 * columns, `power_iterations` rounds of multiplying by E^T and E with re-orthonormalisation, then the SVD of the
 * small projected matrix.  The pair itself is not unique (signs, rotations inside equal singular values); its
 * product is, up to the method's error: ||E - (A_res B_res)^T||_F exceeds the optimum ||E - E_r||_F by a factor
 * that falls geometrically with power_iterations, at a rate set by the decay of E's singular values.
 *
 *   e            in   [N, K] bf16 (salr_residual's output, or any matrix)
 *   r            rank of the pair; oversample >= 0 extra sketch columns; r + oversample <= 128 (else
 *                UNSUPPORTED) and <= min(N, K) (else SHAPE)
 *   omega        in   [K, r + oversample] fp32, row-major: the test matrix, independent standard normal entries
 *                     drawn by the caller (the library draws no random numbers)
 *   a_res        out  [K, r] bf16
 *   b_res        out  [r, N] bf16
 *   sigma        out  [r] fp32, the singular values found, descending; may be NULL
 *   workspace    --   at least salr_residual_adapter_workspace_bytes(N, K, r, oversample) bytes, 256-byte aligned
 *                     (it holds a transposed copy of E and the tall fp32 factors); contents unspecified
 *
 * Constraints: N % 32 == 0, K % 32 == 0, N and K <= 2097120 (else SHAPE); power_iterations <= 64.  A matrix of rank below r yields
 * zero columns / rows for the missing directions.  The workspace query returns 0 for sizes the call would refuse.
 * Errors: INVALID_ARG, SHAPE, UNSUPPORTED, CAPACITY, HIP.
 */
size_t salr_residual_adapter_workspace_bytes(int64_t N, int64_t K, int64_t r, int64_t oversample);
salr_status_t salr_residual_adapter(const uint16_t* e, int64_t N, int64_t K, int64_t r, int64_t oversample,
                                    int64_t power_iterations, const float* omega, uint16_t* a_res, uint16_t* b_res,
                                    float* sigma, void* workspace, size_t workspace_bytes, void* stream);

/*
 * salr_concat_adapters -- Sec. 3.2 ("Concatenating Multi-LoRA adapters"): A_cat = [A_1 ... A_n] side by side
 * and B_cat = [B_1; ...; B_n] stacked, so that (x A_cat) B_cat = sum_i (x A_i) B_i.
 *
 *   a_list, b_list  in   HOST arrays of n DEVICE pointers: A_i [K, ranks[i]] bf16, B_i [ranks[i], N] bf16
 *   ranks           in   HOST array of n ranks r_i >= 0; R = sum r_i <= 65535 (else SHAPE).  An adapter of rank 0
 *                        contributes nothing and its pointers are not looked at.
 *   a_cat           out  [K, R] bf16: columns [sum_{j<i} r_j, sum_{j<=i} r_j) are A_i
 *   b_cat           out  [R, N] bf16: the same range of rows is B_i
 * The host arrays are read before the call returns.  Pure data movement: outputs are bit copies.
 * Errors: INVALID_ARG (null where data is required, negative size or rank), SHAPE, HIP.
 */
salr_status_t salr_concat_adapters(const uint16_t* const* a_list, const uint16_t* const* b_list,
                                   const int64_t* ranks, int64_t n, int64_t K, int64_t N, uint16_t* a_cat,
                                   uint16_t* b_cat, void* stream);

/*
 * Measurement hook (not part of the method): when both events are non-NULL, the next calls of
 * salr_sparse_lowrank_linear on this host thread attach the two events to the launch of the fused
 * decode+GEMM kernel: `start_event` takes the time the kernel begins executing and `stop_event` the
 * time it ends (the adapter pre-kernel stays outside the pair).  Both are hipEvent_t passed as
 * void*, created by the caller with timing enabled.  Pass NULL, NULL to switch the hook off.
 */
void salr_set_kernel_timing_events(void* start_event, void* stop_event);

#ifdef __cplusplus
}
#endif
#endif /* SALR_H */
