/*
 * SALR CPU oracle -- TEST INFRASTRUCTURE, not part of the product.
 *
 * Plain, slow, obviously-correct C for what the SALR inference linear layer computes:
 *
 *     Y = X * decode(bitmap, v)^T + (X * A_cat) * B_cat
 *
 * Only tests, the smoke check and the benchmark's cpu_baseline leg may call it.  It shares no code
 * with the HIP library.  All bf16 tensors cross this interface as raw 16-bit patterns (uint16_t).
 * Floating-point work is done in fp64 on exactly-widened bf16 inputs with no intermediate rounding.
 *
 * Orientation: W is [rows = out features N, cols = in features K] row-major; the paper writes the
 * transpose (y = xW, W in R^{d_in x d_out}), so its "row i, column j" of the bitmap is our
 * "(n, k)" with the bits of one bitmap row running along the contraction dimension.
 *
 * Every function cites the passage of the paper it follows.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

static double bf16_to_f64(uint16_t b) {
    uint32_t u = (uint32_t)b << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

/* magnitude of a bf16 as an integer: monotone in |value| for all non-NaN patterns */
static uint32_t bf16_mag(uint16_t b) { return (uint32_t)(b & 0x7FFFu); }

int salr_oracle_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* ------------------------------------------------------------------------------------------------
 * Magnitude pruning (Sec. 2, the definition of W-hat):  keep an entry if its magnitude is above the
 * threshold that realises the target sparsity, write 0 otherwise.
 *
 * Reading used here: the threshold is taken per row so that exactly `keep` entries of every row
 * survive; entries are ranked by (|w| descending, column ascending), i.e. among equal magnitudes the
 * lower column wins, and the first `keep` of that ranking are kept.  The paper's strict ">" rule would
 * drop all entries tied at the threshold; with 16-bit data ties are common, so the tie-break is what
 * makes nnz hit the target exactly.  Pruned entries become +0.0 (0x0000).
 * ---------------------------------------------------------------------------------------------- */
typedef struct { uint32_t mag; int64_t col; } mag_col_t;

static int cmp_mag_desc_col_asc(const void* a, const void* b) {
    const mag_col_t* x = (const mag_col_t*)a;
    const mag_col_t* y = (const mag_col_t*)b;
    if (x->mag != y->mag) return (x->mag > y->mag) ? -1 : 1;
    if (x->col != y->col) return (x->col < y->col) ? -1 : 1;
    return 0;
}

int salr_oracle_mask_topk_rows(const uint16_t* w, int64_t rows, int64_t cols, int64_t keep,
                               uint16_t* w_hat) {
    if (!w || !w_hat || rows < 0 || cols < 0 || keep < 0 || keep > cols) return 1;
    int fail = 0;
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < rows; ++n) {
        mag_col_t* order = (mag_col_t*)malloc(sizeof(mag_col_t) * (size_t)(cols > 0 ? cols : 1));
        if (!order) {
#pragma omp atomic write
            fail = 1;
            continue;
        }
        for (int64_t k = 0; k < cols; ++k) { order[k].mag = bf16_mag(w[n * cols + k]); order[k].col = k; }
        qsort(order, (size_t)cols, sizeof(mag_col_t), cmp_mag_desc_col_asc);
        for (int64_t k = 0; k < cols; ++k) w_hat[n * cols + k] = 0;
        for (int64_t j = 0; j < keep; ++j) {
            int64_t k = order[j].col;
            w_hat[n * cols + k] = w[n * cols + k];
        }
        free(order);
    }
    return fail;
}

/* The paper's rule exactly as printed (Sec. 2): keep iff |w| > T, with one threshold magnitude for
 * the whole matrix, given by the caller as a bf16 magnitude pattern. */
int salr_oracle_mask_threshold(const uint16_t* w, int64_t count, uint16_t t_mag, uint16_t* w_hat) {
    if (!w || !w_hat || count < 0) return 1;
    for (int64_t i = 0; i < count; ++i) w_hat[i] = (bf16_mag(w[i]) > bf16_mag(t_mag)) ? w[i] : 0;
    return 0;
}

/* ------------------------------------------------------------------------------------------------
 * Bitmap encoding (Sec. 3.3, "Mapping Sparse Weights"): B[n][k] = 1 iff W-hat[n][k] != 0, and the
 * nonzero entries go, in row-major order, into the compact array v.
 *
 * Readings: "nonzero" is a value test, so -0.0 (0x8000) counts as zero; NaN/Inf count as nonzero and
 * their patterns are copied.  Bits are stored 32 per word, bit t of word w of a row is column 32w+t
 * (least significant bit first); read as bytes on a little-endian machine this is the paper's byte
 * mask with bit t of byte b = column 8b+t.  Pad bits of the last word are 0.  The paper does not say
 * how a row's start in v is found; row_offsets[n] = number of nonzeros before row n (n = 0..rows) is
 * added to the format for that.
 * ---------------------------------------------------------------------------------------------- */
int64_t salr_oracle_words_per_row(int64_t cols) { return (cols + 31) / 32; }

int salr_oracle_encode(const uint16_t* w_hat, int64_t rows, int64_t cols, uint32_t* bitmap,
                       uint16_t* values, int64_t values_capacity, uint32_t* row_offsets) {
    if (!w_hat || !bitmap || !row_offsets || rows < 0 || cols < 0) return 1;
    int64_t wpr = salr_oracle_words_per_row(cols);
    int64_t cursor = 0;
    for (int64_t n = 0; n < rows; ++n) {
        row_offsets[n] = (uint32_t)cursor;
        for (int64_t w = 0; w < wpr; ++w) bitmap[n * wpr + w] = 0;
        for (int64_t k = 0; k < cols; ++k) {
            uint16_t bits = w_hat[n * cols + k];
            if (bf16_mag(bits) != 0) {
                bitmap[n * wpr + k / 32] |= (uint32_t)1 << (k % 32);
                if (values) {
                    if (cursor >= values_capacity) return 3;
                    values[cursor] = bits;
                }
                ++cursor;
            }
        }
    }
    row_offsets[rows] = (uint32_t)cursor;
    return 0;
}

/* Decoding as the inverse of the definition above: walk the elements in row-major order with one
 * running cursor into v; a set bit takes the next value, a clear bit gives +0.0. */
int salr_oracle_decode(const uint32_t* bitmap, const uint16_t* values, const uint32_t* row_offsets,
                       int64_t rows, int64_t cols, uint16_t* w_out) {
    if (!bitmap || !row_offsets || !w_out || rows < 0 || cols < 0) return 1;
    int64_t wpr = salr_oracle_words_per_row(cols);
    for (int64_t n = 0; n < rows; ++n) {
        int64_t cursor = row_offsets[n];
        for (int64_t k = 0; k < cols; ++k) {
            uint32_t bit = (bitmap[n * wpr + k / 32] >> (k % 32)) & 1u;
            w_out[n * cols + k] = bit ? values[cursor++] : (uint16_t)0;
        }
        if (cursor != (int64_t)row_offsets[n + 1]) return 2; /* format inconsistent */
    }
    return 0;
}

/* ------------------------------------------------------------------------------------------------
 * The paper's own decoder (Sec. 3.3, byte blocks + lookup table), kept separate from the cursor
 * decoder above so that each checks the other.
 *
 *   mask_{n,b}   = sum_t B[n][8b+t] 2^t                        (byte block b of row n)
 *   k_{n,b}      = popcount(mask_{n,b})                        (length of the block's segment of v)
 *   LUT(mask)_t  = position of bit t among the set bits of mask, or -1 if bit t is clear
 *   W[n][8b+t]   = segment[LUT(mask)_t]  if that entry is >= 0, else 0
 *
 * The table is built by scanning the 8 bits of every mask value and counting set bits seen so far.
 * ---------------------------------------------------------------------------------------------- */
void salr_oracle_build_lut(int8_t* lut /* [256][8] */) {
    for (int m = 0; m < 256; ++m) {
        int seen = 0;
        for (int t = 0; t < 8; ++t) {
            if ((m >> t) & 1) { lut[m * 8 + t] = (int8_t)seen; ++seen; }
            else lut[m * 8 + t] = -1;
        }
    }
}

static int popcount8(unsigned m) {
    int c = 0;
    for (int t = 0; t < 8; ++t) c += (int)((m >> t) & 1u);
    return c;
}

int salr_oracle_decode_lut(const uint32_t* bitmap, const uint16_t* values, const uint32_t* row_offsets,
                           int64_t rows, int64_t cols, uint16_t* w_out) {
    if (!bitmap || !row_offsets || !w_out || rows < 0 || cols < 0) return 1;
    int8_t lut[256 * 8];
    salr_oracle_build_lut(lut);
    int64_t wpr = salr_oracle_words_per_row(cols);
    const uint8_t* bytes = (const uint8_t*)bitmap; /* little-endian: byte b of a row = columns 8b..8b+7 */
    int64_t blocks = (cols + 7) / 8;
    for (int64_t n = 0; n < rows; ++n) {
        const uint16_t* segment = values ? values + row_offsets[n] : NULL;
        for (int64_t b = 0; b < blocks; ++b) {
            unsigned mask = bytes[n * wpr * 4 + b];
            for (int t = 0; t < 8; ++t) {
                int64_t k = 8 * b + t;
                if (k >= cols) break;
                int l = lut[mask * 8 + t];
                w_out[n * cols + k] = (l >= 0) ? segment[l] : (uint16_t)0;
            }
            if (segment) segment += popcount8(mask);
        }
    }
    return 0;
}

/* ------------------------------------------------------------------------------------------------
 * The layer output (Sec. 3.2, y = xW + sum_i (x A_i) B_i, with the adapters stacked into A_cat and
 * B_cat), in fp64 and in our orientation:
 *
 *   Y[m][n] = sum_k X[m][k] * What[n][k]  +  sum_r ( sum_k X[m][k] * A_cat[k][r] ) * B_cat[r][n]
 *
 * No LoRA scale and no bias: the paper's formula has neither.  R may be 0.
 * ---------------------------------------------------------------------------------------------- */
int salr_oracle_linear(const uint16_t* x, int64_t M, int64_t K, int64_t N, const uint16_t* w_hat,
                       const uint16_t* a_cat, const uint16_t* b_cat, int64_t R, double* y) {
    if (!x || !w_hat || !y || M < 0 || K < 0 || N < 0 || R < 0) return 1;
    if (R > 0 && (!a_cat || !b_cat)) return 1;
    double* T = (double*)calloc((size_t)(M * R > 0 ? M * R : 1), sizeof(double));
    if (!T) return 5;
    /* T = X * A_cat  [M, R] */
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m)
        for (int64_t r = 0; r < R; ++r) {
            double s = 0.0;
            for (int64_t k = 0; k < K; ++k) s += bf16_to_f64(x[m * K + k]) * bf16_to_f64(a_cat[k * R + r]);
            T[m * R + r] = s;
        }
#pragma omp parallel for schedule(static) collapse(2)
    for (int64_t m = 0; m < M; ++m)
        for (int64_t n = 0; n < N; ++n) {
            double s = 0.0;
            for (int64_t k = 0; k < K; ++k) s += bf16_to_f64(x[m * K + k]) * bf16_to_f64(w_hat[n * K + k]);
            double d = 0.0;
            for (int64_t r = 0; r < R; ++r) d += T[m * R + r] * bf16_to_f64(b_cat[r * N + n]);
            y[m * N + n] = s + d;
        }
    free(T);
    return 0;
}

/* The un-concatenated form of the adapter term, sum_i (x A_i) B_i, one adapter at a time
 * (Sec. 3.2, before stacking); adds into y. */
int salr_oracle_adapter_accumulate(const uint16_t* x, int64_t M, int64_t K, int64_t N,
                                   const uint16_t* a_i, const uint16_t* b_i, int64_t r_i, double* y) {
    if (!x || !a_i || !b_i || !y || M < 0 || K < 0 || N < 0 || r_i < 0) return 1;
    for (int64_t m = 0; m < M; ++m)
        for (int64_t r = 0; r < r_i; ++r) {
            double t = 0.0;
            for (int64_t k = 0; k < K; ++k) t += bf16_to_f64(x[m * K + k]) * bf16_to_f64(a_i[k * r_i + r]);
            for (int64_t n = 0; n < N; ++n) y[m * N + n] += t * bf16_to_f64(b_i[r * N + n]);
        }
    return 0;
}

/* ------------------------------------------------------------------------------------------------
 * N:M semi-structured pruning (the pattern the paper's inference-throughput table uses, Sec. 4: 2:4
 * following the protocol of its baseline): in every group of m consecutive columns of a row the n
 * entries of largest magnitude are kept, ties to the lower column, the rest become +0.0.
 * Each group is ranked by brute force.  cols must be a multiple of m.
 * ---------------------------------------------------------------------------------------------- */
int salr_oracle_mask_nm(const uint16_t* w, int64_t rows, int64_t cols, int64_t n_keep, int64_t m_group,
                        uint16_t* w_hat) {
    if (!w || !w_hat || rows < 0 || cols < 0 || m_group <= 0 || n_keep < 0 || n_keep > m_group) return 1;
    if (cols % m_group != 0) return 2;
    for (int64_t r = 0; r < rows; ++r)
        for (int64_t g0 = 0; g0 < cols; g0 += m_group)
            for (int64_t i = 0; i < m_group; ++i) {
                const uint32_t mi = bf16_mag(w[r * cols + g0 + i]);
                int64_t beaten_by = 0; /* entries of the group that rank before entry i */
                for (int64_t j = 0; j < m_group; ++j) {
                    const uint32_t mj = bf16_mag(w[r * cols + g0 + j]);
                    if (mj > mi || (mj == mi && j < i)) ++beaten_by;
                }
                w_hat[r * cols + g0 + i] = (beaten_by < n_keep) ? w[r * cols + g0 + i] : (uint16_t)0;
            }
    return 0;
}

/* ------------------------------------------------------------------------------------------------
 * QSALR (Sec. 4, "Coupled with Quantization"; the size/accuracy table of the 20 % sparsity + NF4
 * variant): the packed nonzero values v of the bitmap format are stored as 4-bit NormalFloat codes.
 *
 * The paper names the data type (NF4, from the QLoRA paper it cites) and nothing else.  Reading taken
 * here: the 16-entry NF4 code book as that paper publishes it (quantiles of N(0,1) scaled to [-1, 1],
 * with an exact zero); blocks of 64 CONSECUTIVE packed values (in the order of v, whatever rows they
 * belong to; the last block may be short) share one scale = the largest magnitude of the block, which
 * is itself one of the bf16 values and so needs no rounding; a value x gets the code of the entry
 * nearest to x / scale, decided without a division: code = number of i in 0..14 with
 * x > fp32(mid_i * scale), mid_i = fp32(0.5 * (c_i + c_{i+1})), all in fp32 (a value exactly on a
 * boundary takes the lower code); two codes per byte, the even-indexed value in the low nibble.
 * Dequantisation: v'[i] = bf16_rne(fp32(c[code] * scale)).  A block of all zeros (cannot occur for
 * packed nonzeros, allowed for generality) has scale +0 and every code 7 (the exact zero).
 * ---------------------------------------------------------------------------------------------- */
static const float kNf4[16] = {
    -1.0f, -0.6961928009986877f, -0.5250730514526367f, -0.39491748809814453f,
    -0.28444138169288635f, -0.18477343022823334f, -0.09105003625154495f, 0.0f,
    0.07958029955625534f, 0.16093020141124725f, 0.24611230194568634f, 0.33791524171829224f,
    0.44070982933044434f, 0.5626170039176941f, 0.7229568362236023f, 1.0f};

void salr_oracle_nf4_codebook(float* out /* [16] */) {
    for (int i = 0; i < 16; ++i) out[i] = kNf4[i];
}

static float bf16_to_f32(uint16_t b) {
    uint32_t u = (uint32_t)b << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return f;
}

static uint16_t f32_to_bf16_rne_bits(float f) {
    uint32_t u;
    memcpy(&u, &f, sizeof u);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (uint16_t)((u >> 16) | 0x0040u); /* NaN stays NaN */
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

int64_t salr_oracle_nf4_blocks(int64_t count) { return (count + 63) / 64; }

int salr_oracle_nf4_quantize(const uint16_t* values, int64_t count, uint8_t* codes /* [(count+1)/2] */,
                             uint16_t* scales /* [(count+63)/64] bf16 */) {
    if (count < 0 || (count > 0 && (!values || !codes || !scales))) return 1;
    for (int64_t i = 0; i < (count + 1) / 2; ++i) codes[i] = 0;
    for (int64_t b0 = 0; b0 < count; b0 += 64) {
        const int64_t b1 = b0 + 64 < count ? b0 + 64 : count;
        uint16_t amax = 0; /* magnitude pattern: for finite bf16 the integer order is the order of |x| */
        for (int64_t i = b0; i < b1; ++i) {
            const uint16_t mag = (uint16_t)(values[i] & 0x7FFFu);
            if (mag > amax) amax = mag;
        }
        scales[b0 / 64] = amax;
        const float s = bf16_to_f32(amax);
        for (int64_t i = b0; i < b1; ++i) {
            const float x = bf16_to_f32(values[i]);
            int code = 0;
            if (amax == 0) {
                code = 7;
            } else {
                for (int k = 0; k < 15; ++k) {
                    const volatile float mid = 0.5f * (kNf4[k] + kNf4[k + 1]);
                    const volatile float edge = mid * s; /* one fp32 product, rounded once */
                    if (x > edge) ++code;
                }
            }
            codes[i / 2] |= (uint8_t)(code << (4 * (i & 1)));
        }
    }
    return 0;
}

int salr_oracle_nf4_dequantize(const uint8_t* codes, const uint16_t* scales, int64_t count, uint16_t* values_out) {
    if (count < 0 || (count > 0 && (!codes || !scales || !values_out))) return 1;
    for (int64_t i = 0; i < count; ++i) {
        const int code = (codes[i / 2] >> (4 * (i & 1))) & 15;
        const volatile float p = kNf4[code] * bf16_to_f32(scales[i / 64]);
        values_out[i] = f32_to_bf16_rne_bits(p);
    }
    return 0;
}
