/*
 * Sanitizer driver for the CPU oracle (test infrastructure): compiled together with oracle/salr_oracle.c under
 * -fsanitize=address,undefined and run by tests/test_oracle_sanitize.py.  It walks every oracle entry point over
 * ragged shapes (columns that are no multiple of 8 or 32, empty rows and matrices, full rows, keep = 0 and keep =
 * cols) with exactly-sized heap buffers, so that any access past a buffer, any misaligned or overflowing
 * arithmetic stops the program; it also checks the round trip encode -> decode and that both decoders agree.
 * Exit status 0 = clean.
 */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

int salr_oracle_mask_topk_rows(const uint16_t*, int64_t, int64_t, int64_t, uint16_t*);
int salr_oracle_mask_threshold(const uint16_t*, int64_t, uint16_t, uint16_t*);
int salr_oracle_mask_nm(const uint16_t*, int64_t, int64_t, int64_t, int64_t, uint16_t*);
int64_t salr_oracle_words_per_row(int64_t);
int salr_oracle_encode(const uint16_t*, int64_t, int64_t, uint32_t*, uint16_t*, int64_t, uint32_t*);
int salr_oracle_decode(const uint32_t*, const uint16_t*, const uint32_t*, int64_t, int64_t, uint16_t*);
int salr_oracle_decode_lut(const uint32_t*, const uint16_t*, const uint32_t*, int64_t, int64_t, uint16_t*);
int salr_oracle_linear(const uint16_t*, int64_t, int64_t, int64_t, const uint16_t*, const uint16_t*, const uint16_t*,
                       int64_t, double*);
int salr_oracle_adapter_accumulate(const uint16_t*, int64_t, int64_t, int64_t, const uint16_t*, const uint16_t*, int64_t,
                                   double*);
int salr_oracle_nf4_quantize(const uint16_t*, int64_t, uint8_t*, uint16_t*);
int salr_oracle_nf4_dequantize(const uint8_t*, const uint16_t*, int64_t, uint16_t*);

static uint64_t rng_state = 0x2601169912345ULL;
static uint32_t rnd(void) {
    rng_state = rng_state * 6364136223846793005ULL + 1442695040888963407ULL;
    return (uint32_t)(rng_state >> 33);
}
/* a finite bf16 pattern of modest magnitude (exponent 112..127), either sign, a few exact zeros and -0.0 */
static uint16_t rnd_bf16(void) {
    uint32_t r = rnd();
    if (r % 37 == 0) return 0;
    if (r % 41 == 0) return 0x8000u;
    return (uint16_t)(((r >> 3) & 0x8000u) | ((112u + (r >> 8) % 16u) << 7) | (r & 0x7Fu));
}
static void* xmalloc(size_t n) {
    void* p = malloc(n ? n : 1);
    if (!p) { fprintf(stderr, "out of memory\n"); exit(2); }
    return p;
}
#define CHECK(cond)                                                             \
    do {                                                                        \
        if (!(cond)) { fprintf(stderr, "%s:%d: %s\n", __FILE__, __LINE__, #cond); exit(1); } \
    } while (0)

static void one_shape(int64_t rows, int64_t cols, int64_t keep) {
    const size_t n = (size_t)(rows * cols);
    uint16_t* w = xmalloc(2 * n);
    uint16_t* w_hat = xmalloc(2 * n);
    uint16_t* back = xmalloc(2 * n);
    uint16_t* back2 = xmalloc(2 * n);
    for (size_t i = 0; i < n; ++i) w[i] = rnd_bf16();
    CHECK(salr_oracle_mask_topk_rows(w, rows, cols, keep, w_hat) == 0);
    const int64_t wpr = salr_oracle_words_per_row(cols);
    uint32_t* bitmap = xmalloc(4 * (size_t)(rows * wpr));
    uint32_t* offsets = xmalloc(4 * (size_t)(rows + 1));
    CHECK(salr_oracle_encode(w_hat, rows, cols, bitmap, NULL, 0, offsets) == 0);   /* count only */
    const int64_t nnz = offsets[rows];
    CHECK(nnz <= rows * keep);
    uint16_t* values = xmalloc(2 * (size_t)nnz);                                   /* exactly nnz elements */
    CHECK(salr_oracle_encode(w_hat, rows, cols, bitmap, values, nnz, offsets) == 0);
    if (nnz > 0) CHECK(salr_oracle_encode(w_hat, rows, cols, bitmap, values, nnz - 1, offsets) == 3);  /* capacity */
    CHECK(salr_oracle_encode(w_hat, rows, cols, bitmap, values, nnz, offsets) == 0);
    CHECK(salr_oracle_decode(bitmap, values, offsets, rows, cols, back) == 0);
    CHECK(salr_oracle_decode_lut(bitmap, values, offsets, rows, cols, back2) == 0);
    for (size_t i = 0; i < n; ++i) {
        const uint16_t expect = (w_hat[i] & 0x7FFFu) ? w_hat[i] : 0;   /* -0.0 decodes to +0.0 */
        CHECK(back[i] == expect && back2[i] == expect);
    }
    CHECK(salr_oracle_mask_threshold(w, (int64_t)n, 0x3C00u, back) == 0);
    if (cols % 4 == 0) CHECK(salr_oracle_mask_nm(w, rows, cols, 2, 4, back) == 0);
    if (cols % 3 == 0) CHECK(salr_oracle_mask_nm(w, rows, cols, 1, 3, back) == 0);
    /* the packed values as 4-bit codes and back: exactly-sized code and scale buffers, odd counts, short last block */
    {
        uint8_t* codes = xmalloc((size_t)((nnz + 1) / 2));
        uint16_t* scales = xmalloc(2 * (size_t)((nnz + 63) / 64));
        uint16_t* deq = xmalloc(2 * (size_t)nnz);
        CHECK(salr_oracle_nf4_quantize(values, nnz, codes, scales) == 0);
        CHECK(salr_oracle_nf4_dequantize(codes, scales, nnz, deq) == 0);
        for (int64_t i = 0; i < nnz; ++i) CHECK((deq[i] & 0x7FFFu) <= (scales[i / 64] & 0x7FFFu));
        free(deq); free(scales); free(codes);
    }
    /* the layer on this weight: M = 3 rows of X, two adapters of ranks 2 and 1 stacked, and one by one */
    const int64_t M = 3, R = 3;
    uint16_t* x = xmalloc(2 * (size_t)(M * cols));
    uint16_t* a = xmalloc(2 * (size_t)(cols * R));
    uint16_t* b = xmalloc(2 * (size_t)(R * rows));
    double* y = xmalloc(8 * (size_t)(M * rows));
    for (int64_t i = 0; i < M * cols; ++i) x[i] = rnd_bf16();
    for (int64_t i = 0; i < cols * R; ++i) a[i] = rnd_bf16();
    for (int64_t i = 0; i < R * rows; ++i) b[i] = rnd_bf16();
    CHECK(salr_oracle_linear(x, M, cols, rows, w_hat, a, b, R, y) == 0);
    CHECK(salr_oracle_linear(x, M, cols, rows, w_hat, NULL, NULL, 0, y) == 0);
    CHECK(salr_oracle_adapter_accumulate(x, M, cols, rows, a, b, 0, y) == 0);
    uint16_t* a1 = xmalloc(2 * (size_t)cols);
    for (int64_t k = 0; k < cols; ++k) a1[k] = a[k * R + 2];
    CHECK(salr_oracle_adapter_accumulate(x, M, cols, rows, a1, b + 2 * rows, 1, y) == 0);
    free(a1); free(y); free(b); free(a); free(x);
    free(values); free(offsets); free(bitmap); free(back2); free(back); free(w_hat); free(w);
}

int main(void) {
    static const int64_t rows_list[] = {0, 1, 2, 5, 17};
    static const int64_t cols_list[] = {0, 1, 7, 8, 9, 31, 32, 33, 64, 96, 100, 255, 260};
    int shapes = 0;
    for (size_t i = 0; i < sizeof rows_list / sizeof rows_list[0]; ++i)
        for (size_t j = 0; j < sizeof cols_list / sizeof cols_list[0]; ++j) {
            const int64_t cols = cols_list[j];
            const int64_t keeps[] = {0, cols / 3, cols - cols / 2, cols};
            for (size_t q = 0; q < 4; ++q) {
                one_shape(rows_list[i], cols, keeps[q]);
                ++shapes;
            }
        }
    printf("oracle sanitize: %d shapes clean\n", shapes);
    return 0;
}
