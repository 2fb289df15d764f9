// Host-side declarations shared between the C boundary and the kernel files.
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stddef.h>
#include <stdint.h>

namespace salr {

hipError_t launch_encode(const uint16_t* w, int64_t rows, int64_t cols, uint32_t* bitmap, uint16_t* values,
                         int64_t capacity, uint32_t* row_offsets, hipStream_t stream);

hipError_t launch_decode(const uint32_t* bitmap, const uint16_t* values, const uint32_t* row_offsets, int64_t rows,
                         int64_t cols, uint16_t* out, hipStream_t stream);

hipError_t launch_mask_rows(const uint16_t* w, int64_t rows, int64_t cols, int64_t keep, uint16_t* out,
                            hipStream_t stream);

hipError_t launch_mask_nm(const uint16_t* w, int64_t rows, int64_t cols, int n_keep, int m_group, uint16_t* out,
                          hipStream_t stream);

hipError_t launch_residual(const uint16_t* w, const uint16_t* w_hat, int64_t rows, int64_t cols, uint16_t* e,
                           hipStream_t stream);

// Host arrays of n device pointers / ranks; R = sum of the ranks.
constexpr int kConcatBatch = 16;
hipError_t launch_concat(const uint16_t* const* a_list, const uint16_t* const* b_list, const int64_t* ranks, int64_t n,
                         int64_t K, int64_t N, int64_t R, uint16_t* a_cat, uint16_t* b_cat, hipStream_t stream);

// Residual adapter: rank-r factors of E [N, K] by subspace iteration with l = r + oversample columns (l <= 128)
constexpr int64_t kSvdMaxColumns = 128;
size_t residual_adapter_workspace_bytes(int64_t N, int64_t K, int64_t l);
hipError_t launch_residual_adapter(const uint16_t* e, int64_t N, int64_t K, int64_t r, int64_t l, int64_t iterations,
                                   const float* omega, uint16_t* a_res, uint16_t* b_res, float* sigma, void* workspace,
                                   hipStream_t stream);

// Columns of the bf16 workspace matrix T = X * A_cat: R rounded up to the MFMA k-step.
inline int64_t adapter_rank_padded(int64_t R) { return (R + 31) / 32 * 32; }

struct LinearArgs {
    const uint16_t* x;
    int64_t M, K, N;
    const uint32_t* bitmap;
    const uint16_t* values;
    const uint32_t* row_offsets;
    const uint16_t* a_cat;
    const uint16_t* b_cat;
    int64_t R;
    uint16_t* y;
    uint16_t* t;  // workspace (see linear_workspace_bytes)
    bool lean = false;  // large batches: no room for a decoded copy of the weight, take the fused kernel
    const uint32_t* slice_table = nullptr;  // optional: the layer's slice table (see kSliceTableSlices)
    bool build_table = false;  // slice_table points into the workspace and the adapter pre-kernel fills it in this call
    // QSALR on the large-batch path: `values` is null and the decode stage reads these (nnz values, 4-bit codes)
    const uint8_t* codes = nullptr;
    const uint16_t* scales = nullptr;
    int64_t nnz = 0;
};

// Slice table of a layer (a derived, kernel-private index; the three arrays of the format stay what is checked): for
// row n and slice w of the small-batch kernel's 8 wave slices (chunks [C w / 8, C (w + 1) / 8) of the row's
// C = ceil(K / 128) chunks of 128 columns) two uint32: the index in `values` of the slice's first value, and the most
// nonzeros any one chunk of the slice holds.
constexpr int kSliceTableSlices = 8;
inline size_t slice_table_bytes(int64_t N) { return (size_t)N * kSliceTableSlices * 2 * sizeof(uint32_t); }
hipError_t launch_build_slice_table(const uint32_t* bitmap, const uint32_t* row_offsets, int64_t N, int64_t K, uint32_t* table,
                                    hipStream_t stream);

// Optional events recorded around the fused kernel's launch (measurement hook of the boundary).
struct TimingEvents {
    hipEvent_t start = nullptr;
    hipEvent_t stop = nullptr;
};
extern thread_local TimingEvents g_timing_events;

// Launch `kernel`; when both events are set they receive the kernel's own begin/end timestamps.
#define SALR_LAUNCH(kernel, grid, block, stream, ev, ...)                                                    \
    do {                                                                                                      \
        if ((ev).start != nullptr && (ev).stop != nullptr)                                                    \
            hipExtLaunchKernelGGL(kernel, grid, block, 0, stream, (ev).start, (ev).stop, 0, __VA_ARGS__);     \
        else                                                                                                  \
            hipLaunchKernelGGL(kernel, grid, block, 0, stream, __VA_ARGS__);                                  \
    } while (0)

// Small-batch path: M <= kStreamMaxM; T = X * A_cat arrives as kStreamTSlices split-K partials (fp32).
constexpr int64_t kStreamMaxM = 64;
constexpr int kStreamTSlices = 16;
constexpr int kMaxRankPadded = 256;  // R <= 256: pitch of the T tile the streaming kernels keep in LDS

// Large-batch path: M > kStreamMaxM decodes the weight once into a dense scratch matrix, then runs a dense MFMA
// GEMM on it (k-steps of 64).
inline bool uses_twostage(int64_t M, int64_t K) { return M > kStreamMaxM && K >= 64 && K % 64 == 0; }

inline size_t round_up_256(size_t b) { return (b + 255) / 256 * 256; }

// Workspace layout of the large-batch paths (M > kStreamMaxM): T [M, Rpad] bf16, the transposed padded adapter
// a_t [Rpad, K] bf16, the split-K partials of T, then (two-stage path only) the decoded weight [N, K] bf16 and the
// split-K partials of Y; each 256-byte aligned.
inline size_t adapter_t_bytes(int64_t M, int64_t R) {
    return R > 0 ? round_up_256((size_t)M * (size_t)adapter_rank_padded(R) * sizeof(uint16_t)) : 0;
}
inline size_t adapter_at_bytes(int64_t K, int64_t R) {
    return R > 0 ? round_up_256((size_t)K * (size_t)adapter_rank_padded(R) * sizeof(uint16_t)) : 0;
}
// T = X * A_cat splits K over workgroups (fp32 partials [ksplit, M, Rpad], added up in a fixed order).
inline int adapter_rows_per_block(int64_t M) { return M >= 4096 ? 256 : 64; }
inline int adapter_ksplit(int64_t M, int64_t K) {
    const int64_t rows = adapter_rows_per_block(M);
    const int64_t blocks = (M + rows - 1) / rows, units = K / 32;
    int s = 1;
    while (s < 64 && blocks * s * 2 <= 1024 && units / (s * 2) >= 8) s *= 2;
    return s;
}
// Up to kAdapterSmallM rows the small-batch pre-kernel computes T (one launch of many short workgroups reading A_cat as it
// is, kStreamTSlices fp32 partials) and the reducing pass sums them; above, the transposing pass + tall product + sum.
constexpr int64_t kAdapterSmallM = 1024;
inline bool adapter_uses_prekernel(int64_t M) { return M <= kAdapterSmallM; }
inline size_t adapter_partial_bytes(int64_t M, int64_t K, int64_t R) {
    if (R > 0 && adapter_uses_prekernel(M))
        return round_up_256((size_t)kStreamTSlices * (size_t)M * (size_t)adapter_rank_padded(R) * sizeof(float));
    const int s = adapter_ksplit(M, K);
    return (R > 0 && s > 1) ? round_up_256((size_t)s * (size_t)M * (size_t)adapter_rank_padded(R) * sizeof(float)) : 0;
}
inline size_t twostage_dense_offset(int64_t M, int64_t K, int64_t R) {
    return adapter_t_bytes(M, R) + adapter_at_bytes(K, R) + adapter_partial_bytes(M, K, R);
}

// Split of K over workgroups in the dense stage of the two-stage path: used when the 256 x 128 output tiles are
// too few for the 256 CUs.  Needs N % 4 == 0 (vector stores of the reducing pass) and an even split of the 64-wide
// k-steps; the fp32 partial tiles [ksplit, M, N] follow the dense weight in the workspace.
inline int dense_ksplit(int64_t M, int64_t K, int64_t N) {
    const int64_t tiles = ((M + 255) / 256) * ((N + 127) / 128);
    const int64_t steps = K / 64;
    if (tiles >= 128 || N % 4 != 0) return 1;
    int s = 1;
    while (s < 8 && tiles * s * 2 <= 256 && steps % (s * 2) == 0 && steps / (s * 2) >= 4) s *= 2;
    return s;
}

// Row-tiled streaming path (one pass over the compressed weight, X shared by the 128 rows of a workgroup): batches of
// 9 to 128 tokens on layers whose rows come in whole 128-column chunks.  K is split over workgroups when the
// 128-row tiles alone would leave most of the chip idle; the fp32 partial outputs [ksplit, M, N] follow T in the
// workspace.  Measured against the other paths on the Llama-3 shapes: ahead from 33 tokens on everywhere (by 15 to
// 45 %), from 9 tokens on where the layer has thousands of rows; below that the small-batch kernel, whose waves
// run independently of each other, is as fast or faster.
constexpr int64_t kRowtileMaxM = 128;
inline int rowtile_ksplit(int64_t M, int64_t K, int64_t N) {
    const int64_t tiles = (N + 127) / 128, chunks = K / 128;
    if (N % 4 != 0) return 1;   // the reducing pass stores four outputs per thread
    // up to 64 tokens two workgroups share a CU (and hide each other's barriers), above that one fills it
    const int64_t enough = M <= 64 ? 448 : 224;
    int s = 1;
    while (s < 16 && tiles * s < enough && chunks / (s * 2) >= 4) s *= 2;
    return s;
}
inline bool rowtile_possible(int64_t M, int64_t K) { return M <= kRowtileMaxM && K >= 128 && K % 128 == 0; }
inline bool uses_rowtile(int64_t M, int64_t K, int64_t N) {
    if (!rowtile_possible(M, K)) return false;
    if (N % 4 != 0 && N < 64 * 128) return false;   // K cannot be split and the row tiles are few
    return M > 32 || (M > 8 && N >= 8192);
}
// T of the row-tiled path: the split-K partials of the small-batch pre-kernel
inline size_t rowtile_t_bytes(int64_t M, int64_t K, int64_t R) {
    if (R <= 0) return 0;
    return round_up_256((size_t)kStreamTSlices * (size_t)M * (size_t)adapter_rank_padded(R) * sizeof(float));
}
inline size_t rowtile_workspace_bytes(int64_t M, int64_t K, int64_t N, int64_t R) {
    const int ks = rowtile_ksplit(M, K, N);
    return rowtile_t_bytes(M, K, R) + (ks > 1 ? round_up_256((size_t)ks * (size_t)M * (size_t)N * sizeof(float)) : 0);
}

// The linear on 2:4-masked weights (sparse matrix-core instructions, no decode stage): same tiling, K split and
// workspace as the row-tiled path; other shapes go through launch_linear.
inline bool uses_2of4_kernel(int64_t M, int64_t K, int64_t N) {
    return rowtile_possible(M, K) && !(N % 4 != 0 && N < 64 * 128);
}
// above 128 tokens: a tiled GEMM on the sparse MFMA (k-steps of 64 columns, four outputs per store); its workspace is
// the T part of the large-batch layout, which the general call's workspace contains
// Taken where its tiles fill the chip without crowding it (measured on the Llama-3 shapes: 14 to 32 % ahead of the
// decode + dense GEMM path there): >= 192 tiles of 256 x 256 (one workgroup per CU); on layers of >= 8192 rows from
// 128 tiles of 128 x 128 on; on smaller layers with 192 to 320 of them (about one workgroup per CU: with two the
// 128 x 128 tiles, which read more LDS per flop, are level with the other path, and below 192 the chip is not full).
constexpr int64_t kGemm2of4BigTilesMin = 192;
inline bool uses_2of4_gemm(int64_t M, int64_t K, int64_t N) {
    if (!(M > kRowtileMaxM && K >= 64 && K % 64 == 0 && N % 4 == 0)) return false;
    const int64_t big = ((M + 255) / 256) * ((N + 255) / 256), small = ((M + 127) / 128) * ((N + 127) / 128);
    if (big >= kGemm2of4BigTilesMin) return true;
    return N >= 8192 ? small >= 128 : (small >= 192 && small <= 320);
}
hipError_t launch_check_2of4(const uint32_t* bitmap, int64_t rows, int64_t cols, uint32_t* flag, hipStream_t stream);

// decode-sized batches (M <= 16, K % 128 == 0, 12288 <= K <= 32768): the streaming kernel that reads every bitmap word once
bool linear_slice_takes(int64_t M, int64_t K, int64_t N);
// Shapes that launch_linear sends down the two-stage path when the workspace has room for the decoded copy
inline bool linear_takes_twostage(int64_t M, int64_t K, int64_t N) {
    return M > kStreamMaxM && !uses_rowtile(M, K, N) && uses_twostage(M, K);
}
// A call without a slice table of the caller's builds one for itself where the adapter pre-kernel runs anyway (R > 0)
// and a kernel that gains more from it than the build costs follows: the small-batch streaming kernel on rows of whole
// chunks, and the row-tiled kernel when its split of K starts where table slices do.  (The long-row kernel reads a
// caller's table but gains less from it than reading the bitmap a second time costs: 70B down_proj M = 1, kernel +
// pre-kernel 87.3 us without, 89.3 us with.)  The table sits behind the rest of the workspace.
inline bool builds_slice_table(int64_t M, int64_t K, int64_t N, int64_t R) {
    if (R <= 0 || M <= 0 || N <= 0 || K < 128 || K % 128 != 0) return false;
    if (uses_rowtile(M, K, N)) return kSliceTableSlices % rowtile_ksplit(M, K, N) == 0;
    if (linear_slice_takes(M, K, N)) return false;
    return M <= kStreamMaxM;
}
inline size_t linear_workspace_bytes_without_table(int64_t M, int64_t K, int64_t N, int64_t R);
// Workspace the linear needs: the small-batch path keeps fp32 split-K partials of T; the others see above.
inline size_t linear_workspace_bytes(int64_t M, int64_t K, int64_t N, int64_t R) {
    const size_t b = linear_workspace_bytes_without_table(M, K, N, R);
    return builds_slice_table(M, K, N, R) ? b + round_up_256(slice_table_bytes(N)) : b;
}
inline size_t linear_workspace_bytes_without_table(int64_t M, int64_t K, int64_t N, int64_t R) {
    if (M <= 0 || N <= 0) return 0;
    if (uses_rowtile(M, K, N)) return rowtile_workspace_bytes(M, K, N, R);
    if (M <= kStreamMaxM)
        return R > 0 ? round_up_256((size_t)kStreamTSlices * (size_t)M * (size_t)adapter_rank_padded(R) * sizeof(float)) : 0;
    size_t b = twostage_dense_offset(M, K, R);
    if (uses_twostage(M, K)) {
        b += round_up_256((size_t)N * (size_t)K * sizeof(uint16_t));
        const int ks = dense_ksplit(M, K, N);
        if (ks > 1) b += round_up_256((size_t)ks * (size_t)M * (size_t)N * sizeof(float));
    }
    return b;
}

// The least the layer runs with: where the preferred path decodes the weight into the workspace (large batches), the
// fused kernel needs the adapter part only.
inline size_t linear_workspace_bytes_lean(int64_t M, int64_t K, int64_t N, int64_t R) {
    if (M <= 0 || N <= 0) return 0;
    if (!uses_rowtile(M, K, N) && M > kStreamMaxM && uses_twostage(M, K)) return twostage_dense_offset(M, K, R);
    return linear_workspace_bytes(M, K, N, R);
}

// Backward pass of the layer: dx [M, K], da [K, R], db [R, N]; any of them may be null (not computed)
size_t linear_backward_workspace_bytes(int64_t M, int64_t K, int64_t N, int64_t R, bool want_dx, bool want_dadb);
hipError_t launch_linear_backward(const uint16_t* x, const uint16_t* dy, int64_t M, int64_t K, int64_t N,
                                  const uint32_t* bitmap, const uint16_t* values, const uint32_t* row_offsets,
                                  const uint16_t* a_cat, const uint16_t* b_cat, int64_t R, uint16_t* dx, uint16_t* da,
                                  uint16_t* db, void* workspace, hipStream_t stream);

// QSALR: the packed values as 4-bit NormalFloat codes, one bf16 scale per 64 values
hipError_t launch_nf4_quantize(const uint16_t* values, int64_t count, uint8_t* codes, uint16_t* scales, hipStream_t stream);
hipError_t launch_nf4_dequantize(const uint8_t* codes, const uint16_t* scales, int64_t count, uint16_t* out, hipStream_t stream);
// bytes of the dequantised packed values at the start of the QSALR layer's workspace (16-byte vectors, 256-byte aligned)
inline size_t qsalr_values_bytes(int64_t nnz) { return round_up_256((size_t)((nnz + 7) / 8 * 8) * sizeof(uint16_t)); }
// QSALR at small batches (M <= 64, K a multiple of 128, nnz > 0): the streaming kernel that reads the 4-bit codes itself.
// Its workspace: the split-K partials of T (with adapters), then the call's slice table; args.t and args.slice_table
// point at the two, args.values is not used.
bool linear_nf4_takes(int64_t M, int64_t K, int64_t N, int64_t nnz);
size_t linear_nf4_table_offset(int64_t M, int64_t R);
size_t linear_nf4_workspace_bytes(int64_t M, int64_t N, int64_t R);
hipError_t launch_linear_nf4(const LinearArgs& args, const uint8_t* codes, const uint16_t* scales, int64_t nnz,
                             hipStream_t stream, const TimingEvents& ev);

// QSALR: decode from the 4-bit codes (the row-per-workgroup decode kernel's limits: cols % 8 == 0, 16-byte aligned out)
bool decode_nf4_takes(int64_t rows, int64_t cols, int64_t nnz, const void* codes, const void* out);
hipError_t launch_decode_nf4(const uint32_t* bitmap, const uint8_t* codes, const uint16_t* scales, int64_t nnz,
                             const uint32_t* row_offsets, int64_t rows, int64_t cols, uint16_t* out, hipStream_t stream);
// decode into the transposed dense matrix out_t [cols, rows] (cols a multiple of 128, 16-byte aligned buffers)
bool decode_transposed_takes(int64_t rows, int64_t cols, const void* values, const void* out_t);
hipError_t launch_decode_transposed(const uint32_t* bitmap, const uint16_t* values, const uint32_t* row_offsets, int64_t rows,
                                    int64_t cols, uint16_t* out_t, hipStream_t stream);
hipError_t launch_linear(const LinearArgs& args, hipStream_t stream);
// count bf16 zeros (+0.0) at out
hipError_t launch_fill_zero(uint16_t* out, int64_t count, hipStream_t stream);
hipError_t launch_linear_stream(const LinearArgs& args, hipStream_t stream, const TimingEvents& ev);
hipError_t launch_linear_slice(const LinearArgs& args, hipStream_t stream, const TimingEvents& ev);
hipError_t launch_linear_twostage(const LinearArgs& args, hipStream_t stream, const TimingEvents& ev);
// the same shapes without a decoded copy of the weight: decode stage and MFMA stage in one kernel (K % 64 == 0)
hipError_t launch_linear_tiled(const LinearArgs& args, hipStream_t stream, const TimingEvents& ev);
hipError_t launch_linear_rowtile(const LinearArgs& args, hipStream_t stream, const TimingEvents& ev);
hipError_t launch_linear_2of4(const LinearArgs& args, hipStream_t stream, const TimingEvents& ev);
hipError_t launch_gemm_2of4(const LinearArgs& args, hipStream_t stream, const TimingEvents& ev);
// split-K partials of T = X * A_cat (small batches): fp32 [kStreamTSlices, M, Rpad] at the start of the workspace
void launch_adapter_partial(const LinearArgs& args, hipStream_t stream);
// the same into `partial` [kStreamTSlices, M, Rpad] (no slice table)
void launch_adapter_partial_to(const LinearArgs& args, float* partial, hipStream_t stream);
// T = X * A_cat in bf16 [M, Rpad] at the start of the workspace (every path with M > kStreamMaxM)
void launch_adapter_t(const LinearArgs& args, hipStream_t stream);
// x [M, K] bf16 times the transpose of a_t [Rpad, K] bf16 (Rpad % 32 == 0, K % 32 == 0), K split over `ksplit`
// slices: bf16 t [M, Rpad] (one slice, !keep_fp32) or fp32 partial [ksplit, M, Rpad]
// Products that contract over the rows of in [M, C] (M % 32 == 0): partial [ksplit][C][Rpad] fp32; tn_ksplit picks the
// split of M (about four workgroups per CU, at least two steps of 32 rows each)
inline int tn_ksplit(int64_t C, int64_t M) {
    const int64_t blocks = (C + 63) / 64, steps = M / 32;
    int s = 1;
    while (s < 64 && blocks * s * 2 <= 1024 && steps / (s * 2) >= 2) s *= 2;
    return s;
}
void launch_tall_tn(const uint16_t* in, int64_t M, int64_t C, const uint16_t* s_t, int Rpad, int ksplit, float* partial,
                    hipStream_t stream);
void launch_tall_product(const uint16_t* x, int64_t M, int64_t K, const uint16_t* a_t, int Rpad, int ksplit, uint16_t* t,
                         float* partial, bool keep_fp32, hipStream_t stream);
// a_t [Rpad, K] = A_cat [K, R]^T, rows R .. Rpad - 1 zero
void launch_adapter_transpose(const uint16_t* a_cat, int64_t K, int R, int Rpad, uint16_t* a_t, hipStream_t stream);
// out [C, R] = in [R, C]^T (bf16); R <= 65535 * 32
void launch_transpose_bf16(const uint16_t* in, int64_t R, int64_t C, uint16_t* out, hipStream_t stream);
// y [M, N] = x [M, K] * wd [N, K]^T (+ t [M, Rpad] * b_cat [R, N], pitch N, when R > 0): the dense MFMA stage with its
// tile choice; K % 64 == 0; partial holds dense_ksplit(M, K, N) fp32 copies of y when that is > 1
void launch_dense_stage(const uint16_t* x, int64_t M, int64_t K, int64_t N, const uint16_t* wd, const uint16_t* t,
                        const uint16_t* b_cat, int R, int Rpad, uint16_t* y, float* partial, const TimingEvents& ev,
                        hipStream_t stream);
// out[i] = bf16(sum over z < ksplit of partial[z * count + i]); count % 4 == 0
void launch_splitk_reduce(const float* partial, int64_t count, int ksplit, uint16_t* out, hipStream_t stream);

}  // namespace salr
