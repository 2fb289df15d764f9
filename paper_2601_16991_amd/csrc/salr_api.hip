// C boundary: argument validation on the host, then kernels enqueued on the caller's stream.
#include "../../include/salr.h"

#include "salr_internal.hpp"

#include <atomic>

namespace {

// Scratch of salr_sparse_lowrank_linear_noalloc: part of the code object, so every GPU that loads the library holds
// its own copy at its own address.  In host code the name stands for the symbol, not for device memory: the address
// comes from hipGetSymbolAddress, once per device, and only that address is handed to kernels.
static __device__ __align__(256) unsigned char scratch[SALR_NOALLOC_SCRATCH_BYTES];
constexpr int kMaxDevices = 64;
std::atomic<void*> g_scratch_ptr[kMaxDevices];

// Address of the current device's copy of `scratch` (looked up on the first call on that device).
hipError_t scratch_of_current_device(void** out) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    void* p = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (p == nullptr) {
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (p == nullptr) return hipErrorInvalidSymbol;
        g_scratch_ptr[dev].store(p, std::memory_order_release);   // racing first calls store the same address
    }
    *out = p;
    return hipSuccess;
}

constexpr int64_t kMaxRows = 2147483647LL;        // gridDim.x
constexpr int64_t kMaxCols = 2147483647LL - 31;   // so that ceil(cols/32)*32 stays in int32 range
constexpr int64_t kMaxRank = 256;
constexpr int64_t kMaxM = 65535LL * 64;           // gridDim.y of the generic kernel
constexpr int64_t kMaxSvdDim = 65535LL * 32;      // gridDim.y of the transposing kernel

// QSALR calls whose decode stage reads the 4-bit codes itself: the two-stage path (large batches, K % 64 == 0) within the
// row decode kernel's limits (rows of at most 524288 columns); the workspace is then the plain layer's.
bool qsalr_decodes_codes(int64_t M, int64_t K, int64_t N, int64_t nnz) {
    return nnz > 0 && K > 0 && salr::linear_takes_twostage(M, K, N) && (K / 32 + 15) / 16 <= 1024;
}

}  // namespace

extern "C" {

const char* salr_status_string(salr_status_t status) {
    switch (status) {
        case SALR_OK: return "ok";
        case SALR_ERR_INVALID_ARG: return "invalid argument (null pointer or negative size)";
        case SALR_ERR_SHAPE: return "sizes violate a constraint of this entry point";
        case SALR_ERR_CAPACITY: return "buffer or workspace too small";
        case SALR_ERR_UNSUPPORTED: return "unsupported request";
        case SALR_ERR_HIP: return "HIP runtime error while enqueuing";
    }
    return "unknown status";
}

int64_t salr_bitmap_words_per_row(int64_t cols) { return cols < 0 ? -1 : (cols + 31) / 32; }

salr_status_t salr_magnitude_mask_rows(const uint16_t* w, int64_t rows, int64_t cols, int64_t keep, uint16_t* w_hat,
                                       void* stream) {
    if (rows < 0 || cols < 0 || keep < 0 || keep > cols) return SALR_ERR_INVALID_ARG;
    if (rows > 0 && cols > 0 && (!w || !w_hat)) return SALR_ERR_INVALID_ARG;
    if (rows > kMaxRows || cols > kMaxCols) return SALR_ERR_SHAPE;
    hipError_t e = salr::launch_mask_rows(w, rows, cols, keep, w_hat, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? SALR_OK : SALR_ERR_HIP;
}

salr_status_t salr_magnitude_mask_nm(const uint16_t* w, int64_t rows, int64_t cols, int64_t n_keep, int64_t m_group,
                                     uint16_t* w_hat, void* stream) {
    if (rows < 0 || cols < 0 || m_group < 1 || n_keep < 0 || n_keep > m_group) return SALR_ERR_INVALID_ARG;
    if (rows > 0 && cols > 0 && (!w || !w_hat)) return SALR_ERR_INVALID_ARG;
    if (m_group > 64) return SALR_ERR_UNSUPPORTED;
    if (rows > kMaxRows || cols > kMaxCols || cols % m_group != 0) return SALR_ERR_SHAPE;
    if (cols > 0 && rows > (kMaxRows * 256) / (cols / m_group)) return SALR_ERR_SHAPE;  // one thread per group
    hipError_t e = salr::launch_mask_nm(w, rows, cols, (int)n_keep, (int)m_group, w_hat,
                                        static_cast<hipStream_t>(stream));
    return e == hipSuccess ? SALR_OK : SALR_ERR_HIP;
}

salr_status_t salr_encode_bitmap(const uint16_t* w_dense, int64_t rows, int64_t cols, uint32_t* bitmap,
                                 uint16_t* values, int64_t values_capacity, uint32_t* row_offsets, void* stream) {
    if (rows < 0 || cols < 0) return SALR_ERR_INVALID_ARG;
    if (!row_offsets) return SALR_ERR_INVALID_ARG;
    if (rows > 0 && cols > 0 && (!w_dense || !bitmap)) return SALR_ERR_INVALID_ARG;
    if (values && values_capacity < 0) return SALR_ERR_INVALID_ARG;
    if (rows > kMaxRows || cols > kMaxCols) return SALR_ERR_SHAPE;
    if (cols > 0 && rows > (int64_t)0xFFFFFFFFLL / cols) return SALR_ERR_SHAPE;  // nnz must fit uint32
    hipError_t e = salr::launch_encode(w_dense, rows, cols, bitmap, values, values_capacity, row_offsets,
                                       static_cast<hipStream_t>(stream));
    return e == hipSuccess ? SALR_OK : SALR_ERR_HIP;
}

salr_status_t salr_decode(const uint32_t* bitmap, const uint16_t* values, const uint32_t* row_offsets, int64_t rows,
                          int64_t cols, uint16_t* w_dense_out, void* stream) {
    if (rows < 0 || cols < 0) return SALR_ERR_INVALID_ARG;
    if (rows > 0 && cols > 0 && (!bitmap || !row_offsets || !w_dense_out)) return SALR_ERR_INVALID_ARG;
    if (rows > kMaxRows || cols > kMaxCols) return SALR_ERR_SHAPE;
    hipError_t e = salr::launch_decode(bitmap, values, row_offsets, rows, cols, w_dense_out,
                                       static_cast<hipStream_t>(stream));
    return e == hipSuccess ? SALR_OK : SALR_ERR_HIP;
}

salr_status_t salr_residual(const uint16_t* w, const uint16_t* w_hat, int64_t rows, int64_t cols, uint16_t* e, void* stream) {
    if (rows < 0 || cols < 0) return SALR_ERR_INVALID_ARG;
    if (rows > 0 && cols > 0 && (!w || !w_hat || !e)) return SALR_ERR_INVALID_ARG;
    if (rows > kMaxRows || cols > kMaxCols) return SALR_ERR_SHAPE;
    if (cols > 0 && rows > (kMaxRows * 2048) / cols) return SALR_ERR_SHAPE;   // 2048 elements per workgroup
    hipError_t err = salr::launch_residual(w, w_hat, rows, cols, e, static_cast<hipStream_t>(stream));
    return err == hipSuccess ? SALR_OK : SALR_ERR_HIP;
}

salr_status_t salr_concat_adapters(const uint16_t* const* a_list, const uint16_t* const* b_list, const int64_t* ranks,
                                   int64_t n, int64_t K, int64_t N, uint16_t* a_cat, uint16_t* b_cat, void* stream) {
    if (n < 0 || K < 0 || N < 0) return SALR_ERR_INVALID_ARG;
    if (n == 0) return SALR_OK;
    if (!a_list || !b_list || !ranks) return SALR_ERR_INVALID_ARG;
    if (K > kMaxCols || N > kMaxRows) return SALR_ERR_SHAPE;
    int64_t R = 0;
    for (int64_t i = 0; i < n; ++i) {
        if (ranks[i] < 0) return SALR_ERR_INVALID_ARG;
        if (ranks[i] > 0 && ((K > 0 && !a_list[i]) || (N > 0 && !b_list[i]))) return SALR_ERR_INVALID_ARG;
        R += ranks[i];
        if (R > 65535) return SALR_ERR_SHAPE;   // rows of B_cat are a grid dimension
    }
    if (R > 0 && K > (kMaxRows * 256) / R) return SALR_ERR_SHAPE;   // one thread per element of A_cat
    if (R == 0) return SALR_OK;
    if ((K > 0 && !a_cat) || (N > 0 && !b_cat)) return SALR_ERR_INVALID_ARG;
    hipError_t err = salr::launch_concat(a_list, b_list, ranks, n, K, N, R, a_cat, b_cat, static_cast<hipStream_t>(stream));
    return err == hipSuccess ? SALR_OK : SALR_ERR_HIP;
}

size_t salr_residual_adapter_workspace_bytes(int64_t N, int64_t K, int64_t r, int64_t oversample) {
    if (N <= 0 || K <= 0 || r <= 0 || oversample < 0 || N % 32 != 0 || K % 32 != 0 || N > kMaxSvdDim || K > kMaxSvdDim) return 0;
    if (r + oversample > salr::kSvdMaxColumns || r + oversample > (N < K ? N : K)) return 0;
    return salr::residual_adapter_workspace_bytes(N, K, r + oversample);
}

salr_status_t salr_residual_adapter(const uint16_t* e, int64_t N, int64_t K, int64_t r, int64_t oversample,
                                    int64_t power_iterations, const float* omega, uint16_t* a_res, uint16_t* b_res,
                                    float* sigma, void* workspace, size_t workspace_bytes, void* stream) {
    if (N < 0 || K < 0 || r < 0 || oversample < 0 || power_iterations < 0) return SALR_ERR_INVALID_ARG;
    if (N == 0 || K == 0 || r == 0) return SALR_OK;
    if (!e || !omega || !a_res || !b_res) return SALR_ERR_INVALID_ARG;
    if (N % 32 != 0 || K % 32 != 0 || N > kMaxSvdDim || K > kMaxSvdDim) return SALR_ERR_SHAPE;
    if (r + oversample > (N < K ? N : K)) return SALR_ERR_SHAPE;
    if (r + oversample > salr::kSvdMaxColumns || power_iterations > 64) return SALR_ERR_UNSUPPORTED;
    const size_t need = salr::residual_adapter_workspace_bytes(N, K, r + oversample);
    if (!workspace || workspace_bytes < need) return SALR_ERR_CAPACITY;
    hipError_t err = salr::launch_residual_adapter(e, N, K, r, r + oversample, power_iterations, omega, a_res, b_res, sigma,
                                                   workspace, static_cast<hipStream_t>(stream));
    return err == hipSuccess ? SALR_OK : SALR_ERR_HIP;
}

size_t salr_linear_workspace_bytes(int64_t M, int64_t K, int64_t N, int64_t R) {
    if (M <= 0 || K < 0 || N <= 0 || R < 0 || R > kMaxRank || K % 32 != 0) return 0;
    return salr::linear_workspace_bytes(M, K, N, R);
}

size_t salr_linear_workspace_bytes_min(int64_t M, int64_t K, int64_t N, int64_t R) {
    if (M <= 0 || K < 0 || N <= 0 || R < 0 || R > kMaxRank || K % 32 != 0) return 0;
    return salr::linear_workspace_bytes_lean(M, K, N, R);
}

size_t salr_slice_table_bytes(int64_t N, int64_t K) {
    if (N <= 0 || K < 0 || K % 32 != 0 || N > kMaxRows || K > kMaxCols) return 0;
    return salr::slice_table_bytes(N);
}

salr_status_t salr_build_slice_table(const uint32_t* bitmap, const uint32_t* row_offsets, int64_t N, int64_t K,
                                     uint32_t* slice_table, size_t slice_table_bytes, void* stream) {
    if (N < 0 || K < 0) return SALR_ERR_INVALID_ARG;
    if (N == 0) return SALR_OK;
    if (!row_offsets || !slice_table || (K > 0 && !bitmap)) return SALR_ERR_INVALID_ARG;
    if (K % 32 != 0) return SALR_ERR_SHAPE;
    if (N > kMaxRows || K > kMaxCols) return SALR_ERR_SHAPE;
    if (slice_table_bytes < salr::slice_table_bytes(N)) return SALR_ERR_CAPACITY;
    hipError_t e = salr::launch_build_slice_table(bitmap, row_offsets, N, K, slice_table, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? SALR_OK : SALR_ERR_HIP;
}

static salr_status_t linear_entry(const uint16_t* x, int64_t M, int64_t K, int64_t N, const uint32_t* bitmap,
                                  const uint16_t* values, const uint32_t* row_offsets, const uint32_t* slice_table,
                                  const uint16_t* a_cat, const uint16_t* b_cat, int64_t R, uint16_t* y, void* workspace,
                                  size_t workspace_bytes, void* stream, const uint8_t* codes = nullptr,
                                  const uint16_t* scales = nullptr, int64_t nnz = 0) {
    if (M < 0 || K < 0 || N < 0 || R < 0) return SALR_ERR_INVALID_ARG;
    if (M == 0 || N == 0) return SALR_OK;
    if (!y) return SALR_ERR_INVALID_ARG;
    if (K > 0 && (!x || !bitmap || !row_offsets)) return SALR_ERR_INVALID_ARG;
    if (K > 0 && R > 0 && (!a_cat || !b_cat)) return SALR_ERR_INVALID_ARG;
    if (K % 32 != 0) return SALR_ERR_SHAPE;
    if (N > kMaxRows || K > kMaxCols) return SALR_ERR_SHAPE;
    if (R > kMaxRank || M > kMaxM) return SALR_ERR_UNSUPPORTED;
    if (K == 0) {   // empty contraction: X W-hat^T and X A_cat are empty sums, so Y = 0; no operand is read
        hipError_t e0 = salr::launch_fill_zero(y, M * N, static_cast<hipStream_t>(stream));
        return e0 == hipSuccess ? SALR_OK : SALR_ERR_HIP;
    }
    const size_t need = salr_linear_workspace_bytes(M, K, N, R);
    const size_t least = salr::linear_workspace_bytes_lean(M, K, N, R);
    const size_t have = workspace ? workspace_bytes : 0;
    if (have < least) return SALR_ERR_CAPACITY;
    salr::LinearArgs a;
    a.x = x; a.M = M; a.K = K; a.N = N;
    a.bitmap = bitmap; a.values = values; a.row_offsets = row_offsets;
    a.a_cat = a_cat; a.b_cat = b_cat; a.R = R;
    a.y = y;
    a.t = static_cast<uint16_t*>(workspace);
    a.lean = have < need;   // no room for the decoded copy: decode stage and MFMA stage in one kernel
    a.slice_table = slice_table;
    if (codes != nullptr) {   // QSALR on the two-stage path (the caller has checked that this call takes it)
        if (!salr::linear_takes_twostage(M, K, N) || a.lean) return SALR_ERR_UNSUPPORTED;
        a.values = nullptr; a.codes = codes; a.scales = scales; a.nnz = nnz;
    }
    if (!slice_table && have >= need && salr::builds_slice_table(M, K, N, R)) {   // none of the caller's: this call's own
        a.slice_table = reinterpret_cast<const uint32_t*>(static_cast<char*>(workspace) +
                                                          salr::linear_workspace_bytes_without_table(M, K, N, R));
        a.build_table = true;
    }
    hipError_t e = salr::launch_linear(a, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? SALR_OK : SALR_ERR_HIP;
}

salr_status_t salr_sparse_lowrank_linear(const uint16_t* x, int64_t M, int64_t K, int64_t N, const uint32_t* bitmap,
                                         const uint16_t* values, const uint32_t* row_offsets, const uint16_t* a_cat,
                                         const uint16_t* b_cat, int64_t R, uint16_t* y, void* workspace,
                                         size_t workspace_bytes, void* stream) {
    return linear_entry(x, M, K, N, bitmap, values, row_offsets, nullptr, a_cat, b_cat, R, y, workspace, workspace_bytes, stream);
}

salr_status_t salr_sparse_lowrank_linear_prepared(const uint16_t* x, int64_t M, int64_t K, int64_t N, const uint32_t* bitmap,
                                                  const uint16_t* values, const uint32_t* row_offsets,
                                                  const uint32_t* slice_table, const uint16_t* a_cat, const uint16_t* b_cat,
                                                  int64_t R, uint16_t* y, void* workspace, size_t workspace_bytes,
                                                  void* stream) {
    if (M > 0 && N > 0 && K > 0 && !slice_table) return SALR_ERR_INVALID_ARG;
    return linear_entry(x, M, K, N, bitmap, values, row_offsets, slice_table, a_cat, b_cat, R, y, workspace, workspace_bytes,
                        stream);
}

salr_status_t salr_sparse_lowrank_linear_noalloc(const uint16_t* x, int64_t M, int64_t K, int64_t N, const uint32_t* bitmap,
                                                 const uint16_t* values, const uint32_t* row_offsets,
                                                 const uint16_t* a_cat, const uint16_t* b_cat, int64_t R, uint16_t* y,
                                                 void* stream) {
    if (M < 0 || K < 0 || N < 0 || R < 0) return SALR_ERR_INVALID_ARG;
    if (M == 0 || N == 0) return SALR_OK;
    if (K % 32 != 0) return SALR_ERR_SHAPE;
    if (R > kMaxRank) return SALR_ERR_UNSUPPORTED;
    size_t need = K > 0 ? salr::linear_workspace_bytes(M, K, N, R) : 0;
    if (need > SALR_NOALLOC_SCRATCH_BYTES && K > 0) need = salr::linear_workspace_bytes_lean(M, K, N, R);   // large batches: fused kernel
    if (need > SALR_NOALLOC_SCRATCH_BYTES) return SALR_ERR_CAPACITY;
    void* ws = nullptr;
    if (need > 0 && scratch_of_current_device(&ws) != hipSuccess) return SALR_ERR_HIP;
    return salr_sparse_lowrank_linear(x, M, K, N, bitmap, values, row_offsets, a_cat, b_cat, R, y, ws, need, stream);
}

salr_status_t salr_nf4_quantize_values(const uint16_t* values, int64_t count, uint8_t* codes, uint16_t* scales, void* stream) {
    if (count < 0) return SALR_ERR_INVALID_ARG;
    if (count == 0) return SALR_OK;
    if (!values || !codes || !scales) return SALR_ERR_INVALID_ARG;
    if (count > (int64_t)0xFFFFFFFFLL) return SALR_ERR_SHAPE;
    hipError_t e = salr::launch_nf4_quantize(values, count, codes, scales, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? SALR_OK : SALR_ERR_HIP;
}

salr_status_t salr_nf4_dequantize_values(const uint8_t* codes, const uint16_t* scales, int64_t count, uint16_t* values_out,
                                         void* stream) {
    if (count < 0) return SALR_ERR_INVALID_ARG;
    if (count == 0) return SALR_OK;
    if (!codes || !scales || !values_out) return SALR_ERR_INVALID_ARG;
    if (count > (int64_t)0xFFFFFFFFLL) return SALR_ERR_SHAPE;
    hipError_t e = salr::launch_nf4_dequantize(codes, scales, count, values_out, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? SALR_OK : SALR_ERR_HIP;
}

size_t salr_qsalr_linear_workspace_bytes(int64_t M, int64_t K, int64_t N, int64_t R, int64_t nnz) {
    if (M <= 0 || K < 0 || N <= 0 || R < 0 || R > kMaxRank || K % 32 != 0 || nnz < 0) return 0;
    if (salr::linear_nf4_takes(M, K, N, nnz)) return salr::linear_nf4_workspace_bytes(M, N, R);   // no bf16 copy of the values
    if (qsalr_decodes_codes(M, K, N, nnz)) return salr::linear_workspace_bytes(M, K, N, R);      // nor here
    return salr::qsalr_values_bytes(nnz) + salr::linear_workspace_bytes(M, K, N, R);
}

salr_status_t salr_qsalr_linear(const uint16_t* x, int64_t M, int64_t K, int64_t N, const uint32_t* bitmap, const uint8_t* codes,
                                const uint16_t* scales, const uint32_t* row_offsets, int64_t nnz, const uint16_t* a_cat,
                                const uint16_t* b_cat, int64_t R, uint16_t* y, void* workspace, size_t workspace_bytes,
                                void* stream) {
    if (M < 0 || K < 0 || N < 0 || R < 0 || nnz < 0) return SALR_ERR_INVALID_ARG;
    if (M == 0 || N == 0) return SALR_OK;
    if (nnz > 0 && (!codes || !scales)) return SALR_ERR_INVALID_ARG;
    if (K % 32 != 0) return SALR_ERR_SHAPE;
    if (nnz > (int64_t)0xFFFFFFFFLL || (K > 0 && nnz > N * K)) return SALR_ERR_SHAPE;
    if (R > kMaxRank) return SALR_ERR_UNSUPPORTED;
    if (salr::linear_nf4_takes(M, K, N, nnz)) {   // small batches: the kernel that reads the codes itself
        if (!y || !x || !bitmap || !row_offsets) return SALR_ERR_INVALID_ARG;
        if (R > 0 && (!a_cat || !b_cat)) return SALR_ERR_INVALID_ARG;
        if (N > kMaxRows || K > kMaxCols) return SALR_ERR_SHAPE;
        const size_t fused = salr::linear_nf4_workspace_bytes(M, N, R);
        if (!workspace || workspace_bytes < fused) return SALR_ERR_CAPACITY;
        salr::LinearArgs a;
        a.x = x; a.M = M; a.K = K; a.N = N;
        a.bitmap = bitmap; a.values = nullptr; a.row_offsets = row_offsets;
        a.a_cat = a_cat; a.b_cat = b_cat; a.R = R;
        a.y = y;
        a.t = static_cast<uint16_t*>(workspace);
        a.slice_table = reinterpret_cast<const uint32_t*>(static_cast<char*>(workspace) + salr::linear_nf4_table_offset(M, R));
        hipError_t e = salr::launch_linear_nf4(a, codes, scales, nnz, static_cast<hipStream_t>(stream), salr::g_timing_events);
        return e == hipSuccess ? SALR_OK : SALR_ERR_HIP;
    }
    if (qsalr_decodes_codes(M, K, N, nnz)) {   // large batches: the decode stage reads the codes
        const size_t lw = salr::linear_workspace_bytes(M, K, N, R);
        if (!workspace || workspace_bytes < lw) return SALR_ERR_CAPACITY;
        return linear_entry(x, M, K, N, bitmap, nullptr, row_offsets, nullptr, a_cat, b_cat, R, y, workspace, workspace_bytes, stream,
                            codes, scales, nnz);
    }
    const size_t vbytes = salr::qsalr_values_bytes(nnz);
    const size_t need = vbytes + (K > 0 ? salr::linear_workspace_bytes(M, K, N, R) : 0);
    if (need > 0 && (!workspace || workspace_bytes < need)) return SALR_ERR_CAPACITY;
    uint16_t* values = static_cast<uint16_t*>(workspace);
    if (K > 0 && nnz > 0) {
        hipError_t e = salr::launch_nf4_dequantize(codes, scales, nnz, values, static_cast<hipStream_t>(stream));
        if (e != hipSuccess) return SALR_ERR_HIP;
    }
    return salr_sparse_lowrank_linear(x, M, K, N, bitmap, values, row_offsets, a_cat, b_cat, R, y,
                                      static_cast<char*>(workspace) + vbytes, workspace_bytes - vbytes, stream);
}

size_t salr_linear_2of4_workspace_bytes(int64_t M, int64_t K, int64_t N, int64_t R) {
    const size_t general = salr_linear_workspace_bytes(M, K, N, R);
    if (M <= 0 || K <= 0 || N <= 0 || R < 0 || R > kMaxRank || K % 32 != 0 || !salr::uses_2of4_kernel(M, K, N)) return general;
    const size_t fast = salr::rowtile_workspace_bytes(M, K, N, R);
    return fast > general ? fast : general;
}

salr_status_t salr_sparse_lowrank_linear_2of4(const uint16_t* x, int64_t M, int64_t K, int64_t N, const uint32_t* bitmap,
                                              const uint16_t* values, const uint32_t* row_offsets, const uint16_t* a_cat,
                                              const uint16_t* b_cat, int64_t R, uint16_t* y, void* workspace,
                                              size_t workspace_bytes, void* stream) {
    if (M < 0 || K < 0 || N < 0 || R < 0) return SALR_ERR_INVALID_ARG;
    if (M == 0 || N == 0) return SALR_OK;
    if (K % 32 != 0) return SALR_ERR_SHAPE;
    const bool small = salr::uses_2of4_kernel(M, K, N);        // up to 128 tokens: the streaming kernels
    const bool large = salr::uses_2of4_gemm(M, K, N);           // above: the tiled GEMM
    if (K == 0 || (!small && !large))   // shapes the sparse-MFMA kernels do not take: the general path
        return salr_sparse_lowrank_linear(x, M, K, N, bitmap, values, row_offsets, a_cat, b_cat, R, y, workspace, workspace_bytes,
                                          stream);
    if (!y || !row_offsets || !x || !bitmap || !values) return SALR_ERR_INVALID_ARG;
    if (R > 0 && (!a_cat || !b_cat)) return SALR_ERR_INVALID_ARG;
    if (N > kMaxRows || K > kMaxCols) return SALR_ERR_SHAPE;
    if (R > kMaxRank || M > kMaxM) return SALR_ERR_UNSUPPORTED;
    const size_t need = salr_linear_2of4_workspace_bytes(M, K, N, R);
    if (need > 0 && (!workspace || workspace_bytes < need)) return SALR_ERR_CAPACITY;
    salr::LinearArgs a;
    a.x = x; a.M = M; a.K = K; a.N = N;
    a.bitmap = bitmap; a.values = values; a.row_offsets = row_offsets;
    a.a_cat = a_cat; a.b_cat = b_cat; a.R = R;
    a.y = y;
    a.t = static_cast<uint16_t*>(workspace);
    hipError_t e = small ? salr::launch_linear_2of4(a, static_cast<hipStream_t>(stream), salr::g_timing_events)
                         : salr::launch_gemm_2of4(a, static_cast<hipStream_t>(stream), salr::g_timing_events);
    return e == hipSuccess ? SALR_OK : SALR_ERR_HIP;
}

salr_status_t salr_bitmap_is_2of4(const uint32_t* bitmap, int64_t rows, int64_t cols, uint32_t* result, void* stream) {
    if (rows < 0 || cols < 0 || !result) return SALR_ERR_INVALID_ARG;
    if (rows > 0 && cols > 0 && !bitmap) return SALR_ERR_INVALID_ARG;
    if (cols % 32 != 0) return SALR_ERR_SHAPE;
    if (rows > kMaxRows || cols > kMaxCols) return SALR_ERR_SHAPE;
    hipError_t e = salr::launch_check_2of4(bitmap, rows, cols, result, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? SALR_OK : SALR_ERR_HIP;
}

static salr_status_t backward_shape_check(int64_t M, int64_t K, int64_t N, int64_t R, bool want_dx, bool want_dadb) {
    if (K % 32 != 0) return SALR_ERR_SHAPE;
    if (N > kMaxSvdDim || K > kMaxCols || M > kMaxM) return SALR_ERR_SHAPE;
    if (R > kMaxRank) return SALR_ERR_UNSUPPORTED;
    if (want_dx && N % 64 != 0) return SALR_ERR_UNSUPPORTED;
    if (R > 0 && N % 32 != 0) return SALR_ERR_UNSUPPORTED;
    if (want_dadb && R > 0 && (M % 32 != 0 || M > kMaxSvdDim)) return SALR_ERR_UNSUPPORTED;
    return SALR_OK;
}

size_t salr_linear_backward_workspace_bytes(int64_t M, int64_t K, int64_t N, int64_t R, int want_dx, int want_dadb) {
    if (M <= 0 || K <= 0 || N <= 0 || R < 0) return 0;
    if (backward_shape_check(M, K, N, R, want_dx != 0, want_dadb != 0) != SALR_OK) return 0;
    return salr::linear_backward_workspace_bytes(M, K, N, R, want_dx != 0, want_dadb != 0);
}

salr_status_t salr_sparse_lowrank_linear_backward(const uint16_t* x, const uint16_t* dy, int64_t M, int64_t K, int64_t N,
                                                  const uint32_t* bitmap, const uint16_t* values,
                                                  const uint32_t* row_offsets, const uint16_t* a_cat, const uint16_t* b_cat,
                                                  int64_t R, uint16_t* dx, uint16_t* da, uint16_t* db, void* workspace,
                                                  size_t workspace_bytes, void* stream) {
    if (M < 0 || K < 0 || N < 0 || R < 0) return SALR_ERR_INVALID_ARG;
    if (M == 0 || K == 0 || N == 0) return SALR_OK;
    const bool want_dx = dx != nullptr, want_dadb = R > 0 && (da != nullptr || db != nullptr);
    if (!want_dx && !want_dadb) return SALR_OK;
    if (!dy) return SALR_ERR_INVALID_ARG;
    if (want_dx && (!bitmap || !row_offsets)) return SALR_ERR_INVALID_ARG;
    if (R > 0 && (!a_cat || !b_cat)) return SALR_ERR_INVALID_ARG;
    if (want_dadb && !x) return SALR_ERR_INVALID_ARG;
    const salr_status_t st = backward_shape_check(M, K, N, R, want_dx, want_dadb);
    if (st != SALR_OK) return st;
    const size_t need = salr::linear_backward_workspace_bytes(M, K, N, R, want_dx, want_dadb);
    if (need > 0 && (!workspace || workspace_bytes < need)) return SALR_ERR_CAPACITY;
    hipError_t e = salr::launch_linear_backward(x, dy, M, K, N, bitmap, values, row_offsets, a_cat, b_cat, R, dx,
                                                want_dadb ? da : nullptr, want_dadb ? db : nullptr, workspace,
                                                static_cast<hipStream_t>(stream));
    return e == hipSuccess ? SALR_OK : SALR_ERR_HIP;
}

void salr_set_kernel_timing_events(void* start_event, void* stop_event) {
    salr::g_timing_events.start = static_cast<hipEvent_t>(start_event);
    salr::g_timing_events.stop = static_cast<hipEvent_t>(stop_event);
}

}  // extern "C"
