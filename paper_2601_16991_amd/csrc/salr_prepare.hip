// Model-preparation steps around the linear layer (not on its per-token path):
//   residual_kernel        E = W - What                               (paper Sec. 3.1)
//   concat_a_kernel / concat_b_kernel   A_cat = [A_1 ... A_n], B_cat = [B_1; ...; B_n]   (Sec. 3.2)
// All three are plain streams over their operands (HBM-bound, no reuse).
#include "salr_device.hpp"
#include "salr_internal.hpp"
#include "salr_linear_common.hpp"

namespace salr {

// E = bf16(f32(W) - f32(What)), 8 elements per thread.  For a masked What (each entry the entry of W or zero) the
// difference is exact: the entry of W where it was pruned, +0 where it was kept.
template <bool kVec>
__global__ __launch_bounds__(256) void residual_kernel(const uint16_t* __restrict__ w, const uint16_t* __restrict__ w_hat,
                                                        int64_t count, uint16_t* __restrict__ e) {
    const int64_t i0 = ((int64_t)blockIdx.x * 256 + threadIdx.x) * 8;
    if (i0 >= count) return;
    uint16_t a[8], b[8], o[8];
    if (kVec && i0 + 8 <= count) {
        *reinterpret_cast<uint4*>(a) = *reinterpret_cast<const uint4*>(w + i0);
        *reinterpret_cast<uint4*>(b) = *reinterpret_cast<const uint4*>(w_hat + i0);
#pragma unroll
        for (int j = 0; j < 8; ++j) o[j] = f32_to_bf16_rne(bf16_bits_to_f32(a[j]) - bf16_bits_to_f32(b[j]));
        *reinterpret_cast<uint4*>(e + i0) = *reinterpret_cast<const uint4*>(o);
    } else {
        for (int j = 0; j < 8 && i0 + j < count; ++j)
            e[i0 + j] = f32_to_bf16_rne(bf16_bits_to_f32(w[i0 + j]) - bf16_bits_to_f32(w_hat[i0 + j]));
    }
}

hipError_t launch_residual(const uint16_t* w, const uint16_t* w_hat, int64_t rows, int64_t cols, uint16_t* e,
                           hipStream_t stream) {
    const int64_t count = rows * cols;
    if (count == 0) return hipSuccess;
    const bool vec = (((uintptr_t)w | (uintptr_t)w_hat | (uintptr_t)e) & 15) == 0;
    const unsigned grid = (unsigned)((count + 2047) / 2048);
    if (vec) hipLaunchKernelGGL(residual_kernel<true>, dim3(grid), dim3(256), 0, stream, w, w_hat, count, e);
    else hipLaunchKernelGGL(residual_kernel<false>, dim3(grid), dim3(256), 0, stream, w, w_hat, count, e);
    return hipGetLastError();
}

// Up to kConcatBatch adapters per launch, their pointers and rank offsets passed by value.
struct ConcatBatch {
    const uint16_t* src[kConcatBatch];
    int first[kConcatBatch + 1];   // first column (A) / row (B) of adapter i inside the concatenation; [n] = end
    int n;
};

// A_cat[k][first_i + c] = A_i[k][c]: one thread per element of the batch's column range (rows of 2 r_i bytes do
// not line up with anything wider).
__global__ __launch_bounds__(256) void concat_a_kernel(ConcatBatch batch, int64_t K, int R, uint16_t* __restrict__ a_cat) {
    const int width = batch.first[batch.n] - batch.first[0];
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= K * width) return;
    const int64_t k = idx / width;
    const int col = batch.first[0] + (int)(idx % width);
    int i = 0;
    while (i + 1 < batch.n && col >= batch.first[i + 1]) ++i;
    const int r = batch.first[i + 1] - batch.first[i];
    a_cat[k * R + col] = batch.src[i][k * r + (col - batch.first[i])];
}

// B_cat[first_i + c][:] = B_i[c][:]: whole rows are contiguous on both sides; 8 elements per thread where the
// addresses allow 16-byte accesses.
template <bool kVec>
__global__ __launch_bounds__(256) void concat_b_kernel(ConcatBatch batch, int64_t N, uint16_t* __restrict__ b_cat) {
    const int row = batch.first[0] + (int)blockIdx.y;
    int i = 0;
    while (i + 1 < batch.n && row >= batch.first[i + 1]) ++i;
    const uint16_t* src = batch.src[i] + (int64_t)(row - batch.first[i]) * N;
    uint16_t* dst = b_cat + (int64_t)row * N;
    const int64_t c0 = ((int64_t)blockIdx.x * 256 + threadIdx.x) * 8;
    if (c0 >= N) return;
    if (kVec && c0 + 8 <= N) {
        *reinterpret_cast<uint4*>(dst + c0) = *reinterpret_cast<const uint4*>(src + c0);
    } else {
        for (int j = 0; j < 8 && c0 + j < N; ++j) dst[c0 + j] = src[c0 + j];
    }
}

hipError_t launch_concat(const uint16_t* const* a_list, const uint16_t* const* b_list, const int64_t* ranks, int64_t n,
                         int64_t K, int64_t N, int64_t R, uint16_t* a_cat, uint16_t* b_cat, hipStream_t stream) {
    int first = 0;
    for (int64_t base = 0; base < n; base += kConcatBatch) {
        const int cnt = (int)(n - base < kConcatBatch ? n - base : kConcatBatch);
        ConcatBatch a{}, b{};
        a.n = b.n = cnt;
        bool vec = N % 8 == 0 && ((uintptr_t)b_cat & 15) == 0;
        for (int i = 0; i < cnt; ++i) {
            a.src[i] = a_list[base + i];
            b.src[i] = b_list[base + i];
            a.first[i] = b.first[i] = first;
            first += (int)ranks[base + i];
            vec = vec && ((uintptr_t)b.src[i] & 15) == 0;
        }
        a.first[cnt] = b.first[cnt] = first;
        const int width = first - a.first[0];
        if (width == 0) continue;
        if (K > 0)
            hipLaunchKernelGGL(concat_a_kernel, dim3((unsigned)((K * width + 255) / 256)), dim3(256), 0, stream, a, K, (int)R,
                               a_cat);
        if (N > 0) {
            const dim3 grid((unsigned)((N + 2047) / 2048), (unsigned)width);
            if (vec) hipLaunchKernelGGL(concat_b_kernel<true>, grid, dim3(256), 0, stream, b, N, b_cat);
            else hipLaunchKernelGGL(concat_b_kernel<false>, grid, dim3(256), 0, stream, b, N, b_cat);
        }
    }
    return hipGetLastError();
}

}  // namespace salr
