// First adapter stage of the large-batch paths (paper Sec. 3.2): T = X * A_cat, plus the small passes around it
// (transposed copy of A_cat, fixed-order sum of split-K partials, also used by the dense stage).
#include "salr_device.hpp"
#include "salr_internal.hpp"
#include "salr_linear_common.hpp"

namespace salr {

// ---------------------------------------------------------------------------------------------------
// T = X * A_cat for the large-batch paths (Sec. 3.2, first concatenated GEMM), bf16 output [M, Rpad].
// A_cat arrives transposed and zero padded, a_t [Rpad, K] (written by the transposing pre-pass), so that
// both MFMA operands are plain 16-byte loads along k.  The product is a stream over X (it is read once, nothing
// else is large), so the grid is made wide: workgroup (b, z) = 64 kMB rows of X times slice z of K, wave w owns
// 16 kMB of the rows (each a_t operand it loads is used for kMB row blocks: at kMB = 1 the a_t requests are kRT
// times the X requests and their L2 traffic, not X, sets the pace), the four waves walk the slice in step.
// kRT rank tiles of 16 columns per pass over the slice (all of them in one pass up to rank 128); 16x16x32 bf16
// MFMAs; with more than one slice the fp32 partial results go to partial[z] and splitk_reduce_kernel adds
// them in a fixed order.  Padding columns come out as exact zeros.  keep_fp32: the caller wants the fp32 sums
// (the subspace iteration of the residual adapter), so even a single slice goes to partial[0].
// ---------------------------------------------------------------------------------------------------
template <int kMB, int kRT, int kDepth>
__global__ __launch_bounds__(256) void adapter_t_kernel(const uint16_t* __restrict__ x, int64_t M, int64_t K,
                                                        const uint16_t* __restrict__ a_t, int Rpad, int ksplit,
                                                        uint16_t* __restrict__ t, float* __restrict__ partial,
                                                        int keep_fp32) {
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int i16 = lane & 15, g = lane >> 4;
    const int64_t m0 = ((int64_t)blockIdx.x * 4 + wave) * 16 * kMB;
    if (m0 >= M) return;   // wave-uniform; the kernel has no barrier
    const int z = blockIdx.y;
    const int64_t units = K >> 5;
    const int64_t per_slice = (units + ksplit - 1) / ksplit;
    const int64_t u_begin = z * per_slice < units ? z * per_slice : units;
    const int64_t u_end = (z + 1) * per_slice < units ? (z + 1) * per_slice : units;
    const int64_t len = u_end - u_begin;
    const uint16_t* xrow[kMB];
#pragma unroll
    for (int mb = 0; mb < kMB; ++mb) {
        const int64_t mrow = m0 + 16 * mb + i16;
        xrow[mb] = x + (mrow < M ? mrow : M - 1) * K + 8 * g;
    }
    for (int rb = 0; rb < Rpad; rb += 16 * kRT) {
        // a pass starts inside the Rpad columns (loop bound); tiles of it that lie past them are clamped, not stored
        const uint16_t* arow[kRT];
#pragma unroll
        for (int rt = 0; rt < kRT; ++rt) {
            const int r = rb + 16 * rt + i16;
            arow[rt] = a_t + (int64_t)(r < Rpad ? r : Rpad - 1) * K + 8 * g;
        }
        f32x4 acc[kMB][kRT];
#pragma unroll
        for (int mb = 0; mb < kMB; ++mb)
#pragma unroll
            for (int rt = 0; rt < kRT; ++rt) acc[mb][rt] = f32x4{0.f, 0.f, 0.f, 0.f};
        // kDepth k-steps per trip with every load issued before the first MFMA: the kernel lives on loads in flight
        for (int64_t i0 = 0; i0 < len; i0 += kDepth) {
            uint4 aq[kDepth][kMB], bq[kDepth][kRT];
#pragma unroll
            for (int d = 0; d < kDepth; ++d) {
                const int64_t i = i0 + d < len ? i0 + d : len - 1;   // past the end: reload the last step, not used
                const int64_t k0 = (u_begin + i) << 5;
#pragma unroll
                for (int mb = 0; mb < kMB; ++mb) aq[d][mb] = *reinterpret_cast<const uint4*>(xrow[mb] + k0);
#pragma unroll
                for (int rt = 0; rt < kRT; ++rt) bq[d][rt] = *reinterpret_cast<const uint4*>(arow[rt] + k0);
            }
#pragma unroll
            for (int d = 0; d < kDepth; ++d) {
                if (i0 + d < len) {   // wave-uniform
#pragma unroll
                    for (int mb = 0; mb < kMB; ++mb)
#pragma unroll
                        for (int rt = 0; rt < kRT; ++rt)
                            acc[mb][rt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(aq[d][mb]), as_bf16x8(bq[d][rt]),
                                                                                  acc[mb][rt], 0, 0, 0);
                }
            }
        }
        // accumulator layout of the 16x16 MFMA: lane holds column lane % 16, rows 4 (lane / 16) + e
#pragma unroll
        for (int mb = 0; mb < kMB; ++mb)
#pragma unroll
            for (int rt = 0; rt < kRT; ++rt) {
                const int r = rb + 16 * rt + i16;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int64_t m = m0 + 16 * mb + 4 * g + e;
                    if (m < M && r < Rpad) {
                        if (ksplit == 1 && !keep_fp32) t[m * Rpad + r] = f32_to_bf16_rne(acc[mb][rt][e]);
                        else partial[((int64_t)z * M + m) * Rpad + r] = acc[mb][rt][e];
                    }
                }
            }
    }
}

// out = bf16(sum over z of partial[z]), four elements per thread (count % 4 == 0), z in ascending order.
__global__ __launch_bounds__(256) void splitk_reduce_kernel(const float* __restrict__ partial, int64_t count, int ksplit,
                                                            uint16_t* __restrict__ out) {
    const int64_t i = ((int64_t)blockIdx.x * 256 + threadIdx.x) * 4;
    if (i >= count) return;
    float4 s = *reinterpret_cast<const float4*>(partial + i);
    for (int z = 1; z < ksplit; ++z) {
        const float4 p = *reinterpret_cast<const float4*>(partial + (int64_t)z * count + i);
        s.x += p.x; s.y += p.y; s.z += p.z; s.w += p.w;
    }
    uint2 o;
    o.x = (uint32_t)f32_to_bf16_rne(s.x) | ((uint32_t)f32_to_bf16_rne(s.y) << 16);
    o.y = (uint32_t)f32_to_bf16_rne(s.z) | ((uint32_t)f32_to_bf16_rne(s.w) << 16);
    *reinterpret_cast<uint2*>(out + i) = o;
}

void launch_splitk_reduce(const float* partial, int64_t count, int ksplit, uint16_t* out, hipStream_t stream) {
    hipLaunchKernelGGL(splitk_reduce_kernel, dim3((unsigned)((count / 4 + 255) / 256)), dim3(256), 0, stream, partial, count,
                       ksplit, out);
}

// a_t[r][k] = A_cat[k][r] for r < R, 0 for R <= r < Rpad: one thread per k and block of 8 ranks.
__global__ __launch_bounds__(256) void adapter_transpose_kernel(const uint16_t* __restrict__ a_cat, int64_t K, int R,
                                                                 int Rpad, uint16_t* __restrict__ a_t) {
    const int64_t k = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (k >= K) return;
    const int r0 = 8 * blockIdx.y;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const int r = r0 + j;
        a_t[(int64_t)r * K + k] = r < R ? a_cat[k * R + r] : (uint16_t)0;
    }
}

void launch_adapter_transpose(const uint16_t* a_cat, int64_t K, int R, int Rpad, uint16_t* a_t, hipStream_t stream) {
    hipLaunchKernelGGL(adapter_transpose_kernel, dim3((unsigned)((K + 255) / 256), Rpad / 8), dim3(256), 0, stream, a_cat, K, R,
                       Rpad, a_t);
}

template <int kMB, int kDepth>
static void launch_tall_product_rt(int rank_tiles, dim3 grid, hipStream_t stream, const uint16_t* x, int64_t M, int64_t K,
                                   const uint16_t* a_t, int Rpad, int ksplit, uint16_t* t, float* partial, int keep) {
    switch (rank_tiles) {
#define SALR_CASE(RT)                                                                                                   \
    case RT:                                                                                                            \
        hipLaunchKernelGGL((adapter_t_kernel<kMB, RT, kDepth>), grid, dim3(256), 0, stream, x, M, K, a_t, Rpad, ksplit, t, \
                           partial, keep);                                                                              \
        break;
        SALR_CASE(2) SALR_CASE(3) SALR_CASE(4) SALR_CASE(5) SALR_CASE(6) SALR_CASE(7) SALR_CASE(8)
#undef SALR_CASE
        default: break;
    }
}

void launch_tall_product(const uint16_t* x, int64_t M, int64_t K, const uint16_t* a_t, int Rpad, int ksplit, uint16_t* t,
                         float* partial, bool keep_fp32, hipStream_t stream) {
    const int rows = adapter_rows_per_block(M);
    const dim3 grid((unsigned)((M + rows - 1) / rows), (unsigned)ksplit);
    // rank tiles of 16 columns per pass over the slice: as few passes as eight tiles at a time allow, evenly filled
    const int tiles = Rpad / 16, passes = (tiles + 7) / 8;
    const int rank_tiles = (tiles + passes - 1) / passes;
    const int keep = keep_fp32 ? 1 : 0;
    if (rows == 256) launch_tall_product_rt<4, 2>(rank_tiles, grid, stream, x, M, K, a_t, Rpad, ksplit, t, partial, keep);
    else launch_tall_product_rt<1, 4>(rank_tiles, grid, stream, x, M, K, a_t, Rpad, ksplit, t, partial, keep);
}

void launch_adapter_t(const LinearArgs& a, hipStream_t stream) {
    const int R = (int)a.R, Rpad = (int)adapter_rank_padded(a.R);
    char* base = reinterpret_cast<char*>(a.t);
    uint16_t* a_t = reinterpret_cast<uint16_t*>(base + adapter_t_bytes(a.M, a.R));
    float* partial = reinterpret_cast<float*>(base + adapter_t_bytes(a.M, a.R) + adapter_at_bytes(a.K, a.R));
    launch_adapter_transpose(a.a_cat, a.K, R, Rpad, a_t, stream);
    const int ksplit = adapter_ksplit(a.M, a.K);
    launch_tall_product(a.x, a.M, a.K, a_t, Rpad, ksplit, a.t, partial, false, stream);
    if (ksplit > 1) launch_splitk_reduce(partial, a.M * Rpad, ksplit, a.t, stream);
}

}  // namespace salr
