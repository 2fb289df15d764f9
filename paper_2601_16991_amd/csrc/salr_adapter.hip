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

// ---------------------------------------------------------------------------------------------------
// Products that contract over the ROWS of a large row-major matrix (the adapter gradients of the backward pass,
// dA = X^T T' and dB^T = dY^T T): partial[z][c][r] = sum over the rows m of slice z of in[m][c] * s_t[r][m], with
// in [M, C] bf16 and the small factor given transposed, s_t [Rpad, M].  The large matrix is read once, row-wise and
// coalesced, and transposed on the way into the MFMA operand by an LDS tile: no transposed copy of it in memory.
//   workgroup (b, z): columns 64 b .. 64 b + 63 (wave w the 16 columns 16 w ..), row slice z (whole steps of 32 rows);
//   per step the 256 threads copy the tile [32 rows x 64 columns] into one of two LDS buffers (the next tile's request
//   is in flight while this one is multiplied); lane (i, g) gathers in[8 g .. 8 g + 7][16 w + i] from it as the A
//   operand of 16x16x32 bf16 MFMAs, the B operand s_t[16 rt + i][8 g ..] is a plain 16-byte load; kRT rank tiles per
//   pass over the slice.  fp32 partials [ksplit][C][Rpad]; padding columns of Rpad come out as zeros (s_t is zero there).
// M % 32 == 0.
// ---------------------------------------------------------------------------------------------------
constexpr int kTnPitch = 64 + 8;   // bf16 elements per tile row

template <int kRT>
__global__ __launch_bounds__(256) void tall_tn_kernel(const uint16_t* __restrict__ in, int64_t M, int64_t C,
                                                      const uint16_t* __restrict__ s_t, int Rpad, int ksplit,
                                                      float* __restrict__ partial) {
    __shared__ __attribute__((aligned(16))) uint16_t tile[2][32 * kTnPitch];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int i16 = lane & 15, g = lane >> 4;
    const int64_t c0 = (int64_t)blockIdx.x * 64;
    const int z = blockIdx.y;
    const int64_t steps = M >> 5;
    const int64_t per_slice = (steps + ksplit - 1) / ksplit;
    const int64_t s_begin = z * per_slice < steps ? z * per_slice : steps;
    const int64_t s_end = (z + 1) * per_slice < steps ? (z + 1) * per_slice : steps;
    // this thread's 16 bytes of a tile: row tid / 8, columns 8 (tid % 8) ..; columns past C are clamped (never stored)
    const int trow = tid >> 3, tvec = tid & 7;
    const bool vec_ok = (C & 7) == 0;
    auto load_tile = [&](int64_t step) -> uint4 {
        const int64_t m = (step << 5) + trow;
        const int64_t c = c0 + 8 * tvec;
        if (vec_ok) {
            const int64_t cc = c + 8 <= C ? c : C - 8;   // a clamped vector holds other columns: they are not stored
            return *reinterpret_cast<const uint4*>(in + m * C + cc);
        }
        uint32_t e[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) e[j] = in[m * C + (c + j < C ? c + j : C - 1)];
        return make_uint4(e[0] | (e[1] << 16), e[2] | (e[3] << 16), e[4] | (e[5] << 16), e[6] | (e[7] << 16));
    };
    for (int rb = 0; rb < Rpad; rb += 16 * kRT) {
        f32x4 acc[kRT];
#pragma unroll
        for (int rt = 0; rt < kRT; ++rt) acc[rt] = f32x4{0.f, 0.f, 0.f, 0.f};
        const uint16_t* srow[kRT];
#pragma unroll
        for (int rt = 0; rt < kRT; ++rt) {
            const int r = rb + 16 * rt + i16;
            srow[rt] = s_t + (int64_t)(r < Rpad ? r : Rpad - 1) * M + 8 * g;
        }
        if (s_begin < s_end) {
            uint4 next = load_tile(s_begin);
            int buf = 0;
            for (int64_t step = s_begin; step < s_end; ++step) {
                *reinterpret_cast<uint4*>(&tile[buf][trow * kTnPitch + 8 * tvec]) = next;
                if (step + 1 < s_end) next = load_tile(step + 1);
                uint4 bq[kRT];
#pragma unroll
                for (int rt = 0; rt < kRT; ++rt) bq[rt] = *reinterpret_cast<const uint4*>(srow[rt] + (step << 5));
                __syncthreads();   // the tile is complete; the buffer written two steps ago has been read by everyone
                const uint16_t* col = &tile[buf][(8 * g) * kTnPitch + 16 * wave + i16];
                uint32_t e[8];
#pragma unroll
                for (int j = 0; j < 8; ++j) e[j] = col[j * kTnPitch];
                const uint4 aq = make_uint4(e[0] | (e[1] << 16), e[2] | (e[3] << 16), e[4] | (e[5] << 16), e[6] | (e[7] << 16));
#pragma unroll
                for (int rt = 0; rt < kRT; ++rt)
                    acc[rt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(aq), as_bf16x8(bq[rt]), acc[rt], 0, 0, 0);
                buf ^= 1;
            }
        }
        __syncthreads();   // before the next pass writes buffer 0 again
        // accumulator layout of the 16x16 MFMA: lane holds column lane % 16 (rank), rows 4 (lane / 16) + e (matrix column)
#pragma unroll
        for (int rt = 0; rt < kRT; ++rt) {
            const int r = rb + 16 * rt + i16;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int64_t c = c0 + 16 * wave + 4 * g + e;
                if (c < C && r < Rpad) partial[((int64_t)z * C + c) * Rpad + r] = acc[rt][e];
            }
        }
    }
}

// partial [ksplit][C][Rpad] fp32 = slices of in^T [C, M] * s_t^T [M, Rpad]
void launch_tall_tn(const uint16_t* in, int64_t M, int64_t C, const uint16_t* s_t, int Rpad, int ksplit, float* partial,
                    hipStream_t stream) {
    const dim3 grid((unsigned)((C + 63) / 64), (unsigned)ksplit);
    const int tiles = Rpad / 16;
    if (tiles % 4 == 0) hipLaunchKernelGGL(tall_tn_kernel<4>, grid, dim3(256), 0, stream, in, M, C, s_t, Rpad, ksplit, partial);
    else hipLaunchKernelGGL(tall_tn_kernel<2>, grid, dim3(256), 0, stream, in, M, C, s_t, Rpad, ksplit, partial);
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
    if (adapter_uses_prekernel(a.M)) {   // two launches: split-K partials from A_cat as it is, then their sum
        launch_adapter_partial_to(a, partial, stream);
        launch_splitk_reduce(partial, a.M * Rpad, kStreamTSlices, a.t, stream);
        return;
    }
    launch_adapter_transpose(a.a_cat, a.K, R, Rpad, a_t, stream);
    const int ksplit = adapter_ksplit(a.M, a.K);
    launch_tall_product(a.x, a.M, a.K, a_t, Rpad, ksplit, a.t, partial, false, stream);
    if (ksplit > 1) launch_splitk_reduce(partial, a.M * Rpad, ksplit, a.t, stream);
}

}  // namespace salr
