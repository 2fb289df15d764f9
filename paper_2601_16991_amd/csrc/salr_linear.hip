// The SALR linear layer  Y = X * What^T + (X * A_cat) * B_cat  (paper Sec. 3.2 and 3.3).
//
// This file: the dispatch between the kernels, and
//   linear_generic_kernel   any shape: 64 x 64 output tile per workgroup, decode of a 64 x 32 weight
//                           tile into LDS per k-step, bf16 MFMA, adapters as extra k-steps
#include <hip/hip_ext.h>

#include "salr_device.hpp"
#include "salr_internal.hpp"
#include "salr_linear_common.hpp"

namespace salr {

// ---------------------------------------------------------------------------------------------------
// Generic fused kernel.  Workgroup = 4 waves, output tile 64 (m) x 64 (n), k-step 32.
//   decode stage : thread (row = tid/4, byte = tid%4) expands one byte mask of its weight row into
//                  8 bf16 in the LDS tile Ws (Sec. 3.3 reconstruction rule), keeping the row's cursor
//                  into the packed values in a register;
//   MFMA stage   : each wave owns a 32 x 32 sub-tile = 2 x 2 v_mfma_f32_16x16x32_bf16 tiles;
//   adapters     : after the K loop the same accumulators take ceil(R/32) more k-steps with
//                  X-tile := T[m, r] and W-tile := B_cat[r, n] (Sec. 3.2 fused into the output tile).
// ---------------------------------------------------------------------------------------------------
constexpr int kGenThreads = 256;
constexpr int kGenTM = 64, kGenTN = 64, kGenTK = 32;
constexpr int kGenPitch = kGenTK + 8;  // bf16 elements; 80-byte rows keep 16-byte alignment and spread banks

// Packed values read straight from global memory (dword index clamped to the last valid dword).
__device__ __forceinline__ void expand_nibble_global(const uint32_t* __restrict__ values32, int64_t last_dw,
                                                     const uint32_t* lut, int64_t cursor, uint32_t nib,
                                                     uint32_t& out01, uint32_t& out23) {
    const int64_t dw = cursor >> 1;
    const uint32_t shift = (uint32_t)(cursor & 1) * 2u;
    const int64_t i0 = dw < last_dw ? dw : last_dw;
    const int64_t i1 = dw + 1 < last_dw ? dw + 1 : last_dw;
    const int64_t i2 = dw + 2 < last_dw ? dw + 2 : last_dw;
    const uint32_t d0 = values32[i0], d1 = values32[i1], d2 = values32[i2];
    const uint32_t e0 = __builtin_amdgcn_alignbyte(d1, d0, shift);
    const uint32_t e1 = __builtin_amdgcn_alignbyte(d2, d1, shift);
    const uint2 sel = *reinterpret_cast<const uint2*>(lut + 2 * nib);
    out01 = __builtin_amdgcn_perm(e1, e0, sel.x);
    out23 = __builtin_amdgcn_perm(e1, e0, sel.y);
}

__global__ __launch_bounds__(kGenThreads) void linear_generic_kernel(
    const uint16_t* __restrict__ x, int64_t M, int64_t K, int64_t N, const uint32_t* __restrict__ bitmap,
    const uint16_t* __restrict__ values, const uint32_t* __restrict__ row_offsets, const uint16_t* __restrict__ t,
    const uint16_t* __restrict__ b_cat, int R, int Rpad, uint16_t* __restrict__ y) {
    __shared__ __attribute__((aligned(16))) uint16_t Xs[kGenTM * kGenPitch];
    __shared__ __attribute__((aligned(16))) uint16_t Ws[kGenTN * kGenPitch];
    __shared__ uint32_t lut[kNibbleLutWords];
    nibble_lut_init(lut);

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int64_t n0 = (int64_t)blockIdx.x * kGenTN;
    const int64_t m0 = (int64_t)blockIdx.y * kGenTM;
    const int64_t wpr = K / 32;

    // loader / decoder role of this thread
    const int lrow = tid >> 2;  // 0..63
    const int lseg = tid & 3;   // 8-element segment of the 32-wide k-step
    const int64_t xm = m0 + lrow;
    const int64_t wn_row = n0 + lrow;
    const bool x_ok = xm < M;
    const bool w_ok = wn_row < N;
    const uint32_t* values32 = reinterpret_cast<const uint32_t*>(values);
    const int64_t nnz = row_offsets[N];
    const int64_t last_dw = nnz > 0 ? (nnz - 1) >> 1 : 0;
    int64_t cursor = w_ok ? (int64_t)row_offsets[wn_row] : 0;

    f32x4 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};

    __syncthreads();  // lut ready

    const int a_row = wm * 32 + (lane & 15);
    const int b_row = wn * 32 + (lane & 15);
    const int k_off = 8 * (lane >> 4);

    for (int64_t k0 = 0; k0 < K; k0 += kGenTK) {
        uint4 xq = make_uint4(0, 0, 0, 0);
        if (x_ok) xq = *reinterpret_cast<const uint4*>(x + xm * K + k0 + 8 * lseg);
        uint4 wq = make_uint4(0, 0, 0, 0);
        if (w_ok) {
            const uint32_t word = bitmap[wn_row * wpr + (k0 >> 5)];
            const uint32_t m8 = (word >> (8 * lseg)) & 0xFFu;
            if (m8) {
                const int64_t c = cursor + __popc(word & ((1u << (8 * lseg)) - 1u));
                const uint32_t lo = m8 & 0xFu, hi = m8 >> 4;
                expand_nibble_global(values32, last_dw, lut, c, lo, wq.x, wq.y);
                expand_nibble_global(values32, last_dw, lut, c + __popc(lo), hi, wq.z, wq.w);
            }
            cursor += __popc(word);
        }
        *reinterpret_cast<uint4*>(&Xs[lrow * kGenPitch + 8 * lseg]) = xq;
        *reinterpret_cast<uint4*>(&Ws[lrow * kGenPitch + 8 * lseg]) = wq;
        __syncthreads();
        bf16x8 a[2], b[2];
#pragma unroll
        for (int i = 0; i < 2; ++i) a[i] = *reinterpret_cast<const bf16x8*>(&Xs[(a_row + 16 * i) * kGenPitch + k_off]);
#pragma unroll
        for (int j = 0; j < 2; ++j) b[j] = *reinterpret_cast<const bf16x8*>(&Ws[(b_row + 16 * j) * kGenPitch + k_off]);
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
        __syncthreads();
    }

    // adapter k-steps: X-tile := T[m, r0 + c], W-tile := B_cat[r0 + c, n]
    for (int r0 = 0; r0 < Rpad; r0 += kGenTK) {
        uint4 xq = make_uint4(0, 0, 0, 0);
        if (x_ok) xq = *reinterpret_cast<const uint4*>(t + xm * Rpad + r0 + 8 * lseg);
        uint32_t e[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int r = r0 + 8 * lseg + j;
            e[j] = (w_ok && r < R) ? (uint32_t)b_cat[(int64_t)r * N + wn_row] : 0u;
        }
        const uint4 wq = make_uint4(e[0] | (e[1] << 16), e[2] | (e[3] << 16), e[4] | (e[5] << 16), e[6] | (e[7] << 16));
        *reinterpret_cast<uint4*>(&Xs[lrow * kGenPitch + 8 * lseg]) = xq;
        *reinterpret_cast<uint4*>(&Ws[lrow * kGenPitch + 8 * lseg]) = wq;
        __syncthreads();
        bf16x8 a[2], b[2];
#pragma unroll
        for (int i = 0; i < 2; ++i) a[i] = *reinterpret_cast<const bf16x8*>(&Xs[(a_row + 16 * i) * kGenPitch + k_off]);
#pragma unroll
        for (int j = 0; j < 2; ++j) b[j] = *reinterpret_cast<const bf16x8*>(&Ws[(b_row + 16 * j) * kGenPitch + k_off]);
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
        __syncthreads();
    }

    // accumulator layout of the 16x16 MFMA: lane holds column (lane % 16), rows 4 * (lane / 16) + e
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int64_t n = n0 + wn * 32 + 16 * j + (lane & 15);
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int64_t m = m0 + wm * 32 + 16 * i + 4 * (lane >> 4) + e;
                if (m < M && n < N) y[m * N + n] = f32_to_bf16_rne(acc[i][j][e]);
            }
        }
}

// +0.0 into `count` bf16 elements (the layer's output when the contraction is empty)
__global__ __launch_bounds__(256) void fill_zero_kernel(uint16_t* __restrict__ out, int64_t count) {
    const int64_t stride = (int64_t)gridDim.x * 256;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < count; i += stride) out[i] = 0;
}

hipError_t launch_fill_zero(uint16_t* out, int64_t count, hipStream_t stream) {
    if (count <= 0) return hipSuccess;
    const int64_t blocks = (count + 255) / 256;
    hipLaunchKernelGGL(fill_zero_kernel, dim3((unsigned)(blocks < 65536 ? blocks : 65536)), dim3(256), 0, stream, out, count);
    return hipGetLastError();
}

thread_local TimingEvents g_timing_events;

hipError_t launch_linear(const LinearArgs& a, hipStream_t stream) {
    if (a.M == 0 || a.N == 0) return hipSuccess;
    if (uses_rowtile(a.M, a.K, a.N)) return launch_linear_rowtile(a, stream, g_timing_events);
    if (linear_slice_takes(a.M, a.K, a.N)) return launch_linear_slice(a, stream, g_timing_events);
    if (a.M <= kStreamMaxM) return launch_linear_stream(a, stream, g_timing_events);
    if (uses_twostage(a.M, a.K))
        return a.lean ? launch_linear_tiled(a, stream, g_timing_events) : launch_linear_twostage(a, stream, g_timing_events);
    const int R = (int)a.R;
    const int Rpad = (int)adapter_rank_padded(a.R);
    if (R > 0) launch_adapter_t(a, stream);
    const TimingEvents ev = g_timing_events;
    dim3 grid((unsigned)((a.N + kGenTN - 1) / kGenTN), (unsigned)((a.M + kGenTM - 1) / kGenTM));
    SALR_LAUNCH(linear_generic_kernel, grid, dim3(kGenThreads), stream, ev, a.x, a.M, a.K, a.N, a.bitmap, a.values,
                a.row_offsets, (const uint16_t*)a.t, a.b_cat, R, Rpad, a.y);
    return hipGetLastError();
}

}  // namespace salr
