// QSALR (paper Sec. 4, "Coupled with Quantization"): the packed nonzero values of the bitmap format as 4-bit
// NormalFloat codes with one scale per block of 64 consecutive values.
//
// The paper names the data type (NF4, from the QLoRA paper it cites) and gives no further detail; the reading is:
//   levels   the 16 published NF4 levels (normal quantiles scaled to [-1, 1], exact zero at index 7);
//   scale    per block of 64 consecutive packed values (the last block may be short): the block's largest magnitude,
//            which is one of its bf16 values, so it is stored as bf16 without rounding;
//   code     the level nearest to x / scale, decided without a division: the number of boundaries
//            fp32(mid_k * scale), mid_k = fp32(0.5 (c_k + c_{k+1})), k = 0..14, that x exceeds (a value on a boundary
//            takes the lower code); two codes per byte, the even-indexed value in the low nibble;
//   value    bf16_rne(fp32(level[code] * scale)).
// Every decision is a comparison of fp32 numbers that are each one correctly rounded product, so the codes are
// reproducible bit for bit.
#include "salr_device.hpp"
#include "salr_internal.hpp"
#include "salr_linear_common.hpp"
#include "salr_nf4.hpp"

namespace salr {

// One wave per block of 64 values: lane i owns value 64 b + i.
__global__ __launch_bounds__(256) void nf4_quantize_kernel(const uint16_t* __restrict__ values, int64_t count,
                                                           uint8_t* __restrict__ codes, uint16_t* __restrict__ scales) {
    const int lane = threadIdx.x & 63;
    const int64_t block = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    const int64_t i = block * kNf4Block + lane;
    if (block * kNf4Block >= count) return;   // wave-uniform; no barrier in this kernel
    const bool mine = i < count;
    const uint32_t bits = mine ? values[i] : 0u;
    uint32_t amax = bits & 0x7FFFu;            // magnitude pattern: integer order = order of |x| for finite bf16
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) {
        const uint32_t o = (uint32_t)__shfl_xor((int)amax, d, 64);
        amax = o > amax ? o : amax;
    }
    if (lane == 0) scales[block] = (uint16_t)amax;
    const float s = bf16_bits_to_f32(amax);
    const float x = bf16_bits_to_f32(bits);
    uint32_t code = 0;
    if (amax == 0) {
        code = 7;
    } else {
#pragma unroll
        for (int k = 0; k < 15; ++k) {
            const float mid = __fmul_rn(0.5f, __fadd_rn(kNf4Levels[k], kNf4Levels[k + 1]));
            code += x > __fmul_rn(mid, s) ? 1u : 0u;
        }
    }
    if (!mine) code = 0;                       // the unused high nibble of an odd count stays 0
    const uint32_t hi = (uint32_t)__shfl_down((int)code, 1, 64);
    if (mine && (lane & 1) == 0) codes[i >> 1] = (uint8_t)(code | (hi << 4));
}

// Eight values per thread: one dword of codes in, 16 bytes of bf16 out (scalar at the ragged end).
__global__ __launch_bounds__(256) void nf4_dequantize_kernel(const uint8_t* __restrict__ codes,
                                                             const uint16_t* __restrict__ scales, int64_t count,
                                                             uint16_t* __restrict__ out) {
    const int64_t i0 = ((int64_t)blockIdx.x * 256 + threadIdx.x) * 8;
    if (i0 >= count) return;
    const float s = bf16_bits_to_f32(scales[i0 / kNf4Block]);   // 8 divides 64: one scale per thread
    uint32_t e[8];
    if (i0 + 8 <= count) {
        const uint32_t c = *reinterpret_cast<const uint32_t*>(codes + (i0 >> 1));
#pragma unroll
        for (int j = 0; j < 8; ++j) e[j] = f32_to_bf16_rne(__fmul_rn(kNf4Levels[(c >> (4 * j)) & 15u], s));
        *reinterpret_cast<uint4*>(out + i0) = make_uint4(e[0] | (e[1] << 16), e[2] | (e[3] << 16), e[4] | (e[5] << 16), e[6] | (e[7] << 16));
    } else {
        for (int64_t i = i0; i < count; ++i) {
            const uint32_t c = (codes[i >> 1] >> (4 * (i & 1))) & 15u;
            out[i] = f32_to_bf16_rne(__fmul_rn(kNf4Levels[c], s));
        }
    }
}

hipError_t launch_nf4_quantize(const uint16_t* values, int64_t count, uint8_t* codes, uint16_t* scales, hipStream_t stream) {
    if (count <= 0) return hipSuccess;
    const int64_t blocks = (count + kNf4Block - 1) / kNf4Block;
    hipLaunchKernelGGL(nf4_quantize_kernel, dim3((unsigned)((blocks + 3) / 4)), dim3(256), 0, stream, values, count, codes, scales);
    return hipGetLastError();
}

hipError_t launch_nf4_dequantize(const uint8_t* codes, const uint16_t* scales, int64_t count, uint16_t* out, hipStream_t stream) {
    if (count <= 0) return hipSuccess;
    const int64_t threads = (count + 7) / 8;
    hipLaunchKernelGGL(nf4_dequantize_kernel, dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, stream, codes, scales, count, out);
    return hipGetLastError();
}

}  // namespace salr
