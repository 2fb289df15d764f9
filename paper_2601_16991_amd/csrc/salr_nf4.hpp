// The 4-bit NormalFloat code of QSALR (paper Sec. 4, "Coupled with Quantization") as the kernels see it: the 16 levels
// and the value rule bf16(fp32(level * scale)), eight codes at a time.
#pragma once

#include "salr_device.hpp"

namespace salr {

constexpr int kNf4Block = 64;   // packed values per scale

// the published NF4 levels: normal quantiles scaled to [-1, 1], ascending, exact zero at index 7
static __device__ __constant__ float kNf4Levels[16] = {
    -1.0f, -0.6961928009986877f, -0.5250730514526367f, -0.39491748809814453f,
    -0.28444138169288635f, -0.18477343022823334f, -0.09105003625154495f, 0.0f,
    0.07958029955625534f, 0.16093020141124725f, 0.24611230194568634f, 0.33791524171829224f,
    0.44070982933044434f, 0.5626170039176941f, 0.7229568362236023f, 1.0f};

typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));

// two floats -> two bf16 (round to nearest even), the first in the low half
__device__ __forceinline__ uint32_t pack_bf16_rne(float a, float b) {
    const f32x2_t v = {a, b};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}

// Dequantise the eight codes of c with one scale: eight bf16, value 0 in the low half of .x.  `levels`: the 16 levels
// in LDS (a 16-entry table covers 16 banks once, so the lanes of a wave never conflict on it).
__device__ __forceinline__ uint4 nf4_decode8(uint32_t c, float scale, const float* levels) {
    float w[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) w[j] = __fmul_rn(levels[(c >> (4 * j)) & 15u], scale);
    return make_uint4(pack_bf16_rne(w[0], w[1]), pack_bf16_rne(w[2], w[3]), pack_bf16_rne(w[4], w[5]),
                      pack_bf16_rne(w[6], w[7]));
}

}  // namespace salr
