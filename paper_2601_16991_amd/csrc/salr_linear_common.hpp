// Small device helpers shared by the linear-layer kernels.
#pragma once

#include "salr_device.hpp"

namespace salr {

// fp32 -> bf16, round to nearest even; NaN stays a quiet NaN.
__device__ __forceinline__ uint16_t f32_to_bf16_rne(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (uint16_t)((u >> 16) | 0x0040u);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

__device__ __forceinline__ float bf16_bits_to_f32(uint32_t b) { return __uint_as_float(b << 16); }

__device__ __forceinline__ bf16x8 as_bf16x8(const uint4& q) { return __builtin_bit_cast(bf16x8, q); }

// One block of 256 threads builds the slice-table entries of 32 rows (see kSliceTableSlices in salr_internal.hpp):
// eight lanes per row, one per slice; a lane walks the chunks of its slice (16 bytes = 128 columns a load, four loads
// in flight), then an exclusive scan over the row's eight lanes turns slice counts into value indices.  Used by
// salr_build_slice_table and, for calls without a table of the caller's, by extra blocks of the small-batch adapter
// pre-kernel.  (Two other shapes were measured and were slower inside the pre-kernel: a wave per row with wave scans,
// and the rows staged through LDS.)
constexpr int kSliceTableRowsPerBlock = 32;

__device__ __forceinline__ void slice_table_block(const uint32_t* __restrict__ bitmap, const uint32_t* __restrict__ row_offsets,
                                                  int64_t N, int64_t K, uint32_t* __restrict__ table, int64_t block,
                                                  int tid) {
    constexpr int kSlices = 8;
    const int64_t n = block * kSliceTableRowsPerBlock + (tid >> 3);
    const int w = tid & 7;
    const int64_t wpr = K >> 5;
    const int64_t chunks = (wpr + 3) / 4;
    const int64_t c_begin = chunks * w / kSlices, c_end = chunks * (w + 1) / kSlices;
    uint32_t count = 0, longest = 0;
    if (n < N) {
        const uint32_t* brow = bitmap + n * wpr;
        if ((wpr & 3) == 0) {
#pragma unroll 4
            for (int64_t c = c_begin; c < c_end; ++c) {
                const uint4 q = *reinterpret_cast<const uint4*>(brow + 4 * c);
                const uint32_t len = __popc(q.x) + __popc(q.y) + __popc(q.z) + __popc(q.w);
                count += len;
                longest = len > longest ? len : longest;
            }
        } else {
            for (int64_t c = c_begin; c < c_end; ++c) {
                uint32_t len = 0;
                for (int64_t q = 4 * c; q < 4 * c + 4 && q < wpr; ++q) len += __popc(brow[q]);
                count += len;
                longest = len > longest ? len : longest;
            }
        }
    }
    uint32_t incl = count;   // the lanes of a row are consecutive
#pragma unroll
    for (int o = 1; o < kSlices; o <<= 1) {
        const uint32_t up = __shfl_up(incl, o, kSlices);
        if (w >= o) incl += up;
    }
    if (n < N) {
        uint2 e;
        e.x = row_offsets[n] + (incl - count);
        e.y = longest;
        *reinterpret_cast<uint2*>(table + (n * kSlices + w) * 2) = e;
    }
}

}  // namespace salr
