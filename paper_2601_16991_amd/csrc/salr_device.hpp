// Device-side helpers shared by the SALR kernels (gfx950 only, wave64).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace salr {

constexpr int kWave = 64;

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

__device__ __forceinline__ int lane_id() { return threadIdx.x & (kWave - 1); }

// "Nonzero" is a value test on the bf16 pattern: both zeros have no magnitude bits.
__device__ __forceinline__ uint32_t bf16_is_nonzero(uint32_t bits16) { return (bits16 & 0x7FFFu) != 0u; }

// 8-bit mask of the nonzero halves of four dwords holding eight bf16 (element 0 in the low half of q.x).
__device__ __forceinline__ uint32_t nonzero_mask8(uint4 q) {
    uint32_t m = 0;
    m |= bf16_is_nonzero(q.x) << 0;
    m |= bf16_is_nonzero(q.x >> 16) << 1;
    m |= bf16_is_nonzero(q.y) << 2;
    m |= bf16_is_nonzero(q.y >> 16) << 3;
    m |= bf16_is_nonzero(q.z) << 4;
    m |= bf16_is_nonzero(q.z >> 16) << 5;
    m |= bf16_is_nonzero(q.w) << 6;
    m |= bf16_is_nonzero(q.w >> 16) << 7;
    return m;
}

constexpr int kUnit = 8;  // columns a thread handles per step = one byte of bitmap = one 16-byte load

// Eight consecutive bf16 of a row starting at column 8u, zero-filled past the row end.
template <bool kVec>
__device__ __forceinline__ uint4 load_unit(const uint16_t* row, int64_t cols, int64_t u) {
    uint4 q = make_uint4(0, 0, 0, 0);
    const int64_t k0 = u * kUnit;
    if (k0 >= cols) return q;
    if constexpr (kVec) {
        q = *reinterpret_cast<const uint4*>(row + k0);
    } else {
        uint32_t e[kUnit];
#pragma unroll
        for (int j = 0; j < kUnit; ++j) e[j] = (k0 + j < cols) ? row[k0 + j] : 0u;
        q.x = e[0] | (e[1] << 16);
        q.y = e[2] | (e[3] << 16);
        q.z = e[4] | (e[5] << 16);
        q.w = e[6] | (e[7] << 16);
    }
    return q;
}

__device__ __forceinline__ uint32_t unit_elem(const uint4& q, int j) {
    const uint32_t d = (j < 2) ? q.x : (j < 4) ? q.y : (j < 6) ? q.z : q.w;
    return (j & 1) ? (d >> 16) : (d & 0xFFFFu);
}

// Inclusive scan of one value per lane across the wave.
__device__ __forceinline__ uint32_t wave_inclusive_scan(uint32_t v) {
    const int lane = lane_id();
#pragma unroll
    for (int d = 1; d < kWave; d <<= 1) {
        uint32_t o = __shfl_up(v, d, kWave);
        if (lane >= d) v += o;
    }
    return v;
}

// Exclusive scan over a block of kThreads (multiple of 64); `total` gets the block sum.
// `scratch` needs kThreads/64 + 1 words of LDS.  All threads must call it.
template <int kThreads>
__device__ __forceinline__ uint32_t block_exclusive_scan(uint32_t v, uint32_t* scratch, uint32_t& total) {
    constexpr int kWaves = kThreads / kWave;
    const int wave = threadIdx.x / kWave;
    const int lane = lane_id();
    uint32_t incl = wave_inclusive_scan(v);
    __syncthreads();  // scratch may still be read from a previous call
    if (lane == kWave - 1) scratch[wave] = incl;
    __syncthreads();
    uint32_t base = 0, sum = 0;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
        uint32_t s = scratch[w];
        if (w < wave) base += s;
        sum += s;
    }
    total = sum;
    return base + incl - v;
}

// ---------------------------------------------------------------------------------------------------
// Nibble expansion: the reconstruction rule of Sec. 3.3 applied to 4 columns at a time.
//
// For a 4-bit mask `nib` whose set bits own the next popcount(nib) packed values, the four output
// bf16 slots (two dwords) are produced by two byte permutes of the 8 bytes that hold those values.
// The permute selectors depend only on `nib`: slot s takes value number popcount(nib & (2^s - 1)) if
// bit s is set, and the constant 0 otherwise.  They sit in a 16-entry table in LDS (the counterpart of
// the paper's 256 x 8 lookup table, at nibble instead of byte granularity so that the 128-byte table
// covers each LDS bank once and lookups never conflict).
// ---------------------------------------------------------------------------------------------------
constexpr int kNibbleLutWords = 32;  // 16 entries x 2 selectors

__device__ __forceinline__ void nibble_lut_entry(uint32_t nib, uint32_t& sel_lo, uint32_t& sel_hi) {
    uint32_t sel[2] = {0, 0};
    uint32_t seen = 0;
    for (int s = 0; s < 4; ++s) {
        uint32_t two;  // selector bytes for the low and high byte of slot s
        if ((nib >> s) & 1u) {
            two = (2u * seen) | ((2u * seen + 1u) << 8);
            ++seen;
        } else {
            two = 0x0C0Cu;  // selector value 12 yields the constant byte 0x00
        }
        sel[s >> 1] |= two << (16 * (s & 1));
    }
    sel_lo = sel[0];
    sel_hi = sel[1];
}

// Fill the LDS table; the caller synchronises before use.
__device__ __forceinline__ void nibble_lut_init(uint32_t* lut) {
    if (threadIdx.x < 16) {
        uint32_t a, b;
        nibble_lut_entry(threadIdx.x, a, b);
        lut[2 * threadIdx.x] = a;
        lut[2 * threadIdx.x + 1] = b;
    }
}

// Expand 4 columns.  `stage` is an LDS copy (as dwords) of packed values, `cursor` the element index
// in it of the first value owned by this nibble.  Reads stage[cursor/2 .. cursor/2 + 2], so the
// staging buffer must extend 2 dwords past the last valid one.
__device__ __forceinline__ void expand_nibble(const uint32_t* stage, const uint32_t* lut, uint32_t cursor,
                                              uint32_t nib, uint32_t& out01, uint32_t& out23) {
    const uint32_t dw = cursor >> 1;
    const uint32_t shift = (cursor & 1u) * 2u;  // bytes
    const uint32_t d0 = stage[dw], d1 = stage[dw + 1], d2 = stage[dw + 2];
    const uint32_t e0 = __builtin_amdgcn_alignbyte(d1, d0, shift);
    const uint32_t e1 = __builtin_amdgcn_alignbyte(d2, d1, shift);
    const uint2 sel = *reinterpret_cast<const uint2*>(lut + 2 * nib);
    out01 = __builtin_amdgcn_perm(e1, e0, sel.x);
    out23 = __builtin_amdgcn_perm(e1, e0, sel.y);
}

// Expand the 8 columns of one byte mask into four dwords (element 0 in the low half of .x).
__device__ __forceinline__ uint4 expand_byte(const uint32_t* stage, const uint32_t* lut, uint32_t cursor,
                                             uint32_t mask8) {
    uint4 o;
    const uint32_t lo = mask8 & 0xFu, hi = (mask8 >> 4) & 0xFu;
    expand_nibble(stage, lut, cursor, lo, o.x, o.y);
    expand_nibble(stage, lut, cursor + __popc(lo), hi, o.z, o.w);
    return o;
}

}  // namespace salr
