// Bitmap encoder and standalone decoder (paper Sec. 3.3, "Mapping Sparse Weights").
//
// Encoding is three launches on the caller's stream:
//   1. encode_count_kernel   one workgroup per row: bitmap words + the row's nonzero count
//   2. row_scan_kernel       one workgroup: counts -> row_offsets (exclusive prefix, in place)
//   3. encode_compact_kernel one workgroup per row: order-preserving compaction of the nonzeros
// Decoding is one launch, one workgroup per row.  All of it is integer/bit work; the traffic is the
// dense matrix (2 B/element) against bitmap + values (1/8 + 2(1-p) B/element).
#include "salr_device.hpp"
#include "salr_internal.hpp"
#include "salr_linear_common.hpp"

namespace salr {

constexpr int kCodecThreads = 256;             // 4 waves
constexpr int kChunkValuesMax = kCodecThreads * kUnit;  // packed values one step can own

template <bool kVec>
__global__ __launch_bounds__(kCodecThreads) void encode_count_kernel(const uint16_t* __restrict__ w,
                                                                     int64_t cols, int64_t wpr,
                                                                     uint32_t* __restrict__ bitmap,
                                                                     uint32_t* __restrict__ row_offsets) {
    __shared__ uint32_t scratch[kCodecThreads / kWave];
    const int64_t n = blockIdx.x;
    const uint16_t* row = w + n * cols;
    const int64_t units = wpr * 4;  // whole words: pad bytes are produced as zeros
    uint32_t count = 0;
    for (int64_t base = 0; base < units; base += kCodecThreads) {
        const int64_t u = base + threadIdx.x;
        const uint32_t m = nonzero_mask8(load_unit<kVec>(row, cols, u));
        count += __popc(m);
        // four neighbouring lanes hold the four bytes of one word
        const uint32_t b1 = __shfl_down(m, 1, kWave);
        const uint32_t b2 = __shfl_down(m, 2, kWave);
        const uint32_t b3 = __shfl_down(m, 3, kWave);
        if ((threadIdx.x & 3) == 0 && u < units) bitmap[n * wpr + (u >> 2)] = m | (b1 << 8) | (b2 << 16) | (b3 << 24);
    }
#pragma unroll
    for (int d = kWave / 2; d > 0; d >>= 1) count += __shfl_down(count, d, kWave);
    if (lane_id() == 0) scratch[threadIdx.x / kWave] = count;
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t s = 0;
        for (int i = 0; i < kCodecThreads / kWave; ++i) s += scratch[i];
        row_offsets[n + 1] = s;  // the scan turns counts into offsets in place
    }
}

constexpr int kScanThreads = 1024;

// row_offsets[1..rows] holds per-row counts on entry and inclusive prefix sums on exit; [0] = 0.
__global__ __launch_bounds__(kScanThreads) void row_scan_kernel(uint32_t* __restrict__ row_offsets, int64_t rows) {
    __shared__ uint32_t scratch[kScanThreads / kWave];
    uint32_t carry = 0;
    for (int64_t base = 0; base < rows; base += kScanThreads) {
        const int64_t i = base + threadIdx.x;
        const uint32_t v = (i < rows) ? row_offsets[i + 1] : 0u;
        uint32_t total;
        const uint32_t excl = block_exclusive_scan<kScanThreads>(v, scratch, total);
        if (i < rows) row_offsets[i + 1] = carry + excl + v;
        carry += total;
    }
    if (threadIdx.x == 0) row_offsets[0] = 0;
}

template <bool kVec>
__global__ __launch_bounds__(kCodecThreads) void encode_compact_kernel(const uint16_t* __restrict__ w,
                                                                       int64_t cols,
                                                                       const uint32_t* __restrict__ row_offsets,
                                                                       uint16_t* __restrict__ values,
                                                                       int64_t capacity) {
    __shared__ uint32_t scratch[kCodecThreads / kWave];
    const int64_t n = blockIdx.x;
    const uint16_t* row = w + n * cols;
    const int64_t units = (cols + kUnit - 1) / kUnit;
    int64_t cursor = row_offsets[n];
    for (int64_t base = 0; base < units; base += kCodecThreads) {
        const int64_t u = base + threadIdx.x;
        const uint4 q = load_unit<kVec>(row, cols, u);
        const uint32_t m = nonzero_mask8(q);
        uint32_t total;
        const uint32_t excl = block_exclusive_scan<kCodecThreads>(__popc(m), scratch, total);
        int64_t idx = cursor + excl;
#pragma unroll
        for (int j = 0; j < kUnit; ++j) {
            if ((m >> j) & 1u) {
                if (idx < capacity) values[idx] = (uint16_t)unit_elem(q, j);
                ++idx;
            }
        }
        cursor += total;
    }
}

// Standalone decoder: per step the workgroup owns 2048 columns of its row; the packed values of the
// step are one contiguous piece of `values`, copied to LDS with aligned dword loads and expanded there.
template <bool kVec>
__global__ __launch_bounds__(kCodecThreads) void decode_kernel(const uint32_t* __restrict__ bitmap,
                                                               const uint16_t* __restrict__ values,
                                                               const uint32_t* __restrict__ row_offsets,
                                                               int64_t rows, int64_t cols, int64_t wpr,
                                                               uint16_t* __restrict__ out) {
    __shared__ uint32_t stage[kChunkValuesMax / 2 + 8];
    __shared__ uint32_t lut[kNibbleLutWords];
    __shared__ uint32_t scratch[kCodecThreads / kWave];
    nibble_lut_init(lut);
    __syncthreads();
    const int64_t n = blockIdx.x;
    const uint8_t* mask_bytes = reinterpret_cast<const uint8_t*>(bitmap + n * wpr);
    const uint32_t* values32 = reinterpret_cast<const uint32_t*>(values);
    uint16_t* row_out = out + n * cols;
    const int64_t units = (cols + kUnit - 1) / kUnit;
    const int64_t nnz = row_offsets[rows];
    int64_t g = row_offsets[n];  // element index in `values` of the next unread value of this row
    for (int64_t base = 0; base < units; base += kCodecThreads) {
        const int64_t u = base + threadIdx.x;
        const uint32_t m = (u < units) ? mask_bytes[u] : 0u;
        uint32_t total;
        const uint32_t excl = block_exclusive_scan<kCodecThreads>(__popc(m), scratch, total);
        const uint32_t parity = (uint32_t)(g & 1);
        const int64_t gdw = g >> 1;
        const uint32_t ndw = (parity + total + 1) >> 1;
        for (uint32_t j = threadIdx.x; j < ndw; j += kCodecThreads) {
            const int64_t e = 2 * (gdw + j);
            uint32_t d;
            if (e + 1 < nnz) d = values32[gdw + j];
            else d = (e < nnz) ? (uint32_t)values[e] : 0u;  // last, half-filled dword of the array
            stage[j] = d;
        }
        __syncthreads();
        if (u < units) {
            const uint4 q = expand_byte(stage, lut, parity + excl, m);
            const int64_t k0 = u * kUnit;
            if constexpr (kVec) {
                *reinterpret_cast<uint4*>(row_out + k0) = q;
            } else {
#pragma unroll
                for (int j = 0; j < kUnit; ++j)
                    if (k0 + j < cols) row_out[k0 + j] = (uint16_t)unit_elem(q, j);
            }
        }
        g += total;
        // the next step's block scan synchronises before `stage` is overwritten
    }
}

// Decoder for rows whose output can be written with 16-byte stores.  One workgroup per row, but the waves
// work on their own: a row is cut into groups of 512 columns (one byte mask per lane), a first pass popcounts
// the bitmap row into per-group start offsets (the only block barriers), then every wave takes groups on its
// own -- wave scan of the byte popcounts, the group's values (one contiguous piece, at most 65 aligned 16-byte
// vectors) copied into the wave's LDS slot, nibble expansion, one 16-byte store per lane -- with the loads of
// its next group already in flight.
constexpr int kDecWaves = kCodecThreads / kWave;
constexpr int kDecMaxGroups = 1024;   // rows up to 524288 columns

__global__ __launch_bounds__(kCodecThreads) void decode_rows_kernel(const uint32_t* __restrict__ bitmap,
                                                                    const uint16_t* __restrict__ values,
                                                                    const uint32_t* __restrict__ row_offsets, int64_t cols,
                                                                    int64_t wpr, uint16_t* __restrict__ out) {
    __shared__ uint32_t prefix[kDecMaxGroups + 1];
    __shared__ __attribute__((aligned(16))) uint32_t slot[kDecWaves][65 * 4 + 8];
    __shared__ uint32_t lut[kNibbleLutWords];
    nibble_lut_init(lut);
    const int lane = lane_id();
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    const int64_t n = blockIdx.x;
    const uint32_t* brow = bitmap + n * wpr;
    const int groups = (int)((wpr + 15) / 16);
    // ---- pass 1: nonzeros per group of 16 words, then their exclusive prefix
    for (int g = threadIdx.x >> 4; g < groups; g += kCodecThreads / 16) {
        const int64_t w = 16 * (int64_t)g + (lane & 15);
        uint32_t c = w < wpr ? __popc(brow[w]) : 0u;
#pragma unroll
        for (int d = 8; d > 0; d >>= 1) c += __shfl_xor(c, d, kWave);
        if ((lane & 15) == 0) prefix[g + 1] = c;
    }
    __syncthreads();
    if (wave == 0) {
        uint32_t carry = 0;
        for (int base = 0; base < groups; base += kWave) {
            const int g = base + lane;
            const uint32_t c = g < groups ? prefix[g + 1] : 0u;
            const uint32_t incl = wave_inclusive_scan(c);
            if (g < groups) prefix[g + 1] = carry + incl;
            carry += __shfl(incl, kWave - 1, kWave);
        }
        if (lane == 0) prefix[0] = 0;
    }
    __syncthreads();
    // ---- pass 2
    const uint8_t* mask_bytes = reinterpret_cast<const uint8_t*>(brow);
    const uint4* values128 = reinterpret_cast<const uint4*>(values);
    uint16_t* row_out = out + n * cols;
    const int64_t units = (cols + kUnit - 1) / kUnit;
    const uint32_t row_start = row_offsets[n];
    uint32_t* my_slot = slot[wave];
    auto group_loads = [&](int g, uint32_t& m, uint4& v, uint32_t& off, uint32_t& nv, uint32_t& vbase) {
        const int64_t u = 64 * (int64_t)g + lane;
        m = (g < groups && u < units) ? mask_bytes[u] : 0u;
        const uint32_t gi = g < groups ? g : groups - 1;
        const uint32_t cursor = row_start + prefix[gi];
        const uint32_t total = g < groups ? prefix[gi + 1] - prefix[gi] : 0u;
        off = cursor & 7u;
        nv = total ? (off + total + 7u) >> 3 : 0u;
        // lanes past the piece repeat its last vector (clamped, not predicated); an empty piece loads nothing new
        const uint32_t li = nv ? ((uint32_t)lane < nv ? lane : nv - 1u) : 0u;
        vbase = cursor >> 3;
        v = nv ? values128[vbase + li] : make_uint4(0, 0, 0, 0);
    };
    uint32_t m, off, nv, vbase;
    uint4 v;
    group_loads(wave, m, v, off, nv, vbase);
    for (int g = wave; g < groups; g += kDecWaves) {
        uint32_t m2, off2, nv2, vbase2;
        uint4 v2;
        group_loads(g + kDecWaves, m2, v2, off2, nv2, vbase2);   // next group of this wave, in flight while this one expands
        const uint32_t incl = wave_inclusive_scan(__popc(m));
        if ((uint32_t)lane < nv) reinterpret_cast<uint4*>(my_slot)[lane] = v;
        // a full group that starts off a vector boundary spans 65 vectors: the last one is fetched on the spot
        if (__builtin_amdgcn_readfirstlane(nv) > 64u && lane == 0) reinterpret_cast<uint4*>(my_slot)[64] = values128[vbase + 64];
        __builtin_amdgcn_wave_barrier();
        const uint4 q = expand_byte(my_slot, lut, off + incl - __popc(m), m);
        __builtin_amdgcn_wave_barrier();
        const int64_t u = 64 * (int64_t)g + lane;
        if (u < units) *reinterpret_cast<uint4*>(row_out + u * kUnit) = q;
        m = m2; v = v2; off = off2; nv = nv2; vbase = vbase2;
    }
}

static bool vec_ok(const void* p, int64_t cols) {
    return (cols % kUnit == 0) && ((reinterpret_cast<uintptr_t>(p) & 15u) == 0);
}

hipError_t launch_encode(const uint16_t* w, int64_t rows, int64_t cols, uint32_t* bitmap, uint16_t* values,
                         int64_t capacity, uint32_t* row_offsets, hipStream_t stream) {
    const int64_t wpr = (cols + 31) / 32;
    const bool vec = vec_ok(w, cols);
    if (rows > 0) {
        if (vec) hipLaunchKernelGGL(encode_count_kernel<true>, dim3((unsigned)rows), dim3(kCodecThreads), 0, stream, w, cols, wpr, bitmap, row_offsets);
        else hipLaunchKernelGGL(encode_count_kernel<false>, dim3((unsigned)rows), dim3(kCodecThreads), 0, stream, w, cols, wpr, bitmap, row_offsets);
    }
    hipLaunchKernelGGL(row_scan_kernel, dim3(1), dim3(kScanThreads), 0, stream, row_offsets, rows);
    if (values != nullptr && rows > 0 && cols > 0) {
        if (vec) hipLaunchKernelGGL(encode_compact_kernel<true>, dim3((unsigned)rows), dim3(kCodecThreads), 0, stream, w, cols, row_offsets, values, capacity);
        else hipLaunchKernelGGL(encode_compact_kernel<false>, dim3((unsigned)rows), dim3(kCodecThreads), 0, stream, w, cols, row_offsets, values, capacity);
    }
    return hipGetLastError();
}

hipError_t launch_decode(const uint32_t* bitmap, const uint16_t* values, const uint32_t* row_offsets, int64_t rows,
                         int64_t cols, uint16_t* out, hipStream_t stream) {
    if (rows == 0 || cols == 0) return hipSuccess;
    const int64_t wpr = (cols + 31) / 32;
    if (vec_ok(out, cols) && (wpr + 15) / 16 <= kDecMaxGroups && (reinterpret_cast<uintptr_t>(values) & 15u) == 0)
        hipLaunchKernelGGL(decode_rows_kernel, dim3((unsigned)rows), dim3(kCodecThreads), 0, stream, bitmap, values, row_offsets, cols, wpr, out);
    else if (vec_ok(out, cols))
        hipLaunchKernelGGL(decode_kernel<true>, dim3((unsigned)rows), dim3(kCodecThreads), 0, stream, bitmap, values, row_offsets, rows, cols, wpr, out);
    else
        hipLaunchKernelGGL(decode_kernel<false>, dim3((unsigned)rows), dim3(kCodecThreads), 0, stream, bitmap, values, row_offsets, rows, cols, wpr, out);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------------
// Slice table (see salr_internal.hpp; the block's work is slice_table_block in salr_linear_common.hpp).  Runs once per
// layer.
// ---------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void slice_table_kernel(const uint32_t* __restrict__ bitmap,
                                                          const uint32_t* __restrict__ row_offsets, int64_t N, int64_t K,
                                                          uint32_t* __restrict__ table) {
    slice_table_block(bitmap, row_offsets, N, K, table, (int64_t)blockIdx.x, (int)threadIdx.x);
}

hipError_t launch_build_slice_table(const uint32_t* bitmap, const uint32_t* row_offsets, int64_t N, int64_t K, uint32_t* table,
                                    hipStream_t stream) {
    if (N <= 0) return hipSuccess;
    hipLaunchKernelGGL(slice_table_kernel, dim3((unsigned)((N + kSliceTableRowsPerBlock - 1) / kSliceTableRowsPerBlock)),
                       dim3(256), 0, stream, bitmap, row_offsets, N, K, table);
    return hipGetLastError();
}

}  // namespace salr
