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
#include "salr_nf4.hpp"

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

// kNf4 (QSALR, paper Sec. 4): `values` are the 4-bit codes, eight to a dword where the bf16 kernel has a 16-byte vector of
// eight values; a lane dequantises its dword (all eight codes lie in one scale block of 64) on the way into the slot,
// and everything after that is the same.  scale_last: index of the last scale.
template <bool kNf4>
__global__ __launch_bounds__(kCodecThreads) void decode_rows_kernel(const uint32_t* __restrict__ bitmap,
                                                                    const uint16_t* __restrict__ values,
                                                                    const uint32_t* __restrict__ row_offsets, int64_t cols,
                                                                    int64_t wpr, uint16_t* __restrict__ out,
                                                                    const uint16_t* __restrict__ scales, uint32_t scale_last) {
    __shared__ uint32_t prefix[kDecMaxGroups + 1];
    __shared__ float levels[16];
    if (kNf4 && threadIdx.x < 16) levels[threadIdx.x] = kNf4Levels[threadIdx.x];
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
    const uint32_t* codes32 = reinterpret_cast<const uint32_t*>(values);
    // vector j of the packed values as requested (16 bytes of bf16; or dword j of the codes in .x and its scale in .y)
    // and as it goes into the slot (the codes dequantised: only then does the wave wait for the request)
    auto fetch = [&](uint32_t j) -> uint4 {
        if constexpr (kNf4) {
            const uint32_t blk = j >> 3;
            return make_uint4(codes32[j], scales[blk < scale_last ? blk : scale_last], 0u, 0u);
        } else {
            return values128[j];
        }
    };
    auto ready = [&](const uint4& q) -> uint4 {
        if constexpr (kNf4) return nf4_decode8(q.x, bf16_bits_to_f32(q.y), levels);
        else return q;
    };
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
        v = nv ? fetch(vbase + li) : make_uint4(0, 0, 0, 0);
    };
    uint32_t m, off, nv, vbase;
    uint4 v;
    group_loads(wave, m, v, off, nv, vbase);
    for (int g = wave; g < groups; g += kDecWaves) {
        uint32_t m2, off2, nv2, vbase2;
        uint4 v2;
        group_loads(g + kDecWaves, m2, v2, off2, nv2, vbase2);   // next group of this wave, in flight while this one expands
        const uint32_t incl = wave_inclusive_scan(__popc(m));
        if ((uint32_t)lane < nv) reinterpret_cast<uint4*>(my_slot)[lane] = ready(v);
        // a full group that starts off a vector boundary spans 65 vectors: the last one is fetched on the spot
        if (__builtin_amdgcn_readfirstlane(nv) > 64u && lane == 0) reinterpret_cast<uint4*>(my_slot)[64] = ready(fetch(vbase + 64));
        __builtin_amdgcn_wave_barrier();
        const uint4 q = expand_byte(my_slot, lut, off + incl - __popc(m), m);
        __builtin_amdgcn_wave_barrier();
        const int64_t u = 64 * (int64_t)g + lane;
        if (u < units) *reinterpret_cast<uint4*>(row_out + u * kUnit) = q;
        m = m2; v = v2; off = off2; nv = nv2; vbase = vbase2;
    }
}

static bool vec_ok(const void* p, int64_t cols);

// QSALR: decode from the 4-bit codes straight into the dense matrix (no bf16 copy of the values in between)
bool decode_nf4_takes(int64_t rows, int64_t cols, int64_t nnz, const void* codes, const void* out) {
    const int64_t wpr = (cols + 31) / 32;
    return rows > 0 && cols > 0 && nnz > 0 && vec_ok(out, cols) && (wpr + 15) / 16 <= kDecMaxGroups &&
           (reinterpret_cast<uintptr_t>(codes) & 3u) == 0;
}

hipError_t launch_decode_nf4(const uint32_t* bitmap, const uint8_t* codes, const uint16_t* scales, int64_t nnz,
                             const uint32_t* row_offsets, int64_t rows, int64_t cols, uint16_t* out, hipStream_t stream) {
    const int64_t wpr = (cols + 31) / 32;
    hipLaunchKernelGGL(decode_rows_kernel<true>, dim3((unsigned)rows), dim3(kCodecThreads), 0, stream, bitmap,
                       reinterpret_cast<const uint16_t*>(codes), row_offsets, cols, wpr, out, scales,
                       (uint32_t)((nnz + kNf4Block - 1) / kNf4Block - 1));
    return hipGetLastError();
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
        hipLaunchKernelGGL(decode_rows_kernel<false>, dim3((unsigned)rows), dim3(kCodecThreads), 0, stream, bitmap, values,
                           row_offsets, cols, wpr, out, (const uint16_t*)nullptr, 0u);
    else if (vec_ok(out, cols))
        hipLaunchKernelGGL(decode_kernel<true>, dim3((unsigned)rows), dim3(kCodecThreads), 0, stream, bitmap, values, row_offsets, rows, cols, wpr, out);
    else
        hipLaunchKernelGGL(decode_kernel<false>, dim3((unsigned)rows), dim3(kCodecThreads), 0, stream, bitmap, values, row_offsets, rows, cols, wpr, out);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------------
// Decode into the TRANSPOSED dense matrix, out_t [cols, rows] (the backward pass contracts over the weight's rows and
// wants them contiguous): the reconstruction rule of Sec. 3.3 as in the kernels above, with the transposition done in
// LDS on the way out, so that the dense matrix crosses memory once instead of three times (decode, then read and
// write again to transpose).  cols % 128 == 0, rows % 64 == 0.
//   workgroup (b, z): rows 64 b .. 64 b + 63 (wave w the 16 rows 16 w ..), chunks [C z / ksl, C (z + 1) / ksl) of the
//   C = cols / 128 chunks of 128 columns.  Per chunk lane (n = lane%16, g = lane/16) expands byte g of the four bitmap
//   words of row n, as in the small-batch linear, and writes its 32 values into an LDS tile [128 columns][64 rows];
//   after a barrier the 256 threads store the tile's rows, 128 bytes each, with 16-byte stores.
//   The packed values of the next chunk are in flight while this one is expanded.
// ---------------------------------------------------------------------------------------------------
constexpr int kDtWaves = 4;
constexpr int kDtThreads = kDtWaves * 64;
constexpr int kDtRows = 16 * kDtWaves;
constexpr int kDtPitch = kDtRows + 8;     // bf16 elements per tile row: 144 bytes, 16-byte aligned, banks spread
constexpr int kDtSlotDwords = 68;         // per row and chunk: 17 vectors of 16 B (128 values + misalignment)

struct DtStage {
    uint4 bm;
    uint4 vq[3];
    uint32_t off, nv, vbase;
};

__global__ __launch_bounds__(kDtThreads) void decode_transposed_kernel(const uint32_t* __restrict__ bitmap,
                                                                       const uint16_t* __restrict__ values,
                                                                       const uint32_t* __restrict__ row_offsets, int64_t rows,
                                                                       int64_t cols, int ksl, uint16_t* __restrict__ out_t) {
    __shared__ __attribute__((aligned(16))) uint16_t tile[128 * kDtPitch];
    __shared__ __attribute__((aligned(16))) uint32_t slots[kDtWaves * 16 * kDtSlotDwords + 8];
    __shared__ uint32_t lut[kNibbleLutWords];
    nibble_lut_init(lut);
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int n = lane & 15, g = lane >> 4;
    const int64_t n0 = (int64_t)blockIdx.x * kDtRows;
    const int64_t row = n0 + 16 * wave + n;
    const int64_t row_c = row;   // rows % 64 == 0: every row of the block exists
    const int64_t wpr = cols >> 5;
    const int64_t chunks = wpr >> 2;
    const int z = blockIdx.y;
    const int64_t c_begin = chunks * z / ksl, c_end = chunks * (z + 1) / ksl;   // the same for the whole workgroup
    const uint32_t* brow = bitmap + row_c * wpr;
    // nonzeros of the row left of the slice: the 4 lanes of a row share the words, 8 loads in flight each
    uint32_t cur = row_offsets[row_c];
    {
        uint32_t before = 0;
        for (int64_t c0 = 0; c0 < c_begin; c0 += 32) {
            uint4 q[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int64_t c = c0 + g + 4 * i;
                q[i] = *reinterpret_cast<const uint4*>(brow + (c < c_begin ? c : 0) * 4);
            }
#pragma unroll
            for (int i = 0; i < 8; ++i)
                before += (c0 + g + 4 * i < c_begin) ? __popc(q[i].x) + __popc(q[i].y) + __popc(q[i].z) + __popc(q[i].w) : 0u;
        }
        before += __shfl_xor(before, 16, 64);
        before += __shfl_xor(before, 32, 64);
        cur += before;
    }
    const uint4* values128 = reinterpret_cast<const uint4*>(values);
    uint32_t* slot = slots + (wave * 16 + n) * kDtSlotDwords;
    // chunks past the slice read its last chunk and count as empty (no conditional load in the stream)
    auto issue = [&](DtStage& st, int64_t c) {
        uint4 bm = *reinterpret_cast<const uint4*>(brow + (c < c_end ? c : c_end - 1) * 4);
        const uint32_t keep = c < c_end ? 0xFFFFFFFFu : 0u;
        bm.x &= keep; bm.y &= keep; bm.z &= keep; bm.w &= keep;
        st.bm = bm;
        const uint32_t len = __popc(bm.x) + __popc(bm.y) + __popc(bm.z) + __popc(bm.w);
        st.off = cur & 7u;
        st.nv = len ? (st.off + len + 7u) >> 3 : 0u;
        st.vbase = cur >> 3;
        const uint32_t last = st.nv ? st.nv - 1u : 0u;
        // an empty piece reads the bitmap instead (always mapped: cols >= 128 gives every row 16 bytes)
        const uint4* vb = st.nv ? values128 + st.vbase : reinterpret_cast<const uint4*>(brow);
        cur += len;
#pragma unroll
        for (int i = 0; i < 3; ++i) {
            const uint32_t v = g + 4 * i;
            st.vq[i] = vb[v < last ? v : last];
        }
    };
    __syncthreads();   // the lookup table
    if (c_begin >= c_end) return;   // the same for the whole workgroup
    DtStage st[2];
    issue(st[0], c_begin);
    issue(st[1], c_begin + 1);
    for (int64_t c = c_begin; c < c_end; c += 2) {
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            if (c + i < c_end) {   // the same for the whole workgroup
                const DtStage& s0 = st[i];
#pragma unroll
                for (int v = 0; v < 3; ++v) *reinterpret_cast<uint4*>(slot + 4 * (g + 4 * v)) = s0.vq[v];
                if (s0.nv > 12u) {   // a piece of more than 89 values: fetch the rest now
#pragma unroll
                    for (int v3 = 3; v3 < 5; ++v3) {
                        const uint32_t v = g + 4 * v3;
                        if (v < 17u) *reinterpret_cast<uint4*>(slot + 4 * v) = values128[s0.vbase + (v < s0.nv - 1u ? v : s0.nv - 1u)];
                    }
                }
                __builtin_amdgcn_wave_barrier();
                const uint32_t words[4] = {s0.bm.x, s0.bm.y, s0.bm.z, s0.bm.w};
                uint32_t c_local = s0.off;
#pragma unroll
                for (int s = 0; s < 4; ++s) {
                    const uint32_t word = words[s];
                    const uint32_t m8 = (word >> (8 * g)) & 0xFFu;
                    const uint32_t cb = c_local + __popc(word & ((1u << (8 * g)) - 1u));
                    const uint4 wq = expand_byte(slot, lut, cb, m8);
                    c_local += __popc(word);
                    const uint32_t e[4] = {wq.x, wq.y, wq.z, wq.w};
                    uint16_t* col = tile + (32 * s + 8 * g) * kDtPitch + 16 * wave + n;   // column 32 s + 8 g of the chunk
#pragma unroll
                    for (int j = 0; j < 8; ++j) col[j * kDtPitch] = (uint16_t)(e[j >> 1] >> (16 * (j & 1)));
                }
                issue(st[i], c + i + 2);
                // barriers that wait for LDS traffic only: the requests of the next chunks stay in flight
                asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");   // the tile is complete
                const int64_t k0 = (c + i) * 128;
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    const int idx = tid + kDtThreads * t;
                    const int kr = idx >> 3, v = idx & 7;
                    *reinterpret_cast<uint4*>(out_t + (k0 + kr) * rows + n0 + 8 * v) =
                        *reinterpret_cast<const uint4*>(tile + kr * kDtPitch + 8 * v);
                }
                asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");   // the tile may be overwritten
            }
        }
    }
}

bool decode_transposed_takes(int64_t rows, int64_t cols, const void* values, const void* out_t) {
    return rows > 0 && rows % kDtRows == 0 && cols >= 128 && cols % 128 == 0 && (reinterpret_cast<uintptr_t>(values) & 15u) == 0 &&
           (reinterpret_cast<uintptr_t>(out_t) & 15u) == 0;
}

hipError_t launch_decode_transposed(const uint32_t* bitmap, const uint16_t* values, const uint32_t* row_offsets, int64_t rows,
                                    int64_t cols, uint16_t* out_t, hipStream_t stream) {
    const int64_t blocks = (rows + kDtRows - 1) / kDtRows, chunks = cols / 128;
    int64_t ksl = (1024 + blocks - 1) / blocks;   // about four workgroups per CU
    ksl = ksl < 1 ? 1 : (ksl > chunks ? chunks : ksl);
    if (ksl > 65535) ksl = 65535;
    hipLaunchKernelGGL(decode_transposed_kernel, dim3((unsigned)blocks, (unsigned)ksl), dim3(kDtThreads), 0, stream, bitmap, values,
                       row_offsets, rows, cols, (int)ksl, out_t);
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
