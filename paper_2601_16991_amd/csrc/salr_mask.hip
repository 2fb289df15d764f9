// Magnitude pruning masks (paper Sec. 2: static mask from a magnitude threshold; Sec. 4: the N:M
// pattern of the inference-throughput comparison).
//
// Row mask: one workgroup per row keeps the `keep` entries of largest |w|, ties to the lower column.
// The threshold is the largest 15-bit magnitude pattern T with count(|w| >= T) >= keep, found by a
// two-level radix select: a histogram of the exponent (the top 8 of the 15 bits) locates T's exponent,
// a histogram of the 7 mantissa bits inside that exponent locates the rest (two passes over the row,
// which sits in LDS when it fits; the histograms are per wave, to spread the LDS atomics);
// every entry above T is kept, and of the entries equal to T the first keep - count(|w| > T) in
// column order (a block scan over the row).  bf16 magnitudes order like their bit patterns, so all of
// it is integer work and the result is exact.  Traffic: the matrix once in, once out.
#include "salr_device.hpp"
#include "salr_internal.hpp"

namespace salr {

constexpr int kMaskThreads = 256;
constexpr int kMaskWaves = kMaskThreads / kWave;
constexpr int64_t kMaskLdsBytesMax = 56 * 1024;  // dynamic LDS a row may take beside the histograms without raising the default limit

__device__ __forceinline__ uint32_t mag15(uint32_t bits16) { return bits16 & 0x7FFFu; }

template <bool kLds, bool kVec>
__global__ __launch_bounds__(kMaskThreads) void mask_rows_kernel(const uint16_t* __restrict__ w, int64_t cols,
                                                                 int64_t keep, uint16_t* __restrict__ out) {
    extern __shared__ uint4 row_lds[];        // kLds: the row, ceil(cols/8) units, zero padded
    __shared__ uint32_t scan_scratch[kMaskWaves + 1];
    const int64_t n = blockIdx.x;
    const uint16_t* row = w + n * cols;
    uint16_t* row_out = out + n * cols;
    const int64_t units = (cols + kUnit - 1) / kUnit;
    const int tid = threadIdx.x;
    const int wave = tid / kWave;

    if constexpr (kLds) {
        for (int64_t u = tid; u < units; u += kMaskThreads) row_lds[u] = load_unit<kVec>(row, cols, u);
        __syncthreads();
    }
    auto unit = [&](int64_t u) -> uint4 {
        if constexpr (kLds) return row_lds[u];
        else return load_unit<kVec>(row, cols, u);
    };
    // Histogram pass: bins[wave][key] += 1 for every entry whose `filter` holds; then the bin of the
    // `want`-th largest key (want >= 1) and the number of entries in bins above it.
    __shared__ uint32_t bins[kMaskWaves][256];
    __shared__ uint32_t found[2];
    auto select_bin = [&](int nbins, auto key_of, auto filter, uint32_t want, uint32_t& bin, uint32_t& above_bin) {
        for (int i = tid; i < kMaskWaves * 256; i += kMaskThreads) bins[i >> 8][i & 255] = 0u;
        __syncthreads();
        for (int64_t u = tid; u < units; u += kMaskThreads) {
            const uint4 q = unit(u);
#pragma unroll
            for (int j = 0; j < kUnit; ++j) {
                const uint32_t m = mag15(unit_elem(q, j));
                if (u * kUnit + j < cols && filter(m)) atomicAdd(&bins[wave][key_of(m)], 1u);
            }
        }
        __syncthreads();
        // thread i owns key nbins - 1 - i: the exclusive scan then counts the entries with a larger key
        const int key = nbins - 1 - tid;
        uint32_t h = 0;
        if (tid < nbins)
#pragma unroll
            for (int w = 0; w < kMaskWaves; ++w) h += bins[w][key];
        uint32_t total;
        const uint32_t larger = block_exclusive_scan<kMaskThreads>(h, scan_scratch, total);
        if (tid < nbins && larger < want && larger + h >= want) {
            found[0] = (uint32_t)key;
            found[1] = larger;
        }
        __syncthreads();
        bin = found[0];
        above_bin = found[1];
        __syncthreads();   // found and bins are reused by the next call
    };

    // T = max { t : count(|w| >= t) >= keep }; above = count(|w| > T).  keep == 0 keeps nothing: T is the largest
    // pattern and nothing is allowed in as a tie.
    uint32_t T = 0x7FFFu, above = 0u;
    if (keep > 0) {
        uint32_t expo, above_expo, mant, above_mant;
        select_bin(256, [](uint32_t m) { return m >> 7; }, [](uint32_t) { return true; }, (uint32_t)keep, expo, above_expo);
        select_bin(128, [](uint32_t m) { return m & 0x7Fu; }, [&](uint32_t m) { return (m >> 7) == expo; },
                   (uint32_t)keep - above_expo, mant, above_mant);
        T = (expo << 7) | mant;
        above = above_expo + above_mant;
    }
    // Entries strictly above T all survive; ties at T fill the remaining places from the left.
    const uint32_t ties_wanted = (uint32_t)(keep - (int64_t)above);

    uint32_t ties_before = 0;  // ties in the columns left of this step
    for (int64_t base = 0; base < units; base += kMaskThreads) {
        const int64_t u = base + tid;
        const int64_t k0 = u * kUnit;
        uint4 q = make_uint4(0, 0, 0, 0);
        if (u < units) q = unit(u);
        uint32_t e[kUnit];
        uint32_t my_ties = 0;
#pragma unroll
        for (int j = 0; j < kUnit; ++j) {
            e[j] = unit_elem(q, j);
            my_ties += (k0 + j < cols) && (mag15(e[j]) == T);
        }
        uint32_t step_ties;
        uint32_t tie_rank = ties_before + block_exclusive_scan<kMaskThreads>(my_ties, scan_scratch, step_ties);
        ties_before += step_ties;
#pragma unroll
        for (int j = 0; j < kUnit; ++j) {
            const uint32_t m = mag15(e[j]);
            bool kept = m > T;
            if (m == T && k0 + j < cols) {
                kept = tie_rank < ties_wanted;
                ++tie_rank;
            }
            if (!kept) e[j] = 0u;
        }
        if (u < units) {
            if constexpr (kVec) {
                uint4 o;
                o.x = e[0] | (e[1] << 16);
                o.y = e[2] | (e[3] << 16);
                o.z = e[4] | (e[5] << 16);
                o.w = e[6] | (e[7] << 16);
                *reinterpret_cast<uint4*>(row_out + k0) = o;
            } else {
#pragma unroll
                for (int j = 0; j < kUnit; ++j)
                    if (k0 + j < cols) row_out[k0 + j] = (uint16_t)e[j];
            }
        }
    }
}

// Row mask for rows of up to 64 * kUPL units (8 columns each) that allow 16-byte accesses: ONE WAVE per row, the
// row in registers (lane l holds units l, l + 64, ...), the threshold by a bit search with wave reductions, the tie
// ranking with wave scans: no LDS, no barrier.  Four rows per workgroup.
template <int kUPL>
__global__ __launch_bounds__(kMaskThreads) void mask_rows_wave_kernel(const uint16_t* __restrict__ w, int64_t rows, int64_t cols,
                                                                      int64_t keep, uint16_t* __restrict__ out) {
    const int lane = lane_id();
    const int wave = threadIdx.x / kWave;
    const int64_t n = (int64_t)blockIdx.x * kMaskWaves + wave;
    if (n >= rows) return;   // wave-uniform; nothing below synchronises across waves
    const uint16_t* row = w + n * cols;
    uint16_t* row_out = out + n * cols;
    const int units = (int)(cols / kUnit);
    uint4 q[kUPL];
#pragma unroll
    for (int i = 0; i < kUPL; ++i) {
        const int u = lane + kWave * i;
        q[i] = u < units ? *reinterpret_cast<const uint4*>(row + (int64_t)u * kUnit) : make_uint4(0, 0, 0, 0);
    }
    // Magnitudes two to a dword with bit 15 of each half set: (m | 0x8000) - t never borrows for t <= 0x7FFF, so one
    // 32-bit subtraction compares both halves, and bit 15 of a half of the difference says m >= t.
    uint32_t pm[kUPL][4];
#pragma unroll
    for (int i = 0; i < kUPL; ++i) {
        pm[i][0] = (q[i].x & 0x7FFF7FFFu) | 0x80008000u;
        pm[i][1] = (q[i].y & 0x7FFF7FFFu) | 0x80008000u;
        pm[i][2] = (q[i].z & 0x7FFF7FFFu) | 0x80008000u;
        pm[i][3] = (q[i].w & 0x7FFF7FFFu) | 0x80008000u;
    }
    // entries of the row with magnitude >= t (1 <= t <= 0x7FFF; the zero padding never counts), in every lane
    auto row_count_ge = [&](uint32_t t) -> uint32_t {
        const uint32_t tt = t | (t << 16);
        uint32_t c = 0;
#pragma unroll
        for (int i = 0; i < kUPL; ++i)
#pragma unroll
            for (int d = 0; d < 4; ++d) c += __popc((pm[i][d] - tt) & 0x80008000u);
#pragma unroll
        for (int d = 1; d < kWave; d <<= 1) c += __shfl_xor(c, d, kWave);
        return c;
    };
    // T = max { t : count(|w| >= t) >= keep }, built bit by bit from the top (15 passes over the registers;
    // a histogram select needs fewer passes but its LDS atomics pile up on the few exponents real weights have)
    uint32_t T = 0;
    for (int bit = 14; bit >= 0; --bit) {
        const uint32_t cand = T | (1u << bit);
        if ((int64_t)row_count_ge(cand) >= keep) T = cand;
    }
    const uint32_t above = (T == 0x7FFFu) ? 0u : row_count_ge(T + 1u);
    const uint32_t ties_wanted = (uint32_t)(keep - (int64_t)above);
    uint32_t ties_before = 0;   // ties in the units before round i (units run lane-fastest, so rounds are in column order)
#pragma unroll
    for (int i = 0; i < kUPL; ++i) {
        const int u = lane + kWave * i;
        uint32_t e[kUnit], my_ties = 0;
#pragma unroll
        for (int j = 0; j < kUnit; ++j) {
            e[j] = unit_elem(q[i], j);
            my_ties += (u < units) && (mag15(e[j]) == T);
        }
        uint32_t tie_rank = ties_before;
        if (__builtin_amdgcn_ballot_w64(my_ties != 0) != 0) {   // wave-uniform; most rounds of real data hold no tie
            const uint32_t incl = wave_inclusive_scan(my_ties);
            tie_rank += incl - my_ties;
            ties_before += __shfl(incl, kWave - 1, kWave);
        }
#pragma unroll
        for (int j = 0; j < kUnit; ++j) {
            const uint32_t m = mag15(e[j]);
            bool kept = m > T;
            if (m == T) {
                kept = tie_rank < ties_wanted;
                ++tie_rank;
            }
            if (!kept) e[j] = 0u;
        }
        if (u < units) {
            uint4 o;
            o.x = e[0] | (e[1] << 16);
            o.y = e[2] | (e[3] << 16);
            o.z = e[4] | (e[5] << 16);
            o.w = e[6] | (e[7] << 16);
            *reinterpret_cast<uint4*>(row_out + (int64_t)u * kUnit) = o;
        }
    }
}

// N:M mask, one thread per group of m consecutive columns: entry i survives iff fewer than n entries
// of its group come before it in the order (larger magnitude first, lower column first among equals).
template <int kM>
__global__ __launch_bounds__(256) void mask_nm_fixed_kernel(const uint16_t* __restrict__ w, int64_t groups,
                                                            int n_keep, uint16_t* __restrict__ out) {
    typedef uint16_t group_t __attribute__((ext_vector_type(kM)));  // 2*kM bytes, aligned because cols % kM == 0
    const int64_t g = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (g >= groups) return;
    const group_t v = reinterpret_cast<const group_t*>(w)[g];
    group_t o;
#pragma unroll
    for (int i = 0; i < kM; ++i) {
        const uint32_t mi = mag15(v[i]);
        int before = 0;
#pragma unroll
        for (int j = 0; j < kM; ++j) {
            const uint32_t mj = mag15(v[j]);
            before += (mj > mi) || (mj == mi && j < i);
        }
        o[i] = before < n_keep ? v[i] : (uint16_t)0;
    }
    reinterpret_cast<group_t*>(out)[g] = o;
}

__global__ __launch_bounds__(256) void mask_nm_any_kernel(const uint16_t* __restrict__ w, int64_t groups,
                                                          int n_keep, int m_group, uint16_t* __restrict__ out) {
    const int64_t g = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (g >= groups) return;
    const uint16_t* src = w + g * m_group;
    uint16_t* dst = out + g * m_group;
    for (int i = 0; i < m_group; ++i) {
        const uint32_t mi = mag15(src[i]);
        int before = 0;
        for (int j = 0; j < m_group; ++j) {
            const uint32_t mj = mag15(src[j]);
            before += (mj > mi) || (mj == mi && j < i);
        }
        dst[i] = before < n_keep ? src[i] : (uint16_t)0;
    }
}

hipError_t launch_mask_rows(const uint16_t* w, int64_t rows, int64_t cols, int64_t keep, uint16_t* out,
                            hipStream_t stream) {
    if (rows == 0 || cols == 0) return hipSuccess;
    const int64_t units = (cols + kUnit - 1) / kUnit;
    const size_t row_bytes = (size_t)units * sizeof(uint4);
    const bool lds = row_bytes <= (size_t)kMaskLdsBytesMax;
    const bool vec = (cols % kUnit == 0) && (((reinterpret_cast<uintptr_t>(w) | reinterpret_cast<uintptr_t>(out)) & 15u) == 0);
    if (vec && units <= kWave * 16) {   // the row fits the registers of one wave
        const dim3 wgrid((unsigned)((rows + kMaskWaves - 1) / kMaskWaves));
        if (units <= kWave * 4) hipLaunchKernelGGL((mask_rows_wave_kernel<4>), wgrid, dim3(kMaskThreads), 0, stream, w, rows, cols, keep, out);
        else if (units <= kWave * 8) hipLaunchKernelGGL((mask_rows_wave_kernel<8>), wgrid, dim3(kMaskThreads), 0, stream, w, rows, cols, keep, out);
        else hipLaunchKernelGGL((mask_rows_wave_kernel<16>), wgrid, dim3(kMaskThreads), 0, stream, w, rows, cols, keep, out);
        return hipGetLastError();
    }
    const dim3 grid((unsigned)rows), block(kMaskThreads);
    const size_t dyn = lds ? row_bytes : 0;
    if (lds && vec) hipLaunchKernelGGL((mask_rows_kernel<true, true>), grid, block, dyn, stream, w, cols, keep, out);
    else if (lds) hipLaunchKernelGGL((mask_rows_kernel<true, false>), grid, block, dyn, stream, w, cols, keep, out);
    else if (vec) hipLaunchKernelGGL((mask_rows_kernel<false, true>), grid, block, dyn, stream, w, cols, keep, out);
    else hipLaunchKernelGGL((mask_rows_kernel<false, false>), grid, block, dyn, stream, w, cols, keep, out);
    return hipGetLastError();
}

hipError_t launch_mask_nm(const uint16_t* w, int64_t rows, int64_t cols, int n_keep, int m_group, uint16_t* out,
                          hipStream_t stream) {
    const int64_t groups = rows * (cols / m_group);
    if (groups == 0) return hipSuccess;
    const dim3 grid((unsigned)((groups + 255) / 256)), block(256);
    const bool aligned = (((reinterpret_cast<uintptr_t>(w) | reinterpret_cast<uintptr_t>(out)) & 15u) == 0);
    if (aligned && m_group == 2) hipLaunchKernelGGL((mask_nm_fixed_kernel<2>), grid, block, 0, stream, w, groups, n_keep, out);
    else if (aligned && m_group == 4) hipLaunchKernelGGL((mask_nm_fixed_kernel<4>), grid, block, 0, stream, w, groups, n_keep, out);
    else if (aligned && m_group == 8) hipLaunchKernelGGL((mask_nm_fixed_kernel<8>), grid, block, 0, stream, w, groups, n_keep, out);
    else hipLaunchKernelGGL(mask_nm_any_kernel, grid, block, 0, stream, w, groups, n_keep, m_group, out);
    return hipGetLastError();
}

}  // namespace salr
