// Magnitude pruning masks (paper Sec. 2: static mask from a magnitude threshold; Sec. 4: the N:M
// pattern of the inference-throughput comparison).
//
// Row mask: one workgroup per row keeps the `keep` entries of largest |w|, ties to the lower column.
// The threshold is the largest 15-bit magnitude pattern T with count(|w| >= T) >= keep, found by
// fixing its bits from the top (15 counting passes over the row, which sits in LDS when it fits);
// every entry above T is kept, and of the entries equal to T the first keep - count(|w| > T) in
// column order (a block scan over the row).  bf16 magnitudes order like their bit patterns, so all of
// it is integer work and the result is exact.  Traffic: the matrix once in, once out.
#include "salr_device.hpp"
#include "salr_internal.hpp"

namespace salr {

constexpr int kMaskThreads = 256;
constexpr int kMaskWaves = kMaskThreads / kWave;
constexpr int64_t kMaskLdsBytesMax = 60 * 1024;  // dynamic LDS a row may take without raising the default limit

__device__ __forceinline__ uint32_t mag15(uint32_t bits16) { return bits16 & 0x7FFFu; }

// Entries of the eight in q whose magnitude is >= t (t >= 1, so zero padding never counts).
__device__ __forceinline__ uint32_t count_ge8(const uint4& q, uint32_t t) {
    uint32_t c = 0;
    c += mag15(q.x) >= t;
    c += mag15(q.x >> 16) >= t;
    c += mag15(q.y) >= t;
    c += mag15(q.y >> 16) >= t;
    c += mag15(q.z) >= t;
    c += mag15(q.z >> 16) >= t;
    c += mag15(q.w) >= t;
    c += mag15(q.w >> 16) >= t;
    return c;
}

template <bool kLds, bool kVec>
__global__ __launch_bounds__(kMaskThreads) void mask_rows_kernel(const uint16_t* __restrict__ w, int64_t cols,
                                                                 int64_t keep, uint16_t* __restrict__ out) {
    extern __shared__ uint4 row_lds[];        // kLds: the row, ceil(cols/8) units, zero padded
    __shared__ uint32_t red[2][kMaskWaves];   // count reductions, two slots so one barrier per pass is enough
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
    // Number of entries of the row with magnitude >= t, known to every thread.  `slot` alternates.
    auto row_count_ge = [&](uint32_t t, int slot) -> uint32_t {
        uint32_t c = 0;
        for (int64_t u = tid; u < units; u += kMaskThreads) c += count_ge8(unit(u), t);
#pragma unroll
        for (int d = kWave / 2; d > 0; d >>= 1) c += __shfl_down(c, d, kWave);
        if (lane_id() == 0) red[slot][wave] = c;
        __syncthreads();
        uint32_t s = 0;
#pragma unroll
        for (int i = 0; i < kMaskWaves; ++i) s += red[slot][i];
        return s;
    };

    // T = max { t : count(|w| >= t) >= keep }, built bit by bit (count(>= 0) = cols >= keep always holds).
    uint32_t T = 0;
    int slot = 0;
    for (int bit = 14; bit >= 0; --bit) {
        const uint32_t cand = T | (1u << bit);
        if ((int64_t)row_count_ge(cand, slot) >= keep) T = cand;
        slot ^= 1;
    }
    // Entries strictly above T all survive; ties at T fill the remaining places from the left.
    const uint32_t above = (T == 0x7FFFu) ? 0u : row_count_ge(T + 1u, slot);
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
