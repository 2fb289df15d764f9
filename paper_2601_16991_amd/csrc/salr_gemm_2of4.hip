// The SALR linear on 2:4-masked weights for large batches (M > 128): a tiled GEMM on the sparse matrix-core
// instruction whose sparse operand is the SALR format as it is (Sec. 3.3: packed values, bitmap), so that there is
// neither a decode stage nor a dense copy of the weight, and the weight tile in LDS is half as wide as a dense one.
//
//   workgroup   4 waves, output tile 128 (n) x 128 (m), k-step 64 columns; wave (wn, wm) owns 64 x 64 = 4 x 4 tiles
//               of v_smfmac_f32_16x16x64_bf16 (one instruction per tile and step), D[n][m] (the sparse operand is the
//               first one, so the weight rows are the rows of D);
//   LDS         per k-step, double buffered: the X tile [128 x 64] (row pitch 144 bytes), the packed values of the
//               weight tile [128 rows x 32 values] (row pitch 80 bytes; a row's values of a k-step are 64 contiguous
//               bytes of `values` at row_offsets[n] + columns / 2) and the index fields of the tile's bitmap words [128 x 2]; fetched one
//               step ahead into registers, written to LDS after the barrier that retires the buffer; one barrier per
//               step;
//   operands    lane (n, kb) of the sparse operand: the 4 stored values of columns 8 kb .. 8 kb + 7 of a 32-column
//               half step (8 bytes from the values tile) and its index byte (byte kb of the word of index fields); lane (m, kb) of the dense operand: X[m][8 kb .. 8 kb + 7] of the half step;
//   adapters    after the K loop, dense MFMAs with B_cat columns as first and T = X A_cat (bf16, from the large-batch
//               adapter stage) as second operand add into the same D[n][m] (Sec. 3.2);
//   output      a lane holds four consecutive outputs n of one token: one 8-byte store.
// Consecutive workgroup ids land on different XCDs; all m-tiles of an n-tile stay on one XCD (one L2 holds its weights).
// As in the small-batch 2:4 kernels the precondition is the caller's and value offsets are clamped to the stored count.
#include <hip/hip_ext.h>

#include "salr_device.hpp"
#include "salr_internal.hpp"
#include "salr_linear_common.hpp"

namespace salr {

constexpr int kG4K = 64;
constexpr int kG4XPitch = 72;   // bf16 elements per X tile row: 144 bytes, 16 rows x 16 bytes then cover all banks once
constexpr int kG4WPitch = 40;   // bf16 elements per values tile row: 80 bytes
constexpr int kG4Xcds = 8;

typedef __bf16 bf16x16 __attribute__((ext_vector_type(16)));
typedef uint32_t g4_u32x4 __attribute__((ext_vector_type(4)));   // native vectors: the compiler keeps arrays of them in registers
typedef uint32_t g4_u32x2 __attribute__((ext_vector_type(2)));

// per nibble with two set bits at p0 < p1: p0 | p1 << 2 (the index field of the sparse MFMA)
__device__ __forceinline__ uint32_t g4_index_codes(uint32_t w) {
    const uint32_t ones = 0x11111111u;
    const uint32_t b0 = w & ones, b1 = (w >> 1) & ones, b2 = (w >> 2) & ones, b3 = (w >> 3) & ones;
    const uint32_t n0 = b0 ^ ones, n1 = b1 ^ ones, n2 = b2 ^ ones;
    return (n0 & b1) | ((n0 & n1) << 1) | ((b3 | n2) << 2) | ((b3 | b2) << 3);
}

// kWN x kWM waves; a wave owns kNI x kMJ tiles of 16 x 16: output tile 16 kNI kWN (n) x 16 kMJ kWM (m).
template <int kWN, int kWM, int kNI, int kMJ>
__global__ __launch_bounds__(64 * kWN * kWM, kWN * kWM <= 4 ? 2 : 1) void gemm_2of4_kernel(
    const uint16_t* __restrict__ x, int64_t M, int64_t K, int64_t N, const uint32_t* __restrict__ bitmap,
    const uint16_t* __restrict__ values, const uint32_t* __restrict__ row_offsets, const uint16_t* __restrict__ t,
    const uint16_t* __restrict__ b_cat, int R, int Rpad, uint16_t* __restrict__ y, int m_tiles, int n_tiles) {
    constexpr int kG4N = 16 * kNI * kWN, kG4M = 16 * kMJ * kWM, kG4Threads = 64 * kWN * kWM;
    constexpr int kXV = kG4M * 8 / kG4Threads;                              // 16-byte vectors per thread and step
    constexpr int kWV = (kG4N * 4 + kG4Threads - 1) / kG4Threads;           // (a 224-row tile leaves the last waves idle here)
    static_assert(kXV * kG4Threads == kG4M * 8 && kG4N * 2 <= kG4Threads && (kG4N * 4) % 64 == 0 && (kG4N * 2) % 64 == 0,
                  "loader shape: whole waves take part or sit out");
    __shared__ __attribute__((aligned(16))) uint16_t xs[2][kG4M * kG4XPitch];
    __shared__ __attribute__((aligned(16))) uint16_t ws[2][kG4N * kG4WPitch];
    __shared__ uint32_t bms[2][kG4N * 2];

    const int bid = blockIdx.x;
    const int xcd = bid % kG4Xcds, local = bid / kG4Xcds;
    const int nt = (local / m_tiles) * kG4Xcds + xcd;
    const int mt = local % m_tiles;
    if (nt >= n_tiles) return;  // uniform for the workgroup, before any barrier
    const int64_t n0 = (int64_t)nt * kG4N, m0 = (int64_t)mt * kG4M;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wn = wave / kWM, wm = wave % kWM;
    const int li = lane & 15, kb = lane >> 4;
    const int64_t wpr = K >> 5;
    const int64_t steps = K / kG4K;

    // ---- loader roles.  X: 4 vectors of 16 bytes per thread and step; values: 2; bitmap: one word.
    const uint16_t* xsrc[kXV];
    int xdst[kXV];
#pragma unroll
    for (int j = 0; j < kXV; ++j) {
        const int idx = tid + kG4Threads * j, row = idx >> 3, seg = idx & 7;
        const int64_t m = m0 + row < M ? m0 + row : M - 1;   // rows past M repeat row M-1; never stored
        xsrc[j] = x + m * K + 8 * seg;
        xdst[j] = row * kG4XPitch + 8 * seg;
    }
    const uint32_t nnz = row_offsets[N];
    const uint32_t e_max = nnz >= 8u ? nnz - 8u : 0u;
    const uint16_t* vsrc = nnz >= 8u ? values : x;   // (a weight this small cannot meet the precondition)
    // The values tile is stored so that a lane of the sparse operand finds its two sets of four values side by side
    // (one 16-byte read): quad q (values 4 q .. 4 q + 3 of the row's 32) belongs to set (q / 2) % 2 of lane block
    // q / 4 + 2 (q % 2) and goes to element 8 block + 4 set of the row.
    uint32_t wbase[kWV];
    int wdst[kWV][2];
#pragma unroll
    for (int j = 0; j < kWV; ++j) {
        const int idx = tid + kG4Threads * j, row = (idx >> 2) < kG4N ? (idx >> 2) : kG4N - 1, seg = idx & 3;
        const int64_t n = n0 + row < N ? n0 + row : N - 1;   // rows past N repeat row N-1; never stored
        wbase[j] = row_offsets[n] + 8u * (uint32_t)seg;
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int q = 2 * seg + h;
            wdst[j][h] = row * kG4WPitch + 8 * ((q >> 2) + 2 * (q & 1)) + 4 * ((q >> 1) & 1);
        }
    }
    const int brow = (tid >> 1) < kG4N ? (tid >> 1) : kG4N - 1, bw = tid & 1;
    const bool b_loader = tid < 2 * kG4N;   // wave-uniform, like the w_loader conditions below
    const uint32_t* bsrc = bitmap + (n0 + brow < N ? n0 + brow : N - 1) * wpr + bw;

    g4_u32x4 xr[kXV], wr[kWV];
    uint32_t br = 0;
    auto load_regs = [&](int64_t s) {
#pragma unroll
        for (int j = 0; j < kXV; ++j) xr[j] = *reinterpret_cast<const g4_u32x4*>(xsrc[j] + s * kG4K);
#pragma unroll
        for (int j = 0; j < kWV; ++j) {
            if (tid + kG4Threads * j < kG4N * 4) {
                uint32_t e = wbase[j] + 32u * (uint32_t)s;
                e = (e < e_max ? e : e_max) & ~7u;   // in bounds and 16-byte aligned whatever the offsets are
                wr[j] = *reinterpret_cast<const g4_u32x4*>(vsrc + e);
            }
        }
        if (b_loader) br = bsrc[2 * s];
    };
    auto store_regs = [&](int buf) {
#pragma unroll
        for (int j = 0; j < kXV; ++j) *reinterpret_cast<g4_u32x4*>(&xs[buf][xdst[j]]) = xr[j];
#pragma unroll
        for (int j = 0; j < kWV; ++j) {
            if (tid + kG4Threads * j < kG4N * 4) {
                *reinterpret_cast<g4_u32x2*>(&ws[buf][wdst[j][0]]) = g4_u32x2{wr[j].x, wr[j].y};
                *reinterpret_cast<g4_u32x2*>(&ws[buf][wdst[j][1]]) = g4_u32x2{wr[j].z, wr[j].w};
            }
        }
        if (b_loader) bms[buf][2 * brow + bw] = g4_index_codes(br);   // the index fields of the word's four bytes, computed once per tile
    };

    f32x4 acc[kNI][kMJ];
#pragma unroll
    for (int i = 0; i < kNI; ++i)
#pragma unroll
        for (int j = 0; j < kMJ; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};

    // One v_smfmac_f32_16x16x64_bf16 per tile pair and step.  Its operands (layout found with a probe on the device:
    // unit values in the dense operand, coded values and index patterns in the sparse one): lane (m, kb) of the dense
    // operand holds columns 16 kb .. 16 kb + 15 of the step; lane (n, kb) of the sparse one holds two sets of four
    // stored values, those of columns c .. c + 7 and c + 16 .. c + 23 with c = 32 (kb % 2) + 8 (kb / 2), and 16 index
    // bits: the index byte of the first set below that of the second.
    auto compute = [&](int buf) {
        bf16x8 a[kNI];
        int idx[kNI];
        bf16x16 b[kMJ];
        const int sh = 8 * (kb >> 1);                   // bitmap byte of the first set: byte kb / 2 of word kb % 2
#pragma unroll
        for (int i = 0; i < kNI; ++i) {
            const int nrow = 16 * kNI * wn + 16 * i + li;
            const uint32_t cw = bms[buf][2 * nrow + (kb & 1)];
            idx[i] = (int)(((cw >> sh) & 0xFFu) | ((cw >> (sh + 8)) & 0xFF00u));
            a[i] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const g4_u32x4*>(&ws[buf][nrow * kG4WPitch + 8 * kb]));
        }
#pragma unroll
        for (int j = 0; j < kMJ; ++j) {
            const uint16_t* xrow = &xs[buf][(16 * kMJ * wm + 16 * j + li) * kG4XPitch + 16 * kb];
            const g4_u32x4 b0 = *reinterpret_cast<const g4_u32x4*>(xrow), b1 = *reinterpret_cast<const g4_u32x4*>(xrow + 8);
            uint32_t w16[8] = {b0.x, b0.y, b0.z, b0.w, b1.x, b1.y, b1.z, b1.w};
            __builtin_memcpy(&b[j], w16, 32);
        }
#pragma unroll
        for (int i = 0; i < kNI; ++i)
#pragma unroll
            for (int j = 0; j < kMJ; ++j)
                acc[i][j] = __builtin_amdgcn_smfmac_f32_16x16x64_bf16(a[i], b[j], acc[i][j], idx[i], 0, 0);
    };

    load_regs(0);
    store_regs(0);
    if (steps > 1) load_regs(1);
    __syncthreads();
    auto step = [&](int64_t s, int buf) {
        if (s + 1 < steps) store_regs(buf ^ 1);   // the buffer read one step ago: all waves are past that barrier
        if (s + 2 < steps) load_regs(s + 2);
        compute(buf);
        __syncthreads();                          // publishes step s + 1, retires step s
    };
    int64_t s = 0;
    for (; s + 1 < steps; s += 2) {   // two steps per trip: the buffer indices are constants
        step(s, 0);
        step(s + 1, 1);
    }
    if (s < steps) step(s, 0);

    // ---- adapter k-steps of 32 (Sec. 3.2): first operand = B_cat columns of the weight rows, second = T rows
    if (R > 0) {
        for (int rs = 0; rs < (Rpad >> 5); ++rs) {
            g4_u32x4 bq[kNI], tq[kMJ];
#pragma unroll
            for (int i = 0; i < kNI; ++i) {
                const int64_t n = n0 + 16 * kNI * wn + 16 * i + li;
                const int64_t nc = n < N ? n : N - 1;
                uint32_t e[8];
#pragma unroll
                for (int j = 0; j < 8; ++j) {  // rows past R meet the zero padding of T; clamp instead of predicating
                    const int r = rs * 32 + 8 * kb + j;
                    e[j] = (uint32_t)b_cat[(int64_t)(r < R ? r : R - 1) * N + nc];
                }
                bq[i] = g4_u32x4{e[0] | (e[1] << 16), e[2] | (e[3] << 16), e[4] | (e[5] << 16), e[6] | (e[7] << 16)};
            }
#pragma unroll
            for (int j = 0; j < kMJ; ++j) {
                const int64_t m = m0 + 16 * kMJ * wm + 16 * j + li;
                tq[j] = *reinterpret_cast<const g4_u32x4*>(t + (m < M ? m : M - 1) * Rpad + rs * 32 + 8 * kb);
            }
#pragma unroll
            for (int i = 0; i < kNI; ++i)
#pragma unroll
                for (int j = 0; j < kMJ; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, bq[i]), __builtin_bit_cast(bf16x8, tq[j]), acc[i][j], 0, 0, 0);
        }
    }

    // ---- store: lane holds token 16 j + lane % 16 of the wave's 64, outputs 16 i + 4 (lane / 16) + e (N % 4 == 0)
#pragma unroll
    for (int i = 0; i < kNI; ++i)
#pragma unroll
        for (int j = 0; j < kMJ; ++j) {
            const int64_t m = m0 + 16 * kMJ * wm + 16 * j + li;
            const int64_t nn = n0 + 16 * kNI * wn + 16 * i + 4 * kb;
            if (m < M && nn < N) {
                const uint32_t lo = (uint32_t)f32_to_bf16_rne(acc[i][j][0]) | ((uint32_t)f32_to_bf16_rne(acc[i][j][1]) << 16);
                const uint32_t hi = (uint32_t)f32_to_bf16_rne(acc[i][j][2]) | ((uint32_t)f32_to_bf16_rne(acc[i][j][3]) << 16);
                *reinterpret_cast<uint2*>(y + m * N + nn) = make_uint2(lo, hi);
            }
        }
}

template <int kWN, int kWM, int kNI, int kMJ>
static void launch_gemm_2of4_t(const LinearArgs& a, hipStream_t stream, const TimingEvents& ev) {
    constexpr int tile_n = 16 * kNI * kWN, tile_m = 16 * kMJ * kWM;
    const int m_tiles = (int)((a.M + tile_m - 1) / tile_m), n_tiles = (int)((a.N + tile_n - 1) / tile_n);
    const int n_groups = (n_tiles + kG4Xcds - 1) / kG4Xcds;
    const dim3 grid((unsigned)(n_groups * m_tiles * kG4Xcds));
    SALR_LAUNCH((gemm_2of4_kernel<kWN, kWM, kNI, kMJ>), grid, dim3(64 * kWN * kWM), stream, ev, a.x, a.M, a.K, a.N, a.bitmap,
                a.values, a.row_offsets, (const uint16_t*)a.t, a.b_cat, (int)a.R, (int)adapter_rank_padded(a.R), a.y, m_tiles,
                n_tiles);
}

hipError_t launch_gemm_2of4(const LinearArgs& a, hipStream_t stream, const TimingEvents& ev) {
    if (a.R > 0) launch_adapter_t(a, stream);   // T = X A_cat, bf16 [M, Rpad], at the start of the workspace
    // 256 x 256 tiles (8 waves, one workgroup per CU) where they fill the chip, else 128 x 128 (4 waves, two per CU);
    // 224 rows instead of 256 where that needs less time in whole rounds of the 256 CUs (a round costs its tile width)
    const int64_t m_tiles = (a.M + 255) / 256;
    const int64_t t256 = m_tiles * ((a.N + 255) / 256), t224 = m_tiles * ((a.N + 223) / 224);
    const int64_t cost256 = (t256 + 255) / 256 * 256, cost224 = (t224 + 255) / 256 * 224;
    if (t256 >= kGemm2of4BigTilesMin && cost224 < cost256) launch_gemm_2of4_t<2, 4, 7, 4>(a, stream, ev);
    else if (t256 >= kGemm2of4BigTilesMin) launch_gemm_2of4_t<2, 4, 8, 4>(a, stream, ev);
    else launch_gemm_2of4_t<2, 2, 4, 4>(a, stream, ev);
    return hipGetLastError();
}

}  // namespace salr
