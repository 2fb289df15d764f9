// The SALR linear on 2:4-masked weights (the N:M protocol of the paper's inference-throughput table, Sec. 4) for
// batches of up to 128 tokens, on the sparse matrix-core instruction of CDNA: no expansion of the bitmap at all.
//
// A weight whose every aligned group of four columns holds exactly two stored values is, as it sits in the SALR
// format (Sec. 3.3: bitmap + packed values in row-major order), already the operand that
// v_smfmac_f32_16x16x32_bf16 takes: lane (i, kb) of the sparse operand supplies the four stored values of columns
// 8 kb .. 8 kb + 7 of row i, two per group of four, together with one index byte (bits [1:0] and [3:2]: positions of
// the two values inside the first group, bits [5:4] and [7:6]: inside the second).  The four stored values of one
// bitmap byte are eight contiguous bytes of `values` at a position that follows from the row offset alone
// (row_offsets[n] + columns / 2), and the index byte follows from the bitmap byte by a few bit operations, so the
// kernel is the row-tiled streaming kernel without its decode stage: no LDS staging of values, no cursor, no lookup
// table, and a quarter of the vector instructions.
//
//   workgroup    128 consecutive weight rows and one slice of K, 8 waves of 16 rows, the waves walk the slice in step,
//                chunk by chunk (128 columns); the chunk's X tile is loaded once per workgroup into LDS (as in the
//                row-tiled kernel: registers S chunks ahead, LDS one chunk ahead, one barrier per chunk);
//   lane (n, g)  takes bitmap word g of the chunk for row n: one 4-byte load, and the word's 16 stored values: two
//                16-byte loads (the four lanes of a row read 128 contiguous bytes).  Instruction s of the chunk
//                multiplies byte s of every word: k-block g of that instruction is columns 32 g + 8 s .. + 7, and
//                the X operand is read from the tile to match (the order of the contraction index is free);
//   output       D[n][m]: a lane holds four consecutive outputs n of one token m (one 8-byte store);
//   adapters     as in the row-tiled kernel, with the operands of the dense MFMA swapped (B_cat columns as the first
//                operand, T as the second) so that they add into the same D[n][m].
//
// The precondition (every group 2-of-4) is the caller's: salr_bitmap_is_2of4 checks it once per layer.  Without it the
// result is unspecified, but every address stays inside the buffers: value offsets are clamped to the stored count.
#include <hip/hip_ext.h>

#include "salr_device.hpp"
#include "salr_internal.hpp"
#include "salr_linear_common.hpp"

namespace salr {

constexpr int kS4Waves = 8;
constexpr int kS4Threads = kS4Waves * 64;
constexpr int kS4ChunkCols = 128;

typedef uint32_t s4_u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t s4_u32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
template <bool kHalf> struct S4UnitType { using type = s4_u32x4; };
template <> struct S4UnitType<true> { using type = s4_u32x2; };

struct S4Stage {
    uint32_t word;       // bitmap word g of the chunk
    s4_u32x4 v0, v1;     // its 16 stored values
};

// Index bytes of the sparse MFMA for the four bytes of a bitmap word whose nibbles have two set bits each:
// per nibble, code = p0 | p1 << 2 with p0 < p1 the positions of the set bits.
__device__ __forceinline__ uint32_t index_codes_2of4(uint32_t w) {
    const uint32_t ones = 0x11111111u;
    const uint32_t b0 = w & ones, b1 = (w >> 1) & ones, b2 = (w >> 2) & ones, b3 = (w >> 3) & ones;
    const uint32_t n0 = b0 ^ ones, n1 = b1 ^ ones, n2 = b2 ^ ones;
    const uint32_t p0_lo = n0 & b1;        // p0 == 1
    const uint32_t p0_hi = n0 & n1;        // p0 == 2
    const uint32_t p1_lo = b3 | n2;        // p1 == 3 or p1 == 1
    const uint32_t p1_hi = b3 | b2;        // p1 == 3 or p1 == 2
    return p0_lo | (p0_hi << 1) | (p1_lo << 2) | (p1_hi << 3);
}

// MT m-tiles of 16 tokens (M <= 16 MT), S chunks in flight per wave.  K % 128 == 0.
template <int MT, int S>
__global__ __launch_bounds__(kS4Threads, MT <= 4 ? 4 : 2) void linear_2of4_kernel(
    const uint16_t* __restrict__ x, int M, int64_t K, int64_t N, const uint32_t* __restrict__ bitmap,
    const uint16_t* __restrict__ values, const uint32_t* __restrict__ row_offsets, const float* __restrict__ t_partial,
    const uint16_t* __restrict__ b_cat, int R, int Rpad, int ksplit, uint16_t* __restrict__ y, float* __restrict__ y_partial) {
    constexpr int kRows = 16 * MT;                       // X rows of the tile (M padded)
    constexpr int kXsElems = kRows * kS4ChunkCols;       // bf16 elements of one X tile
    __shared__ __attribute__((aligned(16))) uint16_t xs[2 * kXsElems];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int n = lane & 15;
    const int g = lane >> 4;
    const int z = blockIdx.y;
    const int64_t n0 = (int64_t)blockIdx.x * (16 * kS4Waves) + 16 * wave;
    // rows past N (last workgroup only) are computed as copies of row N-1 and dropped at the store
    const int64_t row_c = n0 + n < N ? n0 + n : N - 1;
    const int64_t wpr = K >> 5;
    const int64_t chunks_total = wpr >> 2;
    const int64_t c_begin = chunks_total * z / ksplit;          // the same for all waves of the workgroup
    const int64_t c_end = chunks_total * (z + 1) / ksplit;

    // where the stored values of (row, chunk c, word g) start: half the columns to the left of them
    const uint32_t nnz = row_offsets[N];
    const uint32_t e_max = nnz >= 16u ? nnz - 16u : 0u;
    const uint16_t* vsrc = nnz >= 16u ? values : x;   // (a weight this small cannot meet the precondition: read X instead)
    const uint32_t e_row = row_offsets[row_c] + 16u * (uint32_t)g;
    const uint32_t* bword = bitmap + row_c * wpr + g;

    // Chunks past the slice reload its last chunk and are not used.  No load of the stream is conditional.
    auto issue = [&](S4Stage& st, int64_t c) {
        const int64_t cc = c < c_end ? c : c_end - 1;
        st.word = bword[cc * 4];
        uint32_t e = e_row + 64u * (uint32_t)cc;
        e = (e < e_max ? e : e_max) & ~7u;   // in bounds and 16-byte aligned whatever the offsets are
        st.v0 = *reinterpret_cast<const s4_u32x4*>(vsrc + e);
        st.v1 = *reinterpret_cast<const s4_u32x4*>(vsrc + e + 8);
    };

    // ---- X tile loader (as in the row-tiled kernel): every thread moves kXPer units of the tile
    using XUnit = typename S4UnitType<MT == 1>::type;
    constexpr int kUnitElems = sizeof(XUnit) / 2;
    constexpr int kUnitsPerRow = kS4ChunkCols / kUnitElems;
    constexpr int kXPer = kRows * kUnitsPerRow / kS4Threads;
    static_assert(kXPer * kS4Threads == kRows * kUnitsPerRow, "the threads cover the tile exactly");
    const uint16_t* xsrc[kXPer];
    int xdst[kXPer];
#pragma unroll
    for (int j = 0; j < kXPer; ++j) {
        const int idx = tid + kS4Threads * j;
        const int r = idx / kUnitsPerRow, e = (idx % kUnitsPerRow) * kUnitElems;
        const int v = e >> 3;
        xsrc[j] = x + (int64_t)(r < M ? r : M - 1) * K + e;   // rows past M repeat row M-1; never stored
        xdst[j] = r * kS4ChunkCols + 8 * (v ^ (r & 15)) + (e & 7);
    }
    XUnit xring[S][kXPer];
    auto load_x = [&](XUnit (&xr)[kXPer], int64_t c) {
        const int64_t cc = c < c_end ? c : c_end - 1;
#pragma unroll
        for (int j = 0; j < kXPer; ++j) xr[j] = *reinterpret_cast<const XUnit*>(xsrc[j] + cc * kS4ChunkCols);
    };
    auto store_x = [&](const XUnit (&xr)[kXPer], int buf) {
#pragma unroll
        for (int j = 0; j < kXPer; ++j) *reinterpret_cast<XUnit*>(&xs[buf * kXsElems + xdst[j]]) = xr[j];
    };

    // first operand of the first rank step (Sec. 3.2): lane (n, g) holds B_cat[8 g + j][row], j = 0..7
    const bool adapters = R > 0 && z == 0;
    auto load_b_cat = [&](int rs) -> uint4 {
        const int r0 = rs * 32 + 8 * g;
        uint32_t e[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {  // rows past R meet the zero padding of T; clamp instead of predicating
            const int r = r0 + j < R ? r0 + j : R - 1;
            e[j] = (uint32_t)b_cat[(int64_t)r * N + row_c];
        }
        return make_uint4(e[0] | (e[1] << 16), e[2] | (e[3] << 16), e[4] | (e[5] << 16), e[6] | (e[7] << 16));
    };
    uint4 bq0 = make_uint4(0, 0, 0, 0);
    if (adapters) bq0 = load_b_cat(0);

    f32x4 acc[MT];
#pragma unroll
    for (int i = 0; i < MT; ++i) acc[i] = f32x4{0.f, 0.f, 0.f, 0.f};

    // the chunk's four sparse MFMAs per m-tile: instruction s takes byte s of this lane's word
    auto consume = [&](const S4Stage& st, const uint16_t* xt) {
        const int idx = (int)index_codes_2of4(st.word);
        const uint32_t vals[8] = {st.v0.x, st.v0.y, st.v0.z, st.v0.w, st.v1.x, st.v1.y, st.v1.z, st.v1.w};
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            const uint16_t* xrow = xt + (16 * mt + n) * kS4ChunkCols;
            uint4 xq[4];
#pragma unroll
            for (int s = 0; s < 4; ++s) xq[s] = *reinterpret_cast<const uint4*>(xrow + 8 * ((4 * g + s) ^ n));
            const bf16x4 a0 = __builtin_bit_cast(bf16x4, make_uint2(vals[0], vals[1]));
            const bf16x4 a1 = __builtin_bit_cast(bf16x4, make_uint2(vals[2], vals[3]));
            const bf16x4 a2 = __builtin_bit_cast(bf16x4, make_uint2(vals[4], vals[5]));
            const bf16x4 a3 = __builtin_bit_cast(bf16x4, make_uint2(vals[6], vals[7]));
            acc[mt] = __builtin_amdgcn_smfmac_f32_16x16x32_bf16(a0, as_bf16x8(xq[0]), acc[mt], idx, 0, 0);
            acc[mt] = __builtin_amdgcn_smfmac_f32_16x16x32_bf16(a1, as_bf16x8(xq[1]), acc[mt], idx, 0, 1);
            acc[mt] = __builtin_amdgcn_smfmac_f32_16x16x32_bf16(a2, as_bf16x8(xq[2]), acc[mt], idx, 0, 2);
            acc[mt] = __builtin_amdgcn_smfmac_f32_16x16x32_bf16(a3, as_bf16x8(xq[3]), acc[mt], idx, 0, 3);
        }
    };

    if (c_begin < c_end) {
        S4Stage st[S];
#pragma unroll
        for (int d = 0; d < S; ++d) {
            load_x(xring[d], c_begin + d);
            issue(st[d], c_begin + d);
        }
        store_x(xring[0], 0);
        load_x(xring[0], c_begin + S);
        __syncthreads();
        int buf = 0;
        int64_t c = c_begin;
        // rounds whose prefetches all lie inside the slice run without a condition (the compiler then leaves the
        // younger requests in flight when it waits for one), the last rounds with them
        for (; c + 2 * S <= c_end; c += S) {
#pragma unroll
            for (int i = 0; i < S; ++i) {
                consume(st[i], xs + buf * kXsElems);
                issue(st[i], c + i + S);
                store_x(xring[(i + 1) % S], buf ^ 1);   // tile c + i + 1 into the buffer read one chunk ago
                load_x(xring[(i + 1) % S], c + i + 1 + S);
                __syncthreads();                        // publishes tile c + i + 1, retires tile c + i
                buf ^= 1;
            }
        }
        for (; c < c_end; c += S) {
#pragma unroll
            for (int i = 0; i < S; ++i) {
                if (c + i < c_end) {   // the same for the whole workgroup
                    consume(st[i], xs + buf * kXsElems);
                    if (c + i + S < c_end) issue(st[i], c + i + S);
                    if (c + i + 1 < c_end) store_x(xring[(i + 1) % S], buf ^ 1);
                    if (c + i + 1 + S < c_end) load_x(xring[(i + 1) % S], c + i + 1 + S);
                    __syncthreads();
                    buf ^= 1;
                }
            }
        }
    }

    // ---- adapter k-steps (Sec. 3.2): first operand = B_cat columns of this wave's rows, second = T rows from LDS
    if (adapters) {   // the same for the whole workgroup
        uint16_t* t_lds = xs;   // [M][Rpad]; the X tiles are retired (last barrier of the loop)
        const int groups = M * (Rpad >> 2);  // float4 groups of T
        for (int i = tid; i < groups; i += kS4Threads) {
            float4 sum = make_float4(0.f, 0.f, 0.f, 0.f);
            const float4* p = reinterpret_cast<const float4*>(t_partial) + i;
#pragma unroll
            for (int sl = 0; sl < kStreamTSlices; ++sl) {
                const float4 v = p[(int64_t)sl * groups];
                sum.x += v.x; sum.y += v.y; sum.z += v.z; sum.w += v.w;
            }
            uint2 o;
            o.x = (uint32_t)f32_to_bf16_rne(sum.x) | ((uint32_t)f32_to_bf16_rne(sum.y) << 16);
            o.y = (uint32_t)f32_to_bf16_rne(sum.z) | ((uint32_t)f32_to_bf16_rne(sum.w) << 16);
            *reinterpret_cast<uint2*>(&t_lds[4 * i]) = o;
        }
        __syncthreads();
        for (int rs = 0; rs < (Rpad >> 5); ++rs) {
            const uint4 bq = rs == 0 ? bq0 : load_b_cat(rs);
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
                const int m = 16 * mt + n;
                const uint4 tq = *reinterpret_cast<const uint4*>(&t_lds[(m < M ? m : M - 1) * Rpad + rs * 32 + 8 * g]);
                acc[mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(bq), as_bf16x8(tq), acc[mt], 0, 0, 0);
            }
        }
    }

    // ---- store: lane holds token 16 mt + lane % 16, outputs n0 + 4 (lane / 16) + e
    const int64_t nn = n0 + 4 * g;
    const bool vec_store = (N & 3) == 0;   // then a lane's four outputs are all inside or all outside, and aligned
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        const int m = 16 * mt + n;
        if (m >= M) continue;
        if (ksplit == 1) {
            uint16_t* dst = y + (int64_t)m * N + nn;
            const uint16_t o0 = f32_to_bf16_rne(acc[mt][0]), o1 = f32_to_bf16_rne(acc[mt][1]);
            const uint16_t o2 = f32_to_bf16_rne(acc[mt][2]), o3 = f32_to_bf16_rne(acc[mt][3]);
            if (vec_store) {
                if (nn < N) *reinterpret_cast<uint2*>(dst) = make_uint2((uint32_t)o0 | ((uint32_t)o1 << 16), (uint32_t)o2 | ((uint32_t)o3 << 16));
            } else {
                if (nn + 0 < N) dst[0] = o0;
                if (nn + 1 < N) dst[1] = o1;
                if (nn + 2 < N) dst[2] = o2;
                if (nn + 3 < N) dst[3] = o3;
            }
        } else if (nn < N) {   // K is split only where N % 4 == 0
            *reinterpret_cast<float4*>(y_partial + ((int64_t)z * M + m) * N + nn) =
                make_float4(acc[mt][0], acc[mt][1], acc[mt][2], acc[mt][3]);
        }
    }
}

// ---------------------------------------------------------------------------------------------------
// Up to 32 tokens: the shape of the small-batch streaming kernel.  A workgroup owns 16 weight rows for the whole
// contraction, its 8 waves split K into contiguous slices and meet only in the final sum through LDS, so there is
// no barrier in the stream, no split of K over workgroups and no reducing launch.  Per chunk a lane (n, g) loads
// bitmap word g and its 16 stored values of row n (4 + 32 bytes) and, as lane (m, g) of the dense operand, the 32
// activations X[m][32 g .. 32 g + 31] of the chunk (64 contiguous bytes, from the L2); S chunks are in flight.
// Wave w applies rank step w of the adapters (T summed from the pre-kernel's partials into LDS).
// ---------------------------------------------------------------------------------------------------
template <int MT>
struct S4WaveStage {
    uint32_t word;
    s4_u32x4 v0, v1;
    s4_u32x4 xq[4 * MT];   // xq[4 mt + s]: X[16 mt + m][32 g + 8 s .. + 7] of the chunk
};

template <int MT, int S>
__global__ __launch_bounds__(kS4Threads, 4) void linear_2of4_stream_kernel(
    const uint16_t* __restrict__ x, int M, int64_t K, int64_t N, const uint32_t* __restrict__ bitmap,
    const uint16_t* __restrict__ values, const uint32_t* __restrict__ row_offsets, const float* __restrict__ t_partial,
    const uint16_t* __restrict__ b_cat, int R, int Rpad, uint16_t* __restrict__ y) {
    constexpr int kTRows = 16 * MT;
    __shared__ __attribute__((aligned(16))) float red[kS4Waves * MT * 256];
    __shared__ __attribute__((aligned(16))) uint16_t t_lds[kTRows * kMaxRankPadded];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int n = lane & 15;
    const int g = lane >> 4;
    const int64_t n0 = (int64_t)blockIdx.x * 16;
    const int64_t row_c = n0 + n < N ? n0 + n : N - 1;   // rows past N are copies of row N-1, dropped at the store
    const int64_t wpr = K >> 5;
    const int64_t chunks_total = wpr >> 2;
    const int64_t c_begin = chunks_total * wave / kS4Waves;
    const int64_t c_end = chunks_total * (wave + 1) / kS4Waves;

    const uint32_t nnz = row_offsets[N];
    const uint32_t e_max = nnz >= 16u ? nnz - 16u : 0u;
    const uint16_t* vsrc = nnz >= 16u ? values : x;
    const uint32_t e_row = row_offsets[row_c] + 16u * (uint32_t)g;
    const uint32_t* bword = bitmap + row_c * wpr + g;
    const uint16_t* xrow[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        const int m = 16 * mt + n;
        xrow[mt] = x + (int64_t)(m < M ? m : M - 1) * K + 32 * g;   // tokens past M repeat token M-1; never stored
    }

    auto issue = [&](S4WaveStage<MT>& st, int64_t c) {
        const int64_t cc = c < chunks_total ? c : chunks_total - 1;   // past the row: any chunk will do, it is not used
        st.word = bword[cc * 4];
        uint32_t e = e_row + 64u * (uint32_t)cc;
        e = (e < e_max ? e : e_max) & ~7u;   // in bounds and 16-byte aligned whatever the offsets are
        st.v0 = *reinterpret_cast<const s4_u32x4*>(vsrc + e);
        st.v1 = *reinterpret_cast<const s4_u32x4*>(vsrc + e + 8);
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int s = 0; s < 4; ++s)
                st.xq[4 * mt + s] = *reinterpret_cast<const s4_u32x4*>(xrow[mt] + cc * kS4ChunkCols + 8 * s);
    };

    // first operand of this wave's rank step (Sec. 3.2): lane (n, g) holds B_cat[32 wave + 8 g + j][row], j = 0..7
    const bool has_rank_step = R > 0 && wave * 32 < Rpad;
    uint4 bq = make_uint4(0, 0, 0, 0);
    if (has_rank_step) {
        const int r0 = wave * 32 + 8 * g;
        uint32_t e[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {  // rows past R meet the zero padding of T; clamp instead of predicating
            const int r = r0 + j < R ? r0 + j : R - 1;
            e[j] = (uint32_t)b_cat[(int64_t)r * N + row_c];
        }
        bq = make_uint4(e[0] | (e[1] << 16), e[2] | (e[3] << 16), e[4] | (e[5] << 16), e[6] | (e[7] << 16));
    }

    // T = sum of the pre-kernel's split-K partials, rounded once to bf16, kept in LDS
    if (R > 0) {
        const int groups = M * (Rpad >> 2);  // float4 groups of T
        for (int i = tid; i < groups; i += kS4Threads) {
            float4 sum = make_float4(0.f, 0.f, 0.f, 0.f);
            const float4* p = reinterpret_cast<const float4*>(t_partial) + i;
#pragma unroll
            for (int sl = 0; sl < kStreamTSlices; ++sl) {
                const float4 v = p[(int64_t)sl * groups];
                sum.x += v.x; sum.y += v.y; sum.z += v.z; sum.w += v.w;
            }
            const int m = i / (Rpad >> 2), r4 = i % (Rpad >> 2);
            uint2 o;
            o.x = (uint32_t)f32_to_bf16_rne(sum.x) | ((uint32_t)f32_to_bf16_rne(sum.y) << 16);
            o.y = (uint32_t)f32_to_bf16_rne(sum.z) | ((uint32_t)f32_to_bf16_rne(sum.w) << 16);
            *reinterpret_cast<uint2*>(&t_lds[m * kMaxRankPadded + 4 * r4]) = o;
        }
    }

    f32x4 acc[MT];
#pragma unroll
    for (int i = 0; i < MT; ++i) acc[i] = f32x4{0.f, 0.f, 0.f, 0.f};

    auto consume = [&](const S4WaveStage<MT>& st) {
        const int idx = (int)index_codes_2of4(st.word);
        const bf16x4 a0 = __builtin_bit_cast(bf16x4, make_uint2(st.v0.x, st.v0.y));
        const bf16x4 a1 = __builtin_bit_cast(bf16x4, make_uint2(st.v0.z, st.v0.w));
        const bf16x4 a2 = __builtin_bit_cast(bf16x4, make_uint2(st.v1.x, st.v1.y));
        const bf16x4 a3 = __builtin_bit_cast(bf16x4, make_uint2(st.v1.z, st.v1.w));
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            acc[mt] = __builtin_amdgcn_smfmac_f32_16x16x32_bf16(a0, __builtin_bit_cast(bf16x8, st.xq[4 * mt + 0]), acc[mt], idx, 0, 0);
            acc[mt] = __builtin_amdgcn_smfmac_f32_16x16x32_bf16(a1, __builtin_bit_cast(bf16x8, st.xq[4 * mt + 1]), acc[mt], idx, 0, 1);
            acc[mt] = __builtin_amdgcn_smfmac_f32_16x16x32_bf16(a2, __builtin_bit_cast(bf16x8, st.xq[4 * mt + 2]), acc[mt], idx, 0, 2);
            acc[mt] = __builtin_amdgcn_smfmac_f32_16x16x32_bf16(a3, __builtin_bit_cast(bf16x8, st.xq[4 * mt + 3]), acc[mt], idx, 0, 3);
        }
    };

    if (c_begin < c_end) {
        S4WaveStage<MT> st[S];
#pragma unroll
        for (int i = 0; i < S; ++i) issue(st[i], c_begin + i);   // (chunks past the slice are loaded and dropped)
        int64_t c = c_begin;
        for (; c + 2 * S <= c_end; c += S) {   // rounds without a condition, see the row-tiled kernel below
#pragma unroll
            for (int i = 0; i < S; ++i) {
                consume(st[i]);
                issue(st[i], c + i + S);
            }
        }
        for (; c < c_end; c += S) {
#pragma unroll
            for (int i = 0; i < S; ++i) {
                if (c + i < c_end) consume(st[i]);   // wave-uniform conditions
                if (c + i + S < c_end) issue(st[i], c + i + S);
            }
        }
    }

    __syncthreads();  // T in LDS is complete

    // ---- adapter k-step of this wave (Sec. 3.2): first operand = B_cat columns, second = T rows from LDS
    if (has_rank_step) {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            const int m = 16 * mt + n;
            const uint4 tq = *reinterpret_cast<const uint4*>(&t_lds[(m < M ? m : M - 1) * kMaxRankPadded + wave * 32 + 8 * g]);
            acc[mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(bq), as_bf16x8(tq), acc[mt], 0, 0, 0);
        }
    }

    // ---- add up the waves' accumulators and store: a lane of the sum holds token 16 mt + l % 16, outputs 4 (l / 16) + e
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int e = 0; e < 4; ++e) red[((wave * MT + mt) * 4 + e) * 64 + lane] = acc[mt][e];
    __syncthreads();
    for (int idx = tid; idx < MT * 256; idx += kS4Threads) {
        const int l = idx & 63, e = (idx >> 6) & 3, mt = idx >> 8;
        float s = 0.f;
#pragma unroll
        for (int w = 0; w < kS4Waves; ++w) s += red[((w * MT + mt) * 4 + e) * 64 + l];
        const int m = 16 * mt + (l & 15);
        const int64_t nn = n0 + 4 * (l >> 4) + e;
        if (m < M && nn < N) y[(int64_t)m * N + nn] = f32_to_bf16_rne(s);
    }
}

template <int MT, int S>
static void launch_2of4_stream_t(const LinearArgs& a, const float* t_partial, hipStream_t stream, const TimingEvents& ev) {
    const dim3 grid((unsigned)((a.N + 15) / 16));
    SALR_LAUNCH((linear_2of4_stream_kernel<MT, S>), grid, dim3(kS4Threads), stream, ev, a.x, (int)a.M, a.K, a.N, a.bitmap,
                a.values, a.row_offsets, t_partial, a.b_cat, (int)a.R, (int)adapter_rank_padded(a.R), a.y);
}

template <int MT, int S>
static void launch_2of4_t(const LinearArgs& a, const float* t_partial, int ksplit, float* y_partial, hipStream_t stream,
                          const TimingEvents& ev) {
    const dim3 grid((unsigned)((a.N + 16 * kS4Waves - 1) / (16 * kS4Waves)), (unsigned)ksplit);
    SALR_LAUNCH((linear_2of4_kernel<MT, S>), grid, dim3(kS4Threads), stream, ev, a.x, (int)a.M, a.K, a.N, a.bitmap, a.values,
                a.row_offsets, t_partial, a.b_cat, (int)a.R, (int)adapter_rank_padded(a.R), ksplit, a.y, y_partial);
}

hipError_t launch_linear_2of4(const LinearArgs& a, hipStream_t stream, const TimingEvents& ev) {
    const int ksplit = rowtile_ksplit(a.M, a.K, a.N);
    char* base = reinterpret_cast<char*>(a.t);
    const float* t_partial = reinterpret_cast<const float*>(base);
    if (a.R > 0) launch_adapter_partial(a, stream);   // split-K partials of T, summed inside the kernel
    float* y_partial = reinterpret_cast<float*>(base + rowtile_t_bytes(a.M, a.K, a.R));
    // Up to 16 tokens the barrier-free kernel is ahead where the call is short (layers of up to 2^25 elements: no
    // reducing launch, no split of K) and, on any layer, up to 4 tokens (little X to pull through the L2 per workgroup);
    // measured on the Llama-3 shapes.
    if (a.M <= 16 && (a.M <= 4 || a.N * a.K <= (int64_t(1) << 25))) {
        launch_2of4_stream_t<1, 4>(a, t_partial, stream, ev);
        return hipGetLastError();
    }
    if (a.M <= 16) launch_2of4_t<1, 4>(a, t_partial, ksplit, y_partial, stream, ev);
    else if (a.M <= 32) launch_2of4_t<2, 4>(a, t_partial, ksplit, y_partial, stream, ev);
    else if (a.M <= 64) launch_2of4_t<4, 2>(a, t_partial, ksplit, y_partial, stream, ev);
    else launch_2of4_t<8, 2>(a, t_partial, ksplit, y_partial, stream, ev);
    if (ksplit > 1) launch_splitk_reduce(y_partial, a.M * a.N, ksplit, a.y, stream);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------------
// flag[0] = 1 iff every aligned group of four columns of the bitmap has exactly two set bits.
// ---------------------------------------------------------------------------------------------------
__global__ void flag_set_kernel(uint32_t* flag, uint32_t value) {
    if (threadIdx.x == 0 && blockIdx.x == 0) flag[0] = value;
}

__global__ __launch_bounds__(256) void check_2of4_kernel(const uint32_t* __restrict__ bitmap, int64_t words,
                                                         uint32_t* __restrict__ flag) {
    bool bad = false;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < words; i += (int64_t)gridDim.x * 256) {
        const uint32_t w = bitmap[i];
        const uint32_t pairs = (w & 0x55555555u) + ((w >> 1) & 0x55555555u);
        const uint32_t nibbles = (pairs & 0x33333333u) + ((pairs >> 2) & 0x33333333u);
        bad |= nibbles != 0x22222222u;
    }
    if (bad) flag[0] = 0u;   // every writer stores the same value
}

hipError_t launch_check_2of4(const uint32_t* bitmap, int64_t rows, int64_t cols, uint32_t* flag, hipStream_t stream) {
    const int64_t words = rows * (cols / 32);
    const bool possible = rows > 0 && cols > 0 && cols % 32 == 0;
    hipLaunchKernelGGL(flag_set_kernel, dim3(1), dim3(64), 0, stream, flag, possible ? 1u : 0u);
    if (possible) {
        const int64_t blocks = (words + 255) / 256;
        hipLaunchKernelGGL(check_2of4_kernel, dim3((unsigned)(blocks < 4096 ? blocks : 4096)), dim3(256), 0, stream, bitmap, words,
                           flag);
    }
    return hipGetLastError();
}

}  // namespace salr
