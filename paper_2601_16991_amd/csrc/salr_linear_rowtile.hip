// Row-tiled streaming path of the SALR linear (paper Sec. 3.2 / 3.3) for layers with many rows and batches of up to
// 128 tokens: one pass over the compressed weight, like the small-batch kernel, but with the activations shared
// inside the workgroup instead of every wave fetching its own.
//
// A workgroup owns 128 consecutive rows of What and one slice of K; wave w owns rows 16 w .. 16 w + 15 of the tile
// for the whole slice.  The waves walk the slice in step, chunk by chunk (128 columns):
//   weights      as in the small-batch kernel: lane (n = lane%16, g = lane/16) takes byte g of each bitmap word of
//                row n; the row's packed values of the chunk (one contiguous piece) are fetched S chunks ahead with
//                16-byte loads, parked in the wave's LDS slot and expanded by the nibble rule of Sec. 3.3 straight
//                into the B operand of a 16x16x32 bf16 MFMA;
//   activations  the chunk's X tile [16 MT rows x 128 columns] is loaded ONCE per workgroup (one 16-byte vector per
//                thread and 32 rows) S chunks ahead into registers, written to LDS one chunk ahead, and read from
//                there by all eight waves as the A operand.  A wave of the small-batch kernel pulls all of X through the L2 for its 16 rows; here
//                128 rows share one copy, so a layer of N rows moves N / 128 copies of X instead of N / 16.
//                16-byte vectors of a row are stored at index v ^ (row % 16): the operand reads of a wave (16 rows,
//                the same four vectors each) then cover every LDS bank equally.
//   one barrier per chunk: it publishes the next X tile and retires the one just read.
//   adapters     slice 0 adds the rank steps after its loop: T = X A_cat (summed from the pre-kernel's split-K partials
//                and rounded to bf16 once) sits in LDS where the X tiles were; every wave multiplies it with the
//                B_cat columns of its own rows.
//   output       every wave owns its 16 output columns outright: bf16 to y, or fp32 to partial[slice] when K is split
//                (not enough 128-row tiles to fill the chip twice over), summed in slice order by the reducing pass.
// Tried and left out: 16 waves per workgroup walking the two halves of K side by side and adding them up through
// LDS, in place of a split of K over two workgroups per CU.  It saves the reducing launch, but the barrier then
// holds 16 waves in step, and on the 70B gate/up shape it was 10 to 18 % slower than the split.
#include <hip/hip_ext.h>

#include "salr_device.hpp"
#include "salr_internal.hpp"
#include "salr_linear_common.hpp"

namespace salr {

constexpr int kRtWaves = 8;
constexpr int kRtThreads = kRtWaves * 64;
constexpr int kRtChunkWords = 4;      // bitmap words per row per chunk
constexpr int kRtChunkCols = 128;
constexpr int kRtSlotDwords = 68;     // LDS per row per chunk: 17 vectors of 16 B (128 values + misalignment)

struct RowStage {
    uint4 bm;         // the chunk's 4 bitmap words of this lane's row
    uint4 vq[3];      // this lane's share of the first 12 vectors of the row's packed-value piece
    uint32_t off;     // element offset of the piece inside its first 16-byte vector
    uint32_t nv;      // vectors in the piece
    uint32_t vbase;   // index of its first vector in `values`
};

// native vector types (a 16-byte and an 8-byte one) that the compiler keeps in registers
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
template <bool kHalf> struct XUnitType { using type = u32x4; };
template <> struct XUnitType<true> { using type = u32x2; };

__device__ __forceinline__ uint32_t popc4(const uint4& q) { return __popc(q.x) + __popc(q.y) + __popc(q.z) + __popc(q.w); }

// MT m-tiles of 16 rows (M <= 16 MT), S chunks of packed values in flight per wave.  K % 128 == 0.  Up to 4 m-tiles
// the kernel keeps to 128 registers so that two workgroups share a CU and run through each other's barriers.
template <int MT, int S>
__global__ __launch_bounds__(kRtThreads, MT <= 4 ? 4 : 2) void linear_rowtile_kernel(
    const uint16_t* __restrict__ x, int M, int64_t K, int64_t N, const uint32_t* __restrict__ bitmap,
    const uint16_t* __restrict__ values, const uint32_t* __restrict__ row_offsets, const float* __restrict__ t_partial,
    const uint16_t* __restrict__ b_cat, int R, int Rpad, int ksplit, uint16_t* __restrict__ y, float* __restrict__ y_partial,
    const uint32_t* __restrict__ slice_table) {
    constexpr int kRows = 16 * MT;                                    // X rows of the tile (M padded)
    constexpr int kXsElems = kRows * kRtChunkCols;                    // bf16 elements of one X tile
    __shared__ __attribute__((aligned(16))) uint16_t xs[2 * kXsElems];
    __shared__ __attribute__((aligned(16))) uint32_t slots[kRtWaves * 16 * kRtSlotDwords + 8];
    __shared__ uint32_t lut_all[kRtWaves][kNibbleLutWords];  // one copy per wave: filled and used wave-synchronously

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int n = lane & 15;
    const int g = lane >> 4;
    const int z = blockIdx.y;
    const int64_t n0 = (int64_t)blockIdx.x * (16 * kRtWaves) + 16 * wave;
    const int64_t row = n0 + n;
    // Rows past N (last workgroup only) are computed as copies of row N-1 and dropped at the store: every wave
    // takes part in every barrier and no load needs a per-lane predicate.
    const int64_t row_c = row < N ? row : N - 1;
    const int64_t wpr = K >> 5;
    const int64_t chunks_total = wpr / kRtChunkWords;
    const int64_t c_begin = chunks_total * z / ksplit;          // the same for all waves of the workgroup
    const int64_t c_end = chunks_total * (z + 1) / ksplit;
    const uint32_t* brow = bitmap + row_c * wpr;
    uint32_t* lut = lut_all[wave];

    uint32_t cur = row_offsets[row_c];  // element index in `values` of the row's next value

    // Chunks past the slice read its last chunk and count as empty.  No load of the stream is conditional: the
    // compiler can then count the requests that are younger than the one a wave waits for, and leaves them in flight.
    auto load_bitmap_chunk = [&](int64_t c) -> uint4 {
        uint4 q = *reinterpret_cast<const uint4*>(brow + (c < c_end ? c : c_end - 1) * kRtChunkWords);
        const uint32_t keep = c < c_end ? 0xFFFFFFFFu : 0u;
        q.x &= keep; q.y &= keep; q.z &= keep; q.w &= keep;
        return q;
    };
    uint4 bmq[S];  // bitmap ring: the chunks that are issued next
#pragma unroll
    for (int i = 0; i < S; ++i) bmq[i] = load_bitmap_chunk(c_begin + i);

    // ---- X tile loader: every thread moves kXPer units of the tile (16 bytes; 8 bytes with one m-tile, where the
    // tile has only 256 vectors for 512 threads): unit idx = tid + kRtThreads j belongs to tile row idx / units-per-row
    using XUnit = typename XUnitType<MT == 1>::type;
    constexpr int kUnitElems = sizeof(XUnit) / 2;                 // bf16 elements per unit
    constexpr int kUnitsPerRow = kRtChunkCols / kUnitElems;
    constexpr int kXPer = kRows * kUnitsPerRow / kRtThreads;     // units per thread
    static_assert(kXPer * kRtThreads == kRows * kUnitsPerRow, "the threads cover the tile exactly");
    const uint16_t* xsrc[kXPer];
    int xdst[kXPer];
#pragma unroll
    for (int j = 0; j < kXPer; ++j) {
        const int idx = tid + kRtThreads * j;
        const int r = idx / kUnitsPerRow, e = (idx % kUnitsPerRow) * kUnitElems;   // row, first element of the unit
        const int v = e >> 3;                                                      // its 16-byte vector
        xsrc[j] = x + (int64_t)(r < M ? r : M - 1) * K + e;   // rows past M repeat row M-1; never stored
        xdst[j] = r * kRtChunkCols + 8 * (v ^ (r & 15)) + (e & 7);
    }
    // tile j of the slice waits in register set j % S from S chunks before it is read until it is written to LDS
    XUnit xring[S][kXPer];
    auto load_x = [&](XUnit (&xr)[kXPer], int64_t c) {
        const int64_t cc = c < c_end ? c : c_end - 1;   // past the slice: reload its last tile (its weights count as zero)
#pragma unroll
        for (int j = 0; j < kXPer; ++j) xr[j] = *reinterpret_cast<const XUnit*>(xsrc[j] + cc * kRtChunkCols);
    };
    auto store_x = [&](const XUnit (&xr)[kXPer], int buf) {
#pragma unroll
        for (int j = 0; j < kXPer; ++j) *reinterpret_cast<XUnit*>(&xs[buf * kXsElems + xdst[j]]) = xr[j];
    };
    if (c_begin < c_end) {
#pragma unroll
        for (int d = 0; d < S; ++d) load_x(xring[d], c_begin + d);
    }

    // B operand of the first rank step (Sec. 3.2): lane (n, g) holds B_cat[8 g + j][row], j = 0..7
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

    if (lane < 16) {
        uint32_t a, b;
        nibble_lut_entry(lane, a, b);
        lut[2 * lane] = a;
        lut[2 * lane + 1] = b;
    }
    __builtin_amdgcn_wave_barrier();

    // ---- nonzeros of the row left of the slice: from the layer's slice table when the call has one and the slice
    // starts where one of the table's eight does (K split 1, 2, 4 or 8 ways); else the 4 lanes of a row share the words,
    // 8 loads in flight each
    if (slice_table != nullptr && kSliceTableSlices % ksplit == 0) {   // the same for the whole grid
        cur = slice_table[((int64_t)row_c * kSliceTableSlices + z * (kSliceTableSlices / ksplit)) * 2];
    } else {
        uint32_t before = 0;
        for (int64_t c0 = 0; c0 < c_begin; c0 += 32) {
            uint4 q[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int64_t c = c0 + g + 4 * i;
                q[i] = *reinterpret_cast<const uint4*>(brow + (c < c_begin ? c : 0) * kRtChunkWords);
            }
#pragma unroll
            for (int i = 0; i < 8; ++i) before += (c0 + g + 4 * i < c_begin) ? popc4(q[i]) : 0u;
        }
        before += __shfl_xor(before, 16, 64);
        before += __shfl_xor(before, 32, 64);
        cur += before;
    }

    const uint4* values128 = reinterpret_cast<const uint4*>(values);
    uint32_t* slot = slots + (wave * 16 + n) * kRtSlotDwords;

    f32x4 acc[MT];
#pragma unroll
    for (int i = 0; i < MT; ++i) acc[i] = f32x4{0.f, 0.f, 0.f, 0.f};

    // Request the first 12 vectors of the chunk's piece.  Lanes whose vector lies past the piece re-read its last
    // vector (never used); an empty piece reads the start of X instead (always mapped).
    auto issue = [&](RowStage& st, const uint4 bm) {
        st.bm = bm;
        const uint32_t len = popc4(bm);
        st.off = cur & 7u;
        st.nv = len ? (st.off + len + 7u) >> 3 : 0u;
        st.vbase = cur >> 3;
        const uint32_t last = st.nv ? st.nv - 1u : 0u;
        const uint4* vb = st.nv ? values128 + st.vbase : reinterpret_cast<const uint4*>(x);
        cur += len;
#pragma unroll
        for (int i = 0; i < 3; ++i) {
            const uint32_t v = g + 4 * i;
            st.vq[i] = vb[v < last ? v : last];
        }
    };

    // Park the piece in LDS, expand the 4 byte masks of this lane, multiply with the X tile.
    auto consume = [&](const RowStage& st, const uint16_t* xt) {
#pragma unroll
        for (int i = 0; i < 3; ++i) *reinterpret_cast<uint4*>(slot + 4 * (g + 4 * i)) = st.vq[i];
        if (st.nv > 12u) {   // a piece of more than ~89 values (rare at the sparsities of the paper): fetch the rest now
#pragma unroll
            for (int i = 3; i < 5; ++i) {
                const uint32_t v = g + 4 * i;
                if (v < 17u) *reinterpret_cast<uint4*>(slot + 4 * v) = values128[st.vbase + (v < st.nv - 1u ? v : st.nv - 1u)];
            }
        }
        __builtin_amdgcn_wave_barrier();  // LDS executes a wave's accesses in order: writes above land first
        const uint32_t words[kRtChunkWords] = {st.bm.x, st.bm.y, st.bm.z, st.bm.w};
        uint32_t c_local = st.off;
#pragma unroll
        for (int s = 0; s < kRtChunkWords; ++s) {
            const uint32_t word = words[s];
            const uint32_t m8 = (word >> (8 * g)) & 0xFFu;
            const uint32_t cb = c_local + __popc(word & ((1u << (8 * g)) - 1u));
            const uint4 wq = expand_byte(slot, lut, cb, m8);
            c_local += __popc(word);
            const bf16x8 b = as_bf16x8(wq);
            const int vx = 8 * ((4 * s + g) ^ n);   // where vector 4 s + g of rows n, 16 + n, .. sits
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
                const uint4 aq = *reinterpret_cast<const uint4*>(xt + (16 * mt + n) * kRtChunkCols + vx);
                acc[mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(aq), b, acc[mt], 0, 0, 0);
            }
        }
        __builtin_amdgcn_wave_barrier();  // reads above are issued before the next chunk overwrites the slot
    };

    if (c_begin < c_end) {
        RowStage st[S];
#pragma unroll
        for (int i = 0; i < S; ++i) {
            issue(st[i], bmq[i]);
            bmq[i] = load_bitmap_chunk(c_begin + i + S);
        }
        store_x(xring[0], 0);
        load_x(xring[0], c_begin + S);
        __syncthreads();
        int buf = 0;
        int64_t c = c_begin;
        // Rounds of S chunks whose prefetches all lie inside the slice run without a condition: with no load of the
        // round conditional the compiler counts the requests younger than the one a wave waits for and leaves them in
        // flight (behind a branch it waits for everything).
        for (; c + 2 * S <= c_end; c += S) {
#pragma unroll
            for (int i = 0; i < S; ++i) {
                consume(st[i], xs + buf * kXsElems);
                issue(st[i], bmq[i]);
                bmq[i] = load_bitmap_chunk(c + i + 2 * S);
                // tile c + i + 1 into the buffer read one chunk ago (all waves are past that barrier)
                store_x(xring[(i + 1) % S], buf ^ 1);
                load_x(xring[(i + 1) % S], c + i + 1 + S);
                __syncthreads();    // publishes tile c + i + 1, retires tile c + i
                buf ^= 1;
            }
        }
        // the last rounds: nothing is requested past the slice
        for (; c < c_end; c += S) {
#pragma unroll
            for (int i = 0; i < S; ++i) {
                if (c + i < c_end) {   // the same for the whole workgroup
                    consume(st[i], xs + buf * kXsElems);
                    if (c + i + S < c_end) issue(st[i], bmq[i]);
                    if (c + i + 1 < c_end) store_x(xring[(i + 1) % S], buf ^ 1);
                    if (c + i + 1 + S < c_end) load_x(xring[(i + 1) % S], c + i + 1 + S);
                    __syncthreads();
                    buf ^= 1;
                }
            }
        }
    }

    // ---- adapter k-steps (Sec. 3.2): A operand = T rows from LDS, B operand = B_cat columns of this wave's rows
    if (adapters) {   // the same for the whole workgroup
        uint16_t* t_lds = xs;   // [M][Rpad]; the X tiles are retired (last barrier of the loop)
        const int groups = M * (Rpad >> 2);  // float4 groups of T
        for (int i = tid; i < groups; i += kRtThreads) {
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
                const uint4 aq = *reinterpret_cast<const uint4*>(&t_lds[(m < M ? m : M - 1) * Rpad + rs * 32 + 8 * g]);
                acc[mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(aq), as_bf16x8(bq), acc[mt], 0, 0, 0);
            }
        }
    }

    // ---- store: lane holds column `row`, rows 16 mt + 4 g + e
    if (row < N) {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int m = 16 * mt + 4 * g + e;
                if (m < M) {
                    if (ksplit == 1) y[(int64_t)m * N + row] = f32_to_bf16_rne(acc[mt][e]);
                    else y_partial[((int64_t)z * M + m) * N + row] = acc[mt][e];
                }
            }
    }
}

template <int MT, int S>
static void launch_rowtile_t(const LinearArgs& a, const float* t_partial, int ksplit, float* y_partial, hipStream_t stream,
                             const TimingEvents& ev) {
    const dim3 grid((unsigned)((a.N + 16 * kRtWaves - 1) / (16 * kRtWaves)), (unsigned)ksplit);
    SALR_LAUNCH((linear_rowtile_kernel<MT, S>), grid, dim3(kRtThreads), stream, ev, a.x, (int)a.M, a.K, a.N, a.bitmap, a.values,
                a.row_offsets, t_partial, a.b_cat, (int)a.R, (int)adapter_rank_padded(a.R), ksplit, a.y, y_partial, a.slice_table);
}

hipError_t launch_linear_rowtile(const LinearArgs& a, hipStream_t stream, const TimingEvents& ev) {
    const int ksplit = rowtile_ksplit(a.M, a.K, a.N);
    char* base = reinterpret_cast<char*>(a.t);
    const float* t_partial = reinterpret_cast<const float*>(base);
    if (a.R > 0) launch_adapter_partial(a, stream);   // split-K partials of T, summed inside the kernel
    float* y_partial = reinterpret_cast<float*>(base + rowtile_t_bytes(a.M, a.K, a.R));
    if (a.M <= 16) launch_rowtile_t<1, 2>(a, t_partial, ksplit, y_partial, stream, ev);
    else if (a.M <= 32) launch_rowtile_t<2, 2>(a, t_partial, ksplit, y_partial, stream, ev);
    else if (a.M <= 64) launch_rowtile_t<4, 2>(a, t_partial, ksplit, y_partial, stream, ev);
    else launch_rowtile_t<8, 2>(a, t_partial, ksplit, y_partial, stream, ev);
    if (ksplit > 1) launch_splitk_reduce(y_partial, a.M * a.N, ksplit, a.y, stream);
    return hipGetLastError();
}

}  // namespace salr
