// Small-batch (M <= 64) path of the SALR linear: one pass over the compressed weight, HBM-bound.
//
// A workgroup owns 16 consecutive rows of What (= 16 outputs n) for the whole contraction; its NW
// waves split K into contiguous slices and run independently of each other until the final reduction:
//
//   per wave, per chunk of 128 columns (4 bitmap words per row):
//     decode stage  lane (n = lane%16, g = lane/16) takes byte g of each word of row n.  The packed
//                   values of the chunk (one contiguous piece per row) are fetched with 16-byte loads
//                   two chunks ahead, parked in LDS, and expanded by the nibble rule of Sec. 3.3
//                   straight into the B operand of a 16x16x32 bf16 MFMA -- the 8 columns of one byte
//                   mask are exactly the 8 k-values one lane feeds to that instruction;
//     MFMA stage    X rows come from global memory (L2-resident, shared by all workgroups) as the A
//                   operand; fp32 accumulators [16 m x 16 n] per m-tile.
//   adapters       the rank dimension is appended as extra k-steps: A operand = T (summed from the
//                   split-K partials of the adapter pre-kernel), B operand = B_cat columns (Sec. 3.2).
//   epilogue       accumulators of the NW waves are summed through LDS, rounded to bf16, stored.
//
// The row cursor into `values` at the start of a wave's slice is the row offset plus the popcount of
// the row's earlier bitmap words; a short pre-pass over the workgroup's bitmap rows computes it.
#include <hip/hip_ext.h>

#include "salr_device.hpp"
#include "salr_internal.hpp"
#include "salr_linear_common.hpp"

namespace salr {

constexpr int kStreamRows = 16;         // weight rows per workgroup
constexpr int kChunkWords = 4;          // bitmap words per row per chunk (128 columns)
constexpr int kSlotDwords = 68;         // LDS per row per chunk: 17 vectors of 16 B (128 values + misalignment)
constexpr int kMaxVecPerLane = 5;       // 17 vectors over the 4 lanes of a row

template <int MT, int NV>
struct StreamStage {
    uint4 bm;                           // the chunk's 4 bitmap words of this lane's row
    uint4 vq[NV];                       // this lane's share of the row's packed-value piece
    uint4 xq[kChunkWords * MT];         // X operands of the chunk's 4 k-steps
    uint32_t off;                       // element offset of the piece inside its first 16-byte vector
    uint32_t nv;                        // vectors in the piece
};

// MT m-tiles of 16 rows, NW waves per workgroup, S chunks in flight per wave.
// kOwnPrefix: every wave popcounts the bitmap words left of its slice itself (short rows), so the
// workgroup needs no barrier before the stream starts; otherwise the waves exchange slice counts.
// kTable: the cursors come ready-made from the layer's slice table (salr_build_slice_table: for every row and each of
// the 8 wave slices the index of the slice's first value and the most nonzeros any chunk of it holds): one 8-byte
// request in place of the row offset, the rest of the slice's bitmap and the words left of it, and no barrier.
template <int MT, int NW, int S, bool kVecBitmap, bool kOwnPrefix, bool kTable = false>
__global__ __launch_bounds__(NW * 64, (S == 2 && MT == 1) ? 4 : 1) void linear_stream_kernel(
    const uint16_t* __restrict__ x, int M, int64_t K, int64_t N, const uint32_t* __restrict__ bitmap,
    const uint16_t* __restrict__ values, const uint32_t* __restrict__ row_offsets,
    const float* __restrict__ t_partial, const uint16_t* __restrict__ b_cat, int R, int Rpad,
    uint16_t* __restrict__ y, const uint32_t* __restrict__ slice_table) {
    static_assert(!kTable || NW == kSliceTableSlices, "the table holds one entry per wave slice");
    constexpr int kThreads = NW * 64;
    constexpr int kStageDwords = NW * kStreamRows * kSlotDwords + 8;
    constexpr int kRedFloats = NW * MT * 256;
    constexpr int kSmemDwords = kStageDwords > kRedFloats ? kStageDwords : kRedFloats;
    constexpr int kTRows = 16 * MT;
    __shared__ __attribute__((aligned(16))) uint32_t smem[kSmemDwords];
    __shared__ __attribute__((aligned(16))) uint16_t t_lds[kTRows * kMaxRankPadded];  // T = X * A_cat, bf16
    __shared__ uint32_t lut_all[NW][kNibbleLutWords];  // one copy per wave: filled and used wave-synchronously
    __shared__ uint32_t slice_count[NW][kStreamRows];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // scalar: conditions on it branch uniformly
    const int n = lane & 15;
    const int g = lane >> 4;
    const int64_t n0 = (int64_t)blockIdx.x * kStreamRows;
    const int64_t row = n0 + n;
    const bool row_ok = row < N;
    const int64_t wpr = K >> 5;
    const int64_t chunks_total = (wpr + kChunkWords - 1) / kChunkWords;
    const int64_t c_begin = chunks_total * wave / NW;
    const int64_t c_end = chunks_total * (wave + 1) / NW;
    uint32_t* lut = lut_all[wave];
    // Rows past N (last workgroup only) are computed as copies of row N-1 and dropped at the store,
    // so no load below needs a per-lane predicate: every address is clamped into range instead.
    const int64_t row_c = row_ok ? row : N - 1;
    const uint32_t* brow = bitmap + row_c * wpr;

    // first requests of the kernel: row offset, bitmap of the first S chunks, adapter operands
    uint32_t cur;           // element index in `values` of the row's next value
    uint32_t longest = 0;   // most nonzeros any 128-column chunk of the slice holds (per lane)
    if constexpr (kTable) {
        const uint2 e = *reinterpret_cast<const uint2*>(slice_table + ((int64_t)row_c * kSliceTableSlices + wave) * 2);
        cur = e.x;
        longest = e.y;
    } else {
        cur = row_offsets[row_c];
    }

    auto load_bitmap_chunk = [&](int64_t c) -> uint4 {
        uint4 q = make_uint4(0, 0, 0, 0);
        if (c < c_end) {  // wave-uniform when c is
            if constexpr (kVecBitmap) {
                q = *reinterpret_cast<const uint4*>(brow + c * kChunkWords);
            } else {
                const int64_t w0 = c * kChunkWords;
                q.x = brow[w0];
                if (w0 + 1 < wpr) q.y = brow[w0 + 1];
                if (w0 + 2 < wpr) q.z = brow[w0 + 2];
                if (w0 + 3 < wpr) q.w = brow[w0 + 3];
            }
        }
        return q;
    };

    uint4 bmq[S];  // bitmap ring: chunks [c, c + S) ahead of the stages
#pragma unroll
    for (int i = 0; i < S; ++i) bmq[i] = load_bitmap_chunk(c_begin + i);

    // B operand of this wave's rank step (Sec. 3.2): lane (n, g) holds B_cat[32*wave + 8g + j][row], j = 0..7
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
        for (int i = tid; i < groups; i += kThreads) {
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

    if (lane < 16) {
        uint32_t a, b;
        nibble_lut_entry(lane, a, b);
        lut[2 * lane] = a;
        lut[2 * lane + 1] = b;
    }
    __builtin_amdgcn_wave_barrier();

    // ---- pre-pass: nonzeros of this wave's slice per row.  The first S chunks are already in
    // registers (all 4 lanes of a row hold them); the 4 lanes split the rest.
    if constexpr (!kTable) {
        uint32_t head = 0, tail = 0;
#pragma unroll
        for (int i = 0; i < S; ++i) {
            const uint32_t len = __popc(bmq[i].x) + __popc(bmq[i].y) + __popc(bmq[i].z) + __popc(bmq[i].w);
            head += len;
            longest = len > longest ? len : longest;
        }
        for (int64_t c = c_begin + S + g; c < c_end; c += 4) {
            const uint4 q = load_bitmap_chunk(c);
            const uint32_t len = __popc(q.x) + __popc(q.y) + __popc(q.z) + __popc(q.w);
            tail += len;
            longest = len > longest ? len : longest;
        }
        if constexpr (kOwnPrefix) {
            // nonzeros left of the slice: at most 7 chunks per lane (rows of <= 32 chunks), all in flight at once
            uint32_t before = 0;
            uint4 left[7];  // no branches: chunks past the slice start re-read chunk 0 and are dropped
#pragma unroll
            for (int i = 0; i < 7; ++i) {
                const int64_t c = g + 4 * i;
                left[i] = *reinterpret_cast<const uint4*>(brow + (c < c_begin ? c : 0) * kChunkWords);
            }
#pragma unroll
            for (int i = 0; i < 7; ++i) {
                const uint32_t cnt = __popc(left[i].x) + __popc(left[i].y) + __popc(left[i].z) + __popc(left[i].w);
                before += (g + 4 * i < c_begin) ? cnt : 0u;
            }
            before += __shfl_xor(before, 16, 64);
            before += __shfl_xor(before, 32, 64);
            cur += before;
        } else {
            tail += __shfl_xor(tail, 16, 64);
            tail += __shfl_xor(tail, 32, 64);
            if (g == 0) slice_count[wave][n] = head + tail;
        }
    }
    if constexpr (!kOwnPrefix && !kTable) {
        __syncthreads();
        for (int w = 0; w < wave; ++w) cur += slice_count[w][n];
    }

    const uint4* values128 = reinterpret_cast<const uint4*>(values);
    uint32_t* slot = smem + (wave * kStreamRows + n) * kSlotDwords;

    f32x4 acc[MT];
#pragma unroll
    for (int i = 0; i < MT; ++i) acc[i] = f32x4{0.f, 0.f, 0.f, 0.f};

    // A piece of up to 89 values spans at most 12 vectors (3 per lane); denser chunks need 5 per lane.
    const bool dense_slice = __builtin_amdgcn_ballot_w64(longest > 89u) != 0;  // wave-uniform

    // X rows of this lane: row 16 mt + n, its 8 k of a k-step at + 8 g (rows past M are computed on row M-1's data
    // and never stored)
    const uint16_t* xrow[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        const int m = 16 * mt + n;
        xrow[mt] = x + (int64_t)(m < M ? m : M - 1) * K + 8 * g;
    }

    // Fetch everything chunk c needs: NV value vectors per lane and the X operands of its 4 k-steps.
    // Lanes whose vector lies past the piece re-read its last vector (never used); an empty piece reads
    // the start of X instead (always mapped).  No per-lane branches: all requests go out back to back.
    auto issue = [&](auto& st, const uint4 bm, int64_t c) {
        constexpr int NV = sizeof(st.vq) / sizeof(uint4);
        st.bm = bm;
        const uint32_t len = __popc(bm.x) + __popc(bm.y) + __popc(bm.z) + __popc(bm.w);
        st.off = cur & 7u;
        st.nv = len ? (st.off + len + 7u) >> 3 : 0u;
        const uint32_t last = st.nv ? st.nv - 1u : 0u;
        const uint4* vb = st.nv ? values128 + (cur >> 3) : reinterpret_cast<const uint4*>(x);
        cur += len;
#pragma unroll
        for (int i = 0; i < NV; ++i) {
            const uint32_t v = g + 4 * i;
            st.vq[i] = vb[v < last ? v : last];
        }
        if constexpr (kVecBitmap && MT >= 2) {
            // whole chunks only (K % 128 == 0): one address per row tile, the 4 k-steps at constant offsets (with one
            // row tile the two registers of the hoisted pointer cost more than the address arithmetic they save)
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
                if (16 * mt + n < M) {   // lanes of rows past M request nothing: their accumulator rows are never stored
                    const uint16_t* xc = xrow[mt] + c * (kChunkWords * 32);
#pragma unroll
                    for (int s = 0; s < kChunkWords; ++s) st.xq[s * MT + mt] = *reinterpret_cast<const uint4*>(xc + 32 * s);
                }
            }
        } else {
#pragma unroll
            for (int s = 0; s < kChunkWords; ++s) {
                int64_t k = (c * kChunkWords + s) * 32 + 8 * g;
                if constexpr (!kVecBitmap) k = k < K ? k : K - 8;  // ragged last chunk: the weight operand is zero there
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) {
                    const int m = 16 * mt + n;
                    if (m < M) st.xq[s * MT + mt] = *reinterpret_cast<const uint4*>(x + (int64_t)m * K + k);
                }
            }
        }
    };

    // Park the piece in LDS, expand the 4 byte masks of this lane, run the MFMAs.
    auto consume = [&](const auto& st) {
        constexpr int NV = sizeof(st.vq) / sizeof(uint4);
#pragma unroll
        for (int i = 0; i < NV; ++i) {
            const uint32_t v = g + 4 * i;
            if (NV <= 4 || v < 17u) *reinterpret_cast<uint4*>(slot + 4 * v) = st.vq[i];
        }
        __builtin_amdgcn_wave_barrier();  // LDS executes a wave's accesses in order: writes above land first
        const uint32_t words[kChunkWords] = {st.bm.x, st.bm.y, st.bm.z, st.bm.w};
        uint32_t c_local = st.off;
#pragma unroll
        for (int s = 0; s < kChunkWords; ++s) {
            const uint32_t word = words[s];
            const uint32_t m8 = (word >> (8 * g)) & 0xFFu;
            const uint32_t cb = c_local + __popc(word & ((1u << (8 * g)) - 1u));
            const uint4 wq = expand_byte(slot, lut, cb, m8);
            c_local += __popc(word);
            const bf16x8 b = as_bf16x8(wq);
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
                acc[mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(st.xq[s * MT + mt]), b, acc[mt], 0, 0, 0);
        }
        __builtin_amdgcn_wave_barrier();  // reads above are issued before the next chunk overwrites the slot
    };

    const int64_t n_chunks = c_end - c_begin;
    if (n_chunks == S && !dense_slice) {
        // the whole slice is in flight at once: straight-line code, each chunk waits for its own data only
        StreamStage<MT, 3> st[S];
#pragma unroll
        for (int i = 0; i < S; ++i) issue(st[i], bmq[i], c_begin + i);
#pragma unroll
        for (int i = 0; i < S; ++i) consume(st[i]);
    } else if (n_chunks > 0 && !dense_slice) {
        StreamStage<MT, 3> st[S];
#pragma unroll
        for (int i = 0; i < S; ++i) {
            if (c_begin + i < c_end) {
                issue(st[i], bmq[i], c_begin + i);
                bmq[i] = load_bitmap_chunk(c_begin + i + S);
            }
        }
        for (int64_t c = c_begin; c < c_end; c += S) {
#pragma unroll
            for (int i = 0; i < S; ++i) {
                if (c + i < c_end) consume(st[i]);  // wave-uniform conditions
                if (c + i + S < c_end) {
                    issue(st[i], bmq[i], c + i + S);
                    bmq[i] = load_bitmap_chunk(c + i + 2 * S);
                }
            }
        }
    } else if (n_chunks > 0) {
        // dense pieces (more than ~70 % nonzeros in some chunk): 5 vectors per lane, two chunks in flight
        StreamStage<MT, kMaxVecPerLane> da, db;
        uint4 bm_next = bmq[0];
        auto step = [&](auto& st, int64_t c) {
            issue(st, bm_next, c);
            bm_next = (c + 1 - c_begin < S) ? bmq[(c + 1 - c_begin) % S] : load_bitmap_chunk(c + 1);
        };
        step(da, c_begin);
        for (int64_t c = c_begin; c < c_end; c += 2) {
            if (c + 1 < c_end) step(db, c + 1);
            consume(da);
            if (c + 2 < c_end) step(da, c + 2);
            if (c + 1 < c_end) consume(db);
        }
    }

    __syncthreads();  // every wave is done with its staging slots; T in LDS is complete

    // ---- adapter k-step of this wave (Sec. 3.2): A operand = T rows from LDS, B operand = bq
    if (has_rank_step) {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            const int m = 16 * mt + n;
            const uint4 aq = *reinterpret_cast<const uint4*>(&t_lds[(m < M ? m : M - 1) * kMaxRankPadded + wave * 32 + 8 * g]);
            acc[mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(aq), as_bf16x8(bq), acc[mt], 0, 0, 0);
        }
    }

    // ---- reduce the waves' accumulators and store
    float* red = reinterpret_cast<float*>(smem);
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int e = 0; e < 4; ++e) red[((wave * MT + mt) * 4 + e) * 64 + lane] = acc[mt][e];
    __syncthreads();
    for (int idx = tid; idx < MT * 256; idx += kThreads) {
        const int l = idx & 63;
        const int e = (idx >> 6) & 3;
        const int mt = idx >> 8;
        float s = 0.f;
#pragma unroll
        for (int w = 0; w < NW; ++w) s += red[((w * MT + mt) * 4 + e) * 64 + l];
        const int m = 16 * mt + 4 * (l >> 4) + e;
        const int64_t nn = n0 + (l & 15);
        if (m < M && nn < N) y[(int64_t)m * N + nn] = f32_to_bf16_rne(s);
    }
}

// ---------------------------------------------------------------------------------------------------
// Split-K partials of T = X * A_cat for the small-batch path (Sec. 3.2, first concatenated GEMM).
// Workgroup (slice b, rank tile rt, row block) sums k over its slice for 16 columns of T and 64 rows of X
// with 16x16x32 bf16 MFMAs and writes t_partial[b][m][16 rt + r] (fp32; columns >= R as zeros).
// The main kernel adds the slices up, so no atomics and no zeroed workspace are needed.
//   A operand: lane (m, g) = X[m][k0 + 8g .. +8)            (one 16-byte load)
//   B operand: lane (r, g) = A_cat[k0 + 8g + j][16 rt + r]   (8 two-byte loads, j = 0..7)
// ---------------------------------------------------------------------------------------------------
constexpr int kTpWaves = 4;
constexpr int kTpThreads = kTpWaves * 64;
constexpr int kTpBatch = 4;   // k-steps a wave has in flight

// Blocks past the product's (a one-dimensional grid: product blocks first) build the layer's slice table for this call when
// the caller brought none: the bitmap is read once here, in the shadow of the product's round trips, and the main kernel
// starts from ready cursors (see kTable).
__global__ __launch_bounds__(kTpThreads) void adapter_partial_kernel(const uint16_t* __restrict__ x, int M, int64_t K,
                                                                     const uint16_t* __restrict__ a_cat, int R, int Rpad,
                                                                     int slices, float* __restrict__ t_partial,
                                                                     int product_blocks, const uint32_t* __restrict__ bitmap,
                                                                     const uint32_t* __restrict__ row_offsets, int64_t N,
                                                                     uint32_t* __restrict__ table_out) {
    __shared__ float red[kTpWaves][4][4][64];
    static_assert(kTpThreads == 256, "slice_table_block is written for 256 threads");
    if ((int)blockIdx.x >= product_blocks) {   // the same for the whole workgroup
        slice_table_block(bitmap, row_offsets, N, K, table_out, (int64_t)blockIdx.x - product_blocks, (int)threadIdx.x);
        return;
    }
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int i16 = lane & 15, g = lane >> 4;
    const int rank_tiles = Rpad >> 4;
    const int b = (int)blockIdx.x % slices, rt = ((int)blockIdx.x / slices) % rank_tiles;
    const int row_block = (int)blockIdx.x / (slices * rank_tiles);
    const int64_t units = K >> 5;  // k-steps of 32 columns
    const int64_t u_begin = units * b / slices, u_end = units * (b + 1) / slices;
    const int r = 16 * rt + i16;
    const int r_c = r < R ? r : R - 1;  // padded columns read a valid column and are zeroed at the store
    const int m_base = 64 * row_block;  // 64 rows of X per workgroup
    const int mtiles = ((M - m_base < 64 ? M - m_base : 64) + 15) >> 4;
    f32x4 acc[4];
#pragma unroll
    for (int mt = 0; mt < 4; ++mt) acc[mt] = f32x4{0.f, 0.f, 0.f, 0.f};
    // kTpBatch k-steps per trip with all their loads issued before the first MFMA: the kernel is a handful of dependent
    // round trips long, so they are taken side by side (steps past the slice reload its last step and are skipped)
    for (int64_t u0 = u_begin + wave; u0 < u_end; u0 += kTpWaves * kTpBatch) {
        uint4 bq[kTpBatch], aq[kTpBatch][4];
#pragma unroll
        for (int t = 0; t < kTpBatch; ++t) {
            const int64_t u = u0 + kTpWaves * t < u_end ? u0 + kTpWaves * t : u_end - 1;
            const int64_t k0 = (u << 5) + 8 * g;
            uint32_t e[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) e[j] = a_cat[(k0 + j) * R + r_c];
            bq[t] = make_uint4(e[0] | (e[1] << 16), e[2] | (e[3] << 16), e[4] | (e[5] << 16), e[6] | (e[7] << 16));
#pragma unroll
            for (int mt = 0; mt < 4; ++mt) {
                if (mt < mtiles) {  // uniform
                    const int m = m_base + 16 * mt + i16;
                    aq[t][mt] = *reinterpret_cast<const uint4*>(x + (int64_t)(m < M ? m : M - 1) * K + k0);
                }
            }
        }
#pragma unroll
        for (int t = 0; t < kTpBatch; ++t) {
            if (u0 + kTpWaves * t < u_end) {  // uniform
#pragma unroll
                for (int mt = 0; mt < 4; ++mt)
                    if (mt < mtiles)
                        acc[mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(aq[t][mt]), as_bf16x8(bq[t]), acc[mt], 0, 0, 0);
            }
        }
    }
#pragma unroll
    for (int mt = 0; mt < 4; ++mt)
#pragma unroll
        for (int e = 0; e < 4; ++e) red[wave][mt][e][lane] = acc[mt][e];
    __syncthreads();
    // accumulator layout: lane holds T[16 mt + 4 (lane / 16) + e][16 rt + lane % 16]
    for (int idx = threadIdx.x; idx < mtiles * 256; idx += kTpThreads) {
        const int l = idx & 63, e = (idx >> 6) & 3, mt = idx >> 8;
        float s = 0.f;
#pragma unroll
        for (int w = 0; w < kTpWaves; ++w) s += red[w][mt][e][l];
        const int m = m_base + 16 * mt + 4 * (l >> 4) + e;
        const int rr = 16 * rt + (l & 15);
        if (m < M) t_partial[((int64_t)b * M + m) * Rpad + rr] = rr < R ? s : 0.f;
    }
}

static void launch_adapter_partial_impl(const LinearArgs& a, float* partial, bool build_table, hipStream_t stream) {
    const int R = (int)a.R, Rpad = (int)adapter_rank_padded(a.R);
    const int product_blocks = kStreamTSlices * (Rpad / 16) * (int)((a.M + 63) / 64);
    const int table_blocks = build_table ? (int)((a.N + kSliceTableRowsPerBlock - 1) / kSliceTableRowsPerBlock) : 0;
    hipLaunchKernelGGL(adapter_partial_kernel, dim3((unsigned)(product_blocks + table_blocks)), dim3(kTpThreads), 0, stream, a.x,
                       (int)a.M, a.K, a.a_cat, R, Rpad, kStreamTSlices, partial, product_blocks, a.bitmap, a.row_offsets, a.N,
                       const_cast<uint32_t*>(build_table ? a.slice_table : nullptr));
}

void launch_adapter_partial(const LinearArgs& a, hipStream_t stream) {
    launch_adapter_partial_impl(a, reinterpret_cast<float*>(a.t), a.build_table, stream);
}

void launch_adapter_partial_to(const LinearArgs& a, float* partial, hipStream_t stream) {
    launch_adapter_partial_impl(a, partial, false, stream);
}

template <int MT, int NW, int S>
static void launch_stream_t(const LinearArgs& a, hipStream_t stream, const TimingEvents& ev) {
    const int R = (int)a.R, Rpad = (int)adapter_rank_padded(a.R);
    float* t_partial = reinterpret_cast<float*>(a.t);
    if (R > 0) launch_adapter_partial(a, stream);
    // the optional events take the kernel's own begin/end timestamps (null events = plain launch)
    const unsigned grid = (unsigned)((a.N + kStreamRows - 1) / kStreamRows);
    const int64_t wpr = a.K / 32;
    const uint32_t* no_table = nullptr;
    if (a.slice_table != nullptr && wpr % kChunkWords == 0)   // prepared layer: cursors from its slice table
        SALR_LAUNCH((linear_stream_kernel<MT, NW, S, true, false, true>), dim3(grid), dim3(NW * 64), stream, ev, a.x, (int)a.M,
                    a.K, a.N, a.bitmap, a.values, a.row_offsets, (const float*)t_partial, a.b_cat, R, Rpad, a.y, a.slice_table);
    else if (wpr % kChunkWords != 0)  // bitmap rows are not multiples of 16 bytes: scalar bitmap loads
        SALR_LAUNCH((linear_stream_kernel<MT, NW, S, false, false>), dim3(grid), dim3(NW * 64), stream, ev, a.x, (int)a.M, a.K,
                    a.N, a.bitmap, a.values, a.row_offsets, (const float*)t_partial, a.b_cat, R, Rpad, a.y, no_table);
    else if (wpr / kChunkWords <= 32 && S != 2)  // short rows and one workgroup per CU: barrier-free start (two workgroups
                                                 // per CU hide each other's barrier, and the bitmap words left of a slice,
                                                 // which every wave would fetch again, are a third of the L2 reads)
        SALR_LAUNCH((linear_stream_kernel<MT, NW, S, true, true>), dim3(grid), dim3(NW * 64), stream, ev, a.x, (int)a.M, a.K,
                    a.N, a.bitmap, a.values, a.row_offsets, (const float*)t_partial, a.b_cat, R, Rpad, a.y, no_table);
    else
        SALR_LAUNCH((linear_stream_kernel<MT, NW, S, true, false>), dim3(grid), dim3(NW * 64), stream, ev, a.x, (int)a.M, a.K,
                    a.N, a.bitmap, a.values, a.row_offsets, (const float*)t_partial, a.b_cat, R, Rpad, a.y, no_table);
}

hipError_t launch_linear_stream(const LinearArgs& a, hipStream_t stream, const TimingEvents& ev) {
    constexpr int NW = 8;
    // More row groups than two per CU: the leaner variant (2 chunks in flight, 128 registers) lets two
    // workgroups share a CU, so one group's start-up and reduction overlap the other's stream.
    const bool many_groups = (a.N + kStreamRows - 1) / kStreamRows >= 2 * 256;
    if (a.M <= 16 && many_groups) launch_stream_t<1, NW, 2>(a, stream, ev);
    else if (a.M <= 16) launch_stream_t<1, NW, 4>(a, stream, ev);
    else if (a.M <= 32) launch_stream_t<2, NW, 3>(a, stream, ev);
    else launch_stream_t<4, NW, 2>(a, stream, ev);
    return hipGetLastError();
}

}  // namespace salr
