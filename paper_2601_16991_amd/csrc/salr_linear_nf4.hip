// Small-batch (M <= 64) QSALR linear (paper Sec. 4, "Coupled with Quantization"; the layer of Sec. 3.2 / 3.3): the
// small-batch streaming kernel reading the packed values as 4-bit NormalFloat codes, so the weight crosses the memory
// system at 1 bit + 4.25 bits per stored value and is never written back in bf16.
//
// Work split, X operands, adapters and epilogue are those of salr_linear_stream.hip: a workgroup owns 16 weight rows,
// its 8 waves split K into the slices of the layer's slice table, lane (n = lane%16, g = lane/16) takes byte g of each
// bitmap word of row n.  What differs is the decode stage, per chunk of 128 columns:
//   request     the row's piece of codes (up to 128 nibbles, at any nibble offset: at most five 16-byte vectors of 32
//               codes; lane g asks for vector g and for dword g of the fifth).  A vector of 32 codes never straddles
//               two scale blocks (64 values), so each request comes with ONE scale;
//   dequantise  every lane turns its 40 codes into bf16 -- level from a 16-entry table, times the scale, rounded to
//               bf16 (the value rule of the code: bf16(fp32(level * scale))) -- and parks them in the row's LDS slot,
//               which then holds the piece as the bf16 kernel's slot does;
//   expand      as there: the nibble rule of Sec. 3.3 (two byte permutes per four columns) straight into the B operand
//               of a 16x16x32 bf16 MFMA.
// The result equals that of the small-batch streaming kernel on the dequantised values bit for bit (finite scales):
// the same products enter the same MFMA chain in the same order.
#include <hip/hip_ext.h>

#include "salr_device.hpp"
#include "salr_internal.hpp"
#include "salr_linear_common.hpp"
#include "salr_nf4.hpp"

namespace salr {

constexpr int kQRows = 16;            // weight rows per workgroup
constexpr int kQWaves = 8;
constexpr int kQChunkWords = 4;       // bitmap words per row per chunk (128 columns)
constexpr int kQSlotDwords = 84;      // LDS per row per chunk: 160 bf16 (five vectors of 32 codes, dequantised) + 2
                                      // dwords that the expansion may read past them; 84 n mod 64 are 16 different
                                      // multiples of 4, so the rows of a wave start in different banks
constexpr int kQLevelWords = 16;

template <int MT>
struct NfStage {
    uint4 bm;                        // the chunk's 4 bitmap words of this lane's row
    uint4 cq;                        // vector g of the row's piece of codes (32 codes)
    uint32_t c4;                     // dword g of its fifth vector (8 codes)
    uint4 xq[kQChunkWords * MT];     // X operands of the chunk's 4 k-steps
    uint32_t sc, sc4;                // bf16 scales of the blocks that vector g and the fifth vector lie in
    uint32_t off;                    // nibble offset of the piece inside its first vector (0..31)
};

// MT m-tiles of 16 rows, S chunks in flight per wave.  K % 128 == 0, nnz > 0.
template <int MT, int S>
__global__ __launch_bounds__(kQWaves * 64, (S == 2 && MT == 1) ? 4 : 1) void linear_nf4_kernel(
    const uint16_t* __restrict__ x, int M, int64_t K, int64_t N, const uint32_t* __restrict__ bitmap,
    const uint8_t* __restrict__ codes, const uint16_t* __restrict__ scales, uint32_t scale_last,
    const uint32_t* __restrict__ slice_table, const float* __restrict__ t_partial, const uint16_t* __restrict__ b_cat,
    int R, int Rpad, uint16_t* __restrict__ y) {
    static_assert(kQWaves == kSliceTableSlices, "the table holds one entry per wave slice");
    constexpr int NW = kQWaves;
    constexpr int kThreads = NW * 64;
    constexpr int kStageDwords = NW * kQRows * kQSlotDwords;
    constexpr int kRedFloats = NW * MT * 256;
    constexpr int kSmemDwords = kStageDwords > kRedFloats ? kStageDwords : kRedFloats;
    constexpr int kTRows = 16 * MT;
    __shared__ __attribute__((aligned(16))) uint32_t smem[kSmemDwords];
    __shared__ __attribute__((aligned(16))) uint16_t t_lds[kTRows * kMaxRankPadded];  // T = X * A_cat, bf16
    __shared__ uint32_t lut_all[NW][kNibbleLutWords];   // one copy per wave: filled and used wave-synchronously
    __shared__ float level_all[NW][kQLevelWords];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int n = lane & 15;
    const int g = lane >> 4;
    const int64_t n0 = (int64_t)blockIdx.x * kQRows;
    const int64_t row = n0 + n;
    const int64_t wpr = K >> 5;
    const int64_t chunks_total = wpr / kQChunkWords;
    const int64_t c_begin = chunks_total * wave / NW;
    const int64_t c_end = chunks_total * (wave + 1) / NW;
    uint32_t* lut = lut_all[wave];
    float* levels = level_all[wave];
    // Rows past N (last workgroup only) are computed as copies of row N-1 and dropped at the store.
    const int64_t row_c = row < N ? row : N - 1;
    const uint32_t* brow = bitmap + row_c * wpr;

    // index in the packed values of the first value of this wave's slice of the row
    uint32_t cur = slice_table[((int64_t)row_c * kSliceTableSlices + wave) * 2];

    auto load_bitmap_chunk = [&](int64_t c) -> uint4 {
        uint4 q = make_uint4(0, 0, 0, 0);
        if (c < c_end) q = *reinterpret_cast<const uint4*>(brow + c * kQChunkWords);   // wave-uniform when c is
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
        levels[lane] = kNf4Levels[lane];
    }
    __builtin_amdgcn_wave_barrier();

    const uint4* codes128 = reinterpret_cast<const uint4*>(codes);
    uint32_t* slot = smem + (wave * kQRows + n) * kQSlotDwords;

    f32x4 acc[MT];
#pragma unroll
    for (int i = 0; i < MT; ++i) acc[i] = f32x4{0.f, 0.f, 0.f, 0.f};

    // X rows of this lane: row 16 mt + n, its 8 k of a k-step at + 8 g
    const uint16_t* xrow[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        const int m = 16 * mt + n;
        xrow[mt] = x + (int64_t)(m < M ? m : M - 1) * K + 8 * g;
    }

    // Request everything chunk c needs.  Lanes whose vector lies past the piece re-read its last vector (never used);
    // an empty piece reads the start of X instead (always mapped); scale indices are clamped to the last block.
    auto issue = [&](NfStage<MT>& st, const uint4 bm, int64_t c) {
        st.bm = bm;
        const uint32_t len = __popc(bm.x) + __popc(bm.y) + __popc(bm.z) + __popc(bm.w);
        st.off = cur & 31u;
        const uint32_t vbase = cur >> 5;
        const uint32_t nv = len ? (st.off + len + 31u) >> 5 : 0u;
        const uint32_t last = nv ? nv - 1u : 0u;
        const uint32_t v_mine = (uint32_t)g < last ? (uint32_t)g : last;
        const uint32_t v_fifth = 4u < last ? 4u : last;
        const uint4* vb = nv ? codes128 + vbase : reinterpret_cast<const uint4*>(x);
        st.cq = vb[v_mine];
        st.c4 = reinterpret_cast<const uint32_t*>(vb + v_fifth)[g];
        const uint32_t blk = (vbase + v_mine) >> 1, blk4 = (vbase + v_fifth) >> 1;   // 64 values = two vectors per block
        st.sc = scales[blk < scale_last ? blk : scale_last];
        st.sc4 = scales[blk4 < scale_last ? blk4 : scale_last];
        cur += len;
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            if (16 * mt + n < M) {   // lanes of rows past M request nothing: their accumulator rows are never stored
                const uint16_t* xc = xrow[mt] + c * (kQChunkWords * 32);
#pragma unroll
                for (int s = 0; s < kQChunkWords; ++s) st.xq[s * MT + mt] = *reinterpret_cast<const uint4*>(xc + 32 * s);
            }
        }
    };

    // Dequantise this lane's codes into the row's slot, expand the 4 byte masks of this lane, run the MFMAs.
    auto consume = [&](const NfStage<MT>& st) {
        const float sa = __uint_as_float(st.sc << 16), s4 = __uint_as_float(st.sc4 << 16);   // bf16 -> fp32
        uint4* slot4 = reinterpret_cast<uint4*>(slot);
        slot4[4 * g + 0] = nf4_decode8(st.cq.x, sa, levels);   // values 32 g .. 32 g + 31 of the slot
        slot4[4 * g + 1] = nf4_decode8(st.cq.y, sa, levels);
        slot4[4 * g + 2] = nf4_decode8(st.cq.z, sa, levels);
        slot4[4 * g + 3] = nf4_decode8(st.cq.w, sa, levels);
        slot4[16 + g] = nf4_decode8(st.c4, s4, levels);        // values 128 + 8 g .. of the fifth vector
        __builtin_amdgcn_wave_barrier();  // LDS executes a wave's accesses in order: writes above land first
        const uint32_t words[kQChunkWords] = {st.bm.x, st.bm.y, st.bm.z, st.bm.w};
        uint32_t c_local = st.off;
#pragma unroll
        for (int s = 0; s < kQChunkWords; ++s) {
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
    if (n_chunks == S) {
        // the whole slice is in flight at once: straight-line code, each chunk waits for its own data only
        NfStage<MT> st[S];
#pragma unroll
        for (int i = 0; i < S; ++i) issue(st[i], bmq[i], c_begin + i);
#pragma unroll
        for (int i = 0; i < S; ++i) consume(st[i]);
    } else if (n_chunks > 0) {
        NfStage<MT> st[S];
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

bool linear_nf4_takes(int64_t M, int64_t K, int64_t N, int64_t nnz) {
    return M > 0 && M <= kStreamMaxM && N > 0 && K >= 128 && K % 128 == 0 && nnz > 0;
}

// Workspace of the fused call: the split-K partials of T (with adapters), then the call's slice table.
size_t linear_nf4_table_offset(int64_t M, int64_t R) {
    return R > 0 ? round_up_256((size_t)kStreamTSlices * (size_t)M * (size_t)adapter_rank_padded(R) * sizeof(float)) : 0;
}
size_t linear_nf4_workspace_bytes(int64_t M, int64_t N, int64_t R) {
    return linear_nf4_table_offset(M, R) + round_up_256(slice_table_bytes(N));
}

template <int MT, int S>
static void launch_nf4_t(const LinearArgs& a, const uint8_t* codes, const uint16_t* scales, int64_t nnz, hipStream_t stream,
                         const TimingEvents& ev) {
    const int R = (int)a.R, Rpad = (int)adapter_rank_padded(a.R);
    const unsigned grid = (unsigned)((a.N + kQRows - 1) / kQRows);
    const uint32_t scale_last = (uint32_t)((nnz + 63) / 64 - 1);
    SALR_LAUNCH((linear_nf4_kernel<MT, S>), dim3(grid), dim3(kQWaves * 64), stream, ev, a.x, (int)a.M, a.K, a.N, a.bitmap, codes,
                scales, scale_last, a.slice_table, reinterpret_cast<const float*>(a.t), a.b_cat, R, Rpad, a.y);
}

// a.t: the partials of T (R > 0), a.slice_table: room for the table (built here), a.values unused.
hipError_t launch_linear_nf4(const LinearArgs& a_in, const uint8_t* codes, const uint16_t* scales, int64_t nnz,
                             hipStream_t stream, const TimingEvents& ev) {
    LinearArgs a = a_in;
    if (a.R > 0) {   // the adapter pre-kernel builds the table in its extra workgroups
        a.build_table = true;
        launch_adapter_partial(a, stream);
    } else {
        hipError_t e = launch_build_slice_table(a.bitmap, a.row_offsets, a.N, a.K, const_cast<uint32_t*>(a.slice_table), stream);
        if (e != hipSuccess) return e;
    }
    const bool many_groups = (a.N + kQRows - 1) / kQRows >= 2 * 256;
    if (a.M <= 16 && many_groups) launch_nf4_t<1, 2>(a, codes, scales, nnz, stream, ev);
    else if (a.M <= 16) launch_nf4_t<1, 4>(a, codes, scales, nnz, stream, ev);
    else if (a.M <= 32) launch_nf4_t<2, 3>(a, codes, scales, nnz, stream, ev);
    else launch_nf4_t<4, 2>(a, codes, scales, nnz, stream, ev);
    return hipGetLastError();
}

}  // namespace salr
