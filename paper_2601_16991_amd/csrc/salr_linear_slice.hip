// Decode-sized batches (M <= 16) of the SALR linear on long rows of whole 128-column chunks: one pass over the
// compressed weight, HBM-bound.  The shape of the small-batch kernel (a workgroup owns 16 consecutive rows of What for
// the whole contraction, its 8 waves split K into contiguous slices and meet only for the final sum), with what a
// compute unit's memory path has to carry cut down:
//
//   round trip 1  row offset; the slice's bitmap, every word ONCE per wave: lane (n, g) loads the four words of chunk
//               4 b + g of row n (b = group of four chunks) and the other lanes of the row get them by lane shuffles
//               when the chunk is decoded.  The waves exchange their per-row nonzero counts through LDS (one
//               barrier), which places every wave's cursor into `values`: no bitmap word is read twice, where the
//               small-batch kernel re-reads the words left of each slice.
//   round trip 2  packed values: a group's values of one row (4 chunks = 512 columns) are ONE contiguous piece;
//               the 4 lanes of a row fetch it with 16-byte loads (40 vectors ahead, more when the piece is consumed),
//               the next group's piece while this one is decoded; then X (from the L2), four chunks ahead.
//   decode + MFMA  as in the other streaming kernels: the piece is parked in the wave's LDS slot and expanded by the
//               nibble rule of Sec. 3.3 straight into the B operand of a 16x16x32 bf16 MFMA.
//   adapters (Sec. 3.2), reduction over the waves, store: as in the small-batch kernel.
// Measured against the small-batch kernel on the Llama-3 shapes: 10 to 14 % ahead from K = 14336 on; level or behind
// on shorter rows (where one workgroup per compute unit, which the 147 KB of slots allow, covers too few round trips).
#include <hip/hip_ext.h>

#include "salr_device.hpp"
#include "salr_internal.hpp"
#include "salr_linear_common.hpp"

namespace salr {

constexpr int kSlRows = 16;           // weight rows per workgroup
constexpr int kSlWaves = 8;
constexpr int kSlThreads = kSlWaves * 64;
constexpr int kSlChunkWords = 4;      // bitmap words per row and chunk (128 columns)
constexpr int kSlGroup = 4;           // chunks per group: one bitmap load per lane, one piece of values per row
constexpr int kSlEager = 10;          // value vectors per lane requested ahead: 40 vectors hold >= 313 of a group's 512 values
constexpr int64_t kSlMinK = 12288;   // rows from here on take this kernel (>= 12 chunks per wave)
constexpr int kSlSlotDwords = 268;    // LDS per row: 66 vectors of 16 B (512 values + misalignment) + pad; 268 = 12 mod 64 banks

// a native 16-byte vector: an array of these that is written inside a loop stays in registers (an array of uint4 structs does not)
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ uint32_t slice_popc4(const uint4& q) { return __popc(q.x) + __popc(q.y) + __popc(q.z) + __popc(q.w); }

// kMaxGroups: groups of four chunks a wave's slice may have (K <= 8 waves * kMaxGroups * 512 columns)
// kTable: the cursor at the start of the wave's slice comes from the layer's slice table (the slices are the same
// eight), so the waves need not exchange their counts and the workgroup starts without a barrier.
template <int kMaxGroups, bool kTable = false>
__global__ __launch_bounds__(kSlThreads, 1) void linear_slice_kernel(
    const uint16_t* __restrict__ x, int M, int64_t K, int64_t N, const uint32_t* __restrict__ bitmap,
    const uint16_t* __restrict__ values, const uint32_t* __restrict__ row_offsets,
    const float* __restrict__ t_partial, const uint16_t* __restrict__ b_cat, int R, int Rpad,
    uint16_t* __restrict__ y, const uint32_t* __restrict__ slice_table) {
    static_assert(kSlWaves == kSliceTableSlices, "the table holds one entry per wave slice");
    __shared__ __attribute__((aligned(16))) uint32_t slots[kSlWaves * kSlRows * kSlSlotDwords + 8];
    __shared__ __attribute__((aligned(16))) uint16_t t_lds[16 * kMaxRankPadded];  // T = X * A_cat, bf16
    __shared__ uint32_t lut_all[kSlWaves][kNibbleLutWords];  // one copy per wave: filled and used wave-synchronously
    __shared__ __attribute__((aligned(16))) uint32_t slice_count[kSlRows][kSlWaves];
    static_assert(kSlWaves * 256 <= kSlWaves * kSlRows * kSlSlotDwords, "the final reduction reuses the slots");

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // scalar: conditions on it branch uniformly
    const int n = lane & 15;
    const int g = lane >> 4;
    const int64_t n0 = (int64_t)blockIdx.x * kSlRows;
    const int64_t row = n0 + n;
    // Rows past N (last workgroup only) are computed as copies of row N-1 and dropped at the store,
    // so no load below needs a per-lane predicate: every address is clamped into range instead.
    const int64_t row_c = row < N ? row : N - 1;
    const int64_t wpr = K >> 5;
    const int chunks_total = (int)(wpr / kSlChunkWords);
    const int c_begin = chunks_total * wave / kSlWaves;
    const int c_end = chunks_total * (wave + 1) / kSlWaves;
    const int n_chunks = c_end - c_begin;
    const int n_groups = (n_chunks + kSlGroup - 1) / kSlGroup;   // <= kMaxGroups (the host's choice of kernel)
    const uint32_t* brow = bitmap + row_c * wpr;
    uint32_t* lut = lut_all[wave];

    // ---- round trip 1: row offset and the slice's bitmap, chunk 4 b + g of the slice in lane (n, g)
    uint32_t cur;  // element index in `values` of the row's next value
    if constexpr (kTable) cur = slice_table[((int64_t)row_c * kSliceTableSlices + wave) * 2];
    else cur = row_offsets[row_c];
    uint4 bw[kMaxGroups];
#pragma unroll
    for (int b = 0; b < kMaxGroups; ++b) {
        bw[b] = make_uint4(0, 0, 0, 0);
        if (b < n_groups) {   // wave-uniform
            const int c = c_begin + kSlGroup * b + g;
            const uint4 q = *reinterpret_cast<const uint4*>(brow + (int64_t)(c < c_end ? c : c_end - 1) * kSlChunkWords);
            const uint32_t keep = c < c_end ? 0xFFFFFFFFu : 0u;   // chunks past the slice count as empty
            bw[b] = make_uint4(q.x & keep, q.y & keep, q.z & keep, q.w & keep);
        }
    }

    // ---- requests that are not needed before the stream is over: they ride behind round trip 1
    const int t_groups = R > 0 ? M * (Rpad >> 2) : 0;   // float4 groups of T
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

    if (lane < 16) {
        uint32_t a, b;
        nibble_lut_entry(lane, a, b);
        lut[2 * lane] = a;
        lut[2 * lane + 1] = b;
    }

    // ---- nonzeros per group and row (every lane of a row gets the row's sum), and of the whole slice
    uint32_t glen[kMaxGroups];
    uint32_t slice_total = 0;
#pragma unroll
    for (int b = 0; b < kMaxGroups; ++b) {
        uint32_t v = slice_popc4(bw[b]);
        v += __shfl_xor(v, 16, 64);
        v += __shfl_xor(v, 32, 64);
        glen[b] = v;
        slice_total += v;
    }
    if constexpr (!kTable) {
        if (g == 0) slice_count[n][wave] = slice_total;
        __syncthreads();
        const uint4 lo = *reinterpret_cast<const uint4*>(&slice_count[n][0]);
        const uint4 hi = *reinterpret_cast<const uint4*>(&slice_count[n][4]);
        const uint32_t cnt[kSlWaves] = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
#pragma unroll
        for (int w = 0; w < kSlWaves - 1; ++w) cur += w < wave ? cnt[w] : 0u;
    }

    const u32x4* values128 = reinterpret_cast<const u32x4*>(values);
    uint32_t* slot = slots + (wave * kSlRows + n) * kSlSlotDwords;

    // ---- round trip 2: the piece of group 0; the piece of the group after is requested when this one is in LDS.
    // Lanes whose vector lies past the piece re-read its last vector (never used); an empty piece reads the start of X
    // instead (always mapped).  No per-lane branches: all requests go out back to back.
    u32x4 vq[kSlEager];
    uint32_t off = 0, nv = 0;
    const u32x4* vb = reinterpret_cast<const u32x4*>(x);
    auto issue_values = [&](uint32_t len) {
        off = cur & 7u;
        nv = len ? (off + len + 7u) >> 3 : 0u;
        const uint32_t last = nv ? nv - 1u : 0u;
        vb = nv ? values128 + (cur >> 3) : reinterpret_cast<const u32x4*>(x);
        cur += len;
#pragma unroll
        for (int i = 0; i < kSlEager; ++i) {
            const uint32_t v = g + 4 * i;
            vq[i] = vb[v < last ? v : last];
        }
    };
    if (n_groups > 0) issue_values(glen[0]);

    // X operands: lane (m, g) holds X[m][k0 + 8g .. +8) of a k-step; ring of the next four chunks.  Lanes of rows past M
    // request nothing (what comes back from memory is counted per lane, and with one token 15 of 16 lanes would fetch
    // copies); their accumulator rows are never stored, so it does not matter what their registers hold.
    const uint16_t* xrow = x + (int64_t)(n < M ? n : M - 1) * K + 8 * g;
    const bool x_lane = n < M;
    u32x4 xq[kSlGroup][kSlChunkWords];
#pragma unroll
    for (int c = 0; c < kSlGroup; ++c)
#pragma unroll
        for (int s = 0; s < kSlChunkWords; ++s) xq[c][s] = u32x4{0u, 0u, 0u, 0u};
    auto load_x = [&](u32x4 (&q)[kSlChunkWords], int c) {
        if (x_lane) {
            const uint16_t* xc = xrow + (int64_t)c * (kSlChunkWords * 32);
#pragma unroll
            for (int s = 0; s < kSlChunkWords; ++s) q[s] = *reinterpret_cast<const u32x4*>(xc + 32 * s);
        }
    };
#pragma unroll
    for (int c = 0; c < kSlGroup; ++c)
        if (c < n_chunks) load_x(xq[c], c_begin + c);   // wave-uniform

    // T = sum of the pre-kernel's split-K partials, rounded once to bf16, kept in LDS
    for (int i = tid; i < t_groups; i += kSlThreads) {
        float4 sum = make_float4(0.f, 0.f, 0.f, 0.f);
        const float4* p = reinterpret_cast<const float4*>(t_partial) + i;
#pragma unroll
        for (int sl = 0; sl < kStreamTSlices; ++sl) {
            const float4 v = p[(int64_t)sl * t_groups];
            sum.x += v.x; sum.y += v.y; sum.z += v.z; sum.w += v.w;
        }
        const int m = i / (Rpad >> 2), r4 = i % (Rpad >> 2);
        uint2 o;
        o.x = (uint32_t)f32_to_bf16_rne(sum.x) | ((uint32_t)f32_to_bf16_rne(sum.y) << 16);
        o.y = (uint32_t)f32_to_bf16_rne(sum.z) | ((uint32_t)f32_to_bf16_rne(sum.w) << 16);
        *reinterpret_cast<uint2*>(&t_lds[m * kMaxRankPadded + 4 * r4]) = o;
    }

    f32x4 acc = f32x4{0.f, 0.f, 0.f, 0.f};

    for (int b = 0; b < n_groups; ++b) {
        // park the piece in LDS: the vectors requested ahead, then (pieces of more than 40 vectors: denser than ~60 %)
        // the rest, fetched now
#pragma unroll
        for (int i = 0; i < kSlEager; ++i) *reinterpret_cast<u32x4*>(slot + 4 * (g + 4 * i)) = vq[i];
        for (uint32_t v = 4 * kSlEager + g; v < nv; v += 4) *reinterpret_cast<u32x4*>(slot + 4 * v) = vb[v];
        __builtin_amdgcn_wave_barrier();  // LDS executes a wave's accesses in order: writes above land first
        uint32_t c_local = off;
        const uint4 words_mine = bw[0];
        // the registers of the piece are free again: request the next group's
        if (b + 1 < n_groups) issue_values(glen[kMaxGroups > 1 ? 1 : 0]);
#pragma unroll
        for (int c = 0; c < kSlGroup; ++c) {
            if (kSlGroup * b + c < n_chunks) {   // wave-uniform
                // the chunk's four bitmap words of row n sit in lane (n, c)
                const int src = 4 * (n + 16 * c);
                const uint32_t words[kSlChunkWords] = {(uint32_t)__builtin_amdgcn_ds_bpermute(src, (int)words_mine.x),
                                                        (uint32_t)__builtin_amdgcn_ds_bpermute(src, (int)words_mine.y),
                                                        (uint32_t)__builtin_amdgcn_ds_bpermute(src, (int)words_mine.z),
                                                        (uint32_t)__builtin_amdgcn_ds_bpermute(src, (int)words_mine.w)};
#pragma unroll
                for (int s = 0; s < kSlChunkWords; ++s) {
                    const uint32_t word = words[s];
                    const uint32_t m8 = (word >> (8 * g)) & 0xFFu;
                    const uint32_t cb = c_local + __popc(word & ((1u << (8 * g)) - 1u));
                    const uint4 wq = expand_byte(slot, lut, cb, m8);
                    c_local += __popc(word);
                    acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, xq[c][s]), as_bf16x8(wq), acc, 0, 0, 0);
                }
                const int next = c_begin + kSlGroup * (b + 1) + c;
                if (next < c_end) load_x(xq[c], next);
            }
        }
        __builtin_amdgcn_wave_barrier();  // reads above are issued before the next piece overwrites the slot
        // the next group's bitmap words and length move up
#pragma unroll
        for (int i = 0; i + 1 < kMaxGroups; ++i) {
            bw[i] = bw[i + 1];
            glen[i] = glen[i + 1];
        }
    }

    __syncthreads();  // every wave is done with its slot; T in LDS is complete

    // ---- adapter k-step of this wave (Sec. 3.2): A operand = T rows from LDS, B operand = bq
    if (has_rank_step) {
        const uint4 aq = *reinterpret_cast<const uint4*>(&t_lds[(n < M ? n : M - 1) * kMaxRankPadded + wave * 32 + 8 * g]);
        acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(aq), as_bf16x8(bq), acc, 0, 0, 0);
    }

    // ---- reduce the waves' accumulators and store
    float* red = reinterpret_cast<float*>(slots);
#pragma unroll
    for (int e = 0; e < 4; ++e) red[(wave * 4 + e) * 64 + lane] = acc[e];
    __syncthreads();
    if (tid < 256) {
        const int l = tid & 63;
        const int e = tid >> 6;
        float s = 0.f;
#pragma unroll
        for (int w = 0; w < kSlWaves; ++w) s += red[(w * 4 + e) * 64 + l];
        const int m = 4 * (l >> 4) + e;
        const int64_t nn = n0 + (l & 15);
        if (m < M && nn < N) y[(int64_t)m * N + nn] = f32_to_bf16_rne(s);
    }
}

bool linear_slice_takes(int64_t M, int64_t K, int64_t N) {
    (void)N;
    if (M > 16 || K < kSlMinK || K % 128 != 0) return false;
    const int64_t chunks = K / 128;
    const int64_t per_wave = (chunks + kSlWaves - 1) / kSlWaves;
    return (per_wave + kSlGroup - 1) / kSlGroup <= 8;
}

template <int kMaxGroups>
static void launch_slice_t(const LinearArgs& a, const float* t_partial, unsigned grid, hipStream_t stream,
                           const TimingEvents& ev) {
    const int R = (int)a.R, Rpad = (int)adapter_rank_padded(a.R);
    const uint32_t* no_table = nullptr;
    if (a.slice_table != nullptr)   // prepared layer
        SALR_LAUNCH((linear_slice_kernel<kMaxGroups, true>), dim3(grid), dim3(kSlThreads), stream, ev, a.x, (int)a.M, a.K, a.N,
                    a.bitmap, a.values, a.row_offsets, t_partial, a.b_cat, R, Rpad, a.y, a.slice_table);
    else
        SALR_LAUNCH((linear_slice_kernel<kMaxGroups, false>), dim3(grid), dim3(kSlThreads), stream, ev, a.x, (int)a.M, a.K, a.N,
                    a.bitmap, a.values, a.row_offsets, t_partial, a.b_cat, R, Rpad, a.y, no_table);
}

hipError_t launch_linear_slice(const LinearArgs& a, hipStream_t stream, const TimingEvents& ev) {
    const float* t_partial = reinterpret_cast<const float*>(a.t);
    if (a.R > 0) launch_adapter_partial(a, stream);
    const unsigned grid = (unsigned)((a.N + kSlRows - 1) / kSlRows);
    const int64_t per_wave = (a.K / 128 + kSlWaves - 1) / kSlWaves;
    const int groups = (int)((per_wave + kSlGroup - 1) / kSlGroup);
    if (groups <= 1) launch_slice_t<1>(a, t_partial, grid, stream, ev);
    else if (groups <= 4) launch_slice_t<4>(a, t_partial, grid, stream, ev);
    else launch_slice_t<8>(a, t_partial, grid, stream, ev);
    return hipGetLastError();
}

}  // namespace salr
