// Large batches (M > 64) without a decoded copy of the weight: the two-stage pipeline of Sec. 3.3 ("Pipeline Design")
// inside one kernel, the stages connected by double-buffered LDS tiles.
//
// Workgroup = 8 waves, output tile 256 (m) x 128 (n), k-step 32, two workgroups per CU (4 waves per SIMD), LDS
// tiles double-buffered:
//
//   X tile       travels from memory straight into LDS (global_load_lds, 16 bytes per lane): the four lanes of
//                a row fetch its 64 bytes of the k-step, no registers and no VALU involved;
//   decode stage (all threads, for k-step s+1 while the MFMAs of step s run)
//       thread (row = tid/4, q = tid%4) owns byte q of the bitmap word of one weight row of the tile.  Packed
//       values arrive per 64-column chunk: each row's piece is contiguous in `values`, is fetched by the row's
//       four threads with 16-byte loads a chunk ahead, parked in the row's LDS slot and expanded with the
//       nibble rule (Sec. 3.3) into the dense LDS tile Ws;
//   MFMA stage   wave (wm, wn) owns 64 (m) x 64 (n): 2 x 2 tiles of v_mfma_f32_32x32x16_bf16;
//   adapters (Sec. 3.2): after the K loop the same accumulators take Rpad/32 more k-steps with
//       Xs := T (bf16, from adapter_t_kernel) and Ws := B_cat columns.
//
// Consecutive workgroup ids land on different XCDs (8 of them, each with its own L2); the id -> tile
// map keeps all m-tiles of one n-tile on the same XCD so the compressed rows are fetched into one L2.
// Every m-tile decodes the weight tile again, and the decode instructions share the SIMDs with the MFMAs: with a
// workspace for a decoded copy (2 N K bytes) the call decodes once into memory and runs a dense MFMA kernel instead
// (salr_linear_twostage.hip), which is faster at every M > 64 that was measured.  This kernel is what runs when the
// caller gives the layer no room for that copy: the weight then never exists in dense form outside LDS.
#include "salr_device.hpp"
#include "salr_internal.hpp"
#include "salr_linear_common.hpp"

namespace salr {

constexpr int kTM = 256, kTN = 128, kTK = 32;
constexpr int kTiledThreads = 512;
constexpr int kPitch = kTK;              // bf16 elements per LDS tile row: 64 bytes = four 16-byte segments, no padding
constexpr int kSlotDw = 36;              // 9 vectors of 16 B: 64 values + misalignment
constexpr int kXcds = 8;

// LDS tiles are swizzled instead of padded: segment s of row r sits at segment s ^ ((r >> 2) & 3).  Sixteen
// consecutive lanes then cover all sixteen 16-byte bank groups of a 256-byte LDS line both when an MFMA
// operand is read (16 rows, one segment) and when the tiles are written (8 rows x 2 or 4 rows x 4 segments).
__device__ __forceinline__ int swz(int row, int seg) { return (seg ^ ((row >> 2) & 3)) * 8; }


__global__ __launch_bounds__(kTiledThreads, 4) void linear_tiled_kernel(
    const uint16_t* __restrict__ x, int64_t M, int64_t K, int64_t N, const uint32_t* __restrict__ bitmap,
    const uint16_t* __restrict__ values, const uint32_t* __restrict__ row_offsets, const uint16_t* __restrict__ t,
    const uint16_t* __restrict__ b_cat, int R, int Rpad, uint16_t* __restrict__ y, int m_tiles, int n_tiles) {
    // two separate arrays, not one [2][...]: the compiler orders LDS reads against the asynchronous loads
    // into LDS per variable, and reads of one buffer must not wait for loads into the other
    __shared__ __attribute__((aligned(16))) uint16_t Xs0[kTM * kPitch];
    __shared__ __attribute__((aligned(16))) uint16_t Xs1[kTM * kPitch];
    __shared__ __attribute__((aligned(16))) uint16_t Ws[2][kTN * kPitch];
    __shared__ __attribute__((aligned(16))) uint32_t stage[kTN * kSlotDw + 8];
    __shared__ uint32_t lut[kNibbleLutWords];

    // ---- tile of this workgroup
    const int bid = blockIdx.x;
    const int xcd = bid % kXcds, local = bid / kXcds;
    const int nt = (local / m_tiles) * kXcds + xcd;
    const int mt = local % m_tiles;
    if (nt >= n_tiles) return;  // uniform for the workgroup, before any barrier
    const int64_t m0 = (int64_t)mt * kTM, n0 = (int64_t)nt * kTN;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave >> 1, wn = wave & 1;

    nibble_lut_init(lut);

    // ---- both roles use the same split: four threads per tile row, thread q owns 8 of the row's 32 columns.
    // Loader: segment q of X rows wr and wr + 128 (the four lanes of a row fetch 64 contiguous bytes).
    // Decoder: byte q of the bitmap word of weight row wr.
    const int wr = tid >> 2, q = tid & 3;
    const int64_t xrow0 = (m0 + wr < M) ? m0 + wr : M - 1;   // rows past the edge recompute the last row; never stored
    const int64_t xrow1 = (m0 + wr + 128 < M) ? m0 + wr + 128 : M - 1;
    // X tiles go from memory straight into LDS (no registers): a wave's load instruction fills 1 KB = its 16
    // rows of 64 bytes, lane l landing on 16-byte slot l.  Slot (row, p) holds logical segment p ^ swizzle(row),
    // so that is the segment the lane fetches.
    const int xseg = q ^ ((wr >> 2) & 3);
    const uint16_t* xptr0 = x + xrow0 * K + 8 * xseg;
    const uint16_t* xptr1 = x + xrow1 * K + 8 * xseg;
    const int64_t wrow = (n0 + wr < N) ? n0 + wr : N - 1;
    const int64_t wpr = K >> 5;
    const uint32_t* brow = bitmap + wrow * wpr;
    const uint4* values128 = reinterpret_cast<const uint4*>(values);
    uint32_t* slot = stage + wr * kSlotDw;
    uint32_t cur = row_offsets[wrow];  // element index in `values` of the row's next unfetched value
    const int64_t steps = K / kTK;
    const int64_t chunks = steps / 2;   // K % 64 == 0 on this path

    auto load_bitmap = [&](int64_t c) -> uint2 {
        return (c < chunks) ? *reinterpret_cast<const uint2*>(brow + 2 * c) : make_uint2(0, 0);
    };
    typedef const __attribute__((address_space(1))) void* gptr_t;
    typedef __attribute__((address_space(3))) void* lptr_t;
    // request X tile of k-step s into buffer `buf`; completion is awaited (vmcnt) before the barrier that
    // publishes the buffer
    auto fetch_x = [&](int buf, int64_t s) {
        const int64_t sc = s < steps ? s : steps - 1;  // past the end: reload the last step (unused)
        uint16_t* dst = (buf ? Xs1 : Xs0) + (wave * 16) * kPitch;
        __builtin_amdgcn_global_load_lds((gptr_t)(xptr0 + sc * kTK), (lptr_t)dst, 16, 0, 0);
        __builtin_amdgcn_global_load_lds((gptr_t)(xptr1 + sc * kTK), (lptr_t)(dst + 128 * kPitch), 16, 0, 0);
    };
    auto x_landed = [&]() { __builtin_amdgcn_s_waitcnt(0x0F70); };  // vmcnt(0)
    // One staged value chunk (the packed values of 64 columns of the row, contiguous in `values`) lives in
    // plain registers: this thread's two 16-byte vectors of the piece, the piece's first vector, the index
    // of its last vector, the element offset of the piece inside its first vector and its vector count.
    uint4 vq0, vq1;
    const uint4* vb;
    uint32_t v_last, v_off, v_nv;
    auto v_issue = [&](uint2 w) {
        const uint32_t len = __popc(w.x) + __popc(w.y);
        v_off = cur & 7u;
        v_nv = len ? (v_off + len + 7u) >> 3 : 0u;
        vb = v_nv ? values128 + (cur >> 3) : reinterpret_cast<const uint4*>(x);
        v_last = v_nv ? v_nv - 1u : 0u;
        cur += len;
        // clamped, not predicated: both requests go out back to back.  A ninth vector exists only in
        // pieces denser than ~90 %; v_store fetches it on the spot.
        vq0 = vb[(uint32_t)q < v_last ? (uint32_t)q : v_last];
        vq1 = vb[(uint32_t)q + 4u < v_last ? (uint32_t)q + 4u : v_last];
    };
    uint32_t c_local = 0;  // cursor inside the slot
    // park the chunk in the row's LDS slot (only the row's own four threads, lanes of one wave, touch it)
    auto v_store = [&]() {
        uint4* sv = reinterpret_cast<uint4*>(slot);
        sv[q] = vq0;
        sv[q + 4] = vq1;
        if (__builtin_amdgcn_ballot_w64(v_nv > 8u)) {  // rare, wave-uniform
            if (q == 0) sv[8] = vb[8u < v_last ? 8u : v_last];
        }
        __builtin_amdgcn_wave_barrier();
        c_local = v_off;  // the slot's cursor restarts at the piece's offset
    };
    // expand this thread's byte mask of `word` into Ws[buf]
    auto decode = [&](int buf, uint32_t word) {
        const uint32_t cb = c_local + __popc(word & ((1u << (8 * q)) - 1u));
        const uint4 qa = expand_byte(slot, lut, cb, (word >> (8 * q)) & 0xFFu);
        c_local += __popc(word);
        *reinterpret_cast<uint4*>(&Ws[buf][wr * kPitch + swz(wr, q)]) = qa;
    };

    f32x16 acc00 = {0}, acc01 = {0}, acc10 = {0}, acc11 = {0};

    // operand lane: row lane%32 of a 32-row block, k-group lane/32 (+2 for the second half of the k-step);
    // rows 32 or 64 further down share the swizzle term
    const int frag_row = lane & 31;
    const int frag_k0 = swz(frag_row, lane >> 5), frag_k1 = swz(frag_row, (lane >> 5) + 2);
    auto mfma_step = [&](int buf) {
        const uint16_t* xa = (buf ? Xs1 : Xs0) + (wm * 64 + frag_row) * kPitch;
        const uint16_t* wb = &Ws[buf][(wn * 64 + frag_row) * kPitch];
        auto frag = [](const uint16_t* p) { return *reinterpret_cast<const bf16x8*>(p); };
        const bf16x8 a00 = frag(xa + frag_k0), a10 = frag(xa + 32 * kPitch + frag_k0);
        const bf16x8 b00 = frag(wb + frag_k0), b10 = frag(wb + 32 * kPitch + frag_k0);
        const bf16x8 a01 = frag(xa + frag_k1), a11 = frag(xa + 32 * kPitch + frag_k1);
        const bf16x8 b01 = frag(wb + frag_k1), b11 = frag(wb + 32 * kPitch + frag_k1);
        acc00 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a00, b00, acc00, 0, 0, 0);
        acc01 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a00, b10, acc01, 0, 0, 0);
        acc10 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a10, b00, acc10, 0, 0, 0);
        acc11 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a10, b10, acc11, 0, 0, 0);
        acc00 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a01, b01, acc00, 0, 0, 0);
        acc01 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a01, b11, acc01, 0, 0, 0);
        acc10 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a11, b01, acc10, 0, 0, 0);
        acc11 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a11, b11, acc11, 0, 0, 0);
    };

    // ---- prologue: bitmap of chunks 0..2, values of chunk 0 parked and of chunk 1 requested, tile 0 in buffer 0
    uint2 bm0 = load_bitmap(0), bm1 = load_bitmap(1), bm2 = load_bitmap(2);
    fetch_x(0, 0);
    v_issue(bm0);
    __syncthreads();  // lut
    v_store();
    decode(0, bm0.x);
    v_issue(bm1);
    x_landed();
    __syncthreads();

    // ---- main loop: one value chunk (2 k-steps, one bitmap pair) per iteration.  Within a k-step the MFMAs
    // read buffer s%2 while the loaders fill buffer (s+1)%2, so the two halves may run in either order: even
    // waves fill first, odd waves multiply first.  Two workgroups share a CU (4 waves per SIMD), so decode
    // and LDS latency of some waves overlaps the MFMAs of the others.
    const bool fill_first = (wave & 1) == 0;
    for (int64_t c = 0; c < chunks; ++c) {
        const int64_t s0 = 2 * c;
        // step s0 (tile in buffer 0): decode tile s0+1 from the parked chunk, word 1
        fetch_x(1, s0 + 1);
        if (!fill_first) mfma_step(0);
        decode(1, bm0.y);
        if (fill_first) mfma_step(0);
        x_landed();
        __syncthreads();
        // step s0+1 (buffer 1): chunk c+1 becomes current; decode tile s0+2 (its word 0); request chunk c+2
        fetch_x(0, s0 + 2);
        if (!fill_first) mfma_step(1);
        v_store();
        decode(0, bm1.x);
        v_issue(bm2);
        bm0 = bm1;
        bm1 = bm2;
        bm2 = load_bitmap(c + 3);
        if (fill_first) mfma_step(1);
        x_landed();
        __syncthreads();
    }

    // ---- adapter k-steps (Sec. 3.2): Xs := T[m, r0 .. r0+31], Ws := B_cat[r0 .. r0+31, n]
    if (R > 0) {
        const int64_t bn = (n0 + (tid & 127) < N) ? n0 + (tid & 127) : N - 1;
        const int rr4 = tid >> 7;                  // rank row 4 i + rr4 of the k-step: segment i / 2 of tile row tid % 128
        const int bf = ((tid & 127) >> 2) & 3;     // that row's swizzle term
        for (int r0 = 0; r0 < Rpad; r0 += kTK) {
            uint16_t* xs = &Xs0[wr * kPitch + swz(wr, q)];   // row wr + 128 has the same swizzle term
            *reinterpret_cast<uint4*>(xs) = *reinterpret_cast<const uint4*>(t + xrow0 * Rpad + r0 + 8 * q);
            *reinterpret_cast<uint4*>(xs + 128 * kPitch) = *reinterpret_cast<const uint4*>(t + xrow1 * Rpad + r0 + 8 * q);
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int rr = 4 * i + rr4;
                const int rg = r0 + rr;
                const uint16_t v = b_cat[(int64_t)(rg < R ? rg : R - 1) * N + bn];
                Ws[0][(tid & 127) * kPitch + (((i >> 1) ^ bf) << 3) + 4 * (i & 1) + rr4] = rg < R ? v : (uint16_t)0;
            }
            __syncthreads();
            mfma_step(0);
            __syncthreads();
        }
    }

    // ---- store: accumulator register e of a 32x32 tile holds row 8*(e/4) + 4*(lane/32) + e%4, column lane%32
    auto store_tile = [&](const f32x16& a, int i, int j) {
        const int64_t n = n0 + wn * 64 + 32 * j + (lane & 31);
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            const int64_t m = m0 + wm * 64 + 32 * i + 8 * (e >> 2) + 4 * (lane >> 5) + (e & 3);
            if (m < M && n < N) y[m * N + n] = f32_to_bf16_rne(a[e]);
        }
    };
    store_tile(acc00, 0, 0);
    store_tile(acc01, 0, 1);
    store_tile(acc10, 1, 0);
    store_tile(acc11, 1, 1);
}

hipError_t launch_linear_tiled(const LinearArgs& a, hipStream_t stream, const TimingEvents& ev) {
    const int R = (int)a.R, Rpad = (int)adapter_rank_padded(a.R);
    if (R > 0) launch_adapter_t(a, stream);
    const int m_tiles = (int)((a.M + kTM - 1) / kTM);
    const int n_tiles = (int)((a.N + kTN - 1) / kTN);
    const int n_groups = (n_tiles + kXcds - 1) / kXcds;
    const unsigned grid = (unsigned)(n_groups * m_tiles * kXcds);
    SALR_LAUNCH(linear_tiled_kernel, dim3(grid), dim3(kTiledThreads), stream, ev, a.x, a.M, a.K, a.N, a.bitmap, a.values,
                a.row_offsets, (const uint16_t*)a.t, a.b_cat, R, Rpad, a.y, m_tiles, n_tiles);
    return hipGetLastError();
}

}  // namespace salr
