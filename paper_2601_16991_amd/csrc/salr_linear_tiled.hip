// Large-batch path of the SALR linear (M > 64): MFMA-bound, the two-stage pipeline of Sec. 3.3.
//
// Workgroup = 8 waves, output tile 256 (m) x 256 (n), k-step 32, everything double-buffered in LDS:
//
//   decode stage (all threads, for k-step s+1 while the MFMAs of step s run)
//       thread (row = tid/2, half = tid%2) owns one weight row of the tile and two byte masks of the
//       row's bitmap word.  Packed values arrive per 64-column chunk: each row's piece is contiguous in
//       `values`, is fetched by the row's two threads with 16-byte loads two chunks ahead, parked in the
//       row's LDS slot and expanded with the nibble rule (Sec. 3.3) into the dense LDS tile Ws.
//   MFMA stage
//       wave (wm, wn) owns 128 (m) x 64 (n): 4 x 2 tiles of v_mfma_f32_32x32x16_bf16, 128 accumulator
//       registers; A fragments from the X tile Xs, B fragments from Ws (row pitch 80 B: conflict-free
//       16-byte LDS reads for the 32-row operand layout).
//   adapters (Sec. 3.2): after the K loop the same accumulators take Rpad/32 more k-steps with
//       Xs := T (bf16, from adapter_t_mfma_kernel) and Ws := B_cat columns.
//
// Consecutive workgroup ids land on different XCDs (8 of them, each with its own L2); the id -> tile
// map keeps all m-tiles of one n-tile on the same XCD so the compressed rows are fetched into one L2.
#include "salr_device.hpp"
#include "salr_internal.hpp"
#include "salr_linear_common.hpp"

namespace salr {

constexpr int kTM = 256, kTN = 256, kTK = 32;
constexpr int kTiledThreads = 512;
constexpr int kPitch = kTK + 8;          // bf16 elements per LDS tile row (80 bytes)
constexpr int kSlotDw = 36;              // 9 vectors of 16 B: 64 values + misalignment
constexpr int kXcds = 8;

struct XPair {
    uint4 a, b;      // 16 bf16 of one X row
};

// One staged value chunk of a row lives in plain registers (named per ring slot): the thread's share of
// the piece (every second 16-byte vector), the piece's first vector, the index of its last vector, the
// element offset of the piece inside its first vector and its vector count.
#define SALR_VC_DECL(n) uint4 n##_q0, n##_q1, n##_q2; const uint4* n##_vb; uint32_t n##_last, n##_off, n##_nv
#define SALR_VC_ARGS(n) n##_q0, n##_q1, n##_q2, n##_vb, n##_last, n##_off, n##_nv

__global__ __launch_bounds__(kTiledThreads) void linear_tiled_kernel(
    const uint16_t* __restrict__ x, int64_t M, int64_t K, int64_t N, const uint32_t* __restrict__ bitmap,
    const uint16_t* __restrict__ values, const uint32_t* __restrict__ row_offsets, const uint16_t* __restrict__ t,
    const uint16_t* __restrict__ b_cat, int R, int Rpad, uint16_t* __restrict__ y, int m_tiles, int n_tiles) {
    __shared__ __attribute__((aligned(16))) uint16_t Xs[2][kTM * kPitch];
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
    const int wm = wave >> 2, wn = wave & 3;

    nibble_lut_init(lut);

    // ---- loader / decoder role: row r of the tile, half h
    const int r = tid >> 1, h = tid & 1;
    const int64_t xrow = (m0 + r < M) ? m0 + r : M - 1;   // rows past the edge recompute the last row; never stored
    const int64_t wrow = (n0 + r < N) ? n0 + r : N - 1;
    const uint16_t* xptr = x + xrow * K + 16 * h;
    const int64_t wpr = K >> 5;
    const uint32_t* brow = bitmap + wrow * wpr;
    const uint4* values128 = reinterpret_cast<const uint4*>(values);
    uint32_t* slot = stage + r * kSlotDw;
    uint32_t cur = row_offsets[wrow];  // element index in `values` of the row's next unfetched value
    const int64_t steps = K / kTK;
    const int64_t supers = steps / 4;   // K % 128 == 0 on this path

    auto load_bitmap = [&](int64_t q) -> uint4 {
        return (q < supers) ? *reinterpret_cast<const uint4*>(brow + 4 * q) : make_uint4(0, 0, 0, 0);
    };
    auto load_x = [&](int64_t s) -> XPair {
        const int64_t sc = s < steps ? s : steps - 1;  // past the end: reload the last step (unused)
        const uint4* p = reinterpret_cast<const uint4*>(xptr + sc * kTK);
        XPair v;
        v.a = p[0];
        v.b = p[1];
        return v;
    };
    auto store_x = [&](int buf, const XPair src) {
        uint4* p = reinterpret_cast<uint4*>(&Xs[buf][r * kPitch + 16 * h]);
        p[0] = src.a;
        p[1] = src.b;
    };
    // request the packed values of the next chunk of this row (bitmap words w0, w1)
    auto v_issue = [&](uint4& q0, uint4& q1, uint4& q2, const uint4*& vb, uint32_t& last, uint32_t& off, uint32_t& nv,
                       uint32_t w0, uint32_t w1) {
        const uint32_t len = __popc(w0) + __popc(w1);
        off = cur & 7u;
        nv = len ? (off + len + 7u) >> 3 : 0u;
        vb = nv ? values128 + (cur >> 3) : reinterpret_cast<const uint4*>(x);
        last = nv ? nv - 1u : 0u;
        cur += len;
        // clamped, not predicated: the three requests go out back to back.  Vectors 6..8 exist only in
        // pieces denser than ~70 %; v_store fetches them on the spot.
        q0 = vb[h < last ? h : last];
        q1 = vb[h + 2 < last ? h + 2 : last];
        q2 = vb[h + 4 < last ? h + 4 : last];
    };
    uint32_t c_local = 0;  // cursor inside the slot
    // park the chunk in the row's LDS slot (only the row's own two threads ever touch the slot)
    auto v_store = [&](const uint4& q0, const uint4& q1, const uint4& q2, const uint4* vb, uint32_t last, uint32_t off,
                       uint32_t nv) {
        uint4* sv = reinterpret_cast<uint4*>(slot);
        sv[h] = q0;
        sv[h + 2] = q1;
        sv[h + 4] = q2;
        if (__builtin_amdgcn_ballot_w64(nv > 6u)) {  // rare, wave-uniform
            sv[h + 6] = vb[h + 6 < last ? h + 6 : last];
            if (h == 0) sv[8] = vb[8u < last ? 8u : last];  // the slot holds 9 vectors
        }
        __builtin_amdgcn_wave_barrier();
        c_local = off;  // the slot's cursor restarts at the piece's offset
    };
    // expand this thread's two byte masks of `word` into Ws[buf]
    auto decode = [&](int buf, uint32_t word) {
        const uint32_t half = (word >> (16 * h)) & 0xFFFFu;
        const uint32_t cb = c_local + (h ? __popc(word & 0xFFFFu) : 0u);
        const uint32_t ma = half & 0xFFu, mb = half >> 8;
        const uint4 qa = expand_byte(slot, lut, cb, ma);
        const uint4 qb = expand_byte(slot, lut, cb + __popc(ma), mb);
        c_local += __popc(word);
        uint4* p = reinterpret_cast<uint4*>(&Ws[buf][r * kPitch + 16 * h]);
        p[0] = qa;
        p[1] = qb;
    };

    f32x16 acc00 = {0}, acc01 = {0}, acc10 = {0}, acc11 = {0}, acc20 = {0}, acc21 = {0}, acc30 = {0}, acc31 = {0};

    const int frag_row = lane & 31, frag_k = 8 * (lane >> 5);
    auto mfma_step = [&](int buf) {
        const uint16_t* xa = &Xs[buf][(wm * 128 + frag_row) * kPitch + frag_k];
        const uint16_t* wb = &Ws[buf][(wn * 64 + frag_row) * kPitch + frag_k];
        auto frag = [](const uint16_t* p) { return *reinterpret_cast<const bf16x8*>(p); };
        // all twelve 16-byte fragment reads of the step are in flight before the first MFMA issues
        const bf16x8 a00 = frag(xa), a10 = frag(xa + 32 * kPitch), a20 = frag(xa + 64 * kPitch), a30 = frag(xa + 96 * kPitch);
        const bf16x8 b00 = frag(wb), b10 = frag(wb + 32 * kPitch);
        const bf16x8 a01 = frag(xa + 16), a11 = frag(xa + 32 * kPitch + 16), a21 = frag(xa + 64 * kPitch + 16),
                     a31 = frag(xa + 96 * kPitch + 16);
        const bf16x8 b01 = frag(wb + 16), b11 = frag(wb + 32 * kPitch + 16);
        acc00 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a00, b00, acc00, 0, 0, 0);
        acc01 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a00, b10, acc01, 0, 0, 0);
        acc10 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a10, b00, acc10, 0, 0, 0);
        acc11 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a10, b10, acc11, 0, 0, 0);
        acc20 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a20, b00, acc20, 0, 0, 0);
        acc21 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a20, b10, acc21, 0, 0, 0);
        acc30 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a30, b00, acc30, 0, 0, 0);
        acc31 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a30, b10, acc31, 0, 0, 0);
        acc00 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a01, b01, acc00, 0, 0, 0);
        acc01 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a01, b11, acc01, 0, 0, 0);
        acc10 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a11, b01, acc10, 0, 0, 0);
        acc11 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a11, b11, acc11, 0, 0, 0);
        acc20 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a21, b01, acc20, 0, 0, 0);
        acc21 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a21, b11, acc21, 0, 0, 0);
        acc30 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a31, b01, acc30, 0, 0, 0);
        acc31 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a31, b11, acc31, 0, 0, 0);
    };

    // ---- prologue: bitmap of 3 super-steps, values of chunks 0 and 1, X of steps 0..2, tile 0 decoded
    uint4 bm0 = load_bitmap(0), bm1 = load_bitmap(1), bm2 = load_bitmap(2);
    XPair xr0 = load_x(0), xr1;
    SALR_VC_DECL(vc0);
    SALR_VC_DECL(vc1);
    v_issue(SALR_VC_ARGS(vc0), bm0.x, bm0.y);
    v_issue(SALR_VC_ARGS(vc1), bm0.z, bm0.w);
    __syncthreads();  // lut
    store_x(0, xr0);
    xr1 = load_x(1);
    xr0 = load_x(2);
    v_store(SALR_VC_ARGS(vc0));
    decode(0, bm0.x);
    v_issue(SALR_VC_ARGS(vc0), bm1.x, bm1.y);  // chunk 2
    __syncthreads();

    // ---- main loop: one super-step (4 k-steps, 2 value chunks, one bitmap vector) per iteration.
    // Within a k-step the MFMAs read buffer s%2 while the loaders fill buffer (s+1)%2, so the two halves
    // may run in either order: waves 0-3 fill first, waves 4-7 multiply first.  Waves w and w+4 share a
    // SIMD, so on every SIMD one wave's decode overlaps the other wave's MFMAs.
    const bool fill_first = wave < 4;
    for (int64_t q = 0; q < supers; ++q) {
        const int64_t s0 = 4 * q;
        // step s0 (tile in buffer 0): decode tile s0+1 from chunk 2q, word 1
        if (!fill_first) mfma_step(0);
        store_x(1, xr1);
        xr1 = load_x(s0 + 3);
        decode(1, bm0.y);
        if (fill_first) mfma_step(0);
        __syncthreads();
        // step s0+1 (buffer 1): chunk 2q+1 becomes current; decode tile s0+2, word 2; request chunk 2q+3
        if (!fill_first) mfma_step(1);
        store_x(0, xr0);
        xr0 = load_x(s0 + 4);
        v_store(SALR_VC_ARGS(vc1));
        decode(0, bm0.z);
        v_issue(SALR_VC_ARGS(vc1), bm1.z, bm1.w);
        if (fill_first) mfma_step(1);
        __syncthreads();
        // step s0+2 (buffer 0): decode tile s0+3, word 3
        if (!fill_first) mfma_step(0);
        store_x(1, xr1);
        xr1 = load_x(s0 + 5);
        decode(1, bm0.w);
        if (fill_first) mfma_step(0);
        __syncthreads();
        // step s0+3 (buffer 1): chunk 2q+2 becomes current; decode tile s0+4 (word 0 of the next super-step);
        // request chunk 2q+4; rotate the bitmap ring
        if (!fill_first) mfma_step(1);
        store_x(0, xr0);
        xr0 = load_x(s0 + 6);
        v_store(SALR_VC_ARGS(vc0));
        decode(0, bm1.x);
        v_issue(SALR_VC_ARGS(vc0), bm2.x, bm2.y);
        bm0 = bm1;
        bm1 = bm2;
        bm2 = load_bitmap(q + 3);
        if (fill_first) mfma_step(1);
        __syncthreads();
    }

    // ---- adapter k-steps (Sec. 3.2): Xs := T[m, r0 .. r0+31], Ws := B_cat[r0 .. r0+31, n]
    if (R > 0) {
        const int64_t bn = (n0 + (tid & 255) < N) ? n0 + (tid & 255) : N - 1;
        const int rr2 = tid >> 8;
        for (int r0 = 0; r0 < Rpad; r0 += kTK) {
            const uint4* tp = reinterpret_cast<const uint4*>(t + xrow * Rpad + r0 + 16 * h);
            XPair tq;
            tq.a = tp[0];
            tq.b = tp[1];
            store_x(0, tq);
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int rr = 2 * i + rr2;
                const int rg = r0 + rr;
                const uint16_t v = b_cat[(int64_t)(rg < R ? rg : R - 1) * N + bn];
                Ws[0][(tid & 255) * kPitch + rr] = rg < R ? v : (uint16_t)0;
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
            const int64_t m = m0 + wm * 128 + 32 * i + 8 * (e >> 2) + 4 * (lane >> 5) + (e & 3);
            if (m < M && n < N) y[m * N + n] = f32_to_bf16_rne(a[e]);
        }
    };
    store_tile(acc00, 0, 0);
    store_tile(acc01, 0, 1);
    store_tile(acc10, 1, 0);
    store_tile(acc11, 1, 1);
    store_tile(acc20, 2, 0);
    store_tile(acc21, 2, 1);
    store_tile(acc30, 3, 0);
    store_tile(acc31, 3, 1);
}

// ---------------------------------------------------------------------------------------------------
// T = X * A_cat for the tiled path (Sec. 3.2, first concatenated GEMM): workgroup (m-block of 64 rows,
// rank tile of 16 columns), 4 waves split K, 16x16x32 bf16 MFMAs, LDS reduction, bf16 output
// [M, Rpad] with zero padding columns.
// ---------------------------------------------------------------------------------------------------
constexpr int kTmWaves = 16;

__global__ __launch_bounds__(kTmWaves * 64) void adapter_t_mfma_kernel(const uint16_t* __restrict__ x, int64_t M, int64_t K,
                                                                       const uint16_t* __restrict__ a_cat, int R, int Rpad,
                                                                       uint16_t* __restrict__ t) {
    __shared__ float red[kTmWaves][4][4][64];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int i16 = lane & 15, g = lane >> 4;
    const int64_t m0 = (int64_t)blockIdx.x * 64;
    const int rt = blockIdx.y;
    const int rc = 16 * rt + i16 < R ? 16 * rt + i16 : R - 1;
    const int64_t units = K >> 5;
    f32x4 acc[4];
#pragma unroll
    for (int mt = 0; mt < 4; ++mt) acc[mt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll 4
    for (int64_t u = wave; u < units; u += kTmWaves) {
        const int64_t k0 = (u << 5) + 8 * g;
        uint32_t e[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) e[j] = a_cat[(k0 + j) * R + rc];
        const uint4 bq = make_uint4(e[0] | (e[1] << 16), e[2] | (e[3] << 16), e[4] | (e[5] << 16), e[6] | (e[7] << 16));
#pragma unroll
        for (int mt = 0; mt < 4; ++mt) {
            const int64_t m = m0 + 16 * mt + i16;
            const uint4 aq = *reinterpret_cast<const uint4*>(x + (m < M ? m : M - 1) * K + k0);
            acc[mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(aq), as_bf16x8(bq), acc[mt], 0, 0, 0);
        }
    }
#pragma unroll
    for (int mt = 0; mt < 4; ++mt)
#pragma unroll
        for (int e = 0; e < 4; ++e) red[wave][mt][e][lane] = acc[mt][e];
    __syncthreads();
    for (int idx = threadIdx.x; idx < 1024; idx += kTmWaves * 64) {
        const int l = idx & 63, e = (idx >> 6) & 3, mt = idx >> 8;
        float s = 0.f;
#pragma unroll
        for (int w = 0; w < kTmWaves; ++w) s += red[w][mt][e][l];
        const int64_t m = m0 + 16 * mt + 4 * (l >> 4) + e;
        const int rr = 16 * rt + (l & 15);
        if (m < M) t[m * Rpad + rr] = rr < R ? f32_to_bf16_rne(s) : (uint16_t)0;
    }
}

hipError_t launch_linear_tiled(const LinearArgs& a, hipStream_t stream, const TimingEvents& ev) {
    const int R = (int)a.R, Rpad = (int)adapter_rank_padded(a.R);
    if (R > 0)
        hipLaunchKernelGGL(adapter_t_mfma_kernel, dim3((unsigned)((a.M + 63) / 64), Rpad / 16), dim3(kTmWaves * 64), 0, stream,
                           a.x, a.M, a.K, a.a_cat, R, Rpad, a.t);
    const int m_tiles = (int)((a.M + kTM - 1) / kTM);
    const int n_tiles = (int)((a.N + kTN - 1) / kTN);
    const int n_groups = (n_tiles + kXcds - 1) / kXcds;
    const unsigned grid = (unsigned)(n_groups * m_tiles * kXcds);
    SALR_LAUNCH(linear_tiled_kernel, dim3(grid), dim3(kTiledThreads), stream, ev, a.x, a.M, a.K, a.N, a.bitmap, a.values,
                a.row_offsets, (const uint16_t*)a.t, a.b_cat, R, Rpad, a.y, m_tiles, n_tiles);
    return hipGetLastError();
}

}  // namespace salr
