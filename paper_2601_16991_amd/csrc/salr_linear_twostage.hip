// Large-batch path of the SALR linear (M > 64): the two stages of Sec. 3.3 ("Pipeline Design") as two kernels.
//
//   stage 1  bitmap decode of the whole weight into a dense bf16 scratch matrix (the decode kernel of the codec,
//            once per call: a kernel that decodes into LDS tiles next to its MFMAs repeats the decode for every
//            256-row block of X and was slower at every M > 64, see below);
//   stage 2  dense_gemm_kernel: Y = X * Wd^T (+ T * B_cat, Sec. 3.2) on the matrix cores.
//
// dense_gemm_kernel: output tile 256 (m) x 64 kWN (n); wave (wm, wn) owns 32 kMI x 64 = kMI x 2 tiles of
// v_mfma_f32_32x32x16_bf16 (128 x 64 per wave, 8 waves, on 256 x 256 tiles; 64 x 64 on 256 x 128 tiles when the
// wide ones would not fill the chip).  A k-step is 64 wide so that every row of a tile is one whole 128-byte line: at 64
// bytes per row the L2 sees twice the requests for the same bytes and its request rate, not its bandwidth,
// limits the kernel.  Both operand tiles travel from memory straight into LDS (global_load_lds, 16 bytes per
// lane, no registers, no VALU) into a ring of kStages stages; one barrier per step, in its middle, publishes the
// stage that is multiplied next and retires the one read last.  LDS rows are 128 bytes, swizzled (segment s of row r at
// s ^ ((r >> 1) & 7)) so that operand reads are conflict-free; a load instruction of a wave fills 8 consecutive
// rows, lane l landing on 16-byte slot l, so lane l fetches the segment that belongs there.
#include "salr_device.hpp"
#include "salr_internal.hpp"
#include "salr_linear_common.hpp"

namespace salr {

constexpr int kDM = 256, kDK = 64;
constexpr int kDXcds = 8;

// segment (16 bytes = 8 bf16) position of logical segment `seg` in LDS row `row`, in elements
__device__ __forceinline__ int dswz(int row, int seg) { return (seg ^ ((row >> 1) & 7)) * 8; }

// Output tile 256 x (32 kNI kWN); wave (wm, wn) owns 32 kMI rows x 32 kNI columns, so there are (8 / kMI) kWN
// waves, always 8 here (2 per SIMD, which leaves room in the registers to fetch the operands of the next 16 k
// while the current ones are multiplied):
//   <4, 2, 4>  256 x 256 tile, 128 x 64 per wave;   <1, 7, 1>  256 x 224 tile, 32 x 224 per wave (for N where
//   224-wide tiles fill whole rounds of the 256 CUs and 256-wide ones do not);   <2, 2, 2>  256 x 128 tile.
// K % 64 == 0.
template <int kMI, int kNI, int kWN, int kStages>
__global__ __launch_bounds__(64 * (8 / kMI) * kWN, (8 / kMI) * kWN / 4) void dense_gemm_kernel(
    const uint16_t* __restrict__ x, int64_t M, int64_t K, int64_t N, const uint16_t* __restrict__ wd,
    const uint16_t* __restrict__ t, const uint16_t* __restrict__ b_cat, int R, int Rpad, uint16_t* __restrict__ y,
    int m_tiles, int n_tiles, int ksplit, float* __restrict__ partial) {
    constexpr int kDN = 32 * kNI * kWN;
    constexpr int kWaves = (8 / kMI) * kWN;
    constexpr int kXLoads = kDM / (8 * kWaves);                 // load instructions per wave and step for the X tile (8 rows each)
    constexpr int kWLoads = (kDN + 8 * kWaves - 1) / (8 * kWaves);   // ... and for the W tile; the last one may be partial
    constexpr bool kWRagged = kDN % (8 * kWaves) != 0;          // only the first waves take part in the last W load
    constexpr int kLoads = kXLoads + kWLoads;
    static_assert(kDM % (8 * kWaves) == 0 && kDN % 8 == 0, "tile/wave shape");
    static_assert(!kWRagged || kStages == 2, "a partial load makes the in-flight count differ between waves: wait for all");
    __shared__ __attribute__((aligned(16))) uint16_t Xs[kStages][kDM * kDK];
    __shared__ __attribute__((aligned(16))) uint16_t Ws[kStages][kDN * kDK];

    // consecutive workgroup ids land on different XCDs; all m-tiles of an n-tile stay on one XCD (one L2)
    const int bid = blockIdx.x;
    const int xcd = bid % kDXcds, local = bid / kDXcds;
    const int nt = (local / m_tiles) * kDXcds + xcd;
    const int mt = local % m_tiles;
    if (nt >= n_tiles) return;  // uniform for the workgroup, before any barrier
    const int64_t m0 = (int64_t)mt * kDM, n0 = (int64_t)nt * kDN;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / kWN, wn = wave % kWN;

    // split K: workgroup z = blockIdx.y multiplies k-steps [z, z + 1) * steps of its tile and leaves an fp32
    // partial tile in partial[z]; splitk_reduce_kernel adds them up.  The adapters ride with z = 0.
    const int kz = blockIdx.y;
    const int64_t steps = K / kDK / ksplit;
    const int64_t k_first = kz * steps * kDK;

    // loader role: load j of wave w fills tile rows 8 (w + kWaves j) .. + 7; lane l lands on slot l % 8 of row l / 8
    const int lrow = 8 * wave + (lane >> 3);          // row of load 0; load j is 8 kWaves j rows further down
    const int lseg = (lane & 7) ^ ((lrow >> 1) & 7);  // logical segment stored in the lane's slot (same for all j)
    const uint16_t* xptr[kXLoads];
    const uint16_t* wptr[kWLoads];
#pragma unroll
    for (int j = 0; j < kXLoads; ++j) {
        const int64_t row = m0 + lrow + 8 * kWaves * j;
        xptr[j] = x + (row < M ? row : M - 1) * K + k_first + 8 * lseg;  // rows past the edge repeat the last row; never stored
    }
#pragma unroll
    for (int j = 0; j < kWLoads; ++j) {
        const int64_t row = n0 + lrow + 8 * kWaves * j;
        wptr[j] = wd + (row < N ? row : N - 1) * K + k_first + 8 * lseg;
    }

    // One 16-byte-per-lane load from memory straight into LDS: lane l of the wave lands on lds_base + 16 l.
    // Written as assembly so that the waits stay under this kernel's control (vmcnt below): handed to the
    // compiler as a builtin, every barrier of the loop would wait for ALL requests, also the newest ones.
    auto load_to_lds = [&](const uint16_t* src, uint16_t* lds_base) {
        const uint32_t lds_off = __builtin_amdgcn_readfirstlane(
            (uint32_t)(uintptr_t)(__attribute__((address_space(3))) void*)lds_base);
        asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off"
                     :
                     : "v"(src), "s"(lds_off)
                     : "memory", "m0");
    };
    auto fetch = [&](uint16_t* xs, uint16_t* ws, int64_t s) {
        const int64_t sc = s < steps ? s : steps - 1;  // past the end: reload the last step (unused)
#pragma unroll
        for (int j = 0; j < kXLoads; ++j) load_to_lds(xptr[j] + sc * kDK, xs + (8 * wave + 8 * kWaves * j) * kDK);
#pragma unroll
        for (int j = 0; j < kWLoads; ++j) {
            if (!kWRagged || j + 1 < kWLoads || 8 * (wave + kWaves * j) < kDN)   // wave-uniform
                load_to_lds(wptr[j] + sc * kDK, ws + (8 * wave + 8 * kWaves * j) * kDK);
        }
    };
    // the requests of the newest kStages - 2 steps may stay in flight, everything older has landed
    static_assert((kStages - 2) * kLoads <= 15, "vmcnt immediate");
    static_assert(kStages >= 2, "the stage that is read and the one that lands are different ones");
    auto older_landed = [&]() { __builtin_amdgcn_s_waitcnt(0x0F70 | ((kStages - 2) * kLoads)); };

    f32x16 acc[kMI][kNI];
#pragma unroll
    for (int i = 0; i < kMI; ++i)
#pragma unroll
        for (int j = 0; j < kNI; ++j) acc[i][j] = f32x16{0};
    // operand lane: row lane % 32 of a 32-row block, segment 2 j + lane / 32 in sub-step j (16 of the 64 k);
    // rows 32 or 64 further down share the swizzle term
    const int frag_row = lane & 31;
    const int fsw = (frag_row >> 1) & 7, fhalf = lane >> 5;
    struct Frags {
        bf16x8 a[kMI], b[kNI];
    };
    auto load_frags = [&](const uint16_t* xa, const uint16_t* wb, int j) -> Frags {
        const int fk = ((2 * j + fhalf) ^ fsw) * 8;
        Frags f;
#pragma unroll
        for (int i = 0; i < kMI; ++i) f.a[i] = *reinterpret_cast<const bf16x8*>(xa + 32 * i * kDK + fk);
#pragma unroll
        for (int j = 0; j < kNI; ++j) f.b[j] = *reinterpret_cast<const bf16x8*>(wb + 32 * j * kDK + fk);
        return f;
    };
    auto multiply = [&](const Frags& f) {
#pragma unroll
        for (int i = 0; i < kMI; ++i)
#pragma unroll
            for (int j = 0; j < kNI; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.a[i], f.b[j], acc[i][j], 0, 0, 0);
    };
    // one k-step of 32 (two sub-steps) on stage 0: the shape of an adapter step
    auto rank_step = [&]() {
        const uint16_t* xa = Xs[0] + (wm * 32 * kMI + frag_row) * kDK;
        const uint16_t* wb = Ws[0] + (wn * 32 * kNI + frag_row) * kDK;
        const Frags r0 = load_frags(xa, wb, 0);
        const Frags r1 = load_frags(xa, wb, 1);
        multiply(r0);
        multiply(r1);
    };

    // ---- k loop.  The ring holds steps s .. s + kStages - 1.  The one barrier of a step sits in its middle, after
    // the last operand read of stage `cur`: it retires that stage (refilled at once with step s + kStages) and
    // publishes stage `nxt`, whose first operands are then requested under the MFMAs of the step's second half, so
    // that no wave starts a step with an empty matrix pipe.
    // Operands are requested one sub-step before they are multiplied.  The scheduling fences keep the compiler from
    // sinking the reads down to their first use, where every one of them would be waited for with nothing else to
    // issue (only where three sets of operands fit into the registers beside the accumulators).
    constexpr bool kFenced = kMI * kNI * 16 + 12 * (kMI + kNI) <= 200;
    auto fence = [&]() {
        if constexpr (kFenced) __builtin_amdgcn_sched_barrier(0);
    };
    for (int p = 0; p < kStages; ++p) fetch(Xs[p], Ws[p], p);
    // step 0 has landed (a count of requests allowed in flight only where every wave issues the same number)
    __builtin_amdgcn_s_waitcnt(0x0F70 | ((kWRagged || (kStages - 1) * kLoads > 15) ? 0 : (kStages - 1) * kLoads));
    __syncthreads();
    const uint16_t* xa0 = Xs[0] + (wm * 32 * kMI + frag_row) * kDK;
    const uint16_t* wb0 = Ws[0] + (wn * 32 * kNI + frag_row) * kDK;
    Frags f0 = load_frags(xa0, wb0, 0);
    Frags f1 = load_frags(xa0, wb0, 1);
    int cur = 0, nxt = 1;
    for (int64_t s = 0; s < steps; ++s) {
        const uint16_t* xa = Xs[cur] + (wm * 32 * kMI + frag_row) * kDK;
        const uint16_t* wb = Ws[cur] + (wn * 32 * kNI + frag_row) * kDK;
        const uint16_t* xn = Xs[nxt] + (wm * 32 * kMI + frag_row) * kDK;
        const uint16_t* wn_ = Ws[nxt] + (wn * 32 * kNI + frag_row) * kDK;
        const Frags f2 = load_frags(xa, wb, 2);
        fence();
        multiply(f0);
        fence();
        const Frags f3 = load_frags(xa, wb, 3);
        fence();
        multiply(f1);
        fence();
        older_landed();    // this wave's requests for step s + 1 have landed
        __syncthreads();   // ... and everybody's; every wave has read all it needs of stage `cur`
        fetch(Xs[cur], Ws[cur], s + kStages);
        f0 = load_frags(xn, wn_, 0);
        fence();
        multiply(f2);
        fence();
        f1 = load_frags(xn, wn_, 1);
        fence();
        multiply(f3);
        fence();
        cur = nxt;
        nxt = nxt + 1 == kStages ? 0 : nxt + 1;
    }
    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): no request may land after this point
    __syncthreads();

    // ---- adapter k-steps of 32 (Sec. 3.2): Xs[0] := T[m, r0 .. r0+31], Ws[0] := B_cat[r0 .. r0+31, n] (transposed),
    // both in segments 0..3 of the rows
    if (R > 0 && kz == 0) {
        const int trow = tid >> 2, tseg = tid & 3; // T: four threads per row, 256 tile rows in 256 / (kWaves 16) passes
        for (int r0 = 0; r0 < Rpad; r0 += 32) {
#pragma unroll
            for (int j = 0; j < kDM / (16 * kWaves); ++j) {
                const int row = trow + 16 * kWaves * j;
                const int64_t m = (m0 + row < M) ? m0 + row : M - 1;
                *reinterpret_cast<uint4*>(&Xs[0][row * kDK + dswz(row, tseg)]) =
                    *reinterpret_cast<const uint4*>(t + m * Rpad + r0 + 8 * tseg);
            }
            // element (rank row rr, output column bcol) of the 32 x kDN block: consecutive threads take consecutive columns
            for (int idx = tid; idx < 32 * kDN; idx += 64 * kWaves) {
                const int rr = idx / kDN, bcol = idx % kDN;   // segment rr / 8, element rr % 8 of tile row bcol
                const int rg = r0 + rr;
                const int64_t bn = (n0 + bcol < N) ? n0 + bcol : N - 1;
                const uint16_t v = b_cat[(int64_t)(rg < R ? rg : R - 1) * N + bn];
                Ws[0][bcol * kDK + dswz(bcol, rr >> 3) + (rr & 7)] = rg < R ? v : (uint16_t)0;
            }
            __syncthreads();
            rank_step();
            __syncthreads();
        }
    }

    // ---- store: accumulator register e of a 32x32 tile holds row 8*(e/4) + 4*(lane/32) + e%4, column lane%32
#pragma unroll
    for (int i = 0; i < kMI; ++i)
#pragma unroll
        for (int j = 0; j < kNI; ++j) {
            const int64_t n = n0 + wn * 32 * kNI + 32 * j + (lane & 31);
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int64_t m = m0 + wm * 32 * kMI + 32 * i + 8 * (e >> 2) + 4 * (lane >> 5) + (e & 3);
                if (m < M && n < N) {
                    if (ksplit == 1) y[m * N + n] = f32_to_bf16_rne(acc[i][j][e]);
                    else partial[((int64_t)kz * M + m) * N + n] = acc[i][j][e];
                }
            }
        }
}

void launch_dense_stage(const uint16_t* x, int64_t M, int64_t K, int64_t N, const uint16_t* wd, const uint16_t* t,
                        const uint16_t* b_cat, int R, int Rpad, uint16_t* y, float* partial, const TimingEvents& ev,
                        hipStream_t stream) {
    const int m_tiles = (int)((M + kDM - 1) / kDM);
    // Tile width: 256 or 224 columns, whichever needs less time in whole rounds of the 256 CUs (one workgroup per
    // CU, so a round costs its tile width); 128, with K split over workgroups if need be, when neither fills the chip.
    const int64_t t256 = (int64_t)m_tiles * ((N + 255) / 256), t224 = (int64_t)m_tiles * ((N + 223) / 224);
    const int64_t cost256 = (t256 + 255) / 256 * 256, cost224 = (t224 + 255) / 256 * 224;
    const int tn = t256 < 224 ? 128 : (cost224 < cost256 ? 224 : 256);
    const int n_tiles = (int)((N + tn - 1) / tn);
    const int n_groups = (n_tiles + kDXcds - 1) / kDXcds;
    const int ksplit = tn == 128 ? dense_ksplit(M, K, N) : 1;
    const dim3 grid((unsigned)(n_groups * m_tiles * kDXcds), (unsigned)ksplit);
    if (tn == 256)
        SALR_LAUNCH((dense_gemm_kernel<4, 2, 4, 2>), grid, dim3(512), stream, ev, x, M, K, N, wd, t, b_cat, R, Rpad, y, m_tiles,
                    n_tiles, ksplit, partial);
    else if (tn == 224)
        SALR_LAUNCH((dense_gemm_kernel<1, 7, 1, 2>), grid, dim3(512), stream, ev, x, M, K, N, wd, t, b_cat, R, Rpad, y, m_tiles,
                    n_tiles, ksplit, partial);
    else
        SALR_LAUNCH((dense_gemm_kernel<2, 2, 2, 3>), grid, dim3(512), stream, ev, x, M, K, N, wd, t, b_cat, R, Rpad, y, m_tiles,
                    n_tiles, ksplit, partial);
    if (ksplit > 1) launch_splitk_reduce(partial, M * N, ksplit, y, stream);
}

hipError_t launch_linear_twostage(const LinearArgs& a, hipStream_t stream, const TimingEvents& ev) {
    const int R = (int)a.R, Rpad = (int)adapter_rank_padded(a.R);
    uint16_t* wd = reinterpret_cast<uint16_t*>(reinterpret_cast<char*>(a.t) + twostage_dense_offset(a.M, a.K, a.R));
    hipError_t e = a.codes != nullptr
                       ? launch_decode_nf4(a.bitmap, a.codes, a.scales, a.nnz, a.row_offsets, a.N, a.K, wd, stream)
                       : launch_decode(a.bitmap, a.values, a.row_offsets, a.N, a.K, wd, stream);
    if (e != hipSuccess) return e;
    if (R > 0) launch_adapter_t(a, stream);
    float* partial = reinterpret_cast<float*>(reinterpret_cast<char*>(wd) + round_up_256((size_t)a.N * (size_t)a.K * sizeof(uint16_t)));
    launch_dense_stage(a.x, a.M, a.K, a.N, wd, a.t, a.b_cat, R, Rpad, a.y, partial, ev, stream);
    return hipGetLastError();
}

}  // namespace salr
