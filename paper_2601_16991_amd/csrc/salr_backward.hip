// Backward pass of the SALR layer  Y = X What^T + (X A_cat) B_cat  (the layer of paper Sec. 3.2 / 3.3; fine-tuning,
// whose throughput Sec. 4 compares, runs it every step).  The pruned base weight is frozen, the adapters train:
//     dX = dY What + (dY B_cat^T) A_cat^T        [M, K]
//     dA = X^T (dY B_cat^T)                      [K, R]
//     dB = (X A_cat)^T dY                        [R, N]
// Everything is a product this library already has a kernel for, on operands laid out so that the contraction
// index is the contiguous one:
//     dX  the dense MFMA stage on dY and the TRANSPOSED decoded weight [K, N] (decoded straight into that layout when
//         K is a multiple of 128, else decode and a bf16 transpose), with
//         T' = dY B_cat^T [M, Rpad] and A_cat^T [Rpad, K] riding along as its adapter steps;
//     T' and T = X A_cat: the tall-product kernel of the adapter stage (B_cat's rows already run along N);
//     dA, dB: products that contract over the rows of X and dY: the row-contracting tall product (tall_tn_kernel), which
//         transposes its tiles of the large operand in LDS, against T'^T and T^T [Rpad, M].
// As in the forward pass T and T' are rounded to bf16 once; sums are fp32; outputs bf16.
#include "salr_device.hpp"
#include "salr_internal.hpp"
#include "salr_linear_common.hpp"

namespace salr {

// out [Rpad, N] = in [R, N] followed by zero rows
__global__ __launch_bounds__(256) void pad_rows_kernel(const uint16_t* __restrict__ in, int R, int64_t N,
                                                       uint16_t* __restrict__ out) {
    const int row = blockIdx.y;
    const int64_t c = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (c >= N) return;
    out[(int64_t)row * N + c] = row < R ? in[(int64_t)row * N + c] : (uint16_t)0;
}

// out [rows, R] (transposed == 0) or out [R, rows] (transposed == 1) = bf16 of the first R columns of
// sum over z < ksplit of partial[z] ([rows, Rpad] fp32), z ascending
__global__ __launch_bounds__(256) void reduce_columns_kernel(const float* __restrict__ partial, int64_t rows, int Rpad, int ksplit,
                                                             int R, int transposed, uint16_t* __restrict__ out) {
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= rows * R) return;
    // consecutive threads take consecutive output elements
    const int64_t row = transposed ? idx % rows : idx / R;
    const int r = (int)(transposed ? idx / rows : idx % R);
    float s = 0.f;
    for (int z = 0; z < ksplit; ++z) s += partial[((int64_t)z * rows + row) * Rpad + r];
    out[idx] = f32_to_bf16_rne(s);
}

struct BackwardPlan {
    int Rpad, ks_tp, ks_t, ks_da, ks_db, ks_y;
    size_t off_wd, off_wt, off_tp, off_at, off_bpad, off_tt, off_small_t, off_tpart, off_ypart, total;
};

static BackwardPlan backward_plan(int64_t M, int64_t K, int64_t N, int64_t R, bool want_dx, bool want_dadb) {
    BackwardPlan p{};
    p.Rpad = (int)adapter_rank_padded(R);
    p.ks_tp = adapter_ksplit(M, N);   // T' = dY B^T: rows M, contraction N
    p.ks_t = adapter_ksplit(M, K);    // T  = X A:     rows M, contraction K
    p.ks_da = tn_ksplit(K, M);        // dA: rows K, contraction M
    p.ks_db = tn_ksplit(N, M);        // dB: rows N, contraction M
    p.ks_y = want_dx ? dense_ksplit(M, N, K) : 1;
    size_t o = 0;
    auto take = [&](size_t bytes) { const size_t at = o; o += round_up_256(bytes); return at; };
    p.off_wd = take(want_dx ? (size_t)N * K * 2 : 0);
    p.off_wt = take(want_dx ? (size_t)N * K * 2 : 0);
    p.off_tp = take(R > 0 ? (size_t)M * p.Rpad * 2 : 0);
    p.off_at = take(R > 0 ? (size_t)K * p.Rpad * 2 : 0);
    p.off_bpad = take(R > 0 ? (size_t)N * p.Rpad * 2 : 0);
    const bool grads = want_dadb && R > 0;
    p.off_tt = take(grads ? (size_t)M * p.Rpad * 2 : 0);
    p.off_small_t = take(grads ? (size_t)2 * M * p.Rpad * 2 : 0);   // T^T and T'^T
    size_t part = 0;
    if (R > 0) {
        part = (size_t)p.ks_tp * M;
        if (grads) {
            const size_t c[3] = {(size_t)p.ks_t * M, (size_t)p.ks_da * K, (size_t)p.ks_db * N};
            for (size_t v : c) part = v > part ? v : part;
        }
    }
    p.off_tpart = take(part * p.Rpad * sizeof(float));
    p.off_ypart = take(p.ks_y > 1 ? (size_t)p.ks_y * M * K * sizeof(float) : 0);
    p.total = o;
    return p;
}

size_t linear_backward_workspace_bytes(int64_t M, int64_t K, int64_t N, int64_t R, bool want_dx, bool want_dadb) {
    return backward_plan(M, K, N, R, want_dx, want_dadb).total;
}

hipError_t launch_linear_backward(const uint16_t* x, const uint16_t* dy, int64_t M, int64_t K, int64_t N,
                                  const uint32_t* bitmap, const uint16_t* values, const uint32_t* row_offsets,
                                  const uint16_t* a_cat, const uint16_t* b_cat, int64_t R64, uint16_t* dx, uint16_t* da,
                                  uint16_t* db, void* workspace, hipStream_t stream) {
    const bool want_dx = dx != nullptr, want_dadb = (da != nullptr || db != nullptr);
    const BackwardPlan p = backward_plan(M, K, N, R64, want_dx, want_dadb);
    const int R = (int)R64, Rpad = p.Rpad;
    char* ws = static_cast<char*>(workspace);
    uint16_t* wd = reinterpret_cast<uint16_t*>(ws + p.off_wd);
    uint16_t* wt = reinterpret_cast<uint16_t*>(ws + p.off_wt);
    uint16_t* tp = reinterpret_cast<uint16_t*>(ws + p.off_tp);
    uint16_t* at = reinterpret_cast<uint16_t*>(ws + p.off_at);
    uint16_t* bpad = reinterpret_cast<uint16_t*>(ws + p.off_bpad);
    uint16_t* tt = reinterpret_cast<uint16_t*>(ws + p.off_tt);
    uint16_t* tt_t = reinterpret_cast<uint16_t*>(ws + p.off_small_t);
    uint16_t* tp_t = tt_t + (size_t)M * Rpad;
    float* tpart = reinterpret_cast<float*>(ws + p.off_tpart);
    float* ypart = reinterpret_cast<float*>(ws + p.off_ypart);

    if (R > 0) {   // T' = dY B_cat^T, needed by dX and dA
        hipLaunchKernelGGL(pad_rows_kernel, dim3((unsigned)((N + 255) / 256), (unsigned)Rpad), dim3(256), 0, stream, b_cat, R, N, bpad);
        launch_tall_product(dy, M, N, bpad, Rpad, p.ks_tp, tp, tpart, false, stream);
        if (p.ks_tp > 1) launch_splitk_reduce(tpart, M * Rpad, p.ks_tp, tp, stream);
        launch_adapter_transpose(a_cat, K, R, Rpad, at, stream);
    }
    if (want_dx) {
        hipError_t e;
        if (decode_transposed_takes(N, K, values, wt)) {   // straight into the transposed dense weight
            e = launch_decode_transposed(bitmap, values, row_offsets, N, K, wt, stream);
            if (e != hipSuccess) return e;
        } else {
            e = launch_decode(bitmap, values, row_offsets, N, K, wd, stream);
            if (e != hipSuccess) return e;
            launch_transpose_bf16(wd, N, K, wt, stream);
        }
        const TimingEvents none;
        launch_dense_stage(dy, M, N, K, wt, tp, at, R, Rpad, dx, ypart, none, stream);
    }
    if (want_dadb && R > 0) {
        if (da != nullptr) {   // dA = X^T T'
            launch_transpose_bf16(tp, M, Rpad, tp_t, stream);
            launch_tall_tn(x, M, K, tp_t, Rpad, p.ks_da, tpart, stream);
            hipLaunchKernelGGL(reduce_columns_kernel, dim3((unsigned)((K * R + 255) / 256)), dim3(256), 0, stream, tpart, K, Rpad,
                               p.ks_da, R, 0, da);
        }
        if (db != nullptr) {   // dB = T^T dY with T = X A_cat
            launch_tall_product(x, M, K, at, Rpad, p.ks_t, tt, tpart, false, stream);
            if (p.ks_t > 1) launch_splitk_reduce(tpart, M * Rpad, p.ks_t, tt, stream);
            launch_transpose_bf16(tt, M, Rpad, tt_t, stream);
            launch_tall_tn(dy, M, N, tt_t, Rpad, p.ks_db, tpart, stream);
            hipLaunchKernelGGL(reduce_columns_kernel, dim3((unsigned)((N * R + 255) / 256)), dim3(256), 0, stream, tpart, N, Rpad,
                               p.ks_db, R, 1, db);
        }
    }
    return hipGetLastError();
}

}  // namespace salr
