// Residual adapter (paper Sec. 3.1, "Sparsity Preservation Pruning"): factors A_res [K, r], B_res [r, N] of the best
// rank-r approximation of the residual E [N, K], so that (A_res B_res)^T ~ E_r.
//
// The paper asks for the truncated SVD of E and names no algorithm.  Here: randomized subspace iteration with a
// caller-supplied Gaussian test matrix Omega [K, l], l = r + oversample (a published method: range finder with power
// iterations, then the SVD of the small projected matrix).  With L = l rounded up to 16:
//     Y = E Omega;  Q = orth(Y);   q times { Z = E^T Q;  Z = orth(Z);  Y = E Z;  Q = orth(Y) };   Z = E^T Q
//     Z^T Z = U~ diag(s^2) U~^T  (l x l, Jacobi);   A_res = Z U~_r s_r^{-1/2},   B_res = s_r^{1/2} (Q U~_r)^T
// (E ~ Q Q^T E = Q Z^T, and Z = V~ S U~^T gives E ~ (Q U~) S V~^T.)
//
// Kernels: the two big products stream E (or its transposed copy) once each through launch_tall_product, the MFMA
// kernel of the adapter stage, with the fp32 matrix on the other side split into bf16 high and low parts (2 L
// columns, added up again by fold_reduce_kernel); orth = CholeskyQR twice (gram_partial_kernel, chol_inverse_kernel,
// apply_kernel); the l x l eigenproblem runs in one workgroup (eig_kernel).  Everything small is fp32.
#include "salr_device.hpp"
#include "salr_internal.hpp"
#include "salr_linear_common.hpp"

namespace salr {

// out [C, R] = in [R, C]^T, bf16, 32 x 32 tiles through LDS
__global__ __launch_bounds__(256) void transpose_bf16_kernel(const uint16_t* __restrict__ in, int64_t R, int64_t C,
                                                             uint16_t* __restrict__ out) {
    __shared__ uint16_t tile[32][33];
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
    const int64_t c0 = (int64_t)blockIdx.x * 32, r0 = (int64_t)blockIdx.y * 32;
    for (int i = ty; i < 32; i += 8)
        if (r0 + i < R && c0 + tx < C) tile[i][tx] = in[(r0 + i) * C + c0 + tx];
    __syncthreads();
    for (int i = ty; i < 32; i += 8)
        if (c0 + i < C && r0 + tx < R) out[(c0 + i) * R + r0 + tx] = tile[tx][i];
}

void launch_transpose_bf16(const uint16_t* in, int64_t R, int64_t C, uint16_t* out, hipStream_t stream) {
    if (R == 0 || C == 0) return;
    hipLaunchKernelGGL(transpose_bf16_kernel, dim3((unsigned)((C + 31) / 32), (unsigned)((R + 31) / 32)), dim3(256), 0, stream, in, R,
                       C, out);
}

// fp32 v = hi + lo with hi = bf16(v), lo = bf16(v - hi): 16 significant bits survive
__device__ __forceinline__ void split_bf16(float v, uint16_t& hi, uint16_t& lo) {
    hi = f32_to_bf16_rne(v);
    lo = f32_to_bf16_rne(v - bf16_bits_to_f32(hi));
}

// in [rows, l] fp32 -> out_t [2 L, rows] bf16: row c = high parts of column c, row L + c = low parts; columns
// l .. L - 1 are zero
__global__ __launch_bounds__(256) void split_transpose_kernel(const float* __restrict__ in, int64_t rows, int l, int L,
                                                              uint16_t* __restrict__ out_t) {
    const int64_t row = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (row >= rows) return;
    for (int c = 0; c < L; ++c) {
        uint16_t hi = 0, lo = 0;
        if (c < l) split_bf16(in[row * l + c], hi, lo);
        out_t[(int64_t)c * rows + row] = hi;
        out_t[(int64_t)(L + c) * rows + row] = lo;
    }
}

// y [rows, L] = sum over slices z of (partial[z][row][j] + partial[z][row][L + j]), z ascending
__global__ __launch_bounds__(256) void fold_reduce_kernel(const float* __restrict__ partial, int64_t rows, int L, int ksplit,
                                                          float* __restrict__ y) {
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int quads = L / 4;
    if (idx >= rows * quads) return;
    const int64_t row = idx / quads;
    const int j = (int)(idx % quads) * 4;
    float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int z = 0; z < ksplit; ++z) {
        const float* p = partial + ((int64_t)z * rows + row) * (2 * L);
        const float4 a = *reinterpret_cast<const float4*>(p + j);
        const float4 b = *reinterpret_cast<const float4*>(p + L + j);
        s.x += a.x + b.x; s.y += a.y + b.y; s.z += a.z + b.z; s.w += a.w + b.w;
    }
    *reinterpret_cast<float4*>(y + row * L + j) = s;
}

// gp[b] = Y_b^T Y_b for the kGramRows rows of block b (L = 16 TL columns); thread (ti, tj) owns entries (ti + 16 u, tj + 16 v)
constexpr int kGramRows = 128;
template <int TL>
__global__ __launch_bounds__(256) void gram_partial_kernel(const float* __restrict__ y, int64_t rows, float* __restrict__ gp) {
    constexpr int L = 16 * TL;
    __shared__ float ys[32][L + 4];
    const int tid = threadIdx.x, ti = tid >> 4, tj = tid & 15;
    float acc[TL][TL];
#pragma unroll
    for (int u = 0; u < TL; ++u)
#pragma unroll
        for (int v = 0; v < TL; ++v) acc[u][v] = 0.f;
    const int64_t r_begin = (int64_t)blockIdx.x * kGramRows;
    const int64_t r_end = r_begin + kGramRows < rows ? r_begin + kGramRows : rows;
    for (int64_t r0 = r_begin; r0 < r_end; r0 += 32) {
        for (int i = tid; i < 32 * L; i += 256) {
            const int rr = i / L, c = i % L;
            ys[rr][c] = r0 + rr < r_end ? y[(r0 + rr) * L + c] : 0.f;
        }
        __syncthreads();
        for (int rr = 0; rr < 32; ++rr) {
            float a[TL], b[TL];
#pragma unroll
            for (int u = 0; u < TL; ++u) a[u] = ys[rr][ti + 16 * u];
#pragma unroll
            for (int v = 0; v < TL; ++v) b[v] = ys[rr][tj + 16 * v];
#pragma unroll
            for (int u = 0; u < TL; ++u)
#pragma unroll
                for (int v = 0; v < TL; ++v) acc[u][v] += a[u] * b[v];
        }
        __syncthreads();
    }
    float* g = gp + (int64_t)blockIdx.x * L * L;
#pragma unroll
    for (int u = 0; u < TL; ++u)
#pragma unroll
        for (int v = 0; v < TL; ++v) g[(ti + 16 * u) * L + tj + 16 * v] = acc[u][v];
}

// g = sum of the partial Gram matrices in block order, one thread per entry (the loads of a thread are independent,
// so they overlap; inside the one-workgroup kernels below the same sum would be a chain of round trips)
__global__ __launch_bounds__(256) void gram_reduce_kernel(const float* __restrict__ gp, int nblocks, int count,
                                                          float* __restrict__ g) {
    const int idx = blockIdx.x * 256 + threadIdx.x;
    if (idx >= count) return;
    float s = 0.f;
    int b = 0;
    for (; b + 8 <= nblocks; b += 8) {
        float t[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) t[u] = gp[(int64_t)(b + u) * count + idx];
#pragma unroll
        for (int u = 0; u < 8; ++u) s += t[u];
    }
    for (; b < nblocks; ++b) s += gp[(int64_t)b * count + idx];
    g[idx] = s;
}

// One workgroup: G (the summed Gram matrix) = R^T R (Cholesky, R upper triangular),
// rinv = R^{-1}, so that Y rinv has orthonormal columns.  A column whose pivot falls below kDropRel of its own
// squared norm depends on the columns before it: it gets a zero column in rinv, i.e. it leaves the basis.
constexpr float kDropRel = 3e-6f;
template <int TL>
__global__ __launch_bounds__(256) void chol_inverse_kernel(const float* __restrict__ gsum, float* __restrict__ rinv) {
    constexpr int L = 16 * TL;
    __shared__ float g[L][L + 1];
    __shared__ float x[L][L + 1];
    __shared__ float diag0[L];
    __shared__ int dropped[L];
    const int tid = threadIdx.x;
    for (int idx = tid; idx < L * L; idx += 256) g[idx / L][idx % L] = gsum[idx];
    __syncthreads();
    if (tid < L) diag0[tid] = g[tid][tid];
    __syncthreads();
    // Right-looking elimination on the raw rows: step c subtracts g[c][i] g[c][j] / g[c][c] from the trailing part
    // and leaves row c alone, so one barrier per step is enough; the rows are scaled to R afterwards.
    {
        const int ti = tid >> 4, tj = tid & 15;
        for (int c = 0; c < L; ++c) {
            const float d = g[c][c];
            if (d > kDropRel * diag0[c] && d > 0.f) {   // the same decision in every thread
                const float inv_d = 1.f / d;
                for (int i = c + 1 + ti; i < L; i += 16) {
                    const float gi = g[c][i] * inv_d;
                    for (int j = c + 1 + tj; j < L; j += 16)
                        if (j >= i) g[i][j] -= gi * g[c][j];
                }
            }
            __syncthreads();
        }
    }
    if (tid < L) {
        const int c = tid;
        const float d = g[c][c];
        const bool ok = d > kDropRel * diag0[c] && d > 0.f;
        dropped[c] = ok ? 0 : 1;
        const float scale = ok ? 1.f / sqrtf(d) : 0.f;
        for (int j = c + 1; j < L; ++j) g[c][j] *= scale;
        g[c][c] = ok ? sqrtf(d) : 1.f;
    }
    __syncthreads();
    // X = R^{-1} in 16 x 16 blocks.  Diagonal blocks by back substitution (one thread per column, 16 steps deep);
    // above the diagonal  X[I][J] = -X[I][I] * sum_{P = I+1 .. J} R[I][P] X[P][J],  block row I descending, every
    // thread one entry of the 16 x 16 product: the block columns J are independent of each other.
    for (int idx = tid; idx < L * L; idx += 256) x[idx / L][idx % L] = 0.f;
    __syncthreads();
    if (tid < L && !dropped[tid]) {
        const int j = tid, j0 = j & ~15;
        x[j][j] = 1.f / g[j][j];
        for (int i = j - 1; i >= j0; --i) {
            float s = 0.f;
            for (int p = i + 1; p <= j; ++p) s += g[i][p] * x[p][j];
            x[i][j] = -s / g[i][i];
        }
    }
    __syncthreads();
    {
        __shared__ float tmp[TL][16][17];
        const int bi = tid >> 4, bj = tid & 15;   // entry (bi, bj) of a 16 x 16 block
        for (int step = 1; step < TL; ++step) {   // block row I = J - step for every block column J >= step
            for (int J = step; J < TL; ++J) {
                const int I = J - step;
                float s = 0.f;
                for (int P = I + 1; P <= J; ++P)
#pragma unroll
                    for (int c = 0; c < 16; ++c) s += g[16 * I + bi][16 * P + c] * x[16 * P + c][16 * J + bj];
                tmp[J][bi][bj] = s;
            }
            __syncthreads();
            for (int J = step; J < TL; ++J) {
                const int I = J - step;
                float s = 0.f;
#pragma unroll
                for (int c = 0; c < 16; ++c) s += x[16 * I + bi][16 * I + c] * tmp[J][c][bj];
                x[16 * I + bi][16 * J + bj] = dropped[16 * J + bj] ? 0.f : -s;
            }
            __syncthreads();
        }
    }
    for (int idx = tid; idx < L * L; idx += 256) rinv[idx] = x[idx / L][idx % L];
}

// out = in [rows, L] * m [L, L] for 64 rows per workgroup; thread (tr, tc) owns rows 4 tr .. + 3, columns tc + 16 u.
//   mode 0: out32 [rows, L] fp32 (may be `in`: a workgroup reads its rows before it writes them) and
//           out16 [2 L, pitch] bf16 = the transposed high and low parts (the other side of the next product)
//   mode 1: out16 [rows, ncols] bf16                      mode 2: out16 [ncols, pitch] bf16, transposed
// rows % 4 == 0 and pitch % 4 == 0 (the transposed stores are 8 bytes wide).
template <int TL>
__global__ __launch_bounds__(256) void apply_kernel(const float* in, int64_t rows, const float* __restrict__ m, int mode,
                                                    int ncols, float* out32, uint16_t* __restrict__ out16, int64_t pitch) {
    constexpr int L = 16 * TL;
    __shared__ float ms[L][L];
    __shared__ float ins[64][L + 1];
    const int tid = threadIdx.x, tr = tid >> 4, tc = tid & 15;
    const int64_t r0 = (int64_t)blockIdx.x * 64;
    for (int idx = tid; idx < L * L; idx += 256) ms[idx / L][idx % L] = m[idx];
    for (int idx = tid; idx < 64 * L; idx += 256) {
        const int rr = idx / L, c = idx % L;
        ins[rr][c] = r0 + rr < rows ? in[(r0 + rr) * L + c] : 0.f;
    }
    __syncthreads();
    float acc[4][TL];
#pragma unroll
    for (int q = 0; q < 4; ++q)
#pragma unroll
        for (int u = 0; u < TL; ++u) acc[q][u] = 0.f;
    for (int p = 0; p < L; ++p) {
        float a[4], b[TL];
#pragma unroll
        for (int q = 0; q < 4; ++q) a[q] = ins[4 * tr + q][p];
#pragma unroll
        for (int u = 0; u < TL; ++u) b[u] = ms[p][tc + 16 * u];
#pragma unroll
        for (int q = 0; q < 4; ++q)
#pragma unroll
            for (int u = 0; u < TL; ++u) acc[q][u] += a[q] * b[u];
    }
    const int64_t row = r0 + 4 * tr;   // rows % 4 == 0: the thread's four rows are all inside or all outside
    if (row >= rows) return;
#pragma unroll
    for (int u = 0; u < TL; ++u) {
        const int c = tc + 16 * u;
        if (mode == 0) {
            uint16_t hi[4], lo[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                out32[(row + q) * L + c] = acc[q][u];
                split_bf16(acc[q][u], hi[q], lo[q]);
            }
            *reinterpret_cast<uint2*>(out16 + (int64_t)c * pitch + row) =
                make_uint2(hi[0] | ((uint32_t)hi[1] << 16), hi[2] | ((uint32_t)hi[3] << 16));
            *reinterpret_cast<uint2*>(out16 + (int64_t)(L + c) * pitch + row) =
                make_uint2(lo[0] | ((uint32_t)lo[1] << 16), lo[2] | ((uint32_t)lo[3] << 16));
        } else if (c < ncols) {
            uint16_t h[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) h[q] = f32_to_bf16_rne(acc[q][u]);
            if (mode == 1) {
#pragma unroll
                for (int q = 0; q < 4; ++q) out16[(row + q) * ncols + c] = h[q];
            } else {
                *reinterpret_cast<uint2*>(out16 + (int64_t)c * pitch + row) =
                    make_uint2(h[0] | ((uint32_t)h[1] << 16), h[2] | ((uint32_t)h[3] << 16));
            }
        }
    }
}

// One workgroup: G = sum of partial Gram matrices of Z (= Z^T Z, symmetric l x l), G = U~ diag(lambda) U~^T by
// cyclic Jacobi with the L / 2 disjoint rotations of a round-robin round applied together, eigenvalues ranked in
// descending order; then  ma[:, k] = u_k lambda_k^{-1/4},  mb[:, k] = u_k lambda_k^{1/4}  for the r largest (other
// columns zero) and sigma[k] = sqrt(lambda_k).
constexpr int kJacobiSweeps = 8;   // upper bound (fp32 Jacobi on up to 128 columns is through by then); a sweep that meets nothing worth rotating ends the loop
template <int TL>
__global__ __launch_bounds__(256) void eig_kernel(const float* gsum, int r, float* __restrict__ ma, float* mb,
                                                  float* __restrict__ sigma) {
    constexpr int L = 16 * TL, H = L / 2;
    __shared__ float a[L][L + 1];
    __shared__ float v[L][L + 1];
    __shared__ float rot[H][2];
    __shared__ int pair[H][2];
    __shared__ float lam[L];
    __shared__ int order[L];
    const int tid = threadIdx.x, nthreads = blockDim.x;
    __shared__ float off_max[H];
    __shared__ int done;
    for (int idx = tid; idx < L * L; idx += nthreads) {   // gsum may be the memory that mb goes to at the end
        a[idx / L][idx % L] = gsum[idx];
        v[idx / L][idx % L] = idx / L == idx % L ? 1.f : 0.f;
    }
    __syncthreads();
    for (int sweep = 0; sweep < kJacobiSweeps; ++sweep) {
        if (tid < H) off_max[tid] = 0.f;
        for (int t = 0; t < L - 1; ++t) {
            if (tid < H) {   // round t of the round-robin schedule: index L - 1 stays put, the others turn
                int p = tid == 0 ? L - 1 : (t + tid) % (L - 1);
                int q = tid == 0 ? t : (t - tid + (L - 1)) % (L - 1);
                if (p > q) { const int s = p; p = q; q = s; }
                const float app = a[p][p], aqq = a[q][q], apq = a[p][q];
                float c = 1.f, s = 0.f;
                if (fabsf(apq) > 1e-30f) {
                    const float theta = (aqq - app) / (2.f * apq);
                    const float tt = copysignf(1.f, theta) / (fabsf(theta) + sqrtf(1.f + theta * theta));
                    c = 1.f / sqrtf(1.f + tt * tt);
                    s = tt * c;
                }
                off_max[tid] = fmaxf(off_max[tid], fabsf(apq));
                pair[tid][0] = p; pair[tid][1] = q;
                rot[tid][0] = c; rot[tid][1] = s;
            }
            __syncthreads();
            // The items of a phase touch disjoint entries; they are taken kBatch at a time with all reads before
            // the first write, or every item would wait for the LDS round trip of the one before it.
            constexpr int kBatch = 4;
            for (int base = tid; base < H * L; base += nthreads * kBatch) {   // columns p, q of a and of v
                int p[kBatch], q[kBatch], k[kBatch];
                float c[kBatch], s[kBatch], ap[kBatch], aq[kBatch], vp[kBatch], vq[kBatch];
#pragma unroll
                for (int b = 0; b < kBatch; ++b) {
                    const int idx = base + b * nthreads;
                    const int pr = idx < H * L ? idx / L : 0;
                    k[b] = idx < H * L ? idx % L : -1;
                    p[b] = pair[pr][0]; q[b] = pair[pr][1];
                    c[b] = rot[pr][0]; s[b] = rot[pr][1];
                    const int kk = k[b] < 0 ? 0 : k[b];
                    ap[b] = a[kk][p[b]]; aq[b] = a[kk][q[b]];
                    vp[b] = v[kk][p[b]]; vq[b] = v[kk][q[b]];
                }
#pragma unroll
                for (int b = 0; b < kBatch; ++b) {
                    if (k[b] < 0) continue;
                    a[k[b]][p[b]] = c[b] * ap[b] - s[b] * aq[b];
                    a[k[b]][q[b]] = s[b] * ap[b] + c[b] * aq[b];
                    v[k[b]][p[b]] = c[b] * vp[b] - s[b] * vq[b];
                    v[k[b]][q[b]] = s[b] * vp[b] + c[b] * vq[b];
                }
            }
            __syncthreads();
            for (int base = tid; base < H * L; base += nthreads * kBatch) {   // rows p, q of a
                int p[kBatch], q[kBatch], k[kBatch];
                float c[kBatch], s[kBatch], ap[kBatch], aq[kBatch];
#pragma unroll
                for (int b = 0; b < kBatch; ++b) {
                    const int idx = base + b * nthreads;
                    const int pr = idx < H * L ? idx / L : 0;
                    k[b] = idx < H * L ? idx % L : -1;
                    p[b] = pair[pr][0]; q[b] = pair[pr][1];
                    c[b] = rot[pr][0]; s[b] = rot[pr][1];
                    const int kk = k[b] < 0 ? 0 : k[b];
                    ap[b] = a[p[b]][kk]; aq[b] = a[q[b]][kk];
                }
#pragma unroll
                for (int b = 0; b < kBatch; ++b) {
                    if (k[b] < 0) continue;
                    a[p[b]][k[b]] = c[b] * ap[b] - s[b] * aq[b];
                    a[q[b]][k[b]] = s[b] * ap[b] + c[b] * aq[b];
                }
            }
            __syncthreads();
        }
        // converged when no off-diagonal entry met in this sweep exceeds a few fp32 roundings of the largest diagonal entry
        if (tid == 0) {
            float off = 0.f, dmax = 0.f;
            for (int i = 0; i < H; ++i) off = fmaxf(off, off_max[i]);
            for (int i = 0; i < L; ++i) dmax = fmaxf(dmax, fabsf(a[i][i]));
            done = off <= 5e-7f * dmax ? 1 : 0;
        }
        __syncthreads();
        if (done) break;
    }
    if (tid < L) lam[tid] = a[tid][tid] > 0.f ? a[tid][tid] : 0.f;
    __syncthreads();
    if (tid < L) {
        int rk = 0;
        for (int j = 0; j < L; ++j) rk += (lam[j] > lam[tid] || (lam[j] == lam[tid] && j < tid)) ? 1 : 0;
        order[tid] = rk;
    }
    __syncthreads();
    float lmax = 0.f;
    for (int j = 0; j < L; ++j) lmax = lam[j] > lmax ? lam[j] : lmax;
    for (int idx = tid; idx < L * L; idx += nthreads) {
        const int p = idx / L, i = idx % L;
        const int rk = order[i];
        float fa = 0.f, fb = 0.f;
        if (rk < r && lam[i] > 1e-12f * lmax) {
            fb = sqrtf(sqrtf(lam[i]));
            fa = 1.f / fb;
        }
        ma[p * L + rk] = v[p][i] * fa;
        mb[p * L + rk] = v[p][i] * fb;
    }
    if (sigma != nullptr && tid < L && order[tid] < r) sigma[order[tid]] = sqrtf(lam[tid]);
}

// ---------------------------------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------------------------------
struct SvdPlan {
    int L, ks_n, ks_k, gram_blocks;
    size_t off_et, off_y, off_z, off_bt, off_partial, off_gp, off_small, total;
};

static SvdPlan svd_plan(int64_t N, int64_t K, int64_t l) {
    SvdPlan p;
    p.L = (int)((l + 15) / 16 * 16);
    p.ks_n = adapter_ksplit(N, K);   // rows N, contraction over K
    p.ks_k = adapter_ksplit(K, N);   // rows K, contraction over N
    const int64_t big = N > K ? N : K;
    p.gram_blocks = (int)((big + kGramRows - 1) / kGramRows);
    size_t o = 0;
    p.off_et = o; o += round_up_256((size_t)N * K * sizeof(uint16_t));
    p.off_y = o; o += round_up_256((size_t)N * p.L * sizeof(float));
    p.off_z = o; o += round_up_256((size_t)K * p.L * sizeof(float));
    p.off_bt = o; o += round_up_256((size_t)2 * p.L * big * sizeof(uint16_t));
    const size_t pn = (size_t)p.ks_n * N, pk = (size_t)p.ks_k * K;
    p.off_partial = o; o += round_up_256((pn > pk ? pn : pk) * 2 * p.L * sizeof(float));
    p.off_gp = o; o += round_up_256((size_t)p.gram_blocks * p.L * p.L * sizeof(float));
    p.off_small = o; o += round_up_256((size_t)2 * p.L * p.L * sizeof(float));
    p.total = o;
    return p;
}

size_t residual_adapter_workspace_bytes(int64_t N, int64_t K, int64_t l) { return svd_plan(N, K, l).total; }

template <int TL>
static void run_svd(const uint16_t* e, int64_t N, int64_t K, int r, int l, int iterations, const float* omega,
                    uint16_t* a_res, uint16_t* b_res, float* sigma, char* ws, const SvdPlan& p, hipStream_t stream) {
    constexpr int L = 16 * TL;
    uint16_t* et = reinterpret_cast<uint16_t*>(ws + p.off_et);
    float* y = reinterpret_cast<float*>(ws + p.off_y);
    float* z = reinterpret_cast<float*>(ws + p.off_z);
    uint16_t* bt = reinterpret_cast<uint16_t*>(ws + p.off_bt);
    float* partial = reinterpret_cast<float*>(ws + p.off_partial);
    float* gp = reinterpret_cast<float*>(ws + p.off_gp);
    float* small_a = reinterpret_cast<float*>(ws + p.off_small);
    float* small_b = small_a + L * L;

    auto product = [&](const uint16_t* mat, int64_t rows, int64_t cols, int ks, float* out) {   // out = mat * (bt as fp32)^T
        launch_tall_product(mat, rows, cols, bt, 2 * L, ks, nullptr, partial, true, stream);
        hipLaunchKernelGGL(fold_reduce_kernel, dim3((unsigned)((rows * (L / 4) + 255) / 256)), dim3(256), 0, stream, partial, rows,
                           L, ks, out);
    };
    auto gram = [&](const float* buf, int64_t rows) {   // small_b = buf^T buf
        const int nb = (int)((rows + kGramRows - 1) / kGramRows);
        hipLaunchKernelGGL((gram_partial_kernel<TL>), dim3(nb), dim3(256), 0, stream, buf, rows, gp);
        hipLaunchKernelGGL(gram_reduce_kernel, dim3((L * L + 255) / 256), dim3(256), 0, stream, gp, nb, L * L, small_b);
    };
    // CholeskyQR; leaves the transposed split copy in bt.  Inside the iteration one pass is enough (it only has to
    // keep the columns from collapsing onto the leading direction); the basis that the result is built on gets two.
    auto orth = [&](float* buf, int64_t rows, int passes) {
        for (int pass = 0; pass < passes; ++pass) {
            gram(buf, rows);
            hipLaunchKernelGGL((chol_inverse_kernel<TL>), dim3(1), dim3(256), 0, stream, small_b, small_a);
            hipLaunchKernelGGL((apply_kernel<TL>), dim3((unsigned)((rows + 63) / 64)), dim3(256), 0, stream, buf, rows, small_a, 0,
                               L, buf, bt, rows);
        }
    };

    launch_transpose_bf16(e, N, K, et, stream);
    hipLaunchKernelGGL(split_transpose_kernel, dim3((unsigned)((K + 255) / 256)), dim3(256), 0, stream, omega, K, l, L, bt);
    product(e, N, K, p.ks_n, y);                      // Y = E Omega
    orth(y, N, iterations == 0 ? 2 : 1);              // Q
    product(et, K, N, p.ks_k, z);                     // Z = E^T Q
    for (int it = 0; it < iterations; ++it) {
        orth(z, K, 1);
        product(e, N, K, p.ks_n, y);
        orth(y, N, it + 1 == iterations ? 2 : 1);
        product(et, K, N, p.ks_k, z);
    }
    gram(z, K);
    hipLaunchKernelGGL((eig_kernel<TL>), dim3(1), dim3(256), 0, stream, small_b, r, small_a, small_b, sigma);
    hipLaunchKernelGGL((apply_kernel<TL>), dim3((unsigned)((K + 63) / 64)), dim3(256), 0, stream, z, K, small_a, 1, r,
                       (float*)nullptr, a_res, (int64_t)r);
    hipLaunchKernelGGL((apply_kernel<TL>), dim3((unsigned)((N + 63) / 64)), dim3(256), 0, stream, y, N, small_b, 2, r,
                       (float*)nullptr, b_res, N);
}

hipError_t launch_residual_adapter(const uint16_t* e, int64_t N, int64_t K, int64_t r, int64_t l, int64_t iterations,
                                   const float* omega, uint16_t* a_res, uint16_t* b_res, float* sigma, void* workspace,
                                   hipStream_t stream) {
    const SvdPlan p = svd_plan(N, K, l);
    char* ws = static_cast<char*>(workspace);
    switch (p.L / 16) {
        case 1: run_svd<1>(e, N, K, (int)r, (int)l, (int)iterations, omega, a_res, b_res, sigma, ws, p, stream); break;
        case 2: run_svd<2>(e, N, K, (int)r, (int)l, (int)iterations, omega, a_res, b_res, sigma, ws, p, stream); break;
        case 3: run_svd<3>(e, N, K, (int)r, (int)l, (int)iterations, omega, a_res, b_res, sigma, ws, p, stream); break;
        case 4: run_svd<4>(e, N, K, (int)r, (int)l, (int)iterations, omega, a_res, b_res, sigma, ws, p, stream); break;
        case 5: run_svd<5>(e, N, K, (int)r, (int)l, (int)iterations, omega, a_res, b_res, sigma, ws, p, stream); break;
        case 6: run_svd<6>(e, N, K, (int)r, (int)l, (int)iterations, omega, a_res, b_res, sigma, ws, p, stream); break;
        case 7: run_svd<7>(e, N, K, (int)r, (int)l, (int)iterations, omega, a_res, b_res, sigma, ws, p, stream); break;
        case 8: run_svd<8>(e, N, K, (int)r, (int)l, (int)iterations, omega, a_res, b_res, sigma, ws, p, stream); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

}  // namespace salr
