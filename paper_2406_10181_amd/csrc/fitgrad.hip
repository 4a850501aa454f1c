// Gradient of the data term of projector fitting with respect to the stored projector values
// (the minimisation in MaybeUpdate, Alg. 1; Eq. 2):
//     F(P, Q) = 1/2 || P P^T G Q Q^T - G ||_F^2,    gP[i][k] = dF / dP_val[i][k],   gQ[j][k] = dF / dQ_val[j][k].
// With S = P^T G Q, R = P S Q^T - G, Z = P^T R Q the chain rule gives
//     dF/dPhat = (R Q) S^T + (G Q) Z^T,          dF/dQhat = (R^T P) S + (G^T P) Z,
// and everything that involves R collapses onto r x r matrices, because
//     R Q = P S (Q^T Q) - G Q,    R^T P = Q S^T (P^T P) - G^T P,    Z = (P^T P) S (Q^T Q) - S.
// So with C_P = P^T P, C_Q = Q^T Q, S1 = S C_Q, X = C_P S (all r x r):
//     dF/dPhat[i][a] = sum_k' P_val[i][k'] M1[P_idx[i][k']][a] + sum_b T[i][b] D[a][b],      M1 = S1 S^T,
//     dF/dQhat[j][b] = sum_k' Q_val[j][k'] M2[Q_idx[j][k']][b] + sum_a Y[a][j] D[a][b],      M2 = S^T X,
//     D = Z - S = C_P S1 - 2 S,     T = G Q (m x r),     Y = P^T G (r x n).
// G is streamed twice: once by the compress kernels (T and S, as in every training step) and once, row by
// row through the column-sorted copy of P in the plan, for Y.  The dense r x r products run in fp32 on the
// matrix cores; the rest is gathers and fp32 dot products.  No m x n temporary exists.
#include <cstring>

#include "lsp_internal.h"

namespace lsp {

typedef float f32x4 __attribute__((ext_vector_type(4)));

// Y[a][j] = sum over the entries (i, v) of row a of P^T of v * G[i][j]: one workgroup per (piece of a row of
// P^T, tile of columns); a thread owns VEC consecutive columns.  Rows cut into pieces (heavily skewed
// projectors) add up with atomics on a Y that k_zero_if_split cleared.
constexpr int kThreadsY = 128;
template <typename D, int VEC>
__global__ __launch_bounds__(kThreadsY) void k_gather_rows(const typename D::elem* __restrict__ G, const uint8_t* __restrict__ plan,
                                                          float* __restrict__ Y, int m, int n, int r, int d) {
    PlanHeaderPtr H = as_const<PlanHeader>(plan);
    if (H->magic != kPlanMagic || H->m != m || H->n != n || H->r != r || H->d != d) return;
    const int item = blockIdx.x;
    if (item >= H->p_nitems) return;
    const auto* itp = as_const<int32_t>(plan + H->off_p_item) + 4 * item;
    const RowItem it{itp[0], itp[1], itp[2], itp[3]};
    const uint2* ent = reinterpret_cast<const uint2*>(plan + H->off_p_ent) + it.start;
    const int64_t j0 = ((int64_t)blockIdx.y * kThreadsY + threadIdx.x) * VEC;
    if (j0 >= n) return;
    float acc[VEC];
#pragma unroll
    for (int q = 0; q < VEC; ++q) acc[q] = 0.0f;
    for (int e = 0; e < it.len; ++e) {
        const uint2 en = ent[e];                                    // uniform over the workgroup
        const float v = __uint_as_float(en.y);
        const typename D::elem* row = G + (int64_t)en.x * n + j0;
        if constexpr (VEC == 8) {                                   // 16-bit storage, n % 8 == 0
            const uint4 x = *reinterpret_cast<const uint4*>(row);
            const uint32_t w[4] = {x.x, x.y, x.z, x.w};
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                acc[2 * q]     = fmaf(v, widen<D>((uint16_t)(w[q] & 0xFFFFu)), acc[2 * q]);
                acc[2 * q + 1] = fmaf(v, widen<D>((uint16_t)(w[q] >> 16)), acc[2 * q + 1]);
            }
        } else if constexpr (VEC == 4) {                            // fp32 storage, n % 4 == 0
            const f32x4 x = *reinterpret_cast<const f32x4*>(row);
            acc[0] = fmaf(v, x.x, acc[0]); acc[1] = fmaf(v, x.y, acc[1]);
            acc[2] = fmaf(v, x.z, acc[2]); acc[3] = fmaf(v, x.w, acc[3]);
        } else {
            acc[0] = fmaf(v, widen<D>(row[0]), acc[0]);
        }
    }
    float* dst = Y + (int64_t)it.a * n + j0;
#pragma unroll
    for (int q = 0; q < VEC; ++q) {
        if (it.atomic) atomicAdd(dst + q, acc[q]);
        else dst[q] = acc[q];
    }
}

__global__ __launch_bounds__(256) void k_zero_if_split(const uint8_t* __restrict__ plan, float* __restrict__ Y, int64_t count) {
    PlanHeaderPtr H = as_const<PlanHeader>(plan);
    if (H->magic != kPlanMagic || !H->p_any_split) return;
    for (int64_t k = (int64_t)blockIdx.x * 256 + threadIdx.x; k < count; k += (int64_t)gridDim.x * 256) Y[k] = 0.0f;
}

// gP[i][k] = sum_k' P_val[i][k'] M1[P_idx[i][k']][a] + sum_b T[i][b] D[a][b],  a = P_idx[i][k]: one wave per
// row i, the dot product over b spread over its lanes.
__global__ __launch_bounds__(256) void k_grad_left(const float* __restrict__ T, const float* __restrict__ Dm, const float* __restrict__ M1,
                                                   const int32_t* __restrict__ P_idx, const float* __restrict__ P_val,
                                                   int m, int r, int d, float* __restrict__ gP) {
    const int lane = threadIdx.x & 63;
    const int64_t i = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (i >= m) return;
    const float* Ti = T + i * r;
    for (int k = 0; k < d; ++k) {
        const int a = P_idx[i * d + k];
        const float* Da = Dm + (int64_t)a * r;
        float acc = 0.0f;
        for (int b = lane; b < r; b += 64) acc = fmaf(Ti[b], Da[b], acc);
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) acc += __shfl_down(acc, off);
        if (lane == 0) {
            float g = acc;
            for (int k2 = 0; k2 < d; ++k2) g = fmaf(P_val[i * d + k2], M1[(int64_t)P_idx[i * d + k2] * r + a], g);
            gP[i * d + k] = g;
        }
    }
}

// gQ[j][k] = sum_k' Q_val[j][k'] M2[Q_idx[j][k']][b] + sum_a Y[a][j] D[a][b],  b = Q_idx[j][k]: a workgroup takes
// 16 columns j (the reads of Y are then contiguous) and cuts the sum over a into 16 interleaved slices, one per
// group of 16 threads; the slices' sums meet in LDS and are added in slice order.  Eight entries of a row at a time.
constexpr int kGradCols = 16, kGradSlices = 16;
__global__ __launch_bounds__(kGradCols * kGradSlices) void k_grad_right(const float* __restrict__ Y, const float* __restrict__ Dm, const float* __restrict__ M2,
                                                                      const int32_t* __restrict__ Q_idx, const float* __restrict__ Q_val,
                                                                      int n, int r, int d, float* __restrict__ gQ) {
    __shared__ float part[kGradSlices][kGradCols][8];
    const int jl = threadIdx.x % kGradCols, sl = threadIdx.x / kGradCols;
    const int64_t j = (int64_t)blockIdx.x * kGradCols + jl;
    const bool live = j < n;
    const int64_t jc = live ? j : (int64_t)n - 1;
    for (int k0 = 0; k0 < d; k0 += 8) {
        int b[8];
        float acc[8];
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            b[q] = k0 + q < d ? Q_idx[jc * d + k0 + q] : 0;
            acc[q] = 0.0f;
        }
        for (int a = sl; a < r; a += kGradSlices) {
            const float y = Y[(int64_t)a * n + jc];
            const float* Da = Dm + (int64_t)a * r;
#pragma unroll
            for (int q = 0; q < 8; ++q) acc[q] = fmaf(y, Da[b[q]], acc[q]);
        }
#pragma unroll
        for (int q = 0; q < 8; ++q) part[sl][jl][q] = acc[q];
        __syncthreads();
        if (sl == 0 && live) {
#pragma unroll
            for (int q = 0; q < 8; ++q) {
                if (k0 + q < d) {
                    float g = 0.0f;
                    for (int t = 0; t < kGradSlices; ++t) g += part[t][jl][q];
                    for (int k2 = 0; k2 < d; ++k2) g = fmaf(Q_val[j * d + k2], M2[(int64_t)Q_idx[j * d + k2] * r + b[q]], g);
                    gQ[j * d + k0 + q] = g;
                }
            }
        }
        __syncthreads();
    }
}

// floats of workspace: T (m r) | S, C_P, C_Q, S1, X, D, M1, M2 (8 r^2) | Y (r n)
size_t fitgrad_workspace_floats(int64_t m, int64_t n, int32_t r) {
    const size_t rr = (size_t)r * (size_t)r;
    return align_up((size_t)m * r, 64) + 8 * align_up(rr, 64) + align_up((size_t)r * (size_t)n, 64);
}

template <typename D>
static hipError_t launch_gather(const void* G, const uint8_t* plan, float* Y, int64_t m, int64_t n, int32_t r, int32_t d, hipStream_t st) {
    using E = typename D::elem;
    const unsigned items = (unsigned)plan_max_items(m, r, d);
    auto tiles = [&](int vec) { return (unsigned)((n + (int64_t)kThreadsY * vec - 1) / ((int64_t)kThreadsY * vec)); };
    if (D::size == 2 && n % 8 == 0)
        hipLaunchKernelGGL((k_gather_rows<D, 8>), dim3(items, tiles(8)), dim3(kThreadsY), 0, st, static_cast<const E*>(G), plan, Y, (int)m, (int)n, (int)r, (int)d);
    else if (D::size == 4 && n % 4 == 0)
        hipLaunchKernelGGL((k_gather_rows<D, 4>), dim3(items, tiles(4)), dim3(kThreadsY), 0, st, static_cast<const E*>(G), plan, Y, (int)m, (int)n, (int)r, (int)d);
    else
        hipLaunchKernelGGL((k_gather_rows<D, 1>), dim3(items, tiles(1)), dim3(kThreadsY), 0, st, static_cast<const E*>(G), plan, Y, (int)m, (int)n, (int)r, (int)d);
    return hipGetLastError();
}

hipError_t launch_fitgrad(const void* G, const uint8_t* plan, const int32_t* P_idx, const float* P_val,
                          const int32_t* Q_idx, const float* Q_val, int64_t m, int64_t n, int32_t r, int32_t d,
                          float* gP, float* gQ, float* ws, lsp_dtype dtype, hipStream_t st) {
    const size_t rr = align_up((size_t)r * (size_t)r, 64);
    float* T = ws;
    float* S = T + align_up((size_t)m * r, 64);
    float* CP = S + rr; float* CQ = CP + rr; float* S1 = CQ + rr; float* X = S1 + rr;
    float* Dm = X + rr; float* M1 = Dm + rr; float* M2 = M1 + rr;
    float* Y = M2 + rr;
    hipError_t e;
    // T = G Q and S = P^T T: the compress kernels (a plan of another problem leaves S full of NaN, which then
    // reaches every output)
    CompressGroup g;
    memset(&g, 0, sizeof(g));
    g.count = 1; g.G[0] = G; g.plan[0] = plan; g.T[0] = T; g.S[0] = S; g.m[0] = (int32_t)m; g.n[0] = (int32_t)n;
    if ((e = launch_compress_planned(g, r, d, dtype, st)) != hipSuccess) return e;
    // C_P = P^T P, C_Q = Q^T Q (adjacent: one clearing pass)
    if ((e = launch_zero(CP, (int64_t)(2 * rr), st)) != hipSuccess) return e;
    if ((e = launch_gram(P_idx, P_val, P_idx, P_val, m, d, r, CP, st)) != hipSuccess) return e;
    if ((e = launch_gram(Q_idx, Q_val, Q_idx, Q_val, n, d, r, CQ, st)) != hipSuccess) return e;
    // the r x r chain
    if ((e = launch_gemm_rr(S, CQ, S1, r, false, false, 0.0f, nullptr, st)) != hipSuccess) return e;     // S1 = S C_Q
    if ((e = launch_gemm_rr(CP, S, X, r, false, false, 0.0f, nullptr, st)) != hipSuccess) return e;      // X  = C_P S
    if ((e = launch_gemm_rr(CP, S1, Dm, r, false, false, -2.0f, S, st)) != hipSuccess) return e;         // D  = C_P S1 - 2 S
    if ((e = launch_gemm_rr(S1, S, M1, r, false, true, 0.0f, nullptr, st)) != hipSuccess) return e;      // M1 = S1 S^T
    if ((e = launch_gemm_rr(S, X, M2, r, true, false, 0.0f, nullptr, st)) != hipSuccess) return e;       // M2 = S^T X
    // Y = P^T G
    hipLaunchKernelGGL(k_zero_if_split, dim3(1024), dim3(256), 0, st, plan, Y, (int64_t)r * n);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    switch (dtype) {
        case LSP_F32:  e = launch_gather<F32>(G, plan, Y, m, n, r, d, st); break;
        case LSP_F16:  e = launch_gather<F16>(G, plan, Y, m, n, r, d, st); break;
        default:       e = launch_gather<BF16>(G, plan, Y, m, n, r, d, st); break;
    }
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(k_grad_left, dim3((unsigned)((m + 3) / 4)), dim3(256), 0, st, T, Dm, M1, P_idx, P_val, (int)m, (int)r, (int)d, gP);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    hipLaunchKernelGGL(k_grad_right, dim3((unsigned)((n + kGradCols - 1) / kGradCols)), dim3(kGradCols * kGradSlices), 0, st, Y, Dm, M2, Q_idx, Q_val, (int)n, (int)r, (int)d, gQ);
    return hipGetLastError();
}

}  // namespace lsp
