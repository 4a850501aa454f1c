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
#include <algorithm>
#include <cstring>
#include <type_traits>

#include "lsp_internal.h"

namespace lsp {

typedef float f32x4 __attribute__((ext_vector_type(4)));

// Y[a][j] = sum over the entries (i, v) of row a of P^T of v * G[i][j]: one workgroup per (piece of a row of
// P^T, tile of 64 VEC columns); a lane owns VEC consecutive columns, and the four waves take a quarter of the
// piece's entries each; their sums meet in LDS and are added in wave order.  Rows cut into pieces (heavily
// skewed projectors) add up with atomics on a Y that k_zero_if_split cleared.
// Every row of G is wanted by d rows of Y, so G goes from L2 to the CUs d times: that traffic (268 MB at
// 4096 x 4096, d = 8, 16-bit) is what the kernel's time is made of, whatever the shape of the workgroups.  HBM
// sees G once: workgroup b runs on XCD b % 8 (the dispatcher deals workgroups round-robin), and the grid is laid
// out so that one XCD takes every row of Y for a column tile before its next tile, so a tile of G (m rows of
// 64 VEC elements, 2 MB at m = 4096) stays in that XCD's L2 for its d visits.
constexpr int kThreadsY = 256, kWavesY = kThreadsY / kWave, kXcds = 8;
template <typename D, int VEC>
__global__ __launch_bounds__(kThreadsY) void k_gather_rows(const typename D::elem* __restrict__ G, const uint8_t* __restrict__ plan,
                                                          float* __restrict__ Y, int m, int n, int r, int d, int items, int tiles) {
    __shared__ float part[kWavesY][kWave * VEC];
    PlanHeaderPtr H = as_const<PlanHeader>(plan);
    if (H->magic != kPlanMagic || H->m != m || H->n != n || H->r != r || H->d != d) return;
    const int seq = blockIdx.x / kXcds;                             // position in this XCD's sequence: items fastest
    const int item = seq % items, tile = (seq / items) * kXcds + blockIdx.x % kXcds;
    if (item >= H->p_nitems || tile >= tiles) return;
    const auto* itp = as_const<int32_t>(plan + H->off_p_item) + 4 * item;
    const RowItem it{itp[0], itp[1], itp[2], itp[3]};
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    const int e_begin = (int)((int64_t)it.len * wave / kWavesY), e_end = (int)((int64_t)it.len * (wave + 1) / kWavesY);
    const uint2* ent = reinterpret_cast<const uint2*>(plan + H->off_p_ent) + it.start;
    const int64_t tile0 = (int64_t)tile * kWave * VEC;
    const int64_t j0 = tile0 + lane * VEC;
    const bool live = j0 < n;                                       // n % VEC == 0: a lane's columns are all in or all out
    float acc[VEC];
#pragma unroll
    for (int q = 0; q < VEC; ++q) acc[q] = 0.0f;
    // a lane's piece of a row: 8 bytes of 16-bit storage or 16 bytes of fp32 (VEC == 4), else one element
    using Piece = typename std::conditional<VEC == 1, typename D::elem, typename std::conditional<D::size == 2, uint2, f32x4>::type>::type;
    auto load = [&](uint2 en) { return *reinterpret_cast<const Piece*>(G + (int64_t)en.x * n + j0); };
    auto add = [&](uint2 en, Piece x) {                             // entries are added in their stored order
        const float v = __uint_as_float(en.y);
        if constexpr (VEC == 1) {
            acc[0] = fmaf(v, widen<D>(x), acc[0]);
        } else if constexpr (D::size == 2) {
            acc[0] = fmaf(v, widen<D>((uint16_t)(x.x & 0xFFFFu)), acc[0]); acc[1] = fmaf(v, widen<D>((uint16_t)(x.x >> 16)), acc[1]);
            acc[2] = fmaf(v, widen<D>((uint16_t)(x.y & 0xFFFFu)), acc[2]); acc[3] = fmaf(v, widen<D>((uint16_t)(x.y >> 16)), acc[3]);
        } else {
            acc[0] = fmaf(v, x.x, acc[0]); acc[1] = fmaf(v, x.y, acc[1]);
            acc[2] = fmaf(v, x.z, acc[2]); acc[3] = fmaf(v, x.w, acc[3]);
        }
    };
    if (live) {
        // eight rows of G in flight per lane: a row piece is one load whose latency nothing else hides
        constexpr int kInFlight = 8;
        int e = e_begin;
        for (; e + kInFlight <= e_end; e += kInFlight) {
            uint2 en[kInFlight];                                    // uniform over the wave
            Piece x[kInFlight];
#pragma unroll
            for (int u = 0; u < kInFlight; ++u) en[u] = ent[e + u];
#pragma unroll
            for (int u = 0; u < kInFlight; ++u) x[u] = load(en[u]);
#pragma unroll
            for (int u = 0; u < kInFlight; ++u) add(en[u], x[u]);
        }
        for (; e < e_end; ++e) {
            const uint2 en = ent[e];
            add(en, load(en));
        }
    }
#pragma unroll
    for (int q = 0; q < VEC; ++q) part[wave][q * kWave + lane] = acc[q];     // column lane * VEC + q of the tile
    __syncthreads();
    for (int c = threadIdx.x; c < kWave * VEC; c += kThreadsY) {
        const int64_t j = tile0 + c;
        if (j >= n) break;
        const int slot = (c % VEC) * kWave + c / VEC;
        float sum = part[0][slot];
#pragma unroll
        for (int w = 1; w < kWavesY; ++w) sum += part[w][slot];
        float* dst = Y + (int64_t)it.a * n + j;
        if (it.atomic) atomicAdd(dst, sum);
        else *dst = sum;
    }
}

__global__ __launch_bounds__(256) void k_zero_if_split(const uint8_t* __restrict__ plan, float* __restrict__ Y, int64_t count) {
    PlanHeaderPtr H = as_const<PlanHeader>(plan);
    if (H->magic != kPlanMagic || !H->p_any_split) return;
    for (int64_t k = (int64_t)blockIdx.x * 256 + threadIdx.x; k < count; k += (int64_t)gridDim.x * 256) Y[k] = 0.0f;
}

// gP[i][k] = sum_k' P_val[i][k'] M1[P_idx[i][k']][a] + sum_b T[i][b] D[a][b],  a = P_idx[i][k]: one wave per
// row i, the dot product over b spread over its lanes; lane k' < d also carries the k'-th term of the first
// sum into the same lane reduction (d <= 64).  Four entries of the row at a time, so that their loads overlap.
__global__ __launch_bounds__(256) void k_grad_left(const float* __restrict__ T, const float* __restrict__ Dm, const float* __restrict__ M1,
                                                   const int32_t* __restrict__ P_idx, const float* __restrict__ P_val,
                                                   int m, int r, int d, float* __restrict__ gP) {
    const int lane = threadIdx.x & 63;
    const int64_t i = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (i >= m) return;
    const float* Ti = T + i * r;
    const bool mine = lane < d;
    const float pv = mine ? P_val[i * d + lane] : 0.0f;
    const int64_t prow = mine ? (int64_t)P_idx[i * d + lane] * r : 0;
    for (int k0 = 0; k0 < d; k0 += 4) {
        int a[4];
        float acc[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            a[q] = P_idx[i * d + min(k0 + q, d - 1)];
            acc[q] = mine ? pv * M1[prow + a[q]] : 0.0f;
        }
        for (int b = lane; b < r; b += 64) {
            const float t = Ti[b];
#pragma unroll
            for (int q = 0; q < 4; ++q) acc[q] = fmaf(t, Dm[(int64_t)a[q] * r + b], acc[q]);
        }
#pragma unroll
        for (int q = 0; q < 4; ++q) {
#pragma unroll
            for (int off = 32; off > 0; off >>= 1) acc[q] += __shfl_down(acc[q], off);
            if (lane == 0 && k0 + q < d) gP[i * d + k0 + q] = acc[q];
        }
    }
}

// gQ[j][k] = sum_k' Q_val[j][k'] M2[Q_idx[j][k']][b] + sum_a Y[a][j] D[a][b],  b = Q_idx[j][k].  The second sum
// gathers one element of every row of D per (j, k): from memory that is one cache line per term.  So a workgroup
// takes 128 columns j and a slice of the range of a, brings the rows of D of that slice (and the matching piece
// of Y) through LDS a few rows at a time, and every thread gathers from LDS: thread (j, g) owns entry k = k0 + g
// of column j, eight entries of a column at a time.  Each slice leaves its sums in a list of its own (the terms
// of the first sum are dealt over the slices as well), and k_grad_right_finish adds the lists in slice order.
constexpr int kGradCols = 128, kGradEnt = 8, kGradThreads = kGradCols * kGradEnt;
constexpr int kGradLdsFloats = 8192;                                // rows of D staged at a time: kGradLdsFloats / r, at most 16
constexpr int kGradMaxRows = 16, kGradMaxSlices = 16;
__global__ __launch_bounds__(kGradThreads) void k_grad_right(const float* __restrict__ Y, const float* __restrict__ Dm, const float* __restrict__ M2,
                                                           const int32_t* __restrict__ Q_idx, const float* __restrict__ Q_val,
                                                           int n, int r, int d, int rows, int a_per_slice, float* __restrict__ part) {
    __shared__ float Ds[kGradLdsFloats];
    __shared__ float Ys[kGradMaxRows][kGradCols];
    const int jl = threadIdx.x % kGradCols, g = threadIdx.x / kGradCols;
    const int64_t j0 = (int64_t)blockIdx.x * kGradCols, j = j0 + jl;
    const int a_begin = blockIdx.y * a_per_slice, a_end = min(r, a_begin + a_per_slice);
    for (int k0 = 0; k0 < d; k0 += kGradEnt) {
        const bool mine = j < n && k0 + g < d;
        const int b = mine ? Q_idx[j * d + k0 + g] : 0;
        float acc = 0.0f;
        for (int a0 = a_begin; a0 < a_end; a0 += rows) {
            const int here = min(rows, a_end - a0);
            __syncthreads();                                        // the previous rows have been used
            for (int q = threadIdx.x; q < here * r; q += kGradThreads) Ds[q] = Dm[(int64_t)a0 * r + q];
            for (int q = threadIdx.x; q < here * kGradCols; q += kGradThreads) {
                const int64_t jj = j0 + q % kGradCols;
                Ys[q / kGradCols][q % kGradCols] = jj < n ? Y[(int64_t)(a0 + q / kGradCols) * n + jj] : 0.0f;
            }
            __syncthreads();
            for (int t = 0; t < here; ++t) acc = fmaf(Ys[t][jl], Ds[t * r + b], acc);
        }
        if (mine) {
            for (int k2 = blockIdx.y; k2 < d; k2 += gridDim.y)      // the terms of the first sum, dealt over the slices
                acc = fmaf(Q_val[j * d + k2], M2[(int64_t)Q_idx[j * d + k2] * r + b], acc);
            part[(int64_t)blockIdx.y * n * d + j * d + k0 + g] = acc;
        }
    }
}

__global__ __launch_bounds__(256) void k_grad_right_finish(const float* __restrict__ part, float* __restrict__ gQ, int64_t count, int slices) {
    for (int64_t k = (int64_t)blockIdx.x * 256 + threadIdx.x; k < count; k += (int64_t)gridDim.x * 256) {
        float s = part[k];
        for (int q = 1; q < slices; ++q) s += part[(int64_t)q * count + k];
        gQ[k] = s;
    }
}

// floats of workspace: T (m r) | S, C_P, C_Q, S1, X, D, M1, M2 (8 r^2) | Y (r n) | the slices' lists of gQ
size_t fitgrad_workspace_floats(int64_t m, int64_t n, int32_t r, int32_t d) {
    const size_t rr = (size_t)r * (size_t)r;
    return align_up((size_t)m * r, 64) + 8 * align_up(rr, 64) + align_up((size_t)r * (size_t)n, 64) + (size_t)kGradMaxSlices * (size_t)n * d;
}

template <typename D>
static hipError_t launch_gather(const void* G, const uint8_t* plan, float* Y, int64_t m, int64_t n, int32_t r, int32_t d, hipStream_t st) {
    using E = typename D::elem;
    const int items = (int)plan_max_items(m, r, d);
    auto launch = [&](auto vec) {
        constexpr int VEC = decltype(vec)::value;
        const int tiles = (int)((n + (int64_t)kWave * VEC - 1) / ((int64_t)kWave * VEC));
        const int64_t grid = (int64_t)items * ((tiles + kXcds - 1) / kXcds) * kXcds;
        if (grid > INT32_MAX) return hipErrorInvalidValue;
        hipLaunchKernelGGL((k_gather_rows<D, VEC>), dim3((unsigned)grid), dim3(kThreadsY), 0, st, static_cast<const E*>(G), plan, Y,
                           (int)m, (int)n, (int)r, (int)d, items, tiles);
        return hipGetLastError();
    };
    // four columns per lane when rows start on the piece's alignment (G itself is 16-byte aligned)
    if (n % 4 == 0) return launch(std::integral_constant<int, 4>{});
    return launch(std::integral_constant<int, 1>{});
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
    float* gq_part = Y + align_up((size_t)r * (size_t)n, 64);
    hipError_t e;
    // T = G Q and S = P^T T: the compress kernels (a plan of another problem leaves S full of NaN, which then
    // reaches every output)
    CompressGroup g;
    memset(&g, 0, sizeof(g));
    g.count = 1; g.G[0] = G; g.plan[0] = plan; g.T[0] = T; g.S[0] = S; g.m[0] = (int32_t)m; g.n[0] = (int32_t)n;
    if ((e = launch_compress_planned(g, r, d, dtype, st)) != hipSuccess) return e;
    // C_P = P^T P, C_Q = Q^T Q
    GramBatch grams{};
    grams.p[0] = GramPair{P_idx, P_val, P_idx, P_val, m, CP};
    grams.p[1] = GramPair{Q_idx, Q_val, Q_idx, Q_val, n, CQ};
    if ((e = launch_gram(grams, 2, d, r, st)) != hipSuccess) return e;
    // the r x r chain: two launches of independent products
    GemmBatch first{}, second{};
    first.p[0] = GemmProblem{S, CQ, S1, nullptr, 0.0f, 0};                                               // S1 = S C_Q
    first.p[1] = GemmProblem{CP, S, X, nullptr, 0.0f, 0};                                                // X  = C_P S
    second.p[0] = GemmProblem{CP, S1, Dm, S, -2.0f, 0};                                                  // D  = C_P S1 - 2 S
    second.p[1] = GemmProblem{S1, S, M1, nullptr, 0.0f, kGemmTB};                                        // M1 = S1 S^T
    second.p[2] = GemmProblem{S, X, M2, nullptr, 0.0f, kGemmTA};                                         // M2 = S^T X
    if ((e = launch_gemm_rr_batch(first, 2, r, st)) != hipSuccess) return e;
    if ((e = launch_gemm_rr_batch(second, 3, r, st)) != hipSuccess) return e;
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
    // enough slices of the range of a for two workgroups per CU, each a whole number of LDS loads
    const int rows = std::max(1, std::min(kGradMaxRows, kGradLdsFloats / (int)r));
    const int colblocks = (int)((n + kGradCols - 1) / kGradCols);
    const int want = std::max(1, std::min({(512 + colblocks - 1) / colblocks, ((int)r + rows - 1) / rows, kGradMaxSlices}));
    const int a_per_slice = (((int)r + want - 1) / want + rows - 1) / rows * rows;
    const int slices = ((int)r + a_per_slice - 1) / a_per_slice;
    hipLaunchKernelGGL(k_grad_right, dim3((unsigned)colblocks, (unsigned)slices), dim3(kGradThreads), 0, st, Y, Dm, M2, Q_idx, Q_val,
                       (int)n, (int)r, (int)d, rows, a_per_slice, gq_part);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    const int64_t count = n * d;
    hipLaunchKernelGGL(k_grad_right_finish, dim3((unsigned)std::min<int64_t>((count + 255) / 256, 2048)), dim3(256), 0, st, gq_part, gQ, count, slices);
    return hipGetLastError();
}

}  // namespace lsp
