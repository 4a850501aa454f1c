// Optimiser-state re-projection (MaybeUpdate in Alg. 1, its last two assignments): when the
// projectors of a matrix are replaced, the subspace moments follow,
//     M <- (P^T P_prev) M (Q_prev^T Q),      V <- (P^T P_prev)^2 V (Q_prev^T Q)^2,
// the squares taken element by element.  Two steps:
//   1. A = P^T P_prev and B = Q_prev^T Q, r x r: products of two ELL matrices with the same rows;
//      row i adds its d x d products val * val' at (idx, idx').  Scatter with fp32 atomics (a few
//      hundred thousand of them on a 1 MB matrix that stays in L2).
//   2. four dense r x r products in fp32 on the matrix cores (v_mfma_f32_32x32x2_f32): X = A M,
//      M = X B, X = (A o A) V, V = X (B o B); the squares are taken while the tiles are staged.
// Runs once per change of projectors; nothing here is on the per-step path.
#include "lsp_internal.h"

namespace lsp {

typedef float f32x16 __attribute__((ext_vector_type(16)));

__global__ __launch_bounds__(256) void k_zero(float* __restrict__ p, int64_t count) {
    for (int64_t k = (int64_t)blockIdx.x * 256 + threadIdx.x; k < count; k += (int64_t)gridDim.x * 256) p[k] = 0.0f;
}

// C[L_idx[i][k]][R_idx[i][k']] += L_val[i][k] * R_val[i][k']  for all rows i: C = L^T R.
// One thread per (row, k, k').
__global__ __launch_bounds__(256) void k_gram(const int32_t* __restrict__ L_idx, const float* __restrict__ L_val,
                                              const int32_t* __restrict__ R_idx, const float* __restrict__ R_val,
                                              int64_t rows, int d, int r, float* __restrict__ C) {
    const int64_t total = rows * d * d;
    for (int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x; t < total; t += (int64_t)gridDim.x * 256) {
        const int64_t i = t / (d * d);
        const int k = (int)(t - i * d * d) / d, k2 = (int)(t - i * d * d) % d;
        const float v = L_val[i * d + k] * R_val[i * d + k2];
        if (v != 0.0f) atomicAdd(&C[(int64_t)L_idx[i * d + k] * r + R_idx[i * d + k2]], v);
    }
}

// C = op(A) op(B) + beta E, all r x r row-major fp32; op squares every element (SQ*) or transposes the
// operand (T*) while its tiles are staged.
// A workgroup of four waves makes a 32 x 32 tile of C (many small tiles: r is a few hundred, and
// every CU should get one).  The K range goes by in 64-wide tiles staged through LDS; inside a
// tile the four waves take 16 consecutive k each with v_mfma_f32_32x32x2_f32 -- lane l supplies
// A[i = l % 32][k = l / 32] and B[k = l / 32][j = l % 32] and holds
// C[8 (v / 4) + 4 (l / 32) + v % 4][l % 32] in accumulator register v -- and their four partial
// tiles are added through LDS at the end, in wave order.
constexpr int kTileMN = 32, kTileK = 64;
constexpr int kTileElems = kTileMN * kTileK / 256;                  // elements of each tile a thread stages
template <bool SQA, bool SQB, bool TA, bool TB>
__global__ __launch_bounds__(256) void k_gemm_rr(const float* __restrict__ A, const float* __restrict__ B,
                                                 float* __restrict__ C, int r, float beta, const float* __restrict__ E) {
    __shared__ float As[kTileMN][kTileK + 1];
    __shared__ float Bs[kTileK][kTileMN + 1];
    __shared__ float Cs[4][16][64];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int row0 = blockIdx.y * kTileMN, col0 = blockIdx.x * kTileMN;
    f32x16 acc;
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[v] = 0.0f;
    // the next pair of tiles is fetched into registers while the matrix cores work on the current one;
    // consecutive threads read consecutive addresses whichever way the operand lies in memory
    float an[kTileElems], bn[kTileElems];
    auto fetch = [&](int k0) {
#pragma unroll
        for (int e = 0; e < kTileElems; ++e) {
            const int q = tid + e * 256;
            const int ar = TA ? q % kTileMN : q / kTileK, ak = TA ? q / kTileMN : q % kTileK;
            const bool aok = row0 + ar < r && k0 + ak < r;
            const float a = !aok ? 0.0f : TA ? A[(int64_t)(k0 + ak) * r + row0 + ar] : A[(int64_t)(row0 + ar) * r + k0 + ak];
            an[e] = SQA ? a * a : a;
            const int bk = TB ? q % kTileK : q / kTileMN, bc = TB ? q / kTileK : q % kTileMN;
            const bool bok = k0 + bk < r && col0 + bc < r;
            const float b = !bok ? 0.0f : TB ? B[(int64_t)(col0 + bc) * r + k0 + bk] : B[(int64_t)(k0 + bk) * r + col0 + bc];
            bn[e] = SQB ? b * b : b;
        }
    };
    fetch(0);
    for (int k0 = 0; k0 < r; k0 += kTileK) {
#pragma unroll
        for (int e = 0; e < kTileElems; ++e) {
            const int q = tid + e * 256;
            As[TA ? q % kTileMN : q / kTileK][TA ? q / kTileMN : q % kTileK] = an[e];
            Bs[TB ? q % kTileK : q / kTileMN][TB ? q / kTileK : q % kTileMN] = bn[e];
        }
        __syncthreads();
        if (k0 + kTileK < r) fetch(k0 + kTileK);
#pragma unroll
        for (int kk = wave * (kTileK / 4); kk < (wave + 1) * (kTileK / 4); kk += 2)
            acc = __builtin_amdgcn_mfma_f32_32x32x2f32(As[lane & 31][kk + (lane >> 5)],
                                                       Bs[kk + (lane >> 5)][lane & 31], acc, 0, 0, 0);
        __syncthreads();
    }
#pragma unroll
    for (int v = 0; v < 16; ++v) Cs[wave][v][lane] = acc[v];
    __syncthreads();
    if (wave == 0) {
        const int j = col0 + (lane & 31);
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int i = row0 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
            float sum = ((Cs[0][v][lane] + Cs[1][v][lane]) + Cs[2][v][lane]) + Cs[3][v][lane];
            if (i < r && j < r) {
                if (E) sum = fmaf(beta, E[(int64_t)i * r + j], sum);
                C[(int64_t)i * r + j] = sum;
            }
        }
    }
}

static dim3 blocks_for(int64_t count) { return dim3((unsigned)((count + 255) / 256 > 2048 ? 2048 : (count + 255) / 256)); }

hipError_t launch_zero(float* p, int64_t count, hipStream_t st) {
    hipLaunchKernelGGL(k_zero, blocks_for(count), dim3(256), 0, st, p, count);
    return hipGetLastError();
}

hipError_t launch_gram(const int32_t* L_idx, const float* L_val, const int32_t* R_idx, const float* R_val,
                       int64_t rows, int32_t d, int32_t r, float* C, hipStream_t st) {
    hipLaunchKernelGGL(k_gram, blocks_for(rows * d * d), dim3(256), 0, st, L_idx, L_val, R_idx, R_val, rows, (int)d, (int)r, C);
    return hipGetLastError();
}

hipError_t launch_gemm_rr(const float* A, const float* B, float* C, int32_t r, bool ta, bool tb,
                          float beta, const float* E, hipStream_t st) {
    const dim3 grid((unsigned)((r + kTileMN - 1) / kTileMN), (unsigned)((r + kTileMN - 1) / kTileMN));
    if (ta && tb) return hipErrorInvalidValue;                       // not needed anywhere
    if (ta)      hipLaunchKernelGGL((k_gemm_rr<false, false, true, false>), grid, dim3(256), 0, st, A, B, C, (int)r, beta, E);
    else if (tb) hipLaunchKernelGGL((k_gemm_rr<false, false, false, true>), grid, dim3(256), 0, st, A, B, C, (int)r, beta, E);
    else         hipLaunchKernelGGL((k_gemm_rr<false, false, false, false>), grid, dim3(256), 0, st, A, B, C, (int)r, beta, E);
    return hipGetLastError();
}

hipError_t launch_reproject(const int32_t* P_idx, const float* P_val, const int32_t* Pp_idx, const float* Pp_val,
                            const int32_t* Q_idx, const float* Q_val, const int32_t* Qp_idx, const float* Qp_val,
                            int64_t m, int64_t n, int32_t r, int32_t d, float* M, float* V, float* workspace,
                            hipStream_t st) {
    const int64_t rr = (int64_t)r * r;
    float* A = workspace;
    float* B = workspace + rr;
    float* X = workspace + 2 * rr;
    hipLaunchKernelGGL(k_zero, blocks_for(2 * rr), dim3(256), 0, st, A, 2 * rr);
    hipLaunchKernelGGL(k_gram, blocks_for(m * d * d), dim3(256), 0, st, P_idx, P_val, Pp_idx, Pp_val, m, (int)d, (int)r, A);
    hipLaunchKernelGGL(k_gram, blocks_for(n * d * d), dim3(256), 0, st, Qp_idx, Qp_val, Q_idx, Q_val, n, (int)d, (int)r, B);
    const dim3 grid((unsigned)((r + kTileMN - 1) / kTileMN), (unsigned)((r + kTileMN - 1) / kTileMN));
    const float* none = nullptr;
    hipLaunchKernelGGL((k_gemm_rr<false, false, false, false>), grid, dim3(256), 0, st, A, M, X, (int)r, 0.0f, none);
    hipLaunchKernelGGL((k_gemm_rr<false, false, false, false>), grid, dim3(256), 0, st, X, B, M, (int)r, 0.0f, none);
    if (V) {
        hipLaunchKernelGGL((k_gemm_rr<true, false, false, false>), grid, dim3(256), 0, st, A, V, X, (int)r, 0.0f, none);
        hipLaunchKernelGGL((k_gemm_rr<false, true, false, false>), grid, dim3(256), 0, st, X, B, V, (int)r, 0.0f, none);
    }
    return hipGetLastError();
}

}  // namespace lsp
