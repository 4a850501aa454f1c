// Decompress and apply:  W <- rn(W - P S Q^T)  (Alg. 1, apply step; Alg. 3, last step of the
// layer loop).  One kernel, one fused read-modify-write pass over W:
//   phase 1  U = P S for the workgroup's R rows of W (gathers d rows of S per row, S stays in
//            L2), stored in LDS as [4-row plane][column b][4 rows] fp32;
//   phase 2  every thread owns CPT consecutive columns j, keeps the d (column, value) pairs of
//            their rows of Q in registers, and for each 4-row plane gathers U with one 128-bit
//            LDS read per pair; W is read, updated in fp32 and rounded once.
// Bandwidth-bound (read + write of W); no matrix cores (sparse gather + fp32 FMA).
#include "lsp_internal.h"

namespace lsp {

constexpr int kThreadsD = 256;

template <typename D, int CPT> struct Vec;     // CPT consecutive elements of W
template <> struct Vec<F32, 4>  { float4 v; };
template <> struct Vec<F16, 4>  { uint2 v; };
template <> struct Vec<BF16, 4> { uint2 v; };

template <typename D> __device__ __forceinline__ void vec_widen(const Vec<D, 4>& x, float out[4]);
template <> __device__ __forceinline__ void vec_widen<F32>(const Vec<F32, 4>& x, float out[4]) {
    out[0] = x.v.x; out[1] = x.v.y; out[2] = x.v.z; out[3] = x.v.w;
}
template <> __device__ __forceinline__ void vec_widen<F16>(const Vec<F16, 4>& x, float out[4]) {
    out[0] = widen<F16>((uint16_t)(x.v.x & 0xFFFFu)); out[1] = widen<F16>((uint16_t)(x.v.x >> 16));
    out[2] = widen<F16>((uint16_t)(x.v.y & 0xFFFFu)); out[3] = widen<F16>((uint16_t)(x.v.y >> 16));
}
template <> __device__ __forceinline__ void vec_widen<BF16>(const Vec<BF16, 4>& x, float out[4]) {
    out[0] = __uint_as_float(x.v.x << 16); out[1] = __uint_as_float(x.v.x & 0xFFFF0000u);
    out[2] = __uint_as_float(x.v.y << 16); out[3] = __uint_as_float(x.v.y & 0xFFFF0000u);
}
template <typename D> __device__ __forceinline__ Vec<D, 4> vec_narrow(const float in[4]);
template <> __device__ __forceinline__ Vec<F32, 4> vec_narrow<F32>(const float in[4]) {
    return {make_float4(in[0], in[1], in[2], in[3])};
}
template <> __device__ __forceinline__ Vec<F16, 4> vec_narrow<F16>(const float in[4]) {
    return {make_uint2((uint32_t)narrow<F16>(in[0]) | ((uint32_t)narrow<F16>(in[1]) << 16),
                       (uint32_t)narrow<F16>(in[2]) | ((uint32_t)narrow<F16>(in[3]) << 16))};
}
template <> __device__ __forceinline__ Vec<BF16, 4> vec_narrow<BF16>(const float in[4]) {
    return {make_uint2((uint32_t)narrow<BF16>(in[0]) | ((uint32_t)narrow<BF16>(in[1]) << 16),
                       (uint32_t)narrow<BF16>(in[2]) | ((uint32_t)narrow<BF16>(in[3]) << 16))};
}

// phase 1, shared by both kernels:  Us[plane][b] (float4 = 4 rows) = sum_k P_val[i][k] S[P_idx[i][k]][b]
// `plane` is the distance between planes in float4 units (>= r).
template <int RG>
__device__ __forceinline__ void build_u_tile(float4* Us, const float* __restrict__ S,
                                             const int32_t* __restrict__ P_idx, const float* __restrict__ P_val,
                                             int64_t i0, int m, int r, int d, int plane) {
    for (int b = threadIdx.x; b < r; b += kThreadsD) {
#pragma unroll
        for (int g = 0; g < RG; ++g) {
            float u[4] = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const int64_t i = i0 + g * 4 + t;
                if (i < m) {
                    for (int k = 0; k < d; ++k) {
                        const int a = P_idx[i * d + k];           // uniform over the workgroup
                        const float v = P_val[i * d + k];
                        u[t] = fmaf(v, S[(int64_t)a * r + b], u[t]);
                    }
                }
            }
            Us[g * plane + b] = make_float4(u[0], u[1], u[2], u[3]);
        }
    }
}

// Fast kernel: DD = compile-time d, 4 columns per thread, n % 4 == 0.  PS = bytes between the
// 4-row planes of U in LDS, a compile-time constant >= 16 r so that the plane offset folds into the
// immediate offset of the LDS read and a gather costs no address arithmetic.
template <typename D, int RG, int DD, int PS>
__global__ __launch_bounds__(kThreadsD) void k_decompress(typename D::elem* __restrict__ W, const float* __restrict__ S,
                                                         const int32_t* __restrict__ P_idx, const float* __restrict__ P_val,
                                                         const int32_t* __restrict__ Q_idx, const float* __restrict__ Q_val,
                                                         int m, int n, int r) {
    extern __shared__ __align__(16) uint8_t smem[];
    float4* Us = reinterpret_cast<float4*>(smem);
    constexpr int R = 4 * RG;
    constexpr int CPT = 4;
    const int64_t i0 = (int64_t)blockIdx.x * R;
    build_u_tile<RG>(Us, S, P_idx, P_val, i0, m, r, DD, PS / 16);
    __syncthreads();

    for (int64_t j0 = (int64_t)threadIdx.x * CPT; j0 < n; j0 += (int64_t)kThreadsD * CPT) {
        // the CPT rows of Q owned by this thread: DD (column, value) pairs each
        uint32_t off[CPT][DD];
        float val[CPT][DD];
        const int32_t* qi = Q_idx + j0 * DD;
        const float* qv = Q_val + j0 * DD;
#pragma unroll
        for (int c = 0; c < CPT; ++c)
#pragma unroll
            for (int k = 0; k < DD; ++k) {
                off[c][k] = (uint32_t)qi[c * DD + k] * 16u;
                val[c][k] = qv[c * DD + k];
            }
#pragma unroll
        for (int g = 0; g < RG; ++g) {
            float acc[4][CPT];
#pragma unroll
            for (int t = 0; t < 4; ++t)
#pragma unroll
                for (int c = 0; c < CPT; ++c) acc[t][c] = 0.0f;
#pragma unroll
            for (int c = 0; c < CPT; ++c)
#pragma unroll
                for (int k = 0; k < DD; ++k) {
                    const float4 u = *reinterpret_cast<const float4*>(smem + off[c][k] + g * PS);
                    acc[0][c] = fmaf(val[c][k], u.x, acc[0][c]);
                    acc[1][c] = fmaf(val[c][k], u.y, acc[1][c]);
                    acc[2][c] = fmaf(val[c][k], u.z, acc[2][c]);
                    acc[3][c] = fmaf(val[c][k], u.w, acc[3][c]);
                }
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const int64_t i = i0 + g * 4 + t;
                if (i < m) {
                    Vec<D, CPT>* p = reinterpret_cast<Vec<D, CPT>*>(W + i * (int64_t)n + j0);
                    float w[4];
                    vec_widen<D>(*p, w);
#pragma unroll
                    for (int c = 0; c < CPT; ++c) w[c] -= acc[t][c];
                    *p = vec_narrow<D>(w);
                }
            }
        }
    }
}

// Generic kernel: any n and d, one column per thread.
template <typename D, int RG>
__global__ __launch_bounds__(kThreadsD) void k_decompress_any(typename D::elem* __restrict__ W, const float* __restrict__ S,
                                                             const int32_t* __restrict__ P_idx, const float* __restrict__ P_val,
                                                             const int32_t* __restrict__ Q_idx, const float* __restrict__ Q_val,
                                                             int m, int n, int r, int d) {
    extern __shared__ __align__(16) uint8_t smem[];
    float4* Us = reinterpret_cast<float4*>(smem);
    constexpr int R = 4 * RG;
    const int64_t i0 = (int64_t)blockIdx.x * R;
    build_u_tile<RG>(Us, S, P_idx, P_val, i0, m, r, d, r);
    __syncthreads();
    for (int64_t j = threadIdx.x; j < n; j += kThreadsD) {
        float acc[RG][4];
#pragma unroll
        for (int g = 0; g < RG; ++g) acc[g][0] = acc[g][1] = acc[g][2] = acc[g][3] = 0.0f;
        for (int k = 0; k < d; ++k) {
            const int b = Q_idx[j * d + k];
            const float v = Q_val[j * d + k];
#pragma unroll
            for (int g = 0; g < RG; ++g) {
                const float4 u = Us[g * r + b];
                acc[g][0] = fmaf(v, u.x, acc[g][0]); acc[g][1] = fmaf(v, u.y, acc[g][1]);
                acc[g][2] = fmaf(v, u.z, acc[g][2]); acc[g][3] = fmaf(v, u.w, acc[g][3]);
            }
        }
#pragma unroll
        for (int g = 0; g < RG; ++g)
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const int64_t i = i0 + g * 4 + t;
                if (i < m) {
                    typename D::elem* p = W + i * (int64_t)n + j;
                    *p = narrow<D>(widen<D>(*p) - acc[g][t]);
                }
            }
    }
}

template <typename D, int RG, int PS>
static hipError_t launch_d(void* W, const float* S, const int32_t* P_idx, const float* P_val,
                           const int32_t* Q_idx, const float* Q_val, int64_t m, int64_t n, int32_t r, int32_t d,
                           hipStream_t st) {
    using E = typename D::elem;
    const unsigned grid = (unsigned)((m + RG * 4 - 1) / (RG * 4));
    const bool fast = (n % 4) == 0 && (d == 2 || d == 4 || d == 8 || d == 16);
    hipError_t e;
#define LSP_LAUNCH_FAST(DDV)                                                                                   \
    do {                                                                                                       \
        auto kern = k_decompress<D, RG, DDV, PS>;                                                              \
        const size_t lds = (size_t)RG * PS;                                                                    \
        e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds); \
        if (e != hipSuccess) return e;                                                                         \
        hipLaunchKernelGGL(kern, dim3(grid), dim3(kThreadsD), lds, st, reinterpret_cast<E*>(W), S, P_idx, P_val, \
                           Q_idx, Q_val, (int)m, (int)n, (int)r);                                              \
    } while (0)
    if (fast && d == 2) LSP_LAUNCH_FAST(2);
    else if (fast && d == 4) LSP_LAUNCH_FAST(4);
    else if (fast && d == 8) LSP_LAUNCH_FAST(8);
    else if (fast && d == 16) LSP_LAUNCH_FAST(16);
    else {
        auto kern = k_decompress_any<D, RG>;
        const size_t lds = (size_t)RG * r * 16;
        e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL(kern, dim3(grid), dim3(kThreadsD), lds, st, reinterpret_cast<E*>(W), S, P_idx, P_val,
                           Q_idx, Q_val, (int)m, (int)n, (int)r, (int)d);
    }
#undef LSP_LAUNCH_FAST
    return hipGetLastError();
}

template <typename D>
static hipError_t launch_d_rg(void* W, const float* S, const int32_t* P_idx, const float* P_val,
                              const int32_t* Q_idx, const float* Q_val, int64_t m, int64_t n, int32_t r, int32_t d,
                              hipStream_t st) {
    if (r <= 256)  return launch_d<D, 4, 4096>(W, S, P_idx, P_val, Q_idx, Q_val, m, n, r, d, st);
    if (r <= 512)  return launch_d<D, 4, 8192>(W, S, P_idx, P_val, Q_idx, Q_val, m, n, r, d, st);
    if (r <= 1024) return launch_d<D, 4, 16384>(W, S, P_idx, P_val, Q_idx, Q_val, m, n, r, d, st);
    return launch_d<D, 2, 32768>(W, S, P_idx, P_val, Q_idx, Q_val, m, n, r, d, st);
}

hipError_t launch_decompress(void* W, const float* S, const int32_t* P_idx, const float* P_val,
                             const int32_t* Q_idx, const float* Q_val,
                             int64_t m, int64_t n, int32_t r, int32_t d, lsp_dtype dtype, hipStream_t st) {
    switch (dtype) {
        case LSP_F32:  return launch_d_rg<F32>(W, S, P_idx, P_val, Q_idx, Q_val, m, n, r, d, st);
        case LSP_F16:  return launch_d_rg<F16>(W, S, P_idx, P_val, Q_idx, Q_val, m, n, r, d, st);
        default:       return launch_d_rg<BF16>(W, S, P_idx, P_val, Q_idx, Q_val, m, n, r, d, st);
    }
}

__global__ __launch_bounds__(256) void k_validate(const int32_t* __restrict__ idx, int64_t count, int r, int32_t* flag) {
    int bad = 0;
    for (int64_t k = (int64_t)blockIdx.x * 256 + threadIdx.x; k < count; k += (int64_t)gridDim.x * 256) {
        const int v = idx[k];
        bad |= (v < 0 || v >= r);
    }
    if (bad) *flag = 1;
}

__global__ void k_clear_flag(int32_t* flag) { *flag = 0; }

hipError_t launch_validate(const int32_t* idx, int64_t count, int32_t r, int32_t* flag, hipStream_t st) {
    hipLaunchKernelGGL(k_clear_flag, dim3(1), dim3(1), 0, st, flag);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const int64_t blocks = (count + 255) / 256;
    hipLaunchKernelGGL(k_validate, dim3((unsigned)(blocks > 2048 ? 2048 : blocks)), dim3(256), 0, st, idx, count, (int)r, flag);
    return hipGetLastError();
}

}  // namespace lsp
