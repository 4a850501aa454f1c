// Dense-projector ablation of the compress step (Def. 1 makes the projectors (d, r)-sparse; with dense
// projectors of the same shape S = P^T G Q is a plain contraction and belongs on the matrix cores):
//     T^T = Q^T G^T   (r x m, kept in storage precision),      S = P^T T   (r x r, fp32).
// Both products are C[M][N] = sum_k A[M][k] B[N][k] with A and B stored row-major and k running along
// the rows ("NT"), which is how all four operands lie when the caller hands in the transposed dense
// projectors P^T (r x m) and Q^T (r x n): G (m x n) is B of the first product, its result T^T (r x m) is
// B of the second.  One kernel serves both.
//
// A workgroup of four waves makes a 64 x 128 tile of C; wave (wm, wn) the 32 x 64 part at (32 wm, 64 wn)
// as two 32 x 32 tiles of v_mfma_f32_32x32x16 (bf16 or f16): lane l supplies A[i = l % 32][k = 8 (l / 32) ..
// + 7] and B[j = l % 32][the same k] as one 128-bit register group each and holds
// C[8 (v / 4) + 4 (l / 32) + v % 4][l % 32] in accumulator register v.  The K range goes by in 64-wide
// tiles through LDS (rows padded by 16 bytes, so that the 16 lanes that read together hit 16 different
// bank quads); the next pair of tiles is fetched into registers while the matrix cores work on the current one.
// The second product has few tiles (r x r) and a long K (= m): its K range is cut into slices that write
// partial sums, added in a fixed order by a small kernel (no atomics: the result does not depend on timing).
#include "lsp_internal.h"

namespace lsp {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));

constexpr int kDenseBM = 64, kDenseBN = 128, kDenseBK = 64;
constexpr int kDenseThreads = 256;
constexpr int kDenseRowBytes = kDenseBK * 2 + 16;                   // one row of a tile in LDS
constexpr int kDenseSlices = 8;                                     // K slices of the second product

template <typename D> __device__ __forceinline__ f32x16 mfma_32x32x16(u32x4 a, u32x4 b, f32x16 c);
template <> __device__ __forceinline__ f32x16 mfma_32x32x16<BF16>(u32x4 a, u32x4 b, f32x16 c) {
    bf16x8 x, y;
    __builtin_memcpy(&x, &a, 16); __builtin_memcpy(&y, &b, 16);
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(x, y, c, 0, 0, 0);
}
template <> __device__ __forceinline__ f32x16 mfma_32x32x16<F16>(u32x4 a, u32x4 b, f32x16 c) {
    f16x8 x, y;
    __builtin_memcpy(&x, &a, 16); __builtin_memcpy(&y, &b, 16);
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(x, y, c, 0, 0, 0);
}

// C (+ slice * M * N when SPLIT) = A[M][k0 .. k1) B[N][k0 .. k1)^T.  M % 64 == 0, N % 128 == 0, K % 64 == 0
// (checked by the caller); lda = ldb = K elements.  OUT16: C is stored in the storage type, else in fp32.
template <typename D, bool OUT16>
__global__ __launch_bounds__(kDenseThreads) void k_dense_nt(const typename D::elem* __restrict__ A, const typename D::elem* __restrict__ B,
                                                            void* __restrict__ Cout, int M, int N, int K, int kslice) {
    __shared__ __align__(16) uint8_t As[kDenseBM * kDenseRowBytes];
    __shared__ __align__(16) uint8_t Bs[kDenseBN * kDenseRowBytes];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int row0 = blockIdx.y * kDenseBM, col0 = blockIdx.x * kDenseBN;
    const int k_begin = blockIdx.z * kslice, k_end = min(K, k_begin + kslice);
    f32x16 acc[2];
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[t][v] = 0.0f;
    // a thread stages 2 x 16 bytes of the A tile (64 rows x 128 bytes) and 4 x 16 bytes of the B tile (128 rows)
    u32x4 an[2], bn[4];
    auto fetch = [&](int k0) {
#pragma unroll
        for (int e = 0; e < 2; ++e) {
            const int q = tid + e * kDenseThreads, rr = q >> 3, seg = q & 7;
            an[e] = *reinterpret_cast<const u32x4*>(A + (int64_t)(row0 + rr) * K + k0 + seg * 8);
        }
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int q = tid + e * kDenseThreads, rr = q >> 3, seg = q & 7;
            bn[e] = stream_load(reinterpret_cast<const u32x4*>(B + (int64_t)(col0 + rr) * K + k0 + seg * 8));
        }
    };
    fetch(k_begin);
    for (int k0 = k_begin; k0 < k_end; k0 += kDenseBK) {
#pragma unroll
        for (int e = 0; e < 2; ++e) {
            const int q = tid + e * kDenseThreads;
            *reinterpret_cast<u32x4*>(As + (q >> 3) * kDenseRowBytes + (q & 7) * 16) = an[e];
        }
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int q = tid + e * kDenseThreads;
            *reinterpret_cast<u32x4*>(Bs + (q >> 3) * kDenseRowBytes + (q & 7) * 16) = bn[e];
        }
        __syncthreads();
        if (k0 + kDenseBK < k_end) fetch(k0 + kDenseBK);
        const uint8_t* ap = As + (wm * 32 + (lane & 31)) * kDenseRowBytes + (lane >> 5) * 16;
        const uint8_t* bp = Bs + (wn * 64 + (lane & 31)) * kDenseRowBytes + (lane >> 5) * 16;
#pragma unroll
        for (int kk = 0; kk < kDenseBK / 16; ++kk) {                // 16 k per instruction: 32 bytes of a row
            const u32x4 a = *reinterpret_cast<const u32x4*>(ap + kk * 32);
            const u32x4 b0 = *reinterpret_cast<const u32x4*>(bp + kk * 32);
            const u32x4 b1 = *reinterpret_cast<const u32x4*>(bp + 32 * kDenseRowBytes + kk * 32);
            acc[0] = mfma_32x32x16<D>(a, b0, acc[0]);
            acc[1] = mfma_32x32x16<D>(a, b1, acc[1]);
        }
        __syncthreads();
    }
    const int64_t base = (int64_t)blockIdx.z * M * N;
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int i = row0 + wm * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
            const int j = col0 + wn * 64 + t * 32 + (lane & 31);
            if constexpr (OUT16) static_cast<typename D::elem*>(Cout)[(int64_t)i * N + j] = narrow<D>(acc[t][v]);
            else static_cast<float*>(Cout)[base + (int64_t)i * N + j] = acc[t][v];
        }
}

// S = sum of the slices' partial sums, in slice order
__global__ __launch_bounds__(256) void k_dense_reduce(const float* __restrict__ part, float* __restrict__ S, int64_t count, int slices) {
    for (int64_t k = (int64_t)blockIdx.x * 256 + threadIdx.x; k < count; k += (int64_t)gridDim.x * 256) {
        float s = part[k];
        for (int q = 1; q < slices; ++q) s += part[(int64_t)q * count + k];
        S[k] = s;
    }
}

size_t dense_workspace_bytes(int64_t m, int32_t r) {
    return align_up((size_t)r * (size_t)m * 2, 256) + (size_t)kDenseSlices * r * r * sizeof(float);
}

template <typename D>
static hipError_t launch_dense_t(const void* G, const void* Pt, const void* Qt, int64_t m, int64_t n, int32_t r, float* S,
                                 uint8_t* ws, hipStream_t st) {
    using E = typename D::elem;
    E* Tt = reinterpret_cast<E*>(ws);
    float* part = reinterpret_cast<float*>(ws + align_up((size_t)r * (size_t)m * 2, 256));
    // T^T [r][m] = Q^T [r][n] (G [m][n])^T
    hipLaunchKernelGGL((k_dense_nt<D, true>), dim3((unsigned)(m / kDenseBN), (unsigned)(r / kDenseBM), 1), dim3(kDenseThreads), 0, st,
                       static_cast<const E*>(Qt), static_cast<const E*>(G), static_cast<void*>(Tt), (int)r, (int)m, (int)n, (int)n);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    // S [r][r] = P^T [r][m] (T^T [r][m])^T, K = m in slices of whole tiles
    const int kslice = (int)(((m / kDenseBK + kDenseSlices - 1) / kDenseSlices) * kDenseBK);
    const int slices = (int)((m + kslice - 1) / kslice);
    hipLaunchKernelGGL((k_dense_nt<D, false>), dim3((unsigned)(r / kDenseBN), (unsigned)(r / kDenseBM), (unsigned)slices), dim3(kDenseThreads), 0, st,
                       static_cast<const E*>(Pt), static_cast<const E*>(Tt), static_cast<void*>(part), (int)r, (int)r, (int)m, kslice);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    const int64_t rr = (int64_t)r * r;
    hipLaunchKernelGGL(k_dense_reduce, dim3((unsigned)((rr + 255) / 256)), dim3(256), 0, st, part, S, rr, slices);
    return hipGetLastError();
}

bool dense_shape_ok(int64_t m, int64_t n, int32_t r) {
    return m % kDenseBN == 0 && n % kDenseBK == 0 && r % kDenseBN == 0;
}

hipError_t launch_compress_dense(const void* G, const void* Pt, const void* Qt, int64_t m, int64_t n, int32_t r, float* S,
                                 uint8_t* workspace, lsp_dtype dtype, hipStream_t st) {
    return dtype == LSP_F16 ? launch_dense_t<F16>(G, Pt, Qt, m, n, r, S, workspace, st)
                            : launch_dense_t<BF16>(G, Pt, Qt, m, n, r, S, workspace, st);
}

}  // namespace lsp
