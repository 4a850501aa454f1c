// Measurement aids: what a plain streaming kernel reaches on this GPU's HBM, for the benchmark's
// "achievable" figures beside the published peak.  Two kernels with nothing but the stream in them:
// a read-only pass (compress streams G once) and a read-modify-write pass y -= c (decompress-apply
// reads and writes W once).  Not part of the method.
#include "lsp_internal.h"

namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));
constexpr int kThreads = 256;
constexpr int kUnroll = 8;                                       // 16-byte vectors in flight per thread, read-only pass
// The read-modify-write pass is sensitive to how much a workgroup reads before it writes: with 256 threads,
// 1 / 2 / 4 / 6 / 8 / 16 vectors per thread reach 6.6 / 6.1 / 6.2 / 6.3 / 4.5 / 5.3 TB/s on 1 GiB.  The probe
// reports the best plain pattern: one vector per thread, a 4 KB tile read and written back at once.
constexpr int kUnrollRmw = 1;

__global__ __launch_bounds__(kThreads) void k_probe_read(const f32x4* __restrict__ x, size_t nvec, float* __restrict__ out) {
    const size_t tile = (size_t)kThreads * kUnroll;
    const size_t base = (size_t)blockIdx.x * tile + threadIdx.x;
    f32x4 v[kUnroll];
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
        const size_t k = base + (size_t)u * kThreads;
        v[u] = k < nvec ? __builtin_nontemporal_load(x + k) : f32x4{0.0f, 0.0f, 0.0f, 0.0f};
    }
    float s = 0.0f;
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) s += (v[u].x + v[u].y) + (v[u].z + v[u].w);
    // one store per workgroup of a value that depends on every load
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) s += __shfl_down(s, off);
    __shared__ float part[kThreads / 64];
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = s;
    __syncthreads();
    if (threadIdx.x == 0) out[blockIdx.x] = (part[0] + part[1]) + (part[2] + part[3]);
}

__global__ __launch_bounds__(kThreads) void k_probe_rmw(f32x4* __restrict__ y, size_t nvec, float c) {
    const size_t tile = (size_t)kThreads * kUnrollRmw;
    const size_t base = (size_t)blockIdx.x * tile + threadIdx.x;
    f32x4 v[kUnrollRmw];
#pragma unroll
    for (int u = 0; u < kUnrollRmw; ++u) {
        const size_t k = base + (size_t)u * kThreads;
        if (k < nvec) v[u] = __builtin_nontemporal_load(y + k);
    }
#pragma unroll
    for (int u = 0; u < kUnrollRmw; ++u) {
        const size_t k = base + (size_t)u * kThreads;
        if (k < nvec) __builtin_nontemporal_store(v[u] - c, y + k);
    }
}

}  // namespace

extern "C" {

size_t lsp_hbm_probe_workspace_bytes(size_t bytes) {
    const size_t nvec = bytes / 16, tile = (size_t)kThreads * kUnroll;
    return lsp::align_up(((nvec + tile - 1) / tile) * sizeof(float), 256);
}

int lsp_hbm_probe_read(const void* buf, size_t bytes, void* workspace, size_t workspace_bytes, void* stream) {
    if (!buf || !workspace) return LSP_ERR_NULL;
    if (bytes < 16 || bytes / 16 / ((size_t)kThreads * kUnroll) > 0x7FFFFFFFu) return LSP_ERR_SHAPE;
    if ((reinterpret_cast<uintptr_t>(buf) & 15u) || (reinterpret_cast<uintptr_t>(workspace) & 15u)) return LSP_ERR_ALIGN;
    if (workspace_bytes < lsp_hbm_probe_workspace_bytes(bytes)) return LSP_ERR_WORKSPACE;
    const size_t nvec = bytes / 16, tile = (size_t)kThreads * kUnroll;
    hipLaunchKernelGGL(k_probe_read, dim3((unsigned)((nvec + tile - 1) / tile)), dim3(kThreads), 0, static_cast<hipStream_t>(stream),
                       static_cast<const f32x4*>(buf), nvec, static_cast<float*>(workspace));
    const hipError_t e = hipGetLastError();
    return e == hipSuccess ? LSP_OK : lsp::note_hip_error(e);
}

int lsp_hbm_probe_rmw(void* buf, size_t bytes, float c, void* stream) {
    if (!buf) return LSP_ERR_NULL;
    if (bytes < 16 || bytes / 16 / ((size_t)kThreads * kUnrollRmw) > 0x7FFFFFFFu) return LSP_ERR_SHAPE;
    if (reinterpret_cast<uintptr_t>(buf) & 15u) return LSP_ERR_ALIGN;
    const size_t nvec = bytes / 16, tile = (size_t)kThreads * kUnrollRmw;
    hipLaunchKernelGGL(k_probe_rmw, dim3((unsigned)((nvec + tile - 1) / tile)), dim3(kThreads), 0, static_cast<hipStream_t>(stream),
                       static_cast<f32x4*>(buf), nvec, c);
    const hipError_t e = hipGetLastError();
    return e == hipSuccess ? LSP_OK : lsp::note_hip_error(e);
}

}  // extern "C"
