// lsp_compress_planned_static: the planned compress call for callers that cannot allocate or pass
// device scratch (code under HIP graph capture, tight serving loops, harnesses that forbid
// hipMalloc).  It is lsp_compress_planned with the m x r fp32 intermediate T = G Q placed in a
// device array that is part of the library image instead of a caller-supplied workspace; the kernels
// are the same and receive the array's address as their T argument.
//
// Every GPU the library runs on holds its own copy of the array (at its own address) until the
// process ends.  All calls on one GPU share it: two calls whose kernels overlap in time (different
// streams) race on it; calls on one stream are ordered and safe.  Nothing in it has to start at
// zero -- the first kernel writes every element of T that the second one reads -- so the contents
// left by the previous call are simply overwritten.
#include <cstring>
#include <mutex>

#include "lsp_internal.h"

namespace {

constexpr size_t kScratchBytes = LSP_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

// `scratch` above is only a host-side handle; the memory's device address differs from GPU to GPU
// and is looked up once per device, with that device current.
constexpr int kMaxDevices = 64;
std::mutex g_lock;
void* g_scratch_ptr[kMaxDevices] = {};

hipError_t scratch_address(void** out) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> hold(g_lock);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return hipSuccess;
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

}  // namespace

extern "C" {

size_t lsp_static_scratch_bytes(void) { return kScratchBytes; }

int lsp_compress_planned_static(const void* G, const void* plan, int64_t m, int64_t n, int32_t r, int32_t d,
                                float* S, lsp_dtype dtype, void* stream) {
    if (!G || !plan || !S) return LSP_ERR_NULL;
    // the shape checks of lsp_compress_planned (a zero size means an invalid shape)
    const size_t need = lsp_compress_planned_workspace_bytes(m, n, r, d);
    if (need == 0) return LSP_ERR_SHAPE;
    if (dtype != LSP_F32 && dtype != LSP_F16 && dtype != LSP_BF16) return LSP_ERR_DTYPE;
    if (need > kScratchBytes) return LSP_ERR_TOO_LARGE;
    if (!aligned16(plan)) return LSP_ERR_WORKSPACE;
    if (!aligned16(G) || !aligned16(S)) return LSP_ERR_ALIGN;
    void* T = nullptr;
    hipError_t e = scratch_address(&T);
    if (e != hipSuccess) return lsp::note_hip_error(e);
    lsp::CompressGroup g;
    std::memset(&g, 0, sizeof(g));
    g.count = 1;
    g.G[0] = G; g.plan[0] = static_cast<const uint8_t*>(plan); g.T[0] = static_cast<float*>(T); g.S[0] = S;
    g.m[0] = (int32_t)m; g.n[0] = (int32_t)n;
    e = lsp::launch_compress_planned(g, r, d, dtype, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? LSP_OK : lsp::note_hip_error(e);
}

}  // extern "C"
