// extern "C" entry points: argument checks, workspace carving, kernel launches.
#include <algorithm>
#include <cstring>
#include <vector>

#include "lsp_internal.h"

namespace {
thread_local int g_last_hip_error = 0;
}

namespace lsp {
// Remembers the raw HIP error for lsp_last_hip_error() and returns LSP_ERR_LAUNCH.
int note_hip_error(hipError_t e) {
    g_last_hip_error = (int)e;
    return LSP_ERR_LAUNCH;
}
}  // namespace lsp

namespace {

int fail_launch(hipError_t e) { return lsp::note_hip_error(e); }

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

int check_shape(int64_t m, int64_t n, int32_t r, int32_t d) {
    if (m <= 0 || n <= 0 || r <= 0 || d <= 0) return LSP_ERR_SHAPE;
    if (d > r || r > LSP_MAX_R || d > LSP_MAX_D) return LSP_ERR_SHAPE;
    if (m > INT32_MAX || n > INT32_MAX) return LSP_ERR_SHAPE;
    if (m > ((int64_t)1 << 40) / n) return LSP_ERR_SHAPE;
    if (m * d > INT32_MAX || n * d > INT32_MAX) return LSP_ERR_SHAPE;   // plan offsets are 32-bit
    return LSP_OK;
}

int check_dtype(lsp_dtype t) { return (t == LSP_F32 || t == LSP_F16 || t == LSP_BF16) ? LSP_OK : LSP_ERR_DTYPE; }

size_t t_bytes(int64_t m, int32_t r) { return lsp::align_up((size_t)m * (size_t)r * sizeof(float), 256); }

}  // namespace

extern "C" {

size_t lsp_plan_build_workspace_bytes(int64_t m, int64_t n, int32_t r, int32_t d) {
    if (check_shape(m, n, r, d) != LSP_OK) return 0;
    return lsp::plan_build_workspace_bytes(m, n, r, d);
}

// raw entry: T | plan | scratch of the plan build | status word
size_t lsp_compress_workspace_bytes(int64_t m, int64_t n, int32_t r, int32_t d) {
    if (check_shape(m, n, r, d) != LSP_OK) return 0;
    return t_bytes(m, r) + lsp::align_up(lsp::plan_bytes(m, n, r, d), 256) + lsp::plan_build_workspace_bytes(m, n, r, d) + 256;
}

size_t lsp_compress_planned_workspace_bytes(int64_t m, int64_t n, int32_t r, int32_t d) {
    if (check_shape(m, n, r, d) != LSP_OK) return 0;
    return t_bytes(m, r);
}

size_t lsp_workspace_bytes(int64_t m, int64_t n, int32_t r, int32_t d, lsp_dtype dtype) {
    if (check_shape(m, n, r, d) != LSP_OK || check_dtype(dtype) != LSP_OK) return 0;
    size_t need = t_bytes(m, r);                                                    // both compress entries
    need = std::max(need, lsp_estimation_bias_workspace_bytes(m, n, r, d));
    need = std::max(need, lsp_reproject_state_workspace_bytes(r));
    need = std::max(need, lsp_bias_gradient_workspace_bytes(m, n, r, d));
    return need;
}

size_t lsp_plan_bytes(int64_t m, int64_t n, int32_t r, int32_t d) {
    if (check_shape(m, n, r, d) != LSP_OK) return 0;
    return lsp::plan_bytes(m, n, r, d);
}

int lsp_compress(const void* G, const int32_t* P_idx, const float* P_val, const int32_t* Q_idx, const float* Q_val,
                 int64_t m, int64_t n, int32_t r, int32_t d, float* S, lsp_dtype dtype,
                 void* workspace, size_t workspace_bytes, void* stream) {
    if (!G || !P_idx || !P_val || !Q_idx || !Q_val || !S) return LSP_ERR_NULL;
    int rc = check_shape(m, n, r, d);
    if (rc != LSP_OK) return rc;
    rc = check_dtype(dtype);
    if (rc != LSP_OK) return rc;
    if (!workspace || workspace_bytes < lsp_compress_workspace_bytes(m, n, r, d)) return LSP_ERR_WORKSPACE;
    if (!aligned16(workspace)) return LSP_ERR_WORKSPACE;
    if (!aligned16(G) || !aligned16(S) || !aligned16(P_idx) || !aligned16(P_val) || !aligned16(Q_idx) || !aligned16(Q_val))
        return LSP_ERR_ALIGN;
    // A plan is built on the device into the workspace, the planned kernels run on it, and the scatter-form
    // kernels follow, which do their work only if the build found the columns too skewed for a plan.
    uint8_t* ws = static_cast<uint8_t*>(workspace);
    float* T = reinterpret_cast<float*>(ws);
    uint8_t* plan = ws + t_bytes(m, r);
    uint8_t* scratch = plan + lsp::align_up(lsp::plan_bytes(m, n, r, d), 256);
    int32_t* status = reinterpret_cast<int32_t*>(scratch + lsp::plan_build_workspace_bytes(m, n, r, d));
    hipStream_t st = static_cast<hipStream_t>(stream);
    hipError_t e = lsp::launch_plan_build(P_idx, P_val, Q_idx, Q_val, m, n, r, d, plan, scratch, status, st);
    if (e != hipSuccess) return fail_launch(e);
    lsp::CompressGroup g;
    std::memset(&g, 0, sizeof(g));
    g.count = 1; g.G[0] = G; g.plan[0] = plan; g.T[0] = T; g.S[0] = S; g.m[0] = (int32_t)m; g.n[0] = (int32_t)n;
    if ((e = lsp::launch_compress_planned(g, r, d, dtype, st)) != hipSuccess) return fail_launch(e);
    e = lsp::launch_compress_raw(G, P_idx, P_val, Q_idx, Q_val, m, n, r, d, S, dtype, T, status, st);
    return e == hipSuccess ? LSP_OK : fail_launch(e);
}

int lsp_plan_build_async(const int32_t* P_idx, const float* P_val, const int32_t* Q_idx, const float* Q_val,
                         int64_t m, int64_t n, int32_t r, int32_t d, void* plan, size_t plan_bytes,
                         void* workspace, size_t workspace_bytes, int32_t* status, void* stream) {
    if (!P_idx || !P_val || !Q_idx || !Q_val) return LSP_ERR_NULL;
    int rc = check_shape(m, n, r, d);
    if (rc != LSP_OK) return rc;
    if (!plan || plan_bytes < lsp::plan_bytes(m, n, r, d) || !aligned16(plan)) return LSP_ERR_WORKSPACE;
    if (!workspace || workspace_bytes < lsp::plan_build_workspace_bytes(m, n, r, d) || !aligned16(workspace)) return LSP_ERR_WORKSPACE;
    if (!aligned16(P_idx) || !aligned16(P_val) || !aligned16(Q_idx) || !aligned16(Q_val)) return LSP_ERR_ALIGN;
    hipError_t e = lsp::launch_plan_build(P_idx, P_val, Q_idx, Q_val, m, n, r, d, static_cast<uint8_t*>(plan),
                                          static_cast<uint8_t*>(workspace), status, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? LSP_OK : fail_launch(e);
}

int lsp_plan_build(const int32_t* P_idx, const float* P_val, const int32_t* Q_idx, const float* Q_val,
                   int64_t m, int64_t n, int32_t r, int32_t d, void* plan, size_t plan_bytes, void* stream) {
    if (!P_idx || !P_val || !Q_idx || !Q_val) return LSP_ERR_NULL;
    int rc = check_shape(m, n, r, d);
    if (rc != LSP_OK) return rc;
    const size_t need = lsp::plan_bytes(m, n, r, d);
    if (!plan || plan_bytes < need || !aligned16(plan)) return LSP_ERR_WORKSPACE;
    if (!aligned16(P_idx) || !aligned16(P_val) || !aligned16(Q_idx) || !aligned16(Q_val)) return LSP_ERR_ALIGN;
    hipStream_t st = static_cast<hipStream_t>(stream);
    // a set-up call: scratch for the device-side build is allocated here and released before returning
    const size_t ws_bytes = lsp::plan_build_workspace_bytes(m, n, r, d) + 256;
    uint8_t* ws = nullptr;
    hipError_t e = hipMalloc(reinterpret_cast<void**>(&ws), ws_bytes);
    if (e != hipSuccess) return fail_launch(e);
    int32_t* status = reinterpret_cast<int32_t*>(ws + ws_bytes - 256);
    int32_t host_status = LSP_ERR_LAUNCH;
    e = lsp::launch_plan_build(P_idx, P_val, Q_idx, Q_val, m, n, r, d, static_cast<uint8_t*>(plan), ws, status, st);
    if (e == hipSuccess) e = hipMemcpyAsync(&host_status, status, sizeof(int32_t), hipMemcpyDeviceToHost, st);
    const hipError_t e2 = hipStreamSynchronize(st);                 // also before the scratch is released
    (void)hipFree(ws);
    if (e != hipSuccess) return fail_launch(e);
    if (e2 != hipSuccess) return fail_launch(e2);
    return host_status;
}

int lsp_plan_build_host(const int32_t* P_idx, const float* P_val, const int32_t* Q_idx, const float* Q_val,
                        int64_t m, int64_t n, int32_t r, int32_t d, void* plan_host, size_t plan_bytes) {
    if (!P_idx || !P_val || !Q_idx || !Q_val) return LSP_ERR_NULL;
    int rc = check_shape(m, n, r, d);
    if (rc != LSP_OK) return rc;
    if (!plan_host || plan_bytes < lsp::plan_bytes(m, n, r, d)) return LSP_ERR_WORKSPACE;
    for (int64_t k = 0; k < m * d; ++k) if (P_idx[k] < 0 || P_idx[k] >= r) return LSP_ERR_INDEX;
    for (int64_t k = 0; k < n * d; ++k) if (Q_idx[k] < 0 || Q_idx[k] >= r) return LSP_ERR_INDEX;
    return lsp::build_plan_host(P_idx, P_val, Q_idx, Q_val, m, n, r, d, static_cast<uint8_t*>(plan_host));
}

size_t lsp_compress_dense_workspace_bytes(int64_t m, int64_t n, int32_t r) {
    if (check_shape(m, n, r, 1) != LSP_OK || !lsp::dense_shape_ok(m, n, r)) return 0;
    return lsp::dense_workspace_bytes(m, r);
}

int lsp_compress_dense(const void* G, const void* Pt, const void* Qt, int64_t m, int64_t n, int32_t r, float* S,
                       lsp_dtype dtype, void* workspace, size_t workspace_bytes, void* stream) {
    if (!G || !Pt || !Qt || !S) return LSP_ERR_NULL;
    int rc = check_shape(m, n, r, 1);
    if (rc != LSP_OK) return rc;
    if (!lsp::dense_shape_ok(m, n, r)) return LSP_ERR_SHAPE;
    if (dtype != LSP_F16 && dtype != LSP_BF16) return LSP_ERR_DTYPE;
    if (!workspace || workspace_bytes < lsp::dense_workspace_bytes(m, r) || !aligned16(workspace)) return LSP_ERR_WORKSPACE;
    if (!aligned16(G) || !aligned16(Pt) || !aligned16(Qt) || !aligned16(S)) return LSP_ERR_ALIGN;
    hipError_t e = lsp::launch_compress_dense(G, Pt, Qt, m, n, r, S, static_cast<uint8_t*>(workspace), dtype, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? LSP_OK : fail_launch(e);
}

int lsp_compress_planned_grouped(const lsp_compress_item* items, int32_t count, int32_t r, int32_t d,
                                 lsp_dtype dtype, void* stream) {
    if (!items) return LSP_ERR_NULL;
    if (count <= 0 || count > LSP_MAX_GROUP) return LSP_ERR_SHAPE;
    int rc = check_dtype(dtype);
    if (rc != LSP_OK) return rc;
    lsp::CompressGroup g;
    std::memset(&g, 0, sizeof(g));
    g.count = count;
    for (int p = 0; p < count; ++p) {
        const lsp_compress_item& it = items[p];
        if (!it.G || !it.plan || !it.S) return LSP_ERR_NULL;
        rc = check_shape(it.m, it.n, r, d);
        if (rc != LSP_OK) return rc;
        if (!it.workspace || it.workspace_bytes < lsp_compress_planned_workspace_bytes(it.m, it.n, r, d)) return LSP_ERR_WORKSPACE;
        if (!aligned16(it.workspace) || !aligned16(it.plan)) return LSP_ERR_WORKSPACE;
        if (!aligned16(it.G) || !aligned16(it.S)) return LSP_ERR_ALIGN;
        for (int q = 0; q < p; ++q)                            // problems of a group run concurrently
            if (items[q].workspace == it.workspace || items[q].S == it.S) return LSP_ERR_WORKSPACE;
        g.G[p] = it.G; g.plan[p] = static_cast<const uint8_t*>(it.plan);
        g.T[p] = static_cast<float*>(it.workspace); g.S[p] = it.S;
        g.m[p] = (int32_t)it.m; g.n[p] = (int32_t)it.n;
    }
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (lsp::compress_group_uniform(g)) {
        hipError_t e = lsp::launch_compress_planned(g, r, d, dtype, st);
        return e == hipSuccess ? LSP_OK : fail_launch(e);
    }
    for (int p = 0; p < count; ++p) {                          // mixed kernel variants: one launch per problem
        lsp::CompressGroup one;
        std::memset(&one, 0, sizeof(one));
        one.count = 1;
        one.G[0] = g.G[p]; one.plan[0] = g.plan[p]; one.T[0] = g.T[p]; one.S[0] = g.S[p]; one.m[0] = g.m[p]; one.n[0] = g.n[p];
        hipError_t e = lsp::launch_compress_planned(one, r, d, dtype, st);
        if (e != hipSuccess) return fail_launch(e);
    }
    return LSP_OK;
}

int lsp_compress_planned(const void* G, const void* plan, int64_t m, int64_t n, int32_t r, int32_t d,
                         float* S, lsp_dtype dtype, void* workspace, size_t workspace_bytes, void* stream) {
    if (!G || !plan || !S) return LSP_ERR_NULL;
    lsp_compress_item it;
    it.G = G; it.plan = plan; it.S = S; it.workspace = workspace; it.workspace_bytes = workspace_bytes; it.m = m; it.n = n;
    return lsp_compress_planned_grouped(&it, 1, r, d, dtype, stream);
}

int lsp_decompress_apply_grouped(const lsp_apply_item* items, int32_t count, int32_t r, int32_t d,
                                 lsp_dtype dtype, void* stream) {
    if (!items) return LSP_ERR_NULL;
    if (count <= 0 || count > LSP_MAX_GROUP) return LSP_ERR_SHAPE;
    int rc = check_dtype(dtype);
    if (rc != LSP_OK) return rc;
    lsp::ApplyGroup g;
    std::memset(&g, 0, sizeof(g));
    g.count = count;
    for (int p = 0; p < count; ++p) {
        const lsp_apply_item& it = items[p];
        if (!it.W || !it.S || !it.P_idx || !it.P_val || !it.Q_idx || !it.Q_val) return LSP_ERR_NULL;
        rc = check_shape(it.m, it.n, r, d);
        if (rc != LSP_OK) return rc;
        if (!aligned16(it.W) || !aligned16(it.S) || !aligned16(it.P_idx) || !aligned16(it.P_val) || !aligned16(it.Q_idx) ||
            !aligned16(it.Q_val))
            return LSP_ERR_ALIGN;
        for (int q = 0; q < p; ++q)
            if (items[q].W == it.W) return LSP_ERR_SHAPE;      // one matrix twice in a group would race
        g.W[p] = it.W; g.S[p] = it.S; g.P_idx[p] = it.P_idx; g.P_val[p] = it.P_val; g.Q_idx[p] = it.Q_idx; g.Q_val[p] = it.Q_val;
        g.m[p] = (int32_t)it.m; g.n[p] = (int32_t)it.n;
    }
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (lsp::apply_group_uniform(g, r, d)) {
        hipError_t e = lsp::launch_decompress(g, r, d, dtype, st);
        return e == hipSuccess ? LSP_OK : fail_launch(e);
    }
    for (int p = 0; p < count; ++p) {
        lsp::ApplyGroup one;
        std::memset(&one, 0, sizeof(one));
        one.count = 1;
        one.W[0] = g.W[p]; one.S[0] = g.S[p]; one.P_idx[0] = g.P_idx[p]; one.P_val[0] = g.P_val[p];
        one.Q_idx[0] = g.Q_idx[p]; one.Q_val[0] = g.Q_val[p]; one.m[0] = g.m[p]; one.n[0] = g.n[p];
        hipError_t e = lsp::launch_decompress(one, r, d, dtype, st);
        if (e != hipSuccess) return fail_launch(e);
    }
    return LSP_OK;
}

int lsp_decompress_apply(void* W, const float* S, const int32_t* P_idx, const float* P_val,
                         const int32_t* Q_idx, const float* Q_val,
                         int64_t m, int64_t n, int32_t r, int32_t d, lsp_dtype dtype, void* stream) {
    if (!W || !S || !P_idx || !P_val || !Q_idx || !Q_val) return LSP_ERR_NULL;
    lsp_apply_item it;
    it.W = W; it.S = S; it.P_idx = P_idx; it.P_val = P_val; it.Q_idx = Q_idx; it.Q_val = Q_val; it.m = m; it.n = n;
    return lsp_decompress_apply_grouped(&it, 1, r, d, dtype, stream);
}

size_t lsp_estimation_bias_workspace_bytes(int64_t m, int64_t n, int32_t r, int32_t d) {
    if (check_shape(m, n, r, d) != LSP_OK) return 0;
    return lsp::align_up((size_t)lsp::bias_blocks(m, r) * 2 * sizeof(float), 256);
}

int lsp_estimation_bias(const void* G, const float* S, const int32_t* P_idx, const float* P_val,
                        const int32_t* Q_idx, const float* Q_val,
                        int64_t m, int64_t n, int32_t r, int32_t d, float* out,
                        void* workspace, size_t workspace_bytes, lsp_dtype dtype, void* stream) {
    if (!G || !S || !P_idx || !P_val || !Q_idx || !Q_val || !out) return LSP_ERR_NULL;
    int rc = check_shape(m, n, r, d);
    if (rc != LSP_OK) return rc;
    rc = check_dtype(dtype);
    if (rc != LSP_OK) return rc;
    if (!workspace || workspace_bytes < lsp_estimation_bias_workspace_bytes(m, n, r, d) || !aligned16(workspace))
        return LSP_ERR_WORKSPACE;
    if (!aligned16(G) || !aligned16(S) || !aligned16(P_idx) || !aligned16(P_val) || !aligned16(Q_idx) || !aligned16(Q_val))
        return LSP_ERR_ALIGN;
    lsp::ApplyGroup g;
    std::memset(&g, 0, sizeof(g));
    g.count = 1;
    g.W[0] = const_cast<void*>(G);                 // read only: the kernels built for the norms store nothing
    g.S[0] = S; g.P_idx[0] = P_idx; g.P_val[0] = P_val; g.Q_idx[0] = Q_idx; g.Q_val[0] = Q_val;
    g.m[0] = (int32_t)m; g.n[0] = (int32_t)n;
    hipError_t e = lsp::launch_bias(g, r, d, dtype, static_cast<float*>(workspace), out, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? LSP_OK : fail_launch(e);
}

int lsp_projector_reorder_host(const int32_t* idx, const float* val, int64_t rows, int32_t d, int32_t r,
                               int32_t* idx_out, float* val_out) {
    if (!idx || !val || !idx_out || !val_out) return LSP_ERR_NULL;
    if (rows <= 0 || d <= 0 || r <= 0 || d > r || r > LSP_MAX_R || d > LSP_MAX_D || rows * d > INT32_MAX) return LSP_ERR_SHAPE;
    if (idx == idx_out || val == val_out) return LSP_ERR_SHAPE;
    return lsp::reorder_rows_host(idx, val, rows, d, r, idx_out, val_out);
}

int lsp_projector_reorder(const int32_t* idx, const float* val, int64_t rows, int32_t d, int32_t r,
                          int32_t* idx_out, float* val_out, void* stream) {
    if (!idx || !val || !idx_out || !val_out) return LSP_ERR_NULL;
    if (rows <= 0 || d <= 0 || r <= 0 || d > r || r > LSP_MAX_R || d > LSP_MAX_D || rows * d > INT32_MAX) return LSP_ERR_SHAPE;
    if (idx == idx_out || val == val_out) return LSP_ERR_SHAPE;
    hipStream_t st = static_cast<hipStream_t>(stream);
    // Order after whatever produced the arrays on this stream, bring them to the host, reorder, send back.
    hipError_t e = hipStreamSynchronize(st);
    if (e != hipSuccess) return fail_launch(e);
    const size_t count = (size_t)rows * (size_t)d;
    std::vector<int32_t> hi(count), ho(count);
    std::vector<float> hv(count), hw(count);
    if ((e = hipMemcpy(hi.data(), idx, count * 4, hipMemcpyDeviceToHost)) != hipSuccess) return fail_launch(e);
    if ((e = hipMemcpy(hv.data(), val, count * 4, hipMemcpyDeviceToHost)) != hipSuccess) return fail_launch(e);
    const int rc = lsp::reorder_rows_host(hi.data(), hv.data(), rows, d, r, ho.data(), hw.data());
    if (rc != LSP_OK) return rc;
    if ((e = hipMemcpy(idx_out, ho.data(), count * 4, hipMemcpyHostToDevice)) != hipSuccess) return fail_launch(e);
    if ((e = hipMemcpy(val_out, hw.data(), count * 4, hipMemcpyHostToDevice)) != hipSuccess) return fail_launch(e);
    return LSP_OK;
}

size_t lsp_reproject_state_workspace_bytes(int32_t r) {
    if (r <= 0 || r > LSP_MAX_R) return 0;
    return lsp::align_up((size_t)4 * (size_t)r * (size_t)r * sizeof(float), 256);   // A, B and two products in flight
}

int lsp_reproject_state(const int32_t* P_idx, const float* P_val, const int32_t* Pprev_idx, const float* Pprev_val,
                        const int32_t* Q_idx, const float* Q_val, const int32_t* Qprev_idx, const float* Qprev_val,
                        int64_t m, int64_t n, int32_t r, int32_t d, float* M, float* V,
                        void* workspace, size_t workspace_bytes, void* stream) {
    if (!P_idx || !P_val || !Pprev_idx || !Pprev_val || !Q_idx || !Q_val || !Qprev_idx || !Qprev_val || !M) return LSP_ERR_NULL;
    int rc = check_shape(m, n, r, d);
    if (rc != LSP_OK) return rc;
    if (!workspace || workspace_bytes < lsp_reproject_state_workspace_bytes(r) || !aligned16(workspace)) return LSP_ERR_WORKSPACE;
    if (!aligned16(M) || (V && !aligned16(V))) return LSP_ERR_ALIGN;
    if (M == V) return LSP_ERR_SHAPE;
    hipError_t e = lsp::launch_reproject(P_idx, P_val, Pprev_idx, Pprev_val, Q_idx, Q_val, Qprev_idx, Qprev_val,
                                         m, n, r, d, M, V, static_cast<float*>(workspace), static_cast<hipStream_t>(stream));
    return e == hipSuccess ? LSP_OK : fail_launch(e);
}

int lsp_plan_refresh_values(void* plan, const float* P_val, const float* Q_val,
                            int64_t m, int64_t n, int32_t r, int32_t d, void* stream) {
    if (!plan || !P_val || !Q_val) return LSP_ERR_NULL;
    int rc = check_shape(m, n, r, d);
    if (rc != LSP_OK) return rc;
    if (!aligned16(plan)) return LSP_ERR_WORKSPACE;
    if (!aligned16(P_val) || !aligned16(Q_val)) return LSP_ERR_ALIGN;
    hipError_t e = lsp::launch_plan_refresh(static_cast<uint8_t*>(plan), P_val, Q_val, m, n, r, d, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? LSP_OK : fail_launch(e);
}

size_t lsp_bias_gradient_workspace_bytes(int64_t m, int64_t n, int32_t r, int32_t d) {
    if (check_shape(m, n, r, d) != LSP_OK) return 0;
    return lsp::align_up(lsp::fitgrad_workspace_floats(m, n, r, d) * sizeof(float), 256);
}

int lsp_bias_gradient(const void* G, const void* plan,
                      const int32_t* P_idx, const float* P_val, const int32_t* Q_idx, const float* Q_val,
                      int64_t m, int64_t n, int32_t r, int32_t d, float* gP, float* gQ,
                      void* workspace, size_t workspace_bytes, lsp_dtype dtype, void* stream) {
    if (!G || !plan || !P_idx || !P_val || !Q_idx || !Q_val || !gP || !gQ) return LSP_ERR_NULL;
    int rc = check_shape(m, n, r, d);
    if (rc != LSP_OK) return rc;
    rc = check_dtype(dtype);
    if (rc != LSP_OK) return rc;
    if (!workspace || workspace_bytes < lsp_bias_gradient_workspace_bytes(m, n, r, d) || !aligned16(workspace) || !aligned16(plan))
        return LSP_ERR_WORKSPACE;
    if (!aligned16(G) || !aligned16(P_idx) || !aligned16(P_val) || !aligned16(Q_idx) || !aligned16(Q_val) || !aligned16(gP) || !aligned16(gQ))
        return LSP_ERR_ALIGN;
    hipError_t e = lsp::launch_fitgrad(G, static_cast<const uint8_t*>(plan), P_idx, P_val, Q_idx, Q_val, m, n, r, d, gP, gQ,
                                       static_cast<float*>(workspace), dtype, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? LSP_OK : fail_launch(e);
}

int lsp_validate_projector(const int32_t* idx, int64_t rows, int32_t d, int32_t r, int32_t* flag, void* stream) {
    if (!idx || !flag) return LSP_ERR_NULL;
    if (rows <= 0 || d <= 0 || r <= 0) return LSP_ERR_SHAPE;
    hipStream_t st = static_cast<hipStream_t>(stream);
    hipError_t e = lsp::launch_validate(idx, rows * d, r, flag, st);
    if (e != hipSuccess) return fail_launch(e);
    int32_t host_flag = 0;
    if ((e = hipMemcpyAsync(&host_flag, flag, sizeof(int32_t), hipMemcpyDeviceToHost, st)) != hipSuccess) return fail_launch(e);
    if ((e = hipStreamSynchronize(st)) != hipSuccess) return fail_launch(e);
    return host_flag ? LSP_ERR_INDEX : LSP_OK;
}

const char* lsp_strerror(int code) {
    switch (code) {
        case LSP_OK:            return "ok";
        case LSP_ERR_NULL:      return "a required pointer is NULL";
        case LSP_ERR_SHAPE:     return "invalid shape (m, n, r, d must be positive, d <= r, within supported maxima)";
        case LSP_ERR_DTYPE:     return "unknown dtype";
        case LSP_ERR_WORKSPACE: return "workspace or plan buffer missing, misaligned or too small";
        case LSP_ERR_LAUNCH:    return "HIP runtime error (see lsp_last_hip_error)";
        case LSP_ERR_INDEX:     return "projector index outside [0, r)";
        case LSP_ERR_ALIGN:     return "a base pointer is not 16-byte aligned";
        case LSP_ERR_SKEW:      return "projector columns used too unevenly for a plan (use lsp_compress)";
        case LSP_ERR_TOO_LARGE: return "problem needs more scratch than the library's static array holds (lsp_static_scratch_bytes); "
                                       "use the entry that takes a workspace";
        default:                return "unknown lsp_status";
    }
}

int lsp_last_hip_error(void) { return g_last_hip_error; }
int lsp_version(void) { return 100; }

}  // extern "C"
