// Device-side maintenance of a projector plan.
//
// Values-only refresh: projector fitting (the minimisation in MaybeUpdate, Alg. 1 / Eq. 2) changes the stored
// values of P and Q in every iteration and leaves their positions alone.  The plan records, for every value it
// holds, the flat ELL position it came from, so new values are dropped in place by one small kernel; nothing
// is sorted again and the host is not involved.
#include <algorithm>

#include "lsp_internal.h"

namespace lsp {

__global__ __launch_bounds__(256) void k_plan_refresh(uint8_t* __restrict__ plan, const float* __restrict__ P_val,
                                                      const float* __restrict__ Q_val, int m, int n, int r, int d) {
    const PlanHeader* H = reinterpret_cast<const PlanHeader*>(plan);
    if (H->magic != kPlanMagic || H->m != m || H->n != n || H->r != r || H->d != d) return;   // not this problem's plan
    const int64_t nq = (int64_t)H->q_total_rows * kWave, np = (int64_t)m * d;
    uint2* rows = reinterpret_cast<uint2*>(plan + H->off_q_rows);
    const uint32_t* qsrc = reinterpret_cast<const uint32_t*>(plan + H->off_q_src);
    uint2* pent = reinterpret_cast<uint2*>(plan + H->off_p_ent);
    const uint32_t* psrc = reinterpret_cast<const uint32_t*>(plan + H->off_p_src);
    const int64_t stride = (int64_t)gridDim.x * 256;
    for (int64_t k = (int64_t)blockIdx.x * 256 + threadIdx.x; k < nq + np; k += stride) {
        if (k < nq) {
            const uint32_t s = qsrc[k];
            if (s != kNoSource) rows[k].y = __float_as_uint(Q_val[s]);
        } else {
            const int64_t e = k - nq;
            pent[e].y = __float_as_uint(P_val[psrc[e]]);
        }
    }
}

hipError_t launch_plan_refresh(uint8_t* plan, const float* P_val, const float* Q_val,
                               int64_t m, int64_t n, int32_t r, int32_t d, hipStream_t st) {
    const int64_t work = (int64_t)plan_max_rows(n, r, d) * kWave + m * d;
    const unsigned blocks = (unsigned)std::min<int64_t>((work + 255) / 256, 2048);
    hipLaunchKernelGGL(k_plan_refresh, dim3(blocks), dim3(256), 0, st, plan, P_val, Q_val, (int)m, (int)n, (int)r, (int)d);
    return hipGetLastError();
}

}  // namespace lsp
