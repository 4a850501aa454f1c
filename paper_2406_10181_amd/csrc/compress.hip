// Compress: S = P^T G Q  (Alg. 1, compress step; Alg. 3, projected gradient of a layer).
//
// Two kernels per call, both gather-form and free of global atomics in the common case:
//   A  T = G Q     one workgroup per block of 16 rows of G; G is streamed once from HBM in
//                  chunks of kChunk columns and staged in LDS transposed, one 16-byte unit per
//                  column and group of rows (8 rows in storage precision for fp16 / bf16, 4 rows
//                  widened to fp32 otherwise), so one 128-bit LDS read serves 8 (4) rows; each
//                  lane owns one column b of T and walks the plan's list of (column of G, value)
//                  pairs of b, accumulating in registers.  With one column per lane the plan deals
//                  the lists of every chunk to the waves by length, and the partial sums change
//                  lanes between chunks (swap_owner).
//   B  S = P^T T   one wave per piece of a row of P^T and 1/8 of the columns; reads rows of T.
// The path streams G once; its main loop is bound by vector-ALU issue (16 widenings and 16 FMAs
// per pair and 16 rows for bf16), not by HBM.  No matrix cores are involved because the
// projectors are sparse (d entries per row, Def. 1) and the work is gather + fp32 FMA.

#include "compress_common.h"

namespace lsp {

// ----------------------------------------------------------------------------------------------
// Kernel B, general variant (any r): S[a][stripe] (+)= sum_e v_e T[i_e][stripe] for one piece of a
// row of P^T and one stripe of 256 columns, one column per thread.
constexpr int kThreadsB = 256;
constexpr int kStripeQuads = 64;                              // column quads (float4) per stripe
__global__ __launch_bounds__(kThreadsB) void k_compress_pt(const CompressGroup grp, int r, int d, int nstripes) {
    const CompressProblem pr = group_pick(grp, (int)blockIdx.x, true);
    const uint8_t* __restrict__ plan = pr.plan;
    const float* __restrict__ T = pr.T;
    float* __restrict__ S = pr.S;
    const int block = pr.block_pt;
    PlanHeaderPtr H = as_const<PlanHeader>(plan);
    if (!plan_matches(H, pr.m, pr.n, r, d)) return;                   // kernel A has filled S with NaN
    const int stripe = block % nstripes, item = block / nstripes;
    if (item >= H->p_nitems) return;
    const auto* itp = as_const<int32_t>(plan + H->off_p_item) + 4 * item;    // RowItem, field by field
    const RowItem it{itp[0], itp[1], itp[2], itp[3]};
    const uint2* ent = reinterpret_cast<const uint2*>(plan + H->off_p_ent) + it.start;
    for (int b = stripe * kStripeQuads * 4 + threadIdx.x; b < min(r, (stripe + 1) * kStripeQuads * 4); b += kThreadsB) {
        float acc = 0.0f;
        for (int e = 0; e < it.len; ++e) {
            const uint2 en = ent[e];
            acc = fmaf(__uint_as_float(en.y), T[(int64_t)en.x * r + b], acc);
        }
        float* dst = S + (int64_t)it.a * r + b;
        if (it.atomic) atomicAdd(dst, acc); else *dst = acc;
    }
}

// Kernel B, the usual variant (r % 4 == 0), XCD-aware.  The columns of T are cut into 8 stripes, one per XCD:
// workgroups are dealt to the 8 XCDs round-robin, so with stripe = blockIdx % 8 an XCD only ever
// touches its own m x r/8 slice of T, which fits its 4 MB L2 -- T comes from HBM once instead of
// once per use (each row of T is used by d rows of S).  Each of the 4 waves of a workgroup takes
// one piece of a row of P^T; its 64 lanes form 64/LG groups of LG lanes (LG = 16, 32 or 64 >= quads
// per stripe), group g takes entries g, g + groups, ...; the groups' sums meet through lane
// exchanges in a fixed order.
template <int LG>
__global__ __launch_bounds__(kThreadsB) void k_compress_pt8(const CompressGroup grp, int r, int d, int sq) {
    constexpr int NG = kWave / LG;                            // entry groups per wave
    const CompressProblem pr = group_pick(grp, (int)blockIdx.x, true);
    const uint8_t* __restrict__ plan = pr.plan;
    const float* __restrict__ T = pr.T;
    float* __restrict__ S = pr.S;
    const int block = pr.block_pt;
    PlanHeaderPtr H = as_const<PlanHeader>(plan);
    if (!plan_matches(H, pr.m, pr.n, r, d)) return;                   // kernel A has filled S with NaN
    const int stripe = block & 7;
    const int item = (block >> 3) * (kThreadsB / kWave) + (int)(threadIdx.x >> 6);
    if (item >= H->p_nitems) return;
    const auto* itp = as_const<int32_t>(plan + H->off_p_item) + 4 * item;    // RowItem, field by field
    const RowItem it{itp[0], itp[1], itp[2], itp[3]};
    const uint2* ent = reinterpret_cast<const uint2*>(plan + H->off_p_ent) + it.start;
    const int lane = threadIdx.x & 63;
    const int grp_e = lane / LG, ql = lane % LG;
    const int b4 = stripe * sq + ql;
    const bool live = ql < sq && b4 < (r >> 2);
    const float* Tcol = T + (live ? b4 * 4 : 0);
    f32x4 acc = {0.0f, 0.0f, 0.0f, 0.0f};
    // The piece's entries are loaded once, 64 at a time (one per lane), and handed to the groups by
    // lane exchange, so that the loads of T do not each wait for a load of their entry and can
    // all be in flight together.
    for (int base = 0; base < it.len; base += kWave) {
        const int e_mine = base + lane;
        const uint2 mine = e_mine < it.len ? ent[e_mine] : make_uint2(0u, 0u);
        const int steps = (min(it.len - base, (int)kWave) + NG - 1) / NG;      // uniform over the wave
        constexpr int kBlock = 16;                                              // loads of T in flight per lane
        for (int k0 = 0; k0 < steps; k0 += kBlock) {
            f32x4 x[kBlock];
            float v[kBlock];
#pragma unroll
            for (int k = 0; k < kBlock; ++k) {
                const int src = min((k0 + k) * NG + grp_e, (int)kWave - 1);     // lane holding entry base + (k0+k)*NG + grp
                const uint32_t row = (uint32_t)__shfl((int)mine.x, src);
                v[k] = __uint_as_float((uint32_t)__shfl((int)mine.y, src));
                const bool on = k0 + k < steps && (k0 + k) * NG + grp_e < kWave;
                if (!on) v[k] = 0.0f;
                x[k] = *reinterpret_cast<const f32x4*>(Tcol + (int64_t)(on ? row : 0u) * r);
            }
#pragma unroll
            for (int k = 0; k < kBlock; ++k) {
                acc.x = fmaf(v[k], x[k].x, acc.x); acc.y = fmaf(v[k], x[k].y, acc.y);
                acc.z = fmaf(v[k], x[k].z, acc.z); acc.w = fmaf(v[k], x[k].w, acc.w);
            }
        }
    }
#pragma unroll
    for (int step = LG; step < kWave; step *= 2) {            // group g adds group g ^ (step / LG)
        acc.x += __shfl_xor(acc.x, step); acc.y += __shfl_xor(acc.y, step);
        acc.z += __shfl_xor(acc.z, step); acc.w += __shfl_xor(acc.w, step);
    }
    if (lane < LG && live) {
        float* dst = S + (int64_t)it.a * r + b4 * 4;
        if (it.atomic) {
            atomicAdd(dst + 0, acc.x); atomicAdd(dst + 1, acc.y); atomicAdd(dst + 2, acc.z); atomicAdd(dst + 3, acc.w);
        } else {
            *reinterpret_cast<f32x4*>(dst) = acc;
        }
    }
}

// ----------------------------------------------------------------------------------------------
// Plan-free variant used by the raw-ELL entry: same mathematics in scatter form.
//   T tile in LDS, every (row, column j, entry k) adds G[i][j] * Q_val[j][k] to T[i][Q_idx[j][k]];
//   then S[P_idx[i][k]][:] += P_val[i][k] * T[i][:] with global atomics (S zeroed first).
constexpr int kRawRows = 16;
template <typename D>
__global__ __launch_bounds__(256) void k_raw_gq(const typename D::elem* __restrict__ G,
                                               const int32_t* __restrict__ Q_idx, const float* __restrict__ Q_val,
                                               float* __restrict__ T, int m, int n, int r, int d, const int32_t* __restrict__ gate) {
    extern __shared__ __align__(16) uint8_t smem[];
    if (gate && *gate != LSP_ERR_SKEW) return;                        // the planned kernels have done the work
    float* Tl = reinterpret_cast<float*>(smem);
    const int64_t i0 = (int64_t)blockIdx.x * kRawRows;
    for (int k = threadIdx.x; k < kRawRows * r; k += 256) Tl[k] = 0.0f;
    __syncthreads();
    for (int64_t j = threadIdx.x; j < n; j += 256) {
        float g[kRawRows];
#pragma unroll
        for (int t = 0; t < kRawRows; ++t) g[t] = (i0 + t < m) ? widen<D>(G[(i0 + t) * (int64_t)n + j]) : 0.0f;
        for (int k = 0; k < d; ++k) {
            const int b = Q_idx[j * d + k];
            const float v = Q_val[j * d + k];
#pragma unroll
            for (int t = 0; t < kRawRows; ++t) atomicAdd(&Tl[t * r + b], g[t] * v);
        }
    }
    __syncthreads();
    for (int k = threadIdx.x; k < kRawRows * r; k += 256) {
        const int t = k / r;
        if (i0 + t < m) T[(i0 + t) * (int64_t)r + (k - t * r)] = Tl[k];
    }
}

__global__ __launch_bounds__(256) void k_fill_zero(float* __restrict__ p, int64_t count, const int32_t* __restrict__ gate) {
    if (gate && *gate != LSP_ERR_SKEW) return;
    for (int64_t k = (int64_t)blockIdx.x * 256 + threadIdx.x; k < count; k += (int64_t)gridDim.x * 256) p[k] = 0.0f;
}

__global__ __launch_bounds__(256) void k_raw_pt(const float* __restrict__ T, const int32_t* __restrict__ P_idx,
                                               const float* __restrict__ P_val, float* __restrict__ S, int r, int d,
                                               const int32_t* __restrict__ gate) {
    if (gate && *gate != LSP_ERR_SKEW) return;
    const int64_t i = blockIdx.x;
    for (int k = 0; k < d; ++k) {
        const int a = P_idx[i * d + k];
        const float v = P_val[i * d + k];
        for (int b = threadIdx.x; b < r; b += 256) atomicAdd(&S[(int64_t)a * r + b], v * T[i * r + b]);
    }
}

// ----------------------------------------------------------------------------------------------
bool compress_group_uniform(const CompressGroup& g) {
    for (int p = 1; p < g.count; ++p)
        if ((g.n[p] % 8 == 0) != (g.n[0] % 8 == 0)) return false;     // selects vector or element-wise loads
    return true;
}

// Row blocks per workgroup of kernel A: several on big grids (grouped calls) of the 16-bit kernel
static int gq_blocks_per_wg(const CompressGroup& g, lsp_dtype dtype) {
    if (dtype == LSP_F32 || g.n[0] % 8 != 0) return 1;
    int64_t rows = 0;
    for (int p = 0; p < g.count; ++p) rows += g.m[p];
    return rows >= 16384 ? 2 : 1;
}

// Rows of a row block of kernel A: the 16-bit kernel and the 32-bit-staged kernel differ
static int gq_block_rows(const CompressGroup& g, lsp_dtype dtype) {
    return (dtype != LSP_F32 && g.n[0] % 8 == 0) ? kRowsGQ16 : kRowsGQ;
}

static hipError_t launch_gq(const CompressGroup& g, int32_t r, int32_t d, int blocks_per_wg, lsp_dtype dtype, hipStream_t st) {
    if (dtype != LSP_F32 && g.n[0] % 8 == 0)
        return dtype == LSP_F16 ? launch_gq16_f16(g, r, d, blocks_per_wg, st) : launch_gq16_bf16(g, r, d, blocks_per_wg, st);
    return launch_gq_staged32(g, r, d, dtype, st);
}

// The hardware hands the workgroups of a launch to the CUs in index order as CUs fall free, so the
// order of the problems inside a group is the order of a greedy list schedule: the problems whose
// workgroups run longest (widest matrices: work per row block grows with n) go first, and the
// short ones fill in behind them.
static void longest_first(CompressGroup& g) {
    for (int a = 1; a < g.count; ++a)
        for (int b = a; b > 0 && g.n[b] > g.n[b - 1]; --b) {
            std::swap(g.G[b], g.G[b - 1]); std::swap(g.plan[b], g.plan[b - 1]); std::swap(g.T[b], g.T[b - 1]);
            std::swap(g.S[b], g.S[b - 1]); std::swap(g.m[b], g.m[b - 1]); std::swap(g.n[b], g.n[b - 1]);
        }
}

hipError_t launch_compress_planned(CompressGroup& g, int32_t r, int32_t d, lsp_dtype dtype, hipStream_t st) {
    const int nstripes = (r + kStripeQuads * 4 - 1) / (kStripeQuads * 4);
    const bool striped = (r % 4) == 0;
    longest_first(g);
    const int bpw = gq_blocks_per_wg(g, dtype), rows = gq_block_rows(g, dtype);
    g.first_gq[0] = g.first_pt[0] = 0;
    for (int p = 0; p < g.count; ++p) {
        g.first_gq[p + 1] = g.first_gq[p] + (int32_t)(((g.m[p] + rows - 1) / rows + bpw - 1) / bpw);
        const int32_t items = (int32_t)plan_max_items(g.m[p], r, d);
        g.first_pt[p + 1] = g.first_pt[p] + (striped ? ((items + 3) / 4) * 8 : items * nstripes);
    }
    hipError_t e = launch_gq(g, r, d, bpw, dtype, st);
    if (e != hipSuccess) return e;
    const unsigned blocks = (unsigned)g.first_pt[g.count];
    if (striped) {
        const int sq = ((r >> 2) + 7) / 8;
        if (sq <= 16)      hipLaunchKernelGGL(k_compress_pt8<16>, dim3(blocks), dim3(kThreadsB), 0, st, g, (int)r, (int)d, sq);
        else if (sq <= 32) hipLaunchKernelGGL(k_compress_pt8<32>, dim3(blocks), dim3(kThreadsB), 0, st, g, (int)r, (int)d, sq);
        else               hipLaunchKernelGGL(k_compress_pt8<64>, dim3(blocks), dim3(kThreadsB), 0, st, g, (int)r, (int)d, sq);
        return hipGetLastError();
    }
    hipLaunchKernelGGL(k_compress_pt, dim3(blocks), dim3(kThreadsB), 0, st, g, (int)r, (int)d, nstripes);
    return hipGetLastError();
}

template <typename D>
static hipError_t launch_raw_gq(const void* G, const int32_t* Q_idx, const float* Q_val, float* T,
                                int64_t m, int64_t n, int32_t r, int32_t d, const int32_t* gate, hipStream_t st) {
    const size_t lds = (size_t)kRawRows * r * sizeof(float);
    hipError_t e = allow_dynamic_lds<k_raw_gq<D>>((size_t)kRawRows * LSP_MAX_R * sizeof(float));
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(k_raw_gq<D>, dim3((unsigned)((m + kRawRows - 1) / kRawRows)), dim3(256), lds, st,
                       reinterpret_cast<const typename D::elem*>(G), Q_idx, Q_val, T, (int)m, (int)n, (int)r, (int)d, gate);
    return hipGetLastError();
}

hipError_t launch_compress_raw(const void* G, const int32_t* P_idx, const float* P_val,
                               const int32_t* Q_idx, const float* Q_val,
                               int64_t m, int64_t n, int32_t r, int32_t d,
                               float* S, lsp_dtype dtype, float* T, const int32_t* gate, hipStream_t st) {
    hipError_t e;
    switch (dtype) {
        case LSP_F32:  e = launch_raw_gq<F32>(G, Q_idx, Q_val, T, m, n, r, d, gate, st); break;
        case LSP_F16:  e = launch_raw_gq<F16>(G, Q_idx, Q_val, T, m, n, r, d, gate, st); break;
        default:       e = launch_raw_gq<BF16>(G, Q_idx, Q_val, T, m, n, r, d, gate, st); break;
    }
    if (e != hipSuccess) return e;
    const int64_t rr = (int64_t)r * r;
    hipLaunchKernelGGL(k_fill_zero, dim3((unsigned)((rr + 255) / 256 > 1024 ? 1024 : (rr + 255) / 256)), dim3(256), 0, st, S, rr, gate);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(k_raw_pt, dim3((unsigned)m), dim3(256), 0, st, T, P_idx, P_val, S, (int)r, (int)d, gate);
    return hipGetLastError();
}

}  // namespace lsp

