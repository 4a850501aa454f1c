// Decompress and apply:  W <- rn(W - P S Q^T)  (Alg. 1, apply step; Alg. 3, last step of the
// layer loop).  One kernel, one fused read-modify-write pass over W:
//   phase 1  U = P S for the workgroup's R rows of W (gathers d rows of S per row, S stays in
//            L2), stored in LDS as [4-row plane][column b][4 rows] fp32;
//   phase 2  every thread owns CPT consecutive columns j, keeps the d (column, value) pairs of
//            their rows of Q in registers, and for each 4-row plane gathers U with one 128-bit
//            LDS read per pair; W is read, updated in fp32 and rounded once.
// Bandwidth-bound (read + write of W); no matrix cores (sparse gather + fp32 FMA).
//
// The same kernels, built with NORMS, serve the estimation bias of Def. 2 (the test MaybeUpdate
// makes in Alg. 1): with S = P^T G Q they rebuild P S Q^T tile by tile in registers, read G where
// the apply step reads W, and instead of storing anything add up (P S Q^T - G)^2 and G^2; every
// workgroup leaves its two sums in a list that k_bias_finish adds in a fixed order.
#include <utility>

#include "lsp_internal.h"

namespace lsp {

constexpr int kThreadsD = 256;   // generic kernel
typedef float f32x4 __attribute__((ext_vector_type(4)));

template <typename D, int CPT> struct Vec;     // CPT consecutive elements of W
template <> struct Vec<F32, 4>  { f32x4 v; };
template <> struct Vec<F32, 2>  { float x, y; };
template <> struct Vec<F16, 4>  { uint32_t x, y; };
template <> struct Vec<BF16, 4> { uint32_t x, y; };
template <> struct Vec<F16, 2>  { uint32_t x; };
template <> struct Vec<BF16, 2> { uint32_t x; };

template <typename D> __device__ __forceinline__ void pair_widen(uint32_t p, float& lo, float& hi);
template <> __device__ __forceinline__ void pair_widen<F16>(uint32_t p, float& lo, float& hi) {
    lo = widen<F16>((uint16_t)(p & 0xFFFFu)); hi = widen<F16>((uint16_t)(p >> 16));
}
template <> __device__ __forceinline__ void pair_widen<BF16>(uint32_t p, float& lo, float& hi) {
    lo = __uint_as_float(p << 16); hi = __uint_as_float(p & 0xFFFF0000u);
}
template <typename D> __device__ __forceinline__ uint32_t pair_narrow(float lo, float hi) {
    return (uint32_t)narrow<D>(lo) | ((uint32_t)narrow<D>(hi) << 16);
}

template <typename D, int CPT> __device__ __forceinline__ void vec_widen(const Vec<D, CPT>& x, float* out) {
    if constexpr (D::size == 4) {
        if constexpr (CPT == 4) { out[0] = x.v.x; out[1] = x.v.y; out[2] = x.v.z; out[3] = x.v.w; }
        else { out[0] = x.x; out[1] = x.y; }
    } else {
        pair_widen<D>(x.x, out[0], out[1]);
        if constexpr (CPT == 4) pair_widen<D>(x.y, out[2], out[3]);
    }
}
template <typename D, int CPT> __device__ __forceinline__ Vec<D, CPT> vec_narrow(const float* in) {
    Vec<D, CPT> o;
    if constexpr (D::size == 4) {
        if constexpr (CPT == 4) { o.v.x = in[0]; o.v.y = in[1]; o.v.z = in[2]; o.v.w = in[3]; }
        else { o.x = in[0]; o.y = in[1]; }
    } else {
        o.x = pair_narrow<D>(in[0], in[1]);
        if constexpr (CPT == 4) o.y = pair_narrow<D>(in[2], in[3]);
    }
    return o;
}

// Sums x and y over the workgroup (NT threads) and lets thread 0 store them; `red` is LDS nobody
// else uses any more.  Fixed order: the result does not depend on timing.
template <int NT>
__device__ __forceinline__ void block_sum2(float x, float y, float2* red, float2* dst) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        x += __shfl_down(x, off);
        y += __shfl_down(y, off);
    }
    __syncthreads();
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = make_float2(x, y);
    __syncthreads();
    if (threadIdx.x == 0) {
        float2 t = red[0];
        for (int w = 1; w < NT / 64; ++w) { t.x += red[w].x; t.y += red[w].y; }
        *dst = t;
    }
}

// phase 1 (generic kernel):  Us[plane][b] (float4 = 4 rows) = sum_k P_val[i][k] S[P_idx[i][k]][b]
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

// phase 1 (fast kernel, r % 4 == 0): the R*DD (row of S, value) pairs of the tile go to LDS first,
// then every work item (row t of the tile, 4 consecutive columns b) issues its DD 128-bit loads of
// S back to back, so the whole gather costs two memory round trips.
template <int RG, int DD, int PS, int NT>
__device__ __forceinline__ void build_u_tile_fast(uint8_t* smem, int2* pent, const float* __restrict__ S,
                                                  const int32_t* __restrict__ P_idx, const float* __restrict__ P_val,
                                                  int64_t i0, int m, int r) {
    constexpr int R = 4 * RG;
    for (int q = threadIdx.x; q < R * DD; q += NT) {
        const int64_t i = i0 + q / DD;
        int2 e = make_int2(0, 0);                                   // rows past m: value 0, row 0 of S
        if (i < m) e = make_int2(P_idx[i * DD + q % DD], __float_as_int(P_val[i * DD + q % DD]));
        pent[q] = e;
    }
    __syncthreads();
    const int r4 = r >> 2;
    for (int q = threadIdx.x; q < r4 * R; q += NT) {
        const int row = q / r4, b4 = q - row * r4;                  // row of the tile, column quad
        f32x4 x[DD];
#pragma unroll
        for (int k = 0; k < DD; ++k)
            x[k] = *reinterpret_cast<const f32x4*>(S + (int64_t)pent[row * DD + k].x * r + b4 * 4);
        f32x4 u = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
        for (int k = 0; k < DD; ++k) {
            const float v = __int_as_float(pent[row * DD + k].y);
            u.x = fmaf(v, x[k].x, u.x); u.y = fmaf(v, x[k].y, u.y);
            u.z = fmaf(v, x[k].z, u.z); u.w = fmaf(v, x[k].w, u.w);
        }
        // Us[plane][b] is a float4 over the plane's 4 rows: element (b, t) lives at float index 4 b + t
        float* dst = reinterpret_cast<float*>(smem + (row >> 2) * PS) + (b4 * 4) * 4 + (row & 3);
        dst[0] = u.x; dst[4] = u.y; dst[8] = u.z; dst[12] = u.w;
    }
}

// Fast kernel: DD = compile-time d, CPT columns per thread, n % CPT == 0, r % 4 == 0.  PS = bytes
// between the 4-row planes of U in LDS, a compile-time constant >= 16 r so that the plane offset
// folds into the immediate offset of the LDS read and a gather costs no address arithmetic.
// All loads of a pass (the thread's rows of Q and its R x CPT patch of W) are issued before the
// gathers start, so one pass costs one HBM round trip; many waves per CU overlap the passes.
template <typename D, int RG, int DD, int PS, int NT, int CPT, int kDepth, bool NORMS>
__global__ __launch_bounds__(NT) void k_decompress(const ApplyGroup grp, int r, float2* __restrict__ partial, int split_from) {
    extern __shared__ __align__(16) uint8_t smem[];
    constexpr int R = 4 * RG;
    constexpr int NE = CPT * DD;                                    // entries owned by a thread in one pass
    static_assert(NE % 4 == 0, "entries are loaded 4 at a time");
    // Row blocks from split_from on are shared by two workgroups, each with half of the passes (both build
    // the tile of U): the last workgroups of a launch are then half as long, and the CUs finish closer together.
    int bx = (int)blockIdx.x, half = 0, halves = 1;
    if (bx >= split_from) {
        const int t = bx - split_from;
        bx = split_from + (t >> 1); half = t & 1; halves = 2;
    }
    const int prob = group_find(grp.first, grp.count, bx);
    typename D::elem* __restrict__ W = static_cast<typename D::elem*>(grp.W[prob]);
    const float* __restrict__ S = grp.S[prob];
    const int32_t* __restrict__ P_idx = grp.P_idx[prob];
    const float* __restrict__ P_val = grp.P_val[prob];
    const int32_t* __restrict__ Q_idx = grp.Q_idx[prob];
    const float* __restrict__ Q_val = grp.Q_val[prob];
    const int m = grp.m[prob], n = grp.n[prob];
    const int block = bx - grp.first[prob];
    const int64_t i0 = (int64_t)block * R;
    int2* pent = reinterpret_cast<int2*>(smem + RG * PS);
    const f32x4* Us4 = reinterpret_cast<const f32x4*>(smem);

    // one pass = this thread's CPT columns: their rows of Q (NE pairs, flat index c * DD + k) and
    // the R x CPT patch of W
    struct Pass { int4 qi[NE / 4]; f32x4 qv[NE / 4]; Vec<D, CPT> wv[R]; };
    auto load_pass = [&](int64_t j0, Pass& p) {
        const int4* qip = reinterpret_cast<const int4*>(Q_idx + j0 * DD);
        const f32x4* qvp = reinterpret_cast<const f32x4*>(Q_val + j0 * DD);
#pragma unroll
        for (int k = 0; k < NE / 4; ++k) {
            if constexpr (kNoApplyQ) {
                p.qi[k] = make_int4((int)(threadIdx.x + k) & 255, (int)(threadIdx.x * 3 + k) & 255, (int)(threadIdx.x * 5 + k) & 255, (int)(threadIdx.x * 7 + k) & 255);
                p.qv[k] = f32x4{0.1f, 0.2f, 0.3f, 0.4f};
            } else {
                p.qi[k] = qip[k];
                p.qv[k] = qvp[k];
            }
        }
#pragma unroll
        for (int t = 0; t < R; ++t) {
            const int64_t i = i0 + t < m ? i0 + t : m - 1;         // rows past m: any valid row, never stored
            p.wv[t] = stream_load(reinterpret_cast<const Vec<D, CPT>*>(W + i * (int64_t)n + j0));
        }
    };
    auto idx_of = [](const Pass& p, int e) -> uint32_t {
        const int4 q = p.qi[e >> 2];
        return (uint32_t)((e & 3) == 0 ? q.x : (e & 3) == 1 ? q.y : (e & 3) == 2 ? q.z : q.w);
    };
    auto val_of = [](const Pass& p, int e) -> float {
        const f32x4 q = p.qv[e >> 2];
        return (e & 3) == 0 ? q.x : (e & 3) == 1 ? q.y : (e & 3) == 2 ? q.z : q.w;
    };

    // Passes are visited in an order rotated by the workgroup's position inside its XCD
    // (workgroups are dealt to the 8 XCDs round-robin): all workgroups read the same Q arrays, and
    // without the rotation they would all ask the same few L2 channels for the same lines at once.
    const int64_t step = (int64_t)NT * CPT;
    const int npass_all = (int)((n + step - 1) / step);
    const int p_lo = half * ((npass_all + 1) / 2);
    const int npass = halves == 1 ? npass_all : (half == 0 ? (npass_all + 1) / 2 : npass_all / 2);   // passes of this workgroup
    const int rot = (int)((block / 8) % npass_all);
    auto pass_col = [&](int p) -> int64_t {
        int q = p_lo + p + rot;
        if (q >= npass_all) q -= npass_all;
        return (int64_t)q * step + (int64_t)threadIdx.x * CPT;
    };
    float num = 0.0f, den = 0.0f;                                   // NORMS: this thread's sums of squares
    auto compute_pass = [&](const Pass& cur, int64_t j0) {
#pragma unroll
        for (int g = 0; g < RG; ++g) {
            float acc[4][CPT];
#pragma unroll
            for (int t = 0; t < 4; ++t)
#pragma unroll
                for (int c = 0; c < CPT; ++c) acc[t][c] = 0.0f;
            if constexpr (kNoApplyMath) acc[0][0] = val_of(cur, 0) + __int_as_float((int)idx_of(cur, 0));
            else
#pragma unroll
            for (int c = 0; c < CPT; ++c)
#pragma unroll
                for (int k = 0; k < DD; ++k) {
                    const uint32_t unit = kNoConflicts ? ((idx_of(cur, c * DD + k) & ~15u) | (threadIdx.x & 15u)) : idx_of(cur, c * DD + k);
                    const f32x4 u = Us4[unit + g * (PS / 16)];
                    const float v = val_of(cur, c * DD + k);
                    acc[0][c] = fmaf(v, u.x, acc[0][c]);
                    acc[1][c] = fmaf(v, u.y, acc[1][c]);
                    acc[2][c] = fmaf(v, u.z, acc[2][c]);
                    acc[3][c] = fmaf(v, u.w, acc[3][c]);
                }
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const int64_t i = i0 + g * 4 + t;
                if (i < m) {
                    float w[CPT];
                    vec_widen<D, CPT>(cur.wv[g * 4 + t], w);
                    if constexpr (NORMS) {
#pragma unroll
                        for (int c = 0; c < CPT; ++c) {
                            const float diff = acc[t][c] - w[c];
                            num = fmaf(diff, diff, num);
                            den = fmaf(w[c], w[c], den);
                        }
                    } else {
#pragma unroll
                        for (int c = 0; c < CPT; ++c) w[c] -= acc[t][c];
                        stream_store(reinterpret_cast<Vec<D, CPT>*>(W + i * (int64_t)n + j0), vec_narrow<D, CPT>(w));
                    }
                }
            }
        }
    };

    // kDepth passes live in fixed register slots: one being computed, the others in flight.
    // (Copying a slot to another would wait for its loads.)
    Pass slot[kDepth];
    auto load_if = [&](int p, Pass& s) {
        if (p < npass) {
            const int64_t j = pass_col(p);
            if (j < n) load_pass(j, s);
        }
    };
    auto compute_if = [&](int p, const Pass& s) {
        if (p < npass) {
            const int64_t j = pass_col(p);
            if (j < n) compute_pass(s, j);
        }
    };
#pragma unroll
    for (int k = 0; k + 1 < kDepth; ++k) load_if(k, slot[k]);       // in flight while the U tile is built
    if constexpr (!kNoApplyU) build_u_tile_fast<RG, DD, PS, NT>(smem, pent, S, P_idx, P_val, i0, m, r);
    __syncthreads();
    for (int p = 0; p < npass; p += kDepth) {
#pragma unroll
        for (int k = 0; k < kDepth; ++k) {
            load_if(p + k + kDepth - 1, slot[(k + kDepth - 1) % kDepth]);
            compute_if(p + k, slot[k]);
        }
    }
    if constexpr (NORMS) block_sum2<NT>(num, den, reinterpret_cast<float2*>(smem), partial + blockIdx.x);
}

// Generic kernel: any n and d, one column per thread.
template <typename D, int RG, bool NORMS>
__global__ __launch_bounds__(kThreadsD) void k_decompress_any(typename D::elem* __restrict__ W, const float* __restrict__ S,
                                                             const int32_t* __restrict__ P_idx, const float* __restrict__ P_val,
                                                             const int32_t* __restrict__ Q_idx, const float* __restrict__ Q_val,
                                                             int m, int n, int r, int d, float2* __restrict__ partial) {
    extern __shared__ __align__(16) uint8_t smem[];
    float4* Us = reinterpret_cast<float4*>(smem);
    constexpr int R = 4 * RG;
    const int64_t i0 = (int64_t)blockIdx.x * R;
    build_u_tile<RG>(Us, S, P_idx, P_val, i0, m, r, d, r);
    __syncthreads();
    float num = 0.0f, den = 0.0f;                                   // NORMS: this thread's sums of squares
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
                    if constexpr (NORMS) {
                        const float w = widen<D>(*p), diff = acc[g][t] - w;
                        num = fmaf(diff, diff, num);
                        den = fmaf(w, w, den);
                    } else {
                        *p = narrow<D>(widen<D>(*p) - acc[g][t]);
                    }
                }
            }
    }
    if constexpr (NORMS) {
        __syncthreads();                                            // the tile of U is no longer read
        block_sum2<kThreadsD>(num, den, reinterpret_cast<float2*>(smem), partial + blockIdx.x);
    }
}

// Adds the workgroups' sums in order (in double) and forms the bias:
// out[0] = ||P S Q^T - G||_F^2, out[1] = ||G||_F^2, out[2] = sqrt(out[0] / out[1]).
__global__ __launch_bounds__(256) void k_bias_finish(const float2* __restrict__ partial, int count, float* __restrict__ out) {
    __shared__ double sx[256], sy[256];
    double x = 0.0, y = 0.0;
    for (int k = threadIdx.x; k < count; k += 256) { x += (double)partial[k].x; y += (double)partial[k].y; }
    sx[threadIdx.x] = x; sy[threadIdx.x] = y;
    __syncthreads();
    for (int off = 128; off > 0; off >>= 1) {
        if ((int)threadIdx.x < off) { sx[threadIdx.x] += sx[threadIdx.x + off]; sy[threadIdx.x] += sy[threadIdx.x + off]; }
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        out[0] = (float)sx[0]; out[1] = (float)sy[0];
        out[2] = (float)sqrt(sx[0] / sy[0]);
    }
}

// The fast kernel needs n % 4 == 0, r % 4 == 0 and d in {2, 4, 8, 16}; a group takes it only if all
// of its problems qualify.
static bool fast_shape(int32_t n, int32_t r, int32_t d) {
    return (n % 4) == 0 && (r % 4) == 0 && (d == 2 || d == 4 || d == 8 || d == 16);
}
bool apply_group_uniform(const ApplyGroup& g, int32_t r, int32_t d) {
    for (int p = 1; p < g.count; ++p)
        if (fast_shape(g.n[p], r, d) != fast_shape(g.n[0], r, d)) return false;
    return g.count == 1 || fast_shape(g.n[0], r, d);                // the generic kernel takes one problem at a time
}

// Row blocks at the end of a big launch of 32-row workgroups that are shared by two workgroups each: half a
// round of the 256 CUs (measured on the seven matrices of a 6.7B-style layer: 0 / 96 / 128 / 160 / 192 / 256
// blocks give 216 / 214 / 212 / 212 / 219 / 217 us per launch -- beyond that the second build of U costs more
// than the shorter tail saves).
constexpr int kTailSplitBlocks = 128;

template <typename D, int RG, int PS, int NT, int CPT, int DEPTH, bool NORMS = false>
static hipError_t launch_d(ApplyGroup& g, int32_t r, int32_t d, hipStream_t st, float2* partial = nullptr) {
    using E = typename D::elem;
    // widest matrices first: workgroups are started in index order as CUs fall free, and a workgroup's
    // run time grows with n, so the long ones should not be the last to start
    for (int a = 1; a < g.count; ++a)
        for (int b = a; b > 0 && g.n[b] > g.n[b - 1]; --b) {
            std::swap(g.W[b], g.W[b - 1]); std::swap(g.S[b], g.S[b - 1]); std::swap(g.P_idx[b], g.P_idx[b - 1]);
            std::swap(g.P_val[b], g.P_val[b - 1]); std::swap(g.Q_idx[b], g.Q_idx[b - 1]); std::swap(g.Q_val[b], g.Q_val[b - 1]);
            std::swap(g.m[b], g.m[b - 1]); std::swap(g.n[b], g.n[b - 1]);
        }
    g.first[0] = 0;
    for (int p = 0; p < g.count; ++p) g.first[p + 1] = g.first[p] + (g.m[p] + RG * 4 - 1) / (RG * 4);
    const int row_blocks = g.first[g.count];
    // big launches of 32-row workgroups: the last row blocks go to two workgroups each (see the kernel)
    const int tail = (!NORMS && RG == 8) ? std::min(row_blocks, kTailSplitBlocks) : 0;
    const int split_from = row_blocks - tail;
    const unsigned grid = (unsigned)(row_blocks + tail);
    hipError_t e;
    // d = 16: a pass holds 32 (column, value) pairs per thread, so only one pass fits the registers
#define LSP_LAUNCH_FAST(DDV)                                                                                   \
    do {                                                                                                       \
        constexpr auto kern = k_decompress<D, RG, DDV, PS, NT, CPT, (DDV == 16 ? 1 : DEPTH), NORMS>;                  \
        constexpr size_t lds = (size_t)RG * PS + (size_t)RG * 4 * DDV * sizeof(int2);                          \
        if ((e = allow_dynamic_lds<kern>(lds)) != hipSuccess) return e;                                        \
        hipLaunchKernelGGL(kern, dim3(grid), dim3(NT), lds, st, g, (int)r, partial, split_from);               \
    } while (0)
    if (!fast_shape(g.n[0], r, d)) {
        constexpr auto kern = k_decompress_any<D, RG, NORMS>;
        const size_t lds = (size_t)RG * r * 16;
        if ((e = allow_dynamic_lds<kern>((size_t)RG * LSP_MAX_R * 16)) != hipSuccess) return e;
        hipLaunchKernelGGL(kern, dim3(grid), dim3(kThreadsD), lds, st, static_cast<E*>(g.W[0]), g.S[0], g.P_idx[0], g.P_val[0],
                           g.Q_idx[0], g.Q_val[0], (int)g.m[0], (int)g.n[0], (int)r, (int)d, partial);
    }
    else if (d == 2) LSP_LAUNCH_FAST(2);
    else if (d == 4) LSP_LAUNCH_FAST(4);
    else if (d == 8) LSP_LAUNCH_FAST(8);
    else LSP_LAUNCH_FAST(16);
#undef LSP_LAUNCH_FAST
    return hipGetLastError();
}

// Rows per workgroup: 16 (four planes of U in LDS), 8 when the tile of U would not fit otherwise.
// Passes held in registers: three when the grid is small (few workgroups per CU, so each has to
// keep more bytes in flight itself), two otherwise.  Big grids (grouped calls) use workgroups of
// 256 threads, two of which share a CU and cover each other's set-up phase; when the tile of U
// allows it (256 < r <= 512) they use 32 rows per workgroup instead, so that the rows of Q are
// streamed from L2 half as often, with 512 threads: a row of the patch of W is then a 2 KB piece
// per pass, and the read-modify-write stream of W runs measurably faster on longer pieces (plain
// streaming kernels with this access pattern: 4.9 TB/s with 1 KB pieces, 5.4 TB/s with 2 KB ones).
template <typename D>
static hipError_t launch_d_shape(ApplyGroup& g, int32_t r, int32_t d, hipStream_t st) {
    constexpr int NT = 512, CPT = 2;
    int64_t blocks = 0;
    for (int p = 0; p < g.count; ++p) blocks += (g.m[p] + 15) / 16;
    const bool deep = blocks <= 512;
    const bool many = blocks >= 1024;
#define LSP_D_CASE(RGV, PSV)                                                          \
    return many ? launch_d<D, RGV, PSV, 256, CPT, 3>(g, r, d, st) :                   \
           deep ? launch_d<D, RGV, PSV, NT, CPT, 3>(g, r, d, st)                      \
                : launch_d<D, RGV, PSV, NT, CPT, 2>(g, r, d, st)
    if (r <= 256) LSP_D_CASE(4, 4096);
    if (256 < r && r <= 512 && many) return launch_d<D, 8, 8192, NT, CPT, 2>(g, r, d, st);    // 32 rows per workgroup
    if (r <= 512) LSP_D_CASE(4, 8192);
    if (r <= 1024) LSP_D_CASE(4, 16384);
    LSP_D_CASE(2, 32768);
#undef LSP_D_CASE
}

// Estimation bias: one problem, 16 (or 8) rows per workgroup, two passes deep.
int64_t bias_blocks(int64_t m, int32_t r) { return r <= 1024 ? (m + 15) / 16 : (m + 7) / 8; }

template <typename D>
static hipError_t launch_bias_shape(ApplyGroup& g, int32_t r, int32_t d, float2* partial, hipStream_t st) {
    if (r <= 256)  return launch_d<D, 4, 4096, 512, 2, 2, true>(g, r, d, st, partial);
    if (r <= 512)  return launch_d<D, 4, 8192, 512, 2, 2, true>(g, r, d, st, partial);
    if (r <= 1024) return launch_d<D, 4, 16384, 512, 2, 2, true>(g, r, d, st, partial);
    return launch_d<D, 2, 32768, 512, 2, 2, true>(g, r, d, st, partial);
}

hipError_t launch_bias(ApplyGroup& g, int32_t r, int32_t d, lsp_dtype dtype, float* partial, float* out, hipStream_t st) {
    float2* part = reinterpret_cast<float2*>(partial);
    hipError_t e;
    switch (dtype) {
        case LSP_F32:  e = launch_bias_shape<F32>(g, r, d, part, st); break;
        case LSP_F16:  e = launch_bias_shape<F16>(g, r, d, part, st); break;
        default:       e = launch_bias_shape<BF16>(g, r, d, part, st); break;
    }
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(k_bias_finish, dim3(1), dim3(256), 0, st, part, (int)bias_blocks(g.m[0], r), out);
    return hipGetLastError();
}

hipError_t launch_decompress(ApplyGroup& g, int32_t r, int32_t d, lsp_dtype dtype, hipStream_t st) {
    switch (dtype) {
        case LSP_F32:  return launch_d_shape<F32>(g, r, d, st);
        case LSP_F16:  return launch_d_shape<F16>(g, r, d, st);
        default:       return launch_d_shape<BF16>(g, r, d, st);
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
