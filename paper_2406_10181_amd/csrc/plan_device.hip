// Device-side construction and maintenance of a projector plan.
//
// The plan is the column-sorted copy of the two ELL projectors that the compress kernels walk
// (layout: lsp_internal.h; the host builder in plan.cpp defines its contents).  The projectors
// change when MaybeUpdate (Alg. 1) replaces them, and their values change in every iteration of
// the fitting loop, so a plan has to be cheap to make where the projectors live: on the GPU.
//
// Build.  The same bytes as the host builder, from kernels only, asynchronously on one stream:
//   1. one 64-bit key per stored entry, (chunk, subspace column, flat ELL position) for Q and
//      (subspace row, flat ELL position) for P, sorted by the device radix sort; the keys are
//      unique, so the sorted order is the (column, row, k) order of the host's counting sorts;
//   2. list boundaries by binary search; owners per column of T (long lists are shared between
//      lanes, spare lanes go to the longest lists), virtual columns, slots;
//   3. per chunk: the 512 lists dealt to the waves by length (rank by counting), segment lengths;
//   4. the waves' stream positions, then the interleaved (LDS offset, value) rows;
//   5. the rows of P^T cut into pieces.
// Errors that only the data can show (an index outside [0, r), columns too skewed for a plan) are
// left in a device status word and invalidate the plan's magic, so that a later compress call
// with it fills S with NaN instead of following it.
//
// Values-only refresh.  The plan records, for every value it holds, the flat ELL position it came
// from, so new values are dropped in place by one small kernel.
#include <algorithm>

#include <rocprim/device/device_radix_sort.hpp>

#include "lsp_internal.h"

namespace lsp {

// ---------------------------------------------------------------------------------------------
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

// ---------------------------------------------------------------------------------------------
// Build.  Scratch (device, caller's workspace), carved by build_scratch():
struct BuildScratch {
    uint64_t* keys_a;      // max(n, m) * d
    uint64_t* keys_b;      // max(n, m) * d
    uint32_t* start_q;     // nchunks * r + 1: first sorted position of each (chunk, column) list
    uint32_t* start_p;     // r + 1
    int32_t*  owners;      // r
    int32_t*  first_v;     // r + 1
    int32_t*  v_col;       // kMaxSlots * 512: column of a virtual column, -1 if none
    int32_t*  v_own;       // kMaxSlots * 512: which owner of its column it is
    uint32_t* seg_start;   // nchunks * kMaxSlots * 8: first stream row of each segment
    int32_t*  item_base;   // r + 1
    int32_t*  status;      // [0] lsp_status of the build, [1] nslots, [2] total rows, [3] build abandoned
    void*     sort_tmp;
    size_t    sort_tmp_bytes;
};

static int bits_for(uint64_t count) { int b = 1; while (b < 63 && ((uint64_t)1 << b) < count) ++b; return b; }

static size_t sort_tmp_bytes(size_t count) {
    size_t bytes = 0;
    uint64_t* none = nullptr;
    (void)rocprim::radix_sort_keys(nullptr, bytes, none, none, count, 0u, 64u, (hipStream_t)0, false);   // size query only
    return bytes;
}

static size_t build_scratch(uint8_t* base, int64_t m, int64_t n, int32_t r, int32_t d, BuildScratch* out) {
    const size_t nchunks = (size_t)((n + kChunk - 1) / kChunk);
    const size_t maxn = (size_t)std::max(m, n) * (size_t)d;
    size_t o = 0;
    auto take = [&](size_t bytes) { const size_t at = o; o = align_up(o + bytes, 256); return base ? base + at : nullptr; };
    BuildScratch s;
    s.keys_a = reinterpret_cast<uint64_t*>(take(maxn * 8));
    s.keys_b = reinterpret_cast<uint64_t*>(take(maxn * 8));
    s.start_q = reinterpret_cast<uint32_t*>(take((nchunks * (size_t)r + 1) * 4));
    s.start_p = reinterpret_cast<uint32_t*>(take(((size_t)r + 1) * 4));
    s.owners = reinterpret_cast<int32_t*>(take((size_t)r * 4));
    s.first_v = reinterpret_cast<int32_t*>(take(((size_t)r + 1) * 4));
    s.v_col = reinterpret_cast<int32_t*>(take((size_t)kMaxSlots * kThreadsGQ * 4));
    s.v_own = reinterpret_cast<int32_t*>(take((size_t)kMaxSlots * kThreadsGQ * 4));
    s.seg_start = reinterpret_cast<uint32_t*>(take(nchunks * kMaxSlots * kWavesGQ * 4));
    s.item_base = reinterpret_cast<int32_t*>(take(((size_t)r + 1) * 4));
    s.status = reinterpret_cast<int32_t*>(take(256));
    s.sort_tmp_bytes = sort_tmp_bytes(maxn);
    s.sort_tmp = take(s.sort_tmp_bytes);
    if (out) *out = s;
    return o;
}

size_t plan_build_workspace_bytes(int64_t m, int64_t n, int32_t r, int32_t d) { return build_scratch(nullptr, m, n, r, d, nullptr); }

typedef PlanLayout DevLayout;

__global__ __launch_bounds__(256) void k_fill_u32(uint32_t* __restrict__ p, int64_t count, uint32_t v) {
    for (int64_t k = (int64_t)blockIdx.x * 256 + threadIdx.x; k < count; k += (int64_t)gridDim.x * 256) p[k] = v;
}

// key of stored entry e = row * d + k: (list << ebits) | e, list = chunk * r + column for Q (chunk_rows = kChunk)
// and the subspace row for P (chunk_rows = 0).  An index outside [0, r) is recorded and replaced by 0.
__global__ __launch_bounds__(256) void k_build_keys(const int32_t* __restrict__ idx, int64_t count, int d, int r, int chunk_rows,
                                                    int ebits, uint64_t* __restrict__ keys, int32_t* __restrict__ status) {
    bool bad = false;
    for (int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x; e < count; e += (int64_t)gridDim.x * 256) {
        int b = idx[e];
        if (b < 0 || b >= r) { bad = true; b = 0; }
        const int64_t row = e / d;
        const uint64_t list = (chunk_rows ? (uint64_t)(row / chunk_rows) * (uint64_t)r : 0u) + (uint64_t)b;
        keys[e] = (list << ebits) | (uint64_t)e;
    }
    if (bad) status[0] = LSP_ERR_INDEX;
}

// start[l] = first sorted position whose list is >= l, for l = 0 .. nlists
__global__ __launch_bounds__(256) void k_list_bounds(const uint64_t* __restrict__ sorted, int64_t count, int ebits, int64_t nlists,
                                                     uint32_t* __restrict__ start) {
    for (int64_t l = (int64_t)blockIdx.x * 256 + threadIdx.x; l <= nlists; l += (int64_t)gridDim.x * 256) {
        const uint64_t want = (uint64_t)l << ebits;
        int64_t lo = 0, hi = count;
        while (lo < hi) {
            const int64_t mid = (lo + hi) >> 1;
            if (sorted[mid] < want) lo = mid + 1; else hi = mid;
        }
        start[l] = (uint32_t)lo;
    }
}

// share of owner o (of k) of the list [s0, s1): the same integer arithmetic as the host builder
__device__ __forceinline__ void share_of(uint32_t s0, uint32_t s1, int o, int k, int32_t& lo, int32_t& hi) {
    const int64_t len = (int64_t)s1 - (int64_t)s0;
    lo = (int32_t)s0 + (int32_t)(len * o / k);
    hi = (int32_t)s0 + (int32_t)(len * (o + 1) / k);
}

// Owners per column, virtual columns, header: one workgroup of 512 threads.
__global__ __launch_bounds__(kThreadsGQ) void k_q_owners(uint8_t* __restrict__ plan, DevLayout L, int m, int n, int r, int d, int nchunks,
                                                         int cap, const uint32_t* __restrict__ start_q, int32_t* __restrict__ owners_g,
                                                         int32_t* __restrict__ first_v_g, int32_t* __restrict__ v_col,
                                                         int32_t* __restrict__ v_own, int32_t* __restrict__ status) {
    __shared__ int32_t s_own[LSP_MAX_R], s_long[LSP_MAX_R], s_first[LSP_MAX_R + 1];
    __shared__ int32_t s_part[kThreadsGQ];
    __shared__ int32_t s_vneed;
    const int tid = threadIdx.x;
    int mine = 0;
    for (int b = tid; b < r; b += kThreadsGQ) {
        int32_t longest = 0;
        for (int c = 0; c < nchunks; ++c)
            longest = max(longest, (int32_t)(start_q[(int64_t)c * r + b + 1] - start_q[(int64_t)c * r + b]));
        s_long[b] = longest;
        s_own[b] = max(1, (longest + cap - 1) / cap);
        mine += s_own[b];
    }
    s_part[tid] = mine;
    __syncthreads();
    if (tid == 0) { int t = 0; for (int k = 0; k < kThreadsGQ; ++k) t += s_part[k]; s_vneed = t; }
    __syncthreads();
    const int vneed = s_vneed;
    // lanes left over go, one at a time, to the column whose owners have the longest share (ties: the lower
    // column), as long as that share is at least 64 pairs.  One wave does it, each lane keeping its columns
    // (b = lane + 64 q; r < 512 here, because every column has an owner already) in registers.
    if (vneed < kThreadsGQ && tid < kWave) {
        int own_l[8], long_l[8];
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            const int b = tid + kWave * q;
            own_l[q] = b < r ? s_own[b] : 1; long_l[q] = b < r ? s_long[b] : -1;
        }
        for (int spare = kThreadsGQ - vneed; spare > 0; --spare) {
            double best = -1.0; int best_b = 0x7FFFFFFF;
#pragma unroll
            for (int q = 0; q < 8; ++q) {
                const int b = tid + kWave * q;
                const double sh = (double)long_l[q] / (double)own_l[q];
                if (b < r && (sh > best || (sh == best && b < best_b))) { best = sh; best_b = b; }
            }
#pragma unroll
            for (int off = 32; off > 0; off >>= 1) {
                const double ob = __shfl_xor(best, off); const int obb = __shfl_xor(best_b, off);
                if (ob > best || (ob == best && obb < best_b)) { best = ob; best_b = obb; }
            }
            if (best < 64.0) break;                                  // uniform over the wave
#pragma unroll
            for (int q = 0; q < 8; ++q)
                if (best_b == tid + kWave * q) own_l[q]++;
        }
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            const int b = tid + kWave * q;
            if (b < r) s_own[b] = own_l[q];
        }
    }
    __syncthreads();
    if (tid == 0) {                                                  // first virtual column of each column
        int t = 0;
        for (int b = 0; b < r; ++b) { s_first[b] = t; t += s_own[b]; }
        s_first[r] = t;
    }
    __syncthreads();
    const int V = s_first[r];
    PlanHeader* H = reinterpret_cast<PlanHeader*>(plan);
    if (V > kMaxSlots * kThreadsGQ) {                                // more lists than the lanes can carry: no plan
        if (tid == 0) {
            if (status[0] == LSP_OK) status[0] = LSP_ERR_SKEW;
            status[3] = 1;                                           // the later kernels of the build do nothing
        }
        return;
    }
    const int nslots = max(1, (V + kThreadsGQ - 1) / kThreadsGQ);
    for (int v = tid; v < kMaxSlots * kThreadsGQ; v += kThreadsGQ) { v_col[v] = -1; v_own[v] = 0; }
    __syncthreads();
    int shared = 0;
    for (int b = tid; b < r; b += kThreadsGQ) {
        owners_g[b] = s_own[b];
        first_v_g[b] = s_first[b];
        shared |= s_own[b] > 1;
        for (int o = 0; o < s_own[b]; ++o) { v_col[s_first[b] + o] = b; v_own[s_first[b] + o] = o; }
    }
    if (tid == 0) first_v_g[r] = V;
    shared = __syncthreads_or(shared);
    uint16_t* vcol = reinterpret_cast<uint16_t*>(plan + L.off_q_vcol);
    uint16_t* vcnt = reinterpret_cast<uint16_t*>(plan + L.off_q_vcnt);
    for (int v = tid; v < nslots * kThreadsGQ; v += kThreadsGQ) {
        const int b = v_col[v];
        vcol[v] = b < 0 ? (uint16_t)kNoColumn : (uint16_t)((uint32_t)b | (s_own[b] > 1 ? kSharedColumn : 0u));
        vcnt[v] = (b >= 0 && v_own[v] == 0) ? (uint16_t)s_own[b] : (uint16_t)0;
    }
    if (tid == 0) {
        H->magic = kPlanMagic; H->m = m; H->n = n; H->r = r; H->d = d; H->nchunks = nchunks;
        H->nslots = nslots; H->nvcols = V; H->list_cap = cap;
        H->q_any_shared = shared ? 1 : 0; H->q_permuted = nslots == 1 ? 1 : 0;
        H->off_q_seg = L.off_q_seg; H->off_q_vcol = L.off_q_vcol; H->off_q_vcnt = L.off_q_vcnt; H->off_q_perm = L.off_q_perm;
        H->off_q_rows = L.off_q_rows; H->off_p_item = L.off_p_item; H->off_p_ent = L.off_p_ent; H->total_bytes = L.total;
        H->off_q_src = L.off_q_src; H->off_p_src = L.off_p_src;
        status[1] = nslots;
    }
}

// Per chunk: which virtual column each thread walks (lists dealt to the waves by length when there is one
// slot) and the segment lengths.  One workgroup of 512 threads per chunk.
__global__ __launch_bounds__(kThreadsGQ) void k_q_deal(uint8_t* __restrict__ plan, DevLayout L, int r, const uint32_t* __restrict__ start_q,
                                                       const int32_t* __restrict__ owners, const int32_t* __restrict__ v_col,
                                                       const int32_t* __restrict__ v_own, const int32_t* __restrict__ status) {
    if (status[3]) return;
    const int nslots = status[1];
    const int c = blockIdx.x, tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    __shared__ int32_t s_len[kThreadsGQ];
    __shared__ uint16_t s_order[kThreadsGQ];
    uint32_t* seg = reinterpret_cast<uint32_t*>(plan + L.off_q_seg);
    uint16_t* perm = reinterpret_cast<uint16_t*>(plan + L.off_q_perm);
    auto len_of = [&](int v) -> int32_t {
        const int b = v_col[v];
        if (b < 0) return 0;
        int32_t lo, hi;
        share_of(start_q[(int64_t)c * r + b], start_q[(int64_t)c * r + b + 1], v_own[v], owners[b], lo, hi);
        return hi - lo;
    };
    const bool permuted = nslots == 1;
    const int k_of_w = w < kWavesGQ / 2 ? w : kWavesGQ + kWavesGQ / 2 - 1 - w;      // group of 64 lists that wave w walks
    if (permuted) {
        const int32_t mylen = len_of(tid);
        s_len[tid] = mylen;
        __syncthreads();
        int rank = 0;                                                // longest first; equal lengths keep their order
        for (int u = 0; u < kThreadsGQ; ++u) {
            const int32_t lu = s_len[u];
            rank += (lu > mylen) || (lu == mylen && u < tid);
        }
        s_order[rank] = (uint16_t)tid;
        __syncthreads();
    } else {
        s_order[tid] = (uint16_t)tid;
        __syncthreads();
    }
    const int walked_p = s_order[k_of_w * kWave + lane];
    perm[(size_t)c * kThreadsGQ + tid] = (uint16_t)walked_p;
    for (int s = 0; s < nslots; ++s) {
        const int v = permuted ? walked_p : s * kThreadsGQ + tid;
        int32_t longest = len_of(v);
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) longest = max(longest, __shfl_xor(longest, off));
        if (lane == 0) seg[((size_t)c * nslots + s) * kWavesGQ + w] = (uint32_t)((longest + kSegBatch - 1) / kSegBatch * kSegBatch);
    }
}

// Stream positions: wave w's rows are contiguous over all chunks and slots, followed by kStreamSlack padding rows.
__global__ __launch_bounds__(64) void k_q_rowstart(uint8_t* __restrict__ plan, DevLayout L, int nchunks, uint32_t* __restrict__ seg_start,
                                                   int32_t* __restrict__ status) {
    if (status[3]) return;
    const int nslots = status[1];
    const uint32_t* seg = reinterpret_cast<const uint32_t*>(plan + L.off_q_seg);
    __shared__ uint32_t s_total[kWavesGQ];
    const int w = threadIdx.x;
    if (w < kWavesGQ) {
        uint32_t t = 0;
        for (int cs = 0; cs < nchunks * nslots; ++cs) t += seg[(size_t)cs * kWavesGQ + w];
        s_total[w] = t + kStreamSlack;
    }
    __syncthreads();
    if (w < kWavesGQ) {
        uint32_t row = 0;
        for (int k = 0; k < w; ++k) row += s_total[k];
        PlanHeader* H = reinterpret_cast<PlanHeader*>(plan);
        H->q_stream_row[w] = row;
        for (int cs = 0; cs < nchunks * nslots; ++cs) {
            seg_start[(size_t)cs * kWavesGQ + w] = row;
            row += seg[(size_t)cs * kWavesGQ + w];
        }
        if (w == kWavesGQ - 1) { H->q_total_rows = (int32_t)(row + kStreamSlack); status[2] = (int32_t)(row + kStreamSlack); }
    }
}

// The interleaved rows: block (cs, w) writes one segment; blocks past the segments write a wave's slack rows.
__global__ __launch_bounds__(256) void k_q_rows(uint8_t* __restrict__ plan, DevLayout L, int r, int d, int nchunks, int ebits,
                                                const uint64_t* __restrict__ sorted, const float* __restrict__ Q_val,
                                                const uint32_t* __restrict__ start_q, const int32_t* __restrict__ owners,
                                                const int32_t* __restrict__ v_col, const int32_t* __restrict__ v_own,
                                                const uint32_t* __restrict__ seg_start, const int32_t* __restrict__ status) {
    if (status[3]) return;
    const int nslots = status[1];
    const uint32_t* seg = reinterpret_cast<const uint32_t*>(plan + L.off_q_seg);
    const uint16_t* perm = reinterpret_cast<const uint16_t*>(plan + L.off_q_perm);
    uint2* rows = reinterpret_cast<uint2*>(plan + L.off_q_rows);
    uint32_t* qsrc = reinterpret_cast<uint32_t*>(plan + L.off_q_src);
    const uint2 pad_pair = make_uint2((uint32_t)kChunk * 16u, 0u);
    auto slot_of = [](size_t rw, int lane) { return ((rw >> 1) * kWave + (size_t)lane) * 2 + (rw & 1); };
    const int nseg = nchunks * nslots * kWavesGQ;
    const int blk = blockIdx.x;
    if (blk >= nseg + kWavesGQ) return;
    if (blk >= nseg) {                                               // slack rows behind wave w's stream
        const int w = blk - nseg;
        const PlanHeader* H = reinterpret_cast<const PlanHeader*>(plan);
        const uint32_t end = w + 1 < kWavesGQ ? H->q_stream_row[w + 1] : (uint32_t)status[2];
        for (int q = threadIdx.x; q < kStreamSlack * kWave; q += 256) {
            const size_t slot = slot_of((size_t)end - kStreamSlack + q / kWave, q % kWave);
            rows[slot] = pad_pair; qsrc[slot] = kNoSource;
        }
        return;
    }
    const int cs = blk / kWavesGQ, w = blk % kWavesGQ, c = cs / nslots, s = cs % nslots;
    const int len = (int)seg[(size_t)cs * kWavesGQ + w];
    const uint32_t row0 = seg_start[(size_t)cs * kWavesGQ + w];
    __shared__ int32_t s_lo[kWave], s_n[kWave];
    if (threadIdx.x < kWave) {
        const int lane = threadIdx.x;
        const int v = nslots == 1 ? (int)perm[(size_t)c * kThreadsGQ + w * kWave + lane] : s * kThreadsGQ + w * kWave + lane;
        const int b = v_col[v];
        int32_t lo = 0, hi = 0;
        if (b >= 0) share_of(start_q[(int64_t)c * r + b], start_q[(int64_t)c * r + b + 1], v_own[v], owners[b], lo, hi);
        s_lo[lane] = lo; s_n[lane] = hi - lo;
    }
    __syncthreads();
    const uint64_t emask = ((uint64_t)1 << ebits) - 1;
    for (int q = threadIdx.x; q < len * kWave; q += 256) {
        const int e = q / kWave, lane = q % kWave;
        const size_t slot = slot_of((size_t)row0 + e, lane);
        if (e < s_n[lane]) {
            const uint32_t src = (uint32_t)(sorted[s_lo[lane] + e] & emask);       // flat position j * d + k
            const uint32_t jl = (src / (uint32_t)d) - (uint32_t)c * kChunk;
            rows[slot] = make_uint2(chunk_col_offset(jl), __float_as_uint(Q_val[src]));
            qsrc[slot] = src;
        } else {
            rows[slot] = pad_pair; qsrc[slot] = kNoSource;
        }
    }
}

// Rows of P^T: pieces of at most kRowPiece entries; one workgroup.
__global__ __launch_bounds__(kThreadsGQ) void k_p_items(uint8_t* __restrict__ plan, DevLayout L, int r, const uint32_t* __restrict__ start_p,
                                                        int32_t* __restrict__ item_base, const int32_t* __restrict__ status) {
    if (status[3]) return;
    __shared__ int32_t s_cnt[LSP_MAX_R];
    __shared__ int32_t s_any;
    const int tid = threadIdx.x;
    if (tid == 0) s_any = 0;
    __syncthreads();
    for (int a = tid; a < r; a += kThreadsGQ) {
        const int32_t n_a = (int32_t)(start_p[a + 1] - start_p[a]);
        s_cnt[a] = max(1, (n_a + kRowPiece - 1) / kRowPiece);
        if (n_a > kRowPiece) s_any = 1;
    }
    __syncthreads();
    if (tid == 0) {
        int t = 0;
        for (int a = 0; a < r; ++a) { item_base[a] = t; t += s_cnt[a]; }
        item_base[r] = t;
        PlanHeader* H = reinterpret_cast<PlanHeader*>(plan);
        H->p_nitems = t; H->p_any_split = s_any;
    }
    __syncthreads();
    RowItem* items = reinterpret_cast<RowItem*>(plan + L.off_p_item);
    for (int a = tid; a < r; a += kThreadsGQ) {
        const int32_t s0 = (int32_t)start_p[a], s1 = (int32_t)start_p[a + 1];
        const int split = (s1 - s0) > kRowPiece;
        int at = item_base[a];
        if (s1 == s0) { items[at] = RowItem{a, s0, 0, 0}; continue; }
        for (int32_t s = s0; s < s1; s += kRowPiece) items[at++] = RowItem{a, s, min((int32_t)kRowPiece, s1 - s), split};
    }
}

__global__ __launch_bounds__(256) void k_p_entries(uint8_t* __restrict__ plan, DevLayout L, int64_t count, int d, int ebits,
                                                   const uint64_t* __restrict__ sorted, const float* __restrict__ P_val,
                                                   const int32_t* __restrict__ status) {
    if (status[3]) return;
    uint2* pent = reinterpret_cast<uint2*>(plan + L.off_p_ent);
    uint32_t* psrc = reinterpret_cast<uint32_t*>(plan + L.off_p_src);
    const uint64_t emask = ((uint64_t)1 << ebits) - 1;
    for (int64_t p = (int64_t)blockIdx.x * 256 + threadIdx.x; p < count; p += (int64_t)gridDim.x * 256) {
        const uint32_t src = (uint32_t)(sorted[p] & emask);
        pent[p] = make_uint2(src / (uint32_t)d, __float_as_uint(P_val[src]));
        psrc[p] = src;
    }
}

// A failed build leaves no plan behind: the magic is cleared, so compress calls with this buffer fill S with NaN.
__global__ void k_plan_seal(uint8_t* __restrict__ plan, const int32_t* __restrict__ status, int32_t* __restrict__ status_out) {
    if (status[0] != LSP_OK) reinterpret_cast<PlanHeader*>(plan)->magic = 0u;
    if (status_out) *status_out = status[0];
}

hipError_t launch_plan_build(const int32_t* P_idx, const float* P_val, const int32_t* Q_idx, const float* Q_val,
                             int64_t m, int64_t n, int32_t r, int32_t d, uint8_t* plan, uint8_t* workspace,
                             int32_t* status_out, hipStream_t st) {
    BuildScratch S;
    build_scratch(workspace, m, n, r, d, &S);
    const DevLayout L = plan_layout(m, n, r, d);
    const int nchunks = (int)((n + kChunk - 1) / kChunk);
    const int cap = plan_list_cap(r, d);
    const int64_t nq = n * d, np = m * d;
    const int ebits_q = bits_for((uint64_t)nq), ebits_p = bits_for((uint64_t)np);
    const int lbits_q = bits_for((uint64_t)nchunks * (uint64_t)r + 1), lbits_p = bits_for((uint64_t)r + 1);
    auto grid_for = [](int64_t count) { return dim3((unsigned)std::min<int64_t>((count + 255) / 256, 4096)); };
    hipError_t e;
    hipLaunchKernelGGL(k_fill_u32, grid_for((int64_t)(L.total / 4)), dim3(256), 0, st, reinterpret_cast<uint32_t*>(plan), (int64_t)(L.total / 4), 0u);
    hipLaunchKernelGGL(k_fill_u32, dim3(1), dim3(256), 0, st, reinterpret_cast<uint32_t*>(S.status), (int64_t)64, 0u);
    // ---- Q
    hipLaunchKernelGGL(k_build_keys, grid_for(nq), dim3(256), 0, st, Q_idx, nq, (int)d, (int)r, (int)kChunk, ebits_q, S.keys_a, S.status);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    size_t tmp = S.sort_tmp_bytes;
    if ((e = rocprim::radix_sort_keys(S.sort_tmp, tmp, S.keys_a, S.keys_b, (size_t)nq, 0u, (unsigned)(ebits_q + lbits_q), st, false)) != hipSuccess) return e;
    hipLaunchKernelGGL(k_list_bounds, grid_for((int64_t)nchunks * r + 1), dim3(256), 0, st, S.keys_b, nq, ebits_q, (int64_t)nchunks * r, S.start_q);
    hipLaunchKernelGGL(k_q_owners, dim3(1), dim3(kThreadsGQ), 0, st, plan, L, (int)m, (int)n, (int)r, (int)d, nchunks, cap, S.start_q,
                       S.owners, S.first_v, S.v_col, S.v_own, S.status);
    hipLaunchKernelGGL(k_q_deal, dim3((unsigned)nchunks), dim3(kThreadsGQ), 0, st, plan, L, (int)r, S.start_q, S.owners, S.v_col, S.v_own, S.status);
    hipLaunchKernelGGL(k_q_rowstart, dim3(1), dim3(64), 0, st, plan, L, nchunks, S.seg_start, S.status);
    hipLaunchKernelGGL(k_q_rows, dim3((unsigned)(nchunks * kMaxSlots * kWavesGQ + kWavesGQ)), dim3(256), 0, st, plan, L, (int)r, (int)d, nchunks,
                       ebits_q, S.keys_b, Q_val, S.start_q, S.owners, S.v_col, S.v_own, S.seg_start, S.status);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    // ---- P (the key buffers are free again: work on one stream is ordered)
    hipLaunchKernelGGL(k_build_keys, grid_for(np), dim3(256), 0, st, P_idx, np, (int)d, (int)r, 0, ebits_p, S.keys_a, S.status);
    tmp = S.sort_tmp_bytes;
    if ((e = rocprim::radix_sort_keys(S.sort_tmp, tmp, S.keys_a, S.keys_b, (size_t)np, 0u, (unsigned)(ebits_p + lbits_p), st, false)) != hipSuccess) return e;
    hipLaunchKernelGGL(k_list_bounds, grid_for((int64_t)r + 1), dim3(256), 0, st, S.keys_b, np, ebits_p, (int64_t)r, S.start_p);
    hipLaunchKernelGGL(k_p_items, dim3(1), dim3(kThreadsGQ), 0, st, plan, L, (int)r, S.start_p, S.item_base, S.status);
    hipLaunchKernelGGL(k_p_entries, grid_for(np), dim3(256), 0, st, plan, L, np, (int)d, ebits_p, S.keys_b, P_val, S.status);
    hipLaunchKernelGGL(k_plan_seal, dim3(1), dim3(1), 0, st, plan, S.status, status_out);
    return hipGetLastError();
}

}  // namespace lsp
