// Compress, kernel A, fp32-staged variant: T = G Q for fp32 storage and for rows that are not whole
// 8-element groups (any storage type).  See compress.hip for the path as a whole.
#include "compress_common.h"

namespace lsp {

// ----------------------------------------------------------------------------------------------
// eight consecutive elements of one row, as loaded
template <typename D> struct Oct;
template <> struct Oct<F32>  { float4 lo, hi; };
template <> struct Oct<F16>  { uint4 v; };
template <> struct Oct<BF16> { uint4 v; };

template <typename D> __device__ __forceinline__ Oct<D> oct_zero();
template <> __device__ __forceinline__ Oct<F32> oct_zero<F32>() { return {make_float4(0, 0, 0, 0), make_float4(0, 0, 0, 0)}; }
template <> __device__ __forceinline__ Oct<F16> oct_zero<F16>() { return {make_uint4(0, 0, 0, 0)}; }
template <> __device__ __forceinline__ Oct<BF16> oct_zero<BF16>() { return {make_uint4(0, 0, 0, 0)}; }

template <typename D> __device__ __forceinline__ Oct<D> oct_load(const typename D::elem* p);
template <> __device__ __forceinline__ Oct<F32> oct_load<F32>(const float* p) {
    const float4* q = reinterpret_cast<const float4*>(p);
    return {stream_load(q), stream_load(q + 1)};
}
template <> __device__ __forceinline__ Oct<F16> oct_load<F16>(const uint16_t* p) { return {stream_load(reinterpret_cast<const uint4*>(p))}; }
template <> __device__ __forceinline__ Oct<BF16> oct_load<BF16>(const uint16_t* p) { return {stream_load(reinterpret_cast<const uint4*>(p))}; }

// element-wise, bounds-checked variant for ragged or unaligned rows
template <typename D> __device__ __forceinline__ void oct_gather(const typename D::elem* row, int64_t col0, int64_t n, float out[8]) {
#pragma unroll
    for (int q = 0; q < 8; ++q) out[q] = (col0 + q < n) ? widen<D>(row[col0 + q]) : 0.0f;
}

template <typename D> __device__ __forceinline__ void oct_widen(const Oct<D>& o, float out[8]);
template <> __device__ __forceinline__ void oct_widen<F32>(const Oct<F32>& o, float out[8]) {
    out[0] = o.lo.x; out[1] = o.lo.y; out[2] = o.lo.z; out[3] = o.lo.w;
    out[4] = o.hi.x; out[5] = o.hi.y; out[6] = o.hi.z; out[7] = o.hi.w;
}
template <> __device__ __forceinline__ void oct_widen<BF16>(const Oct<BF16>& o, float out[8]) {
    const uint32_t w[4] = {o.v.x, o.v.y, o.v.z, o.v.w};
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        out[2 * q]     = __uint_as_float(w[q] << 16);
        out[2 * q + 1] = __uint_as_float(w[q] & 0xFFFF0000u);
    }
}
template <> __device__ __forceinline__ void oct_widen<F16>(const Oct<F16>& o, float out[8]) {
    const uint32_t w[4] = {o.v.x, o.v.y, o.v.z, o.v.w};
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        out[2 * q]     = widen<F16>((uint16_t)(w[q] & 0xFFFFu));
        out[2 * q + 1] = widen<F16>((uint16_t)(w[q] >> 16));
    }
}

// ----------------------------------------------------------------------------------------------
// Kernel A.  One workgroup = 16 rows of G (4 planes of 4 rows), 512 threads, one lane per
// (virtual) column of T; the lane keeps its 16 partial sums per owned column in registers for the
// whole kernel, so there is no flush and no atomic in the main loop.
// LDS: 4 planes of kPlaneStride bytes (staged chunk of G, fp32); at the very end the same memory
// holds the T tile [16][r] when partial sums of several owners have to meet.
// Each wave reads one linear stream of plan rows (64 x (LDS offset, value)); segment lengths come
// from a small table (scalar loads).
// VEC: rows are 8-element aligned (n % 8 == 0), vector loads; otherwise element-wise loads.

// Global -> register -> LDS staging of one chunk of G, shared by both variants of kernel A.
template <typename D, bool VEC>
struct ChunkStager {
    static constexpr int UNITS = kPlanes * (kChunk / 8);      // (plane, column octet) units per chunk
    static constexpr int UPT = UNITS / kThreadsGQ;            // units per thread
    static_assert(UNITS % kThreadsGQ == 0, "staging assumes whole units per thread");
    Oct<D> pre[VEC ? UPT : 1][VEC ? 4 : 1];
    float  preg[VEC ? 1 : UPT][VEC ? 1 : 4][VEC ? 1 : 8];

    __device__ __forceinline__ void fetch(const typename D::elem* __restrict__ G, int64_t i0, int m, int n, int c, int tid) {
#pragma unroll
        for (int u = 0; u < UPT; ++u) {
            const int unit = tid + u * kThreadsGQ;
            const int plane = unit / (kChunk / 8), oct = unit % (kChunk / 8);
            const int64_t col0 = (int64_t)c * kChunk + (int64_t)oct * 8;
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const int64_t row = i0 + plane * 4 + t;
                const bool ok = row < m && col0 < n;
                if constexpr (VEC) {
                    // always load (from a clamped, valid address) and select afterwards: a branch
                    // around the load would make the wave wait for each load in turn
                    const int64_t rowc = row < m ? row : (int64_t)m - 1, colc = col0 < n ? col0 : 0;
                    pre[u][t] = oct_load<D>(G + rowc * (int64_t)n + colc);
                    if (!ok) pre[u][t] = oct_zero<D>();
                } else {
                    if (ok) oct_gather<D>(G + row * (int64_t)n, col0, n, preg[u][t]);
                    else {
#pragma unroll
                        for (int q = 0; q < 8; ++q) preg[u][t][q] = 0.0f;
                    }
                }
            }
        }
    }
    __device__ __forceinline__ void stage(uint8_t* smem, int tid) const {
#pragma unroll
        for (int u = 0; u < UPT; ++u) {
            const int unit = tid + u * kThreadsGQ;
            const int plane = unit / (kChunk / 8), oct = unit % (kChunk / 8);
            float f[4][8];
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                if constexpr (VEC) oct_widen<D>(pre[u][t], f[t]);
                else {
#pragma unroll
                    for (int q = 0; q < 8; ++q) f[t][q] = preg[u][t][q];
                }
            }
            uint8_t* base = smem + plane * kPlaneStride + oct * 16;
#pragma unroll
            for (int q = 0; q < 8; ++q)
                *reinterpret_cast<f32x4*>(base + q * (kChunk / 8) * 16) = f32x4{f[0][q], f[1][q], f[2][q], f[3][q]};
        }
    }
};

// the staged values of the two columns named by e, for all 16 rows
__device__ __forceinline__ void gather_pair(const uint8_t* smem, const u32x4 e, f32x4 (&x)[2][kPlanes]) {
#pragma unroll
    for (int h = 0; h < 2; ++h)
#pragma unroll
        for (int g = 0; g < kPlanes; ++g)
            x[h][g] = *reinterpret_cast<const f32x4*>(smem + (h ? e.z : e.x) + g * kPlaneStride);
}
__device__ __forceinline__ void fma_pair(const u32x4 e, const f32x4 (&x)[2][kPlanes], float (&acc)[kPlanes][4]) {
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const float v = __uint_as_float(h ? e.w : e.y);
#pragma unroll
        for (int g = 0; g < kPlanes; ++g) {
            acc[g][0] = fmaf(v, x[h][g].x, acc[g][0]);
            acc[g][1] = fmaf(v, x[h][g].y, acc[g][1]);
            acc[g][2] = fmaf(v, x[h][g].z, acc[g][2]);
            acc[g][3] = fmaf(v, x[h][g].w, acc[g][3]);
        }
    }
}

// acc[g][t] += value * (staged G)[row 4g+t][column] for the two (offset, value) pairs of e
__device__ __forceinline__ void consume_pair(const uint8_t* smem, const u32x4 e, float (&acc)[kPlanes][4]) {
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const uint32_t off = h ? e.z : e.x;
        const float v = __uint_as_float(h ? e.w : e.y);
#pragma unroll
        for (int g = 0; g < kPlanes; ++g) {
            const f32x4 x = *reinterpret_cast<const f32x4*>(smem + off + g * kPlaneStride);
            acc[g][0] = fmaf(v, x.x, acc[g][0]);
            acc[g][1] = fmaf(v, x.y, acc[g][1]);
            acc[g][2] = fmaf(v, x.z, acc[g][2]);
            acc[g][3] = fmaf(v, x.w, acc[g][3]);
        }
    }
}


// Common case: every lane owns at most one column (nslots == 1).  The wave's plan stream is
// consumed as one flat sequence of batches, kPrefetch batches deep in registers, running ahead
// across chunk boundaries; a chunk boundary only costs the two barriers around the staging.
template <typename D, bool VEC>
__device__ __forceinline__ void gq_one_slot(ChunkStager<D, VEC>& stg, uint8_t* smem, const typename D::elem* __restrict__ G,
                                            const uint8_t* __restrict__ plan, PlanHeaderPtr H,
                                            float* __restrict__ T, int64_t i0, int m, int n, int r,
                                            int tid, int lane, int wave) {
    const int nchunks = H->nchunks;
    const auto* seg = as_const<uint32_t>(plan + H->off_q_seg) + wave;
    const u32x4* rp = reinterpret_cast<const u32x4*>(plan + H->off_q_rows) + (size_t)(H->q_stream_row[wave] >> 1) * kWave + lane;
    const uint32_t mycol = as_const<uint16_t>(plan + H->off_q_vcol)[tid];
    const uint16_t* __restrict__ perm = reinterpret_cast<const uint16_t*>(plan + H->off_q_perm) + tid;
    uint32_t walked = perm[0];                                        // virtual column whose list this thread walks

    // Ring of kPrefetch batches with fixed register slots: slot k is consumed, then refilled with
    // the batch kPrefetch further on.  (Shifting the ring instead would make every iteration wait
    // for the newest load.)  Slot 0 holds the oldest batch at the start of each chunk; a chunk
    // whose batch count is not a multiple of kPrefetch leaves the ring rotated, which is undone
    // once per chunk, behind the staging barrier, when the loads in flight have long landed.
    u32x4 ring[kPrefetch][kBatchLoads];
#pragma unroll
    for (int k = 0; k < kPrefetch; ++k)
#pragma unroll
        for (int q = 0; q < kBatchLoads; ++q) ring[k][q] = rp[(size_t)(k * kBatchLoads + q) * kWave];
    rp += (size_t)kPrefetch * kBatchLoads * kWave;

    float acc[1][kPlanes][4];
#pragma unroll
    for (int g = 0; g < kPlanes; ++g) acc[0][g][0] = acc[0][g][1] = acc[0][g][2] = acc[0][g][3] = 0.0f;

    auto step = [&](u32x4 (&slot)[kBatchLoads]) {
        // gathers of pair q+1 are issued before the multiply-adds of pair q, not further ahead, so
        // that at most two pairs of gathered data (64 registers) are live
        f32x4 x[2][2][kPlanes];
        gather_pair(smem, slot[0], x[0]);
#pragma unroll
        for (int q = 0; q < kBatchLoads; ++q) {
            if (q + 1 < kBatchLoads) gather_pair(smem, slot[q + 1], x[(q + 1) & 1]);
            __builtin_amdgcn_sched_barrier(0);
            fma_pair(slot[q], x[q & 1], acc[0]);
            __builtin_amdgcn_sched_barrier(0);
        }
#pragma unroll
        for (int q = 0; q < kBatchLoads; ++q) slot[q] = rp[(size_t)q * kWave];
        rp += (size_t)kBatchLoads * kWave;
    };

    int rot = 0;                                                      // slots the ring is rotated by
    for (int c = 0; c < nchunks; ++c) {
        __syncthreads();                                              // everyone is done reading the previous chunk
        stg.stage(smem, tid);
        __syncthreads();
        if (c + 1 < nchunks) stg.fetch(G, i0, m, n, c + 1, tid);
        const uint32_t next = c + 1 < nchunks ? (uint32_t)perm[(size_t)(c + 1) * kThreadsGQ] : (uint32_t)tid;
        if (rot != 0) {
            u32x4 t[kPrefetch][kBatchLoads];
#pragma unroll
            for (int k = 0; k < kPrefetch; ++k)
#pragma unroll
                for (int q = 0; q < kBatchLoads; ++q) {
                    t[k][q] = ring[(k + 1) % kPrefetch][q];
                    if (rot == 2) t[k][q] = ring[(k + 2) % kPrefetch][q];
                    if (rot == 3) t[k][q] = ring[(k + 3) % kPrefetch][q];
                }
#pragma unroll
            for (int k = 0; k < kPrefetch; ++k)
#pragma unroll
                for (int q = 0; q < kBatchLoads; ++q) ring[k][q] = t[k][q];
        }
        static_assert(kPrefetch == 4, "the rotation above is written for four slots");
        const int nb = (int)(seg[c * kWavesGQ] / kSegBatch);
        for (int g = nb / kPrefetch; g > 0; --g) {
            step(ring[0]); step(ring[1]); step(ring[2]); step(ring[3]);
        }
        rot = nb % kPrefetch;
        if (rot > 0) step(ring[0]);
        if (rot > 1) step(ring[1]);
        if (rot > 2) step(ring[2]);
        // the sums move to the lanes that walk the columns next; after the last chunk, home (thread t: column t)
        swap_owner(smem, reinterpret_cast<float(&)[kRowsGQ]>(acc), walked, next);   // through the LDS of the chunk just consumed
        walked = next;
    }
    if (H->q_any_shared) {
        write_tile_shared<1>(smem, plan, H, T, reinterpret_cast<const float(&)[1][kRowsGQ]>(acc), 1, i0, m, r, tid);
    } else if (mycol != kNoColumn) {
#pragma unroll
        for (int g = 0; g < kPlanes; ++g)
#pragma unroll
            for (int t = 0; t < 4; ++t)
                if (i0 + g * 4 + t < m) T[(i0 + g * 4 + t) * (int64_t)r + mycol] = acc[0][g][t];
    }
}

// General case (up to kMaxSlots columns per lane): slot by slot inside each chunk, one batch ahead.
template <typename D, bool VEC>
__device__ __attribute__((noinline)) void gq_any_slots(ChunkStager<D, VEC> stg, uint8_t* smem, const typename D::elem* __restrict__ G,
                                             const uint8_t* __restrict__ plan, PlanHeaderPtr H,
                                             float* __restrict__ T, int64_t i0, int m, int n, int r,
                                             int tid, int lane, int wave) {
    const int nchunks = H->nchunks;
    const int nslots = H->nslots;
    const auto* seg = as_const<uint32_t>(plan + H->off_q_seg);
    const u32x4* rp = reinterpret_cast<const u32x4*>(plan + H->off_q_rows) + (size_t)(H->q_stream_row[wave] >> 1) * kWave + lane;

    float acc[kMaxSlots][kPlanes][4];
#pragma unroll
    for (int s = 0; s < kMaxSlots; ++s)
#pragma unroll
        for (int g = 0; g < kPlanes; ++g) acc[s][g][0] = acc[s][g][1] = acc[s][g][2] = acc[s][g][3] = 0.0f;

    u32x4 cur[kBatchLoads], nxt[kBatchLoads];
#pragma unroll
    for (int q = 0; q < kBatchLoads; ++q) cur[q] = rp[(size_t)q * kWave];

    for (int c = 0; c < nchunks; ++c) {
        __syncthreads();                     // everyone is done reading the previous chunk
        stg.stage(smem, tid);
        __syncthreads();
        if (c + 1 < nchunks) stg.fetch(G, i0, m, n, c + 1, tid);
#pragma unroll
        for (int s = 0; s < kMaxSlots; ++s) {
            if (s < nslots) {
                const int nb = (int)(seg[(c * nslots + s) * kWavesGQ + wave] / kSegBatch);
                for (int b = 0; b < nb; ++b) {
#pragma unroll
                    for (int q = 0; q < kBatchLoads; ++q) nxt[q] = rp[(size_t)(kBatchLoads + q) * kWave];   // one batch ahead
#pragma unroll
                    for (int q = 0; q < kBatchLoads; ++q) consume_pair(smem, cur[q], acc[s]);
#pragma unroll
                    for (int q = 0; q < kBatchLoads; ++q) cur[q] = nxt[q];
                    rp += (size_t)kBatchLoads * kWave;
                }
            }
        }
    }
    write_tile_shared<kMaxSlots>(smem, plan, H, T, reinterpret_cast<const float(&)[kMaxSlots][kRowsGQ]>(acc), nslots, i0, m, r, tid);
}

template <typename D, bool VEC>
__global__ __launch_bounds__(kThreadsGQ) void k_compress_gq(const CompressGroup grp, int r, int d) {
    extern __shared__ __align__(16) uint8_t smem[];
    const CompressProblem pr = group_pick(grp, (int)blockIdx.x, false);
    const typename D::elem* __restrict__ G = static_cast<const typename D::elem*>(pr.G);
    const uint8_t* __restrict__ plan = pr.plan;
    float* __restrict__ T = pr.T;
    float* __restrict__ S = pr.S;
    const int m = pr.m, n = pr.n;
    const int block = pr.block_gq, nblocks = pr.nblocks_gq;
    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int64_t i0 = (int64_t)block * kRowsGQ;

    ChunkStager<D, VEC> stg;
    stg.fetch(G, i0, m, n, 0, tid);                                   // depends on nothing but the arguments

    PlanHeaderPtr H = as_const<PlanHeader>(plan);
    if (!plan_matches(H, m, n, r, d)) {                               // not a plan for this problem
        poison_s(S, r, block, nblocks, tid, kThreadsGQ);
        return;
    }
    // S must start at zero only when some row of P^T was cut into pieces (kernel B then adds).
    if (H->p_any_split) {
        const int64_t total = (int64_t)r * r;
        for (int64_t k = (int64_t)block * kThreadsGQ + tid; k < total; k += (int64_t)nblocks * kThreadsGQ) S[k] = 0.0f;
    }
    if (tid < kPlanes) *reinterpret_cast<f32x4*>(smem + tid * kPlaneStride + kChunk * 16) = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
    if (H->nslots == 1) gq_one_slot<D, VEC>(stg, smem, G, plan, H, T, i0, m, n, r, tid, lane, wave);
    else                gq_any_slots<D, VEC>(stg, smem, G, plan, H, T, i0, m, n, r, tid, lane, wave);
}


template <typename D>
static hipError_t launch_one(const CompressGroup& g, int32_t r, int32_t d, hipStream_t st) {
    constexpr size_t lds = (size_t)kPlanes * kPlaneStride;   // >= 64 r bytes for every supported r
    const bool vec = (g.n[0] % 8) == 0;
    const unsigned grid = (unsigned)g.first_gq[g.count];
    hipError_t e;
    if (vec) {
        if ((e = allow_dynamic_lds<k_compress_gq<D, true>>(lds)) != hipSuccess) return e;
        hipLaunchKernelGGL((k_compress_gq<D, true>), dim3(grid), dim3(kThreadsGQ), lds, st, g, (int)r, (int)d);
    } else {
        if ((e = allow_dynamic_lds<k_compress_gq<D, false>>(lds)) != hipSuccess) return e;
        hipLaunchKernelGGL((k_compress_gq<D, false>), dim3(grid), dim3(kThreadsGQ), lds, st, g, (int)r, (int)d);
    }
    return hipGetLastError();
}

hipError_t launch_gq_staged32(const CompressGroup& g, int32_t r, int32_t d, lsp_dtype dtype, hipStream_t st) {
    switch (dtype) {
        case LSP_F32:  return launch_one<F32>(g, r, d, st);
        case LSP_F16:  return launch_one<F16>(g, r, d, st);
        default:       return launch_one<BF16>(g, r, d, st);
    }
}

}  // namespace lsp
