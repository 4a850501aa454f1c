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

#include <utility>

#include "lsp_internal.h"

namespace lsp {

constexpr int kPlaneStride = kChunk * 16 + 16;   // bytes; last 16 bytes of a plane stay zero
typedef float f32x4 __attribute__((ext_vector_type(4)));

// A plan is only followed when its header names this very problem: the offsets and counts in it
// index S and T with the call's r and m, so a plan built for other sizes (or a buffer that holds no
// plan at all) must not be walked.  Kernel A then fills S with NaN, which is how the caller sees
// the mistake, and kernel B does nothing; all kernels exit normally.
__device__ __forceinline__ bool plan_matches(PlanHeaderPtr H, int m, int n, int r, int d) {
    return H->magic == kPlanMagic && H->m == m && H->n == n && H->r == r && H->d == d;
}
__device__ __forceinline__ void poison_s(float* __restrict__ S, int r, int block, int nblocks, int tid, int nthreads) {
    const int64_t total = (int64_t)r * r;
    for (int64_t k = (int64_t)block * nthreads + tid; k < total; k += (int64_t)nblocks * nthreads) S[k] = __builtin_nanf("");
}

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
constexpr int kPlanes = 4;
constexpr int kRowsGQ = 4 * kPlanes;
constexpr int kBatchLoads = kSegBatch / 2;                    // 128-bit loads per batch of plan rows

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

// Partial sums of several owners of one column meet in LDS: every lane parks its 16 sums at its
// virtual column, [16][nslots * 512] floats; the first owner of a column then adds the owners'
// sums in owner order (they sit side by side) and stores the column of T.  No atomics, so the
// result does not depend on timing.  Called by all threads of the workgroup.
template <int NS>
__device__ __forceinline__ void write_tile_shared(uint8_t* smem, const uint8_t* plan, PlanHeaderPtr H, float* __restrict__ T,
                                                  const float (&acc)[NS][kRowsGQ], int nslots, int64_t i0, int m, int r, int tid) {
    __syncthreads();                                                  // the staged chunk is no longer read
    float* Tl = reinterpret_cast<float*>(smem);
    const int V = nslots * kThreadsGQ;
    const auto* vcol = as_const<uint16_t>(plan + H->off_q_vcol);
    const auto* vcnt = as_const<uint16_t>(plan + H->off_q_vcnt);
#pragma unroll
    for (int s = 0; s < NS; ++s) {
        if (s < nslots) {
#pragma unroll
            for (int t = 0; t < kRowsGQ; ++t) Tl[t * V + s * kThreadsGQ + tid] = acc[s][t];
        }
    }
    __syncthreads();
#pragma unroll
    for (int s = 0; s < NS; ++s) {
        if (s < nslots) {
            const int v = s * kThreadsGQ + tid;
            const int owners = vcnt[v];
            if (owners > 0) {
                const uint32_t bb = vcol[v] & 0x7FFFu;
                for (int t = 0; t < kRowsGQ; ++t) {
                    float sum = Tl[t * V + v];
                    for (int o = 1; o < owners; ++o) sum += Tl[t * V + v + o];
                    if (i0 + t < m) T[(i0 + t) * (int64_t)r + bb] = sum;
                }
            }
        }
    }
}

// Hands the 16 partial sums of every virtual column from the lane that walked its list in one
// chunk to the lane that walks it in the next (`from`, `to`: virtual columns of this thread; the
// plan deals the lists of each chunk to the waves by length).  They pass through the first 32 KB
// of `area`, the LDS of the chunk consumed last: the first barrier makes sure nobody reads that
// chunk any more (and publishes whatever was written to other LDS before the call), the last one
// that the area may be staged into again.  Called by all threads.
__device__ __forceinline__ void swap_owner(uint8_t* area, float (&acc)[16], uint32_t from, uint32_t to) {
    f32x4* X = reinterpret_cast<f32x4*>(area);
    __syncthreads();
#pragma unroll
    for (int q = 0; q < 4; ++q)
        X[q * kThreadsGQ + from] = f32x4{acc[4 * q], acc[4 * q + 1], acc[4 * q + 2], acc[4 * q + 3]};   // lanes spread over all banks
    __syncthreads();
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const f32x4 a = X[q * kThreadsGQ + to];
        acc[4 * q] = a[0]; acc[4 * q + 1] = a[1]; acc[4 * q + 2] = a[2]; acc[4 * q + 3] = a[3];
    }
    __syncthreads();
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

// ----------------------------------------------------------------------------------------------
// 16-bit storage types (fp16, bf16), n % 8 == 0, one column per lane: G is staged as it is stored,
// 8 rows to a 16-byte LDS unit ([plane of 8 rows][column][8 rows]), so one 128-bit gather serves
// eight rows (half the LDS bytes per pair) and a chunk takes half the space: the LDS holds two
// chunks, the one being consumed and the one being staged, with one barrier per chunk.  The
// elements are widened in registers when they are used (exact: a shift or mask for bf16, a
// conversion for fp16).
constexpr int kPlanes16 = 2;                                          // planes of 8 rows
constexpr int kBufStride16 = kPlanes16 * kPlaneStride;                // bytes between the two chunk buffers
static_assert(2 * kBufStride16 == kPlanes * kPlaneStride, "both layouts use the same LDS allocation");

template <typename D> __device__ __forceinline__ void widen2(uint32_t w, float& lo, float& hi);
template <> __device__ __forceinline__ void widen2<BF16>(uint32_t w, float& lo, float& hi) {
    lo = __uint_as_float(w << 16); hi = __uint_as_float(w & 0xFFFF0000u);
}
template <> __device__ __forceinline__ void widen2<F16>(uint32_t w, float& lo, float& hi) {
    typedef _Float16 h2 __attribute__((ext_vector_type(2)));
    h2 h; __builtin_memcpy(&h, &w, 4);
    lo = (float)h.x; hi = (float)h.y;
}

struct ChunkStager16 {
    u32x4 pre[8];                                                     // 8 rows x 8 columns, as stored
    uint32_t live = 0;                                                // bit t: pre[t] holds data of the matrix

    template <typename E>
    __device__ __forceinline__ void fetch(const E* __restrict__ G, int64_t i0, int m, int n, int c, int tid) {
        const int plane = tid / (kChunk / 8), oct = tid % (kChunk / 8);
        const int64_t col0 = (int64_t)c * kChunk + (int64_t)oct * 8;
        const int64_t colc = col0 < n ? col0 : 0;                    // clamped: always a valid address
        live = 0;
#pragma unroll
        for (int t = 0; t < 8; ++t) {
            const int64_t row = i0 + plane * 8 + t;
            const int64_t rowc = row < m ? row : (int64_t)m - 1;
            pre[t] = stream_load(reinterpret_cast<const u32x4*>(G + rowc * (int64_t)n + colc));
            live |= (row < m && col0 < n) ? (1u << t) : 0u;
        }
    }
    // transposes the 8x8 block and writes its 8 units (column q: rows 0..7) into buffer `buf`
    __device__ __forceinline__ void stage(uint8_t* smem, int buf, int tid) {
        const int plane = tid / (kChunk / 8), oct = tid % (kChunk / 8);
        if (live != 0xFFu) {
#pragma unroll
            for (int t = 0; t < 8; ++t)
                if (!((live >> t) & 1u)) pre[t] = u32x4{0u, 0u, 0u, 0u};
        }
        uint8_t* base = smem + buf * kBufStride16 + plane * kPlaneStride + oct * 16;
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            u32x4 unit;
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const uint32_t a = pre[2 * k][q >> 1], b = pre[2 * k + 1][q >> 1];   // rows 2k, 2k+1; columns q&~1, q|1
                unit[k] = (q & 1) ? ((a >> 16) | (b & 0xFFFF0000u)) : ((a & 0xFFFFu) | (b << 16));
            }
            *reinterpret_cast<u32x4*>(base + q * (kChunk / 8) * 16) = unit;
        }
    }
};

__device__ __forceinline__ void gather_pair16(const uint8_t* buf, const u32x4 e, u32x4 (&x)[2][kPlanes16]) {
#pragma unroll
    for (int h = 0; h < 2; ++h)
#pragma unroll
        for (int g = 0; g < kPlanes16; ++g)
            x[h][g] = *reinterpret_cast<const u32x4*>(buf + (h ? e.z : e.x) + g * kPlaneStride);
}
template <typename D>
__device__ __forceinline__ void fma_pair16(const u32x4 e, const u32x4 (&x)[2][kPlanes16], float (&acc)[kRowsGQ]) {
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const float v = __uint_as_float(h ? e.w : e.y);
#pragma unroll
        for (int g = 0; g < kPlanes16; ++g)
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                float lo, hi;
                widen2<D>(x[h][g][k], lo, hi);
                acc[g * 8 + 2 * k]     = fmaf(v, lo, acc[g * 8 + 2 * k]);
                acc[g * 8 + 2 * k + 1] = fmaf(v, hi, acc[g * 8 + 2 * k + 1]);
            }
    }
}

// One workgroup walks `nblk` consecutive blocks of 16 rows (several when the grid is big: the first
// chunk of the next block is fetched and staged while the last chunk of the current one is
// consumed, and the stores of T go out under the next block's work, so that the set-up and the
// tail of a block cost nothing but for the first and the last one).
template <typename D>
__device__ __forceinline__ void gq16_one_slot(ChunkStager16& stg, uint8_t* smem, const typename D::elem* __restrict__ G,
                                              const uint8_t* __restrict__ plan, PlanHeaderPtr H,
                                              float* __restrict__ T, int64_t i0, int nblk, int m, int n, int r,
                                              int tid, int lane, int wave) {
    const int nchunks = H->nchunks;
    const auto* seg = as_const<uint32_t>(plan + H->off_q_seg) + wave;
    const u32x4* rp0 = reinterpret_cast<const u32x4*>(plan + H->off_q_rows) + (size_t)(H->q_stream_row[wave] >> 1) * kWave + lane;
    const u32x4* rp = rp0;
    const uint32_t mycol = as_const<uint16_t>(plan + H->off_q_vcol)[tid];
    const bool shared = H->q_any_shared != 0;
    const uint16_t* __restrict__ perm = reinterpret_cast<const uint16_t*>(plan + H->off_q_perm) + tid;
    const uint32_t first = perm[0];
    uint32_t walked = first;                                          // virtual column whose list this thread walks

    // ring of kPrefetch batches of plan rows in fixed register slots (see gq_one_slot)
    u32x4 ring[kPrefetch][kBatchLoads];
    auto ring_restart = [&]() {
        rp = rp0;
#pragma unroll
        for (int k = 0; k < kPrefetch; ++k)
#pragma unroll
            for (int q = 0; q < kBatchLoads; ++q) ring[k][q] = rp[(size_t)(k * kBatchLoads + q) * kWave];
        rp += (size_t)kPrefetch * kBatchLoads * kWave;
    };
    ring_restart();

    float acc[1][kRowsGQ];
#pragma unroll
    for (int t = 0; t < kRowsGQ; ++t) acc[0][t] = 0.0f;

    const uint8_t* buf = smem;
    auto step = [&](u32x4 (&slot)[kBatchLoads]) {
        u32x4 x[2][2][kPlanes16];
        gather_pair16(buf, slot[0], x[0]);
#pragma unroll
        for (int q = 0; q < kBatchLoads; ++q) {
            if (q + 1 < kBatchLoads) gather_pair16(buf, slot[q + 1], x[(q + 1) & 1]);
            __builtin_amdgcn_sched_barrier(0);
            fma_pair16<D>(slot[q], x[q & 1], acc[0]);
            __builtin_amdgcn_sched_barrier(0);
        }
#pragma unroll
        for (int q = 0; q < kBatchLoads; ++q) slot[q] = rp[(size_t)q * kWave];
        rp += (size_t)kBatchLoads * kWave;
    };

    stg.stage(smem, 0, tid);                                          // chunk 0 of the first block (fetched by the caller)
    __syncthreads();
    int rot = 0, c = 0, blk = 0;
    const int units = nblk * nchunks;                                 // (row block, chunk) pairs, in order
    for (int u = 0; u < units; ++u) {
        if (rot != 0) {                                               // undo the slot rotation left by the previous chunk
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
        const bool last_chunk = c + 1 == nchunks;
        const uint32_t next = last_chunk ? (uint32_t)tid : (uint32_t)perm[(size_t)(c + 1) * kThreadsGQ];
        if (u + 1 < units)                                            // next chunk, maybe of the next block: lands while this one is consumed
            stg.fetch(G, i0 + (int64_t)(last_chunk ? blk + 1 : blk) * kRowsGQ, m, n, last_chunk ? 0 : c + 1, tid);
        buf = smem + (u & 1) * kBufStride16;
        const bool more = u + 1 < units;
        // The next chunk is staged (into the buffer nobody reads now) in the middle of this one's
        // work rather than at its end, where every wave would wait for it; only a block's last
        // chunk with shared columns stages later, behind the merge that uses the same LDS.
        const bool stage_early = more && !(last_chunk && shared);
        const int nb = (int)(seg[c * kWavesGQ] / kSegBatch);
        const int groups = nb / kPrefetch, before = groups < 2 ? groups : 2;
        for (int g = before; g > 0; --g) {
            step(ring[0]); step(ring[1]); step(ring[2]); step(ring[3]);
        }
        if (stage_early) stg.stage(smem, (u + 1) & 1, tid);
        for (int g = groups - before; g > 0; --g) {
            step(ring[0]); step(ring[1]); step(ring[2]); step(ring[3]);
        }
        rot = nb % kPrefetch;
        if (rot > 0) step(ring[0]);
        if (rot > 1) step(ring[1]);
        if (rot > 2) step(ring[2]);
        // The sums move to the lanes that walk the columns in the next chunk; after the last chunk
        // of a block they go home (thread t: virtual column t) and out to T.
        if (last_chunk && more) { ring_restart(); rot = 0; }          // the stream starts over; in flight during the stores
        swap_owner(smem + (u & 1) * kBufStride16, acc[0], walked, next);
        if (last_chunk) {
            const int64_t ib = i0 + (int64_t)blk * kRowsGQ;
            if (shared) {
                write_tile_shared<1>(smem, plan, H, T, acc, 1, ib, m, r, tid);   // uses the LDS of the first chunk buffer
                if (more) {
                    __syncthreads();                                  // before that LDS is staged into again
                    stg.stage(smem, (u + 1) & 1, tid);
                    __syncthreads();
                }
            } else if (mycol != kNoColumn) {
#pragma unroll
                for (int t = 0; t < kRowsGQ; ++t)
                    if (ib + t < m) T[(ib + t) * (int64_t)r + mycol] = acc[0][t];
            }
        }
        if (last_chunk) {                                             // the block's sums are out
#pragma unroll
            for (int t = 0; t < kRowsGQ; ++t) acc[0][t] = 0.0f;
            c = 0; ++blk;
            walked = first;
        } else {
            ++c;
            walked = next;
        }
    }
}

// Several columns per lane (r > 512, or columns used so unevenly that they were split), 16-bit
// storage: the same staging, plan ring and block walk as gq16_one_slot, the lane's columns taken
// slot by slot inside each chunk.  A lane keeps its columns for all chunks (no dealing by length:
// the sums of NS columns per lane would not fit through LDS cheaply).
template <typename D, int NS>
__device__ __forceinline__ void gq16_multi_slot(ChunkStager16& stg, uint8_t* smem, const typename D::elem* __restrict__ G,
                                                const uint8_t* __restrict__ plan, PlanHeaderPtr H,
                                                float* __restrict__ T, int64_t i0, int nblk, int m, int n, int r,
                                                int tid, int lane, int wave) {
    const int nchunks = H->nchunks, nslots = H->nslots;
    const auto* seg = as_const<uint32_t>(plan + H->off_q_seg) + wave;
    const u32x4* rp0 = reinterpret_cast<const u32x4*>(plan + H->off_q_rows) + (size_t)(H->q_stream_row[wave] >> 1) * kWave + lane;
    const u32x4* rp = rp0;
    const auto* vcol = as_const<uint16_t>(plan + H->off_q_vcol);
    const bool shared = H->q_any_shared != 0;

    u32x4 ring[kPrefetch][kBatchLoads];                               // fixed register slots (see gq_one_slot)
    auto ring_restart = [&]() {
        rp = rp0;
#pragma unroll
        for (int k = 0; k < kPrefetch; ++k)
#pragma unroll
            for (int q = 0; q < kBatchLoads; ++q) ring[k][q] = rp[(size_t)(k * kBatchLoads + q) * kWave];
        rp += (size_t)kPrefetch * kBatchLoads * kWave;
    };
    ring_restart();

    float acc[NS][kRowsGQ];
#pragma unroll
    for (int s = 0; s < NS; ++s)
#pragma unroll
        for (int t = 0; t < kRowsGQ; ++t) acc[s][t] = 0.0f;

    const uint8_t* buf = smem;
    auto step = [&](u32x4 (&slot)[kBatchLoads], float (&a)[kRowsGQ]) {
        u32x4 x[2][2][kPlanes16];
        gather_pair16(buf, slot[0], x[0]);
#pragma unroll
        for (int q = 0; q < kBatchLoads; ++q) {
            if (q + 1 < kBatchLoads) gather_pair16(buf, slot[q + 1], x[(q + 1) & 1]);
            __builtin_amdgcn_sched_barrier(0);
            fma_pair16<D>(slot[q], x[q & 1], a);
            __builtin_amdgcn_sched_barrier(0);
        }
#pragma unroll
        for (int q = 0; q < kBatchLoads; ++q) slot[q] = rp[(size_t)q * kWave];
        rp += (size_t)kBatchLoads * kWave;
    };
    static_assert(kPrefetch == 4, "the rotation below is written for four slots");
    auto unrotate = [&](int rot) {                                    // slot 0 holds the oldest batch again
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
    };

    stg.stage(smem, 0, tid);                                          // chunk 0 of the first block (fetched by the caller)
    __syncthreads();
    int rot = 0, c = 0, blk = 0;
    const int units = nblk * nchunks;
    for (int u = 0; u < units; ++u) {
        const bool last_chunk = c + 1 == nchunks;
        const bool more = u + 1 < units;
        if (more)
            stg.fetch(G, i0 + (int64_t)(last_chunk ? blk + 1 : blk) * kRowsGQ, m, n, last_chunk ? 0 : c + 1, tid);
        buf = smem + (u & 1) * kBufStride16;
#pragma unroll
        for (int s = 0; s < NS; ++s) {
            if (s < nslots) {
                unrotate(rot);
                const int nb = (int)(seg[(c * nslots + s) * kWavesGQ] / kSegBatch);
                for (int g = nb / kPrefetch; g > 0; --g) {
                    step(ring[0], acc[s]); step(ring[1], acc[s]); step(ring[2], acc[s]); step(ring[3], acc[s]);
                }
                rot = nb % kPrefetch;
                if (rot > 0) step(ring[0], acc[s]);
                if (rot > 1) step(ring[1], acc[s]);
                if (rot > 2) step(ring[2], acc[s]);
            }
        }
        if (last_chunk) {                                             // the block's 16 sums per column are complete
            const int64_t ib = i0 + (int64_t)blk * kRowsGQ;
            if (more) { ring_restart(); rot = 0; }                    // the stream starts over; in flight during the stores
            if (shared) {
                write_tile_shared<NS>(smem, plan, H, T, acc, nslots, ib, m, r, tid);   // uses the LDS of both chunk buffers
                if (more) {
                    __syncthreads();                                  // before that LDS is staged into again
                    if (tid < kPlanes) *reinterpret_cast<f32x4*>(smem + tid * kPlaneStride + kChunk * 16) = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
                }
            } else {
#pragma unroll
                for (int s = 0; s < NS; ++s) {
                    const uint32_t col = s < nslots ? (uint32_t)vcol[s * kThreadsGQ + tid] : kNoColumn;
                    if (col != kNoColumn) {
#pragma unroll
                        for (int t = 0; t < kRowsGQ; ++t)
                            if (ib + t < m) T[(ib + t) * (int64_t)r + col] = acc[s][t];
                    }
                }
            }
#pragma unroll
            for (int s = 0; s < NS; ++s)
#pragma unroll
                for (int t = 0; t < kRowsGQ; ++t) acc[s][t] = 0.0f;
            c = 0; ++blk;
        } else {
            ++c;
        }
        if (more) stg.stage(smem, (u + 1) & 1, tid);                  // the other buffer: nobody reads it now
        __syncthreads();                                              // the next chunk is staged; this one is no longer read
    }
}

// Kernel A for fp16 / bf16 with n % 8 == 0.
template <typename D>
__global__ __launch_bounds__(kThreadsGQ) void k_compress_gq16(const CompressGroup grp, int r, int d, int blocks_per_wg) {
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
    const int64_t i0 = (int64_t)block * blocks_per_wg * kRowsGQ;
    const int nblk = min(blocks_per_wg, (int)((m - i0 + kRowsGQ - 1) / kRowsGQ));   // row blocks of this workgroup

    PlanHeaderPtr H = as_const<PlanHeader>(plan);
    if (!plan_matches(H, m, n, r, d)) {                               // not a plan for this problem
        poison_s(S, r, block, nblocks, tid, kThreadsGQ);
        return;
    }
    if (H->p_any_split) {
        const int64_t total = (int64_t)r * r;
        for (int64_t k = (int64_t)block * kThreadsGQ + tid; k < total; k += (int64_t)nblocks * kThreadsGQ) S[k] = 0.0f;
    }
    if (tid < kPlanes) *reinterpret_cast<f32x4*>(smem + tid * kPlaneStride + kChunk * 16) = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
    ChunkStager16 stg;
    stg.fetch(G, i0, m, n, 0, tid);
    if (H->nslots == 1)      gq16_one_slot<D>(stg, smem, G, plan, H, T, i0, nblk, m, n, r, tid, lane, wave);
    else if (H->nslots == 2) gq16_multi_slot<D, 2>(stg, smem, G, plan, H, T, i0, nblk, m, n, r, tid, lane, wave);
    else                     gq16_multi_slot<D, kMaxSlots>(stg, smem, G, plan, H, T, i0, nblk, m, n, r, tid, lane, wave);
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
    int64_t blocks = 0;
    for (int p = 0; p < g.count; ++p) blocks += (g.m[p] + kRowsGQ - 1) / kRowsGQ;
    return blocks >= 1024 ? 2 : 1;
}

template <typename D>
static hipError_t launch_gq(const CompressGroup& g, int32_t r, int32_t d, int blocks_per_wg, hipStream_t st) {
    constexpr size_t lds = (size_t)kPlanes * kPlaneStride;   // >= 64 r bytes for every supported r
    const bool vec = (g.n[0] % 8) == 0;
    const unsigned grid = (unsigned)g.first_gq[g.count];
    hipError_t e;
    if constexpr (D::size == 2) {
        if (vec) {
            if ((e = allow_dynamic_lds<k_compress_gq16<D>>(lds)) != hipSuccess) return e;
            hipLaunchKernelGGL(k_compress_gq16<D>, dim3(grid), dim3(kThreadsGQ), lds, st, g, (int)r, (int)d, blocks_per_wg);
            return hipGetLastError();
        }
    }
    if (vec) {
        if ((e = allow_dynamic_lds<k_compress_gq<D, true>>(lds)) != hipSuccess) return e;
        hipLaunchKernelGGL((k_compress_gq<D, true>), dim3(grid), dim3(kThreadsGQ), lds, st, g, (int)r, (int)d);
    } else {
        if ((e = allow_dynamic_lds<k_compress_gq<D, false>>(lds)) != hipSuccess) return e;
        hipLaunchKernelGGL((k_compress_gq<D, false>), dim3(grid), dim3(kThreadsGQ), lds, st, g, (int)r, (int)d);
    }
    return hipGetLastError();
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
    const int bpw = gq_blocks_per_wg(g, dtype);
    g.first_gq[0] = g.first_pt[0] = 0;
    for (int p = 0; p < g.count; ++p) {
        g.first_gq[p + 1] = g.first_gq[p] + (int32_t)(((g.m[p] + kRowsGQ - 1) / kRowsGQ + bpw - 1) / bpw);
        const int32_t items = (int32_t)plan_max_items(g.m[p], r, d);
        g.first_pt[p + 1] = g.first_pt[p] + (striped ? ((items + 3) / 4) * 8 : items * nstripes);
    }
    hipError_t e;
    switch (dtype) {
        case LSP_F32:  e = launch_gq<F32>(g, r, d, bpw, st); break;
        case LSP_F16:  e = launch_gq<F16>(g, r, d, bpw, st); break;
        default:       e = launch_gq<BF16>(g, r, d, bpw, st); break;
    }
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
