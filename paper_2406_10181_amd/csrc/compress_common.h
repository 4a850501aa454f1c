// Pieces shared by the translation units of the compress path (kernel A in its 16-bit and its
// fp32-staged variants, kernel B and the launchers).
#pragma once

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


// Kernel A: one workgroup = 16 rows of G, 512 threads, one lane per (virtual) column of T.
constexpr int kPlanes = 4;                                    // 4-row planes of an fp32-staged chunk
constexpr int kRowsGQ = 4 * kPlanes;
constexpr int kBatchLoads = kSegBatch / 2;                    // 128-bit loads per batch of plan rows

// Partial sums of several owners of one column meet in LDS: every lane parks its 16 sums at its
// virtual column, [16][nslots * 512] floats; the first owner of a column then adds the owners'
// sums in owner order (they sit side by side) and stores the column of T.  No atomics, so the
// result does not depend on timing.  Called by all threads of the workgroup.
template <int NS, int R = kRowsGQ>
__device__ __forceinline__ void write_tile_shared(uint8_t* smem, const uint8_t* plan, PlanHeaderPtr H, float* __restrict__ T,
                                                  const float (&acc)[NS][R], int nslots, int64_t i0, int m, int r, int tid) {
    __syncthreads();                                                  // the staged chunk is no longer read
    float* Tl = reinterpret_cast<float*>(smem);
    const int V = nslots * kThreadsGQ;
    const auto* vcol = as_const<uint16_t>(plan + H->off_q_vcol);
    const auto* vcnt = as_const<uint16_t>(plan + H->off_q_vcnt);
#pragma unroll
    for (int s = 0; s < NS; ++s) {
        if (s < nslots) {
#pragma unroll
            for (int t = 0; t < R; ++t) Tl[t * V + s * kThreadsGQ + tid] = acc[s][t];
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
                for (int t = 0; t < R; ++t) {
                    float sum = Tl[t * V + v];
                    for (int o = 1; o < owners; ++o) sum += Tl[t * V + v + o];
                    if (i0 + t < m) T[(i0 + t) * (int64_t)r + bb] = sum;
                }
            }
        }
    }
}

// Hands the R partial sums of every virtual column from the lane that walked its list in one
// chunk to the lane that walks it in the next (`from`, `to`: virtual columns of this thread; the
// plan deals the lists of each chunk to the waves by length).  They pass through the first 2 R KB
// of `area`, the LDS of the chunk consumed last: the first barrier makes sure nobody reads that
// chunk any more (and publishes whatever was written to other LDS before the call), the last one
// that the area may be staged into again.  Called by all threads.
template <int R>
__device__ __forceinline__ void swap_owner(uint8_t* area, float (&acc)[R], uint32_t from, uint32_t to) {
    f32x4* X = reinterpret_cast<f32x4*>(area);
    __syncthreads();
#pragma unroll
    for (int q = 0; q < R / 4; ++q)
        X[q * kThreadsGQ + from] = f32x4{acc[4 * q], acc[4 * q + 1], acc[4 * q + 2], acc[4 * q + 3]};   // lanes spread over all banks
    __syncthreads();
#pragma unroll
    for (int q = 0; q < R / 4; ++q) {
        const f32x4 a = X[q * kThreadsGQ + to];
        acc[4 * q] = a[0]; acc[4 * q + 1] = a[1]; acc[4 * q + 2] = a[2]; acc[4 * q + 3] = a[3];
    }
    __syncthreads();
}


// Development aid, compiled in only with -DLSP_PHASE_TIMING (build.py --phase-timing builds such a library beside the
// normal one; phase_timing.py reads it out): the one-column walker of the 16-bit kernel A adds up, per wave, the core
// clock cycles it spends in each phase of a chunk and leaves them in a device array.
#ifdef LSP_PHASE_TIMING
constexpr int kPhaseSlots = 16;                               // per wave: 12 phase sums, cycles, start, wall clock, spare
constexpr int kPhaseMaxWG = 8192;
static __device__ unsigned long long g_phase[kPhaseMaxWG * kWavesGQ * kPhaseSlots];   // one copy per translation unit
struct PhaseClock {
    unsigned long long sum[12] = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
    unsigned long long last, begin, wall;
    __device__ __forceinline__ PhaseClock() { last = begin = clock64(); wall = wall_clock64(); }
    __device__ __forceinline__ void tick(int phase) { const unsigned long long now = clock64(); sum[phase] += now - last; last = now; }
    __device__ __forceinline__ void count(int slot, unsigned long long k) { sum[slot] += k; }
    __device__ __forceinline__ void store(int wave, int lane) {
        if (lane != 0 || blockIdx.x >= kPhaseMaxWG) return;
        unsigned long long* o = g_phase + ((size_t)blockIdx.x * kWavesGQ + wave) * kPhaseSlots;
        for (int k = 0; k < 12; ++k) o[k] = sum[k];
        o[12] = clock64() - begin; o[13] = begin; o[14] = wall_clock64() - wall; o[15] = wall;
    }
};
#else
struct PhaseClock {
    __device__ __forceinline__ void tick(int) {}
    __device__ __forceinline__ void count(int, unsigned long long) {}
    __device__ __forceinline__ void store(int, int) {}
};
#endif
// phases of a chunk in gq16_one_slot: staging of the block's first chunk, top of the chunk loop, fetch of the next
// chunk and segment length, the batches before the staging, staging, the remaining batches, exchange of the sums;
// slots 5, 7, 8 count batches
enum : int { kPhFirstStage = 0, kPhTop = 1, kPhFetch = 2, kPhFirst = 3, kPhStage = 4, kPhBatches = 5, kPhRest = 6, kPhNFirst = 7,
             kPhNRest = 8, kPhSwap = 9 };

// Launchers of kernel A (first_gq filled in): fp16 / bf16 with rows of whole 8-element groups, and the rest.
// rows of G per row block of the 16-bit kernel (a workgroup holds that many rows of two chunks in LDS)
constexpr int kRowsGQ16 = 8;
hipError_t launch_gq16_bf16(const CompressGroup& g, int32_t r, int32_t d, int blocks_per_wg, hipStream_t st);
hipError_t launch_gq16_f16(const CompressGroup& g, int32_t r, int32_t d, int blocks_per_wg, hipStream_t st);
hipError_t launch_gq_staged32(const CompressGroup& g, int32_t r, int32_t d, lsp_dtype dtype, hipStream_t st);

}  // namespace lsp
