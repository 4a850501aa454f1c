// Compress, kernel A, 16-bit variant (fp16 / bf16 storage, rows of whole 8-element groups): the template
// code; compress_gq16_bf16.hip and compress_gq16_f16.hip instantiate it.  See compress.hip for the path as a whole.
#pragma once

#include "compress_common.h"

namespace lsp {

// ----------------------------------------------------------------------------------------------
// 16-bit storage types (fp16, bf16), n % 8 == 0: G is staged as it is stored, 8 rows to a 16-byte LDS
// unit ([plane of 8 rows][column][8 rows]), so one 128-bit gather serves eight rows, and the LDS holds two
// chunks, the one being consumed and the one being staged, with one barrier per chunk.  The elements are
// widened in registers when they are used (exact: a shift or mask for bf16, a conversion for fp16).
// RP = planes of 8 rows per workgroup.  With RP = 1 (8 rows, 64 KB of LDS, at most 128 registers per lane) two
// workgroups share a CU, four waves per SIMD: a single wave issues a vector instruction only every 5 to 6
// cycles, so a SIMD needs more than two resident waves to stay busy while some of them wait at a barrier.
template <typename D> __device__ __forceinline__ void widen2(uint32_t w, float& lo, float& hi);
template <> __device__ __forceinline__ void widen2<BF16>(uint32_t w, float& lo, float& hi) {
    lo = __uint_as_float(w << 16); hi = __uint_as_float(w & 0xFFFF0000u);
}
template <> __device__ __forceinline__ void widen2<F16>(uint32_t w, float& lo, float& hi) {
    typedef _Float16 h2 __attribute__((ext_vector_type(2)));
    h2 h; __builtin_memcpy(&h, &w, 4);
    lo = (float)h.x; hi = (float)h.y;
}

// Rows 2k and 2k+1 of two adjacent columns sit in the dwords a (row 2k) and b (row 2k+1); the unit
// of the even column takes their low halves, that of the odd column their high halves (one byte permute).
__device__ __forceinline__ uint32_t pair_rows(uint32_t a, uint32_t b, bool odd_column) {
    return __builtin_amdgcn_perm(b, a, odd_column ? 0x07060302u : 0x05040100u);
}

// Fetches and stages a chunk of 8 RP rows.  Rows past the matrix are read from its last row and columns
// past it from its first ones (always a valid address): what they hold is never used, as the plan
// has no entry for such a column and the sums of such a row are not stored.  The rows of a thread
// are the same for the whole wave, so the row addresses are scalar.
template <int RP> struct ChunkStager16;

// RP = 2: a thread fetches 8 rows x 8 columns (one 16-byte load per row)
template <> struct ChunkStager16<2> {
    u32x4 pre[8];                                                     // 8 rows x 8 columns, as stored

    template <typename E>
    __device__ __forceinline__ void fetch(const E* __restrict__ G, int64_t i0, int m, int n, int c, int tid, int wave) {
        const int plane = wave / (kWavesGQ / 2), oct = tid % (kChunk / 8);
        const uint32_t col0 = (uint32_t)c * kChunk + (uint32_t)oct * 8;
        const uint32_t byte0 = (col0 < (uint32_t)n ? col0 : 0u) * (uint32_t)sizeof(E);
        const int64_t first = i0 + plane * 8;                        // may lie past the matrix (second plane of a ragged block)
        const int64_t top = first < m ? first : (int64_t)m - 1;
        const int last = (int)(m - 1 - top < 7 ? m - 1 - top : 7);   // rows of this plane inside the matrix, less one
        const char* base = reinterpret_cast<const char*>(G + top * (int64_t)n) + byte0;
        const uint64_t stride = (uint64_t)n * sizeof(E);
#pragma unroll
        for (int t = 0; t < 8; ++t) {
            pre[t] = stream_load(reinterpret_cast<const u32x4*>(base));
            base += t < last ? stride : 0;
        }
    }
    // transposes the 8x8 block and writes its 8 units (column q: rows 0..7) into buffer `buf`
    __device__ __forceinline__ void stage(uint8_t* smem, int buf, int tid) {
        const int plane = tid / (kChunk / 8), oct = tid % (kChunk / 8);
        uint8_t* base = smem + buf * (2 * kPlaneStride) + plane * kPlaneStride + oct * 16;
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            u32x4 unit;
#pragma unroll
            for (int k = 0; k < 4; ++k) unit[k] = pair_rows(pre[2 * k][q >> 1], pre[2 * k + 1][q >> 1], q & 1);
            *reinterpret_cast<u32x4*>(base + q * (kChunk / 8) * 16) = unit;
        }
    }
};

// RP = 1: a thread fetches 8 rows x 4 columns (one 8-byte load per row): 512 threads cover the 2048 columns
template <> struct ChunkStager16<1> {
    u32x2 pre[8];

    template <typename E>
    __device__ __forceinline__ void fetch(const E* __restrict__ G, int64_t i0, int m, int n, int c, int tid, int) {
        const uint32_t col0 = (uint32_t)c * kChunk + (uint32_t)tid * 4;
        const uint32_t byte0 = (col0 < (uint32_t)n ? col0 : 0u) * (uint32_t)sizeof(E);   // n % 8 == 0
        const int last = (int)(m - 1 - i0 < 7 ? m - 1 - i0 : 7);     // rows of the block inside the matrix, less one (i0 < m)
        const char* base = reinterpret_cast<const char*>(G + i0 * (int64_t)n) + byte0;
        const uint64_t stride = (uint64_t)n * sizeof(E);
#pragma unroll
        for (int t = 0; t < 8; ++t) {
            pre[t] = stream_load(reinterpret_cast<const u32x2*>(base));
            base += t < last ? stride : 0;
        }
    }
    // transposes the 8x4 block and writes its 4 units (column q: rows 0..7) into buffer `buf`
    __device__ __forceinline__ void stage(uint8_t* smem, int buf, int tid) {
        // local column j = 4 tid + q sits at unit (j & 7) * (kChunk / 8) + (j >> 3)
        uint8_t* base = smem + buf * kPlaneStride + ((4 * (tid & 1)) * (kChunk / 8) + (tid >> 1)) * 16;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            u32x4 unit;
#pragma unroll
            for (int k = 0; k < 4; ++k) unit[k] = pair_rows(pre[2 * k][q >> 1], pre[2 * k + 1][q >> 1], q & 1);
            *reinterpret_cast<u32x4*>(base + q * (kChunk / 8) * 16) = unit;
        }
    }
};

template <int RP>
__device__ __forceinline__ void gather_pair16(const uint8_t* buf, const u32x4 e, u32x4 (&x)[2][RP]) {
#pragma unroll
    for (int h = 0; h < 2; ++h)
#pragma unroll
        for (int g = 0; g < RP; ++g)
            if constexpr (kNoGathers) x[h][g] = e;
            else if constexpr (kNoConflicts) {                        // inside the chunk only (the always-zero unit lies behind it)
                const uint32_t off = h ? e.z : e.x;
                x[h][g] = *reinterpret_cast<const u32x4*>(buf + (off < kChunk * 16u ? (off & ~0xF0u) | ((threadIdx.x & 15u) << 4) : off) + g * kPlaneStride);
            }
            else x[h][g] = *reinterpret_cast<const u32x4*>(buf + (h ? e.z : e.x) + g * kPlaneStride);
}
template <typename D, int RP>
__device__ __forceinline__ void fma_pair16(const u32x4 e, const u32x4 (&x)[2][RP], float (&acc)[8 * RP]) {
    if constexpr (kNoFmas) {
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
            for (int g = 0; g < RP; ++g) acc[g * 8 + h] = __uint_as_float(__float_as_uint(acc[g * 8 + h]) ^ x[h][g][0] ^ x[h][g][3]);
        return;
    }
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const float v = __uint_as_float(h ? e.w : e.y);
#pragma unroll
        for (int g = 0; g < RP; ++g)
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
template <typename D, int RP>
__device__ __forceinline__ void gq16_one_slot(ChunkStager16<RP>& stg, uint8_t* smem, const typename D::elem* __restrict__ G,
                                              const uint8_t* __restrict__ plan, PlanHeaderPtr H,
                                              float* __restrict__ T, int64_t i0, int nblk, int m, int n, int r,
                                              int tid, int lane, int wave) {
    constexpr int R = 8 * RP;                                         // rows of a row block
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

    float acc[1][R];
#pragma unroll
    for (int t = 0; t < R; ++t) acc[0][t] = 0.0f;

    const uint8_t* buf = smem;
    auto step = [&](u32x4 (&slot)[kBatchLoads]) {
        u32x4 x[2][2][RP];
        gather_pair16<RP>(buf, slot[0], x[0]);
#pragma unroll
        for (int q = 0; q < kBatchLoads; ++q) {
            if (q + 1 < kBatchLoads) gather_pair16<RP>(buf, slot[q + 1], x[(q + 1) & 1]);
            __builtin_amdgcn_sched_barrier(0);
            fma_pair16<D, RP>(slot[q], x[q & 1], acc[0]);
            __builtin_amdgcn_sched_barrier(0);
        }
        if constexpr (kNoStream) {
#pragma unroll
            for (int q = 0; q < kBatchLoads; ++q) { slot[q].x = (slot[q].x + 272u) & 0x7FF0u; slot[q].z = (slot[q].z + 528u) & 0x7FF0u; }
        } else {
#pragma unroll
            for (int q = 0; q < kBatchLoads; ++q) slot[q] = rp[(size_t)q * kWave];
            rp += (size_t)kBatchLoads * kWave;
        }
    };

    PhaseClock clk;                                                   // empty unless built for phase timing
    stg.stage(smem, 0, tid);                                          // chunk 0 of the first block (fetched by the caller)
    __syncthreads();
    clk.tick(kPhFirstStage);
    // Batch k of a chunk sits in ring slot (rot + k) % kPrefetch, where rot is what the chunks before left over:
    // the walk enters the unrolled slot sequence at slot rot instead of moving the ring's registers.
    static_assert(kPrefetch == 4, "the slot walk below is written for four slots");
    int rot = 0, c = 0, blk = 0;
    const int units = nblk * nchunks;                                 // (row block, chunk) pairs, in order
    int nb_next = (int)(seg[0] / kSegBatch);                          // batches of this wave in the coming chunk
    for (int u = 0; u < units; ++u) {
        const bool last_chunk = c + 1 == nchunks;
        const uint32_t next = last_chunk ? (uint32_t)tid : (uint32_t)perm[(size_t)(c + 1) * kThreadsGQ];
        const int nb = kNoBatches ? 0 : nb_next;
        nb_next = (int)(seg[(last_chunk ? 0 : c + 1) * kWavesGQ] / kSegBatch);   // arrives while this chunk is walked
        clk.tick(kPhTop);
        if (u + 1 < units)                                            // next chunk, maybe of the next block: lands while this one is consumed
            stg.fetch(G, i0 + (int64_t)(last_chunk ? blk + 1 : blk) * R, m, n, last_chunk ? 0 : c + 1, tid, wave);
        buf = smem + (u & 1) * (RP * kPlaneStride);
        const bool more = u + 1 < units;
        // The next chunk is staged (into the buffer nobody reads now) in the middle of this one's
        // work rather than at its end, where every wave would wait for it; only a block's last
        // chunk with shared columns stages later, behind the merge that uses the same LDS.
        const bool stage_early = more && !(last_chunk && shared);
        int left = nb;
        clk.tick(kPhFetch);
        switch (rot) {                                                // up to the ring's slot 0
            case 1: if (left > 0) { step(ring[1]); --left; } [[fallthrough]];
            case 2: if (left > 0) { step(ring[2]); --left; } [[fallthrough]];
            case 3: if (left > 0) { step(ring[3]); --left; } [[fallthrough]];
            default: break;
        }
        const int groups = left / kPrefetch, before = groups < 2 ? groups : 2;
        for (int g = before; g > 0; --g) {
            step(ring[0]); step(ring[1]); step(ring[2]); step(ring[3]);
        }
        clk.tick(kPhFirst);
        if (stage_early && !kNoStaging) stg.stage(smem, (u + 1) & 1, tid);
        clk.tick(kPhStage);
        for (int g = groups - before; g > 0; --g) {
            step(ring[0]); step(ring[1]); step(ring[2]); step(ring[3]);
        }
        left -= groups * kPrefetch;
        if (left > 0) step(ring[0]);
        if (left > 1) step(ring[1]);
        if (left > 2) step(ring[2]);
        rot = (rot + nb) % kPrefetch;
        clk.tick(kPhRest);
        clk.count(kPhNFirst, (unsigned)(4 * before)); clk.count(kPhNRest, (unsigned)(nb - 4 * before)); clk.count(kPhBatches, (unsigned)nb);
        // The sums move to the lanes that walk the columns in the next chunk; after the last chunk
        // of a block they go home (thread t: virtual column t) and out to T.
        if (last_chunk && more) { ring_restart(); rot = 0; }          // the stream starts over; in flight during the stores
        if constexpr (kNoExchange) __syncthreads();
        else swap_owner<R>(smem + (u & 1) * (RP * kPlaneStride), acc[0], walked, next);
        clk.tick(kPhSwap);
        if (last_chunk) {
            const int64_t ib = i0 + (int64_t)blk * R;
            if (shared) {
                write_tile_shared<1, R>(smem, plan, H, T, acc, 1, ib, m, r, tid);   // uses the LDS of the first chunk buffer
                if (more) {
                    __syncthreads();                                  // before that LDS is staged into again
                    stg.stage(smem, (u + 1) & 1, tid);
                    __syncthreads();
                }
            } else if (mycol != kNoColumn) {
                if constexpr (kNoTStore) {
                    if (acc[0][0] == 123.456f) T[0] = acc[0][1] + acc[0][2] + acc[0][3] + acc[0][4] + acc[0][5] + acc[0][6] + acc[0][7];
                } else {
#pragma unroll
                    for (int t = 0; t < R; ++t)
                        if (ib + t < m) T[(ib + t) * (int64_t)r + mycol] = acc[0][t];
                }
            }
        }
        if (last_chunk) {                                             // the block's sums are out
#pragma unroll
            for (int t = 0; t < R; ++t) acc[0][t] = 0.0f;
            c = 0; ++blk;
            walked = first;
        } else {
            ++c;
            walked = next;
        }
    }
    clk.store(wave, lane);
}

// Several columns per lane (r > 512, or columns used so unevenly that they were split), 16-bit
// storage: the same staging, plan ring and block walk as gq16_one_slot, the lane's columns taken
// slot by slot inside each chunk.  A lane keeps its columns for all chunks (no dealing by length:
// the sums of NS columns per lane would not fit through LDS cheaply).
template <typename D, int NS, int RP>
__device__ __forceinline__ void gq16_multi_slot(ChunkStager16<RP>& stg, uint8_t* smem, const typename D::elem* __restrict__ G,
                                                const uint8_t* __restrict__ plan, PlanHeaderPtr H,
                                                float* __restrict__ T, int64_t i0, int nblk, int m, int n, int r,
                                                int tid, int lane, int wave) {
    constexpr int R = 8 * RP;                                         // rows of a row block
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

    float acc[NS][R];
#pragma unroll
    for (int s = 0; s < NS; ++s)
#pragma unroll
        for (int t = 0; t < R; ++t) acc[s][t] = 0.0f;

    const uint8_t* buf = smem;
    auto step = [&](u32x4 (&slot)[kBatchLoads], float (&a)[R]) {
        u32x4 x[2][2][RP];
        gather_pair16<RP>(buf, slot[0], x[0]);
#pragma unroll
        for (int q = 0; q < kBatchLoads; ++q) {
            if (q + 1 < kBatchLoads) gather_pair16<RP>(buf, slot[q + 1], x[(q + 1) & 1]);
            __builtin_amdgcn_sched_barrier(0);
            fma_pair16<D, RP>(slot[q], x[q & 1], a);
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
            stg.fetch(G, i0 + (int64_t)(last_chunk ? blk + 1 : blk) * R, m, n, last_chunk ? 0 : c + 1, tid, wave);
        buf = smem + (u & 1) * (RP * kPlaneStride);
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
            const int64_t ib = i0 + (int64_t)blk * R;
            if (more) { ring_restart(); rot = 0; }                    // the stream starts over; in flight during the stores
            if (shared) {
                write_tile_shared<NS, R>(smem, plan, H, T, acc, nslots, ib, m, r, tid);   // uses the LDS of both chunk buffers
                if (more) {
                    __syncthreads();                                  // before that LDS is staged into again
                    if (tid < 2 * RP) *reinterpret_cast<f32x4*>(smem + tid * kPlaneStride + kChunk * 16) = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
                }
            } else {
#pragma unroll
                for (int s = 0; s < NS; ++s) {
                    const uint32_t col = s < nslots ? (uint32_t)vcol[s * kThreadsGQ + tid] : kNoColumn;
                    if (col != kNoColumn) {
#pragma unroll
                        for (int t = 0; t < R; ++t)
                            if (ib + t < m) T[(ib + t) * (int64_t)r + col] = acc[s][t];
                    }
                }
            }
#pragma unroll
            for (int s = 0; s < NS; ++s)
#pragma unroll
                for (int t = 0; t < R; ++t) acc[s][t] = 0.0f;
            c = 0; ++blk;
        } else {
            ++c;
        }
        if (more) stg.stage(smem, (u + 1) & 1, tid);                  // the other buffer: nobody reads it now
        __syncthreads();                                              // the next chunk is staged; this one is no longer read
    }
}

// Kernel A for fp16 / bf16 with n % 8 == 0: R = 8 RP rows per row block.
template <typename D, int RP>
__global__ __launch_bounds__(kThreadsGQ, RP == 1 ? 4 : 1) void k_compress_gq16(const CompressGroup grp, int r, int d, int blocks_per_wg) {
    constexpr int R = 8 * RP;
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
    const int64_t i0 = (int64_t)block * blocks_per_wg * R;
    const int nblk = min(blocks_per_wg, (int)((m - i0 + R - 1) / R));   // row blocks of this workgroup

    ChunkStager16<RP> stg;
    stg.fetch(G, i0, m, n, 0, tid, wave);                             // in flight while the plan's header arrives
    PlanHeaderPtr H = as_const<PlanHeader>(plan);
    if (!plan_matches(H, m, n, r, d)) {                               // not a plan for this problem
        poison_s(S, r, block, nblocks, tid, kThreadsGQ);
        return;
    }
    if (H->p_any_split) {
        const int64_t total = (int64_t)r * r;
        for (int64_t k = (int64_t)block * kThreadsGQ + tid; k < total; k += (int64_t)nblocks * kThreadsGQ) S[k] = 0.0f;
    }
    if (tid < 2 * RP) *reinterpret_cast<f32x4*>(smem + tid * kPlaneStride + kChunk * 16) = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
    if (H->nslots == 1)      gq16_one_slot<D, RP>(stg, smem, G, plan, H, T, i0, nblk, m, n, r, tid, lane, wave);
    else if (H->nslots == 2) gq16_multi_slot<D, 2, RP>(stg, smem, G, plan, H, T, i0, nblk, m, n, r, tid, lane, wave);
    else                     gq16_multi_slot<D, kMaxSlots, RP>(stg, smem, G, plan, H, T, i0, nblk, m, n, r, tid, lane, wave);
}


template <typename D>
static hipError_t launch_gq16(const CompressGroup& g, int32_t r, int32_t d, int blocks_per_wg, hipStream_t st) {
    constexpr int RP = kRowsGQ16 / 8;
    constexpr size_t lds = (size_t)2 * RP * kPlaneStride;    // two chunk buffers of RP 8-row planes
    hipError_t e;
    if ((e = allow_dynamic_lds<k_compress_gq16<D, RP>>(lds)) != hipSuccess) return e;
    hipLaunchKernelGGL((k_compress_gq16<D, RP>), dim3((unsigned)g.first_gq[g.count]), dim3(kThreadsGQ), lds, st, g, (int)r, (int)d, blocks_per_wg);
    return hipGetLastError();
}

}  // namespace lsp
