// Compress, kernel A, 16-bit variant (fp16 / bf16 storage, rows of whole 8-element groups): the template
// code; compress_gq16_bf16.hip and compress_gq16_f16.hip instantiate it.  See compress.hip for the path as a whole.
#pragma once

#include <cstdlib>

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
            x[h][g] = *reinterpret_cast<const u32x4*>(buf + (h ? e.z : e.x) + g * kPlaneStride);
}
template <typename D, int RP>
__device__ __forceinline__ void fma_pair16(const u32x4 e, const u32x4 (&x)[2][RP], float (&acc)[8 * RP]) {
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

// The launch has a fixed number of workgroups (two per CU) that stay until the group's work is done and take
// the row blocks of the group, one at a time and in group order, from a counter in device memory: a workgroup
// started anew pays for the launch, the plan header, its first chunk of G and the first plan rows with nothing
// to overlap them, a workgroup that goes on to its next row block overlaps all of that with the block before.
// (A fixed share of the blocks per workgroup instead of the counter leaves the CUs idle at the end: the two
// workgroups of a CU do not advance at the same speed.)  A group with no more row blocks than that is launched
// with one workgroup per row block and no counter.
//
// Per problem of the group, in LDS: what the kernel needs of it.  Thread 0 fills the table from the by-value
// group with compile-time indices; a problem is then picked with a run-time index from LDS (indexing the
// by-value group that way would make the compiler copy it to scratch memory, see group_pick).
struct ProblemTable {
    const void* G[kMaxGroup]; const uint8_t* plan[kMaxGroup]; float* T[kMaxGroup]; float* S[kMaxGroup];
    int32_t m[kMaxGroup], n[kMaxGroup], first[kMaxGroup + 1];         // first: row blocks of the group before this problem
    int32_t ticket[2];                                                // row blocks drawn ahead (see Tickets)
};
__device__ __forceinline__ void fill_table(const CompressGroup& g, ProblemTable* out) {
#pragma unroll
    for (int p = 0; p < kMaxGroup; ++p) {
        if (p < g.count) {
            out->G[p] = g.G[p]; out->plan[p] = g.plan[p]; out->T[p] = g.T[p]; out->S[p] = g.S[p];
            out->m[p] = g.m[p]; out->n[p] = g.n[p];
        }
        out->first[p] = g.first_gq[p < g.count ? p : g.count];
    }
    out->first[kMaxGroup] = g.first_gq[g.count];
}
template <typename X> __device__ __forceinline__ X* uniform_ptr(X* const* slot) {   // a pointer every lane reads from the same LDS slot
    const uint32_t* w = reinterpret_cast<const uint32_t*>(slot);
    const uint64_t v = (uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((int)w[0]) | ((uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((int)w[1]) << 32);
    // the table holds device-memory addresses: saying so keeps the loads and stores through them on the vector-memory
    // path of global memory (a pointer of unknown origin would be accessed with flat instructions, which tie the
    // LDS and the vector-memory counters together)
    typedef X __attribute__((address_space(1))) GX;
    return (X*)reinterpret_cast<GX*>(v);
}
__device__ __forceinline__ int uniform_int(const int32_t* slot) { return __builtin_amdgcn_readfirstlane(*slot); }
__device__ __forceinline__ int problem_of(const ProblemTable* t, int unit) {   // unit < first[kMaxGroup]
    int p = 0;
    while (unit >= uniform_int(&t->first[p + 1])) ++p;
    return p;
}

// The row blocks a workgroup works on: `cur` now, `nxt` after it (both indices into the group's row blocks; at
// or past `total`: none).  The one after `nxt` is drawn from the counter when a block is begun and read when
// it ends, so that the counter's latency stays hidden and the block after the current one is always known
// early enough to fetch its first chunk ahead.  One lane of the last wave draws (that wave walks short lists
// and has time to wait for the counter); the value passes through LDS, two slots in turn, with the barriers of
// the block in between.
struct Tickets {
    uint32_t* counter;                                                // null: one row block per workgroup, nothing to draw
    int32_t*  slot;
    int       cur, nxt, total, drawn;
    __device__ __forceinline__ void draw(int tid) {
        if (counter && tid == kThreadsGQ - kWave) slot[drawn & 1] = (int32_t)atomicAdd(counter, 1u);
    }
    __device__ __forceinline__ void advance() {                       // after a barrier that follows draw()
        cur = nxt;
        nxt = counter ? __builtin_amdgcn_readfirstlane(slot[drawn & 1]) : total;
        ++drawn;
    }
};

// Fetches the first chunk of the row block a workgroup goes on to when that block belongs to another problem.
template <typename E, int RP>
__device__ __forceinline__ void fetch_ahead(ChunkStager16<RP>& stg, const ProblemTable* tab, int unit, int tid, int wave) {
    const int q = problem_of(tab, unit);
    stg.fetch(static_cast<const E*>(uniform_ptr(&tab->G[q])), (int64_t)(unit - uniform_int(&tab->first[q])) * (8 * RP),
              uniform_int(&tab->m[q]), uniform_int(&tab->n[q]), 0, tid, wave);
}

// When some row of P^T is cut into pieces, kernel B adds into S, which therefore starts at zero; the row blocks
// of a problem share that work (block b of nblocks takes every nblocks-th run of 512 elements).
__device__ __forceinline__ void zero_share_of_s(float* __restrict__ S, int r, int block, int nblocks, int tid) {
    const int64_t total = (int64_t)r * r;
    for (int64_t k = (int64_t)block * kThreadsGQ + tid; k < total; k += (int64_t)nblocks * kThreadsGQ) S[k] = 0.0f;
}

// One workgroup walks row blocks of 8 RP rows, beginning in problem p (whose plan has one column per lane), for
// as long as its tickets name blocks of one-column plans: the first chunk of the next block is fetched and
// staged while the last chunk of the current one is consumed, the plan ring is refilled for it, and the
// stores of T go out under the next block's work, so that the set-up and the tail of a block cost nothing but
// for the first and the last one -- also when the next block belongs to the next problem of the group.  Chunk 0
// of the first block has been fetched by the caller; on return chunk 0 of the block tk.cur (if any) has been.
template <typename D, int RP>
__device__ __forceinline__ void gq16_one_slot(ChunkStager16<RP>& stg, uint8_t* smem, const ProblemTable* tab, int p, int r, int d,
                                              int tid, int lane, int wave, Tickets& tk, PhaseClock& clk) {
    typedef typename D::elem E;
    constexpr int R = 8 * RP;                                         // rows of a row block
    // the problem the walk is in
    const E* __restrict__ G; const uint8_t* __restrict__ plan; PlanHeaderPtr H; float* __restrict__ T; float* __restrict__ S;
    int m, n, first_p, end_p, nchunks; bool shared, split;
    const LSP_CONST_AS uint32_t* seg; const u32x4* rp0; const uint16_t* __restrict__ perm; uint32_t mycol, first;
    auto stream_start = [&](const uint8_t* pl, PlanHeaderPtr Hq) {
        return reinterpret_cast<const u32x4*>(pl + Hq->off_q_rows) + (size_t)(Hq->q_stream_row[wave] >> 1) * kWave + lane;
    };
    auto enter = [&](int q) {                                         // the plan of problem q has been checked
        G = static_cast<const E*>(uniform_ptr(&tab->G[q])); plan = uniform_ptr(&tab->plan[q]);
        T = uniform_ptr(&tab->T[q]); S = uniform_ptr(&tab->S[q]);
        m = uniform_int(&tab->m[q]); n = uniform_int(&tab->n[q]);
        first_p = uniform_int(&tab->first[q]); end_p = uniform_int(&tab->first[q + 1]);
        H = as_const<PlanHeader>(plan);
        nchunks = H->nchunks; shared = H->q_any_shared != 0; split = H->p_any_split != 0;
        seg = as_const<uint32_t>(plan + H->off_q_seg) + wave;
        rp0 = stream_start(plan, H);
        perm = reinterpret_cast<const uint16_t*>(plan + H->off_q_perm) + tid;
        mycol = as_const<uint16_t>(plan + H->off_q_vcol)[tid];
        first = perm[0];
    };
    enter(p);
    const u32x4* rp = rp0;
    uint32_t walked = first;                                          // virtual column whose list this thread walks

    // ring of kPrefetch batches of plan rows in fixed register slots (see gq_one_slot)
    u32x4 ring[kPrefetch][kBatchLoads];
    auto ring_restart = [&](const u32x4* from) {
        rp = from;
#pragma unroll
        for (int k = 0; k < kPrefetch; ++k)
#pragma unroll
            for (int q = 0; q < kBatchLoads; ++q) ring[k][q] = rp[(size_t)(k * kBatchLoads + q) * kWave];
        rp += (size_t)kPrefetch * kBatchLoads * kWave;
    };
    ring_restart(rp0);

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
#pragma unroll
        for (int q = 0; q < kBatchLoads; ++q) slot[q] = rp[(size_t)q * kWave];
        rp += (size_t)kBatchLoads * kWave;
    };

    clk.resume();
    stg.stage(smem, 0, tid);                                          // chunk 0 of the first block (fetched by the caller)
    __syncthreads();
    clk.tick(kPhFirstStage);
    // Batch k of a chunk sits in ring slot (rot + k) % kPrefetch, where rot is what the chunks before left over:
    // the walk enters the unrolled slot sequence at slot rot instead of moving the ring's registers.
    static_assert(kPrefetch == 4, "the slot walk below is written for four slots");
    int rot = 0, c = 0;
    int64_t ib = (int64_t)(tk.cur - first_p) * R;                     // first row of the block
    int nb_next = (int)(seg[0] / kSegBatch);                          // batches of this wave in the coming chunk
    for (int u = 0; ; ++u) {                                          // (row block, chunk) pairs, in order
        if (c == 0) {
            tk.draw(tid);
            if (split) zero_share_of_s(S, r, (int)(ib / R), end_p - first_p, tid);
        }
        const bool last_chunk = c + 1 == nchunks;
        const bool more_here = tk.nxt < end_p;                        // the block after this one belongs to this problem too
        const bool leaving = last_chunk && !more_here && tk.nxt < tk.total;   // ... or to the next problem
        const uint32_t next = last_chunk ? (uint32_t)tid : (uint32_t)perm[(size_t)(c + 1) * kThreadsGQ];
        const int nb = nb_next;
        if (!last_chunk || more_here)
            nb_next = (int)(seg[(last_chunk ? 0 : c + 1) * kWavesGQ] / kSegBatch);   // arrives while this chunk is walked
        clk.tick(kPhTop);
        int q = p; PlanHeaderPtr Hq = H;                              // the problem of the next block
        if (!last_chunk) {                                            // the next chunk lands while this one is consumed
            stg.fetch(G, ib, m, n, c + 1, tid, wave);
        } else if (more_here) {
            stg.fetch(G, (int64_t)(tk.nxt - first_p) * R, m, n, 0, tid, wave);
        } else if (leaving) {
            q = problem_of(tab, tk.nxt);
            stg.fetch(static_cast<const E*>(uniform_ptr(&tab->G[q])), (int64_t)(tk.nxt - uniform_int(&tab->first[q])) * R,
                      uniform_int(&tab->m[q]), uniform_int(&tab->n[q]), 0, tid, wave);
            Hq = as_const<PlanHeader>(uniform_ptr(&tab->plan[q]));
        }
        buf = smem + (u & 1) * (RP * kPlaneStride);
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
        // does the walk go on into the next problem?  (its header has had the first batches to arrive)
        const bool chain = leaving && plan_matches(Hq, uniform_int(&tab->m[q]), uniform_int(&tab->n[q]), r, d) && Hq->nslots == 1;
        const bool more = !last_chunk || more_here || chain;
        // The next chunk is staged (into the buffer nobody reads now) in the middle of this one's
        // work rather than at its end, where every wave would wait for it; only a block's last
        // chunk with shared columns stages later, behind the merge that uses the same LDS.
        const bool stage_early = more && !(last_chunk && shared);
        if (stage_early) stg.stage(smem, (u + 1) & 1, tid);
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
        if (last_chunk && more) {                                     // the stream starts over (that of the next problem, maybe); in flight during the stores
            ring_restart(chain ? stream_start(uniform_ptr(&tab->plan[q]), Hq) : rp0);
            rot = 0;
        }
        swap_owner<R>(smem + (u & 1) * (RP * kPlaneStride), acc[0], walked, next);
        clk.tick(kPhSwap);
        if (last_chunk) {
            if (shared) {
                write_tile_shared<1, R>(smem, plan, H, T, acc, 1, ib, m, r, tid);   // uses the LDS of the first chunk buffer
                if (more) {
                    __syncthreads();                                  // before that LDS is staged into again
                    stg.stage(smem, (u + 1) & 1, tid);
                    __syncthreads();
                }
            } else if (mycol != kNoColumn) {
#pragma unroll
                for (int t = 0; t < R; ++t)
                    if (ib + t < m) T[(ib + t) * (int64_t)r + mycol] = acc[0][t];
            }
        }
        if (last_chunk) {                                             // the block's sums are out
            tk.advance();
            if (!more) break;
            if (chain) {
                p = q;
                enter(p);
                nb_next = (int)(seg[0] / kSegBatch);
            }
#pragma unroll
            for (int t = 0; t < R; ++t) acc[0][t] = 0.0f;
            c = 0; ib = (int64_t)(tk.cur - first_p) * R;
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
template <typename D, int NS, int RP>
__device__ __forceinline__ void gq16_multi_slot(ChunkStager16<RP>& stg, uint8_t* smem, const typename D::elem* __restrict__ G,
                                                const uint8_t* __restrict__ plan, PlanHeaderPtr H,
                                                float* __restrict__ T, float* __restrict__ S, int m, int n, int r,
                                                int tid, int lane, int wave, Tickets& tk, int first_p, int end_p, const ProblemTable* tab) {
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
    int rot = 0, c = 0;
    int64_t ib = (int64_t)(tk.cur - first_p) * R;                     // first row of the block
    for (int u = 0; ; ++u) {                                          // (row block, chunk) pairs, in order
        if (c == 0) {
            tk.draw(tid);
            if (H->p_any_split) zero_share_of_s(S, r, (int)(ib / R), end_p - first_p, tid);
        }
        const bool last_chunk = c + 1 == nchunks;
        const bool more_here = tk.nxt < end_p;                        // the block after this one belongs to this problem too
        const bool more = !last_chunk || more_here;
        if (!last_chunk)
            stg.fetch(G, ib, m, n, c + 1, tid, wave);
        else if (more_here)
            stg.fetch(G, (int64_t)(tk.nxt - first_p) * R, m, n, 0, tid, wave);
        else if (tk.nxt < tk.total)
            fetch_ahead<typename D::elem, RP>(stg, tab, tk.nxt, tid, wave);
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
        if (last_chunk) {                                             // the block's sums per column are complete
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
            c = 0;
        } else {
            ++c;
        }
        if (more) stg.stage(smem, (u + 1) & 1, tid);                  // the other buffer: nobody reads it now
        __syncthreads();                                              // the next chunk is staged; this one is no longer read
        if (last_chunk) {
            tk.advance();
            if (!more_here) break;
            ib = (int64_t)(tk.cur - first_p) * R;
        }
    }
}

// Kernel A for fp16 / bf16 with n % 8 == 0: R = 8 RP rows per row block.  `counter` (device memory, zero at the
// start of the launch) is null when the launch has one workgroup per row block.
template <typename D, int RP>
__global__ __launch_bounds__(kThreadsGQ, RP == 1 ? 4 : 1) void k_compress_gq16(const CompressGroup grp, int r, int d, uint32_t* counter) {
    constexpr int R = 8 * RP;
    typedef typename D::elem E;
    extern __shared__ __align__(16) uint8_t smem[];
    ProblemTable* tab = reinterpret_cast<ProblemTable*>(smem + 2 * RP * kPlaneStride);
    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    if (tid == 0) fill_table(grp, tab);
    if (tid == kThreadsGQ - kWave) tab->ticket[0] = counter ? (int32_t)atomicAdd(counter, 2u) : (int32_t)blockIdx.x;
    if (tid < 2 * RP) *reinterpret_cast<f32x4*>(smem + tid * kPlaneStride + kChunk * 16) = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
    __syncthreads();
    Tickets tk;
    tk.counter = counter; tk.slot = tab->ticket; tk.total = grp.first_gq[grp.count]; tk.drawn = 1;
    tk.cur = __builtin_amdgcn_readfirstlane(tab->ticket[0]);          // a workgroup's first two row blocks lie side by side
    tk.nxt = counter ? tk.cur + 1 : tk.total;
    if (tk.cur >= tk.total) return;
    PhaseClock clk;                                                   // empty unless built for phase timing
    ChunkStager16<RP> stg;
    fetch_ahead<E, RP>(stg, tab, tk.cur, tid, wave);                  // in flight while the plan's header arrives
    for (bool first = true; tk.cur < tk.total; first = false) {
        const int p = problem_of(tab, tk.cur);
        const E* __restrict__ G = static_cast<const E*>(uniform_ptr(&tab->G[p]));
        const uint8_t* __restrict__ plan = uniform_ptr(&tab->plan[p]);
        float* __restrict__ T = uniform_ptr(&tab->T[p]);
        float* __restrict__ S = uniform_ptr(&tab->S[p]);
        const int m = uniform_int(&tab->m[p]), n = uniform_int(&tab->n[p]);
        const int first_p = uniform_int(&tab->first[p]), end_p = uniform_int(&tab->first[p + 1]);
        if (!first) __syncthreads();                                  // the LDS of the problem before is no longer read
        PlanHeaderPtr H = as_const<PlanHeader>(plan);
        if (!plan_matches(H, m, n, r, d)) {                           // not a plan for this problem: its row blocks only mark S
            while (tk.cur < end_p) {
                tk.draw(tid);
                poison_s(S, r, tk.cur - first_p, end_p - first_p, tid, kThreadsGQ);
                __syncthreads();
                tk.advance();
            }
            if (tk.cur < tk.total) fetch_ahead<E, RP>(stg, tab, tk.cur, tid, wave);
        }
        else if (H->nslots == 1) gq16_one_slot<D, RP>(stg, smem, tab, p, r, d, tid, lane, wave, tk, clk);
        else if (H->nslots == 2) gq16_multi_slot<D, 2, RP>(stg, smem, G, plan, H, T, S, m, n, r, tid, lane, wave, tk, first_p, end_p, tab);
        else                     gq16_multi_slot<D, kMaxSlots, RP>(stg, smem, G, plan, H, T, S, m, n, r, tid, lane, wave, tk, first_p, end_p, tab);
    }
    clk.store(wave, lane);
}

template <typename D> __global__ void k_zero_counter(uint32_t* counter) { if (threadIdx.x < 2) counter[threadIdx.x] = 0u; }

// workgroups that stay on the device together: two per CU (what the LDS of a CU holds)
static int gq16_resident_workgroups() {
    constexpr int kMaxDevices = 64;
    static std::atomic<int> cus[kMaxDevices];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return 512;
    int v = cus[dev].load(std::memory_order_relaxed);
    if (v == 0) {
        if (hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || v <= 0) v = 256;
        cus[dev].store(v, std::memory_order_relaxed);
    }
    return 2 * v;
}

template <typename D>
static hipError_t launch_gq16(const CompressGroup& g, int32_t r, int32_t d, uint32_t* counter, hipStream_t st) {
    constexpr int RP = kRowsGQ16 / 8;
    constexpr size_t lds = (size_t)2 * RP * kPlaneStride + sizeof(ProblemTable);   // two chunk buffers of RP 8-row planes, the table
    hipError_t e;
    if ((e = allow_dynamic_lds<k_compress_gq16<D, RP>>(lds)) != hipSuccess) return e;
    static const int expmode = getenv("LSP_EXP") ? atoi(getenv("LSP_EXP")) : 0;
    const int total = g.first_gq[g.count], resident = expmode == 1 ? (1 << 30) : expmode > 1 ? expmode : gq16_resident_workgroups();
    if (total <= resident) {
        hipLaunchKernelGGL((k_compress_gq16<D, RP>), dim3((unsigned)total), dim3(kThreadsGQ), lds, st, g, (int)r, (int)d, (uint32_t*)nullptr);
        return hipGetLastError();
    }
    hipLaunchKernelGGL(k_zero_counter<D>, dim3(1), dim3(64), 0, st, counter);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    hipLaunchKernelGGL((k_compress_gq16<D, RP>), dim3((unsigned)resident), dim3(kThreadsGQ), lds, st, g, (int)r, (int)d, counter);
    return hipGetLastError();
}

}  // namespace lsp
