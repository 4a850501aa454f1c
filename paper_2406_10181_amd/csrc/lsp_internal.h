// Internal declarations shared by the translation units of the HIP library (not installed).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include <atomic>

#include "lsp.h"

namespace lsp {

// ------------------------------------------------------------------------------------------
// Tiling constants of the compress kernels (the plan layout depends on them).
// ------------------------------------------------------------------------------------------
constexpr int kChunk      = 2048;  // columns of G staged in LDS at a time
constexpr int kWave       = 64;    // gfx950 wavefront
constexpr int kThreadsGQ  = 512;   // threads of the T = G Q kernel: one lane per (virtual) column of T
constexpr int kWavesGQ    = kThreadsGQ / kWave;
constexpr int kMaxSlots   = 4;     // a lane owns at most this many virtual columns
constexpr int kSegBatch   = 4;     // segment lengths are multiples of this many rows
constexpr int kPrefetch   = 4;     // batches of plan rows a wave holds in registers (one consumed, the rest in flight)
constexpr int kStreamSlack = kPrefetch * kSegBatch;   // readable padding rows after the last segment
constexpr int kRowPiece   = 256;   // a row list of P^T longer than this is cut into pieces
constexpr uint32_t kNoColumn = 0xFFFFu;      // virtual column slot without a column
constexpr uint32_t kSharedColumn = 0x8000u;  // flag: the column is owned by several lanes

static inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// Development aid: -DLSP_ABLATE=<bits> builds a library in which pieces of the two hot kernels are left out, to see
// what each costs (build.py --ablations, ablation.py).  Such a library computes WRONG results by design and is
// never loaded by the binding; the normal build has LSP_ABLATE = 0 and all of these are false.
#ifndef LSP_ABLATE
#define LSP_ABLATE 0
#endif
constexpr bool kNoExchange  = (LSP_ABLATE & 0x001) != 0;   // kernel A: the sums stay with their lanes between chunks (one barrier instead)
constexpr bool kNoStaging   = (LSP_ABLATE & 0x002) != 0;   // kernel A: no chunk is written to LDS (nor fetched: the loads are dead)
constexpr bool kNoBatches   = (LSP_ABLATE & 0x004) != 0;   // kernel A: no plan row is walked
constexpr bool kNoGathers   = (LSP_ABLATE & 0x008) != 0;   // kernel A: the plan entry itself stands in for the gathered unit
constexpr bool kNoFmas      = (LSP_ABLATE & 0x010) != 0;   // kernel A: one exclusive-or per gathered unit instead of 16 + 16 instructions
constexpr bool kNoStream    = (LSP_ABLATE & 0x020) != 0;   // kernel A: the plan ring is never refilled (stale entries, scrambled)
constexpr bool kNoConflicts = (LSP_ABLATE & 0x040) != 0;   // both: lane k of every 16 gathers from bank quad k
constexpr bool kNoTStore    = (LSP_ABLATE & 0x080) != 0;   // kernel A: T is not stored
constexpr bool kNoApplyMath = (LSP_ABLATE & 0x100) != 0;   // apply kernel: no gathers of U, no FMAs
constexpr bool kNoApplyQ    = (LSP_ABLATE & 0x200) != 0;   // apply kernel: the rows of Q are made up, not loaded
constexpr bool kNoApplyU    = (LSP_ABLATE & 0x400) != 0;   // apply kernel: U = P S is not built

// Remembers the raw HIP error for lsp_last_hip_error() and returns LSP_ERR_LAUNCH.
int note_hip_error(hipError_t e);

// LDS byte offset, inside one 4-row plane, of local column j of a staged chunk.
// Columns are stored as [j & 7][j >> 3] in units of 16 bytes (4 rows x fp32), so that the 64
// lanes of a staging wave, which hold 8 consecutive columns each, write consecutive units.
__host__ __device__ static inline uint32_t chunk_col_offset(uint32_t j) {
    return (((j & 7u) * (kChunk / 8)) + (j >> 3)) * 16u;
}

// ------------------------------------------------------------------------------------------
// Plan: column-sorted projector copies, laid out for the compress kernels.
// All offsets are bytes from the start of the plan buffer and multiples of 16.
//
// Q part.  Every column b of T = G Q is owned by one lane of the 512-thread workgroup, which keeps
// the column's partial sums in registers.  A column whose list of (column j of
// G, value) pairs is longer than list_cap inside some chunk gets several owners ("virtual
// columns"), each taking an equal share of the list in every chunk; the owners' sums are added at
// the end, in a fixed order.  Lanes left over (r < 512) are given to the columns with the longest
// shares, so that all lanes of the workgroup carry about the same load.  Virtual column v sits in
// slot v / 512, lane v % 512 -- except that with one slot (q_permuted) the lane that walks a
// column's list changes from chunk to chunk: inside each chunk the 512 lists are dealt to the waves
// by length, longest first (a wave is as slow as its longest list, so lists of like length go
// together; the two waves that share a SIMD get a long and a short group), and the kernel hands
// the partial sums from lane to lane between chunks.  q_perm[c][t] is the virtual column that
// thread t walks in chunk c.  For each (chunk, slot, wave) the
// 64 lists are padded to a common length (a multiple of kSegBatch) with pairs that point at an
// always-zero LDS unit, and stored lane-interleaved two rows at a time: rows 2p and 2p+1 form
// 64 x (LDS offset, value bits, LDS offset, value bits), one 128-bit load per lane.
// The rows of one wave are contiguous over all chunks and slots (chunk-major), so a wave reads
// one linear stream.
// ------------------------------------------------------------------------------------------
struct PlanHeader {            // first 256 bytes of the plan buffer
    uint32_t magic;            // kPlanMagic
    int32_t  m, n, r, d;
    int32_t  nchunks;          // ceil(n / kChunk)
    int32_t  nslots;           // virtual columns per lane (1 .. kMaxSlots)
    int32_t  nvcols;           // virtual columns in use
    int32_t  q_total_rows;     // rows of all wave streams, slack included
    int32_t  p_nitems;         // pieces of rows of P^T
    int32_t  p_any_split;      // 1 if some row of P^T was cut (S must start at zero)
    int32_t  list_cap;         // longest list a lane walks in one chunk
    uint32_t q_stream_row[kWavesGQ];   // first row of each wave's stream
    int32_t  q_any_shared;     // 1 if some column of T has several owners
    int32_t  q_permuted;       // 1 if the owner of a virtual column changes per chunk (q_perm; one slot only)
    uint32_t pad[2];
    // section offsets
    uint64_t off_q_seg;        // uint32[nchunks][nslots][kWavesGQ]  rows of each segment
    uint64_t off_q_vcol;       // uint16[nslots * 512]               column b (| kSharedColumn) or kNoColumn
    uint64_t off_q_rows;       // uint4[q_total_rows / 2][64]
    uint64_t off_p_item;       // RowItem[p_nitems]
    uint64_t off_p_ent;        // uint2[m*d]                         (row i, value bits)
    uint64_t total_bytes;
    uint64_t off_q_vcnt;       // uint16[nslots * 512]               owners of the column if this is its first owner, else 0
    uint64_t off_q_perm;       // uint16[nchunks][512]               virtual column walked by thread t in chunk c
    // where every stored value came from, so that new values can be dropped into an existing plan when only
    // the values of the projectors change (lsp_plan_refresh_values): flat ELL positions row * d + k
    uint64_t off_q_src;        // uint32[q_total_rows][64], laid out like q_rows; kNoSource for padding pairs
    uint64_t off_p_src;        // uint32[m*d], parallel to p_ent
    uint64_t pad2[2];
};
static_assert(sizeof(PlanHeader) == 192, "PlanHeader layout");
constexpr uint32_t kPlanMagic = 0x4C535038u;   // "LSP8"
constexpr uint32_t kNoSource = 0xFFFFFFFFu;    // q_src of a padding pair
constexpr size_t   kPlanHeaderBytes = 256;

struct RowItem   { int32_t a; int32_t start; int32_t len; int32_t atomic; };

// Copy of an ELL projector with the entries of each row ordered against LDS bank conflicts in the
// decompress kernels (host arrays; the matrix itself is unchanged).
int reorder_rows_host(const int32_t* idx, const float* val, int64_t rows, int32_t d, int32_t r,
                      int32_t* idx_out, float* val_out);

// Byte offsets of the plan's sections (they depend on the shape only).
struct PlanLayout { size_t off_q_seg, off_q_vcol, off_q_vcnt, off_q_perm, off_q_rows, off_p_item, off_p_ent, off_q_src, off_p_src, total; };
PlanLayout plan_layout(int64_t m, int64_t n, int32_t r, int32_t d);

// Upper bounds (depend on shapes only) used to size the plan buffer.
int    plan_list_cap(int32_t r, int32_t d);
size_t plan_max_rows(int64_t n, int32_t r, int32_t d);
size_t plan_max_items(int64_t m, int32_t r, int32_t d);
size_t plan_bytes(int64_t m, int64_t n, int32_t r, int32_t d);

// Host-side builder: fills `host_plan` (plan_bytes() bytes) from host copies of the ELL arrays.
// Returns LSP_OK, or LSP_ERR_SKEW when the columns of Q are so unevenly used that more than
// kMaxSlots * 512 virtual columns would be needed.
int build_plan_host(const int32_t* P_idx, const float* P_val, const int32_t* Q_idx, const float* Q_val,
                    int64_t m, int64_t n, int32_t r, int32_t d, uint8_t* host_plan);

// ------------------------------------------------------------------------------------------
// Groups: several independent problems (same r, d, dtype) served by one launch per kernel, so that
// workgroups of different matrices fill the CUs together.  Passed to the kernels by value.
// first[p] .. first[p+1] are the workgroups of problem p.
// ------------------------------------------------------------------------------------------
constexpr int kMaxGroup = LSP_MAX_GROUP;
struct CompressGroup {
    const void*    G[kMaxGroup];
    const uint8_t* plan[kMaxGroup];
    float*         T[kMaxGroup];
    float*         S[kMaxGroup];
    int32_t        m[kMaxGroup], n[kMaxGroup];
    int32_t        first_gq[kMaxGroup + 1];      // workgroups of the T = G Q kernel
    int32_t        first_pt[kMaxGroup + 1];      // workgroups of the S = P^T T kernel
    int32_t        count;
};
struct ApplyGroup {
    void*          W[kMaxGroup];
    const float*   S[kMaxGroup];
    const int32_t* P_idx[kMaxGroup];
    const float*   P_val[kMaxGroup];
    const int32_t* Q_idx[kMaxGroup];
    const float*   Q_val[kMaxGroup];
    int32_t        m[kMaxGroup], n[kMaxGroup];
    int32_t        first[kMaxGroup + 1];
    int32_t        count;
};

#if defined(__HIPCC__)
// The problem that owns workgroup `block`, picked with compile-time indices only: indexing the
// by-value group with a run-time index would make the compiler copy it to scratch memory and turn
// every address derived from it into a per-lane (vector) value, so that the small uniform loads of
// the kernels (plan header, segment table) would go through the vector memory path and wait for
// all the data loads in flight.  Everything returned is wave-uniform and lives in scalar registers.
struct CompressProblem { const void* G; const uint8_t* plan; float* T; float* S; int32_t m, n, block_gq, nblocks_gq, block_pt; };
__device__ __forceinline__ CompressProblem group_pick(const CompressGroup& g, int block, bool kernel_b) {
    CompressProblem o{g.G[0], g.plan[0], g.T[0], g.S[0], g.m[0], g.n[0], block, g.first_gq[1], block};
#pragma unroll
    for (int p = 1; p < kMaxGroup; ++p) {
        const bool hit = p < g.count && block >= (kernel_b ? g.first_pt[p] : g.first_gq[p]);
        if (hit) {
            o.G = g.G[p]; o.plan = g.plan[p]; o.T = g.T[p]; o.S = g.S[p]; o.m = g.m[p]; o.n = g.n[p];
            o.block_gq = block - g.first_gq[p]; o.nblocks_gq = g.first_gq[p + 1] - g.first_gq[p];
            o.block_pt = block - g.first_pt[p];
        }
    }
    return o;
}
// index of the problem that owns workgroup `block` (uniform; count <= kMaxGroup); the decompress
// kernels use this run-time index: they have no small uniform loads to protect, and measured faster
__device__ __forceinline__ int group_find(const int32_t* first, int count, int block) {
    int p = 0;
    while (p + 1 < count && block >= first[p + 1]) ++p;
    return p;
}
#endif

// ------------------------------------------------------------------------------------------
// Kernel launchers (each returns hipSuccess or the launch error).  The group launchers fill in
// first_* themselves; all problems of a group must agree on what selects the kernel variant
// (see compress_group_uniform / apply_group_uniform).
// ------------------------------------------------------------------------------------------
bool       compress_group_uniform(const CompressGroup& g);
bool       apply_group_uniform(const ApplyGroup& g, int32_t r, int32_t d);
hipError_t launch_compress_planned(CompressGroup& g, int32_t r, int32_t d, lsp_dtype dtype, hipStream_t st);
// Scatter form on raw ELL arrays.  gate (device, may be null): the kernels run only if *gate == LSP_ERR_SKEW.
hipError_t launch_compress_raw(const void* G, const int32_t* P_idx, const float* P_val,
                               const int32_t* Q_idx, const float* Q_val,
                               int64_t m, int64_t n, int32_t r, int32_t d,
                               float* S, lsp_dtype dtype, float* T, const int32_t* gate, hipStream_t st);
hipError_t launch_decompress(ApplyGroup& g, int32_t r, int32_t d, lsp_dtype dtype, hipStream_t st);
// Dense-projector ablation of compress on the matrix cores (dense.hip): Pt = P^T [r][m], Qt = Q^T [r][n] in the
// storage type of G (fp16 / bf16); workspace of dense_workspace_bytes(m, r); shapes must pass dense_shape_ok.
bool       dense_shape_ok(int64_t m, int64_t n, int32_t r);
size_t     dense_workspace_bytes(int64_t m, int32_t r);
hipError_t launch_compress_dense(const void* G, const void* Pt, const void* Qt, int64_t m, int64_t n, int32_t r, float* S,
                                 uint8_t* workspace, lsp_dtype dtype, hipStream_t st);
// Estimation bias (Def. 2): `partial` holds bias_blocks(m, r) pairs of floats, `out` three floats.
int64_t    bias_blocks(int64_t m, int32_t r);
hipError_t launch_bias(ApplyGroup& g, int32_t r, int32_t d, lsp_dtype dtype, float* partial, float* out, hipStream_t st);
// Optimiser-state re-projection (MaybeUpdate, Alg. 1): workspace holds 3 r^2 floats; V may be null.
hipError_t launch_reproject(const int32_t* P_idx, const float* P_val, const int32_t* Pp_idx, const float* Pp_val,
                            const int32_t* Q_idx, const float* Q_val, const int32_t* Qp_idx, const float* Qp_val,
                            int64_t m, int64_t n, int32_t r, int32_t d, float* M, float* V, float* workspace,
                            hipStream_t st);
hipError_t launch_validate(const int32_t* idx, int64_t count, int32_t r, int32_t* flag, hipStream_t st);
// Values-only refresh of a plan (same indices, new values).
hipError_t launch_plan_refresh(uint8_t* plan, const float* P_val, const float* Q_val,
                               int64_t m, int64_t n, int32_t r, int32_t d, hipStream_t st);
// Device-side plan build (plan_device.hip): the bytes of build_plan_host, from kernels on `st`; workspace of
// plan_build_workspace_bytes(); status_out (device, may be null) receives LSP_OK / LSP_ERR_INDEX / LSP_ERR_SKEW.
size_t     plan_build_workspace_bytes(int64_t m, int64_t n, int32_t r, int32_t d);
hipError_t launch_plan_build(const int32_t* P_idx, const float* P_val, const int32_t* Q_idx, const float* Q_val,
                             int64_t m, int64_t n, int32_t r, int32_t d, uint8_t* plan, uint8_t* workspace,
                             int32_t* status_out, hipStream_t st);
// C = op(A) op(B) + beta E on r x r fp32 matrices (matrix cores): up to kMaxGemmBatch independent products of
// one size in a launch (no product may read what another of the same launch writes).  flags: transpose an
// operand (not both), square an operand element by element; E may be null.
constexpr int kMaxGemmBatch = 3;
constexpr int kGemmTA = 1, kGemmTB = 2, kGemmSqA = 4, kGemmSqB = 8;
struct GemmProblem { const float* A; const float* B; float* C; const float* E; float beta; int32_t flags; };
struct GemmBatch { GemmProblem p[kMaxGemmBatch]; };
hipError_t launch_gemm_rr_batch(const GemmBatch& batch, int count, int32_t r, hipStream_t st);
// C = L^T R (r x r, overwritten) for two ELL matrices with the same number of rows; one or two independent
// pairs per launch.
struct GramPair { const int32_t* L_idx; const float* L_val; const int32_t* R_idx; const float* R_val; int64_t rows; float* C; };
struct GramBatch { GramPair p[2]; };
hipError_t launch_gram(const GramBatch& batch, int count, int32_t d, int32_t r, hipStream_t st);
hipError_t launch_zero(float* p, int64_t count, hipStream_t st);
// Gradient of 1/2 ||P P^T G Q Q^T - G||_F^2 with respect to the stored projector values (fitgrad.hip).
size_t     fitgrad_workspace_floats(int64_t m, int64_t n, int32_t r, int32_t d);
hipError_t launch_fitgrad(const void* G, const uint8_t* plan, const int32_t* P_idx, const float* P_val,
                          const int32_t* Q_idx, const float* Q_val, int64_t m, int64_t n, int32_t r, int32_t d,
                          float* gP, float* gQ, float* workspace, lsp_dtype dtype, hipStream_t st);

// ------------------------------------------------------------------------------------------
// Storage types on the device.
// ------------------------------------------------------------------------------------------
struct F32 { using elem = float;    static constexpr int size = 4; };
struct F16 { using elem = uint16_t; static constexpr int size = 2; };
struct BF16{ using elem = uint16_t; static constexpr int size = 2; };

#if defined(__HIPCC__)
// Lets kernel `Kern` use up to `bytes` of dynamic LDS.  The attribute belongs to the (kernel, device)
// pair and does not change afterwards, so the runtime is asked once per pair, not on every launch of
// the per-step path.
template <auto Kern>
static inline hipError_t allow_dynamic_lds(size_t bytes) {
    static std::atomic<uint64_t> done{0};                   // bit k: set on device k (devices >= 64: always asked)
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 64 && ((done.load(std::memory_order_acquire) >> dev) & 1u)) return hipSuccess;
    e = hipFuncSetAttribute(reinterpret_cast<const void*>(Kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
    if (e == hipSuccess && dev < 64) done.fetch_or((uint64_t)1 << dev, std::memory_order_release);
    return e;
}

// Streaming accesses to the big matrices (each byte of G and W is touched once per call): marked
// non-temporal so that they do not evict the small, heavily re-read operands (S, the projector
// arrays, the plan) from the XCD's L2.
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
template <typename V> __device__ __forceinline__ V stream_load(const V* p) {
    static_assert(sizeof(V) == 4 || sizeof(V) == 8 || sizeof(V) == 16, "4, 8 or 16 bytes");
    V out;
    if constexpr (sizeof(V) == 4) { uint32_t t = __builtin_nontemporal_load(reinterpret_cast<const uint32_t*>(p)); __builtin_memcpy(&out, &t, 4); }
    else if constexpr (sizeof(V) == 8) { u32x2 t = __builtin_nontemporal_load(reinterpret_cast<const u32x2*>(p)); __builtin_memcpy(&out, &t, 8); }
    else { u32x4 t = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p)); __builtin_memcpy(&out, &t, 16); }
    return out;
}
template <typename V> __device__ __forceinline__ void stream_store(V* p, const V& v) {
    static_assert(sizeof(V) == 4 || sizeof(V) == 8 || sizeof(V) == 16, "4, 8 or 16 bytes");
    if constexpr (sizeof(V) == 4) { uint32_t t; __builtin_memcpy(&t, &v, 4); __builtin_nontemporal_store(t, reinterpret_cast<uint32_t*>(p)); }
    else if constexpr (sizeof(V) == 8) { u32x2 t; __builtin_memcpy(&t, &v, 8); __builtin_nontemporal_store(t, reinterpret_cast<u32x2*>(p)); }
    else { u32x4 t; __builtin_memcpy(&t, &v, 16); __builtin_nontemporal_store(t, reinterpret_cast<u32x4*>(p)); }
}

// Read-only tables of the plan (header, segment lengths, column tables) are read through the
// constant address space: the kernels never write the plan, and a uniform load from that address
// space is a scalar load, which does not share the counter (and the waits) of the vector loads
// that stream G and the plan rows.
#define LSP_CONST_AS __attribute__((address_space(4)))
template <typename T> __device__ __forceinline__ const LSP_CONST_AS T* as_const(const void* p) {
    return (const LSP_CONST_AS T*)(uintptr_t)p;
}
typedef const LSP_CONST_AS PlanHeader* PlanHeaderPtr;

template <typename D> __device__ __forceinline__ float widen(typename D::elem x);
template <> __device__ __forceinline__ float widen<F32>(float x) { return x; }
template <> __device__ __forceinline__ float widen<F16>(uint16_t x) {
    _Float16 h; __builtin_memcpy(&h, &x, 2); return (float)h;
}
template <> __device__ __forceinline__ float widen<BF16>(uint16_t x) {
    return __uint_as_float(((uint32_t)x) << 16);
}
template <typename D> __device__ __forceinline__ typename D::elem narrow(float x);
template <> __device__ __forceinline__ float narrow<F32>(float x) { return x; }
template <> __device__ __forceinline__ uint16_t narrow<F16>(float x) {
    _Float16 h = (_Float16)x; uint16_t u; __builtin_memcpy(&u, &h, 2); return u;   // nearest-even
}
template <> __device__ __forceinline__ uint16_t narrow<BF16>(float x) {
    __bf16 h = (__bf16)x; uint16_t u; __builtin_memcpy(&u, &h, 2); return u;       // nearest-even
}
#endif

}  // namespace lsp
