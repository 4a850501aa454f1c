// Internal declarations shared by the translation units of the HIP library (not installed).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "lsp.h"

namespace lsp {

// ------------------------------------------------------------------------------------------
// Tiling constants of the compress kernels (the plan layout depends on them).
// ------------------------------------------------------------------------------------------
constexpr int kChunk      = 1024;  // columns of G staged in LDS at a time
constexpr int kWave       = 64;    // gfx950 wavefront
constexpr int kListMax    = 64;    // a (chunk, column) list longer than this is cut into pieces
constexpr int kRowPiece   = 128;   // a row list of P^T longer than this is cut into pieces
constexpr uint32_t kNoColumn = 0xFFFFu;      // lane has no piece in this round
constexpr uint32_t kSharedColumn = 0x8000u;  // flag on a piece's column: the list was cut, several lanes add to it

static inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// LDS byte offset, inside one 4-row plane, of local column j of a staged chunk.
// Columns are stored as [j & 7][j >> 3] in units of 16 bytes (4 rows x fp32), so that the 64
// lanes of a staging wave, which hold 8 consecutive columns each, write consecutive units.
__host__ __device__ static inline uint32_t chunk_col_offset(uint32_t j) {
    return (((j & 7u) * (kChunk / 8)) + (j >> 3)) * 16u;
}

// ------------------------------------------------------------------------------------------
// Plan: column-sorted projector copies, laid out for the compress kernels.
// All offsets are bytes from the start of the plan buffer and multiples of 16.
// ------------------------------------------------------------------------------------------
struct PlanHeader {            // first 256 bytes of the plan buffer
    uint32_t magic;            // kPlanMagic
    int32_t  m, n, r, d;
    int32_t  nchunks;          // ceil(n / kChunk)
    int32_t  q_total_rounds;   // rounds over all chunks
    int32_t  p_nitems;         // pieces of rows of P^T
    int32_t  p_any_split;      // 1 if some row of P^T was cut (S must start at zero)
    uint32_t pad[7];
    // section offsets
    uint64_t off_q_chunk;      // ChunkInfo[nchunks]
    uint64_t off_q_round;      // RoundInfo[q_total_rounds]
    uint64_t off_q_cols;       // uint16[q_total_rounds][64]   column b of each lane's piece
    uint64_t off_q_ent;        // uint2[slots]                  (LDS offset, value bits)
    uint64_t off_p_item;       // RowItem[p_nitems]
    uint64_t off_p_ent;        // uint2[m*d]                    (row i, value bits)
    uint64_t total_bytes;
    uint64_t pad2[9];
};
static_assert(sizeof(PlanHeader) == 192, "PlanHeader layout");
constexpr uint32_t kPlanMagic = 0x4C535031u;   // "LSP1"
constexpr size_t   kPlanHeaderBytes = 256;

struct ChunkInfo { int32_t first_round; int32_t nrounds; };
struct RoundInfo { uint32_t ent_offset; int32_t len; };         // ent_offset in entries
struct RowItem   { int32_t a; int32_t start; int32_t len; int32_t atomic; };

// Upper bounds (depend on shapes only) used to size the plan buffer.
size_t plan_max_rounds(int64_t n, int32_t r, int32_t d);
size_t plan_max_slots(int64_t n, int32_t r, int32_t d);
size_t plan_max_items(int64_t m, int32_t r, int32_t d);
size_t plan_bytes(int64_t m, int64_t n, int32_t r, int32_t d);

// Host-side builder: fills `host_plan` (plan_bytes() bytes) from host copies of the ELL arrays.
void build_plan_host(const int32_t* P_idx, const float* P_val, const int32_t* Q_idx, const float* Q_val,
                     int64_t m, int64_t n, int32_t r, int32_t d, uint8_t* host_plan);

// ------------------------------------------------------------------------------------------
// Kernel launchers (each returns hipSuccess or the launch error).
// ------------------------------------------------------------------------------------------
hipError_t launch_compress_planned(const void* G, const uint8_t* plan, int64_t m, int64_t n, int32_t r, int32_t d,
                                   float* S, lsp_dtype dtype, float* T, hipStream_t st);
hipError_t launch_compress_raw(const void* G, const int32_t* P_idx, const float* P_val,
                               const int32_t* Q_idx, const float* Q_val,
                               int64_t m, int64_t n, int32_t r, int32_t d,
                               float* S, lsp_dtype dtype, float* T, hipStream_t st);
hipError_t launch_decompress(void* W, const float* S, const int32_t* P_idx, const float* P_val,
                             const int32_t* Q_idx, const float* Q_val,
                             int64_t m, int64_t n, int32_t r, int32_t d, lsp_dtype dtype, hipStream_t st);
hipError_t launch_validate(const int32_t* idx, int64_t count, int32_t r, int32_t* flag, hipStream_t st);

// ------------------------------------------------------------------------------------------
// Storage types on the device.
// ------------------------------------------------------------------------------------------
struct F32 { using elem = float;    static constexpr int size = 4; };
struct F16 { using elem = uint16_t; static constexpr int size = 2; };
struct BF16{ using elem = uint16_t; static constexpr int size = 2; };

#if defined(__HIPCC__)
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
