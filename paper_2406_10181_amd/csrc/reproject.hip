// Optimiser-state re-projection (MaybeUpdate in Alg. 1, its last two assignments): when the
// projectors of a matrix are replaced, the subspace moments follow,
//     M <- (P^T P_prev) M (Q_prev^T Q),      V <- (P^T P_prev)^2 V (Q_prev^T Q)^2,
// the squares taken element by element.  Two steps:
//   1. A = P^T P_prev and B = Q_prev^T Q, r x r: products of two ELL matrices with the same rows;
//      row i adds its d x d products val * val' at (idx, idx'), with fp32 atomics in LDS on a block
//      of rows of the result that a workgroup owns.
//   2. four dense r x r products in fp32 on the matrix cores (v_mfma_f32_32x32x2_f32): X = A M,
//      X2 = (A o A) V, then M = X B, V = X2 (B o B); the squares are taken while the tiles are staged,
//      and the two independent products of each stage share a launch.
// Runs once per change of projectors; nothing here is on the per-step path.
#include <algorithm>

#include "lsp_internal.h"

namespace lsp {

typedef float f32x16 __attribute__((ext_vector_type(16)));

// C = L^T R for two ELL matrices with the same rows: C[L_idx[i][k]][R_idx[i][k']] += L_val[i][k] * R_val[i][k'].
// Global fp32 atomics are slow here (they go past the per-XCD L2), so a workgroup owns a block of rows of C
// in LDS.  It scans the column index of every entry (i, k) of L and queues, in LDS, those that fall in its
// block; then one thread per (queued entry, k') adds the product with an LDS atomic; then the block is
// written (C needs no clearing).  Scanning and adding are separate so that neither is a chain of dependent
// loads.  An entry that finds the queue full is added by the thread that found it (correct, slow: only
// heavily skewed projectors get there).  blockIdx.y picks one of two independent pairs.  Entries with an
// index outside [0, r) are skipped.  The order of the LDS additions varies: results can differ in the last
// bits from run to run.
constexpr int kGramThreads = 1024, kGramAccFloats = 12288, kGramQueue = 4096, kGramInFlight = 8;
__global__ __launch_bounds__(kGramThreads) void k_gram(const GramBatch batch, int d, int r, int block_rows) {
    __shared__ float acc[kGramAccFloats];
    __shared__ int queue[kGramQueue];
    __shared__ int queued;
    GramPair P = batch.p[0];
    if (blockIdx.y == 1) P = batch.p[1];
    const int a0 = blockIdx.x * block_rows, a1 = min(r, a0 + block_rows);
    const int mine = (a1 - a0) * r;
    const int lane = threadIdx.x & 63;
    for (int q = threadIdx.x; q < mine; q += kGramThreads) acc[q] = 0.0f;
    if (threadIdx.x == 0) queued = 0;
    __syncthreads();
    auto add_entry = [&](int t, int a, int k2) {
        const float v = P.L_val[t];
        const int row = t / d * d;
        const int b = P.R_idx[row + k2];
        const float x = P.R_val[row + k2];
        if (v != 0.0f && (unsigned)b < (unsigned)r) atomicAdd(&acc[(a - a0) * r + b], v * x);
    };
    const int total = (int)(P.rows * d);                            // < 2^31, checked by the host
    for (int t0 = 0; t0 < total; t0 += kGramThreads * kGramInFlight) {       // uniform trip count: the ballots need whole waves
        int a[kGramInFlight];
#pragma unroll
        for (int u = 0; u < kGramInFlight; ++u) {
            const int t = t0 + u * kGramThreads + (int)threadIdx.x;
            a[u] = t < total ? P.L_idx[t] : -1;
        }
#pragma unroll
        for (int u = 0; u < kGramInFlight; ++u) {
            const bool hit = a[u] >= a0 && a[u] < a1;
            const uint64_t mask = __ballot(hit);
            if (mask == 0) continue;
            int base = 0;
            if (lane == __ffsll((long long)mask) - 1) base = atomicAdd(&queued, __popcll(mask));
            base = __shfl(base, __ffsll((long long)mask) - 1);
            if (hit) {
                const int t = t0 + u * kGramThreads + (int)threadIdx.x;
                const int slot = base + __popcll(mask & ((1ull << lane) - 1));
                if (slot < kGramQueue) queue[slot] = t;
                else
                    for (int k2 = 0; k2 < d; ++k2) add_entry(t, a[u], k2);
            }
        }
    }
    __syncthreads();
    const int work = min(queued, kGramQueue) * d;
    for (int w0 = threadIdx.x; w0 < work; w0 += kGramThreads * kGramInFlight) {
        // every load of a batch is issued before the first addition: otherwise each item waits for its own
        int t[kGramInFlight], a[kGramInFlight], b[kGramInFlight];
        float v[kGramInFlight], x[kGramInFlight];
#pragma unroll
        for (int u = 0; u < kGramInFlight; ++u) {
            const int w = w0 + u * kGramThreads;
            t[u] = w < work ? queue[w / d] : -1;
        }
#pragma unroll
        for (int u = 0; u < kGramInFlight; ++u) {
            const int tt = max(t[u], 0), k2 = (w0 + u * kGramThreads) % d;
            a[u] = P.L_idx[tt];
            v[u] = P.L_val[tt];
            b[u] = P.R_idx[tt / d * d + k2];
            x[u] = P.R_val[tt / d * d + k2];
        }
#pragma unroll
        for (int u = 0; u < kGramInFlight; ++u)
            if (t[u] >= 0 && v[u] != 0.0f && (unsigned)b[u] < (unsigned)r) atomicAdd(&acc[(a[u] - a0) * r + b[u]], v[u] * x[u]);
    }
    __syncthreads();
    for (int q = threadIdx.x; q < mine; q += kGramThreads) P.C[(int64_t)a0 * r + q] = acc[q];
}

__global__ __launch_bounds__(256) void k_zero(float* __restrict__ p, int64_t count) {
    for (int64_t k = (int64_t)blockIdx.x * 256 + threadIdx.x; k < count; k += (int64_t)gridDim.x * 256) p[k] = 0.0f;
}

// C = op(A) op(B) + beta E, all r x r row-major fp32; op squares every element (sqa, sqb) or transposes the
// operand (ta, tb) while its tiles are staged.  A launch takes up to kMaxGemmBatch independent products of
// one size (blockIdx.z picks one): a product alone is 256 small workgroups at r = 512, one per CU and each a
// chain of load latencies, so independent products share the chip.
// A workgroup of four waves makes a 32 x 32 tile of C (many small tiles: r is a few hundred, and
// every CU should get one).  The K range goes by in 128-wide tiles staged through LDS; inside a
// tile the four waves take 32 consecutive k each with v_mfma_f32_32x32x2_f32 -- lane l supplies
// A[i = l % 32][k = l / 32] and B[k = l / 32][j = l % 32] and holds
// C[8 (v / 4) + 4 (l / 32) + v % 4][l % 32] in accumulator register v -- and their four partial
// tiles are added through LDS at the end, in wave order.
constexpr int kTileMN = 32, kTileK = 128;
constexpr int kTileElems = kTileMN * kTileK / 256;                  // elements of each tile a thread stages
__global__ __launch_bounds__(256) void k_gemm_rr(const GemmBatch batch, int r) {
    __shared__ float As[kTileMN][kTileK + 1];
    __shared__ float Bs[kTileK][kTileMN + 1];
    __shared__ float Cs[4][16][64];
    GemmProblem P = batch.p[0];
#pragma unroll
    for (int z = 1; z < kMaxGemmBatch; ++z)
        if ((int)blockIdx.z == z) P = batch.p[z];
    const float* __restrict__ A = P.A;
    const float* __restrict__ B = P.B;
    const bool ta = P.flags & kGemmTA, tb = P.flags & kGemmTB, sqa = P.flags & kGemmSqA, sqb = P.flags & kGemmSqB;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int row0 = blockIdx.y * kTileMN, col0 = blockIdx.x * kTileMN;
    f32x16 acc;
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[v] = 0.0f;
    // A thread stages elements q = tid + 256 e of each tile; consecutive threads read consecutive addresses
    // whichever way the operand lies in memory.  Element e sits at (row, k) = (ar + e dar, ak + e dak) of the
    // A tile and at (k, col) = (bk + e dbk, bc + e dbc) of the B tile: one base and one step per operand.
    const int ar = ta ? tid % kTileMN : tid / kTileK, ak = ta ? tid / kTileMN : tid % kTileK;
    const int dar = ta ? 0 : 256 / kTileK, dak = ta ? 256 / kTileMN : 0;
    const int bk = tb ? tid % kTileK : tid / kTileMN, bc = tb ? tid / kTileK : tid % kTileMN;
    const int dbk = tb ? 0 : 256 / kTileMN, dbc = tb ? 256 / kTileK : 0;
    const int a_off = ta ? ak * r + row0 + ar : (row0 + ar) * r + ak;      // r * r < 2^31
    const int a_step = ta ? dak * r : dar * r, a_kstep = ta ? r : 1;
    const int b_off = tb ? (col0 + bc) * r + bk : bk * r + col0 + bc;
    const int b_step = tb ? dbc * r : dbk * r, b_kstep = tb ? 1 : r;
    float* const as0 = &As[0][0] + ar * (kTileK + 1) + ak;
    float* const bs0 = &Bs[0][0] + bk * (kTileMN + 1) + bc;
    const int as_step = dar * (kTileK + 1) + dak, bs_step = dbk * (kTileMN + 1) + dbc;
    // the next pair of tiles is fetched into registers while the matrix cores work on the current one
    float an[kTileElems], bn[kTileElems];
    auto fetch = [&](int k0) {
#pragma unroll
        for (int e = 0; e < kTileElems; ++e) {
            const bool aok = row0 + ar + e * dar < r && k0 + ak + e * dak < r;
            const float a = aok ? A[a_off + e * a_step + k0 * a_kstep] : 0.0f;
            an[e] = sqa ? a * a : a;
            const bool bok = k0 + bk + e * dbk < r && col0 + bc + e * dbc < r;
            const float b = bok ? B[b_off + e * b_step + k0 * b_kstep] : 0.0f;
            bn[e] = sqb ? b * b : b;
        }
    };
    fetch(0);
    for (int k0 = 0; k0 < r; k0 += kTileK) {
#pragma unroll
        for (int e = 0; e < kTileElems; ++e) {
            as0[e * as_step] = an[e];
            bs0[e * bs_step] = bn[e];
        }
        __syncthreads();
        if (k0 + kTileK < r) fetch(k0 + kTileK);
#pragma unroll
        for (int kk = wave * (kTileK / 4); kk < (wave + 1) * (kTileK / 4); kk += 2)
            acc = __builtin_amdgcn_mfma_f32_32x32x2f32(As[lane & 31][kk + (lane >> 5)],
                                                       Bs[kk + (lane >> 5)][lane & 31], acc, 0, 0, 0);
        __syncthreads();
    }
#pragma unroll
    for (int v = 0; v < 16; ++v) Cs[wave][v][lane] = acc[v];
    __syncthreads();
    if (wave == 0) {
        const int j = col0 + (lane & 31);
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int i = row0 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
            float sum = ((Cs[0][v][lane] + Cs[1][v][lane]) + Cs[2][v][lane]) + Cs[3][v][lane];
            if (i < r && j < r) {
                if (P.E) sum = fmaf(P.beta, P.E[(int64_t)i * r + j], sum);
                P.C[(int64_t)i * r + j] = sum;
            }
        }
    }
}

// The same product for r % 4 == 0, which is what the training configurations use: everything moves in groups
// of four floats.  Both tiles lie in LDS with k running along the rows (As[i][k], Bs[j][k], rows padded by 16
// bytes); a thread fetches 4 + 4 groups of 16 bytes per K tile -- four consecutive k of one row where the operand
// has k contiguous in memory (A as it is, B transposed: one 16-byte LDS store), else four consecutive rows of
// one k (four 4-byte LDS stores).  Within 8 consecutive k the lanes of half h = l / 32 take k = 4 h .. 4 h + 3
// with one 16-byte LDS load per operand, and the matrix instruction number s of the group multiplies element s of
// both: it sums over k = s and k = 4 + s, and the four of them over all eight.
constexpr int kTileRow4 = kTileK + 4;                               // floats per LDS row
constexpr int kTileGroups = kTileMN * kTileK / 4 / 256;             // 16-byte groups of each tile a thread stages
typedef float f32x4 __attribute__((ext_vector_type(4)));
__global__ __launch_bounds__(256) void k_gemm_rr4(const GemmBatch batch, int r) {
    __shared__ __align__(16) float As[kTileMN * kTileRow4];
    __shared__ __align__(16) float Bs[kTileMN * kTileRow4];
    __shared__ float Cs[4][16][64];
    GemmProblem P = batch.p[0];
#pragma unroll
    for (int z = 1; z < kMaxGemmBatch; ++z)
        if ((int)blockIdx.z == z) P = batch.p[z];
    const float* __restrict__ A = P.A;
    const float* __restrict__ B = P.B;
    const bool ta = P.flags & kGemmTA, tb = P.flags & kGemmTB, sqa = P.flags & kGemmSqA, sqb = P.flags & kGemmSqB;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int row0 = blockIdx.y * kTileMN, col0 = blockIdx.x * kTileMN;
    f32x16 acc;
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[v] = 0.0f;
    // Group q = tid + 256 e of a tile.  k contiguous in memory: row q / 32, k = 4 (q % 32) .. + 3 (rows step by 8
    // with e).  Rows contiguous in memory: k = q / 8, rows 4 (q % 8) .. + 3 (k steps by 32 with e).
    const bool a_kc = !ta, b_kc = tb;
    const int a_mn = a_kc ? tid / 32 : 4 * (tid % 8), a_k = a_kc ? 4 * (tid % 32) : tid / 8;
    const int b_mn = b_kc ? tid / 32 : 4 * (tid % 8), b_k = b_kc ? 4 * (tid % 32) : tid / 8;
    const int a_off = a_kc ? (row0 + a_mn) * r + a_k : a_k * r + row0 + a_mn;    // r * r < 2^31
    const int b_off = b_kc ? (col0 + b_mn) * r + b_k : b_k * r + col0 + b_mn;
    const int a_step = (a_kc ? 8 : 32) * r, b_step = (b_kc ? 8 : 32) * r;
    const int a_kstep = a_kc ? 1 : r, b_kstep = b_kc ? 1 : r;
    float* const as0 = As + a_mn * kTileRow4 + a_k;
    float* const bs0 = Bs + b_mn * kTileRow4 + b_k;
    const int as_step = a_kc ? 8 * kTileRow4 : 32, bs_step = b_kc ? 8 * kTileRow4 : 32;
    f32x4 an[kTileGroups], bn[kTileGroups];
    const f32x4 zero4 = {0.0f, 0.0f, 0.0f, 0.0f};
    auto fetch = [&](int k0) {
#pragma unroll
        for (int e = 0; e < kTileGroups; ++e) {
            const bool aok = row0 + a_mn + (a_kc ? 8 * e : 0) < r && k0 + a_k + (a_kc ? 0 : 32 * e) < r;
            const f32x4 a = aok ? *reinterpret_cast<const f32x4*>(A + a_off + e * a_step + k0 * a_kstep) : zero4;
            an[e] = sqa ? a * a : a;
            const bool bok = col0 + b_mn + (b_kc ? 8 * e : 0) < r && k0 + b_k + (b_kc ? 0 : 32 * e) < r;
            const f32x4 b = bok ? *reinterpret_cast<const f32x4*>(B + b_off + e * b_step + k0 * b_kstep) : zero4;
            bn[e] = sqb ? b * b : b;
        }
    };
    fetch(0);
    const float* ap = As + (lane & 31) * kTileRow4 + wave * (kTileK / 4) + 4 * (lane >> 5);
    const float* bp = Bs + (lane & 31) * kTileRow4 + wave * (kTileK / 4) + 4 * (lane >> 5);
    for (int k0 = 0; k0 < r; k0 += kTileK) {
#pragma unroll
        for (int e = 0; e < kTileGroups; ++e) {
            if (a_kc) *reinterpret_cast<f32x4*>(as0 + e * as_step) = an[e];
            else {
#pragma unroll
                for (int s = 0; s < 4; ++s) as0[e * as_step + s * kTileRow4] = an[e][s];
            }
            if (b_kc) *reinterpret_cast<f32x4*>(bs0 + e * bs_step) = bn[e];
            else {
#pragma unroll
                for (int s = 0; s < 4; ++s) bs0[e * bs_step + s * kTileRow4] = bn[e][s];
            }
        }
        __syncthreads();
        if (k0 + kTileK < r) fetch(k0 + kTileK);
#pragma unroll
        for (int g = 0; g < kTileK / 4 / 8; ++g) {                  // a wave's quarter of the tile, 8 k at a time
            const f32x4 a = *reinterpret_cast<const f32x4*>(ap + 8 * g);
            const f32x4 b = *reinterpret_cast<const f32x4*>(bp + 8 * g);
#pragma unroll
            for (int s = 0; s < 4; ++s) acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a[s], b[s], acc, 0, 0, 0);
        }
        __syncthreads();
    }
#pragma unroll
    for (int v = 0; v < 16; ++v) Cs[wave][v][lane] = acc[v];
    __syncthreads();
    if (wave == 0) {
        const int j = col0 + (lane & 31);
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int i = row0 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
            float sum = ((Cs[0][v][lane] + Cs[1][v][lane]) + Cs[2][v][lane]) + Cs[3][v][lane];
            if (i < r && j < r) {
                if (P.E) sum = fmaf(P.beta, P.E[(int64_t)i * r + j], sum);
                P.C[(int64_t)i * r + j] = sum;
            }
        }
    }
}

static dim3 blocks_for(int64_t count) { return dim3((unsigned)((count + 255) / 256 > 2048 ? 2048 : (count + 255) / 256)); }

hipError_t launch_zero(float* p, int64_t count, hipStream_t st) {
    hipLaunchKernelGGL(k_zero, blocks_for(count), dim3(256), 0, st, p, count);
    return hipGetLastError();
}

hipError_t launch_gram(const GramBatch& batch, int count, int32_t d, int32_t r, hipStream_t st) {
    if (count < 1 || count > 2 || r > kGramAccFloats) return hipErrorInvalidValue;
    for (int z = 0; z < count; ++z)
        if (batch.p[z].rows * d > INT32_MAX) return hipErrorInvalidValue;
    // LDS fp32 atomics go at a few cycles each per CU, so the rows of C are spread over about one workgroup
    // per CU rather than packed into as few as LDS allows (each workgroup scans all of L_idx either way)
    const int block_rows = std::max(1, std::min(kGramAccFloats / (int)r, ((int)r * count + 255) / 256));
    hipLaunchKernelGGL(k_gram, dim3((unsigned)((r + block_rows - 1) / block_rows), (unsigned)count), dim3(kGramThreads), 0, st,
                       batch, (int)d, (int)r, block_rows);
    return hipGetLastError();
}

hipError_t launch_gemm_rr_batch(const GemmBatch& batch, int count, int32_t r, hipStream_t st) {
    if (count < 1 || count > kMaxGemmBatch) return hipErrorInvalidValue;
    for (int z = 0; z < count; ++z)
        if ((batch.p[z].flags & kGemmTA) && (batch.p[z].flags & kGemmTB)) return hipErrorInvalidValue;   // not needed anywhere
    const dim3 grid((unsigned)((r + kTileMN - 1) / kTileMN), (unsigned)((r + kTileMN - 1) / kTileMN), (unsigned)count);
    bool by16 = r % 4 == 0;                                          // the 16-byte path: whole groups, aligned operands
    for (int z = 0; z < count; ++z)
        by16 = by16 && reinterpret_cast<uintptr_t>(batch.p[z].A) % 16 == 0 && reinterpret_cast<uintptr_t>(batch.p[z].B) % 16 == 0;
    if (by16) hipLaunchKernelGGL(k_gemm_rr4, grid, dim3(256), 0, st, batch, (int)r);
    else      hipLaunchKernelGGL(k_gemm_rr, grid, dim3(256), 0, st, batch, (int)r);
    return hipGetLastError();
}

hipError_t launch_reproject(const int32_t* P_idx, const float* P_val, const int32_t* Pp_idx, const float* Pp_val,
                            const int32_t* Q_idx, const float* Q_val, const int32_t* Qp_idx, const float* Qp_val,
                            int64_t m, int64_t n, int32_t r, int32_t d, float* M, float* V, float* workspace,
                            hipStream_t st) {
    const int64_t rr = (int64_t)r * r;
    float* A = workspace;
    float* B = workspace + rr;
    float* X = workspace + 2 * rr;
    GramBatch grams{};
    grams.p[0] = GramPair{P_idx, P_val, Pp_idx, Pp_val, m, A};
    grams.p[1] = GramPair{Qp_idx, Qp_val, Q_idx, Q_val, n, B};
    hipError_t e = launch_gram(grams, 2, d, r, st);
    if (e != hipSuccess) return e;
    // X = A M and X2 = (A o A) V in one launch, then M = X B and V = X2 (B o B) in another
    float* X2 = workspace + 3 * rr;
    GemmBatch left{}, right{};
    left.p[0] = GemmProblem{A, M, X, nullptr, 0.0f, 0};
    left.p[1] = GemmProblem{A, V, X2, nullptr, 0.0f, kGemmSqA};
    right.p[0] = GemmProblem{X, B, M, nullptr, 0.0f, 0};
    right.p[1] = GemmProblem{X2, B, V, nullptr, 0.0f, kGemmSqB};
    if ((e = launch_gemm_rr_batch(left, V ? 2 : 1, r, st)) != hipSuccess) return e;
    return launch_gemm_rr_batch(right, V ? 2 : 1, r, st);
}

}  // namespace lsp
