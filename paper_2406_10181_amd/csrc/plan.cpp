// Projector plan: column-sorted copies of P and Q, packed for the compress kernels.
//
// Compress needs the transposes of the ELL projectors (Def. 1 stores them by row; S = P^T G Q
// consumes them by column).  The projectors stay fixed between subspace refreshes (MaybeUpdate in
// Alg. 1 runs every CheckFreq steps), so the transposition is done once per refresh, here, and
// not in the per-step kernels.  This file only sorts and packs indices and values; it does no
// arithmetic on G, W or S.
#include <algorithm>
#include <cstring>
#include <vector>

#include "lsp_internal.h"

namespace lsp {

size_t plan_max_rounds(int64_t n, int32_t r, int32_t d) {
    const int64_t nchunks = (n + kChunk - 1) / kChunk;
    const int64_t items_per_chunk = (int64_t)r + ((int64_t)kChunk * d + kListMax - 1) / kListMax + 1;
    return (size_t)(nchunks * ((items_per_chunk + kWave - 1) / kWave + 1));
}

size_t plan_max_slots(int64_t n, int32_t r, int32_t d) {
    (void)r;
    const int64_t nchunks = (n + kChunk - 1) / kChunk;
    // Pieces are sorted by length inside a chunk, so the padded size of all rounds after the first
    // is bounded by the entries themselves; the first round adds at most 64 * kListMax.
    return (size_t)(n * d + nchunks * (int64_t)kWave * (kListMax + 1));
}

size_t plan_max_items(int64_t m, int32_t r, int32_t d) {
    return (size_t)((int64_t)r + (m * d + kRowPiece - 1) / kRowPiece + 1);
}

namespace {
struct Layout {
    size_t off_q_chunk, off_q_round, off_q_cols, off_q_ent, off_p_item, off_p_ent, total;
};
Layout plan_layout(int64_t m, int64_t n, int32_t r, int32_t d) {
    Layout L;
    const size_t nchunks = (size_t)((n + kChunk - 1) / kChunk);
    size_t o = kPlanHeaderBytes;
    L.off_q_chunk = o; o = align_up(o + nchunks * sizeof(ChunkInfo), 256);
    L.off_q_round = o; o = align_up(o + plan_max_rounds(n, r, d) * sizeof(RoundInfo), 256);
    L.off_q_cols  = o; o = align_up(o + plan_max_rounds(n, r, d) * kWave * sizeof(uint16_t), 256);
    L.off_q_ent   = o; o = align_up(o + plan_max_slots(n, r, d) * sizeof(uint2), 256);
    L.off_p_item  = o; o = align_up(o + plan_max_items(m, r, d) * sizeof(RowItem), 256);
    L.off_p_ent   = o; o = align_up(o + (size_t)(m * d) * sizeof(uint2), 256);
    L.total = o;
    return L;
}
uint32_t float_bits(float f) { uint32_t u; std::memcpy(&u, &f, 4); return u; }
}  // namespace

size_t plan_bytes(int64_t m, int64_t n, int32_t r, int32_t d) { return plan_layout(m, n, r, d).total; }

void build_plan_host(const int32_t* P_idx, const float* P_val, const int32_t* Q_idx, const float* Q_val,
                     int64_t m, int64_t n, int32_t r, int32_t d, uint8_t* out) {
    const Layout L = plan_layout(m, n, r, d);
    std::memset(out, 0, L.total);
    PlanHeader* H = reinterpret_cast<PlanHeader*>(out);
    const int nchunks = (int)((n + kChunk - 1) / kChunk);
    H->magic = kPlanMagic; H->m = (int32_t)m; H->n = (int32_t)n; H->r = r; H->d = d; H->nchunks = nchunks;
    H->off_q_chunk = L.off_q_chunk; H->off_q_round = L.off_q_round; H->off_q_cols = L.off_q_cols;
    H->off_q_ent = L.off_q_ent; H->off_p_item = L.off_p_item; H->off_p_ent = L.off_p_ent;
    H->total_bytes = L.total;

    ChunkInfo* chunks = reinterpret_cast<ChunkInfo*>(out + L.off_q_chunk);
    RoundInfo* rounds = reinterpret_cast<RoundInfo*>(out + L.off_q_round);
    uint16_t*  cols   = reinterpret_cast<uint16_t*>(out + L.off_q_cols);
    uint2*     qent   = reinterpret_cast<uint2*>(out + L.off_q_ent);

    // ---- Q: per chunk of kChunk columns of G, the entries grouped by subspace column b ----------
    struct Piece { int32_t b; int32_t start; int32_t len; int32_t shared; };
    std::vector<int32_t> cnt((size_t)r + 1), cur((size_t)r);
    std::vector<uint2> sorted;                 // entries of one chunk ordered by (b, j, k)
    std::vector<Piece> pieces;
    int total_rounds = 0;
    size_t slot = 0;
    const uint32_t pad_offset = (uint32_t)kChunk * 16u;     // the always-zero unit of each plane
    for (int c = 0; c < nchunks; ++c) {
        const int64_t j0 = (int64_t)c * kChunk, j1 = std::min<int64_t>(n, j0 + kChunk);
        std::fill(cnt.begin(), cnt.end(), 0);
        for (int64_t j = j0; j < j1; ++j)
            for (int k = 0; k < d; ++k) cnt[(size_t)Q_idx[j * d + k] + 1]++;
        for (int b = 0; b < r; ++b) cnt[(size_t)b + 1] += cnt[(size_t)b];
        sorted.assign((size_t)cnt[(size_t)r], uint2{0, 0});
        for (int b = 0; b < r; ++b) cur[(size_t)b] = cnt[(size_t)b];
        for (int64_t j = j0; j < j1; ++j)
            for (int k = 0; k < d; ++k) {
                const int32_t b = Q_idx[j * d + k];
                sorted[(size_t)cur[(size_t)b]++] = uint2{chunk_col_offset((uint32_t)(j - j0)),
                                                         float_bits(Q_val[j * d + k])};
            }
        pieces.clear();
        for (int b = 0; b < r; ++b)
            for (int32_t s = cnt[(size_t)b]; s < cnt[(size_t)b + 1]; s += kListMax)
                pieces.push_back(Piece{b, s, std::min<int32_t>(kListMax, cnt[(size_t)b + 1] - s),
                                       cnt[(size_t)b + 1] - cnt[(size_t)b] > kListMax});
        std::stable_sort(pieces.begin(), pieces.end(),
                         [](const Piece& x, const Piece& y) { return x.len > y.len; });
        chunks[c].first_round = total_rounds;
        const int nr = (int)((pieces.size() + kWave - 1) / kWave);
        chunks[c].nrounds = nr;
        for (int rho = 0; rho < nr; ++rho) {
            const size_t p0 = (size_t)rho * kWave;
            const int len = pieces[p0].len;
            RoundInfo& ri = rounds[total_rounds];
            ri.ent_offset = (uint32_t)slot; ri.len = len;
            for (int lane = 0; lane < kWave; ++lane) {
                const bool have = p0 + (size_t)lane < pieces.size();
                cols[(size_t)total_rounds * kWave + (size_t)lane] =
                    have ? (uint16_t)(pieces[p0 + (size_t)lane].b | (pieces[p0 + (size_t)lane].shared ? kSharedColumn : 0u))
                         : (uint16_t)kNoColumn;
                for (int e = 0; e < len; ++e) {
                    uint2 v{pad_offset, 0u};
                    if (have && e < pieces[p0 + (size_t)lane].len)
                        v = sorted[(size_t)pieces[p0 + (size_t)lane].start + (size_t)e];
                    qent[slot + (size_t)e * kWave + (size_t)lane] = v;
                }
            }
            slot += (size_t)len * kWave;
            ++total_rounds;
        }
    }
    H->q_total_rounds = total_rounds;

    // ---- P^T: for each subspace row a, the (row of G, value) pairs, cut into pieces -------------
    RowItem* items = reinterpret_cast<RowItem*>(out + L.off_p_item);
    uint2*   pent  = reinterpret_cast<uint2*>(out + L.off_p_ent);
    std::fill(cnt.begin(), cnt.end(), 0);
    for (int64_t i = 0; i < m; ++i)
        for (int k = 0; k < d; ++k) cnt[(size_t)P_idx[i * d + k] + 1]++;
    for (int a = 0; a < r; ++a) cnt[(size_t)a + 1] += cnt[(size_t)a];
    for (int a = 0; a < r; ++a) cur[(size_t)a] = cnt[(size_t)a];
    for (int64_t i = 0; i < m; ++i)
        for (int k = 0; k < d; ++k) {
            const int32_t a = P_idx[i * d + k];
            pent[(size_t)cur[(size_t)a]++] = uint2{(uint32_t)i, float_bits(P_val[i * d + k])};
        }
    int nitems = 0, any_split = 0;
    for (int a = 0; a < r; ++a) {
        const int32_t s0 = cnt[(size_t)a], s1 = cnt[(size_t)a + 1];
        const int split = (s1 - s0) > kRowPiece;
        any_split |= split;
        if (s1 == s0) { items[nitems++] = RowItem{a, s0, 0, 0}; continue; }
        for (int32_t s = s0; s < s1; s += kRowPiece)
            items[nitems++] = RowItem{a, s, std::min<int32_t>(kRowPiece, s1 - s), split};
    }
    H->p_nitems = nitems;
    H->p_any_split = any_split;
}

}  // namespace lsp
