// Projector plan: column-sorted copies of P and Q, packed for the compress kernels.
//
// Compress needs the transposes of the ELL projectors (Def. 1 stores them by row; S = P^T G Q
// consumes them by column).  The projectors stay fixed between subspace refreshes (MaybeUpdate in
// Alg. 1 runs every CheckFreq steps), so the transposition is done once per refresh, here, and
// not in the per-step kernels.  This file only sorts and packs indices and values; it does no
// arithmetic on G, W or S.
#include <algorithm>
#include <cstring>
#include <utility>
#include <vector>

#include "lsp_internal.h"

namespace lsp {

// Longest list one lane may have to walk in one chunk: twice the mean list of a uniformly used
// column (so uniformly drawn projectors are never split), at least 16.
int plan_list_cap(int32_t r, int32_t d) {
    const int64_t mean = ((int64_t)kChunk * d + r - 1) / r;
    return (int)std::max<int64_t>(16, 2 * mean + 8);
}

size_t plan_max_rows(int64_t n, int32_t r, int32_t d) {
    const int64_t nchunks = (n + kChunk - 1) / kChunk;
    const int64_t seg = align_up((size_t)plan_list_cap(r, d), kSegBatch);
    return (size_t)(nchunks * kMaxSlots * kWavesGQ * seg + kWavesGQ * kStreamSlack);
}

size_t plan_max_items(int64_t m, int32_t r, int32_t d) {
    return (size_t)((int64_t)r + (m * d + kRowPiece - 1) / kRowPiece + 1);
}

PlanLayout plan_layout(int64_t m, int64_t n, int32_t r, int32_t d) {
    PlanLayout L;
    const size_t nchunks = (size_t)((n + kChunk - 1) / kChunk);
    size_t o = kPlanHeaderBytes;
    L.off_q_seg  = o; o = align_up(o + nchunks * kMaxSlots * kWavesGQ * sizeof(uint32_t), 256);
    L.off_q_vcol = o; o = align_up(o + (size_t)kMaxSlots * kThreadsGQ * sizeof(uint16_t), 256);
    L.off_q_vcnt = o; o = align_up(o + (size_t)kMaxSlots * kThreadsGQ * sizeof(uint16_t), 256);
    L.off_q_perm = o; o = align_up(o + nchunks * kThreadsGQ * sizeof(uint16_t), 256);
    L.off_q_rows = o; o = align_up(o + plan_max_rows(n, r, d) * kWave * sizeof(uint2), 256);
    L.off_p_item = o; o = align_up(o + plan_max_items(m, r, d) * sizeof(RowItem), 256);
    L.off_p_ent  = o; o = align_up(o + (size_t)(m * d) * sizeof(uint2), 256);
    L.off_q_src  = o; o = align_up(o + plan_max_rows(n, r, d) * kWave * sizeof(uint32_t), 256);
    L.off_p_src  = o; o = align_up(o + (size_t)(m * d) * sizeof(uint32_t), 256);
    L.total = o;
    return L;
}
namespace {
uint32_t float_bits(float f) { uint32_t u; std::memcpy(&u, &f, 4); return u; }
}  // namespace

size_t plan_bytes(int64_t m, int64_t n, int32_t r, int32_t d) { return plan_layout(m, n, r, d).total; }

int build_plan_host(const int32_t* P_idx, const float* P_val, const int32_t* Q_idx, const float* Q_val,
                    int64_t m, int64_t n, int32_t r, int32_t d, uint8_t* out) {
    const PlanLayout L = plan_layout(m, n, r, d);
    const int nchunks = (int)((n + kChunk - 1) / kChunk);
    const int cap = plan_list_cap(r, d);

    // ---- Q: lists of (column j of G, value) per (chunk, subspace column b) -----------------------
    // start[c][b] .. start[c][b+1] index into sorted[c], ordered by (b, j, k)
    std::vector<std::vector<int32_t>> start((size_t)nchunks, std::vector<int32_t>((size_t)r + 1, 0));
    std::vector<std::vector<uint2>> sorted((size_t)nchunks);
    std::vector<std::vector<uint32_t>> sorted_src((size_t)nchunks);      // flat ELL position j * d + k of each sorted pair
    std::vector<int32_t> cur((size_t)r);
    for (int c = 0; c < nchunks; ++c) {
        const int64_t j0 = (int64_t)c * kChunk, j1 = std::min<int64_t>(n, j0 + kChunk);
        auto& st = start[(size_t)c];
        for (int64_t j = j0; j < j1; ++j)
            for (int k = 0; k < d; ++k) st[(size_t)Q_idx[j * d + k] + 1]++;
        for (int b = 0; b < r; ++b) st[(size_t)b + 1] += st[(size_t)b];
        sorted[(size_t)c].assign((size_t)st[(size_t)r], uint2{0, 0});
        sorted_src[(size_t)c].assign((size_t)st[(size_t)r], 0u);
        for (int b = 0; b < r; ++b) cur[(size_t)b] = st[(size_t)b];
        for (int64_t j = j0; j < j1; ++j)
            for (int k = 0; k < d; ++k) {
                const int32_t b = Q_idx[j * d + k];
                sorted_src[(size_t)c][(size_t)cur[(size_t)b]] = (uint32_t)(j * d + k);
                sorted[(size_t)c][(size_t)cur[(size_t)b]++] =
                    uint2{chunk_col_offset((uint32_t)(j - j0)), float_bits(Q_val[j * d + k])};
            }
    }
    // owners per column: enough that no owner's share exceeds `cap` in any chunk; lanes left over
    // go, one at a time, to the column whose owners currently have the longest share (as long as
    // that share is at least 64 pairs)
    std::vector<int32_t> owners((size_t)r, 1), first_v((size_t)r + 1, 0), longest_of((size_t)r, 0);
    int64_t vneed = 0;
    for (int b = 0; b < r; ++b) {
        int32_t longest = 0;
        for (int c = 0; c < nchunks; ++c)
            longest = std::max(longest, start[(size_t)c][(size_t)b + 1] - start[(size_t)c][(size_t)b]);
        longest_of[(size_t)b] = longest;
        owners[(size_t)b] = std::max(1, (longest + cap - 1) / cap);
        vneed += owners[(size_t)b];
    }
    if (vneed < kThreadsGQ) {
        auto share_of = [&](int b) { return (double)longest_of[(size_t)b] / owners[(size_t)b]; };
        std::vector<std::pair<double, int>> heap;
        for (int b = 0; b < r; ++b) heap.emplace_back(share_of(b), -b);           // ties: lower column first
        std::make_heap(heap.begin(), heap.end());
        int64_t spare = kThreadsGQ - vneed;
        while (spare > 0 && !heap.empty()) {
            std::pop_heap(heap.begin(), heap.end());
            const int b = -heap.back().second;
            if (share_of(b) < 64.0) {                             // short lists: the merge would cost more than it saves
                heap.pop_back();
                continue;
            }
            owners[(size_t)b]++;
            --spare;
            heap.back().first = share_of(b);
            std::push_heap(heap.begin(), heap.end());
        }
    }
    for (int b = 0; b < r; ++b) first_v[(size_t)b + 1] = first_v[(size_t)b] + owners[(size_t)b];
    const int V = first_v[(size_t)r];
    if (V > kMaxSlots * kThreadsGQ) return LSP_ERR_SKEW;
    const int nslots = std::max(1, (V + kThreadsGQ - 1) / kThreadsGQ);

    std::memset(out, 0, L.total);
    PlanHeader* H = reinterpret_cast<PlanHeader*>(out);
    H->magic = kPlanMagic; H->m = (int32_t)m; H->n = (int32_t)n; H->r = r; H->d = d; H->nchunks = nchunks;
    H->nslots = nslots; H->nvcols = V; H->list_cap = cap;
    H->off_q_seg = L.off_q_seg; H->off_q_vcol = L.off_q_vcol; H->off_q_vcnt = L.off_q_vcnt; H->off_q_perm = L.off_q_perm; H->off_q_rows = L.off_q_rows;
    H->off_p_item = L.off_p_item; H->off_p_ent = L.off_p_ent; H->total_bytes = L.total;
    H->off_q_src = L.off_q_src; H->off_p_src = L.off_p_src;

    uint32_t* seg  = reinterpret_cast<uint32_t*>(out + L.off_q_seg);
    uint16_t* vcol = reinterpret_cast<uint16_t*>(out + L.off_q_vcol);
    uint2*    rows = reinterpret_cast<uint2*>(out + L.off_q_rows);
    uint32_t* qsrc = reinterpret_cast<uint32_t*>(out + L.off_q_src);
    std::vector<int32_t> v_col((size_t)nslots * kThreadsGQ, -1), v_own((size_t)nslots * kThreadsGQ, 0);
    for (int b = 0; b < r; ++b)
        for (int o = 0; o < owners[(size_t)b]; ++o) {
            const int v = first_v[(size_t)b] + o;
            v_col[(size_t)v] = b; v_own[(size_t)v] = o;
        }
    uint16_t* vcnt = reinterpret_cast<uint16_t*>(out + L.off_q_vcnt);
    for (size_t v = 0; v < v_col.size(); ++v) {
        vcol[v] = v_col[v] < 0 ? (uint16_t)kNoColumn
                               : (uint16_t)((uint32_t)v_col[v] | (owners[(size_t)v_col[v]] > 1 ? kSharedColumn : 0u));
        vcnt[v] = (v_col[v] >= 0 && v_own[v] == 0) ? (uint16_t)owners[(size_t)v_col[v]] : (uint16_t)0;
    }

    // share of owner o of column b in chunk c: [lo, hi) inside the chunk's sorted list of b
    auto share = [&](int c, int b, int o, int32_t& lo, int32_t& hi) {
        const int32_t s0 = start[(size_t)c][(size_t)b], len = start[(size_t)c][(size_t)b + 1] - s0;
        const int k = owners[(size_t)b];
        lo = s0 + (int32_t)((int64_t)len * o / k);
        hi = s0 + (int32_t)((int64_t)len * (o + 1) / k);
    };
    const uint2 pad_pair{(uint32_t)kChunk * 16u, 0u};       // the always-zero unit of each plane
    // rows 2p and 2p+1 are interleaved per lane (every segment has an even number of rows)
    auto row_slot = [](size_t rw, int lane) { return ((rw >> 1) * kWave + (size_t)lane) * 2 + (rw & 1); };
    int any_shared = 0;
    for (int b = 0; b < r; ++b) any_shared |= owners[(size_t)b] > 1;
    H->q_any_shared = any_shared;
    // With one slot the lists of a chunk are dealt to the waves by length: sorted longest first, the
    // k-th group of 64 goes to wave k for k < 4 and to wave 11 - k otherwise, so that the two waves
    // of a SIMD (w and w + 4) get a long and a short group.  walker[c][t]: virtual column of thread t.
    const bool permuted = nslots == 1;
    H->q_permuted = permuted ? 1 : 0;
    uint16_t* perm = reinterpret_cast<uint16_t*>(out + L.off_q_perm);
    std::vector<int32_t> order((size_t)kThreadsGQ), length((size_t)kThreadsGQ);
    for (int c = 0; c < nchunks; ++c) {
        for (int v = 0; v < kThreadsGQ; ++v) {
            order[(size_t)v] = v;
            int32_t lo = 0, hi = 0;
            if (permuted && v_col[(size_t)v] >= 0) share(c, v_col[(size_t)v], v_own[(size_t)v], lo, hi);
            length[(size_t)v] = hi - lo;
        }
        if (permuted)
            std::stable_sort(order.begin(), order.end(),
                             [&](int32_t x, int32_t y) { return length[(size_t)x] > length[(size_t)y]; });
        for (int k = 0; k < kWavesGQ; ++k) {
            const int w = k < kWavesGQ / 2 ? k : kWavesGQ + kWavesGQ / 2 - 1 - k;
            for (int lane = 0; lane < kWave; ++lane)
                perm[(size_t)c * kThreadsGQ + (size_t)w * kWave + (size_t)lane] = (uint16_t)order[(size_t)k * kWave + (size_t)lane];
        }
    }
    size_t row = 0;
    for (int w = 0; w < kWavesGQ; ++w) {
        H->q_stream_row[w] = (uint32_t)row;
        for (int c = 0; c < nchunks; ++c)
            for (int s = 0; s < nslots; ++s) {
                auto walked = [&](int lane) {
                    return permuted ? (size_t)perm[(size_t)c * kThreadsGQ + (size_t)w * kWave + (size_t)lane]
                                    : (size_t)s * kThreadsGQ + (size_t)w * kWave + (size_t)lane;
                };
                int32_t longest = 0;
                for (int lane = 0; lane < kWave; ++lane) {
                    const size_t v = walked(lane);
                    if (v_col[v] < 0) continue;
                    int32_t lo, hi; share(c, v_col[v], v_own[v], lo, hi);
                    longest = std::max(longest, hi - lo);
                }
                const int32_t len = (int32_t)align_up((size_t)longest, kSegBatch);
                seg[((size_t)c * nslots + (size_t)s) * kWavesGQ + (size_t)w] = (uint32_t)len;
                for (int lane = 0; lane < kWave; ++lane) {
                    const size_t v = walked(lane);
                    int32_t lo = 0, hi = 0;
                    if (v_col[v] >= 0) share(c, v_col[v], v_own[v], lo, hi);
                    for (int32_t e = 0; e < len; ++e) {
                        const size_t slot = row_slot(row + (size_t)e, lane);
                        rows[slot] = e < hi - lo ? sorted[(size_t)c][(size_t)(lo + e)] : pad_pair;
                        qsrc[slot] = e < hi - lo ? sorted_src[(size_t)c][(size_t)(lo + e)] : kNoSource;
                    }
                }
                row += (size_t)len;
            }
        for (int e = 0; e < kStreamSlack; ++e, ++row)
            for (int lane = 0; lane < kWave; ++lane) {
                rows[row_slot(row, lane)] = pad_pair;
                qsrc[row_slot(row, lane)] = kNoSource;
            }
    }
    H->q_total_rows = (int32_t)row;

    // ---- P^T: for each subspace row a, the (row of G, value) pairs, cut into pieces -------------
    RowItem* items = reinterpret_cast<RowItem*>(out + L.off_p_item);
    uint2*   pent  = reinterpret_cast<uint2*>(out + L.off_p_ent);
    uint32_t* psrc = reinterpret_cast<uint32_t*>(out + L.off_p_src);
    std::vector<int32_t> cnt((size_t)r + 1, 0);
    for (int64_t i = 0; i < m; ++i)
        for (int k = 0; k < d; ++k) cnt[(size_t)P_idx[i * d + k] + 1]++;
    for (int a = 0; a < r; ++a) cnt[(size_t)a + 1] += cnt[(size_t)a];
    for (int a = 0; a < r; ++a) cur[(size_t)a] = cnt[(size_t)a];
    for (int64_t i = 0; i < m; ++i)
        for (int k = 0; k < d; ++k) {
            const int32_t a = P_idx[i * d + k];
            psrc[(size_t)cur[(size_t)a]] = (uint32_t)(i * d + k);
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
    return LSP_OK;
}

// ---- entry order inside the rows of a projector, for the expand side ---------------------------
// The decompress kernels give lane l of a wave the columns 2 l and 2 l + 1 of a 128-column tile, and
// all 64 lanes gather entry k of their column with one 128-bit LDS read of U[b] (b = the entry's
// index; 16 bytes per b, so the bank group of a read is b mod 16).  The hardware serves such a
// read in four groups of 16 lanes -- (lane >= 32, parity of bits 2..4 of the lane) -- and a group
// costs as many cycles as its most used bank group.  The order of the d entries of a row is free
// (they are summed), so each row's entries are dealt to the d slots such that, slot by slot, the
// lanes of a group meet on a bank group as rarely as a greedy pass manages (12.2 -> 9.2 modelled
// cycles per read on uniformly drawn columns; 7.5 is the floor).
int reorder_rows_host(const int32_t* idx, const float* val, int64_t rows, int32_t d, int32_t r,
                      int32_t* idx_out, float* val_out) {
    if (d > 64) return LSP_ERR_SHAPE;
    for (int64_t k = 0; k < rows * d; ++k)
        if (idx[k] < 0 || idx[k] >= r) return LSP_ERR_INDEX;
    auto group_of = [](int lane) {
        const int q = (lane & 31) >> 2;
        return ((lane >> 5) << 1) | (((q >> 2) ^ (q >> 1) ^ q) & 1);
    };
    std::vector<uint16_t> used((size_t)4 * (size_t)d);       // [group][slot]: bank groups taken
    std::vector<int> slot_of((size_t)d);
    std::vector<char> taken((size_t)d);
    for (int64_t tile = 0; tile < rows; tile += 2 * kWave)
        for (int c = 0; c < 2; ++c) {
            std::fill(used.begin(), used.end(), (uint16_t)0);
            for (int lane = 0; lane < kWave; ++lane) {
                const int64_t j = tile + 2 * lane + c;
                if (j >= rows) break;
                uint16_t* u = used.data() + (size_t)group_of(lane) * (size_t)d;
                std::fill(taken.begin(), taken.end(), (char)0);
                // entries with the fewest admissible slots (bank group still free there) choose first
                for (int e = 0; e < d; ++e) slot_of[(size_t)e] = -1;
                for (int round = 0; round < d; ++round) {
                    int best = -1, best_free = d + 1;
                    for (int e = 0; e < d; ++e) {
                        if (slot_of[(size_t)e] != -1) continue;
                        const uint16_t bit = (uint16_t)(1u << (idx[j * d + e] & 15));
                        int nfree = 0;
                        for (int k = 0; k < d; ++k) nfree += (!taken[(size_t)k] && !(u[k] & bit));
                        if (nfree < best_free) { best_free = nfree; best = e; }
                    }
                    if (best < 0) break;
                    if (best_free == 0) { slot_of[(size_t)best] = -2; continue; }     // no admissible slot: placed below
                    const uint16_t bit = (uint16_t)(1u << (idx[j * d + best] & 15));
                    // among the admissible slots take the one fewest other lanes have used so far
                    int pick = -1, pick_load = 17;
                    for (int k = 0; k < d; ++k)
                        if (!taken[(size_t)k] && !(u[k] & bit)) {
                            const int load = __builtin_popcount(u[k]);
                            if (load < pick_load) { pick_load = load; pick = k; }
                        }
                    slot_of[(size_t)best] = pick; taken[(size_t)pick] = 1;
                }
                for (int e = 0; e < d; ++e) if (slot_of[(size_t)e] == -2) slot_of[(size_t)e] = -1;
                for (int e = 0, k = 0; e < d; ++e) {          // the rest: any slot left
                    if (slot_of[(size_t)e] >= 0) continue;
                    while (taken[(size_t)k]) ++k;
                    slot_of[(size_t)e] = k; taken[(size_t)k] = 1;
                }
                for (int e = 0; e < d; ++e) {
                    const int k = slot_of[(size_t)e];
                    idx_out[j * d + k] = idx[j * d + e];
                    val_out[j * d + k] = val[j * d + e];
                    u[k] |= (uint16_t)(1u << (idx[j * d + e] & 15));
                }
            }
        }
    return LSP_OK;
}

}  // namespace lsp
