"""CPU-only checks of the C-ABI library: it loads, exports every symbol the header declares,
rejects bad arguments before touching the GPU, and its host-side plan builder packs the
projectors correctly (decoded here and replayed with numpy).  No compute call is made."""
import ctypes
import os
import re

import numpy as np
import pytest

import lsp_synth as syn
import paper_2406_10181_amd as L

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CHUNK = 2048
THREADS = 512           # threads of the T = G Q kernel
PAD_OFFSET = CHUNK * 16
BATCH = 4                # segment lengths are multiples of this many plan rows
SLACK = 4 * BATCH        # readable rows behind each wave's stream (the kernel's prefetch depth)


def test_every_declared_symbol_is_exported():
    hdr = open(os.path.join(ROOT, "include", "lsp.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    names = set(re.findall(r"\b(lsp_[a-z_]+)\s*\(", hdr))
    assert {"lsp_compress", "lsp_decompress_apply", "lsp_plan_build", "lsp_compress_planned"} <= names
    lib = L.lib()
    for nm in sorted(names):
        assert hasattr(lib, nm), f"{nm} declared in include/lsp.h but not exported"
    assert L.lsp_version() >= 100


def test_argument_errors_without_gpu():
    big = 1 << 20
    ok = dict(m=64, n=64, r=16, d=2)
    fake = 0x1000          # aligned, never dereferenced: every check below fails before any HIP call
    # NULL pointers
    assert L.lsp_compress(None, fake, fake, fake, fake, 64, 64, 16, 2, fake, 0, fake, big, check=False) == -1
    assert L.lsp_decompress_apply(None, fake, fake, fake, fake, fake, 64, 64, 16, 2, 0, check=False) == -1
    assert L.lsp_compress_planned(fake, None, 64, 64, 16, 2, fake, 0, fake, big, check=False) == -1
    # shapes
    for m, n, r, d in [(0, 64, 16, 2), (64, -1, 16, 2), (64, 64, 0, 2), (64, 64, 16, 0), (64, 64, 4, 8),
                       (64, 64, 4096, 2), (64, 64, 128, 65), (1 << 31, 4, 16, 2)]:
        assert L.lsp_compress(fake, fake, fake, fake, fake, m, n, r, d, fake, 0, fake, big, check=False) == -2
        assert L.lsp_decompress_apply(fake, fake, fake, fake, fake, fake, m, n, r, d, 0, check=False) == -2
        assert L.lsp_plan_bytes(m, n, r, d) == 0
        assert L.lsp_compress_workspace_bytes(m, n, r, d) == 0
    # dtype
    assert L.lsp_compress(fake, fake, fake, fake, fake, 64, 64, 16, 2, fake, 7, fake, big, check=False) == -3
    assert L.lsp_decompress_apply(fake, fake, fake, fake, fake, fake, 64, 64, 16, 2, -1, check=False) == -3
    # workspace too small / missing / misaligned
    need = L.lsp_compress_workspace_bytes(**ok)
    assert need >= 64 * 16 * 4
    assert L.lsp_compress(fake, fake, fake, fake, fake, 64, 64, 16, 2, fake, 0, fake, need - 1, check=False) == -4
    assert L.lsp_compress(fake, fake, fake, fake, fake, 64, 64, 16, 2, fake, 0, None, need, check=False) == -4
    assert L.lsp_compress(fake, fake, fake, fake, fake, 64, 64, 16, 2, fake, 0, fake + 4, need, check=False) == -4
    assert L.lsp_compress_planned(fake, fake, 64, 64, 16, 2, fake, 0, fake, 8, check=False) == -4
    # alignment of data pointers
    assert L.lsp_compress(fake + 2, fake, fake, fake, fake, 64, 64, 16, 2, fake, 0, fake, need, check=False) == -7
    assert L.lsp_decompress_apply(fake, fake + 8, fake, fake, fake, fake, 64, 64, 16, 2, 0, check=False) == -7
    # the estimation-bias call checks its arguments the same way
    bias = lambda *a, **k: L.lsp_estimation_bias(*a, check=False, **k)
    bneed = L.lsp_estimation_bias_workspace_bytes(**ok)
    assert bneed >= (64 // 16) * 8 and L.lsp_estimation_bias_workspace_bytes(0, 64, 16, 2) == 0
    assert bias(None, fake, fake, fake, fake, fake, 64, 64, 16, 2, fake, fake, bneed, 0) == -1
    assert bias(fake, fake, fake, fake, fake, fake, 64, 64, 16, 2, None, fake, bneed, 0) == -1
    assert bias(fake, fake, fake, fake, fake, fake, 64, 64, 4, 8, fake, fake, bneed, 0) == -2
    assert bias(fake, fake, fake, fake, fake, fake, 64, 64, 16, 2, fake, fake, bneed, 9) == -3
    assert bias(fake, fake, fake, fake, fake, fake, 64, 64, 16, 2, fake, fake, bneed - 1, 0) == -4
    assert bias(fake, fake, fake, fake, fake, fake, 64, 64, 16, 2, fake, None, bneed, 0) == -4
    assert bias(fake, fake + 4, fake, fake, fake, fake, 64, 64, 16, 2, fake, fake, bneed, 0) == -7
    # the fitting gradient and the values-only refresh of a plan
    grad = lambda *a, **k: L.lsp_bias_gradient(*a, check=False, **k)
    gneed = L.lsp_bias_gradient_workspace_bytes(**ok)
    assert gneed >= (64 * 16 + 8 * 16 * 16 + 16 * 64) * 4 and L.lsp_bias_gradient_workspace_bytes(64, 64, 4, 8) == 0
    assert L.lsp_workspace_bytes(64, 64, 16, 2, 2) >= gneed and L.lsp_workspace_bytes(64, 64, 16, 2, 9) == 0
    assert grad(None, fake, fake, fake, fake, fake, 64, 64, 16, 2, fake, fake, fake, gneed, 0) == -1
    assert grad(fake, fake, fake, fake, fake, fake, 64, 64, 16, 2, fake, None, fake, gneed, 0) == -1
    assert grad(fake, fake, fake, fake, fake, fake, 64, 64, 16, 0, fake, fake, fake, gneed, 0) == -2
    assert grad(fake, fake, fake, fake, fake, fake, 64, 64, 16, 2, fake, fake, fake, gneed, 3) == -3
    assert grad(fake, fake, fake, fake, fake, fake, 64, 64, 16, 2, fake, fake, fake, gneed - 1, 0) == -4
    assert grad(fake, fake, fake, fake, fake, fake, 64, 64, 16, 2, fake, fake + 4, fake, gneed, 0) == -7
    assert L.lsp_plan_refresh_values(None, fake, fake, 64, 64, 16, 2, None, check=False) == -1
    assert L.lsp_plan_refresh_values(fake, fake, fake, 64, 0, 16, 2, None, check=False) == -2
    assert L.lsp_plan_refresh_values(fake, fake + 4, fake, 64, 64, 16, 2, None, check=False) == -7
    # and so does the state re-projection
    rep = lambda *a, **k: L.lsp_reproject_state(*a, check=False, **k)
    rneed = L.lsp_reproject_state_workspace_bytes(16)
    assert rneed >= 3 * 16 * 16 * 4 and L.lsp_reproject_state_workspace_bytes(0) == 0
    eight = (fake,) * 8
    assert rep(None, *eight[1:], 64, 64, 16, 2, fake, fake + 1024, fake, rneed) == -1
    assert rep(*eight, 64, 64, 16, 2, None, fake, fake, rneed) == -1
    assert rep(*eight, 64, 64, 16, 32, fake, fake + 1024, fake, rneed) == -2
    assert rep(*eight, 64, 64, 16, 2, fake, fake, fake, rneed) == -2           # M and V the same buffer
    assert rep(*eight, 64, 64, 16, 2, fake, fake + 1024, fake, rneed - 1) == -4
    assert rep(*eight, 64, 64, 16, 2, fake + 4, None, fake, rneed) == -7
    assert "NULL" in L.lsp_strerror(-1) and L.lsp_strerror(0) == "ok"
    with pytest.raises(L.LspError):
        L.lsp_compress(None, fake, fake, fake, fake, 64, 64, 16, 2, fake, 0, fake, big)


def test_grouped_argument_errors_without_gpu():
    fake, big = 0x1000, 1 << 20
    one = L.compress_items([(fake, fake, fake, fake, big, 64, 64)])
    assert L.lsp_compress_planned_grouped(None, 1, 16, 2, 0, check=False) == -1
    assert L.lsp_compress_planned_grouped(one, 0, 16, 2, 0, check=False) == -2
    assert L.lsp_compress_planned_grouped(one, 17, 16, 2, 0, check=False) == -2
    assert L.lsp_compress_planned_grouped(one, 1, 16, 2, 9, check=False) == -3
    assert L.lsp_compress_planned_grouped(L.compress_items([(fake, None, fake, fake, big, 64, 64)]), 1, 16, 2, 0, check=False) == -1
    assert L.lsp_compress_planned_grouped(L.compress_items([(fake, fake, fake, fake, 8, 64, 64)]), 1, 16, 2, 0, check=False) == -4
    assert L.lsp_compress_planned_grouped(L.compress_items([(fake, fake, fake, fake, big, 64, 0)]), 1, 16, 2, 0, check=False) == -2
    # two problems sharing a workspace or an S would race
    two = L.compress_items([(fake, fake, fake, fake, big, 64, 64), (fake, fake, 0x2000, fake, big, 64, 64)])
    assert L.lsp_compress_planned_grouped(two, 2, 16, 2, 0, check=False) == -4
    two = L.compress_items([(fake, fake, fake, fake, big, 64, 64), (fake, fake, fake, 0x100000, big, 64, 64)])
    assert L.lsp_compress_planned_grouped(two, 2, 16, 2, 0, check=False) == -4
    a1 = L.apply_items([(fake, fake, fake, fake, fake, fake, 64, 64)])
    assert L.lsp_decompress_apply_grouped(None, 1, 16, 2, 0, check=False) == -1
    assert L.lsp_decompress_apply_grouped(a1, 0, 16, 2, 0, check=False) == -2
    assert L.lsp_decompress_apply_grouped(a1, 1, 16, 2, 5, check=False) == -3
    assert L.lsp_decompress_apply_grouped(L.apply_items([(fake, fake, None, fake, fake, fake, 64, 64)]), 1, 16, 2, 0, check=False) == -1
    assert L.lsp_decompress_apply_grouped(L.apply_items([(fake + 2, fake, fake, fake, fake, fake, 64, 64)]), 1, 16, 2, 0, check=False) == -7
    a2 = L.apply_items([(fake, fake, fake, fake, fake, fake, 64, 64), (fake, fake, fake, fake, fake, fake, 64, 64)])
    assert L.lsp_decompress_apply_grouped(a2, 2, 16, 2, 0, check=False) == -2       # the same W twice
    import ctypes
    assert ctypes.sizeof(L.lsp_compress_item) == 56 and ctypes.sizeof(L.lsp_apply_item) == 64


# ------------------------------------------------------------------ plan decoding
def _decode_col(off):
    unit = off // 16
    return (unit % (CHUNK // 8)) * 8 + unit // (CHUNK // 8)


def _build_host_plan(pb):
    nbytes = L.lsp_plan_bytes(pb.m, pb.n, pb.r, pb.d)
    buf = np.zeros(nbytes, dtype=np.uint8)
    L.lsp_plan_build_host(pb.P_idx, pb.P_val, pb.Q_idx, pb.Q_val, pb.m, pb.n, pb.r, pb.d, buf, nbytes)
    return buf


def _replay_plan(buf, pb):
    """What the plan means: T = G Qhat from the Q part, then S = Phat^T T from the P part.
    The Q streams are walked exactly as the kernel walks them: wave by wave, chunk-major, slot by
    slot, each segment's length from the table; lane l of wave w in slot s walks the list of virtual
    column s*512 + w*64 + l, or, with one slot, of the virtual column the per-chunk table names."""
    hdr32 = buf[:48].view(np.int32)
    assert hdr32[0] == 0x4C535038
    m, n, r, d, nchunks, nslots, nvcols, total_rows, nitems, any_split, cap = [int(x) for x in hdr32[1:12]]
    assert (m, n, r, d) == (pb.m, pb.n, pb.r, pb.d) and nchunks == -(-n // CHUNK)
    assert 1 <= nslots <= 4 and nvcols <= nslots * 512
    stream_row = [int(x) for x in buf[48:80].view(np.uint32)]
    o_seg, o_vcol, o_rows, o_item, o_pent, total = [int(x) for x in buf[96:144].view(np.uint64)]
    assert total == buf.size and all(o % 16 == 0 for o in (o_seg, o_vcol, o_rows, o_item, o_pent))
    assert o_rows + total_rows * 64 * 8 <= o_item
    seg = buf[o_seg:o_seg + nchunks * nslots * 8 * 4].view(np.uint32).reshape(nchunks, nslots, 8)
    vcol = buf[o_vcol:o_vcol + nslots * 512 * 2].view(np.uint16).reshape(nslots, 8, 64)
    # rows 2p and 2p+1 are interleaved per lane: [pair][lane][row parity][offset, value bits]
    assert total_rows % 2 == 0 and all(x % 2 == 0 for x in stream_row)
    rows = buf[o_rows:o_rows + total_rows * 64 * 8].view(np.uint32).reshape(total_rows // 2, 64, 2, 2)
    rows = np.ascontiguousarray(rows.transpose(0, 2, 1, 3)).reshape(total_rows, 64, 2)
    any_shared = int(buf[80:84].view(np.int32)[0])
    permuted = int(buf[84:88].view(np.int32)[0])
    o_perm = int(buf[152:160].view(np.uint64)[0])
    perm = buf[o_perm:o_perm + nchunks * THREADS * 2].view(np.uint16).reshape(nchunks, 8, 64)
    # where every stored value came from (flat ELL position), laid out like the rows / the P entries
    o_qsrc, o_psrc = int(buf[160:168].view(np.uint64)[0]), int(buf[168:176].view(np.uint64)[0])
    assert o_qsrc % 16 == 0 and o_psrc % 16 == 0 and o_pent + m * d * 8 <= o_qsrc and o_qsrc + total_rows * 64 * 4 <= o_psrc
    qsrc = buf[o_qsrc:o_qsrc + total_rows * 64 * 4].view(np.uint32).reshape(total_rows // 2, 64, 2)
    qsrc = np.ascontiguousarray(qsrc.transpose(0, 2, 1)).reshape(total_rows, 64)
    psrc = buf[o_psrc:o_psrc + m * d * 4].view(np.uint32)
    q_seen = np.zeros(n * d, dtype=bool)
    assert permuted == int(nslots == 1) and o_perm % 16 == 0
    if permuted:
        for c in range(nchunks):
            assert sorted(perm[c].reshape(-1).tolist()) == list(range(THREADS)), "every virtual column is walked by one thread"
    G = syn.storage_to_f64(pb.G, pb.dtype)
    T = np.zeros((m, r))
    nent = 0
    owners = {}
    for s in range(nslots):
        for w in range(8):
            for lane in range(64):
                c = int(vcol[s, w, lane])
                if c != 0xFFFF:
                    assert (c & 0x7FFF) < r
                    owners.setdefault(c & 0x7FFF, []).append(bool(c & 0x8000))
    assert sorted(owners) == list(range(r)), "every column has an owner"
    # the owners of a column sit side by side; the first one carries their number, the others 0
    o_vcnt = int(buf[144:152].view(np.uint64)[0])
    vcnt = buf[o_vcnt:o_vcnt + nslots * THREADS * 2].view(np.uint16)
    flat = vcol.reshape(-1)
    v = 0
    while v < flat.size:
        if flat[v] == 0xFFFF:
            assert vcnt[v] == 0
            v += 1
            continue
        k = int(vcnt[v])
        assert k == len(owners[int(flat[v]) & 0x7FFF]) and k >= 1
        assert all((int(flat[v + o]) & 0x7FFF) == (int(flat[v]) & 0x7FFF) and (o == 0 or vcnt[v + o] == 0) for o in range(k))
        v += k
    assert all(all(f) == (len(f) > 1) and (all(f) or not any(f)) for f in owners.values()), \
        "a column is flagged shared exactly when it has several owners"
    assert any_shared == int(any(len(f) > 1 for f in owners.values()))
    longest = np.zeros((nchunks, 8), dtype=np.int64)   # longest real list of each (chunk, wave), one slot
    for w in range(8):
        p = stream_row[w]
        for c in range(nchunks):
            for s in range(nslots):
                ln = int(seg[c, s, w])
                assert ln % BATCH == 0 and ln <= -(-cap // BATCH) * BATCH
                ent = rows[p:p + ln]
                for lane in range(64):
                    col = int(vcol[0].reshape(-1)[perm[c, w, lane]]) if permuted else int(vcol[s, w, lane])
                    for e in range(ln):
                        off = int(ent[e, lane, 0])
                        v = float(ent[e, lane, 1:2].view(np.float32)[0])
                        assert off % 16 == 0 and off <= PAD_OFFSET, "LDS offset inside one plane"
                        src = int(qsrc[p + e, lane])
                        if off == PAD_OFFSET:
                            assert v == 0.0 and src == 0xFFFFFFFF
                            continue
                        if nslots == 1:
                            longest[c, w] = max(longest[c, w], e + 1)
                        assert col != 0xFFFF
                        j = c * CHUNK + _decode_col(off)
                        assert j < n
                        assert src // d == j and not q_seen[src], "the pair's source is an entry of row j of Q, used once"
                        q_seen[src] = True
                        assert int(pb.Q_idx.reshape(-1)[src]) == (col & 0x7FFF) and np.float32(v) == pb.Q_val.reshape(-1)[src]
                        T[:, col & 0x7FFF] += v * G[:, j]
                        nent += 1
                p += ln
        # the kernel prefetches four batches past the end of the stream: harmless rows follow
        assert p + SLACK <= total_rows and (w == 7 or p + SLACK <= stream_row[w + 1])
        tail = rows[p:p + SLACK]
        assert np.all(tail[:, :, 0] == PAD_OFFSET) and np.all(tail[:, :, 1] == 0)
        assert np.all(qsrc[p:p + SLACK] == 0xFFFFFFFF)
    assert nent == n * d
    if permuted:
        # the lists of a chunk are dealt by length: waves 0,1,2,3,7,6,5,4 get ever shorter ones, and
        # no segment is padded by a whole batch
        dealt = longest[:, [0, 1, 2, 3, 7, 6, 5, 4]]
        assert np.all(np.diff(dealt, axis=1) <= 0)
        assert np.all(seg[:, 0, :] - longest < BATCH)
    items = buf[o_item:o_item + nitems * 16].view(np.int32).reshape(nitems, 4)
    pent = buf[o_pent:o_pent + m * d * 8].view(np.uint32).reshape(m * d, 2)
    S = np.zeros((r, r))
    seen = np.zeros(m * d, dtype=bool)
    rows_seen = set()
    for a, start, ln, atomic in items.tolist():
        rows_seen.add(a)
        assert 0 <= ln <= 256 and 0 <= a < r
        for e in range(start, start + ln):
            assert not seen[e]
            seen[e] = True
            i = int(pent[e, 0])
            v = float(pent[e, 1:2].view(np.float32)[0])
            assert i < m
            assert int(psrc[e]) // d == i and int(pb.P_idx.reshape(-1)[psrc[e]]) == a and np.float32(v) == pb.P_val.reshape(-1)[psrc[e]]
            S[a, :] += v * T[i, :]
        if atomic:
            assert any_split == 1
    assert seen.all() and rows_seen == set(range(r))
    assert q_seen.all() and sorted(psrc.tolist()) == list(range(m * d)), "every stored value has exactly one place in the plan"
    return T, S


def _dense(idx, val, r):
    D = np.zeros((idx.shape[0], r))
    for k in range(idx.shape[1]):
        np.add.at(D, (np.arange(idx.shape[0]), idx[:, k]), val[:, k].astype(np.float64))
    return D


@pytest.mark.parametrize("m,n,r,d,dist", [
    (48, 4200, 16, 2, "distinct"),      # three chunks, ragged last chunk
    (40, 2048, 64, 4, "uniform"),
    (33, 2500, 96, 8, "zipf"),          # hot columns get several owners; long rows of P^T are cut
    (2000, 64, 4, 2, "uniform"),        # every row of P^T has ~1000 entries -> pieces + atomic flag
    (24, 3000, 600, 2, "uniform"),      # more columns than lanes: two slots
    (10, 7, 3, 1, "uniform"),
])
def test_plan_replay_matches_dense_definition(m, n, r, d, dist):
    pb = syn.make_problem("t", m, n, r, d, "f32", seed=77 + m, g_std=1.0, index_dist=dist)
    buf = _build_host_plan(pb)
    T, S = _replay_plan(buf, pb)
    G = pb.G.astype(np.float64)
    Ph, Qh = _dense(pb.P_idx, pb.P_val, r), _dense(pb.Q_idx, pb.Q_val, r)
    np.testing.assert_allclose(T, G @ Qh, rtol=0, atol=1e-11 * max(1.0, np.abs(G @ Qh).max()))
    ref = Ph.T @ G @ Qh
    np.testing.assert_allclose(S, ref, rtol=0, atol=1e-10 * max(1.0, np.abs(ref).max()))


def test_plan_build_host_rejects_bad_index_and_small_buffer():
    pb = syn.make_problem("t", 16, 16, 8, 2, "f32", seed=5)
    nbytes = L.lsp_plan_bytes(16, 16, 8, 2)
    buf = np.zeros(nbytes, dtype=np.uint8)
    bad = pb.Q_idx.copy()
    bad[3, 1] = 8
    assert L.lsp_plan_build_host(pb.P_idx, pb.P_val, bad, pb.Q_val, 16, 16, 8, 2, buf, nbytes, check=False) == -6
    bad[3, 1] = -1
    assert L.lsp_plan_build_host(pb.P_idx, pb.P_val, bad, pb.Q_val, 16, 16, 8, 2, buf, nbytes, check=False) == -6
    assert L.lsp_plan_build_host(pb.P_idx, pb.P_val, pb.Q_idx, pb.Q_val, 16, 16, 8, 2, buf, nbytes - 1,
                                 check=False) == -4


def test_plan_build_reports_unplannable_skew():
    # r = 2048 uniformly used columns already fill all 4 x 512 lanes; one hot column on top of
    # that needs extra owners that do not exist -> LSP_ERR_SKEW (the caller falls back to lsp_compress)
    m, n, r, d = 8, 2048, 2048, 16
    rng = np.random.default_rng(3)
    P_idx, P_val = syn.ell_projector(m, r, d, rng)
    Q_idx, Q_val = syn.ell_projector(n, r, d, rng, "distinct")
    nbytes = L.lsp_plan_bytes(m, n, r, d)
    buf = np.zeros(nbytes, dtype=np.uint8)
    assert L.lsp_plan_build_host(P_idx, P_val, Q_idx, Q_val, m, n, r, d, buf, nbytes, check=False) == 0
    Q_idx[:, 0] = 0                      # every row of Q also hits column 0
    assert L.lsp_plan_build_host(P_idx, P_val, Q_idx, Q_val, m, n, r, d, buf, nbytes, check=False) == -8
    assert "unevenly" in L.lsp_strerror(-8)


# ------------------------------------------------------------------ entry order inside projector rows
def _gather_cost(idx):
    """Modelled cycles of the decompress kernels' 128-bit LDS gathers: lane l of a wave owns columns 2l, 2l+1 of a
    128-column tile; a gather (one entry slot of one of the two columns) is served in four groups of 16 lanes
    (lane >= 32, parity of lane bits 2..4), each costing its most used bank group (index mod 16)."""
    groups = [[l for l in range(64) if ((l >= 32) * 2 + (bin((l % 32) // 4).count("1") & 1)) == g] for g in range(4)]
    n, d = idx.shape
    total, steps = 0, 0
    for tile in range(0, n - 127, 128):
        for c in (0, 1):
            for k in range(d):
                total += sum(np.bincount([int(idx[tile + 2 * l + c, k]) % 16 for l in g], minlength=16).max() for g in groups)
                steps += 1
    return total / steps


@pytest.mark.parametrize("rows,r,d,dist", [(1024, 512, 8, "uniform"), (640, 256, 4, "uniform"), (300, 96, 16, "zipf"), (5, 3, 2, "uniform")])
def test_projector_reorder_keeps_the_matrix_and_spreads_the_banks(rows, r, d, dist):
    rng = np.random.default_rng(31 + rows)
    idx, val = syn.ell_projector(rows, r, d, rng, dist)
    oi, ov = np.full_like(idx, -1), np.zeros_like(val)
    L.lsp_projector_reorder_host(idx, val, rows, d, r, oi, ov)
    # every row keeps its (index, value) pairs, as a multiset
    for i in range(rows):
        assert sorted(zip(idx[i].tolist(), val[i].tolist())) == sorted(zip(oi[i].tolist(), ov[i].tolist()))
    if rows >= 128:
        before, after = _gather_cost(idx), _gather_cost(oi)
        assert after <= before
        if dist == "uniform" and d >= 4:
            assert after < 0.85 * before, (before, after)
    # argument errors
    assert L.lsp_projector_reorder_host(idx, val, rows, d, r, idx, ov, check=False) == -2      # in place is refused
    assert L.lsp_projector_reorder_host(None, val, rows, d, r, oi, ov, check=False) == -1
    assert L.lsp_projector_reorder(None, 0x1000, rows, d, r, 0x2000, 0x3000, None, check=False) == -1     # checked before any HIP call
    assert L.lsp_projector_reorder(0x1000, 0x1000, rows, r + 1, r, 0x2000, 0x3000, None, check=False) == -2
    bad = idx.copy(); bad[0, 0] = r
    assert L.lsp_projector_reorder_host(bad, val, rows, d, r, oi, ov, check=False) == -6


def test_dense_compress_refuses_other_shapes_and_types():
    fake = 4096
    assert L.lsp_compress_dense_workspace_bytes(100, 64, 128) == 0
    assert L.lsp_compress_dense(fake, fake, fake, 100, 64, 128, fake, 2, fake, 1 << 30, None, check=False) == -2
    assert L.lsp_compress_dense(fake, fake, fake, 128, 64, 128, fake, 0, fake, 1 << 30, None, check=False) == -3
    assert L.lsp_compress_dense(fake, fake, fake, 128, 64, 128, fake, 2, fake, 16, None, check=False) == -4
    assert L.lsp_compress_dense(None, fake, fake, 128, 64, 128, fake, 2, fake, 1 << 30, None, check=False) == -1
