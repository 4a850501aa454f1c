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
CHUNK = 1024
PAD_OFFSET = CHUNK * 16


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
    assert "NULL" in L.lsp_strerror(-1) and L.lsp_strerror(0) == "ok"
    with pytest.raises(L.LspError):
        L.lsp_compress(None, fake, fake, fake, fake, 64, 64, 16, 2, fake, 0, fake, big)


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
    """What the plan means: T = G Qhat from the Q section, then S = Phat^T T from the P section."""
    hdr32 = buf[:64].view(np.int32)
    assert hdr32[0] == 0x4C535031
    m, n, r, d, nchunks, total_rounds, nitems, any_split = [int(x) for x in hdr32[1:9]]
    assert (m, n, r, d) == (pb.m, pb.n, pb.r, pb.d) and nchunks == -(-n // CHUNK)
    offs = buf[64:64 + 56].view(np.uint64)
    o_chunk, o_round, o_cols, o_ent, o_item, o_pent, total = [int(x) for x in offs]
    assert total == buf.size and all(o % 16 == 0 for o in (o_chunk, o_round, o_cols, o_ent, o_item, o_pent))
    chunks = buf[o_chunk:o_chunk + nchunks * 8].view(np.int32).reshape(nchunks, 2)
    rounds = buf[o_round:o_round + total_rounds * 8].view(np.uint32).reshape(total_rounds, 2)
    cols = buf[o_cols:o_cols + total_rounds * 64 * 2].view(np.uint16).reshape(total_rounds, 64)
    G = syn.storage_to_f64(pb.G, pb.dtype)
    T = np.zeros((m, r))
    used_slots = 0
    nent = 0
    for c in range(nchunks):
        first, nr = int(chunks[c, 0]), int(chunks[c, 1])
        prev_len = None
        for rho in range(first, first + nr):
            eo, ln = int(rounds[rho, 0]), int(rounds[rho, 1])
            assert eo == used_slots, "rounds must be packed back to back"
            assert prev_len is None or ln <= prev_len, "rounds of a chunk are sorted by length"
            prev_len = ln
            assert 1 <= ln <= 64
            ent = buf[o_ent + eo * 8:o_ent + (eo + ln * 64) * 8].view(np.uint32).reshape(ln, 64, 2)
            used_slots += ln * 64
            for lane in range(64):
                b = int(cols[rho, lane])
                if b != 0xFFFF:
                    b &= 0x7FFF                       # bit 15 marks a piece of a cut list
                for e in range(ln):
                    off, vb = int(ent[e, lane, 0]), ent[e, lane, 1:2]
                    v = float(vb.view(np.float32)[0])
                    assert off % 16 == 0 and off <= PAD_OFFSET, "LDS offset inside one plane"
                    if off == PAD_OFFSET:
                        assert v == 0.0
                        continue
                    assert b != 0xFFFF and b < r
                    j = c * CHUNK + _decode_col(off)
                    assert j < n
                    T[:, b] += v * G[:, j]
                    nent += 1
    assert nent == n * d
    max_slots_bytes = o_item - o_ent
    assert used_slots * 8 <= max_slots_bytes
    items = buf[o_item:o_item + nitems * 16].view(np.int32).reshape(nitems, 4)
    pent = buf[o_pent:o_pent + m * d * 8].view(np.uint32).reshape(m * d, 2)
    S = np.zeros((r, r))
    seen = np.zeros(m * d, dtype=bool)
    rows_seen = set()
    for a, start, ln, atomic in items.tolist():
        rows_seen.add(a)
        assert 0 <= ln <= 128 and 0 <= a < r
        for e in range(start, start + ln):
            assert not seen[e]
            seen[e] = True
            i = int(pent[e, 0])
            v = float(pent[e, 1:2].view(np.float32)[0])
            assert i < m
            S[a, :] += v * T[i, :]
        if atomic:
            assert any_split == 1
    assert seen.all() and rows_seen == set(range(r))
    return T, S


def _dense(idx, val, r):
    D = np.zeros((idx.shape[0], r))
    for k in range(idx.shape[1]):
        np.add.at(D, (np.arange(idx.shape[0]), idx[:, k]), val[:, k].astype(np.float64))
    return D


@pytest.mark.parametrize("m,n,r,d,dist", [
    (48, 2100, 16, 2, "distinct"),      # three chunks, ragged last chunk
    (40, 1024, 64, 4, "uniform"),
    (33, 1500, 8, 8, "zipf"),           # lists longer than 64 -> cut into pieces; rows of P^T > 128
    (2000, 64, 4, 2, "uniform"),        # every row of P^T has ~1000 entries -> pieces + atomic flag
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
