"""Pins for the oracle's high-throughput-mode additions (CPU only): group
dedup, the per-expert index list, and the two-level (hierarchical) reduce."""
import numpy as np
import pytest

import ep_inputs as g


def _ht(oracle, cfg, G, T=None, mask=0.0):
    idx, w = g.routing_all(cfg, T)
    if mask:
        idx = g.mask_random(idx, mask, seed=41)
    gidx, fk = oracle.dedup(idx, cfg.E_loc, G)
    ngroups = cfg.R // G
    lay = oracle.layout(idx, cfg.E, cfg.R)
    lay_g = oracle.layout(gidx, ngroups, ngroups)
    return idx, w, gidx, fk, lay, lay_g, ngroups


@pytest.mark.parametrize("cid,G,T,mask", [(1, 1, None, 0.0), (1, 2, None, 0.3), (4, 1, 200, 0.0), (4, 8, 200, 0.1),
                                          (2, 8, 32, 0.0), (5, 2, 150, 0.0)])
def test_dedup_brute_force(oracle, cid, G, T, mask):
    cfg = g.config(cid)
    idx, w, gidx, fk, lay, lay_g, ngroups = _ht(oracle, cfg, G, T, mask)
    S, T_, K = idx.shape
    grp = np.where(idx >= 0, (idx // cfg.E_loc) // G, -1)
    for s in range(S):
        for t in range(T_):
            seen = {}
            for k in range(K):
                gg = grp[s, t, k]
                if gg < 0:
                    assert gidx[s, t, k] == -1 and fk[s, t, k] == -1
                    continue
                if gg not in seen:
                    seen[gg] = k
                    assert gidx[s, t, k] == gg
                else:
                    assert gidx[s, t, k] == -1
                assert fk[s, t, k] == seen[gg]
            # library pin: the kept groups are exactly the distinct groups of the token
            assert sorted(gidx[s, t][gidx[s, t] >= 0].tolist()) == np.unique(grp[s, t][grp[s, t] >= 0]).tolist()
    # one receive row per distinct (source, token, group)
    pairs = {(s, t, int(gg)) for s in range(S) for t in range(T_) for gg in grp[s, t] if gg >= 0}
    assert int(lay_g["expert_offset"][-1]) == len(pairs)
    assert int((gidx >= 0).sum()) == len(pairs)


def test_dedup_special_cases(oracle):
    idx = np.array([[[0, 1, 2, 3], [5, 4, 5 - 5, 7], [-1, 6, -1, 6 + 1]]], np.int32)   # E_loc = 2, 4 ranks
    gidx, fk = oracle.dedup(idx, 2, 1)
    assert gidx[0].tolist() == [[0, -1, 1, -1], [2, -1, 0, 3], [-1, 3, -1, -1]]
    assert fk[0].tolist() == [[0, 0, 2, 2], [0, 0, 2, 3], [-1, 1, -1, 1]]
    gidx2, fk2 = oracle.dedup(idx, 2, 4)                       # all ranks in one group: one copy per token
    assert (gidx2[0] >= 0).sum(axis=1).tolist() == [1, 1, 1]
    assert fk2[0].tolist() == [[0, 0, 0, 0], [0, 0, 0, 0], [-1, 1, -1, 1]]
    # every expert its own group (E_loc = 1, G = 1): nothing is removed
    gidx3, fk3 = oracle.dedup(idx, 1, 1)
    assert np.array_equal(gidx3, idx) and (fk3[idx >= 0] == np.broadcast_to(np.arange(4), idx.shape)[idx >= 0]).all()


@pytest.mark.parametrize("cid,G", [(1, 1), (4, 1), (4, 8), (5, 2)])
def test_index_list_reproduces_the_plain_dispatch(oracle, cid, G):
    """Expert inputs read through the index list from the deduplicated buffer
    equal the receive buffer of the ordinary dispatch, row for row."""
    cfg = g.config(cid, S=1)
    T = min(cfg.T, 120)
    idx, w, gidx, fk, lay, lay_g, ngroups = _ht(oracle, cfg, G, T, 0.1)
    x = g.activations(cfg, 0, T=T)
    rows = int((idx >= 0).sum())
    rows_g = int((gidx >= 0).sum())
    recv, _ = oracle.dispatch_bf16(x, idx[0], lay["dst_row"][0], cfg.E_loc, rows)
    recv_g, wc = oracle.dispatch_bf16(x, gidx[0], lay_g["dst_row"][0], 1, rows_g)
    assert (wc == 1).all() and rows_g <= rows
    index = oracle.gather_index(lay["dst_row"][0], lay_g["dst_row"][0], fk[0], rows)
    assert (index >= 0).all() and index.max() < rows_g
    assert np.array_equal(recv_g[index], recv)
    # rows of one group are contiguous and in token order: the index list of an expert is increasing
    for e in range(cfg.E):
        seg = index[lay["expert_offset"][e]:lay["expert_offset"][e + 1]]
        assert (np.diff(seg) > 0).all()
        grp = (e // cfg.E_loc) // G
        assert ((seg >= lay_g["expert_offset"][grp]) & (seg < lay_g["expert_offset"][grp + 1])).all()


@pytest.mark.parametrize("cid,G,mask", [(1, 1, 0.0), (1, 2, 0.25), (4, 1, 0.0), (4, 8, 0.0), (5, 4, 0.1)])
def test_hierarchical_reduce_against_the_fp64_definition(oracle, cid, G, mask):
    cfg = g.config(cid, S=1)
    T = min(cfg.T, 48)
    idx, w, gidx, fk, lay, lay_g, ngroups = _ht(oracle, cfg, G, T, mask)
    rows = max(1, int((idx >= 0).sum()))
    rows_g = int((gidx >= 0).sum())
    y = g.activations(cfg, 0, tid=g.TID_Y, T=rows)
    dr, drg = lay["dst_row"][0], lay_g["dst_row"][0]
    partial = oracle.combine_partial(y, w[0], dr, fk[0], drg, rows_g)
    ones = np.ones_like(w[0])
    out = oracle.combine(partial, ones, drg)
    # partial rows by definition, in fp64, from an independent gather
    yf = g.bf16_bits_to_f32(y).astype(np.float64)
    pf = g.bf16_bits_to_f32(partial).astype(np.float64)
    ref_total, mag = oracle.combine_f64(y, w[0], dr)
    for t in range(T):
        for j in range(cfg.K):
            if fk[0, t, j] != j:
                continue
            members = [k for k in range(cfg.K) if fk[0, t, k] == j]
            ref = sum(float(w[0, t, k]) * yf[dr[t, k]] for k in members)
            m = sum(abs(float(w[0, t, k])) * np.abs(yf[dr[t, k]]) for k in members)
            bound = 2.0 ** -8 * np.abs(ref) + len(members) * 2.0 ** -24 * m * 1.01 + 2.0 ** -133
            assert (np.abs(pf[drg[t, j]] - ref) <= bound).all()
    # two-level result vs the flat fp64 sum: one bf16 rounding per group, one at the end
    got = g.bf16_bits_to_f32(out).astype(np.float64)
    ngr = (gidx[0] >= 0).sum(axis=1)[:, None]
    bound = 2.0 ** -8 * np.abs(ref_total) + (ngr + 1) * 2.0 ** -8 * mag * 1.01 + 2.0 ** -133
    assert (np.abs(got - ref_total) <= bound).all()
    # and the second level is exactly the ordinary combine of the partial rows
    ref2 = np.where((drg >= 0)[..., None], pf[np.maximum(drg, 0)], 0.0).sum(axis=1)
    assert (np.abs(got - ref2) <= 2.0 ** -8 * np.abs(ref2) * 1.001 + cfg.K * 2.0 ** -24 * np.abs(
        np.where((drg >= 0)[..., None], pf[np.maximum(drg, 0)], 0.0)).sum(axis=1) + 2.0 ** -133).all()


def test_hierarchical_reduce_degenerate_cases(oracle):
    cfg = g.config(1, S=1)
    idx, w = g.routing_all(cfg)
    y = g.activations(cfg, 0, tid=g.TID_Y, T=idx.size)
    lay = oracle.layout(idx, cfg.E, cfg.R)
    flat = oracle.combine(y, w[0], lay["dst_row"][0])
    # one group holds every rank: the single partial IS the flat combine, the second level adds nothing
    gidx, fk = oracle.dedup(idx, cfg.E_loc, cfg.R)
    lay_g = oracle.layout(gidx, 1, 1)
    partial = oracle.combine_partial(y, w[0], lay["dst_row"][0], fk[0], lay_g["dst_row"][0], cfg.T)
    assert np.array_equal(partial[lay_g["dst_row"][0][:, 0]], flat)
    assert np.array_equal(oracle.combine(partial, np.ones_like(w[0]), lay_g["dst_row"][0]), flat)
    # every expert its own group: each partial row is bf16(w_k * y_k)
    gidx, fk = oracle.dedup(idx, 1, 1)
    lay_g = oracle.layout(gidx, cfg.E, cfg.E)
    partial = oracle.combine_partial(y, w[0], lay["dst_row"][0], fk[0], lay_g["dst_row"][0], idx.size)
    yf = g.bf16_bits_to_f32(y)
    for t in range(0, cfg.T, 5):
        for k in range(cfg.K):
            want = g.f32_to_bf16_bits((np.float32(w[0, t, k]) * yf[lay["dst_row"][0, t, k]]).astype(np.float32))
            assert np.array_equal(partial[lay_g["dst_row"][0, t, k]], want)
