"""Pins for the CPU oracle: every function of oracle/dag_oracle.py is checked against something
other than itself -- hand-enumerated fixtures, closed forms, library routines (torch fp64
scaled_dot_product_attention) and invariants -- so that a dropped term, a wrong sign or index, or a
transposed operand fails at least one test.  No GPU needed.
"""
import json
import os

import numpy as np
import pytest
import torch

from oracle import dag_oracle as orc
from workloads import dags

GOLDEN = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "tiny_dags.json")))


def _dag_from_parents(node_len, parents):
    return (np.asarray(node_len, dtype=np.int32),
            dags.bits_from_sets(dags.closure_from_parents(parents)))


def _rand(seed, *shape):
    return np.random.Generator(np.random.PCG64(seed)).standard_normal(shape)


def _sdpa_causal(q, k, v, scale):
    """Library routine: fp64 causal attention. q [T][H][D], k/v [T][H][D] (same head count)."""
    tq = torch.from_numpy(q).permute(1, 0, 2)[None]
    tk = torch.from_numpy(k).permute(1, 0, 2)[None]
    tv = torch.from_numpy(v).permute(1, 0, 2)[None]
    o = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, is_causal=True, scale=scale)
    return o[0].permute(1, 0, 2).numpy()


# ------------------------------------------------------------------ positions (section 4.2)
def test_positions_diamond_golden():
    g = GOLDEN["diamond"]
    L, anc = _dag_from_parents(g["node_len"], g["parents"])
    tok_node, pos = orc.token_meta(L, anc)
    assert tok_node.tolist() == g["tok_node"]
    assert pos.tolist() == g["pos_ids"]


def test_positions_config1_statement():
    g = GOLDEN["config1_positions"]
    L, anc = dags.fork_join(g["prefix"], [g["branch"]] * g["n_branch"], g["join"])
    tok_start, pos_start = orc.node_tables(L, anc)
    assert pos_start[0] == 0
    assert all(pos_start[1 + b] == g["branch_start"] for b in range(g["n_branch"]))
    assert pos_start[-1] == g["join_start"]
    _, pos = orc.token_meta(L, anc)
    assert pos[:128].tolist() == list(range(128))
    assert pos[-64:].tolist() == list(range(192, 256))


@pytest.mark.parametrize("lens", [[5, 3, 9, 1], [7, 7, 7], [1, 20, 4, 4, 2]])
def test_positions_fork_join_closed_form(lens):
    prefix, branches, join = lens[0], lens[1:-1], lens[-1]
    L, anc = dags.fork_join(prefix, branches, join)
    _, pos_start = orc.node_tables(L, anc)
    assert all(pos_start[1 + b] == prefix for b in range(len(branches)))
    assert pos_start[-1] == prefix + max(branches)


def test_positions_linear_chain_is_arange():
    L, anc = dags.linear_chain([3, 1, 5, 2, 8])
    tok_node, pos = orc.token_meta(L, anc)
    assert pos.tolist() == list(range(19))
    assert tok_node.tolist() == [0] * 3 + [1] + [2] * 5 + [3] * 2 + [4] * 8


def test_skip_level_discriminates_the_two_mask_readings():
    g = GOLDEN["skip_level"]
    L, anc = _dag_from_parents(g["node_len"], g["parents"])
    _, pos = orc.token_meta(L, anc)
    m = orc.explicit_mask(L, anc)
    assert np.flatnonzero(m[5]).tolist() == g["ancestor_reading"]["row_of_D"]
    assert pos.tolist() == g["ancestor_reading"]["pos_ids"]
    anc_layer = dags.layerwise_bits(g["levels"])
    _, pos2 = orc.token_meta(L, anc_layer)
    m2 = orc.explicit_mask(L, anc_layer)
    assert np.flatnonzero(m2[5]).tolist() == g["layer_reading"]["row_of_D"]
    assert pos2.tolist() == g["layer_reading"]["pos_ids"]
    # literal Eq. 3 on the layer reading: masked iff j > i, or same layer and different step
    lev = np.repeat(g["levels"], g["node_len"])
    node = np.repeat(np.arange(4), g["node_len"])
    for i in range(6):
        for j in range(6):
            masked = (j > i) or (lev[i] == lev[j] and node[i] != node[j])
            assert m2[i, j] == (not masked)


# ------------------------------------------------------------------ mask (Eq. 3)
def test_mask_diamond_golden():
    g = GOLDEN["diamond"]
    L, anc = _dag_from_parents(g["node_len"], g["parents"])
    m = orc.explicit_mask(L, anc)
    for i, allowed in enumerate(g["allowed"]):
        assert np.flatnonzero(m[i]).tolist() == allowed
    assert orc.useful_pairs(L, anc) == g["useful_pairs"]


def _closed_form_pairs(L, anc):
    sets = dags.sets_from_bits(anc)
    total = 0
    for v, lv in enumerate(L):
        total += int(lv) * sum(int(L[u]) for u in sets[v] if u != v) + int(lv) * (int(lv) + 1) // 2
    return total


def test_mask_counts_closed_form():
    L, anc = dags.fork_join(128, [64] * 4, 64)
    assert orc.useful_pairs(L, anc) == 76000 == _closed_form_pairs(L, anc)
    L, anc = dags.fork_join(2048, [256] * 8, 512)
    assert orc.useful_pairs(L, anc) == 8784128 == _closed_form_pairs(L, anc)
    rng = np.random.Generator(np.random.PCG64(7))
    L, anc, _, _ = dags.random_dag(rng, n_nodes=20, depth=4, len_lo=1, len_hi=9)
    assert orc.useful_pairs(L, anc) == _closed_form_pairs(L, anc)


def test_mask_linear_chain_is_lower_triangular():
    L, anc = dags.linear_chain([4, 1, 6])
    assert np.array_equal(orc.explicit_mask(L, anc), np.tril(np.ones((11, 11), dtype=bool)))


def test_mask_rows_have_self_and_no_future():
    rng = np.random.Generator(np.random.PCG64(11))
    L, anc, _, _ = dags.random_dag(rng, n_nodes=30, depth=5, len_lo=1, len_hi=7)
    m = orc.explicit_mask(L, anc)
    assert m.diagonal().all()
    assert not np.triu(m, 1).any()


# ------------------------------------------------------------------ block map
def test_block_map_diamond_golden():
    g = GOLDEN["diamond"]
    L, anc = _dag_from_parents(g["node_len"], g["parents"])
    bm = orc.block_map(L, anc, *g["tile"])
    assert bm.tolist() == g["block_map"]
    rp, col, flag = orc.block_map_csr(bm)
    assert rp.tolist() == [0, 1, 3, 6, 10]
    assert col.tolist() == [0, 0, 1, 0, 1, 2, 0, 1, 2, 3]
    assert flag.tolist() == [1, 2, 1, 2, 1, 1, 2, 2, 2, 2]


def test_block_map_config2_census():
    # 128x128 tiles: prefix 16 tiles, 8 branches of 2 tiles, join 4 tiles (36 tiles a side).
    # By hand: FULL = prefix below-diagonal 120 + branches x prefix 256 + in-branch 8
    #                 + join x (prefix+branches) 128 + in-join 6 = 518; PARTIAL = 36 diagonal tiles.
    L, anc = dags.fork_join(2048, [256] * 8, 512)
    bm = orc.block_map(L, anc, 128, 128)
    assert bm.shape == (36, 36)
    assert int((bm == orc.FULL).sum()) == 518
    assert int((bm == orc.PARTIAL).sum()) == 36
    assert 518 * 16384 + 36 * 8256 == 8784128


def test_block_map_consistent_with_mask_on_ragged_random_dag():
    rng = np.random.Generator(np.random.PCG64(5))
    L, anc, _, _ = dags.random_dag(rng, n_nodes=12, depth=4, len_lo=1, len_hi=11)
    m = orc.explicit_mask(L, anc)
    T = m.shape[0]
    for tm, tn in [(4, 8), (8, 4), (5, 3)]:
        bm = orc.block_map(L, anc, tm, tn)
        cover = np.zeros_like(m)
        for a in range(bm.shape[0]):
            for b in range(bm.shape[1]):
                sub = m[a * tm:(a + 1) * tm, b * tn:(b + 1) * tn]
                if bm[a, b] == orc.FULL:
                    assert sub.all()
                    cover[a * tm:(a + 1) * tm, b * tn:(b + 1) * tn] = True
                elif bm[a, b] == orc.SKIP:
                    assert not sub.any()
                else:
                    assert sub.any() and not sub.all()
                    cover[a * tm:(a + 1) * tm, b * tn:(b + 1) * tn] = True
        assert not (m & ~cover).any()
        assert bm.shape == (-(-T // tm), -(-T // tn))


def test_full_first_csr_and_launch_tables_golden():
    """The FULL-first row order, the FULL counts, the launch order and the mask-free counts against
    values enumerated by hand (the diamond, and a DAG whose row of D lists a PARTIAL tile in front
    of a FULL one, so that the two row orders differ)."""
    for name in ("diamond", "partial_before_full"):
        g = GOLDEN[name]
        L, anc = _dag_from_parents(g["node_len"], g["parents"])
        tok_node, pos = orc.token_meta(L, anc)
        assert tok_node.tolist() == g["tok_node"] and pos.tolist() == g["pos_ids"]
        m = orc.explicit_mask(L, anc)
        assert [np.nonzero(r)[0].tolist() for r in m] == g["allowed"]
        assert orc.useful_pairs(L, anc) == g["useful_pairs"]
        bm = orc.block_map(L, anc, *g["tile"])
        assert bm.tolist() == g["block_map"]
        want = g["csr_full_first"]
        rp, col, flag, nfull = orc.block_map_csr_full_first(bm)
        assert rp.tolist() == want["rowptr"] and col.tolist() == want["col"]
        assert flag.tolist() == want["flag"] and nfull.tolist() == want["nfull"]
        order, mask_free = orc.launch_tables([bm], [int(np.sum(L))], g["tile"][1])
        assert order.tolist() == want["launch_order"] and mask_free.tolist() == want["mask_free"]
    asc = GOLDEN["partial_before_full"]["csr_ascending"]
    L, anc = _dag_from_parents(GOLDEN["partial_before_full"]["node_len"], GOLDEN["partial_before_full"]["parents"])
    rp, col, flag = orc.block_map_csr(orc.block_map(L, anc, 2, 2))
    assert rp.tolist() == asc["rowptr"] and col.tolist() == asc["col"] and flag.tolist() == asc["flag"]


def test_full_first_csr_properties_on_ragged_random_dags():
    """Same multiset per row as the ascending CSR, FULL before PARTIAL, each group ascending, flags
    equal to the dense map; launch order = a permutation sorted by tile count; mask-free counts by
    brute force over the explicit mask (a tile counts iff all tile_m x tile_n pairs exist and are
    visible)."""
    rng = np.random.Generator(np.random.PCG64(17))
    for tm, tn in [(4, 8), (8, 4), (5, 3), (6, 6)]:
        dag_list = [dags.random_dag(rng, n_nodes=14, depth=4, len_lo=1, len_hi=11)[:2] for _ in range(3)]
        bmaps, Ts, all_counts, brute_free = [], [], [], []
        for L, anc in dag_list:
            bm = orc.block_map(L, anc, tm, tn)
            m = orc.explicit_mask(L, anc)
            T = m.shape[0]
            rp, col, flag = orc.block_map_csr(bm)
            rp2, col2, flag2, nfull = orc.block_map_csr_full_first(bm)
            assert rp.tolist() == rp2.tolist()
            for a in range(bm.shape[0]):
                c, f = col2[rp2[a]:rp2[a + 1]], flag2[rp2[a]:rp2[a + 1]]
                assert sorted(c.tolist()) == col[rp[a]:rp[a + 1]].tolist()
                nf = int(nfull[a])
                assert (f[:nf] == orc.FULL).all() and (f[nf:] == orc.PARTIAL).all()
                assert (np.diff(c[:nf]) > 0).all() and (np.diff(c[nf:]) > 0).all()
                assert all(bm[a, b] == x for b, x in zip(c, f))
                all_counts.append(len(c))
                rows = m[a * tm:(a + 1) * tm]
                brute_free.append(sum(1 for b in range(bm.shape[1]) if (b + 1) * tn <= T and
                                      rows[:, b * tn:(b + 1) * tn].all()))
            bmaps.append(bm)
            Ts.append(T)
        order, mask_free = orc.launch_tables(bmaps, Ts, tn)
        assert sorted(order.tolist()) == list(range(len(all_counts)))
        keys = [(-all_counts[i], i) for i in order]
        assert keys == sorted(keys)
        assert mask_free.tolist() == brute_free


# ------------------------------------------------------------------ rotary embedding
def test_rope_closed_forms():
    # D = 2: one pair, frequency 1: (1, 0) at position p -> (cos p, sin p); (0, 1) -> (-sin p, cos p)
    for p in [0, 1, 5, 1000]:
        out = orc.rope(np.array([[[1.0, 0.0]], [[0.0, 1.0]]]), [p, p], 10000.0)
        assert np.allclose(out[0, 0], [np.cos(p), np.sin(p)], atol=1e-12)
        assert np.allclose(out[1, 0], [-np.sin(p), np.cos(p)], atol=1e-12)
    # D = 4, theta = 10000: pair m = 1 is (x[1], x[3]) and rotates at frequency 10000^(-1/2) = 0.01
    x = np.zeros((1, 1, 4))
    x[0, 0, 1] = 1.0
    out = orc.rope(x, [7], 10000.0)
    assert np.allclose(out[0, 0], [0.0, np.cos(0.07), 0.0, np.sin(0.07)], atol=1e-12)
    # D = 8, theta = 16: frequencies 16^(-m/4) = 1, 1/2, 1/4, 1/8
    x = np.zeros((1, 1, 8))
    x[0, 0, 7] = 2.0                          # second element of pair m = 3
    out = orc.rope(x, [4], 16.0)
    assert np.allclose(out[0, 0, 3], -2.0 * np.sin(0.5), atol=1e-12)
    assert np.allclose(out[0, 0, 7], 2.0 * np.cos(0.5), atol=1e-12)


def test_rope_identity_norm_and_relative_property():
    x = _rand(1, 6, 3, 16)
    assert np.allclose(orc.rope(x, np.zeros(6), 1e4), x)
    pos = np.array([0, 3, 17, 17, 250, 40000])
    y = orc.rope(x, pos, 5e5)
    assert np.allclose((y ** 2).sum(-1), (x ** 2).sum(-1), rtol=1e-12)
    # <rope(a, p1), rope(b, p2)> depends only on p1 - p2
    a, b = _rand(2, 1, 1, 16), _rand(3, 1, 1, 16)
    d1 = (orc.rope(a, [10], 1e4) * orc.rope(b, [3], 1e4)).sum()
    d2 = (orc.rope(a, [1010], 1e4) * orc.rope(b, [1003], 1e4)).sum()
    assert abs(d1 - d2) < 1e-9


# ------------------------------------------------------------------ attention values
def test_linear_chain_equals_library_causal_attention():
    T, H, D = 37, 3, 16
    L, anc = dags.linear_chain([10, 1, 20, 6])
    q, k, v = _rand(4, T, H, D), _rand(5, T, H, D), _rand(6, T, H, D)
    scale = 0.3
    O, lse = orc.attn_prefill(q, k, v, L, anc, scale=scale, row_block=8)
    ref = _sdpa_causal(q, k, v, scale)
    assert np.abs(O - ref).max() < 1e-12
    # lse against the definition log sum exp over the visible prefix
    s = (q[20, 1] @ k[:21, 1].T) * scale
    assert abs(lse[20, 1] - np.log(np.exp(s).sum())) < 1e-12


def test_gqa_head_mapping_against_library():
    T, Hq, Hkv, D = 19, 6, 2, 8
    L, anc = dags.linear_chain([19])
    q, k, v = _rand(7, T, Hq, D), _rand(8, T, Hkv, D), _rand(9, T, Hkv, D)
    O, _ = orc.attn_prefill(q, k, v, L, anc)
    kk = np.repeat(k, Hq // Hkv, axis=1)          # query head h -> kv head h // G
    vv = np.repeat(v, Hq // Hkv, axis=1)
    assert np.abs(O - _sdpa_causal(q, kk, vv, 1.0 / np.sqrt(D))).max() < 1e-12


def test_fork_join_equals_causal_attention_on_each_path():
    """Fork: a branch inherits exactly the prefix context (sections 3.3, 4.3); a branch token's
    output equals plain causal attention with ordinary positions over [prefix, that branch].
    Join: sees prefix and all branches; equals causal attention over the whole concatenation with
    the adaptive rotation applied beforehand."""
    prefix, branches, join = 9, [5, 7, 3], 4
    L, anc = dags.fork_join(prefix, branches, join)
    T, H, D, theta = int(L.sum()), 2, 8, 100.0
    q, k, v = _rand(10, T, H, D), _rand(11, T, H, D), _rand(12, T, H, D)
    _, pos = orc.token_meta(L, anc)
    qr, kr = orc.rope(q, pos, theta), orc.rope(k, pos, theta)
    O, _ = orc.attn_prefill(qr, kr, v, L, anc)
    scale = 1.0 / np.sqrt(D)
    start = prefix
    for bl in branches:
        idx = np.r_[0:prefix, start:start + bl]
        ordinary = np.arange(len(idx))
        ref = _sdpa_causal(orc.rope(q[idx], ordinary, theta), orc.rope(k[idx], ordinary, theta),
                           v[idx], scale)
        assert np.abs(O[idx] - ref).max() < 1e-12
        start += bl
    ref = _sdpa_causal(qr, kr, v, scale)
    assert np.abs(O[-join:] - ref[-join:]).max() < 1e-12
    # and the branches really are isolated: a middle-branch token differs from full causal
    assert np.abs(O[prefix + branches[0] + 1] - ref[prefix + branches[0] + 1]).max() > 1e-6


def test_sibling_order_permutation_invariance():
    prefix, branches, join = 6, [4, 7, 2], 5
    L, anc = dags.fork_join(prefix, branches, join)
    T, H, D, theta = int(L.sum()), 2, 8, 1e4
    q, k, v = _rand(13, T, H, D), _rand(14, T, H, D), _rand(15, T, H, D)
    _, pos = orc.token_meta(L, anc)
    O, _ = orc.attn_prefill(orc.rope(q, pos, theta), orc.rope(k, pos, theta), v, L, anc)
    order = [2, 0, 1]
    starts = np.cumsum([prefix] + branches)
    blocks = [np.arange(starts[b], starts[b] + branches[b]) for b in range(3)]
    perm = np.concatenate([np.arange(prefix)] + [blocks[b] for b in order] + [np.arange(T - join, T)])
    L2, anc2 = dags.fork_join(prefix, [branches[b] for b in order], join)
    _, pos2 = orc.token_meta(L2, anc2)
    O2, _ = orc.attn_prefill(orc.rope(q[perm], pos2, theta), orc.rope(k[perm], pos2, theta),
                             v[perm], L2, anc2)
    assert np.abs(O2 - O[perm]).max() < 1e-12


def test_value_probes_ones_and_one_hot_nodes():
    rng = np.random.Generator(np.random.PCG64(21))
    L, anc, _, _ = dags.random_dag(rng, n_nodes=10, depth=4, len_lo=1, len_hi=6)
    T, N = int(L.sum()), len(L)
    q, k = _rand(16, T, 2, 8), _rand(17, T, 1, 8)
    O, _ = orc.attn_prefill(q, k, np.ones((T, 1, 8)), L, anc)
    assert np.abs(O - 1.0).max() < 1e-12
    tok_node, _ = orc.token_meta(L, anc)
    onehot = np.zeros((T, 1, N))
    onehot[np.arange(T), 0, tok_node] = 1.0
    kk = _rand(18, T, 1, N)
    qq = _rand(19, T, 2, N)
    M, _ = orc.attn_prefill(qq, kk, onehot, L, anc)   # M[i, h, c] = attention mass on node c
    sets = dags.sets_from_bits(anc)
    for i in range(T):
        vi = int(tok_node[i])
        for c in range(N):
            if c != vi and c not in sets[vi]:
                assert M[i, 0, c] == 0.0 and M[i, 1, c] == 0.0
        assert abs(M[i, 0].sum() - 1.0) < 1e-12


def test_position_shift_invariance():
    L, anc = dags.fork_join(5, [3, 4], 2)
    T = int(L.sum())
    q, k, v = _rand(22, T, 2, 8), _rand(23, T, 2, 8), _rand(24, T, 2, 8)
    _, pos = orc.token_meta(L, anc)
    O1, _ = orc.attn_prefill(orc.rope(q, pos, 1e4), orc.rope(k, pos, 1e4), v, L, anc)
    O2, _ = orc.attn_prefill(orc.rope(q, pos + 777, 1e4), orc.rope(k, pos + 777, 1e4), v, L, anc)
    assert np.abs(O1 - O2).max() < 1e-9


def test_rows_and_heads_subset_matches_full():
    L, anc = dags.fork_join(6, [3, 3], 4)
    T = int(L.sum())
    q, k, v = _rand(25, T, 4, 8), _rand(26, T, 2, 8), _rand(27, T, 2, 8)
    O, lse = orc.attn_prefill(q, k, v, L, anc)
    Os, lses = orc.attn_prefill(q, k, v, L, anc, rows=[2, 9, 15], heads=[1, 3])
    assert np.array_equal(Os[[2, 9, 15]][:, [1, 3]], O[[2, 9, 15]][:, [1, 3]])
    assert np.isnan(Os[0]).all() and np.isnan(Os[2, 0]).all()


# ------------------------------------------------------------------ paged KV and decode
def _decode_fixture(seed=31, shared=40, blens=(17, 5, 32), hq=4, hkv=2, d=16):
    st = dags.decode_state(seed, n_seqs=1, n_branches=len(blens), shared_len=shared, branch_len=0,
                           hq=hq, hkv=hkv, d=d, dtype=torch.float64, branch_len_list=list(blens))
    return st


def test_pool_formats_against_independent_packing():
    n_pages, hkv, d = 3, 2, 16
    k_tok = torch.from_numpy(_rand(32, n_pages * 16, hkv, d))
    v_tok = torch.from_numpy(_rand(33, n_pages * 16, hkv, d))
    kp, vp = dags.pack_k_pages(k_tok).numpy(), dags.pack_v_pages(v_tok).numpy()
    for t in [0, 1, 15, 16, 37, 47]:
        for h in range(hkv):
            assert np.array_equal(orc.pool_get_k(kp, t // 16, h, t % 16), k_tok[t, h].numpy())
            assert np.array_equal(orc.pool_get_v(vp, t // 16, h, t % 16), v_tok[t, h].numpy())


def test_decode_equals_last_row_of_prefill():
    shared, blens, hq, hkv, d = 40, (17, 5, 32), 4, 2, 16
    st = _decode_fixture(shared=shared, blens=blens, hq=hq, hkv=hkv, d=d)
    desc, kp, vp = st["desc"], st["k_pool"].numpy(), st["v_pool"].numpy()
    qd = st["q"].numpy()
    Od = orc.attn_decode(desc, qd, kp, vp)
    for r, bl in enumerate(blens):
        K = np.stack([orc.gather_context(desc, r, h, kp, vp)[0] for h in range(hkv)], axis=1)
        V = np.stack([orc.gather_context(desc, r, h, kp, vp)[1] for h in range(hkv)], axis=1)
        T = shared + bl
        assert K.shape == (T, hkv, d)
        L, anc = dags.linear_chain([T])
        q = np.zeros((T, hq, d))
        q[-1] = qd[r]
        O, _ = orc.attn_prefill(q, K, V, L, anc)
        assert np.abs(O[-1] - Od[r]).max() < 1e-12


def test_decode_siblings_share_prefix_pages_and_own_the_rest():
    st = _decode_fixture()
    desc = st["desc"]
    kp, vp = st["k_pool"].numpy(), st["v_pool"].numpy()
    K0, _ = orc.gather_context(desc, 0, 0, kp, vp)
    K1, _ = orc.gather_context(desc, 1, 0, kp, vp)
    assert np.array_equal(K0[:40], K1[:40])
    assert K0.shape[0] == 40 + 17 and K1.shape[0] == 40 + 5
    # first shared token comes from the first shared page, slot 0
    p0 = int(desc["shared_pages"][0])
    assert np.array_equal(K0[0], kp[p0, 0, :, 0, :].reshape(-1))
    # last own token of branch 0 (index 16) sits in its second own page, slot 0
    pb = int(desc["branch_pages"][int(desc["branch_page_off"][0]) + 1])
    assert np.array_equal(K0[-1], kp[pb, 0, :, 0, :].reshape(-1))


def test_lse_merge_any_partition_equals_unsplit():
    K, V, q = _rand(34, 50, 8), _rand(35, 50, 8), _rand(36, 8)
    s = (K @ q) * 0.4
    p = np.exp(s - s.max())
    ref = (p @ V) / p.sum()
    for cuts in [[0, 50], [0, 1, 50], [0, 16, 32, 48, 50], [0, 7, 8, 30, 50]]:
        parts = [orc.partial_attention(q, K[a:b], V[a:b], 0.4) for a, b in zip(cuts[:-1], cuts[1:])]
        assert np.abs(orc.lse_merge(parts) - ref).max() < 1e-12


def test_kv_append_places_rotated_key_in_tail_slot():
    st = _decode_fixture(blens=(17, 5, 32))
    desc = st["desc"]
    kp, vp = st["k_pool"].numpy().copy(), st["v_pool"].numpy().copy()
    before_k = kp.copy()
    k_new, v_new = st["k_new"].numpy(), st["v_new"].numpy()
    orc.kv_append_rope(desc, k_new, v_new, kp, vp, theta=1e4)
    changed = np.argwhere(np.abs(kp - before_k).sum(axis=(1, 2, 4)) > 0)   # (page, slot)
    # exactly one (page, slot) per live branch
    assert len(changed) == 3
    for r, bl in enumerate((17, 5, 32)):
        K, V = orc.gather_context(desc, r, 1, kp, vp)
        pos = int(desc["branch_pos"][r])
        assert pos == 40 + bl - 1
        expect = orc.rope(k_new[r:r + 1], [pos], 1e4)[0, 1]
        assert np.abs(K[-1] - expect).max() < 1e-15
        assert np.array_equal(V[-1], v_new[r, 1])


def test_attn_prefill_compact_rows_mode_is_the_same_computation():
    """compact=True only changes where rows are read and written, not their values."""
    L, anc = dags.fork_join(20, [7, 9], 11)
    T = int(np.sum(L))
    rng = np.random.Generator(np.random.PCG64(5))
    q, k, v = rng.standard_normal((T, 4, 16)), rng.standard_normal((T, 2, 16)), rng.standard_normal((T, 2, 16))
    rows = np.array([0, 5, 21, 30, T - 1])
    O, lse = orc.attn_prefill(q, k, v, L, anc, rows=rows)
    Oc, lsec = orc.attn_prefill(q[rows], k, v, L, anc, rows=rows, compact=True)
    assert np.array_equal(O[rows], Oc) and np.array_equal(lse[rows], lsec)


# ----------------------------------------------------------------------------- decode over KV segments
def _multilevel_dag():
    """root -> (a, b); a -> (a0, a1); b -> (b0, b1, b2); join of a0, a1 and b0; lengths ragged
    against the page size."""
    parents = [[], [0], [0], [1], [1], [2], [2], [2], [3, 4, 5]]
    L = np.asarray([37, 16, 5, 21, 1, 33, 18, 7, 12], dtype=np.int32)
    return L, dags.bits_from_sets(dags.closure_from_parents(parents))


def _segments_fixture(seed=71, hq=4, hkv=2, d=16, live=(8, 6, 7, 4)):
    L, anc = _multilevel_dag()
    st = dags.decode_segments_state(seed, [(L, anc)], [list(live)], hq, hkv, d, dtype=torch.float64)
    return L, anc, st


def test_segment_decode_equals_the_dag_masked_prefill_row():
    """A live node decoding its last token over the segments of its ancestors and its own gives
    the row of DAG-masked attention (Eq. 3) of that token: pins the segment gather to the mask
    definition (partly filled pages, several sharing levels, a join of unequal branches).  The
    unused slots of partly filled pages hold large junk, so reading one slot too many shows."""
    L, anc, st = _segments_fixture()
    q_tok, k_tok, v_tok = (x.numpy() for x in st["tokens"][0])
    O, _ = orc.attn_prefill(q_tok, k_tok, v_tok, L, anc, rows=np.asarray(st["live_tok"]))
    Od = orc.attn_decode_segments(st["desc"], st["q"].numpy(), st["k_pool"].numpy(), st["v_pool"].numpy())
    assert np.abs(O[st["live_tok"]] - Od).max() < 1e-12


def test_segment_decode_context_sizes_and_reader_lists():
    L, anc, st = _segments_fixture()
    desc = st["desc"]
    # live branch 0 is the join (node 8): root, a, b, a0, a1, b0 and itself
    K, _ = orc.gather_segments(desc, 0, 0, st["k_pool"].numpy(), st["v_pool"].numpy())
    assert K.shape[0] == 37 + 16 + 5 + 21 + 1 + 33 + 12
    # live branch 3 is a1 (node 4): root, a, itself
    K, _ = orc.gather_segments(desc, 3, 1, st["k_pool"].numpy(), st["v_pool"].numpy())
    assert K.shape[0] == 37 + 16 + 1
    readers = lambda s: list(desc["seg_readers"][desc["seg_reader_off"][s]:desc["seg_reader_off"][s + 1]])
    assert readers(0) == [0, 1, 2, 3]          # the root is read by every live branch
    assert readers(2) == [0, 1, 2]             # b: the join (through b0), b1, b2
    assert readers(1) == [0, 3] and readers(4) == [0, 3] and readers(3) == [0]
    assert readers(6) == [1] and readers(7) == [2] and readers(8) == [0]


def test_segment_decode_is_independent_of_the_segmentation_and_its_order():
    """Cutting a segment in two (same tokens, other page boundaries) or listing a branch's
    segments in another order leaves the result alone: softmax over a set of keys."""
    hq, hkv, d = 2, 1, 16
    rng = np.random.Generator(np.random.PCG64(72))
    k_tok, v_tok = rng.standard_normal((50, hkv, d)), rng.standard_normal((50, hkv, d))
    q = rng.standard_normal((1, hq, d))
    def build(cuts, order):
        lens = [b - a for a, b in zip(cuts[:-1], cuts[1:])]
        npg = [(n + 15) // 16 for n in lens]
        kp = rng.standard_normal((sum(npg), hkv, d // 8, 16, 8)) * 9
        vp = rng.standard_normal((sum(npg), hkv, d, 16)) * 9
        off = np.concatenate([[0], np.cumsum(npg)]).astype(np.int32)
        for s, (a, b) in enumerate(zip(cuts[:-1], cuts[1:])):
            for t in range(a, b):
                kp[off[s] + (t - a) // 16, :, :, (t - a) % 16, :] = k_tok[t].reshape(hkv, d // 8, 8)
                vp[off[s] + (t - a) // 16, :, :, (t - a) % 16] = v_tok[t]
        n = len(lens)
        desc = dict(n_live=1, n_segments=n, page_size=16, seg_page_off=off,
                    seg_pages=np.arange(sum(npg), dtype=np.int32), seg_len=np.asarray(lens, dtype=np.int32),
                    seg_reader_off=np.arange(n + 1, dtype=np.int32), seg_readers=np.zeros(n, dtype=np.int32),
                    branch_seg_off=np.asarray([0, n], dtype=np.int32), branch_segs=np.asarray(order, dtype=np.int32))
        return orc.attn_decode_segments(desc, q, kp, vp)
    s = np.einsum("thd,hd->th", np.repeat(k_tok, hq // hkv, axis=1), q[0]) / np.sqrt(d)
    p = np.exp(s - s.max(axis=0))
    ref = np.einsum("th,thd->hd", p / p.sum(axis=0), np.repeat(v_tok, hq // hkv, axis=1))
    for cuts, order in [([0, 50], [0]), ([0, 17, 50], [0, 1]), ([0, 17, 50], [1, 0]), ([0, 1, 16, 33, 50], [2, 0, 3, 1])]:
        assert np.abs(build(cuts, order)[0] - ref).max() < 1e-12


def test_two_level_description_as_segments_gives_the_two_level_result():
    st = _decode_fixture(blens=(17, 5, 32))
    kp, vp, q = st["k_pool"].numpy(), st["v_pool"].numpy(), st["q"].numpy()
    sdesc = dags.segments_from_decode_desc(st["desc"])
    assert np.array_equal(orc.attn_decode_segments(sdesc, q, kp, vp), orc.attn_decode(st["desc"], q, kp, vp))


def test_segment_decode_with_reader_lengths_is_chunked_prefill_of_new_nodes():
    """The last n tokens of a node as n live branches, each seeing the node's own segment up to
    itself and the ancestors' segments in full: every such row equals the DAG-masked prefill row
    (Eq. 3: causal inside the node, full visibility of ancestors).  A join prefilled whole, a leaf
    prefilled over its last 5 tokens, a single-token decode beside them."""
    L, anc = _multilevel_dag()
    live, new = [8, 6, 4], [12, 5, 1]
    st = dags.decode_segments_state(73, [(L, anc)], [live], 4, 2, 16, dtype=torch.float64, new_tokens=[new])
    desc = st["desc"]
    assert desc["n_live"] == 18 and len(desc["seg_reader_len"]) == len(desc["seg_readers"])
    # node 8 (12 tokens, all new): its readers see 1..12 of its segment; the root in full
    r8 = desc["seg_reader_len"][desc["seg_reader_off"][8]:desc["seg_reader_off"][9]]
    assert list(r8) == list(range(1, 13))
    assert set(desc["seg_reader_len"][desc["seg_reader_off"][0]:desc["seg_reader_off"][1]]) == {37}
    q_tok, k_tok, v_tok = (x.numpy() for x in st["tokens"][0])
    O, _ = orc.attn_prefill(q_tok, k_tok, v_tok, L, anc, rows=np.asarray(st["live_tok"]))
    Od = orc.attn_decode_segments(desc, st["q"].numpy(), st["k_pool"].numpy(), st["v_pool"].numpy())
    assert np.abs(O[st["live_tok"]] - Od).max() < 1e-12
    # a planted mistake (every reader sees the whole own segment: no causality inside the node) shows
    bad = dict(desc)
    bad["seg_reader_len"] = np.full_like(desc["seg_reader_len"], 1 << 20)
    Ob = orc.attn_decode_segments(bad, st["q"].numpy(), st["k_pool"].numpy(), st["v_pool"].numpy())
    assert np.abs(O[st["live_tok"]] - Ob).max() > 1e-3


# ----------------------------------------------------------------------------- scheduling
def test_frontiers_of_textbook_nets():
    # chain: one transition per frontier
    assert orc.frontier_layers([[], [0], [1], [2]]) == [[0], [1], [2], [3]]
    # fork / join: siblings fire together, the join after all of them (A, B -> C is one transition)
    assert orc.frontier_layers([[], [0], [0], [0], [1, 2, 3]]) == [[0], [1, 2, 3], [4]]
    # two roots, a join of both and a child of one: the child does not wait for the other root's join
    assert orc.frontier_layers([[], [], [0, 1], [0]]) == [[0, 1], [2, 3]]
    # an edge that skips a level does not let a node fire before its slowest parent
    assert orc.frontier_layers([[], [0], [1], [0, 2]]) == [[0], [1], [2], [3]]
    assert orc.frontier_layers([]) == []


def test_frontier_index_is_the_longest_path_and_every_node_fires_once():
    rng = np.random.Generator(np.random.PCG64(90))
    for _ in range(20):
        n = int(rng.integers(1, 40))
        parents = [sorted(set(int(x) for x in rng.integers(0, v, size=int(rng.integers(0, 4))))) if v else []
                   for v in range(n)]
        layers = orc.frontier_layers(parents)
        assert sorted(v for f in layers for v in f) == list(range(n))
        depth = [0] * n                       # longest path to v, by dynamic programming over the topological order
        for v in range(n):
            depth[v] = 1 + max([depth[p] for p in parents[v]], default=-1)
        for k, f in enumerate(layers):
            assert all(depth[v] == k for v in f)


def test_step_counts_parallel_against_serial():
    """Token-by-token generation of prefix -> branches -> join takes prefix + longest branch + join
    steps (the depth of the plan), a chain with the same tokens takes their sum (section 5,
    latency argument); chunks shorten a frontier to ceil(len / chunk)."""
    parents = [[], [0], [0], [0], [1, 2, 3]]
    L = [7, 5, 11, 3, 4]
    steps = orc.schedule_steps(parents, L)
    assert len(steps) == 7 + 11 + 4
    assert sum(n for s in steps for _, _, n in s) == sum(L)
    assert steps[7] == [(1, 0, 1), (2, 0, 1), (3, 0, 1)] and steps[7 + 3] == [(1, 3, 1), (2, 3, 1)]
    assert steps[7 + 10] == [(2, 10, 1)] and steps[-1] == [(4, 3, 1)]
    chain = [[]] + [[v] for v in range(4)]
    assert len(orc.schedule_steps(chain, L)) == sum(L)
    chunked = orc.schedule_steps(parents, L, chunk=[4, 1, 1, 1, 3])
    assert len(chunked) == 2 + 11 + 2
    assert chunked[0] == [(0, 0, 4)] and chunked[1] == [(0, 4, 3)] and chunked[-1] == [(4, 3, 1)]


# ----------------------------------------------------------------------------- backward
def _bwd_fixture(seed=95, hq=4, hkv=2, d=8):
    L, anc = _multilevel_dag()
    L = np.asarray([5, 3, 2, 4, 1, 3, 2, 2, 3], dtype=np.int32)
    T = int(L.sum())
    rng = np.random.Generator(np.random.PCG64(seed))
    q, k, v = rng.standard_normal((T, hq, d)), rng.standard_normal((T, hkv, d)), rng.standard_normal((T, hkv, d))
    dout = rng.standard_normal((T, hq, d))
    return L, anc, q, k, v, dout


def test_backward_equals_central_differences_of_the_forward_oracle():
    """d/dx sum(dout * O(x)) by central differences on sampled entries of q, k and v (GQA: a KV
    entry feeds two query heads; a node with a join: masked pairs carry no gradient)."""
    L, anc, q, k, v, dout = _bwd_fixture()
    dq, dk, dv = orc.attn_prefill_bwd(q, k, v, dout, L, anc, scale=0.4)
    loss = lambda q_, k_, v_: float(np.sum(dout * orc.attn_prefill(q_, k_, v_, L, anc, scale=0.4)[0]))
    rng = np.random.Generator(np.random.PCG64(96))
    eps = 1e-6
    for name, x, g in (("q", q, dq), ("k", k, dk), ("v", v, dv)):
        for _ in range(12):
            idx = tuple(int(rng.integers(n)) for n in x.shape)
            xp, xm = x.copy(), x.copy()
            xp[idx] += eps
            xm[idx] -= eps
            args_p = {"q": (xp, k, v), "k": (q, xp, v), "v": (q, k, xp)}[name]
            args_m = {"q": (xm, k, v), "k": (q, xm, v), "v": (q, k, xm)}[name]
            num = (loss(*args_p) - loss(*args_m)) / (2 * eps)
            assert abs(num - g[idx]) < 1e-7 * max(1.0, abs(num)), (name, idx, num, g[idx])


def test_backward_equals_library_autograd_on_the_explicit_mask():
    L, anc, q, k, v, dout = _bwd_fixture(seed=97, hq=6, hkv=2, d=4)
    dq, dk, dv = orc.attn_prefill_bwd(q, k, v, dout, L, anc)
    tq, tk, tv = (torch.tensor(x, dtype=torch.float64, requires_grad=True) for x in (q, k, v))
    allow = torch.from_numpy(orc.explicit_mask(L, anc))
    G = q.shape[1] // k.shape[1]
    kk, vv = tk.repeat_interleave(G, dim=1), tv.repeat_interleave(G, dim=1)
    S = torch.einsum("ihd,jhd->hij", tq, kk) / np.sqrt(q.shape[2])
    P = torch.softmax(S.masked_fill(~allow[None], float("-inf")), dim=-1)
    O = torch.einsum("hij,jhd->ihd", P, vv)
    (O * torch.from_numpy(dout)).sum().backward()
    for a, b in ((dq, tq.grad), (dk, tk.grad), (dv, tv.grad)):
        assert np.abs(a - b.numpy()).max() < 1e-12


def test_backward_structure():
    """A token nobody but itself sees gets dk, dv only from its own row; masked pairs carry
    nothing: the last token of a leaf node is seen only by itself."""
    L, anc, q, k, v, dout = _bwd_fixture(seed=98)
    dq, dk, dv = orc.attn_prefill_bwd(q, k, v, dout, L, anc)
    t = int(np.cumsum(L)[6] - 1)          # last token of node 6 (a leaf)
    G = q.shape[1] // k.shape[1]
    allow = orc.explicit_mask(L, anc)
    assert allow[:, t].sum() == 1
    for hk in range(k.shape[1]):
        want = np.zeros(v.shape[2])
        for h in range(hk * G, (hk + 1) * G):
            s = (k[allow[t], hk] @ q[t, h]) / np.sqrt(q.shape[2])
            p = np.exp(s - s.max()); p /= p.sum()
            want += p[-1] * dout[t, h]     # the token is the last visible key of its own row
        assert np.abs(dv[t, hk] - want).max() < 1e-12
    assert np.isfinite(dq).all() and np.isfinite(dk).all()
