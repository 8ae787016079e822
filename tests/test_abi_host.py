"""CPU-only checks of the C-ABI library: it loads, exports every symbol include/dagattn.h
declares, and its host-side validation returns the documented error codes before any GPU work
(no compute call is made here, so no GPU is needed)."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from paper_2602_07529_amd import binding as B
from workloads import dags

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE = 0x10000  # a non-null, 16-byte aligned "device pointer"; never dereferenced on these paths


def _declared_functions():
    txt = open(os.path.join(ROOT, "include", "dagattn.h")).read()
    txt = re.sub(r"/\*.*?\*/", "", txt, flags=re.S)
    return sorted(set(re.findall(r"\b(dag_[a-z_0-9]+)\s*\(", txt)))


def test_library_exports_every_declared_symbol():
    names = _declared_functions()
    assert {"dag_meta_sizes", "dag_build_meta", "dag_rope_qk", "dag_attn_prefill", "dag_kv_append_rope",
            "dag_attn_decode", "dag_decode_workspace_bytes", "dag_prefill_workspace_bytes", "dag_prefill_tile_shape",
            "dag_prefill_prepare_v", "dag_attn_prefill_prepared",
            "dag_attn_decode_segments", "dag_decode_segments_workspace_bytes",
            "dag_strerror",
            "dag_version"} <= set(names)
    L = C.CDLL(B.LIB_PATH)
    for n in names:
        assert hasattr(L, n), n


def test_version_and_strerror():
    assert B.dag_version() >= 100
    assert B.dag_strerror(0) == "ok"
    for code in range(-9, 0):
        assert B.dag_strerror(code) not in ("ok", "unknown error")
    assert B.dag_strerror(-99) == "unknown error"


def test_tile_shape_table():
    assert B.dag_prefill_tile_shape(4, 4, 64, B.DAG_F32) == (64, 64)
    assert B.dag_prefill_tile_shape(32, 8, 128, B.DAG_BF16) == (64, 64)
    assert B.dag_prefill_tile_shape(40, 8, 128, B.DAG_BF16) == (64, 64)
    assert B.dag_prefill_tile_shape(16, 8, 64, B.DAG_BF16) == (64, 64)
    assert B.dag_prefill_tile_shape(8, 8, 128, B.DAG_BF16) == (64, 64)
    with pytest.raises(B.DagError) as e:
        B.dag_prefill_tile_shape(6, 4, 128, B.DAG_BF16)
    assert e.value.code == -7
    with pytest.raises(B.DagError):
        B.dag_prefill_tile_shape(8, 8, 96, B.DAG_BF16)


def _desc(dag_list, tile=(64, 64), flags=0, words=None):
    off, lens, bits, W = dags.batch_desc(dag_list)
    return B.DagDesc(off, lens, bits, W if words is None else words, tile[0], tile[1], flags)


def test_meta_sizes_counts():
    one = dags.fork_join(2048, [256] * 8, 512)
    s = B.dag_meta_sizes(_desc([one] * 4))
    assert s.total_nodes == 40 and s.total_tokens == 18432
    assert s.total_qtiles == 4 * 72 and s.total_tiles == 4 * 72 * 72
    # ragged: T = 100 with 32x64 tiles -> 4 query tiles, 2 key tiles
    s = B.dag_meta_sizes(_desc([dags.linear_chain([100])], tile=(32, 64)))
    assert (s.total_qtiles, s.total_tiles) == (4, 8)
    assert s.csr_capacity == 1 + 1 + 2 + 2 + 8      # eight spare entries at the end
    # empty batch and an empty sequence
    s = B.dag_meta_sizes(B.DagDesc(np.zeros(1, np.int32), np.zeros(0, np.int32), np.zeros((0, 1), np.uint64), 1, 32, 64))
    assert s.total_tokens == 0 and s.total_qtiles == 0
    s = B.dag_meta_sizes(B.DagDesc(np.array([0, 0, 1], np.int32), np.array([5], np.int32), np.zeros((1, 1), np.uint64), 1, 32, 64))
    assert s.total_tokens == 5 and s.total_qtiles == 1


def _build_rc(desc, ws_bytes=1 << 20):
    sizes = B.dag_meta_sizes(desc)
    m = B.dag_meta_t()
    m.n_seqs, m.words_per_node = desc.c.n_seqs, desc.c.words_per_node
    m.tile_m, m.tile_n = desc.c.tile_m, desc.c.tile_n
    m.sizes = sizes
    for name, _ in B._META_ARRAYS:
        setattr(m, name, FAKE)
    return B.lib().dag_build_meta(C.byref(desc.c), C.byref(m), C.c_void_p(FAKE), ws_bytes, None)


def test_build_meta_rejects_invalid_dags_before_any_gpu_work():
    # node length < 1
    with pytest.raises(B.DagError) as e:
        B.dag_meta_sizes(B.DagDesc(np.array([0, 2], np.int32), np.array([3, 0], np.int32), np.zeros((2, 1), np.uint64), 1, 32, 64))
    assert e.value.code == -2
    # not topological: node 0 lists node 1 as an ancestor (a cycle 0 <-> 1 looks the same)
    bits = dags.bits_from_sets([{1}, {0}])
    d = B.DagDesc(np.array([0, 2], np.int32), np.array([3, 3], np.int32), bits, 1, 32, 64)
    assert _build_rc(d) == -3
    # self bit alone is ignored, not an error; rejected later only for the tiny workspace
    bits = dags.bits_from_sets([{0}, {0, 1}])
    d = B.DagDesc(np.array([0, 2], np.int32), np.array([3, 3], np.int32), bits, 1, 32, 64)
    assert _build_rc(d, ws_bytes=8) == -6
    # strict closure: 2 lists 1 but not 1's ancestor 0
    bits = dags.bits_from_sets([set(), {0}, {1}])
    d = B.DagDesc(np.array([0, 3], np.int32), np.array([1, 1, 1], np.int32), bits, 1, 32, 64, B.DAG_STRICT_CLOSURE)
    assert _build_rc(d) == -4
    d = B.DagDesc(np.array([0, 3], np.int32), np.array([1, 1, 1], np.int32), bits, 1, 32, 64, 0)
    assert _build_rc(d, ws_bytes=8) == -6          # lax mode accepts it (fails only on the workspace)
    # too few bitset words for the node count
    L, anc = dags.linear_chain([1] * 70)
    with pytest.raises(B.DagError) as e:
        B.dag_meta_sizes(B.DagDesc(np.array([0, 70], np.int32), L, anc[:, :1].copy(), 1, 32, 64))
    assert e.value.code == -2
    # sizes in the meta struct must match the description
    d = _desc([dags.linear_chain([10, 10])])
    sizes = B.dag_meta_sizes(d)
    m = B.dag_meta_t()
    m.n_seqs, m.words_per_node, m.tile_m, m.tile_n = 1, 1, 32, 64
    sizes.total_tokens += 1
    m.sizes = sizes
    assert B.lib().dag_build_meta(C.byref(d.c), C.byref(m), C.c_void_p(FAKE), 1 << 20, None) == -2
    # null description
    assert B.lib().dag_build_meta(None, C.byref(m), C.c_void_p(FAKE), 1 << 20, None) == -1


def test_position_overflow_is_reported():
    lens = np.full(3, 2 ** 30, dtype=np.int32)
    _, anc = dags.linear_chain([1, 1, 1])
    with pytest.raises(B.DagError) as e:
        B.dag_meta_sizes(B.DagDesc(np.array([0, 3], np.int32), lens, anc, 1, 1024, 1024))
    assert e.value.code == -5


def test_rope_and_prefill_argument_errors():
    L = B.lib()
    assert L.dag_rope_qk(C.c_void_p(FAKE), 4, C.c_void_p(FAKE), None, 2, 0, 100, 1e4, B.DAG_BF16, None) == -7
    assert L.dag_rope_qk(C.c_void_p(FAKE), 4, C.c_void_p(FAKE + 4), None, 2, 0, 64, 1e4, B.DAG_BF16, None) == -8
    assert L.dag_rope_qk(None, 4, C.c_void_p(FAKE), None, 2, 0, 64, 1e4, B.DAG_BF16, None) == -1
    assert L.dag_rope_qk(None, 0, C.c_void_p(FAKE), None, 2, 0, 64, 1e4, B.DAG_BF16, None) == 0
    d = _desc([dags.linear_chain([10, 10])])
    m = B.dag_meta_t()
    m.n_seqs, m.words_per_node, m.tile_m, m.tile_n = 1, 1, 64, 64
    m.sizes = B.dag_meta_sizes(d)
    for name, _ in B._META_ARRAYS:
        setattr(m, name, FAKE)
    p = C.c_void_p(FAKE)
    # tile shape of the meta does not match the kernel's (64x64)
    big = 1 << 30
    m.tile_m = 32
    assert L.dag_attn_prefill(C.byref(m), p, p, p, p, None, 8, 8, 128, 0.1, B.DAG_BF16, p, big, None) == -7
    m.tile_m = 64
    assert L.dag_attn_prefill(C.byref(m), p, p, p, p, None, 32, 8, 96, 0.1, B.DAG_BF16, p, big, None) == -7
    assert L.dag_attn_prefill(C.byref(m), None, p, p, p, None, 32, 8, 128, 0.1, B.DAG_BF16, p, big, None) == -1
    assert L.dag_attn_prefill(C.byref(m), C.c_void_p(FAKE + 2), p, p, p, None, 32, 8, 128, 0.1, B.DAG_BF16, p, big,
                              None) == -8
    assert L.dag_attn_prefill(None, p, p, p, p, None, 32, 8, 128, 0.1, B.DAG_BF16, p, big, None) == -1
    # workspace: the bf16 path needs room for the transposed copy of V, the fp32 path needs none
    need = L.dag_prefill_workspace_bytes(C.byref(m), 8, 128, B.DAG_BF16)
    # one key tile x 8 kv heads; counters and the tables of the 256-row query tiles (17 ints per 64-row tile,
    # one per non-skip tile); alignment slack
    assert need == 1 * 8 * 128 * 64 * 2 + 4 * (128 + 64 + 17 * m.sizes.total_qtiles + m.sizes.csr_capacity) + 256
    assert L.dag_prefill_workspace_bytes(C.byref(m), 8, 128, B.DAG_F32) == 0
    assert L.dag_attn_prefill(C.byref(m), p, p, p, p, None, 32, 8, 128, 0.1, B.DAG_BF16, p, need - 1, None) == -6
    assert L.dag_attn_prefill(C.byref(m), p, p, p, p, None, 32, 8, 128, 0.1, B.DAG_BF16, None, 0, None) == -6
    # the two halves validate the same way
    assert L.dag_attn_prefill_prepared(C.byref(m), p, p, p, p, None, 32, 8, 128, 0.1, B.DAG_BF16, p, need - 1, None) == -6
    assert L.dag_attn_prefill_prepared(C.byref(m), None, p, p, p, None, 32, 8, 128, 0.1, B.DAG_BF16, p, big, None) == -1
    assert L.dag_prefill_prepare_v(C.byref(m), p, 32, 8, 128, B.DAG_BF16, p, need - 1, None) == -6
    assert L.dag_prefill_prepare_v(C.byref(m), None, 32, 8, 128, B.DAG_BF16, p, big, None) == -1
    assert L.dag_prefill_prepare_v(C.byref(m), p, 32, 8, 96, B.DAG_BF16, p, big, None) == -7
    assert L.dag_prefill_prepare_v(None, p, 32, 8, 128, B.DAG_BF16, p, big, None) == -1
    assert L.dag_prefill_prepare_v(C.byref(m), C.c_void_p(FAKE + 2), 32, 8, 128, B.DAG_BF16, p, big, None) == -8


def test_decode_argument_errors():
    L = B.lib()
    dd = B.dag_decode_desc_t(1, 2, 16, 4, 2, 2, *([FAKE] * 8))
    p = C.c_void_p(FAKE)
    need = L.dag_decode_workspace_bytes(C.byref(dd), 32, 8, 128)
    assert need > 0
    assert L.dag_attn_decode(C.byref(dd), p, p, p, p, 32, 8, 128, 0.1, p, need - 1, None) == -6
    assert L.dag_attn_decode(C.byref(dd), p, p, p, p, 32, 8, 128, 0.1, None, need, None) == -6
    assert L.dag_attn_decode(C.byref(dd), p, p, p, p, 32, 8, 96, 0.1, p, need, None) == -7
    assert L.dag_attn_decode(C.byref(dd), p, p, p, p, 30, 8, 128, 0.1, p, need, None) == -7
    assert L.dag_attn_decode(C.byref(dd), None, p, p, p, 32, 8, 128, 0.1, p, need, None) == -1
    bad_page = B.dag_decode_desc_t(1, 2, 32, 4, 2, 2, *([FAKE] * 8))
    assert L.dag_attn_decode(C.byref(bad_page), p, p, p, p, 32, 8, 128, 0.1, p, need, None) == -7
    # the variant without a workspace validates the same way and refuses what its array cannot hold
    assert L.dag_attn_decode_static(C.byref(dd), p, p, p, p, 32, 8, 96, 0.1, None) == -7
    assert L.dag_attn_decode_static(C.byref(dd), None, p, p, p, 32, 8, 128, 0.1, None) == -1
    assert L.dag_attn_decode_static(C.byref(bad_page), p, p, p, p, 32, 8, 128, 0.1, None) == -7
    huge = B.dag_decode_desc_t(64, 64 * 32, 16, 1 << 16, 64, 32, *([FAKE] * 8))
    assert L.dag_decode_workspace_bytes(C.byref(huge), 32, 8, 128) > B.DECODE_STATIC_SCRATCH_BYTES
    assert L.dag_attn_decode_static(C.byref(huge), p, p, p, p, 32, 8, 128, 0.1, None) == -6
    assert L.dag_decode_workspace_bytes(C.byref(bad_page), 32, 8, 128) == 0
    assert L.dag_kv_append_rope(C.byref(bad_page), p, p, p, p, 8, 128, 1e4, None) == -7
    assert L.dag_kv_append_rope(C.byref(dd), None, p, p, p, 8, 128, 1e4, None) == -1
    # head dimensions other than 64 and 128 are refused (the kernel's angle tables hold 64 pairs)
    for bad_d in (16, 96, 144, 192, 256):
        assert L.dag_kv_append_rope(C.byref(dd), p, p, p, p, 8, bad_d, 1e4, None) == -7
    empty = B.dag_decode_desc_t(0, 0, 16, 0, 0, 0, *([0] * 8))
    assert L.dag_attn_decode(C.byref(empty), p, p, p, p, 32, 8, 128, 0.1, None, 0, None) == 0
    assert L.dag_kv_append_rope(C.byref(empty), p, p, p, p, 8, 128, 1e4, None) == 0


def test_segment_decode_argument_errors():
    L = B.lib()
    sd = B.dag_decode_seg_desc_t(4, 3, 16, 40, 4, 6, *([FAKE] * 7), None)
    p = C.c_void_p(FAKE)
    need = L.dag_decode_segments_workspace_bytes(C.byref(sd), 32, 8, 128)
    # 40 pages, 3 x 8 x 1 items per split: the split size halves from 128 pages to 8 -> 5 splits
    assert need >= 5 * 6 * 32 * (128 + 2) * 4
    args = (32, 8, 128, 0.1)
    assert L.dag_attn_decode_segments(C.byref(sd), p, p, p, p, *args, p, need - 1, None) == -6
    assert L.dag_attn_decode_segments(C.byref(sd), p, p, p, p, *args, None, need, None) == -6
    assert L.dag_attn_decode_segments(C.byref(sd), p, p, p, p, 32, 8, 96, 0.1, p, need, None) == -7
    assert L.dag_attn_decode_segments(C.byref(sd), p, p, p, p, 30, 8, 128, 0.1, p, need, None) == -7
    assert L.dag_attn_decode_segments(C.byref(sd), None, p, p, p, *args, p, need, None) == -1
    assert L.dag_attn_decode_segments(C.byref(sd), C.c_void_p(FAKE + 2), p, p, p, *args, p, need, None) == -8
    assert L.dag_attn_decode_segments(None, p, p, p, p, *args, p, need, None) == -1
    bad_page = B.dag_decode_seg_desc_t(4, 3, 32, 40, 4, 6, *([FAKE] * 7), None)
    assert L.dag_attn_decode_segments(C.byref(bad_page), p, p, p, p, *args, p, need, None) == -7
    assert L.dag_decode_segments_workspace_bytes(C.byref(bad_page), 32, 8, 128) == 0
    neg = B.dag_decode_seg_desc_t(4, 3, 16, -1, 4, 6, *([FAKE] * 7), None)
    assert L.dag_attn_decode_segments(C.byref(neg), p, p, p, p, *args, p, need, None) == -2
    no_arrays = B.dag_decode_seg_desc_t(4, 3, 16, 40, 4, 6, *([0] * 7), None)
    assert L.dag_attn_decode_segments(C.byref(no_arrays), p, p, p, p, *args, p, need, None) == -1
    empty = B.dag_decode_seg_desc_t(0, 0, 16, 0, 0, 0, *([0] * 7), None)
    assert L.dag_attn_decode_segments(C.byref(empty), p, p, p, p, *args, None, 0, None) == 0


# ----------------------------------------------------------------------------- scheduler (host only)
def _run_schedule(parents, node_len, chunk=None, n_pages=4096):
    sch = B.Scheduler(parents, node_len, n_pages, chunk)
    steps = []
    while True:
        st = sch.step()
        if st is None:
            break
        steps.append(st)
    assert sch.step() is None          # stays finished
    sch.close()
    return steps


def _as_oracle_steps(steps):
    out = []
    for st in steps:
        cur = []
        for v, t in zip(st["live_node"], st["live_token"]):
            if cur and cur[-1][0] == v:
                cur[-1] = (v, cur[-1][1], cur[-1][2] + 1)
            else:
                cur.append((int(v), int(t), 1))
        out.append(cur)
    return out


def test_paged_prefill_argument_errors():
    L = B.lib()
    p = C.c_void_p(FAKE)
    d = B.dag_paged_prefill_desc_t(3, 16, 100, 70, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE)
    # counters + item count, per (node, query tile) slot 17 ints and a row of 18 tile entries of 8 ints; slack
    need = L.dag_prefill_paged_workspace_bytes(C.byref(d))
    assert need == 4 * (128 + 64 + 3 * 2 * (17 + 8 * 18)) + 256
    big = 1 << 30
    args = lambda desc=d, q=p, hq=8, hkv=2, dim=128, ws=p, wsb=big, n_pages=50: L.dag_attn_prefill_paged(
        C.byref(desc), q, p, p, n_pages, p, None, hq, hkv, dim, 0.1, ws, wsb, None)
    assert args(dim=96) == -7 and args(hq=7) == -7
    assert args(q=None) == -1 and args(ws=None) == -6 and args(wsb=need - 1) == -6
    assert args(q=C.c_void_p(FAKE + 2)) == -8
    assert args(n_pages=0) == -2
    bad = B.dag_paged_prefill_desc_t(3, 32, 100, 70, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE)
    assert args(desc=bad) == -7 and L.dag_prefill_paged_workspace_bytes(C.byref(bad)) == 0
    neg = B.dag_paged_prefill_desc_t(3, 16, -1, 70, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE)
    assert args(desc=neg) == -2
    nullarr = B.dag_paged_prefill_desc_t(3, 16, 100, 70, FAKE, None, FAKE, FAKE, FAKE, FAKE)
    assert args(desc=nullarr) == -1
    nothing = B.dag_paged_prefill_desc_t(0, 16, 0, 0, None, None, None, None, None, None)
    assert args(desc=nothing, q=None, ws=None, wsb=0) == 0   # no node: nothing to do, nothing is read
    assert L.dag_attn_prefill_paged(None, p, p, p, 50, p, None, 8, 2, 128, 0.1, p, big, None) == -1


def test_scheduler_steps_equal_the_oracle_schedule():
    from oracle import dag_oracle as orc
    rng = np.random.Generator(np.random.PCG64(91))
    cases = [([[], [0], [0], [0], [1, 2, 3]], [7, 5, 11, 3, 4], None),
             ([[], [0], [0], [0], [1, 2, 3]], [7, 5, 11, 3, 4], [4, 1, 1, 1, 3]),
             ([[], [], [0, 1], [0]], [20, 3, 2, 9], [16, 16, 1, 1])]
    for _ in range(6):
        n = int(rng.integers(1, 30))
        parents = [sorted(set(int(x) for x in rng.integers(0, v, size=int(rng.integers(0, 4))))) if v else []
                   for v in range(n)]
        cases.append((parents, [int(x) for x in rng.integers(1, 40, size=n)],
                      [int(x) for x in rng.integers(1, 9, size=n)]))
    for parents, L, chunk in cases:
        steps = _run_schedule(parents, L, chunk)
        assert _as_oracle_steps(steps) == orc.schedule_steps(parents, L, chunk)
        layers = orc.frontier_layers(parents)
        for st in steps:
            assert set(int(v) for v in st["live_node"]) <= set(layers[st["layer"]])


def test_scheduler_pages_positions_and_descriptions():
    """Fork/join on pages and positions: children start one past the parent's last position,
    the join one past the longest branch; pages are never shared between nodes nor moved; every
    live token reads exactly its ancestors in full and its own node up to itself."""
    from oracle import dag_oracle as orc
    from workloads import dags
    parents = [[], [0], [0], [0], [1, 2, 3]]
    L = [37, 5, 40, 16, 20]
    steps = _run_schedule(parents, L, chunk=[16, 1, 1, 1, 8])
    anc = dags.bits_from_sets(dags.closure_from_parents(parents))
    pos_start = orc.node_tables(np.asarray(L), anc)[1]
    pages_of, seen_pos = {}, {}
    for st in steps:
        for r in range(st["n_live"]):
            v, t = int(st["live_node"][r]), int(st["live_token"][r])
            assert st["branch_pos"][r] == pos_start[v] + t and st["branch_len"][r] == t + 1
            pl = list(st["branch_pages"][st["branch_page_off"][r]:st["branch_page_off"][r + 1]])
            assert len(pl) == (st["seg_len"][list(st["seg_node"]).index(v)] + 15) // 16
            old = pages_of.get(v, [])
            assert pl[:len(old)] == old            # a node's pages only grow
            pages_of[v] = pl
            seen_pos[(v, t)] = True
            mine = st["branch_entries"][st["branch_entry_off"][r]:st["branch_entry_off"][r + 1]]
            read = {}
            for e in mine:
                assert st["seg_readers"][e] == r
                si = int(np.searchsorted(st["seg_reader_off"], e, side="right") - 1)
                read[int(st["seg_node"][si])] = int(st["seg_reader_len"][e])
            want = {u: L[u] for u in orc.ancestors(anc, v)}
            want[v] = t + 1
            assert read == want
        assert st["pages_in_use"] == sum(len(p) for p in pages_of.values())
    flat = [p for pl in pages_of.values() for p in pl]
    assert len(flat) == len(set(flat)) == sum((x + 15) // 16 for x in L)
    assert len(seen_pos) == sum(L)


def test_scheduler_argument_errors_and_page_exhaustion():
    L = B.lib()
    h = C.c_void_p()
    off = (C.c_int32 * 3)(0, 0, 1)
    par = (C.c_int32 * 1)(0)
    ln = (C.c_int32 * 2)(20, 5)
    assert L.dag_sched_create(2, off, par, ln, None, 8, 16, None) == -1
    assert L.dag_sched_create(2, off, par, ln, None, 8, 32, C.byref(h)) == -7
    bad_par = (C.c_int32 * 1)(1)
    assert L.dag_sched_create(2, off, bad_par, ln, None, 8, 16, C.byref(h)) == -3
    bad_len = (C.c_int32 * 2)(20, 0)
    assert L.dag_sched_create(2, off, par, bad_len, None, 8, 16, C.byref(h)) == -2
    # a chain whose positions leave the int32 range is refused when the plan is created
    big = (C.c_int32 * 2)(2 ** 31 - 8, 16)
    assert L.dag_sched_create(2, off, par, big, None, 8, 16, C.byref(h)) == -5 and not h.value
    assert L.dag_sched_create(2, off, par, ln, None, 2, 16, C.byref(h)) == 0      # 3 pages needed, 2 in the pool
    st = B.dag_sched_step_t()
    rcs = []
    for _ in range(26):
        rcs.append(L.dag_sched_step(h, C.byref(st)))
    assert rcs[:20] == [0] * 20 and rcs[20] == -6 and rcs[25] == -6      # node 1 never gets its page
    L.dag_sched_destroy(h)
    L.dag_sched_destroy(None)


def test_backward_argument_errors():
    L = B.lib()
    d = _desc([dags.linear_chain([10, 10])])
    m = B.dag_meta_t()
    m.n_seqs, m.words_per_node, m.tile_m, m.tile_n = 1, 1, 64, 64
    m.sizes = B.dag_meta_sizes(d)
    for name, _ in B._META_ARRAYS:
        setattr(m, name, FAKE)
    p = C.c_void_p(FAKE)
    need = L.dag_prefill_bwd_workspace_bytes(C.byref(m), 32, 8, 128)
    # delta and -lse log2(e), weight and order of the one key tile, first visibility word of the 20 tokens
    assert need == 2 * 2560 + 2 * 256 + 256 + 256
    # five query heads per KV head leave one over: the tile lists of the dQ workgroups that take four query tiles
    # (one entry of the dense block map here, one query tile)
    assert L.dag_prefill_bwd_workspace_bytes(C.byref(m), 40, 8, 128) == 2 * 3328 + 2 * 256 + 256 + 256 + (256 + 256 + 3 * 256)
    args = (32, 8, 128, 0.1, B.DAG_BF16)
    call = lambda *ptrs, a=args, ws=p, nb=need, meta=m: L.dag_attn_prefill_bwd(
        C.byref(meta) if meta is not None else None, *ptrs, *a, ws, nb, None)
    nine = [p] * 9
    assert call(*nine, nb=need - 1) == -6
    assert call(*nine, ws=None) == -6
    assert call(*nine, a=(32, 8, 128, 0.1, 7)) == -7            # no such dtype
    assert call(*nine, a=(32, 8, 96, 0.1, B.DAG_BF16)) == -7
    assert call(*nine, a=(30, 8, 128, 0.1, B.DAG_BF16)) == -7
    for missing in range(9):
        ptrs = list(nine)
        ptrs[missing] = None
        assert call(*ptrs) == -1
    ptrs = list(nine)
    ptrs[7] = C.c_void_p(FAKE + 2)
    assert call(*ptrs) == -8
    assert call(*nine, meta=None) == -1
    m.tile_m = 32
    assert call(*nine) == -7
    m.tile_m = 64
    empty = B.dag_meta_t()
    empty.tile_m, empty.tile_n, empty.words_per_node = 64, 64, 1
    assert call(*nine, ws=None, nb=0, meta=empty) == 0
