"""GPU parity: dag_attn_decode_segments (through the C ABI) against the oracle: contexts as lists
of KV segments with their own lengths, several sharing levels, joins of unequal branches."""
import numpy as np
import pytest
import torch

from oracle import dag_oracle as orc
from paper_2602_07529_amd import binding as B
from workloads import dags
from tests.gpu_util import DEV, check_close

pytestmark = pytest.mark.gpu


def _gpu_decode_segments(desc, q, k_pool, v_pool, hq, hkv, d, scale=None):
    sd = B.SegDecodeDesc(desc, DEV)
    kp, vp, qd = k_pool.to(DEV), v_pool.to(DEV), q.to(DEV)
    out = torch.full_like(qd, float("nan"))
    ws = torch.empty(max(1, B.dag_decode_segments_workspace_bytes(sd, hq, hkv, d)), dtype=torch.uint8, device=DEV)
    B.dag_attn_decode_segments(sd, qd, kp, vp, out, ws, softmax_scale=scale)
    torch.cuda.synchronize()
    return out


def _multilevel(scale_len=1):
    """root -> (a, b); a -> (a0, a1); b -> (b0, b1, b2); one join of a0, a1, b0; every length
    ragged against the page size."""
    parents = [[], [0], [0], [1], [1], [2], [2], [2], [3, 4, 5]]
    L = np.asarray([37, 16, 5, 21, 1, 33, 18, 7, 12], dtype=np.int32) * scale_len
    if scale_len > 1:
        L = L + np.asarray([3, 0, 1, 5, 0, 2, 7, 0, 9], dtype=np.int32)
    return L, dags.bits_from_sets(dags.closure_from_parents(parents))


@pytest.mark.parametrize("hq,hkv,d,scale_len", [(8, 2, 128, 1), (4, 1, 64, 1), (5, 1, 128, 1), (32, 8, 128, 1),
                                                (8, 2, 128, 40), (6, 2, 64, 23), (16, 1, 64, 5), (24, 2, 128, 2)])
def test_multilevel_dags_every_live_branch(hq, hkv, d, scale_len):
    """Two multi-level DAGs and a random one: live leaves, a live join and a live inner node; the
    junk in the unused slots of partly filled pages must not leak (the oracle never reads it)."""
    rng = np.random.Generator(np.random.PCG64(300 + hq + d))
    rd = dags.random_dag(rng, n_nodes=20, depth=5, len_lo=1, len_hi=70)[:2]
    dag_list = [_multilevel(scale_len), _multilevel(1), rd]
    live = [[8, 6, 7, 4], [3, 5], [19, 18, 17, 12, 7]]
    st = dags.decode_segments_state(900 + hq + scale_len, dag_list, live, hq, hkv, d, kv_scale=0.7, q_scale=0.7)
    out = _gpu_decode_segments(st["desc"], st["q"], st["k_pool"], st["v_pool"], hq, hkv, d)
    ref = orc.attn_decode_segments(st["desc"], dags.to_f64(st["q"]), dags.to_f64(st["k_pool"]), dags.to_f64(st["v_pool"]))
    check_close(out, ref, torch.bfloat16, "segment decode out")


def test_matches_dag_masked_prefill_rows_on_the_gpu_too():
    """The same frontier through the prefill kernel: the decode output of a live node equals the
    prefill output row of its last token (both GPU paths, bf16 tolerance twice)."""
    from tests.gpu_util import run_prefill
    hq, hkv, d = 8, 2, 128
    dag_list = [_multilevel(9)]
    st = dags.decode_segments_state(77, dag_list, [[8, 6, 7, 4]], hq, hkv, d, kv_scale=0.7, q_scale=0.7)
    out = _gpu_decode_segments(st["desc"], st["q"], st["k_pool"], st["v_pool"], hq, hkv, d)
    q_tok, k_tok, v_tok = st["tokens"][0]
    o_pre, _, _, _, _ = run_prefill(dag_list, q_tok, k_tok, v_tok, 1e4, rope=False)
    rows = torch.as_tensor(st["live_tok"])
    diff = (out.float().cpu() - o_pre.float().cpu()[rows]).abs().max().item()
    assert diff < 4e-2, diff


def test_many_readers_stack_into_several_row_blocks():
    """One root read by 45 live leaves with 4 query heads per KV head: 180 stacked rows, six row
    blocks, the last one partly filled; leaves of one token up to 40 tokens."""
    hq, hkv, d = 8, 2, 128
    n = 45
    parents = [[]] + [[0]] * n
    L = np.asarray([333] + [1 + (7 * i) % 40 for i in range(n)], dtype=np.int32)
    anc = dags.bits_from_sets(dags.closure_from_parents(parents))
    st = dags.decode_segments_state(41, [(L, anc)], [list(range(1, n + 1))], hq, hkv, d, kv_scale=0.7, q_scale=0.7)
    out = _gpu_decode_segments(st["desc"], st["q"], st["k_pool"], st["v_pool"], hq, hkv, d)
    ref = orc.attn_decode_segments(st["desc"], dags.to_f64(st["q"]), dags.to_f64(st["k_pool"]), dags.to_f64(st["v_pool"]))
    check_close(out, ref, torch.bfloat16, "wide segment decode out")


def test_long_segments_cross_the_page_id_window_and_several_splits(monkeypatch):
    """A 2,500-token root (157 pages) in slices of 70 pages: page ids are fetched 64 at a time and
    a slice crosses a window; the last slice is short and ends in a partly filled page."""
    monkeypatch.setenv("DAGATTN_DECODE_CHUNK_SEG", "70")
    hq, hkv, d = 8, 2, 128
    parents = [[], [0], [0], [1, 2]]
    L = np.asarray([2500, 1130, 17, 3], dtype=np.int32)
    anc = dags.bits_from_sets(dags.closure_from_parents(parents))
    st = dags.decode_segments_state(43, [(L, anc)], [[3, 1]], hq, hkv, d, kv_scale=0.7, q_scale=0.7)
    out = _gpu_decode_segments(st["desc"], st["q"], st["k_pool"], st["v_pool"], hq, hkv, d)
    ref = orc.attn_decode_segments(st["desc"], dags.to_f64(st["q"]), dags.to_f64(st["k_pool"]), dags.to_f64(st["v_pool"]))
    check_close(out, ref, torch.bfloat16, "long segment decode out")


def test_degenerate_descriptions():
    """Segments nobody reads, an empty segment among a branch's segments, a branch whose context
    is its own single token (output = its value vector), and a branch that reads nothing (zeros)."""
    hq, hkv, d = 4, 2, 64
    L, anc = dags.linear_chain([20, 1])
    st = dags.decode_segments_state(45, [(L, anc), dags.linear_chain([1])], [[0], [0]], hq, hkv, d)
    desc = dict(st["desc"])
    # segments: 0 (20 tokens, read by branch 0), 1 (1 token, nobody), 2 (1 token, branch 1);
    # add an empty segment 3 read by branch 0 and a third branch that reads nothing
    desc["n_segments"] = 4
    desc["seg_len"] = np.concatenate([desc["seg_len"], [0]]).astype(np.int32)
    desc["seg_page_off"] = np.concatenate([desc["seg_page_off"], desc["seg_page_off"][-1:]]).astype(np.int32)
    desc["seg_reader_off"] = np.asarray([0, 1, 1, 2, 3], dtype=np.int32)
    desc["seg_readers"] = np.asarray([0, 1, 0], dtype=np.int32)
    desc["n_live"] = 3
    desc["branch_seg_off"] = np.asarray([0, 2, 3, 3], dtype=np.int32)
    desc["branch_segs"] = np.asarray([3, 0, 2], dtype=np.int32)
    dags.add_branch_entries(desc)
    assert list(desc["branch_entries"]) == [2, 0, 1]
    q = torch.cat([st["q"], st["q"][:1]])
    out = _gpu_decode_segments(desc, q, st["k_pool"], st["v_pool"], hq, hkv, d)
    ref = orc.attn_decode_segments(desc, dags.to_f64(q), dags.to_f64(st["k_pool"]), dags.to_f64(st["v_pool"]),
                                   branches=[0, 1])
    check_close(out[:2], ref[:2], torch.bfloat16, "degenerate segment decode out")
    page = int(desc["seg_pages"][desc["seg_page_off"][2]])
    v_tok = st["v_pool"][page, :, :, 0]                       # [hkv][d]: the only visible value
    assert torch.equal(out[1].cpu(), v_tok.repeat_interleave(hq // hkv, dim=0))
    assert torch.equal(out[2].cpu(), torch.zeros_like(out[2].cpu()))


def test_config3_as_segments_sampled_branches_and_against_the_two_level_entry_point():
    """Benchmark config 3 (16 groups x 8 branches, 8192 shared + 1024 own tokens) written as 144
    segments: sampled branches against the oracle, all branches against dag_attn_decode."""
    c = dags.config(2)
    hq, hkv, d = c["hq"], c["hkv"], c["d"]
    st = dags.decode_state(c["seed"], c["n_seqs"], c["n_branch"], c["shared"], c["branch"], hq, hkv, d)
    sdesc = dags.segments_from_decode_desc(st["desc"])
    out = _gpu_decode_segments(sdesc, st["q"], st["k_pool"], st["v_pool"], hq, hkv, d)
    dd = B.DecodeDesc(st["desc"], DEV)
    kp, vp, q = st["k_pool"].to(DEV), st["v_pool"].to(DEV), st["q"].to(DEV)
    out2 = torch.empty_like(q)
    ws = torch.empty(B.dag_decode_workspace_bytes(dd, hq, hkv, d), dtype=torch.uint8, device=DEV)
    B.dag_attn_decode(dd, q, kp, vp, out2, ws)
    torch.cuda.synchronize()
    assert (out.float() - out2.float()).abs().max().item() < 2e-2
    branches = [0, 7, 64, 127]
    ref = orc.attn_decode_segments(sdesc, dags.to_f64(st["q"]), dags.to_f64(st["k_pool"]), dags.to_f64(st["v_pool"]),
                                   branches=branches)
    check_close(out[branches], ref[branches], torch.bfloat16, "config 3 as segments")


@pytest.mark.parametrize("hq,hkv,d,scale_len,new", [(8, 2, 128, 1, [12, 5, 1]), (4, 1, 64, 1, [12, 18, 1]),
                                                    (8, 2, 128, 12, [150, 64, 1]), (5, 1, 128, 3, [40, 33, 2])])
def test_incremental_prefill_of_new_nodes_against_the_cached_context(hq, hkv, d, scale_len, new):
    """Per-reader visible lengths: the last n tokens of a join, of a leaf and of an inner node are
    prefilled together against the paged context (each new token sees its node up to itself and
    the ancestors' segments in full); every row against the oracle, which is pinned to the
    DAG-masked prefill rows.  150 new tokens x 4 heads = 19 row blocks over a 153-token segment:
    row blocks that see nothing of a slice, blocks that end inside a page."""
    dag_list = [_multilevel(scale_len)]
    st = dags.decode_segments_state(600 + hq + scale_len, dag_list, [[8, 6, 4]], hq, hkv, d, kv_scale=0.7,
                                    q_scale=0.7, new_tokens=[new])
    out = _gpu_decode_segments(st["desc"], st["q"], st["k_pool"], st["v_pool"], hq, hkv, d)
    ref = orc.attn_decode_segments(st["desc"], dags.to_f64(st["q"]), dags.to_f64(st["k_pool"]), dags.to_f64(st["v_pool"]))
    check_close(out, ref, torch.bfloat16, "incremental prefill out")


def test_incremental_prefill_in_slices_equals_the_prefill_kernel(monkeypatch):
    """A 700-token node prefilled whole against a 1,000-token parent, in page slices of 20 (so
    that slices lie entirely past the first rows' limits): against the oracle and against the
    prefill kernel's rows for the same tokens."""
    from tests.gpu_util import run_prefill
    monkeypatch.setenv("DAGATTN_DECODE_CHUNK_SEG", "20")
    hq, hkv, d = 4, 1, 128
    dag = dags.linear_chain([1000, 700])
    st = dags.decode_segments_state(81, [dag], [[1]], hq, hkv, d, kv_scale=0.7, q_scale=0.7, new_tokens=[[700]])
    out = _gpu_decode_segments(st["desc"], st["q"], st["k_pool"], st["v_pool"], hq, hkv, d)
    rows = [0, 1, 15, 16, 17, 319, 320, 321, 350, 698, 699]
    ref = orc.attn_decode_segments(st["desc"], dags.to_f64(st["q"]), dags.to_f64(st["k_pool"]), dags.to_f64(st["v_pool"]),
                                   branches=rows)
    check_close(out[rows], ref[rows], torch.bfloat16, "sliced incremental prefill out")
    q_tok, k_tok, v_tok = st["tokens"][0]
    o_pre, _, _, _, _ = run_prefill([dag], q_tok, k_tok, v_tok, 1e4, rope=False)
    assert (out.float().cpu() - o_pre.float().cpu()[1000:]).abs().max().item() < 4e-2
