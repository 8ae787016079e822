"""GPU parity: dag_attn_prefill_paged (through the C ABI) against the oracle's segment attention with
per-reader visible lengths, which is pinned to the DAG-masked prefill definition: the new tokens of
nodes prefilled against cached, paged KV of their predecessors."""
import numpy as np
import pytest
import torch

from oracle import dag_oracle as orc
from paper_2602_07529_amd import binding as B
from workloads import dags
from tests.gpu_util import DEV, check_close

pytestmark = pytest.mark.gpu


def _gpu_prefill_paged(st, hq, hkv, d, want_lse=False):
    pd = B.PagedPrefillDesc(st["paged"], DEV)
    kp, vp, qd = st["k_pool"].to(DEV), st["v_pool"].to(DEV), st["q"].to(DEV)
    out = torch.full_like(qd, float("nan"))
    lse = torch.full((qd.shape[0], hq), float("nan"), dtype=torch.float32, device=DEV) if want_lse else None
    ws = torch.full((max(1, B.dag_prefill_paged_workspace_bytes(pd)),), 0x55, dtype=torch.uint8, device=DEV)
    B.dag_attn_prefill_paged(pd, qd, kp, vp, out, ws, lse=lse)
    torch.cuda.synchronize()
    return (out, lse) if want_lse else out


def _multilevel(scale_len=1):
    """root -> (a, b); a -> (a0, a1); b -> (b0, b1, b2); one join of a0, a1, b0; every length
    ragged against the page size."""
    parents = [[], [0], [0], [1], [1], [2], [2], [2], [3, 4, 5]]
    L = np.asarray([37, 16, 5, 21, 1, 33, 18, 7, 12], dtype=np.int32) * scale_len
    if scale_len > 1:
        L = L + np.asarray([3, 0, 1, 5, 0, 2, 7, 0, 9], dtype=np.int32)
    return L, dags.bits_from_sets(dags.closure_from_parents(parents))


@pytest.mark.parametrize("hq,hkv,d,scale_len,new", [(8, 2, 128, 1, [12, 5, 1]), (4, 1, 64, 1, [12, 18, 1]),
                                                    (8, 2, 128, 12, [150, 64, 1]), (5, 1, 128, 3, [40, 33, 2]),
                                                    (4, 1, 128, 40, [489, 727, 40]), (8, 1, 64, 23, [285, 1, 23]),
                                                    (2, 2, 128, 7, [93, 133, 7])])
def test_new_tokens_of_a_join_a_leaf_and_an_inner_node_every_row(hq, hkv, d, scale_len, new):
    """The last n tokens (in two cases the whole node) of a join, of a leaf and of an inner node are
    prefilled together against the paged context; contexts of up to seven ragged segments, new
    tokens over several query tiles, tiles that straddle segment ends; every row."""
    dag_list = [_multilevel(scale_len)]
    st = dags.decode_segments_state(700 + hq + scale_len, dag_list, [[8, 6, 4]], hq, hkv, d, kv_scale=0.7,
                                    q_scale=0.7, new_tokens=[new])
    out = _gpu_prefill_paged(st, hq, hkv, d)
    ref = orc.attn_decode_segments(st["desc"], dags.to_f64(st["q"]), dags.to_f64(st["k_pool"]), dags.to_f64(st["v_pool"]))
    check_close(out, ref, torch.bfloat16, "paged prefill out")


def test_a_700_token_node_against_a_1000_token_parent_equals_the_packed_prefill():
    """Against the oracle on sampled rows, and every row (output and log-sum-exp) against the packed
    prefill kernel for the same tokens."""
    from tests.gpu_util import run_prefill
    hq, hkv, d = 4, 1, 128
    dag = dags.linear_chain([1000, 700])
    st = dags.decode_segments_state(81, [dag], [[1]], hq, hkv, d, kv_scale=0.7, q_scale=0.7, new_tokens=[[700]])
    out, lse = _gpu_prefill_paged(st, hq, hkv, d, want_lse=True)
    rows = [0, 1, 15, 16, 17, 63, 64, 319, 320, 321, 350, 698, 699]
    ref = orc.attn_decode_segments(st["desc"], dags.to_f64(st["q"]), dags.to_f64(st["k_pool"]), dags.to_f64(st["v_pool"]),
                                   branches=rows)
    check_close(out[rows], ref[rows], torch.bfloat16, "paged prefill out")
    q_tok, k_tok, v_tok = st["tokens"][0]
    o_pre, l_pre, _, _, _ = run_prefill([dag], q_tok, k_tok, v_tok, 1e4, rope=False, want_lse=True)
    assert (out.float().cpu() - o_pre.float().cpu()[1000:]).abs().max().item() < 4e-2
    assert (lse.cpu() - l_pre.cpu()[1000:]).abs().max().item() < 2e-2


def test_many_nodes_with_and_without_new_tokens_sampled_rows():
    """Twelve fork-join sequences, every branch and the join with its own number of new tokens (64
    to 300, some none): items of very different length through the work counter."""
    hq, hkv, d = 8, 2, 128
    rng = np.random.Generator(np.random.PCG64(5))
    dag_list, live, new = [], [], []
    for b in range(12):
        nb = int(rng.integers(2, 6))
        dag_list.append(dags.fork_join(int(rng.integers(200, 1500)), [int(rng.integers(64, 400)) for _ in range(nb)],
                                       int(rng.integers(64, 300))))
        L = dag_list[-1][0]
        live.append(list(range(1, nb + 2)))
        new.append([int(min(L[v], rng.integers(64, 300))) if rng.random() < 0.8 else 1 for v in live[-1]])
    st = dags.decode_segments_state(19, dag_list, live, hq, hkv, d, kv_scale=0.7, q_scale=0.7, new_tokens=new,
                                    keep_tokens=False)
    out = _gpu_prefill_paged(st, hq, hkv, d)
    assert torch.isfinite(out.float()).all()
    rows = sorted(set(int(x) for x in rng.integers(0, st["q"].shape[0], 48)) | {0, st["q"].shape[0] - 1})
    ref = orc.attn_decode_segments(st["desc"], dags.to_f64(st["q"]), dags.to_f64(st["k_pool"]), dags.to_f64(st["v_pool"]),
                                   branches=rows)
    check_close(out[rows], ref[rows], torch.bfloat16, "paged prefill out")


def test_two_calls_in_a_row_share_a_workspace_and_no_node_is_fine():
    hq, hkv, d = 4, 1, 128
    st = dags.decode_segments_state(3, [_multilevel(5)], [[8, 6]], hq, hkv, d, kv_scale=0.7, q_scale=0.7,
                                    new_tokens=[[60, 90]])
    a = _gpu_prefill_paged(st, hq, hkv, d)
    b = _gpu_prefill_paged(st, hq, hkv, d)
    assert torch.equal(a, b)
    empty = dict(st["paged"])
    for k in ("q_off", "ctx_page_off"):
        empty[k] = np.zeros(1, np.int32)
    pd = B.PagedPrefillDesc(empty, DEV)
    q0 = torch.zeros((0, hq, d), dtype=torch.bfloat16, device=DEV)
    B.dag_attn_prefill_paged(pd, q0, st["k_pool"].to(DEV), st["v_pool"].to(DEV), q0.clone(),
                             torch.empty(1, dtype=torch.uint8, device=DEV))
