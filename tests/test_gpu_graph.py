"""GPU: the attention entry points can be captured into a HIP graph (no allocation, no memset,
everything on the capturing stream) and replayed: every replay, with eager work and
synchronisations in between, gives the bits of the eager call."""
import numpy as np
import pytest
import torch

from paper_2602_07529_amd import binding as B
from workloads import dags
from tests.gpu_util import DEV, build_meta

pytestmark = pytest.mark.gpu


def _capture_and_replay(step, out, n_replays=3):
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        for _ in range(2):
            step()
        torch.cuda.synchronize()
        eager = out.clone()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=s):
            step()
        torch.cuda.synchronize()
        for _ in range(n_replays):
            out.zero_()          # eager work between the replays
            torch.cuda.synchronize()
            g.replay()
            torch.cuda.synchronize()
            assert torch.equal(out, eager)


@pytest.mark.parametrize("hq,hkv", [(8, 2), (5, 1)])   # four-head items only; a left-over head on 256-row tiles (two launches)
def test_prefill_prepare_and_attention_in_a_graph(hq, hkv):
    dag_list = [dags.fork_join(300, [100, 90, 64], 70), dags.linear_chain([130, 77])]
    T = int(sum(int(np.sum(L)) for L, _ in dag_list))
    d = 128
    q, k, v = dags.make_qkv(17, T, hq, hkv, d, 0.5, torch.bfloat16)
    _, meta = build_meta(dag_list, hq, hkv, d, torch.bfloat16)
    qd, kd, vd = q.to(DEV), k.to(DEV), v.to(DEV)
    B.dag_rope_qk(meta.get("pos_ids"), qd, kd, 5e5)
    out = torch.zeros_like(qd)
    ws = torch.empty(B.dag_prefill_workspace_bytes(meta, hkv, d, B.DAG_BF16), dtype=torch.uint8, device=DEV)

    def step():
        B.dag_prefill_prepare_v(meta, vd, hq, workspace=ws)
        B.dag_attn_prefill(meta, qd, kd, vd, out, workspace=ws, prepared=True)

    _capture_and_replay(step, out)


@pytest.mark.parametrize("hq,hkv,nb", [(8, 2, 4), (10, 2, 7)])   # 16 stacked rows; 35 rows -> wide groups
def test_decode_step_in_a_graph(hq, hkv, nb):
    d = 128
    st = dags.decode_state(700 + hq, n_seqs=2, n_branches=nb, shared_len=300, branch_len=45, hq=hq, hkv=hkv, d=d)
    dd = B.DecodeDesc(st["desc"], DEV)
    kp, vp = st["k_pool"].to(DEV), st["v_pool"].to(DEV)
    k_new, v_new, q = st["k_new"].to(DEV), st["v_new"].to(DEV), st["q"].to(DEV)
    out = torch.zeros_like(q)
    ws = torch.empty(B.dag_decode_workspace_bytes(dd, hq, hkv, d), dtype=torch.uint8, device=DEV)

    def step():
        B.dag_kv_append_rope(dd, k_new, v_new, kp, vp, 5e5)
        B.dag_attn_decode(dd, q, kp, vp, out, ws)

    _capture_and_replay(step, out)


def test_segment_decode_step_in_a_graph():
    """Plan kernel + item kernel + combination of dag_attn_decode_segments captured and replayed;
    between replays a segment grows by one token (its length lives in device memory), so the
    replayed plan differs from the captured one and must still match an eager call."""
    hq, hkv, d = 8, 2, 128
    parents = [[], [0], [0], [1], [1], [2]]
    L = np.asarray([300, 47, 130, 15, 33, 16], dtype=np.int32)
    anc = dags.bits_from_sets(dags.closure_from_parents(parents))
    st = dags.decode_segments_state(23, [(L, anc)], [[3, 4, 5]], hq, hkv, d, junk_scale=0.5)
    sd = B.SegDecodeDesc(st["desc"], DEV)
    kp, vp, q = st["k_pool"].to(DEV), st["v_pool"].to(DEV), st["q"].to(DEV)
    out = torch.zeros_like(q)
    ws = torch.empty(B.dag_decode_segments_workspace_bytes(sd, hq, hkv, d), dtype=torch.uint8, device=DEV)
    step = lambda: B.dag_attn_decode_segments(sd, q, kp, vp, out, ws)
    _capture_and_replay(step, out)
    # same graph, longer segment: node 3 now shows its 16th slot (junk values, finite) as a token
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=s):
            step()
        sd.t["seg_len"][3] += 1
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        replayed = out.clone()
        out.zero_()
        step()
        torch.cuda.synchronize()
        assert torch.equal(out, replayed)
        assert not torch.equal(out[0], torch.zeros_like(out[0]))


def test_paged_prefill_in_a_graph():
    """Table kernels and the attention launch of dag_attn_prefill_paged, replayed."""
    from tests.test_gpu_prefill_paged import _multilevel
    hq, hkv, d = 8, 2, 128
    st = dags.decode_segments_state(33, [_multilevel(6)], [[8, 6, 4]], hq, hkv, d, kv_scale=0.7, q_scale=0.7,
                                    new_tokens=[[72, 100, 6]])
    pd = B.PagedPrefillDesc(st["paged"], DEV)
    kp, vp, q = st["k_pool"].to(DEV), st["v_pool"].to(DEV), st["q"].to(DEV)
    out = torch.zeros_like(q)
    ws = torch.empty(B.dag_prefill_paged_workspace_bytes(pd), dtype=torch.uint8, device=DEV)
    _capture_and_replay(lambda: B.dag_attn_prefill_paged(pd, q, kp, vp, out, ws), out)
