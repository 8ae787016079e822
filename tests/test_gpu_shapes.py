"""GPU parity on head configurations and batch shapes beside the benchmark ones: one seeded batch of
ragged random DAGs per head configuration (sampled rows of every sequence, output and log-sum-exp),
paged prefill and wide / narrow decode on odd shapes, all against the oracle."""
import numpy as np
import pytest
import torch

from oracle import dag_oracle as orc
from paper_2602_07529_amd import binding as B
from workloads import dags
from tests.gpu_util import DEV, check_close, oracle_prefill, run_prefill

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("hq,hkv,d", [(1, 1, 128), (2, 1, 64), (3, 1, 128), (7, 1, 64), (10, 2, 128), (12, 2, 64),
                                      (13, 1, 128), (6, 6, 64)])
def test_prefill_batches_of_ragged_random_dags(hq, hkv, d):
    rng = np.random.Generator(np.random.PCG64(9900 + 16 * hq + d))
    dag_list = [dags.random_dag(rng, n_nodes=int(rng.integers(14, 60)), depth=int(rng.integers(2, 7)), len_lo=1,
                                len_hi=int(rng.integers(5, 120)))[:2] for _ in range(int(rng.integers(1, 9)))]
    dag_list.append(dags.linear_chain([int(rng.integers(1, 700))]))
    T = int(sum(int(np.sum(L)) for L, _ in dag_list))
    q, k, v = dags.make_qkv(500 + hq, T, hq, hkv, d, 0.5, torch.bfloat16)
    out, lse, _, _, _ = run_prefill(dag_list, q, k, v, 5e5, want_lse=True)
    ref, ref_lse, rows = oracle_prefill(dag_list, q, k, v, 5e5, rows_per_seq=40, seed=hq)
    check_close(out[rows], ref[rows], torch.bfloat16, "prefill")
    assert np.abs(lse.cpu().double().numpy()[rows] - ref_lse[rows]).max() < 2e-2


@pytest.mark.parametrize("hq,hkv,d,nb,shared,own", [(40, 8, 128, 32, 513, 17), (15, 3, 64, 8, 1000, 333),
                                                    (32, 4, 128, 5, 2049, 1), (24, 1, 128, 2, 300, 300),
                                                    (64, 2, 64, 3, 129, 65), (18, 2, 128, 4, 16, 16)])
def test_decode_odd_group_shapes_every_branch(hq, hkv, d, nb, shared, own):
    """Three sibling groups each: 160, 40, 40, 48, 96 and 36 stacked rows per KV head (wide and
    narrow), contexts that end inside a page, a block, a slice."""
    st = dags.decode_state(900 + hq + nb, 3, nb, shared, own, hq, hkv, d, kv_scale=0.5, q_scale=0.5)
    dd = B.DecodeDesc(st["desc"], DEV)
    kp, vp = st["k_pool"].to(DEV), st["v_pool"].to(DEV)
    B.dag_kv_append_rope(dd, st["k_new"].to(DEV), st["v_new"].to(DEV), kp, vp, 5e5)
    qd = st["q"].to(DEV)
    out = torch.empty_like(qd)
    ws = torch.empty(B.dag_decode_workspace_bytes(dd, hq, hkv, d), dtype=torch.uint8, device=DEV)
    B.dag_attn_decode(dd, qd, kp, vp, out, ws)
    torch.cuda.synchronize()
    ref = orc.attn_decode(st["desc"], dags.to_f64(st["q"]), dags.to_f64(kp), dags.to_f64(vp))
    check_close(out, ref, torch.bfloat16, "decode")
