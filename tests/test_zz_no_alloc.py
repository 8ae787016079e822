"""GPU: dag_attn_decode_static (the entry point that allocates nothing: its partial results live in
a device array of the library) against dag_attn_decode, through the C ABI: two calls in a row, the
second with a smaller input, each bit for bit what the workspace variant gives, and within the
parity tolerances of the oracle."""
import numpy as np
import pytest
import torch

from oracle import dag_oracle as orc
from paper_2602_07529_amd import binding as B
from workloads import dags
from tests.gpu_util import DEV, check_close

pytestmark = pytest.mark.gpu


def _both(st, hq, hkv, d):
    dd = B.DecodeDesc(st["desc"], DEV)
    kp, vp, q = st["k_pool"].to(DEV), st["v_pool"].to(DEV), st["q"].to(DEV)
    need = B.dag_decode_workspace_bytes(dd, hq, hkv, d)
    assert 0 < need <= B.DECODE_STATIC_SCRATCH_BYTES
    ws = torch.empty(need, dtype=torch.uint8, device=DEV)
    want = torch.empty_like(q)
    B.dag_attn_decode(dd, q, kp, vp, want, ws)
    torch.cuda.synchronize()
    got = torch.full_like(q, float("nan"))
    mem0 = torch.cuda.memory_allocated()
    B.dag_attn_decode_static(dd, q, kp, vp, got)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == mem0
    return got, want, kp, vp


@pytest.mark.parametrize("hq,hkv,d,nb,first,second", [
    (32, 8, 128, 8, (4, 2048, 300), (2, 513, 37)),     # single-wave items (32 stacked rows)
    (40, 8, 128, 32, (2, 4096, 130), (1, 700, 18)),    # wide sibling groups (160 stacked rows)
    (8, 2, 64, 3, (3, 100, 40), (1, 0, 5)),            # head_dim 64; the second call has no shared context
])
def test_static_decode_two_calls_in_a_row_second_smaller(hq, hkv, d, nb, first, second):
    for i, (n_seqs, shared, own) in enumerate((first, second)):
        st = dags.decode_state(3100 + 10 * hq + i, n_seqs=n_seqs, n_branches=nb, shared_len=shared, branch_len=own,
                               hq=hq, hkv=hkv, d=d, kv_scale=0.5, q_scale=0.5)
        got, want, kp, vp = _both(st, hq, hkv, d)
        assert torch.equal(got, want), "call %d differs from dag_attn_decode" % i
        branches = sorted({0, st["desc"]["n_live"] - 1, st["desc"]["n_live"] // 2})
        ref = orc.attn_decode(st["desc"], dags.to_f64(st["q"]), dags.to_f64(kp), dags.to_f64(vp), branches=branches)
        check_close(got[branches], ref[branches], torch.bfloat16, "static decode, call %d" % i)


def test_static_decode_refuses_what_its_array_cannot_hold():
    st = dags.decode_state(3200, n_seqs=1, n_branches=2, shared_len=64, branch_len=8, hq=8, hkv=2, d=128)
    desc = dict(st["desc"])
    dd = B.DecodeDesc(desc, DEV)
    dd.c.max_shared_pages = 1 << 20          # the host bound sizes the partials: far beyond the array
    dd.c.max_group_size = 1 << 10
    q = st["q"].to(DEV)
    with pytest.raises(B.DagError) as e:
        B.dag_attn_decode_static(dd, q, st["k_pool"].to(DEV), st["v_pool"].to(DEV), torch.empty_like(q))
    assert e.value.code == -6
