"""GPU parity: dag_rope_qk (rotary embedding at adaptive positions) against the oracle."""
import numpy as np
import pytest
import torch

from oracle import dag_oracle as orc
from paper_2602_07529_amd import binding as B
from workloads import dags
from tests.gpu_util import DEV, check_close

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("dtype,d,theta", [(torch.float32, 64, 1e4), (torch.bfloat16, 128, 5e5),
                                           (torch.bfloat16, 64, 1e4), (torch.float32, 128, 1e6)])
def test_rope_matches_oracle(dtype, d, theta):
    T, hq, hkv = 77, 6, 2          # 77 tokens: several blocks and a ragged tail
    q, k, _ = dags.make_qkv(11, T, hq, hkv, d, 1.0, dtype)
    rng = np.random.Generator(np.random.PCG64(3))
    pos = rng.integers(0, 60000, size=T).astype(np.int32)
    pos[:3] = [0, 1, 59999]
    qd, kd = q.to(DEV).clone(), k.to(DEV).clone()
    B.dag_rope_qk(torch.from_numpy(pos).to(DEV), qd, kd, theta)
    torch.cuda.synchronize()
    # fp32: only rounding of the fp32 arithmetic; bf16: one rounding of the result (rel 2^-9)
    check_close(qd, orc.rope(dags.to_f64(q), pos, theta), dtype, "q")
    check_close(kd, orc.rope(dags.to_f64(k), pos, theta), dtype, "k")
    if dtype == torch.float32:
        err = (qd.cpu().double().numpy() - orc.rope(dags.to_f64(q), pos, theta))
        assert np.abs(err).max() < 2e-6


def test_rope_only_q_or_only_k_and_zero_tokens():
    q, k, _ = dags.make_qkv(12, 9, 4, 2, 64, 1.0, torch.bfloat16)
    pos = torch.arange(9, dtype=torch.int32, device=DEV)
    qd, kd = q.to(DEV).clone(), k.to(DEV).clone()
    B.dag_rope_qk(pos, qd, None, 1e4)
    B.dag_rope_qk(pos, None, kd, 1e4)
    torch.cuda.synchronize()
    check_close(qd, orc.rope(dags.to_f64(q), np.arange(9), 1e4), torch.bfloat16, "q only")
    check_close(kd, orc.rope(dags.to_f64(k), np.arange(9), 1e4), torch.bfloat16, "k only")
    assert torch.equal(qd[0], q[0].to(DEV))       # position 0 is the identity, bit for bit
    B.dag_rope_qk(pos, qd[:0], kd[:0], 1e4)
