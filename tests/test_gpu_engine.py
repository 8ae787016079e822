"""GPU, end to end: a whole plan generated through the scheduler + append + segment decode, token
by token (given nodes in chunks), gives for every token the DAG-masked attention of the prefill
definition (Eq. 2 + Eq. 3 with adaptive positions) -- the oracle's attn_prefill over the finished
DAG -- and takes the number of steps the oracle's schedule has."""
import numpy as np
import pytest
import torch

from oracle import dag_oracle as orc
from paper_2602_07529_amd import engine
from workloads import dags
from tests.gpu_util import DEV, check_close

pytestmark = pytest.mark.gpu


def _check_plan(parents, L, chunk, hq, hkv, d, seed, theta=1e4):
    L = np.asarray(L, dtype=np.int32)
    anc = dags.bits_from_sets(dags.closure_from_parents(parents))
    T = int(L.sum())
    q, k, v = dags.make_qkv(seed, T, hq, hkv, d, 0.7, torch.bfloat16)
    layers = []
    out, n_steps, _, _ = engine.run_plan(parents, L, q.to(DEV), k.to(DEV), v.to(DEV), theta, chunk=chunk,
                                         on_step=lambda st: layers.append(st["layer"]))
    assert n_steps == len(orc.schedule_steps(parents, L, chunk))
    assert layers == sorted(layers) and layers[-1] == len(orc.frontier_layers(parents)) - 1
    _, pos = orc.token_meta(L, anc)
    ks = orc.rope(dags.to_f64(k), pos, theta)
    ref, _ = orc.attn_prefill(dags.to_f64(q), ks, dags.to_f64(v), L, anc)
    check_close(out, ref, torch.bfloat16, "engine out")
    return n_steps


def test_multilevel_plan_with_a_join_token_by_token_and_in_chunks():
    parents = [[], [0], [0], [1], [1], [2], [2], [2], [3, 4, 5]]
    L = [37, 16, 5, 21, 1, 33, 18, 7, 12]
    serial = sum(L)
    n1 = _check_plan(parents, L, None, 8, 2, 128, 11)
    assert n1 == 37 + 16 + 33 + 12 < serial          # depth of the plan, not its size
    n2 = _check_plan(parents, L, [16, 4, 4, 1, 1, 1, 1, 1, 5], 4, 1, 64, 12)
    assert n2 == 3 + 4 + 33 + 3


def test_random_plan_two_roots_gqa5():
    rng = np.random.Generator(np.random.PCG64(14))
    n = 14
    parents = [sorted(set(int(x) for x in rng.integers(0, v, size=int(rng.integers(1, 3))))) if v > 1 else []
               for v in range(n)]
    L = [int(x) for x in rng.integers(1, 30, size=n)]
    chunk = [8 if not parents[v] else 1 for v in range(n)]
    _check_plan(parents, L, chunk, 5, 1, 128, 13)
