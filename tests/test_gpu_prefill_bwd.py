"""GPU parity: dag_attn_prefill_bwd (through the C ABI) against the fp64 oracle's gradients."""
import numpy as np
import pytest
import torch

from oracle import dag_oracle as orc
from paper_2602_07529_amd import binding as B
from workloads import dags
from tests.gpu_util import DEV, build_meta

pytestmark = pytest.mark.gpu


def check_close(got, ref, dtype, what=""):
    """The forward's tolerances (max |diff| <= 2e-2, Frobenius ratio <= 1e-2) with the absolute
    bound scaled by the largest reference magnitude: gradients are sums over rows and query heads
    and reach several units, where the bf16 rounding of the result alone is 2^-9 of the value."""
    g = got.detach().cpu().to(torch.float64).numpy()
    assert np.isfinite(g).all(), what + ": non-finite output"
    max_abs = float(np.abs(g - ref).max())
    rel = float(np.linalg.norm(g - ref) / max(np.linalg.norm(ref), 1e-30))
    atol = 2e-2 * max(1.0, float(np.abs(ref).max()))
    assert max_abs <= atol and rel <= 1e-2, "%s: max_abs %.3e (tol %.1e) rel %.3e (tol 1e-2)" % (what, max_abs, atol, rel)
    return max_abs, rel


def _forward_backward(dag_list, hq, hkv, d, seed, scale=None, theta=5e5):
    T = int(sum(int(np.sum(L)) for L, _ in dag_list))
    q, k, v = dags.make_qkv(seed, T, hq, hkv, d, 0.7, torch.bfloat16)
    dout = dags.make_qkv(seed + 1, T, hq, hkv, d, 1.0, torch.bfloat16)[0]
    _, meta = build_meta(dag_list, hq, hkv, d, torch.bfloat16)
    qd, kd, vd, dod = q.to(DEV).clone(), k.to(DEV).clone(), v.to(DEV), dout.to(DEV)
    B.dag_rope_qk(meta.get("pos_ids"), qd, kd, theta)
    out = torch.empty_like(qd)
    lse = torch.empty(T, hq, dtype=torch.float32, device=DEV)
    B.dag_attn_prefill(meta, qd, kd, vd, out, lse, softmax_scale=scale)
    dq, dk, dv = torch.full_like(qd, float("nan")), torch.full_like(kd, float("nan")), torch.full_like(vd, float("nan"))
    B.dag_attn_prefill_bwd(meta, qd, kd, vd, out, dod, lse, dq, dk, dv, softmax_scale=scale)
    torch.cuda.synchronize()
    return (qd, kd, v, dout), (dq, dk, dv)


def _check_against_oracle(dag_list, inputs, grads, scale=None):
    """The oracle takes one sequence at a time; the tolerances apply to the whole tensors (a
    single-token sequence has dq = dk = 0 exactly, against which no ratio can be taken)."""
    qd, kd, v, dout = inputs
    refs, t0 = [], 0
    for L, anc in dag_list:
        Tb = int(np.sum(L))
        sl = slice(t0, t0 + Tb)
        refs.append(orc.attn_prefill_bwd(dags.to_f64(qd[sl]), dags.to_f64(kd[sl]), dags.to_f64(v[sl]),
                                         dags.to_f64(dout[sl]), L, anc, scale=scale))
        t0 += Tb
    for x, (name, g) in enumerate(zip(("dq", "dk", "dv"), grads)):
        check_close(g, np.concatenate([r[x] for r in refs]), torch.bfloat16, name)


@pytest.mark.parametrize("hq,hkv,d", [(4, 1, 128), (8, 2, 64), (5, 1, 128), (2, 2, 64), (3, 1, 64), (8, 2, 128),
                                      (8, 1, 64), (9, 1, 128), (14, 2, 64)])   # the last three: more than four query heads per KV head
def test_bwd_small_dags_every_head_grouping(hq, hkv, d):
    rng = np.random.Generator(np.random.PCG64(3000 + hq * 10 + d))
    dag_list = [dags.fork_join(100, [37, 64, 5], 70),               # ragged everywhere
                dags.random_dag(rng, n_nodes=14, depth=4, len_lo=1, len_hi=45)[:2],
                dags.linear_chain([1]),
                dags.linear_chain([200])]
    inputs, grads = _forward_backward(dag_list, hq, hkv, d, 4000 + hq + d)
    _check_against_oracle(dag_list, inputs, grads)


def test_bwd_more_than_64_nodes_and_a_scale():
    rng = np.random.Generator(np.random.PCG64(79))
    L, anc, _, _ = dags.random_dag(rng, n_nodes=90, depth=6, len_lo=1, len_hi=12)
    inputs, grads = _forward_backward([(L, anc)], 4, 1, 128, 35, scale=0.05)
    _check_against_oracle([(L, anc)], inputs, grads, scale=0.05)


def test_bwd_is_deterministic_run_to_run():
    dag_list = [dags.fork_join(300, [100, 90], 50)]
    _, g1 = _forward_backward(dag_list, 8, 2, 128, 52)
    _, g2 = _forward_backward(dag_list, 8, 2, 128, 52)
    for a, b in zip(g1, g2):
        assert torch.equal(a, b)


def test_bwd_linear_chain_equals_library_autograd_of_causal_attention():
    """Independent of the oracle: torch autograd (fp32, CPU) of causal SDPA on the GPU-rotated inputs."""
    dag_list = [dags.linear_chain([50, 150, 56])]
    (qd, kd, v, dout), (dq, dk, dv) = _forward_backward(dag_list, 8, 2, 128, 41)
    tq = qd.float().cpu().permute(1, 0, 2)[None].requires_grad_(True)
    tk = kd.float().cpu().permute(1, 0, 2)[None].requires_grad_(True)
    tv = v.float().permute(1, 0, 2)[None].requires_grad_(True)
    o = torch.nn.functional.scaled_dot_product_attention(tq, tk.repeat_interleave(4, dim=1), tv.repeat_interleave(4, dim=1),
                                                         is_causal=True)
    (o * dout.float().permute(1, 0, 2)[None]).sum().backward()
    for name, g, r in (("dq", dq, tq.grad), ("dk", dk, tk.grad), ("dv", dv, tv.grad)):
        check_close(g, r[0].permute(1, 0, 2).double().numpy(), torch.bfloat16, name + " vs autograd")


def test_bwd_config2_one_sequence_one_kv_group_every_row():
    """Benchmark config 2's DAG (2048 -> 8 x 256 -> 512) at full head counts: the whole batch runs
    on the GPU, one sequence's gradients of KV head 1 and its four query heads against the oracle."""
    c = dags.config(1)
    dag_list = dags.config_dags(c)
    inputs, grads = _forward_backward(dag_list, c["hq"], c["hkv"], c["d"], c["seed"] + 5, theta=c["theta"])
    qd, kd, v, dout = inputs
    L, anc = dag_list[1]
    Tb = int(np.sum(L))
    sl = slice(Tb, 2 * Tb)
    ref = orc.attn_prefill_bwd(dags.to_f64(qd[sl]), dags.to_f64(kd[sl]), dags.to_f64(v[sl]), dags.to_f64(dout[sl]),
                               L, anc, kv_heads=[1])
    check_close(grads[0][sl][:, 4:8], ref[0][:, 4:8], torch.bfloat16, "config 2 dq")
    check_close(grads[1][sl][:, 1], ref[1][:, 1], torch.bfloat16, "config 2 dk")
    check_close(grads[2][sl][:, 1], ref[2][:, 1], torch.bfloat16, "config 2 dv")


def test_bwd_config4_one_sequence_one_kv_group_every_row():
    """Benchmark config 4 (random multi-level DAGs; half of the visited tiles take the per-element
    path): the whole batch runs on the GPU, one sequence's gradients of one KV head and its four
    query heads against the oracle."""
    c = dags.config(3)
    dag_list = dags.config_dags(c)
    inputs, grads = _forward_backward(dag_list, c["hq"], c["hkv"], c["d"], c["seed"] + 6, theta=c["theta"])
    qd, kd, v, dout = inputs
    t0 = int(sum(int(np.sum(L)) for L, _ in dag_list[:2]))
    L, anc = dag_list[2]
    sl = slice(t0, t0 + int(np.sum(L)))
    ref = orc.attn_prefill_bwd(dags.to_f64(qd[sl]), dags.to_f64(kd[sl]), dags.to_f64(v[sl]), dags.to_f64(dout[sl]),
                               L, anc, kv_heads=[3])
    check_close(grads[0][sl][:, 12:16], ref[0][:, 12:16], torch.bfloat16, "config 4 dq")
    check_close(grads[1][sl][:, 3], ref[1][:, 3], torch.bfloat16, "config 4 dk")
    check_close(grads[2][sl][:, 3], ref[2][:, 3], torch.bfloat16, "config 4 dv")


def test_bwd_five_query_heads_per_kv_head_at_4k_tokens():
    """The head grouping of benchmark config 5 (five query heads per KV head) on a fork-join of
    4096 tokens: every gradient element against the oracle."""
    dag_list = [dags.fork_join(2048, [256] * 6, 512)]
    inputs, grads = _forward_backward(dag_list, 10, 2, 128, 88, theta=1e6)
    _check_against_oracle(dag_list, inputs, grads)


def test_bwd_fp32_config1_and_ragged_dags():
    """The fp32 accuracy path (benchmark config 1: 128 -> 4 x 64 -> 64, 4 heads, D 64; then ragged
    DAGs with GQA at D 128): gradients within 1e-4 of the oracle's (absolute bound scaled by the
    largest reference magnitude, as for bf16)."""
    c = dags.config(0)
    rng = np.random.Generator(np.random.PCG64(77))
    for dag_list, hq, hkv, d, scale, theta in [
            (dags.config_dags(c), c["hq"], c["hkv"], c["d"], c["scale"], c["theta"]),
            ([dags.fork_join(70, [33, 64], 31), dags.random_dag(rng, n_nodes=10, depth=4, len_lo=1, len_hi=30)[:2]],
             4, 2, 128, 1.0, 1e4)]:
        T = int(sum(int(np.sum(L)) for L, _ in dag_list))
        q, k, v = dags.make_qkv(61, T, hq, hkv, d, scale, torch.float32)
        dout = dags.make_qkv(62, T, hq, hkv, d, 1.0, torch.float32)[0]
        _, meta = build_meta(dag_list, hq, hkv, d, torch.float32)
        qd, kd, vd, dod = q.to(DEV).clone(), k.to(DEV).clone(), v.to(DEV), dout.to(DEV)
        B.dag_rope_qk(meta.get("pos_ids"), qd, kd, theta)
        out = torch.empty_like(qd)
        lse = torch.empty(T, hq, dtype=torch.float32, device=DEV)
        B.dag_attn_prefill(meta, qd, kd, vd, out, lse)
        dq, dk, dv = torch.full_like(qd, float("nan")), torch.full_like(kd, float("nan")), torch.full_like(vd, float("nan"))
        B.dag_attn_prefill_bwd(meta, qd, kd, vd, out, dod, lse, dq, dk, dv)
        torch.cuda.synchronize()
        refs, t0 = [], 0
        for L, anc in dag_list:
            Tb = int(np.sum(L))
            sl = slice(t0, t0 + Tb)
            refs.append(orc.attn_prefill_bwd(dags.to_f64(qd[sl]), dags.to_f64(kd[sl]), dags.to_f64(v[sl]),
                                             dags.to_f64(dout[sl]), L, anc))
            t0 += Tb
        for x, (name, g) in enumerate(zip(("dq", "dk", "dv"), (dq, dk, dv))):
            ref = np.concatenate([r[x] for r in refs])
            got = g.cpu().double().numpy()
            assert np.isfinite(got).all()
            assert np.abs(got - ref).max() <= 1e-4 * max(1.0, np.abs(ref).max()), name
            assert np.linalg.norm(got - ref) / np.linalg.norm(ref) <= 1e-4, name


def test_bwd_random_batches_on_the_pipelined_kernels():
    """Head dimension 128 with three or more query heads per KV head (the shapes the two pipelined
    kernels take): batches of random DAGs, fork-joins with ragged and with tile-aligned nodes,
    chains; one to three sequences, up to 90 nodes (more than one visibility word), G = 3, 4, 5, 8."""
    rng = np.random.Generator(np.random.PCG64(2026))
    for case in range(12):
        hkv = int(rng.integers(1, 3))
        hq = hkv * int(rng.choice([3, 4, 5, 8]))
        dag_list = []
        for _ in range(int(rng.integers(1, 4))):
            kind = int(rng.integers(0, 4))
            if kind == 0:
                n = int(rng.integers(6, 90))
                L, anc, _, _ = dags.random_dag(rng, n_nodes=n, depth=int(rng.integers(2, min(n, 7))), len_lo=1,
                                               len_hi=int(rng.integers(3, 40)))
                dag_list.append((L, anc))
            elif kind == 1:
                dag_list.append(dags.fork_join(int(rng.integers(1, 400)),
                                               [int(rng.integers(1, 200)) for _ in range(int(rng.integers(1, 6)))],
                                               int(rng.integers(1, 150))))
            elif kind == 2:
                dag_list.append(dags.fork_join(64 * int(rng.integers(1, 5)),
                                               [64 * int(rng.integers(1, 3)) for _ in range(int(rng.integers(2, 5)))],
                                               64 * int(rng.integers(1, 3))))
            else:
                dag_list.append(dags.linear_chain([int(rng.integers(1, 300)) for _ in range(int(rng.integers(1, 4)))]))
        inputs, grads = _forward_backward(dag_list, hq, hkv, 128, 9000 + case)
        _check_against_oracle(dag_list, inputs, grads)


def test_bwd_tiles_made_of_many_short_nodes():
    """The masked iterations build Eq. 3 of a tile from the runs of equal node ids among its 64
    tokens: here tiles of up to 64 runs (64 nodes of one or two tokens), a tile that is one long run
    cut by the diagonal, nodes that end exactly on tile boundaries, and a ragged last tile; one
    visibility word per node, head shapes of both pipelined kernels."""
    rng = np.random.Generator(np.random.PCG64(777))
    L1, anc1, _, _ = dags.random_dag(rng, n_nodes=64, depth=6, len_lo=1, len_hi=2)
    L2, anc2, _, _ = dags.random_dag(rng, n_nodes=40, depth=5, len_lo=1, len_hi=9)
    dag_list = [(L1, anc1), dags.fork_join(64, [1] * 40 + [64, 63], 5), (L2, anc2),
                dags.fork_join(130, [64, 64, 2, 62], 64), dags.linear_chain([1] * 64)]
    for hq, hkv in ((4, 1), (10, 2)):
        inputs, grads = _forward_backward(dag_list, hq, hkv, 128, 600 + hq)
        _check_against_oracle(dag_list, inputs, grads)


@pytest.mark.parametrize("hq,hkv", [(1, 1), (2, 1), (3, 1), (5, 1), (6, 1), (7, 1), (10, 2)])
def test_bwd_left_over_heads_on_four_query_tiles(hq, hkv):
    """Head groupings that leave heads over (not a multiple of four per KV head) run dQ workgroups of one head on four
    consecutive query tiles: sequences of 1, 2, 3, 4, 5 and 9 query tiles and one of a single token
    (groups that end before their fourth tile), a sequence with more than 64 nodes (two visibility
    words: its masked tiles take the general walk with one block-map entry per wave pair), tiles
    that only some of the four query tiles see."""
    rng = np.random.Generator(np.random.PCG64(4242 + hq))
    many = dags.random_dag(rng, n_nodes=90, depth=6, len_lo=1, len_hi=14)[:2]
    dag_list = [dags.linear_chain([1]), dags.linear_chain([50]), dags.fork_join(70, [30, 20], 8),
                dags.fork_join(64, [64, 40], 20), many, dags.fork_join(100, [90, 64, 33], 17),
                dags.random_dag(rng, n_nodes=30, depth=5, len_lo=1, len_hi=40)[:2], dags.fork_join(256, [64] * 4, 64)]
    inputs, grads = _forward_backward(dag_list, hq, hkv, 128, 800 + hq)
    _check_against_oracle(dag_list, inputs, grads)


@pytest.mark.parametrize("hq,hkv", [(5, 1), (4, 1), (6, 2)])
def test_bwd_batch_with_sequences_without_nodes(hq, hkv):
    """Sequences without a node in front of, between and behind the real ones (the tables that count
    query tiles and groups of four query tiles over the sequences must step over them)."""
    real = [dags.fork_join(100, [90, 64, 33], 17), dags.linear_chain([300, 40])]
    lens = np.concatenate([real[0][0], real[1][0]]).astype(np.int32)
    bits = np.concatenate([real[0][1], real[1][1]])
    n0, n1 = len(real[0][0]), len(real[1][0])
    desc = B.DagDesc(np.array([0, 0, n0, n0, n0 + n1, n0 + n1], np.int32), lens, bits, 1, 64, 64)
    meta = B.DagMeta(desc, B.dag_meta_sizes(desc), DEV)
    B.dag_build_meta(desc, meta)
    T = int(lens.sum())
    q, k, v = dags.make_qkv(7, T, hq, hkv, 128, 0.7, torch.bfloat16)
    dout = dags.make_qkv(8, T, hq, hkv, 128, 1.0, torch.bfloat16)[0].to(DEV)
    qd, kd, vd = q.to(DEV), k.to(DEV), v.to(DEV)
    B.dag_rope_qk(meta.get("pos_ids"), qd, kd, 5e5)
    out = torch.empty_like(qd)
    lse = torch.empty(T, hq, dtype=torch.float32, device=DEV)
    B.dag_attn_prefill(meta, qd, kd, vd, out, lse)
    dq, dk, dv = (torch.full_like(x, float("nan")) for x in (qd, kd, vd))
    B.dag_attn_prefill_bwd(meta, qd, kd, vd, out, dout, lse, dq, dk, dv)
    torch.cuda.synchronize()
    _check_against_oracle(real, (qd, kd, v, dout), (dq, dk, dv))
