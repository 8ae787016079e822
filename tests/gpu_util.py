"""Helpers shared by the GPU parity tests: run the library through its binding, run the oracle on
the same inputs, and compare to the stated tolerances."""
import numpy as np
import torch

from oracle import dag_oracle as orc
from paper_2602_07529_amd import binding as B
from workloads import dags

DEV = "cuda:0"

# Tolerances of the parity bar: bf16 outputs max-abs 2e-2 and relative (Frobenius) 1e-2;
# fp32 path 1e-4 for both.
TOL = {torch.bfloat16: (2e-2, 1e-2), torch.float32: (1e-4, 1e-4)}


def build_meta(dag_list, hq, hkv, d, dtype, flags=0):
    code = B.DAG_F32 if dtype == torch.float32 else B.DAG_BF16
    tm, tn = B.dag_prefill_tile_shape(hq, hkv, d, code)
    off, lens, bits, W = dags.batch_desc(dag_list)
    desc = B.DagDesc(off, lens, bits, W, tm, tn, flags)
    sizes = B.dag_meta_sizes(desc)
    meta = B.DagMeta(desc, sizes, DEV)
    B.dag_build_meta(desc, meta)
    return desc, meta


def oracle_meta(dag_list, tm, tn):
    """Oracle tables for a batch, concatenated the way the library lays them out."""
    out = dict(cu_seqlens=[0], tok_node=[], pos_ids=[], node_tok_start=[], node_pos_start=[], node_vis=[],
               qtile_start=[0], block_map_off=[0], block_map=[], rowptr=[0], col=[], flag=[], cnt=[],
               useful_pairs=[])
    W = max(a.shape[1] for _, a in dag_list) if dag_list else 1
    for L, anc in dag_list:
        tok_start, pos_start = orc.node_tables(L, anc)
        tn_, pos = orc.token_meta(L, anc)
        bm = orc.block_map(L, anc, tm, tn)
        out.setdefault("bmaps", []).append(bm)
        rp, col, flag, nfull = orc.block_map_csr_full_first(bm)
        out.setdefault("nfull", []).append(nfull)
        out["cu_seqlens"].append(out["cu_seqlens"][-1] + len(tn_))
        out["tok_node"].append(tn_)
        out["pos_ids"].append(pos)
        out["node_tok_start"].append(tok_start[:-1])
        out["node_pos_start"].append(pos_start)
        vis = np.zeros((anc.shape[0], W), dtype=np.uint64)
        vis[:, :anc.shape[1]] = orc.node_vis(anc)
        out["node_vis"].append(vis.reshape(-1))
        out["qtile_start"].append(out["qtile_start"][-1] + bm.shape[0])
        out["block_map_off"].append(out["block_map_off"][-1] + bm.size)
        out["block_map"].append(bm.reshape(-1))
        base = out["rowptr"][-1]
        out["rowptr"].extend((base + rp[1:]).tolist())
        out["col"].append(col)
        out["flag"].append(flag)
        out["cnt"].extend(np.diff(rp).tolist())
        out["useful_pairs"].append(orc.useful_pairs(L, anc))
    cat = lambda xs, dt: np.concatenate(xs).astype(dt) if xs else np.zeros(0, dt)
    res = dict(
        cu_seqlens=np.array(out["cu_seqlens"]), tok_node=cat(out["tok_node"], np.int64),
        pos_ids=cat(out["pos_ids"], np.int64), node_tok_start=cat(out["node_tok_start"], np.int64),
        node_pos_start=cat(out["node_pos_start"], np.int64), node_vis=cat(out["node_vis"], np.uint64),
        qtile_start=np.array(out["qtile_start"]), block_map_off=np.array(out["block_map_off"]),
        block_map=cat(out["block_map"], np.uint8), qtile_rowptr=np.array(out["rowptr"]),
        qtile_col=cat(out["col"], np.int64), qtile_flag=cat(out["flag"], np.uint8),
        qtile_nfull=cat(out.get("nfull", []), np.int64),
        useful_pairs=np.array(out["useful_pairs"], dtype=np.int64))
    cnt = np.array(out["cnt"], dtype=np.int64)
    # launch order and mask-free counts: the oracle's statement of the library's rules
    seq_of = np.repeat(np.arange(len(dag_list)), np.diff(res["qtile_start"]))
    seq_T = np.diff(res["cu_seqlens"])
    order, mask_free = orc.launch_tables(out["bmaps"], seq_T, tn)
    res["qtile_order"] = order
    # launch descriptors: {token offset, tokens, first row, CSR start, tiles, mask-free tiles, node offset, tile id}
    node_start = np.concatenate([[0], np.cumsum([len(L) for L, _ in dag_list])])
    ktiles = [-(-int(np.sum(L)) // tn) for L, _ in dag_list]
    res["ktile_start"] = np.concatenate([[0], np.cumsum(ktiles)]).astype(np.int64)
    desc = np.zeros((len(cnt), 8), dtype=np.int64)
    for oi, qt in enumerate(order):
        b = int(seq_of[qt])
        desc[oi] = [res["cu_seqlens"][b], seq_T[b], (qt - res["qtile_start"][b]) * tm, res["qtile_rowptr"][qt],
                    cnt[qt], mask_free[qt], node_start[b], res["ktile_start"][b]]
    res["qtile_desc"] = desc.reshape(-1)
    return res


def assert_meta_equal(meta, ref):
    torch.cuda.synchronize()
    nnz = int(ref["qtile_rowptr"][-1])
    for name in ("cu_seqlens", "tok_node", "pos_ids", "node_tok_start", "node_pos_start", "qtile_start", "ktile_start",
                 "block_map_off", "block_map", "qtile_rowptr", "qtile_nfull", "qtile_order", "qtile_desc",
                 "useful_pairs"):
        got = meta.get(name).cpu().numpy().astype(np.int64)
        assert got.shape == ref[name].shape, name
        assert np.array_equal(got, ref[name].astype(np.int64)), name
    got = meta.get("node_vis").cpu().numpy().view(np.uint64)
    assert np.array_equal(got, ref["node_vis"]), "node_vis"
    assert np.array_equal(meta.t["qtile_col"][:nnz].cpu().numpy().astype(np.int64), ref["qtile_col"]), "qtile_col"
    assert np.array_equal(meta.t["qtile_flag"][:nnz].cpu().numpy(), ref["qtile_flag"]), "qtile_flag"


def check_close(got, ref, dtype, what=""):
    """got: torch tensor (any float dtype); ref: numpy fp64.  Applies the parity tolerances."""
    g = got.detach().cpu().to(torch.float64).numpy()
    assert np.isfinite(g).all(), what + ": non-finite output"
    diff = np.abs(g - ref)
    max_abs = float(diff.max()) if diff.size else 0.0
    rel = float(np.linalg.norm(g - ref) / max(np.linalg.norm(ref), 1e-30)) if diff.size else 0.0
    atol, rtol = TOL[dtype]
    assert max_abs <= atol and rel <= rtol, "%s: max_abs %.3e (tol %.1e) rel %.3e (tol %.1e)" % (
        what, max_abs, atol, rel, rtol)
    return max_abs, rel


def run_prefill(dag_list, q, k, v, theta, rope=True, want_lse=False):
    """Full library path: build_meta -> rope (in place on copies) -> prefill.  Returns (out, lse, meta)."""
    hq, hkv, d = q.shape[1], k.shape[1], q.shape[2]
    _, meta = build_meta(dag_list, hq, hkv, d, q.dtype)
    qd, kd, vd = q.to(DEV).clone(), k.to(DEV).clone(), v.to(DEV)
    if rope:
        B.dag_rope_qk(meta.get("pos_ids"), qd, kd, theta)
    out = torch.empty_like(qd)
    lse = torch.empty(q.shape[0], hq, dtype=torch.float32, device=DEV) if want_lse else None
    B.dag_attn_prefill(meta, qd, kd, vd, out, lse)
    torch.cuda.synchronize()
    return out, lse, meta, qd, kd


def oracle_prefill(dag_list, q, k, v, theta, rows_per_seq=None, seed=0, heads=None):
    """Oracle outputs for the batch.  rows_per_seq = None -> every row; else a seeded sample of that
    many rows per sequence (always including the first and last row of the sequence).
    Returns (ref [T][Hq][D] with NaN where not computed, list of global row indices computed)."""
    q64, k64, v64 = dags.to_f64(q), dags.to_f64(k), dags.to_f64(v)
    T, hq, d = q64.shape
    ref = np.full((T, hq, d), np.nan)
    lse = np.full((T, hq), np.nan)
    rows_all = []
    t0 = 0
    rng = np.random.Generator(np.random.PCG64(seed))
    for L, anc in dag_list:
        Tb = int(np.sum(L))
        _, pos = orc.token_meta(L, anc)
        qs = orc.rope(q64[t0:t0 + Tb], pos, theta)
        ks = orc.rope(k64[t0:t0 + Tb], pos, theta)
        if rows_per_seq is None or rows_per_seq >= Tb:
            rows = None
            sel = np.arange(Tb)
        else:
            sel = np.unique(np.concatenate([[0, Tb - 1], rng.choice(Tb, size=rows_per_seq, replace=False)]))
            rows = sel
        O, l = orc.attn_prefill(qs, ks, v64[t0:t0 + Tb], L, anc, rows=rows, heads=heads)
        ref[t0:t0 + Tb] = O
        lse[t0:t0 + Tb] = l
        rows_all.append(t0 + sel)
        t0 += Tb
    return ref, lse, np.concatenate(rows_all)
