"""GPU parity: dag_kv_append_rope and dag_attn_decode (through the C ABI) against the oracle."""
import numpy as np
import pytest
import torch

from oracle import dag_oracle as orc
from paper_2602_07529_amd import binding as B
from workloads import dags
from tests.gpu_util import DEV, check_close

pytestmark = pytest.mark.gpu


def _gpu_decode(st, hq, hkv, d, theta, append=True):
    dd = B.DecodeDesc(st["desc"], DEV)
    kp, vp = st["k_pool"].to(DEV), st["v_pool"].to(DEV)
    if append:
        B.dag_kv_append_rope(dd, st["k_new"].to(DEV), st["v_new"].to(DEV), kp, vp, theta)
    q = st["q"].to(DEV)
    out = torch.empty_like(q)
    ws = torch.empty(B.dag_decode_workspace_bytes(dd, hq, hkv, d), dtype=torch.uint8, device=DEV)
    B.dag_attn_decode(dd, q, kp, vp, out, ws)
    torch.cuda.synchronize()
    return out, kp, vp


def _oracle_pools_after_append(st, theta):
    """Oracle append on fp64 copies, then rounded to bf16 exactly as the storage format is."""
    kp, vp = dags.to_f64(st["k_pool"]), dags.to_f64(st["v_pool"])
    orc.kv_append_rope(st["desc"], dags.to_f64(st["k_new"]), dags.to_f64(st["v_new"]), kp, vp, theta)
    return kp, vp


@pytest.mark.parametrize("hq,hkv,d,nb,shared,blens", [
    (8, 2, 128, 3, 100, [17, 5, 32]),        # ragged shared context and tails
    (32, 8, 128, 8, 512, [64] * 8),          # 32 rows per (group, kv head) like config 3
    (10, 2, 128, 7, 48, [1, 2, 3, 16, 17, 31, 33]),   # G = 5; 35 rows -> two row blocks
    (4, 4, 64, 2, 0, [40, 9]),               # no shared context at all, MHA, D = 64
    (16, 2, 128, 1, 33, [1]),                # a single branch whose own context is just its token
    (12, 2, 64, 9, 200, [3, 40, 16, 1, 7, 64, 33, 2, 20]),   # G = 6; 54 rows -> two row blocks, D = 64
    (24, 2, 128, 11, 77, [5] * 11),          # G = 12; 132 rows -> five row blocks, the last one partly filled
    (12, 2, 128, 30, 330, [3, 17, 1] * 10),  # G = 6; 180 rows -> six row blocks: two of them split over wave pairs
    (10, 2, 64, 16, 1000, [2] * 16),         # G = 5; 160 rows -> five row blocks at D = 64, 63 pages of shared context
])
def test_decode_small_cases_all_branches(hq, hkv, d, nb, shared, blens):
    st = dags.decode_state(500 + hq + nb, n_seqs=2, n_branches=nb, shared_len=shared, branch_len=0,
                           hq=hq, hkv=hkv, d=d, branch_len_list=blens * 2)
    theta = 5e5
    out, kp, vp = _gpu_decode(st, hq, hkv, d, theta)
    okp, ovp = _oracle_pools_after_append(st, theta)
    # appended keys: GPU pool equals the oracle's rotated key rounded to bf16 (tolerance of one rounding)
    check_close(kp, okp, torch.bfloat16, "k pool after append")
    assert torch.equal(vp.cpu(), torch.from_numpy(ovp).to(torch.bfloat16))
    # attention: the oracle reads the GPU-written pools so that only the attention is compared
    ref = orc.attn_decode(st["desc"], dags.to_f64(st["q"]), dags.to_f64(kp), dags.to_f64(vp))
    check_close(out, ref, torch.bfloat16, "decode out")


@pytest.mark.parametrize("hq,hkv,nb", [(8, 2, 3), (10, 2, 8)])
def test_decode_long_slices_cross_the_page_id_window(monkeypatch, hq, hkv, nb):
    """Slices of more than 64 pages (forced through the development knobs; the default plan cuts a
    small batch into short slices): the kernels fetch page ids 64 at a time, here they have to
    move on to a second and a third window.  Narrow group (12 rows) and wide group (40 rows)."""
    monkeypatch.setenv("DAGATTN_DECODE_CHUNK_A", "200")
    monkeypatch.setenv("DAGATTN_DECODE_CHUNK_B", "200")
    d, theta = 128, 5e5
    st = dags.decode_state(900 + hq, n_seqs=1, n_branches=nb, shared_len=150 * 16 + 5, branch_len=70 * 16 + 3,
                           hq=hq, hkv=hkv, d=d)
    out, kp, vp = _gpu_decode(st, hq, hkv, d, theta)
    ref = orc.attn_decode(st["desc"], dags.to_f64(st["q"]), dags.to_f64(kp), dags.to_f64(vp))
    check_close(out, ref, torch.bfloat16, "decode out, long slices")


def test_decode_config3_full_size_sampled_branches():
    c = dags.config(2)
    st = dags.decode_state(c["seed"], c["n_seqs"], c["n_branch"], c["shared"], c["branch"], c["hq"], c["hkv"], c["d"])
    out, kp, vp = _gpu_decode(st, c["hq"], c["hkv"], c["d"], c["theta"])
    branches = [0, 7, 8, 63, 127]
    ref = orc.attn_decode(st["desc"], dags.to_f64(st["q"]), dags.to_f64(kp), dags.to_f64(vp), branches=branches)
    check_close(out[branches], ref[branches], torch.bfloat16, "config 3 decode")
    # siblings of one group with identical queries and identical own pages would coincide; here they
    # differ, but the shared part must be common: run again with own length 1 for branch 0 only
    assert torch.isfinite(out.float()).all()


def test_decode_growing_branches_over_steps_config5_shape_reduced():
    # config-5 shape (G = 5, 32 live branches per sequence) at a reduced context; 3 decode steps
    hq, hkv, d, nb = 40, 8, 128, 32
    st = dags.decode_state(77, n_seqs=1, n_branches=nb, shared_len=1024, branch_len=30, hq=hq, hkv=hkv, d=d,
                           kv_scale=0.5, q_scale=0.5, spare_pages=64)
    desc = st["desc"]
    kp, vp = st["k_pool"].to(DEV), st["v_pool"].to(DEV)
    rng = np.random.Generator(np.random.PCG64(78))
    spare = list(range(st["n_pages"] - 64, st["n_pages"]))
    for step in range(3):
        # grow every branch by one token (allocating a fresh page when the tail page is full)
        new_pages, off = [], [0]
        for r in range(nb):
            pages = list(desc["branch_pages"][desc["branch_page_off"][r]:desc["branch_page_off"][r + 1]])
            if desc["branch_len"][r] % 16 == 0:
                pages.append(spare.pop())
            new_pages += pages
            off.append(len(new_pages))
        desc["branch_pages"] = np.array(new_pages, dtype=np.int32)
        desc["branch_page_off"] = np.array(off, dtype=np.int32)
        desc["branch_len"] = desc["branch_len"] + 1
        desc["branch_pos"] = (desc["shared_len"][0] + desc["branch_len"] - 1).astype(np.int32)
        k_new = dags.normal_tensor(rng, (nb, hkv, d), 0.5, torch.bfloat16)
        v_new = dags.normal_tensor(rng, (nb, hkv, d), 0.5, torch.bfloat16)
        q = dags.normal_tensor(rng, (nb, hq, d), 0.5, torch.bfloat16)
        dd = B.DecodeDesc(desc, DEV)
        B.dag_kv_append_rope(dd, k_new.to(DEV), v_new.to(DEV), kp, vp, 1e6)
        out = torch.empty(nb, hq, d, dtype=torch.bfloat16, device=DEV)
        ws = torch.empty(B.dag_decode_workspace_bytes(dd, hq, hkv, d), dtype=torch.uint8, device=DEV)
        B.dag_attn_decode(dd, q.to(DEV), kp, vp, out, ws)
        torch.cuda.synchronize()
        branches = [0, 13, 31]
        ref = orc.attn_decode(desc, dags.to_f64(q), dags.to_f64(kp), dags.to_f64(vp), branches=branches)
        check_close(out[branches], ref[branches], torch.bfloat16, "step %d" % step)


def test_decode_256_steps_of_growing_branches_every_branch_every_step():
    """A run of decode steps as the execution phase makes them (config-3 shape at a reduced context:
    two sibling groups of 8 branches, G = 4): every step appends one token per branch (a fresh page
    whenever a tail page is full: sixteen times per branch here), decodes, and every branch is
    checked against the oracle on the pools as they stand; 256 steps, the length of a decode run of
    the benchmark configurations."""
    hq, hkv, d, nb, n_seqs = 32, 8, 128, 8, 2
    st = dags.decode_state(91, n_seqs=n_seqs, n_branches=nb, shared_len=300, branch_len=7, hq=hq, hkv=hkv, d=d,
                           kv_scale=0.5, q_scale=0.5, spare_pages=n_seqs * nb * 17)
    desc = st["desc"]
    kp, vp = st["k_pool"].to(DEV), st["v_pool"].to(DEV)
    rng = np.random.Generator(np.random.PCG64(92))
    spare = list(range(st["n_pages"] - n_seqs * nb * 17, st["n_pages"]))
    R = n_seqs * nb
    group_of = np.repeat(np.arange(n_seqs), nb)
    for step in range(256):
        new_pages, off = [], [0]
        for r in range(R):
            pages = list(desc["branch_pages"][desc["branch_page_off"][r]:desc["branch_page_off"][r + 1]])
            if desc["branch_len"][r] % 16 == 0:
                pages.append(spare.pop())
            new_pages += pages
            off.append(len(new_pages))
        desc["branch_pages"] = np.array(new_pages, dtype=np.int32)
        desc["branch_page_off"] = np.array(off, dtype=np.int32)
        desc["branch_len"] = desc["branch_len"] + 1
        desc["branch_pos"] = (desc["shared_len"][group_of] + desc["branch_len"] - 1).astype(np.int32)
        k_new = dags.normal_tensor(rng, (R, hkv, d), 0.5, torch.bfloat16)
        v_new = dags.normal_tensor(rng, (R, hkv, d), 0.5, torch.bfloat16)
        q = dags.normal_tensor(rng, (R, hq, d), 0.5, torch.bfloat16)
        dd = B.DecodeDesc(desc, DEV)
        B.dag_kv_append_rope(dd, k_new.to(DEV), v_new.to(DEV), kp, vp, 1e6)
        out = torch.empty(R, hq, d, dtype=torch.bfloat16, device=DEV)
        ws = torch.empty(B.dag_decode_workspace_bytes(dd, hq, hkv, d), dtype=torch.uint8, device=DEV)
        B.dag_attn_decode(dd, q.to(DEV), kp, vp, out, ws)
        torch.cuda.synchronize()
        ref = orc.attn_decode(desc, dags.to_f64(q), dags.to_f64(kp), dags.to_f64(vp))
        check_close(out, ref, torch.bfloat16, "step %d" % step)


def test_decode_equals_last_row_of_gpu_prefill():
    """Cross-check of the two GPU paths: decoding the last token of a branch equals the last row of a
    prefill over [prefix, branch] (both within tolerance of the same oracle value)."""
    hq, hkv, d, prefix, bl = 8, 2, 128, 64, 32
    T = prefix + bl
    q, k, v = dags.make_qkv(91, T, hq, hkv, d, 0.5, torch.bfloat16)
    from tests.gpu_util import run_prefill
    out_p, _, meta, qd, kd = run_prefill([dags.linear_chain([prefix, bl])], q, k, v, 5e5)
    kp = dags.pack_k_pages(kd.cpu()).to(DEV)
    vp = dags.pack_v_pages(v).to(DEV)
    desc = dict(n_groups=1, n_live=1, page_size=16, group_branch_off=np.array([0, 1]), shared_page_off=np.array([0, 4]),
                shared_pages=np.arange(4), shared_len=np.array([prefix]), branch_page_off=np.array([0, 2]),
                branch_pages=np.array([4, 5]), branch_len=np.array([bl]), branch_pos=np.array([T - 1]))
    dd = B.DecodeDesc(desc, DEV)
    out = torch.empty(1, hq, d, dtype=torch.bfloat16, device=DEV)
    ws = torch.empty(B.dag_decode_workspace_bytes(dd, hq, hkv, d), dtype=torch.uint8, device=DEV)
    B.dag_attn_decode(dd, qd[-1:].contiguous(), kp, vp, out, ws)
    torch.cuda.synchronize()
    assert (out[0].float() - out_p[-1].float()).abs().max().item() < 2e-2


@pytest.mark.parametrize("own_len", [513, 768])
def test_decode_config5_full_size_sampled_branches(own_len):
    """Benchmark config 5 decode at full size: 2 sequences x 32 live branches, shared prefix 32,768
    tokens, G = 5 (160 stacked rows per group and KV head), at its first and its last step."""
    c = dags.config(4)
    st = dags.decode_state(c["seed"] + own_len, 2, c["n_branch"], c["prefix"], own_len, c["hq"], c["hkv"], c["d"],
                           kv_scale=0.5, q_scale=0.5)
    out, kp, vp = _gpu_decode(st, c["hq"], c["hkv"], c["d"], c["theta"])
    branches = [0, 31, 32, 50, 63]
    ref = orc.attn_decode(st["desc"], dags.to_f64(st["q"]), dags.to_f64(kp), dags.to_f64(vp), branches=branches)
    check_close(out[branches], ref[branches], torch.bfloat16, "config 5 decode")
    assert torch.isfinite(out.float()).all()


@pytest.mark.parametrize("hq,hkv,d,nb,shared,own", [(40, 8, 128, 32, 3000, 2100), (12, 2, 64, 20, 777, 1300),
                                                    (16, 2, 128, 9, 50, 4000), (10, 1, 128, 7, 0, 700)])
def test_decode_wide_groups_with_long_own_lists(hq, hkv, d, nb, shared, own):
    """Wide sibling groups (more than 32 stacked rows per KV head) whose own page lists are long
    enough to be cut into several slices, odd page counts, a shared context shorter than one
    slice, and none at all (the single-wave path then takes everything): every branch."""
    st = dags.decode_state(7000 + hq + nb, 2, nb, shared, own, hq, hkv, d, kv_scale=0.5, q_scale=0.5)
    out, kp, vp = _gpu_decode(st, hq, hkv, d, 5e5)
    branches = sorted(set(range(0, 2 * nb, 3)) | {2 * nb - 1})
    ref = orc.attn_decode(st["desc"], dags.to_f64(st["q"]), dags.to_f64(kp), dags.to_f64(vp), branches=branches)
    check_close(out[branches], ref[branches], torch.bfloat16, "wide decode, long own lists")
    assert torch.isfinite(out.float()).all()


def test_decode_config5_every_branch_of_one_kv_head():
    """Benchmark config 5 decode at full size, middle of its 256 steps (own length 640): all 64
    live branches, the five query heads of one KV head, against the oracle."""
    c = dags.config(4)
    st = dags.decode_state(c["seed"] + 640, 2, c["n_branch"], c["prefix"], 640, c["hq"], c["hkv"], c["d"],
                           kv_scale=0.5, q_scale=0.5)
    out, kp, vp = _gpu_decode(st, c["hq"], c["hkv"], c["d"], c["theta"])
    ref = orc.attn_decode(st["desc"], dags.to_f64(st["q"]), dags.to_f64(kp), dags.to_f64(vp), kv_heads=[6])
    check_close(out[:, 30:35], ref[:, 30:35], torch.bfloat16, "config 5 decode, kv head 6")


@pytest.mark.parametrize("hq,hkv,d,nb,shared,blens", [
    (8, 2, 128, 3, 100, [17, 5, 32]),             # single-wave items, ragged shared context and tails
    (10, 2, 128, 16, 1000, [2, 19, 33, 16] * 4),  # 80 stacked rows: the wide kernel for the shared context
])
def test_decode_ignores_non_finite_bits_in_unused_slots(hq, hkv, d, nb, shared, blens):
    """The slots of a partly filled last page that hold no token yet (and pages of the pool that
    belong to nobody) carry NaN and infinity bit patterns: no result may depend on them."""
    st = dags.decode_state(900 + nb, n_seqs=2, n_branches=nb, shared_len=shared, branch_len=0,
                           hq=hq, hkv=hkv, d=d, branch_len_list=blens * 2, spare_pages=2)
    desc = st["desc"]
    kp, vp = st["k_pool"], st["v_pool"]
    poison = [float("nan"), float("inf"), float("-inf")]

    def poison_tail(pages, n_tok, salt):
        used = n_tok % 16
        if used and len(pages):
            kp[int(pages[-1]), :, :, used:, :] = poison[salt % 3]
            vp[int(pages[-1]), :, :, used:] = poison[(salt + 1) % 3]

    for g in range(int(desc["n_groups"])):
        poison_tail(desc["shared_pages"][desc["shared_page_off"][g]:desc["shared_page_off"][g + 1]],
                    int(desc["shared_len"][g]), g)
    for r in range(int(desc["n_live"])):
        poison_tail(desc["branch_pages"][desc["branch_page_off"][r]:desc["branch_page_off"][r + 1]],
                    int(desc["branch_len"][r]), r)
    unused = sorted(set(range(st["n_pages"])) - set(desc["shared_pages"].tolist()) - set(desc["branch_pages"].tolist()))
    assert len(unused) == 2
    kp[unused] = float("nan")
    vp[unused] = float("nan")
    out, kpd, vpd = _gpu_decode(st, hq, hkv, d, 5e5, append=False)
    assert torch.isfinite(out.float()).all()
    ref = orc.attn_decode(desc, dags.to_f64(st["q"]), dags.to_f64(kpd), dags.to_f64(vpd))
    check_close(out, ref, torch.bfloat16, "decode with poisoned unused slots")
