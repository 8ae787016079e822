"""Seeded synthetic inputs shared by the tests, the benchmark and the smoke check.

This module only *builds inputs*: DAG node tables (lengths + ancestor bitsets), random Q/K/V
values, page tables and the storage packing of the paged KV pools.  It contains none of the
attention method's arithmetic (no positions, masks, rotary embedding, softmax) and imports neither
the GPU library nor the CPU oracle.

The DAG shapes stand in for the topologies the paper reports (Table 3: a single linear chain,
multiple independent chains = fork/join, complex intersecting = multi-level DAG with joins); the
paper's own dataset is not used.
"""
import numpy as np
import torch

SEED0 = 260207529
PAGE = 16


# ----------------------------------------------------------------------------- DAG node tables
def words_for(n_nodes):
    return max(1, (n_nodes + 63) // 64)


def bits_from_sets(anc_sets, n_words=None):
    """anc_sets: list of iterables of ancestor ids -> uint64 [N][W]."""
    n = len(anc_sets)
    W = words_for(n) if n_words is None else n_words
    out = np.zeros((n, W), dtype=np.uint64)
    for v, s in enumerate(anc_sets):
        for u in s:
            out[v, u >> 6] |= np.uint64(1) << np.uint64(u & 63)
    return out


def sets_from_bits(anc):
    n = anc.shape[0]
    return [{u for u in range(n) if (int(anc[v, u >> 6]) >> (u & 63)) & 1} for v in range(n)]


def closure_from_parents(parents):
    """parents[v] = iterable of direct predecessors (< v).  Returns transitive ancestor sets."""
    anc = []
    for v, ps in enumerate(parents):
        s = set()
        for p in ps:
            assert p < v
            s.add(p)
            s |= anc[p]
        anc.append(s)
    return anc


def linear_chain(lengths):
    """Single chain: node v depends on v-1."""
    parents = [[] if v == 0 else [v - 1] for v in range(len(lengths))]
    return np.asarray(lengths, dtype=np.int32), bits_from_sets(closure_from_parents(parents))


def fork_join(prefix_len, branch_lens, join_len=None):
    """prefix -> len(branch_lens) sibling branches -> (optional) one join node."""
    lens = [prefix_len] + list(branch_lens)
    parents = [[]] + [[0] for _ in branch_lens]
    if join_len is not None:
        lens.append(join_len)
        parents.append(list(range(1, 1 + len(branch_lens))))
    return np.asarray(lens, dtype=np.int32), bits_from_sets(closure_from_parents(parents))


def random_dag(rng, n_nodes=64, depth=6, fan_lo=1, fan_hi=4, join_prob=0.3,
               len_lo=32, len_hi=256):
    """Multi-level DAG: `depth` levels, exactly `n_nodes` nodes, fan-out U{fan_lo..fan_hi} per
    node, nodes at level >= 2 become joins of 2-3 parents with probability join_prob.
    Node ids are assigned level by level, so they are a topological order.
    Returns (node_len int32[N], anc uint64[N][W], parents list, level list).
    """
    if n_nodes < depth:
        raise ValueError("random_dag: %d nodes cannot fill %d levels" % (n_nodes, depth))
    while True:
        levels = [[0]]
        parents = [[]]
        nxt = 1
        ok = True
        for lv in range(1, depth):
            remaining_levels = depth - 1 - lv          # levels still to come after this one
            budget = n_nodes - nxt - remaining_levels  # nodes this level may take at most
            if budget < 1:
                ok = False
                break
            # keep the level sizes balanced: at most twice an even share of what is left
            budget = min(budget, 2 * -(-(n_nodes - nxt) // (remaining_levels + 1)))
            cur = []
            for p in levels[lv - 1]:
                f = int(rng.integers(fan_lo, fan_hi + 1))
                for _ in range(f):
                    if len(cur) < budget:
                        parents.append([p])
                        cur.append(nxt)
                        nxt += 1
            if lv == depth - 1:
                # last level absorbs what is left so that the node count is exact
                while nxt < n_nodes:
                    p = levels[lv - 1][int(rng.integers(0, len(levels[lv - 1])))]
                    parents.append([p])
                    cur.append(nxt)
                    nxt += 1
            if not cur:
                ok = False
                break
            levels.append(cur)
        if ok and nxt == n_nodes and len(levels) == depth:
            break
    level_of = [0] * n_nodes
    for lv, ids in enumerate(levels):
        for v in ids:
            level_of[v] = lv
    for lv in range(2, depth):
        prev = levels[lv - 1]
        for v in levels[lv]:
            if len(prev) >= 2 and rng.random() < join_prob:
                extra = int(rng.integers(1, 3))
                cand = [p for p in prev if p not in parents[v]]
                rng.shuffle(cand)
                parents[v] = sorted(parents[v] + cand[:extra])
    anc = closure_from_parents(parents)
    lens = rng.integers(len_lo, len_hi + 1, size=n_nodes).astype(np.int32)
    return lens, bits_from_sets(anc), parents, level_of


def layerwise_bits(level_of):
    """Ancestor bitsets of the literal layer-wise mask: every node of an earlier layer is visible."""
    n = len(level_of)
    return bits_from_sets([{u for u in range(v) if level_of[u] < level_of[v]} for v in range(n)])


def batch_desc(dags):
    """Concatenate per-sequence (node_len, anc) pairs into the batched host description."""
    n_seqs = len(dags)
    W = max(a.shape[1] for _, a in dags)
    node_offsets = np.zeros(n_seqs + 1, dtype=np.int32)
    lens, bits = [], []
    for b, (l, a) in enumerate(dags):
        node_offsets[b + 1] = node_offsets[b] + len(l)
        lens.append(np.asarray(l, dtype=np.int32))
        aa = np.zeros((a.shape[0], W), dtype=np.uint64)
        aa[:, :a.shape[1]] = a
        bits.append(aa)
    return node_offsets, np.concatenate(lens), np.concatenate(bits, axis=0), W


# ----------------------------------------------------------------------------- values
def normal_tensor(rng, shape, scale, dtype):
    """Standard normal fp32 * scale, rounded once (RNE) to `dtype` (torch.float32 / bfloat16)."""
    x = rng.standard_normal(size=shape, dtype=np.float32) * np.float32(scale)
    return torch.from_numpy(x).to(dtype)


def make_qkv(seed, T, hq, hkv, d, scale, dtype):
    rng = np.random.Generator(np.random.PCG64(seed))
    q = normal_tensor(rng, (T, hq, d), scale, dtype)
    k = normal_tensor(rng, (T, hkv, d), scale, dtype)
    v = normal_tensor(rng, (T, hkv, d), scale, dtype)
    return q, k, v


def to_f64(t):
    """Exact upcast of a torch tensor (fp32 / bf16) to a numpy fp64 array."""
    return t.detach().cpu().to(torch.float64).numpy()


# ----------------------------------------------------------------------------- paged KV storage
def pack_k_pages(k_tok):
    """k_tok [n_pages*16][Hkv][D] (token-major) -> K pool format [n_pages][Hkv][D/8][16][8]."""
    n, hkv, d = k_tok.shape
    assert n % PAGE == 0 and d % 8 == 0
    x = k_tok.reshape(n // PAGE, PAGE, hkv, d // 8, 8)
    return x.permute(0, 2, 3, 1, 4).contiguous()


def pack_v_pages(v_tok):
    """v_tok [n_pages*16][Hkv][D] -> V pool format [n_pages][Hkv][D][16]."""
    n, hkv, d = v_tok.shape
    assert n % PAGE == 0
    x = v_tok.reshape(n // PAGE, PAGE, hkv, d)
    return x.permute(0, 2, 3, 1).contiguous()


def decode_state(seed, n_seqs, n_branches, shared_len, branch_len, hq, hkv, d,
                 kv_scale=1.0, q_scale=1.0, dtype=torch.bfloat16, spare_pages=0,
                 branch_len_list=None):
    """Branch-parallel decode state: every sequence is one sibling group whose `n_branches`
    live branches share `shared_len` context tokens and own `branch_len` tokens each (the
    last own token is the one being decoded).  Page ids are a seeded random permutation of the
    pool, so pages are non-contiguous.  `branch_len_list` (length n_seqs*n_branches) overrides
    the per-branch own length.  Pools are filled with N(0,1)*kv_scale directly in pool format.
    Returns a dict with the pools, q, and the int32 description arrays (numpy).
    """
    rng = np.random.Generator(np.random.PCG64(seed))
    n_live = n_seqs * n_branches
    if branch_len_list is None:
        branch_len_list = [branch_len] * n_live
    blens = np.asarray(branch_len_list, dtype=np.int32)
    shared_pages_per = (shared_len + PAGE - 1) // PAGE
    bpages = (blens + PAGE - 1) // PAGE
    n_pages = n_seqs * shared_pages_per + int(bpages.sum()) + spare_pages
    perm = rng.permutation(n_pages).astype(np.int32)
    cur = 0
    group_branch_off = np.arange(0, n_live + 1, n_branches, dtype=np.int32)
    shared_page_off = np.zeros(n_seqs + 1, dtype=np.int32)
    shared_pages = []
    for g in range(n_seqs):
        shared_pages.append(perm[cur:cur + shared_pages_per])
        cur += shared_pages_per
        shared_page_off[g + 1] = shared_page_off[g] + shared_pages_per
    branch_page_off = np.zeros(n_live + 1, dtype=np.int32)
    branch_pages = []
    for r in range(n_live):
        branch_pages.append(perm[cur:cur + bpages[r]])
        cur += int(bpages[r])
        branch_page_off[r + 1] = branch_page_off[r] + bpages[r]
    k_pool = normal_tensor(rng, (n_pages, hkv, d // 8, PAGE, 8), kv_scale, dtype)
    v_pool = normal_tensor(rng, (n_pages, hkv, d, PAGE), kv_scale, dtype)
    q = normal_tensor(rng, (n_live, hq, d), q_scale, dtype)
    k_new = normal_tensor(rng, (n_live, hkv, d), kv_scale, dtype)
    v_new = normal_tensor(rng, (n_live, hkv, d), kv_scale, dtype)
    desc = dict(
        n_groups=n_seqs, n_live=n_live, page_size=PAGE,
        group_branch_off=group_branch_off,
        shared_page_off=shared_page_off,
        shared_pages=np.concatenate(shared_pages).astype(np.int32) if shared_pages_per else np.zeros(0, np.int32),
        shared_len=np.full(n_seqs, shared_len, dtype=np.int32),
        branch_page_off=branch_page_off,
        branch_pages=np.concatenate(branch_pages).astype(np.int32),
        branch_len=blens,
        branch_pos=(shared_len + blens - 1).astype(np.int32),
    )
    return dict(desc=desc, k_pool=k_pool, v_pool=v_pool, q=q, k_new=k_new, v_new=v_new,
                n_pages=n_pages)


def decode_algorithmic_bytes(desc, hkv, d, elem_bytes=2):
    """Bytes one decode step must read: every shared page once per sibling group plus every
    branch's own tokens, K and V."""
    toks = int(np.sum(desc["shared_len"])) + int(np.sum(desc["branch_len"]))
    return toks * hkv * d * 2 * elem_bytes


def decode_segments_state(seed, dag_list, live_list, hq, hkv, d, kv_scale=1.0, q_scale=1.0,
                          dtype=torch.bfloat16, junk_scale=4.0, spare_pages=3, keep_tokens=True,
                          new_tokens=None):
    """Decode state of a general DAG frontier: one KV *segment* per node of every DAG in
    `dag_list` ((node_len, anc) pairs), stored in its own pages (the last page of a segment is
    partly filled when the node length is no multiple of the page size; its unused slots hold
    large random junk that no reader may touch).  `live_list[b]` names the live nodes of DAG b:
    each is decoding its last token and reads the segments of its ancestors and its own.
    With `new_tokens[b][i]` = n > 1 the last n tokens of live node i of DAG b are all live (the
    node is being prefilled n tokens at a time against the cached context): n branches, oldest
    first, each seeing the node's segment up to itself ("seg_reader_len", one entry per
    reader-list position; the full segment length for every other reader).
    Segment ids and live-branch ids are global (DAG after DAG).  Returns the pools, the query
    of every live branch, the token-level q/k/v of every DAG (for a dense cross-check; with
    keep_tokens=False only the live tokens get a query and nothing token-level is kept) and the
    int32 description arrays:
      seg_page_off/seg_pages/seg_len        pages and token count of each segment
      seg_reader_off/seg_readers            live branches that read the segment (ascending)
      branch_seg_off/branch_segs            segments each live branch reads (ascending node id)
      branch_entry_off/branch_entries       the same relation as positions in seg_readers
    and, under "paged", the same frontier as a paged-prefill description (one entry per live node:
    its rows of q, the pages of its context with their token counts, where its own pages start).
    """
    rng = np.random.Generator(np.random.PCG64(seed))
    seg_len, seg_np = [], []
    paged = dict(q_off=[0], ctx_page_off=[0], ctx_pages=[], ctx_page_len=[], own_page=[], own_len=[], page_size=PAGE)
    for L, _ in dag_list:
        for x in L:
            seg_len.append(int(x))
            seg_np.append((int(x) + PAGE - 1) // PAGE)
    n_pages = int(np.sum(seg_np)) + spare_pages
    perm = rng.permutation(n_pages).astype(np.int32)
    # (without token-level arrays the pools are drawn in place with the token scale and only the
    # unused slots of partly filled pages are overwritten with junk)
    k_pool = normal_tensor(rng, (n_pages, hkv, d // 8, PAGE, 8), junk_scale if keep_tokens else kv_scale, dtype)
    v_pool = normal_tensor(rng, (n_pages, hkv, d, PAGE), junk_scale if keep_tokens else kv_scale, dtype)
    seg_page_off = np.zeros(len(seg_len) + 1, dtype=np.int32)
    seg_page_off[1:] = np.cumsum(seg_np)
    seg_pages = perm[:seg_page_off[-1]].copy()
    readers = [[] for _ in seg_len]
    reader_len = [[] for _ in seg_len]
    dag_index = 0
    branch_segs, q_rows, toks, live_tok = [], [], [], []
    s0 = 0
    for (L, anc), live in zip(dag_list, live_list):
        T = int(np.sum(L))
        if keep_tokens:
            q_tok, k_tok, v_tok = make_qkv(int(rng.integers(1 << 30)), T, hq, hkv, d, 1.0, dtype)
            q_tok, k_tok, v_tok = q_tok * q_scale, k_tok * kv_scale, v_tok * kv_scale
            toks.append((q_tok, k_tok, v_tok))
        else:
            q_tok = k_tok = v_tok = None
        start = np.concatenate([[0], np.cumsum(L)]).astype(np.int64)
        for u, n in enumerate(L):
            pg = torch.from_numpy(seg_pages[seg_page_off[s0 + u]:seg_page_off[s0 + u + 1]].astype(np.int64))
            if not keep_tokens:
                used = int(n) % PAGE
                if used:
                    k_pool[pg[-1], :, :, used:, :] = normal_tensor(rng, (hkv, d // 8, PAGE - used, 8), junk_scale, dtype)
                    v_pool[pg[-1], :, :, used:] = normal_tensor(rng, (hkv, d, PAGE - used), junk_scale, dtype)
                continue
            i = torch.arange(int(n))
            k_pool[pg[i // PAGE], :, :, i % PAGE, :] = k_tok[start[u]:start[u + 1]].reshape(int(n), hkv, d // 8, 8)
            v_pool[pg[i // PAGE], :, :, i % PAGE] = v_tok[start[u]:start[u + 1]]
        sets = sets_from_bits(anc)
        for li, v in enumerate(live):
            n_new = 1 if new_tokens is None else int(new_tokens[dag_index][li])
            mine = sorted(set(int(u) for u in sets[v]) | {int(v)})
            # the same live node as one entry of the paged-prefill description: the pages of its
            # ancestors' segments in node order, then its own, with the tokens each page holds
            for u in [u for u in mine if u != v] + [int(v)]:
                if u == v:
                    paged["own_page"].append(len(paged["ctx_pages"]) - paged["ctx_page_off"][-1])
                pg = seg_pages[seg_page_off[s0 + u]:seg_page_off[s0 + u + 1]]
                paged["ctx_pages"].extend(int(x) for x in pg)
                paged["ctx_page_len"].extend(min(PAGE, int(L[u]) - PAGE * j) for j in range(len(pg)))
            paged["ctx_page_off"].append(len(paged["ctx_pages"]))
            paged["own_len"].append(int(L[v]))
            paged["q_off"].append(paged["q_off"][-1] + n_new)
            for i in range(n_new):
                r = len(branch_segs)
                tok = int(start[v + 1]) - n_new + i
                branch_segs.append([s0 + u for u in mine])
                for u in mine:
                    readers[s0 + u].append(r)
                    reader_len[s0 + u].append(int(L[u]) if u != v else tok - int(start[v]) + 1)
                q_rows.append(q_tok[tok] if keep_tokens else normal_tensor(rng, (hq, d), q_scale, dtype))
                live_tok.append(tok)
        s0 += len(L)
        dag_index += 1
    n_live = len(branch_segs)
    seg_reader_off = np.zeros(len(seg_len) + 1, dtype=np.int32)
    seg_reader_off[1:] = np.cumsum([len(x) for x in readers])
    branch_seg_off = np.zeros(n_live + 1, dtype=np.int32)
    branch_seg_off[1:] = np.cumsum([len(x) for x in branch_segs])
    flat = lambda ll: np.asarray([x for l in ll for x in l], dtype=np.int32)
    desc = dict(
        n_live=n_live, n_segments=len(seg_len), page_size=PAGE,
        seg_page_off=seg_page_off, seg_pages=seg_pages.astype(np.int32),
        seg_len=np.asarray(seg_len, dtype=np.int32),
        seg_reader_off=seg_reader_off, seg_readers=flat(readers),
        branch_seg_off=branch_seg_off, branch_segs=flat(branch_segs),
    )
    if new_tokens is not None:
        desc["seg_reader_len"] = flat(reader_len)
    add_branch_entries(desc)
    return dict(desc=desc, k_pool=k_pool, v_pool=v_pool, q=torch.stack(q_rows) if q_rows else
                torch.zeros((0, hq, d), dtype=dtype), tokens=toks, live_tok=live_tok, n_pages=n_pages,
                paged={k: (np.asarray(x, dtype=np.int32) if isinstance(x, list) else x) for k, x in paged.items()})


def add_branch_entries(desc):
    """branch_entries[e]: position in seg_readers where the branch of entry e of branch_segs is
    listed among the readers of that segment (pure bookkeeping: the inverse of the reader lists)."""
    off, readers = np.asarray(desc["seg_reader_off"]), np.asarray(desc["seg_readers"])
    bso, bs = np.asarray(desc["branch_seg_off"]), np.asarray(desc["branch_segs"])
    ent = np.zeros(len(bs), dtype=np.int32)
    for r in range(int(desc["n_live"])):
        for e in range(int(bso[r]), int(bso[r + 1])):
            s = int(bs[e])
            ent[e] = off[s] + int(np.nonzero(readers[off[s]:off[s + 1]] == r)[0][0])
    desc["branch_entry_off"] = bso.astype(np.int32)
    desc["branch_entries"] = ent
    return desc


def segments_from_decode_desc(desc):
    """The two-level description of decode_state (shared context + own tokens per branch) written
    as segments: one per sibling group's shared context, one per live branch."""
    ng, nl = int(desc["n_groups"]), int(desc["n_live"])
    gbo = np.asarray(desc["group_branch_off"])
    sp = np.diff(np.asarray(desc["shared_page_off"]))
    bp = np.diff(np.asarray(desc["branch_page_off"]))
    seg_page_off = np.concatenate([[0], np.cumsum(np.concatenate([sp, bp]))]).astype(np.int32)
    readers = [list(range(int(gbo[g]), int(gbo[g + 1]))) for g in range(ng)] + [[r] for r in range(nl)]
    group_of = np.searchsorted(gbo, np.arange(nl), side="right") - 1
    branch_segs = [[int(group_of[r]), ng + r] for r in range(nl)]
    flat = lambda ll: np.asarray([x for l in ll for x in l], dtype=np.int32)
    return add_branch_entries(dict(
        n_live=nl, n_segments=ng + nl, page_size=PAGE,
        seg_page_off=seg_page_off,
        seg_pages=np.concatenate([desc["shared_pages"], desc["branch_pages"]]).astype(np.int32),
        seg_len=np.concatenate([desc["shared_len"], desc["branch_len"]]).astype(np.int32),
        seg_reader_off=np.concatenate([[0], np.cumsum([len(x) for x in readers])]).astype(np.int32),
        seg_readers=flat(readers),
        branch_seg_off=np.arange(0, 2 * nl + 1, 2, dtype=np.int32), branch_segs=flat(branch_segs),
    ))


def decode_segments_algorithmic_bytes(desc, hkv, d, elem_bytes=2):
    """Bytes one decode step must read: K and V of every segment that has a reader, once."""
    has = np.diff(np.asarray(desc["seg_reader_off"])) > 0
    return int(np.sum(np.asarray(desc["seg_len"])[has])) * hkv * d * 2 * elem_bytes


# ----------------------------------------------------------------------------- the five configs
def config(idx):
    """Shapes of the five benchmark configurations (index 0..4)."""
    cfgs = [
        dict(name="tiny_fork_join_f32", kind="prefill", batch=1, prefix=128, n_branch=4, branch=64,
             join=64, hq=4, hkv=4, d=64, scale=1.0, theta=10000.0, dtype="f32"),
        dict(name="llama3_8b_prefill_bf16", kind="prefill", batch=4, prefix=2048, n_branch=8,
             branch=256, join=512, hq=32, hkv=8, d=128, scale=0.5, theta=500000.0, dtype="bf16"),
        dict(name="branch_decode_bf16", kind="decode", n_seqs=16, n_branch=8, shared=8192,
             branch=1024, hq=32, hkv=8, d=128, scale=1.0, theta=500000.0, dtype="bf16"),
        dict(name="random_dag_prefill_bf16", kind="prefill_random", batch=8, n_nodes=64, depth=6,
             hq=32, hkv=8, d=128, scale=0.5, theta=500000.0, dtype="bf16"),
        dict(name="qwen32b_long_bf16", kind="prefill+decode", batch=2, prefix=32768, n_branch=32,
             branch=512, join=1024, decode_steps=256, hq=40, hkv=8, d=128, scale=0.5,
             theta=1000000.0, dtype="bf16"),
    ]
    c = dict(cfgs[idx])
    c["seed"] = SEED0 + idx
    return c


def config_dags(c):
    """List of per-sequence (node_len, anc) for a prefill-type config."""
    if c["kind"] == "prefill_random":
        rng = np.random.Generator(np.random.PCG64(c["seed"]))
        out = []
        for _ in range(c["batch"]):
            lens, anc, _, _ = random_dag(rng, c["n_nodes"], c["depth"])
            out.append((lens, anc))
        return out
    one = fork_join(c["prefix"], [c["branch"]] * c["n_branch"], c["join"])
    return [one for _ in range(c["batch"])]
