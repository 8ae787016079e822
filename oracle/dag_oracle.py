"""CPU oracle for DAG-structured attention (MedVerse attention, paper sections 3.2-3.3, 4.2, 4.3).

TEST INFRASTRUCTURE ONLY.  This module is the slow, plain, fp64 definition of what the GPU library
computes.  It may be imported by tests/, by __graft_entry__.smoke() and by the cpu_baseline leg of
bench.py, and by nothing else.  It shares no code with the HIP path and never imports it.

Conventions (the paper is silent or loose on several; these are the readings used):
  * A sequence is a DAG of N nodes (reasoning states / Petri-net places, section 3.1-3.2).  Node v
    has L[v] >= 1 tokens.  Tokens are stored node after node in node-id order, and node ids are a
    topological order: anc(v) is a subset of {0..v-1}.
  * anc is a uint64 array [N][W]; bit u of row v set  <=>  node u is an ancestor of node v.  The
    self bit is ignored on input.
  * Visibility (section 4.2 Eq. 3 generalised to the ancestor closure the engine text of section
    3.3 / 4.3 describes): token i sees token j  iff  (same node and j <= i) or node(j) in
    anc(node(i)).  A caller who wants the literal layer-wise Eq. 3 passes anc(v) = all nodes of
    earlier layers.
  * Adaptive positions (section 4.2, "Adaptive Position Indices"): a node without ancestors starts
    at 0; otherwise it starts one past the largest position used by any ancestor.  Siblings with
    the same ancestor set therefore start at the same index (fork alignment) and a join resumes
    after its longest predecessor.
  * P(i) of Eq. 2 is rotary embedding, rotate-half pairing (m, m + D/2), frequency theta^(-2m/D).
  * Scores are scaled by softmax_scale (1/sqrt(D) by default), which Eq. 2 leaves out.
  * Paged KV (section 3.2 token tau=(h,k): KV passed by page reference; section 4.3 Fork: the
    prefix pages are shared by all sibling branches).  Page size 16.  Pool storage formats:
        K pool [n_pages][Hkv][D/8][16][8]   element (page, h, slot, d) at [page, h, d//8, slot, d%8]
        V pool [n_pages][Hkv][D][16]        element (page, h, slot, d) at [page, h, d, slot]
"""
import numpy as np

PAGE = 16
SKIP, PARTIAL, FULL = 0, 1, 2


# ----------------------------------------------------------------------------- node level
def _has_bit(anc, v, u):
    return (int(anc[v, u >> 6]) >> (u & 63)) & 1 == 1


def ancestors(anc, v):
    """Ancestor ids of node v as a list (self bit ignored)."""
    n = anc.shape[0]
    return [u for u in range(n) if u != v and _has_bit(anc, v, u)]


def node_tables(node_len, anc):
    """Section 4.2 adaptive position rule at node granularity.

    Returns (tok_start[N+1], pos_start[N]) as int64.
    """
    L = [int(x) for x in node_len]
    n = len(L)
    tok_start = np.zeros(n + 1, dtype=np.int64)
    for v in range(n):
        tok_start[v + 1] = tok_start[v] + L[v]
    pos_start = np.zeros(n, dtype=np.int64)
    for v in range(n):
        a = ancestors(anc, v)
        if a:
            pos_start[v] = 1 + max(int(pos_start[u]) + L[u] - 1 for u in a)
    return tok_start, pos_start


def token_meta(node_len, anc):
    """Per-token node id and adaptive position id (int64 arrays of length T)."""
    tok_start, pos_start = node_tables(node_len, anc)
    n = len(node_len)
    T = int(tok_start[n])
    tok_node = np.zeros(T, dtype=np.int64)
    pos_ids = np.zeros(T, dtype=np.int64)
    for v in range(n):
        t0, t1 = int(tok_start[v]), int(tok_start[v + 1])
        tok_node[t0:t1] = v
        pos_ids[t0:t1] = int(pos_start[v]) + np.arange(t1 - t0)
    return tok_node, pos_ids


def node_vis(anc):
    """Visibility bitset per node: ancestors plus the node itself."""
    out = np.array(anc, dtype=np.uint64, copy=True)
    for v in range(out.shape[0]):
        out[v, v >> 6] |= np.uint64(1) << np.uint64(v & 63)
    return out


def node_allow_matrix(anc):
    """A[v][u] = True iff u is an ancestor of v (self excluded)."""
    n = anc.shape[0]
    A = np.zeros((n, n), dtype=bool)
    for v in range(n):
        for u in ancestors(anc, v):
            A[v, u] = True
    return A


# ----------------------------------------------------------------------------- mask
def mask_rows(node_len, anc, i0, i1):
    """Rows [i0, i1) of the explicit T x T boolean visibility mask (Eq. 3, ancestor reading)."""
    tok_node, _ = token_meta(node_len, anc)
    A = node_allow_matrix(anc)
    T = tok_node.shape[0]
    i = np.arange(i0, i1)[:, None]
    j = np.arange(T)[None, :]
    ni = tok_node[i0:i1][:, None]
    nj = tok_node[None, :]
    same = (ni == nj) & (j <= i)
    return same | A[ni, nj]


def explicit_mask(node_len, anc):
    T = int(np.sum(node_len))
    return mask_rows(node_len, anc, 0, T)


def useful_pairs(node_len, anc):
    """Number of visible (query, key) pairs, counted from the explicit mask."""
    T = int(np.sum(node_len))
    total = 0
    for i0 in range(0, T, 1024):
        total += int(mask_rows(node_len, anc, i0, min(T, i0 + 1024)).sum())
    return total


def block_map(node_len, anc, tile_m, tile_n):
    """Tile classification by brute force over in-range pairs: 0 skip / 1 partial / 2 full.

    Tiles restart at the beginning of the sequence; returns uint8 [QT][KT].
    """
    T = int(np.sum(node_len))
    QT = (T + tile_m - 1) // tile_m
    KT = (T + tile_n - 1) // tile_n
    out = np.zeros((QT, KT), dtype=np.uint8)
    for a in range(QT):
        rows = mask_rows(node_len, anc, a * tile_m, min(T, (a + 1) * tile_m))
        for b in range(KT):
            sub = rows[:, b * tile_n:min(T, (b + 1) * tile_n)]
            if not sub.any():
                out[a, b] = SKIP
            elif sub.all():
                out[a, b] = FULL
            else:
                out[a, b] = PARTIAL
    return out


def block_map_csr(bmap):
    """CSR over the non-skip tiles of a dense block map, key tiles ascending."""
    QT, KT = bmap.shape
    row_ptr = np.zeros(QT + 1, dtype=np.int64)
    col, flag = [], []
    for a in range(QT):
        for b in range(KT):
            if bmap[a, b] != SKIP:
                col.append(b)
                flag.append(int(bmap[a, b]))
        row_ptr[a + 1] = len(col)
    return row_ptr, np.array(col, dtype=np.int64), np.array(flag, dtype=np.uint8)


def block_map_csr_full_first(bmap):
    """The library's CSR row order: within a row the FULL tiles first (key tiles ascending), then
    the PARTIAL tiles (ascending).  Also returns the number of FULL tiles per row."""
    QT, KT = bmap.shape
    row_ptr = np.zeros(QT + 1, dtype=np.int64)
    nfull = np.zeros(QT, dtype=np.int64)
    col, flag = [], []
    for a in range(QT):
        for want in (FULL, PARTIAL):
            for b in range(KT):
                if bmap[a, b] == want:
                    col.append(b)
                    flag.append(want)
            if want == FULL:
                nfull[a] = len(col) - row_ptr[a]
        row_ptr[a + 1] = len(col)
    return row_ptr, np.array(col, dtype=np.int64), np.array(flag, dtype=np.uint8), nfull


def launch_tables(bmaps, seq_tokens, tile_n):
    """How the library starts its prefill work, written out from its stated rules (no passage of
    the paper; the block map and everything derived from it is the library's own device).  For a
    batch of dense block maps (one per sequence, query tiles numbered sequence after sequence):
      order     -- every query tile of the batch, most non-skip key tiles first, ties by index;
      mask_free -- per query tile, how many of its FULL tiles need no mask at all: a FULL tile
                   whose keys run past the end of the sequence (ragged last key tile) still needs
                   the length limit and does not count.
    Returns (order, mask_free) as int64 arrays."""
    counts, mask_free = [], []
    for bmap, T in zip(bmaps, seq_tokens):
        for a in range(bmap.shape[0]):
            counts.append(sum(1 for b in range(bmap.shape[1]) if bmap[a, b] != SKIP))
            mask_free.append(sum(1 for b in range(bmap.shape[1])
                                 if bmap[a, b] == FULL and (b + 1) * tile_n <= int(T)))
    order = sorted(range(len(counts)), key=lambda i: (-counts[i], i))
    return np.array(order, dtype=np.int64), np.array(mask_free, dtype=np.int64)


# ----------------------------------------------------------------------------- rotary embedding
def rope(x, pos, theta):
    """Rotate x[T][H][D] (any float dtype, upcast to fp64) by angle pos[t] * theta^(-2m/D).

    Pairing is (m, m + D/2) for m in [0, D/2)  (Eq. 2's P(i) read as rotary embedding).
    """
    x = np.asarray(x, dtype=np.float64)
    D = x.shape[-1]
    half = D // 2
    m = np.arange(half, dtype=np.float64)
    omega = np.float64(theta) ** (-2.0 * m / D)
    phi = np.asarray(pos, dtype=np.float64)[:, None] * omega[None, :]      # [T][half]
    c = np.cos(phi)[:, None, :]
    s = np.sin(phi)[:, None, :]
    lo, hi = x[..., :half], x[..., half:]
    out = np.empty_like(x)
    out[..., :half] = lo * c - hi * s
    out[..., half:] = hi * c + lo * s
    return out


# ----------------------------------------------------------------------------- prefill attention
def attn_prefill(q, k, v, node_len, anc, scale=None, row_block=128, rows=None, heads=None, compact=False):
    """O_i = sum_j softmax_j(q_i . k_j * scale + M_ij) v_j with the DAG mask (Eq. 2 + Eq. 3).

    q [T][Hq][D], k, v [T][Hkv][D] are the already-rotated inputs.  Query head h uses KV head
    h // (Hq/Hkv).  Returns (O [T][Hq][D], lse [T][Hq]) in fp64.  `rows` / `heads` optionally
    restrict the computation to a subset (other entries are left NaN).  With compact=True (and
    `rows` given) q holds only the selected rows, q[i] being row rows[i], and the outputs are
    [len(rows)][Hq][...] in the same order: for sequences too long to hold whole in fp64.
    """
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    T = k.shape[0]
    _, Hq, D = q.shape
    Hkv = k.shape[1]
    G = Hq // Hkv
    if scale is None:
        scale = 1.0 / np.sqrt(D)
    O = np.full((q.shape[0], Hq, D), np.nan)
    lse = np.full((q.shape[0], Hq), np.nan)
    head_list = list(range(Hq)) if heads is None else list(heads)
    if rows is None:
        blocks = [np.arange(i0, min(T, i0 + row_block)) for i0 in range(0, T, row_block)]
    else:
        rows = np.asarray(rows)
        blocks = [rows[i:i + row_block] for i in range(0, len(rows), row_block)]
    tok_node, _ = token_meta(node_len, anc)
    A = node_allow_matrix(anc)
    j = np.arange(T)[None, :]
    done = 0
    for blk in blocks:
        # where the rows of this block sit in q / O: at their own index, or packed in order
        at = np.arange(done, done + len(blk)) if compact else blk
        done += len(blk)
        ni = tok_node[blk][:, None]
        allow = ((ni == tok_node[None, :]) & (j <= blk[:, None])) | A[ni, tok_node[None, :]]
        for h in head_list:
            S = (q[at, h, :] @ k[:, h // G, :].T) * scale
            S[~allow] = -np.inf
            mrow = S.max(axis=1, keepdims=True)
            P = np.exp(S - mrow)
            lrow = P.sum(axis=1, keepdims=True)
            O[at, h, :] = (P @ v[:, h // G, :]) / lrow
            lse[at, h] = (mrow + np.log(lrow))[:, 0]
    return O, lse


def attn_prefill_bwd(q, k, v, dout, node_len, anc, scale=None, kv_heads=None):
    """Gradients of L = sum(dout * O) for O = attn_prefill(q, k, v) (Eq. 2 + Eq. 3; the paper
    fine-tunes through this mask, section 4.2), written out from the definition in fp64:
        P = softmax_row(scale * Q K^T + M),  O = P V,  delta_i = sum_d dO_id O_id,
        dV = P^T dO,  dP = dO V^T,  dS = P * (dP - delta),  dQ = scale * dS K,  dK = scale * dS^T Q,
    the gradients of a KV head summed over its query heads.  q and k are the rotated tensors;
    returns (dq, dk, dv) with their shapes (with kv_heads given, only those KV heads and their
    query heads are computed, the rest stays zero)."""
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    dout = np.asarray(dout, dtype=np.float64)
    T, Hq, D = q.shape
    Hkv = k.shape[1]
    G = Hq // Hkv
    if scale is None:
        scale = 1.0 / np.sqrt(D)
    allow = explicit_mask(node_len, anc)
    dq, dk, dv = np.zeros_like(q), np.zeros_like(k), np.zeros_like(v)
    for h in range(Hq):
        hk = h // G
        if kv_heads is not None and hk not in kv_heads:
            continue
        S = (q[:, h, :] @ k[:, hk, :].T) * scale
        S[~allow] = -np.inf
        P = np.exp(S - S.max(axis=1, keepdims=True))
        P /= P.sum(axis=1, keepdims=True)
        O = P @ v[:, hk, :]
        delta = np.sum(dout[:, h, :] * O, axis=1, keepdims=True)
        dP = dout[:, h, :] @ v[:, hk, :].T
        dS = P * (dP - delta)
        dv[:, hk, :] += P.T @ dout[:, h, :]
        dq[:, h, :] = (dS @ k[:, hk, :]) * scale
        dk[:, hk, :] += (dS.T @ q[:, h, :]) * scale
    return dq, dk, dv


# ----------------------------------------------------------------------------- paged KV
def pool_get_k(k_pool, page, h, slot):
    """Key vector [D] of (page, kv head, slot) from the K pool format [P][Hkv][D/8][16][8]."""
    return np.asarray(k_pool[page, h, :, slot, :], dtype=np.float64).reshape(-1)


def pool_get_v(v_pool, page, h, slot):
    """Value vector [D] of (page, kv head, slot) from the V pool format [P][Hkv][D][16]."""
    return np.asarray(v_pool[page, h, :, slot], dtype=np.float64)


def kv_append_rope(desc, k_new, v_new, k_pool, v_pool, theta):
    """Write each live branch's new token into the tail of its own page list (in place).

    The key is rotated at the branch's adaptive position; the slot is branch_len-1 counted over
    the branch's own pages.  Pools are float arrays in the formats above; stores keep the pool's
    dtype rounding to the caller (the caller passes arrays of the storage precision).
    """
    n_live = len(desc["branch_len"])
    k_rot = rope(k_new, desc["branch_pos"], theta)
    for r in range(n_live):
        idx = int(desc["branch_len"][r]) - 1
        page = int(desc["branch_pages"][int(desc["branch_page_off"][r]) + idx // PAGE])
        slot = idx % PAGE
        Hkv = k_pool.shape[1]
        for h in range(Hkv):
            k_pool[page, h, :, slot, :] = k_rot[r, h].reshape(-1, 8)
            v_pool[page, h, :, slot] = np.asarray(v_new[r, h], dtype=np.float64)
    return k_rot


def gather_context(desc, r, h, k_pool, v_pool):
    """K, V [ctx][D] seen by live branch r on KV head h: shared tokens, then its own tokens."""
    g = int(np.searchsorted(np.asarray(desc["group_branch_off"]), r, side="right") - 1)
    Ks, Vs = [], []
    for t in range(int(desc["shared_len"][g])):
        page = int(desc["shared_pages"][int(desc["shared_page_off"][g]) + t // PAGE])
        Ks.append(pool_get_k(k_pool, page, h, t % PAGE))
        Vs.append(pool_get_v(v_pool, page, h, t % PAGE))
    for t in range(int(desc["branch_len"][r])):
        page = int(desc["branch_pages"][int(desc["branch_page_off"][r]) + t // PAGE])
        Ks.append(pool_get_k(k_pool, page, h, t % PAGE))
        Vs.append(pool_get_v(v_pool, page, h, t % PAGE))
    return np.array(Ks), np.array(Vs)


def attn_decode(desc, q, k_pool, v_pool, scale=None, branches=None, kv_heads=None):
    """One decode step: o = softmax(q . K^T * scale) V over each branch's context, fp64.

    q [n_live][Hq][D] already rotated.  Returns O [n_live][Hq][D] (NaN for the branches and the
    query heads of the KV heads not asked for).
    """
    q = np.asarray(q, dtype=np.float64)
    n_live, Hq, D = q.shape
    Hkv = k_pool.shape[1]
    G = Hq // Hkv
    if scale is None:
        scale = 1.0 / np.sqrt(D)
    O = np.full((n_live, Hq, D), np.nan)
    for r in (range(n_live) if branches is None else branches):
        for hk in (range(Hkv) if kv_heads is None else kv_heads):
            K, V = gather_context(desc, r, hk, k_pool, v_pool)
            for h in range(hk * G, (hk + 1) * G):
                s = (K @ q[r, h]) * scale
                p = np.exp(s - s.max())
                O[r, h] = (p @ V) / p.sum()
    return O


def gather_segments(sdesc, r, h, k_pool, v_pool):
    """K, V [ctx][D] seen by live branch r on KV head h when contexts are lists of KV segments
    (section 3.2: a token carries references to cached blocks; section 4.3: a Fork hands the same
    context to every child, a Join the histories of all its predecessors): the first seg_len[s]
    tokens of every segment s the branch reads, in the order listed.  With "seg_reader_len" (one
    entry per reader-list position) the branch sees only that many leading tokens of the segment:
    a token of a node that is being prefilled sees the node's tokens up to itself (the same-node
    case of Eq. 3)."""
    Ks, Vs = [], []
    limits = sdesc.get("seg_reader_len")
    for e in range(int(sdesc["branch_seg_off"][r]), int(sdesc["branch_seg_off"][r + 1])):
        s = int(sdesc["branch_segs"][e])
        n = int(sdesc["seg_len"][s])
        if limits is not None:
            r0, r1 = int(sdesc["seg_reader_off"][s]), int(sdesc["seg_reader_off"][s + 1])
            pos = [x for x in range(r0, r1) if int(sdesc["seg_readers"][x]) == r]
            assert len(pos) == 1, "branch %d must be listed once among the readers of segment %d" % (r, s)
            n = min(n, max(0, int(limits[pos[0]])))
        for t in range(n):
            page = int(sdesc["seg_pages"][int(sdesc["seg_page_off"][s]) + t // PAGE])
            Ks.append(pool_get_k(k_pool, page, h, t % PAGE))
            Vs.append(pool_get_v(v_pool, page, h, t % PAGE))
    return np.array(Ks), np.array(Vs)


def attn_decode_segments(sdesc, q, k_pool, v_pool, scale=None, branches=None):
    """One decode step over segment lists: o = softmax(q . K^T * scale) V over the tokens of the
    segments each live branch reads (Eq. 2 with membership as the only mask), fp64.

    q [n_live][Hq][D] already rotated.  Returns O [n_live][Hq][D] (NaN for branches not asked).
    """
    q = np.asarray(q, dtype=np.float64)
    n_live, Hq, D = q.shape
    Hkv = k_pool.shape[1]
    G = Hq // Hkv
    if scale is None:
        scale = 1.0 / np.sqrt(D)
    O = np.full((n_live, Hq, D), np.nan)
    for r in (range(n_live) if branches is None else branches):
        for hk in range(Hkv):
            K, V = gather_segments(sdesc, r, hk, k_pool, v_pool)
            for h in range(hk * G, (hk + 1) * G):
                s = (K @ q[r, h]) * scale
                p = np.exp(s - s.max())
                O[r, h] = (p @ V) / p.sum()
    return O


# ----------------------------------------------------------------------------- log-sum-exp merge
def partial_attention(qvec, K, V, scale):
    """Un-normalised partial over a key subset: (o = sum_j e^{s_j-m} v_j, m = max s, l = sum e^{s_j-m})."""
    s = (np.asarray(K, dtype=np.float64) @ np.asarray(qvec, dtype=np.float64)) * scale
    m = s.max()
    p = np.exp(s - m)
    return p @ np.asarray(V, dtype=np.float64), m, p.sum()


def lse_merge(partials):
    """Combine partials [(o, m, l), ...]: m = max m_s; l = sum l_s e^{m_s-m}; o = sum o_s e^{m_s-m} / l."""
    m = max(p[1] for p in partials)
    l = sum(p[2] * np.exp(p[1] - m) for p in partials)
    o = sum(p[0] * np.exp(p[1] - m) for p in partials)
    return o / l


# ----------------------------------------------------------------------------- scheduling (section 3.3)
def frontier_layers(parents):
    """Enabled-transition frontiers F_0, F_1, ... of Eq. 1 under the execution loop of section 3.3.

    Node v is the output place of one transition whose input places are parents[v] (converging
    edges form one transition, diverging edges one transition per child); nodes without parents
    have an empty pre-set.  The marking is the set of places that hold a token; a transition is
    enabled when every input place is marked and its output place is empty; all enabled
    transitions fire, then the marking advances and the frontier is recomputed, until nothing is
    enabled.  Returns the list of frontiers (lists of node ids, ascending)."""
    n = len(parents)
    marked = [False] * n
    layers = []
    while True:
        frontier = [v for v in range(n) if not marked[v] and all(marked[p] for p in parents[v])]
        if not frontier:
            return layers
        layers.append(frontier)
        for v in frontier:
            marked[v] = True


def schedule_steps(parents, node_len, chunk=None):
    """The engine's steps: frontier after frontier; within a frontier every transition advances
    by chunk[v] tokens per step (1 = token-by-token generation; more = a node whose text is
    given and is prefilled in pieces) until its node_len[v] tokens exist, and the frontier is
    complete when its longest transition is.  Returns a list of steps, each a list of
    (node, first new token inside the node, number of new tokens), nodes ascending."""
    chunk = [1] * len(parents) if chunk is None else chunk
    steps = []
    for frontier in frontier_layers(parents):
        done = {v: 0 for v in frontier}
        while any(done[v] < int(node_len[v]) for v in frontier):
            step = []
            for v in frontier:
                n = min(int(chunk[v]), int(node_len[v]) - done[v])
                if n > 0:
                    step.append((v, done[v], n))
                    done[v] += n
            steps.append(step)
    return steps
