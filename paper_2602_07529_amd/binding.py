"""ctypes binding of libdagattn.so: argument marshalling only.

Every step of the path runs in the library's HIP kernels; PyTorch is used for device memory and
for the current stream handle.  There is no CPU fallback: if the library is missing, loading
raises.  Function names match the C ABI declared in include/dagattn.h.
"""
import ctypes as C
import os

import numpy as np
import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("DAGATTN_LIB") or os.path.join(_PKG, "libdagattn.so")

DAG_F32, DAG_BF16 = 0, 1
DAG_STRICT_CLOSURE = 1
TILE_SKIP, TILE_PARTIAL, TILE_FULL = 0, 1, 2
PAGE = 16


class DagError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__("dagattn error %d: %s" % (code, msg))
        self.code = code


class dag_desc_t(C.Structure):
    _fields_ = [("n_seqs", C.c_int32), ("node_offsets", C.c_void_p), ("node_len", C.c_void_p),
                ("anc_bits", C.c_void_p), ("words_per_node", C.c_int32), ("tile_m", C.c_int32),
                ("tile_n", C.c_int32), ("flags", C.c_uint32)]


class dag_meta_sizes_t(C.Structure):
    _fields_ = [("total_nodes", C.c_int64), ("total_tokens", C.c_int64), ("total_qtiles", C.c_int64),
                ("total_ktiles", C.c_int64), ("total_tiles", C.c_int64), ("csr_capacity", C.c_int64),
                ("workspace_bytes", C.c_int64)]


_META_ARRAYS = [("cu_seqlens", torch.int32), ("node_start", torch.int32), ("tok_node", torch.int32),
                ("pos_ids", torch.int32), ("node_tok_start", torch.int32), ("node_pos_start", torch.int32),
                ("node_vis", torch.int64), ("qtile_start", torch.int32), ("ktile_start", torch.int32),
                ("block_map_off", torch.int64),
                ("block_map", torch.uint8), ("qtile_rowptr", torch.int32), ("qtile_col", torch.int32),
                ("qtile_flag", torch.uint8), ("qtile_nfull", torch.int32), ("qtile_order", torch.int32), ("qtile_desc", torch.int32),
                ("useful_pairs", torch.int64)]


class dag_meta_t(C.Structure):
    _fields_ = ([("n_seqs", C.c_int32), ("words_per_node", C.c_int32), ("tile_m", C.c_int32),
                 ("tile_n", C.c_int32), ("sizes", dag_meta_sizes_t)] +
                [(name, C.c_void_p) for name, _ in _META_ARRAYS])


class dag_decode_desc_t(C.Structure):
    _fields_ = [("n_groups", C.c_int32), ("n_live", C.c_int32), ("page_size", C.c_int32),
                ("max_shared_pages", C.c_int32), ("max_branch_pages", C.c_int32),
                ("max_group_size", C.c_int32),
                ("group_branch_off", C.c_void_p), ("shared_page_off", C.c_void_p),
                ("shared_pages", C.c_void_p), ("shared_len", C.c_void_p),
                ("branch_page_off", C.c_void_p), ("branch_pages", C.c_void_p),
                ("branch_len", C.c_void_p), ("branch_pos", C.c_void_p)]


_SEG_ARRAYS = ("seg_page_off", "seg_pages", "seg_len", "seg_reader_off", "seg_readers", "branch_entry_off",
               "branch_entries")


class dag_decode_seg_desc_t(C.Structure):
    _fields_ = ([("n_live", C.c_int32), ("n_segments", C.c_int32), ("page_size", C.c_int32),
                 ("max_seg_pages", C.c_int32), ("max_readers", C.c_int32), ("total_readers", C.c_int32)] +
                [(name, C.c_void_p) for name in _SEG_ARRAYS] + [("seg_reader_len", C.c_void_p)])


_PAGED_ARRAYS = ("q_off", "ctx_page_off", "ctx_pages", "ctx_page_len", "own_page", "own_len")


class dag_paged_prefill_desc_t(C.Structure):
    _fields_ = ([("n_nodes", C.c_int32), ("page_size", C.c_int32), ("max_new", C.c_int32),
                 ("max_ctx_pages", C.c_int32)] + [(name, C.c_void_p) for name in _PAGED_ARRAYS])


_SCHED_ARRAYS = ("live_node", "live_token", "branch_page_off", "branch_pages", "branch_len", "branch_pos",
                 "seg_node", "seg_page_off", "seg_pages", "seg_len", "seg_reader_off", "seg_readers",
                 "seg_reader_len", "branch_entry_off", "branch_entries")


class dag_sched_step_t(C.Structure):
    _fields_ = ([(name, C.c_int32) for name in ("n_live", "layer", "n_segments", "max_seg_pages", "max_readers",
                                                "total_readers", "n_branch_pages", "n_seg_pages", "pages_in_use")] +
                [(name, C.POINTER(C.c_int32)) for name in _SCHED_ARRAYS])


_lib = None


def lib():
    """Load the shared library (raises if it has not been built)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("libdagattn.so is not built: run `python -m paper_2602_07529_amd.build` "
                               "(there is no CPU fallback)")
        L = C.CDLL(LIB_PATH)
        vp, i32, i64, f32 = C.c_void_p, C.c_int32, C.c_int64, C.c_float
        L.dag_prefill_tile_shape.argtypes = [i32, i32, i32, C.c_int, C.POINTER(i32), C.POINTER(i32)]
        L.dag_meta_sizes.argtypes = [C.POINTER(dag_desc_t), C.POINTER(dag_meta_sizes_t)]
        L.dag_build_meta.argtypes = [C.POINTER(dag_desc_t), C.POINTER(dag_meta_t), vp, C.c_size_t, vp]
        L.dag_rope_qk.argtypes = [vp, i64, vp, vp, i32, i32, i32, f32, C.c_int, vp]
        L.dag_attn_prefill.argtypes = [C.POINTER(dag_meta_t), vp, vp, vp, vp, vp, i32, i32, i32, f32,
                                       C.c_int, vp, C.c_size_t, vp]
        L.dag_attn_prefill_prepared.argtypes = L.dag_attn_prefill.argtypes
        L.dag_prefill_prepare_v.argtypes = [C.POINTER(dag_meta_t), vp, i32, i32, i32, C.c_int, vp, C.c_size_t, vp]
        L.dag_prefill_workspace_bytes.argtypes = [C.POINTER(dag_meta_t), i32, i32, C.c_int]
        L.dag_prefill_workspace_bytes.restype = C.c_size_t
        L.dag_prefill_bwd_workspace_bytes.argtypes = [C.POINTER(dag_meta_t), i32, i32, i32]
        L.dag_prefill_bwd_workspace_bytes.restype = C.c_size_t
        L.dag_attn_prefill_bwd.argtypes = [C.POINTER(dag_meta_t), vp, vp, vp, vp, vp, vp, vp, vp, vp, i32, i32, i32,
                                           f32, C.c_int, vp, C.c_size_t, vp]
        L.dag_kv_append_rope.argtypes = [C.POINTER(dag_decode_desc_t), vp, vp, vp, vp, i32, i32, f32, vp]
        L.dag_decode_workspace_bytes.argtypes = [C.POINTER(dag_decode_desc_t), i32, i32, i32]
        L.dag_decode_workspace_bytes.restype = C.c_size_t
        L.dag_attn_decode.argtypes = [C.POINTER(dag_decode_desc_t), vp, vp, vp, vp, i32, i32, i32, f32,
                                      vp, C.c_size_t, vp]
        L.dag_attn_decode_static.argtypes = [C.POINTER(dag_decode_desc_t), vp, vp, vp, vp, i32, i32, i32, f32, vp]
        L.dag_decode_segments_workspace_bytes.argtypes = [C.POINTER(dag_decode_seg_desc_t), i32, i32, i32]
        L.dag_decode_segments_workspace_bytes.restype = C.c_size_t
        L.dag_attn_decode_segments.argtypes = [C.POINTER(dag_decode_seg_desc_t), vp, vp, vp, vp, i32, i32, i32, f32,
                                               vp, C.c_size_t, vp]
        L.dag_prefill_paged_workspace_bytes.argtypes = [C.POINTER(dag_paged_prefill_desc_t)]
        L.dag_prefill_paged_workspace_bytes.restype = C.c_size_t
        L.dag_attn_prefill_paged.argtypes = [C.POINTER(dag_paged_prefill_desc_t), vp, vp, vp, i32, vp, vp, i32, i32,
                                             i32, f32, vp, C.c_size_t, vp]
        L.dag_copy_calibration.argtypes = [vp, vp, C.c_size_t, vp]
        L.dag_sched_create.argtypes = [i32, vp, vp, vp, vp, i32, i32, C.POINTER(vp)]
        L.dag_sched_destroy.argtypes = [vp]
        L.dag_sched_destroy.restype = None
        L.dag_sched_step.argtypes = [vp, C.POINTER(dag_sched_step_t)]
        L.dag_strerror.argtypes = [C.c_int]
        L.dag_strerror.restype = C.c_char_p
        L.dag_version.restype = C.c_int
        for name in ("dag_prefill_tile_shape", "dag_meta_sizes", "dag_build_meta", "dag_rope_qk",
                     "dag_attn_prefill", "dag_attn_prefill_prepared", "dag_prefill_prepare_v",
                     "dag_kv_append_rope", "dag_attn_decode", "dag_attn_decode_static", "dag_attn_decode_segments",
                     "dag_sched_create", "dag_attn_prefill_paged", "dag_copy_calibration",
                     "dag_attn_prefill_bwd",
                     "dag_sched_step"):
            getattr(L, name).restype = C.c_int
        _lib = L
    return _lib


def _check(rc):
    if rc != 0:
        raise DagError(rc, lib().dag_strerror(rc).decode())


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _ptr(t):
    return C.c_void_p(t.data_ptr()) if t is not None else C.c_void_p(0)


def _dtype_code(t):
    if t.dtype == torch.float32:
        return DAG_F32
    if t.dtype == torch.bfloat16:
        return DAG_BF16
    raise TypeError("unsupported dtype %s" % t.dtype)


def dag_strerror(code):
    return lib().dag_strerror(code).decode()


def dag_version():
    return lib().dag_version()


def dag_prefill_tile_shape(hq, hkv, head_dim, dtype_code):
    tm, tn = C.c_int32(0), C.c_int32(0)
    _check(lib().dag_prefill_tile_shape(hq, hkv, head_dim, dtype_code, C.byref(tm), C.byref(tn)))
    return tm.value, tn.value


class DagDesc:
    """Host-side node table (keeps the numpy arrays alive for the ctypes struct)."""

    def __init__(self, node_offsets, node_len, anc_bits, words_per_node, tile_m, tile_n, flags=0):
        self.node_offsets = np.ascontiguousarray(node_offsets, dtype=np.int32)
        self.node_len = np.ascontiguousarray(node_len, dtype=np.int32)
        self.anc_bits = np.ascontiguousarray(anc_bits, dtype=np.uint64)
        self.c = dag_desc_t(len(self.node_offsets) - 1, self.node_offsets.ctypes.data,
                            self.node_len.ctypes.data, self.anc_bits.ctypes.data,
                            words_per_node, tile_m, tile_n, flags)


def dag_meta_sizes(desc):
    out = dag_meta_sizes_t()
    _check(lib().dag_meta_sizes(C.byref(desc.c), C.byref(out)))
    return out


class DagMeta:
    """Device tables written by dag_build_meta (torch tensors + the ctypes struct pointing at them)."""

    def __init__(self, desc, sizes, device):
        n = desc.c.n_seqs
        W = desc.c.words_per_node
        counts = dict(cu_seqlens=n + 1, node_start=n + 1, tok_node=sizes.total_tokens,
                      pos_ids=sizes.total_tokens, node_tok_start=sizes.total_nodes,
                      node_pos_start=sizes.total_nodes, node_vis=sizes.total_nodes * W,
                      qtile_start=n + 1, ktile_start=n + 1, block_map_off=n + 1, block_map=sizes.total_tiles,
                      qtile_rowptr=sizes.total_qtiles + 1, qtile_col=sizes.csr_capacity,
                      qtile_flag=sizes.csr_capacity, qtile_nfull=sizes.total_qtiles, qtile_order=sizes.total_qtiles, qtile_desc=sizes.total_qtiles * 8,
                      useful_pairs=n)
        self.sizes = sizes
        self.t = {name: torch.empty(max(int(counts[name]), 1), dtype=dt, device=device)
                  for name, dt in _META_ARRAYS}
        self.counts = counts
        self.c = dag_meta_t()
        self.c.n_seqs, self.c.words_per_node = n, W
        self.c.tile_m, self.c.tile_n = desc.c.tile_m, desc.c.tile_n
        self.c.sizes = sizes
        for name, _ in _META_ARRAYS:
            setattr(self.c, name, self.t[name].data_ptr())
        self.workspace = torch.empty(max(int(sizes.workspace_bytes), 16), dtype=torch.uint8, device=device)

    def get(self, name):
        """Valid prefix of a table as a torch tensor."""
        return self.t[name][:int(self.counts[name])]


def dag_build_meta(desc, meta):
    _check(lib().dag_build_meta(C.byref(desc.c), C.byref(meta.c), _ptr(meta.workspace),
                                meta.workspace.numel(), _stream()))


def dag_rope_qk(pos_ids, q, k, theta):
    ref = q if q is not None else k
    n_tokens, d = ref.shape[0], ref.shape[-1]
    hq = q.shape[1] if q is not None else 0
    hkv = k.shape[1] if k is not None else 0
    _check(lib().dag_rope_qk(_ptr(pos_ids), n_tokens, _ptr(q), _ptr(k), hq, hkv, d, float(theta),
                             _dtype_code(ref), _stream()))


def dag_prefill_workspace_bytes(meta, hkv, head_dim, dtype_code):
    return int(lib().dag_prefill_workspace_bytes(C.byref(meta.c), hkv, head_dim, dtype_code))


def _prefill_workspace(meta, hkv, d, like, workspace):
    if workspace is not None:
        return workspace
    need = dag_prefill_workspace_bytes(meta, hkv, d, _dtype_code(like))
    ws = getattr(meta, "prefill_ws", None)
    if ws is None or ws.numel() < need:
        ws = torch.empty(max(need, 256), dtype=torch.uint8, device=like.device)
        meta.prefill_ws = ws
    return ws


def dag_attn_prefill(meta, q, k, v, out, lse=None, softmax_scale=None, workspace=None, prepared=False):
    """`workspace`: uint8 device tensor of dag_prefill_workspace_bytes(); when omitted one is
    allocated (torch) and kept on `meta` for the following calls.  prepared=True calls
    dag_attn_prefill_prepared (the workspace already holds what dag_prefill_prepare_v wrote)."""
    T, hq, d = q.shape
    hkv = k.shape[1]
    if softmax_scale is None:
        softmax_scale = 1.0 / float(d) ** 0.5
    workspace = _prefill_workspace(meta, hkv, d, q, workspace)
    fn = lib().dag_attn_prefill_prepared if prepared else lib().dag_attn_prefill
    _check(fn(C.byref(meta.c), _ptr(q), _ptr(k), _ptr(v), _ptr(out), _ptr(lse), hq, hkv, d, float(softmax_scale),
              _dtype_code(q), _ptr(workspace), workspace.numel(), _stream()))


def dag_prefill_prepare_v(meta, v, hq, workspace=None):
    hkv, d = v.shape[1], v.shape[2]
    workspace = _prefill_workspace(meta, hkv, d, v, workspace)
    _check(lib().dag_prefill_prepare_v(C.byref(meta.c), _ptr(v), hq, hkv, d, _dtype_code(v), _ptr(workspace),
                                       workspace.numel(), _stream()))


class DecodeDesc:
    """Device copies of the decode description arrays + the ctypes struct."""

    def __init__(self, desc, device):
        self.t = {}
        for name in ("group_branch_off", "shared_page_off", "shared_pages", "shared_len",
                     "branch_page_off", "branch_pages", "branch_len", "branch_pos"):
            arr = np.ascontiguousarray(desc[name], dtype=np.int32)
            if arr.size == 0:
                arr = np.zeros(1, dtype=np.int32)
            self.t[name] = torch.from_numpy(arr).to(device)
        ng, nl = int(desc["n_groups"]), int(desc["n_live"])
        sp = np.diff(np.asarray(desc["shared_page_off"])) if ng else np.zeros(0)
        bp = np.diff(np.asarray(desc["branch_page_off"])) if nl else np.zeros(0)
        gs = np.diff(np.asarray(desc["group_branch_off"])) if ng else np.zeros(0)
        self.c = dag_decode_desc_t(ng, nl, int(desc["page_size"]),
                                   int(sp.max()) if sp.size else 0, int(bp.max()) if bp.size else 0,
                                   int(gs.max()) if gs.size else 0,
                                   *[self.t[n].data_ptr() for n in
                                     ("group_branch_off", "shared_page_off", "shared_pages", "shared_len",
                                      "branch_page_off", "branch_pages", "branch_len", "branch_pos")])


def dag_kv_append_rope(ddesc, k_new, v_new, k_pool, v_pool, theta):
    hkv, d = k_new.shape[1], k_new.shape[2]
    _check(lib().dag_kv_append_rope(C.byref(ddesc.c), _ptr(k_new), _ptr(v_new), _ptr(k_pool), _ptr(v_pool),
                                    hkv, d, float(theta), _stream()))


def dag_decode_workspace_bytes(ddesc, hq, hkv, head_dim):
    return int(lib().dag_decode_workspace_bytes(C.byref(ddesc.c), hq, hkv, head_dim))


def dag_attn_decode(ddesc, q, k_pool, v_pool, out, workspace, softmax_scale=None):
    n_live, hq, d = q.shape
    hkv = k_pool.shape[1]
    if softmax_scale is None:
        softmax_scale = 1.0 / float(d) ** 0.5
    _check(lib().dag_attn_decode(C.byref(ddesc.c), _ptr(q), _ptr(k_pool), _ptr(v_pool), _ptr(out), hq, hkv, d,
                                 float(softmax_scale), _ptr(workspace), workspace.numel(), _stream()))


DECODE_STATIC_SCRATCH_BYTES = 32 << 20


def dag_attn_decode_static(ddesc, q, k_pool, v_pool, out, softmax_scale=None):
    """dag_attn_decode without a workspace: the partial results live in the library's own device
    array (DAG_ERR_WORKSPACE when the description needs more than DECODE_STATIC_SCRATCH_BYTES)."""
    n_live, hq, d = q.shape
    hkv = k_pool.shape[1]
    if softmax_scale is None:
        softmax_scale = 1.0 / float(d) ** 0.5
    _check(lib().dag_attn_decode_static(C.byref(ddesc.c), _ptr(q), _ptr(k_pool), _ptr(v_pool), _ptr(out), hq, hkv, d,
                                        float(softmax_scale), _stream()))


class SegDecodeDesc:
    """Device copies of the segment-form decode description arrays + the ctypes struct."""

    def __init__(self, desc, device):
        self.t = {}
        for name in _SEG_ARRAYS:
            arr = np.ascontiguousarray(desc[name], dtype=np.int32)
            if arr.size == 0:
                arr = np.zeros(1, dtype=np.int32)
            self.t[name] = torch.from_numpy(arr).to(device)
        ns, nl = int(desc["n_segments"]), int(desc["n_live"])
        sp = np.diff(np.asarray(desc["seg_page_off"])) if ns else np.zeros(0)
        rd = np.diff(np.asarray(desc["seg_reader_off"])) if ns else np.zeros(0)
        self.c = dag_decode_seg_desc_t(nl, ns, int(desc["page_size"]),
                                       int(sp.max()) if sp.size else 0, int(rd.max()) if rd.size else 0,
                                       int(rd.sum()) if rd.size else 0,
                                       *[self.t[n].data_ptr() for n in _SEG_ARRAYS], None)
        if desc.get("seg_reader_len") is not None:
            arr = np.ascontiguousarray(desc["seg_reader_len"], dtype=np.int32)
            self.t["seg_reader_len"] = torch.from_numpy(arr if arr.size else np.zeros(1, np.int32)).to(device)
            self.c.seg_reader_len = self.t["seg_reader_len"].data_ptr()


def dag_decode_segments_workspace_bytes(sdesc, hq, hkv, head_dim):
    return int(lib().dag_decode_segments_workspace_bytes(C.byref(sdesc.c), hq, hkv, head_dim))


def dag_attn_decode_segments(sdesc, q, k_pool, v_pool, out, workspace, softmax_scale=None):
    n_live, hq, d = q.shape
    hkv = k_pool.shape[1]
    if softmax_scale is None:
        softmax_scale = 1.0 / float(d) ** 0.5
    _check(lib().dag_attn_decode_segments(C.byref(sdesc.c), _ptr(q), _ptr(k_pool), _ptr(v_pool), _ptr(out), hq, hkv,
                                          d, float(softmax_scale), _ptr(workspace), workspace.numel(), _stream()))


def dag_copy_calibration(dst, src):
    """Plain copy by the library's own kernel (the reference point of the HBM counters)."""
    _check(lib().dag_copy_calibration(_ptr(dst), _ptr(src), src.numel() * src.element_size(), _stream()))


class PagedPrefillDesc:
    """Device copies of the paged-prefill description arrays + the ctypes struct.  `desc`: dict with the six
    arrays of dag_paged_prefill_desc_t (host, int32) and page_size."""

    def __init__(self, desc, device):
        self.t = {}
        for name in _PAGED_ARRAYS:
            arr = np.ascontiguousarray(desc[name], dtype=np.int32)
            self.t[name] = torch.from_numpy(arr if arr.size else np.zeros(1, np.int32)).to(device)
        q_off = np.asarray(desc["q_off"])
        p_off = np.asarray(desc["ctx_page_off"])
        n_nodes = len(q_off) - 1
        self.n_rows = int(q_off[-1])
        self.c = dag_paged_prefill_desc_t(n_nodes, int(desc["page_size"]),
                                          int(np.diff(q_off).max()) if n_nodes else 0,
                                          int(np.diff(p_off).max()) if n_nodes else 0,
                                          *[self.t[n].data_ptr() for n in _PAGED_ARRAYS])


def dag_prefill_paged_workspace_bytes(pdesc):
    return int(lib().dag_prefill_paged_workspace_bytes(C.byref(pdesc.c)))


def dag_attn_prefill_paged(pdesc, q, k_pool, v_pool, out, workspace, lse=None, softmax_scale=None):
    _, hq, d = q.shape
    hkv = k_pool.shape[1]
    if softmax_scale is None:
        softmax_scale = 1.0 / float(d) ** 0.5
    _check(lib().dag_attn_prefill_paged(C.byref(pdesc.c), _ptr(q), _ptr(k_pool), _ptr(v_pool), k_pool.shape[0],
                                        _ptr(out), _ptr(lse) if lse is not None else None, hq, hkv, d,
                                        float(softmax_scale), _ptr(workspace), workspace.numel(), _stream()))


class Scheduler:
    """dag_sched_*: the host-side scheduler of the execution phase.  step() returns a dict of
    numpy copies of the step's arrays (None when the net is finished)."""

    def __init__(self, parents, node_len, n_pages, chunk=None, page_size=16):
        n = len(parents)
        off = np.zeros(n + 1, dtype=np.int32)
        off[1:] = np.cumsum([len(p) for p in parents])
        flat = np.asarray([x for p in parents for x in p] or [0], dtype=np.int32)
        ln = np.ascontiguousarray(node_len, dtype=np.int32)
        ch = None if chunk is None else np.ascontiguousarray(chunk, dtype=np.int32)
        self.h = C.c_void_p()
        _check(lib().dag_sched_create(n, off.ctypes.data, flat.ctypes.data, ln.ctypes.data if n else None,
                                      None if ch is None else ch.ctypes.data, int(n_pages), int(page_size),
                                      C.byref(self.h)))

    def step(self):
        st = dag_sched_step_t()
        _check(lib().dag_sched_step(self.h, C.byref(st)))
        if st.n_live == 0:
            return None
        sizes = dict(live_node=st.n_live, live_token=st.n_live, branch_page_off=st.n_live + 1,
                     branch_pages=st.n_branch_pages, branch_len=st.n_live, branch_pos=st.n_live,
                     seg_node=st.n_segments, seg_page_off=st.n_segments + 1, seg_pages=st.n_seg_pages,
                     seg_len=st.n_segments, seg_reader_off=st.n_segments + 1, seg_readers=st.total_readers,
                     seg_reader_len=st.total_readers, branch_entry_off=st.n_live + 1,
                     branch_entries=st.total_readers)
        out = {k: np.ctypeslib.as_array(getattr(st, k), shape=(n,)).copy() if n else np.zeros(0, np.int32)
               for k, n in sizes.items()}
        out.update(n_live=st.n_live, layer=st.layer, n_segments=st.n_segments, page_size=16,
                   pages_in_use=st.pages_in_use)
        return out

    def close(self):
        if self.h:
            lib().dag_sched_destroy(self.h)
            self.h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def dag_prefill_bwd_workspace_bytes(meta, hq, hkv, head_dim):
    return int(lib().dag_prefill_bwd_workspace_bytes(C.byref(meta.c), hq, hkv, head_dim))


def dag_attn_prefill_bwd(meta, q, k, v, out, dout, lse, dq, dk, dv, softmax_scale=None, workspace=None):
    T, hq, d = q.shape
    hkv = k.shape[1]
    if softmax_scale is None:
        softmax_scale = 1.0 / float(d) ** 0.5
    if workspace is None:
        workspace = torch.empty(int(lib().dag_prefill_bwd_workspace_bytes(C.byref(meta.c), hq, hkv, d)),
                                dtype=torch.uint8, device=q.device)
    _check(lib().dag_attn_prefill_bwd(C.byref(meta.c), _ptr(q), _ptr(k), _ptr(v), _ptr(out), _ptr(dout), _ptr(lse),
                                      _ptr(dq), _ptr(dk), _ptr(dv), hq, hkv, d, float(softmax_scale),
                                      _dtype_code(q), _ptr(workspace), workspace.numel(), _stream()))
