"""Example driver of the execution phase for ONE attention layer: the host-side scheduler
(dag_sched_*) decides the live transitions of every step, this loop uploads its descriptions and
calls dag_kv_append_rope and dag_attn_decode_segments on the tokens it names.  The "model" is a
table of per-token q / k / v rows (synthetic), so the loop shows the data flow of the engine, not
a language model.  Argument marshalling only: positions, pages, frontiers come from the scheduler,
attention from the kernels."""
import numpy as np
import torch

from . import binding as B


def run_plan(parents, node_len, q_tok, k_tok, v_tok, theta, n_pages=None, chunk=None, softmax_scale=None,
             on_step=None):
    """Generates every node of the plan (tokens stored node after node in q_tok [T][hq][d],
    k_tok / v_tok [T][hkv][d], bf16 on the GPU; q already rotated, k rotated by the append at the
    adaptive position).  Returns (out [T][hq][d], number of steps, k_pool, v_pool)."""
    dev = q_tok.device
    T, hq, d = q_tok.shape
    hkv = k_tok.shape[1]
    node_len = np.asarray(node_len, dtype=np.int64)
    node_start = np.concatenate([[0], np.cumsum(node_len)])
    if n_pages is None:
        n_pages = int(np.sum((node_len + 15) // 16))
    k_pool = torch.zeros((n_pages, hkv, d // 8, 16, 8), dtype=q_tok.dtype, device=dev)
    v_pool = torch.zeros((n_pages, hkv, d, 16), dtype=q_tok.dtype, device=dev)
    out = torch.zeros_like(q_tok)
    sch = B.Scheduler(parents, node_len, n_pages, chunk)
    ws = torch.empty(1 << 20, dtype=torch.uint8, device=dev)
    n_steps = 0
    zero = np.zeros(1, dtype=np.int32)
    while True:
        st = sch.step()
        if st is None:
            break
        idx = torch.from_numpy(node_start[st["live_node"]] + st["live_token"]).to(dev)
        q, k_new, v_new = q_tok.index_select(0, idx), k_tok.index_select(0, idx), v_tok.index_select(0, idx)
        append = dict(n_groups=0, n_live=st["n_live"], page_size=16, group_branch_off=zero, shared_page_off=zero,
                      shared_pages=zero, shared_len=zero, branch_page_off=st["branch_page_off"],
                      branch_pages=st["branch_pages"], branch_len=st["branch_len"], branch_pos=st["branch_pos"])
        B.dag_kv_append_rope(B.DecodeDesc(append, dev), k_new, v_new, k_pool, v_pool, theta)
        sd = B.SegDecodeDesc(st, dev)
        need = B.dag_decode_segments_workspace_bytes(sd, hq, hkv, d)
        if need > ws.numel():
            ws = torch.empty(need, dtype=torch.uint8, device=dev)
        o = torch.empty_like(q)
        B.dag_attn_decode_segments(sd, q, k_pool, v_pool, o, ws, softmax_scale=softmax_scale)
        out.index_copy_(0, idx, o)
        n_steps += 1
        if on_step is not None:
            on_step(st)
    sch.close()
    return out, n_steps, k_pool, v_pool
