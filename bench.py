#!/usr/bin/env python3
"""Benchmark of the DAG-attention hot path on one MI355X.

One step = one pass of the whole hot path over one batch of seeded synthetic input:
  prefill segment (workload "llama3_8b_prefill_bf16", benchmark config 2):
      dag_build_meta -> dag_rope_qk -> dag_attn_prefill (as its two halves: prepare_v, attention)
  decode segment  (workload "branch_decode_bf16", benchmark config 3):
      dag_kv_append_rope -> dag_attn_decode (shared-prefix items + own items + LSE merge)
Inputs are resident in HBM before the timed region.  `value` is the prefill segment's useful
TFLOP/s (4*D*Hq*visible pairs / segment time); the decode segment is reported in "decode".
Beside the timed region, each with a roofline object of its own: the largest configuration
(benchmark config 5: prefill of 2 x 50,176 tokens with 40 query heads, and its 64-branch decode
over a 32,768-token prefix), the random multi-level DAGs of config 4, the segment form of the
decode step and the backward of the prefill attention.
Prints ONE JSON line on stdout.
"""
import argparse
import json
import os
import sys
import time

import numpy as np
import torch

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

from paper_2602_07529_amd import binding as B  # noqa: E402
from workloads import dags  # noqa: E402

MFMA_BF16_PEAK_TFLOPS = 2500.0   # MI355X dense bf16
HBM_PEAK_GBS = 8000.0            # MI355X HBM3E
# HBM bytes per launch come from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this file (one
# counter per run), scaled by what the same counter reads for a plain 256 MiB copy.  They are
# measured, not computed here: `python bench.py --write-traffic <fetch csv> <write csv>` turns the
# two counter files into profiles/traffic.json, which a normal run reads (kernels that are not in
# the file report null).
TRAFFIC_JSON = os.path.join(ROOT, "profiles", "traffic.json")
CALIBRATION_KIB = 256 * 1024


def write_traffic(workload, fetch_csv, write_csv, out_path=TRAFFIC_JSON):
    """Per kernel of one workload (a `--only` choice): mean FETCH_SIZE / WRITE_SIZE per dispatch,
    scaled so that the calibration copy (--copy-calibration: one 256 MiB device copy) reads and
    writes exactly its size.  Other workloads' entries in the file are kept."""
    import csv
    import collections
    import re

    def per_kernel(path):
        agg = collections.defaultdict(list)
        for r in csv.DictReader(open(path)):
            agg[r["Kernel_Name"]].append(float(r["Counter_Value"]))
        return agg

    def short(name):   # "void (anonymous namespace)::k_decode<128>(DecodeArgs)" -> "k_decode<128>"
        m = re.search(r"(k_[A-Za-z0-9_]+(<[^>]*>)?)", name)
        return m.group(1).replace(" ", "") if m else None

    try:
        out = json.load(open(out_path))
    except Exception:
        out = {}
    out["_about"] = ("HBM-side bytes per launch from rocprofv3 --pmc FETCH_SIZE and WRITE_SIZE runs of "
                     "`bench.py --only WORKLOAD --steps 3 --warmup 1 --copy-calibration --no-cpu-baseline`, "
                     "written by bench.py --write-traffic; scale = 256 MiB / what the counter reads for a "
                     "plain 256 MiB copy")
    entry = out.setdefault("workloads", {})[workload] = {"kernels": {}}
    for key, path in (("fetch", fetch_csv), ("write", write_csv)):
        agg = per_kernel(path)
        # the calibration copy: the library's own copy kernel on 256 MiB
        cal = [v for k, v in agg.items() if short(k) == "k_copy_calibration"]
        scale = CALIBRATION_KIB / (sum(cal[0]) / len(cal[0])) if cal else None
        entry[key + "_scale"] = scale
        for k, v in agg.items():
            name = short(k)
            if name is None or scale is None or name == "k_copy_calibration":
                continue
            v = v[len(v) // 2:]   # the later dispatches: steady state
            d = entry["kernels"].setdefault(name, {})
            d[key + "_bytes"] = int(sum(v) / len(v) * scale * 1024)
            d[key + "_dispatches"] = len(v)
    with open(out_path, "w") as f:
        json.dump(out, f, indent=1, sort_keys=True)
    return out


def traffic_of(workload, *kernels):
    """Measured bytes per launch (read + written) of the named kernels of a workload, summed; None
    when the summary file has no entry for one of them."""
    try:
        t = json.load(open(TRAFFIC_JSON))["workloads"][workload]["kernels"]
        return int(sum(t[k]["fetch_bytes"] + t[k]["write_bytes"] for k in kernels))
    except Exception:
        return None


def _ensure_built():
    if not os.path.exists(B.LIB_PATH):
        from paper_2602_07529_amd import build
        build.build()


CLOCK_RAMP_STEPS = 40


class PrefillWork:
    def __init__(self, cfg, dev, device_values=False):
        """device_values: draw Q/K/V with torch's seeded generator on the GPU (same distribution,
        N(0,1) x scale rounded to bf16) instead of numpy on the host; used for the large legs, whose
        host generation alone would take longer than their timed work."""
        self.cfg = cfg
        self.dag_list = dags.config_dags(cfg)
        self.T = int(sum(int(np.sum(L)) for L, _ in self.dag_list))
        hq, hkv, d = cfg["hq"], cfg["hkv"], cfg["d"]
        dtype = torch.float32 if cfg["dtype"] == "f32" else torch.bfloat16
        if device_values:
            gen = torch.Generator(device=dev).manual_seed(cfg["seed"])
            draw = lambda h: (torch.randn(self.T, h, d, device=dev, generator=gen) * cfg["scale"]).to(dtype)
            self.q0, self.k0, self.v = draw(hq), draw(hkv), draw(hkv)
        else:
            q, k, v = dags.make_qkv(cfg["seed"], self.T, hq, hkv, d, cfg["scale"], dtype)
            self.q0, self.k0, self.v = q.to(dev), k.to(dev), v.to(dev)
        self.q, self.k = torch.empty_like(self.q0), torch.empty_like(self.k0)
        self.out = torch.empty_like(self.q0)
        code = B.DAG_F32 if dtype == torch.float32 else B.DAG_BF16
        tm, tn = B.dag_prefill_tile_shape(hq, hkv, d, code)
        off, lens, bits, W = dags.batch_desc(self.dag_list)
        self.desc = B.DagDesc(off, lens, bits, W, tm, tn, 0)
        self.meta = B.DagMeta(self.desc, B.dag_meta_sizes(self.desc), dev)
        self.theta = cfg["theta"]

    def refresh_inputs(self):
        """Restore the un-rotated Q/K (RoPE works in place).  Not needed between timed steps: a
        step rotates Q and K once more, which changes neither shapes nor magnitudes."""
        self.q.copy_(self.q0)
        self.k.copy_(self.k0)

    def run(self, ev=None):
        """ev: three events (torch's current stream is the one the library launches on)."""
        if ev:
            ev[0].record()
        B.dag_build_meta(self.desc, self.meta)
        B.dag_rope_qk(self.meta.get("pos_ids"), self.q, self.k, self.theta)
        B.dag_prefill_prepare_v(self.meta, self.v, self.cfg["hq"])
        if ev:
            ev[1].record()
        # dag_attn_prefill = prepare_v + this call; launched separately here so that the events
        # bracket exactly one kernel (k_prefill_bf16), the one the roofline is quoted on
        B.dag_attn_prefill(self.meta, self.q, self.k, self.v, self.out, prepared=True)
        if ev:
            ev[2].record()

    def algorithmic_bytes(self):
        """Q read and out written once, K and the transposed V read once."""
        c = self.cfg
        return (2 * self.T * c["hq"] + 2 * self.T * c["hkv"]) * c["d"] * 2

    def useful_flops(self):
        pairs = int(self.meta.get("useful_pairs").sum().item())
        return 4.0 * self.cfg["d"] * self.cfg["hq"] * pairs, pairs


class DecodeWork:
    def __init__(self, cfg, dev, copies=2):
        self.cfg = cfg
        st = dags.decode_state(cfg["seed"], cfg["n_seqs"], cfg["n_branch"], cfg["shared"], cfg["branch"],
                               cfg["hq"], cfg["hkv"], cfg["d"])
        self.desc_np = st["desc"]
        self.dd = B.DecodeDesc(st["desc"], dev)
        # several copies of the pools, used in turn, so that no step finds its K/V in the 256 MB
        # last-level cache from the step before (two copies of 1 GiB for config 3; the 0.4 GiB of
        # config 5 needs more turns)
        kp, vp = st["k_pool"].to(dev), st["v_pool"].to(dev)
        self.pools = [(kp, vp)] + [(kp.clone(), vp.clone()) for _ in range(copies - 1)]
        self.turn = 0
        self.q, self.k_new, self.v_new = st["q"].to(dev), st["k_new"].to(dev), st["v_new"].to(dev)
        self.out = torch.empty_like(self.q)
        self.ws = torch.empty(B.dag_decode_workspace_bytes(self.dd, cfg["hq"], cfg["hkv"], cfg["d"]),
                              dtype=torch.uint8, device=dev)
        self.bytes = dags.decode_algorithmic_bytes(st["desc"], cfg["hkv"], cfg["d"])
        self.n_live = st["desc"]["n_live"]

    def run(self, ev=None):
        kp, vp = self.pools[self.turn]
        self.turn = (self.turn + 1) % len(self.pools)
        if ev:
            ev[0].record()
        B.dag_kv_append_rope(self.dd, self.k_new, self.v_new, kp, vp, self.cfg["theta"])
        if ev:
            ev[1].record()
        B.dag_attn_decode(self.dd, self.q, kp, vp, self.out, self.ws)
        if ev:
            ev[2].record()


class SegDecodeWork:
    """A three-level decode frontier for dag_attn_decode_segments: 16 sequences, each a root of
    4096 tokens, two mid-level nodes of 2048 and four live leaves under each with 1000..1063 own
    tokens (ragged last pages); shapes of config 3.  Reported beside the main line, not part of
    `value`."""

    def __init__(self, cfg, dev, n_seqs=16):
        self.cfg = cfg
        rng = np.random.Generator(np.random.PCG64(cfg["seed"] + 77))
        parents = [[], [0], [0]] + [[1]] * 4 + [[2]] * 4
        anc = dags.bits_from_sets(dags.closure_from_parents(parents))
        dag_list = [(np.asarray([4096, 2048, 2048] + [1000 + int(rng.integers(64)) for _ in range(8)], dtype=np.int32),
                     anc) for _ in range(n_seqs)]
        st = dags.decode_segments_state(cfg["seed"] + 78, dag_list, [list(range(3, 11))] * n_seqs, cfg["hq"],
                                        cfg["hkv"], cfg["d"], keep_tokens=False)
        self.sd = B.SegDecodeDesc(st["desc"], dev)
        kp, vp = st["k_pool"].to(dev), st["v_pool"].to(dev)
        self.pools = [(kp, vp), (kp.clone(), vp.clone())]   # used in turn, as in DecodeWork
        self.turn = 0
        self.q = st["q"].to(dev)
        self.out = torch.empty_like(self.q)
        self.ws = torch.empty(B.dag_decode_segments_workspace_bytes(self.sd, cfg["hq"], cfg["hkv"], cfg["d"]),
                              dtype=torch.uint8, device=dev)
        self.bytes = dags.decode_segments_algorithmic_bytes(st["desc"], cfg["hkv"], cfg["d"])
        self.n_live, self.n_segments = st["desc"]["n_live"], st["desc"]["n_segments"]

    def run(self):
        kp, vp = self.pools[self.turn]
        self.turn ^= 1
        B.dag_attn_decode_segments(self.sd, self.q, kp, vp, self.out, self.ws)


def paged_prefill_leg(cfg, dev, steps, warmup, n_new=256, cached=1024):
    """Beside the timed region: dag_attn_prefill_paged on contexts of config 3's shape -- per
    sequence a shared prefix and 8 nodes with `cached` tokens in their pages, each prefilling
    n_new further tokens at once (their K/V already appended).  Useful FLOPs: 4 D per (new token,
    visible token, query head)."""
    nb, n_seqs = cfg["n_branch"], cfg["n_seqs"]
    dag = dags.fork_join(cfg["shared"], [cached + n_new] * nb, None)
    st = dags.decode_segments_state(cfg["seed"] + 55, [dag] * n_seqs, [list(range(1, nb + 1))] * n_seqs, cfg["hq"],
                                    cfg["hkv"], cfg["d"], keep_tokens=False, new_tokens=[[n_new] * nb] * n_seqs)
    pd = B.PagedPrefillDesc(st["paged"], dev)
    kp, vp, q = st["k_pool"].to(dev), st["v_pool"].to(dev), st["q"].to(dev)
    out = torch.empty_like(q)
    ws = torch.empty(B.dag_prefill_paged_workspace_bytes(pd), dtype=torch.uint8, device=dev)
    pairs = n_seqs * nb * sum(cfg["shared"] + cached + i + 1 for i in range(n_new))
    flops = 4.0 * cfg["d"] * cfg["hq"] * pairs
    for _ in range(warmup):
        B.dag_attn_prefill_paged(pd, q, kp, vp, out, ws)
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
    for e0, e1 in ev:
        e0.record()
        B.dag_attn_prefill_paged(pd, q, kp, vp, out, ws)
        e1.record()
    torch.cuda.synchronize()
    ms = float(np.mean([e0.elapsed_time(e1) for e0, e1 in ev]))
    tf = flops / (ms * 1e-3) / 1e12
    kern = "k_prefill_bf16<128,4,2,true>"
    return {"metric": "dag_attn_prefill_paged_useful_tflops", "value": tf, "unit": "TFLOP/s", "ms_per_call": ms,
            "calls": steps,
            "config": {"workload": "paged_node_prefill_bf16", "n_seqs": n_seqs, "nodes": n_seqs * nb,
                       "new_tokens_per_node": n_new, "cached_tokens_per_node": cached, "shared_prefix": cfg["shared"],
                       "hq": cfg["hq"], "hkv": cfg["hkv"], "head_dim": cfg["d"], "page_size": 16, "useful_pairs": pairs},
            "roofline": {"bound": "mfma", "kernel": "k_paged_rows+k_wide_order+" + kern, "achieved": tf,
                         "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": tf / MFMA_BF16_PEAK_TFLOPS,
                         "traffic": traffic_of("paged", kern)}}


def cpu_baseline(pw, n_seq=3):
    """The oracle as it stands, timed on the host cores on a bounded sample of the prefill workload:
    the first n_seq sequences, every row, every query head (10 - 20 s of CPU work)."""
    from oracle import dag_oracle as orc
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count()
    cfg = pw.cfg
    heads = list(range(cfg["hq"]))
    n_seq = min(n_seq, len(pw.dag_list))
    dt, pairs, t0_tok, rows = 0.0, 0, 0, 0
    for L, anc in pw.dag_list[:n_seq]:
        Tb = int(np.sum(L))
        q64 = dags.to_f64(pw.q0[t0_tok:t0_tok + Tb].cpu())
        k64 = dags.to_f64(pw.k0[t0_tok:t0_tok + Tb].cpu())
        v64 = dags.to_f64(pw.v[t0_tok:t0_tok + Tb].cpu())
        t0 = time.perf_counter()
        _, pos = orc.token_meta(L, anc)
        qs, ks = orc.rope(q64, pos, cfg["theta"]), orc.rope(k64, pos, cfg["theta"])
        orc.attn_prefill(qs, ks, v64, L, anc, heads=heads)
        dt += time.perf_counter() - t0
        pairs += orc.useful_pairs(L, anc)
        t0_tok += Tb
        rows += Tb
    flops = 4.0 * cfg["d"] * len(heads) * pairs
    return {"value": flops / dt / 1e12, "unit": "TFLOP/s", "cores": int(cores), "kind": "oracle",
            "sample": "sequences 0..%d of %d, all %d rows, %d of %d query heads, fp64 numpy; %.1f s"
                      % (n_seq - 1, cfg["batch"], rows, len(heads), cfg["hq"], dt)}


def _events(n):
    return [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(n)]


def backward_timing(pw, dev, calls, warmup):
    """dag_attn_prefill_bwd on a prefill workload (after one forward that leaves the log-sum-exp):
    ms per call between two events, and the same as useful TFLOP/s (2.5 x the forward's)."""
    cfg = pw.cfg
    lse = torch.empty(pw.T, cfg["hq"], dtype=torch.float32, device=dev)
    B.dag_attn_prefill(pw.meta, pw.q, pw.k, pw.v, pw.out, lse)
    dout = torch.randn(pw.q.shape, device=dev, generator=torch.Generator(device=dev).manual_seed(cfg["seed"])).to(pw.q.dtype)
    dq, dk, dv = torch.empty_like(pw.q), torch.empty_like(pw.k), torch.empty_like(pw.v)
    ws = torch.empty(B.dag_prefill_bwd_workspace_bytes(pw.meta, cfg["hq"], cfg["hkv"], cfg["d"]), dtype=torch.uint8, device=dev)
    bwd = lambda: B.dag_attn_prefill_bwd(pw.meta, pw.q, pw.k, pw.v, pw.out, dout, lse, dq, dk, dv, workspace=ws)
    for _ in range(warmup):
        bwd()
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    ev[0].record()
    for _ in range(calls):
        bwd()
    ev[1].record()
    torch.cuda.synchronize()
    ms = ev[0].elapsed_time(ev[1]) / calls
    flops, _ = pw.useful_flops()
    return ms, 2.5 * flops / (ms * 1e-3) / 1e12


def bwd_kernels(G):
    """The launches of dag_attn_prefill_bwd at head dimension 128 with G query heads per KV head: groups of
    four heads on one query tile (k_bwd_dq2<false>), the left-over heads on four query tiles each."""
    wide = G % 4
    dq = (("k_bwd_dq2<false>",) if G - wide > 0 else ()) + (("k_bwd_wide_rows", "k_bwd_dq2<true>") if wide else ())
    return ("k_bwd_delta<128>", "k_bwd_tokvis") + dq + ("k_bwd_weights", "k_bwd_order", "k_bwd_dkv2")


def prefill_leg(cfg, dev, launches, warmup, workload_key, with_bwd=False):
    """An extra prefill workload beside the timed region: the whole prefill path `launches` times,
    the attention kernel bracketed by events of its own.  Returns the JSON object of the leg."""
    pw = PrefillWork(cfg, dev, device_values=True)
    pw.refresh_inputs()
    for _ in range(warmup):
        pw.run()
    ev = _events(launches)
    for e in ev:
        pw.run(e)
    torch.cuda.synchronize()
    ms_path = float(np.mean([e[0].elapsed_time(e[2]) for e in ev]))
    attn = [e[1].elapsed_time(e[2]) for e in ev]
    ms_attn = float(np.mean(attn))
    flops, pairs = pw.useful_flops()
    tf = flops / (ms_attn * 1e-3) / 1e12
    bmap = pw.meta.get("block_map")
    census = {"full": int((bmap == B.TILE_FULL).sum().item()), "partial": int((bmap == B.TILE_PARTIAL).sum().item())}
    # the launches of one call: four-head items on 64-row tiles, left-over heads (one or two) on 256-row tiles
    g = cfg["hq"] // cfg["hkv"]
    wide = g % 4 if g % 4 < 3 else 0
    kerns = (["k_prefill_bf16<%d,4,2,false>" % cfg["d"]] if g > wide else []) + \
            (["k_prefill_bf16<%d,1,8,false>" % cfg["d"]] if wide else [])
    bwd = None
    if with_bwd:
        ms_bwd, tf_bwd = backward_timing(pw, dev, 3, 1)
        bwd = {"metric": "dag_attn_prefill_bwd_useful_tflops", "value": tf_bwd, "unit": "TFLOP/s", "ms_per_call": ms_bwd,
               "calls": 3, "roofline": {"bound": "mfma", "kernel": "+".join(bwd_kernels(cfg["hq"] // cfg["hkv"])), "achieved": tf_bwd,
                                        "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                                        "frac": tf_bwd / MFMA_BF16_PEAK_TFLOPS,
                                        "traffic": traffic_of(workload_key, *bwd_kernels(cfg["hq"] // cfg["hkv"]))}}
    return {"metric": "dag_attn_prefill_useful_tflops", "value": flops / (ms_path * 1e-3) / 1e12, "unit": "TFLOP/s",
            "prefill_bwd": bwd,
            "launches": launches, "ms_prefill_path(meta+rope+attn)": ms_path, "ms_attn_kernel": ms_attn,
            "min_ms_attn_kernel": float(np.min(attn)),
            "config": {"workload": cfg["name"], "batch": cfg["batch"], "tokens": pw.T, "hq": cfg["hq"],
                       "hkv": cfg["hkv"], "head_dim": cfg["d"], "useful_pairs": pairs, "tiles_64x64": census,
                       "values": "torch generator on the device, seed %d" % cfg["seed"]},
            "roofline": {"bound": "mfma", "kernel": "+".join(kerns), "achieved": tf, "peak": MFMA_BF16_PEAK_TFLOPS,
                         "unit": "TFLOP/s", "frac": tf / MFMA_BF16_PEAK_TFLOPS,
                         "traffic": traffic_of(workload_key, *kerns), "algorithmic_bytes": pw.algorithmic_bytes()}}


def decode_leg(cfg, dev, steps, warmup, workload_key, kernels, copies):
    """An extra decode workload beside the timed region: `steps` decode steps one after the other,
    dag_attn_decode bracketed by events of its own."""
    dw = DecodeWork(cfg, dev, copies=copies)
    for _ in range(warmup):
        dw.run()
    ev = _events(steps)
    for e in ev:
        dw.run(e)
    torch.cuda.synchronize()
    ms_step = float(np.mean([e[0].elapsed_time(e[2]) for e in ev]))
    att = [e[1].elapsed_time(e[2]) for e in ev]
    ms_att = float(np.mean(att))
    gbs = dw.bytes / (ms_att * 1e-3) / 1e9
    return {"metric": "branch_decode_tok_per_s_one_attention_layer", "value": dw.n_live / (ms_step * 1e-3),
            "unit": "tok/s", "ms_per_decode_step": ms_step, "ms_attn_kernels": ms_att,
            "min_ms_attn_kernels": float(np.min(att)), "steps": steps,
            "config": {"workload": cfg["name"], "n_seqs": cfg["n_seqs"], "live_branches": dw.n_live,
                       "shared_prefix": cfg["shared"], "branch_len": cfg["branch"], "hq": cfg["hq"], "hkv": cfg["hkv"],
                       "page_size": 16, "pool_copies_used_in_turn": copies},
            "roofline": {"bound": "hbm", "kernel": "+".join(kernels), "achieved": gbs, "peak": HBM_PEAK_GBS,
                         "unit": "GB/s", "frac": gbs / HBM_PEAK_GBS, "algorithmic_bytes": dw.bytes,
                         "traffic": traffic_of(workload_key, *kernels)}}


def config5_decode_cfg():
    """Decode state of benchmark config 5: 2 sequences x 32 live branches at own length 640 (the
    middle of the 256 steps, 513..768) over the 32768-token prefix, 40 query / 8 KV heads."""
    c = dags.config(4)
    return dict(name="qwen32b_long_decode_bf16", seed=c["seed"] + 1000, n_seqs=c["batch"], n_branch=c["n_branch"],
                shared=c["prefix"], branch=c["branch"] + c["decode_steps"] // 2, hq=c["hq"], hkv=c["hkv"], d=c["d"],
                theta=c["theta"])


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--only", choices=["all", "main", "config4", "config5", "paged"], default="all",
                    help="main = the timed region (configs 2 and 3) with the segment decode and the backward; "
                         "config4 / config5 = only that leg (for profiler runs)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one plain 256 MiB device copy by the library's copy kernel (untimed): under "
                         "rocprofv3 --pmc its FETCH_SIZE / WRITE_SIZE give the scale of those counters")
    ap.add_argument("--write-traffic", nargs=3, metavar=("WORKLOAD", "FETCH_CSV", "WRITE_CSV"),
                    help="no GPU work: turn two rocprofv3 counter files of a `--only WORKLOAD "
                         "--copy-calibration` run into that workload's entry of profiles/traffic.json")
    args = ap.parse_args()
    if args.write_traffic:
        print(json.dumps(write_traffic(*args.write_traffic)["workloads"][args.write_traffic[0]], indent=1))
        return
    if args.gpus != 1:
        print("bench.py: this build measures one GPU only (the path shards by sequence or KV head without any "
              "exchange inside attention, so N GPUs run N copies of this job); run with --gpus 1", file=sys.stderr)
        sys.exit(2)
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        sys.exit(2)
    _ensure_built()
    dev = "cuda:0"
    torch.cuda.set_device(0)
    if args.copy_calibration:
        src = torch.ones(256 << 20, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        B.dag_copy_calibration(dst, src)
        torch.cuda.synchronize()
        del src, dst
    extra = {}
    if args.only in ("all", "config5"):
        c5 = dags.config(4)
        c5["name"] = "qwen32b_long_prefill_bf16"
        n5 = max(1, min(args.steps, 4))
        extra["config5_prefill"] = prefill_leg(c5, dev, n5, min(args.warmup, 2), "config5", with_bwd=True)
        torch.cuda.empty_cache()
        extra["config5_decode"] = decode_leg(config5_decode_cfg(), dev, args.steps, args.warmup + 20, "config5",
                                             ("k_decode_wide<128>", "k_decode_merge<128>"), copies=4)
    if args.only in ("all", "config4"):
        extra["config4_prefill"] = prefill_leg(dags.config(3), dev, max(1, min(args.steps, 20)),
                                               min(args.warmup, 5) + 10, "config4", with_bwd=True)
    if args.only in ("all", "paged"):
        extra["paged_prefill"] = paged_prefill_leg(dags.config(2), dev, max(1, min(args.steps, 10)), min(args.warmup, 3))
        torch.cuda.empty_cache()
    if args.only in ("config4", "config5", "paged"):
        print(json.dumps(extra))
        return
    torch.cuda.empty_cache()

    pw = PrefillWork(dags.config(1), dev)
    dw = DecodeWork(dags.config(2), dev)
    pw.refresh_inputs()
    # From a cold start the GPU needs some tens of milliseconds of load to reach its sustained
    # clocks (the first ~20 steps run about 12 % slower than all later ones), so a fixed number of
    # untimed steps comes first, whatever --warmup says; then the W warm-up steps proper.
    for _ in range(CLOCK_RAMP_STEPS + args.warmup):
        pw.run()
        dw.run()
    pev = _events(args.steps)
    dev_ev = _events(args.steps)

    # exactly `steps` steps between two synchronisations; the host runs ahead of the GPU, so the
    # per-kernel event intervals below contain no launch gaps
    torch.cuda.synchronize()
    wall0 = time.perf_counter()
    # the K steps' work in the order a serving job does it: the prefill passes, then the decode
    # steps one after the other (a decode step right after a prefill pass runs ~12 % slower than in
    # a run of decode steps)
    for i in range(args.steps):
        pw.run(pev[i])
    for i in range(args.steps):
        dw.run(dev_ev[i])
    torch.cuda.synchronize()
    wall = time.perf_counter() - wall0
    pre_ms = [e[0].elapsed_time(e[2]) for e in pev]
    attn_ms = [e[1].elapsed_time(e[2]) for e in pev]
    dec_ms = [e[0].elapsed_time(e[2]) for e in dev_ev]
    deck_ms = [e[1].elapsed_time(e[2]) for e in dev_ev]
    step_ms = [wall * 1e3 / args.steps]

    # beside the timed region: the segment form of the decode step on a three-level frontier
    sw = SegDecodeWork(dags.config(2), dev)
    for _ in range(args.warmup):
        sw.run()
    sev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    sev[0].record()
    for _ in range(args.steps):
        sw.run()
    sev[1].record()
    torch.cuda.synchronize()
    ms_seg = sev[0].elapsed_time(sev[1]) / args.steps
    seg_gbs = sw.bytes / (ms_seg * 1e-3) / 1e9

    # beside the timed region: the backward of the prefill attention on the same workload
    n_bwd = max(1, min(args.steps, 10))
    ms_bwd, bwd_tf = backward_timing(pw, dev, n_bwd, min(args.warmup, 3))

    flops, pairs = pw.useful_flops()
    mean = lambda xs: float(np.mean(xs))
    ms_step, ms_pre, ms_attn, ms_dec, ms_deck = map(mean, (step_ms, pre_ms, attn_ms, dec_ms, deck_ms))
    tflops_seg = flops / (ms_pre * 1e-3) / 1e12
    tflops_kernel = flops / (ms_attn * 1e-3) / 1e12
    dec_gbs = dw.bytes / (ms_deck * 1e-3) / 1e9
    cfg = pw.cfg
    bwd_k = bwd_kernels(cfg["hq"] // cfg["hkv"])
    res = {
        "metric": "dag_attn_prefill_useful_tflops",
        "value": tflops_seg,
        "unit": "TFLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": cfg["name"], "batch": cfg["batch"], "tokens_per_seq": pw.T // cfg["batch"],
                   "dag": "prefix %d -> %d branches x %d -> join %d" % (cfg["prefix"], cfg["n_branch"], cfg["branch"], cfg["join"]),
                   "hq": cfg["hq"], "hkv": cfg["hkv"], "head_dim": cfg["d"], "useful_pairs": pairs,
                   "decode_workload": dw.cfg["name"]},
        "segments_ms": {"prefill_path(meta+rope+attn)": ms_pre, "prefill_attn_kernel": ms_attn,
                        "decode_path(append+attn+merge)": ms_dec, "decode_attn_kernels": ms_deck,
                        "min_prefill_attn_kernel": float(np.min(attn_ms)), "min_decode_attn_kernels": float(np.min(deck_ms))},
        "roofline": {"bound": "mfma", "kernel": "k_prefill_bf16<128,4,2,false>", "achieved": tflops_kernel,
                     "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": tflops_kernel / MFMA_BF16_PEAK_TFLOPS,
                     "traffic": traffic_of("main", "k_prefill_bf16<128,4,2,false>"), "algorithmic_bytes": pw.algorithmic_bytes()},
        "decode": {"metric": "branch_decode_tok_per_s_one_attention_layer",
                   "value": dw.n_live / (ms_dec * 1e-3), "unit": "tok/s", "ms_per_decode_step": ms_dec,
                   "config": {"workload": dw.cfg["name"], "n_seqs": dw.cfg["n_seqs"], "live_branches": dw.n_live,
                              "shared_prefix": dw.cfg["shared"], "branch_len": dw.cfg["branch"], "page_size": 16},
                   "roofline": {"bound": "hbm", "kernel": "k_decode<128>+k_decode_merge<128>", "achieved": dec_gbs,
                                "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": dec_gbs / HBM_PEAK_GBS,
                                "algorithmic_bytes": dw.bytes,
                                "traffic": traffic_of("main", "k_decode<128>", "k_decode_merge<128>")}},
        "decode_segments": {"metric": "segment_decode_tok_per_s_one_attention_layer",
                            "value": sw.n_live / (ms_seg * 1e-3), "unit": "tok/s", "ms_per_decode_step": ms_seg,
                            "config": {"workload": "three_level_frontier_bf16", "n_seqs": 16, "segments": sw.n_segments,
                                       "live_branches": sw.n_live, "levels": "root 4096 | 2 x 2048 | 8 x 1000..1063",
                                       "page_size": 16},
                            "roofline": {"bound": "hbm", "kernel": "k_seg_plan+k_decode_seg<128>+k_decode_seg_merge<128>",
                                         "achieved": seg_gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                                         "frac": seg_gbs / HBM_PEAK_GBS, "algorithmic_bytes": sw.bytes,
                                         "traffic": traffic_of("main", "k_seg_plan", "k_decode_seg<128>",
                                                               "k_decode_seg_merge<128>")}},
        "prefill_bwd": {"metric": "dag_attn_prefill_bwd_useful_tflops", "value": bwd_tf,
                        "unit": "TFLOP/s", "ms_per_call": ms_bwd, "calls": n_bwd,
                        "useful_flops": "2.5 x forward (five products per visible pair)",
                        "roofline": {"bound": "mfma", "kernel": "+".join(bwd_k),
                                     "achieved": bwd_tf, "peak": MFMA_BF16_PEAK_TFLOPS,
                                     "unit": "TFLOP/s", "frac": bwd_tf / MFMA_BF16_PEAK_TFLOPS,
                                     "traffic": traffic_of("main", *bwd_k)}},
        "wall_s_timed_loop": wall,
    }
    res.update(extra)
    if not args.no_cpu_baseline:
        res["cpu_baseline"] = cpu_baseline(pw)
    print(json.dumps(res))


if __name__ == "__main__":
    main()
