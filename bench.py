#!/usr/bin/env python3
"""Benchmark of the DAG-attention hot path on one MI355X.

One step = one pass of the whole hot path over one batch of seeded synthetic input:
  prefill segment (workload "llama3_8b_prefill_bf16", benchmark config 2):
      dag_build_meta -> dag_rope_qk -> dag_attn_prefill (as its two halves: prepare_v, attention)
  decode segment  (workload "branch_decode_bf16", benchmark config 3):
      dag_kv_append_rope -> dag_attn_decode (shared-prefix items + own items + LSE merge)
Inputs are resident in HBM before the timed region.  `value` is the prefill segment's useful
TFLOP/s (4*D*Hq*visible pairs / segment time); the decode segment is reported in "decode".
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
# HBM bytes per launch from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this file, scaled by
# what the same counters read for a plain 256 MiB copy (profiles/k_prefill_bf16__*.txt and
# profiles/k_decode__*.txt hold the commands and the raw readings); measured, not computed here.
TRAFFIC_PREFILL_KERNEL = (1237150 + 147528) * 1024      # k_prefill_bf16, read + written
TRAFFIC_DECODE_KERNELS = (1053639 + 10400 + 11819 + 1024) * 1024   # k_decode + k_decode_merge
# (profiles/k_decode_seg__*.txt and profiles/k_bwd__*.txt)
TRAFFIC_SEG_DECODE_KERNELS = (8 + 8 + 1058683 + 8322 + 9290 + 1024) * 1024   # k_seg_plan + k_decode_seg + k_decode_seg_merge
TRAFFIC_BWD_KERNELS = (294941 + 2304 + 769233 + 165872 + 2536551 + 73728 + 256 + 156) * 1024   # delta, dq, dkv, the three small ones


def _ensure_built():
    if not os.path.exists(B.LIB_PATH):
        from paper_2602_07529_amd import build
        build.build()


CLOCK_RAMP_STEPS = 40


class PrefillWork:
    def __init__(self, cfg, dev):
        self.cfg = cfg
        self.dag_list = dags.config_dags(cfg)
        self.T = int(sum(int(np.sum(L)) for L, _ in self.dag_list))
        hq, hkv, d = cfg["hq"], cfg["hkv"], cfg["d"]
        dtype = torch.float32 if cfg["dtype"] == "f32" else torch.bfloat16
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
    def __init__(self, cfg, dev):
        self.cfg = cfg
        st = dags.decode_state(cfg["seed"], cfg["n_seqs"], cfg["n_branch"], cfg["shared"], cfg["branch"],
                               cfg["hq"], cfg["hkv"], cfg["d"])
        self.desc_np = st["desc"]
        self.dd = B.DecodeDesc(st["desc"], dev)
        # two copies of the pools, used in turn, so that no step finds any of its 1 GiB of K/V in the
        # 256 MB last-level cache from the step before
        kp, vp = st["k_pool"].to(dev), st["v_pool"].to(dev)
        self.pools = [(kp, vp), (kp.clone(), vp.clone())]
        self.turn = 0
        self.q, self.k_new, self.v_new = st["q"].to(dev), st["k_new"].to(dev), st["v_new"].to(dev)
        self.out = torch.empty_like(self.q)
        self.ws = torch.empty(B.dag_decode_workspace_bytes(self.dd, cfg["hq"], cfg["hkv"], cfg["d"]),
                              dtype=torch.uint8, device=dev)
        self.bytes = dags.decode_algorithmic_bytes(st["desc"], cfg["hkv"], cfg["d"])
        self.n_live = st["desc"]["n_live"]

    def run(self, ev=None):
        kp, vp = self.pools[self.turn]
        self.turn ^= 1
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


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one plain 256 MiB device copy (untimed): under rocprofv3 --pmc its "
                         "FETCH_SIZE / WRITE_SIZE give the scale of those counters")
    args = ap.parse_args()
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
    pw = PrefillWork(dags.config(1), dev)
    dw = DecodeWork(dags.config(2), dev)

    if args.copy_calibration:
        src = torch.ones(256 << 20, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    pw.refresh_inputs()
    # From a cold start the GPU needs some tens of milliseconds of load to reach its sustained
    # clocks (the first ~20 steps run about 12 % slower than all later ones), so a fixed number of
    # untimed steps comes first, whatever --warmup says; then the W warm-up steps proper.
    for _ in range(CLOCK_RAMP_STEPS + args.warmup):
        pw.run()
        dw.run()
    new_events = lambda: [torch.cuda.Event(enable_timing=True) for _ in range(3)]
    pev = [new_events() for _ in range(args.steps)]
    dev_ev = [new_events() for _ in range(args.steps)]

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
    lse = torch.empty(pw.T, pw.cfg["hq"], dtype=torch.float32, device=dev)
    B.dag_attn_prefill(pw.meta, pw.q, pw.k, pw.v, pw.out, lse)
    dout = torch.randn(pw.q.shape, device=dev, generator=torch.Generator(device=dev).manual_seed(pw.cfg["seed"])).to(pw.q.dtype)
    dq, dk, dv = torch.empty_like(pw.q), torch.empty_like(pw.k), torch.empty_like(pw.v)
    bws = torch.empty(B.dag_prefill_bwd_workspace_bytes(pw.meta, pw.cfg["hq"], pw.cfg["hkv"], pw.cfg["d"]),
                      dtype=torch.uint8, device=dev)
    bwd = lambda: B.dag_attn_prefill_bwd(pw.meta, pw.q, pw.k, pw.v, pw.out, dout, lse, dq, dk, dv, workspace=bws)
    n_bwd = max(1, min(args.steps, 10))
    for _ in range(min(args.warmup, 3)):
        bwd()
    bev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    bev[0].record()
    for _ in range(n_bwd):
        bwd()
    bev[1].record()
    torch.cuda.synchronize()
    ms_bwd = bev[0].elapsed_time(bev[1]) / n_bwd

    flops, pairs = pw.useful_flops()
    mean = lambda xs: float(np.mean(xs))
    ms_step, ms_pre, ms_attn, ms_dec, ms_deck = map(mean, (step_ms, pre_ms, attn_ms, dec_ms, deck_ms))
    tflops_seg = flops / (ms_pre * 1e-3) / 1e12
    tflops_kernel = flops / (ms_attn * 1e-3) / 1e12
    dec_gbs = dw.bytes / (ms_deck * 1e-3) / 1e9
    cfg = pw.cfg
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
        "roofline": {"bound": "mfma", "kernel": "k_prefill_bf16", "achieved": tflops_kernel,
                     "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": tflops_kernel / MFMA_BF16_PEAK_TFLOPS,
                     "traffic": TRAFFIC_PREFILL_KERNEL, "algorithmic_bytes": pw.algorithmic_bytes()},
        "decode": {"metric": "branch_decode_tok_per_s_one_attention_layer",
                   "value": dw.n_live / (ms_dec * 1e-3), "unit": "tok/s", "ms_per_decode_step": ms_dec,
                   "config": {"workload": dw.cfg["name"], "n_seqs": dw.cfg["n_seqs"], "live_branches": dw.n_live,
                              "shared_prefix": dw.cfg["shared"], "branch_len": dw.cfg["branch"], "page_size": 16},
                   "roofline": {"bound": "hbm", "kernel": "k_decode(+k_decode_merge)", "achieved": dec_gbs,
                                "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": dec_gbs / HBM_PEAK_GBS,
                                "algorithmic_bytes": dw.bytes, "traffic": TRAFFIC_DECODE_KERNELS}},
        "decode_segments": {"metric": "segment_decode_tok_per_s_one_attention_layer",
                            "value": sw.n_live / (ms_seg * 1e-3), "unit": "tok/s", "ms_per_decode_step": ms_seg,
                            "config": {"workload": "three_level_frontier_bf16", "n_seqs": 16, "segments": sw.n_segments,
                                       "live_branches": sw.n_live, "levels": "root 4096 | 2 x 2048 | 8 x 1000..1063",
                                       "page_size": 16},
                            "roofline": {"bound": "hbm", "kernel": "k_seg_plan+k_decode_seg+k_decode_seg_merge",
                                         "achieved": seg_gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                                         "frac": seg_gbs / HBM_PEAK_GBS, "algorithmic_bytes": sw.bytes,
                                         "traffic": TRAFFIC_SEG_DECODE_KERNELS}},
        "prefill_bwd": {"metric": "dag_attn_prefill_bwd_useful_tflops", "value": 2.5 * flops / (ms_bwd * 1e-3) / 1e12,
                        "unit": "TFLOP/s", "ms_per_call": ms_bwd, "calls": n_bwd,
                        "useful_flops": "2.5 x forward (five products per visible pair)",
                        "roofline": {"bound": "mfma", "kernel": "k_bwd_delta+k_bwd_transpose+k_bwd_dq+k_bwd_dkv",
                                     "achieved": 2.5 * flops / (ms_bwd * 1e-3) / 1e12, "peak": MFMA_BF16_PEAK_TFLOPS,
                                     "unit": "TFLOP/s", "frac": 2.5 * flops / (ms_bwd * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS,
                                     "traffic": TRAFFIC_BWD_KERNELS}},
        "wall_s_timed_loop": wall,
    }
    if not args.no_cpu_baseline:
        res["cpu_baseline"] = cpu_baseline(pw)
    print(json.dumps(res))


if __name__ == "__main__":
    main()
