#!/usr/bin/env python3
"""Benchmark of the APB-V host-share hot path on one MI355X.

One "step" = one layer's hot path for one virtual host at the headline workload: apbv_compress_kv on the
local context block (batch 1) followed by apbv_host_attention over [anchor | passing | local(causal)].
Inputs are synthetic (seeded, Qwen2.5-VL-3B-shaped; see paper_2601_21444_amd/workloads.py) and resident
in HBM before the timed region.  The passing blocks that preceding hosts would send are produced, untimed,
by running the same compression kernel on their generated context blocks.

Prints ONE JSON line.  `value` is the useful attention FLOP rate of the whole step (visible (q,k)
pairs x 4d flops, divided by the wall time of compress + attention).  `roofline` describes the dominant
kernel (attention, bf16 MFMA bound) from HIP-event timings taken inside the timed region;
`roofline_compress` describes the score/select/gather pipeline at a batch whose working set exceeds the
256 MB last-level cache (HBM bound); `cpu_baseline` is the fp64 oracle timed on this machine's host cores on
a bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_MFMA_TFLOPS = 2500.0   # MI355X dense bf16 MFMA, published
PEAK_HBM_GBPS = 8000.0           # MI355X HBM3E, published



def measured_traffic(rel: str, library_version: int):
    """HBM traffic per launch (bytes) as measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (each scaled by the same
    counter's reading for a copy of known size).  The figure is not measured by this run: it is read from the committed
    summary `rel` (profiles/..._<workload>_pmc.txt), which ends with a line
        TRAFFIC_BYTES_PER_LAUNCH <bytes> library_version <v>
    and is reported only for the workload it was measured on and only while the library still has the version it
    was measured with; otherwise (None, None).  Returns (bytes, path relative to the repository)."""
    try:
        with open(os.path.join(ROOT, rel)) as f:
            lines = [ln.split() for ln in f if ln.startswith("TRAFFIC_BYTES_PER_LAUNCH")]
    except OSError:
        return None, None
    for w in lines:
        if len(w) >= 4 and w[2] == "library_version" and int(w[3]) == library_version:
            return int(w[1]), rel
    return None, None



def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default=None, help="workload name (default: the headline config)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-compress-roofline", action="store_true")
    ap.add_argument("--cpu-rows", type=int, default=6144, help="query rows the oracle is timed on")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also run one plain 1 GiB device copy (reference dispatch for scaling rocprofv3 FETCH_SIZE/WRITE_SIZE)")
    ap.add_argument("--no-extras", action="store_true", help="skip the short timings of the query-block, physical-host "
                    "and alternative-reduction entry points")
    ap.add_argument("--no-per-config", action="store_true", help="skip the short timings of the other configurations")
    ap.add_argument("--reducer-batch", type=int, default=0,
                    help="also time the whole compression call under each score reduction at this batch (0: skip)")
    ap.add_argument("--compress-batch", type=int, default=96,
                    help="batch of the HBM-bound compression measurement (working set far beyond the 256 MB cache)")
    return ap.parse_args()


def main():
    args = parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build covers one GPU (one virtual host's share); --gpus N with N > 1 is not "
              "supported -- the sequence-parallel exchange between hosts is outside the single-GPU hot path.",
              file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import paper_2601_21444_amd as apbv
    from paper_2601_21444_amd import workloads as wl

    apbv.load_library()
    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    torch.cuda.set_device(0)

    name = args.workload or wl.HEADLINE
    cfg = wl.CONFIGS[name]
    x = wl.generate(cfg)

    def dev(bits):
        return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).view(torch.bfloat16).cuda()

    q_probe, q, k_a, v_a, k, v = (dev(a) for a in (x.q_probe, x.q, x.k_anchor, x.v_anchor, x.k, x.v))
    scale = 1.0 / math.sqrt(cfg.head_dim)

    # Passing block = compressed blocks of the preceding hosts (what the all-gather would deliver).
    kps, vps = [], []
    for kb, vb in zip(x.k_prev, x.v_prev):
        _, a, b = apbv.apbv_compress_kv(q_probe, dev(kb), dev(vb), cfg.l_p)
        kps.append(a)
        vps.append(b)
    empty = torch.empty((0, cfg.n_kv_heads, cfg.head_dim), dtype=torch.bfloat16, device="cuda")
    k_p = torch.cat(kps) if kps else empty
    v_p = torch.cat(vps) if vps else empty
    torch.cuda.synchronize()

    # Pre-allocated outputs and workspace: nothing is allocated inside the timed region.
    ws = torch.empty(max(apbv.apbv_compress_workspace_bytes(1, cfg.n_kv_heads, cfg.head_dim, cfg.L, cfg.l_p), 256),
                     dtype=torch.uint8, device="cuda")
    idx = torch.empty((1, cfg.n_kv_heads, cfg.l_p), dtype=torch.int32, device="cuda")
    k_c = torch.empty((1, cfg.l_p, cfg.n_kv_heads, cfg.head_dim), dtype=torch.bfloat16, device="cuda")
    v_c = torch.empty_like(k_c)
    out = torch.empty((1, cfg.L, cfg.n_q_heads, cfg.head_dim), dtype=torch.bfloat16, device="cuda")

    def step(ev=None):
        if ev:
            ev[0].record()
        apbv.apbv_compress_kv(q_probe, k, v, cfg.l_p, workspace=ws, idx_out=idx, k_c_out=k_c, v_c_out=v_c)
        if ev:
            ev[1].record()
        apbv.apbv_host_attention(q, k_a, v_a, k_p, v_p, k, v, scale, out=out)
        if ev:
            ev[2].record()

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    events = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(events[i])
    torch.cuda.synchronize()
    t1 = time.perf_counter()

    ms_per_step = (t1 - t0) * 1e3 / args.steps
    comp_ms = sorted(e[0].elapsed_time(e[1]) for e in events)
    attn_ms = sorted(e[1].elapsed_time(e[2]) for e in events)
    attn_avg_ms = sum(attn_ms) / len(attn_ms)
    comp_avg_ms = sum(comp_ms) / len(comp_ms)
    flops = cfg.attention_flops
    attn_tflops = flops / (attn_avg_ms * 1e-3) / 1e12
    value = flops / (ms_per_step * 1e-3) / 1e12

    result = {
        "metric": "host-share attention TFLOP/s (% bf16 MFMA peak) + compress GB/s, ms/layer",
        "value": round(value, 2),
        "unit": "TFLOP/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {
            "workload": f"{name}: Hq {cfg.n_q_heads} / Hkv {cfg.n_kv_heads} / d {cfg.head_dim}, local {cfg.L}, anchor {cfg.l_a}, "
                        f"{cfg.P} passing blocks of top-{cfg.l_p}, probe n_q {cfg.n_q}, batch 1",
            "attention_flops": flops,
            "compress_bytes": cfg.compress_bytes,
        },
        "library_version": apbv.apbv_version(),
        "ms_per_layer": round(ms_per_step, 4),
        "attention": {"ms_avg": round(attn_avg_ms, 4), "ms_median": round(attn_ms[len(attn_ms) // 2], 4),
                      "ms_min": round(attn_ms[0], 4), "ms_max": round(attn_ms[-1], 4),
                      "tflops": round(attn_tflops, 2), "pct_bf16_mfma_peak": round(100 * attn_tflops / PEAK_BF16_MFMA_TFLOPS, 2)},
        "compress_batch1": {"us_avg": round(comp_avg_ms * 1e3, 2), "us_median": round(comp_ms[len(comp_ms) // 2] * 1e3, 2),
                            "us_min": round(comp_ms[0] * 1e3, 2),
                            "gbps": round(cfg.compress_bytes / (comp_avg_ms * 1e-3) / 1e9, 2)},
        "roofline": {"bound": "mfma", "kernel": "host_attention_kernel", "achieved": round(attn_tflops, 2),
                     "peak": PEAK_BF16_MFMA_TFLOPS, "unit": "TFLOP/s", "frac": round(attn_tflops / PEAK_BF16_MFMA_TFLOPS, 4),
                     "traffic": None, "traffic_source": None},
    }
    result["roofline"]["traffic"], result["roofline"]["traffic_source"] = measured_traffic(
        f"profiles/host_attention_{name}_pmc.txt", apbv.apbv_version())


    # The per-layer call again, free of the host: 20 calls captured in one HIP graph, replayed.  (The per-step
    # figures above are bracketed by one event pair per call and queued from Python; a serving loop would replay
    # the layer step from a graph.)
    result["compress_batch1"]["us_graph_replay"] = round(graph_replay_us(
        torch, lambda: apbv.apbv_compress_kv(q_probe, k, v, cfg.l_p, workspace=ws, idx_out=idx, k_c_out=k_c, v_c_out=v_c)), 2)

    # the two virtual hosts of a physical host as one batched call (Sec. 4.3)
    k2, v2, qp2 = (t.unsqueeze(0).repeat(2, 1, 1, 1) for t in (k, v, q_probe))
    ws2 = torch.empty(apbv.apbv_compress_workspace_bytes(2, cfg.n_kv_heads, cfg.head_dim, cfg.L, cfg.l_p), dtype=torch.uint8, device="cuda")
    idx2 = torch.empty((2, cfg.n_kv_heads, cfg.l_p), dtype=torch.int32, device="cuda")
    kc2 = torch.empty((2, cfg.l_p, cfg.n_kv_heads, cfg.head_dim), dtype=torch.bfloat16, device="cuda")
    vc2 = torch.empty_like(kc2)
    ms2 = timed(torch, lambda: apbv.apbv_compress_kv(qp2, k2, v2, cfg.l_p, workspace=ws2, idx_out=idx2, k_c_out=kc2, v_c_out=vc2),
                iters=20)
    result["compress_batch2"] = {"us_avg": round(ms2 * 1e3, 2), "gbps": round(2 * cfg.compress_bytes / (ms2 * 1e-3) / 1e9, 2)}
    del k2, v2, qp2

    if args.calibration_copy:
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        src.fill_(1)
        torch.cuda.synchronize()
        dst.copy_(src)          # one elementwise copy kernel: reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        del src, dst
    if not args.no_compress_roofline:
        result["roofline_compress"] = compress_roofline(apbv, torch, cfg, q_probe, k, v, args.compress_batch)
        rc = result["roofline_compress"]
        rc["traffic"], rc["traffic_source"] = measured_traffic(
            f"profiles/compress_{name}_batch{args.compress_batch}_pmc.txt", apbv.apbv_version())
    if not args.no_per_config:
        result["per_config"] = per_config(apbv, torch, np, wl, name, result)
    if not args.no_extras:
        result["extras"] = extras(apbv, torch, cfg, q_probe, q, k_a, v_a, k_p, v_p, k, v, scale)
    if args.reducer_batch > 0:
        result["reducers_batched"] = reducers_batched(apbv, torch, cfg, q_probe, k, v, scale, args.reducer_batch)
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(np, x, cfg, scale, args.cpu_rows)
    print(json.dumps(result), flush=True)


def timed(torch, fn, iters=10, warmup=3):
    """Average milliseconds per call of fn() on the current stream (HIP events)."""
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(iters):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / iters


def graph_replay_us(torch, fn, calls=20, replays=20):
    """Microseconds per call of fn() when `calls` of them are captured in one HIP graph and the graph is replayed."""
    g = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        fn()                                    # first call outside the capture (the library's one-time set-up)
        torch.cuda.synchronize()
        with torch.cuda.graph(g, stream=side):
            for _ in range(calls):
                fn()
    torch.cuda.synchronize()
    for _ in range(3):
        g.replay()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(replays):
        g.replay()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) * 1e3 / (calls * replays)


def per_config(apbv, torch, np, wl, headline, headline_result):
    """Every configuration of workloads.CONFIGS through the two calls of the hot path, a few launches each (context
    beside the headline fields; the headline's own entry repeats the figures of the timed steps)."""
    out = {}
    for name, cfg in wl.CONFIGS.items():
        if name == headline:
            a, c = headline_result["attention"], headline_result["compress_batch1"]
            out[name] = {"attention_ms": a["ms_avg"], "tflops": a["tflops"], "frac_bf16_mfma_peak": round(a["tflops"] / PEAK_BF16_MFMA_TFLOPS, 4),
                         "compress_us": c["us_avg"], "compress_us_graph_replay": c["us_graph_replay"]}
            continue
        x = wl.generate(cfg)

        def dev(bits):
            return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).view(torch.bfloat16).cuda()
        q_probe, q, k_a, v_a, k, v = (dev(a) for a in (x.q_probe, x.q, x.k_anchor, x.v_anchor, x.k, x.v))
        kps, vps = [], []
        for kb, vb in zip(x.k_prev, x.v_prev):
            _, a, b = apbv.apbv_compress_kv(q_probe, dev(kb), dev(vb), cfg.l_p)
            kps.append(a)
            vps.append(b)
        empty = torch.empty((0, cfg.n_kv_heads, cfg.head_dim), dtype=torch.bfloat16, device="cuda")
        k_p = torch.cat(kps) if kps else empty
        v_p = torch.cat(vps) if vps else empty
        ws = torch.empty(max(apbv.apbv_compress_workspace_bytes(1, cfg.n_kv_heads, cfg.head_dim, cfg.L, cfg.l_p), 256),
                         dtype=torch.uint8, device="cuda")
        idx = torch.empty((1, cfg.n_kv_heads, cfg.l_p), dtype=torch.int32, device="cuda")
        k_c = torch.empty((1, cfg.l_p, cfg.n_kv_heads, cfg.head_dim), dtype=torch.bfloat16, device="cuda")
        v_c = torch.empty_like(k_c)
        o = torch.empty((1, cfg.L, cfg.n_q_heads, cfg.head_dim), dtype=torch.bfloat16, device="cuda")
        scale = 1.0 / math.sqrt(cfg.head_dim)
        ms_a = timed(torch, lambda: apbv.apbv_host_attention(q, k_a, v_a, k_p, v_p, k, v, scale, out=o), iters=20, warmup=5)
        ms_c = timed(torch, lambda: apbv.apbv_compress_kv(q_probe, k, v, cfg.l_p, workspace=ws, idx_out=idx, k_c_out=k_c,
                                                          v_c_out=v_c), iters=50, warmup=5)
        us_g = graph_replay_us(torch, lambda: apbv.apbv_compress_kv(q_probe, k, v, cfg.l_p, workspace=ws, idx_out=idx,
                                                                    k_c_out=k_c, v_c_out=v_c))
        tf = cfg.attention_flops / (ms_a * 1e-3) / 1e12
        out[name] = {"attention_ms": round(ms_a, 4), "tflops": round(tf, 2),
                     "frac_bf16_mfma_peak": round(tf / PEAK_BF16_MFMA_TFLOPS, 4), "compress_us": round(ms_c * 1e3, 2),
                     "compress_us_graph_replay": round(us_g, 2)}
        del x, q_probe, q, k_a, v_a, k, v, k_p, v_p, kps, vps, o
    return out


def extras(apbv, torch, cfg, q_probe, q, k_a, v_a, k_p, v_p, k, v, scale):
    """Short timings of the entry points beyond the two-call hot path, at the same workload's shapes (context, not
    part of `value`): the query block's attention with and without the key split, a physical host's three attention
    problems in one launch and in three, and the alternative score reductions."""
    hq, hkv, d = cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim
    empty = torch.empty((0, hkv, d), dtype=torch.bfloat16, device="cuda")
    out = {}
    # query block of n_q tokens over this host's anchor + context block (Eq. 5), no causal segment
    n_keys = cfg.l_a + cfg.L
    q_out = torch.empty((1, cfg.n_q, hq, d), dtype=torch.bfloat16, device="cuda")
    nb = apbv.apbv_query_attention_workspace_bytes(1, hq, d, cfg.n_q, n_keys, 0)
    qws = torch.empty(max(nb, 256), dtype=torch.uint8, device="cuda")
    ms_split = timed(torch, lambda: apbv.apbv_query_attention(q_probe, k_a, v_a, k, v, empty, empty, scale, out=q_out,
                                                              workspace=qws))
    ms_plain = timed(torch, lambda: apbv.apbv_host_attention(q_probe, k_a, v_a, k, v, empty, empty, scale, out=q_out))
    out["query_attention"] = {"n_q": cfg.n_q, "keys": n_keys, "us_key_split": round(ms_split * 1e3, 1),
                              "us_unsplit": round(ms_plain * 1e3, 1)}
    # physical host 0 of 8: anchor block, virtual host 0 (no passing keys), virtual host 15 (15 passing blocks)
    def passing(n_blocks):
        reps = -(-n_blocks // max(cfg.P, 1))
        return (torch.cat([k_p] * reps)[: n_blocks * cfg.l_p].contiguous(), torch.cat([v_p] * reps)[: n_blocks * cfg.l_p].contiguous())
    if cfg.P > 0:
        kp15, vp15 = passing(15)
        qa = q[: cfg.l_a].contiguous()
        probs = [(qa, empty, empty, empty, empty, k_a, v_a),
                 (q, k_a, v_a, empty, empty, k, v),
                 (q, k_a, v_a, kp15, vp15, k, v)]
        outs = [torch.empty((p[0].shape[0], hq, d), dtype=torch.bfloat16, device="cuda") for p in probs]
        with_out = [p + (o,) for p, o in zip(probs, outs)]
        flops = sum(4.0 * hq * d * (p[0].shape[0] * (p[1].shape[0] + p[3].shape[0]) + p[0].shape[0] * (p[0].shape[0] + 1) / 2)
                    for p in probs)
        ms_group = timed(torch, lambda: apbv.apbv_host_attention_group(with_out, scale))

        def separate():
            for p, o in zip(probs, outs):
                apbv.apbv_host_attention(*p, scale, out=o)
        ms_sep = timed(torch, separate)
        out["physical_host"] = {"problems": "anchor 2048 causal; block with 0 passing keys; block with 15 x l_p passing keys",
                                "ms_one_launch": round(ms_group, 4), "ms_three_launches": round(ms_sep, 4),
                                "tflops_one_launch": round(flops / (ms_group * 1e-3) / 1e12, 1)}
    # alternative reductions of the score matrix, whole compression call at batch 1
    red = {}
    for name in ("sum", "max", "softmax_sum"):
        nbytes = apbv.apbv_compress_reduced_workspace_bytes(name, 1, hq, hkv, d, cfg.n_q, cfg.L, cfg.l_p)
        rws = torch.empty(max(nbytes, 256), dtype=torch.uint8, device="cuda")
        idx = torch.empty((1, hkv, cfg.l_p), dtype=torch.int32, device="cuda")
        k_c = torch.empty((1, cfg.l_p, hkv, d), dtype=torch.bfloat16, device="cuda")
        v_c = torch.empty_like(k_c)
        ms = timed(torch, lambda: apbv.apbv_compress_kv(q_probe, k, v, cfg.l_p, reducer=name, softmax_scale=scale,
                                                        workspace=rws, idx_out=idx, k_c_out=k_c, v_c_out=v_c), iters=20)
        red[name] = round(ms * 1e3, 1)
    out["compress_us_by_reducer"] = red
    return out


def reducers_batched(apbv, torch, cfg, q_probe, k, v, scale, batch):
    """The whole compression call under each reduction of the score matrix at a batch that fills the chip (the block
    repeated; timing only).  The matrix reductions form n_q*G x L logits per KV head on the matrix cores."""
    hq, hkv, d = cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim
    qp, kb, vb = (t.unsqueeze(0).repeat(batch, 1, 1, 1) for t in (q_probe, k, v))
    idx = torch.empty((batch, hkv, cfg.l_p), dtype=torch.int32, device="cuda")
    k_c = torch.empty((batch, cfg.l_p, hkv, d), dtype=torch.bfloat16, device="cuda")
    v_c = torch.empty_like(k_c)
    out = {"batch": batch, "logit_flops_per_call": 2.0 * batch * hq * cfg.n_q * cfg.L * d}
    for name in ("sum", "max", "softmax_sum"):
        nbytes = apbv.apbv_compress_reduced_workspace_bytes(name, batch, hq, hkv, d, cfg.n_q, cfg.L, cfg.l_p)
        rws = torch.empty(max(nbytes, 256), dtype=torch.uint8, device="cuda")
        ms = timed(torch, lambda: apbv.apbv_compress_kv(qp, kb, vb, cfg.l_p, reducer=name, softmax_scale=scale,
                                                        workspace=rws, idx_out=idx, k_c_out=k_c, v_c_out=v_c), iters=20, warmup=5)
        out[name + "_us"] = round(ms * 1e3, 1)
    return out


def compress_roofline(apbv, torch, cfg, q_probe, k, v, batch):
    """Compression at a batch whose rotating working set exceeds the 256 MB last-level cache, so the
    K stream really comes from HBM: two buffer sets of `batch` copies each, alternated."""
    sets = []
    for s in range(2):
        kb = k.unsqueeze(0).repeat(batch, 1, 1, 1)
        vb = v.unsqueeze(0).repeat(batch, 1, 1, 1)
        # decorrelate the copies a little so no two rows of the batch are the same cache lines
        kb = kb.roll(shifts=s + 1, dims=1).contiguous()
        sets.append((kb, vb))
    qp = q_probe.unsqueeze(0).repeat(batch, 1, 1, 1)
    ws = torch.empty(apbv.apbv_compress_workspace_bytes(batch, cfg.n_kv_heads, cfg.head_dim, cfg.L, cfg.l_p),
                     dtype=torch.uint8, device="cuda")
    idx = torch.empty((batch, cfg.n_kv_heads, cfg.l_p), dtype=torch.int32, device="cuda")
    k_c = torch.empty((batch, cfg.l_p, cfg.n_kv_heads, cfg.head_dim), dtype=torch.bfloat16, device="cuda")
    v_c = torch.empty_like(k_c)
    iters = 100
    for i in range(20):
        kb, vb = sets[i % 2]
        apbv.apbv_compress_kv(qp, kb, vb, cfg.l_p, workspace=ws, idx_out=idx, k_c_out=k_c, v_c_out=v_c)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for i in range(iters):
        kb, vb = sets[i % 2]
        apbv.apbv_compress_kv(qp, kb, vb, cfg.l_p, workspace=ws, idx_out=idx, k_c_out=k_c, v_c_out=v_c)
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / iters
    nbytes = cfg.compress_bytes * batch
    gbps = nbytes / (ms * 1e-3) / 1e9
    # the streaming pass on its own (l_p = 0: pooled query + scores, nothing selected or gathered); its
    # algorithmic bytes are the K block read once
    for i in range(10):
        apbv.apbv_compress_kv(qp, sets[i % 2][0], sets[i % 2][1], 0, workspace=ws)
    torch.cuda.synchronize()
    e0.record()
    for i in range(iters):
        kb, vb = sets[i % 2]
        apbv.apbv_compress_kv(qp, kb, vb, 0, workspace=ws)
    e1.record()
    torch.cuda.synchronize()
    ms_score = e0.elapsed_time(e1) / iters
    k_bytes = cfg.L * cfg.n_kv_heads * cfg.head_dim * 2 * batch
    gbps_score = k_bytes / (ms_score * 1e-3) / 1e9
    return {"bound": "hbm", "kernel": "pool+score+select+gather", "batch": batch, "achieved": round(gbps, 1),
            "peak": PEAK_HBM_GBPS, "unit": "GB/s", "frac": round(gbps / PEAK_HBM_GBPS, 4),
            "ms_per_call": round(ms, 4), "algorithmic_bytes_per_call": nbytes,
            "score_pass": {"kernel": "pool+score (l_p = 0)", "achieved": round(gbps_score, 1), "unit": "GB/s",
                           "frac": round(gbps_score / PEAK_HBM_GBPS, 4), "ms_per_call": round(ms_score, 4),
                           "algorithmic_bytes_per_call": k_bytes}}


def cpu_baseline(np, x, cfg, scale, n_rows):
    """The fp64 oracle as it stands, on this machine's host cores, on a bounded sample: the whole
    compression of the local block, and complete attention rows for an evenly spaced subset of query
    positions (all heads).  Reported as useful TFLOP/s on the same visible-pair FLOP count."""
    import oracle
    cores = len(os.sched_getaffinity(0))
    k_p, v_p = oracle.make_passing_block(x.q_probe, x.k_prev, x.v_prev, cfg.l_p, cfg.n_kv_heads, cfg.head_dim)
    t0 = time.perf_counter()
    oracle.compress_kv(x.q_probe, x.k, x.v, cfg.l_p)
    t_comp = time.perf_counter() - t0
    rows = np.linspace(0, cfg.L - 1, num=min(n_rows, cfg.L)).astype(np.int64)
    t0 = time.perf_counter()
    oracle.host_attention(x.q, x.k_anchor, x.v_anchor, k_p, v_p, x.k, x.v, scale, rows=rows, chunk=128)
    t_att = time.perf_counter() - t0
    n_vis = cfg.l_a + cfg.P * cfg.l_p
    pairs = int(np.sum(rows + 1 + n_vis))
    flops = 4 * cfg.head_dim * pairs * cfg.n_q_heads
    tflops = flops / t_att / 1e12
    return {"value": round(tflops, 5), "unit": "TFLOP/s", "cores": cores, "kind": "oracle",
            "sample": f"{len(rows)} evenly spaced query rows of {cfg.L} (all {cfg.n_q_heads} heads, full key rows) in "
                      f"{t_att:.2f} s; whole-block compress oracle {t_comp * 1e3:.1f} ms "
                      f"({cfg.compress_bytes / t_comp / 1e9:.3f} GB/s)",
            "attention_seconds_per_layer_extrapolated": round(cfg.attention_flops / (tflops * 1e12), 2),
            "compress_seconds_per_layer": round(t_comp, 4)}


if __name__ == "__main__":
    main()
