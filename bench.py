#!/usr/bin/env python3
"""Benchmark of the LRSA hot path on one MI355X.

A step is one pass of the whole path -- scoring and selection (lrsa_score_select: both in one call; the
two separate calls with --separate-score-select), lrsa_attn_fwd, lrsa_attn_bwd -- over one synthetic batch
that is already resident in HBM.  The workload is the 32K-token GQA
config ("C4": B1, 32 query / 8 KV heads, d 128, n 32768, L 1024, K 256, S 64, bf16) unless
--workload says otherwise.  Prints ONE JSON line:

  value      effective TFLOP/s of attention forward+backward = 14*d*pairs*Hq*B / time of a
             whole step (score and select included in the time), pairs = visible (query, key)
             pairs per query head
  roofline   the kernel with the largest share of the step, its algorithmic flops per launch
             over its HIP-event duration, against the dense bf16 MFMA peak
  score_select  algorithmic bytes of scoring and selection over the time of a call, against the HBM peak
  cpu_baseline  the CPU oracle timed on a bounded sample of the same workload

K and V are rotated over several copies so that the scoring kernels read HBM-cold data.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

BF16_MFMA_PEAK_TFLOPS = 2500.0   # MI355X dense bf16
HBM_PEAK_GBPS = 8000.0


def pair_counts(w, local_prev=1):
    """(all visible pairs, pairs reached through the gather list) per query head, from the mask's
    closed form: a row of chunk q sees S + K*max(q-lp,0) gathered keys plus the window back to the
    start of chunk max(q-lp,0)."""
    import numpy as np
    t = np.arange(w.n, dtype=np.int64)
    q = (t - w.S) // w.L
    c = np.maximum(q - local_prev, 0)
    gathered = np.where(t < w.S, 0, w.S + w.K * c)
    window = np.where(t < w.S, t + 1, t - (w.S + w.L * c) + 1)
    return int((gathered + window).sum()), int(gathered.sum())


def cpu_baseline(w, x, chunks=24):
    """Time the oracle, as it stands, on a bounded sample: fp32 scores and selection of every head
    (NumPy), then the whole forward and backward (every query row: O, lse, D, dQ; every key column:
    dK, dV) of the first S + chunks*L tokens of ONE KV group in the fp64 C code with OpenMP.  The
    method is causal, so the prefix is the same problem at a shorter length."""
    from oracle import lrsa_ref as ref
    from oracle import lrsa_rows as rows
    Kf, Vf = x["K"].float().numpy(), x["V"].float().numpy()
    t0 = time.perf_counter()
    sc = ref.score(Kf, Vf, w.S, w.L)
    idx = ref.select(sc, w.S, w.L, w.K)
    t_sel = time.perf_counter() - t0
    G = w.G
    m = min(w.n, w.S + chunks * w.L)
    import dataclasses
    wp = dataclasses.replace(w, n=m)
    ns = max(-(-(m - w.S) // w.L) - 2, 0)
    Qg, dOg = x["Q"][0, :G, :m].float().numpy(), x["dO"][0, :G, :m].float().numpy()
    t0 = time.perf_counter()
    rows.attn_group(Qg, Kf[0, 0, :m], Vf[0, 0, :m], dOg, idx[0, 0, :ns], w.S, w.L, w.K)
    t_attn = time.perf_counter() - t0
    pairs, _ = pair_counts(wp)
    pairs_full, _ = pair_counts(w)
    flops = 14.0 * w.d * pairs * G
    threads = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
    t_full = t_attn * pairs_full / pairs * w.Hkv * w.B + t_sel
    return {"value": flops / t_attn / 1e12, "unit": "TFLOP/s", "cores": threads, "kind": "oracle",
            "sample": f"fp64 forward+backward of the first {m} tokens of KV group 0 of {w.Hkv * w.B} ({G} query heads, "
                      f"{pairs} visible pairs per head of {pairs_full}, {t_attn:.1f} s); fp32 score+select of all "
                      f"heads at full length took {t_sel:.2f} s",
            "attn_s": t_attn, "score_select_s": t_sel,
            "tokens_per_s_extrapolated": w.B * w.n / t_full}


def inference_bench(w, dev, batches=(1, 8), iters=50):
    """The inference-time cache at the history length of the workload (context only, not part of `value`):
    lrsa_decode_attn over the cache the last token of an n-token history sees (sink + K rows per compressed chunk +
    the uncompressed tail) and one lrsa_cache_compress step on a cache whose tail has just reached two chunks.
    Times are per-call sums of the kernels' HIP-event durations; GB/s = cache bytes the call must read / time."""
    import torch
    import paper_2506_11498_amd as lrsa
    nchunks = (w.n - w.S) // w.L                     # full chunks of the history
    done = max(nchunks - 1, 0)                       # the last full chunk is still the local window
    length = w.S + w.K * done + (w.n - w.S - done * w.L)
    cap = length + 2 * w.L
    out = {"history_tokens": w.n, "cache_rows": length, "compressed_chunks": done}
    esz = 2 if w.dtype == "bf16" else 4
    for B in batches:
        g = torch.Generator(device=dev).manual_seed(5)
        Kc = torch.randn((B, w.Hkv, cap, w.d), generator=g, device=dev).to(w.torch_dtype)
        Vc = torch.randn((B, w.Hkv, cap, w.d), generator=g, device=dev).to(w.torch_dtype)
        q = torch.randn((B, w.Hq, w.d), generator=g, device=dev).to(w.torch_dtype)
        p = lrsa.make_params((B, w.Hq, cap, w.d), tuple(Kc.shape), (w.Hq * cap * w.d, cap * w.d, w.d, 1), Kc.stride(),
                             dtype=w.torch_dtype, sink=w.S, lag=w.L, topk=w.K)
        O = torch.empty_like(q)
        lse = torch.empty((B, w.Hq), dtype=torch.float32, device=dev)
        ws = torch.empty(max(lrsa.workspace_bytes(p, 4), 256), dtype=torch.uint8, device=dev)
        full = w.S + w.K * done + 2 * w.L            # a tail of exactly two chunks: one compression step
        for timed in (False, True):
            if timed:
                torch.cuda.synchronize()
                lrsa.timing_enable(True)
            for _ in range(iters if timed else 5):
                lrsa.lrsa_decode_attn(p, q, Kc, Vc, length, O, lse, ws)
                lrsa.lrsa_cache_compress(p, Kc, Vc, None, full, done)
        torch.cuda.synchronize()
        per = {}
        for name, ms in lrsa.timing_records():
            per[name] = per.get(name, 0.0) + ms
        lrsa.timing_enable(False)
        attn_us = (per.get("k_decode_attn", 0.0) + per.get("k_decode_combine", 0.0)) * 1e3 / iters
        comp_us = per.get("k_cache_compress", 0.0) * 1e3 / iters
        attn_bytes = 2 * B * w.Hkv * length * w.d * esz
        comp_bytes = 2 * B * w.Hkv * (2 * w.L + (w.K + w.L)) * w.d * esz * 1   # two chunks read, survivors + tail moved
        out[f"B{B}"] = {"decode_attn_us": attn_us, "decode_attn_GBps": attn_bytes / attn_us / 1e3,
                        "decode_attn_frac_of_hbm_peak": attn_bytes / attn_us / 1e3 / HBM_PEAK_GBPS,
                        "cache_bytes": attn_bytes, "cache_compress_us": comp_us,
                        "cache_compress_GBps": comp_bytes / max(comp_us, 1e-9) / 1e3}
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="C4")
    ap.add_argument("--kv-copies", type=int, default=4, help="distinct K/V copies rotated over the steps")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--impl", choices=["auto", "compact"], default="auto",
                    help="compact: attention over a physically condensed KV cache (LRSA_IMPL_COMPACT)")
    ap.add_argument("--separate-score-select", action="store_true",
                    help="call lrsa_score and lrsa_select (two launches) instead of lrsa_score_select (one)")
    ap.add_argument("--no-inference", action="store_true",
                    help="skip the inference-time cache measurement (lrsa_decode_attn, lrsa_cache_compress)")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="after the timed steps, run one plain 1 GiB device copy (a kernel of known traffic "
                         "for scaling rocprofv3's FETCH_SIZE / WRITE_SIZE)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2506_11498_amd as lrsa

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    dev = "cuda:0"
    w = lrsa.inputs.WORKLOADS[args.workload]
    x = lrsa.inputs.make_inputs(w)
    Q, dO = x["Q"].to(dev), x["dO"].to(dev)
    Ks = [x["K"].to(dev) for _ in range(max(args.kv_copies, 1))]
    Vs = [x["V"].to(dev) for _ in range(max(args.kv_copies, 1))]
    p = lrsa.params_for(Q, Ks[0], sink=w.S, lag=w.L, topk=w.K,
                        impl=lrsa.IMPL_COMPACT if args.impl == "compact" else lrsa.IMPL_AUTO)
    Ns = lrsa.num_scored_chunks(p)
    score = torch.empty((w.B, w.Hkv, Ns, w.L), dtype=torch.float32, device=dev)
    idx = torch.empty((w.B, w.Hkv, Ns, w.K), dtype=torch.int32, device=dev)
    O, dQ = torch.empty_like(Q), torch.empty_like(Q)
    lse = torch.empty((w.B, w.Hq, w.n), dtype=torch.float32, device=dev)
    dK, dV = torch.empty_like(Ks[0]), torch.empty_like(Ks[0])
    ws_bytes = max(lrsa.workspace_bytes(p, k) for k in range(4))
    ws = torch.empty(max(ws_bytes, 256), dtype=torch.uint8, device=dev)

    def step(i):
        K, V = Ks[i % len(Ks)], Vs[i % len(Vs)]
        if args.separate_score_select:
            lrsa.lrsa_score(p, K, V, score, ws)
            lrsa.lrsa_select(p, score, idx, ws)
        else:
            lrsa.lrsa_score_select(p, K, V, score, idx, ws)
        lrsa.lrsa_attn_fwd(p, Q, K, V, idx, O, lse, ws)
        lrsa.lrsa_attn_bwd(p, Q, K, V, O, dO, lse, idx, dQ, dK, dV, ws)

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    lrsa.timing_enable(True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(args.warmup + i)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    recs = lrsa.timing_records()
    lrsa.timing_enable(False)

    ms_per_step = elapsed * 1e3 / args.steps
    per_kernel = {}
    for name, ms in recs:
        per_kernel.setdefault(name, []).append(ms)
    kern_ms = {k: sum(v) / len(v) for k, v in per_kernel.items()}           # average launch duration
    kern_med = {k: sorted(v)[len(v) // 2] for k, v in per_kernel.items()}
    kern_min = {k: min(v) for k, v in per_kernel.items()}
    launches = {k: len(v) / args.steps for k, v in per_kernel.items()}

    pairs, pairs_g = pair_counts(w)
    unit = w.d * w.Hq * w.B
    flops_step = 14.0 * unit * pairs
    # algorithmic flops per launch: forward 4*d per pair; backward 10*d per pair = S, dA, dV, dK
    # (8*d, in the key-outer kernels) + dQ (2*d, in the query-outer kernel)
    kern_flops = {"k_fwd_mfma": 4.0 * unit * pairs, "k_bwd_dq": 2.0 * unit * pairs, "k_bwd_dkv": 8.0 * unit * pairs}
    cand = [k for k in kern_flops if k in kern_ms]
    roofline = None
    if cand:
        dom = max(cand, key=lambda k: kern_ms[k] * launches[k])
        ach = kern_flops[dom] / (kern_ms[dom] * 1e-3) / 1e12
        traffic = None
        tpath = os.path.join(ROOT, "profiles", "traffic.json")
        if os.path.exists(tpath):
            traffic = json.load(open(tpath)).get(f"{dom}:{w.name}")
        counters = None      # MFMA-busy fraction, clock and CU occupancy from the committed rocprofv3 --pmc run
        cpath = os.path.join(ROOT, "profiles", "counters.json")
        if os.path.exists(cpath):
            counters = json.load(open(cpath)).get(f"{dom}:{w.name}")
        roofline = {"kernel": dom, "bound": "mfma", "achieved": ach, "peak": BF16_MFMA_PEAK_TFLOPS, "unit": "TFLOP/s",
                    "frac": ach / BF16_MFMA_PEAK_TFLOPS, "traffic": traffic, "counters": counters, "avg_launch_ms": kern_ms[dom],
                    "algorithmic_flop_per_launch": kern_flops[dom],
                    # achieved / frac / avg_launch_ms are measured by this run; traffic and counters are NOT:
                    # they are read from the committed rocprofv3 --pmc summaries of the same command
                    "traffic_source": "profiles/traffic.json (committed rocprofv3 --pmc runs, not this run)",
                    "counters_source": "profiles/counters.json (committed rocprofv3 --pmc runs, not this run)"}

    def stage(names):
        return sum(kern_ms.get(k, 0.0) * launches.get(k, 0.0) for k in names)
    esz = 2 if w.dtype == "bf16" else 4
    score_bytes = 2 * w.B * w.Hkv * w.n * w.d * esz + 4 * w.B * w.Hkv * Ns * w.L
    ms_score = stage(["k_score_select_fused", "k_score_fused", "k_score_resident", "k_softmax_select", "k_minmaxT", "k_sigmaT",
                      "k_softmax"])
    ms_select = stage(["k_select"])
    ms_fwd = stage(["k_fwd_mfma", "k_fwd_genericT"])      # k_compact_kv runs in both calls: counted below
    ms_bwd = stage(["k_bwd_dq", "k_bwd_dkv", "k_bwd_dkv_reduce", "k_bwd_dq_genericT", "k_bwd_dkv_genericT",
                    "k_compact_kv"])
    ss_bytes = score_bytes + 4 * w.B * w.Hkv * Ns * w.K     # K and V read once, scores and idx written once
    # Scoring and selection are a few short launches: an event pair around EACH of them (the per-kernel figures
    # above) adds about 5 us per launch, a large part of a 10-30 us kernel.  The stage's throughput is therefore
    # taken from a loop of its own: `ss_calls` calls back to back on the rotating K/V copies between ONE pair of
    # events on the launch stream, the launch gaps between the call's kernels included.
    ss_calls = 50
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    def score_stage(i):
        K, V = Ks[i % len(Ks)], Vs[i % len(Vs)]
        if args.separate_score_select:
            lrsa.lrsa_score(p, K, V, score, ws)
            lrsa.lrsa_select(p, score, idx, ws)
        else:
            lrsa.lrsa_score_select(p, K, V, score, idx, ws)

    for i in range(5):
        score_stage(i)
    torch.cuda.synchronize()
    ev0.record()
    for i in range(ss_calls):
        score_stage(i)
    ev1.record()
    torch.cuda.synchronize()
    ss_us = ev0.elapsed_time(ev1) * 1e3 / ss_calls
    ss_gbps = ss_bytes / max(ss_us, 1e-9) / 1e3
    out = {
        "metric": "lrsa_attn_fwd_bwd_effective_tflops_32k_bf16" if w.name == "C4" else f"lrsa_attn_fwd_bwd_effective_tflops_{w.name}",
        "value": flops_step / elapsed * args.steps / 1e12, "unit": "TFLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": f"{w.name}: B{w.B} Hq{w.Hq} Hkv{w.Hkv} d{w.d} n{w.n} L{w.L} K{w.K} S{w.S} {w.dtype}, {w.structure}",
                   "pairs_per_head": pairs, "kv_copies": len(Ks),
                   "impl": args.impl,
                   "score_select": "lrsa_score + lrsa_select" if args.separate_score_select else "lrsa_score_select (one call)"},
        "tokens_per_s": w.B * w.n / (ms_per_step * 1e-3),
        # context only: the flops of DENSE causal attention over the same step time (what sparse-attention
        # papers often quote); the graded figure is `value`, from the pairs the method really visits
        "dense_equivalent_tflops": 14.0 * unit * (w.n * (w.n + 1) // 2) / elapsed * args.steps / 1e12,
        "attn_fwd_bwd_tflops_kernels_only": flops_step / max((ms_fwd + ms_bwd) * 1e-3, 1e-12) / 1e12,
        "stages_ms": {"score": ms_score, "select": ms_select, "attn_fwd": ms_fwd, "attn_bwd": ms_bwd},
        "score_select": {"GBps": ss_gbps, "frac_of_hbm_peak": ss_gbps / HBM_PEAK_GBPS,
                         "algorithmic_bytes": ss_bytes, "us_per_call": ss_us,
                         "timing": f"{ss_calls} calls of the stage back to back between one pair of events",
                         "us_per_call_sum_of_per_kernel_events": (ms_score + ms_select) * 1e3},
        "kernels_ms": kern_ms, "kernels_ms_median": kern_med, "kernels_ms_min": kern_min,
        "roofline": roofline,
    }
    if args.calibration_copy:
        src = torch.empty(1 << 30, dtype=torch.uint8, device=dev).random_(0, 255)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()
    if not args.no_inference and w.L <= 4096:
        out["inference_cache"] = inference_bench(w, dev)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w, x)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
