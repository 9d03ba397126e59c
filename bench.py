#!/usr/bin/env python3
"""Decode-step benchmark of libstc on one MI355X.

A step is one pass of the whole hot path over one layer's cache: Quest page
selection (stc_select_pages) followed by routed attention over the selected
pages (stc_decode_attention), for every stream of the batch.  Inputs are
synthetic, resident in HBM before the timed region; the step rotates over
several independent cache replicas and uses a fresh query every step so that
no step is served from the 256 MB last-level cache.

Prints ONE JSON line:
  value / ms_per_step  whole step, averaged over --steps back-to-back steps (HIP events)
  step_us_per_step_events  median / p10 / p90 of the same steps timed one by one
  hbm_GBps / hbm_frac  algorithmic bytes of the step / step time, against 8 TB/s
  calls                the same for stc_select_pages, stc_decode_attention and stc_score_pages
                       alone (each timed over --steps back-to-back launches)
  roofline             the dominant kernel (page scoring: it streams every page bound)
  cpu_baseline         the CPU oracle on a bounded sample of the same workload
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0          # MI355X published HBM3E peak
METRIC = "decode-attention us/step + achieved HBM GB/s (% of peak), Qwen2.5-7B 32K"

# replicas so that the bytes touched between two uses of a cache exceed ~2x the 256 MB
# last-level cache
REPLICAS = {"tiny": 8, "llama2_7b_4k": 4, "qwen25_7b_32k": 6, "llava15_7b_prefix": 4,
            "qwen25_7b_128k": 1}

# HBM bytes per launch of the dominant kernel from rocprofv3 --pmc runs of this file
# (FETCH_SIZE and WRITE_SIZE, scaled by what the same counters read for a copy of known
# size); see profiles/.  None where it has not been measured.
MEASURED_TRAFFIC = {("qwen25_7b_32k", "score_mfma_kernel"): 68624478,
                    ("llama2_7b_4k", "attn_mfma_kernel"): 111299921,
                    ("llava15_7b_prefix", "attn_mfma_kernel"): 175604796}


def algorithmic_bytes(w, mean_kept):
    """Bytes the method must move per decode step (one layer's cache)."""
    P, gd = 16, w.D // w.G
    k = min(w.k_pages, w.NP)
    selecting = w.k_pages < w.NP
    bounds = w.streams * w.NP * 2 * w.D * 2 if selecting else 0
    Kb = w.streams * k * P * w.D * 2
    Vb = w.streams * k * P * mean_kept * gd * 2
    meta = w.streams * k * P * 2 + 2 * w.streams * k * 4      # masks, page offsets, page indices
    score = bounds + (w.B * w.Hq * w.D * 2 + w.streams * w.NP * 4 if selecting else 0)
    return {"select": bounds + w.streams * k * 4, "attention": Kb + Vb + meta, "score": score,
            "step": bounds + Kb + Vb + meta,
            "parts": {"bounds": bounds, "K": Kb, "V": Vb, "meta": meta}}


def build_replicas(stc, W, w, n_rep, dev):
    import torch
    caches = []
    kept = 0
    for r in range(n_rep * w.layers):
        inp = W.make_cache_inputs(w, dev, layer=r)
        K, V, logits = inp["K"], inp["V"], inp["logits"]
        if w.routing == "vlm":
            n_src = w.n_visual + w.n_text
            Kc = torch.empty(w.B, w.Hkv, w.N, w.D, dtype=torch.bfloat16, device=dev)
            Vc = torch.empty_like(Kc)
            stc.stc_compact_tokens(K, inp["token_idx"], Kc, w.B, w.Hkv, n_src, w.N, w.D)
            stc.stc_compact_tokens(V, inp["token_idx"], Vc, w.B, w.Hkv, n_src, w.N, w.D)
            K, V = Kc, Vc
        c = stc.RoutedCache(w.B, w.Hq, w.Hkv, w.D, w.N, w.G, w.k_pages, device=dev,
                            keep_scores=False)
        c.build(K, V, logits=logits, kcount=inp["kcount"], mask_in=inp["mask_in"])
        torch.cuda.synchronize()
        assert int(c.dev_status.item()) == 0
        kept += int(c.tok_off[..., -1].to(torch.int64).sum().item())
        caches.append(c)
        del V, inp
    mean_kept = kept / float(len(caches) * w.streams * w.N)
    return caches, mean_kept


def timed(fn, n, torch):
    """Average milliseconds per call of fn(i) over n back-to-back calls, from HIP events
    recorded on the stream the kernels are launched on (torch's current stream)."""
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    a.record()
    for i in range(n):
        fn(i)
    b.record()
    torch.cuda.synchronize()
    return a.elapsed_time(b) / n


def per_step_times(fn, n, torch):
    """Microseconds of each of n steps, one HIP event pair per step (the event records add a
    little to every step, so these sit slightly above the back-to-back mean)."""
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(n + 1)]
    torch.cuda.synchronize()
    ev[0].record()
    for i in range(n):
        fn(i)
        ev[i + 1].record()
    torch.cuda.synchronize()
    return sorted(ev[i].elapsed_time(ev[i + 1]) * 1e3 for i in range(n))


def cpu_baseline(W, w, dev, budget_s=12.0):
    """The oracle, as it stands, on a bounded sample of streams of the same workload
    (per-step part only: page scores, selection, attention).  Single-threaded numpy."""
    import numpy as np

    from oracle import stc_oracle as O
    w1 = W.shrink(w, B=1)
    inp = W.make_cache_inputs(w1, dev, layer=0)                    # batch element 0 only
    q = W.bf16_bits(W.make_query(w1, 0, dev))
    R = w.R
    prepared = []
    for h in range(min(w.Hkv, 4)):                                 # oracle-built cache (untimed)
        K, V = W.bf16_bits(inp["K"][0, h]), W.bf16_bits(inp["V"][0, h])
        if w.routing == "vlm":
            ti = inp["token_idx"][0].cpu().numpy()
            K, V = K[ti], V[ti]
        if inp["mask_in"] is not None:
            m = W.u16_numpy(inp["mask_in"][0, h]) & np.uint16((1 << w.G) - 1)
        else:
            m = O.route_mask(inp["logits"][0, h].cpu().numpy(), inp["kcount"][0, h].cpu().numpy())
        prepared.append((K, V, m, O.page_bounds(K), q[0, h * R:(h + 1) * R]))
    t0 = time.perf_counter()
    done = 0
    while True:
        K, V, m, bounds, qh = prepared[done % len(prepared)]
        if w.k_pages < w.NP:
            idx = O.select_pages(O.page_scores(qh, bounds), w.k_pages)
        else:
            idx = np.arange(w.NP, dtype=np.int32)
        O.decode_attention(qh, K, V, m, idx, w.G)
        done += 1
        el = time.perf_counter() - t0
        if el > budget_s:
            break
    per_stream = el / done
    return {"value": per_stream * w.streams * w.layers * 1e6, "unit": "us/step", "cores": 1,
            "kind": "oracle",
            "sample": "%d stream-steps of %s (oracle page scores + selection + attention on "
                      "streams of batch element 0, %.1f s of CPU), scaled to the %d streams x %d "
                      "layer(s) of a step" % (done, w.name, el, w.streams, w.layers)}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=300)
    ap.add_argument("--warmup", type=int, default=200)
    ap.add_argument("--workload", default="qwen25_7b_32k")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run 5 plain 256 MiB device copies (a kernel of known traffic, "
                         "to scale rocprofv3's FETCH_SIZE / WRITE_SIZE readings)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no sharding or collectives); "
              "--gpus %d is not supported" % args.gpus, file=sys.stderr)
        sys.exit(2)

    import torch

    import paper_2604_21335_amd as stc
    from paper_2604_21335_amd import workloads as W

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    dev = "cuda:0"
    w = W.WORKLOADS[args.workload]
    n_rep = REPLICAS[w.name]
    caches, mean_kept = build_replicas(stc, W, w, n_rep, dev)
    nq = args.steps + args.warmup
    queries = [W.make_query(w, s, dev) for s in range(min(nq, 64))]
    L, C = w.layers, len(caches)
    selecting = w.k_pages < w.NP
    score_buf = (torch.empty(w.B, w.Hkv, w.NP, dtype=torch.float32, device=dev)
                 if selecting else None)

    def step(i):                       # one decode step = `layers` (select, attend) pairs
        qv = queries[i % len(queries)]
        for lay in range(L):
            caches[(i * L + lay) % C].step(qv)

    def step_two_calls(i):             # the same step through stc_select_pages + stc_decode_attention
        qv = queries[i % len(queries)]
        for lay in range(L):
            caches[(i * L + lay) % C].step(qv, one_call=False)

    def select_only(i):
        caches[i % C].select(queries[i % len(queries)])

    def attend_only(i):
        caches[i % C].attend(queries[i % len(queries)])

    def score_only(i):
        caches[i % C].score(queries[i % len(queries)], score_buf)

    if args.copy_calibration:
        # float16 so that the kernel's name (MulFunctor<c10::Half>) is unique in the trace
        src = torch.ones(128 << 20, dtype=torch.float16, device=dev)    # 256 MiB
        dst = torch.empty_like(src)
        for _ in range(5):                       # elementwise kernel: reads 256 MiB, writes 256 MiB
            torch.mul(src, 1.0, out=dst)
        torch.cuda.synchronize()
        del src, dst

    for i in range(args.warmup):
        step(i)
    ms_step = timed(step, args.steps, torch)
    ms_two = ms_step
    if selecting:
        for i in range(min(args.warmup, 50)):      # its kernels have not run yet
            step_two_calls(i)
        ms_two = timed(step_two_calls, args.steps, torch)
    ms_sel = timed(select_only, args.steps, torch) if selecting else 0.0
    ms_att = timed(attend_only, args.steps, torch)
    ms_score = timed(score_only, args.steps, torch) if selecting else 0.0
    per = per_step_times(step, args.steps, torch)
    pct = lambda f: per[min(len(per) - 1, int(f * len(per)))]  # noqa: E731

    ab = algorithmic_bytes(w, mean_kept)
    gbps = lambda nbytes, ms: (nbytes / (ms * 1e-3) / 1e9) if ms > 0 else 0.0  # noqa: E731

    def call(ms, nbytes):
        g = gbps(nbytes, ms)
        return {"us": ms * 1e3, "bytes": nbytes, "GBps": g, "frac": g / HBM_PEAK_GBPS}

    step_gbps = gbps(ab["step"] * L, ms_step)
    calls = {"select": call(ms_sel, ab["select"]), "attention": call(ms_att, ab["attention"]),
             "score": call(ms_score, ab["score"]),
             "step_as_two_calls": call(ms_two, ab["step"] * L)}
    # the dominant kernel is the one that moves the most bytes: page scoring where the bounds
    # outweigh the selected K pages and V runs (the headline workload), else the attention kernel
    if selecting and ab["score"] >= ab["attention"]:
        dom, kernel, entry = "score", "score_mfma_kernel", "stc_score_pages"
    else:
        dom, kernel, entry = "attention", "attn_mfma_kernel", "stc_decode_attention"
    roofline = {"bound": "hbm", "kernel": kernel, "entry_point": entry,
                "achieved": calls[dom]["GBps"], "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                "frac": calls[dom]["frac"], "traffic": MEASURED_TRAFFIC.get((w.name, kernel)),
                "algorithmic_bytes": calls[dom]["bytes"], "avg_us": calls[dom]["us"],
                "launches": args.steps}
    out = {
        "metric": METRIC, "value": ms_step * 1e3, "unit": "us/step", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_step,
        "higher_is_better": False, "scaling": "weak", "vs_baseline": None, "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": w.name, "B": w.B, "Hq": w.Hq, "Hkv": w.Hkv, "D": w.D, "N": w.N,
                   "page": 16, "k_pages": min(w.k_pages, w.NP), "G": w.G,
                   "mean_kept_groups": mean_kept, "layers_per_step": L, "cache_replicas": n_rep},
        "step_us_per_step_events": {"median": pct(0.5), "p10": pct(0.1), "p90": pct(0.9)},
        "hbm_GBps": step_gbps, "hbm_frac": step_gbps / HBM_PEAK_GBPS,
        "algorithmic_bytes_per_step": ab["step"] * L, "bytes_parts": ab["parts"],
        "calls": calls, "roofline": roofline,
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(W, w, dev)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
