#!/usr/bin/env python3
"""Benchmark of the hot path on one MI355X.

A step = one pass of the whole hot path over one synthetic batch: `pie_forward` (one Llama-3-8B-shaped
decoder layer over 64 decode requests with prior contexts uniform in [512, 4096] against a 40k-page pool)
followed by `pie_get_next_dist` for the 64 output Embeds (vocab 128256, top-K 256).  Inputs are resident in
HBM before the timed region; the batch has been deserialised (`pie_batch_create`) beforehand.

Prints ONE JSON line: whole-step tokens/s, per-stage times, the roofline of the dominant forward kernel
(paged decode attention, HBM-bound) measured with HIP events on the library's stream, and the CPU oracle
timed on the host cores as a reported baseline.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)
sys.path.insert(0, os.path.join(ROOT, "tests"))

HBM_PEAK_GBS = 8000.0  # MI355X published HBM3E bandwidth
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X published dense bf16 matrix rate
MFMA_RIDGE_ROWS = 312  # rows above which a bf16 GEMM stops being bound by streaming its weights
# HBM bytes per launch of the decode-attention kernel from rocprofv3 counters (FETCH_SIZE scaled by the factor a
# once-streamed weight matrix of known size gives, plus WRITE_SIZE), taken in a profiling session of its own on
# exactly the default configuration (workload c2, 64 requests, one layer, no adapters): reported only when this run
# is that configuration, with the file that holds the counters named beside it; any other run reports null.
PMC_TRAFFIC = {"workload": "c2", "requests": 64, "layers": 1, "lora_rank": 0, "bytes": 527.5e6 + 5.1e6,
               "source": "profiles/c2_decode_pmc.md (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE passes over this command)"}


def mixed_workload_fractions(w_dec, args):
    """A short run of the mixed workload (configs[2]: 8 prefill requests of 1024 tokens + 128 decode requests through
    the same 8B-shaped layer, whose weights are reused) for the MFMA-bound kernels: the four tiled layer GEMMs and
    prefill attention as fractions of the dense bf16 matrix peak, from the library's per-stage HIP events."""
    import numpy as np
    import workloads as W
    from paper_2510_24051_amd import Pie
    w = W.c3_mixed(weights=w_dec.weights, head=w_dec.head, with_head=False)
    b, m = w.batch, w.model
    T = int(b.n_tokens)
    free_ids = np.setdiff1d(np.arange(w.n_embeds, dtype=np.int32), b.in_embed_ids)
    b.out_embed_ids = free_ids[:T].astype(np.int32)
    ctx = Pie(m, w.n_kv_pages, w.n_embeds, max_batch_tokens=T, max_batch_requests=b.n_requests, max_top_k=0,
              max_dist_rows=0)
    ctx.load_layer(0, w.weights)
    ctx.embed_write(b.in_embed_ids, w.embed_bits)
    ctx.kv_write(0, w.prior.page_ids, w.prior.slots, w.prior.k_bits, w.prior.v_bits)
    pb = ctx.batch_create(b, validate=True)
    for _ in range(3):
        ctx.forward(0, pb)
    ctx.synchronize()
    n = 10
    t0 = time.perf_counter()
    for _ in range(n):
        ctx.forward(0, pb)
    ctx.synchronize()
    fwd_ms = (time.perf_counter() - t0) * 1e3 / n
    ctx.set_stage_timing(True)
    acc = {}
    for _ in range(n):
        ctx.forward(0, pb)
        for k, v in ctx.stage_times().items():
            acc[k] = acc.get(k, 0.0) + v / n
    ctx.set_stage_timing(False)
    QD, KD, H, I = m.n_q_heads * m.head_dim, m.n_kv_heads * m.head_dim, m.hidden, m.mlp_dim
    shapes = {"qkv": H * (QD + 2 * KD), "oproj": QD * H, "gateup": 2 * H * I, "down": I * H}
    out = {"workload": "configs[2]: 8 prefill x 1024 (prior U[0,2048]) + 128 decode @2048, one 8B-shaped layer",
           "tokens": T, "forward_ms": round(fwd_ms, 4), "tokens_per_s": round(T / (fwd_ms * 1e-3), 1),
           "peak_TFLOPs": MFMA_BF16_PEAK_TFLOPS, "kernels": {}}
    tot_f, tot_ms = 0.0, 0.0
    for k, elems in shapes.items():
        fl, ms = 2.0 * T * elems, acc.get(k, 0.0)
        tot_f, tot_ms = tot_f + fl, tot_ms + ms
        if ms > 0:
            out["kernels"][k] = {"bound": "mfma", "flops": fl, "ms": round(ms, 4), "TFLOPs": round(fl / ms / 1e9, 1),
                                 "frac": round(fl / ms / 1e9 / MFMA_BF16_PEAK_TFLOPS, 4)}
    if tot_ms > 0:
        out["kernels"]["layer_gemms"] = {"bound": "mfma", "flops": tot_f, "ms": round(tot_ms, 4),
                                         "TFLOPs": round(tot_f / tot_ms / 1e9, 1),
                                         "frac": round(tot_f / tot_ms / 1e9 / MFMA_BF16_PEAK_TFLOPS, 4)}
    G = m.n_q_heads // m.n_kv_heads
    pf = 0
    for r in range(b.n_requests):
        nn = int(b.tok_indptr[r + 1] - b.tok_indptr[r])
        if nn * G > 16:  # prefill path; causal half only, skipped tiles are not counted
            pf += 4 * m.n_q_heads * m.head_dim * (nn * (int(b.kv_len[r]) - nn) + nn * (nn + 1) // 2)
    ms = acc.get("attn_prefill", 0.0)
    if ms > 0:
        out["kernels"]["attn_prefill"] = {"bound": "mfma", "flops": pf, "ms": round(ms, 4), "TFLOPs": round(pf / ms / 1e9, 1),
                                          "frac": round(pf / ms / 1e9 / MFMA_BF16_PEAK_TFLOPS, 4)}
    ms = acc.get("attn_decode", 0.0)
    if ms > 0:
        kvb = pb.work()["kv_bytes_decode"]
        out["kernels"]["attn_decode"] = {"bound": "hbm", "bytes": kvb, "ms": round(ms, 4), "GBs": round(kvb / ms / 1e6, 1),
                                         "frac": round(kvb / ms / 1e6 / HBM_PEAK_GBS, 4)}
    pb.destroy()
    ctx.close()
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="c2", choices=["c2", "c3", "c4", "c5"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-other-workloads", action="store_true",
                    help="default run only: skip the short run of the mixed workload c3 that adds the MFMA-bound kernels' "
                         "fractions of peak (other_workloads) to the line")
    ap.add_argument("--top-k", type=int, default=256)
    ap.add_argument("--requests", type=int, default=64, help="c2 only: number of decode requests (default: the config's 64)")
    ap.add_argument("--lora-rank", type=int, default=0,
                    help="give every request one of two synthetic LoRA adapters of this rank on q, k, v, o "
                         "(forward_with_adapter); 0 = plain forward")
    ap.add_argument("--layers", type=int, default=1,
                    help="run the batch through this many layers (pie_forward_all; every layer gets the same "
                         "synthetic weights and prior KV values); the default 1 is the per-layer metric")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import workloads as W
    from paper_2510_24051_amd import Pie

    t_setup = time.time()
    if args.workload == "c2":
        w = W.c2_decode(top_k=args.top_k, n_requests=args.requests)
        desc = (f"configs[1]: Llama-3-8B-shaped layer, {args.requests} decode requests, prior ctx U[512,4096], "
                "40k-page pool, page 16")
    elif args.workload == "c3":
        w = W.c3_mixed()
        desc = "configs[2]: 8B-shaped layer, 8 prefill x 1024 (prior U[0,2048]) + 128 decode @2048"
    elif args.workload == "c4":
        w = W.c4_prefix_tree(with_head=True)
        w.top_k = args.top_k
        w.dist_rows = np.arange(w.batch.n_tokens, dtype=np.int32)
        desc = "configs[3]: 8B-shaped layer, 256 branches sharing a 4096-token prefix, bitmap masks"
    else:
        w = W.c5_sparse_long()
        desc = "configs[4]: 70B-shaped layer, 16 requests @32768, sink(4)+window(4096) bitmaps"
    b = w.batch
    T = int(b.n_tokens)
    # distinct output Embeds so that every step does identical work on identical inputs
    free_ids = np.setdiff1d(np.arange(w.n_embeds, dtype=np.int32), b.in_embed_ids)
    b.out_embed_ids = free_ids[:T].astype(np.int32)
    dist_ids = b.out_embed_ids[w.dist_rows]
    n_dist = len(dist_ids)

    NL = max(1, args.layers)
    ctx = Pie(w.model, w.n_kv_pages, w.n_embeds, max_batch_tokens=T, max_batch_requests=b.n_requests,
              max_top_k=max(256, w.top_k), max_dist_rows=max(n_dist, 1), n_layers=NL,
              max_adapters=2 if args.lora_rank > 0 else 0, max_lora_rank=max(args.lora_rank, 0))
    if args.lora_rank > 0:
        for a in range(2):
            ctx.load_adapter(a, W.make_adapter(w.model, 2000, a, rank=args.lora_rank, n_layers=NL))
        b.adapter_ids = (np.arange(b.n_requests) % 2).astype(np.int32)
    ctx.load_head(w.head)
    ctx.embed_write(b.in_embed_ids, w.embed_bits)
    for l in range(NL):
        ctx.load_layer(l, w.weights)
        ctx.kv_write(l, w.prior.page_ids, w.prior.slots, w.prior.k_bits, w.prior.v_bits)
    pb = ctx.batch_create(b, validate=True)
    work = pb.work()
    out_ids = torch.empty((n_dist, w.top_k), dtype=torch.int32, device=ctx.device)
    out_probs = torch.empty((n_dist, w.top_k), dtype=torch.float32, device=ctx.device)
    torch.cuda.synchronize()
    print(f"# setup {time.time() - t_setup:.1f}s: {desc}; T={T} R={b.n_requests} "
          f"kv tokens={int(b.kv_len.sum())} visited pages={work['visited_pages']}", file=sys.stderr, flush=True)

    def fwd():
        if NL == 1:
            ctx.forward(0, pb)
        else:
            ctx.forward_all(pb)

    def step():
        fwd()
        ctx.get_next_dist_async(dist_ids, w.top_k, w.temperature, out_ids, out_probs)

    for _ in range(args.warmup):
        step()
    ctx.synchronize()
    torch.cuda.synchronize()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    with torch.cuda.stream(ctx.stream):
        ev0.record()
        for _ in range(args.steps):
            step()
        ev1.record()
    ctx.synchronize()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3 / args.steps
    ev_ms = ev0.elapsed_time(ev1) / args.steps
    ms_per_step = max(wall_ms, ev_ms)

    # forward only (the metric's "per layer" part), same method
    ctx.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        fwd()
    ctx.synchronize()
    fwd_ms = (time.perf_counter() - t0) * 1e3 / args.steps
    # the same calls one by one, each between two events on the library's stream: the median of single calls
    n_single = max(20, min(args.steps, 50))
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n_single)]
    with torch.cuda.stream(ctx.stream):
        for a, b_ in evs:
            a.record()
            fwd()
            b_.record()
    ctx.synchronize()
    fwd_median_ms = float(np.median([a.elapsed_time(b_) for a, b_ in evs]))
    # what a serving loop pays per step on top: deserialising the batch (host checks, work lists, one H2D copy)
    # and releasing it; never part of `value` (inputs resident, batch deserialised before the timed region)
    ctx.synchronize()
    t0 = time.perf_counter()
    n_host = 10
    for _ in range(n_host):
        pb2 = ctx.batch_create(b, validate=False)
        pb2.destroy()
    batch_create_ms = (time.perf_counter() - t0) * 1e3 / n_host

    # per-stage durations: HIP events recorded by the library on its own stream around every stage
    ctx.set_stage_timing(True)
    acc = {}
    n_prof = min(args.steps, 20)
    for _ in range(n_prof):
        ctx.forward(0, pb)  # the stages of one layer (layer 0) also when the step runs several
        ctx.get_next_dist_async(dist_ids, w.top_k, w.temperature, out_ids, out_probs)
        for k, v in ctx.stage_times().items():
            acc[k] = acc.get(k, 0.0) + v
    stages = {k: v / n_prof for k, v in acc.items() if v > 0}
    # Decode attention again with forward calls back to back, for comparison: a kernel that leaves many dirty
    # cache lines behind (get_next_dist once did) slows the next kernel that streams from HBM, and in a model of
    # several layers only the first layer follows get_next_dist.
    attn_b2b_ms = 0.0
    for _ in range(n_prof):
        ctx.forward(0, pb)
        attn_b2b_ms += ctx.stage_times().get("attn_decode", 0.0) / n_prof
    ctx.set_stage_timing(False)

    m = w.model
    kv_token_bytes = 2 * m.n_kv_heads * m.head_dim * 2
    # algorithmic HBM bytes of decode attention: every distinct visited page once (requests that share pages
    # do not multiply them); `logical` counts a page once per request that sees it, `requested` is what the
    # kernel asks the memory system for after grouping such requests
    shared = work["kv_bytes_unique"] != work["kv_bytes_decode"]
    if shared or b.mask_indptr is not None:
        attn_bytes = work["kv_bytes_unique"]  # pages with at least one visible key, each once
    else:  # inferred causal, nothing shared: every KV token of every decode-path request once
        G = m.n_q_heads // m.n_kv_heads
        attn_bytes = kv_token_bytes * sum(int(b.kv_len[r]) for r in range(b.n_requests)
                                          if (b.tok_indptr[r + 1] - b.tok_indptr[r]) * G <= 16)
    attn_ms = stages.get("attn_decode", 0.0)
    achieved = attn_bytes / (attn_ms * 1e-3) / 1e9 if attn_ms > 0 else 0.0
    roofline = {"kernel": "attn_decode_kernel", "bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": None, "traffic_source": None,
                "algorithmic_bytes": attn_bytes, "avg_ms": round(attn_ms, 5)}
    if (args.workload, args.requests, NL, args.lora_rank) == (PMC_TRAFFIC["workload"], PMC_TRAFFIC["requests"],
                                                               PMC_TRAFFIC["layers"], PMC_TRAFFIC["lora_rank"]):
        roofline["traffic"], roofline["traffic_source"] = PMC_TRAFFIC["bytes"], PMC_TRAFFIC["source"]
    if attn_b2b_ms > 0:
        roofline["forward_calls_back_to_back"] = {"avg_ms": round(attn_b2b_ms, 5),
                                                  "achieved": round(attn_bytes / (attn_b2b_ms * 1e-3) / 1e9, 1)}
    if shared and attn_ms > 0:
        roofline["shared_pages"] = {
            "logical_bytes": work["kv_bytes_decode"], "requested_bytes": work["kv_bytes_requested"],
            "requested_GBs": round(work["kv_bytes_requested"] / (attn_ms * 1e-3) / 1e9, 1),
            "note": "requests alias prefix pages: the kernel is bound by cache reads of the requested bytes, not by HBM"}

    weight_elems = (m.hidden * (m.n_q_heads + 2 * m.n_kv_heads) * m.head_dim + m.n_q_heads * m.head_dim * m.hidden
                    + 3 * m.hidden * m.mlp_dim)
    weight_bytes = 2 * weight_elems
    lm_bytes = 2 * m.vocab * m.hidden
    gemm_ms = sum(stages.get(k, 0.0) for k in ("qkv", "oproj", "gateup", "down"))
    extra = {
        "lm_head": {"bound": "hbm", "algorithmic_bytes": lm_bytes, "ms": round(stages.get("lm_head", 0.0), 5),
                    "achieved_GBs": round(lm_bytes / (stages["lm_head"] * 1e-3) / 1e9, 1) if stages.get("lm_head") else None},
    }
    if T < MFMA_RIDGE_ROWS:  # few rows: the GEMMs stream their weights once (HBM-bound)
        extra["layer_gemms"] = {"bound": "hbm", "algorithmic_bytes": weight_bytes, "ms": round(gemm_ms, 5),
                                "achieved_GBs": round(weight_bytes / (gemm_ms * 1e-3) / 1e9, 1) if gemm_ms else None}
    else:  # many rows: dense bf16 contractions (MFMA-bound)
        gemm_flops = 2 * T * weight_elems
        extra["layer_gemms"] = {"bound": "mfma", "algorithmic_flops": gemm_flops, "ms": round(gemm_ms, 5),
                                "achieved_TFLOPs": round(gemm_flops / (gemm_ms * 1e-3) / 1e12, 1),
                                "frac": round(gemm_flops / (gemm_ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4)}
        gu_flops, gu_ms = 2 * T * m.hidden * 2 * m.mlp_dim, stages.get("gateup", 0.0)
        if gu_ms > 0:
            # the dominant kernel of this workload is the gate/up contraction, not decode attention
            extra["decode_attention"] = roofline
            roofline = {"kernel": "gemm_large_async_kernel (gate/up + SwiGLU)", "bound": "mfma",
                        "achieved": round(gu_flops / (gu_ms * 1e-3) / 1e12, 1), "peak": MFMA_BF16_PEAK_TFLOPS,
                        "unit": "TFLOP/s", "frac": round(gu_flops / (gu_ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4),
                        "traffic": None, "algorithmic_flops": gu_flops, "avg_ms": round(gu_ms, 5)}
    pf_ms = stages.get("attn_prefill", 0.0)
    if pf_ms > 0:
        G = m.n_q_heads // m.n_kv_heads
        pf_flops = 0
        for r in range(b.n_requests):
            n = int(b.tok_indptr[r + 1] - b.tok_indptr[r])
            if n * G > 16:  # prefill path; causal half only, skipped tiles are not counted
                prior = int(b.kv_len[r]) - n
                pf_flops += 4 * m.n_q_heads * m.head_dim * (n * prior + n * (n + 1) // 2)
        extra["attn_prefill"] = {"bound": "mfma", "algorithmic_flops": pf_flops, "ms": round(pf_ms, 5),
                                 "achieved_TFLOPs": round(pf_flops / (pf_ms * 1e-3) / 1e12, 1),
                                 "frac": round(pf_flops / (pf_ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4)}

    other = None
    if args.workload == "c2" and args.requests == 64 and NL == 1 and args.lora_rank == 0 and not args.no_other_workloads:
        other = {"c3": mixed_workload_fractions(w, args)}

    cpu = None
    if not args.no_cpu_baseline:
        from oracle import pie_oracle as O
        from helpers import oracle_pools
        kv, emb = oracle_pools(w)
        # bounded sample: all rows when the batch is small, else the decode rows' worth of evenly spaced rows
        rows = None if T <= 512 else np.unique(np.linspace(0, T - 1, 64).astype(np.int64))
        n_rows = T if rows is None else len(rows)
        dist_sample = dist_ids if n_dist <= 64 else dist_ids[:: max(1, n_dist // 16)]
        tc = time.perf_counter()
        O.forward(w.model, w.weights, kv, emb, b, rows=rows)
        t_fwd = time.perf_counter() - tc
        tc = time.perf_counter()
        O.get_next_dist(w.model, w.head, emb, dist_sample, w.top_k, w.temperature)
        t_dist = time.perf_counter() - tc
        # scale each part to the whole step (the oracle's cost is linear in rows)
        cpu_s = NL * t_fwd * T / n_rows + t_dist * n_dist / max(len(dist_sample), 1)
        sample = (f"one layer over {n_rows} of {T} tokens ({t_fwd:.1f}s) + get_next_dist on {len(dist_sample)} of {n_dist} rows "
                  f"({t_dist:.1f}s), scaled to one whole step of {NL} layer(s); float64 NumPy")
        try:
            from threadpoolctl import threadpool_info
            cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
        except Exception:
            cores = os.cpu_count()
        cpu = {"value": round(T / cpu_s, 3), "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
               "sample": sample}

    line = {
        "metric": "forward tokens/s per layer (8B shape) + decode-attn HBM GB/s % of peak",
        "value": round(T / (ms_per_step * 1e-3), 1), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 5), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": desc, "tokens_per_step": T, "requests": int(b.n_requests), "dist_rows": n_dist,
                   "top_k": int(w.top_k), "layers": NL, "lora_rank": int(args.lora_rank),
                   "step": ("pie_forward (1 layer)" if NL == 1 else f"pie_forward_all ({NL} layers)") + " + pie_get_next_dist"},
        "forward_only": {"tokens_per_s": round(T / (fwd_ms * 1e-3), 1), "ms": round(fwd_ms, 5),
                         "median_ms_single_calls": round(fwd_median_ms, 5)},
        "host": {"batch_create_plus_destroy_ms": round(batch_create_ms, 4),
                 "step_including_batch_create_ms": round(ms_per_step + batch_create_ms, 4),
                 "note": "deserialising the batch is host work outside `value`; it can run while the GPU executes the previous step"},
        "stages_ms": {k: round(v, 5) for k, v in stages.items()},
        "roofline": roofline, "other_kernels": extra, "other_workloads": other, "cpu_baseline": cpu,
    }
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
