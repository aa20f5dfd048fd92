#!/usr/bin/env python3
"""Benchmark of the PSD hot path on one MI355X.

A "step" is one whole decode of the workload: every block of every sequence run through
Alg. 1 (stage-1 forward + top-1 confidence, policy commit, draft build, batched
verification forward, hierarchical acceptance) by psd_decode_block, inputs and weights
resident in HBM.  Prints ONE JSON line: decoded tokens/s (whole job), tokens per forward
(TPF), the roofline figure of the dominant kernel measured live with HIP events, and the
CPU oracle timed on a bounded sample.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 3] [--logit-scale 1.0]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

MFMA_BF16_PEAK_TFLOPS = 2500.0     # MI355X dense bf16
HBM_PEAK_GBS = 8000.0

# HBM-side bytes per launch of the SwiGLU contraction at config 3, from two rocprofv3 --pmc runs (FETCH_SIZE,
# WRITE_SIZE) scaled by what the same counters read for a plain 256 MiB copy (factors 2.00 and 1.00); commands
# and tables in profiles/config3_hbm_traffic_pmc.md.  (fetched, written) MiB for the verification launch
# (2048 tokens, 768 workgroups) and the stage-1 launch (512 tokens, 192 workgroups) of the 256x256 tile.
SWIGLU_TRAFFIC_MIB = {"config": 3, "tile": "256x256, 8 wavefronts, LDS rings 2/3",
                      "verify": (584.2, 48.6), "stage1": (230.6, 12.0)}


def cpu_baseline(workload, stats_tokens, n_stage1, n_verify, threads_hint):
    """Times the oracle as it stands on a bounded sample: forward + confidence of one
    sequence at the workload's N on 1-layer and 2-layer cuts of the model (same widths and
    vocabulary).  Per-layer and per-call costs are extrapolated to the full depth and to
    the call counts of the measured decode (the oracle runs each sequence of a batched
    verification separately)."""
    import numpy as np
    import psd_inputs as inp
    from oracle import psd_oracle as orc
    shape, N, L = workload.shape, workload.seq_len, workload.block_len
    tokens = inp.initial_state(workload)[0]
    times = {}
    for nl in (1, 2):
        cut = inp.cut_down(shape, n_layers=nl)
        host = inp.draw_model(cut, N)
        t0 = time.perf_counter()
        orc.forward_confidence(host, tokens, workload.prompt_len, L)
        times[nl] = time.perf_counter() - t0
        del host
    per_layer = max(times[2] - times[1], 1e-9)
    rest = max(times[1] - per_layer, 0.0)
    t_seq = shape.n_layers * per_layer + rest
    total = (n_stage1 + n_verify * workload.n_drafts) * t_seq
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = threads_hint
    return {"value": stats_tokens / total, "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
            "sample": f"oracle forward+confidence of one {N}-token sequence on 1- and 2-layer cuts of the model "
                      f"({times[1]:.2f}s, {times[2]:.2f}s), extrapolated to {shape.n_layers} layers and to the "
                      f"{n_stage1} stage-1 + {n_verify}x{workload.n_drafts} verify sequence-forwards of one decode",
            "seconds_per_sequence_forward": t_seq}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--config", type=int, default=3, help="BASELINE configuration index (1-5)")
    ap.add_argument("--logit-scale", type=float, default=1.0)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-also", action="store_true",
                    help="skip the short extra measurement of config 2 (the small launch-latency-bound model) that a default run appends")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 256 MiB device copy (a known-size reference for scaling rocprofv3's "
                         "FETCH_SIZE / WRITE_SIZE counters)")
    ap.add_argument("--attention", choices=["bidirectional", "block-causal", "approx-cache"], default="bidirectional",
                    help="block-causal: the same shapes as a context-causal block model (App. A) decoded on the block rows "
                         "against an exact prefix KV cache (prefill included in the step); approx-cache: the bidirectional model "
                         "under the approximate prefix + suffix cache (one exact call per block, block rows otherwise; results "
                         "differ from the exact decode)")
    ap.add_argument("--max-blocks", type=int, default=0,
                    help="decode only the first blocks of the generation region (0 = all); tokens/s counts what was decoded")
    ap.add_argument("--calibrate-graph", action="store_true",
                    help="instead of the benchmark: decode the workload once per candidate draft graph (chains of depth 1-8, "
                         "wider steps, subset lattices) and print tokens/s and TPF of each, and the winner")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU only (no collectives, no sharding); run with --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import dataclasses
    import numpy as np
    import torch
    import psd_inputs as inp
    import paper_2605_15609_amd as psd
    from paper_2605_15609_amd.synthetic import synthetic_model

    if not os.path.exists(psd.library_path()):
        from paper_2605_15609_amd import build
        build.build()
    w = inp.WORKLOADS[args.config]
    if args.logit_scale != 1.0:
        w = dataclasses.replace(w, shape=dataclasses.replace(w.shape, logit_scale=args.logit_scale))
    approx = args.attention == "approx-cache"
    cached = args.attention == "block-causal"
    if cached:
        w = dataclasses.replace(w, shape=dataclasses.replace(w.shape, attention="block_causal"))
    shape = w.shape
    torch.cuda.set_device(0)
    t0 = time.perf_counter()
    model = synthetic_model(shape, w.seq_len, "cuda:0", threads=16)
    torch.cuda.synchronize()
    t_weights = time.perf_counter() - t0
    tokens0 = torch.from_numpy(inp.initial_state(w)).to("cuda:0")
    policy, graph = psd.Policy(w.tau, w.k_min, w.k_max), psd.chain_graph(w.n_drafts)

    if args.calibrate_graph:
        names = [f"chain K={k}" for k in range(1, 9)] + ["chain K=3 width=2", "chain K=4 width=2", "lattice depth=2",
                                                         "lattice depth=3"]
        cands = [psd.chain_graph(k) for k in range(1, 9)] + [psd.chain_graph(3, 2), psd.chain_graph(4, 2),
                                                             psd.lattice_graph(2), psd.lattice_graph(3)]
        if approx:
            sys.exit("bench.py: --calibrate-graph runs the exact decode or the block-causal cached one")
        kv = psd.KvCache(model, w.batch, w.seq_len) if cached else None
        psd.psd_calibrate_graph(model, tokens0, w.prompt_len, w.block_len, policy, cands[:1], kv)     # warm-up
        best, scores = psd.psd_calibrate_graph(model, tokens0, w.prompt_len, w.block_len, policy, cands, kv)
        print(json.dumps({"mode": "calibrate_graph", "config": {"workload": f"config {w.index}: {shape.name}, B={w.batch}, prompt {w.prompt_len}, {w.gen_len} generated, L={w.block_len}",
                                                                "attention": args.attention, "tau": w.tau},
                          "best": names[best],
                          "candidates": [{"graph": n, "K": g.K, "tokens_per_s": round(sc["tokens_per_s"], 2),
                                          "tpf": round(sc["tpf"], 4), "seconds": round(sc["seconds"], 4)}
                                         for n, g, sc in zip(names, cands, scores)]}))
        return

    n_blocks = w.gen_len // w.block_len
    if args.max_blocks > 0:
        n_blocks = min(n_blocks, args.max_blocks)
    gen_end = w.prompt_len + n_blocks * w.block_len

    cache = psd.KvCache(model, w.batch, w.seq_len) if cached else psd.KvCache(model, w.batch, w.seq_len - w.block_len) if approx else None
    prefill_ms = []

    def one_decode():
        toks = tokens0.clone()
        stats = [psd.Stats() for _ in range(w.batch)]
        if cached:
            cache.reset()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            psd.psd_kv_prefill(model, toks, w.prompt_len, w.block_len, cache)
            e1.record()
            prefill_ms.append((e0, e1))
        for block_start in range(w.prompt_len, gen_end, w.block_len):
            if cached:
                stats = psd.psd_decode_block_cached(model, toks, block_start, w.block_len, policy, graph, cache, stats)
            elif approx:
                stats = psd.psd_decode_block_approx(model, toks, block_start, w.block_len, policy, graph, cache, stats)
            else:
                stats = psd.psd_decode_block(model, toks, block_start, w.block_len, policy, graph, stats)
        return toks, stats

    for _ in range(args.warmup):
        one_decode()
    torch.cuda.synchronize()

    # dominant kernel: the SwiGLU gate/up contraction of the verification forward
    bf16 = shape.dtype == "bf16"
    lib = psd.load_library()
    if bf16:
        # the tile the dispatcher picks for the verification pass's SwiGLU contraction
        rows_per_seq = w.block_len if (cached or approx) else w.seq_len        # rows a model call runs over
        swiglu_tile = lib.psd_kernel_gemm_tile(w.batch * w.n_drafts * rows_per_seq, shape.d_ffn, 3)
        model.probe_begin(3, swiglu_tile)
        model.probe_begin(4, 0)
    t0 = time.perf_counter()
    for _ in range(args.steps):
        toks, stats = one_decode()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    roofline, lm_head = None, None
    if bf16:
        hms, hcalls, hbytes = model.probe_end(4)
        if hcalls > 0 and hms > 0:
            gbs = hbytes / (hms * 1e-3) / 1e9
            # rows per pass from the byte count (V d 2 + rows (d 2 + 8)); above the ridge (315 FLOP/B) the pass is MFMA work
            w_bytes = shape.vocab * shape.d_model * 2.0
            avg_rows = (hbytes / hcalls - w_bytes) / (shape.d_model * 2.0 + 8.0)
            lm_head = {"bound": "hbm", "achieved": gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": gbs / HBM_PEAK_GBS,
                       "calls": int(hcalls), "avg_pass_us": hms * 1e3 / hcalls, "bytes_per_pass": hbytes / hcalls,
                       "avg_rows": avg_rows,
                       "what": "LM-head confidence pass (final norm, weight stream, merge), stage-1 and verify calls together"}
            if avg_rows > 315:
                tfl = 2.0 * avg_rows * shape.vocab * shape.d_model * hcalls / (hms * 1e-3) / 1e12
                lm_head.update({"bound": "mfma", "achieved": tfl, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                                "frac": tfl / MFMA_BF16_PEAK_TFLOPS})
        ms, launches, flops = model.probe_end(3)
        if launches > 0 and ms > 0:
            achieved = flops / (ms * 1e-3) / 1e12
            roofline = {"bound": "mfma", "achieved": achieved, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                        "frac": achieved / MFMA_BF16_PEAK_TFLOPS, "traffic": None,
                        "kernel": f"mfma::gemm_bf16_kernel, SwiGLU gate/up contraction, tile {lib.psd_kernel_gemm_tile_name(swiglu_tile).decode()}", "launches": int(launches),
                        "avg_launch_us": ms * 1e3 / launches, "flops_per_launch": flops / launches}
            # rows per launch from the FLOP count (4 d F per row); below the ridge (315 FLOP/B) the launch is a
            # weight stream: algorithmic bytes = both weight matrices once + activations in + out
            rows_total = flops / (4.0 * shape.d_model * shape.d_ffn)
            by = launches * 2.0 * shape.d_ffn * shape.d_model * 2 + rows_total * (shape.d_model + shape.d_ffn) * 2
            if flops / by < 315:
                gbs = by / (ms * 1e-3) / 1e9
                roofline.update({"bound": "hbm", "achieved": gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": gbs / HBM_PEAK_GBS,
                                 "bytes_per_launch": by / launches, "tflops": achieved})

    if args.calibrate_copy:
        src = torch.ones(64 << 20, dtype=torch.float32, device="cuda:0")
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    if roofline is not None:
        # context for `frac`: what a loop of nothing but MFMAs sustains here on real (non-zero) operand data
        from paper_2605_15609_amd.binding import kernel_mfma_rate
        ops = (torch.randn(1 << 16, device="cuda:0") * 0.5).to(torch.bfloat16)
        roofline["mfma_only_loop_random_operands_tflops"] = kernel_mfma_rate(ops)
        roofline["mfma_only_loop_zero_operands_tflops"] = kernel_mfma_rate(torch.zeros_like(ops))

    assert not bool((toks[:, :gen_end] == shape.mask_id).any()), "decode left masked positions"
    n_tokens = w.batch * n_blocks * w.block_len
    invocations = sum(s.invocations for s in stats)
    n_verify = sum(sum(s.depth_hist) for s in stats)
    n_stage1 = invocations - n_verify
    if roofline is not None and w.index == SWIGLU_TRAFFIC_MIB["config"] and w.batch == 1 and \
            lib.psd_kernel_gemm_tile_name(swiglu_tile).decode() == SWIGLU_TRAFFIC_MIB["tile"]:
        # per launch, averaged over this decode's mix of verification and stage-1 launches like `achieved`
        v, s1 = sum(SWIGLU_TRAFFIC_MIB["verify"]), sum(SWIGLU_TRAFFIC_MIB["stage1"])
        roofline["traffic"] = (n_verify * v + n_stage1 * s1) / max(1, invocations) * 2 ** 20
        roofline["traffic_unit"] = "bytes per launch (rocprofv3 FETCH_SIZE + WRITE_SIZE, copy-calibrated; profiles/config3_hbm_traffic_pmc.md)"
        roofline["algorithmic_bytes_per_launch"] = ((n_verify * w.n_drafts + n_stage1) * w.seq_len * (shape.d_model + shape.d_ffn) * 2
                                                    / max(1, invocations) + 2 * shape.d_ffn * shape.d_model * 2)
    tpf = sum(s.tokens for s in stats) / max(1, invocations)
    value = args.steps * n_tokens / elapsed

    # whole-forward accounting for the verification pass (MFMA utilisation of the model call)
    # (per-sequence call counts: a stage-1 call is one sequence-forward, a verify call K of them)
    rows_call = w.block_len if (cached or approx) else w.seq_len
    work_v = psd.forward_work(model, w.n_drafts, rows_call, w.block_len)
    work_1 = psd.forward_work(model, 1, rows_call, w.block_len)
    total = lambda wk: wk["gemm_flops"] + wk["attn_flops"] + wk["head_flops"]
    flops_decode = n_stage1 * total(work_1) + n_verify * total(work_v)
    if approx:   # the call that enters a block runs over the whole sequence
        flops_decode += n_blocks * w.batch * (total(psd.forward_work(model, 1, w.seq_len, w.block_len)) - total(work_1))
    out = {
        "metric": "decoded tokens/s (PSD, tokens per forward in config.tpf)", "value": value, "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": elapsed / args.steps * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if bf16 else "f32", "data": "synthetic",
        "config": {"workload": f"config {w.index}: {shape.name}, B={w.batch}, prompt {w.prompt_len} Zipf tokens, "
                               f"{n_blocks * w.block_len} generated in blocks of {w.block_len}, K={w.n_drafts} chain, tau={w.tau}",
                   "tpf": tpf, "invocations": int(invocations), "stage1_calls": int(n_stage1),
                   "verify_calls": int(n_verify), "logit_scale": shape.logit_scale,
                   "tokens_policy": int(sum(s.tokens_policy for s in stats)),
                   "tokens_draft": int(sum(s.tokens_draft for s in stats)),
                   "tokens_postverify": int(sum(s.tokens_postverify for s in stats)),
                   "model_tflops_per_s_whole_decode": flops_decode / (elapsed / args.steps) / 1e12,
                   "weights_setup_s": t_weights, "attention": args.attention},
        "roofline": roofline,
        "lm_head_roofline": lm_head,
    }
    if cached:
        torch.cuda.synchronize()
        out["config"]["prefill_ms"] = float(np.mean([a.elapsed_time(b) for a, b in prefill_ms[-args.steps:]]))
        out["config"]["workload"] += ", context-causal block attention with prefix KV cache (prefill inside the step)"
    if approx:
        out["config"]["workload"] += (", approximate prefix + suffix KV cache (one exact whole-sequence call per block, block rows "
                                      "against frozen keys / values otherwise; results differ from the exact decode)")
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w, n_tokens, n_stage1, n_verify, os.cpu_count() or 1)
    else:
        out["cpu_baseline"] = None
    if args.config == 3 and not cached and not approx and not args.no_also and args.max_blocks == 0:
        # context: the small configuration (8 layers, d_model 512), whose model call is ~90 kernels of a few
        # microseconds each -- bound by kernel granularity, no roofline claim
        del model
        w2 = inp.WORKLOADS[2]
        m2 = synthetic_model(w2.shape, w2.seq_len, "cuda:0", threads=16)
        t2 = torch.from_numpy(inp.initial_state(w2)).to("cuda:0")
        pol2, g2 = psd.Policy(w2.tau, w2.k_min, w2.k_max), psd.chain_graph(w2.n_drafts)

        def decode2():
            toks = t2.clone()
            return psd.decode(m2, toks, w2.prompt_len, w2.block_len, pol2, g2)

        decode2()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        reps = 5
        for _ in range(reps):
            st2 = decode2()
        torch.cuda.synchronize()
        dt = (time.perf_counter() - t0) / reps
        out["also"] = {"config 2 (small-bf16, B=1, 128-token prompt, 256 generated, L=32, K=4)": {
            "tokens_per_s": w2.batch * w2.gen_len / dt, "ms_per_decode": dt * 1e3,
            "tpf": sum(s.tokens for s in st2) / max(1, sum(s.invocations for s in st2)),
            "invocations": int(sum(s.invocations for s in st2)), "bound": "kernel granularity (about 90 kernels of 3-14 us per model call, GPU 97 % busy)"}}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
