#!/usr/bin/env python3
"""Benchmark of the rollout decode step on one MI355X.

A "step" is one pass of the whole hot path (work list, embedding, every layer's norms, products,
RoPE + cache append, split-K attention and combine, LM head, argmax) over one batch of synthetic
sequences whose weights and KV cache are already resident in HBM.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload 7b-b128] [--breakdown]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0     # MI355X published HBM3E bandwidth


# HBM bytes per attention launch at workload 7b-b128 from rocprofv3 FETCH_SIZE / WRITE_SIZE runs scaled by a plain
# copy (profiles/attn_splitk_7b-b128_hbm_traffic.txt).  Valid only for the kernel source they were taken with.
PMC_TRAFFIC = {"workload": "7b-b128",
               "attention_hip_sha256": "11c5439d0fe03dfc65f9e7571695422881c8be675a5bff743dad012a6a914306",
               "fetch_bytes": 2165.63e6, "write_bytes": 9.45e6}


def measured_traffic(workload_name):
    import hashlib
    src = os.path.join(os.path.dirname(os.path.abspath(__file__)), "paper_2511_00796_amd", "csrc", "attention.hip")
    try:
        sha = hashlib.sha256(open(src, "rb").read()).hexdigest()
    except OSError:
        return None
    if sha != PMC_TRAFFIC["attention_hip_sha256"] or workload_name != PMC_TRAFFIC["workload"]:
        return None                      # the kernel changed since the counters were taken
    return PMC_TRAFFIC["fetch_bytes"] + PMC_TRAFFIC["write_bytes"]


def cpu_baseline(wl, dw_host, sample_rows, sample_layers, kv_fp8=False):
    """Time the CPU oracle, as it stands, on a bounded sample of the same workload: `sample_rows` sequences through
    `sample_layers` layers plus embedding and LM head.  Rows are independent and run one per core, so with all layers
    the figure is simply rows / seconds; with fewer layers the per-layer time is scaled to the full depth (and the
    sample text says so).  Returns the JSON object."""
    import dataclasses

    import numpy as np

    import oracle
    s = wl.shape
    rows = dw_host["rows"]
    sub = dataclasses.replace(s, n_layers=sample_layers)
    cfg = oracle.make_config(sub, kv_fp8=kv_fp8)
    w = oracle.Weights(dw_host["globals"], dw_host["layers"])
    ctx, table = dw_host["ctx"][rows], dw_host["table_rows"]
    kv = oracle.PagedKV(cfg, dw_host["num_blocks"])
    start = np.concatenate([[0], np.cumsum(ctx)]).astype(np.int32)
    for l in range(sample_layers):
        kv.fill(l, dw_host["k"][l], dw_host["v"][l], start, table)
    toks = dw_host["tokens"][rows]
    t0 = time.perf_counter()
    oracle.decode_step(cfg, w, kv, toks, ctx, ctx + 1, table)
    t_layers = time.perf_counter() - t0
    what = "%d of %d sequences (shortest, longest, seeded random)" % (len(rows), wl.batch)
    if sample_layers == s.n_layers:
        return {"value": len(rows) / t_layers, "unit": "tokens/s", "cores": oracle.num_threads(), "kind": "oracle",
                "sample": "%s through all %d layers, embedding and LM head: one whole oracle step of those rows, %.1f s of CPU "
                          "work; rows are independent, tokens/s = rows / seconds, nothing extrapolated"
                          % (what, s.n_layers, t_layers)}
    cfg0 = oracle.make_config(dataclasses.replace(s, n_layers=0))
    t0 = time.perf_counter()
    oracle.decode_step(cfg0, w, kv, toks, ctx, ctx + 1, table)
    t_head = time.perf_counter() - t0
    per_layer = max(t_layers - t_head, 0.0) / sample_layers
    full = per_layer * s.n_layers + t_head
    return {"value": len(rows) / full, "unit": "tokens/s", "cores": oracle.num_threads(), "kind": "oracle",
            "sample": "%s through %d of %d layers + embedding and LM head, %.1f s of CPU work; per-layer time scaled to %d layers"
                      % (what, sample_layers, s.n_layers, t_layers + t_head, s.n_layers)}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="7b-b128",
                    help="1.5b-b64, 1.5b-b256-longtail, 7b-b128 (default, the configuration the metric is quoted on) or "
                         "14b-b64; tiny-b4 fits the caches and is a parity case only")
    ap.add_argument("--batch", type=int, default=0, metavar="B",
                    help="override the workload's batch (same model shape and length law; reported as <workload>@bB): how "
                         "the kernels behave at other row counts, e.g. 4 rows = one m-group")
    ap.add_argument("--breakdown", action="store_true", help="extra untimed steps with every kernel class bracketed by events")
    ap.add_argument("--graph", action="store_true",
                    help="time replays of ONE HIP graph holding a whole step instead of eager launches (reported as such; the "
                         "dominant kernel is then timed in a separate eager pass)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-rows", type=int, default=16,
                    help="sequences the CPU baseline recomputes (default 16: one per host core of the GPU box, ~20 s of CPU work "
                         "at 7B; 128 = the whole batch, ~2 min)")
    ap.add_argument("--cpu-layers", type=int, default=0, help="layers of the CPU baseline (default 0 = all)")
    ap.add_argument("--sample", type=float, default=0.0, metavar="T",
                    help="time decode_step_sample at this temperature instead of the greedy step (reported as such)")
    ap.add_argument("--top-p", type=float, default=1.0, metavar="P",
                    help="with --sample: nucleus truncation (decode_step_top_p) at this mass")
    ap.add_argument("--prefill", type=int, default=0, metavar="P",
                    help="instead of decode steps, time prompt processing: 128 prompts of P tokens through prefill_chunk, "
                         "256 token rows per call (reported as prompt tokens/s)")
    ap.add_argument("--prefill-streams", type=int, default=1, choices=[1, 2, 4], metavar="S",
                    help="with --prefill: S engines over one copy of the packed weights, each with its own workspace, "
                         "cache and stream, processing different prompts concurrently")
    ap.add_argument("--prefill-rows-per-call", type=int, default=256, metavar="M",
                    help="with --prefill: rows per call; above 256 (a multiple of 256 that divides P) the calls go through "
                         "prefill_rows, whose products run over all rows of the call at once")
    ap.add_argument("--prefill-prompts", type=int, default=32, metavar="Q",
                    help="with --prefill-rows-per-call above 256: prompts per pass (32; fewer for counter runs)")
    ap.add_argument("--prefill-rows-per-seq", type=int, default=256, metavar="N",
                    help="with --prefill: consecutive positions of one prompt per call (256 = one prompt per call, "
                         "2 = all 128 prompts in every call)")
    ap.add_argument("--weight-swap", action="store_true",
                    help="instead of decode steps, time re-packing a whole policy version (hx_weights_pack of every tensor, "
                         "sources resident on the GPU) into the live engine")
    ap.add_argument("--kv-dtype", choices=["bf16", "fp8"], default="bf16",
                    help="element type of the KV cache: bf16 (the contract the headline metric is quoted on) or the "
                         "8-bit E4M3 variant (reported as such; its CPU baseline runs the oracle's 8-bit variant)")
    ap.add_argument("--copy-calibration", type=int, default=0, metavar="MiB",
                    help="run only a plain device copy of this size (5 launches): the known traffic against which "
                         "the FETCH_SIZE / WRITE_SIZE counters of a profiler run are scaled")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (the decode step has no cross-GPU path); "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    from paper_2511_00796_amd import binding, synth, workload

    if args.copy_calibration:
        n = args.copy_calibration << 20
        src = torch.empty(n, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration_bytes_read": n, "copy_calibration_bytes_written": n, "launches": 5}))
        return

    binding.load()
    if args.workload not in synth.WORKLOADS or synth.WORKLOADS[args.workload].kv_fill != "normal":
        print("bench.py: --workload must be one of %s (tiny-b4 is cache-resident: a parity case, not a bench line)"
              % ", ".join(n for n, w in synth.WORKLOADS.items() if w.kv_fill == "normal"), file=sys.stderr)
        sys.exit(2)
    wl = synth.WORKLOADS[args.workload]
    if args.batch:
        import dataclasses
        wl = dataclasses.replace(wl, batch=args.batch, name="%s@b%d" % (wl.name, args.batch))
    s = wl.shape
    ctx = synth.context_lengths(wl)
    if args.cpu_layers <= 0 or args.cpu_layers > s.n_layers:
        args.cpu_layers = s.n_layers

    # rows and layers the CPU baseline will recompute (copied to the host while the workload is built)
    host = None
    if not args.no_cpu_baseline:
        rows = {int(np.argmin(ctx)), int(np.argmax(ctx))}
        rng = np.random.default_rng(wl.seed)
        while len(rows) < min(args.cpu_rows, wl.batch):
            rows.add(int(rng.integers(0, wl.batch)))
        rows = np.array(sorted(rows))
        seq_start = np.concatenate([[0], np.cumsum(ctx)]).astype(np.int64)
        nblk = (ctx[rows].astype(np.int64) + 1 + 15) // 16
        width = int(nblk.max())
        table_rows = np.full((len(rows), width), -1, dtype=np.int32)
        at = 0
        for i, n in enumerate(nblk):
            table_rows[i, :n] = np.arange(at, at + n)
            at += int(n)
        host = {"rows": rows, "ctx": ctx, "layers": [], "k": [], "v": [], "table_rows": table_rows, "num_blocks": at,
                "tokens": synth.token_ids(wl, wl.batch)}

        def tap(kind, layer, t):
            if kind == "globals":
                host["globals"] = {k: synth.as_u16(v) for k, v in t.items()}
            elif layer < args.cpu_layers:
                if kind == "layer":
                    host["layers"].append({k: synth.as_u16(v) for k, v in t.items()})
                else:
                    for name in ("k", "v"):
                        host[name].append(np.concatenate(
                            [synth.as_u16(t[name][seq_start[r]: seq_start[r] + ctx[r]]) for r in rows]))
    else:
        tap = None

    if args.prefill:
        P, B, R = args.prefill, 128, 256
        kvd = binding.HX_KV_FP8_E4M3 if args.kv_dtype == "fp8" else binding.HX_KV_BF16
        eng = binding.Engine(s, R, P + 1, kv_dtype=kvd)
        for l in range(s.n_layers):
            eng.pack_layer(l, synth.layer_weights(s, l, wl.seed, device=torch.device("cuda")))
        eng.pack_globals(synth.global_weights(s, wl.seed, device=torch.device("cuda")))
        lens = np.full(B, P + 1, dtype=np.int32)
        table, nb = synth.block_table(lens, s.block_size, wl.seed)
        kvc = binding.KVCache(eng, nb)
        kvc.pool.zero_()
        n_streams = args.prefill_streams
        # further engines share the packed weights; each has its own workspace, cache and stream
        lanes = [(eng, kvc, torch.cuda.current_stream())]
        for _ in range(1, 1 if args.prefill_rows_per_call > 256 else n_streams):
            e2 = binding.Engine(s, R, P + 1, kv_dtype=kvd, weights=eng.weights)
            k2 = binding.KVCache(e2, nb)
            k2.pool.zero_()
            lanes.append((e2, k2, torch.cuda.Stream()))
        if args.prefill_rows_per_call > 256:
            # M consecutive positions of one prompt per call, through prefill_rows
            M = args.prefill_rows_per_call
            assert M % 256 == 0 and P % M == 0
            table_d = torch.from_numpy(table).cuda()
            toks = torch.randint(0, s.vocab, (M,), dtype=torch.int32, device="cuda")
            pos_of_call = [torch.arange(M, dtype=torch.int32, device="cuda") + c * M for c in range(P // M)]
            len_of_call = [p + 1 for p in pos_of_call]
            # calls on different streams share the engine (weights, layouts) and differ in workspace and cache
            wide_lanes = []
            for i in range(n_streams):
                kv_i = kvc if i == 0 else binding.KVCache(eng, nb)
                kv_i.pool.zero_()
                st_i = torch.cuda.current_stream() if i == 0 else torch.cuda.Stream()
                wide_lanes.append((kv_i, st_i, torch.empty(binding.prefill_workspace_bytes(eng.cfg, M), dtype=torch.uint8, device="cuda")))
            wide_ws = wide_lanes[0][2]
            n_seq = min(B, args.prefill_prompts)                  # 32 prompts are enough for a steady figure
            assert n_seq % n_streams == 0
            rows_of_seq = [table_d[g:g + 1].expand(M, -1).contiguous() for g in range(n_seq)]
            calls = n_seq * (P // M)
            torch.cuda.synchronize()

            def run_wide():
                for g in range(0, n_seq, n_streams):
                    for c in range(P // M):
                        for i, (kv_i, st_i, ws_i) in enumerate(wide_lanes):
                            with torch.cuda.stream(st_i):
                                eng.prefill_rows(kv_i, toks, pos_of_call[c], len_of_call[c], rows_of_seq[g + i], ws_i)

            run_wide()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            run_wide()
            torch.cuda.synchronize()
            dt = time.perf_counter() - t0
            eng.profile_enable(["gemm_gate_up"])
            for c in range(2):
                eng.prefill_rows(kvc, toks, pos_of_call[c % (P // M)], len_of_call[c % (P // M)], rows_of_seq[0], wide_ws)
            torch.cuda.synchronize()
            gu_ms, gu_n = eng.profile_read("gemm_gate_up")
            eng.profile_enable([])
            gu_avg_ms = gu_ms / max(gu_n, 1)
            gu_flops = 2.0 * M * s.hidden * 2 * s.intermediate
            call_flops = 2.0 * M * (s.weight_elements() - s.hidden * s.vocab)
            print(json.dumps({"metric": "prompt tokens/s through prefill_rows (rows = prompt tokens)",
                              "value": M * calls / dt, "unit": "tokens/s", "n_gpus": 1, "seconds": dt, "calls": calls,
                              "rows_per_call": M, "ms_per_call": dt / calls * 1e3,
                              "config": {"workload": "%s-prefill" % s.name, "prompts": n_seq, "prompt_len": P, "rows_per_call": M,
                                         "streams": n_streams, "kv_cache": "fp8-e4m3" if args.kv_dtype == "fp8" else "bf16"},
                              "data": "synthetic", "dtype": "bf16",
                              "product_flops_over_call_time_TFLOPs": call_flops / (dt / calls) / 1e12,
                              "roofline": {"kernel": "gemm_wide_kernel (gate|up product over all rows of the call)", "bound": "mfma",
                                           "achieved": gu_flops / (gu_avg_ms * 1e-3) / 1e12, "peak": 2500.0, "unit": "TFLOP/s",
                                           "frac": gu_flops / (gu_avg_ms * 1e-3) / 1e12 / 2500.0, "traffic": None,
                                           "launches_timed": int(gu_n), "avg_launch_ms": gu_avg_ms,
                                           "algorithmic_flops_per_launch": gu_flops}}))
            return
        per_seq = args.prefill_rows_per_seq                  # consecutive positions of each sequence per call
        assert R % per_seq == 0 and P % per_seq == 0 and B % (R // per_seq) == 0
        seqs_per_call = R // per_seq
        seq_of_row = torch.arange(R, device="cuda") // per_seq
        off_of_row = (torch.arange(R, device="cuda") % per_seq).to(torch.int32)
        table_d = torch.from_numpy(table).cuda()
        table_rows = [table_d[seq_of_row + g * seqs_per_call].contiguous() for g in range(B // seqs_per_call)]
        toks = torch.randint(0, s.vocab, (R,), dtype=torch.int32, device="cuda")
        calls = (B // seqs_per_call) * (P // per_seq)
        assert (B // seqs_per_call) % n_streams == 0

        pos_of_chunk = [off_of_row + c * per_seq for c in range(P // per_seq)]
        len_of_chunk = [p + 1 for p in pos_of_chunk]
        torch.cuda.synchronize()                              # the arguments exist before any stream reads them

        def run():
            for g in range(0, B // seqs_per_call, n_streams):   # a set of sequences at a time, each from position 0 to P
                for c in range(P // per_seq):
                    for i, (e_i, kv_i, st_i) in enumerate(lanes):
                        with torch.cuda.stream(st_i):
                            e_i.prefill_chunk(kv_i, toks, pos_of_chunk[c], len_of_chunk[c], table_rows[g + i])

        run()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        run()
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        # the kernel a call spends most time in: the gate|up product (HIP events around it, 8 calls)
        eng.profile_enable(["gemm_gate_up"])
        for c in range(8):
            cc = c % (P // per_seq)
            eng.prefill_chunk(kvc, toks, pos_of_chunk[cc], len_of_chunk[cc], table_rows[0])
        torch.cuda.synchronize()
        gu_ms, gu_n = eng.profile_read("gemm_gate_up")
        eng.profile_enable([])
        gu_avg_ms = gu_ms / max(gu_n, 1)
        gu_flops = 2.0 * R * s.hidden * 2 * s.intermediate
        call_flops = 2.0 * R * (s.weight_elements() - s.hidden * s.vocab)      # products of a call (no LM head)
        print(json.dumps({"metric": "prompt tokens/s through prefill_chunk (rows = prompt tokens)",
                          "value": R * calls / dt, "unit": "tokens/s", "n_gpus": 1, "seconds": dt, "calls": calls,
                          "rows_per_call": R, "ms_per_call": dt / calls * 1e3,
                          "config": {"workload": "%s-prefill" % s.name, "prompts": B, "prompt_len": P, "rows_per_sequence_per_call": per_seq,
                                     "streams": n_streams, "kv_cache": "fp8-e4m3" if args.kv_dtype == "fp8" else "bf16"},
                          "data": "synthetic",
                          "dtype": "bf16",
                          "product_flops_over_call_time_TFLOPs": call_flops / (dt / calls) / 1e12,
                          "roofline": {"kernel": "gemm_stream_kernel (gate|up product, 256 rows)", "bound": "mfma",
                                       "achieved": gu_flops / (gu_avg_ms * 1e-3) / 1e12, "peak": 2500.0, "unit": "TFLOP/s",
                                       "frac": gu_flops / (gu_avg_ms * 1e-3) / 1e12 / 2500.0, "traffic": None,
                                       "launches_timed": int(gu_n), "avg_launch_ms": gu_avg_ms,
                                       "algorithmic_flops_per_launch": gu_flops}}))
        return

    t_build = time.perf_counter()
    fp8 = args.kv_dtype == "fp8"
    dw = workload.build(wl, tap=tap, kv_dtype=binding.HX_KV_FP8_E4M3 if fp8 else binding.HX_KV_BF16)
    torch.cuda.synchronize()
    t_build = time.perf_counter() - t_build
    eng = dw.engine
    nbytes = dw.bytes()

    if args.weight_swap:
        # one layer's logical tensors serve as the source of every layer (the values do not matter for the timing)
        src_layer = synth.layer_weights(s, 0, wl.seed + 1, device=torch.device("cuda"))
        src_glob = synth.global_weights(s, wl.seed + 1, device=torch.device("cuda"))
        torch.cuda.synchronize()

        def swap():
            for l in range(s.n_layers):
                eng.pack_layer(l, src_layer)
            eng.pack_globals(src_glob)

        swap()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(3):
            swap()
        torch.cuda.synchronize()
        dt = (time.perf_counter() - t0) / 3
        wbytes = s.weight_elements() * 2
        print(json.dumps({"metric": "policy version swap: bf16 weights re-packed into the streaming layout", "value": wbytes / dt / 1e9,
                          "unit": "GB/s of weights", "n_gpus": 1, "seconds_per_swap": dt, "weights_bytes": wbytes,
                          "hbm_bytes_moved": 2 * wbytes, "decode_steps_equivalent": dt / 14.2e-3,
                          "config": {"workload": wl.name, "model_shape": s.name}, "data": "synthetic", "dtype": "bf16"}))
        return

    if args.sample > 0:
        s_tok = torch.zeros(wl.batch, dtype=torch.int32, device="cuda")
        s_lp = torch.zeros(wl.batch, dtype=torch.float32, device="cuda")

        def one_step():
            if args.top_p < 1.0:
                eng.decode_step_top_p(dw.kv, dw.tokens, dw.positions, dw.seq_lens_d, dw.table_d, args.sample, args.top_p,
                                      wl.seed, dw.logits, s_tok, s_lp)
            else:
                eng.decode_step_sample(dw.kv, dw.tokens, dw.positions, dw.seq_lens_d, dw.table_d, args.sample, wl.seed,
                                       dw.logits, s_tok, s_lp)
    else:
        one_step = dw.step

    for _ in range(args.warmup):
        one_step()
    torch.cuda.synchronize()
    # HIP events around the dominant kernel only, and around every 4th of its launches (layers 0, 4, 8, ...: the same
    # K/V lengths in every layer): a pair of events costs the stream ~5 us, 0.15 ms per step if all 28 were bracketed
    if args.graph:
        # one graph = one step; no events inside the capture, so the attention kernel is timed in an eager pass after
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            with torch.cuda.graph(graph, stream=side):
                one_step()
        torch.cuda.current_stream().wait_stream(side)
        for _ in range(args.warmup):
            graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            graph.replay()
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        eng.profile_enable(["attention"], every=4)
        for _ in range(args.steps):
            one_step()
        torch.cuda.synchronize()
    else:
        eng.profile_enable(["attention"], every=4)
        t0 = time.perf_counter()
        for _ in range(args.steps):
            one_step()
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
    attn_ms, attn_n = eng.profile_read("attention")
    eng.profile_enable([])

    # spread of single steps: a second pass with a pair of events per step (outside the timed region)
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
    marks[0].record()
    for i in range(args.steps):
        one_step()
        marks[i + 1].record()
    torch.cuda.synchronize()
    per_step = sorted(marks[i].elapsed_time(marks[i + 1]) for i in range(args.steps))

    ms_per_step = dt / args.steps * 1e3
    tokens_per_s = wl.batch / (dt / args.steps)
    kv_bytes_per_launch = nbytes["kv"] / s.n_layers
    attn_avg_ms = attn_ms / max(attn_n, 1)
    achieved = kv_bytes_per_launch / (attn_avg_ms * 1e-3) / 1e9

    out = {
        "metric": "decode tokens/s on 1 MI355X (7B, batch 128) + % of HBM peak GB/s",
        "value": tokens_per_s, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": wl.name, "model_shape": s.name, "batch": wl.batch, "kv_lengths": "%s[%d,%d]" % (wl.length_law, wl.lo, wl.hi),
                   "total_kv_tokens": int(dw.seq_lens.sum()), "block_size": s.block_size, "attention_waves": eng.attention_waves(), "launch": "hip graph replay" if args.graph else "eager",
                   "kv_cache": "fp8-e4m3" if fp8 else "bf16",
                   "token_choice": ("sample T=%g%s + logprob" % (args.sample, " top-p %g" % args.top_p if args.top_p < 1 else ""))
                   if args.sample > 0 else "greedy"},
        "step_hbm": {"algorithmic_bytes": nbytes["total"], "weights_bytes": nbytes["weights"], "kv_bytes": nbytes["kv"],
                     "achieved_GBps": nbytes["total"] / (dt / args.steps) / 1e9,
                     "frac_of_peak": nbytes["total"] / (dt / args.steps) / 1e9 / HBM_PEAK_GBS},
        "roofline": {"kernel": "attn_splitk_fp8_kernel" if fp8 else "attn_splitk_kernel", "bound": "hbm",
                     "achieved": achieved, "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS, "traffic": None if fp8 else measured_traffic(wl.name),
                     "traffic_unit": "bytes per launch",
                     "traffic_source": "rocprofv3 FETCH_SIZE + WRITE_SIZE of an earlier run of this kernel source, scaled by a "
                                       "plain copy: profiles/attn_splitk_7b-b128_hbm_traffic.txt (null once the source changed)",
                     "launches_timed": int(attn_n), "avg_launch_ms": attn_avg_ms,
                     "algorithmic_bytes_per_launch": kv_bytes_per_launch},
        "step_spread_ms": {"min": per_step[0], "median": per_step[len(per_step) // 2], "max": per_step[-1]},
        "setup_s": t_build,
    }

    if args.breakdown:
        eng.profile_enable(binding.KERNEL_CLASSES)
        for _ in range(3):
            one_step()
        torch.cuda.synchronize()
        bd = {}
        for k in binding.KERNEL_CLASSES:
            ms, n = eng.profile_read(k)
            bd[k] = {"ms_per_step": ms / 3, "launches_per_step": n // 3}
        eng.profile_enable([])
        out["breakdown"] = bd

    if host is not None:
        out["cpu_baseline"] = cpu_baseline(wl, host, args.cpu_rows, args.cpu_layers, kv_fp8=fp8)
        out["cpu_baseline"]["gpu_over_cpu"] = tokens_per_s / out["cpu_baseline"]["value"]
    print(json.dumps(out))


if __name__ == "__main__":
    main()
