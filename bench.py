#!/usr/bin/env python3
"""Benchmark of the stairs-assisted greedy generation hot path on one MI355X.

One "step" = one stairs decode of G tokens after an (untimed, separately reported) prefill of
the workload's prompt: draft k-step proposal, stair verification forward at M = k+1 rows,
per-row argmax, validation walk, KV rollback, repeated until G tokens exist.  Weights, KV
caches and the prompt are resident in HBM when the timed region starts.

Prints ONE JSON line: metric / value / unit (generated tokens per second of the decode phase at the best draft
length of a short sweep), the run's shape, "roofline" (the dominant kernel, the gate/up projection, against the HBM
peak: algorithmic bytes over its mean in-situ duration from HIP-event pairs, plus the isolated figure and the
measured counter traffic), "cpu_baseline" (the CPU oracle on a bounded sample of the same workload) and the extra
legs: verification time against k, adaptive draft length, sampling, several sequences, encoder-decoder pairs.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0           # MI355X published HBM3E peak
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "k_gemm_bf16_gateup_cfg4_7b_pmc.txt")


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def measured_traffic(kernel_key):
    """HBM bytes per launch of the dominant kernel from the committed rocprofv3 --pmc summary: lines
    'kernel: <name>', 'commit: <hash>', 'traffic_bytes_per_launch: N'.  None when the summary is missing or was taken
    on another kernel than the one this run times (the figure would silently be stale)."""
    fields = {}
    try:
        for line in open(TRAFFIC_FILE):
            if ":" in line:
                key, val = line.split(":", 1)
                fields.setdefault(key.strip(), val.strip())
    except OSError:
        return None, None
    if kernel_key not in fields.get("kernel", "") or "traffic_bytes_per_launch" not in fields:
        return None, None
    return float(fields["traffic_bytes_per_launch"]), fields.get("commit")


def cpu_baseline(w, target, draft, prompt, k, sample_P, sample_G):
    """The oracle's cached stairs loop, as it stands, on the host cores: same model pair, the
    first sample_P prompt tokens, sample_G generated tokens; timed after its prefill, like
    the GPU."""
    import numpy as np
    from oracle import stairs_oracle as so
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info() if p.get("user_api") == "blas"] or [1])
    except Exception:
        threads = os.cpu_count()
    T = so.OracleModel(target, np.float32, keep=True)
    D = so.OracleModel(draft, np.float32, keep=True) if k > 0 else None
    t0 = time.time()
    for m in [T] + ([D] if D is not None else []):          # decode the bf16 weights once (data loading)
        m.tok_emb(), m.lm_head(), m.final_norm()
        for l in range(m.n_layers):
            for name in m.inp.layers[l]:
                m.layer(l, name)
    t_load = time.time() - t0
    st = so.CachedStairs(T, D, prompt[:sample_P], sample_P + sample_G + k + 2)
    t1 = time.time()
    gen = st.run(sample_G, k)
    dt = time.time() - t1
    log(f"[cpu_baseline] weights decoded in {t_load:.1f}s, prefill {t1 - t0 - t_load:.1f}s, "
        f"{sample_G} tokens in {dt:.2f}s over {len(gen.iterations)} iterations")
    return {"value": sample_G / dt, "unit": "tokens/s", "cores": int(threads), "kind": "oracle",
            "sample": f"same model pair and k={k}; first {sample_P} prompt tokens, {sample_G} generated tokens, "
                      f"decode phase only (after the oracle's own cached prefill); numpy float32",
            "iterations": len(gen.iterations), "seconds": dt}


def encdec_leg(name):
    """Stairs with an encoder-decoder pair: source encoded once, G decoder tokens, plain greedy (k = 0) against
    every k of the workload; decode phase only (encoding reported beside it)."""
    import numpy as np
    import paper_2407_19947_amd as pkg
    import synth_inputs as si
    w = si.ENCDEC_WORKLOADS[name]
    target, draft = si.make_encdec_pair(w)
    src = si.make_source(w)
    G, ks = w["G"], w["ks"]
    out = {"source_len": len(src), "generate": G, "target": w["target"], "draft": w["draft"], "k_sweep": {}}
    with pkg.StairsEncDec(target, draft, k_max=max(ks), max_src=len(src), max_seq=G + max(ks) + 8,
                          start_token=si.DECODER_START) as eng:
        eng.generate(src, G, 0)                                   # warm-up (graph capture, first touch)
        base, st0 = eng.generate(src, G, 0)
        out["plain_greedy_tokens_per_s"] = G / (st0.ms_decode * 1e-3)
        out["encode_ms"] = st0.ms_prefill
        out["greedy_ms_per_token"] = st0.ms_decode / G
        out["decoder_weight_GBps_at_k0"] = target.decoder_bytes_streamed() / (st0.ms_decode / G * 1e-3) / 1e9
        best = None
        for k in ks:
            eng.generate(src, G, k)
            toks, st = eng.generate(src, G, k)
            assert np.array_equal(toks, base), "stairs changed the output of the encoder-decoder pair"
            tps = G / (st.ms_decode * 1e-3)
            out["k_sweep"][str(k)] = {"tokens_per_s": tps, "iterations": st.iterations,
                                      "mean_tokens_per_iteration": G / st.iterations,
                                      "ms_verify_per_iteration": st.ms_verify / st.iterations,
                                      "ms_draft_per_iteration": st.ms_draft / st.iterations}
            if best is None or tps > best[1]:
                best = (k, tps)
        out["best_k"], out["tokens_per_s"] = best
        out["time_reduction_vs_plain_greedy_pct"] = 100.0 * (1.0 - out["plain_greedy_tokens_per_s"] / best[1])
    log(f"[bench] encoder-decoder {name}: greedy {out['plain_greedy_tokens_per_s']:.0f} tok/s, stairs k={best[0]} "
        f"{best[1]:.0f} tok/s ({out['time_reduction_vs_plain_greedy_pct']:.1f} % less time), encode {out['encode_ms']:.1f} ms")
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--workload", default="cfg4_7b")
    ap.add_argument("--k", default="auto", help="draft length (stair rows = k+1); 'auto' = the best of a short sweep")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-sweep", action="store_true", help="skip the verify-vs-k sweep and the per-kernel table")
    ap.add_argument("--cpu-sample", default="64,96", help="prompt tokens, generated tokens of the CPU sample")
    ap.add_argument("--encdec", default="t5_large_shape,t5_3b_shape",
                    help="encoder-decoder workloads of the extra leg (comma separated, empty = none)")
    ap.add_argument("--only-encdec", action="store_true", help="run the encoder-decoder leg alone and print its results")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU only (no collectives, no sharding); use --gpus 1")

    import numpy as np
    import torch
    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    torch.cuda.set_device(0)
    if args.only_encdec:
        print(json.dumps({"encoder_decoder": {name: encdec_leg(name) for name in args.encdec.split(",") if name}}), flush=True)
        return
    import paper_2407_19947_amd as pkg
    import synth_inputs as si

    w = si.WORKLOADS[args.workload]
    P, G = w["P"], w["G"]
    t0 = time.time()
    target, draft = si.make_pair(w, threads=min(16, os.cpu_count() or 8))
    prompt = si.make_prompt(w)
    log(f"[bench] {args.workload}: weights drawn in {time.time() - t0:.1f}s "
        f"(target {target.n_params() / 1e9:.2f}B, draft {draft.n_params() / 1e9:.2f}B params)")
    k_max = 16
    t0 = time.time()
    eng = pkg.Stairs(target, draft, k_max=k_max, max_seq=P + G + k_max + 8)
    log(f"[bench] context built in {time.time() - t0:.1f}s")

    # draft length: the workload sweeps k; the headline is quoted at the k that generates fastest here
    k_table = {}
    if args.k == "auto":
        for kk in (1, 2, 3, 4, 6, 8):
            eng.prefill(prompt)
            t1 = time.perf_counter()
            _, st = eng.decode(G, kk)
            k_table[str(kk)] = {"tokens_per_s": G / (time.perf_counter() - t1), "iterations": st.iterations}
        k = int(max(k_table, key=lambda q: k_table[q]["tokens_per_s"]))
        log(f"[bench] k sweep: " + ", ".join(f"k={q}: {v['tokens_per_s']:.0f} tok/s" for q, v in k_table.items()) + f" -> k={k}")
    else:
        k = int(args.k)
    decode_s, prefill_ms, stats_last, toks0 = [], [], None, None
    for step in range(args.warmup + args.steps):
        eng.prefill(prompt)
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        toks, st = eng.decode(G, k)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t1
        if toks0 is None:
            toks0 = toks.copy()
        assert np.array_equal(toks, toks0), "generation is not reproducible"
        if step >= args.warmup:
            decode_s.append(dt)
            stats_last = st
        log(f"[bench] step {step}: decode {dt * 1e3:.1f} ms ({G / dt:.1f} tok/s), iterations {st.iterations}, "
            f"accepted {st.accepted}, draft {st.ms_draft:.1f} ms, verify {st.ms_verify:.1f} ms")
    total = sum(decode_s)
    value = G * len(decode_s) / total
    per_step = sorted(G / t for t in decode_s)
    spread = {"median": per_step[len(per_step) // 2], "min": per_step[0], "max": per_step[-1]}
    # prefill, once, timed through generate()
    _, stg = eng.generate(prompt, 1, 0)
    prefill_ms = stg.ms_prefill

    # plain greedy on the same GPU (the paper's "original" comparator), one step
    eng.prefill(prompt)
    t1 = time.perf_counter()
    toks_plain, st_plain = eng.decode(G, 0)
    plain_s = time.perf_counter() - t1
    assert np.array_equal(toks_plain, toks0), "stairs output differs from plain greedy"

    # ---- roofline of the dominant kernel: gate/up projection GEMM at M = k+1 rows ----------
    # in situ: whole verification forwards at the decode's context length, every layer's gate/up launch recording its
    # own start and end events (the HIP events of the launch itself: nothing is added to the stream, and the figure
    # agrees with what rocprofv3 reports for the same launches); also the reading of an event pair recorded around
    # the launch (which contains the pair's own cost) and of an empty pair;
    # isolated: the same kernel launched back to back, cycling through the layers' matrices
    M = k + 1
    ctx_mid = P + G // 2
    ms_situ, bytes_gu = eng.time_kernel(10, M, ctx_mid, 4)
    ms_around, _ = eng.time_kernel(8, M, ctx_mid, 4)
    ms_pair, _ = eng.time_kernel(9, M, ctx_mid, 4)      # what an event pair reads with no kernel inside
    ms_iso, _ = eng.time_kernel(0, M, 0, 4 * target.n_layers)
    achieved = bytes_gu / (ms_situ * 1e-3) / 1e9
    kernel_key = f"k_gemm_bf16_rows<{M}, gate/up" if M <= 7 else f"k_gemm_bf16_wide<{(M + 15) // 16},"
    kname = (f"k_gemm_bf16_rows<{M}, gate/up> (whole activation block in LDS, a work-group walks its share of the weight tiles)"
             if M <= 7 else
             f"k_gemm_bf16_wide<{(M + 15) // 16}, NT> (activation fragments from L2, a wave owns NT weight tiles over its share of k)")
    # the committed counter summary is of the default workload's kernel: no figure for another workload or row count
    traffic, traffic_commit = measured_traffic(kernel_key) if args.workload == "cfg4_7b" else (None, None)
    roofline = {"bound": "hbm", "kernel": kname + ": gate/up projection + SwiGLU at M = k+1 rows",
                "achieved": achieved, "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBPS,
                "traffic": traffic, "traffic_source": (f"profiles/{os.path.basename(TRAFFIC_FILE)} at commit {traffic_commit}"
                                                       if traffic is not None else None),
                "bytes_per_launch": bytes_gu, "ms_per_launch": ms_situ,
                "launches_timed": 4 * target.n_layers,
                "how": "in situ: start/end HIP events of each layer's launch inside whole verification forwards",
                "event_pair_around_launch_ms": ms_around, "empty_event_pair_ms": ms_pair,
                "event_pair_around_launch_frac": bytes_gu / (ms_around * 1e-3) / 1e9 / HBM_PEAK_GBPS,
                "isolated_ms_per_launch": ms_iso, "isolated_GBps": bytes_gu / (ms_iso * 1e-3) / 1e9,
                "isolated_frac": bytes_gu / (ms_iso * 1e-3) / 1e9 / HBM_PEAK_GBPS}
    # second denominator: what a plain copy kernel (1 GiB read + 1 GiB written) streams on this machine
    copy_bytes = 1 << 30
    ms_copy = pkg.stairs_copy_probe(copy_bytes, 4)
    copy_gbps = 2 * copy_bytes / (ms_copy * 1e-3) / 1e9
    roofline["measured_stream_GBps"] = copy_gbps
    roofline["frac_of_measured_stream"] = achieved / copy_gbps
    extras = {"copy_probe_GBps": copy_gbps}

    if not args.no_sweep:
        names = {0: "gemm_gate_up", 1: "gemm_qkv", 2: "gemm_wo", 3: "gemm_down", 4: "gemm_lm_head", 5: "attention"}
        per_kernel = {}
        for which, name in names.items():
            ms, by = eng.time_kernel(which, M, ctx_mid, 2 * target.n_layers)
            per_kernel[name] = {"ms": ms, "GB/s": by / (ms * 1e-3) / 1e9}
        extras["per_kernel_at_M"] = per_kernel
        sweep = {}
        for kk in range(0, k_max + 1):
            ms, by = eng.time_kernel(6, kk + 1, ctx_mid, 3)
            sweep[str(kk)] = {"ms": ms, "GB/s": by / (ms * 1e-3) / 1e9, "frac": by / (ms * 1e-3) / 1e9 / HBM_PEAK_GBPS}
        extras["verify_vs_k"] = sweep
        extras["verify_vs_k_max_over_k0"] = max(v["ms"] for v in sweep.values()) / sweep["0"]["ms"]
        # the spec quantities beside the dominant kernel's: the whole verification at the headline's k and one
        # draft step, algorithmic bytes (all matrices + keys and values of the context) over measured time
        extras["verify"] = dict(sweep[str(k)], k=k, rows=k + 1, context=ctx_mid)
        ms, by = eng.time_kernel(7, 1, ctx_mid, 8)
        extras["draft_step"] = {"ms": ms, "GB/s": by / (ms * 1e-3) / 1e9, "frac": by / (ms * 1e-3) / 1e9 / HBM_PEAK_GBPS}
    # ---- draft length following the acceptance (same output, other iteration count) -----------------------
    if not args.no_sweep:
        eng.prefill(prompt)
        t1 = time.perf_counter()
        toks_a, st_a = eng.decode_adaptive(G, 2)
        dt_a = time.perf_counter() - t1
        assert np.array_equal(toks_a, toks0), "adaptive draft length changed the output"
        extras["adaptive_draft_length"] = {"k_first": 2, "k_max": k_max, "tokens_per_s": G / dt_a,
                                           "iterations": st_a.iterations,
                                           "mean_tokens_per_iteration": G / max(1, st_a.iterations)}
        log(f"[bench] adaptive draft length: {G / dt_a:.0f} tok/s, {st_a.iterations} iterations")

    # ---- sampling variant: assistant and main model sample at a temperature, keep / replace validation --------
    if not args.no_sweep:
        sampled = {}
        for temp in (0.02, 0.1, 1.0):
            eng.prefill(prompt)
            eng.decode_sampled(G, k, temp, 1)                      # graph capture
            eng.prefill(prompt)
            toks_s, st_s = eng.decode_sampled(G, k, temp, 1)
            sampled[f"T{temp}"] = {"temperature": temp, "k": k, "tokens_per_s": G / (st_s.ms_decode * 1e-3),
                                   "iterations": st_s.iterations, "mean_tokens_per_iteration": G / st_s.iterations,
                                   "ms_verify_per_iteration": st_s.ms_verify / st_s.iterations,
                                   "ms_draft_per_iteration": st_s.ms_draft / st_s.iterations,
                                   "distinct_tokens": int(len(set(toks_s.tolist())))}
            log(f"[bench] sampled T={temp} k={k}: {sampled[f'T{temp}']['tokens_per_s']:.0f} tok/s, "
                f"{st_s.iterations} iterations, verify {sampled[f'T{temp}']['ms_verify_per_iteration']:.2f} ms/iteration")
        extras["sampled"] = sampled

    # ---- several sequences per forward (not the headline: the workload is one sequence) -------------------
    # B prompts of the workload's length share every weight pass: aggregate tokens/s of stairs_generate_batch,
    # decode phase, prompt 0 is the workload's prompt and must reproduce its tokens bit for bit
    if not args.no_sweep and w["dtype"] == "bf16":
        rngp = np.random.default_rng([w["seed"], 4242])
        V = w["target"]["vocab"]
        # every sequence has K/V caches of its own (both models, half precision): as many slots as fit 128 GB
        kv_per_seq = sum(2 * 2 * m.n_layers * m.n_heads * m.head_dim for m in (target, draft)) * (P + G + k_max + 8)
        n_seq = 64
        while n_seq > 8 and n_seq * kv_per_seq > 128e9:
            n_seq //= 2
        prompts = [prompt] + [rngp.integers(0, V, P).astype(np.int32) for _ in range(n_seq - 1)]
        eng.reserve_batch(n_seq)
        batched = {}
        flop_per_row = 2.0 * 2.0 * target.n_params()          # high and low part of every activation
        for B, kk in ((2, k), (4, k), (8, k), (8, 3), (16, k), (16, 3), (32, k), (64, k)):
            rows = B * (kk + 1)
            if rows > 256 or B > n_seq:
                continue
            toks_b, st_b = eng.generate_batch(prompts[:B], G, kk)
            if rows <= 64:      # the weight-streaming kernels: bit for bit the sequence alone
                assert np.array_equal(toks_b[0], toks0), "a sequence of the batch differs from the same sequence alone"
            ms_v = st_b.ms_verify / max(1, st_b.iterations)
            batched[f"B{B}_k{kk}"] = {"sequences": B, "k": kk, "rows_per_forward": rows,
                                      "kernels": "decode (weight-streaming)" if rows <= 64 else "block (MFMA GEMM)",
                                      "tokens_per_s": B * G / (st_b.ms_decode * 1e-3), "iterations": st_b.iterations,
                                      "ms_verify_per_iteration": ms_v,
                                      "verify_weight_GBps": target.weight_bytes_streamed() / (ms_v * 1e-3) / 1e9,
                                      "verify_mfma_frac": flop_per_row * rows / (ms_v * 1e-3) / 2.5e15,
                                      "ms_draft_per_iteration": st_b.ms_draft / max(1, st_b.iterations),
                                      "prefill_ms": st_b.ms_prefill,
                                      "tokens_equal_sequence_alone": bool(np.array_equal(toks_b[0], toks0))}
            log(f"[bench] batch B={B} k={kk} ({rows} rows): {batched[f'B{B}_k{kk}']['tokens_per_s']:.0f} tok/s aggregate, "
                f"{st_b.iterations} iterations, verify {ms_v:.2f} ms/iteration, "
                f"MFMA {100 * batched[f'B{B}_k{kk}']['verify_mfma_frac']:.1f} %")
        extras["batched_sequences"] = batched
    eng.close()

    # ---- encoder-decoder pairs in the shapes of the paper's checkpoints (not the headline) -----------------
    if not args.no_sweep and args.encdec:
        extras["encoder_decoder"] = {name: encdec_leg(name) for name in args.encdec.split(",") if name}

    out = {
        "metric": "generated tokens/sec (stairs greedy, 7B-class target)" if "7b" in args.workload
                  else "generated tokens/sec (stairs greedy)",
        "value": value, "unit": "tokens/s", "n_gpus": 1, "steps": len(decode_s), "warmup": args.warmup,
        "ms_per_step": 1e3 * total / len(decode_s), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": w["dtype"], "data": "synthetic",
        "config": {"workload": args.workload, "prompt_len": P, "generate": G, "k": k, "stair_rows": k + 1,
                   "timed_region": "decode phase (prefill excluded)"},
        "tokens_per_s_over_steps": spread,
        "iterations_per_step": stats_last.iterations, "mean_tokens_per_iteration": G / stats_last.iterations,
        "accept_hist": list(stats_last.accept_hist)[:k + 1],
        "ms_draft_per_step": stats_last.ms_draft, "ms_verify_per_step": stats_last.ms_verify,
        "prefill_ms": prefill_ms, "k_sweep": k_table,
        # prompt ingestion (outside the timed region): the layer projections of both models over the P-1 ingested rows,
        # each activation issued as a high and a low bf16 part, against the dense bf16 MFMA peak
        "prefill": {"ms": prefill_ms, "rows": P - 1, "tokens_per_s": (P - 1) / (prefill_ms * 1e-3),
                    "issued_mfma_frac_of_2.5PFLOPs": (2.0 * 2.0 * (P - 1) * sum(m.n_params() - m.vocab * m.d_model for m in (target, draft))
                                                      / (prefill_ms * 1e-3) / 2.5e15) if w["dtype"] == "bf16" else None},
        "plain_greedy_tokens_per_s": G / plain_s,
        "time_reduction_vs_plain_greedy_pct": 100.0 * (1.0 - (total / len(decode_s)) / plain_s),
        "paper_context": "paper reports 9.58-17.24 % inference-time reduction (T5-3B / T5-large + T5-small, MacBook Pro M2 32 GB)",
        "roofline": roofline,
    }
    out.update(extras)
    if not args.no_cpu_baseline:
        sp, sg = (int(x) for x in args.cpu_sample.split(","))
        out["cpu_baseline"] = cpu_baseline(w, target, draft, prompt, k, min(sp, P), sg)
        out["gpu_over_cpu_baseline"] = value / out["cpu_baseline"]["value"]
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
