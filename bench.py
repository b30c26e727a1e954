"""Benchmark of the pruned prefill: TTFT and prompt tokens/s on one MI355X.

One step = one whole prefill (embedding, 32 pruned decoder layers with scoring / selection /
compaction / Aux Cache writes, final norm, LM head) of the 7B-shaped model on a 3376-token
synthetic prompt already resident in HBM.  Prints ONE JSON line.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_FP8_TFLOPS = 5000.0         # MI355X dense fp8 matrix peak
PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0
PMC_PROFILE = os.path.join(ROOT, "profiles", "gemm_attention_7b_3376_pmc.md")


def gate_up_traffic_bytes():
    """Bytes per launch the dominant kernel (gate/up GEMM, SwiGLU epilogue) moves through the L2s'
    fabric side, averaged over the 32 launches of a 7b_3376 step: rocprofv3 FETCH_SIZE x 2 KiB +
    WRITE_SIZE x 1 KiB, factors calibrated on a 1 GiB copy.  Read from the committed counter summary
    (the line "Gate/up projection, all four stages: <x> MB per launch"); None if it is not there."""
    import re
    try:
        m = re.search(r"Gate/up projection, all four stages: ([0-9.]+) MB per launch", open(PMC_PROFILE).read())
    except OSError:
        return None
    return float(m.group(1)) * 1e6 if m else None


STEP_KERNEL = {"gemm_gate_up": "gemm_pp_kernel<4,2,2,4,EPI_SWIGLU> (RMSNorm scale + gate/up projection + SiLU*mul; at 355 rows "
                               "the same epilogue under gemm_psk_kernel<2,4,3,2,EPI_SWIGLU>)",
               "gemm_qkv": "gemm_pp_kernel<4,2,2,4,EPI_QKV_ROPE128> (RMSNorm scale + QKV projection + RoPE + V^T)",
               "gemm_down": "gemm_pp_kernel<4,2,2,4,EPI_RESIDUAL> (down projection + residual + row sums of squares)",
               "gemm_o": "gemm_pp_kernel<4,2,2,4,EPI_RESIDUAL> (O projection + residual + row sums of squares)"}


def kernel_sweep(args, torch, B) -> int:
    """Stand-alone timing of the HBM-bound steps at 7B row width (H=32, hd=128, d=4096).

    Each measurement flushes the caches first (a 1 GiB fill between launches), so the bytes
    really come from HBM; the rate is algorithmic bytes / event time of the launch alone."""
    dev = "cuda:0"
    H, hd, d = 32, 128, 4096
    flush = torch.empty(1 << 28, dtype=torch.int32, device=dev)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)

    def timed(fn, reps=5):
        best, tot = 1e9, 0.0
        fn()                                   # first call pays one-time set-up
        for _ in range(reps):
            flush.fill_(1)
            torch.cuda.synchronize()
            e0.record(); fn(); e1.record()
            torch.cuda.synchronize()
            ms = e0.elapsed_time(e1)
            best = min(best, ms); tot += ms
        return tot / reps, best

    rows = []
    g = torch.Generator(dev).manual_seed(7)
    # calibration: what a plain device-to-device copy of 1 GiB reaches on this machine
    src = torch.empty(1 << 28, dtype=torch.int32, device=dev).fill_(3)
    dst = torch.empty_like(src)
    avg, best = timed(lambda: dst.copy_(src))
    rows.append({"kernel": "plain copy 1 GiB (torch, calibration)", "n": 1, "bytes": 2 << 30, "avg_us": round(avg * 1e3, 2),
                 "best_us": round(best * 1e3, 2), "gbs": round((2 << 30) / (avg * 1e-3) / 1e9, 1)})
    del src, dst
    for n in (3376, 8192, 36864, 262144):
        k = torch.randn(n, d, device=dev, generator=g).to(torch.bfloat16)
        q_last = torch.randn(d, device=dev, generator=g).to(torch.bfloat16)
        s = torch.empty(n, dtype=torch.float32, device=dev)
        scratch = torch.empty(B.lazyllm_op_score_scratch_bytes(n, H), dtype=torch.uint8, device=dev)
        avg, best = timed(lambda: B.lazyllm_op_score(q_last, k, s, scratch, n, H, hd))
        byt = n * d * 2 + d * 2 + 4 * n
        rows.append({"kernel": "score (Eq. 1, three launches)", "n": n, "bytes": byt, "avg_us": round(avg * 1e3, 2),
                     "best_us": round(best * 1e3, 2), "gbs": round(byt / (avg * 1e-3) / 1e9, 1)})
        kk = max(1, (n * 7 + 9) // 10)
        keep = torch.empty(kk, dtype=torch.int32, device=dev)
        prune = torch.empty(max(1, n - kk), dtype=torch.int32, device=dev)
        sc = torch.rand(n, device=dev, generator=g)
        avg, best = timed(lambda: B.lazyllm_op_select(sc, n, kk, keep, prune))
        rows.append({"kernel": "select (one workgroup)", "n": n, "bytes": 8 * n, "avg_us": round(avg * 1e3, 2),
                     "best_us": round(best * 1e3, 2), "gbs": round(8 * n / (avg * 1e-3) / 1e9, 2)})
        B.lazyllm_op_select(sc, n, kk, keep, prune)
        pos = torch.arange(n, dtype=torch.int32, device=dev)
        h_out = torch.empty(kk, d, dtype=torch.bfloat16, device=dev)
        aux = torch.empty(max(1, n - kk), d, dtype=torch.bfloat16, device=dev)
        pos_out = torch.empty(kk, dtype=torch.int32, device=dev)
        aux_pos = torch.empty(max(1, n - kk), dtype=torch.int32, device=dev)
        avg, best = timed(lambda: B.lazyllm_op_gather(k, pos, keep, kk, prune, n - kk, h_out, pos_out, aux, aux_pos, d))
        byt = 2 * n * d * 2 + 16 * n
        rows.append({"kernel": "gather + aux scatter", "n": n, "bytes": byt, "avg_us": round(avg * 1e3, 2),
                     "best_us": round(best * 1e3, 2), "gbs": round(byt / (avg * 1e-3) / 1e9, 1)})
        x = torch.empty_like(k)
        gain = torch.ones(d, dtype=torch.bfloat16, device=dev)
        avg, best = timed(lambda: B.lazyllm_op_rmsnorm(k, gain, x, n, d, 1e-5))
        byt = 2 * n * d * 2
        rows.append({"kernel": "rmsnorm", "n": n, "bytes": byt, "avg_us": round(avg * 1e3, 2),
                     "best_us": round(best * 1e3, 2), "gbs": round(byt / (avg * 1e-3) / 1e9, 1)})
        del k, x, h_out, aux
    V = 32000
    w = (torch.randn(V, d, device=dev, generator=g) * 0.02).to(torch.bfloat16)
    hl = torch.randn(d, device=dev, generator=g).to(torch.bfloat16)
    gain = torch.ones(d, dtype=torch.bfloat16, device=dev)
    xf = torch.empty(d, dtype=torch.float32, device=dev)
    lg = torch.empty(V, dtype=torch.float32, device=dev)
    avg, best = timed(lambda: B.lazyllm_op_lm_head(hl, gain, w, xf, lg, d, V, 1e-5))
    rows.append({"kernel": "final norm + LM head", "n": 1, "bytes": V * d * 2, "avg_us": round(avg * 1e3, 2),
                 "best_us": round(best * 1e3, 2), "gbs": round(V * d * 2 / (avg * 1e-3) / 1e9, 1)})
    # empty-launch floor for reference
    one = torch.zeros(1, dtype=torch.float32, device=dev)
    keep1 = torch.empty(1, dtype=torch.int32, device=dev)
    avg, best = timed(lambda: B.lazyllm_op_select(one, 1, 1, keep1, keep1))
    rows.append({"kernel": "launch floor (select on 1 token)", "n": 1, "bytes": 8, "avg_us": round(avg * 1e3, 2),
                 "best_us": round(best * 1e3, 2), "gbs": 0.0})
    print(json.dumps({"mode": "kernels", "peak_hbm_gbs": PEAK_HBM_GBS, "rows": rows}))
    for r in rows:
        print("%-34s n=%7d  %9.2f us (best %9.2f)  %8.1f GB/s  %5.1f %% of 8 TB/s" % (
            r["kernel"], r["n"], r["avg_us"], r["best_us"], r["gbs"], 100.0 * r["gbs"] / PEAK_HBM_GBS), file=sys.stderr)
    return 0


def schedule_sweep(args, wl, shape, n_tokens, timed, B) -> int:
    """TTFT against the share of token-layers computed, for the schedule families the paper compares: one pruning
    layer at varying depth and keep ratio (section "Drop Rate in Different Layers"), all pruning at once after the
    first few layers (the static-pruning baseline of section "Results"), and progressive schedules (section
    "Inference with LazyLLM").  Accuracy needs trained weights and is not measured; this is the cost axis."""
    L = shape.n_layers
    steps, warmup = max(3, args.steps // 4), 2
    dense_ms, _ = timed([], steps, warmup)
    grid = [("dense", [])]
    grid.append(("progressive (workload's own)", list(wl.schedule)))
    if L >= 32:
        grid.append(("progressive 90/70/50/30 % at 6/12/18/24", [(6, 900), (12, 778), (18, 714), (24, 600)]))
        grid.append(("progressive 50 % at 4/12/20", [(4, 500), (12, 500), (20, 500)]))
    for layer in sorted({max(1, L // 16), max(1, L // 8)}):
        for permille in (700, 500, 300):
            grid.append(("static: all pruning at layer %d, keep %d %%" % (layer, permille // 10), [(layer, permille)]))
    for layer in sorted({max(1, (L * q) // 8) for q in range(2, 8)}):
        for permille in (900, 700, 500, 300, 100):
            grid.append(("one pruning layer %d, keep %d %%" % (layer, permille // 10), [(layer, permille)]))
    rows = []
    for name, schedule in grid:
        ms, out = timed(schedule, steps, warmup)
        assert out.status == 0
        tl = sum(out.n_tokens)
        rows.append({"schedule": name, "keep_permille_of_survivors": schedule,
                     "token_layers_frac": round(tl / (n_tokens * L), 4), "ttft_ms": round(ms, 3),
                     "speedup_vs_dense": round(dense_ms / ms, 3)})
    print(json.dumps({"mode": "schedules", "workload": wl.name, "prompt_tokens": n_tokens, "steps": steps,
                      "dense_ttft_ms": round(dense_ms, 3), "rows": rows}))
    for r in rows:
        print("%-48s token-layers %5.1f %%  TTFT %8.3f ms  x%.2f" % (
            r["schedule"], 100 * r["token_layers_frac"], r["ttft_ms"], r["speedup_vs_dense"]), file=sys.stderr)
    return 0


def decode_bench(args, wl, shape, model, ids, sched, n_tokens, torch, B) -> int:
    """Decoding steps after the workload's prefill (Sec. 3.2, "Aux Cache"; Sec. 5.3's "% of prompt tokens
    computed" and generation time), pruned and unpruned.  A step is timed from its launch to the
    completion of its logits; tokens are chosen greedily on the device (the argmax is not timed)."""
    steps = args.decode
    L = shape.n_layers
    runs = {}
    for name, schedule in (("lazy", sched), ("dense", [])):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        out = model.prefill(ids, schedule)
        torch.cuda.synchronize()
        prefill_ms = (time.perf_counter() - t0) * 1e3
        tok = torch.argmax(out.logits[0]).to(torch.int32).reshape(1)
        gen = B.Generation(model, schedule, out, n_tokens + steps + 1)
        torch.cuda.synchronize()
        rows = []
        for t in range(steps):
            t0 = time.perf_counter()
            so = gen.step(tok)
            torch.cuda.synchronize()
            ms = (time.perf_counter() - t0) * 1e3
            tok = torch.argmax(so.logits).to(torch.int32).reshape(1)
            stage_rows = sorted(set(so.n_ran), reverse=True)
            rows.append({"step": t + 1, "ms": round(ms, 3), "token_layers_run": int(sum(so.n_ran)),
                         "most_rows_in_a_layer": max(so.n_ran)})
            assert so.status == 0
        prof = None
        if name == "dense":
            # one more unpruned step with per-launch events: where a step's time goes, and the rate at
            # which its largest launch (the gate/up projection: 2 * d_ffn * d_model bf16 weights) streams
            B.lazyllm_profile_begin()
            so = gen.step(tok)
            recs = B.lazyllm_profile_end(1 << 16)
            by = {}
            for r in recs:
                a = by.setdefault(r["step"], [0.0, 0])
                a[0] += r["ms"]; a[1] += 1
            gu_ms, gu_n = by["gemm_gate_up"]
            gu_bytes = 2.0 * 2.0 * shape.d_ffn * shape.d_model
            achieved = gu_bytes / (gu_ms / gu_n * 1e-3) / 1e9
            prof = {"ms_by_step": {k: round(v[0], 4) for k, v in sorted(by.items(), key=lambda kv: -kv[1][0])},
                    "roofline": {"bound": "hbm", "kernel": "gemm_skinny_kernel<EPI_SWIGLU> (gate/up projection, one token row)",
                                 "achieved": round(achieved, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s",
                                 "frac": round(achieved / PEAK_HBM_GBS, 4), "avg_launch_ms": round(gu_ms / gu_n, 5),
                                 "algorithmic_bytes_per_launch": gu_bytes, "traffic": None}}
        view = gen.view()
        computed = float(sum(float(view["has_kv"][l][:n_tokens].float().mean()) for l in range(L)) / L)
        runs[name] = {"prefill_ms": round(prefill_ms, 3), "steps": rows, "profiled_step": prof,
                      "decode_ms_total": round(sum(r["ms"] for r in rows), 3),
                      "generation_ms": round(prefill_ms + sum(r["ms"] for r in rows), 3),
                      "prompt_token_layers_computed": round(computed, 4)}
        gen.close()
    lazy, dense = runs["lazy"], runs["dense"]
    print(json.dumps({"mode": "decode", "workload": wl.name, "prompt_tokens": n_tokens, "new_tokens": steps,
                      "generation_speedup_vs_dense": round(dense["generation_ms"] / lazy["generation_ms"], 3),
                      "lazy": lazy, "dense": dense}))
    for name in ("lazy", "dense"):
        r = runs[name]
        print("%-5s prefill %8.3f ms  %d steps %9.3f ms  total %9.3f ms  prompt token-layers computed %5.1f %%" % (
            name, r["prefill_ms"], steps, r["decode_ms_total"], r["generation_ms"],
            100 * r["prompt_token_layers_computed"]), file=sys.stderr)
        for row in r["steps"][:12] + ([r["steps"][-1]] if steps > 12 else []):
            print("      step %3d  %8.3f ms  token-layers run %6d  most rows in a layer %5d" % (
                row["step"], row["ms"], row["token_layers_run"], row["most_rows_in_a_layer"]), file=sys.stderr)
    return 0


def fused_compaction_study(args, wl, model, ids, sched, cu, scale, torch, B) -> int:
    """Sec. 3.2's gather as a kernel of its own (kept rows copied into a compact buffer) against the form
    that leaves them in place and lets the next layer's QKV and O projections read them through the index.
    The two forms alternate (three rounds of `steps` prefills each); a profiled pass of each gives the
    times of the steps that differ, at the pruning layers only."""
    prune_layers = [l for l, p in sched if p < 1000]
    res = {}
    for rnd in range(3):
        for name, flags in (("separate", 0), ("fused", B.LAZYLLM_FUSE_COMPACTION)):
            for _ in range(3):
                model.prefill(ids, sched, cu_seqlens=cu, embed_scale=scale, flags=flags)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(args.steps):
                out = model.prefill(ids, sched, cu_seqlens=cu, embed_scale=scale, flags=flags)
            torch.cuda.synchronize()
            assert out.status == 0
            res.setdefault(name, []).append(round((time.perf_counter() - t0) * 1e3 / args.steps, 4))
    steps = {}
    for name, flags in (("separate", 0), ("fused", B.LAZYLLM_FUSE_COMPACTION)):
        B.lazyllm_profile_begin()
        for _ in range(args.steps):
            model.prefill(ids, sched, cu_seqlens=cu, embed_scale=scale, flags=flags)
        recs = B.lazyllm_profile_end(1 << 20)
        by = {}
        for r in recs:
            if r["layer"] in prune_layers and r["step"] in ("gather", "gemm_qkv", "gemm_o"):
                by[(r["layer"], r["step"])] = by.get((r["layer"], r["step"]), 0.0) + r["ms"] / args.steps
        steps[name] = {"layer %d %s" % k: round(v * 1e3, 2) for k, v in sorted(by.items())}
    print(json.dumps({"study": "compaction as a kernel vs folded into the next layer's operand loads",
                      "workload": wl.name, "steps": args.steps, "ttft_ms": res,
                      "us_per_step_at_pruning_layers": steps}))
    return 0


def band_height_sweep(args, torch, B) -> int:
    """The dominant GEMM alone (gate/up projection of the 7B shape at 3376 rows, 256x256 ping-pong tiles)
    against the height of the tile-walk band: the number of tile rows that share a run of W column blocks in
    one XCD's L2.  Under `rocprofv3 --pmc FETCH_SIZE` the launches of one band height are told apart by their
    order, which the lines printed here give.  The weights rotate over 8 copies, so none is L2-resident from
    the launch before."""
    dev = "cuda:0"
    N, K, M = 22016, 4096, 3376
    n_w, reps, warm = 8, max(args.steps, 4), 4
    ws = []
    for _ in range(n_w):
        w = (torch.randn(N, K, device=dev) * 0.02).to(torch.bfloat16)
        wb = torch.empty_like(w)
        B.lazyllm_op_pack_weight_ksteps(w, N, K, K, wb)
        ws.append(wb)
        del w
    a = torch.randn(M, K, device=dev).to(torch.bfloat16)
    c = torch.zeros(M, N // 2, device=dev, dtype=torch.bfloat16)
    rows = []
    for gm in (1, 2, 4, 7, 14):
        e = B.EPI_SWIGLU | (5 << 8) | (gm << 16) | (1 << 29)     # forced: 256x256 ping-pong tiles, band height gm
        for i in range(warm):
            B.lazyllm_op_gemm(a, ws[i % n_w], c, None, M, N, K, K, K, N // 2, e)
        torch.cuda.synchronize()
        t0 = torch.cuda.Event(enable_timing=True)
        t1 = torch.cuda.Event(enable_timing=True)
        t0.record()
        for i in range(reps):
            B.lazyllm_op_gemm(a, ws[i % n_w], c, None, M, N, K, K, K, N // 2, e)
        t1.record()
        torch.cuda.synchronize()
        us = t0.elapsed_time(t1) / reps * 1e3
        rows.append({"band_height": gm, "launches": warm + reps, "us_per_launch": round(us, 1),
                     "tflops": round(2.0 * M * N * K / us / 1e6, 1)})
        print("band height %2d: %d launches (%d warm-up + %d timed), %.1f us per launch, %.0f TFLOP/s" % (
            gm, warm + reps, warm, reps, us, rows[-1]["tflops"]), file=sys.stderr, flush=True)
    print(json.dumps({"study": "tile-walk band height, gate/up projection", "M": M, "N": N, "K": K,
                      "rows": rows}))
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="7b_3376")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-baseline-layers", type=int, default=0, metavar="N",
                    help="time the CPU checker on the first N layers only and scale by token-layers "
                         "(default 0: the whole pruned prefill, all layers, timed as it is)")
    ap.add_argument("--no-other-workloads", action="store_true",
                    help="skip the short timings of the other workloads (tiny512, 7b_8192, needles, batch of 8)")
    ap.add_argument("--no-dense", action="store_true", help="skip the unpruned comparison run")
    ap.add_argument("--breakdown", action="store_true", help="print the per-step time table to stderr")
    ap.add_argument("--kernels", action="store_true",
                    help="instead of the prefill, time the bandwidth-bound steps (scoring, selection, "
                         "compaction, LM head) alone over a sweep of token counts with cold caches")
    ap.add_argument("--band-heights", action="store_true",
                    help="instead of the prefill, time the dominant GEMM alone under tile-walk bands of 1, 2, 4, 7 "
                         "and 14 tile rows (--steps launches each)")
    ap.add_argument("--schedules", action="store_true",
                    help="instead of the headline line, time the prefill under a grid of keep schedules: one "
                         "pruning layer at varying depth and keep ratio (the paper's drop-rate study), pruning "
                         "all at once after the first few layers (its static-pruning baseline), progressive")
    ap.add_argument("--prefill-flags", type=int, default=0, metavar="BITS",
                    help="LAZYLLM_* flag bits for the timed prefills (4 = compaction folded into the next layer)")
    ap.add_argument("--fused-compaction", action="store_true",
                    help="study: the prefill with the compaction folded into the next layer's operand loads "
                         "(LAZYLLM_FUSE_COMPACTION) against the copying form, alternating, with the times of the "
                         "steps involved at the three pruning layers")
    ap.add_argument("--decode", type=int, default=0, metavar="STEPS",
                    help="instead of the headline line, run the prefill and then this many decoding steps "
                         "with Aux Cache revival (greedy tokens), and the same with no pruning; prints the time "
                         "of every step, the tokens revived and the share of prompt tokens computed")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU only: the pruned prefill of one prompt is a single-GPU job "
              "(--gpus %d refused)" % args.gpus, file=sys.stderr)
        return 2

    import numpy as np
    import torch
    from paper_2407_14057_amd import binding as B
    from paper_2407_14057_amd import synth

    if args.kernels:
        return kernel_sweep(args, torch, B)
    if args.band_heights:
        return band_height_sweep(args, torch, B)

    wl = synth.WORKLOADS[args.workload]
    shape = wl.shape
    dev = "cuda:0"
    torch.cuda.set_device(0)
    wdev = "cpu" if shape.d_model <= 512 else dev
    f8 = shape.gemm_dtype == 1                      # projections in the 8-bit variant (not the headline)
    weights = synth.make_weights(shape, wl.weight_seed, wdev)
    if wdev == "cpu":
        weights = {k: ([t.to(dev) for t in v] if isinstance(v, list) else v.to(dev)) for k, v in weights.items()}
    # the CPU checker gets the same bytes (bf16 bit patterns on the host); the 8-bit variant's checker
    # is slow (per-row quantisation in numpy), so its sample is the first layer unless told otherwise
    cpu_layers = args.cpu_baseline_layers if args.cpu_baseline_layers > 0 else (1 if f8 else 0)
    cpu_layers = min(cpu_layers, shape.n_layers)
    want_cpu = not args.no_cpu_baseline and len(wl.seqlens) == 1
    host_bits = None
    if want_cpu:
        if cpu_layers:
            host_bits = {k: ([synth.layer_to_host_bits(weights, l)[k] for l in range(cpu_layers)] if isinstance(v, list)
                             else v.cpu().view(torch.int16).numpy().view(np.uint16)) for k, v in weights.items()}
        else:
            host_bits = synth.weights_to_host_bits(weights)
    # checksum of the inputs as the library gets them (bf16 bit patterns summed per tensor as integers,
    # tensors weighted by their order), so that two reports can be told to be about the same bytes
    wsum, idx = 0, 0
    for name in sorted(weights):
        for t in (weights[name] if isinstance(weights[name], list) else [weights[name]]):
            idx += 1
            wsum = (wsum + idx * int(t.view(torch.int16).to(torch.int64).sum().item())) % (1 << 61)
    model = B.Model(shape.as_dict(), weights, dev)
    del weights
    torch.cuda.empty_cache()

    inp = synth.make_workload_inputs(wl)
    ids = torch.from_numpy(inp["token_ids"]).to(dev)
    ids_sum = int(np.dot(inp["token_ids"].astype(np.int64), np.arange(1, inp["token_ids"].shape[0] + 1)) % (1 << 61))
    scale = None if inp["embed_scale"] is None else torch.from_numpy(inp["embed_scale"]).to(dev)
    cu = [int(x) for x in inp["cu_seqlens"]]
    sched = list(wl.schedule)
    n_tokens = int(ids.numel())

    def step(schedule):
        return model.prefill(ids, schedule, cu_seqlens=cu, embed_scale=scale, flags=args.prefill_flags)

    def timed(schedule, steps, warmup):
        for _ in range(warmup):
            step(schedule)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            out = step(schedule)
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / steps, out

    if args.fused_compaction:
        return fused_compaction_study(args, wl, model, ids, sched, cu, scale, torch, B)
    if args.schedules:
        return schedule_sweep(args, wl, shape, n_tokens, timed, B)
    if args.decode:
        return decode_bench(args, wl, shape, model, ids, sched, n_tokens, torch, B)

    ms, out = timed(sched, args.steps, args.warmup)
    assert out.status == 0
    dense_ms = None
    if not args.no_dense:
        dense_ms, _ = timed([], max(3, args.steps // 4), 2)

    # ---- each prefill timed on its own (event pair on the stream the prefill runs on): median, min
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
           for _ in range(max(args.steps, 20))]
    for a, b in evs:
        a.record(); step(sched); b.record()
    torch.cuda.synchronize()
    each = sorted(a.elapsed_time(b) for a, b in evs)
    ttft_median, ttft_min = each[len(each) // 2], each[0]

    # ---- per-launch timing (hipEvents on the prefill's stream), same steps again
    B.lazyllm_profile_begin()
    for _ in range(args.steps):
        step(sched)
    recs = B.lazyllm_profile_end(1 << 20)
    by_step = {}
    for r in recs:
        a = by_step.setdefault(r["step"], [0.0, 0.0, 0])
        a[0] += r["ms"]; a[1] += r["work"]; a[2] += 1
    gemm_steps = ("gemm_qkv", "gemm_o", "gemm_gate_up", "gemm_down")
    dom = max(gemm_steps, key=lambda s: by_step.get(s, [0, 0, 0])[0])
    dms, dwork, dn = by_step[dom]
    achieved = dwork / (dms * 1e-3) / 1e12                       # TFLOP/s over this step's launches
    traffic = gate_up_traffic_bytes() if (dom == "gemm_gate_up" and wl.name == "7b_3376") else None
    peak = PEAK_FP8_TFLOPS if f8 else PEAK_BF16_TFLOPS
    kernel = ("quantize_rows_f8_kernel + gemm_f8_kernel (%s)" % dom) if f8 else STEP_KERNEL[dom]
    roofline = {"bound": "mfma", "kernel": kernel, "achieved": round(achieved, 1),
                "peak": peak, "unit": "TFLOP/s", "frac": round(achieved / peak, 4),
                "avg_launch_ms": round(dms / dn, 5), "flops_per_launch": dwork / dn, "traffic": traffic,
                "algorithmic_bytes_per_launch": None}
    if dom == "gemm_gate_up":
        # operands read once + activation written once, averaged over the step's launches
        rows_avg = sum(r["rows"] for r in recs if r["step"] == dom) / max(1, dn)
        roofline["algorithmic_bytes_per_launch"] = round(
            2.0 * (rows_avg * shape.d_model + 2.0 * shape.d_ffn * shape.d_model + rows_avg * shape.d_ffn))
    total_prof_ms = sum(v[0] for v in by_step.values()) / args.steps
    breakdown = {}
    for s, (tms, work, cnt) in sorted(by_step.items(), key=lambda kv: -kv[1][0]):
        per = tms / args.steps
        rate = work / (tms * 1e-3) if tms > 0 else 0.0
        is_flop = s.startswith("gemm") or s == "attention"
        breakdown[s] = {"ms_per_step": round(per, 4), "launches_per_step": cnt // args.steps,
                        ("tflops" if is_flop else "gbs"): round(rate / (1e12 if is_flop else 1e9), 1)}
    if args.breakdown:
        print(json.dumps(breakdown, indent=1), file=sys.stderr)
        by_rows = {}
        for r in recs:
            a = by_rows.setdefault((r["step"], r["rows"]), [0.0, 0.0, 0])
            a[0] += r["ms"]; a[1] += r["work"]; a[2] += 1
        for (st, rows), (tms, work, cnt) in sorted(by_rows.items()):
            if st.startswith("gemm") or st == "attention":
                print("%-14s rows=%6d  avg %8.1f us  %7.1f TFLOP/s" % (st, rows, tms / cnt * 1e3, work / (tms * 1e-3) / 1e12),
                      file=sys.stderr)
            else:
                print("%-14s rows=%6d  avg %8.1f us  %7.1f GB/s" % (st, rows, tms / cnt * 1e3, work / (tms * 1e-3) / 1e9),
                      file=sys.stderr)

    total_flops = sum(by_step[s][1] for s in gemm_steps + ("attention",) if s in by_step) / args.steps

    # ---- a TTFT sample that counts the host's enqueue time: the stream is idle when the call starts
    synced = []
    for _ in range(min(args.steps, 10)):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        step(sched)
        torch.cuda.synchronize()
        synced.append((time.perf_counter() - t0) * 1e3)
    synced.sort()

    # ---- what Eq. 1 costs inside the prefill: the same profiled pass with scores only where a
    # pruning layer consumes them (the attention kernel then skips the logit side output and the
    # gate/up launch its finishing workgroups on the other layers)
    score_cost = None
    if len(cu) == 2:
        B.lazyllm_profile_begin()
        for _ in range(args.steps):
            model.prefill(ids, sched, cu_seqlens=cu, embed_scale=scale, flags=B.LAZYLLM_SCORE_ONLY_USED)
        recs_u = B.lazyllm_profile_end(1 << 20)
        tot_u = {}
        for r in recs_u:
            tot_u[r["step"]] = tot_u.get(r["step"], 0.0) + r["ms"]
        score_cost = {k: round((by_step[k][0] - tot_u.get(k, 0.0)) / args.steps, 4) for k in ("attention", "gemm_gate_up")}
        score_cost["note"] = ("ms per prefill that scoring all 32 layers adds to these two steps, against scoring "
                              "only the %d layers whose successor prunes" % len([1 for _, p in sched if p < 1000]))

    # ---- the other workloads, a few steps each (same model where the shape is the same)
    others = None
    if wl.name == "7b_3376" and not args.no_other_workloads:
        others = {}
        for name in ("tiny512", "7b_8192", "7b_3376_needles", "7b_batch8"):
            w2 = synth.WORKLOADS[name]
            m2 = model
            if w2.shape != shape:
                wt = synth.make_weights(w2.shape, w2.weight_seed, "cpu")
                wt = {k: ([t.to(dev) for t in v] if isinstance(v, list) else v.to(dev)) for k, v in wt.items()}
                m2 = B.Model(w2.shape.as_dict(), wt, dev)
            i2 = synth.make_workload_inputs(w2)
            ids2 = torch.from_numpy(i2["token_ids"]).to(dev)
            sc2 = None if i2["embed_scale"] is None else torch.from_numpy(i2["embed_scale"]).to(dev)
            cu2 = [int(x) for x in i2["cu_seqlens"]]

            def timed2(schedule, steps, warmup):
                for _ in range(warmup):
                    m2.prefill(ids2, schedule, cu_seqlens=cu2, embed_scale=sc2)
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                for _ in range(steps):
                    o2 = m2.prefill(ids2, schedule, cu_seqlens=cu2, embed_scale=sc2)
                torch.cuda.synchronize()
                return (time.perf_counter() - t0) * 1e3 / steps, o2
            k2 = 5 if ids2.numel() < 20000 else 3
            ms2, o2 = timed2(list(w2.schedule), k2, 2)
            assert o2.status == 0
            d2, _ = timed2([], 3, 1)
            others[name] = {"prompt_tokens": int(ids2.numel()), "batch": len(cu2) - 1, "steps": k2,
                            "ttft_ms": round(ms2, 4), "tokens_per_s": round(ids2.numel() / (ms2 * 1e-3), 1),
                            "dense_ttft_ms": round(d2, 4), "pruned_vs_dense_speedup": round(d2 / ms2, 3),
                            "tokens_per_layer_stage": sorted(set(o2.n_tokens), reverse=True)}
            if m2 is not model:
                m2.close()
            del ids2, o2
            torch.cuda.empty_cache()

    # ---- the CPU checker, as it stands, timed on this machine's host cores (rank 0, N=1): the whole
    # pruned prefill of the same prompt with the same weights -- embedding, all layers with its own
    # scoring, selection and compaction, final norm, LM head -- in its fp32 variant
    cpu = None
    if want_cpu:
        from oracle import lazyllm_oracle as O
        sd = shape.as_dict()
        t0 = time.perf_counter()
        ref = O.prefill(sd, host_bits, inp["token_ids"], sched, dtype=np.float32, embed_scale=inp["embed_scale"],
                        n_layers=(cpu_layers or None), gemm8=f8)
        t_cpu = time.perf_counter() - t0
        counts = B.lazyllm_keep_counts(n_tokens, shape.n_layers, sched)
        if cpu_layers:
            est_total = t_cpu * sum(counts) / sum(counts[:cpu_layers])
            sample = ("the first %d of %d layers of the pruned prefill (fp32 variant) took %.1f s; scaled by "
                      "token-layers (%d of %d) to the whole call" % (cpu_layers, shape.n_layers, t_cpu, sum(counts),
                                                                      sum(counts[:cpu_layers])))
        else:
            est_total = t_cpu
            sample = ("whole pruned prefill of the same %d-token prompt, all %d layers, the checker's own selections, "
                      "fp32 variant (numpy): %.1f s" % (n_tokens, shape.n_layers, t_cpu))
            same = int(np.argmax(ref.logits)) == int(torch.argmax(out.logits[0]).item())
            sample += "; first token %s the GPU's" % ("equals" if same else "differs from")
        try:
            cores = len(os.sched_getaffinity(0))
        except AttributeError:
            cores = os.cpu_count()
        env_threads = os.environ.get("OMP_NUM_THREADS")
        if env_threads:
            cores = min(cores, int(env_threads))
        cpu = {"value": round(n_tokens / est_total, 2), "unit": "tokens/s", "cores": cores, "kind": "oracle",
               "dtype": "f32", "seconds": round(t_cpu, 2), "sample": sample}

    line = {
        "metric": "pruned-prefill TTFT (ms) + prompt tokens/s, 7B shape, 3376-token prompt"
                  + (" [8-bit projections variant: not the headline arithmetic]" if f8 else ""),
        "value": round(n_tokens / (ms * 1e-3), 1), "unit": "tokens/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "fp8_e4m3 projections (weights and activations, fp32 accumulation), bf16 elsewhere" if f8 else "bf16",
        "data": "synthetic",
        "inputs": {"weight_seed": wl.weight_seed, "prompt_seed": wl.prompt_seed,
                   "weights_checksum": wsum, "token_ids_checksum": ids_sum},
        "config": {"workload": wl.name,
                   "shape": "%d layers, d %d, %dx%d heads (%d K,V heads), ffn %d, vocab %d" % (
                       shape.n_layers, shape.d_model, shape.n_heads, shape.head_dim, shape.kv_heads, shape.d_ffn,
                       shape.vocab),
                   "prompt_tokens": n_tokens, "batch": len(cu) - 1,
                   "keep_schedule_permille_of_survivors": sched,
                   "tokens_per_layer_stage": sorted(set(out.n_tokens), reverse=True),
                   **({"prefill_flags": args.prefill_flags} if args.prefill_flags else {})},
        "ttft_ms": round(ms, 4), "ttft_ms_median": round(ttft_median, 4), "ttft_ms_min": round(ttft_min, 4),
        "ttft_ms_host_synced_median": round(synced[len(synced) // 2], 4),
        "ttft_runs": len(each), "dense_ttft_ms": None if dense_ms is None else round(dense_ms, 4),
        "pruned_vs_dense_speedup": None if dense_ms is None else round(dense_ms / ms, 3),
        "whole_call_tflops": round(total_flops / (ms * 1e-3) / 1e12, 1),
        "whole_call_mfma_frac": None if f8 else round(total_flops / (ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4),
        "profiled_ms_per_step": round(total_prof_ms, 4),
        "roofline": roofline, "cpu_baseline": cpu, "other_workloads": others,
        "scoring_cost_ms": score_cost, "breakdown": breakdown,
    }
    print(json.dumps(line))
    model.close()
    return 0


if __name__ == "__main__":
    sys.exit(main())
