#!/usr/bin/env python3
"""Benchmark of the ANPD verification path on one MI355X.

A "step" is one pass of the whole hot path: draft k tokens from the multi-level
N-gram table (host), one verification forward over the k+1-row window against
the paged KV cache (HIP kernels), greedy argmax, longest-prefix acceptance, KV
commit / rollback, table update (paper, Algorithm 1, one loop iteration).

Prints ONE JSON line.  ``value`` is verification steps per second with the
weights, the cache and the prompt already resident in HBM.  The line also
carries accepted tokens/s, the ANPD / greedy speed-up, the roofline of the
dominant kernel (the small-M weight-streaming GEMM) and the CPU oracle timed
on this machine's host cores.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0  # MI355X published peak


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def timed_steps(fn, n, torch):
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(n):
        fn()
    torch.cuda.synchronize()
    return time.perf_counter() - t0


def sweep(args, torch, B, synth) -> int:
    """Step time over L x M (seeded N(0,1) cache, random window ids): the question whether a window of
    k + 1 rows costs what one row costs (paper, Section 3.1, "Parallel Decoding"), and whether paging costs
    bandwidth.  One JSON line per (L, page order) on stdout, a table on stderr."""
    wl = synth.WORKLOADS[args.workload]
    shape = wl["shape"]
    path = {"auto": B.GEMM_AUTO, "dot": B.GEMM_DOT, "mfma": B.GEMM_MFMA, "launches": B.GEMM_MFMA_LAUNCHES}[args.gemm_path]
    lengths = [128] if args.workload == "tiny" else [512, 1024, 2048, 4096]
    rows = [1, 2, 4, 6, 8, 9, 16, 17]
    cap = max(lengths) + 64
    weights = synth.make_weights(shape, wl["seed"], device="cuda")
    model = B.Model(shape, weights, max_window=32, max_positions=cap, gemm_path=path)
    kv = B.KVCache(model, cap)
    for layer in range(shape.n_layers):
        k, v = synth.kv_fill(shape, 7, layer, max(lengths), device="cuda")
        kv.write(layer, 0, k.float().contiguous(), v.float().contiguous())
    torch.cuda.synchronize()
    weight_bytes = 2 * shape.n_params_streamed if shape.dtype == "bf16" else 4 * shape.n_params_streamed
    n_pages = kv.num_pages
    perm = sorted(range(n_pages), key=lambda i: synth.splitmix64(0xABCD + i))
    log("%-9s %-6s" % ("pages", "L") + "".join("  M=%-2d ms (GB/s)" % m for m in rows))
    for order_name, order in (("identity", list(range(n_pages))), ("permuted", perm)):
        kv.truncate(0)
        kv.set_page_order(order)
        for layer in range(shape.n_layers):
            k, v = synth.kv_fill(shape, 7, layer, max(lengths), device="cuda")
            kv.write(layer, 0, k.float().contiguous(), v.float().contiguous())
        for L in lengths:
            line, rec = "%-9s %-6d" % (order_name, L), {}
            for M in rows:
                win = synth.random_tokens(shape.vocab, M, 11 + M)

                def step():
                    kv.truncate(L)
                    B.verify(model, kv, win, B.APPEND)

                for _ in range(max(3, args.warmup // 4)):
                    step()
                n = max(10, args.steps // 4)
                dt = timed_steps(step, n, torch)
                ms = 1e3 * dt / n
                gbs = (weight_bytes + shape.kv_bytes_per_token * L) / (ms * 1e-3) / 1e9
                line += "  %6.3f (%4.0f)" % (ms, gbs)
                rec[str(M)] = round(ms, 4)
            log(line)
            print(json.dumps({"sweep": args.workload, "pages": order_name, "L": L, "ms_per_step_by_rows": rec,
                              "gemm_path": args.gemm_path}))
    kv.close()
    model.close()
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="llama7b", choices=["tiny", "llama7b", "llama13b", "long7b", "glm6b"])
    ap.add_argument("--gemm-path", default="auto", choices=["auto", "dot", "mfma", "launches"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-steps", type=int, default=2)
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run a plain 1 GiB elementwise copy five times (reference for HBM traffic counters)")
    ap.add_argument("--sweep", action="store_true",
                    help="kernel sweep instead of the headline run: step time over cache length x window rows on a "
                         "seeded cache, with the identity page table and a seeded permutation; prints a table")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no sharding, no collectives); use --gpus 1",
              file=sys.stderr)
        return 2

    import torch
    from paper_2404_08698_amd import binding as B
    from paper_2404_08698_amd import synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    B.lib()  # fail loudly if the HIP library is missing

    if args.copy_calibration:
        # a kernel of known traffic: reads 1 GiB, writes 1 GiB (256 Mi floats, y = x * 1)
        cx = torch.ones(1 << 28, dtype=torch.float32, device="cuda")
        cy = torch.empty_like(cx)
        for _ in range(5):
            torch.mul(cx, 1.0, out=cy)
        torch.cuda.synchronize()
        del cx, cy

    if args.sweep:
        return sweep(args, torch, B, synth)

    wl = synth.WORKLOADS[args.workload]
    shape = wl["shape"]
    K, n_min, n_max = wl["k"], wl["n_min"], wl["n_max"]
    prompt = synth.workload_prompt(args.workload)
    path = {"auto": B.GEMM_AUTO, "dot": B.GEMM_DOT, "mfma": B.GEMM_MFMA, "launches": B.GEMM_MFMA_LAUNCHES}[args.gemm_path]
    gen = wl["gen"]
    max_tokens = len(prompt) + gen + 2 * (K + 2) + 32

    t0 = time.perf_counter()
    weights = synth.make_weights(shape, wl["seed"], device="cuda")
    torch.cuda.synchronize()
    log("weights generated on the GPU in %.1f s" % (time.perf_counter() - t0))
    model = B.Model(shape, weights, max_window=32, max_positions=max_tokens, gemm_path=path)
    kv = B.KVCache(model, max_tokens)
    table = B.NgramTable(n_min, n_max, shape.vocab)

    # ---- prompt (outside the timed steps): LLM(prompt) in one pass on the matrix cores, timed once
    # warm next to the same prompt appended through the verification step in 32-row windows
    pws = torch.empty(max(B.prefill_workspace_bytes(model, len(prompt)), 256), dtype=torch.uint8, device="cuda")
    t0 = time.perf_counter()
    c_win = B.prefill_windows(model, kv, prompt)
    torch.cuda.synchronize()
    kv.truncate(0)
    t0 = time.perf_counter()
    B.prefill_windows(model, kv, prompt)
    torch.cuda.synchronize()
    t_win = time.perf_counter() - t0
    kv.truncate(0)
    c0 = B.prefill(model, kv, prompt, workspace=pws)
    kv.truncate(0)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    c0 = B.prefill(model, kv, prompt, workspace=pws)
    torch.cuda.synchronize()
    t_one = time.perf_counter() - t0
    del pws
    # every weight meets every row twice (hi and lo term of the split activation)
    prompt_flop = 2.0 * 2.0 * shape.n_params_streamed * len(prompt)
    prompt_info = {"tokens": len(prompt), "one_pass_ms": round(1e3 * t_one, 3), "windowed_ms": round(1e3 * t_win, 3),
                   "one_pass_mfma_tflops": round(prompt_flop / t_one / 1e12, 1),
                   "one_pass_frac_of_bf16_mfma_peak": round(prompt_flop / t_one / 2.5e15, 4),
                   "same_first_token": c0 == c_win}
    log("prompt of %d tokens: one pass %.2f ms, in windows %.2f ms" % (len(prompt), 1e3 * t_one, 1e3 * t_win))
    L0 = kv.length

    # Every region below generates at most `gen` tokens past the prompt and then starts
    # over from the prefilled cache, so the cache length stays the workload's.
    def restart():
        kv.truncate(L0)
        table.reset()
        table.update(prompt)

    # ---- plain greedy decoding on the GPU: windows of one row
    cont = [c0]
    g = {"c": c0, "n": 0}

    def greedy_step():
        if g["n"] >= gen + K + 2:
            kv.truncate(L0)
            g.update(c=c0, n=0)
        _, nxt = B.verify(model, kv, [g["c"]], B.VERIFY)
        g["c"] = nxt
        g["n"] += 1
        if len(cont) <= gen + K + 2:
            cont.append(nxt)

    for _ in range(gen + K + 2):     # also records the greedy continuation (untimed warm-up)
        greedy_step()
    kv.truncate(L0)
    g.update(c=c0, n=0)
    dt_g = timed_steps(greedy_step, args.steps, torch)
    greedy_tokens_per_s = args.steps / dt_g
    log("greedy: %.1f tokens/s (%.3f ms/step)" % (greedy_tokens_per_s, 1e3 * dt_g / args.steps))

    # ---- ANPD steps at the workload's window size.  Every step updates and queries the N-gram
    # table (the host rows of the path).  A random-weight model does not reuse its prompt, so the
    # table rarely answers; the window is then filled to K drafts from a script that follows the
    # true greedy continuation for a seeded number of tokens and is wrong afterwards, which makes
    # verification, acceptance and rollback run at a hit ratio inside the paper's range.
    st = {"i": 0, "tokens": 0, "acc": 0, "prop": 0, "n": 0, "len_sum": 0, "mln": 0}

    def scripted(i, n):
        right = synth.splitmix64(977 + n) % (K + 1)
        if synth.splitmix64(55 + n) % 100 < 35:
            right = 0
        return cont[i + 1:i + 1 + right] + [(t + 1) % shape.vocab for t in cont[i + 1 + right:i + 1 + K]], right

    def anpd_step():
        if st["i"] + K + 1 >= gen:
            restart()
            st["i"] = 0
        i = st["i"]
        table.update([cont[i]])
        drafts, _ = table.propose(K)
        if len(drafts) == K:
            st["mln"] += 1
            right = None
        else:
            drafts, right = scripted(i, st["n"])
        st["len_sum"] += L0 + i
        a, nxt = B.verify(model, kv, [cont[i]] + drafts, B.VERIFY)
        if nxt != cont[i + 1 + a] or (right is not None and a != right):
            raise RuntimeError("verification diverged from greedy decoding at token %d" % i)
        if a:
            table.update(drafts[:a])
        st["i"] = i + 1 + a
        st["tokens"] += 1 + a
        st["acc"] += a
        st["prop"] += len(drafts)
        st["n"] += 1

    restart()
    for _ in range(args.warmup):
        anpd_step()
    st.update(tokens=0, acc=0, prop=0, len_sum=0, mln=0)
    dt = timed_steps(anpd_step, args.steps, torch)
    steps_per_s = args.steps / dt
    ms_per_step = 1e3 * dt / args.steps
    anpd_tokens_per_s = st["tokens"] / dt
    alpha = st["acc"] / st["prop"] if st["prop"] else 0.0
    kbar = st["prop"] / args.steps
    L_mid = st["len_sum"] // args.steps
    tokens_per_step = st["tokens"] / args.steps
    mln_windows = st["mln"]
    log("ANPD (window %d rows): %.1f steps/s, %.3f ms/step, alpha %.3f, tokens/step %.2f" %
        (K + 1, steps_per_s, ms_per_step, alpha, tokens_per_step))

    # ---- the same steps again with per-kernel events on the launch stream (roofline leg)
    model.profile(True)
    dt_ev = timed_steps(anpd_step, args.steps, torch)
    prof = model.profile_read()
    model.profile(False)
    gemm_cats = [c_ for c_ in B.PROF_CATEGORIES if c_.startswith("gemm")]
    el = 2 if shape.dtype == "bf16" else 4
    weight_bytes = shape.n_params_streamed * el
    kv_bytes = shape.kv_bytes_per_token * L_mid
    kernels = {c_: round(prof["ms"][c_] / max(1, prof["steps"]), 4) for c_ in B.PROF_CATEGORIES}
    log("per-step kernel time by category (ms, events):", kernels)
    if prof["ms"]["step"] > 0:
        # the step ran as one persistent kernel: that kernel is the dominant one
        dom_ms = prof["ms"]["step"] / max(1, prof["intervals"]["step"])
        dom_bytes = weight_bytes + kv_bytes
        dom_name = "verify_mega_kernel (the whole step in one launch: weights once + KV once)"
        dom_launches = 1
    else:
        dom_ms = sum(prof["ms"][c_] for c_ in gemm_cats) / max(1, prof["steps"])
        dom_launches = sum(prof["intervals"][c_] for c_ in gemm_cats) / max(1, prof["steps"])
        dom_bytes = weight_bytes
        dom_name = "small-M weight-streaming GEMM (all %d launches of a step)" % round(dom_launches)
    dom_gbs = dom_bytes / (dom_ms * 1e-3) / 1e9 if dom_ms > 0 else 0.0
    # HBM bytes per launch of the persistent kernel from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE
    # (profiles/verify_step_llama7b_hbm_traffic.md): 13 773 MB read + 25 MB written
    traffic = {"llama7b": 13.773e9 + 0.025e9}.get(args.workload) if shape.dtype == "bf16" else None

    # ---- ANPD driven by the N-gram table alone (Algorithm 1 as printed), reported beside it
    ms_ = {"c": c0, "proposed": 0, "accepted": 0, "tokens": 0, "since": 0}

    def mln_step():
        if ms_["since"] >= gen:
            restart()
            ms_.update(c=c0, since=0)
        table.update([ms_["c"]])
        drafts, _ = table.propose(K)
        a, nxt = B.verify(model, kv, [ms_["c"]] + drafts, B.VERIFY)
        if a:
            table.update(drafts[:a])
        ms_["proposed"] += len(drafts)
        ms_["accepted"] += a
        ms_["tokens"] += 1 + a
        ms_["since"] += 1 + a
        ms_["c"] = nxt

    restart()
    dt_m = timed_steps(mln_step, args.steps, torch)
    mln_only = {"steps": args.steps, "steps_per_s": round(args.steps / dt_m, 2),
                "accepted_tokens_per_s": round(ms_["tokens"] / dt_m, 2),
                "mean_draft_length": round(ms_["proposed"] / args.steps, 3),
                "alpha": round(ms_["accepted"] / ms_["proposed"], 4) if ms_["proposed"] else 0.0,
                "speedup_vs_gpu_greedy": round(ms_["tokens"] / dt_m / greedy_tokens_per_s, 3)}
    log("N-gram drafts only:", mln_only)

    step_bytes = weight_bytes + kv_bytes
    out = {
        "metric": "verify steps/sec (LLaMA-7B shape bf16, ANPD window k+1 = %d)" % (K + 1)
        if args.workload == "llama7b" else "verify steps/sec (%s, window k+1 = %d)" % (args.workload, K + 1),
        "value": round(steps_per_s, 2),
        "unit": "steps/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": shape.dtype, "data": "synthetic",
        "config": {"workload": args.workload, "prompt_tokens": len(prompt), "kv_length_mid": L_mid,
                   "window_rows": K + 1, "mln_levels": [n_min, n_max], "gemm_path": args.gemm_path,
                   "weights": "seeded ~N(0,0.02)", "stream": "copy-heavy order-2 Markov",
                   "drafts": "N-gram table updated and queried every step; windows it cannot fill are "
                             "completed to k drafts by a script following the greedy continuation "
                             "for a seeded number of tokens"},
        "accepted_tokens_per_s": round(anpd_tokens_per_s, 2),
        "tokens_per_step": round(tokens_per_step, 4),
        "draft_hit_ratio": round(alpha, 4), "mean_draft_length": round(kbar, 3),
        "gpu_greedy_tokens_per_s": round(greedy_tokens_per_s, 2),
        "speedup_vs_gpu_greedy": round(anpd_tokens_per_s / greedy_tokens_per_s, 3),
        "bound_alpha_k_plus_1": round(alpha * kbar + 1, 3),
        "windows_drafted_by_ngram_table": mln_windows,
        "ngram_drafts_only": mln_only,
        "step_hbm_frac_of_peak": round(step_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
        "step_algorithmic_bytes": step_bytes,
        "ms_per_step_with_events": round(1e3 * dt_ev / args.steps, 4),
        "kernel_ms_per_step": kernels,
        "prompt": prompt_info,
        "paper_context": "paper reports end-to-end speed-ups of 1.95x-3.67x on RTX-3090 (Table 1); not comparable",
        "roofline": {"bound": "hbm", "kernel": dom_name,
                     "achieved": round(dom_gbs, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(dom_gbs / HBM_PEAK_GBS, 4), "traffic": traffic,
                     "algorithmic_bytes_per_launch": dom_bytes / dom_launches,
                     "avg_launch_us": round(1e3 * dom_ms / dom_launches, 3),
                     # the weight access pattern alone, non-temporal loads, steady state
                     # (profiles/weight_stream_probe.md; 5700-6300 in bursts of the size of one GEMM phase)
                     "measured_read_ceiling_gbs": 7100.0},
    }

    # ---- CPU oracle on this machine's host cores: a bounded sample of the same workload
    if not args.no_cpu_baseline:
        from oracle import decoder as od
        t0 = time.perf_counter()
        w_host = {k_: ([t.cpu() for t in v] if isinstance(v, list) else v.cpu()) for k_, v in weights.items()}
        Ls = min(len(prompt), 512)
        dec = od.Decoder(shape, w_host, Ls + 2 * (K + 1) * args.cpu_steps + 8)
        for layer in range(shape.n_layers):
            kk, vv = synth.kv_fill(shape, 99, layer, Ls)
            dec.kv_load(layer, 0, kk.float().numpy(), vv.float().numpy())
        dec.set_length(Ls)
        log("oracle set-up (weights to host, seeded cache): %.1f s" % (time.perf_counter() - t0))
        win = synth.random_tokens(shape.vocab, K + 1, 123)
        t0 = time.perf_counter()
        for _ in range(args.cpu_steps):
            dec.predict(win)
        dt_c = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": round(args.cpu_steps / dt_c, 4), "unit": "steps/s",
                               "cores": od.num_threads(), "kind": "oracle",
                               "sample": "%d verify steps of %d rows over a seeded %d-token cache, fp64 oracle" %
                                         (args.cpu_steps, K + 1, Ls)}
        log("oracle: %.3f steps/s on %d threads" % (args.cpu_steps / dt_c, od.num_threads()))
    else:
        out["cpu_baseline"] = None

    print(json.dumps(out), flush=True)
    kv.close()
    model.close()
    table.close()
    return 0


if __name__ == "__main__":
    sys.exit(main())
