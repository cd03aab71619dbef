"""Benchmark of the constrained-decoding mask hot path on one MI355X.

A step = one pass of the whole per-step path over one batch: batched mask
fill (kernel b) + in-place -inf apply (kernel c) for the serving workload
(batch 128, vocabulary 151936, 128 distinct string-heavy schema grammars,
bf16 logits), with everything it reads resident in device memory: the mask
caches, the logits and the matcher states (xgm_batch_*), done in one launch
(xgm_batch_fill_and_apply: mask written, logits masked).  Timed beside it: the
same step as two calls (fill, then apply), both forms from host-side matcher
states (stacks packed on the host and uploaded every step), and the kernels
that accept a token per row on the device.  The mask caches (kernel a) are
built during set-up and their throughput is reported too.  Prints ONE JSON
line on stdout.
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

HBM_PEAK_GBS = 8000.0                      # MI355X HBM3E, published
# HBM bytes per launch from the FETCH_SIZE / WRITE_SIZE counter runs summarised in
# profiles/serving_step_counters.txt (scaled by what the counters read for a plain copy of known size).
# Set to None whenever a kernel changes after the counters were taken.
TRAFFIC_FILL_BYTES = 13.9e6
TRAFFIC_APPLY_BYTES = 33.9e6
TRAFFIC_FUSED_BYTES = 54.3e6


def log(*a):
    print("[bench]", *a, file=sys.stderr, flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=1000)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--rows", type=int, default=128, help="batch size (default: the serving workload's 128)")
    ap.add_argument("--vocab", type=int, default=151936)
    ap.add_argument("--pool", type=int, default=16, help="number of pre-walked state sets cycled through")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-build-bench", action="store_true")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this path runs on one GPU (rows and vocabulary slices are independent; "
              "nothing is exchanged between devices). Run with --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import paper_2411_15100_amd as xgm
    import synth_inputs as si
    from paper_2411_15100_amd import workloads as wl

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    stream = wl.current_stream()
    t_setup = time.time()
    work = wl.ServingWorkload(n_rows=args.rows, vocab_size=args.vocab, pool=args.pool, log=log)
    B, V, W = work.B, work.V, work.W
    log(f"set-up done in {time.time() - t_setup:.1f} s; context-dependent fraction at the stack tops "
        f"{work.uncertain_fraction:.3f}")

    # ---- warm-up, then the timed region: exactly K steps between two synchronisations
    # (the step is the one-launch form, xgm_batch_fill_and_apply: mask written, logits masked)
    for k in range(args.warmup):
        work.fused_step_device(k, stream)
    torch.cuda.synchronize()
    work.refresh_logits()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(args.steps):
        work.fused_step_device(k, stream)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    overflow = xgm.overflow_total()

    # ---- the same K steps as two calls (fill, then apply), states resident on the device
    work.refresh_logits()
    torch.cuda.synchronize()
    t0t = time.perf_counter()
    for k in range(args.steps):
        work.step_device(k, stream)
    torch.cuda.synchronize()
    two_call_us = (time.perf_counter() - t0t) * 1e6 / args.steps

    # ---- the same K steps from host-side matcher states (pack + upload over PCIe every step)
    for k in range(min(args.warmup, 10)):
        work.step(k, stream)
    work.refresh_logits()
    torch.cuda.synchronize()
    t0h = time.perf_counter()
    for k in range(args.steps):
        work.step(k, stream)
    torch.cuda.synchronize()
    host_state_us = (time.perf_counter() - t0h) * 1e6 / args.steps

    # ---- the same K steps again with HIP events around each kernel (same stream)
    work.refresh_logits()
    torch.cuda.synchronize()
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(args.steps)]
    for k in range(args.steps):
        ev[k][0].record()
        work.fill_device(k, stream)
        ev[k][1].record()
        work.apply(k, stream)
        ev[k][2].record()
    torch.cuda.synchronize()
    fill_us = np.array([e[0].elapsed_time(e[1]) for e in ev]) * 1e3
    apply_us = np.array([e[1].elapsed_time(e[2]) for e in ev]) * 1e3

    # ---- the one-launch step with HIP events around each call (same stream)
    work.refresh_logits()
    torch.cuda.synchronize()
    evf = [[torch.cuda.Event(enable_timing=True) for _ in range(2)] for _ in range(args.steps)]
    for k in range(args.steps):
        evf[k][0].record()
        work.fused_step_device(k, stream)
        evf[k][1].record()
    torch.cuda.synchronize()
    fused_call_us = np.array([e[0].elapsed_time(e[1]) for e in evf]) * 1e3
    work.refresh_logits()
    torch.cuda.synchronize()
    t0f = time.perf_counter()
    for k in range(args.steps):
        work.fused_step(k, stream)
    torch.cuda.synchronize()
    host_state_fused_us = (time.perf_counter() - t0f) * 1e6 / args.steps

    # ---- accepting one token per row on the device (accept kernel, then plan and two-byte tables in one launch), then one step back
    accept_us = []
    w0 = work.sets[0]
    work.fill(0, stream)
    torch.cuda.synchronize()
    allowed0 = wl.unpack_rows(work.d_mask.cpu().numpy(), V)
    allowed0[:, work.vocab.stop_ids] = False
    picks = si.pick_tokens(np.random.Generator(np.random.PCG64(1)), allowed0, w0.info.structural, w0.info.is_stop, 0.35)
    d_picks = torch.tensor(picks, dtype=torch.int32, device="cuda")
    d_back = torch.tensor((picks >= 0).astype(np.int32), dtype=torch.int32, device="cuda")
    accept_batch = xgm.DeviceBatch(w0.matchers, history=1, stream=stream)
    for k in range(40):
        a0, a1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a0.record()
        accept_batch.accept_tokens(d_picks.data_ptr(), stream)
        a1.record()
        accept_batch.rollback(d_back.data_ptr(), stream)
        torch.cuda.synchronize()
        if k >= 8:
            accept_us.append(a0.elapsed_time(a1) * 1e3)
    assert not accept_batch.status(stream).any()
    del accept_batch

    # ---- what this box writes at best: a plain fill of the same rotating logits buffers
    for t in work.logits:
        t.fill_(0.5)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    n_fill = 64
    e0.record()
    for k in range(n_fill):
        work.logits[k % len(work.logits)].fill_(0.25)
    e1.record()
    torch.cuda.synchronize()
    plain_fill_us = e0.elapsed_time(e1) * 1e3 / n_fill
    plain_fill_gbs = 2.0 * B * V / (plain_fill_us * 1e-6) / 1e9
    # ... and a plain copy between them (read + write of 38.9 MB each), the streaming rate of this machine
    e0.record()
    for k in range(n_fill):
        work.logits[k % len(work.logits)].copy_(work.logits[(k + 3) % len(work.logits)])
    e1.record()
    torch.cuda.synchronize()
    plain_copy_us = e0.elapsed_time(e1) * 1e3 / n_fill
    plain_copy_gbs = 2.0 * 2.0 * B * V / (plain_copy_us * 1e-6) / 1e9
    work.refresh_logits()

    # ---- the fill kernel by itself: events inside the library around its two launches
    up_us, fk_us = [], []
    for k in range(args.steps):
        a, b_ = xgm.debug_fill_timed(work.sets[k % len(work.sets)].batch, work.d_mask.data_ptr(), stream)
        up_us.append(a)
        fk_us.append(b_)
    up_us, fk_us = np.array(up_us), np.array(fk_us)

    # ---- algorithmic work per launch (averaged over the state sets in use)
    n_sets = len(work.sets)
    rejected, acc_words, unc_tokens, steps_count, sector_bytes = [], [], [], [], []
    for k in range(n_sets):
        work.fill(k, stream)
        torch.cuda.synchronize()
        words = work.d_mask.cpu().numpy()
        allowed = int(np.unpackbits(words.view(np.uint8)).sum())
        rejected.append(B * V - allowed)
        # the same count at the memory's granularity: a 64-byte piece of a bf16 row (32 logits = one mask word)
        # with no allowed logit is written, one with allowed and rejected logits is read and written
        mw = words.view(np.uint32)[:, : V // 32]
        sector_bytes.append(64.0 * int((mw == 0).sum()) + 128.0 * int(((mw != 0) & (mw != 0xFFFFFFFF)).sum()))
        w = work.sets[k]
        n_stacks = sum(m.num_stacks() for m in w.matchers)
        acc_words.append(n_stacks * W)
        unc_tokens.append(sum(c.num_uncertain(m.stack(s)[-1]) for m, c in zip(w.matchers, work.caches)
                              for s in range(m.num_stacks())))
        steps_count.append(xgm.debug_fill_count_steps(w.batch, work.d_mask.data_ptr(), stream))
    # apply: the mask words are read once, a rejected bf16 logit is 2 bytes written, nothing else is needed
    apply_bytes = 4.0 * B * W + 2.0 * float(np.mean(rejected))
    # fill: accepted words of every stack top read, list entries of every stack top read, mask words written
    fill_bytes = 4.0 * float(np.mean(acc_words)) + 4.0 * float(np.mean(unc_tokens)) + 4.0 * B * W
    fill_us_avg, apply_us_avg = float(fill_us.mean()), float(apply_us.mean())
    # the one-launch step: what fill moves plus the rejected logits (the mask is not read again)
    fused_bytes = fill_bytes + 2.0 * float(np.mean(rejected))
    fused_us_avg = float(fused_call_us.mean())
    roof_fused = {"kernel": "fill_kernel<false, 2> (mask fill and -inf apply in one launch, device-resident states)",
                  "bound": "hbm", "kernel_us": fused_us_avg, "achieved": fused_bytes / (fused_us_avg * 1e-6) / 1e9,
                  "peak": HBM_PEAK_GBS, "unit": "GB/s", "traffic": TRAFFIC_FUSED_BYTES, "bytes_per_launch": fused_bytes,
                  "bytes_per_launch_in_64_byte_pieces": fill_bytes + float(np.mean(sector_bytes)),
                  "note": "the launch lasts as long as its slowest workgroup's token walks plus the drain of the "
                          "logits stores; the byte count is what the method must move"}
    roof_fused["frac"] = roof_fused["achieved"] / HBM_PEAK_GBS
    roof_apply = {"kernel": "apply_kernel<2>", "bound": "hbm", "achieved": apply_bytes / (apply_us_avg * 1e-6) / 1e9,
                  "peak": HBM_PEAK_GBS, "unit": "GB/s", "traffic": TRAFFIC_APPLY_BYTES, "bytes_per_launch": apply_bytes,
                  "read_modify_write_bytes_per_launch": 2.0 * 2.0 * B * V + 4.0 * B * W,
                  "bytes_per_launch_in_64_byte_pieces": 4.0 * B * W + float(np.mean(sector_bytes)),
                  "achieved_on_64_byte_pieces_GB/s": (4.0 * B * W + float(np.mean(sector_bytes))) / (apply_us_avg * 1e-6) / 1e9,
                  "plain_fill_of_the_same_buffers": {"us": plain_fill_us, "GB/s": plain_fill_gbs},
                  "plain_copy_between_the_same_buffers": {"us": plain_copy_us, "GB/s": plain_copy_gbs}}
    roof_apply["frac"] = roof_apply["achieved"] / HBM_PEAK_GBS
    auto_steps = float(np.mean(steps_count))
    fill_kernel_us = fill_us_avg  # HIP events around the launch from device-resident states, on its stream
    roof_fill = {"kernel": "fill_kernel<false, 0> (device-resident states)", "bound": "hbm", "kernel_us": fill_kernel_us,
                 "achieved": fill_bytes / (fill_kernel_us * 1e-6) / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                 "traffic": TRAFFIC_FILL_BYTES, "bytes_per_launch": fill_bytes,
                 "list_entries_per_launch": float(np.mean(unc_tokens)),
                 "automaton_steps_per_launch": auto_steps,
                 "automaton_steps_per_s": auto_steps / (fill_kernel_us * 1e-6),
                 "note": "latency-bound by nature: a few dependent memory rounds per workgroup and a tail of "
                         "token walks; the byte count is what the method must move, not what limits it"}
    roof_fill["frac"] = roof_fill["achieved"] / HBM_PEAK_GBS
    step_bytes = fill_bytes + apply_bytes
    roof_step = {"bound": "hbm", "achieved": step_bytes / (two_call_us * 1e-6) / 1e9, "peak": HBM_PEAK_GBS,
                 "unit": "GB/s", "bytes_per_step": step_bytes, "note": "the two-call step: fill, then apply"}
    roof_step["frac"] = roof_step["achieved"] / HBM_PEAK_GBS

    # ---- cache build throughput (kernel a), generic JSON and the C/SQL-like grammar at V = 128256
    def mean_steps_per_pair(g, toks, rng, n=6000):
        """Automaton steps of the classifying walk on a seeded sample of (node, token) pairs (the same
        walk compiled for the host); a walk that fails on its first byte counts as zero steps: the
        kernel settles such a pair with its first-byte test, without walking."""
        total = 0
        nodes = rng.integers(0, g.num_nodes, size=n)
        ids = rng.integers(0, len(toks), size=n)
        for node, i in zip(nodes, ids):
            t = toks[int(i)]
            if not t:
                continue
            rc, steps = g.debug_walk_host([int(node)], t, True, with_steps=True)
            total += 0 if (rc == 0 and steps <= 1) else steps
        return total / n

    cache_build = None
    if not args.no_build_bench:
        v128 = si.make_vocab("bpe", 128256, 0)
        xv128 = wl.make_xgm_vocab(v128)
        toks128 = v128.tokens()
        lds_rate = xgm.debug_lds_lookup_rate(stream)
        cache_build = {"lds_dependent_lookups_per_s": lds_rate,
                       "note": "steps_per_s = pairs_per_s x the mean automaton steps per pair of a seeded sample; a "
                               "step is 3 to 5 dependent table lookups (header, follow set, class, shape, target); "
                               "the ceiling is a chain of dependent LDS reads with every wave slot busy"}
        for name, text in (("json", si.JSON_GRAMMAR), ("csql", si.CSQL_GRAMMAR)):
            g = xgm.Grammar(text, "root")
            best = whole = None
            for _ in range(3):
                c = xgm.Cache(g, xv128, stream)
                best = c.build_kernel_seconds if best is None else min(best, c.build_kernel_seconds)
                whole = c.build_seconds if whole is None else min(whole, c.build_seconds)
                hostc = c.host_classified
                del c
            sps = mean_steps_per_pair(g, toks128, np.random.Generator(np.random.PCG64(11)))
            cache_build[name] = {"positions": g.num_nodes, "tokens": 128256, "classify_kernel_ms": best * 1e3,
                                 "pairs_per_s": g.num_nodes * 128256 / best, "steps_per_pair": sps,
                                 "steps_per_s": sps * g.num_nodes * 128256 / best,
                                 "lookups_vs_ceiling": 4.0 * sps * g.num_nodes * 128256 / best / lds_rate,
                                 "whole_build_ms": whole * 1e3,
                                 "pairs_per_s_whole_build": g.num_nodes * 128256 / whole,
                                 "host_classified_pairs": hostc}
        toks_s = work.vocab.tokens()
        sps = float(np.mean([mean_steps_per_pair(work.grammars[k], toks_s, np.random.Generator(np.random.PCG64(12 + k)), 1500)
                             for k in (0, 31, 77, 127) if k < len(work.grammars)]))
        pps = work.build_pairs / max(work.build_kernel_seconds, 1e-12)
        cache_build["serving_set_up"] = {"pairs": work.build_pairs, "kernel_s": work.build_kernel_seconds,
                                         "pairs_per_s": pps, "steps_per_pair": sps, "steps_per_s": sps * pps,
                                         "lookups_vs_ceiling": 4.0 * sps * pps / lds_rate}
        nodes = sum(c.num_nodes for c in work.caches)
        kept = sum(c.num_accept_rows for c in work.caches)
        held = sum(c.device_bytes for c in work.caches)
        row_bytes = 4 * xgm.bitmask_words(work.V)
        cache_build["serving_storage"] = {"caches": len(work.caches), "nodes": nodes, "accepted_bitsets_kept": kept,
                                          "device_bytes": held,
                                          "accepted_bitset_bytes_saved": (nodes - kept) * row_bytes,
                                          "note": "the distinct accepted bitsets of a grammar's nodes are kept once each"}

    # ---- the oracle on the host cores, on a bounded sample of the same workload
    cpu_baseline = None
    if not args.no_cpu_baseline:
        import oracle
        toks = work.vocab.tokens()
        threads = oracle.default_threads()
        spent, checks, masks = 0.0, 0, 0
        budget_s = 15.0
        for k in range(n_sets):
            wk = work.sets[k]
            for b in range(B):
                og = oracle.Grammar(work.texts[b], "root")
                om = oracle.EarleyMatcher(og)
                for t in wk.history[b]:
                    assert om.advance(toks[t])
                tt = time.perf_counter()
                om.mask(work.vocab, threads)
                spent += time.perf_counter() - tt
                checks += V
                masks += 1
                if spent > budget_s:
                    break
            if spent > budget_s:
                break
        # one thread, a few masks of the first state set (the paper's brute-force row is a single-thread figure)
        t1s, n1 = 0.0, 0
        for b in range(min(B, 4)):
            om = oracle.EarleyMatcher(oracle.Grammar(work.texts[b], "root"))
            for t in work.sets[0].history[b]:
                assert om.advance(toks[t])
            tt = time.perf_counter()
            om.mask(work.vocab, 1)
            t1s += time.perf_counter() - tt
            n1 += 1
        cpu_model = "unknown"
        try:
            for line in open("/proc/cpuinfo"):
                if line.startswith("model name"):
                    cpu_model = line.split(":", 1)[1].strip()
                    break
        except OSError:
            pass
        cpu_baseline = {"value": checks / spent, "unit": "token checks/s", "cores": threads, "kind": "oracle",
                        "cpu_model": cpu_model, "host_cpus": os.cpu_count(),
                        "single_thread_us_per_mask": t1s / n1 * 1e6,
                        "sample": f"Earley brute-force masks for the first {masks} (state set, row) pairs of the pool, "
                                  f"in order ({checks} token checks, {spent:.1f} s of mask time)",
                        "us_per_mask": spent / (checks / V) * 1e6}

    prop = torch.cuda.get_device_properties(0)
    device = {"name": prop.name, "compute_units": prop.multi_processor_count,
              "memory_GB": round(prop.total_memory / 1e9, 1),
              "peaks_used": {"hbm_GB/s": HBM_PEAK_GBS},
              "measured_streaming_GB/s": {"fill": plain_fill_gbs, "copy": plain_copy_gbs}}
    out = {
        "metric": "vocab token checks/sec + per-step bitmask fill+apply \u00b5s (batch\u00d7vocab)",
        "value": B * V / (ms_per_step * 1e-3),
        "unit": "token checks/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "fill_plus_apply_us": ms_per_step * 1e3,
        "step_form": "one launch (xgm_batch_fill_and_apply); the two-call form is timed in two_call_path",
        "two_call_path": {"fill_plus_apply_us": two_call_us,
                          "note": "xgm_batch_fill_next_token_bitmask, then xgm_apply_token_bitmask_inplace"},
        "host_state_path": {"fill_plus_apply_us": host_state_us, "fused_fill_and_apply_us": host_state_fused_us,
                            "note": "matcher states kept on the host: stacks packed and uploaded over PCIe every step"},
        "device_accept_us": {"mean": float(np.mean(accept_us)), "p50": float(np.median(accept_us)),
                             "note": "one token per row accepted by the accept kernel, then the plan and the two-byte tables in one launch "
                                     "(events around the call); outside the fill+apply step"},
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "u32",
        "logits_dtype": "bf16 (only -inf patterns are stored; no floating-point arithmetic anywhere on the path)",
        "data": "synthetic",
        "config": {"workload": f"serving decode step: batch {B} x vocab {V}, {B} distinct string-heavy schema "
                               f"grammars, bf16 logits [{B},{V}], {n_sets} pre-walked state sets resident on the "
                               f"device, {len(work.logits)} rotating logits buffers",
                   "batch": B, "vocab": V,
                   "context_dependent_fraction_at_tops": work.uncertain_fraction,
                   "context_dependent_fraction_after_narrowing": work.uncertain_fraction_narrowed},
        "kernel_us": {"host_state_fill_kernel_mean": float(fk_us.mean()), "host_state_upload_kernel_mean": float(up_us.mean()),
                      "fused_call_mean": fused_us_avg, "fused_call_p50": float(np.median(fused_call_us)),
                      "fused_call_p99": float(np.percentile(fused_call_us, 99)),
                      "fill_mean": fill_us_avg, "fill_p50": float(np.median(fill_us)), "fill_p99": float(np.percentile(fill_us, 99)),
                      "apply_mean": apply_us_avg, "apply_p50": float(np.median(apply_us)), "apply_p99": float(np.percentile(apply_us, 99))},
        "roofline": roof_fused,
        "roofline_fill": roof_fill,
        "roofline_apply": roof_apply,
        "roofline_two_call_step": roof_step,
        "device": device,
        "walks_on_host_slow_path": int(overflow),
        "cache_build": cache_build,
        "cpu_baseline": cpu_baseline,
    }
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
