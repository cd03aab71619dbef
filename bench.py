"""Benchmark of the constrained-decoding mask hot path on one MI355X.

A step = one pass of the whole per-step path over one batch: batched mask
fill (kernel b) + in-place -inf apply (kernel c) for the serving workload
(batch 128, vocabulary 151936, 128 distinct string-heavy schema grammars,
bf16 logits), with everything it reads resident in device memory: the mask
caches, the logits and the matcher states (xgm_batch_*), done in one launch
(xgm_batch_fill_and_apply: mask written, logits masked).  The headline is the
median of several passes of exactly K such steps, each pass on freshly drawn
logits, after W untimed warm-up steps, between two synchronisations.  Timed beside it, in the same JSON line: the same step as
two calls (fill, then apply), both forms from host-side matcher states, the
whole decode cycle (accept the sampled tokens on the device, then fill and
apply), the smaller workloads (configs 1-3), the mask-cache build (config 4)
and the CPU oracle on a bounded sample.  Prints ONE JSON line on stdout.
"""

from __future__ import annotations

import argparse
import hashlib
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0                      # MI355X HBM3E, published
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "traffic.json")
KERNEL_SOURCES = ["kernels.hip", "kernels.hpp", "walk.hpp"]


def log(*a):
    print("[bench]", *a, file=sys.stderr, flush=True)


def kernel_source_hash() -> str:
    h = hashlib.sha256()
    for name in KERNEL_SOURCES:
        with open(os.path.join(ROOT, "paper_2411_15100_amd", "csrc", name), "rb") as f:
            h.update(f.read())
    return h.hexdigest()[:16]


def counter_traffic():
    """HBM bytes per launch from the FETCH_SIZE / WRITE_SIZE counter runs (written by
    `python -m paper_2411_15100_amd.profile_summary`), or {} if the kernels have changed since."""
    try:
        with open(TRAFFIC_FILE) as f:
            t = json.load(f)
    except (OSError, ValueError):
        return {}
    if t.get("kernel_source_hash") != kernel_source_hash():
        return {}
    return t.get("bytes_per_launch", {})


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=500)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--passes", type=int, default=5, help="passes of --steps steps each; the headline is their median")
    ap.add_argument("--rows", type=int, default=128, help="batch size (default: the serving workload's 128)")
    ap.add_argument("--vocab", type=int, default=151936)
    ap.add_argument("--pool", type=int, default=16, help="number of pre-walked state sets cycled through")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-build-bench", action="store_true")
    ap.add_argument("--no-configs", action="store_true", help="skip the smaller workloads (configs 1-3)")
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
    K, P = args.steps, max(1, args.passes)
    traffic = counter_traffic()

    def timed_passes(step, refresh, passes=P, warmup=0):
        """`passes` passes of exactly K steps, each between two synchronisations and after `warmup` untimed
        steps on freshly drawn logits: microseconds per step of each."""
        out = []
        for _ in range(passes):
            refresh()
            for k in range(warmup):
                step(k, stream)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for k in range(K):
                step(k, stream)
            torch.cuda.synchronize()
            out.append((time.perf_counter() - t0) * 1e6 / K)
        return out

    def event_us(step, refresh, passes=3):
        """Average duration of one launch by HIP events on the launch stream around K back-to-back launches
        (passes as in timed_passes: freshly drawn logits, then the warm-up steps)."""
        out = []
        for _ in range(passes):
            refresh()
            for k in range(args.warmup):
                step(k, stream)
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for k in range(K):
                step(k, stream)
            e1.record()
            torch.cuda.synchronize()
            out.append(e0.elapsed_time(e1) * 1e3 / K)
        return float(np.median(out))

    def per_call_us(step, refresh):
        """HIP events around every single call (each includes its dispatch)."""
        refresh()
        torch.cuda.synchronize()
        ev = [[torch.cuda.Event(enable_timing=True) for _ in range(2)] for _ in range(K)]
        for k in range(K):
            ev[k][0].record()
            step(k, stream)
            ev[k][1].record()
        torch.cuda.synchronize()
        return np.array([a.elapsed_time(b) for a, b in ev]) * 1e3

    def fill_work(matchers):
        """[stacks with a bitset row, level-0, level-1, level-2 list entries] over a batch of host matchers."""
        return np.sum([m.debug_fill_work() for m in matchers], axis=0)

    def step_bytes(matchers_of_set, words_of_set, B, V, W, elem):
        """Algorithmic bytes per launch, averaged over state sets: (fill, apply, fused, fill work, rejected,
        bytes of the logits in 64-byte pieces)."""
        fill_b, rej, work, pieces = [], [], [], []
        per_piece = 64 // elem            # logits per 64-byte piece
        for ms, words in zip(matchers_of_set, words_of_set):
            fw = fill_work(ms)
            work.append(fw)
            # accepted words of every stack top that keeps a bitset row, every list entry once, mask words written
            fill_b.append(4.0 * fw[0] * W + 4.0 * float(fw[1:].sum()) + 4.0 * B * W)
            bits = np.unpackbits(words.view(np.uint8), axis=1, bitorder="little")[:, :V]
            rej.append(float(B * V - int(bits.sum())))
            full = bits[:, : V // per_piece * per_piece].reshape(B, -1, per_piece).sum(axis=2)
            # no logit is read: a piece with a rejected logit in it is written once, whole or under a byte mask
            pieces.append(64.0 * float((full != per_piece).sum()))
        fill_bytes = float(np.mean(fill_b))
        rejected = float(np.mean(rej))
        apply_bytes = 4.0 * B * W + elem * rejected
        return fill_bytes, apply_bytes, fill_bytes + elem * rejected, np.mean(work, axis=0), rejected, float(np.mean(pieces))

    def roofline(kernel, bytes_per_launch, us, traffic_key, **extra):
        r = {"kernel": kernel, "bound": "hbm", "kernel_us": us, "achieved": bytes_per_launch / (us * 1e-6) / 1e9,
             "peak": HBM_PEAK_GBS, "unit": "GB/s", "traffic": traffic.get(traffic_key), "bytes_per_launch": bytes_per_launch}
        r["frac"] = r["achieved"] / HBM_PEAK_GBS
        r.update(extra)
        return r

    # ------------------------------------------------------------------ config 5: the serving decode step
    t_setup = time.time()
    work = wl.ServingWorkload(n_rows=args.rows, vocab_size=args.vocab, pool=args.pool, log=log)
    B, V, W = work.B, work.V, work.W
    n_sets = len(work.sets)
    log(f"set-up done in {time.time() - t_setup:.1f} s; context-dependent fraction at the stack tops "
        f"{work.uncertain_fraction:.3f}")
    refresh = work.refresh_logits
    nothing = lambda: None

    # the headline: passes of exactly K one-launch steps from device-resident states
    fused_passes = timed_passes(work.fused_step_device, refresh, warmup=args.warmup)
    us_per_step = float(np.median(fused_passes))
    overflow = xgm.overflow_total()
    log(f"one-launch step: {us_per_step:.2f} us (passes {[round(x, 2) for x in fused_passes]})")
    two_call_us = float(np.median(timed_passes(work.step_device, refresh, passes=3)))
    host_state_us = float(np.median(timed_passes(work.step, refresh, passes=3, warmup=10)))
    host_state_fused_us = float(np.median(timed_passes(work.fused_step, refresh, passes=3)))
    fill_only_us = float(np.median(timed_passes(work.fill_device, nothing, passes=3)))
    apply_only_us = float(np.median(timed_passes(work.apply, refresh, passes=3)))

    # launch durations by HIP events on the launch stream (K back-to-back launches), and events around every call
    fused_kernel_us = event_us(work.fused_step_device, refresh)
    fill_kernel_us = event_us(work.fill_device, nothing)
    apply_kernel_us = event_us(work.apply, refresh)
    fused_call_us = per_call_us(work.fused_step_device, refresh)
    fill_call_us = per_call_us(work.fill_device, nothing)
    apply_call_us = per_call_us(work.apply, refresh)

    # ---- the whole decode cycle: accept the sampled tokens on the device, then fill and apply, K' real steps.
    # The token sequences are the seeded walks that produced the state sets, replayed from the start states.
    fresh = [xgm.Matcher(cache=c) for c in work.caches]
    cycle_batch = xgm.DeviceBatch(fresh, history=0, stream=stream)
    replays = [torch.tensor(work.replay_tokens(k), dtype=torch.int32, device="cuda") for k in range(n_sets)]
    d_restart = torch.zeros(B, dtype=torch.int32, device="cuda")

    def restart_rows():
        for b, m in enumerate(fresh):
            cycle_batch.set_row(b, m, stream)

    def replay(k, accept_only=False):
        toks = replays[k]
        t = work.logits[k % len(work.logits)]
        for s in range(toks.shape[0]):
            cycle_batch.accept_tokens(toks[s].data_ptr(), stream)
            if not accept_only:
                cycle_batch.fill_and_apply(work.d_mask.data_ptr(), t.data_ptr(), xgm.DTYPE_BF16, V, t.stride(0), stream=stream)
        return toks.shape[0]

    restart_rows()
    replay(0)                                     # warm-up, and a check: the replay ends in state set 0
    assert not cycle_batch.status(stream).any(), "the device refused a token of a recorded walk"
    cycle_batch.fill_next_token_bitmask(work.d_mask.data_ptr(), stream)
    got = work.d_mask.clone()
    work.fill_device(0, stream)
    torch.cuda.synchronize()
    assert torch.equal(got, work.d_mask), "replaying the recorded walk did not reach state set 0"
    cycle_us, accept_us_all, n_cycles = [], [], 0
    for accept_only in (False, True):
        spent, steps = 0.0, 0
        for k in range(n_sets):
            restart_rows()
            work.refresh_logits()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            steps += replay(k, accept_only)
            torch.cuda.synchronize()
            spent += time.perf_counter() - t0
        (accept_us_all if accept_only else cycle_us).append(spent * 1e6 / steps)
        n_cycles = steps
    assert not cycle_batch.status(stream).any()
    decode_cycle = {"us_per_cycle": cycle_us[0], "accept_only_us": accept_us_all[0], "cycles_timed": n_cycles,
                    "note": "xgm_batch_accept_tokens (one kernel: every row's stacks moved on by its token, the next state "
                            "written with where its token lists lie) followed by xgm_batch_fill_and_apply, for every step of "
                            f"the {n_sets} recorded walks that lead from the start states to the state sets, {B} rows; rows "
                            "whose walk is shorter sit out the accept (token id -1) but are still filled and masked"}
    del cycle_batch
    log(f"decode cycle {cycle_us[0]:.2f} us (accept alone {accept_us_all[0]:.2f} us) over {n_cycles} steps")

    # ---- what this box writes at best: a plain fill of the same rotating logits buffers, and a copy between them
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
    e0.record()
    for k in range(n_fill):
        work.logits[k % len(work.logits)].copy_(work.logits[(k + 3) % len(work.logits)])
    e1.record()
    torch.cuda.synchronize()
    plain_copy_us = e0.elapsed_time(e1) * 1e3 / n_fill
    plain_copy_gbs = 2.0 * 2.0 * B * V / (plain_copy_us * 1e-6) / 1e9
    work.refresh_logits()

    # ---- the fill from host-side states: events inside the library around its two launches
    up_us, fk_us = [], []
    for k in range(min(K, 200)):
        a, b_ = xgm.debug_fill_timed(work.sets[k % n_sets].batch, work.d_mask.data_ptr(), stream)
        up_us.append(a)
        fk_us.append(b_)

    # ---- algorithmic work per launch (averaged over the state sets in use)
    words_of_set, steps_count = [], []
    for k in range(n_sets):
        work.fill_device(k, stream)
        torch.cuda.synchronize()
        words_of_set.append(work.d_mask.cpu().numpy())
        steps_count.append(xgm.debug_fill_count_steps(work.sets[k].batch, work.d_mask.data_ptr(), stream))
    fill_bytes, apply_bytes, fused_bytes, fwork, rejected, piece_bytes = step_bytes(
        [w.matchers for w in work.sets], words_of_set, B, V, W, 2)
    ceiling = {"plain_fill_of_the_same_buffers_GB/s": plain_fill_gbs, "plain_copy_between_them_GB/s": plain_copy_gbs,
               "note": "what this box reaches with a plain torch fill / copy of the rotating logits buffers: the attainable "
                       "ceiling for a kernel that writes them, against the published 8 TB/s"}
    roof_fused = roofline("fill_kernel<false, 2> (mask fill and -inf apply in one launch, device-resident states)",
                          fused_bytes, fused_kernel_us, "fill_kernel<false, 2>",
                          bytes_per_launch_in_64_byte_pieces=fill_bytes + piece_bytes,
                          frac_of_measured_fill_rate=fused_bytes / (fused_kernel_us * 1e-6) / 1e9 / plain_fill_gbs,
                          pieces_frac_of_measured_fill_rate=(fill_bytes + piece_bytes) / (fused_kernel_us * 1e-6) / 1e9 / plain_fill_gbs,
                          attainable=ceiling,
                          note="bytes = what the method must move: accepted bitset rows and list entries read, mask words "
                               "written, 2 bytes per rejected bf16 logit written (no logit is read, the mask is not re-read); "
                               "the memory writes 64-byte pieces, whole or under a byte mask: bytes_per_launch_in_64_byte_pieces counts every piece "
                               "that holds a rejected logit once, and pieces_frac_of_measured_fill_rate prices that count against "
                               "the plain fill of the same buffers; kernel_us = HIP "
                               "events on the launch stream around the K back-to-back launches of a pass, divided by K")
    roof_fill = roofline("fill_kernel<false, 0> (device-resident states)", fill_bytes, fill_kernel_us, "fill_kernel<false, 0>",
                         stacks_with_bitset_row=float(fwork[0]), list_entries_per_launch=float(fwork[1:].sum()),
                         automaton_steps_per_launch=float(np.mean(steps_count)),
                         note="a few dependent memory rounds per workgroup (row descriptor, stack headers, bitset row and list "
                              "entries, store): latency, not bytes; the accepted rows of the 16 state sets fit the last-level "
                              "cache, so part of these reads never reaches HBM")
    roof_apply = roofline("apply_kernel<2>", apply_bytes, apply_kernel_us, "apply_kernel<2>",
                          read_modify_write_bytes_per_launch=2.0 * 2.0 * B * V + 4.0 * B * W,
                          bytes_per_launch_in_64_byte_pieces=4.0 * B * W + piece_bytes,
                          frac_of_measured_fill_rate=apply_bytes / (apply_kernel_us * 1e-6) / 1e9 / plain_fill_gbs,
                          pieces_frac_of_measured_fill_rate=(4.0 * B * W + piece_bytes) / (apply_kernel_us * 1e-6) / 1e9 / plain_fill_gbs,
                          attainable=ceiling)
    roof_step = roofline("fill_kernel<false, 0> + apply_kernel<2>", fill_bytes + apply_bytes, two_call_us, None,
                         note="the two-call step: fill, then apply (wall clock per step)")

    # ------------------------------------------------------------------ configs 1-3: the smaller workloads
    configs = {}
    if not args.no_configs:
        specs = [
            ("1", "arithmetic grammar, vocabulary 1024, batch 1, fp32 logits, 8 states along a 64-step walk",
             lambda: ([xgm.Cache(xgm.Grammar(si.ARITH_GRAMMAR, "expr"), wl.make_xgm_vocab(v1))], v1, 0, 64, torch.float32, 1.0, 0.0)),
            ("2", "JSON grammar, vocabulary 32000, batch 1, fp32 logits, 8 states along a 256-step walk",
             lambda: ([xgm.Cache(xgm.Grammar(si.JSON_GRAMMAR, "root"), wl.make_xgm_vocab(v2))], v2, 2, 256, torch.float32, 1.0, 0.35)),
            ("3", "schema grammar, vocabulary 128256, batch 16, bf16 logits, 8 states along a 512-step walk",
             lambda: ([xgm.Cache(xgm.Grammar(si.make_schema_grammar(0), "root"), wl.make_xgm_vocab(v3))] * 16, v3, 3, 512,
                      torch.bfloat16, 2.0, 0.35)),
        ]
        v1, v2, v3 = si.make_vocab("arith", 1024, 0), si.make_vocab("bpe", 32000, 0), si.make_vocab("bpe", 128256, 0)
        for name, what, make in specs:
            caches, vocab, seed, total, dtype, sigma, bias = make()
            sw = wl.WalkedWorkload(caches, vocab, seed, total, pool=8, dtype=dtype, sigma=sigma, structural_bias=bias)
            elem = 4 if dtype == torch.float32 else 2
            words = []
            for k in range(len(sw.sets)):
                sw.fill_device(k, stream)
                torch.cuda.synchronize()
                words.append(sw.d_mask.cpu().numpy())
            fb, ab, ub, _, _, _ = step_bytes([s.matchers for s in sw.sets], words, sw.B, sw.V, sw.W, elem)
            f_us = float(np.median(timed_passes(sw.fill_device, nothing, passes=3, warmup=20)))
            a_us = float(np.median(timed_passes(sw.apply, sw.refresh_logits, passes=3, warmup=20)))
            u_us = float(np.median(timed_passes(sw.fused_step_device, sw.refresh_logits, passes=3, warmup=20)))
            h_us = float(np.median(timed_passes(sw.fused_step, sw.refresh_logits, passes=3, warmup=20)))
            configs[name] = {"workload": what, "batch": sw.B, "vocab": sw.V,
                             "fill_us": f_us, "apply_us": a_us, "fill_plus_apply_one_launch_us": u_us,
                             "one_launch_from_host_side_states_us": h_us,
                             "token_checks_per_s": sw.B * sw.V / (u_us * 1e-6),
                             "bytes_per_launch": {"fill": fb, "apply": ab, "one_launch": ub},
                             "frac": {"fill": fb / (f_us * 1e-6) / 1e9 / HBM_PEAK_GBS, "apply": ab / (a_us * 1e-6) / 1e9 / HBM_PEAK_GBS,
                                      "one_launch": ub / (u_us * 1e-6) / 1e9 / HBM_PEAK_GBS},
                             "note": "wall clock per step over passes of K steps (launch included): at these sizes a step is one "
                                     "launch's latency, so the fractions of the HBM peak are small by nature"}
            log(f"config {name}: fill {f_us:.2f} us, apply {a_us:.2f} us, one launch {u_us:.2f} us")
            del sw

    # ------------------------------------------------------------------ config 4: mask-cache build throughput
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
                       "headline": "pairs_per_s_whole_build: positions x tokens per second of the whole xgm_cache_build call "
                                   "(classification, rank -> id permutation, bitset rows and lists, the per-call-site lists of "
                                   "section 3.2 three frames deep), best of 3; classification_stage = the part of the call up to the point where "
                                   "the section 3.1 classes of every node are known (classify kernel, permutation, row statistics, one "
                                   "synchronisation)",
                       "note": "steps_per_s = pairs_per_s x the mean automaton steps per pair of a seeded sample; a "
                               "step is 3 to 5 dependent table lookups (header, follow set, class, shape, target); "
                               "the ceiling is a chain of dependent LDS reads with every wave slot busy"}
        for name, text in (("json", si.JSON_GRAMMAR), ("csql", si.CSQL_GRAMMAR)):
            g = xgm.Grammar(text, "root")
            best = whole = stage = None
            for _ in range(3):
                c = xgm.Cache(g, xv128, stream)
                best = c.build_kernel_seconds if best is None else min(best, c.build_kernel_seconds)
                whole = c.build_seconds if whole is None else min(whole, c.build_seconds)
                stage = c.build_classify_seconds if stage is None else min(stage, c.build_classify_seconds)
                hostc, stats, held = c.host_classified, c.stats, c.device_bytes
                del c
            sps = mean_steps_per_pair(g, toks128, np.random.Generator(np.random.PCG64(11)))
            cache_build[name] = {"positions": g.num_nodes, "tokens": 128256, "whole_build_ms": whole * 1e3,
                                 "pairs_per_s_whole_build": g.num_nodes * 128256 / whole,
                                 "classification_stage_ms": stage * 1e3,
                                 "pairs_per_s_classification_stage": g.num_nodes * 128256 / stage,
                                 "classify_kernel_ms": best * 1e3, "pairs_per_s_classify_kernel": g.num_nodes * 128256 / best,
                                 "steps_per_pair": sps, "steps_per_s": sps * g.num_nodes * 128256 / best,
                                 "lookups_vs_ceiling": 4.0 * sps * g.num_nodes * 128256 / best / lds_rate,
                                 "host_classified_pairs": hostc, "cache": stats, "cache_device_bytes": held}
        # the same C/SQL cache resolved one frame deep only (XGM_CACHE_DEPTH(1)): faster to build, more to walk per fill
        g = xgm.Grammar(si.CSQL_GRAMMAR, "root")
        shallow = None
        for _ in range(3):
            c = xgm.Cache(g, xv128, stream, depth=1)
            shallow = c.build_seconds if shallow is None else min(shallow, c.build_seconds)
            shallow_stats, shallow_bytes = c.stats, c.device_bytes
            del c
        cache_build["csql_one_frame_deep"] = {"whole_build_ms": shallow * 1e3,
                                              "pairs_per_s_whole_build": g.num_nodes * 128256 / shallow,
                                              "cache": shallow_stats, "cache_device_bytes": shallow_bytes}
        toks_s = work.vocab.tokens()
        sps = float(np.mean([mean_steps_per_pair(work.grammars[k], toks_s, np.random.Generator(np.random.PCG64(12 + k)), 1500)
                             for k in (0, 31, 77, 127) if k < len(work.grammars)]))
        pps = work.build_pairs / max(work.build_kernel_seconds, 1e-12)
        whole_s = sum(c.build_seconds for c in work.caches)
        # the first build of a process also uploads the vocabulary and loads the kernels: kept apart
        rest = work.caches[1:]
        rest_pairs = sum(c.num_nodes for c in rest) * args.vocab
        rest_whole = sum(c.build_seconds for c in rest)
        rest_stage = sum(c.build_classify_seconds for c in rest)
        rest_kernel = sum(c.build_kernel_seconds for c in rest)
        cache_build["serving_set_up"] = {"pairs": work.build_pairs, "classify_kernel_s": work.build_kernel_seconds,
                                         "pairs_per_s_classify_kernel": pps, "whole_builds_s": whole_s,
                                         "first_build_s": work.caches[0].build_seconds,
                                         "after_the_first_build": {
                                             "caches": len(rest), "pairs": rest_pairs, "whole_builds_s": rest_whole,
                                             "classification_stage_s": rest_stage, "classify_kernel_s": rest_kernel,
                                             "pairs_per_s_whole_build": rest_pairs / max(rest_whole, 1e-12),
                                             "pairs_per_s_classification_stage": rest_pairs / max(rest_stage, 1e-12),
                                             "pairs_per_s_classify_kernel": rest_pairs / max(rest_kernel, 1e-12),
                                             "note": "the first build of a process also uploads the vocabulary and loads "
                                                     "the code object"},
                                         "steps_per_pair": sps, "steps_per_s": sps * pps,
                                         "lookups_vs_ceiling": 4.0 * sps * pps / lds_rate}
        st = [c.stats for c in work.caches]
        cache_build["serving_storage"] = {"caches": len(work.caches), "nodes": sum(c.num_nodes for c in work.caches),
                                          "device_bytes": sum(c.device_bytes for c in work.caches),
                                          **{k: sum(s[k] for s in st) for k in st[0]},
                                          "note": "adaptive storage (section 3.1): bitset rows only for nodes that accept many "
                                                  "tokens, lists otherwise; context-dependent tokens resolved per call site "
                                                  "into (node, context) and (node, context, context) lists"}

    if cache_build is not None:
        configs["4"] = {"workload": "mask-cache build: all 128256 tokens at every automaton node, generic JSON grammar and the "
                                    "C/SQL-like grammar",
                        "json_pairs_per_s": cache_build["json"]["pairs_per_s_whole_build"],
                        "csql_pairs_per_s": cache_build["csql"]["pairs_per_s_whole_build"],
                        "json_pairs_per_s_classification_stage": cache_build["json"]["pairs_per_s_classification_stage"],
                        "csql_pairs_per_s_classification_stage": cache_build["csql"]["pairs_per_s_classification_stage"],
                        "json_pairs_per_s_classify_kernel": cache_build["json"]["pairs_per_s_classify_kernel"],
                        "csql_pairs_per_s_classify_kernel": cache_build["csql"]["pairs_per_s_classify_kernel"],
                        "note": "whole xgm_cache_build call (see cache_build)"}

    # ------------------------------------------------------------------ the oracle on the host cores, bounded sample
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
        "metric": "vocab token checks/sec + per-step bitmask fill+apply µs (batch×vocab)",
        "value": B * V / (us_per_step * 1e-6),
        "unit": "token checks/s",
        "n_gpus": 1, "steps": K, "warmup": args.warmup, "passes": P,
        "ms_per_step": us_per_step * 1e-3,
        "fill_plus_apply_us": us_per_step,
        "fill_plus_apply_us_per_pass": fused_passes,
        "step_form": "one launch (xgm_batch_fill_and_apply); median of `passes` passes of exactly `steps` steps, each on "
                     "freshly drawn logits, after `warmup` untimed steps, between two synchronisations; the two-call form is "
                     "timed in two_call_path",
        "two_call_path": {"fill_plus_apply_us": two_call_us, "fill_alone_us": fill_only_us, "apply_alone_us": apply_only_us,
                          "note": "xgm_batch_fill_next_token_bitmask, then xgm_apply_token_bitmask_inplace"},
        "host_state_path": {"fill_plus_apply_us": host_state_us, "fused_fill_and_apply_us": host_state_fused_us,
                            "note": "matcher states kept on the host: stacks packed and uploaded over PCIe every step"},
        "decode_cycle": decode_cycle,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "u32",
        "logits_dtype": "bf16 (only -inf patterns are stored; no floating-point arithmetic anywhere on the path)",
        "data": "synthetic",
        "config": {"workload": f"serving decode step: batch {B} x vocab {V}, {B} distinct string-heavy schema "
                               f"grammars, bf16 logits [{B},{V}], {n_sets} pre-walked state sets resident on the "
                               f"device, {len(work.logits)} rotating logits buffers; a state set holds, per stack, the frames "
                               f"and where its token lists lie in the mask cache (written when the state was entered: by "
                               f"xgm_batch_create here, by the accept kernel in decode_cycle)",
                   "batch": B, "vocab": V,
                   "context_dependent_fraction_at_tops": work.uncertain_fraction,
                   "context_dependent_fraction_after_narrowing": work.uncertain_fraction_narrowed},
        "kernel_us": {"note": "HIP events around every single call (each includes its dispatch); the rooflines use events around "
                              "K back-to-back launches",
                      "host_state_fill_kernel_mean": float(np.mean(fk_us)), "host_state_upload_kernel_mean": float(np.mean(up_us)),
                      "fused_call_mean": float(fused_call_us.mean()), "fused_call_p50": float(np.median(fused_call_us)),
                      "fused_call_p99": float(np.percentile(fused_call_us, 99)),
                      "fill_call_mean": float(fill_call_us.mean()), "fill_call_p50": float(np.median(fill_call_us)),
                      "fill_call_p99": float(np.percentile(fill_call_us, 99)),
                      "apply_call_mean": float(apply_call_us.mean()), "apply_call_p50": float(np.median(apply_call_us)),
                      "apply_call_p99": float(np.percentile(apply_call_us, 99))},
        "roofline": roof_fused,
        "roofline_fill": roof_fill,
        "roofline_apply": roof_apply,
        "roofline_two_call_step": roof_step,
        "configs": configs,
        "device": device,
        "walks_on_host_slow_path": int(overflow),
        "cache_build": cache_build,
        "cpu_baseline": cpu_baseline,
    }
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
