"""Mask-cache build of one grammar, by itself (the workload that rocprofv3 summaries of the build kernels are
taken on):

    python -m paper_2411_15100_amd.build_bench --grammar csql --vocab 128256 --repeat 5

Builds the cache of the generic JSON grammar, the C/SQL-like grammar or a string-heavy schema grammar
`--repeat` times after one untimed build (which uploads the vocabulary) and prints one JSON line with the
best timings: whole call, classification stage, classify kernel, all nodes x all tokens per second.
"""

from __future__ import annotations

import argparse
import json
import os
import sys

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))


def main() -> None:
    ap = argparse.ArgumentParser()
    ap.add_argument("--grammar", choices=["json", "csql", "schema"], default="csql")
    ap.add_argument("--seed", type=int, default=0, help="seed of the schema grammar")
    ap.add_argument("--vocab", type=int, default=128256)
    ap.add_argument("--repeat", type=int, default=5)
    args = ap.parse_args()

    import torch
    import synth_inputs as si
    import paper_2411_15100_amd as xgm
    from paper_2411_15100_amd import workloads as wl

    if not torch.cuda.is_available():
        raise SystemExit("build_bench needs a GPU")
    vocab = si.make_vocab("bpe", args.vocab, 0)
    xv = wl.make_xgm_vocab(vocab)
    text = {"json": si.JSON_GRAMMAR, "csql": si.CSQL_GRAMMAR}.get(args.grammar) or si.make_schema_grammar(
        args.seed, string_heavy=True)
    g = xgm.Grammar(text, "root")
    stream = wl.current_stream()
    xgm.Cache(g, xv, stream)   # untimed: vocabulary upload, code object
    whole = stage = kernel = None
    for _ in range(args.repeat):
        c = xgm.Cache(g, xv, stream)
        whole = min(whole or 1e9, c.build_seconds)
        stage = min(stage or 1e9, c.build_classify_seconds)
        kernel = min(kernel or 1e9, c.build_kernel_seconds)
        stats, held, on_host = c.stats, c.device_bytes, c.host_classified
        del c
    pairs = g.num_nodes * args.vocab
    print(json.dumps({"grammar": args.grammar, "nodes": g.num_nodes, "tokens": args.vocab, "pairs": pairs,
                      "whole_build_ms": whole * 1e3, "classification_stage_ms": stage * 1e3,
                      "classify_kernel_ms": kernel * 1e3, "pairs_per_s_whole_build": pairs / whole,
                      "pairs_per_s_classification_stage": pairs / stage, "pairs_per_s_classify_kernel": pairs / kernel,
                      "host_classified_pairs": on_host, "cache_device_bytes": held, "cache": stats}))


if __name__ == "__main__":
    main()
