"""Throughput of the prefill entry point (bita_prefill) by chunk size:

    python -m paper_2401_12522_amd.prefill_bench 7b [--ctx 1024] [--chunks 64,128,256,512] [--batch 1]

Synthetic weights of the named shape (drawn on the GPU), seeded random context tokens.  For each
chunk size the cache is reset and the same context is prefilled `--reps` times; prints the time
per call and context tokens per second (all sequences)."""
import argparse
import time

import numpy as np
import torch

import synth

from . import binding as B


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("workload", choices=["tiny", "7b", "13b", "70b"])
    ap.add_argument("--ctx", type=int, default=1024)
    ap.add_argument("--chunks", default="64,128,256,512")
    ap.add_argument("--batch", type=int, default=1)
    ap.add_argument("--reps", type=int, default=3)
    ap.add_argument("--seed", type=int, default=0)
    args = ap.parse_args()
    B.lib()
    cfg = synth.get_config(args.workload)
    chunks = [int(c) for c in args.chunks.split(",")]
    smax = (args.ctx + 63) // 64 * 64
    w = synth.SynthWeights(cfg, seed=args.seed, device="cuda")
    model = B.Model(cfg, w, max_pos=smax + 64, free_source=True)
    kv = B.KVState(cfg, cfg.n_layers, args.batch, smax, max(chunks))
    toks = np.stack([synth.random_context(cfg.vocab, args.ctx, args.seed + 7919 * b) for b in range(args.batch)])
    toks = torch.tensor(toks, dtype=torch.int32, device="cuda")
    for chunk in chunks:
        ws = torch.empty(B.lib().bita_prefill_workspace_bytes(model.handle, args.batch, chunk), dtype=torch.uint8, device="cuda")
        ts = []
        for _ in range(args.reps + 1):                  # the first call is a warm-up
            kv.ctx_len.zero_()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            B.prefill(model, kv, 0, toks, chunk, workspace=ws)   # only enqueues: wait for the stream here
            torch.cuda.synchronize()
            ts.append(time.perf_counter() - t0)
        assert bool((kv.ctx_len == args.ctx).all())
        t = float(np.mean(ts[1:]))
        print(f"{args.workload}: batch {args.batch}, ctx {args.ctx}, chunk {chunk}: {t * 1e3:.1f} ms per call, "
              f"{args.batch * args.ctx / t:.0f} tokens/s", flush=True)


if __name__ == "__main__":
    main()
