"""Micro-benchmark of the tree-masked attention entry point (bita_tree_attention), for use
alone or under rocprofv3:

    python -m paper_2401_12522_amd.attention_bench 70b-gqa [--reps 20]

Workloads: `7b` = 32 query / 32 KV heads, one sequence, 1024 cached tokens; `70b-gqa` = 64 query /
8 KV heads, batch 8 with per-sequence context lengths uniform in [1024, 4096] (seeded), the
kernel-only configuration of the problem statement.  Both: head_dim 128, 16 prefix tokens, a
64-node random tree of depth <= 6 plus 4 mask rows, N(0,1) q/K/V in bf16 (q and the pass rows'
K/V with a second, small plane).  Prints time per call and the K/V bytes it has to read."""
import argparse

import numpy as np
import torch

import synth

from . import binding as B

WORKLOADS = {"7b": dict(Hq=32, Hkv=32, batch=1, ctx=(1024, 1024)),
             "70b-gqa": dict(Hq=64, Hkv=8, batch=8, ctx=(1024, 4096))}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("workload", choices=sorted(WORKLOADS))
    ap.add_argument("--reps", type=int, default=20)
    ap.add_argument("--seed", type=int, default=0)
    args = ap.parse_args()
    wl = WORKLOADS[args.workload]
    Hq, Hkv, Bn, hd, P = wl["Hq"], wl["Hkv"], wl["batch"], 128, 16
    rng = np.random.default_rng(args.seed)
    ctx = rng.integers(wl["ctx"][0], wl["ctx"][1] + 1, size=Bn).astype(np.int32)
    tin = synth.attach_mask_groups(synth.random_tree(64, 6, args.seed), [0], 4)
    tmpl = B.TreeTemplate(tin.parent, tin.is_mask, tin.n_tree, 4)
    R = tin.rows
    smax = int(ctx.max()) + 8
    gen = torch.Generator(device="cuda").manual_seed(args.seed)
    g = lambda *s: torch.randn(*s, device="cuda", generator=gen).to(torch.bfloat16)   # noqa: E731
    q, q_lo = g(Bn, R, Hq, hd), g(Bn, R, Hq, hd) * 2.0 ** -9
    kc, vc = g(Bn, Hkv, smax, hd), g(Bn, Hkv, smax, hd)
    kt, vt = g(Bn, Hkv, R, hd), g(Bn, Hkv, R, hd)
    kt_lo, vt_lo = g(Bn, Hkv, R, hd) * 2.0 ** -9, g(Bn, Hkv, R, hd) * 2.0 ** -9
    pk, pv = g(Hkv, P, hd), g(Hkv, P, hd)
    cl = torch.tensor(ctx, dtype=torch.int32, device="cuda")
    hint = int(ctx.max())

    def call():
        return B.tree_attention(tmpl, q, kc, vc, kt, vt, pk, pv, cl, hint, q_lo=q_lo, k_tree_lo=kt_lo, v_tree_lo=vt_lo)

    for _ in range(3):
        call()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(args.reps):
        call()
    e1.record()
    torch.cuda.synchronize()
    us = e0.elapsed_time(e1) * 1e3 / args.reps
    kv_bytes = int(sum(2 * (P + int(c) + 2 * R) * hd * 2 * Hkv for c in ctx))
    flops = int(sum(2 * 2 * 2 * 80 * (P + int(c) + 2 * R) * hd * Hq for c in ctx))   # QK^T and PV, two planes, 80 padded rows
    print(f"{args.workload}: batch {Bn}, ctx {ctx.tolist()}, rows {R}: {us:.1f} us per call; K/V to read "
          f"{kv_bytes / 1e6:.1f} MB ({kv_bytes / us / 1e6:.2f} TB/s), matrix work {flops / 1e9:.1f} GFLOP "
          f"({flops / us / 1e6:.1f} TFLOP/s)")


if __name__ == "__main__":
    main()
