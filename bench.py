#!/usr/bin/env python3
"""Benchmark of the BiTA tree-verify step on one MI355X.

A "step" is one pass of the whole hot path -- build_tree, verify_step (decoder forward
over the token tree + mask rows, tree-masked attention, LM head, argmax/top-k), accept,
compact_kv -- over one batch of synthetic input, replayed from a HIP graph.  Default
workload: the LLaMA-2-7B-shaped configuration (32 layers, d 4096, 32 heads, FFN 11008,
vocab 32000, 16 prompt tokens, 1024-token context, 64-node tree + 4 mask rows, batch 1).

Prints ONE JSON line (see the keys below).  `value` is scored rows per second with every
input resident in HBM; `hbm_gbps` is the algorithmic bytes of a step (weights + K/V cache
+ prompt prefix) divided by the step time.

With no --workload the line's headline is the 7B-shaped step and a `workloads` entry carries
the other half of the metric, the LLaMA-2-70B-shaped step (80 layers, 8 K/V heads, 2048-token
context, 64 steps, compaction included), run in the same process after the first.
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0


# HBM-side bytes (fetch + write) per GEMM launch, averaged over the launches of one step, from the
# FETCH_SIZE / WRITE_SIZE counter runs scaled by a copy kernel (profiles/gemm_traffic_7b.md,
# gemm_traffic_70b.md), 68 rows, batch 1; counters cannot be collected from inside this process,
# so the figure is carried as a constant
GEMM_TRAFFIC_BYTES_PER_LAUNCH = {"7b": 120.9e6, "70b": 459.3e6}
GEMM_TRAFFIC_SOURCE = {"7b": "profiles/gemm_traffic_7b.md", "70b": "profiles/gemm_traffic_70b.md"}
# the same kernel's duration as rocprofv3 --kernel-trace --stats sees it (no event pairs between
# the launches): total GEMM microseconds per step from the committed profile of this workload
ROCPROF_GEMM = {"7b": ("profiles/llama7b_step_kernel_stats.md", 3263.0),
                "70b": ("profiles/llama70b_step_kernel_stats.md", 22169.0)}
# the second leg of the default run (the metric is quoted on both shapes)
SECOND_LEG = {"workload": "70b", "steps": 64, "warmup": 8}
# layer counts of the two oracle passes timed for cpu_baseline (about 10 s of host work at 7B width)
CPU_SAMPLE_LAYERS = (4, 8)


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=128)
    ap.add_argument("--warmup", type=int, default=8)
    ap.add_argument("--workload", default=None, choices=["tiny", "7b", "13b", "70b"],
                    help="default: the 7B-shaped step as the headline plus the 70B-shaped step under `workloads`")
    ap.add_argument("--no-second-leg", action="store_true", help="with no --workload: skip the 70B-shaped leg")
    ap.add_argument("--ctx", type=int, default=None)
    ap.add_argument("--batch", type=int, default=1,
                    help="sequences per step (independent contexts, same template); above 1 the run is "
                         "free-running: planted drafts need the one-sequence planning pass")
    ap.add_argument("--tree", default=None, choices=sorted(TREES),
                    help="draft-tree template (default: full64; tiny workload: its seeded 8-node tree); "
                         "'-pernode' attaches a mask group to every tree node instead of the root only")
    ap.add_argument("--mode", default="planted", choices=["free", "planted"])
    ap.add_argument("--page-size", type=int, default=0,
                    help="keep the KV cache in shuffled pages of this many slots (power of two >= 16; runs free)")
    ap.add_argument("--no-graph", action="store_true")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--calibration-copy-mb", type=int, default=0,
                    help="also run a plain device copy of this many MB a few times (a kernel of known "
                         "traffic, to scale rocprofv3's FETCH_SIZE / WRITE_SIZE readings)")
    return ap.parse_args()


# draft-tree templates of the row-count sweep (Sec. 3.2, compared in Sec. 4.3.4 / Table 4: full trees by per-level top-k, the
# efficient tree of n*k+1 rows; mask groups on the root only or on every node)
TREES = {
    "full64": ("full", [4, 3, 2, 1], 64), "full34": ("full", [3, 2, 2, 1], 34), "full16": ("full", [3, 2, 1, 1], 16),
    "efficient": ("efficient", 5, None),
}
TREES.update({k + "-pernode": v for k, v in list(TREES.items())})


def workload_template(synth, cfg, name, tree=None):
    """Draft-tree shape per workload: small case = seeded random 8-node tree; LLaMA shapes =
    full branching by per-level top-k (4,3,2,1) truncated to 64 rows, one mask group on the
    root, unless --tree names another template."""
    if tree is None and name == "tiny":
        parent = synth.random_tree(8, 3, 0)
    else:
        kind, a, T = TREES[tree or "full64"]
        parent = synth.full_branching_tree(a, T) if kind == "full" else synth.efficient_tree_parents(cfg.n_mask, a)
    per_node = tree is not None and tree.endswith("-pernode")
    return synth.attach_mask_groups(parent, list(range(len(parent))) if per_node else [0], cfg.n_mask)


def tree_shape(tin):
    """children[v] in sibling order (a child's index in it is the candidate column it carries)
    and the depth of the deepest draft row."""
    children = [[] for _ in range(tin.n_tree)]
    depth = [0] * tin.n_tree
    for v in range(1, tin.n_tree):
        children[int(tin.parent[v])].append(v)
        depth[v] = depth[int(tin.parent[v])] + 1
    return children, max(depth)


def planted_walk(children, depth_max, n_levels, rng):
    """A seeded root-to-node walk of the template: how many levels of the reference
    continuation to plant (0..depth_max, cut short at a node without children) and, per level,
    the candidate column (= sibling index) of the node the walk passes through."""
    depth_ok = int(rng.integers(0, depth_max + 1))
    col, v = np.zeros(n_levels, int), 0
    for i in range(depth_ok):
        if not children[v]:
            depth_ok = i
            break
        col[i] = int(rng.integers(0, len(children[v])))
        v = children[v][col[i]]
    return depth_ok, col


def prefill(B, model, kv, cfg, ctx_tokens, chunk=64):
    """Fill the cache with context[:-1] through the library's prefill entry point (chunked
    causal passes).  ctx_tokens: [n] or [batch][n] (equal lengths)."""
    import torch
    ctx_tokens = np.atleast_2d(np.asarray(ctx_tokens))
    if kv.rows < chunk:
        kv.resize_rows(model.n_layers, cfg, chunk)
    toks = torch.tensor(ctx_tokens[:, :-1], dtype=torch.int32, device="cuda").contiguous()
    B.prefill(model, kv, 0, toks, chunk)
    torch.cuda.synchronize()


def cpu_baseline(cfg, wsrc_np, kv_np, tmpl_in, root_token, cand, ctx_len):
    """Time the oracle's step on a bounded sample: the step's token assignment, the forward with
    CPU_SAMPLE_LAYERS[0] and [1] of the model's layers (+ LM head) at full width, selection,
    acceptance walk and K/V commit of those layers; the per-layer cost is extrapolated linearly
    to the full depth.  The oracle is numpy float64; its matrix products run in numpy's
    multi-threaded BLAS, whose thread count is reported as `cores`."""
    import oracle
    from oracle.model import argmax_low, topk_desc
    from oracle.tree import derive_template, ancestors_or_self, build_tree_tokens, accept_walk, compact_kv

    class Src:
        def get(self, name, layer=None):
            return wsrc_np[(name, layer)]
    om = oracle.OracleModel(cfg, Src(), cache_layers=False)
    d = derive_template(tmpl_in.parent, tmpl_in.is_mask, tmpl_in.n_mask)
    ts = []
    na, nb = CPU_SAMPLE_LAYERS
    if cfg.n_layers < nb:
        na, nb = max(1, cfg.n_layers // 2), max(2, cfg.n_layers)
    for nl in (na, nb):
        t0 = time.perf_counter()
        tokens = build_tree_tokens(d, root_token, cand, 0, 0)
        pos = [ctx_len + d.depth[r] for r in range(d.R)]
        vis = [ancestors_or_self(d.parent, r) for r in range(d.R)]
        logits, k, v = oracle.forward_rows(om, tokens, d.is_mask, d.mask_index, pos, vis, kv_np[0], kv_np[1], n_layers=nl)
        greedy = [argmax_low(logits[r]) for r in range(d.T)]
        for g in range(d.G):
            for r in d.group_rows[g]:
                topk_desc(logits[r], d.kmax)
        path, _ = accept_walk(d, tokens, greedy)
        compact_kv(kv_np[0][:nl], kv_np[1][:nl], k, v, path)
        ts.append(time.perf_counter() - t0)
    layer = max((ts[1] - ts[0]) / (nb - na), 1e-9)
    head = max(ts[0] - na * layer, 0.0)
    full = head + cfg.n_layers * layer
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        threads = os.cpu_count() or 1
    return dict(value=d.R / full, unit="tokens/s", cores=int(threads),
                kind=f"oracle (numpy float64, matrix products in multi-threaded BLAS on {int(threads)} threads)",
                ms_per_step=full * 1e3,
                sample=f"one oracle step (token assignment, forward, selection, acceptance, K/V commit) with {na} and "
                       f"{nb} of {cfg.n_layers} layers + LM head at full width ({ts[0]:.1f}s + {ts[1]:.1f}s), the "
                       f"per-layer time extrapolated linearly to {cfg.n_layers} layers")


def run_workload(args, workload, steps, warmup, want_cpu_baseline):
    """One workload from model creation to the result dictionary."""
    import torch
    import synth
    import paper_2401_12522_amd as bita
    from paper_2401_12522_amd import binding as B

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    bita.lib()
    if args.calibration_copy_mb > 0:
        n = args.calibration_copy_mb * (1 << 20) // 4
        src_t = torch.ones(n, dtype=torch.float32, device="cuda")
        dst_t = torch.empty_like(src_t)
        for _ in range(4):
            torch.add(src_t, 1.0, out=dst_t)      # reads n*4 bytes, writes n*4 bytes
        torch.cuda.synchronize()
        del src_t, dst_t
    cfg = synth.get_config(workload)
    NB = args.batch
    if NB < 1:
        sys.exit("bench.py: --batch must be at least 1")
    if NB > 1 and args.mode == "planted":
        print("bench.py: --batch above 1 runs free (no planted drafts)", file=sys.stderr)
        args.mode = "free"
    if args.page_size and args.mode == "planted":
        print("bench.py: a paged cache runs free (no planted drafts)", file=sys.stderr)
        args.mode = "free"
    ctx_n = args.ctx or {"tiny": 64, "7b": 1024, "13b": 2048, "70b": 2048}[workload]
    tin = workload_template(synth, cfg, workload, args.tree)
    R = tin.rows
    children, depth_max = tree_shape(tin)
    total_steps = warmup + steps
    smax = ctx_n + (total_steps + 2) * (depth_max + 1) + 64
    smax = (smax + 63) // 64 * 64

    # ---- model: weights drawn on the GPU, packed layer by layer ----------------------------
    w = synth.SynthWeights(cfg, seed=args.seed, device="cuda")
    keep_layers = tuple(range(min(CPU_SAMPLE_LAYERS[1], cfg.n_layers)))
    wsrc_np = {}
    if want_cpu_baseline:
        for l in keep_layers:
            for n in ("wq", "wk", "wv", "wo", "w_gate", "w_up", "w_down", "attn_norm", "ffn_norm",
                      "prompt_k", "prompt_v"):
                wsrc_np[(n, l)] = w.numpy(n, l)
        for n in ("tok_emb", "mask_emb", "lm_head", "final_norm"):
            wsrc_np[(n, None)] = w.numpy(n)
    model = bita.Model(cfg, w, max_pos=smax + 64, free_source=True)
    tmpl = bita.TreeTemplate(tin.parent, tin.is_mask, tin.n_tree, cfg.n_mask)
    if args.page_size:
        kv = bita.PagedKVState(cfg, cfg.n_layers, NB, smax, R, args.page_size, seed=args.seed)
    else:
        kv = bita.KVState(cfg, cfg.n_layers, NB, smax, R)
    ctx_all = np.stack([synth.random_context(cfg.vocab, ctx_n, args.seed + 7919 * b) for b in range(NB)])
    ctx_tokens = ctx_all[0]
    prefill(B, model, kv, cfg, ctx_all)
    kv.resize_rows(cfg.n_layers, cfg, R)
    ctx0 = int(kv.ctx_len[0])
    assert ctx0 == ctx_n - 1 and bool((kv.ctx_len == ctx0).all())
    k_snap, v_snap = kv.k_cache.clone(), kv.v_cache.clone()

    kmax = tmpl.kmax
    buf = bita.StepBuffers(model, tmpl, NB, kmax)
    last_tokens = torch.tensor(ctx_all[:, -1].astype(np.int32), device="cuda")
    hint = ctx0 + (total_steps + 1) * (depth_max + 1)

    def reset_state():
        kv.k_cache.copy_(k_snap)
        kv.v_cache.copy_(v_snap)
        kv.ctx_len.fill_(ctx0)
        buf.bonus.copy_(last_tokens)
        buf.next_group.zero_()
        buf.next_shift.fill_(cfg.n_mask)        # first pass: no candidates, all drafts inactive
        buf.topk_ids.zero_()

    cand_buf = torch.zeros((1, cfg.n_mask, kmax), dtype=torch.int32, device="cuda")

    def one_step():
        if args.mode == "planted":
            B.decode_step(model, kv, hint, tmpl, buf, 1, buf.bonus, cand_buf)
        else:
            B.decode_step(model, kv, hint, tmpl, buf, NB, buf.bonus, buf.topk_ids, buf.next_group, buf.next_shift)

    reset_state()
    one_step()                                   # eager once (sets kernel attributes)
    torch.cuda.synchronize()
    graph = None
    if not args.no_graph:
        graph = torch.cuda.CUDAGraph()
        st = torch.cuda.Stream()
        with torch.cuda.stream(st):
            with torch.cuda.graph(graph, stream=st):
                one_step()
        torch.cuda.synchronize()

    def launch_step():
        if graph is not None:
            graph.replay()
        else:
            one_step()

    # ---- planted drafts ---------------------------------------------------------------------
    # Random-init weights never predict their own continuation, so candidates are planted from
    # a reference continuation obtained by plain one-token-per-pass greedy decoding on the
    # device.  The plan is made in an untimed dry run with the host in the loop: whenever the
    # tree pass and the one-row pass disagree on a token (a near-tie decided differently by
    # two summation orders), the reference is regenerated from the current state.  The kernels
    # are deterministic, so the timed run, replaying the recorded candidate tables from the
    # same initial state, follows the dry run exactly.
    cand_all, plan_acc, resyncs, dry_emitted, ar_ms_per_token = None, [], 0, None, None
    if args.mode == "planted":
        t1 = synth.attach_mask_groups(np.array([-1], np.int32), [], cfg.n_mask)
        tm1 = B.TreeTemplate(t1.parent, t1.is_mask, 1, cfg.n_mask)
        kv_ref = bita.KVState(cfg, cfg.n_layers, 1, smax, 1)
        b1 = B.StepBuffers(model, tm1, 1, 1)
        B.decode_step(model, kv_ref, smax - 8, tm1, b1, 1, b1.bonus, None)
        torch.cuda.synchronize()
        g1 = torch.cuda.CUDAGraph()
        st1 = torch.cuda.Stream()
        with torch.cuda.stream(st1):
            with torch.cuda.graph(g1, stream=st1):
                B.decode_step(model, kv_ref, smax - 8, tm1, b1, 1, b1.bonus, None)
        torch.cuda.synchronize()

        def reference_from_current(n):
            """Greedy continuation of the main state: n tokens, one row per pass."""
            kv_ref.k_cache.copy_(kv.k_cache)
            kv_ref.v_cache.copy_(kv.v_cache)
            kv_ref.ctx_len.copy_(kv.ctx_len)
            b1.bonus.copy_(buf.bonus)
            out_toks = torch.zeros(n, dtype=torch.int32, device="cuda")
            for i in range(n):
                g1.replay()
                out_toks[i:i + 1].copy_(b1.bonus)
            torch.cuda.synchronize()
            return out_toks.cpu().tolist()

        reset_state()
        tabs, dry_emitted = [], []
        ref, pos = reference_from_current((depth_max + 1) * 8), 0
        for t in range(total_steps):
            if len(ref) - pos < depth_max + 2:
                ref, pos = reference_from_current((depth_max + 1) * 8), 0
            rng = np.random.default_rng(1000 + t)
            depth_ok, col = planted_walk(children, depth_max, cfg.n_mask, rng)
            tab = synth.planted_candidates(ref[pos:], cfg.n_mask, kmax, depth_ok, col, cfg.vocab, 50 + t)
            tabs.append(tab)
            cand_buf.copy_(torch.tensor(tab[None], dtype=torch.int32))
            launch_step()
            torch.cuda.synchronize()
            na = int(buf.n_acc[0])
            em = buf.emitted[0, :na].cpu().tolist()
            dry_emitted.append(em)
            plan_acc.append(na)
            if em == ref[pos:pos + na]:
                pos += na
            else:                                 # near-tie decided differently: re-reference
                resyncs += 1
                ref, pos = reference_from_current((depth_max + 1) * 8), 0
        cand_all = torch.tensor(np.stack(tabs)[:, None], dtype=torch.int32, device="cuda")
        # the one-row greedy pass (plain autoregressive decoding with the same kernels), timed
        # beside the tree step: the paper's speedup is (this) x (tokens per step) / (step time)
        n_ar = 32
        reference_from_current(4)
        e_a, e_b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e_a.record()
        for _ in range(n_ar):
            g1.replay()
        e_b.record()
        torch.cuda.synchronize()
        ar_ms_per_token = e_a.elapsed_time(e_b) / n_ar
        del kv_ref
    reset_state()

    emitted_log = torch.zeros((total_steps, NB, depth_max + 1), dtype=torch.int32, device="cuda")
    nacc_log = torch.zeros((total_steps, NB), dtype=torch.int32, device="cuda")

    def run(t):
        if args.mode == "planted":
            cand_buf.copy_(cand_all[t])
        launch_step()
        emitted_log[t].copy_(buf.emitted)
        nacc_log[t].copy_(buf.n_acc)

    for t in range(warmup):
        run(t)
    torch.cuda.synchronize()
    ctx_start = kv.ctx_len.cpu().numpy().astype(np.int64)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    for t in range(warmup, total_steps):
        run(t)
    e1.record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    gpu_ms = e0.elapsed_time(e1)
    ms_per_step = wall * 1e3 / steps

    nacc = nacc_log.cpu().numpy()
    em = emitted_log.cpu().numpy()
    replay_ok = None
    if args.mode == "planted":
        replay_ok = all(em[t, 0, : nacc[t, 0]].tolist() == dry_emitted[t] for t in range(total_steps))
    grown = np.concatenate([np.zeros((1, NB), np.int64), np.cumsum(nacc[warmup:], axis=0)[:-1]])
    ctx_lens = ctx_start[None, :] + grown                      # [steps][batch] context length seen by each step
    kv_bytes = float(np.mean([cfg.kv_bytes([int(c) for c in row]) for row in ctx_lens]))
    bytes_per_step = cfg.weight_bytes() + kv_bytes
    gbps = bytes_per_step / (ms_per_step * 1e-3) / 1e9

    # ---- spread of the step time: the same run once more, an event behind every step -----------
    # (outside the timed region above; an event between two replays costs a queue packet)
    reset_state()
    for t in range(warmup):
        run(t)
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
    marks[0].record()
    for t in range(warmup, total_steps):
        run(t)
        marks[t - warmup + 1].record()
    torch.cuda.synchronize()
    per_step = np.array([marks[i].elapsed_time(marks[i + 1]) for i in range(steps)])
    step_ms = {"median": float(np.median(per_step)), "p10": float(np.percentile(per_step, 10)),
               "p90": float(np.percentile(per_step, 90)), "min": float(per_step.min()), "max": float(per_step.max()),
               "source": "HIP events behind every step of a second, untimed run of the same %d steps" % steps}

    # ---- dominant kernel (the skinny GEMM): HIP events around every launch, eager passes ------
    n_gemm = 4 * cfg.n_layers + 1
    prof_steps = max(1, min(4, steps))
    B.profile_enable(n_gemm * prof_steps)
    for t in range(prof_steps):
        one_step()
    torch.cuda.synchronize()
    g_ms, g_bytes = B.profile_read(n_gemm * prof_steps)
    gemm_avg_us = float(np.mean(g_ms)) * 1e3
    gemm_gbps = float(np.sum(g_bytes)) / (float(np.sum(g_ms)) * 1e-3) / 1e9
    standard = R == 68 and NB == 1 and not args.page_size
    prof_file, prof_gemm_us = ROCPROF_GEMM.get(workload, (None, None))
    roofline = {"bound": "hbm", "kernel": "gemm_skinny_kernel (all %d launches of a step)" % n_gemm,
                "achieved": gemm_gbps, "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": gemm_gbps / HBM_PEAK_GBPS,
                "frac_source": "HIP events recorded by the library around every GEMM launch on the launch stream, "
                               "%d eager steps run right after the timed graph replays (an event pair adds about "
                               "3 us to a launch, so this reads lower than rocprofv3)" % prof_steps,
                "frac_rocprof": (float(np.mean(g_bytes)) * n_gemm / (prof_gemm_us * 1e-6) / 1e9 / HBM_PEAK_GBPS
                                 if (standard and prof_gemm_us) else None),
                "frac_rocprof_source": prof_file if (standard and prof_gemm_us) else None,
                "traffic": GEMM_TRAFFIC_BYTES_PER_LAUNCH.get(workload) if standard else None,
                "traffic_source": ("rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of the stand-alone GEMM at this "
                                   "step's shapes, scaled by a copy kernel, committed in " + GEMM_TRAFFIC_SOURCE[workload]
                                   + " (a constant in bench.py, not measured by this run)")
                                  if (standard and workload in GEMM_TRAFFIC_SOURCE) else None,
                "avg_launch_us": gemm_avg_us,
                "bytes_per_launch": float(np.mean(g_bytes)),
                "gemm_ms_per_step": float(np.sum(g_ms)) / prof_steps}

    out = {
        "metric": "tree_verify_scored_tokens_per_s", "value": R * NB * steps / wall, "unit": "tokens/s",
        "n_gpus": 1, "steps": steps, "warmup": warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": f"llama2-{workload}-shaped random-init, ctx {ctx_n}, batch {NB}, "
                               f"{tin.n_tree}-node tree ({args.tree or 'default'}) + {R - tin.n_tree} mask rows, P={cfg.n_prompt}, mode {args.mode}",
                   "rows": R, "batch": NB, "graph": graph is not None, "page_size": args.page_size or None},
        "hbm_gbps": gbps, "hbm_frac_of_peak": gbps / HBM_PEAK_GBPS, "bytes_per_step": bytes_per_step,
        "gpu_ms_per_step": gpu_ms / steps, "step_ms": step_ms, "mean_accepted": float(np.mean(nacc[warmup:])),
        "generated_tokens_per_s": float(np.sum(nacc[warmup:])) / wall,
        "planted_resyncs": resyncs if args.mode == "planted" else None,
        "one_row_pass_ms": ar_ms_per_token,
        "speedup_over_one_row_passes": (ar_ms_per_token * float(np.mean(nacc[warmup:])) / ms_per_step
                                        if ar_ms_per_token else None),
        "timed_run_equals_dry_run": replay_ok,
        "roofline": roofline, "cpu_baseline": None,
    }

    if want_cpu_baseline:
        kv_np = ([k_snap[l, 0, :, :ctx0].permute(1, 0, 2).float().cpu().numpy() for l in keep_layers],
                 [v_snap[l, 0, :, :ctx0].permute(1, 0, 2).float().cpu().numpy() for l in keep_layers])
        cand = np.random.default_rng(3).integers(0, cfg.vocab, size=(cfg.n_mask, kmax)).astype(np.int32)
        out["cpu_baseline"] = cpu_baseline(cfg, wsrc_np, kv_np, tin, int(ctx_tokens[-1]), cand, ctx0)
    return out


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)
    headline = args.workload or "7b"
    out = run_workload(args, headline, args.steps, args.warmup, not args.no_cpu_baseline)
    plain = args.batch == 1 and not args.tree and not args.page_size and args.mode == "planted" and not args.ctx
    if args.workload is None and not args.no_second_leg and plain:
        import gc
        import torch
        gc.collect()
        torch.cuda.empty_cache()
        leg = SECOND_LEG
        t0 = time.perf_counter()
        try:
            res = run_workload(args, leg["workload"], leg["steps"], leg["warmup"], False)
            keep = ("steps", "warmup", "ms_per_step", "value", "unit", "config", "hbm_gbps", "hbm_frac_of_peak",
                    "bytes_per_step", "step_ms", "mean_accepted", "generated_tokens_per_s", "planted_resyncs", "one_row_pass_ms",
                    "speedup_over_one_row_passes", "timed_run_equals_dry_run", "roofline")
            entry = {k: res[k] for k in keep}
            entry["includes"] = "build_tree, verify_step, accept, compact_kv per step (one HIP graph)"
        except Exception as e:                    # the headline stands on its own; say why the leg is absent
            entry = {"error": f"{type(e).__name__}: {e}"}
        entry["leg_wall_s"] = time.perf_counter() - t0
        out["workloads"] = {leg["workload"]: entry}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
