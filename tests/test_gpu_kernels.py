"""Kernel-level parity (GPU): skinny GEMM, tree-masked attention, integer kernels and the
vocabulary selection, each against the oracle through the C ABI."""
import numpy as np
import pytest
import torch

import oracle
import synth
from oracle.model import attend_row, topk_desc, argmax_low
from oracle.tree import derive_template, ancestors_or_self, build_tree_tokens, accept_walk, next_group_and_shift

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def bita():
    import paper_2401_12522_amd as b
    b.lib()
    return b


@pytest.mark.parametrize("M,N,K", [(1, 16, 32), (5, 48, 256), (68, 1024, 256), (68, 256, 688),
                                   (68, 4096, 4096), (80, 12288, 4096), (100, 1024, 1376), (16, 32000, 256),
                                   (272, 512, 512)])
def test_gemm_matches_float64_matmul(bita, M, N, K):
    g = torch.Generator().manual_seed(M * 7 + N)
    a = (torch.randn(M, K, generator=g)).to(torch.bfloat16)
    w = (torch.randn(N, K, generator=g) * 0.05).to(torch.bfloat16)
    ref = a.to(torch.float64).numpy() @ w.to(torch.float64).numpy().T
    wp = bita.pack_weight(w.cuda())
    out = bita.gemm(a.cuda(), wp, N).cpu().numpy()
    torch.cuda.synchronize()
    scale = np.abs(ref).max()
    assert np.abs(out - ref).max() <= 2e-5 * scale + 1e-6, (np.abs(out - ref).max(), scale)


@pytest.mark.parametrize("M,N,K", [(68, 4096, 4096), (68, 22016, 4096), (12, 256, 688), (1, 1024, 256),
                                   # other row counts: 2, 3, 7 and 10 m-tiles per pass, two passes, the wide variant
                                   (25, 4096, 1024), (40, 2048, 4096), (105, 4096, 2048), (170, 1024, 4096),
                                   (320, 2048, 1024), (25, 57344, 512), (105, 57344, 512), (333, 512, 688),
                                   # a last m-tile at most half full keeps both planes in one fragment
                                   # (rows 1..8 and 65..72); 9, 64 and 73 rows sit just outside
                                   (3, 2048, 1024), (4, 22016, 512), (5, 1024, 4096), (8, 4096, 688), (9, 1024, 1024),
                                   (64, 2048, 1024), (65, 4096, 1024), (69, 22016, 512), (72, 1024, 4096), (73, 2048, 688)])
def test_gemm_two_plane_activation(bita, M, N, K):
    """A = hi + lo (two bf16 planes): the product must match float64 on the summed operand
    to fp32-accumulation accuracy, i.e. the activation rounding is gone."""
    g = torch.Generator().manual_seed(N + K)
    a32 = torch.randn(M, K, generator=g)
    hi = a32.to(torch.bfloat16)
    lo = (a32 - hi.float()).to(torch.bfloat16)
    w = (torch.randn(N, K, generator=g) * 0.05).to(torch.bfloat16)
    a_sum = hi.to(torch.float64) + lo.to(torch.float64)
    ref = a_sum.numpy() @ w.to(torch.float64).numpy().T
    out = bita.gemm(hi.cuda(), bita.pack_weight(w.cuda()), N, a_lo=lo.cuda()).cpu().numpy()
    scale = np.abs(ref).max()
    assert np.abs(out - ref).max() <= 2e-5 * scale + 1e-6
    # and it is closer to the unrounded product than a single plane can be
    full = a32.to(torch.float64).numpy() @ w.to(torch.float64).numpy().T
    assert np.abs(out - full).max() <= 3e-4 * scale


@pytest.mark.parametrize("M,N,K,mt_pass", [(170, 12288, 4096, 6), (105, 57344, 1024, 7), (512, 4096, 11008, 8),
                                            (265, 22016, 512, 9)])
def test_gemm_tall_row_passes(bita, M, N, K, mt_pass):
    """Many-row shapes for which the launch heuristic takes tall row passes (6 to 9 m-tiles per pass
    and 16 weight tiles per workgroup and k group) instead of passes of 5: with and without a
    k split, a ragged last m-tile, a last pass shorter than the others."""
    from paper_2401_12522_amd import binding as BB
    plan = BB.gemm_plan_info(M, N, K)
    assert plan["variant"] == 12 and plan["mt_pass"] == mt_pass, plan
    g = torch.Generator().manual_seed(N + K + M)
    a32 = torch.randn(M, K, generator=g)
    hi = a32.to(torch.bfloat16)
    lo = (a32 - hi.float()).to(torch.bfloat16)
    w = (torch.randn(N, K, generator=g) * 0.05).to(torch.bfloat16)
    out = bita.gemm(hi.cuda(), bita.pack_weight(w.cuda()), N, a_lo=lo.cuda()).cpu().numpy()
    # float64 reference on a seeded sample of 2048 columns (every row): the full product of the
    # largest case is 46 GFLOP on the host
    cols = np.sort(np.random.default_rng(M).choice(N, size=min(N, 2048), replace=False))
    a_sum = (hi.to(torch.float64) + lo.to(torch.float64)).numpy()
    ref = a_sum @ w[torch.tensor(cols)].to(torch.float64).numpy().T
    scale = np.abs(ref).max()
    assert np.isfinite(out).all()
    assert np.abs(out[:, cols] - ref).max() <= 2e-5 * scale + 1e-6
    # the columns outside the sample: against the same library run in passes of 5 m-tiles
    BB.lib().bita_tune_gemm(-2, -1)
    try:
        assert BB.gemm_plan_info(M, N, K)["mt_pass"] == 0
        base = bita.gemm(hi.cuda(), bita.pack_weight(w.cuda()), N, a_lo=lo.cuda()).cpu().numpy()
    finally:
        BB.lib().bita_tune_gemm(-1, -1)
    assert np.abs(out - base).max() <= 2e-5 * scale + 1e-6


def _attention_case(bita, B, Hq, Hkv, hd, P, ctx_lens, tree_parent, attach, n_mask, seed, smax=None,
                    two_plane_q=True):
    """Returns (worst error of the bf16 output, worst error of output + residual plane)."""
    rng = np.random.default_rng(seed)
    tin = synth.attach_mask_groups(tree_parent, attach, n_mask)
    d = derive_template(tin.parent, tin.is_mask, n_mask)
    R = d.R
    smax = smax or (max(ctx_lens) + 8)
    r16 = lambda *s: synth.bf16_round(rng.normal(size=s))   # noqa: E731
    q_full = rng.normal(size=(B, R, Hq, hd))
    q_hi = synth.bf16_round(q_full)
    q_lo = synth.bf16_round(q_full - q_hi) if two_plane_q else None
    q = q_hi + (q_lo if two_plane_q else 0.0)          # what the kernel is given, exactly
    kc, vc = r16(B, Hkv, smax, hd), r16(B, Hkv, smax, hd)
    kt, vt = r16(B, Hkv, R, hd), r16(B, Hkv, R, hd)
    kt_lo = vt_lo = None
    if two_plane_q:     # the pass rows' K/V carry a second plane too (large here, so that a
        kt_lo = r16(B, Hkv, R, hd) * 0.25               # dropped or misplaced plane fails the test)
        vt_lo = r16(B, Hkv, R, hd) * 0.25
    pk, pv = (r16(Hkv, P, hd), r16(Hkv, P, hd)) if P else (None, None)
    tmpl = bita.TreeTemplate(tin.parent, tin.is_mask, tin.n_tree, n_mask)
    tb = lambda a: None if a is None else torch.tensor(a).to(torch.bfloat16).cuda()   # noqa: E731
    out = bita.tree_attention(tmpl, tb(q_hi), tb(kc), tb(vc), tb(kt), tb(vt), tb(pk), tb(pv),
                              torch.tensor(ctx_lens, dtype=torch.int32, device="cuda"), max(ctx_lens),
                              q_lo=tb(q_lo), k_tree_lo=tb(kt_lo), v_tree_lo=tb(vt_lo), two_plane_out=True)
    torch.cuda.synchronize()
    out, out_lo = (x.to(torch.float64).cpu().numpy().reshape(B, R, Hq, hd) for x in out)
    out2 = out + out_lo
    if two_plane_q:
        kt, vt = kt + kt_lo, vt + vt_lo                 # what the kernel is given, exactly
    worst = worst2 = 0.0
    for b in range(B):
        Lc = ctx_lens[b]
        for r in range(R):
            vis = ancestors_or_self(d.parent, r)
            ks = [kc[b, :, :Lc].transpose(1, 0, 2), kt[b][:, vis].transpose(1, 0, 2)]
            vs = [vc[b, :, :Lc].transpose(1, 0, 2), vt[b][:, vis].transpose(1, 0, 2)]
            if d.is_mask[r] and P:
                ks.insert(0, pk.transpose(1, 0, 2))
                vs.insert(0, pv.transpose(1, 0, 2))
            ref = attend_row(q[b, r], np.concatenate(ks), np.concatenate(vs), Hq, Hkv)
            worst = max(worst, np.abs(out[b, r] - ref).max())
            worst2 = max(worst2, np.abs(out2[b, r] - ref).max())
    return worst, worst2


# bf16 output rounding (2^-9 relative on values of order 1) plus bf16 probabilities: 2e-2 abs
ATT_TOL = 2e-2
# Regression bound on the two-plane output (value + rounding residual, the form the step hands to
# the output projection), about ten times the measured error (3e-7 .. 1.4e-5 over the cases
# below, 1.4e-6 at the grouped-query benchmark shape).  One key wrongly visible or hidden among a
# few thousand moves an output by about 1e-3: this bound sees it at every context length of the
# cases below, the 2e-2 above only at the short ones.
ATT_TWO_PLANE_REGRESSION = 1e-4


@pytest.mark.parametrize("case", [
    dict(B=1, Hq=4, Hkv=4, hd=64, P=8, ctx=[63], T=8, depth=3, attach=[0], n=4),
    dict(B=1, Hq=4, Hkv=2, hd=64, P=8, ctx=[300], T=8, depth=3, attach=[0, 3], n=4),
    dict(B=2, Hq=4, Hkv=1, hd=128, P=16, ctx=[130, 517], T=64, depth=6, attach=[0], n=4),
    dict(B=1, Hq=2, Hkv=2, hd=128, P=0, ctx=[0], T=5, depth=2, attach=[0], n=2),
    dict(B=1, Hq=2, Hkv=2, hd=128, P=16, ctx=[1], T=1, depth=0, attach=[], n=4),
    dict(B=3, Hq=8, Hkv=1, hd=128, P=16, ctx=[1024, 96, 2047], T=64, depth=5, attach=[0], n=4),
    dict(B=1, Hq=2, Hkv=1, hd=64, P=4, ctx=[200], T=21, depth=4, attach=list(range(21)), n=4),
    # three query heads per K/V head (no pairing), a context long enough for a key split by
    # length (more than 256 chunks), and the largest template (512 rows, 32 row tiles)
    dict(B=2, Hq=3, Hkv=1, hd=128, P=16, ctx=[77, 400], T=20, depth=4, attach=[0], n=4),
    dict(B=1, Hq=2, Hkv=2, hd=128, P=16, ctx=[9000], T=8, depth=3, attach=[0], n=4),
    dict(B=1, Hq=2, Hkv=1, hd=64, P=8, ctx=[50], T=508, depth=9, attach=[0], n=4),
])
def test_tree_attention_matches_oracle(bita, case):
    parent = synth.random_tree(case["T"], max(case["depth"], 1), 11) if case["T"] > 1 else np.array([-1], np.int32)
    err, err2 = _attention_case(bita, case["B"], case["Hq"], case["Hkv"], case["hd"], case["P"], case["ctx"],
                                parent, case["attach"], case["n"], seed=5)
    print(f"attention {case['Hq']}/{case['Hkv']} heads, ctx {case['ctx']}: bf16 out {err:.2e}, two planes {err2:.2e}", flush=True)
    assert err < ATT_TOL, err
    assert err2 < ATT_TWO_PLANE_REGRESSION, err2


def test_tree_attention_at_the_grouped_query_benchmark_shape(bita):
    """The kernel-only configuration: 64 query heads on 8 K/V heads, head dim 128, 16 prefix
    tokens, batch 8 with seeded context lengths uniform in [1024, 4096], 64 tree rows of depth
    <= 6 plus 4 mask rows, N(0, 1) K/V.  Every row of every sequence against the oracle's
    attention over its explicit key list."""
    ctx = [int(x) for x in np.random.default_rng(4).integers(1024, 4097, size=8)]
    ctx[0], ctx[7] = 4096, 1024                           # both ends of the range are present
    parent = synth.random_tree(64, 6, 11)
    err, err2 = _attention_case(bita, 8, 64, 8, 128, 16, ctx, parent, [0], 4, seed=21, smax=4096 + 8)
    print(f"attention 64/8 heads, batch 8, ctx {ctx}: bf16 out {err:.2e}, two planes {err2:.2e}", flush=True)
    assert err < ATT_TOL, err
    assert err2 < ATT_TWO_PLANE_REGRESSION, err2


def test_tree_attention_chain_equals_causal(bita):
    """Special case: a chain template is plain causal attention over [cache | chain]."""
    err, err2 = _attention_case(bita, 1, 4, 4, 64, 0, [100], synth.chain_tree(40), [], 4, seed=6)
    assert err < ATT_TOL and err2 < ATT_TWO_PLANE_REGRESSION, (err, err2)
    err, err2 = _attention_case(bita, 1, 4, 4, 64, 0, [100], synth.chain_tree(40), [], 4, seed=6, two_plane_q=False)
    assert err < ATT_TOL and err2 < ATT_TWO_PLANE_REGRESSION, (err, err2)


def test_select_orders_equal_values_by_index(bita):
    """Selection alone on crafted logits: runs of equal maxima, equal values across the 16-byte
    and thread strides, +0 / -0, negative-only rows, very large and very small magnitudes.
    Greedy index and sorted top-k must equal the oracle's (value descending, lower id first)."""
    from oracle.model import argmax_low, topk_desc
    n_mask, kmax, V = 4, 6, 32000
    par = synth.full_branching_tree([2, 2], 7)
    tin = synth.attach_mask_groups(par, [0], n_mask)
    tmpl = bita.TreeTemplate(tin.parent, tin.is_mask, tin.n_tree, n_mask)
    R = tin.rows
    rng = np.random.default_rng(12)
    lg = rng.normal(size=(2, R, V)).astype(np.float32)
    lg[0, 0, [5, 4099, 31999]] = 9.0                      # three equal maxima, far apart
    lg[0, 1, :] = -3.5                                    # a constant row
    lg[0, 2, :] = -np.abs(lg[0, 2, :]) - 1.0              # all negative ...
    lg[0, 2, [17, 16]] = -0.25                            # ... with an equal pair as maximum
    lg[0, 3, :] = -1.0
    lg[0, 3, 777] = -0.0                                  # -0 and +0 are one value: the lower id wins
    lg[0, 3, 20000] = 0.0
    lg[0, 4, :] = 1e-30 * rng.normal(size=V)              # tiny magnitudes of both signs
    lg[0, 5, [1, 2, 3]] = [3e38, -3e38, 3e38]             # near the float range
    for r in range(tin.n_tree, R):                        # mask rows: ties inside and across the top-k
        lg[1, r, :] = np.round(lg[1, r, :] * 2) / 2       # many equal values
        lg[1, r, [31990 - r, 8, 4104]] = 40.0
    dev = torch.tensor(lg, device="cuda")
    am, ids, val = bita.select(tmpl, dev, kmax)
    torch.cuda.synchronize()
    am, ids, val = am.cpu().numpy(), ids.cpu().numpy(), val.cpu().numpy()
    d = derive_template(tin.parent, tin.is_mask, n_mask)
    for b in range(2):
        for r in range(d.T):
            assert am[b, r] == argmax_low(lg[b, r].astype(np.float64)), (b, r)
        for j, r in enumerate(range(d.T, R)):
            ref_ids, ref_val = topk_desc(lg[b, r].astype(np.float64), kmax)
            assert ids[b, j].tolist() == list(ref_ids), (b, r)
            assert np.array_equal(val[b, j].astype(np.float64) + 0.0, np.asarray(ref_val) + 0.0), (b, r)


def test_integer_kernels_match_oracle(bita):
    rng = np.random.default_rng(0)
    for trial in range(40):
        T = int(rng.integers(1, 70))
        n = int(rng.integers(1, 5))
        parent = synth.random_tree(T, int(rng.integers(1, 7)), trial)
        per_node = trial % 3 == 0 and T <= 40
        tin = synth.attach_mask_groups(parent, list(range(T)) if per_node else [0], n)
        d = derive_template(tin.parent, tin.is_mask, n)
        tmpl = bita.TreeTemplate(tin.parent, tin.is_mask, tin.n_tree, n)
        assert (tmpl.rows, tmpl.n_tree, tmpl.n_groups, tmpl.depth, tmpl.kmax) == (d.R, d.T, d.G, d.tree_depth, d.kmax)
        if d.kmax > 64:          # wider than the library's top-k limit: must be refused, not run
            from paper_2401_12522_amd.binding import BitaError, build_tree
            z = torch.zeros((1, d.G * n, d.kmax), dtype=torch.int32, device="cuda")
            with pytest.raises(BitaError):
                build_tree(tmpl, z[0, 0, :1], z, None, None, 1, torch.zeros((1, d.R), dtype=torch.int32, device="cuda"))
            continue
        B = 3
        vocab = 5
        kmax = d.kmax
        cand = rng.integers(0, vocab, size=(B, d.G * n, kmax)).astype(np.int32)
        roots = rng.integers(0, vocab, size=B).astype(np.int32)
        groups = rng.integers(0, d.G, size=B).astype(np.int32)
        shifts = rng.integers(0, n + 1, size=B).astype(np.int32)
        dev = lambda a: torch.tensor(a, dtype=torch.int32, device="cuda")   # noqa: E731
        token = torch.zeros((B, d.R), dtype=torch.int32, device="cuda")
        from paper_2401_12522_amd import binding as BB
        BB.build_tree(tmpl, dev(roots), dev(cand), dev(groups), dev(shifts), B, token)
        greedy = rng.integers(0, vocab, size=(B, d.T)).astype(np.int32)

        class Buf:
            pass
        buf = Buf()
        buf.token, buf.argmax = token, dev(greedy)
        z = lambda *s: torch.zeros(s, dtype=torch.int32, device="cuda")   # noqa: E731
        buf.path, buf.emitted = z(B, d.tree_depth + 1), z(B, d.tree_depth + 1)
        buf.n_acc, buf.bonus, buf.next_group, buf.next_shift = z(B), z(B), z(B), z(B)
        BB.accept(tmpl, buf, B)
        torch.cuda.synchronize()
        for b in range(B):
            ref_tok = build_tree_tokens(d, roots[b], cand[b], int(groups[b]), int(shifts[b]))
            assert token[b].cpu().tolist() == ref_tok
            path, bonus = accept_walk(d, ref_tok, list(greedy[b]))
            na = int(buf.n_acc[b])
            assert na == len(path) and buf.path[b, :na].cpu().tolist() == path
            assert all(x == -1 for x in buf.path[b, na:].cpu().tolist())
            assert int(buf.bonus[b]) == bonus
            assert buf.emitted[b, :na].cpu().tolist() == [ref_tok[c] for c in path[1:]] + [bonus]
            g, s = next_group_and_shift(d, path)
            assert (int(buf.next_group[b]), int(buf.next_shift[b])) == (g, s)


def test_template_errors(bita):
    from paper_2401_12522_amd.binding import BitaError
    for parent, is_mask, T, n in [([-1, 1], [0, 0], 2, 1), ([0, 0], [0, 0], 2, 1), ([-1, 0, 0], [0, 1, 0], 2, 1),
                                  ([-1, 0, 1], [0, 1, 1], 1, 3), ([-1, 0, 0], [0, 1, 1], 1, 1)]:
        with pytest.raises(BitaError) as e:
            bita.TreeTemplate(parent, is_mask, T, n)
        assert e.value.code == -2
