"""Micro-benchmark of the skinny GEMM entry point (bita_gemm) on the projection shapes of the
LLaMA-2 configurations, for use under rocprofv3:

    python -m paper_2401_12522_amd.gemm_bench 7b-qkv [--rows 68] [--reps 40] [--copy-mb 1024]

`7b-step` / `70b-step` run the five matrices of a layer (and the LM head) one after the other and
print, beside each, the sum over the launches of one step (layers x four matrices + LM head);
`--rows` takes a comma-separated list; `--no-tall` restricts many-row launches to passes of 5
m-tiles (bita_tune_gemm(-2, -1)) for a same-box comparison of the two pass forms.

Each repetition runs on a different copy of the weight matrix (at least 1.5 GB of copies in
rotation), so that no launch finds its weights in a cache.  --copy-mb also runs a plain
elementwise kernel that reads and writes that many MB, a launch of known traffic against which
the profiler's FETCH_SIZE / WRITE_SIZE readings can be scaled.  Prints the wall time per call
(three kernels: fragment layout, GEMM, split-K reduction); kernel-only figures come from the
profiler."""
import argparse

import torch

from . import binding as B

SHAPES = {
    "7b-qkv": (12288, 4096), "7b-o": (4096, 4096), "7b-gateup": (22016, 4096), "7b-down": (4096, 11008),
    "7b-lm": (32000, 4096),
    "70b-qkv": (10240, 8192), "70b-o": (8192, 8192), "70b-gateup": (57344, 8192), "70b-down": (8192, 28672),
    "70b-lm": (32000, 8192),
}


LAYERS = {"7b": 32, "70b": 80}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("shape", choices=sorted(SHAPES) + ["7b-step", "70b-step"])
    ap.add_argument("--rows", default="68")
    ap.add_argument("--reps", type=int, default=40)
    ap.add_argument("--copy-mb", type=int, default=0)
    ap.add_argument("--no-tall", action="store_true")
    args = ap.parse_args()
    L = B.lib()
    if args.no_tall:
        L.bita_tune_gemm(-2, -1)
    rows = [int(x) for x in args.rows.split(",")]
    if args.shape.endswith("-step"):
        wl = args.shape.split("-")[0]
        total = {m: 0.0 for m in rows}
        for name in ("qkv", "o", "gateup", "down", "lm"):
            for m in rows:
                us = one(L, f"{wl}-{name}", m, min(args.reps, 12), 0)
                total[m] += us * (1 if name == "lm" else LAYERS[wl])
        for m in rows:
            print(f"{args.shape}: rows {m}: {total[m] / 1e3:.3f} ms for the GEMM launches of one step "
                  f"({LAYERS[wl]} layers x 4 + LM head; layout and reduction kernels included)")
        return
    for m in rows:
        one(L, args.shape, m, args.reps, args.copy_mb)


def one(L, shape, M, reps, copy_mb):
    class A:
        pass
    args = A()
    args.shape, args.reps, args.copy_mb = shape, reps, copy_mb
    N, K = SHAPES[args.shape]
    nbytes = N * K * 2
    ncopy = max(2, int(1.5e9 // nbytes))
    g = torch.Generator(device="cuda").manual_seed(0)
    # bf16 bit patterns of finite values below 2^-7, directly in the packed layout (any layout is a matrix)
    wp = [torch.randint(0x3000, 0x3C00, (B.packed_bytes(N, K) // 2,), dtype=torch.int16, device="cuda",
                        generator=g).view(torch.uint8) for _ in range(ncopy)]
    a = torch.randn(2, M, K, device="cuda", generator=g).to(torch.bfloat16)
    ws = torch.empty(L.bita_gemm_workspace_bytes(M, N, K), dtype=torch.uint8, device="cuda")
    out = torch.empty((M, N), dtype=torch.float32, device="cuda")
    if args.copy_mb > 0:
        n = args.copy_mb * (1 << 20) // 4
        src = torch.ones(n, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(4):
            torch.add(src, 1.0, out=dst)
        torch.cuda.synchronize()

    def call(i):
        B._check(L.bita_gemm(a[0].data_ptr(), a[1].data_ptr(), M, K, K, wp[i % ncopy].data_ptr(), N,
                             ws.data_ptr(), ws.numel(), out.data_ptr(), torch.cuda.current_stream().cuda_stream))

    for i in range(3):
        call(i)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for i in range(args.reps):
        call(i)
    e1.record()
    torch.cuda.synchronize()
    us = e0.elapsed_time(e1) * 1e3 / args.reps
    plan = B.gemm_plan_info(M, N, K)
    print(f"{args.shape}: N {N} K {K} rows {M}: {nbytes / 1e6:.1f} MB of weights, {us:.1f} us per call "
          f"({nbytes / us / 1e6:.2f} TB/s incl. layout and reduction kernels; workgroup shape {plan['variant']}, "
          f"{plan['splits']} k splits, {plan['mt_pass'] or '-'} m-tiles per tall pass)", flush=True)
    return us


if __name__ == "__main__":
    main()
