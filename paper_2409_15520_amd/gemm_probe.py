"""Stand-alone rates of the bf16 MFMA path on the current GPU: the matrix cores alone (with zero and with random
operand bits, with and without the main loop's LDS fragment reads) and gemm_bf16_kernel on given shapes, tile
configurations and weight distributions.  Context for the roofline fractions bench.py reports.

    python -m paper_2409_15520_amd.gemm_probe                       # defaults: the 7B-shaped projections
    python -m paper_2409_15520_amd.gemm_probe --shapes 8192x4096x4096 --cfgs 6,14,15 --weights normal,zeros --rotate 6

Shapes are MxNxK (out[M, N] = x[M, K] w[N, K]^T).  --rotate R cycles through R operand sets so that nothing is warm
in the caches.  Prints one line per measurement."""
import argparse

import torch

from . import mpz_debug_gemm_bf16, mpz_debug_mfma_probe


def _time(fn, reps):
    for _ in range(3):
        fn(0)
    torch.cuda.synchronize()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    for i in range(reps):
        fn(i)
    b.record()
    torch.cuda.synchronize()
    return a.elapsed_time(b) / reps      # ms


def mfma_ceiling(stream):
    g = torch.Generator(device="cuda")
    g.manual_seed(1)
    out = torch.empty(256 * 512, dtype=torch.float32, device="cuda")
    ops = {"zeros": torch.zeros(12288, dtype=torch.bfloat16, device="cuda"),
           "random N(0,1)": torch.randn(12288, generator=g, device="cuda").to(torch.bfloat16)}
    iters = 20000
    for name, t in ops.items():
        for with_lds in (False, True):
            ms = _time(lambda i: mpz_debug_mfma_probe(t.data_ptr(), 256, iters, with_lds, out.data_ptr(), stream), 5)
            tf = 256 * 8 * iters * 8 * 32768.0 / ms / 1e9
            print(f"MFMA loop, operands {name}, {'6 LDS fragment reads per 8 MFMAs' if with_lds else 'registers only'}: "
                  f"{tf:.0f} TFLOP/s", flush=True)


def gemm_rates(stream, shapes, cfgs, weights, rotate, reps):
    g = torch.Generator(device="cuda")
    g.manual_seed(2)
    for (m, n, k) in shapes:
        for wd in weights:
            xs = [torch.randn(m, k, generator=g, device="cuda").to(torch.bfloat16) for _ in range(rotate)]
            if wd == "zeros":
                ws = [torch.zeros(n, k, dtype=torch.bfloat16, device="cuda") for _ in range(rotate)]
            else:
                ws = [(torch.randn(n, k, generator=g, device="cuda") * 0.02).to(torch.bfloat16) for _ in range(rotate)]
            outs = [torch.empty(m, n, dtype=torch.bfloat16, device="cuda") for _ in range(rotate)]
            for cfg in cfgs:
                def fn(i):
                    j = i % rotate
                    mpz_debug_gemm_bf16(m, n, k, xs[j].data_ptr(), ws[j].data_ptr(), None, -1, outs[j].data_ptr(), False,
                                        stream, cfg)
                ms = _time(fn, reps)
                print(f"GEMM {m}x{n}x{k}, tile configuration {cfg}, weights {wd}, {rotate} operand set(s): "
                      f"{ms * 1e3:.1f} us, {2.0 * m * n * k / ms / 1e9:.0f} TFLOP/s", flush=True)
            del xs, ws, outs


def main():
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--shapes", default="8192x4096x4096,8192x12288x4096,8192x4096x11008,32768x8192x2048")
    ap.add_argument("--cfgs", default="6", help="tile configurations (0 = chosen by shape)")
    ap.add_argument("--weights", default="normal,zeros")
    ap.add_argument("--rotate", type=int, default=1)
    ap.add_argument("--reps", type=int, default=30)
    ap.add_argument("--no-mfma-loop", action="store_true")
    args = ap.parse_args()
    stream = torch.cuda.current_stream().cuda_stream
    if not args.no_mfma_loop:
        mfma_ceiling(stream)
    shapes = [tuple(int(v) for v in s.split("x")) for s in args.shapes.split(",") if s]
    gemm_rates(stream, shapes, [int(c) for c in args.cfgs.split(",")], args.weights.split(","), args.rotate, args.reps)


if __name__ == "__main__":
    main()
