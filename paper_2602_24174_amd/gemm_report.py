"""The tiled GEMM at the projection shapes of the verify steps (tasc_calibration_gemm), beside the vendor library.

    python -m paper_2602_24174_amd.gemm_report [--no-vendor]

1. A sweep of k on one full round of 256 x 256 tiles (2048 x 8192 outputs on 256 compute units): the slope is the cost of the
   main loop per 1024 of k, the intercept what a launch pays whatever its k (dispatch, first fetch, epilogue, drain).
2. The verify-step shapes of the three larger workloads (rows = batch x (k + 1)), each with the epilogue and k-slices the
   forward uses, and the time of torch.matmul (the vendor's GEMM library: plain bf16 output, no epilogue) for the same
   operand shapes -- the attainable rate at these shapes, not part of the product path.
"""
import argparse
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

STORE, RESID, SWIGLU, PARTIAL = 0, 1, 2, 4
PEAK_TFLOPS = 2500.0


def vendor_us(torch, M, N, K, iters=30):
    a = torch.randn(M, K, device="cuda", dtype=torch.bfloat16)
    w = torch.randn(N, K, device="cuda", dtype=torch.bfloat16)
    for _ in range(5):
        a @ w.t()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(iters):
        a @ w.t()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / iters * 1e3


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--no-vendor", action="store_true", help="skip the torch.matmul column")
    args = ap.parse_args()
    import torch
    import workload as W
    import paper_2602_24174_amd as T

    print("k sweep, one round of 256 x 256 tiles (M 2048, N 8192), microseconds per launch")
    rows = []
    for epi, name in ((SWIGLU, "SwiGLU, bf16 out"), (STORE, "fp32 store")):
        ts = [(K, T.tasc_calibration_gemm(2048, 8192, K, epi)) for K in (512, 1024, 2048, 4096, 8192)]
        slope = (ts[-1][1] - ts[-2][1]) / ((ts[-1][0] - ts[-2][0]) / 1024)
        fixed = ts[0][1] - slope * ts[0][0] / 1024
        ideal = 2.0 * 256 * 256 * 1024 / (PEAK_TFLOPS * 1e6 / 256)
        print(f"  {name:18s} " + "  ".join(f"k {K}: {us:6.1f}" for K, us in ts) +
              f"   -> {slope:.1f} us per 1024 of k ({ideal:.1f} at the MFMA peak: {ideal / slope:.0%}), {fixed:.1f} us per launch whatever k")
        rows.append((name, slope, fixed))

    print("verify-step projections (rows = batch x (k + 1)); TFLOP/s and the share of the 2.5 PFLOP/s peak in brackets")
    for cname in ("cfg5", "cfg4", "cfg3"):
        c = W.get_config(cname)
        M = c.batch * (c.k + 1)
        nqkv, nqo = (c.n_heads + 2 * c.n_kv_heads) * c.head_dim, c.n_heads * c.head_dim
        shapes = [("qkv", nqkv, c.d_model), ("output", c.d_model, nqo), ("gate/up + SwiGLU", 2 * c.d_ffn, c.d_model), ("down", c.d_model, c.d_ffn)]
        for name, N, K in shapes:
            if N % 128:
                continue
            epi = SWIGLU if name.startswith("gate") else STORE
            us = T.tasc_calibration_gemm(M, N, K, epi)
            line = f"  {cname} {name:17s} M {M:5d} N {N:6d} K {K:5d}: one slice {us:7.1f} us ({2.0 * M * N * K / us / 1e6:6.0f} TFLOP/s, {2.0 * M * N * K / us / 1e6 / PEAK_TFLOPS:.2f})"
            if name in ("qkv", "output", "down"):
                sl = [(s, T.tasc_calibration_gemm(M, N, K, PARTIAL, s)) for s in (2, 3, 4, 5, 6, 7, 8) if K // 64 >= 4 * s]
                line += "; k-sliced (the ordered reduction is a kernel of its own) " + " ".join(f"{s}: {us:.1f}" for s, us in sl)
            if not args.no_vendor:
                line += f"; vendor GEMM {vendor_us(torch, M, N, K):7.1f} us"
            print(line, flush=True)


if __name__ == "__main__":
    main()
