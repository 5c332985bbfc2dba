"""The tile loops of the head kernels as plain GEMMs beside the vendor GEMM (hipBLASLt through torch.mm)
on the shapes the library launches, plus the two-workgroups-per-CU layout that was tried and rejected.

    python -m paper_2510_11062_amd.bench_gemm

One JSON line per case: variant, shape, TFLOP/s, shader clock.  Shapes (bf16, fp32 accumulate):
  forward / dZ   vocabulary x tokens of one launch x H          151808 x 16384 x 2048   (short k)
  dHidden        tokens x H x vocabulary                         16384 x 2048 x 151936   (long k)
  dW             vocabulary x H x tokens of a super-chunk, both operands k-major  151808 x 2048 x 32768
  a square case  8192^3
nt4 / km4 are the same loops with 4 wavefronts of 128 x 128 per workgroup instead of 8 of 64 x 128: the
library uses them where k is long (dHidden, dW) and the 8-wavefront form where k = H (forward).
The probe (csrc/gemm_probe.hip, built by build.py) runs the library's own loop without any epilogue;
torch.mm is timed with the output written.  A measurement aid: nothing in the library calls this.
"""
from __future__ import annotations

import json
import os
import subprocess
import sys
import time

import torch

PKG = os.path.dirname(os.path.abspath(__file__))
PROBE = os.path.join(PKG, "gemm_probe")

SHAPES = [
    ("forward / dZ (short k)", "nt", 151808, 16384, 2048),
    ("forward / dZ (short k), 4 wavefronts", "nt4", 151808, 16384, 2048),
    ("dHidden (long k)", "nt", 16384, 2048, 151936),
    ("dHidden (long k), 4 wavefronts", "nt4", 16384, 2048, 151936),
    ("dW (k-major operands)", "km", 151808, 2048, 32768),
    ("dW (k-major operands), 4 wavefronts", "km4", 151808, 2048, 32768),
    ("square", "nt", 8192, 8192, 8192),
    ("microbenchmark shape", "nt", 37888, 32768, 1984),
    ("microbenchmark shape, two workgroups per CU (rejected layout)", "wg2", 37888, 32768, 1952),
]


def vendor(label, variant, M, N, K, iters=4):
    dev = torch.device("cuda:0")
    if variant.startswith("km"):
        a = torch.randn(K, M, device=dev, dtype=torch.bfloat16)
        b = torch.randn(K, N, device=dev, dtype=torch.bfloat16)
        fn = lambda: a.T @ b
    else:
        a = torch.randn(M, K, device=dev, dtype=torch.bfloat16)
        b = torch.randn(N, K, device=dev, dtype=torch.bfloat16)
        fn = lambda: a @ b.T
    for _ in range(2):
        fn()
    torch.cuda.synchronize()
    t = time.perf_counter()
    for _ in range(iters):
        fn()
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t) / iters
    return {"case": label, "variant": "torch.mm (vendor GEMM)", "M": M, "N": N, "K": K, "ms": dt * 1e3,
            "tflops": 2.0 * M * N * K / dt / 1e12}


def probe(label, variant, M, N, K):
    out = subprocess.run([PROBE, variant, str(M), str(N), str(K)], capture_output=True, text=True, timeout=600)
    if out.returncode != 0:
        raise RuntimeError(f"gemm_probe {variant} {M} {N} {K} failed: {out.stdout} {out.stderr}")
    rec = json.loads([l for l in out.stdout.splitlines() if l.startswith("{")][-1])
    rec["case"] = label
    rec["check"] = [l for l in out.stdout.splitlines() if "check" in l][-1]
    return rec


def main():
    if not torch.cuda.is_available():
        print("needs a GPU", file=sys.stderr)
        sys.exit(2)
    if not os.path.exists(PROBE):
        print(f"{PROBE} is missing: run python -m paper_2510_11062_amd.build", file=sys.stderr)
        sys.exit(2)
    for label, variant, M, N, K in SHAPES:
        print(json.dumps(probe(label, variant, M, N, K)), flush=True)
        if variant in ("nt", "km"):     # one vendor line per shape
            print(json.dumps(vendor(label, variant, M, N, K)), flush=True)


if __name__ == "__main__":
    main()
