"""Microbenchmark of the MFMA GEMM kernel on the shapes of the 20M-class worker step, each with
the epilogue the step uses, through the C ABI (als_k_gemm_ex).  Optional arguments force tile
variants, e.g. ``python -m paper_2401_09135_amd.gemm_bench 256x128x1 128x128x2`` (tile M x tile N
x LDS buffers); without arguments only the library's automatic choice is timed."""
from __future__ import annotations

import sys

import torch

from . import binding as A

T = 16384   # tokens per worker step (32 sequences of 512)
# name, M, N, K, a_layout, b_layout, epilogue (-1: plain store to fp32, 0: store bf16, 1 residual, 2 GELU, 3 x derivative)
SHAPES = [("qkv", T, 1536, 512, 0, 0, 0), ("wo+res", T, 512, 512, 0, 0, 1), ("ffn1+gelu", T, 2048, 512, 0, 0, 2),
          ("ffn2+res", T, 512, 2048, 0, 0, 1), ("head bf16", T, 8192, 512, 0, 0, 0),
          ("dffn2*gp", T, 2048, 512, 0, 1, 3), ("dffn1 f32", T, 512, 2048, 0, 1, -1), ("dqkv f32", T, 512, 1536, 0, 1, -1),
          ("do bf16", T, 512, 512, 0, 1, 0), ("dhead f32", T, 512, 8192, 0, 1, -1),
          ("dw ffn1", 512, 2048, T, 1, 0, 0), ("dw ffn2", 2048, 512, T, 1, 0, 0), ("dw qkv", 512, 1536, T, 1, 0, 0),
          ("dw wo", 512, 512, T, 1, 0, 0),
          ("dw head", 512, 8192, T, 1, 0, 0), ("square 8192", 8192, 8192, 8192, 0, 1, 0)]


def run(name, M, N, K, al, bl, epi, tile, ws, iters=20, dev="cuda:0"):
    a = torch.randn((M, K) if al == 0 else (K, M), device=dev).to(torch.bfloat16)
    b = torch.randn((K, N) if bl == 0 else (N, K), device=dev).to(torch.bfloat16)
    e = max(epi, 0)
    out_f32 = e == 1 or al == 1 or epi == -1
    c = torch.empty(M, N, dtype=torch.float32 if out_f32 else torch.bfloat16, device=dev)
    R = torch.randn(M, N, device=dev) if e == 1 else None
    C2 = torch.empty(M, N, dtype=torch.bfloat16, device=dev) if e == 2 else None
    U = torch.randn(M, N, device=dev).to(torch.bfloat16) if e == 3 else None
    A.lib.als_k_set_gemm_tile(*tile)
    f = lambda: A.k_gemm_ex(a, b, c, M, N, K, al, bl, True, e, R, C2, U, ws if al == 1 else None)
    try:
        for _ in range(10):   # first launches on fresh buffers run up to 10 % slower
            f()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(iters):
            f()
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / iters
        print(f"{name:12s} M{M:<6d} N{N:<5d} K{K:<6d} tile={tile}: {ms * 1e3:8.1f} us {2.0 * M * N * K / ms / 1e9:6.0f} TFLOP/s",
              flush=True)
    except A.AlsError as ex:
        print(f"{name:12s} tile={tile}: not supported ({str(ex)[:50]})", flush=True)
    finally:
        A.lib.als_k_set_gemm_tile(0, 0, 0)


def main(argv):
    ws = torch.empty(64 << 20, dtype=torch.uint8, device="cuda:0")     # split-K scratch
    tiles = [(0, 0, 0)] + [tuple(int(x) for x in t.split("x")) for t in argv]
    for sh in SHAPES:
        for t in tiles:
            run(*sh, t, ws)


if __name__ == "__main__":
    main(sys.argv[1:])
