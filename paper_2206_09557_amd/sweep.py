"""Latency against footprint over (q, g) at one layer shape (paper section 3.4, figure 4b:
batch-1 latency follows the memory footprint of eq. 4, and a small group size raises it).

    python -m paper_2206_09557_amd.sweep [--m 12288 --n 12288 --iters 50]

The kernel is data-oblivious, so the packed buffers are filled with random key bytes and
random positive fp16 scales directly on the device (no quantiser run): sizes, layouts and
access pattern are those of a packed layer.  Copies of every configuration worth about 1 GB
rotate, so that neither the L2 nor the 256 MB Infinity Cache serves the weights.  Prints a markdown table.
"""
from __future__ import annotations

import argparse
import sys


def main(argv=None):
    ap = argparse.ArgumentParser()
    ap.add_argument("--m", type=int, default=12288)
    ap.add_argument("--n", type=int, default=12288)
    ap.add_argument("--iters", type=int, default=50)
    ap.add_argument("--q", type=str, default="1,2,3,4,5,6,7,8")
    ap.add_argument("--g", type=str, default="32,64,128,256,0")
    ap.add_argument("--preset", choices=["none", "workloads"], default="none",
                    help="workloads: every layer of the workload list (1024^2; OPT-13B q=4; OPT-175B q=3; LLaMA-65B "
                         "q in 2..4 x g in 32, 64, 128, row-wise with offsets) instead of one shape")
    ap.add_argument("--layout", choices=["planes", "planes_z", "shared"], default="planes",
                    help="planes: q scales per group (eq. 4); planes_z: plus one offset per group; "
                         "shared: one scale and one offset per group (uniformly quantised weights, appendix C)")
    args = ap.parse_args(argv)

    import torch

    from . import lutgemm as L

    if not torch.cuda.is_available():
        print("sweep: no GPU visible", file=sys.stderr)
        return 2
    L.lib()
    stream = torch.cuda.current_stream().cuda_stream
    gen = torch.Generator(device="cuda").manual_seed(1234)
    rows = []
    if args.preset == "workloads":
        from . import synth
        cases = [("1024^2", 1024, 1024, 3, 128, "planes")]
        cases += [(f"OPT-13B {k}", *synth.OPT_13B[k], 4, 128, "planes") for k in ("qkv", "out", "fc1", "fc2")]
        cases += [(f"OPT-175B {k}", *synth.OPT_175B[k], 3, 128, "planes") for k in ("qkv", "out", "fc1", "fc2")]
        cases += [(f"LLaMA-65B {k}", *synth.LLAMA_65B[k], q, g, "planes_z")
                  for k in ("qkv", "out", "gate_up", "down") for q in (2, 3, 4) for g in (32, 64, 128, 0)]
    else:
        cases = [("", args.m, args.n, q, g, args.layout) for q in [int(v) for v in args.q.split(",")]
                 for g in [int(v) for v in args.g.split(",")]]
    for name, m, n, q, g, layout in cases:
        x = torch.randn(n, device="cuda", generator=gen).half()
        y = torch.empty(m, dtype=torch.float16, device="cuda")
        args.layout = layout
        nb = L.lutgemm_bits_bytes(m, n, q)
        na = L.lutgemm_alpha_shared_bytes(m, n, g) if args.layout == "shared" else L.lutgemm_alpha_bytes(m, n, q, g)
        nz = 0 if args.layout == "planes" else L.lutgemm_z_bytes(m, n, g)
        copies = max(2, min(80, -(-int(1.0e9) // (nb + na + nz))))   # about 1 GB in rotation: nothing stays cached
        bits = [torch.randint(0, 256, (nb,), dtype=torch.uint8, device="cuda", generator=gen) for _ in range(copies)]
        alpha = [(torch.rand(na // 2, device="cuda", generator=gen) * 0.05 + 0.001).half() for _ in range(copies)]
        zs = [None] * copies if nz == 0 else [(torch.rand(nz // 2, device="cuda", generator=gen) * 0.02 - 0.01).half()
                                              for _ in range(copies)]
        flags = L.LUTGEMM_Y_F16 | (L.LUTGEMM_ALPHA_SHARED if args.layout == "shared" else 0)
        wsb = L.lutgemm_workspace_bytes(m, n, q, g)
        ws = torch.empty(wsb, dtype=torch.uint8, device="cuda")
        L.lutgemm_workspace_init(ws, wsb, stream)

        def go(i):
            L.lutgemm_gemv(x, bits[i % copies], alpha[i % copies], zs[i % copies], y, q, g, 8, m, n, flags, ws, wsb,
                           stream)

        for i in range(5):
            go(i)
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for i in range(args.iters):
            go(i)
        b.record()
        torch.cuda.synchronize()
        us = a.elapsed_time(b) * 1e3 / args.iters
        gg = n if g == 0 else g
        footprint = m * n * q // 8 + na + nz                    # bits + scales (+ offsets), bytes
        rows.append((name, m, n, layout, q, g, footprint, us))
        del bits, alpha, zs, ws
        print(f"[sweep] {name} {m}x{n} q={q} g={g or 'row'}: {us:.2f} us", file=sys.stderr, flush=True)
    if args.preset == "workloads":
        print("| layer | m x n | q | g | offsets | footprint MB | us / GEMV | GB/s | % of 8 TB/s |")
        print("|---|---|---|---|---|---|---|---|---|")
        for name, m, n, layout, q, g, fp, us in rows:
            print(f"| {name} | {m} x {n} | {q} | {g or 'row'} | {'yes' if layout != 'planes' else 'no'} | {fp / 1e6:.2f} | "
                  f"{us:.2f} | {fp / us / 1e3:.0f} | {fp / us / 1e3 / 80:.1f} |")
        return 0
    print(f"layout: {rows[0][3]}, m = {rows[0][1]}, n = {rows[0][2]}")
    print()
    print(f"| q | g | footprint MB | us / GEMV | GB/s | us per MB |")
    print("|---|---|---|---|---|---|")
    for _, _, _, _, q, g, fp, us in rows:
        print(f"| {q} | {g or 'row'} | {fp / 1e6:.2f} | {us:.2f} | {fp / us / 1e3:.0f} | {us / (fp / 1e6):.3f} |")
    return 0


if __name__ == "__main__":
    sys.exit(main())
