"""Times single kernels of the generation library through their rl_op_* entry points (MI355X, synthetic operands).

    python -m paper_2406_14088_amd.opbench gemm --m 16384 --n 4096 --k 4096 --kernel tiled_packed
    python -m paper_2406_14088_amd.opbench gemm --m 128 --n 12288 --k 4096 --kernel packed --terms 2 --splits 2
    python -m paper_2406_14088_amd.opbench gemm --m 128 --n 11008 --k 4096 --kernel skinny --epilogue swiglu
    python -m paper_2406_14088_amd.opbench attention --batch 128 --heads 32 --kv-heads 32 --pos 255

The projection weights rotate over enough copies to exceed the caches (every launch streams them from HBM, as in a decode
step); `--iters` launches are timed between two HIP events on the launch stream.  Prints one line per case: microseconds per
launch, executed TFLOP/s and weight (or KV) GB/s.  Not used by the library, the tests or bench.py.
"""
from __future__ import annotations

import argparse

EPILOGUES = {"f32": 0, "swiglu": 1, "acc": 2}


def _time(fn, iters):
    import torch
    for _ in range(5):   # clocks and caches settle
        fn()
    torch.cuda.synchronize()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    for _ in range(iters):
        fn()
    b.record()
    torch.cuda.synchronize()
    return a.elapsed_time(b) / iters * 1e3


def bench_gemm(args):
    import torch
    from . import ops
    dev = "cuda:0"
    M, N, K = args.m, args.n, args.k
    epi = EPILOGUES[args.epilogue]
    nmat = 2 if epi == 1 else 1
    torch.manual_seed(0)
    A = torch.randn((args.terms * M, K), device=dev).to(torch.float16)
    if args.terms == 2:
        A[M:] *= 2.0 ** -11
    A_lo = A[M:] if args.terms == 2 else None
    copies = max(2, min(16, int(600e6 // (nmat * N * K * 2)))) if M <= 256 else 1
    Ws = [[(torch.randn((N, K), device=dev) * 0.02).to(torch.bfloat16) for _ in range(nmat)] for _ in range(copies)]
    Ps = None
    if args.kernel in ("packed", "tiled_packed", "packed_halves"):
        Ps = []
        for ws in Ws:
            row = []
            for w in ws:
                p = torch.empty((ops.packed_weight_bytes(N, K) // 2,), dtype=torch.int16, device=dev)
                ops.pack_weights(w, p)
                row.append(p)
            Ps.append(row)
    splits = args.splits if epi == 0 else 1
    if epi == 1:
        out = torch.empty((M, N), dtype=torch.float16, device=dev)
    else:
        out = torch.zeros((splits, M, N), dtype=torch.float32, device=dev)
    i = [0]

    def fn():
        c = i[0] % copies
        i[0] += 1
        if args.kernel == "packed":
            ops.gemm_packed(A[:M], Ps[c], [N] * nmat, K, out, N, A_lo=A_lo, M=M, split_stride=M * N, splits=splits, epilogue=epi,
                            nb=args.nb, rows_per_wg=args.rows_per_wg, depth=args.depth)
        elif args.kernel == "packed_halves":
            ops.gemm_packed_swiglu_halves(A[:M], Ps[c][0], Ps[c][1], N, K, out, N, M=M, depth=args.depth)
        elif args.kernel == "tiled_packed":
            ops.gemm_tiled_packed(A[:M], Ws[c], Ps[c], out, N, M=M, epilogue=epi, A_lo=A_lo)
        else:
            ops.gemm(A[:M], Ws[c], out, N, M=M, split_stride=M * N, splits=splits, epilogue=epi,
                     kernel=1 if args.kernel == "skinny" else 2, A_lo=A_lo)
    us = _time(fn, args.iters)
    flop = 2.0 * M * N * K * nmat * args.terms
    wbytes = nmat * N * K * 2
    print(f"gemm {args.kernel} M={M} N={N} K={K} epilogue={args.epilogue} terms={args.terms} splits={splits}: "
          f"{us:.1f} us  {flop / us / 1e6:.0f} TFLOP/s  weights {wbytes / us / 1e3:.0f} GB/s")


def bench_attention(args):
    import torch
    from . import ops
    dev = "cuda:0"
    B, Hq, Hkv, hd, pos = args.batch, args.heads, args.kv_heads, args.head_dim, args.pos
    S = args.max_seq or pos + 129
    torch.manual_seed(0)
    q = torch.randn((B, Hq, hd), device=dev)
    ks = vs = None
    if args.block_scaled:
        kc = torch.randint(-32767, 32768, (B, Hkv, S, hd), device=dev, dtype=torch.int32).to(torch.int16)
        vc = torch.randint(-32767, 32768, (B, Hkv, S, hd), device=dev, dtype=torch.int32).to(torch.int16)
        ks = torch.rand((B, Hkv, S), device=dev) / 32767 + 1e-5
        vs = torch.rand((B, Hkv, S), device=dev) / 32767 + 1e-5
    else:
        kc = torch.randn((B, Hkv, S, hd), device=dev).to(torch.float16)
        vc = torch.randn((B, Hkv, S, hd), device=dev).to(torch.float16)
    d_len = torch.full((1,), pos, dtype=torch.int32, device=dev)
    out = torch.empty((B, Hq * hd), dtype=torch.float16, device=dev)
    ws = torch.empty((max(1, ops.decode_attention_ws_floats(B, Hq, hd, args.nsplit)),), device=dev)
    us = _time(lambda: ops.decode_attention(q, kc, vc, d_len, out, ws, B, Hq, Hkv, hd, S, args.nsplit, kscale=ks, vscale=vs), args.iters)
    kv = 2.0 * B * Hkv * (pos + 1) * hd * 2
    print(f"decode attention B={B} heads={Hq}/{Hkv} hd={hd} position={pos} nsplit={args.nsplit}: {us:.1f} us  KV {kv / us / 1e3:.0f} GB/s")


def main():
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    sub = ap.add_subparsers(dest="what", required=True)
    g = sub.add_parser("gemm")
    g.add_argument("--m", type=int, default=128)
    g.add_argument("--n", type=int, default=4096)
    g.add_argument("--k", type=int, default=4096)
    g.add_argument("--kernel", default="packed", choices=["skinny", "tiled", "tiled_packed", "packed", "packed_halves"])
    g.add_argument("--epilogue", default="f32", choices=list(EPILOGUES))
    g.add_argument("--terms", type=int, default=1, choices=[1, 2], help="2: activations as a two-term half split")
    g.add_argument("--splits", type=int, default=1, help="K splits (fp32 partial outputs; epilogue f32 only)")
    g.add_argument("--nb", type=int, default=0, help="packed: column blocks per wavefront (0: the library's plan)")
    g.add_argument("--rows-per-wg", type=int, default=0, help="packed: 32, 64 or 128 activation rows per workgroup (0: by M)")
    g.add_argument("--depth", type=int, default=0, help="packed: weight chunks in flight, 2 or 4")
    g.add_argument("--iters", type=int, default=20)
    a = sub.add_parser("attention")
    a.add_argument("--batch", type=int, default=128)
    a.add_argument("--heads", type=int, default=32)
    a.add_argument("--kv-heads", type=int, default=32)
    a.add_argument("--head-dim", type=int, default=128)
    a.add_argument("--pos", type=int, default=255)
    a.add_argument("--max-seq", type=int, default=0)
    a.add_argument("--nsplit", type=int, default=1)
    a.add_argument("--iters", type=int, default=20)
    a.add_argument("--block-scaled", action="store_true")
    args = ap.parse_args()
    if args.what == "gemm":
        if args.epilogue == "swiglu" and args.terms == 2:
            ap.error("the SwiGLU projection takes one-term activations")
        if args.kernel == "packed_halves" and args.epilogue != "swiglu":
            ap.error("packed_halves is the fused gate/up projection: --epilogue swiglu")
        if args.terms == 2 and args.kernel == "skinny":
            ap.error("the row-major skinny kernel takes the second term as extra rows, not as --terms 2")
        bench_gemm(args)
    else:
        bench_attention(args)


if __name__ == "__main__":
    main()
