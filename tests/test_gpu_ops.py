"""GPU parity of every single kernel (rl_op_* entry points of the C ABI) against the CPU oracle's
sub-functions on the same seeded inputs.  Sizes span several tiles and ragged tails.

Number formats: weights are bf16, activations and cache slabs are IEEE half ("f16"); both sides get
identical values.  Tolerances (derived from the arithmetic): the kernels accumulate in fp32 (relative
error ~1e-6 per term, growing like sqrt(K)); outputs stored as f16 carry one rounding (relative
2^-11); weights below 2^-14 in magnitude are widened onto the f16 subnormal grid (absolute 2^-25).
Attention additionally uses a fast exponential (relative ~2e-6) and, in prefill, probabilities
rounded to f16 for the matrix cores (relative 2^-11 per term of a convex combination).
"""
import numpy as np
import pytest
import torch

from oracle import orc
from tests.gpu_util import F16_EPS, DEV, bits, np64, randn_bf16, randn_f16, randn_f32, step

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ops():
    from paper_2406_14088_amd import ops as o
    return o


def test_embed_exact(ops):
    emb = randn_bf16((1000, 264), 1)
    tok = torch.tensor([0, 999, 5, 5, 123, 77], dtype=torch.int32, device=DEV)
    x = torch.empty((6, 264), dtype=torch.float32, device=DEV)
    ops.embed(tok, emb, x)
    torch.cuda.synchronize()
    assert torch.equal(x, emb[tok.long()].float())


@pytest.mark.parametrize("d", [256, 4096, 5120, 8192])
@pytest.mark.parametrize("nsplit", [0, 3])
def test_add_rmsnorm(ops, d, nsplit):
    M = 5
    x = randn_f32((M, d), 10 + d, std=2.0)
    part = randn_f32((max(nsplit, 1), M, d), 11 + d)
    gain = (1.0 + 0.3 * randn_f32((d,), 12)).to(torch.bfloat16)
    h = torch.empty((M, d), dtype=torch.float16, device=DEV)
    h_lo = torch.empty((M, d), dtype=torch.float16, device=DEV) if nsplit else None
    x0 = x.clone()
    ops.add_rmsnorm(x, part, nsplit, M * d, gain, 1e-5, h, h_lo)
    torch.cuda.synchronize()
    xs = np64(x0) + (np64(part[:nsplit]).sum(0) if nsplit else 0.0)
    assert np.abs(np64(x) - xs).max() <= 1e-6 * (1 + np.abs(xs).max())
    ref = orc.rmsnorm(xs, bits(gain), float(np.float32(1e-5)))
    err = np.abs(np64(h) - ref)
    assert (err <= 0.5 * F16_EPS * np.abs(ref) * 1.01 + 1e-6).all()
    if h_lo is not None:     # two-term split: h + h_lo reproduces the fp32 value (fp32 arithmetic: ~1e-6 relative)
        err2 = np.abs(np64(h) + np64(h_lo) - ref)
        assert (err2 <= 2e-6 * np.abs(ref) + 1e-7).all(), err2.max()


GEMM_CASES = [
    # M, K, rows of up to three matrices, splits, kernel (1 skinny / 2 tiled)
    (1, 256, (256,), 1, 1), (4, 688, (256,), 2, 1), (4, 256, (256, 256, 256), 1, 1), (33, 688, (1000, 72), 3, 1),
    (128, 4096, (512, 128, 128), 4, 1), (200, 1024, (688,), 2, 1), (256, 512, (300,), 1, 1), (64, 256, (1024,), 1, 1),
    (64, 688, (256,), 1, 2), (300, 256, (688, 256), 1, 2), (130, 1000, (1000,), 1, 2), (1024, 256, (16384,), 1, 2),
    (1100, 136, (16400,), 1, 2),
]


@pytest.mark.parametrize("M,K,rows,splits,kernel", GEMM_CASES)
def test_gemm_f32(ops, M, K, rows, splits, kernel):
    step(f"gemm M={M} K={K} rows={rows} splits={splits} kernel={kernel}")
    A = randn_f16((M, K), 20 + M)
    Ws = [randn_bf16((r, K), 30 + i + r, std=0.05) for i, r in enumerate(rows)]
    N = sum(rows)
    out = torch.full((splits, M, N), float("nan"), dtype=torch.float32, device=DEV)
    ops.gemm(A, Ws, out, N, split_stride=M * N, splits=splits, epilogue=0, kernel=kernel)
    torch.cuda.synchronize()
    got = np64(out).sum(0)
    ref = np.concatenate([orc.linear(bits(w), np64(A)) for w in Ws], axis=1)
    tol = 2e-6 * np.sqrt(K) * (np.abs(ref).max() + 1.0)
    assert np.isfinite(got).all()
    assert np.abs(got - ref).max() <= tol, (np.abs(got - ref).max(), tol)


@pytest.mark.parametrize("M,kernel", [(4, 1), (128, 1), (70, 2), (600, 2)])
def test_gemm_row_stride_and_accumulate(ops, M, kernel):
    # A with a row stride (the LM head reads the last prompt position of every sequence) and the residual-add epilogue
    K, N, T = 256, 264, 3
    buf = randn_f16((M * T, K), 40)
    A = buf[T - 1::T]
    assert A.stride(0) == T * K
    W = randn_bf16((N, K), 41, std=0.05)
    out = randn_f32((M, N), 42)
    base = np64(out)
    ops.gemm(A, [W], out, N, M=M, lda=T * K, epilogue=2, kernel=kernel)
    torch.cuda.synchronize()
    ref = base + orc.linear(bits(W), np64(A))
    assert np.abs(np64(out) - ref).max() <= 1e-4


@pytest.mark.parametrize("M,K,N,epilogue", [(300, 256, 688, 0), (1100, 136, 300, 0), (600, 1000, 264, 2)])
def test_gemm_tiled_two_term_activations(ops, M, K, N, epilogue):
    """(A + A_lo) W^T in one pass of the large-M kernel: the K loop walks [A | A_lo] against [W | W]."""
    both = randn_f16((2 * M, K), 43)
    both[M:] *= 2.0 ** -11
    A, A_lo = both[:M], both[M:]
    W = randn_bf16((N, K), 44, std=0.05)
    out = randn_f32((M, N), 45)
    base = np64(out) if epilogue == 2 else 0.0
    ops.gemm(A, [W], out, N, epilogue=epilogue, kernel=2, A_lo=A_lo)
    torch.cuda.synchronize()
    ref = base + orc.linear(bits(W), np64(A) + np64(A_lo))
    tol = 2e-6 * np.sqrt(K) * (np.abs(ref).max() + 1.0)
    assert np.abs(np64(out) - ref).max() <= tol


@pytest.mark.parametrize("M,K,F,kernel", [(4, 256, 688, 1), (128, 512, 1000, 1), (256, 256, 72, 1), (100, 256, 688, 2),
                                          (1024, 128, 8200, 2)])
def test_gemm_swiglu(ops, M, K, F, kernel):
    step(f"swiglu M={M} K={K} F={F} kernel={kernel}")
    A = randn_f16((M, K), 50)
    Wg, Wu = randn_bf16((F, K), 51, std=0.1), randn_bf16((F, K), 52, std=0.1)
    out = torch.zeros((M, F), dtype=torch.float16, device=DEV)
    ops.gemm(A, [Wg, Wu], out, F, epilogue=1, kernel=kernel)
    torch.cuda.synchronize()
    g, u = orc.linear(bits(Wg), np64(A)), orc.linear(bits(Wu), np64(A))
    ref = g / (1.0 + np.exp(-g)) * u
    err = np.abs(np64(out) - ref)
    assert (err <= 0.5 * F16_EPS * np.abs(ref) * 1.02 + 2e-5).all(), err.max()


def pack(ops, W):
    N, K = W.shape
    P = torch.full((ops.packed_weight_bytes(N, K) // 2,), -1, dtype=torch.int16, device=DEV)
    ops.pack_weights(W, P)
    return P


TILED_PACKED_CASES = [
    # M, K, rows, epilogue, two activation terms: all at least 256 tiles of 256 x 256 (below that the call runs rl_op_gemm's kernel)
    (1100, 136, (16400,), 0, False), (1024, 256, (8192, 4200, 4100), 0, False), (1030, 200, (13100,), 0, True),
    (1100, 72, (16400,), 2, False), (1281, 104, (300, 13000), 2, True), (1024, 128, (8200, 8200), 1, False), (1300, 1000, (6600, 6600), 1, False),
]


@pytest.mark.parametrize("M,K,rows,epilogue,two_terms", TILED_PACKED_CASES)
def test_gemm_tiled_from_fragment_order_copies_equals_the_register_staged_kernel(ops, M, K, rows, epilogue, two_terms):
    """Same products, same order of the sums over K: the direct-to-LDS main loop stores the bits the register-staged one does
    (whose oracle parity its own tests establish); one output row is also checked against the oracle directly."""
    step(f"tiled packed M={M} K={K} rows={rows} epilogue={epilogue} two_terms={two_terms}")
    A = randn_f16(((2 if two_terms else 1) * M, K), 60 + M)
    if two_terms:
        A[M:] *= 2.0 ** -11
    A_lo = A[M:] if two_terms else None
    Ws = [randn_bf16((r, K), 61 + i, std=0.05) for i, r in enumerate(rows)]
    Ps = [pack(ops, W) for W in Ws]
    N = rows[0] if epilogue == 1 else sum(rows)
    if epilogue == 1:
        ref, out = (torch.zeros((M, N), dtype=torch.float16, device=DEV) for _ in range(2))
    else:
        base = randn_f32((M, N), 62)
        ref, out = base.clone(), base.clone()
    ops.gemm(A[:M], Ws, ref, N, M=M, epilogue=epilogue, kernel=2, A_lo=A_lo)
    ops.gemm_tiled_packed(A[:M], Ws, Ps, out, N, M=M, epilogue=epilogue, A_lo=A_lo)
    torch.cuda.synchronize()
    bits_of = (lambda x: x.view(torch.int16)) if epilogue == 1 else (lambda x: x.view(torch.int32))
    assert torch.equal(bits_of(out), bits_of(ref))
    m = M - 3
    x = np64(A[m]) + (np64(A[M + m]) if two_terms else 0.0)
    y = [np64(W) @ x for W in Ws]
    if epilogue == 1:
        want = y[0] / (1.0 + np.exp(-y[0])) * y[1]
        assert (np.abs(np64(out[m]) - want) <= 0.5 * F16_EPS * np.abs(want) * 1.02 + 2e-5).all()
    else:
        want = np.concatenate(y) + (np64(base[m]) if epilogue == 2 else 0.0)
        assert np.abs(np64(out[m]) - want).max() <= 2e-6 * np.sqrt(K) * (np.abs(want).max() + 1.0)


def test_gemm_tiled_from_fragment_order_copies_with_a_row_stride(ops):
    """Activation rows wider than K (a column slice of a larger buffer) and a K that ends inside a 32-wide stage."""
    M, K, N, pad = 1040, 168, 16640, 24
    buf = randn_f16((M, K + pad), 70)
    A = buf[:, :K]
    assert A.stride(0) == K + pad
    W = randn_bf16((N, K), 71, std=0.05)
    P = pack(ops, W)
    ref = torch.zeros((M, N), dtype=torch.float32, device=DEV)
    out = torch.full((M, N), float("nan"), dtype=torch.float32, device=DEV)
    ops.gemm(A, [W], ref, N, M=M, epilogue=0, kernel=2)
    ops.gemm_tiled_packed(A, [W], [P], out, N, M=M, epilogue=0)
    torch.cuda.synchronize()
    assert torch.equal(out.view(torch.int32), ref.view(torch.int32))
    want = np64(A[M - 1]) @ np64(W).T
    assert np.abs(np64(out[M - 1]) - want).max() <= 2e-6 * np.sqrt(K) * (np.abs(want).max() + 1.0)


@pytest.mark.parametrize("M,K,F,depth", [(4, 256, 688, 4), (128, 512, 1000, 2), (256, 256, 72, 4), (128, 4096, 1100, 4), (77, 1000, 200, 2),
                                          (200, 136, 96, 0)])
def test_gemm_packed_swiglu_on_k_halves_equals_the_row_major_kernel(ops, M, K, F, depth):
    """Same column sums in the same order (K halves of each 128-wide chunk, ascending chunks, half 0 + half 1): the kernel
    over fragment-order copies stores the bits the row-major kernel stores; one row also against the oracle."""
    step(f"swiglu halves M={M} K={K} F={F} depth={depth}")
    A = randn_f16((M, K), 80 + M)
    Wg, Wu = randn_bf16((F, K), 81, std=0.1), randn_bf16((F, K), 82, std=0.1)
    ref = torch.zeros((M, F), dtype=torch.float16, device=DEV)
    out = torch.full((M, F), -1.0, dtype=torch.float16, device=DEV)
    ops.gemm(A, [Wg, Wu], ref, F, epilogue=1, kernel=1)
    ops.gemm_packed_swiglu_halves(A, pack(ops, Wg), pack(ops, Wu), F, K, out, F, depth=depth)
    torch.cuda.synchronize()
    assert torch.equal(out.view(torch.int16), ref.view(torch.int16))
    m = M - 1
    g, u = np64(Wg) @ np64(A[m]), np64(Wu) @ np64(A[m])
    want = g / (1.0 + np.exp(-g)) * u
    assert (np.abs(np64(out[m]) - want) <= 0.5 * F16_EPS * np.abs(want) * 1.02 + 2e-5).all()


def f16_toward_zero(x32):
    """float32 -> float16, rounded toward zero (what the weight widening does; exact for normal halves)."""
    h = x32.astype(np.float16)
    over = np.abs(h.astype(np.float32)) > np.abs(x32)
    return np.where(over, np.nextafter(h, np.float16(0)), h)


@pytest.mark.parametrize("N,K", [(32, 16), (100, 72), (688, 256), (1000, 1000)])
def test_pack_weights_layout(ops, N, K):
    # index work: every element of the packed buffer is compared bit for bit with the stated layout
    W = randn_bf16((N, K), 70 + N, std=0.05)
    P = pack(ops, W)
    torch.cuda.synchronize()
    nbl, ks = -(-N // 32), -(-K // 16)
    got = P.cpu().numpy().view(np.uint16).reshape(nbl, ks, 64, 8)
    w32 = (W.cpu().view(torch.int16).numpy().astype(np.uint16).astype(np.uint32) << 16).view(np.float32)
    full = np.zeros((nbl * 32, ks * 16), np.float16)
    full[:N, :K] = f16_toward_zero(w32)
    lane = np.arange(64)
    rows = (np.arange(nbl)[:, None, None, None] * 32 + (lane & 31)[None, None, :, None])
    cols = (np.arange(ks)[None, :, None, None] * 16 + ((lane >> 5) * 8)[None, None, :, None] + np.arange(8)[None, None, None, :])
    ref = full[rows, cols].view(np.uint16)
    assert (got == ref).all()


PACKED_CASES = [
    # M, K, rows of up to three matrices, splits, blocks per wavefront, activation terms, rows per workgroup
    (1, 256, (256,), 1, 1, 1, 0), (4, 688, (256,), 2, 2, 1, 32), (4, 256, (256, 256, 256), 1, 1, 2, 64),
    (33, 688, (1000, 72), 3, 2, 1, 32), (128, 4096, (512, 128, 128), 4, 1, 2, 128), (200, 1024, (688,), 2, 2, 2, 64),
    (256, 512, (300,), 1, 1, 1, 32), (64, 264, (1024,), 1, 2, 1, 0), (128, 2048, (2048,), 16, 1, 1, 64), (77, 72, (40,), 1, 0, 1, 0),
    (130, 520, (1100, 200), 2, 1, 2, 32), (100, 1000, (2000,), 3, 2, 1, 64),
]


@pytest.mark.parametrize("M,K,rows,splits,nb,terms,rpw", PACKED_CASES)
def test_gemm_packed_f32(ops, M, K, rows, splits, nb, terms, rpw):
    step(f"gemm_packed M={M} K={K} rows={rows} splits={splits} nb={nb} terms={terms} rows_per_wg={rpw}")
    A = randn_f16((M, K), 20 + M)
    A_lo = randn_f16((M, K), 21 + M) * 2.0 ** -11 if terms == 2 else None
    Ws = [randn_bf16((r, K), 30 + i + r, std=0.05) for i, r in enumerate(rows)]
    Ps = [pack(ops, w) for w in Ws]
    N = sum(rows)
    out = torch.full((splits, M, N), float("nan"), dtype=torch.float32, device=DEV)
    ops.gemm_packed(A, Ps, rows, K, out, N, A_lo=A_lo, split_stride=M * N, splits=splits, epilogue=0, nb=nb, rows_per_wg=rpw,
                    depth=(0, 2, 4)[(M + K) % 3])
    torch.cuda.synchronize()
    got = np64(out).sum(0)
    a = np64(A) + (np64(A_lo) if terms == 2 else 0.0)
    ref = np.concatenate([orc.linear(bits(w), a) for w in Ws], axis=1)
    tol = 2e-6 * np.sqrt(K) * (np.abs(ref).max() + 1.0)
    assert np.isfinite(got).all()
    assert np.abs(got - ref).max() <= tol, (np.abs(got - ref).max(), tol)


@pytest.mark.parametrize("M,K,V,two", [(4, 256, 1000, False), (128, 512, 32000, False), (200, 256, 1024, True), (5, 136, 128256, False),
                                       (130, 264, 3000, True)])
def test_lm_head_with_fused_greedy_choice(ops, M, K, V, two):
    """The LM-head projection whose epilogue starts the greedy choice: logits as the plain packed projection gives them (the
    oracle's within fp32 accumulation), tokens exactly the lowest argmax of those logits -- with ties planted across
    different 128-column passes, a NaN row (-1), a vocabulary that ends inside a pass -- and the same tokens when the
    logits are not stored at all."""
    step(f"lm head + greedy choice M={M} K={K} V={V} two-term={two}")
    A = randn_f16((M, K), 70)
    A_lo = (randn_f16((M, K), 71) * 2.0 ** -11).to(torch.float16) if two else None
    W = randn_bf16((V, K), 72, std=0.05)
    a = np64(A) + (np64(A_lo) if two else 0.0)
    ref = orc.linear(bits(W), a)
    # ties at the top: the weight row of a row's best column copied to a column 130 (or more) below or above it
    planted = {}
    for m in range(0, min(M, 4)):
        c = int(np.argmax(ref[m]))
        c2 = c - 130 - m if c - 130 - m >= 0 else c + 130 + m
        W[c2] = W[c]
        planted[m] = min(c, c2)
    ref = orc.linear(bits(W), a)
    if M > 4:
        A[4] = float("nan")
    P = pack(ops, W)
    logits = torch.zeros((M, V), dtype=torch.float32, device=DEV)
    nxt = torch.full((M,), -7, dtype=torch.int32, device=DEV)
    nxt2 = torch.full((M,), -7, dtype=torch.int32, device=DEV)
    ops.lm_head_argmax(A, P, V, K, nxt, logits=logits, A_lo=A_lo)
    ops.lm_head_argmax(A, P, V, K, nxt2, logits=None, A_lo=A_lo)
    torch.cuda.synchronize()
    got, tok = np64(logits), nxt.cpu().numpy()
    rows = [m for m in range(M) if m != 4]
    tol = 2e-6 * np.sqrt(K) * (np.abs(ref[rows]).max() + 1.0)
    assert np.abs(got[rows] - ref[rows]).max() <= tol
    for m in range(M):
        assert tok[m] == orc.argmax(got[m]), m                     # index work is exact (-1 for the NaN row)
    if M > 4:
        assert tok[4] == -1 and np.isnan(got[4]).all()
    for m, c in planted.items():
        if m != 4:
            assert tok[m] == c and got[m, c] == got[m].max() and (got[m] == got[m].max()).sum() >= 2, m
    assert np.array_equal(nxt2.cpu().numpy(), tok)
    assert rows and ops.lm_head_argmax_ws_floats(M, V) == 2 * M * ((V + 127) // 128)


@pytest.mark.parametrize("M,nb,rpw", [(4, 1, 0), (128, 2, 64), (200, 1, 32)])
def test_gemm_packed_row_stride_and_accumulate(ops, M, nb, rpw):
    K, N, T = 256, 264, 3
    buf = randn_f16((M * T, K), 40)
    A = buf[T - 1::T]
    W = randn_bf16((N, K), 41, std=0.05)
    out = randn_f32((M, N), 42)
    base = np64(out)
    ops.gemm_packed(A, [pack(ops, W)], (N,), K, out, N, M=M, lda=T * K, epilogue=2, nb=nb, rows_per_wg=rpw, depth=4)
    torch.cuda.synchronize()
    ref = base + orc.linear(bits(W), np64(A))
    assert np.abs(np64(out) - ref).max() <= 1e-4


@pytest.mark.parametrize("M,K,F,rpw", [(4, 256, 688, 0), (128, 512, 1000, 32), (256, 256, 72, 64), (130, 1000, 4128, 128)])
def test_gemm_packed_swiglu(ops, M, K, F, rpw):
    step(f"packed swiglu M={M} K={K} F={F} rows_per_wg={rpw}")
    A = randn_f16((M, K), 50)
    Wg, Wu = randn_bf16((F, K), 51, std=0.1), randn_bf16((F, K), 52, std=0.1)
    out = torch.zeros((M, F), dtype=torch.float16, device=DEV)
    ops.gemm_packed(A, [pack(ops, Wg), pack(ops, Wu)], (F, F), K, out, F, epilogue=1, rows_per_wg=rpw, depth=(4, 2)[M % 2])
    torch.cuda.synchronize()
    g, u = orc.linear(bits(Wg), np64(A)), orc.linear(bits(Wu), np64(A))
    ref = g / (1.0 + np.exp(-g)) * u
    err = np.abs(np64(out) - ref)
    assert (err <= 0.5 * F16_EPS * np.abs(ref) * 1.02 + 2e-5).all(), err.max()


@pytest.mark.parametrize("style", [0, 1])
@pytest.mark.parametrize("hd,Hq,Hkv", [(64, 4, 4), (128, 8, 2)])
def test_rope_append(ops, style, hd, Hq, Hkv):
    S, nseq, nsplit = 40, 3, 2
    tab = torch.empty((S, hd // 2, 2), dtype=torch.float32, device=DEV)
    ops.build_rope_table(tab, S, hd, 10000.0)
    ld = (Hq + 2 * Hkv) * hd
    for (T, b0, pos0, nb) in [(7, 1, 0, 2), (1, 0, 23, 3)]:     # a prefill-like and a decode-like call
        M = nb * T
        qkv = randn_f32((nsplit, M, ld), 60 + T)
        kc = torch.zeros((nseq, Hkv, S, hd), dtype=torch.float16, device=DEV)
        vc = torch.zeros_like(kc)
        qf = torch.empty((M, Hq * hd), dtype=torch.float32, device=DEV)
        qb = torch.empty((M, Hq * hd), dtype=torch.float16, device=DEV)
        d_pos = torch.tensor([pos0], dtype=torch.int32, device=DEV)
        ops.rope_append(qkv, nsplit, M * ld, M, T, b0, d_pos, tab, style, Hq, Hkv, hd, S, qf, qb, kc, vc)
        torch.cuda.synchronize()
        tot = np64(qkv).sum(0)
        kcn, vcn = np64(kc), np64(vc)
        seen = np.zeros((nseq, S), bool)
        for m in range(M):
            b, pos = b0 + m // T, pos0 + m % T
            seen[b, pos] = True
            q = orc.rope(tot[m, : Hq * hd].reshape(Hq, hd), pos, 10000.0, style)
            k = orc.rope(tot[m, Hq * hd: (Hq + Hkv) * hd].reshape(Hkv, hd), pos, 10000.0, style)
            v = tot[m, (Hq + Hkv) * hd:].reshape(Hkv, hd)
            assert np.abs(np64(qf[m]).reshape(Hq, hd) - q).max() <= 2e-6 * (1 + np.abs(q).max())
            assert (np.abs(np64(qb[m]).reshape(Hq, hd) - q) <= 0.5 * F16_EPS * np.abs(q) * 1.01 + 1e-6).all()
            assert (np.abs(kcn[b, :, pos] - k) <= 0.5 * F16_EPS * np.abs(k) * 1.01 + 1e-6).all()
            assert (np.abs(vcn[b, :, pos] - v) <= 0.5 * F16_EPS * np.abs(v) * 1.01 + 1e-6).all()
        untouched = ~seen[:, None, :, None]                              # nothing else was touched
        assert (np.where(untouched, kcn, 0) == 0).all() and (np.where(untouched, vcn, 0) == 0).all()


@pytest.mark.parametrize("hd,Hq,Hkv", [(128, 8, 8), (128, 8, 2), (128, 16, 1), (64, 4, 4), (64, 6, 2), (128, 8, 1)])
@pytest.mark.parametrize("length,nsplit", [(0, 1), (5, 1), (130, 1), (130, 3), (1000, 8), (2, 4)])
def test_decode_attention(ops, hd, Hq, Hkv, length, nsplit):
    step(f"decode attention hd={hd} Hq={Hq} Hkv={Hkv} len={length} nsplit={nsplit}")
    B, S = 3, 1024
    q = randn_f32((B, Hq * hd), 70, std=1.5)
    kc = randn_f16((B, Hkv, S, hd), 71)
    vc = randn_f16((B, Hkv, S, hd), 72)
    # rows past the visible range must never be used: poison them
    kc[:, :, length + 1:] = float("nan")
    vc[:, :, length + 1:] = float("nan")
    d_len = torch.tensor([length], dtype=torch.int32, device=DEV)
    out = torch.zeros((B, Hq * hd), dtype=torch.float16, device=DEV)
    ws = torch.empty(max(ops.decode_attention_ws_floats(B, Hq, hd, nsplit), 1), dtype=torch.float32, device=DEV)
    ops.decode_attention(q, kc, vc, d_len, out, ws, B, Hq, Hkv, hd, S, nsplit)
    torch.cuda.synchronize()
    qn, kn, vn, on = np64(q).reshape(B, Hq, hd), np64(kc), np64(vc), np64(out).reshape(B, Hq, hd)
    g = Hq // Hkv
    for b in range(B):
        for u in range(Hq):
            ref = orc.attend(qn[b, u], kn[b, u // g, : length + 1], vn[b, u // g, : length + 1])
            err = np.abs(on[b, u] - ref)
            assert (err <= 0.5 * F16_EPS * np.abs(ref) * 1.02 + 2e-5).all(), (b, u, err.max())


@pytest.mark.parametrize("style", [0, 1])
@pytest.mark.parametrize("hd,Hq,Hkv", [(128, 8, 8), (128, 8, 2), (128, 16, 2), (64, 4, 4), (64, 6, 2), (128, 8, 1)])
@pytest.mark.parametrize("length,nsplit", [(0, 1), (5, 1), (130, 3), (1000, 8), (2, 4)])
def test_decode_attention_fused_with_rope_and_append(ops, style, hd, Hq, Hkv, length, nsplit):
    """One kernel = rotary embedding of the new q/k, append of the new k/v row, attention over positions 0 .. length."""
    step(f"fused decode attention style={style} hd={hd} Hq={Hq} Hkv={Hkv} len={length} nsplit={nsplit}")
    B, S, nq = 3, 1024, 2
    ld = (Hq + 2 * Hkv) * hd
    tab = torch.empty((S, hd // 2, 2), dtype=torch.float32, device=DEV)
    ops.build_rope_table(tab, S, hd, 10000.0)
    qkv = randn_f32((nq, B, ld), 73, std=0.8)
    kc = randn_f16((B, Hkv, S, hd), 71)
    vc = randn_f16((B, Hkv, S, hd), 72)
    kc[:, :, length:] = float("nan")     # the row of the new position is NOT in the cache yet; later rows are never used
    vc[:, :, length:] = float("nan")
    k_before, v_before = kc.clone(), vc.clone()
    d_len = torch.tensor([length], dtype=torch.int32, device=DEV)
    out = torch.zeros((B, Hq * hd), dtype=torch.float16, device=DEV)
    ws = torch.empty(max(ops.decode_attention_ws_floats(B, Hq, hd, nsplit), 1), dtype=torch.float32, device=DEV)
    ops.decode_attention_fused(qkv, nq, B * ld, tab, style, kc, vc, d_len, out, ws, B, Hq, Hkv, hd, S, nsplit)
    torch.cuda.synchronize()
    tot = np64(qkv).sum(0)
    kn, vn, on = np64(kc), np64(vc), np64(out).reshape(B, Hq, hd)
    g = Hq // Hkv
    for b in range(B):
        q = orc.rope(tot[b, : Hq * hd].reshape(Hq, hd), length, 10000.0, style)
        k = orc.rope(tot[b, Hq * hd: (Hq + Hkv) * hd].reshape(Hkv, hd), length, 10000.0, style)
        v = tot[b, (Hq + Hkv) * hd:].reshape(Hkv, hd)
        # the appended rows: the rotated k and the plain v, rounded once to f16
        assert (np.abs(kn[b, :, length] - k) <= 0.5 * F16_EPS * np.abs(k) * 1.01 + 1e-6).all()
        assert (np.abs(vn[b, :, length] - v) <= 0.5 * F16_EPS * np.abs(v) * 1.01 + 1e-6).all()
        for u in range(Hq):
            # attention over the cache as it now stands (the stored, rounded new row included)
            ref = orc.attend(q[u], kn[b, u // g, : length + 1], vn[b, u // g, : length + 1])
            err = np.abs(on[b, u] - ref)
            assert (err <= 0.5 * F16_EPS * np.abs(ref) * 1.02 + 3e-5).all(), (b, u, err.max())
    # nothing but the new row changed (bit patterns: NaN payloads included)
    kb, ka = k_before.cpu().view(torch.int16).numpy().copy(), kc.cpu().view(torch.int16).numpy().copy()
    vb, va = v_before.cpu().view(torch.int16).numpy().copy(), vc.cpu().view(torch.int16).numpy().copy()
    ka[:, :, length] = kb[:, :, length]
    va[:, :, length] = vb[:, :, length]
    assert (ka == kb).all() and (va == vb).all()


@pytest.mark.parametrize("hd,Hq,Hkv", [(128, 4, 4), (128, 8, 2), (64, 4, 1)])
@pytest.mark.parametrize("T", [1, 16, 100, 300])
def test_prefill_attention(ops, hd, Hq, Hkv, T):
    step(f"prefill attention hd={hd} Hq={Hq} Hkv={Hkv} T={T}")
    nb, b0, S, nseq = 2, 1, 320, 3
    q = randn_f16((nb * T, Hq * hd), 80, std=1.5)
    kc = randn_f16((nseq, Hkv, S, hd), 81)
    vc = randn_f16((nseq, Hkv, S, hd), 82)
    kc[:, :, T:] = float("nan")
    vc[:, :, T:] = float("nan")
    out = torch.zeros((nb * T, Hq * hd), dtype=torch.float16, device=DEV)
    ops.prefill_attention(q, kc, vc, out, nb, b0, T, Hq, Hkv, hd, S)
    torch.cuda.synchronize()
    qn, kn, vn = np64(q).reshape(nb, T, Hq, hd), np64(kc), np64(vc)
    on = np64(out).reshape(nb, T, Hq, hd)
    g = Hq // Hkv
    worst = 0.0
    for b in range(nb):
        for u in range(Hq):
            for i in sorted(set(min(i, T - 1) for i in [0, 1, T // 2, T - 1] + list(range(0, T, 7)))):
                ref = orc.attend(qn[b, i, u], kn[b0 + b, u // g, : i + 1], vn[b0 + b, u // g, : i + 1])
                err = np.abs(on[b, i, u] - ref)
                worst = max(worst, err.max())
                # probabilities are rounded to f16 (2^-11 relative each) before the second product
                bound = 0.5 * F16_EPS * np.abs(ref) * 1.02 + 2.0 ** -11 * np.abs(vn[b0 + b, u // g, : i + 1]).max() + 2e-5
                assert (err <= bound).all(), (b, u, i, err.max())
    step(f"  worst abs error {worst:.2e}")


@pytest.mark.parametrize("V", [1024, 32000, 128256])
def test_argmax(ops, V):
    B = 6
    lg = randn_f32((B, V), 90)
    lg[1, 17] = 50.0
    lg[1, 4000 % V] = 50.0                     # tie: lowest index wins
    lg[2, :] = -3.0                            # all equal
    lg[3, V - 1] = 99.0
    lg[4, 5] = float("nan")
    lg[5, :] = -torch.abs(lg[5, :]) - 1.0      # all negative
    nxt = torch.full((B,), -7, dtype=torch.int32, device=DEV)
    ops.argmax(lg, nxt)
    torch.cuda.synchronize()
    ln = np64(lg)
    for b in range(B):
        assert int(nxt[b]) == orc.argmax(ln[b]), b
    assert int(nxt[1]) == min(17, 4000 % V) and int(nxt[2]) == 0 and int(nxt[3]) == V - 1 and int(nxt[4]) == -1


@pytest.mark.parametrize("M,V,T,m_first", [(7, 97, 4, 0), (64, 1000, 16, 32), (33, 32000, 11, 22), (5, 128256, 5, 0)])
def test_logprob_gather(ops, M, V, T, m_first):
    """out[g] = log softmax(row)[next token]; rows that end a sequence get 0."""
    step(f"logprob gather M={M} V={V} T={T} m_first={m_first}")
    logits = randn_f32((M, V), 90 + M, std=2.5)
    total = m_first + M + 1
    g = torch.Generator(device="cpu").manual_seed(91)
    tokens = torch.randint(0, V, (total,), generator=g, dtype=torch.int32).to(DEV)
    out = torch.full((total,), float("nan"), dtype=torch.float32, device=DEV)
    ops.logprob_gather(logits, tokens, T, m_first, out)
    torch.cuda.synchronize()
    ln, tn, on = np64(logits), tokens.cpu().numpy(), np64(out)
    assert np.isnan(on[:m_first]).all() and np.isnan(on[m_first + M:]).all()       # rows outside the block are untouched
    for r in range(M):
        gidx = m_first + r
        if gidx % T == T - 1:
            assert on[gidx] == 0.0
        else:
            ref = orc.token_logprob(ln[r], int(tn[gidx + 1]))
            # fp32 exp/log and a 512-way merge of (max, sum) pairs: a few ulp of the log-sum (|lse| <= ~20)
            assert abs(on[gidx] - ref) <= 2e-5 * (1.0 + abs(ref)), (r, on[gidx], ref)


def test_empty_inputs_enqueue_nothing(ops):
    """M = 0 / B = 0: every entry point returns success and leaves its outputs alone.  (Called through the C ABI directly:
    an empty torch tensor has a NULL pointer, which the entry points reject.)"""
    from paper_2406_14088_amd.binding import lib
    L = lib()
    d, V = 64, 97
    sentinel = lambda *shape, dtype=torch.float32: torch.full(shape, 7.0, dtype=dtype, device=DEV)
    emb, gain, W = randn_bf16((V, d), 1), randn_bf16((d,), 2), randn_bf16((96, d), 3)
    x, h, out, lg = sentinel(2, d), sentinel(2, d, dtype=torch.float16), sentinel(2, 96), sentinel(2, V)
    A = randn_f16((2, d), 4)
    toks = torch.zeros((2,), dtype=torch.int32, device=DEV)
    nxt = torch.full((2,), 5, dtype=torch.int32, device=DEV)
    kc = torch.zeros((1, 1, 8, 64), dtype=torch.float16, device=DEV)
    P = torch.zeros(ops.packed_weight_bytes(96, d) // 2, dtype=torch.int16, device=DEV)
    ops.pack_weights(W, P)
    p = lambda t: t.data_ptr()
    rcs = [
        L.rl_op_embed(p(toks), p(emb), p(x), 0, d, V, None),
        L.rl_op_add_rmsnorm(p(x), None, 0, 0, p(gain), 1e-5, p(h), None, 0, d, None),
        L.rl_op_gemm(p(A), None, d, p(W), None, None, 96, 0, 0, 0, d, p(out), 96, 0, 1, 0, 1, None, None),
        L.rl_op_gemm(p(A), None, d, p(W), None, None, 96, 0, 0, 0, d, p(out), 96, 0, 1, 0, 2, None, None),
        L.rl_op_gemm_packed(p(A), None, d, p(P), None, None, 96, 0, 0, 0, d, p(out), 96, 0, 1, 0, 0, 0, 0, None, None),
        L.rl_op_argmax(p(lg), 0, V, p(nxt), None),
        L.rl_op_decode_attention(p(x), p(kc), p(kc), p(toks), 0, p(h), None, 0, 1, 1, 64, 8, 1, None, None, None, None, None),
        L.rl_op_prefill_attention(p(h), p(kc), p(kc), p(h), 0, 0, 1, 1, 1, 64, 8, None, None, None, None, None),
        L.rl_op_logprob_gather(p(lg), V, 0, V, p(toks), 4, 0, p(x), None),
    ]
    torch.cuda.synchronize()
    assert rcs == [0] * len(rcs), rcs
    assert (x == 7).all() and (h == 7).all() and (out == 7).all() and (nxt == 5).all() and (lg == 7).all()


def cdf_interval(x64, temperature):
    z = (x64 - x64.max()) / temperature
    e = np.exp(z)
    c = np.cumsum(e) / e.sum()
    return np.concatenate([[0.0], c])


@pytest.mark.parametrize("B,V,temperature", [(5, 97, 1.0), (16, 1000, 0.7), (8, 32000, 1.0), (3, 128256, 1.3), (4, 1500, 0.05)])
def test_sampling_kernel(ops, B, V, temperature):
    """Index decided by floating point: the returned token must be a valid inversion of the row's own cumulative softmax
    (the draw lies in the token's probability interval up to fp32 summation error), and equal to the oracle's token whenever
    the draw is not within that error of an interval end."""
    step(f"sample B={B} V={V} T={temperature}")
    logits = randn_f32((B, V), 95 + B, std=2.0)
    g = torch.Generator(device="cpu").manual_seed(96)
    rounds, delta, exact, total = (6 if V <= 2000 else 2), 3e-5, 0, 0
    for r in range(rounds):
        u = torch.rand((B,), generator=g, dtype=torch.float32)
        if r == 0:
            u[0] = 0.0
        if r == 1:
            u[0] = float(np.nextafter(np.float32(1.0), np.float32(0.0)))
        nxt = torch.full((B,), -7, dtype=torch.int32, device=DEV)
        ops.sample(logits, temperature, u.to(DEV), nxt)
        torch.cuda.synchronize()
        got = nxt.cpu().numpy()
        for b in range(B):
            x = np64(logits[b])
            c = cdf_interval(x, temperature)
            ub, v = float(u[b]), int(got[b])
            assert 0 <= v < V
            assert c[v] - delta <= ub <= c[v + 1] + delta, (b, v, ub, c[v], c[v + 1])
            want = orc.sample(x, temperature, ub)
            total += 1
            if min(abs(ub - c[want]), abs(ub - c[want + 1])) > delta:
                assert v == want
                exact += 1
    if V <= 2000:       # with a large vocabulary most probability intervals are no wider than the summation error
        assert exact >= 0.9 * total
    # determinism, and NaN rows
    a = torch.empty((B,), dtype=torch.int32, device=DEV)
    b2 = torch.empty((B,), dtype=torch.int32, device=DEV)
    ud = torch.full((B,), 0.3712, dtype=torch.float32, device=DEV)
    ops.sample(logits, temperature, ud, a)
    ops.sample(logits, temperature, ud, b2)
    bad = logits.clone()
    bad[1, V // 2] = float("nan")
    c2 = torch.empty((B,), dtype=torch.int32, device=DEV)
    ops.sample(bad, temperature, ud, c2)
    torch.cuda.synchronize()
    assert torch.equal(a, b2) and int(c2[1]) == -1 and torch.equal(c2[2:], a[2:]) and int(c2[0]) == int(a[0])


@pytest.mark.parametrize("hd,Hq,Hkv,nsplit", [(128, 4, 4, 1), (128, 8, 2, 3), (64, 4, 2, 1)])
def test_per_sequence_lengths_in_rope_append_and_attention(ops, hd, Hq, Hkv, nsplit):
    """Ragged batches: every sequence appends and attends at its own length (pos_stride / len_stride = 1)."""
    B, S, style = 4, 256, 1
    lens = [0, 7, 130, 255]
    ld = (Hq + 2 * Hkv) * hd
    tab = torch.empty((S, hd // 2, 2), dtype=torch.float32, device=DEV)
    ops.build_rope_table(tab, S, hd, 10000.0)
    qkv = randn_f32((1, B, ld), 97, std=0.8)
    kc, vc = randn_f16((B, Hkv, S, hd), 98), randn_f16((B, Hkv, S, hd), 99)
    for b, n in enumerate(lens):                      # nothing at or beyond a sequence's own length may be used
        kc[b, :, n:] = float("nan")
        vc[b, :, n:] = float("nan")
    d_len = torch.tensor(lens, dtype=torch.int32, device=DEV)
    qf = torch.empty((B, Hq * hd), dtype=torch.float32, device=DEV)
    ops.rope_append(qkv, 1, B * ld, B, 1, 0, d_len, tab, style, Hq, Hkv, hd, S, qf, None, kc, vc, pos_stride=1)
    out = torch.zeros((B, Hq * hd), dtype=torch.float16, device=DEV)
    ws = torch.empty(max(ops.decode_attention_ws_floats(B, Hq, hd, nsplit), 1), dtype=torch.float32, device=DEV)
    ops.decode_attention(qf, kc, vc, d_len, out, ws, B, Hq, Hkv, hd, S, nsplit, len_stride=1)
    torch.cuda.synchronize()
    tot, kn, vn, on = np64(qkv)[0], np64(kc), np64(vc), np64(out).reshape(B, Hq, hd)
    g = Hq // Hkv
    for b, n in enumerate(lens):
        q = orc.rope(tot[b, : Hq * hd].reshape(Hq, hd), n, 10000.0, style)
        k = orc.rope(tot[b, Hq * hd: (Hq + Hkv) * hd].reshape(Hkv, hd), n, 10000.0, style)
        assert (np.abs(kn[b, :, n] - k) <= 0.5 * F16_EPS * np.abs(k) * 1.01 + 1e-6).all()
        assert np.isnan(kn[b, :, n + 1:]).all()                       # rows past the new one stay untouched
        for u in range(Hq):
            ref = orc.attend(q[u], kn[b, u // g, : n + 1], vn[b, u // g, : n + 1])
            assert (np.abs(on[b, u] - ref) <= 0.5 * F16_EPS * np.abs(ref) * 1.02 + 3e-5).all(), (b, u)


@pytest.mark.parametrize("hd,Hq,Hkv,nsplit,page", [(128, 4, 4, 1, 16), (128, 8, 2, 3, 64), (64, 4, 2, 2, 32), (128, 16, 2, 1, 128)])
def test_paged_decode_attention_equals_contiguous(ops, hd, Hq, Hkv, nsplit, page):
    """A paged cache is a layout, not another computation: the same rows reached through shuffled page lists give
    the same output bit for bit (and, by the contiguous kernel's own test, the oracle's attention)."""
    B, S = 5, 320
    lens = [0, 15, 16, 200, 319]                      # positions of the newest row: page borders, one row, the whole cache
    kc, vc = randn_f16((B, Hkv, S, hd), 201), randn_f16((B, Hkv, S, hd), 202)
    q = randn_f32((B, Hq * hd), 203, std=0.7)
    d_len = torch.tensor(lens, dtype=torch.int32, device=DEV)
    pps = (S + page - 1) // page
    n_pages = B * pps + 3
    rng = np.random.default_rng(204)
    perm = rng.permutation(n_pages)[: B * pps].reshape(B, pps)
    k_pool = torch.full((n_pages, Hkv, page, hd), float("nan"), dtype=torch.float16, device=DEV)
    v_pool = torch.full((n_pages, Hkv, page, hd), float("nan"), dtype=torch.float16, device=DEV)
    for b in range(B):
        for i in range(pps):
            lo, hi = i * page, min((i + 1) * page, S)
            if lo > lens[b]:
                continue                              # pages a sequence has not reached stay NaN: they must not be read
            k_pool[perm[b, i], :, : hi - lo] = kc[b, :, lo:hi]
            v_pool[perm[b, i], :, : hi - lo] = vc[b, :, lo:hi]
    for b, n in enumerate(lens):                      # and inside the last page nothing beyond the newest row
        i, r = n // page, n % page
        k_pool[perm[b, i], :, r + 1:] = float("nan")
        v_pool[perm[b, i], :, r + 1:] = float("nan")
    table = torch.tensor(perm, dtype=torch.int32, device=DEV)
    ws = torch.empty(max(ops.decode_attention_ws_floats(B, Hq, hd, nsplit), 1), dtype=torch.float32, device=DEV)
    ref = torch.zeros((B, Hq * hd), dtype=torch.float16, device=DEV)
    ops.decode_attention(q, kc, vc, d_len, ref, ws, B, Hq, Hkv, hd, S, nsplit, len_stride=1)
    got = torch.zeros((B, Hq * hd), dtype=torch.float16, device=DEV)
    ops.decode_attention_paged(q, k_pool, v_pool, table, page, d_len, got, ws, B, Hq, Hkv, hd, S, nsplit, len_stride=1)
    torch.cuda.synchronize()
    assert not torch.isnan(got).any()
    assert torch.equal(got.view(torch.int16), ref.view(torch.int16))
    # one sequence against the oracle directly
    b, g = 3, Hq // Hkv
    kn, vn, on = np64(kc), np64(vc), np64(got).reshape(B, Hq, hd)
    for u in range(Hq):
        want = orc.attend(np64(q).reshape(B, Hq, hd)[b, u], kn[b, u // g, : lens[b] + 1], vn[b, u // g, : lens[b] + 1])
        assert (np.abs(on[b, u] - want) <= 0.5 * F16_EPS * np.abs(want) * 1.02 + 3e-5).all()


@pytest.mark.parametrize("hd,Hq,Hkv,nsplit,page", [(128, 4, 4, 1, 16), (128, 8, 2, 3, 64), (64, 4, 2, 2, 32), (128, 16, 2, 1, 128),
                                                   (128, 32, 4, 2, 16)])
def test_paged_decode_attention_over_block_scaled_rows(ops, hd, Hq, Hkv, nsplit, page):
    """Block-scaled rows (int16 elements, one fp32 scale per row) through shuffled page lists: bit-equal to the contiguous
    cache for the vector kernel and for the matrix-core kernel of grouped-query shapes, and the oracle's attention."""
    B, S = 5, 320
    lens = [0, 15, 16, 200, 319]
    kc, ks, kn = _random_block_scaled((B, Hkv, S, hd), 211)
    vc, vs, vn = _random_block_scaled((B, Hkv, S, hd), 212)
    q = randn_f32((B, Hq * hd), 213, std=0.7)
    d_len = torch.tensor(lens, dtype=torch.int32, device=DEV)
    pps = (S + page - 1) // page
    n_pages = B * pps + 3
    perm = np.random.default_rng(214).permutation(n_pages)[: B * pps].reshape(B, pps)
    # rows a sequence has not reached hold the largest elements and NaN scales: they must not reach the result
    k_pool = torch.full((n_pages, Hkv, page, hd), 32767, dtype=torch.int16, device=DEV)
    v_pool = torch.full((n_pages, Hkv, page, hd), 32767, dtype=torch.int16, device=DEV)
    ks_pool = torch.full((n_pages, Hkv, page), float("nan"), dtype=torch.float32, device=DEV)
    vs_pool = torch.full((n_pages, Hkv, page), float("nan"), dtype=torch.float32, device=DEV)
    for b in range(B):
        for i in range(pps):
            lo, hi = i * page, min((i + 1) * page, S)
            n = min(hi, lens[b] + 1) - lo
            if n <= 0:
                continue
            k_pool[perm[b, i], :, :n] = kc[b, :, lo: lo + n]
            v_pool[perm[b, i], :, :n] = vc[b, :, lo: lo + n]
            ks_pool[perm[b, i], :, :n] = ks[b, :, lo: lo + n]
            vs_pool[perm[b, i], :, :n] = vs[b, :, lo: lo + n]
    table = torch.tensor(perm, dtype=torch.int32, device=DEV)
    ws = torch.empty(max(ops.decode_attention_ws_floats(B, Hq, hd, nsplit), 1), dtype=torch.float32, device=DEV)
    ref = torch.zeros((B, Hq * hd), dtype=torch.float16, device=DEV)
    ops.decode_attention(q, kc, vc, d_len, ref, ws, B, Hq, Hkv, hd, S, nsplit, len_stride=1, kscale=ks, vscale=vs)
    got = torch.zeros((B, Hq * hd), dtype=torch.float16, device=DEV)
    ops.decode_attention_paged(q, k_pool, v_pool, table, page, d_len, got, ws, B, Hq, Hkv, hd, S, nsplit, len_stride=1,
                               kscale=ks_pool, vscale=vs_pool)
    torch.cuda.synchronize()
    assert not torch.isnan(got).any() and not torch.isnan(ref).any()
    assert torch.equal(got.view(torch.int16), ref.view(torch.int16))
    g = Hq // Hkv
    on = np64(got).reshape(B, Hq, hd)
    for b in (1, 3):
        for u in range(Hq):
            want = orc.attend(np64(q).reshape(B, Hq, hd)[b, u], kn[b, u // g, : lens[b] + 1], vn[b, u // g, : lens[b] + 1])
            assert (np.abs(on[b, u] - want) <= 0.5 * F16_EPS * np.abs(want) * 1.02 + 3e-5).all()


def test_paged_decode_attention_rejects_bad_page_sizes(ops):
    t = torch.zeros((1, 64), dtype=torch.int32, device=DEV)
    x = torch.zeros((4096,), dtype=torch.float16, device=DEV)
    qf = torch.zeros((128,), dtype=torch.float32, device=DEV)
    from paper_2406_14088_amd import RlGenError
    for page in (0, 8, 24, 8192):
        with pytest.raises(RlGenError):
            ops.decode_attention_paged(qf, x, x, t, page, t, x, None, 1, 1, 1, 128, 16, 1)
    with pytest.raises(RlGenError):                   # the page lists must cover S positions
        ops.decode_attention_paged(qf, x, x, t, 16, t, x, None, 1, 1, 1, 128, 16 * 64 + 1, 1)


@pytest.mark.parametrize("Hq,Hkv,nsplit", [(8, 2, 1), (8, 1, 1), (16, 1, 2), (32, 4, 5)])
def test_grouped_query_decode_attention_tile_tails(ops, Hq, Hkv, nsplit):
    """The matrix-core kernel for grouped-query shapes works on tiles of 16 cache rows in a ring of LDS stages: every
    residue of the visible length modulo the tile, fewer tiles than stages, and splits that receive nothing."""
    hd, S = 128, 256
    lens = [0, 1, 14, 15, 16, 17, 30, 31, 32, 33, 46, 47, 48, 49, 63, 64, 65, 100, 127, 128, 129, 200, 254, 255]
    B = len(lens)
    q = randn_f32((B, Hq * hd), 301, std=1.2)
    kc, vc = randn_f16((B, Hkv, S, hd), 302), randn_f16((B, Hkv, S, hd), 303)
    for b, n in enumerate(lens):
        kc[b, :, n + 1:] = float("nan")
        vc[b, :, n + 1:] = float("nan")
    d_len = torch.tensor(lens, dtype=torch.int32, device=DEV)
    out = torch.zeros((B, Hq * hd), dtype=torch.float16, device=DEV)
    ws = torch.empty(max(ops.decode_attention_ws_floats(B, Hq, hd, nsplit), 1), dtype=torch.float32, device=DEV)
    ops.decode_attention(q, kc, vc, d_len, out, ws, B, Hq, Hkv, hd, S, nsplit, len_stride=1)
    torch.cuda.synchronize()
    qn, kn, vn, on = np64(q).reshape(B, Hq, hd), np64(kc), np64(vc), np64(out).reshape(B, Hq, hd)
    g = Hq // Hkv
    for b, n in enumerate(lens):
        for u in range(Hq):
            ref = orc.attend(qn[b, u], kn[b, u // g, : n + 1], vn[b, u // g, : n + 1])
            err = np.abs(on[b, u] - ref)
            assert (err <= 0.5 * F16_EPS * np.abs(ref) * 1.02 + 2e-5).all(), (b, n, u, err.max())


@pytest.mark.parametrize("Hq,Hkv,two_terms", [(8, 8, True), (16, 2, False), (9, 3, True)])
def test_qkv_projection_with_rotary_epilogue_equals_the_two_kernels(ops, Hq, Hkv, two_terms):
    """The prefill QKV projection that rotates and appends in its own epilogue stores, bit for bit, what the fp32
    projection followed by rope_append stores (the oracle parity of those two is established by their own tests)."""
    hd, K, T, nseq, b0, S = 128, 256, 40, 205, 3, 64        # 8200 rows: a ragged last tile, bands that wrap to the next sequence
    M = nseq * T
    n_all = (Hq + 2 * Hkv) * hd
    A = randn_f16(((2 if two_terms else 1) * M, K), 401)
    if two_terms:
        A[M:] *= 2.0 ** -11                                   # a second term of the size it has in the generator
    Wq, Wk, Wv = randn_bf16((Hq * hd, K), 402, 0.05), randn_bf16((Hkv * hd, K), 403, 0.05), randn_bf16((Hkv * hd, K), 404, 0.05)
    tab = torch.empty((S, hd // 2, 2), dtype=torch.float32, device=DEV)
    ops.build_rope_table(tab, S, hd, 10000.0)
    A_lo = A[M:] if two_terms else None
    # reference: fp32 projection, then rope_append
    part = torch.empty((M, n_all), dtype=torch.float32, device=DEV)
    ops.gemm(A[:M], [Wq, Wk, Wv], part, n_all, M=M, epilogue=0, kernel=2, A_lo=A_lo)
    zero = torch.zeros((1,), dtype=torch.int32, device=DEV)
    q_ref = torch.zeros((M, Hq * hd), dtype=torch.float16, device=DEV)
    kc_ref = torch.zeros((b0 + nseq, Hkv, S, hd), dtype=torch.float16, device=DEV)
    vc_ref = torch.zeros_like(kc_ref)
    ops.rope_append(part, 1, M * n_all, M, T, b0, zero, tab, 1, Hq, Hkv, hd, S, None, q_ref, kc_ref, vc_ref)
    q = torch.zeros_like(q_ref)
    kc, vc = torch.zeros_like(kc_ref), torch.zeros_like(vc_ref)
    ops.gemm_rope(A[:M], Wq, Wk, Wv, Hq, Hkv, hd, M, T, b0, tab, 1, S, q, kc, vc, A_lo=A_lo)
    torch.cuda.synchronize()
    assert q_ref.abs().max() > 0 and kc_ref.abs().max() > 0
    assert torch.equal(q.view(torch.int16), q_ref.view(torch.int16))
    assert torch.equal(kc.view(torch.int16), kc_ref.view(torch.int16))
    assert torch.equal(vc.view(torch.int16), vc_ref.view(torch.int16))
    # the same with both operands copied global -> LDS directly (fragment-order weight copies)
    q2, kc2, vc2 = torch.zeros_like(q_ref), torch.zeros_like(kc_ref), torch.zeros_like(vc_ref)
    ops.gemm_rope(A[:M], Wq, Wk, Wv, Hq, Hkv, hd, M, T, b0, tab, 1, S, q2, kc2, vc2, A_lo=A_lo, Ps=[pack(ops, W) for W in (Wq, Wk, Wv)])
    torch.cuda.synchronize()
    for got, want in ((q2, q_ref), (kc2, kc_ref), (vc2, vc_ref)):
        assert torch.equal(got.view(torch.int16), want.view(torch.int16))
    # one row against the oracle directly (sequence b0 + 7, position 11)
    m = 7 * T + 11
    x = np64(A[m]) + (np64(A[M + m]) if two_terms else 0.0)
    for name, W, H, got in (("q", Wq, Hq, np64(q[m]).reshape(Hq, hd)), ("k", Wk, Hkv, np64(kc[b0 + 7, :, 11])), ("v", Wv, Hkv, np64(vc[b0 + 7, :, 11]))):
        y = (np64(W) @ x).reshape(H, hd)
        want = y if name == "v" else orc.rope(y, 11, 10000.0, 1)
        assert (np.abs(got - want) <= 0.5 * F16_EPS * np.abs(want) * 1.05 + 2e-4).all(), name


def test_rotary_epilogue_is_refused_where_it_does_not_apply(ops):
    from paper_2406_14088_amd import RlGenError
    x = torch.zeros((4096, 256), dtype=torch.float16, device=DEV)
    w = torch.zeros((1024, 256), dtype=torch.bfloat16, device=DEV)
    t = torch.zeros((64, 64, 2), dtype=torch.float32, device=DEV)
    for hd, style, T, M in ((64, 1, 40, 4000), (128, 0, 40, 4000), (128, 1, 16, 4000), (128, 1, 40, 512)):
        with pytest.raises(RlGenError):
            ops.gemm_rope(x, w, w, w, 8, 8, hd, M, T, 0, t, style, 64, x, x, x)


@pytest.mark.parametrize("hd,Hq,Hkv,nsplit", [(128, 4, 4, 1), (128, 8, 1, 2), (64, 4, 2, 1)])
def test_decode_attention_skips_ended_sequences(ops, hd, Hq, Hkv, nsplit):
    """Sequences flagged as ended are not attended: their output rows keep what they held, the others are unaffected."""
    B, S, n = 6, 128, 70
    q = randn_f32((B, Hq * hd), 501)
    kc, vc = randn_f16((B, Hkv, S, hd), 502), randn_f16((B, Hkv, S, hd), 503)
    done = torch.tensor([0, 1, 0, 0, 1, 1], dtype=torch.int32, device=DEV)
    kc[done.bool()] = float("nan")                        # an ended sequence's cache must not be touched
    vc[done.bool()] = float("nan")
    d_len = torch.tensor([n], dtype=torch.int32, device=DEV)
    ws = torch.zeros(max(ops.decode_attention_ws_floats(B, Hq, hd, nsplit), 1), dtype=torch.float32, device=DEV)
    ref = torch.full((B, Hq * hd), 7.0, dtype=torch.float16, device=DEV)
    ops.decode_attention(q, kc, vc, d_len, ref, ws, B, Hq, Hkv, hd, S, nsplit)
    out = torch.full((B, Hq * hd), 7.0, dtype=torch.float16, device=DEV)
    ws.zero_()
    ops.decode_attention(q, kc, vc, d_len, out, ws, B, Hq, Hkv, hd, S, nsplit, d_done=done)
    torch.cuda.synchronize()
    live = ~done.bool()
    assert torch.equal(out[live].view(torch.int16), ref[live].view(torch.int16)) and not torch.isnan(out[live]).any()
    if nsplit == 1:
        assert (out[done.bool()] == 7.0).all()
    else:                                                 # the merge of the (untouched, zeroed) partials writes the row
        assert not torch.isinf(out[done.bool()]).any()


# ---------------------------------------------------------------------------------------------------------------------
# Block-scaled cache rows (int16 elements, one fp32 scale per row) and two-term half outputs
# ---------------------------------------------------------------------------------------------------------------------
def _random_block_scaled(shape, seed):
    """A cache area as the kernels store it: random int16 elements and positive fp32 row scales, plus the fp64 values
    q * scale they stand for (exactly representable, so both sides read identical numbers)."""
    g = torch.Generator(device="cpu").manual_seed(seed)
    qi = torch.randint(-32767, 32768, shape, generator=g, dtype=torch.int32).to(torch.int16)
    sc = (torch.rand(shape[:-1], generator=g) * 2.0 + 0.5) * (1.0 / 32767.0)
    vals = qi.to(torch.float64) * sc.to(torch.float32).to(torch.float64)[..., None]
    return qi.to(DEV), sc.to(torch.float32).to(DEV), vals.numpy()


@pytest.mark.parametrize("style", [0, 1])
@pytest.mark.parametrize("hd,Hq,Hkv", [(64, 4, 4), (128, 8, 2), (128, 3, 3)])
def test_rope_append_block_scaled_rows(ops, style, hd, Hq, Hkv):
    """The appended rows as int16 * scale: scale = max|x| / 32767 of the (position, kv head) row, elements within half a
    step of the oracle's rotated values; the largest element of a row is +-32767; nothing else is touched."""
    S, nseq, nsplit = 40, 3, 2
    tab = torch.empty((S, hd // 2, 2), dtype=torch.float32, device=DEV)
    ops.build_rope_table(tab, S, hd, 10000.0)
    ld = (Hq + 2 * Hkv) * hd
    for (T, b0, pos0, nb) in [(7, 1, 0, 2), (1, 0, 23, 3)]:
        M = nb * T
        qkv = randn_f32((nsplit, M, ld), 160 + T)
        qkv[:, 0, Hq * hd: Hq * hd + hd] = 0.0           # one all-zero K row: scale 0, elements 0
        kc = torch.zeros((nseq, Hkv, S, hd), dtype=torch.int16, device=DEV)
        vc = torch.zeros_like(kc)
        ks = torch.full((nseq, Hkv, S), -1.0, dtype=torch.float32, device=DEV)
        vs = torch.full((nseq, Hkv, S), -1.0, dtype=torch.float32, device=DEV)
        qf = torch.empty((M, Hq * hd), dtype=torch.float32, device=DEV)
        d_pos = torch.tensor([pos0], dtype=torch.int32, device=DEV)
        qh = torch.zeros((M, Hq * hd), dtype=torch.float16, device=DEV)
        ql = torch.zeros_like(qh)
        ops.rope_append(qkv, nsplit, M * ld, M, T, b0, d_pos, tab, style, Hq, Hkv, hd, S, qf, qh, kc, vc, kscale=ks, vscale=vs, q_f16_lo=ql)
        torch.cuda.synchronize()
        assert torch.equal(qh, qf.to(torch.float16)) and torch.equal(ql, (qf - qh.float()).to(torch.float16))
        tot = np64(qkv).sum(0)
        kq, vq, ksn, vsn = kc.cpu().numpy().astype(np.float64), vc.cpu().numpy().astype(np.float64), np64(ks), np64(vs)
        seen = np.zeros((nseq, S), bool)
        for m in range(M):
            b, pos = b0 + m // T, pos0 + m % T
            seen[b, pos] = True
            k = orc.rope(tot[m, Hq * hd: (Hq + Hkv) * hd].reshape(Hkv, hd), pos, 10000.0, style)
            v = tot[m, (Hq + Hkv) * hd:].reshape(Hkv, hd)
            for ref, qv, sc in ((k, kq[b, :, pos], ksn[b, :, pos]), (v, vq[b, :, pos], vsn[b, :, pos])):
                amax = np.abs(ref).max(-1)
                assert (np.abs(sc - amax / 32767.0) <= 3e-6 * amax / 32767.0 + 1e-30).all()
                assert (np.abs(qv * sc[:, None] - ref) <= 0.5 * sc[:, None] * 1.001 + 1e-6 * np.abs(ref)).all()
                assert ((np.abs(qv).max(-1) == 32767) | (amax == 0)).all()
        untouched = ~seen[:, None, :]
        assert (np.where(untouched[..., None], kq, 0) == 0).all() and (np.where(untouched[..., None], vq, 0) == 0).all()
        assert (np.where(untouched, ksn, -1.0) == -1.0).all() and (np.where(untouched, vsn, -1.0) == -1.0).all()


@pytest.mark.parametrize("hd,Hq,Hkv", [(128, 8, 8), (128, 8, 2), (128, 16, 2), (64, 4, 4), (64, 6, 2)])
@pytest.mark.parametrize("length,nsplit", [(0, 1), (5, 1), (130, 3), (1000, 8), (2, 4)])
def test_decode_attention_block_scaled_rows_and_two_term_output(ops, hd, Hq, Hkv, length, nsplit):
    """Decode attention over int16 * scale rows (every head grouping runs on the vector kernel then), with the second
    half term of the output: out alone is the oracle's value to half precision, out + out_lo to fp32 arithmetic."""
    B, S = 3, 1024
    q = randn_f32((B, Hq * hd), 170, std=1.5)
    kc, ks, kn = _random_block_scaled((B, Hkv, S, hd), 171)
    vc, vs, vn = _random_block_scaled((B, Hkv, S, hd), 172)
    ks[:, :, length + 1:] = float("nan")          # rows past the visible range must never be used
    vs[:, :, length + 1:] = float("nan")
    d_len = torch.tensor([length], dtype=torch.int32, device=DEV)
    out = torch.zeros((B, Hq * hd), dtype=torch.float16, device=DEV)
    out_lo = torch.zeros_like(out)
    ws = torch.empty(max(ops.decode_attention_ws_floats(B, Hq, hd, nsplit), 1), dtype=torch.float32, device=DEV)
    ops.decode_attention(q, kc, vc, d_len, out, ws, B, Hq, Hkv, hd, S, nsplit, kscale=ks, vscale=vs, out_lo=out_lo)
    torch.cuda.synchronize()
    qn, on, ln = np64(q).reshape(B, Hq, hd), np64(out).reshape(B, Hq, hd), np64(out_lo).reshape(B, Hq, hd)
    g = Hq // Hkv
    for b in range(B):
        for u in range(Hq):
            ref = orc.attend(qn[b, u], kn[b, u // g, : length + 1], vn[b, u // g, : length + 1])
            assert (np.abs(on[b, u] - ref) <= 0.5 * F16_EPS * np.abs(ref) * 1.02 + 2e-5).all(), (b, u)
            assert (np.abs(on[b, u] + ln[b, u] - ref) <= 2e-5 * (1 + np.abs(ref))).all(), (b, u, np.abs(on[b, u] + ln[b, u] - ref).max())


@pytest.mark.parametrize("kind", ["vector", "matrix", "block_scaled", "matrix_block_scaled"])
@pytest.mark.parametrize("length", [2047, 4095])
def test_decode_attention_at_long_context_lengths(ops, kind, length):
    """Cached lengths of the long-context workload (prompt 2048, generation to 4096 positions): the vector kernel (one query
    head per kv head, IEEE half rows), the matrix-core kernel (8 query heads per kv head) and both kernels over
    block-scaled rows, each split over the sequence as the generator splits it, against the oracle row by row."""
    hd, S = 128, 4096
    B, Hq, Hkv = (2, 16, 2) if kind.startswith("matrix") else (2, 4, 4)
    nsplit = 4
    step(f"decode attention, {kind} kernel, {length + 1} cached rows")
    q = randn_f32((B, Hq * hd), 180, std=1.5)
    if kind.endswith("block_scaled"):
        kc, ks, kn = _random_block_scaled((B, Hkv, S, hd), 181)
        vc, vs, vn = _random_block_scaled((B, Hkv, S, hd), 182)
    else:
        kc, vc, ks, vs = randn_f16((B, Hkv, S, hd), 181), randn_f16((B, Hkv, S, hd), 182), None, None
        kn, vn = np64(kc), np64(vc)
    d_len = torch.tensor([length], dtype=torch.int32, device=DEV)
    out = torch.zeros((B, Hq * hd), dtype=torch.float16, device=DEV)
    ws = torch.empty(max(ops.decode_attention_ws_floats(B, Hq, hd, nsplit), 1), dtype=torch.float32, device=DEV)
    ops.decode_attention(q, kc, vc, d_len, out, ws, B, Hq, Hkv, hd, S, nsplit, kscale=ks, vscale=vs)
    torch.cuda.synchronize()
    qn, on = np64(q).reshape(B, Hq, hd), np64(out).reshape(B, Hq, hd)
    g = Hq // Hkv
    for b in range(B):
        for u in range(Hq):
            ref = orc.attend(qn[b, u], kn[b, u // g, : length + 1], vn[b, u // g, : length + 1])
            assert (np.abs(on[b, u] - ref) <= 0.5 * F16_EPS * np.abs(ref) * 1.02 + 3e-5).all(), (b, u, np.abs(on[b, u] - ref).max())


@pytest.mark.parametrize("hd,Hq,Hkv", [(128, 4, 4), (128, 8, 2), (64, 4, 1)])
@pytest.mark.parametrize("T", [1, 16, 100, 300])
def test_prefill_attention_block_scaled_rows_and_two_term_output(ops, hd, Hq, Hkv, T):
    """Prefill attention over int16 * scale rows: every element enters the matrix cores as hi + lo, so only q and the
    probabilities carry a half rounding."""
    nb, b0, S, nseq = 2, 1, 320, 3
    qf = randn_f32((nb * T, Hq * hd), 190, std=1.5)
    q = qf.to(torch.float16)
    q_lo = (qf - q.float()).to(torch.float16)             # the two terms the projection's epilogue stores
    kc, ks, kn = _random_block_scaled((nseq, Hkv, S, hd), 191)
    vc, vs, vn = _random_block_scaled((nseq, Hkv, S, hd), 192)
    ks[:, :, T:] = float("nan")
    vs[:, :, T:] = float("nan")
    out = torch.zeros((nb * T, Hq * hd), dtype=torch.float16, device=DEV)
    out_lo = torch.zeros_like(out)
    ops.prefill_attention(q, kc, vc, out, nb, b0, T, Hq, Hkv, hd, S, kscale=ks, vscale=vs, out_lo=out_lo, q_lo=q_lo)
    torch.cuda.synchronize()
    qn = (np64(q) + np64(q_lo)).reshape(nb, T, Hq, hd)
    on, ln = np64(out).reshape(nb, T, Hq, hd), np64(out_lo).reshape(nb, T, Hq, hd)
    g = Hq // Hkv
    for b in range(nb):
        for u in range(Hq):
            for i in sorted(set(min(i, T - 1) for i in [0, 1, T // 2, T - 1] + list(range(0, T, 7)))):
                ref = orc.attend(qn[b, i, u], kn[b0 + b, u // g, : i + 1], vn[b0 + b, u // g, : i + 1])
                # every operand is a two-term sum: what is left is fp32 arithmetic and the fast exponential
                small = 3e-5 * (1 + np.abs(vn[b0 + b, u // g, : i + 1]).max())
                assert (np.abs(on[b, i, u] - ref) <= 0.5 * F16_EPS * np.abs(ref) * 1.02 + small).all(), (b, u, i)
                assert (np.abs(on[b, i, u] + ln[b, i, u] - ref) <= small + 2e-6 * np.abs(ref)).all(), (b, u, i, np.abs(on[b, i, u] + ln[b, i, u] - ref).max())


@pytest.mark.parametrize("M,K,F,kind", [(4, 256, 688, "halves"), (128, 512, 1000, "halves"), (77, 1000, 200, "packed"),
                                        (300, 256, 688, "packed"), (600, 264, 520, "tiled")])
def test_swiglu_two_term_output(ops, M, K, F, kind):
    """The SwiGLU epilogues' second half term: out is the oracle's value to half precision, out + out_lo to fp32 arithmetic."""
    A = randn_f16((M, K), 200)
    Wg, Wu = randn_bf16((F, K), 201, std=0.05), randn_bf16((F, K), 202, std=0.05)
    out = torch.zeros((M, F), dtype=torch.float16, device=DEV)
    out_lo = torch.zeros_like(out)
    if kind == "tiled":
        ops.gemm(A, [Wg, Wu], out, F, epilogue=1, kernel=2, out_lo=out_lo)
    else:
        Pg = torch.zeros(ops.packed_weight_bytes(F, K) // 2, dtype=torch.int16, device=DEV)
        Pu = torch.zeros_like(Pg)
        ops.pack_weights(Wg, Pg)
        ops.pack_weights(Wu, Pu)
        if kind == "halves":
            ops.gemm_packed_swiglu_halves(A, Pg, Pu, F, K, out, F, out_lo=out_lo)
        else:
            ops.gemm_packed(A, [Pg, Pu], [F, F], K, out, F, epilogue=1, out_lo=out_lo)
    torch.cuda.synchronize()
    gate = orc.linear(bits(Wg), np64(A))
    up = orc.linear(bits(Wu), np64(A))
    ref = np.vectorize(orc.silu)(gate) * up
    tol = 3e-6 * np.sqrt(K) * (np.abs(np64(A)).max() * 0.05 * np.sqrt(K)) * (1 + np.abs(up)) + 1e-6
    assert (np.abs(np64(out) - ref) <= 0.5 * F16_EPS * np.abs(ref) * 1.02 + tol).all()
    assert (np.abs(np64(out) + np64(out_lo) - ref) <= tol + 2e-6 * np.abs(ref)).all(), np.abs(np64(out) + np64(out_lo) - ref).max()


@pytest.mark.parametrize("Hq,Hkv,two_terms", [(8, 8, True), (16, 2, False)])
def test_qkv_projection_with_rotary_epilogue_block_scaled_equals_the_two_kernels(ops, Hq, Hkv, two_terms):
    """The prefill projection that rotates and stores in its epilogue writes the same int16 rows and scales as the fp32
    projection followed by rope_append (the row maximum and the quantisation are the same operations on the same bits);
    one row is checked against the oracle directly."""
    hd, K, T, nseq, b0, S = 128, 256, 40, 205, 3, 64        # 8200 rows: a ragged last tile, bands that wrap to the next sequence
    M = nseq * T
    n_all = (Hq + 2 * Hkv) * hd
    A = randn_f16(((2 if two_terms else 1) * M, K), 411)
    if two_terms:
        A[M:] *= 2.0 ** -11
    A_lo = A[M:] if two_terms else None
    Wq, Wk, Wv = randn_bf16((Hq * hd, K), 412, 0.05), randn_bf16((Hkv * hd, K), 413, 0.05), randn_bf16((Hkv * hd, K), 414, 0.05)
    tab = torch.empty((S, hd // 2, 2), dtype=torch.float32, device=DEV)
    ops.build_rope_table(tab, S, hd, 10000.0)
    mk = lambda: (torch.zeros((b0 + nseq, Hkv, S, hd), dtype=torch.int16, device=DEV),
                  torch.zeros((b0 + nseq, Hkv, S), dtype=torch.float32, device=DEV))
    (kc1, ks1), (vc1, vs1), (kc2, ks2), (vc2, vs2) = mk(), mk(), mk(), mk()
    q1 = torch.zeros((M, Hq * hd), dtype=torch.float16, device=DEV)
    q2, l1, l2 = torch.zeros_like(q1), torch.zeros_like(q1), torch.zeros_like(q1)
    ops.gemm_rope(A[:M], Wq, Wk, Wv, Hq, Hkv, hd, M, T, b0, tab, 1, S, q1, kc1, vc1, A_lo=A_lo, kscale=ks1, vscale=vs1, q_f16_lo=l1)
    part = torch.zeros((M, n_all), dtype=torch.float32, device=DEV)
    ops.gemm(A[:M], [Wq, Wk, Wv], part, n_all, M=M, kernel=2, A_lo=A_lo)
    zero = torch.zeros((1,), dtype=torch.int32, device=DEV)
    ops.rope_append(part, 1, M * n_all, M, T, b0, zero, tab, 1, Hq, Hkv, hd, S, None, q2, kc2, vc2, kscale=ks2, vscale=vs2, q_f16_lo=l2)
    torch.cuda.synchronize()
    assert torch.equal(l1, l2) and l1.abs().max() > 0
    assert torch.equal(q1, q2) and torch.equal(kc1, kc2) and torch.equal(vc1, vc2) and torch.equal(ks1, ks2) and torch.equal(vs1, vs2)
    assert ks1[b0:, :, :T].min() > 0 and ks1[:b0].abs().max() == 0 and ks1[:, :, T:].abs().max() == 0
    m = 7 * T + 11
    x = np64(A[m]) + (np64(A[M + m]) if two_terms else 0.0)
    for name, W, got, sc in (("k", Wk, kc1[b0 + 7, :, 11], ks1[b0 + 7, :, 11]), ("v", Wv, vc1[b0 + 7, :, 11], vs1[b0 + 7, :, 11])):
        y = (np64(W) @ x).reshape(Hkv, hd)
        want = y if name == "v" else orc.rope(y, 11, 10000.0, 1)
        deq = got.cpu().numpy().astype(np.float64) * np64(sc)[:, None]
        assert (np.abs(deq - want) <= 0.51 * np64(sc)[:, None] + 2e-4).all(), name
