"""Range of the half-precision activation path: what happens at and beyond +-65504.

The library states (header of the C ABI): every fp32 -> half conversion saturates at +-65504, values below that are
exact to half precision, nothing finite ever turns into inf or NaN, and block-scaled cache rows have no such limit.
The oracle has no limit at all, so the expected value of a saturating output is the oracle's value clamped here, in the
test: first term clamp(y, +-65504) rounded to half, second term clamp(y - first, +-65504) rounded to half.
"""
import numpy as np
import pytest
import torch

from oracle import orc
from tests.gpu_util import F16_EPS, DEV, bits, np64, randn_bf16, randn_f16, randn_f32, step
from workload import ModelShape, Workload, make_prompts, make_weights

pytestmark = pytest.mark.gpu
HMAX = 65504.0


@pytest.fixture(scope="module")
def ops():
    from paper_2406_14088_amd import ops as o
    return o


def clamp1(y):
    return np.clip(y, -HMAX, HMAX)


def clamp2(y):
    """what two saturating half terms can carry"""
    return np.clip(y, -2 * HMAX, 2 * HMAX)


def check_terms(hi, lo, ref, tol):
    hi, lo = np64(hi), (np64(lo) if lo is not None else None)
    assert np.isfinite(hi).all()
    assert (np.abs(hi - clamp1(ref)) <= 0.5 * F16_EPS * np.abs(clamp1(ref)) * 1.02 + tol).all(), np.abs(hi - clamp1(ref)).max()
    assert (np.abs(hi[np.abs(ref) > HMAX * 1.001]) == HMAX).all()
    if lo is not None:
        assert np.isfinite(lo).all()
        err = np.abs(hi + lo - clamp2(ref))
        assert (err <= 0.5 * F16_EPS * np.abs(lo) * 1.02 + 2e-6 * np.abs(ref) + tol).all(), err.max()
    return int((np.abs(ref) > HMAX).sum()), int((np.abs(ref) > 2 * HMAX).sum())


@pytest.mark.parametrize("d", [256, 4096])
def test_normalised_rows_beyond_the_half_limit(ops, d):
    """RMSNorm gains of 2^15 .. 2^17: most normalised elements (order 1 before the gain) leave the half range."""
    M = 6
    x = randn_f32((M, d), 900 + d, std=2.0)
    part = randn_f32((2, M, d), 901 + d)
    gain = ((1.0 + 0.3 * randn_f32((d,), 902)) * 2.0 ** 15 * (1 + (torch.arange(d, device=DEV) % 3))).to(torch.bfloat16)
    h = torch.empty((M, d), dtype=torch.float16, device=DEV)
    h_lo = torch.empty_like(h)
    xs = np64(x) + np64(part).sum(0)
    ops.add_rmsnorm(x, part, 2, M * d, gain, 1e-5, h, h_lo)
    torch.cuda.synchronize()
    ref = orc.rmsnorm(xs, bits(gain), float(np.float32(1e-5)))
    # fp32 sums of x and the partials: an absolute error of ~1e-7 * |x| before the gain, i.e. ~1e-6 * gain after it
    over, over2 = check_terms(h, h_lo, ref, 1e-6 * np.abs(np64(gain))[None, :] + 2e-6 * np.abs(ref))
    assert over > M * d // 10 and over2 > 0 and over < M * d          # the case covers both sides of both limits


@pytest.mark.parametrize("M,K,F,kind", [(4, 256, 688, "skinny"), (4, 256, 688, "halves"), (128, 512, 1000, "halves"),
                                        (77, 1000, 200, "packed"), (300, 256, 688, "packed"), (600, 264, 520, "tiled")])
def test_swiglu_outputs_beyond_the_half_limit(ops, M, K, F, kind):
    """Gate and up values of a few hundred: products from well inside the half range to ten times beyond it."""
    step(f"swiglu range M={M} K={K} F={F} {kind}")
    a_std, w_std = 30.0, 0.5
    A = randn_f16((M, K), 910, std=a_std)
    Wg, Wu = randn_bf16((F, K), 911, std=w_std), randn_bf16((F, K), 912, std=w_std)
    out = torch.zeros((M, F), dtype=torch.float16, device=DEV)
    out_lo = torch.zeros_like(out) if kind != "skinny" else None
    if kind == "skinny":
        ops.gemm(A, [Wg, Wu], out, F, epilogue=1, kernel=1)
    elif kind == "tiled":
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
    gate, up = orc.linear(bits(Wg), np64(A)), orc.linear(bits(Wu), np64(A))
    ref = np.vectorize(orc.silu)(gate) * up
    # fp32 accumulation of K terms of size a_std * w_std: absolute error of gate and of up, carried into the product
    acc = 3e-6 * np.sqrt(K) * (np.abs(np64(A)).max() * w_std * np.sqrt(K))
    tol = acc * (1 + np.abs(up) + np.abs(gate)) + 1e-6
    over, over2 = check_terms(out, out_lo, ref, tol)
    assert over > 0 and over2 > 0 and over < M * F // 2


@pytest.mark.parametrize("block_scaled", [False, True])
def test_appended_rows_beyond_the_half_limit(ops, block_scaled):
    """Projection outputs of order 1e5 into rope_append: half cache rows and the half copy of q saturate, block-scaled rows
    keep their relative precision (their scale is fp32)."""
    hd, Hq, Hkv, S, T, nb, b0, pos0 = 128, 4, 2, 24, 5, 2, 1, 3
    tab = torch.empty((S, hd // 2, 2), dtype=torch.float32, device=DEV)
    ops.build_rope_table(tab, S, hd, 10000.0)
    ld, M = (Hq + 2 * Hkv) * hd, nb * T
    qkv = randn_f32((1, M, ld), 920, std=5e4)
    dt = torch.int16 if block_scaled else torch.float16
    kc = torch.zeros((b0 + nb, Hkv, S, hd), dtype=dt, device=DEV)
    vc = torch.zeros_like(kc)
    ks = torch.zeros((b0 + nb, Hkv, S), dtype=torch.float32, device=DEV) if block_scaled else None
    vs = torch.zeros_like(ks) if block_scaled else None
    qf = torch.empty((M, Hq * hd), dtype=torch.float32, device=DEV)
    qh = torch.zeros((M, Hq * hd), dtype=torch.float16, device=DEV)
    ql = torch.zeros_like(qh)
    d_pos = torch.tensor([pos0], dtype=torch.int32, device=DEV)
    ops.rope_append(qkv, 1, M * ld, M, T, b0, d_pos, tab, 1, Hq, Hkv, hd, S, qf, qh, kc, vc, kscale=ks, vscale=vs, q_f16_lo=ql)
    torch.cuda.synchronize()
    tot = np64(qkv)[0]
    n_over = 0
    for m in range(M):
        b, pos = b0 + m // T, pos0 + m % T
        q = orc.rope(tot[m, : Hq * hd].reshape(Hq, hd), pos, 10000.0, 1)
        k = orc.rope(tot[m, Hq * hd: (Hq + Hkv) * hd].reshape(Hkv, hd), pos, 10000.0, 1)
        v = tot[m, (Hq + Hkv) * hd:].reshape(Hkv, hd)
        n_over += check_terms(qh[m].reshape(Hq, hd), ql[m].reshape(Hq, hd), q, 3e-6 * np.abs(q).max())[0]
        if block_scaled:
            for ref, rows, sc in ((k, kc[b, :, pos], ks[b, :, pos]), (v, vc[b, :, pos], vs[b, :, pos])):
                sc = np64(sc)
                amax = np.abs(ref).max(-1)
                assert (np.abs(sc - amax / 32767.0) <= 3e-6 * amax / 32767.0).all()
                assert (np.abs(rows.cpu().numpy().astype(np.float64) * sc[:, None] - ref) <= 0.5 * sc[:, None] * 1.001 + 1e-6 * np.abs(ref)).all()
        else:
            n_over += check_terms(kc[b, :, pos], None, k, 3e-6 * np.abs(k).max())[0]
            n_over += check_terms(vc[b, :, pos], None, v, 3e-6 * np.abs(v).max())[0]
    assert n_over > 0


@pytest.mark.parametrize("Hq,Hkv", [(4, 2), (16, 2)])
def test_decode_attention_over_rows_at_the_half_limit(ops, Hq, Hkv):
    """Half cache rows holding +-65504 and queries of order 100: scores of order 1e8, a one-hot softmax; the output is a
    cache row, finite, and the oracle's (vector kernel, and the matrix-core kernel of grouped-query shapes)."""
    B, hd, S, length = 2, 128, 160, 150
    q = randn_f32((B, Hq * hd), 930, std=100.0)
    kc = randn_f16((B, Hkv, S, hd), 931, std=3e4)          # torch's conversion gives inf beyond the range: bring those back
    vc = randn_f16((B, Hkv, S, hd), 932, std=3e4)
    kc, vc = torch.nan_to_num(kc, posinf=HMAX, neginf=-HMAX), torch.nan_to_num(vc, posinf=HMAX, neginf=-HMAX)
    assert (kc.abs() == HMAX).any() and (vc.abs() == HMAX).any()
    d_len = torch.tensor([length], dtype=torch.int32, device=DEV)
    out = torch.zeros((B, Hq * hd), dtype=torch.float16, device=DEV)
    out_lo = torch.zeros_like(out)
    for nsplit in (1, 3):
        ws = torch.empty(max(ops.decode_attention_ws_floats(B, Hq, hd, nsplit), 1), dtype=torch.float32, device=DEV)
        ops.decode_attention(q, kc, vc, d_len, out, ws, B, Hq, Hkv, hd, S, nsplit, out_lo=out_lo)
        torch.cuda.synchronize()
        qn, kn, vn = np64(q).reshape(B, Hq, hd), np64(kc), np64(vc)
        for b in range(B):
            for u in range(Hq):
                ref = orc.attend(qn[b, u], kn[b, u // (Hq // Hkv), : length + 1], vn[b, u // (Hq // Hkv), : length + 1])
                check_terms(out[b].reshape(Hq, hd)[u], out_lo[b].reshape(Hq, hd)[u], ref, 1e-6 * np.abs(ref).max() + 1e-6)


def scaled_gains(W, attn=1.0, ffn=1.0, final=1.0):
    """powers of two on the gain vectors: exact in bf16"""
    out = dict(W)
    out["attn_norm"] = [t * attn for t in W["attn_norm"]]
    out["ffn_norm"] = [t * ffn for t in W["ffn_norm"]]
    out["final_norm"] = W["final_norm"] * final
    return out


def run(shape, W, B, P, G, precision, packed, compare):
    from paper_2406_14088_amd import Generator
    prompts = make_prompts(Workload("t", 31, shape, B, P, G))
    om = orc.OracleModel(shape, orc.weights_to_numpy(W), B, P + G)
    gen = Generator(shape, {k: ([t.to(DEV) for t in v] if isinstance(v, list) else v.to(DEV)) for k, v in W.items()}, B, P + G,
                    packed=packed, precision=precision)
    o_logits, tok = om.prefill(prompts.numpy())
    g_logits, g_next = gen.prefill(prompts.to(DEV))
    torch.cuda.synchronize()
    compare(np64(g_logits), g_next.cpu().numpy(), o_logits)
    for _ in range(G - 1):
        o_logits, nxt = om.decode_step(tok)
        g_logits, g_next = gen.decode_step(torch.from_numpy(tok).to(DEV))
        torch.cuda.synchronize()
        compare(np64(g_logits), g_next.cpu().numpy(), o_logits)
        tok = nxt
    gen.close()


@pytest.mark.parametrize("packed", [True, False])
@pytest.mark.parametrize("precision", [1, 2, 3])
def test_generation_with_large_activations_inside_the_range(precision, packed):
    """FFN-norm gains of 64 (SwiGLU outputs up to ~1e4, the FFN dominating the residual stream) and a final-norm gain of
    1024 (LM-head inputs up to ~4e3, logits of a few hundred): everything stays inside the half range, so the result is the
    oracle's to the usual tolerance, which scales with the logits, i.e. with the final gain."""
    shape = ModelShape(3, 512, 4, 4, 128, 1384, 2048)
    W = scaled_gains(make_weights(shape, 31, device="cpu"), ffn=64.0, final=1024.0)
    worst = [0.0, 0.0]

    def compare(gl, gn, ol):
        assert np.isfinite(gl).all()
        assert np.array_equal(gn, np.array([orc.argmax(r) for r in gl]))
        worst[0] = max(worst[0], np.abs(gl - ol).max())
        worst[1] = max(worst[1], np.abs(ol).max())

    run(shape, W, 5, 20, 4, precision, packed, compare)
    step(f"  level {precision} packed={packed}: max-abs logit error {worst[0]:.3e} on logits up to {worst[1]:.1f} (tolerance {3e-2 * 1024:.1f})")
    assert worst[1] > 100.0 and worst[0] <= 3e-2 * 1024.0


@pytest.mark.parametrize("packed", [True, False])
@pytest.mark.parametrize("precision", [1, 2, 3])
@pytest.mark.parametrize("which", ["attention", "ffn", "all", "all_grouped_query"])
def test_generation_beyond_the_range_stays_finite(which, precision, packed):
    """Gains of 2^17 on the attention norms (normalised rows, q, k and v past 65504), on the FFN norms (SwiGLU outputs of order
    1e9), on everything: outputs saturate, so the oracle (no limit) is no reference any more; what must hold is what the
    header promises: finite logits, tokens that are the argmax of those logits, no fault."""
    shape = ModelShape(3, 1024, 8, 1, 128, 1000, 2048) if which == "all_grouped_query" else ModelShape(3, 512, 4, 4, 128, 1384, 2048)
    big = 2.0 ** 17
    W = scaled_gains(make_weights(shape, 32, device="cpu", std=0.05), attn=big if which != "ffn" else 1.0,
                     ffn=big if which != "attention" else 1.0, final=big if which.startswith("all") else 1.0)
    seen = [0]

    def compare(gl, gn, ol):
        assert np.isfinite(gl).all()
        assert np.array_equal(gn, np.array([orc.argmax(r) for r in gl]))
        assert np.abs(gl).max() > 0
        seen[0] += 1

    run(shape, W, 130, 6, 3, precision, packed, compare)
    assert seen[0] == 3
