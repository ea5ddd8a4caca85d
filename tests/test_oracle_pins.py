"""Pins for the CPU oracle: checks against what the paper and the mathematics fix, never against itself.

Citations: paper Section 2.1 (generation = prefill forward pass + single-token decode loop), Appendix A
(model-configuration table with exact parameter counts; fixed-length synthetic prompts).
"""
import os

import numpy as np
import pytest

from oracle import orc
from tests import ref_numpy
from workload import LLAMA3_TABLE_SHAPES, PRESETS, ModelShape, make_prompts, make_weights

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def small_shape(**kw):
    base = dict(n_layers=2, hidden=32, n_heads=4, n_kv_heads=2, head_dim=8, ffn=48, vocab=64,
                rope_base=10000.0, rms_eps=1e-5, rope_style=1)
    base.update(kw)
    return ModelShape(**base)


def rand_weights(shape, seed=0, std=0.2, gains_random=True):
    """float32 weights with NON-unit gains so that a misplaced or dropped gain is caught."""
    r = np.random.default_rng(seed)
    d, qd, kvd = shape.hidden, shape.n_heads * shape.head_dim, shape.n_kv_heads * shape.head_dim

    def mat(n, k):
        return (r.standard_normal((n, k)) * std).astype(np.float32)

    def gain():
        return (1.0 + 0.3 * r.standard_normal(d)).astype(np.float32) if gains_random else np.ones(d, np.float32)

    L = shape.n_layers
    return {
        "tok_emb": mat(shape.vocab, d), "final_norm": gain(), "lm_head": mat(shape.vocab, d),
        "attn_norm": [gain() for _ in range(L)], "ffn_norm": [gain() for _ in range(L)],
        "wq": [mat(qd, d) for _ in range(L)], "wk": [mat(kvd, d) for _ in range(L)],
        "wv": [mat(kvd, d) for _ in range(L)], "wo": [mat(d, qd) for _ in range(L)],
        "w_gate": [mat(shape.ffn, d) for _ in range(L)], "w_up": [mat(shape.ffn, d) for _ in range(L)],
        "w_down": [mat(d, shape.ffn) for _ in range(L)],
    }


def to64(W):
    return {k: ([a.astype(np.float64) for a in v] if isinstance(v, list) else v.astype(np.float64)) for k, v in W.items()}


def rand_tokens(shape, B, T, seed=1):
    return np.random.default_rng(seed).integers(0, shape.vocab, (B, T)).astype(np.int32)


# ------------------------------------------------------------------ parameter inventory (paper's table)

def test_param_count_matches_paper_table():
    rows = [l.split() for l in open(os.path.join(GOLDEN, "llama3_param_counts.txt")) if l.strip() and not l.startswith("#")]
    assert len(rows) == 4
    for name, hidden, ffn, layers, heads, kv, vocab, total, wo_out in rows:
        s = LLAMA3_TABLE_SHAPES[name]
        assert (s.hidden, s.ffn, s.n_layers, s.n_heads, s.n_kv_heads, s.vocab) == tuple(
            int(v) for v in (hidden, ffn, layers, heads, kv, vocab))
        assert orc.param_count(s) == int(total)
        assert orc.param_count(s) - s.vocab * s.hidden == int(wo_out)


def test_param_count_counts_actual_tensors():
    s = small_shape()
    W = rand_weights(s)
    n = sum(sum(a.size for a in v) if isinstance(v, list) else v.size for v in W.values())
    assert orc.param_count(s) == n


def test_kv_bytes_closed_form():
    # 7B multi-head shape in bf16: 2 (K and V) * 32 layers * 4096 * 2 bytes = 0.5 MiB per token and sequence
    assert orc.kv_bytes_per_token(PRESETS["llama7b"].shape, 2) == 524288
    assert orc.kv_bytes_per_token(PRESETS["llama70b"].shape, 2) == 2 * 80 * 8 * 128 * 2


# ------------------------------------------------------------------ sub-functions

def test_linear_is_x_times_w_transposed():
    r = np.random.default_rng(3)
    W = r.standard_normal((7, 13)).astype(np.float32)
    X = r.standard_normal((5, 13))
    assert np.allclose(orc.linear(W, X), X @ W.astype(np.float64).T, rtol=0, atol=1e-12)
    # a non-square case where a transposed operand cannot go unnoticed: W = row selector
    W = np.zeros((2, 3), np.float32); W[0, 2] = 1.0; W[1, 0] = 2.0
    assert np.array_equal(orc.linear(W, np.array([[1.0, 5.0, 7.0]])), np.array([[7.0, 2.0]]))


def test_linear_bf16_bits_are_widened_exactly():
    # 0x3F80 = 1.0, 0xC000 = -2.0, 0x3DCD ~ 0.1001 (bf16)
    W = np.array([[0x3F80, 0xC000, 0x3DCD]], dtype=np.uint16)
    x = np.array([[1.0, 1.0, 1.0]])
    third = np.array([0x3DCD << 16], dtype=np.uint32).view(np.float32)[0]
    assert orc.linear(W, x)[0, 0] == 1.0 - 2.0 + float(third)


def test_rmsnorm_pins():
    r = np.random.default_rng(4)
    x = r.standard_normal(64)
    one = np.ones(64, np.float32)
    y = orc.rmsnorm(x, one, 0.0)
    assert abs(np.sqrt((y * y).mean()) - 1.0) < 1e-12                      # unit RMS for unit gain
    assert np.allclose(orc.rmsnorm(37.5 * x, one, 0.0), y, atol=1e-12)     # scale invariance at eps = 0
    g = r.standard_normal(64).astype(np.float32)
    assert np.allclose(orc.rmsnorm(x, g, 1e-5), g * x / np.sqrt((x * x).mean() + 1e-5), atol=1e-12)
    # d = 1 closed form: eps sits inside the square root, added to the mean
    assert abs(orc.rmsnorm(np.array([3.0]), np.array([2.0], np.float32), 7.0)[0] - 2.0 * 3.0 / 4.0) < 1e-15


@pytest.mark.parametrize("style", [0, 1])
def test_rope_pins(style):
    r = np.random.default_rng(5)
    v = r.standard_normal(16)
    assert np.array_equal(orc.rope(v, 0, 10000.0, style), v)               # position 0 is the identity
    w = orc.rope(v, 11, 10000.0, style)
    ia = (lambda k: 2 * k) if style == 0 else (lambda k: k)
    ib = (lambda k: 2 * k + 1) if style == 0 else (lambda k: k + 8)
    for k in range(8):                                                     # each pair keeps its length
        assert abs(np.hypot(w[ia(k)], w[ib(k)]) - np.hypot(v[ia(k)], v[ib(k)])) < 1e-12
    # pair 0 turns by exactly `pos` radians, counter-clockwise; pair r by pos * base^(-2r/hd)
    e = np.zeros(16); e[ia(0)] = 1.0
    w = orc.rope(e, 3, 10000.0, style)
    assert abs(w[ia(0)] - np.cos(3.0)) < 1e-15 and abs(w[ib(0)] - np.sin(3.0)) < 1e-15
    e = np.zeros(16); e[ia(4)] = 1.0
    w = orc.rope(e, 3, 10000.0, style)
    ang = 3.0 * 10000.0 ** (-2.0 * 4 / 16)                                 # = 3 / 100
    assert abs(ang - 0.03) < 1e-15
    assert abs(w[ia(4)] - np.cos(ang)) < 1e-15 and abs(w[ib(4)] - np.sin(ang)) < 1e-15
    # a huge base freezes every pair but the first
    w = orc.rope(v, 9, 1e300, style)
    keep = [i for k in range(1, 8) for i in (ia(k), ib(k))]
    assert np.allclose(w[keep], v[keep], atol=1e-12)


@pytest.mark.parametrize("style", [0, 1])
def test_rope_relative_position_property(style):
    r = np.random.default_rng(6)
    q, k = r.standard_normal(32), r.standard_normal(32)
    ref = orc.rope(q, 9, 10000.0, style) @ orc.rope(k, 4, 10000.0, style)
    for shift in (1, 17, 300):
        got = orc.rope(q, 9 + shift, 10000.0, style) @ orc.rope(k, 4 + shift, 10000.0, style)
        assert abs(got - ref) < 1e-10


def brute_attention(q, K, V):
    """explicit O(n*hd) loops with python floats"""
    n, hd = K.shape
    s = [sum(float(q[e]) * float(K[j, e]) for e in range(hd)) / np.sqrt(hd) for j in range(n)]
    m = max(s)
    p = [np.exp(v - m) for v in s]
    z = sum(p)
    return np.array([sum(p[j] / z * float(V[j, e]) for j in range(n)) for e in range(hd)])


def test_attend_pins():
    r = np.random.default_rng(7)
    for n, hd in [(1, 4), (3, 2), (8, 8), (5, 6)]:
        q, K, V = r.standard_normal(hd), r.standard_normal((n, hd)), r.standard_normal((n, hd))
        assert np.allclose(orc.attend(q, K, V), brute_attention(q, K, V), atol=1e-13)
    q, K, V = r.standard_normal(8), r.standard_normal((1, 8)), r.standard_normal((1, 8))
    assert np.array_equal(orc.attend(q, K, V), V[0])                        # one key: output is its value
    K, V = r.standard_normal((6, 8)), r.standard_normal((6, 8))
    assert np.allclose(orc.attend(np.zeros(8), K, V), V.mean(0), atol=1e-14)  # uniform scores: mean of values
    # softmax shift invariance: adding one vector to every key shifts all scores equally
    assert np.allclose(orc.attend(q, K + 3.0, V), orc.attend(q, K, V), atol=1e-12)
    # large scores stay finite and pick the dominating key
    big = orc.attend(100.0 * np.ones(8), np.vstack([np.ones(8), -np.ones(8), 0.5 * np.ones(8)]), np.eye(3, 8))
    assert np.all(np.isfinite(big)) and np.allclose(big, np.eye(3, 8)[0], atol=1e-12)
    # scale is 1/sqrt(hd): two keys with q.k = hd*ln(3)/sqrt(hd)... check through the probability ratio
    hd = 4
    q = np.ones(hd); K = np.array([np.full(hd, np.log(3.0) / 2.0), np.zeros(hd)]); V = np.array([[1.0, 0, 0, 0], [0, 1.0, 0, 0]])
    o = orc.attend(q, K, V)                                                 # scores: (4*ln3/2)/2 = ln 3 and 0
    assert abs(o[0] - 0.75) < 1e-14 and abs(o[1] - 0.25) < 1e-14


def test_silu_and_argmax_pins():
    assert orc.silu(0.0) == 0.0
    assert abs(orc.silu(40.0) - 40.0) < 1e-12 and abs(orc.silu(-40.0)) < 1e-12
    assert abs(orc.silu(1.0) - 1.0 / (1.0 + np.exp(-1.0))) < 1e-16
    assert abs(orc.silu(-2.0) + 2.0 / (1.0 + np.exp(2.0))) < 1e-16
    assert orc.argmax(np.array([1.0, 5.0, 5.0, 2.0])) == 1                  # ties: lowest index
    assert orc.argmax(np.array([-3.0, -1.0, -2.0])) == 1
    assert orc.argmax(np.zeros(9)) == 0
    assert orc.argmax(np.array([0.0, np.nan])) == -1


# ------------------------------------------------------------------ whole model

@pytest.mark.parametrize("style", [0, 1])
@pytest.mark.parametrize("kv_heads", [4, 2, 1])
def test_forward_all_matches_independent_numpy_statement(style, kv_heads):
    s = small_shape(rope_style=style, n_kv_heads=kv_heads)
    W = rand_weights(s, seed=10 + kv_heads)
    tok = rand_tokens(s, 3, 9)
    m = orc.OracleModel(s, W, 3, 9)
    got = m.forward_all(tok)
    ref = ref_numpy.forward_all(s, to64(W), tok)
    assert np.abs(got - ref).max() < 1e-10


def test_tiny_preset_shape_matches_numpy_statement():
    s = PRESETS["tiny"].shape
    W = rand_weights(s, seed=21, std=0.05)
    tok = rand_tokens(s, 2, 6)
    m = orc.OracleModel(s, W, 2, 6)
    assert np.abs(m.forward_all(tok) - ref_numpy.forward_all(s, to64(W), tok)).max() < 1e-10


def test_zero_layers_closed_form():
    s = small_shape(n_layers=0)
    W = rand_weights(s, seed=22)
    tok = rand_tokens(s, 2, 5)
    m = orc.OracleModel(s, W, 2, 5)
    e = W["tok_emb"].astype(np.float64)[tok]
    h = W["final_norm"] * e / np.sqrt((e * e).mean(-1, keepdims=True) + float(np.float32(s.rms_eps)))
    assert np.abs(m.forward_all(tok) - h @ W["lm_head"].astype(np.float64).T).max() < 1e-12


def test_zero_output_projections_make_layers_identity():
    s = small_shape()
    W = rand_weights(s, seed=23)
    for l in range(s.n_layers):
        W["wo"][l][:] = 0.0
        W["w_down"][l][:] = 0.0
    tok = rand_tokens(s, 2, 5)
    W0 = {k: ([] if isinstance(v, list) else v) for k, v in W.items()}
    got = orc.OracleModel(s, W, 2, 5).forward_all(tok)
    ref = orc.OracleModel(small_shape(n_layers=0), W0, 2, 5).forward_all(tok)
    assert np.array_equal(got, ref)


def test_zero_gate_kills_ffn_only():
    s = small_shape(n_layers=1)
    W = rand_weights(s, seed=24)
    tok = rand_tokens(s, 1, 4)
    base = orc.OracleModel(s, W, 1, 4).forward_all(tok)
    W2 = {k: ([a.copy() for a in v] if isinstance(v, list) else v) for k, v in W.items()}
    W2["w_gate"][0][:] = 0.0                      # silu(0) * up = 0  -> FFN contributes nothing
    W3 = {k: ([a.copy() for a in v] if isinstance(v, list) else v) for k, v in W.items()}
    W3["w_down"][0][:] = 0.0
    a = orc.OracleModel(s, W2, 1, 4).forward_all(tok)
    b = orc.OracleModel(s, W3, 1, 4).forward_all(tok)
    assert np.array_equal(a, b) and np.abs(a - base).max() > 1e-3


def test_causality_prefix_and_future_independence():
    s = small_shape()
    W = rand_weights(s, seed=25)
    tok = rand_tokens(s, 2, 10)
    m = orc.OracleModel(s, W, 2, 10)
    full = m.forward_all(tok)
    for t in (0, 3, 8):
        assert np.array_equal(m.forward_all(tok[:, : t + 1])[:, t], full[:, t])
    tok2 = tok.copy()
    tok2[:, 6:] = (tok2[:, 6:] + 7) % s.vocab
    other = m.forward_all(tok2)
    assert np.array_equal(other[:, :6], full[:, :6]) and np.abs(other[:, 6:] - full[:, 6:]).max() > 1e-3


def test_batch_independence():
    s = small_shape()
    W = rand_weights(s, seed=26)
    tok = rand_tokens(s, 4, 6)
    m = orc.OracleModel(s, W, 4, 6)
    full = m.forward_all(tok)
    perm = np.array([2, 0, 3, 1])
    assert np.array_equal(m.forward_all(tok[perm]), full[perm])
    assert np.array_equal(m.forward_all(tok[1:2]), full[1:2])


def test_cached_route_equals_plain_definition():
    s = small_shape()
    W = rand_weights(s, seed=27)
    P, G, B = 5, 6, 3
    tok = rand_tokens(s, B, P + G)
    m = orc.OracleModel(s, W, B, P + G)
    full = m.forward_all(tok)
    logits, nxt = m.prefill(tok[:, :P])
    assert np.abs(logits - full[:, P - 1]).max() < 1e-12
    assert np.array_equal(nxt, full[:, P - 1].argmax(-1))
    for i in range(G):                                 # teacher forcing with the given tokens
        logits, nxt = m.decode_step(tok[:, P + i])
        assert np.abs(logits - full[:, P + i]).max() < 1e-12
        assert np.array_equal(nxt, full[:, P + i].argmax(-1))
    # prefill(P) == prefill(P-k) followed by k decode steps
    m.reset()
    m.prefill(tok[:, : P - 3])
    for i in range(3):
        logits, _ = m.decode_step(tok[:, P - 3 + i])
    assert np.abs(logits - full[:, P - 1]).max() < 1e-12


def test_feeding_a_sequence_in_spans_equals_plain_definition():
    """prefill(first piece) + extend(further pieces of any length) reaches the logits of the plain, cache-free forward pass
    at every span end, and decode steps continue from there (the route the long-context GPU tests take on the oracle)."""
    s = small_shape(n_kv_heads=2)
    W = rand_weights(s, seed=31)
    B, T = 2, 17
    tok = rand_tokens(s, B, T)
    m = orc.OracleModel(s, W, B, T)
    full = m.forward_all(tok)
    logits, _ = m.prefill(tok[:, :4])
    assert np.abs(logits - full[:, 3]).max() < 1e-12
    at = 4
    for n in (1, 5, 3, 2):
        logits = m.extend(tok[:, at: at + n])
        at += n
        assert np.abs(logits - full[:, at - 1]).max() < 1e-12
    assert m.extend(tok[:, at: at + 1], want_logits=False) is None
    logits, nxt = m.decode_step(tok[:, at + 1])
    assert np.abs(logits - full[:, at + 1]).max() < 1e-12 and np.array_equal(nxt, full[:, at + 1].argmax(-1))
    with pytest.raises(orc.OracleError) as e:          # capacity
        m.extend(tok[:, :1])
    assert e.value.code == -3


def test_gqa_equals_mha_with_replicated_kv_rows():
    s = small_shape(n_kv_heads=2)
    W = rand_weights(s, seed=28)
    tok = rand_tokens(s, 2, 7)
    got = orc.OracleModel(s, W, 2, 7).forward_all(tok)
    smha = small_shape(n_kv_heads=4)
    W2 = dict(W)
    rep = lambda a: np.repeat(a.reshape(2, s.head_dim, -1), 2, axis=0).reshape(4 * s.head_dim, -1)
    W2["wk"] = [rep(a) for a in W["wk"]]
    W2["wv"] = [rep(a) for a in W["wv"]]
    ref = orc.OracleModel(smha, W2, 2, 7).forward_all(tok)
    assert np.abs(got - ref).max() < 1e-12


def test_rope_styles_equivalent_under_row_permutation():
    s1 = small_shape(rope_style=1)
    s0 = small_shape(rope_style=0)
    W = rand_weights(s1, seed=29)
    hd, half = s1.head_dim, s1.head_dim // 2
    # style-1 row r (first half) / r+half (second half) of a head  <->  style-0 rows 2r / 2r+1
    perm_head = np.empty(hd, dtype=int)
    perm_head[0::2] = np.arange(half)
    perm_head[1::2] = np.arange(half) + half

    def permute(a):
        H = a.shape[0] // hd
        idx = (np.arange(H)[:, None] * hd + perm_head[None, :]).reshape(-1)
        return a[idx]

    W0 = dict(W)
    W0["wq"] = [permute(a) for a in W["wq"]]
    W0["wk"] = [permute(a) for a in W["wk"]]
    tok = rand_tokens(s1, 2, 7)
    a = orc.OracleModel(s1, W, 2, 7).forward_all(tok)
    b = orc.OracleModel(s0, W0, 2, 7).forward_all(tok)
    assert np.abs(a - b).max() < 1e-11


def test_bf16_bits_and_fp32_values_give_the_same_results():
    import torch
    s = small_shape()
    W = rand_weights(s, seed=30)
    Wt = {k: ([torch.from_numpy(a).to(torch.bfloat16) for a in v] if isinstance(v, list) else torch.from_numpy(v).to(torch.bfloat16))
          for k, v in W.items()}
    tok = rand_tokens(s, 2, 5)
    a = orc.OracleModel(s, orc.weights_to_numpy(Wt, as_bf16_bits=True), 2, 5).forward_all(tok)
    b = orc.OracleModel(s, orc.weights_to_numpy(Wt, as_bf16_bits=False), 2, 5).forward_all(tok)
    assert np.abs(a - b).max() < 1e-12        # same values; only the summation order of the two loops may differ


def test_error_paths():
    s = small_shape()
    W = rand_weights(s, seed=31)
    m = orc.OracleModel(s, W, 2, 6)
    with pytest.raises(orc.OracleError):
        m.decode_step(np.zeros(2, np.int32))                 # decode before prefill
    with pytest.raises(orc.OracleError):
        m.prefill(np.zeros((3, 4), np.int32))                # batch over capacity
    with pytest.raises(orc.OracleError):
        m.prefill(np.full((2, 4), s.vocab, np.int32))        # token id out of range
    m.prefill(np.zeros((2, 6), np.int32))
    with pytest.raises(orc.OracleError):
        m.decode_step(np.zeros(2, np.int32))                 # sequence capacity reached
    with pytest.raises(orc.OracleError):
        orc.OracleModel(small_shape(n_kv_heads=3), W, 1, 1)  # heads not divisible by kv heads


# ---------------------------------------------------------------------------------------------- token log-probability
def test_token_logprob_pins():
    """log-softmax gather: a library routine (scipy), closed forms and invariants."""
    from scipy.special import log_softmax, logsumexp
    rng = np.random.default_rng(77)
    x = rng.normal(0, 3.0, size=1000)
    ref = log_softmax(x)
    for t in (0, 1, 499, 999):
        assert abs(orc.token_logprob(x, t) - ref[t]) <= 1e-12
    # probabilities sum to one
    assert abs(logsumexp([orc.token_logprob(x, t) for t in range(1000)])) <= 1e-10
    # uniform logits: -log n, whatever the common value
    for c in (0.0, -7.5, 1e4):
        assert abs(orc.token_logprob(np.full(64, c), 5) + np.log(64)) <= 1e-12
    # shift invariance, and no overflow for large logits
    assert abs(orc.token_logprob(x + 900.0, 3) - orc.token_logprob(x, 3)) <= 1e-9
    assert np.isfinite(orc.token_logprob(np.array([800.0, -800.0, 0.0]), 1))
    # two logits: log sigmoid of the difference
    assert abs(orc.token_logprob(np.array([1.25, -0.5]), 0) + np.log1p(np.exp(-1.75))) <= 1e-14
    # a planted mistake would show: gathering the wrong index or dropping the max term
    assert abs(orc.token_logprob(np.array([0.0, np.log(3.0)]), 1) - np.log(0.75)) <= 1e-14
    assert np.isnan(orc.token_logprob(x, 1000)) and np.isnan(orc.token_logprob(x, -1))


def test_sequence_logprobs_follow_the_next_token():
    wl = PRESETS["tiny"]
    W = make_weights(wl.shape, wl.index, device="cpu")
    om = orc.OracleModel(wl.shape, orc.weights_to_numpy(W), 2, 8)
    toks = make_prompts(wl, batch=2, prompt_len=8).numpy()
    logits = om.forward_all(toks)
    lp = orc.sequence_logprobs(logits, toks)
    assert lp.shape == (2, 7) and (lp < 0).all()
    from scipy.special import log_softmax
    assert abs(lp[1, 3] - log_softmax(logits[1, 3])[toks[1, 4]]) <= 1e-12     # position i scores token i+1
    # causality carries over: the first k log-probs depend only on the first k+1 tokens
    toks2 = toks.copy()
    toks2[:, 6:] = (toks2[:, 6:] + 1) % wl.shape.vocab
    lp2 = orc.sequence_logprobs(om.forward_all(toks2), toks2)
    assert np.array_equal(lp[:, :5], lp2[:, :5]) and not np.array_equal(lp[:, 5:], lp2[:, 5:])
    om.close()


# ---------------------------------------------------------------------------------------------- temperature sampling
def test_sampling_by_inversion_pins():
    from scipy.special import softmax
    rng = np.random.default_rng(5)
    x = rng.normal(0, 2.0, size=50)
    # against the library: index where the cumulative softmax first exceeds u
    for temp in (0.5, 1.0, 2.0):
        cdf = np.cumsum(softmax(x / temp))
        for u in (0.0, 0.1234, 0.5, 0.87, 0.999):
            assert orc.sample(x, temp, u) == int(np.searchsorted(cdf, u, side="right"))
    # uniform logits: the u-th equal slice
    for u, want in ((0.0, 0), (0.249, 0), (0.251, 1), (0.99, 3)):
        assert orc.sample(np.zeros(4), 1.0, u) == want
    # two logits with probabilities 1/4 and 3/4
    two = np.array([0.0, np.log(3.0)])
    assert orc.sample(two, 1.0, 0.2499) == 0 and orc.sample(two, 1.0, 0.2501) == 1
    # temperature scales the logits: at T = 2 the same logits give 1/(1+sqrt 3) and the rest
    b = 1.0 / (1.0 + np.sqrt(3.0))
    assert orc.sample(two, 2.0, b - 1e-6) == 0 and orc.sample(two, 2.0, b + 1e-6) == 1
    # cold temperature concentrates on the argmax; a probability-zero tail is never drawn
    assert all(orc.sample(x, 1e-3, u) == int(np.argmax(x)) for u in (0.0, 0.5, 0.999999))
    assert orc.sample(np.array([0.0, -5000.0]), 1.0, 0.9999999999) == 0
    # empirical frequencies follow the probabilities (20000 evenly spaced draws: exact up to 1/20000 per cell)
    p = softmax(x)
    counts = np.bincount([orc.sample(x, 1.0, (i + 0.5) / 20000) for i in range(20000)], minlength=50)
    assert np.abs(counts / 20000 - p).max() <= 1.5 / 20000
    # invalid input
    assert orc.sample(x, 0.0, 0.5) == -1 and orc.sample(np.array([0.0, np.nan]), 1.0, 0.5) == -1


def test_oracle_under_address_and_undefined_behaviour_sanitizers():
    """Every entry point of orc.c driven on tiny, exactly-sized models (grouped-query, both weight formats, both rotary
    styles, no layers, refusals) in a build with AddressSanitizer, LeakSanitizer and UndefinedBehaviorSanitizer: any access
    out of bounds, leak on an error path or undefined arithmetic aborts the run."""
    import subprocess
    from oracle import build as orc_build
    exe = orc_build.build_sanitize_check()
    r = subprocess.run([exe], capture_output=True, text=True, timeout=120,
                       env={**os.environ, "ASAN_OPTIONS": "detect_leaks=1:abort_on_error=0", "OMP_NUM_THREADS": "4"})
    assert r.returncode == 0, r.stdout + r.stderr
    assert "orc sanitize check: ok" in r.stdout
