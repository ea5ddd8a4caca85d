"""End-to-end GPU parity: rl_gen_prefill / rl_gen_decode_step (C ABI) against the CPU oracle on the same
seeded weights and prompts, under teacher forcing (the GPU is fed the oracle's greedy tokens).

Gate (the stated target): per-step logits max-abs error <= 3e-2 and >= 99 % greedy-token agreement.
Greedy tokens are additionally required to be a valid argmax of the GPU's own logits (bit-exact index work).
Where a floating-point value decides the token, two answers are defensible when the oracle's own logits of the
two candidates are closer than twice the measured logit error: every disagreement must be such a near tie.
The 99 % gate is applied strictly (near ties count as misses) to every case with at least 200 compared tokens
and to the union of all cases of this module (test_zz_overall_agreement).
"""
import numpy as np
import pytest
import torch

from oracle import orc
from tests.gpu_util import DEV, np64, step
from workload import PRESETS, ModelShape, Workload, make_prompts, make_weights

pytestmark = pytest.mark.gpu
LOGIT_TOL = 3e-2
TOTALS = {"agree": 0, "total": 0}


def run_teacher_forced(shape, seed_index, B, P, G, graph=True, max_batch=None, max_seq=None, std=0.02, packed=True, gain_std=0.0,
                       precision=0):
    from paper_2406_14088_amd import Generator
    wl = Workload("t", seed_index, shape, B, P, G)
    W = make_weights(shape, seed_index, device="cpu", std=std, gain_std=gain_std)
    Wg = {k: ([t.to(DEV) for t in v] if isinstance(v, list) else v.to(DEV)) for k, v in W.items()}
    prompts = make_prompts(wl)
    om = orc.OracleModel(shape, orc.weights_to_numpy(W), B, P + G)
    gen = Generator(shape, Wg, max_batch or B, max_seq or (P + G), packed=packed, precision=precision)
    gen.set_graph(graph)
    o_logits, o_next = om.prefill(prompts.numpy())
    g_logits, g_next = gen.prefill(prompts.to(DEV))
    torch.cuda.synchronize()
    errs, agree, total = [], 0, 0

    def compare(gl, gn, ol, on):
        nonlocal agree, total
        gl64 = np64(gl)
        assert np.isfinite(gl64).all()
        errs.append(np.abs(gl64 - ol).max())
        gn = gn.cpu().numpy()
        # index work is exact: the returned token is the lowest argmax of the GPU's own fp32 logits
        assert np.array_equal(gn, np.array([orc.argmax(r) for r in gl64]))
        agree += int((gn == on).sum())
        total += len(on)
        for b in np.nonzero(gn != on)[0]:       # a disagreement must be a near tie in the oracle's own logits
            assert ol[b, on[b]] - ol[b, gn[b]] <= 2.0 * errs[-1], (b, on[b], gn[b], ol[b, on[b]] - ol[b, gn[b]], errs[-1])

    compare(g_logits, g_next, o_logits, o_next)
    tok = o_next
    for i in range(G - 1):
        o_logits, o_next = om.decode_step(tok)
        g_logits, g_next = gen.decode_step(torch.from_numpy(tok).to(DEV))
        torch.cuda.synchronize()
        compare(g_logits, g_next, o_logits, o_next)
        tok = o_next
    assert gen.state() == (B, P + G - 1)
    gen.close()
    TOTALS["agree"] += agree
    TOTALS["total"] += total
    return max(errs), agree / total, errs, total


def check(shape, seed_index, B, P, G, **kw):
    worst, agreement, errs, total = run_teacher_forced(shape, seed_index, B, P, G, **kw)
    step(f"  max-abs logit error {worst:.3e}, greedy agreement {agreement:.4f} over {len(errs)} steps / {total} tokens")
    assert worst <= LOGIT_TOL
    if total >= 200:
        assert agreement >= 0.99
    return worst, agreement


@pytest.mark.parametrize("packed", [True, False])
@pytest.mark.parametrize("graph", [True, False])
def test_tiny_config_full_workload(graph, packed):
    wl = PRESETS["tiny"]
    step(f"tiny preset: B={wl.batch} P={wl.prompt_len} G={wl.gen_len} graph={graph} packed={packed}")
    check(wl.shape, wl.index, wl.batch, wl.prompt_len, wl.gen_len, graph=graph, packed=packed)


def test_tiny_interleaved_rope_and_spare_capacity():
    from dataclasses import replace
    wl = PRESETS["tiny"]
    check(replace(wl.shape, rope_style=0), 11, 3, 9, 5, max_batch=5, max_seq=40)


@pytest.mark.parametrize("packed", [True, False])
@pytest.mark.parametrize("shape", [ModelShape(4, 512, 4, 4, 128, 1384, 2048), ModelShape(3, 512, 8, 2, 64, 1000, 2048)])
def test_distinct_random_gains_reach_their_own_norms(shape, packed):
    """Every RMSNorm gain vector drawn as 1 + 0.3 N(0, 1) (attention norm and FFN norm of each layer, final norm): with
    unit gains any two of them could be swapped unnoticed; with these, a gain reaching the wrong norm moves the logits far
    beyond the tolerance (a swapped pair changes them by ~0.3 relative)."""
    worst, _ = check(shape, 16, 5, 40, 6, packed=packed, gain_std=0.3)
    # the test has teeth: the oracle itself, fed weights with two gain vectors exchanged, is far from the product
    from paper_2406_14088_amd import Generator
    W = make_weights(shape, 16, device="cpu", gain_std=0.3)
    Ws = dict(W)
    Ws["ffn_norm"] = list(W["ffn_norm"])
    Ws["attn_norm"] = list(W["attn_norm"])
    Ws["ffn_norm"][1], Ws["attn_norm"][2] = W["attn_norm"][2], W["ffn_norm"][1]
    prompts = make_prompts(Workload("t", 16, shape, 5, 40, 6))
    wrong, _ = orc.OracleModel(shape, orc.weights_to_numpy(Ws), 5, 46).prefill(prompts.numpy())
    gen = Generator(shape, {k: ([t.to(DEV) for t in v] if isinstance(v, list) else v.to(DEV)) for k, v in W.items()}, 5, 46, packed=packed)
    g_logits, _ = gen.prefill(prompts.to(DEV))
    torch.cuda.synchronize()
    gen.close()
    assert np.abs(np64(g_logits) - wrong).max() > 10 * LOGIT_TOL


@pytest.mark.parametrize("precision", [1, 2, 3])
@pytest.mark.parametrize("shape", [ModelShape(3, 512, 4, 4, 128, 1384, 2048), ModelShape(3, 1024, 8, 1, 128, 1000, 2048)])
def test_precision_levels(shape, precision):
    """Each level of rl_gen_shape.precision on a multi-head and a grouped-query shape, packed and row-major decode paths,
    more than 128 rows per step included (all within the tolerance; the levels differ in how far inside)."""
    step(f"precision {precision}, Hq/Hkv {shape.n_heads}/{shape.n_kv_heads}")
    check(shape, 17, 6, 33, 5, precision=precision)
    check(shape, 17, 6, 33, 5, precision=precision, packed=False)
    check(shape, 17, 130, 5, 3, precision=precision)


def test_gqa_small_model():
    s = ModelShape(3, 512, 8, 2, 64, 1000, 2048)
    check(s, 12, 5, 21, 6)


def test_gate_up_copies_for_some_layers_only():
    """An arena with room for the gate/up copies of two of three layers: those layers run the fused projection from
    the copies, the third from the row-major weights; the model as a whole stays within the oracle's tolerance."""
    from paper_2406_14088_amd import Generator
    s = ModelShape(3, 512, 8, 2, 64, 1000, 2048)
    W = make_weights(s, 12, device=DEV)
    for want, arg in ((2, 2), (3, True), (0, False)):
        gen = Generator(s, W, 5, 32, pack_gate_up=arg)
        assert gen.packed_gate_up_layers() == want
        gen.close()
    import paper_2406_14088_amd.binding as binding
    orig = binding.Generator.__init__

    def two_layers(self, *a, **kw):
        kw["pack_gate_up"] = 2
        orig(self, *a, **kw)
    binding.Generator.__init__ = two_layers
    try:
        check(s, 12, 130, 4, 4)        # more than 128 rows per decode step: the copies are used where they exist
    finally:
        binding.Generator.__init__ = orig


def test_batch_256_and_above_uses_wide_tiles():
    s = ModelShape(1, 256, 4, 4, 64, 688, 1024)
    check(s, 13, 256, 3, 3)
    check(s, 13, 256, 3, 3, packed=False)
    check(s, 14, 300, 2, 3)     # more than 256 rows per decode step: the tiled projection path


def test_long_sequences_split_attention():
    # long prompt (several attention tiles, ragged tail) and sequence-split decode attention
    s = ModelShape(2, 256, 2, 1, 128, 512, 1024)
    check(s, 15, 2, 333, 4, max_seq=2048)


@pytest.mark.parametrize("packed", [True, False])
def test_width_of_7b_reduced_depth(packed):
    s = PRESETS["llama7b"].shape.with_layers(2)
    step(f"7B width (hidden 4096, 32 heads, FFN 11008, vocab 32000), 2 layers, packed={packed}")
    check(s, 2, 4, 32, 4, packed=packed)


def test_width_of_13b_reduced_depth():
    s = PRESETS["llama13b"].shape.with_layers(1)
    step("13B width (hidden 5120, 40 heads, FFN 13824), 1 layer")
    check(s, 3, 2, 24, 3)


def test_width_of_70b_gqa_reduced_depth():
    s = PRESETS["llama70b"].shape.with_layers(1)
    step("70B width (hidden 8192, 64/8 heads, FFN 28672), 1 layer")
    check(s, 5, 2, 16, 3)


def test_width_of_the_papers_llama3_7b_row_reduced_depth():
    """The paper's own model-configuration table, 7B row: grouped-query attention 32/8, FFN 14336, vocabulary 128256
    (LM head of 1.05 GB, argmax over 128256 logits; 128256 = 2^8 * 3 * 167 exercises the tile tails)."""
    from workload.configs import LLAMA3_TABLE_SHAPES
    s = LLAMA3_TABLE_SHAPES["7B"].with_layers(1)
    step("LLaMA-3 7B row width (hidden 4096, 32/8 heads, FFN 14336, vocab 128256), 1 layer")
    check(s, 6, 3, 20, 3)


def test_width_of_the_papers_llama3_34b_row_reduced_depth():
    """34B row of the same table: hidden 8192, 64/8 heads, FFN 22016 (= 2^9 * 43), vocabulary 128256."""
    from workload.configs import LLAMA3_TABLE_SHAPES
    s = LLAMA3_TABLE_SHAPES["34B"].with_layers(1)
    step("LLaMA-3 34B row width (hidden 8192, 64/8 heads, FFN 22016, vocab 128256), 1 layer")
    check(s, 7, 2, 12, 3)


@pytest.mark.parametrize("case", ["tiny", "7b_width", "chunked_head", "tiny_level3", "7b_width_level3_row_major"])
def test_inference_call_logprobs(case):
    """rl_gen_logprobs: one forward pass over whole sequences, log-probability of every following token.
    |d logp| <= |d logit_target| + |d logsumexp| <= 2 * LOGIT_TOL (the logits themselves are within LOGIT_TOL)."""
    from paper_2406_14088_amd import Generator
    kw = {}
    if case.startswith("tiny"):
        shape, idx, B, T = PRESETS["tiny"].shape, 1, 5, 90       # 450 rows: the large-M projection kernel serves the LM head
        if case == "tiny_level3":                                # the LM head takes the final norm's low term as well
            kw = {"precision": 3}
    elif case == "7b_width_level3_row_major":                    # 72 rows and no fragment-order copies: tile kernel, two terms
        shape, idx, B, T, kw = PRESETS["llama7b"].shape.with_layers(2), 2, 3, 24, {"precision": 3, "packed": False}
    elif case == "7b_width":
        shape, idx, B, T = PRESETS["llama7b"].shape.with_layers(2), 2, 3, 24
    else:   # more rows than one block of the LM head holds (vocabulary large against the workspace)
        shape, idx, B, T = ModelShape(1, 256, 4, 4, 64, 688, 50000), 21, 6, 100
    step(f"inference call {case}: B={B} T={T} vocab={shape.vocab}")
    wl = Workload("t", idx, shape, B, T, 0)
    W = make_weights(shape, idx, device="cpu")
    Wg = {k: ([t.to(DEV) for t in v] if isinstance(v, list) else v.to(DEV)) for k, v in W.items()}
    toks = make_prompts(wl)
    om = orc.OracleModel(shape, orc.weights_to_numpy(W), B, T)
    want = orc.sequence_logprobs(om.forward_all(toks.numpy()), toks.numpy())
    om.close()
    gen = Generator(shape, Wg, B, T + 1, **kw)
    got = gen.logprobs(toks.to(DEV))
    torch.cuda.synchronize()
    gn = np64(got)
    assert gn.shape == (B, T) and (gn[:, T - 1] == 0).all()
    err = np.abs(gn[:, : T - 1] - want).max()
    step(f"  max-abs log-prob error {err:.3e}")
    assert err <= 2 * LOGIT_TOL
    # the call leaves the cache as a prefill of the same tokens would: a decode step may follow
    assert gen.state() == (B, T)
    ref = Generator(shape, Wg, B, T + 1, **kw)
    ref.prefill(toks.to(DEV))
    nxt = torch.zeros((B,), dtype=torch.int32, device=DEV)
    a, _ = gen.decode_step(nxt)
    b, _ = ref.decode_step(nxt)
    torch.cuda.synchronize()
    assert torch.equal(a, b)
    gen.close()
    ref.close()


@pytest.mark.parametrize("precision", [0, 3])
@pytest.mark.parametrize("fp32_weights", [False, True])
def test_inference_call_scalar_head(fp32_weights, precision):
    """rl_gen_values: the Critic/Reward form of the inference call.  A scalar head w gives, at every position, what the LM
    head would give for a vocabulary row equal to w: the oracle runs the same decoder with w as row 0 of its LM head."""
    from paper_2406_14088_amd import Generator
    shape, idx, B, T = ModelShape(2, 256, 4, 2, 64, 688, 300), 23, 5, 70
    wl = Workload("t", idx, shape, B, T, 0)
    W = make_weights(shape, idx, device="cpu", dtype=torch.float32 if fp32_weights else torch.bfloat16)
    head = W["lm_head"][0].clone()
    Wg = {k: ([t.to(DEV) for t in v] if isinstance(v, list) else v.to(DEV)) for k, v in W.items()}
    toks = make_prompts(wl)
    om = orc.OracleModel(shape, orc.weights_to_numpy(W, as_bf16_bits=not fp32_weights), B, T)
    want = om.forward_all(toks.numpy())[:, :, 0]
    om.close()
    gen = Generator(shape, Wg, B, T, precision=precision)
    got = np64(gen.values(toks.to(DEV), head.to(DEV)))
    torch.cuda.synchronize()
    err = np.abs(got - want).max()
    step(f"  scalar head, level {precision}: max-abs error {err:.3e}")
    assert got.shape == (B, T) and err <= LOGIT_TOL and gen.state() == (B, T)
    gen.close()


def test_prefill_equals_incremental_decode_on_device():
    """Causality/caching invariant on the GPU itself: prefill(P) and prefill(P-k) + k decode steps give the
    same last-position logits up to the bf16 path's own rounding differences."""
    from paper_2406_14088_amd import Generator
    s = ModelShape(2, 512, 8, 4, 64, 1000, 2048)
    W = make_weights(s, 16, device=DEV)
    wl = Workload("t", 16, s, 3, 40, 1)
    prompts = make_prompts(wl, device=DEV)
    gen = Generator(s, W, 3, 48)
    full, _ = gen.prefill(prompts)
    full = full.clone()
    _, _ = gen.prefill(prompts[:, :33].contiguous())
    lg = None
    for i in range(33, 40):
        lg, _ = gen.decode_step(prompts[:, i].contiguous())
    torch.cuda.synchronize()
    assert (full - lg).abs().max().item() <= 2e-2
    gen.close()


def test_free_running_generation_is_deterministic_and_graph_invariant():
    from paper_2406_14088_amd import Generator
    wl = PRESETS["tiny"]
    W = make_weights(wl.shape, wl.index, device=DEV)
    prompts = make_prompts(wl, device=DEV)
    runs = []
    for graph in (False, True, True):
        gen = Generator(wl.shape, W, wl.batch, wl.max_seq)
        gen.set_graph(graph)
        _, a = gen.prefill(prompts)
        b = torch.empty_like(a)
        toks, logs = [a.clone()], []
        for i in range(wl.gen_len - 1):
            lg, _ = gen.decode_step(a, next_tokens=b)   # ping-pong buffers, as the benchmark does
            torch.cuda.synchronize()
            toks.append(b.clone())
            logs.append(lg.clone())
            a, b = b, a
        runs.append((torch.stack(toks), torch.stack(logs)))
        gen.close()
    for t, l in runs[1:]:
        assert torch.equal(t, runs[0][0]) and torch.equal(l, runs[0][1])


def test_repacking_follows_a_weight_update():
    """The fragment-order copies are a snapshot: after the weight tensors change in place (a training step between two
    generation phases) pack_weights() must be called, and then the step computes with the new weights."""
    from paper_2406_14088_amd import Generator
    wl = PRESETS["tiny"]
    W = make_weights(wl.shape, wl.index, device=DEV)
    W2 = make_weights(wl.shape, wl.index + 40, device=DEV)
    prompts = make_prompts(wl, device=DEV)
    ref = Generator(wl.shape, W2, wl.batch, wl.max_seq, packed=False)
    want, _ = ref.prefill(prompts)
    gen = Generator(wl.shape, W, wl.batch, wl.max_seq)
    before, _ = gen.prefill(prompts)
    for k, v in W.items():                      # in-place update of every borrowed tensor
        for dst, src in zip(v if isinstance(v, list) else [v], W2[k] if isinstance(v, list) else [W2[k]]):
            dst.copy_(src)
    gen.pack_weights()
    after, _ = gen.prefill(prompts)
    torch.cuda.synchronize()
    assert (before - want).abs().max() > 1e-2          # the two weight sets really differ
    assert (after - want).abs().max() <= 1e-3          # same weights, packed vs row-major: fp32 summation order only
    with pytest.raises(Exception):
        lib_small = torch.empty(256, dtype=torch.uint8, device=DEV)
        gen._check(__import__("paper_2406_14088_amd").binding.lib().rl_gen_pack_weights(gen._h, lib_small.data_ptr(), 256, None), "pack")
    ref.close()
    gen.close()


def test_degenerate_models_and_inputs():
    """No layers (logits = LM head of the normalised embedding), a one-token prompt, a batch of one, capacity filled to the
    last position, and token ids outside the vocabulary (clamped on the device: no fault)."""
    from paper_2406_14088_amd import Generator
    from dataclasses import replace
    wl = PRESETS["tiny"]
    check(wl.shape.with_layers(0), 31, 2, 3, 3)        # L = 0
    check(wl.shape, 32, 1, 1, 4)                       # B = 1, P = 1
    check(replace(wl.shape, vocab=97, ffn=72), 33, 3, 5, 3)   # sizes that are no multiple of any tile
    W = make_weights(wl.shape, wl.index, device=DEV)
    gen = Generator(wl.shape, W, 2, 5)
    bad = torch.tensor([[5, -3, 2000000, 7], [1, 2, 3, 4]], dtype=torch.int32, device=DEV)
    clamped = torch.tensor([[5, 0, wl.shape.vocab - 1, 7], [1, 2, 3, 4]], dtype=torch.int32, device=DEV)
    a, _ = gen.prefill(bad)
    b, _ = gen.prefill(clamped)
    lg, _ = gen.decode_step(torch.tensor([-1, 3], dtype=torch.int32, device=DEV))      # fills the cache to max_seq
    torch.cuda.synchronize()
    assert torch.equal(a, b) and torch.isfinite(lg).all() and gen.state() == (2, 5)
    gen.close()


def test_graph_cache_eviction_and_internal_logit_buffer():
    """More distinct (token, next) buffer pairs than the library keeps captured graphs for, and decode steps that keep the
    logits in the library's own workspace: tokens must equal those of a plain eager run."""
    from paper_2406_14088_amd import Generator
    wl = PRESETS["tiny"]
    W = make_weights(wl.shape, wl.index, device=DEV)
    prompts = make_prompts(wl, device=DEV)
    ref = Generator(wl.shape, W, wl.batch, wl.max_seq)
    ref.set_graph(False)
    _, t = ref.prefill(prompts)
    want = [t.clone()]
    for _ in range(wl.gen_len - 1):
        _, t = ref.decode_step(want[-1])
        want.append(t.clone())
    ref.close()
    gen = Generator(wl.shape, W, wl.batch, wl.max_seq)
    bufs = [torch.empty((wl.batch,), dtype=torch.int32, device=DEV) for _ in range(11)]   # 11 buffers: 11 distinct pairs in a ring
    gen.prefill(prompts, next_tokens=bufs[0])
    got = [bufs[0].clone()]
    for i in range(wl.gen_len - 1):
        a, b = bufs[i % 11], bufs[(i + 1) % 11]
        gen.decode_step(a, next_tokens=b, want_logits=False)
        got.append(b.clone())
    torch.cuda.synchronize()
    for g, w_ in zip(got, want):
        assert torch.equal(g, w_)
    gen.close()


@pytest.mark.parametrize("graph", [False, True])
def test_sampled_generation(graph):
    """Generation with temperature sampling: the library draws nothing, the caller refreshes the uniform draws between steps.
    Every returned token must be a valid inversion of the step's own logits (which the other tests tie to the oracle), both for
    prefill and for (graph-replayed) decode steps; switching back gives the greedy tokens again."""
    from paper_2406_14088_amd import Generator
    wl = PRESETS["tiny"]
    W = make_weights(wl.shape, wl.index, device=DEV)
    prompts = make_prompts(wl, device=DEV)
    B, temperature, delta = wl.batch, 0.9, 3e-5
    gen = Generator(wl.shape, W, B, wl.max_seq)
    gen.set_graph(graph)
    u = torch.zeros((B,), dtype=torch.float32, device=DEV)
    gen.set_sampling(temperature, u)
    rng = torch.Generator(device="cpu").manual_seed(7)

    def valid(logits, tokens, draws):
        for b in range(B):
            x = np64(logits[b])
            e = np.exp((x - x.max()) / temperature)
            c = np.concatenate([[0.0], np.cumsum(e) / e.sum()])
            v = int(tokens[b])
            assert c[v] - delta <= float(draws[b]) <= c[v + 1] + delta

    draws = torch.rand((B,), generator=rng)
    u.copy_(draws)
    lg, tok = gen.prefill(prompts)
    torch.cuda.synchronize()
    valid(lg, tok.cpu(), draws)
    seen_non_greedy = not torch.equal(tok.cpu(), lg.argmax(-1).int().cpu())
    nxt = torch.empty_like(tok)
    for i in range(8):
        draws = torch.rand((B,), generator=rng)
        u.copy_(draws)
        lg, _ = gen.decode_step(tok, next_tokens=nxt)
        torch.cuda.synchronize()
        valid(lg, nxt.cpu(), draws)
        seen_non_greedy |= not torch.equal(nxt.cpu(), lg.argmax(-1).int().cpu())
        tok, nxt = nxt, tok
    assert seen_non_greedy                       # the draws really steer the tokens
    gen.set_sampling(0.0)
    lg, t2 = gen.decode_step(tok)
    torch.cuda.synchronize()
    assert torch.equal(t2.cpu().long(), (lg == lg.max(-1, keepdim=True).values).int().argmax(-1).cpu())
    gen.close()


def test_per_kernel_timing_counts_every_launch():
    """rl_gen_profile: while on, every kernel launch of prefill and decode is bracketed by events on the caller's stream; the
    counts per kernel class follow from the model depth, and results are the same as without timing."""
    from paper_2406_14088_amd import Generator
    wl = PRESETS["tiny"]
    L = wl.shape.n_layers
    W = make_weights(wl.shape, wl.index, device=DEV)
    prompts = make_prompts(wl, device=DEV)
    gen = Generator(wl.shape, W, wl.batch, wl.max_seq)
    lg0, t0 = gen.prefill(prompts)
    lg1, _ = gen.decode_step(t0)
    ref = (lg0.clone(), lg1.clone())
    gen.profile(True)
    gen.profile_read()
    lg0, t0 = gen.prefill(prompts)
    lg1, _ = gen.decode_step(t0)
    prof = gen.profile_read()
    gen.profile(False)
    torch.cuda.synchronize()
    assert torch.equal(lg0, ref[0]) and torch.equal(lg1, ref[1])
    n = {k: v["launches"] for k, v in prof.items()}
    assert n["embed"] == 2 and n["add_rmsnorm"] == 2 * (2 * L + 1) and n["gemm_qkv"] == 2 * L and n["rope_append"] == 2 * L
    assert n["decode_attention"] == L and n["prefill_attention"] == L and n["gemm_o"] == 2 * L and n["gemm_gate_up"] == 2 * L
    assert n["gemm_down"] == 2 * L and n["gemm_lm_head"] == 2 and n["argmax"] == 2
    assert all(v["ms"] > 0 for k, v in prof.items() if v["launches"])
    again = gen.profile_read()                      # reading clears the sums
    assert all(v["launches"] == 0 for v in again.values())
    gen.close()


@pytest.mark.parametrize("precision,packed", [(0, True), (3, True), (3, False)])
def test_ragged_prompts_against_the_oracle(precision, packed):
    """Prompts of different lengths in one batch: every sequence must behave exactly as if it were alone (the oracle runs
    them one by one at their own lengths), through prefill and teacher-forced decode steps at per-sequence positions."""
    from paper_2406_14088_amd import Generator
    shape = ModelShape(2, 256, 4, 2, 64, 688, 1000)
    B, T, steps = 5, 40, 4
    lens = [40, 1, 17, 33, 8]
    W = make_weights(shape, 41, device="cpu")
    Wg = {k: ([t.to(DEV) for t in v] if isinstance(v, list) else v.to(DEV)) for k, v in W.items()}
    toks = make_prompts(Workload("t", 41, shape, B, T, 0))
    gen = Generator(shape, Wg, B, T + steps, precision=precision, packed=packed)
    g_logits, g_next = gen.prefill_ragged(toks.to(DEV), torch.tensor(lens, dtype=torch.int32, device=DEV))
    torch.cuda.synchronize()
    assert gen.read_state() == (lens, [0] * B)
    Wn = orc.weights_to_numpy(W)
    oms = []
    worst = 0.0
    feed = np.zeros((B,), np.int32)
    for b in range(B):
        om = orc.OracleModel(shape, Wn, 1, T + steps)
        ol, on = om.prefill(toks[b: b + 1, : lens[b]].numpy())
        worst = max(worst, np.abs(np64(g_logits[b]) - ol[0]).max())
        feed[b] = on[0]
        oms.append(om)
    for i in range(steps):
        g_logits, g_next = gen.decode_step(torch.from_numpy(feed).to(DEV))
        torch.cuda.synchronize()
        for b in range(B):
            ol, on = oms[b].decode_step(feed[b: b + 1])
            worst = max(worst, np.abs(np64(g_logits[b]) - ol[0]).max())
            feed[b] = on[0]
        assert gen.read_state()[0] == [n + i + 1 for n in lens]
    for om in oms:
        om.close()
    step(f"  ragged batch, level {precision}, packed={packed}: max-abs logit error {worst:.3e}")
    assert worst <= LOGIT_TOL
    gen.close()


def _shuffled_pages(capacity, page, n_pages, seed):
    """Page lists that scatter every sequence over the pool (no two runs of positions adjacent on purpose)."""
    need = [(c + page - 1) // page for c in capacity]
    perm = [int(v) for v in np.random.default_rng(seed).permutation(n_pages)]
    rows, at = [], 0
    for n in need:
        rows.append(perm[at: at + n])
        at += n
    width = max(max(need), 1)
    return [r + [-1] * (width - len(r)) for r in rows]


@pytest.mark.parametrize("graph", [False, True])
@pytest.mark.parametrize("page", [16, 64])
def test_paged_cache_equals_contiguous_cache(graph, page):
    """Ragged prompts over a paged cache whose pool holds just what the sequences need, pages scattered: logits and
    tokens equal those of the contiguous cache bit for bit (which the ragged test ties to the oracle), and one
    sequence is also checked against the oracle directly."""
    from paper_2406_14088_amd import Generator
    shape = ModelShape(2, 256, 4, 2, 64, 688, 1000)
    B, T, steps = 5, 40, 6
    lens = [40, 1, 17, 33, 8]
    capacity = [n + steps for n in lens]
    W = make_weights(shape, 43, device="cpu")
    Wg = {k: ([t.to(DEV) for t in v] if isinstance(v, list) else v.to(DEV)) for k, v in W.items()}
    toks = make_prompts(Workload("t", 43, shape, B, T, 0)).to(DEV)
    d_lens = torch.tensor(lens, dtype=torch.int32, device=DEV)
    n_pages = sum((c + page - 1) // page for c in capacity)

    def run(gen):
        gen.set_graph(graph)
        out = []
        lg, nx = gen.prefill_ragged(toks, d_lens)
        out.append((lg.clone(), nx.clone()))
        for _ in range(steps):
            lg, nx = gen.decode_step(out[-1][1])
            out.append((lg.clone(), nx.clone()))
        torch.cuda.synchronize()
        return out

    flat = Generator(shape, Wg, B, T + steps)
    want = run(flat)
    flat_bytes = flat.kv_arena.numel()
    flat.close()
    paged = Generator(shape, Wg, B, T + steps, page_size=page, n_pages=n_pages)
    assert paged.pool_pages() == n_pages
    if page == 16:
        assert paged.kv_arena.numel() < flat_bytes                 # the point of paging: memory follows the real lengths
    paged.set_block_table(_shuffled_pages(capacity, page, n_pages, 44), capacity)
    got = run(paged)
    assert paged.read_state() == ([n + steps for n in lens], [0] * B)
    for i, ((lw, nw), (lg, ng)) in enumerate(zip(want, got)):
        assert torch.equal(lg.view(torch.int32), lw.view(torch.int32)), i
        assert torch.equal(ng, nw), i
    # sequence 2 alone on the oracle, fed the tokens the batch produced
    b = 2
    om = orc.OracleModel(shape, orc.weights_to_numpy(W), 1, T + steps)
    ol, _ = om.prefill(toks[b: b + 1, : lens[b]].cpu().numpy())
    worst = np.abs(np64(got[0][0][b]) - ol[0]).max()
    for i in range(steps):
        ol, _ = om.decode_step(got[i][1][b: b + 1].cpu().numpy())
        worst = max(worst, np.abs(np64(got[i + 1][0][b]) - ol[0]).max())
    om.close()
    assert worst <= LOGIT_TOL
    paged.close()
    # the inference call over a paged cache: every sequence needs T positions for it
    cap_T = [T] * B
    pages_T = sum((c + page - 1) // page for c in cap_T)
    paged = Generator(shape, Wg, B, T + steps, page_size=page, n_pages=pages_T + 2)
    paged.set_block_table(_shuffled_pages(cap_T, page, pages_T + 2, 45), cap_T)
    lp = paged.logprobs(toks)
    flat = Generator(shape, Wg, B, T + steps)
    lp_want = flat.logprobs(toks)
    torch.cuda.synchronize()
    assert torch.equal(lp.view(torch.int32), lp_want.view(torch.int32))
    flat.close()
    paged.close()


def test_paged_ragged_prefill_through_the_fused_projection_and_grouped_query_attention():
    """A model wide enough for the kernels the small paged tests do not reach: head_dim 128 with 4 query heads per kv head
    (matrix-core decode attention through page lists) and a prefill of 2880 rows (QKV projection that rotates and appends
    in its epilogue, honouring page lists and per-sequence lengths).  Paged equals contiguous bit for bit; two sequences
    are checked against the oracle run alone."""
    from paper_2406_14088_amd import Generator
    shape = ModelShape(1, 4096, 32, 8, 128, 1024, 1000)
    B, T, steps, page = 30, 96, 3, 32
    rng = np.random.default_rng(51)
    lens = [int(v) for v in rng.integers(1, T + 1, size=B)]
    lens[0], lens[1] = T, 33
    capacity = [n + steps for n in lens]
    W = make_weights(shape, 51, device="cpu")
    Wg = {k: ([t.to(DEV) for t in v] if isinstance(v, list) else v.to(DEV)) for k, v in W.items()}
    toks = make_prompts(Workload("t", 51, shape, B, T, 0)).to(DEV)
    d_lens = torch.tensor(lens, dtype=torch.int32, device=DEV)
    n_pages = sum((c + page - 1) // page for c in capacity)

    def run(gen):
        out = []
        lg, nx = gen.prefill_ragged(toks, d_lens)
        out.append((lg.clone(), nx.clone()))
        for _ in range(steps):
            lg, nx = gen.decode_step(out[-1][1])
            out.append((lg.clone(), nx.clone()))
        torch.cuda.synchronize()
        return out

    flat = Generator(shape, Wg, B, T + steps)
    want = run(flat)
    flat.close()
    paged = Generator(shape, Wg, B, T + steps, page_size=page, n_pages=n_pages)
    paged.set_block_table(_shuffled_pages(capacity, page, n_pages, 52), capacity)
    got = run(paged)
    paged.close()
    for i, ((lw, nw), (lg, ng)) in enumerate(zip(want, got)):
        assert torch.equal(lg.view(torch.int32), lw.view(torch.int32)), i
        assert torch.equal(ng, nw), i
    Wn = orc.weights_to_numpy(W)
    worst = 0.0
    for b in (1, 7):
        om = orc.OracleModel(shape, Wn, 1, T + steps)
        ol, _ = om.prefill(toks[b: b + 1, : lens[b]].cpu().numpy())
        worst = max(worst, np.abs(np64(got[0][0][b]) - ol[0]).max())
        for i in range(steps):
            ol, _ = om.decode_step(got[i][1][b: b + 1].cpu().numpy())
            worst = max(worst, np.abs(np64(got[i + 1][0][b]) - ol[0]).max())
        om.close()
    step(f"  fused projection + paged grouped-query attention: max-abs logit error {worst:.3e}")
    assert worst <= LOGIT_TOL


def test_paged_cache_capacity_is_checked_on_the_host():
    """Nothing is launched that would store a row outside a sequence's pages: the calls fail with E_CAPACITY / E_STATE."""
    from paper_2406_14088_amd import Generator, RlGenError
    wl = PRESETS["tiny"]
    W = make_weights(wl.shape, wl.index, device=DEV)
    prompts = make_prompts(wl, device=DEV)
    B, P, page = wl.batch, wl.prompt_len, 16
    gen = Generator(wl.shape, W, B, wl.max_seq, page_size=page, n_pages=2 * B)
    with pytest.raises(RlGenError) as e:               # no page lists yet
        gen.prefill(prompts)
    assert e.value.code == -4
    rows = [[2 * b, 2 * b + 1] for b in range(B)]
    for bad, code in (([[0, 1]] + [[0, 3]] + rows[2:], -2),          # page 0 named twice
                      ([[0, 2 * B]] + rows[1:], -3),                # outside the pool
                      ([[0, -1]] + rows[1:], -3)):
        with pytest.raises(RlGenError) as e:
            gen.set_block_table(bad, [2 * page] * B)
        assert e.value.code == code
    with pytest.raises(RlGenError) as e:               # more positions than the rows of the table can name
        gen.set_block_table(rows, [2 * page + 1] * B)
    assert e.value.code in (-2, -3)
    gen.set_block_table(rows, [P - 1] + [2 * page] * (B - 1))
    with pytest.raises(RlGenError) as e:               # sequence 0 cannot hold its prompt
        gen.prefill(prompts)
    assert e.value.code == -3
    cap = [P + 2] + [2 * page] * (B - 1)
    gen.set_block_table(rows, cap)
    _, t = gen.prefill(prompts)
    _, t = gen.decode_step(t)
    _, t = gen.decode_step(t)
    with pytest.raises(RlGenError) as e:               # a third appended row would not fit sequence 0
        gen.decode_step(t)
    assert e.value.code == -3
    assert gen.read_state()[0] == [P + 2] * B
    gen.set_block_table(rows, [2 * page] * B)           # more room for sequence 0 in the page it already has: goes on
    gen.decode_step(t)
    torch.cuda.synchronize()
    assert gen.read_state()[0] == [P + 3] * B
    gen.close()


def test_paged_cache_ended_sequence_stops_counting():
    """Once the host has read the end flags, an ended sequence no longer needs room, and it stores nothing more: the
    other sequences produce what they produce without an end token."""
    from paper_2406_14088_amd import Generator, RlGenError
    wl = PRESETS["tiny"]
    W = make_weights(wl.shape, wl.index, device=DEV)
    prompts = make_prompts(wl, device=DEV)
    B, P, G, page = wl.batch, wl.prompt_len, wl.gen_len, 16
    flat = Generator(wl.shape, W, B, wl.max_seq)
    _, t = flat.prefill(prompts)
    free = [t.clone()]
    for _ in range(G - 1):
        free.append(flat.decode_step(free[-1])[1].clone())
    torch.cuda.synchronize()
    flat.close()
    eos = int(free[1][0])                               # sequence 0 ends with the token of its first decode step
    rows = [[2 * b + 1, 2 * b] for b in range(B)]
    gen = Generator(wl.shape, W, B, wl.max_seq, page_size=page, n_pages=2 * B)
    cap = [P + 1] + [2 * page] * (B - 1)               # sequence 0 has room for exactly the one row it stores before ending
    gen.set_block_table(rows, cap)
    gen.set_eos(eos)
    _, t = gen.prefill(prompts)
    if int(t[0]) == eos:
        pytest.skip("the first token already is the end token")
    _, t = gen.decode_step(t)                           # stores row P of sequence 0 and returns eos for it
    with pytest.raises(RlGenError):                     # the host does not know yet that sequence 0 has ended
        gen.decode_step(t)
    lens, done = gen.read_state()
    assert done[0] == 1 and lens[0] == P + 1
    out = [None, t.clone()]
    for _ in range(G - 2):
        out.append(gen.decode_step(out[-1])[1].clone())
    torch.cuda.synchronize()
    for k in range(1, G):
        assert int(out[k][0]) == eos
        for b in range(1, B):
            if not any(int(free[j][b]) == eos for j in range(k + 1)):
                assert int(out[k][b]) == int(free[k][b]), (k, b)
    gen.close()


@pytest.mark.parametrize("sampling", [False, True])
def test_generate_call_runs_the_batch_in_portions(sampling):
    """rl_gen_generate on a generator smaller than the batch: portions of max_batch sequences, each prefilled and decoded
    to the end before the next.  Equal, token for token, to the step calls run portion by portion; and every greedy token
    is a best token of the oracle's own logits (teacher-forced on what the GPU generated) within the logit tolerance."""
    from paper_2406_14088_amd import Generator
    shape = ModelShape(2, 256, 4, 2, 64, 688, 1000)
    B, P, G, portion = 10, 12, 8, 4
    W = make_weights(shape, 47, device="cpu")
    Wg = {k: ([t.to(DEV) for t in v] if isinstance(v, list) else v.to(DEV)) for k, v in W.items()}
    prompts = make_prompts(Workload("t", 47, shape, B, P, 0)).to(DEV)
    gen = Generator(shape, Wg, portion, P + G - 1)
    u = None
    if sampling:
        u = torch.rand((G, B), generator=torch.Generator().manual_seed(48)).to(DEV)
        ubuf = torch.zeros((portion,), dtype=torch.float32, device=DEV)
        gen.set_sampling(0.9, ubuf)
    out = gen.generate(prompts, G, u)
    again = gen.generate(prompts, G, u)                     # second call: the decode steps are replayed from the captured graph
    torch.cuda.synchronize()
    assert out.shape == (B, G) and torch.equal(out, again)
    for b0 in range(0, B, portion):
        nb = min(portion, B - b0)
        if sampling:
            ubuf[:nb] = u[0, b0: b0 + nb]
        _, t = gen.prefill(prompts[b0: b0 + nb].contiguous())
        assert torch.equal(t, out[b0: b0 + nb, 0])
        for g in range(1, G):
            if sampling:
                ubuf[:nb] = u[g, b0: b0 + nb]
            _, t = gen.decode_step(t)
            assert torch.equal(t, out[b0: b0 + nb, g]), (b0, g)
    gen.close()
    if sampling:
        return                                              # the sampled choice itself is tied to the oracle by the step-call tests
    om = orc.OracleModel(shape, orc.weights_to_numpy(W), B, P + G)
    toks = out.cpu().numpy()
    ol, _ = om.prefill(prompts.cpu().numpy())
    for g in range(G):
        for b in range(B):
            assert ol[b, toks[b, g]] >= ol[b].max() - 2 * LOGIT_TOL, (b, g)
        if g + 1 < G:
            ol, _ = om.decode_step(toks[:, g].copy())
    om.close()


def test_generate_call_argument_errors():
    from paper_2406_14088_amd import Generator, RlGenError
    wl = PRESETS["tiny"]
    W = make_weights(wl.shape, wl.index, device=DEV)
    prompts = make_prompts(wl, device=DEV)
    gen = Generator(wl.shape, W, 2, wl.prompt_len + 3)
    with pytest.raises(RlGenError) as e:                    # prompt + 5 generated tokens store 4 rows too many... one too many
        gen.generate(prompts, 5)
    assert e.value.code == -3
    gen.set_sampling(1.0, torch.zeros((2,), dtype=torch.float32, device=DEV))
    with pytest.raises(RlGenError) as e:                    # sampling without draws
        gen.generate(prompts, 2)
    assert e.value.code == -1
    gen.set_sampling(0.0)
    out = gen.generate(prompts, 4)                          # exactly fills the cache
    torch.cuda.synchronize()
    assert out.shape == (wl.batch, 4) and int(out.min()) >= 0
    gen.close()


@pytest.mark.parametrize("graph", [False, True])
def test_end_token_stops_a_sequence(graph):
    """With an end token set, a sequence that produces it keeps returning it, stops growing and leaves the others alone."""
    from paper_2406_14088_amd import Generator
    wl = PRESETS["tiny"]
    W = make_weights(wl.shape, wl.index, device=DEV)
    prompts = make_prompts(wl, device=DEV)
    B, G = wl.batch, wl.gen_len

    def run(eos):
        gen = Generator(wl.shape, W, B, wl.max_seq)
        gen.set_graph(graph)
        gen.set_eos(eos)
        _, t = gen.prefill(prompts)
        out = [t.clone()]
        for _ in range(G - 1):
            _, t2 = gen.decode_step(out[-1])
            out.append(t2.clone())
        torch.cuda.synchronize()
        state = gen.read_state()
        gen.close()
        return torch.stack(out).cpu().numpy(), state          # [G, B]

    free, (lens_free, done_free) = run(-1)
    assert done_free == [0] * B and lens_free == [wl.prompt_len + G - 1] * B
    b_stop, k_stop = 1, 5
    eos = int(free[k_stop, b_stop])                           # the token sequence 1 produces at step 5 becomes the end token
    got, (lens, done) = run(eos)
    for b in range(B):
        hits = np.nonzero(free[:, b] == eos)[0]
        if len(hits) == 0:
            assert (got[:, b] == free[:, b]).all() and done[b] == 0 and lens[b] == wl.prompt_len + G - 1
        else:
            k = int(hits[0])                                   # first time the free run of this sequence emits the end token
            assert (got[: k + 1, b] == free[: k + 1, b]).all() and (got[k:, b] == eos).all() and done[b] == 1
            assert lens[b] == wl.prompt_len + k                # the prompt plus the k tokens fed back before it ended
    assert done[b_stop] == 1


@pytest.mark.parametrize("graph", [False, True])
@pytest.mark.parametrize("cache", ["contiguous", "paged"])
def test_batch_compaction_after_the_end_token(cache, graph):
    """rl_gen_compact: ended sequences leave the batch, the others move up (cache rows of a contiguous cache, page lists of
    a paged one), later steps run on fewer rows -- and every sequence still produces exactly the tokens of the uncompacted
    run, each of them the argmax of logits that are the oracle's (teacher-forced on those tokens) within the tolerance."""
    from paper_2406_14088_amd import Generator, RlGenError
    shape = ModelShape(2, 256, 4, 2, 64, 688, 48)                 # a small vocabulary: the end token comes up often
    B, P, G, page = 14, 9, 20, 16
    W = make_weights(shape, 61, device="cpu", std=0.05)
    Wg = {k: ([t.to(DEV) for t in v] if isinstance(v, list) else v.to(DEV)) for k, v in W.items()}
    prompts = make_prompts(Workload("t", 61, shape, B, P, G)).to(DEV)

    def make():
        if cache == "paged":
            cap = [P + G] * B
            n_pages = sum((c + page - 1) // page for c in cap)
            gen = Generator(shape, Wg, B, P + G, page_size=page, n_pages=n_pages)
            gen.set_block_table(_shuffled_pages(cap, page, n_pages, 62), cap)
        else:
            gen = Generator(shape, Wg, B, P + G)
        gen.set_graph(graph)
        return gen

    # the free run picks the end token: what most sequences emit somewhere, at different steps
    gen = make()
    _, t = gen.prefill(prompts)
    free = [t.clone()]
    for _ in range(G - 1):
        free.append(gen.decode_step(free[-1])[1].clone())
    free = torch.stack(free).cpu().numpy()                         # [G, B]
    gen.close()
    first = {}
    for v in range(shape.vocab):
        hit = [int(np.nonzero(free[:, b] == v)[0][0]) if (free[:, b] == v).any() else -1 for b in range(B)]
        first[v] = hit
    eos = max(first, key=lambda v: (len({h for h in first[v] if h >= 0}), sum(h >= 0 for h in first[v])))
    ends = first[eos]
    assert sum(h >= 0 for h in ends) >= 4 and len({h for h in ends if h >= 0}) >= 3, ends
    step(f"  end token {eos}: sequences end after {ends} tokens (-1: never)")

    # uncompacted run with the end token
    gen = make()
    gen.set_eos(eos)
    _, t = gen.prefill(prompts)
    plain = [t.clone()]
    for _ in range(G - 1):
        plain.append(gen.decode_step(plain[-1])[1].clone())
    plain = torch.stack(plain).cpu().numpy()
    gen.close()

    # compacted run: compaction after every second step; rows[i] = original sequence of batch row i
    gen = make()
    gen.set_eos(eos)
    lg, t = gen.prefill(prompts)
    rows = list(range(B))
    tokens = {b: [] for b in range(B)}
    logits = {b: [] for b in range(B)}
    sizes = []
    for g in range(G):
        tn, ln = t.cpu().numpy(), np64(lg)
        for i, b in enumerate(rows):
            tokens[b].append(int(tn[i]))
            logits[b].append(ln[i])
        if g == G - 1 or not rows:
            break
        if g % 2 == 1:
            kept = gen.compact(t)
            rows = [rows[k] for k in kept]
            assert gen.state()[0] == len(rows)
            lens, done = gen.read_state()
            assert done == [0] * len(rows) and lens == [P + len(tokens[b]) - 1 for b in rows]
            t = t[: len(rows)].contiguous()
        sizes.append(len(rows))
        if not rows:
            with pytest.raises(RlGenError):
                gen.decode_step(torch.zeros((1,), dtype=torch.int32, device=DEV))
            break
        lg, t = gen.decode_step(t)
    torch.cuda.synchronize()
    gen.close()
    assert sizes[-1] < B, sizes                                    # the batch did shrink
    step(f"  batch sizes over the steps: {sizes}")

    worst = 0.0
    Wn = orc.weights_to_numpy(W)
    for b in range(B):
        n = len(tokens[b])
        assert tokens[b] == [int(v) for v in plain[:n, b]], b      # the same tokens as without compaction ...
        if n < G:
            assert tokens[b][-1] == eos or ends[b] < 0             # ... and a sequence only leaves once it has ended
            assert (plain[n:, b] == eos).all()
        om = orc.OracleModel(shape, Wn, 1, P + G)
        ol, _ = om.prefill(prompts[b: b + 1].cpu().numpy())
        n = tokens[b].index(eos) + 1 if eos in tokens[b] else n    # what an ended sequence returns afterwards is not compared
        for k in range(n):
            worst = max(worst, np.abs(logits[b][k] - ol[0]).max())
            assert tokens[b][k] == orc.argmax(logits[b][k])
            if k + 1 < n:
                ol, _ = om.decode_step(np.array([tokens[b][k]], np.int32))
        om.close()
    step(f"  max-abs logit error of the compacted run {worst:.3e}")
    assert worst <= LOGIT_TOL


def test_batch_compaction_when_nobody_or_everybody_has_ended():
    from paper_2406_14088_amd import Generator, RlGenError
    wl = PRESETS["tiny"]
    W = make_weights(wl.shape, wl.index, device=DEV)
    prompts = make_prompts(wl, device=DEV)[:1].contiguous()
    gen = Generator(wl.shape, W, 1, wl.max_seq)
    with pytest.raises(RlGenError):
        gen.compact()                                              # no sequences yet
    _, t = gen.prefill(prompts)
    assert gen.compact(t) == [0] and gen.state() == (1, wl.prompt_len)        # nobody has ended: nothing changes
    _, t2 = gen.decode_step(t)
    gen.set_eos(int(t2.item()))                                    # what the sequence is about to repeat ends it
    gen.reset()
    _, t = gen.prefill(prompts)
    _, t2 = gen.decode_step(t)
    assert gen.read_state() == ([wl.prompt_len + 1], [1])
    assert gen.compact(t2) == [] and gen.state() == (0, 0)         # everybody has ended: an empty generator
    with pytest.raises(RlGenError):
        gen.decode_step(t2)
    gen.set_eos(-1)
    _, t3 = gen.prefill(prompts)                                   # ... that takes a new batch
    assert torch.equal(t3, t)
    gen.close()


def test_error_paths_on_device():
    from paper_2406_14088_amd import Generator, RlGenError
    wl = PRESETS["tiny"]
    W = make_weights(wl.shape, wl.index, device=DEV)
    gen = Generator(wl.shape, W, 2, 6)
    tok = torch.zeros((2,), dtype=torch.int32, device=DEV)
    with pytest.raises(RlGenError) as e:
        gen.decode_step(tok)
    assert e.value.code == -4
    with pytest.raises(RlGenError) as e:
        gen.prefill(torch.zeros((3, 4), dtype=torch.int32, device=DEV))
    assert e.value.code == -3
    with pytest.raises(RlGenError) as e:
        gen.prefill(torch.zeros((2, 7), dtype=torch.int32, device=DEV))
    assert e.value.code == -3 and gen.state() == (0, 0)
    gen.prefill(torch.zeros((2, 6), dtype=torch.int32, device=DEV))
    with pytest.raises(RlGenError) as e:
        gen.decode_step(tok)
    assert e.value.code == -3 and gen.state() == (2, 6)
    gen.reset()
    assert gen.state() == (0, 0)
    gen.close()


def test_fp32_weights_are_converted_once():
    from paper_2406_14088_amd import Generator
    wl = PRESETS["tiny"]
    Wb = make_weights(wl.shape, wl.index, device=DEV)
    Wf = {k: ([t.float() for t in v] if isinstance(v, list) else v.float()) for k, v in Wb.items()}
    prompts = make_prompts(wl, device=DEV)
    a = Generator(wl.shape, Wb, wl.batch, wl.max_seq)
    b = Generator(wl.shape, Wf, wl.batch, wl.max_seq)
    la, na = a.prefill(prompts)
    lb, nb = b.prefill(prompts)
    torch.cuda.synchronize()
    assert torch.equal(la, lb) and torch.equal(na, nb)
    a.close(); b.close()


def test_zz_overall_agreement():
    """Strict greedy-token agreement over every teacher-forced token compared by the tests above."""
    if TOTALS["total"] < 1000:
        pytest.skip("needs the whole module to have run")
    rate = TOTALS["agree"] / TOTALS["total"]
    step(f"overall greedy agreement {rate:.4f} over {TOTALS['total']} tokens")
    assert rate >= 0.99
