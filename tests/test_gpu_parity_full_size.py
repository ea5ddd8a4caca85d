"""GPU parity at the sizes the benchmark workloads run at: full depth, full width, the workload's batch on the GPU, and the
oracle recomputing sampled sequences one by one (sequences are independent) fed with the GPU's own tokens, so both sides
see identical inputs at every step.

Gate (the stated target): per-step logits max-abs error <= 3e-2 and >= 99 % greedy-token agreement, near ties counted as
misses; every miss must be a near tie in the oracle's own logits (gap <= 2 x the step's error); the GPU's tokens must be
the lowest argmax of its own logits (index work is exact).
"""
import numpy as np
import pytest
import torch

from oracle import orc
from tests.gpu_util import DEV, np64, step
from workload import PRESETS, make_prompts, make_weights

pytestmark = pytest.mark.gpu
LOGIT_TOL = 3e-2


def lowest_argmax(lg):
    return (lg == lg.max(-1, keepdim=True).values).int().argmax(-1)   # first index of the maximum


class Tally:
    """Running comparison of GPU logits / tokens with the oracle's."""

    def __init__(self, label):
        self.label, self.worst, self.sq, self.n, self.agree, self.total = label, 0.0, 0.0, 0, 0, 0
        self.block = [0.0, 0.0, 0, 0, 0]

    def add(self, i, g_logits, g_tokens, o_logits, o_next):
        gl, gn = np64(g_logits), g_tokens.cpu().numpy()
        assert np.isfinite(gl).all()
        d = gl - o_logits
        err = float(np.abs(d).max())
        assert err <= LOGIT_TOL, (self.label, i, err)
        assert np.array_equal(gn, np.array([orc.argmax(r) for r in gl]))
        for b in np.nonzero(gn != o_next)[0]:
            assert o_logits[b, o_next[b]] - o_logits[b, gn[b]] <= 2.0 * err, (self.label, i, b)
        hit = int((gn == o_next).sum())
        self.worst = max(self.worst, err)
        self.sq += float((d * d).sum()); self.n += d.size
        self.agree += hit; self.total += len(gn)
        blk = self.block
        blk[0] = max(blk[0], err); blk[1] += float((d * d).sum()); blk[2] += d.size; blk[3] += hit; blk[4] += len(gn)
        return gn

    def flush(self, upto):
        blk = self.block
        if blk[2]:
            step(f"  {self.label} steps to {upto}: worst {blk[0]:.3e}, rms {np.sqrt(blk[1] / blk[2]):.3e}, agreement {blk[3]}/{blk[4]}")
        self.block = [0.0, 0.0, 0, 0, 0]

    def finish(self, need_rate=True):
        rms = np.sqrt(self.sq / max(self.n, 1))
        step(f"  {self.label}: worst {self.worst:.3e}, rms {rms:.3e}, greedy agreement {self.agree}/{self.total} "
             f"({100.0 * self.agree / max(self.total, 1):.2f} %)")
        if need_rate:
            assert self.agree >= 0.99 * self.total
        return self.worst, rms


def generate_on_gpu(gen, prompts, G, sample, keep_steps=None):
    """Free-running greedy generation of the whole batch (tokens fed back on the device, as bench.py runs it); keeps the
    logits and tokens of the sampled sequences (at the steps in keep_steps, default all) and checks whole-batch properties."""
    B = prompts.shape[0]
    bufs = [torch.empty((B,), dtype=torch.int32, device=DEV) for _ in range(2)]
    lg = gen.prefill(prompts, next_tokens=bufs[0])[0]
    assert torch.isfinite(lg).all() and torch.equal(bufs[0].long(), lowest_argmax(lg))
    logits, tokens = {0: lg[sample].clone()}, [bufs[0][sample].clone()]
    cur = 0
    for i in range(1, G):
        lg, _ = gen.decode_step(bufs[cur], next_tokens=bufs[1 - cur])
        cur = 1 - cur
        tokens.append(bufs[cur][sample].clone())
        if keep_steps is None or i in keep_steps:
            logits[i] = lg[sample].clone()
        if i % 64 == 0 or i == G - 1:        # whole-batch properties that hold at any size
            assert torch.isfinite(lg).all() and torch.equal(bufs[cur].long(), lowest_argmax(lg))
    torch.cuda.synchronize()
    return logits, tokens


def test_benchmark_workload_full_size_sampled():
    """The benchmark configuration itself (LLaMA-7B shape, all 32 layers, batch 128, prompt 128, 256 generated tokens,
    packed weights, HIP-graph decode): the GPU runs the whole batch exactly as bench.py does; the oracle recomputes eight
    sampled sequences over all 256 steps: 2048 greedy decisions, 65 M logits."""
    from paper_2406_14088_amd import Generator
    wl = PRESETS["llama7b"]
    shape, B, P, G = wl.shape, wl.batch, wl.prompt_len, wl.gen_len
    sample = [5, 21, 40, 63, 77, 90, 104, 127]
    step("7B full depth: drawing weights on the GPU")
    W = make_weights(shape, wl.index, device=DEV)
    prompts = make_prompts(wl, device=DEV)
    gen = Generator(shape, W, B, wl.max_seq)
    g_logits, g_tokens = generate_on_gpu(gen, prompts, G, sample)
    assert gen.state() == (B, P + G - 1)
    gen.close()
    step("copying weights to the host for the oracle")
    Wn = orc.weights_to_numpy(W)
    del W
    om = orc.OracleModel(shape, Wn, len(sample), P + G)
    step("oracle prefill of the sampled sequences")
    o_logits, o_next = om.prefill(prompts[sample].cpu().numpy())
    tally = Tally("7B, 32 layers, batch 128")
    for i in range(G):
        gn = tally.add(i, g_logits[i], g_tokens[i], o_logits, o_next)
        if i % 32 == 31:
            tally.flush(i)
        if i < G - 1:
            o_logits, o_next = om.decode_step(gn)      # the oracle is fed the GPU's tokens
    om.close()
    tally.finish()


def test_13b_workload_full_depth_sampled():
    """LLaMA-13B shape at all 40 layers, batch 256, prompt 256 (the workload's own numbers) on the GPU; the oracle recomputes
    two sampled sequences through the prompt and the first decode steps."""
    from paper_2406_14088_amd import Generator
    wl = PRESETS["llama13b"]
    shape, B, P, G = wl.shape, wl.batch, wl.prompt_len, 8
    sample = [17, 201]
    step("13B full depth: drawing weights on the GPU")
    W = make_weights(shape, wl.index, device=DEV)
    prompts = make_prompts(wl, device=DEV)
    gen = Generator(shape, W, B, P + G)
    g_logits, g_tokens = generate_on_gpu(gen, prompts, G, sample)
    gen.close()
    step("copying weights to the host for the oracle")
    Wn = orc.weights_to_numpy(W)
    del W
    om = orc.OracleModel(shape, Wn, len(sample), P + G)
    pn = prompts[sample].cpu().numpy()
    step("oracle prefill of the sampled sequences (in spans of 64 positions)")
    om.prefill(pn[:, :64])
    for at in range(64, P - 64, 64):
        om.extend(pn[:, at: at + 64], want_logits=False)
    step("  oracle prompt done")
    o_logits = om.extend(pn[:, P - 64:])
    o_next = np.array([orc.argmax(r) for r in o_logits], dtype=np.int32)
    tally = Tally("13B, 40 layers, batch 256")
    for i in range(G):
        gn = tally.add(i, g_logits[i], g_tokens[i], o_logits, o_next)
        if i < G - 1:
            o_logits, o_next = om.decode_step(gn)
    om.close()
    tally.finish(need_rate=False)       # 16 decisions: the rate is gated where the sample is large enough


def test_long_context_workload_full_depth_prompt():
    """The long-context workload (LLaMA-7B shape, batch 32, prompt 2048) at all 32 layers: the oracle recomputes one
    sequence's 2048-position prompt and the decode steps at positions 2048 .. 2050."""
    from paper_2406_14088_amd import Generator
    wl = PRESETS["llama7b_long"]
    shape, B, P, G = wl.shape, wl.batch, wl.prompt_len, 4
    sample = [9]
    W = make_weights(shape, wl.index, device=DEV)
    prompts = make_prompts(wl, device=DEV)
    gen = Generator(shape, W, B, wl.max_seq)          # the cache at its full 4096-position capacity
    g_logits, g_tokens = generate_on_gpu(gen, prompts, G, sample)
    gen.close()
    Wn = orc.weights_to_numpy(W)
    del W
    om = orc.OracleModel(shape, Wn, 1, P + G)
    pn = prompts[sample].cpu().numpy()
    step("oracle: 2048-position prompt in spans of 128")
    om.prefill(pn[:, :128])
    for at in range(128, P - 128, 128):
        om.extend(pn[:, at: at + 128], want_logits=False)
        if at % 512 == 0:
            step(f"  oracle at position {at}")
    o_logits = om.extend(pn[:, P - 128:])
    o_next = np.array([orc.argmax(r) for r in o_logits], dtype=np.int32)
    tally = Tally("7B, 32 layers, prompt 2048")
    for i in range(G):
        gn = tally.add(i, g_logits[i], g_tokens[i], o_logits, o_next)
        if i < G - 1:
            o_logits, o_next = om.decode_step(gn)
    om.close()
    tally.finish(need_rate=False)


def test_long_context_workload_to_the_last_position():
    """The long-context workload's lengths (prompt 2048, generation to position 4094, batch 32, the cache at 4096 positions) at
    the 7B width and 4 of the 32 layers, so that the oracle can follow one sequence all the way: logits compared at the
    first decode step, around position 3000 and at the last positions."""
    from paper_2406_14088_amd import Generator
    wl = PRESETS["llama7b_long"]
    shape, B, P, G = wl.shape.with_layers(4), wl.batch, wl.prompt_len, wl.gen_len
    sample = [20]
    keep = {0, 1, 2, 952, 953, G - 3, G - 2, G - 1}       # step i decodes at position P + i - 1
    W = make_weights(shape, wl.index, device=DEV)
    prompts = make_prompts(wl, device=DEV)
    gen = Generator(shape, W, B, wl.max_seq)
    g_logits, g_tokens = generate_on_gpu(gen, prompts, G, sample, keep_steps=keep)
    assert gen.state() == (B, P + G - 1)
    gen.close()
    Wn = orc.weights_to_numpy(W)
    del W
    om = orc.OracleModel(shape, Wn, 1, P + G)
    seq = np.concatenate([prompts[sample].cpu().numpy(), torch.stack(g_tokens, 1).cpu().numpy()], axis=1)   # [1, P + G]
    tally = Tally("7B width, 4 layers, positions to 4094")
    at = 0
    for i in sorted(keep):          # logits of step i follow the token at position P + i - 1
        end = P + i
        while at < end:
            n = min(128, end - at)
            last = at + n == end
            o_logits = om.extend(seq[:, at: at + n], want_logits=last) if at else om.prefill(seq[:, :n])[0]
            at += n
            if at % 1024 == 0:
                step(f"  oracle at position {at}")
        o_next = np.array([orc.argmax(r) for r in o_logits], dtype=np.int32)
        tally.add(i, g_logits[i], g_tokens[i], o_logits, o_next)
    om.close()
    tally.finish(need_rate=False)


def test_70b_workload_full_depth_sampled():
    """LLaMA-70B shape (64 query / 8 kv heads, hidden 8192) at all 80 layers, the workload's batch of 64 on the GPU with a
    short prompt; the oracle recomputes two sequences."""
    from paper_2406_14088_amd import Generator
    wl = PRESETS["llama70b"]
    shape, B, P, G = wl.shape, wl.batch, 24, 4
    sample = [3, 50]
    torch.cuda.empty_cache()
    free, _ = torch.cuda.mem_get_info()
    if free < 200 * 2 ** 30:
        pytest.skip("needs 200 GB of free device memory")
    step("70B full depth: drawing weights on the GPU")
    W = make_weights(shape, wl.index, device=DEV)
    prompts = make_prompts(wl, prompt_len=P, device=DEV)
    gen = Generator(shape, W, B, P + G)
    g_logits, g_tokens = generate_on_gpu(gen, prompts, G, sample)
    gen.close()
    step("copying weights to the host for the oracle, tensor by tensor")
    Wn = {}
    for k in list(W.keys()):       # 138 GB: keep the runner informed while it moves
        Wn.update(orc.weights_to_numpy({k: W.pop(k)}))
        step(f"  {k} on the host")
    del W
    torch.cuda.empty_cache()
    om = orc.OracleModel(shape, Wn, len(sample), P + G)
    step("oracle prefill of the sampled sequences")
    o_logits, o_next = om.prefill(prompts[sample].cpu().numpy())
    tally = Tally("70B, 80 layers, batch 64")
    for i in range(G):
        gn = tally.add(i, g_logits[i], g_tokens[i], o_logits, o_next)
        if i < G - 1:
            o_logits, o_next = om.decode_step(gn)
            step(f"  oracle decode step {i + 1}")
    om.close()
    tally.finish(need_rate=False)
