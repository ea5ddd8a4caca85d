"""Seeded weight and prompt generators (inputs only; none of the method's arithmetic).

Every tensor is drawn from its own generator seeded by (workload index, layer,
tensor slot), so a reduced-depth model is exactly a prefix of the full one and a
tensor's values do not depend on which other tensors were generated.

Recipe: embedding and all projection matrices ~ N(0, 0.02^2); RMSNorm gains are
1.0 (gain_std > 0: every gain vector drawn as 1 + gain_std * N(0, 1) instead).  Values are rounded once (round-to-nearest-even, torch's conversion) to
bf16 so that the CPU oracle and the GPU path consume identical weights; the
oracle widens them, the GPU path uses them as they are.
"""
from __future__ import annotations

from typing import Dict, List

import torch

from .configs import ModelShape, Workload

LAYER_TENSORS = ("attn_norm", "wq", "wk", "wv", "wo", "ffn_norm", "w_gate", "w_up", "w_down")
WEIGHT_ORDER = ("tok_emb",) + LAYER_TENSORS + ("final_norm", "lm_head")
_SLOT = {name: i for i, name in enumerate(WEIGHT_ORDER)}


def _tensor_shape(s: ModelShape, name: str):
    qd, kvd = s.n_heads * s.head_dim, s.n_kv_heads * s.head_dim
    return {
        "tok_emb": (s.vocab, s.hidden), "lm_head": (s.vocab, s.hidden),
        "attn_norm": (s.hidden,), "ffn_norm": (s.hidden,), "final_norm": (s.hidden,),
        "wq": (qd, s.hidden), "wk": (kvd, s.hidden), "wv": (kvd, s.hidden), "wo": (s.hidden, qd),
        "w_gate": (s.ffn, s.hidden), "w_up": (s.ffn, s.hidden), "w_down": (s.hidden, s.ffn),
    }[name]


def _draw(seed_index: int, layer: int, name: str, shape, device, dtype, std: float, gain_std: float = 0.0):
    g = torch.Generator(device=device)
    g.manual_seed((1000 + seed_index) * 1_000_003 + (layer + 1) * 101 + _SLOT[name])
    if name.endswith("norm"):
        if gain_std == 0.0:
            return torch.ones(shape, dtype=dtype, device=device)
        # distinct gains per norm (tests of which gain reaches which norm): 1 + gain_std * N(0, 1), rounded to bf16
        t = 1.0 + gain_std * torch.randn(shape, generator=g, device=device, dtype=torch.float32)
        return t.to(torch.bfloat16).to(dtype)
    t = torch.randn(shape, generator=g, device=device, dtype=torch.float32) * std
    return t.to(torch.bfloat16).to(dtype)


def make_weights(shape: ModelShape, seed_index: int, device="cpu", dtype=torch.bfloat16,
                 std: float = 0.02, gain_std: float = 0.0) -> Dict[str, object]:
    """Returns {"tok_emb": T, "final_norm": T, "lm_head": T, <layer tensor>: [T]*L}.

    All values are exactly representable in bf16 whatever `dtype` is.  The CPU
    and GPU generators of torch produce different streams: draw once on one
    device and copy, never draw the "same" weights twice on different devices.
    """
    out: Dict[str, object] = {}
    for name in ("tok_emb", "final_norm", "lm_head"):
        out[name] = _draw(seed_index, -1, name, _tensor_shape(shape, name), device, dtype, std, gain_std)
    for name in LAYER_TENSORS:
        lst: List[torch.Tensor] = []
        for layer in range(shape.n_layers):
            lst.append(_draw(seed_index, layer, name, _tensor_shape(shape, name), device, dtype, std, gain_std))
        out[name] = lst
    return out


def make_prompts(w: Workload, batch: int | None = None, prompt_len: int | None = None,
                 device="cpu") -> torch.Tensor:
    """Uniform random token ids, int32 [batch, prompt_len], seeded by the workload index."""
    b = w.batch if batch is None else batch
    p = w.prompt_len if prompt_len is None else prompt_len
    g = torch.Generator(device="cpu")
    g.manual_seed(2000 + w.index)
    full = torch.randint(0, w.shape.vocab, (max(b, w.batch), max(p, w.prompt_len)), generator=g,
                         dtype=torch.int32)
    return full[:b, :p].contiguous().to(device)
