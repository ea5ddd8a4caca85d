"""Helpers shared by the GPU parity tests (no arithmetic of the method)."""
import numpy as np
import torch

DEV = "cuda:0"
BF16_EPS = 2.0 ** -7      # bf16 spacing relative to the value (8 significant bits); rounding error <= half of it
F16_EPS = 2.0 ** -10      # IEEE half spacing relative to the value (11 significant bits)


def randn_bf16(shape, seed, std=1.0, device=DEV):
    g = torch.Generator(device="cpu").manual_seed(seed)
    return (torch.randn(shape, generator=g) * std).to(torch.bfloat16).to(device)


def randn_f16(shape, seed, std=1.0, device=DEV):
    g = torch.Generator(device="cpu").manual_seed(seed)
    return (torch.randn(shape, generator=g) * std).to(torch.float16).to(device)


def randn_f32(shape, seed, std=1.0, device=DEV):
    g = torch.Generator(device="cpu").manual_seed(seed)
    return (torch.randn(shape, generator=g) * std).to(device)


def np64(t):
    return t.detach().to("cpu").to(torch.float64).numpy()


def bits(t):
    """bf16 tensor -> uint16 numpy bit patterns (what the oracle borrows)"""
    return t.detach().cpu().contiguous().view(torch.int16).numpy().view(np.uint16)


_PROGRESS = None


def step(msg):
    """Progress line of a long test: printed, and appended to a log file in the output folder under the repository root, so that
    a runner that watches that folder sees the test is alive even when pytest captures the output."""
    global _PROGRESS
    print(msg, flush=True)
    try:
        if _PROGRESS is None:
            import os
            root = os.environ.get("GRAFT_REPO_ROOT") or os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
            d = os.path.join(root, "gpurun_out")
            os.makedirs(d, exist_ok=True)
            _PROGRESS = os.path.join(d, "test_progress.log")
        with open(_PROGRESS, "a") as f:
            f.write(msg + "\n")
    except OSError:
        pass
