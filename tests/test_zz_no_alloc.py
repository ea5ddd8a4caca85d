"""The entry point that allocates nothing (rl_op_decode_attention_noalloc: split partials in the library's built-in scratch
array) against rl_op_decode_attention on the same inputs, through the C ABI: two calls in a row, the second with a smaller
input, IEEE-half and block-scaled cache rows, and the size limit."""
import numpy as np
import pytest
import torch

from tests.gpu_util import DEV, randn_f16, randn_f32

pytestmark = pytest.mark.gpu


def _case(ops, B, Hq, Hkv, hd, S, length, nsplit, seed, block_scaled):
    q = randn_f32((B, Hq * hd), seed, std=1.5)
    if block_scaled:
        g = torch.Generator(device="cpu").manual_seed(seed + 1)
        kc = torch.randint(-32767, 32768, (B, Hkv, S, hd), generator=g, dtype=torch.int32).to(torch.int16).to(DEV)
        vc = torch.randint(-32767, 32768, (B, Hkv, S, hd), generator=g, dtype=torch.int32).to(torch.int16).to(DEV)
        ks = ((torch.rand((B, Hkv, S), generator=g) + 0.5) / 32767.0).to(DEV)
        vs = ((torch.rand((B, Hkv, S), generator=g) + 0.5) / 32767.0).to(DEV)
    else:
        kc, vc, ks, vs = randn_f16((B, Hkv, S, hd), seed + 1), randn_f16((B, Hkv, S, hd), seed + 2), None, None
    d_len = torch.tensor([length], dtype=torch.int32, device=DEV)
    want = torch.zeros((B, Hq * hd), dtype=torch.float16, device=DEV)
    want_lo = torch.zeros_like(want)
    ws = torch.empty(max(ops.decode_attention_ws_floats(B, Hq, hd, nsplit), 1), dtype=torch.float32, device=DEV)
    ops.decode_attention(q, kc, vc, d_len, want, ws, B, Hq, Hkv, hd, S, nsplit, kscale=ks, vscale=vs, out_lo=want_lo)
    got = torch.zeros_like(want)
    got_lo = torch.zeros_like(want)
    ops.decode_attention_noalloc(q, kc, vc, d_len, got, B, Hq, Hkv, hd, S, nsplit, kscale=ks, vscale=vs, out_lo=got_lo)
    torch.cuda.synchronize()
    assert want.abs().max() > 0
    # same kernels on the same inputs: the two entry points agree to the bit (the stated tolerance is met with room to spare)
    assert torch.equal(got.view(torch.int16), want.view(torch.int16))
    assert torch.equal(got_lo.view(torch.int16), want_lo.view(torch.int16))


@pytest.mark.parametrize("block_scaled", [False, True])
def test_no_alloc_entry_point_two_calls_in_a_row(block_scaled):
    from paper_2406_14088_amd import ops
    _case(ops, 8, 16, 4, 128, 640, 500, 4, 900, block_scaled)     # partials of 8 x 16 x 4 splits
    _case(ops, 3, 4, 4, 64, 160, 100, 2, 910, block_scaled)       # a smaller call reuses the front of the same scratch
    _case(ops, 5, 8, 8, 128, 64, 40, 1, 920, block_scaled)        # no split: the scratch is not touched


def test_no_alloc_entry_point_rejects_what_does_not_fit():
    from paper_2406_14088_amd import lib, ops
    B, Hq, hd, nsplit = 4096, 64, 128, 16                          # 4096 x 64 x 16 x 130 floats = 2.2 GB of partials
    assert ops.decode_attention_ws_floats(B, Hq, hd, nsplit) * 4 > (16 << 20)
    x = torch.zeros(16, dtype=torch.float32, device=DEV)
    rc = lib().rl_op_decode_attention_noalloc(x.data_ptr(), x.data_ptr(), x.data_ptr(), x.data_ptr(), 0, x.data_ptr(), B, Hq, 8, hd, 16,
                                              nsplit, None, None, None, None, None)
    assert rc == -3
    assert b"scratch" in lib().rl_gen_last_error(None)
    assert lib().rl_op_decode_attention_noalloc(None, None, None, None, 0, None, 1, 1, 1, 64, 1, 1, None, None, None, None, None) == -1
