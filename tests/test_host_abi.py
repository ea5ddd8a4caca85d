"""Host-only checks of the C-ABI library: it loads, exports every declared symbol, and its host logic
(shape validation, closed forms, argument errors) behaves as include/rl_gen.h states.  No GPU compute."""
import ctypes as C
import os
import re

import pytest

from workload import LLAMA3_TABLE_SHAPES, PRESETS

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def binding():
    from paper_2406_14088_amd import binding as b
    b.lib()
    return b


def declared_symbols():
    names = set()
    for hdr in ("rl_gen.h", "rl_gen_ops.h"):
        text = open(os.path.join(ROOT, "include", hdr)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names |= set(re.findall(r"\b(rl_(?:gen|op)_[a-z0-9_]+)\s*\(", text))
    return names


def test_every_declared_symbol_is_exported_and_bound(binding):
    L = binding.lib()
    decl = declared_symbols()
    assert decl == set(binding.EXPORTED_SYMBOLS)
    for name in decl:
        assert getattr(L, name) is not None


def test_param_count_matches_paper_table_and_presets(binding):
    rows = [l.split() for l in open(os.path.join(ROOT, "tests", "golden", "llama3_param_counts.txt"))
            if l.strip() and not l.startswith("#")]
    for name, *_cfg, total, _ in rows:
        assert binding.param_count(LLAMA3_TABLE_SHAPES[name]) == int(total)
    # benchmark shapes: counted tensor by tensor
    for wl in PRESETS.values():
        s = wl.shape
        qd, kvd, d = s.n_heads * s.head_dim, s.n_kv_heads * s.head_dim, s.hidden
        per_layer = qd * d + 2 * kvd * d + d * qd + 3 * d * s.ffn + 2 * d
        assert binding.param_count(s) == 2 * s.vocab * d + s.n_layers * per_layer + d


def test_kv_bytes_closed_form(binding):
    s = PRESETS["llama7b"].shape
    # 16-bit elements: 0.5 MiB per token and sequence; level 1 keeps IEEE half rows
    assert binding.kv_bytes(s, 1, 1, precision=1) == 524288
    assert binding.kv_bytes(s, 128, 384, precision=1) == 524288 * 128 * 384
    # block-scaled rows (the default level of this shape): one fp32 scale per (layer, K|V, kv head) row of 128 elements
    assert binding.precision_level(s) == 2 and binding.kv_block_scaled(s)
    assert binding.kv_bytes(s, 1, 1) == 524288 + 2 * 32 * 32 * 4
    assert binding.kv_bytes(s, 128, 384) == (524288 + 2 * 32 * 32 * 4) * 128 * 384
    s70 = PRESETS["llama70b"].shape
    assert binding.precision_level(s70) == 3 and binding.kv_block_scaled(s70)
    assert binding.kv_bytes(s70, 64, 384) == 2 * 80 * 8 * (128 * 2 + 4) * 64 * 384
    assert binding.kv_bytes(s70, 64, 384, precision=2) == 2 * 80 * 8 * 128 * 2 * 64 * 384   # grouped-query shape: half rows at level 2
    assert not binding.kv_block_scaled(s70, precision=2) and not binding.kv_block_scaled(s, precision=1)
    assert binding.precision_level(s, precision=3) == 3
    assert binding.validate_shape(binding.RlGenShape.from_model(s, 1, 1, precision=4)) == -2
    assert binding.work_bytes(s, 128, 384) > 0


def test_shape_validation(binding):
    from dataclasses import replace
    s = PRESETS["tiny"].shape
    assert binding.validate_shape(s, 4, 32) == 0
    assert binding.validate_shape(replace(s, n_kv_heads=3), 4, 32) == -2      # heads not divisible
    assert binding.validate_shape(replace(s, head_dim=32), 4, 32) == -2       # hidden != heads * head_dim
    assert binding.validate_shape(replace(s, ffn=690), 4, 32) == -2           # ffn % 8
    assert binding.validate_shape(replace(s, rope_style=2), 4, 32) == -2
    assert binding.validate_shape(s, 0, 32) == -2
    assert binding.kv_bytes(replace(s, n_kv_heads=3), 4, 32) == 0


def test_null_arguments_are_rejected_without_a_gpu(binding):
    L = binding.lib()
    cs = binding.RlGenShape.from_model(PRESETS["tiny"].shape, 4, 32)
    out = C.c_void_p()
    assert L.rl_gen_create(C.byref(cs), None, None, 0, None, 0, C.byref(out)) == -1
    assert L.rl_gen_prefill(None, None, 1, 1, None, None, None) == -1
    assert L.rl_gen_decode_step(None, None, None, None, None) == -1
    assert L.rl_gen_reset(None) == -1
    L.rl_gen_destroy(None)
    assert L.rl_op_argmax(None, 1, 1, None, None) == -1
    assert L.rl_op_gemm(None, None, 8, None, None, None, 1, 0, 0, 1, 8, None, 1, 0, 1, 0, 0, None, None) == -1
    assert L.rl_gen_kernel_class_name(4) == b"decode_attention"
    assert len(binding.KERNEL_CLASSES) == 13


def test_page_bytes_and_page_planning_on_the_host(binding):
    s = PRESETS["llama7b"].shape
    assert binding.page_bytes(s, 16, precision=1) == 16 * 524288    # a page of 16 positions: 16 x the per-token bytes
    assert binding.page_bytes(s, 64) * 6 == binding.kv_bytes(s, 1, 384)
    assert binding.page_bytes(s, 16) == 16 * binding.kv_bytes(s, 1, 1)
    for bad in (0, 8, 24, 100, 8192, -16):
        assert binding.page_bytes(s, bad) == 0
    # consecutive pages, ceil(capacity / page) per sequence, -1 in the unused entries
    used, table = binding.plan_pages([33, 0, 16, 1], 16, 10, 4)
    assert used == 5
    assert table == [[0, 1, 2, -1], [-1, -1, -1, -1], [3, -1, -1, -1], [4, -1, -1, -1]]
    assert binding.plan_pages([], 16, 0, 4) == (0, [])
    from paper_2406_14088_amd import RlGenError
    for cap, n_pages, pps, code in (([33, 16], 3, 4, -3),           # the pool is one page short
                                    ([65], 10, 4, -3),              # more pages than a row of the table holds
                                    ([-1], 10, 4, -2)):
        with pytest.raises(RlGenError) as e:
            binding.plan_pages(cap, 16, n_pages, pps)
        assert e.value.code == code
    L = binding.lib()
    assert L.rl_gen_plan_pages(None, 1, 16, 1, 1, None) == -1
    assert L.rl_gen_set_block_table(None, None, None, 1, 1, None) == -1
    assert L.rl_gen_pool_pages(None) == -1
    cs = binding.RlGenShape.from_model(PRESETS["tiny"].shape, 4, 32)
    out = C.c_void_p()
    assert L.rl_gen_create_paged(C.byref(cs), None, None, 0, None, 0, 16, C.byref(out)) == -1


def test_host_logic_under_address_and_undefined_behaviour_sanitizers():
    """The host side of the C ABI (validation, arena sizing up to byte counts that need 64 bits, page planning into
    exactly-sized tables, argument checks of the entry points) in a build with AddressSanitizer and
    UndefinedBehaviorSanitizer on the host code; nothing in it needs a GPU."""
    import os
    import subprocess
    from paper_2406_14088_amd import build as lib_build
    exe = lib_build.build_host_sanitize_check()
    r = subprocess.run([exe], capture_output=True, text=True, timeout=120,
                       env={**os.environ, "ASAN_OPTIONS": "detect_leaks=0"})   # the HIP runtime's own start-up allocations are not ours
    assert r.returncode == 0, r.stdout + r.stderr
    assert "host sanitize check: ok" in r.stdout
