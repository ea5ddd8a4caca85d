"""ctypes binding of librl_gen.so: same names as the C ABI, argument marshalling only.

torch is used for device memory (arenas, I/O tensors) and for the current stream; every step of the
generation path runs inside the library's HIP kernels.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, List, Optional

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "librl_gen.so")
_LIB = None

STATUS = {0: "OK", -1: "E_NULL", -2: "E_SHAPE", -3: "E_CAPACITY", -4: "E_STATE", -5: "E_HIP"}
KERNEL_CLASSES = ("embed", "add_rmsnorm", "gemm_qkv", "rope_append", "decode_attention", "attention_merge",
                  "prefill_attention", "gemm_o", "gemm_gate_up", "gemm_down", "gemm_lm_head", "argmax", "misc")
LAYER_NAMES = ("attn_norm", "wq", "wk", "wv", "wo", "ffn_norm", "w_gate", "w_up", "w_down")


class RlGenError(RuntimeError):
    def __init__(self, code: int, where: str, text: str = ""):
        super().__init__(f"{where}: {STATUS.get(code, code)} {text}".strip())
        self.code = code


class RlGenShape(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_layers", "hidden", "n_heads", "n_kv_heads", "head_dim", "ffn", "vocab")] + [
        ("rope_base", C.c_float), ("rms_eps", C.c_float), ("rope_style", C.c_int32), ("weight_dtype", C.c_int32),
        ("max_batch", C.c_int32), ("max_seq", C.c_int32), ("precision", C.c_int32)]

    @classmethod
    def from_model(cls, shape, max_batch: int, max_seq: int, weight_dtype: int = 1, precision: int = 0) -> "RlGenShape":
        return cls(shape.n_layers, shape.hidden, shape.n_heads, shape.n_kv_heads, shape.head_dim, shape.ffn, shape.vocab,
                   shape.rope_base, shape.rms_eps, shape.rope_style, weight_dtype, max_batch, max_seq, precision)


class RlGenWeights(C.Structure):
    _fields_ = [("tok_emb", C.c_void_p)] + [(n, C.POINTER(C.c_void_p)) for n in LAYER_NAMES] + [
        ("final_norm", C.c_void_p), ("lm_head", C.c_void_p)]


def lib():
    """Loads the built library; raises if it is missing (there is no fallback path)."""
    global _LIB
    if _LIB is not None:
        return _LIB
    # torch first: the library must bind to the same HIP runtime instance that owns the device memory
    # and streams it is handed (two runtimes in one process do not share allocations)
    import torch  # noqa: F401
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is not built: run `python -m paper_2406_14088_amd.build` "
                           "(or __graft_entry__.build()) first; this package has no fallback path")
    L = C.CDLL(LIB_PATH)
    vp, i32, i64, sz, f32 = C.c_void_p, C.c_int32, C.c_int64, C.c_size_t, C.c_float
    sp = C.POINTER(RlGenShape)
    sig = {
        "rl_gen_validate_shape": (C.c_int, [sp]),
        "rl_gen_param_count": (i64, [sp]),
        "rl_gen_kv_bytes": (sz, [sp]),
        "rl_gen_precision_level": (C.c_int, [sp]),
        "rl_gen_kv_block_scaled": (C.c_int, [sp]),
        "rl_gen_work_bytes": (sz, [sp]),
        "rl_gen_create": (C.c_int, [sp, C.POINTER(RlGenWeights), vp, sz, vp, sz, C.POINTER(vp)]),
        "rl_gen_page_bytes": (sz, [sp, i32]),
        "rl_gen_create_paged": (C.c_int, [sp, C.POINTER(RlGenWeights), vp, sz, vp, sz, i32, C.POINTER(vp)]),
        "rl_gen_pool_pages": (C.c_int, [vp]),
        "rl_gen_set_block_table": (C.c_int, [vp, C.POINTER(i32), C.POINTER(i32), i32, i32, vp]),
        "rl_gen_plan_pages": (i32, [C.POINTER(i32), i32, i32, i32, i32, C.POINTER(i32)]),
        "rl_gen_packed_bytes": (sz, [sp]),
        "rl_gen_packed_bytes_full": (sz, [sp]),
        "rl_gen_prefers_packed_gate_up": (C.c_int, [sp]),
        "rl_gen_packed_gate_up_layers": (C.c_int, [vp]),
        "rl_gen_pack_weights": (C.c_int, [vp, vp, sz, vp]),
        "rl_gen_prefill": (C.c_int, [vp, vp, i32, i32, vp, vp, vp]),
        "rl_gen_prefill_ragged": (C.c_int, [vp, vp, vp, i32, i32, vp, vp, vp]),
        "rl_gen_set_eos": (C.c_int, [vp, i32]),
        "rl_gen_read_state": (C.c_int, [vp, C.POINTER(i32), C.POINTER(i32), vp]),
        "rl_gen_compact": (C.c_int, [vp, vp, C.POINTER(i32), C.POINTER(i32), vp]),
        "rl_gen_decode_step": (C.c_int, [vp, vp, vp, vp, vp]),
        "rl_gen_generate": (C.c_int, [vp, vp, i32, i32, i32, vp, vp, vp]),
        "rl_gen_logprobs": (C.c_int, [vp, vp, i32, i32, vp, vp]),
        "rl_gen_values": (C.c_int, [vp, vp, i32, i32, vp, vp, vp]),
        "rl_gen_set_graph": (C.c_int, [vp, i32]),
        "rl_gen_set_qkv_terms": (C.c_int, [vp, i32]),
        "rl_gen_set_sampling": (C.c_int, [vp, f32, vp]),
        "rl_gen_reset": (C.c_int, [vp]),
        "rl_gen_state": (C.c_int, [vp, C.POINTER(i32), C.POINTER(i32)]),
        "rl_gen_destroy": (None, [vp]),
        "rl_gen_last_error": (C.c_char_p, [vp]),
        "rl_gen_profile": (C.c_int, [vp, i32]),
        "rl_gen_profile_read": (C.c_int, [vp, C.POINTER(i32), C.POINTER(f32), vp]),
        "rl_gen_kernel_class_name": (C.c_char_p, [i32]),
        "rl_op_embed": (C.c_int, [vp, vp, vp, i32, i32, i32, vp]),
        "rl_op_add_rmsnorm": (C.c_int, [vp, vp, i32, sz, vp, f32, vp, vp, i32, i32, vp]),
        "rl_op_gemm": (C.c_int, [vp, vp, i64, vp, vp, vp, i32, i32, i32, i32, i32, vp, i64, sz, i32, i32, i32, vp, vp]),
        "rl_op_gemm_rope": (C.c_int, [vp, vp, i64, vp, vp, vp, vp, vp, vp, i32, i32, i32, i32, i32, i32, i32, vp, i32, i32, vp, vp, vp, vp, vp, vp, vp]),
        "rl_op_gemm_packed_swiglu_halves": (C.c_int, [vp, i64, vp, vp, i32, i32, i32, vp, i64, i32, vp, vp]),
        "rl_op_gemm_tiled_packed": (C.c_int, [vp, vp, i64, vp, vp, vp, vp, vp, vp, i32, i32, i32, i32, i32, vp, i64, i32, vp]),
        "rl_op_packed_weight_bytes": (sz, [i32, i32]),
        "rl_op_pack_weights": (C.c_int, [vp, vp, i32, i32, vp]),
        "rl_op_gemm_packed": (C.c_int, [vp, vp, i64, vp, vp, vp, i32, i32, i32, i32, i32, vp, i64, sz, i32, i32, i32, i32, i32, vp, vp]),
        "rl_op_lm_head_argmax_ws_floats": (C.c_size_t, [i32, i32]),
        "rl_op_lm_head_argmax": (C.c_int, [vp, vp, i64, vp, i32, i32, i32, vp, i64, vp, vp, vp]),
        "rl_op_build_rope_table": (C.c_int, [vp, i32, i32, f32]),
        "rl_op_rope_append": (C.c_int, [vp, i32, sz, i32, i32, i32, vp, i32, vp, i32, i32, i32, i32, i32, vp, vp, vp, vp, vp, vp, vp, vp]),
        "rl_op_decode_attention": (C.c_int, [vp, vp, vp, vp, i32, vp, vp, i32, i32, i32, i32, i32, i32, vp, vp, vp, vp, vp]),
        "rl_op_decode_attention_ws_floats": (sz, [i32, i32, i32, i32]),
        "rl_op_decode_attention_noalloc": (C.c_int, [vp, vp, vp, vp, i32, vp, i32, i32, i32, i32, i32, i32, vp, vp, vp, vp, vp]),
        "rl_op_decode_attention_paged": (C.c_int, [vp, vp, vp, vp, i32, i32, vp, i32, vp, vp, i32, i32, i32, i32, i32, i32, vp, vp, vp]),
        "rl_op_decode_attention_fused": (C.c_int, [vp, i32, sz, vp, i32, vp, vp, vp, i32, vp, vp, i32, i32, i32, i32, i32, i32, vp]),
        "rl_op_prefill_attention": (C.c_int, [vp, vp, vp, vp, i32, i32, i32, i32, i32, i32, i32, vp, vp, vp, vp, vp]),
        "rl_op_argmax": (C.c_int, [vp, i32, i32, vp, vp]),
        "rl_op_sample": (C.c_int, [vp, i32, i32, f32, vp, vp, vp]),
        "rl_op_logprob_gather": (C.c_int, [vp, i64, i32, i32, vp, i32, i64, vp, vp]),
        "rl_op_copy": (C.c_int, [vp, vp, sz, vp]),
    }
    for name, (res, args) in sig.items():
        fn = getattr(L, name)
        fn.restype = res
        fn.argtypes = args
    L._signatures = sig
    _LIB = L
    return L


EXPORTED_SYMBOLS = (
    "rl_gen_validate_shape", "rl_gen_param_count", "rl_gen_kv_bytes", "rl_gen_precision_level", "rl_gen_kv_block_scaled", "rl_gen_work_bytes", "rl_gen_create", "rl_gen_page_bytes", "rl_gen_create_paged", "rl_gen_pool_pages", "rl_gen_set_block_table", "rl_gen_plan_pages", "rl_gen_packed_bytes", "rl_gen_packed_bytes_full", "rl_gen_prefers_packed_gate_up", "rl_gen_packed_gate_up_layers",
    "rl_gen_pack_weights", "rl_gen_prefill", "rl_gen_prefill_ragged", "rl_gen_set_eos", "rl_gen_read_state", "rl_gen_compact", "rl_gen_logprobs", "rl_gen_values",
    "rl_gen_decode_step", "rl_gen_generate", "rl_gen_set_graph", "rl_gen_set_qkv_terms", "rl_gen_set_sampling", "rl_gen_reset", "rl_gen_state", "rl_gen_destroy", "rl_gen_last_error",
    "rl_gen_profile", "rl_gen_profile_read", "rl_gen_kernel_class_name", "rl_op_embed", "rl_op_add_rmsnorm", "rl_op_gemm",
    "rl_op_gemm_rope", "rl_op_gemm_tiled_packed", "rl_op_packed_weight_bytes", "rl_op_pack_weights", "rl_op_gemm_packed", "rl_op_lm_head_argmax_ws_floats", "rl_op_lm_head_argmax", "rl_op_gemm_packed_swiglu_halves", "rl_op_build_rope_table", "rl_op_rope_append", "rl_op_decode_attention", "rl_op_decode_attention_ws_floats", "rl_op_decode_attention_noalloc", "rl_op_decode_attention_paged", "rl_op_decode_attention_fused",
    "rl_op_prefill_attention", "rl_op_argmax", "rl_op_sample", "rl_op_logprob_gather", "rl_op_copy")


def _shape_of(shape, max_batch=1, max_seq=1, weight_dtype=1, precision=0) -> RlGenShape:
    return shape if isinstance(shape, RlGenShape) else RlGenShape.from_model(shape, max_batch, max_seq, weight_dtype, precision)


def precision_level(shape, precision=0) -> int:
    return int(lib().rl_gen_precision_level(C.byref(_shape_of(shape, precision=precision))))


def kv_block_scaled(shape, precision=0) -> bool:
    return int(lib().rl_gen_kv_block_scaled(C.byref(_shape_of(shape, precision=precision)))) == 1


def validate_shape(shape, max_batch=1, max_seq=1) -> int:
    return int(lib().rl_gen_validate_shape(C.byref(_shape_of(shape, max_batch, max_seq))))


def param_count(shape) -> int:
    return int(lib().rl_gen_param_count(C.byref(_shape_of(shape))))


def kv_bytes(shape, max_batch=1, max_seq=1, precision=0) -> int:
    return int(lib().rl_gen_kv_bytes(C.byref(_shape_of(shape, max_batch, max_seq, precision=precision))))


def work_bytes(shape, max_batch=1, max_seq=1) -> int:
    return int(lib().rl_gen_work_bytes(C.byref(_shape_of(shape, max_batch, max_seq))))


def page_bytes(shape, page_size: int, precision=0) -> int:
    return int(lib().rl_gen_page_bytes(C.byref(_shape_of(shape, precision=precision)), int(page_size)))


def plan_pages(capacity, page_size: int, n_pages: int, pages_per_seq: int):
    """Consecutive pool pages for sequences of the given capacities: (pages used, table as a list of rows)."""
    B = len(capacity)
    cap = (C.c_int32 * max(B, 1))(*[int(c) for c in capacity])
    tab = (C.c_int32 * max(B * pages_per_seq, 1))()
    used = int(lib().rl_gen_plan_pages(cap, B, int(page_size), int(n_pages), int(pages_per_seq), tab))
    if used < 0:
        raise RlGenError(used, "rl_gen_plan_pages")
    flat = list(tab)[: B * pages_per_seq]
    return used, [flat[b * pages_per_seq:(b + 1) * pages_per_seq] for b in range(B)]


def _ptr(t) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _stream() -> int:
    import torch
    return torch.cuda.current_stream().cuda_stream


class Generator:
    """rl_gen handle plus the torch tensors (weights, arenas) it borrows.

    weights: dict as produced by workload.make_weights, tensors on the GPU, all bf16 or all fp32.
    packed: also hold fragment-order copies of the projection matrices (what the decode step streams);
    call pack_weights() again after the weight tensors were updated in place.
    """

    def __init__(self, shape, weights: Dict[str, object], max_batch: int, max_seq: int, packed: bool = True,
                 page_size: int = 0, n_pages: int = 0, pack_gate_up: Optional[bool] = None, precision: int = 0):
        import torch
        self._h = None
        any_w = weights["tok_emb"]
        wd = 1 if any_w.dtype == torch.bfloat16 else 0
        if wd == 0 and any_w.dtype != torch.float32:
            raise TypeError("weights must be bf16 or fp32")
        self.shape = shape
        self.cshape = RlGenShape.from_model(shape, max_batch, max_seq, wd, precision)
        self._keep: List[object] = []

        def hold(t):
            if not t.is_cuda or not t.is_contiguous() or t.dtype != any_w.dtype:
                raise TypeError("weights must be contiguous GPU tensors of one dtype")
            self._keep.append(t)
            return t.data_ptr()

        w = RlGenWeights()
        w.tok_emb, w.final_norm, w.lm_head = hold(weights["tok_emb"]), hold(weights["final_norm"]), hold(weights["lm_head"])
        self._arrays = []
        for name in LAYER_NAMES:
            arr = (C.c_void_p * max(shape.n_layers, 1))()
            lst = weights[name]
            if len(lst) != shape.n_layers:
                raise ValueError(f"{name}: expected {shape.n_layers} tensors")
            for l, t in enumerate(lst):
                arr[l] = hold(t)
            self._arrays.append(arr)
            setattr(w, name, C.cast(arr, C.POINTER(C.c_void_p)))
        L = lib()
        rc = L.rl_gen_validate_shape(C.byref(self.cshape))
        if rc != 0:
            raise RlGenError(rc, "rl_gen_validate_shape")
        nwork = L.rl_gen_work_bytes(C.byref(self.cshape))
        self.page_size = int(page_size)
        if page_size:   # paged cache: the arena is a pool of n_pages pages
            pb = L.rl_gen_page_bytes(C.byref(self.cshape), int(page_size))
            if pb == 0 and shape.n_layers > 0:
                raise RlGenError(-2, "rl_gen_page_bytes", f"page size {page_size}")
            nkv = pb * int(n_pages)
        else:
            nkv = L.rl_gen_kv_bytes(C.byref(self.cshape))
        dev = any_w.device
        self.kv_arena = torch.empty(max(nkv, 256), dtype=torch.uint8, device=dev)
        self.work_arena = torch.empty(nwork, dtype=torch.uint8, device=dev)
        h = C.c_void_p()
        if page_size:
            rc = L.rl_gen_create_paged(C.byref(self.cshape), C.byref(w), self.kv_arena.data_ptr(), nkv,
                                       self.work_arena.data_ptr(), nwork, int(page_size), C.byref(h))
        else:
            rc = L.rl_gen_create(C.byref(self.cshape), C.byref(w), self.kv_arena.data_ptr(), nkv, self.work_arena.data_ptr(),
                                 nwork, C.byref(h))
        if rc != 0:
            raise RlGenError(rc, "rl_gen_create", L.rl_gen_last_error(None).decode())
        self._h = h
        self.max_batch, self.max_seq = max_batch, max_seq
        self.packed_arena = None
        # copies of the gate/up pair too?  None: where the library says its fragment-order kernel is the faster one
        # (an int: at most that many layers)
        self._gate_up_layer_limit = pack_gate_up if isinstance(pack_gate_up, int) and not isinstance(pack_gate_up, bool) else None
        self.pack_gate_up = bool(L.rl_gen_prefers_packed_gate_up(C.byref(self.cshape)) == 1) if pack_gate_up is None else bool(pack_gate_up)
        if packed:
            self.pack_weights()

    def pack_weights(self):
        """(Re)builds the fragment-order weight copies from the current contents of the weight tensors."""
        import torch
        if self.packed_arena is None:
            n = lib().rl_gen_packed_bytes(C.byref(self.cshape))
            if self.pack_gate_up and self.shape.n_layers > 0:
                # the copies are optional: as many layers as fit while leaving room for everything else
                full = lib().rl_gen_packed_bytes_full(C.byref(self.cshape))
                pair = (full - n) // self.shape.n_layers
                free, _ = torch.cuda.mem_get_info(self.kv_arena.device)
                layers = min(self.shape.n_layers, max(0, (free - (8 << 30) - n) // pair))
                if self._gate_up_layer_limit is not None:
                    layers = min(layers, self._gate_up_layer_limit)
                n += layers * pair
                self.pack_gate_up = layers > 0
            self.packed_arena = torch.empty(max(n, 256), dtype=torch.uint8, device=self.kv_arena.device)
        self._check(lib().rl_gen_pack_weights(self._h, self.packed_arena.data_ptr(), self.packed_arena.numel(), _stream()),
                    "rl_gen_pack_weights")

    def packed_gate_up_layers(self) -> int:
        return int(lib().rl_gen_packed_gate_up_layers(self._h))

    def unpack_weights(self):
        """Back to the row-major weights for every projection."""
        self._check(lib().rl_gen_pack_weights(self._h, None, 0, _stream()), "rl_gen_pack_weights")

    def _check(self, rc: int, where: str):
        if rc != 0:
            raise RlGenError(rc, where, lib().rl_gen_last_error(self._h).decode())

    def prefill(self, tokens, logits=None, next_tokens=None):
        """tokens: int32 GPU tensor [B, T].  Returns (logits fp32 [B, V], next int32 [B])."""
        import torch
        B, T = tokens.shape
        assert tokens.dtype == torch.int32 and tokens.is_cuda and tokens.is_contiguous()
        if logits is None:
            logits = torch.empty((B, self.shape.vocab), dtype=torch.float32, device=tokens.device)
        if next_tokens is None:
            next_tokens = torch.empty((B,), dtype=torch.int32, device=tokens.device)
        self._check(lib().rl_gen_prefill(self._h, tokens.data_ptr(), B, T, _ptr(logits), _ptr(next_tokens), _stream()),
                    "rl_gen_prefill")
        return logits, next_tokens

    def prefill_ragged(self, tokens, lens, logits=None, next_tokens=None):
        """tokens: int32 GPU tensor [B, T] (padded), lens: int32 GPU tensor [B].  Returns (logits of each sequence's last
        prompt position, next)."""
        import torch
        B, T = tokens.shape
        assert tokens.dtype == torch.int32 and tokens.is_cuda and tokens.is_contiguous()
        assert lens.dtype == torch.int32 and lens.is_cuda and lens.is_contiguous() and lens.numel() == B
        if logits is None:
            logits = torch.empty((B, self.shape.vocab), dtype=torch.float32, device=tokens.device)
        if next_tokens is None:
            next_tokens = torch.empty((B,), dtype=torch.int32, device=tokens.device)
        self._check(lib().rl_gen_prefill_ragged(self._h, tokens.data_ptr(), lens.data_ptr(), B, T, _ptr(logits), _ptr(next_tokens),
                                                _stream()), "rl_gen_prefill_ragged")
        return logits, next_tokens

    def pool_pages(self) -> int:
        return int(lib().rl_gen_pool_pages(self._h))

    def set_block_table(self, table, capacity):
        """table: rows of pool page numbers (one row per sequence), capacity: positions reserved per sequence."""
        B = len(capacity)
        pps = max(len(r) for r in table) if B else 1
        flat = (C.c_int32 * max(B * pps, 1))()
        for b, row in enumerate(table):
            for i, v in enumerate(row):
                flat[b * pps + i] = int(v)
        cap = (C.c_int32 * max(B, 1))(*[int(c) for c in capacity])
        self._check(lib().rl_gen_set_block_table(self._h, flat, cap, B, pps, _stream()), "rl_gen_set_block_table")

    def set_eos(self, eos: int):
        self._check(lib().rl_gen_set_eos(self._h, int(eos)), "rl_gen_set_eos")

    def read_state(self):
        """(lengths, end flags) of the current sequences as Python lists."""
        b, _ = self.state()
        lens, done = (C.c_int32 * max(b, 1))(), (C.c_int32 * max(b, 1))()
        self._check(lib().rl_gen_read_state(self._h, lens, done, _stream()), "rl_gen_read_state")
        return list(lens)[:b], list(done)[:b]

    def compact(self, tokens=None):
        """Drops the ended sequences from the batch (rl_gen_compact).  tokens: optional int32 GPU tensor [B], permuted in place;
        returns the old row of every remaining row as a list (the first len(list) entries of `tokens` are the new batch)."""
        b, _ = self.state()
        kept, n = (C.c_int32 * max(b, 1))(), C.c_int32(0)
        self._check(lib().rl_gen_compact(self._h, _ptr(tokens), kept, C.byref(n), _stream()), "rl_gen_compact")
        return list(kept)[: n.value]

    def decode_step(self, tokens, logits=None, next_tokens=None, want_logits=True):
        """tokens: int32 GPU tensor [B].  Returns (logits or None, next)."""
        import torch
        assert tokens.dtype == torch.int32 and tokens.is_cuda and tokens.is_contiguous()
        B = tokens.shape[0]
        if logits is None and want_logits:
            logits = torch.empty((B, self.shape.vocab), dtype=torch.float32, device=tokens.device)
        if next_tokens is None:
            next_tokens = torch.empty((B,), dtype=torch.int32, device=tokens.device)
        self._check(lib().rl_gen_decode_step(self._h, tokens.data_ptr(), _ptr(logits), _ptr(next_tokens), _stream()),
                    "rl_gen_decode_step")
        return logits, next_tokens

    def generate(self, prompts, G: int, u=None, out=None):
        """prompts: int32 GPU tensor [B, P] (B may exceed max_batch: sequential portions).  Returns int32 [B, G]."""
        import torch
        B, P = prompts.shape
        assert prompts.dtype == torch.int32 and prompts.is_cuda and prompts.is_contiguous()
        if u is not None:
            assert u.dtype == torch.float32 and u.is_cuda and u.is_contiguous() and tuple(u.shape) == (G, B)
        if out is None:
            out = torch.empty((B, G), dtype=torch.int32, device=prompts.device)
        self._check(lib().rl_gen_generate(self._h, prompts.data_ptr(), B, P, int(G), _ptr(u), out.data_ptr(), _stream()),
                    "rl_gen_generate")
        return out

    def logprobs(self, tokens, logp=None):
        """tokens: int32 GPU tensor [B, T].  Returns fp32 [B, T]: log-probability of token i+1 at position i (last column 0)."""
        import torch
        B, T = tokens.shape
        assert tokens.dtype == torch.int32 and tokens.is_cuda and tokens.is_contiguous()
        if logp is None:
            logp = torch.empty((B, T), dtype=torch.float32, device=tokens.device)
        self._check(lib().rl_gen_logprobs(self._h, tokens.data_ptr(), B, T, logp.data_ptr(), _stream()), "rl_gen_logprobs")
        return logp

    def values(self, tokens, head, out=None):
        """tokens: int32 GPU tensor [B, T]; head: GPU tensor [hidden] of the weights' dtype.  Returns fp32 [B, T]."""
        import torch
        B, T = tokens.shape
        assert tokens.dtype == torch.int32 and tokens.is_cuda and tokens.is_contiguous()
        assert head.is_cuda and head.is_contiguous() and head.numel() == self.shape.hidden and head.dtype == self._keep[0].dtype
        if out is None:
            out = torch.empty((B, T), dtype=torch.float32, device=tokens.device)
        self._check(lib().rl_gen_values(self._h, tokens.data_ptr(), B, T, head.data_ptr(), out.data_ptr(), _stream()), "rl_gen_values")
        return out

    def set_graph(self, enabled: bool):
        self._check(lib().rl_gen_set_graph(self._h, int(enabled)), "rl_gen_set_graph")

    def set_sampling(self, temperature: float, u=None):
        """temperature > 0: sample with the uniform draws in `u` (fp32 GPU tensor [max_batch], refreshed by the caller between
        steps); temperature <= 0: greedy."""
        self._sample_u = u           # keep the borrowed tensor alive
        self._check(lib().rl_gen_set_sampling(self._h, float(temperature), _ptr(u)), "rl_gen_set_sampling")

    def set_qkv_terms(self, terms: int):
        self._check(lib().rl_gen_set_qkv_terms(self._h, int(terms)), "rl_gen_set_qkv_terms")

    def reset(self):
        self._check(lib().rl_gen_reset(self._h), "rl_gen_reset")

    def state(self):
        b, n = C.c_int32(), C.c_int32()
        self._check(lib().rl_gen_state(self._h, C.byref(b), C.byref(n)), "rl_gen_state")
        return b.value, n.value

    def profile(self, enabled: bool):
        self._check(lib().rl_gen_profile(self._h, int(enabled)), "rl_gen_profile")

    def profile_read(self) -> Dict[str, Dict[str, float]]:
        n = len(KERNEL_CLASSES)
        launches, ms = (C.c_int32 * n)(), (C.c_float * n)()
        self._check(lib().rl_gen_profile_read(self._h, launches, ms, _stream()), "rl_gen_profile_read")
        return {KERNEL_CLASSES[i]: {"launches": int(launches[i]), "ms": float(ms[i])} for i in range(n)}

    def close(self):
        if getattr(self, "_h", None):
            lib().rl_gen_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class _Ops:
    """Single-kernel entry points (rl_op_*), tensors in, status checked."""

    @staticmethod
    def _ck(rc, name):
        if rc != 0:
            raise RlGenError(rc, name)

    def embed(self, tokens, emb, x):
        self._ck(lib().rl_op_embed(tokens.data_ptr(), emb.data_ptr(), x.data_ptr(), tokens.numel(), emb.shape[1], emb.shape[0],
                                   _stream()), "rl_op_embed")

    def add_rmsnorm(self, x, part, nsplit, part_stride, gain, eps, h, h_lo=None):
        M, d = x.shape
        self._ck(lib().rl_op_add_rmsnorm(x.data_ptr(), _ptr(part), nsplit, part_stride, gain.data_ptr(), eps, h.data_ptr(), _ptr(h_lo), M, d,
                                         _stream()), "rl_op_add_rmsnorm")

    def gemm(self, A, Ws, out, ldc, M=None, lda=None, split_stride=0, splits=1, epilogue=0, kernel=0, A_lo=None, out_lo=None):
        K = Ws[0].shape[1]
        ptrs = [w.data_ptr() for w in Ws] + [None] * (3 - len(Ws))
        rows = [w.shape[0] for w in Ws] + [0] * (3 - len(Ws))
        M = A.shape[0] if M is None else M
        lda = A.stride(0) if lda is None else lda
        self._ck(lib().rl_op_gemm(A.data_ptr(), _ptr(A_lo), lda, ptrs[0], ptrs[1], ptrs[2], rows[0], rows[1], rows[2], M, K, out.data_ptr(),
                                  ldc, split_stride, splits, epilogue, kernel, _ptr(out_lo), _stream()), "rl_op_gemm")

    def gemm_tiled_packed(self, A, Ws, Ps, out, ldc, M=None, epilogue=0, A_lo=None):
        K = Ws[0].shape[1]
        wp = [w.data_ptr() for w in Ws] + [None] * (3 - len(Ws))
        pp = [x.data_ptr() for x in Ps] + [None] * (3 - len(Ps))
        rows = [w.shape[0] for w in Ws] + [0] * (3 - len(Ws))
        M = A.shape[0] if M is None else M
        self._ck(lib().rl_op_gemm_tiled_packed(A.data_ptr(), _ptr(A_lo), A.stride(0), wp[0], wp[1], wp[2], pp[0], pp[1], pp[2], rows[0],
                                               rows[1], rows[2], M, K, out.data_ptr(), ldc, epilogue, _stream()), "rl_op_gemm_tiled_packed")

    def gemm_rope(self, A, Wq, Wk, Wv, Hq, Hkv, hd, M, T, b0, rope_tab, rope_style, S, q_f16, kc, vc, A_lo=None, Ps=None,
                  kscale=None, vscale=None, q_f16_lo=None):
        K = Wq.shape[1]
        pq, pk, pv = (x.data_ptr() for x in Ps) if Ps else (None, None, None)
        self._ck(lib().rl_op_gemm_rope(A.data_ptr(), _ptr(A_lo), A.stride(0), Wq.data_ptr(), Wk.data_ptr(), Wv.data_ptr(), pq, pk, pv, Hq, Hkv, hd, M, K,
                                       T, b0, rope_tab.data_ptr(), rope_style, S, q_f16.data_ptr(), kc.data_ptr(), vc.data_ptr(), _ptr(kscale), _ptr(vscale),
                                       _ptr(q_f16_lo), _stream()),
                 "rl_op_gemm_rope")

    def gemm_packed_swiglu_halves(self, A, Pg, Pu, F, K, out, ldc, M=None, depth=0, out_lo=None):
        M = A.shape[0] if M is None else M
        self._ck(lib().rl_op_gemm_packed_swiglu_halves(A.data_ptr(), A.stride(0), Pg.data_ptr(), Pu.data_ptr(), F, M, K, out.data_ptr(),
                                                       ldc, depth, _ptr(out_lo), _stream()), "rl_op_gemm_packed_swiglu_halves")

    def packed_weight_bytes(self, N, K):
        return int(lib().rl_op_packed_weight_bytes(N, K))

    def pack_weights(self, W, P):
        N, K = W.shape
        self._ck(lib().rl_op_pack_weights(W.data_ptr(), P.data_ptr(), N, K, _stream()), "rl_op_pack_weights")

    def gemm_packed(self, A, Ps, rows, K, out, ldc, A_lo=None, M=None, lda=None, split_stride=0, splits=1, epilogue=0, nb=0,
                    rows_per_wg=0, depth=0, out_lo=None):
        ptrs = [q.data_ptr() for q in Ps] + [None] * (3 - len(Ps))
        rows = list(rows) + [0] * (3 - len(rows))
        M = A.shape[0] if M is None else M
        lda = A.stride(0) if lda is None else lda
        self._ck(lib().rl_op_gemm_packed(A.data_ptr(), _ptr(A_lo), lda, ptrs[0], ptrs[1], ptrs[2], rows[0], rows[1], rows[2], M, K,
                                         out.data_ptr(), ldc, split_stride, splits, epilogue, nb, rows_per_wg, depth, _ptr(out_lo), _stream()), "rl_op_gemm_packed")

    def lm_head_argmax_ws_floats(self, M, V):
        return int(lib().rl_op_lm_head_argmax_ws_floats(M, V))

    def lm_head_argmax(self, A, P, V, K, nxt, logits=None, A_lo=None, ws=None):
        import torch
        M = A.shape[0]
        if ws is None:
            ws = torch.empty(max(int(lib().rl_op_lm_head_argmax_ws_floats(M, V)), 1), dtype=torch.float32, device=A.device)
        self._ck(lib().rl_op_lm_head_argmax(A.data_ptr(), _ptr(A_lo), A.stride(0), P.data_ptr(), V, M, K, _ptr(logits),
                                            logits.stride(0) if logits is not None else V, ws.data_ptr(), nxt.data_ptr(), _stream()),
                 "rl_op_lm_head_argmax")

    def build_rope_table(self, tab, max_seq, head_dim, base):
        self._ck(lib().rl_op_build_rope_table(tab.data_ptr(), max_seq, head_dim, base), "rl_op_build_rope_table")

    def rope_append(self, qkv, nsplit, split_stride, M, T, b0, d_pos0, rope_tab, rope_style, Hq, Hkv, hd, S, q_f32, q_bf16, kc, vc,
                    pos_stride=0, kscale=None, vscale=None, q_f16_lo=None):
        self._ck(lib().rl_op_rope_append(qkv.data_ptr(), nsplit, split_stride, M, T, b0, d_pos0.data_ptr(), pos_stride, rope_tab.data_ptr(),
                                         rope_style, Hq, Hkv, hd, S, _ptr(q_f32), _ptr(q_bf16), kc.data_ptr(), vc.data_ptr(),
                                         _ptr(kscale), _ptr(vscale), _ptr(q_f16_lo), _stream()), "rl_op_rope_append")

    def decode_attention_ws_floats(self, B, Hq, hd, nsplit):
        return int(lib().rl_op_decode_attention_ws_floats(B, Hq, hd, nsplit))

    def decode_attention(self, q, kc, vc, d_len, out, ws, B, Hq, Hkv, hd, S, nsplit, len_stride=0, d_done=None, kscale=None,
                         vscale=None, out_lo=None):
        self._ck(lib().rl_op_decode_attention(q.data_ptr(), kc.data_ptr(), vc.data_ptr(), d_len.data_ptr(), len_stride, out.data_ptr(),
                                              _ptr(ws), B, Hq, Hkv, hd, S, nsplit, _ptr(d_done), _ptr(kscale), _ptr(vscale), _ptr(out_lo),
                                              _stream()), "rl_op_decode_attention")

    def decode_attention_noalloc(self, q, kc, vc, d_len, out, B, Hq, Hkv, hd, S, nsplit, len_stride=0, d_done=None, kscale=None,
                                 vscale=None, out_lo=None):
        self._ck(lib().rl_op_decode_attention_noalloc(q.data_ptr(), kc.data_ptr(), vc.data_ptr(), d_len.data_ptr(), len_stride,
                                                      out.data_ptr(), B, Hq, Hkv, hd, S, nsplit, _ptr(d_done), _ptr(kscale),
                                                      _ptr(vscale), _ptr(out_lo), _stream()), "rl_op_decode_attention_noalloc")

    def decode_attention_paged(self, q, k_pool, v_pool, table, page_size, d_len, out, ws, B, Hq, Hkv, hd, S, nsplit, len_stride=0,
                               kscale=None, vscale=None):
        self._ck(lib().rl_op_decode_attention_paged(q.data_ptr(), k_pool.data_ptr(), v_pool.data_ptr(), table.data_ptr(),
                                                    table.shape[1], page_size, d_len.data_ptr(), len_stride, out.data_ptr(), _ptr(ws),
                                                    B, Hq, Hkv, hd, S, nsplit, _ptr(kscale), _ptr(vscale), _stream()),
                 "rl_op_decode_attention_paged")

    def decode_attention_fused(self, qkv, nsplit_qkv, split_stride, rope_tab, rope_style, kc, vc, d_len, out, ws, B, Hq, Hkv, hd, S,
                               nsplit, len_stride=0):
        self._ck(lib().rl_op_decode_attention_fused(qkv.data_ptr(), nsplit_qkv, split_stride, rope_tab.data_ptr(), rope_style,
                                                    kc.data_ptr(), vc.data_ptr(), d_len.data_ptr(), len_stride, out.data_ptr(), _ptr(ws), B, Hq,
                                                    Hkv, hd, S, nsplit, _stream()), "rl_op_decode_attention_fused")

    def prefill_attention(self, q, kc, vc, out, nb, b0, T, Hq, Hkv, hd, S, kscale=None, vscale=None, out_lo=None, q_lo=None):
        self._ck(lib().rl_op_prefill_attention(q.data_ptr(), kc.data_ptr(), vc.data_ptr(), out.data_ptr(), nb, b0, T, Hq, Hkv,
                                               hd, S, _ptr(kscale), _ptr(vscale), _ptr(out_lo), _ptr(q_lo), _stream()), "rl_op_prefill_attention")

    def sample(self, logits, temperature, u, nxt):
        B, V = logits.shape
        self._ck(lib().rl_op_sample(logits.data_ptr(), B, V, float(temperature), u.data_ptr(), nxt.data_ptr(), _stream()), "rl_op_sample")

    def logprob_gather(self, logits, tokens, T, m_first, out):
        M, V = logits.shape
        self._ck(lib().rl_op_logprob_gather(logits.data_ptr(), logits.stride(0), M, V, tokens.data_ptr(), T, m_first, out.data_ptr(),
                                            _stream()), "rl_op_logprob_gather")

    def copy(self, src, dst):
        self._ck(lib().rl_op_copy(src.data_ptr(), dst.data_ptr(), src.numel() * src.element_size(), _stream()), "rl_op_copy")

    def argmax(self, logits, nxt):
        B, V = logits.shape
        self._ck(lib().rl_op_argmax(logits.data_ptr(), B, V, nxt.data_ptr(), _stream()), "rl_op_argmax")


ops = _Ops()
