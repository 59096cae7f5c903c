"""ctypes binding of libifkv.so (include/ifkv.h).

Argument marshalling only: every step of the path runs in the library's HIP
kernels.  torch is used to allocate device memory and to name the stream.  If
the library has not been built the import of any entry point fails loudly;
there is no fallback.
"""
from __future__ import annotations

import ctypes as C
import math
import os
from typing import List, Optional, Sequence, Tuple

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libifkv.so")

IFKV_OK, IFKV_EINVAL, IFKV_ESHAPE, IFKV_EDTYPE, IFKV_ENOMEM, IFKV_EHIP = 0, -1, -2, -3, -4, -5
IFKV_F32, IFKV_BF16 = 0, 1
IFKV_ROPE_HALF, IFKV_ROPE_INTERLEAVED = 0, 1
IFKV_FLAG_FORCE_GENERIC = 1
IFKV_FLAG_VALIDATE = 2

EXPORTS = (
    "ifkv_create", "ifkv_destroy", "ifkv_last_error", "ifkv_version",
    "ifkv_reposition_keys", "ifkv_score_tokens", "ifkv_reposition_score", "ifkv_select_topk", "ifkv_select_topk_noalloc",
    "ifkv_recompute_attention", "ifkv_splice_kv", "ifkv_rope_rows", "ifkv_chunk_counts", "ifkv_reorder_chunks",
    "ifkv_copy_bytes", "ifkv_mfma_probe", "ifkv_mfma_probe_sink_floats",   # include/ifkv_calibrate.h
    "ifkv_set_tuning", "ifkv_attention_plan",                                # include/ifkv_debug.h
)


class LayerDesc(C.Structure):
    _fields_ = [
        ("dtype", C.c_int32), ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32),
        ("head_dim", C.c_int32), ("rope_theta", C.c_double), ("inv_freq", C.POINTER(C.c_double)),
        ("pairing", C.c_int32), ("sm_scale", C.c_float), ("max_ctx", C.c_int64),
        ("max_prompt", C.c_int32), ("flags", C.c_uint32),
        ("token_stride", C.c_int64), ("head_stride", C.c_int64),
    ]


class IfkvError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"ifkv error {code}: {msg}")
        self.code = code


_lib = None


def load_library() -> C.CDLL:
    """Loads libifkv.so; raises if it has not been built (no fallback path)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(
            f"{LIB_PATH} is missing: build it with `python -m paper_2603_05353_amd.build` "
            "(there is no fallback implementation)")
    lib = C.CDLL(LIB_PATH)
    vp, i32, i64 = C.c_void_p, C.c_int32, C.c_int64
    lib.ifkv_create.argtypes = [C.POINTER(vp), C.POINTER(LayerDesc), vp]
    lib.ifkv_create.restype = C.c_int
    lib.ifkv_destroy.argtypes = [vp]
    lib.ifkv_destroy.restype = None
    lib.ifkv_last_error.argtypes = [vp]
    lib.ifkv_last_error.restype = C.c_char_p
    lib.ifkv_version.argtypes = []
    lib.ifkv_version.restype = C.c_char_p
    lib.ifkv_reposition_keys.argtypes = [vp, i32, C.POINTER(vp), C.POINTER(vp), C.POINTER(i32),
                                         C.POINTER(i32), C.POINTER(i32), C.POINTER(i64), vp, vp,
                                         C.POINTER(i64), C.POINTER(i64)]
    lib.ifkv_reposition_keys.restype = C.c_int
    lib.ifkv_score_tokens.argtypes = [vp, vp, i64, vp, i32, vp, i32, vp]
    lib.ifkv_score_tokens.restype = C.c_int
    lib.ifkv_reposition_score.argtypes = [vp, i32, C.POINTER(vp), C.POINTER(vp), C.POINTER(i32), C.POINTER(i32),
                                          C.POINTER(i32), C.POINTER(i64), vp, vp, C.POINTER(i64), C.POINTER(i64),
                                          vp, i32, vp, i32, vp]
    lib.ifkv_reposition_score.restype = C.c_int
    lib.ifkv_select_topk.argtypes = [vp, vp, i64, C.c_double, i64, vp, C.POINTER(i64)]
    lib.ifkv_select_topk.restype = C.c_int
    lib.ifkv_select_topk_noalloc.argtypes = [vp, vp, i64, C.c_double, i64, vp, C.POINTER(i64)]
    lib.ifkv_select_topk_noalloc.restype = C.c_int
    lib.ifkv_recompute_attention.argtypes = [vp, vp, vp, i64, vp, vp, i64, vp, vp]
    lib.ifkv_recompute_attention.restype = C.c_int
    lib.ifkv_splice_kv.argtypes = [vp, vp, vp, vp, i64, vp, vp, i64]
    lib.ifkv_splice_kv.restype = C.c_int
    lib.ifkv_rope_rows.argtypes = [vp, vp, vp, i64, i32]
    lib.ifkv_rope_rows.restype = C.c_int
    lib.ifkv_chunk_counts.argtypes = [vp, vp, i64, i32, C.POINTER(i64), i64, vp]
    lib.ifkv_chunk_counts.restype = C.c_int
    lib.ifkv_reorder_chunks.argtypes = [vp, i32, C.POINTER(i32), C.POINTER(i32), C.POINTER(i32), C.POINTER(i32)]
    lib.ifkv_reorder_chunks.restype = C.c_int
    lib.ifkv_copy_bytes.argtypes = [vp, vp, vp, i64]
    lib.ifkv_copy_bytes.restype = C.c_int
    lib.ifkv_mfma_probe.argtypes = [vp, i32, i64, vp, C.POINTER(C.c_double)]
    lib.ifkv_mfma_probe.restype = C.c_int
    lib.ifkv_mfma_probe_sink_floats.argtypes = []
    lib.ifkv_mfma_probe_sink_floats.restype = i64
    lib.ifkv_set_tuning.argtypes = [vp, C.c_char_p, i64]
    lib.ifkv_set_tuning.restype = C.c_int
    lib.ifkv_attention_plan.argtypes = [vp, i64, i64, C.POINTER(C.c_int64)]
    lib.ifkv_attention_plan.restype = C.c_int
    _lib = lib
    return lib


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _i32_array(x: Optional[Sequence[int]]):
    if x is None:
        return None
    return (C.c_int32 * len(x))(*[int(v) for v in x])


def _i64_array(x: Optional[Sequence[int]]):
    if x is None:
        return None
    return (C.c_int64 * len(x))(*[int(v) for v in x])


_TORCH_DTYPE = {"f32": torch.float32, "bf16": torch.bfloat16}
_ENUM_DTYPE = {"f32": IFKV_F32, "bf16": IFKV_BF16}


class Layer:
    """One ifkv_ctx: a layer shape bound to a HIP stream."""

    def __init__(self, dtype: str, n_q_heads: int, n_kv_heads: int, head_dim: int, rope_theta: float,
                 max_ctx: int, max_prompt: int, pairing: str = "half", sm_scale: float = 0.0,
                 inv_freq: Optional[Sequence[float]] = None, flags: int = 0,
                 stream: Optional[int] = None, device: str = "cuda:0",
                 token_stride: int = 0, head_stride: int = 0):
        self._lib = load_library()
        self._recording = None
        self.dtype = dtype
        self.torch_dtype = _TORCH_DTYPE[dtype]
        self.n_q_heads, self.n_kv_heads, self.head_dim = n_q_heads, n_kv_heads, head_dim
        self.device = device
        desc = LayerDesc()
        desc.dtype = _ENUM_DTYPE[dtype]
        desc.n_q_heads, desc.n_kv_heads, desc.head_dim = n_q_heads, n_kv_heads, head_dim
        desc.rope_theta = float(rope_theta)
        self._freq = None
        if inv_freq is not None:
            self._freq = (C.c_double * len(inv_freq))(*[float(v) for v in inv_freq])
            desc.inv_freq = C.cast(self._freq, C.POINTER(C.c_double))
        desc.pairing = IFKV_ROPE_HALF if pairing == "half" else IFKV_ROPE_INTERLEAVED
        desc.sm_scale = float(sm_scale)
        desc.max_ctx, desc.max_prompt, desc.flags = int(max_ctx), int(max_prompt), int(flags)
        desc.token_stride, desc.head_stride = int(token_stride), int(head_stride)
        self.token_stride = int(token_stride) or n_kv_heads * head_dim
        self.head_stride = int(head_stride) or head_dim
        self.max_ctx = int(max_ctx)
        if stream is None and torch.cuda.is_available():
            stream = torch.cuda.current_stream().cuda_stream
        self._ctx = C.c_void_p()
        rc = self._lib.ifkv_create(C.byref(self._ctx), C.byref(desc), C.c_void_p(stream or 0))
        if rc != IFKV_OK:
            raise IfkvError(rc, self._lib.ifkv_last_error(None).decode())

    # -- plumbing -----------------------------------------------------------
    def close(self):
        if getattr(self, "_ctx", None) is not None and self._ctx.value:
            self._lib.ifkv_destroy(self._ctx)
            self._ctx = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _check(self, rc: int):
        if rc != IFKV_OK:
            raise IfkvError(rc, self._lib.ifkv_last_error(self._ctx).decode())

    def _invoke(self, cfunc, *cargs):
        """One C call of a stage; while bind() records, the call is also kept for replay."""
        if self._recording is not None:
            self._recording.append((cfunc, cargs))
        self._check(cfunc(*cargs))

    def bind(self, stage: str, *args, **kw):
        """Marshals a stage call once and returns a function that repeats it: stage(*args, **kw) runs
        once now (checks, buffer look-ups, ctypes arrays), the returned function only re-issues the C
        call(s) with the same arguments.  For loops that call a stage many times on the same buffers
        (benchmarks, graph capture) without paying the Python-side marshalling every time."""
        self._recording = []
        try:
            result = getattr(self, stage)(*args, **kw)
        finally:
            calls, self._recording = self._recording, None
        check, keep = self._check, (args, kw, result)

        def replay(_keep=keep):
            for cfunc, cargs in calls:
                check(cfunc(*cargs))
        return replay

    def _empty(self, *shape, dtype=None):
        return torch.empty(*shape, dtype=dtype or self.torch_dtype, device=self.device)

    def empty_cache(self, n_rows: int) -> torch.Tensor:
        """A concatenated cache [n_rows, H_kv, d] in the layout the layer was created with."""
        return torch.empty_strided((int(n_rows), self.n_kv_heads, self.head_dim), (self.token_stride, self.head_stride, 1),
                                   dtype=self.torch_dtype, device=self.device)

    # Argument marshalling: a pointer is only taken from a tensor that is what the C call expects
    # (device, dtype, shape, layout); anything else would be read as garbage or out of bounds.
    def _packed(self, t: Optional[torch.Tensor], name: str, tail: Tuple[int, ...], dtype=None, rows: Optional[int] = None):
        if t is None:
            return None
        want = dtype or self.torch_dtype
        if not t.is_cuda or t.dtype != want:
            raise ValueError(f"{name}: expected a {want} tensor on the GPU, got {t.dtype} on {t.device}")
        if tuple(t.shape[1:]) != tuple(tail) or (rows is not None and t.shape[0] < rows):
            raise ValueError(f"{name}: expected shape [{'R' if rows is None else rows}, {', '.join(map(str, tail))}], got {tuple(t.shape)}")
        if not t.is_contiguous():
            raise ValueError(f"{name}: must be contiguous")
        return t.data_ptr()

    def _cache(self, t: Optional[torch.Tensor], name: str):
        if t is None:
            return None
        if not t.is_cuda or t.dtype != self.torch_dtype:
            raise ValueError(f"{name}: expected a {self.torch_dtype} tensor on the GPU, got {t.dtype} on {t.device}")
        if t.dim() != 3 or tuple(t.shape[1:]) != (self.n_kv_heads, self.head_dim):
            raise ValueError(f"{name}: expected shape [T, {self.n_kv_heads}, {self.head_dim}], got {tuple(t.shape)}")
        if t.shape[0] > 1 and tuple(t.stride()) != (self.token_stride, self.head_stride, 1):
            raise ValueError(f"{name}: strides {tuple(t.stride())} are not the layer's ({self.token_stride}, {self.head_stride}, 1)")
        return t.data_ptr()

    # -- the five stages ------------------------------------------------------
    def _repo_args(self, k_chunks, v_chunks, chunk_order, cached_pos0, delta_override, k_out, v_out):
        n = len(k_chunks)
        lens = [int(t.shape[0]) for t in k_chunks]
        N = sum(lens)
        if k_out is None:
            k_out = self.empty_cache(N)
        if v_chunks is not None and v_out is None:
            v_out = self.empty_cache(N)
        kv_tail = (self.n_kv_heads, self.head_dim)
        kp = (C.c_void_p * n)(*[self._packed(t, "k_chunks[i]", kv_tail) if t.shape[0] else None for t in k_chunks])
        vp = None
        if v_chunks is not None:
            if [int(t.shape[0]) for t in v_chunks] != lens:
                raise ValueError("v_chunks: lengths differ from k_chunks")
            vp = (C.c_void_p * n)(*[self._packed(t, "v_chunks[i]", kv_tail) if t.shape[0] else None for t in v_chunks])
        if k_out.shape[0] < N or (v_out is not None and v_out.shape[0] < N):
            raise ValueError("k_out / v_out: fewer rows than the chunks hold")
        starts = (C.c_int64 * max(n, 1))()
        n_ctx = C.c_int64()
        args = (self._ctx, n, kp, vp, _i32_array(lens), _i32_array(chunk_order), _i32_array(cached_pos0),
                _i64_array(delta_override), self._cache(k_out, "k_out"), self._cache(v_out, "v_out"), starts, C.byref(n_ctx))
        return args, k_out, v_out, starts, n_ctx, n, N

    def reposition_keys(self, k_chunks: List[torch.Tensor], v_chunks: Optional[List[torch.Tensor]] = None,
                        chunk_order: Optional[Sequence[int]] = None,
                        cached_pos0: Optional[Sequence[int]] = None,
                        delta_override: Optional[Sequence[int]] = None,
                        k_out: Optional[torch.Tensor] = None, v_out: Optional[torch.Tensor] = None
                        ) -> Tuple[torch.Tensor, Optional[torch.Tensor], List[int], int]:
        args, k_out, v_out, starts, n_ctx, n, _ = self._repo_args(k_chunks, v_chunks, chunk_order, cached_pos0,
                                                                   delta_override, k_out, v_out)
        self._invoke(self._lib.ifkv_reposition_keys, *args)
        return k_out, v_out, [int(starts[i]) for i in range(n)], int(n_ctx.value)

    def reposition_score(self, k_chunks: List[torch.Tensor], v_chunks: Optional[List[torch.Tensor]],
                         q_prompt: torch.Tensor, chunk_order: Optional[Sequence[int]] = None,
                         cached_pos0: Optional[Sequence[int]] = None, delta_override: Optional[Sequence[int]] = None,
                         k_out: Optional[torch.Tensor] = None, v_out: Optional[torch.Tensor] = None,
                         k_prompt: Optional[torch.Tensor] = None, scores: Optional[torch.Tensor] = None,
                         accumulate: bool = False):
        """ifkv_reposition_score: stages 1 and 2 in one call.  Returns (k_out, v_out, starts, n_ctx, scores)."""
        args, k_out, v_out, starts, n_ctx, n, N = self._repo_args(k_chunks, v_chunks, chunk_order, cached_pos0,
                                                                   delta_override, k_out, v_out)
        m = int(q_prompt.shape[0])
        if scores is None:
            scores = self._empty(N, dtype=torch.float32)
        self._invoke(self._lib.ifkv_reposition_score, 
            *args, self._packed(q_prompt, "q_prompt", (self.n_q_heads, self.head_dim)), m,
            self._packed(k_prompt, "k_prompt", (self.n_kv_heads, self.head_dim), rows=m), int(accumulate),
            self._packed(scores, "scores", (), dtype=torch.float32, rows=N))
        return k_out, v_out, [int(starts[i]) for i in range(n)], int(n_ctx.value), scores

    def score_tokens(self, k_global: torch.Tensor, q_prompt: torch.Tensor,
                     k_prompt: Optional[torch.Tensor] = None, scores: Optional[torch.Tensor] = None,
                     accumulate: bool = False) -> torch.Tensor:
        n_ctx, m = int(k_global.shape[0]), int(q_prompt.shape[0])
        if scores is None:
            scores = self._empty(n_ctx, dtype=torch.float32)
        self._invoke(self._lib.ifkv_score_tokens, 
            self._ctx, self._cache(k_global, "k_global"), n_ctx, self._packed(q_prompt, "q_prompt", (self.n_q_heads, self.head_dim)), m,
            self._packed(k_prompt, "k_prompt", (self.n_kv_heads, self.head_dim), rows=m), int(accumulate),
            self._packed(scores, "scores", (), dtype=torch.float32, rows=n_ctx))
        return scores

    def select_topk(self, scores: torch.Tensor, ratio: float = 0.0, k: int = -1,
                    idx_out: Optional[torch.Tensor] = None) -> torch.Tensor:
        n_ctx = int(scores.shape[0])
        k_out = C.c_int64()
        sp = self._packed(scores, "scores", (), dtype=torch.float32)
        if idx_out is None:   # the library knows the budget: ask it, then bring a buffer of that size
            self._invoke(self._lib.ifkv_select_topk, self._ctx, sp, n_ctx, float(ratio), int(k), None, C.byref(k_out))
            idx_out = self._empty(max(int(k_out.value), 1), dtype=torch.int32)
        self._invoke(self._lib.ifkv_select_topk, self._ctx, sp, n_ctx, float(ratio), int(k),
                                               self._packed(idx_out, "idx_out", (), dtype=torch.int32), C.byref(k_out))
        if idx_out.shape[0] < int(k_out.value):
            raise ValueError("idx_out: fewer entries than k")   # (checked by budget_of before the call in careful code)
        return idx_out[: int(k_out.value)]

    def budget_of(self, n_ctx: int, ratio: float = 0.0, k: int = -1) -> int:
        """k = floor(ratio * n_ctx) as the library evaluates it (no GPU work)."""
        k_out = C.c_int64()
        self._invoke(self._lib.ifkv_select_topk, self._ctx, None, int(n_ctx), float(ratio), int(k), None, C.byref(k_out))
        return int(k_out.value)

    def select_topk_noalloc(self, scores: torch.Tensor, idx_out: torch.Tensor, ratio: float = 0.0, k: int = -1) -> torch.Tensor:
        """ifkv_select_topk_noalloc: the caller brings idx_out; the call allocates nothing."""
        k_out = C.c_int64()
        self._invoke(self._lib.ifkv_select_topk_noalloc, self._ctx, self._packed(scores, "scores", (), dtype=torch.float32),
                                                       int(scores.shape[0]), float(ratio), int(k),
                                                       self._packed(idx_out, "idx_out", (), dtype=torch.int32), C.byref(k_out))
        return idx_out[: int(k_out.value)]

    def recompute_attention(self, q_sel: torch.Tensor, row_pos: torch.Tensor, k_cache: torch.Tensor,
                            v_cache: torch.Tensor, out: Optional[torch.Tensor] = None,
                            return_lse: bool = False):
        n_rows, n_kv = int(q_sel.shape[0]), int(k_cache.shape[0])
        if out is None:
            out = self._empty(n_rows, self.n_q_heads, self.head_dim)
        lse = self._empty(n_rows, self.n_q_heads, dtype=torch.float32) if return_lse else None
        qh = (self.n_q_heads, self.head_dim)
        self._invoke(self._lib.ifkv_recompute_attention, 
            self._ctx, self._packed(q_sel, "q_sel", qh), self._packed(row_pos, "row_pos", (), dtype=torch.int32, rows=n_rows), n_rows,
            self._cache(k_cache, "k_cache"), self._cache(v_cache, "v_cache"), n_kv, self._packed(out, "out", qh, rows=n_rows),
            self._packed(lse, "lse", (self.n_q_heads,), dtype=torch.float32, rows=n_rows))
        return (out, lse) if return_lse else out

    def splice_kv(self, k_new: torch.Tensor, v_new: Optional[torch.Tensor], idx: torch.Tensor,
                  k_cache: torch.Tensor, v_cache: Optional[torch.Tensor]) -> None:
        n = int(idx.shape[0])
        kv_tail = (self.n_kv_heads, self.head_dim)
        self._invoke(self._lib.ifkv_splice_kv, self._ctx, self._packed(k_new, "k_new", kv_tail, rows=n),
                                             self._packed(v_new, "v_new", kv_tail, rows=n),
                                             self._packed(idx, "idx", (), dtype=torch.int32), n,
                                             self._cache(k_cache, "k_cache"), self._cache(v_cache, "v_cache"), int(k_cache.shape[0]))

    def rope_rows(self, x: torch.Tensor, pos: torch.Tensor) -> torch.Tensor:
        """In place; x [R, n_heads, d], pos int32 [R]."""
        if x.dim() != 3 or x.shape[2] != self.head_dim:
            raise ValueError(f"x: expected [R, n_heads, {self.head_dim}], got {tuple(x.shape)}")
        self._invoke(self._lib.ifkv_rope_rows, self._ctx, self._packed(x, "x", tuple(x.shape[1:])),
                                             self._packed(pos, "pos", (), dtype=torch.int32, rows=int(x.shape[0])),
                                             int(x.shape[0]), int(x.shape[1]))
        return x

    def chunk_counts(self, idx: torch.Tensor, slot_start: Sequence[int], n_ctx: int,
                     counts_out: Optional[torch.Tensor] = None) -> torch.Tensor:
        n_slots = len(slot_start)
        if counts_out is None:
            counts_out = self._empty(max(n_slots, 1), dtype=torch.int32)
        self._invoke(self._lib.ifkv_chunk_counts, self._ctx, self._packed(idx, "idx", (), dtype=torch.int32), int(idx.shape[0]), n_slots,
                                                _i64_array(slot_start), int(n_ctx),
                                                self._packed(counts_out, "counts_out", (), dtype=torch.int32, rows=n_slots))
        return counts_out[:n_slots]

    def reorder_chunks(self, order_in: Optional[Sequence[int]], slot_counts: Sequence[int],
                       chunk_len: Sequence[int]) -> List[int]:
        n = len(chunk_len)
        out = (C.c_int32 * max(n, 1))()
        self._check(self._lib.ifkv_reorder_chunks(self._ctx, n, _i32_array(order_in), _i32_array(slot_counts),
                                                  _i32_array(chunk_len), out))
        return [int(out[i]) for i in range(n)]

    def set_tuning(self, key: str, value: int) -> None:
        """Tuning / testing knob of include/ifkv_debug.h (host only)."""
        self._check(self._lib.ifkv_set_tuning(self._ctx, key.encode(), int(value)))

    def attention_plan(self, n_rows: int, n_kv: int) -> dict:
        """How recompute_attention would serve such a call (include/ifkv_debug.h; host only)."""
        out = (C.c_int64 * 5)()
        self._check(self._lib.ifkv_attention_plan(self._ctx, int(n_rows), int(n_kv), out))
        return dict(zip(("launches", "parts", "part_tiles", "partial_bytes", "scratch_bytes"), (int(x) for x in out)))

    def copy_bytes(self, dst: torch.Tensor, src: torch.Tensor) -> None:
        self._check(self._lib.ifkv_copy_bytes(self._ctx, _ptr(dst), _ptr(src), src.numel() * src.element_size()))

    def mfma_probe_sink_floats(self) -> int:
        return int(self._lib.ifkv_mfma_probe_sink_floats())

    def mfma_probe(self, pattern: int, iterations: int, sink: Optional[torch.Tensor] = None) -> float:
        """Launch the matrix-pipe calibration loop; returns the flops one launch performs."""
        need = self.mfma_probe_sink_floats()
        if sink is None:
            sink = torch.empty(need, dtype=torch.float32, device=self.device)
        if sink.dtype != torch.float32 or sink.numel() < need:
            raise ValueError(f"mfma_probe: sink must hold {need} float32")
        flops = C.c_double(0.0)
        self._check(self._lib.ifkv_mfma_probe(self._ctx, int(pattern), int(iterations), _ptr(sink), C.byref(flops)))
        return float(flops.value)
