"""ctypes binding of libspan.so: same names as include/span.h, argument marshalling only.

Device buffers are torch tensors (PyTorch is used for device memory and streams only);
their data pointers are handed to the C ABI unchanged.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

# PyTorch owns the device memory handed to the library, so both must talk to ONE HIP
# runtime instance.  Importing torch first loads its bundled libamdhip64 (soname
# libamdhip64.so.7); libspan.so's dependency of that soname then binds to the copy already
# in the process instead of pulling a second runtime from /opt/rocm.
import torch  # noqa: F401

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libspan.so")

if not os.path.exists(LIB_PATH):
    raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2312_08361_amd.build` "
                      "(the HIP path has no fallback)")
lib = C.CDLL(LIB_PATH)

SPAN_MAX_CALL_SESSIONS = 64
SPAN_ARCH_LLAMA, SPAN_ARCH_BLOOM = 0, 1
SPAN_IO_BF16, SPAN_IO_F32 = 0, 1
(SPAN_OK, SPAN_E_INVALID, SPAN_E_BAD_SESSION, SPAN_E_CACHE_FULL, SPAN_E_TOO_LONG, SPAN_E_MIXED_SPANS,
 SPAN_E_DUPLICATE, SPAN_E_HIP, SPAN_E_TOO_MANY_TOKENS, SPAN_E_NOT_EMPTY, SPAN_E_NO_SLOT) = (
    0, -1, -2, -3, -4, -5, -6, -7, -8, -9, -10)


class span_config(C.Structure):
    _fields_ = [("arch", C.c_int32), ("n_blocks", C.c_int32), ("d_model", C.c_int32),
                ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32),
                ("d_ff", C.c_int32), ("norm_eps", C.c_float), ("rope_base", C.c_float),
                ("page_tokens", C.c_int32), ("max_pages", C.c_int32), ("max_sessions", C.c_int32),
                ("max_session_tokens", C.c_int32), ("max_batch_tokens", C.c_int32),
                ("io_dtype", C.c_int32), ("dry_run", C.c_int32), ("weight_bits", C.c_int32),
                ("levels", C.c_float * 16)]


WEIGHT_FIELDS = ["norm1_g", "norm1_b", "wq", "bq", "wk", "bk", "wv", "bv", "wo", "bo",
                 "norm2_g", "norm2_b", "w_gate", "w_up", "b_up", "w_down", "b_down"]


class span_block_weights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in WEIGHT_FIELDS]


EXPORTS = ["span_query_sizes", "span_create", "span_destroy", "span_session_open", "span_session_close",
           "span_session_length", "span_forward", "span_replay", "span_reorder", "span_hidden_encode",
           "span_hidden_decode", "span_train_sizes", "span_train_attach", "span_train_forward", "span_backward",
           "span_debug_free_pages",
           "span_debug_page_table", "span_debug_read_kv", "span_debug_tap", "span_debug_profile", "span_debug_profile_read", "span_debug_ceilings", "span_op_lowbit_scratch", "span_op_quantize",
           "span_op_linear_lowbit", "span_op_linear_scratch", "span_op_linear",
           "span_op_attn_decode_scratch", "span_op_attn_decode", "span_op_attn_decode_static", "span_last_error"]

_p = C.c_void_p
lib.span_query_sizes.argtypes = [C.POINTER(span_config), C.POINTER(C.c_size_t), C.POINTER(C.c_size_t), C.POINTER(C.c_size_t)]
lib.span_create.argtypes = [C.POINTER(span_config), C.POINTER(span_block_weights), _p, _p, _p, _p, C.POINTER(_p)]
lib.span_destroy.argtypes = [_p]
lib.span_session_open.argtypes = [_p, C.c_int, C.c_int, C.c_int, C.POINTER(C.c_int32)]
lib.span_session_close.argtypes = [_p, C.c_int32]
lib.span_session_length.argtypes = [_p, C.c_int32, C.POINTER(C.c_int)]
lib.span_forward.argtypes = [_p, C.c_int, C.POINTER(C.c_int32), C.POINTER(C.c_int), _p, _p, _p]
lib.span_replay.argtypes = [_p, C.c_int, C.POINTER(C.c_int32), C.POINTER(C.c_int), _p, _p, _p]
lib.span_reorder.argtypes = [_p, C.c_int, C.POINTER(C.c_int32), C.POINTER(C.c_int), _p]
lib.span_train_sizes.argtypes = [C.POINTER(span_config), C.c_int, C.POINTER(C.c_size_t), C.POINTER(C.c_size_t)]
lib.span_train_attach.argtypes = [_p, C.POINTER(span_block_weights), _p, _p, C.c_int, _p]
lib.span_train_forward.argtypes = [_p, C.c_int, C.c_int, C.c_int, C.POINTER(C.c_int), _p, _p, _p]
lib.span_backward.argtypes = [_p, C.c_int, C.c_int, C.c_int, C.POINTER(C.c_int), _p, _p, _p, _p, _p]
lib.span_debug_free_pages.argtypes = [_p, C.POINTER(C.c_int)]
lib.span_debug_page_table.argtypes = [_p, C.c_int32, C.POINTER(C.c_int32), C.POINTER(C.c_int)]
lib.span_debug_read_kv.argtypes = [_p, C.c_int32, C.c_int, C.c_int, C.c_int, _p, _p, _p]
lib.span_debug_tap.argtypes = [_p, C.c_int, C.c_int, C.c_int32, C.c_int, C.c_int, C.c_int, _p, C.c_size_t]
lib.span_debug_profile.argtypes = [_p, C.c_int]
lib.span_debug_profile_read.argtypes = [_p, C.c_int, C.POINTER(C.c_int), C.POINTER(C.c_float)]
lib.span_debug_ceilings.argtypes = [_p, C.c_size_t, _p, C.POINTER(C.c_float), C.POINTER(C.c_float), _p]
lib.span_hidden_encode.argtypes = [_p, C.c_int, C.c_int, C.c_int, C.c_int, C.POINTER(C.c_float), _p, _p, _p]
lib.span_hidden_decode.argtypes = [_p, _p, C.c_int, C.c_int, C.c_int, C.POINTER(C.c_float), C.c_int, _p, _p]
lib.span_op_lowbit_scratch.argtypes = [C.c_int, C.c_int, C.c_int]
lib.span_op_lowbit_scratch.restype = C.c_size_t
lib.span_op_quantize.argtypes = [_p, C.c_int, C.c_int, C.c_int, C.POINTER(C.c_float), _p, _p, _p, _p]
lib.span_op_linear_lowbit.argtypes = [_p, _p, _p, C.c_int, C.c_int, C.c_int, C.c_int, C.POINTER(C.c_float), _p, _p]
lib.span_op_linear_scratch.argtypes = [C.c_int, C.c_int, C.c_int]
lib.span_op_linear_scratch.restype = C.c_size_t
lib.span_op_linear.argtypes = [_p, _p, _p, C.c_int, C.c_int, C.c_int, C.c_int, _p, _p]
lib.span_op_attn_decode_scratch.argtypes = [C.c_int] * 5
lib.span_op_attn_decode_scratch.restype = C.c_size_t
lib.span_op_attn_decode.argtypes = [_p, _p, _p, C.POINTER(C.c_int), C.c_int, C.c_int, C.c_int, C.c_int, C.c_int,
                                    C.c_int, _p, _p, _p, _p]
lib.span_op_attn_decode_static.argtypes = [_p, _p, _p, C.POINTER(C.c_int), C.c_int, C.c_int, C.c_int, C.c_int, C.c_int,
                                           C.c_int, _p, _p, _p]
lib.span_last_error.restype = C.c_char_p
for _n in EXPORTS:
    if _n not in ("span_op_linear_scratch", "span_op_lowbit_scratch", "span_op_attn_decode_scratch", "span_last_error"):
        getattr(lib, _n).restype = C.c_int


class SpanError(RuntimeError):
    def __init__(self, code: int, message: str):
        super().__init__(f"span error {code}: {message}")
        self.code = code


def span_last_error() -> str:
    return lib.span_last_error().decode()


def _check(rc: int) -> None:
    if rc != 0:
        raise SpanError(rc, span_last_error())


def _ptr(t) -> Optional[int]:
    """Device (or host) pointer of a torch tensor, None -> NULL."""
    return None if t is None else t.data_ptr()


def _ints(values: Sequence[int], ctype=C.c_int):
    return (ctype * max(len(values), 1))(*values)


def make_config(**kw) -> span_config:
    cfg = span_config()
    cfg.page_tokens = 16
    for k, v in kw.items():
        if not hasattr(cfg, k):
            raise TypeError(f"span_config has no field {k}")
        if k == "levels":
            v = (C.c_float * 16)(*[float(a) for a in v])
        setattr(cfg, k, v)
    return cfg


def span_query_sizes(cfg: span_config):
    w, k, s = C.c_size_t(), C.c_size_t(), C.c_size_t()
    _check(lib.span_query_sizes(C.byref(cfg), C.byref(w), C.byref(k), C.byref(s)))
    return w.value, k.value, s.value


def span_create(cfg: span_config, weights, weight_arena, kv_arena, workspace, stream: int = 0) -> int:
    """weights: per block, a dict name -> torch bf16 device tensor (or None in dry-run)."""
    arr = None
    if weights is not None:
        arr = (span_block_weights * len(weights))()
        for b, w in enumerate(weights):
            for name in WEIGHT_FIELDS:
                setattr(arr[b], name, _ptr(w.get(name)))
    out = _p()
    _check(lib.span_create(C.byref(cfg), arr, _ptr(weight_arena), _ptr(kv_arena), _ptr(workspace), stream, C.byref(out)))
    return out.value


def span_destroy(span: int) -> None:
    _check(lib.span_destroy(span))


def span_session_open(span: int, first_block: int, n_blocks: int, max_len: int) -> int:
    out = C.c_int32()
    _check(lib.span_session_open(span, first_block, n_blocks, max_len, C.byref(out)))
    return out.value


def span_session_close(span: int, session: int) -> None:
    _check(lib.span_session_close(span, session))


def span_session_length(span: int, session: int) -> int:
    out = C.c_int()
    _check(lib.span_session_length(span, session, C.byref(out)))
    return out.value


def span_forward(span: int, sessions: Sequence[int], n_tokens: Sequence[int], x, y, stream: int = 0) -> None:
    _check(lib.span_forward(span, len(sessions), _ints(sessions, C.c_int32), _ints(n_tokens), _ptr(x), _ptr(y), stream))


def span_replay(span: int, sessions: Sequence[int], n_tokens: Sequence[int], x_past, y_all, stream: int = 0) -> None:
    _check(lib.span_replay(span, len(sessions), _ints(sessions, C.c_int32), _ints(n_tokens), _ptr(x_past), _ptr(y_all), stream))


def span_reorder(span: int, sessions: Sequence[int], hypo_ids: Sequence[int], stream: int = 0) -> None:
    _check(lib.span_reorder(span, len(sessions), _ints(sessions, C.c_int32), _ints(hypo_ids), stream))


def _weight_array(weights):
    arr = (span_block_weights * len(weights))()
    for b, w in enumerate(weights):
        for name in WEIGHT_FIELDS:
            setattr(arr[b], name, _ptr(w.get(name)))
    return arr


def span_train_sizes(cfg: span_config, max_tokens: int):
    w, s = C.c_size_t(), C.c_size_t()
    _check(lib.span_train_sizes(C.byref(cfg), max_tokens, C.byref(w), C.byref(s)))
    return w.value, s.value


def span_train_attach(span: int, weights, weight_t_arena, scratch, max_tokens: int, stream: int = 0) -> None:
    arr = None if weights is None else _weight_array(weights)
    _check(lib.span_train_attach(span, arr, _ptr(weight_t_arena), _ptr(scratch), max_tokens, stream))


def span_train_forward(span: int, first_block: int, n_blocks: int, lens: Sequence[int], x, y, stream: int = 0) -> None:
    _check(lib.span_train_forward(span, first_block, n_blocks, len(lens), _ints(lens), _ptr(x), _ptr(y), stream))


def span_backward(span: int, first_block: int, n_blocks: int, lens: Sequence[int], x, grad_y, grad_x, y_out=None,
                  stream: int = 0) -> None:
    _check(lib.span_backward(span, first_block, n_blocks, len(lens), _ints(lens), _ptr(x), _ptr(grad_y), _ptr(grad_x),
                             _ptr(y_out), stream))


def span_debug_free_pages(span: int) -> int:
    out = C.c_int()
    _check(lib.span_debug_free_pages(span, C.byref(out)))
    return out.value


def span_debug_page_table(span: int, session: int):
    n = C.c_int()
    _check(lib.span_debug_page_table(span, session, None, C.byref(n)))
    buf = (C.c_int32 * max(n.value, 1))()
    _check(lib.span_debug_page_table(span, session, buf, C.byref(n)))
    return list(buf[: n.value])


def span_debug_read_kv(span: int, session: int, block: int, pos0: int, n: int, k_out, v_out, stream: int = 0) -> None:
    _check(lib.span_debug_read_kv(span, session, block, pos0, n, _ptr(k_out), _ptr(v_out), stream))


(SPAN_K_NORM, SPAN_K_SKINNY, SPAN_K_TILED, SPAN_K_ATTN_DECODE, SPAN_K_ATTN_MERGE, SPAN_K_ATTN_PREFILL,
 SPAN_K_CLASSES) = range(7)


def span_debug_profile(span: int, enable: int) -> None:
    _check(lib.span_debug_profile(span, enable))


def span_debug_profile_read(span: int, kernel_class: int):
    """-> (number of launches, summed duration in ms) of one kernel class."""
    n, ms = C.c_int(), C.c_float()
    _check(lib.span_debug_profile_read(span, kernel_class, C.byref(n), C.byref(ms)))
    return n.value, ms.value


def _levels(levels):
    return None if levels is None else (C.c_float * 16)(*[float(a) for a in levels])


def span_debug_ceilings(buf, nbytes: int, out, stream: int = 0):
    r, m = C.c_float(), C.c_float()
    _check(lib.span_debug_ceilings(_ptr(buf), nbytes, _ptr(out), C.byref(r), C.byref(m), stream))
    return r.value, m.value


def _levels256(levels):
    return (C.c_float * 256)(*[float(a) for a in levels])


def span_hidden_encode(x, x_f32: int, M: int, d: int, block: int, levels, codes_out, absmax_out, stream: int = 0) -> None:
    _check(lib.span_hidden_encode(_ptr(x), x_f32, M, d, block, _levels256(levels), _ptr(codes_out), _ptr(absmax_out), stream))


def span_hidden_decode(codes, absmax, M: int, d: int, block: int, levels, y_f32: int, y, stream: int = 0) -> None:
    _check(lib.span_hidden_decode(_ptr(codes), _ptr(absmax), M, d, block, _levels256(levels), y_f32, _ptr(y), stream))


def span_op_lowbit_scratch(M: int, N: int, K: int) -> int:
    return lib.span_op_lowbit_scratch(M, N, K)


def span_op_quantize(w, N: int, K: int, bits: int, levels, codes_out, absmax_out, scratch, stream: int = 0) -> None:
    _check(lib.span_op_quantize(_ptr(w), N, K, bits, _levels(levels), _ptr(codes_out), _ptr(absmax_out), _ptr(scratch), stream))


def span_op_linear_lowbit(x, w, y, M: int, N: int, K: int, bits: int, levels, scratch, stream: int = 0) -> None:
    _check(lib.span_op_linear_lowbit(_ptr(x), _ptr(w), _ptr(y), M, N, K, bits, _levels(levels), _ptr(scratch), stream))


def span_op_linear_scratch(M: int, N: int, K: int) -> int:
    return lib.span_op_linear_scratch(M, N, K)


def span_op_linear(x, w, y, M: int, N: int, K: int, path: int, scratch, stream: int = 0) -> None:
    _check(lib.span_op_linear(_ptr(x), _ptr(w), _ptr(y), M, N, K, path, _ptr(scratch), stream))


def span_op_attn_decode_scratch(B: int, L_max: int, Hq: int, Hkv: int, hd: int) -> int:
    return lib.span_op_attn_decode_scratch(B, L_max, Hq, Hkv, hd)


def span_op_attn_decode(q, k, v, lens: Sequence[int], B: int, L_max: int, Hq: int, Hkv: int, hd: int,
                        alibi: int, out, logits, scratch, stream: int = 0) -> None:
    _check(lib.span_op_attn_decode(_ptr(q), _ptr(k), _ptr(v), _ints(lens), B, L_max, Hq, Hkv, hd, alibi,
                                   _ptr(out), _ptr(logits), _ptr(scratch), stream))


def span_op_attn_decode_static(q, k, v, lens: Sequence[int], B: int, L_max: int, Hq: int, Hkv: int, hd: int,
                               alibi: int, out, logits, stream: int = 0) -> None:
    _check(lib.span_op_attn_decode_static(_ptr(q), _ptr(k), _ptr(v), _ints(lens), B, L_max, Hq, Hkv, hd, alibi,
                                          _ptr(out), _ptr(logits), stream))


TAP_Q_ROT, TAP_K_ROT, TAP_LOGITS = 1, 2, 3


def span_debug_tap(span, what: int, block: int, session: int, head: int, q0: int, nq: int, out, out_bytes: int) -> None:
    _check(lib.span_debug_tap(span, what, block, session, head, q0, nq, _ptr(out), out_bytes))
