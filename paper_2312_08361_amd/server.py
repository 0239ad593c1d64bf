"""Device-memory plumbing around the C ABI: allocates the three arenas as torch tensors,
uploads seeded weights, and keeps them alive.  No arithmetic of the method lives here."""
from __future__ import annotations

from typing import Dict, Optional, Sequence

import numpy as np
import torch

from . import binding as B


def config_for(shape, *, max_pages: int, max_sessions: int, max_session_tokens: int,
               max_batch_tokens: int, io_f32: bool = True, dry_run: bool = False, weight_bits: int = 0,
               levels=None) -> B.span_config:
    extra = {} if levels is None else {"levels": levels}
    return B.make_config(weight_bits=weight_bits, **extra, arch=B.SPAN_ARCH_LLAMA if shape.arch == "llama" else B.SPAN_ARCH_BLOOM,
                         n_blocks=shape.n_blocks, d_model=shape.d_model, n_q_heads=shape.n_q_heads,
                         n_kv_heads=shape.n_kv_heads, head_dim=shape.head_dim, d_ff=shape.d_ff,
                         norm_eps=shape.norm_eps, rope_base=shape.rope_base, max_pages=max_pages,
                         max_sessions=max_sessions, max_session_tokens=max_session_tokens,
                         max_batch_tokens=max_batch_tokens, io_dtype=B.SPAN_IO_F32 if io_f32 else B.SPAN_IO_BF16,
                         dry_run=int(dry_run))


def bf16_tensor_from_bits(bits: np.ndarray, device) -> torch.Tensor:
    """uint16 bf16 bit patterns (numpy) -> torch bf16 tensor on `device`, bits unchanged."""
    t = torch.from_numpy(bits.view(np.int16)).to(device)
    return t.view(torch.bfloat16)


def to_bf16(a: np.ndarray, device) -> torch.Tensor:
    """fp32 numpy -> torch bf16 on `device` (torch's cast rounds to nearest even; values that are
    bf16-representable already, as every seeded input is, pass unchanged)."""
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(device).to(torch.bfloat16)


class SpanServer:
    """Owns the arenas of one span_t.  `weights` is a workloads.SpanWeights (or any
    sequence of {name: fp32 ndarray holding bf16-representable values})."""

    def __init__(self, cfg: B.span_config, weights: Optional[Sequence[Dict[str, np.ndarray]]], device="cuda:0",
                 keep_canonical: bool = False):
        self.cfg = cfg
        self.device = torch.device(device)
        wb, kb, sb = B.span_query_sizes(cfg)
        self.sizes = (wb, kb, sb)
        self.stream = 0
        if cfg.dry_run:
            self.span = B.span_create(cfg, None, None, None, None)
            return
        self.weight_arena = torch.empty(wb, dtype=torch.uint8, device=self.device)
        self.kv_arena = torch.empty(kb, dtype=torch.uint8, device=self.device)
        self.workspace = torch.empty(sb, dtype=torch.uint8, device=self.device)
        self.stream = torch.cuda.current_stream(self.device).cuda_stream
        # Upload and pack block by block so that the canonical copies can be freed early.
        self.span = None
        canon = []
        for b in range(cfg.n_blocks):
            wd = weights[b]
            up = (lambda a: torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(self.device)) \
                if cfg.weight_bits == 32 else (lambda a: to_bf16(a, self.device))
            canon.append({k: (v if isinstance(v, torch.Tensor) else up(v)) for k, v in wd.items()})
        self.span = B.span_create(cfg, canon, self.weight_arena, self.kv_arena, self.workspace, self.stream)
        torch.cuda.synchronize(self.device)
        self.canonical = canon if keep_canonical else None

    def open(self, max_len: int, first_block: int = 0, n_blocks: Optional[int] = None) -> int:
        n_blocks = self.cfg.n_blocks - first_block if n_blocks is None else n_blocks
        return B.span_session_open(self.span, first_block, n_blocks, max_len)

    def close(self, session: int) -> None:
        B.span_session_close(self.span, session)

    def _io(self, x_np: np.ndarray) -> torch.Tensor:
        if self.cfg.io_dtype == B.SPAN_IO_F32:
            return torch.from_numpy(np.ascontiguousarray(x_np, dtype=np.float32)).to(self.device)
        return to_bf16(x_np, self.device)

    def forward(self, sessions, n_tokens, x, replay: bool = False) -> torch.Tensor:
        """x: numpy [sum T, d] (uploaded) or a device tensor of the io dtype.  Returns y (device)."""
        xt = self._io(x) if isinstance(x, np.ndarray) else x
        y = torch.empty_like(xt)
        fn = B.span_replay if replay else B.span_forward
        fn(self.span, sessions, n_tokens, xt, y, self.stream)
        return y

    def attach_training(self, max_tokens: int) -> None:
        """Allocates and binds the arenas of the training-time passes (needs keep_canonical=True)."""
        compressed = self.cfg.weight_bits in (8, 4)
        if not compressed and getattr(self, "canonical", None) is None:
            raise RuntimeError("create the server with keep_canonical=True to attach training")
        wt, sc = B.span_train_sizes(self.cfg, max_tokens)
        self.train_sizes = (wt, sc)
        self.weight_t_arena = None if compressed else torch.empty(wt, dtype=torch.uint8, device=self.device)
        self.train_scratch = torch.empty(sc, dtype=torch.uint8, device=self.device)
        B.span_train_attach(self.span, None if compressed else self.canonical, self.weight_t_arena, self.train_scratch,
                            max_tokens, self.stream)
        torch.cuda.synchronize(self.device)

    def train_forward(self, lens, x, first_block: int = 0, n_blocks: Optional[int] = None) -> torch.Tensor:
        n_blocks = self.cfg.n_blocks - first_block if n_blocks is None else n_blocks
        xt = self._io(x) if isinstance(x, np.ndarray) else x
        y = torch.empty_like(xt)
        B.span_train_forward(self.span, first_block, n_blocks, lens, xt, y, self.stream)
        return y

    def backward(self, lens, x, grad_y, first_block: int = 0, n_blocks: Optional[int] = None, want_y: bool = False):
        """Returns grad_x (and y when want_y), device tensors of the io dtype."""
        n_blocks = self.cfg.n_blocks - first_block if n_blocks is None else n_blocks
        xt = self._io(x) if isinstance(x, np.ndarray) else x
        gt = self._io(grad_y) if isinstance(grad_y, np.ndarray) else grad_y
        gx = torch.empty_like(xt)
        y = torch.empty_like(xt) if want_y else None
        B.span_backward(self.span, first_block, n_blocks, lens, xt, gt, gx, y, self.stream)
        return (gx, y) if want_y else gx

    def reorder(self, sessions, hypo_ids) -> None:
        B.span_reorder(self.span, sessions, hypo_ids, self.stream)

    def read_kv(self, session: int, block: int, pos0: int, n: int):
        shp = (n, self.cfg.n_kv_heads, self.cfg.head_dim)
        dt = torch.float32 if self.cfg.weight_bits == 32 else torch.bfloat16
        k = torch.empty(shp, dtype=dt, device=self.device)
        v = torch.empty(shp, dtype=dt, device=self.device)
        B.span_debug_read_kv(self.span, session, block, pos0, n, k, v, self.stream)
        return k, v

    def destroy(self) -> None:
        if getattr(self, "span", None):
            B.span_destroy(self.span)
            self.span = None

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass
