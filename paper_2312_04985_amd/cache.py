"""Device buffers of one decode cache and convenience wrappers over the binding.

Allocation and bookkeeping only (torch owns the memory); all work is done by libsparq.
"""
from __future__ import annotations

from typing import Optional

import torch

from . import binding as B


class DecodeCache:
    """K, Kt, V, v_mean, seq_lens and the workspace for one (B, H, H_kv, S_max, d_h) cache."""

    def __init__(self, Bsz: int, H: int, H_kv: int, S_max: int, d_h: int, r: int, k: int, dtype,
                 device="cuda", flags: int = 0, poison: Optional[float] = None):
        if S_max % 64:
            raise ValueError("S_max must be a multiple of 64")
        self.B, self.H, self.H_kv, self.S_max, self.d_h, self.r, self.k = Bsz, H, H_kv, S_max, d_h, r, k
        self.dtype, self.device = dtype, torch.device(device)
        self.shape = B.make_shape(Bsz, H, H_kv, S_max, d_h, r, k, dtype, flags)
        mk = torch.zeros if poison is None else (lambda *a, **kw: torch.full(*a, fill_value=poison, **kw))
        self.tiled = bool(flags & B.SPARQ_FLAG_TILED_K)
        if self.tiled:
            # one key copy in tiles of 8 positions (channel-major inside a tile) + the rows that wait for their tile
            self.K = mk((Bsz, H_kv, S_max // 8, d_h, 8), dtype=dtype, device=self.device)
            self.Kt = mk((Bsz, H_kv, 8, d_h), dtype=dtype, device=self.device)
        else:
            self.K = mk((Bsz, H_kv, S_max, d_h), dtype=dtype, device=self.device)
            # with SPARQ_FLAG_SINGLE_K at construction there is no second key copy at all
            self.Kt = None if flags & B.SPARQ_FLAG_SINGLE_K else mk((Bsz, H_kv, d_h, S_max), dtype=dtype, device=self.device)
        self.V = mk((Bsz, H_kv, S_max, d_h), dtype=dtype, device=self.device)
        self.v_mean = torch.zeros((Bsz, H_kv, d_h), dtype=torch.float32, device=self.device)
        self.seq_lens = torch.zeros((Bsz,), dtype=torch.int32, device=self.device)
        self.workspace = torch.zeros((B.sparq_workspace_bytes(self.shape),), dtype=torch.uint8, device=self.device)
        B.sparq_workspace_init(self.workspace)
        self.cache = B.make_cache(self.K, self.Kt, self.V, self.v_mean, self.seq_lens)
        self._v_mean_alt = None      # second (v_mean, seq_lens) pair for the one-launch step, made on first use
        self._seq_lens_alt = None

    def with_params(self, r: int, k: int, flags: int = 0, local_window: int = 0, S_bound: int = 0):
        """The same buffers seen through another (r, k, flags, local window, bound on the lengths) setting."""
        self.r, self.k = r, k
        self.shape = B.make_shape(self.B, self.H, self.H_kv, self.S_max, self.d_h, r, k, self.dtype, flags, local_window, S_bound)
        need = B.sparq_workspace_bytes(self.shape)          # the plan, and with it the scratch size, may change
        if need > self.workspace.numel():
            self.workspace = torch.zeros((need,), dtype=torch.uint8, device=self.device)
            B.sparq_workspace_init(self.workspace)
        return self

    def with_bound(self, S_bound: int):
        """Promise that no sequence is (or, in a step, becomes) longer than S_bound, a multiple of 64 (0: S_max): kernels
        and workspace are then chosen for that length instead of the buffers' S_max."""
        return self.with_params(self.r, self.k, self.shape.flags, self.shape.local_window, S_bound)

    def append(self, k_new: torch.Tensor, v_new: torch.Tensor, n_new_per_seq: Optional[torch.Tensor] = None, stream=None):
        """k_new, v_new: [B, H_kv, n_new, d_h] (or [B, H_kv, d_h] for one row)."""
        n_new = 1 if k_new.dim() == 3 else k_new.shape[2]
        B.sparq_kv_append(self.shape, self.cache, k_new, v_new, n_new, n_new_per_seq, self.workspace, stream)

    def decode(self, q: torch.Tensor, k_per_seq: Optional[torch.Tensor] = None, aux: bool = False,
               idx_stride: Optional[int] = None, out: Optional[torch.Tensor] = None, stream=None):
        out = torch.empty((self.B, self.H, self.d_h), dtype=self.dtype, device=self.device) if out is None else out
        if not aux:
            B.sparq_decode(self.shape, self.cache, q, k_per_seq, out, None, None, None, self.workspace, stream)
            return out
        stride = idx_stride if idx_stride is not None else min(self.k, self.S_max)
        alpha = torch.empty((self.B, self.H), dtype=torch.float32, device=self.device)
        idx = torch.empty((self.B, self.H, stride), dtype=torch.int32, device=self.device)
        chan = torch.empty((self.B, self.H, self.r), dtype=torch.int32, device=self.device)
        B.sparq_decode(self.shape, self.cache, q, k_per_seq, out, alpha, idx, chan, self.workspace, stream)
        return out, alpha, idx, chan

    def step(self, k_new: torch.Tensor, v_new: torch.Tensor, q: torch.Tensor, k_per_seq: Optional[torch.Tensor] = None,
             aux: bool = False, idx_stride: Optional[int] = None, out: Optional[torch.Tensor] = None, stream=None):
        """Append one row and decode in one launch (sparq_decode_step); the (v_mean, seq_lens) pair that
        the call wrote becomes the current one."""
        if self._v_mean_alt is None:
            self._v_mean_alt = torch.empty_like(self.v_mean)
            self._seq_lens_alt = torch.empty_like(self.seq_lens)
        out = torch.empty((self.B, self.H, self.d_h), dtype=self.dtype, device=self.device) if out is None else out
        alpha = idx = chan = None
        if aux:
            stride = idx_stride if idx_stride is not None else min(self.k, self.S_max)
            alpha = torch.empty((self.B, self.H), dtype=torch.float32, device=self.device)
            idx = torch.empty((self.B, self.H, stride), dtype=torch.int32, device=self.device)
            chan = torch.empty((self.B, self.H, self.r), dtype=torch.int32, device=self.device)
        B.sparq_decode_step(self.shape, self.cache, k_new, v_new, self._v_mean_alt, self._seq_lens_alt, q, k_per_seq,
                            out, alpha, idx, chan, self.workspace, stream)
        self.v_mean, self._v_mean_alt = self._v_mean_alt, self.v_mean
        self.seq_lens, self._seq_lens_alt = self._seq_lens_alt, self.seq_lens
        self.cache = B.make_cache(self.K, self.Kt, self.V, self.v_mean, self.seq_lens)
        return (out, alpha, idx, chan) if aux else out

    def dense(self, q: torch.Tensor, out: Optional[torch.Tensor] = None, stream=None):
        out = torch.empty((self.B, self.H, self.d_h), dtype=self.dtype, device=self.device) if out is None else out
        B.dense_decode(self.shape, self.cache, q, out, self.workspace, stream)
        return out

    def key_rows(self) -> torch.Tensor:
        """The cached keys as rows [B, H_kv, S_max, d_h], whatever the layout (a copy for the tiled layout: tiles
        un-tiled, the rows still waiting for their tile taken from the small buffer; bookkeeping for tests)."""
        if not self.tiled:
            return self.K
        rows = self.K.permute(0, 1, 2, 4, 3).reshape(self.B, self.H_kv, self.S_max, self.d_h).clone()
        lens = self.seq_lens.cpu().tolist()
        for b, s in enumerate(lens):
            fl = s & ~7
            if s > fl:
                rows[b, :, fl:s] = self.Kt[b, :, :s - fl]
        return rows

    def error_flags(self) -> int:
        return B.sparq_async_error(self.workspace)
