"""Device-memory plumbing around the C entry points: allocates the state, code,
scale and workspace buffers of a batch of layer tensors with torch and keeps the
host pointer arrays.  No codec arithmetic happens here."""
from __future__ import annotations

from typing import List, Optional, Sequence

import torch

import paper_2507_17511_amd as cf

_TORCH_DT = {cf.CF_F32: torch.float32, cf.CF_BF16: torch.bfloat16}


class CodecSession:
    def __init__(self, descs: Sequence[cf.cf_tensor_desc], opts: Optional[cf.cf_options] = None,
                 device: str | torch.device = "cuda:0", stream: Optional[torch.cuda.Stream] = None):
        self.descs = list(descs)
        self.opts = opts if opts is not None else cf.options()
        self.device = torch.device(device)
        self.n = len(self.descs)
        self.recon: List[torch.Tensor] = []
        self.err: List[torch.Tensor] = []
        self.codes: List[torch.Tensor] = []
        self.scales: List[torch.Tensor] = []
        for d in self.descs:
            cb, sb, _, _ = cf.cf_sizes(d, self.opts)
            shape = (d.n_tokens, d.n_channels)
            self.recon.append(torch.empty(shape, dtype=_TORCH_DT[d.dtype], device=self.device))
            self.err.append(torch.empty(shape, dtype=_TORCH_DT[self.opts.err_dtype], device=self.device))
            codes_shape = (cb,) if d.scale in (cf.CF_SPARSE_NM, cf.CF_LOWRANK) else (d.n_tokens, cb // d.n_tokens)   # two arrays in one buffer
            self.codes.append(torch.empty(codes_shape, dtype=torch.uint8, device=self.device))
            self.scales.append(torch.empty(sb // 4, dtype=torch.float32, device=self.device))
        self.ws_bytes = cf.cf_workspace_bytes(self.descs, self.opts)
        if self.ws_bytes == 0:
            raise cf.CFError(cf.CF_ERR_UNSUPPORTED, "cf_workspace_bytes")
        self.workspace = torch.empty(self.ws_bytes, dtype=torch.uint8, device=self.device)
        assert self.workspace.data_ptr() % 256 == 0
        self._stream = stream
        with torch.cuda.device(self.device):
            self.ctx = cf.cf_init(self.descs, self.opts, self.workspace, self.ws_bytes, self.stream_handle)
        self.p_recon = cf.ptr_array(self.recon)
        self.p_err = cf.ptr_array(self.err)
        self.p_codes = cf.ptr_array(self.codes)
        self.p_scales = cf.ptr_array(self.scales)

    @property
    def stream_handle(self) -> int:
        s = self._stream if self._stream is not None else torch.cuda.current_stream(self.device)
        return s.cuda_stream

    def _slice(self, arr, first, count):
        if first == 0 and count == self.n:
            return arr
        return cf.ptr_array([arr[k] for k in range(first, first + count)])

    def _x(self, x, count):
        if len(x) != count:
            raise ValueError(f"expected {count} x tensors, got {len(x)}")
        return x if not isinstance(x, (list, tuple)) else cf.ptr_array(x)

    def warmup(self, x0, first: int = 0, count: Optional[int] = None) -> None:
        count = self.n - first if count is None else count
        cf.cf_warmup(self.ctx, first, count, self._x(x0, count), self._slice(self.p_recon, first, count),
                     self._slice(self.p_err, first, count), self.stream_handle)

    def step_fused(self, x, first: int = 0, count: Optional[int] = None) -> None:
        count = self.n - first if count is None else count
        cf.cf_step_fused(self.ctx, first, count, self._x(x, count), self._slice(self.p_recon, first, count),
                         self._slice(self.p_err, first, count), self._slice(self.p_codes, first, count),
                         self._slice(self.p_scales, first, count), self.stream_handle)

    def compress(self, x, first: int = 0, count: Optional[int] = None) -> None:
        count = self.n - first if count is None else count
        cf.cf_compress(self.ctx, first, count, self._x(x, count), self._slice(self.p_recon, first, count),
                       self._slice(self.p_err, first, count), self._slice(self.p_codes, first, count),
                       self._slice(self.p_scales, first, count), self.stream_handle)

    def decompress(self, first: int = 0, count: Optional[int] = None, recon=None) -> None:
        count = self.n - first if count is None else count
        p_recon = self._slice(self.p_recon, first, count) if recon is None else cf.ptr_array(recon)
        cf.cf_decompress(self.ctx, first, count, self._slice(self.p_codes, first, count),
                         self._slice(self.p_scales, first, count), p_recon, self.stream_handle)

    def close(self) -> None:
        if self.ctx is not None:
            torch.cuda.synchronize(self.device)
            cf.cf_destroy(self.ctx)
            self.ctx = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
