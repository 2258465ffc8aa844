"""Shared plumbing of the GPU parity tests: runs the HIP library and the CPU oracle
side by side on the same tensors and compares every output.

Tolerances (the build's stated bar): packed codes bit-exact; scales,
reconstructions and error buffers within 1e-6 relative in fp32 and within 1 bf16
ulp where stored as bf16.  Because both sides evaluate the same fp32 expression
tree with one rounding per operation, the comparison also demands bit equality
and reports the tolerance figures if that ever fails.
"""
from __future__ import annotations

from concurrent.futures import ThreadPoolExecutor
from typing import List, Optional, Sequence

import numpy as np
import torch

import oracle
import paper_2507_17511_amd as cf
from paper_2507_17511_amd.session import CodecSession
from workloads import as_numpy

REL_TOL_F32 = 1e-6
BF16_ULP_TOL = 1


def oracle_config(d: cf.cf_tensor_desc, opts: cf.cf_options) -> oracle.Config:
    # naive compression is a function of its own in the oracle, not an error-feedback mode
    ef = 0 if opts.ef == cf.CF_EF_NAIVE else int(opts.ef)
    return oracle.Config(int(d.n_tokens), int(d.n_channels), dtype=int(d.dtype), bits=int(d.bits), scale=int(d.scale),
                         group=int(d.group) if d.scale in (cf.CF_SCALE_GROUP, cf.CF_SPARSE_NM) else 128, ef=ef,
                         err_dtype=int(opts.err_dtype))


def bf16_to_f32(bits: np.ndarray) -> np.ndarray:
    return (bits.astype(np.uint32) << 16).view(np.float32)


def assert_same(name: str, got: np.ndarray, want: np.ndarray, kind: str):
    """kind: 'bytes' (bit-exact integers), 'f32', 'bf16' (uint16 patterns)."""
    got = np.ascontiguousarray(got).reshape(-1)
    want = np.ascontiguousarray(want).reshape(-1)
    assert got.shape == want.shape, f"{name}: shape {got.shape} vs {want.shape}"
    if kind == "bytes":
        bad = np.flatnonzero(got != want)
        assert bad.size == 0, f"{name}: {bad.size} of {got.size} bytes differ, first at {bad[:5]}"
        return
    if kind == "f32":
        gb, wb = got.view(np.uint32), want.view(np.uint32)
        if np.array_equal(gb, wb):
            return
        g, w = got.astype(np.float64), want.astype(np.float64)
        rel = np.abs(g - w) / np.maximum(np.abs(w), 1e-30)
        within = bool(np.all((rel <= REL_TOL_F32) | (np.abs(g - w) <= 1e-30)))
        bad = np.flatnonzero(gb != wb)
        raise AssertionError(f"{name}: {bad.size} of {got.size} fp32 values differ in bits (max rel {rel.max():.3e}; "
                             f"within the 1e-6 tolerance: {within}), first at {bad[:5]}: got {got[bad[:3]]}, want {want[bad[:3]]}")
    if kind == "bf16":
        if np.array_equal(got, want):
            return
        # ulp distance on the ordered integer line of bf16 patterns
        def key(b):
            b = b.astype(np.int32)
            return np.where(b & 0x8000, 0x8000 - (b & 0x7fff), 0x8000 + b)
        dist = np.abs(key(got) - key(want))
        bad = np.flatnonzero(got != want)
        raise AssertionError(f"{name}: {bad.size} of {got.size} bf16 values differ (max {dist.max()} ulp; "
                             f"within the 1-ulp tolerance: {bool(dist.max() <= BF16_ULP_TOL)}), first at {bad[:5]}")
    raise ValueError(kind)


def kind_of(dtype: int) -> str:
    return "bf16" if dtype == cf.CF_BF16 else "f32"


class OracleState:
    """The oracle's copy of the state of a set of tensors."""

    def __init__(self, descs: Sequence[cf.cf_tensor_desc], opts: cf.cf_options, which: Optional[Sequence[int]] = None):
        self.descs = list(descs)
        self.opts = opts
        self.which = list(range(len(self.descs))) if which is None else list(which)
        self.cfg = {t: oracle_config(self.descs[t], opts) for t in self.which}
        self.recon = {}
        self.err = {}
        self.codes = {}
        self.scales = {}

    def warmup(self, t: int, x0: np.ndarray):
        self.recon[t], self.err[t] = oracle.warmup(self.cfg[t], x0)

    def step(self, t: int, x: np.ndarray):
        if self.opts.ef == cf.CF_EF_NAIVE:
            # Sec. 3.1's baseline: recon_t = D(C(x_t)).  The library also reports e_t = x_t - D; the
            # oracle's stages give D, and one fp32 subtraction gives what e must hold.
            cfg = self.cfg[t]
            self.recon[t], self.codes[t], self.scales[t] = oracle.naive(cfg, x)
            if cfg.scale == oracle.SPARSE_NM:
                dec = oracle.nm_unpack(cfg, self.codes[t])
            else:
                dec = oracle.decode(cfg, oracle.unpack(cfg, self.codes[t]), self.scales[t])
            xf = bf16_to_f32(x) if cfg.dtype == oracle.BF16 else x       # widening is exact: a 16-bit shift
            lost = (xf.reshape(cfg.shape).astype(np.float32) - dec).astype(np.float32)
            self.err[t] = oracle.f32_to_bf16(lost) if cfg.err_dtype == oracle.BF16 else lost
            return
        self.codes[t], self.scales[t] = oracle.step(self.cfg[t], x, self.recon[t], self.err[t])


def compare_tensor(tag: str, sess: CodecSession, orc: OracleState, t: int, check_codes: bool = True):
    d = sess.descs[t]
    if check_codes:
        got = as_numpy(sess.codes[t])
        if d.scale == cf.CF_SPARSE_NM:      # the bytes between the masks and the 16-byte aligned values are unspecified
            got = got.copy().reshape(-1)
            n_mask = int(d.n_tokens) * int(d.n_channels) // 8
            got[n_mask:(n_mask + 15) // 16 * 16] = 0
        assert_same(f"{tag} codes[{t}]", got, orc.codes[t], "bytes")
        assert_same(f"{tag} scales[{t}]", as_numpy(sess.scales[t]), orc.scales[t], "f32")
    assert_same(f"{tag} recon[{t}]", as_numpy(sess.recon[t]), orc.recon[t], kind_of(d.dtype))
    assert_same(f"{tag} err[{t}]", as_numpy(sess.err[t]), orc.err[t], kind_of(sess.opts.err_dtype))


def run_parity(descs, opts, xs_per_step: List[List[torch.Tensor]], mode: str = "fused", device="cuda:0",
               which: Optional[Sequence[int]] = None, threads: int = 8, tag: str = ""):
    """xs_per_step[s][t]: device tensor of tensor t at step s (step 0 = warm-up).
    mode: 'fused' | 'split' (cf_compress then cf_decompress).  Compares after every step."""
    sess = CodecSession(descs, opts, device=device)
    orc = OracleState(descs, opts, which)
    try:
        sess.warmup(xs_per_step[0])
        torch.cuda.synchronize()
        with ThreadPoolExecutor(max_workers=threads) as pool:
            list(pool.map(lambda t: orc.warmup(t, as_numpy(xs_per_step[0][t])), orc.which))
            for t in orc.which:
                compare_tensor(f"{tag} warm-up", sess, orc, t, check_codes=False)
            for s in range(1, len(xs_per_step)):
                if mode == "fused":
                    sess.step_fused(xs_per_step[s])
                else:
                    sess.compress(xs_per_step[s])
                    sess.decompress()
                cf.cf_check_device(sess.ctx, sess.stream_handle)     # synchronises; raises if a bounded wait expired
                list(pool.map(lambda t: orc.step(t, as_numpy(xs_per_step[s][t])), orc.which))
                for t in orc.which:
                    compare_tensor(f"{tag} step {s}", sess, orc, t)
    finally:
        sess.close()
    return sess, orc


def drift_stream(shape, dtype: int, steps: int, seed: int, sigma: float = 0.05, device="cuda:0") -> List[torch.Tensor]:
    """x_0 ~ N(0,1), x_t = x_{t-1} + sigma N(0,1), in the codec's storage dtype."""
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    x = torch.randn(shape, generator=g, device=device, dtype=torch.float32)
    out = []
    for _ in range(steps):
        out.append(x.to(torch.bfloat16).contiguous() if dtype == cf.CF_BF16 else x.clone())
        x = x + sigma * torch.randn(shape, generator=g, device=device, dtype=torch.float32)
    return out
