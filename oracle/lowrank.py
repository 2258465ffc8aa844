"""CPU oracle for the low-rank compressor of CompactFusion (arxiv 2507.17511).  TEST INFRASTRUCTURE ONLY:
nothing in the product path may import it.

What it computes, in fp64 with numpy, step by step as the paper states it:

  * Alg. 3 (App. D "Low-Rank Compression"), rank-r subspace iteration on the residual A [tokens, channels]:
    Q <- orthogonalize(Q0);  T times: Z <- A^T (A Q), Q <- orthogonalize(Z);  U <- A Q;  V <- Q.
  * The residual recursion around it (Sec. 3.1, 3.2; App. D "Residual Base and Error Feedback"):
    A = x_t - recon_{t-1},  D = U V^T,  e_t = A - D,  recon_t = recon_{t-1} + D.

Readings (the paper is silent or garbled on these):
  * The start matrix Q0 [channels, r] is an input: the caller draws it ("randomly sample Q").
  * orthogonalize = Gram-Schmidt in column order (what PowerSGD, which the paper adapts, uses).  A column whose
    remainder after projection is below 1e-4 of its own length carries no new direction and becomes zero, so a
    residual of rank < r yields zero columns instead of amplified rounding noise.
  * Alg. 3 as printed also orthonormalises U, which would drop the magnitudes from U V^T; U = A Q is kept
    un-normalised, so that U V^T = A Q Q^T is the orthogonal projection of A onto span(Q).
  * The factors travel in the storage dtype of the tensor (bf16: round to nearest even) and D is formed from the
    travelled values, so that sender and receiver add the same D and the rounding loss stays in e.
  * INT4 factors (Sec. 3.4 and App. D name them, no format is given): factor_bits = 4 sends every factor row of
    r entries as one fp32 scale s = absmax / 7 and nibbles q = clamp(rint(f / s), -7, 7) (round half to even,
    two's complement, entry k in byte k // 2, even k in the low nibble); D is formed from q * s.  Like everything
    else here the decision is taken in fp64, on the fp64 factor and the scale as it travels (absmax / 7 rounded
    once to fp32); an implementation that works in fp32 may decide a nibble the other way only where f / s lies
    within its own factor error of a half-integer, which is what its parity test has to show.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Tuple

import numpy as np

F32, BF16 = 0, 1
DROP = 1e-4


@dataclass(frozen=True)
class LowRankConfig:
    n_tokens: int
    n_channels: int
    dtype: int = BF16
    rank: int = 32
    iters: int = 1
    factor_bits: int = 0        # 0: factors in the storage dtype; 4: INT4 nibbles + one fp32 scale per factor row

    @property
    def np_dtype(self):
        return np.uint16 if self.dtype == BF16 else np.float32


def bf16_to_f64(h: np.ndarray) -> np.ndarray:
    return (h.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def rne_bf16(f: np.ndarray) -> np.ndarray:
    """fp64/fp32 values -> bf16 bit patterns: first to fp32 (nearest), then nearest-even on the 16 dropped bits."""
    u = np.ascontiguousarray(f, dtype=np.float32).view(np.uint32).astype(np.uint64)
    u = u + 0x7FFF + ((u >> 16) & 1)
    return (u >> 16).astype(np.uint16)


def widen(a: np.ndarray, dtype: int) -> np.ndarray:
    return bf16_to_f64(a) if dtype == BF16 else a.astype(np.float64)


def narrow(a: np.ndarray, dtype: int) -> np.ndarray:
    return rne_bf16(a) if dtype == BF16 else a.astype(np.float32)


def quantise_rows(F: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
    """INT4 factor rows: -> (nibble bytes uint8 [rows, r // 2], scales fp32 [rows])."""
    f = np.asarray(F, dtype=np.float64)
    s = (np.abs(f).max(axis=1) / 7.0).astype(np.float32)            # the scale travels as fp32
    safe = np.where(s == 0, 1.0, s.astype(np.float64))
    q = np.clip(np.rint(f / safe[:, None]), -7, 7).astype(np.int32)
    q[s == 0] = 0
    u = (q & 0xF).astype(np.uint8)
    return (u[:, 0::2] | (u[:, 1::2] << 4)).astype(np.uint8), s


def unpack_nibbles(nibbles: np.ndarray) -> np.ndarray:
    """-> int32 [rows, r]: the signed 4-bit integers."""
    b = np.asarray(nibbles, dtype=np.uint8)
    u = np.empty((b.shape[0], 2 * b.shape[1]), dtype=np.int32)
    u[:, 0::2] = b & 0xF
    u[:, 1::2] = b >> 4
    return np.where(u >= 8, u - 16, u)


def dequantise_rows(nibbles: np.ndarray, scales: np.ndarray) -> np.ndarray:
    """-> fp64 [rows, r]: q * s (exact in fp64: a 3-bit integer times an fp32 value)."""
    return unpack_nibbles(nibbles).astype(np.float64) * np.asarray(scales, dtype=np.float32).astype(np.float64)[:, None]


def factors_to_wire(cfg: LowRankConfig, F: np.ndarray):
    """A factor as it travels: storage-dtype array, or (nibbles, scales) for INT4."""
    return quantise_rows(F) if cfg.factor_bits == 4 else narrow(F, cfg.dtype)


def factors_from_wire(cfg: LowRankConfig, W, rows: int) -> np.ndarray:
    if cfg.factor_bits == 4:
        return dequantise_rows(W[0].reshape(rows, cfg.rank // 2), W[1].reshape(rows))
    return widen(W, cfg.dtype).reshape(rows, cfg.rank)


def orthogonalize(Z: np.ndarray) -> np.ndarray:
    """Gram-Schmidt over the columns, left to right (each column is projected twice, which in fp64 changes
    nothing beyond 1e-16 and keeps the loop free of cancellation)."""
    Z = np.array(Z, dtype=np.float64)
    Q = np.zeros_like(Z)
    for k in range(Z.shape[1]):
        v = Z[:, k].copy()
        start = np.sqrt(v @ v)
        for _ in range(2):
            v = v - Q[:, :k] @ (Q[:, :k].T @ v)
        left = np.sqrt(v @ v)
        if start > 0.0 and left > DROP * start:
            Q[:, k] = v / left
    return Q


def subspace_iteration(A: np.ndarray, Q0: np.ndarray, iters: int) -> Tuple[np.ndarray, np.ndarray]:
    """Alg. 3.  Returns U [tokens, r] = A Q and V [channels, r] = Q."""
    A = np.asarray(A, dtype=np.float64)
    Q = orthogonalize(Q0)
    for _ in range(iters):
        Z = A.T @ (A @ Q)
        Q = orthogonalize(Z)
    return A @ Q, Q


def compress(cfg: LowRankConfig, x: np.ndarray, recon: np.ndarray, q0: np.ndarray):
    """Sender half.  Returns (U_wire, V_wire, err fp32); recon is not touched."""
    A = widen(x, cfg.dtype).reshape(cfg.n_tokens, cfg.n_channels) - widen(recon, cfg.dtype).reshape(cfg.n_tokens, cfg.n_channels)
    U, V = subspace_iteration(A, np.asarray(q0, dtype=np.float64).reshape(cfg.n_channels, cfg.rank), cfg.iters)
    Uw, Vw = factors_to_wire(cfg, U), factors_to_wire(cfg, V)
    D = factors_from_wire(cfg, Uw, cfg.n_tokens) @ factors_from_wire(cfg, Vw, cfg.n_channels).T
    return Uw, Vw, (A - D).astype(np.float32)


def decode(cfg: LowRankConfig, Uw: np.ndarray, Vw: np.ndarray) -> np.ndarray:
    return factors_from_wire(cfg, Uw, cfg.n_tokens) @ factors_from_wire(cfg, Vw, cfg.n_channels).T


def decompress(cfg: LowRankConfig, Uw: np.ndarray, Vw: np.ndarray, recon: np.ndarray) -> np.ndarray:
    """Receiver half.  Returns the new reconstruction in the storage dtype."""
    return narrow(widen(recon, cfg.dtype).reshape(cfg.n_tokens, cfg.n_channels) + decode(cfg, Uw, Vw), cfg.dtype)


def step(cfg: LowRankConfig, x: np.ndarray, recon: np.ndarray, q0: np.ndarray):
    """One codec step.  Returns (U_wire, V_wire, err, new recon)."""
    Uw, Vw, err = compress(cfg, x, recon, q0)
    return Uw, Vw, err, decompress(cfg, Uw, Vw, recon)
