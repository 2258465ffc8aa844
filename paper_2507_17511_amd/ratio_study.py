"""Compression ratio against steady-state error for every compressor of the library, under the same residual /
error-feedback recursion (Sec. 3.1-3.3 and the "tunable ratios" claim of Sec. 1): 1-/2-/4-bit quantisers with
channel, rank-1 and group scales, the N:M block sparsifier and the rank-32 low-rank compressor.

All codec work runs in the HIP library; this module drives it over one synthetic stream and takes norms:

  ratio        = bytes of the activation / bytes on the wire (codes + scales, as cf_sizes reports them)
  total error  = mean (recon_t - x_t)^2 over the last quarter of the steps, relative to the mean square of the
                 step-to-step change of the stream (so "1.0" means: as wrong as not updating at all)

The stream is the stationary one of error_study (x_t = rho x_{t-1} + sqrt(1 - rho^2) n_t) with half of the change's
energy in a rank-16 part and half in full-rank noise.  With feedback on, a compressor that keeps a fraction delta of
the residual's energy settles near (1 - delta) / delta times the step-to-step change: the quantisers (delta 0.6 to
0.99) stay far below 1, while 32 directions of 512 or one value of eight cannot hold a mostly full-rank change and
end above it -- the "high-rank / low-rank mismatch" and the collapse of extreme sparsity that Sec. 3.3 describes.

Run:  python -m paper_2507_17511_amd.ratio_study [--tokens 1024] [--channels 1024] [--steps 28]
"""
from __future__ import annotations

import argparse
from typing import Dict, List, Tuple

import torch

import paper_2507_17511_amd as cf
from paper_2507_17511_amd.session import CodecSession

CODECS: List[Tuple[str, int, int, int]] = [        # name, bits, scale kind, group (a name ending in "INT4 factors" sets that flag)
    ("4-bit, group-128 scales", 4, cf.CF_SCALE_GROUP, 128),
    ("4-bit, channel scales", 4, cf.CF_SCALE_CHANNEL, 128),
    ("2-bit, channel scales", 2, cf.CF_SCALE_CHANNEL, 128),
    ("2-bit, rank-1 scales", 2, cf.CF_SCALE_RANK1, 128),
    ("1-bit, channel scales", 1, cf.CF_SCALE_CHANNEL, 128),
    ("1-bit, rank-1 scales", 1, cf.CF_SCALE_RANK1, 128),
    ("4 of 8 kept", 4, cf.CF_SPARSE_NM, 8),
    ("2 of 8 kept", 2, cf.CF_SPARSE_NM, 8),
    ("1 of 8 kept", 1, cf.CF_SPARSE_NM, 8),
    ("rank 32, T = 1", 1, cf.CF_LOWRANK, 32),
    ("rank 32, T = 2", 2, cf.CF_LOWRANK, 32),
    ("rank 32, T = 2, INT4 factors", 2, cf.CF_LOWRANK, 32),
]


def stream(n: int, c: int, steps: int, rho: float, seed: int, device: str):
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    x = torch.randn((n, c), generator=g, device=device)
    out = []
    for _ in range(steps):
        out.append(x.to(torch.bfloat16).contiguous())
        low = torch.randn((n, 16), generator=g, device=device) @ torch.randn((16, c), generator=g, device=device) / 4.0
        x = rho * x + (1.0 - rho * rho) ** 0.5 * (0.7 * torch.randn((n, c), generator=g, device=device) + 0.7 * low)
    return out


def run(n_tokens: int = 1024, n_channels: int = 1024, steps: int = 28, rho: float = 0.995, seed: int = 0,
        device: str = "cuda:0") -> Dict[str, Dict[str, float]]:
    xs = stream(n_tokens, n_channels, steps, rho, seed, device)
    change = sum(float((xs[t].double() - xs[t - 1].double()).pow(2).mean()) for t in range(1, steps)) / (steps - 1)
    g = torch.Generator(device=device)
    g.manual_seed(seed + 1)
    out = {}
    for name, bits, scale, group in CODECS:
        d = cf.desc(n_tokens, n_channels, cf.CF_BF16, bits, scale, group)
        opts = cf.options(flags=cf.CF_FLAG_LOWRANK_INT4 if name.endswith("INT4 factors") else 0)
        codes_bytes, scales_bytes, recon_bytes, _ = cf.cf_sizes(d, opts)
        wire = codes_bytes + (0 if scale == cf.CF_LOWRANK else scales_bytes)      # the low-rank start matrix does not travel
        sess = CodecSession([d], opts, device=device)
        errs = []
        try:
            sess.warmup([xs[0]])
            for t in range(1, steps):
                if scale == cf.CF_LOWRANK:
                    sess.scales[0].copy_(torch.randn(sess.scales[0].shape, generator=g, device=device))
                sess.step_fused([xs[t]])
                cf.cf_check_device(sess.ctx, sess.stream_handle)
                errs.append(float((sess.recon[0].double() - xs[t].double()).pow(2).mean()))
        finally:
            sess.close()
        tail = errs[-max(1, len(errs) // 4):]
        out[name] = {"ratio": recon_bytes / wire, "total_error": sum(tail) / len(tail) / change}
    return out


def main() -> None:
    ap = argparse.ArgumentParser(description=__doc__.split("\n\n")[0])
    ap.add_argument("--tokens", type=int, default=1024)
    ap.add_argument("--channels", type=int, default=1024)
    ap.add_argument("--steps", type=int, default=28)
    ap.add_argument("--rho", type=float, default=0.995)
    a = ap.parse_args()
    res = run(a.tokens, a.channels, a.steps, a.rho)
    print(f"[{a.tokens}, {a.channels}] bf16, {a.steps} steps, rho = {a.rho}; error relative to the stream's step-to-step change")
    print(f"{'compressor':<30} {'ratio':>8} {'total error':>12}")
    for name, r in res.items():
        print(f"{name:<30} {r['ratio']:>7.1f}x {r['total_error']:>12.4f}")


if __name__ == "__main__":
    main()
