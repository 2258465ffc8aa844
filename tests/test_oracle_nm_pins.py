"""Pins for the oracle's N:M block sparsifier (arxiv 2507.17511, Sec. 3.4 "Optimized Compression
Kernels" names it; block shape, tie rule and wire format are this build's reading, so nothing here
is a value the paper prints: parity is unpinned by the paper and pinned by mathematics instead).

What fixes the oracle: brute force over all subsets of a block, numpy's stable sort, hand-written
wire bytes, exact round trips, the top-k contraction bound (1 - N/M), the energy identity and the
telescoping invariant of the residual recursion.
"""
import itertools

import numpy as np
import pytest

from test_oracle_pins import _run, _stream, bf16_bits, bf16_vals

NM = [(1, 8), (2, 8), (4, 8), (2, 16), (4, 32)]


def nm_cfg(cfo, N, C, keep, block, dtype=None, **kw):
    return cfo.Config(N, C, dtype=cfo.F32 if dtype is None else dtype, bits=keep, scale=cfo.SPARSE_NM, group=block, **kw)


@pytest.mark.parametrize("keep,block", NM)
def test_kept_set_is_the_best_subset_bruteforce(cfo, keep, block):
    """Of all C(M, N) subsets of a block the kept one carries the most magnitude (continuous random
    values: no ties, the optimum is unique)."""
    if block > 16:
        pytest.skip("C(32, 4) subsets per block is left to the sort pin")
    rng = np.random.default_rng(keep * 100 + block)
    z = rng.standard_normal((6, 2 * block)).astype(np.float32)
    kept = cfo.nm_select(nm_cfg(cfo, 6, 2 * block, keep, block), z)
    for i in range(6):
        for b in range(2):
            blk = np.abs(z[i, b * block:(b + 1) * block]).astype(np.float64)
            best = max(itertools.combinations(range(block), keep), key=lambda s: blk[list(s)].sum())
            assert sorted(np.flatnonzero(kept[i, b * block:(b + 1) * block])) == sorted(best)


@pytest.mark.parametrize("keep,block", NM)
def test_kept_set_matches_stable_sort_with_ties(cfo, keep, block):
    """numpy's stable descending sort of |z| takes equal magnitudes in channel order: its first N
    entries are the kept set, also when most magnitudes tie (values drawn from {0, +-1, +-2})."""
    rng = np.random.default_rng(7)
    for z in (rng.standard_normal((16, 4 * block)).astype(np.float32),
              rng.integers(-2, 3, size=(16, 4 * block)).astype(np.float32)):
        kept = cfo.nm_select(nm_cfg(cfo, 16, 4 * block, keep, block), z)
        assert kept.reshape(16, 4, block).sum(axis=2).tolist() == [[keep] * 4] * 16
        for i in range(16):
            for b in range(4):
                blk = np.abs(z[i, b * block:(b + 1) * block])
                order = np.argsort(-blk, kind="stable")[:keep]
                assert sorted(np.flatnonzero(kept[i, b * block:(b + 1) * block])) == sorted(order)


def test_ties_zeros_and_non_finite(cfo):
    cfg = nm_cfg(cfo, 1, 8, 2, 8)
    sel = lambda *v: cfo.nm_select(cfg, np.array([v], dtype=np.float32))[0].tolist()
    assert sel(0, 0, 0, 0, 0, 0, 0, 0) == [1, 1, 0, 0, 0, 0, 0, 0]              # all equal: lowest channels
    assert sel(-0.0, 0, 0, 0, 0, 0, 0, -0.0) == [1, 1, 0, 0, 0, 0, 0, 0]        # -0 and +0 have equal magnitude
    assert sel(1, -1, 1, -1, 1, -1, 1, -1) == [1, 1, 0, 0, 0, 0, 0, 0]          # sign does not matter
    assert sel(1, 2, 3, -3, 2, 1, 0, 0) == [0, 0, 1, 1, 0, 0, 0, 0]
    assert sel(1, 2, 3, -3, 3, 1, 0, 0) == [0, 0, 1, 1, 0, 0, 0, 0]             # three-way tie: first two
    inf, nan = np.inf, np.nan
    assert sel(1, inf, 5, -inf, 2, 0, 0, 0) == [0, 1, 0, 1, 0, 0, 0, 0]
    assert sel(1, inf, 5, nan, 2, 0, 0, 0) == [0, 1, 0, 1, 0, 0, 0, 0]          # NaN orders above infinity
    assert sel(nan, inf, nan, nan, 2, 0, 0, 0)[:4] in ([1, 0, 1, 0], [1, 0, 0, 1], [0, 0, 1, 1])   # exactly two kept
    assert sum(sel(nan, nan, nan, nan, nan, nan, nan, nan)) == 2


def test_wire_hand_written_bytes(cfo):
    """One token, 16 channels, 2:8.  Block 0 keeps channels 1 and 6, block 1 keeps channels 8 and 15."""
    z = np.zeros((1, 16), dtype=np.float32)
    z[0, [1, 6, 8, 15]] = [1.5, -2.0, 0.25, -1.0]
    z[0, [2, 9]] = [0.125, -0.0625]                      # smaller: dropped
    for dtype in (cfo.F32, cfo.BF16):
        cfg = nm_cfg(cfo, 1, 16, 2, 8, dtype=dtype)
        wire = cfo.nm_pack(cfg, z, cfo.nm_select(cfg, z))
        off = cfo.nm_values_offset(cfg)
        assert off == 16                                  # 2 mask bytes, values start at the next multiple of 16
        assert wire[:2].tolist() == [0b01000010, 0b10000001] and not wire[2:16].any()
        if dtype == cfo.F32:
            assert wire.size == 16 + 4 * 4
            assert wire[off:].view(np.float32).tolist() == [1.5, -2.0, 0.25, -1.0]
        else:
            assert wire.size == 16 + 4 * 2
            assert wire[off:].view(np.uint16).tolist() == [0x3FC0, 0xC000, 0x3E80, 0xBF80]
        d = cfo.nm_unpack(cfg, wire)
        want = np.zeros((1, 16), dtype=np.float32)
        want[0, [1, 6, 8, 15]] = [1.5, -2.0, 0.25, -1.0]
        assert np.array_equal(d, want) and not np.signbit(d[0, 0])


def test_wire_sizes(cfo):
    """2:8 on 16-bit activations: a block of 16 bytes travels as 1 mask byte + 2 values = 5 bytes."""
    for (keep, block), dtype, per_block in (((2, 8), "BF16", 1 + 4), ((1, 8), "BF16", 1 + 2), ((4, 8), "F32", 1 + 16),
                                            ((2, 16), "BF16", 2 + 4), ((4, 32), "BF16", 4 + 8)):
        cfg = nm_cfg(cfo, 4096, 3072, keep, block, dtype=getattr(cfo, dtype))
        n_blocks = 4096 * 3072 // block
        assert cfo.codes_bytes(cfg) == n_blocks * per_block       # 4096 * 3072 / 8 mask bytes is a multiple of 16
        assert cfo.alloc_scales(cfg).size == 0
    assert cfo.nm_values_offset(nm_cfg(cfo, 3, 8, 1, 8)) == 16    # 3 mask bytes round up


@pytest.mark.parametrize("keep,block", NM)
def test_exact_round_trip_when_the_block_is_sparse_enough(cfo, keep, block):
    """Blocks with at most N non-zero residuals, representable in the storage dtype, pass unchanged:
    D == z, nothing is lost, and the reconstruction equals the input."""
    rng = np.random.default_rng(3)
    N, C = 32, 4 * block
    for dtype in (cfo.F32, cfo.BF16):
        x0 = rng.integers(-8, 9, size=(N, C)).astype(np.float32)
        delta = np.zeros((N, C), dtype=np.float32)
        for i in range(N):
            for b in range(C // block):
                where = rng.choice(block, size=rng.integers(0, keep + 1), replace=False)
                delta[i, b * block + where] = rng.integers(-4, 5, size=where.size) * 0.25
        x1 = x0 + delta
        enc = (lambda a: bf16_bits(a)) if dtype == cfo.BF16 else (lambda a: a.copy())
        cfg = nm_cfg(cfo, N, C, keep, block, dtype=dtype)
        hist = _run(cfo, cfg, [enc(x0), enc(x1)])
        recon, err = hist[1][0], hist[1][1]
        assert np.array_equal(recon, enc(x1)) and not err.any()
        assert np.array_equal(cfo.nm_unpack(cfg, hist[1][2]), delta)


@pytest.mark.parametrize("keep,block", NM)
def test_contraction_bound_and_energy_identity(cfo, keep, block):
    """Keeping the N largest of M loses at most a fraction 1 - N/M of the block's energy (the
    delta-compressor property of App. H with delta = N/M), and with fp32 values nothing is rounded,
    so ||z - D||^2 = ||z||^2 - ||D||^2 exactly up to fp64 summation."""
    rng = np.random.default_rng(11)
    N, C = 64, 8 * block
    z = (rng.standard_normal((N, C)) * np.exp(rng.standard_normal((N, C)))).astype(np.float32)
    cfg = nm_cfg(cfo, N, C, keep, block)
    d = cfo.nm_unpack(cfg, cfo.nm_pack(cfg, z, cfo.nm_select(cfg, z)))
    zb = z.astype(np.float64).reshape(N, C // block, block)
    db = d.astype(np.float64).reshape(N, C // block, block)
    lost = ((zb - db) ** 2).sum(axis=2)
    assert np.all(lost <= (1 - keep / block) * (zb ** 2).sum(axis=2) * (1 + 1e-12))
    assert np.allclose(lost, (zb ** 2).sum(axis=2) - (db ** 2).sum(axis=2), rtol=1e-9, atol=1e-12)
    assert np.all((db != 0).sum(axis=2) <= keep)


@pytest.mark.parametrize("ef", [0, 1, 2])
@pytest.mark.parametrize("keep,block", [(2, 8), (4, 32)])
def test_telescoping_invariant_fp32(cfo, keep, block, ef):
    C = 128
    cfg = nm_cfg(cfo, 96, C, keep, block, ef=ef)
    xs = _stream(cfo, cfo.F32, C=C)
    hist = _run(cfo, cfg, xs)
    for t in range(1, len(xs)):
        target = xs[t].astype(np.float64)
        if ef == cfo.EF_LITERAL:
            target = target + hist[t - 1][1].astype(np.float64)
        big = np.max(np.abs(np.stack([hist[t][0], hist[t - 1][0], xs[t], hist[t][1], hist[t - 1][1]])), axis=0)
        tol = 4 * np.spacing(big.astype(np.float32)) + 1e-30
        assert np.all(np.abs(hist[t][0].astype(np.float64) + hist[t][1].astype(np.float64) - target) <= tol)


def test_telescoping_invariant_bf16_and_split_equals_step(cfo):
    C = 128
    cfg = nm_cfg(cfo, 96, C, 2, 8, dtype=cfo.BF16)
    xs = _stream(cfo, cfo.BF16, C=C)
    hist = _run(cfo, cfg, xs)
    for t in range(1, len(xs)):
        recon = bf16_vals(hist[t][0]).astype(np.float64)
        gap = np.abs(recon + hist[t][1].astype(np.float64) - bf16_vals(xs[t]).astype(np.float64))
        assert np.all(gap <= np.abs(recon) * 2.0 ** -8 * 1.01 + 1e-6)
    # sender half then receiver half == one step
    recon, err = cfo.warmup(cfg, xs[0])
    for t in range(1, 4):
        wire, s = cfo.compress(cfg, xs[t], recon, err)
        cfo.decompress(cfg, wire, s, recon)
        assert np.array_equal(wire, hist[t][2]) and np.array_equal(recon, hist[t][0]) and np.array_equal(err, hist[t][1])


def test_error_feedback_reaches_every_coordinate(cfo):
    """Why sparsifiers need the feedback: without it a 1:8 sparsifier never updates a coordinate whose
    change stays below its block's maximum; with it the left-over grows until it is sent, so the
    total error stays bounded (Sec. 3.2), while it keeps growing without."""
    rng = np.random.default_rng(2)
    N, C, T = 64, 64, 40
    x = rng.standard_normal((N, C)).astype(np.float32)
    xs = [x.copy()]
    drift = (0.02 * (1 + np.arange(C) % 8)).astype(np.float32)       # channel 7 of each block always moves most
    for _ in range(T):
        x = (x + drift).astype(np.float32)
        xs.append(x.copy())
    err_ef = [float(np.abs(h[0] - xx).max()) for h, xx in zip(_run(cfo, nm_cfg(cfo, N, C, 1, 8, ef=cfo.EF_RECON), xs), xs)]
    err_no = [float(np.abs(h[0] - xx).max()) for h, xx in zip(_run(cfo, nm_cfg(cfo, N, C, 1, 8, ef=cfo.EF_OFF), xs), xs)]
    assert err_no[-1] > 0.9 * T * 0.02 * 7                             # channel 6 is never sent: error ~ T * drift
    assert max(err_ef) < 8 * 0.16 * 1.5                                # bounded by about a block's drift per round
    assert err_ef[-1] < err_no[-1] / 3


def test_rejects_bad_nm_configs(cfo):
    for keep, block, C in ((0, 8, 64), (8, 8, 64), (2, 12, 96), (2, 128, 256), (2, 16, 72)):
        with pytest.raises(ValueError):
            cfo.warmup(nm_cfg(cfo, 8, C, keep, block), np.zeros((8, C), dtype=np.float32))
