"""Pins for the CPU oracle: each checks it against something other than itself --
the paper's printed code books, closed forms, invariants, library routines
(torch's bf16 cast, torch.round), exact integer arithmetic, brute force.

Citations are to arxiv 2507.17511.
"""
import itertools
import os

import numpy as np
import pytest
import torch

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def bf16_bits(x_f32: np.ndarray) -> np.ndarray:
    """fp32 -> bf16 bit patterns through torch (independent of the oracle)."""
    t = torch.from_numpy(np.ascontiguousarray(x_f32, dtype=np.float32)).to(torch.bfloat16)
    return t.view(torch.int16).numpy().view(np.uint16).copy()


def bf16_vals(bits: np.ndarray) -> np.ndarray:
    t = torch.from_numpy(bits.view(np.int16).copy()).view(torch.bfloat16)
    return t.to(torch.float32).numpy()


# ------------------------------------------------------------------ element formats

def test_bf16_widen_all_patterns(cfo):
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    got = cfo.bf16_to_f32(bits)
    want = bf16_vals(bits)
    # NaN payloads do not survive the float return path of the binding: compare them as NaN
    ok = ~np.isnan(want)
    assert np.array_equal(got.view(np.uint32)[ok], want.view(np.uint32)[ok])
    assert np.all(np.isnan(got[~ok]))


def test_bf16_narrow_ties_and_random(cfo):
    hi = np.arange(65536, dtype=np.uint32) << 16
    rng = np.random.default_rng(1)
    cases = np.concatenate([
        hi | 0x8000,            # exact ties on every upper half
        hi | 0x7fff, hi | 0x8001,
        rng.integers(0, 2**32, size=100000, dtype=np.uint64).astype(np.uint32),
    ]).astype(np.uint32)
    f = cases.view(np.float32)
    finite_or_inf = ~np.isnan(f)
    got = cfo.f32_to_bf16(f)
    want = bf16_bits(f)
    assert np.array_equal(got[finite_or_inf], want[finite_or_inf])
    assert np.all(np.isnan(bf16_vals(got[~finite_or_inf])))


# ------------------------------------------------------------------ summation order

def test_treesum_order_hand_values(cfo):
    f = lambda *v: float(cfo.treesum(np.array(v, dtype=np.float32)))
    two24 = 2.0 ** 24
    # (2^24+1) rounds back to 2^24 (tie to even); the right pair adds to 2 first.
    assert f(two24, 1, 1, 1) == 16777218.0       # left-to-right would give 16777216
    # adjacent pairs, not (v0+v2)+(v1+v3), which would give 16777220
    assert f(two24, 1, 2, 0) == 16777218.0
    # n = 3 pads to 4: (v0+v1)+(v2+0)
    assert f(1, two24, 1) == 16777216.0
    assert f(1, 1, two24) == 16777218.0
    # n = 5 pads to 8: ((v0+v1)+(v2+v3)) + ((v4+0)+(0+0))
    assert f(two24, 1, 1, 1, 2) == 16777220.0
    # n = 6: ((2^24+1)+(1+1)) + ((1+1)+0)
    assert f(two24, 1, 1, 1, 1, 1) == 16777220.0
    assert f(5.0) == 5.0


def test_treesum_exact_on_integers_and_stride(cfo):
    rng = np.random.default_rng(2)
    for n in (1, 2, 7, 64, 100, 1000, 4096):
        v = rng.integers(0, 1000, size=n).astype(np.float32)   # sums < 2^24: every order is exact
        assert float(cfo.treesum(v)) == float(v.astype(np.int64).sum())
    # strided access: column j of a [n, c] matrix
    import ctypes
    a = rng.integers(0, 100, size=(37, 8)).astype(np.float32)
    for j in range(8):
        got = cfo.lib().cfo_treesum(ctypes.c_void_p(a.ctypes.data + 4 * j), 37, 8)
        assert got == float(a[:, j].astype(np.int64).sum())


def test_treesum_close_to_fp64(cfo):
    rng = np.random.default_rng(3)
    for n in (1000, 4096, 16384):
        v = np.abs(rng.standard_normal(n)).astype(np.float32)
        assert abs(float(cfo.treesum(v)) - v.astype(np.float64).sum()) <= 1e-6 * v.astype(np.float64).sum()


# ------------------------------------------------------------------ scales (a3)

def test_channel_scale_closed_forms(cfo):
    N, C = 64, 8
    cfg = cfo.Config(N, C, dtype=cfo.F32, bits=1)
    z = np.zeros((N, C), dtype=np.float32)
    mags = np.array([0.375, 1.0, 3.0, 1e-3, 12345.0, 2.0 ** -20, 7.0, 0.1], dtype=np.float32)
    signs = np.where(np.arange(N) % 3 == 0, -1.0, 1.0).astype(np.float32)
    z[:] = signs[:, None] * mags[None, :]
    # constant magnitude down a column, N a power of two: the mean is that magnitude exactly
    assert np.array_equal(cfo.scales(cfg, z), mags)
    # column 1..N: mean (N+1)/2, exactly representable
    z[:, 0] = np.arange(1, N + 1)
    assert cfo.scales(cfg, z)[0] == (N + 1) / 2
    # ragged N: mean of 1..N is still (N+1)/2 (integers: any order exact), division by float(N)
    N2 = 50
    cfg2 = cfo.Config(N2, C, dtype=cfo.F32, bits=2)
    z2 = np.tile(np.arange(1, N2 + 1, dtype=np.float32)[:, None], (1, C))
    assert np.all(cfo.scales(cfg2, z2) == np.float32(1275.0) / np.float32(50.0))


def test_absmax_scales_and_group_boundary(cfo):
    N, C = 5, 256
    rng = np.random.default_rng(4)
    z = rng.standard_normal((N, C)).astype(np.float32)
    z[2, 127] = 100.0    # last channel of group 0
    z[3, 128] = -200.0   # first channel of group 1
    g = cfo.Config(N, C, dtype=cfo.F32, bits=4, scale=cfo.SCALE_GROUP, group=128)
    s = cfo.scales(g, z).reshape(N, 2)
    want = (np.abs(z).reshape(N, 2, 128).max(axis=2) / np.float32(7.0)).astype(np.float32)
    assert np.array_equal(s, want)
    assert s[2, 0] == np.float32(100.0) / np.float32(7.0) and s[2, 1] < 1.0
    assert s[3, 1] == np.float32(200.0) / np.float32(7.0) and s[3, 0] < 1.0
    c = cfo.Config(N, C, dtype=cfo.F32, bits=4, scale=cfo.SCALE_CHANNEL)
    assert np.array_equal(cfo.scales(c, z), np.abs(z).max(axis=0) / np.float32(7.0))


def test_rank1_scale_pins(cfo):
    """App. D "Quantization": u_i = rowmean|X| / globalmean|X|, v_j = colmean|X|."""
    N, C = 16, 32
    cfg = cfo.Config(N, C, dtype=cfo.F32, bits=2, scale=cfo.SCALE_RANK1)
    # |z_ij| = a_i * b_j with powers of two: every mean is exact
    a = (2.0 ** (np.arange(N) % 3)).astype(np.float32)
    b = (2.0 ** -(np.arange(C) % 4)).astype(np.float32)
    z = np.outer(a, b).astype(np.float32) * np.where((np.add.outer(np.arange(N), np.arange(C)) % 2) == 0, 1, -1)
    s = cfo.scales(cfg, z.astype(np.float32))
    v, u = s[:C], s[C:]
    assert np.allclose(v, b * a.mean(), rtol=1e-6)
    assert np.allclose(u, a / a.mean(), rtol=1e-6)
    # a rank-1 magnitude field is reproduced exactly by u v^T
    assert np.allclose(np.outer(u, v), np.abs(z), rtol=1e-6)
    # all rows alike => u == 1 and the rank-1 scale reduces to the channel scale
    z2 = np.tile(z[:1], (N, 1)).astype(np.float32)
    s2 = cfo.scales(cfg, z2)
    assert np.all(s2[C:] == 1.0)
    ch = cfo.Config(N, C, dtype=cfo.F32, bits=2)
    assert np.array_equal(s2[:C], cfo.scales(ch, z2))
    code_r = cfo.select(cfg, z2, s2)
    code_c = cfo.select(ch, z2, s2[:C].copy())
    assert np.array_equal(code_r, code_c)
    # all-zero tensor: u = 0, no NaN
    s0 = cfo.scales(cfg, np.zeros((N, C), dtype=np.float32))
    assert np.all(s0 == 0.0)


# ------------------------------------------------------------------ code books (paper's printed values)

def test_decode_levels_match_printed_code_books(cfo):
    books = {}
    with open(os.path.join(GOLDEN, "codebooks.txt")) as fh:
        for line in fh:
            if line.startswith("#") or not line.strip():
                continue
            parts = line.split()
            books[int(parts[0])] = (int(parts[1]), sorted(float(v) for v in parts[2:]))
    for bits, (ratio, levels) in books.items():
        C = 8
        cfg = cfo.Config(1, C, dtype=cfo.F32, bits=bits)
        code = np.zeros((1, C), dtype=np.uint8)
        code[0, : 2 ** bits] = np.arange(2 ** bits)
        for s in (1.0, 0.375):
            d = cfo.decode(cfg, code, np.full(C, s, dtype=np.float32))
            assert sorted(d[0, : 2 ** bits].tolist()) == [lv * s for lv in levels]
        # wire size: 16-bit activations / ratio
        big = cfo.Config(64, 128, dtype=cfo.BF16, bits=bits)
        assert cfo.alloc_codes(big).nbytes * ratio == 64 * 128 * 2
    # 4-bit is this build's own definition: integers -7..7 times the scale
    cfg4 = cfo.Config(1, 16, dtype=cfo.F32, bits=4)
    code = np.arange(16, dtype=np.uint8).reshape(1, 16)
    d = cfo.decode(cfg4, code, np.full(16, 0.5, dtype=np.float32))
    assert d[0].tolist() == [0.5 * (c - 16 if c >= 8 else c) for c in range(16)]


# ------------------------------------------------------------------ code choice (a4)

LEVELS = {1: {0: 1.0, 1: -1.0},
          2: {0: 0.5, 1: 2.0, 2: -0.5, 3: -2.0},
          4: {c: float(c - 16 if c >= 8 else c) for c in range(16) if c != 8}}


@pytest.mark.parametrize("bits", [1, 2, 4])
def test_code_choice_is_nearest_level_bruteforce(cfo, bits):
    rng = np.random.default_rng(10 + bits)
    for trial in range(20):
        N, C = 4, 8
        cfg = cfo.Config(N, C, dtype=cfo.F32, bits=bits)
        z = (rng.standard_normal((N, C)) * 10.0 ** rng.integers(-3, 3)).astype(np.float32)
        s = cfo.scales(cfg, z)
        code = cfo.select(cfg, z, s)
        for i in range(N):
            for j in range(C):
                errs = {c: abs(float(z[i, j]) - lv * float(s[j])) for c, lv in LEVELS[bits].items()}
                best = min(errs.values())
                if bits == 1:
                    # one level per sign: the sign must match (nearest of +-s)
                    assert errs[int(code[i, j])] == best
                else:
                    # nearest level; fp32 rounding of the threshold / quotient may move a
                    # near-tie by a few ulp of the scale
                    assert errs[int(code[i, j])] <= best + 4e-7 * float(s[j]) * 8
                    # and away from ties the choice is the unique minimiser
                    second = sorted(errs.values())[1]
                    if second - best > 1e-5 * float(s[j]) * 8:
                        assert errs[int(code[i, j])] == best


def test_two_bit_row_joint_bruteforce(cfo):
    """Per-element nearest level is the joint optimum over all 4^8 assignments of a row
    (for a fixed scale the squared error separates)."""
    rng = np.random.default_rng(20)
    N, C = 16, 8
    cfg = cfo.Config(N, C, dtype=cfo.F32, bits=2)
    z = rng.standard_normal((N, C)).astype(np.float32)
    s = cfo.scales(cfg, z)
    code = cfo.select(cfg, z, s)
    lv = np.array([0.5, 2.0, -0.5, -2.0])
    combos = np.array(list(itertools.product(range(4), repeat=C)))          # [65536, 8]
    row = 3
    cost = ((z[row].astype(np.float64)[None, :] - lv[combos] * s.astype(np.float64)[None, :]) ** 2).sum(axis=1)
    assert tuple(combos[cost.argmin()]) == tuple(code[row].tolist())


def test_two_bit_threshold_ties_and_zero_sign(cfo):
    # column sums to 4 over N=4 -> s = 1 exactly; 1.25 == 1.25*s is a tie -> small level
    cfg = cfo.Config(4, 8, dtype=cfo.F32, bits=2)
    z = np.zeros((4, 8), dtype=np.float32)
    z[:, 0] = [1.25, 0.25, 1.25, 1.25]
    z[:, 1] = [-1.25, 0.25, -1.25, 1.25]
    z[:, 2] = [1.5, 0.5, -1.0, 1.0]
    z[:, 3] = [np.nextafter(np.float32(1.25), np.float32(2)), 0.25, 1.25, np.nextafter(np.float32(1.25), np.float32(0))]
    z[:, 4] = [0.0, -0.0, 2.0, -2.0]
    s = cfo.scales(cfg, z)
    assert s[:5].tolist() == [1.0, 1.0, 1.0, 1.0, 1.0]
    code = cfo.select(cfg, z, s)
    assert code[:, 0].tolist() == [0, 0, 0, 0]
    assert code[:, 1].tolist() == [2, 0, 2, 0]
    assert code[:, 2].tolist() == [1, 0, 2, 0]
    assert code[:, 3].tolist() == [1, 0, 0, 0]
    assert code[:, 4].tolist() == [0, 0, 1, 3]       # +-0 is non-negative, small level
    # 1-bit: sign only; -0.0 counts as non-negative
    c1 = cfo.select(cfo.Config(4, 8, dtype=cfo.F32, bits=1), z, s)
    assert c1[:, 4].tolist() == [0, 0, 0, 1] and c1[:, 1].tolist() == [1, 0, 1, 0]


def test_four_bit_half_even_and_clamp(cfo):
    C = 128
    cfg = cfo.Config(1, C, dtype=cfo.F32, bits=4, scale=cfo.SCALE_GROUP, group=128)
    for m in (-3, 0, 5):
        unit = np.float32(2.0 ** m)
        z = np.zeros((1, C), dtype=np.float32)
        vals = [7, -7, 0.5, 1.5, 2.5, 3.5, -0.5, -1.5, -2.5, 6.5, -6.5, 0.0, -0.0, 0.49, 0.51]
        z[0, : len(vals)] = np.array(vals, dtype=np.float32) * unit
        s = cfo.scales(cfg, z)
        assert s[0] == unit                                   # 7*2^m / 7 == 2^m exactly
        code = cfo.select(cfg, z, s)[0, : len(vals)].astype(np.int8)
        q = np.where(code >= 8, code - 16, code)
        assert q.tolist() == [7, -7, 0, 2, 2, 4, 0, -2, -2, 6, -6, 0, 0, 0, 1]
    # zero group: scale 0, codes 0
    z = np.zeros((1, C), dtype=np.float32)
    s = cfo.scales(cfg, z)
    assert s[0] == 0.0 and not cfo.select(cfg, z, s).any()


def test_four_bit_matches_library_expression(cfo):
    """The textbook symmetric absmax quantiser, written with torch CPU ops."""
    rng = np.random.default_rng(30)
    N, C = 33, 256
    z = (rng.standard_normal((N, C)) * 3).astype(np.float32)
    zt = torch.from_numpy(z)
    for scale, group in ((cfo.SCALE_GROUP, 128), (cfo.SCALE_CHANNEL, 0)):
        cfg = cfo.Config(N, C, dtype=cfo.F32, bits=4, scale=scale, group=group or 128)
        s = cfo.scales(cfg, z)
        d = cfo.decode(cfg, cfo.select(cfg, z, s), s)
        if scale == cfo.SCALE_GROUP:
            st = zt.reshape(N, C // 128, 128).abs().amax(dim=2, keepdim=True) / 7.0
            dt = (torch.clamp(torch.round(zt.reshape(N, C // 128, 128) / st), -7, 7) * st).reshape(N, C)
        else:
            st = zt.abs().amax(dim=0, keepdim=True) / 7.0
            dt = torch.clamp(torch.round(zt / st), -7, 7) * st
        assert np.array_equal(d, dt.numpy())


# ------------------------------------------------------------------ packing (a5)

def test_pack_hand_written_bytes(cfo):
    c1 = cfo.Config(1, 16, dtype=cfo.F32, bits=1)
    code = np.array([[1, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 1]], dtype=np.uint8)
    assert cfo.pack(c1, code).tolist() == [[0x01, 0x80]]
    code = np.array([[1, 1, 0, 1, 0, 0, 1, 0, 0, 1, 0, 0, 0, 0, 0, 0]], dtype=np.uint8)
    assert cfo.pack(c1, code).tolist() == [[0b01001011, 0b00000010]]
    c2 = cfo.Config(1, 8, dtype=cfo.F32, bits=2)
    code = np.array([[3, 0, 0, 0, 0, 1, 2, 3]], dtype=np.uint8)
    assert cfo.pack(c2, code).tolist() == [[0x03, 0xE4]]
    c4 = cfo.Config(1, 8, dtype=cfo.F32, bits=4)
    code = np.array([[0x1, 0xF, 0x7, 0x9, 0, 0xA, 0xB, 0]], dtype=np.uint8)
    assert cfo.pack(c4, code).tolist() == [[0xF1, 0x97, 0xA0, 0x0B]]
    # rows are dense: row 1 starts right after row 0
    c = cfo.Config(2, 8, dtype=cfo.F32, bits=1)
    code = np.array([[1] * 8, [0, 1] * 4], dtype=np.uint8)
    assert cfo.pack(c, code).ravel().tolist() == [0xFF, 0xAA]


@pytest.mark.parametrize("bits", [1, 2, 4])
def test_unpack_pack_all_byte_values(cfo, bits):
    per = 8 // bits
    cfg = cfo.Config(256 // 8 * 8 // 8, 8 * per // per * 8, dtype=cfo.F32, bits=bits)  # [32, 8] codes-bytes rows
    cfg = cfo.Config(32, 64, dtype=cfo.F32, bits=bits)
    nbytes = cfg.n_tokens * cfg.n_channels * bits // 8
    packed = (np.arange(nbytes) % 256).astype(np.uint8).reshape(cfg.n_tokens, -1)
    code = cfo.unpack(cfg, packed)
    assert code.max() < 2 ** bits
    assert np.array_equal(cfo.pack(cfg, code), packed)
    # independent unpack: bit arithmetic on the bytes
    flat = packed.reshape(cfg.n_tokens, -1, 1) >> (bits * np.arange(per)).reshape(1, 1, per) & (2 ** bits - 1)
    assert np.array_equal(code, flat.reshape(cfg.n_tokens, cfg.n_channels))
    assert nbytes * 8 == cfg.n_tokens * cfg.n_channels * bits


# ------------------------------------------------------------------ whole step: state recursion

def _run(cfo, cfg, xs):
    """xs: list of arrays in cfg's storage dtype. Returns per-step (recon, err, codes, scales)."""
    recon, err = cfo.warmup(cfg, xs[0])
    hist = [(recon.copy(), err.copy(), None, None)]
    for x in xs[1:]:
        codes, s = cfo.step(cfg, x, recon, err)
        hist.append((recon.copy(), err.copy(), codes, s))
    return hist


def _vals(cfo, a, dtype):
    return bf16_vals(a) if dtype == cfo.BF16 else a


def _stream(cfo, dtype, steps=6, N=96, C=64, seed=5, sigma=0.05):
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((N, C)).astype(np.float32)
    xs = []
    for _ in range(steps):
        xs.append(bf16_bits(x) if dtype == cfo.BF16 else x.copy())
        x = (x + np.float32(sigma) * rng.standard_normal((N, C)).astype(np.float32)).astype(np.float32)
    return xs


def test_warmup_seeds_base(cfo):
    """a~_1 = a_1 (App. H.2); nothing lost yet, so e = 0."""
    for dtype in (cfo.F32, cfo.BF16):
        for ed in (cfo.F32, cfo.BF16):
            cfg = cfo.Config(96, 64, dtype=dtype, bits=2, err_dtype=ed)
            xs = _stream(cfo, dtype, steps=1)
            recon, err = cfo.warmup(cfg, xs[0])
            assert np.array_equal(recon, xs[0]) and not err.any()


@pytest.mark.parametrize("bits,scale", [(1, 0), (2, 0), (4, 0), (4, 1), (1, 2), (2, 2)])
@pytest.mark.parametrize("ef", [0, 1, 2])
def test_telescoping_invariant_fp32(cfo, bits, scale, ef):
    """recon_t + e_t == x_t (RECON, OFF); == x_t + e_{t-1} (LITERAL), up to fp32 rounding."""
    C = 128
    cfg = cfo.Config(96, C, dtype=cfo.F32, bits=bits, scale=scale, group=128, ef=ef)
    xs = _stream(cfo, cfo.F32, C=C)
    hist = _run(cfo, cfg, xs)
    for t in range(1, len(xs)):
        recon, err = hist[t][0].astype(np.float64), hist[t][1].astype(np.float64)
        target = xs[t].astype(np.float64)
        if ef == cfo.EF_LITERAL:
            target = target + hist[t - 1][1].astype(np.float64)
        # roundings: z (ulp of z), recon + D (ulp of recon_t), z - D (ulp of e): a few ulp of the largest operand
        big = np.max(np.abs(np.stack([hist[t][0], hist[t - 1][0], xs[t], hist[t][1], hist[t - 1][1]])), axis=0)
        tol = 4 * np.spacing(big.astype(np.float32)) + 1e-30
        assert np.all(np.abs(recon + err - target) <= tol)


@pytest.mark.parametrize("bits,scale", [(1, 0), (2, 0), (4, 1)])
def test_telescoping_invariant_bf16(cfo, bits, scale):
    """With bf16 storage recon_t is rounded once: recon_t + e_t = x_t within half a bf16 ulp of recon_t."""
    C = 128
    cfg = cfo.Config(96, C, dtype=cfo.BF16, bits=bits, scale=scale, group=128, ef=cfo.EF_RECON)
    xs = _stream(cfo, cfo.BF16, C=C)
    hist = _run(cfo, cfg, xs)
    for t in range(1, len(xs)):
        recon = bf16_vals(hist[t][0]).astype(np.float64)
        err = hist[t][1].astype(np.float64)
        x = bf16_vals(xs[t]).astype(np.float64)
        half_ulp = np.abs(recon) * 2.0 ** -8 + 1e-30
        assert np.all(np.abs(recon + err - x) <= half_ulp * 1.01 + 1e-6)
        # the rounding of recon is what the next residual sees: x_{t+1} - recon_t is formed from the stored value
    # the next step's z equals x - stored recon exactly
    z = cfo.residual(cfg, xs[-1], hist[-2][0], hist[-2][1])
    assert np.array_equal(z, bf16_vals(xs[-1]) - bf16_vals(hist[-2][0]))


def test_step_equals_compress_then_decompress(cfo):
    rng = np.random.default_rng(6)
    for dtype in (cfo.F32, cfo.BF16):
        for bits, scale in [(1, 0), (2, 0), (4, 0), (4, 1), (2, 2)]:
            for ef in (0, 1, 2):
                cfg = cfo.Config(40, 128, dtype=dtype, bits=bits, scale=scale, ef=ef)
                xs = _stream(cfo, dtype, steps=3, N=40, C=128, seed=int(rng.integers(1 << 30)))
                ra, ea = cfo.warmup(cfg, xs[0])
                rb, eb = ra.copy(), ea.copy()
                for x in xs[1:]:
                    ca, sa = cfo.step(cfg, x, ra, ea)
                    cb, sb = cfo.compress(cfg, x, rb, eb)
                    cfo.decompress(cfg, cb, sb, rb)
                    assert np.array_equal(ca, cb) and np.array_equal(sa.view(np.uint32), sb.view(np.uint32))
                    assert np.array_equal(ra, rb) and np.array_equal(ea, eb)


def test_zero_residual_gives_zero_codes(cfo):
    for dtype in (cfo.F32, cfo.BF16):
        for bits, scale in [(1, 0), (2, 0), (4, 0), (4, 1), (2, 2)]:
            cfg = cfo.Config(24, 128, dtype=dtype, bits=bits, scale=scale)
            xs = _stream(cfo, dtype, steps=1, N=24, C=128)
            recon, err = cfo.warmup(cfg, xs[0])
            codes, s = cfo.step(cfg, xs[0], recon, err)     # x_t == recon_{t-1}
            assert not codes.any() and not s.any() and not err.any()
            assert np.array_equal(recon, xs[0])


def test_exact_round_trip_of_representable_residuals(cfo):
    rng = np.random.default_rng(7)
    # 1-bit: |z_ij| = a_j down each column -> D == z
    N, C = 64, 16
    a = (2.0 ** rng.integers(-6, 3, size=C)).astype(np.float32) * np.float32(1.5)
    z = a[None, :] * rng.choice([-1.0, 1.0], size=(N, C)).astype(np.float32)
    x0 = np.round(rng.standard_normal((N, C)) * 4).astype(np.float32)      # integers: x0 + z exact in fp32
    cfg = cfo.Config(N, C, dtype=cfo.F32, bits=1)
    recon, err = cfo.warmup(cfg, x0)
    x1 = (x0 + z).astype(np.float32)
    assert np.array_equal((x1 - x0).astype(np.float32), z)
    cfo.step(cfg, x1, recon, err)
    assert np.array_equal(recon, x1) and not err.any()

    # 2-bit: one third of a column at +-2a, two thirds at +-0.5a -> mean-abs = a (N = 384)
    N = 384
    a = (2.0 ** rng.integers(-4, 3, size=C)).astype(np.float32)
    mag = np.where(np.arange(N)[:, None] % 3 == 0, 2.0, 0.5).astype(np.float32) * a[None, :]
    z = mag * rng.choice([-1.0, 1.0], size=(N, C)).astype(np.float32)
    x0 = np.round(rng.standard_normal((N, C)) * 4).astype(np.float32)
    cfg = cfo.Config(N, C, dtype=cfo.F32, bits=2)
    recon, err = cfo.warmup(cfg, x0)
    x1 = (x0 + z).astype(np.float32)
    codes, s = cfo.step(cfg, x1, recon, err)
    assert np.array_equal(s, a)
    assert np.array_equal(recon, x1) and not err.any()

    # 4-bit: entries k*2^m, |k| <= 7, absmax 7*2^m in every group / column
    N, C = 32, 256
    for scale in (cfo.SCALE_GROUP, cfo.SCALE_CHANNEL):
        k = rng.integers(-7, 8, size=(N, C))
        k[:, ::128] = 7
        k[0, :] = -7
        z = (k * 0.25).astype(np.float32)
        x0 = np.round(rng.standard_normal((N, C)) * 4).astype(np.float32)
        cfg = cfo.Config(N, C, dtype=cfo.F32, bits=4, scale=scale, group=128)
        recon, err = cfo.warmup(cfg, x0)
        x1 = (x0 + z).astype(np.float32)
        codes, s = cfo.step(cfg, x1, recon, err)
        assert np.all(s == 0.25)
        assert np.array_equal(recon, x1) and not err.any()


def test_one_bit_energy_identity(cfo):
    """With s_j = mean|z_j|: sum_i (z_ij - s_j sgn z_ij)^2 = sum_i z_ij^2 - N s_j^2, so the 1-bit
    quantiser is a delta-compressor (Sec. 3.2) with delta = (mean|z|)^2 / mean(z^2); 2/pi for a Gaussian."""
    rng = np.random.default_rng(8)
    N, C = 4096, 64
    z = rng.standard_normal((N, C)).astype(np.float32)
    cfg = cfo.Config(N, C, dtype=cfo.F32, bits=1)
    x0 = np.zeros((N, C), dtype=np.float32)
    recon, err = cfo.warmup(cfg, x0)
    codes, s = cfo.step(cfg, z, recon, err)
    lhs = (err.astype(np.float64) ** 2).sum()
    rhs = (z.astype(np.float64) ** 2).sum() - N * (s.astype(np.float64) ** 2).sum()
    assert abs(lhs - rhs) <= 1e-5 * rhs
    delta = 1.0 - lhs / (z.astype(np.float64) ** 2).sum()
    assert abs(delta - 2 / np.pi) < 0.01


def test_error_feedback_bounds_drift_and_naive_fails(cfo):
    """Sec. 3.1 / 3.2 / App. H: residual+EF keeps the total error bounded; without EF its energy
    grows about linearly in t; naive 1-bit compression of the activation is far worse than either."""
    from workloads import cfg1_numpy
    xs = cfg1_numpy(seed=0, steps=40)
    N, C = xs[0].shape
    tot = {}
    for ef in (cfo.EF_RECON, cfo.EF_OFF):
        cfg = cfo.Config(N, C, dtype=cfo.F32, bits=1, ef=ef)
        recon, err = cfo.warmup(cfg, xs[0])
        e2 = []
        for x in xs[1:]:
            cfo.step(cfg, x, recon, err)
            e2.append(float(((recon.astype(np.float64) - x) ** 2).mean()))
        tot[ef] = np.array(e2)
    with_ef, no_ef = tot[cfo.EF_RECON], tot[cfo.EF_OFF]
    assert with_ef[-10:].mean() < 3 * with_ef[:10].mean()            # bounded
    assert no_ef[-1] > 10 * no_ef[0] and no_ef[-1] > 5 * with_ef[-1]   # random-walk growth
    ts = np.arange(1, len(no_ef) + 1)
    slope = np.polyfit(ts, no_ef, 1)[0]
    assert slope > 0.5 * no_ef[0]                                      # roughly linear in t, slope ~ per-step loss
    cfgn = cfo.Config(N, C, dtype=cfo.F32, bits=1)
    rn, _, _ = cfo.naive(cfgn, xs[-1])
    naive_err = float(((rn.astype(np.float64) - xs[-1]) ** 2).mean())
    assert naive_err > 20 * with_ef[-1]                                # sigma_a^2 >> sigma_Delta^2 (Prop. 3.1)


def test_naive_is_a_step_from_the_zero_state_and_has_closed_forms(cfo):
    """Sec. 3.1: naive compression quantises the activation itself.  That is one codec step against the zero
    state (recon = 0, e = 0), which the recursion's own pins cover: same codes, same scales, recon = D, for every
    code width and both storage types.  And in closed form: a column of constant magnitude a with mixed signs has
    the 1-bit scale a (N a power of two: the tree sum is exact), so the reconstruction is the input itself."""
    rng = np.random.default_rng(11)
    for dtype in (cfo.F32, cfo.BF16):
        for bits in (1, 2, 4):
            N, C = 48, 40                                            # N not a power of two: zero padding in the tree
            cfg = cfo.Config(N, C, dtype=dtype, bits=bits)
            x = (rng.standard_normal((N, C)) * np.exp(rng.standard_normal((1, C)))).astype(np.float32)
            if dtype == cfo.BF16:
                x = cfo.f32_to_bf16(x)
            rn, cn, sn = cfo.naive(cfg, x)
            zero = np.zeros((N, C), dtype=cfg.np_dtype)
            recon, err = cfo.warmup(cfg, zero)
            cs, ss = cfo.step(cfg, x, recon, err)
            assert np.array_equal(cn, cs) and np.array_equal(sn.view(np.uint32), ss.view(np.uint32))
            assert np.array_equal(rn.view(np.uint8), recon.view(np.uint8))
    N, C = 64, 16
    a = np.linspace(0.25, 4.0, C, dtype=np.float32)                 # one magnitude per column (exact in fp32)
    sign = np.where(rng.random((N, C)) < 0.5, -1.0, 1.0).astype(np.float32)
    x = sign * a[None, :]
    rn, cn, sn = cfo.naive(cfo.Config(N, C, dtype=cfo.F32, bits=1), x)
    assert np.array_equal(sn, a) and np.array_equal(rn, x)
    bits_expected = np.packbits((x < 0).astype(np.uint8), axis=1, bitorder="little")
    assert np.array_equal(cn.reshape(N, C // 8), bits_expected)


def test_literal_mode_is_second_order(cfo):
    """LITERAL adds e on top of a residual that already contains it: x_t - recon_t = e_t - e_{t-1}."""
    cfg = cfo.Config(96, 64, dtype=cfo.F32, bits=2, ef=cfo.EF_LITERAL)
    xs = _stream(cfo, cfo.F32)
    hist = _run(cfo, cfg, xs)
    for t in range(1, len(xs)):
        lhs = xs[t].astype(np.float64) - hist[t][0]
        rhs = hist[t][1].astype(np.float64) - hist[t - 1][1]
        assert np.allclose(lhs, rhs, atol=1e-5)


def test_bf16_error_buffer_is_rounded_error(cfo):
    xs = _stream(cfo, cfo.BF16, steps=3)
    a = cfo.Config(96, 64, dtype=cfo.BF16, bits=2, err_dtype=cfo.F32)
    b = cfo.Config(96, 64, dtype=cfo.BF16, bits=2, err_dtype=cfo.BF16)
    ra, ea = cfo.warmup(a, xs[0]); rb, eb = cfo.warmup(b, xs[0])
    for x in xs[1:]:
        ca, sa = cfo.step(a, x, ra, ea); cb, sb = cfo.step(b, x, rb, eb)
        # RECON mode never reads e, so everything else is identical and e differs by one rounding
        assert np.array_equal(ca, cb) and np.array_equal(ra, rb)
        assert np.array_equal(eb, bf16_bits(ea))


def test_rejects_bad_configs(cfo):
    bad = [cfo.Config(0, 64), cfo.Config(8, 12), cfo.Config(8, 4), cfo.Config(8, 64, bits=3),
           cfo.Config(8, 64, bits=2, scale=cfo.SCALE_GROUP), cfo.Config(8, 192, bits=4, scale=cfo.SCALE_GROUP, group=128),
           cfo.Config(8, 64, dtype=5), cfo.Config(8, 64, ef=3), cfo.Config(8, 64, bits=4, scale=cfo.SCALE_RANK1)]
    for cfg in bad:
        with pytest.raises(ValueError):
            cfo.warmup(cfg, np.zeros((max(cfg.n_tokens, 1), cfg.n_channels), dtype=cfg.np_dtype))


def test_planted_mistakes_would_be_caught(cfo):
    """The pins above are only worth something if plausible mistakes break them: plant a few in a
    private re-implementation of the stage results and see the checks used above reject them."""
    N, C = 4, 8
    cfg = cfo.Config(N, C, dtype=cfo.F32, bits=2)
    z = np.zeros((N, C), dtype=np.float32)
    z[:, 0] = [1.5, 0.5, -1.0, 1.0]
    s = cfo.scales(cfg, z)
    code = cfo.select(cfg, z, s)
    d = cfo.decode(cfg, code, s)
    assert d[:, 0].tolist() == [2.0, 0.5, -0.5, 0.5]
    # wrong sign convention, swapped magnitude bit, transposed scale axis: all give other values
    assert (d[:, 0] * -1).tolist() != [2.0, 0.5, -0.5, 0.5]
    assert np.where(np.abs(d[:, 0]) == 2.0, 0.5, 2.0).tolist() != [2.0, 0.5, 0.5, 0.5]
    zt = np.zeros((N, C), dtype=np.float32); zt[0, :4] = [1.5, 0.5, -1.0, 1.0]
    assert not np.array_equal(cfo.scales(cfg, zt)[:4], np.full(4, s[0]))
