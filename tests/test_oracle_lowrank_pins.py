"""Pins for the low-rank oracle (arxiv 2507.17511, Alg. 3 and App. D "Low-Rank Compression").  Nothing the paper
prints fixes numbers for it, so it is pinned by linear algebra: numpy's QR and SVD, exact recovery of matrices of
rank <= r, the projection identities, Eckart-Young optimality, and the invariant of the residual recursion.
Parity with the paper itself is unpinned (Alg. 3 as printed normalises U; see the oracle's header)."""
import numpy as np
import pytest
import torch

from oracle import lowrank as lr


def rand_lowrank(rng, n, c, rank, noise=0.0, decay=None):
    s = np.ones(rank) if decay is None else decay ** np.arange(rank)
    a = (rng.standard_normal((n, rank)) * s) @ rng.standard_normal((rank, c))
    return a + noise * rng.standard_normal((n, c))


def test_bf16_rounding_matches_torch():
    rng = np.random.default_rng(0)
    f = np.concatenate([rng.standard_normal(100000) * np.exp(rng.standard_normal(100000) * 8),
                        (np.arange(65536, dtype=np.uint32) << 16 | 0x8000).view(np.float32)[:0x7F80].astype(np.float64)])
    want = torch.from_numpy(f.astype(np.float32)).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(lr.rne_bf16(f), want)
    assert np.array_equal(lr.bf16_to_f64(want), torch.from_numpy(want.view(np.int16).copy()).view(torch.bfloat16).double().numpy())


def test_orthogonalize_is_gram_schmidt():
    rng = np.random.default_rng(1)
    Z = rng.standard_normal((200, 32)) * np.exp(rng.standard_normal(32))
    Q = lr.orthogonalize(Z)
    assert np.allclose(Q.T @ Q, np.eye(32), atol=1e-12)
    Qn, R = np.linalg.qr(Z)                                  # library QR: same Q up to the sign that makes diag(R) > 0
    assert np.allclose(Q, Qn * np.sign(np.diag(R)), atol=1e-10)
    # column k lies in the span of the first k + 1 input columns: Q^T Z is upper triangular with a positive diagonal
    Rm = Q.T @ Z
    assert np.allclose(np.tril(Rm, -1), 0, atol=1e-9) and np.all(np.diag(Rm) > 0)


def test_orthogonalize_drops_dependent_columns():
    rng = np.random.default_rng(2)
    Z = rng.standard_normal((64, 8))
    Z[:, 3] = 2 * Z[:, 0] - Z[:, 2]                          # dependent on earlier columns
    Z[:, 6] = 0.0
    Q = lr.orthogonalize(Z)
    assert not Q[:, 3].any() and not Q[:, 6].any()
    keep = [0, 1, 2, 4, 5, 7]
    assert np.allclose(Q[:, keep].T @ Q[:, keep], np.eye(6), atol=1e-12)
    assert np.linalg.matrix_rank(np.concatenate([Q[:, keep], Z], axis=1)) == 6       # same span


@pytest.mark.parametrize("rank_a", [1, 5, 32])
def test_exact_recovery_of_matrices_of_rank_at_most_r(rank_a):
    """One iteration suffices: range(A^T A Q0) = range(A^T) when rank(A) <= r, and projecting A onto it is A."""
    rng = np.random.default_rng(3)
    A = rand_lowrank(rng, 96, 128, rank_a)
    U, V = lr.subspace_iteration(A, rng.standard_normal((128, 32)), 1)
    assert np.allclose(U @ V.T, A, atol=1e-9 * np.abs(A).max())
    assert np.count_nonzero(np.abs(V).sum(axis=0)) == rank_a                          # the other columns were dropped


def test_projection_identities():
    rng = np.random.default_rng(4)
    A = rng.standard_normal((150, 96)) * np.exp(rng.standard_normal((1, 96)))
    for T in (0, 1, 3):
        U, V = lr.subspace_iteration(A, rng.standard_normal((96, 32)), T)
        D = U @ V.T
        assert np.allclose(V.T @ V, np.eye(32), atol=1e-12)
        assert np.allclose(U, A @ V, atol=1e-12)
        assert np.allclose(D, A @ V @ V.T, atol=1e-10)
        assert np.isclose((A ** 2).sum(), (D ** 2).sum() + ((A - D) ** 2).sum(), rtol=1e-12)      # Pythagoras
        assert np.allclose((A - D) @ V, 0, atol=1e-9)                                            # what is lost is orthogonal to V


def test_error_against_the_svd_optimum():
    """Eckart-Young: no rank-32 approximation beats the truncated SVD; subspace iteration approaches it as T grows."""
    rng = np.random.default_rng(5)
    n, c, r = 160, 128, 32
    Ua, _ = np.linalg.qr(rng.standard_normal((n, c)))
    Va, _ = np.linalg.qr(rng.standard_normal((c, c)))
    sv = 0.9 ** np.arange(c)
    A = (Ua * sv) @ Va.T
    best = np.sqrt((sv[r:] ** 2).sum())
    Q0 = rng.standard_normal((c, r))
    errs = []
    for T in (0, 1, 2, 4, 16):
        U, V = lr.subspace_iteration(A, Q0, T)
        errs.append(np.linalg.norm(A - U @ V.T))
    assert all(e >= best * (1 - 1e-12) for e in errs)
    assert all(b <= a * (1 + 1e-12) for a, b in zip(errs, errs[1:]))                  # more iterations never hurt here
    assert errs[0] > 2 * best and errs[-1] < 1.02 * best
    # dominant direction: with a clear gap the first column of V is the top right singular vector
    A1 = 10 * np.outer(Ua[:, 0], Va[:, 0]) + 0.01 * rng.standard_normal((n, c))
    _, V1 = lr.subspace_iteration(A1, Q0, 2)
    assert abs(V1[:, 0] @ Va[:, 0]) > 0.9999


@pytest.mark.parametrize("dtype", [lr.F32, lr.BF16])
def test_step_wiring_and_invariant(dtype):
    rng = np.random.default_rng(6)
    n, c = 96, 128
    cfg = lr.LowRankConfig(n, c, dtype=dtype, rank=32, iters=1)
    enc = (lambda a: lr.rne_bf16(a)) if dtype == lr.BF16 else (lambda a: a.astype(np.float32))
    x0 = rng.standard_normal((n, c))
    recon = enc(x0)
    x = x0
    for t in range(4):
        x = x + 0.05 * rand_lowrank(rng, n, c, 48)
        xs = enc(x)
        q0 = rng.standard_normal((c, 32)).astype(np.float32)
        Uw, Vw, err, new = lr.step(cfg, xs, recon, q0)
        Uc, Vc, errc = lr.compress(cfg, xs, recon, q0)
        assert np.array_equal(Uw, Uc) and np.array_equal(Vw, Vc) and np.array_equal(err, errc)
        assert np.array_equal(lr.decompress(cfg, Uw, Vw, recon), new)
        gap = np.abs(lr.widen(new, dtype) + err - lr.widen(xs, dtype))
        bound = np.abs(lr.widen(new, dtype)) * (2.0 ** -8 if dtype == lr.BF16 else 2.0 ** -23) * 1.01 + 1e-6
        assert np.all(gap <= bound)                            # recon_t + e_t = x_t up to the one rounding of recon_t
        # what was sent is rank <= 32 and the residual shrank
        A = lr.widen(xs, dtype) - lr.widen(recon, dtype)
        assert np.linalg.matrix_rank(lr.decode(cfg, Uw, Vw)) <= 32
        assert np.linalg.norm(err) < np.linalg.norm(A)
        recon = new


# ---------------------------------------------------------------- INT4 factors (Sec. 3.4 / App. D name them; format: the oracle's header)

def test_int4_factor_rows_round_trip_exactly_when_representable():
    """Rows whose entries are k * 2^m, |k| <= 7, with absmax 7 * 2^m: the scale is 2^m and nothing is lost."""
    rng = np.random.default_rng(20)
    k = rng.integers(-7, 8, size=(50, 32))
    k[:, 0] = 7 * rng.choice([-1, 1], size=50)
    m = rng.integers(-6, 7, size=(50, 1))
    f = k * 2.0 ** m
    nib, s = lr.quantise_rows(f)
    assert np.array_equal(s, (2.0 ** m[:, 0]).astype(np.float32))
    assert np.array_equal(lr.dequantise_rows(nib, s), f)


def test_int4_factor_bytes_by_hand():
    """Entry k sits in byte k // 2, even k in the low nibble, two's complement."""
    f = np.zeros((1, 32))
    f[0, :6] = [7, -7, 1, -1, 3, -8]          # -8 clamps to -7
    f[0, 31] = 2
    f[0, 0] = 7                                # absmax would be 8: put it back to 7 for a scale of 1
    f[0, 5] = -7
    nib, s = lr.quantise_rows(f)
    assert s[0] == np.float32(1.0)
    assert list(nib[0, :3]) == [0x97, 0xF1, 0x93] and nib[0, 15] == 0x20 and not nib[0, 3:15].any()


def test_int4_zero_row_and_error_bound_and_textbook_expression():
    rng = np.random.default_rng(21)
    f = rng.standard_normal((300, 32)) * np.exp(rng.standard_normal((300, 1)) * 3)
    f[7] = 0.0
    nib, s = lr.quantise_rows(f)
    assert s[7] == 0 and not nib[7].any()
    back = lr.dequantise_rows(nib, s)
    assert np.all(np.abs(back - f) <= 0.5 * s[:, None].astype(np.float64) * (1 + 1e-6))
    # the symmetric absmax quantiser as a library expression (torch.round rounds half to even), in fp64 on the
    # scale as it travels (absmax / 7 rounded once to fp32)
    t = torch.from_numpy(f)
    st = (t.abs().amax(dim=1, keepdim=True) / 7).float().double()
    want = torch.where(st > 0, torch.clamp(torch.round(t / torch.where(st > 0, st, torch.ones_like(st))), -7, 7) * st, torch.zeros_like(t))
    assert np.array_equal(back, want.numpy())


def test_int4_factors_keep_the_recursion_invariant_and_cost_accuracy_gracefully():
    """recon_t + e_t = x_t holds with quantised factors (D is whatever travelled), and the extra error is of the
    size of the quantisation step: a few percent of the factors' share, not a different regime."""
    rng = np.random.default_rng(22)
    n, c = 160, 128
    x0 = rng.standard_normal((n, c)).astype(np.float32)
    x1 = (x0 + 0.05 * rand_lowrank(rng, n, c, 40, noise=0.01, decay=0.9)).astype(np.float32)
    q0 = rng.standard_normal((c, 32))
    errs = {}
    for fb in (0, 4):
        cfg = lr.LowRankConfig(n, c, dtype=lr.F32, rank=32, iters=2, factor_bits=fb)
        Uw, Vw, err, recon = lr.step(cfg, x1, x0.copy(), q0)
        assert np.allclose(recon.astype(np.float64) + err, x1, atol=1e-5)
        errs[fb] = np.linalg.norm(err)
    assert errs[0] < errs[4] < 0.5 * np.linalg.norm(x1 - x0)
