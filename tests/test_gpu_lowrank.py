"""GPU parity of the low-rank compressor (Alg. 3; App. D "Low-Rank Compression") against the fp64 oracle.

The path is floating-point linear algebra on the matrix cores (fp32 in, fp32 accumulate), so the bar is a
tolerance, derived here from the arithmetic:
  * factors against the oracle: an fp32 dot product over C <= 3072 channels carries a relative error of about
    sqrt(C) * 2^-24 ~ 3e-6 of the operand norms, Gram-Schmidt passes it on multiplied by the conditioning of Z
    (below 100 for the test matrices): WIRE_TOL = 2e-4 of the largest factor entry is asserted, 1e-5 is what is
    seen.  bf16 factors may also differ by one bf16 ulp where the fp32 value sits next to a rounding boundary.
  * error buffer and reconstruction against the ORACLE's end state, element by element, at the tolerance that
    the factor tolerance implies: with |dU| <= E_U and |dV| <= E_V entry-wise (the bounds just asserted),
        |U V^T - Uo Vo^T| <= E_U |Vo|^T + |Uo| E_V^T + E_U E_V^T =: T_D,
    the device's 32-term fp32 dot product adds 1e-5 of sum_k |U_ik V_jk|, and the stored values one rounding
    each (2^-24 of e in fp32; half a bf16 ulp of the reconstruction on either side).
  * as a second, sharper assertion, D, e and recon against an fp64 evaluation of the GPU's OWN travelled
    factors, which is free of the factors' sensitivity.
  * INT4 factors: the oracle decides every nibble in fp64; the device, working in fp32 on its own factors, may
    decide one the other way only where the oracle's f / s lies within the factor tolerance of the half-integer
    between the two nibbles.  That is asserted per nibble, and T_D is formed from the per-entry bounds that follow
    (one quantisation step where the nibble flipped, 7 x the scale tolerance elsewhere).
"""
import sys

import numpy as np
import pytest
import torch

import paper_2507_17511_amd as cf
from oracle import lowrank as lr
from paper_2507_17511_amd.session import CodecSession
from workloads import as_numpy

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
R = 32
WIRE_TOL = 2e-4       # factors: share of the largest entry (see the module docstring)


def say(msg):
    print(f"[case] {msg}", flush=True)
    sys.stdout.flush()


def stream(n, c, dtype, steps, seed, rank=48, decay=0.93, noise=0.02):
    """x_0 ~ N(0,1); each step adds a matrix with a geometrically decaying spectrum plus a little full-rank noise."""
    g = torch.Generator(device=DEV)
    g.manual_seed(seed)
    x = torch.randn((n, c), generator=g, device=DEV)
    sv = decay ** torch.arange(rank, device=DEV, dtype=torch.float32)
    out = []
    for _ in range(steps):
        out.append(x.to(torch.bfloat16).contiguous() if dtype == cf.CF_BF16 else x.clone())
        left = torch.randn((n, rank), generator=g, device=DEV) * sv
        right = torch.randn((rank, c), generator=g, device=DEV)
        x = x + 0.05 * (left @ right) / rank ** 0.5 + noise * 0.05 * torch.randn((n, c), generator=g, device=DEV)
    return out


def start_matrices(c, steps, seed):
    g = torch.Generator(device=DEV)
    g.manual_seed(seed)
    return [torch.randn((c, R), generator=g, device=DEV) for _ in range(steps)]


def split_wire(codes: np.ndarray, n, c, dtype):
    flat = codes.reshape(-1)
    if dtype == cf.CF_BF16:
        w = flat.view(np.uint16)
    else:
        w = flat.view(np.float32)
    return w[:n * R].reshape(n, R).copy(), w[n * R:(n + c) * R].reshape(c, R).copy()


def check_step(tag, cfg, sess, t, x, recon_before, q0, wire_tol=WIRE_TOL):
    n, c, dt = cfg.n_tokens, cfg.n_channels, cfg.dtype
    Ug, Vg = split_wire(as_numpy(sess.codes[t]), n, c, dt)
    Uo, Vo, erro, recono = lr.step(cfg, x, recon_before, q0)
    U64, V64, Uo64, Vo64 = lr.widen(Ug, dt), lr.widen(Vg, dt), lr.widen(Uo, dt), lr.widen(Vo, dt)
    ulp = 2.0 ** -7 if dt == lr.BF16 else 0.0      # one bf16 step is between 2^-8 and 2^-7 of the value
    bounds = []
    for name, got, want in (("U", U64, Uo64), ("V", V64, Vo64)):
        tol = wire_tol * np.abs(want).max() + ulp * np.abs(want)
        worst = float((np.abs(got - want) - ulp * np.abs(want)).max() / np.abs(want).max())
        assert np.all(np.abs(got - want) <= tol), f"{tag}: factor {name} off by {worst:.2e} of its largest entry"
        bounds.append(tol)
    # the subspace itself (independent of the basis)
    proj_gap = np.linalg.norm(V64 @ V64.T - Vo64 @ Vo64.T)
    assert proj_gap < (0.05 if dt == lr.BF16 else 1e-3), f"{tag}: projector differs by {proj_gap:.2e}"
    check_against_oracle_state(tag, cfg, sess, t, U64, V64, Uo64, Vo64, bounds[0], bounds[1], erro, recono, recon_before)
    check_from_own_factors(tag, cfg, sess, t, x, recon_before, U64, V64)
    return float(np.abs(U64 - Uo64).max() / np.abs(Uo64).max()), float(np.abs(V64 - Vo64).max())


def check_against_oracle_state(tag, cfg, sess, t, U64, V64, Uo64, Vo64, E_U, E_V, erro, recono, recon_before):
    """e and recon against the oracle's end state, at the tolerance the entry-wise factor bounds E_U, E_V imply."""
    n, c, dt = cfg.n_tokens, cfg.n_channels, cfg.dtype
    T_D = E_U @ np.abs(Vo64).T + np.abs(Uo64) @ E_V.T + E_U @ E_V.T
    terms = np.abs(U64) @ np.abs(V64).T                                     # what the device's fp32 dot product sums
    err = as_numpy(sess.err[t]).astype(np.float64).reshape(n, c)
    erro = erro.astype(np.float64).reshape(n, c)
    tol_e = T_D + 1e-5 * terms + 2.0 ** -22 * np.abs(erro) + 1e-30
    worst = float((np.abs(err - erro) / tol_e).max())
    assert worst <= 1.0, f"{tag}: error buffer is {worst:.2f} x its tolerance away from the oracle's"
    recon = lr.widen(as_numpy(sess.recon[t]), dt).reshape(n, c)
    recono = lr.widen(recono, dt).reshape(n, c)
    half_ulp = (2.0 ** -8 if dt == lr.BF16 else 2.0 ** -23) * 1.01
    tol_r = T_D + 1e-5 * terms + half_ulp * (np.abs(recon) + np.abs(recono)) + 1e-30
    worst_r = float((np.abs(recon - recono) / tol_r).max())
    assert worst_r <= 1.0, f"{tag}: reconstruction is {worst_r:.2f} x its tolerance away from the oracle's"
    return worst, worst_r


def check_from_own_factors(tag, cfg, sess, t, x, recon_before, U64, V64):
    """D, e and recon against an fp64 evaluation of the factors the GPU itself put on the wire."""
    n, c, dt = cfg.n_tokens, cfg.n_channels, cfg.dtype
    A = lr.widen(x, dt).reshape(n, c) - lr.widen(recon_before, dt).reshape(n, c)
    D = U64 @ V64.T
    terms = np.abs(U64) @ np.abs(V64).T
    err = as_numpy(sess.err[t]).astype(np.float64).reshape(n, c)
    assert np.all(np.abs(err - (A - D)) <= 1e-5 * terms + 1e-6 * np.abs(A) + 1e-30), f"{tag}: e != A - U V^T"
    recon = lr.widen(as_numpy(sess.recon[t]), dt).reshape(n, c)
    target = lr.widen(recon_before, dt).reshape(n, c) + D
    half_ulp = (2.0 ** -8 if dt == lr.BF16 else 2.0 ** -23) * np.abs(target) * 1.01
    assert np.all(np.abs(recon - target) <= half_ulp + 1e-5 * terms + 1e-30), f"{tag}: recon != recon + U V^T"


def check_int4_step(tag, cfg, sess, t, x, recon_before, q0, wire_tol=WIRE_TOL):
    """INT4 factors: scales, every nibble, then the end state against the oracle's and against the GPU's own factors.
    Returns how many nibbles sit on a decision boundary (and went the other way)."""
    n, c, dt = cfg.n_tokens, cfg.n_channels, cfg.dtype
    Ug, Vg = split_wire_int4(as_numpy(sess.codes[t]).view(np.uint8), n, c)
    Uo, Vo, erro, recono = lr.step(cfg, x, recon_before, q0)
    A = lr.widen(x, dt).reshape(n, c) - lr.widen(recon_before, dt).reshape(n, c)
    F_U, F_V = lr.subspace_iteration(A, np.asarray(q0, dtype=np.float64).reshape(c, R), cfg.iters)     # the oracle's fp64 factors
    flips, bounds, deq = 0, [], []
    for name, (gn, gs), (on, os_), F in (("U", Ug, Uo, F_U), ("V", Vg, Vo, F_V)):
        big_s, big_f = np.abs(os_).max(), np.abs(F).max()
        tol_s = wire_tol * big_s
        assert np.all(np.abs(gs - os_) <= tol_s), f"{tag}: {name} scales off by {np.abs(gs - os_).max() / big_s:.2e} of the largest"
        qg, qo = lr.unpack_nibbles(gn), lr.unpack_nibbles(on)
        differ = qg != qo
        s64 = os_.astype(np.float64)[:, None]
        safe = np.where(s64 == 0, 1.0, s64)
        where = np.nonzero(differ)
        if where[0].size:
            assert np.all(np.abs(qg - qo)[where] == 1), f"{tag}: a {name} nibble is off by more than one step"
            boundary = (qg + qo)[where] / 2.0                   # the half-integer between the two decisions
            dist = np.abs((F / safe)[where] - boundary)          # how far the oracle's value is from it, in steps
            allowed = (wire_tol * big_f / safe)[where[0], 0] + 1e-6
            worst = float((dist / allowed).max())
            assert worst <= 1.0, f"{tag}: a {name} nibble differs where the oracle's value is {worst:.1f} x the factor tolerance from the boundary"
        flips += int(differ.sum())
        bounds.append(np.where(differ, np.maximum(gs, os_).astype(np.float64)[:, None] * 1.001, 7.0 * tol_s))
        deq.append((lr.dequantise_rows(gn, gs), lr.dequantise_rows(on, os_)))
    (U64, Uo64), (V64, Vo64) = deq
    check_against_oracle_state(tag, cfg, sess, t, U64, V64, Uo64, Vo64, bounds[0], bounds[1], erro, recono, recon_before)
    check_from_own_factors(tag, cfg, sess, t, x, recon_before, U64, V64)
    return flips


@pytest.mark.parametrize("dtype", [cf.CF_F32, cf.CF_BF16])
@pytest.mark.parametrize("iters", [1, 2])
@pytest.mark.parametrize("mode", ["fused", "split"])
def test_lowrank_parity(dtype, iters, mode):
    for k, (n, c) in enumerate([(96, 128), (203, 1024), (300, 3072), (64, 32), (1, 64), (517, 96)]):
        say(f"lowrank dtype={dtype} T={iters} mode={mode} N={n} C={c}")
        d = cf.desc(n, c, dtype, iters, cf.CF_LOWRANK, R)
        cfg = lr.LowRankConfig(n, c, dtype=dtype, rank=R, iters=iters)
        xs = stream(n, c, dtype, 4, 900 + k)
        q0s = start_matrices(c, 4, 950 + k)
        sess = CodecSession([d], cf.options(), device=DEV)
        try:
            sess.warmup([xs[0]])
            for s in range(1, 4):
                before = as_numpy(sess.recon[0]).copy()
                sess.scales[0].copy_(q0s[s].reshape(-1))
                if mode == "fused":
                    sess.step_fused([xs[s]])
                else:
                    sess.compress([xs[s]])
                    sess.decompress()
                cf.cf_check_device(sess.ctx, sess.stream_handle)
                du, dv = check_step(f"N{n}C{c} step {s}", cfg, sess, 0, as_numpy(xs[s]), before, as_numpy(q0s[s]))
            say(f"   factors within {du:.1e} (U, relative) and {dv:.1e} (V, absolute) of the oracle")
        finally:
            sess.close()


def split_wire_int4(codes: np.ndarray, n, c):
    """U nibbles [N, 16], V nibbles [C, 16], U scales [N] fp32, V scales [C] fp32."""
    flat = codes.reshape(-1)
    assert flat.size == (n + c) * 20
    un, vn = flat[:n * 16].reshape(n, 16), flat[n * 16:(n + c) * 16].reshape(c, 16)
    sc = flat[(n + c) * 16:].view(np.float32)
    return (un.copy(), sc[:n].copy()), (vn.copy(), sc[n:].copy())


@pytest.mark.parametrize("dtype", [cf.CF_F32, cf.CF_BF16])
@pytest.mark.parametrize("mode", ["fused", "split"])
def test_lowrank_int4_factors(dtype, mode):
    """CF_FLAG_LOWRANK_INT4: the factors travel as nibbles with one fp32 scale per factor row.  The scales must
    agree with the oracle's to the factor tolerance; a nibble may differ from the oracle's (decided in fp64) only
    by one step and only where the oracle's value lies within the factor tolerance of the boundary between the
    two; e and recon are then checked against the oracle's end state and against the GPU's own factors."""
    for k, (n, c) in enumerate([(96, 128), (203, 1024), (300, 3072), (1, 64), (517, 96)]):
        say(f"lowrank int4 factors dtype={dtype} mode={mode} N={n} C={c}")
        d = cf.desc(n, c, dtype, 1 + k % 2, cf.CF_LOWRANK, R)
        cfg = lr.LowRankConfig(n, c, dtype=dtype, rank=R, iters=1 + k % 2, factor_bits=4)
        xs = stream(n, c, dtype, 4, 1300 + k)
        q0s = start_matrices(c, 4, 1350 + k)
        sess = CodecSession([d], cf.options(flags=cf.CF_FLAG_LOWRANK_INT4), device=DEV)
        try:
            assert sess.codes[0].numel() * sess.codes[0].element_size() == (n + c) * 20
            sess.warmup([xs[0]])
            for s in range(1, 4):
                before = as_numpy(sess.recon[0]).copy()
                sess.scales[0].copy_(q0s[s].reshape(-1))
                if mode == "fused":
                    sess.step_fused([xs[s]])
                else:
                    sess.compress([xs[s]])
                    sess.decompress()
                cf.cf_check_device(sess.ctx, sess.stream_handle)
                flips = check_int4_step(f"int4 N{n}C{c} step {s}", cfg, sess, 0, as_numpy(xs[s]), before, as_numpy(q0s[s]))
                assert flips <= 2 + 0.005 * (n + c) * R, f"{flips} nibbles sit on a decision boundary: too many to be chance"
            say(f"   {flips} of {(n + c) * R} nibbles sat on a decision boundary and went the other way at the last step")
        finally:
            sess.close()


def test_lowrank_int4_sizes():
    o = cf.options(flags=cf.CF_FLAG_LOWRANK_INT4)
    assert cf.cf_sizes(cf.desc(4096, 3072, cf.CF_BF16, 1, cf.CF_LOWRANK, R), o)[0] == (4096 + 3072) * 20
    assert cf.cf_sizes(cf.desc(4096, 3072, cf.CF_BF16, 1, cf.CF_LOWRANK, R))[0] == (4096 + 3072) * 64


def test_lowrank_exact_for_residuals_of_small_rank():
    """A residual of rank 5 < 32 comes through unchanged (fp32 storage), and the unused columns are dropped."""
    n, c = 200, 256
    g = torch.Generator(device=DEV)
    g.manual_seed(4)
    x0 = torch.randn((n, c), generator=g, device=DEV)
    delta = torch.randn((n, 5), generator=g, device=DEV) @ torch.randn((5, c), generator=g, device=DEV)
    x1 = x0 + 0.1 * delta
    q0 = torch.randn((c, R), generator=g, device=DEV)
    sess = CodecSession([cf.desc(n, c, cf.CF_F32, 1, cf.CF_LOWRANK, R)], cf.options(), device=DEV)
    try:
        sess.warmup([x0])
        sess.scales[0].copy_(q0.reshape(-1))
        sess.step_fused([x1])
        cf.cf_check_device(sess.ctx, sess.stream_handle)
        _, V = split_wire(as_numpy(sess.codes[0]), n, c, cf.CF_F32)
        assert np.count_nonzero(np.abs(V).sum(axis=0)) == 5
        assert float((sess.recon[0] - x1).abs().max()) < 1e-4 * float((x1 - x0).abs().max())
        assert float(sess.err[0].abs().max()) < 1e-4 * float((x1 - x0).abs().max())
    finally:
        sess.close()


def test_lowrank_four_iterations_and_zero_residual():
    """T = 4 (the basis is re-orthogonalised after every product, so the conditioning does not compound), and an
    unchanged tensor: A = 0 gives Z = 0, every column is dropped, the factors and D are zero and the state stays."""
    n, c = 300, 1024
    d = cf.desc(n, c, cf.CF_BF16, 4, cf.CF_LOWRANK, R)
    cfg = lr.LowRankConfig(n, c, dtype=lr.BF16, rank=R, iters=4)
    xs = stream(n, c, cf.CF_BF16, 3, 77)
    q0s = start_matrices(c, 4, 78)
    sess = CodecSession([d], cf.options(), device=DEV)
    try:
        sess.warmup([xs[0]])
        for s in (1, 2):
            before = as_numpy(sess.recon[0]).copy()
            sess.scales[0].copy_(q0s[s].reshape(-1))
            sess.step_fused([xs[s]])
            cf.cf_check_device(sess.ctx, sess.stream_handle)
            check_step(f"T4 step {s}", cfg, sess, 0, as_numpy(xs[s]), before, as_numpy(q0s[s]))
        # now feed the reconstruction itself: the residual is exactly zero
        same = sess.recon[0].clone()
        sess.scales[0].copy_(q0s[3].reshape(-1))
        sess.step_fused([same])
        cf.cf_check_device(sess.ctx, sess.stream_handle)
        U, V = split_wire(as_numpy(sess.codes[0]), n, c, cf.CF_BF16)
        assert not U.any() and not V.any()
        assert torch.equal(sess.recon[0], same) and not bool(sess.err[0].any())
    finally:
        sess.close()


def test_lowrank_in_a_mixed_batch_and_receiver():
    """Low-rank tensors next to quantised and sparsified ones in one call; a receiver fed the wire reaches the
    sender's reconstruction bit for bit (both ends add the same D)."""
    from helpers import OracleState, compare_tensor
    descs = [cf.desc(203, 1024, cf.CF_BF16, 1, cf.CF_LOWRANK, R), cf.desc(130, 264, cf.CF_BF16, 2, cf.CF_SCALE_CHANNEL),
             cf.desc(96, 128, cf.CF_F32, 2, cf.CF_LOWRANK, R), cf.desc(67, 3072, cf.CF_BF16, 2, cf.CF_SPARSE_NM, 8)]
    xs = [stream(int(d.n_tokens), int(d.n_channels), int(d.dtype), 3, 70 + t) for t, d in enumerate(descs)]
    q0 = {0: start_matrices(1024, 3, 5), 2: start_matrices(128, 3, 6)}
    send = CodecSession(descs, cf.options(), device=DEV)
    recv = CodecSession(descs, cf.options(), device=DEV)
    orc = OracleState(descs, cf.options(), [1, 3])
    try:
        first = [x[0] for x in xs]
        send.warmup(first)
        recv.warmup(first)
        for t in (1, 3):
            orc.warmup(t, as_numpy(first[t]))
        for s in (1, 2):
            now = [x[s] for x in xs]
            before = {t: as_numpy(send.recon[t]).copy() for t in (0, 2)}
            for t in (0, 2):
                send.scales[t].copy_(q0[t][s].reshape(-1))
            send.step_fused(now)
            cf.cf_check_device(send.ctx, send.stream_handle)
            for t in (0, 2):
                cfg = lr.LowRankConfig(int(descs[t].n_tokens), int(descs[t].n_channels), dtype=int(descs[t].dtype), rank=R,
                                       iters=int(descs[t].bits))
                check_step(f"mixed t{t} step {s}", cfg, send, t, as_numpy(now[t]), before[t], as_numpy(q0[t][s]))
            for t in (1, 3):
                orc.step(t, as_numpy(now[t]))
                compare_tensor(f"mixed step {s}", send, orc, t)
            for t in range(len(descs)):
                recv.codes[t].copy_(send.codes[t])
                if recv.scales[t].numel():
                    recv.scales[t].copy_(send.scales[t])
            recv.decompress()
            cf.cf_check_device(recv.ctx, recv.stream_handle)
            for t in range(len(descs)):
                assert torch.equal(recv.recon[t], send.recon[t]), f"receiver differs on tensor {t} at step {s}"
    finally:
        send.close()
        recv.close()


def test_lowrank_int4_in_a_mixed_batch_and_receiver():
    """The INT4-factor context next to quantised and sparsified tensors: those are untouched by the flag (bit-exact
    against the oracle), and a receiver fed the wire reaches the sender's reconstruction bit for bit."""
    from helpers import OracleState, compare_tensor
    opts = cf.options(flags=cf.CF_FLAG_LOWRANK_INT4)
    descs = [cf.desc(203, 1024, cf.CF_BF16, 1, cf.CF_LOWRANK, R), cf.desc(130, 264, cf.CF_BF16, 2, cf.CF_SCALE_CHANNEL),
             cf.desc(96, 128, cf.CF_F32, 2, cf.CF_LOWRANK, R), cf.desc(67, 3072, cf.CF_BF16, 2, cf.CF_SPARSE_NM, 16)]
    xs = [stream(int(d.n_tokens), int(d.n_channels), int(d.dtype), 3, 170 + t) for t, d in enumerate(descs)]
    q0 = {0: start_matrices(1024, 3, 15), 2: start_matrices(128, 3, 16)}
    send, recv = CodecSession(descs, opts, device=DEV), CodecSession(descs, opts, device=DEV)
    orc = OracleState(descs, opts, [1, 3])
    try:
        first = [x[0] for x in xs]
        send.warmup(first)
        recv.warmup(first)
        for t in (1, 3):
            orc.warmup(t, as_numpy(first[t]))
        for s in (1, 2):
            now = [x[s] for x in xs]
            before = {t: as_numpy(send.recon[t]).copy() for t in (0, 2)}
            for t in (0, 2):
                send.scales[t].copy_(q0[t][s].reshape(-1))
            send.step_fused(now)
            cf.cf_check_device(send.ctx, send.stream_handle)
            for t in (0, 2):
                n, c = int(descs[t].n_tokens), int(descs[t].n_channels)
                cfg = lr.LowRankConfig(n, c, dtype=int(descs[t].dtype), rank=R, iters=int(descs[t].bits), factor_bits=4)
                check_int4_step(f"int4 mixed t{t} step {s}", cfg, send, t, as_numpy(now[t]), before[t], as_numpy(q0[t][s]))
            for t in (1, 3):
                orc.step(t, as_numpy(now[t]))
                compare_tensor(f"int4 mixed step {s}", send, orc, t)
            for t in range(len(descs)):
                recv.codes[t].copy_(send.codes[t])
                if recv.scales[t].numel():
                    recv.scales[t].copy_(send.scales[t])
            recv.decompress()
            cf.cf_check_device(recv.ctx, recv.stream_handle)
            for t in range(len(descs)):
                assert torch.equal(recv.recon[t], send.recon[t]), f"receiver differs on tensor {t} at step {s}"
    finally:
        send.close()
        recv.close()


def test_lowrank_rejections():
    for d, status in ((cf.desc(64, 100, cf.CF_BF16, 1, cf.CF_LOWRANK, R), cf.CF_ERR_SHAPE),       # C not a multiple of 32
                      (cf.desc(64, 4096, cf.CF_BF16, 1, cf.CF_LOWRANK, R), cf.CF_ERR_SHAPE),      # C above 3072
                      (cf.desc(64, 128, cf.CF_BF16, 1, cf.CF_LOWRANK, 8), cf.CF_ERR_UNSUPPORTED)):
        with pytest.raises(cf.CFError) as ei:
            cf.cf_sizes(d)
        assert ei.value.status == status
    good = cf.desc(64, 128, cf.CF_BF16, 1, cf.CF_LOWRANK, R)
    assert cf.cf_sizes(good)[:2] == ((64 + 128) * R * 2, 128 * R * 4)
    assert cf.cf_workspace_bytes([good], cf.options(ef=cf.CF_EF_OFF)) == 0     # only the default feedback mode


def test_lowrank_full_shape():
    """[4096, 3072] bf16, rank 32, T = 1 and 2, in one batch: factors against the fp64 oracle, error and
    reconstruction re-derived from the travelled factors."""
    n, c = 4096, 3072
    descs = [cf.desc(n, c, cf.CF_BF16, 1 + t % 2, cf.CF_LOWRANK, R) for t in range(4)]
    xs = [stream(n, c, cf.CF_BF16, 3, 300 + t) for t in range(4)]
    q0s = [start_matrices(c, 3, 400 + t) for t in range(4)]
    sess = CodecSession(descs, cf.options(), device=DEV)
    try:
        sess.warmup([x[0] for x in xs])
        for s in (1, 2):
            before = [as_numpy(sess.recon[t]).copy() for t in range(4)]
            for t in range(4):
                sess.scales[t].copy_(q0s[t][s].reshape(-1))
            sess.step_fused([x[s] for x in xs])
            cf.cf_check_device(sess.ctx, sess.stream_handle)
            for t in range(4):
                cfg = lr.LowRankConfig(n, c, dtype=lr.BF16, rank=R, iters=1 + t % 2)
                du, dv = check_step(f"full t{t} step {s}", cfg, sess, t, as_numpy(xs[t][s]), before[t], as_numpy(q0s[t][s]))
                say(f"lowrank full shape tensor {t} step {s}: factors within {du:.1e} (U, relative), {dv:.1e} (V, absolute)")
    finally:
        sess.close()
