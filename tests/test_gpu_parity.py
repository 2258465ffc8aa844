"""GPU parity: the HIP library against the CPU oracle, element by element, through
the C ABI, on seeded inputs small enough for the oracle but spanning several
tiles, ragged tails, every code width, scale kind, error-feedback mode and
storage dtype.  Bars are stated in tests/helpers.py."""
import sys

import numpy as np
import pytest
import torch

import paper_2507_17511_amd as cf
from helpers import (OracleState, assert_same, compare_tensor, drift_stream, kind_of, oracle_config, run_parity)
from paper_2507_17511_amd.session import CodecSession
from workloads import CONFIGS, ActivationStream, as_numpy, cfg1_numpy

pytestmark = pytest.mark.gpu

DEV = "cuda:0"
CH, GR = cf.CF_SCALE_CHANNEL, cf.CF_SCALE_GROUP


def say(msg):
    print(f"[case] {msg}", flush=True)
    sys.stdout.flush()


# (N, C): several row tiles with a ragged last one; C spans one full 1024-channel
# column tile plus a partial one (1096 = 137 chunks), a single chunk, and 3072.
SHAPES = [(203, 1096), (67, 3072), (9, 8), (1, 128), (130, 2176)]
COMBOS = [(1, CH), (2, CH), (4, CH), (4, GR)]


@pytest.mark.parametrize("bits,scale", COMBOS)
@pytest.mark.parametrize("dtype", [cf.CF_BF16, cf.CF_F32])
@pytest.mark.parametrize("mode", ["fused", "split"])
@pytest.mark.parametrize("flags", [cf.CF_FLAG_SINGLE_PASS, cf.CF_FLAG_TWO_KERNEL])
def test_parity_shapes(bits, scale, dtype, mode, flags):
    """flags: the single-pass kernel (default where it applies) and the two-kernel path must both match the oracle."""
    if scale == GR and flags == cf.CF_FLAG_TWO_KERNEL:
        pytest.skip("group scales take the same path either way")
    for k, (n, c) in enumerate(SHAPES):
        if scale == GR and c % 128:
            continue
        say(f"shapes bits={bits} scale={scale} dtype={dtype} mode={mode} flags={flags} N={n} C={c}")
        d = cf.desc(n, c, dtype, bits, scale)
        xs = drift_stream((n, c), dtype, steps=4, seed=100 + k, device=DEV)
        run_parity([d], cf.options(flags=flags), [[x] for x in xs], mode=mode, tag=f"N{n}C{c}")


@pytest.mark.parametrize("ef", [cf.CF_EF_RECON, cf.CF_EF_LITERAL, cf.CF_EF_OFF])
@pytest.mark.parametrize("err_dtype", [cf.CF_F32, cf.CF_BF16])
def test_parity_ef_modes_and_err_dtypes(ef, err_dtype):
    n, c = 203, 1152
    for bits, scale in COMBOS:
        for dtype in (cf.CF_BF16, cf.CF_F32):
            say(f"ef={ef} err_dtype={err_dtype} bits={bits} scale={scale} dtype={dtype}")
            d = cf.desc(n, c, dtype, bits, scale)
            xs = drift_stream((n, c), dtype, steps=5, seed=7 * bits + ef, device=DEV)
            run_parity([d], cf.options(ef=ef, err_dtype=err_dtype), [[x] for x in xs], mode="fused")


@pytest.mark.parametrize("tile_rows", [8, 16, 32, 64])
def test_parity_every_tile_height(tile_rows):
    """The tree over rows is split differently for every tile height; scales must not move."""
    n, c = 333, 1096
    for bits in (1, 2, 4):
        say(f"tile_rows={tile_rows} bits={bits}")
        d = cf.desc(n, c, cf.CF_BF16, bits, CH)
        xs = drift_stream((n, c), cf.CF_BF16, steps=3, seed=bits, device=DEV)
        run_parity([d], cf.options(tile_rows=tile_rows), [[x] for x in xs])


@pytest.mark.parametrize("encode_rows", [1, 2, 3, 8, 64])
def test_parity_every_encode_height(encode_rows):
    """Rows per workgroup of the element-wise kernels, on channel counts with (1152, 3072) and
    without (1096, 8) whole quads of lanes (the gathered code stores need them)."""
    for k, (n, c) in enumerate([(67, 1152), (130, 1096), (9, 8), (33, 3072)]):
        for bits, scale in COMBOS:
            if scale == GR and c % 128:
                continue
            say(f"encode_rows={encode_rows} N={n} C={c} bits={bits} scale={scale}")
            d = cf.desc(n, c, cf.CF_BF16, bits, scale)
            xs = drift_stream((n, c), cf.CF_BF16, steps=3, seed=11 * k + bits, device=DEV)
            for mode in ("fused", "split"):
                run_parity([d], cf.options(encode_rows=encode_rows), [[x] for x in xs], mode=mode)


def _mixed_batch():
    descs = [cf.desc(203, 1096, cf.CF_BF16, 1, CH), cf.desc(64, 3072, cf.CF_BF16, 2, CH),
             cf.desc(100, 256, cf.CF_F32, 4, GR), cf.desc(77, 1024, cf.CF_BF16, 4, CH),
             cf.desc(256, 64, cf.CF_F32, 2, CH), cf.desc(19, 384, cf.CF_BF16, 4, GR),
             cf.desc(40, 8, cf.CF_F32, 1, CH)]
    streams = [drift_stream((d.n_tokens, d.n_channels), d.dtype, steps=4, seed=40 + k, device=DEV)
               for k, d in enumerate(descs)]
    xs = [[streams[t][s] for t in range(len(descs))] for s in range(4)]
    return descs, xs


@pytest.mark.parametrize("mode", ["fused", "split"])
@pytest.mark.parametrize("flags", [cf.CF_FLAG_SINGLE_PASS, cf.CF_FLAG_TWO_KERNEL])
def test_parity_batched_mixed_launch(mode, flags):
    """One call covers tensors of different shapes, dtypes, widths and scale kinds."""
    say(f"mixed batch mode={mode} flags={flags}")
    descs, xs = _mixed_batch()
    run_parity(descs, cf.options(flags=flags), xs, mode=mode)


def test_single_pass_many_row_blocks_and_stripes():
    """Reduction groups of several items (N = 1500: 6 row blocks of 256, ragged) over 9 stripes (C = 1096),
    several tensors deep, so that workgroups take more than one item each."""
    say("single pass, deep")
    descs = [cf.desc(1500, 1096, cf.CF_BF16, (1, 2, 4)[t % 3], CH) for t in range(6)]
    descs += [cf.desc(700, 520, cf.CF_F32, (2, 4, 1)[t % 3], CH) for t in range(3)]
    streams = [drift_stream((d.n_tokens, d.n_channels), d.dtype, steps=3, seed=70 + k, device=DEV)
               for k, d in enumerate(descs)]
    xs = [[streams[t][s] for t in range(len(descs))] for s in range(3)]
    run_parity(descs, cf.options(flags=cf.CF_FLAG_SINGLE_PASS), xs, mode="fused")
    run_parity(descs, cf.options(flags=cf.CF_FLAG_TWO_KERNEL), xs, mode="fused")
    run_parity(descs, cf.options(), xs, mode="fused")


def test_single_pass_stripe_width_rule_boundaries():
    """The single-pass kernel takes 256-channel stripes for contexts whose tallest channel-scale tensor makes at most
    12 items per group with 128-channel ones (bf16: N <= 3072), 128-channel stripes otherwise: contexts on both sides
    of the boundary (N = 3072 / 3328) and at N = 4096 with and without a 1-bit tensor, ragged in both directions,
    against the oracle."""
    cases = [[(3072, 264, 1), (1000, 1096, 2)],                 # wide, groups of 24 and 8 items
             [(3328, 264, 1), (1000, 1096, 2)],                 # narrow, groups of 13 and 4
             [(4096, 264, 4), (4000, 136, 2)],                  # narrow, groups of 16
             [(4096, 264, 4), (4000, 136, 1)]]                  # narrow, groups of 16
    for k, shapes in enumerate(cases):
        say(f"stripe width boundary case {k}: {shapes}")
        descs = [cf.desc(n, c, cf.CF_BF16, bits, CH) for n, c, bits in shapes]
        streams = [drift_stream((d.n_tokens, d.n_channels), d.dtype, steps=3, seed=270 + 10 * k + t, device=DEV) for t, d in enumerate(descs)]
        xs = [[streams[t][s] for t in range(len(descs))] for s in range(3)]
        for mode in ("fused", "split"):
            run_parity(descs, cf.options(flags=cf.CF_FLAG_SINGLE_PASS), xs, mode=mode)


def test_single_pass_long_groups_and_fixed_grid():
    """Groups of 157 items (N = 40000), as one workgroup per item and as a fixed grid of workgroups that loop
    over the items (CF_FLAG_FIXED_GRID)."""
    say("single pass, long groups")
    descs = [cf.desc(40000, 72, cf.CF_BF16, (1, 2, 4)[t % 3], CH) for t in range(6)]
    streams = [drift_stream((d.n_tokens, d.n_channels), d.dtype, steps=3, seed=170 + k, device=DEV)
               for k, d in enumerate(descs)]
    xs = [[streams[t][s] for t in range(len(descs))] for s in range(3)]
    run_parity(descs, cf.options(flags=cf.CF_FLAG_SINGLE_PASS), xs, mode="fused")
    run_parity(descs, cf.options(flags=cf.CF_FLAG_SINGLE_PASS | cf.CF_FLAG_FIXED_GRID), xs, mode="fused")


@pytest.mark.parametrize("ef", [cf.CF_EF_RECON, cf.CF_EF_LITERAL, cf.CF_EF_OFF, cf.CF_EF_NAIVE])
@pytest.mark.parametrize("err_dtype", [cf.CF_F32, cf.CF_BF16])
def test_single_pass_every_feedback_mode(ef, err_dtype):
    """The single-pass kernel in every error-feedback mode (items are 256 rows of bf16 without the error buffer as an
    operand, 128 with it, half of that for fp32), ragged in both directions, several row blocks and stripes deep,
    fused and split, also as a fixed grid."""
    descs = [cf.desc(1500, 1096, cf.CF_BF16, (1, 2, 4)[t % 3], CH) for t in range(3)]
    descs += [cf.desc(700, 520, cf.CF_F32, (2, 4, 1)[t % 3], CH) for t in range(3)]
    descs += [cf.desc(130, 72, cf.CF_BF16, 2, CH), cf.desc(1, 8, cf.CF_F32, 1, CH)]
    streams = [drift_stream((d.n_tokens, d.n_channels), d.dtype, steps=4, seed=370 + 10 * ef + k, device=DEV)
               for k, d in enumerate(descs)]
    xs = [[streams[t][s] for t in range(len(descs))] for s in range(4)]
    for mode in ("fused", "split"):
        if ef == cf.CF_EF_NAIVE and mode == "split":
            continue            # naive compression has no separate receiver step in the oracle harness
        say(f"single pass ef={ef} err_dtype={err_dtype} mode={mode}")
        run_parity(descs, cf.options(ef=ef, err_dtype=err_dtype, flags=cf.CF_FLAG_SINGLE_PASS), xs, mode=mode)
    run_parity(descs, cf.options(ef=ef, err_dtype=err_dtype, flags=cf.CF_FLAG_SINGLE_PASS | cf.CF_FLAG_FIXED_GRID), xs, mode="fused")


@pytest.mark.parametrize("ef", [cf.CF_EF_RECON, cf.CF_EF_OFF])
def test_single_pass_gives_up_and_redoes(ef):
    """CF_FLAG_TEST_NO_WAIT: a workgroup that does not find every partial sum of its stripe at its first look gives
    its item up, and the second launch of the call does it.  Same bits as ever, and the give-up path did run."""
    descs = [cf.desc(1500, 1096, cf.CF_BF16, (1, 2, 4)[t % 3], CH) for t in range(4)]
    descs += [cf.desc(700, 520, cf.CF_F32, (2, 4, 1)[t % 3], CH) for t in range(2)]
    streams = [drift_stream((d.n_tokens, d.n_channels), d.dtype, steps=3, seed=470 + 10 * ef + k, device=DEV)
               for k, d in enumerate(descs)]
    xs = [[streams[t][s] for t in range(len(descs))] for s in range(3)]
    for extra in (0, cf.CF_FLAG_FIXED_GRID):
        say(f"single pass without waiting, ef={ef}, flags +{extra}")
        sess, _ = run_parity(descs, cf.options(ef=ef, flags=cf.CF_FLAG_SINGLE_PASS | cf.CF_FLAG_TEST_NO_WAIT | extra), xs, mode="fused")
    # the counter of the last call, on a session that is still open
    sess = CodecSession(descs, cf.options(ef=ef, flags=cf.CF_FLAG_SINGLE_PASS | cf.CF_FLAG_TEST_NO_WAIT), device=DEV)
    quiet = CodecSession(descs, cf.options(ef=ef, flags=cf.CF_FLAG_SINGLE_PASS), device=DEV)
    try:
        for c in (sess, quiet):
            c.warmup(xs[0])
            c.step_fused(xs[1])
        n_gave_up = cf.cf_given_up_items(sess.ctx, sess.stream_handle)
        say(f"   {n_gave_up} items were given up and redone; {cf.cf_given_up_items(quiet.ctx, quiet.stream_handle)} in the ordinary run")
        assert n_gave_up > 0, "the give-up path was not exercised"
        assert cf.cf_given_up_items(quiet.ctx, quiet.stream_handle) == 0
        for t in range(len(descs)):
            assert torch.equal(sess.recon[t], quiet.recon[t]) and torch.equal(sess.codes[t], quiet.codes[t])
    finally:
        sess.close()
        quiet.close()


def test_single_pass_next_to_other_work_on_the_device():
    """cf_step_fused on one stream while a second stream of the same priority keeps the device busy with unrelated
    kernels: the outputs are the bits of a quiet run, and the oracle's."""
    descs = [cf.desc(4096, 3072, cf.CF_BF16, (1, 2, 4)[t % 3], CH) for t in range(6)]
    streams = [drift_stream((4096, 3072), cf.CF_BF16, steps=3, seed=570 + k, sigma=0.02, device=DEV) for k in range(len(descs))]
    xs = [[streams[t][s] for t in range(len(descs))] for s in range(3)]
    busy, quiet = CodecSession(descs, cf.options(), device=DEV), CodecSession(descs, cf.options(), device=DEV)
    other = torch.cuda.Stream(device=DEV)           # default priority, like the codec's
    a = torch.randn(4096, 4096, device=DEV)
    try:
        for c in (busy, quiet):
            c.warmup(xs[0])
        torch.cuda.synchronize()
        for s in (1, 2):
            quiet.step_fused(xs[s])
            torch.cuda.synchronize()
            with torch.cuda.stream(other):          # matrix products and element-wise kernels, queued ahead and behind
                for _ in range(40):
                    b = a @ a
                    a = torch.tanh(b * 1e-3)
            busy.step_fused(xs[s])
            with torch.cuda.stream(other):
                for _ in range(40):
                    b = a @ a
                    a = torch.tanh(b * 1e-3)
            cf.cf_check_device(busy.ctx, busy.stream_handle)
            torch.cuda.synchronize()
            say(f"step {s} next to a busy stream: {cf.cf_given_up_items(busy.ctx, busy.stream_handle)} items given up and redone")
            for t in range(len(descs)):
                assert torch.equal(busy.recon[t], quiet.recon[t]), f"recon[{t}] differs from the quiet run at step {s}"
                assert torch.equal(busy.err[t], quiet.err[t]) and torch.equal(busy.codes[t], quiet.codes[t])
                assert torch.equal(busy.scales[t], quiet.scales[t])
    finally:
        busy.close()
        quiet.close()
    # and the oracle, on the same inputs (one tensor of each width)
    run_parity(descs[:3], cf.options(), [x[:3] for x in xs], mode="fused")


@pytest.mark.parametrize("case", [0, 1, 2, 3])
def test_single_pass_random_shapes(case):
    """Seeded random batches: token counts that leave ragged items (items are 256 rows of bf16, 128 of fp32),
    channel counts that leave ragged stripes (128 channels) and ragged lane quads, mixed dtypes and widths."""
    rng = np.random.default_rng(1000 + case)
    descs = []
    for t in range(7):
        n = int(rng.integers(1, 2600))
        c = 8 * int(rng.integers(1, 260))
        descs.append(cf.desc(n, c, int(rng.integers(0, 2)), (1, 2, 4)[int(rng.integers(0, 3))], CH))
    say("single pass, random shapes: " + ", ".join(f"[{d.n_tokens},{d.n_channels}]{'bf16' if d.dtype else 'f32'}/{d.bits}" for d in descs))
    streams = [drift_stream((int(d.n_tokens), int(d.n_channels)), int(d.dtype), steps=3, seed=1100 + 10 * case + k, device=DEV)
               for k, d in enumerate(descs)]
    xs = [[streams[t][s] for t in range(len(descs))] for s in range(3)]
    for mode in ("fused", "split"):
        run_parity(descs, cf.options(flags=cf.CF_FLAG_SINGLE_PASS), xs, mode=mode)


def test_subrange_calls_match_whole_batch():
    """Calling [first, first+count) pieces, in any order, equals one whole-batch call."""
    say("subrange")
    descs, xs = _mixed_batch()
    a = CodecSession(descs, device=DEV)
    b = CodecSession(descs, device=DEV)
    a.warmup(xs[0])
    b.warmup(xs[0][4:], first=4, count=3)
    b.warmup(xs[0][:4], first=0, count=4)
    for s in range(1, 4):
        a.step_fused(xs[s])
        b.step_fused(xs[s][5:], first=5, count=2)
        b.step_fused(xs[s][:2], first=0, count=2)
        b.step_fused(xs[s][2:5], first=2, count=3)
        torch.cuda.synchronize()
        for t in range(len(descs)):
            for name in ("codes", "scales", "recon", "err"):
                assert torch.equal(getattr(a, name)[t].view(torch.uint8), getattr(b, name)[t].view(torch.uint8)), (s, t, name)
    a.close(); b.close()


def test_fused_is_bit_identical_to_compress_then_decompress():
    say("fused == split")
    descs, xs = _mixed_batch()
    for opts in (cf.options(), cf.options(ef=cf.CF_EF_LITERAL, err_dtype=cf.CF_BF16), cf.options(ef=cf.CF_EF_OFF)):
        a = CodecSession(descs, opts, device=DEV)
        b = CodecSession(descs, opts, device=DEV)
        a.warmup(xs[0]); b.warmup(xs[0])
        for s in range(1, 4):
            a.step_fused(xs[s])
            b.compress(xs[s])
            recon_before = [r.clone() for r in b.recon]
            torch.cuda.synchronize()
            for t in range(len(descs)):      # cf_compress leaves recon alone
                assert torch.equal(b.recon[t].view(torch.uint8), recon_before[t].view(torch.uint8))
            b.decompress()
            torch.cuda.synchronize()
            for t in range(len(descs)):
                for name in ("codes", "scales", "recon", "err"):
                    assert torch.equal(getattr(a, name)[t].view(torch.uint8), getattr(b, name)[t].view(torch.uint8)), (s, t, name)
        a.close(); b.close()


def test_receiver_tracks_sender_through_the_wire():
    """A receiver that only ever sees codes and scales keeps the same reconstruction as the sender."""
    say("receiver")
    descs, xs = _mixed_batch()
    snd = CodecSession(descs, device=DEV)
    rcv = CodecSession(descs, device=DEV)
    snd.warmup(xs[0]); rcv.warmup(xs[0])          # the warm-up step travels uncompressed
    for s in range(1, 4):
        snd.step_fused(xs[s])
        for t in range(len(descs)):               # "the wire": the packed buffers
            rcv.codes[t].copy_(snd.codes[t]); rcv.scales[t].copy_(snd.scales[t])
        rcv.decompress()
        torch.cuda.synchronize()
        for t in range(len(descs)):
            assert torch.equal(snd.recon[t].view(torch.uint8), rcv.recon[t].view(torch.uint8))
    snd.close(); rcv.close()


# ------------------------------------------------------------------ degenerate and edge inputs

def test_zero_residual_and_exact_round_trip_on_gpu():
    say("zero residual / representable")
    rng = np.random.default_rng(3)
    for bits, scale in COMBOS:
        n, c = 384, 256
        d = cf.desc(n, c, cf.CF_F32, bits, scale)
        x0 = torch.from_numpy(np.round(rng.standard_normal((n, c)) * 4).astype(np.float32)).to(DEV)
        s = CodecSession([d], device=DEV)
        s.warmup([x0])
        s.step_fused([x0])                        # x_t == recon_{t-1}
        torch.cuda.synchronize()
        assert not s.codes[0].any() and not s.scales[0].any() and not s.err[0].any()
        assert torch.equal(s.recon[0], x0)
        # representable residuals come back exactly
        if bits == 1:
            z = 0.375 * rng.choice([-1.0, 1.0], size=(n, c))
        elif bits == 2:
            z = np.where(np.arange(n)[:, None] % 3 == 0, 2.0, 0.5) * 0.25 * rng.choice([-1.0, 1.0], size=(n, c))
        else:
            k = rng.integers(-7, 8, size=(n, c)); k[:, ::128] = 7; k[0, :] = -7
            z = k * 0.5
        x1 = x0 + torch.from_numpy(z.astype(np.float32)).to(DEV)
        s.step_fused([x1])
        torch.cuda.synchronize()
        assert torch.equal(s.recon[0], x1) and not s.err[0].any()
        s.close()


def test_extreme_values_stay_in_parity():
    """Large dynamic range, exact ties of the 2-bit threshold and 4-bit half-way points, signed zeros."""
    say("extremes")
    rng = np.random.default_rng(5)
    n, c = 64, 256
    base = rng.standard_normal((n, c)).astype(np.float32)
    scalecol = (10.0 ** rng.integers(-12, 12, size=c)).astype(np.float32)
    x0 = np.zeros((n, c), dtype=np.float32)
    x1 = base * scalecol[None, :]
    x1[:, 0] = np.where(np.arange(n) % 4 == 1, 0.25, 1.25)          # mean 1.0 -> 1.25 is an exact tie
    x1[:, 1] = 0.0
    x1[:, 2] = -0.0
    x1[::2, 3] = 3.5; x1[1::2, 3] = 7.0                              # 4-bit: 3.5/1.0 is a half-way point
    x1[:, 4] = 2.0 ** -130                                           # denormal column
    for bits, scale in COMBOS:
        for dtype in (cf.CF_F32, cf.CF_BF16):
            d = cf.desc(n, c, dtype, bits, scale)
            conv = (lambda a: torch.from_numpy(a).to(DEV).to(torch.bfloat16)) if dtype == cf.CF_BF16 else (lambda a: torch.from_numpy(a).to(DEV))
            run_parity([d], cf.options(), [[conv(x0)], [conv(x1)], [conv(x1 * 0.5)]], tag=f"extreme b{bits}s{scale}d{dtype}")


# ------------------------------------------------------------------ argument and state errors (need a context)

def test_argument_and_state_errors():
    say("errors")
    d = cf.desc(32, 128, cf.CF_BF16, 2, CH)
    s = CodecSession([d, d], device=DEV)
    x = [torch.zeros(32, 128, dtype=torch.bfloat16, device=DEV) for _ in range(2)]
    with pytest.raises(cf.CFError) as ei:          # not warmed up
        s.step_fused(x)
    assert ei.value.status == cf.CF_ERR_STATE
    with pytest.raises(cf.CFError) as ei:
        s.decompress()
    assert ei.value.status == cf.CF_ERR_STATE
    s.warmup(x[:1], first=0, count=1)
    with pytest.raises(cf.CFError) as ei:          # tensor 1 still cold
        s.step_fused(x)
    assert ei.value.status == cf.CF_ERR_STATE
    s.step_fused(x[:1], first=0, count=1)
    s.warmup(x)
    P = cf.ptr_array
    good = dict(x=P(x), recon=s.p_recon, err=s.p_err, codes=s.p_codes, scales=s.p_scales)

    def call(**kw):
        a = dict(good); a.update(kw)
        cf.cf_step_fused(s.ctx, 0, 2, a["x"], a["recon"], a["err"], a["codes"], a["scales"], s.stream_handle)

    for bad in (dict(x=None), dict(codes=P([s.codes[0], 0])), dict(x=P([x[0].data_ptr() + 2, x[1]])),
                dict(x=s.p_recon), dict(scales=s.p_codes)):
        with pytest.raises(cf.CFError) as ei:
            call(**bad)
        assert ei.value.status == cf.CF_ERR_INVALID_ARG
    for first, count in ((-1, 1), (0, 3), (2, 1), (1, -1)):
        with pytest.raises(cf.CFError) as ei:
            cf.cf_step_fused(s.ctx, first, count, good["x"], good["recon"], good["err"], good["codes"], good["scales"], s.stream_handle)
        assert ei.value.status == cf.CF_ERR_INVALID_ARG
    cf.cf_step_fused(s.ctx, 1, 0, good["x"], good["recon"], good["err"], good["codes"], good["scales"], s.stream_handle)  # empty range: no-op
    # nothing above may have changed state: a valid step still matches the oracle
    torch.cuda.synchronize()
    orc = OracleState([d, d], s.opts)
    for t in range(2):
        orc.warmup(t, as_numpy(x[t]))
    x1 = drift_stream((32, 128), cf.CF_BF16, 2, seed=1, device=DEV)
    s.step_fused([x1[0], x1[1]])
    torch.cuda.synchronize()
    for t in range(2):
        orc.step(t, as_numpy(x1[t]))
        compare_tensor("after errors", s, orc, t)
    s.close()


def test_resume_from_saved_state():
    """State is only (recon, err): a new context handed the same buffers continues identically."""
    say("resume")
    d = cf.desc(100, 1096, cf.CF_BF16, 2, CH)
    xs = drift_stream((100, 1096), cf.CF_BF16, 6, seed=9, device=DEV)
    a = CodecSession([d], device=DEV)
    a.warmup([xs[0]])
    for s in range(1, 6):
        a.step_fused([xs[s]])
    b = CodecSession([d], device=DEV)
    b.warmup([xs[0]])
    for s in range(1, 3):
        b.step_fused([xs[s]])
    torch.cuda.synchronize()
    c = CodecSession([d], device=DEV)
    c.recon[0].copy_(b.recon[0]); c.err[0].copy_(b.err[0])
    cf.cf_set_warm(c.ctx, 0, 1, True)
    for s in range(3, 6):
        c.step_fused([xs[s]])
    torch.cuda.synchronize()
    for name in ("codes", "scales", "recon", "err"):
        assert torch.equal(getattr(a, name)[0].view(torch.uint8), getattr(c, name)[0].view(torch.uint8)), name
    a.close(); b.close(); c.close()


# ------------------------------------------------------------------ the five configurations, reduced

def test_cfg1_tiny_exactly_as_stated():
    """Config 1 at its real size: fp32 [256, 64], 5 steps, 2-bit per-channel, numpy seed 0."""
    say("cfg1")
    xs = cfg1_numpy(seed=0, steps=5)
    d = cf.desc(256, 64, cf.CF_F32, 2, CH)
    for mode in ("fused", "split"):
        run_parity([d], cf.options(), [[torch.from_numpy(x).to(DEV)] for x in xs], mode=mode, tag="cfg1")


@pytest.mark.parametrize("name,shrink", [
    ("cfg2_flux_patch", dict(n_tensors=4, n_tokens=200, steps=5)),
    ("cfg3_kv_fullseq", dict(n_tensors=4, n_tokens=520, steps=4)),
    ("cfg4_video", dict(n_tensors=3, n_tokens=300, steps=6)),
    ("cfg5_batched_mixed", dict(n_tensors=6, n_tokens=260, steps=4)),
])
def test_configs_reduced(name, shrink):
    """The recipe of configs 2-5 (3072 channels, outliers, decaying drift, heavy tails, mixed widths)
    at a token and layer count the oracle handles in seconds."""
    say(name)
    wl = CONFIGS[name].scaled(**shrink)
    stream = ActivationStream(wl, device=DEV)
    scale = GR if wl.scale == "group" else CH
    descs = [cf.desc(wl.n_tokens, wl.n_channels, cf.CF_BF16, wl.bits_of(t), scale, wl.group) for t in range(wl.n_tensors)]
    xs = [[x.clone() for x in stream.current]]
    for _ in range(1, wl.steps):
        xs.append([x.clone() for x in stream.advance()])
    for flags in (0, cf.CF_FLAG_SINGLE_PASS, cf.CF_FLAG_TWO_KERNEL):
        run_parity(descs, cf.options(flags=flags), xs, mode="fused", tag=f"{name} flags={flags}")


# ---------------------------------------------------------------- rank-1 scales u v^T (App. D "Quantization")

R1 = cf.CF_SCALE_RANK1


def token_outlier_stream(shape, dtype, steps, seed):
    """A drift whose per-token magnitude spans two decades: what the row factor u is for."""
    n, c = shape
    g = torch.Generator(device=DEV)
    g.manual_seed(seed)
    row_gain = torch.exp(torch.randn((n, 1), generator=g, device=DEV) * 1.5)
    x = torch.randn(shape, generator=g, device=DEV)
    out = []
    for _ in range(steps):
        out.append(x.to(torch.bfloat16).contiguous() if dtype == cf.CF_BF16 else x.clone())
        x = x + 0.05 * row_gain * torch.randn(shape, generator=g, device=DEV)
    return out


@pytest.mark.parametrize("bits", [1, 2])
@pytest.mark.parametrize("dtype", [cf.CF_BF16, cf.CF_F32])
@pytest.mark.parametrize("mode", ["fused", "split"])
def test_parity_rank1_shapes(bits, dtype, mode):
    """Row sums cross lanes, the two waves of a tile and several column tiles; the total crosses the
    1024 lanes of the finalising block with one row (N <= 1024) or several (N = 2500) per lane."""
    for k, (n, c) in enumerate(SHAPES + [(2500, 264), (1025, 1032)]):
        say(f"rank1 bits={bits} dtype={dtype} mode={mode} N={n} C={c}")
        d = cf.desc(n, c, dtype, bits, R1)
        xs = token_outlier_stream((n, c), dtype, steps=4, seed=300 + k)
        run_parity([d], cf.options(), [[x] for x in xs], mode=mode, tag=f"rank1 N{n}C{c}")


@pytest.mark.parametrize("ef", [cf.CF_EF_RECON, cf.CF_EF_LITERAL, cf.CF_EF_OFF])
def test_parity_rank1_ef_modes_tile_heights(ef):
    n, c = 333, 1096
    for tile_rows in (0, 8, 16, 32, 64):
        for err_dtype in (cf.CF_F32, cf.CF_BF16):
            say(f"rank1 ef={ef} tile_rows={tile_rows} err_dtype={err_dtype}")
            d = cf.desc(n, c, cf.CF_BF16, 2, R1)
            xs = token_outlier_stream((n, c), cf.CF_BF16, steps=4, seed=17 + ef)
            run_parity([d], cf.options(ef=ef, err_dtype=err_dtype, tile_rows=tile_rows), [[x] for x in xs])


def test_parity_rank1_zero_residual_and_mixed_batch():
    """An unchanged tensor has mean |z| = 0, for which u is defined as 0; and rank-1 tensors share
    one batch (and one launch of every kernel) with channel- and group-scaled ones.  The single-pass
    flag is accepted and ignored for a context that holds a rank-1 tensor."""
    n, c = 130, 1152
    x = drift_stream((n, c), cf.CF_BF16, steps=1, seed=5, device=DEV)[0]
    say("rank1 zero residual")
    run_parity([cf.desc(n, c, cf.CF_BF16, 1, R1)], cf.options(), [[x], [x], [x]], tag="rank1 zero")
    descs = [cf.desc(203, 1096, cf.CF_BF16, 2, R1), cf.desc(64, 256, cf.CF_F32, 4, GR), cf.desc(67, 3072, cf.CF_BF16, 1, CH),
             cf.desc(1500, 136, cf.CF_F32, 1, R1), cf.desc(9, 8, cf.CF_BF16, 2, R1)]
    streams = [token_outlier_stream((int(d.n_tokens), int(d.n_channels)), int(d.dtype), 4, 40 + t) for t, d in enumerate(descs)]
    for flags in (0, cf.CF_FLAG_SINGLE_PASS, cf.CF_FLAG_TWO_KERNEL):
        say(f"rank1 mixed batch flags={flags}")
        run_parity(descs, cf.options(flags=flags), [[s[k] for s in streams] for k in range(4)], tag="rank1 mixed")


def test_rank1_beats_channel_scale_on_token_outliers():
    """Why the paper uses u v^T: with token-wise outliers the rank-1 scale leaves a smaller error
    than the channel scale at the same code width (both computed by the library)."""
    n, c = 512, 1024
    xs = token_outlier_stream((n, c), cf.CF_F32, steps=2, seed=9)
    rel = {}
    for scale in (CH, R1):
        sess = CodecSession([cf.desc(n, c, cf.CF_F32, 2, scale)], cf.options(), device=DEV)
        try:
            sess.warmup([xs[0]])
            sess.step_fused([xs[1]])
            cf.cf_check_device(sess.ctx, sess.stream_handle)
            rel[scale] = float((sess.recon[0] - xs[1]).norm() / (xs[1] - xs[0]).norm())
        finally:
            sess.close()
    say(f"relative residual error: channel {rel[CH]:.3f}, rank-1 {rel[R1]:.3f}")
    assert rel[R1] < rel[CH]


# ---------------------------------------------------------------- naive compression (Sec. 3.1) and the error study

@pytest.mark.parametrize("bits,scale", COMBOS + [(1, R1), (2, R1)])
@pytest.mark.parametrize("dtype", [cf.CF_BF16, cf.CF_F32])
@pytest.mark.parametrize("mode", ["fused", "split"])
def test_parity_naive_compression(bits, scale, dtype, mode):
    """CF_EF_NAIVE: codes and scales of x_t itself, recon_t = D, e_t = x_t - D; the state of the step
    before is never read (it is deliberately left holding other values by the warm-up)."""
    for k, (n, c) in enumerate([(203, 1152), (9, 8), (67, 3072)]):
        if scale == GR and c % 128:
            continue
        for err_dtype in (cf.CF_F32, cf.CF_BF16):
            say(f"naive bits={bits} scale={scale} dtype={dtype} mode={mode} err_dtype={err_dtype} N={n} C={c}")
            d = cf.desc(n, c, dtype, bits, scale)
            xs = drift_stream((n, c), dtype, steps=3, seed=500 + k, sigma=0.3, device=DEV)
            run_parity([d], cf.options(ef=cf.CF_EF_NAIVE, err_dtype=err_dtype), [[x] for x in xs], mode=mode, tag="naive")


@pytest.mark.parametrize("bits", [1, 2])
def test_error_study_orders_the_strategies_as_the_paper_does(bits):
    """Sec. 3.1-3.3 on a synthetic stationary stream with sigma_Delta^2 / sigma_a^2 = 0.01: naive compression is
    far worse than residual compression; without feedback the total error keeps growing; with feedback it
    settles.  All numbers come from the library's own state buffers."""
    from paper_2507_17511_amd import error_study
    res = error_study.run(n_tokens=512, n_channels=1024, steps=28, bits=bits, rho=0.995, seed=3, device=DEV)
    checks = error_study.ordering_holds(res)
    say(f"error study bits={bits}: total error at the last step naive {res['naive']['total'][-1]:.3e}, "
        f"residual {res['residual']['total'][-1]:.3e}, residual+ef {res['residual+ef']['total'][-1]:.3e}")
    assert all(checks.values()), checks
    # 1-bit on a Gaussian signal loses 1 - 2/pi of the energy: the delta of the paper's compressor model
    if bits == 1:
        assert abs(res["naive"]["compression"][-1] - (1 - 2 / np.pi)) < 0.02


# ---------------------------------------------------------------- N:M block sparsifier (Sec. 3.4)

NMK = cf.CF_SPARSE_NM


def tie_stream(shape, dtype, steps, seed):
    """Small integers times 1/4: most magnitudes inside a block of 8 tie, many residuals are exactly zero."""
    g = torch.Generator(device=DEV)
    g.manual_seed(seed)
    x = torch.randint(-8, 9, shape, generator=g, device=DEV).float()
    out = []
    for _ in range(steps):
        out.append(x.to(torch.bfloat16).contiguous() if dtype == cf.CF_BF16 else x.clone())
        x = x + 0.25 * torch.randint(-2, 3, shape, generator=g, device=DEV).float()
    return out


@pytest.mark.parametrize("block", [8, 16])
@pytest.mark.parametrize("keep", [1, 2, 4])
@pytest.mark.parametrize("dtype", [cf.CF_BF16, cf.CF_F32])
@pytest.mark.parametrize("mode", ["fused", "split"])
def test_parity_nm_shapes(keep, dtype, mode, block):
    """Masks, kept values, error and reconstruction, on continuous drifts and on drifts full of ties;
    channel counts with (1152, 3072) and without (1096, 8; 16-channel blocks: 1104, 16) whole quads of lanes."""
    shapes = SHAPES + [(33, 1152)]
    if block == 16:
        shapes = [s for s in shapes if s[1] % 16 == 0] + [(203, 1104), (9, 16), (131, 48)]
    for k, (n, c) in enumerate(shapes):
        for maker in (drift_stream_local, tie_stream):
            say(f"nm keep={keep} of {block} dtype={dtype} mode={mode} N={n} C={c} {maker.__name__}")
            d = cf.desc(n, c, dtype, keep, NMK, block)
            xs = maker((n, c), dtype, 4, 700 + k)
            run_parity([d], cf.options(), [[x] for x in xs], mode=mode, tag=f"nm N{n}C{c}")


def drift_stream_local(shape, dtype, steps, seed):
    return drift_stream(shape, dtype, steps=steps, seed=seed, device=DEV)


@pytest.mark.parametrize("ef", [cf.CF_EF_RECON, cf.CF_EF_LITERAL, cf.CF_EF_OFF, cf.CF_EF_NAIVE])
def test_parity_nm_ef_modes_err_dtypes_heights(ef):
    for err_dtype in (cf.CF_F32, cf.CF_BF16):
        for encode_rows in (0, 3, 64):
            for keep, dtype, block in ((1, cf.CF_BF16, 8), (2, cf.CF_BF16, 8), (4, cf.CF_F32, 8), (2, cf.CF_BF16, 16), (4, cf.CF_F32, 16)):
                n, c = (203, 1096) if block == 8 else (203, 1104)
                say(f"nm ef={ef} err_dtype={err_dtype} encode_rows={encode_rows} keep={keep} of {block} dtype={dtype}")
                d = cf.desc(n, c, dtype, keep, NMK, block)
                xs = drift_stream((n, c), dtype, steps=4, seed=31 + ef, device=DEV)
                run_parity([d], cf.options(ef=ef, err_dtype=err_dtype, encode_rows=encode_rows), [[x] for x in xs])


def test_parity_nm_zero_residual():
    """An unchanged tensor: every magnitude in a block ties at zero, the lowest channels are 'kept' with value 0,
    D = 0, and the state stays as it is."""
    n, c = 130, 1152
    x = drift_stream((n, c), cf.CF_BF16, steps=1, seed=5, device=DEV)[0]
    for keep in (1, 2, 4):
        say(f"nm zero residual keep={keep}")
        sess, orc = run_parity([cf.desc(n, c, cf.CF_BF16, keep, NMK, 8)], cf.options(), [[x], [x], [x]], tag="nm zero")
        masks = orc.codes[0][:n * c // 8]
        assert np.all(masks == (1 << keep) - 1) and not orc.codes[0][(n * c // 8 + 15) // 16 * 16:].any()
        say(f"nm zero residual keep={keep} of 16")
        sess, orc = run_parity([cf.desc(n, c, cf.CF_BF16, keep, NMK, 16)], cf.options(), [[x], [x], [x]], tag="nm zero 16")
        masks = orc.codes[0][:n * c // 8].reshape(-1, 2)
        assert np.all(masks[:, 0] == (1 << keep) - 1) and not masks[:, 1].any()


def test_parity_nm_in_a_mixed_batch():
    """Sparsified tensors share a batch with quantised ones, with and without the single-pass kernel
    taking the channel-scaled tensors."""
    descs = [cf.desc(203, 1096, cf.CF_BF16, 2, NMK, 8), cf.desc(64, 256, cf.CF_F32, 4, GR), cf.desc(300, 1024, cf.CF_BF16, 1, CH),
             cf.desc(67, 3072, cf.CF_F32, 1, NMK, 8), cf.desc(9, 8, cf.CF_BF16, 4, NMK, 8), cf.desc(130, 264, cf.CF_BF16, 2, CH),
             cf.desc(203, 1104, cf.CF_BF16, 2, NMK, 16), cf.desc(67, 3072, cf.CF_BF16, 1, NMK, 16)]
    streams = [drift_stream((int(d.n_tokens), int(d.n_channels)), int(d.dtype), 4, 60 + t, device=DEV) for t, d in enumerate(descs)]
    for flags in (0, cf.CF_FLAG_SINGLE_PASS, cf.CF_FLAG_TWO_KERNEL):
        for mode in ("fused", "split"):
            say(f"nm mixed batch flags={flags} mode={mode}")
            run_parity(descs, cf.options(flags=flags), [[s[k] for s in streams] for k in range(4)], mode=mode, tag="nm mixed")


# ---------------------------------------------------------------- HIP graph capture

@pytest.mark.parametrize("flags", [0, cf.CF_FLAG_TWO_KERNEL])
def test_step_replays_from_a_hip_graph(flags):
    """A serving loop can capture one cf_step_fused call in a HIP graph and replay it every step: the call
    allocates nothing, clears its scratch with a fill kernel and passes its pointers in kernel arguments.  Every
    replay is checked against an eager context fed the same inputs (default path: the single-pass kernel, one
    workgroup per item; and the two-kernel path), with eager work and synchronisations between the replays."""
    descs = [cf.desc(2048, 1024, cf.CF_BF16, (1, 2, 4)[t % 3], CH) for t in range(3)]
    descs += [cf.desc(300, 1152, cf.CF_BF16, 4, GR), cf.desc(203, 1096, cf.CF_BF16, 2, NMK, 8)]
    steps = 6
    streams = [drift_stream((int(d.n_tokens), int(d.n_channels)), int(d.dtype), steps, 800 + t, device=DEV) for t, d in enumerate(descs)]
    eager = CodecSession(descs, cf.options(flags=flags), device=DEV)
    graphed = CodecSession(descs, cf.options(flags=flags), device=DEV)
    try:
        first = [s[0] for s in streams]
        eager.warmup(first)
        graphed.warmup(first)
        static_x = [s[1].clone() for s in streams]
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):                     # step 1 eagerly on the capture stream's side (uploads the pointer table)
            graphed.step_fused(static_x)
        torch.cuda.current_stream().wait_stream(side)
        eager.step_fused([s[1] for s in streams])
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            graphed.step_fused(static_x)
        for k in range(2, steps):
            for t in range(len(descs)):
                static_x[t].copy_(streams[t][k])
            g.replay()
            cf.cf_check_device(graphed.ctx, graphed.stream_handle)
            eager.step_fused([s[k] for s in streams])
            cf.cf_check_device(eager.ctx, eager.stream_handle)
            for t in range(len(descs)):
                for name in ("codes", "scales", "recon", "err"):
                    a, b = getattr(graphed, name)[t], getattr(eager, name)[t]
                    if name == "codes" and descs[t].scale == NMK:      # the pad between masks and values is never written
                        n_mask = int(descs[t].n_tokens) * int(descs[t].n_channels) // 8
                        a, b = a.clone(), b.clone()
                        a[n_mask:(n_mask + 15) // 16 * 16] = 0
                        b[n_mask:(n_mask + 15) // 16 * 16] = 0
                    assert torch.equal(a.view(torch.uint8).reshape(-1), b.view(torch.uint8).reshape(-1)), \
                        f"replay {k}: {name}[{t}] differs from the eager run"
            say(f"graph replay {k} (flags={flags}) matches the eager run")
    finally:
        eager.close()
        graphed.close()
