"""GPU parity at the full sizes of configurations 2-5, in the launch shape bench.py times
(one cf_step_fused call per step over ALL layer tensors, default options).

What the oracle checks element by element (it needs about 0.5 s per [4096, 3072] tensor-step, 2 s per
[16384, 3072] one, on one core; eight run side by side):
  * every layer tensor for codec steps 1 and 2, and
  * three sampled layers (first, middle, last; for config 5 one of each code width, for config 3 a K
    and a V tensor) through every codec step (27 for configs 2, 3 and 5, 49 for config 4), on the default
    path and, for config 5, on the two-kernel path as well.
What is checked for EVERY tensor at EVERY step, on the GPU with torch: the telescoping invariant
recon_t + e_t == x_t within half a bf16 ulp of recon_t (the one rounding of the stored
reconstruction), and that no bounded wait expired (cf_check_device).
"""
import sys
import time
from concurrent.futures import ThreadPoolExecutor

import pytest
import torch

import paper_2507_17511_amd as cf
from helpers import OracleState, compare_tensor
from paper_2507_17511_amd.session import CodecSession
from workloads import CONFIGS, ActivationStream, as_numpy

pytestmark = [pytest.mark.gpu, pytest.mark.timeout(900)]      # these follow whole configurations: minutes, not seconds
DEV = "cuda:0"


def say(msg):
    print(f"[case] {msg}", flush=True)
    sys.stdout.flush()


def invariant_holds(sess: CodecSession, xs, t: int) -> bool:
    recon = sess.recon[t].float()
    gap = (recon + sess.err[t] - xs[t].float()).abs()
    bound = recon.abs() * 2.0 ** -8 * 1.01 + 1e-6       # half a bf16 ulp of recon (8 significand bits)
    return bool((gap <= bound).all())


def run_full(name: str, sampled, follow_steps=None, all_layer_steps=2, flags=0):
    wl = CONFIGS[name]
    scale = cf.CF_SCALE_GROUP if wl.scale == "group" else cf.CF_SCALE_CHANNEL
    descs = [cf.desc(wl.n_tokens, wl.n_channels, cf.CF_BF16, wl.bits_of(t), scale, wl.group) for t in range(wl.n_tensors)]
    opts = cf.options(flags=flags)
    t0 = time.time()
    stream = ActivationStream(wl, device=DEV)
    sess = CodecSession(descs, opts, device=DEV)
    everything = list(range(wl.n_tensors))
    orc = OracleState(descs, opts, everything)
    n_steps = wl.steps if follow_steps is None else min(wl.steps, follow_steps + 1)
    try:
        sess.warmup(stream.current)
        torch.cuda.synchronize()
        with ThreadPoolExecutor(max_workers=8) as pool:
            list(pool.map(lambda t: orc.warmup(t, as_numpy(stream.current[t])), everything))
            for t in everything:
                compare_tensor(f"{name} warm-up", sess, orc, t, check_codes=False)
            say(f"{name}: warm-up of {wl.n_tensors} tensors checked ({time.time() - t0:.0f}s)")
            for s in range(1, n_steps):
                xs = stream.advance()
                cf.cf_step_fused(sess.ctx, 0, sess.n, cf.ptr_array(xs), sess.p_recon, sess.p_err, sess.p_codes,
                                 sess.p_scales, sess.stream_handle)
                cf.cf_check_device(sess.ctx, sess.stream_handle)
                bad = [t for t in everything if not invariant_holds(sess, xs, t)]
                assert not bad, f"{name} step {s}: recon + e != x on tensors {bad[:8]}"
                which = everything if s <= all_layer_steps else list(sampled)
                if s == all_layer_steps + 1:          # drop the oracle state of the layers no longer followed
                    for t in everything:
                        if t not in sampled:
                            orc.recon.pop(t, None); orc.err.pop(t, None); orc.codes.pop(t, None); orc.scales.pop(t, None)
                list(pool.map(lambda t: orc.step(t, as_numpy(xs[t])), which))
                for t in which:
                    compare_tensor(f"{name} step {s}", sess, orc, t)
                say(f"{name}: step {s}/{n_steps - 1}: {len(which)} tensors bit-exact, invariant on all "
                    f"({time.time() - t0:.0f}s)")
    finally:
        sess.close()


def test_cfg2_flux_patch_full():
    run_full("cfg2_flux_patch", sampled=(0, 28, 56))


def test_cfg3_kv_fullseq_full():
    run_full("cfg3_kv_fullseq", sampled=(0, 57, 113))          # K of layer 0, V of layer 28, V of layer 56


def test_cfg4_video_full():
    run_full("cfg4_video", sampled=(0, 21, 41))


def test_cfg5_batched_mixed_full():
    run_full("cfg5_batched_mixed", sampled=(0, 28, 56))        # bits 1, 2, 4


def test_cfg5_two_kernel_path_full():
    """The two-kernel path at full size (the default runs the single-pass kernel, whose reduction groups
    span 32 workgroups here)."""
    run_full("cfg5_batched_mixed", sampled=(3, 31, 53), flags=cf.CF_FLAG_TWO_KERNEL)


# ---------------------------------------------------------------- the widened rows at the size of configuration 3

def _full_shape_case(name, descs, opts, seed, steps=3):
    """A few [4096, 3072] bf16 tensors, every one checked against the oracle at every step."""
    t0 = time.time()
    wl = CONFIGS["cfg3_kv_fullseq"].scaled(n_tensors=len(descs), seed=seed)
    stream = ActivationStream(wl, device=DEV)
    sess = CodecSession(descs, opts, device=DEV)
    everything = list(range(len(descs)))
    orc = OracleState(descs, opts, everything)
    try:
        sess.warmup(stream.current)
        with ThreadPoolExecutor(max_workers=8) as pool:
            list(pool.map(lambda t: orc.warmup(t, as_numpy(stream.current[t])), everything))
            for s in range(1, steps + 1):
                xs = stream.advance()
                sess.step_fused(xs)
                cf.cf_check_device(sess.ctx, sess.stream_handle)
                list(pool.map(lambda t: orc.step(t, as_numpy(xs[t])), everything))
                for t in everything:
                    compare_tensor(f"{name} step {s}", sess, orc, t)
                say(f"{name}: step {s}/{steps}: {len(descs)} tensors bit-exact ({time.time() - t0:.0f}s)")
    finally:
        sess.close()


def test_rank1_scales_full_shape():
    descs = [cf.desc(4096, 3072, cf.CF_BF16, 1 + t % 2, cf.CF_SCALE_RANK1) for t in range(6)]
    _full_shape_case("rank-1 scales", descs, cf.options(), seed=21)


def test_nm_sparsifier_full_shape():
    descs = [cf.desc(4096, 3072, cf.CF_BF16, (1, 2, 4)[t % 3], cf.CF_SPARSE_NM, 8) for t in range(6)]
    _full_shape_case("N:M sparsifier", descs, cf.options(), seed=22)


def test_naive_and_no_feedback_full_shape():
    descs = [cf.desc(4096, 3072, cf.CF_BF16, (1, 2, 4)[t % 3], cf.CF_SCALE_CHANNEL) for t in range(3)]
    _full_shape_case("naive", descs, cf.options(ef=cf.CF_EF_NAIVE), seed=23, steps=2)
    _full_shape_case("no feedback", descs, cf.options(ef=cf.CF_EF_OFF), seed=24, steps=2)
