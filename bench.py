#!/usr/bin/env python3
"""Benchmark of the fused residual codec on one MI355X.

A step is one cf_step_fused call over ALL layer tensors of a workload (the whole
hot path: residual, error feedback, scales, codes, packing, decode, error and
reconstruction update), with the step's activations already resident in HBM.
The metric is algorithmic GB/s through the codec: every input read once and
every output written once, per element
    x + recon(read) + recon(write) + err(write) + bits/8 + scales,
divided by the wall time of a step; it is reported against the 8 TB/s HBM peak.

Prints ONE JSON line: metric, value (GB/s), ms_per_step, config, per-kernel times
from HIP events, `roofline` (the dominant kernel: its algorithmic bytes per launch
over its measured duration against the HBM peak, plus the HBM traffic a committed
rocprofv3 counter run recorded for it), `cpu_baseline` (the CPU oracle on a bounded
sample) and, with the default --workload all, one entry per configuration.  Inputs
are seeded synthetic activation streams (workloads/), standing in for FLUX.1-dev
and CogVideoX-2b activations.
"""
from __future__ import annotations

import argparse
import ctypes
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0   # MI355X HBM3E, published peak

DEFAULT_WORKLOAD = "cfg3_kv_fullseq"


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="all", help="one of workloads.CONFIGS, or all (every config; the headline is cfg3_kv_fullseq)")
    ap.add_argument("--ef", type=int, default=0, help="cf_ef_mode (0 = RECON)")
    ap.add_argument("--flags", type=int, default=0, help="cf_options.flags")
    ap.add_argument("--err-dtype", default="f32", choices=("f32", "bf16"), help="dtype of the error buffer (the metric is quoted with f32)")
    ap.add_argument("--tile-rows", type=int, default=0)
    ap.add_argument("--encode-rows", type=int, default=0)
    ap.add_argument("--tensors", type=int, default=0, help="override the workload's tensor count (exploration only)")
    ap.add_argument("--nm-block", type=int, default=8, choices=(8, 16), help="with --scale nm: channels per block")
    ap.add_argument("--scale", default="", choices=("", "channel", "group", "rank1", "nm", "lowrank"), help="override the workload's scale kind (exploration only)")
    ap.add_argument("--bits", type=int, default=0, help="override the workload's code width (exploration only)")
    ap.add_argument("--split", action="store_true", help="time cf_compress + cf_decompress (sender and receiver halves) instead of cf_step_fused (exploration only)")
    ap.add_argument("--sub-batch", type=int, default=0, help="issue the step as calls over ranges of this many tensors (exploration only)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-kernel-events", action="store_true")
    ap.add_argument("--quiet", action="store_true")
    return ap.parse_args()


def log(args, *a):
    if not args.quiet:
        print(*a, file=sys.stderr, flush=True)


# ------------------------------------------------------------------ HIP events (for per-kernel durations)

class HipEvents:
    def __init__(self):
        self.hip = ctypes.CDLL("libamdhip64.so.7")   # the runtime torch already loaded
        self.hip.hipEventCreate.argtypes = [ctypes.POINTER(ctypes.c_void_p)]
        self.hip.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p, ctypes.c_void_p]
        self.hip.hipEventDestroy.argtypes = [ctypes.c_void_p]
        self.hip.hipEventSynchronize.argtypes = [ctypes.c_void_p]
        self.all = []

    def create(self, n):
        out = []
        for _ in range(n):
            e = ctypes.c_void_p()
            rc = self.hip.hipEventCreate(ctypes.byref(e))
            if rc != 0:
                raise RuntimeError(f"hipEventCreate failed: {rc}")
            out.append(e.value)
            self.all.append(e.value)
        return out

    def elapsed_ms(self, a, b) -> float:
        ms = ctypes.c_float()
        rc = self.hip.hipEventElapsedTime(ctypes.byref(ms), a, b)
        if rc != 0:
            raise RuntimeError(f"hipEventElapsedTime failed: {rc}")
        return float(ms.value)

    def destroy(self):
        for e in self.all:
            self.hip.hipEventDestroy(e)
        self.all = []


# ------------------------------------------------------------------ workload accounting

ERR_BYTES = 4       # bytes of one error-buffer element (set from --err-dtype)
LOWRANK_INT4 = False    # --flags has CF_FLAG_LOWRANK_INT4: 20 bytes per factor row instead of 32 values


def bytes_per_element(wl, bits: int, ef: int) -> float:
    err_bytes = ERR_BYTES
    sx = 4 if wl.dtype == "f32" else 2
    b = sx + sx + sx + err_bytes + code_bytes_per_element(wl, bits)     # x, recon read, recon write, err write, codes
    if ef in (1, 2):
        b += err_bytes                                  # LITERAL / OFF also read err
    if ef == 3:
        b -= sx                                         # naive compression never reads recon
    b += scale_bytes_per_element(wl)
    return b


def code_bytes_per_element(wl, bits: int) -> float:
    if wl.scale == "nm":                                # a mask bit per channel and `bits` values per block of `group`
        return 1 / 8.0 + bits * (4 if wl.dtype == "f32" else 2) / float(wl.group)
    if wl.scale == "lowrank":                           # U [N, 32] and V [C, 32] in the storage dtype
        row_bytes = 20 if LOWRANK_INT4 else 32 * (4 if wl.dtype == "f32" else 2)
        return (wl.n_tokens + wl.n_channels) * row_bytes / (wl.n_tokens * wl.n_channels)
    return bits / 8.0


def scale_bytes_per_element(wl) -> float:
    if wl.scale == "nm":
        return 0.0
    if wl.scale == "lowrank":                           # the start matrix Q0 [C, 32] fp32 is an input
        return 32 * 4.0 / wl.n_tokens
    if wl.scale == "group":
        return 4.0 / wl.group
    if wl.scale == "rank1":                             # v[C] and u[N]
        return 4.0 / wl.n_tokens + 4.0 / wl.n_channels
    return 4.0 / wl.n_tokens


def step_bytes(wl, ef: int) -> float:
    per_tensor = wl.n_tokens * wl.n_channels
    return sum(per_tensor * bytes_per_element(wl, wl.bits_of(t), ef) for t in range(wl.n_tensors))


def apply_overrides(wl, args):
    if args.tensors:
        wl = wl.scaled(n_tensors=args.tensors)
    if args.scale:
        wl = wl.scaled(scale=args.scale, group={"nm": args.nm_block, "lowrank": 32}.get(args.scale, wl.group))
    if args.bits:
        wl = wl.scaled(bits=(args.bits,))
    return wl


def run_workload(name: str, args, events: HipEvents | None):
    import torch

    import paper_2507_17511_amd as cf
    from paper_2507_17511_amd.session import CodecSession
    from workloads import CONFIGS, ActivationStream

    wl = CONFIGS[name]
    wl = apply_overrides(wl, args)
    dev = "cuda:0"
    dt = cf.CF_F32 if wl.dtype == "f32" else cf.CF_BF16
    scale = {"group": cf.CF_SCALE_GROUP, "rank1": cf.CF_SCALE_RANK1, "nm": cf.CF_SPARSE_NM,
             "lowrank": cf.CF_LOWRANK}.get(wl.scale, cf.CF_SCALE_CHANNEL)
    descs = [cf.desc(wl.n_tokens, wl.n_channels, dt, wl.bits_of(t), scale, wl.group) for t in range(wl.n_tensors)]
    opts = cf.options(ef=args.ef, flags=args.flags, tile_rows=args.tile_rows, encode_rows=args.encode_rows,
                      err_dtype=cf.CF_BF16 if args.err_dtype == "bf16" else cf.CF_F32)

    t0 = time.time()
    stream = ActivationStream(wl, device=dev)
    x0 = [x.clone() for x in stream.current]
    # a ring of consecutive stream states x_1..x_R; the timed loop walks it back and forth so that
    # every step sees an input one drift step away from the last (real residual statistics)
    R = 4
    ring = [[x.clone() for x in stream.advance()] for _ in range(R)]
    del stream
    torch.cuda.synchronize()
    log(args, f"[{name}] inputs ready in {time.time() - t0:.1f}s "
              f"({wl.n_tensors} x [{wl.n_tokens},{wl.n_channels}] {wl.dtype}, bits {tuple(wl.bits)}, {wl.scale} scale)")

    sess = CodecSession(descs, opts, device=dev)
    if wl.scale == "lowrank":                           # the start matrices the caller draws (Alg. 3, first line)
        g = torch.Generator(device=dev)
        g.manual_seed(wl.seed)
        for q0 in sess.scales:
            q0.copy_(torch.randn(q0.shape, generator=g, device=dev))
    p_ring = [cf.ptr_array(xs) for xs in ring]
    order = list(range(R)) + list(range(R - 2, 0, -1))      # 0 1 2 3 2 1 | 0 1 ...

    sub = args.sub_batch
    if sub:
        def sl(arr, lo, hi):
            return cf.ptr_array([arr[i] for i in range(lo, hi)])
        ranges = [(lo, min(lo + sub, sess.n)) for lo in range(0, sess.n, sub)]
        sub_ptrs = [[(lo, hi - lo, sl(pr, lo, hi), sl(sess.p_recon, lo, hi), sl(sess.p_err, lo, hi),
                      sl(sess.p_codes, lo, hi), sl(sess.p_scales, lo, hi)) for lo, hi in ranges] for pr in p_ring]

    def step(k, on_call=None):
        """on_call(i): called before the i-th entry-point call of the step (the instrumented pass arms its events there)."""
        if on_call is None:
            on_call = lambda i: None
        if sub:
            for lo, cnt, px, pr, pe, pc, ps in sub_ptrs[order[k % len(order)]]:
                cf.cf_step_fused(sess.ctx, lo, cnt, px, pr, pe, pc, ps, sess.stream_handle)
            return
        if args.split:
            on_call(0)
            cf.cf_compress(sess.ctx, 0, sess.n, p_ring[order[k % len(order)]], sess.p_recon, sess.p_err,
                           sess.p_codes, sess.p_scales, sess.stream_handle)
            on_call(1)
            cf.cf_decompress(sess.ctx, 0, sess.n, sess.p_codes, sess.p_scales, sess.p_recon, sess.stream_handle)
            on_call(2)
            return
        on_call(0)
        cf.cf_step_fused(sess.ctx, 0, sess.n, p_ring[order[k % len(order)]], sess.p_recon, sess.p_err,
                         sess.p_codes, sess.p_scales, sess.stream_handle)

    sess.warmup(x0)
    k = 0
    verified = None
    for w in range(args.warmup):
        step(k); k += 1
        if w == 0 and not args.no_cpu_baseline and wl.scale != "lowrank":
            # outside the timed region: the first tensor's outputs of this step against the CPU oracle, bit for bit
            verified = verify_first_tensor(wl, args, sess, x0[0], ring[order[0]][0])
    torch.cuda.synchronize()
    t_start = time.perf_counter()
    for _ in range(args.steps):
        step(k); k += 1
    torch.cuda.synchronize()
    wall = time.perf_counter() - t_start
    ms_per_step = wall * 1e3 / args.steps

    nbytes = step_bytes(wl, args.ef)
    act_bytes = wl.n_tensors * wl.n_tokens * wl.n_channels * (4 if wl.dtype == "f32" else 2)
    res = {
        "workload": name,
        "ms_per_step": ms_per_step,
        "algorithmic_bytes_per_step": nbytes,
        "gbps": nbytes / (ms_per_step * 1e-3) / 1e9,
        "activation_gbps": act_bytes / (ms_per_step * 1e-3) / 1e9,
        "bytes_per_element": nbytes / (wl.n_tensors * wl.n_tokens * wl.n_channels),
    }
    res["frac_of_hbm_peak"] = res["gbps"] / HBM_PEAK_GBPS

    # second, instrumented pass: HIP events around every kernel the library launches, on its stream
    if events is not None:
        n_prof = min(args.steps, 10)
        # one event set per entry-point call (a split step makes two; a sub-batched one is not instrumented per call)
        sets = [[events.create(32) for _ in range(2)] for _ in range(n_prof)]
        names = [[[], []] for _ in range(n_prof)]
        for s in range(n_prof):
            def on_call(i, s=s):
                if i > 0:           # collect the names of the call that just ended
                    n_launch = min(cf.cf_profile_launch_count(sess.ctx), 16)
                    names[s][i - 1] = [cf.cf_profile_kernel_name(sess.ctx, j) for j in range(n_launch)]
                if i < 2 and (i == 0 or args.split):
                    cf.cf_profile_next_call(sess.ctx, sets[s][i], 16)
            if sub:
                cf.cf_profile_next_call(sess.ctx, sets[s][0], 16)
                step(k)
            else:
                step(k, on_call)
                if not args.split:
                    on_call(1)
            k += 1
            if sub:
                n_launch = min(cf.cf_profile_launch_count(sess.ctx), 16)
                names[s][0] = [cf.cf_profile_kernel_name(sess.ctx, j) for j in range(n_launch)]
        torch.cuda.synchronize()
        per_kernel = {}
        for s in range(n_prof):
            for c in range(2):
                for i, nm in enumerate(names[s][c]):
                    per_kernel.setdefault(nm, []).append(events.elapsed_ms(sets[s][c][2 * i], sets[s][c][2 * i + 1]))
        res["kernel_ms"] = {nm: sum(v) / len(v) for nm, v in per_kernel.items()}
        res["kernel_launches_per_step"] = {nm: len(v) / n_prof for nm, v in per_kernel.items()}
    cf.cf_check_device(sess.ctx, sess.stream_handle)           # raises if anything went wrong on the device
    res["given_up_items_last_step"] = cf.cf_given_up_items(sess.ctx, sess.stream_handle)
    res["first_step_matches_oracle"] = verified
    sess.close()
    del sess, ring, x0
    torch.cuda.empty_cache()
    return res, wl


def verify_first_tensor(wl, args, sess, x0, x1) -> bool:
    """Tensor 0 after warm-up with x0 and one codec step with x1: codes, scales, error buffer and reconstruction must
    be the CPU oracle's bits.  Raises on a mismatch (a wrong kernel must not produce a benchmark line)."""
    import numpy as np
    import torch

    import oracle
    from workloads import as_numpy

    torch.cuda.synchronize()
    scale = {"group": oracle.SCALE_GROUP, "rank1": oracle.SCALE_RANK1, "nm": oracle.SPARSE_NM}.get(wl.scale, oracle.SCALE_CHANNEL)
    cfg = oracle.Config(wl.n_tokens, wl.n_channels, dtype=oracle.F32 if wl.dtype == "f32" else oracle.BF16, bits=wl.bits_of(0),
                        scale=scale, group=wl.group, ef=0 if args.ef == 3 else args.ef,
                        err_dtype=oracle.BF16 if args.err_dtype == "bf16" else oracle.F32)
    if args.ef == 3:        # naive compression is a function of its own in the oracle: reconstruction, codes, scales
        recon, codes, scales = oracle.naive(cfg, as_numpy(x1))
        err = None
    else:
        recon, err = oracle.warmup(cfg, as_numpy(x0))
        codes, scales = oracle.step(cfg, as_numpy(x1), recon, err)
    got_codes = as_numpy(sess.codes[0]).reshape(-1).copy()
    if wl.scale == "nm":            # the bytes between the masks and the 16-byte aligned values are never written
        n_mask = wl.n_tokens * wl.n_channels // 8
        got_codes[n_mask:(n_mask + 15) // 16 * 16] = 0
    checks = {"codes": np.array_equal(got_codes, codes.reshape(-1)),
              "scales": np.array_equal(as_numpy(sess.scales[0]).view(np.uint32).reshape(-1), scales.view(np.uint32).reshape(-1)),
              "recon": np.array_equal(as_numpy(sess.recon[0]).reshape(-1), recon.reshape(-1))}
    if err is not None:
        checks["err"] = np.array_equal(as_numpy(sess.err[0]).reshape(-1), err.reshape(-1))
    bad = [name for name, ok in checks.items() if not ok]
    if bad:
        raise RuntimeError(f"{wl.name}: tensor 0 differs from the CPU oracle after the first step in {bad}")
    return True


def dominant_kernel(res):
    km = res.get("kernel_ms") or {}
    if not km:
        return None, None
    nm = max(km, key=lambda n: km[n] * res["kernel_launches_per_step"][n])
    return nm, km[nm]


def kernel_algorithmic_bytes(nm: str, wl, ef: int, split: bool = False) -> float:
    """Algorithmic bytes one launch of kernel `nm` moves (every operand of that kernel once).  split: the step runs
    as cf_compress + cf_decompress, so the sender's kernels do not write the reconstruction."""
    total = 0.0
    for t in range(wl.n_tensors):
        n = wl.n_tokens * wl.n_channels
        sx = 4 if wl.dtype == "f32" else 2
        bits = wl.bits_of(t)
        scale_b = scale_bytes_per_element(wl)
        if nm == "k_colreduce":
            per = (1 if ef == 3 else 2) * sx + (ERR_BYTES if ef in (1, 2) else 0)
        elif nm in ("k_encode", "k_encode_nm"):     # reads x, recon (+err); writes codes, err, recon
            per = (2 if split else 3) * sx + ERR_BYTES + code_bytes_per_element(wl, bits) + (ERR_BYTES if ef in (1, 2) else 0) + scale_b
            if ef == 3:
                per -= sx
        elif nm in ("k_lr_project", "k_lr_backproject"):     # re-form A from x and recon
            per = 2 * sx
        elif nm == "k_lr_apply":                            # reads x, recon and the factors; writes err, recon
            per = (2 if split else 3) * sx + ERR_BYTES + code_bytes_per_element(wl, bits)
        elif nm == "k_decode":
            per = 2 * sx + code_bytes_per_element(wl, bits) + scale_b
        else:                            # a kernel that does the whole step (the sender's half of it when split)
            per = bytes_per_element(wl, bits, ef) - (sx if split else 0)
        total += n * per
    return total


def cpu_baseline(wl, ef: int, budget_s: float = 15.0):
    """The oracle as it stands, single-threaded, on a bounded sample of the same workload."""
    import numpy as np
    import torch

    import oracle
    from workloads import ActivationStream, as_numpy

    small = wl.scaled(n_tensors=min(wl.n_tensors, 3))
    stream = ActivationStream(small, device="cpu")
    cfgs = [oracle.Config(wl.n_tokens, wl.n_channels, dtype=oracle.F32 if wl.dtype == "f32" else oracle.BF16,
                          bits=wl.bits_of(t), scale={"group": oracle.SCALE_GROUP, "rank1": oracle.SCALE_RANK1, "nm": oracle.SPARSE_NM}.get(wl.scale, oracle.SCALE_CHANNEL),
                          group=wl.group, ef=ef) for t in range(small.n_tensors)]
    state = [oracle.warmup(cfgs[t], as_numpy(stream.current[t])) for t in range(small.n_tensors)]
    done, spent, nbytes = 0, 0.0, 0.0
    while spent < budget_s and done < 64:
        xs = [as_numpy(x) for x in stream.advance()]
        for t in range(small.n_tensors):
            t0 = time.perf_counter()
            oracle.step(cfgs[t], xs[t], state[t][0], state[t][1])
            spent += time.perf_counter() - t0
            nbytes += wl.n_tokens * wl.n_channels * bytes_per_element(wl, wl.bits_of(t), ef)
            done += 1
            if spent >= budget_s:
                break
    return {"value": nbytes / spent / 1e9, "unit": "GB/s", "cores": 1, "kind": "oracle",
            "sample": f"{done} tensor-steps of [{wl.n_tokens},{wl.n_channels}] {wl.dtype} from {wl.name} "
                      f"(first {small.n_tensors} layers), {spent:.1f}s single-threaded C oracle",
            "seconds_per_tensor_step": spent / done}


def source_fingerprint() -> str:
    """Hash of the library's sources: a recorded profile only describes the kernels it was taken from."""
    import glob
    import hashlib
    h = hashlib.sha256()
    for path in sorted(glob.glob(os.path.join(ROOT, "paper_2507_17511_amd", "csrc", "*"))):
        h.update(os.path.basename(path).encode())
        h.update(open(path, "rb").read())
    return h.hexdigest()[:12]


def read_traffic(kernel: str, workload: str):
    """HBM bytes per launch from the committed rocprofv3 --pmc summary of this kernel and workload: a RECORDED value
    (the counters cannot be read inside this run), used only if it was taken from the sources as they are now.
    -> (bytes or None, note)"""
    rel = os.path.join("profiles", f"traffic_{kernel}_{workload}.txt")
    path = os.path.join(ROOT, rel)
    if not os.path.exists(path):
        return None, "no recorded counter run for this kernel and workload"
    value, recorded = None, None
    for line in open(path):
        if line.startswith("hbm_bytes_per_launch:"):
            value = float(line.split(":")[1])
        if line.startswith("source_fingerprint:"):
            recorded = line.split(":")[1].strip()
    now = source_fingerprint()
    if recorded != now:
        return None, f"{rel} was recorded for sources {recorded}, these are {now}: not used"
    return value, f"recorded in {rel} (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, sources {recorded}); not measured in this run"


def main():
    global ERR_BYTES, LOWRANK_INT4
    args = parse_args()
    ERR_BYTES = 2 if args.err_dtype == "bf16" else 4
    LOWRANK_INT4 = bool(args.flags & 0x4)
    if args.gpus != 1:
        print("bench.py: this build measures ONE GPU only (the packed-code buffer in HBM stands in for the wire; "
              "there is no multi-GPU path): run with --gpus 1", file=sys.stderr)
        sys.exit(2)
    import torch

    import paper_2507_17511_amd as cf
    from workloads import CONFIGS
    cf.lib()
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    events = None if args.no_kernel_events else HipEvents()

    names = list(CONFIGS) if args.workload == "all" else [args.workload]
    results = {}
    for nm in names:
        r, wl = run_workload(nm, args, events)
        results[nm] = (r, wl)
        log(args, f"[{nm}] {r['ms_per_step']:.3f} ms/step  {r['gbps']:.0f} GB/s algorithmic "
                  f"({100 * r['frac_of_hbm_peak']:.1f}% of {HBM_PEAK_GBPS:.0f})  kernels: {r.get('kernel_ms')}")
    head = DEFAULT_WORKLOAD if args.workload == "all" else args.workload
    r, wl = results[head]

    kname, kms = dominant_kernel(r)
    roofline = None
    if kname is not None:
        kb = kernel_algorithmic_bytes(kname, wl, args.ef, args.split)
        achieved = kb / (kms * 1e-3) / 1e9
        if args.scale or args.bits or args.tensors or args.ef or args.split or args.flags or args.err_dtype != "f32":
            traffic, traffic_note = None, "counter runs are recorded for the default options only"
        else:
            traffic, traffic_note = read_traffic(kname, head)
        roofline = {"bound": "hbm", "kernel": kname, "achieved": achieved, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                    "frac": achieved / HBM_PEAK_GBPS, "traffic": traffic, "traffic_source": traffic_note,
                    "algorithmic_bytes_per_launch": kb, "avg_launch_ms": kms}
    mfma = None
    if wl.scale == "lowrank" and r.get("kernel_ms"):        # the dense contractions: 2 * 32 flops per element and launch
        flops = 2.0 * 32 * wl.n_tensors * wl.n_tokens * wl.n_channels
        mfma = {nm: {"tflops": flops / (ms * 1e-3) / 1e12, "peak_fp32_mfma": 157.3, "frac": flops / (ms * 1e-3) / 1e12 / 157.3}
                for nm, ms in r["kernel_ms"].items() if nm in ("k_lr_project", "k_lr_backproject", "k_lr_apply")}
    cpu = None if (args.no_cpu_baseline or wl.scale == "lowrank" or args.err_dtype != "f32") else cpu_baseline(wl, args.ef)
    if events is not None:
        events.destroy()

    out = {
        "metric": "activation GB/s through fused residual codec (% of MI355X HBM peak)",
        "value": r["gbps"], "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": r["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": head, "tensors": wl.n_tensors, "shape": [wl.n_tokens, wl.n_channels],
                   "storage": wl.dtype, "bits": list(wl.bits), "scale": wl.scale, "ef_mode": args.ef,
                   "launch": "one cf_step_fused call per step over all tensors"},
        "pct_of_hbm_peak": 100.0 * r["frac_of_hbm_peak"],
        "activation_gbps": r["activation_gbps"],
        "bytes_per_element": r["bytes_per_element"],
        "kernel_ms": r.get("kernel_ms"),
        "roofline": roofline,
        "mfma": mfma,
        "cpu_baseline": cpu,
        "first_step_matches_oracle": r.get("first_step_matches_oracle"),
        "source_fingerprint": source_fingerprint(),
    }
    if len(results) > 1:
        out["all_workloads"] = {nm: {k: v for k, v in rr.items() if k != "workload"} for nm, (rr, _) in results.items()}
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
