"""cf_step_fused_static, the entry point for callers that cannot allocate device memory: through the C ABI,
against cf_step_fused (the existing entry point it is a variant of), bit for bit in every output, on calls in a
row that share the library's static scratch -- the second with a smaller input, the third back to the first."""
import pytest
import torch

import paper_2507_17511_amd as cf
from helpers import drift_stream
from paper_2507_17511_amd.session import CodecSession

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
_DT = {cf.CF_F32: torch.float32, cf.CF_BF16: torch.bfloat16}


class StaticState:
    """Caller-owned state and outputs for the static entry point (allocated up front, as such a caller would)."""

    def __init__(self, descs, opts, x0):
        self.descs, self.opts = list(descs), opts
        self.recon = [x.clone() for x in x0]                                    # recon_0 = x_0
        self.err = [torch.zeros(x.shape, dtype=_DT[opts.err_dtype], device=DEV) for x in x0]      # e_0 = 0
        self.codes, self.scales = [], []
        for d in self.descs:
            cb, sb, _, _ = cf.cf_sizes(d, opts)
            self.codes.append(torch.zeros(cb, dtype=torch.uint8, device=DEV))
            self.scales.append(torch.zeros(max(sb // 4, 1), dtype=torch.float32, device=DEV))

    def step(self, x):
        cf.cf_step_fused_static(self.descs, self.opts, x, self.recon, self.err, self.codes, self.scales,
                                torch.cuda.current_stream().cuda_stream)


def same_bits(a: torch.Tensor, b: torch.Tensor) -> bool:
    return torch.equal(a.contiguous().view(torch.uint8).reshape(-1), b.contiguous().view(torch.uint8).reshape(-1))


def compare(tag, st: StaticState, sess: CodecSession):
    torch.cuda.synchronize()
    for t, d in enumerate(st.descs):
        assert same_bits(st.recon[t], sess.recon[t]), f"{tag}: recon[{t}] differs from cf_step_fused"
        assert same_bits(st.err[t], sess.err[t]), f"{tag}: err[{t}] differs"
        got, want = st.codes[t], sess.codes[t].reshape(-1)
        if d.scale == cf.CF_SPARSE_NM:          # the bytes between the masks and the 16-byte aligned values are never written
            n_mask = int(d.n_tokens) * int(d.n_channels) // 8
            got, want = got.clone(), want.clone()
            got[n_mask:(n_mask + 15) // 16 * 16] = 0
            want[n_mask:(n_mask + 15) // 16 * 16] = 0
        assert same_bits(got, want), f"{tag}: codes[{t}] differ"
        if sess.scales[t].numel():
            assert same_bits(st.scales[t][:sess.scales[t].numel()], sess.scales[t]), f"{tag}: scales[{t}] differ"


def test_static_entry_point_matches_cf_step_fused_on_calls_in_a_row():
    opts = cf.options()
    big = [cf.desc(2048, 1024, cf.CF_BF16, 1, cf.CF_SCALE_CHANNEL),        # 64 items: the single-pass kernel, its partials in the scratch
           cf.desc(300, 384, cf.CF_BF16, 4, cf.CF_SCALE_GROUP, 128),
           cf.desc(130, 1096, cf.CF_BF16, 2, cf.CF_SPARSE_NM, 8),
           cf.desc(517, 264, cf.CF_BF16, 2, cf.CF_SCALE_CHANNEL)]
    small = [cf.desc(256, 64, cf.CF_F32, 2, cf.CF_SCALE_CHANNEL), cf.desc(96, 384, cf.CF_BF16, 4, cf.CF_SCALE_GROUP, 128)]
    assert 0 < cf.cf_workspace_bytes(small, opts) < cf.cf_workspace_bytes(big, opts) <= cf.CF_STATIC_SCRATCH_BYTES
    xs_big = [drift_stream((int(d.n_tokens), int(d.n_channels)), int(d.dtype), 4, 500 + t) for t, d in enumerate(big)]
    xs_small = [drift_stream((int(d.n_tokens), int(d.n_channels)), int(d.dtype), 3, 600 + t) for t, d in enumerate(small)]
    ref_big, ref_small = CodecSession(big, opts, device=DEV), CodecSession(small, opts, device=DEV)
    try:
        ref_big.warmup([x[0] for x in xs_big])
        ref_small.warmup([x[0] for x in xs_small])
        st_big = StaticState(big, opts, [x[0] for x in xs_big])
        st_small = StaticState(small, opts, [x[0] for x in xs_small])
        # call 1: the larger input
        ref_big.step_fused([x[1] for x in xs_big])
        st_big.step([x[1] for x in xs_big])
        compare("call 1 (large)", st_big, ref_big)
        # call 2, straight after: a smaller input over the same scratch (other tables, other partial sizes)
        ref_small.step_fused([x[1] for x in xs_small])
        st_small.step([x[1] for x in xs_small])
        compare("call 2 (small)", st_small, ref_small)
        # calls 3 and 4: back to the large tensors, then the small ones again; state carries on in the caller's buffers
        ref_big.step_fused([x[2] for x in xs_big])
        st_big.step([x[2] for x in xs_big])
        compare("call 3 (large again)", st_big, ref_big)
        ref_small.step_fused([x[2] for x in xs_small])
        st_small.step([x[2] for x in xs_small])
        compare("call 4 (small again)", st_small, ref_small)
        # the same tensors twice in a row (tables reused)
        ref_big.step_fused([x[3] for x in xs_big])
        st_big.step([x[3] for x in xs_big])
        compare("call 5 (large, tables kept)", st_big, ref_big)
        cf.cf_check_device(ref_big.ctx, ref_big.stream_handle)
    finally:
        ref_big.close()
        ref_small.close()


def test_static_entry_point_rejects_what_its_scratch_cannot_hold():
    opts = cf.options()
    many = [cf.desc(4096, 3072, cf.CF_BF16, 2, cf.CF_SCALE_CHANNEL) for _ in range(40)]
    assert cf.cf_workspace_bytes(many, opts) > cf.CF_STATIC_SCRATCH_BYTES
    null = [0] * len(many)
    with pytest.raises(cf.CFError) as ei:       # validated before any pointer is looked at
        cf.cf_step_fused_static(many, opts, null, null, null, null, null, None)
    assert ei.value.status == cf.CF_ERR_WORKSPACE
    with pytest.raises(cf.CFError) as ei:
        cf.cf_step_fused_static([cf.desc(64, 100, cf.CF_BF16, 2, cf.CF_SCALE_CHANNEL)], opts, [0], [0], [0], [0], [0], None)
    assert ei.value.status == cf.CF_ERR_SHAPE
