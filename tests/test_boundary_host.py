"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every
symbol the header declares, sizes buffers correctly and rejects bad descriptors
before touching a device."""
import ctypes
import os
import re

import pytest

import paper_2507_17511_amd as cf

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "compactfusion.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(cf_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = declared_functions()
    assert {"cf_init", "cf_compress", "cf_decompress", "cf_step_fused"} <= set(names)
    L = ctypes.CDLL(cf.LIB_PATH)
    for n in names:
        assert hasattr(L, n), f"{n} is declared in compactfusion.h but not exported"
    assert sorted(cf.EXPORTS) == names
    for n in names:
        assert callable(getattr(cf, n)), f"binding lacks {n}"


def test_status_strings():
    seen = {cf.cf_status_string(s) for s in range(7)}
    assert len(seen) == 7 and "ok" in seen
    assert cf.cf_status_string(99) == "unknown status"


def test_sizes_follow_the_layouts():
    # codes: N * C * bits / 8 bytes, i.e. 16x / 8x / 4x smaller than 16-bit activations
    for bits, ratio in ((1, 16), (2, 8), (4, 4)):
        d = cf.desc(4096, 3072, cf.CF_BF16, bits, cf.CF_SCALE_CHANNEL)
        codes, scales, recon, err = cf.cf_sizes(d)
        assert codes * ratio == 4096 * 3072 * 2
        assert scales == 3072 * 4 and recon == 4096 * 3072 * 2 and err == 4096 * 3072 * 4
    d = cf.desc(16384, 3072, cf.CF_BF16, 4, cf.CF_SCALE_GROUP, 128)
    codes, scales, recon, err = cf.cf_sizes(d, cf.options(err_dtype=cf.CF_BF16))
    assert codes == 16384 * 3072 // 2 and scales == 16384 * 24 * 4 and err == recon == 16384 * 3072 * 2
    d = cf.desc(256, 64, cf.CF_F32, 2)
    assert cf.cf_sizes(d) == (256 * 16, 64 * 4, 256 * 64 * 4, 256 * 64 * 4)
    d = cf.desc(4096, 3072, cf.CF_BF16, 2, cf.CF_SCALE_RANK1)          # v[C] then u[N]
    assert cf.cf_sizes(d)[1] == (3072 + 4096) * 4
    # the workspace of a rank-1 tensor also holds one partial row sum per token and column tile
    two = cf.options(flags=cf.CF_FLAG_TWO_KERNEL)
    ch = cf.cf_workspace_bytes([cf.desc(4096, 3072, cf.CF_BF16, 2, cf.CF_SCALE_CHANNEL)], two)
    assert cf.cf_workspace_bytes([d], two) >= ch + 4096 * 3 * 4


BAD = [
    (cf.desc(0, 64), cf.CF_ERR_SHAPE),
    (cf.desc(16, 4), cf.CF_ERR_SHAPE),
    (cf.desc(16, 12), cf.CF_ERR_SHAPE),
    (cf.desc(16, 192, cf.CF_BF16, 4, cf.CF_SCALE_GROUP, 128), cf.CF_ERR_SHAPE),     # C % group
    (cf.desc(16, 256, cf.CF_BF16, 4, cf.CF_SCALE_GROUP, 64), cf.CF_ERR_SHAPE),      # group != 128
    (cf.desc(16, 256, cf.CF_BF16, 2, cf.CF_SCALE_GROUP, 128), cf.CF_ERR_UNSUPPORTED),
    (cf.desc(16, 64, cf.CF_BF16, 3), cf.CF_ERR_UNSUPPORTED),
    (cf.desc(16, 64, 7, 2), cf.CF_ERR_UNSUPPORTED),
    (cf.desc(16, 64, cf.CF_BF16, 2, 9), cf.CF_ERR_UNSUPPORTED),
    (cf.desc(16, 64, cf.CF_BF16, 4, cf.CF_SCALE_RANK1), cf.CF_ERR_UNSUPPORTED),         # u v^T goes with 1-/2-bit codes
    (cf.desc(16, 128 * 1024 + 8, cf.CF_BF16, 2, cf.CF_SCALE_RANK1), cf.CF_ERR_SHAPE),   # more than 128 column tiles
]


@pytest.mark.parametrize("d,status", BAD)
def test_bad_descriptors_are_rejected_before_any_device_work(d, status):
    with pytest.raises(cf.CFError) as ei:
        cf.cf_sizes(d)
    assert ei.value.status == status
    assert cf.cf_workspace_bytes([d]) == 0
    with pytest.raises(cf.CFError) as ei:
        cf.cf_init([cf.desc(16, 64), d], None, 0x1000, 1 << 30)
    assert ei.value.status == status


def test_bad_options_and_workspace():
    good = cf.desc(64, 128)
    for opts in (cf.options(ef=5), cf.options(err_dtype=3), cf.options(flags=0x80), cf.options(tile_rows=12)):
        with pytest.raises(cf.CFError) as ei:
            cf.cf_sizes(good, opts)
        assert ei.value.status == cf.CF_ERR_UNSUPPORTED
        assert cf.cf_workspace_bytes([good], opts) == 0
    need = cf.cf_workspace_bytes([good])
    assert need > 0 and need % 256 == 0
    for ws, nbytes in ((None, need), (0x1010, need), (0x1000, need - 1)):
        with pytest.raises(cf.CFError) as ei:
            cf.cf_init([good], None, ws, nbytes)
        assert ei.value.status == cf.CF_ERR_WORKSPACE
    with pytest.raises(cf.CFError) as ei:
        cf.cf_init([], None, 0x1000, 1 << 20)
    assert ei.value.status == cf.CF_ERR_INVALID_ARG


def test_workspace_grows_with_channel_scale_partials():
    ch = cf.desc(4096, 3072, cf.CF_BF16, 2, cf.CF_SCALE_CHANNEL)
    gr = cf.desc(4096, 3072, cf.CF_BF16, 4, cf.CF_SCALE_GROUP, 128)
    o = cf.options(tile_rows=32)
    a, b = cf.cf_workspace_bytes([ch], o), cf.cf_workspace_bytes([gr], o)
    assert a > b > 0
    # partial sums: one fp32 row of C per tile row-block
    assert a - b >= (4096 // 32) * 3072 * 4
    assert cf.cf_workspace_bytes([ch] * 8, o) > 7 * (a - b)


def test_calls_on_null_context_fail_cleanly():
    p = cf.ptr_array([0x1000])
    for fn, args in ((cf.cf_warmup, (None, 0, 1, p, p, p)), (cf.cf_step_fused, (None, 0, 1, p, p, p, p, p)),
                     (cf.cf_compress, (None, 0, 1, p, p, p, p, p)), (cf.cf_decompress, (None, 0, 1, p, p, p)),
                     (cf.cf_set_warm, (None, 0, 1, True))):
        with pytest.raises(cf.CFError) as ei:
            fn(*args)
        assert ei.value.status == cf.CF_ERR_INVALID_ARG
    cf.cf_destroy(None)
    assert cf.cf_last_hip_error(None) == 0


def test_lowrank_int4_factor_sizes():
    o = cf.options(flags=cf.CF_FLAG_LOWRANK_INT4)
    d = cf.desc(4096, 3072, cf.CF_BF16, 1, cf.CF_LOWRANK, 32)
    assert cf.cf_sizes(d, o)[0] == (4096 + 3072) * 20              # 16 nibble bytes and one fp32 scale per factor row
    assert cf.cf_sizes(d)[0] == (4096 + 3072) * 64
    with pytest.raises(cf.CFError) as ei:
        cf.cf_sizes(d, cf.options(flags=0x40))                           # not a flag
    assert ei.value.status == cf.CF_ERR_UNSUPPORTED


def test_nm_sizes_and_block_lengths():
    for group in (4, 32):
        with pytest.raises(cf.CFError) as ei:
            cf.cf_sizes(cf.desc(16, 64, cf.CF_BF16, 2, cf.CF_SPARSE_NM, group))
        assert ei.value.status == cf.CF_ERR_UNSUPPORTED
    with pytest.raises(cf.CFError) as ei:
        cf.cf_sizes(cf.desc(16, 72, cf.CF_BF16, 2, cf.CF_SPARSE_NM, 16))       # 72 channels are not whole blocks of 16
    assert ei.value.status == cf.CF_ERR_SHAPE
    assert cf.cf_sizes(cf.desc(4096, 3072, cf.CF_BF16, 2, cf.CF_SPARSE_NM, 16))[0] == 4096 * 192 * (2 + 4)
    codes, scales, recon, err = cf.cf_sizes(cf.desc(4096, 3072, cf.CF_BF16, 2, cf.CF_SPARSE_NM, 8))
    assert scales == 0 and codes == 4096 * 384 * (1 + 4)           # 16-byte blocks travel as 5 bytes
    assert cf.cf_sizes(cf.desc(3, 8, cf.CF_F32, 1, cf.CF_SPARSE_NM, 8))[0] == 16 + 3 * 4
