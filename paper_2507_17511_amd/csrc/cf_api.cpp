// C-ABI layer of the residual codec: argument validation, workspace layout,
// per-call pointer tables and kernel sequencing.  No arithmetic of the method
// happens here; see cf_kernels.hip, cf_single_pass.hip and cf_lowrank.hip.  Declarations and their citations of
// arxiv 2507.17511 are in include/compactfusion.h.
#include "compactfusion.h"

#include <cstdint>
#include <cstring>
#include <new>
#include <vector>

#include "cf_internal.h"

using namespace cf;

namespace {

constexpr size_t kAlign = 256;
inline size_t align_up(size_t v) { return (v + kAlign - 1) / kAlign * kAlign; }

struct Layout {
    size_t off_descs = 0, off_ptrs = 0, off_tile_prefix = 0, off_fin_prefix = 0, off_partials = 0;
    size_t off_item_prefix = 0, off_item_tensor = 0, off_gave_up = 0, off_error = 0, off_p_partials = 0;
    std::vector<uint32_t> item_prefix;
    size_t n_items = 0;
    int32_t max_group_items = 0;   // largest reduction group of the single-pass path
    bool sp_wide = false;          // single-pass items are kStripeChannelsWide channels wide (short tensors)
    bool single_pass = false;      // every channel-scale tensor has single-pass geometry
    size_t total = 0;
    std::vector<TensorDev> dev;
    std::vector<uint32_t> tile_prefix, fin_prefix, ew_prefix, dec_prefix;
    size_t off_ew_prefix = 0, off_dec_prefix = 0;
    bool any_channel = false, any_rank1 = false, any_lowrank = false;
    int64_t min_channel_scale_tokens = INT64_MAX;
};

cf_status check_opts(const cf_options *o, cf_options &out)
{
    out.ef = CF_EF_RECON;
    out.err_dtype = CF_F32;
    out.flags = 0;
    out.tile_rows = 0;
    out.encode_rows = 0;
    if (!o) return CF_OK;
    if (o->ef != CF_EF_RECON && o->ef != CF_EF_LITERAL && o->ef != CF_EF_OFF && o->ef != CF_EF_NAIVE) return CF_ERR_UNSUPPORTED;
    if (o->err_dtype != CF_F32 && o->err_dtype != CF_BF16) return CF_ERR_UNSUPPORTED;
    if (o->flags & ~(CF_FLAG_SINGLE_PASS | CF_FLAG_TWO_KERNEL | CF_FLAG_LOWRANK_INT4 | CF_FLAG_FIXED_GRID | CF_FLAG_TEST_NO_WAIT))
        return CF_ERR_UNSUPPORTED;
    if (o->tile_rows != 0 && o->tile_rows != 8 && o->tile_rows != 16 && o->tile_rows != 32 && o->tile_rows != 64)
        return CF_ERR_UNSUPPORTED;
    if (o->encode_rows < 0 || o->encode_rows > 64) return CF_ERR_UNSUPPORTED;
    out = *o;
    return CF_OK;
}

cf_status check_desc(const cf_tensor_desc &d)
{
    if (d.n_tokens < 1 || d.n_channels < 8 || d.n_channels % 8 != 0) return CF_ERR_SHAPE;
    if (d.n_channels > (int64_t)1 << 30 || d.n_tokens > (int64_t)1 << 24) return CF_ERR_SHAPE;
    if (d.n_tokens > ((int64_t)1 << 46) / d.n_channels) return CF_ERR_SHAPE;
    if (d.dtype != CF_F32 && d.dtype != CF_BF16) return CF_ERR_UNSUPPORTED;
    if (d.bits != 1 && d.bits != 2 && d.bits != 4) return CF_ERR_UNSUPPORTED;
    if (d.scale == CF_SCALE_CHANNEL) return CF_OK;
    if (d.scale == CF_SCALE_GROUP) {
        if (d.bits != 4) return CF_ERR_UNSUPPORTED;
        if (d.group != 128 || d.n_channels % 128 != 0) return CF_ERR_SHAPE;
        return CF_OK;
    }
    if (d.scale == CF_LOWRANK) {        // bits = subspace iterations T, group = rank
        if (d.group != kLowRankRank) return CF_ERR_UNSUPPORTED;
        if (d.n_channels % 32 != 0 || d.n_channels > kLowRankMaxChannels) return CF_ERR_SHAPE;
        return CF_OK;
    }
    if (d.scale == CF_SPARSE_NM) {      // bits = N values kept of every group = M channels
        if (d.group != 8 && d.group != 16) return CF_ERR_UNSUPPORTED;
        if (d.n_channels % d.group != 0) return CF_ERR_SHAPE;
        return CF_OK;                   // bits in {1, 2, 4} was checked above
    }
    if (d.scale == CF_SCALE_RANK1) {
        if (d.bits == 4) return CF_ERR_UNSUPPORTED;                  // the paper's u v^T goes with its 1-/2-bit code books
        if (d.n_channels > (int64_t)kMaxRank1Colblocks * kTileChannels) return CF_ERR_SHAPE;
        return CF_OK;
    }
    return CF_ERR_UNSUPPORTED;
}

size_t dtype_size(int32_t dt) { return dt == CF_BF16 ? 2 : 4; }

struct BufferBytes {
    size_t codes, scales, recon, err;      // recon is also the size of x
};

// Byte sizes of one (valid) tensor's buffers.
BufferBytes buffer_bytes(const cf_tensor_desc &d, const cf_options &o)
{
    BufferBytes b;
    const size_t n = (size_t)d.n_tokens, c = (size_t)d.n_channels;
    if (d.scale == CF_LOWRANK) {        // U [N, 32] then V [C, 32] in the storage dtype; the scales entry is the input Q0 [C, 32] fp32
        // 4-bit factors: 16 nibble bytes and one fp32 scale per factor row
        b.codes = (o.flags & CF_FLAG_LOWRANK_INT4) ? (n + c) * 20 : (n + c) * kLowRankRank * dtype_size(d.dtype);
        b.scales = c * kLowRankRank * sizeof(float);
    } else if (d.scale == CF_SPARSE_NM) {      // one mask byte per block of 8, then (16-byte aligned) bits values per block
        b.codes = (n * (c / 8) + 15) / 16 * 16 + n * (c / (size_t)d.group) * (size_t)d.bits * dtype_size(d.dtype);
        b.scales = 0;
    } else {
        b.codes = n * (c * (size_t)d.bits / 8);
        b.scales = sizeof(float) * (d.scale == CF_SCALE_GROUP ? n * (c / 128) : d.scale == CF_SCALE_RANK1 ? c + n : c);
    }
    b.recon = n * c * dtype_size(d.dtype);
    b.err = n * c * dtype_size(o.err_dtype);
    return b;
}

inline bool overlap(const void *a, size_t na, const void *b, size_t nb)
{
    if (!a || !b || na == 0 || nb == 0) return false;
    const uintptr_t pa = reinterpret_cast<uintptr_t>(a), pb = reinterpret_cast<uintptr_t>(b);
    return pa < pb + nb && pb < pa + na;
}

// Rows per tile: as large as still leaves the batched grid a few thousand
// workgroups (256 CUs, several resident workgroups each).
int pick_rb_rows(const cf_tensor_desc *descs, int32_t n, const cf_options &o)
{
    if (o.tile_rows) return o.tile_rows;
    const int cands[] = {64, 32, 16, 8};
    for (int rb : cands) {
        uint64_t tiles = 0;
        for (int32_t t = 0; t < n; ++t) {
            uint64_t rbn = (uint64_t)((descs[t].n_tokens + rb - 1) / rb);
            uint64_t cbn = (uint64_t)((descs[t].n_channels / kChunk + kTileThreads - 1) / kTileThreads);
            tiles += rbn * cbn;
        }
        if (tiles >= 4096) return rb;
    }
    return 8;
}

cf_status make_layout(const cf_tensor_desc *descs, int32_t n, const cf_options &o, Layout &L)
{
    if (!descs || n < 1) return CF_ERR_INVALID_ARG;
    for (int32_t t = 0; t < n; ++t) {
        cf_status st = check_desc(descs[t]);
        if (st != CF_OK) return st;
    }
    const int rb = pick_rb_rows(descs, n, o);
    L.dev.resize(n);
    L.tile_prefix.assign(n + 1, 0);
    L.ew_prefix.assign(n + 1, 0);
    L.dec_prefix.assign(n + 1, 0);
    uint64_t ew_tiles = 0, dec_tiles = 0;
    L.fin_prefix.assign(n + 1, 0);
    uint64_t tiles = 0, fins = 0, items = 0;
    size_t partial_bytes = 0, p_partial_bytes = 0;
    L.item_prefix.assign(n + 1, 0);
    L.single_pass = (o.flags & CF_FLAG_TWO_KERNEL) == 0;
    for (int32_t t = 0; t < n; ++t)
        if (descs[t].scale == CF_SCALE_RANK1) L.single_pass = false;   // the single-pass kernel knows channel scales only
    // Single-pass item shape: 256 lanes, each with single_pass_rows_per_lane rows, cover kStripeChannels channels by
    // default; when even the tallest channel-scale tensor would make at most 12 items per group that way (bf16:
    // N <= 3072), items half as tall and twice as wide measure equal or faster.  [N, 3072] bf16 batches of equal
    // size, 128 -> 256 channels, 1- / 2- / 4-bit codes: N = 1024 1.57 / 1.61 / 1.65 -> 1.47 / 1.55 / 1.52 ms,
    // N = 2048 1.49 / 1.51 / 1.60 -> 1.52 / 1.48 / 1.55, N = 3072 1.47 / 1.52 / 1.61 -> 1.46 / 1.50 / 1.58,
    // N = 4096 1.50 / 1.55 / 1.62 -> 1.53 / 1.56 / 1.65, N = 6144 1.56 / 1.59 / 1.68 -> 1.62 / 1.66 / 1.77.
    auto narrow_item_rows = [&](int32_t dtype) { return (kPersistThreads / (kStripeChannels / kChunk)) * single_pass_rows_per_lane(dtype, o.ef); };
    int64_t narrow_max_group = 0;
    for (int32_t t = 0; t < n; ++t)
        if (descs[t].scale == CF_SCALE_CHANNEL) {
            const int64_t rows = narrow_item_rows(descs[t].dtype);
            const int64_t g = (descs[t].n_tokens + rows - 1) / rows;
            if (g > narrow_max_group) narrow_max_group = g;
        }
    L.sp_wide = L.single_pass && narrow_max_group > 0 && narrow_max_group <= 12;
    const int stripe_channels = L.sp_wide ? kStripeChannelsWide : kStripeChannels;
    for (int32_t t = 0; t < n; ++t) {
        const cf_tensor_desc &d = descs[t];
        TensorDev &v = L.dev[t];
        std::memset(&v, 0, sizeof v);
        v.n_tokens = d.n_tokens;
        v.n_channels = (int32_t)d.n_channels;
        v.n_chunks = (int32_t)(d.n_channels / kChunk);
        v.dtype = d.dtype;
        v.bits = d.bits;
        v.scale = d.scale;
        v.nm_block = d.scale == CF_SPARSE_NM ? (uint32_t)d.group : (d.scale == CF_LOWRANK && (o.flags & CF_FLAG_LOWRANK_INT4)) ? 4u : 0u;
        v.rb_rows = rb;
        v.n_rowblocks = (int32_t)((d.n_tokens + rb - 1) / rb);
        v.n_colblocks = (v.n_chunks + kTileThreads - 1) / kTileThreads;
        v.tile_begin = (uint32_t)tiles;
        v.fin_begin = (uint32_t)fins;
        L.tile_prefix[t] = (uint32_t)tiles;
        L.fin_prefix[t] = (uint32_t)fins;
        tiles += (uint64_t)v.n_rowblocks * (uint64_t)v.n_colblocks;
        // element-wise kernels do best with short-lived workgroups: a lane never has to wait for
        // its own stores before it can use its next loads
        v.ew_rows = 1;
        v.ew_n_rowblocks = (int32_t)((d.n_tokens + v.ew_rows - 1) / v.ew_rows);
        v.ew_tile_begin = (uint32_t)ew_tiles;
        L.ew_prefix[t] = (uint32_t)ew_tiles;
        ew_tiles += (uint64_t)v.ew_n_rowblocks * (uint64_t)v.n_colblocks;
        if (ew_tiles > 0x7fffffffull) return CF_ERR_SHAPE;
        // the receiver's kernel moves 4 bytes per element, not 10: two rows per workgroup (loaded together, then
        // stored together) keep the workgroup count down; measured 1.43 -> 1.08 ms on 114 x [4096, 3072]
        v.dec_rows = o.encode_rows ? o.encode_rows : 2;
        v.dec_n_rowblocks = (int32_t)((d.n_tokens + v.dec_rows - 1) / v.dec_rows);
        v.dec_tile_begin = (uint32_t)dec_tiles;
        L.dec_prefix[t] = (uint32_t)dec_tiles;
        dec_tiles += (uint64_t)v.dec_n_rowblocks * (uint64_t)v.n_colblocks;
        fins += (uint64_t)((d.n_channels + kFinalizeThreads - 1) / kFinalizeThreads);
        if (tiles > 0x7fffffffull || fins > 0x7fffffffull) return CF_ERR_SHAPE;
        if (d.scale == CF_SCALE_CHANNEL || d.scale == CF_SCALE_RANK1) {
            L.any_channel = true;
            v.partial_off = partial_bytes;   // relative; rebased below
            partial_bytes += align_up((size_t)v.n_rowblocks * (size_t)d.n_channels * sizeof(float));
        }
        if (d.scale == CF_LOWRANK) {
            if (o.ef != CF_EF_RECON) return CF_ERR_UNSUPPORTED;
            L.any_lowrank = true;
            v.lr_p_off = partial_bytes;
            partial_bytes += align_up((size_t)d.n_tokens * kLowRankRank * sizeof(float));
            v.lr_z_off = partial_bytes;
            partial_bytes += align_up((size_t)d.n_channels * kLowRankRank * sizeof(float));
            v.lr_q_off = partial_bytes;
            partial_bytes += align_up((size_t)d.n_channels * kLowRankRank * sizeof(float));
        }
        if (d.scale == CF_SCALE_RANK1) {
            L.any_rank1 = true;
            v.rowpart_off = partial_bytes;
            partial_bytes += align_up((size_t)d.n_tokens * (size_t)v.n_colblocks * sizeof(float));
        }
        L.item_prefix[t] = (uint32_t)items;
        if (d.scale == CF_SCALE_CHANNEL && d.n_tokens < L.min_channel_scale_tokens) L.min_channel_scale_tokens = d.n_tokens;
        if (d.scale == CF_SCALE_CHANNEL && L.single_pass) {
            v.p_rows = narrow_item_rows(d.dtype) / (L.sp_wide ? 2 : 1);
            v.p_n_rb = (int32_t)((d.n_tokens + v.p_rows - 1) / v.p_rows);
            v.p_n_stripes = (int32_t)((d.n_channels + stripe_channels - 1) / stripe_channels);
            v.p_item_begin = (uint32_t)items;
            v.p_partial_off = p_partial_bytes;               // relative; rebased below
            p_partial_bytes += align_up((size_t)v.p_n_rb * (size_t)d.n_channels * sizeof(float));
            items += (uint64_t)v.p_n_rb * (uint64_t)v.p_n_stripes;
            if (v.p_n_rb > L.max_group_items) L.max_group_items = v.p_n_rb;
            if (items > 0x7fffffffull) return CF_ERR_SHAPE;
        }
    }
    L.tile_prefix[n] = (uint32_t)tiles;
    L.ew_prefix[n] = (uint32_t)ew_tiles;
    L.dec_prefix[n] = (uint32_t)dec_tiles;
    L.fin_prefix[n] = (uint32_t)fins;
    L.item_prefix[n] = (uint32_t)items;

    size_t off = 0;
    L.off_descs = off;        off = align_up(off + sizeof(TensorDev) * (size_t)n);
    L.off_ptrs = off;         off = align_up(off + sizeof(TensorPtrs) * (size_t)n);
    L.off_tile_prefix = off;  off = align_up(off + sizeof(uint32_t) * (size_t)(n + 1));
    L.off_fin_prefix = off;   off = align_up(off + sizeof(uint32_t) * (size_t)(n + 1));
    L.off_ew_prefix = off;    off = align_up(off + sizeof(uint32_t) * (size_t)(n + 1));
    L.off_dec_prefix = off;   off = align_up(off + sizeof(uint32_t) * (size_t)(n + 1));
    L.off_partials = off;     off = align_up(off + partial_bytes);
    L.off_item_prefix = off;  off = align_up(off + sizeof(uint32_t) * (size_t)(n + 1));
    L.off_item_tensor = off;  off = align_up(off + sizeof(uint32_t) * (size_t)items);
    L.n_items = (size_t)items;
    L.off_gave_up = off;      off = align_up(off + sizeof(uint32_t) * (size_t)items);
    L.off_error = off;        off = align_up(off + sizeof(uint32_t) * 64);      // error word, and the give-up counter 128 bytes on
    L.off_p_partials = off;   off = align_up(off + p_partial_bytes);
    L.total = off;
    for (int32_t t = 0; t < n; ++t) {
        if (descs[t].scale == CF_SCALE_CHANNEL || descs[t].scale == CF_SCALE_RANK1) {
            L.dev[t].partial_off += L.off_partials;
            L.dev[t].p_partial_off += L.off_p_partials;
        }
        if (descs[t].scale == CF_SCALE_RANK1) L.dev[t].rowpart_off += L.off_partials;
        if (descs[t].scale == CF_LOWRANK) {
            L.dev[t].lr_p_off += L.off_partials;
            L.dev[t].lr_z_off += L.off_partials;
            L.dev[t].lr_q_off += L.off_partials;
        }
    }
    return CF_OK;
}

inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

}  // namespace

struct cf_ctx {
    std::vector<cf_tensor_desc> descs;
    Layout L;
    cf_options opts;
    uint8_t *ws = nullptr;
    size_t ws_bytes = 0;
    std::vector<TensorPtrs> ptrs;      // what the workspace table currently holds (once the uploads on ptrs_stream have run)
    hipStream_t ptrs_stream = nullptr; // stream the pointer uploads were enqueued on
    bool ptrs_synced = false;          // the table matches `ptrs` for work enqueued on ptrs_stream from now on
    std::vector<uint8_t> warm;
    int32_t last_hip = 0;
    int device = 0;
    int persist_grid[2][2] = {{0, 0}, {0, 0}};   // co-resident workgroups of k_single_pass<err dtype, fused>

    // benchmark instrumentation (cf_profile_next_call)
    std::vector<hipEvent_t> prof_events;
    bool prof_armed = false;
    int32_t prof_count = 0;
    const char *prof_names[16] = {};

    BatchView view() const
    {
        BatchView v;
        v.descs = reinterpret_cast<const TensorDev *>(ws + L.off_descs);
        v.ptrs = reinterpret_cast<const TensorPtrs *>(ws + L.off_ptrs);
        v.tile_prefix = reinterpret_cast<const uint32_t *>(ws + L.off_tile_prefix);
        v.fin_prefix = reinterpret_cast<const uint32_t *>(ws + L.off_fin_prefix);
        v.ew_prefix = reinterpret_cast<const uint32_t *>(ws + L.off_ew_prefix);
        v.dec_prefix = reinterpret_cast<const uint32_t *>(ws + L.off_dec_prefix);
        v.item_prefix = reinterpret_cast<const uint32_t *>(ws + L.off_item_prefix);
        v.item_tensor = reinterpret_cast<const uint32_t *>(ws + L.off_item_tensor);
        v.error_flag = reinterpret_cast<uint32_t *>(ws + L.off_error);
        v.gave_up_items = reinterpret_cast<uint32_t *>(ws + L.off_gave_up);
        v.workspace = ws;
        v.n_tensors = (int32_t)descs.size();
        return v;
    }

    LaunchRange range(int32_t first, int32_t count) const
    {
        LaunchRange r;
        r.first = first;
        r.count = count;
        r.tile_lo = L.tile_prefix[first];
        r.tile_hi = L.tile_prefix[first + count];
        r.ew_lo = L.ew_prefix[first];
        r.ew_hi = L.ew_prefix[first + count];
        r.dec_lo = L.dec_prefix[first];
        r.dec_hi = L.dec_prefix[first + count];
        r.fin_lo = L.fin_prefix[first];
        r.fin_hi = L.fin_prefix[first + count];
        r.sp_xcd_major = 0;
        r.sp_wait_polls = kWaitPolls;
        r.sp_redo = 0;
        r.item_lo = L.item_prefix[first];
        r.item_hi = L.item_prefix[first + count];
        r.only_group_scale = 0;
        r.naive = opts.ef == CF_EF_NAIVE;
        r.dts = descs[first].dtype;
        r.lr_max_channels = 0;
        r.lr_max_tokens = 0;
        r.p_partial_lo = ~(uint64_t)0;
        r.p_partial_hi = 0;
        for (int32_t t = first; t < first + count; ++t) {
            const TensorDev &dv = L.dev[t];
            if (dv.p_rows == 0) continue;
            const uint64_t bytes = align_up((size_t)dv.p_n_rb * (size_t)dv.n_channels * sizeof(float));
            if (dv.p_partial_off < r.p_partial_lo) r.p_partial_lo = dv.p_partial_off;
            if (dv.p_partial_off + bytes > r.p_partial_hi) r.p_partial_hi = dv.p_partial_off + bytes;
        }
        if (r.p_partial_hi == 0) r.p_partial_lo = 0;
        for (int32_t t = first; t < first + count; ++t) {
            if (descs[t].dtype != descs[first].dtype) r.dts = 2;
            if (descs[t].scale == CF_LOWRANK) {
                if (descs[t].n_channels > r.lr_max_channels) r.lr_max_channels = (int32_t)descs[t].n_channels;
                if (descs[t].n_tokens > r.lr_max_tokens) r.lr_max_tokens = descs[t].n_tokens;
            }
        }
        return r;
    }

    // anything for k_encode (with_channel: channel-scale tensors too; not when the single-pass kernel took them)
    bool range_has_quantised(int32_t first, int32_t count, bool with_channel) const
    {
        for (int32_t t = first; t < first + count; ++t) {
            const int sc = descs[t].scale;
            if (sc == CF_SCALE_GROUP || sc == CF_SCALE_RANK1 || (with_channel && sc == CF_SCALE_CHANNEL)) return true;
        }
        return false;
    }

    bool range_has_sparse(int32_t first, int32_t count, int block) const   // anything for k_encode_nm of that block length
    {
        for (int32_t t = first; t < first + count; ++t)
            if (descs[t].scale == CF_SPARSE_NM && descs[t].group == block) return true;
        return false;
    }

    bool range_has_channel(int32_t first, int32_t count) const      // anything that needs the reduction kernels
    {
        for (int32_t t = first; t < first + count; ++t)
            if (descs[t].scale == CF_SCALE_CHANNEL || descs[t].scale == CF_SCALE_RANK1) return true;
        return false;
    }

    int range_lowrank_iters(int32_t first, int32_t count) const       // most subspace iterations any tensor asks for; -1 = no such tensor
    {
        int iters = -1;
        for (int32_t t = first; t < first + count; ++t)
            if (descs[t].scale == CF_LOWRANK && descs[t].bits > iters) iters = descs[t].bits;
        return iters;
    }

    bool range_has_elementwise(int32_t first, int32_t count) const    // anything k_encode / k_decode handle
    {
        for (int32_t t = first; t < first + count; ++t)
            if (descs[t].scale != CF_LOWRANK) return true;
        return false;
    }

    bool range_has_rank1(int32_t first, int32_t count) const
    {
        for (int32_t t = first; t < first + count; ++t)
            if (descs[t].scale == CF_SCALE_RANK1) return true;
        return false;
    }
};

namespace {

cf_status check_range(const cf_ctx *ctx, int32_t first, int32_t count)
{
    if (!ctx) return CF_ERR_INVALID_ARG;
    if (first < 0 || count < 0 || (int64_t)first + count > (int64_t)ctx->descs.size()) return CF_ERR_INVALID_ARG;
    return CF_OK;
}

cf_status check_warm(const cf_ctx *ctx, int32_t first, int32_t count)
{
    for (int32_t t = first; t < first + count; ++t)
        if (!ctx->warm[t]) return CF_ERR_STATE;
    return CF_OK;
}

// Validates one pointer array (host array of `count` device pointers).
cf_status check_ptrs(const void *const *arr, int32_t count)
{
    if (!arr) return CF_ERR_INVALID_ARG;
    for (int32_t k = 0; k < count; ++k)
        if (!arr[k] || !aligned16(arr[k])) return CF_ERR_INVALID_ARG;
    return CF_OK;
}

// Scale buffers: the N:M sparsifier has none, its entries are ignored and may be null.
cf_status check_scale_ptrs(const cf_ctx *ctx, int32_t first, int32_t count, const void *const *arr)
{
    if (!arr) return CF_ERR_INVALID_ARG;
    for (int32_t k = 0; k < count; ++k) {
        if (ctx->descs[first + k].scale == CF_SPARSE_NM) {
            if (arr[k] && !aligned16(arr[k])) return CF_ERR_INVALID_ARG;
        } else if (!arr[k] || !aligned16(arr[k])) {
            return CF_ERR_INVALID_ARG;
        }
    }
    return CF_OK;
}

cf_status device_fail(cf_ctx *ctx, hipError_t e)
{
    ctx->last_hip = (int32_t)e;
    return CF_ERR_DEVICE;
}

// Builds a context over `workspace` and brings its tables there.  Everything travels inside kernel arguments
// (no host-to-device copy, no memset), so this works wherever a kernel launch does.
cf_status make_ctx(cf_ctx **out, const cf_tensor_desc *descs, int32_t n_tensors, const cf_options &o, void *workspace,
                   size_t workspace_bytes, hipStream_t s)
{
    cf_ctx *ctx = new (std::nothrow) cf_ctx;
    if (!ctx) return CF_ERR_INVALID_ARG;
    cf_status st = make_layout(descs, n_tensors, o, ctx->L);
    if (st != CF_OK) { delete ctx; return st; }
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) % kAlign) != 0 || workspace_bytes < ctx->L.total) {
        delete ctx;
        return CF_ERR_WORKSPACE;
    }
    ctx->descs.assign(descs, descs + n_tensors);
    ctx->opts = o;
    ctx->ws = static_cast<uint8_t *>(workspace);
    ctx->ws_bytes = workspace_bytes;
    ctx->ptrs.resize(n_tensors);
    std::memset(ctx->ptrs.data(), 0, sizeof(TensorPtrs) * (size_t)n_tensors);
    ctx->warm.assign(n_tensors, 0);

    const Layout &L = ctx->L;
    const size_t prefix_bytes = sizeof(uint32_t) * (size_t)(n_tensors + 1);
    hipError_t e = hipGetDevice(&ctx->device);
    if (e == hipSuccess) e = launch_upload_bytes(L.dev.data(), ctx->ws + L.off_descs, sizeof(TensorDev) * (size_t)n_tensors, s);
    if (e == hipSuccess) e = launch_upload_bytes(L.tile_prefix.data(), ctx->ws + L.off_tile_prefix, prefix_bytes, s);
    if (e == hipSuccess) e = launch_upload_bytes(L.fin_prefix.data(), ctx->ws + L.off_fin_prefix, prefix_bytes, s);
    if (e == hipSuccess) e = launch_upload_bytes(L.ew_prefix.data(), ctx->ws + L.off_ew_prefix, prefix_bytes, s);
    if (e == hipSuccess) e = launch_upload_bytes(L.dec_prefix.data(), ctx->ws + L.off_dec_prefix, prefix_bytes, s);
    if (e == hipSuccess) e = launch_upload_bytes(L.item_prefix.data(), ctx->ws + L.off_item_prefix, prefix_bytes, s);
    if (e == hipSuccess && L.n_items > 0)
        e = launch_fill_item_tensor(reinterpret_cast<const uint32_t *>(ctx->ws + L.off_item_prefix),
                                    reinterpret_cast<uint32_t *>(ctx->ws + L.off_item_tensor), n_tensors, s);
    if (e == hipSuccess) e = launch_fill_words(ctx->ws + L.off_ptrs, 0u, sizeof(TensorPtrs) * (size_t)n_tensors / 4, s);
    if (e == hipSuccess) e = launch_fill_words(ctx->ws + L.off_error, 0u, 64, s);
    if (e == hipSuccess && L.single_pass && L.max_group_items > 0) {
        int n_cu = 0;
        e = hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, ctx->device);
        if (e == hipSuccess)
            for (int et = 0; et < 2; ++et)
                for (int fu = 0; fu < 2; ++fu)
                    ctx->persist_grid[et][fu] = persistent_max_blocks_per_cu(o.ef, et, fu != 0, L.sp_wide) * n_cu;
    }
    if (e != hipSuccess) {
        (void)hipGetLastError();
        delete ctx;
        return CF_ERR_DEVICE;
    }
    *out = ctx;
    return CF_OK;
}

// Runs one launch; when the call is being profiled, brackets it with the caller's events.
template <class F>
hipError_t launch(cf_ctx *ctx, hipStream_t s, const char *name, F &&f)
{
    const int32_t k = ctx->prof_count;
    const bool rec = ctx->prof_armed && (size_t)(2 * k + 1) < ctx->prof_events.size();
    if (ctx->prof_armed && k < 16) ctx->prof_names[k] = name;
    if (ctx->prof_armed) ctx->prof_count = k + 1;
    hipError_t e = hipSuccess;
    if (rec) e = hipEventRecord(ctx->prof_events[2 * k], s);
    if (e == hipSuccess) e = f();
    if (e == hipSuccess && rec) e = hipEventRecord(ctx->prof_events[2 * k + 1], s);
    return e;
}

struct ProfileScope {      // a profiled call is exactly one entry-point call
    cf_ctx *ctx;
    explicit ProfileScope(cf_ctx *c) : ctx(c) { if (ctx->prof_armed) ctx->prof_count = 0; }
    ~ProfileScope() { ctx->prof_armed = false; }
};

// Brings the workspace pointer table up to date for [first, first+count).
// Arrays that an entry point does not take are passed as nullptr and keep
// their last value.  Nothing is launched when no pointer changed.
// The last batch of pointer sets of a call, left for the call's next kernel to write (see sync_ptrs).
struct DeferredPtrs {
    PtrChunk chunk;
    TensorPtrs *dst = nullptr;
    int n = 0;
    DeferredPtrs() { std::memset(&chunk, 0, sizeof chunk); }
};

// defer: the caller's next launch is a kernel that can write one batch of pointer sets itself (k_reset_partials):
// the last batch is handed back instead of launched.
cf_status sync_ptrs(cf_ctx *ctx, int32_t first, int32_t count, const void *const *x, void *const *recon,
                    void *const *err, void *const *codes, void *const *scales, hipStream_t s, DeferredPtrs *defer = nullptr)
{
    bool changed = false;
    for (int32_t k = 0; k < count; ++k) {
        TensorPtrs &p = ctx->ptrs[first + k];
        TensorPtrs q = p;
        if (x) q.x = x[k];
        if (recon) q.recon = recon[k];
        if (err) q.err = err[k];
        if (codes) q.codes = static_cast<uint8_t *>(codes[k]);
        if (scales) q.scales = static_cast<float *>(scales[k]);
        if (std::memcmp(&p, &q, sizeof p) != 0) {
            p = q;
            changed = true;
        }
    }
    // The mirror describes the table as work enqueued on ptrs_stream after the last upload sees it.  On another
    // stream nothing orders that upload before this call, and while a stream is being captured into a graph the
    // upload is recorded, not run (nobody knows whether or when the graph will): in both cases the whole table
    // is uploaded, and after a captured call it counts as unknown again.
    hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(s, &cap) != hipSuccess) {
        (void)hipGetLastError();
        cap = hipStreamCaptureStatusNone;
    }
    const bool capturing = cap != hipStreamCaptureStatusNone;
    const bool whole = capturing || !ctx->ptrs_synced || ctx->ptrs_stream != s;
    if (!changed && !whole) return CF_OK;
    const int32_t lo = whole ? 0 : first, n = whole ? (int32_t)ctx->ptrs.size() : count;
    TensorPtrs *table = reinterpret_cast<TensorPtrs *>(ctx->ws + ctx->L.off_ptrs);
    ctx->ptrs_synced = false;
    for (int32_t k0 = 0; k0 < n; k0 += kMaxUploadTensors) {
        int m = n - k0 < kMaxUploadTensors ? n - k0 : kMaxUploadTensors;
        PtrChunk chunk;
        std::memset(&chunk, 0, sizeof chunk);
        for (int k = 0; k < m; ++k) chunk.p[k] = ctx->ptrs[lo + k0 + k];
        if (defer && k0 + m == n) {     // the caller's next kernel takes this one along
            defer->chunk = chunk;
            defer->dst = table + lo + k0;
            defer->n = m;
            break;
        }
        hipError_t e = launch(ctx, s, "k_upload_ptrs", [&] { return launch_upload_ptrs(chunk, table + lo + k0, m, s); });
        if (e != hipSuccess) return device_fail(ctx, e);       // the table counts as unknown: the next call uploads all of it
    }
    ctx->ptrs_synced = !capturing;
    ctx->ptrs_stream = s;
    return CF_OK;
}

// Alg. 3 on the low-rank tensors of the range: Q <- orth(Q0); T x { P <- A Q; Z <- A^T P; Q <- orth(Z) };
// U <- A Q; then D = U V^T, error and reconstruction.
cf_status run_lowrank_sender(cf_ctx *ctx, int32_t first, int32_t count, const BatchView &v, const LaunchRange &r,
                             bool fused, hipStream_t s)
{
    const int iters = ctx->range_lowrank_iters(first, count);
    if (iters < 0) return CF_OK;
    if (count > 65535) return CF_ERR_SHAPE;     // the low-rank kernels index the tensors of a call with blockIdx.y
    hipError_t e = launch(ctx, s, "k_lr_orth", [&] { return launch_lr_orth(v, r, true, 0, s); });
    if (e != hipSuccess) return device_fail(ctx, e);
    for (int it = 1; it <= iters; ++it) {       // tensors that asked for fewer iterations sit the later ones out
        e = launch(ctx, s, "k_lr_project", [&] { return launch_lr_project(v, r, false, it, s); });
        if (e != hipSuccess) return device_fail(ctx, e);
        e = launch(ctx, s, "k_lr_backproject", [&] { return launch_lr_backproject(v, r, it, s); });
        if (e != hipSuccess) return device_fail(ctx, e);
        e = launch(ctx, s, "k_lr_orth", [&] { return launch_lr_orth(v, r, false, it, s); });
        if (e != hipSuccess) return device_fail(ctx, e);
    }
    e = launch(ctx, s, "k_lr_project", [&] { return launch_lr_project(v, r, true, 0, s); });
    if (e != hipSuccess) return device_fail(ctx, e);
    if (ctx->opts.flags & CF_FLAG_LOWRANK_INT4) {
        e = launch(ctx, s, "k_lr_quant_u", [&] { return launch_lr_quant_u(v, r, s); });
        if (e != hipSuccess) return device_fail(ctx, e);
    }
    e = launch(ctx, s, "k_lr_apply", [&] { return launch_lr_encode(v, r, ctx->opts.err_dtype, fused, s); });
    if (e != hipSuccess) return device_fail(ctx, e);
    return CF_OK;
}

// The row-local encoders over the element-wise tiles of the range: k_encode for the quantisers (channel-scale
// tensors only when with_channel: not when the single-pass kernel already took them, r.only_group_scale),
// k_encode_nm for the sparsifier (once per block length); each only if the range holds such a tensor.
hipError_t run_row_local(cf_ctx *ctx, int32_t first, int32_t count, const BatchView &v, const LaunchRange &r, bool fused,
                         bool with_channel, hipStream_t s)
{
    const int ef = ctx->opts.ef, et = ctx->opts.err_dtype;
    hipError_t e = hipSuccess;
    if (ctx->range_has_quantised(first, count, with_channel)) {
        e = launch(ctx, s, "k_encode", [&] { return launch_encode(v, r, ef, et, fused, s); });
        if (e != hipSuccess) return e;
    }
    for (int pair = 0; pair < 2 && e == hipSuccess; ++pair)
        if (ctx->range_has_sparse(first, count, pair ? 16 : 8))
            e = launch(ctx, s, "k_encode_nm", [&] { return launch_encode_nm(v, r, ef, et, fused, pair != 0, s); });
    return e;
}

cf_status run_sender(cf_ctx *ctx, int32_t first, int32_t count, const void *const *x, void *const *recon,
                     void *const *err, void *const *codes, void *const *scales, void *stream, bool fused)
{
    cf_status st = check_range(ctx, first, count);
    if (st != CF_OK) return st;
    if (count == 0) return CF_OK;
    if ((st = check_ptrs(x, count)) != CF_OK) return st;
    if ((st = check_ptrs(recon, count)) != CF_OK) return st;
    if ((st = check_ptrs(err, count)) != CF_OK) return st;
    if ((st = check_ptrs(codes, count)) != CF_OK) return st;
    if ((st = check_scale_ptrs(ctx, first, count, reinterpret_cast<const void *const *>(scales))) != CF_OK) return st;
    for (int32_t k = 0; k < count; ++k) {       // the buffers of one tensor must not overlap one another
        const BufferBytes b = buffer_bytes(ctx->descs[first + k], ctx->opts);
        const void *px = x[k], *pr = recon[k], *pe = err[k], *pc = codes[k], *ps = scales[k];
        if (overlap(px, b.recon, pr, b.recon) || overlap(px, b.recon, pe, b.err) || overlap(pr, b.recon, pe, b.err)) return CF_ERR_INVALID_ARG;
        if (overlap(pc, b.codes, px, b.recon) || overlap(pc, b.codes, pr, b.recon) || overlap(pc, b.codes, pe, b.err)) return CF_ERR_INVALID_ARG;
        if (overlap(ps, b.scales, px, b.recon) || overlap(ps, b.scales, pr, b.recon) || overlap(ps, b.scales, pe, b.err) ||
            overlap(ps, b.scales, pc, b.codes))
            return CF_ERR_INVALID_ARG;
    }
    if ((st = check_warm(ctx, first, count)) != CF_OK) return st;

    hipStream_t s = static_cast<hipStream_t>(stream);
    ProfileScope prof(ctx);
    BatchView v = ctx->view();
    LaunchRange r = ctx->range(first, count);
    const int ef = ctx->opts.ef, et = ctx->opts.err_dtype;
    hipError_t e;
    const int grid = ctx->persist_grid[et == CF_BF16 ? 1 : 0][fused ? 1 : 0];
    // unless asked for: not for tiny batches (the wait chain costs more than a second read) nor for short tensors
    // (an item is 128 or 256 rows tall: most of its lanes would idle)
    const bool forced = (ctx->opts.flags & CF_FLAG_SINGLE_PASS) != 0;
    // nor for very tall ones (groups of more than 48 items: measured on [N, 3072] bf16 batches of equal size, single pass
    // against two kernels: N = 8192 1.64 / 1.91 ms, 12288 1.80 / 1.88, 16384 2.04 / 1.91, 32768 2.34 / 1.92)
    const bool worth_it = forced || (r.item_hi - r.item_lo >= 64u && ctx->L.min_channel_scale_tokens >= 256 && ctx->L.max_group_items <= 48);
    // (a group larger than what the device holds at once would have its first workgroups wait for ones that cannot
    // start before they leave: correct, they give up and the redo launch does them, but slow: such tensors take two kernels)
    const bool single_pass = ctx->L.single_pass && grid >= ctx->L.max_group_items && grid >= 1 && r.item_hi > r.item_lo && worth_it;
    // the call's pointers go to the table first; the single pass's first kernel takes the last batch of them along
    DeferredPtrs defer;
    if ((st = sync_ptrs(ctx, first, count, x, recon, err, codes, scales, s, single_pass ? &defer : nullptr)) != CF_OK) return st;
    if (single_pass) {
        // channel-scale tensors: one pass, the operands stay in registers across the scale reduction
        e = launch(ctx, s, "k_reset_partials", [&] { return launch_reset_partials(v, r, defer.chunk, defer.dst, defer.n, s); });
        if (e != hipSuccess) {
            ctx->ptrs_synced = false;       // the batch that kernel was to write never reached the table
            return device_fail(ctx, e);
        }
        // measured on [N, 3072] bf16 batches: up to 4 row blocks per tensor a run of consecutive items per XCD is
        // 4-20 % faster (the stripes of a code row meet in one L2), from 6 on dealing them round the XCDs is 8-15 % faster
        r.sp_xcd_major = ctx->L.max_group_items <= 4;
        r.sp_wait_polls = (ctx->opts.flags & CF_FLAG_TEST_NO_WAIT) ? 0u : kWaitPolls;
        const bool one_shot = (ctx->opts.flags & CF_FLAG_FIXED_GRID) == 0;
        e = launch(ctx, s, "k_single_pass", [&] { return launch_single_pass(v, r, ef, et, fused, ctx->L.sp_wide, grid, one_shot, false, s); });
        if (e != hipSuccess) return device_fail(ctx, e);
        // the items whose workgroup gave up waiting (normally none: the launch is empty)
        e = launch(ctx, s, "k_single_pass_redo", [&] { return launch_single_pass(v, r, ef, et, fused, ctx->L.sp_wide, grid, one_shot, true, s); });
        if (e != hipSuccess) return device_fail(ctx, e);
        r.only_group_scale = 1;
        if ((e = run_row_local(ctx, first, count, v, r, fused, false, s)) != hipSuccess) return device_fail(ctx, e);
        return run_lowrank_sender(ctx, first, count, v, r, fused, s);
    }
    if (ctx->range_has_channel(first, count)) {
        e = launch(ctx, s, "k_colreduce", [&] { return launch_colreduce(v, r, ef, et, s); });
        if (e != hipSuccess) return device_fail(ctx, e);
        e = launch(ctx, s, "k_finalize", [&] { return launch_finalize(v, r, s); });
        if (e != hipSuccess) return device_fail(ctx, e);
        if (ctx->range_has_rank1(first, count)) {
            e = launch(ctx, s, "k_finalize_rank1", [&] { return launch_finalize_rank1(v, r, s); });
            if (e != hipSuccess) return device_fail(ctx, e);
        }
    }
    if ((e = run_row_local(ctx, first, count, v, r, fused, true, s)) != hipSuccess) return device_fail(ctx, e);
    return run_lowrank_sender(ctx, first, count, v, r, fused, s);
}

}  // namespace

extern "C" {

const char *cf_status_string(cf_status s)
{
    switch (s) {
    case CF_OK: return "ok";
    case CF_ERR_INVALID_ARG: return "invalid argument";
    case CF_ERR_SHAPE: return "unsupported shape";
    case CF_ERR_UNSUPPORTED: return "unsupported configuration";
    case CF_ERR_STATE: return "tensor not warmed up";
    case CF_ERR_WORKSPACE: return "workspace too small or misaligned";
    case CF_ERR_DEVICE: return "HIP call failed";
    }
    return "unknown status";
}

cf_status cf_sizes(const cf_tensor_desc *desc, const cf_options *opts, size_t *codes_bytes, size_t *scales_bytes,
                   size_t *recon_bytes, size_t *err_bytes)
{
    if (!desc) return CF_ERR_INVALID_ARG;
    cf_options o;
    cf_status st = check_opts(opts, o);
    if (st != CF_OK) return st;
    if ((st = check_desc(*desc)) != CF_OK) return st;
    BufferBytes b = buffer_bytes(*desc, o);
    if (codes_bytes) *codes_bytes = b.codes;
    if (scales_bytes) *scales_bytes = b.scales;
    if (recon_bytes) *recon_bytes = b.recon;
    if (err_bytes) *err_bytes = b.err;
    return CF_OK;
}

size_t cf_workspace_bytes(const cf_tensor_desc *descs, int32_t n_tensors, const cf_options *opts)
{
    cf_options o;
    if (check_opts(opts, o) != CF_OK) return 0;
    Layout L;
    if (make_layout(descs, n_tensors, o, L) != CF_OK) return 0;
    return L.total;
}

cf_status cf_init(cf_ctx **out, const cf_tensor_desc *descs, int32_t n_tensors, const cf_options *opts,
                  void *workspace, size_t workspace_bytes, void *stream)
{
    if (!out) return CF_ERR_INVALID_ARG;
    *out = nullptr;
    cf_options o;
    cf_status st = check_opts(opts, o);
    if (st != CF_OK) return st;
    return make_ctx(out, descs, n_tensors, o, workspace, workspace_bytes, static_cast<hipStream_t>(stream));
}

void cf_destroy(cf_ctx *ctx) { delete ctx; }

int32_t cf_last_hip_error(const cf_ctx *ctx) { return ctx ? ctx->last_hip : 0; }

cf_status cf_profile_next_call(cf_ctx *ctx, void *const *events, int32_t n_pairs)
{
    if (!ctx || n_pairs < 0 || (n_pairs > 0 && !events)) return CF_ERR_INVALID_ARG;
    ctx->prof_events.clear();
    for (int32_t k = 0; k < 2 * n_pairs; ++k) {
        if (!events[k]) { ctx->prof_events.clear(); return CF_ERR_INVALID_ARG; }
        ctx->prof_events.push_back(static_cast<hipEvent_t>(events[k]));
    }
    ctx->prof_armed = n_pairs > 0;
    ctx->prof_count = 0;
    return CF_OK;
}

cf_status cf_check_device(cf_ctx *ctx, void *stream)
{
    if (!ctx) return CF_ERR_INVALID_ARG;
    hipError_t e = hipStreamSynchronize(static_cast<hipStream_t>(stream));
    uint32_t flag = 0;
    if (e == hipSuccess) e = hipMemcpy(&flag, ctx->ws + ctx->L.off_error, sizeof flag, hipMemcpyDeviceToHost);
    if (e != hipSuccess) return device_fail(ctx, e);
    if (flag) {
        ctx->last_hip = 0;
        return CF_ERR_DEVICE;
    }
    return CF_OK;
}

cf_status cf_given_up_items(cf_ctx *ctx, void *stream, uint32_t *count)
{
    if (!ctx || !count) return CF_ERR_INVALID_ARG;
    hipError_t e = hipStreamSynchronize(static_cast<hipStream_t>(stream));
    uint32_t n = 0;
    if (e == hipSuccess)
        e = hipMemcpy(&n, ctx->ws + ctx->L.off_error + sizeof(uint32_t) * kGaveUpWord, sizeof n, hipMemcpyDeviceToHost);
    if (e != hipSuccess) return device_fail(ctx, e);
    *count = n;
    return CF_OK;
}

int32_t cf_profile_launch_count(const cf_ctx *ctx) { return ctx ? ctx->prof_count : 0; }

const char *cf_profile_kernel_name(const cf_ctx *ctx, int32_t k)
{
    if (!ctx || k < 0 || k >= ctx->prof_count || k >= 16) return nullptr;
    return ctx->prof_names[k];
}

cf_status cf_set_warm(cf_ctx *ctx, int32_t first, int32_t count, int32_t warm)
{
    cf_status st = check_range(ctx, first, count);
    if (st != CF_OK) return st;
    for (int32_t t = first; t < first + count; ++t) ctx->warm[t] = warm ? 1 : 0;
    return CF_OK;
}

cf_status cf_warmup(cf_ctx *ctx, int32_t first, int32_t count, const void *const *x0, void *const *recon,
                    void *const *err, void *stream)
{
    cf_status st = check_range(ctx, first, count);
    if (st != CF_OK) return st;
    if (count == 0) return CF_OK;
    if ((st = check_ptrs(x0, count)) != CF_OK) return st;
    if ((st = check_ptrs(recon, count)) != CF_OK) return st;
    if ((st = check_ptrs(err, count)) != CF_OK) return st;
    for (int32_t k = 0; k < count; ++k) {
        const BufferBytes b = buffer_bytes(ctx->descs[first + k], ctx->opts);
        if (overlap(x0[k], b.recon, recon[k], b.recon) || overlap(x0[k], b.recon, err[k], b.err) || overlap(recon[k], b.recon, err[k], b.err))
            return CF_ERR_INVALID_ARG;
    }
    hipStream_t s = static_cast<hipStream_t>(stream);
    if ((st = sync_ptrs(ctx, first, count, x0, recon, err, nullptr, nullptr, s)) != CF_OK) return st;
    hipError_t e = launch_warmup(ctx->view(), ctx->range(first, count), ctx->opts.err_dtype, s);
    if (e != hipSuccess) return device_fail(ctx, e);
    for (int32_t t = first; t < first + count; ++t) ctx->warm[t] = 1;
    return CF_OK;
}

cf_status cf_compress(cf_ctx *ctx, int32_t first, int32_t count, const void *const *x, const void *const *recon,
                      void *const *err, void *const *codes, void *const *scales, void *stream)
{
    return run_sender(ctx, first, count, x, const_cast<void *const *>(reinterpret_cast<const void *const *>(recon)), err,
                      codes, scales, stream, false);
}

cf_status cf_step_fused(cf_ctx *ctx, int32_t first, int32_t count, const void *const *x, void *const *recon,
                        void *const *err, void *const *codes, void *const *scales, void *stream)
{
    return run_sender(ctx, first, count, x, recon, err, codes, scales, stream, true);
}

cf_status cf_decompress(cf_ctx *ctx, int32_t first, int32_t count, const void *const *codes,
                        const void *const *scales, void *const *recon, void *stream)
{
    cf_status st = check_range(ctx, first, count);
    if (st != CF_OK) return st;
    if (count == 0) return CF_OK;
    if ((st = check_ptrs(codes, count)) != CF_OK) return st;
    if ((st = check_scale_ptrs(ctx, first, count, scales)) != CF_OK) return st;
    if ((st = check_ptrs(recon, count)) != CF_OK) return st;
    for (int32_t k = 0; k < count; ++k) {
        const BufferBytes b = buffer_bytes(ctx->descs[first + k], ctx->opts);
        if (overlap(codes[k], b.codes, recon[k], b.recon)) return CF_ERR_INVALID_ARG;
        if (overlap(scales[k], b.scales, codes[k], b.codes) || overlap(scales[k], b.scales, recon[k], b.recon)) return CF_ERR_INVALID_ARG;
    }
    if ((st = check_warm(ctx, first, count)) != CF_OK) return st;
    hipStream_t s = static_cast<hipStream_t>(stream);
    ProfileScope prof(ctx);
    st = sync_ptrs(ctx, first, count, nullptr, recon, nullptr, const_cast<void *const *>(codes),
                   const_cast<void *const *>(scales), s);
    if (st != CF_OK) return st;
    hipError_t e = hipSuccess;
    if (ctx->range_has_elementwise(first, count)) {
        e = launch(ctx, s, "k_decode", [&] { return launch_decode(ctx->view(), ctx->range(first, count), s); });
        if (e != hipSuccess) return device_fail(ctx, e);
    }
    if (ctx->range_lowrank_iters(first, count) >= 0) {
        e = launch(ctx, s, "k_lr_apply", [&] { return launch_lr_decode(ctx->view(), ctx->range(first, count), s); });
        if (e != hipSuccess) return device_fail(ctx, e);
    }
    return CF_OK;
}

namespace {
constexpr int kMaxStaticDevices = 64;
cf_ctx *g_static_ctx[kMaxStaticDevices];       // the context over each device's static scratch, kept while the tensors stay the same
}  // namespace

cf_status cf_step_fused_static(const cf_tensor_desc *descs, int32_t n_tensors, const cf_options *opts, const void *const *x,
                               void *const *recon, void *const *err, void *const *codes, void *const *scales, void *stream)
{
    cf_options o;
    cf_status st = check_opts(opts, o);
    if (st != CF_OK) return st;
    if (!descs || n_tensors < 1) return CF_ERR_INVALID_ARG;
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxStaticDevices) {
        (void)hipGetLastError();
        return CF_ERR_DEVICE;
    }
    hipStream_t s = static_cast<hipStream_t>(stream);
    cf_ctx *&ctx = g_static_ctx[dev];
    const bool same = ctx && ctx->descs.size() == (size_t)n_tensors &&
                      std::memcmp(ctx->descs.data(), descs, sizeof(cf_tensor_desc) * (size_t)n_tensors) == 0 &&
                      std::memcmp(&ctx->opts, &o, sizeof o) == 0;
    if (!same) {
        delete ctx;
        ctx = nullptr;
        void *ws = nullptr;
        if (static_scratch(&ws) != hipSuccess) {
            (void)hipGetLastError();
            return CF_ERR_DEVICE;
        }
        // lays the tables out in the scratch array afresh (CF_ERR_WORKSPACE if these tensors need more than it holds)
        st = make_ctx(&ctx, descs, n_tensors, o, ws, kStaticScratchBytes, s);
        if (st != CF_OK) return st;
        for (auto &w : ctx->warm) w = 1;        // the caller vouches for recon and err
    }
    return run_sender(ctx, 0, n_tensors, x, recon, err, codes, scales, stream, true);
}

}  // extern "C"
