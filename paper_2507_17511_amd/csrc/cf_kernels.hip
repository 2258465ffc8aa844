// gfx950 kernels of the residual codec (arxiv 2507.17511: Sec. 3.1, Sec. 3.2,
// App. D "Quantization", App. H).  Everything here is bandwidth-bound
// element-wise or reduction work: 128-bit loads, fp32 arithmetic in registers
// with one rounding per operation (the file is compiled with
// -ffp-contract=off), integer code packing, in-place state updates.  No MFMA:
// nothing is a dense contraction.
//
// Tiled kernels: one workgroup of 128 lanes per tile of rb_rows x 1024
// channels; lane l owns channels [8l, 8l+8) of the tile (one 128-bit bf16
// load per row), so a wave reads 1 KiB of contiguous row per instruction.
// A batched grid covers the tiles of many tensors; a workgroup finds its
// tensor by binary search in a prefix array of tile counts.  Each workgroup
// copies its tensor's descriptor and pointers into registers once: nothing is
// re-read from the tables after a store.
#include "cf_device.h"
#include "cf_internal.h"

namespace cf {
namespace {

using namespace dev;

// ---------------------------------------------------------------- tile lookup

struct TileCtx {
    TensorDev d;        // by value: lives in scalar registers
    TensorPtrs p;
    int rowblock, colblock;
    int rows;           // rows per tile of the kernel at hand
};

// DTS: the storage dtype of every tensor in the launch when it is uniform (F32 or BF16: the other
// dtype's code is then not even compiled in, which keeps the register count down), 2 when mixed.
template <int DTS> __device__ __forceinline__ bool is_bf16(const TensorDev &d) { return DTS == 2 ? d.dtype == BF16 : DTS == BF16; }

// Which tiling of a tensor a kernel walks: the reduction's, the element-wise one (short tiles) or the receiver's.
constexpr int TILES_REDUCE = 0, TILES_EW = 1, TILES_DECODE = 2;

template <int KIND>
__device__ __forceinline__ TileCtx locate_tile_of(const BatchView &v, const LaunchRange &r)
{
    const uint32_t lo = KIND == TILES_EW ? r.ew_lo : KIND == TILES_DECODE ? r.dec_lo : r.tile_lo;
    const uint32_t *prefix = KIND == TILES_EW ? v.ew_prefix : KIND == TILES_DECODE ? v.dec_prefix : v.tile_prefix;
    uint32_t tile = lo + blockIdx.x;
    int t = find_slot(prefix, r.first, r.first + r.count, tile);
    TileCtx c;
    c.d = v.descs[t];
    c.p = v.ptrs[t];
    uint32_t local = tile - (KIND == TILES_EW ? c.d.ew_tile_begin : KIND == TILES_DECODE ? c.d.dec_tile_begin : c.d.tile_begin);
    c.colblock = (int)(local % (uint32_t)c.d.n_colblocks);
    c.rowblock = (int)(local / (uint32_t)c.d.n_colblocks);
    c.rows = KIND == TILES_EW ? c.d.ew_rows : KIND == TILES_DECODE ? c.d.dec_rows : c.d.rb_rows;
    return c;
}

template <bool EW>
__device__ __forceinline__ TileCtx locate_tile(const BatchView &v, const LaunchRange &r)
{
    return locate_tile_of<EW ? TILES_EW : TILES_REDUCE>(v, r);
}

// ---------------------------------------------------------------- a0 warm-up

template <int DT, int ET>
__device__ __forceinline__ void warmup_tile(const TileCtx &c)
{
    const TensorDev &d = c.d;
    int chunk = c.colblock * kTileThreads + (int)threadIdx.x;
    const bool cvalid = chunk < d.n_chunks;
    const int lane = (int)threadIdx.x & 63;
    const int run_chunk0 = chunk - lane, run_valid = d.n_chunks - run_chunk0;    // the wave's 64 chunks: first, and how many exist
    const int64_t i = c.rowblock;                   // element-wise tiles are one row tall
    const int64_t e = i * d.n_channels + (int64_t)chunk * kChunk;
    if (cvalid) {
        Raw8<DT> x;
        x.load_stream(c.p.x, e);
        if (DT == BF16) x.store_stream(c.p.recon, e); else x.store(c.p.recon, e);
    }
    if (ET == F32) {        // zeros need no exchange: every lane fills the pieces a whole-line store gives it
        const f32x4 zero[2] = {(f32x4)(0.0f), (f32x4)(0.0f)};
        lines_store_stream<64>(static_cast<float *>(c.p.err) + i * d.n_channels + (int64_t)run_chunk0 * kChunk, lane, run_valid, zero);
    } else if (cvalid) {
        Raw8<ET> zero;
        zero.zero();
        zero.store_stream(c.p.err, e);
    }
}

template <int ET, int DTS>
__global__ __launch_bounds__(kTileThreads) void k_warmup(BatchView v, LaunchRange r)
{
    TileCtx c = locate_tile<true>(v, r);
    if (is_bf16<DTS>(c.d)) warmup_tile<BF16, ET>(c); else warmup_tile<F32, ET>(c);
}

// ---------------------------------------------------------------- a3, first level: per-tile column partials

// |z| of 8 consecutive rows, combined as a balanced tree:
// ((r0+r1)+(r2+r3)) + ((r4+r5)+(r6+r7)).  Rows past the end count as +0, which
// is exactly the zero padding of the tree.
// R1 (rank-1 scales): also the sum of |z| over the wave's 512 channels of each of the 8 rows, as
// a balanced tree over the channels (8 in the lane, then lane pairs upwards); every lane takes
// part, lanes past the last chunk contribute zeros.
template <int DT, int EF, int ET, bool IS_MAX, bool R1>
__device__ __forceinline__ F8 rows8(const TensorDev &d, const TensorPtrs &p, int chunk, int64_t row, float (&wave_rowsum)[8])
{
    Raw8<DT> xr[8], br[8];
    Raw8<ET> er[8];
#pragma unroll
    for (int r = 0; r < 8; ++r) {
        int64_t i = row + r;
        if (i < d.n_tokens && (!R1 || chunk < d.n_chunks)) {
            int64_t e = i * d.n_channels + (int64_t)chunk * kChunk;
            xr[r].load_stream(p.x, e);       // streaming: the batch is far larger than any cache
            if (EF != EF_NAIVE) br[r].load_stream(p.recon, e); else br[r].zero();
            if (EF == EF_LITERAL || EF == EF_OFF) er[r].load(p.err, e); else er[r].zero();
        } else {
            xr[r].zero();
            br[r].zero();
            er[r].zero();
        }
    }
    F8 a[8];
#pragma unroll
    for (int r = 0; r < 8; ++r) {
        F8 z = residual8<EF>(xr[r].widen(), br[r].widen(), er[r].widen());
#pragma unroll
        for (int k = 0; k < 8; ++k) a[r].v[k] = fabsf(z.v[k]);
        if (R1) {
            const float lane = ((a[r].v[0] + a[r].v[1]) + (a[r].v[2] + a[r].v[3])) + ((a[r].v[4] + a[r].v[5]) + (a[r].v[6] + a[r].v[7]));
            wave_rowsum[r] = wave_tree_sum(lane);
        }
    }
    F8 t;
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        float s01 = comb<IS_MAX>(a[0].v[k], a[1].v[k]), s23 = comb<IS_MAX>(a[2].v[k], a[3].v[k]);
        float s45 = comb<IS_MAX>(a[4].v[k], a[5].v[k]), s67 = comb<IS_MAX>(a[6].v[k], a[7].v[k]);
        float s03 = comb<IS_MAX>(s01, s23), s47 = comb<IS_MAX>(s45, s67);
        t.v[k] = comb<IS_MAX>(s03, s47);
    }
    return t;
}

template <int DT, int EF, int ET, bool IS_MAX, bool R1>
__device__ __forceinline__ void colreduce_tile(const TileCtx &c, uint8_t *ws)
{
    const TensorDev &d = c.d;
    int chunk = c.colblock * kTileThreads + (int)threadIdx.x;
    if (!R1 && chunk >= d.n_chunks) return;
    __shared__ float tile_rowsum[kTileThreads / 64][64];      // [wave][row of the tile]
    const int64_t tile_row0 = (int64_t)c.rowblock * d.rb_rows;
    int64_t row = tile_row0;
    // Balanced tree over the tile's rb_rows = 8 * nb rows (nb in {1,2,4,8}) as three
    // nested two-way loops: level k combines two results of level k-1.  The loops
    // stay rolled so that only one batch of 16 row loads is in flight per lane.
    const int nb = d.rb_rows >> 3;
    const int n0 = nb >= 2 ? 2 : 1, n1 = nb >= 4 ? 2 : 1, n2 = nb >= 8 ? 2 : 1;
    F8 s0, s1, s2;
#pragma unroll 1
    for (int h2 = 0; h2 < n2; ++h2) {
#pragma unroll 1
        for (int h1 = 0; h1 < n1; ++h1) {
#pragma unroll 1
            for (int h0 = 0; h0 < n0; ++h0) {
                float wave_rowsum[8];
                F8 t = rows8<DT, EF, ET, IS_MAX, R1>(d, c.p, chunk, row, wave_rowsum);
                if (R1 && (threadIdx.x & 63) == 0) {
#pragma unroll
                    for (int q = 0; q < 8; ++q) tile_rowsum[threadIdx.x >> 6][(int)(row - tile_row0) + q] = wave_rowsum[q];
                }
                row += 8;
#pragma unroll
                for (int k = 0; k < 8; ++k) s0.v[k] = (h0 == 0) ? t.v[k] : comb<IS_MAX>(s0.v[k], t.v[k]);
            }
#pragma unroll
            for (int k = 0; k < 8; ++k) s1.v[k] = (h1 == 0) ? s0.v[k] : comb<IS_MAX>(s1.v[k], s0.v[k]);
        }
#pragma unroll
        for (int k = 0; k < 8; ++k) s2.v[k] = (h2 == 0) ? s1.v[k] : comb<IS_MAX>(s2.v[k], s1.v[k]);
    }
    if (chunk < d.n_chunks) {
        float *partial = reinterpret_cast<float *>(ws + d.partial_off) + (int64_t)c.rowblock * d.n_channels + (int64_t)chunk * kChunk;
        Raw8<F32> out;
        out.narrow(s2);
        out.store(partial, 0);
    }
    if (R1) {       // the tile's two waves cover channels [0,512) and [512,1024) of the tile: lower + upper
        __syncthreads();
        const int q = (int)threadIdx.x;
        if (q < d.rb_rows && tile_row0 + q < d.n_tokens) {
            float *rowpart = reinterpret_cast<float *>(ws + d.rowpart_off);
            rowpart[(tile_row0 + q) * d.n_colblocks + c.colblock] = tile_rowsum[0][q] + tile_rowsum[1][q];
        }
    }
}

template <int EF, int ET, int DTS>
__global__ __launch_bounds__(kTileThreads) void k_colreduce(BatchView v, LaunchRange r)
{
    TileCtx c = locate_tile<false>(v, r);
    const TensorDev &d = c.d;
    if (d.scale != SCALE_CHANNEL && d.scale != SCALE_RANK1) return;  // row-local codecs: nothing to reduce
    if (is_bf16<DTS>(d)) {
        if (d.scale == SCALE_RANK1) colreduce_tile<BF16, EF, ET, false, true>(c, v.workspace);
        else if (d.bits == 4) colreduce_tile<BF16, EF, ET, true, false>(c, v.workspace);
        else colreduce_tile<BF16, EF, ET, false, false>(c, v.workspace);
    } else {
        if (d.scale == SCALE_RANK1) colreduce_tile<F32, EF, ET, false, true>(c, v.workspace);
        else if (d.bits == 4) colreduce_tile<F32, EF, ET, true, false>(c, v.workspace);
        else colreduce_tile<F32, EF, ET, false, false>(c, v.workspace);
    }
}

// ---------------------------------------------------------------- a3, second level: tree over tile partials

// One lane per column: continues the same binary tree over the n_rowblocks
// partials (zero padded to a power of two), then s = sum / N or max / 7.
__global__ __launch_bounds__(kFinalizeThreads) void k_finalize(BatchView v, LaunchRange r)
{
    uint32_t blk = r.fin_lo + blockIdx.x;
    int t = find_slot(v.fin_prefix, r.first, r.first + r.count, blk);
    const TensorDev d = v.descs[t];
    if (d.scale != SCALE_CHANNEL && d.scale != SCALE_RANK1) return;
    int col = (int)(blk - d.fin_begin) * kFinalizeThreads + (int)threadIdx.x;
    if (col >= d.n_channels) return;
    const CF_GLOBAL float *partial = gconst<float>(v.workspace + d.partial_off) + col;
    const int64_t C = d.n_channels;
    float res, s;
    if (d.bits == 4) {
        res = tree_over<true, 18>(d.n_rowblocks, [&](int i) { return partial[(int64_t)i * C]; });
        s = res / 7.0f;
    } else {
        res = tree_over<false, 18>(d.n_rowblocks, [&](int i) { return partial[(int64_t)i * C]; });
        s = res / (float)d.n_tokens;
    }
    gmut<float>(v.ptrs[t].scales)[col] = s;
}

// Rank-1 scales (App. D "Quantization"): u_i = (rowsum_i / C) / (sum_i rowsum_i / (N C)), written
// behind v in the scales buffer.  One block per tensor: lane t owns an aligned block of B rows
// (B a power of two); a row's sum is the tree over its 1024-channel tile sums, the total is the
// tree over the rows (in the lane, then across lanes in LDS).
__global__ __launch_bounds__(kRank1Threads) void k_finalize_rank1(BatchView v, LaunchRange r)
{
    const int t = r.first + (int)blockIdx.x;
    const TensorDev d = v.descs[t];
    if (d.scale != SCALE_RANK1) return;
    __shared__ float lane_total[kRank1Threads];
    const CF_GLOBAL float *rowpart = gconst<float>(v.workspace + d.rowpart_off);
    CF_GLOBAL float *u = gmut<float>(v.ptrs[t].scales) + d.n_channels;
    const int64_t N = d.n_tokens;
    const int ncb = d.n_colblocks;
    int64_t B = 1;
    while (B * kRank1Threads < N) B <<= 1;
    const int64_t first = (int64_t)threadIdx.x * B;
    auto rowsum = [&](int64_t i) { return tree_over<false, 4>(ncb, [&](int cb) { return rowpart[i * ncb + cb]; }); };
    // pass 1: row sums (kept in u for pass 2) and this lane's block total
    const int nmine = first >= N ? 0 : (int)(N - first < B ? N - first : B);
    lane_total[threadIdx.x] = tree_over<false, 12>(nmine, [&](int q) {
        const float rs = rowsum(first + q);
        u[first + q] = rs;
        return rs;
    });
    __syncthreads();
    for (int w = 1; w < kRank1Threads; w <<= 1) {
        if ((threadIdx.x & (2 * w - 1)) == 0) lane_total[threadIdx.x] = lane_total[threadIdx.x] + lane_total[threadIdx.x + w];
        __syncthreads();
    }
    const float total = lane_total[0];
    const float gmean = total / (float)(N * (int64_t)d.n_channels);
    for (int q = 0; q < nmine; ++q) {
        const float rmean = u[first + q] / (float)d.n_channels;
        u[first + q] = gmean == 0.0f ? 0.0f : rmean / gmean;
    }
}

// ---------------------------------------------------------------- a4-a8: encode (+ fused state update)

// MODE: 0 = channel scales read from memory, 1 = group scales computed in the wave,
// 2 = rank-1 scales u_i * v_j (v read once per lane, u once per row).
// Every lane stays alive (lanes past the last chunk of the row are masked): the group maximum and the
// whole-line store of an fp32 error row are wave-wide exchanges.  `patch`: the wave's 2 KB of LDS.
template <int DT, int BITS, int MODE, int EF, int ET, bool FUSED>
__device__ __forceinline__ void encode_tile(const TileCtx &c, float *patch)
{
    const TensorDev &d = c.d;
    const TensorPtrs &p = c.p;
    int chunk = c.colblock * kTileThreads + (int)threadIdx.x;
    const bool cvalid = chunk < d.n_chunks;
    const int lane = (int)threadIdx.x & 63;
    const int run_chunk0 = chunk - lane;                                // first chunk of the wave's 64
    const int run_valid = d.n_chunks - run_chunk0;                      // chunks of the wave that exist (may exceed 64 or be <= 0)
    const int64_t row0 = c.rowblock;            // element-wise tiles are one row tall
    const int64_t C = d.n_channels;
    const int64_t row_bytes = C * BITS / 8;
    const int n_groups = d.n_channels >> 7;
    const bool wide = (d.n_channels & 31) == 0;

    F8 s = {}, vj = {};
    if (MODE == 0 && cvalid) s = load_scales8(p.scales, (int64_t)chunk * kChunk);
    if (MODE == 2 && cvalid) vj = load_scales8(p.scales, (int64_t)chunk * kChunk);

    // One row per workgroup (the element-wise tiling): a lane never has to wait for its own stores
    // before it can use its next loads, and the register file holds one row's worth, not four.
    const int64_t i = row0;
    const int64_t e = i * C + (int64_t)chunk * kChunk;
    Raw8<DT> xr, br;
    Raw8<ET> er;
    if (cvalid) {
        xr.load(p.x, e);
        // fused: the line is written back by this workgroup, and the streaming hint on its load pays (cfg4 4.09 -> 3.98 ms)
        if (EF == EF_NAIVE) br.zero();
        else if (FUSED) br.load_stream(p.recon, e);
        else br.load(p.recon, e);
        if (EF == EF_LITERAL || EF == EF_OFF) er.load(p.err, e); else er.zero();
    } else {
        xr.zero();
        br.zero();
        er.zero();
    }
    F8 b = br.widen();
    F8 eold = er.widen();
    F8 z = residual8<EF>(xr.widen(), b, eold);
    if (MODE == 1) {
        float m = 0.0f;
#pragma unroll
        for (int k = 0; k < 8; ++k) m = fmaxf(m, fabsf(z.v[k]));
        m = row16_max(m);
        float sg = m / 7.0f;
#pragma unroll
        for (int k = 0; k < 8; ++k) s.v[k] = sg;
        if (cvalid && (threadIdx.x & 15) == 0) gmut<float>(p.scales)[i * n_groups + (chunk >> 4)] = sg;
    }
    if (MODE == 2) {
        const float ui = gconst<float>(p.scales)[C + i];
#pragma unroll
        for (int k = 0; k < 8; ++k) s.v[k] = ui * vj.v[k];
    }
    F8 dq;
    uint32_t packed = quant8<BITS>(z, s, dq);
    if (cvalid) store_codes_wide<BITS>(p.codes + i * row_bytes, chunk, packed, wide);
    F8 enew;
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        float lost = z.v[k] - dq.v[k];
        if (EF == EF_OFF) lost = eold.v[k] + lost;
        enew.v[k] = lost;
    }
    if (ET == F32) {                    // whole 128-byte lines per store, streaming
        f32x4 pieces[2];
        lines_exchange<64>(patch, lane, enew, pieces);
        lines_store_stream<64>(static_cast<float *>(p.err) + i * C + (int64_t)run_chunk0 * kChunk, lane, run_valid, pieces);
    } else if (cvalid) {
        Raw8<ET> eo;
        eo.narrow(enew);
        eo.store_stream(p.err, e);
    }
    if (FUSED && cvalid) {
        F8 nb;
#pragma unroll
        for (int k = 0; k < 8; ++k) nb.v[k] = (EF == EF_NAIVE) ? dq.v[k] : b.v[k] + dq.v[k];
        Raw8<DT> out;
        out.narrow(nb);
        if (DT == BF16) out.store_stream(p.recon, e); else out.store(p.recon, e);
    }
}

// N:M block sparsifier (Sec. 3.4), blocks of 8 channels: one lane selects, packs and decodes its own
// block; the row's mask bytes go where 1-bit codes would, the kept values behind all masks.
template <int DT, int KEEP, bool PAIR, int EF, int ET, bool FUSED>
__device__ __forceinline__ void nm_encode_tile(const TileCtx &c, float *patch)
{
    const TensorDev &d = c.d;
    const TensorPtrs &p = c.p;
    const int chunk = c.colblock * kTileThreads + (int)threadIdx.x;
    const bool cvalid = chunk < d.n_chunks;         // every lane stays alive for the whole-line store of the error row
    const int lane = (int)threadIdx.x & 63;
    const int run_chunk0 = chunk - lane, run_valid = d.n_chunks - run_chunk0;
    const int64_t i = c.rowblock;                   // element-wise tiles are one row tall
    const int64_t C = d.n_channels;
    const bool wide = (d.n_channels & 31) == 0;
    constexpr int kValueBytes = KEEP * (DT == BF16 ? 2 : 4);
    uint8_t *values = p.codes + ((d.n_tokens * d.n_chunks + 15) / 16) * 16;
    const int64_t e = i * C + (int64_t)chunk * kChunk;
    Raw8<DT> xr, br;
    Raw8<ET> er;
    if (cvalid) {
        xr.load(p.x, e);
        // fused: the line is written back by this workgroup, and the streaming hint on its load pays
        if (EF == EF_NAIVE) br.zero();
        else if (FUSED) br.load_stream(p.recon, e);
        else br.load(p.recon, e);
        if (EF == EF_LITERAL || EF == EF_OFF) er.load(p.err, e); else er.zero();
    } else {
        xr.zero();
        br.zero();
        er.zero();
    }
    const F8 b = br.widen();
    const F8 eold = er.widen();
    const F8 z = residual8<EF>(xr.widen(), b, eold);
    const uint32_t mask = nm_select8<KEEP, PAIR>(z);
    uint32_t vals[KEEP];
    F8 dq;
    nm_values8<DT, KEEP>(z, mask, vals, dq);
    if (cvalid) store_codes_wide<1>(p.codes + i * d.n_chunks, chunk, mask, wide);
    if (PAIR) {
        // the even lane writes the block: its own kept values, then the odd lane's
        const int mine = __builtin_popcount(mask);
        uint32_t theirs[KEEP], block[KEEP];
#pragma unroll
        for (int q = 0; q < KEEP; ++q) theirs[q] = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)vals[q], 0xB1, 0xF, 0xF, false);
#pragma unroll
        for (int q = 0; q < KEEP; ++q) {
            uint32_t from_theirs = 0u;
#pragma unroll
            for (int t = 0; t < KEEP; ++t) from_theirs = (q - mine == t) ? theirs[t] : from_theirs;
            block[q] = q < mine ? vals[q] : from_theirs;
        }
        uint8_t *dst = values + (i * (d.n_chunks >> 1) + (chunk >> 1)) * kValueBytes;
        if (DT == BF16 && KEEP == 1 && wide) {
            // two blocks of a lane quad share one dword (whole quads are active: 32 | C)
            const uint32_t next = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)block[0], 0xAA, 0xF, 0xF, false);   // quad_perm [2,2,2,2]
            if (cvalid && (chunk & 3) == 0) *gmut<uint32_t>(dst) = (block[0] & 0xFFFFu) | (next << 16);
        } else if (cvalid && (chunk & 1) == 0) {
            nm_store_values<DT, KEEP>(dst, chunk >> 1, block, false);
        }
    } else if (cvalid) {
        nm_store_values<DT, KEEP>(values + (i * d.n_chunks + chunk) * kValueBytes, chunk, vals, wide);
    }
    F8 enew;
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        float lost = z.v[k] - dq.v[k];
        if (EF == EF_OFF) lost = eold.v[k] + lost;
        enew.v[k] = lost;
    }
    if (ET == F32) {                    // whole 128-byte lines per store, streaming
        f32x4 pieces[2];
        lines_exchange<64>(patch, lane, enew, pieces);
        lines_store_stream<64>(static_cast<float *>(p.err) + i * C + (int64_t)run_chunk0 * kChunk, lane, run_valid, pieces);
    } else if (cvalid) {
        Raw8<ET> eo;
        eo.narrow(enew);
        eo.store_stream(p.err, e);
    }
    if (FUSED && cvalid) {
        F8 nb;
#pragma unroll
        for (int k = 0; k < 8; ++k) nb.v[k] = (EF == EF_NAIVE) ? dq.v[k] : b.v[k] + dq.v[k];
        Raw8<DT> out;
        out.narrow(nb);
        if (DT == BF16) out.store_stream(p.recon, e); else out.store(p.recon, e);
    }
}

template <int DT, bool PAIR, int EF, int ET, bool FUSED>
__device__ __forceinline__ void nm_encode_dispatch(const TileCtx &c, float *patch)
{
    const TensorDev &d = c.d;
    if (d.bits == 1) nm_encode_tile<DT, 1, PAIR, EF, ET, FUSED>(c, patch);
    else if (d.bits == 2) nm_encode_tile<DT, 2, PAIR, EF, ET, FUSED>(c, patch);
    else nm_encode_tile<DT, 4, PAIR, EF, ET, FUSED>(c, patch);
}

template <int DT, int EF, int ET, bool FUSED>
__device__ __forceinline__ void encode_dispatch(const TileCtx &c, float *patch)
{
    const TensorDev &d = c.d;
    if (d.scale == SCALE_GROUP) { encode_tile<DT, 4, 1, EF, ET, FUSED>(c, patch); return; }
    if (d.scale == SCALE_RANK1) {
        if (d.bits == 1) encode_tile<DT, 1, 2, EF, ET, FUSED>(c, patch);
        else encode_tile<DT, 2, 2, EF, ET, FUSED>(c, patch);
        return;
    }
    if (d.bits == 1) encode_tile<DT, 1, 0, EF, ET, FUSED>(c, patch);
    else if (d.bits == 2) encode_tile<DT, 2, 0, EF, ET, FUSED>(c, patch);
    else encode_tile<DT, 4, 0, EF, ET, FUSED>(c, patch);
}

template <int EF, int ET, bool FUSED, int DTS>
__global__ __launch_bounds__(kTileThreads) void k_encode(BatchView v, LaunchRange r)
{
    __shared__ __attribute__((aligned(16))) float patches[kTileThreads / 64][512];      // 2 KB per wave: an fp32 error row's way to whole lines
    TileCtx c = locate_tile<true>(v, r);
    if (r.only_group_scale && c.d.scale == SCALE_CHANNEL) return;   // covered by the single-pass kernel
    if (c.d.scale == LOWRANK || c.d.scale == SPARSE_NM) return;     // have kernels of their own
    float *patch = patches[(int)threadIdx.x >> 6];
    if (is_bf16<DTS>(c.d)) encode_dispatch<BF16, EF, ET, FUSED>(c, patch);
    else encode_dispatch<F32, EF, ET, FUSED>(c, patch);
}

// The sparsifier's tensors, over the same tiles; PAIR: those with 16-channel blocks, else those with 8-channel
// blocks.  Kernels of their own: the selection over 16-channel blocks needs half as many registers again as the
// quantisers, and in one kernel every tensor would pay for that in occupancy.
template <int EF, int ET, bool FUSED, bool PAIR, int DTS>
__global__ __launch_bounds__(kTileThreads) void k_encode_nm(BatchView v, LaunchRange r)
{
    __shared__ __attribute__((aligned(16))) float patches[kTileThreads / 64][512];
    TileCtx c = locate_tile<true>(v, r);
    if (c.d.scale != SPARSE_NM || (c.d.nm_block == 16) != PAIR) return;
    float *patch = patches[(int)threadIdx.x >> 6];
    if (is_bf16<DTS>(c.d)) nm_encode_dispatch<BF16, PAIR, EF, ET, FUSED>(c, patch);
    else nm_encode_dispatch<F32, PAIR, EF, ET, FUSED>(c, patch);
}

// ---------------------------------------------------------------- a6 + a8: receiver decode

// replace: recon_t = D (naive compression) instead of recon_{t-1} + D.
template <int DT, int BITS, int MODE>
__device__ __forceinline__ void decode_tile(const TileCtx &c, bool replace)
{
    const TensorDev &d = c.d;
    const TensorPtrs &p = c.p;
    int chunk = c.colblock * kTileThreads + (int)threadIdx.x;
    if (chunk >= d.n_chunks) return;
    int64_t row0 = (int64_t)c.rowblock * c.rows;
    int64_t row1 = row0 + c.rows < d.n_tokens ? row0 + c.rows : d.n_tokens;
    const int64_t C = d.n_channels;
    const int64_t row_bytes = C * BITS / 8;
    const int n_groups = d.n_channels >> 7;
    F8 s, vj;
    if (MODE == 0) s = load_scales8(p.scales, (int64_t)chunk * kChunk);
    if (MODE == 2) vj = load_scales8(p.scales, (int64_t)chunk * kChunk);
    constexpr int U = 4;
    for (int64_t i0 = row0; i0 < row1; i0 += U) {
        Raw8<DT> br[U];
        uint32_t pk[U];
        float sg[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            int64_t i = i0 + u;
            if (i < row1) {
                // streaming hint: the line is written back by this workgroup (measured 5 % faster than a plain load)
                if (!replace) br[u].load_stream(p.recon, i * C + (int64_t)chunk * kChunk); else br[u].zero();
                pk[u] = load_codes<BITS>(p.codes + i * row_bytes, chunk);
                sg[u] = (MODE == 1) ? gconst<float>(p.scales)[i * n_groups + (chunk >> 4)]
                                    : (MODE == 2) ? gconst<float>(p.scales)[C + i] : 0.0f;
            } else {
                br[u].zero();
                pk[u] = 0;
                sg[u] = 0.0f;
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            int64_t i = i0 + u;
            if (i >= row1) break;
            if (MODE == 1) {
#pragma unroll
                for (int k = 0; k < 8; ++k) s.v[k] = sg[u];
            }
            if (MODE == 2) {
#pragma unroll
                for (int k = 0; k < 8; ++k) s.v[k] = sg[u] * vj.v[k];
            }
            F8 dq, b = br[u].widen(), nb;
            dequant8<BITS>(pk[u], s, dq);
#pragma unroll
            for (int k = 0; k < 8; ++k) nb.v[k] = replace ? dq.v[k] : b.v[k] + dq.v[k];
            Raw8<DT> out;
            out.narrow(nb);
            if (DT == BF16) out.store_stream(p.recon, i * C + (int64_t)chunk * kChunk);     // a whole line per 8 lanes, written once
            else out.store(p.recon, i * C + (int64_t)chunk * kChunk);
        }
    }
}

template <int DT, int KEEP, bool PAIR>
__device__ __forceinline__ void nm_decode_tile(const TileCtx &c, bool replace)
{
    const TensorDev &d = c.d;
    const TensorPtrs &p = c.p;
    const int chunk = c.colblock * kTileThreads + (int)threadIdx.x;
    if (chunk >= d.n_chunks) return;
    const int64_t row0 = (int64_t)c.rowblock * c.rows;
    const int64_t row1 = row0 + c.rows < d.n_tokens ? row0 + c.rows : d.n_tokens;
    const int64_t C = d.n_channels;
    constexpr int kValueBytes = KEEP * (DT == BF16 ? 2 : 4);
    const uint8_t *values = p.codes + ((d.n_tokens * d.n_chunks + 15) / 16) * 16;
    constexpr int U = 2;                                    // rows loaded together, then stored together
    for (int64_t i0 = row0; i0 < row1; i0 += U) {
        Raw8<DT> br[U];
        uint32_t mask[U];
        uint32_t vals[U][KEEP];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t i = i0 + u;
            if (i < row1) {
                // streaming hint: the line is written back by this workgroup (measured 5 % faster than a plain load)
                if (!replace) br[u].load_stream(p.recon, i * C + (int64_t)chunk * kChunk); else br[u].zero();
                mask[u] = load_codes<1>(p.codes + i * d.n_chunks, chunk);
                if (PAIR) nm_load_values<DT, KEEP>(values + (i * (d.n_chunks >> 1) + (chunk >> 1)) * kValueBytes, vals[u]);
                else nm_load_values<DT, KEEP>(values + (i * d.n_chunks + chunk) * kValueBytes, vals[u]);
            } else {
                br[u].zero();
                mask[u] = 0;
#pragma unroll
                for (int q = 0; q < KEEP; ++q) vals[u][q] = 0;
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t i = i0 + u;
            if (i >= row1) break;                           // uniform over the workgroup
            F8 dq, nb;
            int first = 0;
            if (PAIR) {     // the odd lane's values come after the even lane's
                const int lower = __builtin_popcount((uint32_t)__builtin_amdgcn_update_dpp(0, (int)mask[u], 0xB1, 0xF, 0xF, false));
                first = (chunk & 1) ? lower : 0;
            }
            nm_scatter8<DT, KEEP>(mask[u], vals[u], dq, first);
            const F8 b = br[u].widen();
#pragma unroll
            for (int k = 0; k < 8; ++k) nb.v[k] = replace ? dq.v[k] : b.v[k] + dq.v[k];
            Raw8<DT> out;
            out.narrow(nb);
            if (DT == BF16) out.store_stream(p.recon, i * C + (int64_t)chunk * kChunk);
            else out.store(p.recon, i * C + (int64_t)chunk * kChunk);
        }
    }
}

template <int DT> __device__ __forceinline__ void decode_dispatch(const TileCtx &c, bool replace)
{
    const TensorDev &d = c.d;
    if (d.scale == SPARSE_NM) {
        if (d.nm_block == 16) {
            if (d.bits == 1) nm_decode_tile<DT, 1, true>(c, replace);
            else if (d.bits == 2) nm_decode_tile<DT, 2, true>(c, replace);
            else nm_decode_tile<DT, 4, true>(c, replace);
        } else {
            if (d.bits == 1) nm_decode_tile<DT, 1, false>(c, replace);
            else if (d.bits == 2) nm_decode_tile<DT, 2, false>(c, replace);
            else nm_decode_tile<DT, 4, false>(c, replace);
        }
        return;
    }
    if (d.scale == SCALE_GROUP) { decode_tile<DT, 4, 1>(c, replace); return; }
    if (d.scale == SCALE_RANK1) {
        if (d.bits == 1) decode_tile<DT, 1, 2>(c, replace); else decode_tile<DT, 2, 2>(c, replace);
        return;
    }
    if (d.bits == 1) decode_tile<DT, 1, 0>(c, replace);
    else if (d.bits == 2) decode_tile<DT, 2, 0>(c, replace);
    else decode_tile<DT, 4, 0>(c, replace);
}

template <int DTS>
__global__ __launch_bounds__(kTileThreads) void k_decode(BatchView v, LaunchRange r)
{
    TileCtx c = locate_tile_of<TILES_DECODE>(v, r);
    if (c.d.scale == LOWRANK) return;
    if (is_bf16<DTS>(c.d)) decode_dispatch<BF16>(c, r.naive != 0); else decode_dispatch<F32>(c, r.naive != 0);
}

// ---------------------------------------------------------------- table uploads and fills

// The per-call device pointers travel in the kernel arguments (captured at
// launch, so the host arrays may be reused at once) and are written to the
// workspace table by one small block.
__global__ void k_upload_ptrs(PtrChunk chunk, TensorPtrs *dst, int n)
{
    int i = (int)threadIdx.x;
    if (i < n) dst[i] = chunk.p[i];
}

// The same way for the context's own tables (descriptors, prefix arrays): no host-to-device copy, so a
// context can be set up where copies from pageable memory are not allowed.
__global__ void k_upload_words(WordChunk chunk, uint32_t *dst, int n)
{
    for (int i = (int)threadIdx.x; i < n; i += (int)blockDim.x) dst[i] = chunk.w[i];
}

__global__ void k_fill_words(uint32_t *dst, uint32_t value, uint32_t n)
{
    for (uint32_t i = blockIdx.x * blockDim.x + threadIdx.x; i < n; i += gridDim.x * blockDim.x) dst[i] = value;
}

// item_tensor[i] = t for the items [item_prefix[t], item_prefix[t + 1]) of tensor t = blockIdx.x
__global__ void k_fill_item_tensor(const uint32_t *item_prefix, uint32_t *item_tensor)
{
    const uint32_t t = blockIdx.x, lo = item_prefix[t], hi = item_prefix[t + 1];
    for (uint32_t i = lo + threadIdx.x; i < hi; i += blockDim.x) item_tensor[i] = t;
}

}  // namespace

// ---------------------------------------------------------------- host-side launchers

hipError_t launch_upload_ptrs(const PtrChunk &chunk, TensorPtrs *dst, int n, hipStream_t s)
{
    hipLaunchKernelGGL(k_upload_ptrs, dim3(1), dim3(kMaxUploadTensors), 0, s, chunk, dst, n);
    return hipGetLastError();
}

hipError_t launch_upload_bytes(const void *src, void *dst, size_t bytes, hipStream_t s)
{
    const uint32_t *from = static_cast<const uint32_t *>(src);      // tables are arrays of 4-byte words
    uint32_t *to = static_cast<uint32_t *>(dst);
    size_t words = bytes / 4;
    while (words > 0) {
        WordChunk chunk;
        const int n = words < (size_t)kUploadWords ? (int)words : kUploadWords;
        for (int i = 0; i < n; ++i) chunk.w[i] = from[i];
        hipLaunchKernelGGL(k_upload_words, dim3(1), dim3(256), 0, s, chunk, to, n);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
        from += n;
        to += n;
        words -= (size_t)n;
    }
    return hipSuccess;
}

hipError_t launch_fill_words(void *dst, uint32_t value, size_t n_words, hipStream_t s)
{
    if (n_words == 0) return hipSuccess;
    const size_t want = (n_words + 255) / 256;
    hipLaunchKernelGGL(k_fill_words, dim3((unsigned)(want < 1024 ? want : 1024)), dim3(256), 0, s, static_cast<uint32_t *>(dst), value,
                       (uint32_t)n_words);
    return hipGetLastError();
}

hipError_t launch_fill_item_tensor(const uint32_t *item_prefix, uint32_t *item_tensor, int n_tensors, hipStream_t s)
{
    if (n_tensors <= 0) return hipSuccess;
    hipLaunchKernelGGL(k_fill_item_tensor, dim3((unsigned)n_tensors), dim3(256), 0, s, item_prefix, item_tensor);
    return hipGetLastError();
}

// Launches KERNEL<ARGS..., DTS> for the range's dtype selector, with `pad_lds` bytes of dynamic LDS (see kCapLdsBytes).
// The row-local kernels need few registers, and left alone 16 of their workgroups would share a CU.  They run
// faster with about 12 (measured on 42 x [16384, 3072] bf16, 4-bit group codes: 16 resident 3.71 ms, 12 3.53 ms,
// 10 3.52 ms, 8 3.57 ms, 6 4.07 ms; the receiver's kernel 1.54 -> 1.49 ms): with more, too many streams of reads
// and writes are open at once.  Dynamic LDS that nobody touches is what caps them: kCapLdsBytes per workgroup
// in total, 12 of which fit the 160 KB of a CU.
constexpr unsigned kCapLdsBytes = 13312;
#define CF_LAUNCH_DTS(KERNEL, ...)                                                                      \
    do {                                                                                                \
        if (r.dts == 0) hipLaunchKernelGGL((KERNEL<__VA_ARGS__, 0>), grid, block, pad_lds, s, v, r);            \
        else if (r.dts == 1) hipLaunchKernelGGL((KERNEL<__VA_ARGS__, 1>), grid, block, pad_lds, s, v, r);       \
        else hipLaunchKernelGGL((KERNEL<__VA_ARGS__, 2>), grid, block, pad_lds, s, v, r);                       \
    } while (0)

#define CF_LAUNCH_EF_ET(KERNEL, ...)                                                                    \
    do {                                                                                                \
        if (err_dtype == BF16) {                                                                        \
            if (ef == EF_RECON) CF_LAUNCH_DTS(KERNEL, EF_RECON, BF16 __VA_ARGS__);                      \
            else if (ef == EF_LITERAL) CF_LAUNCH_DTS(KERNEL, EF_LITERAL, BF16 __VA_ARGS__);             \
            else if (ef == EF_NAIVE) CF_LAUNCH_DTS(KERNEL, EF_NAIVE, BF16 __VA_ARGS__);                 \
            else CF_LAUNCH_DTS(KERNEL, EF_OFF, BF16 __VA_ARGS__);                                       \
        } else {                                                                                        \
            if (ef == EF_RECON) CF_LAUNCH_DTS(KERNEL, EF_RECON, F32 __VA_ARGS__);                       \
            else if (ef == EF_LITERAL) CF_LAUNCH_DTS(KERNEL, EF_LITERAL, F32 __VA_ARGS__);              \
            else if (ef == EF_NAIVE) CF_LAUNCH_DTS(KERNEL, EF_NAIVE, F32 __VA_ARGS__);                  \
            else CF_LAUNCH_DTS(KERNEL, EF_OFF, F32 __VA_ARGS__);                                        \
        }                                                                                               \
    } while (0)

hipError_t launch_warmup(const BatchView &v, const LaunchRange &r, int err_dtype, hipStream_t s)
{
    dim3 grid(r.ew_hi - r.ew_lo), block(kTileThreads);
    if (grid.x == 0) return hipSuccess;
    const unsigned pad_lds = 0;
    if (err_dtype == BF16) CF_LAUNCH_DTS(k_warmup, BF16);
    else CF_LAUNCH_DTS(k_warmup, F32);
    return hipGetLastError();
}

hipError_t launch_colreduce(const BatchView &v, const LaunchRange &r, int ef, int err_dtype, hipStream_t s)
{
    dim3 grid(r.tile_hi - r.tile_lo), block(kTileThreads);
    if (grid.x == 0) return hipSuccess;
    const unsigned pad_lds = 0;
    CF_LAUNCH_EF_ET(k_colreduce);
    return hipGetLastError();
}

hipError_t launch_finalize(const BatchView &v, const LaunchRange &r, hipStream_t s)
{
    dim3 grid(r.fin_hi - r.fin_lo), block(kFinalizeThreads);
    if (grid.x == 0) return hipSuccess;
    hipLaunchKernelGGL(k_finalize, grid, block, 0, s, v, r);
    return hipGetLastError();
}

hipError_t launch_finalize_rank1(const BatchView &v, const LaunchRange &r, hipStream_t s)
{
    if (r.count == 0) return hipSuccess;
    hipLaunchKernelGGL(k_finalize_rank1, dim3(r.count), dim3(kRank1Threads), 0, s, v, r);
    return hipGetLastError();
}

hipError_t launch_encode(const BatchView &v, const LaunchRange &r, int ef, int err_dtype, bool fused, hipStream_t s)
{
    dim3 grid(r.ew_hi - r.ew_lo), block(kTileThreads);
    if (grid.x == 0) return hipSuccess;
    const unsigned pad_lds = kCapLdsBytes - (unsigned)sizeof(float) * 512 * (kTileThreads / 64);       // the kernel's own patches count
    if (fused) CF_LAUNCH_EF_ET(k_encode, , true);
    else CF_LAUNCH_EF_ET(k_encode, , false);
    return hipGetLastError();
}

hipError_t launch_encode_nm(const BatchView &v, const LaunchRange &r, int ef, int err_dtype, bool fused, bool pair, hipStream_t s)
{
    dim3 grid(r.ew_hi - r.ew_lo), block(kTileThreads);
    if (grid.x == 0) return hipSuccess;
    const unsigned pad_lds = kCapLdsBytes - (unsigned)sizeof(float) * 512 * (kTileThreads / 64);
    if (pair) {
        if (fused) CF_LAUNCH_EF_ET(k_encode_nm, , true, true);
        else CF_LAUNCH_EF_ET(k_encode_nm, , false, true);
    } else {
        if (fused) CF_LAUNCH_EF_ET(k_encode_nm, , true, false);
        else CF_LAUNCH_EF_ET(k_encode_nm, , false, false);
    }
    return hipGetLastError();
}

hipError_t launch_decode(const BatchView &v, const LaunchRange &r, hipStream_t s)
{
    dim3 grid(r.dec_hi - r.dec_lo), block(kTileThreads);
    if (grid.x == 0) return hipSuccess;
    if (r.dts == 0) hipLaunchKernelGGL(k_decode<0>, grid, block, kCapLdsBytes, s, v, r);
    else if (r.dts == 1) hipLaunchKernelGGL(k_decode<1>, grid, block, kCapLdsBytes, s, v, r);
    else hipLaunchKernelGGL(k_decode<2>, grid, block, kCapLdsBytes, s, v, r);
    return hipGetLastError();
}

}  // namespace cf
