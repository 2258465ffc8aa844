// Internal interface between the C-ABI layer (cf_api.cpp) and the gfx950
// kernels (cf_kernels.hip).  Not installed; not part of the ABI.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace cf {

// Every tile of the tiled kernels is TILE_ROWS(rb) x TILE_CHANNELS: 128 lanes
// each own 8 consecutive channels (one 128-bit load of bf16).
constexpr int kTileThreads = 128;
constexpr int kChunk = 8;                                   // channels per lane
constexpr int kTileChannels = kTileThreads * kChunk;        // 1024
constexpr int kFinalizeThreads = 256;                       // columns per finalise block
constexpr int kRank1Threads = 1024;                         // one block per tensor finishes the token scales u
constexpr int kMaxRank1Colblocks = 128;                     // rank-1 scales: C <= 128 * 1024
constexpr int kMaxUploadTensors = 64;                       // pointer sets per upload launch
// Single-pass path: one workgroup of 256 lanes keeps an item of p_rows x 128
// channels (x and recon, raw) in registers between the scale reduction and the
// encode; lanes are 16 chunks x 16 row-lanes, so a row segment is 256 bytes of
// bf16 and a row's 1-bit codes of one item are 16 bytes.  Measured on 114 x
// [4096, 3072] bf16: 64- / 128- / 256-channel stripes (8 / 16 / 32 items per
// reduction group) 2.94 / 2.86 / 2.92 ms; 32-channel ones (64-byte segments)
// were 50 % slower.  Short tensors do better with the wide stripe (items half
// as tall, twice as many per group): 57 x [1024, 3072] 0.417 -> 0.382 ms; a
// context whose tallest channel-scale tensor makes at most 12 items per group
// with the narrow stripe (bf16: N <= 3072) takes the wide one.
constexpr int kPersistThreads = 256;
constexpr int kStripeChannels = 128;
constexpr int kStripeChannelsWide = 2 * kStripeChannels;    // 256
// Rows a lane of the single-pass kernel keeps in registers: 128 VGPRs of raw operands, i.e. 16 rows of bf16 x and
// recon, half as many of fp32, half as many again when the error buffer is an operand too (CF_EF_LITERAL = 1,
// CF_EF_OFF = 2).  Measured on 114 x [4096, 3072] bf16 (two waves per SIMD): 16 rows 2.65 ms; 8 rows at three
// waves per SIMD 2.97 ms, at four (spills) 4.8 ms.  dtype: cf_dtype (CF_F32 = 0).
constexpr int single_pass_rows_per_lane(int dtype, int ef) { return 16 / (dtype == 0 ? 2 : 1) / ((ef == 1 || ef == 2) ? 2 : 1); }
// A workgroup polls a missing partial this many times (a microsecond or two each) before it gives its item up.
constexpr uint32_t kWaitPolls = 4096;
constexpr int kGaveUpWord = 32;                             // 128 bytes behind the error word: how many items the call's first launch gave up
constexpr int kRedoGrid = 512;                              // workgroups of the launch that does them

// Static description of one tensor; built at cf_init, lives in the workspace.
struct alignas(16) TensorDev {
    int64_t n_tokens;
    int32_t n_channels;
    int32_t n_chunks;       // C / 8
    int32_t dtype;          // cf_dtype
    int32_t bits;           // 1 | 2 | 4
    int32_t scale;          // cf_scale_kind
    int32_t rb_rows;        // rows per tile (power of two, multiple of 8)
    int32_t n_rowblocks;    // ceil(N / rb_rows)
    int32_t n_colblocks;    // ceil(n_chunks / 128)
    uint32_t tile_begin;    // id of this tensor's first tile in the batched grids
    uint32_t fin_begin;     // id of its first finalise block
    uint64_t partial_off;   // byte offset in the workspace of partial[n_rowblocks][C] (channel scales)
    // single-pass path (channel scales): items of p_rows x kStripeChannels (or kStripeChannelsWide)
    uint64_t p_partial_off; // byte offset of partial[p_n_rb][C]
    int32_t p_rows;         // rows per item (row-lanes x single_pass_rows_per_lane); 0 = tensor not on this path
    int32_t p_n_rb;         // ceil(N / p_rows): items per reduction group
    int32_t p_n_stripes;    // ceil(C / stripe width of the context): reduction groups of this tensor
    uint32_t p_item_begin;  // id of this tensor's first item
    uint32_t p_pad_;
    // element-wise kernels (warm-up, encode, decode): short tiles of ew_rows x 1024 channels
    int32_t ew_rows;
    int32_t ew_n_rowblocks; // ceil(N / ew_rows)
    uint32_t ew_tile_begin;
    // the receiver's kernel does less per row and likes taller tiles: dec_rows x 1024 channels
    int32_t dec_rows;
    int32_t dec_n_rowblocks;
    uint32_t dec_tile_begin;
    uint32_t dec_pad_;
    // rank-1 scales: per-row sums of |z| over each 1024-channel tile, rowpart[N][n_colblocks]
    uint32_t nm_block;      // N:M sparsifier: M, channels per block (8 or 16)
                            // low-rank compressor: 4 when the factors travel as 4-bit integers, else 0
    uint64_t rowpart_off;
    // low-rank compressor: P = A Q [N][32], Z = A^T P [C][32], Q in the order k_lr_project reads it (all fp32)
    uint64_t lr_p_off, lr_z_off, lr_q_off;
};

static_assert(sizeof(TensorDev) % 4 == 0, "tables travel as 4-byte words");

// Per-call device pointers of one tensor; uploaded into the workspace.
struct TensorPtrs {
    const void *x;
    void *recon;
    void *err;
    uint8_t *codes;
    float *scales;
};

struct PtrChunk {
    TensorPtrs p[kMaxUploadTensors];
};

// A piece of one of the context's tables on its way to the workspace inside a kernel's arguments.
constexpr int kUploadWords = 896;
struct WordChunk {
    uint32_t w[kUploadWords];
};

// Device view of a context's workspace.
struct BatchView {
    const TensorDev *descs;     // [n_tensors]
    const TensorPtrs *ptrs;     // [n_tensors]
    const uint32_t *tile_prefix;    // [n_tensors + 1] reduction tiles
    const uint32_t *ew_prefix;      // [n_tensors + 1] element-wise tiles
    const uint32_t *dec_prefix;     // [n_tensors + 1] decode tiles
    const uint32_t *fin_prefix;     // [n_tensors + 1]
    const uint32_t *item_prefix;    // [n_tensors + 1] items of the single-pass path
    const uint32_t *item_tensor;    // [n_items] tensor of every item: one load where a search over the prefix would be seven
    uint32_t *error_flag;           // set if the redo launch finds a partial missing (cannot happen); kGaveUpWord words on: the give-up counter
    uint32_t *gave_up_items;        // [n_items] the items the first launch of a call gave up
    uint8_t *workspace;
    int32_t n_tensors;
};

struct LaunchRange {
    int32_t first, count;       // tensors
    uint32_t tile_lo, tile_hi;  // reduction tiles of [first, first+count)
    uint32_t ew_lo, ew_hi;      // element-wise tiles
    uint32_t dec_lo, dec_hi;    // decode tiles
    uint32_t fin_lo, fin_hi;    // finalise blocks
    uint32_t item_lo, item_hi;  // single-pass items
    uint32_t sp_xcd_major;      // single-pass kernel: deal the items XCD-major (a run of consecutive items per XCD)
    uint32_t sp_wait_polls;     // single-pass kernel: polls of a missing partial before the workgroup gives its item up
    uint32_t sp_redo;           // single-pass kernel: this is the launch over the given-up items
    uint64_t p_partial_lo, p_partial_hi;    // workspace bytes holding the single-pass partials of the range
    int32_t dts;                // storage dtype of every tensor in the range (cf_dtype), or 2 if mixed
    int32_t only_group_scale;   // tiled encode: skip tensors the single-pass kernel covers
    int32_t naive;              // decode: recon_t = D instead of recon_{t-1} + D (CF_EF_NAIVE)
    int32_t lr_max_channels;    // low-rank tensors of the range: largest C and N (0 = none)
    int64_t lr_max_tokens;
};

enum class Op { Compress, StepFused };

hipError_t launch_upload_ptrs(const PtrChunk &chunk, TensorPtrs *dst, int n, hipStream_t s);
// Host tables (multiples of 4 bytes) to the workspace through kernel arguments; fills; the item -> tensor table
hipError_t launch_upload_bytes(const void *src, void *dst, size_t bytes, hipStream_t s);
hipError_t launch_fill_words(void *dst, uint32_t value, size_t n_words, hipStream_t s);
hipError_t launch_fill_item_tensor(const uint32_t *item_prefix, uint32_t *item_tensor, int n_tensors, hipStream_t s);

// The library's own scratch for callers that cannot allocate (cf_static.hip): one array per device, resolved on
// first use with that device current.
constexpr size_t kStaticScratchBytes = (size_t)16 << 20;
hipError_t static_scratch(void **ptr);
hipError_t launch_warmup(const BatchView &v, const LaunchRange &r, int err_dtype, hipStream_t s);
hipError_t launch_colreduce(const BatchView &v, const LaunchRange &r, int ef, int err_dtype, hipStream_t s);
hipError_t launch_finalize(const BatchView &v, const LaunchRange &r, hipStream_t s);
hipError_t launch_finalize_rank1(const BatchView &v, const LaunchRange &r, hipStream_t s);
hipError_t launch_encode(const BatchView &v, const LaunchRange &r, int ef, int err_dtype, bool fused, hipStream_t s);
hipError_t launch_encode_nm(const BatchView &v, const LaunchRange &r, int ef, int err_dtype, bool fused, bool pair, hipStream_t s);
hipError_t launch_decode(const BatchView &v, const LaunchRange &r, hipStream_t s);

// Low-rank compressor (cf_lowrank.hip): rank 32, C a multiple of 32 and at most kLowRankMaxChannels.
constexpr int kLowRankRank = 32;
constexpr int kLowRankMaxChannels = 3072;
// min_iters: only tensors whose descriptor asks for at least that many subspace iterations take part
hipError_t launch_lr_orth(const BatchView &v, const LaunchRange &r, bool from_q0, int min_iters, hipStream_t s);
hipError_t launch_lr_project(const BatchView &v, const LaunchRange &r, bool wire, int min_iters, hipStream_t s);
hipError_t launch_lr_backproject(const BatchView &v, const LaunchRange &r, int min_iters, hipStream_t s);
// 4-bit factors: U from P (fp32, in the workspace) onto the wire, after the last projection
hipError_t launch_lr_quant_u(const BatchView &v, const LaunchRange &r, hipStream_t s);
hipError_t launch_lr_encode(const BatchView &v, const LaunchRange &r, int err_dtype, bool fused, hipStream_t s);
hipError_t launch_lr_decode(const BatchView &v, const LaunchRange &r, hipStream_t s);

// Single-pass kernel (channel scales, every error-feedback mode).
int persistent_max_blocks_per_cu(int ef, int err_dtype, bool fused, bool wide);
// wide: items of kStripeChannelsWide channels (the layout's choice, fixed at cf_init); one_shot: a workgroup per
// item, else `grid` workgroups that loop over the items
hipError_t launch_single_pass(const BatchView &v, const LaunchRange &r, int ef, int err_dtype, bool fused, bool wide, int grid,
                             bool one_shot, bool redo, hipStream_t s);
// also writes `n` pointer sets of the call to the table (dst), which saves the call a launch of k_upload_ptrs; n may be 0
hipError_t launch_reset_partials(const BatchView &v, const LaunchRange &r, const PtrChunk &chunk, TensorPtrs *dst, int n, hipStream_t s);

}  // namespace cf
