// Single-pass kernel for channel scales (arxiv 2507.17511, App. D
// "Quantization": v_j = mean_i |z_ij| needs every token of a channel before
// any code of that channel can be chosen).
//
// A two-kernel design reads x and recon twice from HBM.  Here a workgroup
// keeps its share of the operands in registers across the reduction instead:
//   item  = p_rows x 128 channels of one tensor, owned by one workgroup of 256
//           lanes (16 chunks of 8 channels x 16 row-lanes), 128 VGPRs of raw
//           operands per lane: 256 rows of bf16 x and recon (Sec. 3.2's feedback
//           folded into the residual against the reconstruction), half as many
//           of fp32, half as many again when the error buffer is an operand too
//           (the literal and the no-feedback recursions); for contexts of short
//           tensors half as tall and 256 channels wide (32 chunks x 8 row-lanes);
//   group = the items of one such stripe of one tensor; only they have
//           to agree on that stripe's scales, so there is no grid-wide barrier,
//           and different groups drift apart, which keeps HBM busy while some
//           workgroups wait.
// Per item: load -> |z| tree over the lane's rows -> LDS tree over row-lanes
// -> publish the item's partial (an aligned power-of-two block of the channel
// tree) -> every workgroup of the group fetches the group's partials as they
// appear and finishes the tree itself -> scales -> codes, error and
// reconstruction straight from the registers.
//
// A partial is its own ready flag: the buffer is filled with a pattern no
// partial can take before the kernel starts, and a reader fetches a slot again
// until it has changed.  One store and one load per hop; no counter.
//
// Forward progress does not depend on how the hardware schedules workgroups.
// Items are numbered group-major and dealt to the workgroups in index order
// (or, for short tensors, XCD-major: see the kernel), so the items of a group
// start at about the same time and a waiter normally sees the partials within
// microseconds.  But no workgroup waits for ever: one that has polled a slot
// `sp_wait_polls` times in vain GIVES ITS ITEM UP.  Up to that point it has
// written nothing but its own partial (codes, error and reconstruction are all
// written after the wait), so it only appends the item to a list in the
// workspace and goes on (or exits, which frees its slot for the workgroups the
// others are waiting for).  Every workgroup publishes its partial before it
// waits, so when the kernel has ended every partial of the call is there, and a
// second, normally empty launch of the same kernel walks the list and does the
// given-up items without any waiting.  The pass therefore always ends, on a
// device shared with other kernels and with a dispatcher that does not go by
// index too, and the outputs are the same bits either way.
#include "cf_device.h"
#include "cf_internal.h"

namespace cf {
namespace {

using namespace dev;

__device__ __forceinline__ void publish(float *p, float v) { __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ __forceinline__ float fetch(const float *p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }

// A partial that has not been published yet reads as this pattern: a negative NaN with every
// mantissa bit set, which neither a sum of magnitudes nor a maximum of magnitudes can produce.
constexpr uint32_t kUnpublished = 0xFFFFFFFFu;

constexpr int kPollBatch = 8;       // leaves fetched (and re-fetched) together

// tree_over whose leaves are other workgroups' partials: a leaf that still reads as kUnpublished is
// fetched again until its owner has stored it, at most max_polls times (then ok = false and the
// result is meaningless).  The data word is its own ready flag, so a group needs no counter and no
// second round trip.
template <bool IS_MAX, int LV>
__device__ __forceinline__ float tree_over_published(int n, const float *mine, int64_t stride, uint32_t max_polls, bool &ok)
{
    constexpr int NB = kPollBatch;
    float stack[LV];
#pragma unroll
    for (int l = 0; l < LV; ++l) stack[l] = 0.0f;
    const int nbatch = (n + NB - 1) / NB;
    int bpad = 1;
    while (bpad < nbatch) bpad <<= 1;
    for (int b = 0; b < bpad; ++b) {
        float vals[NB];
#pragma unroll
        for (int u = 0; u < NB; ++u) vals[u] = (b * NB + u < n) ? fetch(mine + (int64_t)(b * NB + u) * stride) : 0.0f;
        uint32_t polls = 0;
        for (;;) {
            uint32_t pending = 0;
#pragma unroll
            for (int u = 0; u < NB; ++u) pending |= (__float_as_uint(vals[u]) == kUnpublished ? 1u : 0u) << u;
            if (pending == 0) break;
            if (polls >= max_polls) { ok = false; break; }
            __builtin_amdgcn_s_sleep(1);
#pragma unroll
            for (int u = 0; u < NB; ++u)
                if ((pending >> u) & 1u) vals[u] = fetch(mine + (int64_t)(b * NB + u) * stride);
            ++polls;
        }
        // balanced tree over the batch: neighbours, then neighbours of neighbours, ...
#pragma unroll
        for (int w = 1; w < NB; w <<= 1)
#pragma unroll
            for (int u = 0; u < NB; u += 2 * w) vals[u] = comb<IS_MAX>(vals[u], vals[u + w]);
        tree_push<LV, IS_MAX>(stack, vals[0], b);
    }
    return tree_top<LV, IS_MAX>(stack);
}

// SCH: channels per stripe (kStripeChannels or kStripeChannelsWide); the 256 lanes are SCH / 8 chunks across
// by 2048 / SCH row-lanes down.
template <int SCH> struct alignas(16) Shared {
    float red[kPersistThreads / (SCH / kChunk)][SCH];       // 8 KB: level 2 of the tree; afterwards the waves' patches for whole-line stores
    float scale[SCH];
    uint32_t ok;
};

template <int DT, int BITS, int EF, int ET, bool FUSED, int SCH>
__device__ __forceinline__ bool persist_item(const BatchView &v, const LaunchRange &r, const TensorDev &d, const TensorPtrs &p, int stripe,
                                             int rb, Shared<SCH> &sh)
{
    constexpr int kStripeChannels = SCH, kStripeChunks = SCH / kChunk, kRowLanes = kPersistThreads / kStripeChunks;
    constexpr int RPT = single_pass_rows_per_lane(DT, EF);      // rows per lane
    constexpr bool IS_MAX = BITS == 4;
    constexpr bool HAS_B = EF != EF_NAIVE;                      // recon is an operand
    constexpr bool HAS_E = EF == EF_LITERAL || EF == EF_OFF;    // the error buffer is an operand
    const int tid = (int)threadIdx.x, cl = tid & (kStripeChunks - 1), rl = tid / kStripeChunks;
    const int chunk = stripe * kStripeChunks + cl;
    const bool cvalid = chunk < d.n_chunks;
    const int64_t row0 = (int64_t)rb * d.p_rows + rl * RPT;
    const int64_t C = d.n_channels;

    // ---- load the lane's rows (raw), all in flight at once
    Raw8<DT> xr[RPT], br[HAS_B ? RPT : 1];
    Raw8<ET> er[HAS_E ? RPT : 1];
#pragma unroll
    for (int k = 0; k < RPT; ++k) {
        const int64_t row = row0 + k;
        if (cvalid && row < d.n_tokens) {
            const int64_t e = row * C + (int64_t)chunk * kChunk;
            xr[k].load_stream(p.x, e);       // read once: keep the caches for the partials and the outputs
            if (HAS_B) br[HAS_B ? k : 0].load_stream(p.recon, e);
            if (HAS_E) er[HAS_E ? k : 0].load_stream(p.err, e);
        } else {                                    // zero padding of the tree / masked lanes
            xr[k].zero();
            if (HAS_B) br[HAS_B ? k : 0].zero();
            if (HAS_E) er[HAS_E ? k : 0].zero();
        }
    }
    const F8 none = {};

    // ---- a3, level 1: balanced tree over the lane's RPT consecutive rows
    // (a binary-counter stack: after row k the slots hold the partial trees of the rows seen so far;
    // k is a compile-time constant after unrolling, so every branch below folds away)
    constexpr int LVR = (RPT == 32) ? 6 : (RPT == 16) ? 5 : (RPT == 8) ? 4 : (RPT == 4) ? 3 : 2;
    F8 st[LVR];
#pragma unroll
    for (int k = 0; k < RPT; ++k) {
        F8 z = residual8<EF>(xr[k].widen(), HAS_B ? br[HAS_B ? k : 0].widen() : none, HAS_E ? er[HAS_E ? k : 0].widen() : none);
        F8 a;
#pragma unroll
        for (int j = 0; j < 8; ++j) a.v[j] = fabsf(z.v[j]);
        bool carry = true;
#pragma unroll
        for (int l = 0; l < LVR; ++l) {
            if (carry) {
                if ((k >> l) & 1) {
#pragma unroll
                    for (int j = 0; j < 8; ++j) a.v[j] = comb<IS_MAX>(st[l].v[j], a.v[j]);
                } else {
                    st[l] = a;
                    carry = false;
                }
            }
        }
    }
    {
        const F8 &top = st[LVR - 1];
        f32x4 *dst = reinterpret_cast<f32x4 *>(&sh.red[rl][cl * kChunk]);
        f32x4 lo, hi;
        lo.x = top.v[0]; lo.y = top.v[1]; lo.z = top.v[2]; lo.w = top.v[3];
        hi.x = top.v[4]; hi.y = top.v[5]; hi.z = top.v[6]; hi.w = top.v[7];
        dst[0] = lo;
        dst[1] = hi;
    }
    if (tid == 0) sh.ok = 1u;
    __syncthreads();

    // ---- level 2: tree over the row-lanes (consecutive RPT-row blocks); one lane per channel
    const bool owner = tid < kStripeChannels;
    const int64_t col = owner ? (int64_t)stripe * kStripeChannels + tid : C;
    float *partial = reinterpret_cast<float *>(v.workspace + d.p_partial_off);
    if (owner) {
        float lanes[kRowLanes];
#pragma unroll
        for (int q = 0; q < kRowLanes; ++q) lanes[q] = sh.red[q][tid];
#pragma unroll
        for (int w = 1; w < kRowLanes; w <<= 1)
#pragma unroll
            for (int q = 0; q < kRowLanes; q += 2 * w) lanes[q] = comb<IS_MAX>(lanes[q], lanes[q + w]);
        if (col < C) publish(partial + (int64_t)rb * C + col, lanes[0]);
    }
    // The partials are agent-scope atomic stores (written through to where the other XCDs read them)
    // and every partial is its own ready flag: nothing to drain, no arrival to count.

    // ---- level 3: the same tree continued over the group's item partials as they appear, then the scale
    if (col < C) {
        bool ok = true;
        const float res = tree_over_published<IS_MAX, 10>(d.p_n_rb, partial + col, C, r.sp_wait_polls, ok);
        const float s = IS_MAX ? res / 7.0f : res / (float)d.n_tokens;
        sh.scale[tid] = s;
        if (!ok) sh.ok = 0u;                        // a partial did not come in time
        if (ok && rb == 0) gmut<float>(p.scales)[col] = s;
    }
    __syncthreads();
    if (!sh.ok) return false;                       // uniform: nothing of this item has been written but its partial

    // ---- a4-a8 from the registers.  z is formed again from the raw operands: keeping the first
    // phase's fp32 residuals alive across the wait would double the register footprint.
#pragma unroll
    for (int k = 0; k < RPT; ++k) {
        xr[k].opaque();
        if (HAS_B) br[HAS_B ? k : 0].opaque();
        if (HAS_E) er[HAS_E ? k : 0].opaque();
    }
    F8 s;
    {
        const f32x4 *src = reinterpret_cast<const f32x4 *>(&sh.scale[cl * kChunk]);
        f32x4 a = src[0], b = src[1];
        s.v[0] = a.x; s.v[1] = a.y; s.v[2] = a.z; s.v[3] = a.w;
        s.v[4] = b.x; s.v[5] = b.y; s.v[6] = b.z; s.v[7] = b.w;
    }
    const int64_t row_bytes = C * BITS / 8;
    const bool wide = (d.n_channels & 31) == 0;
    // fp32 error rows go out as whole lines (see lines_exchange): a run is the kStripeChunks lanes of one row
    // segment; the wave's patch is its 2 KB of `red`, which nobody reads any more
    float *patch = &sh.red[0][0] + (tid >> 6) * 512;
    const int run_valid = d.n_chunks - stripe * kStripeChunks;
#pragma unroll
    for (int k = 0; k < RPT; ++k) {
        const int64_t row = row0 + k;
        const bool rvalid = row < d.n_tokens;
        __builtin_amdgcn_sched_barrier(0);      // one row at a time: keeps the live set inside the register budget
        const int64_t e = row * C + (int64_t)chunk * kChunk;
        const F8 b = HAS_B ? br[HAS_B ? k : 0].widen() : none;
        const F8 eold = HAS_E ? er[HAS_E ? k : 0].widen() : none;
        const F8 z = residual8<EF>(xr[k].widen(), b, eold);         // masked lanes and rows hold zeros
        F8 dq;
        uint32_t packed = quant8<BITS>(z, s, dq);
        if (rvalid && cvalid) store_codes_wide<BITS>(p.codes + row * row_bytes, chunk, packed, wide);
        F8 enew;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            float lost = z.v[j] - dq.v[j];
            if (EF == EF_OFF) lost = eold.v[j] + lost;
            enew.v[j] = lost;
        }
        if (ET == F32) {
            f32x4 pieces[2];
            lines_exchange<kStripeChunks>(patch, tid & 63, enew, pieces);
            if (rvalid)
                lines_store_stream<kStripeChunks>(static_cast<float *>(p.err) + row * C + (int64_t)stripe * kStripeChannels, cl,
                                                  run_valid, pieces);
        } else if (rvalid && cvalid) {
            Raw8<ET> eo;
            eo.narrow(enew);
            eo.store_stream(p.err, e);
        }
        if (FUSED && rvalid && cvalid) {
            F8 nb;
#pragma unroll
            for (int j = 0; j < 8; ++j) nb.v[j] = (EF == EF_NAIVE) ? dq.v[j] : b.v[j] + dq.v[j];
            Raw8<DT> out;
            out.narrow(nb);
            if (DT == BF16) out.store_stream(p.recon, e); else out.store(p.recon, e);
        }
    }
    return true;
}

template <int EF, int ET, bool FUSED, int SCH>
__global__ __launch_bounds__(kPersistThreads, 2) void k_single_pass(BatchView v, LaunchRange r)
{
    __shared__ Shared<SCH> sh;
    // Workgroups are handed to the 8 XCDs in turn (blockIdx.x % 8).  Taking item b in workgroup b runs the
    // consecutive items of a reduction group on different XCDs at the same time, and a tensor whose row
    // blocks number a multiple of 8 keeps each of them on one XCD, whose L2 then sees all stripes of a code row.  Short tensors
    // (few items per group) do better XCD-major, a run of consecutive items per XCD; the host chooses.
    // The second launch of a call (r.sp_redo): the items the first one gave up, from the list it left.
    uint32_t *const gave_up = v.error_flag + kGaveUpWord;
    const uint32_t n_todo = r.sp_redo ? *gconst<uint32_t>(gave_up) : r.item_hi - r.item_lo;
    uint32_t vb = blockIdx.x;
    if (r.sp_xcd_major && !r.sp_redo) {
        const uint32_t q = gridDim.x >> 3, rem = gridDim.x & 7u, xcd = blockIdx.x & 7u;
        vb = xcd * q + (xcd < rem ? xcd : rem) + (blockIdx.x >> 3);
    }
    for (uint32_t k = vb; k < n_todo; k += gridDim.x) {
        const uint32_t item = r.sp_redo ? v.gave_up_items[k] : r.item_lo + k;
        const int t = (int)v.item_tensor[item];
        const TensorDev d = v.descs[t];                             // by value: scalar registers, never re-read
        const TensorPtrs p = v.ptrs[t];
        const uint32_t local = item - d.p_item_begin;               // group-major: stripe, then row block
        const int stripe = (int)(local / (uint32_t)d.p_n_rb);
        const int rb = (int)(local % (uint32_t)d.p_n_rb);
        bool done;
        if (d.dtype == BF16) {
            if (d.bits == 1) done = persist_item<BF16, 1, EF, ET, FUSED, SCH>(v, r, d, p, stripe, rb, sh);
            else if (d.bits == 2) done = persist_item<BF16, 2, EF, ET, FUSED, SCH>(v, r, d, p, stripe, rb, sh);
            else done = persist_item<BF16, 4, EF, ET, FUSED, SCH>(v, r, d, p, stripe, rb, sh);
        } else {
            if (d.bits == 1) done = persist_item<F32, 1, EF, ET, FUSED, SCH>(v, r, d, p, stripe, rb, sh);
            else if (d.bits == 2) done = persist_item<F32, 2, EF, ET, FUSED, SCH>(v, r, d, p, stripe, rb, sh);
            else done = persist_item<F32, 4, EF, ET, FUSED, SCH>(v, r, d, p, stripe, rb, sh);
        }
        if (!done && threadIdx.x == 0) {
            if (r.sp_redo) {        // cannot happen: every partial was published before the first launch ended
                __hip_atomic_store(v.error_flag, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            } else {
                const uint32_t slot = __hip_atomic_fetch_add(gave_up, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                *gmut<uint32_t>(v.gave_up_items + slot) = item;
            }
        }
        __syncthreads();            // a looping workgroup reuses the shared arrays for its next item
    }
}

// Every partial starts a call as "unpublished" (a fill kernel, so the call can be captured in a graph).  The
// first kernel of a single pass also takes the call's last batch of device pointers to the table (see
// k_upload_ptrs): one launch fewer per call.
__global__ void k_reset_partials(u32x4 *words, uint64_t n_vec, uint32_t *gave_up, PtrChunk chunk, TensorPtrs *dst, int n)
{
    if (blockIdx.x == 0 && threadIdx.x == 0) *gmut<uint32_t>(gave_up) = 0u;        // the list of given-up items is empty
    if (blockIdx.x == 0 && (int)threadIdx.x < n) dst[threadIdx.x] = chunk.p[threadIdx.x];
    const u32x4 fill = (u32x4)(kUnpublished);
    for (uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n_vec; i += (uint64_t)gridDim.x * blockDim.x)
        *gmut<u32x4>(words + i) = fill;
}

template <int EF, int ET, bool FUSED, int SCH> const void *persistent_fn() { return reinterpret_cast<const void *>(&k_single_pass<EF, ET, FUSED, SCH>); }

template <int EF, int SCH> const void *pick_width(int err_dtype, bool fused)
{
    if (err_dtype == BF16) return fused ? persistent_fn<EF, BF16, true, SCH>() : persistent_fn<EF, BF16, false, SCH>();
    return fused ? persistent_fn<EF, F32, true, SCH>() : persistent_fn<EF, F32, false, SCH>();
}

template <int EF> const void *pick_ef(int err_dtype, bool fused, bool wide)
{
    return wide ? pick_width<EF, kStripeChannelsWide>(err_dtype, fused) : pick_width<EF, kStripeChannels>(err_dtype, fused);
}

const void *pick(int ef, int err_dtype, bool fused, bool wide)
{
    if (ef == EF_LITERAL) return pick_ef<EF_LITERAL>(err_dtype, fused, wide);
    if (ef == EF_OFF) return pick_ef<EF_OFF>(err_dtype, fused, wide);
    if (ef == EF_NAIVE) return pick_ef<EF_NAIVE>(err_dtype, fused, wide);
    return pick_ef<EF_RECON>(err_dtype, fused, wide);
}

}  // namespace

int persistent_max_blocks_per_cu(int ef, int err_dtype, bool fused, bool wide)
{
    int n = 0;
    hipError_t e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, pick(ef, err_dtype, fused, wide), kPersistThreads, 0);
    if (e != hipSuccess) { (void)hipGetLastError(); return 0; }
    return n;
}

hipError_t launch_reset_partials(const BatchView &v, const LaunchRange &r, const PtrChunk &chunk, TensorPtrs *dst, int n, hipStream_t s)
{
    static_assert(kMaxUploadTensors <= 256, "one block of k_reset_partials writes the pointer sets");
    const bool none = r.p_partial_hi <= r.p_partial_lo;
    if (none && n == 0) return hipSuccess;
    const uint64_t n_vec = none ? 0 : (r.p_partial_hi - r.p_partial_lo) / 16;      // offsets are multiples of 256
    const uint64_t want = n_vec == 0 ? 1 : (n_vec + 255) / 256;
    hipLaunchKernelGGL(k_reset_partials, dim3((unsigned)(want < 2048 ? want : 2048)), dim3(256), 0, s,
                       reinterpret_cast<u32x4 *>(v.workspace + r.p_partial_lo), n_vec, v.error_flag + kGaveUpWord, chunk, dst, n);
    return hipGetLastError();
}

// one_shot: one workgroup per item instead of a smaller grid whose workgroups loop over the items.
// A workgroup that loops has to drain its stores before its next loads count as returned (the loads and
// stores of a wave share one in-order counter); one that exits leaves the draining to the memory system
// while the next workgroup already loads: measured faster by 15 % (114 x [4096, 3072] bf16: 2.65 against 3.04 ms).  Neither form needs co-residency to
// finish (see the top of the file); the looping grid is for callers who share the device with other work
// and want the codec to hold a fixed number of workgroup slots.  redo: the second launch of a call, over
// the items the first one gave up (kRedoGrid workgroups; all of them leave at once when the list is empty).
hipError_t launch_single_pass(const BatchView &v, const LaunchRange &r, int ef, int err_dtype, bool fused, bool wide, int grid,
                             bool one_shot, bool redo, hipStream_t s)
{
    if (r.item_hi == r.item_lo) return hipSuccess;
    uint32_t items = r.item_hi - r.item_lo;
    if ((uint32_t)grid > items) grid = (int)items;
    if (grid < 1) grid = 1;
    BatchView vv = v;
    LaunchRange rr = r;
    rr.sp_redo = redo ? 1u : 0u;
    if (redo) rr.sp_wait_polls = 0u;        // every partial is there; nothing to wait for
    const uint32_t n_wg = redo ? (items < (uint32_t)kRedoGrid ? items : (uint32_t)kRedoGrid) : one_shot ? items : (uint32_t)grid;
    void *args[] = {&vv, &rr};
    return hipLaunchKernel(pick(ef, err_dtype, fused, wide), dim3(n_wg), dim3(kPersistThreads), args, 0, s);
}

}  // namespace cf
