// Single-pass kernel for channel scales (arxiv 2507.17511, App. D
// "Quantization": v_j = mean_i |z_ij| needs every token of a channel before
// any code of that channel can be chosen).
//
// A two-kernel design reads x and recon twice from HBM.  Here a workgroup
// keeps its share of x and recon in registers across the reduction instead:
//   item  = p_rows x 128 channels of one tensor (256 rows of bf16, 128 of fp32:
//           128 VGPRs of raw data per lane), owned by one workgroup of 256 lanes
//           (16 chunks of 8 channels x 16 row-lanes); for contexts of short
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
// Items are numbered group-major and dealt to the workgroups in index order
// (or, for short tensors, XCD-major: see the kernel), so the items of a group
// start at about the same time.  Every wait ends
// because the waited-for items are running or about to start: under a
// cooperative launch (a co-resident grid that loops over the items, at least
// as large as the largest group) by construction; under an ordinary launch of
// one workgroup per item because workgroups start in index order (see
// launch_single_pass).  Waits are bounded all the same: on expiry the workgroup
// raises the error flag and leaves.
#include "cf_device.h"
#include "cf_internal.h"

#ifndef CF_POLL_BATCH
#define CF_POLL_BATCH 8
#endif

namespace cf {
namespace {

using namespace dev;

__device__ __forceinline__ void publish(float *p, float v) { __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ __forceinline__ float fetch(const float *p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }

// A partial that has not been published yet reads as this pattern: a negative NaN with every
// mantissa bit set, which neither a sum of magnitudes nor a maximum of magnitudes can produce.
constexpr uint32_t kUnpublished = 0xFFFFFFFFu;

// tree_over whose leaves are other workgroups' partials: a leaf that still reads as kUnpublished is
// fetched again (bounded) until its owner has stored it.  The data word is its own ready flag, so
// a group needs no counter and no second round trip.
template <bool IS_MAX, int LV>
__device__ __forceinline__ float tree_over_published(int n, const float *mine, int64_t stride, bool &ok)
{
    constexpr int NB = CF_POLL_BATCH;               // leaves fetched (and re-fetched) together
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
        uint32_t spins = 0;
        for (;;) {
            uint32_t pending = 0;
#pragma unroll
            for (int u = 0; u < NB; ++u) pending |= (__float_as_uint(vals[u]) == kUnpublished ? 1u : 0u) << u;
            if (pending == 0) break;
#ifdef CF_EXP_NOWAIT
            break;      // timing experiment only: wrong scales
#endif
            if (spins >= kSpinLimit) { ok = false; break; }
            __builtin_amdgcn_s_sleep(1);
#pragma unroll
            for (int u = 0; u < NB; ++u)
                if ((pending >> u) & 1u) vals[u] = fetch(mine + (int64_t)(b * NB + u) * stride);
            ++spins;
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
#ifndef CF_SP_LDS_ROWS
#define CF_SP_LDS_ROWS 0
#endif
template <int SCH> struct alignas(16) Shared {
    float red[kPersistThreads / (SCH / kChunk)][SCH];
    float scale[SCH];
    uint32_t ok;
    u32x4 stage[CF_SP_LDS_ROWS > 0 ? CF_SP_LDS_ROWS : 1][kPersistThreads];     // recon rows that wait in LDS instead of registers
};

// A lane's own slot of a staged row (only the lane itself ever touches it: no barrier).
template <int DT> __device__ __forceinline__ void stage_put(u32x4 (*stage)[kPersistThreads], int k, int tid, const Raw8<DT> &r);
template <> __device__ __forceinline__ void stage_put<BF16>(u32x4 (*stage)[kPersistThreads], int k, int tid, const Raw8<BF16> &r) { stage[k][tid] = r.w; }
template <> __device__ __forceinline__ void stage_put<F32>(u32x4 (*stage)[kPersistThreads], int k, int tid, const Raw8<F32> &r)
{
    stage[2 * k][tid] = __builtin_bit_cast(u32x4, r.a);
    stage[2 * k + 1][tid] = __builtin_bit_cast(u32x4, r.b);
}
template <int DT> __device__ __forceinline__ Raw8<DT> stage_get(u32x4 (*stage)[kPersistThreads], int k, int tid);
template <> __device__ __forceinline__ Raw8<BF16> stage_get<BF16>(u32x4 (*stage)[kPersistThreads], int k, int tid)
{
    Raw8<BF16> r;
    r.w = stage[k][tid];
    return r;
}
template <> __device__ __forceinline__ Raw8<F32> stage_get<F32>(u32x4 (*stage)[kPersistThreads], int k, int tid)
{
    Raw8<F32> r;
    r.a = __builtin_bit_cast(f32x4, stage[2 * k][tid]);
    r.b = __builtin_bit_cast(f32x4, stage[2 * k + 1][tid]);
    return r;
}

template <int DT, int BITS, int ET, bool FUSED, int SCH>
__device__ __forceinline__ bool persist_item(const BatchView &v, const TensorDev &d, const TensorPtrs &p, int stripe,
                                             int rb, Shared<SCH> &sh)
{
    constexpr int kStripeChannels = SCH, kStripeChunks = SCH / kChunk, kRowLanes = kPersistThreads / kStripeChunks;
    constexpr int RPT = (DT == BF16) ? CF_SP_RPT : CF_SP_RPT / 2;      // rows per lane
    constexpr bool IS_MAX = BITS == 4;
    const int tid = (int)threadIdx.x, cl = tid & (kStripeChunks - 1), rl = tid / kStripeChunks;
    const int chunk = stripe * kStripeChunks + cl;
    const bool cvalid = chunk < d.n_chunks;
    const int64_t row0 = (int64_t)rb * d.p_rows + rl * RPT;
    const int64_t C = d.n_channels;

    // ---- load the lane's rows (raw), all in flight at once.  The first LR rows of recon wait in LDS,
    // not in registers (loaded first, so that they have arrived and gone to LDS while the rest is on its way).
    constexpr int LR = (DT == BF16) ? CF_SP_LDS_ROWS : CF_SP_LDS_ROWS / 2;
    Raw8<DT> xr[RPT], br[RPT - LR > 0 ? RPT - LR : 1];
    {
        Raw8<DT> tmp[LR > 0 ? LR : 1];
#pragma unroll
        for (int k = 0; k < LR; ++k) {
            const int64_t row = row0 + k;
            if (cvalid && row < d.n_tokens) tmp[k].load_stream(p.recon, row * C + (int64_t)chunk * kChunk);
            else tmp[k].zero();
        }
#pragma unroll
        for (int k = 0; k < RPT; ++k) {
            const int64_t row = row0 + k;
            if (cvalid && row < d.n_tokens) {
                const int64_t e = row * C + (int64_t)chunk * kChunk;
#ifdef CF_EXP_X_PLAIN
                xr[k].load(p.x, e);
#else
                xr[k].load_stream(p.x, e);       // read once: keep the caches for the partials and the outputs
#endif
                if (k >= LR) br[k >= LR ? k - LR : 0].load_stream(p.recon, e);
            } else {                                    // zero padding of the tree / masked lanes
                xr[k].zero();
                if (k >= LR) br[k >= LR ? k - LR : 0].zero();
            }
        }
#pragma unroll
        for (int k = 0; k < LR; ++k) stage_put<DT>(sh.stage, k, tid, tmp[k]);
    }
    auto recon_row = [&](int k) -> Raw8<DT> { return k < LR ? stage_get<DT>(sh.stage, k < LR ? k : 0, tid) : br[k >= LR ? k - LR : 0]; };

    // ---- a3, level 1: balanced tree over the lane's RPT consecutive rows
    // (a binary-counter stack: after row k the slots hold the partial trees of the rows seen so far;
    // k is a compile-time constant after unrolling, so every branch below folds away)
    constexpr int LVR = (RPT == 32) ? 6 : (RPT == 16) ? 5 : (RPT == 8) ? 4 : (RPT == 4) ? 3 : 2;
    F8 st[LVR];
    const F8 none = {};
#pragma unroll
    for (int k = 0; k < RPT; ++k) {
        F8 z = residual8<EF_RECON>(xr[k].widen(), recon_row(k).widen(), none);
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
        const float res = tree_over_published<IS_MAX, 10>(d.p_n_rb, partial + col, C, ok);
        const float s = IS_MAX ? res / 7.0f : res / (float)d.n_tokens;
        sh.scale[tid] = s;
        if (rb == 0) gmut<float>(p.scales)[col] = s;
        if (!ok) {                                  // a bounded wait expired: flag it and leave
            sh.ok = 0u;
            __hip_atomic_store(v.error_flag, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
    __syncthreads();
    if (!sh.ok) return false;

    // ---- a4-a8 from the registers.  z is formed again from the raw operands: keeping the first
    // phase's fp32 residuals alive across the wait would double the register footprint.
#pragma unroll
    for (int k = 0; k < RPT; ++k) {
        xr[k].opaque();
        if (k >= LR) br[k >= LR ? k - LR : 0].opaque();
    }
    {
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
            F8 b = recon_row(k).widen();
            F8 z = residual8<EF_RECON>(xr[k].widen(), b, none);     // masked lanes and rows hold zeros
            F8 dq;
            uint32_t packed = quant8<BITS>(z, s, dq);
            if (rvalid && cvalid) store_codes_wide<BITS>(p.codes + row * row_bytes, chunk, packed, wide);
            F8 enew;
#pragma unroll
            for (int j = 0; j < 8; ++j) enew.v[j] = z.v[j] - dq.v[j];
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
                for (int j = 0; j < 8; ++j) nb.v[j] = b.v[j] + dq.v[j];
                Raw8<DT> out;
                out.narrow(nb);
                if (DT == BF16) out.store_stream(p.recon, e); else out.store(p.recon, e);
            }
        }
    }
    return true;
}

template <int ET, bool FUSED, int SCH>
__global__ __launch_bounds__(kPersistThreads, CF_SP_WAVES) void k_single_pass(BatchView v, LaunchRange r)
{
    __shared__ Shared<SCH> sh;
    // Workgroups are handed to the 8 XCDs in turn (blockIdx.x % 8).  Taking item b in workgroup b runs the
    // consecutive items of a reduction group on different XCDs at the same time, and a tensor whose row
    // blocks number a multiple of 8 keeps each of them on one XCD, whose L2 then sees all stripes of a code row.  Short tensors
    // (few items per group) do better XCD-major, a run of consecutive items per XCD; the host chooses.
    uint32_t vb = blockIdx.x;
    if (r.sp_xcd_major) {
        const uint32_t q = gridDim.x >> 3, rem = gridDim.x & 7u, xcd = blockIdx.x & 7u;
        vb = xcd * q + (xcd < rem ? xcd : rem) + (blockIdx.x >> 3);
    }
    for (uint32_t item = r.item_lo + vb; item < r.item_hi; item += gridDim.x) {
        const int t = (int)v.item_tensor[item];
        const TensorDev d = v.descs[t];                             // by value: scalar registers, never re-read
        const TensorPtrs p = v.ptrs[t];
        const uint32_t local = item - d.p_item_begin;               // group-major: stripe, then row block
#ifdef CF_EXP_RBMAJOR
        const int stripe = (int)(local % (uint32_t)d.p_n_stripes);
        const int rb = (int)(local / (uint32_t)d.p_n_stripes);
#else
        const int stripe = (int)(local / (uint32_t)d.p_n_rb);
        const int rb = (int)(local % (uint32_t)d.p_n_rb);
#endif
        bool ok;
        if (d.dtype == BF16) {
            if (d.bits == 1) ok = persist_item<BF16, 1, ET, FUSED, SCH>(v, d, p, stripe, rb, sh);
            else if (d.bits == 2) ok = persist_item<BF16, 2, ET, FUSED, SCH>(v, d, p, stripe, rb, sh);
            else ok = persist_item<BF16, 4, ET, FUSED, SCH>(v, d, p, stripe, rb, sh);
        } else {
            if (d.bits == 1) ok = persist_item<F32, 1, ET, FUSED, SCH>(v, d, p, stripe, rb, sh);
            else if (d.bits == 2) ok = persist_item<F32, 2, ET, FUSED, SCH>(v, d, p, stripe, rb, sh);
            else ok = persist_item<F32, 4, ET, FUSED, SCH>(v, d, p, stripe, rb, sh);
        }
        if (!ok) return;                                            // uniform over the workgroup
    }
}

// Every partial starts a call as "unpublished" (a fill kernel, so the call can be captured in a graph).
__global__ void k_reset_partials(u32x4 *words, uint64_t n_vec)
{
    const u32x4 fill = (u32x4)(kUnpublished);
    for (uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n_vec; i += (uint64_t)gridDim.x * blockDim.x)
        *gmut<u32x4>(words + i) = fill;
}

template <int ET, bool FUSED, int SCH> const void *persistent_fn() { return reinterpret_cast<const void *>(&k_single_pass<ET, FUSED, SCH>); }

template <int SCH> const void *pick_width(int err_dtype, bool fused)
{
    if (err_dtype == BF16) return fused ? persistent_fn<BF16, true, SCH>() : persistent_fn<BF16, false, SCH>();
    return fused ? persistent_fn<F32, true, SCH>() : persistent_fn<F32, false, SCH>();
}

const void *pick(int err_dtype, bool fused, bool wide)
{
    return wide ? pick_width<kStripeChannelsWide>(err_dtype, fused) : pick_width<kStripeChannels>(err_dtype, fused);
}

}  // namespace

int persistent_max_blocks_per_cu(int err_dtype, bool fused, bool wide)
{
    int n = 0;
    hipError_t e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, pick(err_dtype, fused, wide), kPersistThreads, 0);
    if (e != hipSuccess) { (void)hipGetLastError(); return 0; }
    return n;
}

hipError_t launch_reset_partials(const BatchView &v, const LaunchRange &r, hipStream_t s)
{
    if (r.p_partial_hi <= r.p_partial_lo) return hipSuccess;
    const uint64_t n_vec = (r.p_partial_hi - r.p_partial_lo) / 16;      // offsets are multiples of 256
    const uint64_t want = (n_vec + 255) / 256;
    hipLaunchKernelGGL(k_reset_partials, dim3((unsigned)(want < 2048 ? want : 2048)), dim3(256), 0, s,
                       reinterpret_cast<u32x4 *>(v.workspace + r.p_partial_lo), n_vec);
    return hipGetLastError();
}

// one_shot: one workgroup per item under an ordinary launch instead of a co-resident grid that loops.
// A workgroup that loops has to drain its stores before its next loads count as returned (the loads and
// stores of a wave share one in-order counter); one that exits leaves the draining to the memory system
// while the next workgroup already loads.  Without co-residency every wait still ends because workgroups
// are started in index order, each XCD taking those of its residue class in order, and under either dealing
// an XCD walks its items in ascending order: take the oldest group with an unfinished item; every older
// group has finished and left, so whatever an XCD still holds from before one of this group's unstarted
// items belongs to this group too, and as long as the XCD's share of `grid` (the co-resident capacity)
// exceeds the group a slot is free and the item starts.  The caller passes one_shot only when an XCD's
// share of `grid` holds a whole group.  Should the assumption ever fail, the bounded wait raises the error flag.
hipError_t launch_single_pass(const BatchView &v, const LaunchRange &r, int err_dtype, bool fused, bool wide, int grid,
                             bool one_shot, hipStream_t s)
{
    if (r.item_hi == r.item_lo) return hipSuccess;
    uint32_t items = r.item_hi - r.item_lo;
    if ((uint32_t)grid > items) grid = (int)items;
    BatchView vv = v;
    LaunchRange rr = r;
    void *args[] = {&vv, &rr};
    if (one_shot) return hipLaunchKernel(pick(err_dtype, fused, wide), dim3(items), dim3(kPersistThreads), args, 0, s);
    return hipLaunchCooperativeKernel(pick(err_dtype, fused, wide), dim3(grid), dim3(kPersistThreads), args, 0, s);
}

}  // namespace cf
