// Low-rank compressor (arxiv 2507.17511, Alg. 3 and App. D "Low-Rank Compression") under the
// residual recursion of Sec. 3.1: A = x_t - recon_{t-1} [tokens, channels] is sent as rank-32 factors
// U = A Q [tokens, 32], V = Q [channels, 32] found by T steps of subspace iteration
//     Q <- orth(Q0);  T x { Z <- A^T (A Q);  Q <- orth(Z) };  U <- A Q,
// and both ends add D = U V^T to the reconstruction; e_t = A - D stays at the sender.
//
// This is the one dense contraction of the codec, so it runs on the matrix cores: every product is a
// chain of v_mfma_f32_32x32x2_f32 (fp32 in, fp32 accumulate; 32 = the rank fills the N side of the
// tile exactly).  A is never materialised: each pass re-forms it from x and recon (4 bytes per element
// in bf16 storage, the same as reading an fp32 A would cost) and is bound by that stream.
//
// Operand layouts are chosen so that every lane feeds the MFMA straight from a 128-bit row-major
// load, with no staging through LDS.  The instruction computes D[m][n] += sum_k A[m][k] B[k][n] with
// lane l holding A[l % 32][l / 32] and B[l / 32][l % 32]: any relabelling of k that both operands share,
// and any relabelling of m or n that the epilogue undoes, is free.
//   project      P = A Q     m = token, k = channel: a lane loads 16 consecutive channels of its token
//                            and spends them on 16 instructions; Q is kept in that per-lane order.
//   backproject  Z = A^T P   m = channel, k = token: a lane loads 8 consecutive channels of its token and
//                            spends them on 8 accumulator tiles (tile j holds channels = j mod 8).
//   encode       D^T = V U^T m = channel (relabelled so that a lane ends up with 16 consecutive channels
//                            of its token), n = token, k = rank.
#include "cf_device.h"
#include "cf_internal.h"

namespace cf {
namespace {

using namespace dev;

typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kRank = 32;
constexpr float kDrop2 = 1e-8f;     // (1e-4)^2: a column left with less than 1e-4 of its length is dropped

__device__ __forceinline__ f32x16 mfma32(float a, float b, f32x16 c) { return __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, c, 0, 0, 0); }

template <int DT> __device__ __forceinline__ void load16(const void *base, int64_t elem, float (&out)[16])
{
    Raw8<DT> lo, hi;
    lo.load(base, elem);
    hi.load(base, elem + 8);
    const F8 a = lo.widen(), b = hi.widen();
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        out[k] = a.v[k];
        out[8 + k] = b.v[k];
    }
}

// 16 consecutive elements of the residual x - recon of one token, or zeros.
template <int DT> __device__ __forceinline__ void residual16(const TensorPtrs &p, int64_t elem, bool valid, float (&z)[16])
{
    if (valid) {
        float x[16], b[16];
        load16<DT>(p.x, elem, x);
        load16<DT>(p.recon, elem, b);
#pragma unroll
        for (int k = 0; k < 16; ++k) z[k] = x[k] - b[k];
    } else {
#pragma unroll
        for (int k = 0; k < 16; ++k) z[k] = 0.0f;
    }
}

__device__ __forceinline__ uint8_t *wire_u(const TensorPtrs &p) { return p.codes; }
__device__ __forceinline__ uint8_t *wire_v(const TensorDev &d, const TensorPtrs &p)
{
    return p.codes + d.n_tokens * kRank * (d.dtype == BF16 ? 2 : 4);
}

// Factors as 4-bit integers (Sec. 3.4 and App. D name INT4 factors; the format is this library's): every
// factor row of 32 entries has one fp32 scale s = absmax / 7 and travels as 32 nibbles q = clamp(rint(f / s),
// -7, 7), two's complement, entry k in byte k / 2, even k in the low nibble -- the 4-bit group quantiser of
// the activations with the rank index in place of the channel.  On the wire: U nibbles [N, 16 bytes],
// V nibbles [C, 16 bytes], U scales [N] fp32, V scales [C] fp32.
__device__ __forceinline__ bool factors_int4(const TensorDev &d) { return d.nm_block == 4u; }
__device__ __forceinline__ uint8_t *wire4_u(const TensorPtrs &p) { return p.codes; }
__device__ __forceinline__ uint8_t *wire4_v(const TensorDev &d, const TensorPtrs &p) { return p.codes + d.n_tokens * 16; }
__device__ __forceinline__ float *wire4_u_scales(const TensorDev &d, const TensorPtrs &p)
{
    return reinterpret_cast<float *>(p.codes + (d.n_tokens + (int64_t)d.n_channels) * 16);
}
__device__ __forceinline__ float *wire4_v_scales(const TensorDev &d, const TensorPtrs &p) { return wire4_u_scales(d, p) + d.n_tokens; }

// One factor row (32 fp32 values) onto the wire.
__device__ __forceinline__ void quantise_factor_row(const float (&f)[kRank], uint8_t *nibbles16, float *scale)
{
    float amax = 0.0f;
#pragma unroll
    for (int k = 0; k < kRank; ++k) amax = fmaxf(amax, fabsf(f[k]));
    const float s = amax / 7.0f;
    u32x4 w;
#pragma unroll
    for (int g = 0; g < 4; ++g) {
        F8 z, sv, dq;
#pragma unroll
        for (int k = 0; k < 8; ++k) { z.v[k] = f[8 * g + k]; sv.v[k] = s; }
        const uint32_t packed = quant8<4>(z, sv, dq);
        if (g == 0) w.x = packed; else if (g == 1) w.y = packed; else if (g == 2) w.z = packed; else w.w = packed;
    }
    *gmut<u32x4>(nibbles16) = w;
    *gmut<float>(scale) = s;
}

// ---------------------------------------------------------------- P = A Q  (and U on the wire)

// A wave owns 64 tokens (two accumulator tiles that share the Q operand), a workgroup of two waves 128, and walks
// the channels 64 at a time.  The MFMA wants a lane to hold one token's channels, memory wants
// neighbouring lanes on neighbouring channels: the wave reads its [64 tokens][64 channels] of x and
// recon row-major (8 lanes = 128 bytes of a bf16 row), leaves the residual in its own LDS patch and
// picks it up again with lane (m, h) on token m (and m + 32), channels 16 * h ... of each 32-channel step.
// Q is read in its per-lane order: step s (32 channels), lane l, 16 floats at ((s * 64 + l) * 16).
constexpr int kProjThreads = 128;                           // two waves: their LDS patches stay under 64 KB at four workgroups per CU
constexpr int kProjTokens = 128;
constexpr int kProjChannels = 64;
constexpr int kProjPitch = kProjChannels + 4;               // floats per token row of the patch

template <int DT>
__device__ __forceinline__ void lr_project_body(const BatchView &v, const TensorDev &d, const TensorPtrs &p, bool wire, float *patch)
{
    const int lane = (int)threadIdx.x & 63, wave = (int)threadIdx.x >> 6;
    const int m = lane & 31, h = lane >> 5;
    const int64_t row_base = (int64_t)blockIdx.x * kProjTokens + wave * 64;
    if (row_base >= d.n_tokens) return;                     // uniform over the wave
    const int64_t C = d.n_channels;
    const CF_GLOBAL f32x4 *qs = gconst<f32x4>(v.workspace + d.lr_q_off);
    f32x16 acc0 = {}, acc1 = {};
    const int steps = d.n_channels / 32;
    const int chunk = lane & 7, trow = lane >> 3;           // row-major side: 8 chunks of 8 channels, 8 tokens per sweep
    // The loads of the next 64 channels are issued as soon as the current ones have gone to the patch,
    // so that they are in flight while the 64 MFMAs of the current ones run.
    Raw8<DT> xr[8], br[8];
    auto fetch = [&](int s0) {
        const int ch = s0 * 32 + chunk * 8;
#pragma unroll
        for (int it = 0; it < 8; ++it) {
            const int64_t tok = row_base + trow + 8 * it;
            if (s0 < steps && tok < d.n_tokens && ch < d.n_channels) {
                xr[it].load(p.x, tok * C + ch);
                br[it].load(p.recon, tok * C + ch);
            } else {
                xr[it].zero();
                br[it].zero();
            }
        }
    };
    fetch(0);
    for (int s0 = 0; s0 < steps; s0 += 2) {
#pragma unroll
        for (int it = 0; it < 8; ++it) {
            const F8 x = xr[it].widen(), b = br[it].widen();
            f32x4 lo, hi;
            lo.x = x.v[0] - b.v[0]; lo.y = x.v[1] - b.v[1]; lo.z = x.v[2] - b.v[2]; lo.w = x.v[3] - b.v[3];
            hi.x = x.v[4] - b.v[4]; hi.y = x.v[5] - b.v[5]; hi.z = x.v[6] - b.v[6]; hi.w = x.v[7] - b.v[7];
            f32x4 *dst = reinterpret_cast<f32x4 *>(patch + (trow + 8 * it) * kProjPitch + chunk * 8);
            dst[0] = lo;
            dst[1] = hi;
        }
        // Q first, then the prefetch: loads return in issue order, so the MFMAs below wait for Q only
        float q[2][16];
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const CF_GLOBAL f32x4 *qp = qs + ((int64_t)(s0 + u < steps ? s0 + u : s0) * 64 + lane) * 4;
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const f32x4 wq = qp[k];
                q[u][4 * k] = wq.x; q[u][4 * k + 1] = wq.y; q[u][4 * k + 2] = wq.z; q[u][4 * k + 3] = wq.w;
            }
        }
        fetch(s0 + 2);
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            if (s0 + u < steps) {                           // uniform over the wave
                float z0[16], z1[16];
                const f32x4 *a0 = reinterpret_cast<const f32x4 *>(patch + m * kProjPitch + 32 * u + 16 * h);
                const f32x4 *a1 = reinterpret_cast<const f32x4 *>(patch + (m + 32) * kProjPitch + 32 * u + 16 * h);
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    const f32x4 w0 = a0[k], w1 = a1[k];
                    z0[4 * k] = w0.x; z0[4 * k + 1] = w0.y; z0[4 * k + 2] = w0.z; z0[4 * k + 3] = w0.w;
                    z1[4 * k] = w1.x; z1[4 * k + 1] = w1.y; z1[4 * k + 2] = w1.z; z1[4 * k + 3] = w1.w;
                }
#pragma unroll
                for (int j = 0; j < 16; ++j) {
                    acc0 = mfma32(z0[j], q[u][j], acc0);
                    acc1 = mfma32(z1[j], q[u][j], acc1);
                }
            }
        }
        __builtin_amdgcn_wave_barrier();
    }
    // accumulator register i of lane (m, h): row 8 * (i / 4) + 4 * h + i % 4 of the tile, column m
    CF_GLOBAL float *P = gmut<float>(v.workspace + d.lr_p_off);
    uint8_t *U = wire_u(p);
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const int row = 8 * (i >> 2) + 4 * h + (i & 3);
#pragma unroll
        for (int half = 0; half < 2; ++half) {
            const int64_t rr = row_base + 32 * half + row;
            const float val = half ? acc1[i] : acc0[i];
            if (rr < d.n_tokens) {
                P[rr * kRank + m] = val;
                if (wire && !factors_int4(d)) {     // 4-bit factors are quantised from P by k_lr_quant_u
                    if (DT == BF16) gmut<uint16_t>(U)[rr * kRank + m] = (uint16_t)bf16_rne(val);
                    else gmut<float>(U)[rr * kRank + m] = val;
                }
            }
        }
    }
}

// min_iters: tensors that asked for fewer subspace iterations than this sit the launch out.
__global__ __launch_bounds__(kProjThreads, 2) void k_lr_project(BatchView v, LaunchRange r, int wire, int min_iters)
{
    __shared__ __attribute__((aligned(16))) float patches[kProjThreads / 64][64 * kProjPitch];
    const int t = r.first + (int)blockIdx.y;
    const TensorDev d = v.descs[t];
    if (d.scale != LOWRANK || d.bits < min_iters) return;
    const TensorPtrs p = v.ptrs[t];
    float *patch = patches[(int)threadIdx.x >> 6];
    if (d.dtype == BF16) lr_project_body<BF16>(v, d, p, wire != 0, patch);
    else lr_project_body<F32>(v, d, p, wire != 0, patch);
}

// ---------------------------------------------------------------- Z = A^T P

// A workgroup owns a stripe of 256 channels; its 4 waves split the tokens and add their tiles up
// through LDS in wave order.  Lane (q, h): channels 8q..8q+7 of the stripe, token 2 * pair + h.
template <int DT>
__device__ __forceinline__ void lr_backproject_body(const BatchView &v, const TensorDev &d, const TensorPtrs &p, float *sum)
{
    const int lane = (int)threadIdx.x & 63, wave = (int)threadIdx.x >> 6;
    const int q = lane & 31, h = lane >> 5;
    const int ch0 = (int)blockIdx.x * 256 + 8 * q;
    const bool cvalid = ch0 < d.n_channels;
    const int64_t C = d.n_channels;
    const int64_t n_pairs = (d.n_tokens + 1) / 2;
    const int64_t per_wave = (n_pairs + 3) / 4;
    const int64_t lo = wave * per_wave;
    const int64_t hi = lo + per_wave < n_pairs ? lo + per_wave : n_pairs;
    const CF_GLOBAL float *P = gconst<float>(v.workspace + d.lr_p_off);
    f32x16 acc[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[j] = (f32x16){};
    constexpr int U = (DT == F32) ? 2 : 4;                  // token pairs per batch (fp32 rows take twice the registers); the next batch is in flight during the MFMAs
    Raw8<DT> xr[U], br[U];
    float pv[U];
    auto fetch = [&](int64_t pair0) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t row = 2 * (pair0 + u) + h;
            const bool rvalid = pair0 + u < hi && row < d.n_tokens;
            if (rvalid && cvalid) {
                xr[u].load(p.x, row * C + ch0);
                br[u].load(p.recon, row * C + ch0);
            } else {
                xr[u].zero();
                br[u].zero();
            }
            pv[u] = rvalid ? P[row * kRank + q] : 0.0f;
        }
    };
    fetch(lo);
    for (int64_t pair0 = lo; pair0 < hi; pair0 += U) {
        float z[U][8], pn[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const F8 x = xr[u].widen(), b = br[u].widen();
#pragma unroll
            for (int j = 0; j < 8; ++j) z[u][j] = x.v[j] - b.v[j];
            pn[u] = pv[u];
        }
        fetch(pair0 + U);
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int j = 0; j < 8; ++j) acc[j] = mfma32(z[u][j], pn[u], acc[j]);
    }
    // tile j, register i of lane (q, h): channel 8 * rho + j of the stripe with rho = 8 * (i / 4) + 4 * h + i % 4, column q
    for (int w = 0; w < 4; ++w) {
        if (wave == w) {
#pragma unroll
            for (int j = 0; j < 8; ++j)
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const int rho = 8 * (i >> 2) + 4 * h + (i & 3);
                    const int idx = (8 * rho + j) * kRank + q;
                    sum[idx] = (w == 0) ? acc[j][i] : sum[idx] + acc[j][i];
                }
        }
        __syncthreads();
    }
    CF_GLOBAL float *Z = gmut<float>(v.workspace + d.lr_z_off);
    for (int k = (int)threadIdx.x; k < 256 * kRank; k += 256) {
        const int ch = (int)blockIdx.x * 256 + k / kRank;
        if (ch < d.n_channels) Z[(int64_t)ch * kRank + (k % kRank)] = sum[k];
    }
}

__global__ __launch_bounds__(256, 2) void k_lr_backproject(BatchView v, LaunchRange r, int min_iters)
{
    __shared__ float sum[256 * kRank];
    const int t = r.first + (int)blockIdx.y;
    const TensorDev d = v.descs[t];
    if (d.scale != LOWRANK || d.bits < min_iters) return;
    if ((int)blockIdx.x * 256 >= d.n_channels) return;      // uniform over the workgroup
    const TensorPtrs p = v.ptrs[t];
    if (d.dtype == BF16) lr_backproject_body<BF16>(v, d, p, sum);
    else lr_backproject_body<F32>(v, d, p, sum);
}

// ---------------------------------------------------------------- Q = orth(Z)

// Gram-Schmidt over the 32 columns, left to right, every column projected twice; one workgroup of
// 1024 lanes per tensor holds the matrix in registers (3 channel rows per lane: C <= 3072).  A column
// left with less than 1e-4 of its length is dropped (zero): a residual of rank < 32 then gives zero
// columns rather than amplified rounding noise.  Writes Q in the per-lane order k_lr_project reads,
// and V = Q on the wire.
constexpr int kOrthThreads = 1024;
constexpr int kOrthRows = 3;

struct OrthShared {
    float part[kOrthThreads / 64][kRank + 1];
    float total[kRank + 1];
};

// Sums `val` over the workgroup into sh.total[slot]; the caller places the barriers.
__device__ __forceinline__ void orth_partial(OrthShared &sh, int slot, float val)
{
    const float w = wave_tree_sum(val);
    if (((int)threadIdx.x & 63) == 0) sh.part[(int)threadIdx.x >> 6][slot] = w;
}

__device__ __forceinline__ void orth_finish(OrthShared &sh, int n_slots)
{
    __syncthreads();
    if ((int)threadIdx.x < n_slots) {
        float s = 0.0f;
#pragma unroll
        for (int w = 0; w < kOrthThreads / 64; ++w) s += sh.part[w][threadIdx.x];
        sh.total[threadIdx.x] = s;
    }
    __syncthreads();
}

// Column K: project it on the finished columns 0..K-1 (twice), then normalise or drop it.  K is a
// template parameter so that every register of the matrix is addressed statically.
template <int K>
__device__ __forceinline__ void orth_column(float (&a)[kOrthRows][kRank], OrthShared &sh)
{
    float start2 = 0.0f;
#pragma unroll
    for (int pass = 0; pass < 2; ++pass) {
        // <q_j, a_K> for every finished column j < K, and (first pass) the column's own length
#pragma unroll
        for (int j = 0; j < K; ++j) {
            float dot = 0.0f;
#pragma unroll
            for (int rr = 0; rr < kOrthRows; ++rr) dot += a[rr][j] * a[rr][K];
            orth_partial(sh, j, dot);
        }
        if (pass == 0) {
            float own = 0.0f;
#pragma unroll
            for (int rr = 0; rr < kOrthRows; ++rr) own += a[rr][K] * a[rr][K];
            orth_partial(sh, K, own);
        }
        orth_finish(sh, pass == 0 ? K + 1 : K);
        if (pass == 0) start2 = sh.total[K];
#pragma unroll
        for (int j = 0; j < K; ++j) {
            const float c = sh.total[j];
#pragma unroll
            for (int rr = 0; rr < kOrthRows; ++rr) a[rr][K] -= c * a[rr][j];
        }
    }
    float own = 0.0f;
#pragma unroll
    for (int rr = 0; rr < kOrthRows; ++rr) own += a[rr][K] * a[rr][K];
    orth_partial(sh, 0, own);
    orth_finish(sh, 1);
    const float left2 = sh.total[0];
    const bool keep = start2 > 0.0f && left2 > kDrop2 * start2;
    const float len = sqrtf(left2);
#pragma unroll
    for (int rr = 0; rr < kOrthRows; ++rr) a[rr][K] = keep ? a[rr][K] / len : 0.0f;
    __syncthreads();                                        // sh.total is rewritten by the next column
}

template <int K>
__device__ __forceinline__ void orth_columns_from(float (&a)[kOrthRows][kRank], OrthShared &sh)
{
    orth_column<K>(a, sh);
    if constexpr (K + 1 < kRank) orth_columns_from<K + 1>(a, sh);
}

__global__ __launch_bounds__(kOrthThreads) void k_lr_orth(BatchView v, LaunchRange r, int from_q0, int min_iters)
{
    __shared__ OrthShared sh;
    const int t = r.first + (int)blockIdx.x;
    const TensorDev d = v.descs[t];
    if (d.scale != LOWRANK || d.bits < min_iters) return;
    const TensorPtrs p = v.ptrs[t];
    const CF_GLOBAL f32x4 *src = from_q0 ? gconst<f32x4>(p.scales) : gconst<f32x4>(v.workspace + d.lr_z_off);
    float a[kOrthRows][kRank];
#pragma unroll
    for (int rr = 0; rr < kOrthRows; ++rr) {
        const int ch = (int)threadIdx.x + kOrthThreads * rr;
#pragma unroll
        for (int k = 0; k < kRank / 4; ++k) {
            f32x4 w = {};
            if (ch < d.n_channels) w = src[(int64_t)ch * (kRank / 4) + k];
            a[rr][4 * k] = w.x; a[rr][4 * k + 1] = w.y; a[rr][4 * k + 2] = w.z; a[rr][4 * k + 3] = w.w;
        }
    }
    orth_columns_from<0>(a, sh);
    CF_GLOBAL float *qs = gmut<float>(v.workspace + d.lr_q_off);
    uint8_t *V = wire_v(d, p);
#pragma unroll
    for (int rr = 0; rr < kOrthRows; ++rr) {
        const int ch = (int)threadIdx.x + kOrthThreads * rr;
        if (ch >= d.n_channels) continue;
        const int s = ch >> 5, c = ch & 31, hh = c >> 4, j = c & 15;
#pragma unroll
        for (int n = 0; n < kRank; ++n) {
            qs[((int64_t)s * 64 + hh * 32 + n) * 16 + j] = a[rr][n];
            if (factors_int4(d)) continue;
            if (d.dtype == BF16) gmut<uint16_t>(V)[(int64_t)ch * kRank + n] = (uint16_t)bf16_rne(a[rr][n]);
            else gmut<float>(V)[(int64_t)ch * kRank + n] = a[rr][n];
        }
        if (factors_int4(d)) quantise_factor_row(a[rr], wire4_v(d, p) + (int64_t)ch * 16, wire4_v_scales(d, p) + ch);
    }
}

// 4-bit factors: U = P (fp32, in the workspace) onto the wire, one lane per token.
__global__ __launch_bounds__(256) void k_lr_quant_u(BatchView v, LaunchRange r)
{
    const int t = r.first + (int)blockIdx.y;
    const TensorDev d = v.descs[t];
    if (d.scale != LOWRANK || !factors_int4(d)) return;
    const TensorPtrs p = v.ptrs[t];
    const int64_t row = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (row >= d.n_tokens) return;
    const CF_GLOBAL f32x4 *src = gconst<f32x4>(v.workspace + d.lr_p_off) + row * (kRank / 4);
    float f[kRank];
#pragma unroll
    for (int k = 0; k < kRank / 4; ++k) {
        const f32x4 w = src[k];
        f[4 * k] = w.x; f[4 * k + 1] = w.y; f[4 * k + 2] = w.z; f[4 * k + 3] = w.w;
    }
    quantise_factor_row(f, wire4_u(p) + row * 16, wire4_u_scales(d, p) + row);
}

// ---------------------------------------------------------------- D = U V^T, error and reconstruction

// 16 consecutive rank entries (16 * h ...) of one row of a factor on the wire, widened.
// int4: `base` holds rows of 16 nibble bytes and `scales` one fp32 per row.
template <int DT> __device__ __forceinline__ void factor16(const uint8_t *base, const float *scales, bool int4, int64_t row, int h,
                                                           bool valid, float (&out)[16])
{
    const int64_t r0 = valid ? row : 0;                             // row 0 always exists; its values are discarded
    if (int4) {                                                     // uniform over the launch's tensor
        const u32x2 w = *gconst<u32x2>(base + r0 * 16 + 8 * h);
        const float s = *gconst<float>(scales + r0);
        F8 sv, lo, hi;
#pragma unroll
        for (int k = 0; k < 8; ++k) sv.v[k] = s;
        dequant8<4>(w.x, sv, lo);
        dequant8<4>(w.y, sv, hi);
#pragma unroll
        for (int k = 0; k < 8; ++k) { out[k] = lo.v[k]; out[8 + k] = hi.v[k]; }
    } else {
        load16<DT>(base, r0 * kRank + 16 * h, out);
    }
#pragma unroll
    for (int k = 0; k < 16; ++k) out[k] = valid ? out[k] : 0.0f;
}

// A wave owns 32 tokens and kApplySpan channels, which it walks in tiles of 64 (a workgroup that
// looped over all channels would have to drain its stores before each tile's loads count as returned).  The MFMA leaves lane (n, h) with
// channel n of 16 tokens, which is the wrong way round for row-major memory, so the tile of D goes
// through the wave's own LDS patch [32 tokens][64 channels] and comes back as 8 consecutive channels
// of one token per lane: 8 lanes then cover 128 bytes of a bf16 row (256 of the fp32 error row).
// SENDER: also forms A again and writes e = A - D.  UPDATE: writes recon + D.
constexpr int kApplyChannels = 64;
#ifndef CF_APPLY_SPAN
#define CF_APPLY_SPAN 128
#endif
constexpr int kApplySpan = CF_APPLY_SPAN;                   // channels per workgroup
constexpr int kApplyPitch = kApplyChannels + 4;             // floats per token row of the patch

template <int DT, int ET, bool SENDER, bool UPDATE>
__device__ __forceinline__ void lr_apply_body(const TensorDev &d, const TensorPtrs &p, float *patch, float *epatch)
{
    const int lane = (int)threadIdx.x & 63, wave = (int)threadIdx.x >> 6;
    const int n = lane & 31, h = lane >> 5;
    const int n_spans = (d.n_channels + kApplySpan - 1) / kApplySpan;
    const int span = (int)(blockIdx.x % (unsigned)n_spans);
    const int64_t tok_base = (int64_t)(blockIdx.x / (unsigned)n_spans) * 128 + wave * 32;
    if (tok_base >= d.n_tokens) return;                     // uniform over the wave
    const int64_t C = d.n_channels;
    float u[16];
    const bool int4 = factors_int4(d);
    factor16<DT>(int4 ? wire4_u(p) : wire_u(p), wire4_u_scales(d, p), int4, tok_base + n, h, tok_base + n < d.n_tokens, u);
    const uint8_t *V = int4 ? wire4_v(d, p) : wire_v(d, p);
    const float *Vs = wire4_v_scales(d, p);
    const int sub_lo = span * (kApplySpan / 32);
    const int n_sub = d.n_channels / 32 < sub_lo + kApplySpan / 32 ? d.n_channels / 32 : sub_lo + kApplySpan / 32;
    const int chunk = lane & 7, trow = lane >> 3;           // row-major side: 8 chunks of 8 channels, 8 tokens per sweep
    for (int sub0 = sub_lo; sub0 < n_sub; sub0 += 2) {
        const int cnt = n_sub - sub0 < 2 ? 1 : 2;
        // Issue order matters because loads return in order: first the V rows the MFMAs need, then the
        // tile's x and recon, which are only needed once D has come back through the patch.
        float vv[2][16];
#pragma unroll
        for (int c = 0; c < 2; ++c) factor16<DT>(V, Vs, int4, (int64_t)(sub0 + (c < cnt ? c : 0)) * 32 + n, h, true, vv[c]);
        Raw8<DT> xr[4], br[4];
        bool live[4];
#pragma unroll
        for (int it = 0; it < 4; ++it) {
            const int64_t tok = tok_base + trow + 8 * it;
            live[it] = tok < d.n_tokens && chunk * 8 < cnt * 32;
            const int64_t e0 = tok * C + (int64_t)sub0 * 32 + chunk * 8;
            if (live[it]) {
                if (UPDATE) br[it].load_stream(p.recon, e0);        // written back below: the streaming hint pays
                else br[it].load(p.recon, e0);
                if (SENDER) xr[it].load(p.x, e0); else xr[it].zero();
            } else {
                br[it].zero();
                xr[it].zero();
            }
        }
#pragma unroll
        for (int c = 0; c < 2; ++c) {
            if (c < cnt) {                                  // uniform over the wave
                f32x16 acc = {};
#pragma unroll
                for (int j = 0; j < 16; ++j) acc = mfma32(u[j], vv[c][j], acc);
#pragma unroll
                for (int i = 0; i < 16; ++i) patch[(8 * (i >> 2) + 4 * h + (i & 3)) * kApplyPitch + c * 32 + n] = acc[i];
            }
        }
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int it = 0; it < 4; ++it) {
            const int tl = trow + 8 * it;
            const int64_t tok = tok_base + tl;
            // every lane goes through the exchange of the error row (dead lanes carry values nobody stores)
            const f32x4 *src = reinterpret_cast<const f32x4 *>(patch + tl * kApplyPitch + chunk * 8);
            const f32x4 d0 = src[0], d1 = src[1];
            F8 D;
            D.v[0] = d0.x; D.v[1] = d0.y; D.v[2] = d0.z; D.v[3] = d0.w;
            D.v[4] = d1.x; D.v[5] = d1.y; D.v[6] = d1.z; D.v[7] = d1.w;
            const int64_t e0 = tok * C + (int64_t)sub0 * 32 + chunk * 8;
            const F8 b = br[it].widen();
            if (SENDER) {
                const F8 x = xr[it].widen();
                F8 lost;
#pragma unroll
                for (int k = 0; k < 8; ++k) {
                    const float z = x.v[k] - b.v[k];
                    lost.v[k] = z - D.v[k];
                }
                if (ET == F32) {        // the 8 lanes of a token row send its 256 bytes as two whole lines
                    f32x4 pieces[2];
                    lines_exchange<8>(epatch, lane, lost, pieces);
                    if (tok < d.n_tokens)
                        lines_store_stream<8>(static_cast<float *>(p.err) + tok * C + (int64_t)sub0 * 32, chunk, cnt * 4, pieces);
                } else if (live[it]) {
                    Raw8<ET> eo;
                    eo.narrow(lost);
                    eo.store_stream(p.err, e0);
                }
            }
            if (UPDATE && live[it]) {
                F8 nb;
#pragma unroll
                for (int k = 0; k < 8; ++k) nb.v[k] = b.v[k] + D.v[k];
                Raw8<DT> out;
                out.narrow(nb);
                if (DT == BF16) out.store_stream(p.recon, e0); else out.store(p.recon, e0);
            }
        }
        __builtin_amdgcn_wave_barrier();
    }
}

template <int ET, bool SENDER, bool UPDATE>
__global__ __launch_bounds__(256) void k_lr_apply(BatchView v, LaunchRange r)
{
    __shared__ __attribute__((aligned(16))) float patches[4][32 * kApplyPitch];
    const int t = r.first + (int)blockIdx.y;
    const TensorDev d = v.descs[t];
    if (d.scale != LOWRANK) return;
    const TensorPtrs p = v.ptrs[t];
    __shared__ __attribute__((aligned(16))) float epatches[4][512];       // the error rows' way to whole lines (2 KB per wave)
    float *patch = patches[(int)threadIdx.x >> 6];
    float *epatch = epatches[(int)threadIdx.x >> 6];
    if (d.dtype == BF16) lr_apply_body<BF16, ET, SENDER, UPDATE>(d, p, patch, epatch);
    else lr_apply_body<F32, ET, SENDER, UPDATE>(d, p, patch, epatch);
}

}  // namespace

hipError_t launch_lr_orth(const BatchView &v, const LaunchRange &r, bool from_q0, int min_iters, hipStream_t s)
{
    if (r.count == 0) return hipSuccess;
    hipLaunchKernelGGL(k_lr_orth, dim3(r.count), dim3(kOrthThreads), 0, s, v, r, from_q0 ? 1 : 0, min_iters);
    return hipGetLastError();
}

hipError_t launch_lr_project(const BatchView &v, const LaunchRange &r, bool wire, int min_iters, hipStream_t s)
{
    if (r.count == 0 || r.lr_max_tokens == 0) return hipSuccess;
    dim3 grid((unsigned)((r.lr_max_tokens + kProjTokens - 1) / kProjTokens), (unsigned)r.count);
    hipLaunchKernelGGL(k_lr_project, grid, dim3(kProjThreads), 0, s, v, r, wire ? 1 : 0, min_iters);
    return hipGetLastError();
}

hipError_t launch_lr_backproject(const BatchView &v, const LaunchRange &r, int min_iters, hipStream_t s)
{
    if (r.count == 0 || r.lr_max_channels == 0) return hipSuccess;
    dim3 grid((unsigned)((r.lr_max_channels + 255) / 256), (unsigned)r.count);
    hipLaunchKernelGGL(k_lr_backproject, grid, dim3(256), 0, s, v, r, min_iters);
    return hipGetLastError();
}

// Blocks of 128 tokens x kApplySpan channels, for the largest low-rank tensor of the range; a tensor with
// fewer channel spans sees block indices beyond its own and returns at once (tok_base >= n_tokens).
static unsigned apply_blocks(const LaunchRange &r)
{
    return (unsigned)((r.lr_max_tokens + 127) / 128) * (unsigned)((r.lr_max_channels + kApplySpan - 1) / kApplySpan);
}

hipError_t launch_lr_quant_u(const BatchView &v, const LaunchRange &r, hipStream_t s)
{
    if (r.count == 0 || r.lr_max_tokens == 0) return hipSuccess;
    dim3 grid((unsigned)((r.lr_max_tokens + 255) / 256), (unsigned)r.count);
    hipLaunchKernelGGL(k_lr_quant_u, grid, dim3(256), 0, s, v, r);
    return hipGetLastError();
}

hipError_t launch_lr_encode(const BatchView &v, const LaunchRange &r, int err_dtype, bool fused, hipStream_t s)
{
    if (r.count == 0 || r.lr_max_tokens == 0) return hipSuccess;
    dim3 grid(apply_blocks(r), (unsigned)r.count), block(256);
    if (err_dtype == BF16) {
        if (fused) hipLaunchKernelGGL((k_lr_apply<BF16, true, true>), grid, block, 0, s, v, r);
        else hipLaunchKernelGGL((k_lr_apply<BF16, true, false>), grid, block, 0, s, v, r);
    } else {
        if (fused) hipLaunchKernelGGL((k_lr_apply<F32, true, true>), grid, block, 0, s, v, r);
        else hipLaunchKernelGGL((k_lr_apply<F32, true, false>), grid, block, 0, s, v, r);
    }
    return hipGetLastError();
}

hipError_t launch_lr_decode(const BatchView &v, const LaunchRange &r, hipStream_t s)
{
    if (r.count == 0 || r.lr_max_tokens == 0) return hipSuccess;
    dim3 grid(apply_blocks(r), (unsigned)r.count);
    hipLaunchKernelGGL((k_lr_apply<F32, false, true>), grid, dim3(256), 0, s, v, r);
    return hipGetLastError();
}

}  // namespace cf
