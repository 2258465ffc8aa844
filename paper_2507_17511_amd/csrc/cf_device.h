// Device-side building blocks shared by the codec kernels: element formats,
// the residual (a1, a2), code selection / packing / decode (a4-a6) and a 16-lane
// DPP maximum.  All value arithmetic is fp32 with one rounding per operation
// (translation units including this are compiled with -ffp-contract=off).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace cf {
namespace dev {

constexpr int F32 = 0, BF16 = 1;
constexpr int SCALE_CHANNEL = 0, SCALE_GROUP = 1;
constexpr int EF_RECON = 0, EF_LITERAL = 1, EF_OFF = 2;

// ---------------------------------------------------------------- element formats

__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

// fp32 -> bf16, round to nearest, ties to even, on the 16 dropped bits.
__device__ __forceinline__ uint32_t bf16_rne(float f)
{
    uint32_t u = __float_as_uint(f);
    u += 0x7fffu + ((u >> 16) & 1u);
    return u >> 16;
}

struct F8 {
    float v[8];
};

// Raw 8-element vectors as they sit in memory.
template <int DT> struct Raw8;
template <> struct Raw8<BF16> {
    uint4 w;
    __device__ __forceinline__ void zero() { w = make_uint4(0, 0, 0, 0); }
    // Makes the registers opaque to the optimiser: values derived from them earlier are not reused.
    __device__ __forceinline__ void opaque() { asm volatile("" : "+v"(w.x), "+v"(w.y), "+v"(w.z), "+v"(w.w)); }
    __device__ __forceinline__ void load(const void *base, int64_t elem) { w = *reinterpret_cast<const uint4 *>(static_cast<const uint16_t *>(base) + elem); }
    __device__ __forceinline__ void store(void *base, int64_t elem) const { *reinterpret_cast<uint4 *>(static_cast<uint16_t *>(base) + elem) = w; }
    __device__ __forceinline__ F8 widen() const
    {
        F8 f;
        f.v[0] = bf16_lo(w.x); f.v[1] = bf16_hi(w.x);
        f.v[2] = bf16_lo(w.y); f.v[3] = bf16_hi(w.y);
        f.v[4] = bf16_lo(w.z); f.v[5] = bf16_hi(w.z);
        f.v[6] = bf16_lo(w.w); f.v[7] = bf16_hi(w.w);
        return f;
    }
    __device__ __forceinline__ void narrow(const F8 &f)
    {
        w.x = bf16_rne(f.v[0]) | (bf16_rne(f.v[1]) << 16);
        w.y = bf16_rne(f.v[2]) | (bf16_rne(f.v[3]) << 16);
        w.z = bf16_rne(f.v[4]) | (bf16_rne(f.v[5]) << 16);
        w.w = bf16_rne(f.v[6]) | (bf16_rne(f.v[7]) << 16);
    }
};
template <> struct Raw8<F32> {
    float4 a, b;
    __device__ __forceinline__ void zero() { a = make_float4(0, 0, 0, 0); b = a; }
    __device__ __forceinline__ void opaque()
    {
        asm volatile("" : "+v"(a.x), "+v"(a.y), "+v"(a.z), "+v"(a.w));
        asm volatile("" : "+v"(b.x), "+v"(b.y), "+v"(b.z), "+v"(b.w));
    }
    __device__ __forceinline__ void load(const void *base, int64_t elem)
    {
        const float4 *p = reinterpret_cast<const float4 *>(static_cast<const float *>(base) + elem);
        a = p[0];
        b = p[1];
    }
    __device__ __forceinline__ void store(void *base, int64_t elem) const
    {
        float4 *p = reinterpret_cast<float4 *>(static_cast<float *>(base) + elem);
        p[0] = a;
        p[1] = b;
    }
    __device__ __forceinline__ F8 widen() const
    {
        F8 f;
        f.v[0] = a.x; f.v[1] = a.y; f.v[2] = a.z; f.v[3] = a.w;
        f.v[4] = b.x; f.v[5] = b.y; f.v[6] = b.z; f.v[7] = b.w;
        return f;
    }
    __device__ __forceinline__ void narrow(const F8 &f)
    {
        a = make_float4(f.v[0], f.v[1], f.v[2], f.v[3]);
        b = make_float4(f.v[4], f.v[5], f.v[6], f.v[7]);
    }
};

// ---------------------------------------------------------------- a1 + a2

// z from the raw operands; the order of the two fp32 operations is fixed.
template <int EF>
__device__ __forceinline__ F8 residual8(const F8 &x, const F8 &b, const F8 &e)
{
    F8 z;
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        float r = x.v[k] - b.v[k];
        if (EF == EF_LITERAL) r = r + e.v[k];
        if (EF == EF_OFF) r = r - e.v[k];
        z.v[k] = r;
    }
    return z;
}

// ---------------------------------------------------------------- a4 + a5 + a6

// Codes of 8 consecutive channels, packed least significant first, and their
// decoded values.  BITS == 4 divides (IEEE) and rounds half to even.
template <int BITS>
__device__ __forceinline__ uint32_t quant8(const F8 &z, const F8 &s, F8 &d)
{
    uint32_t packed = 0;
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        float v = z.v[k], sc = s.v[k];
        if (BITS == 1) {
            bool neg = v < 0.0f;
            packed |= (neg ? 1u : 0u) << k;
            d.v[k] = neg ? -sc : sc;
        } else if (BITS == 2) {
            bool neg = v < 0.0f;
            bool big = fabsf(v) > 1.25f * sc;
            packed |= ((neg ? 2u : 0u) | (big ? 1u : 0u)) << (2 * k);
            float m = big ? 2.0f * sc : 0.5f * sc;
            d.v[k] = neg ? -m : m;
        } else {
            float t = v / sc;
            float r = rintf(t);
            r = fminf(fmaxf(r, -7.0f), 7.0f);
            int q = (sc != 0.0f) ? (int)r : 0;
            packed |= ((uint32_t)q & 0xFu) << (4 * k);
            d.v[k] = (float)q * sc;
        }
    }
    return packed;
}

template <int BITS>
__device__ __forceinline__ void dequant8(uint32_t packed, const F8 &s, F8 &d)
{
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        float sc = s.v[k];
        if (BITS == 1) {
            d.v[k] = ((packed >> k) & 1u) ? -sc : sc;
        } else if (BITS == 2) {
            uint32_t c = (packed >> (2 * k)) & 3u;
            float m = (c & 1u) ? 2.0f * sc : 0.5f * sc;
            d.v[k] = (c & 2u) ? -m : m;
        } else {
            int q = ((int)(packed << (28 - 4 * k))) >> 28;      // sign-extended nibble
            d.v[k] = (float)q * sc;
        }
    }
}

template <int BITS> __device__ __forceinline__ void store_codes(uint8_t *row, int chunk, uint32_t packed)
{
    if (BITS == 1) row[chunk] = (uint8_t)packed;
    else if (BITS == 2) reinterpret_cast<uint16_t *>(row)[chunk] = (uint16_t)packed;
    else reinterpret_cast<uint32_t *>(row)[chunk] = packed;
}

template <int BITS> __device__ __forceinline__ uint32_t load_codes(const uint8_t *row, int chunk)
{
    if (BITS == 1) return row[chunk];
    if (BITS == 2) return reinterpret_cast<const uint16_t *>(row)[chunk];
    return reinterpret_cast<const uint32_t *>(row)[chunk];
}

// Max over the 16 lanes of a DPP row (16 lanes x 8 channels = one group of 128).
// All 64 lanes must be active.
__device__ __forceinline__ float row16_max(float m)
{
    int v;
    v = __builtin_amdgcn_update_dpp(0, __float_as_int(m), 0xB1, 0xF, 0xF, false);   // quad_perm [1,0,3,2]
    m = fmaxf(m, __int_as_float(v));
    v = __builtin_amdgcn_update_dpp(0, __float_as_int(m), 0x4E, 0xF, 0xF, false);   // quad_perm [2,3,0,1]
    m = fmaxf(m, __int_as_float(v));
    v = __builtin_amdgcn_update_dpp(0, __float_as_int(m), 0x141, 0xF, 0xF, false);  // row_half_mirror
    m = fmaxf(m, __int_as_float(v));
    v = __builtin_amdgcn_update_dpp(0, __float_as_int(m), 0x140, 0xF, 0xF, false);  // row_mirror
    m = fmaxf(m, __int_as_float(v));
    return m;
}


// Largest t in [lo, hi) with prefix[t] <= id.
__device__ __forceinline__ int find_slot(const uint32_t *prefix, int lo, int hi, uint32_t id)
{
    while (hi - lo > 1) {
        int mid = (lo + hi) >> 1;
        if (prefix[mid] <= id) lo = mid; else hi = mid;
    }
    return lo;
}

}  // namespace dev
}  // namespace cf
