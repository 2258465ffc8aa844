// Device-side building blocks shared by the codec kernels: element formats,
// the residual (a1, a2), code selection / packing / decode (a4-a6) and a 16-lane
// DPP maximum.  All value arithmetic is fp32 with one rounding per operation
// (translation units including this are compiled with -ffp-contract=off).
//
// Memory access goes through global-address-space pointers to native vector
// types, so that every load and store is a global_* instruction of 128 bits.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace cf {
namespace dev {

constexpr int F32 = 0, BF16 = 1;
constexpr int SCALE_CHANNEL = 0, SCALE_GROUP = 1, SCALE_RANK1 = 2, SPARSE_NM = 3, LOWRANK = 4;
constexpr int EF_RECON = 0, EF_LITERAL = 1, EF_OFF = 2, EF_NAIVE = 3;

#define CF_GLOBAL __attribute__((address_space(1)))

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

template <typename T> __device__ __forceinline__ const CF_GLOBAL T *gconst(const void *p) { return (const CF_GLOBAL T *)p; }
template <typename T> __device__ __forceinline__ CF_GLOBAL T *gmut(void *p) { return (CF_GLOBAL T *)p; }

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

// Raw 8-element vectors as they sit in memory.  `elem` is an element index from
// `base`.  load_stream / store_stream mark data that is touched once (they map
// to the non-temporal forms).
template <int DT> struct Raw8;
template <> struct Raw8<BF16> {
    u32x4 w;
    __device__ __forceinline__ void zero() { w = (u32x4)(0u); }
    __device__ __forceinline__ void load(const void *base, int64_t elem) { w = *gconst<u32x4>(static_cast<const uint16_t *>(base) + elem); }
    __device__ __forceinline__ void load_stream(const void *base, int64_t elem) { w = __builtin_nontemporal_load(gconst<u32x4>(static_cast<const uint16_t *>(base) + elem)); }
    __device__ __forceinline__ void store(void *base, int64_t elem) const { *gmut<u32x4>(static_cast<uint16_t *>(base) + elem) = w; }
    __device__ __forceinline__ void store_stream(void *base, int64_t elem) const { __builtin_nontemporal_store(w, gmut<u32x4>(static_cast<uint16_t *>(base) + elem)); }
    // Uniform base pointer plus a 32-bit per-lane byte offset: the scalar-base form of the global
    // instructions, which needs no 64-bit address arithmetic in vector registers.
    __device__ __forceinline__ void load_at(const void *ubase, uint32_t off) { w = *gconst<u32x4>(static_cast<const char *>(ubase) + off); }
    __device__ __forceinline__ void store_at(void *ubase, uint32_t off) const { *gmut<u32x4>(static_cast<char *>(ubase) + off) = w; }
    // Makes the registers opaque to the optimiser: values derived from them earlier are not reused.
    __device__ __forceinline__ void opaque() { asm volatile("" : "+v"(w)); }
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
    f32x4 a, b;
    __device__ __forceinline__ void zero() { a = (f32x4)(0.0f); b = a; }
    __device__ __forceinline__ void load(const void *base, int64_t elem)
    {
        const CF_GLOBAL f32x4 *p = gconst<f32x4>(static_cast<const float *>(base) + elem);
        a = p[0];
        b = p[1];
    }
    __device__ __forceinline__ void load_stream(const void *base, int64_t elem)
    {
        const CF_GLOBAL f32x4 *p = gconst<f32x4>(static_cast<const float *>(base) + elem);
        a = __builtin_nontemporal_load(p);
        b = __builtin_nontemporal_load(p + 1);
    }
    __device__ __forceinline__ void store(void *base, int64_t elem) const
    {
        CF_GLOBAL f32x4 *p = gmut<f32x4>(static_cast<float *>(base) + elem);
        p[0] = a;
        p[1] = b;
    }
    __device__ __forceinline__ void store_stream(void *base, int64_t elem) const
    {
        CF_GLOBAL f32x4 *p = gmut<f32x4>(static_cast<float *>(base) + elem);
        __builtin_nontemporal_store(a, p);
        __builtin_nontemporal_store(b, p + 1);
    }
    __device__ __forceinline__ void load_at(const void *ubase, uint32_t off)
    {
        const CF_GLOBAL f32x4 *p = gconst<f32x4>(static_cast<const char *>(ubase) + off);
        a = p[0];
        b = p[1];
    }
    __device__ __forceinline__ void store_at(void *ubase, uint32_t off) const
    {
        CF_GLOBAL f32x4 *p = gmut<f32x4>(static_cast<char *>(ubase) + off);
        p[0] = a;
        p[1] = b;
    }
    __device__ __forceinline__ void opaque()
    {
        asm volatile("" : "+v"(a));
        asm volatile("" : "+v"(b));
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
        a.x = f.v[0]; a.y = f.v[1]; a.z = f.v[2]; a.w = f.v[3];
        b.x = f.v[4]; b.y = f.v[5]; b.z = f.v[6]; b.w = f.v[7];
    }
};

// ---------------------------------------------------------------- fp32 rows to memory as whole lines

// A lane's 8 fp32 values are 32 bytes, so a plain pair of 128-bit stores half-fills every 64-byte
// request, and a streaming store (which nothing merges on the way) would reach memory in pieces.
// Instead the lanes of a wave pass their values through a wave-private LDS patch (2 KB: the image
// of what the wave writes) and take them back so that store h of a run covers bytes
// [h * 16 * RUN, (h + 1) * 16 * RUN) of it: whole 128-byte lines per instruction.  RUN = lanes
// whose outputs are contiguous in memory (a divisor of 64).  Lane j of a run then holds pieces
// j and RUN + j (16 bytes each) of the run's 2 * RUN pieces; piece q belongs to channel chunk q / 2.
__device__ __forceinline__ void wave_lds_fence()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

template <int RUN>
__device__ __forceinline__ void lines_exchange(float *patch, int lane, const F8 &v, f32x4 (&out)[2])
{
    f32x4 *img = reinterpret_cast<f32x4 *>(patch);
    f32x4 lo, hi;
    lo.x = v.v[0]; lo.y = v.v[1]; lo.z = v.v[2]; lo.w = v.v[3];
    hi.x = v.v[4]; hi.y = v.v[5]; hi.z = v.v[6]; hi.w = v.v[7];
    img[2 * lane] = lo;
    img[2 * lane + 1] = hi;
    wave_lds_fence();
    const int first = (lane / RUN) * 2 * RUN, j = lane % RUN;
    out[0] = img[first + j];
    out[1] = img[first + RUN + j];
    wave_lds_fence();                   // the next exchange overwrites the patch
}

// `run` points at the first byte of the run in memory; n_valid = channel chunks of the run that exist.
template <int RUN>
__device__ __forceinline__ void lines_store_stream(void *run, int j, int n_valid, const f32x4 (&pieces)[2])
{
    CF_GLOBAL f32x4 *dst = gmut<f32x4>(run);
    if ((j >> 1) < n_valid) __builtin_nontemporal_store(pieces[0], dst + j);
    if (((RUN + j) >> 1) < n_valid) __builtin_nontemporal_store(pieces[1], dst + RUN + j);
}

// ---------------------------------------------------------------- a1 + a2

// z from the raw operands; the order of the two fp32 operations is fixed.
template <int EF>
__device__ __forceinline__ F8 residual8(const F8 &x, const F8 &b, const F8 &e)
{
    F8 z;
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        float r = (EF == EF_NAIVE) ? x.v[k] : x.v[k] - b.v[k];     // naive: the activation itself (Sec. 3.1)
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

// `row` points at the first code byte of the token; a lane owns `BITS` bytes of it.
template <int BITS> __device__ __forceinline__ void store_codes(uint8_t *row, int chunk, uint32_t packed)
{
    if (BITS == 1) gmut<uint8_t>(row)[chunk] = (uint8_t)packed;
    else if (BITS == 2) gmut<uint16_t>(row)[chunk] = (uint16_t)packed;
    else gmut<uint32_t>(row)[chunk] = packed;
}

// The same, with the code bytes of neighbouring lanes gathered into one dword
// first (sub-dword stores are slow): 1-bit, the four lanes of a quad; 2-bit,
// two lanes.  `wide` (uniform over the wave) says that rows are a multiple of
// four bytes long and that a tensor's lanes come in whole quads; all lanes of a
// quad must be active.
// `mine` is the address of the lane's own BITS code bytes; `chunk` its chunk index in the row.
template <int BITS> __device__ __forceinline__ void store_codes_ptr(uint8_t *mine, int chunk, uint32_t packed, bool wide)
{
    if (BITS == 4) {
        *gmut<uint32_t>(mine) = packed;
        return;
    }
    if (!wide) {
        if (BITS == 1) *gmut<uint8_t>(mine) = (uint8_t)packed;
        else *gmut<uint16_t>(mine) = (uint16_t)packed;
        return;
    }
    const int me = (int)packed;
    if (BITS == 1) {
        const uint32_t b1 = (uint32_t)__builtin_amdgcn_update_dpp(0, me, 0x55, 0xF, 0xF, false);   // quad_perm [1,1,1,1]
        const uint32_t b2 = (uint32_t)__builtin_amdgcn_update_dpp(0, me, 0xAA, 0xF, 0xF, false);   // quad_perm [2,2,2,2]
        const uint32_t b3 = (uint32_t)__builtin_amdgcn_update_dpp(0, me, 0xFF, 0xF, 0xF, false);   // quad_perm [3,3,3,3]
        const uint32_t w = (packed & 0xFFu) | ((b1 & 0xFFu) << 8) | ((b2 & 0xFFu) << 16) | (b3 << 24);
        if ((chunk & 3) == 0) *gmut<uint32_t>(mine) = w;
    } else {
        const uint32_t h1 = (uint32_t)__builtin_amdgcn_update_dpp(0, me, 0xF5, 0xF, 0xF, false);   // quad_perm [1,1,3,3]
        const uint32_t w = (packed & 0xFFFFu) | (h1 << 16);
        if ((chunk & 1) == 0) *gmut<uint32_t>(mine) = w;
    }
}

template <int BITS> __device__ __forceinline__ void store_codes_wide(uint8_t *row, int chunk, uint32_t packed, bool wide)
{
    store_codes_ptr<BITS>(row + chunk * BITS, chunk, packed, wide);
}

template <int BITS> __device__ __forceinline__ uint32_t load_codes(const uint8_t *row, int chunk)
{
    if (BITS == 1) return gconst<uint8_t>(row)[chunk];
    if (BITS == 2) return gconst<uint16_t>(row)[chunk];
    return gconst<uint32_t>(row)[chunk];
}

__device__ __forceinline__ F8 load_scales8(const float *scales, int64_t first)
{
    Raw8<F32> r;
    r.load(scales, first);
    return r.widen();
}

// ---------------------------------------------------------------- N:M block sparsifier, M = 8

// Sec. 3.4 names an N:M block sparsifier; here a block is the 8 channels of one lane.  Returns
// the mask of the KEEP elements of largest magnitude (bit k = channel k).  Magnitudes are ordered
// by the bit pattern of |z|, equal ones by channel: element k is kept iff fewer than KEEP elements
// come before it.  28 comparisons, no cross-lane traffic.
// PAIR: the block is 16 channels, this lane's 8 and those of the lane next to it (lane ^ 1; the even lane
// holds the lower channels); both lanes must be active.  The neighbour's magnitudes come over DPP.
template <int KEEP, bool PAIR = false> __device__ __forceinline__ uint32_t nm_select8(const F8 &z)
{
    uint32_t key[8];
    int before[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        key[k] = __float_as_uint(z.v[k]) & 0x7fffffffu;
        before[k] = 0;
    }
#pragma unroll
    for (int j = 0; j < 8; ++j)
#pragma unroll
        for (int k = j + 1; k < 8; ++k) {
            const bool j_first = key[j] >= key[k];      // j < k: a tie goes to j
            before[k] += j_first ? 1 : 0;
            before[j] += j_first ? 0 : 1;
        }
    if (PAIR) {
        // Only a lane's own first KEEP can be among the block's first KEEP, and an element that some other
        // element of the neighbour precedes is preceded by all of the neighbour's first KEEP too (or is out
        // anyway), so the lanes exchange their first KEEP magnitudes only.  The receiver counts `theirs > mine`:
        // the even lane's channels win ties, so it sends magnitude + 1 (at most 0x80000000, no wrap); a zero
        // stands for "nothing" and precedes no one.
        const uint32_t bias = (threadIdx.x & 1u) ? 0u : 1u;
        int extra[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) extra[k] = 0;
        if (KEEP <= 2) {
            uint32_t first[KEEP];
#pragma unroll
            for (int q = 0; q < KEEP; ++q) first[q] = 0u;
#pragma unroll
            for (int k = 0; k < 8; ++k)
#pragma unroll
                for (int q = 0; q < KEEP; ++q) first[q] = before[k] == q ? key[k] + bias : first[q];
#pragma unroll
            for (int q = 0; q < KEEP; ++q) {
                const uint32_t theirs = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)first[q], 0xB1, 0xF, 0xF, false);   // quad_perm [1,0,3,2]
#pragma unroll
                for (int k = 0; k < 8; ++k) extra[k] += theirs > key[k] ? 1 : 0;
            }
        } else {
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const uint32_t send = before[j] < KEEP ? key[j] + bias : 0u;
                const uint32_t theirs = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)send, 0xB1, 0xF, 0xF, false);
#pragma unroll
                for (int k = 0; k < 8; ++k) extra[k] += theirs > key[k] ? 1 : 0;
            }
        }
#pragma unroll
        for (int k = 0; k < 8; ++k) before[k] += extra[k];
    }
    uint32_t mask = 0;
#pragma unroll
    for (int k = 0; k < 8; ++k) mask |= (before[k] < KEEP ? 1u : 0u) << k;
    return mask;
}

// The kept values in channel order as they travel (bf16: rounded to nearest even, 16-bit patterns;
// fp32: the bits of z), and D: the travelled value where kept, +0 elsewhere.
template <int DT, int KEEP> __device__ __forceinline__ void nm_values8(const F8 &z, uint32_t mask, uint32_t (&vals)[KEEP], F8 &d)
{
#pragma unroll
    for (int r = 0; r < KEEP; ++r) vals[r] = 0u;
    int r = 0;
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        const bool kept = (mask >> k) & 1u;
        const uint32_t raw = (DT == BF16) ? bf16_rne(z.v[k]) : __float_as_uint(z.v[k]);
        const float back = (DT == BF16) ? __uint_as_float(raw << 16) : z.v[k];
        d.v[k] = kept ? back : 0.0f;
#pragma unroll
        for (int q = 0; q < KEEP; ++q) vals[q] = (kept && r == q) ? raw : vals[q];
        r += kept ? 1 : 0;
    }
}

// Receiver side: D from the mask and the travelled values.  Mask bits beyond the KEEP-th are ignored.
// `first`: how many of the block's values belong to lower channels than this lane's (16-channel blocks).
template <int DT, int KEEP> __device__ __forceinline__ void nm_scatter8(uint32_t mask, const uint32_t (&vals)[KEEP], F8 &d, int first = 0)
{
    int r = first;
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        const bool set = ((mask >> k) & 1u) && r < KEEP;
        uint32_t raw = 0u;
#pragma unroll
        for (int q = 0; q < KEEP; ++q) raw = (r == q) ? vals[q] : raw;
        const float v = (DT == BF16) ? __uint_as_float(raw << 16) : __uint_as_float(raw);
        d.v[k] = set ? v : 0.0f;
        r += set ? 1 : 0;
    }
}

// A lane's KEEP values are KEEP * (2 | 4) contiguous bytes at `mine`: 2 bytes are paired with the
// neighbour lane's into one dword (see store_codes_ptr), the rest are dword vectors.
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
template <int DT, int KEEP> __device__ __forceinline__ void nm_store_values(uint8_t *mine, int chunk, const uint32_t (&vals)[KEEP], bool wide)
{
    if (DT == BF16) {
        if (KEEP == 1) store_codes_ptr<2>(mine, chunk, vals[0], wide);
        else if (KEEP == 2) *gmut<uint32_t>(mine) = vals[0] | (vals[1] << 16);
        else {
            u32x2 w;
            w.x = vals[0] | (vals[1] << 16);
            w.y = vals[2] | (vals[3] << 16);
            *gmut<u32x2>(mine) = w;
        }
    } else {
        if (KEEP == 1) *gmut<uint32_t>(mine) = vals[0];
        else if (KEEP == 2) {
            u32x2 w;
            w.x = vals[0]; w.y = vals[1];
            *gmut<u32x2>(mine) = w;
        } else {
            u32x4 w;
            w.x = vals[0]; w.y = vals[1]; w.z = vals[2]; w.w = vals[3];
            *gmut<u32x4>(mine) = w;
        }
    }
}

template <int DT, int KEEP> __device__ __forceinline__ void nm_load_values(const uint8_t *mine, uint32_t (&vals)[KEEP])
{
    if (DT == BF16) {
        if (KEEP == 1) vals[0] = *gconst<uint16_t>(mine);
        else if (KEEP == 2) {
            const uint32_t w = *gconst<uint32_t>(mine);
            vals[0] = w & 0xffffu; vals[1] = w >> 16;
        } else {
            const u32x2 w = *gconst<u32x2>(mine);
            vals[0] = w.x & 0xffffu; vals[1] = w.x >> 16; vals[2] = w.y & 0xffffu; vals[3] = w.y >> 16;
        }
    } else {
        if (KEEP == 1) vals[0] = *gconst<uint32_t>(mine);
        else if (KEEP == 2) {
            const u32x2 w = *gconst<u32x2>(mine);
            vals[0] = w.x; vals[1] = w.y;
        } else {
            const u32x4 w = *gconst<u32x4>(mine);
            vals[0] = w.x; vals[1] = w.y; vals[2] = w.z; vals[3] = w.w;
        }
    }
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

// Sum over the 64 lanes of a wave as a balanced tree over the lane index (lane pairs, then pairs
// of pairs, ...): every lane ends up with the total.  After the two quad steps the lanes of a quad
// agree, so the mirror steps pair quad with quad and half-row with half-row exactly as an xor
// butterfly would.  All 64 lanes must be active.
__device__ __forceinline__ float wave_tree_sum(float v)
{
    v = v + __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0xB1, 0xF, 0xF, false));   // lane ^ 1
    v = v + __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x4E, 0xF, 0xF, false));   // lane ^ 2
    v = v + __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x141, 0xF, 0xF, false));  // other quad of 8
    v = v + __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x140, 0xF, 0xF, false));  // other half of 16
    v = v + __shfl_xor(v, 16);
    v = v + __shfl_xor(v, 32);
    return v;
}

template <bool IS_MAX> __device__ __forceinline__ float comb(float a, float b) { return IS_MAX ? fmaxf(a, b) : a + b; }

// Balanced binary tree over values pushed in index order 0, 1, 2, ...: slot l of
// the stack holds the tree over an aligned block of 2^l indices.  After 2^k
// pushes the total is in slot k and every other slot is empty (+0).  Every slot
// is addressed statically.
template <int LV, bool IS_MAX>
__device__ __forceinline__ void tree_push(float (&stack)[LV], float val, int index, bool active = true)
{
    // Written with selects, not branches: the slots must stay in registers.
    bool carry = active;
#pragma unroll
    for (int l = 0; l < LV; ++l) {
        const bool bit = (index >> l) & 1;
        const float merged = comb<IS_MAX>(stack[l], val);
        stack[l] = carry ? (bit ? 0.0f : val) : stack[l];     // a merged slot is emptied (+0)
        val = (carry && bit) ? merged : val;
        carry = carry && bit;
    }
}

// After a power-of-two number of pushes exactly one slot is occupied and the
// others hold +0, so combining all slots (in any order) returns the total
// unchanged: adding +0, or taking the maximum with +0, is exact for the
// non-negative values reduced here.
template <int LV, bool IS_MAX> __device__ __forceinline__ float tree_top(const float (&stack)[LV])
{
    float res = stack[0];
#pragma unroll
    for (int l = 1; l < LV; ++l) res = comb<IS_MAX>(res, stack[l]);
    return res;
}

// Tree sum (or max) over n values `fetch(i)`, i = 0..n-1, zero padded to a power of
// two.  Values are taken in aligned batches of 16 whose loads are issued
// together; a batch is reduced as a 16-leaf tree in registers and the batch
// results go through the stack (n <= 16 * 2^(LV-1)).  Padding is +0, which
// leaves sums and maxima of non-negative values unchanged, so a short last
// batch or n < 16 gives exactly the tree over the padded range.
template <bool IS_MAX, int LV, class Fetch>
__device__ __forceinline__ float tree_over(int n, Fetch fetch)
{
    constexpr int NB = 16;
    float stack[LV];
#pragma unroll
    for (int l = 0; l < LV; ++l) stack[l] = 0.0f;
    const int nbatch = (n + NB - 1) / NB;
    int bpad = 1;
    while (bpad < nbatch) bpad <<= 1;
    for (int b = 0; b < bpad; ++b) {             // batches past the last are all padding (+0)
        float vals[NB];
#pragma unroll
        for (int u = 0; u < NB; ++u) vals[u] = (b * NB + u < n) ? fetch(b * NB + u) : 0.0f;
        float p2[8], p4[4];
#pragma unroll
        for (int u = 0; u < 8; ++u) p2[u] = comb<IS_MAX>(vals[2 * u], vals[2 * u + 1]);
#pragma unroll
        for (int u = 0; u < 4; ++u) p4[u] = comb<IS_MAX>(p2[2 * u], p2[2 * u + 1]);
        const float lo8 = comb<IS_MAX>(p4[0], p4[1]), hi8 = comb<IS_MAX>(p4[2], p4[3]);
        tree_push<LV, IS_MAX>(stack, comb<IS_MAX>(lo8, hi8), b);
    }
    return tree_top<LV, IS_MAX>(stack);
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
