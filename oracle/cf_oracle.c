/*
 * CPU oracle for the CompactFusion residual codec.  TEST INFRASTRUCTURE ONLY
 * (see cf_oracle.h).  Plain single-threaded C; every floating-point operation
 * below is one IEEE fp32 operation, written as a separate statement where the
 * order matters.  Build: gcc -O2 -ffp-contract=off -fno-fast-math.
 */
#include "cf_oracle.h"

#include <math.h>
#include <stdlib.h>
#include <string.h>

/* ------------------------------------------------------------------ */
/* Element formats                                                     */
/* ------------------------------------------------------------------ */

/* bf16 is the upper half of an IEEE binary32: widening is exact. */
float cfo_bf16_to_f32(uint16_t h)
{
    uint32_t u = (uint32_t)h << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return f;
}

/* Narrowing rounds to nearest, ties to even, on the 16 discarded bits.
 * NaN stays NaN (quiet bit forced); infinities and overflow to infinity fall
 * out of the integer carry. */
uint16_t cfo_f32_to_bf16(float f)
{
    uint32_t u;
    memcpy(&u, &f, sizeof u);
    if ((u & 0x7fffffffu) > 0x7f800000u)
        return (uint16_t)((u >> 16) | 0x0040u);
    uint32_t keep_lsb = (u >> 16) & 1u;
    u += 0x7fffu + keep_lsb;
    return (uint16_t)(u >> 16);
}

/* The same narrowing over an array (one call instead of one per element from Python). */
void cfo_f32_to_bf16_array(const float *src, uint16_t *dst, int64_t n)
{
    for (int64_t k = 0; k < n; ++k) dst[k] = cfo_f32_to_bf16(src[k]);
}

static float load_elem(const void *p, int dtype, int64_t k)
{
    if (dtype == CFO_BF16)
        return cfo_bf16_to_f32(((const uint16_t *)p)[k]);
    return ((const float *)p)[k];
}

static void store_elem(void *p, int dtype, int64_t k, float v)
{
    if (dtype == CFO_BF16)
        ((uint16_t *)p)[k] = cfo_f32_to_bf16(v);
    else
        ((float *)p)[k] = v;
}

/* ------------------------------------------------------------------ */
/* Configuration                                                       */
/* ------------------------------------------------------------------ */

int cfo_check(const cfo_config *cfg)
{
    if (!cfg) return -1;
    if (cfg->n_tokens < 1 || cfg->n_channels < 8 || cfg->n_channels % 8 != 0) return -1;
    if (cfg->dtype != CFO_F32 && cfg->dtype != CFO_BF16) return -1;
    if (cfg->err_dtype != CFO_F32 && cfg->err_dtype != CFO_BF16) return -1;
    if (cfg->scale == CFO_SPARSE_NM) {  /* bits = N kept of every group = M channels */
        if (cfg->group < 8 || cfg->group > 64 || cfg->group % 8 != 0 || cfg->n_channels % cfg->group != 0) return -1;
        if (cfg->bits < 1 || cfg->bits >= cfg->group) return -1;
        if (cfg->ef != CFO_EF_RECON && cfg->ef != CFO_EF_LITERAL && cfg->ef != CFO_EF_OFF) return -1;
        return 0;
    }
    if (cfg->bits != 1 && cfg->bits != 2 && cfg->bits != 4) return -1;
    if (cfg->ef != CFO_EF_RECON && cfg->ef != CFO_EF_LITERAL && cfg->ef != CFO_EF_OFF) return -1;
    if (cfg->scale == CFO_SCALE_GROUP) {
        if (cfg->bits != 4) return -1;
        if (cfg->group < 8 || cfg->group % 8 != 0 || cfg->n_channels % cfg->group != 0) return -1;
    } else if (cfg->scale == CFO_SCALE_RANK1) {
        if (cfg->bits == 4) return -1; /* the paper's rank-1 scale goes with its 1-/2-bit code books */
    } else if (cfg->scale != CFO_SCALE_CHANNEL) {
        return -1;
    }
    return 0;
}

int64_t cfo_nm_values_offset(const cfo_config *cfg)
{
    int64_t mask_bytes = cfg->n_tokens * (cfg->n_channels / 8);
    return (mask_bytes + 15) / 16 * 16;
}

int64_t cfo_codes_bytes(const cfo_config *cfg)
{
    if (cfg->scale == CFO_SPARSE_NM) {
        int64_t elem = cfg->dtype == CFO_BF16 ? 2 : 4;
        return cfo_nm_values_offset(cfg) + cfg->n_tokens * (cfg->n_channels / cfg->group) * cfg->bits * elem;
    }
    return cfg->n_tokens * (cfg->n_channels * cfg->bits / 8);
}

/* CHANNEL: s[j], C values.  GROUP: s[i][g], N*(C/group) values.
 * RANK1: v[0..C) followed by u[0..N). */
int64_t cfo_scales_count(const cfo_config *cfg)
{
    if (cfg->scale == CFO_SCALE_GROUP) return cfg->n_tokens * (cfg->n_channels / cfg->group);
    if (cfg->scale == CFO_SCALE_RANK1) return cfg->n_channels + cfg->n_tokens;
    if (cfg->scale == CFO_SPARSE_NM) return 0;
    return cfg->n_channels;
}

/* ------------------------------------------------------------------ */
/* Summation order                                                     */
/* ------------------------------------------------------------------ */

/* The paper gives v_j = (1/N) sum_i |X_ij| (App. D "Quantization") without an
 * order; codes must be reproducible bit for bit, so the order is fixed here:
 * a balanced binary tree over the index, the range padded with +0 up to the
 * next power of two.  T(lo,hi) = v[lo] if hi-lo == 1, else T(lo,mid)+T(mid,hi). */
static float tree(const float *v, int64_t n, int64_t stride, int64_t lo, int64_t hi)
{
    if (lo >= n) return 0.0f; /* padding */
    if (hi - lo == 1) return v[lo * stride];
    int64_t mid = lo + (hi - lo) / 2;
    float a = tree(v, n, stride, lo, mid);
    float b = tree(v, n, stride, mid, hi);
    float s = a + b;
    return s;
}

float cfo_treesum(const float *v, int64_t n, int64_t stride)
{
    int64_t p = 1;
    while (p < n) p *= 2;
    return tree(v, n, stride, 0, p);
}

/* ------------------------------------------------------------------ */
/* a1 + a2: what is compressed                                         */
/* ------------------------------------------------------------------ */

/* r = x_t - recon_{t-1} is the residual against the previous reconstruction
 * (Sec. 3.1; App. H: Delta a*_t = a*_t - a~_{t-1}).
 *   EF_RECON   z = r.  Because the base is the reconstruction, r already equals
 *              (true residual) + (error left over from the last step): the
 *              feedback of Sec. 3.2 is implicit (App. H, end of "Analysis
 *              Without Error Feedback").
 *   EF_LITERAL z = r + e: the stored error added on top of r, as a literal
 *              reading of "residual, plus error buffer" would have it.
 *   EF_OFF     z = r - e = x_t - x_{t-1}: the true residual, i.e. the paper's
 *              no-feedback ablation; e then accumulates the total error. */
void cfo_residual(const cfo_config *cfg, const void *x, const void *recon, const void *err, float *z)
{
    int64_t total = cfg->n_tokens * cfg->n_channels;
    for (int64_t k = 0; k < total; ++k) {
        float xv = load_elem(x, cfg->dtype, k);
        float bv = load_elem(recon, cfg->dtype, k);
        float r = xv - bv;
        if (cfg->ef == CFO_EF_LITERAL) {
            float e = load_elem(err, cfg->err_dtype, k);
            r = r + e;
        } else if (cfg->ef == CFO_EF_OFF) {
            float e = load_elem(err, cfg->err_dtype, k);
            r = r - e;
        }
        z[k] = r;
    }
}

/* ------------------------------------------------------------------ */
/* a3: scales                                                          */
/* ------------------------------------------------------------------ */

/* 1-/2-bit, CHANNEL: s_j = (sum_i |z_ij|) / N, the paper's v_j with u = 1.
 * 1-/2-bit, RANK1:   the paper's u v^T: v_j as above and
 *                    u_i = (rowsum_i / C) / (sum_i rowsum_i / (N*C)), u_i = 0 if the
 *                    tensor is all zero; rowsum_i is the tree sum over channels.
 * 4-bit (not in the paper for activations): symmetric absmax scale
 *                    s = max|z| / 7 over the column (CHANNEL) or over `group`
 *                    consecutive channels of one token (GROUP). */
void cfo_scales(const cfo_config *cfg, const float *z, float *scales)
{
    int64_t N = cfg->n_tokens, C = cfg->n_channels;
    if (cfg->bits == 4) {
        if (cfg->scale == CFO_SCALE_GROUP) {
            int64_t G = cfg->group, ng = C / G;
            for (int64_t i = 0; i < N; ++i)
                for (int64_t g = 0; g < ng; ++g) {
                    float m = 0.0f;
                    for (int64_t j = g * G; j < (g + 1) * G; ++j) {
                        float a = fabsf(z[i * C + j]);
                        if (a > m) m = a;
                    }
                    scales[i * ng + g] = m / 7.0f;
                }
        } else {
            for (int64_t j = 0; j < C; ++j) {
                float m = 0.0f;
                for (int64_t i = 0; i < N; ++i) {
                    float a = fabsf(z[i * C + j]);
                    if (a > m) m = a;
                }
                scales[j] = m / 7.0f;
            }
        }
        return;
    }

    float *a = (float *)malloc(sizeof(float) * (size_t)(N * C));
    for (int64_t k = 0; k < N * C; ++k) a[k] = fabsf(z[k]);
    for (int64_t j = 0; j < C; ++j) {
        float sum = cfo_treesum(a + j, N, C);
        scales[j] = sum / (float)N;
    }
    if (cfg->scale == CFO_SCALE_RANK1) {
        float *u = scales + C;
        float *rowsum = (float *)malloc(sizeof(float) * (size_t)N);
        for (int64_t i = 0; i < N; ++i) rowsum[i] = cfo_treesum(a + i * C, C, 1);
        float total = cfo_treesum(rowsum, N, 1);
        float gmean = total / (float)(N * C);
        for (int64_t i = 0; i < N; ++i) {
            float rmean = rowsum[i] / (float)C;
            u[i] = (gmean == 0.0f) ? 0.0f : rmean / gmean;
        }
        free(rowsum);
    }
    free(a);
}

/* The scale that applies to element (i, j). */
static float scale_at(const cfo_config *cfg, const float *scales, int64_t i, int64_t j)
{
    if (cfg->scale == CFO_SCALE_GROUP) {
        int64_t ng = cfg->n_channels / cfg->group;
        return scales[i * ng + j / cfg->group];
    }
    if (cfg->scale == CFO_SCALE_RANK1) {
        float u = scales[cfg->n_channels + i];
        float v = scales[j];
        float s = u * v;
        return s;
    }
    return scales[j];
}

/* ------------------------------------------------------------------ */
/* a4: code selection                                                  */
/* ------------------------------------------------------------------ */

/* 1-bit: q(X) = +-1 -> one sign bit (1 = negative; +-0 is non-negative).
 * 2-bit: q(X) in {-2,-0.5,+0.5,+2}: bit 1 = sign, bit 0 = magnitude
 *        (0 -> 0.5, 1 -> 2).  The nearest level is chosen, so the magnitude bit
 *        is set when |z| exceeds the midpoint 1.25*s (one fp32 product); a tie
 *        keeps the small level.
 * 4-bit: q = round-half-even(z / s) clamped to [-7, 7], stored as a
 *        two's-complement nibble; s == 0 gives q = 0. */
void cfo_select(const cfo_config *cfg, const float *z, const float *scales, uint8_t *code)
{
    int64_t N = cfg->n_tokens, C = cfg->n_channels;
    for (int64_t i = 0; i < N; ++i)
        for (int64_t j = 0; j < C; ++j) {
            float v = z[i * C + j];
            float s = scale_at(cfg, scales, i, j);
            uint8_t c;
            if (cfg->bits == 1) {
                c = (v < 0.0f) ? 1 : 0;
            } else if (cfg->bits == 2) {
                float thr = 1.25f * s;
                c = (uint8_t)(((v < 0.0f) ? 2 : 0) | ((fabsf(v) > thr) ? 1 : 0));
            } else {
                int q = 0;
                if (s != 0.0f) {
                    float t = v / s;
                    float r = rintf(t); /* default rounding mode: nearest, ties to even */
                    if (r > 7.0f) r = 7.0f;
                    if (r < -7.0f) r = -7.0f;
                    q = (int)r;
                }
                c = (uint8_t)(q & 0xF);
            }
            code[i * C + j] = c;
        }
}

/* ------------------------------------------------------------------ */
/* a5: packing                                                         */
/* ------------------------------------------------------------------ */

/* Paper silent.  Codes run along the channels of a token, least significant
 * bits first: byte k of a row holds channels (8/bits)*k ... (8/bits)*k + 8/bits - 1,
 * channel (8/bits)*k + m in bits [bits*m, bits*m + bits). Rows are dense. */
void cfo_pack(const cfo_config *cfg, const uint8_t *code, uint8_t *packed)
{
    int64_t N = cfg->n_tokens, C = cfg->n_channels;
    int per = 8 / cfg->bits;
    int64_t row_bytes = C / per;
    for (int64_t i = 0; i < N; ++i)
        for (int64_t k = 0; k < row_bytes; ++k) {
            unsigned byte = 0;
            for (int m = 0; m < per; ++m)
                byte |= (unsigned)code[i * C + k * per + m] << (cfg->bits * m);
            packed[i * row_bytes + k] = (uint8_t)byte;
        }
}

void cfo_unpack(const cfo_config *cfg, const uint8_t *packed, uint8_t *code)
{
    int64_t N = cfg->n_tokens, C = cfg->n_channels;
    int per = 8 / cfg->bits;
    int64_t row_bytes = C / per;
    unsigned mask = (1u << cfg->bits) - 1u;
    for (int64_t i = 0; i < N; ++i)
        for (int64_t j = 0; j < C; ++j) {
            unsigned byte = packed[i * row_bytes + j / per];
            code[i * C + j] = (uint8_t)((byte >> (cfg->bits * (j % per))) & mask);
        }
}

/* ------------------------------------------------------------------ */
/* a6: decode                                                          */
/* ------------------------------------------------------------------ */

/* Q(X) = q(X) (.) scale (App. D "Quantization"): level times scale. */
void cfo_decode(const cfo_config *cfg, const uint8_t *code, const float *scales, float *d)
{
    int64_t N = cfg->n_tokens, C = cfg->n_channels;
    for (int64_t i = 0; i < N; ++i)
        for (int64_t j = 0; j < C; ++j) {
            unsigned c = code[i * C + j];
            float s = scale_at(cfg, scales, i, j);
            float v;
            if (cfg->bits == 1) {
                v = c ? -s : s;
            } else if (cfg->bits == 2) {
                float m = (c & 1u) ? 2.0f * s : 0.5f * s;
                v = (c & 2u) ? -m : m;
            } else {
                int q = (c & 8u) ? (int)c - 16 : (int)c;
                v = (float)q * s;
            }
            d[i * C + j] = v;
        }
}

/* ------------------------------------------------------------------ */
/* N:M block sparsifier                                                */
/* ------------------------------------------------------------------ */

/* Sec. 3.4 names an N:M block sparsifier (selection in linear time, regular
 * memory access, in place of a global top-k) and gives no more.  Reading:
 * blocks are M consecutive channels of one token; the N elements of largest
 * magnitude are kept; magnitudes are ordered by the bit pattern of |z| (the
 * numeric order for everything but NaN, which sorts above infinity, so the
 * order is total); of equal magnitudes the lower channel wins.
 * Element k is kept iff fewer than N elements of its block come before it in
 * that order. */
static uint32_t magnitude_key(float v)
{
    uint32_t u;
    memcpy(&u, &v, sizeof u);
    return u & 0x7fffffffu;
}

void cfo_nm_select(const cfo_config *cfg, const float *z, uint8_t *keep)
{
    int64_t N = cfg->n_tokens, C = cfg->n_channels;
    int M = cfg->group, K = cfg->bits;
    for (int64_t i = 0; i < N; ++i)
        for (int64_t b = 0; b < C / M; ++b) {
            const float *blk = z + i * C + b * M;
            for (int k = 0; k < M; ++k) {
                int before = 0;
                for (int j = 0; j < M; ++j) {
                    uint32_t kj = magnitude_key(blk[j]), kk = magnitude_key(blk[k]);
                    if (kj > kk || (kj == kk && j < k)) ++before;
                }
                keep[i * C + b * M + k] = (uint8_t)(before < K);
            }
        }
}

/* The kept values travel in the storage dtype of the tensor (bf16 values are
 * rounded to nearest even; what the rounding loses stays in the error). */
void cfo_nm_pack(const cfo_config *cfg, const float *z, const uint8_t *keep, uint8_t *wire)
{
    int64_t N = cfg->n_tokens, C = cfg->n_channels;
    int M = cfg->group, K = cfg->bits;
    int64_t row_mask_bytes = C / 8;
    void *values = wire + cfo_nm_values_offset(cfg);
    memset(wire, 0, (size_t)cfo_codes_bytes(cfg));
    for (int64_t i = 0; i < N; ++i)
        for (int64_t b = 0; b < C / M; ++b) {
            int r = 0;
            for (int k = 0; k < M; ++k) {
                int64_t j = b * M + k;
                if (!keep[i * C + j]) continue;
                wire[i * row_mask_bytes + j / 8] |= (uint8_t)(1u << (j % 8));
                store_elem(values, cfg->dtype, (i * (C / M) + b) * K + r, z[i * C + j]);
                ++r;
            }
        }
}

/* D: the transmitted value where the mask bit is set, +0 elsewhere. */
void cfo_nm_unpack(const cfo_config *cfg, const uint8_t *wire, float *d)
{
    int64_t N = cfg->n_tokens, C = cfg->n_channels;
    int M = cfg->group, K = cfg->bits;
    int64_t row_mask_bytes = C / 8;
    const void *values = wire + cfo_nm_values_offset(cfg);
    for (int64_t i = 0; i < N; ++i)
        for (int64_t b = 0; b < C / M; ++b) {
            int r = 0;
            for (int k = 0; k < M; ++k) {
                int64_t j = b * M + k;
                int set = (wire[i * row_mask_bytes + j / 8] >> (j % 8)) & 1;
                float v = 0.0f;
                if (set && r < K) {
                    v = load_elem(values, cfg->dtype, (i * (C / M) + b) * K + r);
                    ++r;
                }
                d[i * C + j] = v;
            }
        }
}

/* ------------------------------------------------------------------ */
/* a7, a8: state updates                                               */
/* ------------------------------------------------------------------ */

/* The error is what compression lost, kept at the sender (Sec. 3.2).
 * RECON, LITERAL: e_t = z - D.  OFF: e_t = e_{t-1} + (z - D) (it is never fed
 * back, so it accumulates). */
static void update_err(const cfo_config *cfg, const float *z, const float *d, void *err)
{
    int64_t total = cfg->n_tokens * cfg->n_channels;
    for (int64_t k = 0; k < total; ++k) {
        float lost = z[k] - d[k];
        if (cfg->ef == CFO_EF_OFF) {
            float e = load_elem(err, cfg->err_dtype, k);
            lost = e + lost;
        }
        store_elem(err, cfg->err_dtype, k, lost);
    }
}

/* a~_t = a~_{t-1} + C(Delta a*_t) (App. H), rounded once to the storage dtype. */
static void update_recon(const cfo_config *cfg, const float *d, void *recon)
{
    int64_t total = cfg->n_tokens * cfg->n_channels;
    for (int64_t k = 0; k < total; ++k) {
        float b = load_elem(recon, cfg->dtype, k);
        float nb = b + d[k];
        store_elem(recon, cfg->dtype, k, nb);
    }
}

/* ------------------------------------------------------------------ */
/* Whole operations                                                    */
/* ------------------------------------------------------------------ */

/* Warm-up: the step is sent uncompressed and seeds the base, a~_1 = a_1
 * (App. D "Warmup Implementation"; App. H.2); nothing was lost, so e = 0. */
int cfo_warmup(const cfo_config *cfg, const void *x0, void *recon, void *err)
{
    if (cfo_check(cfg)) return -1;
    int64_t total = cfg->n_tokens * cfg->n_channels;
    for (int64_t k = 0; k < total; ++k) {
        store_elem(recon, cfg->dtype, k, load_elem(x0, cfg->dtype, k));
        store_elem(err, cfg->err_dtype, k, 0.0f);
    }
    return 0;
}

typedef struct {
    float *z, *d;
    uint8_t *code;
} work;

static int work_alloc(const cfo_config *cfg, work *w)
{
    size_t total = (size_t)(cfg->n_tokens * cfg->n_channels);
    w->z = (float *)malloc(total * sizeof(float));
    w->d = (float *)malloc(total * sizeof(float));
    w->code = (uint8_t *)malloc(total);
    return (w->z && w->d && w->code) ? 0 : -1;
}

static void work_free(work *w)
{
    free(w->z);
    free(w->d);
    free(w->code);
}

/* Sender half: everything up to the wire, plus the sender-side error. */
int cfo_compress(const cfo_config *cfg, const void *x, const void *recon, void *err,
                 uint8_t *codes, float *scales)
{
    if (cfo_check(cfg)) return -1;
    work w;
    if (work_alloc(cfg, &w)) { work_free(&w); return -1; }
    cfo_residual(cfg, x, recon, err, w.z);      /* a1, a2 */
    if (cfg->scale == CFO_SPARSE_NM) {
        cfo_nm_select(cfg, w.z, w.code);
        cfo_nm_pack(cfg, w.z, w.code, codes);
        cfo_nm_unpack(cfg, codes, w.d);
    } else {
        cfo_scales(cfg, w.z, scales);               /* a3 */
        cfo_select(cfg, w.z, scales, w.code);       /* a4 */
        cfo_pack(cfg, w.code, codes);               /* a5 */
        cfo_decode(cfg, w.code, scales, w.d);       /* a6 */
    }
    update_err(cfg, w.z, w.d, err);             /* a7 */
    work_free(&w);
    return 0;
}

/* Receiver half: from the wire to the new reconstruction. */
int cfo_decompress(const cfo_config *cfg, const uint8_t *codes, const float *scales, void *recon)
{
    if (cfo_check(cfg)) return -1;
    work w;
    if (work_alloc(cfg, &w)) { work_free(&w); return -1; }
    if (cfg->scale == CFO_SPARSE_NM) {
        cfo_nm_unpack(cfg, codes, w.d);
    } else {
        cfo_unpack(cfg, codes, w.code);
        cfo_decode(cfg, w.code, scales, w.d);       /* a6 */
    }
    update_recon(cfg, w.d, recon);              /* a8 */
    work_free(&w);
    return 0;
}

/* One full step on one tensor, in the order the method states it. */
int cfo_step(const cfo_config *cfg, const void *x, void *recon, void *err,
             uint8_t *codes, float *scales)
{
    if (cfo_check(cfg)) return -1;
    work w;
    if (work_alloc(cfg, &w)) { work_free(&w); return -1; }
    cfo_residual(cfg, x, recon, err, w.z);      /* a1, a2 */
    if (cfg->scale == CFO_SPARSE_NM) {
        cfo_nm_select(cfg, w.z, w.code);
        cfo_nm_pack(cfg, w.z, w.code, codes);
        cfo_nm_unpack(cfg, codes, w.d);
    } else {
        cfo_scales(cfg, w.z, scales);               /* a3 */
        cfo_select(cfg, w.z, scales, w.code);       /* a4 */
        cfo_pack(cfg, w.code, codes);               /* a5 */
        cfo_decode(cfg, w.code, scales, w.d);       /* a6 */
    }
    update_err(cfg, w.z, w.d, err);             /* a7 */
    update_recon(cfg, w.d, recon);              /* a8 */
    work_free(&w);
    return 0;
}

/* Naive compression (Sec. 3.1): C applied to the activation itself,
 * recon_t = D(C(x_t)); no base, no error buffer. */
int cfo_naive(const cfo_config *cfg, const void *x, void *recon, uint8_t *codes, float *scales)
{
    if (cfo_check(cfg)) return -1;
    work w;
    if (work_alloc(cfg, &w)) { work_free(&w); return -1; }
    int64_t total = cfg->n_tokens * cfg->n_channels;
    for (int64_t k = 0; k < total; ++k) w.z[k] = load_elem(x, cfg->dtype, k);
    if (cfg->scale == CFO_SPARSE_NM) {
        cfo_nm_select(cfg, w.z, w.code);
        cfo_nm_pack(cfg, w.z, w.code, codes);
        cfo_nm_unpack(cfg, codes, w.d);
    } else {
        cfo_scales(cfg, w.z, scales);
        cfo_select(cfg, w.z, scales, w.code);
        cfo_pack(cfg, w.code, codes);
        cfo_decode(cfg, w.code, scales, w.d);
    }
    for (int64_t k = 0; k < total; ++k) store_elem(recon, cfg->dtype, k, w.d[k]);
    work_free(&w);
    return 0;
}
