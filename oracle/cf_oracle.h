/*
 * CPU oracle for the CompactFusion residual codec.  TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, single-threaded C implementation of what one codec step
 * computes, written from the paper (arxiv 2507.17511):
 *   - residual against the stored reconstruction            Sec. 3.1; App. H (residual recursion)
 *   - error feedback kept at the sender                      Sec. 3.2; App. D "Residual Base and Error Feedback"
 *   - warm-up seeds the base with the uncompressed tensor    App. D "Warmup Implementation"; App. H.2
 *   - 1-bit / 2-bit code books and the channel scale v_j     App. D "Quantization"
 *   - N:M block sparsifier under the same residual recursion  Sec. 3.4 (named there, not specified:
 *     block shape, tie rule and wire format are this build's reading; parity unpinned by the paper)
 * Where the paper is silent (4-bit codes, scale groups, packing, tie rules,
 * summation order) the readings are stated at each function.
 *
 * It shares no code with the HIP library and must never be linked, imported
 * or called by the product path: only the tests, the smoke check and the
 * benchmark's cpu-baseline leg may use it.
 *
 * All value arithmetic is IEEE fp32 with one rounding per operation
 * (compile with -ffp-contract=off, no fast-math); codes and packing are
 * integer work.  Tensors are dense row-major [n_tokens, n_channels].
 */
#ifndef CF_ORACLE_H
#define CF_ORACLE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum { CFO_F32 = 0, CFO_BF16 = 1 };
enum { CFO_SCALE_CHANNEL = 0, CFO_SCALE_GROUP = 1, CFO_SCALE_RANK1 = 2, CFO_SPARSE_NM = 3 };
enum { CFO_EF_RECON = 0, CFO_EF_LITERAL = 1, CFO_EF_OFF = 2 };

typedef struct {
    int64_t n_tokens;    /* N */
    int64_t n_channels;  /* C, multiple of 8 */
    int32_t dtype;       /* dtype of x and recon: CFO_F32 | CFO_BF16 */
    int32_t bits;        /* 1, 2 or 4; with CFO_SPARSE_NM: N, the values kept per block */
    int32_t scale;       /* CFO_SCALE_*, or CFO_SPARSE_NM for the N:M block sparsifier (no scales) */
    int32_t group;       /* channels per group when scale == GROUP; with CFO_SPARSE_NM: M, the block length */
    int32_t ef;          /* CFO_EF_* */
    int32_t err_dtype;   /* dtype of the error buffer */
} cfo_config;

/* Element conversions (bf16 <-> fp32), exported so tests can pin them. */
float    cfo_bf16_to_f32(uint16_t h);
uint16_t cfo_f32_to_bf16(float f);
void     cfo_f32_to_bf16_array(const float *src, uint16_t *dst, int64_t n);

/* Balanced binary-tree sum of v[0], v[stride], ..., v[(n-1)*stride]. */
float cfo_treesum(const float *v, int64_t n, int64_t stride);

/* Stages of one step, each on whole tensors (fp32 work arrays). */
void cfo_residual(const cfo_config *cfg, const void *x, const void *recon, const void *err, float *z);
void cfo_scales(const cfo_config *cfg, const float *z, float *scales);
void cfo_select(const cfo_config *cfg, const float *z, const float *scales, uint8_t *code);
void cfo_pack(const cfo_config *cfg, const uint8_t *code, uint8_t *packed);
void cfo_unpack(const cfo_config *cfg, const uint8_t *packed, uint8_t *code);
void cfo_decode(const cfo_config *cfg, const uint8_t *code, const float *scales, float *d);

/* N:M block sparsifier (scale == CFO_SPARSE_NM): of every M consecutive channels of a token the N of
 * largest magnitude are kept.  keep[i*C + j] is 1 for a kept element.  The wire holds one mask bit per
 * element (bit j%8 of byte j/8 of the token's C/8 mask bytes), then, from cfo_nm_values_offset on, the
 * kept values in the storage dtype, token-major, N per block in channel order. */
void cfo_nm_select(const cfo_config *cfg, const float *z, uint8_t *keep);
void cfo_nm_pack(const cfo_config *cfg, const float *z, const uint8_t *keep, uint8_t *wire);
void cfo_nm_unpack(const cfo_config *cfg, const uint8_t *wire, float *d);
int64_t cfo_nm_values_offset(const cfo_config *cfg);

/* Sizes in bytes/elements of the per-tensor buffers. */
int64_t cfo_codes_bytes(const cfo_config *cfg);
int64_t cfo_scales_count(const cfo_config *cfg);

/* Whole operations.  Return 0, or -1 for a configuration the oracle rejects. */
int cfo_check(const cfo_config *cfg);
int cfo_warmup(const cfo_config *cfg, const void *x0, void *recon, void *err);
int cfo_compress(const cfo_config *cfg, const void *x, const void *recon, void *err,
                 uint8_t *codes, float *scales);
int cfo_decompress(const cfo_config *cfg, const uint8_t *codes, const float *scales, void *recon);
int cfo_step(const cfo_config *cfg, const void *x, void *recon, void *err,
             uint8_t *codes, float *scales);

/* Naive compression (the paper's failing baseline, Sec. 3.1): the activation
 * itself is compressed and the reconstruction is its decode; no state. */
int cfo_naive(const cfo_config *cfg, const void *x, void *recon, uint8_t *codes, float *scales);

#ifdef __cplusplus
}
#endif
#endif
