/* Runs the C oracle over small ragged tensors in every configuration it supports, under AddressSanitizer and
 * UndefinedBehaviorSanitizer: every buffer is allocated at exactly the size the oracle's own size functions give,
 * so any access past an end is caught.  Values are not checked here (the pins do that). */
#include <math.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "cf_oracle.h"

static unsigned long long g_state = 88172645463325252ULL;
static float rnd(void)      /* xorshift, roughly uniform in [-1, 1) */
{
    g_state ^= g_state << 13; g_state ^= g_state >> 7; g_state ^= g_state << 17;
    return (float)((double)(g_state >> 11) / 9007199254740992.0 * 2.0 - 1.0);
}

static int run(cfo_config cfg, int naive)
{
    if (cfo_check(&cfg) != 0) return 0;        /* an unsupported combination: nothing to run */
    const size_t n = (size_t)(cfg.n_tokens * cfg.n_channels);
    const size_t es = cfg.dtype == CFO_BF16 ? 2 : 4, ee = cfg.err_dtype == CFO_BF16 ? 2 : 4;
    void *x = malloc(n * es), *recon = malloc(n * es), *err = malloc(n * ee);
    uint8_t *codes = malloc((size_t)cfo_codes_bytes(&cfg));
    const size_t ns = (size_t)cfo_scales_count(&cfg);
    float *scales = malloc(ns ? ns * sizeof(float) : 4);
    int rc = 0;
    for (int step = 0; step < 3 && rc == 0; ++step) {
        for (size_t i = 0; i < n; ++i) {
            const float v = rnd() * (i % 97 == 0 ? 20.0f : 1.0f);
            if (cfg.dtype == CFO_BF16) ((uint16_t *)x)[i] = cfo_f32_to_bf16(v); else ((float *)x)[i] = v;
        }
        if (step == 0) rc = cfo_warmup(&cfg, x, recon, err);
        else if (naive) rc = cfo_naive(&cfg, x, recon, codes, scales);
        else if (step == 1) rc = cfo_step(&cfg, x, recon, err, codes, scales);
        else {
            rc = cfo_compress(&cfg, x, recon, err, codes, scales);
            if (rc == 0) rc = cfo_decompress(&cfg, codes, scales, recon);
        }
    }
    free(x); free(recon); free(err); free(codes); free(scales);
    return rc;
}

int main(void)
{
    const int shapes[][2] = {{1, 8}, {9, 8}, {67, 136}, {130, 264}, {33, 1024}};
    int ran = 0;
    for (unsigned s = 0; s < sizeof shapes / sizeof shapes[0]; ++s)
        for (int dtype = 0; dtype < 2; ++dtype)
            for (int err_dtype = 0; err_dtype < 2; ++err_dtype)
                for (int ef = 0; ef < 3; ++ef)
                    for (int bits = 1; bits <= 4; bits *= 2) {
                        const struct { int scale, group; } kinds[] = {{CFO_SCALE_CHANNEL, 128}, {CFO_SCALE_GROUP, 128}, {CFO_SCALE_RANK1, 128},
                                                                      {CFO_SPARSE_NM, 8}, {CFO_SPARSE_NM, 16}, {CFO_SPARSE_NM, 32}};
                        for (unsigned k = 0; k < sizeof kinds / sizeof kinds[0]; ++k) {
                            cfo_config cfg;
                            memset(&cfg, 0, sizeof cfg);
                            cfg.n_tokens = shapes[s][0]; cfg.n_channels = shapes[s][1]; cfg.dtype = dtype; cfg.bits = bits;
                            cfg.scale = kinds[k].scale; cfg.group = kinds[k].group; cfg.ef = ef; cfg.err_dtype = err_dtype;
                            if (run(cfg, 0) != 0) { printf("oracle step failed\n"); return 1; }
                            if (ef == 0 && run(cfg, 1) != 0) { printf("oracle naive failed\n"); return 1; }
                            ++ran;
                        }
                    }
    float v[37];
    for (int i = 0; i < 37; ++i) v[i] = rnd();
    if (!isfinite(cfo_treesum(v, 37, 1)) || !isfinite(cfo_treesum(v, 12, 3))) return 1;
    printf("oracle: %d configurations ran clean\n", ran);
    return 0;
}
