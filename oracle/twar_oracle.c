/* twar_oracle.c -- see twar_oracle.h.  TEST INFRASTRUCTURE ONLY. */
#include "twar_oracle.h"

#include <stddef.h>

int twar_oracle_predict(const twar_params *p, int ch, int a, int b, int c)
{
    int64_t acc = (int64_t)p->w[ch][0] * a + (int64_t)p->w[ch][1] * b + (int64_t)p->w[ch][2] * c +
                  p->bias[ch] + 8192;
    int64_t v = acc >= 0 ? acc / 16384 : -((-acc + 16383) / 16384); /* floor(acc / 2^14) */
    return v < 0 ? 0 : (v > 255 ? 255 : (int)v);
}

/* value of channel ch at (u, v) of one image, 0 outside (the padding row and column) */
static int at(const uint8_t *im, uint32_t w, int64_t u, int64_t v, int ch)
{
    if (u < 0 || v < 0) return 0;
    return im[((size_t)u * w + (size_t)v) * 3 + ch];
}

static void predict_pixel(const twar_params *p, const uint8_t *x, uint32_t w, int64_t u, int64_t v,
                          int out[3])
{
    /* the pixel's own R and G must already be in x when G and B are predicted */
    out[0] = twar_oracle_predict(p, 0, at(x, w, u - 1, v - 1, 0), at(x, w, u - 1, v, 0), at(x, w, u, v - 1, 0));
    out[1] = twar_oracle_predict(p, 1, at(x, w, u, v - 1, 1), at(x, w, u, v - 1, 0), at(x, w, u, v, 0));
    out[2] = twar_oracle_predict(p, 2, at(x, w, u, v - 1, 2), at(x, w, u, v - 1, 1), at(x, w, u, v, 1));
}

void twar_oracle_forward(const twar_params *p, uint32_t n, uint32_t h, uint32_t w, const uint8_t *img,
                         uint8_t *res)
{
    uint32_t i;
    int64_t u, v;
    for (i = 0; i < n; ++i) {
        const uint8_t *x = img + (size_t)i * h * w * 3;
        uint8_t *r = res + (size_t)i * h * w * 3;
        for (u = 0; u < h; ++u)
            for (v = 0; v < w; ++v) {
                int pr[3], c;
                predict_pixel(p, x, w, u, v, pr);
                for (c = 0; c < 3; ++c)
                    r[((size_t)u * w + (size_t)v) * 3 + c] = (uint8_t)((at(x, w, u, v, c) - pr[c]) & 255);
            }
    }
}

void twar_oracle_inverse(const twar_params *p, uint32_t n, uint32_t h, uint32_t w, const uint8_t *res,
                         uint8_t *img)
{
    uint32_t i;
    int64_t u, v;
    for (i = 0; i < n; ++i) {
        const uint8_t *r = res + (size_t)i * h * w * 3;
        uint8_t *x = img + (size_t)i * h * w * 3;
        /* raster order, R then G then B inside a pixel: every context value is known in time */
        for (u = 0; u < h; ++u)
            for (v = 0; v < w; ++v) {
                size_t o = ((size_t)u * w + (size_t)v) * 3;
                int pr;
                pr = twar_oracle_predict(p, 0, at(x, w, u - 1, v - 1, 0), at(x, w, u - 1, v, 0), at(x, w, u, v - 1, 0));
                x[o] = (uint8_t)((r[o] + pr) & 255);
                pr = twar_oracle_predict(p, 1, at(x, w, u, v - 1, 1), at(x, w, u, v - 1, 0), x[o]);
                x[o + 1] = (uint8_t)((r[o + 1] + pr) & 255);
                pr = twar_oracle_predict(p, 2, at(x, w, u, v - 1, 2), at(x, w, u, v - 1, 1), x[o + 1]);
                x[o + 2] = (uint8_t)((r[o + 2] + pr) & 255);
            }
    }
}
