/*
 * twar_oracle.h -- plain CPU reference of the Three-Way Auto-regressive residual transform.
 *
 * TEST INFRASTRUCTURE ONLY (as pilc_oracle.h): never part of the product path, shares no code
 * with the HIP implementation.
 *
 * What it follows (arXiv 2206.05279, Sec. 3.1, eqs. (2)-(4)): every subpixel is predicted from
 * three already known values,
 *   R(u,v) from R(u-1,v-1), R(u-1,v), R(u,v-1)          (up-left, up, left)
 *   G(u,v) from G(u,v-1),   R(u,v-1), R(u,v)            (left G, left R, this pixel's R)
 *   B(u,v) from B(u,v-1),   G(u,v-1), G(u,v)            (left B, left G, this pixel's G)
 * each with three weights and a bias (12 parameters), u the row and v the column, the image
 * padded with one row on top and one column on the left; the residual r = x - x^ is what the
 * coder sees, and the inverse recovers x from r exactly because it can form the same x^.
 *
 * Readings where the paper is silent: the padding is zeros; the weights are fixed point (Q2.14,
 * bias in the same scale: Q8.14), x^ = clamp((w . ctx + bias + 2^13) >> 14, 0, 255) with an
 * arithmetic shift (round half up); the residual is taken mod 256 (the coder works in uint8
 * space, Sec. 3.3), so r = (x - x^) mod 256 and x = (r + x^) mod 256.
 * Layout: uint8 [n, h, w, 3], channel-interleaved, as everywhere in this library.
 */
#ifndef TWAR_ORACLE_H
#define TWAR_ORACLE_H
#include <stdint.h>
#ifdef __cplusplus
extern "C" {
#endif

typedef struct {
    int16_t w[3][3]; /* [channel][context value, in the order listed above], Q2.14 */
    int32_t bias[3]; /* Q8.14 */
} twar_params;

int twar_oracle_predict(const twar_params *p, int channel, int a, int b, int c);
void twar_oracle_forward(const twar_params *p, uint32_t n, uint32_t h, uint32_t w, const uint8_t *img,
                         uint8_t *res);
void twar_oracle_inverse(const twar_params *p, uint32_t n, uint32_t h, uint32_t w, const uint8_t *res,
                         uint8_t *img);
#ifdef __cplusplus
}
#endif
#endif
