/*
 * mix_oracle.h -- plain, slow, single-threaded CPU reference for coding uint8
 * subpixels under a mixture of K logistic laws with the rANS lanes of
 * pilc_oracle.h.
 *
 * TEST INFRASTRUCTURE ONLY.  It exists to check the GPU library, is never part
 * of the product path and shares nothing with the HIP implementation.  It is
 * built on pilc_oracle.c (same directory): the single-law arithmetic (edge
 * CDF, inverse scale, mean shift, lane geometry, rANS recurrences) is the one
 * pinned there.
 *
 * What it follows (arXiv 2206.05279): Sec. 2 ("Entropy Coder" and the "Data
 * transfer" item of Sec. 1) names the workload -- a dynamic rANS coder driven
 * by a mixture of ten logistic laws per symbol -- as what makes
 * earlier learned codecs slow; the paper gives no formula for it.  The coder
 * is that of App. A eqs. (11)-(12) and Sec. 3.2 (integer masses P_x summing to
 * 2^M, C_x their running sum).  Readings taken here, all integer:
 *   - a pixel carries K weights in Q0.15 that sum to 2^15 exactly (one set
 *     for its three subpixels); a subpixel carries K means (Q8.8) and K
 *     log-scales (Q4.12);
 *   - the mixed 24-bit edge CDF is F(k) = floor(sum_j wt_j * F_j(k) / 2^15)
 *     with F_j the single-law edge CDF of pilc_oracle_edge_cdf, and
 *     C(k) = k + floor(F(k) * (2^M - 256) / 2^24), C(0) = 0, C(256) = 2^M:
 *     every value keeps a mass of at least 1, and K = 1 is the single law;
 *   - G is conditioned on R, and B on R and G (Sec. 3.1 eqs. (3)-(4)), by
 *     shifting every component's mean with that component's own innovations
 *     and the image's three coefficients, as pilc_oracle_mean_shift does;
 *   - the container is that of pilc_oracle_encode with the magic "PMIX" and K
 *     in header bytes 44..47.
 *
 * Parity pins (tests/test_oracle_mix.py): K = 1 and K equal components give
 * the single-law tables and container; masses against the float64 closed form
 * of the weighted sum of logistic differences; table invariants; exact round
 * trips; coded length against the cross entropy and against a big-integer
 * arithmetic coder; rejection of weights that do not sum to 2^15.
 */
#ifndef MIX_ORACLE_H
#define MIX_ORACLE_H

#include "pilc_oracle.h"

#ifdef __cplusplus
extern "C" {
#endif

#define MIX_ORACLE_MAX_K 16

/* Array layouts: mu, log_scale [n,h,w,3,K]; weight [n,h,w,K]; chan_coef [n,3]; img [n,h,w,3]. */

/* C(k), k = 0..256, of one subpixel: mu_eff[K] effective Q8.8 means, log_scale[K] Q4.12,
 * weight[K] Q0.15 summing to 2^15. */
uint32_t mix_oracle_cum(const int64_t *mu_eff, const int16_t *log_scale, const uint16_t *weight,
                        int num_comp, int prec_bits, int k);

/* (cum, freq) of every subpixel in image layout.  PILC_ORACLE_E_ARG for a bad geometry, K
 * outside 1..16 or a pixel whose weights do not sum to 2^15. */
int mix_oracle_symbol_tables(const pilc_oracle_geom *g, int num_comp, const uint8_t *img,
                             const uint16_t *mu, const int16_t *log_scale, const uint16_t *weight,
                             const int16_t *chan_coef, uint32_t *cum_out, uint32_t *freq_out);

uint64_t mix_oracle_max_coded_bytes(const pilc_oracle_geom *g);

int mix_oracle_encode(const pilc_oracle_geom *g, int num_comp, const uint8_t *img,
                      const uint16_t *mu, const int16_t *log_scale, const uint16_t *weight,
                      const int16_t *chan_coef, uint8_t *coded, uint64_t coded_capacity,
                      uint64_t *coded_bytes);

int mix_oracle_decode(const pilc_oracle_geom *g, int num_comp, const uint8_t *coded,
                      uint64_t coded_bytes, const uint16_t *mu, const int16_t *log_scale,
                      const uint16_t *weight, const int16_t *chan_coef, uint8_t *img_out);

#ifdef __cplusplus
}
#endif
#endif
