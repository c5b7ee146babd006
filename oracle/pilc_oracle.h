/*
 * pilc_oracle.h -- plain, slow, single-threaded CPU reference of the PILC
 * entropy-coding stage.
 *
 * TEST INFRASTRUCTURE ONLY.  This code exists to check the GPU library; it is
 * never part of the product path.  It shares no source, header, table
 * generator or helper with the HIP implementation.  Only the test-suite, the
 * smoke check and the benchmark's cpu_baseline leg may load it.
 *
 * What it follows (arXiv 2206.05279):
 *   - Sec. 3.2, first paragraphs: a constant M is chosen, every symbol x gets an
 *     integer mass P_x with sum_x P_x = 2^M, and C_x = sum_{i<x} P_i.
 *   - App. A, eqs. (11)-(12): the original rANS recurrences
 *         encode  S <- 2^M * floor(S / P_x) + C_x + (S mod P_x)
 *         decode  S <- P_x * floor(S / 2^M) + (S mod 2^M) - C_x
 *     with the symbol found by a search on S mod 2^M, and the state kept in a
 *     fixed range so that the work is O(n)  (App. A, paragraph after eq. (12)).
 *   - Sec. 3.1 (eq. 7) / Sec. 3.3: every subpixel follows a logistic law with
 *     location mu and scale s, restricted to the 256 values 0..255.
 *   - Sec. 3.1, eqs. (3)-(4): G is conditioned on R, and B on R and G, of the
 *     same pixel.
 *   - Sec. 4.1: every byte needed to decode counts towards the coded size.
 *
 * The paper fixes no number format, state range or container.  The readings
 * taken (all integer, no floating point at run time) are documented with each
 * function below.
 *
 * Parity pins: every function here is pinned by tests that do not call it to
 * produce their own expectation -- closed forms in float64, table invariants,
 * hand-computed worked examples, a big-integer arithmetic coder, and a
 * degenerate uniform-table case with a hand-derivable stream length.  Nothing
 * in the paper prints an actual rANS bitstream, so byte-level agreement of the
 * container is pinned only by those properties plus oracle<->GPU identity.
 */
#ifndef PILC_ORACLE_H
#define PILC_ORACLE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Geometry of a batch: n images of h x w pixels, 3 interleaved channels. */
typedef struct {
    uint32_t n, h, w;
    uint32_t prec_bits; /* M, 10..16 */
    uint32_t lane_mode; /* 0: flat pixel ranges of lane_a pixels; 1: tiles lane_a x lane_b (h x w) */
    uint32_t lane_a, lane_b;
} pilc_oracle_geom;

enum {
    PILC_ORACLE_OK = 0,
    PILC_ORACLE_E_ARG = -1,
    PILC_ORACLE_E_CAPACITY = -3,
    PILC_ORACLE_E_TOO_LARGE = -4,
    PILC_ORACLE_E_FORMAT = -5,
    PILC_ORACLE_E_CORRUPT = -6
};

/* ---- table constants (built once, in double precision) ------------------- */
/* T[i]  = round(2^24 * sigmoid((i-1024)/64)),  i = 0..2048
 * EH[i] = round(2^26 * exp(4 - i/64)),         i = 0..639
 * EL[j] = round(2^31 * exp(-j/4096)),          j = 0..63                      */
const uint32_t *pilc_oracle_table_sigmoid(void); /* 2049 entries */
const uint32_t *pilc_oracle_table_exp_hi(void);  /* 640 entries  */
const uint32_t *pilc_oracle_table_exp_lo(void);  /* 64 entries   */

/* ---- per-symbol arithmetic ------------------------------------------------ */

/* Number of lanes of a geometry, or 0 if the geometry is invalid. */
uint64_t pilc_oracle_lane_count(const pilc_oracle_geom *g);

/* Pixels in lane j (clipped lanes are shorter), and the flat pixel index
 * (into n*h*w) of the t-th pixel of lane j in decode order. */
uint64_t pilc_oracle_lane_pixels(const pilc_oracle_geom *g, uint64_t lane);
uint64_t pilc_oracle_lane_pixel_index(const pilc_oracle_geom *g, uint64_t lane, uint64_t t);

/* Channel-conditional mean shift (innovation form of the conditioning in
 * Sec. 3.1 eqs. (3)-(4)).  x: the pixel's three values; mu: Q8.8 means;
 * coef: Q2.14 (a_GR, a_BR, a_BG).  out: effective Q8.8 means (may leave
 * [0,65535]; not clamped). */
void pilc_oracle_mean_shift(const uint8_t x[3], const uint16_t mu[3], const int16_t coef[3],
                            int64_t out[3]);

/* Q6.25 value of exp(-log_scale), log_scale in Q4.12 clamped to [-4, 6). */
int64_t pilc_oracle_inv_scale(int32_t log_scale_q);

/* F(k): 24-bit logistic CDF at the edge k - 1/2, k = 1..255. */
uint32_t pilc_oracle_edge_cdf(int64_t mu_eff, int64_t inv_s, int k);

/* C(k), k = 0..256: cumulative integer frequency, C(0)=0, C(256)=2^M. */
uint32_t pilc_oracle_cum(int64_t mu_eff, int32_t log_scale_q, int prec_bits, int k);

/* (cum, freq) of every subpixel, in image layout [n,h,w,3]. */
int pilc_oracle_symbol_tables(const pilc_oracle_geom *g, const uint8_t *img, const uint16_t *mu,
                              const int16_t *log_scale, const int16_t *chan_coef,
                              uint32_t *cum_out, uint32_t *freq_out);

/* sum over subpixels of (M - log2 freq), float64. */
double pilc_oracle_cross_entropy_bits(const pilc_oracle_geom *g, const uint8_t *img,
                                      const uint16_t *mu, const int16_t *log_scale,
                                      const int16_t *chan_coef);

/* ---- rANS core on explicit tables ---------------------------------------- */
/* Encode count symbols whose (cum,freq) are given in decode order.  words_out
 * (capacity count) receives the 16-bit words in decoder read order; returns the
 * number of words and the flushed state. */
int pilc_oracle_rans_encode_tables(const uint32_t *cum, const uint32_t *freq, uint64_t count,
                                   int prec_bits, uint16_t *words_out, uint64_t *nwords_out,
                                   uint32_t *state_out);

/* Decode the slot sequence of a lane given explicit per-position tables:
 * table_cum[t*257 + k] = C_t(k), k = 0..256.  Returns symbols. */
int pilc_oracle_rans_decode_tables(const uint32_t *table_cum, uint64_t count, int prec_bits,
                                   const uint16_t *words, uint64_t nwords, uint32_t state,
                                   uint8_t *sym_out);

/* ---- container ------------------------------------------------------------ */
uint64_t pilc_oracle_max_coded_bytes(const pilc_oracle_geom *g);

int pilc_oracle_encode(const pilc_oracle_geom *g, const uint8_t *img, const uint16_t *mu,
                       const int16_t *log_scale, const int16_t *chan_coef, uint8_t *coded,
                       uint64_t coded_capacity, uint64_t *coded_bytes);

int pilc_oracle_decode(const pilc_oracle_geom *g, const uint8_t *coded, uint64_t coded_bytes,
                       const uint16_t *mu, const int16_t *log_scale, const int16_t *chan_coef,
                       uint8_t *img_out);

#ifdef __cplusplus
}
#endif
#endif
