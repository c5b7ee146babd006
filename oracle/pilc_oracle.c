/*
 * pilc_oracle.c -- see pilc_oracle.h.  TEST INFRASTRUCTURE ONLY: a plain,
 * single-threaded, int64-everywhere reference.  No blocking, no fusion, no
 * tricks: each function is the definition written out so that it can be
 * checked against the paper (arXiv 2206.05279) by eye.
 */
#include "pilc_oracle.h"

#include <math.h>
#include <stdlib.h>
#include <string.h>

/* ------------------------------------------------------------------------- */
/* Tables                                                                     */
/* ------------------------------------------------------------------------- */

#define SIG_N 2049
#define EH_N 640
#define EL_N 64

static uint32_t g_sig[SIG_N];
static uint32_t g_eh[EH_N];
static uint32_t g_el[EL_N];
static int g_tables_ready = 0;

static void build_tables(void)
{
    int i;
    if (g_tables_ready)
        return;
    for (i = 0; i < SIG_N; ++i) {
        double t = ((double)i - 1024.0) / 64.0;
        double s = 1.0 / (1.0 + exp(-t));
        g_sig[i] = (uint32_t)floor(16777216.0 * s + 0.5);
    }
    for (i = 0; i < EH_N; ++i)
        g_eh[i] = (uint32_t)floor(67108864.0 * exp(4.0 - (double)i / 64.0) + 0.5);
    for (i = 0; i < EL_N; ++i)
        g_el[i] = (uint32_t)floor(2147483648.0 * exp(-(double)i / 4096.0) + 0.5);
    g_tables_ready = 1;
}

const uint32_t *pilc_oracle_table_sigmoid(void) { build_tables(); return g_sig; }
const uint32_t *pilc_oracle_table_exp_hi(void) { build_tables(); return g_eh; }
const uint32_t *pilc_oracle_table_exp_lo(void) { build_tables(); return g_el; }

/* floor division by a power of two for a signed value (C's >> on negative
 * values is implementation-defined, so spell it out). */
static int64_t floor_shift(int64_t v, int bits)
{
    int64_t d = (int64_t)1 << bits;
    int64_t q = v / d;
    if ((v % d) != 0 && v < 0)
        q -= 1;
    return q;
}

/* ------------------------------------------------------------------------- */
/* Geometry                                                                   */
/* ------------------------------------------------------------------------- */

static int geom_ok(const pilc_oracle_geom *g)
{
    uint64_t hw;
    if (!g || g->n == 0 || g->h == 0 || g->w == 0)
        return 0;
    if (g->prec_bits < 10 || g->prec_bits > 16)
        return 0;
    hw = (uint64_t)g->h * g->w;
    if (g->lane_mode == 0) {
        if (g->lane_a == 0)
            return 0;
        if (hw % g->lane_a != 0 && g->lane_a % hw != 0)
            return 0;
        return 1;
    }
    if (g->lane_mode == 1)
        return g->lane_a != 0 && g->lane_b != 0;
    return 0;
}

static uint64_t ceil_div(uint64_t a, uint64_t b) { return (a + b - 1) / b; }

uint64_t pilc_oracle_lane_count(const pilc_oracle_geom *g)
{
    if (!geom_ok(g))
        return 0;
    if (g->lane_mode == 0)
        return ceil_div((uint64_t)g->n * g->h * g->w, g->lane_a);
    return (uint64_t)g->n * ceil_div(g->h, g->lane_a) * ceil_div(g->w, g->lane_b);
}

/* A tile lane: which image, where its top-left corner is, and its clipped size. */
static void tile_of_lane(const pilc_oracle_geom *g, uint64_t lane, uint64_t *img, uint64_t *y0,
                         uint64_t *x0, uint64_t *th, uint64_t *tw)
{
    uint64_t tiles_y = ceil_div(g->h, g->lane_a);
    uint64_t tiles_x = ceil_div(g->w, g->lane_b);
    uint64_t per_img = tiles_y * tiles_x;
    uint64_t r = lane % per_img;
    uint64_t ty = r / tiles_x, tx = r % tiles_x;
    *img = lane / per_img;
    *y0 = ty * g->lane_a;
    *x0 = tx * g->lane_b;
    *th = (*y0 + g->lane_a <= g->h) ? g->lane_a : g->h - *y0;
    *tw = (*x0 + g->lane_b <= g->w) ? g->lane_b : g->w - *x0;
}

uint64_t pilc_oracle_lane_pixels(const pilc_oracle_geom *g, uint64_t lane)
{
    if (g->lane_mode == 0) {
        uint64_t total = (uint64_t)g->n * g->h * g->w;
        uint64_t first = lane * g->lane_a;
        uint64_t last = first + g->lane_a;
        if (last > total)
            last = total;
        return last - first;
    } else {
        uint64_t img, y0, x0, th, tw;
        tile_of_lane(g, lane, &img, &y0, &x0, &th, &tw);
        return th * tw;
    }
}

uint64_t pilc_oracle_lane_pixel_index(const pilc_oracle_geom *g, uint64_t lane, uint64_t t)
{
    if (g->lane_mode == 0) {
        return lane * g->lane_a + t;
    } else {
        uint64_t img, y0, x0, th, tw;
        tile_of_lane(g, lane, &img, &y0, &x0, &th, &tw);
        return (img * g->h + y0 + t / tw) * g->w + x0 + t % tw;
    }
}

/* ------------------------------------------------------------------------- */
/* Per-symbol arithmetic                                                      */
/* ------------------------------------------------------------------------- */

/* round-to-nearest division by 2^14 of a signed product (ties towards +inf) */
static int64_t rsh14(int64_t v) { return floor_shift(v + 8192, 14); }

void pilc_oracle_mean_shift(const uint8_t x[3], const uint16_t mu[3], const int16_t coef[3],
                            int64_t out[3])
{
    /* innovations of the already-coded channels, Q8.8, against the UNSHIFTED means */
    int64_t e_r = (int64_t)x[0] * 256 - (int64_t)mu[0];
    int64_t e_g = (int64_t)x[1] * 256 - (int64_t)mu[1];
    out[0] = (int64_t)mu[0];
    out[1] = (int64_t)mu[1] + rsh14((int64_t)coef[0] * e_r);
    out[2] = (int64_t)mu[2] + rsh14((int64_t)coef[1] * e_r) + rsh14((int64_t)coef[2] * e_g);
}

int64_t pilc_oracle_inv_scale(int32_t log_scale_q)
{
    int64_t ls = log_scale_q;
    int64_t u;
    uint64_t prod;
    build_tables();
    if (ls < -16384)
        ls = -16384;
    if (ls > 24575)
        ls = 24575;
    u = ls + 16384; /* 0 .. 40959, i.e. (log_scale + 4) in Q4.12 */
    prod = (uint64_t)g_eh[u >> 6] * (uint64_t)g_el[u & 63];
    return (int64_t)(prod >> 32);
}

uint32_t pilc_oracle_edge_cdf(int64_t mu_eff, int64_t inv_s, int k)
{
    int64_t d, p, z, w, i, r, t0, t1;
    build_tables();
    d = 256 * (int64_t)k - 128 - mu_eff; /* edge k - 1/2 minus the mean, Q8.8 */
    p = d * inv_s;                       /* Q.33 */
    z = floor_shift(p, 17);              /* Q.16 */
    if (z < -(1 << 20))
        z = -(1 << 20);
    if (z > (1 << 20) - 1)
        z = (1 << 20) - 1;
    w = z + (1 << 20); /* 0 .. 2^21-1 */
    i = w >> 10;       /* 0 .. 2047 */
    r = w & 1023;
    t0 = g_sig[i];
    t1 = g_sig[i + 1];
    return (uint32_t)(t0 + (((t1 - t0) * r) >> 10));
}

static uint32_t cum_with_inv(int64_t mu_eff, int64_t inv_s, int prec_bits, int k)
{
    int64_t spread = ((int64_t)1 << prec_bits) - 256;
    if (k <= 0)
        return 0;
    if (k >= 256)
        return (uint32_t)1 << prec_bits;
    return (uint32_t)(k + (((int64_t)pilc_oracle_edge_cdf(mu_eff, inv_s, k) * spread) >> 24));
}

uint32_t pilc_oracle_cum(int64_t mu_eff, int32_t log_scale_q, int prec_bits, int k)
{
    return cum_with_inv(mu_eff, pilc_oracle_inv_scale(log_scale_q), prec_bits, k);
}

int pilc_oracle_symbol_tables(const pilc_oracle_geom *g, const uint8_t *img, const uint16_t *mu,
                              const int16_t *log_scale, const int16_t *chan_coef,
                              uint32_t *cum_out, uint32_t *freq_out)
{
    uint64_t hw, p, total;
    int c;
    if (!geom_ok(g))
        return PILC_ORACLE_E_ARG;
    hw = (uint64_t)g->h * g->w;
    total = (uint64_t)g->n * hw;
    for (p = 0; p < total; ++p) {
        int64_t mu_eff[3];
        pilc_oracle_mean_shift(img + 3 * p, mu + 3 * p, chan_coef + 3 * (p / hw), mu_eff);
        for (c = 0; c < 3; ++c) {
            int v = img[3 * p + c];
            int64_t inv_s = pilc_oracle_inv_scale(log_scale[3 * p + c]);
            uint32_t lo = cum_with_inv(mu_eff[c], inv_s, (int)g->prec_bits, v);
            uint32_t hi = cum_with_inv(mu_eff[c], inv_s, (int)g->prec_bits, v + 1);
            cum_out[3 * p + c] = lo;
            freq_out[3 * p + c] = hi - lo;
        }
    }
    return PILC_ORACLE_OK;
}

double pilc_oracle_cross_entropy_bits(const pilc_oracle_geom *g, const uint8_t *img,
                                      const uint16_t *mu, const int16_t *log_scale,
                                      const int16_t *chan_coef)
{
    uint64_t hw, p, total;
    double bits = 0.0;
    int c;
    if (!geom_ok(g))
        return -1.0;
    hw = (uint64_t)g->h * g->w;
    total = (uint64_t)g->n * hw;
    for (p = 0; p < total; ++p) {
        int64_t mu_eff[3];
        pilc_oracle_mean_shift(img + 3 * p, mu + 3 * p, chan_coef + 3 * (p / hw), mu_eff);
        for (c = 0; c < 3; ++c) {
            int v = img[3 * p + c];
            int64_t inv_s = pilc_oracle_inv_scale(log_scale[3 * p + c]);
            uint32_t lo = cum_with_inv(mu_eff[c], inv_s, (int)g->prec_bits, v);
            uint32_t hi = cum_with_inv(mu_eff[c], inv_s, (int)g->prec_bits, v + 1);
            bits += (double)g->prec_bits - log2((double)(hi - lo));
        }
    }
    return bits;
}

/* ------------------------------------------------------------------------- */
/* rANS core: state in [2^16, 2^32), 16-bit words                             */
/* ------------------------------------------------------------------------- */

#define RANS_LOW ((uint64_t)1 << 16)

int pilc_oracle_rans_encode_tables(const uint32_t *cum, const uint32_t *freq, uint64_t count,
                                   int prec_bits, uint16_t *words_out, uint64_t *nwords_out,
                                   uint32_t *state_out)
{
    uint64_t s = RANS_LOW;
    uint64_t emitted = 0;
    uint64_t t, a, b;
    if (prec_bits < 1 || prec_bits > 16)
        return PILC_ORACLE_E_ARG;
    /* symbols are pushed last-first so that the decoder pops them first-last */
    for (t = count; t-- > 0;) {
        uint64_t f = freq[t], c = cum[t];
        if (f == 0 || c + f > ((uint64_t)1 << prec_bits))
            return PILC_ORACLE_E_ARG;
        /* keep the state below 2^32 after the step: move 16 bits out first */
        if (s >= (f << (32 - prec_bits))) {
            words_out[emitted++] = (uint16_t)(s & 0xFFFF);
            s >>= 16;
        }
        /* App. A eq. (11) */
        s = ((s / f) << prec_bits) + c + (s % f);
    }
    /* words were produced in emission order; the decoder reads them in reverse */
    for (a = 0, b = emitted; a + 1 < b; ++a, --b) {
        uint16_t tmp = words_out[a];
        words_out[a] = words_out[b - 1];
        words_out[b - 1] = tmp;
    }
    *nwords_out = emitted;
    *state_out = (uint32_t)s;
    return PILC_ORACLE_OK;
}

int pilc_oracle_rans_decode_tables(const uint32_t *table_cum, uint64_t count, int prec_bits,
                                   const uint16_t *words, uint64_t nwords, uint32_t state,
                                   uint8_t *sym_out)
{
    uint64_t s = state, next = 0, t;
    uint64_t mask = ((uint64_t)1 << prec_bits) - 1;
    for (t = 0; t < count; ++t) {
        const uint32_t *cdf = table_cum + t * 257;
        uint64_t slot = s & mask;
        int x = 0;
        while (x < 255 && cdf[x + 1] <= slot)
            ++x;
        if (!(cdf[x] <= slot && slot < cdf[x + 1]))
            return PILC_ORACLE_E_CORRUPT;
        sym_out[t] = (uint8_t)x;
        /* App. A eq. (12) */
        s = (uint64_t)(cdf[x + 1] - cdf[x]) * (s >> prec_bits) + slot - cdf[x];
        if (s < RANS_LOW) {
            if (next >= nwords)
                return PILC_ORACLE_E_CORRUPT;
            s = (s << 16) | words[next++];
        }
    }
    if (s != RANS_LOW || next != nwords)
        return PILC_ORACLE_E_CORRUPT;
    return PILC_ORACLE_OK;
}

/* ------------------------------------------------------------------------- */
/* Container                                                                  */
/* ------------------------------------------------------------------------- */

#define HEADER_BYTES 64
#define FORMAT_VERSION 1u

static void put_u16(uint8_t *p, uint32_t v) { p[0] = (uint8_t)v; p[1] = (uint8_t)(v >> 8); }
static void put_u32(uint8_t *p, uint32_t v) { put_u16(p, v & 0xFFFF); put_u16(p + 2, v >> 16); }
static void put_u64(uint8_t *p, uint64_t v) { put_u32(p, (uint32_t)v); put_u32(p + 4, (uint32_t)(v >> 32)); }
static uint32_t get_u16(const uint8_t *p) { return (uint32_t)p[0] | ((uint32_t)p[1] << 8); }
static uint32_t get_u32(const uint8_t *p) { return get_u16(p) | (get_u16(p + 2) << 16); }
static uint64_t get_u64(const uint8_t *p) { return (uint64_t)get_u32(p) | ((uint64_t)get_u32(p + 4) << 32); }

uint64_t pilc_oracle_max_coded_bytes(const pilc_oracle_geom *g)
{
    uint64_t lanes = pilc_oracle_lane_count(g);
    uint64_t sym = (uint64_t)g->n * g->h * g->w * 3;
    if (lanes == 0)
        return 0;
    /* at most one 16-bit word per symbol, one 32-bit state per lane */
    return HEADER_BYTES + 4 * (lanes + 1) + 4 * lanes + 2 * sym;
}

int pilc_oracle_encode(const pilc_oracle_geom *g, const uint8_t *img, const uint16_t *mu,
                       const int16_t *log_scale, const int16_t *chan_coef, uint8_t *coded,
                       uint64_t coded_capacity, uint64_t *coded_bytes)
{
    uint64_t lanes, lane, hw, table_bytes, payload = 0, max_sym = 0;
    uint32_t *cum = NULL, *freq = NULL;
    uint16_t *words = NULL;
    uint8_t *offsets, *body;
    int rc = PILC_ORACLE_OK;

    if (!geom_ok(g) || !img || !mu || !log_scale || !chan_coef || !coded || !coded_bytes)
        return PILC_ORACLE_E_ARG;
    lanes = pilc_oracle_lane_count(g);
    if (lanes >= 0xFFFFFFFFull)
        return PILC_ORACLE_E_TOO_LARGE;
    hw = (uint64_t)g->h * g->w;
    table_bytes = 4 * (lanes + 1);
    if (coded_capacity < HEADER_BYTES + table_bytes)
        return PILC_ORACLE_E_CAPACITY;
    offsets = coded + HEADER_BYTES;
    body = offsets + table_bytes;

    for (lane = 0; lane < lanes; ++lane) {
        uint64_t s = 3 * pilc_oracle_lane_pixels(g, lane);
        if (s > max_sym)
            max_sym = s;
    }
    cum = (uint32_t *)malloc(max_sym * sizeof(uint32_t));
    freq = (uint32_t *)malloc(max_sym * sizeof(uint32_t));
    words = (uint16_t *)malloc(max_sym * sizeof(uint16_t));
    if (!cum || !freq || !words) {
        rc = PILC_ORACLE_E_ARG;
        goto done;
    }

    for (lane = 0; lane < lanes; ++lane) {
        uint64_t npix = pilc_oracle_lane_pixels(g, lane);
        uint64_t t, nwords = 0, bytes, k;
        uint32_t state = 0;
        /* the lane's symbols in decode order: pixels in lane order, R,G,B inside */
        for (t = 0; t < npix; ++t) {
            uint64_t p = pilc_oracle_lane_pixel_index(g, lane, t);
            int64_t mu_eff[3];
            int c;
            pilc_oracle_mean_shift(img + 3 * p, mu + 3 * p, chan_coef + 3 * (p / hw), mu_eff);
            for (c = 0; c < 3; ++c) {
                int v = img[3 * p + c];
                int64_t inv_s = pilc_oracle_inv_scale(log_scale[3 * p + c]);
                uint32_t lo = cum_with_inv(mu_eff[c], inv_s, (int)g->prec_bits, v);
                uint32_t hi = cum_with_inv(mu_eff[c], inv_s, (int)g->prec_bits, v + 1);
                cum[3 * t + c] = lo;
                freq[3 * t + c] = hi - lo;
            }
        }
        rc = pilc_oracle_rans_encode_tables(cum, freq, 3 * npix, (int)g->prec_bits, words, &nwords,
                                            &state);
        if (rc != PILC_ORACLE_OK)
            goto done;
        bytes = 4 + 2 * nwords;
        if (payload + bytes >= ((uint64_t)1 << 32)) {
            rc = PILC_ORACLE_E_TOO_LARGE;
            goto done;
        }
        if (HEADER_BYTES + table_bytes + payload + bytes > coded_capacity) {
            rc = PILC_ORACLE_E_CAPACITY;
            goto done;
        }
        put_u32(offsets + 4 * lane, (uint32_t)payload);
        put_u32(body + payload, state);
        for (k = 0; k < nwords; ++k)
            put_u16(body + payload + 4 + 2 * k, words[k]);
        payload += bytes;
    }
    put_u32(offsets + 4 * lanes, (uint32_t)payload);

    memset(coded, 0, HEADER_BYTES);
    memcpy(coded, "PILC", 4);
    put_u32(coded + 4, FORMAT_VERSION);
    put_u32(coded + 8, g->n);
    put_u32(coded + 12, g->h);
    put_u32(coded + 16, g->w);
    put_u32(coded + 20, 3);
    put_u32(coded + 24, g->prec_bits);
    put_u32(coded + 28, g->lane_mode);
    put_u32(coded + 32, g->lane_a);
    put_u32(coded + 36, g->lane_b);
    put_u32(coded + 40, (uint32_t)lanes);
    put_u64(coded + 48, payload);
    *coded_bytes = HEADER_BYTES + table_bytes + payload;

done:
    free(cum);
    free(freq);
    free(words);
    return rc;
}

int pilc_oracle_decode(const pilc_oracle_geom *g, const uint8_t *coded, uint64_t coded_bytes,
                       const uint16_t *mu, const int16_t *log_scale, const int16_t *chan_coef,
                       uint8_t *img_out)
{
    uint64_t lanes, lane, hw, table_bytes, payload;
    const uint8_t *offsets, *body;
    uint64_t mask;

    if (!geom_ok(g) || !coded || !mu || !log_scale || !chan_coef || !img_out)
        return PILC_ORACLE_E_ARG;
    lanes = pilc_oracle_lane_count(g);
    hw = (uint64_t)g->h * g->w;
    mask = ((uint64_t)1 << g->prec_bits) - 1;
    if (coded_bytes < HEADER_BYTES)
        return PILC_ORACLE_E_FORMAT;
    if (memcmp(coded, "PILC", 4) != 0 || get_u32(coded + 4) != FORMAT_VERSION)
        return PILC_ORACLE_E_FORMAT;
    if (get_u32(coded + 8) != g->n || get_u32(coded + 12) != g->h || get_u32(coded + 16) != g->w ||
        get_u32(coded + 20) != 3 || get_u32(coded + 24) != g->prec_bits ||
        get_u32(coded + 28) != g->lane_mode || get_u32(coded + 32) != g->lane_a ||
        get_u32(coded + 36) != g->lane_b || get_u32(coded + 40) != lanes)
        return PILC_ORACLE_E_FORMAT;
    payload = get_u64(coded + 48);
    table_bytes = 4 * (lanes + 1);
    if (coded_bytes != HEADER_BYTES + table_bytes + payload)
        return PILC_ORACLE_E_FORMAT;
    offsets = coded + HEADER_BYTES;
    body = offsets + table_bytes;
    if (get_u32(offsets) != 0 || get_u32(offsets + 4 * lanes) != payload)
        return PILC_ORACLE_E_CORRUPT;

    for (lane = 0; lane < lanes; ++lane) {
        uint64_t begin = get_u32(offsets + 4 * lane);
        uint64_t end = get_u32(offsets + 4 * (lane + 1));
        uint64_t npix = pilc_oracle_lane_pixels(g, lane);
        uint64_t pos, s, t;
        if (end < begin || end > payload || end - begin < 4 || ((end - begin) & 1))
            return PILC_ORACLE_E_CORRUPT;
        s = get_u32(body + begin);
        pos = begin + 4;
        for (t = 0; t < npix; ++t) {
            uint64_t p = pilc_oracle_lane_pixel_index(g, lane, t);
            uint8_t x[3] = {0, 0, 0};
            int c;
            for (c = 0; c < 3; ++c) {
                int64_t mu_eff[3];
                int64_t inv_s = pilc_oracle_inv_scale(log_scale[3 * p + c]);
                uint64_t slot = s & mask;
                uint32_t lo_c, hi_c;
                int lo = 0, hi = 256;
                /* channels decoded so far are in x[]; later entries are unused by
                 * the mean of channel c */
                pilc_oracle_mean_shift(x, mu + 3 * p, chan_coef + 3 * (p / hw), mu_eff);
                /* binary search for the value v with C(v) <= slot < C(v+1) */
                while (hi - lo > 1) {
                    int mid = (lo + hi) / 2;
                    if (cum_with_inv(mu_eff[c], inv_s, (int)g->prec_bits, mid) <= slot)
                        lo = mid;
                    else
                        hi = mid;
                }
                lo_c = cum_with_inv(mu_eff[c], inv_s, (int)g->prec_bits, lo);
                hi_c = cum_with_inv(mu_eff[c], inv_s, (int)g->prec_bits, lo + 1);
                x[c] = (uint8_t)lo;
                /* App. A eq. (12) */
                s = (uint64_t)(hi_c - lo_c) * (s >> g->prec_bits) + slot - lo_c;
                if (s < RANS_LOW) {
                    if (pos + 2 > end)
                        return PILC_ORACLE_E_CORRUPT;
                    s = (s << 16) | get_u16(body + pos);
                    pos += 2;
                }
            }
            img_out[3 * p + 0] = x[0];
            img_out[3 * p + 1] = x[1];
            img_out[3 * p + 2] = x[2];
        }
        if (s != RANS_LOW || pos != end)
            return PILC_ORACLE_E_CORRUPT;
    }
    return PILC_ORACLE_OK;
}
