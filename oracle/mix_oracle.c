/* mix_oracle.c -- see mix_oracle.h.  TEST INFRASTRUCTURE ONLY. */
#include "mix_oracle.h"

#include <stdlib.h>
#include <string.h>

#define RANS_LOW ((uint64_t)1 << 16)
#define HEADER_BYTES 64
#define FORMAT_VERSION 1u

static void put_u16(uint8_t *p, uint32_t v) { p[0] = (uint8_t)v; p[1] = (uint8_t)(v >> 8); }
static void put_u32(uint8_t *p, uint32_t v) { put_u16(p, v & 0xFFFF); put_u16(p + 2, v >> 16); }
static void put_u64(uint8_t *p, uint64_t v) { put_u32(p, (uint32_t)v); put_u32(p + 4, (uint32_t)(v >> 32)); }
static uint32_t get_u16(const uint8_t *p) { return (uint32_t)p[0] | ((uint32_t)p[1] << 8); }
static uint32_t get_u32(const uint8_t *p) { return get_u16(p) | (get_u16(p + 2) << 16); }
static uint64_t get_u64(const uint8_t *p) { return (uint64_t)get_u32(p) | ((uint64_t)get_u32(p + 4) << 32); }

uint32_t mix_oracle_cum(const int64_t *mu_eff, const int16_t *log_scale, const uint16_t *weight,
                        int num_comp, int prec_bits, int k)
{
    uint64_t sum = 0, f;
    int j;
    if (k <= 0)
        return 0;
    if (k >= 256)
        return (uint32_t)1 << prec_bits;
    for (j = 0; j < num_comp; ++j)
        sum += (uint64_t)weight[j] *
               pilc_oracle_edge_cdf(mu_eff[j], pilc_oracle_inv_scale(log_scale[j]), k);
    f = sum >> 15; /* the mixed 24-bit edge CDF */
    return (uint32_t)k + (uint32_t)((f * (((uint64_t)1 << prec_bits) - 256)) >> 24);
}

static int weights_ok(const uint16_t *weight, int num_comp)
{
    uint32_t s = 0;
    int j;
    for (j = 0; j < num_comp; ++j)
        s += weight[j];
    return s == (1u << 15);
}

/* Effective means of channel c of pixel p for every component: the single-law mean shift applied
 * to component j's three means with the values x decoded so far (later entries are not used). */
static void comp_means(int num_comp, const uint8_t x[3], const uint16_t *mu_px, const int16_t *coef,
                       int c, int64_t *mu_eff)
{
    int j;
    for (j = 0; j < num_comp; ++j) {
        uint16_t m3[3];
        int64_t e3[3];
        m3[0] = mu_px[0 * num_comp + j];
        m3[1] = mu_px[1 * num_comp + j];
        m3[2] = mu_px[2 * num_comp + j];
        pilc_oracle_mean_shift(x, m3, coef, e3);
        mu_eff[j] = e3[c];
    }
}

static int args_ok(const pilc_oracle_geom *g, int num_comp)
{
    return pilc_oracle_lane_count(g) != 0 && num_comp >= 1 && num_comp <= MIX_ORACLE_MAX_K;
}

int mix_oracle_symbol_tables(const pilc_oracle_geom *g, int num_comp, const uint8_t *img,
                             const uint16_t *mu, const int16_t *log_scale, const uint16_t *weight,
                             const int16_t *chan_coef, uint32_t *cum_out, uint32_t *freq_out)
{
    uint64_t hw, total, p;
    if (!args_ok(g, num_comp) || !img || !mu || !log_scale || !weight || !chan_coef || !cum_out ||
        !freq_out)
        return PILC_ORACLE_E_ARG;
    hw = (uint64_t)g->h * g->w;
    total = (uint64_t)g->n * hw;
    for (p = 0; p < total; ++p) {
        int c;
        if (!weights_ok(weight + p * num_comp, num_comp))
            return PILC_ORACLE_E_ARG;
        for (c = 0; c < 3; ++c) {
            int64_t mu_eff[MIX_ORACLE_MAX_K];
            const int16_t *ls = log_scale + (3 * p + c) * num_comp;
            int v = img[3 * p + c];
            uint32_t lo, hi;
            comp_means(num_comp, img + 3 * p, mu + 3 * p * num_comp, chan_coef + 3 * (p / hw), c,
                       mu_eff);
            lo = mix_oracle_cum(mu_eff, ls, weight + p * num_comp, num_comp, (int)g->prec_bits, v);
            hi = mix_oracle_cum(mu_eff, ls, weight + p * num_comp, num_comp, (int)g->prec_bits, v + 1);
            cum_out[3 * p + c] = lo;
            freq_out[3 * p + c] = hi - lo;
        }
    }
    return PILC_ORACLE_OK;
}

uint64_t mix_oracle_max_coded_bytes(const pilc_oracle_geom *g) { return pilc_oracle_max_coded_bytes(g); }

int mix_oracle_encode(const pilc_oracle_geom *g, int num_comp, const uint8_t *img,
                      const uint16_t *mu, const int16_t *log_scale, const uint16_t *weight,
                      const int16_t *chan_coef, uint8_t *coded, uint64_t coded_capacity,
                      uint64_t *coded_bytes)
{
    uint64_t lanes, lane, total, table_bytes, payload = 0, max_sym = 0;
    uint32_t *cum = NULL, *freq = NULL, *lane_cum = NULL, *lane_freq = NULL;
    uint16_t *words = NULL;
    uint8_t *offsets, *body;
    int rc;

    if (!args_ok(g, num_comp) || !img || !mu || !log_scale || !weight || !chan_coef || !coded ||
        !coded_bytes)
        return PILC_ORACLE_E_ARG;
    lanes = pilc_oracle_lane_count(g);
    if (lanes >= 0xFFFFFFFFull)
        return PILC_ORACLE_E_TOO_LARGE;
    total = (uint64_t)g->n * g->h * g->w;
    table_bytes = 4 * (lanes + 1);
    if (coded_capacity < HEADER_BYTES + table_bytes)
        return PILC_ORACLE_E_CAPACITY;
    offsets = coded + HEADER_BYTES;
    body = offsets + table_bytes;

    /* the masses of every subpixel first (the encoder knows all values), then lane by lane */
    cum = (uint32_t *)malloc(3 * total * sizeof(uint32_t));
    freq = (uint32_t *)malloc(3 * total * sizeof(uint32_t));
    for (lane = 0; lane < lanes; ++lane) {
        uint64_t s = 3 * pilc_oracle_lane_pixels(g, lane);
        if (s > max_sym)
            max_sym = s;
    }
    lane_cum = (uint32_t *)malloc(max_sym * sizeof(uint32_t));
    lane_freq = (uint32_t *)malloc(max_sym * sizeof(uint32_t));
    words = (uint16_t *)malloc(max_sym * sizeof(uint16_t));
    if (!cum || !freq || !lane_cum || !lane_freq || !words) {
        rc = PILC_ORACLE_E_ARG;
        goto done;
    }
    rc = mix_oracle_symbol_tables(g, num_comp, img, mu, log_scale, weight, chan_coef, cum, freq);
    if (rc != PILC_ORACLE_OK)
        goto done;

    for (lane = 0; lane < lanes; ++lane) {
        uint64_t npix = pilc_oracle_lane_pixels(g, lane);
        uint64_t t, nwords = 0, bytes, k;
        uint32_t state = 0;
        int c;
        for (t = 0; t < npix; ++t) {
            uint64_t p = pilc_oracle_lane_pixel_index(g, lane, t);
            for (c = 0; c < 3; ++c) {
                lane_cum[3 * t + c] = cum[3 * p + c];
                lane_freq[3 * t + c] = freq[3 * p + c];
            }
        }
        rc = pilc_oracle_rans_encode_tables(lane_cum, lane_freq, 3 * npix, (int)g->prec_bits, words,
                                            &nwords, &state);
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
    memcpy(coded, "PMIX", 4);
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
    put_u32(coded + 44, (uint32_t)num_comp);
    put_u64(coded + 48, payload);
    *coded_bytes = HEADER_BYTES + table_bytes + payload;
    rc = PILC_ORACLE_OK;

done:
    free(cum);
    free(freq);
    free(lane_cum);
    free(lane_freq);
    free(words);
    return rc;
}

int mix_oracle_decode(const pilc_oracle_geom *g, int num_comp, const uint8_t *coded,
                      uint64_t coded_bytes, const uint16_t *mu, const int16_t *log_scale,
                      const uint16_t *weight, const int16_t *chan_coef, uint8_t *img_out)
{
    uint64_t lanes, lane, hw, total, table_bytes, payload, mask, p;
    const uint8_t *offsets, *body;

    if (!args_ok(g, num_comp) || !coded || !mu || !log_scale || !weight || !chan_coef || !img_out)
        return PILC_ORACLE_E_ARG;
    lanes = pilc_oracle_lane_count(g);
    hw = (uint64_t)g->h * g->w;
    total = (uint64_t)g->n * hw;
    for (p = 0; p < total; ++p)
        if (!weights_ok(weight + p * num_comp, num_comp))
            return PILC_ORACLE_E_ARG;
    mask = ((uint64_t)1 << g->prec_bits) - 1;
    if (coded_bytes < HEADER_BYTES)
        return PILC_ORACLE_E_FORMAT;
    if (memcmp(coded, "PMIX", 4) != 0 || get_u32(coded + 4) != FORMAT_VERSION)
        return PILC_ORACLE_E_FORMAT;
    if (get_u32(coded + 8) != g->n || get_u32(coded + 12) != g->h || get_u32(coded + 16) != g->w ||
        get_u32(coded + 20) != 3 || get_u32(coded + 24) != g->prec_bits ||
        get_u32(coded + 28) != g->lane_mode || get_u32(coded + 32) != g->lane_a ||
        get_u32(coded + 36) != g->lane_b || get_u32(coded + 40) != lanes ||
        get_u32(coded + 44) != (uint32_t)num_comp)
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
            uint8_t x[3] = {0, 0, 0};
            int c;
            p = pilc_oracle_lane_pixel_index(g, lane, t);
            for (c = 0; c < 3; ++c) {
                int64_t mu_eff[MIX_ORACLE_MAX_K];
                const int16_t *ls = log_scale + (3 * p + c) * num_comp;
                const uint16_t *wt = weight + p * num_comp;
                uint64_t slot = s & mask;
                uint32_t lo_c, hi_c;
                int v = 0, hi = 256;
                comp_means(num_comp, x, mu + 3 * p * num_comp, chan_coef + 3 * (p / hw), c, mu_eff);
                /* binary search (App. A, text after eq. (12)) for the value v with
                 * C(v) <= slot < C(v+1); C is increasing */
                while (hi - v > 1) {
                    int mid = (v + hi) / 2;
                    if (mix_oracle_cum(mu_eff, ls, wt, num_comp, (int)g->prec_bits, mid) <= slot)
                        v = mid;
                    else
                        hi = mid;
                }
                lo_c = mix_oracle_cum(mu_eff, ls, wt, num_comp, (int)g->prec_bits, v);
                hi_c = mix_oracle_cum(mu_eff, ls, wt, num_comp, (int)g->prec_bits, v + 1);
                x[c] = (uint8_t)v;
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
