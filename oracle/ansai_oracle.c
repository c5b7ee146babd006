/* ansai_oracle.c -- see ansai_oracle.h.  TEST INFRASTRUCTURE ONLY. */
#include "ansai_oracle.h"

#include <stdlib.h>
#include <string.h>

static int model_ok(const ansai_model *md)
{
    int i, x;
    if (!md || !md->mass || md->prec_bits < 1 || md->prec_bits > 15 || md->num_dist < 1 ||
        md->num_dist > 255 || md->num_sym < 2 || md->num_sym > 256)
        return 0;
    for (i = 0; i < md->num_dist; ++i) {
        uint64_t sum = 0;
        for (x = 0; x < md->num_sym; ++x) {
            if (md->mass[i * md->num_sym + x] == 0) return 0;
            sum += md->mass[i * md->num_sym + x];
        }
        if (sum != ((uint64_t)1 << md->prec_bits)) return 0;
    }
    return 1;
}

int ansai_oracle_build_tables(const ansai_model *md, int32_t *delta, uint32_t *phi, uint8_t *theta,
                              uint8_t *nbits, uint16_t *next)
{
    uint32_t top;
    int i, x, xs;
    if (!model_ok(md)) return -1;
    top = (uint32_t)1 << md->prec_bits;
    xs = md->num_sym;
    for (i = 0; i < md->num_dist; ++i) {
        uint32_t cum = 0;
        for (x = 0; x < xs; ++x) {
            uint32_t p = md->mass[i * xs + x], s;
            int k = 0;
            while ((p << k) < top) ++k; /* the k with P_x 2^k in [2^M, 2^(M+1)) */
            delta[i * xs + x] = (int32_t)k * (int32_t)top - (int32_t)(p << k);
            phi[i * xs + x] = top - p + cum;
            /* Alg. 2 carried out for every state value that decodes to x */
            for (s = cum; s < cum + p; ++s) {
                uint32_t t = s - cum + p; /* in [P_x, 2 P_x) */
                int b = 0;
                while ((t << b) < top) ++b; /* pops until the state is back above 2^M */
                theta[(size_t)i * top + s] = (uint8_t)x;
                nbits[(size_t)i * top + s] = (uint8_t)b;
                next[(size_t)i * top + s] = (uint16_t)((t << b) - top);
            }
            cum += p;
        }
    }
    return 0;
}

/* Number of significant bits of v (0 for v = 0). */
static int bit_length(uint32_t v)
{
    int n = 0;
    while (v) { ++n; v >>= 1; }
    return n;
}

/* The modified rANS of Sec. 3.2 (Algs. 1-2) without tables, a symbol's whole group of bits at
 * once.  Push of x under masses P, C: the state v in [2^M, 2^(M+1)) gives up its b low bits, b the
 * smallest count with floor(v / 2^b) < 2 P_x (which leaves the rest in [P_x, 2 P_x)), and becomes
 * 2^M + (rest - P_x) + C_x.  b follows from the bit lengths of v and of 2 P_x - 1: shifting by
 * their difference makes the lengths equal, and one more shift is needed exactly if the rest is
 * still above 2 P_x - 1. */
int64_t ansai_oracle_encode_piece_direct(const ansai_model *md, const uint8_t *sym,
                                         const uint8_t *dist, int64_t count, uint8_t *bits_out,
                                         uint32_t *state_out)
{
    uint32_t top, v;
    int64_t n = 0, t;
    if (!model_ok(md)) return -1;
    top = (uint32_t)1 << md->prec_bits;
    v = top; /* the initial state */
    for (t = count - 1; t >= 0; --t) {
        const uint32_t *row;
        uint32_t p, c = 0;
        int x, b, i;
        if (dist[t] >= md->num_dist || sym[t] >= md->num_sym) return -1;
        row = md->mass + (size_t)md->num_sym * dist[t];
        p = row[sym[t]];
        for (x = 0; x < sym[t]; ++x) c += row[x];
        b = bit_length(v) - bit_length(2 * p - 1);
        if (b < 0) b = 0;
        if ((v >> b) >= 2 * p) ++b;
        for (i = 0; i < b; ++i) bits_out[n++] = (uint8_t)((v >> i) & 1); /* bit 0 first */
        v = top + ((v >> b) - p) + c;
    }
    *state_out = v;
    return n;
}

/* Pop: x is the symbol whose interval [C_x, C_x + P_x) holds v - 2^M; t = v - 2^M - C_x + P_x lies
 * in [P_x, 2 P_x), and the b = M + 1 - (bit length of t) bits pushed last return below it, the
 * last pushed one highest, which puts the state back into [2^M, 2^(M+1)). */
int ansai_oracle_decode_piece_direct(const ansai_model *md, const uint8_t *dist, int64_t count,
                                     const uint8_t *bits, int64_t nbits, uint32_t state,
                                     uint8_t *sym_out)
{
    uint32_t top, v;
    int64_t t;
    if (!model_ok(md)) return -1;
    top = (uint32_t)1 << md->prec_bits;
    if (state < top || state >= 2 * top) return -6;
    v = state;
    for (t = 0; t < count; ++t) {
        const uint32_t *row;
        uint32_t c = 0, r = v - top, u;
        int x = 0, b, i;
        if (dist[t] >= md->num_dist) return -1;
        row = md->mass + (size_t)md->num_sym * dist[t];
        while (c + row[x] <= r) c += row[x++];
        sym_out[t] = (uint8_t)x;
        u = r - c + row[x];
        b = md->prec_bits + 1 - bit_length(u);
        if (nbits < b) return -6;
        for (i = 0; i < b; ++i) u = (u << 1) | bits[--nbits];
        v = u;
    }
    return (v == top && nbits == 0) ? 0 : -6;
}

#define HDR 64
static void put32(uint8_t *p, uint32_t v)
{
    p[0] = (uint8_t)v; p[1] = (uint8_t)(v >> 8); p[2] = (uint8_t)(v >> 16); p[3] = (uint8_t)(v >> 24);
}
static uint32_t get32(const uint8_t *p)
{
    return (uint32_t)p[0] | ((uint32_t)p[1] << 8) | ((uint32_t)p[2] << 16) | ((uint32_t)p[3] << 24);
}

uint64_t ansai_oracle_max_coded_bytes(uint32_t pieces, uint32_t count, int m)
{
    uint64_t words = ((uint64_t)count * (uint64_t)m + 31) / 32;
    return HDR + 4 * ((uint64_t)pieces + 1) + (uint64_t)pieces * (8 + 4 * words);
}

typedef struct {
    int32_t *delta;
    uint32_t *phi;
    uint8_t *theta, *nbits;
    uint16_t *next;
} tables;

static int tables_make(const ansai_model *md, tables *tb)
{
    size_t dx = (size_t)md->num_dist * md->num_sym, ds = (size_t)md->num_dist << md->prec_bits;
    tb->delta = (int32_t *)malloc(dx * 4);
    tb->phi = (uint32_t *)malloc(dx * 4);
    tb->theta = (uint8_t *)malloc(ds);
    tb->nbits = (uint8_t *)malloc(ds);
    tb->next = (uint16_t *)malloc(ds * 2);
    return ansai_oracle_build_tables(md, tb->delta, tb->phi, tb->theta, tb->nbits, tb->next);
}
static void tables_free(tables *tb)
{
    free(tb->delta); free(tb->phi); free(tb->theta); free(tb->nbits); free(tb->next);
}

int ansai_oracle_encode(const ansai_model *md, uint32_t pieces, uint32_t count, const uint8_t *sym,
                        const uint8_t *dist, uint8_t *coded, uint64_t capacity,
                        uint64_t *coded_bytes)
{
    tables tb;
    uint32_t top;
    uint64_t table = 4 * ((uint64_t)pieces + 1), payload = 0, i;
    uint8_t *offs, *body;
    int m, rc = 0;
    if (!model_ok(md) || pieces == 0 || count == 0 || !sym || !dist || !coded || !coded_bytes) return -1;
    m = md->prec_bits;
    top = (uint32_t)1 << m;
    if (capacity < ansai_oracle_max_coded_bytes(pieces, count, m)) return -3;
    tables_make(md, &tb);
    offs = coded + HDR;
    body = offs + table;
    for (i = 0; i < pieces && rc == 0; ++i) {
        const uint8_t *x = sym + i * (uint64_t)count, *di = dist + i * (uint64_t)count;
        uint8_t *rec = body + payload;
        uint32_t s = top, nbits = 0, words = 0, k;
        int64_t t;
        for (t = (int64_t)count - 1; t >= 0; --t) {
            uint32_t e, b;
            if (di[t] >= md->num_dist || x[t] >= md->num_sym) { rc = -1; break; }
            e = (uint32_t)di[t] * (uint32_t)md->num_sym + x[t];
            b = (uint32_t)(tb.delta[e] + (int32_t)s) >> m; /* Alg. 3 */
            for (k = 0; k < b; ++k, ++nbits) {             /* the last b bits of S, bit 0 first */
                if ((nbits & 31) == 0) put32(rec + 8 + 4 * words++, 0);
                rec[8 + (nbits >> 3)] |= (uint8_t)(((s >> k) & 1u) << (nbits & 7));
            }
            s = (s >> b) + tb.phi[e];
        }
        put32(rec, s);
        put32(rec + 4, nbits);
        put32(offs + 4 * i, (uint32_t)payload);
        payload += 8 + 4 * (uint64_t)words;
    }
    tables_free(&tb);
    if (rc) return rc;
    put32(offs + 4 * (uint64_t)pieces, (uint32_t)payload);
    memset(coded, 0, HDR);
    memcpy(coded, "PANS", 4);
    put32(coded + 4, 1);
    put32(coded + 8, pieces);
    put32(coded + 12, count);
    put32(coded + 16, (uint32_t)m);
    put32(coded + 20, (uint32_t)md->num_dist);
    put32(coded + 24, (uint32_t)md->num_sym);
    put32(coded + 48, (uint32_t)payload);
    put32(coded + 52, (uint32_t)(payload >> 32));
    *coded_bytes = HDR + table + payload;
    return 0;
}

int ansai_oracle_decode(const ansai_model *md, uint32_t pieces, uint32_t count, const uint8_t *dist,
                        const uint8_t *coded, uint64_t coded_bytes, uint8_t *sym_out)
{
    tables tb;
    uint32_t top;
    uint64_t table = 4 * ((uint64_t)pieces + 1), payload, i;
    const uint8_t *offs, *body;
    int rc = 0;
    if (!model_ok(md) || pieces == 0 || count == 0 || !dist || !coded || !sym_out) return -1;
    top = (uint32_t)1 << md->prec_bits;
    if (coded_bytes < HDR + table || memcmp(coded, "PANS", 4) != 0 || get32(coded + 4) != 1 ||
        get32(coded + 8) != pieces || get32(coded + 12) != count ||
        get32(coded + 16) != (uint32_t)md->prec_bits || get32(coded + 20) != (uint32_t)md->num_dist ||
        get32(coded + 24) != (uint32_t)md->num_sym)
        return -5;
    payload = (uint64_t)get32(coded + 48) | ((uint64_t)get32(coded + 52) << 32);
    if (coded_bytes != HDR + table + payload) return -5;
    tables_make(md, &tb);
    offs = coded + HDR;
    body = offs + table;
    for (i = 0; i < pieces && rc == 0; ++i) {
        uint64_t begin = get32(offs + 4 * i), end = get32(offs + 4 * (i + 1));
        const uint8_t *rec = body + begin, *di = dist + i * (uint64_t)count;
        uint32_t s, nbits, t;
        if (end < begin + 8 || end > payload || ((begin | end) & 3)) { rc = -6; break; }
        s = get32(rec);
        nbits = get32(rec + 4);
        if (s < top || s >= 2 * top || end - begin != 8 + 4 * (((uint64_t)nbits + 31) / 32)) { rc = -6; break; }
        for (t = 0; t < count; ++t) {
            uint32_t e, b, v = 0, k;
            if (di[t] >= md->num_dist) { rc = -1; break; }
            e = (uint32_t)di[t] * top + (s - top);
            sym_out[i * (uint64_t)count + t] = tb.theta[e]; /* Alg. 4 */
            b = tb.nbits[e];
            if (b > nbits) { rc = -6; break; }
            nbits -= b;
            for (k = 0; k < b; ++k) v |= (uint32_t)((rec[8 + ((nbits + k) >> 3)] >> ((nbits + k) & 7)) & 1u) << k;
            s = top + tb.next[e] + v;
        }
        if (rc == 0 && (s != top || nbits != 0)) rc = -6;
    }
    tables_free(&tb);
    return rc;
}

void ansai_oracle_center(const uint8_t *in, const uint8_t *mu, uint64_t n, int inverse, uint8_t *out)
{
    uint64_t i;
    for (i = 0; i < n; ++i) {
        int v = inverse ? (int)in[i] + (int)mu[i] - 128 : (int)in[i] - (int)mu[i] + 128;
        out[i] = (uint8_t)(((v % 256) + 256) % 256);
    }
}
