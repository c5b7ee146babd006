// Wave-per-lane kernels for batches with few, long lanes (gfx950, 64-wide wavefronts).
//
// A rANS lane is a strictly serial chain (App. A eqs. (11)-(12) of arXiv 2206.05279: every
// state depends on the previous one), so a batch with a few thousand lanes cannot fill the chip
// with one thread per lane.  Here one wavefront owns one lane:
//   - everything that does not depend on the state (parameter loads, exp/sigmoid table work,
//     (cum,freq) of known symbols, reciprocals) is done 64 pixels at a time, one pixel per
//     thread, and handed to the serial part through v_readlane;
//   - the state, the stream position and all control flow are wave-uniform, so they live in
//     scalar registers;
//   - decode replaces the bisection for the symbol (App. A: "binary search is needed") by one
//     64-candidate evaluation of C(k) around the predicted mean plus a ballot.
#pragma once

#include "pilc_device.hpp"

namespace pilc {

constexpr int kWavesPerBlock = 4;

__device__ __forceinline__ uint32_t uniform(uint32_t v) { return __builtin_amdgcn_readfirstlane(v); }
__device__ __forceinline__ uint32_t read_lane(uint32_t v, uint32_t l)
{
    return (uint32_t)__builtin_amdgcn_readlane((int)v, (int)l);
}
// value `val` into thread l's copy of a vector register (compare + select)
__device__ __forceinline__ uint32_t write_lane(uint32_t val, uint32_t l, uint32_t old)
{
    return (threadIdx.x & 63u) == l ? val : old;
}

// Flat pixel index of the t-th pixel of a lane (rows of sh.tw pixels, g.w apart).
__device__ __forceinline__ uint32_t lane_pixel(const Geo &g, const LaneShape &sh, uint32_t t)
{
    uint32_t row = t / sh.tw;
    return sh.first + row * g.w + (t - row * sh.tw);
}

// --------------------------------------------------------------------------------------------
// Decode, one wavefront per lane.
// --------------------------------------------------------------------------------------------
struct WaveReader {
    const uint16_t *payload;
    uint32_t pos, stop;   // 16-bit word indices into the payload (uniform)
    uint32_t base;        // first word held in `buf` (even, uniform)
    uint32_t buf;         // per thread: words base+2j (low half) and base+2j+1 (high half)
    uint32_t lane_id;

    __device__ __forceinline__ void fill(uint32_t from)
    {
        base = from & ~1u;
        uint32_t a = base + 2u * lane_id;
        uint32_t lo = a < stop ? payload[a] : 0u;
        uint32_t hi = a + 1u < stop ? payload[a + 1u] : 0u;
        buf = lo | (hi << 16);
    }
    // next word of the lane (caller checked pos < stop)
    __device__ __forceinline__ uint32_t next()
    {
        uint32_t idx = pos - base;
        if (idx >= 128u) {
            fill(pos);
            idx = pos - base;
        }
        uint32_t w = read_lane(buf, idx >> 1);
        ++pos;
        return (idx & 1u) ? (w >> 16) : (w & 0xFFFFu);
    }
};

__global__ __launch_bounds__(64 * kWavesPerBlock) void k_decode_wave(
    Geo g, const uint8_t *__restrict__ coded, const uint16_t *__restrict__ mu,
    const int16_t *__restrict__ ls, const int16_t *__restrict__ coef, uint8_t *__restrict__ out,
    int *__restrict__ status_code, const unsigned long long *__restrict__ status_payload)
{
    __shared__ LdsTables tab;
    load_tables(tab);
    if (*status_code != 0) return;
    const uint32_t lane_id = threadIdx.x & 63u;
    const uint32_t lane = blockIdx.x * kWavesPerBlock + uniform(threadIdx.x >> 6);
    if (lane >= g.lanes) return;
    const LaneShape sh = lane_shape(g, lane);
    const uint32_t m_bits = g.prec_bits;
    const uint32_t spread = (1u << m_bits) - 256u;
    const uint32_t mask = (1u << m_bits) - 1u;
    const uint32_t top = 1u << m_bits;
    const uint32_t payload_bytes = (uint32_t)*status_payload;

    const uint32_t *offsets = reinterpret_cast<const uint32_t *>(coded + 64);
    WaveReader rd;
    rd.payload = reinterpret_cast<const uint16_t *>(coded + 64 + 4ull * ((size_t)g.lanes + 1));
    rd.lane_id = lane_id;
    const uint32_t begin = offsets[lane], end = offsets[lane + 1];
    if (end < begin || end > payload_bytes || end - begin < 4u || ((begin | end) & 1u)) {
        if (lane_id == 0) atomicMax(status_code, 6);
        return;
    }
    rd.pos = begin >> 1;
    rd.stop = end >> 1;
    uint32_t S = (uint32_t)rd.payload[rd.pos] | ((uint32_t)rd.payload[rd.pos + 1] << 16);
    S = uniform(S);
    rd.pos += 2;
    rd.fill(rd.pos);
    bool bad = false;

    for (uint32_t t0 = 0; t0 < sh.npx; t0 += 64u) {
        const uint32_t nb = min(64u, sh.npx - t0);
        // ---- vector part: thread j prepares pixel t0 + j ----
        const bool valid = lane_id < nb;
        const uint32_t p = lane_pixel(g, sh, t0 + (valid ? lane_id : 0u));
        const size_t s = (size_t)p * 3;
        const uint32_t im = p / g.hw;
        const uint32_t v_m01 = (uint32_t)mu[s] | ((uint32_t)mu[s + 1] << 16);
        const uint32_t v_m2 = mu[s + 2];
        const uint32_t v_i0 = inv_scale(ls[s], tab);
        const uint32_t v_i1 = inv_scale(ls[s + 1], tab);
        const uint32_t v_i2 = inv_scale(ls[s + 2], tab);
        const uint32_t v_a01 = (uint32_t)(uint16_t)coef[3 * im] | ((uint32_t)(uint16_t)coef[3 * im + 1] << 16);
        const uint32_t v_a2 = (uint32_t)(int)coef[3 * im + 2];
        uint32_t v_out = 0;

        // ---- serial part: one pixel after the other, all values wave-uniform ----
        for (uint32_t i = 0; i < nb; ++i) {
            const uint32_t m01 = read_lane(v_m01, i);
            const int m_r = (int)(m01 & 0xFFFFu), m_g = (int)(m01 >> 16);
            const int m_b = (int)read_lane(v_m2, i);
            const uint32_t a01 = read_lane(v_a01, i);
            const int a_gr = (int)(short)(a01 & 0xFFFFu), a_br = (int)(short)(a01 >> 16);
            const int a_bg = (int)read_lane(v_a2, i);
            uint32_t inv[3] = {read_lane(v_i0, i), read_lane(v_i1, i), read_lane(v_i2, i)};
            int x[3] = {0, 0, 0};
#pragma unroll
            for (int c = 0; c < 3; ++c) {
                int me = m_r;
                if (c == 1) me = m_g + rsh14(a_gr * (x[0] * 256 - m_r));
                if (c == 2) me = m_b + rsh14(a_br * (x[0] * 256 - m_r)) + rsh14(a_bg * (x[1] * 256 - m_g));
                const uint32_t slot = S & mask;
                // 64 candidates C(base + j); the symbol is base + (#candidates <= slot) - 1
                int base = min(max(((me + 128) >> 8) - 31, 0), 193);
                uint32_t cv, cnt;
                for (;;) {
                    const int k = base + (int)lane_id;
                    cv = cum_inner(min(max(k, 1), 255), me, inv[c], spread, tab);
                    cv = k <= 0 ? 0u : cv;
                    cv = k >= 256 ? top : cv;
                    cnt = (uint32_t)__popcll(__ballot(cv <= slot));
                    if (cnt == 0u)
                        base = max(base - 63, 0);      // C(0) = 0 <= slot ends this at base 0
                    else if (cnt == 64u)
                        base = min(base + 63, 193);    // C(256) = 2^M > slot ends this at base 193
                    else
                        break;
                }
                x[c] = base + (int)cnt - 1;
                const uint32_t c_lo = read_lane(cv, cnt - 1u), c_hi = read_lane(cv, cnt);
                // App. A eq. (12)
                S = (c_hi - c_lo) * (S >> m_bits) + slot - c_lo;
                if (S < (1u << 16)) {
                    if (rd.pos < rd.stop) {
                        S = (S << 16) | rd.next();
                    } else {
                        bad = true;
                        S |= 1u << 16;
                    }
                }
            }
            v_out = write_lane((uint32_t)x[0] | ((uint32_t)x[1] << 8) | ((uint32_t)x[2] << 16), i, v_out);
        }
        if (valid) {
            out[s] = (uint8_t)v_out;
            out[s + 1] = (uint8_t)(v_out >> 8);
            out[s + 2] = (uint8_t)(v_out >> 16);
        }
    }
    if ((bad || S != (1u << 16) || rd.pos != rd.stop) && lane_id == 0) atomicMax(status_code, 6);
}

// --------------------------------------------------------------------------------------------
// Encode, one wavefront per lane.  Per 64 pixels: every thread computes (cum,freq) and an
// exact reciprocal of freq for its pixel's three symbols; then the wave pushes the 192 symbols
// last-first through the scalar state (App. A eq. (11)).  Words are collected 128 at a time in
// a vector register and written to the lane's scratch slot from its end downwards.
// --------------------------------------------------------------------------------------------

// Magic number of the round-up division by f for 32-bit dividends (Granlund & Montgomery):
// with l = ceil(log2 f), m = floor(2^32 * (2^l - f) / f) + 1,
// floor(n / f) = (t + ((n - t) >> min(l,1))) >> max(l-1,0),  t = mulhi(m, n).
__device__ __forceinline__ uint32_t div_magic(uint32_t f)
{
    uint32_t l = f > 1u ? 32u - (uint32_t)__clz(f - 1u) : 0u;
    unsigned long long num = ((1ull << l) - f) << 32;
    return (uint32_t)(num / f) + 1u;
}

__global__ __launch_bounds__(64 * kWavesPerBlock) void k_encode_wave(
    Geo g, const uint8_t *__restrict__ img, const uint16_t *__restrict__ mu,
    const int16_t *__restrict__ ls, const int16_t *__restrict__ coef, uint16_t *__restrict__ scratch,
    uint32_t *__restrict__ lane_words, uint32_t *__restrict__ lane_state)
{
    __shared__ LdsTables tab;
    load_tables(tab);
    const uint32_t lane_id = threadIdx.x & 63u;
    const uint32_t lane = blockIdx.x * kWavesPerBlock + uniform(threadIdx.x >> 6);
    if (lane >= g.lanes) return;
    const LaneShape sh = lane_shape(g, lane);
    const uint32_t m_bits = g.prec_bits;
    const uint32_t spread = (1u << m_bits) - 256u;
    const uint32_t top = 1u << m_bits;
    uint16_t *slot_end = scratch + (size_t)sh.sym_base + 3u * sh.npx;

    uint32_t S = 1u << 16;
    uint32_t nwords = 0;      // words emitted so far (uniform)
    uint32_t pending = 0;     // even-numbered word waiting for its partner (uniform)
    uint32_t v_words = 0;     // thread j: words 128k+2j (high half) and 128k+2j+1 (low half)

    // Writes the first `count` words of the current 128-word group to the slot.  Word e of the
    // lane lives at slot_end[-1 - e].
    auto flush = [&](uint32_t group, uint32_t count) {
        uint32_t e = 128u * group + 2u * lane_id;
        if (2u * lane_id < count) slot_end[-1 - (ptrdiff_t)e] = (uint16_t)(v_words >> 16);
        if (2u * lane_id + 1u < count) slot_end[-2 - (ptrdiff_t)e] = (uint16_t)(v_words & 0xFFFFu);
    };

    const uint32_t batches = (sh.npx + 63u) / 64u;
    for (uint32_t b = batches; b-- > 0u;) {
        const uint32_t t0 = b * 64u;
        const uint32_t nb = min(64u, sh.npx - t0);
        // ---- vector part ----
        const bool valid = lane_id < nb;
        const uint32_t p = lane_pixel(g, sh, t0 + (valid ? lane_id : 0u));
        const size_t s = (size_t)p * 3;
        const uint32_t im = p / g.hw;
        int x[3] = {img[s], img[s + 1], img[s + 2]};
        int m[3] = {mu[s], mu[s + 1], mu[s + 2]};
        int me[3];
        {
            int e_r = x[0] * 256 - m[0], e_g = x[1] * 256 - m[1];
            me[0] = m[0];
            me[1] = m[1] + rsh14((int)coef[3 * im] * e_r);
            me[2] = m[2] + rsh14((int)coef[3 * im + 1] * e_r) + rsh14((int)coef[3 * im + 2] * e_g);
        }
        uint32_t v_cf[3], v_mg[3];
#pragma unroll
        for (int c = 0; c < 3; ++c) {
            uint32_t inv_s = inv_scale(ls[s + c], tab);
            uint32_t lo = x[c] == 0 ? 0u : cum_inner(x[c], me[c], inv_s, spread, tab);
            uint32_t hi = x[c] == 255 ? top : cum_inner(x[c] + 1, me[c], inv_s, spread, tab);
            v_cf[c] = lo | ((hi - lo) << 16);   // cum < 2^16, freq <= 2^16 - 255
            v_mg[c] = div_magic(hi - lo);
        }
        // ---- serial part ----
        for (uint32_t i = nb; i-- > 0u;) {
#pragma unroll
            for (int c = 2; c >= 0; --c) {
                const uint32_t cf = read_lane(v_cf[c], i);
                const uint32_t mg = read_lane(v_mg[c], i);
                const uint32_t f = cf >> 16, cm = cf & 0xFFFFu;
                if (S >= (f << (32u - m_bits))) {
                    const uint32_t word = S & 0xFFFFu;
                    S >>= 16;
                    if (nwords & 1u) {
                        v_words = write_lane((pending << 16) | word, (nwords >> 1) & 63u, v_words);
                        if ((nwords & 127u) == 127u) flush(nwords >> 7, 128u);
                    } else {
                        pending = word;
                    }
                    ++nwords;
                }
                const uint32_t l = f > 1u ? 32u - (uint32_t)__clz(f - 1u) : 0u;
                const uint32_t t = __umulhi(mg, S);
                const uint32_t q = (t + ((S - t) >> min(l, 1u))) >> (l > 0u ? l - 1u : 0u);
                S = S + cm + q * (top - f);   // = (q << M) + (S - q*f) + cum
            }
        }
    }
    // last, partial group
    if (nwords & 1u) v_words = write_lane(pending << 16, (nwords >> 1) & 63u, v_words);
    if (nwords & 127u) flush(nwords >> 7, nwords & 127u);
    if (lane_id == 0) {
        lane_words[lane] = nwords;
        lane_state[lane] = S;
    }
}

}  // namespace pilc
