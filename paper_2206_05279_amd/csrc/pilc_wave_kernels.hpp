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
//   - decode replaces the bisection for the symbol (App. A searches for it by bisection) by one
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
//
// Per symbol the 64 threads evaluate C(k) at the 64 candidates k = base..base+63 of a window
// centred on the predicted mean; a ballot of C(k) <= slot counts how many lie at or below the
// slot, which names the symbol (App. A: the x with C_x <= S mod 2^M < C_x + P_x).  The common
// case (window inside 1..255 and within 2^15 Q8.8 units of the mean, symbol inside the window)
// takes a short exact evaluation with 24-bit multiplies; everything else goes through
// find_symbol_slow, which walks windows with the general 64-bit evaluation.
// --------------------------------------------------------------------------------------------
struct Found {
    uint32_t x, c_lo, c_hi;
};

__device__ __noinline__ Found find_symbol_slow(int me, uint32_t inv_s, uint32_t slot,
                                               uint32_t m_bits, const LdsTables &tab)
{
    const int lane_id = (int)(threadIdx.x & 63u);
    const uint32_t spread = (1u << m_bits) - 256u, top = 1u << m_bits;
    int base = min(max(((me + 128) >> 8) - 31, 0), 193);
    uint32_t cv, cnt;
    for (;;) {
        const int k = base + lane_id;  // 0..256
        cv = cum_inner(min(max(k, 1), 255), me, inv_s, spread, tab);
        cv = k <= 0 ? 0u : cv;
        cv = k >= 256 ? top : cv;
        cnt = (uint32_t)__popcll(__ballot(cv <= slot));
        if (cnt == 0u)
            base = max(base - 63, 0);    // C(0) = 0 <= slot ends this at base 0
        else if (cnt == 64u)
            base = min(base + 63, 193);  // C(256) = 2^M > slot ends this at base 193
        else
            break;
    }
    Found r;
    r.x = (uint32_t)base + cnt - 1u;
    r.c_lo = read_lane(cv, cnt - 1u);
    r.c_hi = read_lane(cv, cnt);
    return r;
}

// Wave-wide buffer of the next 64 stream words, one per thread.
struct WaveReader {
    const uint16_t *payload;
    uint32_t pos, stop;  // 16-bit word indices into the payload (uniform)
    uint32_t base;       // word index held by thread 0 (uniform)
    uint32_t buf;        // this thread's word
    uint32_t lane_id;

    // words past `stop` read as 0: an overrun is detected at the end of the lane (pos != stop)
    __device__ __forceinline__ void fill(uint32_t from)
    {
        base = from;
        uint32_t a = base + lane_id;
        buf = a < stop ? (uint32_t)payload[a] : 0u;
    }
    __device__ __forceinline__ uint32_t next()
    {
        uint32_t idx = pos - base;
        if (idx >= 64u) {
            fill(pos);
            idx = 0u;
        }
        ++pos;
        return read_lane(buf, idx);
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
    uint32_t S = uniform((uint32_t)rd.payload[rd.pos] | ((uint32_t)rd.payload[rd.pos + 1] << 16));
    rd.pos += 2;
    rd.fill(rd.pos);

    const int d0 = 256 * (int)lane_id - 128;  // candidate edge j - 1/2 relative to the window base

    // One symbol.  `win` packs the window chosen for mean `me`: bits 0..7 base (1..192),
    // bit 8 set when the short evaluation is valid for this window.
    auto decode_symbol = [&](int me, uint32_t win, uint32_t inv_s, uint32_t inv_a,
                             uint32_t inv_b) -> uint32_t {
        const uint32_t slot = S & mask;
        const int base = (int)(win & 0xFFu);
        const int d = d0 + ((base << 8) - me);
        // z = floor(d * inv_s / 2^17) with inv_s = inv_a * 2^16 + inv_b, |d| <= 2^15
        const int t = __mul24(d, (int)inv_b) >> 16;
        int w = ((__mul24(d, (int)inv_a) + t) >> 1) + (1 << 20);
        w = min(max(w, 0), (1 << 21) - 1);
        const uint2 cell = tab.sig[w >> 10];
        const uint32_t f24 = cell.x + (__umul24(cell.y, (uint32_t)w & 1023u) >> 10);
        const uint32_t cv = (uint32_t)base + lane_id + scale_mass(f24, spread);
        const uint32_t cnt = (uint32_t)__popcll(__ballot(cv <= slot));
        uint32_t x, c_lo, c_hi;
        if (__builtin_expect((win & 0x100u) != 0u && cnt - 1u < 63u, 1)) {
            x = (uint32_t)base + cnt - 1u;
            c_lo = read_lane(cv, cnt - 1u);
            c_hi = read_lane(cv, cnt);
        } else {
            Found r = find_symbol_slow(me, inv_s, slot, m_bits, tab);
            // keep the chain in scalar registers: the call returns through vector registers
            x = uniform(r.x);
            c_lo = uniform(r.c_lo);
            c_hi = uniform(r.c_hi);
        }
        // App. A eq. (12)
        S = (c_hi - c_lo) * (S >> m_bits) + slot - c_lo;
        if (S < (1u << 16)) S = (S << 16) | rd.next();
        return x;
    };
    // window for a mean: base = clamp(round(mean) - 31, 1, 192); the short evaluation needs
    // |256*k - 128 - mean| <= 2^15 for k in the window, true when the unclamped base is in
    // [-63, 255]
    auto window_of = [](int me) -> uint32_t {
        const int b0 = ((me + 128) >> 8) - 31;
        const uint32_t ok = (uint32_t)(b0 + 63) <= 318u ? 0x100u : 0u;
        return (uint32_t)min(max(b0, 1), 192) | ok;
    };

    for (uint32_t t0 = 0; t0 < sh.npx; t0 += 64u) {
        const uint32_t nb = min(64u, sh.npx - t0);
        // ---- vector part: thread j prepares pixel t0 + j ----
        const bool valid = lane_id < nb;
        const uint32_t p = lane_pixel(g, sh, t0 + (valid ? lane_id : 0u));
        const size_t s = (size_t)p * 3;
        const uint32_t im = p / g.hw;
        const uint32_t v_m01 = (uint32_t)mu[s] | ((uint32_t)mu[s + 1] << 16);
        const uint32_t v_m2 = (uint32_t)mu[s + 2] | (window_of((int)mu[s]) << 16);
        const uint32_t v_i0 = inv_scale(ls[s], tab);
        const uint32_t v_i1 = inv_scale(ls[s + 1], tab);
        const uint32_t v_i2 = inv_scale(ls[s + 2], tab);
        const uint32_t v_a01 =
            (uint32_t)(uint16_t)coef[3 * im] | ((uint32_t)(uint16_t)coef[3 * im + 1] << 16);
        const uint32_t v_a2 = (uint32_t)(int)coef[3 * im + 2];
        uint32_t v_out = 0;

        // ---- serial part: one pixel after the other, all values wave-uniform ----
        for (uint32_t i = 0; i < nb; ++i) {
            const uint32_t m01 = read_lane(v_m01, i), m2w = read_lane(v_m2, i);
            const int m_r = (int)(m01 & 0xFFFFu), m_g = (int)(m01 >> 16), m_b = (int)(m2w & 0xFFFFu);
            const uint32_t a01 = read_lane(v_a01, i);
            const int a_gr = (int)(short)(a01 & 0xFFFFu), a_br = (int)a01 >> 16;
            const int a_bg = (int)read_lane(v_a2, i);
            const uint32_t i0 = read_lane(v_i0, i), i1 = read_lane(v_i1, i), i2 = read_lane(v_i2, i);

            const uint32_t x_r = decode_symbol(m_r, m2w >> 16, i0, i0 >> 16, i0 & 0xFFFFu);
            const int e_r = (int)(x_r << 8) - m_r;
            const int me_g = m_g + rsh14_mul(a_gr, e_r);
            const uint32_t x_g = decode_symbol(me_g, window_of(me_g), i1, i1 >> 16, i1 & 0xFFFFu);
            const int e_g = (int)(x_g << 8) - m_g;
            const int me_b = m_b + rsh14_mul(a_br, e_r) + rsh14_mul(a_bg, e_g);
            const uint32_t x_b = decode_symbol(me_b, window_of(me_b), i2, i2 >> 16, i2 & 0xFFFFu);
            v_out = write_lane(x_r | (x_g << 8) | (x_b << 16), i, v_out);
        }
        if (valid) {
            out[s] = (uint8_t)v_out;
            out[s + 1] = (uint8_t)(v_out >> 8);
            out[s + 2] = (uint8_t)(v_out >> 16);
        }
    }
    if ((S != (1u << 16) || rd.pos != rd.stop) && lane_id == 0) atomicMax(status_code, 6);
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
            me[1] = m[1] + rsh14_mul((int)coef[3 * im], e_r);
            me[2] = m[2] + rsh14_mul((int)coef[3 * im + 1], e_r) + rsh14_mul((int)coef[3 * im + 2], e_g);
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
