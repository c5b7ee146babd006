// rANS lanes under a mixture of K logistic laws per subpixel, one thread per lane (gfx950).
//
// Sec. 2 of arXiv 2206.05279 names this workload (a dynamic rANS coder fed a mixture of ten
// logistic laws per symbol) as what holds earlier learned codecs near 1 MB/s; the coder itself is
// App. A eqs. (11)-(12).  A pixel has K weights (Q0.15, summing to 2^15), a subpixel K means and
// K log-scales.  The mixed 24-bit edge CDF is F(k) = floor(sum_j w_j F_j(k) / 2^15) with F_j the
// single-law edge CDF, and C(k) = k + floor(F(k) (2^M - 256) / 2^24); the channel conditioning
// of Sec. 3.1 eqs. (3)-(4) shifts every component's mean with that component's own innovations.
//
// K is a run-time value, so nothing per component lives in registers.  A thread first copies
// the 7 K 16-bit parameters of a pixel into its own LDS slots in one burst of loads (every
// 128-byte line of the arrays is then asked for by one or two bursts rather than by dozens of
// separate loads spread over the pixel's work), then, before a subpixel is coded, turns the
// channel's components into {shifted mean, 1/scale} pairs in further slots; every evaluation of
// C(k) walks those.  All slots are [index][thread] arrays of dwords, so a wavefront's accesses
// are conflict free.  The 16-bit words go through the thread-per-lane scratch layout and packer.
#pragma once

#include "pilc_lane_kernels.hpp"

namespace pilc {

constexpr int kMixMaxComp = 16;
constexpr int kMixThreads = 256;

struct MixArgs {
    const uint16_t *mu;      // [px][3][K]
    const int16_t *ls;       // [px][3][K]
    const uint16_t *weight;  // [px][K]
    const int16_t *coef;     // [n][3]
    uint32_t k;
};

// Dynamic LDS of the mixture kernels: K {mean, 1/scale} pairs per thread as [component][thread]
// 8-byte elements, then per thread the pixel's raw means (3 K halfwords), log-scales (3 K) and
// weights (K), each rounded up to dwords, as [dword][thread].
struct MixSlots {
    uint2 *pairs;    // this thread's column of the pairs
    uint32_t *base;  // this thread's column of the raw parameters
    uint32_t k, stride, raw_ls, raw_w;
    static constexpr uint32_t raw_mu = 0u;
    __device__ __forceinline__ MixSlots(uint32_t *lds, uint32_t k_)
        : pairs(reinterpret_cast<uint2 *>(lds) + threadIdx.x),
          base(lds + 2u * k_ * blockDim.x + threadIdx.x), k(k_), stride(blockDim.x),
          raw_ls((3u * k_ + 1u) / 2u), raw_w(2u * ((3u * k_ + 1u) / 2u))
    {
    }
    __device__ __forceinline__ uint32_t &dword(uint32_t i) const { return base[i * stride]; }
    // halfword e of the array that starts at dword `first`
    __device__ __forceinline__ uint32_t half(uint32_t first, uint32_t e) const
    {
        return reinterpret_cast<const uint16_t *>(&base[(first + (e >> 1)) * stride])[e & 1u];
    }
    __device__ __forceinline__ void set_half(uint32_t first, uint32_t e, uint32_t v) const
    {
        reinterpret_cast<uint16_t *>(&base[(first + (e >> 1)) * stride])[e & 1u] = (uint16_t)v;
    }
    __device__ __forceinline__ void set_pair(uint32_t j, int me, uint32_t inv_s) const
    {
        pairs[j * stride] = make_uint2((uint32_t)me, inv_s);
    }
};

static inline size_t mix_lds_bytes(uint32_t k)
{
    return (size_t)kMixThreads * 4u * (2u * k + 2u * ((3u * k + 1u) / 2u) + (k + 1u) / 2u);
}

// The pixel's parameters into the slots; false if its weights do not sum to 2^15.
__device__ __forceinline__ bool mix_load_pixel(const MixArgs &a, uint32_t p, const MixSlots &s)
{
    const size_t px = (size_t)p * 3u * a.k;
    if ((a.k & 1u) == 0u && ((reinterpret_cast<uintptr_t>(a.mu) | reinterpret_cast<uintptr_t>(a.ls) |
                              reinterpret_cast<uintptr_t>(a.weight)) & 3u) == 0u) {
        // even K: a pixel's block of every array is a whole number of aligned dwords
        const uint32_t *gm = reinterpret_cast<const uint32_t *>(a.mu + px);
        const uint32_t *gl = reinterpret_cast<const uint32_t *>(a.ls + px);
        const uint32_t *gw = reinterpret_cast<const uint32_t *>(a.weight + (size_t)p * a.k);
        const uint32_t n3 = 3u * a.k / 2u, n1 = a.k / 2u;
        for (uint32_t i = 0; i < n3; ++i) s.dword(s.raw_mu + i) = gm[i];
        for (uint32_t i = 0; i < n3; ++i) s.dword(s.raw_ls + i) = gl[i];
        for (uint32_t i = 0; i < n1; ++i) s.dword(s.raw_w + i) = gw[i];
    } else {
        for (uint32_t e = 0; e < 3u * a.k; ++e) s.set_half(s.raw_mu, e, a.mu[px + e]);
        for (uint32_t e = 0; e < 3u * a.k; ++e) s.set_half(s.raw_ls, e, (uint16_t)a.ls[px + e]);
        for (uint32_t e = 0; e < a.k; ++e) s.set_half(s.raw_w, e, a.weight[(size_t)p * a.k + e]);
    }
    uint32_t sum = 0;
    for (uint32_t j = 0; j < a.k; ++j) sum += s.half(s.raw_w, j);
    return sum == (1u << 15);
}

// Even K with dword-aligned arrays: a pixel's raw parameters are 3 K / 2 + 3 K / 2 + K / 2 whole
// dwords, and the kernels keep the NEXT pixel's dwords in registers while they work on the
// current one, so that the loads have a pixel's worth of arithmetic to arrive in.
constexpr int kMixPreMu = 3 * kMixMaxComp / 2, kMixPreW = kMixMaxComp / 2;
struct MixAhead {
    uint32_t m[kMixPreMu], l[kMixPreMu], w[kMixPreW];
};

__device__ __forceinline__ bool mix_can_run_ahead(const MixArgs &a)
{
    return (a.k & 1u) == 0u && ((reinterpret_cast<uintptr_t>(a.mu) | reinterpret_cast<uintptr_t>(a.ls) |
                                 reinterpret_cast<uintptr_t>(a.weight)) & 3u) == 0u;
}

__device__ __forceinline__ void mix_fetch_ahead(const MixArgs &a, uint32_t p, MixAhead &r)
{
    const size_t px = (size_t)p * 3u * a.k;
    const uint32_t *gm = reinterpret_cast<const uint32_t *>(a.mu + px);
    const uint32_t *gl = reinterpret_cast<const uint32_t *>(a.ls + px);
    const uint32_t *gw = reinterpret_cast<const uint32_t *>(a.weight + (size_t)p * a.k);
    const uint32_t n3 = 3u * a.k / 2u, n1 = a.k / 2u;
#pragma unroll
    for (int i = 0; i < kMixPreMu; ++i)
        if ((uint32_t)i < n3) r.m[i] = gm[i];
#pragma unroll
    for (int i = 0; i < kMixPreMu; ++i)
        if ((uint32_t)i < n3) r.l[i] = gl[i];
#pragma unroll
    for (int i = 0; i < kMixPreW; ++i)
        if ((uint32_t)i < n1) r.w[i] = gw[i];
}

// The fetched pixel into the slots; false if its weights do not sum to 2^15.
__device__ __forceinline__ bool mix_store_ahead(const MixAhead &r, const MixSlots &s)
{
    const uint32_t n3 = 3u * s.k / 2u, n1 = s.k / 2u;
    uint32_t sum = 0;
#pragma unroll
    for (int i = 0; i < kMixPreMu; ++i)
        if ((uint32_t)i < n3) s.dword(s.raw_mu + i) = r.m[i];
#pragma unroll
    for (int i = 0; i < kMixPreMu; ++i)
        if ((uint32_t)i < n3) s.dword(s.raw_ls + i) = r.l[i];
#pragma unroll
    for (int i = 0; i < kMixPreW; ++i)
        if ((uint32_t)i < n1) {
            s.dword(s.raw_w + i) = r.w[i];
            sum += (r.w[i] & 0xFFFFu) + (r.w[i] >> 16);
        }
    return sum == (1u << 15);
}

// {shifted mean, 1/scale} of every component of channel `ch` of the loaded pixel into the pair
// slots; x_r and x_g are the pixel's red and green values (used for ch >= 1 and ch == 2).
__device__ __forceinline__ void mix_load_channel(const MixSlots &s, int ch, int x_r, int x_g, int a_gr,
                                                 int a_br, int a_bg, const LdsTables &tab)
{
    for (uint32_t j = 0; j < s.k; ++j) {
        int me = (int)s.half(s.raw_mu, (uint32_t)ch * s.k + j);
        if (ch >= 1) {
            const int e_r = x_r * 256 - (int)s.half(s.raw_mu, j);
            if (ch == 1) {
                me += rsh14_mul(a_gr, e_r);
            } else {
                const int e_g = x_g * 256 - (int)s.half(s.raw_mu, s.k + j);
                me += rsh14_mul(a_br, e_r) + rsh14_mul(a_bg, e_g);
            }
        }
        const int l = (int)(short)s.half(s.raw_ls, (uint32_t)ch * s.k + j);
        s.set_pair(j, me, inv_scale(l, tab));
    }
}

// C(k), 1 <= k <= 255, from the slots.
__device__ __forceinline__ uint32_t mix_cum_inner(int k, const MixSlots &s, uint32_t spread,
                                                  const LdsTables &tab)
{
    auto term = [&](uint32_t j) -> unsigned long long {
        const uint2 c = s.pairs[j * s.stride];
        return (unsigned long long)s.half(s.raw_w, j) * edge_cdf(256 * k + (-128 - (int)c.x), c.y, tab);
    };
    // four (then two) components per round, so that their table reads are in flight together
    unsigned long long acc = 0ull;
    uint32_t j = 0;
    for (; j + 3u < s.k; j += 4u) {
        const unsigned long long t0 = term(j), t1 = term(j + 1u), t2 = term(j + 2u), t3 = term(j + 3u);
        acc += (t0 + t1) + (t2 + t3);
    }
    if (j + 1u < s.k) {
        const unsigned long long t0 = term(j), t1 = term(j + 1u);
        acc += t0 + t1;
        j += 2u;
    }
    if (j < s.k) acc += term(j);
    return (uint32_t)k + scale_mass((uint32_t)(acc >> 15), spread);
}

__global__ __launch_bounds__(kMixThreads) void k_mix_encode(
    Geo g, const uint8_t *__restrict__ img, MixArgs a, uint16_t *__restrict__ scratch,
    uint32_t lane_cap, uint32_t *__restrict__ lane_words, uint32_t *__restrict__ lane_state,
    int *__restrict__ status_code)
{
    __shared__ LdsTables tab;
    extern __shared__ uint32_t mix_lds[];
    load_tables(tab);
    const uint32_t lane = blockIdx.x * blockDim.x + threadIdx.x;
    if (lane >= g.lanes) return;
    const MixSlots slots(mix_lds, a.k);
    const LaneShape sh = lane_shape(g, lane);
    const uint32_t m_bits = g.prec_bits;
    const uint32_t spread = (1u << m_bits) - 256u, top = 1u << m_bits;

    uint16_t *wout = scratch + lane_scratch_base(lane, lane_cap);
    uint32_t nwords = 0, S = 1u << 16;
    bool ok = true;
    // pixels last-first, and B, G, R inside a pixel (App. A eq. (11) runs against the decoder)
    const bool ahead = mix_can_run_ahead(a);
    MixAhead pre;
    uint32_t pre_x = 0, im_now = 0xFFFFFFFFu;
    int a_gr = 0, a_br = 0, a_bg = 0;
    auto fetch_pixel_bytes = [&](uint32_t q) -> uint32_t {
        const uint8_t *b = img + 3 * (size_t)q;
        return (uint32_t)b[0] | ((uint32_t)b[1] << 8) | ((uint32_t)b[2] << 16);
    };
    if (ahead && sh.npx != 0u) {
        const uint32_t q = lane_pixel(g, sh, sh.npx - 1u);
        mix_fetch_ahead(a, q, pre);
        pre_x = fetch_pixel_bytes(q);
    }
    for (uint32_t t = sh.npx; t-- > 0u;) {
        const uint32_t p = lane_pixel(g, sh, t);
        const uint32_t im = p / g.hw;
        if (im != im_now) {
            im_now = im;
            a_gr = a.coef[3 * im]; a_br = a.coef[3 * im + 1]; a_bg = a.coef[3 * im + 2];
        }
        uint32_t xb;
        if (ahead) {
            ok = mix_store_ahead(pre, slots) && ok;
            xb = pre_x;
            if (t != 0u) {
                const uint32_t q = lane_pixel(g, sh, t - 1u);
                mix_fetch_ahead(a, q, pre);
                pre_x = fetch_pixel_bytes(q);
            }
        } else {
            ok = mix_load_pixel(a, p, slots) && ok;
            xb = fetch_pixel_bytes(p);
        }
        const int x[3] = {(int)(xb & 0xFFu), (int)((xb >> 8) & 0xFFu), (int)(xb >> 16)};
#pragma unroll 1
        for (int ch = 2; ch >= 0; --ch) {
            mix_load_channel(slots, ch, x[0], x[1], a_gr, a_br, a_bg, tab);
            const int v = ch == 0 ? x[0] : (ch == 1 ? x[1] : x[2]);
            const uint32_t lo = v == 0 ? 0u : mix_cum_inner(v, slots, spread, tab);
            const uint32_t hi = v == 255 ? top : mix_cum_inner(v + 1, slots, spread, tab);
            const uint32_t f = hi - lo;
            if (S >= (f << (32u - m_bits))) {
                *wout = (uint16_t)(S & 0xFFFFu);
                wout += 64;
                ++nwords;
                S >>= 16;
            }
            uint32_t rem;
            const uint32_t q = div_small(S, f, __builtin_amdgcn_rcpf((float)f), m_bits < 12u, rem);
            S = (q << m_bits) + rem + lo;
        }
    }
    if (!ok) atomicMax(status_code, 7);
    lane_words[lane] = nwords;
    lane_state[lane] = S;
}

// Decoded bytes of consecutive addresses, gathered into aligned 8-byte stores; single bytes only
// up to the first 8-byte boundary of a run and for what is left at its end.
struct ByteRun {
    unsigned __int128 acc;
    uint32_t n;   // bytes in acc (< 11)
    size_t addr;  // where the first of them goes
    __device__ __forceinline__ void begin(size_t a) { acc = 0; n = 0u; addr = a; }
    __device__ __forceinline__ void put3(uint8_t *out, uint32_t v)
    {
        acc |= (unsigned __int128)v << (8u * n);
        n += 3u;
        while (n != 0u && (addr & 7u) != 0u) {
            out[addr++] = (uint8_t)acc;
            acc >>= 8;
            --n;
        }
        if (n >= 8u) {
            *reinterpret_cast<unsigned long long *>(out + addr) = (unsigned long long)acc;
            acc >>= 64;
            n -= 8u;
            addr += 8u;
        }
    }
    __device__ __forceinline__ void end(uint8_t *out)
    {
        while (n != 0u) {
            out[addr++] = (uint8_t)acc;
            acc >>= 8;
            --n;
        }
    }
};

__global__ __launch_bounds__(kMixThreads) void k_mix_decode(
    Geo g, const uint8_t *__restrict__ coded, MixArgs a, uint8_t *__restrict__ out,
    int *__restrict__ status_code, const unsigned long long *__restrict__ status_payload)
{
    __shared__ LdsTables tab;
    extern __shared__ uint32_t mix_lds[];
    load_tables(tab);
    if (*status_code != 0) return;  // uniform: written by an earlier kernel
    const uint32_t lane = blockIdx.x * blockDim.x + threadIdx.x;
    if (lane >= g.lanes) return;
    const MixSlots slots(mix_lds, a.k);
    const LaneShape sh = lane_shape(g, lane);
    const uint32_t m_bits = g.prec_bits;
    const uint32_t spread = (1u << m_bits) - 256u, mask = (1u << m_bits) - 1u;
    const uint32_t payload_bytes = (uint32_t)*status_payload;

    const uint32_t *offsets = reinterpret_cast<const uint32_t *>(coded + 64);
    const uint16_t *payload =
        reinterpret_cast<const uint16_t *>(coded + 64 + 4ull * ((size_t)g.lanes + 1));
    const uint32_t begin = offsets[lane], end = offsets[lane + 1];
    if (end < begin || end > payload_bytes || end - begin < 4u || ((begin | end) & 1u)) {
        atomicMax(status_code, 6);
        return;
    }
    const uint32_t adj = (uint32_t)(reinterpret_cast<uintptr_t>(payload) & 31u);
    const uint16_t *base = reinterpret_cast<const uint16_t *>(reinterpret_cast<const uint8_t *>(payload) - adj);
    const uint32_t first = (adj + begin) >> 1;
    const uint32_t lim = (uint32_t)(((unsigned long long)adj + payload_bytes + 1ull) >> 1);
    WordStream words;
    words.open(base, first, lim);
    uint32_t S = words.take(base, lim);
    S |= words.take(base, lim) << 16;

    bool ok = true;
    ByteRun run;
    run.begin(0);
    uint32_t p_next = 0xFFFFFFFFu;  // the pixel that would continue the current run of bytes
    const bool ahead = mix_can_run_ahead(a);
    MixAhead pre;
    uint32_t im_now = 0xFFFFFFFFu;
    int a_gr = 0, a_br = 0, a_bg = 0;
    if (ahead && sh.npx != 0u) mix_fetch_ahead(a, lane_pixel(g, sh, 0u), pre);
    for (uint32_t t = 0; t < sh.npx; ++t) {
        const uint32_t p = lane_pixel(g, sh, t);
        if (p != p_next) {  // a new row of the lane
            run.end(out);
            run.begin(3 * (size_t)p);
        }
        p_next = p + 1u;
        const uint32_t im = p / g.hw;
        if (im != im_now) {
            im_now = im;
            a_gr = a.coef[3 * im]; a_br = a.coef[3 * im + 1]; a_bg = a.coef[3 * im + 2];
        }
        if (ahead) {
            ok = mix_store_ahead(pre, slots) && ok;
            if (t + 1u < sh.npx) mix_fetch_ahead(a, lane_pixel(g, sh, t + 1u), pre);
        } else {
            ok = mix_load_pixel(a, p, slots) && ok;
        }
        int x_r = 0, x_g = 0, x_b = 0;
#pragma unroll 1
        for (int ch = 0; ch < 3; ++ch) {
            mix_load_channel(slots, ch, x_r, x_g, a_gr, a_br, a_bg, tab);
            const uint32_t slot = S & mask;
            // the symbol is in lo .. lo + 2 * step - 1, and c_hi = C(lo + 2 * step)
            int lo = 0;
            uint32_t c_lo = 0u, c_hi = 1u << m_bits;
#pragma unroll 1
            for (int step = 128; step >= 1; step >>= 1) {
                const uint32_t cv = mix_cum_inner(lo + step, slots, spread, tab);
                const bool ge = cv <= slot;
                lo = ge ? lo + step : lo;
                c_lo = ge ? cv : c_lo;
                c_hi = ge ? c_hi : cv;
            }
            // App. A eq. (12)
            // the mass is at most 2^16 and S >> M below 2^22: a 24-bit multiply is exact
            S = (uint32_t)__umul24(c_hi - c_lo, S >> m_bits) + slot - c_lo;
            if (S < (1u << 16)) S = (S << 16) | words.take(base, lim);
            x_b = ch == 2 ? lo : x_b;
            x_g = ch == 1 ? lo : x_g;
            x_r = ch == 0 ? lo : x_r;
        }
        run.put3(out, (uint32_t)x_r | ((uint32_t)x_g << 8) | ((uint32_t)x_b << 16));
    }
    run.end(out);
    if (!ok) atomicMax(status_code, 7);
    if (S != (1u << 16) || words.taken(first) != (end - begin) >> 1) atomicMax(status_code, 6);
}

}  // namespace pilc
