// rANS lanes under a mixture of K logistic laws per subpixel, one thread per lane (gfx950).
//
// Sec. 2 of arXiv 2206.05279 names this workload (a dynamic rANS coder fed "a distribution mixed
// by 10 logistic ones") as what holds earlier learned codecs near 1 MB/s; the coder itself is
// App. A eqs. (11)-(12).  A pixel has K weights (Q0.15, summing to 2^15), a subpixel K means and
// K log-scales.  The mixed 24-bit edge CDF is F(k) = floor(sum_j w_j F_j(k) / 2^15) with F_j the
// single-law edge CDF, and C(k) = k + floor(F(k) (2^M - 256) / 2^24); the channel conditioning
// of Sec. 3.1 eqs. (3)-(4) shifts every component's mean with that component's own innovations.
//
// K is a run-time value, so nothing per component lives in registers: before a subpixel is coded
// the thread puts {shifted mean, 1/scale} and the weight of every component in its own LDS slots
// ([component][thread], so a wavefront's accesses are conflict free), and every evaluation of
// C(k) walks them.  The 16-bit words go through the thread-per-lane scratch layout and packer.
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

// Dynamic LDS of the mixture kernels: per component and thread a {mean, 1/scale} pair and a weight.
struct MixSlots {
    uint2 *pair;       // [K][blockDim.x]
    uint32_t *weight;  // [K][blockDim.x]
    __device__ __forceinline__ MixSlots(uint8_t *raw, uint32_t k)
        : pair(reinterpret_cast<uint2 *>(raw) + threadIdx.x),
          weight(reinterpret_cast<uint32_t *>(raw + (size_t)k * blockDim.x * sizeof(uint2)) + threadIdx.x)
    {
    }
};

static inline size_t mix_lds_bytes(uint32_t k) { return (size_t)k * kMixThreads * (sizeof(uint2) + 4); }

// The pixel's weights into the slots; false if they do not sum to 2^15.
__device__ __forceinline__ bool mix_load_weights(const MixArgs &a, uint32_t p, const MixSlots &s)
{
    uint32_t sum = 0;
    for (uint32_t j = 0; j < a.k; ++j) {
        const uint32_t w = a.weight[(size_t)p * a.k + j];
        s.weight[j * blockDim.x] = w;
        sum += w;
    }
    return sum == (1u << 15);
}

// {shifted mean, 1/scale} of every component of channel `ch` of pixel p into the slots; x_r and
// x_g are the pixel's red and green values (used for ch >= 1 and ch == 2).
__device__ __forceinline__ void mix_load_channel(const MixArgs &a, uint32_t p, int ch, int x_r, int x_g,
                                                 int a_gr, int a_br, int a_bg, const MixSlots &s,
                                                 const LdsTables &tab)
{
    const size_t px = (size_t)p * 3u * a.k;
    for (uint32_t j = 0; j < a.k; ++j) {
        int me = a.mu[px + (size_t)ch * a.k + j];
        if (ch >= 1) {
            const int e_r = x_r * 256 - (int)a.mu[px + j];
            if (ch == 1) {
                me += rsh14(a_gr * e_r);
            } else {
                const int e_g = x_g * 256 - (int)a.mu[px + a.k + j];
                me += rsh14(a_br * e_r) + rsh14(a_bg * e_g);
            }
        }
        const uint32_t inv_s = inv_scale(a.ls[px + (size_t)ch * a.k + j], tab);
        s.pair[j * blockDim.x] = make_uint2((uint32_t)me, inv_s);
    }
}

// C(k), 1 <= k <= 255, from the slots.
__device__ __forceinline__ uint32_t mix_cum_inner(int k, uint32_t ncomp, const MixSlots &s,
                                                  uint32_t spread, const LdsTables &tab)
{
    unsigned long long acc = 0ull;
    for (uint32_t j = 0; j < ncomp; ++j) {
        const uint2 c = s.pair[j * blockDim.x];
        const uint32_t w = s.weight[j * blockDim.x];
        acc += (unsigned long long)w * edge_cdf(256 * k + (-128 - (int)c.x), c.y, tab);
    }
    return (uint32_t)k + scale_mass((uint32_t)(acc >> 15), spread);
}

__global__ __launch_bounds__(kMixThreads) void k_mix_encode(
    Geo g, const uint8_t *__restrict__ img, MixArgs a, uint16_t *__restrict__ scratch,
    uint32_t lane_cap, uint32_t *__restrict__ lane_words, uint32_t *__restrict__ lane_state,
    int *__restrict__ status_code)
{
    __shared__ LdsTables tab;
    extern __shared__ __align__(16) uint8_t mix_lds[];
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
    for (uint32_t t = sh.npx; t-- > 0u;) {
        const uint32_t p = lane_pixel(g, sh, t);
        const uint32_t im = p / g.hw;
        const int a_gr = a.coef[3 * im], a_br = a.coef[3 * im + 1], a_bg = a.coef[3 * im + 2];
        const int x[3] = {img[3 * (size_t)p], img[3 * (size_t)p + 1], img[3 * (size_t)p + 2]};
        ok = mix_load_weights(a, p, slots) && ok;
#pragma unroll 1
        for (int ch = 2; ch >= 0; --ch) {
            mix_load_channel(a, p, ch, x[0], x[1], a_gr, a_br, a_bg, slots, tab);
            const int v = ch == 0 ? x[0] : (ch == 1 ? x[1] : x[2]);
            const uint32_t lo = v == 0 ? 0u : mix_cum_inner(v, a.k, slots, spread, tab);
            const uint32_t hi = v == 255 ? top : mix_cum_inner(v + 1, a.k, slots, spread, tab);
            const uint32_t f = hi - lo;
            if (S >= (f << (32u - m_bits))) {
                *wout = (uint16_t)(S & 0xFFFFu);
                wout += 64;
                ++nwords;
                S >>= 16;
            }
            uint32_t rem;
            const uint32_t q = div_small(S, f, __builtin_amdgcn_rcpf((float)f), rem);
            S = (q << m_bits) + rem + lo;
        }
    }
    if (!ok) atomicMax(status_code, 7);
    lane_words[lane] = nwords;
    lane_state[lane] = S;
}

__global__ __launch_bounds__(kMixThreads) void k_mix_decode(
    Geo g, const uint8_t *__restrict__ coded, MixArgs a, uint8_t *__restrict__ out,
    int *__restrict__ status_code, const unsigned long long *__restrict__ status_payload)
{
    __shared__ LdsTables tab;
    extern __shared__ __align__(16) uint8_t mix_lds[];
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
    for (uint32_t t = 0; t < sh.npx; ++t) {
        const uint32_t p = lane_pixel(g, sh, t);
        const uint32_t im = p / g.hw;
        const int a_gr = a.coef[3 * im], a_br = a.coef[3 * im + 1], a_bg = a.coef[3 * im + 2];
        ok = mix_load_weights(a, p, slots) && ok;
        int x_r = 0, x_g = 0;
#pragma unroll 1
        for (int ch = 0; ch < 3; ++ch) {
            mix_load_channel(a, p, ch, x_r, x_g, a_gr, a_br, a_bg, slots, tab);
            const uint32_t slot = S & mask;
            // the symbol is in lo .. lo + 2 * step - 1, and c_hi = C(lo + 2 * step)
            int lo = 0;
            uint32_t c_lo = 0u, c_hi = 1u << m_bits;
#pragma unroll 1
            for (int step = 128; step >= 1; step >>= 1) {
                const uint32_t cv = mix_cum_inner(lo + step, a.k, slots, spread, tab);
                const bool ge = cv <= slot;
                lo = ge ? lo + step : lo;
                c_lo = ge ? cv : c_lo;
                c_hi = ge ? c_hi : cv;
            }
            // App. A eq. (12)
            S = (c_hi - c_lo) * (S >> m_bits) + slot - c_lo;
            if (S < (1u << 16)) S = (S << 16) | words.take(base, lim);
            out[3 * (size_t)p + ch] = (uint8_t)lo;
            x_g = ch == 1 ? lo : x_g;
            x_r = ch == 0 ? lo : x_r;
        }
    }
    if (!ok) atomicMax(status_code, 7);
    if (S != (1u << 16) || words.taken(first) != (end - begin) >> 1) atomicMax(status_code, 6);
}

}  // namespace pilc
