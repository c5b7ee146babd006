// rANS lanes under a mixture of K logistic laws per subpixel, one thread per lane (gfx950).
//
// Sec. 2 of arXiv 2206.05279 names this workload (a dynamic rANS coder fed a mixture of ten
// logistic laws per symbol) as what holds earlier learned codecs near 1 MB/s; the coder itself is
// App. A eqs. (11)-(12).  A pixel has K weights (Q0.15, summing to 2^15), a subpixel K means and
// K log-scales.  The mixed 24-bit edge CDF is F(k) = floor(sum_j w_j F_j(k) / 2^15) with F_j the
// single-law edge CDF, and C(k) = k + floor(F(k) (2^M - 256) / 2^24); the channel conditioning
// of Sec. 3.1 eqs. (3)-(4) shifts every component's mean with that component's own innovations.
//
// In the general kernels K is a run-time value, so nothing per component lives in registers (the
// kernels built for one K keep the channel's components and the pixel's weights there; they are
// the same kernels with the component count as a template argument).  A thread first copies
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
// weights (K), each rounded up to dwords, as [dword][thread].  The kernels built for one K have
// neither the pairs nor the weights there.
constexpr uint32_t kMixImageBlock = 32;   // bytes of the image a thread of the encoder keeps in LDS
constexpr uint32_t kMixWeightBlock = 64;  // bytes of the weights a thread keeps there (kernels built for one K)

struct MixSlots {
    uint2 *pairs;    // this thread's column of the pairs
    uint32_t *base;  // this thread's column of the raw parameters
    uint32_t k, stride, raw_ls, raw_w, image_block, weight_block;
    static constexpr uint32_t raw_mu = 0u;
    __device__ __forceinline__ MixSlots(uint32_t *lds, uint32_t k_, bool with_pairs = true)
        : pairs(reinterpret_cast<uint2 *>(lds) + threadIdx.x),
          base(lds + (with_pairs ? 2u * k_ * blockDim.x : 0u) + threadIdx.x), k(k_), stride(blockDim.x),
          raw_ls((3u * k_ + 1u) / 2u), raw_w(2u * ((3u * k_ + 1u) / 2u)),
          image_block(2u * ((3u * k_ + 1u) / 2u) + (with_pairs ? (k_ + 1u) / 2u : 0u)),
          weight_block(image_block + kMixImageBlock / 4u)
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

// with_pairs false: the kernels built for one K, which keep the pairs and the weights in registers.
// The blocks of image bytes and of weights are the encoder's (the decoder's columns have them too,
// unused: one layout for both).
static inline size_t mix_lds_bytes(uint32_t k, bool with_pairs)
{
    return (size_t)kMixThreads * 4u *
           ((with_pairs ? 2u * k + (k + 1u) / 2u : kMixWeightBlock / 4u) + 2u * ((3u * k + 1u) / 2u) +
            kMixImageBlock / 4u);
}

// An aligned block of kBytes of global memory in a thread's LDS column ([dword][thread]), loaded
// when an address outside it is asked for.  With the lines long gone from the L2 when a lane
// reaches its next pixel, every separate load costs a fetch of its whole 128-byte line; through a
// block a line is asked for 128 / kBytes times instead of once per pixel.  A block that holds a
// byte of an array lies inside the array's pages even where it reaches past its ends.
template <uint32_t kBytes> struct LdsBlock {
    uint32_t *col;
    uint32_t stride;
    uintptr_t tag;  // address of the block held; 1: none
    __device__ __forceinline__ LdsBlock(uint32_t *column, uint32_t stride_) : col(column), stride(stride_), tag(1u) {}
    __device__ __forceinline__ uint32_t dword(uintptr_t at)  // the aligned dword that holds byte `at`
    {
        const uintptr_t blk = at & ~(uintptr_t)(kBytes - 1u);
        if (blk != tag) {
            const uint4 *src = reinterpret_cast<const uint4 *>(blk);
            uint4 v[kBytes / 16u];
#pragma unroll
            for (uint32_t i = 0; i < kBytes / 16u; ++i) v[i] = src[i];
#pragma unroll
            for (uint32_t i = 0; i < kBytes / 16u; ++i) {
                col[(4u * i) * stride] = v[i].x;
                col[(4u * i + 1u) * stride] = v[i].y;
                col[(4u * i + 2u) * stride] = v[i].z;
                col[(4u * i + 3u) * stride] = v[i].w;
            }
            tag = blk;
        }
        return col[(((uint32_t)at & (kBytes - 1u)) >> 2) * stride];
    }
};

// The encoder's image bytes.
struct PixelBytes {
    LdsBlock<kMixImageBlock> block;
    __device__ __forceinline__ PixelBytes(const MixSlots &s) : block(s.base + s.image_block * s.stride, s.stride) {}
    __device__ __forceinline__ uint32_t byte(const uint8_t *a)
    {
        const uintptr_t at = reinterpret_cast<uintptr_t>(a);
        return (block.dword(at) >> (8u * ((uint32_t)at & 3u))) & 0xFFu;
    }
    // R | G << 8 | B << 16 of pixel q, highest address first: the encoder walks its lane backwards
    __device__ __forceinline__ uint32_t pixel(const uint8_t *img, uint32_t q)
    {
        const uint8_t *a = img + 3 * (size_t)q;
        const uint32_t b = byte(a + 2), g = byte(a + 1), r = byte(a);
        return r | (g << 8) | (b << 16);
    }
};

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

// Dword-aligned arrays: a pixel's raw parameters lie in ceil(3 K / 2) + ceil(3 K / 2) + ceil(K / 2)
// aligned dwords (for odd K the blocks of every other pixel start on the upper half of a dword and
// end on a lower half: the same number of dwords, one halfword of a neighbour at either end), and
// the kernels keep the NEXT pixel's dwords in registers while they work on the current one, so that
// the loads have a pixel's worth of arithmetic to arrive in.
// kK is the component count a kernel was built for, 0 for the kernels that take it at run time
// (those run ahead for even K only).
template <int kK> struct MixAhead {
    static constexpr int kComp = kK > 0 ? kK : kMixMaxComp;
    static constexpr int kMu = (3 * kComp + 1) / 2, kW = (kComp + 1) / 2;
    uint32_t m[kMu], l[kMu], w[kW];
};

// The components of the channel being coded, in registers: only in the kernels built for one K,
// where every index into these arrays is a compile-time constant.
template <int kK> struct MixRegs {
    int c0[kK > 0 ? kK : 1];          // edge_offset of the shifted mean
    uint32_t inv_s[kK > 0 ? kK : 1];  // 1 / scale
    uint32_t w[kK > 0 ? kK : 1];      // the pixel's weights
};

__device__ __forceinline__ bool mix_can_run_ahead(const MixArgs &a)
{
    return (a.k & 1u) == 0u && ((reinterpret_cast<uintptr_t>(a.mu) | reinterpret_cast<uintptr_t>(a.ls) |
                                 reinterpret_cast<uintptr_t>(a.weight)) & 3u) == 0u;
}

// kWeights false: the weights come some other way (the encoder built for one K has an LdsBlock).
template <int kK, bool kWeights = true>
__device__ __forceinline__ void mix_fetch_ahead(const MixArgs &a, uint32_t p, MixAhead<kK> &r)
{
    const uint32_t k = kK > 0 ? (uint32_t)kK : a.k;
    const size_t px = (size_t)p * 3u * k;  // in halfwords: the aligned dwords from px / 2 on
    const uint32_t *gm = reinterpret_cast<const uint32_t *>(a.mu) + (px >> 1);
    const uint32_t *gl = reinterpret_cast<const uint32_t *>(a.ls) + (px >> 1);
    const uint32_t *gw = reinterpret_cast<const uint32_t *>(a.weight) + (((size_t)p * k) >> 1);
    const uint32_t n3 = (3u * k + 1u) / 2u, n1 = (k + 1u) / 2u;
#pragma unroll
    for (int i = 0; i < MixAhead<kK>::kMu; ++i)
        if ((uint32_t)i < n3) r.m[i] = gm[i];
#pragma unroll
    for (int i = 0; i < MixAhead<kK>::kMu; ++i)
        if ((uint32_t)i < n3) r.l[i] = gl[i];
    if constexpr (kWeights) {
#pragma unroll
        for (int i = 0; i < MixAhead<kK>::kW; ++i)
            if ((uint32_t)i < n1) r.w[i] = gw[i];
    }
}

// The weights of pixel p into `regs`, through the thread's block (dword-aligned array), highest
// address first: the encoder walks its lane backwards.  False if they do not sum to 2^15.
template <int kK>
__device__ __forceinline__ bool mix_load_weights(const MixArgs &a, uint32_t p, LdsBlock<kMixWeightBlock> &block,
                                                 MixRegs<kK> &regs)
{
    const uintptr_t at = reinterpret_cast<uintptr_t>(a.weight + (size_t)p * kK);
    uint32_t sum = 0;
    if constexpr (kK % 2 == 0) {
#pragma unroll
        for (int i = kK / 2 - 1; i >= 0; --i) {
            const uint32_t w2 = block.dword(at + 4u * i);
            regs.w[2 * i] = w2 & 0xFFFFu;
            regs.w[2 * i + 1] = w2 >> 16;
        }
    } else {  // a halfword at a time: the pixel's weights start on either half of a dword
#pragma unroll
        for (int j = kK - 1; j >= 0; --j) {
            const uintptr_t b = at + 2u * j;
            const uint32_t w2 = block.dword(b);
            regs.w[j] = (b & 2u) ? w2 >> 16 : w2 & 0xFFFFu;
        }
    }
#pragma unroll
    for (int j = 0; j < kK; ++j) sum += regs.w[j];
    return sum == (1u << 15);
}

// The fetched pixel into the slots, its weights into `regs` in the kernels built for one K; false
// if the weights do not sum to 2^15.  kWeights as above (then true).  `upper`: the pixel's blocks
// start on the upper half of the first dword fetched (odd K, every other pixel) and are moved down
// by a halfword on the way.
template <int kK, bool kWeights = true>
__device__ __forceinline__ bool mix_store_ahead(const MixAhead<kK> &r, const MixSlots &s, MixRegs<kK> &regs,
                                                bool upper)
{
    constexpr bool kOdd = kK % 2 != 0;
    const uint32_t n3 = (3u * s.k + 1u) / 2u, n1 = (s.k + 1u) / 2u;
    auto lowered = [&](const uint32_t *d, int i, int n) {  // dword i of the block, from the n fetched
        if constexpr (!kOdd) return d[i];
        const uint32_t next = i + 1 < n ? d[i + 1] : 0u;
        return upper ? __builtin_amdgcn_alignbit(next, d[i], 16) : d[i];
    };
    uint32_t sum = 0;
#pragma unroll
    for (int i = 0; i < MixAhead<kK>::kMu; ++i)
        if ((uint32_t)i < n3) s.dword(s.raw_mu + i) = lowered(r.m, i, MixAhead<kK>::kMu);
#pragma unroll
    for (int i = 0; i < MixAhead<kK>::kMu; ++i)
        if ((uint32_t)i < n3) s.dword(s.raw_ls + i) = lowered(r.l, i, MixAhead<kK>::kMu);
    if constexpr (!kWeights) return true;
#pragma unroll
    for (int i = 0; i < MixAhead<kK>::kW; ++i)
        if ((uint32_t)i < n1) {
            const uint32_t w2 = lowered(r.w, i, MixAhead<kK>::kW);
            if constexpr (kK > 0) {
                regs.w[2 * i] = w2 & 0xFFFFu;
                sum += w2 & 0xFFFFu;
                if (2 * i + 1 < kK) {
                    regs.w[2 * i + 1] = w2 >> 16;
                    sum += w2 >> 16;
                }
            } else {
                s.dword(s.raw_w + i) = w2;
                sum += (w2 & 0xFFFFu) + (w2 >> 16);
            }
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

// The same into registers, two components (one dword of each raw array) at a time.
template <int kK>
__device__ __forceinline__ void mix_load_channel(const MixSlots &s, MixRegs<kK> &regs, int ch, int x_r,
                                                 int x_g, int a_gr, int a_br, int a_bg, const LdsTables &tab)
{
    static_assert(kK > 0, "built for one component count");
    if constexpr (kK % 2 != 0) {  // a channel's block starts on either half of a dword: halfword reads
#pragma unroll
        for (int j = 0; j < kK; ++j) {
            int me = (int)s.half(s.raw_mu, (uint32_t)ch * kK + j);
            if (ch >= 1) {
                const int e_r = x_r * 256 - (int)s.half(s.raw_mu, j);
                if (ch == 1)
                    me += rsh14_mul(a_gr, e_r);
                else
                    me += rsh14_mul(a_br, e_r) + rsh14_mul(a_bg, x_g * 256 - (int)s.half(s.raw_mu, kK + j));
            }
            regs.c0[j] = edge_offset(me);
            regs.inv_s[j] = inv_scale((int)(short)s.half(s.raw_ls, (uint32_t)ch * kK + j), tab);
        }
        return;
    }
    const uint32_t *mu_r = s.base + s.raw_mu * s.stride;
    const uint32_t *mu_g = mu_r + (kK / 2) * s.stride;
    const uint32_t *mu_c = mu_r + (uint32_t)ch * (kK / 2) * s.stride;
    const uint32_t *ls_c = s.base + (s.raw_ls + (uint32_t)ch * (kK / 2)) * s.stride;
#pragma unroll
    for (int jj = 0; jj < kK / 2; ++jj) {
        const uint32_t m2 = mu_c[jj * s.stride], l2 = ls_c[jj * s.stride];
        int me[2] = {(int)(m2 & 0xFFFFu), (int)(m2 >> 16)};
        if (ch >= 1) {
            const uint32_t r2 = mu_r[jj * s.stride];
            const int e_r[2] = {x_r * 256 - (int)(r2 & 0xFFFFu), x_r * 256 - (int)(r2 >> 16)};
            if (ch == 1) {
                me[0] += rsh14_mul(a_gr, e_r[0]);
                me[1] += rsh14_mul(a_gr, e_r[1]);
            } else {
                const uint32_t g2 = mu_g[jj * s.stride];
                me[0] += rsh14_mul(a_br, e_r[0]) + rsh14_mul(a_bg, x_g * 256 - (int)(g2 & 0xFFFFu));
                me[1] += rsh14_mul(a_br, e_r[1]) + rsh14_mul(a_bg, x_g * 256 - (int)(g2 >> 16));
            }
        }
        regs.c0[2 * jj] = edge_offset(me[0]);
        regs.c0[2 * jj + 1] = edge_offset(me[1]);
        regs.inv_s[2 * jj] = inv_scale((int)(short)(l2 & 0xFFFFu), tab);
        regs.inv_s[2 * jj + 1] = inv_scale((int)(short)(l2 >> 16), tab);
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

// C(k), 1 <= k <= 255, from the registers: all kK table reads are in flight together.
template <int kK>
__device__ __forceinline__ uint32_t mix_cum_inner(int k, const MixRegs<kK> &regs, uint32_t spread,
                                                  const LdsTables &tab)
{
    unsigned long long acc = 0ull;
#pragma unroll
    for (int j = 0; j < kK; ++j)
        acc += (unsigned long long)regs.w[j] * edge_cdf(256 * k + regs.c0[j], regs.inv_s[j], tab);
    return (uint32_t)k + scale_mass((uint32_t)(acc >> 15), spread);
}

// kK > 0: built for that many components (even, dword-aligned arrays: the host checks), which then
// live in registers; kK == 0: any K, components in LDS.
template <int kK>
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
    const MixSlots slots(mix_lds, kK > 0 ? (uint32_t)kK : a.k, kK == 0);
    const LaneShape sh = lane_shape(g, lane);
    const uint32_t m_bits = g.prec_bits;
    const uint32_t spread = (1u << m_bits) - 256u, top = 1u << m_bits;

    uint16_t *wout = scratch + lane_scratch_base(lane, lane_cap);
    uint32_t nwords = 0, S = 1u << 16;
    bool ok = true;
    // pixels last-first, and B, G, R inside a pixel (App. A eq. (11) runs against the decoder)
    const bool ahead = kK > 0 || mix_can_run_ahead(a);
    MixAhead<kK> pre;
    MixRegs<kK> regs;
    PixelBytes bytes(slots);
    LdsBlock<kMixWeightBlock> weights(slots.base + slots.weight_block * slots.stride, slots.stride);
    uint32_t im_now = 0xFFFFFFFFu;
    int a_gr = 0, a_br = 0, a_bg = 0;
    // built for one K: the weights reach the registers through a block in LDS, which costs a wait
    // when the block runs out and saves most of their traffic (the decoder, bound by its
    // arithmetic, keeps fetching them ahead with the other parameters)
    constexpr bool kAheadW = kK == 0;
    if (ahead && sh.npx != 0u) mix_fetch_ahead<kK, kAheadW>(a, lane_pixel(g, sh, sh.npx - 1u), pre);
    for (uint32_t t = sh.npx; t-- > 0u;) {
        const uint32_t p = lane_pixel(g, sh, t);
        const uint32_t im = g.by_hw.div(p);
        if (im != im_now) {
            im_now = im;
            a_gr = a.coef[3 * im]; a_br = a.coef[3 * im + 1]; a_bg = a.coef[3 * im + 2];
        }
        if (ahead) {
            ok = mix_store_ahead<kK, kAheadW>(pre, slots, regs, (kK & 1) != 0 && (p & 1u) != 0u) && ok;
            if constexpr (!kAheadW) ok = mix_load_weights<kK>(a, p, weights, regs) && ok;
            if (t != 0u) mix_fetch_ahead<kK, kAheadW>(a, lane_pixel(g, sh, t - 1u), pre);
        } else {
            ok = mix_load_pixel(a, p, slots) && ok;
        }
        const uint32_t xb = bytes.pixel(img, p);
        const int x[3] = {(int)(xb & 0xFFu), (int)((xb >> 8) & 0xFFu), (int)(xb >> 16)};
#pragma unroll 1
        for (int ch = 2; ch >= 0; --ch) {
            const int v = ch == 0 ? x[0] : (ch == 1 ? x[1] : x[2]);
            uint32_t lo, hi;
            if constexpr (kK > 0) {
                mix_load_channel(slots, regs, ch, x[0], x[1], a_gr, a_br, a_bg, tab);
                lo = v == 0 ? 0u : mix_cum_inner(v, regs, spread, tab);
                hi = v == 255 ? top : mix_cum_inner(v + 1, regs, spread, tab);
            } else {
                mix_load_channel(slots, ch, x[0], x[1], a_gr, a_br, a_bg, tab);
                lo = v == 0 ? 0u : mix_cum_inner(v, slots, spread, tab);
                hi = v == 255 ? top : mix_cum_inner(v + 1, slots, spread, tab);
            }
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

template <int kK>  // as k_mix_encode
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
    const MixSlots slots(mix_lds, kK > 0 ? (uint32_t)kK : a.k, kK == 0);
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
    const bool ahead = kK > 0 || mix_can_run_ahead(a);
    MixAhead<kK> pre;
    MixRegs<kK> regs;
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
        const uint32_t im = g.by_hw.div(p);
        if (im != im_now) {
            im_now = im;
            a_gr = a.coef[3 * im]; a_br = a.coef[3 * im + 1]; a_bg = a.coef[3 * im + 2];
        }
        if (ahead) {
            ok = mix_store_ahead(pre, slots, regs, (kK & 1) != 0 && (p & 1u) != 0u) && ok;
            if (t + 1u < sh.npx) mix_fetch_ahead(a, lane_pixel(g, sh, t + 1u), pre);
        } else {
            ok = mix_load_pixel(a, p, slots) && ok;
        }
        int x_r = 0, x_g = 0, x_b = 0;
#pragma unroll 1
        for (int ch = 0; ch < 3; ++ch) {
            if constexpr (kK > 0)
                mix_load_channel(slots, regs, ch, x_r, x_g, a_gr, a_br, a_bg, tab);
            else
                mix_load_channel(slots, ch, x_r, x_g, a_gr, a_br, a_bg, tab);
            const uint32_t slot = S & mask;
            // the symbol is in lo .. lo + 2 * step - 1, and c_hi = C(lo + 2 * step)
            int lo = 0;
            uint32_t c_lo = 0u, c_hi = 1u << m_bits;
#pragma unroll 1
            for (int step = 128; step >= 1; step >>= 1) {
                uint32_t cv;
                if constexpr (kK > 0)
                    cv = mix_cum_inner(lo + step, regs, spread, tab);
                else
                    cv = mix_cum_inner(lo + step, slots, spread, tab);
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
