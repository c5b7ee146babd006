// Decoder for batches with few, long lanes: G threads of a wavefront own one lane (gfx950).
//
// A wavefront carries 64/G lanes side by side, all in vector registers, so that the serial
// part of a step (App. A eq. (12) of arXiv 2206.05279) costs one instruction stream for 64/G
// lanes.  Per symbol the G threads of a lane evaluate C(k) at G candidates k = base..base+G-1
// around the predicted mean; a ballot counts the candidates at or below the slot, which names
// the symbol (App. A: the x with C_x <= S mod 2^M < C_x + P_x).  Every thread also computes
// the next state as if its own candidate were the symbol, and the winner's value is fetched
// with one cross-lane read; the stream word a refill would need is fetched ahead of time.
// Values that are the same for all threads of a lane ("lane-uniform") are simply replicated.
#pragma once

#include <type_traits>

#include "pilc_device.hpp"

namespace pilc {

constexpr int kGroupWavesPerBlock = 4;

// thread i receives the value of thread i + 1 of the wavefront (thread 63 keeps 0)
__device__ __forceinline__ uint32_t from_next_thread(uint32_t v)
{
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x130 /* wave_shl:1 */, 0xF, 0xF, false);
}

// thread i of a 16-thread row receives the value of thread (i + 1) mod 16 of the same row
__device__ __forceinline__ uint32_t from_next_in_row(uint32_t v)
{
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x12F /* row_ror:15 */, 0xF, 0xF, false);
}

// G threads per lane, C candidates per thread: the window of a symbol is W = G * C values wide.
template <int G, int C>
__global__ __launch_bounds__(64 * kGroupWavesPerBlock) void k_decode_group(
    Geo g, const uint8_t *__restrict__ coded, const uint16_t *__restrict__ mu,
    const int16_t *__restrict__ ls, const int16_t *__restrict__ coef, uint8_t *__restrict__ out,
    int *__restrict__ status_code, const unsigned long long *__restrict__ status_payload)
{
    static_assert(G == 16 || G == 32 || G == 64, "threads per lane");
    static_assert(C == 1 || (C == 2 && G == 16), "two candidates per thread only with 16-thread rows");
    constexpr int L = 64 / G;
    constexpr int W = G * C;                     // candidates per symbol
    constexpr int kBaseMax = 256 - W;            // candidates stay within 1..255
    constexpr int kHalf = W / 2 - 1;             // window starts this far below the rounded mean
    constexpr int kOkLo = 256 * W - 32895;       // means for which |256 k - 128 - mean| <= 2^15
    constexpr int kOkHi = 98176 - 256 * W;       //   holds over the whole (clamped) window
    __shared__ LdsTables tab;
    load_tables(tab);
    if (*status_code != 0) return;

    const uint32_t tid = threadIdx.x & 63u;
    const uint32_t grp = tid / G, j = tid % G, gbase = grp * G;
    const uint32_t lane = (blockIdx.x * kGroupWavesPerBlock + (threadIdx.x >> 6)) * L + grp;
    const bool has_lane = lane < g.lanes;
    const LaneShape sh = lane_shape(g, has_lane ? lane : 0u);
    const uint32_t m_bits = g.prec_bits;
    const uint32_t spread = (1u << m_bits) - 256u, mask = (1u << m_bits) - 1u;
    const uint32_t payload_bytes = (uint32_t)*status_payload;
    const uint32_t *offsets = reinterpret_cast<const uint32_t *>(coded + 64);
    const uint16_t *payload =
        reinterpret_cast<const uint16_t *>(coded + 64 + 4ull * ((size_t)g.lanes + 1));

    // lane-uniform state: S, and the stream position as wbase + (widx - gbase)
    uint32_t npx = 0, stop = 0, S = 1u << 16, wbase = 0;
    if (has_lane) {
        const uint32_t begin = offsets[lane], end = offsets[lane + 1];
        if (end < begin || end > payload_bytes || end - begin < 4u || ((begin | end) & 1u)) {
            if (j == 0) atomicMax(status_code, 6);
        } else {
            npx = sh.npx;
            stop = end >> 1;
            wbase = begin >> 1;
            S = (uint32_t)payload[wbase] | ((uint32_t)payload[wbase + 1] << 16);
            wbase += 2;
        }
    }
    // the lane's next G stream words, one per thread; words past `stop` read as 0 and an
    // overrun shows at the end of the lane as a position different from `stop`
    uint32_t wbuf = wbase + j < stop ? (uint32_t)payload[wbase + j] : 0u;
    uint32_t widx = gbase;  // wavefront thread that holds the lane's next word

    // candidate edge relative to the window base: thread j holds candidates j and (C == 2) j + G
    const int d0 = 256 * (int)j - 128;

    auto bperm = [](uint32_t src_thread, uint32_t v) -> uint32_t {
        return (uint32_t)__builtin_amdgcn_ds_bpermute((int)(src_thread << 2), (int)v);
    };
    auto group_count = [&](bool pred) -> uint32_t {
        const unsigned long long m = __ballot(pred);
        if (G == 64) return (uint32_t)__popcll(m);
        if (G == 32) return (uint32_t)__popc(grp ? (uint32_t)(m >> 32) : (uint32_t)m);
        return (uint32_t)__popc((uint32_t)(m >> gbase) & 0xFFFFu);
    };
    // Window of a symbol with effective mean `me`, packed: bits 0..7 base = clamp(round(me) -
    // kHalf, 1, kBaseMax); bit 8 set when the short evaluation is NOT exact for it; bits 9..31
    // sc = 256 * base - me (signed), so that candidate j sits at d = 256 j - 128 + sc.
    auto pack_window = [](int me) -> uint32_t {
        const int base = min(max((me + (128 - 256 * kHalf)) >> 8, 1), kBaseMax);
        const uint32_t notok = (uint32_t)(me - kOkLo) > (uint32_t)(kOkHi - kOkLo) ? 0x100u : 0u;
        return ((uint32_t)((base << 8) - me) << 9) | notok | (uint32_t)base;
    };

    // One symbol of every lane of the wavefront.  `pk` is its packed window; `next(x)` gives
    // the packed window of the following symbol if this one decodes to x (evaluated by every
    // thread for its own candidate, before the slot is compared).  Returns the value; leaves the
    // winner's next window in pk_next; updates S and the stream position of lanes with `act`.
    auto decode_symbol = [&](auto ragged, bool act, uint32_t pk, uint32_t inv_s, auto next,
                             uint32_t &pk_next) -> uint32_t {
        const uint32_t slot = S & mask;
        const uint32_t wnext = bperm(widx, wbuf);  // the word a refill would consume
        int base = (int)(pk & 0xFFu);
        const int sc = (int)pk >> 9;
        // candidates of a window the short form cannot evaluate compare against 2^32 - 1: a miss
        const uint32_t slot_eff = slot | (uint32_t)((int)(pk << 23) >> 31);
        uint32_t cv[C], spec[C];
        uint32_t cnt = 0;
#pragma unroll
        for (int c = 0; c < C; ++c) {
            const int d = d0 + 256 * G * c + sc;
            // z = floor(d * inv_s / 2^17) with inv_s = a * 2^16 + b and |d| <= 2^15
            const int t = __mul24(d, (int)(inv_s & 0xFFFFu)) >> 16;
            // clamp z to [-2^20, 2^20 - 1]; the table cell is 1024 + (z >> 10), the fraction z & 1023
            const int z = min(max((__mul24(d, (int)(inv_s >> 16)) + t) >> 1, -(1 << 20)), (1 << 20) - 1);
            const uint2 cell = (tab.sig + 1024)[z >> 10];
            spec[c] = next((uint32_t)base + j + (uint32_t)(G * c));
            const uint32_t f24 = cell.x + (__umul24(cell.y, (uint32_t)z & 1023u) >> 10);
            cv[c] = (uint32_t)base + j + (uint32_t)(G * c) + scale_mass(f24, spread);
        }
#pragma unroll
        for (int c = 0; c < C; ++c) cnt += group_count(cv[c] <= slot_eff);
        bool bad = cnt - 1u >= (uint32_t)(W - 1);
        if (ragged) bad = bad && act;
        if (__builtin_expect(__any(bad), 0)) {
            // general evaluation; windows walk towards the slot: C(0) = 0 <= slot ends a walk
            // down at base 0, C(256) = 2^M > slot ends a walk up at base 257 - W.  With the narrow
            // 16-candidate window a walk can be long, so there a coarse pass comes first: the lane's
            // candidates look at every 16th value, the count of those at or below the slot names the
            // band that holds the symbol (C(0) = 0 always counts), and the walk starts at that band.
            // (Wider windows keep the plain walk: the extra code slowed their common case.)
            constexpr bool kCoarse = W == 16;
            constexpr int kBand = 256 / W;
            const int me = (base << 8) - sc;
            const bool redo = bad;
            int step = (pk & 0x100u) != 0u ? 0 : (cnt == 0u ? -(W - 1) : (W - 1));
            if (kCoarse) {
                uint32_t below = 0;
#pragma unroll
                for (int c = 0; c < C; ++c)
                    below += group_count(cum_at(kBand * ((int)j + G * c), me, inv_s, m_bits, tab) <= slot);
                if (bad) {
                    base = min(max((int)(below - 1u) * kBand, 0), 257 - W);
                    step = 0;
                }
            }
            do {
                if (bad) {
                    base = min(max(base + step, 0), 257 - W);
#pragma unroll
                    for (int c = 0; c < C; ++c)
                        cv[c] = cum_at(base + (int)j + G * c, me, inv_s, m_bits, tab);
                }
                uint32_t n = 0;
#pragma unroll
                for (int c = 0; c < C; ++c) n += group_count(redo ? cv[c] <= slot : cv[c] <= slot_eff);
                cnt = n;
                if (bad) {
                    bad = cnt - 1u >= (uint32_t)(W - 1);
                    step = cnt == 0u ? -(W - 1) : (W - 1);
                }
            } while (__any(bad));
            if (redo) {
#pragma unroll
                for (int c = 0; c < C; ++c) spec[c] = next((uint32_t)base + j + (uint32_t)(G * c));
            }
        }
        // App. A eq. (12), computed by every thread as if its own candidates were the symbol
        const uint32_t q = S >> m_bits;
        uint32_t sj, sp, winner;
        if (C == 1) {
            const uint32_t cvn = from_next_thread(cv[0]);
            sj = __umul24(cvn - cv[0], q) + (slot - cv[0]);
            sp = spec[0];
            winner = gbase + cnt - 1u;
        } else {
            // candidate j + G follows candidate j of the row's next thread; candidate G follows G - 1
            const uint32_t n0 = from_next_in_row(cv[0]), n1 = from_next_in_row(cv[C - 1]);
            const uint32_t cvn0 = j == (uint32_t)(G - 1) ? n1 : n0;
            const uint32_t s0 = __umul24(cvn0 - cv[0], q) + (slot - cv[0]);
            const uint32_t s1 = __umul24(n1 - cv[C - 1], q) + (slot - cv[C - 1]);
            const bool upper = cnt > (uint32_t)G;  // the symbol is one of the second candidates
            sj = upper ? s1 : s0;
            sp = upper ? spec[C - 1] : spec[0];
            winner = gbase + ((cnt - 1u) & (uint32_t)(G - 1));
        }
        uint32_t s_new = bperm(winner, sj);
        pk_next = bperm(winner, sp);
        const bool refill = s_new < (1u << 16);
        s_new = refill ? (s_new << 16) | wnext : s_new;
        if (ragged) {
            S = act ? s_new : S;
            widx += (act && refill) ? 1u : 0u;
        } else {
            S = s_new;
            widx += refill ? 1u : 0u;
        }
        return (uint32_t)base + cnt - 1u;
    };

    for (uint32_t t0 = 0; __any(t0 < npx); t0 += G) {
        const uint32_t nb = t0 < npx ? min((uint32_t)G, npx - t0) : 0u;
        // ---- thread j prepares pixel t0 + j of its lane ----
        const bool valid = j < nb;
        const uint32_t p = lane_pixel(g, sh, valid ? t0 + j : 0u);
        const size_t s = (size_t)p * 3;
        const uint32_t im = p / g.hw;
        const uint32_t v_m01 = (uint32_t)mu[s] | ((uint32_t)mu[s + 1] << 16);
        const uint32_t v_mba = (uint32_t)mu[s + 2] | ((uint32_t)(uint16_t)coef[3 * im + 2] << 16);
        const uint32_t v_a01 =
            (uint32_t)(uint16_t)coef[3 * im] | ((uint32_t)(uint16_t)coef[3 * im + 1] << 16);
        const uint32_t v_pkr = pack_window((int)mu[s]);
        const uint32_t v_i0 = inv_scale(ls[s], tab);
        const uint32_t v_i1 = inv_scale(ls[s + 1], tab);
        const uint32_t v_i2 = inv_scale(ls[s + 2], tab);
        uint32_t v_out = 0;

        auto pixels = [&](auto ragged) {
            for (uint32_t i = 0; ragged ? __any(i < nb) : i < (uint32_t)G; ++i) {
                const bool act = i < nb;
                const uint32_t src = gbase + i;
                const uint32_t m01 = bperm(src, v_m01), mba = bperm(src, v_mba), a01 = bperm(src, v_a01);
                const uint32_t pk_r = bperm(src, v_pkr);
                const uint32_t i0 = bperm(src, v_i0), i1 = bperm(src, v_i1), i2 = bperm(src, v_i2);
                const int m_r = (int)(m01 & 0xFFFFu), m_g = (int)(m01 >> 16), m_b = (int)(mba & 0xFFFFu);
                const int a_gr = (int)(short)(a01 & 0xFFFFu), a_br = (int)a01 >> 16, a_bg = (int)mba >> 16;
                // keep three words of the stream in the buffer for this pixel
                if ((!ragged || act) && widx - gbase + 3u > (uint32_t)G) {
                    wbase += widx - gbase;
                    widx = gbase;
                    wbuf = wbase + j < stop ? (uint32_t)payload[wbase + j] : 0u;
                }
                uint32_t pk_g, pk_b, unused;
                const uint32_t x_r = decode_symbol(ragged, act, pk_r, i0, [&](uint32_t x) {
                    return pack_window(m_g + rsh14_mul(a_gr, ((int)(x << 8) - m_r)));
                }, pk_g);
                const int mb1 = m_b + rsh14_mul(a_br, ((int)(x_r << 8) - m_r));
                const uint32_t x_g = decode_symbol(ragged, act, pk_g, i1, [&](uint32_t x) {
                    return pack_window(mb1 + rsh14_mul(a_bg, ((int)(x << 8) - m_g)));
                }, pk_b);
                const uint32_t x_b = decode_symbol(ragged, act, pk_b, i2, [](uint32_t) { return 0u; }, unused);
                v_out = j == i ? (x_r | (x_g << 8) | (x_b << 16)) : v_out;
            }
        };
        if (__all(nb == (uint32_t)G))
            pixels(std::false_type{});
        else
            pixels(std::true_type{});
        if (valid) {
            out[s] = (uint8_t)v_out;
            out[s + 1] = (uint8_t)(v_out >> 8);
            out[s + 2] = (uint8_t)(v_out >> 16);
        }
    }
    if (has_lane && npx != 0u && (S != (1u << 16) || wbase + (widx - gbase) != stop) && j == 0)
        atomicMax(status_code, 6);
}

}  // namespace pilc
