// Workgroup-cooperative encoder for batches with few, long lanes (gfx950).
//
// The rANS push (App. A eq. (11) of arXiv 2206.05279) is a serial chain per lane, but only
// the state update itself is serial: the symbol's (cum, freq) and an exact reciprocal of freq
// do not depend on the state.  A workgroup owns 16 lanes.  Wave 0 keeps the 16 states, one per
// thread, and does nothing but the chain; the other seven waves run ahead by one batch of 28
// pixels per lane (one pixel per thread) and leave, per symbol, one ready-made 16-byte record in
// LDS (see
// encode_record).  One barrier per batch hands a buffer over; the two roles never wait for each
// other inside a batch.  The chain is branch-free: a word is stored on every step, below the
// lane's words so far, and counted only when the state renormalises.
#pragma once

#include "pilc_device.hpp"

namespace pilc {

constexpr int kEncLanes = 16;             // lanes per workgroup (threads 0..15 of wave 0 chain)
constexpr int kEncProducerWaves = 7;      // waves 1..7 prepare records
constexpr int kEncThreads = 64 * (1 + kEncProducerWaves);
constexpr int kEncPix = 64 * kEncProducerWaves / kEncLanes;  // pixels per lane and batch (28)
constexpr int kEncSyms = 3 * kEncPix;

// floor(2^32 * a / f) for a < f < 2^17, by two 16-bit digits of long division
__device__ __forceinline__ uint32_t frac32(uint32_t a, uint32_t f)
{
    uint32_t n1 = a << 16;
    uint32_t q1 = n1 / f;
    uint32_t r1 = n1 - q1 * f;
    uint32_t q0 = (r1 << 16) / f;
    return (q1 << 16) | q0;
}

// v >> (top byte of w): one instruction that takes its shift count from byte 3 of a register
__device__ __forceinline__ uint32_t shift_right_by_top_byte(uint32_t v, uint32_t w)
{
    uint32_t r;
    asm("v_lshrrev_b32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:BYTE_3 src1_sel:DWORD"
        : "=v"(r)
        : "v"(w), "v"(v));
    return r;
}

// Record of one symbol for the chain: { T, m, add, k | sh << 24 } such that one step is
//     if (S > T) { emit low 16 bits; S >>= 16; }
//     t = mulhi(m, S);  q = (t + ((S - t) >> 1)) >> sh;  S = S + add + q * k.
// For f >= 2 this is App. A eq. (11) with the division by f done by multiplication (Granlund &
// Montgomery, round-up method, l = ceil(log2 f), m = floor(2^32 (2^l - f) / f) + 1, sh = l - 1):
// T = (f << (32-M)) - 1, add = cum, k = 2^M - f, since (q << M) + (S - q f) + cum = S + cum + q k.
// For f = 1 the same formula with m = 2^32 - 1, sh = 0 yields q = S - 1, so add = cum + 2^M - 1
// makes up for the missing k.  An all-identity record (T = 2^32 - 1, add = k = 0) skips a slot.
// k and sh share a word without any unpacking: the 24-bit multiply looks at the low 24 bits only,
// and the shift takes its count from the top byte.
__device__ __forceinline__ uint4 encode_record(uint32_t cum, uint32_t f, uint32_t m_bits)
{
    const uint32_t k = (1u << m_bits) - f;
    if (f == 1u) return make_uint4((1u << (32u - m_bits)) - 1u, 0xFFFFFFFFu, cum + k, k);
    const uint32_t l = 32u - (uint32_t)__clz(f - 1u);
    const uint32_t magic = frac32((1u << l) - f, f) + 1u;
    return make_uint4((f << (32u - m_bits)) - 1u, magic, cum, k | ((l - 1u) << 24));
}

__global__ __launch_bounds__(kEncThreads) void k_encode_block(
    Geo g, const uint8_t *__restrict__ img, const uint16_t *__restrict__ mu,
    const int16_t *__restrict__ ls, const int16_t *__restrict__ coef, uint16_t *__restrict__ scratch,
    uint32_t *__restrict__ lane_words, uint32_t *__restrict__ lane_state)
{
    __shared__ LdsTables tab;
    __shared__ uint4 rec[2][kEncSyms][kEncLanes];
    __shared__ uint32_t s_max_px;
    if (threadIdx.x == 0) s_max_px = 0;
    load_tables(tab);  // ends with a barrier

    const uint32_t tid = threadIdx.x;
    const uint32_t lane0 = blockIdx.x * kEncLanes;
    const uint32_t nl = min((uint32_t)kEncLanes, g.lanes - lane0);
    const uint32_t m_bits = g.prec_bits;
    const uint32_t spread = (1u << m_bits) - 256u, top = 1u << m_bits;

    const bool producer = tid >= 64u;
    const uint32_t q = tid - 64u;
    const uint32_t my = producer ? q / kEncPix : tid;  // lane of the workgroup this thread serves
    const uint32_t pj = producer ? q - my * kEncPix : 0u;
    const bool has_lane = my < nl;
    LaneShape sh = lane_shape(g, lane0 + (has_lane ? my : 0u));
    if (!producer && has_lane) atomicMax(&s_max_px, sh.npx);
    __syncthreads();
    const uint32_t batches = (s_max_px + kEncPix - 1u) / kEncPix;

    // chain state (threads 0..nl-1 of wave 0)
    uint32_t S = 1u << 16;
    // index into scratch, one past the lane's slot (block_slot_end: one spare word below every slot)
    const uint32_t slot_end = block_slot_end(sh, lane0 + (has_lane ? my : 0u));
    uint32_t wat = slot_end - 1u;  // where the next word goes: just below the lane's words so far

    // producers: the nine input values of the pixel of batch b, loaded one batch ahead
    struct PixelIn {
        int x[3], m[3], ls[3], a[3];
        bool valid;
    };
    auto fetch = [&](uint32_t b) {
        PixelIn in;
        const uint32_t idx = b * kEncPix + pj;  // pixel counted from the lane's end
        in.valid = has_lane && idx < sh.npx;
        const uint32_t t = in.valid ? sh.npx - 1u - idx : 0u;
        const uint32_t row = t / sh.tw;
        const uint32_t p = sh.first + row * g.w + (t - row * sh.tw);
        const size_t s = (size_t)p * 3;
        const uint32_t im = g.by_hw.div(p);
#pragma unroll
        for (int c = 0; c < 3; ++c) {
            in.x[c] = img[s + c];
            in.m[c] = mu[s + c];
            in.ls[c] = ls[s + c];
            in.a[c] = coef[3 * im + c];
        }
        return in;
    };
    auto produce = [&](const PixelIn &in, uint32_t buf) {
        if (!(my < (uint32_t)kEncLanes)) return;
        const int e_r = in.x[0] * 256 - in.m[0], e_g = in.x[1] * 256 - in.m[1];
        const int me[3] = {in.m[0], in.m[1] + rsh14_mul(in.a[0], e_r),
                           in.m[2] + rsh14_mul(in.a[1], e_r) + rsh14_mul(in.a[2], e_g)};
#pragma unroll
        for (int c = 0; c < 3; ++c) {
            const uint32_t inv_s = inv_scale(in.ls[c], tab);
            const uint32_t lo = in.x[c] == 0 ? 0u : cum_inner(in.x[c], me[c], inv_s, spread, tab);
            const uint32_t hi = in.x[c] == 255 ? top : cum_inner(in.x[c] + 1, me[c], inv_s, spread, tab);
            // the chain walks a batch last symbol first: pixel pj from the end, B before G before R
            rec[buf][3u * pj + (2 - c)][my] =
                in.valid ? encode_record(lo, hi - lo, m_bits) : make_uint4(0xFFFFFFFFu, 0u, 0u, 0u);
        }
    };

    auto consume = [&](uint32_t buf) {
        // all records of the batch first: the loads do not depend on the state
        uint4 r[kEncSyms];
#pragma unroll
        for (int k = 0; k < kEncSyms; ++k) r[k] = rec[buf][k][my];
#pragma unroll
        for (int k = 0; k < kEncSyms; ++k) {
            // The word is stored on every step, just below the words already there, and counted
            // only when the state renormalises: an uncounted word is overwritten by the next one
            // or stays below the lane's first word.  After i symbols at most i words are counted
            // and the slot has room for one per symbol, so the store stays in the slot, or, for the
            // empty steps after a lane's last symbol, in the spare word below it.
            const bool emit = S > r[k].x;
            scratch[wat] = (uint16_t)(S & 0xFFFFu);
            wat -= emit ? 1u : 0u;
            S = emit ? S >> 16 : S;
            const uint32_t t = __umulhi(r[k].y, S);
            // the shift count is the top byte of the record's last word (picked by the shift itself),
            // the multiplier its low 24 bits (all the 24-bit multiply looks at)
            const uint32_t quo = shift_right_by_top_byte(t + ((S - t) >> 1), r[k].w);
            S = S + r[k].z + __umul24(quo, r[k].w);
        }
    };

    PixelIn cur = {};
    if (producer) {
        cur = fetch(0);
        produce(cur, 0);
        cur = fetch(1);
    }
    __syncthreads();
    for (uint32_t b = 0; b < batches; ++b) {
        if (producer) {
            const PixelIn nxt = fetch(b + 2u);
            if (b + 1u < batches) produce(cur, (b + 1u) & 1u);
            cur = nxt;
        } else if (tid < (uint32_t)kEncLanes && has_lane) {
            consume(b & 1u);
        }
        __syncthreads();
    }
    if (!producer && has_lane) {
        lane_words[lane0 + my] = slot_end - 1u - wat;
        lane_state[lane0 + my] = S;
    }
}

}  // namespace pilc
