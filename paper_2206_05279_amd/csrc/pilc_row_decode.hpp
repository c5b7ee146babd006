// Decoder for batches with few, long lanes: a row of 16 threads owns one lane (gfx950).
//
// A lane is a serial chain (App. A eq. (12) of arXiv 2206.05279: every state depends on the one
// before), so with a few thousand lanes a wavefront must be alone on its SIMD and the time is
// (symbols per lane) x (instructions the wavefront issues per symbol) x 4 cycles.  This kernel
// is built to keep that instruction count low:
//   - a wavefront carries four lanes, one per 16-thread row, so 4096 lanes still leave every SIMD
//     of the chip with at most one wavefront;
//   - per symbol every thread evaluates C(k) at two neighbouring candidates of a 32-value window
//     around the predicted mean (exact 24-bit form), together with the mass up to its successor;
//     once the state is known, one subtraction and one compare per candidate tell the thread
//     whether it holds the symbol (App. A: the x with C_x <= S mod 2^M < C_x + P_x), every thread
//     forms the next state for its own candidates, and an OR over the row (four rotate-and-OR
//     steps on the data-parallel-primitive path, no LDS round trip, no ballot) hands the one
//     non-zero value to all 16 threads;
//   - a pixel is decoded without a branch: whether every symbol was inside its window is
//     looked at once per pixel, and a pixel with a symbol outside (or with a mean so far out
//     that the 24-bit form is not exact) is decoded again from the state saved at its start by a
//     bounded two-level search with the general evaluation (32 values eight apart, then the nine
//     of the band);
//   - the candidates of a pixel's first channel do not depend on decoded values and are evaluated
//     while the previous pixel is still being decoded;
//   - per-pixel parameters are prepared 16 pixels at a time, one pixel per thread, two batches
//     ahead of their use, and handed over through LDS; the 96 stream words a batch can reach are
//     fetched a batch ahead and wait in LDS, and the word a refill would take is read ahead of
//     time;
//   - none of that, nor the stores of the decoded pixels, is done by the wavefront that decodes:
//     every decoding wavefront has a second wavefront on its SIMD, its stager, which does it a
//     batch ahead in the issue slots the decoder leaves empty (a decoder that staged its own
//     batches spent 6 % of its time on it).  The two hand over through counts in LDS.
// Every loop has a trip count fixed by the geometry; the waits of the hand-over are bounded by the
// constant-rate clock and end in a time-out error.
#pragma once

#include <type_traits>

#include "pilc_device.hpp"

namespace pilc {

constexpr int kRowWaves = 4;                  // wavefronts per workgroup
constexpr int kRowLanes = 4 * kRowWaves;      // lanes per workgroup
constexpr int kRowBatch = 16;                 // pixels prepared at a time, one per thread of the row
constexpr int kRowWords = 112;                // stream words kept per lane and batch: a batch takes at
                                              // most 48 and is fetched before the previous one's 48
constexpr int kRowWindow = 32;                // candidates per symbol
constexpr int kRowBaseMax = 256 - kRowWindow; // window bases 0..224: candidates stay within 0..255
constexpr int kRowRedoLimit = 4;              // a batch with this many pixels outside their windows sends
constexpr int kRowSearchBatches = 7;          // the wavefront's next 7 batches straight to the search

// OR over the 16 threads of a row, result in every thread: rotate right by 1, 2, 4, 8 and OR.
__device__ __forceinline__ uint32_t row_or(uint32_t v)
{
    v |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x121 /* row_ror:1 */, 0xF, 0xF, false);
    v |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x122 /* row_ror:2 */, 0xF, 0xF, false);
    v |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x124 /* row_ror:4 */, 0xF, 0xF, false);
    v |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x128 /* row_ror:8 */, 0xF, 0xF, false);
    return v;
}

// The same for two values at once, the steps of the two reductions taken in turn: a step reads
// what the step before it wrote, so two independent reductions fill each other's waiting time.
__device__ __forceinline__ void row_or2(uint32_t &a, uint32_t &b)
{
#define PILC_ROW_OR_STEP(ctrl)                                                                  \
    a |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)a, ctrl, 0xF, 0xF, false);               \
    b |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)b, ctrl, 0xF, 0xF, false);
    PILC_ROW_OR_STEP(0x121)
    PILC_ROW_OR_STEP(0x122)
    PILC_ROW_OR_STEP(0x124)
    PILC_ROW_OR_STEP(0x128)
#undef PILC_ROW_OR_STEP
}

// thread j of a row receives the value of thread (j + 1) mod 16 of the same row
__device__ __forceinline__ uint32_t row_next(uint32_t v)
{
    return (uint32_t)__builtin_amdgcn_mov_dpp((int)v, 0x12F /* row_ror:15 */, 0xF, 0xF, true);
}

// floor((a * e + 2^13) / 2^14) for a Q2.14 coefficient and an innovation e of at most 18 bits
__device__ __forceinline__ int rsh14_mad(int a, int e) { return mad_i24(a, e, 8192) >> 14; }

// What one pixel's preparing thread leaves in LDS for the row (64 bytes).  1/s is the Q6.25
// inverse scale; "split" means (>> 17, & 0x1FFFF), the form the 24-bit evaluation takes.
struct RowPixel {
    uint4 r;  // m_r (Q8.8), 1/s of R split, 1/s of R whole
    uint4 a;  // m_g, m_b (Q8.8), a_gr, a_br (Q2.14, sign-extended)
    uint4 b;  // a_bg, 1/s of G split, 1/s of B >> 17
    uint4 c;  // 1/s of B & 0x1FFFF, 1/s of G whole, 1/s of B whole, window of R: base | exact << 16
};

// The candidates of one symbol as a thread holds them: C(k) at k = base + 2 j and base + 2 j + 1
// and the masses up to their successors (0 for a candidate that cannot be the symbol).
struct RowCand {
    uint32_t cv0, cv1, f0, f1;
    int base;
    bool ok;  // the 24-bit evaluation is exact for this window
};

// kStaged: with a stager per decoding wavefront (see above).  That form keeps twice the LDS per
// lane (the first channel's candidates of two batches), so only one workgroup of 16 lanes fits a
// compute unit; it is for batches of up to 16 lanes per compute unit.  Without it a decoding
// wavefront stages its own batches, and two workgroups share a compute unit.
template <bool kRagged, bool kStaged>
__global__ __launch_bounds__((kStaged ? 2 : 1) * 64 * kRowWaves) void k_decode_rows(
    Geo g, const uint8_t *__restrict__ coded, const uint16_t *__restrict__ mu,
    const int16_t *__restrict__ ls, const int16_t *__restrict__ coef, uint8_t *__restrict__ out,
    int *__restrict__ status_code, const unsigned long long *__restrict__ status_payload,
    unsigned long long wait_ticks, uint32_t withhold)
{
    // wait_ticks: the bound of a wait between a decoding wavefront and its stager, in ticks of the
    // constant-rate clock; withhold: the stagers never say that a batch is ready (tests of the
    // give-up path)
    __shared__ LdsTables tab;
    __shared__ RowPixel stage[2][kRowLanes][kRowBatch];
    __shared__ uint16_t words[2][kRowLanes][kRowWords];
    // C(k) at the two candidates of every thread for the first channel of every pixel of a batch,
    // 16 bits each (a candidate is at most 255, so C is below 2^M <= 2^16)
    __shared__ uint32_t first_cand[kStaged ? 2 : 1][kStaged ? kRowLanes : 1][kRowBatch][16];
    // The workgroup has two wavefronts per four lanes: one decodes, the other (its stager) prepares
    // the next batch's parameters and stream words in LDS meanwhile.  What passes between them:
    __shared__ uint32_t s_word_base[2][kRowLanes];  // stream position of words[buf][lane][0]
    // Of batch b, in slot b & 1: the lane's stream position at its start and its 16 decoded pixels.
    // (The decoder writes a slot again two batches later, and cannot start that batch before the
    // stager, which reads the slot first, has staged it.)
    __shared__ uint32_t s_pos[2][kRowLanes];
    __shared__ uint32_t s_out[2][kStaged ? kRowLanes : 1][kRowBatch];
    __shared__ uint32_t s_posted[kRowWaves];        // batches the decoding wavefront has finished
    __shared__ uint32_t s_staged[kRowWaves];        // batches the stager has made ready
    __shared__ uint32_t s_abort;                    // a wait was given up: everybody leaves
    if (threadIdx.x < (uint32_t)kRowWaves) {
        s_posted[threadIdx.x] = 0u;
        s_staged[threadIdx.x] = 0u;
    }
    // Whether the call has failed already is looked at once for the whole workgroup: were every
    // wavefront to look for itself, another workgroup's error could come between the looks, and a
    // wavefront would wait for a partner that has left.
    __shared__ int s_failed;
    if (threadIdx.x == 0u) {
        s_abort = 0u;
        s_failed = *status_code;
    }
    load_tables(tab);  // ends with a barrier
    if (s_failed != 0) return;

    const bool stager = kStaged && threadIdx.x >= 64u * kRowWaves;
    const uint32_t tix = threadIdx.x - (stager ? 64u * kRowWaves : 0u);  // index among the threads of its kind
    const uint32_t tid = tix & 63u, wv = tix >> 6;
    const uint32_t j = tid & 15u, gbase = tid & 48u;
    const uint32_t lrow = tix >> 4;  // lane slot of the workgroup
    // a row beyond the last lane decodes the last lane once more and keeps the result to itself,
    // so that every row of a wavefront always does valid work
    const bool has_lane = blockIdx.x * kRowLanes + lrow < g.lanes;
    const uint32_t lane = has_lane ? blockIdx.x * kRowLanes + lrow : g.lanes - 1u;
    const LaneShape sh = lane_shape(g, lane);
    const uint32_t m_bits = g.prec_bits;
    const uint32_t mask = (1u << m_bits) - 1u, top = 1u << m_bits;
    const uint32_t sp8 = (top - 256u) >> 8;  // 2^M - 256 = 256 * sp8
    const uint32_t payload_bytes = (uint32_t)*status_payload;
    const uint32_t *offsets = reinterpret_cast<const uint32_t *>(coded + 64);
    const uint16_t *payload =
        reinterpret_cast<const uint16_t *>(coded + 64 + 4ull * ((size_t)g.lanes + 1));
    const uint2 *sig = tab.sig;

    // row-uniform state: S, the stream position `pos` (word index into the payload) and the end
    // of the lane's words `stop`
    uint32_t npx = 0, stop = 0, S = 1u << 16, pos = 0;
    {
        const uint32_t begin = offsets[lane], end = offsets[lane + 1];
        if (end < begin || end > payload_bytes || end - begin < 4u || ((begin | end) & 1u)) {
            if (j == 0 && has_lane) atomicMax(status_code, 6);
        } else {
            npx = sh.npx;
            stop = end >> 1;
            pos = begin >> 1;
            S = (uint32_t)payload[pos] | ((uint32_t)payload[pos + 1] << 16);
            pos += 2;
        }
    }
    // The stream words from `from` on, thread j those at j, j + 16, ...: words past `stop` read
    // as 0, and an overrun shows at the end of the lane as pos != stop.
    struct Ahead {
        uint32_t w[kRowWords / 16];
    };
    auto fetch_words = [&](uint32_t from) {
        Ahead a;
#pragma unroll
        for (int r = 0; r < kRowWords / 16; ++r) {
            const uint32_t at = from + 16u * r + j;
            a.w[r] = at < stop ? (uint32_t)payload[at] : 0u;
        }
        return a;
    };

    // ---- per-pixel parameters: thread j prepares pixel t0 + j of its lane ----
    struct Raw {
        uint32_t m[3];
        int l[3], a[3];
    };
    auto fetch_raw = [&](uint32_t t0) {
        Raw r;
        const uint32_t t = t0 + j;
        const uint32_t p = lane_pixel(g, sh, t < npx ? t : 0u);
        const size_t s = (size_t)p * 3;
        const uint32_t im = g.by_hw.div(p);
#pragma unroll
        for (int c = 0; c < 3; ++c) {
            r.m[c] = mu[s + c];
            r.l[c] = ls[s + c];
            r.a[c] = coef[3 * im + c];
        }
        return r;
    };
    auto window_base = [](int me) { return min(max((me - (256 * (kRowWindow / 2 - 1) - 128)) >> 8, 0), kRowBaseMax); };
    auto window_exact = [](int me) { return (uint32_t)(me + 8576) <= (uint32_t)(73600 + 8576); };
    auto put_stage = [&](const Raw &r, uint32_t buf) {
        const uint32_t i0 = inv_scale(r.l[0], tab), i1 = inv_scale(r.l[1], tab), i2 = inv_scale(r.l[2], tab);
        RowPixel px;
        px.r = make_uint4(r.m[0], i0 >> 17, i0 & 0x1FFFFu, i0);
        px.a = make_uint4(r.m[1], r.m[2], (uint32_t)r.a[0], (uint32_t)r.a[1]);
        px.b = make_uint4((uint32_t)r.a[2], i1 >> 17, i1 & 0x1FFFFu, i2 >> 17);
        px.c = make_uint4(i2 & 0x1FFFFu, i1, i2,
                          (uint32_t)window_base((int)r.m[0]) | (window_exact((int)r.m[0]) ? 1u << 16 : 0u));
        stage[buf][lrow][j] = px;
    };

    // Window of a symbol with effective mean `me`, and this thread's candidates k = base + 2 j and
    // base + 2 j + 1 in it.  With 1/s = inv_hi * 2^17 + inv_lo the clamped
    // z = floor(d * (1/s) / 2^17) = d * inv_hi + floor(d * inv_lo / 2^17) is exact in 32-bit
    // arithmetic with 24-bit multiplies while |d| <= 2^14, d = 256 k - 128 - mean; that holds over the
    // whole window for means in -8576 .. 73600.
    // The evaluation comes in two halves so that the wait for one symbol's table cells can be
    // filled with another symbol's arithmetic: `aim` goes as far as asking for the cells,
    // `finish` takes it from there.
    struct RowAim {
        uint2 cell[2];
        int z[2];
        int base, k0;
        bool ok;
    };
    const int j2 = 2 * (int)j;
    auto aim = [&](int me, uint32_t inv_hi, uint32_t inv_lo) {
        RowAim am;
        am.base = window_base(me);
        am.ok = window_exact(me);
        am.k0 = am.base + j2;
        const int d0 = 256 * am.k0 - 128 - me;
#pragma unroll
        for (int c = 0; c < 2; ++c) {
            const int d = d0 + 256 * c;
            const int t = mul_i24(d, (int)inv_lo) >> 17;
            am.z[c] = min(max(mad_i24(d, (int)inv_hi, t), -(1 << 20)), (1 << 20) - 1);
            am.cell[c] = (sig + 1024)[am.z[c] >> 10];
        }
        return am;
    };
    // C(k) at the thread's two candidates, from the cells `aim` asked for
    auto cum_pair = [&](const RowAim &am, uint32_t cv[2]) {
#pragma unroll
        for (int c = 0; c < 2; ++c) {
            const uint32_t f24 =
                am.cell[c].x + ((uint32_t)__umul24(am.cell[c].y, (uint32_t)am.z[c] & 1023u) >> 16);
            cv[c] = (uint32_t)(am.k0 + c) + ((uint32_t)__umul24(f24, sp8) >> 16);
        }
        cv[0] = am.k0 == 0 ? 0u : cv[0];  // C(0) = 0
    };
    // The candidates of a symbol from its two values of C.  The second candidate is followed by the
    // next thread's first; candidate 31 by C(base + 32), which is known only when it is C(256) = 2^M.
    auto with_masses = [&](uint32_t cv0, uint32_t cv1, int base, bool ok) {
        RowCand cd;
        const uint32_t from_next = row_next(cv0);
        const uint32_t after = j == 15u ? (base == kRowBaseMax ? top : cv1) : from_next;
        cd.cv0 = cv0;
        cd.cv1 = cv1;
        cd.f0 = cv1 - cv0;
        cd.f1 = after - cv1;
        cd.base = base;
        cd.ok = ok;
        return cd;
    };
    auto finish = [&](const RowAim &am) {
        uint32_t cv[2];
        cum_pair(am, cv);
        return with_masses(cv[0], cv[1], am.base, am.ok);
    };
    // the same for a pixel's first channel, whose two values of C the stager has left in LDS
    auto first_channel = [&](uint32_t pair, uint32_t window) {
        return with_masses(pair & 0xFFFFu, pair >> 16, (int)(window & 0xFFFFu), (window >> 16) != 0u);
    };
    // (stager) the first channel of the 16 pixels staged in `buf`, every thread its two candidates
    auto put_first_cand = [&](uint32_t buf) {
        wave_lds_sync();  // the parameters were written by this wavefront
#pragma unroll 4
        for (int i = 0; i < kRowBatch; ++i) {
            const uint4 r = stage[buf][lrow][i].r;
            uint32_t cv[2];
            cum_pair(aim((int)r.x, r.y, r.z), cv);
            first_cand[buf][lrow][i][j] = cv[0] | (cv[1] << 16);
        }
    };

    const uint32_t xw0 = 2u * j | 256u, xw1 = xw0 | 1u;  // what a winning candidate contributes
    const uint16_t *my_words = words[0][lrow];  // the current batch's words, from `wbase` on
    uint32_t wbase = pos;
    uint32_t wnext = 0;  // the word at `pos`
    // One symbol of the four lanes of the wavefront, no branch.  Returns the value (meaningless
    // where the window does not hold the symbol: bit 8 of `seen` is then cleared); updates S, pos,
    // wnext of rows with `act`.
    auto decode_symbol = [&](bool act, const RowCand &cd, uint32_t &seen) -> uint32_t {
        const uint32_t slot = S & mask, q = S >> m_bits;
        const uint32_t t0 = slot - cd.cv0, t1 = slot - cd.cv1;
        const bool win0 = t0 < cd.f0, win1 = t1 < cd.f1;
        // App. A eq. (12) as if this thread's candidate were the symbol: the mass is at most 2^16
        // and S >> M below 2^22, so the 24-bit multiply is exact
        const uint32_t s0 = (uint32_t)__umul24(cd.f0, q) + t0, s1 = (uint32_t)__umul24(cd.f1, q) + t1;
        // at most one of the two is the symbol (no nested choice: it would become a branch)
        uint32_t s_new = (win0 ? s0 : 0u) | (win1 ? s1 : 0u);
        uint32_t xw = (win0 ? xw0 : 0u) | (win1 ? xw1 : 0u);
        row_or2(xw, s_new);
        // (kept as one value: left free, the compiler splits the last step of the reduction into a
        // move, an OR and a three-operand AND for the two uses of xw below, four instructions for two)
        asm("" : "+v"(xw));
        seen &= cd.ok ? xw : 0u;
        const bool refill = s_new < (1u << 16);
        const uint32_t s_ref = (s_new << 16) | wnext;
        if (kRagged) {
            S = act ? (refill ? s_ref : s_new) : S;
            pos += (act && refill) ? 1u : 0u;
        } else {
            S = refill ? s_ref : s_new;
            pos += refill ? 1u : 0u;
        }
        wnext = my_words[pos - wbase];
        return (uint32_t)cd.base + (xw & 255u);
    };
    // The same by a bounded search with the general evaluation, on the state (Sr, pr): every 8th
    // value first (C(0) = 0 always counts), then the nine values of the band.
    auto search_symbol = [&](int me, uint32_t inv_s, uint32_t &Sr, uint32_t &pr) -> uint32_t {
        auto row_count = [&](bool pred) -> uint32_t {
            return (uint32_t)__popc((uint32_t)(__ballot(pred) >> gbase) & 0xFFFFu);
        };
        const uint32_t slot = Sr & mask, q = Sr >> m_bits;
        const uint32_t below = row_count(cum_at(8 * (int)j, me, inv_s, m_bits, tab) <= slot) +
                               row_count(cum_at(8 * (int)j + 128, me, inv_s, m_bits, tab) <= slot);
        const int kb = 8 * ((int)below - 1);
        const uint32_t cf = cum_at(min(kb + (int)j, 256), me, inv_s, m_bits, tab);
        const uint32_t n = row_count(j <= 8u && cf <= slot);  // 1..8: C(kb) <= slot < C(kb + 8)
        const uint32_t c_lo = (uint32_t)__builtin_amdgcn_ds_bpermute((int)((gbase + n - 1u) << 2), (int)cf);
        const uint32_t c_hi = (uint32_t)__builtin_amdgcn_ds_bpermute((int)((gbase + n) << 2), (int)cf);
        uint32_t s_new = (uint32_t)__umul24(c_hi - c_lo, q) + (slot - c_lo);
        if (s_new < (1u << 16)) {
            s_new = (s_new << 16) | my_words[pr - wbase];
            ++pr;
        }
        Sr = s_new;
        return (uint32_t)kb + n - 1u;
    };

    // Hand-over between a decoding wavefront and its stager: a count in LDS, raised by one thread
    // after the wavefront's LDS writes are done, and waited for by the whole partner wavefront.  A
    // wait is bounded by the constant-rate clock; who gives up says so to everybody (no wavefront
    // is left waiting) and the call ends in a time-out error.
    auto raise = [&](uint32_t *count, uint32_t value) {
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
        if (tid == 0u) __hip_atomic_store(count, value, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    };
    auto wait_for = [&](uint32_t *count, uint32_t value) -> bool {
        if (__hip_atomic_load(count, __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_WORKGROUP) >= value) return true;
        const unsigned long long since = wall_clock64();
        for (;;) {
            if (__hip_atomic_load(count, __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_WORKGROUP) >= value) return true;
            if (__hip_atomic_load(&s_abort, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP) != 0u) return false;
            if (wall_clock64() - since > wait_ticks) {
                __hip_atomic_store(&s_abort, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
                if (tid == 0u) atomicMax(status_code, 8);
                return false;
            }
            __builtin_amdgcn_s_sleep(8);
        }
    };
    auto put_words = [&](const Ahead &a, uint32_t buf, uint32_t from) {
#pragma unroll
        for (int r = 0; r < kRowWords / 16; ++r) words[buf][lrow][16 * r + j] = (uint16_t)a.w[r];
        if (j == 0u) s_word_base[buf][lrow] = from;
    };

    // the pixels of the batch that began at pixel t0 of the lane, from slot `slot`, to the image
    auto store_batch = [&](uint32_t t0, uint32_t slot) {
        const uint32_t nb = t0 < npx ? min((uint32_t)kRowBatch, npx - t0) : 0u;
        if (j < nb && has_lane) {
            const uint32_t v = s_out[slot][lrow][j];
            const size_t s = (size_t)lane_pixel(g, sh, t0 + j) * 3;
            out[s] = (uint8_t)v;
            out[s + 1] = (uint8_t)(v >> 8);
            out[s + 2] = (uint8_t)(v >> 16);
        }
    };

    if (kStaged && stager) {
        // Batch 0 first; then, while the partner decodes batch b, the parameters of batch b + 1 (loaded
        // a batch ago) and its stream words: the 112 words from where the stream stood when batch b
        // began, of which batch b takes at most 48 and batch b + 1 at most 48 more; and the pixels of
        // batch b - 1 go to the image.
        put_stage(fetch_raw(0), 0);
        Raw raw_next = fetch_raw(kRowBatch);
        put_first_cand(0u);
        put_words(fetch_words(pos), 0u, pos);
        if (!withhold) raise(&s_staged[wv], 1u);
        uint32_t from = pos, t0 = 0, b = 0;
        for (; __any(t0 < npx); t0 += kRowBatch, ++b) {
            const uint32_t buf = b & 1u;
            if (b != 0u) {
                // the partner has finished batch b - 1: buffer buf ^ 1 is free, and the position is known
                if (!wait_for(&s_posted[wv], b)) return;
                from = s_pos[buf][lrow];
                store_batch(t0 - kRowBatch, buf ^ 1u);
            }
            const Ahead ahead = fetch_words(from);
            put_stage(raw_next, buf ^ 1u);
            raw_next = fetch_raw(t0 + 2 * kRowBatch);
            put_first_cand(buf ^ 1u);
            put_words(ahead, buf ^ 1u, from);
            if (!withhold) raise(&s_staged[wv], b + 2u);
        }
        if (b != 0u && wait_for(&s_posted[wv], b)) store_batch(t0 - kRowBatch, (b & 1u) ^ 1u);  // the last batch's pixels
        return;
    }

    uint32_t search_batches = 0;  // wavefront-uniform: batches still to decode by search alone
    // (without a stager) batch 0 staged, batch 1 in flight
    Raw raw_next = {};
    Ahead ahead = {};
    uint32_t ahead_base = pos;
    if (!kStaged) {
        put_stage(fetch_raw(0), 0);
        raw_next = fetch_raw(kRowBatch);
        ahead = fetch_words(pos);
    }
    for (uint32_t t0 = 0, b = 0; __any(t0 < npx); t0 += kRowBatch, ++b) {
        const uint32_t buf = b & 1u;
        const uint32_t nb = t0 < npx ? min((uint32_t)kRowBatch, npx - t0) : 0u;
        if (kStaged) {
            if (!wait_for(&s_staged[wv], b + 1u)) break;
            my_words = words[buf][lrow];
            wbase = s_word_base[buf][lrow];
        } else {
            // this batch's words (fetched a batch ago, from where the stream stood then) into LDS, the
            // next batch's requested from where the stream stands now; the next batch's parameters
            // staged from the registers loaded a batch ago, and the batch after that requested
            my_words = words[buf][lrow];
            wbase = ahead_base;
#pragma unroll
            for (int r = 0; r < kRowWords / 16; ++r) words[buf][lrow][16 * r + j] = (uint16_t)ahead.w[r];
            ahead = fetch_words(pos);
            ahead_base = pos;
            put_stage(raw_next, buf ^ 1u);
            raw_next = fetch_raw(t0 + 2 * kRowBatch);
            wave_lds_sync();
        }
        wnext = my_words[pos - wbase];

        const RowPixel *px = stage[buf][lrow];
        uint32_t v_out = 0;
        // The three symbols of a pixel by search, on the state (Sr, pr).
        auto search_pixel = [&](const RowPixel &cur, uint32_t &Sr, uint32_t &pr, uint32_t &y_r, uint32_t &y_g,
                                uint32_t &y_b) {
            const int m_r = (int)cur.r.x, m_g = (int)cur.a.x, m_b = (int)cur.a.y;
            const int a_gr = (int)cur.a.z, a_br = (int)cur.a.w, a_bg = (int)cur.b.x;
            y_r = search_symbol(m_r, cur.r.w, Sr, pr);
            const int f_r = (int)(y_r << 8) - m_r;
            y_g = search_symbol(m_g + rsh14_mul(a_gr, f_r), cur.c.y, Sr, pr);
            y_b = search_symbol(m_b + rsh14_mul(a_br, f_r) + rsh14_mul(a_bg, (int)(y_g << 8) - m_g), cur.c.z,
                                Sr, pr);
        };
        if (search_batches != 0) {
            // data the model does not fit (such as uniformly random pixels): the windows are not tried
            --search_batches;
            for (uint32_t i = 0; kRagged ? __any(i < nb) : i < (uint32_t)kRowBatch; ++i) {
                uint32_t Sr = S, pr = pos, y_r, y_g, y_b;
                search_pixel(px[i], Sr, pr, y_r, y_g, y_b);
                if (!kRagged || i < nb) {
                    S = Sr;
                    pos = pr;
                }
                v_out = j == i ? (y_r | (y_g << 8) | (y_b << 16)) : v_out;
            }
        } else {
            uint32_t redone = 0;  // pixels of this batch that had a symbol outside its window
            // One pixel: `cur` holds its parameters (read from LDS a pixel ago), `nxt` receives the
            // next pixel's, and `cr` enters with this pixel's first-channel candidates and leaves
            // with the next pixel's.
            auto pixel = [&](uint32_t i, const RowPixel &cur, RowPixel &nxt, RowCand &cr) {
                const bool act = i < nb;
                nxt = px[(i + 1u) & (kRowBatch - 1)];
                const uint32_t next_pair = kStaged ? first_cand[buf][lrow][(i + 1u) & (kRowBatch - 1)][j] : 0u;
                __builtin_amdgcn_sched_barrier(0);  // asked for here, used a pixel later
                const int m_r = (int)cur.r.x, m_g = (int)cur.a.x, m_b = (int)cur.a.y;
                const int a_gr = (int)cur.a.z, a_br = (int)cur.a.w, a_bg = (int)cur.b.x;
                const uint32_t S0 = S, pos0 = pos;
                uint32_t seen = 256u;

                uint32_t x_r = decode_symbol(act, cr, seen);
                const int e_r = (int)(x_r << 8) - m_r;
                const int me_g = m_g + rsh14_mad(a_gr, e_r);
                const RowAim ag = aim(me_g, cur.b.y, cur.b.z);
                __builtin_amdgcn_sched_barrier(0);
                const int mb1 = m_b + rsh14_mad(a_br, e_r);
                // The next pixel's first channel depends on no decoded value.  The stager has evaluated
                // it, and what is left to do fills the wait for this channel's table cells; without a
                // stager its evaluation fills the waits of the two channels that do depend.
                RowCand cr_next = {};
                RowAim an = {};
                if (kStaged)
                    cr_next = first_channel(next_pair, nxt.c.w);
                else
                    an = aim((int)nxt.r.x, nxt.r.y, nxt.r.z);
                __builtin_amdgcn_sched_barrier(0);
                const RowCand cg = finish(ag);
                uint32_t x_g = decode_symbol(act, cg, seen);
                const int me_b = mb1 + rsh14_mad(a_bg, (int)(x_g << 8) - m_g);
                const RowAim ab = aim(me_b, cur.b.w, cur.c.x);
                __builtin_amdgcn_sched_barrier(0);
                if (kStaged) {
                    cr = cr_next;
                } else {
                    cr = finish(an);
                    __builtin_amdgcn_sched_barrier(0);
                }
                const RowCand cb = finish(ab);
                uint32_t x_b = decode_symbol(act, cb, seen);

                bool bad = (seen & 256u) == 0u;
                if (kRagged) bad = bad && act;
                if (__builtin_expect(__any(bad), 0)) {
                    // the pixel once more, from the state at its start, for the rows that need it
                    uint32_t Sr = S0, pr = pos0, y_r, y_g, y_b;
                    search_pixel(cur, Sr, pr, y_r, y_g, y_b);
                    if (bad) {
                        S = Sr;
                        pos = pr;
                        x_r = y_r;
                        x_g = y_g;
                        x_b = y_b;
                    }
                    wnext = my_words[pos - wbase];
                    ++redone;
                }
                v_out = j == i ? (x_r | (x_g << 8) | (x_b << 16)) : v_out;
            };
            RowPixel pe = px[0], po;
            RowCand cr = kStaged ? first_channel(first_cand[buf][lrow][0][j], pe.c.w)
                                 : finish(aim((int)pe.r.x, pe.r.y, pe.r.z));
            for (uint32_t i = 0; kRagged ? __any(i < nb) : i < (uint32_t)kRowBatch; i += 2) {
                pixel(i, pe, po, cr);
                pixel(i + 1u, po, pe, cr);
            }
            if (redone >= (uint32_t)kRowRedoLimit) search_batches = kRowSearchBatches;
        }
        if (kStaged) {
            // the pixels and the position go to the stager, which may then go on to the batch after next
            s_out[buf][lrow][j] = v_out;
            if (j == 0u) s_pos[buf ^ 1u][lrow] = pos;
            raise(&s_posted[wv], b + 1u);
        } else if (j < nb && has_lane) {
            const size_t s = (size_t)lane_pixel(g, sh, t0 + j) * 3;
            out[s] = (uint8_t)v_out;
            out[s + 1] = (uint8_t)(v_out >> 8);
            out[s + 2] = (uint8_t)(v_out >> 16);
        }
    }
    if (has_lane && npx != 0u && (S != (1u << 16) || pos != stop) && j == 0) atomicMax(status_code, 6);
}

}  // namespace pilc
