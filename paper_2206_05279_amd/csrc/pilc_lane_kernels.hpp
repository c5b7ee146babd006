// One thread per lane: the kernels for batches with many lanes (gfx950).
//
// Every thread walks its own lane (App. A eqs. (11)-(12) of arXiv 2206.05279 are serial per
// lane), so neighbouring threads read memory a whole lane apart.  A lane is consumed in chunks of
// 8 pixels held in registers: when the geometry keeps every chunk 8-pixel aligned (kVec) the
// 24 + 48 + 48 bytes of a chunk arrive as 64- and 128-bit loads, and decoded pixels leave as
// 64-bit stores; otherwise, and for ragged chunk tails, the same registers are filled element by
// element.  The coded words, which a thread produces or consumes one at a time, never go to
// memory one at a time: the encoder writes them to a scratch laid out [word number][thread], so
// that the 64 lanes of a wavefront fill whole lines, and the decoder reads them through a ring
// of 32 words per thread in LDS that is refilled with 16-byte loads between chunks.
#pragma once

#include <type_traits>

#include "pilc_device.hpp"

namespace pilc {

constexpr int kChunk = 8;  // pixels per chunk
constexpr int kLaneMaxThreads = 256;  // the lane kernels run in workgroups of 64 or 256

struct Chunk {
    int x[kChunk][3];   // pixel values (encode)
    int m[kChunk][3];   // mu, Q8.8
    int l[kChunk][3];   // log-scale, Q4.12
};

__device__ __forceinline__ int byte_of(const uint32_t *w, int i) { return (w[i >> 2] >> (8 * (i & 3))) & 0xFF; }
__device__ __forceinline__ int half_of(const uint32_t *w, int i) { return (w[i >> 1] >> (16 * (i & 1))) & 0xFFFF; }

// Fills `c` with the pixels p .. p+len-1 (len <= 8).  kVec: p is a multiple of 8 and the arrays
// are 16-byte aligned, so a full chunk is 3 x 8 bytes of pixels and 3 x 16 bytes of each parameter.
template <bool kVec, bool kPixels>
__device__ __forceinline__ void load_chunk(Chunk &c, uint32_t p, uint32_t len,
                                           const uint8_t *__restrict__ img,
                                           const uint16_t *__restrict__ mu,
                                           const int16_t *__restrict__ ls)
{
    const size_t s = (size_t)p * 3;
    if (kVec && len == (uint32_t)kChunk) {
        uint32_t wm[12], wl[12];
        const uint4 *pm = reinterpret_cast<const uint4 *>(mu + s);
        const uint4 *pl = reinterpret_cast<const uint4 *>(ls + s);
#pragma unroll
        for (int q = 0; q < 3; ++q) {
            const uint4 a = pm[q], b = pl[q];
            wm[4 * q] = a.x; wm[4 * q + 1] = a.y; wm[4 * q + 2] = a.z; wm[4 * q + 3] = a.w;
            wl[4 * q] = b.x; wl[4 * q + 1] = b.y; wl[4 * q + 2] = b.z; wl[4 * q + 3] = b.w;
        }
        uint32_t wx[6] = {0, 0, 0, 0, 0, 0};
        if (kPixels) {
            const uint2 *px = reinterpret_cast<const uint2 *>(img + s);
#pragma unroll
            for (int q = 0; q < 3; ++q) {
                const uint2 a = px[q];
                wx[2 * q] = a.x; wx[2 * q + 1] = a.y;
            }
        }
#pragma unroll
        for (int i = 0; i < kChunk; ++i)
#pragma unroll
            for (int ch = 0; ch < 3; ++ch) {
                if (kPixels) c.x[i][ch] = byte_of(wx, 3 * i + ch);
                c.m[i][ch] = half_of(wm, 3 * i + ch);
                c.l[i][ch] = (int)(short)half_of(wl, 3 * i + ch);
            }
    } else {
#pragma unroll
        for (int i = 0; i < kChunk; ++i)
#pragma unroll
            for (int ch = 0; ch < 3; ++ch) {
                const bool in = (uint32_t)i < len;
                const size_t e = in ? s + 3 * i + ch : s;
                if (kPixels) c.x[i][ch] = img[e];
                c.m[i][ch] = mu[e];
                c.l[i][ch] = ls[e];
            }
    }
}

// The 8 pixels held in the words wx (6 dwords of pixels), wm and wl (12 dwords each) into `c`.
template <bool kPixels>
__device__ __forceinline__ void unpack_chunk(Chunk &c, const uint32_t *wx, const uint32_t *wm,
                                             const uint32_t *wl)
{
#pragma unroll
    for (int i = 0; i < kChunk; ++i)
#pragma unroll
        for (int ch = 0; ch < 3; ++ch) {
            if (kPixels) c.x[i][ch] = byte_of(wx, 3 * i + ch);
            c.m[i][ch] = half_of(wm, 3 * i + ch);
            c.l[i][ch] = (int)(short)half_of(wl, 3 * i + ch);
        }
}

// Two neighbouring chunks (16 pixels from p, a multiple of 16) as raw words: 96 bytes of each
// parameter array and 48 of pixels in 16-byte loads.  Taking two chunks at a time halves the
// number of times a thread comes back to a 128-byte line.
struct ChunkPair {
    uint32_t wx[12], wm[24], wl[24];
};
template <bool kPixels>
__device__ __forceinline__ void load_pair(ChunkPair &r, uint32_t p, const uint8_t *__restrict__ img,
                                          const uint16_t *__restrict__ mu,
                                          const int16_t *__restrict__ ls)
{
    const size_t s = (size_t)p * 3;
    const uint4 *pm = reinterpret_cast<const uint4 *>(mu + s);
    const uint4 *pl = reinterpret_cast<const uint4 *>(ls + s);
#pragma unroll
    for (int q = 0; q < 6; ++q) {
        const uint4 a = pm[q], b = pl[q];
        r.wm[4 * q] = a.x; r.wm[4 * q + 1] = a.y; r.wm[4 * q + 2] = a.z; r.wm[4 * q + 3] = a.w;
        r.wl[4 * q] = b.x; r.wl[4 * q + 1] = b.y; r.wl[4 * q + 2] = b.z; r.wl[4 * q + 3] = b.w;
    }
    if (kPixels) {
        const uint4 *px = reinterpret_cast<const uint4 *>(img + s);
#pragma unroll
        for (int q = 0; q < 3; ++q) {
            const uint4 a = px[q];
            r.wx[4 * q] = a.x; r.wx[4 * q + 1] = a.y; r.wx[4 * q + 2] = a.z; r.wx[4 * q + 3] = a.w;
        }
    }
}

// Whole-line feeding of ChunkPair for flat lanes made of 64-pixel groups that start on a 128-byte
// line of the parameter arrays (a group is three lines of each, a line 21 1/3 pixels).  A pair of
// chunks takes 96 bytes of each array, so three of every four pairs straddle a line; asked for by
// the pair, every line would be fetched twice, because it has left the caches when the thread
// comes back to it.  Here a thread asks for whole lines, eight 16-byte pieces at once, when a pair
// first needs one, and carries the pieces the pair does not use in registers to the pairs that
// do: every line is fetched once.  The pixels go the same way in halves of a group (96 bytes).
// `v` is the pair's number within its group (0..3); forward feeds pairs in the order 0,1,2,3,
// backward in the order 3,2,1,0.
struct LineCarry {
    uint4 m[6], l[6], x[3];
};
__device__ __forceinline__ void put_piece(uint32_t *w, int i, const uint4 &q)
{
    w[4 * i] = q.x; w[4 * i + 1] = q.y; w[4 * i + 2] = q.z; w[4 * i + 3] = q.w;
}
// One array's share of a pair: `grp` points at the group's 24 pieces.  Every piece is loaded
// straight into the place it is used from (the pair's words or the carry), so no more registers
// are alive than the pair and the carry take.
__device__ __forceinline__ void load_piece(uint32_t *w, int i, const uint4 *__restrict__ src)
{
    put_piece(w, i, *src);
}
template <bool kBackward>
__device__ __forceinline__ void feed_array(uint32_t *w, uint4 *carry, uint32_t v, const uint4 *__restrict__ grp)
{
    // forward:  v=0 line A: use A0-5, keep A6,7 | v=1 line B: kept + B0-3, keep B4-7 |
    //           v=2 line C: kept + C0,1, keep C2-7 | v=3: kept
    // backward: v=3 line C: use C2-7, keep C0,1 | v=2 line B: B4-7 + kept, keep B0-3 |
    //           v=1 line A: A6,7 + kept, keep A0-5 | v=0: kept
    if (!kBackward) {
        switch (v) {
        case 0:
#pragma unroll
            for (int i = 0; i < 6; ++i) load_piece(w, i, grp + i);
            carry[0] = grp[6]; carry[1] = grp[7];
            break;
        case 1:
            put_piece(w, 0, carry[0]); put_piece(w, 1, carry[1]);
#pragma unroll
            for (int i = 0; i < 4; ++i) load_piece(w, 2 + i, grp + 8 + i);
#pragma unroll
            for (int i = 0; i < 4; ++i) carry[i] = grp[12 + i];
            break;
        case 2:
#pragma unroll
            for (int i = 0; i < 4; ++i) put_piece(w, i, carry[i]);
            load_piece(w, 4, grp + 16); load_piece(w, 5, grp + 17);
#pragma unroll
            for (int i = 0; i < 6; ++i) carry[i] = grp[18 + i];
            break;
        default:
#pragma unroll
            for (int i = 0; i < 6; ++i) put_piece(w, i, carry[i]);
            break;
        }
    } else {
        switch (v) {
        case 3:
#pragma unroll
            for (int i = 0; i < 6; ++i) load_piece(w, i, grp + 18 + i);
            carry[0] = grp[16]; carry[1] = grp[17];
            break;
        case 2:
#pragma unroll
            for (int i = 0; i < 4; ++i) load_piece(w, i, grp + 12 + i);
            put_piece(w, 4, carry[0]); put_piece(w, 5, carry[1]);
#pragma unroll
            for (int i = 0; i < 4; ++i) carry[i] = grp[8 + i];
            break;
        case 1:
            load_piece(w, 0, grp + 6); load_piece(w, 1, grp + 7);
#pragma unroll
            for (int i = 0; i < 4; ++i) put_piece(w, 2 + i, carry[i]);
#pragma unroll
            for (int i = 0; i < 6; ++i) carry[i] = grp[i];
            break;
        default:
#pragma unroll
            for (int i = 0; i < 6; ++i) put_piece(w, i, carry[i]);
            break;
        }
    }
}
// The pair `v` of the group whose first pixel is `pg` (a multiple of 64 pixels from the lane's start).
template <bool kBackward, bool kPixels>
__device__ __forceinline__ void feed_pair(ChunkPair &r, LineCarry &c, uint32_t v, uint32_t pg,
                                          const uint8_t *__restrict__ img, const uint16_t *__restrict__ mu,
                                          const int16_t *__restrict__ ls)
{
    const size_t s = (size_t)pg * 3;
    feed_array<kBackward>(r.wm, c.m, v, reinterpret_cast<const uint4 *>(mu + s));
    feed_array<kBackward>(r.wl, c.l, v, reinterpret_cast<const uint4 *>(ls + s));
    if (kPixels) {
        const uint4 *px = reinterpret_cast<const uint4 *>(img + s);  // 12 pieces a group, 3 a pair
        const bool fresh = kBackward ? (v & 1u) != 0u : (v & 1u) == 0u;  // first pair of its half
        if (fresh) {
            const uint32_t h = 6u * (v >> 1);
            uint4 n[6];
#pragma unroll
            for (int i = 0; i < 6; ++i) n[i] = px[h + i];
#pragma unroll
            for (int i = 0; i < 3; ++i) {
                put_piece(r.wx, i, kBackward ? n[3 + i] : n[i]);
                c.x[i] = kBackward ? n[i] : n[3 + i];
            }
        } else {
#pragma unroll
            for (int i = 0; i < 3; ++i) put_piece(r.wx, i, c.x[i]);
        }
    }
}

// floor(n / f) and the remainder for f <= 2^16 and n / f < 2^(32-M) (true after the
// renormalisation of the encoder), given rf = 1/f to float accuracy.  Conversion, reciprocal and
// product are each within 2^-24, 2^-23 and 2^-24 of exact, so scaling the estimate by 1 - 2^-21
// keeps it at or below n / f and within 3.25 * 2^-22 of it: the truncated estimate is the
// quotient or, for quotients below 2^20 (M >= 12), one less; for M = 10 and 11 up to four less
// (`more_fixups`, the same for every thread of the launch).
__device__ __forceinline__ uint32_t div_small(uint32_t n, uint32_t f, float rf, bool more_fixups,
                                              uint32_t &rem)
{
    uint32_t q = (uint32_t)(((float)n * rf) * 0.999999523162841796875f);
    uint32_t r = n - (uint32_t)__umul24(q, f);  // q < 2^22 and f < 2^24; q * f <= n
    if (more_fixups) {
#pragma unroll
        for (int i = 0; i < 3; ++i)
            if (r >= f) { r -= f; q += 1u; }
    }
    if (r >= f) { r -= f; q += 1u; }
    rem = r;
    return q;
}

// Chunk c of a lane: rows of sh.tw pixels, g.w apart, each cut into pieces of 8 pixels.
struct ChunkPos {
    uint32_t p, len;
};
__device__ __forceinline__ ChunkPos chunk_pos(const Geo &g, const LaneShape &sh, uint32_t per_row,
                                              uint32_t c)
{
    const uint32_t row = c / per_row, k = c - row * per_row;
    ChunkPos r;
    r.p = sh.first + row * g.w + k * kChunk;
    r.len = min((uint32_t)kChunk, sh.tw - k * kChunk);
    return r;
}

// --------------------------------------------------------------------------------------------
// Encode.  Symbols are pushed last-first (App. A eq. (11)), so the 16-bit words come out in the
// reverse of the order the decoder reads them.  Scratch is laid out per wavefront as
// [word number][thread]: the k-th word of the 64 lanes of a wavefront share a 128-byte line, and
// since neighbouring lanes emit at nearly the same pace a line is complete soon after it is first
// touched.  `lane_cap` is the room every lane has (words); the packer reads a lane's words back
// from the highest number down.
// --------------------------------------------------------------------------------------------
__device__ __forceinline__ size_t lane_scratch_base(uint32_t lane, uint32_t lane_cap)
{
    return (size_t)(lane & ~63u) * lane_cap + (lane & 63u);
}

// kPair (with kVec): every row of every lane is a whole number of 16-pixel pairs of chunks that
// start at multiples of 16 pixels, and the arrays allow 16-byte loads.
// kLine (with kPair, flat lanes): lanes are whole 64-pixel groups that start on 128-byte lines.
// Encodes lane `lane` into its column of the scratch; returns the number of words, the final
// state in `state_out`.
template <bool kVec, bool kPair, bool kLine>
__device__ __forceinline__ uint32_t encode_lane(const Geo &g, uint32_t lane, const uint8_t *__restrict__ img,
                                                const uint16_t *__restrict__ mu,
                                                const int16_t *__restrict__ ls,
                                                const int16_t *__restrict__ coef,
                                                uint16_t *__restrict__ scratch, uint32_t lane_cap,
                                                const LdsTables &tab, uint32_t &state_out)
{
    const LaneShape sh = lane_shape(g, lane);
    const uint32_t m_bits = g.prec_bits;
    const uint32_t spread = (1u << m_bits) - 256u, top = 1u << m_bits;
    const uint32_t per_row = (sh.tw + kChunk - 1) / kChunk;
    const uint32_t chunks = per_row * (sh.npx / sh.tw);

    uint16_t *wout = scratch + lane_scratch_base(lane, lane_cap);  // the lane's next word
    uint32_t nwords = 0;
    uint32_t S = 1u << 16;

    const bool more_fixups = m_bits < 12u;

    auto encode_chunk = [&](const Chunk &ck, const ChunkPos cp) {
        // a chunk never straddles two images when kVec; otherwise take the image per pixel
        uint32_t im = g.by_hw.div(cp.p);
        int a_gr = coef[3 * im], a_br = coef[3 * im + 1], a_bg = coef[3 * im + 2];
        // The chunk in two halves of four pixels, the later half first.  Phase 1 of a half:
        // (cum | freq << 16) of its 12 symbols; nothing there depends on the state, so the
        // evaluations overlap freely.  Phase 2: the serial chain (App. A eq. (11)), last symbol
        // first.  (Halves, and 1/freq formed in phase 2, keep the registers of the whole-line
        // variant at three wavefronts per SIMD.)
        constexpr int kHalf = kChunk / 2;
#pragma unroll
        for (int hb = 1; hb >= 0; --hb) {
            uint32_t cf[3 * kHalf];
#pragma unroll
            for (int ii = 0; ii < kHalf; ++ii) {
                const int i = kHalf * hb + ii;
                if (!kVec && (uint32_t)i < cp.len) {
                    const uint32_t im_i = g.by_hw.div(cp.p + i);
                    if (im_i != im) {
                        im = im_i;
                        a_gr = coef[3 * im]; a_br = coef[3 * im + 1]; a_bg = coef[3 * im + 2];
                    }
                }
                const int e_r = ck.x[i][0] * 256 - ck.m[i][0], e_g = ck.x[i][1] * 256 - ck.m[i][1];
                const int me[3] = {ck.m[i][0], ck.m[i][1] + rsh14_mul(a_gr, e_r),
                                   ck.m[i][2] + rsh14_mul(a_br, e_r) + rsh14_mul(a_bg, e_g)};
#pragma unroll
                for (int ch = 0; ch < 3; ++ch) {
                    const int x = ck.x[i][ch];
                    const uint32_t inv_s = inv_scale(ck.l[i][ch], tab);
                    const int c0 = edge_offset(me[ch]);
                    const uint32_t lo = x == 0 ? 0u : cum_inner_at(x, c0, inv_s, spread, tab);
                    const uint32_t hi = x == 255 ? top : cum_inner_at(x + 1, c0, inv_s, spread, tab);
                    cf[3 * ii + ch] = lo | ((hi - lo) << 16);  // cum < 2^16, freq <= 2^16 - 255
                }
            }
#pragma unroll
            for (int kk = 3 * kHalf - 1; kk >= 0; --kk) {
                if ((uint32_t)(3 * kHalf * hb + kk) < 3u * cp.len) {
                    const uint32_t f = cf[kk] >> 16, lo = cf[kk] & 0xFFFFu;
                    if (S >= (f << (32u - m_bits))) {
                        *wout = (uint16_t)(S & 0xFFFFu);
                        wout += 64;
                        ++nwords;
                        S >>= 16;
                    }
                    uint32_t rem;
                    const uint32_t q = div_small(S, f, __builtin_amdgcn_rcpf((float)f), more_fixups, rem);
                    S = (q << m_bits) + rem + lo;
                }
            }
        }
    };

    if (kVec && kPair) {
        // chunks 2i and 2i + 1 of a lane are neighbours in a row; the right one is coded first
        LineCarry carry;
        for (uint32_t c = chunks; c >= 2u; c -= 2u) {
            const ChunkPos left = chunk_pos(g, sh, per_row, c - 2u);
            ChunkPair raw;
            if (kLine) {
                const uint32_t pair = (c - 2u) >> 1;  // pairs of a flat lane are 16 pixels apart
                feed_pair<true, true>(raw, carry, pair & 3u, sh.first + 16u * (pair & ~3u), img, mu, ls);
            } else {
                load_pair<true>(raw, left.p, img, mu, ls);
            }
            auto half = [&](auto h) {  // h: which chunk of the pair, as a compile-time constant
                constexpr int kH = decltype(h)::value;
                Chunk ck;
                unpack_chunk<true>(ck, raw.wx + 6 * kH, raw.wm + 12 * kH, raw.wl + 12 * kH);
                ChunkPos cp;
                cp.p = left.p + (uint32_t)(kChunk * kH);
                cp.len = (uint32_t)kChunk;
                encode_chunk(ck, cp);
            };
            half(std::integral_constant<int, 1>{});
            half(std::integral_constant<int, 0>{});
        }
    } else {
        for (uint32_t c = chunks; c-- > 0u;) {
            const ChunkPos cp = chunk_pos(g, sh, per_row, c);
            Chunk ck;
            load_chunk<kVec, true>(ck, cp.p, cp.len, img, mu, ls);
            encode_chunk(ck, cp);
        }
    }
    state_out = S;
    return nwords;
}

// --------------------------------------------------------------------------------------------
// One-pass encode: the workgroup that has coded a group of lanes also places them in the
// container.  It needs the bytes of all lanes before the group, which it gets by looking back over
// the descriptors of the groups before it (a group's bytes are published as soon as they are
// known, and the bytes of everything up to and including the group once its workgroup has looked
// back).  Groups are handed out by a ticket counter, so every group with a smaller number has been
// taken by a workgroup that is running, and no workgroup ever waits for a larger number: the
// smallest unfinished group never waits at all.  A workgroup codes its next group before it looks
// back for the one it has just coded, so the groups before that one have usually been coded by
// then and the wait is short; the placing (memory) of one group overlaps the coding (arithmetic)
// of others on the same compute unit.  The wait is bounded all the same: a workgroup that sees an
// empty descriptor for longer than `wait_ticks` of the constant-rate clock raises ST_TIMEOUT, marks
// its own descriptor as abandoned and leaves, and every workgroup that meets an abandoned
// descriptor does the same, so the grid drains.
// --------------------------------------------------------------------------------------------
struct OnePass {
    unsigned long long *desc;  // [groups], zero before the launch; null: two-pass encode
    uint32_t *ticket;          // zero before the launch
    Status *status;
    uint8_t *coded;            // the container: header, offset table, payload
    unsigned long long payload_capacity;  // bytes the payload may take
    unsigned long long wait_ticks;
    uint32_t groups;           // groups of blockDim.x lanes
    uint32_t withhold_first;   // tests of the give-up path: group 0 publishes nothing
    HeaderWords head;
};
constexpr unsigned long long kDescOwn = 1ull, kDescUpTo = 2ull, kDescAbandoned = 3ull;
constexpr int kTailRows = 32;  // word numbers a wavefront moves through its LDS tile at a time

__device__ __forceinline__ void desc_publish(const OnePass &op, uint32_t group, unsigned long long v,
                                             unsigned long long flag)
{
    __hip_atomic_store(&op.desc[group], (v << 2) | flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Bytes of the workgroup's lanes before this thread's lane; *total = bytes of all its lanes.
// Ends with a barrier (after which every word the workgroup's lanes stored is visible to it).
__device__ __forceinline__ unsigned long long group_bytes_before(uint32_t t, unsigned long long bytes,
                                                                 unsigned long long *total)
{
    __shared__ unsigned long long s_wave_sum[kLaneMaxThreads / 64];
    const uint32_t wl = t & 63u, wv = t >> 6, nwaves = blockDim.x >> 6;
    unsigned long long inc = bytes;
    for (int d = 1; d < 64; d <<= 1) {
        const unsigned long long o = __shfl_up(inc, d, 64);
        if (wl >= (uint32_t)d) inc += o;
    }
    __syncthreads();  // the previous use of s_wave_sum is over
    if (wl == 63u) s_wave_sum[wv] = inc;
    __syncthreads();
    unsigned long long before = 0, all = 0;
    for (uint32_t i = 0; i < nwaves; ++i) {
        if (i < wv) before += s_wave_sum[i];
        all += s_wave_sum[i];
    }
    *total = all;
    return before + inc - bytes;
}

// Looks back for group `group` (its own bytes: `total`), then every wavefront places its 64
// lanes.  Returns false if the workgroup has to leave (abandoned wait).
__device__ __forceinline__ bool place_group(const OnePass &op, const Geo &g, uint32_t t, uint32_t group,
                                            unsigned long long total, unsigned long long before,
                                            uint32_t nwords, uint32_t S, uint32_t lane_cap,
                                            const uint16_t *__restrict__ scratch)
{
    __shared__ unsigned long long s_base;
    __shared__ int s_abandon;
    __shared__ __align__(4) uint16_t s_tile[kLaneMaxThreads / 64][kTailRows * kPackTileStride];
    const uint32_t wl = t & 63u, wv = t >> 6;
    const uint32_t lane = group * blockDim.x + t;
    const bool active = lane < g.lanes;

    if (wv == 0u) {
        unsigned long long running = 0;
        int abandon = 0;
        if (group != 0u) {
            long long pos = (long long)group;  // descriptors below pos are still to be added
            const unsigned long long t0 = wall_clock64();
            for (;;) {
                const long long idx = pos - 1 - (long long)wl;
                const unsigned long long d =
                    idx >= 0 ? __hip_atomic_load(&op.desc[idx], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)
                             : kDescUpTo;  // before the first group: nothing, and final
                const unsigned long long f = d & 3ull;
                const unsigned long long m_upto = __ballot(f == kDescUpTo);
                // the descriptors that matter: from the nearest one back to the first final sum
                const unsigned long long need =
                    m_upto ? ((2ull << (__ffsll((long long)m_upto) - 1)) - 1ull) : ~0ull;
                if (__ballot(f == kDescAbandoned) & need) {
                    abandon = 1;
                    break;
                }
                if (__ballot(f == 0ull) & need) {
                    if (wall_clock64() - t0 > op.wait_ticks) {
                        abandon = 2;
                        break;
                    }
                    __builtin_amdgcn_s_sleep(4);
                    continue;
                }
                unsigned long long v = ((need >> wl) & 1ull) ? d >> 2 : 0ull;
                for (int dd = 32; dd >= 1; dd >>= 1) v += __shfl_xor(v, dd, 64);
                running += v;
                if (m_upto) break;
                pos -= 64;
            }
            if (wl == 0u) {
                if (abandon) {
                    desc_publish(op, group, 0ull, kDescAbandoned);
                    if (abandon == 2) atomicMax(&op.status->code, (int)ST_TIMEOUT);
                } else {
                    desc_publish(op, group, running + total, kDescUpTo);
                }
            }
        }
        if (wl == 0u) {
            s_base = running;
            s_abandon = abandon;
        }
    }
    __syncthreads();
    const unsigned long long base = s_base, upto = base + total;
    const bool leave = s_abandon != 0;
    __syncthreads();  // s_base and s_abandon may be written again
    if (leave) return false;
    uint32_t *offsets = reinterpret_cast<uint32_t *>(op.coded + kHeaderBytes);
    uint16_t *payload = reinterpret_cast<uint16_t *>(op.coded + kHeaderBytes + 4ull * ((size_t)g.lanes + 1ull));
    if (group + 1u == op.groups && t == 0u) {
        // the last group knows the size of the payload: header and closing offset
        uint32_t *h = reinterpret_cast<uint32_t *>(op.coded);
        for (int i = 0; i < 12; ++i) h[i] = op.head.w[i];
        h[12] = (uint32_t)upto;
        h[13] = (uint32_t)(upto >> 32);
        h[14] = 0u;
        h[15] = 0u;
        offsets[g.lanes] = (uint32_t)upto;
        op.status->payload_bytes = upto;
    }
    if (upto >= (1ull << 32) || upto > op.payload_capacity) {
        // this group's lanes do not fit: nothing of them is written (the groups before it that did
        // fit have been written inside the capacity); later groups will find the same
        if (t == 0u) atomicMax(&op.status->code, upto >= (1ull << 32) ? (int)ST_TOO_LARGE : (int)ST_CAPACITY);
        return true;
    }

    // From here on a wavefront meets no other: the words of its 64 lanes are rows of 64 in the
    // scratch ([word number][thread]); 32 rows at a time go through an LDS tile and leave as runs
    // of 32 consecutive words of a lane, two lanes per instruction.
    const uint32_t first = (uint32_t)((base + before) >> 1);  // payload word index of the lane's state
    if (active) {
        offsets[lane] = (uint32_t)(base + before);
        payload[first] = (uint16_t)S;
        payload[first + 1u] = (uint16_t)(S >> 16);
    }
    const uint32_t my_nw = active ? nwords : 0u;
    uint32_t max_nw = my_nw;
    for (int dd = 32; dd >= 1; dd >>= 1) max_nw = max(max_nw, (uint32_t)__shfl_xor((int)max_nw, dd, 64));
    const uint16_t *rows = scratch + (size_t)(lane - wl) * lane_cap;
    uint16_t *tile = s_tile[wv];
    const uint32_t half = wl >> 5, u = wl & 31u;
    for (uint32_t k0 = 0; k0 < max_nw; k0 += kTailRows) {
        wave_lds_sync();
        // two rows an instruction, a dword (two lanes) a thread; all rows of the turn are asked for
        // before the first is stored (guarded one by one, every load would wait for the one before);
        // rows past the last one repeat it and are never read
        uint32_t v[kTailRows / 2];
#pragma unroll
        for (int j = 0; j < kTailRows / 2; ++j)
            v[j] = *reinterpret_cast<const uint32_t *>(rows + (size_t)min(k0 + 2u * j + half, max_nw - 1u) * 64u + 2u * u);
#pragma unroll
        for (int j = 0; j < kTailRows / 2; ++j)
            *reinterpret_cast<uint32_t *>(&tile[(2u * j + half) * kPackTileStride + 2u * u]) = v[j];
        wave_lds_sync();
#pragma unroll 4
        for (int j = 0; j < 32; ++j) {  // lanes 2 j and 2 j + 1; thread u of a half has word numbers k0 + u, + 32, ...
            const uint32_t i = 2u * j + half;
            const uint32_t nw_i = (uint32_t)__shfl((int)my_nw, (int)i, 64);
            const uint32_t first_i = (uint32_t)__shfl((int)first, (int)i, 64);
#pragma unroll
            for (uint32_t part = 0; part < (uint32_t)kTailRows; part += 32u) {
                const uint32_t k = k0 + part + u;
                if (k < nw_i) payload[first_i + 2u + (nw_i - 1u - k)] = tile[(part + u) * kPackTileStride + i];
            }
        }
    }
    return true;
}

// kOnePass: the kernel also places the lanes in the container (`op`); otherwise it leaves word
// counts and states for the scan and pack kernels.  (Three wavefronts per SIMD are asked for: the
// one-pass whole-line variant would otherwise settle at 175 registers, two wavefronts.)
template <bool kOnePass, bool kVec, bool kPair, bool kLine = false>
__global__ __launch_bounds__(kLaneMaxThreads) __attribute__((amdgpu_waves_per_eu(3))) void k_encode_lanes(Geo g, const uint8_t *__restrict__ img,
                               const uint16_t *__restrict__ mu, const int16_t *__restrict__ ls,
                               const int16_t *__restrict__ coef, uint16_t *__restrict__ scratch,
                               uint32_t lane_cap, uint32_t *__restrict__ lane_words,
                               uint32_t *__restrict__ lane_state, OnePass op)
{
    __shared__ LdsTables tab;
    load_tables(tab);  // ends with a barrier
    if (!kOnePass) {
        const uint32_t lane = blockIdx.x * blockDim.x + threadIdx.x;
        if (lane >= g.lanes) return;
        uint32_t S;
        const uint32_t nwords = encode_lane<kVec, kPair, kLine>(g, lane, img, mu, ls, coef, scratch, lane_cap, tab, S);
        lane_words[lane] = nwords;
        lane_state[lane] = S;
        return;
    }
    // what the group coded last still needs: kept in LDS while the next group is coded
    __shared__ uint32_t s_ticket;
    __shared__ uint32_t s_words[kLaneMaxThreads], s_state[kLaneMaxThreads];
    __shared__ unsigned long long s_before[kLaneMaxThreads];
    bool have = false;
    uint32_t last_group = 0u;
    unsigned long long last_total = 0ull;
    for (;;) {
        // the thread index afresh in every round: nothing derived from it (LDS addresses of the
        // arrays below, wavefront numbers) is to be carried in registers through the coding
        uint32_t t = threadIdx.x;
        asm volatile("" : "+v"(t));
        if (t == 0u) s_ticket = atomicAdd(op.ticket, 1u);
        __syncthreads();
        const uint32_t group = s_ticket;
        if (group < op.groups) {
            const uint32_t lane = group * blockDim.x + t;
            uint32_t nwords = 0u, S = 0u;
            if (lane < g.lanes)
                nwords = encode_lane<kVec, kPair, kLine>(g, lane, img, mu, ls, coef, scratch, lane_cap, tab, S);
            t = threadIdx.x;
            asm volatile("" : "+v"(t));  // (as above: what follows starts from the thread index again)
            unsigned long long total;
            const bool coded = group * blockDim.x + t < g.lanes;
            const unsigned long long before = group_bytes_before(t, coded ? 4ull + 2ull * nwords : 0ull, &total);
            if (t == 0u && !(group == 0u && op.withhold_first))
                desc_publish(op, group, total, group == 0u ? kDescUpTo : kDescOwn);
            if (have && !place_group(op, g, t, last_group, last_total, s_before[t], s_words[t], s_state[t],
                                     lane_cap, scratch))
                return;
            s_words[t] = nwords;  // a thread reads back only what it wrote itself
            s_state[t] = S;
            s_before[t] = before;
            last_group = group;
            last_total = total;
            have = true;
        } else {
            if (have) place_group(op, g, t, last_group, last_total, s_before[t], s_words[t], s_state[t], lane_cap, scratch);
            return;
        }
    }
}

// --------------------------------------------------------------------------------------------
// Decode.  The symbol is found by an 8-step bisection on C(k) (App. A names a binary search).
// --------------------------------------------------------------------------------------------

// A lane's 16-bit words, fetched as aligned 32-byte pairs of 16-byte pieces, a piece ahead of
// their use: a refill of the state (App. A eq. (12)) never waits for memory, and a 128-byte line
// of the stream is asked for four times instead of once per word.  A piece is loaded only if it
// starts below `lim`, the end of the container: it then holds at least one byte of it and cannot
// leave the container's last page.  Words beyond the lane's own end are whatever follows; a lane
// that takes them fails its final check of the number of words taken.
struct WordStream {
    uint32_t w0, w1, w2, w3;  // the words not yet taken from the current piece, lowest first
    uint4 x, y;               // the piece after the current one; the piece after that when the
                              // current one is the second of its pair
    uint32_t next;            // word offset from `base` of the next pair to load
    uint32_t count;           // words of the current pair skipped or taken, plus 16 per pair done:
                              // bits 0..2 count within a piece, bit 3 tells the piece of the pair

    // the 8 words at word offset `off` of the 32-byte aligned `base`, if they start below `lim`
    __device__ __forceinline__ static uint4 fetch(const uint16_t *base, uint32_t off, uint32_t lim)
    {
        return off < lim ? *reinterpret_cast<const uint4 *>(base + off) : make_uint4(0u, 0u, 0u, 0u);
    }
    // the lane's first word is at word offset `first` < lim
    __device__ __forceinline__ void open(const uint16_t *base, uint32_t first, uint32_t lim)
    {
        const uint32_t q = first & ~7u;
        const uint4 c = fetch(base, q, lim);
        x = fetch(base, q + 8u, lim);
        y = make_uint4(0u, 0u, 0u, 0u);
        if ((first & 8u) != 0u) y = fetch(base, q + 16u, lim);  // second piece: x, y are the next pair
        next = (first & ~15u) + 16u + (first & 8u) * 2u;
        const uint32_t skip = first & 7u;  // words of the first piece before `first`
        unsigned long long lo = (unsigned long long)c.x | ((unsigned long long)c.y << 32);
        unsigned long long hi = (unsigned long long)c.z | ((unsigned long long)c.w << 32);
        if (skip >= 4u) {
            lo = hi >> (16u * (skip - 4u));
            hi = 0ull;
        } else if (skip != 0u) {
            lo = (lo >> (16u * skip)) | (hi << (64u - 16u * skip));
            hi >>= 16u * skip;
        }
        w0 = (uint32_t)lo; w1 = (uint32_t)(lo >> 32); w2 = (uint32_t)hi; w3 = (uint32_t)(hi >> 32);
        count = first & 15u;
    }
    __device__ __forceinline__ uint32_t take(const uint16_t *base, uint32_t lim)
    {
        const uint32_t wd = w0 & 0xFFFFu;
        w0 = __builtin_amdgcn_alignbit(w1, w0, 16);
        w1 = __builtin_amdgcn_alignbit(w2, w1, 16);
        w2 = __builtin_amdgcn_alignbit(w3, w2, 16);
        w3 >>= 16;
        if ((++count & 7u) == 0u) {
            w0 = x.x; w1 = x.y; w2 = x.z; w3 = x.w;
            if ((count & 8u) != 0u) {  // now in the second piece of a pair: fetch the next pair
                x = fetch(base, next, lim);
                y = fetch(base, next + 8u, lim);
                next += 16u;
            } else {
                x = y;
            }
        }
        return wd;
    }
    // words taken by a stream opened at word offset `first`
    __device__ __forceinline__ uint32_t taken(uint32_t first) const { return count - (first & 15u); }
};

// The same stream for a decoder that works in chunks of at most kRingChunk symbols: the words wait
// in a ring of 64 per thread in LDS.  Before a chunk the ring is looked at: while it still holds 32
// words or more nothing happens (a chunk takes at most 24), otherwise it is filled to the brim with
// aligned 16-byte loads, four to eight at once, together with the chunk's parameter loads.  No
// refill inside the chunk ever touches memory or branches on the fill level, and a 128-byte line of
// the stream is asked for by one or two fills, not by eight.  A thread's 64 words lie side by side
// (rows of 33 dwords, so that the threads of a wavefront start in different banks): the word at
// stream position pos is one 16-bit read at (pos mod 64), fetched ahead of its use.
constexpr int kRingChunk = 24;
constexpr int kRingPieces = 8;                      // 16-byte pieces per thread: 64 words
constexpr int kRingWordsHeld = 8 * kRingPieces;
constexpr int kRingRow = kRingWordsHeld + 2;        // 16-bit elements per thread, padding included
constexpr int kRingMaxThreads = kLaneMaxThreads;
static_assert(3 * kChunk <= kRingChunk, "a chunk must not take more words than the ring guarantees");

struct WordRing {
    typedef uint32_t __attribute__((may_alias)) word_pair;  // two ring words stored at once
    uint16_t *row;      // this thread's 64 words
    uint32_t pos;       // word offset (from the 16-byte aligned `base`) of the next word
    uint32_t filled;    // word offset up to which the ring holds the stream: a multiple of 8
    uint32_t nextw;     // the word at `pos`

    __device__ __forceinline__ static uint4 fetch(const uint16_t *base, uint32_t off, uint32_t lim)
    {
        return off < lim ? *reinterpret_cast<const uint4 *>(base + off) : make_uint4(0u, 0u, 0u, 0u);
    }
    __device__ __forceinline__ uint32_t peek() const { return row[pos & (kRingWordsHeld - 1)]; }
    // Brings `filled` to (pos rounded down to 8) + 64 if fewer than 32 words are held.
    __device__ __forceinline__ void fill(const uint16_t *base, uint32_t lim)
    {
        if ((int)(filled - pos) < 32) {  // signed: at the opening `filled` may lie below `pos`
            const uint32_t want = (pos & ~7u) + kRingWordsHeld;
            const uint32_t n = (want - filled) >> 3;  // 4..8
            uint4 piece[kRingPieces];
#pragma unroll
            for (int i = 0; i < kRingPieces; ++i)
                if ((uint32_t)i < n) piece[i] = fetch(base, filled + 8u * i, lim);
#pragma unroll
            for (int i = 0; i < kRingPieces; ++i)
                if ((uint32_t)i < n) {
                    word_pair *d = reinterpret_cast<word_pair *>(row + ((filled + 8u * i) & (kRingWordsHeld - 1)));
                    d[0] = piece[i].x; d[1] = piece[i].y; d[2] = piece[i].z; d[3] = piece[i].w;
                }
            filled = want;
        }
        nextw = peek();
    }
    // the lane's first word is at word offset `first` < lim
    __device__ __forceinline__ void open(uint16_t *ring, const uint16_t *base, uint32_t first, uint32_t lim)
    {
        row = ring + threadIdx.x * kRingRow;
        pos = first;
        filled = first & ~7u;
        fill(base, lim);
    }
    __device__ __forceinline__ uint32_t take()
    {
        const uint32_t wd = nextw;
        ++pos;
        nextw = peek();  // at most kRingChunk takes between fills: pos stays below `filled`
        return wd;
    }
};

template <bool kVec, bool kPair, bool kLine = false>
__global__ __launch_bounds__(kLaneMaxThreads) void k_decode_lanes(Geo g, const uint8_t *__restrict__ coded,
                               const uint16_t *__restrict__ mu, const int16_t *__restrict__ ls,
                               const int16_t *__restrict__ coef, uint8_t *__restrict__ out,
                               int *__restrict__ status_code,
                               const unsigned long long *__restrict__ status_payload)
{
    __shared__ LdsTables tab;
    __shared__ __align__(16) uint16_t ring[kRingRow * kRingMaxThreads];  // [thread][word]
    load_tables(tab);
    if (*status_code != 0) return;  // uniform: written by an earlier kernel
    const uint32_t lane = blockIdx.x * blockDim.x + threadIdx.x;
    if (lane >= g.lanes) return;
    const LaneShape sh = lane_shape(g, lane);
    const uint32_t m_bits = g.prec_bits;
    const uint32_t spread = (1u << m_bits) - 256u, mask = (1u << m_bits) - 1u;
    const uint32_t payload_bytes = (uint32_t)*status_payload;
    const uint32_t per_row = (sh.tw + kChunk - 1) / kChunk;
    const uint32_t chunks = per_row * (sh.npx / sh.tw);

    const uint32_t *offsets = reinterpret_cast<const uint32_t *>(coded + 64);
    const uint16_t *payload =
        reinterpret_cast<const uint16_t *>(coded + 64 + 4ull * ((size_t)g.lanes + 1));
    const uint32_t begin = offsets[lane], end = offsets[lane + 1];
    if (end < begin || end > payload_bytes || end - begin < 4u || ((begin | end) & 1u)) {
        atomicMax(status_code, 6);
        return;
    }
    // word offsets from the last 16-byte boundary at or below the payload (the payload is < 4 GiB)
    const uint32_t adj = (uint32_t)(reinterpret_cast<uintptr_t>(payload) & 15u);
    const uint16_t *base = reinterpret_cast<const uint16_t *>(reinterpret_cast<const uint8_t *>(payload) - adj);
    const uint32_t first = (adj + begin) >> 1;
    const uint32_t lim = (uint32_t)(((unsigned long long)adj + payload_bytes + 1ull) >> 1);
    WordRing words;
    words.open(ring, base, first, lim);
    uint32_t S = words.take();
    S |= words.take() << 16;

    // decodes the chunk into its 24 bytes (6 dwords)
    // tiles and flat lanes no longer than an image lie in one image: its coefficients are loaded once
    auto decode_chunk = [&](const Chunk &ck, const ChunkPos cp, uint32_t *wout) {
        // (the plain division on purpose: with g.by_hw the whole-line variant needs 171 registers
        // instead of 167 and loses its third wavefront per SIMD)
        uint32_t im = cp.p / g.hw;
        int a_gr = coef[3 * im], a_br = coef[3 * im + 1], a_bg = coef[3 * im + 2];
#pragma unroll
        for (int b = 0; b < 6; ++b) wout[b] = 0u;
#pragma unroll
        for (int i = 0; i < kChunk; ++i) {
            if ((uint32_t)i < cp.len) {
                if (!kVec) {
                    const uint32_t im_i = (cp.p + i) / g.hw;
                    if (im_i != im) {
                        im = im_i;
                        a_gr = coef[3 * im]; a_br = coef[3 * im + 1]; a_bg = coef[3 * im + 2];
                    }
                }
                int x[3] = {0, 0, 0};
#pragma unroll
                for (int ch = 0; ch < 3; ++ch) {
                    int me = ck.m[i][0];
                    if (ch == 1) me = ck.m[i][1] + rsh14_mul(a_gr, (x[0] * 256 - ck.m[i][0]));
                    if (ch == 2)
                        me = ck.m[i][2] + rsh14_mul(a_br, (x[0] * 256 - ck.m[i][0])) +
                             rsh14_mul(a_bg, (x[1] * 256 - ck.m[i][1]));
                    const uint32_t inv_s = inv_scale(ck.l[i][ch], tab);
                    const uint32_t slot = S & mask;
                    const int c0 = edge_offset(me);
                    // the symbol is in lo .. lo + 2 * step - 1, and c_hi = C(lo + 2 * step)
                    int lo = 0;
                    uint32_t c_lo = 0u, c_hi = 1u << m_bits;
#pragma unroll
                    for (int step = 128; step >= 1; step >>= 1) {
                        const uint32_t cm = cum_inner_at(lo + step, c0, inv_s, spread, tab);
                        const bool ge = cm <= slot;
                        lo = ge ? lo + step : lo;
                        c_lo = ge ? cm : c_lo;
                        c_hi = ge ? c_hi : cm;
                    }
                    x[ch] = lo;
                    // App. A eq. (12)
                    // the mass is at most 2^16 and S >> M below 2^22: a 24-bit multiply is exact
                    S = (uint32_t)__umul24(c_hi - c_lo, S >> m_bits) + slot - c_lo;
                    if (S < (1u << 16)) S = (S << 16) | words.take();
                    const int b = 3 * i + ch;
                    wout[b >> 2] |= (uint32_t)lo << (8 * (b & 3));
                }
            }
        }
    };

    if (kVec && kPair) {
        // two neighbouring chunks per round: 96 bytes of each parameter array in, 48 bytes out
        LineCarry carry;
        for (uint32_t c = 0; c + 2u <= chunks; c += 2u) {
            const ChunkPos left = chunk_pos(g, sh, per_row, c);
            ChunkPair raw;
            if (kLine) {
                const uint32_t pair = c >> 1;
                feed_pair<false, false>(raw, carry, pair & 3u, sh.first + 16u * (pair & ~3u), nullptr, mu, ls);
            } else {
                load_pair<false>(raw, left.p, nullptr, mu, ls);
            }
            uint32_t wout[12];
            auto half = [&](auto h) {  // h: which chunk of the pair, as a compile-time constant
                constexpr int kH = decltype(h)::value;
                words.fill(base, lim);
                Chunk ck;
                unpack_chunk<false>(ck, nullptr, raw.wm + 12 * kH, raw.wl + 12 * kH);
                ChunkPos cp;
                cp.p = left.p + (uint32_t)(kChunk * kH);
                cp.len = (uint32_t)kChunk;
                decode_chunk(ck, cp, wout + 6 * kH);
            };
            half(std::integral_constant<int, 0>{});
            half(std::integral_constant<int, 1>{});
            uint4 *po = reinterpret_cast<uint4 *>(out + (size_t)left.p * 3);
            po[0] = make_uint4(wout[0], wout[1], wout[2], wout[3]);
            po[1] = make_uint4(wout[4], wout[5], wout[6], wout[7]);
            po[2] = make_uint4(wout[8], wout[9], wout[10], wout[11]);
        }
    } else {
        for (uint32_t c = 0; c < chunks; ++c) {
            const ChunkPos cp = chunk_pos(g, sh, per_row, c);
            Chunk ck;
            load_chunk<kVec, false>(ck, cp.p, cp.len, nullptr, mu, ls);
            words.fill(base, lim);  // its loads travel with the chunk's
            uint32_t wout[6];
            decode_chunk(ck, cp, wout);
            const size_t s = (size_t)cp.p * 3;
            if (kVec && cp.len == (uint32_t)kChunk) {
                uint2 *po = reinterpret_cast<uint2 *>(out + s);
                po[0] = make_uint2(wout[0], wout[1]);
                po[1] = make_uint2(wout[2], wout[3]);
                po[2] = make_uint2(wout[4], wout[5]);
            } else {
#pragma unroll
                for (int b = 0; b < 3 * kChunk; ++b)
                    if ((uint32_t)b < 3u * cp.len) out[s + b] = (uint8_t)(wout[b >> 2] >> (8 * (b & 3)));
            }
        }
    }
    if (S != (1u << 16) || words.pos - first != (end - begin) >> 1) atomicMax(status_code, 6);
}

}  // namespace pilc
