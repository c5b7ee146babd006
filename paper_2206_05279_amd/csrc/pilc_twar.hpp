// The Three-Way Auto-regressive residual transform of Sec. 3.1 (eqs. (2)-(4)) for gfx950.
//
//   R(u,v) is predicted from R(u-1,v-1), R(u-1,v), R(u,v-1)   (up-left, up, left)
//   G(u,v)                from G(u,v-1),   R(u,v-1), R(u,v)     (left G, left R, this pixel's R)
//   B(u,v)                from B(u,v-1),   G(u,v-1), G(u,v)     (left B, left G, this pixel's G)
// with three weights and a bias each, zero padding above and to the left, and the residual
// r = (x - x^) mod 256.  Forward, every pixel is independent (k_twar_forward).  Inverse, a pixel
// needs its left, upper and upper-left neighbours: the paper's schedule runs the red channel along
// anti-diagonals and then green and blue column by column; here a wavefront takes 64 rows, one
// per thread, and walks the anti-diagonals once, recovering R, G and B of a pixel in the same
// step (G and B only need values of the same row, which the thread already holds), with the two
// values a row needs from the row above passed down by a cross-lane shift (k_twar_inverse).
//
// Included at the end of pilc.hip.
#pragma once

namespace pilc {

struct TwarK {
    int w[3][3];  // Q2.14
    int bias[3];  // Q8.14
};

__device__ __forceinline__ int twar_predict(const TwarK &p, int ch, int a, int b, int c)
{
    // 16-bit weights times 8-bit values: 24-bit multiplies are exact and run at full rate
    const int acc = __mul24(p.w[ch][0], a) + __mul24(p.w[ch][1], b) + __mul24(p.w[ch][2], c) + p.bias[ch] + 8192;
    return min(max(acc >> 14, 0), 255);  // arithmetic shift: floor
}

// (a + b) mod 256 for a pixel value: one instruction that adds and keeps the low byte.
__device__ __forceinline__ int add_low_byte(int a, int b)
{
    int r;
    asm("v_add_u32_sdwa %0, %1, %2 dst_sel:BYTE_0 dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:DWORD"
        : "=v"(r)
        : "v"(a), "v"(b));
    return r;
}

// (byte kByte of a + b) mod 256
template <int kByte>
__device__ __forceinline__ int add_byte_of(uint32_t a, int b)
{
    int r;
    if (kByte == 0)
        asm("v_add_u32_sdwa %0, %1, %2 dst_sel:BYTE_0 dst_unused:UNUSED_PAD src0_sel:BYTE_0 src1_sel:DWORD" : "=v"(r) : "v"(a), "v"(b));
    else if (kByte == 1)
        asm("v_add_u32_sdwa %0, %1, %2 dst_sel:BYTE_0 dst_unused:UNUSED_PAD src0_sel:BYTE_1 src1_sel:DWORD" : "=v"(r) : "v"(a), "v"(b));
    else
        asm("v_add_u32_sdwa %0, %1, %2 dst_sel:BYTE_0 dst_unused:UNUSED_PAD src0_sel:BYTE_2 src1_sel:DWORD" : "=v"(r) : "v"(a), "v"(b));
    return r;
}

// One thread per pixel.  A workgroup takes 256 / w whole rows (or one row, in steps of 256
// pixels, when w > 256); neighbouring threads read neighbouring bytes and the row above comes from
// the caches.
__global__ __launch_bounds__(256) void k_twar_forward(TwarK p, uint32_t rows, uint32_t h, uint32_t w,
                                                      uint32_t rows_per_block,
                                                      const uint8_t *__restrict__ img,
                                                      uint8_t *__restrict__ res)
{
    const uint32_t local = threadIdx.x / w, v0 = threadIdx.x % w;
    const uint32_t row = blockIdx.x * rows_per_block + local;
    if (local >= rows_per_block || row >= rows) return;
    const uint32_t u = row % h;
    const size_t row_off = (size_t)row * w * 3u;
    for (uint32_t v = v0; v < w; v += 256u) {  // one turn unless w > 256
        const uint8_t *x = img + row_off + 3u * v;
        const int r0 = x[0], g0 = x[1], b0 = x[2];
        int rl = 0, gl = 0, bl = 0, ru = 0, rul = 0;
        if (v > 0) {
            rl = x[-3];
            gl = x[-2];
            bl = x[-1];
        }
        if (u > 0) {
            ru = x[-3ll * (long long)w];
            if (v > 0) rul = x[-3ll * (long long)w - 3];
        }
        uint8_t *o = res + row_off + 3u * v;
        o[0] = (uint8_t)(r0 - twar_predict(p, 0, rul, ru, rl));
        o[1] = (uint8_t)(g0 - twar_predict(p, 1, gl, rl, r0));
        o[2] = (uint8_t)(b0 - twar_predict(p, 2, bl, gl, g0));
    }
}

// Byte b (-4 <= b < 12) of the 16 bytes {prev, c0, c1, c2}, b = 0 being the first byte of c0.
template <int B>
__device__ __forceinline__ int byte_at(uint32_t prev, uint32_t c0, uint32_t c1, uint32_t c2)
{
    constexpr int i = B + 4;
    const uint32_t word = i < 4 ? prev : (i < 8 ? c0 : (i < 12 ? c1 : c2));
    return (int)((word >> (8 * (i & 3))) & 255u);
}

// Four pixels (12 bytes, three dwords) per thread, for rows that are a whole number of such
// groups in 4-byte aligned arrays: dword loads and stores only.
__global__ __launch_bounds__(256) void k_twar_forward4(TwarK p, uint32_t groups, FastDiv by_h,
                                                       FastDiv by_groups_per_row,
                                                       const uint32_t *__restrict__ img,
                                                       uint32_t *__restrict__ res)
{
    const uint32_t gi = blockIdx.x * blockDim.x + threadIdx.x;
    if (gi >= groups) return;
    const uint32_t groups_per_row = by_groups_per_row.d;
    const uint32_t row = by_groups_per_row.div(gi), k = gi - row * groups_per_row;
    const uint32_t u = row - by_h.div(row) * by_h.d;
    const uint32_t *x = img + (size_t)gi * 3u;
    const uint32_t c0 = x[0], c1 = x[1], c2 = x[2];
    const uint32_t prev = k > 0 ? x[-1] : 0u;  // the pixel to the left of the group (its last 3 bytes)
    uint32_t u0 = 0u, u1 = 0u, u2 = 0u, uprev = 0u;
    if (u > 0) {
        const uint32_t *y = x - (size_t)groups_per_row * 3u;
        u0 = y[0];
        u1 = y[1];
        u2 = y[2];
        uprev = k > 0 ? y[-1] : 0u;
    }
    uint32_t out[3] = {0u, 0u, 0u};
#define PILC_TWAR_PIXEL(J)                                                                         \
    {                                                                                              \
        const int r0 = byte_at<3 * J>(prev, c0, c1, c2), g0 = byte_at<3 * J + 1>(prev, c0, c1, c2); \
        const int b0 = byte_at<3 * J + 2>(prev, c0, c1, c2);                                       \
        const int rl = byte_at<3 * J - 3>(prev, c0, c1, c2), gl = byte_at<3 * J - 2>(prev, c0, c1, c2); \
        const int bl = byte_at<3 * J - 1>(prev, c0, c1, c2);                                       \
        const int ru = byte_at<3 * J>(uprev, u0, u1, u2), rul = byte_at<3 * J - 3>(uprev, u0, u1, u2); \
        const uint32_t e0 = (uint32_t)(r0 - twar_predict(p, 0, rul, ru, rl)) & 255u;               \
        const uint32_t e1 = (uint32_t)(g0 - twar_predict(p, 1, gl, rl, r0)) & 255u;                \
        const uint32_t e2 = (uint32_t)(b0 - twar_predict(p, 2, bl, gl, g0)) & 255u;                \
        out[(3 * J) >> 2] |= e0 << (8 * ((3 * J) & 3));                                            \
        out[(3 * J + 1) >> 2] |= e1 << (8 * ((3 * J + 1) & 3));                                    \
        out[(3 * J + 2) >> 2] |= e2 << (8 * ((3 * J + 2) & 3));                                    \
    }
    PILC_TWAR_PIXEL(0)
    PILC_TWAR_PIXEL(1)
    PILC_TWAR_PIXEL(2)
    PILC_TWAR_PIXEL(3)
#undef PILC_TWAR_PIXEL
    uint32_t *o = res + (size_t)gi * 3u;
    o[0] = out[0];
    o[1] = out[1];
    o[2] = out[2];
}

// A flat copy by one wavefront: `total` >= 1 elements, element lane + 64 i, four of them a turn, so
// that four loads are under way together (taken one at a time, every load waits for the one
// before).  Loads past the end read the last element again instead of being skipped (a register
// that is only sometimes written costs more in moves than the load it saves); stores past the end
// are skipped.
template <typename T>
__device__ __forceinline__ void flat_copy(const T *__restrict__ src, T *__restrict__ dst, uint32_t total, uint32_t lane)
{
    for (uint32_t base = 0; base < total; base += 256u) {  // the same for the whole wavefront
        T v[4];
#pragma unroll
        for (uint32_t k = 0; k < 4u; ++k) v[k] = src[min(base + lane + 64u * k, total - 1u)];
#pragma unroll
        for (uint32_t k = 0; k < 4u; ++k)
            if (base + lane + 64u * k < total) dst[base + lane + 64u * k] = v[k];
    }
}

// A wavefront per group of up to 64 rows: whole images when h <= 64 (64 / h of them side by side),
// else the bands of 64 rows of one image one after the other, the last row's red values of a band
// kept in LDS for the first row of the next.  kTile: the group's residuals are copied to LDS
// first and the pixels copied back at the end, so that global memory only sees whole, coalesced
// rows; without it every thread reads and writes its row in place in global memory.  The tile is
// the group exactly as it lies in memory (its rows are contiguous there), copied as a flat run of
// elements of type T (16 bytes, 4 bytes or single bytes: what the sizes and addresses allow); the
// skew between rows keeps the threads' accesses on different banks without any padding.
constexpr int kTwarWaves = 4;

template <bool kTile, typename T>
__global__ __launch_bounds__(64 * kTwarWaves) void k_twar_inverse(TwarK p, uint32_t n, uint32_t h,
                                                                  uint32_t w, uint32_t last_bytes,
                                                                  const uint8_t *__restrict__ res,
                                                                  uint8_t *__restrict__ img)
{
    extern __shared__ uint8_t twar_lds[];
    const uint32_t wave = threadIdx.x >> 6, lane = threadIdx.x & 63u;
    const uint32_t per = h <= 64u ? 64u / h : 1u;          // images side by side in a wavefront
    const uint32_t groups = (n + per - 1u) / per;
    const uint32_t g = blockIdx.x * kTwarWaves + wave;
    if (g >= groups) return;
    const uint32_t bands = h <= 64u ? 1u : (h + 63u) / 64u;
    // LDS of this wavefront: [last_bytes >= w, a multiple of 16: red values of the row above a band][tile]
    const uint32_t row_stride = 3u * w;
    uint8_t *lastrow = twar_lds + (size_t)wave * (last_bytes + (kTile ? 64u * row_stride : 0u));
    uint8_t *tile = lastrow + last_bytes;
    const size_t row_bytes = (size_t)w * 3u;

    for (uint32_t band = 0; band < bands; ++band) {
        // this thread's row
        uint32_t image, u;
        bool have;
        if (h <= 64u) {
            image = g * per + lane / h;
            u = lane % h;
            have = lane < per * h && image < n;
        } else {
            image = g;
            u = band * 64u + lane;
            have = u < h;
        }
        const size_t row_off = ((size_t)image * h + u) * row_bytes;
        const uint32_t rows_here = h <= 64u ? min(per, n - g * per) * h : min(64u, h - band * 64u);
        if (kTile) {  // the group's rows are contiguous in memory: copy them row by row
            const size_t first = h <= 64u ? (size_t)g * per * h * row_bytes : ((size_t)g * h + band * 64u) * row_bytes;
            wave_lds_sync();
            flat_copy(reinterpret_cast<const T *>(res + first), reinterpret_cast<T *>(tile),
                      rows_here * row_stride / (uint32_t)sizeof(T), lane);
            wave_lds_sync();
        }
        const bool top = u == 0u;                // the row above is padding: its two weights are zero here
        const int w_upleft = top ? 0 : p.w[0][0], w_up = top ? 0 : p.w[0][1];
        // the rounding biases in vector registers of their own: as scalar operands they would be
        // copied into one at every use (a multiply-add takes one scalar operand, and has a weight)
        int bias_r = p.bias[0] + 8192, bias_g = p.bias[1] + 8192, bias_b = p.bias[2] + 8192;
        asm volatile("" : "+v"(bias_r), "+v"(bias_g), "+v"(bias_b));
        // likewise the weights of the multiply-adds that are written out below
        int w_g0 = p.w[1][0], w_g1 = p.w[1][1], w_b0 = p.w[2][0], w_b1 = p.w[2][1];
        asm volatile("" : "+v"(w_g0), "+v"(w_g1), "+v"(w_b0), "+v"(w_b1));
        const bool from_lds = lane == 0u && !top;  // the row above belongs to the previous band
        int rl = 0, gl = 0, bl = 0;
        int above = 0;  // the red value above the pixel decoded last: above-left of the next one
        // row k of an image (or band) runs k positions behind row 0: w + rows - 1 steps in all
        const uint32_t skew = h <= 64u ? lane % h : lane;
        const uint32_t steps = w + min(h, 64u) - 1u;
        for (uint32_t d = 0; d < steps; ++d) {
            int up = __builtin_amdgcn_update_dpp(0, rl, 0x138 /* wave_shr:1 */, 0xF, 0xF, true);
            const int v = (int)d - (int)skew;
            const bool on = have && v >= 0 && v < (int)w;
            if (from_lds && on) up = lastrow[v];
            if (on) {
                int r0, r1, r2;
                if (kTile) {
                    const uint8_t *s = tile + lane * row_stride + 3u * v;
                    r0 = s[0];
                    r1 = s[1];
                    r2 = s[2];
                } else {
                    const uint8_t *s = res + row_off + 3u * v;
                    r0 = s[0];
                    r1 = s[1];
                    r2 = s[2];
                }
                // Three multiply-adds each.  What only needs the pixel to the left comes first, so
                // that each new value can take the place of the one it replaces; the operand that
                // arrives last (the value just decoded) goes into the last multiply-add.
                auto clamp8 = [](int acc) { return min(max(acc >> 14, 0), 255); };
                const int tg = mad_i24(w_g1, rl, mad_i24(w_g0, gl, bias_g));
                const int tb = mad_i24(w_b1, gl, mad_i24(w_b0, bl, bias_b));
                const int tr = mad_i24(w_up, up, mad_i24(w_upleft, above, bias_r));
                const int xr = add_low_byte(r0, clamp8(__mul24(p.w[0][2], rl) + tr));
                const int xg = add_low_byte(r1, clamp8(__mul24(p.w[1][2], xr) + tg));
                const int xb = add_low_byte(r2, clamp8(__mul24(p.w[2][2], xg) + tb));
                if (kTile) {
                    uint8_t *o = tile + lane * row_stride + 3u * v;
                    o[0] = (uint8_t)xr;
                    o[1] = (uint8_t)xg;
                    o[2] = (uint8_t)xb;
                } else {
                    uint8_t *o = img + row_off + 3u * v;
                    o[0] = (uint8_t)xr;
                    o[1] = (uint8_t)xg;
                    o[2] = (uint8_t)xb;
                }
                // the last row of a band leaves its red values for the next band; it runs 63
                // positions behind the first row's reads of the same buffer
                if (bands > 1u && lane == 63u) lastrow[v] = (uint8_t)xr;
                above = up;
                rl = xr;
                gl = xg;
                bl = xb;
            }
        }
        if (kTile) {
            const size_t first = h <= 64u ? (size_t)g * per * h * row_bytes : ((size_t)g * h + band * 64u) * row_bytes;
            wave_lds_sync();
            flat_copy(reinterpret_cast<const T *>(tile), reinterpret_cast<T *>(img + first),
                      rows_here * row_stride / (uint32_t)sizeof(T), lane);
        }
        wave_lds_sync();
    }
}

// Images taller than 64 rows whose rows are whole 16-pixel chunks in 16-byte aligned arrays: a
// thread per row, every wavefront 64 rows, all wavefronts of a workgroup under way at once.
// Thread t of the workgroup runs t + 16 (t / 64) positions behind thread 0, so inside a wavefront
// a row still gets the two values it needs from the row above by a cross-lane shift, and the first
// row of a wavefront finds them in LDS, where the last row of the wavefront above left them 17
// steps earlier; a workgroup barrier every 16 steps separates the two.  A row passes through a
// three-chunk ring in LDS (a chunk is 16 pixels, 48 bytes): the chunk the row is in, the next one,
// and the one it left, which is written back and then filled again; what is to fill it was asked
// for a turn earlier and waits in registers.  The chunks of a wavefront's 64 rows are moved as 192
// pieces of 16 bytes, three neighbouring threads taking the 48 contiguous bytes of one row.  The
// work goes in blocks of 16 steps: barrier, chunk turn, then 16 steps without a branch on anything
// but the loop count (a step used to spend more time in its dozen branches than in its arithmetic).
//
// kBands false: a workgroup per image, every wavefront turns the chunks of its own rows before its
// 16 steps; images with more rows than a workgroup has threads go in rounds, the last row's red
// values of a round kept in LDS for the first row of the next.
// kBands true (few images): an image is cut into bands of rows, a workgroup per band, so that one
// image keeps several compute units busy.  Here the workgroup has a second set of wavefronts, the
// movers: mover k turns the chunks of wavefront k's rows while wavefront k decodes (with one
// or two decoding wavefronts on a SIMD a turn's trip to memory and back, a third of a block's
// time, is not hidden by anything else).  The first row of a band needs the red values of the last
// row of the band above, which belongs to another workgroup: the mover of that row publishes, after
// every chunk it has written back to the image, how many chunks of the row are final (a counter per
// band in global memory; the row's bytes and the count are stored at device scope, the count once
// no store of the wavefront is outstanding), and three threads of the first mover of the band below
// fetch the chunk of that row two chunks ahead of their first row from the image as soon as the
// counter allows (acquire at device scope).  Bands number themselves with a ticket taken at
// their start (image-major), so the band above is always a workgroup that is already running, and
// it never waits for the band below.  The wait is bounded by the constant-rate clock; a band that
// gives up sets an abort word, every band that sees it while waiting leaves too, and the host
// returns PILC_E_TIMEOUT.
constexpr int kTallLag = 16;         // steps between barriers = extra lag per wavefront
constexpr int kTallChunk = 48;       // bytes of a chunk of 16 pixels
constexpr int kTallRing = 3 * kTallChunk;
constexpr int kTallStride = kTallRing + 4;  // LDS bytes per thread: 37 dwords, odd
constexpr int kTallMaxThreads = 768;
constexpr int kTallLead = 32;        // steps a wavefront runs before its first pixel (two chunk turns)
// a band's progress counter has a 128-byte line to itself (32 words): the band below polls it while
// the band's own mover writes it
constexpr uint32_t kBandStride = 32;

struct TallBands {
    uint32_t bands, band_rows;
    uint32_t *progress;   // [images * bands]: chunks of the band's last row that are final
    uint32_t *ticket;
    uint32_t *abort_word;
    unsigned long long wait_ticks;
    uint32_t withhold;    // tests of the give-up path: nothing is published
};

template <bool kBands>
__global__ __launch_bounds__(kTallMaxThreads) void k_twar_inverse_tall(TwarK p, uint32_t h, uint32_t w,
                                                                       uint32_t rounds, TallBands tb,
                                                                       const uint8_t *__restrict__ res,
                                                                       uint8_t *__restrict__ img)
{
    extern __shared__ uint8_t twar_lds[];
    __shared__ uint32_t s_id;
    __shared__ int s_abort;
    // (bands) the second half of the workgroup are the movers: wavefront waves + k moves the chunks of
    // wavefront k's rows between memory and the ring while wavefront k decodes
    const uint32_t nt = kBands ? blockDim.x >> 1 : blockDim.x, waves = nt >> 6;
    const bool mover = kBands && threadIdx.x >= nt;
    const uint32_t wave = (threadIdx.x >> 6) - (mover ? waves : 0u), lane = threadIdx.x & 63u;
    const uint32_t thread = wave * 64u + lane;  // the row of the workgroup this thread decodes (a mover: none)
    uint32_t image = blockIdx.x, band = 0u, id = 0u;
    if (kBands) {
        if (threadIdx.x == 0u) {
            s_id = atomicAdd(tb.ticket, 1u);
            s_abort = 0;
        }
        __syncthreads();
        id = s_id;
        image = id / tb.bands;
        band = id % tb.bands;
    }
    uint8_t *my = twar_lds + (size_t)thread * kTallStride;
    uint8_t *hand = twar_lds + (size_t)nt * kTallStride;  // [wavefront][64]: red of its last row, by column mod 64
    // red of the row above the workgroup's first row: the whole row of the round before, or (bands) a
    // ring of 32 values filled from the image
    uint8_t *carry = hand + waves * 64u;
    const size_t row_bytes = (size_t)w * 3u;
    const int chunks = (int)(w >> 4);
    const int lag = (int)(wave * (64u + kTallLag));
    // a mover asks for a chunk three turns before its row enters it, a decoding wavefront two
    constexpr int kLead = kBands ? kTallLead + kTallLag : kTallLead;
    // local steps -kLead .. w + 63 + 16: the last lane's last chunk is written back by then
    const uint32_t total = kLead + w + 80u + (waves - 1u) * (64u + kTallLag);
    const uint32_t rows_here = kBands ? tb.band_rows : nt;
    // where the first thread of this wavefront finds the red values above its row
    const uint8_t *above_ptr = wave != 0u ? hand + (wave - 1u) * 64u : carry;
    const uint32_t above_mask = wave != 0u ? 63u : (kBands ? 31u : 0xFFFFFFFFu);
    const bool first_lane = lane == 0u;
    // the rounding biases and the weights of the multiply-adds written out below in vector
    // registers of their own (as scalar operands they would be copied into one at every use)
    int bias_r = p.bias[0] + 8192, bias_g = p.bias[1] + 8192, bias_b = p.bias[2] + 8192;
    int w_r0 = p.w[0][0], w_r1 = p.w[0][1], w_g0 = p.w[1][0], w_g1 = p.w[1][1], w_b0 = p.w[2][0], w_b1 = p.w[2][1];
    asm volatile("" : "+v"(bias_r), "+v"(bias_g), "+v"(bias_b));
    asm volatile("" : "+v"(w_r0), "+v"(w_r1), "+v"(w_g0), "+v"(w_g1), "+v"(w_b0), "+v"(w_b1));

    for (uint32_t round = 0; round < rounds; ++round) {
        const uint32_t u = kBands ? band * tb.band_rows + thread : round * nt + thread;
        const bool have = !mover && thread < rows_here && u < h;
        const bool last_row = have && (u + 1u == h || thread + 1u == rows_here);
        const bool keeps_row = !kBands && last_row;  // leaves its red values for the next round
        const bool has_above = wave != 0u || (kBands ? band != 0u : round != 0u);
        // (bands) the three threads that fetch the row above the band, 16 bytes of a chunk each
        const bool fetches = mover && band != 0u && wave == 0u && lane < 3u;
        const uint4 *above_src = reinterpret_cast<const uint4 *>(
            img + ((size_t)image * h + (kBands && band != 0u ? band * tb.band_rows - 1u : 0u)) * row_bytes);
        const uint32_t *above_progress = tb.progress + (size_t)(id - (band != 0u ? 1u : 0u)) * kBandStride;
        uint4 above_ahead = make_uint4(0u, 0u, 0u, 0u);
        uint32_t above_done = 0u;  // chunks of the row above known to be final

        // The 64 rows of a wavefront move one chunk on per turn, as 192 pieces of 16 bytes: piece k of
        // the turn is piece k mod 3 of row k / 3, so three neighbouring threads move the 48 contiguous
        // bytes of one row's chunk.  These are this thread's three pieces.
        uint32_t piece_row[3];
        bool piece_have[3];
        const uint4 *piece_src[3];
        uint4 *piece_dst[3];
        uint8_t *piece_lds[3];
#pragma unroll
        for (int i = 0; i < 3; ++i) {
            const uint32_t k = 64u * i + lane, r = (k * 171u) >> 9, part = k - 3u * r;  // r = k / 3 for k < 192
            const uint32_t t = wave * 64u + r;
            const uint32_t ur = kBands ? band * tb.band_rows + t : round * nt + t;
            piece_row[i] = r;
            piece_have[i] = t < rows_here && ur < h;
            const size_t off = ((size_t)image * h + (piece_have[i] ? ur : 0u)) * row_bytes + 16u * part;
            piece_src[i] = reinterpret_cast<const uint4 *>(res + off);
            piece_dst[i] = reinterpret_cast<uint4 *>(img + off);
            piece_lds[i] = twar_lds + (size_t)t * kTallStride + 16u * part;
        }
        // (bands) the thread of the band's last row, which the band below waits for
        const uint32_t pub_thread = kBands ? min(rows_here, h - band * tb.band_rows) - 1u : 0u;
        const uint32_t pub_wave = kBands && band + 1u < tb.bands ? pub_thread >> 6 : 0xFFFFFFFFu;
        const uint32_t pub_lane = pub_thread & 63u;
        bool piece_published[3];
#pragma unroll
        for (int i = 0; i < 3; ++i) piece_published[i] = wave == pub_wave && piece_row[i] == pub_lane;
        uint4 ahead[3] = {};  // this thread's three pieces of the chunks asked for in the last turn

        // One chunk turn of the rows of this wavefront, whose thread 0 stands at column d0: row r is in
        // chunk c = (d0 - r) >> 4.  Chunk c - 1 was left for good and is written back; chunk c + kFill,
        // asked for a turn ago, goes into the ring; chunk c + kFill + 1 is asked for.  The ring has
        // three slots (chunk mod 3): a decoding wavefront that turns its own rows fills the slot its
        // rows enter during the coming 16 steps (kFill 1); a mover works beside the wavefront that is
        // in chunks c and c + 1, so it fills the slot it has just read out (kFill 2), a turn before
        // that wavefront needs it.  What is written back is read out of the ring first; the ring is
        // filled before the stores are issued: loads and stores share one counter of outstanding
        // accesses, and a wait for last turn's loads placed after this turn's stores would wait for
        // the stores too.
        auto turn = [&](int d0, int kFill) {
            uint4 back[3];
            bool backs[3];
#pragma unroll
            for (int i = 0; i < 3; ++i) {
                const int c_prev = ((d0 - (int)piece_row[i]) >> 4) - 1;
                backs[i] = piece_have[i] && c_prev >= 0 && c_prev < chunks;
                const uint32_t *q = reinterpret_cast<const uint32_t *>(
                    piece_lds[i] + ((uint32_t)(c_prev + 48) % 3u) * kTallChunk);
                back[i] = make_uint4(q[0], q[1], q[2], q[3]);
            }
#pragma unroll
            for (int i = 0; i < 3; ++i) {
                const int c_fill = ((d0 - (int)piece_row[i]) >> 4) + kFill;
                if (piece_have[i] && c_fill >= 0 && c_fill < chunks) {
                    uint32_t *q = reinterpret_cast<uint32_t *>(piece_lds[i] + ((uint32_t)(c_fill + 48) % 3u) * kTallChunk);
                    q[0] = ahead[i].x;
                    q[1] = ahead[i].y;
                    q[2] = ahead[i].z;
                    q[3] = ahead[i].w;
                }
            }
#pragma unroll
            for (int i = 0; i < 3; ++i) {
                if (!backs[i]) continue;
                uint4 *to = piece_dst[i] + 3 * (((d0 - (int)piece_row[i]) >> 4) - 1);
                if (kBands && piece_published[i]) {
                    // the band's last row, which another workgroup reads: stores at device scope go
                    // through to memory, so that no write-back of the whole L2 is needed to publish them
                    uint32_t *t32 = reinterpret_cast<uint32_t *>(to);
                    __hip_atomic_store(t32 + 0, back[i].x, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    __hip_atomic_store(t32 + 1, back[i].y, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    __hip_atomic_store(t32 + 2, back[i].z, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    __hip_atomic_store(t32 + 3, back[i].w, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                } else {
                    *to = back[i];
                }
            }
            if (kBands && wave == pub_wave && !tb.withhold) {
                // chunks 0 .. c - 1 of the band's last row are final.  Its pieces were stored by threads
                // of this wavefront, at device scope; once the wavefront has no store outstanding they
                // are in memory, and the count may follow (a release fence would do the same and also
                // write the whole L2 back: 2.5 us each, a third of a block of 16 steps).
                const int c = (d0 - (int)pub_lane) >> 4;
                if (c >= 1 && c <= chunks) {
                    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
                    if (lane == pub_lane)
                        __hip_atomic_store(tb.progress + (size_t)id * kBandStride, (uint32_t)c, __ATOMIC_RELAXED,
                                           __HIP_MEMORY_SCOPE_AGENT);
                }
            }
#pragma unroll
            for (int i = 0; i < 3; ++i) {
                const int c_ask = ((d0 - (int)piece_row[i]) >> 4) + kFill + 1;
                // (a piece with nothing to ask for reads the row's first chunk: no branch round a load)
                const bool asks = piece_have[i] && c_ask >= 0 && c_ask < chunks;
                ahead[i] = piece_src[i][asks ? 3 * c_ask : 0];
            }
        };

        int rl = 0, gl = 0, bl = 0;
        int prev_up = 0;  // the red value above the pixel decoded last: above-left of the next one
        uint32_t ptr = 0;             // ring offset of the pixel about to be decoded
        for (uint32_t D0 = 0; D0 < total; D0 += kTallLag) {
            __syncthreads();
            if (kBands && s_abort) return;  // the same for every thread: written before the barrier
            const int d0 = (int)D0 - lag - kLead;  // this wavefront's step; lane 0 is at column d0
            if (d0 < -kLead || d0 >= (int)(w + 80u)) continue;  // (the same for the whole wavefront)
            if (fetches) {
                // thread 0 of the band enters chunk T now: the red values of chunk T + 1 of the row
                // above, fetched a turn ago, go to the ring (the half that thread is not reading), and
                // chunk T + 2 is fetched as soon as it is final
                const int T = d0 >> 4;
                if (T + 1 >= 0 && T + 1 < chunks) {
                    // this thread holds bytes 16 lane .. 16 lane + 15 of the chunk; red is every third
                    const uint32_t wd[4] = {above_ahead.x, above_ahead.y, above_ahead.z, above_ahead.w};
                    const uint32_t skip = (3u - (16u * lane) % 3u) % 3u;  // offset of the first red byte
#pragma unroll
                    for (uint32_t k = 0; k < 6u; ++k) {
                        const uint32_t o = skip + 3u * k;  // byte within these 16
                        if (o < 16u) {
                            const uint32_t px = (16u * lane + o) / 3u;  // pixel within the chunk
                            carry[(16u * (uint32_t)(T + 1) + px) & 31u] = (uint8_t)(wd[o >> 2] >> (8u * (o & 3u)));
                        }
                    }
                }
                if (T + 2 >= 0 && T + 2 < chunks) {
                    const unsigned long long t0 = wall_clock64();
                    while (above_done < (uint32_t)(T + 3)) {  // what is known to be final does not need asking
                        above_done = __hip_atomic_load(above_progress, __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_AGENT);
                        if (above_done >= (uint32_t)(T + 3)) break;
                        if (__hip_atomic_load(tb.abort_word, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0u) {
                            s_abort = 1;
                            break;
                        }
                        if (wall_clock64() - t0 > tb.wait_ticks) {
                            s_abort = 1;
                            __hip_atomic_store(tb.abort_word, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                            break;
                        }
                        __builtin_amdgcn_s_sleep(32);
                    }
                    if (!s_abort) above_ahead = above_src[3 * (T + 2) + (int)lane];
                }
            }
            if (mover) {
                turn(d0, 2);
                continue;
            }
            if (!kBands) {
                turn(d0, 1);
                wave_lds_sync();
            }
            // ---- 16 steps ----
            // The 16 steps.  Within a pixel green waits for red and blue for green, three chains of
            // dependent instructions one after the other, and a wavefront alone on its SIMD has
            // nothing else to issue meanwhile; red of the next pixel, however, only needs red.  So
            // the channels run skewed: turn i decodes red of pixel i, green of pixel i - 1 and blue
            // of pixel i - 2, which do not depend on each other, and two more turns drain the block
            // (at its end every pixel is whole, as the chunk turns and the barrier expect).
            // A pixel's three residual bytes are asked for a step ahead, as the two aligned dwords
            // that hold them (the second may be the spare bytes behind the ring), and taken apart
            // when used: a byte read is widened where it is read, and that use would put the wait for
            // it right behind the read; the wait stands before the next reads are issued, because
            // LDS answers in order.  The next pixel's ring offset is never this pixel's; what the
            // last step asks for is not used.
            // The values above the 16 pixels that the wavefront's first thread decodes in this block
            // (columns d0 .. d0 + 15: 16 neighbouring bytes, all written before the last barrier, the
            // last of them 17 steps ago) are read once, by every thread alike.
            int v = d0 - (int)lane;
            bool on = have && (uint32_t)v < w;
            auto ring_dwords = [&](uint32_t at) { return reinterpret_cast<const uint32_t *>(my + (at & ~3u)); };
            uint32_t above16[4] = {0u, 0u, 0u, 0u};
            if (has_above) {
                const uint32_t at = (d0 >= 0 && (uint32_t)d0 < w ? (uint32_t)d0 : 0u) & above_mask;
                const uint32_t *a = reinterpret_cast<const uint32_t *>(above_ptr + at);
#pragma unroll
                for (int k = 0; k < 4; ++k) above16[k] = a[k];
            }
            uint32_t e_lo = ring_dwords(ptr)[0], e_hi = ring_dwords(ptr)[1];
            uint8_t *const spare = my + kTallRing;  // the four bytes after the ring: where writes of idle steps go
            auto clamp8 = [](int acc) { return min(max(acc >> 14, 0), 255); };
            // what a pixel's later channels need from its earlier ones, one and two turns later
            struct InFlight {
                uint32_t e;     // its residual bytes
                uint8_t *q;     // where it goes in the ring (the spare bytes for an idle step)
                bool on;
                int left_r, xr; // red to its left, its own red
                int left_g, xg; // green to its left, its own green
            };
            InFlight one = {}, two = {};  // the pixels of one and two turns ago
#pragma unroll
            for (int i = 0; i < kTallLag + 2; ++i) {
                InFlight now = {};
                int xr = 0;
                if (i < kTallLag) {
                    // the wait for what the last step asked for stands here, before this step asks
                    asm volatile("" : "+v"(e_lo), "+v"(e_hi));
                    now.on = on;
                    now.e = __builtin_amdgcn_alignbyte(e_hi, e_lo, ptr & 3u);  // bytes ptr .. ptr + 3 of the ring
                    now.q = on ? my + ptr : spare;
                    const uint32_t nptr = ptr + 3u == (uint32_t)kTallRing ? 0u : ptr + 3u;
                    ptr = on ? nptr : ptr;
                    e_lo = ring_dwords(ptr)[0];
                    e_hi = ring_dwords(ptr)[1];
                }
                // ---- red of this turn's pixel, green of the one before, blue of the one before that:
                // three multiply-adds each; what only needs the pixel to the left comes first, the
                // operand that arrives last (the value just decoded) goes into the last of them
                int acc_r = 0, acc_g = 0, acc_b = 0;
                if (i < kTallLag) {
                    const int above = (int)((above16[i >> 2] >> (8 * (i & 3))) & 0xFFu);
                    int up = __builtin_amdgcn_update_dpp(0, rl, 0x138 /* wave_shr:1 */, 0xF, 0xF, true);
                    // the first thread of a wavefront: the row above belongs to another wavefront, to
                    // the round or band before, or is padding
                    up = first_lane ? above : up;
                    const int upleft = prev_up;
                    prev_up = on ? up : prev_up;
                    acc_r = mad_i24(p.w[0][2], rl, mad_i24(w_r1, up, mad_i24(w_r0, upleft, bias_r)));
                }
                if (i >= 1 && i <= kTallLag)
                    acc_g = mad_i24(p.w[1][2], one.xr, mad_i24(w_g1, one.left_r, mad_i24(w_g0, gl, bias_g)));
                if (i >= 2)
                    acc_b = mad_i24(p.w[2][2], two.xg, mad_i24(w_b1, two.left_g, mad_i24(w_b0, bl, bias_b)));
                if (i < kTallLag) {
                    xr = add_byte_of<0>(now.e, clamp8(acc_r));
                    now.left_r = rl;
                    now.xr = xr;
                    const uint32_t col = on ? (uint32_t)v : 0u;
                    uint8_t *const to_next_wave = on && lane == 63u ? hand + wave * 64u + (col & 63u) : spare + 3;
                    *to_next_wave = (uint8_t)xr;
                    if (on && keeps_row) carry[col] = (uint8_t)xr;
                    rl = on ? xr : rl;
                }
                if (i >= 1 && i <= kTallLag) {
                    const int xg = add_byte_of<1>(one.e, clamp8(acc_g));
                    one.left_g = gl;
                    one.xg = xg;
                    gl = one.on ? xg : gl;
                }
                if (i >= 2) {
                    const int xb = add_byte_of<2>(two.e, clamp8(acc_b));
                    bl = two.on ? xb : bl;
                    two.q[0] = (uint8_t)two.xr;
                    two.q[1] = (uint8_t)two.xg;
                    two.q[2] = (uint8_t)xb;
                }
                two = one;
                one = now;
                if (i < kTallLag) {
                    ++v;
                    on = have && (uint32_t)v < w;
                }
            }
        }
        __syncthreads();
    }
}

// Progress counters of the band kernel: a few sets in device globals (the entry points take no
// workspace), handed out under a lock so that concurrent calls do not share one; a call that finds
// none free uses the workgroup-per-image kernel instead.  Layout of a set: the progress counters of
// up to 4096 bands, kBandStride words apart (2 MB for the four sets), then the ticket and the abort
// word.
constexpr int kBandSlots = 4;
constexpr uint32_t kBandFlags = 4096 * kBandStride;
static __device__ uint32_t g_band_flags[kBandSlots][kBandFlags + 2];
static std::mutex g_band_mutex;
static bool g_band_in_use[kBandSlots];
static std::map<int, uint32_t *> g_band_base;  // per device: address of g_band_flags there

__global__ void k_band_clear(uint32_t *flags, uint32_t n)
{
    const uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) flags[i] = 0u;
    if (i < 2u) flags[kBandFlags + i] = 0u;
}

// A free set of counters on the current device (null if none), and its release.
static uint32_t *band_flags_acquire(int *slot_out)
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return nullptr;
    std::lock_guard<std::mutex> lock(g_band_mutex);
    auto it = g_band_base.find(dev);
    if (it == g_band_base.end()) {
        void *ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(g_band_flags)) != hipSuccess) return nullptr;
        it = g_band_base.emplace(dev, static_cast<uint32_t *>(ptr)).first;
    }
    for (int i = 0; i < kBandSlots; ++i)
        if (!g_band_in_use[i]) {
            g_band_in_use[i] = true;
            *slot_out = i;
            return it->second + (size_t)i * (kBandFlags + 2);
        }
    return nullptr;
}
static void band_flags_release(int slot)
{
    std::lock_guard<std::mutex> lock(g_band_mutex);
    g_band_in_use[slot] = false;
}

static int make_twar(const pilc_twar_params *in, uint32_t n, uint32_t h, uint32_t w, TwarK *k)
{
    if (!in || n == 0 || h == 0 || w == 0) return PILC_E_ARG;
    if ((uint64_t)n * h * w * 3 + 4096 >= (1ull << 40)) return PILC_E_TOO_LARGE;
    if (w > 65535u) return PILC_E_TOO_LARGE;
    for (int c = 0; c < 3; ++c) {
        for (int j = 0; j < 3; ++j) k->w[c][j] = in->w[c][j];
        // the sum of three products and the bias must stay inside 32 bits: |w| <= 2^15, values <= 255
        if (in->bias[c] > (1 << 30) || in->bias[c] < -(1 << 30)) return PILC_E_ARG;
        k->bias[c] = in->bias[c];
    }
    return PILC_OK;
}

}  // namespace pilc

extern "C" {

int pilc_twar_forward(uint32_t n, uint32_t h, uint32_t w, const uint8_t *img_dev,
                      const pilc_twar_params *params_host, uint8_t *res_dev, void *hip_stream)
{
    TwarK k;
    int rc = make_twar(params_host, n, h, w, &k);
    if (rc != PILC_OK) return rc;
    if (!img_dev || !res_dev || img_dev == res_dev) return PILC_E_ARG;
    hipStream_t stream = (hipStream_t)hip_stream;
    const uint64_t rows = (uint64_t)n * h;
    if (rows >= (1ull << 31)) return PILC_E_TOO_LARGE;
    const uint32_t rpb = w >= 256 ? 1u : 256u / w;
    const uint32_t blocks = (uint32_t)((rows + rpb - 1) / rpb);
    Timer timer(stream);
    const uint64_t groups = rows * (w / 4);
    if (w % 4 == 0 && ((((uintptr_t)img_dev) | ((uintptr_t)res_dev)) & 3) == 0 && groups < (1ull << 32))
        k_twar_forward4<<<(uint32_t)((groups + 255) / 256), 256, 0, stream>>>(
            k, (uint32_t)groups, FastDiv::make(h), FastDiv::make(w / 4), reinterpret_cast<const uint32_t *>(img_dev),
            reinterpret_cast<uint32_t *>(res_dev));
    else
        k_twar_forward<<<blocks, 256, 0, stream>>>(k, (uint32_t)rows, h, w, rpb, img_dev, res_dev);
    timer.mark("k_twar_forward");
    HIP_TRY(hipGetLastError());
    HIP_TRY(hipStreamSynchronize(stream));
    timer.finish();
    return PILC_OK;
}

int pilc_twar_inverse(uint32_t n, uint32_t h, uint32_t w, const uint8_t *res_dev,
                      const pilc_twar_params *params_host, uint8_t *img_dev, void *hip_stream)
{
    TwarK k;
    int rc = make_twar(params_host, n, h, w, &k);
    if (rc != PILC_OK) return rc;
    if (!img_dev || !res_dev || img_dev == res_dev) return PILC_E_ARG;
    hipStream_t stream = (hipStream_t)hip_stream;
    const uint32_t per = h <= 64 ? 64 / h : 1;
    const uint32_t groups = (n + per - 1) / per;
    const uint32_t blocks = (groups + kTwarWaves - 1) / kTwarWaves;
    const uint32_t last_bytes = (w + 15u) & ~15u;
    const size_t tile_lds = (size_t)kTwarWaves * (last_bytes + 64u * (size_t)w * 3u);
    // the element of the tile copies: every group (whole images, or a band of 64 rows) must start
    // and end on a multiple of it
    const uint32_t row_bytes = w * 3u;
    const uintptr_t both = (uintptr_t)img_dev | (uintptr_t)res_dev;
    const bool whole_images = h <= 64;
    const uint32_t unit_bytes = whole_images ? h * row_bytes : row_bytes;
    const int elem = unit_bytes % 16u == 0u && (both & 15) == 0 ? 16 : unit_bytes % 4u == 0u && (both & 3) == 0 ? 4 : 1;
    Timer timer(stream);
    const bool tall = h > 64 && w % 16 == 0 && w <= 16384 && ((((uintptr_t)img_dev) | ((uintptr_t)res_dev)) & 15) == 0;
    // few tall images: bands of up to 256 rows in workgroups of their own, four decoding wavefronts
    // (one per SIMD) and their four movers (on 30 frames of 1080 x 1920: five bands of 216 rows
    // 0.49 ms, six of 180 0.50, three of 360 0.57; one workgroup per frame 2.2)
    uint32_t bands = tall && n < 256u ? (h + 255u) / 256u : 1u;
    int slot = -1;
    uint32_t *flags = nullptr;
    if (bands > 1u && (uint64_t)n * bands * kBandStride <= kBandFlags) flags = band_flags_acquire(&slot);
    if (tall && flags) {
        const uint32_t band_rows = (h + bands - 1) / bands;
        bands = (h + band_rows - 1) / band_rows;
        const uint32_t nt = (band_rows + 63u) & ~63u;
        const size_t lds = (size_t)nt * kTallStride + (nt / 64) * 64 + 32;
        int dev = 0, khz = 0;
        const unsigned long long wait = g_one_pass_wait.load(std::memory_order_relaxed);
        if (hipGetDevice(&dev) != hipSuccess ||
            hipDeviceGetAttribute(&khz, hipDeviceAttributeWallClockRate, dev) != hipSuccess || khz <= 0)
            khz = 100000;
        rc = allow_large_lds(reinterpret_cast<const void *>(k_twar_inverse_tall<true>));
        uint32_t aborted = 0u;
        if (rc == PILC_OK) {
            k_band_clear<<<(n * bands * kBandStride + 255u) / 256u, 256, 0, stream>>>(flags, n * bands * kBandStride);
            const TallBands tb = {bands, band_rows, flags, flags + kBandFlags, flags + kBandFlags + 1,
                                  wait ? wait : 2000ull * (unsigned long long)khz,
                                  (uint32_t)g_one_pass_withhold.load(std::memory_order_relaxed)};
            // a decoding and a moving wavefront per 64 rows
            k_twar_inverse_tall<true><<<n * bands, 2u * nt, lds, stream>>>(k, h, w, 1u, tb, res_dev, img_dev);
            timer.mark("k_twar_inverse");
            hipError_t e = hipGetLastError();
            if (e == hipSuccess)
                e = hipMemcpyAsync(&aborted, flags + kBandFlags + 1, sizeof(aborted), hipMemcpyDeviceToHost, stream);
            if (e == hipSuccess) e = hipStreamSynchronize(stream);
            if (e != hipSuccess) rc = hip_fail(e, "k_twar_inverse_bands");
        }
        band_flags_release(slot);
        if (rc != PILC_OK) return rc;
        timer.finish();
        return aborted ? PILC_E_TIMEOUT : PILC_OK;
    }
    if (tall) {
        // as few rounds as the workgroup size allows, of equal size (three rounds of 512, 512 and 56
        // rows of a 1080-row frame took 2.8 ms where two rounds of 540 take 2.2)
        const uint32_t rounds = (h + kTallMaxThreads - 1) / kTallMaxThreads;
        const uint32_t per = (h + rounds - 1) / rounds;
        const uint32_t nt = (per + 63u) & ~63u;
        const size_t lds = (size_t)nt * kTallStride + (nt / 64) * 64 + w;
        if ((rc = allow_large_lds(reinterpret_cast<const void *>(k_twar_inverse_tall<false>))) != PILC_OK) return rc;
        k_twar_inverse_tall<false><<<n, nt, lds, stream>>>(k, h, w, rounds, TallBands{}, res_dev, img_dev);
    } else if (tile_lds <= 64 * 1024) {
        if (elem == 16)
            k_twar_inverse<true, u32x4><<<blocks, 64 * kTwarWaves, tile_lds, stream>>>(k, n, h, w, last_bytes, res_dev, img_dev);
        else if (elem == 4)
            k_twar_inverse<true, uint32_t><<<blocks, 64 * kTwarWaves, tile_lds, stream>>>(k, n, h, w, last_bytes, res_dev, img_dev);
        else
            k_twar_inverse<true, uint8_t><<<blocks, 64 * kTwarWaves, tile_lds, stream>>>(k, n, h, w, last_bytes, res_dev, img_dev);
    } else {
        k_twar_inverse<false, uint8_t><<<blocks, 64 * kTwarWaves, (size_t)kTwarWaves * last_bytes, stream>>>(
            k, n, h, w, last_bytes, res_dev, img_dev);
    }
    timer.mark("k_twar_inverse");
    HIP_TRY(hipGetLastError());
    HIP_TRY(hipStreamSynchronize(stream));
    timer.finish();
    return PILC_OK;
}

}  // extern "C"
