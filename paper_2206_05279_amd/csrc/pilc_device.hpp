// Device-side arithmetic shared by the libpilc kernels (gfx950 only).
//
// Everything here is integer and must produce, bit for bit, the tables that Sec. 3.2 of
// arXiv 2206.05279 asks for (integer masses summing to 2^M with C_x their running sum) from a
// logistic law with location mu and scale s on 0..255 (Sec. 3.1 eq. (7), Sec. 3.3), after the
// channel conditioning of Sec. 3.1 eqs. (3)-(4).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace pilc {

constexpr int kSigEntries = 2048;  // interpolation cells of the sigmoid table
constexpr int kExpHiEntries = 640;
constexpr int kExpLoEntries = 64;

// Constant tables in device globals, filled by the host once per device.
//   g_sig_cell[i] = { T[i], (T[i+1]-T[i]) * 64 },  T[i] = round(2^24 * sigmoid((i-1024)/64))
//     (the slope is below 2^16, so slope * 64 * r for a 10-bit r stays below 2^32 and its upper
//     half is floor(slope * r / 2^10): the interpolation is one multiply and one add of a half)
//   g_exp_hi[i]   = round(2^26 * exp(4 - i/64)),  g_exp_lo[j] = round(2^31 * exp(-j/4096))
extern __device__ uint2 g_sig_cell[kSigEntries];
extern __device__ uint32_t g_exp_hi[kExpHiEntries];
extern __device__ uint32_t g_exp_lo[kExpLoEntries];

// LDS copy of the tables; every coding kernel stages them once per workgroup.
struct LdsTables {
    uint2 sig[kSigEntries];
    uint32_t exp_hi[kExpHiEntries];
    uint32_t exp_lo[kExpLoEntries];
};

__device__ __forceinline__ void load_tables(LdsTables &t)
{
    for (int i = threadIdx.x; i < kSigEntries; i += blockDim.x) t.sig[i] = g_sig_cell[i];
    for (int i = threadIdx.x; i < kExpHiEntries; i += blockDim.x) t.exp_hi[i] = g_exp_hi[i];
    for (int i = threadIdx.x; i < kExpLoEntries; i += blockDim.x) t.exp_lo[i] = g_exp_lo[i];
    __syncthreads();
}

// Sixteen bytes as the compiler's own vector type (arrays of it stay in registers where arrays of
// the HIP struct type of the same size go to private memory).
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// Orders this wavefront's LDS accesses: LDS instructions of one wavefront execute in order, so
// all that is needed is that the compiler keeps them in order too.
__device__ __forceinline__ void wave_lds_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// 24-bit signed multiply and multiply-add as the single instructions they are.  (Written through
// the 32-bit product, the compiler first sign-extends operands it cannot prove to be 24 bits wide,
// which costs more instructions than the multiply.)  Operands must lie within +-2^23; only plain
// vector ALU instructions consume the results.
__device__ __forceinline__ int mul_i24(int a, int b)
{
    int r;
    asm("v_mul_i32_i24 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
    return r;
}
__device__ __forceinline__ int mad_i24(int a, int b, int c)
{
    int r;
    asm("v_mad_i32_i24 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
    return r;
}
// Division of a 32-bit number by a divisor fixed at launch (1 <= d < 2^31), as one multiply-high,
// an add, a subtract and two shifts: with l = ceil(log2 d) and m = floor(2^32 (2^l - d) / d) + 1,
// n / d = (t + ((n - t) >> 1)) >> (l - 1) for t = floor(m n / 2^32) and l >= 1; d = 1 is passed on.
// (The division the compiler makes from `/` goes through a float reciprocal and two corrections:
// some fifteen instructions.)
struct FastDiv {
    uint32_t m, s, d;
    static FastDiv make(uint32_t d)
    {
        FastDiv f;
        uint32_t l = 0;
        while ((1ull << l) < d) ++l;
        f.m = l == 0 ? 0u : (uint32_t)((((1ull << l) - d) << 32) / d + 1ull);
        f.s = l == 0 ? 0u : l - 1u;
        f.d = d;
        return f;
    }
    __device__ __forceinline__ uint32_t div(uint32_t n) const
    {
        if (d == 1u) return n;  // the same for every thread
        const uint32_t t = __umulhi(m, n);
        return (t + ((n - t) >> 1)) >> s;
    }
};

// Batch geometry as the kernels see it (derived on the host from pilc_geom).
struct Geo {
    uint32_t n, h, w, hw;
    uint32_t prec_bits;
    uint32_t lane_mode, lane_a, lane_b;
    uint32_t tiles_x, tiles_per_img;  // mode 1
    uint32_t total_px;                // n*h*w   (< 2^32 / 3)
    uint32_t lanes;
    FastDiv by_hw;                    // which image a pixel belongs to: once a chunk or pixel in every kernel
};

// One lane's pixel set: `npx` pixels starting at flat pixel `first`, laid out as rows of `tw`
// pixels with a stride of `w` pixels between row starts (flat lanes are a single row).
struct LaneShape {
    uint32_t first, npx, tw;
    uint32_t sym_base;  // symbols of all lanes before this one (lane-major order)
};

__device__ __forceinline__ LaneShape lane_shape(const Geo &g, uint32_t lane)
{
    LaneShape s;
    if (g.lane_mode == 0) {
        uint64_t first = (uint64_t)lane * g.lane_a;
        uint64_t last = first + g.lane_a;
        if (last > g.total_px) last = g.total_px;
        s.first = (uint32_t)first;
        s.npx = (uint32_t)(last - first);
        s.tw = s.npx;
        s.sym_base = 3u * s.first;
    } else {
        uint32_t img = lane / g.tiles_per_img;
        uint32_t r = lane - img * g.tiles_per_img;
        uint32_t ty = r / g.tiles_x, tx = r - ty * g.tiles_x;
        uint32_t y0 = ty * g.lane_a, x0 = tx * g.lane_b;
        uint32_t th = min(g.lane_a, g.h - y0);
        uint32_t tw = min(g.lane_b, g.w - x0);
        s.first = (img * g.h + y0) * g.w + x0;
        s.npx = th * tw;
        s.tw = tw;
        // tiles above cover y0 full rows; tiles to the left in this tile row are th high
        s.sym_base = 3u * (img * g.hw + y0 * g.w + x0 * th);
    }
    return s;
}

// Where lane `lane`'s words end in the scratch of the few-lane encoder: slots in lane order, one
// word per symbol, and one spare word below every slot.
__device__ __forceinline__ uint32_t block_slot_end(const LaneShape &sh, uint32_t lane)
{
    return sh.sym_base + 3u * sh.npx + lane + 1u;
}

// Flat pixel index of the t-th pixel of a lane (rows of sh.tw pixels, g.w apart).
__device__ __forceinline__ uint32_t lane_pixel(const Geo &g, const LaneShape &sh, uint32_t t)
{
    if (g.lane_mode == 0) return sh.first + t;  // a flat lane is one run of pixels (the same for every thread)
    uint32_t row = t / sh.tw;
    return sh.first + row * g.w + (t - row * sh.tw);
}

// Rounded Q2.14 * Q8.8 product: floor((v + 2^13) / 2^14).
__device__ __forceinline__ int rsh14(int v) { return (v + 8192) >> 14; }

// rsh14(a * e) for a Q2.14 coefficient a (16 bits) and an innovation e = 256 x - mu (18 bits): the
// product is below 2^31 in magnitude, so the 24-bit multiply-add gives it exactly at full rate.
__device__ __forceinline__ int rsh14_mul(int a, int e) { return (__mul24(a, e) + 8192) >> 14; }

// Q6.25 value of exp(-log_scale); log_scale Q4.12 clamped to [-4, 6).
__device__ __forceinline__ uint32_t inv_scale(int ls, const LdsTables &t)
{
    int u = min(max(ls, -16384), 24575) + 16384;
    return __umulhi(t.exp_hi[u >> 6], t.exp_lo[u & 63]);
}

// F(k) in 24 bits at the edge k - 1/2:  d = 256*k - 128 - mu'  (Q8.8), inv_s Q6.25 < 2^31.
// z = clamp(floor(d * inv_s / 2^17), -2^20, 2^20 - 1) and w = z + 2^20 is bits 17..48 of the
// 64-bit value d * inv_s + 2^37; z saturates exactly when the high word of that sum leaves 0..63.
// Clamping the high word to -1..64 first keeps the saturated cases on their side of 0..2^21 - 1
// after the shift (all ones above bit 14, or bit 21 set), so one more clamp finishes the job.
__device__ __forceinline__ uint32_t edge_cdf(int d, uint32_t inv_s, const LdsTables &t)
{
    long long p = (long long)d * (long long)(int)inv_s + (1ll << 37);  // Q.33
    asm("" : "+v"(p));  // keep the clamps below on 32-bit words
    const int hi = min(max((int)(p >> 32), -1), 64);
    const int v = (int)__builtin_amdgcn_alignbit((uint32_t)hi, (uint32_t)p, 17);
    const uint32_t w = (uint32_t)min(max(v, 0), (1 << 21) - 1);
    const uint2 cell = t.sig[w >> 10];
    return cell.x + ((uint32_t)__umul24(cell.y, w & 1023u) >> 16);
}

// floor(f * (2^M - 256) / 2^24) for a 24-bit f:  2^M - 256 = 256 * (spread >> 8) and the product
// f * (spread >> 8) stays below 2^32 for M <= 16.
__device__ __forceinline__ uint32_t scale_mass(uint32_t f, uint32_t spread)
{
    return (uint32_t)__umul24(f, spread >> 8) >> 16;  // the builtin's result type is int
}

// C(k), 1 <= k <= 255:  k + floor(F(k) * (2^M - 256) / 2^24).
__device__ __forceinline__ uint32_t cum_inner(int k, int mu_eff, uint32_t inv_s, uint32_t spread,
                                              const LdsTables &t)
{
    return (uint32_t)k + scale_mass(edge_cdf(256 * k + (-128 - mu_eff), inv_s, t), spread);
}

// -128 - mu' in a register of its own: the edge offset of C(k) is then one shift-and-add per k,
// instead of being formed again from a packed parameter at every evaluation.
__device__ __forceinline__ int edge_offset(int mu_eff)
{
    int c0 = -128 - mu_eff;
    asm("" : "+v"(c0));
    return c0;
}

// C(k), 1 <= k <= 255, from c0 = edge_offset(mu').
__device__ __forceinline__ uint32_t cum_inner_at(int k, int c0, uint32_t inv_s, uint32_t spread,
                                                 const LdsTables &t)
{
    return (uint32_t)k + scale_mass(edge_cdf(256 * k + c0, inv_s, t), spread);
}

// C(k) for any k in 0..256.
__device__ __forceinline__ uint32_t cum_at(int k, int mu_eff, uint32_t inv_s, uint32_t prec_bits,
                                           const LdsTables &t)
{
    uint32_t spread = (1u << prec_bits) - 256u;
    if (k <= 0) return 0u;
    if (k >= 256) return 1u << prec_bits;
    return cum_inner(k, mu_eff, inv_s, spread, t);
}

}  // namespace pilc
