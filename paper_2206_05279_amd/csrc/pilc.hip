// libpilc: kernels and C ABI of the PILC entropy-coding stage for gfx950 (arXiv 2206.05279).
//
// Path per call
//   encode: lane kernel (mean shift -> (cum,freq) -> rANS, words to per-lane scratch slots)
//           -> 3-step prefix scan of lane byte counts (offset table + header)
//           -> pack (lane streams copied to their offsets)
//   decode: header check -> lane kernel (search of the symbol, state update, refill)
// Lane kernels: pilc_lane_kernels.hpp (thread per lane), pilc_block_encode.hpp and
// pilc_row_decode.hpp (few long lanes).
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <atomic>
#include <map>
#include <mutex>
#include <utility>

#include "../../include/pilc.h"
#include "pilc_device.hpp"

namespace pilc {

__device__ uint2 g_sig_cell[kSigEntries];
__device__ uint32_t g_exp_hi[kExpHiEntries];
__device__ uint32_t g_exp_lo[kExpLoEntries];

constexpr uint32_t kHeaderBytes = 64;

// status word kinds (device side), mapped to PILC_E_* on the host
constexpr uint32_t kMagicPilc = 0x434C4950u;  // "PILC"
constexpr uint32_t kMagicMix = 0x58494D50u;   // "PMIX"
enum : int { ST_OK = 0, ST_TOO_LARGE = 4, ST_FORMAT = 5, ST_CORRUPT = 6, ST_CAPACITY = 3, ST_PARAMS = 7, ST_TIMEOUT = 8 };

struct Status {
    int code;
    uint32_t ticket;  // the one-pass encoder's workgroups number themselves from it
    unsigned long long payload_bytes;
};

// --------------------------------------------------------------------------------------------
// Per-pixel helper: effective means of the three channels (Sec. 3.1 eqs. (3)-(4), innovation
// form).  e_G uses the unshifted mu_G so the three means are independent of each other.
// --------------------------------------------------------------------------------------------
__device__ __forceinline__ void mean_shift(const int x[3], const int m[3], int a_gr, int a_br,
                                           int a_bg, int out[3])
{
    int e_r = x[0] * 256 - m[0];
    int e_g = x[1] * 256 - m[1];
    out[0] = m[0];
    out[1] = m[1] + rsh14_mul(a_gr, e_r);
    out[2] = m[2] + rsh14_mul(a_br, e_r) + rsh14_mul(a_bg, e_g);
}

// --------------------------------------------------------------------------------------------
// pilc_symbol_tables: one thread per pixel.
// --------------------------------------------------------------------------------------------
__global__ void k_symbol_tables(Geo g, const uint8_t *__restrict__ img,
                                const uint16_t *__restrict__ mu, const int16_t *__restrict__ ls,
                                const int16_t *__restrict__ coef, uint32_t *__restrict__ cum_out,
                                uint32_t *__restrict__ freq_out)
{
    __shared__ LdsTables tab;
    load_tables(tab);
    uint32_t p = blockIdx.x * blockDim.x + threadIdx.x;
    if (p >= g.total_px) return;
    size_t s = (size_t)p * 3;
    uint32_t im = g.by_hw.div(p);
    int x[3] = {img[s], img[s + 1], img[s + 2]};
    int m[3] = {mu[s], mu[s + 1], mu[s + 2]};
    int me[3];
    mean_shift(x, m, coef[3 * im], coef[3 * im + 1], coef[3 * im + 2], me);
    for (int c = 0; c < 3; ++c) {
        uint32_t inv_s = inv_scale(ls[s + c], tab);
        uint32_t lo = cum_at(x[c], me[c], inv_s, g.prec_bits, tab);
        uint32_t hi = cum_at(x[c] + 1, me[c], inv_s, g.prec_bits, tab);
        cum_out[s + c] = lo;
        freq_out[s + c] = hi - lo;
    }
}

// --------------------------------------------------------------------------------------------
// Prefix scan of per-item byte counts into a container's offset table.
// --------------------------------------------------------------------------------------------
constexpr int kScanThreads = 256;
constexpr int kScanItems = 4;
constexpr int kScanTile = kScanThreads * kScanItems;

__device__ __forceinline__ unsigned long long block_exclusive_scan(unsigned long long v,
                                                                   unsigned long long *total)
{
    __shared__ unsigned long long wave_sum[kScanThreads / 64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    unsigned long long inc = v;
    for (int d = 1; d < 64; d <<= 1) {
        unsigned long long o = __shfl_up(inc, d, 64);
        if (lane >= d) inc += o;
    }
    if (lane == 63) wave_sum[wave] = inc;
    __syncthreads();
    unsigned long long base = 0, all = 0;
    for (int i = 0; i < kScanThreads / 64; ++i) {
        if (i < wave) base += wave_sum[i];
        all += wave_sum[i];
    }
    __syncthreads();
    *total = all;
    return base + inc - v;
}

// Bytes an item (a lane, a piece) takes in the payload, from the count its coder left behind:
// base + unit * ((count + add) >> shift).
struct ItemBytes {
    uint32_t base, unit, add, shift;
    __device__ __forceinline__ unsigned long long operator()(uint32_t count) const
    {
        return (unsigned long long)base + (unsigned long long)unit * ((count + add) >> shift);
    }
};

// The first twelve 32-bit words of a container header (the payload size follows them).
struct HeaderWords {
    uint32_t w[12];
};

__global__ void k_scan_partials(uint32_t items, ItemBytes bytes, const uint32_t *__restrict__ counts,
                                unsigned long long *__restrict__ block_sums)
{
    uint32_t base = blockIdx.x * kScanTile + threadIdx.x * kScanItems;
    unsigned long long v = 0;
    for (int i = 0; i < kScanItems; ++i)
        if (base + i < items) v += bytes(counts[base + i]);
    unsigned long long total;
    block_exclusive_scan(v, &total);
    if (threadIdx.x == 0) block_sums[blockIdx.x] = total;
}

// Single workgroup: exclusive scan of the block sums in place; writes the header.
__global__ void k_scan_spine(HeaderWords head, uint32_t items, uint32_t nblocks,
                             unsigned long long *__restrict__ block_sums,
                             uint8_t *__restrict__ coded, unsigned long long coded_capacity,
                             Status *__restrict__ status)
{
    unsigned long long carry = 0;
    for (uint32_t b0 = 0; b0 < nblocks; b0 += kScanThreads) {
        uint32_t i = b0 + threadIdx.x;
        unsigned long long v = i < nblocks ? block_sums[i] : 0ull, total;
        unsigned long long ex = block_exclusive_scan(v, &total);
        if (i < nblocks) block_sums[i] = carry + ex;
        carry += total;
    }
    if (threadIdx.x == 0) {
        status->payload_bytes = carry;
        unsigned long long need = kHeaderBytes + 4ull * ((unsigned long long)items + 1ull) + carry;
        if (status->code == ST_OK) {  // an earlier error stays
            if (carry >= (1ull << 32))
                status->code = ST_TOO_LARGE;
            else if (need > coded_capacity)
                status->code = ST_CAPACITY;
        }
        uint32_t *h = reinterpret_cast<uint32_t *>(coded);
        for (int i = 0; i < 12; ++i) h[i] = head.w[i];
        h[12] = (uint32_t)carry;
        h[13] = (uint32_t)(carry >> 32);
        h[14] = 0u;
        h[15] = 0u;
    }
}

__global__ void k_scan_apply(uint32_t items, ItemBytes bytes, const uint32_t *__restrict__ counts,
                             const unsigned long long *__restrict__ block_sums,
                             uint32_t *__restrict__ offsets)
{
    uint32_t base = blockIdx.x * kScanTile + threadIdx.x * kScanItems;
    unsigned long long item[kScanItems], v = 0;
    for (int i = 0; i < kScanItems; ++i) {
        item[i] = base + i < items ? bytes(counts[base + i]) : 0ull;
        v += item[i];
    }
    unsigned long long total;
    unsigned long long ex = block_exclusive_scan(v, &total) + block_sums[blockIdx.x];
    for (int i = 0; i < kScanItems; ++i) {
        if (base + i < items) offsets[base + i] = (uint32_t)ex;
        ex += item[i];
        // the closing entry offsets[items] = payload size
        if (base + i + 1 == items) offsets[items] = (uint32_t)ex;
    }
}

// --------------------------------------------------------------------------------------------
// Pack: a workgroup copies the streams of a run of consecutive lanes (their bytes are contiguous
// in the payload).  Offsets, scratch positions and states of the run sit in LDS; each payload
// word finds its lane by bisection there.
// --------------------------------------------------------------------------------------------
constexpr int kPackMaxLanes = 256;

__global__ __launch_bounds__(256) void k_pack(Geo g, uint32_t lanes_per_block,
                                              const uint16_t *__restrict__ scratch,
                                              const uint32_t *__restrict__ lane_state,
                                              const uint32_t *__restrict__ offsets,
                                              uint16_t *__restrict__ payload,
                                              const Status *__restrict__ status)
{
    if (status->code != ST_OK) return;
    __shared__ uint32_t s_off[kPackMaxLanes + 1];
    __shared__ uint32_t s_src[kPackMaxLanes];    // scratch index of the lane's first word
    __shared__ uint32_t s_state[kPackMaxLanes];
    const uint32_t l0 = blockIdx.x * lanes_per_block;
    const uint32_t n = min(lanes_per_block, g.lanes - l0);
    for (uint32_t i = threadIdx.x; i < n; i += blockDim.x) {
        const uint32_t begin = offsets[l0 + i], end = offsets[l0 + i + 1];
        const LaneShape sh = lane_shape(g, l0 + i);
        s_off[i] = begin;
        if (i + 1 == n) s_off[n] = end;
        s_src[i] = block_slot_end(sh, l0 + i) - ((end - begin - 4u) >> 1);
        s_state[i] = lane_state[l0 + i];
    }
    __syncthreads();
    const uint32_t w_begin = s_off[0] >> 1, w_end = s_off[n] >> 1;
    if (w_begin == w_end) return;
    // four words per thread and turn, so that four loads are under way together (words past the
    // end read the last one again and are not written)
    for (uint32_t w0 = w_begin + threadIdx.x; w0 - threadIdx.x < w_end; w0 += 4u * blockDim.x) {
        uint16_t v[4];
#pragma unroll
        for (uint32_t k = 0; k < 4u; ++k) {
            const uint32_t byte = 2u * min(w0 + k * blockDim.x, w_end - 1u);
            uint32_t lo = 0, hi = n - 1;  // largest i with s_off[i] <= byte
            while (lo < hi) {
                const uint32_t mid = (lo + hi + 1) >> 1;
                if (s_off[mid] <= byte)
                    lo = mid;
                else
                    hi = mid - 1;
            }
            const uint32_t local = byte - s_off[lo];
            // a lane's state is its first four bytes; for those the load goes to the word below the
            // lane's words (inside its slot: a lane has a pixel or more) and is not used
            const uint16_t word = scratch[local < 4u ? s_src[lo] - 1u : s_src[lo] + ((local - 4u) >> 1)];
            v[k] = local < 4u ? (uint16_t)(s_state[lo] >> (8u * local)) : word;
        }
#pragma unroll
        for (uint32_t k = 0; k < 4u; ++k)
            if (w0 + k * blockDim.x < w_end) payload[w0 + k * blockDim.x] = v[k];
    }
}

// The packer for the thread-per-lane encoder, whose scratch is [word number][thread] per 64
// lanes with room for lane_cap words each, the words of a lane in the reverse of the stream
// order.  A workgroup owns 64 lanes: it reads kPackTile word numbers at a time as whole 128-byte
// rows into an LDS tile and writes every lane's piece of the stream from there, 64 consecutive words
// per wavefront instruction.  kPackTile word numbers a turn: the more, the longer the runs a lane's
// words are written in (128 for lanes of up to 256 symbols, where more would mostly be read in
// vain, 256 for longer ones; on the stress workload 64 / 128 / 256 take 0.61 / 0.52 / 0.47 ms).
constexpr int kPackTileStride = 66;  // 16-bit elements: 33 dwords, odd, so a column read spreads over the banks

template <int kPackTile>
__global__ __launch_bounds__(256) void k_pack_by_thread(uint32_t lanes, uint32_t lane_cap,
                                                        const uint16_t *__restrict__ scratch,
                                                        const uint32_t *__restrict__ lane_state,
                                                        const uint32_t *__restrict__ offsets,
                                                        uint16_t *__restrict__ payload,
                                                        const Status *__restrict__ status)
{
    if (status->code != ST_OK) return;
    __shared__ uint32_t s_first[64];  // payload word index of the lane's state
    __shared__ uint32_t s_nw[64];     // words after the state
    __shared__ uint32_t s_max;
    __shared__ __align__(4) uint16_t tile[kPackTile * kPackTileStride];
    const uint32_t t = threadIdx.x;
    const uint32_t l0 = blockIdx.x * 64u;
    if (t == 0) s_max = 0u;
    __syncthreads();
    if (t < 64u) {
        uint32_t nw = 0u, first = 0u;
        if (l0 + t < lanes) {
            const uint32_t begin = offsets[l0 + t], end = offsets[l0 + t + 1];
            const uint32_t st = lane_state[l0 + t];
            first = begin >> 1;
            nw = (end - begin - 4u) >> 1;
            payload[first] = (uint16_t)st;
            payload[first + 1u] = (uint16_t)(st >> 16);
            atomicMax(&s_max, nw);
        }
        s_first[t] = first;
        s_nw[t] = nw;
    }
    __syncthreads();
    const uint32_t max_nw = s_max;
    const uint16_t *rows = scratch + (size_t)l0 * lane_cap;
    for (uint32_t k0 = 0; k0 < max_nw; k0 += kPackTile) {
        // rows k0 .. k0 + 63 of the block, two lanes (one dword) per thread and 8 rows apart; all
        // eight are asked for before the first is stored (guarded one by one, every load would wait
        // for the one before); rows past the last one repeat it and are never read
        uint32_t v[kPackTile / 8];
#pragma unroll
        for (int j = 0; j < kPackTile / 8; ++j) {
            const uint32_t r = min(k0 + (t >> 5) + 8u * j, max_nw - 1u);
            v[j] = *reinterpret_cast<const uint32_t *>(rows + (size_t)r * 64u + 2u * (t & 31u));
        }
#pragma unroll
        for (int j = 0; j < kPackTile / 8; ++j)
            *reinterpret_cast<uint32_t *>(&tile[((t >> 5) + 8u * j) * kPackTileStride + 2u * (t & 31u)]) = v[j];
        __syncthreads();
        // wavefront w writes lanes 16 w .. 16 w + 15; its thread u has word numbers k0 + u, k0 + 64 + u, ...
#pragma unroll 4
        for (int j = 0; j < 16; ++j) {
            const uint32_t i = (t >> 6) * 16u + j;
            const uint32_t nw = s_nw[i];
#pragma unroll
            for (uint32_t part = 0; part < (uint32_t)kPackTile; part += 64u) {
                const uint32_t row = part + (t & 63u), k = k0 + row;
                if (k < nw) payload[s_first[i] + 2u + (nw - 1u - k)] = tile[row * kPackTileStride + i];
            }
        }
        __syncthreads();
    }
}

// --------------------------------------------------------------------------------------------
// Decode.
// --------------------------------------------------------------------------------------------
__global__ void k_init_status(Status *status)
{
    status->code = ST_OK;
    status->ticket = 0;
    status->payload_bytes = 0;
}

// The same, and the look-back descriptors of the one-pass encoder cleared.
__global__ void k_init_one_pass(Status *status, unsigned long long *desc, uint32_t n)
{
    const uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i == 0u) {
        status->code = ST_OK;
        status->ticket = 0;
        status->payload_bytes = 0;
    }
    if (i < n) desc[i] = 0ull;
}

// `word11` is header word 11 for containers that use it (the number of mixture components);
// containers that leave it reserved pass 0 and it is not looked at.
__global__ void k_check_header(Geo g, uint32_t magic, uint32_t word11,
                               const uint8_t *__restrict__ coded, unsigned long long coded_bytes,
                               Status *__restrict__ status)
{
    const uint32_t *h = reinterpret_cast<const uint32_t *>(coded);
    int st = ST_OK;
    unsigned long long payload = (unsigned long long)h[12] | ((unsigned long long)h[13] << 32);
    if (h[0] != magic || h[1] != PILC_VERSION) st = ST_FORMAT;
    if (word11 != 0u && h[11] != word11) st = ST_FORMAT;
    if (h[2] != g.n || h[3] != g.h || h[4] != g.w || h[5] != 3u || h[6] != g.prec_bits ||
        h[7] != g.lane_mode || h[8] != g.lane_a || h[9] != g.lane_b || h[10] != g.lanes)
        st = ST_FORMAT;
    if (coded_bytes != kHeaderBytes + 4ull * ((unsigned long long)g.lanes + 1ull) + payload)
        st = ST_FORMAT;
    if (st == ST_OK) {
        const uint32_t *offsets = h + kHeaderBytes / 4;
        if (payload >= (1ull << 32) || offsets[0] != 0u || offsets[g.lanes] != (uint32_t)payload)
            st = ST_CORRUPT;
    }
    status->code = st;
    status->payload_bytes = payload;
}

}  // namespace pilc

#include "pilc_lane_kernels.hpp"
#include "pilc_block_encode.hpp"
#include "pilc_row_decode.hpp"
#include "pilc_mix.hpp"

namespace pilc {

// --------------------------------------------------------------------------------------------
// Host side
// --------------------------------------------------------------------------------------------
// 0 chosen from the lane count, 1 thread per lane, 2 the kernels for few long lanes, 3 thread per
// lane with the one-pass encoder (the lane kernel also scans and packs)
static std::atomic<int> g_kernel_policy{0};
static std::atomic<int> g_ansai_decode_waves{0};  // 0: chosen per call
// Bound of a look-back wait of the one-pass encoder in ticks of the constant-rate clock (0: two
// seconds), and the switch that makes its first workgroup publish nothing (tests only).
static std::atomic<unsigned long long> g_one_pass_wait{0};
static std::atomic<int> g_one_pass_withhold{0};

// The few-lane kernels pay off while there are too few lanes to fill the chip with one thread
// each (256 CUs x 4 SIMDs x 64 threads = 65,536 threads for a single wave per SIMD).  Measured
// on CIFAR-shaped data cut into lanes of different lengths, the block encoder is ahead of the
// thread-per-lane encoder up to about 28K lanes (1.85 against 2.15 ms at 25,000 lanes, 1.74
// against 1.13 ms at 50,000) and the row decoder up to about 13K (7.8 against 15.5 ms at 6250
// lanes, 7.5 against 7.8 ms at 12,500, 6.4 against 4.2 ms at 25,000; on uniformly random pixels
// 5.3 against 7.7 ms at 8192 lanes, 4.7 against 3.9 ms at 16,384).
static bool use_few_lane_kernels(const Geo &g, bool decode)
{
    const int policy = g_kernel_policy.load(std::memory_order_relaxed);
    if (policy == 1 || policy == 3) return false;
    if (policy == 2) return true;
    return g.lanes <= (decode ? 12288u : 28672u);
}

thread_local char t_hip_error[256] = "";
thread_local float t_timing_ms[16];
thread_local const char *t_timing_name[16];
thread_local int t_timing_count = 0;
static std::atomic<int> g_timing_enabled{0};

static int hip_fail(hipError_t e, const char *what)
{
    snprintf(t_hip_error, sizeof(t_hip_error), "%s: %s", what, hipGetErrorString(e));
    return PILC_E_HIP;
}

#define HIP_TRY(expr)                                   \
    do {                                                \
        hipError_t e_ = (expr);                         \
        if (e_ != hipSuccess) return hip_fail(e_, #expr); \
    } while (0)

static std::mutex g_table_mutex;
static bool g_table_ready[64] = {false};

static int ensure_tables()
{
    int dev = 0;
    HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= 64) return PILC_E_ARG;
    std::lock_guard<std::mutex> lock(g_table_mutex);
    if (g_table_ready[dev]) return PILC_OK;
    static uint32_t sig[kSigEntries + 1];
    static uint2 cell[kSigEntries];
    static uint32_t eh[kExpHiEntries], el[kExpLoEntries];
    for (int i = 0; i <= kSigEntries; ++i)
        sig[i] = (uint32_t)std::llround(std::ldexp(1.0 / (1.0 + std::exp(-(i - 1024) / 64.0)), 24));
    for (int i = 0; i < kSigEntries; ++i) cell[i] = make_uint2(sig[i], (sig[i + 1] - sig[i]) << 6);
    for (int i = 0; i < kExpHiEntries; ++i)
        eh[i] = (uint32_t)std::llround(std::ldexp(std::exp(4.0 - i / 64.0), 26));
    for (int i = 0; i < kExpLoEntries; ++i)
        el[i] = (uint32_t)std::llround(std::ldexp(std::exp(-i / 4096.0), 31));
    HIP_TRY(hipMemcpyToSymbol(HIP_SYMBOL(g_sig_cell), cell, sizeof(cell)));
    HIP_TRY(hipMemcpyToSymbol(HIP_SYMBOL(g_exp_hi), eh, sizeof(eh)));
    HIP_TRY(hipMemcpyToSymbol(HIP_SYMBOL(g_exp_lo), el, sizeof(el)));
    HIP_TRY(hipDeviceSynchronize());
    g_table_ready[dev] = true;
    return PILC_OK;
}

static uint64_t ceil_div64(uint64_t a, uint64_t b) { return (a + b - 1) / b; }

// Validates a geometry and derives the kernel-side view.  Returns PILC_OK / PILC_E_*.
static int make_geo(const pilc_geom *in, Geo *g)
{
    if (!in || in->n == 0 || in->h == 0 || in->w == 0) return PILC_E_ARG;
    if (in->prec_bits < 10 || in->prec_bits > 16) return PILC_E_ARG;
    uint64_t hw = (uint64_t)in->h * in->w;
    uint64_t total = hw * in->n;
    uint64_t lanes;
    if (in->lane_mode == 0) {
        if (in->lane_a == 0) return PILC_E_ARG;
        if (hw % in->lane_a != 0 && in->lane_a % hw != 0) return PILC_E_ARG;
        lanes = ceil_div64(total, in->lane_a);
    } else if (in->lane_mode == 1) {
        if (in->lane_a == 0 || in->lane_b == 0) return PILC_E_ARG;
        lanes = (uint64_t)in->n * ceil_div64(in->h, in->lane_a) * ceil_div64(in->w, in->lane_b);
    } else {
        return PILC_E_ARG;
    }
    // 32-bit symbol indices and lane numbers inside the kernels
    if (total * 3 + lanes + 4096 >= (1ull << 32)) return PILC_E_TOO_LARGE;
    g->n = in->n;
    g->h = in->h;
    g->w = in->w;
    g->hw = (uint32_t)hw;
    g->prec_bits = in->prec_bits;
    g->lane_mode = in->lane_mode;
    g->lane_a = in->lane_a;
    g->lane_b = in->lane_b;
    g->tiles_x = in->lane_mode == 1 ? (uint32_t)ceil_div64(in->w, in->lane_b) : 1u;
    g->tiles_per_img =
        in->lane_mode == 1 ? (uint32_t)(ceil_div64(in->h, in->lane_a) * g->tiles_x) : 1u;
    g->total_px = (uint32_t)total;
    g->lanes = (uint32_t)lanes;
    g->by_hw = FastDiv::make(g->hw);
    return PILC_OK;
}

static size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }

// Symbols of the longest lane.
static uint32_t max_lane_symbols(const Geo &g)
{
    const uint64_t px = g.lane_mode == 0 ? (uint64_t)(g.lane_a < g.total_px ? g.lane_a : g.total_px)
                                         : (uint64_t)(g.lane_a < g.h ? g.lane_a : g.h) *
                                               (g.lane_b < g.w ? g.lane_b : g.w);
    return (uint32_t)(3u * px);
}

struct Workspace {
    size_t status_off, words_off, state_off, sums_off, desc_off, scratch_off, total;
    uint32_t scan_blocks;
};

static Workspace layout(const Geo &g)
{
    Workspace w;
    w.scan_blocks = (uint32_t)ceil_div64(g.lanes, kScanTile);
    size_t off = 0;
    w.status_off = off;
    off = align256(off + sizeof(Status));
    w.words_off = off;
    off = align256(off + 4 * (size_t)g.lanes);
    w.state_off = off;
    off = align256(off + 4 * (size_t)g.lanes);
    w.sums_off = off;
    off = align256(off + 8 * (size_t)w.scan_blocks);
    w.desc_off = off;  // one look-back descriptor per workgroup of the one-pass encoder (>= 64 lanes each)
    off = align256(off + 8 * (size_t)ceil_div64(g.lanes, 64));
    w.scratch_off = off;
    // one 16-bit word per symbol, plus one spare word per lane for the branch-free encoder; the
    // thread-per-lane encoder gives every lane of a block of 64 the room of the longest lane
    const size_t linear = (size_t)g.total_px * 3 + g.lanes + 64;
    const size_t by_thread = (((size_t)g.lanes + 63) & ~(size_t)63) * max_lane_symbols(g);
    off = align256(off + 2 * (linear > by_thread ? linear : by_thread));
    w.total = off;
    return w;
}

static int status_to_error(int st)
{
    switch (st) {
    case ST_OK: return PILC_OK;
    case ST_CAPACITY: return PILC_E_CAPACITY;
    case ST_TOO_LARGE: return PILC_E_TOO_LARGE;
    case ST_FORMAT: return PILC_E_FORMAT;
    case ST_PARAMS: return PILC_E_ARG;
    case ST_TIMEOUT: return PILC_E_TIMEOUT;
    default: return PILC_E_CORRUPT;
    }
}

// Optional per-kernel event timing on the caller's stream.  The events are created once per host
// thread and device and reused by every later call.
struct EventPool {
    int dev = -1;
    hipEvent_t ev[17];
};
thread_local EventPool t_events;

struct Timer {
    hipStream_t stream;
    hipEvent_t *ev = nullptr;
    const char *name[16];
    int n = 0;
    bool on;
    explicit Timer(hipStream_t s, bool allowed = true)
        : stream(s), on(allowed && g_timing_enabled.load(std::memory_order_relaxed) != 0)
    {
        t_timing_count = 0;
        if (!on) return;
        int dev = -1;
        if (hipGetDevice(&dev) != hipSuccess) {
            on = false;
            return;
        }
        if (t_events.dev != dev) {
            if (t_events.dev >= 0)
                for (auto &e : t_events.ev) (void)hipEventDestroy(e);
            t_events.dev = -1;
            for (auto &e : t_events.ev)
                if (hipEventCreate(&e) != hipSuccess) {
                    on = false;
                    return;
                }
            t_events.dev = dev;
        }
        ev = t_events.ev;
        (void)hipEventRecord(ev[0], stream);
    }
    void mark(const char *what)
    {
        if (on && n < 16) {
            name[n] = what;
            (void)hipEventRecord(ev[++n], stream);
        }
    }
    void finish()  // call after the stream has been synchronised
    {
        if (!on) return;
        t_timing_name[0] = "total";
        (void)hipEventElapsedTime(&t_timing_ms[0], ev[0], ev[n]);
        for (int i = 0; i < n && i < 15; ++i) {
            t_timing_name[i + 1] = name[i];
            (void)hipEventElapsedTime(&t_timing_ms[i + 1], ev[i], ev[i + 1]);
        }
        t_timing_count = n + 1 > 16 ? 16 : n + 1;
    }
};

// Kernels that take more than 64 KB of dynamic LDS need the limit raised once per device; it is
// raised to all of a compute unit's 160 KB less the kernel's static part, so that no later call
// ever has to change it again.
static std::mutex g_lds_mutex;
static std::map<std::pair<const void *, int>, bool> g_lds_raised;
static int allow_large_lds(const void *kernel)
{
    int dev = 0;
    HIP_TRY(hipGetDevice(&dev));
    std::lock_guard<std::mutex> lock(g_lds_mutex);
    bool &done = g_lds_raised[std::make_pair(kernel, dev)];
    if (!done) {
        hipFuncAttributes fa;
        HIP_TRY(hipFuncGetAttributes(&fa, kernel));
        HIP_TRY(hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize,
                                    160 * 1024 - (int)fa.sharedSizeBytes));
        done = true;
    }
    return PILC_OK;
}

// True when every 8-pixel chunk of every lane starts at a multiple of 8 pixels, never straddles
// two images, and the arrays allow 16-byte (parameters) / 8-byte (pixels) vector accesses.
static bool chunks_aligned(const Geo &g, const void *img, const pilc_params *p)
{
    const bool geo = g.lane_mode == 0 ? (g.lane_a % 8 == 0 && g.hw % 8 == 0)
                                      : (g.w % 8 == 0 && g.lane_b % 8 == 0);
    return geo && ((uintptr_t)img & 7) == 0 && ((uintptr_t)p->mu & 15) == 0 &&
           ((uintptr_t)p->log_scale & 15) == 0;
}

// Workgroup size of the thread-per-lane kernels (at most kRingMaxThreads: the decoder's word ring
// in LDS is sized for that).
// On top of chunks_aligned: every row of every lane is a whole number of 16-pixel chunk pairs
// that start at multiples of 16 pixels, and the pixels allow 16-byte loads.
static bool chunks_pair_up(const Geo &g, const void *img)
{
    const bool geo = g.lane_mode == 0 ? (g.lane_a % 16 == 0 && g.hw % 16 == 0)
                                      : (g.w % 16 == 0 && g.lane_b % 16 == 0);
    return geo && ((uintptr_t)img & 15) == 0;
}

// On top of chunks_pair_up: flat lanes of whole 64-pixel groups (three 128-byte lines of each
// parameter array) that start on a line.
static bool lanes_line_up(const Geo &g, const pilc_params *p)
{
    return g.lane_mode == 0 && g.lane_a % 64 == 0 && g.total_px % g.lane_a == 0 &&
           ((uintptr_t)p->mu & 127) == 0 && ((uintptr_t)p->log_scale & 127) == 0;
}

static int lane_block_threads(const Geo &g) { return g.lanes >= (1u << 16) ? kRingMaxThreads : 64; }

}  // namespace pilc

using namespace pilc;

extern "C" {

uint32_t pilc_version(void) { return PILC_VERSION; }

const char *pilc_strerror(int code)
{
    switch (code) {
    case PILC_OK: return "success";
    case PILC_E_ARG: return "invalid argument (null or misaligned pointer, or bad geometry)";
    case PILC_E_WORKSPACE: return "workspace too small";
    case PILC_E_CAPACITY: return "coded output does not fit the given capacity";
    case PILC_E_TOO_LARGE: return "batch too large for 32-bit offsets";
    case PILC_E_FORMAT: return "container header does not match (magic, version, geometry or size)";
    case PILC_E_CORRUPT: return "container is corrupt (offsets, lane overrun or final state)";
    case PILC_E_HIP: return "HIP runtime failure";
    case PILC_E_TIMEOUT: return "a bounded wait between workgroups ran out";
    default: return "unknown error code";
    }
}

const char *pilc_last_hip_error(void) { return t_hip_error; }

void pilc_set_timing(int enabled) { g_timing_enabled.store(enabled, std::memory_order_relaxed); }

int pilc_set_kernel_policy(int policy)
{
    if (policy < 0 || policy > 3) return PILC_E_ARG;
    g_kernel_policy.store(policy, std::memory_order_relaxed);
    return PILC_OK;
}

void pilc_set_one_pass_wait(uint64_t ticks, int withhold_first)
{
    g_one_pass_wait.store(ticks, std::memory_order_relaxed);
    g_one_pass_withhold.store(withhold_first != 0, std::memory_order_relaxed);
}

int pilc_last_timing(float *ms_out_host, int capacity)
{
    int k = t_timing_count < capacity ? t_timing_count : capacity;
    for (int i = 0; i < k; ++i) ms_out_host[i] = t_timing_ms[i];
    return k;
}

const char *pilc_timing_name(int i)
{
    return (i >= 0 && i < t_timing_count) ? t_timing_name[i] : "";
}

uint64_t pilc_lane_count(const pilc_geom *geom)
{
    Geo g;
    return make_geo(geom, &g) == PILC_OK ? g.lanes : 0;
}

int pilc_workspace_size(const pilc_geom *geom, size_t *workspace_bytes_host,
                        size_t *max_coded_bytes_host)
{
    Geo g;
    int rc = make_geo(geom, &g);
    if (rc != PILC_OK) return rc;
    if (workspace_bytes_host) *workspace_bytes_host = layout(g).total;
    if (max_coded_bytes_host)
        *max_coded_bytes_host = kHeaderBytes + 4 * ((size_t)g.lanes + 1) + 4 * (size_t)g.lanes +
                                2 * (size_t)g.total_px * 3;
    return PILC_OK;
}

static bool params_ok(const pilc_params *p)
{
    return p && p->mu && p->log_scale && p->chan_coef && ((uintptr_t)p->mu & 1) == 0 &&
           ((uintptr_t)p->log_scale & 1) == 0 && ((uintptr_t)p->chan_coef & 1) == 0;
}

int pilc_symbol_tables(const pilc_geom *geom, const uint8_t *img_dev, const pilc_params *params,
                       uint32_t *cum_out_dev, uint32_t *freq_out_dev, void *hip_stream)
{
    Geo g;
    int rc = make_geo(geom, &g);
    if (rc != PILC_OK) return rc;
    if (!img_dev || !params_ok(params) || !cum_out_dev || !freq_out_dev ||
        ((uintptr_t)cum_out_dev & 3) || ((uintptr_t)freq_out_dev & 3))
        return PILC_E_ARG;
    if ((rc = ensure_tables()) != PILC_OK) return rc;
    hipStream_t stream = (hipStream_t)hip_stream;
    uint32_t blocks = (uint32_t)ceil_div64(g.total_px, 256);
    k_symbol_tables<<<blocks, 256, 0, stream>>>(g, img_dev, params->mu, params->log_scale,
                                                params->chan_coef, cum_out_dev, freq_out_dev);
    HIP_TRY(hipGetLastError());
    HIP_TRY(hipStreamSynchronize(stream));
    return PILC_OK;
}

// The body of pilc_encode once the arguments have been checked: `workspace_dev` holds at least
// layout(g).total bytes.  `timed` is false for callers that must not create HIP events.
static int encode_checked(const Geo &g, const uint8_t *img_dev, const pilc_params *params,
                          void *workspace_dev, uint8_t *coded_dev, size_t coded_capacity,
                          uint64_t *coded_bytes_host, hipStream_t stream, bool timed)
{
    const Workspace ws = layout(g);
    const size_t table_end = kHeaderBytes + 4 * ((size_t)g.lanes + 1);
    uint8_t *base = static_cast<uint8_t *>(workspace_dev);
    Status *status = reinterpret_cast<Status *>(base + ws.status_off);
    uint32_t *lane_words = reinterpret_cast<uint32_t *>(base + ws.words_off);
    uint32_t *lane_state = reinterpret_cast<uint32_t *>(base + ws.state_off);
    unsigned long long *sums = reinterpret_cast<unsigned long long *>(base + ws.sums_off);
    uint16_t *scratch = reinterpret_cast<uint16_t *>(base + ws.scratch_off);
    uint32_t *offsets = reinterpret_cast<uint32_t *>(coded_dev + kHeaderBytes);
    uint16_t *payload = reinterpret_cast<uint16_t *>(coded_dev + table_end);

    Timer timer(stream, timed);
    const bool few_lanes = use_few_lane_kernels(g, false);
    const uint32_t lane_cap = few_lanes ? 0u : max_lane_symbols(g);  // selects the scratch layout
    const HeaderWords head = {{kMagicPilc, PILC_VERSION, g.n, g.h, g.w, 3u, g.prec_bits,
                               g.lane_mode, g.lane_a, g.lane_b, g.lanes, 0u}};
    // Policy 3: the lane kernel also scans and packs (one pass).  Not the default: measured 5 %
    // (64 x 64 images, one lane per row) to 10 % (16 x 16 tiles of video frames) slower than the
    // lane kernel followed by the scan and pack kernels.
    const bool one_pass = !few_lanes && g_kernel_policy.load(std::memory_order_relaxed) == 3;
    OnePass op = {};
    if (one_pass) {
        const int bt = lane_block_threads(g);
        const uint32_t nb = (uint32_t)ceil_div64(g.lanes, bt);
        int dev = 0, khz = 0;
        HIP_TRY(hipGetDevice(&dev));
        if (hipDeviceGetAttribute(&khz, hipDeviceAttributeWallClockRate, dev) != hipSuccess || khz <= 0)
            khz = 100000;
        const unsigned long long wait = g_one_pass_wait.load(std::memory_order_relaxed);
        op.desc = reinterpret_cast<unsigned long long *>(base + ws.desc_off);
        op.ticket = &status->ticket;
        op.status = status;
        op.coded = coded_dev;
        op.payload_capacity = coded_capacity - table_end;
        op.wait_ticks = wait ? wait : 2000ull * (unsigned long long)khz;
        op.groups = nb;
        op.withhold_first = (uint32_t)g_one_pass_withhold.load(std::memory_order_relaxed);
        op.head = head;
        k_init_one_pass<<<(nb + 255u) / 256u, 256, 0, stream>>>(status, op.desc, nb);
    } else {
        k_init_status<<<1, 1, 0, stream>>>(status);
    }
    if (few_lanes) {
        k_encode_block<<<(uint32_t)ceil_div64(g.lanes, kEncLanes), kEncThreads, 0, stream>>>(
            g, img_dev, params->mu, params->log_scale, params->chan_coef, scratch, lane_words, lane_state);
    } else {
        const int bt = lane_block_threads(g);
        uint32_t nb = (uint32_t)ceil_div64(g.lanes, bt);
        if (one_pass) {
            // workgroups take groups of lanes from a counter until none is left: no more of them
            // than the chip holds at once (a workgroup that starts late finds nothing to do)
            int dev = 0, cus = 0;
            HIP_TRY(hipGetDevice(&dev));
            if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0)
                cus = 256;
            const uint32_t resident = (uint32_t)cus * (uint32_t)(1024 / bt);
            if (nb > resident) nb = resident;
        }
        const bool vec = chunks_aligned(g, img_dev, params);
        const bool pair = vec && chunks_pair_up(g, img_dev);
        const bool line = pair && lanes_line_up(g, params);
#define PILC_LAUNCH_ENCODE(ONE, VEC, PAIR, LINE)                                                      \
    k_encode_lanes<ONE, VEC, PAIR, LINE><<<nb, bt, 0, stream>>>(g, img_dev, params->mu, params->log_scale, \
                                                               params->chan_coef, scratch, lane_cap,  \
                                                               lane_words, lane_state, op)
        if (one_pass) {
            if (line) PILC_LAUNCH_ENCODE(true, true, true, true);
            else if (pair) PILC_LAUNCH_ENCODE(true, true, true, false);
            else if (vec) PILC_LAUNCH_ENCODE(true, true, false, false);
            else PILC_LAUNCH_ENCODE(true, false, false, false);
        } else {
            if (line) PILC_LAUNCH_ENCODE(false, true, true, true);
            else if (pair) PILC_LAUNCH_ENCODE(false, true, true, false);
            else if (vec) PILC_LAUNCH_ENCODE(false, true, false, false);
            else PILC_LAUNCH_ENCODE(false, false, false, false);
        }
#undef PILC_LAUNCH_ENCODE
    }
    timer.mark(few_lanes ? "k_encode_block" : "k_encode_lanes");
    if (!one_pass) {
        const ItemBytes lane_bytes = {4u, 2u, 0u, 0u};  // a 32-bit state and 16-bit words
        k_scan_partials<<<ws.scan_blocks, kScanThreads, 0, stream>>>(g.lanes, lane_bytes, lane_words, sums);
        k_scan_spine<<<1, kScanThreads, 0, stream>>>(head, g.lanes, ws.scan_blocks, sums, coded_dev,
                                                     (unsigned long long)coded_capacity, status);
        k_scan_apply<<<ws.scan_blocks, kScanThreads, 0, stream>>>(g.lanes, lane_bytes, lane_words, sums,
                                                                  offsets);
        timer.mark("scan");
        // a run of lanes per workgroup: about 16K symbols' worth, at most 256 lanes
        const uint32_t lane_sym = max_lane_symbols(g);
        uint32_t pack_lanes = 16384u / (lane_sym ? lane_sym : 1u);
        pack_lanes = pack_lanes < 1 ? 1 : (pack_lanes > (uint32_t)kPackMaxLanes ? kPackMaxLanes : pack_lanes);
        if (lane_cap != 0u)
            (lane_cap <= 256u ? k_pack_by_thread<128> : k_pack_by_thread<256>)<<<(uint32_t)ceil_div64(g.lanes, 64), 256, 0, stream>>>(
                g.lanes, lane_cap, scratch, lane_state, offsets, payload, status);
        else
            k_pack<<<(uint32_t)ceil_div64(g.lanes, pack_lanes), 256, 0, stream>>>(
                g, pack_lanes, scratch, lane_state, offsets, payload, status);
        timer.mark(lane_cap != 0u ? "k_pack_by_thread" : "k_pack");
    }
    HIP_TRY(hipGetLastError());
    Status host_status;
    HIP_TRY(hipMemcpyAsync(&host_status, status, sizeof(Status), hipMemcpyDeviceToHost, stream));
    HIP_TRY(hipStreamSynchronize(stream));
    timer.finish();
    if (host_status.code != ST_OK) return status_to_error(host_status.code);
    *coded_bytes_host = table_end + host_status.payload_bytes;
    return PILC_OK;
}

int pilc_encode(const pilc_geom *geom, const uint8_t *img_dev, const pilc_params *params,
                void *workspace_dev, size_t workspace_bytes, uint8_t *coded_dev,
                size_t coded_capacity, uint64_t *coded_bytes_host, void *hip_stream)
{
    Geo g;
    int rc = make_geo(geom, &g);
    if (rc != PILC_OK) return rc;
    if (!img_dev || !params_ok(params) || !workspace_dev || !coded_dev || !coded_bytes_host)
        return PILC_E_ARG;
    if (((uintptr_t)workspace_dev & 255) || ((uintptr_t)coded_dev & 15)) return PILC_E_ARG;
    if (workspace_bytes < layout(g).total) return PILC_E_WORKSPACE;
    if (coded_capacity < kHeaderBytes + 4 * ((size_t)g.lanes + 1)) return PILC_E_CAPACITY;
    if ((rc = ensure_tables()) != PILC_OK) return rc;
    return encode_checked(g, img_dev, params, workspace_dev, coded_dev, coded_capacity,
                          coded_bytes_host, (hipStream_t)hip_stream, true);
}

// --------------------------------------------------------------------------------------------
// pilc_encode for callers that cannot allocate device memory: the workspace is a file-scope
// device array.  Every GPU holds its own copy at its own address; the address is asked for once
// per device, with that device current, and host code uses only that pointer (the array's name
// is not a device address in host code).
// --------------------------------------------------------------------------------------------
static __device__ __align__(256) unsigned char scratch[PILC_STATIC_SCRATCH_BYTES];

static std::mutex g_scratch_mutex;
static void *g_scratch_ptr[64] = {nullptr};

static int static_scratch(void **out)
{
    int dev = 0;
    HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= 64) return PILC_E_ARG;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *ptr = nullptr;
        HIP_TRY(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
        if (!ptr || ((uintptr_t)ptr & 255)) {
            snprintf(t_hip_error, sizeof(t_hip_error), "hipGetSymbolAddress(scratch) gave %p", ptr);
            return PILC_E_HIP;
        }
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return PILC_OK;
}

int pilc_encode_static(const pilc_geom *geom, const uint8_t *img_dev, const pilc_params *params,
                       uint8_t *coded_dev, size_t coded_capacity, uint64_t *coded_bytes_host,
                       void *hip_stream)
{
    Geo g;
    int rc = make_geo(geom, &g);
    if (rc != PILC_OK) return rc;
    if (!img_dev || !params_ok(params) || !coded_dev || !coded_bytes_host) return PILC_E_ARG;
    if ((uintptr_t)coded_dev & 15) return PILC_E_ARG;
    if (layout(g).total > (size_t)PILC_STATIC_SCRATCH_BYTES) return PILC_E_WORKSPACE;
    if (coded_capacity < kHeaderBytes + 4 * ((size_t)g.lanes + 1)) return PILC_E_CAPACITY;
    if ((rc = ensure_tables()) != PILC_OK) return rc;
    void *ws = nullptr;
    if ((rc = static_scratch(&ws)) != PILC_OK) return rc;
    // Nothing in the workspace has to start at zero: the status block is set by the first kernel
    // and every count, state and scratch word that is read has been written by this call.
    return encode_checked(g, img_dev, params, ws, coded_dev, coded_capacity, coded_bytes_host,
                          (hipStream_t)hip_stream, false);
}

int pilc_decode(const pilc_geom *geom, const uint8_t *coded_dev, size_t coded_bytes,
                const pilc_params *params, void *workspace_dev, size_t workspace_bytes,
                uint8_t *img_out_dev, void *hip_stream)
{
    Geo g;
    int rc = make_geo(geom, &g);
    if (rc != PILC_OK) return rc;
    if (!coded_dev || !params_ok(params) || !workspace_dev || !img_out_dev) return PILC_E_ARG;
    if (((uintptr_t)workspace_dev & 255) || ((uintptr_t)coded_dev & 15)) return PILC_E_ARG;
    const Workspace ws = layout(g);
    if (workspace_bytes < ws.total) return PILC_E_WORKSPACE;
    const size_t table_end = kHeaderBytes + 4 * ((size_t)g.lanes + 1);
    if (coded_bytes < table_end) return PILC_E_FORMAT;  // cannot even hold header + offsets
    if ((rc = ensure_tables()) != PILC_OK) return rc;

    hipStream_t stream = (hipStream_t)hip_stream;
    Status *status = reinterpret_cast<Status *>(static_cast<uint8_t *>(workspace_dev) + ws.status_off);

    Timer timer(stream);
    k_check_header<<<1, 1, 0, stream>>>(g, kMagicPilc, 0u, coded_dev, (unsigned long long)coded_bytes, status);
    timer.mark("k_check_header");
    const bool few_lanes = use_few_lane_kernels(g, true);
    if (few_lanes) {
        // all lanes alike and made of whole batches of 16 pixels: no per-row activity masks
        const bool even = g.lane_mode == 0 ? (g.lane_a % kRowBatch == 0 && g.total_px % g.lane_a == 0)
                                           : (g.h % g.lane_a == 0 && g.w % g.lane_b == 0 &&
                                              (g.lane_a * g.lane_b) % kRowBatch == 0);
        const uint32_t nblk = (uint32_t)ceil_div64(g.lanes, kRowLanes);
        // a stager beside every decoding wavefront while one workgroup per compute unit holds all lanes
        int dev = 0, cus = 0, khz = 0;
        if (hipGetDevice(&dev) != hipSuccess ||
            hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0)
            cus = 256;
        if (hipDeviceGetAttribute(&khz, hipDeviceAttributeWallClockRate, dev) != hipSuccess || khz <= 0) khz = 100000;
        const bool staged = nblk <= (uint32_t)cus;
        // the bound of the waits between a decoding wavefront and its stager, and the test switch
        const unsigned long long asked = g_one_pass_wait.load(std::memory_order_relaxed);
        const unsigned long long wait_ticks = asked ? asked : 2000ull * (unsigned long long)khz;
        const uint32_t withhold = (uint32_t)g_one_pass_withhold.load(std::memory_order_relaxed);
#define PILC_DECODE_ROWS(RAGGED, STAGED)                                                              \
    k_decode_rows<RAGGED, STAGED><<<nblk, (STAGED ? 2 : 1) * 64 * kRowWaves, 0, stream>>>(           \
        g, coded_dev, params->mu, params->log_scale, params->chan_coef, img_out_dev, &status->code,   \
        &status->payload_bytes, wait_ticks, withhold)
        if (even && staged) PILC_DECODE_ROWS(false, true);
        else if (even) PILC_DECODE_ROWS(false, false);
        else if (staged) PILC_DECODE_ROWS(true, true);
        else PILC_DECODE_ROWS(true, false);
#undef PILC_DECODE_ROWS
    } else {
        const int bt = lane_block_threads(g);
        const uint32_t nb = (uint32_t)ceil_div64(g.lanes, bt);
        if (chunks_aligned(g, img_out_dev, params) && chunks_pair_up(g, img_out_dev) && lanes_line_up(g, params))
            k_decode_lanes<true, true, true><<<nb, bt, 0, stream>>>(g, coded_dev, params->mu, params->log_scale,
                                                                    params->chan_coef, img_out_dev,
                                                                    &status->code, &status->payload_bytes);
        else if (chunks_aligned(g, img_out_dev, params) && chunks_pair_up(g, img_out_dev))
            k_decode_lanes<true, true><<<nb, bt, 0, stream>>>(g, coded_dev, params->mu, params->log_scale,
                                                              params->chan_coef, img_out_dev,
                                                              &status->code, &status->payload_bytes);
        else if (chunks_aligned(g, img_out_dev, params))
            k_decode_lanes<true, false><<<nb, bt, 0, stream>>>(g, coded_dev, params->mu, params->log_scale,
                                                               params->chan_coef, img_out_dev,
                                                               &status->code, &status->payload_bytes);
        else
            k_decode_lanes<false, false><<<nb, bt, 0, stream>>>(g, coded_dev, params->mu,
                                                                params->log_scale, params->chan_coef,
                                                                img_out_dev, &status->code,
                                                                &status->payload_bytes);
    }
    timer.mark(few_lanes ? "k_decode_rows" : "k_decode_lanes");
    HIP_TRY(hipGetLastError());
    Status host_status;
    HIP_TRY(hipMemcpyAsync(&host_status, status, sizeof(Status), hipMemcpyDeviceToHost, stream));
    HIP_TRY(hipStreamSynchronize(stream));
    timer.finish();
    return status_to_error(host_status.code);
}

// --------------------------------------------------------------------------------------------
// Mixture of K logistic laws per subpixel
// --------------------------------------------------------------------------------------------
static bool mix_params_ok(const pilc_mix_params *p)
{
    return p && p->mu && p->log_scale && p->weight && p->chan_coef && p->num_comp >= 1u &&
           p->num_comp <= (uint32_t)kMixMaxComp && ((uintptr_t)p->mu & 1) == 0 &&
           ((uintptr_t)p->log_scale & 1) == 0 && ((uintptr_t)p->weight & 1) == 0 &&
           ((uintptr_t)p->chan_coef & 1) == 0;
}

// The component count a mixture kernel was built for (components in registers: arrays on 4-byte
// boundaries), or 0 for the kernels that take any K at run time.
static int mix_built_for(const pilc_mix_params *p)
{
    const bool aligned =
        (((uintptr_t)p->mu | (uintptr_t)p->log_scale | (uintptr_t)p->weight) & 3) == 0;
    return aligned ? (int)p->num_comp : 0;
}

#define PILC_MIX_KERNEL_FOR(NAME)                                                                \
    static decltype(&NAME<0>) NAME##_for(int built)                                              \
    {                                                                                            \
        switch (built) {                                                                         \
        case 1: return NAME<1>;                                                                  \
        case 2: return NAME<2>;                                                                  \
        case 3: return NAME<3>;                                                                  \
        case 4: return NAME<4>;                                                                  \
        case 5: return NAME<5>;                                                                  \
        case 6: return NAME<6>;                                                                  \
        case 7: return NAME<7>;                                                                  \
        case 8: return NAME<8>;                                                                  \
        case 9: return NAME<9>;                                                                  \
        case 10: return NAME<10>;                                                                \
        case 11: return NAME<11>;                                                                \
        case 12: return NAME<12>;                                                                \
        case 13: return NAME<13>;                                                                \
        case 14: return NAME<14>;                                                                \
        case 15: return NAME<15>;                                                                \
        case 16: return NAME<16>;                                                                \
        default: return NAME<0>;                                                                 \
        }                                                                                        \
    }
PILC_MIX_KERNEL_FOR(k_mix_encode)
PILC_MIX_KERNEL_FOR(k_mix_decode)
#undef PILC_MIX_KERNEL_FOR

int pilc_mix_encode(const pilc_geom *geom, const uint8_t *img_dev, const pilc_mix_params *params,
                    void *workspace_dev, size_t workspace_bytes, uint8_t *coded_dev,
                    size_t coded_capacity, uint64_t *coded_bytes_host, void *hip_stream)
{
    Geo g;
    int rc = make_geo(geom, &g);
    if (rc != PILC_OK) return rc;
    if (!img_dev || !mix_params_ok(params) || !workspace_dev || !coded_dev || !coded_bytes_host)
        return PILC_E_ARG;
    if (((uintptr_t)workspace_dev & 255) || ((uintptr_t)coded_dev & 15)) return PILC_E_ARG;
    const Workspace ws = layout(g);
    if (workspace_bytes < ws.total) return PILC_E_WORKSPACE;
    const size_t table_end = kHeaderBytes + 4 * ((size_t)g.lanes + 1);
    if (coded_capacity < table_end) return PILC_E_CAPACITY;
    if ((rc = ensure_tables()) != PILC_OK) return rc;

    hipStream_t stream = (hipStream_t)hip_stream;
    uint8_t *base = static_cast<uint8_t *>(workspace_dev);
    Status *status = reinterpret_cast<Status *>(base + ws.status_off);
    uint32_t *lane_words = reinterpret_cast<uint32_t *>(base + ws.words_off);
    uint32_t *lane_state = reinterpret_cast<uint32_t *>(base + ws.state_off);
    unsigned long long *sums = reinterpret_cast<unsigned long long *>(base + ws.sums_off);
    uint16_t *scratch = reinterpret_cast<uint16_t *>(base + ws.scratch_off);
    uint32_t *offsets = reinterpret_cast<uint32_t *>(coded_dev + kHeaderBytes);
    uint16_t *payload = reinterpret_cast<uint16_t *>(coded_dev + table_end);
    const MixArgs args = {params->mu, params->log_scale, params->weight, params->chan_coef,
                          params->num_comp};
    const int built = mix_built_for(params);
    const size_t lds = mix_lds_bytes(params->num_comp, built == 0);
    auto kern = k_mix_encode_for(built);
    if ((rc = allow_large_lds(reinterpret_cast<const void *>(kern))) != PILC_OK) return rc;

    Timer timer(stream);
    k_init_status<<<1, 1, 0, stream>>>(status);
    const uint32_t lane_cap = max_lane_symbols(g);
    kern<<<(uint32_t)ceil_div64(g.lanes, kMixThreads), kMixThreads, lds, stream>>>(
        g, img_dev, args, scratch, lane_cap, lane_words, lane_state, &status->code);
    timer.mark("k_mix_encode");
    const ItemBytes lane_bytes = {4u, 2u, 0u, 0u};
    const HeaderWords head = {{kMagicMix, PILC_VERSION, g.n, g.h, g.w, 3u, g.prec_bits, g.lane_mode,
                               g.lane_a, g.lane_b, g.lanes, params->num_comp}};
    k_scan_partials<<<ws.scan_blocks, kScanThreads, 0, stream>>>(g.lanes, lane_bytes, lane_words, sums);
    k_scan_spine<<<1, kScanThreads, 0, stream>>>(head, g.lanes, ws.scan_blocks, sums, coded_dev,
                                                 (unsigned long long)coded_capacity, status);
    k_scan_apply<<<ws.scan_blocks, kScanThreads, 0, stream>>>(g.lanes, lane_bytes, lane_words, sums,
                                                              offsets);
    timer.mark("scan");
    (lane_cap <= 256u ? k_pack_by_thread<128> : k_pack_by_thread<256>)<<<(uint32_t)ceil_div64(g.lanes, 64), 256, 0, stream>>>(
        g.lanes, lane_cap, scratch, lane_state, offsets, payload, status);
    timer.mark("k_pack_by_thread");
    HIP_TRY(hipGetLastError());
    Status host_status;
    HIP_TRY(hipMemcpyAsync(&host_status, status, sizeof(Status), hipMemcpyDeviceToHost, stream));
    HIP_TRY(hipStreamSynchronize(stream));
    timer.finish();
    if (host_status.code != ST_OK) return status_to_error(host_status.code);
    *coded_bytes_host = table_end + host_status.payload_bytes;
    return PILC_OK;
}

int pilc_mix_decode(const pilc_geom *geom, const uint8_t *coded_dev, size_t coded_bytes,
                    const pilc_mix_params *params, void *workspace_dev, size_t workspace_bytes,
                    uint8_t *img_out_dev, void *hip_stream)
{
    Geo g;
    int rc = make_geo(geom, &g);
    if (rc != PILC_OK) return rc;
    if (!coded_dev || !mix_params_ok(params) || !workspace_dev || !img_out_dev) return PILC_E_ARG;
    if (((uintptr_t)workspace_dev & 255) || ((uintptr_t)coded_dev & 15)) return PILC_E_ARG;
    const Workspace ws = layout(g);
    if (workspace_bytes < ws.total) return PILC_E_WORKSPACE;
    const size_t table_end = kHeaderBytes + 4 * ((size_t)g.lanes + 1);
    if (coded_bytes < table_end) return PILC_E_FORMAT;
    if ((rc = ensure_tables()) != PILC_OK) return rc;

    hipStream_t stream = (hipStream_t)hip_stream;
    Status *status = reinterpret_cast<Status *>(static_cast<uint8_t *>(workspace_dev) + ws.status_off);
    const MixArgs args = {params->mu, params->log_scale, params->weight, params->chan_coef,
                          params->num_comp};
    const int built = mix_built_for(params);
    const size_t lds = mix_lds_bytes(params->num_comp, built == 0);
    auto kern = k_mix_decode_for(built);
    if ((rc = allow_large_lds(reinterpret_cast<const void *>(kern))) != PILC_OK) return rc;

    Timer timer(stream);
    k_check_header<<<1, 1, 0, stream>>>(g, kMagicMix, params->num_comp, coded_dev,
                                        (unsigned long long)coded_bytes, status);
    timer.mark("k_check_header");
    kern<<<(uint32_t)ceil_div64(g.lanes, kMixThreads), kMixThreads, lds, stream>>>(
        g, coded_dev, args, img_out_dev, &status->code, &status->payload_bytes);
    timer.mark("k_mix_decode");
    HIP_TRY(hipGetLastError());
    Status host_status;
    HIP_TRY(hipMemcpyAsync(&host_status, status, sizeof(Status), hipMemcpyDeviceToHost, stream));
    HIP_TRY(hipStreamSynchronize(stream));
    timer.finish();
    return status_to_error(host_status.code);
}

}  // extern "C"

#include "pilc_ansai.hpp"
#include "pilc_twar.hpp"
