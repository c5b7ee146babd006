// The table-driven coder of Sec. 3.2 (Alg. 3 "ANS-AI: Encode x", Alg. 4 "ANS-AI: Decode one
// symbol") for gfx950: one thread per piece (Sec. 4.3), the tables of a workgroup in LDS.
//
// What bounds these kernels is memory, not arithmetic (a symbol costs about twenty integer
// instructions, and two to three bytes of HBM traffic), so the layout work is all about moving
// whole cache lines:
//   - the symbol and index rows of a wavefront's 64 pieces are staged through LDS in chunks that
//     are aligned in the arrays, with 16-byte loads in which consecutive threads cover one
//     row's chunk, so every line is fetched once and fully used;
//   - the encoder's words go to a scratch area laid out [wavefront][word][thread], so the 64
//     threads of a wavefront, which emit at nearly the same rate, fill the same lines together;
//   - k_ansai_pack turns that layout into the container's records through an LDS transpose.
//
// Included at the end of pilc.hip (needs its Status, scan kernels, Timer and host helpers).
#pragma once

namespace pilc {

// ---------------------------------------------------------------------------------------------
// Shapes and the table blob
// ---------------------------------------------------------------------------------------------
struct AShape {
    uint32_t pieces, count;  // pieces * count < 2^32
    uint32_t M, D, X;
};

constexpr uint32_t kAnsaiMagic = 0x534E4150u;     // "PANS"
constexpr uint32_t kAnsaiTabMagic = 0x42544150u;  // tag of a built table blob
constexpr int ST_ARG = 1;                         // a symbol / index out of range, or foreign tables

// Device blob written by k_ansai_build: 256-byte header, then
//   enc   uint2 [D*X]         { delta, phi }                       (Alg. 3)
//   theta uint8 [D << M]      symbol                               (Alg. 4)
//   nb    u16 or u32 [D << M] (N - 2^M) << 4 | B; 32-bit entries when M > 12
struct ATabHeader {
    uint32_t magic, M, D, X, ok;
    uint32_t pad[59];
};

struct ATabLayout {
    size_t enc_off, theta_off, nb_off, total;
    bool wide;
};

static inline ATabLayout ansai_tab_layout(uint32_t M, uint32_t D, uint32_t X)
{
    ATabLayout t;
    t.wide = M > 12;
    t.enc_off = sizeof(ATabHeader);
    t.theta_off = (t.enc_off + 8 * (size_t)D * X + 255) & ~(size_t)255;
    t.nb_off = (t.theta_off + ((size_t)D << M) + 255) & ~(size_t)255;
    t.total = (t.nb_off + ((size_t)D << M) * (t.wide ? 4 : 2) + 255) & ~(size_t)255;
    return t;
}

__global__ void k_ansai_build_begin(ATabHeader *head, uint32_t M, uint32_t D, uint32_t X)
{
    head->magic = kAnsaiTabMagic;
    head->M = M;
    head->D = D;
    head->X = X;
    head->ok = 1u;
}

// One workgroup per distribution.  Validates the masses (every P_x >= 1, sum 2^M) and writes
// delta = k 2^M - P_x 2^k for the k with P_x 2^k in [2^M, 2^(M+1)) (App. B, lemma on the range
// of delta), phi = 2^M - P_x + C_x, and for every state value the outcome of Alg. 2: the symbol,
// the number of bits it pops and the state it reaches before they are added.
template <bool kWide>
__global__ __launch_bounds__(256) void k_ansai_build(uint32_t M, uint32_t X,
                                                     const uint32_t *__restrict__ mass,
                                                     ATabHeader *head, uint2 *__restrict__ enc,
                                                     uint8_t *__restrict__ theta,
                                                     void *__restrict__ nb_raw)
{
    __shared__ uint32_t cum[257];
    __shared__ int bad;
    const uint32_t d = blockIdx.x, top = 1u << M;
    if (threadIdx.x == 0) {
        unsigned long long run = 0;
        int b = 0;
        for (uint32_t x = 0; x < X; ++x) {
            const uint32_t p = mass[d * X + x];
            cum[x] = (uint32_t)run;
            if (p == 0 || p > top) b = 1;
            run += p;
        }
        cum[X] = (uint32_t)run;
        if (run != top) b = 1;
        bad = b;
        if (b) atomicExch(&head->ok, 0u);
    }
    __syncthreads();
    if (bad) return;
    for (uint32_t x = threadIdx.x; x < X; x += blockDim.x) {
        const uint32_t p = cum[x + 1] - cum[x];
        const uint32_t k = M - (31u - __clz(p));
        enc[d * X + x] = make_uint2(k * top - (p << k), top - p + cum[x]);
    }
    for (uint32_t s = threadIdx.x; s < top; s += blockDim.x) {
        uint32_t lo = 0, hi = X - 1;  // largest x with cum[x] <= s
        while (lo < hi) {
            const uint32_t mid = (lo + hi + 1) >> 1;
            if (cum[mid] <= s)
                lo = mid;
            else
                hi = mid - 1;
        }
        const uint32_t t = s - cum[lo] + (cum[lo + 1] - cum[lo]);  // in [P_x, 2 P_x)
        const uint32_t len = 32u - __clz(t);
        const uint32_t b = len > M ? 0u : M + 1u - len;
        const uint32_t nrel = (t << b) - top;
        theta[((size_t)d << M) + s] = (uint8_t)lo;
        if (kWide)
            static_cast<uint32_t *>(nb_raw)[((size_t)d << M) + s] = nrel << 4 | b;
        else
            static_cast<uint16_t *>(nb_raw)[((size_t)d << M) + s] = (uint16_t)(nrel << 4 | b);
    }
}

// ---------------------------------------------------------------------------------------------
// Staging of a wavefront's 64 rows through LDS
// ---------------------------------------------------------------------------------------------
// A row is the `count` bytes of one piece in a [pieces, count] array.  It is cut at multiples of
// kChunk bytes of the array; stage number `st` of a row is its st-th chunk from the front
// (decode) or from the back (encode).  In LDS a row takes kChunk/4 + 1 dwords: an odd stride,
// so the 64 threads that each walk their own row hit distinct banks.
template <int kChunk>
struct Stage {
    static constexpr int kVec = kChunk / 16;     // 16-byte vectors per row
    static constexpr int kRow = kChunk / 4 + 1;  // LDS dwords per row
    static constexpr int kDwords = 64 * kRow;    // per wavefront and array
};

// Orders this wavefront's LDS accesses: LDS instructions of one wavefront execute in order, so
// all that is needed is that the compiler keeps them in order too.
__device__ __forceinline__ void wave_lds_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

struct RowStage {
    uint32_t chunk;   // chunk index in the array
    uint32_t lo, hi;  // the row's bytes inside that chunk: [lo, hi), empty when the row has none
};

template <int kChunk>
__device__ __forceinline__ RowStage row_stage(uint32_t piece, uint32_t count, uint32_t st,
                                              bool from_back, bool row_exists)
{
    const uint32_t rb = piece * count, re = rb + count;
    const uint32_t first = rb / kChunk, last = (re - 1u) / kChunk;
    RowStage r;
    r.chunk = from_back ? last - st : first + st;
    if (!row_exists || st > last - first) {
        r.lo = r.hi = 0;
        return r;
    }
    const uint32_t cb = r.chunk * kChunk;
    r.lo = rb > cb ? rb - cb : 0u;
    r.hi = re < cb + kChunk ? re - cb : (uint32_t)kChunk;
    return r;
}

// Cooperative load of stage `st` of the rows of pieces p0 .. p0+np-1 into `rows`.
template <int kChunk>
__device__ __forceinline__ void stage_load(const uint8_t *__restrict__ arr, uint32_t total_bytes,
                                           uint32_t *rows, uint32_t p0, uint32_t np,
                                           uint32_t count, uint32_t st, bool from_back)
{
    using S = Stage<kChunk>;
    const uint32_t lane = threadIdx.x & 63u;
#pragma unroll
    for (int i = 0; i < S::kVec; ++i) {
        const uint32_t idx = i * 64 + lane, r = idx / S::kVec, c = idx % S::kVec;
        const RowStage rs = row_stage<kChunk>(p0 + r, count, st, from_back, r < np);
        if (rs.hi > rs.lo) {
            const uint32_t off = rs.chunk * kChunk + c * 16u;
            uint4 v;
            if (off + 16u <= total_bytes) {
                v = *reinterpret_cast<const uint4 *>(arr + off);
            } else {  // the array ends inside this vector
                uint32_t w0 = 0u, w1 = 0u, w2 = 0u, w3 = 0u;
#pragma unroll
                for (uint32_t k = 0; k < 4u; ++k) {
                    const uint32_t sh8 = 8u * k;
                    if (off + k < total_bytes) w0 |= (uint32_t)arr[off + k] << sh8;
                    if (off + 4u + k < total_bytes) w1 |= (uint32_t)arr[off + 4u + k] << sh8;
                    if (off + 8u + k < total_bytes) w2 |= (uint32_t)arr[off + 8u + k] << sh8;
                    if (off + 12u + k < total_bytes) w3 |= (uint32_t)arr[off + 12u + k] << sh8;
                }
                v = make_uint4(w0, w1, w2, w3);
            }
            uint32_t *dst = rows + r * S::kRow + c * 4u;
            dst[0] = v.x;
            dst[1] = v.y;
            dst[2] = v.z;
            dst[3] = v.w;
        }
    }
}

// Cooperative store of stage `st` (front order) from `rows`: only bytes that belong to a row.
template <int kChunk>
__device__ __forceinline__ void stage_store(uint8_t *__restrict__ arr, const uint32_t *rows,
                                            uint32_t p0, uint32_t np, uint32_t count, uint32_t st)
{
    using S = Stage<kChunk>;
    const uint32_t lane = threadIdx.x & 63u;
#pragma unroll
    for (int i = 0; i < S::kVec; ++i) {
        const uint32_t idx = i * 64 + lane, r = idx / S::kVec, c = idx % S::kVec;
        const RowStage rs = row_stage<kChunk>(p0 + r, count, st, false, r < np);
        const uint32_t vb = c * 16u;
        if (rs.hi > rs.lo && vb < rs.hi && vb + 16u > rs.lo) {
            const uint32_t *src = rows + r * S::kRow + c * 4u;
            const uint32_t off = rs.chunk * kChunk + vb;
            if (rs.lo <= vb && vb + 16u <= rs.hi) {
                *reinterpret_cast<uint4 *>(arr + off) = make_uint4(src[0], src[1], src[2], src[3]);
            } else {
                for (uint32_t k = 0; k < 16u; ++k)
                    if (vb + k >= rs.lo && vb + k < rs.hi)
                        arr[off + k] = (uint8_t)(src[k >> 2] >> (8u * (k & 3u)));
            }
        }
    }
}

__device__ __forceinline__ uint32_t ansai_stage_count(uint32_t count, int chunk)
{
    // a row of `count` bytes starting anywhere touches at most this many chunks
    return (count + 2u * (uint32_t)chunk - 2u) / (uint32_t)chunk;
}

// ---------------------------------------------------------------------------------------------
// Encode (Alg. 3), symbols of a piece taken last-first
// ---------------------------------------------------------------------------------------------
constexpr int kAnsaiEncWaves = 4;

struct EncLane {
    uint32_t S;     // state in [2^M, 2^(M+1))
    uint32_t acc;   // bits pushed and not yet written, low bit first
    uint32_t nacc;  // how many of them, < 32
    uint32_t woff;  // scratch index of the next word
    uint32_t nwords;
    uint32_t bad;
};

template <bool kTabLds>
__device__ __forceinline__ void ansai_push(EncLane &L, uint32_t x, uint32_t d, const AShape &sh,
                                           const uint2 *tab, uint32_t *__restrict__ scratch)
{
    L.bad |= (uint32_t)(x >= sh.X) | (uint32_t)(d >= sh.D);
    const uint32_t idx = min(d, sh.D - 1u) * sh.X + min(x, sh.X - 1u);
    const uint2 e = tab[idx];
    const uint32_t b = (e.x + L.S) >> sh.M;  // Alg. 3: number of bits to push
    const uint32_t low = L.S & ((1u << b) - 1u);
    L.acc |= low << L.nacc;
    uint32_t nn = L.nacc + b;
    if (nn >= 32u) {  // b <= 15, so nacc >= 17 here and the shift below is in 1..15
        scratch[L.woff] = L.acc;
        L.woff += 64u;
        L.nwords += 1u;
        L.acc = low >> (32u - L.nacc);
        nn -= 32u;
    }
    L.nacc = nn;
    L.S = (L.S >> b) + e.y;
}

template <int kChunk, bool kTabLds>
__global__ __launch_bounds__(64 * kAnsaiEncWaves) void k_ansai_encode(
    AShape sh, const uint8_t *__restrict__ sym, const uint8_t *__restrict__ dist,
    const uint2 *__restrict__ enc_tab, uint32_t *__restrict__ scratch, uint32_t maxw,
    uint32_t *__restrict__ piece_bits, uint32_t *__restrict__ piece_state, int *status)
{
    using S = Stage<kChunk>;
    extern __shared__ uint32_t lds[];
    if (*status != ST_OK) return;  // the tables are not the ones this shape needs
    const uint2 *tab = enc_tab;
    uint32_t *stage_base = lds;
    if (kTabLds) {
        uint2 *t = reinterpret_cast<uint2 *>(lds);
        for (uint32_t i = threadIdx.x; i < sh.D * sh.X; i += blockDim.x) t[i] = enc_tab[i];
        tab = t;
        stage_base = lds + 2u * sh.D * sh.X;
        __syncthreads();
    }
    const uint32_t wave = threadIdx.x >> 6, lane = threadIdx.x & 63u;
    const uint32_t gw = blockIdx.x * kAnsaiEncWaves + wave;
    const uint32_t p0 = gw * 64u;
    if (p0 >= sh.pieces) return;
    const uint32_t np = min(64u, sh.pieces - p0);
    uint32_t *srow = stage_base + wave * 2u * S::kDwords;
    uint32_t *drow = srow + S::kDwords;
    const uint32_t total = sh.pieces * sh.count;
    const bool mine = lane < np;

    EncLane L;
    L.S = 1u << sh.M;
    L.acc = 0u;
    L.nacc = 0u;
    L.woff = gw * maxw * 64u + lane;
    L.nwords = 0u;
    L.bad = 0u;

    const uint32_t stages = ansai_stage_count(sh.count, kChunk);
    for (uint32_t st = 0; st < stages; ++st) {
        wave_lds_sync();
        stage_load<kChunk>(sym, total, srow, p0, np, sh.count, st, true);
        stage_load<kChunk>(dist, total, drow, p0, np, sh.count, st, true);
        wave_lds_sync();
        const RowStage rs = row_stage<kChunk>(p0 + lane, sh.count, st, true, mine);
        const uint32_t *ms = srow + lane * S::kRow, *md = drow + lane * S::kRow;
        if (__all(rs.lo == 0u && rs.hi == (uint32_t)kChunk)) {
#pragma unroll 1
            for (int dw = kChunk / 4 - 1; dw >= 0; --dw) {
                const uint32_t s4 = ms[dw], d4 = md[dw];
#pragma unroll
                for (int k = 3; k >= 0; --k)
                    ansai_push<kTabLds>(L, (s4 >> (8 * k)) & 255u, (d4 >> (8 * k)) & 255u, sh, tab, scratch);
            }
        } else {
#pragma unroll 1
            for (int dw = kChunk / 4 - 1; dw >= 0; --dw) {
                const uint32_t s4 = ms[dw], d4 = md[dw];
#pragma unroll
                for (int k = 3; k >= 0; --k)
                    if ((uint32_t)(dw * 4 + k) - rs.lo < rs.hi - rs.lo)
                        ansai_push<kTabLds>(L, (s4 >> (8 * k)) & 255u, (d4 >> (8 * k)) & 255u, sh, tab, scratch);
            }
        }
    }
    if (mine) {
        if (L.nacc) scratch[L.woff] = L.acc;
        piece_bits[p0 + lane] = L.nwords * 32u + L.nacc;
        piece_state[p0 + lane] = L.S;
        if (L.bad) *status = ST_ARG;
    }
}

// ---------------------------------------------------------------------------------------------
// Pack: scratch [wavefront][word][thread] -> records {state, bit count, words} at the offsets
// ---------------------------------------------------------------------------------------------
constexpr int kAnsaiPackWaves = 4;
constexpr int kAnsaiPackRows = 16;

__global__ __launch_bounds__(64 * kAnsaiPackWaves) void k_ansai_pack(
    AShape sh, const uint32_t *__restrict__ scratch, uint32_t maxw,
    const uint32_t *__restrict__ piece_bits, const uint32_t *__restrict__ piece_state,
    const uint32_t *__restrict__ offsets, uint32_t *__restrict__ payload,
    const Status *__restrict__ status)
{
    if (status->code != ST_OK) return;
    __shared__ uint32_t tile[kAnsaiPackWaves][64 * (kAnsaiPackRows + 1)];
    __shared__ uint32_t s_dst[kAnsaiPackWaves][64];  // payload dword index of the piece's words
    __shared__ uint32_t s_nw[kAnsaiPackWaves][64];
    const uint32_t wave = threadIdx.x >> 6, lane = threadIdx.x & 63u;
    const uint32_t gw = blockIdx.x * kAnsaiPackWaves + wave;
    const uint32_t p0 = gw * 64u;
    if (p0 >= sh.pieces) return;
    const uint32_t np = min(64u, sh.pieces - p0);
    uint32_t nw = 0;
    if (lane < np) {
        const uint32_t bits = piece_bits[p0 + lane], at = offsets[p0 + lane] >> 2;
        nw = (bits + 31u) >> 5;
        payload[at] = piece_state[p0 + lane];
        payload[at + 1u] = bits;
        s_dst[wave][lane] = at + 2u;
    }
    s_nw[wave][lane] = nw;
    uint32_t most = nw;
    for (int d = 32; d >= 1; d >>= 1) most = max(most, (uint32_t)__shfl_xor((int)most, d, 64));
    const uint32_t *src = scratch + (size_t)gw * maxw * 64u + lane;
    uint32_t *mine = tile[wave] + lane * (kAnsaiPackRows + 1);
    for (uint32_t j0 = 0; j0 < most; j0 += kAnsaiPackRows) {
        wave_lds_sync();
#pragma unroll
        for (int jj = 0; jj < kAnsaiPackRows; ++jj)
            if (j0 + jj < most) mine[jj] = src[(size_t)(j0 + jj) * 64u];
        wave_lds_sync();
#pragma unroll
        for (int i = 0; i < 16; ++i) {  // 4 pieces per pass, 16 threads each
            const uint32_t r = i * 4 + (lane >> 4), jj = lane & 15u, j = j0 + jj;
            if (j < s_nw[wave][r]) payload[s_dst[wave][r] + j] = tile[wave][r * (kAnsaiPackRows + 1) + jj];
        }
    }
}

// ---------------------------------------------------------------------------------------------
// Decode (Alg. 4)
// ---------------------------------------------------------------------------------------------
__global__ void k_ansai_begin(AShape sh, const ATabHeader *__restrict__ tab, Status *status)
{
    status->code = (tab->magic == kAnsaiTabMagic && tab->ok == 1u && tab->M == sh.M && tab->D == sh.D &&
                    tab->X == sh.X)
                       ? ST_OK
                       : ST_ARG;
    status->pad = 0;
    status->payload_bytes = 0;
}

__global__ void k_ansai_check_header(AShape sh, const uint8_t *__restrict__ coded,
                                     unsigned long long coded_bytes, Status *__restrict__ status)
{
    if (status->code != ST_OK) return;
    const uint32_t *h = reinterpret_cast<const uint32_t *>(coded);
    int st = ST_OK;
    const unsigned long long payload = (unsigned long long)h[12] | ((unsigned long long)h[13] << 32);
    if (h[0] != kAnsaiMagic || h[1] != 1u || h[2] != sh.pieces || h[3] != sh.count || h[4] != sh.M ||
        h[5] != sh.D || h[6] != sh.X)
        st = ST_FORMAT;
    if (coded_bytes != kHeaderBytes + 4ull * ((unsigned long long)sh.pieces + 1ull) + payload)
        st = ST_FORMAT;
    if (st == ST_OK && payload >= (1ull << 32)) st = ST_CORRUPT;
    status->code = st;
    status->payload_bytes = payload;
}

struct DecLane {
    uint32_t s;          // state minus 2^M
    unsigned long long win;  // the top n bits of the stream, right-aligned; win < 2^n
    uint32_t n;          // < 64
    uint32_t widx;       // payload dword index one past the next word to take
    uint32_t wleft;      // words not yet taken
    uint32_t bad, corrupt;
};

__device__ __forceinline__ void ansai_refill(DecLane &L, const uint32_t *__restrict__ payload)
{
    if (L.n < 32u && L.wleft > 0u) {
        L.widx -= 1u;
        L.wleft -= 1u;
        L.win = (L.win << 32) | payload[L.widx];
        L.n += 32u;
    }
}

template <bool kWide>
__device__ __forceinline__ uint32_t ansai_pop(DecLane &L, uint32_t d, const AShape &sh,
                                              const uint8_t *theta, const void *nb_raw)
{
    L.bad |= (uint32_t)(d >= sh.D);
    const uint32_t ti = (min(d, sh.D - 1u) << sh.M) + L.s;
    const uint32_t e = kWide ? static_cast<const uint32_t *>(nb_raw)[ti]
                             : (uint32_t) static_cast<const uint16_t *>(nb_raw)[ti];
    const uint32_t x = theta[ti];
    const uint32_t b = e & 15u;
    L.corrupt |= (uint32_t)(b > L.n);  // the stream ran dry
    L.n = max(L.n, b) - b;
    const uint32_t v = (uint32_t)(L.win >> L.n);  // the last b bits, in the order they were pushed
    L.win -= (unsigned long long)v << L.n;
    L.s = (e >> 4) + v;  // Alg. 4: S <- N[d,S] + popped bits
    return x;
}

template <int kChunk, bool kWide, bool kTabLds>
__global__ __launch_bounds__(1024) void k_ansai_decode(
    AShape sh, const uint8_t *__restrict__ coded, const uint8_t *__restrict__ dist,
    const uint8_t *__restrict__ theta_g, const void *__restrict__ nb_g, uint8_t *__restrict__ out,
    uint32_t maxw, Status *status)
{
    using S = Stage<kChunk>;
    extern __shared__ uint32_t lds[];
    if (status->code != ST_OK) return;
    const uint8_t *theta = theta_g;
    const void *nb = nb_g;
    uint32_t *stage_base = lds;
    if (kTabLds) {
        const uint32_t entries = sh.D << sh.M;  // a multiple of 4 whenever M >= 2; padded otherwise
        const uint32_t th_dw = (entries + 3u) >> 2, nb_dw = kWide ? entries : (entries + 1u) >> 1;
        const uint32_t *tg = reinterpret_cast<const uint32_t *>(theta_g);
        const uint32_t *ng = reinterpret_cast<const uint32_t *>(nb_g);
        for (uint32_t i = threadIdx.x; i < th_dw; i += blockDim.x) lds[i] = tg[i];
        for (uint32_t i = threadIdx.x; i < nb_dw; i += blockDim.x) lds[th_dw + i] = ng[i];
        theta = reinterpret_cast<const uint8_t *>(lds);
        nb = lds + th_dw;
        stage_base = lds + th_dw + nb_dw;
        __syncthreads();
    }
    const uint32_t waves = blockDim.x >> 6;
    const uint32_t wave = threadIdx.x >> 6, lane = threadIdx.x & 63u;
    const uint32_t gw = blockIdx.x * waves + wave;
    const uint32_t p0 = gw * 64u;
    if (p0 >= sh.pieces) return;
    const uint32_t np = min(64u, sh.pieces - p0);
    uint32_t *rows = stage_base + wave * S::kDwords;
    const uint32_t total = sh.pieces * sh.count;
    const uint32_t top = 1u << sh.M;
    const uint32_t *offsets = reinterpret_cast<const uint32_t *>(coded + kHeaderBytes);
    const uint32_t *payload = offsets + sh.pieces + 1u;
    const uint32_t payload_bytes = (uint32_t)status->payload_bytes;

    bool mine = lane < np;
    DecLane L;
    L.s = 0u;
    L.win = 0ull;
    L.n = 0u;
    L.widx = 0u;
    L.wleft = 0u;
    L.bad = 0u;
    L.corrupt = 0u;
    if (mine) {
        const uint32_t begin = offsets[p0 + lane], end = offsets[p0 + lane + 1u];
        bool ok = end >= begin && end - begin >= 8u && end <= payload_bytes && ((begin | end) & 3u) == 0u;
        if (ok) {
            const uint32_t state = payload[begin >> 2], bits = payload[(begin >> 2) + 1u];
            const uint32_t nw = (end - begin - 8u) >> 2;
            // no piece of `count` symbols holds more than maxw words
            ok = nw <= maxw && state >= top && state < 2u * top && bits <= 32u * nw && bits + 31u >= 32u * nw;
            if (ok) {
                L.s = state - top;
                L.widx = (begin >> 2) + 2u + nw;
                L.wleft = nw;
                if (nw > 0u) {  // the last word holds the top 1..32 bits
                    const uint32_t r = bits - 32u * (nw - 1u);
                    L.widx -= 1u;
                    L.wleft -= 1u;
                    L.win = payload[L.widx] & (0xFFFFFFFFu >> (32u - r));
                    L.n = r;
                }
            }
        }
        if (!ok) {
            L.corrupt = 1u;
            mine = false;
        }
    }

    const uint32_t stages = ansai_stage_count(sh.count, kChunk);
    for (uint32_t st = 0; st < stages; ++st) {
        wave_lds_sync();
        stage_load<kChunk>(dist, total, rows, p0, np, sh.count, st, false);
        wave_lds_sync();
        const RowStage rs = row_stage<kChunk>(p0 + lane, sh.count, st, false, mine);
        uint32_t *my = rows + lane * S::kRow;
        if (__all(rs.lo == 0u && rs.hi == (uint32_t)kChunk)) {
#pragma unroll 1
            for (int dw = 0; dw < kChunk / 4; ++dw) {
                const uint32_t d4 = my[dw];
                uint32_t x4 = 0u;
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    if ((k & 1) == 0) ansai_refill(L, payload);
                    x4 |= ansai_pop<kWide>(L, (d4 >> (8 * k)) & 255u, sh, theta, nb) << (8 * k);
                }
                my[dw] = x4;
            }
        } else {
#pragma unroll 1
            for (int dw = 0; dw < kChunk / 4; ++dw) {
                const uint32_t d4 = my[dw];
                uint32_t x4 = 0u;
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    // a check per symbol here: which symbols of a pair run depends on the row
                    if ((uint32_t)(dw * 4 + k) - rs.lo < rs.hi - rs.lo) {
                        ansai_refill(L, payload);
                        x4 |= ansai_pop<kWide>(L, (d4 >> (8 * k)) & 255u, sh, theta, nb) << (8 * k);
                    }
                }
                my[dw] = x4;
            }
        }
        wave_lds_sync();
        stage_store<kChunk>(out, rows, p0, np, sh.count, st);
    }
    if (mine && (L.s != 0u || L.n != 0u || L.wleft != 0u)) L.corrupt = 1u;
    if (L.corrupt)
        status->code = ST_CORRUPT;
    else if (L.bad)
        status->code = ST_ARG;
}

// ---------------------------------------------------------------------------------------------
// Host side
// ---------------------------------------------------------------------------------------------
static int make_ashape(const pilc_ansai_shape *in, AShape *sh)
{
    if (!in || in->pieces == 0 || in->count == 0) return PILC_E_ARG;
    if (in->prec_bits < 1 || in->prec_bits > 15 || in->num_dist < 1 || in->num_dist > 256 ||
        in->num_sym < 2 || in->num_sym > 256 || (1u << in->prec_bits) < in->num_sym)
        return PILC_E_ARG;
    // 32-bit byte offsets into the [pieces, count] arrays and 32-bit scratch word indices
    const uint64_t padded = ((uint64_t)in->pieces + 63) / 64 * 64;
    const uint64_t maxw = ((uint64_t)in->count * in->prec_bits + 31) / 32;
    if (padded * in->count + 4096 >= (1ull << 32) || padded * maxw + 4096 >= (1ull << 32))
        return PILC_E_TOO_LARGE;
    sh->pieces = in->pieces;
    sh->count = in->count;
    sh->M = in->prec_bits;
    sh->D = in->num_dist;
    sh->X = in->num_sym;
    return PILC_OK;
}

struct AWorkspace {
    size_t status_off, bits_off, state_off, sums_off, scratch_off, total;
    uint32_t scan_blocks, maxw, waves;
};

static AWorkspace ansai_layout(const AShape &sh)
{
    AWorkspace w;
    w.scan_blocks = (uint32_t)ceil_div64(sh.pieces, kScanTile);
    w.maxw = (uint32_t)(((uint64_t)sh.count * sh.M + 31) / 32);
    w.waves = (uint32_t)ceil_div64(sh.pieces, 64);
    size_t off = 0;
    w.status_off = off;
    off = align256(off + sizeof(Status));
    w.bits_off = off;
    off = align256(off + 4 * (size_t)sh.pieces);
    w.state_off = off;
    off = align256(off + 4 * (size_t)sh.pieces);
    w.sums_off = off;
    off = align256(off + 8 * (size_t)w.scan_blocks);
    w.scratch_off = off;
    off = align256(off + 4 * (size_t)w.waves * 64 * w.maxw);
    w.total = off;
    return w;
}

static int ansai_status_to_error(int st) { return st == ST_ARG ? PILC_E_ARG : status_to_error(st); }

constexpr int kAnsaiChunk = 64;

// LDS one workgroup may use on gfx950: the whole 160 KB of a compute unit.
constexpr size_t kLdsBytes = 160 * 1024;

}  // namespace pilc

using namespace pilc;

extern "C" {

size_t pilc_ansai_table_bytes(uint32_t prec_bits, uint32_t num_dist, uint32_t num_sym)
{
    pilc_ansai_shape s = {1u, 1u, prec_bits, num_dist, num_sym};
    AShape sh;
    if (make_ashape(&s, &sh) != PILC_OK) return 0;
    return ansai_tab_layout(sh.M, sh.D, sh.X).total;
}

int pilc_ansai_build_tables(uint32_t prec_bits, uint32_t num_dist, uint32_t num_sym,
                            const uint32_t *mass_dev, void *tables_dev, size_t tables_bytes,
                            void *hip_stream)
{
    pilc_ansai_shape s = {1u, 1u, prec_bits, num_dist, num_sym};
    AShape sh;
    int rc = make_ashape(&s, &sh);
    if (rc != PILC_OK) return rc;
    if (!mass_dev || !tables_dev || ((uintptr_t)mass_dev & 3) || ((uintptr_t)tables_dev & 255))
        return PILC_E_ARG;
    const ATabLayout t = ansai_tab_layout(sh.M, sh.D, sh.X);
    if (tables_bytes < t.total) return PILC_E_WORKSPACE;
    hipStream_t stream = (hipStream_t)hip_stream;
    uint8_t *base = static_cast<uint8_t *>(tables_dev);
    ATabHeader *head = reinterpret_cast<ATabHeader *>(base);
    k_ansai_build_begin<<<1, 1, 0, stream>>>(head, sh.M, sh.D, sh.X);
    if (t.wide)
        k_ansai_build<true><<<sh.D, 256, 0, stream>>>(sh.M, sh.X, mass_dev, head,
                                                      reinterpret_cast<uint2 *>(base + t.enc_off),
                                                      base + t.theta_off, base + t.nb_off);
    else
        k_ansai_build<false><<<sh.D, 256, 0, stream>>>(sh.M, sh.X, mass_dev, head,
                                                       reinterpret_cast<uint2 *>(base + t.enc_off),
                                                       base + t.theta_off, base + t.nb_off);
    HIP_TRY(hipGetLastError());
    ATabHeader host;
    HIP_TRY(hipMemcpyAsync(&host, head, sizeof(host), hipMemcpyDeviceToHost, stream));
    HIP_TRY(hipStreamSynchronize(stream));
    return host.ok == 1u ? PILC_OK : PILC_E_ARG;
}

int pilc_ansai_workspace_size(const pilc_ansai_shape *shape, size_t *workspace_bytes_host,
                              size_t *max_coded_bytes_host)
{
    AShape sh;
    int rc = make_ashape(shape, &sh);
    if (rc != PILC_OK) return rc;
    const AWorkspace ws = ansai_layout(sh);
    if (workspace_bytes_host) *workspace_bytes_host = ws.total;
    if (max_coded_bytes_host)
        *max_coded_bytes_host =
            kHeaderBytes + 4 * ((size_t)sh.pieces + 1) + (size_t)sh.pieces * (8 + 4 * (size_t)ws.maxw);
    return PILC_OK;
}

int pilc_ansai_encode(const pilc_ansai_shape *shape, const uint8_t *sym_dev, const uint8_t *dist_dev,
                      const void *tables_dev, void *workspace_dev, size_t workspace_bytes,
                      uint8_t *coded_dev, size_t coded_capacity, uint64_t *coded_bytes_host,
                      void *hip_stream)
{
    AShape sh;
    int rc = make_ashape(shape, &sh);
    if (rc != PILC_OK) return rc;
    if (!sym_dev || !dist_dev || !tables_dev || !workspace_dev || !coded_dev || !coded_bytes_host)
        return PILC_E_ARG;
    if (((uintptr_t)sym_dev & 15) || ((uintptr_t)dist_dev & 15) || ((uintptr_t)tables_dev & 255) ||
        ((uintptr_t)workspace_dev & 255) || ((uintptr_t)coded_dev & 15))
        return PILC_E_ARG;
    const AWorkspace ws = ansai_layout(sh);
    if (workspace_bytes < ws.total) return PILC_E_WORKSPACE;
    const size_t table_end = kHeaderBytes + 4 * ((size_t)sh.pieces + 1);
    if (coded_capacity < table_end) return PILC_E_CAPACITY;

    hipStream_t stream = (hipStream_t)hip_stream;
    uint8_t *base = static_cast<uint8_t *>(workspace_dev);
    Status *status = reinterpret_cast<Status *>(base + ws.status_off);
    uint32_t *piece_bits = reinterpret_cast<uint32_t *>(base + ws.bits_off);
    uint32_t *piece_state = reinterpret_cast<uint32_t *>(base + ws.state_off);
    unsigned long long *sums = reinterpret_cast<unsigned long long *>(base + ws.sums_off);
    uint32_t *scratch = reinterpret_cast<uint32_t *>(base + ws.scratch_off);
    uint32_t *offsets = reinterpret_cast<uint32_t *>(coded_dev + kHeaderBytes);
    uint32_t *payload = reinterpret_cast<uint32_t *>(coded_dev + table_end);
    const ATabLayout t = ansai_tab_layout(sh.M, sh.D, sh.X);
    const uint8_t *tb = static_cast<const uint8_t *>(tables_dev);
    const uint2 *enc_tab = reinterpret_cast<const uint2 *>(tb + t.enc_off);

    Timer timer(stream);
    k_ansai_begin<<<1, 1, 0, stream>>>(sh, reinterpret_cast<const ATabHeader *>(tb), status);
    const uint32_t blocks = (uint32_t)ceil_div64(ws.waves, kAnsaiEncWaves);
    const size_t stage_lds = (size_t)kAnsaiEncWaves * 2 * Stage<kAnsaiChunk>::kDwords * 4;
    const size_t tab_lds = 8 * (size_t)sh.D * sh.X;
    if (tab_lds <= 24576)
        k_ansai_encode<kAnsaiChunk, true><<<blocks, 64 * kAnsaiEncWaves, stage_lds + tab_lds, stream>>>(
            sh, sym_dev, dist_dev, enc_tab, scratch, ws.maxw, piece_bits, piece_state, &status->code);
    else
        k_ansai_encode<kAnsaiChunk, false><<<blocks, 64 * kAnsaiEncWaves, stage_lds, stream>>>(
            sh, sym_dev, dist_dev, enc_tab, scratch, ws.maxw, piece_bits, piece_state, &status->code);
    timer.mark("k_ansai_encode");
    const ItemBytes piece_bytes = {8u, 4u, 31u, 5u};  // state, bit count, 32-bit words
    const HeaderWords head = {{kAnsaiMagic, 1u, sh.pieces, sh.count, sh.M, sh.D, sh.X, 0u, 0u, 0u, 0u, 0u}};
    k_scan_partials<<<ws.scan_blocks, kScanThreads, 0, stream>>>(sh.pieces, piece_bytes, piece_bits, sums);
    k_scan_spine<<<1, kScanThreads, 0, stream>>>(head, sh.pieces, ws.scan_blocks, sums, coded_dev,
                                                 (unsigned long long)coded_capacity, status);
    k_scan_apply<<<ws.scan_blocks, kScanThreads, 0, stream>>>(sh.pieces, piece_bytes, piece_bits, sums,
                                                              offsets);
    timer.mark("scan");
    k_ansai_pack<<<(uint32_t)ceil_div64(ws.waves, kAnsaiPackWaves), 64 * kAnsaiPackWaves, 0, stream>>>(
        sh, scratch, ws.maxw, piece_bits, piece_state, offsets, payload, status);
    timer.mark("k_ansai_pack");
    HIP_TRY(hipGetLastError());
    Status host_status;
    HIP_TRY(hipMemcpyAsync(&host_status, status, sizeof(Status), hipMemcpyDeviceToHost, stream));
    HIP_TRY(hipStreamSynchronize(stream));
    timer.finish();
    if (host_status.code != ST_OK) return ansai_status_to_error(host_status.code);
    *coded_bytes_host = table_end + host_status.payload_bytes;
    return PILC_OK;
}

int pilc_ansai_decode(const pilc_ansai_shape *shape, const uint8_t *coded_dev, size_t coded_bytes,
                      const uint8_t *dist_dev, const void *tables_dev, void *workspace_dev,
                      size_t workspace_bytes, uint8_t *sym_out_dev, void *hip_stream)
{
    AShape sh;
    int rc = make_ashape(shape, &sh);
    if (rc != PILC_OK) return rc;
    if (!coded_dev || !dist_dev || !tables_dev || !workspace_dev || !sym_out_dev) return PILC_E_ARG;
    if (((uintptr_t)sym_out_dev & 15) || ((uintptr_t)dist_dev & 15) || ((uintptr_t)tables_dev & 255) ||
        ((uintptr_t)workspace_dev & 255) || ((uintptr_t)coded_dev & 15))
        return PILC_E_ARG;
    const AWorkspace ws = ansai_layout(sh);
    if (workspace_bytes < ws.total) return PILC_E_WORKSPACE;
    const size_t table_end = kHeaderBytes + 4 * ((size_t)sh.pieces + 1);
    if (coded_bytes < table_end) return PILC_E_FORMAT;
    const size_t lds_max = kLdsBytes;

    hipStream_t stream = (hipStream_t)hip_stream;
    Status *status = reinterpret_cast<Status *>(static_cast<uint8_t *>(workspace_dev) + ws.status_off);
    const ATabLayout t = ansai_tab_layout(sh.M, sh.D, sh.X);
    const uint8_t *tb = static_cast<const uint8_t *>(tables_dev);

    // Workgroup shape: the decode tables in LDS when they leave room for at least four
    // wavefronts' staging rows; as many wavefronts (<= 16) as then fit.
    const size_t entries = (size_t)sh.D << sh.M;
    const size_t tab_lds = ((entries + 3) / 4 + (t.wide ? entries : (entries + 1) / 2)) * 4;
    const size_t row_lds = (size_t)Stage<kAnsaiChunk>::kDwords * 4;
    bool tab_in_lds = tab_lds + 4 * row_lds <= lds_max;
    uint32_t waves = 4;
    if (tab_in_lds) {
        // small tables: several workgroups per compute unit; large ones: one big workgroup
        size_t fit = (lds_max - tab_lds) / row_lds;
        waves = tab_lds <= 16384 ? 4u : (uint32_t)(fit > 16 ? 16 : fit);
    }
    if (const char *e = getenv("PILC_ANSAI_WAVES")) {  // TEMPORARY tuning knob
        int v = atoi(e);
        if (v >= 1 && v <= 16 && (!tab_in_lds || tab_lds + v * row_lds <= lds_max)) waves = (uint32_t)v;
    }
    if (getenv("PILC_ANSAI_NOLDS")) tab_in_lds = false;
    Timer timer(stream);
    k_ansai_begin<<<1, 1, 0, stream>>>(sh, reinterpret_cast<const ATabHeader *>(tb), status);
    k_ansai_check_header<<<1, 1, 0, stream>>>(sh, coded_dev, (unsigned long long)coded_bytes, status);
    timer.mark("k_ansai_check_header");
    // A build of this kernel that needs private memory (register spills) is only ever launched
    // with four wavefronts per workgroup: with more, the wavefronts beyond the fourth of a
    // workgroup were seen to read back wrong spilled values on this machine.  The kernel as
    // written compiles without private memory, so this does not trigger.
#define PILC_ANSAI_DECODE(WIDE, LDS)                                                                  \
    do {                                                                                              \
        auto kern = k_ansai_decode<kAnsaiChunk, WIDE, LDS>;                                           \
        hipFuncAttributes fa;                                                                         \
        HIP_TRY(hipFuncGetAttributes(&fa, reinterpret_cast<const void *>(kern)));                     \
        if (fa.localSizeBytes != 0 && waves > 4) waves = 4;                                           \
        const size_t lds_bytes = (LDS ? tab_lds : 0) + waves * row_lds;                               \
        const uint32_t blocks = (uint32_t)ceil_div64(ws.waves, waves);                                \
        HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void *>(kern),                             \
                                    hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes));    \
        kern<<<blocks, 64 * waves, lds_bytes, stream>>>(sh, coded_dev, dist_dev, tb + t.theta_off,    \
                                                        tb + t.nb_off, sym_out_dev, ws.maxw, status); \
    } while (0)
    if (t.wide) {
        if (tab_in_lds)
            PILC_ANSAI_DECODE(true, true);
        else
            PILC_ANSAI_DECODE(true, false);
    } else {
        if (tab_in_lds)
            PILC_ANSAI_DECODE(false, true);
        else
            PILC_ANSAI_DECODE(false, false);
    }
#undef PILC_ANSAI_DECODE
    timer.mark("k_ansai_decode");
    HIP_TRY(hipGetLastError());
    Status host_status;
    HIP_TRY(hipMemcpyAsync(&host_status, status, sizeof(Status), hipMemcpyDeviceToHost, stream));
    HIP_TRY(hipStreamSynchronize(stream));
    timer.finish();
    return ansai_status_to_error(host_status.code);
}

}  // extern "C"
