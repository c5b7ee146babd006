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
//   enc   uint2 [D][256] + 1  { delta, phi }, index d << 8 | x; the last entry, index D << 8,
//                             is the identity step {-2^M, 0}: no bits pushed, state kept (Alg. 3)
//   theta uint8 [D << M]      symbol                               (Alg. 4)
//   nb    u16 or u32 [D << M] (N - 2^M) << 4 | (15 - B); 32-bit entries when M > 12
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
    t.theta_off = (t.enc_off + 8 * ((size_t)D * 256 + 1) + 255) & ~(size_t)255;
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
    if (d == 0 && threadIdx.x == 0) enc[gridDim.x * 256u] = make_uint2(0u - top, 0u);
    for (uint32_t x = threadIdx.x; x < X; x += blockDim.x) {
        const uint32_t p = cum[x + 1] - cum[x];
        const uint32_t k = M - (31u - __clz(p));
        enc[d * 256u + x] = make_uint2(k * top - (p << k), top - p + cum[x]);
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
            static_cast<uint32_t *>(nb_raw)[((size_t)d << M) + s] = nrel << 4 | (b ^ 15u);
        else
            static_cast<uint16_t *>(nb_raw)[((size_t)d << M) + s] = (uint16_t)(nrel << 4 | (b ^ 15u));
    }
}

// ---------------------------------------------------------------------------------------------
// Moving a wavefront's 64 rows between the arrays and LDS
// ---------------------------------------------------------------------------------------------
// A row is the `count` bytes of one piece in a [pieces, count] array.  Rows are cut at multiples
// of 128 bytes of the array ("lines"); line-stage number `ls` of a row is its ls-th line from the
// front (decode) or from the back (encode).  A wavefront fetches a line-stage of all its rows with
// 16-byte loads in which eight consecutive threads cover one row's line: thread `lane` holds, for
// i = 0..7, bytes [16c, 16c+16) of the line of row 8i + lane/8, with c = lane%8.  Every line is
// thus requested once, whole.  The threads then pass the line through LDS in two halves of 64
// bytes, where thread r finds the bytes of row r; the registers of the second half simply wait.

constexpr uint32_t kLine = 128;

struct RowLine {
    uint32_t line;    // line index in the array
    uint32_t lo, hi;  // the row's bytes inside that line: [lo, hi), empty when the row has none
};

__device__ __forceinline__ RowLine row_line(uint32_t piece, uint32_t count, uint32_t ls,
                                            bool from_back, bool row_exists)
{
    const uint32_t rb = piece * count, re = rb + count;
    const uint32_t first = rb / kLine, last = (re - 1u) / kLine;
    RowLine r;
    r.line = from_back ? last - ls : first + ls;
    if (!row_exists || ls > last - first) {
        r.lo = r.hi = 0;
        return r;
    }
    const uint32_t cb = r.line * kLine;
    r.lo = rb > cb ? rb - cb : 0u;
    r.hi = re < cb + kLine ? re - cb : kLine;
    return r;
}

__device__ __forceinline__ uint32_t line_stage_count(uint32_t count)
{
    // a row of `count` bytes starting anywhere touches at most this many lines
    return (count + 2u * kLine - 2u) / kLine;
}

// Bytes [a, b) of a dword, the others cleared (a, b may lie outside 0..4).
__device__ __forceinline__ uint32_t keep_bytes(uint32_t w, int a, int b)
{
    const uint32_t below_b = b >= 4 ? 0xFFFFFFFFu : (b <= 0 ? 0u : (1u << (8 * b)) - 1u);
    const uint32_t below_a = a >= 4 ? 0xFFFFFFFFu : (a <= 0 ? 0u : (1u << (8 * a)) - 1u);
    return w & below_b & ~below_a;
}

// Fetches line-stage `ls` of the rows of pieces p0 .. p0+np-1: for every row the 16-byte vectors
// of its line that hold at least one of its bytes (they may also hold bytes of its neighbours);
// zeros elsewhere.  A vector is aligned and holds a byte of the array, so it lies inside the
// array's last page even where it reaches past the array's end; such bytes are cleared.  The
// data is used once: the loads are marked non-temporal so that they do not push the lines this
// kernel writes out of the L2 before they are complete.
__device__ __forceinline__ void line_load(const uint8_t *__restrict__ arr, uint32_t total_bytes,
                                          uint32_t p0, uint32_t np, uint32_t count, uint32_t ls,
                                          bool from_back, uint4 (&v)[8])
{
    const uint32_t lane = threadIdx.x & 63u, vb = (lane & 7u) * 16u;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const uint32_t r = i * 8 + (lane >> 3);
        const RowLine rl = row_line(p0 + r, count, ls, from_back, r < np);
        v[i] = make_uint4(0u, 0u, 0u, 0u);
        if (vb < rl.hi && vb + 16u > rl.lo) {
            const uint32_t off = rl.line * kLine + vb;
            const u32x4 t = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(arr + off));
            v[i] = make_uint4(t.x, t.y, t.z, t.w);
            if (off + 16u > total_bytes) {  // at most one vector of the whole grid
                asm volatile("" ::: "memory");  // keep this a branch, not a chain of selects
                const int b = (int)(total_bytes - off);
                v[i] = make_uint4(keep_bytes(t.x, 0, b), keep_bytes(t.y, 0, b - 4), keep_bytes(t.z, 0, b - 8),
                                  keep_bytes(t.w, 0, b - 12));
            }
        }
    }
}

// True if some byte of w is >= limit (1 <= limit <= 255).  `k7` and `use_or` are derived from the
// limit once: k7 = ((limit <= 128 ? 128 : 256) - limit) * 0x01010101.
struct ByteLimit {
    uint32_t k7;
    bool use_or, none;  // none: limit 256, nothing to check
};

__device__ __forceinline__ ByteLimit byte_limit(uint32_t limit)
{
    ByteLimit b;
    b.none = limit >= 256u;
    b.use_or = limit <= 128u;
    b.k7 = ((b.use_or ? 128u : 256u) - (b.none ? 255u : limit)) * 0x01010101u;
    return b;
}

__device__ __forceinline__ uint32_t bytes_at_or_above(uint32_t w, const ByteLimit &b)
{
    const uint32_t t = (w & 0x7F7F7F7Fu) + b.k7;  // bit 7 of a byte: its low 7 bits reach the bound
    return (b.use_or ? (t | w) : (t & w)) & 0x80808080u;
}

// Checks the 8 vectors against a limit; a vector with an offending byte is zeroed (so that no
// table index leaves its table) and reported.
__device__ __forceinline__ uint32_t lines_check(uint4 (&v)[8], const ByteLimit &b)
{
    uint32_t bad = 0u;
    if (b.none) return 0u;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const uint32_t f = bytes_at_or_above(v[i].x, b) | bytes_at_or_above(v[i].y, b) |
                           bytes_at_or_above(v[i].z, b) | bytes_at_or_above(v[i].w, b);
        if (f) v[i] = make_uint4(0u, 0u, 0u, 0u);
        bad |= f;
    }
    return bad;
}

// ---------------------------------------------------------------------------------------------
// Encode (Alg. 3), symbols of a piece taken last-first
// ---------------------------------------------------------------------------------------------
constexpr int kAnsaiEncWaves = 4;
constexpr uint32_t kEncRow = 33;  // LDS dwords per row: 64 table indices of 16 bits, one dword pad

struct EncLane {
    uint32_t S;              // state in [2^M, 2^(M+1))
    unsigned long long acc;  // bits pushed and not yet written, low bit first
    uint32_t nacc;           // how many of them, < 32 between pairs of symbols
    uint32_t woff;           // scratch index of the next word
};

// One step of Alg. 3 with the table entry e = {delta, phi} already fetched.
__device__ __forceinline__ void ansai_push(EncLane &L, const uint2 e, uint32_t M)
{
    const uint32_t b = (e.x + L.S) >> M;  // number of bits to push, <= 15
    const uint32_t low = L.S & ((1u << b) - 1u);
    L.acc |= (unsigned long long)low << L.nacc;
    L.nacc += b;
    L.S = (L.S >> b) + e.y;
}

// Writes a word once 32 bits are there.  Called after every second symbol: two symbols add at
// most 30 bits to fewer than 32, so the accumulator never overflows.
__device__ __forceinline__ void ansai_emit(EncLane &L, uint32_t *__restrict__ scratch)
{
    if (L.nacc >= 32u) {
        scratch[L.woff] = (uint32_t)L.acc;
        L.woff += 64u;
        L.acc >>= 32;
        L.nacc -= 32u;
    }
}

// Puts half `h` of the fetched lines into LDS as table indices d << 8 | x, 16 bits per symbol;
// positions that are not part of a row get the index of the identity step, so that every thread
// can run all 64 positions of the half without asking which are its own.
__device__ __forceinline__ void enc_put(uint32_t *rows, const uint4 (&sv)[8], const uint4 (&dv)[8],
                                        uint32_t h, uint32_t p0, uint32_t np, uint32_t count,
                                        uint32_t ls, uint32_t ident)
{
    const uint32_t lane = threadIdx.x & 63u, c = lane & 7u;
    if ((c >> 2) != h) return;
    const uint32_t vb = c * 16u;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const uint32_t r = i * 8 + (lane >> 3);
        uint32_t *dst = rows + r * kEncRow + (c & 3u) * 8u;
        const RowLine rl = row_line(p0 + r, count, ls, true, r < np);
        const uint32_t s[4] = {sv[i].x, sv[i].y, sv[i].z, sv[i].w};
        const uint32_t d[4] = {dv[i].x, dv[i].y, dv[i].z, dv[i].w};
        uint32_t w[8];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            // bytes {s0, d0, s1, d1} and {s2, d2, s3, d3}
            w[2 * k] = __builtin_amdgcn_perm(d[k], s[k], 0x05010400u);
            w[2 * k + 1] = __builtin_amdgcn_perm(d[k], s[k], 0x07030602u);
        }
        if (vb < rl.lo || vb + 16u > rl.hi) {  // not wholly inside the row
            asm volatile("" ::: "memory");      // keep this a branch, not a chain of selects
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                const uint32_t pos = vb + 2u * k;
                const bool in0 = pos - rl.lo < rl.hi - rl.lo, in1 = pos + 1u - rl.lo < rl.hi - rl.lo;
                w[k] = (in0 ? (w[k] & 0xFFFFu) : ident) | (in1 ? (w[k] & 0xFFFF0000u) : ident << 16);
            }
        }
#pragma unroll
        for (int k = 0; k < 8; ++k) dst[k] = w[k];
    }
}

template <bool kTabLds>
__global__ __launch_bounds__(64 * kAnsaiEncWaves) void k_ansai_encode(
    AShape sh, const uint8_t *__restrict__ sym, const uint8_t *__restrict__ dist,
    const uint2 *__restrict__ enc_tab, uint32_t *__restrict__ scratch, uint32_t maxw,
    uint32_t *__restrict__ piece_bits, uint32_t *__restrict__ piece_state, int *status)
{
    extern __shared__ uint32_t lds[];
    if (*status != ST_OK) return;  // the tables are not the ones this shape needs
    const uint2 *tab = enc_tab;
    uint32_t *stage_base = lds;
    if (kTabLds) {
        uint2 *t = reinterpret_cast<uint2 *>(lds);
        for (uint32_t i = threadIdx.x; i < sh.D * 256u + 1u; i += blockDim.x) t[i] = enc_tab[i];
        tab = t;
        stage_base = lds + 2u * (sh.D * 256u + 1u);
        __syncthreads();
    }
    const uint32_t wave = threadIdx.x >> 6, lane = threadIdx.x & 63u;
    const uint32_t gw = blockIdx.x * kAnsaiEncWaves + wave;
    const uint32_t p0 = gw * 64u;
    if (p0 >= sh.pieces) return;
    const uint32_t np = min(64u, sh.pieces - p0);
    uint32_t *rows = stage_base + wave * 64u * kEncRow;
    const uint32_t total = sh.pieces * sh.count;
    const uint32_t *my = rows + lane * kEncRow;
    const bool mine = lane < np;
    const ByteLimit lim_x = byte_limit(sh.X), lim_d = byte_limit(sh.D);
    const uint32_t M = sh.M;

    EncLane L;
    L.S = 1u << M;
    L.acc = 0ull;
    L.nacc = 0u;
    L.woff = gw * maxw * 64u + lane;
    const uint32_t woff0 = L.woff;
    uint32_t bad = 0u;

    uint4 sv[8], dv[8];
    const uint32_t lines = line_stage_count(sh.count);
    line_load(sym, total, p0, np, sh.count, 0u, true, sv);
    line_load(dist, total, p0, np, sh.count, 0u, true, dv);
    for (uint32_t ls = 0; ls < lines; ++ls) {
        asm volatile("" : "+s"(sh.count));  // recompute the row geometry per line-stage (registers)
        bad |= lines_check(sv, lim_x) | lines_check(dv, lim_d);
#pragma unroll 1
        for (int h = 1; h >= 0; --h) {
            wave_lds_sync();
            enc_put(rows, sv, dv, (uint32_t)h, p0, np, sh.count, ls, sh.D << 8);
            wave_lds_sync();
            if (h == 0 && ls + 1u < lines) {  // the registers are free: fetch the next lines now
                line_load(sym, total, p0, np, sh.count, ls + 1u, true, sv);
                line_load(dist, total, p0, np, sh.count, ls + 1u, true, dv);
            }
#pragma unroll 1
            for (int j = 15; j >= 0; --j) {  // four symbols a turn, last first
                const uint32_t w0 = my[2 * j], w1 = my[2 * j + 1];
                const uint2 e3 = tab[w1 >> 16], e2 = tab[w1 & 0xFFFFu];
                const uint2 e1 = tab[w0 >> 16], e0 = tab[w0 & 0xFFFFu];
                ansai_push(L, e3, M);
                ansai_push(L, e2, M);
                ansai_emit(L, scratch);
                ansai_push(L, e1, M);
                ansai_push(L, e0, M);
                ansai_emit(L, scratch);
            }
        }
    }
    if (mine) {
        if (L.nacc) scratch[L.woff] = (uint32_t)L.acc;
        piece_bits[p0 + lane] = ((L.woff - woff0) >> 6) * 32u + L.nacc;
        piece_state[p0 + lane] = L.S;
    }
    if (bad) atomicMax(status, ST_ARG);  // the same value from every thread that found one
}

// ---------------------------------------------------------------------------------------------
// Pack: scratch [wavefront][word][thread] -> records {state, bit count, words} at the offsets
// ---------------------------------------------------------------------------------------------
constexpr int kAnsaiPackWaves = 4;
constexpr int kAnsaiPackRows = 64;

__global__ __launch_bounds__(64 * kAnsaiPackWaves) void k_ansai_pack(
    AShape sh, const uint32_t *__restrict__ scratch, uint32_t maxw,
    const uint32_t *__restrict__ piece_bits, const uint32_t *__restrict__ piece_state,
    const uint32_t *__restrict__ offsets, uint32_t *__restrict__ payload,
    const Status *__restrict__ status)
{
    if (status->code != ST_OK) return;
    static_assert(kAnsaiPackRows == 64, "a pass writes 64 words of one piece, one per thread");
    __shared__ uint32_t tile[kAnsaiPackWaves][64 * (kAnsaiPackRows + 1)];
    const uint32_t wave = threadIdx.x >> 6, lane = threadIdx.x & 63u;
    const uint32_t gw = blockIdx.x * kAnsaiPackWaves + wave;
    const uint32_t p0 = gw * 64u;
    if (p0 >= sh.pieces) return;
    const uint32_t np = min(64u, sh.pieces - p0);
    uint32_t nw = 0, dst = 0;  // words of this thread's piece and the payload dword index of the first
    if (lane < np) {
        const uint32_t bits = piece_bits[p0 + lane], at = offsets[p0 + lane] >> 2;
        nw = (bits + 31u) >> 5;
        payload[at] = piece_state[p0 + lane];
        payload[at + 1u] = bits;
        dst = at + 2u;
    }
    uint32_t most = nw;
    for (int d = 32; d >= 1; d >>= 1) most = max(most, (uint32_t)__shfl_xor((int)most, d, 64));
    const uint32_t *src = scratch + (size_t)gw * maxw * 64u + lane;
    uint32_t *mine = tile[wave] + lane * (kAnsaiPackRows + 1);
    // A turn moves kAnsaiPackRows words of every piece.  All rows of a turn are asked for before the
    // first is stored (guarded one by one, every load would wait for the one before; rows past the
    // last one repeat it and are never read), and the next turn's rows are asked for before this
    // turn's words are written out, so that they arrive meanwhile.
    uint32_t v[kAnsaiPackRows];
    auto fetch = [&](uint32_t j0) {
#pragma unroll
        for (int jj = 0; jj < kAnsaiPackRows; ++jj) v[jj] = src[(size_t)min(j0 + jj, most - 1u) * 64u];
    };
    if (most != 0u) fetch(0u);
    for (uint32_t j0 = 0; j0 < most; j0 += kAnsaiPackRows) {
        wave_lds_sync();
#pragma unroll
        for (int jj = 0; jj < kAnsaiPackRows; ++jj) mine[jj] = v[jj];
        wave_lds_sync();
        if (j0 + kAnsaiPackRows < most) fetch(j0 + kAnsaiPackRows);
        // pass i writes words j0 .. j0 + 63 of piece i, a word per thread; the piece's length and
        // place come from its thread's registers, and eight tile reads are under way at a time
        const uint32_t j = j0 + lane;
#pragma unroll
        for (int i0 = 0; i0 < 64; i0 += 8) {
            uint32_t word[8];
#pragma unroll
            for (int k = 0; k < 8; ++k) word[k] = tile[wave][(i0 + k) * (kAnsaiPackRows + 1) + lane];
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                const uint32_t nw_i = (uint32_t)__builtin_amdgcn_readlane((int)nw, i0 + k);
                const uint32_t dst_i = (uint32_t)__builtin_amdgcn_readlane((int)dst, i0 + k);
                if (j < nw_i) payload[dst_i + j] = word[k];
            }
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
    status->ticket = 0;
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

// A thread's view of its piece's stream.  The words still to be taken sit in the payload below
// `widx`; the next ones are kept ahead of use in a small per-thread ring in LDS, which is topped
// up with aligned 16-byte loads issued a group of symbols before their data is needed, so no
// step of the decoding chain ever waits for global memory.
// LDS is what limits how many pieces a compute unit decodes at once (the tables take most of
// it), so both per-thread areas are kept small: a ring of three quads and a row of 32 bytes.
constexpr uint32_t kRingWords = 12;   // per thread: three aligned quads
constexpr uint32_t kRingStride = 13;  // odd: threads reading their own rings hit distinct banks
constexpr int kGroupSyms = 8;         // symbols between top-ups; they take at most 4 words (M <= 15)
constexpr uint32_t kPart = 32;        // bytes of a row passed through LDS at a time: a quarter line
constexpr uint32_t kDecRow = 10;      // LDS dwords per row: 32 bytes and a pad that keeps rows 8-byte aligned

struct DecLane {
    uint32_t s;              // state minus 2^M
    unsigned long long win;  // the next n bits of the stream from bit 62 downwards; bit 63 is 0
    int n;                   // <= 63; negative once a corrupt stream has run dry
    uint32_t widx;           // dword index (from the container's start) one past the next word
    uint32_t lp;             // the ring holds the words [lp, widx); a multiple of 4
    uint32_t first;          // dword index of the piece's first word; widx - first words are left
    uint32_t rs;             // ring slot of word widx-1; slots fall with the word index, 0 wraps to 11
    uint32_t ws;             // ring slot of word lp: 0, 4 or 8
    uint32_t cand;           // word widx-1, read ahead from the ring
};

// An aligned quad that holds at least one word of the container: it lies inside the container's
// last page even where it reaches past the container's end.
__device__ __forceinline__ uint4 ansai_quad_load(const uint32_t *__restrict__ cw, uint32_t q)
{
    return *reinterpret_cast<const uint4 *>(cw + q);
}

__device__ __forceinline__ void ansai_ring_put(uint32_t *ring, uint32_t slot, const uint4 &v)
{
    ring[slot] = v.x;
    ring[slot + 1u] = v.y;
    ring[slot + 2u] = v.z;
    ring[slot + 3u] = v.w;
}

// Takes the next word into the window when fewer than 32 bits are left in it.  Written without
// a branch: in a wavefront of 64 streams some thread needs a word at almost every call.
__device__ __forceinline__ void ansai_refill(DecLane &L)
{
    const bool need = L.n < 32 && L.widx > L.first;
    const uint32_t c = need ? L.cand : 0u;
    L.win |= (unsigned long long)c << ((31 - L.n) & 63);  // need implies 0 <= n <= 31
    const uint32_t t = need ? 1u : 0u;
    L.n += (int)(t << 5);
    L.widx -= t;
    const uint32_t below = L.rs == 0u ? kRingWords - 1u : L.rs - 1u;
    L.rs = need ? below : L.rs;
}

__device__ __forceinline__ void ansai_peek(DecLane &L, const uint32_t *ring)
{
    L.cand = ring[L.rs];
}

// One step of Alg. 4.  `dm` = d << M.  The table entry holds N[d,S] - 2^M above its low four
// bits and 15 - B[d,S] in them, so that 31 - B, the shift that leaves the B popped bits (kept in
// the order they were pushed) at the bottom of the window's upper word, is the low five bits of
// (entry | 16).  A stream that has run dry yields zeros here; the count n then ends below zero and
// the piece fails its final check.  With `active` false the step is the identity (no symbol of
// this thread's row at this position).
template <bool kWide, bool kMasked>
__device__ __forceinline__ uint32_t ansai_pop(DecLane &L, uint32_t dm, bool active, const uint8_t *theta,
                                              const void *nb_raw)
{
    const uint32_t ti = dm + L.s;
    uint32_t e = kWide ? static_cast<const uint32_t *>(nb_raw)[ti]
                       : (uint32_t) static_cast<const uint16_t *>(nb_raw)[ti];
    const uint32_t x = theta[ti];
    if (kMasked) e = active ? e : (L.s << 4 | 15u);  // pops nothing, keeps the state
    const uint32_t v = (uint32_t)(L.win >> 32) >> ((e | 16u) & 31u);
    L.s = (e >> 4) + v;  // S <- N[d,S] + popped bits
    const uint32_t b = ~e & 15u;
    L.win = (L.win << b) & 0x7FFFFFFFFFFFFFFFull;
    L.n -= (int)b;
    return x;
}

// The part of [lo, hi) that falls into quarter `ph` of the line, relative to that quarter.
__device__ __forceinline__ void part_range(const RowLine &r, uint32_t ph, uint32_t *lo, uint32_t *hi)
{
    const uint32_t base = ph * kPart;
    *lo = min(max(r.lo, base), base + kPart) - base;
    *hi = min(max(r.hi, base), base + kPart) - base;
}

// Puts quarter `ph` of the fetched index lines into LDS, 32 bytes per row.
__device__ __forceinline__ void dec_put(uint32_t *rows, const uint4 (&dv)[8], uint32_t ph)
{
    const uint32_t lane = threadIdx.x & 63u, c = lane & 7u;
    if ((c >> 1) != ph) return;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        uint2 *dst = reinterpret_cast<uint2 *>(rows + (i * 8 + (lane >> 3)) * kDecRow + (c & 1u) * 4u);
        dst[0] = make_uint2(dv[i].x, dv[i].y);
        dst[1] = make_uint2(dv[i].z, dv[i].w);
    }
}

// Writes the decoded symbols of quarter `ph` of line-stage `ls` from LDS to the output rows:
// only bytes that belong to a row.  Two threads cover a row's 32 bytes.
__device__ __forceinline__ void dec_store(uint8_t *__restrict__ out, const uint32_t *rows, uint32_t p0,
                                          uint32_t np, uint32_t count, uint32_t ls, uint32_t ph)
{
    const uint32_t lane = threadIdx.x & 63u;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const uint32_t r = i * 32 + (lane >> 1), c = lane & 1u;
        const RowLine rl = row_line(p0 + r, count, ls, false, r < np);
        uint32_t lo, hi;
        part_range(rl, ph, &lo, &hi);
        const uint32_t vb = c * 16u;
        if (hi > lo && vb < hi && vb + 16u > lo) {
            const uint32_t *src = rows + r * kDecRow + c * 4u;
            const uint32_t off = rl.line * kLine + ph * kPart + vb;
            if (lo <= vb && vb + 16u <= hi) {
                *reinterpret_cast<uint4 *>(out + off) = make_uint4(src[0], src[1], src[2], src[3]);
            } else {
                for (uint32_t k = 0; k < 16u; ++k)
                    if (vb + k >= lo && vb + k < hi) out[off + k] = (uint8_t)(src[k >> 2] >> (8u * (k & 3u)));
            }
        }
    }
}

// The 32 symbols of one quarter line of this thread's row, in groups of eight.  Before a group
// the quad below the ring is requested when there is room for it (it lies below the quads fetched
// at the start, hence inside the container) and after the group it is stored, so its latency
// hides behind eight symbols of every wavefront on the SIMD.  A group takes at most four words
// and starts with at least four in the ring: with room for a quad (at most 8 words held) the quad
// arrives by the end of the group, without room at least 9 - 4 are left.
// kMasked: positions outside [lo, hi) are skipped by identity steps.
template <bool kWide, bool kMasked>
__device__ __forceinline__ void dec_part(DecLane &L, uint32_t *my, uint32_t *ring,
                                         const uint32_t *__restrict__ cw, uint32_t M, uint32_t lo,
                                         uint32_t hi, const uint8_t *theta, const void *nb)
{
#pragma unroll 1
    for (int g = 0; g < (int)kPart / kGroupSyms; ++g) {
        const uint32_t qb = L.lp - 4u;
        const bool want = L.widx - L.lp <= kRingWords - 4u && L.lp > L.first;
        uint4 q;
        if (want) q = ansai_quad_load(cw, qb);
        ansai_peek(L, ring);
#pragma unroll 1
        for (int hh = 0; hh < kGroupSyms / 4; ++hh) {
            const int dw = g * (kGroupSyms / 4) + hh;
            const uint32_t d4 = my[dw];
            uint32_t x4 = 0u;
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                if ((k & 1) == 0) {
                    ansai_refill(L);
                    ansai_peek(L, ring);
                }
                const uint32_t dm = ((d4 >> (8 * k)) & 255u) << M;
                const bool active = !kMasked || (uint32_t)(dw * 4 + k) - lo < hi - lo;
                x4 |= ansai_pop<kWide, kMasked>(L, dm, active, theta, nb) << (8 * k);
            }
            my[dw] = x4;
        }
        if (want) {
            L.ws = L.ws == 0u ? kRingWords - 4u : L.ws - 4u;
            ansai_ring_put(ring, L.ws, q);
            L.lp = qb;
        }
    }
}

constexpr int kAnsaiDecMaxWaves = 12;

template <bool kWide, bool kTabLds>
__global__ __launch_bounds__(64 * kAnsaiDecMaxWaves) void k_ansai_decode(
    AShape sh, const uint8_t *__restrict__ coded, const uint8_t *__restrict__ dist, const uint8_t *__restrict__ theta_g,
    const void *__restrict__ nb_g, uint8_t *__restrict__ out, uint32_t maxw, Status *status)
{
    extern __shared__ uint32_t lds[];
    if (status->code != ST_OK) return;
    const uint8_t *theta = theta_g;
    const void *nb = nb_g;
    uint32_t *stage_base = lds;
    if (kTabLds) {  // the chain's table first, so that its LDS address is the index times its size
        const uint32_t entries = sh.D << sh.M;
        const uint32_t th_dw = (entries + 3u) >> 2, nb_dw = kWide ? entries : (entries + 1u) >> 1;
        const uint32_t *tg = reinterpret_cast<const uint32_t *>(theta_g);
        const uint32_t *ng = reinterpret_cast<const uint32_t *>(nb_g);
        for (uint32_t i = threadIdx.x; i < nb_dw; i += blockDim.x) lds[i] = ng[i];
        for (uint32_t i = threadIdx.x; i < th_dw; i += blockDim.x) lds[nb_dw + i] = tg[i];
        nb = lds;
        theta = reinterpret_cast<const uint8_t *>(lds + nb_dw);
        stage_base = lds + nb_dw + th_dw;
        __syncthreads();
    }
    const uint32_t waves = blockDim.x >> 6;
    const uint32_t wave = threadIdx.x >> 6, lane = threadIdx.x & 63u;
    const uint32_t gw = blockIdx.x * waves + wave;
    const uint32_t p0 = gw * 64u;
    if (p0 >= sh.pieces) return;
    const uint32_t np = min(64u, sh.pieces - p0);
    uint32_t *rows = stage_base + wave * 64u * (kDecRow + kRingStride);
    uint32_t *ring = rows + 64u * kDecRow + lane * kRingStride;
    uint32_t *my = rows + lane * kDecRow;
    const uint32_t total = sh.pieces * sh.count;
    const uint32_t top = 1u << sh.M, M = sh.M;
    const uint32_t *cw = reinterpret_cast<const uint32_t *>(coded);
    const uint32_t off_dw = kHeaderBytes / 4u, pay_dw = off_dw + sh.pieces + 1u;
    const uint32_t payload_bytes = (uint32_t)status->payload_bytes;
    const ByteLimit lim_d = byte_limit(sh.D);

    bool mine = lane < np;
    uint32_t corrupt = 0u, bad = 0u;
    DecLane L;
    L.s = 0u;
    L.win = 0ull;
    L.n = 0;
    L.widx = pay_dw + 4u;
    L.lp = L.widx & ~3u;
    L.first = L.widx;
    L.rs = 0u;
    L.ws = 0u;
    L.cand = 0u;
    if (mine) {
        const uint32_t begin = cw[off_dw + p0 + lane], end = cw[off_dw + p0 + lane + 1u];
        bool ok = end >= begin && end - begin >= 8u && end <= payload_bytes && ((begin | end) & 3u) == 0u;
        if (ok) {
            const uint32_t rec = pay_dw + (begin >> 2);
            const uint32_t state = cw[rec], bits = cw[rec + 1u];
            const uint32_t nw = (end - begin - 8u) >> 2;
            // no piece of `count` symbols holds more than maxw words
            ok = nw <= maxw && state >= top && state < 2u * top && bits <= 32u * nw && bits + 31u >= 32u * nw;
            if (ok) {
                L.s = state - top;
                L.first = rec + 2u;
                L.widx = L.first + nw;
                if (nw > 0u) {  // the last word holds the top 1..32 bits
                    const uint32_t r = bits - 32u * (nw - 1u);
                    L.widx -= 1u;
                    L.win = (unsigned long long)(cw[L.widx] & (0xFFFFFFFFu >> (32u - r))) << (63u - r);
                    L.n = (int)r;
                }
                // fill the ring with the 12 words that end at the aligned quad holding word widx-1
                L.lp = (L.widx + 3u) & ~3u;
                if (L.widx > L.first) {
                    L.rs = 8u + ((L.widx - 1u) & 3u);
#pragma unroll
                    for (int i = 2; i >= 0; --i) {
                        L.lp -= 4u;
                        ansai_ring_put(ring, 4u * i, ansai_quad_load(cw, L.lp));
                    }
                }
            }
        }
        if (!ok) {
            corrupt = 1u;
            mine = false;
        }
    }

    uint4 dv[8];
    const uint32_t lines = line_stage_count(sh.count);
    line_load(dist, total, p0, np, sh.count, 0u, false, dv);
    for (uint32_t ls = 0; ls < lines; ++ls) {
        // the row geometry is recomputed per line-stage instead of being kept in registers for
        // all the rows a thread helps to move: that keeps the kernel free of register spills
        asm volatile("" : "+s"(sh.count));
        const RowLine rl = row_line(p0 + lane, sh.count, ls, false, mine);
        bad |= lines_check(dv, lim_d);
#pragma unroll 1
        for (uint32_t h = 0; h < kLine / kPart; ++h) {
            wave_lds_sync();
            dec_put(rows, dv, h);
            wave_lds_sync();
            if (h == kLine / kPart - 1u && ls + 1u < lines)
                line_load(dist, total, p0, np, sh.count, ls + 1u, false, dv);
            uint32_t lo, hi;
            part_range(rl, h, &lo, &hi);
            if (__all(lo == 0u && hi == kPart))
                dec_part<kWide, false>(L, my, ring, cw, M, lo, hi, theta, nb);
            else
                dec_part<kWide, true>(L, my, ring, cw, M, lo, hi, theta, nb);
            wave_lds_sync();
            dec_store(out, rows, p0, np, sh.count, ls, h);
        }
    }
    if (mine && (L.s != 0u || L.n != 0 || L.widx != L.first)) corrupt = 1u;
    // many threads may report: the larger code (a damaged container) wins, whatever the order
    if (corrupt)
        atomicMax(&status->code, ST_CORRUPT);
    else if (bad)
        atomicMax(&status->code, ST_ARG);
}

// ---------------------------------------------------------------------------------------------
// Re-centring (Sec. 3.3): code (r - mu + 128) mod 256 so that the distribution index only has to
// tell the scale.  Four bytes per 32-bit lane operation: byte-wise subtraction / addition without
// carries between bytes, and + 128 mod 256 is a flip of every byte's top bit.
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ uint32_t bytes_sub(uint32_t a, uint32_t b)
{
    return ((a | 0x80808080u) - (b & 0x7F7F7F7Fu)) ^ ((a ^ ~b) & 0x80808080u);
}

__device__ __forceinline__ uint32_t bytes_add(uint32_t a, uint32_t b)
{
    return ((a & 0x7F7F7F7Fu) + (b & 0x7F7F7F7Fu)) ^ ((a ^ b) & 0x80808080u);
}

template <bool kInverse>
__global__ __launch_bounds__(256) void k_ansai_center(const uint8_t *in, const uint8_t *__restrict__ mu,
                                                      unsigned long long n, uint8_t *out)  // out may be in
{
    const unsigned long long vecs = n / 16ull, stride = (unsigned long long)gridDim.x * blockDim.x;
    for (unsigned long long i = (unsigned long long)blockIdx.x * blockDim.x + threadIdx.x; i < vecs; i += stride) {
        const uint4 a = reinterpret_cast<const uint4 *>(in)[i], m = reinterpret_cast<const uint4 *>(mu)[i];
        uint4 r;
        if (kInverse) {
            r = make_uint4(bytes_add(a.x ^ 0x80808080u, m.x), bytes_add(a.y ^ 0x80808080u, m.y),
                           bytes_add(a.z ^ 0x80808080u, m.z), bytes_add(a.w ^ 0x80808080u, m.w));
        } else {
            r = make_uint4(bytes_sub(a.x, m.x) ^ 0x80808080u, bytes_sub(a.y, m.y) ^ 0x80808080u,
                           bytes_sub(a.z, m.z) ^ 0x80808080u, bytes_sub(a.w, m.w) ^ 0x80808080u);
        }
        reinterpret_cast<uint4 *>(out)[i] = r;
    }
    if (blockIdx.x == 0 && threadIdx.x < (n & 15ull)) {  // the last, partial vector
        const unsigned long long i = vecs * 16ull + threadIdx.x;
        out[i] = kInverse ? (uint8_t)(in[i] + mu[i] - 128u) : (uint8_t)(in[i] - mu[i] + 128u);
    }
}

// ---------------------------------------------------------------------------------------------
// Host side
// ---------------------------------------------------------------------------------------------
static int make_ashape(const pilc_ansai_shape *in, AShape *sh)
{
    if (!in || in->pieces == 0 || in->count == 0) return PILC_E_ARG;
    if (in->prec_bits < 1 || in->prec_bits > 15 || in->num_dist < 1 || in->num_dist > 255 ||
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

int pilc_ansai_center(const uint8_t *in_dev, const uint8_t *mu_dev, uint64_t count, int inverse,
                      uint8_t *out_dev, void *hip_stream)
{
    if (!in_dev || !mu_dev || !out_dev || count == 0) return PILC_E_ARG;
    if (((uintptr_t)in_dev & 15) || ((uintptr_t)mu_dev & 15) || ((uintptr_t)out_dev & 15)) return PILC_E_ARG;
    hipStream_t stream = (hipStream_t)hip_stream;
    const uint64_t vecs = count / 16;
    uint32_t blocks = (uint32_t)(vecs / 256 > 16384 ? 16384 : (vecs + 255) / 256);
    if (blocks == 0) blocks = 1;
    if (inverse)
        k_ansai_center<true><<<blocks, 256, 0, stream>>>(in_dev, mu_dev, count, out_dev);
    else
        k_ansai_center<false><<<blocks, 256, 0, stream>>>(in_dev, mu_dev, count, out_dev);
    HIP_TRY(hipGetLastError());
    HIP_TRY(hipStreamSynchronize(stream));
    return PILC_OK;
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
    const size_t stage_lds = (size_t)kAnsaiEncWaves * 64 * kEncRow * 4;
    const size_t tab_lds = 8 * ((size_t)sh.D * 256 + 1);
    if (tab_lds <= 24576 + 8)
        k_ansai_encode<true><<<blocks, 64 * kAnsaiEncWaves, stage_lds + tab_lds, stream>>>(
            sh, sym_dev, dist_dev, enc_tab, scratch, ws.maxw, piece_bits, piece_state, &status->code);
    else
        k_ansai_encode<false><<<blocks, 64 * kAnsaiEncWaves, stage_lds, stream>>>(
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

int pilc_set_ansai_decode_waves(int waves)
{
    if (waves < 0 || waves > kAnsaiDecMaxWaves) return PILC_E_ARG;
    g_ansai_decode_waves.store(waves, std::memory_order_relaxed);
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
    // wavefronts' staging rows; as many wavefronts (<= kAnsaiDecMaxWaves) as then fit.
    const size_t entries = (size_t)sh.D << sh.M;
    const size_t tab_lds = ((entries + 3) / 4 + (t.wide ? entries : (entries + 1) / 2)) * 4;
    const size_t row_lds = (size_t)64 * (kDecRow + kRingStride) * 4;
    bool tab_in_lds = tab_lds + 4 * row_lds <= lds_max;
    uint32_t waves = 4;
    if (tab_in_lds) {
        // small tables: several workgroups per compute unit; large ones: one big workgroup
        size_t fit = (lds_max - tab_lds) / row_lds;
        waves = tab_lds <= 16384 ? 4u : (uint32_t)(fit > kAnsaiDecMaxWaves ? kAnsaiDecMaxWaves : fit);
        // a batch too small to fill every compute unit that densely is spread over all of them
        // (a piece is a serial chain: its pace falls with the wavefronts that share its SIMD)
        int dev = 0, cus = 0;
        if (waves > 4u && hipGetDevice(&dev) == hipSuccess &&
            hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && cus > 0) {
            const uint32_t each = (uint32_t)ceil_div64(ws.waves, (uint64_t)cus);
            waves = each < 4u ? 4u : (each < waves ? each : waves);
        }
    }
    const uint32_t asked = (uint32_t)g_ansai_decode_waves.load(std::memory_order_relaxed);
    if (asked != 0u) {  // pilc_set_ansai_decode_waves: that many, if they fit
        const size_t fit = tab_in_lds ? (lds_max - tab_lds) / row_lds : (size_t)kAnsaiDecMaxWaves;
        waves = asked < fit ? asked : (uint32_t)fit;
    }
    Timer timer(stream);
    k_ansai_begin<<<1, 1, 0, stream>>>(sh, reinterpret_cast<const ATabHeader *>(tb), status);
    k_ansai_check_header<<<1, 1, 0, stream>>>(sh, coded_dev, (unsigned long long)coded_bytes, status);
    timer.mark("k_ansai_check_header");
    // A build of this kernel that needed private memory (register spills) once decoded wrongly in
    // the wavefronts beyond the fourth of a workgroup, and the cause was never found.  The kernel as
    // written compiles without private memory; a build that does not is refused rather than run.
#define PILC_ANSAI_DECODE(WIDE, LDS)                                                                  \
    do {                                                                                              \
        auto kern = k_ansai_decode<WIDE, LDS>;                                                        \
        hipFuncAttributes fa;                                                                         \
        HIP_TRY(hipFuncGetAttributes(&fa, reinterpret_cast<const void *>(kern)));                     \
        if (fa.localSizeBytes != 0) {                                                                 \
            snprintf(t_hip_error, sizeof(t_hip_error),                                                \
                     "k_ansai_decode was built with %zu bytes of private memory per thread; this "   \
                     "library only runs a build of it that has none", (size_t)fa.localSizeBytes);     \
            return PILC_E_HIP;                                                                        \
        }                                                                                             \
        const size_t lds_bytes = (LDS ? tab_lds : 0) + waves * row_lds;                               \
        const uint32_t blocks = (uint32_t)ceil_div64(ws.waves, waves);                                \
        if ((rc = allow_large_lds(reinterpret_cast<const void *>(kern))) != PILC_OK) return rc;       \
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
