/*
 * pilc.h -- C ABI of libpilc: the entropy-coding stage of PILC (arXiv 2206.05279)
 * for AMD MI355X (gfx950).
 *
 * The stage turns uint8 subpixels plus per-subpixel distribution parameters into a
 * bitstream and back (Sec. 3.1 "Compress"/"Decompress": the coder receives the symbols
 * and the predicted logistic parameters; the decoder regenerates the same parameters and
 * recovers the symbols losslessly).
 *
 * Conventions for every entry point
 *   - All `*_dev` pointers and the pointers inside pilc_params are DEVICE memory owned by
 *     the caller; pilc_geom, pilc_params and `*_host` pointers are HOST memory.
 *   - The library never allocates or frees device memory on behalf of a call: images,
 *     parameters, workspace and output are caller-owned.  (Three small constant tables
 *     live in the library's own device globals and are filled on first use per device.)
 *   - Work is enqueued on `hip_stream` (a hipStream_t passed as void*, NULL = default
 *     stream).  Every call synchronises that stream before it returns, so the status and
 *     all outputs are final on return.
 *   - Return value: 0 on success, a negative PILC_E_* code otherwise.  No exceptions.  Calls on
 *     different streams may run concurrently, from any threads, if they use different workspaces.
 *     The library's only process-wide state: the constant tables (filled once per device under a
 *     lock), the knobs pilc_set_timing, pilc_set_kernel_policy, pilc_set_one_pass_wait and
 *     pilc_set_ansai_decode_waves (atomic integers, read once at the start of a call), the scratch array of pilc_encode_static, and four
 *     sets of progress counters that calls of pilc_twar_inverse on tall images take turns with.
 *   - Tensors are dense, row-major, channel-interleaved: index ((i*h + y)*w + x)*3 + c.
 */
#ifndef PILC_H
#define PILC_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define PILC_VERSION 1u

enum {
    PILC_OK = 0,
    PILC_E_ARG = -1,       /* null / misaligned pointer, bad geometry                      */
    PILC_E_WORKSPACE = -2, /* workspace smaller than pilc_workspace_size reports            */
    PILC_E_CAPACITY = -3,  /* coded output does not fit coded_capacity (nothing usable out) */
    PILC_E_TOO_LARGE = -4, /* payload would reach 4 GiB (32-bit lane offsets)               */
    PILC_E_FORMAT = -5,    /* decode: bad magic / version / geometry mismatch / size        */
    PILC_E_CORRUPT = -6,   /* decode: offsets not monotone or out of bounds, a lane runs
                              past its end, or does not return to its initial state         */
    PILC_E_HIP = -7,       /* HIP runtime failure (see pilc_last_hip_error)                 */
    PILC_E_TIMEOUT = -8    /* a bounded wait between workgroups or wavefronts ran out (see
                              pilc_set_one_pass_wait); outputs undefined                    */
};

/* Geometry of a batch.  M = prec_bits is the constant of Sec. 3.2 for which every
 * symbol's integer masses sum to 2^M (the paper uses 10..15 for 8-bit data; 16 is also
 * accepted here).  A "lane" is one independent rANS stream:
 *   lane_mode 0: lane j codes the flat pixel range [j*lane_a, min((j+1)*lane_a, n*h*w));
 *                lane_a must divide h*w or be a multiple of it.
 *   lane_mode 1: lane j codes one tile of lane_a rows x lane_b columns; tiles are numbered
 *                row-major inside an image, images in order; edge tiles are clipped.
 * Inside a lane the decode order is raster order of its pixels, R,G,B inside a pixel. */
typedef struct {
    uint32_t n, h, w;   /* images, rows, columns; 3 interleaved channels */
    uint32_t prec_bits; /* M, 10..16 */
    uint32_t lane_mode; /* 0 or 1 */
    uint32_t lane_a, lane_b;
} pilc_geom;

/* Per-subpixel logistic parameters (Sec. 3.1 eq. (7), Sec. 3.3) in fixed point, plus the
 * per-image coefficients that condition G on R and B on R,G of the same pixel (Sec. 3.1
 * eqs. (3)-(4), applied as  mu'_G = mu_G + a_GR*(x_R-mu_R),
 * mu'_B = mu_B + a_BR*(x_R-mu_R) + a_BG*(x_G-mu_G), each product rounded to Q8.8). */
typedef struct {
    const uint16_t *mu;        /* device [n,h,w,3]  Q8.8 unsigned                          */
    const int16_t *log_scale;  /* device [n,h,w,3]  Q4.12, natural log of the scale;
                                  values outside [-4, 6) act as the nearest bound         */
    const int16_t *chan_coef;  /* device [n,3]      Q2.14: a_GR, a_BR, a_BG                */
} pilc_params;

/* Number of lanes of a geometry (Sec. 3.2's independent coder instances, "one thread per
 * piece" in Sec. 4.3); 0 if the geometry is invalid. */
uint64_t pilc_lane_count(const pilc_geom *geom);

/* Sizes a caller must provide: bytes of device workspace for encode and decode of this
 * geometry, and an upper bound of the container size (64-byte header + 4*(lanes+1) offset
 * table + per lane 4 bytes of state + at most one 16-bit word per symbol).
 * Errors: PILC_E_ARG. */
int pilc_workspace_size(const pilc_geom *geom, size_t *workspace_bytes_host,
                        size_t *max_coded_bytes_host);

/* Compress (Sec. 3.1 "Compress", coder part; Sec. 3.2 tables; App. A eq. (11) per symbol).
 *   img_dev        uint8 [n,h,w,3]
 *   params         see pilc_params
 *   workspace_dev  >= workspace_bytes from pilc_workspace_size, 256-byte aligned; contents
 *                  are scratch, undefined afterwards
 *   coded_dev      output container, 16-byte aligned, capacity coded_capacity bytes
 *   coded_bytes_host  receives the container size
 * Container (little endian): 64-byte header {"PILC", version, n, h, w, 3, M, lane_mode,
 * lane_a, lane_b, lanes, 0, payload_bytes u64, 0 u64}; u32 offsets[lanes+1] (exclusive
 * prefix sum of lane byte counts, relative to the payload); payload = for each lane its
 * final 32-bit state followed by its 16-bit words in the order the decoder reads them.
 * Errors: PILC_E_ARG, PILC_E_WORKSPACE, PILC_E_CAPACITY (coded_dev contents undefined),
 * PILC_E_TOO_LARGE, PILC_E_HIP, PILC_E_TIMEOUT. */
int pilc_encode(const pilc_geom *geom, const uint8_t *img_dev, const pilc_params *params,
                void *workspace_dev, size_t workspace_bytes, uint8_t *coded_dev,
                size_t coded_capacity, uint64_t *coded_bytes_host, void *hip_stream);

/* pilc_encode for callers that cannot allocate device memory or carry a workspace: code under
 * HIP graph capture set-up, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments, container, alignment rules and errors as pilc_encode, without the workspace: the
 * scratch memory is an array of PILC_STATIC_SCRATCH_BYTES inside the library (one copy per GPU,
 * held until the process ends), and the call allocates and frees nothing (no HIP events either:
 * pilc_last_timing reports nothing for it).  A geometry whose pilc_workspace_size exceeds
 * PILC_STATIC_SCRATCH_BYTES is refused with PILC_E_WORKSPACE before anything runs (16 MiB holds
 * one 1920x1080 frame, or about 2.7 million pixels in all).  All calls on one GPU share that
 * GPU's array: calls that overlap in time on the same GPU, from any threads or streams, race and
 * give undefined output; calls one after another are independent (nothing is kept between them). */
#define PILC_STATIC_SCRATCH_BYTES (16u << 20)
int pilc_encode_static(const pilc_geom *geom, const uint8_t *img_dev, const pilc_params *params,
                       uint8_t *coded_dev, size_t coded_capacity, uint64_t *coded_bytes_host,
                       void *hip_stream);

/* Decompress (Sec. 3.1 "Decompress", coder part; App. A eq. (12) per symbol, the symbol
 * being the x with C_x <= S mod 2^M < C_x + P_x).  The geometry and parameters must be the
 * ones used to encode.  img_out_dev uint8 [n,h,w,3]; on error its contents are undefined.
 * coded_dev is 16-byte aligned; the decoder reads the stream in aligned 16-byte blocks and may
 * therefore read (never use) up to 15 bytes beyond coded_bytes, inside the block that holds the
 * container's last byte.
 * Errors: PILC_E_ARG, PILC_E_WORKSPACE, PILC_E_FORMAT, PILC_E_CORRUPT, PILC_E_HIP. */
int pilc_decode(const pilc_geom *geom, const uint8_t *coded_dev, size_t coded_bytes,
                const pilc_params *params, void *workspace_dev, size_t workspace_bytes,
                uint8_t *img_out_dev, void *hip_stream);

/* The integer tables of Sec. 3.2 for the symbols actually present: for every subpixel (image
 * layout [n,h,w,3]) its cumulative count C_x and mass P_x (sum_x P_x = 2^M, P_x >= 1).
 * cum_out_dev, freq_out_dev: device uint32 [n,h,w,3].  A verification entry point: encode
 * computes the same values on the fly and never materialises them.
 * Errors: PILC_E_ARG, PILC_E_HIP. */
int pilc_symbol_tables(const pilc_geom *geom, const uint8_t *img_dev, const pilc_params *params,
                       uint32_t *cum_out_dev, uint32_t *freq_out_dev, void *hip_stream);

/* ---- mixture of K logistic laws per subpixel ------------------------------------------
 * The workload Sec. 2 ("Entropy Coder") and the "Data transfer" item of Sec. 1 name as the
 * slow case of earlier learned codecs: a dynamic rANS coder (App. A eqs. (11)-(12)) whose
 * distribution per symbol is a mixture of ten logistic laws.  The paper gives no formula; this
 * library takes: a pixel carries K weights w_j in Q0.15 that sum to 2^15 exactly (shared by its
 * three subpixels), a subpixel K means and K log-scales (formats of pilc_params); the mixed
 * 24-bit edge CDF is F(k) = floor(sum_j w_j F_j(k) / 2^15), F_j the single-law edge CDF, and
 * C(k) = k + floor(F(k) (2^M - 256) / 2^24), so K = 1 is the single law of pilc_encode; G and B
 * are conditioned as in pilc_params, every component's mean shifted with that component's own
 * innovations. */
typedef struct {
    const uint16_t *mu;        /* device [n,h,w,3,K] Q8.8                                  */
    const int16_t *log_scale;  /* device [n,h,w,3,K] Q4.12                                 */
    const uint16_t *weight;    /* device [n,h,w,K]   Q0.15, sum over K = 32768 per pixel   */
    const int16_t *chan_coef;  /* device [n,3]       Q2.14: a_GR, a_BR, a_BG               */
    uint32_t num_comp;         /* K, 1..16                                                 */
} pilc_mix_params;

/* As pilc_encode / pilc_decode (same geometry, workspace size from pilc_workspace_size,
 * alignment, ownership and container), with the magic "PMIX" and K in header word 11 (bytes
 * 44..47).  Runs one thread per lane whatever the number of lanes.
 * Errors: those of pilc_encode / pilc_decode; PILC_E_ARG also for K outside 1..16 and, found on
 * the device, for a pixel whose weights do not sum to 32768 (outputs then undefined). */
int pilc_mix_encode(const pilc_geom *geom, const uint8_t *img_dev, const pilc_mix_params *params,
                    void *workspace_dev, size_t workspace_bytes, uint8_t *coded_dev,
                    size_t coded_capacity, uint64_t *coded_bytes_host, void *hip_stream);
int pilc_mix_decode(const pilc_geom *geom, const uint8_t *coded_dev, size_t coded_bytes,
                    const pilc_mix_params *params, void *workspace_dev, size_t workspace_bytes,
                    uint8_t *img_out_dev, void *hip_stream);

/* Per-kernel timing, off by default.  When enabled, pilc_encode / pilc_decode bracket each
 * kernel with HIP events on the stream the kernel is launched on.  pilc_last_timing returns
 * the durations in milliseconds of the most recent call on the calling thread: index 0 is
 * the whole GPU part of the call, 1.. are its kernels in launch order (pilc_timing_name
 * gives the kernel's function name; "scan" covers the three scan kernels).  Returns the number of entries written (<= capacity), 0 if timing
 * was off. */
void pilc_set_timing(int enabled);
int pilc_last_timing(float *ms_out_host, int capacity);
const char *pilc_timing_name(int index_in_last_call);

/* Which lane kernels encode and decode use: 0 = chosen from the lane count (default), 1 = one
 * thread per lane, 2 = the kernels for few long lanes (workgroup-cooperative encode, a row of 16
 * threads per lane in decode), 3 = one thread per lane with the one-pass encoder (the lane kernel
 * also computes the offsets and places its lanes in the container, instead of leaving that to the
 * scan and pack kernels; measured no faster, kept for comparison).  All choices produce the same
 * bytes; the knob exists for tuning and for testing every kernel on the same input.  Process-wide.
 * Errors: PILC_E_ARG for any other value. */
int pilc_set_kernel_policy(int policy);

/* The one-pass encoder's (policy 3) workgroups learn where their lanes go from the workgroups
 * before them (the scan of Sec. 4.1's container offsets, fused into the lane kernel); a workgroup
 * waits for an earlier one at most `ticks` ticks of the GPU's constant-rate clock (0 = the
 * default, two seconds) and then gives up: the call returns PILC_E_TIMEOUT and every kernel still
 * ends.
 * `withhold_first` != 0 makes the first workgroup publish nothing, which forces that path: for
 * tests of the give-up path only.  The same bound and switch apply to the bands of
 * pilc_twar_inverse and to pilc_decode with few lanes, where every decoding wavefront waits for
 * a second one that prepares its next batch (the switch: nothing is ever said to be ready).
 * Process-wide. */
void pilc_set_one_pass_wait(uint64_t ticks, int withhold_first);

/* ------------------------------------------------------------------------------------------
 * The paper's own coder variant: ANS-AI (Sec. 3.2, Alg. 3 "Encode x", Alg. 4 "Decode one
 * symbol"), the table-driven form of the modified rANS of Alg. 1 / Alg. 2.  The state lives in
 * [2^M, 2^(M+1)); every symbol carries the index d of one of D fixed distributions over X
 * symbols; encode looks up delta[d,x], phi[d,x], decode looks up Theta[d,S], B[d,S], N[d,S].
 * A "piece" is one independent coder instance of `count` symbols (Sec. 4.3: one thread per
 * piece).  Readings the paper leaves open: a piece is encoded last symbol first so that decode
 * returns the symbols in order; the state starts at 2^M and decode must return there with the
 * stream used up; a pushed group of bits keeps its order, bit 0 of S first.
 * Container (little endian): 64-byte header {"PANS", 1, pieces, count, M, D, X, 0.., payload
 * bytes u64 at byte 48, 0}; u32 offsets[pieces+1] (bytes, relative to the payload); per piece
 * {final state u32, bit count u32, ceil(bits/32) words of 32 bits, bit i of the stream at bit
 * i%32 of word i/32}.
 * ------------------------------------------------------------------------------------------ */
typedef struct {
    uint32_t pieces, count; /* independent pieces, symbols per piece; rounded-up pieces*count < 2^32 */
    uint32_t prec_bits;     /* M, 1..15, 2^M >= num_sym */
    uint32_t num_dist;      /* D, 1..255 */
    uint32_t num_sym;       /* X, 2..256 */
} pilc_ansai_shape;

/* Bytes of device memory pilc_ansai_build_tables fills for these M, D, X (0 if invalid):
 * 8*(D*256+1) for delta and phi plus 3*D*2^M (5*D*2^M when M > 12) for Theta, B, N, plus padding. */
size_t pilc_ansai_table_bytes(uint32_t prec_bits, uint32_t num_dist, uint32_t num_sym);

/* Builds the tables of Sec. 3.2 on the device from integer masses.
 *   mass_dev    device uint32 [D, X], every P_x >= 1, each row summing to 2^M
 *   tables_dev  device, 256-byte aligned, tables_bytes >= pilc_ansai_table_bytes(); opaque to
 *               the caller, valid for any number of encode / decode calls with the same M, D, X
 * Errors: PILC_E_ARG (bad sizes or pointers, or masses that break the two conditions above:
 * the blob is then marked unusable), PILC_E_WORKSPACE (tables_bytes too small), PILC_E_HIP. */
int pilc_ansai_build_tables(uint32_t prec_bits, uint32_t num_dist, uint32_t num_sym,
                            const uint32_t *mass_dev, void *tables_dev, size_t tables_bytes,
                            void *hip_stream);

/* Re-centring of Sec. 3.3: the residual r ~ L(mu, s, 0, 255) is coded as (r - mu + 128) mod 256
 * ~ L(128, s, 0, 255), so that the distribution index only has to tell the scale.  mu is the
 * predicted location rounded to an integer.  inverse = 0: out = (in - mu + 128) mod 256 (before
 * pilc_ansai_encode); inverse != 0: out = (in + mu - 128) mod 256 (after pilc_ansai_decode).
 * in_dev, mu_dev, out_dev: device uint8 [count], 16-byte aligned; out_dev may be in_dev.
 * Errors: PILC_E_ARG, PILC_E_HIP. */
int pilc_ansai_center(const uint8_t *in_dev, const uint8_t *mu_dev, uint64_t count, int inverse,
                      uint8_t *out_dev, void *hip_stream);

/* Device workspace needed by pilc_ansai_encode / pilc_ansai_decode and an upper bound of the
 * container size (header + offsets + per piece 8 bytes and ceil(count*M/32) words).
 * Errors: PILC_E_ARG, PILC_E_TOO_LARGE. */
int pilc_ansai_workspace_size(const pilc_ansai_shape *shape, size_t *workspace_bytes_host,
                              size_t *max_coded_bytes_host);

/* Alg. 3 over a batch.  sym_dev, dist_dev: device uint8 [pieces, count], 16-byte aligned;
 * workspace_dev 256-byte aligned scratch; coded_dev 16-byte aligned output.
 * Errors: PILC_E_ARG (also: a symbol >= X or an index >= D in the data, or tables built for
 * other M, D, X), PILC_E_WORKSPACE, PILC_E_CAPACITY, PILC_E_TOO_LARGE, PILC_E_HIP; on error
 * the contents of coded_dev are undefined. */
int pilc_ansai_encode(const pilc_ansai_shape *shape, const uint8_t *sym_dev, const uint8_t *dist_dev,
                      const void *tables_dev, void *workspace_dev, size_t workspace_bytes,
                      uint8_t *coded_dev, size_t coded_capacity, uint64_t *coded_bytes_host,
                      void *hip_stream);

/* Alg. 4 over a batch; dist_dev must hold the indices used to encode.  sym_out_dev: device
 * uint8 [pieces, count], 16-byte aligned; on error its contents are undefined.
 * Errors: PILC_E_ARG (as above), PILC_E_WORKSPACE, PILC_E_FORMAT (header does not match the
 * shape or coded_bytes), PILC_E_CORRUPT (bad offsets or record, a piece that runs out of bits,
 * keeps some, or does not return to the initial state), PILC_E_HIP. */
int pilc_ansai_decode(const pilc_ansai_shape *shape, const uint8_t *coded_dev, size_t coded_bytes,
                      const uint8_t *dist_dev, const void *tables_dev, void *workspace_dev,
                      size_t workspace_bytes, uint8_t *sym_out_dev, void *hip_stream);

/* How many wavefronts a workgroup of pilc_ansai_decode's kernel has: 0 = chosen from the batch and
 * the table size (default: as many as fit beside the tables in LDS, fewer for a batch that would
 * not fill every compute unit that densely), 1 .. 12 = that many (less if fewer fit).  Every
 * choice decodes the same symbols; the knob exists for tuning and for testing every workgroup
 * shape on the same input.  Process-wide.  Errors: PILC_E_ARG for any other value. */
int pilc_set_ansai_decode_waves(int waves);

/* ------------------------------------------------------------------------------------------
 * The Three-Way Auto-regressive residual transform (Sec. 3.1, eqs. (2)-(4)): every subpixel is
 * predicted from three known values -- R(u,v) from R(u-1,v-1), R(u-1,v), R(u,v-1); G(u,v) from
 * G(u,v-1), R(u,v-1), R(u,v); B(u,v) from B(u,v-1), G(u,v-1), G(u,v); u the row, v the column --
 * with three weights and a bias per channel (12 parameters), and the residual goes to the coder.
 * Readings the paper leaves open: zero padding above and to the left; fixed-point weights,
 * x^ = clamp((w . ctx + bias + 2^13) >> 14, 0, 255) with an arithmetic shift; residual
 * r = (x - x^) mod 256, so that x = (r + x^) mod 256.
 * Images: device uint8 [n, h, w, 3], channel-interleaved; input and output must not overlap.
 * ------------------------------------------------------------------------------------------ */
typedef struct {
    int16_t w[3][3]; /* [channel][context value in the order above], Q2.14 */
    int32_t bias[3]; /* Q8.14, |bias| <= 2^30 */
} pilc_twar_params;

/* res = image minus prediction.  Errors: PILC_E_ARG, PILC_E_TOO_LARGE, PILC_E_HIP. */
int pilc_twar_forward(uint32_t n, uint32_t h, uint32_t w, const uint8_t *img_dev,
                      const pilc_twar_params *params_host, uint8_t *res_dev, void *hip_stream);

/* The image back from the residual (Sec. 3.1: the anti-diagonal / column schedule of the paper's
 * decoding figure, here one walk along the anti-diagonals of 64 rows per wavefront).  Fewer than
 * 256 images of more than 256 rows are cut into bands in workgroups of their own that follow each
 * other through counters in the library's device globals; their wait for the band above is bounded
 * like the one-pass encoder's (pilc_set_one_pass_wait) and ends in PILC_E_TIMEOUT.
 * Errors: PILC_E_ARG, PILC_E_TOO_LARGE, PILC_E_HIP, PILC_E_TIMEOUT (img_dev contents undefined). */
int pilc_twar_inverse(uint32_t n, uint32_t h, uint32_t w, const uint8_t *res_dev,
                      const pilc_twar_params *params_host, uint8_t *img_dev, void *hip_stream);

const char *pilc_strerror(int code);
const char *pilc_last_hip_error(void); /* text of the last HIP failure on this thread */
uint32_t pilc_version(void);

#ifdef __cplusplus
}
#endif
#endif
