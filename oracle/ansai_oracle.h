/*
 * ansai_oracle.h -- plain CPU reference of the paper's own table-driven coder.
 *
 * TEST INFRASTRUCTURE ONLY (as pilc_oracle.h): never part of the product path, shares no code
 * with the HIP implementation.
 *
 * What it follows (arXiv 2206.05279, Sec. 3.2):
 *   - Alg. 1 / Alg. 2, the "modified rANS": the state lives in [2^M, 2^(M+1)) and single bits
 *     move to and from a LIFO stream;
 *   - Alg. 3 / Alg. 4, "ANS-AI": the same coder with every loop and search replaced by the
 *     tables delta, phi (encode) and Theta, B, N (decode), indexed by a distribution index d in
 *     [0, D) and a symbol x in [0, X).  phi[d,x] = 2^M - P_x + C_x; delta[d,x] satisfies eq. (5),
 *     and App. B's lemma on the range of delta gives its value: k 2^M - P_x 2^k for the k with
 *     P_x 2^k in [2^M, 2^(M+1)).
 * A "piece" is one independent coder instance (Sec. 4.3: one thread per piece).
 *
 * Readings where the paper is silent: the encoder takes the symbols of a piece last-first so
 * that the decoder returns them first-last; the state starts at 2^M and the decoder must end
 * there with an empty stream; a pushed group of b bits keeps its bit order (bit 0 of S first)
 * inside little-endian 32-bit words, and a pop takes the last b bits back in the same order.
 * Container (little endian): 64-byte header {"PANS", version 1, pieces, symbols per piece, M, D,
 * X, 0.., payload bytes u64 at byte 48, 0}, u32 offsets[pieces+1] (bytes relative to the payload,
 * multiples of 4), then per piece {final state u32, bit count u32, ceil(bits/32) words}.
 *
 * Return codes: 0 ok, -1 bad argument or a symbol / distribution index out of range,
 * -3 capacity, -5 header mismatch, -6 corrupt stream.
 */
#ifndef ANSAI_ORACLE_H
#define ANSAI_ORACLE_H
#include <stdint.h>
#ifdef __cplusplus
extern "C" {
#endif

typedef struct {
    int prec_bits; /* M, 1..15 */
    int num_dist;  /* D, 1..255 (an interface limit; Sec. 4.3 of the paper uses 8) */
    int num_sym;   /* X, 2..256 */
    const uint32_t *mass; /* [D, X] integer masses P_x >= 1, each row sums to 2^M */
} ansai_model;

/* Tables of Sec. 3.2.  delta, phi: [D, X] (int32 / uint32 here; that 16 bits suffice under the
 * lemma's conditions is a tested property, not a storage format).  theta, nbits: [D, 2^M] uint8,
 * next: [D, 2^M] uint16 = N[d,S] - 2^M, all indexed by S - 2^M. */
int ansai_oracle_build_tables(const ansai_model *model, int32_t *delta, uint32_t *phi,
                              uint8_t *theta, uint8_t *nbits, uint16_t *next);

/* One piece with the modified rANS of Sec. 3.2 computed directly from the masses, no tables: per
 * symbol the count of bits that leave the state follows from bit lengths (see the .c file).
 * bits_out (capacity count*M): one bit per byte in push order.  Returns the number of bits (-1 on
 * a bad symbol or index); *state_out is the final state in [2^M, 2^(M+1)). */
int64_t ansai_oracle_encode_piece_direct(const ansai_model *model, const uint8_t *sym,
                                        const uint8_t *dist, int64_t count, uint8_t *bits_out,
                                        uint32_t *state_out);
/* Its inverse: interval search over the running sums, then the bits that restore the state's
 * range, counted from the bit length.  0 on success, -6 if the stream runs dry, is not used up, or
 * the state does not return to its start. */
int ansai_oracle_decode_piece_direct(const ansai_model *model, const uint8_t *dist, int64_t count,
                                    const uint8_t *bits, int64_t nbits, uint32_t state,
                                    uint8_t *sym_out);

uint64_t ansai_oracle_max_coded_bytes(uint32_t pieces, uint32_t count, int prec_bits);

/* A whole batch with the tables of Alg. 3 / Alg. 4.  sym, dist: [pieces, count] uint8. */
int ansai_oracle_encode(const ansai_model *model, uint32_t pieces, uint32_t count,
                        const uint8_t *sym, const uint8_t *dist, uint8_t *coded, uint64_t capacity,
                        uint64_t *coded_bytes);
int ansai_oracle_decode(const ansai_model *model, uint32_t pieces, uint32_t count,
                        const uint8_t *dist, const uint8_t *coded, uint64_t coded_bytes,
                        uint8_t *sym_out);

/* Sec. 3.3: the residual r ~ L(mu, s, 0, 255) is coded as (r - mu + 128) mod 256 ~ L(128, s, 0, 255),
 * so that the distribution index only has to tell the scale.  mu is the predicted location rounded
 * to an integer (a reading: the paper keeps the prediction in the uint8 range).  inverse = 0: out = (r - mu +
 * 128) mod 256; inverse != 0: out = (c + mu - 128) mod 256. */
void ansai_oracle_center(const uint8_t *in, const uint8_t *mu, uint64_t n, int inverse, uint8_t *out);
#ifdef __cplusplus
}
#endif
#endif
