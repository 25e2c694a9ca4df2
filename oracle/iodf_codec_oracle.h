/*
 * CPU oracle for the entropy-coding side of an IODF compressor (arXiv 2206.08869):
 * the factorised discretised-logistic prior over the latents (Sec. 3) evaluated in
 * integers, and range-based asymmetric numeral systems (App. A) in a streaming form.
 *
 * THIS IS TEST INFRASTRUCTURE, not the product; it shares no code, header, table or
 * constant generator with the GPU library.
 *
 * What the paper fixes: the prior's shape, p(z) = sigma((z + 1/2 - mu)/s) -
 * sigma((z - 1/2 - mu)/s) (Sec. 3), and the coder's state recurrences
 * X_t = floor(X_{t-1} / F) * M + C + X_{t-1} mod F and their inverse (App. A), with
 * integer masses F of total M and cumulative masses C.
 * What it leaves open, fixed here (the same readings as the GPU library, written
 * independently):
 *  - mu = 2 * m and s = 2^(l / 16) for the 8-bit mean code m and log-scale code l
 *    of a latent; a latent without a head (flows without heads, the deepest level)
 *    has m = 0, l = 96.
 *  - total mass M = 2^24 over the alphabet r = z - mu in [-8192, 8191]; every symbol
 *    keeps a floor mass of 1, the remaining M - 16384 follows the logistic CDF:
 *    G(r) = (r + 8192) + floor((M - 16384) * S((2r - 1) / (2s)) / 2^30), C = G(r),
 *    F = G(r + 1) - G(r).
 *  - S(t) ~ 2^30 * sigma(t) is a table of correctly rounded values at t = -24 + j/64,
 *    j = 0..3072, linearly interpolated with floor; 0 below -24 and 2^30 above 24.
 *    The argument is formed in fixed point: T = (2r - 1) * INV[l], INV[l] =
 *    round(2^23 * 2^(-l/16)), t = T / 2^24.
 *  - the coder state is 64 bits in [2^31, 2^63), starts at 2^31 (App. A's X_0 = 0
 *    cannot mark the end of a stream), and sheds its low 32 bits as one word when the
 *    next update would leave the interval (X >= F * 2^39).
 *  - a chunk of n symbols is dealt to 16 independent lanes (symbol e -> lane e mod
 *    16); each lane encodes its symbols last-to-first so that decoding returns them
 *    first-to-last, and its words are stored in the order the decoder reads them.
 *  - an image's container is a sequence of little-endian 32-bit words: total word
 *    count; words per (chunk, lane); final states (low, high) per (chunk, lane); then
 *    every lane's words, chunk-major, lane-minor.
 *
 * Pins (tests, CPU only): both tables against 50-digit decimal arithmetic; G
 * monotone with G(-8192) = 0, G(8192) = M and F >= 1; masses against the paper's
 * formula in float64; one coder step against App. A's recurrences in unbounded
 * Python integers; decode(encode) = identity; code length against -sum log2(F / M).
 */
#ifndef IODF_CODEC_ORACLE_H
#define IODF_CODEC_ORACLE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    ORC_MASS_BITS = 24,
    ORC_ALPHA_R = 8192,
    ORC_SIG_BITS = 30,
    ORC_SIG_ENTRIES = 3073,
    ORC_LANES = 16,
    ORC_DEFAULT_M = 0,
    ORC_DEFAULT_L = 96
};

/* Copies of the two tables (for the pins): sig[3073], inv[256] (index l + 128). */
void orc_prior_tables(int32_t* sig, int64_t* inv);

/* S(T): T = t * 2^24. */
int64_t orc_prior_sigmoid(int64_t T);
/* G(r) for -8192 <= r <= 8192 and log-scale code l. */
int64_t orc_prior_cdf(int r, int l);

/* Masses of n latents: C[i] = G(r_i), F[i] = G(r_i + 1) - G(r_i), r_i = z[i] - 2 m[i].
 * m, l may be NULL (defaults). A residual outside the alphabet is clamped into it and
 * counted in the return value. */
int64_t orc_prior_cf(const int32_t* z, const int8_t* m, const int8_t* l, int64_t n, int32_t* C, int32_t* F);

/* One coder update (App. A, encoder recurrence, with the word shed before it when
 * needed). Returns the new state; *word_out is valid when *emitted is 1. */
uint64_t orc_rans_push(uint64_t X, uint32_t C, uint32_t F, int* emitted, uint32_t* word_out);
/* Inverse update for a known symbol (App. A, decoder recurrence), without refill. */
uint64_t orc_rans_pop(uint64_t X, uint32_t C, uint32_t F);

/* Number of header words of a container with n_chunks chunks. */
int64_t orc_codec_header_words(int n_chunks);

/* Encode one image: chunk c holds n[c] latents at z + z_off[c]; its codes are at
 * codes + code_off[c] (n[c] mean codes, then n[c] log-scale codes) or absent when
 * code_off[c] < 0. Writes at most cap words to out; returns the container's size in
 * words (which may exceed cap: then the container is unusable). *n_clamped counts
 * residuals outside the alphabet. */
int64_t orc_codec_encode_image(const int32_t* z, const int8_t* codes, int n_chunks, const int64_t* n,
                               const int64_t* z_off, const int64_t* code_off, uint32_t* out, int64_t cap,
                               int64_t* n_clamped);

/* Decode chunk c of a container into z_chunk (n[c] latents) given its codes
 * (m, l: n[c] each, or NULL). Returns 0, or -1 when the container is malformed or a
 * lane does not end in the initial state with all its words consumed. */
int orc_codec_decode_chunk(const uint32_t* cont, int64_t cont_words, int n_chunks, const int64_t* n, int c,
                           const int8_t* m, const int8_t* l, int32_t* z_chunk);

#ifdef __cplusplus
}
#endif
#endif
