/* CPU oracle of the prior masses and the streaming rANS coder; see iodf_codec_oracle.h.
 * Test infrastructure: plain loops, nothing shared with the GPU library. */
#include "iodf_codec_oracle.h"

#include <math.h>
#include <stdlib.h>
#include <string.h>

#define MASS ((int64_t)1 << ORC_MASS_BITS)
#define RR ((int64_t)ORC_ALPHA_R)
#define STATE_LOW ((uint64_t)1 << 31)

static int32_t g_sig[ORC_SIG_ENTRIES];
static int64_t g_inv[256];
static int g_ready = 0;

/* Tables of the integer prior: 2^30 * sigma(t) at t = -24 + j/64, and 2^23 * 2^(-l/16),
 * both rounded to nearest (computed in long double, far finer than the rounding step). */
static void make_tables(void) {
    if (g_ready) return;
    for (int j = 0; j < ORC_SIG_ENTRIES; ++j) {
        const long double t = -24.0L + (long double)j / 64.0L;
        const long double s = 1.0L / (1.0L + expl(-t));
        g_sig[j] = (int32_t)floorl(s * 1073741824.0L + 0.5L);
    }
    for (int l = -128; l <= 127; ++l)
        g_inv[l + 128] = (int64_t)floorl(exp2l(23.0L - (long double)l / 16.0L) + 0.5L);
    g_ready = 1;
}

void orc_prior_tables(int32_t* sig, int64_t* inv) {
    make_tables();
    if (sig) memcpy(sig, g_sig, sizeof(g_sig));
    if (inv) memcpy(inv, g_inv, sizeof(g_inv));
}

int64_t orc_prior_sigmoid(int64_t T) {
    make_tables();
    const int64_t tmax = (int64_t)24 << 24;
    if (T <= -tmax) return 0;
    if (T >= tmax) return (int64_t)1 << ORC_SIG_BITS;
    const int64_t u = T + tmax;            /* 0 < u < 48 * 2^24 */
    const int64_t j = u >> 18;             /* table step 1/64 = 2^18 units of 2^-24 */
    const int64_t frac = u & (((int64_t)1 << 18) - 1);
    return (int64_t)g_sig[j] + ((((int64_t)g_sig[j + 1] - (int64_t)g_sig[j]) * frac) >> 18);
}

/* Sec. 3: the CDF of the logistic at the lower edge of symbol r is sigma((r - 1/2) / s)
 * = sigma((2r - 1) / (2s)); a floor mass of one per symbol is added underneath. */
int64_t orc_prior_cdf(int r, int l) {
    make_tables();
    const int64_t T = (2 * (int64_t)r - 1) * g_inv[l + 128];
    return ((int64_t)r + RR) + (((MASS - 2 * RR) * orc_prior_sigmoid(T)) >> ORC_SIG_BITS);
}

int64_t orc_prior_cf(const int32_t* z, const int8_t* m, const int8_t* l, int64_t n, int32_t* C, int32_t* F) {
    int64_t clamped = 0;
    for (int64_t i = 0; i < n; ++i) {
        const int mi = m ? m[i] : ORC_DEFAULT_M, li = l ? l[i] : ORC_DEFAULT_L;
        int64_t r = (int64_t)z[i] - 2 * (int64_t)mi;
        if (r < -RR) { r = -RR; ++clamped; }
        if (r > RR - 1) { r = RR - 1; ++clamped; }
        const int64_t c = orc_prior_cdf((int)r, li);
        C[i] = (int32_t)c;
        F[i] = (int32_t)(orc_prior_cdf((int)r + 1, li) - c);
    }
    return clamped;
}

/* App. A, encoder: X_t = floor(X_{t-1} / F) * M + C + X_{t-1} mod F. Before it, the
 * state sheds its low word if the update would leave [2^31, 2^63). */
uint64_t orc_rans_push(uint64_t X, uint32_t C, uint32_t F, int* emitted, uint32_t* word_out) {
    int e = 0;
    if (X >= ((uint64_t)F << 39)) {
        if (word_out) *word_out = (uint32_t)(X & 0xffffffffu);
        X >>= 32;
        e = 1;
    }
    if (emitted) *emitted = e;
    return (X / F) * (uint64_t)MASS + C + (X % F);
}

/* App. A, decoder: X_{t-1} = floor(X_t / M) * F + (X_t mod M - C). */
uint64_t orc_rans_pop(uint64_t X, uint32_t C, uint32_t F) {
    return (uint64_t)F * (X >> ORC_MASS_BITS) + (X & (uint64_t)(MASS - 1)) - C;
}

int64_t orc_codec_header_words(int n_chunks) { return 1 + 3 * (int64_t)n_chunks * ORC_LANES; }

static void put(uint32_t* out, int64_t cap, int64_t idx, uint32_t v) {
    if (idx < cap) out[idx] = v;
}

int64_t orc_codec_encode_image(const int32_t* z, const int8_t* codes, int n_chunks, const int64_t* n,
                               const int64_t* z_off, const int64_t* code_off, uint32_t* out, int64_t cap,
                               int64_t* n_clamped) {
    const int64_t header = orc_codec_header_words(n_chunks);
    int64_t pos = header, clamped = 0;
    for (int c = 0; c < n_chunks; ++c) {
        const int64_t nc = n[c];
        int32_t* C = (int32_t*)malloc((size_t)(nc > 0 ? nc : 1) * sizeof(int32_t));
        int32_t* F = (int32_t*)malloc((size_t)(nc > 0 ? nc : 1) * sizeof(int32_t));
        uint32_t* w = (uint32_t*)malloc((size_t)(nc / ORC_LANES + 2) * sizeof(uint32_t));
        const int8_t* m = code_off[c] >= 0 ? codes + code_off[c] : NULL;
        const int8_t* l = code_off[c] >= 0 ? codes + code_off[c] + nc : NULL;
        clamped += orc_prior_cf(z + z_off[c], m, l, nc, C, F);
        for (int j = 0; j < ORC_LANES; ++j) {
            const int64_t k = j < nc ? (nc - j + ORC_LANES - 1) / ORC_LANES : 0; /* symbols of this lane */
            uint64_t X = STATE_LOW;
            int64_t nw = 0;
            for (int64_t p = k - 1; p >= 0; --p) {
                const int64_t e = p * ORC_LANES + j;
                int emitted;
                uint32_t word;
                X = orc_rans_push(X, (uint32_t)C[e], (uint32_t)F[e], &emitted, &word);
                if (emitted) w[nw++] = word;
            }
            const int64_t slot = (int64_t)c * ORC_LANES + j;
            put(out, cap, 1 + slot, (uint32_t)nw);
            put(out, cap, 1 + (int64_t)n_chunks * ORC_LANES + 2 * slot, (uint32_t)(X & 0xffffffffu));
            put(out, cap, 1 + (int64_t)n_chunks * ORC_LANES + 2 * slot + 1, (uint32_t)(X >> 32));
            /* the decoder reads the words in the reverse of the order they were shed */
            for (int64_t i = 0; i < nw; ++i) put(out, cap, pos + i, w[nw - 1 - i]);
            pos += nw;
        }
        free(C); free(F); free(w);
    }
    put(out, cap, 0, (uint32_t)pos);
    if (n_clamped) *n_clamped = clamped;
    return pos;
}

int orc_codec_decode_chunk(const uint32_t* cont, int64_t cont_words, int n_chunks, const int64_t* n, int c,
                           const int8_t* m, const int8_t* l, int32_t* z_chunk) {
    const int64_t header = orc_codec_header_words(n_chunks);
    if (cont_words < header || (int64_t)cont[0] > cont_words || (int64_t)cont[0] < header || c < 0 || c >= n_chunks)
        return -1;
    const int64_t total = cont[0];
    /* start of this chunk's words: everything of the chunks and lanes before it */
    int64_t pos = header;
    for (int64_t s = 0; s < (int64_t)c * ORC_LANES; ++s) pos += cont[1 + s];
    const int64_t nc = n[c];
    for (int j = 0; j < ORC_LANES; ++j) {
        const int64_t slot = (int64_t)c * ORC_LANES + j;
        const int64_t nw = cont[1 + slot];
        if (pos + nw > total) return -1;
        const uint32_t* w = cont + pos;
        int64_t used = 0;
        uint64_t X = (uint64_t)cont[1 + (int64_t)n_chunks * ORC_LANES + 2 * slot] |
                     ((uint64_t)cont[1 + (int64_t)n_chunks * ORC_LANES + 2 * slot + 1] << 32);
        const int64_t k = j < nc ? (nc - j + ORC_LANES - 1) / ORC_LANES : 0;
        for (int64_t p = 0; p < k; ++p) {
            const int64_t e = p * ORC_LANES + j;
            const int mi = m ? m[e] : ORC_DEFAULT_M, li = l ? l[e] : ORC_DEFAULT_L;
            const int64_t v = (int64_t)(X & (uint64_t)(MASS - 1));
            /* App. A: the symbol is the one whose [C, C + F) holds X mod M */
            int lo = -(int)RR, hi = (int)RR;
            while (hi - lo > 1) {
                const int mid = lo + (hi - lo) / 2;
                if (orc_prior_cdf(mid, li) <= v) lo = mid; else hi = mid;
            }
            const int64_t Cs = orc_prior_cdf(lo, li), Fs = orc_prior_cdf(lo + 1, li) - Cs;
            z_chunk[e] = lo + 2 * mi;
            X = orc_rans_pop(X, (uint32_t)Cs, (uint32_t)Fs);
            if (X < STATE_LOW) {
                if (used >= nw) return -1;
                X = (X << 32) | w[used++];
            }
        }
        if (X != STATE_LOW || used != nw) return -1;
        pos += nw;
    }
    return 0;
}
