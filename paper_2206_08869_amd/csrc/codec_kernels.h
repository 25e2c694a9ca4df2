// Entropy-coding side of the compressor: masses of the discretised-logistic prior
// (Sec. 3) evaluated in integers, and range-based asymmetric numeral systems
// (App. A) in a streaming form with 16 independent lanes per chunk of latents.
// All pointers are device memory unless said otherwise; every call only enqueues.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace iodf {

constexpr int kMassBits = 24;        // total mass M = 2^24
constexpr int kAlphaR = 8192;        // alphabet: residual r = z - mu in [-8192, 8191]
constexpr int kSigBits = 30;         // integer sigmoid S(t) ~ 2^30 * sigma(t)
constexpr int kSigEntries = 3073;    // t = -24 + j / 64
constexpr int kLanes = 16;           // coder lanes per chunk
constexpr int kDefaultM = 0;         // codes of a latent without a head: mu = 0,
constexpr int kDefaultL = 96;        //   s = 2^(96/16) = 64
constexpr int kMaxChunks = 8;

// Host: fills the two tables of the integer prior. sig[j] = round(2^30 * sigma(-24 + j/64)),
// inv[l + 128] = round(2^23 * 2^(-l/16)) (1/(2s) in units of 2^-24 for s = 2^(l/16)).
void codec_make_tables(int32_t* sig, int64_t* inv);

// Where the chunks of one image live (chunk c = level c + 1).
struct ChunkTable {
    int n_chunks;
    int n[kMaxChunks];            // latents
    long long z_off[kMaxChunks];  // offset in an image's z
    long long code_off[kMaxChunks];  // offset of its n mean codes (then n log-scale codes); -1: none
    long long lane_off[kMaxChunks];  // offset of the chunk's lanes in an image's lane scratch (words)
    int lane_cap[kMaxChunks];     // words a lane of this chunk may shed: ceil(n / 16) + 1
};

struct CodecTables {
    const int32_t* sig;   // [kSigEntries]
    const int64_t* inv;   // [256]
};

// errs[0]: residuals outside the alphabet (clamped); errs[1]: containers that did not fit their
// capacity; errs[2]: lanes that did not decode back to the initial state.
hipError_t launch_prior_cf(const CodecTables& t, const ChunkTable& ct, const int32_t* z, long long d,
                           const int8_t* codes, long long d_codes, int batch, int32_t* c_out, int32_t* f_out,
                           unsigned long long* errs, hipStream_t st);

// z, codes -> lane scratch: lane_words[b][lane_words_per_image], lane_meta[b][n_chunks*16][4]
// (word count, state low, state high, 0).
hipError_t launch_rans_encode(const CodecTables& t, const ChunkTable& ct, const int32_t* z, long long d,
                              const int8_t* codes, long long d_codes, int batch, uint32_t* lane_words,
                              long long lane_words_per_image, uint32_t* lane_meta, unsigned long long* errs,
                              hipStream_t st);

// Lane scratch -> one container per image at out + b * cap (at most cap words), sizes[b] = words needed.
hipError_t launch_rans_pack(const ChunkTable& ct, const uint32_t* lane_words, long long lane_words_per_image,
                            const uint32_t* lane_meta, int batch, uint32_t* out, long long cap, uint32_t* sizes,
                            unsigned long long* errs, hipStream_t st);

// Chunk c of every container -> z[b][z_off[c] ..], with the chunk's codes (or none).
hipError_t launch_rans_decode_chunk(const CodecTables& t, const ChunkTable& ct, int c, const uint32_t* cont,
                                    long long cap, int batch, const int8_t* codes, long long d_codes, int32_t* z,
                                    long long d, unsigned long long* errs, hipStream_t st);

}  // namespace iodf
