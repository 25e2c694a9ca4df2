/*
 * libiodf: integer-only inference of an Integer-only Discrete Flow (arXiv
 * 2206.08869) on AMD MI355X (gfx950). C ABI: plain pointers and sizes only.
 *
 * The flow maps an image x in Z^d to a latent z = f(x) of the same size and back
 * (Sec. 3). f is a stack of levels; each level squeezes space to depth, applies K
 * additive couplings  z_a = x_a, z_b = x_b + t(x_a)  (Sec. 3, Eq. 1) and factors
 * half of the channels out. t() is an integer-only network: 8-bit codes, int8 x
 * int8 convolutions with 32-bit accumulator and bias, a per-channel fixed-point
 * rescale back to 8 bit, integer ReLU (Sec. 4.1, Eq. 2-5), with gated-off filters
 * and the matching input columns of their consumers physically removed (Sec. 4.4,
 * Eq. 8); where a residual shortcut needs the unpruned width, a gated-off filter is
 * kept as an all-zero row, which adds exactly the 0 that its removal would.
 *
 * Pointer conventions: "host" = ordinary process memory; "device" = memory of
 * the GPU the context was created on, owned by the caller (for instance a
 * PyTorch-ROCm tensor's data_ptr()). `stream` is a hipStream_t passed as void*
 * (NULL = the default stream). iodf_forward / iodf_inverse only enqueue work on
 * that stream and never synchronise; the caller synchronises before reading.
 * A context must not be used from two streams at once (it owns one workspace).
 * Calls are replayed from HIP graphs kept per (direction, batch, with/without codes): the first
 * call of a shape captures its graph on an internal stream (host work only, a few ms); inputs and
 * outputs pass through internal staging buffers with device-to-device copies on the caller's
 * stream. Setting IODF_NO_GRAPH=1 in the environment before iodf_init launches kernels directly.
 *
 * Every function returns IODF_OK (0) or a negative IODF_E_* code; nothing throws.
 */
#ifndef IODF_H
#define IODF_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct iodf_ctx iodf_ctx;

enum {
    IODF_OK = 0,
    IODF_E_ARG = -1,    /* NULL or out-of-range argument */
    IODF_E_BLOB = -2,   /* malformed model blob (magic, truncation, bad constants) */
    IODF_E_SHAPE = -3,  /* blob is well formed but its layers do not fit the declared family */
    IODF_E_BATCH = -4,  /* batch < 0 or batch > max_batch */
    IODF_E_HIP = -5,    /* a HIP runtime call failed (iodf_last_hip_error has the code) */
    IODF_E_NOMEM = -6,  /* host or device allocation failed */
    IODF_E_SCRATCH = -7 /* iodf_encode_noalloc: the batch needs more than the static scratch holds */
};

/* What iodf_query reports. */
enum {
    IODF_Q_Z_ELEMS = 0,          /* d: int32 latent elements per image (= 3*H*W) */
    IODF_Q_CODE_BYTES = 1,       /* int8 prior-parameter codes per image (0 without heads) */
    IODF_Q_WORKSPACE_BYTES = 2,  /* device memory held by the context */
    IODF_Q_MACS_FORWARD = 3,     /* algorithmic multiply-accumulates per image, kept channels only, true widths */
    IODF_Q_MACS_INVERSE = 4,     /* same for decode (no prior heads) */
    IODF_Q_RANGE_ERRORS = 5,     /* pixels outside [0,255] met by iodf_inverse since the last query;
                                    synchronises the device and resets the counter */
    IODF_Q_MAX_BATCH = 6,
    IODF_Q_IMAGE_H = 7,
    IODF_Q_IMAGE_W = 8,
    IODF_Q_CONV_LAUNCHES = 9,    /* convolution kernels per forward call */
    IODF_Q_WIDE_MACS_FORWARD = 10, /* of IODF_Q_MACS_FORWARD, the part in layers whose C_in and C_out are both >= 128 */
    IODF_Q_CODEC_HEADER_WORDS = 11, /* 32-bit words of a container's header: 1 + 3 * 16 * levels */
    IODF_Q_CODEC_MAX_WORDS = 12,    /* capacity no container exceeds: header + d (a latent sheds at most one word) */
    IODF_Q_CODEC_CLAMPED = 13,      /* latents whose residual z - mu left [-8192, 8191] and was clamped (the image
                                       then does NOT decode back); 13..15 synchronise and reset like RANGE_ERRORS */
    IODF_Q_CODEC_OVERFLOWS = 14,    /* containers that needed more than cap_words (truncated, unusable) */
    IODF_Q_CODEC_BROKEN_LANES = 15, /* coder lanes that iodf_decode could not read back to their initial state
                                       (malformed or foreign container) */
    IODF_Q_NOALLOC_MAX_BATCH = 16   /* largest batch iodf_encode_noalloc accepts for this model (<= max_batch) */
};

/*
 * Build a context from a model blob (Sec. 4.1, 4.4: weights, per-channel rescale
 * constants, binary gates).
 *   out          host; receives the context (caller releases it with iodf_free).
 *   model_blob   host; little-endian, 4-byte aligned fields:
 *                  header 16 x u32: 'IODF','BLB1', version 1, H, W, levels, couplings per
 *                    level, family (0 plain, 1 residual, 2 dense), width, depth, has_heads,
 *                    n_nets, act_unsigned (0 | 1), 3 x reserved (0)
 *                  per network in flow order (level 1 couplings, level 1 head, level 2, ...):
 *                    8 x 32 bit: kind (0 coupling, 1 head), level, C_level, C_in, C_out,
 *                    n_layers, M_in (i32), s_in; then i32 perm[C_level] for couplings;
 *                    per conv layer: 4 x u32 C_out, C_in, k (1|3), flags (bit0 ReLU, bit1
 *                    shortcut); i8 W[C_out][C_in][k][k]; i32 bias[C_out]; i32 M[C_out];
 *                    u8 shift[C_out]; u8 gate[C_out] (1 = keep); arrays padded to 4 bytes.
 *                The blob is copied/repacked; the caller may free it on return. Filters with
 *                gate 0 and the matching input columns of their consumers are removed here,
 *                so they cost nothing at inference.
 *   device_ordinal  HIP device to run on.
 *   max_batch    largest batch later calls may pass (sizes the workspace); >= 1.
 * act_unsigned = 1 selects the paper's hybrid number format (Sec. 4.1, Eq. 3): every tensor that
 * leaves a ReLU holds unsigned codes 0..255 (saturation at 255), read as such by the next
 * convolution and by the shortcut; the input quantiser's output, the translation and the head
 * codes stay signed. Every hidden layer must then carry a ReLU and the last layer none.
 * Constants must satisfy 0 <= M < 2^31, 0 <= shift <= 62, |bias| < 2^30, and for every filter
 * |bias| + X * sum|w| < 2^31 with X = 128 (256 for a layer reading unsigned codes), so that the
 * 32-bit accumulator of Eq. 4-5 cannot overflow for any input; a blob that breaks one of these is
 * refused with IODF_E_BLOB.
 */
int iodf_init(iodf_ctx** out, const void* model_blob, size_t blob_bytes, int device_ordinal, int max_batch);

/*
 * Encode (Sec. 3: z = f(x)).
 *   x_dev      device, uint8 [batch][3][H][W]; read only.
 *   z_dev      device, int32 [batch][d]; per image the concatenation over levels l = 1..L of
 *              the factored-out chunk [C_z,l][h_l][w_l] (last level: all channels).
 *   codes_dev  device, int8 [batch][code bytes], or NULL to skip the prior heads; per image
 *              the concatenation over heads l = 1..L-1 of [2*C_z,l][h_l][w_l]: first C_z,l maps
 *              are the codes of the logistic prior's mean, the rest of its log-scale (Sec. 3).
 * batch may be 0 (no work).
 */
int iodf_forward(iodf_ctx* ctx, const uint8_t* x_dev, int batch, int32_t* z_dev, int8_t* codes_dev, void* stream);

/*
 * Decode (Sec. 3: x = f^{-1}(z)): couplings replayed in reverse, x_b = z_b - t(z_a).
 *   z_dev  device, int32 [batch][d], layout as written by iodf_forward; read only.
 *   x_dev  device, uint8 [batch][3][H][W]. A z that is no image of any x can decode to a
 *          value outside [0,255]: the byte is saturated and counted (IODF_Q_RANGE_ERRORS).
 */
int iodf_inverse(iodf_ctx* ctx, const int32_t* z_dev, int batch, uint8_t* x_dev, void* stream);

/*
 * Compressor: bits = rANS(f(x); p_Z) and back (Sec. 3 prior, Sec. 5.2 "actual encoding", App. A).
 *
 * Prior of a latent z with mean code m and log-scale code l (int8, from the level's head;
 * m = 0, l = 96 for latents without a head): discretised logistic with mu = 2 m, s = 2^(l/16),
 * evaluated in integers: cumulative mass G(r) = (r + 8192) + floor((2^24 - 16384) *
 * S((2r - 1)/(2s)) / 2^30) over the residual r = z - mu in [-8192, 8191], S a 3073-entry table
 * of round(2^30 sigma(t)) at t = -24 + j/64 with linear interpolation; C = G(r), F = G(r+1) - G(r)
 * >= 1, total mass M = 2^24.
 * Coder: App. A's recurrences on a 64-bit state in [2^31, 2^63) that starts at 2^31 and sheds /
 * refills 32-bit words; a level's latents are dealt round-robin to 16 independent lanes.
 * Container of one image (little-endian u32 words): total word count; words per (level, lane);
 * final state (low, high) per (level, lane); then each lane's words in decoding order.
 *
 * iodf_prior_cf: z_dev int32 [batch][d], codes_dev int8 [batch][code bytes] (required when the
 *   model has heads, ignored otherwise) -> c_dev, f_dev int32 [batch][d] (device).
 * iodf_encode: x_dev uint8 [batch][3][H][W] -> words_dev u32 [batch][cap_words] (one container
 *   per image, never written past cap_words) and sizes_dev u32 [batch] (words each container
 *   needs; larger than cap_words means truncated, see IODF_Q_CODEC_OVERFLOWS).
 * iodf_decode: containers -> x_dev. cap_words must be at least the header size. Malformed
 *   containers never cause out-of-range reads; they are counted (IODF_Q_CODEC_BROKEN_LANES).
 * The first of these calls on a context allocates the compressor's device buffers. Calls on one
 * context must not overlap. iodf_codec_tables copies the two tables (host: int32 sig[3073],
 * int64 inv[256] = round(2^23 * 2^(-l/16)) at index l + 128); it needs no GPU.
 */
int iodf_prior_cf(iodf_ctx* ctx, const int32_t* z_dev, const int8_t* codes_dev, int batch, int32_t* c_dev,
                  int32_t* f_dev, void* stream);
int iodf_encode(iodf_ctx* ctx, const uint8_t* x_dev, int batch, uint32_t* words_dev, int64_t cap_words,
                uint32_t* sizes_dev, void* stream);
int iodf_decode(iodf_ctx* ctx, const uint32_t* words_dev, int64_t cap_words, int batch, uint8_t* x_dev, void* stream);
int iodf_codec_tables(int32_t* sig_host, int64_t* inv_host);

/*
 * iodf_encode for callers that cannot allocate device memory: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc. Same arguments, same containers, word for word.
 * The coder's working buffers (the batch's latents and codes, the words each lane sheds, lane
 * states, the prior's tables and the error counters), which iodf_encode allocates on its first
 * call, live in a 64 MiB array that is part of the library's device image; each GPU holds one copy
 * from the moment the library is loaded until the process ends, and iodf_init prepares it. The call
 * allocates and frees nothing and launches the flow kernel by kernel instead of replaying a graph.
 * A batch whose buffers do not fit returns IODF_E_SCRATCH before anything is enqueued
 * (IODF_Q_NOALLOC_MAX_BATCH tells the limit for a model: 554 images of 3x64x64 with prior heads on four levels).
 * All contexts on one GPU share that GPU's array: calls that overlap on one GPU (from any context,
 * on any streams) race; serialise them. The error counters of these calls are shared per GPU too and
 * are reported, and reset, by iodf_query(IODF_Q_CODEC_*) of any context that used this entry point.
 */
int iodf_encode_noalloc(iodf_ctx* ctx, const uint8_t* x_dev, int batch, uint32_t* words_dev, int64_t cap_words,
                        uint32_t* sizes_dev, void* stream);

/*
 * Patch-based coding of images larger than the flow's H x W (Sec. 5.2: a large image is coded as
 * a batch of patches). img_dev: device, planar uint8 [3][img_h][img_w]. The image is covered by a
 * row-major grid of ceil(img_h/H) x ceil(img_w/W) patches; iodf_tile_patches writes patches
 * first_patch .. first_patch + n_patches - 1 to x_dev (uint8 [n_patches][3][H][W], ready for
 * iodf_forward / iodf_encode), reading 128 where a patch sticks out of the image;
 * iodf_untile_patches copies decoded patches back, dropping what lies outside. Patches beyond the
 * grid are an argument error.
 */
int iodf_tile_patches(iodf_ctx* ctx, const uint8_t* img_dev, int img_h, int img_w, int first_patch, int n_patches,
                      uint8_t* x_dev, void* stream);
int iodf_untile_patches(iodf_ctx* ctx, const uint8_t* x_dev, int first_patch, int n_patches, uint8_t* img_dev,
                        int img_h, int img_w, void* stream);

/*
 * One integer-only convolution layer on its own: the isolated shapes the paper times in its
 * architecture argument (Sec. 4.3, Table 1). All tensors are HOST memory, channel-first:
 * x int8 [batch][c_in][h][w], w int8 [c_out][c_in][k][k], bias / m int32 [c_out], shift u8 [c_out]
 * (same constraints as in a blob), y int8 [batch][c_out][h][w] = sat8(relu?(rq(conv(x) + bias))).
 * The layer is packed and run exactly as inside a flow (same kernels, zero padding (k-1)/2); the
 * call allocates and frees its own device buffers, runs the layer once for y and then `iters` more
 * times between two events: *us_per_call (may be NULL) is the mean device time of one launch.
 * k is 1 or 3; h, w <= 8192; c_in, c_out <= 65536; anything else is IODF_E_ARG.
 * Measurement support, not part of the coding path.
 */
int iodf_conv_probe(int device_ordinal, int c_in, int c_out, int k, int h, int w, int batch, int relu,
                    const int8_t* x_host, const int8_t* w_host, const int32_t* bias_host, const int32_t* m_host,
                    const uint8_t* shift_host, int8_t* y_host, int iters, float* us_per_call);

/*
 * iodf_conv_probe plus a per-tile timeline of one more launch that follows `iters` further back-to-back
 * launches (so it sees the clocks of sustained work). timeline_host: int64 [max_tiles][8], one row per
 * output tile that ran (*n_tiles rows): [0..3] the constant 100 MHz counter when the tile's workgroup
 * started on it, when its first k-tile had landed, after its k loop and after its epilogue; [4], [5] the
 * shader-clock counter at start and end, so (row[5] - row[4]) / (row[3] - row[0]) x 100 MHz is the clock the
 * compute unit ran at; [6], [7] zero. Split launches (a last layer cut along K) are not traced.
 * Measurement support for the roofline analysis, not part of the coding path.
 */
int iodf_conv_probe_timeline(int device_ordinal, int c_in, int c_out, int k, int h, int w, int batch, int relu,
                             const int8_t* x_host, const int8_t* w_host, const int32_t* bias_host,
                             const int32_t* m_host, const uint8_t* shift_host, int8_t* y_host, int iters,
                             float* us_per_call, int64_t* timeline_host, int max_tiles, int* n_tiles);

/*
 * Per-kernel timing for roofline reports (the paper reports latency only, Sec. 5.2; this is
 * measurement support, not part of the method). Between begin and end every kernel launch of
 * iodf_forward / iodf_inverse is bracketed by HIP events on the caller's stream (no
 * synchronisation is added). max_launches bounds the launches recorded; later ones run untimed.
 * iodf_profile_end waits for the recorded work, then fills stats (host, caller-owned, up to
 * max_stats entries, one per kernel that ran) and *n_stats.
 */
typedef struct iodf_kernel_stat {
    char name[48];      /* kernel, e.g. "k_quant_in"; a conv kernel's launches are listed per filter size:
                           "conv_igemm<256,256,2,4,4> 3x3" and "conv_igemm<256,256,2,4,4> 1x1"; entries whose
                           name starts with "view:" sum conv launches already listed (the wide layers) */
    int64_t launches;
    double total_ms;    /* sum of event-measured durations */
    int64_t macs;       /* algorithmic multiply-accumulates of those launches (kept channels, true widths) */
    int64_t bytes;      /* algorithmic bytes: live inputs + outputs (+ weights) read or written once */
    int64_t issued_macs; /* multiply-accumulates the matrix cores ran: whole tiles at padded widths (0: not a conv) */
} iodf_kernel_stat;
int iodf_profile_begin(iodf_ctx* ctx, int max_launches);
int iodf_profile_end(iodf_ctx* ctx, iodf_kernel_stat* stats, int max_stats, int* n_stats);

/* Read one IODF_Q_* quantity into *out (host). */
int iodf_query(iodf_ctx* ctx, int what, int64_t* out);

/* Release the context and its device memory. NULL is ignored. */
void iodf_free(iodf_ctx* ctx);

/* Static, NUL-terminated description of an IODF_E_* code. */
const char* iodf_strerror(int code);

/* The hipError_t value behind the most recent IODF_E_HIP on this thread (0 if none). */
int iodf_last_hip_error(void);

#ifdef __cplusplus
}
#endif
#endif
