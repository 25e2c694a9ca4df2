/*
 * CPU oracle for the integer-only inference of an IODF flow (arXiv 2206.08869).
 *
 * THIS IS TEST INFRASTRUCTURE, not the product: a plain, slow, full-width,
 * channel-first implementation in naive loops, used to check the GPU library
 * and timed as a reported CPU baseline. It shares no code, header or table with
 * the GPU path and never compacts gated channels (it masks them).
 *
 * Passages followed: additive coupling (Sec. 3, Eq. 1), integer-only residual
 * block (Sec. 4.1, Eq. 2), hybrid number format (Eq. 3), integer-only
 * convolution with 32-bit accumulator and bias and 8-bit re-quantised outputs
 * (Eq. 4-5 and the paragraph after Eq. 5), integer-only ReLU (Sec. 4.1), binary
 * gated convolution and scatter-add shortcut (Sec. 4.4, Eq. 8), flow macro
 * architecture (Sec. 5, App. B.1).
 *
 * Pins (tests, CPU only): hand-worked requantisation table, brute-force and
 * library convolutions, the asymmetric-kernel example, exact invertibility,
 * closed forms for t == 0 and bias-only t, gate masking == manual row/column
 * deletion, per-image independence, the state bound.
 * Parity unpinned: the prior-parameter heads have no pin of their own beyond
 * being the same convolution stack; the calibration constants are the blob's.
 */
#ifndef IODF_ORACLE_H
#define IODF_ORACLE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct orc_model orc_model;

/* Worker threads used inside a convolution (over output channels). 0 = all cores. */
void orc_set_threads(int n);
int orc_get_threads(void);

/* Requantise: round-half-away-from-zero of a * M / 2^s, in 64-bit. 0 <= s <= 62. */
int64_t orc_rq(int32_t a, int32_t M, int s);
/* Saturate to [-128, 127]. */
int32_t orc_sat8(int64_t u);

/* Eq. 4: acc[c,i,j] = bias[c] + sum_{c',ky,kx} W[c,c',ky,kx] * x[c',i+ky-p,j+kx-p],
 * cross-correlation, zero padding p=(k-1)/2, stride 1; x is [D,h,w], W is
 * [C,D,k,k], acc is [C,h,w] (32-bit). gate may be NULL; a gated-off channel's
 * accumulator is left untouched (its output is defined as 0 by the epilogue). */
void orc_conv_acc(const int8_t* x, int D, int h, int w, const int8_t* W, int C, int k,
                  const int32_t* bias, const uint8_t* gate, int32_t* acc);

/* The same with the input read as unsigned codes 0..255 (Eq. 3: the hybrid format keeps signed
 * 8-bit weights and may use unsigned 8-bit activations). */
void orc_conv_acc_u8(const uint8_t* x, int D, int h, int w, const int8_t* W, int C, int k,
                     const int32_t* bias, const uint8_t* gate, int32_t* acc);

/* Epilogue of one conv layer: y = sat8(relu?((gate ? rq(acc; M_c, s_c) : 0) + shortcut?)). */
void orc_epilogue(const int32_t* acc, int C, int hw, const int32_t* M, const uint8_t* shift,
                  const uint8_t* gate, int relu, const int8_t* shortcut, int8_t* y);

/* Unsigned format: y = min(255, relu((gate ? rq(acc) : 0) + shortcut?)), shortcut and y unsigned.
 * A model whose blob header sets the unsigned flag stores every tensor that leaves a ReLU this
 * way; tensors without a ReLU (the input quantiser's, the translation, the head codes) stay signed. */
void orc_epilogue_u8(const int32_t* acc, int C, int hw, const int32_t* M, const uint8_t* shift,
                     const uint8_t* gate, const uint8_t* shortcut, uint8_t* y);

/* Space-to-depth 2x2: out[4c+2dy+dx, i, j] = in[c, 2i+dy, 2j+dx]; and its inverse. */
void orc_squeeze(const int32_t* in, int C, int H, int W, int32_t* out);
void orc_unsqueeze(const int32_t* in, int C, int H, int W, int32_t* out); /* in [4C,H/2,W/2] -> out [C,H,W] */

/* Model blob (host memory, copied). Returns 0 or a negative error. */
int orc_model_load(const void* blob, size_t bytes, orc_model** out);
void orc_model_free(orc_model* m);
int orc_model_num_nets(const orc_model* m);
int64_t orc_model_d(const orc_model* m);        /* z elements per image */
int64_t orc_model_d_codes(const orc_model* m);  /* code bytes per image */

/* One network (coupling t() or head) on one image: xa [C_in,h,w] int32 is passed
 * through the input quantiser, then the conv stack; out [C_out,h,w] int8. */
int orc_net_eval(const orc_model* m, int net, const int32_t* xa, int h, int w, int8_t* out);

/* Encode: x [B,3,H,W] u8 -> z [B,d] int32, codes [B,d_codes] int8 (codes may be NULL). */
int orc_forward(const orc_model* m, const uint8_t* x, int batch, int32_t* z, int8_t* codes);
/* Decode: z -> x. Values outside [0,255] are saturated and counted in *range_errors. */
int orc_inverse(const orc_model* m, const int32_t* z, int batch, uint8_t* x, int64_t* range_errors);
/* Largest |flow state| seen by the last orc_forward call (for the state bound). */
int64_t orc_last_max_abs_state(void);

/* Compressor built on the flow (Sec. 3, Sec. 5.2, App. A; coder and prior in
 * iodf_codec_oracle.h): x -> one container of 32-bit words per image, written at
 * out + b * cap (at most cap words each); sizes[b] = words the container needs.
 * *n_clamped counts latents whose residual fell outside the prior's alphabet. */
int64_t orc_codec_max_words(const orc_model* m);
int orc_encode(const orc_model* m, const uint8_t* x, int batch, uint32_t* out, int64_t cap, uint32_t* sizes,
               int64_t* n_clamped);
/* Containers -> x. *errors counts malformed lanes and pixels outside [0,255]. */
int orc_decode(const orc_model* m, const uint32_t* cont, int64_t cap, int batch, uint8_t* x, int64_t* errors);

#ifdef __cplusplus
}
#endif
#endif
