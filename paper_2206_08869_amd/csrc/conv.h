// Launch description of one integer-only convolution layer (Sec. 4.1, Eq. 4-5)
// as an implicit GEMM on the int8 matrix cores of gfx950.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace iodf {

enum ConvMode : int {
    MODE_ACT = 0,     // write 8-bit codes, pixel-major (NHWC), optionally + shortcut, ReLU
    MODE_COUPLE = 1,  // last layer of t(): state[b-half] += sign * sat8(rq(acc))   (Eq. 1)
    MODE_CODES = 2,   // last layer of a prior head: write int8 codes channel-first
    MODE_RAW = 3      // store the 32-bit accumulators plus bias[] (no requantise) to `partial` [npix][n_pad]
};

// Second phase of a tap-expanded 3x3 last layer. A 3x3 convolution with few output channels is
// computed as ONE 1x1 GEMM with 9 * c_out rows (row t * c_out + c holds tap t of channel c; its
// raw accumulators go to y), which reads the wide input once instead of nine times; this pass
// then sums, for output pixel (i, j), the nine maps at their shifted positions
//   acc[c](i, j) = sum_t y[(i + ky - 1, j + kx - 1)][t * c_out + c]   (zero outside the image)
// adds the bias, requantises and applies the layer's mode (coupling add or head codes).
struct TapSumArgs {
    const int32_t* y;  // [npix][n_pad]
    int n_pad, c_out, h, w, npix;
    const int32_t* bias;   // [c_out]
    const int32_t* mul;    // [c_out]
    const int32_t* shift;  // [c_out], the full shift
    int mode, relu;
    int32_t* state; int state_c; const int32_t* idx_b; int sign;          // MODE_COUPLE
    int8_t* codes; long long codes_img_stride; long long codes_off;       // MODE_CODES
};
hipError_t launch_tapsum(const TapSumArgs& a, hipStream_t stream);

// The structure is the kernels' argument block, and a launch costs about 0.2 us more for every 64 bytes of
// it (measured on chains of small launches): hence the narrow types, the bit fields and the overlaid
// output fields. 120 bytes.
struct ConvArgs {
    // Activation tensors are int8 in 64-channel planes of zero-bordered images: pixel (b, i, j),
    // channel c lives at
    //   base[(chunk0 + c / 64) * plane + pos(b, i, j) * 64 + c % 64],
    //   pos(b, i, j) = b * (h + 2) * (w + 2) + (i + 1) * (w + 2) + (j + 1),
    // plane = bytes between planes (a fixed property of the buffer, >= batch * (h+2) * (w+2) * 64, < 2^31).
    // The 64-byte k-chunks of consecutive pixels are contiguous (whole cache lines per tile load),
    // a channel concatenation is a range of planes, and the border positions hold code 0 (byte 0; byte
    // -128 for tensors of unsigned codes, see out_unsigned) that nobody ever overwrites: they are the
    // convolution's zero padding.
    const int8_t* in;
    // weights: int8 [cin_pad / 64][taps][n_pad][64]: k-tile major (64-channel plane, then tap), so a
    // [channels][64] tile is contiguous and the taps of one plane follow each other
    const int8_t* wgt;
    // per output channel constants, length n_pad
    const int32_t* bias;
    const int32_t* mul;
    const int32_t* shift;  // rq_fast: shift - 32 (every shift of the layer is >= 33); else the shift itself
    // rq_fast only: smallest accumulator (bias included) whose requantised value reaches the top code
    // (127, or 255 with out_unsigned), saturated to INT32_MAX; lets a ReLU layer clamp before the multiply instead of after it
    const int32_t* clamp_hi;
    int32_t* partial;  // optional split-K scratch: int32 [npix][n_pad], all zero between launches
    union {
        // Optional: memory the next launch will read first (its packed weights and constants, pf_bytes of
        // them). A launch with a handful of tiles adds a few workgroups that touch it, one load per cache
        // line, so that it sits in the L2 of the XCDs that hold tiles when that launch starts.
        const int8_t* pf;
        // Optional per-tile timeline (measurement support; has_trace = 1): the first wave of a workgroup writes,
        // for the output tile in slot s, trace[8 s + 0..3] = the constant 100 MHz counter at tile start, after its
        // first k-tile landed, after the k loop and after the epilogue; [4], [5] = the shader-clock counter at
        // tile start and end. Slots are numbered as blockIdx.x of the plain kernel numbers them.
        long long* trace;
    };
    // What the epilogue writes depends on the mode, and only that mode's fields are read: they share storage.
    union {
        struct {  // MODE_ACT
            int8_t* out;
            unsigned out_plane;
            unsigned short out_chunk0;
            unsigned short shortcut;  // add the 8-bit code already stored at the output location
        };
        struct {  // MODE_COUPLE
            int32_t* state;          // int32 pixel-major [npix][state_c]
            const int32_t* idx_b;    // physical channel of translation channel n
        };
        struct {  // MODE_CODES
            int8_t* codes;           // image b, channel n, pixel q at codes[b * codes_img_stride + codes_off + n * h*w + q]
            unsigned codes_img_stride;
            unsigned codes_off;
        };
    };
    unsigned in_plane;
    unsigned pf_bytes;
    int npix;      // batch * h * w
    int cin_pad;   // channels read per tap, multiple of 64 (padding columns have zero weights)
    int n_pad;     // multiple of 64; rows n >= true C_out are zero
    int n_store;   // channels written (<= n_pad); multiple of 4 in MODE_ACT
    int state_c;
    unsigned short in_chunk0;
    unsigned short h, w;  // feature map size
    unsigned short n_cu;  // compute units of the device the layer runs on (conv_device_cus); decides the launch shape
    unsigned taps : 4;    // 1 (1x1) or 9 (3x3, pad 1, stride 1)
    unsigned rq_fast : 1;
    unsigned relu : 1;
    // Unsigned codes (0..255, stored as code - 128): out_unsigned saturates MODE_ACT results to [0, 255]
    // (the layer then has a ReLU); sc_unsigned says the shortcut bytes are such codes.
    unsigned out_unsigned : 1, sc_unsigned : 1;
    unsigned mode : 3;
    unsigned has_trace : 1;
    int sign : 2;        // +1 encode, -1 decode
    int log2_w : 6, log2_hw : 8;  // filled by launch_conv: log2 of w and of h*w when both are powers of two, else -1
};
static_assert(sizeof(ConvArgs) == 120, "argument block");


// Enqueue the layer on `stream`. Returns hipSuccess or the launch error.
hipError_t launch_conv(const ConvArgs& a, hipStream_t stream);
// Index of the kernel configuration launch_conv picks for `a` (-1: invalid arguments; the last index
// stands for the persistent form of the first tile), the number of configurations, and a printable
// name ("conv_igemm<256,256,2,4,4>").
int conv_pick_tile(const ConvArgs& a);
int conv_num_tiles();
const char* conv_tile_name(int tile);
// Timeline slots launch_conv would use for `a` (see ConvArgs::trace): 8 x int64 each; 0 for invalid arguments.
int conv_trace_slots(const ConvArgs& a);
// Channels x pixels of a tile (0, 0 for an invalid index).
void conv_tile_dims(int tile, int* bc, int* bp);
// Set-up of kernel attributes (dynamic LDS sizes) on the current device.
hipError_t conv_setup();
// Compute units of the current device.
hipError_t conv_device_cus(int* n_cu);

}  // namespace iodf
