// Launchers of the flow-state passes (see flow_kernels.hip). All pointers are device
// memory; every call only enqueues on `st`.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace iodf {

// x u8 [B][3][H][W] -> level-1 state int32 [B][H/2][W/2][12], value - 128.
hipError_t launch_ingest_squeeze(const uint8_t* x, int B, int H, int W, int32_t* s1, hipStream_t st);
// Inverse; pixels outside [0,255] are saturated and counted into *errs.
hipError_t launch_emit_x(const int32_t* s1, int B, int H, int W, uint8_t* x, unsigned long long* errs, hipStream_t st);
// 8-bit codes of the first n_a logical channels (physical idx[c]) of state S [npix][C], npix =
// batch * h * w. xq holds cpad channels (multiple of 64) in 64-channel planes of zero-bordered
// images, `plane` bytes apart; channels >= n_a are written as 0, borders are left alone.
hipError_t launch_quant_in(const int32_t* S, int npix, int h, int w, int C, const int32_t* idx, int n_a, int M, int s,
                           int8_t* xq, int cpad, long long plane, hipStream_t st);
// Split: logical channels >= c_keep go to z (chunk at zoff, image stride d); channels < c_keep
// are squeezed into Snext [B][h/2][w/2][4*c_keep]. c_keep = 0 emits everything (last level).
hipError_t launch_factor_out(const int32_t* S, int B, int h, int w, int C, const int32_t* phi, int c_keep, int32_t* z,
                             long long d, long long zoff, int32_t* Snext, hipStream_t st);
hipError_t launch_unfactor(int32_t* S, int B, int h, int w, int C, const int32_t* phi, int c_keep, const int32_t* z,
                           long long d, long long zoff, const int32_t* Snext, hipStream_t st);
// Patch-based coding of a large image (Sec. 5.2): planar img u8 [3][h][w] <-> patches
// x u8 [n][3][H][W], patches first .. first+n-1 of the row-major grid of ceil(h/H) x ceil(w/W);
// pixels outside the image read as 128 and are dropped on the way back.
hipError_t launch_tile_patches(const uint8_t* img, int h, int w, int H, int W, int first, int n, uint8_t* x,
                               hipStream_t st);
hipError_t launch_untile_patches(const uint8_t* x, int first, int n, int H, int W, uint8_t* img, int h, int w,
                                 hipStream_t st);
// Zero `bytes` (multiple of 4) with a kernel (safe under stream capture).
hipError_t launch_fill_zero(void* p, size_t bytes, hipStream_t st);

}  // namespace iodf
