// Bandwidth-bound passes over the flow state: pixel centring + squeeze, the
// input quantiser of a coupling network, factor-out / split (fused with the next
// level's squeeze), and their inverses (Sec. 3, Eq. 1; Sec. 5 multi-scale levels).
//
// The flow state of a level is int32, pixel-major: S[b][i][j][C]. Channel
// permutations between couplings are never applied to memory: the host composes
// them into an index map phi (logical channel -> physical channel) per coupling.
#include "flow_kernels.h"

namespace iodf {

namespace {

constexpr int TPB = 256;

// S1[b][i][j][4c+2dy+dx] = x[b][c][2i+dy][2j+dx] - 128
__global__ void k_ingest_squeeze(const uint8_t* __restrict__ x, int B, int H, int W, int32_t* __restrict__ s1) {
    const long long n = (long long)B * 3 * H * W;
    for (long long t = blockIdx.x * (long long)blockDim.x + threadIdx.x; t < n; t += (long long)gridDim.x * blockDim.x) {
        // t enumerates the source in its own order, so reads are coalesced
        const int X = (int)(t % W);
        const int Y = (int)((t / W) % H);
        const int c = (int)((t / ((long long)W * H)) % 3);
        const int b = (int)(t / ((long long)W * H * 3));
        const int h = H / 2, w = W / 2;
        const long long o = ((((long long)b * h + Y / 2) * w + X / 2) * 12) + 4 * c + 2 * (Y & 1) + (X & 1);
        s1[o] = (int)x[t] - 128;
    }
}

// x[b][c][2i+dy][2j+dx] = sat_u8(S1[b][i][j][4c+2dy+dx] + 128), counting saturations
__global__ void k_emit_x(const int32_t* __restrict__ s1, int B, int H, int W, uint8_t* __restrict__ x,
                         unsigned long long* __restrict__ errs) {
    const long long n = (long long)B * 3 * H * W;
    unsigned bad = 0;
    for (long long t = blockIdx.x * (long long)blockDim.x + threadIdx.x; t < n; t += (long long)gridDim.x * blockDim.x) {
        const int X = (int)(t % W);
        const int Y = (int)((t / W) % H);
        const int c = (int)((t / ((long long)W * H)) % 3);
        const int b = (int)(t / ((long long)W * H * 3));
        const int h = H / 2, w = W / 2;
        const long long o = ((((long long)b * h + Y / 2) * w + X / 2) * 12) + 4 * c + 2 * (Y & 1) + (X & 1);
        int v = s1[o] + 128;
        if (v < 0) { v = 0; ++bad; }
        if (v > 255) { v = 255; ++bad; }
        x[t] = (uint8_t)v;
    }
    if (bad) atomicAdd(errs, (unsigned long long)bad);
}

__device__ __forceinline__ int rq_in(int a, int M, int s) {
    long long v = (long long)a * (long long)M;
    long long half = s > 0 ? (1LL << (s - 1)) : 0LL;
    long long r = v >= 0 ? ((v + half) >> s) : -((-v + half) >> s);
    return r > 127 ? 127 : (r < -128 ? -128 : (int)r);
}

// Codes of channel c < n_a of pixel p: sat8(rq(S[p][idx[c]]; M, s)).
// xq is laid out in 64-channel planes of zero-bordered images (see conv.h): channel c of pixel
// (b, i, j) at xq[(c / 64) * plane + pos(b, i, j) * 64 + c % 64]. One thread per 4 channels; only the
// dwords that hold a real channel are written: the padding channels up to the next multiple of 64 were
// zeroed when the buffer was allocated and nothing ever writes them (every network of a level reads the
// same number of channels), which at the first level saves seven eighths of the pass's stores.
__global__ void k_quant_in(const int32_t* __restrict__ S, int npix, int h, int w, int C, const int32_t* __restrict__ idx,
                           int n_a, int M, int s, int8_t* __restrict__ xq, long long plane) {
    const int groups = (n_a + 3) / 4;
    const long long n = (long long)npix * groups;
    const int hw = h * w, W2 = w + 2, PP = (h + 2) * W2;
    for (long long t = blockIdx.x * (long long)blockDim.x + threadIdx.x; t < n; t += (long long)gridDim.x * blockDim.x) {
        const int g = (int)(t % groups);
        const int p = (int)(t / groups);
        unsigned packed = 0;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int c = g * 4 + e;
            int v = 0;
            if (c < n_a) v = rq_in(S[(long long)p * C + idx[c]], M, s);
            packed |= ((unsigned)v & 0xffu) << (8 * e);
        }
        const int c0 = g * 4;
        const int b = p / hw, q = p - b * hw, i = q / w, j = q - i * w;
        const long long pos = (long long)b * PP + (i + 1) * W2 + (j + 1);
        *(unsigned*)(xq + (long long)(c0 >> 6) * plane + pos * 64 + (c0 & 63)) = packed;
    }
}

// Split after the last coupling of a level. Logical channel c lives at physical phi[c].
// c >= c_keep: emitted into z (channel-first chunk). c < c_keep: squeezed into the next level.
__global__ void k_factor_out(const int32_t* __restrict__ S, int B, int h, int w, int C, const int32_t* __restrict__ phi,
                             int c_keep, int32_t* __restrict__ z, long long d, long long zoff,
                             int32_t* __restrict__ Snext) {
    const long long n = (long long)B * C * h * w;
    for (long long t = blockIdx.x * (long long)blockDim.x + threadIdx.x; t < n; t += (long long)gridDim.x * blockDim.x) {
        const int j = (int)(t % w);
        const int i = (int)((t / w) % h);
        const int c = (int)((t / ((long long)w * h)) % C);
        const int b = (int)(t / ((long long)w * h * C));
        const int v = S[(((long long)b * h + i) * w + j) * C + phi[c]];
        if (c >= c_keep) {
            z[(long long)b * d + zoff + ((long long)(c - c_keep) * h + i) * w + j] = v;
        } else {
            const int h2 = h / 2, w2 = w / 2;
            Snext[(((long long)b * h2 + i / 2) * w2 + j / 2) * (4 * c_keep) + 4 * c + 2 * (i & 1) + (j & 1)] = v;
        }
    }
}

// Inverse of k_factor_out: rebuild the level's state (in the layout it had after its
// last coupling) from the z chunk and the already decoded next level.
__global__ void k_unfactor(int32_t* __restrict__ S, int B, int h, int w, int C, const int32_t* __restrict__ phi,
                           int c_keep, const int32_t* __restrict__ z, long long d, long long zoff,
                           const int32_t* __restrict__ Snext) {
    const long long n = (long long)B * C * h * w;
    for (long long t = blockIdx.x * (long long)blockDim.x + threadIdx.x; t < n; t += (long long)gridDim.x * blockDim.x) {
        const int j = (int)(t % w);
        const int i = (int)((t / w) % h);
        const int c = (int)((t / ((long long)w * h)) % C);
        const int b = (int)(t / ((long long)w * h * C));
        int v;
        if (c >= c_keep) {
            v = z[(long long)b * d + zoff + ((long long)(c - c_keep) * h + i) * w + j];
        } else {
            const int h2 = h / 2, w2 = w / 2;
            v = Snext[(((long long)b * h2 + i / 2) * w2 + j / 2) * (4 * c_keep) + 4 * c + 2 * (i & 1) + (j & 1)];
        }
        S[(((long long)b * h + i) * w + j) * C + phi[c]] = v;
    }
}

// Patch p (row-major over the grid of ceil(h/H) x ceil(w/W) patches) of a planar image
// img[3][h][w]: x[p - first][c][y][x'] = img[c][py*H + y][px*W + x'], 128 outside the image.
__global__ void k_tile_patches(const uint8_t* __restrict__ img, int h, int w, int H, int W, int first, int n,
                               uint8_t* __restrict__ x) {
    const int pw = (w + W - 1) / W;
    const long long total = (long long)n * 3 * H * W;
    for (long long t = blockIdx.x * (long long)blockDim.x + threadIdx.x; t < total; t += (long long)gridDim.x * blockDim.x) {
        const int xx = (int)(t % W);
        const int yy = (int)((t / W) % H);
        const int c = (int)((t / ((long long)W * H)) % 3);
        const int p = first + (int)(t / ((long long)W * H * 3));
        const int gy = (p / pw) * H + yy, gx = (p % pw) * W + xx;
        x[t] = (gy < h && gx < w) ? img[((long long)c * h + gy) * w + gx] : (uint8_t)128;
    }
}

// Inverse: pixels of the patches that fall inside the image are written back.
__global__ void k_untile_patches(const uint8_t* __restrict__ x, int first, int n, int H, int W, uint8_t* __restrict__ img,
                                 int h, int w) {
    const int pw = (w + W - 1) / W;
    const long long total = (long long)n * 3 * H * W;
    for (long long t = blockIdx.x * (long long)blockDim.x + threadIdx.x; t < total; t += (long long)gridDim.x * blockDim.x) {
        const int xx = (int)(t % W);
        const int yy = (int)((t / W) % H);
        const int c = (int)((t / ((long long)W * H)) % 3);
        const int p = first + (int)(t / ((long long)W * H * 3));
        const int gy = (p / pw) * H + yy, gx = (p % pw) * W + xx;
        if (gy < h && gx < w) img[((long long)c * h + gy) * w + gx] = x[t];
    }
}

__global__ void k_fill_zero(unsigned* __restrict__ p, long long n_words) {
    for (long long t = blockIdx.x * (long long)blockDim.x + threadIdx.x; t < n_words; t += (long long)gridDim.x * blockDim.x)
        p[t] = 0u;
}

int grid_for(long long n) {
    long long g = (n + TPB - 1) / TPB;
    if (g > 256 * 32) g = 256 * 32;
    return g < 1 ? 1 : (int)g;
}

}  // namespace

hipError_t launch_ingest_squeeze(const uint8_t* x, int B, int H, int W, int32_t* s1, hipStream_t st) {
    if (B <= 0) return hipSuccess;
    hipLaunchKernelGGL(k_ingest_squeeze, dim3(grid_for((long long)B * 3 * H * W)), dim3(TPB), 0, st, x, B, H, W, s1);
    return hipGetLastError();
}

hipError_t launch_emit_x(const int32_t* s1, int B, int H, int W, uint8_t* x, unsigned long long* errs, hipStream_t st) {
    if (B <= 0) return hipSuccess;
    hipLaunchKernelGGL(k_emit_x, dim3(grid_for((long long)B * 3 * H * W)), dim3(TPB), 0, st, s1, B, H, W, x, errs);
    return hipGetLastError();
}

hipError_t launch_quant_in(const int32_t* S, int npix, int h, int w, int C, const int32_t* idx, int n_a, int M, int s,
                           int8_t* xq, int cpad, long long plane, hipStream_t st) {
    if (npix <= 0) return hipSuccess;
    if (cpad % 64 || n_a > cpad || h < 1 || w < 1 || npix % (h * w) ||
        plane < (long long)(npix / (h * w)) * (h + 2) * (w + 2) * 64)
        return hipErrorInvalidValue;
    hipLaunchKernelGGL(k_quant_in, dim3(grid_for((long long)npix * ((n_a + 3) / 4))), dim3(TPB), 0, st, S, npix, h, w, C,
                       idx, n_a, M, s, xq, plane);
    return hipGetLastError();
}

hipError_t launch_factor_out(const int32_t* S, int B, int h, int w, int C, const int32_t* phi, int c_keep, int32_t* z,
                             long long d, long long zoff, int32_t* Snext, hipStream_t st) {
    if (B <= 0) return hipSuccess;
    hipLaunchKernelGGL(k_factor_out, dim3(grid_for((long long)B * C * h * w)), dim3(TPB), 0, st, S, B, h, w, C, phi,
                       c_keep, z, d, zoff, Snext);
    return hipGetLastError();
}

hipError_t launch_unfactor(int32_t* S, int B, int h, int w, int C, const int32_t* phi, int c_keep, const int32_t* z,
                           long long d, long long zoff, const int32_t* Snext, hipStream_t st) {
    if (B <= 0) return hipSuccess;
    hipLaunchKernelGGL(k_unfactor, dim3(grid_for((long long)B * C * h * w)), dim3(TPB), 0, st, S, B, h, w, C, phi,
                       c_keep, z, d, zoff, Snext);
    return hipGetLastError();
}

hipError_t launch_tile_patches(const uint8_t* img, int h, int w, int H, int W, int first, int n, uint8_t* x,
                               hipStream_t st) {
    if (n <= 0) return hipSuccess;
    if (h < 1 || w < 1 || H < 1 || W < 1 || first < 0 ||
        (long long)first + n > (long long)((h + H - 1) / H) * ((w + W - 1) / W))
        return hipErrorInvalidValue;
    hipLaunchKernelGGL(k_tile_patches, dim3(grid_for((long long)n * 3 * H * W)), dim3(TPB), 0, st, img, h, w, H, W, first,
                       n, x);
    return hipGetLastError();
}

hipError_t launch_untile_patches(const uint8_t* x, int first, int n, int H, int W, uint8_t* img, int h, int w,
                                 hipStream_t st) {
    if (n <= 0) return hipSuccess;
    if (h < 1 || w < 1 || H < 1 || W < 1 || first < 0 ||
        (long long)first + n > (long long)((h + H - 1) / H) * ((w + W - 1) / W))
        return hipErrorInvalidValue;
    hipLaunchKernelGGL(k_untile_patches, dim3(grid_for((long long)n * 3 * H * W)), dim3(TPB), 0, st, x, first, n, H, W,
                       img, h, w);
    return hipGetLastError();
}

hipError_t launch_fill_zero(void* p, size_t bytes, hipStream_t st) {
    if (bytes == 0) return hipSuccess;
    if (bytes % 4) return hipErrorInvalidValue;
    hipLaunchKernelGGL(k_fill_zero, dim3(grid_for((long long)(bytes / 4))), dim3(TPB), 0, st, (unsigned*)p,
                       (long long)(bytes / 4));
    return hipGetLastError();
}

}  // namespace iodf
