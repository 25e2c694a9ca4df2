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

// Split after the last coupling of a level (factor-out fused with the next level's squeeze). Logical
// channel c lives at physical phi[c]. c >= c_keep: emitted into z (channel-first chunk). c < c_keep:
// squeezed into the next level, Snext[b][i/2][j/2][4c + 2(i&1) + (j&1)].
//
// The state is pixel-major and both outputs are not, so a direct copy is strided on one side. A workgroup
// instead takes a tile of two image rows x jw columns through LDS: it reads the tile's 2 * jw * C words as two
// contiguous runs, then writes z in runs of jw words per (channel, row) and the next level's pixels, each
// 4 * c_keep contiguous words that two rows and two columns of this level make up, in one contiguous run
// per tile. Rows of the LDS tile are padded by one word so that a column walk does not stay on one bank.
struct SplitGeom {
    int B, h, w, C, c_keep, jw, tiles_j, tiles_i;
    long long d, zoff;
};

__device__ __forceinline__ void split_tile(const SplitGeom& g, long long tile, int& b, int& i0, int& j0, int& rows, int& cols) {
    const int tj = (int)(tile % g.tiles_j);
    const long long q = tile / g.tiles_j;
    const int ti = (int)(q % g.tiles_i);
    b = (int)(q / g.tiles_i);
    i0 = 2 * ti;
    j0 = tj * g.jw;
    rows = g.h - i0 < 2 ? g.h - i0 : 2;
    cols = g.w - j0 < g.jw ? g.w - j0 : g.jw;
}

__global__ __launch_bounds__(TPB) void k_factor_out(const int32_t* __restrict__ S, const SplitGeom g,
                                                    const int32_t* __restrict__ phi, int32_t* __restrict__ z,
                                                    int32_t* __restrict__ Snext) {
    extern __shared__ int32_t tile_lds[];  // [2][jw][C + 1]
    const int C = g.C, C1 = C + 1;
    const long long ntiles = (long long)g.B * g.tiles_i * g.tiles_j;
    for (long long tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
        int b, i0, j0, rows, cols;
        split_tile(g, tile, b, i0, j0, rows, cols);
        const int run = cols * C;
        for (int t = threadIdx.x; t < rows * run; t += TPB) {
            const int rr = t / run, rem = t - rr * run;
            const int jj = rem / C, pc = rem - jj * C;
            tile_lds[(rr * g.jw + jj) * C1 + pc] = S[(((long long)b * g.h + i0 + rr) * g.w + j0) * C + rem];
        }
        __syncthreads();
        // emitted channels: runs of `cols` words per (channel, row)
        const int ce = C - g.c_keep;
        for (int t = threadIdx.x; t < ce * rows * cols; t += TPB) {
            const int jj = t % cols, q = t / cols;
            const int rr = q % rows, c = q / rows;
            z[(long long)b * g.d + g.zoff + ((long long)c * g.h + i0 + rr) * g.w + j0 + jj] =
                tile_lds[(rr * g.jw + jj) * C1 + phi[g.c_keep + c]];
        }
        // kept channels: next-level pixel (i0/2, (j0+jj)/2) holds 4*c_keep consecutive words
        if (g.c_keep > 0) {
            const int per = 4 * g.c_keep, npx = cols / 2;
            int32_t* dst = Snext + (((long long)b * (g.h / 2) + i0 / 2) * (g.w / 2) + j0 / 2) * per;
            for (int t = threadIdx.x; t < npx * per; t += TPB) {
                const int px = t / per, k = t - px * per;
                const int c = k >> 2, rr = (k >> 1) & 1, jb = k & 1;
                dst[t] = tile_lds[(rr * g.jw + 2 * px + jb) * C1 + phi[c]];
            }
        }
        __syncthreads();
    }
}

// Inverse of k_factor_out: rebuild the level's state (in the layout it had after its last coupling) from
// the z chunk and the already decoded next level; same tiles, the other way round.
__global__ __launch_bounds__(TPB) void k_unfactor(int32_t* __restrict__ S, const SplitGeom g,
                                                  const int32_t* __restrict__ phi, const int32_t* __restrict__ z,
                                                  const int32_t* __restrict__ Snext) {
    extern __shared__ int32_t tile_lds[];
    const int C = g.C, C1 = C + 1;
    const long long ntiles = (long long)g.B * g.tiles_i * g.tiles_j;
    for (long long tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
        int b, i0, j0, rows, cols;
        split_tile(g, tile, b, i0, j0, rows, cols);
        const int ce = C - g.c_keep;
        for (int t = threadIdx.x; t < ce * rows * cols; t += TPB) {
            const int jj = t % cols, q = t / cols;
            const int rr = q % rows, c = q / rows;
            tile_lds[(rr * g.jw + jj) * C1 + phi[g.c_keep + c]] =
                z[(long long)b * g.d + g.zoff + ((long long)c * g.h + i0 + rr) * g.w + j0 + jj];
        }
        if (g.c_keep > 0) {
            const int per = 4 * g.c_keep, npx = cols / 2;
            const int32_t* src = Snext + (((long long)b * (g.h / 2) + i0 / 2) * (g.w / 2) + j0 / 2) * per;
            for (int t = threadIdx.x; t < npx * per; t += TPB) {
                const int px = t / per, k = t - px * per;
                const int c = k >> 2, rr = (k >> 1) & 1, jb = k & 1;
                tile_lds[(rr * g.jw + 2 * px + jb) * C1 + phi[c]] = src[t];
            }
        }
        __syncthreads();
        const int run = cols * C;
        for (int t = threadIdx.x; t < rows * run; t += TPB) {
            const int rr = t / run, rem = t - rr * run;
            const int jj = rem / C, pc = rem - jj * C;
            S[(((long long)b * g.h + i0 + rr) * g.w + j0) * C + rem] = tile_lds[(rr * g.jw + jj) * C1 + pc];
        }
        __syncthreads();
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

// Tile geometry of the split passes: two rows x jw columns, jw even and as wide as 32 KB of LDS allow.
static bool split_geom(int B, int h, int w, int C, int c_keep, long long d, long long zoff, SplitGeom& g, size_t& lds) {
    if (B <= 0 || h < 1 || w < 1 || C < 1 || c_keep < 0 || c_keep > C) return false;
    if (c_keep > 0 && ((h | w) & 1)) return false;  // a level that is squeezed further has even sides
    int jw = (32 * 1024 / 4) / (2 * (C + 1));
    jw &= ~1;
    if (jw < 2) return false;
    if (jw > w) jw = w;  // (an odd w only occurs at the last level, where nothing is paired)
    g.B = B; g.h = h; g.w = w; g.C = C; g.c_keep = c_keep; g.jw = jw;
    g.tiles_j = (w + jw - 1) / jw;
    g.tiles_i = (h + 1) / 2;
    g.d = d; g.zoff = zoff;
    lds = (size_t)2 * jw * (C + 1) * 4;
    return true;
}

hipError_t launch_factor_out(const int32_t* S, int B, int h, int w, int C, const int32_t* phi, int c_keep, int32_t* z,
                             long long d, long long zoff, int32_t* Snext, hipStream_t st) {
    if (B <= 0) return hipSuccess;
    SplitGeom g;
    size_t lds = 0;
    if (!split_geom(B, h, w, C, c_keep, d, zoff, g, lds) || (c_keep > 0 && !Snext)) return hipErrorInvalidValue;
    const long long ntiles = (long long)B * g.tiles_i * g.tiles_j;
    hipLaunchKernelGGL(k_factor_out, dim3((unsigned)(ntiles > 256 * 16 ? 256 * 16 : ntiles)), dim3(TPB), lds, st, S, g, phi, z,
                       Snext);
    return hipGetLastError();
}

hipError_t launch_unfactor(int32_t* S, int B, int h, int w, int C, const int32_t* phi, int c_keep, const int32_t* z,
                           long long d, long long zoff, const int32_t* Snext, hipStream_t st) {
    if (B <= 0) return hipSuccess;
    SplitGeom g;
    size_t lds = 0;
    if (!split_geom(B, h, w, C, c_keep, d, zoff, g, lds) || (c_keep > 0 && !Snext)) return hipErrorInvalidValue;
    const long long ntiles = (long long)B * g.tiles_i * g.tiles_j;
    hipLaunchKernelGGL(k_unfactor, dim3((unsigned)(ntiles > 256 * 16 ? 256 * 16 : ntiles)), dim3(TPB), lds, st, S, g, phi, z,
                       Snext);
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
