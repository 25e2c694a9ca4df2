// Prior masses (Sec. 3) and the streaming rANS coder (App. A) on the GPU.
//
// Prior of one latent z with 8-bit mean code m and log-scale code l: mu = 2 m, s = 2^(l/16),
// residual r = z - mu in [-8192, 8191]. Cumulative mass of the symbols below r:
//   G(r) = (r + 8192) + floor((M - 16384) * S((2r - 1) / (2s)) / 2^30),   M = 2^24,
// i.e. one unit of floor mass per symbol plus the logistic CDF at the symbol's lower edge,
// sigma((r - 1/2) / s). S is a 3073-entry table of 2^30 * sigma at steps of 1/64 on [-24, 24],
// interpolated linearly with floor. The symbol's masses are C = G(r), F = G(r + 1) - G(r) >= 1.
//
// Coder: 64-bit state X in [2^31, 2^63), initial 2^31. Encoding a symbol first sheds the low
// 32 bits as a word if X >= F * 2^39, then X <- floor(X / F) * M + C + X mod F. Decoding reads
// the slot X mod M, finds the symbol whose [C, C + F) holds it by bisection over r, restores
// X <- F * floor(X / M) + (X mod M) - C and pulls a word back in when X < 2^31.
// A chunk's latents are dealt round-robin to 16 lanes, each an independent stream encoded
// last-to-first. The chains are serial (one thread per lane when encoding, sixteen when
// decoding), so these kernels are bound by dependent integer latency, not by memory or the
// vector units.
#include "codec_kernels.h"

#include <cmath>

namespace iodf {

void codec_make_tables(int32_t* sig, int64_t* inv) {
    for (int j = 0; j < kSigEntries; ++j) {
        const long double t = ((long double)j - 1536.0L) / 64.0L;
        // sigma(t) written so that the exponential never overflows: e^t / (1 + e^t) for t < 0
        long double s;
        if (t < 0) {
            const long double e = std::exp(t);
            s = e / (1.0L + e);
        } else {
            s = 1.0L / (1.0L + std::exp(-t));
        }
        sig[j] = (int32_t)std::llround(std::ldexp(s, kSigBits));
    }
    for (int l = -128; l <= 127; ++l) inv[l + 128] = (int64_t)std::llround(std::exp2((368.0L - (long double)l) / 16.0L));
}

namespace {

constexpr long long kMass = 1LL << kMassBits;
constexpr unsigned long long kStateLow = 1ULL << 31;
constexpr int TPB = 256;

__device__ __forceinline__ void load_sig(int* s_sig, const int32_t* sig) {
    for (int i = threadIdx.x; i < kSigEntries; i += blockDim.x) s_sig[i] = sig[i];
    __syncthreads();
}

__device__ __forceinline__ long long sigm(const int* s_sig, long long T) {
    constexpr long long tmax = 24LL << 24;
    if (T <= -tmax) return 0;
    if (T >= tmax) return 1LL << kSigBits;
    const long long u = T + tmax;
    const int j = (int)(u >> 18);
    const long long frac = u & ((1LL << 18) - 1);
    const long long a = s_sig[j], b = s_sig[j + 1];
    return a + (((b - a) * frac) >> 18);
}

__device__ __forceinline__ int cdf(const int* s_sig, int r, long long inv) {
    const long long T = (2LL * r - 1) * inv;
    return (r + kAlphaR) + (int)(((kMass - 2 * kAlphaR) * sigm(s_sig, T)) >> kSigBits);
}

// codes of latent e of chunk c of one image
__device__ __forceinline__ void codes_of(const ChunkTable& ct, int c, const int8_t* codes_img, int e, int& m, int& l) {
    if (codes_img && ct.code_off[c] >= 0) {
        m = codes_img[ct.code_off[c] + e];
        l = codes_img[ct.code_off[c] + ct.n[c] + e];
    } else {
        m = kDefaultM;
        l = kDefaultL;
    }
}

__device__ __forceinline__ int residual(int z, int m, unsigned& clamped) {
    long long r = (long long)z - 2 * m;
    if (r < -kAlphaR) { r = -kAlphaR; ++clamped; }
    if (r > kAlphaR - 1) { r = kAlphaR - 1; ++clamped; }
    return (int)r;
}

__global__ __launch_bounds__(TPB) void k_prior_cf(const CodecTables t, const ChunkTable ct, const int32_t* __restrict__ z,
                                                  long long d, const int8_t* __restrict__ codes, long long d_codes,
                                                  int batch, int32_t* __restrict__ c_out, int32_t* __restrict__ f_out,
                                                  unsigned long long* errs) {
    __shared__ int s_sig[kSigEntries];
    load_sig(s_sig, t.sig);
    unsigned clamped = 0;
    const long long total = (long long)batch * d;
    for (long long i = blockIdx.x * (long long)blockDim.x + threadIdx.x; i < total; i += (long long)gridDim.x * blockDim.x) {
        const int b = (int)(i / d);
        const long long q = i - (long long)b * d;
        int c = 0;
        while (c + 1 < ct.n_chunks && q >= ct.z_off[c + 1]) ++c;
        const int e = (int)(q - ct.z_off[c]);
        int m, l;
        codes_of(ct, c, codes ? codes + (long long)b * d_codes : nullptr, e, m, l);
        const int r = residual(z[i], m, clamped);
        const long long inv = t.inv[l + 128];
        const int C = cdf(s_sig, r, inv);
        c_out[i] = C;
        f_out[i] = cdf(s_sig, r + 1, inv) - C;
    }
    if (clamped) atomicAdd(errs, (unsigned long long)clamped);
}

__global__ __launch_bounds__(TPB) void k_rans_encode(const CodecTables t, const ChunkTable ct,
                                                     const int32_t* __restrict__ z, long long d,
                                                     const int8_t* __restrict__ codes, long long d_codes, int batch,
                                                     uint32_t* __restrict__ lane_words, long long lwpi,
                                                     uint32_t* __restrict__ lane_meta, unsigned long long* errs) {
    __shared__ int s_sig[kSigEntries];
    load_sig(s_sig, t.sig);
    const int nslots = ct.n_chunks * kLanes;
    const long long tid = blockIdx.x * (long long)blockDim.x + threadIdx.x;
    if (tid >= (long long)batch * nslots) return;
    const int b = (int)(tid / nslots), s = (int)(tid - (long long)b * nslots);
    const int c = s / kLanes, j = s % kLanes;
    const int n = ct.n[c];
    const int k = j < n ? (n - j + kLanes - 1) / kLanes : 0;
    const int32_t* zc = z + (long long)b * d + ct.z_off[c];
    const int8_t* ci = codes ? codes + (long long)b * d_codes : nullptr;
    uint32_t* w = lane_words + (long long)b * lwpi + ct.lane_off[c] + (long long)j * ct.lane_cap[c];
    unsigned long long X = kStateLow;
    unsigned clamped = 0;
    int nw = 0;
    for (int p = k - 1; p >= 0; --p) {
        const int e = p * kLanes + j;
        int m, l;
        codes_of(ct, c, ci, e, m, l);
        const int r = residual(zc[e], m, clamped);
        const long long inv = t.inv[l + 128];
        const unsigned C = (unsigned)cdf(s_sig, r, inv);
        const unsigned F = (unsigned)cdf(s_sig, r + 1, inv) - C;
        if (X >= ((unsigned long long)F << 39)) {  // at most once per symbol, so nw <= k < lane_cap
            w[nw++] = (uint32_t)X;
            X >>= 32;
        }
        const unsigned long long q = X / F;
        X = q * (unsigned long long)kMass + C + (X - q * F);
    }
    uint32_t* mt = lane_meta + ((long long)b * nslots + s) * 4;
    mt[0] = (uint32_t)nw;
    mt[1] = (uint32_t)X;
    mt[2] = (uint32_t)(X >> 32);
    mt[3] = 0;
    if (clamped) atomicAdd(errs, (unsigned long long)clamped);
}

// One workgroup per image. Container: [0] total words; [1 .. 1 + S) words per lane slot;
// then S pairs (state low, state high); then every slot's words in the order the decoder
// reads them (the reverse of the order they were shed). S = n_chunks * 16.
__global__ __launch_bounds__(TPB) void k_rans_pack(const ChunkTable ct, const uint32_t* __restrict__ lane_words,
                                                   long long lwpi, const uint32_t* __restrict__ lane_meta,
                                                   uint32_t* __restrict__ out, long long cap,
                                                   uint32_t* __restrict__ sizes, unsigned long long* errs) {
    __shared__ long long s_off[kMaxChunks * kLanes + 1];
    const int b = blockIdx.x;
    const int nslots = ct.n_chunks * kLanes;
    const long long header = 1 + 3LL * nslots;
    const uint32_t* mt = lane_meta + (long long)b * nslots * 4;
    if (threadIdx.x == 0) {
        long long o = 0;
        for (int s = 0; s < nslots; ++s) { s_off[s] = o; o += mt[4 * s]; }
        s_off[nslots] = o;
    }
    __syncthreads();
    const long long total = header + s_off[nslots];
    uint32_t* ob = out + (long long)b * cap;
    if (threadIdx.x == 0) {
        sizes[b] = (uint32_t)total;
        if (cap > 0) ob[0] = (uint32_t)total;
        if (total > cap) atomicAdd(errs + 1, 1ULL);
    }
    for (int s = threadIdx.x; s < nslots; s += blockDim.x) {
        if (1 + s < cap) ob[1 + s] = mt[4 * s];
        if (1 + nslots + 2 * s < cap) ob[1 + nslots + 2 * s] = mt[4 * s + 1];
        if (1 + nslots + 2 * s + 1 < cap) ob[1 + nslots + 2 * s + 1] = mt[4 * s + 2];
    }
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, nwaves = blockDim.x >> 6;
    for (int s = wave; s < nslots; s += nwaves) {
        const int c = s / kLanes, j = s % kLanes;
        const long long nw = mt[4 * s];
        const uint32_t* w = lane_words + (long long)b * lwpi + ct.lane_off[c] + (long long)j * ct.lane_cap[c];
        for (long long i = lane; i < nw; i += 64) {
            const long long dst = header + s_off[s] + i;
            if (dst < cap) ob[dst] = w[nw - 1 - i];
        }
    }
}

// Sixteen threads serve one lane: each bisection round they test sixteen cut points of the current
// interval at once (a ballot counts how many lie at or below the slot), so the 2^14 residuals are
// isolated in four rounds (16 * 16 * 16 * 4) instead of fourteen. All sixteen keep the same coder
// state; thread 0 of the group writes the latent. A workgroup of 256 threads holds the 16 lanes of
// one image's chunk.
__global__ __launch_bounds__(256) void k_rans_decode_chunk(const CodecTables t, const ChunkTable ct, const int c,
                                                           const uint32_t* __restrict__ cont, long long cap, int batch,
                                                           const int8_t* __restrict__ codes, long long d_codes,
                                                           int32_t* __restrict__ z, long long d,
                                                           unsigned long long* errs) {
    __shared__ int s_sig[kSigEntries];
    load_sig(s_sig, t.sig);
    const int b = blockIdx.x;  // grid = batch
    const int j = threadIdx.x >> 4, helper = threadIdx.x & 15;
    const int grp_shift = (threadIdx.x & 63) & ~15;  // this group's first bit in the wave's ballot
    const int nslots = ct.n_chunks * kLanes;
    const long long header = 1 + 3LL * nslots;  // the host has checked cap >= header
    const uint32_t* cb = cont + (long long)b * cap;
    const int n = ct.n[c];
    const int k = j < n ? (n - j + kLanes - 1) / kLanes : 0;
    const int kmax = (n + kLanes - 1) / kLanes;  // the same for every thread: ballots stay convergent
    int32_t* zc = z + (long long)b * d + ct.z_off[c];
    const int8_t* ci = codes ? codes + (long long)b * d_codes : nullptr;
    const long long total = cb[0];
    bool bad = total > cap || total < header;
    long long pos = header;
    const int slot = c * kLanes + j;
    for (int s = 0; s < slot; ++s) pos += cb[1 + s];
    long long nw = cb[1 + slot];
    if (bad || pos + nw > total) { bad = true; nw = 0; pos = header; }
    const uint32_t* w = cb + pos;  // reads stay below pos + nw <= total <= cap
    long long used = 0;
    unsigned long long X = (unsigned long long)cb[1 + nslots + 2 * slot] |
                           ((unsigned long long)cb[1 + nslots + 2 * slot + 1] << 32);
    for (int p = 0; p < kmax; ++p) {
        const bool active = p < k;
        const int e = active ? p * kLanes + j : 0;
        int m = kDefaultM, l = kDefaultL;
        if (active) codes_of(ct, c, ci, e, m, l);
        const long long inv = t.inv[l + 128];
        const int v = (int)(X & (unsigned long long)(kMass - 1));
        // G(-8192) = 0 <= v < M = G(8192); cut points lo + (helper + 1) * step, the last one of the
        // first three rounds is the interval's end (known to lie above the slot)
        int lo = -kAlphaR;
#pragma unroll
        for (int round = 0; round < 4; ++round) {
            const int step = round == 0 ? 1024 : round == 1 ? 64 : round == 2 ? 4 : 1;
            const int cut = lo + (helper + 1) * step;
            const bool below = (step == 1 ? helper < 3 : helper < 15) && cdf(s_sig, cut, inv) <= v;
            const unsigned long long mask = __ballot(below);
            lo += __popc((unsigned)(mask >> grp_shift) & 0xffffu) * step;
        }
        const int C = cdf(s_sig, lo, inv);
        const int F = cdf(s_sig, lo + 1, inv) - C;
        if (active) {
            if (helper == 0) zc[e] = lo + 2 * m;
            X = (unsigned long long)F * (X >> kMassBits) + (unsigned long long)(v - C);
            if (X < kStateLow) {
                if (used < nw) X = (X << 32) | w[used++];
                else { X <<= 32; bad = true; }
            }
        }
    }
    if (X != kStateLow || used != nw) bad = true;
    if (bad && helper == 0) atomicAdd(errs + 2, 1ULL);
}

int grid_for(long long n, int tpb) {
    long long g = (n + tpb - 1) / tpb;
    if (g > 256 * 16) g = 256 * 16;
    return g < 1 ? 1 : (int)g;
}

bool table_ok(const ChunkTable& ct) { return ct.n_chunks >= 1 && ct.n_chunks <= kMaxChunks; }

}  // namespace

hipError_t launch_prior_cf(const CodecTables& t, const ChunkTable& ct, const int32_t* z, long long d,
                           const int8_t* codes, long long d_codes, int batch, int32_t* c_out, int32_t* f_out,
                           unsigned long long* errs, hipStream_t st) {
    if (batch <= 0) return hipSuccess;
    if (!table_ok(ct) || !z || !c_out || !f_out || !errs || !t.sig || !t.inv) return hipErrorInvalidValue;
    hipLaunchKernelGGL(k_prior_cf, dim3(grid_for((long long)batch * d, TPB)), dim3(TPB), 0, st, t, ct, z, d, codes, d_codes,
                       batch, c_out, f_out, errs);
    return hipGetLastError();
}

hipError_t launch_rans_encode(const CodecTables& t, const ChunkTable& ct, const int32_t* z, long long d,
                              const int8_t* codes, long long d_codes, int batch, uint32_t* lane_words,
                              long long lane_words_per_image, uint32_t* lane_meta, unsigned long long* errs,
                              hipStream_t st) {
    if (batch <= 0) return hipSuccess;
    if (!table_ok(ct) || !z || !lane_words || !lane_meta || !errs || !t.sig || !t.inv) return hipErrorInvalidValue;
    const long long threads = (long long)batch * ct.n_chunks * kLanes;
    hipLaunchKernelGGL(k_rans_encode, dim3((unsigned)((threads + TPB - 1) / TPB)), dim3(TPB), 0, st, t, ct, z, d, codes,
                       d_codes, batch, lane_words, lane_words_per_image, lane_meta, errs);
    return hipGetLastError();
}

hipError_t launch_rans_pack(const ChunkTable& ct, const uint32_t* lane_words, long long lane_words_per_image,
                            const uint32_t* lane_meta, int batch, uint32_t* out, long long cap, uint32_t* sizes,
                            unsigned long long* errs, hipStream_t st) {
    if (batch <= 0) return hipSuccess;
    if (!table_ok(ct) || !lane_words || !lane_meta || !out || !sizes || !errs || cap < 0) return hipErrorInvalidValue;
    hipLaunchKernelGGL(k_rans_pack, dim3(batch), dim3(TPB), 0, st, ct, lane_words, lane_words_per_image, lane_meta, out,
                       cap, sizes, errs);
    return hipGetLastError();
}

hipError_t launch_rans_decode_chunk(const CodecTables& t, const ChunkTable& ct, int c, const uint32_t* cont,
                                    long long cap, int batch, const int8_t* codes, long long d_codes, int32_t* z,
                                    long long d, unsigned long long* errs, hipStream_t st) {
    if (batch <= 0) return hipSuccess;
    if (!table_ok(ct) || c < 0 || c >= ct.n_chunks || !cont || !z || !errs || !t.sig || !t.inv ||
        cap < 1 + 3LL * ct.n_chunks * kLanes)
        return hipErrorInvalidValue;
    hipLaunchKernelGGL(k_rans_decode_chunk, dim3(batch), dim3(256), 0, st, t, ct, c, cont, cap, batch, codes, d_codes, z,
                       d, errs);
    return hipGetLastError();
}

}  // namespace iodf
