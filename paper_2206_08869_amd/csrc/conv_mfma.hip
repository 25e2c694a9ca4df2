// Integer-only convolution (Sec. 4.1, Eq. 4-5) as an implicit GEMM on the gfx950
// int8 matrix cores, with the fixed-point requantise / ReLU / shortcut / coupling
// epilogue fused in.
//
// GEMM view: D[channel][pixel] = sum_k Wgt[channel][k] * Act[k][pixel], k = (tap, c).
// Output channels are the MFMA "A" rows and pixels the "B" columns, so that after
// v_mfma_i32_32x32x32_i8 every lane owns 4 consecutive channels of one pixel per
// register quad: the 8-bit results pack into dword stores along the channel axis of
// the pixel-major activation tensor.
//
// A workgroup computes BC channels x BP pixels. Per 64-byte k-tile it stages a
// [BC][64] weight tile and a [BP][64] activation tile in LDS (row stride 80 bytes,
// which makes the 16-byte fragment reads of 16 consecutive rows bank-conflict free),
// double buffered: the global loads of tile k+1 are in flight while tile k feeds
// the matrix cores. For 3x3 layers the activation tile of tap (ky,kx) is the tile of
// the pixels shifted by (ky-1, kx-1); out-of-image taps are staged as zeros.
#include "conv.h"

#include <stdlib.h>

#include <type_traits>

namespace iodf {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

// Compile-time loop: f(std::integral_constant<int, I>) for I = 0..N-1. Keeps every
// accumulator index a constant so the accumulators stay in registers.
template <int I, int N, class F>
__device__ __forceinline__ void static_for_impl(F&& f) {
    if constexpr (I < N) {
        f(std::integral_constant<int, I>{});
        static_for_impl<I + 1, N>(f);
    }
}
template <int N, class F>
__device__ __forceinline__ void static_for(F&& f) {
    static_for_impl<0, N>(f);
}

constexpr int KT = 64;    // bytes (= int8 values) of K per staged tile
constexpr int ROWB = 80;  // LDS row stride in bytes

// Round-half-away-from-zero of acc * M / 2^s, clamped far outside the 8-bit range
// (the caller saturates to 8 bit after adding at most one 8-bit shortcut).
__device__ __forceinline__ int rq_dev(int acc, int M, int s) {
    long long v = (long long)acc * (long long)M;
    long long half = s > 0 ? (1LL << (s - 1)) : 0LL;
    long long r = v >= 0 ? ((v + half) >> s) : -((-v + half) >> s);
    r = r > (1 << 20) ? (1 << 20) : r;
    r = r < -(1 << 20) ? -(1 << 20) : r;
    return (int)r;
}

__device__ __forceinline__ int sat8_dev(int v) { return v > 127 ? 127 : (v < -128 ? -128 : v); }

template <int BC, int BP, int WC, int WP>
__global__ __launch_bounds__(WC* WP * 64) void conv_igemm(const ConvArgs a, const int npb, const int ncb) {
    constexpr int NT = WC * WP * 64;
    constexpr int WTC = BC / WC, WTP = BP / WP;  // wave tile
    constexpr int TC = WTC / 32, TP = WTP / 32;  // 32x32 MFMA tiles per wave
    constexpr int WU = BC * 4 / NT, AU = BP * 4 / NT;  // 16-byte chunks per thread per k-tile
    constexpr int STAGE = (BC + BP) * ROWB;
    static_assert(WTC % 32 == 0 && WTP % 32 == 0, "wave tile must be a multiple of 32x32");
    static_assert((BC * 4) % NT == 0 && (BP * 4) % NT == 0, "tile rows must divide over the threads");

    extern __shared__ __align__(16) unsigned char lds[];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wc = wave % WC, wp = wave / WC;

    // Workgroups are dealt round-robin to the 8 XCDs. Give each XCD whole pixel
    // blocks (all their channel blocks), so an activation tile is fetched into one L2 only.
    const int bid = blockIdx.x;
    const int xcd = bid & 7, slot = bid >> 3;
    const int pb = (slot / ncb) * 8 + xcd, cb = slot % ncb;
    if (pb >= npb) return;
    const int p0 = pb * BP, c0 = cb * BC;

    const int cpt = a.cin_pad / KT;  // k-tiles per tap
    const int nkt = a.taps * cpt;
    const long long wrow = (long long)nkt * KT;  // bytes per weight row
    const int hw = a.h * a.w;

    const int part = tid & 3;
    const int8_t* wptr[WU];
    int wlds[WU];
#pragma unroll
    for (int u = 0; u < WU; ++u) {
        const int row = (tid >> 2) + u * (NT / 4);
        wptr[u] = a.wgt + (long long)(c0 + row) * wrow + part * 16;
        wlds[u] = row * ROWB + part * 16;
    }
    long long abase[AU];
    unsigned amask[AU];
    int alds[AU];
#pragma unroll
    for (int u = 0; u < AU; ++u) {
        const int row = (tid >> 2) + u * (NT / 4);
        const int m = p0 + row;
        unsigned mask = 0;
        if (m < a.npix) {
            if (a.taps == 9) {
                const int q = m % hw, i = q / a.w, j = q % a.w;
#pragma unroll
                for (int t = 0; t < 9; ++t) {
                    const int ii = i + t / 3 - 1, jj = j + t % 3 - 1;
                    if (ii >= 0 && ii < a.h && jj >= 0 && jj < a.w) mask |= 1u << t;
                }
            } else {
                mask = 1u;
            }
        }
        amask[u] = mask;
        abase[u] = (long long)m * a.in_stride + a.in_off + part * 16;
        alds[u] = BC * ROWB + row * ROWB + part * 16;
    }

    // accumulators start at the 32-bit bias
    v16i acc[TC][TP];
    const int half = lane >> 5, l32 = lane & 31;
    static_for<TC>([&](auto tc_) {
        constexpr int tc = decltype(tc_)::value;
        static_for<4>([&](auto g_) {
            constexpr int g = decltype(g_)::value;
            const int nb = c0 + wc * WTC + tc * 32 + g * 8 + half * 4;
            const v4i b4 = *(const v4i*)(a.bias + nb);
            static_for<TP>([&](auto tp_) {
                constexpr int tp = decltype(tp_)::value;
                acc[tc][tp][g * 4 + 0] = b4[0];
                acc[tc][tp][g * 4 + 1] = b4[1];
                acc[tc][tp][g * 4 + 2] = b4[2];
                acc[tc][tp][g * 4 + 3] = b4[3];
            });
        });
    });

    v4i rw[WU], ra[AU];
    auto gload = [&](int tap, int cc) {
        const long long koff = (long long)(tap * cpt + cc) * KT;
#pragma unroll
        for (int u = 0; u < WU; ++u) rw[u] = *(const v4i*)(wptr[u] + koff);
        const int dpix = a.taps == 9 ? (tap / 3 - 1) * a.w + (tap % 3 - 1) : 0;
        const long long aoff = (long long)dpix * a.in_stride + cc * KT;
#pragma unroll
        for (int u = 0; u < AU; ++u) {
            v4i v = {0, 0, 0, 0};
            if ((amask[u] >> tap) & 1u) v = *(const v4i*)(a.in + abase[u] + aoff);
            ra[u] = v;
        }
    };
    auto lstore = [&](int buf) {
        unsigned char* base = lds + buf * STAGE;
#pragma unroll
        for (int u = 0; u < WU; ++u) *(v4i*)(base + wlds[u]) = rw[u];
#pragma unroll
        for (int u = 0; u < AU; ++u) *(v4i*)(base + alds[u]) = ra[u];
    };

    gload(0, 0);
    lstore(0);
    __syncthreads();
    int tap = 0, cc = 0;
    for (int kt = 0; kt < nkt; ++kt) {
        const int buf = kt & 1;
        if (++cc == cpt) { cc = 0; ++tap; }
        const bool more = kt + 1 < nkt;
        if (more) gload(tap, cc);
        const unsigned char* wl = lds + buf * STAGE + (wc * WTC + l32) * ROWB + half * 16;
        const unsigned char* al = lds + buf * STAGE + BC * ROWB + (wp * WTP + l32) * ROWB + half * 16;
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            v4i wf[TC], af[TP];
#pragma unroll
            for (int tc = 0; tc < TC; ++tc) wf[tc] = *(const v4i*)(wl + tc * 32 * ROWB + ks * 32);
#pragma unroll
            for (int tp = 0; tp < TP; ++tp) af[tp] = *(const v4i*)(al + tp * 32 * ROWB + ks * 32);
            static_for<TC>([&](auto tc_) {
                constexpr int tc = decltype(tc_)::value;
                static_for<TP>([&](auto tp_) {
                    constexpr int tp = decltype(tp_)::value;
                    acc[tc][tp] = __builtin_amdgcn_mfma_i32_32x32x32_i8(wf[tc], af[tp], acc[tc][tp], 0, 0, 0);
                });
            });
        }
        if (more) lstore(buf ^ 1);
        __syncthreads();
    }

    // ---- epilogue: lane owns pixel l32 of each pixel tile and, per register quad g,
    // channels g*8 + half*4 .. +3 of each channel tile
    static_for<TP>([&](auto tp_) {
        constexpr int tp = decltype(tp_)::value;
        const int m = p0 + wp * WTP + tp * 32 + l32;
        if (m >= a.npix) return;
        static_for<TC>([&](auto tc_) {
            constexpr int tc = decltype(tc_)::value;
            static_for<4>([&](auto g_) {
                constexpr int g = decltype(g_)::value;
                const int nb = c0 + wc * WTC + tc * 32 + g * 8 + half * 4;
                if (nb >= a.n_store) return;
                const v4i M4 = *(const v4i*)(a.mul + nb);
                const v4i S4 = *(const v4i*)(a.shift + nb);
                int v[4];
                v[0] = rq_dev(acc[tc][tp][g * 4 + 0], M4[0], S4[0]);
                v[1] = rq_dev(acc[tc][tp][g * 4 + 1], M4[1], S4[1]);
                v[2] = rq_dev(acc[tc][tp][g * 4 + 2], M4[2], S4[2]);
                v[3] = rq_dev(acc[tc][tp][g * 4 + 3], M4[3], S4[3]);
                if (a.mode == MODE_ACT && a.out_map == nullptr) {
                    int8_t* o = a.out + (long long)m * a.out_stride + a.out_off + nb;
                    if (a.shortcut) {
                        const int sc = *(const int*)o;
#pragma unroll
                        for (int e = 0; e < 4; ++e) v[e] += (int)(int8_t)(sc >> (8 * e));
                    }
                    unsigned packed = 0;
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        int y = v[e];
                        if (a.relu) y = y < 0 ? 0 : y;
                        packed |= ((unsigned)sat8_dev(y) & 0xffu) << (8 * e);
                    }
                    *(unsigned*)o = packed;
                } else if (a.mode == MODE_ACT) {
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        if (nb + e >= a.n_store) continue;
                        int8_t* o = a.out + (long long)m * a.out_stride + a.out_off + a.out_map[nb + e];
                        int y = v[e];
                        if (a.shortcut) y += (int)*o;
                        if (a.relu) y = y < 0 ? 0 : y;
                        *o = (int8_t)sat8_dev(y);
                    }
                } else if (a.mode == MODE_COUPLE) {
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        if (nb + e >= a.n_store) continue;
                        int y = v[e];
                        if (a.relu) y = y < 0 ? 0 : y;
                        int32_t* s = a.state + (long long)m * a.state_c + a.idx_b[nb + e];
                        *s += a.sign * sat8_dev(y);
                    }
                } else {
                    const int b = m / hw, q = m % hw;
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        if (nb + e >= a.n_store) continue;
                        int y = v[e];
                        if (a.relu) y = y < 0 ? 0 : y;
                        a.codes[(long long)b * a.codes_img_stride + a.codes_off + (long long)(nb + e) * hw + q] =
                            (int8_t)sat8_dev(y);
                    }
                }
            });
        });
    });
}

namespace {

struct TileCfg {
    int bc, bp;
    size_t lds;
    void (*kern)(const ConvArgs, int, int);
    int threads;
    const char* name;
};

#define IODF_TILE(BC, BP, WC, WP)                                                                   \
    TileCfg {                                                                                       \
        BC, BP, (size_t)2 * (BC + BP) * ROWB, conv_igemm<BC, BP, WC, WP>, WC * WP * 64,             \
            "conv_igemm<" #BC "," #BP "," #WC "," #WP ">"                                           \
    }

const TileCfg kTiles[] = {
    IODF_TILE(256, 256, 2, 2),
    IODF_TILE(128, 128, 2, 2),
    IODF_TILE(64, 256, 1, 4),
    IODF_TILE(64, 64, 2, 2),
};
constexpr int kNumTiles = sizeof(kTiles) / sizeof(kTiles[0]);

int forced_tile() {
    static int v = [] {
        const char* e = getenv("IODF_TILE");
        return e ? atoi(e) : -1;
    }();
    return v;
}

bool args_ok(const ConvArgs& a) {
    return !(a.cin_pad <= 0 || a.cin_pad % KT || a.n_pad <= 0 || a.n_pad % 64 || (a.taps != 1 && a.taps != 9) ||
             a.in_stride % 16 || a.in_off % 16 || a.in_off + a.cin_pad > a.in_stride || a.n_store > a.n_pad ||
             a.n_store < 1 || a.h < 1 || a.w < 1 || a.npix % (a.h * a.w) || !a.in || !a.wgt || !a.bias || !a.mul ||
             !a.shift ||
             (a.mode == MODE_ACT &&
              (!a.out || (!a.out_map && (a.n_store % 4 || a.out_stride % 4 || a.out_off % 4 ||
                                         a.out_off + a.n_store > a.out_stride)))) ||
             (a.mode == MODE_COUPLE && (!a.state || !a.idx_b || a.state_c < 1)) ||
             (a.mode == MODE_CODES && !a.codes) || a.mode < MODE_ACT || a.mode > MODE_CODES);
}

}  // namespace

hipError_t conv_setup() {
    for (int i = 0; i < kNumTiles; ++i) {
        hipError_t e = hipFuncSetAttribute((const void*)kTiles[i].kern, hipFuncAttributeMaxDynamicSharedMemorySize,
                                           (int)kTiles[i].lds);
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

int conv_num_tiles() { return kNumTiles; }
const char* conv_tile_name(int tile) { return tile >= 0 && tile < kNumTiles ? kTiles[tile].name : "?"; }

// Largest tile that still fills the chip; otherwise the valid tile with most workgroups.
int conv_pick_tile(const ConvArgs& a) {
    if (!args_ok(a)) return -1;
    int best = -1;
    long long best_blocks = -1;
    const int forced = forced_tile();
    for (int i = 0; i < kNumTiles; ++i) {
        if (a.n_pad % kTiles[i].bc) continue;
        const long long blocks = (long long)((a.npix + kTiles[i].bp - 1) / kTiles[i].bp) * (a.n_pad / kTiles[i].bc);
        if (i == forced) return i;
        if (blocks >= 256) return i;
        if (blocks > best_blocks) { best_blocks = blocks; best = i; }
    }
    return best;
}

hipError_t launch_conv(const ConvArgs& a, hipStream_t stream) {
    if (a.npix <= 0) return hipSuccess;
    const int best = conv_pick_tile(a);
    if (best < 0) return hipErrorInvalidValue;
    const TileCfg& t = kTiles[best];
    const int npb = (a.npix + t.bp - 1) / t.bp, ncb = a.n_pad / t.bc;
    const int grid = ((npb + 7) / 8) * 8 * ncb;
    hipLaunchKernelGGL(t.kern, dim3(grid), dim3(t.threads), t.lds, stream, a, npb, ncb);
    return hipGetLastError();
}

}  // namespace iodf
