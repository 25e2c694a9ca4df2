// Integer-only convolution (Sec. 4.1, Eq. 4-5) as an implicit GEMM on the gfx950
// int8 matrix cores, with the fixed-point requantise / ReLU / shortcut / coupling
// epilogue fused in.
//
// GEMM view: D[channel][pixel] = sum_k Wgt[channel][k] * Act[k][pixel], k = (tap, c).
// Activations live in 64-channel planes ([c/64][pixel][64]) and weights k-tile major
// ([k/64][channel][64]), so every staged tile is a run of whole cache lines.
// Output channels are the MFMA "A" rows and pixels the "B" columns, so that after
// v_mfma_i32_32x32x32_i8 every lane owns 4 consecutive channels of one pixel per
// register quad: the 8-bit results pack into dword stores along the channel axis of
// the pixel-major activation tensor.
//
// A workgroup computes BC channels x BP pixels, streaming 64-byte k-tiles of both operands
// through a ring of LDS stages (see conv_igemm). For 3x3 layers the activation tile of tap
// (ky,kx) is the tile of the pixels shifted by (ky-1, kx-1) inside zero-bordered images.
#include "conv.h"

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

// Epilogue variants a kernel is compiled for.
enum { EPI_ANY = 0, EPI_FAST = 1, EPI_FAST_RELU = 2 };

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

// Pixel index m -> position of the pixel in the zero-bordered image stack, (b * PP + (i+1) * W2 + (j+1)).
// Image sides that are powers of two (every benchmark shape) take shifts; others divide.
__device__ __forceinline__ int bordered_pos(const ConvArgs& a, int m, int hw, int W2, int PP) {
    int b, i, j;
    if (a.log2_w >= 0 && a.log2_hw >= 0) {
        b = m >> a.log2_hw;
        const int q = m & (hw - 1);
        i = q >> a.log2_w;
        j = q & (a.w - 1);
    } else {
        b = m / hw;
        const int q = m - b * hw;
        i = q / a.w;
        j = q - i * a.w;
    }
    return b * PP + (i + 1) * W2 + (j + 1);
}

// Fast exact requantise for shifts >= 33: with u = |acc| * M = hi * 2^32 + lo, the rounding
// constant 2^(s-1) is a multiple of 2^32, so floor((u + 2^(s-1)) / 2^s) =
// (hi + 2^(s-33)) >> (s-32) and the low word never matters. sh = s - 32 (1..30).
__device__ __forceinline__ int rq_fast_abs(unsigned ua, int M, int sh) {
    return (int)((__umulhi(ua, (unsigned)M) + (1u << (sh - 1))) >> sh);
}

// Epilogue for plain 8-bit pixel-major stores (MODE_ACT, every shift >= 33,
// n_store a multiple of 16). After the requantise each lane holds four dwords of 4 channels
// (register quads g = 0..3: channels g*8 + half*4 ..); three rounds of v_permlane32_swap
// between the two wave halves regroup them into 16 consecutive channels per lane, stored
// with one 16-byte write.
template <int TC, int TP, bool PURE_RELU>
__device__ __forceinline__ void conv_epilogue_fast(const ConvArgs& a, v16i (&acc)[TC][TP], const int pix_base,
                                                   const int ch_base, const int lane, const int hw,
                                                   const int* cst, const int cst_n, const int ch_local) {
    const int half = lane >> 5, l32 = lane & 31;
    const int W2 = a.w + 2, PP = (a.h + 2) * W2;
    // position of each of this lane's pixels in the zero-bordered plane
    long long ppos[TP];
#pragma unroll
    for (int tp = 0; tp < TP; ++tp) {
        int m = pix_base + tp * 32 + l32;
        m = m < a.npix ? m : 0;
        ppos[tp] = (long long)bordered_pos(a, m, hw, W2, PP) * 64;
    }
    // Shortcut codes (Eq. 2) sit where the result goes. Each lane fetches, with one 16-byte load per
    // 32x32 tile, exactly the 16 bytes it will store (all of them before the first store), and the
    // store's three permlane rounds run backwards to bring them into the accumulators' quad layout:
    // v_permlane32_swap undoes itself.
    [[maybe_unused]] v4i scq[TC][TP];
    if constexpr (!PURE_RELU) {
        static_for<TC>([&](auto tc_) {
            constexpr int tc = decltype(tc_)::value;
            static_for<TP>([&](auto tp_) {
                constexpr int tp = decltype(tp_)::value;
                v4i s4 = {0, 0, 0, 0};
                if (a.shortcut) {
                    const int ch0 = ch_base + tc * 32;
                    const bool ok = pix_base + tp * 32 + l32 < a.npix && ch0 + half * 16 < a.n_store;
                    const int8_t* srow =
                        a.out + (long long)(a.out_chunk0 + (ch0 >> 6)) * a.out_plane + ppos[tp] + (ch0 & 63);
                    if (ok) s4 = *(const v4i*)(srow + half * 16);
                }
                scq[tc][tp] = s4;
            });
        });
        if (a.shortcut) {
            static_for<TC>([&](auto tc_) {
                constexpr int tc = decltype(tc_)::value;
                static_for<TP>([&](auto tp_) {
                    constexpr int tp = decltype(tp_)::value;
                    const v4i s4 = scq[tc][tp];  // {x0, w0, x1, w1} of the store below
                    auto x = __builtin_amdgcn_permlane32_swap((unsigned)s4[0], (unsigned)s4[2], false, false);
                    auto w = __builtin_amdgcn_permlane32_swap((unsigned)s4[1], (unsigned)s4[3], false, false);
                    auto q01 = __builtin_amdgcn_permlane32_swap(x[0], w[0], false, false);
                    auto q23 = __builtin_amdgcn_permlane32_swap(x[1], w[1], false, false);
                    scq[tc][tp] = v4i{(int)q01[0], (int)q01[1], (int)q23[0], (int)q23[1]};
                });
            });
        }
    }
    static_for<TC>([&](auto tc_) {
        constexpr int tc = decltype(tc_)::value;
        // bias (PURE_RELU: the clamp bound instead), multiplier, shift - 32 of this lane's 16 channels
        // (staged in LDS), and the rounding constant 2^(shift - 33)
        v4i Bq[4], Mq[4], Sq[4];
        unsigned Rq[4][4];
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            const int nl = ch_local + tc * 32 + g * 8 + half * 4;
            Bq[g] = *(const v4i*)(cst + nl);
            Mq[g] = *(const v4i*)(cst + cst_n + nl);
            Sq[g] = *(const v4i*)(cst + 2 * cst_n + nl);
#pragma unroll
            for (int e = 0; e < 4; ++e) Rq[g][e] = 1u << (Sq[g][e] - 1);
        }
        static_for<TP>([&](auto tp_) {
            constexpr int tp = decltype(tp_)::value;
            const int m = pix_base + tp * 32 + l32;
            const bool live = m < a.npix;
            // channels ch_base + tc*32 .. +31 sit inside one 64-channel plane
            const int ch0 = ch_base + tc * 32;
            int8_t* orow = a.out + (long long)(a.out_chunk0 + (ch0 >> 6)) * a.out_plane + ppos[tp] + (ch0 & 63);
            unsigned pk[4];
            static_for<4>([&](auto g_) {
                constexpr int g = decltype(g_)::value;
                if constexpr (PURE_RELU) {
                    // ReLU without shortcut. The accumulators already hold the bias. Clamping them to
                    // [0, hi] first (hi = the smallest value that requantises to 127; the rescale is
                    // monotone and steps by at most 1) replaces both the ReLU and the saturation, so
                    // every result fits a byte and the last shift can drop it straight into its place
                    // in the packed dword.
                    unsigned q[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        int av;
                        asm("v_med3_i32 %0, %1, 0, %2" : "=v"(av) : "v"(acc[tc][tp][g * 4 + e]), "v"(Bq[g][e]));
                        q[e] = __umulhi((unsigned)av, (unsigned)Mq[g][e]) + Rq[g][e];
                    }
                    unsigned p4 = q[0] >> Sq[g][0];
                    asm("v_lshrrev_b32_sdwa %0, %1, %2 dst_sel:BYTE_1 dst_unused:UNUSED_PRESERVE src0_sel:DWORD "
                        "src1_sel:DWORD" : "+v"(p4) : "v"(Sq[g][1]), "v"(q[1]));
                    asm("v_lshrrev_b32_sdwa %0, %1, %2 dst_sel:BYTE_2 dst_unused:UNUSED_PRESERVE src0_sel:DWORD "
                        "src1_sel:DWORD" : "+v"(p4) : "v"(Sq[g][2]), "v"(q[2]));
                    asm("v_lshrrev_b32_sdwa %0, %1, %2 dst_sel:BYTE_3 dst_unused:UNUSED_PRESERVE src0_sel:DWORD "
                        "src1_sel:DWORD" : "+v"(p4) : "v"(Sq[g][3]), "v"(q[3]));
                    pk[g] = a.out_unsigned ? p4 ^ 0x80808080u : p4;  // code u is stored as u - 128
                    return;
                } else {
                    // Signed results: a shortcut and / or no ReLU. The accumulators hold the bias. In
                    // stored bytes the result is clamp(rq(acc) + shortcut byte, lo, 127): for signed codes
                    // lo is 0 with a ReLU and -128 without; for unsigned codes (stored as code - 128, which
                    // only occur here together with a shortcut of the same format) the two offsets of 128
                    // cancel and ReLU plus saturation to [0, 255] is the clamp to [-128, 127]. The shortcut
                    // byte is added sign-extended straight out of its dword and the clamp's second half
                    // drops the byte into the packed dword.
                    const int sc = scq[tc][tp][g];
                    const int lo2 = (a.relu && !a.out_unsigned) ? 0 : -128;
                    unsigned p4 = 0;
                    static_for<4>([&](auto e_) {
                        constexpr int e = decltype(e_)::value;
                        const int av = acc[tc][tp][g * 4 + e];
                        const int sgn = av >> 31;
                        const unsigned q = (__umulhi((unsigned)((av ^ sgn) - sgn), (unsigned)Mq[g][e]) + Rq[g][e]) >> Sq[g][e];
                        const int r = ((int)q ^ sgn) - sgn;
                        int t;
                        if constexpr (e == 0)
                            asm("v_add_u32_sdwa %0, %1, sext(%2) dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD "
                                "src1_sel:BYTE_0" : "=v"(t) : "v"(r), "v"(sc));
                        else if constexpr (e == 1)
                            asm("v_add_u32_sdwa %0, %1, sext(%2) dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD "
                                "src1_sel:BYTE_1" : "=v"(t) : "v"(r), "v"(sc));
                        else if constexpr (e == 2)
                            asm("v_add_u32_sdwa %0, %1, sext(%2) dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD "
                                "src1_sel:BYTE_2" : "=v"(t) : "v"(r), "v"(sc));
                        else
                            asm("v_add_u32_sdwa %0, %1, sext(%2) dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD "
                                "src1_sel:BYTE_3" : "=v"(t) : "v"(r), "v"(sc));
                        t = t < lo2 ? lo2 : t;
                        const int hi2 = 127;
                        if constexpr (e == 0)
                            asm("v_min_i32_sdwa %0, %1, %2 dst_sel:BYTE_0 dst_unused:UNUSED_PRESERVE src0_sel:DWORD "
                                "src1_sel:DWORD" : "+v"(p4) : "v"(t), "v"(hi2));
                        else if constexpr (e == 1)
                            asm("v_min_i32_sdwa %0, %1, %2 dst_sel:BYTE_1 dst_unused:UNUSED_PRESERVE src0_sel:DWORD "
                                "src1_sel:DWORD" : "+v"(p4) : "v"(t), "v"(hi2));
                        else if constexpr (e == 2)
                            asm("v_min_i32_sdwa %0, %1, %2 dst_sel:BYTE_2 dst_unused:UNUSED_PRESERVE src0_sel:DWORD "
                                "src1_sel:DWORD" : "+v"(p4) : "v"(t), "v"(hi2));
                        else
                            asm("v_min_i32_sdwa %0, %1, %2 dst_sel:BYTE_3 dst_unused:UNUSED_PRESERVE src0_sel:DWORD "
                                "src1_sel:DWORD" : "+v"(p4) : "v"(t), "v"(hi2));
                    });
                    pk[g] = p4;
                }
            });
            // lower half holds channels {0-3, 8-11, 16-19, 24-27}, upper {4-7, 12-15, 20-23, 28-31}
            auto s01 = __builtin_amdgcn_permlane32_swap(pk[0], pk[1], false, false);
            auto s23 = __builtin_amdgcn_permlane32_swap(pk[2], pk[3], false, false);
            // lower: {0-3, 4-7}, {16-19, 20-23}; upper: {8-11, 12-15}, {24-27, 28-31}
            auto x = __builtin_amdgcn_permlane32_swap(s01[0], s23[0], false, false);
            auto w = __builtin_amdgcn_permlane32_swap(s01[1], s23[1], false, false);
            // lower: channels 0-15, upper: channels 16-31
            if (live && ch_base + tc * 32 + half * 16 < a.n_store) {
                v4i o4 = {(int)x[0], (int)w[0], (int)x[1], (int)w[1]};
                *(v4i*)(orow + half * 16) = o4;
            }
        });
    });
}

// General epilogue of one wave tile (any mode, any shift). Lane owns pixel l32 of each
// 32-pixel tile and, per register quad g, channels g*8 + half*4 .. +3 of each 32-channel tile.
template <int TC, int TP>
__device__ __forceinline__ void conv_epilogue(const ConvArgs& a, v16i (&acc)[TC][TP], const int pix_base,
                                              const int ch_base, const int lane, const int hw) {
    const int half = lane >> 5, l32 = lane & 31;
    static_for<TP>([&](auto tp_) {
        constexpr int tp = decltype(tp_)::value;
        const int m = pix_base + tp * 32 + l32;
        if (m >= a.npix) return;
        static_for<TC>([&](auto tc_) {
            constexpr int tc = decltype(tc_)::value;
            static_for<4>([&](auto g_) {
                constexpr int g = decltype(g_)::value;
                const int nb = ch_base + tc * 32 + g * 8 + half * 4;
                if (nb >= a.n_store) return;
                const v4i B4 = *(const v4i*)(a.bias + nb);
                if (a.mode == MODE_RAW) {  // n_pad is a multiple of 64, so the quad is in bounds
                    const v4i r4 = {acc[tc][tp][g * 4 + 0] + B4[0], acc[tc][tp][g * 4 + 1] + B4[1],
                                    acc[tc][tp][g * 4 + 2] + B4[2], acc[tc][tp][g * 4 + 3] + B4[3]};
                    *(v4i*)(a.partial + (long long)m * a.n_pad + nb) = r4;
                    return;
                }
                const v4i M4 = *(const v4i*)(a.mul + nb);
                const v4i S4 = *(const v4i*)(a.shift + nb) + (a.rq_fast ? 32 : 0);
                int v[4];
                v[0] = rq_dev(acc[tc][tp][g * 4 + 0] + B4[0], M4[0], S4[0]);
                v[1] = rq_dev(acc[tc][tp][g * 4 + 1] + B4[1], M4[1], S4[1]);
                v[2] = rq_dev(acc[tc][tp][g * 4 + 2] + B4[2], M4[2], S4[2]);
                v[3] = rq_dev(acc[tc][tp][g * 4 + 3] + B4[3], M4[3], S4[3]);
                if (a.mode == MODE_ACT) {
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        if (nb + e >= a.n_store) continue;
                        const int ch = nb + e;
                        const int bi = m / hw, qi = m - bi * hw, ii = qi / a.w, ji = qi - ii * a.w;
                        const long long pp = (long long)bi * ((a.h + 2) * (a.w + 2)) + (ii + 1) * (a.w + 2) + (ji + 1);
                        int8_t* o = a.out + (long long)(a.out_chunk0 + (ch >> 6)) * a.out_plane + pp * 64 + (ch & 63);
                        int y = v[e];
                        if (a.shortcut) y += (int)*o + (a.sc_unsigned ? 128 : 0);
                        if (a.relu) y = y < 0 ? 0 : y;
                        *o = (int8_t)(a.out_unsigned ? (y > 255 ? 255 : y) - 128 : sat8_dev(y));
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

// Split-K epilogue: add this workgroup's partial sums into the int32 scratch [pixel][n_pad].
// Integer addition is associative, so the result does not depend on arrival order.
template <int TC, int TP>
__device__ __forceinline__ void conv_epilogue_partial(const ConvArgs& a, v16i (&acc)[TC][TP], const int pix_base,
                                                      const int ch_base, const int lane) {
    const int half = lane >> 5, l32 = lane & 31;
    static_for<TP>([&](auto tp_) {
        constexpr int tp = decltype(tp_)::value;
        const int m = pix_base + tp * 32 + l32;
        if (m >= a.npix) return;
        static_for<TC>([&](auto tc_) {
            constexpr int tc = decltype(tc_)::value;
            static_for<4>([&](auto g_) {
                constexpr int g = decltype(g_)::value;
                const int nb = ch_base + tc * 32 + g * 8 + half * 4;
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if (nb + e < a.n_store) atomicAdd(a.partial + (long long)m * a.n_pad + nb + e, acc[tc][tp][g * 4 + e]);
            });
        });
    });
}

// Wait until at most N of this wave's global->LDS loads are outstanding and all of its LDS
// reads have returned, then meet the other waves. Loads retire in order, so "at most N
// outstanding" means every tile but the newest N / (loads per tile) has landed; the LDS-read
// part guarantees that nobody still reads the stage the next loads will overwrite.
template <int N>
__device__ __forceinline__ void wait_tiles_then_barrier() {
    static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
    asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"(N) : "memory");
}

// Timeline of one output tile (see ConvArgs::trace): stamp `which` of slot `slot`.
__device__ __forceinline__ void trace_stamp(const ConvArgs& a, int slot, int which, int tid) {
    if (a.has_trace && tid == 0) {
        a.trace[8LL * slot + which] = (long long)wall_clock64();
        if (which == 0) a.trace[8LL * slot + 4] = (long long)clock64();
        if (which == 3) a.trace[8LL * slot + 5] = (long long)clock64();
    }
}

// Hand-placed LDS fragment reads (see conv_igemm_lean). The destination is an output of the read statement
// and an in/out operand of the wait that covers it, so no use of it can be scheduled ahead of that wait.
template <int OFF>
__device__ __forceinline__ void lds_read_b128(v4i& d, const unsigned addr) {
    static_assert(OFF >= 0 && OFF < 65536, "16-bit offset field");
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(d) : "v"(addr), "n"(OFF));
}
// Marks the fragments as produced here: what uses them stays behind every asm statement before this point.
template <int NWF, int NAF>
__device__ __forceinline__ void tie_frags(v4i (&w)[NWF], v4i (&x)[NAF]) {
#pragma unroll
    for (int i = 0; i < NWF; ++i) asm volatile("" : "+v"(w[i]));
#pragma unroll
    for (int i = 0; i < NAF; ++i) asm volatile("" : "+v"(x[i]));
}
// at most LG LDS operations of this wave outstanding; the fragments w, x are among the completed ones
template <int LG, int NWF, int NAF>
__device__ __forceinline__ void wait_frags(v4i (&w)[NWF], v4i (&x)[NAF]) {
    static_assert(LG >= 0 && LG < 16, "counter width");
    asm volatile("s_waitcnt lgkmcnt(%0)" ::"n"(LG) : "memory");
    tie_frags(w, x);
}
// at most VM vector-memory operations and LG LDS operations of this wave outstanding, then the barrier
template <int VM, int LG, int NWF, int NAF>
__device__ __forceinline__ void wait_frags_then_barrier(v4i (&w)[NWF], v4i (&x)[NAF]) {
    static_assert(VM >= 0 && VM < 64 && LG >= 0 && LG < 16, "counter widths");
    asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(%1)\n\ts_barrier" ::"n"(VM), "n"(LG) : "memory");
    tie_frags(w, x);
}

// BC channels x BP pixels per workgroup, WC x WP waves, NST LDS stages of one 64-byte k-tile.
//
// Tiles go from global memory straight into LDS (global_load_lds_dwordx4): a wave-wide load
// fills 1 KB of LDS with the 16-byte chunks of its 64 lanes in lane order, i.e. 16 rows x 64
// bytes. Lane i fetches k-part (i & 3) ^ ((i >> 4) & 3) of row i >> 2, so the chunk of k-part
// q of row r sits at position q ^ ((r >> 2) & 3) of the row: the 16-byte fragment reads of 16
// consecutive rows then touch every LDS bank exactly once. NST - 1 tiles are in flight while
// one is consumed; each lane issues the same number of loads per tile, so a constant
// s_waitcnt vmcnt() tells when the oldest tile has landed, and one s_barrier per tile both
// publishes it and frees the stage consumed before. Activation planes carry a one-pixel zero
// border per image, so a 3x3 tap is a constant address shift and needs no bounds test; all
// per-tile address arithmetic is scalar, the per-lane parts are computed once.
// Four-wave, three-stage configurations are compiled for two workgroups per CU.
template <int BC, int BP, int WC, int WP, int NST, int EPI>
__global__ __launch_bounds__(WC* WP * 64, (WC * WP == 4 && NST == 3) ? 2 : 1) void conv_igemm(const ConvArgs a) {
    const int npb = (a.npix + BP - 1) / BP, ncb = a.n_pad / BC;  // pixel blocks, channel blocks
    constexpr int NW = WC * WP;
    constexpr int WTC = BC / WC, WTP = BP / WP;  // wave tile
    constexpr int TC = WTC / 32, TP = WTP / 32;  // 32x32 MFMA tiles per wave
    constexpr int WI = BC / 16 / NW, AI = BP / 16 / NW;  // wave-wide loads per wave per k-tile
    constexpr int LPT = WI + AI;
    constexpr int STAGE = (BC + BP) * KT;
    static_assert(WTC % 32 == 0 && WTP % 32 == 0, "wave tile must be a multiple of 32x32");
    static_assert(BC % (16 * NW) == 0 && BP % (16 * NW) == 0, "tile rows must divide over the waves");
    static_assert(NST >= 3 && (NST - 2) * LPT < 64, "pipeline depth must fit the vmcnt counter");

    extern __shared__ __align__(1024) unsigned char lds[];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform, lives in an SGPR
    const int wc = wave % WC, wp = wave / WC;

    // Workgroups are dealt round-robin to the 8 XCDs. Give each XCD whole pixel
    // blocks (all their channel blocks), so an activation tile is fetched into one L2 only.
    const int bid = blockIdx.x;
    const int xcd = bid & 7, slot = bid >> 3;
    const int pb = (slot / ncb) * 8 + xcd, cb = slot % ncb;
    if (pb >= npb) return;
    const int p0 = pb * BP, c0 = cb * BC;
    if (c0 >= a.n_store) return;  // a channel block of padding only
    trace_stamp(a, bid, 0, tid);

    // split-K: blockIdx.y owns a contiguous range of k-tiles and adds its partial sums to a.partial
    const int nkt_all = a.taps * (a.cin_pad / KT);
    const int nsk = gridDim.y, sk = blockIdx.y;
    const int kt0 = (int)((long long)nkt_all * sk / nsk);
    const int nkt = (int)((long long)nkt_all * (sk + 1) / nsk) - kt0;
    const long long wtile = (long long)a.n_pad * KT;  // bytes per weight k-tile
    const int hw = a.h * a.w;
    const int W2 = a.w + 2, PP = (a.h + 2) * W2;  // zero-bordered image geometry

    // What this lane fetches in each wave-wide load: k-part lpart of row lrow of a 16-row
    // segment. Weight segments are contiguous, so the lane offset is a constant; activation
    // rows are pixels, whose position in the bordered plane is computed once here. Rows past
    // the last pixel re-read the last pixel (their results are never stored).
    const int lrow = lane >> 2;
    const int lpart = (lane & 3) ^ ((lane >> 4) & 3);
    const unsigned woffl = (unsigned)(lrow * KT + lpart * 16);
    unsigned aoffl[AI];
#pragma unroll
    for (int u = 0; u < AI; ++u) {
        int m = p0 + (wave * AI + u) * 16 + lrow;
        m = m < a.npix ? m : a.npix - 1;
        aoffl[u] = (unsigned)bordered_pos(a, m, hw, W2, PP) * KT + (unsigned)(lpart * 16);
    }
    const int8_t* const wbase = a.wgt + (long long)(c0 + wave * WI * 16) * KT;
    const int8_t* const abase = a.in + (long long)a.in_chunk0 * a.in_plane;

    // Accumulators start at zero; the 32-bit bias joins in the epilogue. The per-channel
    // constants of this workgroup's BC channels are staged in LDS behind the stage ring (they
    // become visible with the first barrier of the k loop), so the epilogue reads them with
    // LDS latency and its loads do not queue behind the tile loads.
    v16i acc[TC][TP];
    const int half = lane >> 5, l32 = lane & 31;
    static_for<TC>([&](auto tc_) {
        constexpr int tc = decltype(tc_)::value;
        static_for<TP>([&](auto tp_) {
            constexpr int tp = decltype(tp_)::value;
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[tc][tp][r] = 0;
        });
    });
    if constexpr (EPI != EPI_ANY) {
        // the fast epilogues expect the bias in the accumulators from the start (the ReLU one clamps
        // before it rescales): register quad g of tile tc holds channels tc*32 + g*8 + half*4 .. +3
        static_for<TC>([&](auto tc_) {
            constexpr int tc = decltype(tc_)::value;
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const v4i b4 = *(const v4i*)(a.bias + c0 + wc * WTC + tc * 32 + g * 8 + half * 4);
                static_for<TP>([&](auto tp_) {
                    constexpr int tp = decltype(tp_)::value;
#pragma unroll
                    for (int e = 0; e < 4; ++e) acc[tc][tp][g * 4 + e] = b4[e];
                });
            }
        });
    }
    int* const cst = (int*)(lds + NST * STAGE);  // [3][BC]: bias (or clamp bound), multiplier, shift
    int cb_v = 0, cm_v = 0, cs_v = 0;
    if (tid < BC) {
        cb_v = EPI == EPI_FAST_RELU ? a.clamp_hi[c0 + tid] : (EPI == EPI_ANY ? a.bias[c0 + tid] : 0);
        cm_v = a.mul[c0 + tid];
        cs_v = a.shift[c0 + tid];
    }

    typedef const void __attribute__((address_space(1))) * gptr_t;
    typedef void __attribute__((address_space(3))) * lptr_t;
    // Next tile to issue. K runs plane-major, tap-minor: the nine taps of one 64-channel plane
    // are consecutive k-tiles, so they re-read almost the same cache lines back to back. Both
    // source pointers are wave-uniform and advance by scalar additions only: weights by one
    // k-tile; activations by the shift to the next tap (+1 pixel, or to the start of the next
    // kernel row), and after the last tap to tap (0,0) of the next plane. Past the last tile the
    // last one is loaded again into a stage nobody reads, which keeps the loads per step constant.
    int itile = 0, itap = kt0 % a.taps, ikx = itap % 3;
    const int8_t* wt = wbase + (long long)kt0 * wtile;
    // tap (ky, kx) reads pixel (i + ky - 1, j + kx - 1)
    const int8_t* at = abase + (long long)(kt0 / a.taps) * a.in_plane +
                       (a.taps == 9 ? (long long)((itap / 3 - 1) * W2 + (ikx - 1)) * KT : 0LL);
    const long long next_plane = a.in_plane - (a.taps == 9 ? (long long)(2 * W2 + 2) * KT : 0LL);
    auto uniform = [](const int8_t* p) {  // tell the compiler the pointer sits in SGPRs
        const unsigned long long v = (unsigned long long)p;
        const unsigned lo = __builtin_amdgcn_readfirstlane((unsigned)v);
        const unsigned hi = __builtin_amdgcn_readfirstlane((unsigned)(v >> 32));
        return (const int8_t*)(((unsigned long long)hi << 32) | lo);
    };
    auto issue = [&]() {
        unsigned char* sb = lds + (itile % NST) * STAGE;
        const int8_t* wu = uniform(wt);
        const int8_t* au = uniform(at);
#pragma unroll
        for (int u = 0; u < WI; ++u)
            __builtin_amdgcn_global_load_lds((gptr_t)(wu + u * 1024 + woffl), (lptr_t)(sb + (wave * WI + u) * 1024), 16,
                                             0, 0);
#pragma unroll
        for (int u = 0; u < AI; ++u)
            __builtin_amdgcn_global_load_lds((gptr_t)(au + aoffl[u]), (lptr_t)(sb + BC * KT + (wave * AI + u) * 1024),
                                             16, 0, 0);
        ++itile;
        // branch-free advance (selects on scalars); frozen once the last tile has been issued
        const bool go = itile < nkt;
        const bool wrap = itap + 1 == a.taps;
        const bool row = ikx == 2;
        const long long astep = wrap ? next_plane : (long long)((row ? W2 - 2 : 1) * KT);
        wt += go ? wtile : 0LL;
        at += go ? astep : 0LL;
        itap = go ? (wrap ? 0 : itap + 1) : itap;
        ikx = go ? ((wrap || row) ? 0 : ikx + 1) : ikx;
    };

    // The bookkeeping that finds the next k-tile (which tap, which kernel row, which plane, which ring
    // stage) costs the general issue() above some twenty-five scalar instructions and a branch or two per
    // k-tile, and the compiler leaves them as one block between the last MFMA of a step and the barrier. The
    // lean loops below do it at compile time: they are unrolled over lcm(ring stages, 9 taps) steps, so the
    // LDS stage and the tap of every load and fragment read are constants, a tap's address is the plane
    // pointer plus a loop-invariant scalar, and a step has no branch. Launches whose reduction is not split
    // (every hidden layer) take them; the general loop remains for split reductions, which start mid-plane.
    // Small wave tiles (one or two MFMAs per k-step) additionally run at the pace of the wave's instruction
    // stream and of the LDS latency, not of the matrix pipe: they get a ring of nine stages and read their
    // fragments two k-tiles ahead (see below).
    constexpr bool SMALL = TC * TP <= 2 && NST == 9;
    const bool lean = EPI != EPI_ANY || nsk == 1;
    const int8_t* lw = wbase;                                                      // weight k-tile to load next
    const int8_t* la = abase + (a.taps == 9 ? (long long)(-W2 - 1) * KT : 0LL);     // pixel (i-1, j-1) of the plane to load next
    const long long rowstep = (long long)W2 * KT;
    int lissued = 0;
    [[maybe_unused]] auto lean_issue = [&](auto stage_, auto tap_, auto taps_) {
        constexpr int stage = decltype(stage_)::value, tap = decltype(tap_)::value, taps = decltype(taps_)::value;
        unsigned char* sb = lds + stage * STAGE;
        const int8_t* wu = uniform(lw);
#pragma unroll
        for (int u = 0; u < WI; ++u)
            __builtin_amdgcn_global_load_lds((gptr_t)(wu + u * 1024 + woffl), (lptr_t)(sb + (wave * WI + u) * 1024), 16,
                                             0, 0);
        // (the load's immediate offset would shift the LDS address as well, so the tap's offset is added to the pointer)
        const int8_t* au = uniform(la + (taps == 9 ? (tap / 3) * rowstep + (tap % 3) * KT : 0LL));
#pragma unroll
        for (int u = 0; u < AI; ++u)
            __builtin_amdgcn_global_load_lds((gptr_t)(au + aoffl[u]), (lptr_t)(sb + BC * KT + (wave * AI + u) * 1024),
                                             16, 0, 0);
        // past the last k-tile the pointers stay (the same tile lands again in a stage nobody reads)
        ++lissued;
        const bool go = lissued < nkt;
        lw += go ? wtile : 0LL;
        if constexpr (taps == 1 || tap == 8) la += go ? a.in_plane : 0LL;
    };
    if (lean) {
        if (a.taps == 9)
            static_for<NST - 1>([&](auto t_) { lean_issue(t_, t_, std::integral_constant<int, 9>{}); });
        else
            static_for<NST - 1>([&](auto t_) { lean_issue(t_, std::integral_constant<int, 0>{}, std::integral_constant<int, 1>{}); });
    } else if constexpr (EPI == EPI_ANY) {
#pragma unroll
        for (int t = 0; t < NST - 1; ++t) issue();
    }
    if (tid < BC) {
        cst[tid] = cb_v;
        cst[BC + tid] = cm_v;
        cst[2 * BC + tid] = cs_v;
    }

    // Fragment addresses inside a stage: row l32 of each 32-row tile, k-part (2*ks + half).
    // The loop is software pipelined: the fragments of the next 32-deep k-step are read from
    // LDS while the matrix cores work on the current one, and the barrier that publishes tile
    // kt+1 sits between the two k-steps of tile kt.
    const int sw = (l32 >> 2) & 3;
    const int off0 = (half ^ sw) * 16;
    const int wl0 = (wc * WTC + l32) * KT, al0 = BC * KT + (wp * WTP + l32) * KT;
    v4i wf0[TC], af0[TP], wf1[TC], af1[TP];
    auto read_frags = [&](int stage, int ks, v4i (&wf)[TC], v4i (&af)[TP]) {
        const unsigned char* sb = lds + stage * STAGE;
        const int off = off0 ^ (ks * 32);
#pragma unroll
        for (int tc = 0; tc < TC; ++tc) wf[tc] = *(const v4i*)(sb + wl0 + tc * 32 * KT + off);
#pragma unroll
        for (int tp = 0; tp < TP; ++tp) af[tp] = *(const v4i*)(sb + al0 + tp * 32 * KT + off);
    };
    auto mma = [&](v4i (&wf)[TC], v4i (&af)[TP]) {
        static_for<TC>([&](auto tc_) {
            constexpr int tc = decltype(tc_)::value;
            static_for<TP>([&](auto tp_) {
                constexpr int tp = decltype(tp_)::value;
                acc[tc][tp] = __builtin_amdgcn_mfma_i32_32x32x32_i8(wf[tc], af[tp], acc[tc][tp], 0, 0, 0);
            });
        });
    };
    wait_tiles_then_barrier<(NST - 2) * LPT>();  // tile 0 has landed
    trace_stamp(a, bid, 1, tid);
    if (lean) {
        if constexpr (!SMALL) {
            auto big_loop = [&](auto taps_) {
                constexpr int taps = decltype(taps_)::value;
                constexpr int U = taps == 1 ? NST : NST % 9 == 0 ? NST : NST % 3 == 0 ? 3 * NST : 9 * NST;  // lcm(NST, taps)
                read_frags(0, 0, wf0, af0);
                for (int kt = 0; kt < nkt; kt += U) {
                    const int left = nkt - kt;
                    static_for<U>([&](auto i_) {
                        constexpr int i = decltype(i_)::value;
                        constexpr int st = i % NST;
                        if (left > i) {
                            read_frags(st, 1, wf1, af1);
                            mma(wf0, af0);
                            // everybody is past its reads of tile kt+i-1 (they returned before the last barrier), so
                            // its stage takes tile kt+i+NST-1; then wait until tile kt+i+1 has landed for everybody
                            lean_issue(std::integral_constant<int, (i + NST - 1) % NST>{},
                                       std::integral_constant<int, taps == 9 ? (i + NST - 1) % 9 : 0>{}, taps_);
                            wait_tiles_then_barrier<(NST - 2) * LPT>();
                            read_frags((st + 1) % NST, 0, wf0, af0);
                            mma(wf1, af1);
                        }
                    });
                }
            };
            if (a.taps == 9) big_loop(std::integral_constant<int, 9>{});
            else big_loop(std::integral_constant<int, 1>{});
        } else {
            // Fragments of a whole k-tile are read two k-tiles ahead into three rotating register sets, the
            // two k-steps add into separate accumulators (no dependent MFMAs back to back; the integer sums
            // are merged at the end), and the barrier only asks for the LDS reads issued before the previous
            // barrier: no LDS latency is left on the path from one k-tile to the next.
            constexpr int FR = 2 * (TC + TP);
            v4i fw[3][2][TC], fa[3][2][TP];
            v16i acc1[TC][TP];
            static_for<TC>([&](auto tc_) {
                static_for<TP>([&](auto tp_) {
#pragma unroll
                    for (int r = 0; r < 16; ++r) acc1[decltype(tc_)::value][decltype(tp_)::value][r] = 0;
                });
            });
            auto read_tile = [&](int stage, auto set_) {
                constexpr int set = decltype(set_)::value;
                read_frags(stage, 0, fw[set][0], fa[set][0]);
                read_frags(stage, 1, fw[set][1], fa[set][1]);
            };
            auto mma_tile = [&](auto set_) {
                constexpr int set = decltype(set_)::value;
                static_for<TC>([&](auto tc_) {
                    constexpr int tc = decltype(tc_)::value;
                    static_for<TP>([&](auto tp_) {
                        constexpr int tp = decltype(tp_)::value;
                        acc[tc][tp] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fw[set][0][tc], fa[set][0][tp], acc[tc][tp], 0, 0, 0);
                        acc1[tc][tp] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fw[set][1][tc], fa[set][1][tp], acc1[tc][tp], 0, 0, 0);
                    });
                });
            };
            auto lean_loop = [&](auto taps_) {
                constexpr int taps = decltype(taps_)::value;
                read_tile(0, std::integral_constant<int, 0>{});
                wait_tiles_then_barrier<(NST - 3) * LPT>();  // tile 1 has landed (a repeat of tile 0 when there is only one)
                read_tile(1, std::integral_constant<int, 1>{});
                for (int kt = 0; kt < nkt; kt += NST) {
                    const int left = nkt - kt;
                    static_for<NST>([&](auto i_) {
                        constexpr int i = decltype(i_)::value;
                        if (left > i) {
                            // tile kt+i+NST-1 goes into the stage of tile kt+i-1; its tap is (i + 8) mod 9
                            lean_issue(std::integral_constant<int, (i + NST - 1) % NST>{},
                                       std::integral_constant<int, taps == 9 ? (i + 8) % 9 : 0>{}, taps_);
                            // tile kt+i+2 has landed; of this wave's LDS reads only the newest k-tile's may be pending
                            asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(%1)\n\ts_barrier" ::"n"((NST - 3) * LPT), "n"(FR) : "memory");
                            read_tile((i + 2) % NST, std::integral_constant<int, (i + 2) % 3>{});
                            mma_tile(std::integral_constant<int, i % 3>{});
                        }
                    });
                }
            };
            if (a.taps == 9) lean_loop(std::integral_constant<int, 9>{});
            else lean_loop(std::integral_constant<int, 1>{});
            static_for<TC>([&](auto tc_) {
                constexpr int tc = decltype(tc_)::value;
                static_for<TP>([&](auto tp_) {
                    constexpr int tp = decltype(tp_)::value;
#pragma unroll
                    for (int r = 0; r < 16; ++r) acc[tc][tp][r] += acc1[tc][tp][r];
                });
            });
        }
    } else if constexpr (EPI == EPI_ANY) {
        read_frags(0, 0, wf0, af0);
        // One step per k-tile, unrolled NST-fold so that every LDS stage offset is a compile-time constant.
        auto step = [&](auto st_) {
            constexpr int st = decltype(st_)::value;
            read_frags(st, 1, wf1, af1);
            mma(wf0, af0);
            issue();
            wait_tiles_then_barrier<(NST - 2) * LPT>();
            read_frags((st + 1) % NST, 0, wf0, af0);
            mma(wf1, af1);
        };
        for (int kt = 0; kt < nkt; kt += NST) {
            const int left = nkt - kt;
            static_for<NST>([&](auto i_) {
                constexpr int i = decltype(i_)::value;
                if (left > i) step(std::integral_constant<int, i>{});
            });
        }
    }
    trace_stamp(a, bid, 2, tid);

    if constexpr (EPI == EPI_FAST_RELU)
        conv_epilogue_fast<TC, TP, true>(a, acc, p0 + wp * WTP, c0 + wc * WTC, lane, hw, cst, BC, wc * WTC);
    else if constexpr (EPI == EPI_FAST)
        conv_epilogue_fast<TC, TP, false>(a, acc, p0 + wp * WTP, c0 + wc * WTC, lane, hw, cst, BC, wc * WTC);
    else if (nsk > 1)
        conv_epilogue_partial<TC, TP>(a, acc, p0 + wp * WTP, c0 + wc * WTC, lane);
    else
        conv_epilogue<TC, TP>(a, acc, p0 + wp * WTP, c0 + wc * WTC, lane, hw);
    // The loads issued past the last k-tile target stages nobody reads any more, but they must have landed
    // before the wave retires and its LDS goes to another workgroup; they do so while the epilogue runs.
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    trace_stamp(a, bid, 3, tid);
}

// Small and medium tiles, for launches with few pixels (the deep levels of a flow, everything at batch 1).
// With one or two MFMAs per wave and k-step the k loop runs at the pace of a wave's instruction stream and
// of the waits in it, not of the matrix pipe, so this kernel spends as few instructions per k-tile as it
// can and never waits for more than it needs:
//  - nine ring stages (= taps: stage and tap of every load are constants of nine unrolled steps, and a 3x3
//    layer has whole rounds); a wave loads weight rows or pixel rows, not both, and follows its stream with
//    a fixed 64-bit base in SGPRs and a 32-bit position (see below), which gives the address mode
//    "scalar base + 32-bit lane offset": one vector add per load;
//  - the fragments of a k-tile are read two k-tiles ahead into three rotating register sets, by hand-placed
//    ds_reads; only the reads of the newest k-tile may be pending at a barrier, and the wait names the set
//    the following MFMAs use (the compiler, left to itself, puts lgkmcnt(0) before the first use of a
//    fragment, which waits for the reads just issued as well and leaves one LDS latency in every step);
//  - two accumulators per output block take alternate k-steps, so no MFMA waits for the one before it.
// KS = 2 puts twice the waves on the tile: a 64x64 tile gives four waves one MFMA per k-step each, and with
// one wave per SIMD nothing fills the gaps in its stream. Group kh = 0 then multiplies the first 32-deep
// k-step of every k-tile, group kh = 1 the second, every wave issues half the loads, and the two groups'
// partial sums (integers: any order of addition gives the same result) meet once, through LDS, before the
// epilogue, which group 0 runs. Unsplit reductions only.
template <int BC, int BP, int WC, int WP, int KS, int EPI>
__global__ __launch_bounds__(WC* WP* KS * 64, KS) void conv_igemm_lean(const ConvArgs a) {
    const int npb = (a.npix + BP - 1) / BP, ncb = a.n_pad / BC;  // pixel blocks, channel blocks
    static_assert(KS == 1 || KS == 2, "a k-tile has two k-steps");
    constexpr int NST = 9;
    constexpr int NQ = WC * WP, NW = KS * NQ;
    constexpr int WTC = BC / WC, WTP = BP / WP;
    constexpr int TC = WTC / 32, TP = WTP / 32;
    constexpr int KSTEPS = 2 / KS;                        // k-steps of a k-tile that a wave multiplies
    constexpr int WSEG = BC / 16, SEGS = (BC + BP) / 16;  // 16-row segments = wave-wide loads per k-tile
    constexpr int LPT = SEGS / NW;                        // loads per wave per k-tile
    constexpr int STAGE = (BC + BP) * KT;
    constexpr int FR = KSTEPS * (TC + TP);                // fragment reads per wave per k-tile
    constexpr int CST = 2048;                             // bytes set aside for the per-channel constants
    constexpr int G = 65536 / STAGE, NB = (NST + G - 1) / G;  // a ds_read offset has 16 bits: G stages per base address
    static_assert(WTC % 32 == 0 && WTP % 32 == 0, "wave tile must be a multiple of 32x32");
    static_assert(SEGS % NW == 0 && LPT >= 1 && WSEG % LPT == 0, "a wave loads weight rows or pixel rows, not both");
    static_assert((NST - 2) * LPT < 64 && FR < 16, "counter widths");
    static_assert(3 * BC * (int)sizeof(int) <= CST && BC <= NW * 64 && G >= 1, "constants");

    extern __shared__ __align__(1024) unsigned char lds[];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wq = wave % NQ, kh = wave / NQ;
    const int wc = wq % WC, wp = wq / WC;

    const int bid = blockIdx.x;
    const int xcd = bid & 7, slot = bid >> 3;
    const int tile_grid = ((npb + 7) / 8) * 8 * ncb;
    if (bid >= tile_grid) {
        // workgroups beyond the tiles (see ConvArgs::pf): those on an XCD that holds tiles share the lines
        if (xcd >= npb) return;
        const int j = (bid - tile_grid) >> 3, P = ((int)gridDim.x - tile_grid) >> 3;
        const long long lines = (a.pf_bytes + 127) >> 7;
        // four independent loads per round, so that a thread pays one memory latency and not one per line
        const long long stride = (long long)P * blockDim.x;
        int sum = 0;
        for (long long l = (long long)j * blockDim.x + tid; l < lines; l += 4 * stride) {
            const int v0 = *(const int*)(a.pf + (l << 7));
            const int v1 = l + stride < lines ? *(const int*)(a.pf + ((l + stride) << 7)) : 0;
            const int v2 = l + 2 * stride < lines ? *(const int*)(a.pf + ((l + 2 * stride) << 7)) : 0;
            const int v3 = l + 3 * stride < lines ? *(const int*)(a.pf + ((l + 3 * stride) << 7)) : 0;
            sum += v0 + v1 + v2 + v3;
        }
        asm volatile("" ::"v"(sum));  // the loads are the point: keep them
        return;
    }
    const int pb = (slot / ncb) * 8 + xcd, cb = slot % ncb;
    if (pb >= npb) return;
    const int p0 = pb * BP, c0 = cb * BC;
    if (c0 >= a.n_store) return;
    trace_stamp(a, bid, 0, tid);

    const int nkt = a.taps * (a.cin_pad / KT);
    const long long wtile = (long long)a.n_pad * KT;
    const int hw = a.h * a.w;
    const int W2 = a.w + 2, PP = (a.h + 2) * W2;

    // This wave's LPT segments of a stage: weight rows for the first WSEG / LPT waves, pixel rows for the
    // rest. Either way the wave follows one stream: a fixed 64-bit base in SGPRs, a 32-bit position that
    // advances by `inc` bytes per k-tile (weights: one k-tile; pixels of a 1x1 layer: one plane) or by
    // `inc9` after the ninth tap (pixels of a 3x3 layer: one plane), a per-tap byte offset (pixels of a 3x3
    // layer: kernel row and column; the lane offsets already point at pixel (i-1, j-1)), and a last valid
    // position at which it stops: past the last k-tile the same tile lands again in a stage nobody reads,
    // which keeps the loads per step constant. The launcher checks that the positions fit 32 bits.
    const int lrow = lane >> 2;
    const int lpart = (lane & 3) ^ ((lane >> 4) & 3);
    const bool loads_w = wave * LPT < WSEG;
    unsigned loff[LPT];
#pragma unroll
    for (int u = 0; u < LPT; ++u) {
        const int seg = wave * LPT + u;
        int m = p0 + (seg - WSEG) * 16 + lrow;
        m = m < a.npix ? (m < 0 ? 0 : m) : a.npix - 1;
        loff[u] = loads_w ? (unsigned)(seg * 1024 + lrow * KT + lpart * 16)
                          : (unsigned)(bordered_pos(a, m, hw, W2, PP) - (a.taps == 9 ? W2 + 1 : 0)) * KT + (unsigned)(lpart * 16);
    }
    const int planes = a.cin_pad / KT;
    const int8_t* const sbase = loads_w ? a.wgt + (long long)c0 * KT : a.in + (long long)a.in_chunk0 * a.in_plane;
    const unsigned inc = loads_w ? (unsigned)wtile : a.taps == 9 ? 0u : (unsigned)a.in_plane;
    const unsigned inc9 = loads_w ? 0u : (unsigned)a.in_plane;
    const unsigned pos_last = loads_w ? (unsigned)(nkt - 1) * (unsigned)wtile : (unsigned)(planes - 1) * (unsigned)a.in_plane;
    const unsigned trow = loads_w ? 0u : (unsigned)(W2 * KT), tcol = loads_w ? 0u : (unsigned)KT;
    unsigned pos = 0;

    // two accumulators per output block; the first one of group 0 starts at the bias (fast epilogues; the
    // general one adds it itself and reads its constants from global memory)
    const int half = lane >> 5, l32 = lane & 31;
    v16i acc[TC][TP], acc1[TC][TP];
    static_for<TC>([&](auto tc_) {
        constexpr int tc = decltype(tc_)::value;
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            v4i b4 = {0, 0, 0, 0};
            if (EPI != EPI_ANY && kh == 0) b4 = *(const v4i*)(a.bias + c0 + wc * WTC + tc * 32 + g * 8 + half * 4);
            static_for<TP>([&](auto tp_) {
                constexpr int tp = decltype(tp_)::value;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    acc[tc][tp][g * 4 + e] = b4[e];
                    acc1[tc][tp][g * 4 + e] = 0;
                }
            });
        }
    });
    int* const cst = (int*)(lds + NST * STAGE);  // [3][BC]: clamp bound, multiplier, shift
    int cb_v = 0, cm_v = 0, cs_v = 0;
    if (EPI != EPI_ANY && tid < BC) {
        cb_v = EPI == EPI_FAST_RELU ? a.clamp_hi[c0 + tid] : 0;
        cm_v = a.mul[c0 + tid];
        cs_v = a.shift[c0 + tid];
    }

    typedef const void __attribute__((address_space(1))) * gptr_t;
    typedef void __attribute__((address_space(3))) * lptr_t;
    auto issue = [&](auto stage_, auto tap_, auto taps_) {
        constexpr int stage = decltype(stage_)::value, tap = decltype(tap_)::value, taps = decltype(taps_)::value;
        unsigned char* sb = lds + stage * STAGE + wave * (LPT * 1024);
        const unsigned at = taps == 9 ? pos + (tap / 3) * trow + (tap % 3) * tcol : pos;
#pragma unroll
        for (int u = 0; u < LPT; ++u)
            __builtin_amdgcn_global_load_lds((gptr_t)(sbase + (at + loff[u])), (lptr_t)(sb + u * 1024), 16, 0, 0);
        const unsigned nx = pos + (taps == 9 && tap == 8 ? inc + inc9 : inc);
        pos = nx < pos_last ? nx : pos_last;
    };
    if (a.taps == 9)
        static_for<NST - 1>([&](auto t_) { issue(t_, t_, std::integral_constant<int, 9>{}); });
    else
        static_for<NST - 1>([&](auto t_) { issue(t_, std::integral_constant<int, 0>{}, std::integral_constant<int, 1>{}); });
    if (EPI != EPI_ANY && tid < BC) {
        cst[tid] = cb_v;
        cst[BC + tid] = cm_v;
        cst[2 * BC + tid] = cs_v;
    }

    // fragment addresses: row l32 of each 32-row block, k-part (2 * k-step + half), swizzled as the loads put it
    const int sw = (l32 >> 2) & 3;
    const int off0 = (half ^ sw) * 16;
    const unsigned ldsa = (unsigned)(unsigned long long)(lptr_t)lds;
    unsigned wadr[KSTEPS][NB], aadr[KSTEPS][NB];
#pragma unroll
    for (int j = 0; j < KSTEPS; ++j)
#pragma unroll
        for (int b = 0; b < NB; ++b) {
            const int ks = KS == 2 ? kh : j;
            wadr[j][b] = ldsa + b * G * STAGE + (wc * WTC + l32) * KT + (off0 ^ (ks * 32));
            aadr[j][b] = ldsa + b * G * STAGE + BC * KT + (wp * WTP + l32) * KT + (off0 ^ (ks * 32));
        }
    v4i fw[3][KSTEPS * TC], fa[3][KSTEPS * TP];
    auto read_tile = [&](auto stage_, auto set_) {
        constexpr int stage = decltype(stage_)::value, set = decltype(set_)::value;
        static_for<KSTEPS>([&](auto j_) {
            constexpr int j = decltype(j_)::value;
            static_for<TC>([&](auto tc_) {
                constexpr int tc = decltype(tc_)::value;
                lds_read_b128<(stage % G) * STAGE + tc * 32 * KT>(fw[set][j * TC + tc], wadr[j][stage / G]);
            });
            static_for<TP>([&](auto tp_) {
                constexpr int tp = decltype(tp_)::value;
                lds_read_b128<(stage % G) * STAGE + tp * 32 * KT>(fa[set][j * TP + tp], aadr[j][stage / G]);
            });
        });
    };
    // k-tile number i of a round: with one group, k-step 0 adds into acc and k-step 1 into acc1; with two
    // groups a wave has one k-step per k-tile and alternates by k-tile
    auto mma_tile = [&](auto set_, auto i_) {
        constexpr int set = decltype(set_)::value, i = decltype(i_)::value;
        static_for<KSTEPS>([&](auto j_) {
            constexpr int j = decltype(j_)::value;
            constexpr int which = KS == 1 ? j : i % 2;
            static_for<TC>([&](auto tc_) {
                constexpr int tc = decltype(tc_)::value;
                static_for<TP>([&](auto tp_) {
                    constexpr int tp = decltype(tp_)::value;
                    if constexpr (which == 0)
                        acc[tc][tp] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fw[set][j * TC + tc], fa[set][j * TP + tp], acc[tc][tp], 0, 0, 0);
                    else
                        acc1[tc][tp] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fw[set][j * TC + tc], fa[set][j * TP + tp], acc1[tc][tp], 0, 0, 0);
                });
            });
        });
    };
    wait_tiles_then_barrier<(NST - 2) * LPT>();  // tile 0 has landed
    trace_stamp(a, bid, 1, tid);
    auto loop = [&](auto taps_) {
        constexpr int taps = decltype(taps_)::value;
        using I0 = std::integral_constant<int, 0>;
        using I1 = std::integral_constant<int, 1>;
        read_tile(I0{}, I0{});
        // tile 1 has landed (a repeat of tile 0 when there is only one), set 0 has arrived
        wait_tiles_then_barrier<(NST - 3) * LPT>();
        tie_frags(fw[0], fa[0]);
        read_tile(I1{}, I1{});
        for (int kt = 0; kt < nkt; kt += NST) {
            const int left = nkt - kt;
            static_for<NST>([&](auto i_) {
                constexpr int i = decltype(i_)::value;
                // (a 3x3 layer has whole rounds of nine k-tiles)
                if (taps == 9 || left > i) {
                    // tile kt+i+NST-1 goes into the stage of tile kt+i-1; its tap is (i + 8) mod 9
                    issue(std::integral_constant<int, (i + NST - 1) % NST>{},
                          std::integral_constant<int, taps == 9 ? (i + 8) % 9 : 0>{}, taps_);
                    // tile kt+i+2 has landed; of this wave's fragment reads only those of tile kt+i+1 may be pending
                    wait_frags_then_barrier<(NST - 3) * LPT, FR>(fw[i % 3], fa[i % 3]);
                    read_tile(std::integral_constant<int, (i + 2) % NST>{}, std::integral_constant<int, (i + 2) % 3>{});
                    mma_tile(std::integral_constant<int, i % 3>{}, i_);
                }
            });
        }
        // fragment reads past the last k-tile are still on their way to registers the compiler takes for free
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        tie_frags(fw[0], fa[0]);
        tie_frags(fw[1], fa[1]);
        tie_frags(fw[2], fa[2]);
    };
    if (a.taps == 9) loop(std::integral_constant<int, 9>{});
    else loop(std::integral_constant<int, 1>{});
    trace_stamp(a, bid, 2, tid);

    static_for<TC>([&](auto tc_) {
        constexpr int tc = decltype(tc_)::value;
        static_for<TP>([&](auto tp_) {
            constexpr int tp = decltype(tp_)::value;
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[tc][tp][r] += acc1[tc][tp][r];
        });
    });
    if constexpr (KS == 2) {
        // group 1 hands its sums to group 0 through the ring's LDS, once the loads issued past the last
        // k-tile have landed there for every wave (a workgroup then needs 74 KB and two share a CU):
        // 16 bytes per lane and register quad, lane-contiguous
        static_assert(NQ * TC * TP * 4096 <= NST * STAGE, "partial sums fit the ring");
        asm volatile("s_waitcnt vmcnt(0)\n\ts_barrier" ::: "memory");
        unsigned char* const red = lds + wq * (TC * TP * 4096) + lane * 16;
        if (kh == 1) {
            static_for<TC>([&](auto tc_) {
                constexpr int tc = decltype(tc_)::value;
                static_for<TP>([&](auto tp_) {
                    constexpr int tp = decltype(tp_)::value;
#pragma unroll
                    for (int g = 0; g < 4; ++g) {
                        v4i q;
#pragma unroll
                        for (int e = 0; e < 4; ++e) q[e] = acc[tc][tp][g * 4 + e];
                        *(v4i*)(red + ((tc * TP + tp) * 4 + g) * 1024) = q;
                    }
                });
            });
        }
        asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
        if (kh == 0) {
            static_for<TC>([&](auto tc_) {
                constexpr int tc = decltype(tc_)::value;
                static_for<TP>([&](auto tp_) {
                    constexpr int tp = decltype(tp_)::value;
#pragma unroll
                    for (int g = 0; g < 4; ++g) {
                        const v4i q = *(const v4i*)(red + ((tc * TP + tp) * 4 + g) * 1024);
#pragma unroll
                        for (int e = 0; e < 4; ++e) acc[tc][tp][g * 4 + e] += q[e];
                    }
                });
            });
        }
    }
    if (kh == 0) {
        if constexpr (EPI == EPI_FAST_RELU)
            conv_epilogue_fast<TC, TP, true>(a, acc, p0 + wp * WTP, c0 + wc * WTC, lane, hw, cst, BC, wc * WTC);
        else if constexpr (EPI == EPI_FAST)
            conv_epilogue_fast<TC, TP, false>(a, acc, p0 + wp * WTP, c0 + wc * WTC, lane, hw, cst, BC, wc * WTC);
        else
            conv_epilogue<TC, TP>(a, acc, p0 + wp * WTP, c0 + wc * WTC, lane, hw);
    }
    // the loads issued past the last k-tile must have landed before the wave retires and its LDS is reused
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    trace_stamp(a, bid, 3, tid);
}

// Persistent form of conv_igemm for launches with several output tiles per CU (fast epilogues only,
// no split-K, a k-tile count that is a multiple of NST x taps). One workgroup per CU walks the tiles
// blockIdx.x, blockIdx.x + gridDim.x, ... The stream of k-tiles runs on across output tiles: once
// the last k-tile of a tile has been issued the load pointers move to the workgroup's next tile, so
// the loads that conv_igemm spends on dead stages at the end of its k loop fetch the first k-tiles
// of the next output tile here, and these land while the epilogue runs. The epilogue's stores count
// on the same vmcnt as the tile loads; the waits do not depend on when they complete: tile loads
// retire in order among themselves, so while a k-tile has not landed, every tile load issued after
// it is outstanding too, and "at most (NST - 2) * LPT outstanding" cannot hold as long as at least
// that many tile loads were issued after the k-tile in question - which is the case at every wait,
// at the start of a tile included. Per-channel constants, the bias included, take the same road
// as the tiles: four 1 KB loads straight into one of two LDS buffers, issued right behind the last
// k-tile of the previous output tile, so they too are older than the next tile's k-tile 0.
template <int BC, int BP, int WC, int WP, int NST, int EPI>
__global__ __launch_bounds__(WC* WP * 64) void conv_igemm_persist(const ConvArgs a) {
    const int npb = (a.npix + BP - 1) / BP, ncb = a.n_pad / BC;  // pixel blocks, channel blocks
    static_assert(EPI != EPI_ANY, "fast epilogues only");
    static_assert(BC == 256 && WC * WP >= 4, "one wave-wide load per constant array");
    constexpr int NW = WC * WP;
    constexpr int WTC = BC / WC, WTP = BP / WP;
    constexpr int TC = WTC / 32, TP = WTP / 32;
    constexpr int WI = BC / 16 / NW, AI = BP / 16 / NW;
    constexpr int LPT = WI + AI;
    constexpr int STAGE = (BC + BP) * KT;
    static_assert(NST >= 3 && (NST - 2) * LPT < 64, "pipeline depth must fit the vmcnt counter");

    extern __shared__ __align__(1024) unsigned char lds[];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wc = wave % WC, wp = wave / WC;
    const int nkt = a.taps * (a.cin_pad / KT);  // a multiple of NST, and of 9 * NST for 3x3 layers (the launcher checks)
    const long long wtile = (long long)a.n_pad * KT;
    const int hw = a.h * a.w;
    const int W2 = a.w + 2, PP = (a.h + 2) * W2;

    // Tiles are numbered by slot as in conv_igemm (slot & 7 = XCD, whole pixel blocks per XCD);
    // gridDim.x is a multiple of 8, so a workgroup's slots stay on its XCD.
    const int nslots = ((npb + 7) / 8) * 8 * ncb;
    auto slot_tile = [&](int s, int& p0, int& c0) {
        const int xcd = s & 7, q = s >> 3;
        const int pb = (q / ncb) * 8 + xcd, cb = q % ncb;
        p0 = pb * BP;
        c0 = cb * BC;
        return pb < npb && c0 < a.n_store;
    };
    auto next_slot = [&](int s) {
        int p, c;
        while (s < nslots && !slot_tile(s, p, c)) s += (int)gridDim.x;
        return s;
    };
    int cur = next_slot((int)blockIdx.x);
    if (cur >= nslots) return;

    const int lrow = lane >> 2;
    const int lpart = (lane & 3) ^ ((lane >> 4) & 3);
    const unsigned woffl = (unsigned)(lrow * KT + lpart * 16);
    const int8_t* const abase = a.in + (long long)a.in_chunk0 * a.in_plane;

    typedef const void __attribute__((address_space(1))) * gptr_t;
    typedef void __attribute__((address_space(3))) * lptr_t;
    unsigned aoffl[AI];
    const int8_t* wt;
    const int8_t* at;
    int ld_slot, nx_slot;  // slot being loaded, next slot to load
    auto load_setup = [&](int s) {
        int p0, c0;
        slot_tile(s, p0, c0);
#pragma unroll
        for (int u = 0; u < AI; ++u) {
            int m = p0 + (wave * AI + u) * 16 + lrow;
            m = m < a.npix ? m : a.npix - 1;
            aoffl[u] = (unsigned)bordered_pos(a, m, hw, W2, PP) * KT + (unsigned)(lpart * 16);
        }
        wt = a.wgt + (long long)(c0 + wave * WI * 16) * KT;
        at = abase + (a.taps == 9 ? (long long)(-W2 - 1) * KT : 0LL);  // tap (0, 0) reads pixel (i - 1, j - 1)
        ld_slot = s;
    };
    auto uniform = [](const int8_t* p) {
        const unsigned long long v = (unsigned long long)p;
        const unsigned lo = __builtin_amdgcn_readfirstlane((unsigned)v);
        const unsigned hi = __builtin_amdgcn_readfirstlane((unsigned)(v >> 32));
        return (const int8_t*)(((unsigned long long)hi << 32) | lo);
    };
    // [2][4][BC] behind the ring: clamp bound (ReLU epilogue), multiplier, shift, bias of the channels of
    // the tile being computed and of the next one; wave w < 4 fetches array w
    int* const cstbuf = (int*)(lds + NST * STAGE);
    int ctile = 0;  // output tiles whose constants have been requested
    auto load_consts = [&](int s) {
        int p0, c0;
        slot_tile(s, p0, c0);
        if (wave < 4) {
            const int32_t* arr = wave == 0 ? (EPI == EPI_FAST_RELU ? a.clamp_hi : a.mul) : wave == 1 ? a.mul : wave == 2 ? a.shift : a.bias;
            const int8_t* src = uniform((const int8_t*)(arr + c0));
            __builtin_amdgcn_global_load_lds((gptr_t)(src + lane * 16), (lptr_t)(cstbuf + ((ctile & 1) * 4 + wave) * BC), 16, 0, 0);
        }
        ++ctile;
    };
    load_setup(cur);
    load_consts(cur);
    nx_slot = next_slot(cur + (int)gridDim.x);

    const int half = lane >> 5, l32 = lane & 31;
    const int sw = (l32 >> 2) & 3;
    const int off0 = (half ^ sw) * 16;
    const int wl0 = (wc * WTC + l32) * KT, al0 = BC * KT + (wp * WTP + l32) * KT;
    v16i acc[TC][TP];
    v4i wf0[TC], af0[TP], wf1[TC], af1[TP];
    // Fragment reads and the waits for them are placed by hand (lds_read_b128, wait_frags): left to the
    // compiler, every first use of a fragment is preceded by lgkmcnt(0), which also waits for the reads of
    // the next k-step issued just before, so both waves of a SIMD stall for an LDS latency twice per k-tile,
    // at about the same time since the barrier keeps them in step. A ds_read offset has 16 bits and a stage
    // 32 KB: one base address per operand, k-step and pair of stages.
    const unsigned ldsa = (unsigned)(unsigned long long)(lptr_t)lds;
    unsigned wadr[2][2], aadr[2][2];  // [k-step][stage pair]
#pragma unroll
    for (int ks = 0; ks < 2; ++ks)
#pragma unroll
        for (int sp = 0; sp < 2; ++sp) {
            wadr[ks][sp] = ldsa + sp * 2 * STAGE + wl0 + (off0 ^ (ks * 32));
            aadr[ks][sp] = ldsa + sp * 2 * STAGE + al0 + (off0 ^ (ks * 32));
        }
    static_assert(NST == 4 && STAGE + (TC > TP ? TC : TP) * 32 * KT <= 65536, "two stages per base address");
    auto read_frags = [&](auto stage_, auto ks_, v4i (&wf)[TC], v4i (&af)[TP]) {
        constexpr int stage = decltype(stage_)::value, ks = decltype(ks_)::value;
        static_for<TC>([&](auto tc_) {
            constexpr int tc = decltype(tc_)::value;
            lds_read_b128<(stage & 1) * STAGE + tc * 32 * KT>(wf[tc], wadr[ks][stage >> 1]);
        });
        static_for<TP>([&](auto tp_) {
            constexpr int tp = decltype(tp_)::value;
            lds_read_b128<(stage & 1) * STAGE + tp * 32 * KT>(af[tp], aadr[ks][stage >> 1]);
        });
    };
    constexpr int FR = TC + TP;  // fragment reads per k-step
    auto mma = [&](v4i (&wf)[TC], v4i (&af)[TP]) {
        static_for<TC>([&](auto tc_) {
            constexpr int tc = decltype(tc_)::value;
            static_for<TP>([&](auto tp_) {
                constexpr int tp = decltype(tp_)::value;
                acc[tc][tp] = __builtin_amdgcn_mfma_i32_32x32x32_i8(wf[tc], af[tp], acc[tc][tp], 0, 0, 0);
            });
        });
    };

    // The k loop is unrolled over both the ring (NST stages) and the filter taps, U = lcm(NST, taps) steps, so
    // that the LDS stage and the tap of every load are compile-time constants and a step has no branch:
    // a tap's address is the plane pointer plus a loop-invariant scalar, the weights advance by one k-tile,
    // the plane pointer moves on after tap 8. The switch to the workgroup's next output tile (a division or
    // two, the constants' loads) happens at one fixed step of the last round, NST - 1 steps before the end,
    // which is where the load stream crosses into the next tile. With the bookkeeping out of the way the
    // compiler spreads the remaining scalar instructions between the MFMAs instead of leaving them as one
    // block between the last MFMA and the barrier, where both waves of a SIMD used to execute them at the
    // same time with the matrix pipe idle.
    const long long rowstep = (long long)W2 * KT;
    auto issue_static = [&](auto stage_, auto tap_, auto taps_) {
        constexpr int stage = decltype(stage_)::value, tap = decltype(tap_)::value, taps = decltype(taps_)::value;
        unsigned char* sb = lds + stage * STAGE;
        const int8_t* wu = uniform(wt);
#pragma unroll
        for (int u = 0; u < WI; ++u)
            __builtin_amdgcn_global_load_lds((gptr_t)(wu + u * 1024 + woffl), (lptr_t)(sb + (wave * WI + u) * 1024), 16,
                                             0, 0);
        // (the load's immediate offset would shift the LDS address as well, so the tap's offset joins the pointer)
        const int8_t* au = uniform(at + (taps == 9 ? (tap / 3) * rowstep + (tap % 3) * KT : 0LL));
#pragma unroll
        for (int u = 0; u < AI; ++u)
            __builtin_amdgcn_global_load_lds((gptr_t)(au + aoffl[u]), (lptr_t)(sb + BC * KT + (wave * AI + u) * 1024),
                                             16, 0, 0);
        wt += wtile;
        if constexpr (taps == 1 || tap == 8) at += a.in_plane;
    };
    // once per output tile: on to this workgroup's next slot; after the last one the same tile is loaded
    // again into stages nobody reads, which keeps the loads per step constant and every address valid
    auto switch_tile = [&]() {
        const int s = nx_slot < nslots ? nx_slot : ld_slot;
        if (nx_slot < nslots) nx_slot = next_slot(nx_slot + (int)gridDim.x);
        load_setup(s);
        load_consts(s);
    };
    auto run = [&](auto taps_) {
        constexpr int taps = decltype(taps_)::value;
        constexpr int U = taps == 9 ? 9 * NST : NST;   // nkt is a multiple of U (the launcher checks)
        static_for<NST - 1>([&](auto t_) { issue_static(t_, std::integral_constant<int, taps == 9 ? decltype(t_)::value : 0>{}, taps_); });
        for (int n = 0;; ++n) {
            int p0, c0;
            slot_tile(cur, p0, c0);
            int* const cst = cstbuf + (n & 1) * 4 * BC;
            trace_stamp(a, cur, 0, tid);
            // k-tile 0 of this output tile and, before it, its constants have landed (first tile: just
            // issued; later tiles: issued during the previous k loop)
            wait_tiles_then_barrier<(NST - 2) * LPT>();
            trace_stamp(a, cur, 1, tid);
            // accumulators start at the bias (the fast epilogues expect it there)
            static_for<TC>([&](auto tc_) {
                constexpr int tc = decltype(tc_)::value;
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const v4i b4 = *(const v4i*)(cst + 3 * BC + wc * WTC + tc * 32 + g * 8 + half * 4);
                    static_for<TP>([&](auto tp_) {
                        constexpr int tp = decltype(tp_)::value;
#pragma unroll
                        for (int e = 0; e < 4; ++e) acc[tc][tp][g * 4 + e] = b4[e];
                    });
                }
            });
            using I0 = std::integral_constant<int, 0>;
            using I1 = std::integral_constant<int, 1>;
            read_frags(I0{}, I0{}, wf0, af0);
            for (int kt = 0; kt < nkt; kt += U) {
                static_for<U>([&](auto i_) {
                    constexpr int i = decltype(i_)::value;
                    constexpr int st = i % NST;
                    // second k-step's fragments on their way while the first k-step multiplies
                    read_frags(std::integral_constant<int, st>{}, I1{}, wf1, af1);
                    wait_frags<FR>(wf0, af0);
                    mma(wf0, af0);
                    // k-tile kt + i + NST - 1 of the load stream goes into the stage of k-tile kt + i - 1;
                    // in the last round that stream reaches the end of this output tile at step U - NST + 1
                    if constexpr (i == U - NST + 1) {
                        if (kt + U >= nkt) switch_tile();
                    }
                    issue_static(std::integral_constant<int, (i + NST - 1) % NST>{},
                                 std::integral_constant<int, taps == 9 ? (i + NST - 1) % 9 : 0>{}, taps_);
                    // (lgkmcnt(0): nobody still reads the stage that the next step's loads overwrite)
                    wait_tiles_then_barrier<(NST - 2) * LPT>();
                    tie_frags(wf1, af1);
                    read_frags(std::integral_constant<int, (st + 1) % NST>{}, I0{}, wf0, af0);
                    mma(wf1, af1);
                });
            }
            // the reads of the next tile's first fragments are still on their way to registers that the
            // epilogue is free to use
            wait_frags<0>(wf0, af0);
            const int nxt = next_slot(cur + (int)gridDim.x);
            trace_stamp(a, cur, 2, tid);
            if constexpr (EPI == EPI_FAST_RELU)
                conv_epilogue_fast<TC, TP, true>(a, acc, p0 + wp * WTP, c0 + wc * WTC, lane, hw, cst, BC, wc * WTC);
            else
                conv_epilogue_fast<TC, TP, false>(a, acc, p0 + wp * WTP, c0 + wc * WTC, lane, hw, cst, BC, wc * WTC);
            trace_stamp(a, cur, 3, tid);
            if (nxt >= nslots) break;
            cur = nxt;
        }
    };
    if (a.taps == 9) run(std::integral_constant<int, 9>{});
    else run(std::integral_constant<int, 1>{});
    // drain the tail loads (they target stages nobody reads any more) before the wave retires
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
}

// Second phase of a split-K layer: requantise the summed accumulators, apply the layer's
// mode, and leave the scratch zeroed for the next user. One thread per (pixel, channel).
__global__ void conv_splitk_finish(const ConvArgs a) {
    const int hw = a.h * a.w;
    const long long n = (long long)a.npix * a.n_store;
    for (long long t = blockIdx.x * (long long)blockDim.x + threadIdx.x; t < n; t += (long long)gridDim.x * blockDim.x) {
        const int m = (int)(t / a.n_store), c = (int)(t - (long long)m * a.n_store);
        int32_t* ps = a.partial + (long long)m * a.n_pad + c;
        const int av = *ps + a.bias[c];
        *ps = 0;
        int y = rq_dev(av, a.mul[c], a.shift[c] + (a.rq_fast ? 32 : 0));
        if (a.mode == MODE_ACT) {
            const int ch = c;
            const int bi = m / hw, qi = m - bi * hw, ii = qi / a.w, ji = qi - ii * a.w;
            const long long pp = (long long)bi * ((a.h + 2) * (a.w + 2)) + (ii + 1) * (a.w + 2) + (ji + 1);
            int8_t* o = a.out + (long long)(a.out_chunk0 + (ch >> 6)) * a.out_plane + pp * 64 + (ch & 63);
            if (a.shortcut) y += (int)*o + (a.sc_unsigned ? 128 : 0);
            if (a.relu) y = y < 0 ? 0 : y;
            *o = (int8_t)(a.out_unsigned ? (y > 255 ? 255 : y) - 128 : sat8_dev(y));
        } else if (a.mode == MODE_COUPLE) {
            if (a.relu) y = y < 0 ? 0 : y;
            a.state[(long long)m * a.state_c + a.idx_b[c]] += a.sign * sat8_dev(y);
        } else {
            if (a.relu) y = y < 0 ? 0 : y;
            const int b = m / hw, q = m - b * hw;
            a.codes[(long long)b * a.codes_img_stride + a.codes_off + (long long)c * hw + q] = (int8_t)sat8_dev(y);
        }
    }
}

namespace {

struct TileCfg {
    int bc, bp;
    size_t lds;
    void (*kern[3])(const ConvArgs);  // indexed by EPI_*
    int threads;
    const char* name;
};

#define IODF_TILE(BC, BP, WC, WP, NST)                                                              \
    TileCfg {                                                                                       \
        BC, BP, (size_t)NST * (BC + BP) * KT + 3 * BC * sizeof(int),                                 \
            {conv_igemm<BC, BP, WC, WP, NST, EPI_ANY>, conv_igemm<BC, BP, WC, WP, NST, EPI_FAST>,   \
             conv_igemm<BC, BP, WC, WP, NST, EPI_FAST_RELU>},                                       \
            WC * WP * 64,                                                                           \
            "conv_igemm<" #BC "," #BP "," #WC "," #WP "," #NST ">"                                  \
    }

const TileCfg kTiles[] = {
    IODF_TILE(256, 256, 2, 4, 4),
    IODF_TILE(128, 512, 2, 4, 3),
    IODF_TILE(128, 128, 4, 2, 4),
    IODF_TILE(64, 256, 1, 4, 4),
    IODF_TILE(64, 64, 2, 2, 9),
    // four-wave halves of the first two tiles: 72 KB of LDS and at most 256 registers, so two
    // workgroups share a CU (see conv_pick_tile)
    IODF_TILE(256, 128, 2, 2, 3),
    IODF_TILE(128, 256, 2, 2, 3),
    // lean forms of the 64x64 tile (eight waves, the k-steps split between two groups of four) and of the
    // 128x128 tile for layers whose reduction is not split (see conv_igemm_lean)
    TileCfg{64, 64, (size_t)9 * (64 + 64) * KT + 2048,
            {conv_igemm_lean<64, 64, 2, 2, 2, EPI_ANY>, conv_igemm_lean<64, 64, 2, 2, 2, EPI_FAST>, conv_igemm_lean<64, 64, 2, 2, 2, EPI_FAST_RELU>},
            512, "conv_igemm_lean<64,64,2,2,2>"},
    TileCfg{128, 128, (size_t)9 * (128 + 128) * KT + 2048,
            {conv_igemm_lean<128, 128, 4, 2, 1, EPI_ANY>, conv_igemm_lean<128, 128, 4, 2, 1, EPI_FAST>, conv_igemm_lean<128, 128, 4, 2, 1, EPI_FAST_RELU>},
            512, "conv_igemm_lean<128,128,4,2,1>"},
};
constexpr int kNumTiles = sizeof(kTiles) / sizeof(kTiles[0]);
constexpr int kPair256 = 5, kPair128 = 6;  // the two-workgroups-per-CU halves of tiles 0 and 1
constexpr int kSmall = 4, kSmallLean = 7, kMid = 2, kMidLean = 8;  // the 64x64 and 128x128 tiles and their lean forms

// Persistent form of tile 0 (see conv_igemm_persist), by fast epilogue, and its LDS bytes.
void (*const kPersist[3])(const ConvArgs) = {nullptr, conv_igemm_persist<256, 256, 2, 4, 4, EPI_FAST>,
                                                        conv_igemm_persist<256, 256, 2, 4, 4, EPI_FAST_RELU>};
constexpr size_t kPersistLds = (size_t)4 * (256 + 256) * KT + 2 * 4 * 256 * sizeof(int);
constexpr int kPersistTile = kNumTiles;  // what conv_pick_tile answers for a persistent launch of tile 0

// Workgroups of a persistent launch: one per compute unit of the device the layer runs on, a
// multiple of 8 so that a workgroup's tiles stay on its XCD.
int persist_grid(const ConvArgs& a) { return a.n_cu / 8 * 8; }

bool args_ok(const ConvArgs& a) {
    return !(a.cin_pad <= 0 || a.cin_pad % KT || a.n_pad <= 0 || a.n_pad % 64 || (a.taps != 1 && a.taps != 9) ||
             a.in_plane < (long long)(a.npix / (a.h * a.w)) * (a.h + 2) * (a.w + 2) * KT || a.in_plane % 1024 ||
             a.in_plane >= (1u << 31) || a.n_store > a.n_pad ||
             a.n_store < 1 || a.h < 1 || a.w < 1 || a.npix % (a.h * a.w) || !a.in || !a.wgt || !a.bias || !a.mul ||
             !a.shift ||
             (a.mode == MODE_ACT &&
              (!a.out || a.out_plane < (long long)(a.npix / (a.h * a.w)) * (a.h + 2) * (a.w + 2) * KT ||
               a.out_plane % 64)) ||
             (a.mode == MODE_COUPLE && (!a.state || !a.idx_b || a.state_c < 1)) ||
             (a.mode == MODE_CODES && !a.codes) || (a.mode == MODE_RAW && !a.partial) || a.mode > MODE_RAW);
}

}  // namespace

hipError_t conv_setup() {
    for (int i = 0; i < kNumTiles; ++i) {
        for (int v = 0; v < 3; ++v) {
            if (!kTiles[i].kern[v]) continue;
            hipError_t e = hipFuncSetAttribute((const void*)kTiles[i].kern[v],
                                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)kTiles[i].lds);
            if (e != hipSuccess) return e;
        }
    }
    for (int v = 1; v < 3; ++v) {
        hipError_t e = hipFuncSetAttribute((const void*)kPersist[v], hipFuncAttributeMaxDynamicSharedMemorySize,
                                           (int)kPersistLds);
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

hipError_t conv_device_cus(int* n_cu) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e == hipSuccess) e = hipDeviceGetAttribute(n_cu, hipDeviceAttributeMultiprocessorCount, dev);
    return e;
}

int conv_num_tiles() { return kNumTiles + 1; }
const char* conv_tile_name(int tile) {
    if (tile == kPersistTile) return "conv_igemm_persist<256,256,2,4,4>";
    return tile >= 0 && tile < kNumTiles ? kTiles[tile].name : "?";
}
void conv_tile_dims(int tile, int* bc, int* bp) {
    if (tile == kPersistTile) tile = 0;
    const bool ok = tile >= 0 && tile < kNumTiles;
    *bc = ok ? kTiles[tile].bc : 0;
    *bp = ok ? kTiles[tile].bp : 0;
}

int conv_pick_splits(const ConvArgs& a, int tile);

// Epilogue variant a layer runs with.
int pick_epi(const ConvArgs& a) {
    const bool fast = a.mode == MODE_ACT && a.rq_fast && a.n_store % 16 == 0;
    // EPI_FAST covers signed codes, and unsigned ones only where shortcut and result share the format
    const bool fast_signed_ok = a.shortcut ? a.sc_unsigned == a.out_unsigned : !a.out_unsigned;
    return !fast ? EPI_ANY : (a.relu && !a.shortcut && a.clamp_hi) ? EPI_FAST_RELU : fast_signed_ok ? EPI_FAST : EPI_ANY;
}

// Whether the 256x256 tile runs in its persistent form: a tile or more per CU, a fast epilogue and a k-tile
// count that is a whole number of the kernel's unrolled rounds (ring stages x taps). With one tile per
// workgroup nothing is left to overlap, but its branch-free k loop and its constants by DMA still make it
// the faster form (2 % on 3x3 layers, 3-8 % on 1x1 layers).
bool persist_ok(const ConvArgs& a, long long tiles) {
    const int nkt = a.taps * (a.cin_pad / KT);
    return pick_epi(a) != EPI_ANY && nkt % (a.taps == 9 ? 36 : 4) == 0 && persist_grid(a) >= 8 &&
           tiles >= (long long)persist_grid(a);
}

// First tile in table order that still fills the chip (its two-per-CU half when the reduction is
// short); otherwise the valid tile with most workgroups, and among equals the one that multiplies
// the least padding.
static int pick_tile_by_shape(const ConvArgs& a) {
    if (!args_ok(a)) return -1;
    int best = -1;
    long long best_blocks = -1, best_work = 0;
    for (int i = 0; i < kPair256; ++i) {
        if (a.n_pad % kTiles[i].bc) continue;
        const long long blocks = (long long)((a.npix + kTiles[i].bp - 1) / kTiles[i].bp) *
                                 ((a.n_store + kTiles[i].bc - 1) / kTiles[i].bc);
        if (blocks >= 256) {
            // Short reductions: the fixed cost of a tile (first loads, epilogue) outweighs its k-loop.
            // Two half-size workgroups per CU let one's epilogue run under the other's matrix work;
            // worth it only when the big tile would take more than one round and K is short, and only
            // where the big tile cannot run in its persistent form, which hides the same cost better.
            const int alt = i == 0 ? kPair256 : i == 1 ? kPair128 : -1;
            const int nkt = a.taps * (a.cin_pad / KT);
            const int ncb = a.n_pad / kTiles[i].bc;
            if (i == 0 && conv_pick_splits(a, 0) == 1 && persist_ok(a, blocks)) return kPersistTile;
            if (alt >= 0 && blocks > 256 && nkt <= (i == 1 ? 18 : ncb >= 2 ? 16 : 12)) return alt;
            return i;
        }
        const long long work = blocks * kTiles[i].bc * kTiles[i].bp;
        if (blocks > best_blocks || (blocks == best_blocks && work < best_work)) {
            best_blocks = blocks;
            best_work = work;
            best = i;
        }
    }
    return best;
}

int conv_pick_tile(const ConvArgs& a) {
    const int t = pick_tile_by_shape(a);
    // unsplit reductions on the 64x64 and 128x128 tiles take the lean kernel
    // (its load streams keep 32-bit positions)
    const long long nkt = (long long)a.taps * (a.cin_pad / KT);
    const bool fits = nkt * a.n_pad * KT < (1LL << 32) && (long long)(a.cin_pad / KT) * a.in_plane < (1LL << 32);
    if (!fits || (t != kSmall && t != kMid) || conv_pick_splits(a, t) != 1) return t;
    if (t == kSmall) return kSmallLean;
    // the lean 128x128 form fills the LDS of a CU; with more tiles than CUs the four-stage form, two to a CU, is
    // the better one (a second workgroup's loads and epilogue run under the first one's matrix work)
    const long long blocks = (long long)((a.npix + 127) / 128) * ((a.n_store + 127) / 128);
    return blocks <= a.n_cu ? kMidLean : t;
}

// K splits for a layer whose tiles alone cannot fill the chip (only the general epilogue
// supports it, and only when the caller supplied the scratch).
int conv_pick_splits(const ConvArgs& a, int tile) {
    if (a.mode == MODE_RAW || tile == kPersistTile) return 1;  // raw: the scratch is written, not accumulated
    const bool fast = a.mode == MODE_ACT && a.rq_fast && a.n_store % 16 == 0;
    if (fast || !a.partial || tile < 0) return 1;
    const TileCfg& t = kTiles[tile];
    const long long blocks = (long long)((a.npix + t.bp - 1) / t.bp) * ((a.n_store + t.bc - 1) / t.bc);
    const int nkt = a.taps * (a.cin_pad / KT);
    long long s = 512 / (blocks > 0 ? blocks : 1);
    if (s > nkt / 16) s = nkt / 16;
    if (s > 32) s = 32;
    return s < 2 ? 1 : (int)s;
}

int conv_trace_slots(const ConvArgs& a) {
    const int best = conv_pick_tile(a);
    if (best < 0) return 0;
    const TileCfg& t = kTiles[best == kPersistTile ? 0 : best];
    const int npb = (a.npix + t.bp - 1) / t.bp, ncb = a.n_pad / t.bc;
    return ((npb + 7) / 8) * 8 * ncb;
}

hipError_t launch_conv(const ConvArgs& a_in, hipStream_t stream) {
    ConvArgs a = a_in;
    {
        auto lg = [](int v) { int l = 0; while ((1 << l) < v) ++l; return (1 << l) == v ? l : -1; };
        a.log2_w = lg(a.w);
        a.log2_hw = a.log2_w >= 0 ? lg(a.h * a.w) : -1;
    }
    if (a.npix <= 0) return hipSuccess;
    const int best = conv_pick_tile(a);
    if (best < 0) return hipErrorInvalidValue;
    const bool persist = best == kPersistTile;
    const TileCfg& t = kTiles[persist ? 0 : best];
    const int npb = (a.npix + t.bp - 1) / t.bp, ncb = a.n_pad / t.bc;
    const int grid = ((npb + 7) / 8) * 8 * ncb;
    const int epi = pick_epi(a);
    const int splits = conv_pick_splits(a, best);
    // A tile or more per CU, a fast epilogue and whole rounds of the stage ring: one resident
    // workgroup per CU walks its tiles and overlaps each tile's first loads with the epilogue before it.
    if (persist) {
        hipLaunchKernelGGL(kPersist[epi], dim3(persist_grid(a)), dim3(t.threads), kPersistLds, stream, a);
        return hipGetLastError();
    }
    // few tiles, and the next launch's first reads known: eight more workgroups per XCD fetch them (lean kernel only;
    // measured at batch 1 of the gate-pruned flow: 8, 16, 32, 64, 128 extra workgroups give 4.71, 3.77, 3.55, 3.51, 3.50 ms)
    const bool lean_tile = best == kSmallLean || best == kMidLean;
    const int pf_grid = lean_tile && !a.has_trace && a.pf && a.pf_bytes > 0 && (long long)npb * ncb <= 64 ? 64 : 0;
    hipLaunchKernelGGL(t.kern[epi], dim3(grid + pf_grid, splits), dim3(t.threads), t.lds, stream, a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || splits == 1) return e;
    const long long n = (long long)a.npix * a.n_store;
    const int fgrid = (int)((n + 255) / 256 > 4096 ? 4096 : (n + 255) / 256);
    hipLaunchKernelGGL(conv_splitk_finish, dim3(fgrid), dim3(256), 0, stream, a);
    return hipGetLastError();
}

namespace {

__global__ void conv_tapsum(const TapSumArgs a) {
    const int hw = a.h * a.w;
    const long long n = (long long)a.npix * a.c_out;
    for (long long t = blockIdx.x * (long long)blockDim.x + threadIdx.x; t < n; t += (long long)gridDim.x * blockDim.x) {
        const int m = (int)(t / a.c_out), c = (int)(t - (long long)m * a.c_out);
        const int b = m / hw, q = m - b * hw, i = q / a.w, j = q - i * a.w;
        // the state word this thread updates: its address hangs on the channel map, so both loads start
        // before the taps are summed rather than behind them
        int32_t* sp = nullptr;
        int sv = 0;
        const int mul = a.mul[c], shift = a.shift[c];
        if (a.mode == MODE_COUPLE) {
            sp = a.state + (long long)m * a.state_c + a.idx_b[c];
            sv = *sp;
        }
        int acc = a.bias[c];
#pragma unroll
        for (int tap = 0; tap < 9; ++tap) {
            const int ii = i + tap / 3 - 1, jj = j + tap % 3 - 1;
            if (ii >= 0 && ii < a.h && jj >= 0 && jj < a.w)
                acc += a.y[((long long)b * hw + ii * a.w + jj) * a.n_pad + tap * a.c_out + c];
        }
        int y = rq_dev(acc, mul, shift);
        if (a.relu) y = y < 0 ? 0 : y;
        y = sat8_dev(y);
        if (a.mode == MODE_COUPLE)
            *sp = sv + a.sign * y;
        else
            a.codes[(long long)b * a.codes_img_stride + a.codes_off + (long long)c * hw + q] = (int8_t)y;
    }
}

}  // namespace

hipError_t launch_tapsum(const TapSumArgs& a, hipStream_t stream) {
    if (a.npix <= 0) return hipSuccess;
    if (!a.y || !a.bias || !a.mul || !a.shift || a.c_out < 1 || 9 * a.c_out > a.n_pad || a.h < 1 || a.w < 1 ||
        a.npix % (a.h * a.w) || (a.mode == MODE_COUPLE && (!a.state || !a.idx_b)) ||
        (a.mode == MODE_CODES && !a.codes) || (a.mode != MODE_COUPLE && a.mode != MODE_CODES))
        return hipErrorInvalidValue;
    const long long n = (long long)a.npix * a.c_out;
    const int grid = (int)((n + 255) / 256 > 8192 ? 8192 : (n + 255) / 256);
    hipLaunchKernelGGL(conv_tapsum, dim3(grid), dim3(256), 0, stream, a);
    return hipGetLastError();
}

}  // namespace iodf
