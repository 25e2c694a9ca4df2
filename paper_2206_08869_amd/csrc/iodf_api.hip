// C ABI of libiodf: model-blob parsing, gate compaction and weight packing at
// init (Sec. 4.4: gated-off filters and their consumers' input columns are removed),
// and the encode / decode drivers that replay the couplings (Sec. 3, Eq. 1).
#include "../../include/iodf.h"

#include <hip/hip_runtime.h>

#include <algorithm>
#include <array>
#include <climits>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>
#include <string>
#include <vector>

#include "codec_kernels.h"
#include "conv.h"
#include "flow_kernels.h"

using namespace iodf;

namespace {

thread_local int g_last_hip = 0;

#define HIP_TRY(expr)                         \
    do {                                      \
        hipError_t e__ = (expr);              \
        if (e__ != hipSuccess) {              \
            g_last_hip = (int)e__;            \
            return IODF_E_HIP;                \
        }                                     \
    } while (0)

enum { FAM_PLAIN = 0, FAM_RESNET = 1, FAM_DENSE = 2 };
enum { BUF_XQ = 0, BUF_A = 1, BUF_B = 2, NUM_BUFS = 3 };

int round64(int n) { return (n + 63) / 64 * 64; }

// ---- blob (host side view) -------------------------------------------------------

struct HostLayer {
    int C_out, C_in, k, relu, shortcut;
    const int8_t* W;
    const int32_t* bias;
    const int32_t* M;
    const uint8_t* shift;
    const uint8_t* gate;
};

struct HostNet {
    int kind, level, C, C_in, C_out;
    int32_t M_in;
    int s_in;
    const int32_t* perm;
    std::vector<HostLayer> layers;
};

struct HostModel {
    int H, W, levels, couplings, family, width, depth, has_heads;
    int act_unsigned;  // tensors that leave a ReLU hold unsigned codes 0..255 (Eq. 3)
    std::vector<HostNet> nets;
};

size_t pad4(size_t n) { return (n + 3) & ~(size_t)3; }

int parse_blob(const uint8_t* p, size_t bytes, HostModel& m) {
    if (bytes < 64 || ((uintptr_t)p & 3)) return IODF_E_BLOB;
    const uint32_t* h = (const uint32_t*)p;
    if (h[0] != 0x46444F49u || h[1] != 0x31424C42u || h[2] != 1u) return IODF_E_BLOB;
    m.H = (int)h[3]; m.W = (int)h[4]; m.levels = (int)h[5]; m.couplings = (int)h[6]; m.family = (int)h[7];
    m.width = (int)h[8]; m.depth = (int)h[9]; m.has_heads = (int)h[10];
    const uint32_t n_nets = h[11];
    if (h[12] > 1u || h[13] || h[14] || h[15]) return IODF_E_BLOB;  // unknown format flags
    m.act_unsigned = (int)h[12];
    if (m.levels < 1 || m.levels > 8 || m.couplings < 1 || m.couplings > 1024 || m.H < 2 || m.W < 2 || m.H > 8192 ||
        m.W > 8192 || (m.H % (1 << m.levels)) || (m.W % (1 << m.levels)) || m.family < 0 || m.family > 2 ||
        m.has_heads > 1 || m.has_heads < 0)
        return IODF_E_BLOB;
    const uint32_t expect = (uint32_t)(m.levels * m.couplings + (m.has_heads ? m.levels - 1 : 0));
    if (n_nets != expect) return IODF_E_SHAPE;
    size_t pos = 64;
    auto need = [&](size_t n) { return pos + n <= bytes && pos + n >= pos; };
    m.nets.resize(n_nets);
    for (uint32_t n = 0; n < n_nets; ++n) {
        HostNet& net = m.nets[n];
        if (!need(32)) return IODF_E_BLOB;
        const uint32_t* f = (const uint32_t*)(p + pos);
        net.kind = (int)f[0]; net.level = (int)f[1]; net.C = (int)f[2]; net.C_in = (int)f[3]; net.C_out = (int)f[4];
        const uint32_t n_layers = f[5];
        net.M_in = (int32_t)f[6];
        net.s_in = (int)f[7];
        pos += 32;
        if (net.kind < 0 || net.kind > 1 || n_layers < 2 || n_layers > 4096 || f[7] > 62 || net.M_in < 0 ||
            net.C < 2 || net.C > 4096 || net.C_in < 1 || net.C_in > 4096 || net.C_out < 1 || net.C_out > 4096)
            return IODF_E_BLOB;
        net.perm = nullptr;
        if (net.kind == 0) {
            if (!need(4 * (size_t)net.C)) return IODF_E_BLOB;
            net.perm = (const int32_t*)(p + pos);
            pos += 4 * (size_t)net.C;
            std::vector<char> seen(net.C, 0);
            for (int c = 0; c < net.C; ++c) {
                const int32_t pc = net.perm[c];
                if (pc < 0 || pc >= net.C || seen[pc]) return IODF_E_BLOB;
                seen[pc] = 1;
            }
        }
        net.layers.resize(n_layers);
        for (uint32_t l = 0; l < n_layers; ++l) {
            HostLayer& L = net.layers[l];
            if (!need(16)) return IODF_E_BLOB;
            const uint32_t* g = (const uint32_t*)(p + pos);
            pos += 16;
            if (g[0] < 1 || g[0] > 65536 || g[1] < 1 || g[1] > 65536 || (g[2] != 1 && g[2] != 3)) return IODF_E_BLOB;
            L.C_out = (int)g[0]; L.C_in = (int)g[1]; L.k = (int)g[2];
            L.relu = (int)(g[3] & 1u);
            L.shortcut = (int)((g[3] >> 1) & 1u);
            const size_t nw = (size_t)L.C_out * L.C_in * L.k * L.k;
            const size_t co = (size_t)L.C_out;
            if (!need(pad4(nw))) return IODF_E_BLOB;
            L.W = (const int8_t*)(p + pos); pos += pad4(nw);
            if (!need(4 * co)) return IODF_E_BLOB;
            L.bias = (const int32_t*)(p + pos); pos += 4 * co;
            if (!need(4 * co)) return IODF_E_BLOB;
            L.M = (const int32_t*)(p + pos); pos += 4 * co;
            if (!need(pad4(co))) return IODF_E_BLOB;
            L.shift = p + pos; pos += pad4(co);
            if (!need(pad4(co))) return IODF_E_BLOB;
            L.gate = p + pos; pos += pad4(co);
            int kept = 0;
            for (int c = 0; c < L.C_out; ++c) {
                if (L.shift[c] > 62 || L.M[c] < 0 || L.gate[c] > 1) return IODF_E_BLOB;
                if (L.bias[c] >= (1 << 30) || L.bias[c] <= -(1 << 30)) return IODF_E_BLOB;
                kept += L.gate[c];
            }
            if (kept == 0) return IODF_E_BLOB;  // a layer with every filter gated off has no output at all
        }
    }
    if (pos != bytes) return IODF_E_BLOB;
    return IODF_OK;
}

int level_channels(int lv) { return 12 << (lv - 1); }

// Check that the networks fit the flow structure and their family's wiring.
int check_shapes(const HostModel& m) {
    size_t n = 0;
    for (int lv = 1; lv <= m.levels; ++lv) {
        const int C = level_channels(lv);
        for (int k = 0; k < m.couplings; ++k, ++n) {
            const HostNet& N = m.nets[n];
            if (N.kind != 0 || N.level != lv || N.C != C || N.C_in != C / 2 || N.C_out != C - C / 2) return IODF_E_SHAPE;
        }
        if (m.has_heads && lv < m.levels) {
            const HostNet& N = m.nets[n++];
            if (N.kind != 1 || N.level != lv || N.C != C || N.C_in != C / 2 || N.C_out != 2 * (C - C / 2))
                return IODF_E_SHAPE;
        }
    }
    for (const HostNet& N : m.nets) {
        const std::vector<HostLayer>& L = N.layers;
        const int nl = (int)L.size();
        if (L[0].C_in != N.C_in || L[0].k != 3 || L[nl - 1].C_out != N.C_out || L[nl - 1].shortcut || L[0].shortcut)
            return IODF_E_SHAPE;
        for (int c = 0; c < N.C_out; ++c)
            if (!L[nl - 1].gate[c]) return IODF_E_SHAPE;  // the translation / code channels cannot be gated
        // unsigned format: every hidden tensor must leave a ReLU (one format per activation buffer),
        // the translation / codes stay signed
        if (m.act_unsigned) {
            for (int l = 0; l + 1 < nl; ++l)
                if (!L[l].relu) return IODF_E_SHAPE;
            if (L[nl - 1].relu) return IODF_E_SHAPE;
        }
        // Eq. 4-5 accumulate in 32 bits: refuse a layer whose accumulator could leave int32 for some
        // input. Input codes are below 128 in magnitude (256 for unsigned codes, whose stored form adds
        // 128 * sum(w) to the bias); the first layer of a network always reads signed codes.
        for (int l = 0; l < nl; ++l) {
            const long long xmax = (m.act_unsigned && l > 0) ? 256 : 128;
            const long long K = (long long)L[l].C_in * L[l].k * L[l].k;
            if (K * 127 * xmax + (1LL << 30) < (1LL << 31)) continue;  // cannot overflow whatever the weights
            for (int c = 0; c < L[l].C_out; ++c) {
                long long sum = 0;
                const int8_t* w = L[l].W + (size_t)c * K;
                for (long long i = 0; i < K; ++i) sum += w[i] < 0 ? -(long long)w[i] : w[i];
                const long long b = L[l].bias[c] < 0 ? -(long long)L[l].bias[c] : L[l].bias[c];
                if (sum * xmax + b >= (1LL << 31)) return IODF_E_BLOB;
            }
        }
        const int Wd = L[0].C_out;
        if (m.family == FAM_PLAIN) {
            if (nl != 2 || L[1].C_in != Wd) return IODF_E_SHAPE;
        } else if (m.family == FAM_RESNET) {
            if (nl % 2) return IODF_E_SHAPE;
            for (int l = 1; l + 1 < nl; l += 2) {
                if (L[l].C_in != Wd || L[l].shortcut || L[l + 1].C_in != L[l].C_out || L[l + 1].C_out != Wd ||
                    !L[l + 1].shortcut)
                    return IODF_E_SHAPE;
            }
            if (L[nl - 1].C_in != Wd) return IODF_E_SHAPE;
        } else {
            if (nl % 2) return IODF_E_SHAPE;
            const int depth = (nl - 2) / 2;
            for (int l = 1; l <= depth; ++l) {
                const HostLayer &a = L[2 * l - 1], &b = L[2 * l];
                if (a.C_in != l * Wd || a.shortcut || b.C_in != a.C_out || b.C_out != Wd || b.shortcut) return IODF_E_SHAPE;
            }
            if (L[nl - 1].C_in != (depth + 1) * Wd) return IODF_E_SHAPE;
        }
    }
    return IODF_OK;
}

// ---- device plan -------------------------------------------------------------------

struct DevLayer {
    int taps, cin_pad, n_pad, n_store, relu, shortcut, mode, rq_fast;
    int in_buf, in_off;    // input tensor: buffer and first channel (multiple of 64)
    int out_buf, out_off;  // output tensor (MODE_ACT)
    size_t wgt_off, bias_off, mul_off, shift_off;  // byte offsets into the parameter arena
    size_t hi_off = (size_t)-1;                    // rq_fast layers: clamp bound per channel
    // Unsigned format: a code u in 0..255 is stored as the byte u - 128 and planes are bordered with
    // -128, so that the int8 matrix cores see u - 128 everywhere; a layer reading such a tensor adds
    // 128 * (sum of its weights) to its bias, a layer writing one saturates to [0, 255] and stores u - 128.
    bool in_unsigned = false, out_unsigned = false, sc_unsigned = false;
    // tap-expanded 3x3 last layer (see TapSumArgs): the GEMM is 1x1 with 9 * c_out rows and
    // stores raw accumulators; these are the constants of the summing pass
    int expand_c_out = 0, final_mode = 0;
    size_t fin_bias_off = 0, fin_mul_off = 0, fin_shift_off = 0;
    long long macs_per_pixel;                      // algorithmic: kept rows x live columns x taps
    long long bytes_per_pixel;                     // algorithmic: live input codes + kept output codes
    long long wgt_bytes;                           // algorithmic: kept rows x live columns x taps
    bool wide;
};

struct DevNet {
    int kind, level, C, C_in, C_out, cin_pad0;
    int32_t M_in;
    int s_in;
    size_t phi_off;     // byte offset of this coupling's composed index map (int32[C]); heads: the level's last
    std::vector<DevLayer> layers;
};

std::vector<int> kept_rows(const HostLayer& L) {
    std::vector<int> r;
    for (int c = 0; c < L.C_out; ++c)
        if (L.gate[c]) r.push_back(c);
    return r;
}

// Packed position of every original channel of a feature tensor (-1 = removed).
std::vector<int> rank_map(const HostLayer& producer, int base) {
    std::vector<int> pos(producer.C_out, -1);
    int r = 0;
    for (int c = 0; c < producer.C_out; ++c)
        if (producer.gate[c]) pos[c] = base + r++;
    return pos;
}

struct Arena {
    std::vector<uint8_t> host;
    size_t alloc(size_t bytes) {
        const size_t off = (host.size() + 255) & ~(size_t)255;
        host.resize(off + bytes, 0);
        return off;
    }
};

// Append one layer's packed weights and constants to the arena.
//   rows:   original output channels kept, in order
//   colpos: packed input column of each original input channel, or -1
//   masked: rows whose gate is 0 stay in place as all-zero filters with zero bias and multiplier
//           (they output exactly 0, as a removed filter does) instead of being removed; `rows`
//           then lists every channel. Used where the consumer needs the full width anyway.
void pack_layer(Arena& A, const HostLayer& L, const std::vector<int>& rows, const std::vector<int>& colpos, int cin_pad,
                DevLayer& D, bool masked = false) {
    const int taps = L.k * L.k;
    D.taps = taps;
    D.cin_pad = cin_pad;
    D.n_pad = round64((int)rows.size());
    D.relu = L.relu;
    D.shortcut = L.shortcut;
    const size_t wbytes = (size_t)D.n_pad * taps * cin_pad;
    D.wgt_off = A.alloc(wbytes);
    D.bias_off = A.alloc(4 * (size_t)D.n_pad);
    D.mul_off = A.alloc(4 * (size_t)D.n_pad);
    D.shift_off = A.alloc(4 * (size_t)D.n_pad);
    int8_t* w = (int8_t*)(A.host.data() + D.wgt_off);
    int32_t* bias = (int32_t*)(A.host.data() + D.bias_off);
    int32_t* mul = (int32_t*)(A.host.data() + D.mul_off);
    int32_t* sh = (int32_t*)(A.host.data() + D.shift_off);
    int live = 0;
    for (int c = 0; c < L.C_in; ++c) live += colpos[c] >= 0;
    int kept = 0;
    for (size_t n = 0; n < rows.size(); ++n) {
        const int r = rows[n];
        if (masked && !L.gate[r]) { bias[n] = 0; mul[n] = 0; sh[n] = 33; continue; }
        ++kept;
        const int8_t* src = L.W + (size_t)r * L.C_in * taps;
        // input column pc, tap t goes to k-tile (pc / 64) * taps + t, row n, byte pc % 64
        for (int c = 0; c < L.C_in; ++c) {
            const int pc = colpos[c];
            if (pc < 0) continue;
            for (int t = 0; t < taps; ++t)
                w[(((size_t)(pc >> 6) * taps + t) * D.n_pad + n) * 64 + (pc & 63)] = src[(size_t)c * taps + t];
        }
        long long fold = 0;  // sum of the row's kept weights
        if (D.in_unsigned)
            for (int c = 0; c < L.C_in; ++c)
                if (colpos[c] >= 0)
                    for (int t = 0; t < taps; ++t) fold += src[(size_t)c * taps + t];
        bias[n] = (int32_t)(L.bias[r] + 128 * fold);  // |bias| < 2^30 and 128 * 127 * K < 2^30 for K < 66000
        mul[n] = L.M[r];
        sh[n] = L.shift[r];
    }
    // layers whose every shift is >= 33 take the short exact requantise (shift stored minus 32)
    D.rq_fast = 1;
    for (size_t n = 0; n < rows.size(); ++n)
        if (sh[n] < 33) D.rq_fast = 0;
    for (int n = 0; n < D.n_pad; ++n) {
        if (n >= (int)rows.size()) { mul[n] = 0; sh[n] = D.rq_fast ? 33 : 0; }
        if (D.rq_fast) sh[n] -= 32;
    }
    if (D.rq_fast) {
        // Smallest accumulator a >= 0 with (floor(a * M / 2^32) + 2^(sh-1)) >> sh >= top (127, or 255 for
        // unsigned codes), i.e. a * M >= (top * 2^sh - 2^(sh-1)) * 2^32. The rescale factor
        // M / 2^(32+sh) is below 1, so the result there is exactly top; beyond int32 no accumulator
        // reaches it at all.
        D.hi_off = A.alloc(4 * (size_t)D.n_pad);
        int32_t* hi = (int32_t*)(A.host.data() + D.hi_off);
        mul = (int32_t*)(A.host.data() + D.mul_off);  // the arena may have moved
        sh = (int32_t*)(A.host.data() + D.shift_off);
        for (int n = 0; n < D.n_pad; ++n) {
            hi[n] = INT32_MAX;
            if (mul[n] <= 0) continue;
            const unsigned long long top = D.out_unsigned ? 255ULL : 127ULL;
            const unsigned __int128 need = ((unsigned __int128)((top << sh[n]) - (1ULL << (sh[n] - 1)))) << 32;
            const unsigned __int128 a = (need + (unsigned)mul[n] - 1) / (unsigned)mul[n];
            if (a < (unsigned __int128)INT32_MAX) hi[n] = (int32_t)(uint64_t)a;
        }
    }
    D.macs_per_pixel = (long long)kept * live * taps;
    D.bytes_per_pixel = (long long)live + (long long)kept;
    D.wgt_bytes = D.macs_per_pixel;
    D.wide = kept >= 128 && live >= 128;
}

// A 3x3 last layer is tap-expanded from this many (padded) input channels on. Below it the direct
// convolution, whose <= 64 rows waste most of each MFMA, still costs less than writing and re-reading
// the raw maps (measured: the 128-wide residual networks gain 2-7 % from the direct form, the dense
// family with 2304 or 4608 input channels loses 8-9 %).
constexpr int kExpandFromCin = 256;

// Last layer of a network, 3x3 with few output channels, as a 1x1 GEMM over 9 * C_out rows.
void pack_last_expanded(Arena& A, const HostLayer& L, const std::vector<int>& colpos, int cin_pad, int final_mode,
                        DevLayer& D) {
    const int co = L.C_out, rows = 9 * co;
    D.taps = 1;
    D.cin_pad = cin_pad;
    D.n_pad = round64(rows);
    D.n_store = rows;
    D.relu = L.relu;
    D.shortcut = 0;
    D.rq_fast = 0;
    D.mode = MODE_RAW;
    D.expand_c_out = co;
    D.final_mode = final_mode;
    D.wgt_off = A.alloc((size_t)D.n_pad * cin_pad);
    D.bias_off = A.alloc(4 * (size_t)D.n_pad);   // added to the raw accumulators: 0, or the unsigned-input fold
    D.mul_off = A.alloc(4 * (size_t)D.n_pad);
    D.shift_off = A.alloc(4 * (size_t)D.n_pad);
    D.fin_bias_off = A.alloc(4 * (size_t)co);
    D.fin_mul_off = A.alloc(4 * (size_t)co);
    D.fin_shift_off = A.alloc(4 * (size_t)co);
    int8_t* w = (int8_t*)(A.host.data() + D.wgt_off);
    int live = 0;
    for (int c = 0; c < L.C_in; ++c) live += colpos[c] >= 0;
    int32_t* xb = (int32_t*)(A.host.data() + D.bias_off);
    for (int r = 0; r < co; ++r)
        for (int c = 0; c < L.C_in; ++c) {
            const int pc = colpos[c];
            if (pc < 0) continue;
            for (int t = 0; t < 9; ++t) {
                const int8_t wv = L.W[((size_t)r * L.C_in + c) * 9 + t];
                w[((size_t)(pc >> 6) * D.n_pad + (size_t)(t * co + r)) * 64 + (pc & 63)] = wv;
                // a tap that falls outside the image is skipped by the summing pass, fold and all
                if (D.in_unsigned) xb[t * co + r] += 128 * (int32_t)wv;
            }
        }
    int32_t* fb = (int32_t*)(A.host.data() + D.fin_bias_off);
    int32_t* fm = (int32_t*)(A.host.data() + D.fin_mul_off);
    int32_t* fs = (int32_t*)(A.host.data() + D.fin_shift_off);
    for (int r = 0; r < co; ++r) { fb[r] = L.bias[r]; fm[r] = L.M[r]; fs[r] = L.shift[r]; }
    D.macs_per_pixel = (long long)co * live * 9;
    D.bytes_per_pixel = (long long)live + (long long)co + 8LL * rows;  // + raw maps written and read once
    D.wgt_bytes = D.macs_per_pixel;
    D.wide = false;
}

std::vector<int> identity_map(int n) {
    std::vector<int> v(n);
    for (int i = 0; i < n; ++i) v[i] = i;
    return v;
}

// Build the launch list of one network. buf_w[b] is raised to the row width the network needs.
void plan_net(Arena& A, const HostModel& m, const HostNet& N, DevNet& D, int buf_w[NUM_BUFS]) {
    const std::vector<HostLayer>& L = N.layers;
    const int nl = (int)L.size();
    D.kind = N.kind; D.level = N.level; D.C = N.C; D.C_in = N.C_in; D.C_out = N.C_out;
    D.M_in = N.M_in; D.s_in = N.s_in;
    D.cin_pad0 = round64(N.C_in);
    D.layers.resize(nl);
    for (int l = 0; l < nl; ++l) {  // read by the packers below
        D.layers[l].in_unsigned = m.act_unsigned && l > 0;
        D.layers[l].out_unsigned = m.act_unsigned && l + 1 < nl;
        D.layers[l].sc_unsigned = m.act_unsigned && L[l].shortcut;
    }
    buf_w[BUF_XQ] = std::max(buf_w[BUF_XQ], D.cin_pad0);
    const int last_mode = N.kind == 0 ? MODE_COUPLE : MODE_CODES;
    // the last layer: tap-expanded when it is 3x3 over a wide input, else a direct convolution
    auto plan_last = [&](const HostLayer& H, const std::vector<int>& cols, int cin_pad, DevLayer& d) {
        if (H.k == 3 && cin_pad >= kExpandFromCin) {
            pack_last_expanded(A, H, cols, cin_pad, last_mode, d);
        } else {
            pack_layer(A, H, kept_rows(H), cols, cin_pad, d);
            d.mode = last_mode;
            d.n_store = N.C_out;
        }
    };
    auto io = [](DevLayer& d, int ib, int ioff, int /*in width*/, int ob, int ooff, int /*out width*/, int mode) {
        d.in_buf = ib; d.in_off = ioff;
        d.out_buf = ob; d.out_off = ooff;
        d.mode = mode;
    };
    if (m.family == FAM_PLAIN) {
        const std::vector<int> r0 = kept_rows(L[0]);
        const int fw = round64((int)r0.size());
        pack_layer(A, L[0], r0, identity_map(N.C_in), D.cin_pad0, D.layers[0]);
        io(D.layers[0], BUF_XQ, 0, D.cin_pad0, BUF_A, 0, fw, MODE_ACT);
        D.layers[0].n_store = fw;
        plan_last(L[1], rank_map(L[0], 0), fw, D.layers[1]);
        D.layers[1].in_buf = BUF_A; D.layers[1].in_off = 0; D.layers[1].out_buf = -1; D.layers[1].out_off = 0;
        buf_w[BUF_A] = std::max(buf_w[BUF_A], fw);
    } else if (m.family == FAM_RESNET) {
        // BUF_A: residual stream at full width; BUF_B: block-internal feature (compacted)
        const int Wd = L[0].C_out;
        const int rw = round64(Wd);
        buf_w[BUF_A] = std::max(buf_w[BUF_A], rw);
        // The stream keeps its full width (the shortcut adds into unpruned channels, Sec. 4.4), so
        // the layers that write it keep gated-off filters as zero rows: a zero row adds 0 to the
        // shortcut exactly like a removed one, and the store stays a plain full-width one.
        std::vector<int> all_rows(Wd);
        for (int c = 0; c < Wd; ++c) all_rows[c] = c;
        {
            pack_layer(A, L[0], all_rows, identity_map(N.C_in), D.cin_pad0, D.layers[0], true);
            io(D.layers[0], BUF_XQ, 0, D.cin_pad0, BUF_A, 0, rw, MODE_ACT);
            D.layers[0].n_store = rw;
                }
        for (int l = 1; l + 1 < nl; l += 2) {
            const std::vector<int> r1 = kept_rows(L[l]);
            const int tw = round64((int)r1.size());
            buf_w[BUF_B] = std::max(buf_w[BUF_B], tw);
            pack_layer(A, L[l], r1, identity_map(Wd), rw, D.layers[l]);
            io(D.layers[l], BUF_A, 0, rw, BUF_B, 0, tw, MODE_ACT);
            D.layers[l].n_store = tw;
            pack_layer(A, L[l + 1], all_rows, rank_map(L[l], 0), tw, D.layers[l + 1], true);
            io(D.layers[l + 1], BUF_B, 0, tw, BUF_A, 0, rw, MODE_ACT);
            D.layers[l + 1].n_store = rw;
        }
        plan_last(L[nl - 1], identity_map(Wd), rw, D.layers[nl - 1]);
        D.layers[nl - 1].in_buf = BUF_A; D.layers[nl - 1].in_off = 0; D.layers[nl - 1].out_buf = -1;
        D.layers[nl - 1].out_off = 0;
    } else {
        // BUF_A: concatenation of the compacted feature blocks f0..f_depth; BUF_B: bottleneck g
        const int depth = (nl - 2) / 2;
        const int Wd = L[0].C_out;
        std::vector<int> blk_off(depth + 2, 0);
        std::vector<int> catpos;  // packed column of every original concat channel
        for (int j = 0; j <= depth; ++j) {
            const HostLayer& P = j == 0 ? L[0] : L[2 * j];
            const std::vector<int> pm = rank_map(P, blk_off[j]);
            catpos.insert(catpos.end(), pm.begin(), pm.end());
            blk_off[j + 1] = blk_off[j] + round64((int)kept_rows(P).size());
        }
        const int cw = blk_off[depth + 1];
        buf_w[BUF_A] = std::max(buf_w[BUF_A], cw);
        pack_layer(A, L[0], kept_rows(L[0]), identity_map(N.C_in), D.cin_pad0, D.layers[0]);
        io(D.layers[0], BUF_XQ, 0, D.cin_pad0, BUF_A, 0, cw, MODE_ACT);
        D.layers[0].n_store = blk_off[1];
        for (int l = 1; l <= depth; ++l) {
            const HostLayer &P1 = L[2 * l - 1], &P3 = L[2 * l];
            const int gw = round64((int)kept_rows(P1).size());
            buf_w[BUF_B] = std::max(buf_w[BUF_B], gw);
            std::vector<int> cols(catpos.begin(), catpos.begin() + (size_t)l * Wd);
            pack_layer(A, P1, kept_rows(P1), cols, blk_off[l], D.layers[2 * l - 1]);
            io(D.layers[2 * l - 1], BUF_A, 0, cw, BUF_B, 0, gw, MODE_ACT);
            D.layers[2 * l - 1].n_store = gw;
            pack_layer(A, P3, kept_rows(P3), rank_map(P1, 0), gw, D.layers[2 * l]);
            io(D.layers[2 * l], BUF_B, 0, gw, BUF_A, blk_off[l], cw, MODE_ACT);
            D.layers[2 * l].n_store = blk_off[l + 1] - blk_off[l];
        }
        plan_last(L[nl - 1], catpos, cw, D.layers[nl - 1]);
        D.layers[nl - 1].in_buf = BUF_A; D.layers[nl - 1].in_off = 0; D.layers[nl - 1].out_buf = -1;
        D.layers[nl - 1].out_off = 0;
    }
}

}  // namespace

struct iodf_ctx {
    int device = 0, max_batch = 0;
    int n_cu = 0;     // compute units of `device`
    HostModel shape;  // header fields only are used after init
    std::vector<DevNet> nets;
    std::vector<int> first_net;       // per level (1-based)
    std::vector<long long> z_off;     // per level
    std::vector<long long> code_off;  // per level with a head
    long long d = 0, d_codes = 0;
    uint8_t* params = nullptr;        // packed weights, constants, index maps
    size_t params_bytes = 0;
    // Activation buffers per level (1-based): each level has its own image geometry, and the
    // zero borders of its planes must never be overwritten by another geometry's pixels.
    std::vector<std::array<int8_t*, NUM_BUFS>> buf;
    std::vector<std::array<int, NUM_BUFS>> buf_w;   // channels (multiple of 64)
    std::vector<long long> plane;                   // bytes between 64-channel planes = max_batch * (h+2)*(w+2) * 64
    std::vector<int32_t*> state;      // per level (1-based), int32 [B][h][w][C]
    unsigned long long* range_errs = nullptr;
    // Scratch of the last layers, int32 [npix][n_pad]. Two buffers because their users disagree about its
    // state: a tap-expanded layer overwrites `raw` and leaves its maps there, a split-K layer adds into
    // `partial`, which its finishing pass leaves all zero again.
    int32_t* partial = nullptr;
    size_t partial_elems = 0;
    int32_t* raw = nullptr;
    size_t raw_elems = 0;
    size_t workspace_bytes = 0;
    long long macs_fwd = 0, macs_inv = 0, macs_wide = 0;
    int conv_launches = 0;
    // Launch-bound shapes (small batches: ~650 dependent kernels per call) are replayed from a
    // HIP graph. A graph is captured once per (direction, batch, codes) on an internal stream
    // against internal staging buffers for x, z and codes; a call then is: copy in, graph
    // launch, copy out, all on the caller's stream.
    // `done` is recorded after every launch of the graph, so that an entry can be destroyed safely
    struct GraphEntry { int dir, batch, codes; hipGraphExec_t exec; hipEvent_t done; unsigned long long last_use; };
    std::vector<GraphEntry> graphs;   // at most kMaxGraphs, least recently used dropped
    static constexpr size_t kMaxGraphs = 8;
    unsigned long long graph_clock = 0;
    hipStream_t cap_stream = nullptr;
    bool use_graphs = true;
    uint8_t* stage_x = nullptr;
    int32_t* stage_z = nullptr;
    int8_t* stage_codes = nullptr;
    // Compressor (iodf_encode / iodf_decode / iodf_prior_cf): allocated by the first call that needs it
    bool codec_ready = false;
    bool used_static_scratch = false;  // iodf_encode_noalloc ran: its error counters live in the static scratch
    ChunkTable chunks;                 // chunk c = level c + 1
    long long lane_words_per_image = 0;
    int32_t* codec_sig = nullptr;      // tables of the integer prior
    int64_t* codec_inv = nullptr;
    int32_t* codec_z = nullptr;        // [max_batch][d]
    int8_t* codec_codes = nullptr;     // [max_batch][d_codes]
    uint32_t* lane_words = nullptr;    // [max_batch][lane_words_per_image]
    uint32_t* lane_meta = nullptr;     // [max_batch][n_chunks * 16][4]
    unsigned long long* codec_errs = nullptr;  // [3]: clamped residuals, overflowing containers, broken lanes
    // optional per-launch timing (iodf_profile_begin / iodf_profile_end)
    struct ProfRec { int cls; long long macs, bytes, issued; int wide; };  // wide: 1 = wide layer, 2 = at level 1 or 2
    bool prof_on = false;
    std::vector<hipEvent_t> prof_ev;
    std::vector<ProfRec> prof_recs;
};

namespace {

enum { CLS_QUANT_IN = 0, CLS_FILL_ZERO, CLS_INGEST, CLS_FACTOR_OUT, CLS_UNFACTOR, CLS_EMIT_X, CLS_TAPSUM,
       CLS_PRIOR_CF, CLS_RANS_ENCODE, CLS_RANS_PACK, CLS_RANS_DECODE, NUM_FLOW_CLS };
const char* const kFlowClsName[NUM_FLOW_CLS] = {"k_quant_in", "k_fill_zero", "k_ingest_squeeze",
                                                "k_factor_out", "k_unfactor", "k_emit_x", "conv_tapsum",
                                                "k_prior_cf", "k_rans_encode", "k_rans_pack", "k_rans_decode_chunk"};

bool prof_start(iodf_ctx* ctx, hipStream_t st) {
    if (!ctx->prof_on || 2 * (ctx->prof_recs.size() + 1) > ctx->prof_ev.size()) return false;
    return hipEventRecord(ctx->prof_ev[2 * ctx->prof_recs.size()], st) == hipSuccess;
}

void prof_stop(iodf_ctx* ctx, hipStream_t st, int cls, long long macs, long long bytes, long long issued = 0,
               int wide = 0) {
    (void)hipEventRecord(ctx->prof_ev[2 * ctx->prof_recs.size() + 1], st);
    ctx->prof_recs.push_back({cls, macs, bytes, issued, wide});
}

// Multiply-accumulates the matrix cores actually run for a conv launch: whole tiles, padded widths.
long long issued_macs(const ConvArgs& a) {
    int bc = 0, bp = 0;
    conv_tile_dims(conv_pick_tile(a), &bc, &bp);
    if (!bc) return 0;
    const long long px = (long long)((a.npix + bp - 1) / bp) * bp, ch = (long long)((a.n_store + bc - 1) / bc) * bc;
    return px * ch * a.cin_pad * a.taps;
}

// Launch through `call`, bracketed by events when profiling is on.
#define PROF_LAUNCH(ctx, st, cls, macs, bytes, call)        \
    do {                                                    \
        const bool p__ = prof_start(ctx, st);               \
        HIP_TRY(call);                                      \
        if (p__) prof_stop(ctx, st, cls, macs, bytes);      \
    } while (0)

static const int32_t* partial_of(const iodf_ctx* ctx);

// What a layer's launch reads first: its packed weights and, behind them in the parameter buffer, its
// per-channel constants.
static void layer_param_span(const iodf_ctx* ctx, const DevLayer& L, const int8_t** p, unsigned* bytes) {
    size_t end = L.shift_off + 4 * (size_t)L.n_pad;
    if (L.hi_off != (size_t)-1) end = std::max(end, L.hi_off + 4 * (size_t)L.n_pad);
    if (L.mode == MODE_RAW) end = std::max(end, L.fin_shift_off + 4 * (size_t)L.expand_c_out);
    const size_t wbytes = (size_t)L.taps * L.cin_pad * L.n_pad;
    if (end <= L.wgt_off || end > ctx->params_bytes || end - L.wgt_off > wbytes + (1u << 20)) end = L.wgt_off + wbytes;
    *p = (const int8_t*)(ctx->params + L.wgt_off);
    *bytes = (unsigned)std::min<size_t>(end - L.wgt_off, 0xffffffffu);
}

// `next`: the network that runs after this one (its first layer's parameters are prefetched), or nullptr.
int run_net(iodf_ctx* ctx, const DevNet& N, int batch, int mode_sign, int8_t* codes, hipStream_t st,
            const DevNet* next = nullptr) {
    const int lv = N.level;
    const int h = ctx->shape.H >> lv, w = ctx->shape.W >> lv;
    const int npix = batch * h * w;
    const int32_t* phi = (const int32_t*)(ctx->params + N.phi_off);
    const long long plane = ctx->plane[lv];
    PROF_LAUNCH(ctx, st, CLS_QUANT_IN, 0, (long long)npix * (4 * N.C_in + (N.C_in + 3) / 4 * 4),
                launch_quant_in(ctx->state[lv], npix, h, w, N.C, phi, N.C_in, N.M_in, N.s_in, ctx->buf[lv][BUF_XQ],
                                N.cin_pad0, plane, st));
    for (size_t li = 0; li < N.layers.size(); ++li) {
        const DevLayer& L = N.layers[li];
        ConvArgs a;
        memset(&a, 0, sizeof(a));
        {
            const DevLayer* Ln = li + 1 < N.layers.size() ? &N.layers[li + 1] : next && !next->layers.empty() ? &next->layers[0] : nullptr;
            unsigned pfb = 0;
            if (Ln) layer_param_span(ctx, *Ln, &a.pf, &pfb);
            a.pf_bytes = pfb;
        }
        a.in = ctx->buf[lv][L.in_buf];
        a.in_plane = plane;
        a.in_chunk0 = L.in_off / 64;
        a.cin_pad = L.cin_pad;
        a.taps = L.taps;
        a.h = h; a.w = w; a.npix = npix;
        a.n_cu = ctx->n_cu;
        a.wgt = (const int8_t*)(ctx->params + L.wgt_off);
        a.n_pad = L.n_pad;
        a.bias = (const int32_t*)(ctx->params + L.bias_off);
        a.mul = (const int32_t*)(ctx->params + L.mul_off);
        a.shift = (const int32_t*)(ctx->params + L.shift_off);
        a.n_store = L.n_store;
        a.rq_fast = L.rq_fast;
        a.out_unsigned = L.out_unsigned && L.mode == MODE_ACT;
        a.sc_unsigned = L.sc_unsigned;
        a.clamp_hi = L.hi_off == (size_t)-1 ? nullptr : (const int32_t*)(ctx->params + L.hi_off);
        if (L.mode == MODE_RAW) {
            if ((size_t)npix * L.n_pad <= ctx->raw_elems) a.partial = ctx->raw;
        } else if (L.mode != MODE_ACT && (size_t)npix * L.n_pad <= ctx->partial_elems) {
            a.partial = ctx->partial;
        }
        a.mode = L.mode;
        a.relu = L.relu;
        if (L.mode == MODE_ACT) {
            a.out = ctx->buf[lv][L.out_buf];
            a.out_plane = plane;
            a.out_chunk0 = L.out_off / 64;
            a.shortcut = L.shortcut;
        } else if (L.mode == MODE_COUPLE) {
            a.state = ctx->state[lv];
            a.state_c = N.C;
            a.idx_b = phi + N.C_in;
            a.sign = mode_sign;
        } else if (L.mode == MODE_CODES) {
            a.codes = codes;
            a.codes_img_stride = ctx->d_codes;
            a.codes_off = ctx->code_off[lv];
        } else if (!a.partial) {
            return IODF_E_NOMEM;  // cannot happen: the scratch is sized for every raw layer at init
        }
        const int fmode = L.mode == MODE_RAW ? L.final_mode : L.mode;
        const long long extra = fmode == MODE_COUPLE ? 8LL * N.C_out : 0;  // state read + write
        {
            const bool p__ = prof_start(ctx, st);
            HIP_TRY(launch_conv(a, st));
            if (p__)
                prof_stop(ctx, st, NUM_FLOW_CLS + 2 * conv_pick_tile(a) + (a.taps == 9), L.macs_per_pixel * npix,
                          (L.bytes_per_pixel + extra) * npix + L.wgt_bytes, issued_macs(a),
                          L.wide ? (lv <= 2 ? 2 : 1) : 0);
        }
        if (L.mode == MODE_RAW) {
            TapSumArgs t;
            memset(&t, 0, sizeof(t));
            t.y = partial_of(ctx);
            t.n_pad = L.n_pad; t.c_out = L.expand_c_out; t.h = h; t.w = w; t.npix = npix;
            t.bias = (const int32_t*)(ctx->params + L.fin_bias_off);
            t.mul = (const int32_t*)(ctx->params + L.fin_mul_off);
            t.shift = (const int32_t*)(ctx->params + L.fin_shift_off);
            t.mode = L.final_mode; t.relu = L.relu;
            if (L.final_mode == MODE_COUPLE) {
                t.state = ctx->state[lv]; t.state_c = N.C; t.idx_b = phi + N.C_in; t.sign = mode_sign;
            } else {
                t.codes = codes; t.codes_img_stride = ctx->d_codes; t.codes_off = ctx->code_off[lv];
            }
            PROF_LAUNCH(ctx, st, CLS_TAPSUM, 0, (36LL * L.expand_c_out + extra) * npix, launch_tapsum(t, st));
        }
    }
    return IODF_OK;
}

static const int32_t* partial_of(const iodf_ctx* ctx) { return ctx->raw; }

}  // namespace

extern "C" {

static int codec_layout(iodf_ctx* ctx);
static int scratch_setup(int device);

int iodf_last_hip_error(void) { return g_last_hip; }

const char* iodf_strerror(int code) {
    switch (code) {
        case IODF_OK: return "ok";
        case IODF_E_ARG: return "invalid argument";
        case IODF_E_BLOB: return "malformed model blob";
        case IODF_E_SHAPE: return "model layers do not fit the declared flow structure";
        case IODF_E_BATCH: return "batch outside [0, max_batch]";
        case IODF_E_HIP: return "HIP runtime error";
        case IODF_E_NOMEM: return "out of memory";
        case IODF_E_SCRATCH: return "batch needs more than the 64 MiB static scratch of iodf_encode_noalloc";
        default: return "unknown error";
    }
}

int iodf_init(iodf_ctx** out, const void* model_blob, size_t blob_bytes, int device_ordinal, int max_batch) {
    if (!out || !model_blob || max_batch < 1 || device_ordinal < 0) return IODF_E_ARG;
    *out = nullptr;
    // host-side validation comes first: it needs no GPU
    std::vector<uint32_t> copy((blob_bytes + 3) / 4);
    memcpy(copy.data(), model_blob, blob_bytes);
    HostModel hm;
    int rc = parse_blob((const uint8_t*)copy.data(), blob_bytes, hm);
    if (rc != IODF_OK) return rc;
    rc = check_shapes(hm);
    if (rc != IODF_OK) return rc;
    const long long px1 = (long long)max_batch * (hm.H / 2) * (hm.W / 2);
    if (px1 > (1LL << 30)) return IODF_E_BATCH;

    iodf_ctx* ctx = new (std::nothrow) iodf_ctx();
    if (!ctx) return IODF_E_NOMEM;
    ctx->device = device_ordinal;
    ctx->max_batch = max_batch;
    ctx->shape = hm;
    ctx->d = 3LL * hm.H * hm.W;

    // offsets of z chunks / code chunks and network indices per level
    ctx->first_net.assign(hm.levels + 2, 0);
    ctx->z_off.assign(hm.levels + 2, 0);
    ctx->code_off.assign(hm.levels + 2, 0);
    {
        int net = 0;
        long long zo = 0, co = 0;
        for (int lv = 1; lv <= hm.levels; ++lv) {
            const int C = level_channels(lv);
            const long long hw = (long long)(hm.H >> lv) * (hm.W >> lv);
            ctx->first_net[lv] = net;
            ctx->z_off[lv] = zo;
            ctx->code_off[lv] = co;
            net += hm.couplings;
            if (lv < hm.levels) {
                zo += (C - C / 2) * hw;
                if (hm.has_heads) { co += 2LL * (C - C / 2) * hw; ++net; }
            } else {
                zo += C * hw;
            }
        }
        ctx->d_codes = co;
    }
    (void)codec_layout(ctx);  // cannot fail: parse_blob bounds the number of levels

    // plan: pack weights (gate compaction), constants and composed permutations
    Arena A;
    A.host.reserve(blob_bytes + blob_bytes / 2 + (1 << 20));
    ctx->nets.resize(hm.nets.size());
    ctx->buf.assign(hm.levels + 2, std::array<int8_t*, NUM_BUFS>{nullptr, nullptr, nullptr});
    ctx->buf_w.assign(hm.levels + 2, std::array<int, NUM_BUFS>{0, 0, 0});
    ctx->plane.assign(hm.levels + 2, 0);
    {
        size_t n = 0;
        for (int lv = 1; lv <= hm.levels; ++lv) {
            const int C = level_channels(lv);
            std::vector<int> phi = identity_map(C);
            size_t last_off = 0;
            for (int k = 0; k < hm.couplings; ++k, ++n) {
                // logical channel i after this coupling's permutation is the previous logical perm[i]
                std::vector<int> nphi(C);
                for (int i = 0; i < C; ++i) nphi[i] = phi[hm.nets[n].perm[i]];
                phi.swap(nphi);
                last_off = A.alloc(4 * (size_t)C);
                memcpy(A.host.data() + last_off, phi.data(), 4 * (size_t)C);
                ctx->nets[n].phi_off = last_off;
                plan_net(A, hm, hm.nets[n], ctx->nets[n], ctx->buf_w[lv].data());
            }
            if (hm.has_heads && lv < hm.levels) {
                ctx->nets[n].phi_off = last_off;
                plan_net(A, hm, hm.nets[n], ctx->nets[n], ctx->buf_w[lv].data());
                ++n;
            }
        }
    }
    ctx->shape.nets.clear();  // their pointers die with the blob copy; only header fields are kept
    for (const DevNet& N : ctx->nets) {
        const long long hw = (long long)(hm.H >> N.level) * (hm.W >> N.level);
        for (const DevLayer& L : N.layers) {
            ctx->macs_fwd += L.macs_per_pixel * hw;
            if (N.kind == 0) ctx->macs_inv += L.macs_per_pixel * hw;
            if (L.wide) ctx->macs_wide += L.macs_per_pixel * hw;
            ++ctx->conv_launches;
        }
    }

    // device side
    hipError_t e = hipSetDevice(device_ordinal);
    if (e == hipSuccess) e = conv_setup();
    if (e == hipSuccess) e = conv_device_cus(&ctx->n_cu);
    if (e != hipSuccess) { g_last_hip = (int)e; delete ctx; return IODF_E_HIP; }
    rc = scratch_setup(device_ordinal);
    if (rc != IODF_OK) { delete ctx; return rc; }
    auto dev_alloc = [&](void** p, size_t bytes) -> bool {
        if (bytes == 0) bytes = 256;
        hipError_t er = hipMalloc(p, bytes);
        if (er != hipSuccess) { g_last_hip = (int)er; *p = nullptr; return false; }
        ctx->workspace_bytes += bytes;
        return true;
    };
    bool ok = true;
    ctx->params_bytes = A.host.size();
    ok = ok && dev_alloc((void**)&ctx->params, ctx->params_bytes);
    if (ok && ctx->params_bytes) {
        e = hipMemcpy(ctx->params, A.host.data(), ctx->params_bytes, hipMemcpyHostToDevice);
        if (e != hipSuccess) { g_last_hip = (int)e; ok = false; }
    }
    for (int lv = 1; lv <= hm.levels && ok; ++lv) {
        const long long pp = (long long)((hm.H >> lv) + 2) * ((hm.W >> lv) + 2);
        ctx->plane[lv] = ((long long)max_batch * pp * 64 + 1023) / 1024 * 1024;
        if (ctx->plane[lv] >= (1LL << 31)) { iodf_free(ctx); return IODF_E_BATCH; }
        for (int b = 0; b < NUM_BUFS && ok; ++b) {
            const size_t bytes = (size_t)ctx->plane[lv] * (size_t)(std::max(ctx->buf_w[lv][b], 64) / 64);
            ok = dev_alloc((void**)&ctx->buf[lv][b], bytes);
            if (ok) {  // the borders (and everything else) start as code 0: byte 0, or -128 for unsigned tensors
                e = hipMemset(ctx->buf[lv][b], (hm.act_unsigned && b != BUF_XQ) ? 0x80 : 0, bytes);
                if (e != hipSuccess) { g_last_hip = (int)e; ok = false; }
            }
        }
    }
    ctx->state.assign(hm.levels + 2, nullptr);
    for (int lv = 1; lv <= hm.levels && ok; ++lv) {
        const size_t bytes = 4 * (size_t)max_batch * (hm.H >> lv) * (hm.W >> lv) * level_channels(lv);
        ok = dev_alloc((void**)&ctx->state[lv], bytes);
    }
    ok = ok && dev_alloc((void**)&ctx->range_errs, sizeof(unsigned long long));
    {
        const char* ng = getenv("IODF_NO_GRAPH");
        ctx->use_graphs = !(ng && ng[0] == '1');
    }
    if (ctx->use_graphs) {
        ok = ok && dev_alloc((void**)&ctx->stage_x, (size_t)max_batch * ctx->d);
        ok = ok && dev_alloc((void**)&ctx->stage_z, 4 * (size_t)max_batch * ctx->d);
        ok = ok && dev_alloc((void**)&ctx->stage_codes, (size_t)max_batch * std::max<long long>(ctx->d_codes, 1));
        if (ok) {
            e = hipStreamCreateWithFlags(&ctx->cap_stream, hipStreamNonBlocking);
            if (e != hipSuccess) { g_last_hip = (int)e; ok = false; }
        }
    }
    // last-layer scratch: enough for any network at full batch
    for (const DevNet& N : ctx->nets) {
        const size_t px = (size_t)max_batch * (hm.H >> N.level) * (hm.W >> N.level);
        size_t& elems = N.layers.back().mode == MODE_RAW ? ctx->raw_elems : ctx->partial_elems;
        elems = std::max(elems, px * (size_t)N.layers.back().n_pad);
    }
    ok = ok && dev_alloc((void**)&ctx->partial, 4 * ctx->partial_elems);
    ok = ok && dev_alloc((void**)&ctx->raw, 4 * ctx->raw_elems);
    if (ok) {
        e = hipMemset(ctx->partial, 0, std::max<size_t>(4 * ctx->partial_elems, 256));
        if (e != hipSuccess) { g_last_hip = (int)e; ok = false; }
    }
    if (ok) {
        e = hipMemset(ctx->range_errs, 0, sizeof(unsigned long long));
        if (e == hipSuccess) e = hipDeviceSynchronize();
        if (e != hipSuccess) { g_last_hip = (int)e; ok = false; }
    }
    if (!ok) {
        const bool hip_failed = g_last_hip != (int)hipErrorOutOfMemory;
        iodf_free(ctx);
        return hip_failed ? IODF_E_HIP : IODF_E_NOMEM;
    }
    *out = ctx;
    return IODF_OK;
}

void iodf_free(iodf_ctx* ctx) {
    if (!ctx) return;
    (void)hipSetDevice(ctx->device);
    if (ctx->params) (void)hipFree(ctx->params);
    for (auto& lvbuf : ctx->buf)
        for (int8_t* b : lvbuf)
            if (b) (void)hipFree(b);
    for (int32_t* s : ctx->state)
        if (s) (void)hipFree(s);
    if (ctx->range_errs) (void)hipFree(ctx->range_errs);
    for (void* q : {(void*)ctx->codec_sig, (void*)ctx->codec_inv, (void*)ctx->codec_z, (void*)ctx->codec_codes,
                    (void*)ctx->lane_words, (void*)ctx->lane_meta, (void*)ctx->codec_errs})
        if (q) (void)hipFree(q);
    for (auto& g : ctx->graphs) {
        (void)hipEventSynchronize(g.done);
        (void)hipGraphExecDestroy(g.exec);
        (void)hipEventDestroy(g.done);
    }
    if (ctx->cap_stream) (void)hipStreamDestroy(ctx->cap_stream);
    if (ctx->stage_x) (void)hipFree(ctx->stage_x);
    if (ctx->stage_z) (void)hipFree(ctx->stage_z);
    if (ctx->stage_codes) (void)hipFree(ctx->stage_codes);
    if (ctx->partial) (void)hipFree(ctx->partial);
    if (ctx->raw) (void)hipFree(ctx->raw);
    for (hipEvent_t& e : ctx->prof_ev)
        if (e) (void)hipEventDestroy(e);
    delete ctx;
}

static int enqueue_forward(iodf_ctx* ctx, const uint8_t* x_dev, int batch, int32_t* z_dev, int8_t* codes_dev,
                           hipStream_t st) {
    const HostModel& m = ctx->shape;
    PROF_LAUNCH(ctx, st, CLS_INGEST, 0, 5LL * batch * ctx->d,
                launch_ingest_squeeze(x_dev, batch, m.H, m.W, ctx->state[1], st));
    for (int lv = 1; lv <= m.levels; ++lv) {
        const int C = level_channels(lv), h = m.H >> lv, w = m.W >> lv;
        const int n0 = ctx->first_net[lv];
        const bool last = lv == m.levels;
        const bool head = !last && m.has_heads && codes_dev;
        const DevNet* const after_level = last ? nullptr : &ctx->nets[ctx->first_net[lv + 1]];
        for (int k = 0; k < m.couplings; ++k) {
            const DevNet* next = k + 1 < m.couplings ? &ctx->nets[n0 + k + 1] : head ? &ctx->nets[n0 + m.couplings] : after_level;
            const int rc = run_net(ctx, ctx->nets[n0 + k], batch, +1, nullptr, st, next);
            if (rc != IODF_OK) return rc;
        }
        const int32_t* phi = (const int32_t*)(ctx->params + ctx->nets[n0 + m.couplings - 1].phi_off);
        PROF_LAUNCH(ctx, st, CLS_FACTOR_OUT, 0, 8LL * batch * C * h * w,
                    launch_factor_out(ctx->state[lv], batch, h, w, C, phi, last ? 0 : C / 2, z_dev, ctx->d,
                                      ctx->z_off[lv], last ? nullptr : ctx->state[lv + 1], st));
        if (head) {
            const int rc = run_net(ctx, ctx->nets[n0 + m.couplings], batch, +1, codes_dev, st, after_level);
            if (rc != IODF_OK) return rc;
        }
    }
    return IODF_OK;
}

static int enqueue_inverse(iodf_ctx* ctx, const int32_t* z_dev, int batch, uint8_t* x_dev, hipStream_t st) {
    const HostModel& m = ctx->shape;
    for (int lv = m.levels; lv >= 1; --lv) {
        const int C = level_channels(lv), h = m.H >> lv, w = m.W >> lv;
        const int n0 = ctx->first_net[lv];
        const int32_t* phi = (const int32_t*)(ctx->params + ctx->nets[n0 + m.couplings - 1].phi_off);
        const bool last = lv == m.levels;
        PROF_LAUNCH(ctx, st, CLS_UNFACTOR, 0, 8LL * batch * C * h * w,
                    launch_unfactor(ctx->state[lv], batch, h, w, C, phi, last ? 0 : C / 2, z_dev, ctx->d,
                                    ctx->z_off[lv], last ? nullptr : ctx->state[lv + 1], st));
        for (int k = m.couplings - 1; k >= 0; --k) {
            const DevNet* next = k > 0 ? &ctx->nets[n0 + k - 1] : lv > 1 ? &ctx->nets[ctx->first_net[lv - 1] + m.couplings - 1] : nullptr;
            const int rc = run_net(ctx, ctx->nets[n0 + k], batch, -1, nullptr, st, next);
            if (rc != IODF_OK) return rc;
        }
    }
    PROF_LAUNCH(ctx, st, CLS_EMIT_X, 0, 5LL * batch * ctx->d,
                launch_emit_x(ctx->state[1], batch, m.H, m.W, x_dev, ctx->range_errs, st));
    return IODF_OK;
}

// Find or capture the graph of one call shape. Returns nullptr (and *rc) when capture fails.
static iodf_ctx::GraphEntry* get_graph(iodf_ctx* ctx, int dir, int batch, int codes, int* rc) {
    *rc = IODF_OK;
    for (auto& g : ctx->graphs)
        if (g.dir == dir && g.batch == batch && g.codes == codes) {
            g.last_use = ++ctx->graph_clock;
            return &g;
        }
    hipError_t e = hipStreamBeginCapture(ctx->cap_stream, hipStreamCaptureModeThreadLocal);
    if (e != hipSuccess) { g_last_hip = (int)e; *rc = IODF_E_HIP; return nullptr; }
    const int erc = dir == 0 ? enqueue_forward(ctx, ctx->stage_x, batch, ctx->stage_z, codes ? ctx->stage_codes : nullptr,
                                               ctx->cap_stream)
                             : enqueue_inverse(ctx, ctx->stage_z, batch, ctx->stage_x, ctx->cap_stream);
    hipGraph_t graph = nullptr;
    e = hipStreamEndCapture(ctx->cap_stream, &graph);
    if (erc != IODF_OK || e != hipSuccess || !graph) {
        if (graph) (void)hipGraphDestroy(graph);
        if (e != hipSuccess) g_last_hip = (int)e;
        *rc = erc != IODF_OK ? erc : IODF_E_HIP;
        return nullptr;
    }
    hipGraphExec_t exec = nullptr;
    e = hipGraphInstantiate(&exec, graph, nullptr, nullptr, 0);
    (void)hipGraphDestroy(graph);
    if (e != hipSuccess) { g_last_hip = (int)e; *rc = IODF_E_HIP; return nullptr; }
    hipEvent_t done = nullptr;
    e = hipEventCreateWithFlags(&done, hipEventDisableTiming);
    if (e != hipSuccess) { (void)hipGraphExecDestroy(exec); g_last_hip = (int)e; *rc = IODF_E_HIP; return nullptr; }
    if (ctx->graphs.size() >= iodf_ctx::kMaxGraphs) {
        // Drop the least recently used shape. Calls never synchronise, so its last replay may still be
        // running on the caller's stream: wait for the event recorded behind that replay first.
        size_t victim = 0;
        for (size_t i = 1; i < ctx->graphs.size(); ++i)
            if (ctx->graphs[i].last_use < ctx->graphs[victim].last_use) victim = i;
        (void)hipEventSynchronize(ctx->graphs[victim].done);
        (void)hipGraphExecDestroy(ctx->graphs[victim].exec);
        (void)hipEventDestroy(ctx->graphs[victim].done);
        ctx->graphs.erase(ctx->graphs.begin() + (long)victim);
    }
    ctx->graphs.push_back({dir, batch, codes, exec, done, ++ctx->graph_clock});
    return &ctx->graphs.back();
}

int iodf_forward(iodf_ctx* ctx, const uint8_t* x_dev, int batch, int32_t* z_dev, int8_t* codes_dev, void* stream) {
    if (!ctx) return IODF_E_ARG;
    if (batch < 0 || batch > ctx->max_batch) return IODF_E_BATCH;
    if (batch == 0) return IODF_OK;
    if (!x_dev || !z_dev) return IODF_E_ARG;
    hipStream_t st = (hipStream_t)stream;
    HIP_TRY(hipSetDevice(ctx->device));
    if (!ctx->use_graphs || ctx->prof_on) return enqueue_forward(ctx, x_dev, batch, z_dev, codes_dev, st);
    const int codes = (codes_dev && ctx->d_codes) ? 1 : 0;
    int rc;
    iodf_ctx::GraphEntry* g = get_graph(ctx, 0, batch, codes, &rc);
    if (!g) return rc;
    HIP_TRY(hipMemcpyAsync(ctx->stage_x, x_dev, (size_t)batch * ctx->d, hipMemcpyDeviceToDevice, st));
    HIP_TRY(hipGraphLaunch(g->exec, st));
    HIP_TRY(hipEventRecord(g->done, st));
    HIP_TRY(hipMemcpyAsync(z_dev, ctx->stage_z, 4 * (size_t)batch * ctx->d, hipMemcpyDeviceToDevice, st));
    if (codes)
        HIP_TRY(hipMemcpyAsync(codes_dev, ctx->stage_codes, (size_t)batch * ctx->d_codes, hipMemcpyDeviceToDevice, st));
    return IODF_OK;
}

int iodf_inverse(iodf_ctx* ctx, const int32_t* z_dev, int batch, uint8_t* x_dev, void* stream) {
    if (!ctx) return IODF_E_ARG;
    if (batch < 0 || batch > ctx->max_batch) return IODF_E_BATCH;
    if (batch == 0) return IODF_OK;
    if (!x_dev || !z_dev) return IODF_E_ARG;
    hipStream_t st = (hipStream_t)stream;
    HIP_TRY(hipSetDevice(ctx->device));
    if (!ctx->use_graphs || ctx->prof_on) return enqueue_inverse(ctx, z_dev, batch, x_dev, st);
    int rc;
    iodf_ctx::GraphEntry* g = get_graph(ctx, 1, batch, 0, &rc);
    if (!g) return rc;
    HIP_TRY(hipMemcpyAsync(ctx->stage_z, z_dev, 4 * (size_t)batch * ctx->d, hipMemcpyDeviceToDevice, st));
    HIP_TRY(hipGraphLaunch(g->exec, st));
    HIP_TRY(hipEventRecord(g->done, st));
    HIP_TRY(hipMemcpyAsync(x_dev, ctx->stage_x, (size_t)batch * ctx->d, hipMemcpyDeviceToDevice, st));
    return IODF_OK;
}

// ---- compressor: flow + prior + coder ----

// Where the chunks of one image's latents, codes and coder lanes live (host arithmetic only).
static int codec_layout(iodf_ctx* ctx) {
    const HostModel& m = ctx->shape;
    if (m.levels > kMaxChunks) return IODF_E_ARG;
    ChunkTable& ct = ctx->chunks;
    memset(&ct, 0, sizeof(ct));
    ct.n_chunks = m.levels;
    long long lane_off = 0;
    for (int lv = 1; lv <= m.levels; ++lv) {
        const int C = level_channels(lv);
        const long long hw = (long long)(m.H >> lv) * (m.W >> lv);
        const long long n = (lv < m.levels ? C - C / 2 : C) * hw;
        ct.n[lv - 1] = (int)n;
        ct.z_off[lv - 1] = ctx->z_off[lv];
        ct.code_off[lv - 1] = (m.has_heads && lv < m.levels) ? ctx->code_off[lv] : -1;
        ct.lane_cap[lv - 1] = (int)((n + kLanes - 1) / kLanes) + 1;
        ct.lane_off[lv - 1] = lane_off;
        lane_off += (long long)kLanes * ct.lane_cap[lv - 1];
    }
    ctx->lane_words_per_image = lane_off;
    return IODF_OK;
}

// Device buffers and tables of the compressor, on first use.
static int codec_prepare(iodf_ctx* ctx) {
    if (ctx->codec_ready) return IODF_OK;
    const ChunkTable& ct = ctx->chunks;
    const long long lane_off = ctx->lane_words_per_image;
    std::vector<int32_t> sig(kSigEntries);
    std::vector<int64_t> inv(256);
    codec_make_tables(sig.data(), inv.data());
    const size_t B = (size_t)ctx->max_batch;
    struct { void** p; size_t bytes; } want[] = {
        {(void**)&ctx->codec_sig, sizeof(int32_t) * kSigEntries},
        {(void**)&ctx->codec_inv, sizeof(int64_t) * 256},
        {(void**)&ctx->codec_z, 4 * B * (size_t)ctx->d},
        {(void**)&ctx->codec_codes, B * (size_t)std::max<long long>(ctx->d_codes, 1)},
        {(void**)&ctx->lane_words, 4 * B * (size_t)lane_off},
        {(void**)&ctx->lane_meta, 16 * B * (size_t)ct.n_chunks * kLanes},
        {(void**)&ctx->codec_errs, 3 * sizeof(unsigned long long)},
    };
    for (auto& w : want) {
        if (*w.p) continue;
        const hipError_t e = hipMalloc(w.p, w.bytes);
        if (e != hipSuccess) { *w.p = nullptr; g_last_hip = (int)e; return e == hipErrorOutOfMemory ? IODF_E_NOMEM : IODF_E_HIP; }
        ctx->workspace_bytes += w.bytes;
    }
    HIP_TRY(hipMemcpy(ctx->codec_sig, sig.data(), sizeof(int32_t) * kSigEntries, hipMemcpyHostToDevice));
    HIP_TRY(hipMemcpy(ctx->codec_inv, inv.data(), sizeof(int64_t) * 256, hipMemcpyHostToDevice));
    HIP_TRY(hipMemset(ctx->codec_errs, 0, 3 * sizeof(unsigned long long)));
    HIP_TRY(hipDeviceSynchronize());
    ctx->codec_ready = true;
    return IODF_OK;
}

int iodf_codec_tables(int32_t* sig_host, int64_t* inv_host) {
    if (!sig_host || !inv_host) return IODF_E_ARG;
    codec_make_tables(sig_host, inv_host);
    return IODF_OK;
}

int iodf_prior_cf(iodf_ctx* ctx, const int32_t* z_dev, const int8_t* codes_dev, int batch, int32_t* c_dev,
                  int32_t* f_dev, void* stream) {
    if (!ctx) return IODF_E_ARG;
    if (batch < 0 || batch > ctx->max_batch) return IODF_E_BATCH;
    if (batch == 0) return IODF_OK;
    if (!z_dev || !c_dev || !f_dev || (ctx->d_codes && !codes_dev)) return IODF_E_ARG;
    hipStream_t st = (hipStream_t)stream;
    HIP_TRY(hipSetDevice(ctx->device));
    const int rc = codec_prepare(ctx);
    if (rc != IODF_OK) return rc;
    const CodecTables t{ctx->codec_sig, ctx->codec_inv};
    PROF_LAUNCH(ctx, st, CLS_PRIOR_CF, 0, (long long)batch * (12 * ctx->d + ctx->d_codes),
                launch_prior_cf(t, ctx->chunks, z_dev, ctx->d, ctx->d_codes ? codes_dev : nullptr, ctx->d_codes, batch,
                                c_dev, f_dev, ctx->codec_errs, st));
    return IODF_OK;
}

int iodf_encode(iodf_ctx* ctx, const uint8_t* x_dev, int batch, uint32_t* words_dev, int64_t cap_words,
                uint32_t* sizes_dev, void* stream) {
    if (!ctx) return IODF_E_ARG;
    if (batch < 0 || batch > ctx->max_batch) return IODF_E_BATCH;
    if (batch == 0) return IODF_OK;
    if (!x_dev || !words_dev || !sizes_dev || cap_words < 1) return IODF_E_ARG;
    hipStream_t st = (hipStream_t)stream;
    HIP_TRY(hipSetDevice(ctx->device));
    int rc = codec_prepare(ctx);
    if (rc != IODF_OK) return rc;
    // the flow, into the compressor's own latent and code buffers
    rc = iodf_forward(ctx, x_dev, batch, ctx->codec_z, ctx->d_codes ? ctx->codec_codes : nullptr, stream);
    if (rc != IODF_OK) return rc;
    const CodecTables t{ctx->codec_sig, ctx->codec_inv};
    const int8_t* codes = ctx->d_codes ? ctx->codec_codes : nullptr;
    PROF_LAUNCH(ctx, st, CLS_RANS_ENCODE, 0, (long long)batch * (4 * ctx->d + ctx->d_codes),
                launch_rans_encode(t, ctx->chunks, ctx->codec_z, ctx->d, codes, ctx->d_codes, batch, ctx->lane_words,
                                   ctx->lane_words_per_image, ctx->lane_meta, ctx->codec_errs, st));
    PROF_LAUNCH(ctx, st, CLS_RANS_PACK, 0, 0,
                launch_rans_pack(ctx->chunks, ctx->lane_words, ctx->lane_words_per_image, ctx->lane_meta, batch,
                                 words_dev, cap_words, sizes_dev, ctx->codec_errs, st));
    return IODF_OK;
}

// ---- iodf_encode for callers that cannot allocate ----
//
// iodf_encode keeps the coder's device buffers (latents and codes of the batch, the words each lane
// sheds, lane states, the two prior tables, three error counters) in memory that its first call
// allocates. iodf_encode_noalloc keeps the same buffers in this file-scope array instead. Each GPU
// the library runs on holds its own copy of the array at its own address until the process ends;
// host code never uses the array's name as an address, only what hipGetSymbolAddress returned for
// the device at hand.
constexpr size_t kScratchBytes = (size_t)64 << 20;
constexpr size_t kScratchErrsOff = 0;                         // u64[3], kept across calls
constexpr size_t kScratchSigOff = 256;                        // i32[kSigEntries]
constexpr size_t kScratchInvOff = kScratchSigOff + ((sizeof(int32_t) * kSigEntries + 255) & ~(size_t)255);
constexpr size_t kScratchCallOff = kScratchInvOff + sizeof(int64_t) * 256;   // per-call buffers from here
static_assert(kScratchCallOff % 256 == 0, "per-call region must stay aligned");
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

constexpr int kMaxDevices = 64;
static unsigned char* g_scratch_ptr[kMaxDevices];   // device address of `scratch` per device, nullptr = not set up
static std::mutex g_scratch_mutex;

static size_t align256(size_t n) { return (n + 255) & ~(size_t)255; }

// Once per device, with that device current (iodf_init calls this): resolve the array's address on
// the device, upload the prior tables, clear the counters.
static int scratch_setup(int device) {
    if (device < 0 || device >= kMaxDevices) return IODF_E_ARG;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (g_scratch_ptr[device]) return IODF_OK;
    unsigned char* ptr = nullptr;
    HIP_TRY(hipGetSymbolAddress((void**)&ptr, HIP_SYMBOL(scratch)));
    if (!ptr) { g_last_hip = (int)hipErrorInvalidSymbol; return IODF_E_HIP; }
    std::vector<int32_t> sig(kSigEntries);
    std::vector<int64_t> inv(256);
    codec_make_tables(sig.data(), inv.data());
    HIP_TRY(hipMemcpy(ptr + kScratchSigOff, sig.data(), sizeof(int32_t) * kSigEntries, hipMemcpyHostToDevice));
    HIP_TRY(hipMemcpy(ptr + kScratchInvOff, inv.data(), sizeof(int64_t) * 256, hipMemcpyHostToDevice));
    HIP_TRY(hipMemset(ptr + kScratchErrsOff, 0, 3 * sizeof(unsigned long long)));
    HIP_TRY(hipDeviceSynchronize());
    g_scratch_ptr[device] = ptr;
    return IODF_OK;
}

// Bytes of the per-call region a batch needs: latents, codes, lane words, lane states.
static size_t scratch_need(const iodf_ctx* ctx, long long batch) {
    const size_t B = (size_t)batch;
    return align256(4 * B * (size_t)ctx->d) + align256(B * (size_t)std::max<long long>(ctx->d_codes, 1)) +
           align256(4 * B * (size_t)ctx->lane_words_per_image) + align256(16 * B * (size_t)ctx->chunks.n_chunks * kLanes);
}

int iodf_encode_noalloc(iodf_ctx* ctx, const uint8_t* x_dev, int batch, uint32_t* words_dev, int64_t cap_words,
                        uint32_t* sizes_dev, void* stream) {
    if (!ctx) return IODF_E_ARG;
    if (batch < 0 || batch > ctx->max_batch) return IODF_E_BATCH;
    if (batch == 0) return IODF_OK;
    if (!x_dev || !words_dev || !sizes_dev || cap_words < 1) return IODF_E_ARG;
    if (scratch_need(ctx, batch) > kScratchBytes - kScratchCallOff) return IODF_E_SCRATCH;
    unsigned char* const ptr = g_scratch_ptr[ctx->device];  // set by iodf_init on this device
    if (!ptr) return IODF_E_ARG;
    hipStream_t st = (hipStream_t)stream;
    HIP_TRY(hipSetDevice(ctx->device));
    // carve the per-call region; every word read below is written by this call first (the flow writes
    // all latents and codes of the batch, the coder writes each lane's state and the words it counts),
    // so nothing has to be cleared and what an earlier, larger call left behind is never read
    const size_t B = (size_t)batch;
    unsigned char* q = ptr + kScratchCallOff;
    int32_t* zbuf = (int32_t*)q;            q += align256(4 * B * (size_t)ctx->d);
    int8_t* cbuf = (int8_t*)q;              q += align256(B * (size_t)std::max<long long>(ctx->d_codes, 1));
    uint32_t* lane_words = (uint32_t*)q;    q += align256(4 * B * (size_t)ctx->lane_words_per_image);
    uint32_t* lane_meta = (uint32_t*)q;
    unsigned long long* errs = (unsigned long long*)(ptr + kScratchErrsOff);
    const CodecTables t{(const int32_t*)(ptr + kScratchSigOff), (const int64_t*)(ptr + kScratchInvOff)};
    // the flow, launched kernel by kernel (a HIP graph would be instantiated, which allocates)
    int rc = enqueue_forward(ctx, x_dev, batch, zbuf, ctx->d_codes ? cbuf : nullptr, st);
    if (rc != IODF_OK) return rc;
    ctx->used_static_scratch = true;
    const int8_t* codes = ctx->d_codes ? cbuf : nullptr;
    PROF_LAUNCH(ctx, st, CLS_RANS_ENCODE, 0, (long long)batch * (4 * ctx->d + ctx->d_codes),
                launch_rans_encode(t, ctx->chunks, zbuf, ctx->d, codes, ctx->d_codes, batch, lane_words,
                                   ctx->lane_words_per_image, lane_meta, errs, st));
    PROF_LAUNCH(ctx, st, CLS_RANS_PACK, 0, 0,
                launch_rans_pack(ctx->chunks, lane_words, ctx->lane_words_per_image, lane_meta, batch, words_dev,
                                 cap_words, sizes_dev, errs, st));
    return IODF_OK;
}

// Decoding interleaves coder and flow: the latents of a level can be read only after the deeper
// levels are inverted, because the head that parameterises their prior reads the half of the
// level's state that continued downwards.
int iodf_decode(iodf_ctx* ctx, const uint32_t* words_dev, int64_t cap_words, int batch, uint8_t* x_dev, void* stream) {
    if (!ctx) return IODF_E_ARG;
    if (batch < 0 || batch > ctx->max_batch) return IODF_E_BATCH;
    if (batch == 0) return IODF_OK;
    if (!words_dev || !x_dev) return IODF_E_ARG;
    hipStream_t st = (hipStream_t)stream;
    HIP_TRY(hipSetDevice(ctx->device));
    int rc = codec_prepare(ctx);
    if (rc != IODF_OK) return rc;
    const HostModel& m = ctx->shape;
    if (cap_words < 1 + 3LL * m.levels * kLanes) return IODF_E_ARG;  // not even a header
    const CodecTables t{ctx->codec_sig, ctx->codec_inv};
    for (int lv = m.levels; lv >= 1; --lv) {
        const int C = level_channels(lv), h = m.H >> lv, w = m.W >> lv;
        const int n0 = ctx->first_net[lv];
        const int32_t* phi = (const int32_t*)(ctx->params + ctx->nets[n0 + m.couplings - 1].phi_off);
        const bool last = lv == m.levels;
        const bool head = !last && m.has_heads;
        if (head) {
            // kept half back from the deeper level (the emitted half still holds stale values),
            // then the head on it gives this level's codes
            PROF_LAUNCH(ctx, st, CLS_UNFACTOR, 0, 8LL * batch * C * h * w,
                        launch_unfactor(ctx->state[lv], batch, h, w, C, phi, C / 2, ctx->codec_z, ctx->d, ctx->z_off[lv],
                                        ctx->state[lv + 1], st));
            rc = run_net(ctx, ctx->nets[n0 + m.couplings], batch, +1, ctx->codec_codes, st);
            if (rc != IODF_OK) return rc;
        }
        PROF_LAUNCH(ctx, st, CLS_RANS_DECODE, 0, (long long)batch * 5 * ctx->chunks.n[lv - 1],
                    launch_rans_decode_chunk(t, ctx->chunks, lv - 1, words_dev, cap_words, batch,
                                             head ? ctx->codec_codes : nullptr, ctx->d_codes, ctx->codec_z, ctx->d,
                                             ctx->codec_errs, st));
        PROF_LAUNCH(ctx, st, CLS_UNFACTOR, 0, 8LL * batch * C * h * w,
                    launch_unfactor(ctx->state[lv], batch, h, w, C, phi, last ? 0 : C / 2, ctx->codec_z, ctx->d,
                                    ctx->z_off[lv], last ? nullptr : ctx->state[lv + 1], st));
        for (int k = m.couplings - 1; k >= 0; --k) {
            rc = run_net(ctx, ctx->nets[n0 + k], batch, -1, nullptr, st);
            if (rc != IODF_OK) return rc;
        }
    }
    PROF_LAUNCH(ctx, st, CLS_EMIT_X, 0, 5LL * batch * ctx->d,
                launch_emit_x(ctx->state[1], batch, m.H, m.W, x_dev, ctx->range_errs, st));
    return IODF_OK;
}

int iodf_tile_patches(iodf_ctx* ctx, const uint8_t* img_dev, int img_h, int img_w, int first_patch, int n_patches,
                      uint8_t* x_dev, void* stream) {
    if (!ctx || img_h < 1 || img_w < 1 || first_patch < 0 || n_patches < 0) return IODF_E_ARG;
    if (n_patches == 0) return IODF_OK;
    if (!img_dev || !x_dev) return IODF_E_ARG;
    const long long grid = (long long)((img_h + ctx->shape.H - 1) / ctx->shape.H) *
                           ((img_w + ctx->shape.W - 1) / ctx->shape.W);
    if ((long long)first_patch + n_patches > grid) return IODF_E_ARG;
    HIP_TRY(hipSetDevice(ctx->device));
    HIP_TRY(launch_tile_patches(img_dev, img_h, img_w, ctx->shape.H, ctx->shape.W, first_patch, n_patches, x_dev,
                                (hipStream_t)stream));
    return IODF_OK;
}

int iodf_untile_patches(iodf_ctx* ctx, const uint8_t* x_dev, int first_patch, int n_patches, uint8_t* img_dev,
                        int img_h, int img_w, void* stream) {
    if (!ctx || img_h < 1 || img_w < 1 || first_patch < 0 || n_patches < 0) return IODF_E_ARG;
    if (n_patches == 0) return IODF_OK;
    if (!img_dev || !x_dev) return IODF_E_ARG;
    const long long grid = (long long)((img_h + ctx->shape.H - 1) / ctx->shape.H) *
                           ((img_w + ctx->shape.W - 1) / ctx->shape.W);
    if ((long long)first_patch + n_patches > grid) return IODF_E_ARG;
    HIP_TRY(hipSetDevice(ctx->device));
    HIP_TRY(launch_untile_patches(x_dev, first_patch, n_patches, ctx->shape.H, ctx->shape.W, img_dev, img_h, img_w,
                                  (hipStream_t)stream));
    return IODF_OK;
}

// One integer-only convolution layer on its own (Sec. 4.3, Table 1 times three such shapes): host
// tensors in, host tensors out, the same packing and kernels as inside a flow.
static int conv_probe_impl(int device_ordinal, int c_in, int c_out, int k, int h, int w, int batch, int relu,
                           const int8_t* x_host, const int8_t* w_host, const int32_t* bias_host, const int32_t* m_host,
                           const uint8_t* shift_host, int8_t* y_host, int iters, float* us_per_call,
                           int64_t* timeline_host, int max_tiles, int* n_tiles) {
    if (timeline_host && (max_tiles < 1 || !n_tiles)) return IODF_E_ARG;
    if (c_in < 1 || c_out < 1 || (k != 1 && k != 3) || h < 1 || w < 1 || h > 8192 || w > 8192 || batch < 1 || c_in > 65536 || c_out > 65536 ||
        !x_host || !w_host || !bias_host || !m_host || !shift_host || !y_host || iters < 1)
        return IODF_E_ARG;
    for (int c = 0; c < c_out; ++c)
        if (shift_host[c] > 62 || m_host[c] < 0 || bias_host[c] >= (1 << 30) || bias_host[c] <= -(1 << 30)) return IODF_E_ARG;
    HIP_TRY(hipSetDevice(device_ordinal));
    HIP_TRY(conv_setup());
    int n_cu = 0;
    HIP_TRY(conv_device_cus(&n_cu));
    std::vector<uint8_t> gate((size_t)c_out, 1);
    HostLayer L{c_out, c_in, k, relu ? 1 : 0, 0, w_host, bias_host, m_host, shift_host, gate.data()};
    Arena A;
    DevLayer D{};
    const int cin_pad = round64(c_in), n_pad = round64(c_out);
    std::vector<int> rows((size_t)c_out), cols((size_t)c_in);
    for (int i = 0; i < c_out; ++i) rows[i] = i;
    for (int i = 0; i < c_in; ++i) cols[i] = i;
    pack_layer(A, L, rows, cols, cin_pad, D);
    const long long pp = (long long)(h + 2) * (w + 2);
    const long long plane = ((long long)batch * pp * 64 + 1023) / 1024 * 1024;
    if (plane >= (1LL << 31)) return IODF_E_BATCH;
    const size_t in_bytes = (size_t)plane * (cin_pad / 64), out_bytes = (size_t)plane * (n_pad / 64);
    // host staging in the library's plane layout (zero borders, zero padding channels)
    std::vector<int8_t> xin(in_bytes, 0), yout(out_bytes, 0);
    for (int b = 0; b < batch; ++b)
        for (int c = 0; c < c_in; ++c)
            for (int i = 0; i < h; ++i)
                for (int j = 0; j < w; ++j)
                    xin[(size_t)(c / 64) * plane + ((size_t)b * pp + (size_t)(i + 1) * (w + 2) + (j + 1)) * 64 + c % 64] =
                        x_host[(((size_t)b * c_in + c) * h + i) * w + j];
    uint8_t* params = nullptr;
    int8_t *din = nullptr, *dout = nullptr;
    long long* dtrace = nullptr;
    int rc = IODF_OK;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    auto cleanup = [&]() {
        if (dtrace) (void)hipFree(dtrace);
        if (params) (void)hipFree(params);
        if (din) (void)hipFree(din);
        if (dout) (void)hipFree(dout);
        if (e0) (void)hipEventDestroy(e0);
        if (e1) (void)hipEventDestroy(e1);
    };
#define PROBE_TRY(expr)                                                  \
    do {                                                                 \
        const hipError_t e__ = (expr);                                   \
        if (e__ != hipSuccess) { g_last_hip = (int)e__; cleanup(); return IODF_E_HIP; } \
    } while (0)
    PROBE_TRY(hipMalloc((void**)&params, A.host.size()));
    PROBE_TRY(hipMalloc((void**)&din, in_bytes));
    PROBE_TRY(hipMalloc((void**)&dout, out_bytes));
    PROBE_TRY(hipMemcpy(params, A.host.data(), A.host.size(), hipMemcpyHostToDevice));
    PROBE_TRY(hipMemcpy(din, xin.data(), in_bytes, hipMemcpyHostToDevice));
    PROBE_TRY(hipMemset(dout, 0, out_bytes));
    ConvArgs a;
    memset(&a, 0, sizeof(a));

    a.in = din; a.in_plane = plane; a.cin_pad = cin_pad; a.taps = k * k; a.h = h; a.w = w; a.npix = batch * h * w;
    a.n_cu = n_cu;
    a.wgt = (const int8_t*)(params + D.wgt_off); a.n_pad = n_pad;
    a.bias = (const int32_t*)(params + D.bias_off); a.mul = (const int32_t*)(params + D.mul_off);
    a.shift = (const int32_t*)(params + D.shift_off); a.rq_fast = D.rq_fast;
    a.clamp_hi = D.hi_off == (size_t)-1 ? nullptr : (const int32_t*)(params + D.hi_off);
    a.n_store = n_pad; a.mode = MODE_ACT; a.relu = relu ? 1 : 0; a.out = dout; a.out_plane = plane;
    PROBE_TRY(hipEventCreate(&e0));
    PROBE_TRY(hipEventCreate(&e1));
    PROBE_TRY(launch_conv(a, nullptr));  // warm-up, and the run whose output is returned
    PROBE_TRY(hipDeviceSynchronize());
    PROBE_TRY(hipMemcpy(yout.data(), dout, out_bytes, hipMemcpyDeviceToHost));
    PROBE_TRY(hipEventRecord(e0, nullptr));
    for (int i = 0; i < iters; ++i) PROBE_TRY(launch_conv(a, nullptr));
    PROBE_TRY(hipEventRecord(e1, nullptr));
    PROBE_TRY(hipEventSynchronize(e1));
    float ms = 0.f;
    PROBE_TRY(hipEventElapsedTime(&ms, e0, e1));
    if (timeline_host) {
        // once more with the per-tile timeline on, after another run of back-to-back launches so that the
        // traced launch sees the clocks of sustained work
        const int slots = conv_trace_slots(a);
        if (slots < 1) { cleanup(); return IODF_E_ARG; }
        PROBE_TRY(hipMalloc((void**)&dtrace, 64 * (size_t)slots));
        PROBE_TRY(hipMemset(dtrace, 0, 64 * (size_t)slots));
        for (int i = 0; i < iters; ++i) PROBE_TRY(launch_conv(a, nullptr));
        a.trace = dtrace;
        a.has_trace = 1;
        PROBE_TRY(launch_conv(a, nullptr));
        a.trace = nullptr;
        a.has_trace = 0;
        PROBE_TRY(hipDeviceSynchronize());
        std::vector<long long> tl(8 * (size_t)slots);
        PROBE_TRY(hipMemcpy(tl.data(), dtrace, 64 * (size_t)slots, hipMemcpyDeviceToHost));
        int n = 0;
        for (int sl = 0; sl < slots && n < max_tiles; ++sl)
            if (tl[8 * (size_t)sl + 3]) { memcpy(timeline_host + 8 * (size_t)n, &tl[8 * (size_t)sl], 64); ++n; }
        *n_tiles = n;
    }
#undef PROBE_TRY
    if (us_per_call) *us_per_call = 1e3f * ms / (float)iters;
    for (int b = 0; b < batch; ++b)
        for (int c = 0; c < c_out; ++c)
            for (int i = 0; i < h; ++i)
                for (int j = 0; j < w; ++j)
                    y_host[(((size_t)b * c_out + c) * h + i) * w + j] =
                        yout[(size_t)(c / 64) * plane + ((size_t)b * pp + (size_t)(i + 1) * (w + 2) + (j + 1)) * 64 + c % 64];
    cleanup();
    return rc;
}

int iodf_conv_probe(int device_ordinal, int c_in, int c_out, int k, int h, int w, int batch, int relu,
                    const int8_t* x_host, const int8_t* w_host, const int32_t* bias_host, const int32_t* m_host,
                    const uint8_t* shift_host, int8_t* y_host, int iters, float* us_per_call) {
    return conv_probe_impl(device_ordinal, c_in, c_out, k, h, w, batch, relu, x_host, w_host, bias_host, m_host,
                           shift_host, y_host, iters, us_per_call, nullptr, 0, nullptr);
}

int iodf_conv_probe_timeline(int device_ordinal, int c_in, int c_out, int k, int h, int w, int batch, int relu,
                             const int8_t* x_host, const int8_t* w_host, const int32_t* bias_host,
                             const int32_t* m_host, const uint8_t* shift_host, int8_t* y_host, int iters,
                             float* us_per_call, int64_t* timeline_host, int max_tiles, int* n_tiles) {
    if (!timeline_host) return IODF_E_ARG;
    return conv_probe_impl(device_ordinal, c_in, c_out, k, h, w, batch, relu, x_host, w_host, bias_host, m_host,
                           shift_host, y_host, iters, us_per_call, timeline_host, max_tiles, n_tiles);
}

int iodf_profile_begin(iodf_ctx* ctx, int max_launches) {
    if (!ctx || max_launches < 1 || max_launches > (1 << 22)) return IODF_E_ARG;
    if (ctx->prof_on) return IODF_E_ARG;
    HIP_TRY(hipSetDevice(ctx->device));
    ctx->prof_ev.assign(2 * (size_t)max_launches, nullptr);
    for (hipEvent_t& e : ctx->prof_ev) {
        const hipError_t er = hipEventCreate(&e);
        if (er != hipSuccess) {
            for (hipEvent_t& d : ctx->prof_ev)
                if (d) (void)hipEventDestroy(d);
            ctx->prof_ev.clear();
            g_last_hip = (int)er;
            return IODF_E_HIP;
        }
    }
    ctx->prof_recs.clear();
    ctx->prof_recs.reserve((size_t)max_launches);
    ctx->prof_on = true;
    return IODF_OK;
}

int iodf_profile_end(iodf_ctx* ctx, iodf_kernel_stat* stats, int max_stats, int* n_stats) {
    if (!ctx || !stats || !n_stats || max_stats < 1) return IODF_E_ARG;
    if (!ctx->prof_on) return IODF_E_ARG;
    ctx->prof_on = false;
    // classes: the flow-state passes, then every conv tile split into its 1x1 and 3x3 launches, then
    // two views over the same conv launches: the wide layers (C_in and C_out >= 128), all of them and
    // those of levels 1-2 only
    const int nkern = NUM_FLOW_CLS + 2 * conv_num_tiles();
    const int ncls = nkern + 2;
    std::vector<iodf_kernel_stat> acc((size_t)ncls);
    for (int c = 0; c < ncls; ++c) {
        memset(&acc[c], 0, sizeof(iodf_kernel_stat));
        if (c < NUM_FLOW_CLS)
            strncpy(acc[c].name, kFlowClsName[c], sizeof(acc[c].name) - 1);
        else if (c >= nkern)
            strncpy(acc[c].name, c == nkern ? "view: wide conv layers" : "view: wide conv layers, levels 1-2",
                    sizeof(acc[c].name) - 1);
        else
            snprintf(acc[c].name, sizeof(acc[c].name), "%s %s", conv_tile_name((c - NUM_FLOW_CLS) / 2),
                     ((c - NUM_FLOW_CLS) & 1) ? "3x3" : "1x1");
    }
    int rc = IODF_OK;
    for (size_t i = 0; i < ctx->prof_recs.size(); ++i) {
        float ms = 0.f;
        hipError_t e = hipEventSynchronize(ctx->prof_ev[2 * i + 1]);
        if (e == hipSuccess) e = hipEventElapsedTime(&ms, ctx->prof_ev[2 * i], ctx->prof_ev[2 * i + 1]);
        if (e != hipSuccess) { g_last_hip = (int)e; rc = IODF_E_HIP; break; }
        const iodf_ctx::ProfRec& r = ctx->prof_recs[i];
        if (r.cls < 0 || r.cls >= ncls) continue;
        acc[r.cls].launches += 1;
        acc[r.cls].total_ms += ms;
        acc[r.cls].macs += r.macs;
        acc[r.cls].issued_macs += r.issued;
        for (int v = 0; v < r.wide; ++v) {
            iodf_kernel_stat& w = acc[(size_t)(nkern + v)];
            w.launches += 1; w.total_ms += ms; w.macs += r.macs; w.bytes += r.bytes; w.issued_macs += r.issued;
        }
        acc[r.cls].bytes += r.bytes;
    }
    for (hipEvent_t& e : ctx->prof_ev)
        if (e) (void)hipEventDestroy(e);
    ctx->prof_ev.clear();
    ctx->prof_recs.clear();
    int n = 0;
    for (int c = 0; c < ncls && n < max_stats; ++c)
        if (acc[c].launches) stats[n++] = acc[c];
    *n_stats = n;
    return rc;
}

int iodf_query(iodf_ctx* ctx, int what, int64_t* out) {
    if (!ctx || !out) return IODF_E_ARG;
    switch (what) {
        case IODF_Q_Z_ELEMS: *out = ctx->d; return IODF_OK;
        case IODF_Q_CODE_BYTES: *out = ctx->d_codes; return IODF_OK;
        case IODF_Q_WORKSPACE_BYTES: *out = (int64_t)ctx->workspace_bytes; return IODF_OK;
        case IODF_Q_MACS_FORWARD: *out = ctx->macs_fwd; return IODF_OK;
        case IODF_Q_MACS_INVERSE: *out = ctx->macs_inv; return IODF_OK;
        case IODF_Q_WIDE_MACS_FORWARD: *out = ctx->macs_wide; return IODF_OK;
        case IODF_Q_MAX_BATCH: *out = ctx->max_batch; return IODF_OK;
        case IODF_Q_IMAGE_H: *out = ctx->shape.H; return IODF_OK;
        case IODF_Q_IMAGE_W: *out = ctx->shape.W; return IODF_OK;
        case IODF_Q_CONV_LAUNCHES: *out = ctx->conv_launches; return IODF_OK;
        case IODF_Q_RANGE_ERRORS: {
            HIP_TRY(hipSetDevice(ctx->device));
            HIP_TRY(hipDeviceSynchronize());
            unsigned long long v = 0;
            HIP_TRY(hipMemcpy(&v, ctx->range_errs, sizeof(v), hipMemcpyDeviceToHost));
            HIP_TRY(hipMemset(ctx->range_errs, 0, sizeof(v)));
            *out = (int64_t)v;
            return IODF_OK;
        }
        case IODF_Q_CODEC_HEADER_WORDS: *out = 1 + 3LL * ctx->shape.levels * kLanes; return IODF_OK;
        case IODF_Q_CODEC_MAX_WORDS: *out = 1 + 3LL * ctx->shape.levels * kLanes + ctx->d; return IODF_OK;
        case IODF_Q_CODEC_CLAMPED:
        case IODF_Q_CODEC_OVERFLOWS:
        case IODF_Q_CODEC_BROKEN_LANES: {
            *out = 0;
            if (!ctx->codec_ready && !ctx->used_static_scratch) return IODF_OK;
            HIP_TRY(hipSetDevice(ctx->device));
            HIP_TRY(hipDeviceSynchronize());
            unsigned long long* where[2] = {
                ctx->codec_ready ? ctx->codec_errs + (what - IODF_Q_CODEC_CLAMPED) : nullptr,
                ctx->used_static_scratch
                    ? (unsigned long long*)(g_scratch_ptr[ctx->device] + kScratchErrsOff) + (what - IODF_Q_CODEC_CLAMPED)
                    : nullptr};
            for (unsigned long long* p : where) {
                if (!p) continue;
                unsigned long long v = 0;
                HIP_TRY(hipMemcpy(&v, p, sizeof(v), hipMemcpyDeviceToHost));
                HIP_TRY(hipMemset(p, 0, sizeof(v)));
                *out += (int64_t)v;
            }
            return IODF_OK;
        }
        case IODF_Q_NOALLOC_MAX_BATCH: {
            long long lo = 0, hi = ctx->max_batch;  // the need grows with the batch: bisect
            while (lo < hi) {
                const long long mid = (lo + hi + 1) / 2;
                if (scratch_need(ctx, mid) <= kScratchBytes - kScratchCallOff) lo = mid; else hi = mid - 1;
            }
            *out = lo;
            return IODF_OK;
        }
        default: return IODF_E_ARG;
    }
}

}  // extern "C"
