/*
 * CPU oracle for integer-only discrete-flow inference. TEST INFRASTRUCTURE ONLY:
 * see iodf_oracle.h. Plain loops, channel-first tensors, full-width networks with
 * gate masks, one rounding rule. Nothing here is shared with the GPU library.
 */
#include "iodf_oracle.h"
#include "iodf_codec_oracle.h"

#include <omp.h>
#include <stdlib.h>
#include <string.h>

enum { FAM_PLAIN = 0, FAM_RESNET = 1, FAM_DENSE = 2 };

typedef struct {
    int C_out, C_in, k, relu, shortcut;
    const int8_t* W;      /* [C_out][C_in][k][k] */
    const int32_t* bias;  /* [C_out] */
    const int32_t* M;     /* [C_out] */
    const uint8_t* shift; /* [C_out] */
    const uint8_t* gate;  /* [C_out] */
} orc_layer;

typedef struct {
    int kind, level, C, C_in, C_out, n_layers;
    int32_t M_in;
    int s_in;
    const int32_t* perm; /* [C] or NULL */
    orc_layer* layers;
} orc_net;

struct orc_model {
    uint8_t* blob;
    int H, W, levels, couplings, family, width, depth, has_heads, n_nets;
    int act_unsigned; /* tensors that leave a ReLU hold unsigned codes 0..255 (Eq. 3) */
    orc_net* nets;
};

static int g_threads = 0;
static int64_t g_max_abs_state = 0;

void orc_set_threads(int n) { g_threads = n; }
int orc_get_threads(void) { return g_threads > 0 ? g_threads : omp_get_max_threads(); }
int64_t orc_last_max_abs_state(void) { return g_max_abs_state; }

/* ---- arithmetic primitives ------------------------------------------------ */

/* Fixed-point rescale standing in for the real factor s_W s_x / s_y of Eq. 5:
 * the product is exact in 64 bits, then rounded half away from zero. */
int64_t orc_rq(int32_t a, int32_t M, int s) {
    int64_t v = (int64_t)a * (int64_t)M;
    int64_t half = s > 0 ? ((int64_t)1 << (s - 1)) : 0;
    if (v >= 0) return (v + half) >> s;
    return -((-v + half) >> s);
}

int32_t orc_sat8(int64_t u) {
    if (u > 127) return 127;
    if (u < -128) return -128;
    return (int32_t)u;
}

/* Eq. 4 with the input codes read as signed (-128..127) or, for xu != 0, as unsigned
 * (0..255) bytes (Eq. 3: activations after a ReLU may use the unsigned format). */
static void conv_acc_any(const void* xv, int xu, int D, int h, int w, const int8_t* W, int C, int k,
                         const int32_t* bias, const uint8_t* gate, int32_t* acc) {
    const int8_t* x = (const int8_t*)xv;
    const int p = (k - 1) / 2;
    const int nt = orc_get_threads();
#pragma omp parallel for num_threads(nt) schedule(static)
    for (int c = 0; c < C; ++c) {
        if (gate && !gate[c]) continue;
        int32_t* a = acc + (size_t)c * h * w;
        for (int i = 0; i < h * w; ++i) a[i] = bias ? bias[c] : 0;
        for (int cp = 0; cp < D; ++cp) {
            const int8_t* xc = x + (size_t)cp * h * w;
            for (int ky = 0; ky < k; ++ky) {
                for (int kx = 0; kx < k; ++kx) {
                    const int32_t wv = W[(((size_t)c * D + cp) * k + ky) * k + kx];
                    /* output (i,j) reads input (i+ky-p, j+kx-p); outside the map the
                     * input is 0, so only the (i,j) whose source is inside contribute */
                    const int i0 = p - ky > 0 ? p - ky : 0, i1 = h + p - ky < h ? h + p - ky : h;
                    const int j0 = p - kx > 0 ? p - kx : 0, j1 = w + p - kx < w ? w + p - kx : w;
                    for (int i = i0; i < i1; ++i) {
                        int32_t* ar = a + i * w;
                        const int8_t* xr = xc + (i + ky - p) * w + (kx - p);
                        if (xu)
                            for (int j = j0; j < j1; ++j) ar[j] += wv * (int32_t)(uint8_t)xr[j];
                        else
                            for (int j = j0; j < j1; ++j) ar[j] += wv * (int32_t)xr[j];
                    }
                }
            }
        }
    }
}

void orc_conv_acc(const int8_t* x, int D, int h, int w, const int8_t* W, int C, int k,
                  const int32_t* bias, const uint8_t* gate, int32_t* acc) {
    conv_acc_any(x, 0, D, h, w, W, C, k, bias, gate, acc);
}

void orc_conv_acc_u8(const uint8_t* x, int D, int h, int w, const int8_t* W, int C, int k,
                     const int32_t* bias, const uint8_t* gate, int32_t* acc) {
    conv_acc_any(x, 1, D, h, w, W, C, k, bias, gate, acc);
}

/* su: the shortcut bytes are unsigned codes; yu: the output is stored as unsigned codes,
 * saturated to [0, 255] (only meaningful after a ReLU). */
static void epilogue_any(const int32_t* acc, int C, int hw, const int32_t* M, const uint8_t* shift,
                         const uint8_t* gate, int relu, const void* shortcut, int su, void* y, int yu) {
    for (int c = 0; c < C; ++c) {
        for (int i = 0; i < hw; ++i) {
            const size_t o = (size_t)c * hw + i;
            /* a gated-off filter yields exactly 0 (bias included), Eq. 8 */
            int64_t u = (gate && !gate[c]) ? 0 : orc_rq(acc[o], M[c], shift[c]);
            /* the shortcut adds the block input's 8-bit code in the wide integer;
             * it is full width, so this is the scatter-add of Sec. 4.4 */
            if (shortcut) u += su ? (int64_t)((const uint8_t*)shortcut)[o] : (int64_t)((const int8_t*)shortcut)[o];
            if (relu && u < 0) u = 0;
            if (yu) ((uint8_t*)y)[o] = (uint8_t)(u > 255 ? 255 : (u < 0 ? 0 : u));
            else ((int8_t*)y)[o] = (int8_t)orc_sat8(u);
        }
    }
}

void orc_epilogue(const int32_t* acc, int C, int hw, const int32_t* M, const uint8_t* shift,
                  const uint8_t* gate, int relu, const int8_t* shortcut, int8_t* y) {
    epilogue_any(acc, C, hw, M, shift, gate, relu, shortcut, 0, y, 0);
}

void orc_epilogue_u8(const int32_t* acc, int C, int hw, const int32_t* M, const uint8_t* shift,
                     const uint8_t* gate, const uint8_t* shortcut, uint8_t* y) {
    epilogue_any(acc, C, hw, M, shift, gate, 1, shortcut, 1, y, 1);
}

void orc_squeeze(const int32_t* in, int C, int H, int W, int32_t* out) {
    const int h = H / 2, w = W / 2;
    for (int c = 0; c < C; ++c)
        for (int dy = 0; dy < 2; ++dy)
            for (int dx = 0; dx < 2; ++dx)
                for (int i = 0; i < h; ++i)
                    for (int j = 0; j < w; ++j)
                        out[((size_t)(4 * c + 2 * dy + dx) * h + i) * w + j] =
                            in[((size_t)c * H + 2 * i + dy) * W + 2 * j + dx];
}

void orc_unsqueeze(const int32_t* in, int C, int H, int W, int32_t* out) {
    const int h = H / 2, w = W / 2;
    for (int c = 0; c < C; ++c)
        for (int dy = 0; dy < 2; ++dy)
            for (int dx = 0; dx < 2; ++dx)
                for (int i = 0; i < h; ++i)
                    for (int j = 0; j < w; ++j)
                        out[((size_t)c * H + 2 * i + dy) * W + 2 * j + dx] =
                            in[((size_t)(4 * c + 2 * dy + dx) * h + i) * w + j];
}

/* ---- blob ------------------------------------------------------------------ */

static size_t pad4(size_t n) { return (n + 3) & ~(size_t)3; }

int orc_model_load(const void* blob, size_t bytes, orc_model** out) {
    if (!blob || !out || bytes < 64) return -1;
    orc_model* m = (orc_model*)calloc(1, sizeof(*m));
    if (!m) return -2;
    m->blob = (uint8_t*)malloc(bytes);
    if (!m->blob) { free(m); return -2; }
    memcpy(m->blob, blob, bytes);
    const uint32_t* h = (const uint32_t*)m->blob;
    if (h[0] != 0x46444F49u || h[1] != 0x31424C42u || h[2] != 1u) { orc_model_free(m); return -3; }
    m->H = (int)h[3]; m->W = (int)h[4]; m->levels = (int)h[5]; m->couplings = (int)h[6];
    m->family = (int)h[7]; m->width = (int)h[8]; m->depth = (int)h[9]; m->has_heads = (int)h[10];
    m->n_nets = (int)h[11];
    m->act_unsigned = (int)(h[12] & 1u);
    if (m->levels < 1 || m->levels > 8 || m->H <= 0 || m->W <= 0 || (m->H % (1 << m->levels)) ||
        (m->W % (1 << m->levels)) || m->n_nets < 1 || m->n_nets > 4096 || m->family > 2) {
        orc_model_free(m); return -3;
    }
    m->nets = (orc_net*)calloc((size_t)m->n_nets, sizeof(orc_net));
    size_t pos = 64;
#define NEED(n) do { if (pos + (n) > bytes) { orc_model_free(m); return -4; } } while (0)
    for (int n = 0; n < m->n_nets; ++n) {
        orc_net* net = &m->nets[n];
        NEED(32);
        const uint32_t* f = (const uint32_t*)(m->blob + pos);
        net->kind = (int)f[0]; net->level = (int)f[1]; net->C = (int)f[2]; net->C_in = (int)f[3];
        net->C_out = (int)f[4]; net->n_layers = (int)f[5];
        net->M_in = (int32_t)f[6]; net->s_in = (int)f[7];
        pos += 32;
        if (net->n_layers < 1 || net->n_layers > 1024 || net->s_in > 62 || net->M_in < 0 ||
            net->level < 1 || net->level > m->levels) { orc_model_free(m); return -3; }
        if (net->kind == 0) {
            NEED(4 * (size_t)net->C);
            net->perm = (const int32_t*)(m->blob + pos);
            pos += 4 * (size_t)net->C;
            /* must be a permutation of 0..C-1 */
            if (net->C < 2 || net->C > 4096) { orc_model_free(m); return -3; }
            uint8_t seen[4096];
            memset(seen, 0, sizeof(seen));
            for (int c = 0; c < net->C; ++c) {
                const int32_t pc = net->perm[c];
                if (pc < 0 || pc >= net->C || seen[pc]) { orc_model_free(m); return -3; }
                seen[pc] = 1;
            }
        }
        net->layers = (orc_layer*)calloc((size_t)net->n_layers, sizeof(orc_layer));
        for (int l = 0; l < net->n_layers; ++l) {
            orc_layer* L = &net->layers[l];
            NEED(16);
            const uint32_t* g = (const uint32_t*)(m->blob + pos);
            L->C_out = (int)g[0]; L->C_in = (int)g[1]; L->k = (int)g[2];
            L->relu = (int)(g[3] & 1u); L->shortcut = (int)((g[3] >> 1) & 1u);
            pos += 16;
            if (L->C_out < 1 || L->C_in < 1 || (L->k != 1 && L->k != 3)) { orc_model_free(m); return -3; }
            size_t nw = (size_t)L->C_out * L->C_in * L->k * L->k;
            NEED(pad4(nw)); L->W = (const int8_t*)(m->blob + pos); pos += pad4(nw);
            NEED(4 * (size_t)L->C_out); L->bias = (const int32_t*)(m->blob + pos); pos += 4 * (size_t)L->C_out;
            NEED(4 * (size_t)L->C_out); L->M = (const int32_t*)(m->blob + pos); pos += 4 * (size_t)L->C_out;
            NEED(pad4((size_t)L->C_out)); L->shift = m->blob + pos; pos += pad4((size_t)L->C_out);
            NEED(pad4((size_t)L->C_out)); L->gate = m->blob + pos; pos += pad4((size_t)L->C_out);
            for (int c = 0; c < L->C_out; ++c)
                if (L->shift[c] > 62 || L->M[c] < 0) { orc_model_free(m); return -3; }
        }
    }
#undef NEED
    if (pos != bytes) { orc_model_free(m); return -4; }
    *out = m;
    return 0;
}

void orc_model_free(orc_model* m) {
    if (!m) return;
    if (m->nets) {
        for (int n = 0; n < m->n_nets; ++n) free(m->nets[n].layers);
        free(m->nets);
    }
    free(m->blob);
    free(m);
}

int orc_model_num_nets(const orc_model* m) { return m->n_nets; }

static int level_channels(int level) { return 12 << (level - 1); }

int64_t orc_model_d(const orc_model* m) { return (int64_t)3 * m->H * m->W; }

int64_t orc_model_d_codes(const orc_model* m) {
    int64_t n = 0;
    if (!m->has_heads) return 0;
    for (int lv = 1; lv < m->levels; ++lv)
        n += (int64_t)level_channels(lv) * (m->H >> lv) * (m->W >> lv); /* 2 * C/2 code maps */
    return n;
}

/* ---- networks --------------------------------------------------------------- */

/* One conv layer on one image: accumulate (Eq. 4), then the integer epilogue. */
/* In the unsigned format (Eq. 3) a tensor that leaves a ReLU holds codes 0..255; xu / su say
 * whether the input and the shortcut are such tensors, and the output is one iff this layer has
 * a ReLU. Returns whether the output is unsigned. */
static int run_layer(const orc_model* m, const orc_layer* L, const int8_t* x, int xu, int h, int w,
                     const int8_t* shortcut, int su, int32_t* acc, int8_t* y) {
    const int yu = m->act_unsigned && L->relu;
    conv_acc_any(x, xu, L->C_in, h, w, L->W, L->C_out, L->k, L->bias, L->gate, acc);
    epilogue_any(acc, L->C_out, h * w, L->M, L->shift, L->gate, L->relu, shortcut, su, y, yu);
    return yu;
}

int orc_net_eval(const orc_model* m, int n, const int32_t* xa, int h, int w, int8_t* out) {
    if (n < 0 || n >= m->n_nets) return -1;
    const orc_net* net = &m->nets[n];
    const int hw = h * w;
    int maxc = net->C_in > net->C_out ? net->C_in : net->C_out;
    for (int l = 0; l < net->n_layers; ++l)
        if (net->layers[l].C_out > maxc) maxc = net->layers[l].C_out;
    int32_t* acc = (int32_t*)malloc((size_t)maxc * hw * sizeof(int32_t));
    /* input quantiser: the integer translation network sees 8-bit codes of x_a */
    int8_t* q = (int8_t*)malloc((size_t)net->C_in * hw);
    for (int i = 0; i < net->C_in * hw; ++i) q[i] = (int8_t)orc_sat8(orc_rq(xa[i], net->M_in, net->s_in));
    const orc_layer* Ls = net->layers;
    const int nl = net->n_layers;
    int rc = 0;
    if (m->family == FAM_PLAIN) {
        /* conv -> ReLU -> conv */
        if (nl != 2) { rc = -3; goto done; }
        int8_t* f = (int8_t*)malloc((size_t)Ls[0].C_out * hw);
        const int fu = run_layer(m, &Ls[0], q, 0, h, w, NULL, 0, acc, f);
        run_layer(m, &Ls[1], f, fu, h, w, NULL, 0, acc, out);
        free(f);
    } else if (m->family == FAM_RESNET) {
        /* conv_in, blocks r <- ReLU(r + conv1x1(ReLU(conv3x3(r)))) (Eq. 2), conv_out */
        if (nl < 2 || (nl % 2)) { rc = -3; goto done; }
        const int Wd = Ls[0].C_out;
        int8_t* r = (int8_t*)malloc((size_t)Wd * hw);
        int8_t* t1 = (int8_t*)malloc((size_t)Wd * hw);
        int8_t* r2 = (int8_t*)malloc((size_t)Wd * hw);
        int ru = run_layer(m, &Ls[0], q, 0, h, w, NULL, 0, acc, r);
        for (int l = 1; l + 1 < nl; l += 2) {
            const int tu = run_layer(m, &Ls[l], r, ru, h, w, NULL, 0, acc, t1);
            ru = run_layer(m, &Ls[l + 1], t1, tu, h, w, r, ru, acc, r2);
            memcpy(r, r2, (size_t)Wd * hw);
        }
        run_layer(m, &Ls[nl - 1], r, ru, h, w, NULL, 0, acc, out);
        free(r); free(t1); free(r2);
    } else {
        /* dense: f0 = conv_in; g = conv1x1(concat(f0..f_{l-1})); f_l = conv3x3(g);
         * conv_out over concat(f0..f_depth) */
        if (nl < 2 || (nl % 2)) { rc = -3; goto done; }
        const int Wd = Ls[0].C_out;
        const int depth = (nl - 2) / 2;
        int8_t* cat = (int8_t*)malloc((size_t)(depth + 1) * Wd * hw);
        int8_t* g = (int8_t*)malloc((size_t)Wd * hw);
        /* every feature of the concatenation leaves a ReLU, so the whole of it has one format */
        const int cu = run_layer(m, &Ls[0], q, 0, h, w, NULL, 0, acc, cat);
        for (int l = 1; l <= depth; ++l) {
            if (Ls[2 * l - 1].C_in != l * Wd || Ls[2 * l].C_in != Wd) { rc = -3; break; }
            const int gu = run_layer(m, &Ls[2 * l - 1], cat, cu, h, w, NULL, 0, acc, g);
            if (run_layer(m, &Ls[2 * l], g, gu, h, w, NULL, 0, acc, cat + (size_t)l * Wd * hw) != cu) { rc = -3; break; }
        }
        if (!rc) run_layer(m, &Ls[nl - 1], cat, cu, h, w, NULL, 0, acc, out);
        free(cat); free(g);
    }
done:
    free(acc); free(q);
    return rc;
}

/* ---- flow -------------------------------------------------------------------- */

static void track_state(const int32_t* s, size_t n) {
    int64_t mx = g_max_abs_state;
    for (size_t i = 0; i < n; ++i) {
        int64_t a = s[i] < 0 ? -(int64_t)s[i] : s[i];
        if (a > mx) mx = a;
    }
    g_max_abs_state = mx;
}

int orc_forward(const orc_model* m, const uint8_t* x, int batch, int32_t* z, int8_t* codes) {
    const int64_t d = orc_model_d(m), dc = orc_model_d_codes(m);
    g_max_abs_state = 0;
    int32_t* cur = (int32_t*)malloc((size_t)d * sizeof(int32_t));
    int32_t* tmp = (int32_t*)malloc((size_t)d * sizeof(int32_t));
    int8_t* t = (int8_t*)malloc((size_t)d);
    int rc = 0;
    for (int b = 0; b < batch && !rc; ++b) {
        const uint8_t* xb = x + (size_t)b * d;
        int32_t* zb = z + (size_t)b * d;
        int8_t* cb = codes ? codes + (size_t)b * dc : NULL;
        /* pixels are centred once: v = x - 128 */
        for (int64_t i = 0; i < d; ++i) cur[i] = (int32_t)xb[i] - 128;
        int C = 3, H = m->H, W = m->W, net = 0;
        for (int lv = 1; lv <= m->levels && !rc; ++lv) {
            orc_squeeze(cur, C, H, W, tmp);
            C *= 4; H /= 2; W /= 2;
            const int hw = H * W;
            memcpy(cur, tmp, (size_t)C * hw * sizeof(int32_t));
            for (int k = 0; k < m->couplings && !rc; ++k, ++net) {
                const orc_net* N = &m->nets[net];
                if (N->kind != 0 || N->C != C) { rc = -3; break; }
                /* channel permutation, then a = first half, b = second half */
                for (int c = 0; c < C; ++c)
                    memcpy(tmp + (size_t)c * hw, cur + (size_t)N->perm[c] * hw, (size_t)hw * sizeof(int32_t));
                memcpy(cur, tmp, (size_t)C * hw * sizeof(int32_t));
                const int Ca = C / 2;
                rc = orc_net_eval(m, net, cur, H, W, t);
                /* Eq. 1: z_a = x_a, z_b = x_b + t(x_a) */
                for (int i = 0; i < (C - Ca) * hw; ++i) cur[(size_t)Ca * hw + i] += t[i];
                track_state(cur, (size_t)C * hw);
            }
            if (rc) break;
            if (lv < m->levels) {
                /* factor-out: second half is emitted, first half continues and
                 * conditions the prior head */
                const int Ck = C / 2, Cz = C - Ck;
                memcpy(zb, cur + (size_t)Ck * hw, (size_t)Cz * hw * sizeof(int32_t));
                zb += (size_t)Cz * hw;
                if (m->has_heads) {
                    const orc_net* N = &m->nets[net];
                    if (N->kind != 1 || N->C_out != 2 * Cz) { rc = -3; break; }
                    rc = orc_net_eval(m, net, cur, H, W, t);
                    if (cb) { memcpy(cb, t, (size_t)2 * Cz * hw); cb += (size_t)2 * Cz * hw; }
                    ++net;
                }
                C = Ck;
            } else {
                memcpy(zb, cur, (size_t)C * hw * sizeof(int32_t));
            }
        }
    }
    free(cur); free(tmp); free(t);
    return rc;
}

int orc_inverse(const orc_model* m, const int32_t* z, int batch, uint8_t* x, int64_t* range_errors) {
    const int64_t d = orc_model_d(m);
    int64_t errs = 0;
    int32_t* cur = (int32_t*)malloc((size_t)d * sizeof(int32_t));
    int32_t* tmp = (int32_t*)malloc((size_t)d * sizeof(int32_t));
    int8_t* t = (int8_t*)malloc((size_t)d);
    /* index of the first network of each level and offset of each z chunk */
    int first_net[16];
    int64_t z_off[16];
    {
        int net = 0; int64_t off = 0;
        for (int lv = 1; lv <= m->levels; ++lv) {
            first_net[lv] = net;
            z_off[lv] = off;
            net += m->couplings + ((m->has_heads && lv < m->levels) ? 1 : 0);
            const int C = level_channels(lv);
            off += (int64_t)(lv < m->levels ? C - C / 2 : C) * (m->H >> lv) * (m->W >> lv);
        }
    }
    int rc = 0;
    for (int b = 0; b < batch && !rc; ++b) {
        const int32_t* zb = z + (size_t)b * d;
        for (int lv = m->levels; lv >= 1 && !rc; --lv) {
            const int C = level_channels(lv), H = m->H >> lv, W = m->W >> lv, hw = H * W;
            if (lv == m->levels) {
                memcpy(cur, zb + z_off[lv], (size_t)C * hw * sizeof(int32_t));
            } else {
                /* undo factor-out: first half came back from the deeper level (already in cur) */
                const int Ck = C / 2;
                memcpy(cur + (size_t)Ck * hw, zb + z_off[lv], (size_t)(C - Ck) * hw * sizeof(int32_t));
            }
            for (int k = m->couplings - 1; k >= 0 && !rc; --k) {
                const int net = first_net[lv] + k;
                const orc_net* N = &m->nets[net];
                const int Ca = C / 2;
                rc = orc_net_eval(m, net, cur, H, W, t);
                /* Eq. 1 inverted: x_b = z_b - t(z_a) */
                for (int i = 0; i < (C - Ca) * hw; ++i) cur[(size_t)Ca * hw + i] -= t[i];
                /* undo the permutation: permuted[c] = original[perm[c]] */
                for (int c = 0; c < C; ++c)
                    memcpy(tmp + (size_t)N->perm[c] * hw, cur + (size_t)c * hw, (size_t)hw * sizeof(int32_t));
                memcpy(cur, tmp, (size_t)C * hw * sizeof(int32_t));
            }
            orc_unsqueeze(cur, C / 4, 2 * H, 2 * W, tmp);
            memcpy(cur, tmp, (size_t)C * hw * sizeof(int32_t));
        }
        uint8_t* xb = x + (size_t)b * d;
        for (int64_t i = 0; i < d; ++i) {
            int32_t v = cur[i] + 128;
            if (v < 0) { v = 0; ++errs; }
            if (v > 255) { v = 255; ++errs; }
            xb[i] = (uint8_t)v;
        }
    }
    if (range_errors) *range_errors = errs;
    free(cur); free(tmp); free(t);
    return rc;
}

/* ---- compressor: flow + prior + coder (Sec. 3, Sec. 5.2, App. A) ---- */

/* Chunk c = level c + 1: latent count, offset in z, offset in codes (-1: no head). */
static int chunk_tables(const orc_model* m, int64_t* n, int64_t* z_off, int64_t* code_off) {
    int64_t zo = 0, co = 0;
    for (int lv = 1; lv <= m->levels; ++lv) {
        const int C = level_channels(lv);
        const int64_t hw = (int64_t)(m->H >> lv) * (m->W >> lv);
        const int64_t cz = lv < m->levels ? C - C / 2 : C;
        n[lv - 1] = cz * hw;
        z_off[lv - 1] = zo;
        zo += cz * hw;
        if (m->has_heads && lv < m->levels) { code_off[lv - 1] = co; co += 2 * cz * hw; }
        else code_off[lv - 1] = -1;
    }
    return m->levels;
}

int64_t orc_codec_max_words(const orc_model* m) {
    return orc_codec_header_words(m->levels) + orc_model_d(m);
}

int orc_encode(const orc_model* m, const uint8_t* x, int batch, uint32_t* out, int64_t cap, uint32_t* sizes,
               int64_t* n_clamped) {
    const int64_t d = orc_model_d(m), dc = orc_model_d_codes(m);
    int64_t n[16], z_off[16], code_off[16], clamped = 0;
    const int nch = chunk_tables(m, n, z_off, code_off);
    int32_t* z = (int32_t*)malloc((size_t)d * sizeof(int32_t));
    int8_t* codes = (int8_t*)malloc((size_t)(dc > 0 ? dc : 1));
    int rc = 0;
    for (int b = 0; b < batch && !rc; ++b) {
        rc = orc_forward(m, x + (size_t)b * d, 1, z, codes);
        if (rc) break;
        int64_t cl = 0;
        const int64_t w = orc_codec_encode_image(z, codes, nch, n, z_off, code_off, out + (size_t)b * cap, cap, &cl);
        sizes[b] = (uint32_t)w;
        clamped += cl;
    }
    if (n_clamped) *n_clamped = clamped;
    free(z); free(codes);
    return rc;
}

/* Decoding interleaves the coder with the flow: the latents of level lv can only be
 * read once the deeper levels have been inverted, because their prior parameters come
 * from the head on the half that continued downwards. */
int orc_decode(const orc_model* m, const uint32_t* cont, int64_t cap, int batch, uint8_t* x, int64_t* errors) {
    const int64_t d = orc_model_d(m);
    int64_t n[16], z_off[16], code_off[16], errs = 0;
    const int nch = chunk_tables(m, n, z_off, code_off);
    int first_net[16];
    {
        int net = 0;
        for (int lv = 1; lv <= m->levels; ++lv) {
            first_net[lv] = net;
            net += m->couplings + ((m->has_heads && lv < m->levels) ? 1 : 0);
        }
    }
    int32_t* cur = (int32_t*)malloc((size_t)d * sizeof(int32_t));
    int32_t* tmp = (int32_t*)malloc((size_t)d * sizeof(int32_t));
    int8_t* t = (int8_t*)malloc((size_t)d * 2);
    int rc = 0;
    for (int b = 0; b < batch && !rc; ++b) {
        const uint32_t* cb = cont + (size_t)b * cap;
        for (int lv = m->levels; lv >= 1 && !rc; --lv) {
            const int C = level_channels(lv), H = m->H >> lv, W = m->W >> lv, hw = H * W;
            const int Ck = lv == m->levels ? 0 : C / 2;
            const int8_t *mc = NULL, *lc = NULL;
            if (code_off[lv - 1] >= 0) {
                /* head on the kept half (already in cur[0 .. Ck*hw)) */
                rc = orc_net_eval(m, first_net[lv] + m->couplings, cur, H, W, t);
                if (rc) break;
                mc = t;
                lc = t + n[lv - 1];
            }
            if (orc_codec_decode_chunk(cb, cap, nch, n, lv - 1, mc, lc, cur + (size_t)Ck * hw) != 0) ++errs;
            for (int k = m->couplings - 1; k >= 0 && !rc; --k) {
                const int net = first_net[lv] + k;
                const orc_net* N = &m->nets[net];
                const int Ca = C / 2;
                rc = orc_net_eval(m, net, cur, H, W, t);
                for (int i = 0; i < (C - Ca) * hw; ++i) cur[(size_t)Ca * hw + i] -= t[i];
                for (int c = 0; c < C; ++c)
                    memcpy(tmp + (size_t)N->perm[c] * hw, cur + (size_t)c * hw, (size_t)hw * sizeof(int32_t));
                memcpy(cur, tmp, (size_t)C * hw * sizeof(int32_t));
            }
            orc_unsqueeze(cur, C / 4, 2 * H, 2 * W, tmp);
            memcpy(cur, tmp, (size_t)C * hw * sizeof(int32_t));
        }
        uint8_t* xb = x + (size_t)b * d;
        for (int64_t i = 0; i < d; ++i) {
            int32_t v = cur[i] + 128;
            if (v < 0) { v = 0; ++errs; }
            if (v > 255) { v = 255; ++errs; }
            xb[i] = (uint8_t)v;
        }
    }
    if (errors) *errors = errs;
    free(cur); free(tmp); free(t);
    return rc;
}
