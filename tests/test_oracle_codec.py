"""Pins of the entropy-coding oracle (oracle/iodf_codec_oracle.c): the integer
discretised-logistic prior (Sec. 3) and the streaming rANS coder (App. A) are
checked against things other than themselves: 50-digit decimal arithmetic, the
paper's float formula, hand-computed states, unbounded Python integers, the
information content of the symbols, and exact round trips. CPU only."""
import math
from decimal import Decimal, getcontext

import numpy as np
import pytest

import oracle
from synth import CONFIGS, make_blob, make_images
from synth.prng import bits64

M = 1 << 24
R = 8192
LOW = 1 << 31


class SplitMix64:
    """Sequential view of one seeded stream of the generator module."""

    def __init__(self, seed, block=4096):
        self.seed, self.block, self.pos, self.buf = seed, block, 0, []

    def next_u64(self):
        if not self.buf:
            self.buf = [int(v) for v in bits64(self.seed, self.block, self.pos)][::-1]
            self.pos += self.block
        return self.buf.pop()


# ---------------- tables ----------------

def test_sigmoid_table_is_correctly_rounded():
    getcontext().prec = 50
    sig, _ = oracle.prior_tables()
    assert sig.shape == (3073,)
    for j in range(3073):
        t = Decimal(-24) + Decimal(j) / Decimal(64)
        exact = Decimal(1 << 30) / (Decimal(1) + (-t).exp())
        want = int((exact + Decimal("0.5")).to_integral_value(rounding="ROUND_FLOOR"))
        assert int(sig[j]) == want, j
    assert sig[0] == 0 and sig[3072] == 1 << 30 and sig[1536] == 1 << 29
    assert np.all(np.diff(sig.astype(np.int64)) >= 0)


def test_inverse_scale_table_is_correctly_rounded():
    getcontext().prec = 50
    _, inv = oracle.prior_tables()
    ln2 = Decimal(2).ln()
    for l in range(-128, 128):
        exact = ((Decimal(23) - Decimal(l) / Decimal(16)) * ln2).exp()
        want = int((exact + Decimal("0.5")).to_integral_value(rounding="ROUND_FLOOR"))
        assert int(inv[l + 128]) == want, l
    assert inv[128] == 1 << 23          # l = 0: s = 1, 1/(2s) = 2^-1 in units of 2^-24
    assert inv[128 + 16] == 1 << 22     # l = 16: s = 2
    assert inv[128 - 16] == 1 << 24     # l = -16: s = 1/2


def test_integer_sigmoid_tracks_the_real_one():
    # linear interpolation of a 1/64 grid: error <= h^2/8 * max|sigma''| = (1/64)^2/8 * 0.0963 = 2.94e-6,
    # plus rounding of the entries and the floor (< 2 units of 2^-30)
    worst = 0.0
    prev = -1
    for T in range(-26 << 24, 26 << 24, 104729 * 7):
        S = oracle.prior_sigmoid(T)
        assert S >= prev  # monotone
        prev = S
        t = T / float(1 << 24)
        worst = max(worst, abs(S / float(1 << 30) - 1.0 / (1.0 + math.exp(-t))))
    assert worst < 3.0e-6
    assert oracle.prior_sigmoid(-(24 << 24)) == 0 and oracle.prior_sigmoid(24 << 24) == 1 << 30
    assert oracle.prior_sigmoid(0) == 1 << 29
    # exactly on a grid point the table value comes back
    sig, _ = oracle.prior_tables()
    for j in (1, 700, 1536, 2999):
        assert oracle.prior_sigmoid(((j - 1536) << 18)) == int(sig[j])


# ---------------- masses ----------------

@pytest.mark.parametrize("l", [-128, -77, -16, 0, 5, 16, 37, 64, 96, 127])
def test_masses_partition_the_total(l):
    z = np.arange(-R, R, dtype=np.int32)
    C, F, clamped = oracle.prior_cf(z, np.zeros_like(z, np.int8), np.full(z.shape, l, np.int8))
    assert clamped == 0
    C = C.astype(np.int64)
    F = F.astype(np.int64)
    assert C[0] == 0 and C[-1] + F[-1] == M          # G(-R) = 0, G(R) = M
    assert np.all(F >= 1)                             # every symbol can be coded
    assert np.array_equal(C[1:], C[:-1] + F[:-1])     # cumulative
    assert int(F.sum()) == M
    assert oracle.prior_cdf(-R, l) == 0 and oracle.prior_cdf(R, l) == M


def test_all_scales_keep_every_symbol_codable():
    z = np.arange(-R, R, dtype=np.int32)
    m0 = np.zeros_like(z, np.int8)
    for l in range(-128, 128):
        C, F, _ = oracle.prior_cf(z, m0, np.full(z.shape, l, np.int8))
        assert F.min() >= 1 and int(F.astype(np.int64).sum()) == M, l


@pytest.mark.parametrize("l", [-40, -16, 0, 16, 48, 96, 127])
def test_masses_follow_the_discretised_logistic(l):
    # Sec. 3: p(r) = sigma((r + 1/2)/s) - sigma((r - 1/2)/s), s = 2^(l/16). The integer prior
    # gives every symbol a floor mass 1 and spreads M - 2R by the CDF; two floors and two
    # interpolated sigmoids bound the deviation.
    s = 2.0 ** (l / 16.0)
    span = int(min(R - 1, max(8, 12 * s)))
    z = np.arange(-span, span + 1, dtype=np.int32)
    C, F, _ = oracle.prior_cf(z, np.zeros_like(z, np.int8), np.full(z.shape, l, np.int8))
    sg = lambda t: 1.0 / (1.0 + np.exp(-t))
    p = sg((z + 0.5) / s) - sg((z - 0.5) / s)
    want = (1.0 + (M - 2 * R) * p) / M
    assert np.max(np.abs(F / float(M) - want)) < 6.5e-6
    # the mode sits at r = 0 (up to the two floors) and the masses are symmetric around it
    assert int(F[span]) >= int(F.max()) - 2 and abs(int(np.argmax(F)) - span) <= max(1, s / 32)
    assert np.max(np.abs(F.astype(np.int64) - F[::-1].astype(np.int64))) <= 4


def test_mean_code_shifts_by_two_per_step_and_scale_code_is_sixteenth_octaves():
    z = np.arange(-300, 300, dtype=np.int32)
    for m in (-128, -3, 0, 9, 127):
        C, F, _ = oracle.prior_cf(z, np.full(z.shape, m, np.int8), np.full(z.shape, 32, np.int8))
        C0, F0, _ = oracle.prior_cf(z - 2 * m, np.zeros(z.shape, np.int8), np.full(z.shape, 32, np.int8))
        assert np.array_equal(C, C0) and np.array_equal(F, F0)
        assert int(z[np.argmax(F)]) == 2 * m            # the mode is mu = 2 m (a sign slip would give -2 m)
    # l -> l + 16 doubles s: the mass of the central symbol roughly halves (sigma'(0) = 1/4)
    f = [oracle.prior_cf(np.zeros(1, np.int32), np.zeros(1, np.int8), np.full(1, l, np.int8))[1][0] for l in (64, 80, 96)]
    assert abs(f[0] / f[1] - 2.0) < 0.01 and abs(f[1] / f[2] - 2.0) < 0.01
    # defaults: no codes means m = 0, l = 96
    Cd, Fd, _ = oracle.prior_cf(z)
    C96, F96, _ = oracle.prior_cf(z, np.zeros(z.shape, np.int8), np.full(z.shape, 96, np.int8))
    assert np.array_equal(Cd, C96) and np.array_equal(Fd, F96)


def test_residuals_outside_the_alphabet_are_clamped_and_counted():
    z = np.array([-R - 1, -R, R - 1, R, 40000, -40000], np.int32)
    C, F, clamped = oracle.prior_cf(z)
    assert clamped == 4
    assert C[0] == C[1] == 0 and C[2] == C[3] == C[4] and C[5] == 0
    # the mean moves the window
    _, _, cl = oracle.prior_cf(np.array([R + 100], np.int32), np.array([127], np.int8), np.array([0], np.int8))
    assert cl == 0


# ---------------- coder ----------------

def test_push_hand_computed():
    # X = 2^31, C = 3, F = 5: 2^31 = 5 * 429496729 + 3, no word shed (5 * 2^39 > 2^31)
    X, w = oracle.rans_push(LOW, 3, 5)
    assert w is None
    assert X == 429496729 * 16777216 + 3 + 3 == 7205759393726470  # (2^55 - 3 * 2^24) / 5 + 6
    # and back (App. A, decoder): floor(X / M) * F + (X mod M - C)
    assert X % M == 6 and oracle.rans_pop(X, 3, 5) == LOW
    # shedding: X = 5 * 2^39 + 12345 must first drop its low word 12345 -> X = 5 * 2^7 = 640 = 5 * 128
    X2, w2 = oracle.rans_push(5 * (1 << 39) + 12345, 3, 5)
    assert w2 == 12345 and X2 == 128 * M + 3 + 0
    # just below the threshold nothing is shed
    X3, w3 = oracle.rans_push(5 * (1 << 39) - 1, 3, 5)
    assert w3 is None and X3 == ((5 * (1 << 39) - 1) // 5) * M + 3 + (5 * (1 << 39) - 1) % 5 and X3 < 1 << 63


def test_push_matches_the_recurrence_in_unbounded_integers_and_inverts():
    g = SplitMix64(77)
    for _ in range(3000):
        F = 1 + g.next_u64() % (M - 1)
        C = g.next_u64() % (M - F + 1)
        X = LOW + g.next_u64() % ((F << 39) - LOW) if (F << 39) > LOW else LOW
        X1, w = oracle.rans_push(X, C, F)
        assert w is None
        # App. A: X_t = floor(X_{t-1}/F) * M + C + X_{t-1} mod F, in Python's unbounded integers
        assert X1 == (X // F) * M + C + X % F
        assert LOW <= X1 < 1 << 63
        assert C <= X1 % M < C + F                      # the slot names the symbol
        assert oracle.rans_pop(X1, C, F) == X           # decoder recurrence
        # information: the state grows by log2(M/F) bits, up to the rounding of X/F >= 2^7
        assert abs(math.log2(X1 / X) - math.log2(M / F)) < 0.0114 + 1e-9


def _chunks(seed, sizes, with_codes):
    g = SplitMix64(seed)
    n = np.array(sizes, np.int64)
    z_off = np.concatenate([[0], np.cumsum(n)[:-1]]).astype(np.int64)
    code_off, co = [], 0
    for i, k in enumerate(sizes):
        if with_codes[i]:
            code_off.append(co)
            co += 2 * k
        else:
            code_off.append(-1)
    d = int(n.sum())
    codes = np.zeros(max(co, 1), np.int8)
    z = np.zeros(d, np.int32)
    for i, k in enumerate(sizes):
        if with_codes[i]:
            m = np.array([int(g.next_u64() % 256) - 128 for _ in range(k)], np.int8)
            l = np.array([int(g.next_u64() % 160) - 64 for _ in range(k)], np.int8)
            codes[code_off[i]:code_off[i] + k] = m
            codes[code_off[i] + k:code_off[i] + 2 * k] = l
        else:
            m = np.zeros(k, np.int8)
            l = np.full(k, 96, np.int8)
        # latents scattered around their means by a few scales
        s = 2.0 ** (l.astype(np.float64) / 16.0)
        u = np.array([(g.next_u64() % 2000001) / 1e6 - 1.0 for _ in range(k)])
        z[z_off[i]:z_off[i] + k] = np.clip(np.round(2.0 * m + 3.0 * s * u), -R + 256, R - 257).astype(np.int32)
    return z, codes, n, z_off, np.array(code_off, np.int64)


@pytest.mark.parametrize("sizes,with_codes", [
    ((48, 16, 33), (True, True, False)),
    ((5, 1, 0, 17), (True, False, True, True)),      # fewer symbols than lanes, an empty chunk
    ((1536, 768), (True, False)),
])
def test_container_round_trip_layout_and_length(sizes, with_codes):
    z, codes, n, z_off, code_off = _chunks(11 + len(sizes), sizes, with_codes)
    nch = len(sizes)
    header = oracle.codec_header_words(nch)
    assert header == 1 + 3 * nch * 16
    cap = header + int(n.sum()) + 7
    cont, words, clamped = oracle.codec_encode_image(z, codes, n, z_off, code_off, cap)
    assert clamped == 0 and header <= words <= header + int(n.sum())
    assert cont[0] == words and int(cont[1:1 + nch * 16].sum()) == words - header
    assert np.all(cont[words:] == 0)                   # nothing written past the container
    # every chunk decodes back, independently of the others
    for c in range(nch):
        k = int(n[c])
        m = codes[code_off[c]:code_off[c] + k] if code_off[c] >= 0 else None
        l = codes[code_off[c] + k:code_off[c] + 2 * k] if code_off[c] >= 0 else None
        zc, rc = oracle.codec_decode_chunk(cont[:words], n, c, m, l)
        assert rc == 0 and np.array_equal(zc, z[z_off[c]:z_off[c] + k])
    # code length: payload + final states carry the symbols' information content, within the
    # coder's rounding (X/F >= 2^7, so each step is off by less than log2(1 + 2^-7) = 0.0113 bit)
    ideal = 0.0
    for c in range(nch):
        k = int(n[c])
        m = codes[code_off[c]:code_off[c] + k] if code_off[c] >= 0 else None
        l = codes[code_off[c] + k:code_off[c] + 2 * k] if code_off[c] >= 0 else None
        _, F, _ = oracle.prior_cf(z[z_off[c]:z_off[c] + k], m, l)
        ideal += float(np.sum(24.0 - np.log2(F.astype(np.float64))))
    st = cont[1 + nch * 16:1 + 3 * nch * 16].astype(np.uint64)
    states = st[0::2] | (st[1::2] << np.uint64(32))
    assert np.all(states >= np.uint64(LOW))
    info = 32.0 * (words - header) + float(np.sum(np.log2(states.astype(np.float64)) - 31.0))
    assert abs(info - ideal) <= 0.0114 * int(n.sum()) + 1e-6


def test_symbols_are_dealt_to_lanes_round_robin():
    # one improbable latent among cheap ones: the lane that got it ends with the largest state
    for e_far in (0, 18, 37, 63):
        z = np.zeros(64, np.int32)
        z[e_far] = 3000
        n = np.array([64], np.int64)
        cont, words, _ = oracle.codec_encode_image(z, None, n, np.zeros(1, np.int64), np.array([-1], np.int64), 200)
        st = cont[1 + 16:1 + 48].astype(np.uint64)
        states = st[0::2] | (st[1::2] << np.uint64(32))
        shed = cont[1:17]
        info = 32.0 * shed + np.log2(states.astype(np.float64))
        assert int(np.argmax(info)) == e_far % 16
    # header bookkeeping of an empty image
    cont, words, _ = oracle.codec_encode_image(np.zeros(0, np.int32), None, np.array([0], np.int64),
                                               np.zeros(1, np.int64), np.array([-1], np.int64), 60)
    assert words == 49 and cont[0] == 49 and np.all(cont[1:17] == 0)
    assert np.all(cont[17:49:2] == (1 << 31)) and np.all(cont[18:49:2] == 0)   # untouched lanes: state 2^31


def test_malformed_containers_are_rejected_and_capacity_is_respected():
    z, codes, n, z_off, code_off = _chunks(5, (200, 40), (True, False))
    header = oracle.codec_header_words(2)
    cap = header + 240
    cont, words, _ = oracle.codec_encode_image(z, codes, n, z_off, code_off, cap)
    m, l = codes[:200], codes[200:400]
    assert oracle.codec_decode_chunk(cont[:words], n, 0, m, l)[1] == 0
    bad = cont[:words].copy()
    bad[1 + 3] += 1                                     # a lane claims one word more
    assert oracle.codec_decode_chunk(bad, n, 0, m, l)[1] == -1
    bad = cont[:words].copy()
    assert words > header
    bad[words - 1] ^= 0x10                              # payload bit flip (the short chunk sheds no words)
    zc, rc = oracle.codec_decode_chunk(bad, n, 0, m, l)
    assert rc == -1 or not np.array_equal(zc, z[:200])
    bad = cont[:words].copy()
    bad[1 + 2 * 16 + 2 * (16 + 5)] ^= 0x10              # low word of the final state of chunk 1, lane 5
    zc, rc = oracle.codec_decode_chunk(bad, n, 1, None, None)
    assert rc == -1 or not np.array_equal(zc, z[200:])
    assert oracle.codec_decode_chunk(cont[:header - 1], n, 0, m, l)[1] == -1
    # wrong codes at the decoder: the symbols do not come back
    zc, rc = oracle.codec_decode_chunk(cont[:words], n, 0, m, (l.astype(np.int16) + 1).astype(np.int8))
    assert rc == -1 or not np.array_equal(zc, z[:200])
    # a buffer that is too small is never overrun, and the needed size is still reported
    small, need, _ = oracle.codec_encode_image(z, codes, n, z_off, code_off, header + 3)
    assert need == words and small.size == header + 3


# ---------------- whole compressor on small flows ----------------

@pytest.mark.parametrize("name", ["mini_dense", "mini_dense_g", "mini_resnet", "cfg1"])
def test_flow_codec_round_trip(name):
    cfg = CONFIGS[name]
    om = oracle.Model(make_blob(cfg))
    x = make_images(cfg, batch=3)
    cont, sizes, clamped = om.encode(x)
    assert clamped == 0
    assert cont.shape[1] == om.codec_max_words() == oracle.codec_header_words(cfg.levels) + om.d
    x2, errs = om.decode(cont, x.shape[1:])
    assert errs == 0 and np.array_equal(x, x2)
    # the containers hold exactly the flow's latents under the heads' codes
    z, codes = om.forward(x)
    for b in range(3):
        n, z_off, code_off, co, zo = [], [], [], 0, 0
        for lv in range(1, cfg.levels + 1):
            C = 12 << (lv - 1)
            hw = (cfg.H >> lv) * (cfg.W >> lv)
            cz = C - C // 2 if lv < cfg.levels else C
            n.append(cz * hw); z_off.append(zo); zo += cz * hw
            if cfg.heads and lv < cfg.levels:
                code_off.append(co); co += 2 * cz * hw
            else:
                code_off.append(-1)
        ref, words, _ = oracle.codec_encode_image(z[b], codes[b] if om.d_codes else None, n, z_off, code_off,
                                                  cont.shape[1])
        assert words == sizes[b] and np.array_equal(ref, cont[b])
    # images are coded independently
    c1, s1, _ = om.encode(x[1:2])
    assert s1[0] == sizes[1] and np.array_equal(c1[0], cont[1])


def test_decoder_needs_the_heads():
    # with heads the deeper latents condition the shallower ones: corrupting a deep chunk's
    # payload must break the image (it would not if the decoder ignored the heads' inputs)
    cfg = CONFIGS["mini_dense"]
    assert cfg.heads and cfg.levels >= 2
    om = oracle.Model(make_blob(cfg))
    x = make_images(cfg, batch=1)
    cont, sizes, _ = om.encode(x)
    bad = cont.copy()
    bad[0, sizes[0] - 1] ^= 0x4000
    x2, errs = om.decode(bad, x.shape[1:])
    assert errs > 0 or not np.array_equal(x, x2)


# ---------------- patches ----------------

def test_patch_tiling_against_a_reshape_and_by_hand():
    rng = np.random.default_rng(3)
    img = rng.integers(0, 256, size=(3, 8, 12), dtype=np.uint8)
    p = oracle.tile_patches(img, 4, 4)
    # exact multiple: the same thing written as a reshape
    want = img.reshape(3, 2, 4, 3, 4).transpose(1, 3, 0, 2, 4).reshape(6, 3, 4, 4)
    assert np.array_equal(p, want)
    assert np.array_equal(oracle.untile_patches(p, 8, 12), img)
    # ragged: 5 x 7 image, 4 x 4 patches -> 2 x 2 grid, mid-grey outside
    img = np.arange(3 * 5 * 7, dtype=np.uint8).reshape(3, 5, 7)
    p = oracle.tile_patches(img, 4, 4)
    assert p.shape == (4, 3, 4, 4)
    assert p[1, 0, 0, 2] == img[0, 0, 6] and p[1, 0, 0, 3] == 128          # patch (0,1): columns 4..7, 7 is outside
    assert p[2, 2, 0, 1] == img[2, 4, 1] and np.all(p[2, :, 1:, :] == 128)  # patch (1,0): only row 4 is inside
    assert p[3, 1, 0, 2] == img[1, 4, 6] and p[3, 1, 1, 2] == 128
    assert np.array_equal(oracle.untile_patches(p, 5, 7), img)
