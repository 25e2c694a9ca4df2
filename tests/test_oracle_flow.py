"""Pins for the oracle's flow: invertibility, closed forms for degenerate networks,
wiring of the three t() families, gate semantics, batch independence, the state
bound, and rejection of malformed blobs. CPU only."""
from fractions import Fraction

import numpy as np
import pytest

import oracle
from synth import CONFIGS, FlowConfig, DENSE, RESNET, PLAIN, make_blob, make_images, parse_blob
from synth.model import pack_blob

SMALL = ["cfg1", "mini_dense", "mini_dense_g", "mini_resnet", "mini_resnet_g", "odd_dense_g"]
ONE = 1 << 30   # with shift 30: scale exactly 1


def _half_away(q):
    r = int(abs(q) + Fraction(1, 2))
    return r if q >= 0 else -r


def _squeeze_np(a):
    C, H, W = a.shape
    return a.reshape(C, H // 2, 2, W // 2, 2).transpose(0, 2, 4, 1, 3).reshape(4 * C, H // 2, W // 2)


def _layout_chain(v, model, add=None):
    """Closed form of the flow when every translation is a per-channel constant:
    squeeze, permute, add the constants to the second half, split. `add(net_index)`
    returns the constants of that coupling (or None for t == 0)."""
    cur, chunks, net = v, [], 0
    L, K = model["levels"], model["couplings"]
    for lv in range(1, L + 1):
        cur = _squeeze_np(cur)
        for _ in range(K):
            cur = cur[model["nets"][net]["perm"]].copy()
            if add is not None:
                C = cur.shape[0]
                cur[C // 2:] += add(net)[:, None, None]
            net += 1
        C = cur.shape[0]
        if lv < L:
            chunks.append(cur[C // 2:].reshape(-1))
            cur = cur[:C // 2]
            if model["has_heads"]:
                net += 1
        else:
            chunks.append(cur.reshape(-1))
    return np.concatenate(chunks)


# ---- invertibility -------------------------------------------------------------

@pytest.mark.parametrize("name", SMALL)
def test_round_trip_is_exact(name):
    cfg = CONFIGS[name]
    m = oracle.Model(make_blob(cfg))
    for kind in ("filtered", "uniform"):
        x = make_images(cfg, kind=kind)
        z, _ = m.forward(x)
        x2, errs = m.inverse(z, x.shape[1:])
        assert errs == 0 and np.array_equal(x, x2)
    # extreme images
    for val in (0, 255):
        x = np.full((1, 3, cfg.H, cfg.W), val, dtype=np.uint8)
        z, _ = m.forward(x)
        x2, errs = m.inverse(z, x.shape[1:])
        assert errs == 0 and np.array_equal(x, x2)


@pytest.mark.parametrize("name", ["cfg1", "mini_dense", "mini_resnet_g"])
def test_forward_inverts_inverse_on_arbitrary_latents(name):
    # f is a bijection of Z^d: any z whose decoded pixels stay in range maps back to itself
    cfg = CONFIGS[name]
    m = oracle.Model(make_blob(cfg))
    rng = np.random.default_rng(1)
    z = rng.integers(-40, 40, (2, cfg.d)).astype(np.int32)
    x, errs = m.inverse(z, (3, cfg.H, cfg.W))
    assert errs == 0
    z2, _ = m.forward(x)
    assert np.array_equal(z, z2)


def test_inverse_counts_out_of_range_pixels():
    cfg = CONFIGS["cfg1"]
    m = oracle.Model(make_blob(cfg, mode="zero"))
    z = np.zeros((1, cfg.d), dtype=np.int32)
    z[0, 0] = 200      # 200 + 128 > 255
    z[0, 5] = -300     # < 0
    x, errs = m.inverse(z, (3, cfg.H, cfg.W))
    assert errs == 2 and x.max() == 255 and x.min() == 0


# ---- closed forms ----------------------------------------------------------------

@pytest.mark.parametrize("name", ["cfg1", "mini_dense", "mini_resnet", "mid_dense"])
def test_zero_network_gives_pure_layout_chain(name):
    cfg = CONFIGS[name]
    blob = make_blob(cfg, mode="zero")
    model = parse_blob(blob)
    m = oracle.Model(blob)
    x = make_images(cfg, batch=2)
    z, codes = m.forward(x)
    for b in range(2):
        want = _layout_chain(x[b].astype(np.int64) - 128, model)
        assert np.array_equal(z[b], want)
    assert not codes.any()


@pytest.mark.parametrize("name", ["cfg1", "mini_dense", "mini_resnet"])
def test_bias_only_network_adds_constants(name):
    cfg = CONFIGS[name]
    blob = make_blob(cfg, mode="bias_only")
    model = parse_blob(blob)
    m = oracle.Model(blob)

    def consts(net):
        L = model["nets"][net]["layers"][-1]
        return np.array([max(-128, min(127, _half_away(Fraction(int(b) * int(M), 2 ** int(s)))))
                         for b, M, s in zip(L["bias"], L["M"], L["shift"])], dtype=np.int64)

    assert any(consts(n).any() for n in range(len(model["nets"])) if model["nets"][n]["kind"] == 0)
    x = make_images(cfg, batch=2)
    z, codes = m.forward(x)
    for b in range(2):
        assert np.array_equal(z[b], _layout_chain(x[b].astype(np.int64) - 128, model, consts))
    if cfg.heads:
        # head codes are the constants of the head's last layer, one value per code map
        pos = 0
        for n, net in enumerate(model["nets"]):
            if net["kind"] == 1:
                h, w = cfg.level_hw(net["level"])
                c = consts(n)
                blk = codes[0, pos:pos + c.size * h * w].reshape(c.size, h * w)
                assert np.array_equal(blk, np.repeat(c[:, None], h * w, axis=1))
                pos += c.size * h * w
        assert pos == cfg.d_codes


# ---- wiring of the t() families ----------------------------------------------------

def _shift2d(a, dy, dx):
    """out[i,j] = a[i+dy, j+dx], zero outside."""
    h, w = a.shape
    out = np.zeros_like(a)
    ys, xs = slice(max(0, -dy), min(h, h - dy)), slice(max(0, -dx), min(w, w - dx))
    out[ys, xs] = a[max(0, dy):max(0, dy) + (ys.stop - ys.start), max(0, dx):max(0, dx) + (xs.stop - xs.start)]
    return out


def _one_level(family, width, depth, H=8, W=8):
    return FlowConfig("wiring", H, W, 1, 1, 1, family, width, depth, False, seed_id=99)


def _unit(L):
    L["M"][:] = ONE
    L["shift"][:] = 30
    L["bias"][:] = 0
    L["W"][:] = 0


def test_dense_family_wiring_selects_and_shifts():
    Wd, depth = 8, 2
    cfg = _one_level(DENSE, Wd, depth)
    blob = make_blob(cfg, mode="zero")
    model = parse_blob(blob)
    net = model["nets"][0]
    net["M_in"][:] = ONE
    net["s_in"][:] = 30
    Ls = net["layers"]
    for L in Ls:
        _unit(L)
    rng = np.random.default_rng(0)
    xa = rng.integers(-100, 100, (6, 4, 4)).astype(np.int32)
    relu = lambda a: np.maximum(a, 0)
    # conv_in: f0[c] = ReLU(sign_c * xa[c % 6]) read through tap (ky, kx) = (c % 3, 1)
    feats = []
    f0 = np.zeros((Wd, 4, 4), dtype=np.int64)
    for c in range(Wd):
        sgn = 1 if c % 2 == 0 else -1
        Ls[0]["W"][c, c % 6, c % 3, 1] = sgn
        f0[c] = relu(sgn * _shift2d(xa[c % 6], c % 3 - 1, 0))
    feats.append(f0)
    for l in range(1, depth + 1):
        cat = np.concatenate(feats)
        g = np.zeros((Wd, 4, 4), dtype=np.int64)
        for c in range(Wd):
            sel = (3 * c + 5 * l) % (l * Wd)
            Ls[2 * l - 1]["W"][c, sel, 0, 0] = 2        # times 2 ...
            g[c] = relu(cat[sel])
        Ls[2 * l - 1]["shift"][:] = 31                   # ... then halved: exact copy
        f = np.zeros((Wd, 4, 4), dtype=np.int64)
        for c in range(Wd):
            ky, kx = c % 3, (c // 3) % 3
            Ls[2 * l]["W"][c, (c + 1) % Wd, ky, kx] = 1
            f[c] = relu(_shift2d(g[(c + 1) % Wd], ky - 1, kx - 1))
        feats.append(f)
    cat = np.concatenate(feats)
    want = np.zeros((6, 4, 4), dtype=np.int64)
    for c in range(6):
        sel = (7 * c + 3) % ((depth + 1) * Wd)
        Ls[-1]["W"][c, sel, 2, 0] = -1
        want[c] = -_shift2d(cat[sel], 1, -1)
    m = oracle.Model(pack_blob(model))
    got = m.net_eval(0, xa, 6)
    assert want.any() and np.array_equal(got, np.clip(want, -128, 127))


def test_resnet_family_wiring_doubles_through_shortcut():
    Wd, depth = 6, 3
    cfg = _one_level(RESNET, Wd, depth)
    model = parse_blob(make_blob(cfg, mode="zero"))
    net = model["nets"][0]
    net["M_in"][:] = ONE
    net["s_in"][:] = 30
    Ls = net["layers"]
    for L in Ls:
        _unit(L)
    rng = np.random.default_rng(2)
    xa = rng.integers(-30, 30, (6, 4, 4)).astype(np.int32)
    for c in range(Wd):
        Ls[0]["W"][c, c, 1, 1] = 1                  # r = ReLU(xa)
    r = np.maximum(xa.astype(np.int64), 0)
    for b in range(depth):
        c1, c2 = Ls[1 + 2 * b], Ls[2 + 2 * b]
        for c in range(Wd):
            c1["W"][c, c, 1, 2] = 1                 # branch reads the right-hand neighbour
            c2["W"][c, (c + 1) % Wd, 0, 0] = 1      # and rotates channels
        t1 = np.stack([_shift2d(r[c], 0, 1) for c in range(Wd)])
        r = np.minimum(127, r + np.roll(t1, -1, axis=0))   # ReLU is idle on non-negatives; one saturation
    for c in range(6):
        Ls[-1]["W"][c, c, 1, 1] = -1
    m = oracle.Model(pack_blob(model))
    got = m.net_eval(0, xa, 6)
    assert (r == 127).any() and np.array_equal(got, -r)


def test_plain_family_and_input_quantiser():
    cfg = _one_level(PLAIN, 6, 0)
    model = parse_blob(make_blob(cfg, mode="zero"))
    net = model["nets"][0]
    net["M_in"][:] = 3 << 29          # x 1.5 ...
    net["s_in"][:] = 31               # ... / 2 = 0.75
    Ls = net["layers"]
    for L in Ls:
        _unit(L)
    for c in range(6):
        Ls[0]["W"][c, c, 1, 1] = 1
        Ls[1]["W"][c, c, 1, 1] = 1
    xa = np.arange(-48, 48, dtype=np.int32).reshape(6, 4, 4) * 5
    q = np.array([max(-128, min(127, _half_away(Fraction(3 * int(v), 4)))) for v in xa.reshape(-1)]).reshape(xa.shape)
    m = oracle.Model(pack_blob(model))
    assert np.array_equal(m.net_eval(0, xa, 6), np.maximum(q, 0))


def test_coupling_adds_translation_to_second_half_only():
    # one coupling with an identity permutation: z_a = x_a, z_b = x_b + t(x_a)  (Eq. 1)
    cfg = _one_level(PLAIN, 6, 0)
    model = parse_blob(make_blob(cfg))
    model["nets"][0]["perm"][:] = np.arange(12)
    blob = pack_blob(model)
    m = oracle.Model(blob)
    x = make_images(cfg, batch=1, kind="uniform")
    z, _ = m.forward(x)
    s = _squeeze_np(x[0].astype(np.int64) - 128)
    t = m.net_eval(0, s[:6].astype(np.int32), 6)
    zz = z[0].reshape(12, 4, 4)
    assert np.array_equal(zz[:6], s[:6]) and np.array_equal(zz[6:], s[6:] + t) and t.any()


# ---- gates --------------------------------------------------------------------------

def _delete_gated(model):
    """Remove gated-off filters and the consumers' matching input columns by hand."""
    fam = model["family"]
    for net in model["nets"]:
        Ls = net["layers"]
        keep = [L["gate"].astype(bool) for L in Ls]

        def cut(L, rows, cols):
            L["W"] = L["W"][rows][:, cols]
            for key in ("bias", "M", "shift", "gate"):
                L[key] = L[key][rows]

        allrows = lambda L: np.ones(L["W"].shape[0], dtype=bool)
        allcols = lambda L: np.ones(L["W"].shape[1], dtype=bool)
        if fam == DENSE:
            depth = (len(Ls) - 2) // 2
            feat_keep = [keep[0]] + [keep[2 * l] for l in range(1, depth + 1)]
            cut(Ls[0], keep[0], allcols(Ls[0]))
            for l in range(1, depth + 1):
                cut(Ls[2 * l - 1], keep[2 * l - 1], np.concatenate(feat_keep[:l]))
                cut(Ls[2 * l], keep[2 * l], keep[2 * l - 1])
            cut(Ls[-1], allrows(Ls[-1]), np.concatenate(feat_keep))
        elif fam == RESNET:
            # only the block-internal features can be deleted; the residual stream stays
            # full width, so gated stream producers are replaced by all-zero filters
            for l in range(1, len(Ls) - 1, 2):
                cut(Ls[l], keep[l], allcols(Ls[l]))
                cut(Ls[l + 1], allrows(Ls[l + 1]), keep[l])
            for l in [0] + list(range(2, len(Ls) - 1, 2)):
                dead = ~Ls[l]["gate"].astype(bool)
                Ls[l]["W"] = Ls[l]["W"].copy()
                Ls[l]["W"][dead] = 0
                Ls[l]["bias"] = np.where(dead, 0, Ls[l]["bias"])
                Ls[l]["gate"] = np.ones_like(Ls[l]["gate"])
        else:
            cut(Ls[0], keep[0], allcols(Ls[0]))
            cut(Ls[1], allrows(Ls[1]), keep[0])
    if fam == DENSE or fam == PLAIN:
        model["width"] = int(model["nets"][0]["layers"][0]["W"].shape[0])
    return model


@pytest.mark.parametrize("name", ["mini_dense_g", "odd_dense_g", "mini_resnet_g"])
def test_gate_mask_equals_manual_deletion(name):
    cfg = CONFIGS[name]
    blob = make_blob(cfg)
    model = parse_blob(blob)
    n_gated = sum(int((L["gate"] == 0).sum()) for net in model["nets"] for L in net["layers"])
    assert n_gated > 0
    cut = pack_blob(_delete_gated(parse_blob(blob.copy())))
    assert cut.size < blob.size
    x = make_images(cfg)
    z1, c1 = oracle.Model(blob).forward(x)
    z2, c2 = oracle.Model(cut).forward(x)
    assert np.array_equal(z1, z2) and np.array_equal(c1, c2)
    # and the gates do change the result compared with the ungated network
    model_open = parse_blob(blob.copy())
    for net in model_open["nets"]:
        for L in net["layers"]:
            L["gate"][:] = 1
    z3, _ = oracle.Model(pack_blob(model_open)).forward(x)
    assert not np.array_equal(z1, z3)


def test_gate_keep_fraction_is_exact():
    for name in ("mini_dense_g", "odd_dense_g", "mini_resnet_g", "mini_paper_g"):
        cfg = CONFIGS[name]
        model = parse_blob(make_blob(cfg))
        for net in model["nets"]:
            for L in net["layers"]:
                if L["flags"] & 4:
                    assert int(L["gate"].sum()) == int(round(cfg.keep_at(net["level"]) * L["gate"].size))
                else:
                    assert L["gate"].all()


# ---- batch independence, state bound --------------------------------------------------

@pytest.mark.parametrize("name", ["mini_dense", "mini_resnet_g"])
def test_images_are_independent(name):
    cfg = CONFIGS[name]
    m = oracle.Model(make_blob(cfg))
    x = make_images(cfg, batch=3)
    z, c = m.forward(x)
    for i in range(3):
        zi, ci = m.forward(x[i:i + 1])
        assert np.array_equal(zi[0], z[i]) and np.array_equal(ci[0], c[i])


@pytest.mark.parametrize("name", SMALL)
def test_state_bound(name):
    # each coupling moves an element by at most 128 (one signed 8-bit translation)
    cfg = CONFIGS[name]
    m = oracle.Model(make_blob(cfg))
    m.forward(make_images(cfg, kind="uniform"))
    assert m.last_max_abs_state() <= 128 + 128 * cfg.levels * cfg.couplings


def test_threads_do_not_change_results():
    cfg = CONFIGS["mini_dense"]
    m = oracle.Model(make_blob(cfg))
    x = make_images(cfg)
    try:
        oracle.set_threads(1)
        z1, c1 = m.forward(x)
        oracle.set_threads(3)
        z3, c3 = m.forward(x)
    finally:
        oracle.set_threads(0)
    assert np.array_equal(z1, z3) and np.array_equal(c1, c3)


# ---- malformed blobs --------------------------------------------------------------------

def test_bad_blobs_are_rejected():
    cfg = CONFIGS["cfg1"]
    good = make_blob(cfg)
    oracle.Model(good)
    bad = good.copy(); bad[0] ^= 1
    with pytest.raises(ValueError):
        oracle.Model(bad)
    with pytest.raises(ValueError):
        oracle.Model(good[:-4])
    with pytest.raises(ValueError):
        oracle.Model(np.concatenate([good, np.zeros(4, np.uint8)]))
    m = parse_blob(good.copy()); m["nets"][0]["layers"][0]["shift"][0] = 63
    with pytest.raises(ValueError):
        oracle.Model(pack_blob(m))
    m = parse_blob(good.copy()); m["nets"][0]["perm"][0] = m["nets"][0]["perm"][1]
    with pytest.raises(ValueError):
        oracle.Model(pack_blob(m))
    m = parse_blob(good.copy()); m["nets"][0]["layers"][0]["M"][0] = -5
    with pytest.raises(ValueError):
        oracle.Model(pack_blob(m))


# ---- the closed-form requantisation constants give live networks ---------------------------

@pytest.mark.parametrize("name", ["cfg1", "mini_dense", "mini_dense_g", "mini_resnet", "cfg2"])
def test_generated_constants_give_live_translations(name):
    # (M, shift) come from a variance model, not from a calibration pass; check on seeded inputs
    # that every coupling moves its half by a few grey levels and that saturation stays rare
    cfg = CONFIGS[name]
    blob = make_blob(cfg)
    model = parse_blob(blob)
    m = oracle.Model(blob)
    x = make_images(cfg, batch=min(cfg.batch, 2))
    z, codes = m.forward(x)
    for b in range(x.shape[0]):
        base = _layout_chain(x[b].astype(np.int64) - 128, model)
        moved = z[b] != base
        assert moved.mean() > 0.3
    s = _squeeze_np(x[0].astype(np.int64) - 128)[model["nets"][0]["perm"]]
    t = m.net_eval(0, s[:6].astype(np.int32), 6).astype(np.int64)
    assert 1.5 < t.std() < 12.0 and (np.abs(t) >= 127).mean() < 0.01
    if cfg.heads:
        assert 15.0 < codes.astype(np.int64).std() < 70.0


# ---- unsigned activation format (Eq. 3) --------------------------------------------------

def test_unsigned_conv_matches_a_library_convolution():
    import torch
    rng = np.random.default_rng(11)
    x = rng.integers(0, 256, (5, 6, 7)).astype(np.uint8)        # codes above 127 must count as 128..255
    W = rng.integers(-128, 128, (4, 5, 3, 3)).astype(np.int8)
    b = rng.integers(-1000, 1000, 4).astype(np.int32)
    got = oracle.conv_acc_u8(x, W, b)
    ref = torch.nn.functional.conv2d(torch.from_numpy(x.astype(np.float64))[None], torch.from_numpy(W.astype(np.float64)),
                                     torch.from_numpy(b.astype(np.float64)), padding=1)[0].numpy()
    assert np.array_equal(got, ref.astype(np.int64))
    # and it is not the signed reading of the same bytes
    assert not np.array_equal(got, oracle.conv_acc(x.view(np.int8), W, b))


def test_unsigned_epilogue_by_hand():
    acc = np.array([[[-5, 0, 100, 254, 255, 256, 300, 1000]]], np.int32)
    M, sh = np.array([ONE], np.int32), np.array([30], np.uint8)          # rescale by exactly 1
    assert oracle.epilogue_u8(acc, M, sh).reshape(-1).tolist() == [0, 0, 100, 254, 255, 255, 255, 255]
    sc = np.array([[[200, 200, 200, 200, 0, 7, 255, 0]]], np.uint8)      # shortcut codes are unsigned too
    assert oracle.epilogue_u8(acc, M, sh, shortcut=sc).reshape(-1).tolist() == [195, 200, 255, 255, 255, 255, 255, 255]
    half = np.array([ONE], np.int32), np.array([31], np.uint8)           # x 1/2, half away from zero
    assert oracle.epilogue_u8(np.array([[[509, 510, 511, -1, 3]]], np.int32), *half).reshape(-1).tolist() == [255, 255, 255, 0, 2]


def test_unsigned_resnet_wiring_saturates_at_255():
    # the doubling network of the signed pin: in the unsigned format the stream saturates at 255
    Wd, depth = 6, 4
    cfg = _one_level(RESNET, Wd, depth)
    model = parse_blob(make_blob(cfg, mode="zero"))
    model["act_unsigned"] = 1
    net = model["nets"][0]
    net["M_in"][:] = ONE
    net["s_in"][:] = 30
    Ls = net["layers"]
    for L in Ls:
        _unit(L)
    rng = np.random.default_rng(2)
    xa = rng.integers(-30, 60, (6, 4, 4)).astype(np.int32)
    for c in range(Wd):
        Ls[0]["W"][c, c, 1, 1] = 1
    r = np.maximum(xa.astype(np.int64), 0)
    for b in range(depth):
        c1, c2 = Ls[1 + 2 * b], Ls[2 + 2 * b]
        for c in range(Wd):
            c1["W"][c, c, 1, 2] = 1
            c2["W"][c, (c + 1) % Wd, 0, 0] = 1
        t1 = np.stack([_shift2d(r[c], 0, 1) for c in range(Wd)])
        r = np.minimum(255, r + np.roll(t1, -1, axis=0))
    for c in range(6):
        Ls[-1]["W"][c, c, 1, 1] = -1                  # the translation itself is a signed code
    got = oracle.Model(pack_blob(model)).net_eval(0, xa, 6)
    assert (r == 255).any() and ((r > 127) & (r < 255)).any()
    assert np.array_equal(got, np.maximum(-r, -128))


def test_unsigned_dense_wiring_carries_codes_above_127():
    Wd, depth = 8, 2
    cfg = _one_level(DENSE, Wd, depth)
    model = parse_blob(make_blob(cfg, mode="zero"))
    model["act_unsigned"] = 1
    net = model["nets"][0]
    net["M_in"][:] = ONE
    net["s_in"][:] = 30
    Ls = net["layers"]
    for L in Ls:
        _unit(L)
    rng = np.random.default_rng(5)
    xa = rng.integers(-100, 100, (6, 4, 4)).astype(np.int32)
    relu = lambda a: np.maximum(a, 0)
    feats = []
    f0 = np.zeros((Wd, 4, 4), dtype=np.int64)
    for c in range(Wd):
        Ls[0]["W"][c, c % 6, 1, 1] = 3                      # up to 297: saturates at 255
        f0[c] = np.minimum(255, relu(3 * xa[c % 6]))
    feats.append(f0)
    for l in range(1, depth + 1):
        cat = np.concatenate(feats)
        g = np.zeros((Wd, 4, 4), dtype=np.int64)
        for c in range(Wd):
            sel = (3 * c + 5 * l) % (l * Wd)
            Ls[2 * l - 1]["W"][c, sel, 0, 0] = 1
            g[c] = cat[sel]
        f = np.zeros((Wd, 4, 4), dtype=np.int64)
        for c in range(Wd):
            ky, kx = c % 3, (c // 3) % 3
            Ls[2 * l]["W"][c, (c + 1) % Wd, ky, kx] = 1
            f[c] = _shift2d(g[(c + 1) % Wd], ky - 1, kx - 1)
        feats.append(f)
    cat = np.concatenate(feats)
    want = np.zeros((6, 4, 4), dtype=np.int64)
    for c in range(6):
        sel = (7 * c + 3) % ((depth + 1) * Wd)
        Ls[-1]["W"][c, sel, 2, 0] = 1
        Ls[-1]["shift"][:] = 31                             # halve so that 128..255 survive the signed output
        want[c] = _shift2d(cat[sel], 1, -1)
    got = oracle.Model(pack_blob(model)).net_eval(0, xa, 6)
    assert (cat > 127).any()
    halves = np.array([[_half_away(Fraction(int(v), 2)) for v in row] for row in want.reshape(6, -1)]).reshape(6, 4, 4)
    assert np.array_equal(got, np.minimum(halves, 127))        # 255 / 2 rounds to 128 and saturates


@pytest.mark.parametrize("name", ["mini_dense_u", "mini_resnet_gu", "cfg1_u"])
def test_unsigned_flows_round_trip_and_use_the_extra_bit(name):
    cfg = CONFIGS[name]
    blob = make_blob(cfg)
    assert parse_blob(blob)["act_unsigned"] == 1
    m = oracle.Model(blob)
    x = make_images(cfg, batch=2)
    z, codes = m.forward(x)
    x2, errs = m.inverse(z, x.shape[1:])
    assert errs == 0 and np.array_equal(x, x2)
    # the same bytes read as a signed-format model give another flow: codes above 127 exist and matter
    signed = blob.copy()
    signed[48:52] = 0
    z_s, _ = oracle.Model(signed).forward(x)
    assert not np.array_equal(z, z_s)
