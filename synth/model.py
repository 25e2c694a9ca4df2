"""Seeded model blobs: weights, requantisation constants, permutations and gates.

Blob layout (little-endian, every field and array padded to 4 bytes):

  header, 16 x u32: 'IODF', 'BLB1', version=1, H, W, levels, couplings, family,
                    width, depth, has_heads, n_nets, 0, 0, 0, 0
  per network, in flow order (level 1 couplings, level 1 head, level 2 ...):
    8 x 32 bit: kind (0 coupling, 1 head), level, C_level, C_in, C_out, n_layers,
                M_in (i32), s_in
    i32 perm[C_level]                       (couplings only)
    per conv layer:
      4 x u32: C_out, C_in, k, flags (bit0 ReLU, bit1 shortcut, bit2 gated)
      i8  W[C_out][C_in][k][k], i32 bias[C_out], i32 M[C_out],
      u8  shift[C_out], u8 gate[C_out]      (gate 1 = filter kept)

Weights are drawn N(0, 1/fan_in) and quantised symmetrically per output channel:
s_c = max|W_c| / 127, code = clip(round_half_away(W / s_c), -127, 127).

The requantisation constants (M, shift) are chosen without evaluating the
network, from a variance model of the accumulator: the inputs of a layer are
taken as independent with known per-channel mean and variance (post-ReLU codes of
a Gaussian whose 99.9th percentile sits at 127), which gives each output channel
an accumulator mean (cancelled by the bias) and a standard deviation sigma_c; the
multiplier maps 3.29 sigma_c (the 99.9th percentile) to 127 for hidden layers and
prior-parameter codes and to 16 for the translation, so saturation does fire but
rarely. (M, shift) is the normalised pair with M in [2^30, 2^31) closest to that
real scale. Any choice yields a valid flow; the blob fixes one.
"""
from concurrent.futures import ThreadPoolExecutor
import os

import numpy as np

from . import prng
from .configs import net_layers, flow_networks, PLAIN, RESNET, DENSE

BLOB_MAGIC = (0x46444F49, 0x31424C42)   # 'IODF', 'BLB1'
_P999 = 3.29
_SIGMA_Q = 127.0 / _P999                 # std of a code whose 99.9th percentile is 127
_RELU_MEAN = 0.3989422804014327          # E[max(0, g)] for g ~ N(0, 1)
_RELU_VAR = 0.5 - _RELU_MEAN ** 2        # Var[max(0, g)]


def _pad4(n):
    return (n + 3) & ~3


def layer_bytes(co, ci, k):
    return 16 + _pad4(co * ci * k * k) + 4 * co + 4 * co + _pad4(co) + _pad4(co)


def net_bytes(kind, c_level, layers):
    n = 32 + (4 * c_level if kind == 0 else 0)
    for (co, ci, k, *_r) in layers:
        n += layer_bytes(co, ci, k)
    return n


def normalise_scale(scale):
    """(M, shift) with M in [2^30, 2^31) and M / 2^shift closest to `scale` (arrays)."""
    scale = np.asarray(scale, dtype=np.float64)
    e = np.floor(np.log2(scale))
    s = 30 - e
    m = np.rint(scale * np.exp2(s))
    over = m >= 2.0 ** 31
    m = np.where(over, m / 2, m)
    s = np.where(over, s - 1, s)
    s = np.clip(s, 0, 62)
    m = np.clip(m, 1, 2.0 ** 31 - 1)
    return m.astype(np.int64).astype(np.int32), s.astype(np.uint8)


def _rha(a):
    return np.sign(a) * np.floor(np.abs(a) + 0.5)


def _gen_network(cfg, seed, idx, kind, level, c_level, c_in, c_out, n_prev, mode, out):
    """Write network `idx` into the byte buffer `out` (its own slice of the blob)."""
    layers = net_layers(cfg.family, c_in, c_out, cfg.width, cfg.depth, cfg.block_k2)
    pos = 0

    def put(arr):
        nonlocal pos
        b = np.ascontiguousarray(arr).view(np.uint8).reshape(-1)
        out[pos:pos + b.size] = b
        pos += _pad4(b.size)

    # input quantiser of this network: 99.9th percentile of |x_a| -> 127
    sigma_img = 74.0 if cfg.image_kind == "uniform" else 50.0
    p_in = 128.0 + 8.0 * np.sqrt(float(n_prev))
    gain = 127.0 / p_in
    m_in, s_in = normalise_scale(np.array([gain]))
    sigma_state = np.sqrt(sigma_img ** 2 + 12.0 * n_prev)
    put(np.array([kind, level, c_level, c_in, c_out, len(layers)], dtype=np.uint32))
    put(np.array([m_in[0]], dtype=np.int32))
    put(np.array([s_in[0]], dtype=np.uint32))
    if kind == 0:
        put(prng.shuffle(prng.substream(seed, idx, 1), c_level).astype(np.int32))

    # per-channel (mean, variance) model of each feature tensor, for the scales
    in_mean = np.zeros(c_in)
    in_var = np.full(c_in, (gain * sigma_state) ** 2)
    feat_mean, feat_var = [], []          # dense family: statistics of f0..f_l, concatenated
    stream_mean = stream_var = None       # resnet family: statistics of the residual stream
    for li, (co, ci, k, relu, shortcut, gated) in enumerate(layers):
        last = li == len(layers) - 1
        if li > 0:
            if cfg.family == DENSE:
                if k == 1 or last:
                    in_mean, in_var = np.concatenate(feat_mean), np.concatenate(feat_var)
                else:
                    in_mean, in_var = prev_mean, prev_var
            elif cfg.family == RESNET:
                if shortcut:
                    in_mean, in_var = prev_mean, prev_var
                else:
                    in_mean, in_var = stream_mean, stream_var
            else:
                in_mean, in_var = prev_mean, prev_var
        fan_in = ci * k * k
        lseed = prng.substream(seed, idx, 2, li)
        if mode == "random":
            w = prng.normal(prng.substream(lseed, 0), co * fan_in).reshape(co, fan_in)
            w *= 1.0 / np.sqrt(fan_in)
            sc = np.abs(w).max(axis=1, keepdims=True) / 127.0
            wq = np.clip(_rha(w / sc), -127, 127).astype(np.int8)
            del w
        else:
            wq = np.zeros((co, fan_in), dtype=np.int8)
        # gates: exactly round(keep * C_out) filters survive in a gated layer
        gate = np.ones(co, dtype=np.uint8)
        if gated and cfg.keep_at(level) < 1.0:
            n_keep = max(1, int(round(cfg.keep_at(level) * co)))
            order = prng.shuffle(prng.substream(lseed, 1), co)
            gate[:] = 0
            gate[order[:n_keep]] = 1
        # accumulator model
        w3 = wq.reshape(co, ci, k * k).astype(np.float64)
        acc_mean = (w3.sum(axis=2) * in_mean[None, :]).sum(axis=1)
        acc_std = np.sqrt(((w3 ** 2).sum(axis=2) * in_var[None, :]).sum(axis=1))
        del w3
        acc_std = np.maximum(acc_std, 1.0)
        noise = prng.normal(prng.substream(lseed, 2), co)
        if mode == "random":
            bias = np.rint(-acc_mean + 0.3 * acc_std * noise)
        elif mode == "bias_only":
            bias = np.rint(4000.0 * noise)
            acc_std = np.full(co, 4000.0)
        else:
            bias = np.zeros(co)
        bias = np.clip(bias, -(2 ** 30) + 1, 2 ** 30 - 1).astype(np.int32)
        # unsigned post-ReLU codes have one more bit of range
        top = 255.0 if (cfg.act_unsigned and relu) else 127.0
        if last:
            target = 16.0 if kind == 0 else 127.0
        elif shortcut:
            target = (top + 1.0) / 2.0
        else:
            target = top
        if mode == "zero":
            scale = np.ones(co)
        else:
            scale = target / (_P999 * 1.05 * acc_std)
        m, s = normalise_scale(scale)
        flags = (1 if relu else 0) | (2 if shortcut else 0) | (4 if gated else 0)
        put(np.array([co, ci, k, flags], dtype=np.uint32))
        put(wq)
        put(bias)
        put(m)
        put(s)
        put(gate)
        # statistics of this layer's output codes
        sq = target / _P999
        g = gate.astype(np.float64)
        if relu:
            o_mean, o_var = g * _RELU_MEAN * sq, g * _RELU_VAR * sq * sq
        else:
            o_mean, o_var = np.zeros(co), g * sq * sq
        if cfg.family == RESNET and shortcut:
            stream_mean = stream_mean + 0.25 * o_mean
            stream_var = stream_var + 0.5 * o_var
            o_mean, o_var = stream_mean, stream_var
        elif cfg.family == RESNET and li == 0:
            stream_mean, stream_var = o_mean, o_var
        if cfg.family == DENSE and (li == 0 or (k == 3 and not last)):
            feat_mean.append(o_mean)
            feat_var.append(o_var)
        prev_mean, prev_var = o_mean, o_var
    assert pos == out.size, (pos, out.size)


def make_blob(cfg, seed=None, mode="random", threads=None):
    """The model blob of `cfg` as a uint8 array.

    mode "random": seeded weights; "zero": all weights and biases 0 (t == 0);
    "bias_only": weights 0, random biases (t is a per-channel constant).
    """
    seed = (2000 + cfg.seed_id) if seed is None else seed
    nets = flow_networks(cfg)
    sizes = [net_bytes(kind, c, net_layers(cfg.family, ci, co, cfg.width, cfg.depth, cfg.block_k2))
             for (kind, lv, c, ci, co) in nets]
    offs = np.concatenate([[64], 64 + np.cumsum(sizes)]).astype(np.int64)
    blob = np.zeros(int(offs[-1]), dtype=np.uint8)
    hdr = np.array([BLOB_MAGIC[0], BLOB_MAGIC[1], 1, cfg.H, cfg.W, cfg.levels, cfg.couplings,
                    cfg.family, cfg.width, cfg.depth, 1 if cfg.heads else 0, len(nets),
                    1 if cfg.act_unsigned else 0, 0, 0, 0], dtype=np.uint32)
    blob[:64] = hdr.view(np.uint8)
    jobs = []
    n_prev = 0
    for i, (kind, lv, c, ci, co) in enumerate(nets):
        jobs.append((cfg, seed, i, kind, lv, c, ci, co, n_prev, mode, blob[offs[i]:offs[i + 1]]))
        if kind == 0:
            n_prev += 1
    nthreads = threads or min(16, os.cpu_count() or 1, len(jobs))
    if nthreads <= 1 or len(jobs) == 1:
        for j in jobs:
            _gen_network(*j)
    else:
        with ThreadPoolExecutor(nthreads) as ex:
            for f in [ex.submit(_gen_network, *j) for j in jobs]:
                f.result()
    return blob


def parse_blob(blob):
    """Decode a blob into a dict of numpy views (header fields + list of networks).

    Views alias `blob`: editing a weight array in place edits the blob.
    """
    blob = np.asarray(blob, dtype=np.uint8)
    h = blob[:64].view(np.uint32)
    if (int(h[0]), int(h[1])) != BLOB_MAGIC or int(h[2]) != 1:
        raise ValueError("not an IODF model blob")
    model = dict(H=int(h[3]), W=int(h[4]), levels=int(h[5]), couplings=int(h[6]), family=int(h[7]),
                 width=int(h[8]), depth=int(h[9]), has_heads=int(h[10]), act_unsigned=int(h[12]) & 1, nets=[])
    pos = 64

    def take(nbytes, dtype):
        nonlocal pos
        a = blob[pos:pos + nbytes].view(dtype)
        pos += _pad4(nbytes)
        return a

    for _ in range(int(h[11])):
        f = take(24, np.uint32)
        kind, level, c_level, c_in, c_out, n_layers = (int(v) for v in f)
        m_in = take(4, np.int32)
        s_in = take(4, np.uint32)
        net = dict(kind=kind, level=level, C=c_level, C_in=c_in, C_out=c_out, M_in=m_in, s_in=s_in,
                   perm=take(4 * c_level, np.int32) if kind == 0 else None, layers=[])
        for _l in range(n_layers):
            co, ci, k, flags = (int(v) for v in take(16, np.uint32))
            net["layers"].append(dict(
                C_out=co, C_in=ci, k=k, flags=flags,
                W=take(co * ci * k * k, np.int8).reshape(co, ci, k, k),
                bias=take(4 * co, np.int32), M=take(4 * co, np.int32),
                shift=take(co, np.uint8), gate=take(co, np.uint8)))
        model["nets"].append(net)
    if pos != blob.size:
        raise ValueError("trailing bytes in blob")
    return model


def pack_blob(model):
    """Inverse of parse_blob: serialise a (possibly edited) model dict to a blob.

    Layer arrays may have been replaced by arrays of other shapes (for instance
    after deleting filters); C_out / C_in / k are taken from W's shape.
    """
    parts = []

    def put(arr, dtype):
        b = np.ascontiguousarray(np.asarray(arr).astype(dtype, copy=False)).view(np.uint8).reshape(-1)
        parts.append(b)
        if b.size % 4:
            parts.append(np.zeros(4 - b.size % 4, dtype=np.uint8))

    nets = model["nets"]
    put([BLOB_MAGIC[0], BLOB_MAGIC[1], 1, model["H"], model["W"], model["levels"], model["couplings"],
         model["family"], model["width"], model["depth"], model["has_heads"], len(nets),
         model.get("act_unsigned", 0), 0, 0, 0],
        np.uint32)
    for net in nets:
        put([net["kind"], net["level"], net["C"], net["C_in"], net["C_out"], len(net["layers"])], np.uint32)
        put(np.asarray(net["M_in"]).reshape(-1)[:1], np.int32)
        put(np.asarray(net["s_in"]).reshape(-1)[:1], np.uint32)
        if net["kind"] == 0:
            put(net["perm"], np.int32)
        for L in net["layers"]:
            W = np.asarray(L["W"])
            co, ci, k, _k = W.shape
            put([co, ci, k, L["flags"]], np.uint32)
            put(W, np.int8)
            put(L["bias"], np.int32)
            put(L["M"], np.int32)
            put(L["shift"], np.uint8)
            put(L["gate"], np.uint8)
    return np.concatenate(parts)
