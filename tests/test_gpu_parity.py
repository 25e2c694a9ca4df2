"""GPU parity: libiodf (HIP kernels, through the C ABI) against the CPU oracle,
element by element and bit-exact: all arithmetic is integer, so there is no
tolerance anywhere in this file."""
import numpy as np
import pytest

import paper_2206_08869_amd as iodf
from synth import CONFIGS
from util import blob_of, gpu_flow, images, oracle_model, to_gpu

pytestmark = pytest.mark.gpu


def _check_full(name, batch=None, kinds=("filtered",), modes=("random",)):
    import torch
    cfg = CONFIGS[name]
    b = cfg.batch if batch is None else batch
    for mode in modes:
        om = oracle_model(name, mode)
        flow = gpu_flow(name, max_batch=b, mode=mode)
        for kind in kinds:
            x = images(name, batch=b, kind=kind)
            print("parity", name, "batch", b, "images", kind, "mode", mode, flush=True)
            z_ref, c_ref = om.forward(x)
            xg = to_gpu(x)
            z, codes = flow.forward(xg)
            torch.cuda.synchronize()
            assert np.array_equal(z.cpu().numpy(), z_ref), "z differs"
            if cfg.heads:
                assert np.array_equal(codes.cpu().numpy(), c_ref), "codes differ"
            x_ref, errs = om.inverse(z_ref, x.shape[1:])
            assert errs == 0 and np.array_equal(x_ref, x)
            x2 = flow.inverse(z)
            torch.cuda.synchronize()
            assert np.array_equal(x2.cpu().numpy(), x), "round trip differs"
            assert flow.range_errors() == 0
        flow.close()


@pytest.mark.parametrize("name", ["cfg1", "mini_resnet", "mini_dense", "mini_dense_g", "mini_resnet_g",
                                  "odd_dense_g", "rect_dense", "rect_resnet_g", "mini_paper_g",
                                  "mini_dense_u", "mini_resnet_gu", "cfg1_u", "deep6"])
def test_small_flows_match_oracle(name):
    _check_full(name, kinds=("filtered", "uniform"))


@pytest.mark.parametrize("name", ["cfg1", "mini_dense", "mini_resnet"])
def test_degenerate_networks_match_oracle(name):
    _check_full(name, modes=("zero", "bias_only"))


def test_expanded_and_split_k_last_layers_in_one_model():
    """One model whose networks end differently: 3x3 over 2304 channels (tap-expanded, leaves its raw
    maps in the scratch) and 1x1 over 2304 channels on a few pixels (split over K, needs a zeroed
    scratch). The two must not share the buffer."""
    import oracle
    import torch
    from synth import make_blob, make_images
    from synth.configs import DENSE, FlowConfig
    from synth.model import pack_blob, parse_blob
    cfg = FlowConfig("mix_last", 16, 16, 2, 2, 2, DENSE, 256, 8, False, seed_id=31)
    m = parse_blob(make_blob(cfg).copy())
    for n in (1, 3):   # second coupling of each level: keep the centre tap only
        L = m["nets"][n]["layers"][-1]
        L["W"] = np.ascontiguousarray(L["W"][:, :, 1:2, 1:2])
    blob = pack_blob(m)
    x = make_images(cfg)
    om = oracle.Model(blob)
    z_ref, _ = om.forward(x)
    flow = iodf.Flow(blob, max_batch=cfg.batch, device=0)
    for _rep in range(2):   # the second pass starts from whatever the first left in the scratch
        z, _ = flow.forward(to_gpu(x))
        torch.cuda.synchronize()
        assert np.array_equal(z.cpu().numpy(), z_ref)
        x2 = flow.inverse(z)
        torch.cuda.synchronize()
        assert np.array_equal(x2.cpu().numpy(), x)
    flow.close()


def test_mid_dense_matches_oracle():
    _check_full("mid_dense", batch=5)   # 5*256 pixels at level 1: ragged against every pixel tile


def test_cfg2_full_batch_matches_oracle():
    _check_full("cfg2")


def test_cfg2_gated_residual_matches_oracle():
    _check_full("cfg2g")


def test_extreme_images_and_arbitrary_latents():
    import torch
    name = "mini_dense"
    cfg = CONFIGS[name]
    om = oracle_model(name)
    flow = gpu_flow(name, max_batch=4)
    x = np.stack([np.zeros((3, cfg.H, cfg.W), np.uint8), np.full((3, cfg.H, cfg.W), 255, np.uint8)])
    z_ref, c_ref = om.forward(x)
    z, c = flow.forward(to_gpu(x))
    assert np.array_equal(z.cpu().numpy(), z_ref) and np.array_equal(c.cpu().numpy(), c_ref)
    # decode of latents that are no image: same pixels, same count of range errors
    rng = np.random.default_rng(5)
    zz = rng.integers(-300, 300, (3, cfg.d)).astype(np.int32)
    x_ref, errs = om.inverse(zz, (3, cfg.H, cfg.W))
    xg = flow.inverse(to_gpu(zz))
    torch.cuda.synchronize()
    assert errs > 0 and flow.range_errors() == errs
    assert np.array_equal(xg.cpu().numpy(), x_ref)
    assert flow.range_errors() == 0   # the query resets the counter
    flow.close()


def test_batch_edges_and_invariance():
    import torch
    import paper_2206_08869_amd as iodf
    name = "mini_dense_g"
    cfg = CONFIGS[name]
    flow = gpu_flow(name, max_batch=7)
    x = images(name, batch=7)
    xg = to_gpu(x)
    z7, c7 = flow.forward(xg)
    z7, c7 = z7.clone(), c7.clone()
    # image i alone == image i inside the batch; two runs are identical
    for i in (0, 3, 6):
        zi, ci = flow.forward(xg[i:i + 1].contiguous())
        assert torch.equal(zi[0], z7[i]) and torch.equal(ci[0], c7[i])
    z7b, c7b = flow.forward(xg)
    assert torch.equal(z7, z7b) and torch.equal(c7, c7b)
    # codes are optional
    z_nc, none = flow.forward(xg, want_codes=False)
    assert none is None and torch.equal(z_nc, z7)
    # batch 0 is a no-op, batch > max_batch is refused
    z0, c0 = flow.forward(xg[:0].contiguous())
    assert z0.shape[0] == 0
    with pytest.raises(iodf.IodfError) as ei:
        flow.forward(to_gpu(images(name, batch=8)))
    assert ei.value.code == -4
    assert flow.query(iodf.IODF_Q_MAX_BATCH) == 7
    flow.close()


def test_query_reports_algorithmic_macs():
    import paper_2206_08869_amd as iodf
    from synth import macs_per_image
    for name in ("cfg1", "mini_dense", "mini_dense_g", "odd_dense_g", "cfg2"):
        cfg = CONFIGS[name]
        flow = gpu_flow(name, max_batch=1)
        assert flow.query(iodf.IODF_Q_MACS_FORWARD) == macs_per_image(cfg)
        assert flow.query(iodf.IODF_Q_MACS_INVERSE) == macs_per_image(cfg, with_heads=False)
        assert flow.query(iodf.IODF_Q_Z_ELEMS) == cfg.d and flow.query(iodf.IODF_Q_CODE_BYTES) == cfg.d_codes
        flow.close()


def test_graph_replay_equals_eager_launches(monkeypatch):
    # Calls are replayed from a captured HIP graph. Replay each shape several times, with eager
    # work and synchronisations in between, and compare every replay with the eager path.
    import torch
    name = "mini_dense_g"
    cfg = CONFIGS[name]
    monkeypatch.setenv("IODF_NO_GRAPH", "1")
    eager = gpu_flow(name, max_batch=5)
    monkeypatch.delenv("IODF_NO_GRAPH")
    graph = gpu_flow(name, max_batch=5)
    om = oracle_model(name)
    x = images(name, batch=5)
    xg = to_gpu(x)
    z_ref, c_ref = om.forward(x)
    for rep in range(4):
        for b in (5, 2, 1, 5, 3):
            xb = xg[:b].contiguous()
            ze, ce = eager.forward(xb)
            junk = torch.randn(1 << 16, device="cuda").sum()   # unrelated eager work between replays
            zg, cg = graph.forward(xb)
            torch.cuda.synchronize()
            assert torch.equal(ze, zg) and torch.equal(ce, cg), (rep, b)
            assert np.array_equal(zg.cpu().numpy(), z_ref[:b]) and np.array_equal(cg.cpu().numpy(), c_ref[:b])
            xr = graph.inverse(zg)
            zn, none = graph.forward(xb, want_codes=False)
            torch.cuda.synchronize()
            assert torch.equal(xr, xb) and torch.equal(zn, zg) and none is None
            assert float(junk) == float(junk)
    assert graph.range_errors() == 0
    # more shapes than the cache holds: old graphs are dropped and recaptured on demand
    big = gpu_flow(name, max_batch=12)
    xs = to_gpu(images(name, batch=12))
    outs = {}
    for b in list(range(1, 13)) + [1, 2, 12]:
        z, c = big.forward(xs[:b].contiguous())
        torch.cuda.synchronize()
        if b in outs:
            assert torch.equal(outs[b], z)
        outs[b] = z.clone()
        assert torch.equal(z, outs[12][:b]) if 12 in outs else True
    eager.close(); graph.close(); big.close()


def test_contexts_release_their_device_memory():
    import torch
    name = "mini_dense"
    x = to_gpu(images(name, batch=2))
    ref = None

    def cycle(n):
        nonlocal ref
        for _ in range(n):
            flow = gpu_flow(name, max_batch=2)
            z, _ = flow.forward(x)
            w, _ = flow.encode(x)
            assert torch.equal(flow.decode(w), x) and torch.equal(flow.inverse(z), x)
            ref = z.clone() if ref is None else ref
            assert torch.equal(ref, z)
            flow.close()
        torch.cuda.synchronize()
        torch.cuda.empty_cache()
        return torch.cuda.mem_get_info()[0]

    a = cycle(3)
    b = cycle(12)
    assert a - b < (1 << 20), "device memory shrank by %d bytes over 12 contexts" % (a - b)


@pytest.mark.parametrize("c_in,c_out,k,relu,shift_lo", [
    (128, 128, 3, True, 36), (64, 256, 3, True, 36), (32, 512, 3, True, 36),   # the shapes of Table 1
    (40, 72, 1, False, 36), (7, 5, 3, False, 20), (130, 64, 3, True, 20),       # ragged widths, short shifts, no ReLU
])
def test_single_convolution_matches_oracle(c_in, c_out, k, relu, shift_lo):
    _check_single_convolution(c_in, c_out, k, relu, shift_lo, 3, 16, 16)


@pytest.mark.parametrize("c_in,c_out,k,b,side", [
    (512, 512, 1, 80, 32),    # 640 tiles of 256x256 and 8 k-tiles: the 256x128 half tile, two workgroups per CU
    (128, 128, 3, 160, 32),   # 320 tiles of 128x512 and 18 k-tiles: the 128x256 half tile
    (1024, 512, 1, 72, 32),   # 576 tiles, 16 k-tiles: the last reduction length that takes the half tile
    (1088, 512, 1, 72, 32),   # 17 k-tiles: back on the 256x256 tile
    (2048, 512, 1, 96, 32),   # 32 k-tiles, 768 tiles: the persistent form of the 256x256 tile
    (256, 512, 3, 97, 32),    # 3x3, 36 k-tiles, 776 tiles: persistent, workgroups with three and with four tiles
    (1280, 256, 1, 219, 30),  # persistent, one channel block, 197100 pixels (ragged), sides that are no powers of two
    (1280, 256, 1, 92, 30),   # the same layer on 324 tiles (1.3 per CU): workgroups with one and with two tiles
    (512, 512, 1, 92, 30),    # 82800 pixels: a ragged last half tile, image sides that are no powers of two
    (128, 128, 3, 183, 30),   # 164700 pixels, ragged, 3x3
])
def test_single_convolution_on_many_pixels_matches_oracle(c_in, c_out, k, b, side):
    _check_single_convolution(c_in, c_out, k, True, 36, b, side, side)


@pytest.mark.parametrize("c_in,c_out,k,relu,b,side", [
    (256, 256, 3, True, 1, 32),     # 64 tiles of 64x64, 36 k-tiles
    (2304, 256, 1, True, 1, 8),     # 4 tiles, 36 k-tiles
    (1920, 256, 1, False, 3, 4),    # 30 k-tiles, 48 pixels (ragged tile), no ReLU
    (512, 512, 3, True, 2, 4),      # 72 k-tiles, 32 pixels: half a pixel tile
])
def test_single_convolution_on_few_pixels_matches_oracle(c_in, c_out, k, relu, b, side):
    """Hidden layers as a batch-1 call sees them: a handful of small tiles, long reductions."""
    _check_single_convolution(c_in, c_out, k, relu, 36, b, side, side)


@pytest.mark.parametrize("c_in,c_out,k,relu,b,h,w,tiles", [
    (64, 64, 1, True, 1, 4, 4, 1),          # one k-tile: every load past it repeats it
    (640, 64, 1, True, 3, 5, 7, 2),         # ten k-tiles (one round and one step), 105 pixels: a ragged second tile
    (64, 128, 3, False, 2, 6, 6, 4),        # nine k-tiles (one round), shortcut-free no-ReLU epilogue
    (192, 256, 3, True, 16, 8, 8, 64),      # 27 k-tiles, 64 tiles of 64x64
    (128, 512, 3, True, 131, 7, 9, 260),    # 128x128 tile: 65 pixel blocks (the last one ragged) x 4 channel blocks
    (640, 512, 1, True, 128, 8, 8, 256),    # 128x128 tile, ten k-tiles
    (64, 512, 1, False, 128, 8, 8, 256),    # 128x128 tile, one k-tile
])
def test_single_convolution_on_the_small_tile_kernel_matches_oracle(c_in, c_out, k, relu, b, h, w, tiles):
    """Reduction lengths around the nine-step round of the small-tile kernel (1, 9, 10, 27 k-tiles), ragged pixel
    tiles, both of its tile sizes; the timeline's row count (output tiles that ran = pixel blocks x channel blocks)
    tells that the intended tiling ran."""
    _check_single_convolution(c_in, c_out, k, relu, 36, b, h, w)
    rng = np.random.default_rng(3)
    x = rng.integers(0, 128, (b, c_in, h, w)).astype(np.int8)
    W = rng.integers(-128, 128, (c_out, c_in, k, k)).astype(np.int8)
    bias = np.zeros(c_out, np.int32)
    M = np.full(c_out, 1 << 30, np.int32)
    shift = np.full(c_out, 40, np.uint8)
    _, _, tl = iodf.iodf_conv_probe_timeline(x, W, bias, M, shift, relu=relu, iters=1)
    assert tl.shape[0] == tiles


def _check_single_convolution(c_in, c_out, k, relu, shift_lo, b, h, w):
    import oracle
    rng = np.random.default_rng(c_in * 1000 + c_out)
    x = rng.integers(-128, 128, (b, c_in, h, w)).astype(np.int8)
    if relu:
        x = np.maximum(x, 0).astype(np.int8)
    W = rng.integers(-128, 128, (c_out, c_in, k, k)).astype(np.int8)
    bias = rng.integers(-5000, 5000, c_out).astype(np.int32)
    M = rng.integers(1 << 30, (1 << 31) - 1, c_out).astype(np.int32)
    shift = rng.integers(shift_lo, shift_lo + 6, c_out).astype(np.uint8)
    y, us = iodf.iodf_conv_probe(x, W, bias, M, shift, relu=relu, iters=3)
    for i in range(b):
        ref = oracle.epilogue(oracle.conv_acc(x[i], W, bias), M, shift, relu=relu)
        assert np.array_equal(y[i], ref), "image %d" % i
    assert us > 0


def _edge_accumulators(M, shift, top):
    """Per channel, the smallest accumulator a >= 0 whose requantised value round_half_away(a * M / 2^shift)
    reaches `top`: a * M >= (top - 1/2) * 2^shift (exact integer arithmetic)."""
    out = []
    for m, s in zip(M.tolist(), shift.tolist()):
        need = (2 * top - 1) << (s - 1)
        out.append(-(-need // m))
    return np.array(out, dtype=np.int64)


@pytest.mark.parametrize("relu,edge", [(True, "top"), (True, "zero"), (False, "top"), (False, "bottom"), (False, "zero")])
@pytest.mark.parametrize("b,side,c_in", [(2, 16, 64), (136, 32, 256)])
def test_epilogue_at_the_saturation_edges(relu, edge, b, side, c_in):
    """Accumulators placed, for every output channel, exactly around the points where the epilogue's
    result changes regime: the smallest accumulator that requantises to 127 (the fast ReLU epilogue clamps
    the accumulator there BEFORE it rescales), its counterpart at -128 for layers without ReLU, and zero.
    A 1x1 layer whose only non-zero weights are +1 and -1 on two input channels adds delta in -3..3 to a
    per-channel bias, so pixel p of channel c sees bias[c] + delta(p). Small case: the plain kernel; large
    case (139264 pixels, 4 k-tiles): the persistent kernel."""
    import oracle
    c_out = 256
    rng = np.random.default_rng(77 + b)
    M = rng.integers(1 << 30, (1 << 31) - 1, c_out).astype(np.int32)
    shift = rng.integers(33, 47, c_out).astype(np.uint8)
    if edge == "top":
        bias = _edge_accumulators(M, shift, 127)
    elif edge == "bottom":
        bias = -_edge_accumulators(M, shift, 128)
    else:
        bias = np.zeros(c_out, np.int64)
    assert np.abs(bias).max() < (1 << 30)
    bias = bias.astype(np.int32)
    W = np.zeros((c_out, c_in, 1, 1), np.int8)
    W[:, 0] = 1
    W[:, 1] = -1
    x = rng.integers(0, 128, (b, c_in, side, side)).astype(np.int8)   # other channels: arbitrary, zero weights
    delta = (np.arange(b * side * side) % 7 - 3).reshape(b, side, side)
    x[:, 0] = np.maximum(delta, 0)
    x[:, 1] = np.maximum(-delta, 0)
    y, _ = iodf.iodf_conv_probe(x, W, bias, M, shift, relu=relu, iters=1)
    seen = set()
    for i in range(b):
        ref = oracle.epilogue(oracle.conv_acc(x[i], W, bias), M, shift, relu=relu)
        assert np.array_equal(y[i], ref), "image %d" % i
        seen.update(np.unique(ref).tolist())
    # the cases straddle the edge they aim at
    if edge == "top":
        assert 127 in seen and 126 in seen
    elif edge == "bottom":
        assert -128 in seen and -127 in seen
    else:
        assert 0 in seen


@pytest.mark.parametrize("c_in,k,b,side,tiles", [(64, 3, 2, 16, 32), (256, 1, 136, 32, 544)])
def test_conv_probe_timeline(c_in, k, b, side, tiles):
    """The per-tile timeline is measurement support: it must not change the layer's result, report one
    row per output tile that ran, and its stamps must be ordered (start <= first operands <= k loop done
    <= epilogue done) with a plausible shader clock. Small case: plain kernel (64x64 tiles); large case: the
    persistent kernel (256x256 tiles, 544 of them on one workgroup per CU)."""
    c_out = 256
    rng = np.random.default_rng(5 + c_in)
    x = np.maximum(rng.integers(-128, 128, (b, c_in, side, side)), 0).astype(np.int8)
    W = rng.integers(-127, 128, (c_out, c_in, k, k)).astype(np.int8)
    bias = rng.integers(-3000, 3000, c_out).astype(np.int32)
    M = rng.integers(1 << 30, (1 << 31) - 1, c_out).astype(np.int32)
    shift = rng.integers(38, 42, c_out).astype(np.uint8)
    y0, _ = iodf.iodf_conv_probe(x, W, bias, M, shift, relu=True, iters=1)
    y1, us, tl = iodf.iodf_conv_probe_timeline(x, W, bias, M, shift, relu=True, iters=2)
    assert np.array_equal(y0, y1) and us > 0
    assert tl.shape == (tiles, 8)
    assert (tl[:, 0] <= tl[:, 1]).all() and (tl[:, 1] <= tl[:, 2]).all() and (tl[:, 2] <= tl[:, 3]).all()
    wall = (tl[:, 3] - tl[:, 0]).astype(np.float64)          # 10 ns ticks
    ghz = (tl[:, 5] - tl[:, 4]) / np.maximum(wall, 1) * 0.1
    assert (wall > 0).all() and 0.3 < np.median(ghz) < 3.0
