"""GPU parity at the benchmark's full sizes, in the launch configuration bench.py
times. The oracle cannot run whole batches of the width-512 flows in reasonable
time, so a few images of each batch are recomputed by the oracle one by one and
compared bit-exactly; the rest of the batch is covered by properties that hold at
any size: exact round trip, and every image's result being the same when the batch
is cut into ragged chunks (other tile positions, other tile tails) or run alone.

IODF_FULL_PARITY=1 in the environment makes the oracle recompute EVERY image of each
batch instead of the sample (cfg4: about ten minutes of host time).
IODF_FULL_PARITY_ONLY=cfg4 restricts that to one configuration. IODF_PARITY_128=1 checks the
first 64 images and 64 seeded ones of a batch (for batches too large to recompute whole)."""
import os

import numpy as np
import pytest

from synth import CONFIGS
from util import gpu_flow, images, oracle_model, to_gpu

pytestmark = pytest.mark.gpu


def _sampled(capsys, name, batch, sample, invariance=(), chunk=None):
    import torch
    full = os.environ.get("IODF_FULL_PARITY") == "1" and os.environ.get("IODF_FULL_PARITY_ONLY", name) == name
    if full:
        sample = tuple(range(batch))
    elif os.environ.get("IODF_PARITY_128") == "1" and batch > 128 and \
            os.environ.get("IODF_FULL_PARITY_ONLY", name) == name:
        rng = np.random.default_rng(2206)
        sample = tuple(range(64)) + tuple(sorted(int(i) for i in rng.choice(np.arange(64, batch), 64, replace=False)))

    def say(*a):
        with capsys.disabled():   # progress lines must reach the terminal while the test runs
            print("[full-size]", *a, flush=True)

    say(name, "batch", batch, "oracle images", sample)
    flow = gpu_flow(name, max_batch=batch)
    x = images(name, batch=batch)
    xg = to_gpu(x)
    z, codes = flow.forward(xg)
    torch.cuda.synchronize()
    say("gpu forward done")
    x2 = flow.inverse(z)
    torch.cuda.synchronize()
    assert torch.equal(x2, xg), "round trip"
    assert flow.range_errors() == 0
    for i in invariance:
        zi, ci = flow.forward(xg[i:i + 1].contiguous())
        assert torch.equal(zi[0], z[i]) and torch.equal(ci[0], codes[i]), "batch invariance"
    if chunk:
        # the whole batch again in ragged chunks: every image lands in other tiles
        for lo in range(0, batch, chunk):
            hi = min(batch, lo + chunk)
            zi, ci = flow.forward(xg[lo:hi].contiguous())
            assert torch.equal(zi, z[lo:hi]) and torch.equal(ci, codes[lo:hi]), "chunk %d..%d" % (lo, hi)
            xi = flow.inverse(zi)
            assert torch.equal(xi, xg[lo:hi]), "chunked round trip %d..%d" % (lo, hi)
        say("ragged chunks of", chunk, "match")
    zc, cc = z.cpu().numpy(), codes.cpu().numpy()
    flow.close()
    om = oracle_model(name)
    for i in sample:
        z_ref, c_ref = om.forward(x[i:i + 1])
        say("oracle image", i, "done")
        assert np.array_equal(zc[i], z_ref[0]), "z differs from oracle at image %d" % i
        assert np.array_equal(cc[i], c_ref[0]), "codes differ from oracle at image %d" % i


def _spread(batch, n, seed):
    """n image indices of a batch: the first four and the last two (the first and the last tiles of every
    level, whose pixel tiles hold one to sixteen images), two pairs of neighbours around the middle (images
    that share a tile at the deep levels), and seeded others."""
    fixed = [0, 1, 2, 3, batch // 2 - 1, batch // 2, batch // 2 + 3, batch // 2 + 4, batch - 2, batch - 1]
    rng = np.random.default_rng(seed)
    rest = [int(i) for i in rng.permutation(batch) if int(i) not in fixed]
    return tuple(sorted(fixed + rest[:max(0, n - len(fixed))]))


@pytest.mark.timeout(900)
def test_cfg3_sampled(capsys):
    _sampled(capsys, "cfg3", CONFIGS["cfg3"].batch, sample=_spread(256, 32, 3), invariance=(7,), chunk=53)


@pytest.mark.timeout(900)
def test_cfg4_sampled(capsys):
    _sampled(capsys, "cfg4", CONFIGS["cfg4"].batch, sample=_spread(128, 24, 4), invariance=(64,), chunk=37)


@pytest.mark.timeout(600)
def test_paper_network_pruned_sampled(capsys):
    # the paper's own coupling network (8 residual blocks of 3x3 convolutions at 128 channels), pruned
    # hardest at the deepest level; compacted widths 96 / 80 / 48 / 32 are padded to 64-channel planes
    _sampled(capsys, "paper_iodf64", CONFIGS["paper_iodf64"].batch, sample=(0, 101, 255), invariance=(3,), chunk=71)


@pytest.mark.timeout(600)
def test_paper_network_pruned_unsigned_sampled(capsys):
    # the same network with the paper's unsigned activation codes (0..255 after every ReLU)
    _sampled(capsys, "paper_iodf64_u", CONFIGS["paper_iodf64_u"].batch, sample=(1, 254), invariance=(100,), chunk=97)


@pytest.mark.timeout(600)
def test_paper_network_32_sampled(capsys):
    _sampled(capsys, "paper_res32", CONFIGS["paper_res32"].batch, sample=(0, 300, 511), invariance=(9,), chunk=129)


@pytest.mark.timeout(600)
@pytest.mark.parametrize("name", ["wide_resnet", "wide_resnet_u"])
def test_wide_residual_network_sampled(capsys, name):
    # 256-wide shortcut layers on 204800 pixels: the persistent kernel with the shortcut epilogue
    _sampled(capsys, name, CONFIGS[name].batch, sample=(0, 1, 77, 199), invariance=(5,), chunk=67)


@pytest.mark.timeout(900)
def test_cfg5_batch1(capsys):
    # latency shape: batch 1, the whole image against the oracle
    _sampled(capsys, "cfg5", 1, sample=(0,))


@pytest.mark.timeout(900)
def test_cfg5_batch1024_sampled(capsys):
    # throughput shape; oracle on sampled images, batch invariance on the others
    _sampled(capsys, "cfg5", 1024, sample=_spread(1024, 16, 5), invariance=(1, 511), chunk=301)


def _codec_full(capsys, name, batch, sample):
    """Compressor at full size: every image must decode back exactly; sampled containers are
    compared with the oracle's word for word."""
    import torch

    def say(*a):
        with capsys.disabled():
            print("[full-size codec]", *a, flush=True)

    flow = gpu_flow(name, max_batch=batch)
    x = images(name, batch=batch)
    xg = to_gpu(x)
    words, sizes = flow.encode(xg)
    torch.cuda.synchronize()
    say(name, "batch", batch, "encoded; mean bits/dim %.3f" % (32.0 * float(sizes.float().mean()) / flow.d))
    x2 = flow.decode(words)
    torch.cuda.synchronize()
    assert torch.equal(x2, xg), "codec round trip"
    assert flow.codec_errors() == (0, 0, 0) and flow.range_errors() == 0
    wc, sc = words.cpu().numpy().view(np.uint32), sizes.cpu().numpy().view(np.uint32)
    flow.close()
    om = oracle_model(name)
    for i in sample:
        ref, ref_sizes, cl = om.encode(x[i:i + 1])
        say("oracle container", i, "done:", int(ref_sizes[0]), "words")
        assert cl == 0 and ref_sizes[0] == sc[i] and np.array_equal(ref[0], wc[i]), "container %d" % i


@pytest.mark.timeout(900)
def test_cfg4_codec(capsys):
    _codec_full(capsys, "cfg4", CONFIGS["cfg4"].batch, sample=(5, 100))


@pytest.mark.timeout(900)
def test_cfg5_codec_batch1024(capsys):
    _codec_full(capsys, "cfg5", 1024, sample=(13, 1000))
