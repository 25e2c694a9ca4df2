"""GPU parity at the benchmark's full sizes, in the launch configuration bench.py
times. The oracle cannot run whole batches of the width-512 flows in reasonable
time, so a few images of each batch are recomputed by the oracle one by one and
compared bit-exactly; the rest of the batch is covered by properties that hold at
any size: exact round trip and per-image batch invariance."""
import numpy as np
import pytest

from synth import CONFIGS
from util import gpu_flow, images, oracle_model, to_gpu

pytestmark = pytest.mark.gpu


def _sampled(capsys, name, batch, sample, invariance=()):
    import torch

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
    zc, cc = z.cpu().numpy(), codes.cpu().numpy()
    flow.close()
    om = oracle_model(name)
    for i in sample:
        z_ref, c_ref = om.forward(x[i:i + 1])
        say("oracle image", i, "done")
        assert np.array_equal(zc[i], z_ref[0]), "z differs from oracle at image %d" % i
        assert np.array_equal(cc[i], c_ref[0]), "codes differ from oracle at image %d" % i


@pytest.mark.timeout(600)
def test_cfg3_sampled(capsys):
    _sampled(capsys, "cfg3", CONFIGS["cfg3"].batch, sample=(131, 255), invariance=(7,))


@pytest.mark.timeout(900)
def test_cfg4_sampled(capsys):
    _sampled(capsys, "cfg4", CONFIGS["cfg4"].batch, sample=(77,), invariance=(64,))


@pytest.mark.timeout(900)
def test_cfg5_batch1(capsys):
    # latency shape: batch 1, the whole image against the oracle
    _sampled(capsys, "cfg5", 1, sample=(0,))


@pytest.mark.timeout(900)
def test_cfg5_batch1024_sampled(capsys):
    # throughput shape; oracle on one sampled image, batch invariance on others
    _sampled(capsys, "cfg5", 1024, sample=(1023,), invariance=(1, 511))
