"""iodf_encode_noalloc (the entry point for callers that cannot allocate device memory: its coder
buffers live in a static device array) against iodf_encode, through the C ABI: containers and sizes
must be equal word for word, on two calls in a row, the second with a smaller batch of other images
(what the first call left in the shared array must not leak into the second), and a batch beyond
the array's capacity must be refused before anything runs."""
import ctypes

import numpy as np
import pytest

import paper_2206_08869_amd as iodf
from synth import CONFIGS
from util import blob_of, images, to_gpu

pytestmark = pytest.mark.gpu


def _raw_encode(fn, flow, xg, cap):
    import torch
    b = xg.shape[0]
    # poisoned outputs: every word the container claims must have been written by the call
    words = torch.full((b, cap), -1, dtype=torch.int32, device="cuda")
    sizes = torch.full((b,), -1, dtype=torch.int32, device="cuda")
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    fn(flow._ctx, ctypes.c_void_p(xg.data_ptr()), b, ctypes.c_void_p(words.data_ptr()), cap,
       ctypes.c_void_p(sizes.data_ptr()), stream)
    torch.cuda.synchronize()
    return words.cpu().numpy().view(np.uint32), sizes.cpu().numpy().view(np.uint32)


@pytest.mark.parametrize("name", ["mini_dense", "cfg1", "mini_resnet_gu"])
def test_noalloc_encode_equals_encode_on_two_calls(name):
    import torch
    cfg = CONFIGS[name]
    big = max(cfg.batch, 3)
    flow = iodf.Flow(blob_of(name), max_batch=big, device=0)
    cap = flow.query(iodf.IODF_Q_CODEC_MAX_WORDS)
    assert flow.query(iodf.IODF_Q_NOALLOC_MAX_BATCH) == big   # small flows fit whole
    x_all = images(name, batch=big + 2, kind="filtered")
    first, second = x_all[:big], x_all[big:big + 2][::-1].copy()   # second call: fewer, different images
    got = []
    for x in (first, second):
        xg = to_gpu(x)
        got.append(_raw_encode(iodf.iodf_encode_noalloc, flow, xg, cap))
    for x, (w, s) in zip((first, second), got):
        xg = to_gpu(x)
        w_ref, s_ref = _raw_encode(iodf.iodf_encode, flow, xg, cap)
        assert np.array_equal(s, s_ref), "sizes differ"
        for i in range(x.shape[0]):   # words beyond a container's size are unspecified in both
            assert np.array_equal(w[i, :s[i]], w_ref[i, :s_ref[i]]), "container %d differs" % i
        # and they decode back
        x_dec = flow.decode(torch.from_numpy(w.view(np.int32)).cuda())
        torch.cuda.synchronize()
        assert np.array_equal(x_dec.cpu().numpy(), x)
    assert flow.codec_errors() == (0, 0, 0)
    flow.close()


def test_noalloc_encode_refuses_what_does_not_fit():
    import torch
    name = "mini_dense"
    flow = iodf.Flow(blob_of(name), max_batch=20000, device=0)   # 16x16 images: a few KB of scratch each
    limit = flow.query(iodf.IODF_Q_NOALLOC_MAX_BATCH)
    assert 0 < limit < 20000
    cap = flow.query(iodf.IODF_Q_CODEC_MAX_WORDS)
    x = to_gpu(np.repeat(images(name, batch=1), limit + 1, axis=0))
    words = torch.zeros((limit + 1, cap), dtype=torch.int32, device="cuda")
    sizes = torch.zeros((limit + 1,), dtype=torch.int32, device="cuda")
    with pytest.raises(iodf.IodfError) as e:
        flow.encode(x, words=words, sizes=sizes, noalloc=True)
    assert e.value.code == -7
    # the largest batch that fits is accepted and equals the allocating entry point's result
    w1, s1 = flow.encode(x[:limit], words=words[:limit], sizes=sizes[:limit], noalloc=True)
    torch.cuda.synchronize()
    w1, s1 = w1.cpu().numpy().copy(), s1.cpu().numpy().copy()
    w2, s2 = flow.encode(x[:limit])
    torch.cuda.synchronize()
    assert np.array_equal(s1, s2.cpu().numpy())
    n = int(s1[0])
    assert np.array_equal(w1[:, :n], w2.cpu().numpy()[:, :n]) and (s1 == n).all()   # the same image every time
    flow.close()
