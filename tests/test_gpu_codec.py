"""GPU parity of the compressor (prior masses, rANS containers, interleaved decode)
against the CPU oracle, bit for bit, through the C ABI."""
import numpy as np
import pytest

import paper_2206_08869_amd as iodf
from synth import CONFIGS
from util import gpu_flow, images, oracle_model, to_gpu

pytestmark = pytest.mark.gpu


def _u32(t):
    return t.cpu().numpy().view(np.uint32)


def _chunk_layout(cfg):
    n, z_off, code_off, zo, co = [], [], [], 0, 0
    for lv in range(1, cfg.levels + 1):
        C = 12 << (lv - 1)
        hw = (cfg.H >> lv) * (cfg.W >> lv)
        cz = C - C // 2 if lv < cfg.levels else C
        n.append(cz * hw); z_off.append(zo); zo += cz * hw
        if cfg.heads and lv < cfg.levels:
            code_off.append(co); co += 2 * cz * hw
        else:
            code_off.append(-1)
    return n, z_off, code_off


def _oracle_cf(cfg, z, codes):
    import oracle
    n, z_off, code_off = _chunk_layout(cfg)
    C = np.zeros_like(z)
    F = np.zeros_like(z)
    clamped = 0
    for b in range(z.shape[0]):
        for c in range(len(n)):
            k = n[c]
            m = codes[b, code_off[c]:code_off[c] + k] if code_off[c] >= 0 else None
            l = codes[b, code_off[c] + k:code_off[c] + 2 * k] if code_off[c] >= 0 else None
            cc, ff, cl = oracle.prior_cf(z[b, z_off[c]:z_off[c] + k], m, l)
            C[b, z_off[c]:z_off[c] + k] = cc
            F[b, z_off[c]:z_off[c] + k] = ff
            clamped += cl
    return C, F, clamped


@pytest.mark.parametrize("name,batch", [("mini_dense", 5), ("mini_resnet", 3), ("cfg1", 1), ("cfg2", 9)])
def test_prior_masses_match_oracle(name, batch):
    import torch
    cfg = CONFIGS[name]
    flow = gpu_flow(name, max_batch=batch)
    x = images(name, batch=batch)
    z, codes = flow.forward(to_gpu(x))
    C, F = flow.prior_cf(z, codes)
    torch.cuda.synchronize()
    zc = z.cpu().numpy()
    cc = codes.cpu().numpy() if flow.d_codes else np.zeros((batch, 1), np.int8)
    Co, Fo, cl = _oracle_cf(cfg, zc, cc)
    assert np.array_equal(C.cpu().numpy(), Co) and np.array_equal(F.cpu().numpy(), Fo)
    assert flow.codec_errors()[0] == cl == 0
    flow.close()


def test_prior_masses_over_the_whole_alphabet_and_all_codes():
    # synthetic latents and codes (not from a flow): every log-scale code, extreme means,
    # residuals at and beyond both ends of the alphabet
    import torch
    name = "mini_dense"
    cfg = CONFIGS[name]
    flow = gpu_flow(name, max_batch=8)
    d, dc = flow.d, flow.d_codes
    rng = np.random.default_rng(7)
    z = rng.integers(-9000, 9000, size=(8, d), dtype=np.int32)
    z[0, :64] = np.array([-8192, -8193, 8191, 8192, 0, 1, -1, 40000] * 8, np.int32)
    codes = rng.integers(-128, 128, size=(8, dc), dtype=np.int8)
    C, F = flow.prior_cf(to_gpu(z), to_gpu(codes))
    torch.cuda.synchronize()
    Co, Fo, cl = _oracle_cf(cfg, z, codes)
    assert np.array_equal(C.cpu().numpy(), Co) and np.array_equal(F.cpu().numpy(), Fo)
    assert cl > 0 and flow.codec_errors()[0] == cl
    flow.close()


@pytest.mark.parametrize("name,batch", [("mini_dense", 5), ("mini_dense_g", 4), ("mini_resnet", 3),
                                         ("odd_dense_g", 3), ("rect_dense", 3), ("mini_paper_g", 3), ("mini_dense_u", 3), ("mini_resnet_gu", 2), ("deep6", 2), ("cfg1", 1), ("cfg2", 64), ("cfg2g", 7)])
def test_containers_match_oracle_and_decode_everywhere(name, batch):
    import torch
    cfg = CONFIGS[name]
    flow = gpu_flow(name, max_batch=batch)
    x = images(name, batch=batch)
    xg = to_gpu(x)
    words, sizes = flow.encode(xg)
    torch.cuda.synchronize()
    om = oracle_model(name)
    ref, ref_sizes, cl = om.encode(x)
    assert cl == 0
    assert words.shape[1] == ref.shape[1] == flow.query(iodf.IODF_Q_CODEC_MAX_WORDS) == om.codec_max_words()
    assert flow.query(iodf.IODF_Q_CODEC_HEADER_WORDS) == 1 + 48 * cfg.levels
    assert np.array_equal(_u32(sizes), ref_sizes)
    assert np.array_equal(_u32(words), ref)                  # header, states, payload; zeros past the end
    # GPU decodes its own containers and the oracle's; the oracle decodes the GPU's
    assert torch.equal(flow.decode(words), xg)
    assert torch.equal(flow.decode(to_gpu(ref.view(np.int32))), xg)
    x_cpu, errs = om.decode(_u32(words), x.shape[1:])
    assert errs == 0 and np.array_equal(x_cpu, x)
    assert flow.codec_errors() == (0, 0, 0) and flow.range_errors() == 0
    # a smaller batch afterwards reuses the buffers
    if batch > 1:
        w1, s1 = flow.encode(xg[1:2].contiguous())
        assert np.array_equal(_u32(w1)[0], ref[1]) and int(s1[0]) == int(ref_sizes[1])
    flow.close()


def test_capacity_and_malformed_containers():
    import torch
    name, batch = "mini_dense", 6
    flow = gpu_flow(name, max_batch=batch)
    x = images(name, batch=batch)
    xg = to_gpu(x)
    words, sizes = flow.encode(xg)
    need = _u32(sizes).astype(np.int64)
    header = flow.query(iodf.IODF_Q_CODEC_HEADER_WORDS)
    # capacity below what the images need: sizes are still reported, rows never spill into the next
    cap = int(need.min()) - 5
    assert cap > header
    small = torch.full((batch, cap), -1, dtype=torch.int32, device=xg.device)
    _, s2 = flow.encode(xg, cap_words=cap, words=small)
    torch.cuda.synchronize()
    assert np.array_equal(_u32(s2).astype(np.int64), need)
    assert flow.codec_errors()[1] == batch
    assert np.array_equal(_u32(small)[:, 0].astype(np.int64), need)      # each row still starts with its own total
    assert np.array_equal(_u32(small)[:, :cap], _u32(words)[:, :cap])
    # truncated containers are refused lane by lane, without reading outside them
    flow.decode(small)
    assert flow.codec_errors()[2] > 0
    # damaged payload / header: no crash, damage is either detected or changes the image
    bad = words.clone()
    bad[:, header + 3] ^= 0x55
    xb = flow.decode(bad)
    broken = flow.codec_errors()[2]
    assert broken > 0 or not torch.equal(xb, xg)
    bad = words.clone()
    bad[:, 2] += 1000                                                # a lane claims 1000 more words
    flow.decode(bad)
    assert flow.codec_errors()[2] > 0
    bad = words.clone()
    bad[:, 0] = 1 << 30                                              # absurd total
    flow.decode(bad)
    assert flow.codec_errors()[2] > 0
    flow.range_errors()
    # the context still works
    assert torch.equal(flow.decode(words), xg)
    assert flow.codec_errors() == (0, 0, 0)
    # capacity smaller than a header is an argument error
    with pytest.raises(iodf.IodfError):
        flow.decode(torch.zeros((batch, header - 1), dtype=torch.int32, device=xg.device))
    flow.close()


def test_codec_with_and_without_graph_replay(monkeypatch):
    import torch
    name, batch = "mini_dense_g", 4
    x = images(name, batch=batch)
    xg = to_gpu(x)
    flow = gpu_flow(name, max_batch=batch)
    w_a, s_a = flow.encode(xg)
    torch.cuda.synchronize()
    flow.close()
    monkeypatch.setenv("IODF_NO_GRAPH", "1")
    flow = gpu_flow(name, max_batch=batch)
    w_b, s_b = flow.encode(xg)
    assert torch.equal(w_a, w_b) and torch.equal(s_a, s_b)
    assert torch.equal(flow.decode(w_b), xg)
    flow.close()


def test_patch_based_coding_of_a_large_image():
    import oracle
    import torch
    from synth import make_large_image
    name = "mini_dense"           # 16 x 16 patches
    flow = gpu_flow(name, max_batch=7)   # 30 patches in sub-batches of 7, 7, 7, 7, 2
    h, w = 75, 90                 # ragged on both sides: 5 x 6 patches
    img = make_large_image(h, w, seed=1901)
    ig = to_gpu(img)
    assert flow.n_patches(h, w) == 30
    patches = flow.tile_patches(ig)
    ref = oracle.tile_patches(img, 16, 16)
    assert np.array_equal(patches.cpu().numpy(), ref)
    sub = flow.tile_patches(ig, first=11, n=5)
    assert np.array_equal(sub.cpu().numpy(), ref[11:16])
    back = torch.zeros_like(ig)
    flow.untile_patches(patches, back)
    assert torch.equal(back, ig)
    # whole image through the compressor, sub-batch by sub-batch; containers equal the oracle's
    parts = flow.encode_image(ig)
    assert [p[0].shape[0] for p in parts] == [7, 7, 7, 7, 2]
    om = oracle_model(name)
    ref_words, ref_sizes, _ = om.encode(ref)
    got = np.concatenate([_u32(p[0]) for p in parts])
    assert np.array_equal(got, ref_words) and np.array_equal(np.concatenate([_u32(p[1]) for p in parts]), ref_sizes)
    img2 = flow.decode_image(parts, h, w)
    assert torch.equal(img2, ig) and flow.codec_errors() == (0, 0, 0)
    # patches beyond the grid are refused
    with pytest.raises(iodf.IodfError):
        flow.tile_patches(ig, first=28, n=3)
    flow.close()
