"""Pins for the oracle's arithmetic primitives: requantise, saturate, conv, squeeze,
epilogue. Everything here runs on the CPU and checks the oracle against values
worked by hand, exact rational arithmetic, a library convolution and brute force."""
from fractions import Fraction
import os

import numpy as np
import pytest
import torch

import oracle


def _rows(path):
    for line in open(path):
        line = line.split("#")[0].strip()
        if line:
            yield line.split()


def _half_away(q):
    """Round a Fraction to the nearest integer, ties away from zero."""
    n = abs(q)
    r = int(n + Fraction(1, 2))  # floor(|q| + 1/2)
    return r if q >= 0 else -r


# ---- requantise --------------------------------------------------------------

def test_rq_hand_worked_table(golden_dir):
    rows = list(_rows(os.path.join(golden_dir, "rq_table.txt")))
    assert len(rows) >= 29
    for a, M, s, want in rows:
        assert oracle.rq(int(a), int(M), int(s)) == int(want), (a, M, s)


def test_rq_discriminates_rounding_modes():
    # each wrong rule differs from half-away on at least one of these
    assert oracle.rq(5, 1, 1) == 3 and oracle.rq(1, 1, 1) == 1      # half-even gives 2, 0
    assert oracle.rq(3, 1, 1) == 2                                   # floor gives 1
    assert oracle.rq(-5, 1, 1) == -3 and oracle.rq(-1, 1, 1) == -1   # half-up gives -2, 0
    assert oracle.rq(-3, 1, 1) == -2                                 # truncation gives -1


def test_rq_matches_exact_rationals():
    rng = np.random.default_rng(7)
    cases = [(0, 1, 0), (2**31 - 1, 2**31 - 1, 62), (-2**31, 2**31 - 1, 62), (-2**31, 2**31 - 1, 0),
             (2**31 - 1, 2**31 - 1, 0), (1, 1, 62), (-1, 1, 62), (2**30, 2**30, 61), (-(2**30), 2**30, 61)]
    for _ in range(20000):
        s = int(rng.integers(0, 63))
        a = int(rng.integers(-2**31, 2**31))
        M = int(rng.integers(0, 2**31))
        if rng.random() < 0.3:   # force exact ties: a*M odd multiple of 2^(s-1)
            s = int(rng.integers(1, 20))
            M = 1 << (s - 1)
            a = 2 * int(rng.integers(-10**6, 10**6)) + 1
        cases.append((a, M, s))
    for a, M, s in cases:
        assert oracle.rq(a, M, s) == _half_away(Fraction(a * M, 2**s)), (a, M, s)


def test_rq_is_odd_and_monotone():
    M, s = 1518500250, 40
    prev = None
    for a in range(-5000, 5001):
        v = oracle.rq(a, M, s)
        assert v == -oracle.rq(-a, M, s)
        assert prev is None or v >= prev
        prev = v


def test_sat8_table(golden_dir):
    for v, want in _rows(os.path.join(golden_dir, "sat8_table.txt")):
        assert oracle.sat8(int(v)) == int(want)


# ---- convolution ---------------------------------------------------------------

def _read_blocks(path):
    blocks, cur = {}, None
    for line in open(path):
        line = line.split("#")[0].strip()
        if not line:
            continue
        if line.isalpha():
            cur = line
            blocks[cur] = []
        else:
            blocks[cur].append([int(t) for t in line.split()])
    return {k: np.array(v) for k, v in blocks.items()}


def test_conv_asymmetric_kernel_example(golden_dir):
    b = _read_blocks(os.path.join(golden_dir, "conv_asym.txt"))
    acc = oracle.conv_acc(b["input"][None].astype(np.int8), b["kernel"][None, None].astype(np.int8))
    assert np.array_equal(acc[0], b["output"])
    flipped = oracle.conv_acc(b["input"][None].astype(np.int8),
                              b["kernel"][::-1, ::-1][None, None].astype(np.int8))
    assert np.array_equal(flipped[0], -b["output"])


def _brute_conv(x, W, bias):
    """Gather-style loop nest (output-stationary, explicit zero-padded copy)."""
    D, h, w = x.shape
    C, _, k, _ = W.shape
    p = (k - 1) // 2
    xp = np.zeros((D, h + 2 * p, w + 2 * p), dtype=np.int64)
    xp[:, p:p + h, p:p + w] = x
    out = np.zeros((C, h, w), dtype=np.int64)
    for i in range(h):
        for j in range(w):
            for c in range(C):
                tot = int(bias[c])
                for ky in range(k):
                    for kx in range(k):
                        for cp in range(D):
                            tot += int(W[c, cp, ky, kx]) * int(xp[cp, i + ky, j + kx])
                out[c, i, j] = tot
    return out


@pytest.mark.parametrize("D,C,h,w,k", [(1, 1, 1, 1, 3), (2, 3, 4, 5, 3), (3, 2, 5, 3, 1), (5, 4, 2, 2, 3),
                                       (4, 4, 1, 6, 3)])
def test_conv_brute_force_tiny(D, C, h, w, k):
    rng = np.random.default_rng(D * 100 + C * 10 + h)
    x = rng.integers(-128, 128, (D, h, w)).astype(np.int8)
    W = rng.integers(-128, 128, (C, D, k, k)).astype(np.int8)
    bias = rng.integers(-10**6, 10**6, C).astype(np.int32)
    assert np.array_equal(oracle.conv_acc(x, W, bias), _brute_conv(x, W, bias))


@pytest.mark.parametrize("D,C,h,w,k", [(6, 32, 4, 4, 3), (32, 6, 4, 4, 3), (64, 48, 16, 16, 3), (96, 64, 8, 8, 1),
                                       (17, 5, 7, 9, 3)])
def test_conv_matches_library_conv2d(D, C, h, w, k):
    rng = np.random.default_rng(D + C)
    x = rng.integers(-128, 128, (D, h, w)).astype(np.int8)
    W = rng.integers(-128, 128, (C, D, k, k)).astype(np.int8)
    bias = rng.integers(-2**20, 2**20, C).astype(np.int32)
    ref = torch.nn.functional.conv2d(torch.from_numpy(x.astype(np.float64))[None],
                                     torch.from_numpy(W.astype(np.float64)),
                                     torch.from_numpy(bias.astype(np.float64)), padding=(k - 1) // 2)[0]
    assert np.array_equal(oracle.conv_acc(x, W, bias), ref.numpy().astype(np.int64))


def test_conv_is_linear_in_input_and_1x1_is_matmul():
    rng = np.random.default_rng(3)
    x1 = rng.integers(-60, 60, (8, 6, 6)).astype(np.int8)
    x2 = rng.integers(-60, 60, (8, 6, 6)).astype(np.int8)
    W = rng.integers(-128, 128, (5, 8, 3, 3)).astype(np.int8)
    a = oracle.conv_acc(x1, W).astype(np.int64) + oracle.conv_acc(x2, W)
    assert np.array_equal(a, oracle.conv_acc((x1 + x2).astype(np.int8), W))
    W1 = rng.integers(-128, 128, (5, 8, 1, 1)).astype(np.int8)
    mm = W1[:, :, 0, 0].astype(np.int64) @ x1.reshape(8, -1).astype(np.int64)
    assert np.array_equal(oracle.conv_acc(x1, W1).reshape(5, -1), mm)


def test_conv_extreme_values_stay_in_int32():
    # the deepest contraction of the dense family: 4608 channels x 9 taps of (-128)*(-128)
    D = 4608
    x = np.full((D, 3, 3), -128, dtype=np.int8)
    W = np.full((1, D, 3, 3), -128, dtype=np.int8)
    acc = oracle.conv_acc(x, W)
    assert acc[0, 1, 1] == 41472 * 128 * 128 and acc[0, 1, 1] < 2**31
    assert acc[0, 0, 0] == 4 * D * 128 * 128


def test_conv_gate_skips_channel():
    rng = np.random.default_rng(5)
    x = rng.integers(-128, 128, (3, 4, 4)).astype(np.int8)
    W = rng.integers(-128, 128, (4, 3, 3, 3)).astype(np.int8)
    gate = np.array([1, 0, 1, 1], dtype=np.uint8)
    full = oracle.conv_acc(x, W)
    g = oracle.conv_acc(x, W, gate=gate)
    assert np.array_equal(full[[0, 2, 3]], g[[0, 2, 3]])


# ---- epilogue ------------------------------------------------------------------

def test_epilogue_order_relu_shortcut_saturation_gate():
    acc = np.array([[[100, -100, 300, -300, 40]], [[100, -100, 300, -300, 40]]], dtype=np.int32)
    M = np.array([1, 1], dtype=np.int32)
    sh = np.array([1, 1], dtype=np.uint8)          # value / 2, ties away
    y = oracle.epilogue(acc, M, sh)
    assert y.tolist() == [[[50, -50, 127, -128, 20]]] * 2
    y = oracle.epilogue(acc, M, sh, relu=True)
    assert y.tolist() == [[[50, 0, 127, 0, 20]]] * 2
    sc = np.array([[[-60, 60, -100, 127, 127]]] * 2, dtype=np.int8)
    # shortcut is added in the wide integer before ReLU and before the single saturation:
    # 150 + (-100) = 50 (a saturated branch would have given 27); -150 + 127 = -23 -> ReLU 0
    y = oracle.epilogue(acc, M, sh, relu=True, shortcut=sc)
    assert y.tolist() == [[[0, 10, 50, 0, 127]]] * 2
    y = oracle.epilogue(acc, M, sh, relu=False, shortcut=sc)
    assert y.tolist() == [[[-10, 10, 50, -23, 127]]] * 2
    # a gated-off filter contributes exactly 0; the shortcut still passes (scatter-add)
    gate = np.array([1, 0], dtype=np.uint8)
    y = oracle.epilogue(acc, M, sh, gate=gate, relu=True)
    assert y[1].tolist() == [[0, 0, 0, 0, 0]] and y[0].tolist() == [[50, 0, 127, 0, 20]]
    y = oracle.epilogue(acc, M, sh, gate=gate, relu=True, shortcut=sc)
    assert y[1].tolist() == [[0, 60, 0, 127, 127]]


def test_epilogue_per_channel_constants():
    acc = np.array([[[1000]], [[1000]], [[-1000]]], dtype=np.int32)
    M = np.array([1 << 30, 3 << 29, 1 << 30], dtype=np.int32)
    sh = np.array([34, 35, 33], dtype=np.uint8)
    # 1000/16 = 62.5 -> 63 ; 1000*1.5/32 = 46.875 -> 47 ; -1000/8 = -125
    assert oracle.epilogue(acc, M, sh).reshape(-1).tolist() == [63, 47, -125]


# ---- squeeze -------------------------------------------------------------------

def test_squeeze_worked_example(golden_dir):
    want = np.array([[int(t) for t in r] for r in _rows(os.path.join(golden_dir, "squeeze_4x4.txt"))])
    got = oracle.squeeze(np.arange(16, dtype=np.int32).reshape(1, 4, 4))
    assert np.array_equal(got.reshape(4, 4), want)


def test_squeeze_matches_reshape_formulation_and_inverts():
    rng = np.random.default_rng(11)
    a = rng.integers(-1000, 1000, (5, 6, 8)).astype(np.int32)
    # independent formulation: split both axes into (coarse, fine) and move fine to channels
    ref = a.reshape(5, 3, 2, 4, 2).transpose(0, 2, 4, 1, 3).reshape(20, 3, 4)
    got = oracle.squeeze(a)
    assert np.array_equal(got, ref)
    assert np.array_equal(oracle.unsqueeze(got), a)
