"""The oracle under AddressSanitizer + UndefinedBehaviorSanitizer (make -C oracle asan).

The sanitised build is a small driver program around the same C sources. These tests feed it the
hand-worked rounding table (Sec. 4.1 / 4.2: requantisation to 8 bit, round to nearest with ties away
from zero, saturation) and whole small flows of every network family, signed and unsigned, gated and
not; the driver must exit cleanly (no out-of-bounds access, no signed overflow, no misaligned load)
and its outputs must equal those of the optimised library build bit for bit, so neither build's
results depend on undefined behaviour."""
import os
import subprocess

import numpy as np
import pytest

from synth import CONFIGS
from util import blob_of, images, oracle_model

HERE = os.path.dirname(os.path.abspath(__file__))
ORACLE_DIR = os.path.join(os.path.dirname(HERE), "oracle")
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="halt_on_error=1",
           OMP_NUM_THREADS="2")
ENV.pop("LD_PRELOAD", None)   # the sanitiser runtime must come first in the driver's own process


@pytest.fixture(scope="module")
def driver():
    subprocess.check_call(["make", "-s", "-C", ORACLE_DIR, "asan"])
    return os.path.join(ORACLE_DIR, "sanitize_driver")


def _rows(path):
    for line in open(path):
        line = line.split("#")[0].split()
        if line:
            yield [int(v) for v in line]


def test_rounding_tables_under_sanitizers(driver, golden_dir):
    rows = list(_rows(os.path.join(golden_dir, "rq_table.txt")))
    assert len(rows) >= 24
    # plus the extremes of the domain: |a| = 2^31 - 1 and 2^31, M = 2^31 - 1, shifts 0 and 62
    extremes = [(2**31 - 1, 2**31 - 1, 0), (-2**31, 2**31 - 1, 0), (-2**31, 2**31 - 1, 62), (2**31 - 1, 1, 62)]
    text = "".join("%d %d %d\n" % (a, M, s) for a, M, s, *_ in rows) + "".join("%d %d %d\n" % e for e in extremes)
    res = subprocess.run([driver, "rq"], input=text, capture_output=True, text=True, env=ENV, timeout=60)
    assert res.returncode == 0, res.stderr[-2000:]
    assert "runtime error" not in res.stderr and "AddressSanitizer" not in res.stderr
    got = [[int(v) for v in l.split()] for l in res.stdout.split("\n") if l.strip()]
    assert len(got) == len(rows) + len(extremes)
    for (a, M, s, want), (r, sat) in zip(rows, got):
        assert r == want, (a, M, s)
        assert sat == max(-128, min(127, want))
    for (a, M, s), (r, _) in zip(extremes, got[len(rows):]):
        num, den = a * M, 1 << s   # exact: round half away from zero
        want = (abs(num) * 2 + den) // (2 * den) * (1 if num >= 0 else -1)
        assert r == want, (a, M, s)


@pytest.mark.parametrize("name", ["cfg1", "mini_dense_g", "mini_resnet_g", "mini_dense_u", "mini_resnet_gu",
                                  "odd_dense_g", "rect_dense", "mini_paper_g", "deep6"])
def test_small_flows_under_sanitizers(driver, tmp_path, name):
    cfg = CONFIGS[name]
    b = min(cfg.batch, 2)
    blob = np.ascontiguousarray(blob_of(name))
    x = images(name, batch=b)
    (tmp_path / "blob.bin").write_bytes(blob.tobytes())
    (tmp_path / "x.bin").write_bytes(np.ascontiguousarray(x).tobytes())
    out = tmp_path / "out.bin"
    res = subprocess.run([driver, "flow", str(tmp_path / "blob.bin"), str(tmp_path / "x.bin"), str(b), str(out)],
                         capture_output=True, text=True, env=ENV, timeout=300)
    assert res.returncode == 0, res.stderr[-3000:]
    assert "runtime error" not in res.stderr and "AddressSanitizer" not in res.stderr, res.stderr[-3000:]
    info = dict(zip(res.stdout.split()[0::2], (int(v) for v in res.stdout.split()[1::2])))
    assert info["range_errors"] == 0 and info["clamped"] == 0 and info["decode_errors"] == 0
    d, dc, cap = info["d"], info["d_codes"], info["cap"]
    raw = np.frombuffer(out.read_bytes(), np.uint8)
    pos = 0

    def take(n, dtype):
        nonlocal pos
        a = raw[pos:pos + n * np.dtype(dtype).itemsize].view(dtype)
        pos += n * np.dtype(dtype).itemsize
        return a

    z = take(b * d, np.int32).reshape(b, d)
    codes = take(b * dc, np.int8).reshape(b, dc)
    x2 = take(b * d, np.uint8).reshape(x.shape)
    cont = take(b * cap, np.uint32).reshape(b, cap)
    sizes = take(b, np.uint32)
    x3 = take(b * d, np.uint8).reshape(x.shape)
    assert pos == raw.size
    om = oracle_model(name)
    z_ref, c_ref = om.forward(x)
    assert np.array_equal(z, z_ref)
    if cfg.heads:
        assert np.array_equal(codes, c_ref)
    assert np.array_equal(x2, x) and np.array_equal(x3, x)
    w_ref, s_ref, _ = om.encode(x)
    assert np.array_equal(sizes, s_ref) and np.array_equal(cont, w_ref)
