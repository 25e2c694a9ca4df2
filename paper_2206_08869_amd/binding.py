"""Thin ctypes binding of libiodf (argument marshalling only).

Function names mirror the C ABI in include/iodf.h. PyTorch supplies device memory
(tensor.data_ptr()) and the stream; every step of the flow runs in the library's
HIP kernels. There is no CPU fallback: without the built library, calls raise.
"""
import ctypes
import glob
import os
import subprocess

import numpy as np

_PKG = os.path.dirname(os.path.abspath(__file__))
_ROOT = os.path.dirname(_PKG)
LIB_PATH = os.path.join(_PKG, "libiodf.so")
_LIB = None

IODF_Q_Z_ELEMS, IODF_Q_CODE_BYTES, IODF_Q_WORKSPACE_BYTES, IODF_Q_MACS_FORWARD, IODF_Q_MACS_INVERSE, \
    IODF_Q_RANGE_ERRORS, IODF_Q_MAX_BATCH, IODF_Q_IMAGE_H, IODF_Q_IMAGE_W, IODF_Q_CONV_LAUNCHES, \
    IODF_Q_WIDE_MACS_FORWARD, IODF_Q_CODEC_HEADER_WORDS, IODF_Q_CODEC_MAX_WORDS, IODF_Q_CODEC_CLAMPED, \
    IODF_Q_CODEC_OVERFLOWS, IODF_Q_CODEC_BROKEN_LANES, IODF_Q_NOALLOC_MAX_BATCH = range(17)

EXPORTS = ["iodf_init", "iodf_forward", "iodf_inverse", "iodf_query", "iodf_free", "iodf_strerror",
           "iodf_last_hip_error", "iodf_profile_begin", "iodf_profile_end", "iodf_prior_cf", "iodf_encode",
           "iodf_decode", "iodf_codec_tables", "iodf_tile_patches", "iodf_untile_patches",
           "iodf_conv_probe", "iodf_encode_noalloc", "iodf_conv_probe_timeline"]


class KernelStat(ctypes.Structure):
    _fields_ = [("name", ctypes.c_char * 48), ("launches", ctypes.c_int64), ("total_ms", ctypes.c_double),
                ("macs", ctypes.c_int64), ("bytes", ctypes.c_int64), ("issued_macs", ctypes.c_int64)]


class IodfError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__("libiodf: %s (code %d)" % (msg, code))
        self.code = code


def build_library(verbose=False):
    """Compile the HIP sources for gfx950 into libiodf.so (in tree): one object per source, in parallel, then link."""
    from concurrent.futures import ThreadPoolExecutor
    srcs = sorted(glob.glob(os.path.join(_PKG, "csrc", "*.hip")))
    objdir = os.path.join(_PKG, "_build")
    os.makedirs(objdir, exist_ok=True)
    flags = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
             "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-I", os.path.join(_ROOT, "include")]

    def run(cmd):
        res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        out = "\n".join(l for l in res.stdout.splitlines() if "packed-fp32-ops" not in l)
        if res.returncode != 0:
            raise RuntimeError("hipcc failed:\n" + out)
        return out

    objs = [os.path.join(objdir, os.path.basename(s)[:-4] + ".o") for s in srcs]
    with ThreadPoolExecutor(max_workers=min(8, len(srcs))) as pool:
        outs = list(pool.map(lambda so: run(["hipcc"] + flags + ["-c", so[0], "-o", so[1]]), zip(srcs, objs)))
    outs.append(run(["hipcc", "--offload-arch=gfx950", "-fPIC", "-shared", "-o", LIB_PATH] + objs))
    if verbose and "".join(outs).strip():
        print("\n".join(o for o in outs if o.strip()))
    global _LIB
    _LIB = None
    return LIB_PATH


def load_library(build_if_missing=True):
    global _LIB
    if _LIB is not None:
        return _LIB
    if not os.path.exists(LIB_PATH):
        if not build_if_missing:
            raise RuntimeError("libiodf.so is not built (run __graft_entry__.build())")
        build_library()
    L = ctypes.CDLL(LIB_PATH)
    vp, ci = ctypes.c_void_p, ctypes.c_int
    L.iodf_init.restype = ci
    L.iodf_init.argtypes = [ctypes.POINTER(vp), vp, ctypes.c_size_t, ci, ci]
    L.iodf_forward.restype = ci
    L.iodf_forward.argtypes = [vp, vp, ci, vp, vp, vp]
    L.iodf_inverse.restype = ci
    L.iodf_inverse.argtypes = [vp, vp, ci, vp, vp]
    L.iodf_query.restype = ci
    L.iodf_query.argtypes = [vp, ci, ctypes.POINTER(ctypes.c_int64)]
    L.iodf_free.restype = None
    L.iodf_free.argtypes = [vp]
    L.iodf_strerror.restype = ctypes.c_char_p
    L.iodf_strerror.argtypes = [ci]
    L.iodf_last_hip_error.restype = ci
    L.iodf_profile_begin.restype = ci
    L.iodf_profile_begin.argtypes = [vp, ci]
    L.iodf_profile_end.restype = ci
    L.iodf_profile_end.argtypes = [vp, ctypes.POINTER(KernelStat), ci, ctypes.POINTER(ci)]
    L.iodf_prior_cf.restype = ci
    L.iodf_prior_cf.argtypes = [vp, vp, vp, ci, vp, vp, vp]
    L.iodf_encode.restype = ci
    L.iodf_encode.argtypes = [vp, vp, ci, vp, ctypes.c_int64, vp, vp]
    L.iodf_encode_noalloc.restype = ci
    L.iodf_encode_noalloc.argtypes = [vp, vp, ci, vp, ctypes.c_int64, vp, vp]
    L.iodf_decode.restype = ci
    L.iodf_decode.argtypes = [vp, vp, ctypes.c_int64, ci, vp, vp]
    L.iodf_codec_tables.restype = ci
    L.iodf_codec_tables.argtypes = [vp, vp]
    L.iodf_conv_probe.restype = ci
    L.iodf_conv_probe.argtypes = [ci, ci, ci, ci, ci, ci, ci, ci, vp, vp, vp, vp, vp, vp, ci,
                                  ctypes.POINTER(ctypes.c_float)]
    L.iodf_conv_probe_timeline.restype = ci
    L.iodf_conv_probe_timeline.argtypes = [ci, ci, ci, ci, ci, ci, ci, ci, vp, vp, vp, vp, vp, vp, ci,
                                           ctypes.POINTER(ctypes.c_float), vp, ci, ctypes.POINTER(ci)]
    L.iodf_tile_patches.restype = ci
    L.iodf_tile_patches.argtypes = [vp, vp, ci, ci, ci, ci, vp, vp]
    L.iodf_untile_patches.restype = ci
    L.iodf_untile_patches.argtypes = [vp, vp, ci, ci, vp, ci, ci, vp]
    _LIB = L
    return L


def _check(rc):
    if rc != 0:
        L = load_library()
        msg = L.iodf_strerror(rc).decode()
        if rc == -5:
            msg += " (hipError %d)" % L.iodf_last_hip_error()
        raise IodfError(rc, msg)


def iodf_init(blob, device_ordinal=0, max_batch=1):
    """blob: host bytes (numpy uint8 array). Returns an opaque context handle."""
    L = load_library()
    blob = np.ascontiguousarray(blob, dtype=np.uint8)
    h = ctypes.c_void_p()
    _check(L.iodf_init(ctypes.byref(h), blob.ctypes.data_as(ctypes.c_void_p), blob.size, int(device_ordinal),
                       int(max_batch)))
    return h


def iodf_forward(ctx, x_ptr, batch, z_ptr, codes_ptr, stream):
    _check(load_library().iodf_forward(ctx, x_ptr, int(batch), z_ptr, codes_ptr, stream))


def iodf_inverse(ctx, z_ptr, batch, x_ptr, stream):
    _check(load_library().iodf_inverse(ctx, z_ptr, int(batch), x_ptr, stream))


def iodf_prior_cf(ctx, z_ptr, codes_ptr, batch, c_ptr, f_ptr, stream):
    _check(load_library().iodf_prior_cf(ctx, z_ptr, codes_ptr, int(batch), c_ptr, f_ptr, stream))


def iodf_encode(ctx, x_ptr, batch, words_ptr, cap_words, sizes_ptr, stream):
    _check(load_library().iodf_encode(ctx, x_ptr, int(batch), words_ptr, int(cap_words), sizes_ptr, stream))


def iodf_encode_noalloc(ctx, x_ptr, batch, words_ptr, cap_words, sizes_ptr, stream):
    _check(load_library().iodf_encode_noalloc(ctx, x_ptr, int(batch), words_ptr, int(cap_words), sizes_ptr, stream))


def iodf_decode(ctx, words_ptr, cap_words, batch, x_ptr, stream):
    _check(load_library().iodf_decode(ctx, words_ptr, int(cap_words), int(batch), x_ptr, stream))


def iodf_tile_patches(ctx, img_ptr, img_h, img_w, first_patch, n_patches, x_ptr, stream):
    _check(load_library().iodf_tile_patches(ctx, img_ptr, int(img_h), int(img_w), int(first_patch), int(n_patches),
                                            x_ptr, stream))


def iodf_untile_patches(ctx, x_ptr, first_patch, n_patches, img_ptr, img_h, img_w, stream):
    _check(load_library().iodf_untile_patches(ctx, x_ptr, int(first_patch), int(n_patches), img_ptr, int(img_h),
                                              int(img_w), stream))


def iodf_conv_probe(x, w, bias, m, shift, relu=True, iters=20, device_ordinal=0):
    """One conv layer on host arrays: x int8 [B,C_in,h,w], w int8 [C_out,C_in,k,k] -> (y int8 [B,C_out,h,w], us per launch)."""
    x = np.ascontiguousarray(x, np.int8)
    w = np.ascontiguousarray(w, np.int8)
    bias = np.ascontiguousarray(bias, np.int32)
    m = np.ascontiguousarray(m, np.int32)
    shift = np.ascontiguousarray(shift, np.uint8)
    b, c_in, h, wd = x.shape
    c_out, c_in2, k, k2 = w.shape
    assert c_in == c_in2 and k == k2 and bias.size == m.size == shift.size == c_out
    y = np.zeros((b, c_out, h, wd), np.int8)
    us = ctypes.c_float(0)
    p = lambda a: a.ctypes.data_as(ctypes.c_void_p)
    _check(load_library().iodf_conv_probe(int(device_ordinal), c_in, c_out, k, h, wd, b, 1 if relu else 0, p(x), p(w),
                                          p(bias), p(m), p(shift), p(y), int(iters), ctypes.byref(us)))
    return y, float(us.value)


def iodf_conv_probe_timeline(x, w, bias, m, shift, relu=True, iters=20, max_tiles=4096, device_ordinal=0):
    """As iodf_conv_probe, plus the per-tile timeline of one more launch: int64 [n_tiles, 8] (see include/iodf.h)."""
    x = np.ascontiguousarray(x, np.int8)
    w = np.ascontiguousarray(w, np.int8)
    bias = np.ascontiguousarray(bias, np.int32)
    m = np.ascontiguousarray(m, np.int32)
    shift = np.ascontiguousarray(shift, np.uint8)
    b, c_in, h, wd = x.shape
    c_out, c_in2, k, k2 = w.shape
    assert c_in == c_in2 and k == k2 and bias.size == m.size == shift.size == c_out
    y = np.zeros((b, c_out, h, wd), np.int8)
    tl = np.zeros((max_tiles, 8), np.int64)
    us, n = ctypes.c_float(0), ctypes.c_int(0)
    p = lambda a: a.ctypes.data_as(ctypes.c_void_p)
    _check(load_library().iodf_conv_probe_timeline(int(device_ordinal), c_in, c_out, k, h, wd, b, 1 if relu else 0,
                                                   p(x), p(w), p(bias), p(m), p(shift), p(y), int(iters),
                                                   ctypes.byref(us), p(tl), int(max_tiles), ctypes.byref(n)))
    return y, float(us.value), tl[:n.value]


def iodf_codec_tables():
    """(sig int32 [3073], inv int64 [256]) as the library builds them; needs no GPU."""
    sig = np.empty(3073, np.int32)
    inv = np.empty(256, np.int64)
    _check(load_library().iodf_codec_tables(sig.ctypes.data_as(ctypes.c_void_p), inv.ctypes.data_as(ctypes.c_void_p)))
    return sig, inv


def iodf_query(ctx, what):
    v = ctypes.c_int64(0)
    _check(load_library().iodf_query(ctx, int(what), ctypes.byref(v)))
    return int(v.value)


def iodf_profile_begin(ctx, max_launches):
    _check(load_library().iodf_profile_begin(ctx, int(max_launches)))


def iodf_profile_end(ctx):
    """List of dicts, one per kernel that ran since iodf_profile_begin."""
    arr = (KernelStat * 32)()
    n = ctypes.c_int(0)
    _check(load_library().iodf_profile_end(ctx, arr, 32, ctypes.byref(n)))
    return [dict(name=arr[i].name.decode(), launches=int(arr[i].launches), total_ms=float(arr[i].total_ms),
                 macs=int(arr[i].macs), bytes=int(arr[i].bytes), issued_macs=int(arr[i].issued_macs))
            for i in range(n.value)]


def iodf_free(ctx):
    if ctx:
        load_library().iodf_free(ctx)


class Flow:
    """A model on one GPU. Tensors in and out are torch CUDA tensors."""

    def __init__(self, blob, max_batch, device=0):
        import torch
        self._torch = torch
        self.device = torch.device("cuda", device)
        self._ctx = iodf_init(blob, device, max_batch)
        self.max_batch = max_batch
        self.d = iodf_query(self._ctx, IODF_Q_Z_ELEMS)
        self.d_codes = iodf_query(self._ctx, IODF_Q_CODE_BYTES)
        self.H = iodf_query(self._ctx, IODF_Q_IMAGE_H)
        self.W = iodf_query(self._ctx, IODF_Q_IMAGE_W)

    def query(self, what):
        return iodf_query(self._ctx, what)

    def _stream(self):
        return ctypes.c_void_p(self._torch.cuda.current_stream(self.device).cuda_stream)

    def forward(self, x, want_codes=True, z=None, codes=None):
        torch = self._torch
        assert x.is_cuda and x.dtype == torch.uint8 and x.is_contiguous()
        b = x.shape[0]
        assert x.numel() == b * self.d
        if z is None:
            z = torch.empty((b, self.d), dtype=torch.int32, device=self.device)
        if want_codes and self.d_codes and codes is None:
            codes = torch.empty((b, self.d_codes), dtype=torch.int8, device=self.device)
        cp = ctypes.c_void_p(codes.data_ptr()) if (want_codes and codes is not None and b) else None
        iodf_forward(self._ctx, ctypes.c_void_p(x.data_ptr()) if b else None, b,
                     ctypes.c_void_p(z.data_ptr()) if b else None, cp, self._stream())
        return z, codes

    def inverse(self, z, x=None):
        torch = self._torch
        assert z.is_cuda and z.dtype == torch.int32 and z.is_contiguous()
        b = z.shape[0]
        if x is None:
            x = torch.empty((b, 3, self.H, self.W), dtype=torch.uint8, device=self.device)
        iodf_inverse(self._ctx, ctypes.c_void_p(z.data_ptr()) if b else None, b,
                     ctypes.c_void_p(x.data_ptr()) if b else None, self._stream())
        return x

    def prior_cf(self, z, codes=None):
        """Masses (C, F) of every latent under the prior the codes describe."""
        torch = self._torch
        assert z.is_cuda and z.dtype == torch.int32 and z.is_contiguous()
        b = z.shape[0]
        C = torch.empty((b, self.d), dtype=torch.int32, device=self.device)
        F = torch.empty((b, self.d), dtype=torch.int32, device=self.device)
        cp = ctypes.c_void_p(codes.data_ptr()) if (codes is not None and self.d_codes and b) else None
        iodf_prior_cf(self._ctx, ctypes.c_void_p(z.data_ptr()) if b else None, cp, b,
                      ctypes.c_void_p(C.data_ptr()) if b else None, ctypes.c_void_p(F.data_ptr()) if b else None,
                      self._stream())
        return C, F

    def encode(self, x, cap_words=None, words=None, sizes=None, noalloc=False):
        """x u8 [B,3,H,W] -> (containers int32-viewed-as-u32 [B,cap_words], sizes [B] in words).
        noalloc=True calls iodf_encode_noalloc (pass `words` and `sizes`: the call itself allocates nothing)."""
        torch = self._torch
        assert x.is_cuda and x.dtype == torch.uint8 and x.is_contiguous()
        b = x.shape[0]
        cap = int(cap_words or self.query(IODF_Q_CODEC_MAX_WORDS))
        if words is None:
            words = torch.zeros((b, cap), dtype=torch.int32, device=self.device)
        if sizes is None:
            sizes = torch.zeros((b,), dtype=torch.int32, device=self.device)
        (iodf_encode_noalloc if noalloc else iodf_encode)(self._ctx, ctypes.c_void_p(x.data_ptr()) if b else None, b,
                    ctypes.c_void_p(words.data_ptr()) if b else None, cap,
                    ctypes.c_void_p(sizes.data_ptr()) if b else None, self._stream())
        return words, sizes

    def decode(self, words, x=None):
        torch = self._torch
        assert words.is_cuda and words.dtype == torch.int32 and words.is_contiguous() and words.dim() == 2
        b, cap = words.shape
        if x is None:
            x = torch.empty((b, 3, self.H, self.W), dtype=torch.uint8, device=self.device)
        iodf_decode(self._ctx, ctypes.c_void_p(words.data_ptr()) if b else None, cap, b,
                    ctypes.c_void_p(x.data_ptr()) if b else None, self._stream())
        return x

    def n_patches(self, img_h, img_w):
        return -(-img_h // self.H) * -(-img_w // self.W)

    def tile_patches(self, img, first=0, n=None, x=None):
        """Planar image u8 [3,h,w] -> patches u8 [n,3,H,W] (row-major grid, 128 outside the image)."""
        torch = self._torch
        assert img.is_cuda and img.dtype == torch.uint8 and img.is_contiguous() and img.dim() == 3
        _, h, w = img.shape
        n = self.n_patches(h, w) - first if n is None else n
        if x is None:
            x = torch.empty((n, 3, self.H, self.W), dtype=torch.uint8, device=self.device)
        iodf_tile_patches(self._ctx, ctypes.c_void_p(img.data_ptr()), h, w, first, n,
                          ctypes.c_void_p(x.data_ptr()) if n else None, self._stream())
        return x

    def untile_patches(self, x, img, first=0):
        torch = self._torch
        assert x.is_cuda and x.dtype == torch.uint8 and x.is_contiguous()
        assert img.is_cuda and img.dtype == torch.uint8 and img.is_contiguous() and img.dim() == 3
        _, h, w = img.shape
        iodf_untile_patches(self._ctx, ctypes.c_void_p(x.data_ptr()) if x.shape[0] else None, first, x.shape[0],
                            ctypes.c_void_p(img.data_ptr()), h, w, self._stream())
        return img

    def encode_image(self, img):
        """Whole image -> list of (containers, sizes) per sub-batch of at most max_batch patches."""
        _, h, w = img.shape
        total, out = self.n_patches(h, w), []
        for first in range(0, total, self.max_batch):
            n = min(self.max_batch, total - first)
            out.append(self.encode(self.tile_patches(img, first, n)))
        return out

    def decode_image(self, parts, img_h, img_w):
        torch = self._torch
        img = torch.empty((3, img_h, img_w), dtype=torch.uint8, device=self.device)
        first = 0
        for words, _ in parts:
            self.untile_patches(self.decode(words), img, first)
            first += words.shape[0]
        return img

    def codec_errors(self):
        """(clamped residuals, overflowing containers, broken lanes) since the last call; synchronises."""
        return tuple(iodf_query(self._ctx, q) for q in (IODF_Q_CODEC_CLAMPED, IODF_Q_CODEC_OVERFLOWS,
                                                        IODF_Q_CODEC_BROKEN_LANES))

    def profile_begin(self, max_launches):
        iodf_profile_begin(self._ctx, max_launches)

    def profile_end(self):
        return iodf_profile_end(self._ctx)

    def range_errors(self):
        return iodf_query(self._ctx, IODF_Q_RANGE_ERRORS)

    def close(self):
        if getattr(self, "_ctx", None):
            iodf_free(self._ctx)
            self._ctx = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
