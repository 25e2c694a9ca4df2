"""ctypes binding of the CPU oracle (test infrastructure; see iodf_oracle.h).

Only tests, the smoke check and the benchmark's CPU-baseline leg may import this.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB = None


def build(force=False):
    """Compile liboracle.so with gcc (make)."""
    if force:
        subprocess.check_call(["make", "-s", "-C", _HERE, "clean"])
    subprocess.check_call(["make", "-s", "-C", _HERE])
    return os.path.join(_HERE, "liboracle.so")


def lib():
    global _LIB
    if _LIB is None:
        path = os.path.join(_HERE, "liboracle.so")
        srcs = [os.path.join(_HERE, f) for f in ("iodf_oracle.c", "iodf_oracle.h", "iodf_codec_oracle.c",
                                                 "iodf_codec_oracle.h")]
        if not os.path.exists(path) or os.path.getmtime(path) < max(os.path.getmtime(f) for f in srcs):
            build()
        L = ctypes.CDLL(path)
        vp, i32, i64, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_size_t
        ci = ctypes.c_int
        L.orc_rq.restype = i64
        L.orc_rq.argtypes = [i32, i32, ci]
        L.orc_sat8.restype = i32
        L.orc_sat8.argtypes = [i64]
        L.orc_set_threads.argtypes = [ci]
        L.orc_get_threads.restype = ci
        L.orc_conv_acc.restype = None
        L.orc_conv_acc.argtypes = [vp, ci, ci, ci, vp, ci, ci, vp, vp, vp]
        L.orc_epilogue.restype = None
        L.orc_epilogue.argtypes = [vp, ci, ci, vp, vp, vp, ci, vp, vp]
        L.orc_conv_acc_u8.restype = None
        L.orc_conv_acc_u8.argtypes = [vp, ci, ci, ci, vp, ci, ci, vp, vp, vp]
        L.orc_epilogue_u8.restype = None
        L.orc_epilogue_u8.argtypes = [vp, ci, ci, vp, vp, vp, vp, vp]
        L.orc_squeeze.restype = None
        L.orc_squeeze.argtypes = [vp, ci, ci, ci, vp]
        L.orc_unsqueeze.restype = None
        L.orc_unsqueeze.argtypes = [vp, ci, ci, ci, vp]
        L.orc_model_load.restype = ci
        L.orc_model_load.argtypes = [vp, sz, ctypes.POINTER(vp)]
        L.orc_model_free.restype = None
        L.orc_model_free.argtypes = [vp]
        L.orc_model_num_nets.restype = ci
        L.orc_model_num_nets.argtypes = [vp]
        L.orc_model_d.restype = i64
        L.orc_model_d.argtypes = [vp]
        L.orc_model_d_codes.restype = i64
        L.orc_model_d_codes.argtypes = [vp]
        L.orc_net_eval.restype = ci
        L.orc_net_eval.argtypes = [vp, ci, vp, ci, ci, vp]
        L.orc_forward.restype = ci
        L.orc_forward.argtypes = [vp, vp, ci, vp, vp]
        L.orc_inverse.restype = ci
        L.orc_inverse.argtypes = [vp, vp, ci, vp, ctypes.POINTER(i64)]
        L.orc_last_max_abs_state.restype = i64
        u32, u64 = ctypes.c_uint32, ctypes.c_uint64
        L.orc_prior_tables.restype = None
        L.orc_prior_tables.argtypes = [vp, vp]
        L.orc_prior_sigmoid.restype = i64
        L.orc_prior_sigmoid.argtypes = [i64]
        L.orc_prior_cdf.restype = i64
        L.orc_prior_cdf.argtypes = [ci, ci]
        L.orc_prior_cf.restype = i64
        L.orc_prior_cf.argtypes = [vp, vp, vp, i64, vp, vp]
        L.orc_rans_push.restype = u64
        L.orc_rans_push.argtypes = [u64, u32, u32, ctypes.POINTER(ci), ctypes.POINTER(u32)]
        L.orc_rans_pop.restype = u64
        L.orc_rans_pop.argtypes = [u64, u32, u32]
        L.orc_codec_header_words.restype = i64
        L.orc_codec_header_words.argtypes = [ci]
        L.orc_codec_encode_image.restype = i64
        L.orc_codec_encode_image.argtypes = [vp, vp, ci, vp, vp, vp, vp, i64, ctypes.POINTER(i64)]
        L.orc_codec_decode_chunk.restype = ci
        L.orc_codec_decode_chunk.argtypes = [vp, i64, ci, vp, ci, vp, vp, vp]
        L.orc_codec_max_words.restype = i64
        L.orc_codec_max_words.argtypes = [vp]
        L.orc_encode.restype = ci
        L.orc_encode.argtypes = [vp, vp, ci, vp, i64, vp, ctypes.POINTER(i64)]
        L.orc_decode.restype = ci
        L.orc_decode.argtypes = [vp, vp, i64, ci, vp, ctypes.POINTER(i64)]
        _LIB = L
    return _LIB


def _p(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def rq(a, M, s):
    return int(lib().orc_rq(int(a), int(M), int(s)))


def sat8(u):
    return int(lib().orc_sat8(int(u)))


def set_threads(n):
    lib().orc_set_threads(int(n))


def get_threads():
    return int(lib().orc_get_threads())


def conv_acc(x, W, bias=None, gate=None):
    """x int8 [D,h,w], W int8 [C,D,k,k] -> int32 accumulators [C,h,w] (Eq. 4)."""
    x = np.ascontiguousarray(x, dtype=np.int8)
    W = np.ascontiguousarray(W, dtype=np.int8)
    D, h, w = x.shape
    C, D2, k, k2 = W.shape
    assert D == D2 and k == k2
    bias = None if bias is None else np.ascontiguousarray(bias, dtype=np.int32)
    gate = None if gate is None else np.ascontiguousarray(gate, dtype=np.uint8)
    acc = np.zeros((C, h, w), dtype=np.int32)
    lib().orc_conv_acc(_p(x), D, h, w, _p(W), C, k, _p(bias), _p(gate), _p(acc))
    return acc


def conv_acc_u8(x, W, bias=None, gate=None):
    """As conv_acc with x uint8 [D,h,w] read as unsigned codes."""
    x = np.ascontiguousarray(x, dtype=np.uint8)
    W = np.ascontiguousarray(W, dtype=np.int8)
    D, h, w = x.shape
    C, D2, k, k2 = W.shape
    assert D == D2 and k == k2
    bias = None if bias is None else np.ascontiguousarray(bias, dtype=np.int32)
    gate = None if gate is None else np.ascontiguousarray(gate, dtype=np.uint8)
    acc = np.zeros((C, h, w), dtype=np.int32)
    lib().orc_conv_acc_u8(_p(x), D, h, w, _p(W), C, k, _p(bias), _p(gate), _p(acc))
    return acc


def epilogue_u8(acc, M, shift, gate=None, shortcut=None):
    """Unsigned-format epilogue (always with ReLU): uint8 codes saturated to [0, 255]."""
    acc = np.ascontiguousarray(acc, dtype=np.int32)
    C = acc.shape[0]
    hw = int(np.prod(acc.shape[1:]))
    M = np.ascontiguousarray(M, dtype=np.int32)
    shift = np.ascontiguousarray(shift, dtype=np.uint8)
    gate = None if gate is None else np.ascontiguousarray(gate, dtype=np.uint8)
    shortcut = None if shortcut is None else np.ascontiguousarray(shortcut, dtype=np.uint8)
    y = np.zeros(acc.shape, dtype=np.uint8)
    lib().orc_epilogue_u8(_p(acc), C, hw, _p(M), _p(shift), _p(gate), _p(shortcut), _p(y))
    return y


def epilogue(acc, M, shift, gate=None, relu=False, shortcut=None):
    acc = np.ascontiguousarray(acc, dtype=np.int32)
    C = acc.shape[0]
    hw = int(np.prod(acc.shape[1:]))
    M = np.ascontiguousarray(M, dtype=np.int32)
    shift = np.ascontiguousarray(shift, dtype=np.uint8)
    gate = None if gate is None else np.ascontiguousarray(gate, dtype=np.uint8)
    shortcut = None if shortcut is None else np.ascontiguousarray(shortcut, dtype=np.int8)
    y = np.zeros(acc.shape, dtype=np.int8)
    lib().orc_epilogue(_p(acc), C, hw, _p(M), _p(shift), _p(gate), int(relu), _p(shortcut), _p(y))
    return y


def squeeze(a):
    a = np.ascontiguousarray(a, dtype=np.int32)
    C, H, W = a.shape
    out = np.zeros((4 * C, H // 2, W // 2), dtype=np.int32)
    lib().orc_squeeze(_p(a), C, H, W, _p(out))
    return out


def unsqueeze(a):
    a = np.ascontiguousarray(a, dtype=np.int32)
    C4, h, w = a.shape
    out = np.zeros((C4 // 4, 2 * h, 2 * w), dtype=np.int32)
    lib().orc_unsqueeze(_p(a), C4 // 4, 2 * h, 2 * w, _p(out))
    return out


class Model:
    """A loaded model blob."""

    _h = None

    def __init__(self, blob):
        blob = np.ascontiguousarray(blob, dtype=np.uint8)
        h = ctypes.c_void_p()
        rc = lib().orc_model_load(_p(blob), blob.size, ctypes.byref(h))
        if rc != 0:
            raise ValueError("oracle: bad model blob (code %d)" % rc)
        self._h = h
        self.d = int(lib().orc_model_d(h))
        self.d_codes = int(lib().orc_model_d_codes(h))
        self.n_nets = int(lib().orc_model_num_nets(h))

    def close(self):
        if self._h:
            lib().orc_model_free(self._h)
            self._h = None

    def __del__(self):
        self.close()

    def net_eval(self, net, xa, c_out):
        xa = np.ascontiguousarray(xa, dtype=np.int32)
        _, h, w = xa.shape
        out = np.zeros((c_out, h, w), dtype=np.int8)
        rc = lib().orc_net_eval(self._h, net, _p(xa), h, w, _p(out))
        if rc != 0:
            raise RuntimeError("oracle net_eval failed (%d)" % rc)
        return out

    def forward(self, x):
        x = np.ascontiguousarray(x, dtype=np.uint8)
        b = x.shape[0]
        assert x.size == b * self.d
        z = np.zeros((b, self.d), dtype=np.int32)
        codes = np.zeros((b, self.d_codes), dtype=np.int8)
        rc = lib().orc_forward(self._h, _p(x), b, _p(z), _p(codes) if self.d_codes else None)
        if rc != 0:
            raise RuntimeError("oracle forward failed (%d)" % rc)
        return z, codes

    def inverse(self, z, shape):
        z = np.ascontiguousarray(z, dtype=np.int32)
        b = z.shape[0]
        x = np.zeros((b,) + tuple(shape), dtype=np.uint8)
        errs = ctypes.c_int64(0)
        rc = lib().orc_inverse(self._h, _p(z), b, _p(x), ctypes.byref(errs))
        if rc != 0:
            raise RuntimeError("oracle inverse failed (%d)" % rc)
        return x, int(errs.value)

    def codec_max_words(self):
        return int(lib().orc_codec_max_words(self._h))

    def encode(self, x, cap=None):
        """x u8 [B,3,H,W] -> (containers uint32 [B,cap], sizes uint32 [B], clamped count)."""
        x = np.ascontiguousarray(x, dtype=np.uint8)
        cap = int(cap or self.codec_max_words())
        out = np.zeros((x.shape[0], cap), np.uint32)
        sizes = np.zeros(x.shape[0], np.uint32)
        cl = ctypes.c_int64(0)
        rc = lib().orc_encode(self._h, _p(x), x.shape[0], _p(out), cap, _p(sizes), ctypes.byref(cl))
        if rc:
            raise RuntimeError("orc_encode failed: %d" % rc)
        return out, sizes, int(cl.value)

    def decode(self, cont, shape):
        """containers uint32 [B,cap] -> (x u8 [B,*shape], error count)."""
        cont = np.ascontiguousarray(cont, dtype=np.uint32)
        x = np.zeros((cont.shape[0],) + tuple(shape), np.uint8)
        errs = ctypes.c_int64(0)
        rc = lib().orc_decode(self._h, _p(cont), cont.shape[1], cont.shape[0], _p(x), ctypes.byref(errs))
        if rc:
            raise RuntimeError("orc_decode failed: %d" % rc)
        return x, int(errs.value)

    @staticmethod
    def last_max_abs_state():
        return int(lib().orc_last_max_abs_state())


# ---- entropy-coding side (iodf_codec_oracle.h) ----
MASS_BITS, ALPHA_R, SIG_BITS, LANES = 24, 8192, 30, 16


def prior_tables():
    sig = np.empty(3073, np.int32)
    inv = np.empty(256, np.int64)
    lib().orc_prior_tables(_p(sig), _p(inv))
    return sig, inv


def prior_sigmoid(T):
    return int(lib().orc_prior_sigmoid(int(T)))


def prior_cdf(r, l):
    return int(lib().orc_prior_cdf(int(r), int(l)))


def prior_cf(z, m=None, l=None):
    """Masses (C, F) of latents z with mean codes m and log-scale codes l (None: defaults)."""
    z = np.ascontiguousarray(z, np.int32).ravel()
    m = None if m is None else np.ascontiguousarray(m, np.int8).ravel()
    l = None if l is None else np.ascontiguousarray(l, np.int8).ravel()
    C = np.empty(z.size, np.int32)
    F = np.empty(z.size, np.int32)
    clamped = lib().orc_prior_cf(_p(z), _p(m), _p(l), z.size, _p(C), _p(F))
    return C, F, int(clamped)


def rans_push(X, C, F):
    """One encoder update; returns (new state, shed word or None)."""
    e, w = ctypes.c_int(0), ctypes.c_uint32(0)
    X2 = lib().orc_rans_push(int(X), int(C), int(F), ctypes.byref(e), ctypes.byref(w))
    return int(X2), (int(w.value) if e.value else None)


def rans_pop(X, C, F):
    return int(lib().orc_rans_pop(int(X), int(C), int(F)))


def codec_header_words(n_chunks):
    return int(lib().orc_codec_header_words(int(n_chunks)))


def codec_encode_image(z, codes, n, z_off, code_off, cap):
    z = np.ascontiguousarray(z, np.int32)
    codes = None if codes is None else np.ascontiguousarray(codes, np.int8)
    n = np.ascontiguousarray(n, np.int64)
    z_off = np.ascontiguousarray(z_off, np.int64)
    code_off = np.ascontiguousarray(code_off, np.int64)
    out = np.zeros(int(cap), np.uint32)
    cl = ctypes.c_int64(0)
    w = lib().orc_codec_encode_image(_p(z), _p(codes), n.size, _p(n), _p(z_off), _p(code_off), _p(out), int(cap),
                                     ctypes.byref(cl))
    return out, int(w), int(cl.value)


def codec_decode_chunk(cont, n, c, m=None, l=None):
    cont = np.ascontiguousarray(cont, np.uint32)
    n = np.ascontiguousarray(n, np.int64)
    m = None if m is None else np.ascontiguousarray(m, np.int8)
    l = None if l is None else np.ascontiguousarray(l, np.int8)
    zc = np.zeros(int(n[c]), np.int32)
    rc = lib().orc_codec_decode_chunk(_p(cont), cont.size, n.size, _p(n), int(c), _p(m), _p(l), _p(zc))
    return zc, int(rc)


# ---- patch-based coding of a large image (Sec. 5.2) ----

def tile_patches(img, H, W, pad=128):
    """Planar image [3,h,w] -> patches [n,3,H,W] of the row-major grid ceil(h/H) x ceil(w/W);
    pixels outside the image are `pad`. Plain loops: this is the definition."""
    img = np.asarray(img, np.uint8)
    _, h, w = img.shape
    ph, pw = -(-h // H), -(-w // W)
    out = np.full((ph * pw, 3, H, W), pad, np.uint8)
    for py in range(ph):
        for px in range(pw):
            y0, x0 = py * H, px * W
            y1, x1 = min(h, y0 + H), min(w, x0 + W)
            out[py * pw + px, :, :y1 - y0, :x1 - x0] = img[:, y0:y1, x0:x1]
    return out


def untile_patches(patches, h, w):
    patches = np.asarray(patches, np.uint8)
    n, _, H, W = patches.shape
    ph, pw = -(-h // H), -(-w // W)
    assert n == ph * pw
    img = np.zeros((3, h, w), np.uint8)
    for py in range(ph):
        for px in range(pw):
            y0, x0 = py * H, px * W
            y1, x1 = min(h, y0 + H), min(w, x0 + W)
            img[:, y0:y1, x0:x1] = patches[py * pw + px, :, :y1 - y0, :x1 - x0]
    return img
