"""ctypes binding of the CPU oracle (libfadeo.so).

TEST INFRASTRUCTURE ONLY: imported by tests, by the smoke check and by the bench's cpu_baseline leg.
The product package never imports this module.
"""
import ctypes as C
import os

import numpy as np

from .buildlib import LIB, build

F32, BF16 = 0, 1
FROZEN, ONLINE_ADAM = 0, 1

TAPS = ["X", "CACHE", "H_GLOBAL", "H_LOCAL", "ALPHA", "H_MIX", "Y_DOWN", "Z_BMM", "H_A", "H_COARSE",
        "H_EXPAND", "H_OUT", "LOGITS", "PROBS"]


class Config(C.Structure):
    _fields_ = [("struct_size", C.c_uint32), ("abi_version", C.c_uint32),
                ("B", C.c_uint32), ("T", C.c_uint32), ("D", C.c_uint32), ("H", C.c_uint32),
                ("d_low", C.c_uint32), ("cache_chunk", C.c_uint32), ("conv_k", C.c_uint32),
                ("d_cache", C.c_uint32), ("d_e", C.c_uint32), ("ablation", C.c_uint32),
                ("dtype", C.c_uint32), ("update_mode", C.c_uint32),
                ("lr", C.c_float), ("beta1", C.c_float), ("beta2", C.c_float), ("eps", C.c_float),
                ("device", C.c_int32), ("hip_stream", C.c_void_p)]


def make_config(B, T, D, H, d_low=0, cache_chunk=0, conv_k=0, dtype=F32, update_mode=FROZEN,
                lr=0.0, beta1=0.0, beta2=0.0, eps=0.0, d_cache=0, d_e=0, ablation=0):
    c = Config()
    c.struct_size = C.sizeof(Config)
    c.abi_version = 2
    c.B, c.T, c.D, c.H = B, T, D, H
    c.d_low, c.cache_chunk, c.conv_k = d_low, cache_chunk, conv_k
    c.d_cache, c.d_e, c.ablation = d_cache, d_e, ablation
    c.dtype, c.update_mode = dtype, update_mode
    c.lr, c.beta1, c.beta2, c.eps = lr, beta1, beta2, eps
    c.device, c.hip_stream = 0, None
    return c


_lib = None


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(LIB):
            build()
        L = C.CDLL(LIB)
        vp, u8p = C.c_void_p, C.c_void_p
        L.fadeo_weights_nbytes.restype = C.c_size_t
        L.fadeo_weights_nbytes.argtypes = [C.POINTER(Config)]
        L.fadeo_create.argtypes = [C.POINTER(Config), C.POINTER(vp)]
        L.fadeo_load_weights.argtypes = [vp, vp, C.c_size_t]
        L.fadeo_reset.argtypes = [vp]
        L.fadeo_step_probs.argtypes = [vp, u8p, u8p, vp, vp]
        L.fadeo_loss.argtypes = [vp, u8p, u8p, C.POINTER(C.c_double)]
        L.fadeo_backward.argtypes = [vp, u8p, u8p, vp]
        L.fadeo_step_update.argtypes = [vp, u8p, u8p]
        L.fadeo_get_weights.argtypes = [vp, vp, C.c_size_t]
        L.fadeo_tap.restype = C.c_size_t
        L.fadeo_tap.argtypes = [vp, C.c_int, C.c_uint32, vp, C.c_size_t]
        L.fadeo_encode_bound.restype = C.c_size_t
        L.fadeo_encode_bound.argtypes = [vp, C.c_size_t]
        L.fadeo_encode.argtypes = [vp, u8p, C.c_size_t, u8p, C.c_size_t, C.POINTER(C.c_size_t)]
        L.fadeo_decode.argtypes = [vp, u8p, C.c_size_t, u8p, C.c_size_t, C.POINTER(C.c_size_t)]
        L.fadeo_last_code_stats.argtypes = [vp, C.POINTER(C.c_double), C.POINTER(C.c_double),
                                            C.POINTER(C.c_uint64)]
        L.fadeo_quantize.argtypes = [vp, C.c_size_t, vp]
        L.fadeo_coder_encode.argtypes = [vp, u8p, C.c_size_t, u8p, C.c_size_t, C.POINTER(C.c_size_t)]
        L.fadeo_coder_decode.argtypes = [vp, C.c_size_t, u8p, C.c_size_t, u8p]
        L.fadeo_fnv1a64.restype = C.c_uint64
        L.fadeo_fnv1a64.argtypes = [vp, C.c_size_t]
        L.fadeo_last_error.restype = C.c_char_p
        L.fadeo_last_error.argtypes = [vp]
        L.fadeo_destroy.argtypes = [vp]
        _lib = L
    return _lib


class OracleError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__(f"oracle error {code}: {msg}")
        self.code = code


def _p(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _u8(a):
    if a is None:
        return None
    a = np.ascontiguousarray(a, dtype=np.uint8)
    return a


class Oracle:
    """One oracle context. All arrays are host numpy arrays."""

    def __init__(self, cfg: Config):
        self.cfg = cfg
        self.L = lib()
        h = C.c_void_p()
        rc = self.L.fadeo_create(C.byref(cfg), C.byref(h))
        if rc:
            raise OracleError(rc, "create")
        self.h = h
        self.B, self.T = cfg.B, cfg.T
        self.nparams = self.L.fadeo_weights_nbytes(C.byref(cfg)) // 4

    def _chk(self, rc):
        if rc:
            raise OracleError(rc, self.L.fadeo_last_error(self.h).decode())

    def close(self):
        if self.h:
            self.L.fadeo_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def load_weights(self, blob):
        blob = np.ascontiguousarray(blob, dtype=np.float32)
        self._chk(self.L.fadeo_load_weights(self.h, _p(blob), blob.nbytes))

    def reset(self):
        self._chk(self.L.fadeo_reset(self.h))

    def step_probs(self, windows, active=None, want_freq=True, want_probs=True):
        w = _u8(windows).reshape(self.B, self.T)
        a = _u8(active)
        freq = np.zeros((self.B, 256), np.uint16) if want_freq else None
        probs = np.zeros((self.B, 256), np.float32) if want_probs else None
        self._chk(self.L.fadeo_step_probs(self.h, _p(w), _p(a), _p(freq), _p(probs)))
        return freq, probs

    def loss(self, targets, active=None):
        out = C.c_double()
        t, a = _u8(targets), _u8(active)
        self._chk(self.L.fadeo_loss(self.h, _p(t), _p(a), C.byref(out)))
        return out.value

    def backward(self, targets, active=None):
        g = np.zeros(self.nparams, np.float64)
        t, a = _u8(targets), _u8(active)
        self._chk(self.L.fadeo_backward(self.h, _p(t), _p(a), _p(g)))
        return g

    def step_update(self, targets, active=None):
        t, a = _u8(targets), _u8(active)
        self._chk(self.L.fadeo_step_update(self.h, _p(t), _p(a)))

    def get_weights(self):
        w = np.zeros(self.nparams, np.float32)
        self._chk(self.L.fadeo_get_weights(self.h, _p(w), w.nbytes))
        return w

    def tap(self, name, stream):
        which = TAPS.index(name)
        n = self.L.fadeo_tap(self.h, which, stream, None, 0)
        out = np.zeros(n, np.float64)
        self.L.fadeo_tap(self.h, which, stream, _p(out), n)
        return out

    def encode_bound(self, n):
        return self.L.fadeo_encode_bound(self.h, n)

    def encode(self, src):
        src = _u8(src)
        cap = self.encode_bound(src.size)
        dst = np.zeros(cap, np.uint8)
        n = C.c_size_t()
        self._chk(self.L.fadeo_encode(self.h, _p(src), src.size, _p(dst), cap, C.byref(n)))
        return dst[:n.value].copy()

    def decode(self, blob, cap):
        blob = _u8(blob)
        dst = np.zeros(max(cap, 1), np.uint8)
        n = C.c_size_t()
        self._chk(self.L.fadeo_decode(self.h, _p(blob), blob.size, _p(dst), cap, C.byref(n)))
        return dst[:n.value].copy()

    def code_stats(self):
        bf, bp, st = C.c_double(), C.c_double(), C.c_uint64()
        self._chk(self.L.fadeo_last_code_stats(self.h, C.byref(bf), C.byref(bp), C.byref(st)))
        return bf.value, bp.value, st.value


def quantize(p):
    p = np.ascontiguousarray(p, dtype=np.float32).reshape(-1, 256)
    f = np.zeros(p.shape, np.uint16)
    rc = lib().fadeo_quantize(_p(p), p.shape[0], _p(f))
    if rc:
        raise OracleError(rc, "quantize")
    return f


def coder_encode(freq, sym):
    freq = np.ascontiguousarray(freq, dtype=np.uint16).reshape(-1, 256)
    sym = _u8(sym)
    n = sym.size
    cap = 2 * n + 16
    out = np.zeros(cap, np.uint8)
    ln = C.c_size_t()
    rc = lib().fadeo_coder_encode(_p(freq), _p(sym), n, _p(out), cap, C.byref(ln))
    if rc:
        raise OracleError(rc, "coder_encode")
    return out[:ln.value].copy()


def coder_decode(freq, n, data):
    freq = np.ascontiguousarray(freq, dtype=np.uint16).reshape(-1, 256)
    data = _u8(data)
    sym = np.zeros(max(n, 1), np.uint8)
    rc = lib().fadeo_coder_decode(_p(freq), n, _p(data), data.size, _p(sym))
    if rc:
        raise OracleError(rc, "coder_decode")
    return sym[:n].copy()


def fnv1a64(data):
    data = _u8(data)
    return lib().fadeo_fnv1a64(_p(data), data.size)
