"""ctypes marshalling for libfade.so (names mirror include/fade.h). Device buffers are torch tensors on the
context's device; host buffers are numpy arrays."""
import ctypes as C
import os

import numpy as np

from .buildlib import LIB

F32, BF16 = 0, 1
FROZEN, ONLINE_ADAM = 0, 1
ABI_VERSION = 2
TAPS = ["X", "CACHE", "H_GLOBAL", "H_LOCAL", "ALPHA", "H_MIX", "Y_DOWN", "Z_BMM", "H_A", "H_COARSE", "H_EXPAND",
        "H_OUT", "LOGITS", "PROBS"]


class Config(C.Structure):
    _fields_ = [("struct_size", C.c_uint32), ("abi_version", C.c_uint32),
                ("B", C.c_uint32), ("T", C.c_uint32), ("D", C.c_uint32), ("H", C.c_uint32),
                ("d_low", C.c_uint32), ("cache_chunk", C.c_uint32), ("conv_k", C.c_uint32),
                ("d_cache", C.c_uint32), ("d_e", C.c_uint32), ("ablation", C.c_uint32),
                ("dtype", C.c_uint32), ("update_mode", C.c_uint32),
                ("lr", C.c_float), ("beta1", C.c_float), ("beta2", C.c_float), ("eps", C.c_float),
                ("device", C.c_int32), ("hip_stream", C.c_void_p)]


def make_config(B, T, D, H, d_low=0, cache_chunk=0, conv_k=0, dtype=BF16, update_mode=FROZEN, lr=0.0, beta1=0.0,
                beta2=0.0, eps=0.0, device=0, hip_stream=None, d_cache=0, d_e=0, ablation=0):
    c = Config()
    c.struct_size = C.sizeof(Config)
    c.abi_version = ABI_VERSION
    c.B, c.T, c.D, c.H = B, T, D, H
    c.d_low, c.cache_chunk, c.conv_k = d_low, cache_chunk, conv_k
    c.d_cache, c.d_e, c.ablation = d_cache, d_e, ablation
    c.dtype, c.update_mode = dtype, update_mode
    c.lr, c.beta1, c.beta2, c.eps = lr, beta1, beta2, eps
    c.device, c.hip_stream = device, hip_stream
    return c


_lib = None


def lib():
    """Load libfade.so. Fails loudly when it has not been built (python -m paper_2604_07239_amd.buildlib)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB):
            raise FadeError(-7, f"{LIB} is not built: run paper_2604_07239_amd.build() (hipcc, gfx950) first")
        L = C.CDLL(LIB)
        vp, sz = C.c_void_p, C.c_size_t
        L.fade_weights_nbytes.restype = sz
        L.fade_weights_nbytes.argtypes = [C.POINTER(Config)]
        L.fade_create.argtypes = [C.POINTER(Config), C.POINTER(vp)]
        L.fade_load_weights.argtypes = [vp, vp, sz]
        L.fade_reset.argtypes = [vp]
        L.fade_step_probs.argtypes = [vp, vp, vp, vp, vp]
        L.fade_step_update.argtypes = [vp, vp, vp]
        L.fade_encode_bound.restype = sz
        L.fade_encode_bound.argtypes = [vp, sz]
        L.fade_encode.argtypes = [vp, vp, sz, vp, sz, C.POINTER(sz)]
        L.fade_decode.argtypes = [vp, vp, sz, vp, sz, C.POINTER(sz)]
        L.fade_encode_device.argtypes = [vp, vp, sz, sz, sz]
        L.fade_payloads.argtypes = [vp, vp, vp, sz, C.POINTER(sz)]
        L.fade_decode_device.argtypes = [vp, vp, vp, sz, vp, sz, sz, sz]
        L.fade_quantize.argtypes = [vp, vp, sz, vp]
        L.fade_coder_encode_tables.argtypes = [vp, vp, vp, sz, sz, vp, sz, vp]
        L.fade_coder_decode_tables.argtypes = [vp, vp, sz, sz, vp, sz, vp, vp]
        L.fade_coder_encode_tables_noalloc.argtypes = [vp, vp, vp, sz, sz, vp, sz, vp]
        L.fade_tap.restype = sz
        L.fade_tap.argtypes = [vp, C.c_int, vp, sz]
        L.fade_get_weights.argtypes = [vp, vp, sz]
        L.fade_debug_grad.argtypes = [vp, vp, sz]
        L.fade_profile.argtypes = [vp, C.c_int]
        L.fade_profile_read.argtypes = [vp, C.POINTER(C.c_char_p), C.POINTER(C.c_double), C.POINTER(C.c_uint64), C.c_int]
        L.fade_last_error.restype = C.c_char_p
        L.fade_last_error.argtypes = [vp]
        L.fade_destroy.argtypes = [vp]
        _lib = L
    return _lib


class FadeError(RuntimeError):
    def __init__(self, code, msg=""):
        super().__init__(f"libfade error {code}: {msg}")
        self.code = code


def weights_nbytes(cfg):
    return lib().fade_weights_nbytes(C.byref(cfg))


def _hp(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _dp(t):
    return None if t is None else C.c_void_p(t.data_ptr())


class Fade:
    """One libfade context (see include/fade.h for the meaning of every call)."""

    def __init__(self, cfg):
        self.cfg = cfg
        self.L = lib()
        h = C.c_void_p()
        rc = self.L.fade_create(C.byref(cfg), C.byref(h))
        if rc:
            raise FadeError(rc, "fade_create")
        self.h = h
        self.B, self.T = cfg.B, cfg.T

    def _chk(self, rc):
        if rc:
            raise FadeError(rc, self.L.fade_last_error(self.h).decode())

    def close(self):
        if getattr(self, "h", None):
            self.L.fade_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # -- weights / state -------------------------------------------------------------------------
    def load_weights(self, blob):
        blob = np.ascontiguousarray(blob, dtype=np.float32)
        self._chk(self.L.fade_load_weights(self.h, _hp(blob), blob.nbytes))

    def reset(self):
        self._chk(self.L.fade_reset(self.h))

    def get_weights(self):
        n = weights_nbytes(self.cfg)
        out = np.zeros(n // 4, np.float32)
        self._chk(self.L.fade_get_weights(self.h, _hp(out), n))
        return out

    def debug_grad(self):
        n = weights_nbytes(self.cfg)
        out = np.zeros(n // 4, np.float32)
        self._chk(self.L.fade_debug_grad(self.h, _hp(out), n))
        return out

    # -- the step --------------------------------------------------------------------------------
    def step_probs(self, windows_dev, active_dev=None, freq_dev=None, probs_dev=None):
        self._chk(self.L.fade_step_probs(self.h, _dp(windows_dev), _dp(active_dev), _dp(freq_dev), _dp(probs_dev)))

    def step_update(self, targets_dev, active_dev=None):
        self._chk(self.L.fade_step_update(self.h, _dp(targets_dev), _dp(active_dev)))

    def tap(self, name):
        which = TAPS.index(name)
        width = self.L.fade_tap(self.h, which, None, 0)
        if width == 0:
            return None
        out = np.zeros((self.B, width), np.float32)
        if self.L.fade_tap(self.h, which, _hp(out), out.size) != width:
            raise FadeError(-7, "fade_tap")
        return out

    # -- compress / decompress -------------------------------------------------------------------
    def encode_bound(self, n):
        return self.L.fade_encode_bound(self.h, n)

    def encode(self, src):
        src = np.ascontiguousarray(src, dtype=np.uint8)
        cap = self.encode_bound(src.size)
        dst = np.zeros(cap, np.uint8)
        n = C.c_size_t()
        self._chk(self.L.fade_encode(self.h, _hp(src), src.size, _hp(dst), cap, C.byref(n)))
        return dst[:n.value].copy()

    def decode(self, blob, cap):
        blob = np.ascontiguousarray(blob, dtype=np.uint8)
        dst = np.zeros(max(cap, 1), np.uint8)
        n = C.c_size_t()
        self._chk(self.L.fade_decode(self.h, _hp(blob), blob.size, _hp(dst), cap, C.byref(n)))
        return dst[:n.value].copy()

    def encode_device(self, src_dev, n, first_step=0, n_steps=0):
        self._chk(self.L.fade_encode_device(self.h, _dp(src_dev), n, first_step, n_steps))

    def payloads(self):
        lens = np.zeros(self.B, np.uint32)
        total = C.c_size_t()
        rc = self.L.fade_payloads(self.h, _hp(lens), None, 0, C.byref(total))
        if rc not in (0, -5):
            self._chk(rc)
        data = np.zeros(max(total.value, 1), np.uint8)
        self._chk(self.L.fade_payloads(self.h, _hp(lens), _hp(data), data.size, C.byref(total)))
        return lens, data[:total.value]

    def decode_device(self, lens, data, dst_dev, n, first_step=0, n_steps=0):
        if first_step == 0:
            lens = np.ascontiguousarray(lens, dtype=np.uint32)
            data = np.ascontiguousarray(data, dtype=np.uint8)
            self._chk(self.L.fade_decode_device(self.h, _hp(lens), _hp(data) if data.size else None, data.size,
                                                _dp(dst_dev), n, 0, n_steps))
        else:
            self._chk(self.L.fade_decode_device(self.h, None, None, 0, _dp(dst_dev), n, first_step, n_steps))

    # -- stand-alone integer kernels -------------------------------------------------------------
    def quantize(self, probs_dev, freq_dev):
        rows = probs_dev.numel() // 256
        self._chk(self.L.fade_quantize(self.h, _dp(probs_dev), rows, _dp(freq_dev)))

    def coder_encode_tables(self, freq_dev, sym_dev, n_steps, n_streams, out_dev, cap, len_dev):
        self._chk(self.L.fade_coder_encode_tables(self.h, _dp(freq_dev), _dp(sym_dev), n_steps, n_streams, _dp(out_dev), cap, _dp(len_dev)))

    def coder_encode_tables_noalloc(self, freq_dev, sym_dev, n_steps, n_streams, out_dev, cap, len_dev):
        self._chk(self.L.fade_coder_encode_tables_noalloc(self.h, _dp(freq_dev), _dp(sym_dev), n_steps, n_streams, _dp(out_dev), cap, _dp(len_dev)))

    def coder_decode_tables(self, freq_dev, n_steps, n_streams, in_dev, cap, len_dev, sym_dev):
        self._chk(self.L.fade_coder_decode_tables(self.h, _dp(freq_dev), n_steps, n_streams, _dp(in_dev), cap, _dp(len_dev), _dp(sym_dev)))

    # -- profiling -------------------------------------------------------------------------------
    def profile(self, enable):
        self._chk(self.L.fade_profile(self.h, 1 if enable else 0))

    def profile_read(self):
        cap = 64
        names = (C.c_char_p * cap)()
        ms = (C.c_double * cap)()
        cnt = (C.c_uint64 * cap)()
        n = self.L.fade_profile_read(self.h, names, ms, cnt, cap)
        return {names[i].decode(): (ms[i], cnt[i]) for i in range(n)}
