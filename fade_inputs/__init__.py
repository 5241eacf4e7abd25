"""Seeded synthetic inputs shared by tests, bench and the oracle timing: byte streams of the benchmark
configurations and random-init weight blobs. Holds none of the method's arithmetic.

The weight blob is the canonical fp32 layout both libraries accept (an interface, so it is stated here
once more, in the harness's own words): tensors in the order of `tensor_specs`, every matrix row-major
[in][out] so that y = x @ W.
"""
import ctypes as C
import os
import subprocess
from collections import OrderedDict

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
SANITIZE = os.environ.get("FADE_HOST_SANITIZE") == "1"   # separate ASan + UBSan build of the generators (see oracle/buildlib.py)
LIB = os.path.join(HERE, "libfadegen_san.so" if SANITIZE else "libfadegen.so")
SEED_BASE = 0xFADE0000

# name -> (B, T, D, H, dtype, bytes, generator) of the five benchmark configurations, and 6: the model shape the paper
# adopts as its default (Cache_dim = 4096, FNR_dim = 8192 at a 16-byte window) on a 256 MiB text-like input
CONFIGS = OrderedDict([
    (1, dict(B=16, T=32, D=16, H=128, dtype="f32", nbytes=1 << 20, source="markov2")),
    (2, dict(B=1024, T=64, D=32, H=256, dtype="bf16", nbytes=64 << 20, source="text")),
    (3, dict(B=4096, T=64, D=32, H=256, dtype="bf16", nbytes=256 << 20, source="genome")),
    (4, dict(B=4096, T=64, D=32, H=256, dtype="bf16", nbytes=256 << 20, source="float")),
    (5, dict(B=16384, T=64, D=32, H=512, dtype="bf16", nbytes=1 << 30, source="mixed")),
    (6, dict(B=4096, T=16, D=32, H=8192, d_cache=4096, d_e=8192, dtype="bf16", nbytes=256 << 20, source="text")),
])


def build(force: bool = True) -> str:
    src = os.path.join(HERE, "gen.c")
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= os.path.getmtime(src):
        return LIB
    san = ["-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined"] if SANITIZE else []
    subprocess.run(["gcc", "-O2", *san, "-fPIC", "-shared", "-Wall", "-o", LIB, src, "-lm"], check=True)
    return LIB


_lib = None


def _l():
    global _lib
    if _lib is None:
        if not os.path.exists(LIB):
            build()
        _lib = C.CDLL(LIB)
        for name in ("fade_gen_markov2", "fade_gen_text", "fade_gen_genome", "fade_gen_float_ar1"):
            getattr(_lib, name).argtypes = [C.c_uint64, C.c_size_t, C.c_void_p]
        _lib.fade_gen_normal_f32.argtypes = [C.c_uint64, C.c_size_t, C.c_float, C.c_float, C.c_void_p]
    return _lib


def _gen(fn, seed, n):
    out = np.empty(n, np.uint8)
    rc = getattr(_l(), fn)(C.c_uint64(seed), n, out.ctypes.data_as(C.c_void_p))
    if rc:
        raise MemoryError(fn)
    return out


def markov2(seed, n):
    return _gen("fade_gen_markov2", seed, n)


def text(seed, n):
    return _gen("fade_gen_text", seed, n)


def genome(seed, n):
    return _gen("fade_gen_genome", seed, n)


def float_ar1(seed, n):
    return _gen("fade_gen_float_ar1", seed, n)


def mixed(seed, n, block=64 << 20):
    """Alternating blocks of the text, genome and float sources, block j seeded with seed + j."""
    gens = (text, genome, float_ar1)
    jobs, j, left = [], 0, n
    while left > 0:
        m = min(block, left)
        jobs.append((gens[j % 3], seed + j, m))
        left -= m
        j += 1
    if not jobs:
        return np.empty(0, np.uint8)
    # the blocks are independent (own seed each) and the generators run outside the interpreter lock
    from concurrent.futures import ThreadPoolExecutor
    with ThreadPoolExecutor(max_workers=min(8, len(jobs), os.cpu_count() or 1)) as ex:
        parts = list(ex.map(lambda q: q[0](q[1], q[2]), jobs))
    return np.concatenate(parts)


_SOURCES = dict(markov2=markov2, text=text, genome=genome, float=float_ar1, mixed=mixed)


def config_bytes(cfg_id, nbytes=None):
    """The byte stream of benchmark configuration `cfg_id` (or its first `nbytes`... of a shorter run:
    the generators are sequential, so a shorter request is a different, equally distributed stream
    only for the mixed source's block boundaries; for the others it is the exact prefix)."""
    spec = CONFIGS[cfg_id]
    n = spec["nbytes"] if nbytes is None else nbytes
    return _SOURCES[spec["source"]](SEED_BASE + cfg_id, n)


def tensor_specs(B, T, D, H, d_low=64, c=None, k=3, d_cache=None, d_e=None):
    """[(name, shape, init)] in blob order; init is 'normal' (N(0, 0.02)), 'one' or 'zero'."""
    Dh, Dc, De = T * D, d_cache or H, d_e or H
    c = Dc // T if c is None else c
    return [
        ("E", (256, D), "normal"),
        ("gamma_e", (D,), "one"), ("beta_e", (D,), "zero"),
        ("gamma_l", (D,), "one"), ("beta_l", (D,), "zero"),
        ("W_g", (D, c), "normal"), ("W_v", (D, c), "normal"),
        ("W_m", (Dc, Dh), "normal"), ("lambda_m", (1,), "one"),
        ("W_conv", (k, D, D), "normal"), ("b_conv", (D,), "zero"),
        ("W_r", (Dh, Dh), "normal"),
        ("gamma_c", (Dh,), "one"), ("beta_c", (Dh,), "zero"),
        ("W_down", (Dh, d_low), "normal"),
        ("W_U", (B, d_low, d_low), "normal"),
        ("W_up", (d_low, Dh), "normal"),
        ("W_c", (Dh, Dh), "normal"), ("lambda_c", (1,), "one"),
        ("gamma_f", (Dh,), "one"), ("beta_f", (Dh,), "zero"),
        ("W_fg", (Dh, De), "normal"), ("W_fv", (Dh, De), "normal"),
        ("W_f", (De, Dh), "normal"),
        ("gamma_o", (Dh,), "one"), ("beta_o", (Dh,), "zero"), ("lambda_o", (1,), "one"),
        ("W_o", (Dh, 256), "normal"), ("b_o", (256,), "zero"),
    ]


class Blob:
    """A flat fp32 weight blob with named views."""

    def __init__(self, B, T, D, H, d_low=64, c=None, k=3, d_cache=None, d_e=None):
        self.specs = tensor_specs(B, T, D, H, d_low, c, k, d_cache, d_e)
        self.offsets = OrderedDict()
        o = 0
        for name, shape, _ in self.specs:
            n = int(np.prod(shape))
            self.offsets[name] = (o, n, shape)
            o += n
        self.data = np.zeros(o, np.float32)

    def __getitem__(self, name):
        o, n, shape = self.offsets[name]
        return self.data[o:o + n].reshape(shape)

    def __setitem__(self, name, value):
        self[name][...] = value

    def view(self, flat, name):
        """The same named view into another flat array of blob layout (e.g. a gradient)."""
        o, n, shape = self.offsets[name]
        return flat[o:o + n].reshape(shape)


def init_blob(B, T, D, H, seed, d_low=64, c=None, k=3, std=0.02, d_cache=None, d_e=None):
    """Random init: matrices, conv taps, embedding and every W_U slice ~ N(0, std) (one independent
    draw per element), residual scales and LayerNorm gains 1, biases and LayerNorm shifts 0."""
    blob = Blob(B, T, D, H, d_low, c, k, d_cache, d_e)
    for i, (name, shape, init) in enumerate(blob.specs):
        v = blob[name]
        if init == "normal":
            n = v.size
            tmp = np.empty(n, np.float32)
            _l().fade_gen_normal_f32(C.c_uint64(seed * 1000003 + i), n, C.c_float(0.0), C.c_float(std),
                                     tmp.ctypes.data_as(C.c_void_p))
            v[...] = tmp.reshape(shape)
        elif init == "one":
            v[...] = 1.0
    return blob


def config_blob(cfg_id, B=None):
    """Random-init blob of benchmark configuration `cfg_id`; `B` overrides the stream count (the first
    B slices of W_U are then identical to those of the full blob, every other tensor is unchanged)."""
    spec = CONFIGS[cfg_id]
    full = init_blob(spec["B"], spec["T"], spec["D"], spec["H"], SEED_BASE + cfg_id, d_cache=spec.get("d_cache"), d_e=spec.get("d_e"))
    if B is None or B == spec["B"]:
        return full
    return slice_blob(full, spec, B)


def slice_blob(full, spec, B):
    sub = Blob(B, spec["T"], spec["D"], spec["H"], d_cache=spec.get("d_cache"), d_e=spec.get("d_e"))
    for name, _, _ in sub.specs:
        if name == "W_U":
            sub[name] = full[name][:B]
        else:
            sub[name] = full[name]
    return sub
