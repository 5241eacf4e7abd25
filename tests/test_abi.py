"""The C-ABI library loads and exports every symbol include/fade.h declares (no compute without a GPU)."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    txt = open(os.path.join(ROOT, "include", "fade.h")).read()
    txt = re.sub(r"/\*.*?\*/", "", txt, flags=re.S)
    return sorted(set(re.findall(r"\b(fade_[a-z_0-9]+)\s*\(", txt)))


def test_header_declares_the_named_entry_points():
    names = _declared()
    for must in ("fade_create", "fade_load_weights", "fade_step_probs", "fade_encode", "fade_decode", "fade_destroy"):
        assert must in names


def test_library_exports_every_declared_symbol():
    import paper_2604_07239_amd as fa
    if not os.path.exists(fa.LIB):
        fa.build()
    L = C.CDLL(fa.LIB)
    for name in _declared():
        assert hasattr(L, name), name


def test_config_struct_matches_header_size():
    import paper_2604_07239_amd as fa
    assert C.sizeof(fa.Config) == 19 * 4 + 4 + 8   # 14 u32 + 4 float + i32 (+ 4 padding) + pointer (8-aligned)


def test_host_side_validation_needs_no_gpu():
    import paper_2604_07239_amd as fa
    L = fa.lib()
    assert fa.weights_nbytes(fa.make_config(1024, 64, 32, 256)) == 15_490_723 * 4
    assert fa.weights_nbytes(fa.make_config(4, 3, 32, 64)) == 0          # H % T != 0 and no cache_chunk
    # separate cache and refiner widths: only W_m, W_g/W_v (through c) and the three refiner matrices change size
    base, wide = fa.make_config(8, 16, 32, 256), fa.make_config(8, 16, 32, 256, d_cache=512, d_e=1024)
    Dh = 16 * 32
    assert (fa.weights_nbytes(wide) - fa.weights_nbytes(base)) // 4 == (512 - 256) * Dh + 2 * 32 * (32 - 16) + 3 * Dh * (1024 - 256)
    h = C.c_void_p()
    bad = fa.make_config(4, 8, 32, 64)
    bad.abi_version = 99
    assert L.fade_create(C.byref(bad), C.byref(h)) == -1
    assert L.fade_create(C.byref(fa.make_config(4, 8, 24, 64)), C.byref(h)) == -2   # D not supported by the kernels
    assert L.fade_create(None, C.byref(h)) == -1
    import torch
    if not torch.cuda.is_available():
        # no CPU fallback: creating a context without a device fails loudly
        assert L.fade_create(C.byref(fa.make_config(4, 8, 32, 64)), C.byref(h)) == -7
        with pytest.raises(fa.FadeError):
            fa.Fade(fa.make_config(4, 8, 32, 64))


def test_blob_layout_agrees_with_harness_and_oracle():
    """Three statements of the same interface (harness, oracle, library) must give the same size."""
    import fade_inputs as fi
    import oracle as orc
    import paper_2604_07239_amd as fa
    for (B, T, D, H) in ((16, 32, 16, 128), (1024, 64, 32, 256), (7, 8, 32, 64)):
        n = fi.Blob(B, T, D, H).data.size * 4
        assert fa.weights_nbytes(fa.make_config(B, T, D, H)) == n
        assert orc.lib().fadeo_weights_nbytes(orc.make_config(B, T, D, H)) == n
