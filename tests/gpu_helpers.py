"""Helpers for the GPU parity tests: build matching oracle / libfade contexts from one config + blob."""
import numpy as np
import pytest

import fade_inputs as fi
import oracle as orc


def need_gpu():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    return torch


def make_pair(B, T, D, H, dtype, seed=1, update_mode=0, std=0.02, randomize=False, **kw):
    """(libfade context, oracle context, blob) with identical configuration and weights."""
    import paper_2604_07239_amd as fa
    blob = fi.init_blob(B, T, D, H, seed, std=std, d_cache=kw.get("d_cache"), d_e=kw.get("d_e"))
    if randomize:
        rng = np.random.default_rng(seed)
        for name, shape, init in blob.specs:
            if init == "one":
                blob[name] = 1.0 + 0.2 * rng.standard_normal(shape)
            elif init == "zero":
                blob[name] = 0.1 * rng.standard_normal(shape)
    g = fa.Fade(fa.make_config(B, T, D, H, dtype=fa.BF16 if dtype == "bf16" else fa.F32, update_mode=update_mode, **kw))
    g.load_weights(blob.data)
    o = orc.Oracle(orc.make_config(B, T, D, H, dtype=orc.BF16 if dtype == "bf16" else orc.F32, update_mode=update_mode, **kw))
    o.load_weights(blob.data)
    return g, o, blob
