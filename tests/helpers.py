"""Shared test helpers (no method arithmetic): tiny configurations and random blobs."""
import numpy as np

import fade_inputs as fi
import oracle as orc

TINY = dict(B=3, T=4, D=4, H=8, d_low=4, cache_chunk=2, conv_k=3)
# cache, refiner and H all different (D_cache = 12 = 4 slots of 3, D_e = 20): a swapped width shows as a shape or value error
SPLIT_WIDTHS = dict(H=8, d_cache=12, d_e=20, cache_chunk=3)


def tiny_oracle(update_mode=orc.FROZEN, dtype=orc.F32, seed=7, std=0.3, **over):
    kw = dict(TINY)
    kw.update(over)
    cfg = orc.make_config(dtype=dtype, update_mode=update_mode, **kw)
    o = orc.Oracle(cfg)
    blob = fi.init_blob(kw["B"], kw["T"], kw["D"], kw["H"], seed, d_low=kw["d_low"], c=kw["cache_chunk"],
                        k=kw["conv_k"], std=std, d_cache=kw.get("d_cache"), d_e=kw.get("d_e"))
    return o, blob, kw


def randomize_small(blob, rng):
    """Give every non-matrix parameter a non-default value so that dropped gains/shifts/scales show."""
    for name, shape, init in blob.specs:
        if init == "one":
            blob[name] = 1.0 + 0.3 * rng.standard_normal(shape)
        elif init == "zero":
            blob[name] = 0.2 * rng.standard_normal(shape)
