"""End-to-end pins of the oracle's compress/decompress loop (Algorithm 1): byte-exact round trips in both
update modes, ragged and degenerate sizes, the uniform-model size, size vs. model cross-entropy, learning
on a learnable source, and the container's error paths."""
import numpy as np
import pytest

import fade_inputs as fi
import oracle as orc
from helpers import tiny_oracle

HEADER = 64


def _mk(update_mode=orc.FROZEN, B=3, **kw):
    o, blob, k = tiny_oracle(update_mode=update_mode, B=B, std=0.3, **kw)
    o.load_weights(blob.data)
    return o, blob, k


@pytest.mark.parametrize("mode", [orc.FROZEN, orc.ONLINE_ADAM])
@pytest.mark.parametrize("n", [0, 1, 2, 3, 11, 12, 13, 100, 301])
def test_round_trip_sizes(mode, n):
    """B = 3, T = 4: n = 0 (header only), n < B (some streams empty), streams shorter than the window
    (uniform coding only), ragged last stream, and ordinary sizes."""
    o, _, kw = _mk(mode)
    src = np.random.default_rng(n).integers(0, 256, n, dtype=np.uint8)
    blob = o.encode(src)
    assert blob.size >= HEADER + 4 * kw["B"]
    out = o.decode(blob, n)
    np.testing.assert_array_equal(out, src)


def test_uniform_model_costs_eight_bits_per_byte():
    """Zero head: every table is f = 256, so each stream's payload is its bytes + one termination byte."""
    o, blob, kw = tiny_oracle(B=3)
    blob["W_o"] = 0.0
    o.load_weights(blob.data)
    n = 3 * 50
    src = np.random.default_rng(0).integers(0, 256, n, dtype=np.uint8)
    c = o.encode(src)
    assert c.size == HEADER + 4 * 3 + n + 3
    L = n // 3
    body = c[HEADER + 12:]
    for k in range(3):
        assert body[k * (L + 1):(k + 1) * (L + 1)].tobytes() == src[k * L:(k + 1) * L].tobytes() + b"\x40"


def test_size_tracks_model_cross_entropy():
    """Coded payload is within 1 % (+ 2 bytes per stream of termination slack) of the cross-entropy of the
    model's own probabilities on the data, and never below the tables' information content."""
    o, _, kw = _mk(orc.ONLINE_ADAM, B=2, lr=3e-3)
    rng = np.random.default_rng(5)
    n = 2 * 3000
    src = (rng.integers(0, 4, n) * 17 + 40).astype(np.uint8)  # four symbols: learnable quickly
    c = o.encode(src)
    bits_f, bits_p, steps = o.code_stats()
    T, B = kw["T"], 2
    assert steps == n - B * T
    payload_bits = 8 * (c.size - HEADER - 4 * B)
    warm_bits = 8 * B * T
    assert payload_bits >= bits_f + warm_bits - 1e-6
    assert payload_bits <= 1.01 * (bits_p + warm_bits) + 16 * B
    # the online model must have learnt the 4-symbol alphabet: far below 8 bits/byte, above the 2-bit floor
    assert 2.0 <= bits_p / steps < 4.0
    np.testing.assert_array_equal(o.decode(c, n), src)


def test_online_beats_frozen_on_a_learnable_source():
    src = fi.genome(123, 4000)
    of, _, _ = _mk(orc.FROZEN, B=2)
    oo, _, _ = _mk(orc.ONLINE_ADAM, B=2, lr=3e-3)
    assert oo.encode(src).size < 0.7 * of.encode(src).size


def test_container_error_paths():
    o, blob, kw = _mk()
    src = np.random.default_rng(1).integers(0, 256, 90, dtype=np.uint8)
    c = o.encode(src)
    with pytest.raises(orc.OracleError) as e:
        o.decode(c[:40], 90)
    assert e.value.code == -6
    bad = c.copy(); bad[0] ^= 1
    with pytest.raises(orc.OracleError):
        o.decode(bad, 90)
    with pytest.raises(orc.OracleError) as e:
        o.decode(c[:-1], 90)           # truncated payload
    assert e.value.code == -6
    with pytest.raises(orc.OracleError) as e:
        o.decode(c, 10)                # dst too small
    assert e.value.code == -5
    other = blob.data.copy(); other[3] += 1.0
    o.load_weights(other)
    with pytest.raises(orc.OracleError) as e:
        o.decode(c, 90)                # different weights
    assert e.value.code == -4
    o2, b2, _ = tiny_oracle(B=3, conv_k=2)
    o2.load_weights(b2.data)
    with pytest.raises(orc.OracleError) as e:
        o2.decode(c, 90)               # different configuration
    assert e.value.code == -2
    # another ablation level is another model on the same blob (same hash): the header records the level
    o3, b3, _ = tiny_oracle(B=3, ablation=3)
    o3.load_weights(blob.data)
    with pytest.raises(orc.OracleError) as e:
        o3.decode(c, 90)
    assert e.value.code == -2
    c3 = o3.encode(src)
    assert c3[22] == 3 and c[22] == 5
    np.testing.assert_array_equal(o3.decode(c3, 90), src)


def test_bad_configs_rejected():
    import ctypes as C
    L = orc.lib()
    h = C.c_void_p()
    assert L.fadeo_create(C.byref(orc.make_config(B=2, T=3, D=4, H=8)), C.byref(h)) == -2   # H % T
    assert L.fadeo_create(C.byref(orc.make_config(B=2, T=4, D=4, H=8, cache_chunk=3)), C.byref(h)) == -2
    assert L.fadeo_create(C.byref(orc.make_config(B=0, T=4, D=4, H=8)), C.byref(h)) == -2
    o = orc.Oracle(orc.make_config(B=2, T=4, D=4, H=8))
    with pytest.raises(orc.OracleError) as e:
        o.step_probs(np.zeros((2, 4), np.uint8))
    assert e.value.code == -3
