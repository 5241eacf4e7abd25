"""Pins of the oracle's quantiser and arithmetic coder: hand-worked tables, the closed form for the
uniform table, the prefix-code degeneration for dyadic tables, the code-length bound, brute force on
tiny alphabets, and round trips."""
import itertools
import os

import numpy as np
import pytest

import oracle as orc

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _parse_sparse(txt, dtype):
    default, items = None, {}
    for tok in txt.split():
        if tok.startswith("default="):
            default = float(tok.split("=")[1])
        else:
            i, v = tok.split(":")
            items[int(i)] = float(v)
    a = np.full(256, default, dtype)
    for i, v in items.items():
        a[i] = v
    return a


def test_quantizer_hand_worked_cases():
    n = 0
    for line in open(os.path.join(GOLD, "quantizer_cases.txt")):
        if line.startswith("#") or not line.strip():
            continue
        name, p_txt, f_txt = [s.strip() for s in line.split(";")]
        p = _parse_sparse(p_txt, np.float32)
        f = _parse_sparse(f_txt, np.int64)
        np.testing.assert_array_equal(orc.quantize(p)[0].astype(np.int64), f, err_msg=name)
        n += 1
    assert n >= 5


def test_quantizer_properties_random():
    """f >= 1, sum = 2^16 exactly, monotone in p away from the arg-max, for a wide mix of distributions."""
    rng = np.random.default_rng(0)
    rows = []
    rows.append(rng.dirichlet(np.full(256, 1.0), 20000))
    rows.append(rng.dirichlet(np.full(256, 0.05), 20000))            # peaky, many denormal-small tails
    rows.append(rng.dirichlet(np.full(256, 50.0), 10000))            # near uniform
    z = rng.standard_normal((20000, 256)) * rng.uniform(0.1, 30, (20000, 1))
    e = np.exp(z - z.max(1, keepdims=True))
    rows.append(e / e.sum(1, keepdims=True))                         # softmax outputs, sharp to flat
    p = np.concatenate(rows).astype(np.float32)
    p[:1000] *= np.float32(1 + 1e-6)                                  # sum slightly above one
    p[1000:2000] *= np.float32(1 - 1e-6)
    f = orc.quantize(p).astype(np.int64)
    assert f.min() >= 1
    assert np.all(f.sum(1) == 65536)
    # everything except the arg-max entry is exactly 1 + trunc(fp32 product)
    base = 1 + (p * np.float32(65280.0)).astype(np.int64)
    m = base.argmax(1)
    diff = f - base
    mask = np.ones_like(diff, bool)
    mask[np.arange(len(m)), m] = False
    assert np.all(diff[mask] == 0)
    assert np.all(diff[~mask] == 65536 - base.sum(1))


def test_quantizer_rejects_non_finite():
    p = np.full(256, 1 / 256, np.float32)
    p[5] = np.nan
    with pytest.raises(orc.OracleError):
        orc.quantize(p)
    p[5] = -0.1
    with pytest.raises(orc.OracleError):
        orc.quantize(p)


def test_coder_uniform_table_closed_form():
    """With f = 256 everywhere each symbol selects an aligned 2^-8 slice: the coder emits exactly the
    symbol's 8 bits and is back at the full interval, so encode(x) = x followed by the termination bits
    01 padded to one byte (0x40): 8.000 bits per symbol + 1 byte per stream."""
    rng = np.random.default_rng(1)
    for n in (1, 2, 7, 1000):
        x = rng.integers(0, 256, n, dtype=np.uint8)
        f = np.full((n, 256), 256, np.uint16)
        out = orc.coder_encode(f, x)
        assert out.tobytes() == x.tobytes() + b"\x40"
    assert orc.coder_encode(np.zeros((0, 256), np.uint16), np.zeros(0, np.uint8)).size == 0


def test_coder_dyadic_tables_are_a_prefix_code():
    f_row = np.zeros(256, np.uint16)
    f_row[:4] = [32768, 16384, 8192, 8192]
    for line in open(os.path.join(GOLD, "coder_dyadic.txt")):
        if line.startswith("#") or not line.strip():
            continue
        sym_txt, bits_txt = line.split(";")
        sym = np.array([int(s) for s in sym_txt.split()], np.uint8)
        bits = bits_txt.replace(" ", "").strip()
        bits += "0" * (-len(bits) % 8)
        expect = bytes(int(bits[i:i + 8], 2) for i in range(0, len(bits), 8))
        f = np.tile(f_row, (len(sym), 1))
        assert orc.coder_encode(f, sym).tobytes() == expect, line
        np.testing.assert_array_equal(orc.coder_decode(f, len(sym), np.frombuffer(expect, np.uint8)), sym)


def _random_tables(rng, n, conc):
    p = rng.dirichlet(np.full(256, conc), n).astype(np.float32)
    return orc.quantize(p)


@pytest.mark.parametrize("conc", [0.02, 0.3, 5.0])
def test_coder_round_trip_and_length_bound(conc):
    """decode(encode(x)) = x, and the length is within 2 bits (+ padding) of the information content
    sum -log2(f/2^16) from above, and not below it (no code beats its own model)."""
    rng = np.random.default_rng(int(conc * 100))
    n = 5000
    f = _random_tables(rng, n, conc)
    # symbols drawn from the tables themselves (typical) and uniformly (atypical, long codes)
    cdf = np.cumsum(f.astype(np.int64), 1)
    typical = (cdf > rng.integers(0, 65536, (n, 1))).argmax(1).astype(np.uint8)
    for sym in (typical, rng.integers(0, 256, n, dtype=np.uint8)):
        out = orc.coder_encode(f, sym)
        np.testing.assert_array_equal(orc.coder_decode(f, n, out), sym)
        info = -np.log2(f[np.arange(n), sym].astype(np.float64) / 65536.0).sum()
        assert out.size * 8 >= info - 1e-9
        # 32-bit interval arithmetic loses < 2^-15 relative range per symbol on top of the ideal length
        assert out.size * 8 <= np.ceil(info + n * 1e-4) + 2 + 7


def test_coder_brute_force_tiny_alphabet():
    """Every sequence of length <= 4 over three symbols, under three very different tables, decodes to
    itself, and distinct sequences never share an encoding that is a prefix-extension ambiguity."""
    tables = []
    for fr in ([65534, 1, 1], [1, 65534, 1], [21846, 21845, 21845], [40000, 25000, 536]):
        row = np.zeros(256, np.uint16)
        row[:3] = fr
        tables.append(row)
    for row in tables:
        for n in range(1, 5):
            seen = {}
            for seq in itertools.product(range(3), repeat=n):
                sym = np.array(seq, np.uint8)
                f = np.tile(row, (n, 1))
                out = orc.coder_encode(f, sym)
                np.testing.assert_array_equal(orc.coder_decode(f, n, out), sym)
                assert out.tobytes() not in seen, (seq, seen.get(out.tobytes()))
                seen[out.tobytes()] = seq


def test_coder_long_carry_chains():
    """A long run of symbols whose interval straddles the midpoint builds up many pending bits (the
    bit-plus-follow case); the stream must still round-trip."""
    row = np.zeros(256, np.uint16)
    row[:3] = [32767, 2, 32767]   # symbol 1 sits exactly around the midpoint
    n = 300
    sym = np.ones(n, np.uint8)
    sym[-1] = 2
    f = np.tile(row, (n, 1))
    out = orc.coder_encode(f, sym)
    np.testing.assert_array_equal(orc.coder_decode(f, n, out), sym)
    assert out.size * 8 >= (n - 1) * 14


def test_fnv1a64_known_vectors():
    """Published FNV-1a 64-bit test vectors (offset basis for the empty input, and 'a', 'foobar')."""
    assert orc.fnv1a64(np.zeros(0, np.uint8)) == 0xcbf29ce484222325
    assert orc.fnv1a64(np.frombuffer(b"a", np.uint8)) == 0xaf63dc4c8601ec8c
    assert orc.fnv1a64(np.frombuffer(b"foobar", np.uint8)) == 0x85944171f73967e8
