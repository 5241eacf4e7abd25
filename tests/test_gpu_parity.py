"""GPU parity: libfade (HIP, through the C ABI) against the CPU oracle on the same seeded inputs.
Bars: integer work bit-exact; probabilities within 1e-3 absolute per symbol (bf16 path additionally
within 5e-2 relative at random-init scale, fp32 path within 2e-5); compressed size within 0.5 %;
GPU encode -> GPU decode byte-exact."""
import numpy as np
import pytest

import fade_inputs as fi
import oracle as orc
from gpu_helpers import make_pair, need_gpu

pytestmark = pytest.mark.gpu


def _log(msg):
    print(msg, flush=True)


# ---------------------------------------------------------------------------------------------------
# integer kernels
# ---------------------------------------------------------------------------------------------------
def test_quantizer_bit_identical_to_oracle():
    torch = need_gpu()
    g, _, _ = make_pair(4, 8, 32, 64, "bf16")
    rng = np.random.default_rng(0)
    rows = [rng.dirichlet(np.full(256, a), 3000) for a in (1.0, 0.05, 50.0)]
    z = rng.standard_normal((3001, 256)) * rng.uniform(0.1, 30, (3001, 1))  # ragged row count
    e = np.exp(z - z.max(1, keepdims=True))
    rows.append(e / e.sum(1, keepdims=True))
    p = np.concatenate(rows).astype(np.float32)
    p[0] = 1.0 / 256
    p[1] = 0; p[1, 7] = 1.0
    p[2] = 0; p[2, 3] = 0.5; p[2, 9] = 0.5
    _log(f"quantize rows={p.shape[0]}")
    pd = torch.from_numpy(p).cuda()
    fd = torch.zeros(p.shape, dtype=torch.int16, device="cuda")
    g.quantize(pd, fd)
    got = fd.cpu().numpy().view(np.uint16)
    np.testing.assert_array_equal(got, orc.quantize(p))
    bad = p[:4].copy(); bad[1, 5] = np.nan
    with pytest.raises(Exception) as ex:
        g.quantize(torch.from_numpy(bad).cuda(), fd[:4])
    assert ex.value.code == -9


@pytest.mark.parametrize("n_streams,n_steps,conc", [(1, 200, 0.3), (37, 300, 0.05), (260, 64, 5.0)])
def test_coder_bit_identical_on_fixed_tables(n_streams, n_steps, conc):
    torch = need_gpu()
    g, _, _ = make_pair(4, 8, 32, 64, "bf16")
    rng = np.random.default_rng(n_streams)
    f = orc.quantize(rng.dirichlet(np.full(256, conc), n_steps * n_streams).astype(np.float32)).reshape(n_steps, n_streams, 256)
    cdf = np.cumsum(f.astype(np.int64), 2)
    sym = (cdf > rng.integers(0, 65536, (n_steps, n_streams, 1))).argmax(2).astype(np.uint8)
    sym[::7] = rng.integers(0, 256, sym[::7].shape, dtype=np.uint8)  # atypical symbols: long codes, carries
    cap = 2 * n_steps + 16
    _log(f"coder tables streams={n_streams} steps={n_steps}")
    fd = torch.from_numpy(f.view(np.int16)).cuda()
    sd = torch.from_numpy(sym).cuda()
    out = torch.zeros((n_streams, cap), dtype=torch.uint8, device="cuda")
    ln = torch.zeros(n_streams, dtype=torch.int32, device="cuda")
    g.coder_encode_tables(fd, sd, n_steps, n_streams, out, cap, ln)
    out_h, ln_h = out.cpu().numpy(), ln.cpu().numpy()
    for k in range(n_streams):
        ref = orc.coder_encode(f[:, k], sym[:, k])
        assert ln_h[k] == ref.size
        assert out_h[k, :ref.size].tobytes() == ref.tobytes()
    dec = torch.zeros((n_steps, n_streams), dtype=torch.uint8, device="cuda")
    g.coder_decode_tables(fd, n_steps, n_streams, out, cap, ln, dec)
    np.testing.assert_array_equal(dec.cpu().numpy(), sym)


def test_coder_uniform_closed_form_on_gpu():
    """Uniform tables: the payload is the symbols themselves plus 0x40."""
    torch = need_gpu()
    g, _, _ = make_pair(4, 8, 32, 64, "bf16")
    n_streams, n_steps = 5, 40
    sym = np.random.default_rng(1).integers(0, 256, (n_steps, n_streams), dtype=np.uint8)
    f = np.full((n_steps, n_streams, 256), 256, np.uint16)
    cap = 2 * n_steps + 16
    out = torch.zeros((n_streams, cap), dtype=torch.uint8, device="cuda")
    ln = torch.zeros(n_streams, dtype=torch.int32, device="cuda")
    g.coder_encode_tables(torch.from_numpy(f.view(np.int16)).cuda(), torch.from_numpy(sym).cuda(), n_steps, n_streams, out, cap, ln)
    out_h = out.cpu().numpy()
    assert np.all(ln.cpu().numpy() == n_steps + 1)
    for k in range(n_streams):
        assert out_h[k, :n_steps + 1].tobytes() == sym[:, k].tobytes() + b"\x40"


# ---------------------------------------------------------------------------------------------------
# the model step
# ---------------------------------------------------------------------------------------------------
TAP_TOL = {  # absolute tolerance per tap for the bf16 path at unit-scale activations
    "X": 0.02, "CACHE": 0.01, "H_GLOBAL": 0.03, "H_LOCAL": 0.02, "H_MIX": 0.03, "Y_DOWN": 0.05, "Z_BMM": 0.02,
    "H_A": 0.02, "H_COARSE": 0.04, "H_EXPAND": 0.02, "LOGITS": 0.05,
}


ABLATION_TAPS = {1: ("X", "CACHE", "H_GLOBAL", "LOGITS"), 2: ("X", "CACHE", "H_GLOBAL", "H_LOCAL", "H_MIX", "LOGITS"),
                 3: ("H_MIX", "Y_DOWN", "Z_BMM", "H_A", "H_COARSE", "LOGITS"), 4: ("H_MIX", "H_A", "H_COARSE", "LOGITS")}


def _step_parity(B, T, D, H, dtype, steps, randomize, seed, std=0.02, **widths):
    torch = need_gpu()
    g, o, _ = make_pair(B, T, D, H, dtype, seed=seed, randomize=randomize, std=std, **widths)
    rng = np.random.default_rng(seed)
    data = rng.integers(0, 256, (B, T + steps), dtype=np.uint8)
    freq_d = torch.zeros((B, 256), dtype=torch.int16, device="cuda")
    probs_d = torch.zeros((B, 256), dtype=torch.float32, device="cuda")
    worst = 0.0
    for i in range(steps):
        win = np.ascontiguousarray(data[:, i:i + T])
        act = None
        if i == 1 and B > 2:  # one masked step: the masked streams must not advance
            act = np.ones(B, np.uint8); act[1::3] = 0
        _log(f"step_probs B={B} T={T} D={D} H={H} {dtype} step={i}")
        g.step_probs(torch.from_numpy(win).cuda(), None if act is None else torch.from_numpy(act).cuda(), freq_d, probs_d)
        fo, po = o.step_probs(win, act)
        pg = probs_d.cpu().numpy()
        fg = freq_d.cpu().numpy().view(np.uint16)
        live = np.ones(B, bool) if act is None else act.astype(bool)
        dp = np.abs(pg[live] - po[live]).max()
        worst = max(worst, dp)
        assert dp <= 1e-3, f"step {i}: |dp| = {dp}"
        if dtype == "f32":
            assert dp <= 2e-5
            np.testing.assert_allclose(pg[live], po[live], rtol=2e-3)
        else:
            np.testing.assert_allclose(pg[live], po[live], rtol=5e-2, atol=2e-5)
        assert np.all(np.abs(pg[live].astype(np.float64).sum(1) - 1) < 1e-5)
        assert fg[live].min() >= 1 and np.all(fg[live].astype(np.int64).sum(1) == 65536)
        # the table is the exact quantiser image of the GPU's own probabilities
        np.testing.assert_array_equal(fg[live], orc.quantize(pg[live]))
        for name, tol in TAP_TOL.items():
            if widths.get("ablation") and name not in ABLATION_TAPS[widths["ablation"]]:
                continue   # stages past the cut are not computed
            t = g.tap(name)
            assert t is not None, name
            for b in np.flatnonzero(live)[:8]:
                ref = o.tap(name, int(b))
                err = np.abs(t[b] - ref).max()
                lim = tol if dtype == "bf16" else 2e-4
                assert err <= lim * max(1.0, np.abs(ref).max()), f"tap {name} stream {b} step {i}: {err}"
    return worst


@pytest.mark.parametrize("B", [5, 64, 130])
def test_step_parity_bf16_small(B):
    """Small bf16 shapes spanning several row tiles with a ragged tail (B = 5, 130), non-default gains/shifts."""
    _step_parity(B, 8, 32, 64, "bf16", steps=11, randomize=True, seed=B)


@pytest.mark.parametrize("B,T,c", [(5, 32, 8), (7, 64, 8), (67, 32, 8), (5, 32, 4), (7, 64, 4), (67, 64, 4), (9, 32, 16)])
def test_step_parity_bf16_window_kernel_with_tables_in_lds(B, T, c):
    """T = 32 / 64 at D = 32 with cache slots of 8, 16 or 4 elements (4: the benchmark configurations 2-4, whose roll of Eq. 2
    is half a 16-byte piece): the window / cache / conv step runs as the kernel that keeps the per-symbol tables in LDS and
    walks over streams (4 or 2 streams side by side per workgroup), here with a stream count that is no multiple of that
    and, at step 1, masked streams that must not advance. Ten steps: the rolled cache holds entries of several steps."""
    _step_parity(B, T, 32, 64, "bf16", steps=10, randomize=True, seed=B + T + c, d_cache=c * T)


def test_step_parity_bf16_wide_cache():
    _step_parity(33, 16, 32, 128, "bf16", steps=4, randomize=True, seed=3)


@pytest.mark.parametrize("dtype,B,T,D,H,d_cache,d_e", [
    ("bf16", 37, 8, 32, 64, 256, 128),     # cache slots of 32, refiner narrower than the cache
    ("bf16", 70, 16, 32, 128, 1024, 512),  # the paper-default proportions at 1/4 scale: slots of 64, D_e = D_h
    ("bf16", 9, 16, 32, 64, 4096, 1024),   # the widest cache the kernels take: slots of 256
    ("f32", 11, 8, 16, 64, 128, 192),
    ("bf16", 130, 16, 32, 64, 1024, 8192),  # enough column tiles for the refiner's input product to skip split-K
])
def test_step_parity_separate_cache_and_refiner_widths(dtype, B, T, D, H, d_cache, d_e):
    """D_cache and D_e given apart from H (the paper's default model has D_cache = 4096, D_e = 8192)."""
    _step_parity(B, T, D, H, dtype, steps=T + 3 if T <= 8 else 4, randomize=True, seed=B, d_cache=d_cache, d_e=d_e)


@pytest.mark.parametrize("level", [1, 2, 3, 4])
def test_step_parity_ablation_levels(level):
    """The paper's progressive ablation as a configuration switch: the head reads H_global / H_mix / H_a + lambda_c H_mix /
    H_coarse instead of the refiner's output."""
    _step_parity(70, 8, 32, 64, "bf16", steps=10, randomize=True, seed=20 + level, ablation=level)


@pytest.mark.parametrize("level", [1, 2, 3, 4])
def test_step_parity_ablation_levels_fp32(level):
    """The same switch on the fp32 path (both product kernels: the 16-row one of small batches and the general one)."""
    _step_parity(7, 8, 16, 64, "f32", steps=6, randomize=True, seed=40 + level, ablation=level)
    _step_parity(300, 8, 16, 64, "f32", steps=3, randomize=True, seed=50 + level, ablation=level)


def test_ablation_round_trip_and_multi_step_identity(monkeypatch):
    need_gpu()
    import paper_2604_07239_amd as fa
    B, T, D, H, n = 33, 8, 32, 64, 33 * 40 + 7
    blob = fi.init_blob(B, T, D, H, 5, std=0.05)
    src = fi.text(31, n)
    sizes = {}
    for level in (1, 2, 3, 4, 5):
        outs = []
        for steps in ("1", None):
            if steps is None:
                monkeypatch.delenv("FADE_STEPS_PER_PASS", raising=False)
            else:
                monkeypatch.setenv("FADE_STEPS_PER_PASS", steps)
            g = fa.Fade(fa.make_config(B, T, D, H, dtype=fa.BF16, ablation=level))
            g.load_weights(blob.data)
            outs.append(g.encode(src))
            np.testing.assert_array_equal(g.decode(outs[-1], n), src)
            g.close()
        assert outs[0].tobytes() == outs[1].tobytes()
        o = orc.Oracle(orc.make_config(B, T, D, H, dtype=orc.BF16, ablation=level))
        o.load_weights(blob.data)
        co = o.encode(src)
        assert abs(outs[0].size - co.size) <= 0.005 * co.size + B
        sizes[level] = outs[0].size


def test_step_parity_fp32_config1_shape():
    """Benchmark configuration 1's model shape (T = 32, D = 16, H = 128, fp32), B = 16."""
    _step_parity(16, 32, 16, 128, "f32", steps=5, randomize=False, seed=11)


def test_step_parity_fp32_ragged():
    _step_parity(21, 8, 16, 64, "f32", steps=4, randomize=True, seed=12)


def test_step_parity_bf16_config2_shape_sampled():
    """Configuration 2's model shape (T = 64, D = 32, H = 256, bf16) at its full B = 1024 on the GPU; the oracle
    follows the first 24 streams (its W_U slices are those streams' own)."""
    torch = need_gpu()
    import paper_2604_07239_amd as fa
    B, Bo, T, D, H = 1024, 24, 64, 32, 256
    blob = fi.config_blob(2)
    sub = fi.slice_blob(blob, fi.CONFIGS[2], Bo)
    g = fa.Fade(fa.make_config(B, T, D, H, dtype=fa.BF16))
    g.load_weights(blob.data)
    o = orc.Oracle(orc.make_config(Bo, T, D, H, dtype=orc.BF16))
    o.load_weights(sub.data)
    data = fi.config_bytes(2, 1 << 20).reshape(B, -1)[:, :T + 3]
    probs_d = torch.zeros((B, 256), dtype=torch.float32, device="cuda")
    for i in range(3):
        win = np.ascontiguousarray(data[:, i:i + T])
        _log(f"cfg2 shape step {i}")
        g.step_probs(torch.from_numpy(win).cuda(), None, None, probs_d)
        _, po = o.step_probs(win[:Bo])
        pg = probs_d.cpu().numpy()
        assert np.abs(pg[:Bo] - po).max() <= 1e-3
        np.testing.assert_allclose(pg[:Bo], po, rtol=5e-2, atol=2e-5)
        assert np.all(np.abs(pg.astype(np.float64).sum(1) - 1) < 1e-5)


def _sampled_streams_parity(cfg, streams, steps=2):
    """Full batch of a benchmark configuration on the GPU (the launch shapes bench.py times: tile sizes and grids depend on
    B); the oracle follows a sample of streams, each with its own W_U slice. Streams are independent in the frozen step."""
    torch = need_gpu()
    import paper_2604_07239_amd as fa
    spec = fi.CONFIGS[cfg]
    B, T, D, H = spec["B"], spec["T"], spec["D"], spec["H"]
    blob = fi.config_blob(cfg)
    idx = np.asarray(streams)
    widths = dict(d_cache=spec.get("d_cache", 0), d_e=spec.get("d_e", 0))
    sub = fi.Blob(len(idx), T, D, H, **widths)
    for name, _, _ in sub.specs:
        sub[name] = blob[name][idx] if name == "W_U" else blob[name]
    g = fa.Fade(fa.make_config(B, T, D, H, dtype=fa.BF16, **widths))
    g.load_weights(blob.data)
    o = orc.Oracle(orc.make_config(len(idx), T, D, H, dtype=orc.BF16, **widths))
    o.load_weights(sub.data)
    data = fi.config_bytes(cfg, B * 256).reshape(B, -1)[:, :T + steps]
    probs_d = torch.zeros((B, 256), dtype=torch.float32, device="cuda")
    freq_d = torch.zeros((B, 256), dtype=torch.int16, device="cuda")
    for i in range(steps):
        win = np.ascontiguousarray(data[:, i:i + T])
        _log(f"cfg{cfg} full batch B={B} step {i}")
        g.step_probs(torch.from_numpy(win).cuda(), None, freq_d, probs_d)
        _, po = o.step_probs(np.ascontiguousarray(win[idx]))
        pg = probs_d.cpu().numpy()
        assert np.abs(pg[idx] - po).max() <= 1e-3
        np.testing.assert_allclose(pg[idx], po, rtol=5e-2, atol=2e-5)
        # properties that hold for every stream of the batch
        assert np.all(np.isfinite(pg)) and np.all(np.abs(pg.astype(np.float64).sum(1) - 1) < 1e-5)
        fg = freq_d.cpu().numpy().view(np.uint16)
        assert fg.min() >= 1 and np.all(fg.astype(np.int64).sum(1) == 65536)
        np.testing.assert_array_equal(fg[idx], orc.quantize(pg[idx]))


def test_step_parity_config3_full_batch_sampled():
    """B = 4096 (configurations 3 and 4 share the model shape): 256-row tiles in the router / gate products."""
    _sampled_streams_parity(3, list(range(6)) + [1023, 2048, 4000] + list(range(4090, 4096)))


def test_step_parity_paper_default_shape_full_batch_sampled():
    """Configuration 6: T = 16, D = 32, D_cache = 4096, D_e = 8192 at B = 4096, the model the paper adopts as its default.
    The refiner's input product runs without split-K here: folded LayerNorm and GeGLU in its epilogue."""
    _sampled_streams_parity(6, list(range(4)) + [1023, 2048] + list(range(4092, 4096)), steps=2)


def test_step_parity_config5_full_batch_sampled():
    """B = 16384, H = 512: the largest configuration."""
    _sampled_streams_parity(5, list(range(4)) + [5000, 9999] + list(range(16380, 16384)), steps=2)


# ---------------------------------------------------------------------------------------------------
# compress / decompress
# ---------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("dtype,B,T,D,H,n", [
    ("bf16", 5, 8, 32, 64, 0), ("bf16", 5, 8, 32, 64, 3), ("bf16", 5, 8, 32, 64, 37), ("bf16", 5, 8, 32, 64, 1001),
    ("bf16", 70, 8, 32, 64, 70 * 40), ("f32", 16, 32, 16, 128, 16 * 50 + 5),
    ("bf16", 7, 32, 32, 64, 7 * 90 + 5),   # T = 32: tables-in-LDS window kernel, a last stream that ends early
])
def test_round_trip_and_size_vs_oracle(dtype, B, T, D, H, n):
    need_gpu()
    g, o, _ = make_pair(B, T, D, H, dtype, seed=5, std=0.05)
    src = fi.text(77, n) if n else np.zeros(0, np.uint8)
    _log(f"round trip {dtype} B={B} n={n}")
    c = g.encode(src)
    out = g.decode(c, n)
    np.testing.assert_array_equal(out, src)
    co = o.encode(src)
    assert c[:64].tobytes() == co[:64].tobytes()          # identical header (same config, n, weight hash)
    if n >= 1000:
        assert abs(c.size - co.size) <= 0.005 * co.size
    else:
        assert abs(c.size - co.size) <= 2 * B + 0.005 * co.size
    # the oracle can decode the GPU's container only if every table matched bit for bit, which floating
    # point does not promise; what must hold is that each decoder inverts its own encoder
    np.testing.assert_array_equal(o.decode(co, n), src)


@pytest.mark.parametrize("B,T,D,H,n,widths", [(5, 8, 32, 64, 1001, {}), (70, 8, 32, 64, 70 * 45 + 11, {}), (130, 16, 32, 128, 130 * 60 + 3, {}),
                                              (21, 16, 32, 64, 21 * 50 + 5, dict(d_cache=2048, d_e=256))])
def test_multi_step_encode_equals_single_steps(B, T, D, H, n, widths, monkeypatch):
    """Frozen bf16 compression runs several steps of every stream per pass (the model's steps are independent once the
    input is known; only the coder is sequential). The container must be the one single steps produce, byte for byte:
    the decoder, which can only take single steps, has to reproduce every table."""
    torch = need_gpu()
    import paper_2604_07239_amd as fa
    blob = fi.init_blob(B, T, D, H, 5, std=0.05, **widths)
    src = fi.text(21, n)
    outs = {}
    for steps in ("1", "7", None):   # single steps; groups with a ragged last one; the default
        if steps is None:
            monkeypatch.delenv("FADE_STEPS_PER_PASS", raising=False)
        else:
            monkeypatch.setenv("FADE_STEPS_PER_PASS", steps)
        g = fa.Fade(fa.make_config(B, T, D, H, dtype=fa.BF16, **widths))
        g.load_weights(blob.data)
        _log(f"multi-step encode B={B} n={n} steps/pass={steps}")
        outs[steps] = g.encode(src)
        if steps == "7":   # a job in pieces: passes and single steps interleave, so the rolling cache must carry over
            sd = torch.from_numpy(src).cuda()
            L = (n + B - 1) // B
            first = 0
            for cnt in (3, T + 9, 1, 1, 12, 0):
                g.encode_device(sd, n, first, cnt)
                first = min(L, first + cnt) if cnt else L
            lens, data = g.payloads()
            lens1 = np.frombuffer(outs["1"][64:64 + 4 * B].tobytes(), np.uint32)
            np.testing.assert_array_equal(lens, lens1)
            assert data.tobytes() == outs["1"][64 + 4 * B:].tobytes()
        np.testing.assert_array_equal(g.decode(outs[steps], n), src)
        g.close()
    assert outs["1"].tobytes() == outs["7"].tobytes()
    assert outs["1"].tobytes() == outs[None].tobytes()


@pytest.mark.parametrize("chunk", [16, 4])
def test_multi_step_encode_with_explicit_cache_chunk(chunk, monkeypatch):
    """A cache whose slot count differs from the window length (T = 8; 64 / 16 = 4 slots, 64 / 4 = 16 slots): the pass
    that rebuilds the cache from the stream's bytes must pick the symbols the rolling cache appended, also the ones that
    have already left the window. Multi-step containers equal the single-step one byte for byte, both round-trip, and the
    size matches the oracle's."""
    need_gpu()
    import paper_2604_07239_amd as fa
    B, T, D, H, n = 9, 8, 32, 64, 9 * 61 + 4
    blob = fi.init_blob(B, T, D, H, 5, std=0.05, c=chunk)
    src = fi.text(23, n)
    outs = {}
    for steps in ("1", "5", None):
        if steps is None:
            monkeypatch.delenv("FADE_STEPS_PER_PASS", raising=False)
        else:
            monkeypatch.setenv("FADE_STEPS_PER_PASS", steps)
        g = fa.Fade(fa.make_config(B, T, D, H, dtype=fa.BF16, cache_chunk=chunk))
        g.load_weights(blob.data)
        _log(f"multi-step encode cache_chunk={chunk} steps/pass={steps}")
        outs[steps] = g.encode(src)
        np.testing.assert_array_equal(g.decode(outs[steps], n), src)
        g.close()
    assert outs["1"].tobytes() == outs["5"].tobytes()
    assert outs["1"].tobytes() == outs[None].tobytes()
    o = orc.Oracle(orc.make_config(B, T, D, H, dtype=orc.BF16, cache_chunk=chunk))
    o.load_weights(blob.data)
    co = o.encode(src)
    assert abs(outs["1"].size - co.size) <= 0.005 * co.size + 2 * B


def test_multi_step_encode_config2_full_batch():
    """The same identity at benchmark configuration 2's full batch, where a pass carries 16 x 1024 rows through the
    tall-product tiles and in-workgroup split sums that bench.py's frozen compression times."""
    need_gpu()
    import paper_2604_07239_amd as fa
    spec = fi.CONFIGS[2]
    B, T, D, H = spec["B"], spec["T"], spec["D"], spec["H"]
    blob = fi.config_blob(2)
    L = T + 41
    src = np.ascontiguousarray(fi.config_bytes(2, B * 256).reshape(B, -1)[:, :L]).reshape(-1)[:B * L - 700]   # ragged tail
    outs = []
    for steps in ("1", None):
        import os
        if steps is None:
            os.environ.pop("FADE_STEPS_PER_PASS", None)
        else:
            os.environ["FADE_STEPS_PER_PASS"] = steps
        try:
            g = fa.Fade(fa.make_config(B, T, D, H, dtype=fa.BF16))
        finally:
            os.environ.pop("FADE_STEPS_PER_PASS", None)
        g.load_weights(blob.data)
        _log(f"cfg2 multi-step encode, steps/pass={steps}")
        outs.append(g.encode(src))
        if steps is None:
            np.testing.assert_array_equal(g.decode(outs[-1], src.size), src)
        g.close()
    assert outs[0].tobytes() == outs[1].tobytes()
    # sampled (full-length) streams against the oracle, which codes them alone (frozen streams are independent):
    # the payload lengths agree
    idx = np.array([0, 1, 511, 1000])
    sub = fi.Blob(len(idx), T, D, H)
    for name, _, _ in sub.specs:
        sub[name] = blob[name][idx] if name == "W_U" else blob[name]
    o = orc.Oracle(orc.make_config(len(idx), T, D, H, dtype=orc.BF16))
    o.load_weights(sub.data)
    co = o.encode(np.concatenate([src[i * L:(i + 1) * L] for i in idx]))
    lens_g = np.frombuffer(outs[1][64:64 + 4 * B].tobytes(), np.uint32)[idx].astype(np.int64)
    lens_o = np.frombuffer(co[64:64 + 4 * len(idx)].tobytes(), np.uint32).astype(np.int64)
    assert np.all(np.abs(lens_g - lens_o) <= 1 + 0.005 * lens_o), (lens_g, lens_o)


def test_round_trip_separate_cache_and_refiner_widths():
    need_gpu()
    B, n = 21, 21 * 70 + 9
    g, o, _ = make_pair(B, 16, 32, 64, "bf16", seed=5, std=0.05, d_cache=1024, d_e=512)
    src = fi.text(78, n)
    c = g.encode(src)
    np.testing.assert_array_equal(g.decode(c, n), src)
    co = o.encode(src)
    assert c[:64].tobytes() == co[:64].tobytes()          # both record D_e and D_cache in the header
    assert abs(c.size - co.size) <= 0.005 * co.size + B
    g2, _, _ = make_pair(B, 16, 32, 64, "bf16", seed=5, std=0.05, d_cache=1024, d_e=256)
    with pytest.raises(Exception):
        g2.decode(c, n)                                    # another refiner width: refused


def test_one_context_codes_jobs_of_different_sizes():
    """The host-buffer calls stage jobs in buffers the context keeps and grows: a small, a larger and again a smaller job
    on one context give the containers fresh contexts give, and every one round-trips."""
    need_gpu()
    B = 9
    g, _, _ = make_pair(B, 8, 32, 64, "bf16", seed=5, std=0.05)
    for n in (B * 20 + 1, B * 140 + 5, 0, B * 33):
        src = fi.text(79 + n, n) if n else np.zeros(0, np.uint8)
        c = g.encode(src)
        fresh, _, _ = make_pair(B, 8, 32, 64, "bf16", seed=5, std=0.05)
        assert c.tobytes() == fresh.encode(src).tobytes(), n
        np.testing.assert_array_equal(g.decode(c, n), src)
        np.testing.assert_array_equal(fresh.decode(c, n), src)


def test_uniform_model_container_is_exact():
    """Zero head -> every table is f = 256: payload = the bytes + 0x40 per stream, identical to the oracle's."""
    need_gpu()
    import paper_2604_07239_amd as fa
    B, T, D, H = 6, 8, 32, 64
    blob = fi.init_blob(B, T, D, H, 3)
    blob["W_o"] = 0.0
    g = fa.Fade(fa.make_config(B, T, D, H, dtype=fa.BF16))
    g.load_weights(blob.data)
    o = orc.Oracle(orc.make_config(B, T, D, H, dtype=orc.BF16))
    o.load_weights(blob.data)
    src = fi.markov2(9, 6 * 30)
    c = g.encode(src)
    assert c.size == 64 + 4 * B + src.size + B
    assert c.tobytes() == o.encode(src).tobytes()


def test_error_paths_from_host():
    need_gpu()
    import paper_2604_07239_amd as fa
    g, _, blob = make_pair(5, 8, 32, 64, "bf16", seed=5)
    src = fi.text(1, 300)
    c = g.encode(src)
    for bad, code in ((c[:30], -6), (c[:-1], -6), (np.concatenate([c, c[:1]]), -6)):
        with pytest.raises(fa.FadeError) as e:
            g.decode(bad, 300)
        assert e.value.code == code
    m = c.copy(); m[1] ^= 0xff
    with pytest.raises(fa.FadeError) as e:
        g.decode(m, 300)
    assert e.value.code == -6
    with pytest.raises(fa.FadeError) as e:
        g.decode(c, 10)
    assert e.value.code == -5
    w2 = blob.data.copy(); w2[5] += 1
    g.load_weights(w2)
    with pytest.raises(fa.FadeError) as e:
        g.decode(c, 300)
    assert e.value.code == -4
    g.load_weights(blob.data)
    np.testing.assert_array_equal(g.decode(c, 300), src)   # the context survives every error above
    # another ablation level reads the same blob (same hash) as another model: the header's level byte refuses it
    g3 = fa.Fade(fa.make_config(5, 8, 32, 64, ablation=3))
    g3.load_weights(blob.data)
    with pytest.raises(fa.FadeError) as e:
        g3.decode(c, 300)
    assert e.value.code == -2
    g3.close()
    # corrupted payload bytes: the decoder reads only inside each stream's own payload (lengths are checked on the host,
    # reads past a payload's end return zeros), so the call ends with CORRUPT_STREAM or with wrong bytes, never a fault
    rng = np.random.default_rng(3)
    body = 64 + 4 * 5
    for trial in range(6):
        m = c.copy()
        pos = rng.integers(body, c.size, 4)
        m[pos] ^= rng.integers(1, 256, 4).astype(np.uint8)
        try:
            out = g.decode(m, 300)
            assert out.size == 300
        except fa.FadeError as e2:
            assert e2.code == -6
    np.testing.assert_array_equal(g.decode(c, 300), src)
    with pytest.raises(fa.FadeError) as e:
        fa.Fade(fa.make_config(5, 8, 24, 64))               # unsupported D
    assert e.value.code == -2
    g2 = fa.Fade(fa.make_config(5, 8, 32, 64))
    import torch
    with pytest.raises(fa.FadeError) as e:
        g2.step_probs(torch.zeros((5, 8), dtype=torch.uint8, device="cuda"))
    assert e.value.code == -3
