"""Pins of the oracle's model step (Eq. 1-10 of the Method section + head + softmax) against things the
paper and the mathematics fix: closed forms for selector/permutation weights (a matmul with a scaled
selector matrix is a gather, so a transposed operand or a wrong index order shows), special cases,
invariants, and the parameter count the paper's efficiency table prints.
"""
import math

import numpy as np
import pytest

import fade_inputs as fi
import oracle as orc
from helpers import SPLIT_WIDTHS, TINY, randomize_small, tiny_oracle


def gelu(x):
    return np.array([0.5 * v * (1.0 + math.erf(v / math.sqrt(2.0))) for v in np.ravel(x)]).reshape(np.shape(x))


def sigmoid(x):
    return 1.0 / (1.0 + np.exp(-x))


def ln(x, gamma=None, beta=None, eps=1e-5):
    x = np.asarray(x, np.float64)
    h = (x - x.mean()) / np.sqrt(x.var() + eps)
    if gamma is not None:
        h = h * gamma + beta
    return h


def selector(rng, n_in, n_out, lo=0.5, hi=1.5):
    """[n_in][n_out] matrix with one non-zero per column: y[n] = scale[n] * x[src[n]]. src is drawn so that
    the matrix differs from its transpose wherever it is square."""
    src = rng.integers(0, n_in, n_out)
    if n_in == n_out:
        src = np.roll(np.arange(n_in), 1)  # cyclic shift: a permutation that is not an involution
    scale = rng.uniform(lo, hi, n_out) * rng.choice([-1.0, 1.0], n_out)
    W = np.zeros((n_in, n_out), np.float32)
    W[src, np.arange(n_out)] = scale
    return W, src, W[src, np.arange(n_out)].astype(np.float64)


def windows_for(rng, B, T):
    return rng.integers(0, 256, (B, T), dtype=np.uint8)


# ---------------------------------------------------------------------------------------------------
# Table "efficiency": 15.20 M parameters at T=16, D=32, cache 4096, refiner 8192
# ---------------------------------------------------------------------------------------------------
def test_parameter_count_matches_paper_table():
    """The five big matrices W_m [D_cache x D_h], W_r, W_c [D_h x D_h], the GeGLU pair [D_h x D_e] x 2 and
    W_f [D_e x D_h] must total 15,204,352 = the 15.20 M of the efficiency table at T=16, D=32
    (D_h = 512), D_cache = 4096, D_e = 8192. The blob uses one H for both widths, so measure the growth
    in H (it must be D_h for the cache projection plus 3 D_h for the refiner) and the H-free D_h^2 part."""
    def count(H, T=16, D=32):
        cfg = orc.make_config(B=1, T=T, D=D, H=H, cache_chunk=4)
        return orc.lib().fadeo_weights_nbytes(cfg) // 4

    per_h = (count(8192) - count(4096)) // 4096
    Dh = 512
    assert per_h == 4 * Dh
    # D_h^2 part: growth in D_h^2 terms, isolated by differencing T at fixed H
    sq = count(4096) - per_h * 4096  # everything that does not scale with H
    small = 256 * 32 + 4 * 32 + 2 * 32 * 4 + 3 + 3 * 32 * 32 + 32 + 6 * Dh + 2 * Dh * 64 + 64 * 64 + Dh * 256 + 256
    assert sq - small == 2 * Dh * Dh
    total = Dh * 4096 + 3 * Dh * 8192 + (sq - small)
    assert total == 15_204_352


# ---------------------------------------------------------------------------------------------------
# special cases with everything else random
# ---------------------------------------------------------------------------------------------------
@pytest.fixture
def setup():
    rng = np.random.default_rng(11)
    o, blob, kw = tiny_oracle(std=0.4)
    randomize_small(blob, rng)
    return o, blob, kw, rng


def test_probs_sum_to_one_and_tables_valid(setup):
    o, blob, kw, rng = setup
    o.load_weights(blob.data)
    for _ in range(6):
        freq, p = o.step_probs(windows_for(rng, kw["B"], kw["T"]))
        assert np.all(np.abs(p.astype(np.float64).sum(1) - 1.0) < 1e-6)
        assert freq.min() >= 1 and np.all(freq.astype(np.int64).sum(1) == 65536)


def test_zero_head_gives_uniform(setup):
    o, blob, kw, rng = setup
    blob["W_o"] = 0.0
    blob["b_o"] = 0.0
    o.load_weights(blob.data)
    freq, p = o.step_probs(windows_for(rng, kw["B"], kw["T"]))
    assert np.all(p == np.float32(1.0 / 256.0))
    assert np.all(freq == 256)


def test_zero_router_gives_half(setup):
    o, blob, kw, rng = setup
    blob["W_r"] = 0.0
    o.load_weights(blob.data)
    o.step_probs(windows_for(rng, kw["B"], kw["T"]))
    for b in range(kw["B"]):
        assert np.all(o.tap("ALPHA", b) == 0.5)
        np.testing.assert_allclose(o.tap("H_MIX", b), 0.5 * (o.tap("H_GLOBAL", b) + o.tap("H_LOCAL", b)), rtol=1e-14)


def test_zero_up_projection_leaves_scaled_residual(setup):
    o, blob, kw, rng = setup
    blob["W_up"] = 0.0
    blob["lambda_c"] = 0.625
    o.load_weights(blob.data)
    o.step_probs(windows_for(rng, kw["B"], kw["T"]))
    for b in range(kw["B"]):
        np.testing.assert_allclose(o.tap("H_COARSE", b), 0.625 * o.tap("H_MIX", b), rtol=1e-14)


def test_dead_streams_leave_alpha_times_scaled_input(setup):
    """W_m = 0, W_conv = 0, b_conv = 0: psi(0) = 0 on both branches, so H_global = lambda_m X, H_local = 0."""
    o, blob, kw, rng = setup
    blob["W_m"] = 0.0
    blob["W_conv"] = 0.0
    blob["b_conv"] = 0.0
    blob["lambda_m"] = 1.75
    o.load_weights(blob.data)
    o.step_probs(windows_for(rng, kw["B"], kw["T"]))
    for b in range(kw["B"]):
        np.testing.assert_allclose(o.tap("H_LOCAL", b), 0.0, atol=0)
        np.testing.assert_allclose(o.tap("H_MIX", b), o.tap("ALPHA", b) * 1.75 * o.tap("X", b), rtol=1e-14)


# ---------------------------------------------------------------------------------------------------
# closed forms
# ---------------------------------------------------------------------------------------------------
def test_embedding_layernorm_flatten_closed_form():
    """Two-valued embedding rows: E[s] = (a_s,...,a_s, b_s,...,b_s) has mean (a+b)/2 and variance
    ((a-b)/2)^2, so LN gives -+1/sqrt(1 + eps/var) on the two halves. X must hold token j (oldest first)
    in channels [jD, (j+1)D)."""
    rng = np.random.default_rng(3)
    o, blob, kw = tiny_oracle()
    B, T, D = kw["B"], kw["T"], kw["D"]
    a = rng.uniform(-1, 1, 256)
    bb = a + rng.uniform(0.2, 1.0, 256) * rng.choice([-1, 1], 256)
    E = np.zeros((256, D))
    E[:, :D // 2] = a[:, None]
    E[:, D // 2:] = bb[:, None]
    blob["E"] = E
    gamma = rng.uniform(0.5, 1.5, D).astype(np.float32)
    beta = rng.uniform(-0.5, 0.5, D).astype(np.float32)
    blob["gamma_e"] = gamma
    blob["beta_e"] = beta
    o.load_weights(blob.data)
    win = windows_for(rng, B, T)
    o.step_probs(win)
    E32 = blob["E"].astype(np.float64)
    for b in range(B):
        X = o.tap("X", b).reshape(T, D)
        for j in range(T):
            s = win[b, j]
            av, bv = E32[s, 0], E32[s, -1]
            var = ((av - bv) / 2.0) ** 2
            mag = abs(av - bv) / 2.0 / math.sqrt(var + 1e-5)
            sign = np.where(np.arange(D) < D // 2, np.sign(av - bv), np.sign(bv - av))
            np.testing.assert_allclose(X[j], sign * mag * gamma + beta, rtol=1e-12, atol=1e-14)


def _selector_blob(rng, kw):
    """Every matrix a scaled selector, every small parameter random and non-default."""
    B, T, D, H, dl, c, k = kw["B"], kw["T"], kw["D"], kw["H"], kw["d_low"], kw["cache_chunk"], kw["conv_k"]
    Dc, De = kw.get("d_cache") or H, kw.get("d_e") or H
    Dh = T * D
    blob = fi.Blob(B, T, D, H, dl, c, k, kw.get("d_cache"), kw.get("d_e"))
    blob["E"] = rng.standard_normal((256, D))
    randomize_small(blob, rng)
    sel = {}
    for name, (ni, no) in dict(W_g=(D, c), W_v=(D, c), W_m=(Dc, Dh), W_r=(Dh, Dh), W_down=(Dh, dl),
                               W_up=(dl, Dh), W_c=(Dh, Dh), W_fg=(Dh, De), W_fv=(Dh, De), W_f=(De, Dh),
                               W_o=(Dh, 256)).items():
        W, src, sc = selector(rng, ni, no)
        blob[name] = W
        sel[name] = (src, sc)
    conv = []
    Wc = np.zeros((k, D, D), np.float32)
    for r in range(k):
        W, src, sc = selector(rng, D, D)
        src = np.roll(np.arange(D), r + 1)
        W = np.zeros((D, D), np.float32)
        W[src, np.arange(D)] = sc
        Wc[r] = W
        conv.append((src, W[src, np.arange(D)].astype(np.float64)))
    blob["W_conv"] = Wc
    sel["W_conv"] = conv
    wu = []
    WU = np.zeros((B, dl, dl), np.float32)
    for b in range(B):
        src = np.roll(np.arange(dl), b + 1)
        sc = rng.uniform(0.5, 1.5, dl) * (b + 1)
        WU[b][src, np.arange(dl)] = sc
        wu.append((src, WU[b][src, np.arange(dl)].astype(np.float64)))
    blob["W_U"] = WU
    sel["W_U"] = wu
    return blob, sel


def _gather_forward(blob, sel, kw, win, M_prev):
    """The model step when every matrix is a scaled selector: each product x @ W is x[src] * scale."""
    T, D, H, c, k = kw["T"], kw["D"], kw["H"], kw["cache_chunk"], kw["conv_k"]
    f8 = lambda n: blob[n].astype(np.float64)
    g = lambda name, x: x[sel[name][0]] * sel[name][1]
    E = f8("E")
    xe = np.stack([ln(E[s], f8("gamma_e"), f8("beta_e")) for s in win])
    xl = np.stack([ln(E[s], f8("gamma_l"), f8("beta_l")) for s in win])
    X = xe.reshape(-1)
    xt = xe[-1]
    slot = gelu(g("W_g", xt)) * g("W_v", xt)
    M = np.concatenate([M_prev[c:], slot])
    Hg = gelu(g("W_m", M)) + f8("lambda_m")[0] * X
    Hl = np.zeros((T, D))
    for j in range(T):
        acc = f8("b_conv").copy()
        for r in range(k):
            s = j - (k - 1) + r
            if s >= 0:
                src, sc = sel["W_conv"][r]
                acc += xl[s][src] * sc
        Hl[j] = gelu(acc)
    Hl = Hl.reshape(-1)
    alpha = sigmoid(g("W_r", X))
    Hmix = alpha * Hg + (1 - alpha) * Hl
    y = g("W_down", ln(Hmix, f8("gamma_c"), f8("beta_c")))
    return dict(X=X, CACHE=M, H_GLOBAL=Hg, H_LOCAL=Hl, ALPHA=alpha, H_MIX=Hmix, Y_DOWN=y), slot


@pytest.mark.parametrize("widths", [{}, SPLIT_WIDTHS])
def test_selector_network_closed_form(widths):
    rng = np.random.default_rng(5)
    o, _, kw = tiny_oracle(**widths)
    B, T, D, H, dl = kw["B"], kw["T"], kw["D"], kw.get("d_cache") or kw["H"], kw["d_low"]
    blob, sel = _selector_blob(rng, kw)
    o.load_weights(blob.data)
    f8 = lambda n: blob[n].astype(np.float64)
    g = lambda name, x: x[sel[name][0]] * sel[name][1]
    M = [np.zeros(H) for _ in range(B)]
    for step in range(T + 2):  # more steps than cache slots: the roll wraps
        win = windows_for(rng, B, T)
        freq, p = o.step_probs(win)
        for b in range(B):
            exp, _ = _gather_forward(blob, sel, kw, win[b], M[b])
            M[b] = exp["CACHE"]
            src, sc = sel["W_U"][b]
            z = exp["Y_DOWN"][src] * sc
            Ha = g("W_up", z)
            Hc = Ha * sigmoid(g("W_c", exp["H_MIX"])) + f8("lambda_c")[0] * exp["H_MIX"]
            u = ln(Hc, f8("gamma_f"), f8("beta_f"))
            Hexp = gelu(g("W_fg", u)) * g("W_fv", u)
            Hout = gelu(ln(g("W_f", Hexp), f8("gamma_o"), f8("beta_o"))) + f8("lambda_o")[0] * Hc
            logits = g("W_o", Hout) + f8("b_o")
            pe = np.exp(logits - logits.max())
            pe /= pe.sum()
            exp.update(Z_BMM=z, H_A=Ha, H_COARSE=Hc, H_EXPAND=Hexp, H_OUT=Hout, LOGITS=logits, PROBS=pe)
            for name, val in exp.items():
                np.testing.assert_allclose(o.tap(name, b), val, rtol=1e-11, atol=1e-13, err_msg=f"{name} step {step}")
            np.testing.assert_allclose(p[b], pe.astype(np.float32), rtol=0, atol=1e-7)


def test_causal_conv_shift_and_padding():
    """Conv taps that are the identity on one tap only: output token j is psi(b + LN(E[w_{j-(k-1)+r0}])),
    and psi(b) where that index is negative (left zero padding: the window never sees the future)."""
    rng = np.random.default_rng(8)
    o, blob, kw = tiny_oracle()
    B, T, D, k = kw["B"], kw["T"], kw["D"], kw["conv_k"]
    bias = rng.uniform(-0.5, 0.5, D).astype(np.float32)
    for r0 in range(k):
        Wc = np.zeros((k, D, D), np.float32)
        Wc[r0] = np.eye(D)
        blob["W_conv"] = Wc
        blob["b_conv"] = bias
        o.load_weights(blob.data)
        win = windows_for(rng, B, T)
        o.step_probs(win)
        E = blob["E"].astype(np.float64)
        for b in range(B):
            Hl = o.tap("H_LOCAL", b).reshape(T, D)
            for j in range(T):
                s = j - (k - 1) + r0
                pre = bias.astype(np.float64) + (ln(E[win[b, s]]) if s >= 0 else 0.0)
                np.testing.assert_allclose(Hl[j], gelu(pre), rtol=1e-12, atol=1e-14)


# ---------------------------------------------------------------------------------------------------
# invariants
# ---------------------------------------------------------------------------------------------------
def test_rolled_cache_equals_recomputed_window(setup):
    """Frozen weights: after at least T model steps over a sliding window, the rolled cache equals the
    GeGLU slots recomputed from scratch for the T symbols of the current window (slot = function of one
    symbol). Needs exactly T slots: cache_chunk = H / T."""
    o, blob, kw, rng = setup
    B, T, H = kw["B"], kw["T"], kw["H"]
    o.load_weights(blob.data)
    data = rng.integers(0, 256, (B, 3 * T), dtype=np.uint8)
    for i in range(T, 3 * T):
        o.step_probs(data[:, i - T:i])
    rolled = [o.tap("CACHE", b) for b in range(B)]
    c = kw["cache_chunk"]
    for j in range(T):  # feed the final window's symbol j as the newest symbol of a fresh context
        o.reset()
        win = np.zeros((B, T), np.uint8)
        win[:, -1] = data[:, 2 * T - 1 + j]
        o.step_probs(win)
        for b in range(B):
            np.testing.assert_array_equal(o.tap("CACHE", b)[-c:], rolled[b][j * c:(j + 1) * c])


def test_streams_are_independent_and_wu_belongs_to_its_stream(setup):
    """Swapping two streams' windows together with their W_U slices swaps their outputs and leaves the
    third stream untouched; giving stream a the slice of stream b (without swapping windows) changes it."""
    o, blob, kw, rng = setup
    B, T = kw["B"], kw["T"]
    win = windows_for(rng, B, T)
    o.load_weights(blob.data)
    _, p0 = o.step_probs(win)
    blob2 = fi.Blob(B, T, kw["D"], kw["H"], kw["d_low"], kw["cache_chunk"], kw["conv_k"])
    blob2.data[:] = blob.data
    blob2["W_U"][[0, 2]] = blob["W_U"][[2, 0]]
    o.load_weights(blob2.data)
    _, p1 = o.step_probs(win[[2, 1, 0]])
    np.testing.assert_array_equal(p1[0], p0[2])
    np.testing.assert_array_equal(p1[2], p0[0])
    np.testing.assert_array_equal(p1[1], p0[1])
    _, p2 = o.step_probs(win)  # W_U swapped, windows not
    assert np.abs(p2[0] - p0[0]).max() > 1e-6


def test_inactive_streams_do_not_advance(setup):
    o, blob, kw, rng = setup
    B, T = kw["B"], kw["T"]
    o.load_weights(blob.data)
    w1, w2 = windows_for(rng, B, T), windows_for(rng, B, T)
    o.step_probs(w1, active=np.array([1, 0, 1], np.uint8))
    _, pa = o.step_probs(w2)
    o.reset()
    o.step_probs(w1[[0, 2, 2]], active=np.array([1, 0, 1], np.uint8))  # stream 1 masked: its window is irrelevant
    o.reset()
    o2, _, _ = tiny_oracle()
    o2.load_weights(blob.data)
    _, pb = o2.step_probs(w2)  # stream 1 never saw w1
    np.testing.assert_array_equal(pa[1], pb[1])
    assert np.abs(pa[0] - pb[0]).max() > 0


def test_bf16_mode_rounds_matrices_only():
    """bf16 configuration = the same arithmetic on weights rounded to bf16 (round-to-nearest-even): feeding
    pre-rounded matrices to an fp32 context gives the identical result."""
    import torch
    rng = np.random.default_rng(2)
    o16, blob, kw = tiny_oracle(dtype=orc.BF16, std=0.4)
    randomize_small(blob, rng)
    o32, _, _ = tiny_oracle(dtype=orc.F32)
    rounded = fi.Blob(kw["B"], kw["T"], kw["D"], kw["H"], kw["d_low"], kw["cache_chunk"], kw["conv_k"])
    rounded.data[:] = blob.data
    for name, shape, init in blob.specs:
        if init == "normal":
            rounded[name] = torch.from_numpy(blob[name].copy()).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.abs(rounded.data - blob.data).max() > 0
    o16.load_weights(blob.data)
    o32.load_weights(rounded.data)
    win = windows_for(rng, kw["B"], kw["T"])
    np.testing.assert_array_equal(o16.step_probs(win)[1], o32.step_probs(win)[1])


# ---------------------------------------------------------------------------------------------------
# progressive ablation levels (the paper's component table): which feature vector feeds the head
# ---------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("level", [1, 2, 3, 4, 5])
def test_ablation_level_feeds_the_head_from_the_right_stage(level):
    """The stages up to the cut are those of the full model (whose taps the closed-form tests pin), and the head is a
    linear layer + softmax, so the truncated model's probabilities can be recomputed by hand from the full model's taps."""
    rng = np.random.default_rng(31)
    full, blob, kw = tiny_oracle(std=0.4)
    randomize_small(blob, rng)
    full.load_weights(blob.data)
    cut = orc.Oracle(orc.make_config(ablation=level, **kw))
    cut.load_weights(blob.data)
    B, T = kw["B"], kw["T"]
    f8 = lambda n: blob[n].astype(np.float64)
    for step in range(T + 1):
        win = windows_for(rng, B, T)
        full.step_probs(win)
        _, p = cut.step_probs(win)
        for b in range(B):
            feat = {1: full.tap("H_GLOBAL", b), 2: full.tap("H_MIX", b),
                    3: full.tap("H_A", b) + f8("lambda_c")[0] * full.tap("H_MIX", b),
                    4: full.tap("H_COARSE", b), 5: full.tap("H_OUT", b)}[level]
            logits = feat @ f8("W_o") + f8("b_o")
            pe = np.exp(logits - logits.max())
            pe /= pe.sum()
            np.testing.assert_allclose(p[b], pe.astype(np.float32), rtol=0, atol=1e-7)
    if level == 1:   # the global stream alone does not see the conv, router or refiner weights
        other = fi.Blob(B, T, kw["D"], kw["H"], kw["d_low"], kw["cache_chunk"], kw["conv_k"])
        other.data[...] = blob.data
        for name in ("W_conv", "W_r", "W_c", "W_fg", "W_f", "W_up"):
            other[name] = other[name] + 0.5
        a, b2 = orc.Oracle(orc.make_config(ablation=1, **kw)), orc.Oracle(orc.make_config(ablation=1, **kw))
        a.load_weights(blob.data); b2.load_weights(other.data)
        win = windows_for(rng, B, T)
        np.testing.assert_array_equal(a.step_probs(win)[1], b2.step_probs(win)[1])


def test_ablation_level_out_of_range_is_refused():
    import ctypes as C
    L = orc.lib()
    h = C.c_void_p()
    assert L.fadeo_create(C.byref(orc.make_config(B=2, T=4, D=4, H=8, ablation=6)), C.byref(h)) == -2
