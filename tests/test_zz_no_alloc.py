"""The entry point that allocates nothing (fade_coder_encode_tables_noalloc: coder state in the library's own device array)
against the allocating one it mirrors, through the C ABI: same tables and symbols in, byte-identical payloads and lengths
out, on two calls in a row, the second smaller than the first (the shared array keeps the first call's contents)."""
import numpy as np
import pytest

import fade_inputs as fi
import oracle as orc
from gpu_helpers import need_gpu

pytestmark = pytest.mark.gpu


def _case(rng, n_streams, n_steps, conc):
    f = orc.quantize(rng.dirichlet(np.full(256, conc), n_steps * n_streams).astype(np.float32)).reshape(n_steps, n_streams, 256)
    cdf = np.cumsum(f.astype(np.int64), 2)
    sym = (cdf > rng.integers(0, 65536, (n_steps, n_streams, 1))).argmax(2).astype(np.uint8)
    sym[::5] = rng.integers(0, 256, sym[::5].shape, dtype=np.uint8)   # atypical symbols: long codes, carries
    return f, sym


def test_no_alloc_coder_matches_the_allocating_entry_point():
    torch = need_gpu()
    import paper_2604_07239_amd as fa
    B, T, D, H = 4, 8, 32, 64
    g = fa.Fade(fa.make_config(B, T, D, H, dtype=fa.BF16))
    g.load_weights(fi.init_blob(B, T, D, H, 1).data)
    rng = np.random.default_rng(11)
    for n_streams, n_steps, conc in ((301, 90, 0.1), (37, 40, 2.0)):   # the second call is the smaller one
        f, sym = _case(rng, n_streams, n_steps, conc)
        cap = 2 * n_steps + 16
        print(f"no-alloc coder: streams={n_streams} steps={n_steps}", flush=True)
        fd = torch.from_numpy(f.view(np.int16)).cuda()
        sd = torch.from_numpy(sym).cuda()
        res = []
        for call in (g.coder_encode_tables, g.coder_encode_tables_noalloc):
            out = torch.full((n_streams, cap), 0xA5, dtype=torch.uint8, device="cuda")
            ln = torch.full((n_streams,), -1, dtype=torch.int32, device="cuda")
            call(fd, sd, n_steps, n_streams, out, cap, ln)
            res.append((out.cpu().numpy(), ln.cpu().numpy().astype(np.int64)))
        (out_a, len_a), (out_n, len_n) = res
        np.testing.assert_array_equal(len_n, len_a)
        assert len_a.min() > 0
        for k in range(n_streams):
            assert out_n[k, :len_n[k]].tobytes() == out_a[k, :len_a[k]].tobytes(), k
        # and the oracle's coder writes the same bytes (the allocating entry point's own parity bar)
        ref = orc.coder_encode(f[:, 0], sym[:, 0])
        assert out_n[0, :len_n[0]].tobytes() == ref.tobytes()
        # decode what the no-alloc call wrote
        dec = torch.zeros((n_steps, n_streams), dtype=torch.uint8, device="cuda")
        g.coder_decode_tables(fd, n_steps, n_streams, torch.from_numpy(out_n).cuda(), cap, torch.from_numpy(len_n.astype(np.int32)).cuda(), dec)
        np.testing.assert_array_equal(dec.cpu().numpy(), sym)
    with pytest.raises(fa.FadeError) as e:   # beyond the array's size: refused on the host, nothing launched
        g.coder_encode_tables_noalloc(fd, sd, 1, 65537, out, cap, ln)
    assert e.value.code == -1
    g.close()
