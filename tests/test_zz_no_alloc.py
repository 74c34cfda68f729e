"""ink_full_infer_noalloc (full inference with its work memory in a static device array) against
ink_full_infer: every cached table must be identical bit for bit, on two calls in a row that share
the array, the second on a smaller graph, and again after an update batch."""
import numpy as np
import pytest

import synth

pytestmark = pytest.mark.gpu


def _tables(ink, k, select):
    out = []
    for l in range(1, k + 1):
        for which in ((0, 1, 2, 3, 4) if select else (0, 1)):
            out.append(ink.get_layer(l, which).view(np.uint32).copy())
    return out


def _make(cfg):
    from paper_2309_11071_amd import Ink
    src, dst = synth.make_graph(cfg)
    rp, col = synth.in_csr_from_edges(cfg.n_nodes, src, dst)
    return Ink(rp, col, synth.make_features(cfg), synth.make_model(cfg)), (src, dst), int(np.diff(rp).max())


@pytest.mark.parametrize("cfg_id,div_big,div_small", [(1, 1, 4), (4, 256, 1024), (2, 64, 256)])
def test_no_alloc_full_inference_matches(cfg_id, div_big, div_small):
    from paper_2309_11071_amd.binding import make_updates
    big_cfg, small_cfg = synth.get_config(cfg_id, div_big), synth.get_config(cfg_id, div_small)
    select = big_cfg.agg in ("max", "min")
    k = big_cfg.n_layers
    a, (src, dst), maxdeg = _make(big_cfg)
    b, _, _ = _make(small_cfg)
    assert maxdeg > 1024          # long rows exist: the chunked path, whose partial rows live in the array, runs
    a.full_infer(); b.full_infer()
    want_a, want_b = _tables(a, k, select), _tables(b, k, select)
    # two calls in a row on the shared array, the second with the smaller input
    a.full_infer_noalloc()
    b.full_infer_noalloc()
    for got, want in zip(_tables(a, k, select), want_a):
        assert np.array_equal(got, want)
    for got, want in zip(_tables(b, k, select), want_b):
        assert np.array_equal(got, want)
    # after an update the cache rebuilt without allocation equals the one rebuilt with it
    op, bs, bd = synth.BatchSampler(big_cfg, src, dst).next_batch()
    a.apply_updates(make_updates(op, bs, bd))
    a.full_infer_noalloc()
    got = _tables(a, k, select)
    a.full_infer()
    for g, w in zip(got, _tables(a, k, select)):
        assert np.array_equal(g, w)
    a.close(); b.close()


def test_no_alloc_rejects_what_does_not_fit():
    from paper_2309_11071_amd import Ink, InkError
    # GIN staging rows alone (200 000 nodes x 128 floats) exceed the 64 MiB array
    n = 200_000
    rng = np.random.default_rng(3)
    src = rng.integers(0, n, 50_000).astype(np.int32)
    dst = rng.integers(0, n, 50_000).astype(np.int32)
    keep = src != dst
    keys = np.unique(synth.edge_keys(src[keep], dst[keep]))
    src, dst = (keys & 0xFFFFFFFF).astype(np.int32), (keys >> 32).astype(np.int32)
    rp, col = synth.in_csr_from_edges(n, src, dst)
    cfg = synth.WorkloadConfig(4, "t", "gin", "sum", n, 1, False, (16, 16, 16), 128, 2, False)
    X = rng.standard_normal((n, 16)).astype(np.float32)
    ink = Ink(rp, col, X, synth.make_model(cfg))
    ink.full_infer()
    before = ink.get_layer(2, 0)
    with pytest.raises(InkError) as e:
        ink.full_infer_noalloc()
    assert e.value.status == 5 and "scratch" in str(e.value)
    assert np.array_equal(before, ink.get_layer(2, 0))      # refused before anything ran
    ink.full_infer()                                         # the context stays usable
    ink.close()
