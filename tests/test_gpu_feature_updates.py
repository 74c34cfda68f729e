"""Vertex feature updates (ink_update_features) against the oracle's full inference with the new
feature table: the changed rows enter layer 1 as changed sources (Sec. 2.4) and as rows whose own
next embedding depends on them (Sec. 3.2)."""
import numpy as np
import pytest

import synth
from util import Harness
from test_gpu_edge_cases import tiny_model, star

pytestmark = pytest.mark.gpu


def harness(kind, agg, dims, n=1500, e=12000, seed=4, exact=True, integer_features=False):
    cfg = synth.WorkloadConfig(8, "t", kind, agg, n, e, False, tuple(dims), 12, 50, False)
    src, dst = synth.make_graph(cfg)
    rng = np.random.default_rng(seed)
    if integer_features:
        X = rng.integers(-3, 4, size=(n, dims[0])).astype(np.float32)
    else:
        X = rng.standard_normal((n, dims[0])).astype(np.float32)
    return Harness(cfg=cfg, graph=(n, src, dst), X=X, model=tiny_model(kind, agg, dims, seed=seed + 1, hidden=12),
                   precision="f32" if exact else "f64", slack=0.1), rng


@pytest.mark.parametrize("kind,agg,exact", [("sage", "max", True), ("sage", "min", True), ("gin", "max", True),
                                            ("gin", "sum", False), ("sage", "mean", False), ("sage", "sum", False),
                                            ("gcn", "gcn_sym", False)])
def test_random_feature_updates(kind, agg, exact):
    dims = (10, 12, 7)
    h, rng = harness(kind, agg, dims, exact=exact)
    for size in (1, 7, 60, 400):
        ids = rng.choice(h.n, size=size, replace=False)
        rows = rng.standard_normal((size, dims[0])).astype(np.float32)
        res, want = h.feature_step(ids, rows, exact=exact, tol=1e-5)
        assert want.size > 0
    h.check_state(exact=exact, tol=1e-5)
    h.check_bound()
    h.ink.close()


def test_unchanged_and_partly_changed_rows():
    """Rows written with their present values are not events; a single changed column is."""
    dims = (6, 5, 4)
    h, rng = harness("sage", "max", dims, n=400, e=3000, integer_features=True)
    ids = rng.choice(h.n, size=50, replace=False)
    res, want = h.feature_step(ids, h.X[ids].copy())
    assert res["n_changed"] == 0 and want.size == 0
    rows = h.X[ids].copy()
    rows[::2, 3] += 1.0
    res, want = h.feature_step(ids, rows)
    assert res["n_changed"] == want.size
    res, want = h.feature_step(np.zeros(0, np.int32), np.zeros((0, dims[0]), np.float32))
    assert res["n_changed"] == 0
    h.check_state()
    h.check_bound()
    h.ink.close()


def test_holder_gets_worse_and_recovers_on_a_star():
    """Feature changes of the leaf that holds the maximum: a decrease that stays above the
    runner-up changes nothing else, one below it hands the dimensions to the recorded runner-up,
    a second such change exposes the centre, and restoring the rows restores the cache."""
    d = 4
    graph, X = star(12, d, seed=3)
    X[1:13] = np.random.default_rng(5).uniform(0.0, 1.0, size=(12, d)).astype(np.float32)
    X[5] = 10.0            # leaf 5 holds every dimension of the centre, runner-up < 1
    h = Harness(graph=graph, X=X, model=tiny_model("sage", "max", (d, 3, 2), seed=2), precision="f32", profile=True)
    x5 = h.X[5].copy()
    h.feature_step([5], (x5 - 5.0)[None, :])          # 5.0: still above every other leaf
    assert h.ink.stats()["layers"][0]["n_exposed"] == 0
    h.feature_step([5], np.full((1, d), -1.0, np.float32))   # below the runner-up: it takes over
    assert h.ink.stats()["layers"][0]["n_exposed"] == 0
    new_holders = sorted(set(h.ink.get_layer(1, 2)[0].tolist()))
    assert 5 not in new_holders
    rows = np.full((len(new_holders), d), -2.0, np.float32)
    h.feature_step(new_holders, rows)                        # they drop as well, nobody recorded behind: recompute
    assert h.ink.stats()["layers"][0]["n_exposed"] == 1
    h.feature_step([5], x5[None, :])
    h.check_state()
    h.check_bound()
    assert np.array_equal(h.ink.get_layer(1, 2)[0], np.full(d, 5, np.int32))
    h.ink.close()


@pytest.mark.parametrize("kind,agg,exact", [("sage", "max", True), ("gin", "sum", False), ("gcn", "gcn_sym", False)])
def test_feature_and_edge_updates_interleaved(kind, agg, exact):
    dims = (8, 9, 5)
    h, rng = harness(kind, agg, dims, n=800, e=6000, exact=exact)
    for it in range(4):
        ids = rng.choice(h.n, size=30, replace=False)
        h.feature_step(ids, rng.standard_normal((30, dims[0])).astype(np.float32), exact=exact, tol=1e-5)
        src, dst = synth.keys_to_edges(h.keys)
        pick = rng.choice(src.size, size=40, replace=False)
        op = np.concatenate([np.ones(40, np.uint8), np.zeros(40, np.uint8)])
        s = np.concatenate([src[pick], rng.integers(0, h.n, size=40).astype(np.int32)])
        d = np.concatenate([dst[pick], rng.integers(0, h.n, size=40).astype(np.int32)])
        h.step(op, s, d, exact=exact, tol=1e-5)
    h.check_state(exact=exact, tol=1e-5)
    h.check_graph()
    h.ink.close()


def test_wide_features():
    """Feature rows wider than one aggregation block (602 columns)."""
    dims = (602, 16, 8)
    h, rng = harness("sage", "max", dims, n=300, e=2500)
    ids = rng.choice(h.n, size=40, replace=False)
    h.feature_step(ids, rng.standard_normal((40, dims[0])).astype(np.float32))
    h.check_state()
    h.ink.close()


def test_error_paths_leave_the_state_untouched():
    from paper_2309_11071_amd.binding import InkError
    dims = (5, 4, 3)
    h, rng = harness("sage", "max", dims, n=200, e=1200)
    with pytest.raises(InkError):
        h.ink.update_features(np.array([3, 9, 3], np.int32), np.zeros((3, dims[0]), np.float32))
    with pytest.raises(InkError):
        h.ink.update_features(np.array([3, h.n], np.int32), np.zeros((2, dims[0]), np.float32))
    with pytest.raises(InkError):
        h.ink.update_features(np.array([-1], np.int32), np.zeros((1, dims[0]), np.float32))
    h.check_state()
    assert np.array_equal(h.ink.get_layer(0, 0), h.X)
    h.ink.close()


def test_device_resident_arguments_match_host_arguments():
    """Update batches and feature rows handed over as device pointers (batch_mem = device) give the
    same result, bit for bit, as the host-pointer calls that the other tests check against the oracle."""
    import torch
    from paper_2309_11071_amd import Ink
    from paper_2309_11071_amd.binding import make_updates
    dims = (8, 9, 5)
    h, rng = harness("sage", "max", dims, n=900, e=7000)
    rp, col = h.ink.get_graph()
    dev = Ink(rp, col, h.X, h.model, slack_factor=0.1, batch_device=True)
    dev.full_infer()

    def fetch(r):      # copy out of the library-owned device buffers
        from paper_2309_11071_amd.binding import _dtoh
        a = np.empty(r["n_changed"], np.int32)
        b = np.empty((r["n_changed"], dims[-1]), np.float32)
        if r["n_changed"]:
            _dtoh(a, r["changed_ids_ptr"])
            _dtoh(b, r["embeddings_ptr"])
        return a, b

    for it in range(3):
        ids = rng.choice(h.n, size=25, replace=False).astype(np.int32)
        rows = rng.standard_normal((25, dims[0])).astype(np.float32)
        res, _ = h.feature_step(ids, rows)
        t_ids = torch.from_numpy(ids).cuda()
        t_rows = torch.from_numpy(rows).cuda()
        torch.cuda.synchronize()
        a, b = fetch(dev.update_features_device(t_ids.data_ptr(), t_rows.data_ptr(), ids.size))
        assert np.array_equal(a, res["changed_ids"]) and np.array_equal(b.view(np.uint32), res["embeddings"].view(np.uint32))
        src, dst = synth.keys_to_edges(h.keys)
        pick = rng.choice(src.size, size=30, replace=False)
        op = np.concatenate([np.ones(30, np.uint8), np.zeros(30, np.uint8)])
        s = np.concatenate([src[pick], rng.integers(0, h.n, size=30).astype(np.int32)])
        d = np.concatenate([dst[pick], rng.integers(0, h.n, size=30).astype(np.int32)])
        res, _ = h.step(op, s, d)
        upd = make_updates(op, s, d)
        t_upd = torch.from_numpy(upd.view(np.uint8).copy()).cuda()
        torch.cuda.synchronize()
        r = dev.apply_updates_device(t_upd.data_ptr(), upd.size)
        assert (r["n_applied_ins"], r["n_applied_del"], r["n_noop"]) == (res["n_applied_ins"], res["n_applied_del"], res["n_noop"])
        a, b = fetch(r)
        assert np.array_equal(a, res["changed_ids"]) and np.array_equal(b.view(np.uint32), res["embeddings"].view(np.uint32))
    for l in range(1, 3):
        assert np.array_equal(dev.get_layer(l, 0).view(np.uint32), h.ink.get_layer(l, 0).view(np.uint32))
    dev.close()
    h.ink.close()
