"""GPU parity of the accumulative aggregators (sum, mean, degree-normalised sum) against the
fp64 oracle, at the stated tolerance (max row-relative error 1e-5)."""
import numpy as np
import pytest

import synth
from util import Harness
from test_gpu_edge_cases import tiny_model, star, run, arr, INS, DEL

pytestmark = pytest.mark.gpu
TOL = 1e-5


@pytest.mark.parametrize("kind,agg,dims", [
    ("gin", "sum", (12, 20, 9)),
    ("gin", "sum", (128, 128, 128, 172)),
    ("sage", "sum", (16, 8, 4)),
    ("sage", "mean", (16, 8, 4)),
    ("gcn", "gcn_sym", (40, 24, 7)),
    ("gcn", "gcn_sym", (70, 256, 41)),
    ("gcn", "gcn_sym", (12, 8, 8, 5)),
    ("gin", "sum", (500, 32, 8)),          # aggregated rows wider than 256 floats
    ("sage", "mean", (602, 24, 8)),
    ("gin", "sum", (12, 9)),               # a single layer
    ("gcn", "gcn_sym", (12, 9)),
    ("gin", "sum", (6,) * 9),              # the largest layer count the library takes
    ("gcn", "gcn_sym", (20, 64, 7)),       # narrow outputs over whole rows of 2 and 5 k-chunks
    ("gcn", "gcn_sym", (12, 160, 40)),
    ("sage", "mean", (176, 33, 5)),        # mean over 11 k-chunks
    ("sage", "sum", (80, 64, 8)),
])
def test_random_sequences(kind, agg, dims):
    cfg = synth.WorkloadConfig(6, "t", kind, agg, 3000, 20000, False, tuple(dims), 24, 200, False)
    model = tiny_model(kind, agg, dims, seed=len(dims), hidden=24)
    src, dst = synth.make_graph(cfg)
    X = np.random.default_rng(5).standard_normal((cfg.n_nodes, dims[0])).astype(np.float32)
    h = Harness(cfg=cfg, graph=(cfg.n_nodes, src, dst), X=X, model=model, precision="f64", dense_threshold=-1)
    h.check_state(exact=False, tol=TOL)
    for b in range(5):
        op, bs, bd = h.sampler.next_batch()
        res, want = h.step(op, bs, bd, exact=False, tol=TOL)
        assert res["n_changed"] > 0
        h.check_state(exact=False, tol=TOL)
    h.check_graph()
    h.ink.close()


@pytest.mark.parametrize("kind,agg", [("gin", "sum"), ("gcn", "gcn_sym")])
def test_dense_fallback(kind, agg):
    dims = (10, 12, 6)
    cfg = synth.WorkloadConfig(6, "t", kind, agg, 2000, 15000, False, dims, 16, 400, False)
    model = tiny_model(kind, agg, dims, seed=1, hidden=16)
    src, dst = synth.make_graph(cfg)
    X = np.random.default_rng(6).standard_normal((cfg.n_nodes, dims[0])).astype(np.float32)
    h = Harness(cfg=cfg, graph=(cfg.n_nodes, src, dst), X=X, model=model, precision="f64", dense_threshold=1e-4)
    for b in range(3):
        op, bs, bd = h.sampler.next_batch()
        h.step(op, bs, bd, exact=False, tol=TOL)
        assert any(L["dense"] for L in h.ink.stats()["layers"])
        h.check_state(exact=False, tol=TOL)
    h.ink.close()


def test_no_message_is_counted_twice():
    """A source that changed AND gained / lost an out-edge in the same batch (Sec. 2.4.2 notes such
    duplicates are harmless for min/max; for sums they would be wrong)."""
    n, d = 12, 6
    X = np.random.default_rng(8).standard_normal((n, d)).astype(np.float32)
    # 0 -> 1 -> {2,3,4};  5 -> 1
    src, dst = arr([0, 1, 1, 1, 5]), arr([1, 2, 3, 4, 1])
    h = Harness(graph=(n, src, dst), X=X, model=tiny_model("gin", "sum", (d, 6, 5, 4), hidden=8), precision="f64")
    # node 1 changes in layer 1 (gains 6, loses 5) and at the same time gains out-edge 1->7, loses 1->2
    run_tol(h, [(INS, 6, 1), (DEL, 5, 1), (INS, 1, 7), (DEL, 1, 2)])
    h.check_state(exact=False, tol=TOL)
    run_tol(h, [(DEL, 6, 1), (INS, 1, 2), (DEL, 1, 7), (INS, 5, 1)])
    h.check_state(exact=False, tol=TOL)
    h.check_graph()
    h.ink.close()


def run_tol(h, ops):
    op = arr([o for o, _, _ in ops], np.uint8)
    return h.step(op, arr([s for _, s, _ in ops]), arr([d for _, _, d in ops]), exact=False, tol=TOL)


def test_sum_hub_row_and_gcn_degree_change():
    g, X = star(5000, 8, seed=4, extra=6)
    n = g[0]
    for kind, agg in (("gin", "sum"), ("gcn", "gcn_sym")):
        h = Harness(graph=g, X=X, model=tiny_model(kind, agg, (8, 8, 4), hidden=8), precision="f64")
        h.check_state(exact=False, tol=TOL)
        run_tol(h, [(DEL, 7, 0), (INS, n - 1, 0), (INS, 0, n - 2)])
        h.check_state(exact=False, tol=TOL)
        h.ink.close()


@pytest.mark.parametrize("cfg_id", [2, 4])
def test_scaled_configs(cfg_id):
    cfg = synth.get_config(cfg_id, 256 if cfg_id == 4 else 64)
    h = Harness(cfg, precision="f64")
    h.check_state(exact=False, tol=TOL)
    for b in range(3):
        op, bs, bd = h.sampler.next_batch()
        h.step(op, bs, bd, exact=False, tol=TOL)
    h.check_state(exact=False, tol=TOL)
    h.check_graph()
    h.ink.close()


@pytest.mark.parametrize("kind,agg,exact", [("sage", "max", True), ("gin", "sum", False), ("gcn", "gcn_sym", False)])
def test_affected_area_baseline_reaches_the_same_state(kind, agg, exact):
    """The affected-area recompute and the incremental update may be interleaved freely."""
    dims = (10, 12, 6)
    cfg = synth.WorkloadConfig(6, "t", kind, agg, 2000, 15000, False, dims, 16, 100, False)
    model = tiny_model(kind, agg, dims, seed=2, hidden=16)
    src, dst = synth.make_graph(cfg)
    X = np.random.default_rng(7).standard_normal((cfg.n_nodes, dims[0])).astype(np.float32)
    h = Harness(cfg=cfg, graph=(cfg.n_nodes, src, dst), X=X, model=model, precision="f32" if exact else "f64",
                dense_threshold=-1)
    visited = []
    for b in range(4):
        op, bs, bd = h.sampler.next_batch()
        h.step(op, bs, bd, exact=exact, tol=TOL, affected=(b % 2 == 0))
        visited.append(sum(L["n_targets"] for L in h.ink.stats()["layers"]))
        h.check_state(exact=exact, tol=TOL)
    h.check_graph()
    h.ink.close()
