"""User-defined events (ink_apply_user_events): a per-node term per layer, added between the linear
map and the activation, driven by grouped set / add / clear events; checked against the oracle's
full inference with the same terms -- bit for bit for max / min, to the stated metric for sums."""
import numpy as np
import pytest

import oracle
import synth
from util import Harness
from test_gpu_edge_cases import tiny_model

pytestmark = pytest.mark.gpu

SET, ADD, CLEAR = oracle.USER_SET, oracle.USER_ADD, oracle.USER_CLEAR


def _harness(kind, agg, exact, n=3000, dims=(12, 16, 8), seed=3):
    cfg = synth.WorkloadConfig(8, "t", kind, agg, n, 30000, False, dims, 12, 60, False)
    src, dst = synth.make_graph(cfg)
    X = np.random.default_rng(seed).standard_normal((n, dims[0])).astype(np.float32)
    return Harness(cfg=cfg, graph=(n, src, dst), X=X, model=tiny_model(kind, agg, dims, seed=seed, hidden=12),
                   precision="f32" if exact else "f64"), np.random.default_rng(seed + 100)


@pytest.mark.parametrize("kind,agg,exact", [("sage", "max", True), ("sage", "min", True), ("gin", "sum", False),
                                            ("sage", "mean", False), ("gin", "max", True), ("gcn", "gcn_sym", False)])
def test_user_events_match_the_oracle(kind, agg, exact):
    h, rng = _harness(kind, agg, exact)
    n, stride = h.n, 16
    # grouped by (layer, target) in list order: repeated targets, both layers, all three operations
    ev, rows = [], []
    for i in range(300):
        ev.append((int(rng.integers(1, 3)), int(rng.integers(0, 40)), int(rng.choice([SET, ADD, ADD, CLEAR]))))
        rows.append(rng.standard_normal(stride) * 2)
    res, want = h.user_step(ev, np.array(rows, np.float32), exact=exact)
    assert want.size > 0
    assert np.array_equal(h.ink.get_layer(1, 5), h.user_terms[0]) and np.array_equal(h.ink.get_layer(2, 5), h.user_terms[1])
    h.check_state(exact=exact)
    # the terms stay in force: edge batches, feature updates and a rebuilt cache all see them
    for b in range(2):
        op, bs, bd = h.sampler.next_batch()
        h.step(op, bs, bd, exact=exact)
    ids = rng.choice(n, size=30, replace=False)
    h.feature_step(ids, rng.standard_normal((30, h.X.shape[1])).astype(np.float32), exact=exact)
    h.ink.full_infer()
    h.check_state(exact=exact)
    # events that change nothing bitwise give an empty result; clearing restores the plain model
    res, want = h.user_step([(1, 5, ADD), (2, 7, ADD)], np.zeros((2, stride), np.float32), exact=exact)
    assert want.size == 0 and res["n_changed"] == 0
    touched = sorted({(l, t) for l, t, _ in ev})
    h.user_step([(l, t, CLEAR) for l, t in touched], np.zeros((len(touched), stride), np.float32), exact=exact)
    assert not h.ink.get_layer(1, 5).any() and not h.ink.get_layer(2, 5).any()
    h.check_state(exact=exact)
    h.ink.close()


def test_user_events_only_on_the_last_layer_and_many_targets():
    h, rng = _harness("sage", "max", True, n=20000, dims=(8, 8, 6))
    targets = rng.choice(h.n, size=6000, replace=False)         # more rows than the single-workgroup forms take
    ev = [(2, int(t), SET) for t in targets]
    res, want = h.user_step(ev, rng.standard_normal((len(ev), 6)).astype(np.float32))
    assert np.array_equal(want, np.sort(targets))
    st = h.ink.stats()["layers"]
    assert st[0]["n_transformed"] == 0 and st[1]["n_transformed"] == 6000
    h.check_state()
    h.ink.close()


def test_user_event_errors_change_nothing():
    from paper_2309_11071_amd import InkError
    h, rng = _harness("sage", "max", True)
    before = h.ink.get_layer(2, 0)
    row = np.zeros((1, 16), np.float32)
    for ev, code, r in (([(3, 0, SET)], 5, row), ([(0, 0, SET)], 5, row), ([(1, h.n, SET)], 5, row), ([(1, -1, SET)], 5, row),
                        ([(1, 0, 7)], 1, row), ([(1, 0, SET)], 1, np.zeros((1, 8), np.float32))):     # stride 8 < width 16
        with pytest.raises(InkError) as e:
            h.ink.apply_user_events(ev, r)
        assert e.value.status == code
    with pytest.raises(InkError):
        h.ink.get_layer(1, 5)                     # no event ever named the layer: no term table
    assert np.array_equal(before, h.ink.get_layer(2, 0))
    res = h.ink.apply_user_events([], np.zeros((0, 16), np.float32))
    assert res["n_changed"] == 0
    h.ink.close()
