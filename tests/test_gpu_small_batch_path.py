"""The graph-store update has two forms: short batches (at most 4096 entries) run in one workgroup
per direction with one host read-back, longer ones through the device-wide primitives.  Both must
leave the same store, the same Delta E and hence the same result; each is checked against the
oracle, and against the other bit for bit."""
import numpy as np
import pytest

import synth
from util import Harness
from test_gpu_edge_cases import tiny_model
from test_gpu_fuzz import messy_batch

pytestmark = pytest.mark.gpu


def pair(kind, agg, exact, n=5000, e=40000, dims=(8, 8, 6), slack=0.05, **kw):
    cfg = synth.WorkloadConfig(8, "t", kind, agg, n, e, False, dims, 12, 50, False)
    src, dst = synth.make_graph(cfg)
    X = np.random.default_rng(7).integers(-3, 4, size=(n, dims[0])).astype(np.float32)
    mk = lambda limit: Harness(cfg=cfg, graph=(n, src, dst), X=X, model=tiny_model(kind, agg, dims, seed=5, hidden=8),
                               precision="f32" if exact else "f64", slack=slack, small_batch_limit=limit, **kw)
    return mk(0), mk(-1)


@pytest.mark.parametrize("kind,agg,exact", [("sage", "max", True), ("gin", "sum", False), ("gcn", "gcn_sym", False)])
def test_both_forms_agree_and_match_the_oracle(kind, agg, exact):
    a, b = pair(kind, agg, exact)
    rng = np.random.default_rng(31)
    for size in (1, 2, 63, 64, 65, 255, 257, 1000, 1024, 1025, 3000, 4095, 4096, 4097, 9000, 16383, 16384, 16385):
        op, s, d = messy_batch(rng, a.n, a.keys, size)
        ra, _ = a.step(op, s, d, exact=exact, tol=1e-5)
        rb, _ = b.step(op, s, d, exact=exact, tol=1e-5)
        for k in ("n_applied_ins", "n_applied_del", "n_noop", "n_changed"):
            assert ra[k] == rb[k], (size, k)
        assert np.array_equal(ra["changed_ids"], rb["changed_ids"])
        assert np.array_equal(ra["embeddings"].view(np.uint32), rb["embeddings"].view(np.uint32))
    a.check_graph(); b.check_graph()
    for l in (1, 2):
        assert np.array_equal(a.ink.get_layer(l, 0).view(np.uint32), b.ink.get_layer(l, 0).view(np.uint32))
    a.ink.close(); b.ink.close()


def test_degenerate_short_batches():
    """Only self loops, only no-ops, one edge inserted and deleted many times, every op on one node."""
    a, b = pair("sage", "max", True, n=300, e=2000)
    n = a.n
    src, dst = synth.keys_to_edges(a.keys)
    u8 = lambda x: np.asarray(x, np.uint8)
    i32 = lambda x: np.asarray(x, np.int32)
    have = set(synth.edge_keys(src, dst).tolist())
    absent = [(u, v) for u in range(5) for v in range(5, 10)
              if int(synth.edge_keys(np.asarray([u], np.int32), np.asarray([v], np.int32))[0]) not in have]
    cases = [
        (u8([0, 1, 0]), i32([3, 4, 5]), i32([3, 4, 5])),                                   # self loops
        (u8([0] * 4), i32(src[:4]), i32(dst[:4])),                                          # already present
        (u8([1] * len(absent)), i32([p[0] for p in absent]), i32([p[1] for p in absent])),  # already absent
        (u8([0, 1] * 50 + [0]), i32([absent[0][0]] * 101), i32([absent[0][1]] * 101)),      # ends inserted
        (u8([0] * 200), i32(np.arange(20, 220) % n), i32([7] * 200)),                       # one destination
        (u8([0] * 200), i32([9] * 200), i32(np.arange(30, 230) % n)),                       # one source
        (u8([1] * 150), i32(np.arange(20, 170) % n), i32([7] * 150)),                       # and away again
    ]
    for op, s, d in cases:
        ra, _ = a.step(op, s, d)
        rb, _ = b.step(op, s, d)
        assert (ra["n_applied_ins"], ra["n_applied_del"], ra["n_noop"]) == (rb["n_applied_ins"], rb["n_applied_del"], rb["n_noop"])
        assert np.array_equal(ra["changed_ids"], rb["changed_ids"])
        a.check_graph(); b.check_graph()
    a.check_state(); b.check_state()
    a.ink.close(); b.ink.close()


@pytest.mark.parametrize("limit,size", [(0, 300), (0, 3000), (-1, 300), (-1, 10000)])
def test_malformed_device_batches_are_dropped_whole(limit, size):
    """A device-resident batch is validated by the first kernel of the graph stage: one bad entry
    drops the batch before any block is touched, and the next batch is served as usual."""
    import torch
    from paper_2309_11071_amd import Ink
    from paper_2309_11071_amd.binding import InkError, make_updates
    h, _ = pair("sage", "max", True, n=400, e=3000)
    rp, col = h.ink.get_graph()
    dev = Ink(rp, col, h.X, h.model, slack_factor=0.05, batch_device=True, small_batch_limit=limit)
    dev.full_infer()
    before = dev.get_layer(2, 0).copy()
    rng = np.random.default_rng(3)
    op, s, d = messy_batch(rng, h.n, h.keys, size)
    for pos, (bo, bs, bd, code) in enumerate([(0, h.n, 1, 5), (0, 2, -1, 5), (9, 1, 2, 1)]):
        o2, s2, d2 = op.copy(), s.copy(), d.copy()
        o2[17 + pos], s2[17 + pos], d2[17 + pos] = bo, bs, bd
        upd = make_updates(o2, s2, d2)
        t = torch.from_numpy(upd.view(np.uint8).copy()).cuda()
        torch.cuda.synchronize()
        with pytest.raises(InkError) as e:
            dev.apply_updates_device(t.data_ptr(), upd.size)
        assert e.value.status == code
        rp2, col2 = dev.get_graph()
        assert np.array_equal(rp, rp2) and np.array_equal(col, col2)
        assert np.array_equal(before.view(np.uint32), dev.get_layer(2, 0).view(np.uint32))
    res, _ = h.step(op, s, d)
    upd = make_updates(op, s, d)
    t = torch.from_numpy(upd.view(np.uint8).copy()).cuda()
    torch.cuda.synchronize()
    r = dev.apply_updates_device(t.data_ptr(), upd.size)
    assert (r["n_applied_ins"], r["n_applied_del"], r["n_changed"]) == (res["n_applied_ins"], res["n_applied_del"], res["n_changed"])
    assert np.array_equal(dev.get_layer(2, 0).view(np.uint32), h.ink.get_layer(2, 0).view(np.uint32))
    dev.close(); h.ink.close()


@pytest.mark.parametrize("limit", [0, -1])
def test_blocks_and_pools_grow_in_both_forms(limit):
    n, d = 3000, 4
    X = np.random.default_rng(2).standard_normal((n, d)).astype(np.float32)
    h = Harness(graph=(n, np.asarray([1, 2], np.int32), np.asarray([0, 0], np.int32)), X=X,
                model=tiny_model("sage", "max", (d, 4, 4)), slack=0.01, pool_reserve=1024, small_batch_limit=limit)
    for r in range(3):
        lo, hi = 10 + 600 * r, 10 + 600 * (r + 1)
        u = np.arange(lo, hi, dtype=np.int32)
        op = np.zeros(2 * u.size, np.uint8)
        h.step(op, np.concatenate([u, np.full(u.size, 5, np.int32)]), np.concatenate([np.zeros(u.size, np.int32), u]))
        h.check_graph()
    h.check_state()
    h.ink.close()


@pytest.mark.parametrize("kind,agg,exact", [("sage", "max", True), ("gin", "min", True), ("gin", "sum", False),
                                            ("gcn", "gcn_sym", False), ("sage", "mean", False)])
def test_short_layers_on_a_graph_with_a_long_bitmap(kind, agg, exact):
    """Above 16 384 nodes a layer with few events collects its rows from the grouped targets, the
    sources and the degree-changed nodes instead of scanning the changed-row bitmap: small edge
    batches and feature updates, three layers, so that layers of every size class occur."""
    dims = (8, 8, 8, 6)
    n = 20000
    cfg = synth.WorkloadConfig(8, "t", kind, agg, n, 60000, False, dims, 12, 50, False)
    src, dst = synth.make_graph(cfg)
    rng = np.random.default_rng(41)
    X = rng.integers(-3, 4, size=(n, dims[0])).astype(np.float32)
    h = Harness(cfg=cfg, graph=(n, src, dst), X=X, model=tiny_model(kind, agg, dims, seed=5, hidden=8),
                precision="f32" if exact else "f64", slack=0.05, profile=True)
    small_layers = 0
    for size in (1, 3, 20, 90, 300, 700, 2500):
        op, s, d = messy_batch(rng, n, h.keys, size)
        h.step(op, s, d, exact=exact, tol=1e-5)
        small_layers += sum(1 for L in h.ink.stats()["layers"] if 0 < L["n_events"] <= 4096)
        ids = rng.choice(n, size=min(size, 40), replace=False)
        h.feature_step(ids, rng.integers(-3, 4, size=(ids.size, dims[0])).astype(np.float32), exact=exact, tol=1e-5)
    assert small_layers >= 6
    h.check_graph()
    h.check_state(exact=exact, tol=1e-5)
    if exact:
        h.check_bound()
    h.ink.close()


@pytest.mark.parametrize("kind,agg,exact", [("sage", "max", True), ("gin", "sum", False), ("gcn", "gcn_sym", False)])
def test_mixed_stream_of_every_kind_of_call(kind, agg, exact):
    """Edge batches of both forms, feature updates and node arrivals in random order on one
    context (20 000 nodes, three layers); every call is checked against the oracle."""
    from test_gpu_add_nodes import edges_touching
    dims = (8, 8, 8, 6)
    n = 20000
    cfg = synth.WorkloadConfig(8, "t", kind, agg, n, 60000, False, dims, 12, 50, False)
    src, dst = synth.make_graph(cfg)
    rng = np.random.default_rng(77)
    X = rng.integers(-3, 4, size=(n, dims[0])).astype(np.float32)
    h = Harness(cfg=cfg, graph=(n, src, dst), X=X, model=tiny_model(kind, agg, dims, seed=9, hidden=8),
                precision="f32" if exact else "f64", slack=0.05, node_capacity=n + 200)
    for it in range(24):
        what = int(rng.integers(0, 5))
        if what == 0:
            op, s, d = messy_batch(rng, h.n, h.keys, int(rng.integers(1, 60)))
            h.step(op, s, d, exact=exact, tol=1e-5)
        elif what == 1:
            op, s, d = messy_batch(rng, h.n, h.keys, int(rng.integers(300, 4000)))
            h.step(op, s, d, exact=exact, tol=1e-5)
        elif what == 2:
            op, s, d = messy_batch(rng, h.n, h.keys, int(rng.integers(4097, 9000)))
            h.step(op, s, d, exact=exact, tol=1e-5)
        elif what == 3:
            ids = rng.choice(h.n, size=int(rng.integers(1, 80)), replace=False)
            h.feature_step(ids, rng.integers(-3, 4, size=(ids.size, dims[0])).astype(np.float32), exact=exact, tol=1e-5)
        elif h.n + 8 <= n + 200:
            lo = h.n
            h.add_nodes(rng.integers(-3, 4, size=(int(rng.integers(1, 8)), dims[0])).astype(np.float32), exact=exact)
            op, s, d = edges_touching(rng, h, lo, 30)
            h.step(op, s, d, exact=exact, tol=1e-5)
    h.check_graph()
    h.check_state(exact=exact, tol=1e-5)
    if exact:
        h.check_bound()
    h.ink.close()
