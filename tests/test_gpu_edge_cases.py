"""Edge cases of the incremental max/min path on the GPU, each checked against the oracle."""
import numpy as np
import pytest

import oracle
import synth
from util import Harness

pytestmark = pytest.mark.gpu

INS, DEL = 0, 1


def arr(x, dt=np.int32):
    return np.asarray(x, dtype=dt)


def tiny_model(kind, agg, dims, seed=0, hidden=8):
    cfg = synth.WorkloadConfig(7, "t", kind, agg, 1, 1, False, tuple(dims), hidden, 2, False)
    rng = np.random.default_rng(seed)
    model = synth.make_model(cfg, bias_scale=0.3)
    for L in model["layers"]:
        for k in list(L):
            if isinstance(L[k], np.ndarray):
                L[k] = (rng.standard_normal(L[k].shape) * 0.4).astype(np.float32)
    return model


def star(n_leaves, d, seed=0, extra=4):
    """Leaves 1..n_leaves point to 0; `extra` isolated spare nodes follow."""
    n = 1 + n_leaves + extra
    src = np.arange(1, n_leaves + 1, dtype=np.int32)
    dst = np.zeros(n_leaves, np.int32)
    X = np.random.default_rng(seed).standard_normal((n, d)).astype(np.float32)
    return (n, src, dst), X


def run(h, ops):
    op = arr([o for o, _, _ in ops], np.uint8)
    return h.step(op, arr([s for _, s, _ in ops]), arr([d for _, _, d in ops]))


def test_reset_conditions_on_a_star():
    """No reset, covered reset, exposed reset and the equal-value corner cases (Sec. 2.5.1)."""
    g, X = star(6, 4, extra=6)
    # dimension 0: leaf 3 holds the max; dimension 1: leaves 2 and 5 tie (lowest id 2 holds it)
    X[1:7, 0] = [1, 2, 9, 3, 4, 5]
    X[1:7, 1] = [0, 7, 1, 2, 7, 3]
    X[7:, 0] = [10, 9, 8.5, -5, 0, 0]      # spare nodes 7.. used as inserted sources
    X[7:, 1] = [0, 7, 0, -5, 0, 0]
    X[:, 2:4] = -1.0                        # dimensions 2, 3: leaf 6 holds them while it is there
    X[6, 2:4] = 50.0
    model = tiny_model("sage", "max", (4, 4, 3))
    h = Harness(graph=g, X=X, model=model)
    def cond():      # (no deletion, deletion without effect, covered, exposed) of layer 1's only target
        L = h.ink.stats()["layers"][0]
        assert L["n_targets"] == 1
        return (L["n_no_deletion"], L["n_deletion_no_effect"], L["n_covered"], L["n_exposed"])
    run(h, [(DEL, 1, 0)])                         # deletion without effect: no reset
    assert cond() == (0, 1, 0, 0)
    h.check_state()
    run(h, [(DEL, 3, 0), (INS, 7, 0)])            # holder deleted, inserted 10 > 9: covered
    assert cond() == (0, 0, 1, 0)
    h.check_state()
    run(h, [(DEL, 7, 0), (INS, 9, 0)])            # holder deleted, inserted 8.5 < 10 but above every other
    assert cond() == (0, 0, 1, 0)                 # neighbour: covered thanks to the cached runner-up bound
    h.check_state()
    run(h, [(DEL, 9, 0), (INS, 10, 0)])           # holder deleted, inserted -5 is below the others: the
    assert cond() == (0, 0, 1, 0)                 # recorded runner-up (leaf 6, value 5) takes over
    h.check_state()
    assert h.ink.get_layer(1, 2)[0][0] == 6 and h.ink.get_layer(1, 4)[0][0] == -1
    run(h, [(DEL, 6, 0)])                         # that holder leaves too and nobody is recorded behind it: exposed
    assert cond() == (0, 0, 0, 1)
    h.check_state()
    h.check_bound()
    assert (h.ink.get_layer(1, 4)[0] >= 0).all()  # a recompute leaves the exact runner-up and its id
    run(h, [(INS, 8, 0)])                         # dim 1: 8 ties with value 7 but has a higher id
    assert cond() == (1, 0, 0, 0)
    h.check_state()
    run(h, [(DEL, 2, 0)])                         # tie holder leaves: next lowest id takes over
    h.check_state()
    run(h, [(DEL, 5, 0), (INS, 2, 0)])            # holder deleted, equal value comes back: not strictly covered
    h.check_state()
    run(h, [(INS, 11, 0)])                        # insertion that changes nothing: resilient target
    h.check_state()
    h.check_graph()
    h.ink.close()


def test_empty_and_noop_batches():
    g, X = star(5, 4)
    h = Harness(graph=g, X=X, model=tiny_model("sage", "max", (4, 4, 4)))
    res, want = run(h, [])
    assert res["n_changed"] == 0
    res, want = run(h, [(INS, 1, 0), (DEL, 1, 2), (INS, 3, 3), (INS, 6, 0), (DEL, 6, 0), (DEL, 6, 0)])
    assert res["n_changed"] == 0 and res["n_noop"] == 6 and want.size == 0
    res, _ = run(h, [(INS, 6, 0), (INS, 6, 0), (DEL, 2, 0), (INS, 2, 0), (DEL, 2, 0)])
    assert (res["n_applied_ins"], res["n_applied_del"], res["n_noop"]) == (1, 1, 3)
    h.check_state()
    h.check_graph()
    h.ink.close()


def test_first_and_last_edge_of_a_node():
    n, d = 6, 5
    X = np.random.default_rng(3).standard_normal((n, d)).astype(np.float32)
    src, dst = arr([0, 1]), arr([1, 2])
    h = Harness(graph=(n, src, dst), X=X, model=tiny_model("sage", "max", (d, 4, 3)))
    run(h, [(INS, 4, 5)])                 # node 5 had no in-neighbour: cached alpha is not a bound
    h.check_state()
    run(h, [(DEL, 4, 5), (DEL, 0, 1)])    # back to empty: alpha 0, arg -1
    h.check_state()
    assert (h.ink.get_layer(1, 2)[5] == -1).all() and not h.ink.get_layer(1, 1)[5].any()
    h.check_graph()
    h.ink.close()


@pytest.mark.parametrize("kind,agg,dims", [
    ("sage", "min", (8, 8, 8)),
    ("sage", "max", (100, 47, 5)),        # widths that are not multiples of 4 / 32
    ("sage", "max", (256, 130, 256)),     # full-wave rows
    ("sage", "max", (16, 16, 16, 16)),    # three layers
    ("gin", "max", (12, 20, 9)),
    ("gin", "min", (64, 64, 64)),
    ("sage", "max", (602, 64, 8)),        # feature rows wider than one wave covers: column blocks
    ("gin", "max", (300, 40, 6)),
    ("sage", "max", (12, 7)),             # a single layer
    ("sage", "max", (6,) * 9),            # the largest layer count the library takes
    ("sage", "max", (176, 33, 5)),        # narrow outputs, inputs of 11 k-chunks
    ("sage", "max", (48, 64, 40)),        # 3 and 4 k-chunks, one and two column tiles
    ("sage", "min", (256, 8, 8)),         # 16 k-chunks
])
def test_random_sequences(kind, agg, dims):
    cfg = synth.WorkloadConfig(6, "t", kind, agg, 3000, 20000, False, tuple(dims), 24, 300, True)
    model = tiny_model(kind, agg, dims, seed=len(dims), hidden=24)
    rng = np.random.default_rng(5)
    src, dst = synth.make_graph(cfg)
    X = rng.standard_normal((cfg.n_nodes, dims[0])).astype(np.float32)
    X[rng.random(X.shape) < 0.3] = 0.0                      # exact ties
    h = Harness(cfg=cfg, graph=(cfg.n_nodes, src, dst), X=X, model=model)
    h.check_state()
    h.check_bound(exact=True)
    for b in range(4):
        op, bs, bd = h.sampler.next_batch()
        h.step(op, bs, bd)
        h.check_state()
        h.check_bound()
    h.check_graph()
    h.ink.close()


def test_hub_rows_use_the_cooperative_recompute():
    """A node with thousands of in-neighbours (cooperative chunked path) loses the holders of several dimensions."""
    n_leaves, d = 6000, 8
    g, X = star(n_leaves, d, seed=9, extra=8)
    h = Harness(graph=g, X=X, model=tiny_model("sage", "max", (d, 8, 4)))
    h.check_state()
    arg = h.ink.get_layer(1, 2)[0]
    holders = sorted(set(int(a) for a in arg))
    res, _ = run(h, [(DEL, u, 0) for u in holders[:3]])      # the recorded runners-up take over
    assert h.ink.stats()["layers"][0]["n_exposed"] == 0
    h.check_state()
    arg2 = h.ink.get_layer(1, 2)[0]
    res, _ = run(h, [(DEL, int(u), 0) for u in sorted(set(arg2.tolist()) - set(arg.tolist()))])
    assert h.ink.stats()["layers"][0]["n_exposed"] == 1       # nobody recorded behind them: cooperative recompute
    h.check_state()
    h.check_bound(max_nodes=10000)
    assert (h.ink.get_layer(1, 4)[0] >= 0).all()  # the recompute recorded the runner-up of every dimension
    run(h, [(INS, u, 0) for u in holders[:3]] + [(DEL, holders[-1], 0)])
    h.check_state()
    h.check_graph()
    h.ink.close()


def test_blocks_outgrow_their_slack_and_the_pool():
    n, d = 3000, 4
    rng = np.random.default_rng(2)
    X = rng.standard_normal((n, d)).astype(np.float32)
    src, dst = arr([1, 2]), arr([0, 0])
    h = Harness(graph=(n, src, dst), X=X, model=tiny_model("sage", "max", (d, 4, 4)), slack=0.01,
                pool_reserve=1024)     # forces the pool itself to be re-allocated
    for r in range(4):       # node 0 gains hundreds of in-edges, node 5 hundreds of out-edges, per batch
        lo, hi = 10 + 600 * r, 10 + 600 * (r + 1)
        ops = [(INS, u, 0) for u in range(lo, hi)] + [(INS, 5, v) for v in range(lo, hi)]
        run(h, ops)
        h.check_graph()
        h.check_state()
    run(h, [(DEL, u, 0) for u in range(10, 1500)])
    h.check_graph()
    h.check_state()
    h.ink.close()


def test_insert_then_delete_restores_the_cache_exactly():
    cfg = synth.get_config(1, 4)
    h = Harness(cfg)
    before = [h.ink.get_layer(l, w) for l in (1, 2) for w in (0, 1, 2)]
    op, bs, bd = h.sampler.next_batch()
    h.step(op, bs, bd)
    h.step((1 - op)[::-1].copy(), bs[::-1].copy(), bd[::-1].copy())
    after = [h.ink.get_layer(l, w) for l in (1, 2) for w in (0, 1, 2)]
    for a, b in zip(before, after):
        assert np.array_equal(a.view(np.uint32), b.view(np.uint32))
    h.ink.close()


def test_dense_fallback_matches():
    cfg = synth.get_config(1, 8)
    h = Harness(cfg, dense_threshold=1e-4)
    for b in range(3):
        op, bs, bd = h.sampler.next_batch()
        h.step(op, bs, bd)
        assert any(L["dense"] for L in h.ink.stats()["layers"])
        h.check_state()
    h.ink.close()


def test_two_contexts_are_bit_identical():
    cfg = synth.get_config(1, 4)
    a, b = Harness(cfg), Harness(cfg)
    for i in range(3):
        op, bs, bd = a.sampler.next_batch()
        ra, _ = a.step(op, bs, bd)
        rb, _ = b.step(op, bs, bd)
        assert np.array_equal(ra["changed_ids"], rb["changed_ids"])
        assert np.array_equal(ra["embeddings"].view(np.uint32), rb["embeddings"].view(np.uint32))
    a.ink.close(); b.ink.close()


def test_error_paths_leave_the_state_untouched():
    from paper_2309_11071_amd import Ink, InkError
    from paper_2309_11071_amd.binding import make_updates
    g, X = star(5, 4)
    n, src, dst = g
    rp, col = synth.in_csr_from_edges(n, src, dst)
    model = tiny_model("sage", "max", (4, 4, 4))
    ink = Ink(rp, col, X, model)
    with pytest.raises(InkError) as e:
        ink.apply_updates(make_updates(arr([0], np.uint8), arr([1]), arr([2])))
    assert e.value.status == 2                                   # INK_E_STATE
    ink.full_infer()
    h1 = ink.get_layer(2, 0)
    for bad, code in ((make_updates(arr([0, 0], np.uint8), arr([1, n]), arr([2, 0])), 5),
                      (make_updates(arr([0, 0], np.uint8), arr([1, -1]), arr([2, 0])), 5),
                      (make_updates(arr([0, 7], np.uint8), arr([1, 2]), arr([2, 0])), 1)):
        with pytest.raises(InkError) as e:
            ink.apply_updates(bad)
        assert e.value.status == code
    rp2, col2 = ink.get_graph()
    assert np.array_equal(rp, rp2) and np.array_equal(col, col2)
    assert np.array_equal(h1, ink.get_layer(2, 0))
    bad_rp = rp.copy(); bad_rp[-1] += 1
    with pytest.raises(InkError):
        Ink(bad_rp, col, X, model)
    with pytest.raises(InkError):
        Ink(rp, col[::-1].copy(), X, model)                      # rows not ascending
    ink.close()


def test_widest_feature_rows():
    """Feature width at the library's limit (16 384 columns: 64 aggregation blocks, 1 024 k-chunks
    of the combination), next to the widest output (256)."""
    dims = (16384, 256, 5)
    cfg = synth.WorkloadConfig(6, "t", "sage", "max", 400, 3000, False, dims, 8, 60, True)
    model = tiny_model("sage", "max", dims, seed=3)
    for L in model["layers"]:                      # keep the 32 768-term chains well conditioned
        for k in list(L):
            if isinstance(L[k], np.ndarray):
                L[k] = (L[k] * 0.05).astype(np.float32)
    src, dst = synth.make_graph(cfg)
    X = np.random.default_rng(9).standard_normal((cfg.n_nodes, dims[0])).astype(np.float32)
    h = Harness(cfg=cfg, graph=(cfg.n_nodes, src, dst), X=X, model=model, precision="f32")
    h.check_state()
    for b in range(2):
        op, bs, bd = h.sampler.next_batch()
        h.step(op, bs, bd)
    h.check_state()
    h.ink.close()


@pytest.mark.parametrize("small_batch_limit", [0, -1])
def test_many_blocks_relocate_in_one_batch(small_batch_limit):
    """Hundreds of nodes outgrow their edge block in the same batch, with insertions only: every
    workgroup of the apply kernel takes the relocation branch without any earlier barrier, which
    is the case in which the waves of a workgroup must agree on the block's old place and size."""
    n, d = 4000, 4
    rng = np.random.default_rng(5)
    X = rng.standard_normal((n, d)).astype(np.float32)
    src, dst = arr([1, 2, 3]), arr([0, 0, 0])
    h = Harness(graph=(n, src, dst), X=X, model=tiny_model("sage", "max", (d, 4, 4)), slack=0.01,
                small_batch_limit=small_batch_limit)
    for r in range(3):
        # 500 destinations and 500 sources gain 7 edges each: far more than the 4 spare slots of a block
        ops = []
        for v in range(100, 600):
            for j in range(7):
                ops.append((INS, 1000 + (v * 7 + j + 53 * r) % 2900, v))
        ops = [o for o in dict.fromkeys(ops) if o[1] != o[2]]
        run(h, ops[:3900] if small_batch_limit == 0 else ops)
        h.check_graph()
        h.check_state()
    h.ink.close()


def test_condition_counters_of_rows_wider_than_one_block():
    """Aggregated rows of 300 columns are processed as two column blocks; a target's condition
    is tallied once, so the four classes still partition the targets (Sec. 5.2)."""
    dims = (300, 16, 8)
    cfg = synth.WorkloadConfig(6, "t", "sage", "max", 500, 6000, False, dims, 8, 80, True)
    src, dst = synth.make_graph(cfg)
    X = np.random.default_rng(11).standard_normal((cfg.n_nodes, dims[0])).astype(np.float32)
    h = Harness(cfg=cfg, graph=(cfg.n_nodes, src, dst), X=X, model=tiny_model("sage", "max", dims, seed=4))
    for b in range(3):
        op, bs, bd = h.sampler.next_batch()
        h.step(op, bs, bd)
        L = h.ink.stats()["layers"][0]
        assert L["n_targets"] > 0
        assert L["n_no_deletion"] + L["n_deletion_no_effect"] + L["n_covered"] + L["n_exposed"] == L["n_targets"]
        assert L["n_alpha_changed"] <= L["n_targets"]
    h.check_state()
    h.ink.close()


@pytest.mark.parametrize("kind,agg,exact", [("sage", "max", True), ("gin", "min", True), ("gin", "sum", False),
                                            ("gcn", "gcn_sym", False)])
def test_insert_then_delete_restores_the_cache(kind, agg, exact):
    """Inserting a set of edges and deleting the same edges again leaves the edge set as it was: the
    selecting aggregators must return to the very same values, holder ids and embeddings (a selection
    has no memory), the accumulating ones to within the stated tolerance (Sec. 7: the delta method
    may lose precision)."""
    from util import row_rel_err
    dims = (16, 24, 8)
    cfg = synth.WorkloadConfig(6, "t", kind, agg, 2000, 16000, False, dims, 12, 200, False)
    src, dst = synth.make_graph(cfg)
    rng = np.random.default_rng(21)
    X = rng.standard_normal((cfg.n_nodes, dims[0])).astype(np.float32)
    h = Harness(cfg=cfg, graph=(cfg.n_nodes, src, dst), X=X, model=tiny_model(kind, agg, dims, seed=2, hidden=12),
                precision="f32" if exact else "f64")
    which = (0, 1, 2) if exact else (0, 1)
    before = {(l, w): h.ink.get_layer(l, w) for l in (1, 2) for w in which}
    have = set(h.keys.tolist())
    s = rng.integers(0, cfg.n_nodes, size=600).astype(np.int32)
    d = rng.integers(0, cfg.n_nodes, size=600).astype(np.int32)
    new = np.array([a != b and int(k) not in have for a, b, k in zip(s, d, synth.edge_keys(s, d))])
    _, first = np.unique(synth.edge_keys(s, d), return_index=True)
    keep = np.zeros(s.size, bool); keep[first] = True
    s, d = s[new & keep], d[new & keep]
    assert s.size > 400
    res, want = h.step(np.zeros(s.size, np.uint8), s, d, exact=exact)
    assert res["n_applied_ins"] == s.size and want.size > 0
    res, want = h.step(np.ones(s.size, np.uint8), s, d, exact=exact)
    assert res["n_applied_del"] == s.size
    if exact:
        for (l, w), old in before.items():
            assert np.array_equal(h.ink.get_layer(l, w).view(np.uint32), old.view(np.uint32)), (l, w)
    else:       # against the oracle's inference of the restored snapshot, under the metric of the accumulated tables
        h.check_state(exact=False)
        print("restored to within", max(row_rel_err(h.ink.get_layer(l, w), old) for (l, w), old in before.items()))
    h.check_graph()
    h.check_bound()
    h.ink.close()


def test_expansion_over_sources_with_one_or_no_out_edge():
    """Thousands of changed sources that have one out-edge or none: a wave of the expansion kernel
    then covers hundreds of sources, runs of equal offsets included (sources without out-edges)."""
    n, d = 20000, 8
    ids = np.arange(n - 1, dtype=np.int32)
    chain = ids[ids % 3 != 0]                                  # i -> i + 1, every third node has no out-edge
    src = np.concatenate([chain, arr([n - 1, n - 1])])
    dst = np.concatenate([chain + 1, arr([0, 1])])
    rng = np.random.default_rng(13)
    X = rng.standard_normal((n, d)).astype(np.float32)
    h = Harness(graph=(n, src, dst), X=X, model=tiny_model("sage", "max", (d, 8, 8), seed=6))
    h.check_state()
    targets = rng.choice(np.arange(2, n - 1), size=9000, replace=False).astype(np.int32)
    res, want = h.step(np.zeros(targets.size, np.uint8), np.full(targets.size, n - 1, np.int32), targets)
    st = h.ink.stats()["layers"]
    assert st[1]["n_sources"] > 5000 and st[1]["n_events"] > 9000 + 3000
    h.check_state()
    res, want = h.step(np.ones(targets.size, np.uint8), np.full(targets.size, n - 1, np.int32), targets)
    h.check_state()
    h.check_graph()
    h.ink.close()
