"""Pins for the CPU oracle: each test checks it against something other than itself
(brute force from the edge list, dense-matrix closed forms with a library matmul,
hand-computed fixtures, algebraic identities and invariants of the method)."""
import os

import numpy as np
import pytest

import oracle
import synth

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def tiny_graph(n, m, seed, int_vals=False, d=5):
    rng = np.random.default_rng(seed)
    src = rng.integers(0, n, size=m)
    dst = rng.integers(0, n, size=m)
    ok = src != dst
    src, dst = src[ok].astype(np.int32), dst[ok].astype(np.int32)
    keys = np.unique(synth.edge_keys(src, dst))
    src, dst = synth.keys_to_edges(keys)
    if int_vals:       # few distinct values => many exact ties
        X = rng.integers(-2, 3, size=(n, d)).astype(np.float32)
    else:
        X = rng.standard_normal((n, d)).astype(np.float32)
    return src, dst, X


def brute_select(n, src, dst, X, is_min):
    """Second, independent implementation straight from the edge list (no CSR)."""
    d = X.shape[1]
    alpha = np.zeros((n, d), np.float32)
    arg = -np.ones((n, d), np.int32)
    for v in range(n):
        nb = sorted(int(s) for s, t in zip(src, dst) if t == v)
        for i in range(d):
            if not nb:
                continue
            vals = [X[u, i] for u in nb]
            best = min(vals) if is_min else max(vals)
            alpha[v, i] = best
            arg[v, i] = min(u for u in nb if X[u, i] == best)
    return alpha, arg


@pytest.mark.parametrize("seed", range(6))
@pytest.mark.parametrize("is_min", [False, True])
def test_select_matches_brute_force(seed, is_min):
    n = 30 + seed
    src, dst, X = tiny_graph(n, 150, seed, int_vals=(seed % 2 == 0))
    rp, col = synth.in_csr_from_edges(n, src, dst)
    a, g = oracle.agg_select(rp, col, X, is_min=is_min)
    a2, g2 = brute_select(n, src, dst, X, is_min)
    assert np.array_equal(a, a2)
    assert np.array_equal(g, g2)


def _parse_cases(path):
    cases, cur = [], None
    for line in open(path):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        tok = line.split()
        if tok[0] in ("case", "graph"):
            cur = dict(name=tok[1], m={})
            cases.append(cur)
        elif tok[0] == "m":
            cur["m"][int(tok[1])] = [float(x) for x in tok[2:]]
        else:
            cur[tok[0]] = tok[1:]
    return cases


def test_select_golden_ties():
    for c in _parse_cases(os.path.join(GOLD, "select_ties.txt")):
        nb = [int(x) for x in c["in"]]
        n = 8
        X = np.full((n, 3), 99.0, np.float32)        # non-neighbours hold values that would win
        X[:, 2] = -99.0
        for u, row in c["m"].items():
            X[u] = row
        src = np.array(nb, np.int32)
        dst = np.zeros(len(nb), np.int32)
        rp, col = synth.in_csr_from_edges(n, src, dst)
        for is_min, kv, ki in ((False, "max", "argmax"), (True, "min", "argmin")):
            a, g = oracle.agg_select(rp, col, X, is_min=is_min)
            assert np.array_equal(a[0], np.array(c[kv], np.float32)), c["name"]
            assert np.array_equal(g[0], np.array(c[ki], np.int32)), c["name"]


def test_min_is_negated_max_of_negation():
    src, dst, X = tiny_graph(40, 200, 11, int_vals=True)
    rp, col = synth.in_csr_from_edges(40, src, dst)
    amin, gmin = oracle.agg_select(rp, col, X, is_min=True)
    amax, gmax = oracle.agg_select(rp, col, -X, is_min=False)
    assert np.array_equal(amin, -amax + 0.0)
    assert np.array_equal(gmin, gmax)


def dense_adj(n, src, dst):
    A = np.zeros((n, n), np.float64)
    A[dst, src] = 1.0           # row v, column u for edge u -> v
    return A


def test_sum_and_mean_match_dense_matmul():
    n = 35
    src, dst, X = tiny_graph(n, 180, 3)
    rp, col = synth.in_csr_from_edges(n, src, dst)
    A = dense_adj(n, src, dst)
    ref = A @ X.astype(np.float64)
    assert np.allclose(oracle.agg_sum(rp, col, X), ref, rtol=1e-6, atol=1e-6)
    deg = np.maximum(A.sum(1, keepdims=True), 1.0)
    assert np.allclose(oracle.agg_sum(rp, col, X, mean=True), ref / deg, rtol=1e-6, atol=1e-6)


def test_gcn_sym_matches_dense_normalised_adjacency():
    n = 35
    src, dst, X = tiny_graph(n, 180, 4)
    rp, col = synth.in_csr_from_edges(n, src, dst)
    A = dense_adj(n, src, dst) + np.eye(n)
    dinv = 1.0 / np.sqrt(A.sum(1))              # row sums = indeg + 1
    ref = (dinv[:, None] * A * dinv[None, :]) @ X.astype(np.float64)
    assert np.allclose(oracle.agg_gcn_sym(rp, col, X), ref, rtol=1e-6, atol=1e-6)


def test_gcn_sym_golden_star_and_path():
    for c in _parse_cases(os.path.join(GOLD, "gcn_star_path.txt")):
        h = np.array([float(x) for x in c["h"]], np.float32)[:, None]
        e = [tuple(int(t) for t in p.split(">")) for p in c["edges"]]
        src = np.array([p[0] for p in e], np.int32)
        dst = np.array([p[1] for p in e], np.int32)
        rp, col = synth.in_csr_from_edges(h.shape[0], src, dst)
        got = oracle.agg_gcn_sym(rp, col, h)[:, 0]
        want = np.array([float(x) for x in c["a"]])
        assert np.allclose(got, want, rtol=2e-7, atol=0), c["name"]


def test_linear_matches_library_matmul_and_is_not_transposed():
    rng = np.random.default_rng(5)
    x = rng.standard_normal((17, 13)).astype(np.float32)
    W = rng.standard_normal((13, 7)).astype(np.float32)
    b = rng.standard_normal(7).astype(np.float32)
    ref = x.astype(np.float64) @ W.astype(np.float64) + b
    for prec, tol in (("f64", 1e-7), ("f32", 2e-6)):
        y = oracle.linear(x, W, b, relu=False, precision=prec)
        assert np.allclose(y, ref, rtol=tol, atol=tol * 10)
        yr = oracle.linear(x, W, b, relu=True, precision=prec)
        assert np.allclose(yr, np.maximum(ref, 0), rtol=tol, atol=tol * 10)
        assert not np.signbit(yr).any()          # ReLU emits +0 only


def test_linear_exact_on_small_integers():
    rng = np.random.default_rng(6)
    x = rng.integers(-8, 9, size=(9, 20)).astype(np.float32)
    W = rng.integers(-8, 9, size=(20, 6)).astype(np.float32)
    ref = (x.astype(np.int64) @ W.astype(np.int64)).astype(np.float32)
    for prec in ("f64", "f32"):
        assert np.array_equal(oracle.linear(x, W, None, False, prec), ref)


def test_linear_precision_modes_differ_where_rounding_order_says_so():
    # (1 + 2^-12)^2 = 1 + 2^-11 + 2^-24.  An fp32 chain rounds the first product to 1 + 2^-11
    # (tie to even) and the second step cancels it exactly; fp64 accumulation keeps 2^-24.
    a = np.float32(1 + 2.0 ** -12)
    x = np.array([[a, -1.0]], np.float32)
    W = np.array([[a], [np.float32(1 + 2.0 ** -11)]], np.float32)
    assert oracle.linear(x, W, None, False, "f32")[0, 0] == 0.0
    assert oracle.linear(x, W, None, False, "f64")[0, 0] == np.float32(2.0 ** -24)


def small_model(kind, agg, dims, seed, hidden=6, eps=0.0):
    cfg = synth.WorkloadConfig(9, "t", kind, agg, 1, 1, False, tuple(dims), hidden, 2, False)
    rng = np.random.default_rng(seed)
    model = synth.make_model(cfg, bias_scale=0.5)
    model["gin_eps"] = eps
    for L in model["layers"]:                  # re-draw from this test's own seed
        for k in list(L):
            if isinstance(L[k], np.ndarray):
                L[k] = rng.standard_normal(L[k].shape).astype(np.float32) * 0.5
    return model


def relu(x):
    return np.maximum(x, 0.0)


def test_full_infer_sage_against_dense_formula():
    n, dims = 25, (4, 5, 3)
    src, dst, X = tiny_graph(n, 120, 21, d=4)
    rp, col = synth.in_csr_from_edges(n, src, dst)
    model = small_model("sage", "max", dims, 1)
    out = oracle.full_infer(rp, col, X, model)
    h = X.astype(np.float64)
    for l, L in enumerate(model["layers"]):
        a = np.zeros_like(h)
        for v in range(n):
            nb = col[rp[v]:rp[v + 1]]
            if nb.size:
                a[v] = h[nb].max(0)
        z = a @ L["W_neigh"].astype(np.float64) + h @ L["W_self"].astype(np.float64)
        h = relu(z) if l == 0 else z
        assert np.allclose(out["h"][l + 1], h, rtol=1e-5, atol=1e-5)
        h = out["h"][l + 1].astype(np.float64)  # follow the oracle's fp32 tables layer by layer


def test_full_infer_gin_against_dense_formula():
    n, dims = 25, (4, 5, 3)
    src, dst, X = tiny_graph(n, 120, 22, d=4)
    rp, col = synth.in_csr_from_edges(n, src, dst)
    model = small_model("gin", "sum", dims, 2, eps=0.25)
    out = oracle.full_infer(rp, col, X, model)
    A = dense_adj(n, src, dst)
    h = X.astype(np.float64)
    for l, L in enumerate(model["layers"]):
        x = 1.25 * h + A @ h
        z = relu(x @ L["W_neigh"].astype(np.float64) + L["bias"])
        z = z @ L["W_mlp2"].astype(np.float64) + L["bias_mlp2"]
        h = relu(z) if l == 0 else z
        assert np.allclose(out["h"][l + 1], h, rtol=1e-5, atol=1e-5)
        h = out["h"][l + 1].astype(np.float64)


def test_full_infer_gcn_against_dense_formula():
    n, dims = 25, (4, 5, 3)
    src, dst, X = tiny_graph(n, 120, 23, d=4)
    rp, col = synth.in_csr_from_edges(n, src, dst)
    model = small_model("gcn", "gcn_sym", dims, 3)
    out = oracle.full_infer(rp, col, X, model)
    A = dense_adj(n, src, dst) + np.eye(n)
    dinv = 1.0 / np.sqrt(A.sum(1))
    Ah = dinv[:, None] * A * dinv[None, :]
    h = X.astype(np.float64)
    for l, L in enumerate(model["layers"]):
        z = (Ah @ h) @ L["W_neigh"].astype(np.float64) + L["bias"]
        h = relu(z) if l == 0 else z
        assert np.allclose(out["h"][l + 1], h, rtol=1e-5, atol=1e-5)
        h = out["h"][l + 1].astype(np.float64)


def test_one_layer_model_is_one_aggregation_and_one_linear_map():
    n = 20
    src, dst, X = tiny_graph(n, 90, 31, d=4)
    rp, col = synth.in_csr_from_edges(n, src, dst)
    model = small_model("sage", "max", (4, 3), 4)
    out = oracle.full_infer(rp, col, X, model)
    a, g = oracle.agg_select(rp, col, X)
    assert np.array_equal(out["alpha"][1], a) and np.array_equal(out["arg"][1], g)
    L = model["layers"][0]
    ref = a.astype(np.float64) @ L["W_neigh"].astype(np.float64) + X.astype(np.float64) @ L["W_self"].astype(np.float64)
    assert np.allclose(out["h"][1], ref, rtol=1e-5, atol=1e-5)     # last layer: no activation


def test_edgeless_graph():
    n = 6
    X = np.arange(n * 3, dtype=np.float32).reshape(n, 3)
    rp = np.zeros(n + 1, np.int64)
    col = np.zeros(0, np.int32)
    a, g = oracle.agg_select(rp, col, X)
    assert not a.any() and (g == -1).all()
    assert not oracle.agg_sum(rp, col, X).any()
    assert np.allclose(oracle.agg_gcn_sym(rp, col, X), X)       # only the self term, dhat = 1


# ---- batch semantics and invariants of the update problem -------------------------------

def test_apply_batch_net_effect():
    keys = np.array(sorted([(1 << 32) | 0, (2 << 32) | 1]), np.int64)      # 0>1, 1>2
    op = np.array([0, 0, 1, 1, 0, 1, 0, 0], np.uint8)
    src = np.array([0, 3, 1, 4, 5, 5, 6, 6], np.int32)
    dst = np.array([1, 2, 2, 0, 0, 0, 6, 7], np.int32)
    # insert present 0>1 (noop); insert 3>2; delete 1>2; delete absent 4>0 (noop);
    # insert then delete 5>0 (cancel, 2 noops); self loop 6>6 (noop); insert 6>7
    new, n_ins, n_del, n_noop = oracle.apply_batch(keys, op, src, dst)
    want = sorted([(1 << 32) | 0, (2 << 32) | 3, (7 << 32) | 6])
    assert new.tolist() == want
    assert (n_ins, n_del, n_noop) == (2, 1, 5)


def khop_out(n, keys, seeds, k):
    src, dst = synth.keys_to_edges(keys)
    reach = np.zeros(n, bool)
    reach[list(seeds)] = True
    for _ in range(k):
        nxt = reach.copy()
        nxt[dst[reach[src]]] = True
        reach = nxt
    return reach


@pytest.mark.parametrize("kind,agg", [("sage", "max"), ("gin", "sum"), ("gcn", "gcn_sym")])
def test_update_invariants(kind, agg):
    """Empty batch changes nothing; changes stay inside the k-hop out-neighbourhood of the
    changed edges' destinations (Sec. 1: affected area); insert-then-delete restores the
    selection-based state exactly."""
    cfg = synth.get_config(1, 40)
    cfg = synth.WorkloadConfig(1, "t", kind, agg, cfg.n_nodes, cfg.n_edges, True, (6, 5, 4), 5, 10, False)
    src, dst = synth.make_graph(cfg)
    n = cfg.n_nodes
    X = np.random.default_rng(1).standard_normal((n, 6)).astype(np.float32)
    model = small_model(kind, agg, cfg.dims, 8, hidden=5)
    keys = np.unique(synth.edge_keys(src, dst))
    pre = oracle.full_infer(*oracle.csr_from_keys(n, keys), X, model)
    e = np.zeros(0, np.int32)
    k0, a0, d0, z0 = oracle.apply_batch(keys, np.zeros(0, np.uint8), e, e)
    assert np.array_equal(k0, keys) and (a0, d0, z0) == (0, 0, 0)
    sampler = synth.BatchSampler(cfg, src, dst)
    op, bs, bd = sampler.next_batch()
    keys2, n_ins, n_del, n_noop = oracle.apply_batch(keys, op, bs, bd)
    assert (n_ins, n_del, n_noop) == (5, 5, 0)
    cs, cd = sampler.current_edges()
    assert np.array_equal(np.unique(synth.edge_keys(cs, cd)), keys2)     # sampler and oracle agree
    post = oracle.full_infer(*oracle.csr_from_keys(n, keys2), X, model)
    ch = oracle.changed_nodes(pre, post)
    assert ch[0].size == 0
    both = np.union1d(keys, keys2)
    # GCN's degree normalisation lets a destination's own degree change reach its out-neighbours
    # one layer earlier than a plain message change would
    extra = 1 if kind == "gcn" else 0
    for l in (1, 2):
        reach = khop_out(n, both, set(bd.tolist()), l - 1 + extra)
        assert reach[ch[l]].all(), l
    assert ch[2].size > 0
    # reversibility: undo the batch (insert <-> delete, reverse order)
    keys3, _, _, _ = oracle.apply_batch(keys2, (1 - op)[::-1].copy(), bs[::-1].copy(), bd[::-1].copy())
    assert np.array_equal(keys3, keys)
    back = oracle.full_infer(*oracle.csr_from_keys(n, keys3), X, model)
    for l in (1, 2):
        assert np.array_equal(back["h"][l], pre["h"][l])
        if agg == "max":
            assert np.array_equal(back["arg"][l], pre["arg"][l])


@pytest.mark.parametrize("kind,agg", [("sage", "max"), ("gin", "sum"), ("gcn", "gcn_sym")])
def test_feature_change_stays_in_the_out_neighbourhood(kind, agg):
    """What ink_update_features is compared with: after x_v changes for v in S, layer l can only
    change inside the l-hop out-neighbourhood of S (S itself included: the self term of Sec. 3.2,
    GCN's self loop), and S itself does change at layer 1 for a generic new row."""
    n, dims = 60, (5, 6, 4)
    src, dst, X = tiny_graph(n, 260, 41, d=dims[0])
    keys = np.unique(synth.edge_keys(src, dst))
    model = small_model(kind, agg, dims, 9, hidden=5)
    rp, col = oracle.csr_from_keys(n, keys)
    pre = oracle.full_infer(rp, col, X, model)
    S = np.array([3, 17, 44])
    X2 = X.copy()
    X2[S] = np.random.default_rng(5).standard_normal((S.size, dims[0])).astype(np.float32)
    post = oracle.full_infer(rp, col, X2, model)
    ch = oracle.changed_nodes(pre, post)
    assert sorted(ch[0].tolist()) == S.tolist()
    for l in (1, 2):
        reach = khop_out(n, keys, set(S.tolist()), l)
        assert reach[ch[l]].all(), l
    assert ch[2].size > 0


@pytest.mark.parametrize("kind,agg", [("sage", "max"), ("sage", "min"), ("sage", "mean"), ("gin", "sum"),
                                      ("gcn", "gcn_sym")])
def test_isolated_new_node_has_the_closed_form_embedding(kind, agg):
    """What ink_add_nodes is compared with: a node without edges aggregates nothing (alpha = 0,
    argument -1; GCN: d-hat = 1, only its own term), so its embeddings follow from its own row
    alone, and appending it changes no other row."""
    n, dims = 30, (4, 5, 3)
    src, dst, X = tiny_graph(n, 140, 43, d=dims[0])
    keys = np.unique(synth.edge_keys(src, dst))
    model = small_model(kind, agg, dims, 10, hidden=4, eps=0.5) if kind == "gin" else small_model(kind, agg, dims, 10)
    pre = oracle.full_infer(*oracle.csr_from_keys(n, keys), X, model)
    x_new = np.random.default_rng(6).standard_normal((2, dims[0])).astype(np.float32)
    X2 = np.concatenate([X, x_new])
    post = oracle.full_infer(*oracle.csr_from_keys(n + 2, keys), X2, model)
    for l in range(len(dims)):
        assert np.array_equal(post["h"][l][:n], pre["h"][l])
    h = x_new.astype(np.float64)
    for l, L in enumerate(model["layers"]):
        if kind == "sage":
            z = h @ L["W_self"].astype(np.float64) + (L["bias"] if L.get("bias") is not None else 0.0)
        elif kind == "gin":
            z = relu(1.5 * h @ L["W_neigh"].astype(np.float64) + L["bias"])
            z = z @ L["W_mlp2"].astype(np.float64) + L["bias_mlp2"]
        else:
            z = h @ L["W_neigh"].astype(np.float64) + L["bias"]
        h = relu(z) if l == 0 else z
        assert np.allclose(post["h"][l + 1][n:], h, rtol=1e-5, atol=1e-5), l
        h = post["h"][l + 1][n:].astype(np.float64)
    if agg in ("max", "min"):
        assert (post["arg"][1][n:] == -1).all() and (post["alpha"][1][n:] == 0).all()


def test_rows_differ_is_bitwise():
    """The changed-node sets compare bit patterns (the reading of Sec. 2.5.2's "equal" that both
    sides use): +0 and -0 differ, a NaN equals itself, and one differing element marks the row."""
    a = np.array([[0.0, 1.0], [np.nan, 2.0], [3.0, 4.0], [5.0, 6.0]], np.float32)
    b = np.array([[-0.0, 1.0], [np.nan, 2.0], [3.0, 4.0], [5.0, np.nextafter(np.float32(6.0), np.float32(7.0))]], np.float32)
    assert oracle.rows_differ(a, b).tolist() == [True, False, False, True]
    pre = dict(h=[a, a])
    post = dict(h=[a, b])
    ch = oracle.changed_nodes(pre, post)
    assert ch[0].size == 0 and ch[1].tolist() == [0, 3] and ch[1].dtype == np.int32



# ---- user-defined events (Sec. 2.6): a per-node term added between the linear map and the activation
def _user_case(kind, agg, seed=0):
    rng = np.random.default_rng(seed)
    n, dims = 30, (5, 6, 4)
    cfg = synth.WorkloadConfig(9, "t", kind, agg, n, 120, False, dims, 7, 4, False)
    src, dst = synth.make_graph(cfg)
    rp, col = synth.in_csr_from_edges(n, src, dst)
    X = rng.standard_normal((n, dims[0])).astype(np.float32)
    model = synth.make_model(cfg, bias_scale=0.3)
    return n, dims, rp, col, X, model, rng


@pytest.mark.parametrize("kind,agg", [("sage", "max"), ("gin", "sum"), ("gcn", "gcn_sym")])
def test_user_term_is_added_before_the_activation(kind, agg):
    n, dims, rp, col, X, model, rng = _user_case(kind, agg)
    base = oracle.full_infer(rp, col, X, model, "f64")
    none = oracle.full_infer(rp, col, X, model, "f64", [None, None])
    zero = oracle.full_infer(rp, col, X, model, "f64", [np.zeros((n, dims[1]), np.float32), None])
    for a, b, c in zip(base["h"], none["h"], zero["h"]):
        assert np.array_equal(a, b) and np.array_equal(a, c)
    # last layer has no activation: its term shifts the output by exactly that term (up to the final rounding)
    u2 = rng.standard_normal((n, dims[2])).astype(np.float32)
    out = oracle.full_infer(rp, col, X, model, "f64", [None, u2])
    assert np.array_equal(out["h"][1], base["h"][1])
    want = base["h"][2].astype(np.float64) + u2
    assert np.allclose(out["h"][2], want, rtol=0, atol=2e-6 * np.abs(want).max())
    # hidden layer: the activation comes after the term -- a very negative term zeroes the row, and the
    # dense closed form act(lin + u) holds with a library matmul
    u1 = np.zeros((n, dims[1]), np.float32)
    u1[3] = -1e6
    u1[7] = rng.standard_normal(dims[1])
    out = oracle.full_infer(rp, col, X, model, "f64", [u1, None])
    assert np.all(out["h"][1][3] == 0.0)
    lin = dict(model, layers=[dict(model["layers"][0], act="none"), model["layers"][1]])
    pre = oracle.transform(lin, 0, base["alpha"][1], X, "f64").astype(np.float64)
    assert np.allclose(out["h"][1], np.maximum(pre + u1, 0.0), rtol=0, atol=1e-5)
    others = np.ones(n, bool); others[[3, 7]] = False
    assert np.array_equal(out["h"][1][others], base["h"][1][others])


def test_user_events_group_by_layer_and_target_in_list_order():
    widths, n = (3, 2), 5
    r = lambda *x: np.array(x + (9.0,) * (3 - len(x)), np.float32)
    ev = [(1, 2, oracle.USER_SET), (2, 2, oracle.USER_ADD), (1, 2, oracle.USER_ADD), (1, 4, oracle.USER_ADD),
          (1, 4, oracle.USER_CLEAR), (1, 4, oracle.USER_ADD), (2, 0, oracle.USER_SET), (2, 0, oracle.USER_CLEAR)]
    rows = [r(1, 2, 3), r(5, 6), r(10, 20, 30), r(1, 1, 1), r(0, 0, 0), r(7, 8, 9), r(4, 4), r(0, 0)]
    out = oracle.apply_user_events([None, None], widths, n, ev, rows)
    want1 = np.zeros((5, 3), np.float32); want1[2] = (11, 22, 33); want1[4] = (7, 8, 9)
    want2 = np.zeros((5, 2), np.float32); want2[2] = (5, 6)            # only the first width_l entries of a row count
    assert np.array_equal(out[0], want1) and np.array_equal(out[1], want2)
    again = oracle.apply_user_events(out, widths, n, [(1, 2, oracle.USER_CLEAR), (1, 4, oracle.USER_CLEAR), (2, 2, oracle.USER_CLEAR)],
                                     [r(0), r(0), r(0)])
    assert not again[0].any() and not again[1].any()
    assert np.array_equal(out[0], want1)                                # the input terms are not modified


def test_a_user_event_stays_in_the_out_neighbourhood():
    n, dims, rp, col, X, model, rng = _user_case("sage", "max", seed=4)
    base = oracle.full_infer(rp, col, X, model, "f32")
    u1 = np.zeros((n, dims[1]), np.float32)
    u1[5] = rng.standard_normal(dims[1]) * 3
    out = oracle.full_infer(rp, col, X, model, "f32", [u1, None])
    ch1 = np.nonzero(oracle.rows_differ(base["h"][1], out["h"][1]))[0]
    assert set(ch1.tolist()) <= {5}
    outn = {5} | {v for v in range(n) if 5 in col[rp[v]:rp[v + 1]].tolist()}      # 5 and the nodes that aggregate it
    ch2 = np.nonzero(oracle.rows_differ(base["h"][2], out["h"][2]))[0]
    assert set(ch2.tolist()) <= outn


# ---- the "Affected" baseline (Sec. 4.1): recomputing the theoretical affected area gives the full result
@pytest.mark.parametrize("kind,agg", [("sage", "max"), ("gin", "sum"), ("sage", "mean")])
def test_affected_area_recompute_equals_full_inference(kind, agg):
    rng = np.random.default_rng(12)
    n, dims = 300, (6, 5, 5, 4)
    cfg = synth.WorkloadConfig(9, "t", kind, agg, n, 1500, False, dims, 6, 12, False)
    src, dst = synth.make_graph(cfg)
    X = rng.standard_normal((n, dims[0])).astype(np.float32)
    model = synth.make_model(cfg, bias_scale=0.2)
    keys = np.unique(synth.edge_keys(src, dst))
    pre = oracle.full_infer(*oracle.csr_from_keys(n, keys), X, model, "f32")
    sampler = synth.BatchSampler(cfg, src, dst)
    op, bs, bd = sampler.next_batch()
    keys2, _, _, _ = oracle.apply_batch(keys, op, bs, bd)
    rp2, col2 = oracle.csr_from_keys(n, keys2)
    s2, d2 = (keys2 & 0xFFFFFFFF).astype(np.int32), (keys2 >> 32).astype(np.int32)
    orp, ocol = synth.in_csr_from_edges(n, d2, s2)            # roles swapped: out-neighbour lists
    areas = oracle.affected_area(n, orp, ocol, bd, 3)
    # hand check of the area: layer 1 = changed destinations, layer 2 adds their out-neighbours
    assert np.array_equal(areas[0], np.unique(bd))
    want2 = set(np.unique(bd).tolist())
    for v in np.unique(bd).tolist():
        want2 |= set(d2[s2 == v].tolist())
    assert set(areas[1].tolist()) == want2 and set(areas[1].tolist()) <= set(areas[2].tolist())
    got = oracle.affected_infer(rp2, col2, X, model, pre, areas, "f32")
    full = oracle.full_infer(rp2, col2, X, model, "f32")
    for l in range(1, 4):
        assert np.array_equal(got["h"][l].view(np.uint32), full["h"][l].view(np.uint32))
        assert np.array_equal(got["alpha"][l].view(np.uint32), full["alpha"][l].view(np.uint32))
        if full["arg"][l] is not None:
            assert np.array_equal(got["arg"][l], full["arg"][l])
    # and the area is needed: leaving the out-neighbours out of layer 2 must show (the pin is sharp)
    short = [areas[0], areas[0], areas[0]]
    bad = oracle.affected_infer(rp2, col2, X, model, pre, short, "f32")
    assert not np.array_equal(bad["h"][3].view(np.uint32), full["h"][3].view(np.uint32))
