"""Helpers shared by the GPU parity tests (oracle on one side, the C-ABI library on the other)."""
import numpy as np

import oracle
import synth


def row_rel_err(got, ref):
    """Per row: max_i |got - ref| / max(max_i |ref|, tiny); returns the maximum over rows."""
    got = got.astype(np.float64)
    ref = ref.astype(np.float64)
    if got.size == 0:
        return 0.0
    num = np.abs(got - ref).max(axis=1)
    den = np.maximum(np.abs(ref).max(axis=1), 1e-30)
    return float((num / den).max())


def scaled_rel_err(got, ref):
    """Row-relative error for accumulated (sum-type) results: per row max_i |got - ref| divided by
    max(row max |ref|, mean row max of the table).  Rounding errors of a sum scale with the size
    of the summands, so rows that cancel to something small are measured against the table's
    typical magnitude instead of their own."""
    got = got.astype(np.float64)
    ref = ref.astype(np.float64)
    if got.size == 0:
        return 0.0
    rmax = np.abs(ref).max(axis=1)
    floor = max(float(rmax.mean()), 1e-30)
    return float((np.abs(got - ref).max(axis=1) / np.maximum(rmax, floor)).max())


class Harness:
    """Keeps the oracle's view (edge-key set, full inference) next to an Ink context."""

    def __init__(self, cfg=None, model=None, precision="f32", slack=0.25, profile=False, graph=None, X=None,
                 dense_threshold=0.0, pool_reserve=0, node_capacity=0, small_batch_limit=0):
        """Either a workload config, or an explicit graph=(n, src, dst) with features X and a model."""
        from paper_2309_11071_amd import Ink
        self.cfg = cfg
        if graph is None:
            self.src, self.dst = synth.make_graph(cfg)
            self.n = cfg.n_nodes
            self.X = synth.make_features(cfg)
        else:
            self.n, self.src, self.dst = graph
            self.src = np.asarray(self.src, np.int32)
            self.dst = np.asarray(self.dst, np.int32)
            self.X = np.ascontiguousarray(X, np.float32)
        self.model = model if model is not None else synth.make_model(cfg)
        self.precision = precision
        self.keys = np.unique(synth.edge_keys(self.src, self.dst))
        rp, col = oracle.csr_from_keys(self.n, self.keys)
        self.ink = Ink(rp, col, self.X, self.model, slack_factor=slack, profile=profile,
                       dense_threshold=dense_threshold, pool_reserve=pool_reserve, node_capacity=node_capacity,
                       small_batch_limit=small_batch_limit)
        self.ink.full_infer()
        self.ref = oracle.full_infer(rp, col, self.X, self.model, precision)
        self.sampler = synth.BatchSampler(cfg, self.src, self.dst) if cfg is not None else None

    def check_state(self, exact=True, tol=1e-5):
        k = len(self.model["layers"])
        select = self.model["agg"] in ("max", "min")
        for l in range(1, k + 1):
            h = self.ink.get_layer(l, 0)
            if exact:
                assert np.array_equal(h.view(np.uint32), self.ref["h"][l].view(np.uint32)), "h_%d differs" % l
            else:
                err = scaled_rel_err(h, self.ref["h"][l])
                assert err <= tol, "h_%d beyond tolerance: %g" % (l, err)
            if select:
                a = self.ink.get_layer(l, 1)
                g = self.ink.get_layer(l, 2)
                if exact:
                    assert np.array_equal(a.view(np.uint32), self.ref["alpha"][l].view(np.uint32)), "alpha_%d" % l
                    assert np.array_equal(g, self.ref["arg"][l]), "argmax_%d differs" % l

    def check_bound(self, exact=False, max_nodes=4000):
        """The cached bound on the runner-up value (get_layer which=3) must dominate the best value
        among the neighbours other than the holder; right after a full inference it is exact.
        Where a runner-up id is recorded (which=4) it must be a neighbour other than the holder
        that has exactly the bound's value, and no other non-holder may beat it (value, then lower id)."""
        if self.model["agg"] not in ("max", "min") or self.n > max_nodes:
            return
        is_min = self.model["agg"] == "min"
        rp, col = oracle.csr_from_keys(self.n, self.keys)
        for l in range(1, len(self.model["layers"]) + 1):
            m = self.ref["h"][l - 1]
            arg = self.ref["arg"][l]
            ub = self.ink.get_layer(l, 3)
            a2 = self.ink.get_layer(l, 4)
            for v in range(self.n):
                nb = col[rp[v]:rp[v + 1]]
                if nb.size == 0:
                    assert (a2[v] == -1).all(), (l, v)
                    continue
                rows = m[nb].astype(np.float64)                      # [deg, d]
                holder = arg[v][None, :] == nb[:, None]
                worst = np.inf if is_min else -np.inf
                others = np.where(holder, worst, rows)
                true2 = others.min(axis=0) if is_min else others.max(axis=0)
                got = ub[v].astype(np.float64)
                # lowest id among the non-holders that reach the runner-up value (-1: fewer than 2 neighbours)
                first = np.where(others == true2[None, :], nb.astype(np.int64)[:, None], np.int64(1) << 60).min(axis=0)
                true_id = np.where(np.isfinite(true2), first, -1)
                if exact:
                    assert np.array_equal(got, true2), (l, v)
                    assert np.array_equal(a2[v], true_id), (l, v)
                else:
                    assert np.all(got <= true2) if is_min else np.all(got >= true2), (l, v)
                    known = a2[v] >= 0
                    assert np.array_equal(a2[v][known], true_id[known]), (l, v)
                    assert np.array_equal(got[known], true2[known]), (l, v)

    def check_graph(self):
        rp, col = self.ink.get_graph()
        rp2, col2 = oracle.csr_from_keys(self.n, self.keys)
        assert np.array_equal(rp, rp2) and np.array_equal(col, col2), "graph store differs from the oracle's edge set"

    def _compare(self, res, post, exact, tol):
        """Result of an incremental call against the oracle's inference `post` of the new snapshot."""
        want = oracle.changed_nodes(self.ref, post)[-1]
        if exact:
            assert np.array_equal(res["changed_ids"], want), "changed-node set differs"
            assert np.array_equal(res["embeddings"].view(np.uint32), post["h"][-1][want].view(np.uint32))
        else:
            # accumulated aggregators: embeddings within tolerance; the changed sets may differ only in
            # rows whose change is itself below the tolerance (delta updates lose sub-ulp changes, Sec. 7)
            got = res["changed_ids"]
            assert np.all(np.diff(got) > 0)
            hk_pre, hk_post = self.ref["h"][-1], post["h"][-1]
            rmax = np.abs(hk_post).max(axis=1)
            floor = max(float(rmax.mean()), 1e-30)
            delta = np.abs(hk_post.astype(np.float64) - hk_pre).max(axis=1) / np.maximum(rmax, floor)
            sym = np.setxor1d(got, want)
            assert sym.size == 0 or delta[sym].max() <= tol, "changed sets differ in a row that really changed"
            self.last_set_mismatch = int(sym.size)
            floor_rows = np.maximum(np.abs(hk_post[got]).max(axis=1), floor)
            err = np.abs(res["embeddings"].astype(np.float64) - hk_post[got]).max(axis=1) / floor_rows if got.size else np.zeros(0)
            assert got.size == 0 or err.max() <= tol, "returned embeddings beyond tolerance: %g" % err.max()
        return want

    def feature_step(self, ids, rows, exact=True, tol=1e-5):
        """x_v <- rows[i] for v = ids[i] through ink_update_features, against the oracle's full
        inference with the new feature table."""
        ids = np.asarray(ids, np.int32)
        rows = np.ascontiguousarray(rows, np.float32).reshape(ids.size, self.X.shape[1])
        res = self.ink.update_features(ids, rows)
        assert (res["n_applied_ins"], res["n_applied_del"], res["n_noop"]) == (0, 0, 0)
        X2 = self.X.copy()
        X2[ids] = rows
        post = oracle.full_infer(*oracle.csr_from_keys(self.n, self.keys), X2, self.model, self.precision)
        want = self._compare(res, post, exact, tol)
        self.X, self.ref = X2, post
        return res, want

    def add_nodes(self, features, exact=True, tol=1e-5):
        """Appends nodes without edges through ink_add_nodes; the oracle re-runs on the grown graph."""
        features = np.ascontiguousarray(features, np.float32).reshape(-1, self.X.shape[1])
        k = features.shape[0]
        res = self.ink.add_nodes(features)
        n2 = self.n + k
        X2 = np.concatenate([self.X, features], axis=0)
        post = oracle.full_infer(*oracle.csr_from_keys(n2, self.keys), X2, self.model, self.precision)
        ids = np.arange(self.n, n2, dtype=np.int32)
        assert res["n_changed"] == k and np.array_equal(res["changed_ids"], ids)
        for l in range(len(post["h"])):          # the old nodes' rows are untouched by definition
            assert np.array_equal(post["h"][l][:self.n].view(np.uint32), self.ref["h"][l].view(np.uint32))
        want = post["h"][-1][ids]
        if exact:
            assert np.array_equal(res["embeddings"].view(np.uint32), want.view(np.uint32))
        elif k:
            assert scaled_rel_err(res["embeddings"], want) <= tol
        self.n, self.X, self.ref = n2, X2, post
        return res

    def step(self, op, bs, bd, exact=True, tol=1e-5, affected=False):
        from paper_2309_11071_amd.binding import make_updates
        res = self.ink.apply_updates(make_updates(op, bs, bd), affected=affected)
        keys2, n_ins, n_del, n_noop = oracle.apply_batch(self.keys, op, bs, bd)
        assert (res["n_applied_ins"], res["n_applied_del"], res["n_noop"]) == (n_ins, n_del, n_noop)
        post = oracle.full_infer(*oracle.csr_from_keys(self.n, keys2), self.X, self.model, self.precision)
        want = self._compare(res, post, exact, tol)
        self.keys, self.ref = keys2, post
        return res, want
