"""Helpers shared by the GPU parity tests (oracle on one side, the C-ABI library on the other)."""
import numpy as np

import oracle
import synth


def row_rel_err(got, ref):
    """Maximum over rows of the stated per-row metric (see row_err)."""
    e = row_err(got, ref)
    return float(e.max()) if e.size else 0.0


U32 = 2.0 ** -24           # unit roundoff of fp32


def row_err(got, ref):
    """Per row: max_i |got - ref| / max(max_i |ref|, tiny) -- the stated metric, one value per row."""
    got = np.asarray(got, np.float64)
    ref = np.asarray(ref, np.float64)
    if got.size == 0:
        return np.zeros(0)
    return np.abs(got - ref).max(axis=1) / np.maximum(np.abs(ref).max(axis=1), 1e-30)


def magnitude_inference(rowptr, col, X, model, user_terms=None):
    """Per layer l and element, the sum of the absolute values of all the products and summands
    that make up h_l[v][j]: the same inference with |x|, |W|, |b| and no activation, computed by the
    oracle's own routines in fp64.  A rounding error of the fp32 evaluation is a small multiple of
    2^-24 times this magnitude, however far the true value cancels below it."""
    h = np.abs(np.ascontiguousarray(X, np.float32))
    out = [h]
    ab = lambda w: None if w is None else np.abs(w)
    for li, L in enumerate(model["layers"]):
        a, _ = oracle.aggregate(rowptr, col, h, model["agg"] if model["agg"] not in ("max", "min") else "sum")
        if model["kind"] == "sage":
            h = oracle.linear(np.concatenate([a, h], axis=1), np.abs(np.concatenate([L["W_neigh"], L["W_self"]], axis=0)),
                              ab(L.get("bias")), False, "f64")
        elif model["kind"] == "gcn":
            h = oracle.linear(a, np.abs(L["W_neigh"]), ab(L.get("bias")), False, "f64")
        else:
            x = ((1.0 + abs(float(model.get("gin_eps", 0.0)))) * h.astype(np.float64) + a).astype(np.float32)
            z = oracle.linear(x, np.abs(L["W_neigh"]), ab(L.get("bias")), False, "f64")
            h = oracle.linear(z, np.abs(L["W_mlp2"]), ab(L.get("bias_mlp2")), False, "f64")
        if user_terms is not None and user_terms[li] is not None:
            h = (h.astype(np.float64) + np.abs(user_terms[li])).astype(np.float32)
        out.append(h)
    return out


def chain_lengths(model):
    """Terms of the linear maps of each layer (the K of a K-term fp32 chain)."""
    out = []
    for L in model["layers"]:
        k = L["in_dim"] * (2 if model["kind"] == "sage" else 1) + 1
        if model["kind"] == "gin":
            k += int(L.get("mlp_hidden", 0)) + 1
        out.append(k)
    return out


def check_accumulated(got, ref, mag, deg, k_lin, depth, tol=1e-5, what=""):
    """Accumulated (sum-type) results against the fp64 oracle.  Primary bar: the stated per-row
    metric <= tol.  A row beyond it passes only if every element lies within the rounding bound of
    its own summands, depth * (deg + K + 2) * 2^-24 * magnitude (depth layers of a (deg + K)-term
    fp32 evaluation; magnitude from magnitude_inference), i.e. if the row's true value cancels so
    far below its summands that no fp32 evaluation could meet the relative bar.  mag and deg may be
    callables, evaluated only if some row is beyond the strict bar.  Returns the strict maximum and
    how many rows needed the second bound."""
    got = np.asarray(got, np.float64)
    ref = np.asarray(ref, np.float64)
    if got.size == 0:
        return dict(what=what, rows=0, strict_max=0.0, rows_beyond_strict=0)
    err = np.abs(got - ref)
    rmax = np.maximum(np.abs(ref).max(axis=1), 1e-30)
    strict = err.max(axis=1) / rmax
    beyond = np.nonzero(strict > tol)[0]
    if beyond.size:
        mag = mag() if callable(mag) else mag
        deg = deg() if callable(deg) else deg
        bound = (depth * (np.asarray(deg, np.float64)[beyond] + k_lin + 2) * U32)[:, None] * np.asarray(mag, np.float64)[beyond]
        ok = err[beyond] <= np.maximum(bound, tol * rmax[beyond][:, None])
        worst = int(beyond[np.argmin(ok.all(axis=1))])
        assert ok.all(), ("%s: row %d is beyond the relative bar (%.3g) and beyond the rounding bound of its summands"
                          % (what, worst, strict[worst]))
    return dict(what=what, rows=int(strict.size), strict_max=float(strict.max()), rows_beyond_strict=int(beyond.size))


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
        self.user_terms = [None] * len(self.model["layers"])      # oracle-side terms of user-defined events
        self.ref = oracle.full_infer(rp, col, self.X, self.model, precision)
        self.sampler = synth.BatchSampler(cfg, self.src, self.dst) if cfg is not None else None
        self.reports = []          # one entry per accumulated table checked (strict maximum, rows beyond it)
        self.last_set_mismatch = 0
        self._mag_keys = None
        self.k_lin = chain_lengths(self.model)

    def _magnitudes(self):
        """Summand magnitudes and in-degrees of the current snapshot (for check_accumulated)."""
        if self._mag_keys is self.keys and self._mag_X is self.X and self._mag_user is self.user_terms:
            return self
        rp, col = oracle.csr_from_keys(self.n, self.keys)
        self.mag = magnitude_inference(rp, col, self.X, self.model, self.user_terms)
        self.deg = np.diff(rp)
        self.k_lin = chain_lengths(self.model)
        self._mag_keys, self._mag_X, self._mag_user = self.keys, self.X, self.user_terms
        return self

    def check_state(self, exact=True, tol=1e-5):
        k = len(self.model["layers"])
        select = self.model["agg"] in ("max", "min")
        for l in range(1, k + 1):
            h = self.ink.get_layer(l, 0)
            if exact:
                assert np.array_equal(h.view(np.uint32), self.ref["h"][l].view(np.uint32)), "h_%d differs" % l
            else:
                rep = check_accumulated(h, self.ref["h"][l], lambda: self._magnitudes().mag[l], lambda: self._magnitudes().deg,
                                        self.k_lin[l - 1], l, tol, "h_%d" % l)
                self.reports.append(rep)
                print("parity %s: strict max %.3g, %d of %d rows beyond the strict bar (within their rounding bound)"
                      % (rep["what"], rep["strict_max"], rep["rows_beyond_strict"], rep["rows"]))
            if select:
                a = self.ink.get_layer(l, 1)
                g = self.ink.get_layer(l, 2)
                if exact:
                    assert np.array_equal(a.view(np.uint32), self.ref["alpha"][l].view(np.uint32)), "alpha_%d" % l
                    assert np.array_equal(g, self.ref["arg"][l]), "argmax_%d differs" % l

    def check_against_f64(self, tol=1e-5):
        """End-to-end accuracy of the cached embeddings (whatever sequence of updates produced them)
        against an fp64 inference of the current snapshot, under the stated per-row metric; for
        the models whose primary bar is bit-exactness against the fp32-chain oracle."""
        ref64 = oracle.full_infer(*oracle.csr_from_keys(self.n, self.keys), self.X, self.model, "f64", user_terms=self.user_terms)
        out = []
        for l in range(1, len(self.model["layers"]) + 1):
            rep = check_accumulated(self.ink.get_layer(l, 0), ref64["h"][l], lambda: self._magnitudes().mag[l],
                                    lambda: self._magnitudes().deg, self.k_lin[l - 1], l, tol, "h_%d vs fp64" % l)
            print("parity %s: strict max %.3g, %d of %d rows beyond the strict bar (within their rounding bound)"
                  % (rep["what"], rep["strict_max"], rep["rows_beyond_strict"], rep["rows"]))
            out.append(rep)
        return out

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

    def _compare(self, res, post, exact, tol, keys_post=None, X_post=None, n_post=None, user_post=None):
        """Result of an incremental call against the oracle's inference `post` of the new snapshot."""
        want = oracle.changed_nodes(self.ref, post)[-1]
        keys_post = self.keys if keys_post is None else keys_post
        X_post = self.X if X_post is None else X_post
        n_post = self.n if n_post is None else n_post
        user_post = self.user_terms if user_post is None else user_post
        if exact:
            assert np.array_equal(res["changed_ids"], want), "changed-node set differs"
            assert np.array_equal(res["embeddings"].view(np.uint32), post["h"][-1][want].view(np.uint32))
        else:
            # accumulated aggregators: the returned rows meet the bar of check_accumulated; the changed
            # sets may differ only in rows whose true change is itself below the tolerance (a delta
            # that vanishes in fp32, or a change the oracle's single rounding hides; Sec. 7 concedes
            # loss for the delta method), and only in a small part of the set
            got = res["changed_ids"]
            assert np.all(np.diff(got) > 0)
            hk_pre, hk_post = self.ref["h"][-1], post["h"][-1]
            k = len(self.model["layers"])
            memo = {}

            def magnitudes():                      # of the new snapshot; computed only if a row needs its rounding bound
                if not memo:
                    rp2, col2 = oracle.csr_from_keys(n_post, keys_post)
                    memo["mag"] = magnitude_inference(rp2, col2, X_post, self.model, user_post)[k]
                    memo["deg"] = np.diff(rp2)
                return memo
            k_lin = chain_lengths(self.model)[k - 1]
            sym = np.setxor1d(got, want)
            if sym.size:
                delta = row_err(hk_pre[sym], hk_post[sym])
                if np.any(delta > tol):
                    m = magnitudes()
                    bound = (k * (m["deg"][sym] + k_lin + 2) * U32)[:, None] * m["mag"][sym].astype(np.float64)
                    small = np.abs(hk_post[sym].astype(np.float64) - hk_pre[sym]) <= bound
                    assert np.all((delta <= tol) | small.all(axis=1)), "changed sets differ in a row that really changed"
            self.last_set_mismatch = int(sym.size)
            assert sym.size <= max(8, (got.size + want.size) // 100), "changed sets differ in %d rows" % sym.size
            rep = check_accumulated(res["embeddings"], hk_post[got], lambda: magnitudes()["mag"][got],
                                    lambda: magnitudes()["deg"][got], k_lin, k, tol, "returned rows")
            rep["set_mismatch"] = int(sym.size)
            self.reports.append(rep)
            print("parity returned rows: strict max %.3g, %d of %d rows beyond the strict bar; changed sets differ in %d rows"
                  % (rep["strict_max"], rep["rows_beyond_strict"], rep["rows"], sym.size))
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
        post = oracle.full_infer(*oracle.csr_from_keys(self.n, self.keys), X2, self.model, self.precision, self.user_terms)
        want = self._compare(res, post, exact, tol, X_post=X2)
        self.X, self.ref = X2, post
        return res, want

    def user_step(self, events, rows, exact=True, tol=1e-5):
        """User-defined events through ink_apply_user_events, against the oracle's full inference
        with the terms those events leave behind."""
        rows = np.ascontiguousarray(rows, np.float32).reshape(len(events), -1)
        res = self.ink.apply_user_events(events, rows)
        assert (res["n_applied_ins"], res["n_applied_del"], res["n_noop"]) == (0, 0, 0)
        widths = [L["out_dim"] for L in self.model["layers"]]
        terms = oracle.apply_user_events(self.user_terms, widths, self.n, events, rows)
        post = oracle.full_infer(*oracle.csr_from_keys(self.n, self.keys), self.X, self.model, self.precision, terms)
        want = self._compare(res, post, exact, tol, user_post=terms)
        self.user_terms, self.ref = terms, post
        return res, want

    def add_nodes(self, features, exact=True, tol=1e-5):
        """Appends nodes without edges through ink_add_nodes; the oracle re-runs on the grown graph."""
        features = np.ascontiguousarray(features, np.float32).reshape(-1, self.X.shape[1])
        k = features.shape[0]
        res = self.ink.add_nodes(features)
        n2 = self.n + k
        X2 = np.concatenate([self.X, features], axis=0)
        terms = [None if t is None else np.concatenate([t, np.zeros((k, t.shape[1]), np.float32)]) for t in self.user_terms]
        post = oracle.full_infer(*oracle.csr_from_keys(n2, self.keys), X2, self.model, self.precision, terms)
        self.user_terms = terms
        ids = np.arange(self.n, n2, dtype=np.int32)
        assert res["n_changed"] == k and np.array_equal(res["changed_ids"], ids)
        for l in range(len(post["h"])):          # the old nodes' rows are untouched by definition
            assert np.array_equal(post["h"][l][:self.n].view(np.uint32), self.ref["h"][l].view(np.uint32))
        want = post["h"][-1][ids]
        if exact:
            assert np.array_equal(res["embeddings"].view(np.uint32), want.view(np.uint32))
        elif k:
            assert row_err(res["embeddings"], want).max() <= tol
        self.n, self.X, self.ref = n2, X2, post
        return res

    def step(self, op, bs, bd, exact=True, tol=1e-5, affected=False):
        from paper_2309_11071_amd.binding import make_updates
        res = self.ink.apply_updates(make_updates(op, bs, bd), affected=affected)
        keys2, n_ins, n_del, n_noop = oracle.apply_batch(self.keys, op, bs, bd)
        assert (res["n_applied_ins"], res["n_applied_del"], res["n_noop"]) == (n_ins, n_del, n_noop)
        post = oracle.full_infer(*oracle.csr_from_keys(self.n, keys2), self.X, self.model, self.precision, self.user_terms)
        want = self._compare(res, post, exact, tol, keys_post=keys2)
        self.keys, self.ref = keys2, post
        return res, want
