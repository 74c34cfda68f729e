"""CPU oracle (test infrastructure only): plain k-layer GNN inference on a graph snapshot.

Only tests/, the smoke check and the benchmark's cpu_baseline leg may import this package.
It shares no code with the HIP library and never imports it.

The oracle is the definition, not the method: it recomputes every layer for every node on
the snapshot it is given (the paper's "classic method", Sec. 1; "Full", Sec. 4.1).  The
incremental method must reproduce it (Abstract: identical output for min/max).

Model conventions (dict as produced by synth.make_model):
  sage: a = A(h_u : u in N(v));  h' = act(W_neigh^T a + W_self^T h_v)          eqs. (3)(4)
  gcn : a = A(h_u : u in N(v) + {v}) normalised;  h' = act(W^T a + b)          eqs. (1)(2)
  gin : a = sum(h_u : u in N(v));  h' = act(MLP((1 + eps) h_v + a))            eqs. (5)(6)
        MLP = Linear -> ReLU -> Linear
`act` is ReLU on every layer but the last.
"""
import ctypes
import os

import numpy as np

from .build import build as _build

_lib = ctypes.CDLL(_build())
_i64p = ctypes.POINTER(ctypes.c_int64)
_i32p = ctypes.POINTER(ctypes.c_int32)
_f32p = ctypes.POINTER(ctypes.c_float)


def _p(a, t):
    return None if a is None else a.ctypes.data_as(t)


def _c(a, dt):
    return np.ascontiguousarray(a, dtype=dt)


def agg_select(rowptr, col, m, is_min=False):
    """(alpha, arg): per-dimension max (or min) over in-neighbours, lowest id on ties (Sec. 2.1)."""
    rowptr, col, m = _c(rowptr, np.int64), _c(col, np.int32), _c(m, np.float32)
    n, d = rowptr.size - 1, m.shape[1]
    alpha = np.empty((n, d), np.float32)
    arg = np.empty((n, d), np.int32)
    _lib.orc_agg_select(ctypes.c_int64(n), _p(rowptr, _i64p), _p(col, _i32p), _p(m, _f32p),
                        ctypes.c_int32(d), ctypes.c_int32(int(is_min)), _p(alpha, _f32p),
                        _p(arg, _i32p))
    return alpha, arg


def agg_sum(rowptr, col, m, mean=False):
    rowptr, col, m = _c(rowptr, np.int64), _c(col, np.int32), _c(m, np.float32)
    n, d = rowptr.size - 1, m.shape[1]
    alpha = np.empty((n, d), np.float32)
    _lib.orc_agg_sum(ctypes.c_int64(n), _p(rowptr, _i64p), _p(col, _i32p), _p(m, _f32p),
                     ctypes.c_int32(d), ctypes.c_int32(int(mean)), _p(alpha, _f32p))
    return alpha


def agg_gcn_sym(rowptr, col, h):
    rowptr, col, h = _c(rowptr, np.int64), _c(col, np.int32), _c(h, np.float32)
    n, d = rowptr.size - 1, h.shape[1]
    alpha = np.empty((n, d), np.float32)
    _lib.orc_agg_gcn_sym(ctypes.c_int64(n), _p(rowptr, _i64p), _p(col, _i32p), _p(h, _f32p),
                         ctypes.c_int32(d), _p(alpha, _f32p))
    return alpha


def linear(x, W, bias=None, relu=False, precision="f64"):
    """act(x W + b).  precision "f64": fp64 accumulate, round once; "f32": fp32 FMA chain, k ascending."""
    x, W = _c(x, np.float32), _c(W, np.float32)
    bias = None if bias is None else _c(bias, np.float32)
    rows, din = x.shape
    assert W.shape[0] == din
    dout = W.shape[1]
    y = np.empty((rows, dout), np.float32)
    mode = {"f64": 0, "f32": 1}[precision]
    _lib.orc_linear(ctypes.c_int64(rows), ctypes.c_int32(din), ctypes.c_int32(dout),
                    _p(x, _f32p), _p(W, _f32p), _p(bias, _f32p), ctypes.c_int32(int(relu)),
                    ctypes.c_int32(mode), _p(y, _f32p))
    return y


def aggregate(rowptr, col, m, agg):
    """Dispatch on the aggregator name; returns (alpha, arg or None)."""
    if agg == "max":
        return agg_select(rowptr, col, m, is_min=False)
    if agg == "min":
        return agg_select(rowptr, col, m, is_min=True)
    if agg == "sum":
        return agg_sum(rowptr, col, m), None
    if agg == "mean":
        return agg_sum(rowptr, col, m, mean=True), None
    if agg == "gcn_sym":
        return agg_gcn_sym(rowptr, col, m), None
    raise ValueError(agg)


def transform(model, l, alpha, h_prev, precision="f64", user=None):
    """Combination + activation of layer l (0-based): h_l = act(T(alpha_l, h_{l-1})) (Sec. 2.2 item 2).

    user: optional [n][out_dim] term of user-defined events (Sec. 2.6; Sec. 3.2 shows the use: a
    user_apply step adds a user-supplied per-node term to the tensor between the linear map and the
    activation): h_l = act(T(alpha_l, h_{l-1}) + user).  It is added to the rounded result of the
    linear map, in fp64 (precision "f64") or as one fp32 addition ("f32"), before the activation."""
    if user is not None:
        L = model["layers"][l]
        lin = dict(model, layers=[dict(x, act="none") if i == l else x for i, x in enumerate(model["layers"])])
        y = transform(lin, l, alpha, h_prev, precision)
        if precision == "f64":
            y = (y.astype(np.float64) + np.asarray(user, np.float64)).astype(np.float32)
        else:
            y = y + np.asarray(user, np.float32)
        if L["act"] == "relu":
            y = np.where(y > 0, y, np.float32(0.0)).astype(np.float32)
        return y
    L = model["layers"][l]
    relu = L["act"] == "relu"
    kind = model["kind"]
    if kind == "sage":
        x = np.concatenate([alpha, h_prev], axis=1)
        W = np.concatenate([L["W_neigh"], L["W_self"]], axis=0)
        return linear(x, W, L.get("bias"), relu, precision)
    if kind == "gcn":
        return linear(alpha, L["W_neigh"], L.get("bias"), relu, precision)
    if kind == "gin":
        eps = float(model.get("gin_eps", 0.0))
        if precision == "f64":
            x = ((1.0 + eps) * h_prev.astype(np.float64) + alpha.astype(np.float64)).astype(np.float32)
        else:
            x = (np.float32(1.0 + eps) * h_prev).astype(np.float32) + alpha
        z = linear(x, L["W_neigh"], L.get("bias"), True, precision)
        return linear(z, L["W_mlp2"], L.get("bias_mlp2"), relu, precision)
    raise ValueError(kind)


def full_infer(rowptr, col, X, model, precision="f64", user_terms=None):
    """Plain inference.  Returns dict with lists h[0..k], alpha[1..k] (index 0 unused), arg[1..k].
    user_terms: optional list, entry l - 1 = the [n][out_dim_l] term of layer l or None (see transform)."""
    h = [np.ascontiguousarray(X, dtype=np.float32)]
    alpha, arg = [None], [None]
    for l in range(len(model["layers"])):
        a, g = aggregate(rowptr, col, h[l], model["agg"])      # m_{l+1} = h_l (aggregate first)
        alpha.append(a)
        arg.append(g)
        u = None if user_terms is None else user_terms[l]
        h.append(transform(model, l, a, h[l], precision) if u is None else transform(model, l, a, h[l], precision, user=u))
    return dict(h=h, alpha=alpha, arg=arg)


USER_SET, USER_ADD, USER_CLEAR = 0, 1, 2


def apply_user_events(user_terms, widths, n, events, rows):
    """Net effect of an ordered list of user-defined events (Sec. 2.6) on the per-layer user terms.

    events: iterable of (layer 1..k, target, op); rows[i] = the event's row (its first width_l
    entries count).  Events are grouped by (layer, target) and applied in list order to that node's
    term: set replaces it, add adds to it (one fp32 addition per event), clear zeroes it.  Returns
    a new list of terms (a layer never touched stays None)."""
    out = [None if t is None else t.copy() for t in user_terms]
    for (layer, target, op), row in zip(events, rows):
        w = widths[layer - 1]
        if out[layer - 1] is None:
            out[layer - 1] = np.zeros((n, w), np.float32)
        t = out[layer - 1]
        r = np.asarray(row, np.float32)[:w]
        if op == USER_SET:
            t[target] = r
        elif op == USER_ADD:
            t[target] = t[target] + r
        elif op == USER_CLEAR:
            t[target] = 0.0
        else:
            raise ValueError(op)
    return out


def rows_differ(a, b):
    """Boolean mask of rows whose float32 bit patterns differ anywhere (Sec. 2.5.2: a node whose
    embedding equals its previous value is resilient and propagates nothing)."""
    a = np.ascontiguousarray(a, np.float32).view(np.uint32)
    b = np.ascontiguousarray(b, np.float32).view(np.uint32)
    return (a != b).any(axis=1)


def changed_nodes(pre, post):
    """Per-layer ascending id arrays of nodes whose h_l differs bitwise between two inferences."""
    return [np.nonzero(rows_differ(pre["h"][l], post["h"][l]))[0].astype(np.int32)
            for l in range(len(pre["h"]))]


def apply_batch(keys, op, src, dst):
    """Net effect of an ordered update list on an edge set (Sec. 2.1: Delta E is the set of
    edges inserted or removed between two timestamps).

    keys: sorted unique int64 (dst << 32 | src).  op: 0 insert, 1 delete.  The list is applied
    in order to a simple directed graph without self loops: inserting a present edge, deleting
    an absent one or inserting a self loop does nothing.  Returns (new_keys, n_ins, n_del,
    n_noop) where n_ins / n_del count edges whose presence differs between the two snapshots.
    """
    present = {}
    def is_in(k):
        i = np.searchsorted(keys, k)
        return bool(i < keys.size and keys[i] == k)
    for o, s, d in zip(op.tolist(), src.tolist(), dst.tolist()):
        if s == d:
            continue
        k = (d << 32) | s
        if k not in present:
            present[k] = [is_in(k), None]
        present[k][1] = (o == 0)
    add = sorted(k for k, (was, now) in present.items() if now and not was)
    rem = sorted(k for k, (was, now) in present.items() if was and not now)
    out = keys
    if rem:
        out = np.setdiff1d(out, np.array(rem, dtype=np.int64), assume_unique=True)
    if add:
        out = np.union1d(out, np.array(add, dtype=np.int64))
    n = len(op)
    return out, len(add), len(rem), n - len(add) - len(rem)


def csr_from_keys(n, keys):
    """In-neighbour CSR from sorted unique (dst << 32 | src) keys."""
    dst = (keys >> 32).astype(np.int64)
    rowptr = np.zeros(n + 1, dtype=np.int64)
    np.cumsum(np.bincount(dst, minlength=n), out=rowptr[1:])
    return rowptr, (keys & 0xFFFFFFFF).astype(np.int32)


def affected_area(n, out_rowptr, out_col, changed_dst, k):
    """Theoretical affected area of a batch (Sec. 1, Fig. "Inference on a streaming graph" (b);
    Sec. 4.1 "Affected"): layer 1 can change only at the destinations of the changed edges; layer l
    at those of layer l - 1, at their out-neighbours, and again at the changed destinations.
    out_rowptr / out_col: out-neighbour CSR of the NEW snapshot.  Returns k ascending id arrays."""
    seed = np.unique(np.asarray(changed_dst, np.int64))
    areas, cur = [], seed
    for l in range(k):
        if l > 0:
            nb = [out_col[out_rowptr[v]:out_rowptr[v + 1]] for v in cur.tolist()]
            cur = np.unique(np.concatenate([cur, seed] + [x.astype(np.int64) for x in nb])) if nb else seed
        areas.append(cur.astype(np.int32))
    return areas


def affected_infer(rowptr, col, X, model, prev, areas, precision="f64"):
    """The "Affected" baseline (Sec. 4.1): inference on the theoretically affected area only.  Every
    node of areas[l] is recomputed at layer l + 1 from its whole neighbourhood in the new snapshot
    (rowptr, col) whether or not anything it reads changed; every other row is taken from `prev`,
    the inference of the previous snapshot.  Not for the degree-normalised aggregator, whose
    affected area also holds the out-neighbours of every node whose degree changed."""
    if model["agg"] == "gcn_sym":
        raise ValueError("affected_infer: gcn_sym not supported")
    h = [np.ascontiguousarray(X, dtype=np.float32)]
    alpha, arg = [None], [None]
    for l in range(len(model["layers"])):
        rows = areas[l].astype(np.int64)
        sub_rp = np.zeros(rows.size + 1, np.int64)
        np.cumsum(rowptr[rows + 1] - rowptr[rows], out=sub_rp[1:])
        sub_col = np.concatenate([col[rowptr[v]:rowptr[v + 1]] for v in rows.tolist()]) if rows.size else np.zeros(0, np.int32)
        a, g = aggregate(sub_rp, sub_col, h[l], model["agg"])
        al = prev["alpha"][l + 1].copy()
        al[rows] = a
        gl = None
        if g is not None:
            gl = prev["arg"][l + 1].copy()
            gl[rows] = g
        hl = prev["h"][l + 1].copy()
        if rows.size:
            hl[rows] = transform(model, l, a, h[l][rows], precision)
        alpha.append(al); arg.append(gl); h.append(hl)
    return dict(h=h, alpha=alpha, arg=arg)
