"""The pins must be sharp: each plausible mistake planted in the oracle (on the CPU, by replacing
one of its functions with a wrong variant) has to fail at least one of them.  A mutant that
survives means the oracle could carry that mistake unnoticed."""
import numpy as np
import pytest

import oracle
import test_oracle_pins as pins

REAL = {name: getattr(oracle, name) for name in
        ("agg_select", "agg_sum", "agg_gcn_sym", "linear", "transform", "apply_batch", "rows_differ",
         "apply_user_events")}


def _nb_lists(rowptr, col):
    return [col[rowptr[v]:rowptr[v + 1]] for v in range(rowptr.size - 1)]


# ---- wrong variants --------------------------------------------------------------------------
def select_ties_to_highest_id(rowptr, col, m, is_min=False):
    alpha, arg = REAL["agg_select"](rowptr, col, m, is_min)
    for v, nb in enumerate(_nb_lists(np.asarray(rowptr), np.asarray(col))):
        for i in range(m.shape[1]):
            if nb.size:
                arg[v, i] = max(int(u) for u in nb if m[u, i] == alpha[v, i])
    return alpha, arg


def select_empty_row_keeps_sentinel(rowptr, col, m, is_min=False):
    alpha, arg = REAL["agg_select"](rowptr, col, m, is_min)
    deg = np.diff(np.asarray(rowptr))
    alpha[deg == 0] = np.inf if is_min else -np.inf
    return alpha, arg


def select_max_and_min_swapped(rowptr, col, m, is_min=False):
    return REAL["agg_select"](rowptr, col, m, not is_min)


def sum_counts_the_node_itself(rowptr, col, m, mean=False):
    out = REAL["agg_sum"](rowptr, col, m, mean=False) + np.asarray(m, np.float32)
    if mean:
        deg = np.maximum(np.diff(np.asarray(rowptr)), 1).astype(np.float32)
        out = out / deg[:, None]
    return out.astype(np.float32)


def mean_divides_by_degree_plus_one(rowptr, col, m, mean=False):
    out = REAL["agg_sum"](rowptr, col, m, mean=False)
    if mean:
        out = out / (np.diff(np.asarray(rowptr)) + 1).astype(np.float32)[:, None]
    return out.astype(np.float32)


def sum_along_out_edges(rowptr, col, m, mean=False):
    """Transposed adjacency: aggregates over out-neighbours."""
    rowptr, col = np.asarray(rowptr), np.asarray(col)
    n = rowptr.size - 1
    dst = np.repeat(np.arange(n), np.diff(rowptr))
    out = np.zeros((n, m.shape[1]), np.float64)
    np.add.at(out, col, np.asarray(m, np.float64)[dst])
    if mean:
        out = out / np.maximum(np.bincount(col, minlength=n), 1)[:, None]
    return out.astype(np.float32)


def gcn_without_self_loop(rowptr, col, h):
    rowptr, col = np.asarray(rowptr), np.asarray(col)
    n = rowptr.size - 1
    c = 1.0 / np.sqrt(np.diff(rowptr) + 1.0)
    dst = np.repeat(np.arange(n), np.diff(rowptr))
    out = np.zeros((n, h.shape[1]), np.float64)
    np.add.at(out, dst, (c[col] * c[dst])[:, None] * np.asarray(h, np.float64)[col])
    return out.astype(np.float32)


def gcn_row_normalised(rowptr, col, h):
    rowptr, col = np.asarray(rowptr), np.asarray(col)
    n = rowptr.size - 1
    dst = np.repeat(np.arange(n), np.diff(rowptr))
    out = np.asarray(h, np.float64).copy()
    np.add.at(out, dst, np.asarray(h, np.float64)[col])
    return (out / (np.diff(rowptr) + 1.0)[:, None]).astype(np.float32)


def linear_without_bias(x, W, bias=None, relu=False, precision="f64"):
    return REAL["linear"](x, W, None, relu, precision)


def linear_relu_before_bias(x, W, bias=None, relu=False, precision="f64"):
    y = REAL["linear"](x, W, None, relu, precision)
    return y if bias is None else (y + np.asarray(bias, np.float32)).astype(np.float32)


def linear_transposed(x, W, bias=None, relu=False, precision="f64"):
    """Reads the weight array as if it were stored [out][in]."""
    W = np.ascontiguousarray(W, np.float32)
    return REAL["linear"](x, W.ravel().reshape(W.shape[1], W.shape[0]).T, bias, relu, precision)


def linear_f32_mode_accumulates_in_f64(x, W, bias=None, relu=False, precision="f64"):
    return REAL["linear"](x, W, bias, relu, "f64")


def transform_sage_drops_self_term(model, l, alpha, h_prev, precision="f64"):
    if model["kind"] == "sage":
        h_prev = np.zeros_like(h_prev)
    return REAL["transform"](model, l, alpha, h_prev, precision)


def transform_sage_swaps_the_two_weights(model, l, alpha, h_prev, precision="f64"):
    if model["kind"] == "sage" and alpha.shape == h_prev.shape:
        return REAL["transform"](model, l, h_prev, alpha, precision)
    return REAL["transform"](model, l, alpha, h_prev, precision)


def transform_relu_on_every_layer(model, l, alpha, h_prev, precision="f64"):
    return np.maximum(REAL["transform"](model, l, alpha, h_prev, precision), 0.0).astype(np.float32)


def transform_no_relu_on_hidden_layers(model, l, alpha, h_prev, precision="f64"):
    m2 = dict(model)
    m2["layers"] = [dict(L, act="none") for L in model["layers"]]
    return REAL["transform"](m2, l, alpha, h_prev, precision)


def transform_gin_eps_sign(model, l, alpha, h_prev, precision="f64"):
    m2 = dict(model)
    m2["gin_eps"] = -float(model.get("gin_eps", 0.0))
    return REAL["transform"](m2, l, alpha, h_prev, precision)


def transform_gin_forgets_inner_relu(model, l, alpha, h_prev, precision="f64"):
    if model["kind"] != "gin":
        return REAL["transform"](model, l, alpha, h_prev, precision)
    L = model["layers"][l]
    x = ((1.0 + float(model.get("gin_eps", 0.0))) * h_prev + alpha).astype(np.float32)
    z = REAL["linear"](x, L["W_neigh"], L.get("bias"), False, precision)
    return REAL["linear"](z, L["W_mlp2"], L.get("bias_mlp2"), L["act"] == "relu", precision)


def batch_first_op_wins(keys, op, src, dst):
    seen, keep = set(), []
    for i, (s, d) in enumerate(zip(src.tolist(), dst.tolist())):
        if (s, d) not in seen:
            seen.add((s, d))
            keep.append(i)
    keep = np.asarray(keep, np.int64)
    out, a, r, _ = REAL["apply_batch"](keys, op[keep], src[keep], dst[keep])
    return out, a, r, len(op) - a - r


def batch_accepts_self_loops(keys, op, src, dst):
    out, a, r, z = REAL["apply_batch"](keys, op, src, dst)
    loops = [(int(s) << 32) | int(s) for o, s, d in zip(op.tolist(), src.tolist(), dst.tolist()) if s == d and o == 0]
    if loops:
        out2 = np.union1d(out, np.asarray(loops, np.int64))
        a, z = a + out2.size - out.size, z - (out2.size - out.size)
        out = out2
    return out, a, r, z


def rows_differ_by_value(a, b):
    return (np.asarray(a, np.float32) != np.asarray(b, np.float32)).any(axis=1)


def transform_user_term_after_the_activation(model, l, alpha, h_prev, precision="f64", user=None):
    y = REAL["transform"](model, l, alpha, h_prev, precision)
    return y if user is None else (y + np.asarray(user, np.float32)).astype(np.float32)


def transform_ignores_the_user_term(model, l, alpha, h_prev, precision="f64", user=None):
    return REAL["transform"](model, l, alpha, h_prev, precision)


def user_events_add_acts_as_set(user_terms, widths, n, events, rows):
    events = [(l, t, oracle.USER_SET if op == oracle.USER_ADD else op) for l, t, op in events]
    return REAL["apply_user_events"](user_terms, widths, n, events, rows)


def user_events_ignore_the_layer(user_terms, widths, n, events, rows):
    events = [(1, t, op) for l, t, op in events]
    return REAL["apply_user_events"](user_terms, widths, n, events, rows)


def _call(fn, *args):
    return lambda: fn(*args)


ALL_SELECT = [_call(pins.test_select_matches_brute_force, s, m) for s in range(3) for m in (False, True)] + \
    [pins.test_select_golden_ties, pins.test_min_is_negated_max_of_negation, pins.test_edgeless_graph,
     pins.test_full_infer_sage_against_dense_formula]
ALL_SUM = [pins.test_sum_and_mean_match_dense_matmul, pins.test_full_infer_gin_against_dense_formula,
           _call(pins.test_isolated_new_node_has_the_closed_form_embedding, "sage", "mean")]
ALL_GCN = [pins.test_gcn_sym_matches_dense_normalised_adjacency, pins.test_gcn_sym_golden_star_and_path,
           pins.test_full_infer_gcn_against_dense_formula]
ALL_LINEAR = [pins.test_linear_matches_library_matmul_and_is_not_transposed, pins.test_linear_exact_on_small_integers,
              pins.test_linear_precision_modes_differ_where_rounding_order_says_so]
ALL_MODEL = [pins.test_full_infer_sage_against_dense_formula, pins.test_full_infer_gin_against_dense_formula,
             pins.test_full_infer_gcn_against_dense_formula,
             pins.test_one_layer_model_is_one_aggregation_and_one_linear_map]
ALL_BATCH = [pins.test_apply_batch_net_effect]
ALL_USER = [_call(pins.test_user_term_is_added_before_the_activation, "sage", "max"),
            _call(pins.test_user_term_is_added_before_the_activation, "gin", "sum"),
            pins.test_user_events_group_by_layer_and_target_in_list_order,
            pins.test_a_user_event_stays_in_the_out_neighbourhood]
ALL_DIFF = [_call(pins.test_update_invariants, "sage", "max"), pins.test_rows_differ_is_bitwise]

MUTANTS = [
    ("agg_select", select_ties_to_highest_id, ALL_SELECT),
    ("agg_select", select_empty_row_keeps_sentinel, ALL_SELECT),
    ("agg_select", select_max_and_min_swapped, ALL_SELECT),
    ("agg_sum", sum_counts_the_node_itself, ALL_SUM),
    ("agg_sum", mean_divides_by_degree_plus_one, ALL_SUM),
    ("agg_sum", sum_along_out_edges, ALL_SUM),
    ("agg_gcn_sym", gcn_without_self_loop, ALL_GCN),
    ("agg_gcn_sym", gcn_row_normalised, ALL_GCN),
    ("linear", linear_without_bias, ALL_LINEAR + ALL_MODEL),
    ("linear", linear_relu_before_bias, ALL_LINEAR + ALL_MODEL),
    ("linear", linear_transposed, ALL_LINEAR),
    ("linear", linear_f32_mode_accumulates_in_f64, ALL_LINEAR),
    ("transform", transform_sage_drops_self_term, ALL_MODEL),
    ("transform", transform_sage_swaps_the_two_weights, ALL_MODEL),
    ("transform", transform_relu_on_every_layer, ALL_MODEL),
    ("transform", transform_no_relu_on_hidden_layers, ALL_MODEL),
    ("transform", transform_gin_eps_sign, ALL_MODEL),
    ("transform", transform_gin_forgets_inner_relu, ALL_MODEL),
    ("transform", transform_user_term_after_the_activation, ALL_USER),
    ("transform", transform_ignores_the_user_term, ALL_USER),
    ("apply_user_events", user_events_add_acts_as_set, ALL_USER),
    ("apply_user_events", user_events_ignore_the_layer, ALL_USER),
    ("apply_batch", batch_first_op_wins, ALL_BATCH),
    ("apply_batch", batch_accepts_self_loops, ALL_BATCH),
    ("rows_differ", rows_differ_by_value, ALL_DIFF),
]


@pytest.mark.parametrize("attr,mutant,checks", MUTANTS, ids=[m[1].__name__ for m in MUTANTS])
def test_a_planted_mistake_fails_a_pin(monkeypatch, attr, mutant, checks):
    monkeypatch.setattr(oracle, attr, mutant)
    caught = []
    for check in checks:
        try:
            check()
        except AssertionError:
            caught.append(check)
    assert caught, "no pin noticed %s" % mutant.__name__


def test_the_unmodified_oracle_passes_the_same_checks():
    for _, _, checks in MUTANTS:
        for check in checks:
            check()
