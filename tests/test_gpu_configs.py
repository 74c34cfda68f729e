"""Parity at the benchmark's sizes: configs 2 and 3 at full size (the oracle needs 10-20 s per
full inference there), configs 4 and 5 on 1/16-scale replicas (their full size is 20 M nodes).
State after a sequence of batches is compared table by table with a fresh oracle inference of
the final snapshot: an error made by any earlier batch would persist in the cache."""
import numpy as np
import pytest

import oracle
import synth
from util import Harness, scaled_rel_err

pytestmark = pytest.mark.gpu


def test_config3_full_size_exact():
    cfg = synth.get_config(3)
    h = Harness(cfg, precision="f32")
    h.check_state(exact=True)
    from paper_2309_11071_amd.binding import make_updates
    for b in range(2):                      # no oracle in between: only the key set is tracked
        op, bs, bd = h.sampler.next_batch()
        res = h.ink.apply_updates(make_updates(op, bs, bd))
        h.keys, n_ins, n_del, n_noop = oracle.apply_batch(h.keys, op, bs, bd)
        assert (res["n_applied_ins"], res["n_applied_del"], res["n_noop"]) == (n_ins, n_del, n_noop)
    h.ref = oracle.full_infer(*oracle.csr_from_keys(h.n, h.keys), h.X, h.model, "f32")
    h.check_state(exact=True)
    op, bs, bd = h.sampler.next_batch()      # third batch: changed set and embeddings, exactly
    res, want = h.step(op, bs, bd, exact=True)
    assert want.size > 1000
    st = h.ink.stats()["layers"]
    assert st[1]["n_exposed"] > 0 and st[0]["n_events"] == cfg.batch
    h.check_state(exact=True)
    h.check_graph()
    h.ink.close()


def test_config2_full_size_within_tolerance():
    cfg = synth.get_config(2)
    h = Harness(cfg, precision="f64")
    from paper_2309_11071_amd.binding import make_updates
    for b in range(3):
        op, bs, bd = h.sampler.next_batch()
        res = h.ink.apply_updates(make_updates(op, bs, bd))
        h.keys, n_ins, n_del, n_noop = oracle.apply_batch(h.keys, op, bs, bd)
        assert (res["n_applied_ins"], res["n_applied_del"], res["n_noop"]) == (n_ins, n_del, n_noop)
        assert res["n_changed"] > 1000
    post = oracle.full_infer(*oracle.csr_from_keys(h.n, h.keys), h.X, h.model, "f64")
    for l in (1, 2):
        err = scaled_rel_err(h.ink.get_layer(l, 0), post["h"][l])
        assert err <= 1e-5, (l, err)
    ids = res["changed_ids"]
    assert np.array_equal(h.ink.get_layer(2, 0)[ids].view(np.uint32), res["embeddings"].view(np.uint32))
    h.ink.close()


@pytest.mark.parametrize("cfg_id,exact", [(4, False), (5, True)])
def test_configs_4_and_5_at_one_sixteenth(cfg_id, exact):
    cfg = synth.get_config(cfg_id, 16)
    h = Harness(cfg, precision="f32" if exact else "f64")
    h.check_state(exact=exact)
    for b in range(3):
        op, bs, bd = h.sampler.next_batch()
        h.step(op, bs, bd, exact=exact)
    h.check_state(exact=exact)
    h.check_graph()
    h.ink.close()


def test_config5_batch_sizes():
    cfg = synth.get_config(5, 64)
    h = Harness(cfg, precision="f32")
    for B in (1, 10, 100, 1000, 10000):
        op, bs, bd = h.sampler.next_batch(B)
        res, want = h.step(op, bs, bd, exact=True)
    h.check_state(exact=True)
    h.ink.close()
