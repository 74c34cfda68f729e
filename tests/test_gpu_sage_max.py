"""GPU parity of the max/min path against the oracle, through the C ABI."""
import numpy as np
import pytest

import oracle
import synth
from util import Harness, row_rel_err

pytestmark = pytest.mark.gpu


def test_full_infer_cfg1_bit_exact_and_within_tolerance():
    h = Harness(synth.get_config(1))
    h.check_state(exact=True)
    h.check_graph()
    ref64 = oracle.full_infer(*oracle.csr_from_keys(h.n, h.keys), h.X, h.model, "f64")
    for l in (1, 2):
        assert row_rel_err(h.ink.get_layer(l, 0), ref64["h"][l]) <= 1e-5
    h.ink.close()


def test_updates_cfg1_sequence():
    h = Harness(synth.get_config(1))
    total = 0
    for b in range(6):
        op, bs, bd = h.sampler.next_batch()
        res, want = h.step(op, bs, bd)
        total += want.size
        h.check_graph()
        h.check_state(exact=True)
    assert total > 0
    h.ink.close()
