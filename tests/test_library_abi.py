"""Host-side checks that need no GPU: the shared library loads, exports every symbol the header
declares, and the Python struct mirrors match the header's layout."""
import ctypes
import os
import re

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "ink.h")


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ink_[a-z_]+)\s*\(", text)))


def test_header_declares_the_boundary_calls():
    names = declared_functions()
    for must in ("ink_create", "ink_full_infer", "ink_apply_updates", "ink_apply_updates_affected", "ink_update_features", "ink_add_nodes", "ink_get_layer", "ink_get_graph",
                 "ink_get_stats", "ink_set_profiling", "ink_last_error", "ink_destroy"):
        assert must in names


def test_library_exports_every_declared_symbol():
    from paper_2309_11071_amd import binding
    if not os.path.exists(binding.lib_path()):
        pytest.skip("libink.so not built (run __graft_entry__.build())")
    lib = ctypes.CDLL(binding.lib_path())
    for name in declared_functions():
        assert hasattr(lib, name), name


def test_struct_layouts_match_the_header():
    from paper_2309_11071_amd import binding as b
    # compile a tiny C program against the header and compare sizes / offsets
    import subprocess
    import tempfile
    src = r'''
#include <stdio.h>
#include <stddef.h>
#include "ink.h"
int main(void) {
  printf("%zu %zu %zu %zu %zu %zu %zu %zu\n", sizeof(ink_csr), sizeof(ink_layer), sizeof(ink_model),
         sizeof(ink_options), sizeof(ink_edge_update), sizeof(ink_update_result), sizeof(ink_layer_stats),
         sizeof(ink_stats));
  printf("%zu %zu %zu %zu\n", offsetof(ink_options, pool_reserve), offsetof(ink_layer, act),
         offsetof(ink_stats, ms), offsetof(ink_edge_update, src));
  printf("%zu %zu %zu %zu\n", offsetof(ink_options, small_batch_limit), offsetof(ink_options, node_capacity),
         offsetof(ink_options, batch_mem), offsetof(ink_update_result, n_applied_ins));
  return 0;
}
'''
    with tempfile.TemporaryDirectory() as d:
        open(os.path.join(d, "t.c"), "w").write(src)
        exe = os.path.join(d, "t")
        subprocess.check_call(["gcc", "-I", os.path.join(ROOT, "include"), "-o", exe, os.path.join(d, "t.c")])
        out = subprocess.check_output([exe]).decode().split()
    sizes = [int(x) for x in out[:8]]
    mirrors = [b._Csr, b._Layer, b._Model, b._Options, None, b._Result, b._LayerStats, b._Stats]
    for sz, m in zip(sizes, mirrors):
        if m is not None:
            assert ctypes.sizeof(m) == sz, m
    assert b.EDGE_UPDATE_DTYPE.itemsize == sizes[4]
    offs = [int(x) for x in out[8:]]
    assert b._Options.pool_reserve.offset == offs[0]
    assert b._Layer.act.offset == offs[1]
    assert b._Stats.ms.offset == offs[2]
    assert b.EDGE_UPDATE_DTYPE.fields["src"][1] == offs[3]
    assert b._Options.small_batch_limit.offset == offs[4]
    assert b._Options.node_capacity.offset == offs[5]
    assert b._Options.batch_mem.offset == offs[6]
    assert b._Result.n_applied_ins.offset == offs[7]


def test_binding_refuses_to_run_without_the_library(monkeypatch, tmp_path):
    from paper_2309_11071_amd import binding
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "HERE", str(tmp_path))
    with pytest.raises(RuntimeError):
        binding.load_library()


def test_batch_sampler_is_seeded_and_valid():
    import synth
    cfg = synth.get_config(3, 256)
    s, d = synth.make_graph(cfg)
    a = synth.BatchSampler(cfg, s, d)
    b = synth.BatchSampler(cfg, s, d)
    keys = set(synth.edge_keys(s, d).tolist())
    for _ in range(3):
        o1, s1, d1 = a.next_batch()
        o2, s2, d2 = b.next_batch()
        assert np.array_equal(o1, o2) and np.array_equal(s1, s2) and np.array_equal(d1, d2)
        assert (o1 == 1).sum() == cfg.batch // 2
        for o, u, v in zip(o1.tolist(), s1.tolist(), d1.tolist()):
            k = (v << 32) | u
            assert u != v
            if o == 1:
                assert k in keys
                keys.discard(k)
            else:
                assert k not in keys
                keys.add(k)
    cs, cd = a.current_edges()
    assert set(synth.edge_keys(cs, cd).tolist()) == keys
