"""ctypes binding of include/ink.h: argument marshalling only.

Every step of the path runs inside libink.so; this module converts numpy / torch buffers to
the C structs and copies results out.  It fails loudly if the library has not been built.
"""
import ctypes as C
import os

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
INK_MAX_LAYERS = 8
INK_T_NCLASS = 6
TIME_CLASSES = ["graph", "events", "group", "agg", "compact", "transform"]
INK_K_NKERNEL = 8
KERNEL_SLOTS = ["agg_events", "agg_exposed", "agg_long", "agg_full", "sort", "xform"]
STATUS_NAMES = {0: "INK_OK", 1: "INK_E_ARG", 2: "INK_E_STATE", 3: "INK_E_OOM", 4: "INK_E_DEVICE",
                5: "INK_E_RANGE"}
MODEL_KINDS = {"sage": 0, "gcn": 1, "gin": 2}
AGGS = {"max": 0, "min": 1, "sum": 2, "mean": 3, "gcn_sym": 4}

USER_EVENT_DTYPE = np.dtype([("layer", np.int32), ("target", np.int32), ("op", np.int32), ("pad", np.int32)])
USER_SET, USER_ADD, USER_CLEAR = 0, 1, 2
EDGE_UPDATE_DTYPE = np.dtype([("op", np.uint8), ("pad", np.uint8, (3,)), ("src", np.int32),
                              ("dst", np.int32)])
assert EDGE_UPDATE_DTYPE.itemsize == 12


class InkError(RuntimeError):
    def __init__(self, status, msg):
        super().__init__("%s: %s" % (STATUS_NAMES.get(status, status), msg))
        self.status = status


class _Csr(C.Structure):
    _fields_ = [("n_nodes", C.c_int32), ("n_edges", C.c_int64), ("rowptr", C.c_void_p),
                ("col", C.c_void_p)]


class _Layer(C.Structure):
    _fields_ = [("in_dim", C.c_int32), ("out_dim", C.c_int32), ("mlp_hidden", C.c_int32),
                ("W_neigh", C.c_void_p), ("W_self", C.c_void_p), ("bias", C.c_void_p),
                ("W_mlp2", C.c_void_p), ("bias_mlp2", C.c_void_p), ("act", C.c_int32)]


class _Model(C.Structure):
    _fields_ = [("kind", C.c_int32), ("agg", C.c_int32), ("gin_eps", C.c_float),
                ("n_layers", C.c_int32), ("layers", C.POINTER(_Layer))]


class _Options(C.Structure):
    _fields_ = [("mem", C.c_int32), ("hip_stream", C.c_void_p), ("slack_factor", C.c_float),
                ("max_batch", C.c_int32), ("profile", C.c_int32), ("dense_threshold", C.c_float), ("batch_mem", C.c_int32),
                ("small_batch_limit", C.c_int32), ("pool_reserve", C.c_int64), ("node_capacity", C.c_int64)]


class _Result(C.Structure):
    _fields_ = [("n_changed", C.c_int64), ("changed_ids", C.c_void_p), ("embeddings", C.c_void_p),
                ("n_applied_ins", C.c_int64), ("n_applied_del", C.c_int64), ("n_noop", C.c_int64)]


class _LayerStats(C.Structure):
    _fields_ = [(k, C.c_int64) for k in ("n_sources", "n_events", "n_targets", "n_exposed",
                                         "n_regather_nb", "n_alpha_changed", "n_transformed",
                                         "n_changed", "n_no_deletion", "n_deletion_no_effect",
                                         "n_covered")] + [("dense", C.c_int32), ("pad_", C.c_int32),
                                                          ("n_regather_nb_long", C.c_int64),
                                                          ("ms_kernel", C.c_float * INK_K_NKERNEL)]


class _Stats(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("pad_", C.c_int32), ("layer", _LayerStats * INK_MAX_LAYERS),
                ("ms", C.c_float * INK_T_NCLASS), ("launches", C.c_int32 * INK_T_NCLASS),
                ("ms_total", C.c_float), ("pad2_", C.c_float)]


_lib = None


def lib_path():
    """libink.so next to this file, or the build named by INK_LIBRARY (to compare builds)."""
    return os.environ.get("INK_LIBRARY") or os.path.join(HERE, "libink.so")


def load_library():
    """Loads libink.so; raises if it is missing (there is no fallback path)."""
    global _lib
    if _lib is not None:
        return _lib
    path = lib_path()
    if not os.path.exists(path):
        raise RuntimeError("libink.so is not built: run `python -c 'import __graft_entry__ as g; g.build()'`")
    # PyTorch ships a HIP runtime of its own; whichever copy a process loads first is the one that
    # can see the GPU, so torch (the allocator of every device buffer handed to the library) goes first
    import torch
    if torch.cuda.is_available():
        torch.cuda.init()
    lib = C.CDLL(path)
    vp = C.c_void_p
    lib.ink_create.argtypes = [C.POINTER(_Csr), vp, C.c_int32, C.POINTER(_Model), C.POINTER(_Options),
                               C.POINTER(vp)]
    lib.ink_create.restype = C.c_int
    lib.ink_full_infer.argtypes = [vp]
    lib.ink_full_infer.restype = C.c_int
    lib.ink_full_infer_noalloc.argtypes = [vp]
    lib.ink_full_infer_noalloc.restype = C.c_int
    lib.ink_apply_updates.argtypes = [vp, vp, C.c_int64, C.POINTER(_Result)]
    lib.ink_apply_updates.restype = C.c_int
    lib.ink_apply_updates_affected.argtypes = [vp, vp, C.c_int64, C.POINTER(_Result)]
    lib.ink_apply_updates_affected.restype = C.c_int
    lib.ink_update_features.argtypes = [vp, vp, vp, C.c_int64, C.POINTER(_Result)]
    lib.ink_update_features.restype = C.c_int
    lib.ink_apply_user_events.argtypes = [vp, vp, vp, C.c_int32, C.c_int64, C.POINTER(_Result)]
    lib.ink_apply_user_events.restype = C.c_int
    lib.ink_add_nodes.argtypes = [vp, vp, C.c_int64, C.POINTER(_Result)]
    lib.ink_add_nodes.restype = C.c_int
    lib.ink_get_layer.argtypes = [vp, C.c_int32, C.c_int32, C.c_int64, C.c_int64, vp, C.c_int32,
                                  C.POINTER(C.c_int32)]
    lib.ink_get_layer.restype = C.c_int
    lib.ink_get_graph.argtypes = [vp, vp, vp]
    lib.ink_get_graph.restype = C.c_int
    lib.ink_set_profiling.argtypes = [vp, C.c_int32]
    lib.ink_set_profiling.restype = C.c_int
    lib.ink_get_stats.argtypes = [vp, vp, C.c_size_t]
    lib.ink_get_stats.restype = C.c_int
    lib.ink_last_error.argtypes = [vp]
    lib.ink_last_error.restype = C.c_char_p
    lib.ink_destroy.argtypes = [vp]
    lib.ink_destroy.restype = None
    _lib = lib
    return lib


def _ptr(a):
    return None if a is None else C.c_void_p(a.ctypes.data)


def make_updates(op, src, dst):
    """Packs three arrays into the ink_edge_update layout."""
    u = np.zeros(len(op), dtype=EDGE_UPDATE_DTYPE)
    u["op"], u["src"], u["dst"] = op, src, dst
    return u


class Ink:
    """One context.  `model` is the dict layout of synth.make_model (host numpy weights)."""

    def __init__(self, rowptr, col, features, model, slack_factor=0.25, profile=False, stream=None,
                 dense_threshold=0.0, pool_reserve=0, batch_device=False, node_capacity=0, small_batch_limit=0,
                 max_batch=0):
        self._lib = load_library()
        self._h = C.c_void_p()
        rowptr = np.ascontiguousarray(rowptr, np.int64)
        col = np.ascontiguousarray(col, np.int32)
        features = np.ascontiguousarray(features, np.float32)
        keep = [rowptr, col, features]
        layers = (_Layer * len(model["layers"]))()
        for i, L in enumerate(model["layers"]):
            def w(name):
                a = L.get(name)
                if a is None:
                    return None
                a = np.ascontiguousarray(a, np.float32)
                keep.append(a)
                return C.c_void_p(a.ctypes.data)
            layers[i] = _Layer(L["in_dim"], L["out_dim"], int(L.get("mlp_hidden", 0) or 0), w("W_neigh"),
                               w("W_self"), w("bias"), w("W_mlp2"), w("bias_mlp2"),
                               1 if L.get("act", "none") == "relu" else 0)
        m = _Model(MODEL_KINDS[model["kind"]], AGGS[model["agg"]], float(model.get("gin_eps", 0.0)),
                   len(model["layers"]), layers)
        g = _Csr(rowptr.size - 1, col.size, rowptr.ctypes.data, col.ctypes.data if col.size else None)
        o = _Options(0, stream, slack_factor, int(max_batch), int(bool(profile)), dense_threshold,
                     1 if batch_device else 0, small_batch_limit, pool_reserve, node_capacity)
        st = self._lib.ink_create(C.byref(g), features.ctypes.data, features.shape[1], C.byref(m), C.byref(o),
                                  C.byref(self._h))
        if st != 0:
            raise InkError(st, self._lib.ink_last_error(None).decode())
        self.n = rowptr.size - 1
        self.feat_dim = int(features.shape[1])
        self.n_layers = len(model["layers"])
        self.out_dim = model["layers"][-1]["out_dim"]
        self.batch_device = batch_device
        # width of the aggregated rows of each layer (what the aggregation kernels move)
        if model["kind"] == "gcn":
            self.agg_widths = [L["out_dim"] for L in model["layers"]]
        else:
            self.agg_widths = [L["in_dim"] for L in model["layers"]]

    def _check(self, st):
        if st != 0:
            raise InkError(st, self._lib.ink_last_error(self._h).decode())

    def full_infer(self):
        self._check(self._lib.ink_full_infer(self._h))

    def full_infer_noalloc(self):
        self._check(self._lib.ink_full_infer_noalloc(self._h))

    def apply_updates(self, updates, fetch=True, affected=False):
        """updates: structured array (EDGE_UPDATE_DTYPE).  Returns dict; with fetch the changed ids
        and embeddings are copied to host numpy arrays.  affected: run the affected-area baseline."""
        assert not self.batch_device, "context expects device batches"
        updates = np.ascontiguousarray(updates, dtype=EDGE_UPDATE_DTYPE)
        r = _Result()
        fn = self._lib.ink_apply_updates_affected if affected else self._lib.ink_apply_updates
        self._check(fn(self._h, updates.ctypes.data if updates.size else None, updates.size, C.byref(r)))
        out = dict(n_changed=r.n_changed, n_applied_ins=r.n_applied_ins, n_applied_del=r.n_applied_del,
                   n_noop=r.n_noop, changed_ids_ptr=r.changed_ids, embeddings_ptr=r.embeddings)
        if fetch:
            ids = np.empty(r.n_changed, np.int32)
            emb = np.empty((r.n_changed, self.out_dim), np.float32)
            if r.n_changed:
                _dtoh(ids, r.changed_ids)
                _dtoh(emb, r.embeddings)
            out["changed_ids"], out["embeddings"] = ids, emb
        return out

    def apply_updates_device(self, dev_ptr, n, affected=False):
        """Batch already in device memory (context created with batch_device=True); results stay on the device."""
        assert self.batch_device
        r = _Result()
        fn = self._lib.ink_apply_updates_affected if affected else self._lib.ink_apply_updates
        self._check(fn(self._h, C.c_void_p(dev_ptr), n, C.byref(r)))
        return dict(n_changed=r.n_changed, n_applied_ins=r.n_applied_ins, n_applied_del=r.n_applied_del,
                    n_noop=r.n_noop, changed_ids_ptr=r.changed_ids, embeddings_ptr=r.embeddings)

    def update_features(self, node_ids, rows, fetch=True):
        """x_v <- rows[i] for v = node_ids[i] (distinct ids), then incremental propagation.
        Host arrays; same result dict as apply_updates."""
        assert not self.batch_device, "context expects device batches"
        node_ids = np.ascontiguousarray(node_ids, dtype=np.int32)
        rows = np.ascontiguousarray(rows, dtype=np.float32)
        if node_ids.size:
            rows = rows.reshape(node_ids.size, -1)
            assert rows.shape[1] == self.feat_dim, "rows must be [n][feat_dim]"
        r = _Result()
        self._check(self._lib.ink_update_features(self._h, node_ids.ctypes.data if node_ids.size else None,
                                                  rows.ctypes.data if node_ids.size else None, node_ids.size,
                                                  C.byref(r)))
        out = dict(n_changed=r.n_changed, n_applied_ins=r.n_applied_ins, n_applied_del=r.n_applied_del,
                   n_noop=r.n_noop, changed_ids_ptr=r.changed_ids, embeddings_ptr=r.embeddings)
        if fetch:
            ids = np.empty(r.n_changed, np.int32)
            emb = np.empty((r.n_changed, self.out_dim), np.float32)
            if r.n_changed:
                _dtoh(ids, r.changed_ids)
                _dtoh(emb, r.embeddings)
            out["changed_ids"], out["embeddings"] = ids, emb
        return out

    def apply_user_events(self, events, rows, fetch=True):
        """events: list of (layer, target, op) or a USER_EVENT_DTYPE array; rows: [n][stride] float32
        (row i belongs to event i).  Host arrays; same result dict as apply_updates."""
        if not isinstance(events, np.ndarray) or events.dtype != USER_EVENT_DTYPE:
            ev = np.zeros(len(events), dtype=USER_EVENT_DTYPE)
            for i, (layer, target, op) in enumerate(events):
                ev[i] = (layer, target, op, 0)
            events = ev
        events = np.ascontiguousarray(events)
        rows = np.ascontiguousarray(rows, dtype=np.float32).reshape(events.size, -1) if events.size else np.zeros((0, 1), np.float32)
        r = _Result()
        self._check(self._lib.ink_apply_user_events(self._h, events.ctypes.data if events.size else None,
                                                    rows.ctypes.data if events.size else None, rows.shape[1],
                                                    events.size, C.byref(r)))
        out = dict(n_changed=r.n_changed, n_applied_ins=r.n_applied_ins, n_applied_del=r.n_applied_del,
                   n_noop=r.n_noop, changed_ids_ptr=r.changed_ids, embeddings_ptr=r.embeddings)
        if fetch:
            ids = np.empty(r.n_changed, np.int32)
            emb = np.empty((r.n_changed, self.out_dim), np.float32)
            if r.n_changed:
                _dtoh(ids, r.changed_ids)
                _dtoh(emb, r.embeddings)
            out["changed_ids"], out["embeddings"] = ids, emb
        return out

    def add_nodes(self, features, fetch=True):
        """Appends len(features) nodes without edges; returns their ids and final embeddings."""
        assert not self.batch_device, "context expects device batches"
        features = np.ascontiguousarray(features, dtype=np.float32).reshape(-1, self.feat_dim)
        r = _Result()
        self._check(self._lib.ink_add_nodes(self._h, features.ctypes.data if features.size else None,
                                            features.shape[0], C.byref(r)))
        self.n += features.shape[0]
        out = dict(n_changed=r.n_changed, changed_ids_ptr=r.changed_ids, embeddings_ptr=r.embeddings)
        if fetch:
            ids = np.empty(r.n_changed, np.int32)
            emb = np.empty((r.n_changed, self.out_dim), np.float32)
            if r.n_changed:
                _dtoh(ids, r.changed_ids)
                _dtoh(emb, r.embeddings)
            out["changed_ids"], out["embeddings"] = ids, emb
        return out

    def update_features_device(self, ids_ptr, rows_ptr, n):
        """Ids and rows already in device memory (context created with batch_device=True)."""
        assert self.batch_device
        r = _Result()
        self._check(self._lib.ink_update_features(self._h, C.c_void_p(ids_ptr), C.c_void_p(rows_ptr), n, C.byref(r)))
        return dict(n_changed=r.n_changed, n_applied_ins=r.n_applied_ins, n_applied_del=r.n_applied_del,
                    n_noop=r.n_noop, changed_ids_ptr=r.changed_ids, embeddings_ptr=r.embeddings)

    def get_layer(self, layer, which, row0=0, nrows=None):
        nrows = self.n - row0 if nrows is None else nrows
        w = C.c_int32()
        self._check(self._lib.ink_get_layer(self._h, layer, which, 0, 0, None, 0, C.byref(w)))
        out = np.empty((nrows, w.value), np.int32 if which in (2, 4) else np.float32)   # 5: user term, float
        self._check(self._lib.ink_get_layer(self._h, layer, which, row0, nrows, out.ctypes.data, 0, None))
        return out

    def get_graph(self):
        rowptr = np.empty(self.n + 1, np.int64)
        self._check(self._lib.ink_get_graph(self._h, rowptr.ctypes.data, None))
        col = np.empty(int(rowptr[-1]), np.int32)
        self._check(self._lib.ink_get_graph(self._h, rowptr.ctypes.data, col.ctypes.data if col.size else None))
        return rowptr, col

    def set_profiling(self, on):
        self._check(self._lib.ink_set_profiling(self._h, int(bool(on))))

    def stats(self):
        s = _Stats()
        self._check(self._lib.ink_get_stats(self._h, C.byref(s), C.sizeof(s)))
        layers = [{k: getattr(s.layer[i], k) for k, _ in _LayerStats._fields_ if k not in ("pad_", "ms_kernel")}
                  for i in range(s.n_layers)]
        for i, L in enumerate(layers):
            L["ms_kernel"] = {name: s.layer[i].ms_kernel[j] for j, name in enumerate(KERNEL_SLOTS)}
        return dict(layers=layers, ms={TIME_CLASSES[i]: s.ms[i] for i in range(INK_T_NCLASS)},
                    launches={TIME_CLASSES[i]: s.launches[i] for i in range(INK_T_NCLASS)},
                    ms_total=s.ms_total)

    def close(self):
        if self._h:
            self._lib.ink_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def _dtoh(dst, dev_ptr):
    """Device -> host copy through torch (PyTorch is the memory/stream plumbing)."""
    import torch
    n = dst.nbytes
    t = torch.empty(n, dtype=torch.uint8, device="cuda")
    _hip().hipMemcpy(C.c_void_p(t.data_ptr()), C.c_void_p(dev_ptr), C.c_size_t(n), 3)
    dst.view(np.uint8).reshape(-1)[:] = t.cpu().numpy()


_hiprt = None


def _hip():
    global _hiprt
    if _hiprt is None:
        _hiprt = C.CDLL("libamdhip64.so")
    return _hiprt
