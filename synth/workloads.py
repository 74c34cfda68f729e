"""The five benchmark workloads: graph, features, model weights and update batches.

Every array is drawn from numpy's PCG64 with a seed derived from the config number, so the
CPU oracle and the HIP library are always handed identical inputs.  `scale_div` shrinks a
config (nodes, edges and batch size divided by it) into a replica the oracle finishes in
seconds; widths and model structure are unchanged.
"""
from dataclasses import dataclass, replace
import numpy as np

from .rmat import rmat_edges, edge_keys


@dataclass(frozen=True)
class WorkloadConfig:
    cfg_id: int
    name: str
    model: str              # "sage" | "gcn" | "gin"
    agg: str                # "max" | "gcn_sym" | "sum"
    n_nodes: int
    n_edges: int            # unique directed edges drawn (before symmetrisation)
    symmetrise: bool
    dims: tuple             # (feature width, layer-1 out, ..., layer-k out)
    mlp_hidden: int         # GIN only
    batch: int
    hub_biased_deletes: bool
    rmat: tuple = (0.57, 0.19, 0.19)
    graph_seed: int = 0     # 0: 1000 + cfg_id

    @property
    def n_layers(self):
        return len(self.dims) - 1

    def scaled(self, scale_div):
        if scale_div == 1:
            return self
        return replace(self, name=f"{self.name}/div{scale_div}",
                       n_nodes=max(64, self.n_nodes // scale_div),
                       n_edges=max(256, self.n_edges // scale_div),
                       batch=max(2, self.batch // scale_div))


CONFIGS = {
    1: WorkloadConfig(1, "cfg1-sage-max-10k", "sage", "max", 10_000, 100_000, True,
                      (64, 64, 64), 0, 100, False),
    2: WorkloadConfig(2, "cfg2-gcn-sym-233k", "gcn", "gcn_sym", 233_000, 114_000_000, False,
                      (602, 256, 41), 0, 1_000, False),
    3: WorkloadConfig(3, "cfg3-sage-max-2.45M", "sage", "max", 2_450_000, 62_000_000, False,
                      (100, 256, 47), 0, 10_000, True),
    4: WorkloadConfig(4, "cfg4-gin-sum-20M", "gin", "sum", 20_000_000, 400_000_000, False,
                      (128, 128, 128, 172), 128, 10_000, False),
    5: WorkloadConfig(5, "cfg5-sage-max-20M", "sage", "max", 20_000_000, 400_000_000, False,
                      (128, 128, 128, 128), 0, 10_000, False, graph_seed=1004),   # the graph of config 4
}


def get_config(cfg_id, scale_div=1):
    return CONFIGS[cfg_id].scaled(scale_div)


def make_graph(cfg):
    """(src, dst) int32, unique, no self loops, sorted by (dst, src).  Seed 1000 + cfg (config 5 reuses
    the graph of config 4, as its description says)."""
    a, b, c = cfg.rmat
    return rmat_edges(cfg.n_nodes, cfg.n_edges, a, b, c, seed=cfg.graph_seed or 1000 + cfg.cfg_id,
                      symmetrise=cfg.symmetrise)


def make_features(cfg):
    """N x d_0 float32 drawn from N(0, 1).  Seed 2000 + cfg."""
    rng = np.random.Generator(np.random.PCG64(2000 + cfg.cfg_id))
    return rng.standard_normal((cfg.n_nodes, cfg.dims[0]), dtype=np.float32)


def xavier_uniform(rng, fan_in, fan_out):
    """[fan_in][fan_out] float32, uniform in +-sqrt(6 / (fan_in + fan_out))."""
    lim = np.sqrt(6.0 / (fan_in + fan_out))
    return rng.uniform(-lim, lim, size=(fan_in, fan_out)).astype(np.float32)


def make_model(cfg, bias_scale=0.0):
    """Model description as plain dict: kind, agg, eps and per-layer weights (row-major [in][out]).

    ReLU follows every layer but the last.  GraphSAGE has no bias; GCN and GIN biases are
    present and zero unless `bias_scale` is set (tests use a non-zero scale so that a dropped
    bias term is visible).  Seed 3000 + cfg.
    """
    rng = np.random.Generator(np.random.PCG64(3000 + cfg.cfg_id))
    layers = []
    k = cfg.n_layers
    for l in range(k):
        din, dout = cfg.dims[l], cfg.dims[l + 1]
        act = "relu" if l < k - 1 else "none"
        def bias(n):
            return (bias_scale * rng.standard_normal(n)).astype(np.float32)
        if cfg.model == "sage":
            layers.append(dict(in_dim=din, out_dim=dout, act=act,
                               W_neigh=xavier_uniform(rng, din, dout),
                               W_self=xavier_uniform(rng, din, dout), bias=None))
        elif cfg.model == "gcn":
            layers.append(dict(in_dim=din, out_dim=dout, act=act,
                               W_neigh=xavier_uniform(rng, din, dout), bias=bias(dout)))
        elif cfg.model == "gin":
            hid = cfg.mlp_hidden
            layers.append(dict(in_dim=din, out_dim=dout, act=act, mlp_hidden=hid,
                               W_neigh=xavier_uniform(rng, din, hid), bias=bias(hid),
                               W_mlp2=xavier_uniform(rng, hid, dout), bias_mlp2=bias(dout)))
        else:
            raise ValueError(cfg.model)
    return dict(kind=cfg.model, agg=cfg.agg, gin_eps=0.0, layers=layers)


class BatchSampler:
    """Draws update batches against the evolving edge set (seed 4000 + cfg, + batch index).

    A batch of B updates holds B // 2 deletions of existing edges and B - B // 2 insertions
    of absent, non-self-loop pairs; the two halves are then interleaved by a seeded shuffle.
    With `hub_biased_deletes`, 80 % of the deletions are uniform over edges whose destination
    is among the top 1 % of nodes by initial in-degree (ties to the lower id) and 20 % uniform
    over all edges.  The sampler tracks the edge set it has produced so that successive batches
    stay valid; it does no inference arithmetic.
    """

    OP_INSERT, OP_DELETE = 0, 1

    def __init__(self, cfg, src, dst):
        self.cfg = cfg
        self.n = cfg.n_nodes
        self.base = edge_keys(src, dst)              # sorted (dst-major) unique keys
        self.alive = np.ones(self.base.size, dtype=bool)
        self.extra = set()                           # inserted keys not in base (or re-inserted)
        self.batch_idx = 0
        if cfg.hub_biased_deletes:
            indeg = np.bincount(dst, minlength=self.n)
            n_hub = max(1, self.n // 100)
            order = np.lexsort((np.arange(self.n), -indeg))
            hub = np.zeros(self.n, dtype=bool)
            hub[order[:n_hub]] = True
            self.hub_edge_idx = np.nonzero(hub[dst])[0]
        else:
            self.hub_edge_idx = None

    def _present(self, key):
        if key in self.extra:
            return True
        i = np.searchsorted(self.base, key)
        return i < self.base.size and self.base[i] == key and self.alive[i]

    def next_batch(self, batch=None):
        B = self.cfg.batch if batch is None else batch
        rng = np.random.Generator(np.random.PCG64([4000 + self.cfg.cfg_id, self.batch_idx]))
        self.batch_idx += 1
        n_del = B // 2
        n_ins = B - n_del
        del_keys = []
        chosen = set()
        tries = 0
        while len(del_keys) < n_del and tries < 100 * (n_del + 1):
            tries += 1
            if self.hub_edge_idx is not None and rng.random() < 0.8 and self.hub_edge_idx.size:
                i = int(self.hub_edge_idx[rng.integers(self.hub_edge_idx.size)])
            else:
                i = int(rng.integers(self.base.size))
            if not self.alive[i] or i in chosen:
                continue
            chosen.add(i)
            del_keys.append(int(self.base[i]))
        ins_keys = []
        ins_set = set()
        while len(ins_keys) < n_ins:
            s = int(rng.integers(self.n))
            d = int(rng.integers(self.n))
            key = (d << 32) | s
            if s == d or key in ins_set or self._present(key):
                continue
            ins_set.add(key)
            ins_keys.append(key)
        for i in chosen:
            self.alive[i] = False
        for key in ins_keys:
            i = np.searchsorted(self.base, key)
            if i < self.base.size and self.base[i] == key:
                self.alive[i] = True
            else:
                self.extra.add(key)
        keys = np.array(del_keys + ins_keys, dtype=np.int64)
        op = np.array([self.OP_DELETE] * len(del_keys) + [self.OP_INSERT] * len(ins_keys),
                      dtype=np.uint8)
        perm = rng.permutation(keys.size)
        keys, op = keys[perm], op[perm]
        return op, (keys & 0xFFFFFFFF).astype(np.int32), (keys >> 32).astype(np.int32)

    def current_edges(self):
        """(src, dst) of the edge set after all batches drawn so far, sorted by (dst, src)."""
        keys = self.base[self.alive]
        if self.extra:
            keys = np.union1d(keys, np.fromiter(self.extra, dtype=np.int64, count=len(self.extra)))
        return (keys & 0xFFFFFFFF).astype(np.int32), (keys >> 32).astype(np.int32)
