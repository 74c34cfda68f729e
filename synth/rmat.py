"""R-MAT edge generator (recursive-matrix model with quadrant probabilities a, b, c, d).

Stands in for the paper's social-network datasets (Table "Datasets", Sec. 4.1): the
synthetic graphs take their node counts, feature widths and heavy-tailed degree
distribution, not their records.
"""
import numpy as np


def edge_keys(src, dst):
    """Pack directed edges (src -> dst) into sortable int64 keys, destination-major."""
    return (dst.astype(np.int64) << 32) | src.astype(np.int64)


def keys_to_edges(keys):
    return (keys & 0xFFFFFFFF).astype(np.int32), (keys >> 32).astype(np.int32)


def _draw(seed_seq, n, scale, a, b, c, n_nodes):
    """Draw n (src, dst) pairs in [0, 2**scale)^2, one quadrant choice per bit level; returns the
    int64 keys (dst << 32 | src) of the pairs that are in range and not self loops."""
    rng = np.random.Generator(np.random.PCG64(seed_seq))
    src = np.zeros(n, dtype=np.int32)
    dst = np.zeros(n, dtype=np.int32)
    # 16-bit thresholds: quadrant probabilities are honoured to within 2**-16
    t_a, t_ab, t_abc = (int(round(x * 65536)) for x in (a, a + b, a + b + c))
    for _ in range(scale):
        u = rng.integers(0, 65536, size=n, dtype=np.uint16)
        sbit = u >= t_ab                              # quadrants c, d: source bit set
        dbit = ((u >= t_a) & (u < t_ab)) | (u >= t_abc)   # quadrants b, d: destination bit set
        src <<= 1
        src |= sbit
        dst <<= 1
        dst |= dbit
    ok = (src < n_nodes) & (dst < n_nodes) & (src != dst)
    return (dst[ok].astype(np.int64) << 32) | src[ok].astype(np.int64)


def rmat_edges(n_nodes, n_edges, a=0.57, b=0.19, c=0.19, seed=0, symmetrise=False,
               permute=True, chunk=1 << 22, workers=8):
    """Unique directed edges without self loops, as (src, dst) int32 arrays sorted by (dst, src).

    Samples with an endpoint >= n_nodes are rejected; drawing continues in rounds until at least
    `n_edges` distinct pairs exist, then a seeded random subset of exactly `n_edges` is kept.
    With `symmetrise` the reverse of every edge is added afterwards and duplicates dropped, so the
    count is then about 2x n_edges.  A seeded random relabelling spreads the hubs over the id
    range.  Chunks of one round are drawn by worker threads, each from its own child stream of
    the seed, so the result does not depend on the number of workers.
    """
    from concurrent.futures import ThreadPoolExecutor
    root = np.random.SeedSequence(seed)
    rng = np.random.Generator(np.random.PCG64(root.spawn(1)[0]))
    scale = max(1, int(np.ceil(np.log2(max(n_nodes, 2)))))
    have = np.empty(0, dtype=np.int64)
    rounds = 0
    with ThreadPoolExecutor(max_workers=workers) as ex:
        while have.size < n_edges:
            need = n_edges - have.size
            n_draw = int(max(need * 1.25 + 1024, 4096))
            sizes = [min(chunk, n_draw - s0) for s0 in range(0, n_draw, chunk)]
            seeds = root.spawn(len(sizes))
            parts = list(ex.map(lambda t: _draw(t[0], t[1], scale, a, b, c, n_nodes), zip(seeds, sizes)))
            have = np.unique(np.concatenate([have] + parts))
            rounds += 1
            if rounds > 1000:
                raise RuntimeError("R-MAT: cannot reach the requested unique edge count")
    if have.size > n_edges:
        drop = rng.permutation(have.size)[:have.size - n_edges]
        keep = np.ones(have.size, dtype=bool)
        keep[drop] = False
        have = have[keep]
    src = (have & 0xFFFFFFFF)
    dst = (have >> 32)
    if permute:
        perm = rng.permutation(n_nodes).astype(np.int64)
        src, dst = perm[src], perm[dst]
    if symmetrise:
        src, dst = np.concatenate([src, dst]), np.concatenate([dst, src])
    keys = (dst << 32) | src
    keys.sort()
    if symmetrise:
        keys = np.unique(keys)
    return (keys & 0xFFFFFFFF).astype(np.int32), (keys >> 32).astype(np.int32)


def in_csr_from_edges(n_nodes, src, dst, assume_sorted=False):
    """In-neighbour CSR: row v lists the sources u of edges u -> v in ascending order.
    assume_sorted: the edges are already unique and ordered by (dst, src), as rmat_edges returns."""
    if assume_sorted:
        rowptr = np.zeros(n_nodes + 1, dtype=np.int64)
        np.cumsum(np.bincount(dst, minlength=n_nodes), out=rowptr[1:])
        return rowptr, np.ascontiguousarray(src, dtype=np.int32)
    keys = np.unique(edge_keys(np.asarray(src), np.asarray(dst)))
    s, d = keys_to_edges(keys)
    rowptr = np.zeros(n_nodes + 1, dtype=np.int64)
    np.cumsum(np.bincount(d, minlength=n_nodes), out=rowptr[1:])
    return rowptr, s.astype(np.int32)
