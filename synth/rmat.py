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


def _draw(rng, n, scale, a, b, c):
    """Draw n (src, dst) pairs in [0, 2**scale)^2, one quadrant choice per bit level."""
    src = np.zeros(n, dtype=np.int64)
    dst = np.zeros(n, dtype=np.int64)
    ab, abc = a + b, a + b + c
    for _ in range(scale):
        u = rng.random(n, dtype=np.float32)
        sbit = u >= ab                      # quadrants c, d: source bit set
        dbit = ((u >= a) & (u < ab)) | (u >= abc)   # quadrants b, d: destination bit set
        src = (src << 1) | sbit
        dst = (dst << 1) | dbit
    return src, dst


def rmat_edges(n_nodes, n_edges, a=0.57, b=0.19, c=0.19, seed=0, symmetrise=False,
               permute=True, chunk=1 << 24):
    """Unique directed edges without self loops, as (src, dst) int32 arrays sorted by (dst, src).

    Samples with an endpoint >= n_nodes are rejected; drawing continues until `n_edges`
    distinct pairs exist (first occurrences in draw order are kept).  With `symmetrise`
    the reverse of every edge is added afterwards and duplicates dropped, so the count is
    then about 2x n_edges.  A seeded random relabelling spreads the hubs over the id range.
    """
    rng = np.random.Generator(np.random.PCG64(seed))
    scale = max(1, int(np.ceil(np.log2(max(n_nodes, 2)))))
    have = np.empty(0, dtype=np.int64)      # unique keys, in first-occurrence order
    guard = 0
    while have.size < n_edges:
        need = n_edges - have.size
        n_draw = int(min(max(need * 1.3 + 1024, 4096), 4 * chunk))
        parts = []
        for s0 in range(0, n_draw, chunk):
            s, d = _draw(rng, min(chunk, n_draw - s0), scale, a, b, c)
            ok = (s < n_nodes) & (d < n_nodes) & (s != d)
            parts.append((d[ok] << 32) | s[ok])
        cand = np.concatenate([have] + parts)
        _, first = np.unique(cand, return_index=True)
        first.sort()
        have = cand[first]
        guard += 1
        if guard > 10000:
            raise RuntimeError("R-MAT: cannot reach the requested unique edge count")
    have = have[:n_edges]
    src = (have & 0xFFFFFFFF)
    dst = (have >> 32)
    if permute:
        perm = rng.permutation(n_nodes).astype(np.int64)
        src, dst = perm[src], perm[dst]
    if symmetrise:
        src, dst = np.concatenate([src, dst]), np.concatenate([dst, src])
    keys = np.unique((dst << 32) | src)
    return (keys & 0xFFFFFFFF).astype(np.int32), (keys >> 32).astype(np.int32)


def in_csr_from_edges(n_nodes, src, dst):
    """In-neighbour CSR: row v lists the sources u of edges u -> v in ascending order."""
    keys = np.unique(edge_keys(np.asarray(src), np.asarray(dst)))
    s, d = keys_to_edges(keys)
    rowptr = np.zeros(n_nodes + 1, dtype=np.int64)
    np.cumsum(np.bincount(d, minlength=n_nodes), out=rowptr[1:])
    return rowptr, s.astype(np.int32)
