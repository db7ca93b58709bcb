"""Reference neighbour sampler for sampling inference (Section 2: each node aggregates a sampled subset of its
in-neighbours; fan-out 10 in the paper's experiments).  TEST INFRASTRUCTURE ONLY, like the rest of oracle/.

Definition (this build's reading; the paper only names the fan-out):
  * every layer draws its own sample; a row with at most `fanout` in-edges keeps all of them;
  * otherwise it keeps the `fanout` edges with the smallest keys, a uniform sample without replacement, in
    their stored order;
  * the key of the edge stored at position e of `indices` (0 <= e < E) in layer l is the upper 32 bits of output
    number l*E + e + 1 of the SplitMix64 generator (Steele, Lea, Flood 2014) seeded with `seed`; equal keys are
    ordered by position in the row.
Plain numpy, no blocking: keys for all edges, one sort by (row, key, position), ranks within rows.
"""
import numpy as np

GOLDEN = np.uint64(0x9E3779B97F4A7C15)
M1 = np.uint64(0xBF58476D1CE4E5B9)
M2 = np.uint64(0x94D049BB133111EB)


def splitmix64_output(seed, k):
    """Output number k (k = 1, 2, ...) of SplitMix64 started from state `seed`; k may be an array."""
    with np.errstate(over="ignore"):
        z = np.uint64(seed) + GOLDEN * np.asarray(k, dtype=np.uint64)
        z = (z ^ (z >> np.uint64(30))) * M1
        z = (z ^ (z >> np.uint64(27))) * M2
        return z ^ (z >> np.uint64(31))


def sample_csr(indptr, indices, fanout, seed, layer, edge_base=0, total_edges=None):
    """The sampled graph of one layer: (indptr int64, indices int32).  For a slice of consecutive rows of a larger
    graph (indptr rebased to 0, its share of indices), pass the position of the slice's first edge in the full
    `indices` array as `edge_base` and the full edge count as `total_edges`: keys belong to positions in the full
    graph."""
    indptr = np.asarray(indptr, dtype=np.int64)
    indices = np.asarray(indices, dtype=np.int32)
    n, E = indptr.size - 1, indices.size
    deg = np.diff(indptr)
    row = np.repeat(np.arange(n, dtype=np.int64), deg)
    pos = np.arange(E, dtype=np.int64) - indptr[row]
    E_full = E if total_edges is None else int(total_edges)
    with np.errstate(over="ignore"):
        k = np.uint64(layer) * np.uint64(E_full) + np.uint64(edge_base) + np.arange(E, dtype=np.uint64) + np.uint64(1)
    keys = (splitmix64_output(seed, k) >> np.uint64(32)).astype(np.uint32)
    order = np.lexsort((pos, keys, row))            # by row, then key, then position in the row
    rank = np.arange(E, dtype=np.int64) - indptr[row[order]]
    keep = np.zeros(E, dtype=bool)
    keep[order[rank < fanout]] = True
    new_indptr = np.zeros(n + 1, dtype=np.int64)
    np.cumsum(np.minimum(deg, fanout), out=new_indptr[1:])
    return new_indptr, indices[keep]
