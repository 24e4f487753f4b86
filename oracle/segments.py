"""Per-destination reductions (the Gather operator, App. A.1) over edge tensors
laid out in CSR-by-destination order.  Test infrastructure only."""
import numpy as np


def edge_dst(indptr):
    """Destination vertex of every CSR position."""
    n = indptr.shape[0] - 1
    return np.repeat(np.arange(n, dtype=np.int64), np.diff(indptr))


def _starts(indptr):
    counts = np.diff(indptr)
    nz = counts > 0
    return nz, np.asarray(indptr[:-1], dtype=np.int64)[nz]


def segment_sum(indptr, edge_vals):
    """out[v] = sum of edge_vals over the in-edges of v; 0 for an empty row."""
    n = indptr.shape[0] - 1
    out = np.zeros((n,) + edge_vals.shape[1:], dtype=edge_vals.dtype)
    nz, starts = _starts(indptr)
    if starts.size:
        out[nz] = np.add.reduceat(edge_vals, starts, axis=0)
    return out


def segment_max(indptr, edge_vals, empty=0.0):
    """out[v] = max of edge_vals over the in-edges of v; `empty` for an empty row."""
    n = indptr.shape[0] - 1
    out = np.full((n,) + edge_vals.shape[1:], empty, dtype=edge_vals.dtype)
    nz, starts = _starts(indptr)
    if starts.size:
        out[nz] = np.maximum.reduceat(edge_vals, starts, axis=0)
    return out


def restrict_rows(indptr, indices, rows):
    """The same vertex set with only the in-edges of `rows` kept (other rows
    become empty).  Returns (indptr, indices, kept CSR positions)."""
    n = indptr.shape[0] - 1
    keep_row = np.zeros(n, dtype=bool)
    keep_row[np.asarray(rows, dtype=np.int64)] = True
    counts = np.where(keep_row, np.diff(indptr), 0)
    new_indptr = np.zeros(n + 1, dtype=np.int64)
    np.cumsum(counts, out=new_indptr[1:])
    pos = np.flatnonzero(np.repeat(keep_row, np.diff(indptr)))
    return new_indptr, np.asarray(indices)[pos], pos
