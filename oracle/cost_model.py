"""Closed-form operation and IO counts the paper states.  Test infrastructure only."""


def gat_score_ops_original(num_v, num_e, f):
    """u_concat_v (2|E|f) + LP (4|E|f) + LeakyReLU (|E|): Sec. 4, example after Eq. 1."""
    return 2 * num_e * f + 4 * num_e * f + num_e


def gat_score_ops_reorganized(num_v, num_e, f):
    """Two vertex-side projections (4|V|f), then add + LeakyReLU per edge (2|E|): Sec. 4."""
    return 4 * num_v * f + 2 * num_e


def gat_graph_io_unfused(num_v, num_e, h, f):
    """Scatter 4|E|h + ReduceScatter 3|E|h + Aggregate 3|E|hf + |V|hf elements: Sec. 5 example."""
    return 4 * num_e * h + 3 * num_e * h + 3 * num_e * h * f + num_v * h * f


def gat_graph_io_fused(num_v, num_e, h, f):
    """|V|hf + 5|E|h + 2|E|hf elements once intermediates are reused: Sec. 5 example."""
    return num_v * h * f + 5 * num_e * h + 2 * num_e * h * f


def count_gat_score_ops_by_walking(indptr, f, reorganized):
    """Count the same quantities by walking the dataflow edge by edge / vertex by
    vertex (one multiply or add = one op), to pin the closed forms above."""
    n = len(indptr) - 1
    e = int(indptr[-1])
    ops = 0
    if not reorganized:
        for _ in range(e):
            ops += 2 * f              # copy 2f values into the concatenated vector
            ops += 2 * (2 * f)        # dot product of length 2f: 2f multiplies + 2f adds
            ops += 1                  # LeakyReLU
    else:
        for _ in range(n):
            ops += 2 * (2 * f)        # two dot products of length f
        for _ in range(e):
            ops += 1 + 1              # add, LeakyReLU
    return ops
