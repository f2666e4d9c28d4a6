"""Tile plan oracle (test infrastructure only).

Section 3.1: a matrix is partitioned logically into T x T tiles; tiles on the
right and bottom edge are smaller when T does not divide the size.  An output
tile C_ij is one task; the number of k values is the number of steps needed
to finish it.  Algorithm 1 decodes a task id into (i, j); the encoding taken
here is row-major, id = i * nJ + j.
"""


def _ceil_div(a, b):
    return -(-a // b)


def tile_counts(n, t):
    """(full T x T tiles, remaining edge tiles) of an n x n matrix, as section 3.1 counts them."""
    full = (n // t) ** 2
    return full, _ceil_div(n, t) ** 2 - full


def decode_task(task_id, n_j):
    return task_id // n_j, task_id % n_j


def kstep_ranges(K, T):
    return [(k * T, min(K, (k + 1) * T)) for k in range(_ceil_div(K, T))]


def plan_tiles(M, N, K, T):
    """List of tasks: dicts with id, i, j, row range, column range, number of k-steps."""
    if min(M, N, K) < 0 or T <= 0:
        raise ValueError("bad sizes")
    n_i, n_j, n_k = _ceil_div(M, T), _ceil_div(N, T), _ceil_div(K, T)
    tasks = []
    for i in range(n_i):
        for j in range(n_j):
            tasks.append(dict(id=i * n_j + j, i=i, j=j,
                              r0=i * T, r1=min(M, (i + 1) * T),
                              c0=j * T, c1=min(N, (j + 1) * T),
                              n_k=n_k))
    return tasks
