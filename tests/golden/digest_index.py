"""Which entries of a gradient tensor a full-size digest keeps.  Index arithmetic only: used by
make_digests.py (which writes the expected values from the CPU oracle) and by the GPU tests (which
read the same entries of the HIP path's gradients).

Per tensor with more than SMALL elements:
  * a seeded random sample of SAMPLE entries;
  * structured pieces, chosen so that a mistake confined to one tile, one boundary row or the ragged
    tail of a tensor cannot hide between the random entries:
      - the first and the last row,
      - the last 8 rows (the last 8-entry group of a vocabulary-sized tensor),
      - the rows on both sides of the first few and of the last multiple of 256 and of 1024
        (tile and slab boundaries of the kernels that write these tensors),
      - one full 256 x 256 block that straddles tile boundaries in both directions.
Smaller tensors are kept whole."""
import numpy as np

SAMPLE, SMALL = 4096, 65536


def sample_index(name, n):
    if n <= SMALL:
        return np.arange(n)
    seed = int.from_bytes(name.encode(), "little") % (2 ** 31)
    return np.sort(np.random.default_rng(seed).choice(n, size=SAMPLE, replace=False))


def boundary_rows(R):
    rows = {0, R - 1}
    rows.update(range(max(0, R - 8), R))
    for step in (256, 1024):
        mult = [m for m in (step, 2 * step, 3 * step, (R - 1) // step * step) if 0 < m < R]
        for m in mult:
            rows.update((m - 1, m))
    return np.array(sorted(rows), np.int64)


def block_origin(R, C):
    """Top-left corner and size of the kept block: starts 128 entries before the last multiple of 256
    in each direction (so it covers parts of four 256 x 256 tiles and of more 128 x 128 ones)."""
    def one(n):
        size = min(256, n)
        if n <= 256:
            return 0, size
        o = (n - 1) // 256 * 256 - 128
        return max(0, min(o, n - size)), size
    r0, nr = one(R)
    c0, nc = one(C)
    return r0, nr, c0, nc


def pieces(shape):
    """name -> (row index array or slice, column slice) for a large 2-D tensor; {} otherwise."""
    if len(shape) != 2 or shape[0] * shape[1] <= SMALL:
        return {}
    R, C = shape
    r0, nr, c0, nc = block_origin(R, C)
    return {"rows": (boundary_rows(R), slice(0, C)), "block": (slice(r0, r0 + nr), slice(c0, c0 + nc))}


def take(arr, shape, piece):
    rows, cols = piece
    return np.asarray(arr).reshape(shape)[rows, cols]
