"""Shared test helpers: the reader for the small text fixtures under golden/
(`key: v v v` lines and `key:` followed by matrix rows; `#` starts a comment)
and hand-built CSR patterns for edge cases."""
import os

import numpy as np

HERE = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def load_golden(name):
    out, key, rows = {}, None, []

    def flush():
        if key is not None and rows:
            out[key] = np.array(rows, dtype=np.float64)

    with open(os.path.join(HERE, name)) as f:
        for line in f:
            line = line.split("#", 1)[0].strip()
            if not line:
                continue
            if ":" in line:
                flush()
                k, rest = line.split(":", 1)
                key, rows = k.strip(), []
                if rest.strip():
                    out[key] = np.array([float(x) for x in rest.split()], dtype=np.float64)
                    key = None
            else:
                rows.append([float(x) for x in line.split()])
    flush()
    return out


def csr_from_rows(cols_per_row, K):
    """CSR (rowptr, colidx) from a list of per-row column lists, stored in the given order."""
    rowptr = np.zeros(len(cols_per_row) + 1, dtype=np.int32)
    for i, c in enumerate(cols_per_row):
        rowptr[i + 1] = rowptr[i] + len(c)
    colidx = np.array([c for row in cols_per_row for c in row], dtype=np.int32)
    assert colidx.size == 0 or (colidx.min() >= 0 and colidx.max() < K)
    return rowptr, colidx


def edge_patterns(rng):
    """Named adversarial patterns: (name, M, K, rowptr, colidx).  Degenerate cases of the
    row loop of Algorithms 1-3: empty rows (leading, trailing, all), one full row among empty
    ones, all rows of length one, unsorted and duplicated columns, a single column."""
    out = []
    K = 96
    full = list(range(K))
    out.append(("all_empty", 7, K, *csr_from_rows([[] for _ in range(7)], K)))
    out.append(("one_full_row_rest_empty", 9, K, *csr_from_rows([[]] * 4 + [full] + [[]] * 4, K)))
    out.append(("empty_first_last", 6, K, *csr_from_rows([[], [], [1, 5, 9], full, [], []], K)))
    out.append(("all_len_one", 130, K, *csr_from_rows([[int(rng.integers(K))] for _ in range(130)], K)))
    rows = [list(rng.permutation(K)[: int(rng.integers(0, 40))]) for _ in range(50)]
    out.append(("unsorted", 50, K, *csr_from_rows(rows, K)))
    rows = [list(rng.integers(0, 8, size=int(rng.integers(1, 30)))) for _ in range(40)]
    out.append(("duplicates", 40, K, *csr_from_rows(rows, K)))
    out.append(("single_column", 33, 1, *csr_from_rows([[0] * int(rng.integers(0, 3)) for _ in range(33)], 1)))
    lens = [0, 1, 63, 64, 65, 127, 128, 129, 255, 256, 257, 1000]
    K2 = 1024
    rows = [sorted(rng.permutation(K2)[:n].tolist()) for n in lens]
    out.append(("ragged_lengths", len(lens), K2, *csr_from_rows(rows, K2)))
    return out
