"""CPU oracle of the Matrix Market reader (the paper's data set, Section VII "Setup", is distributed in this format:
real square matrices of the SuiteSparse collection).

TEST INFRASTRUCTURE ONLY.  Plain Python, written from the published format description (Boisvert, Pozo, Remington:
"The Matrix Market Exchange Formats: Initial Design", NISTIR 5935), coordinate format:

  banner      %%MatrixMarket matrix coordinate <field> <symmetry>        (case-insensitive)
              field in {real, integer, pattern}; symmetry in {general, symmetric, skew-symmetric}
              (complex / hermitian matrices and the dense "array" format are refused: the library stores reals)
  comments    lines starting with '%', and blank lines, anywhere before the size line
  size line   M N L
  L entries   i j [value], 1-based; pattern entries carry no value and mean 1.0
  symmetry    symmetric: an off-diagonal entry (i, j, v) also stands for (j, i, v);
              skew-symmetric: for (j, i, -v), and diagonal entries are not allowed
  result      triplets sorted by (row, col); entries naming the same position are summed in file order (mirrored
              copies after the entries of the file); explicit zeros stay entries.
"""
from __future__ import annotations


class MtxError(ValueError):
    pass


def read_triplets(path: str):
    """-> (m, n, rows, cols, vals): 0-based triplets sorted by (row, col), duplicates summed."""
    with open(path, "r", newline="\n") as fh:      # lines end with LF; a CR before it is white space
        lines = fh.read().split("\n")
    if not lines or not lines[0].startswith("%%MatrixMarket"):
        raise MtxError("no banner")
    banner = lines[0].split()
    if len(banner) != 5 or banner[1].lower() != "matrix" or banner[2].lower() != "coordinate":
        raise MtxError("only 'matrix coordinate' files are supported")
    field, symmetry = banner[3].lower(), banner[4].lower()
    if field not in ("real", "integer", "pattern") or symmetry not in ("general", "symmetric", "skew-symmetric"):
        raise MtxError("unsupported field or symmetry")
    pos = 1
    while pos < len(lines) and (lines[pos].strip() == "" or lines[pos].lstrip().startswith("%")):
        pos += 1
    if pos >= len(lines):
        raise MtxError("no size line")
    size = lines[pos].split()
    if len(size) != 3:
        raise MtxError("bad size line")
    m, n, count = (int(t) for t in size)
    if m < 1 or n < 1 or count < 0:
        raise MtxError("bad sizes")
    if symmetry != "general" and m != n:
        raise MtxError("a symmetric matrix must be square")
    pos += 1
    direct, mirrored = [], []
    for _ in range(count):
        while pos < len(lines) and lines[pos].strip() == "":
            pos += 1
        if pos >= len(lines):
            raise MtxError("fewer entries than announced")
        tok = lines[pos].split()
        pos += 1
        if len(tok) != (2 if field == "pattern" else 3):
            raise MtxError("bad entry line")
        i, j = int(tok[0]) - 1, int(tok[1]) - 1
        v = 1.0 if field == "pattern" else float(tok[2])
        if not (0 <= i < m and 0 <= j < n):
            raise MtxError("index out of range")
        direct.append((i, j, v))
        if symmetry != "general" and i != j:
            mirrored.append((j, i, v if symmetry == "symmetric" else -v))
        if symmetry == "skew-symmetric" and i == j:
            raise MtxError("diagonal entry in a skew-symmetric matrix")
    if any(l.strip() for l in lines[pos:]):
        raise MtxError("more entries than announced")
    acc = {}
    for i, j, v in direct + mirrored:
        acc[(i, j)] = acc[(i, j)] + v if (i, j) in acc else v
    keys = sorted(acc)
    return m, n, [k[0] for k in keys], [k[1] for k in keys], [acc[k] for k in keys]


def read_csr(path: str):
    """-> (m, n, row_ptr, col_idx, val) as lists."""
    m, n, rows, cols, vals = read_triplets(path)
    row_ptr = [0] * (m + 1)
    for r in rows:
        row_ptr[r + 1] += 1
    for r in range(m):
        row_ptr[r + 1] += row_ptr[r]
    return m, n, row_ptr, cols, vals
