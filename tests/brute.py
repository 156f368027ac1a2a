"""A second, even plainer implementation used only to pin the oracle on tiny inputs.

Pure Python / numpy, written from the method's definition: dict-of-lists partitioning, a dense
fp64 sum for aggregation.  It takes the owner of an index as a *given table*, so it contains no
hash of its own.
"""
import struct

import numpy as np


def is_nonzero_word(f):
    bits = struct.unpack("<I", struct.pack("<f", float(f)))[0] if not isinstance(f, (np.floating,)) else int(
        np.float32(f).view(np.uint32))
    return (bits & 0x7FFFFFFF) != 0


def nonzero_rows(grad2d):
    out = []
    for r in range(grad2d.shape[0]):
        if any(is_nonzero_word(x) for x in grad2d[r]):
            out.append(r)
    return out


def encode(grad2d, owner, n):
    """-> offsets list[n+1], indices list, values list of rows."""
    parts = {p: [] for p in range(n)}
    for r in nonzero_rows(grad2d):
        parts[int(owner[r])].append(r)
    offsets, indices = [0], []
    for p in range(n):
        indices.extend(sorted(parts[p]))
        offsets.append(len(indices))
    values = [grad2d[r].copy() for r in indices]
    return offsets, indices, values


def bitmap(owner, n, nz_rows):
    """-> list over partitions of python ints used as bit strings (bit j = j-th domain row is non-zero)."""
    nzset = set(int(r) for r in nz_rows)
    out = []
    for p in range(n):
        dom = [r for r in range(len(owner)) if owner[r] == p]
        bits = 0
        for j, r in enumerate(dom):
            if r in nzset:
                bits |= 1 << j
        out.append((bits, len(dom)))
    return out


def aggregate_dense(parts, n_rows, row_dim):
    """Dense fp64 sum of the densified parts + set of touched rows."""
    acc = np.zeros((n_rows, row_dim), np.float64)
    touched = set()
    for idx, val in parts:
        for k, r in enumerate(idx):
            acc[int(r)] += np.asarray(val[k], np.float64)
            touched.add(int(r))
    return acc, sorted(touched)


def densify(parts, n_rows, row_dim):
    """Dense fp32 tensor holding every part's rows at their indices, zero elsewhere."""
    out = np.zeros((n_rows, row_dim), np.float32)
    for idx, val in parts:
        for k, r in enumerate(idx):
            out[int(r)] = np.asarray(val[k], np.float32)
    return out


def hier_hash(I, part, slots, n, r1, r2):
    """Algorithm 1's hash memory with Python lists, indices taken in order.  -> (memory as list of
    lists with None for empty cells, serial counts)."""
    mem = [[None] * (r1 + r2) for _ in range(n)]
    counter = [r1] * n
    for t, idx in enumerate(I):
        p = int(part[t])
        for h in slots:
            q = int(h[t])
            if mem[p][q] is None:
                mem[p][q] = int(idx)
                break
        else:
            q = counter[p]
            counter[p] += 1
            if q < r1 + r2:
                mem[p][q] = int(idx)
    return mem, [c - r1 for c in counter]
