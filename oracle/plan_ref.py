"""Reference (numpy) builder of the scheduling plan: TEST INFRASTRUCTURE ONLY.

The plan is integer-only and has exactly one correct value, so the GPU builder is compared
with this one bit for bit.  It shares no code with the GPU library.

The attention backward needs SpMMs with the transposed pattern (Section 2.2: dV = U^T dY,
dK = dZ^T Q); the plan therefore holds the transpose of the CSR pattern, ordered so that each
source row adds its terms in ascending stored position (a stable counting sort).  The degree
classes and chunk tables are this implementation's scheduling contract:

* class(deg)  = 0 for deg == 0, else 1 + ceil(log2(deg))          (deg 1 ->1, 2 ->2, 3..4 ->3, ...)
* bin_rows    = row ids ordered by (class descending, row id ascending); bin_off[k] is the
                start of the rows with class 32-k, k = 0..33 (bin_off[33] = number of rows)
* chunked rows = rows with deg > wave_max_deg: a prefix of bin_rows (wave_max_deg is a power
                of two).  Row r of that prefix is cut into ceil(deg / hub_chunk) chunks of
                hub_chunk consecutive entries; chunk_ptr is the exclusive prefix sum of those
                counts; chunks[c] = (row id, first entry, one-past-last entry, chunks of row).
* hub rows    = rows with deg > hub_chunk (more than one chunk): again a prefix of bin_rows.
"""
from __future__ import annotations

import numpy as np

NUM_CLASSES = 33


def degree_class(deg: np.ndarray) -> np.ndarray:
    deg = np.asarray(deg, dtype=np.int64)
    cls = np.zeros(deg.shape, dtype=np.int64)
    pos = deg > 0
    # 1 + ceil(log2(deg)) with integer arithmetic: bit length of (deg - 1), plus one
    dm1 = deg[pos] - 1
    bitlen = np.zeros(dm1.shape, dtype=np.int64)
    t = dm1.copy()
    while np.any(t > 0):
        bitlen += (t > 0)
        t >>= 1
    cls[pos] = 1 + bitlen
    return cls


def bin_rows_ref(indptr: np.ndarray, wave_max_deg: int, hub_chunk: int) -> dict:
    deg = np.diff(indptr.astype(np.int64))
    n = deg.shape[0]
    key = (NUM_CLASSES - 1) - degree_class(deg)
    order = np.argsort(key, kind="stable").astype(np.int32)
    counts = np.bincount(key, minlength=NUM_CLASSES)
    bin_off = np.zeros(NUM_CLASSES + 1, dtype=np.int64)
    bin_off[1:] = np.cumsum(counts)
    n_chunked = int(np.sum(deg > wave_max_deg))
    n_hub = int(np.sum(deg > hub_chunk))
    rows_c = order[:n_chunked].astype(np.int64)
    assert np.all(deg[rows_c] > wave_max_deg)
    per_row = (deg[rows_c] + hub_chunk - 1) // hub_chunk
    chunk_ptr = np.zeros(n_chunked + 1, dtype=np.int64)
    chunk_ptr[1:] = np.cumsum(per_row)
    chunks = np.zeros((int(chunk_ptr[-1]), 4), dtype=np.int32)
    c = 0
    for r, k in zip(rows_c, per_row):
        b, e = int(indptr[r]), int(indptr[r + 1])
        for s in range(int(k)):
            chunks[c] = (r, b + s * hub_chunk, min(b + (s + 1) * hub_chunk, e), k)
            c += 1
    return dict(bin_rows=order, bin_off=bin_off, n_chunked=n_chunked, n_hub=n_hub,
                chunk_ptr=chunk_ptr, chunks=chunks, n_rows=n)


def transpose_ref(indptr: np.ndarray, indices: np.ndarray, n_src: int) -> dict:
    n_dst = indptr.shape[0] - 1
    nnz = int(indptr[-1])
    dst_of_entry = np.repeat(np.arange(n_dst, dtype=np.int64), np.diff(indptr.astype(np.int64)))
    order = np.argsort(indices[:nnz], kind="stable")
    t_indptr = np.zeros(n_src + 1, dtype=np.int64)
    t_indptr[1:] = np.cumsum(np.bincount(indices[:nnz], minlength=n_src))
    return dict(t_indptr=t_indptr, t_indices=dst_of_entry[order].astype(np.int32),
                t_eid=order.astype(np.int32))


def plan_ref(indptr, indices, n_src, wave_max_deg=128, hub_chunk=2048) -> dict:
    out = {"dst": bin_rows_ref(indptr, wave_max_deg, hub_chunk)}
    tr = transpose_ref(indptr, indices, n_src)
    out.update(tr)
    out["src"] = bin_rows_ref(tr["t_indptr"], wave_max_deg, hub_chunk)
    return out
