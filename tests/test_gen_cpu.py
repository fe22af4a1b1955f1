"""The seeded input generators: reproducible bit for bit (also across thread counts), and the graphs
have the structure the recipe states (CSR by destination, one self-loop per owned row, rows sorted and
free of duplicates, sources in range, the realised sizes the design document lists)."""
import hashlib
import os
import subprocess
import sys

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def digest(w):
    h = hashlib.sha256()
    for a in (w.indptr, w.indices, w.tensor("Q"), w.tensor("K"), w.tensor("V"), w.tensor("dO")):
        h.update(np.ascontiguousarray(a).tobytes())
    return h.hexdigest()


@pytest.mark.parametrize("name,shrink,nnz,max_in", [("tiny", 1, 41_974, 385), ("mid", 1, 1_291_504, 8_924),
                                                    ("large", 64, None, None), ("partition", 64, None, None),
                                                    ("skew", 256, None, None)])
def test_graph_structure(gen, name, shrink, nnz, max_in):
    w = gen.workload(name, shrink)
    ptr, idx = w.indptr, w.indices
    assert ptr.dtype == np.int64 and idx.dtype == np.int32 and len(ptr) == w.n_dst + 1
    assert ptr[0] == 0 and ptr[-1] == len(idx) == w.nnz and np.all(np.diff(ptr) >= 0)
    assert idx.min() >= 0 and idx.max() < w.n_src and w.n_src >= w.n_dst
    if nnz is not None:
        assert w.nnz == nnz and int(np.diff(ptr).max()) == max_in
    dst = np.repeat(np.arange(w.n_dst), np.diff(ptr))
    # rows sorted by source, no duplicate entries
    key = dst.astype(np.int64) * w.n_src + idx
    assert np.all(np.diff(key) > 0)
    # one self-loop per owned row
    assert np.count_nonzero(idx == dst) == w.n_dst
    if name == "large":        # symmetric: every entry has its mirror image
        mirror = idx.astype(np.int64) * w.n_src + dst
        assert np.array_equal(np.sort(mirror), key)
    if name == "partition":    # about 30 % of the sampled entries point at halo rows
        halo = np.count_nonzero(idx >= w.n_dst) / (w.nnz - w.n_dst)
        assert 0.2 < halo < 0.35


def test_same_seed_same_bits_and_thread_count_does_not_matter(gen):
    here = digest(gen.workload("mid", 4))
    assert here == digest(gen.workload("mid", 4))
    code = ("import sys; sys.path.insert(0, %r); sys.path.insert(0, %r); import gen, test_gen_cpu; "
            "print(test_gen_cpu.digest(gen.workload('mid', 4)))" % (ROOT, os.path.join(ROOT, "tests")))
    for threads in ("1", "3"):
        env = dict(os.environ, OMP_NUM_THREADS=threads)
        out = subprocess.run([sys.executable, "-c", code], env=env, capture_output=True, text=True, check=True)
        assert out.stdout.strip() == here, f"OMP_NUM_THREADS={threads} changes the generated inputs"
    assert digest(gen.workload("mid", 8)) != here


def test_normal_tensors(gen):
    x = gen.normal((200_000,), "f32", 12345, 2)
    assert abs(float(x.mean())) < 0.01 and abs(float(x.std()) - 1.0) < 0.01
    assert not np.array_equal(x, gen.normal((200_000,), "f32", 12345, 3))      # another stream
    assert not np.array_equal(x, gen.normal((200_000,), "f32", 12346, 2))      # another seed
    # the bf16 generator is the same stream rounded to nearest even
    b = gen.normal((200_000,), "bf16", 12345, 2)
    u = x.view(np.uint32)
    rne = ((u + 0x7FFF + ((u >> 16) & 1)) >> 16).astype(np.uint16)
    assert np.array_equal(b, rne)
    assert np.array_equal(gen.as_f32(b), gen.bf16_bits_to_f32(b))
