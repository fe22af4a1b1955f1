"""Seeded synthetic inputs shaped like the paper's workloads (Table 2 gives only node and
edge counts; the graphs here are synthetic stand-ins, not the datasets).

This package serves both the CPU oracle's tests and the GPU path; it holds no attention
arithmetic.  Graph sampling and tensor generation run in ``graphgen.cpp`` (built by
``gen.build()``), reached through ctypes.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass, field

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
# SGA_SANITIZE=1 selects a host build with AddressSanitizer + UndefinedBehaviorSanitizer in its own
# file (run python with the ASan runtime preloaded: LD_PRELOAD=$(g++ -print-file-name=libasan.so))
_SANITIZE = os.environ.get("SGA_SANITIZE", "") == "1"
_LIB_PATH = os.path.join(_HERE, "libgraphgen_san.so" if _SANITIZE else "libgraphgen.so")
_CXXFLAGS = (["-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined"]
             if _SANITIZE else ["-O2"])
_lib = None

BASE_SEED = 0x260416715
# stream ids inside one config's seed (0/1 and 6/7 are used by the graph sampler)
STREAM_Q, STREAM_K, STREAM_V, STREAM_DOUT = 2, 3, 4, 5


def build(force: bool = True) -> str:
    """Compile the generator library in-tree."""
    src = os.path.join(_HERE, "graphgen.cpp")
    if force or not os.path.exists(_LIB_PATH):
        subprocess.check_call(
            ["g++", *_CXXFLAGS, "-std=c++17", "-fopenmp", "-fPIC", "-shared", "-o", _LIB_PATH, src]
        )
    return _LIB_PATH


def _load():
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            build()
        lib = ctypes.CDLL(_LIB_PATH)
        i64, u64, dbl, ci, vp = (ctypes.c_int64, ctypes.c_uint64, ctypes.c_double, ctypes.c_int,
                                 ctypes.c_void_p)
        lib.gen_chung_lu.restype = i64
        lib.gen_chung_lu.argtypes = [i64, i64, dbl, dbl, ci, u64, vp, vp]
        lib.gen_rmat.restype = i64
        lib.gen_rmat.argtypes = [ci, i64, dbl, dbl, dbl, ci, dbl, u64, vp, vp]
        lib.gen_normal_f32.restype = None
        lib.gen_normal_f32.argtypes = [vp, i64, u64, u64]
        lib.gen_normal_bf16.restype = None
        lib.gen_normal_bf16.argtypes = [vp, i64, u64, u64]
        _lib = lib
    return _lib


def chung_lu(n, draws, gamma, target_max_deg, symmetric, seed):
    """CSR-by-destination power-law graph with self-loops: (indptr int64, indices int32)."""
    lib = _load()
    cap = draws * (2 if symmetric else 1) + n
    indptr = np.empty(n + 1, dtype=np.int64)
    indices = np.empty(cap, dtype=np.int32)
    nnz = lib.gen_chung_lu(n, draws, gamma, target_max_deg, int(bool(symmetric)), seed,
                           indptr.ctypes.data, indices.ctypes.data)
    return indptr, indices[:nnz].copy() if nnz < cap // 2 else indices[:nnz]


def rmat(scale, draws, a=0.57, b=0.19, c=0.19, halo_log2=-1, halo_prob=0.0, seed=0):
    """CSR-by-destination R-MAT graph with self-loops on the 2^scale owned rows."""
    lib = _load()
    n = 1 << scale
    cap = draws + n
    indptr = np.empty(n + 1, dtype=np.int64)
    indices = np.empty(cap, dtype=np.int32)
    nnz = lib.gen_rmat(scale, draws, a, b, c, halo_log2, halo_prob, seed,
                       indptr.ctypes.data, indices.ctypes.data)
    return indptr, indices[:nnz]


def normal(shape, dtype, seed, stream):
    """N(0,1) samples.  dtype 'f32' -> float32 array; 'bf16' -> uint16 bit patterns (RNE)."""
    lib = _load()
    n = int(np.prod(shape))
    if dtype == "f32":
        out = np.empty(shape, dtype=np.float32)
        lib.gen_normal_f32(out.ctypes.data, n, seed, stream)
    elif dtype == "bf16":
        out = np.empty(shape, dtype=np.uint16)
        lib.gen_normal_bf16(out.ctypes.data, n, seed, stream)
    else:
        raise ValueError(dtype)
    return out


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    """Exact widening of bfloat16 bit patterns to float32."""
    return (bits.astype(np.uint32) << 16).view(np.float32)


def as_f32(x: np.ndarray) -> np.ndarray:
    """Storage array (float32 or bf16 bit patterns) -> float32 values, exactly."""
    return bf16_bits_to_f32(x) if x.dtype == np.uint16 else x


@dataclass
class Workload:
    name: str
    n_dst: int
    n_src: int
    indptr: np.ndarray
    indices: np.ndarray
    heads: int
    head_dim: int
    dtype: str  # 'f32' | 'bf16'
    seed: int
    recipe: str = ""
    _cache: dict = field(default_factory=dict, repr=False)

    @property
    def nnz(self) -> int:
        return int(self.indptr[-1])

    def tensor(self, which: str) -> np.ndarray:
        """'Q' | 'K' | 'V' | 'dO' in storage dtype, shape [rows, heads, head_dim]."""
        rows, stream = {
            "Q": (self.n_dst, STREAM_Q), "K": (self.n_src, STREAM_K),
            "V": (self.n_src, STREAM_V), "dO": (self.n_dst, STREAM_DOUT),
        }[which]
        return normal((rows, self.heads, self.head_dim), self.dtype, self.seed, stream)


# name -> (index in the list of benchmark configurations)
CONFIG_INDEX = {"tiny": 0, "mid": 1, "large": 2, "partition": 3, "skew": 4}


def workload(name: str, shrink: int = 1) -> Workload:
    """One of the five benchmark workloads.  shrink > 1 divides node and draw counts (R-MAT:
    lowers the scale) so the same recipe gives a test-sized instance."""
    idx = CONFIG_INDEX[name]
    seed = BASE_SEED + idx
    if name == "tiny":
        n, draws = 4096 // shrink, 40_000 // shrink
        indptr, indices = chung_lu(n, draws, 2.1, min(512.0, n / 4), False, seed)
        return Workload(name, n, n, indptr, indices, 4, 16, "f32", seed,
                        f"chung-lu directed n={n} draws={draws} gamma=2.1 +self-loops")
    if name == "mid":
        n, draws = 169_343 // shrink, 1_170_000 // shrink
        indptr, indices = chung_lu(n, draws, 2.2, min(13_000.0, n / 4), False, seed)
        return Workload(name, n, n, indptr, indices, 8, 16, "f32", seed,
                        f"chung-lu directed n={n} draws={draws} gamma=2.2 +self-loops")
    if name == "large":
        n, draws = 2_450_000 // shrink, 31_000_000 // shrink
        indptr, indices = chung_lu(n, draws, 2.2, min(17_000.0, n / 4), True, seed)
        return Workload(name, n, n, indptr, indices, 8, 32, "bf16", seed,
                        f"chung-lu symmetric n={n} draws={draws} gamma=2.2 +self-loops")
    lg = max(0, int(round(np.log2(shrink))))
    if name == "partition":
        scale, draws = 21 - lg, 48_000_000 >> lg
        indptr, indices = rmat(scale, draws, halo_log2=scale - 1, halo_prob=0.30, seed=seed)
        n = 1 << scale
        return Workload(name, n, n + (n >> 1), indptr, indices, 4, 64, "bf16", seed,
                        f"rmat scale={scale} draws={draws} halo=2^{scale - 1} p=.30 +self-loops")
    if name == "skew":
        scale, draws = 23 - lg, (1 << 27) >> lg
        indptr, indices = rmat(scale, draws, seed=seed)
        n = 1 << scale
        return Workload(name, n, n, indptr, indices, 1, 64, "bf16", seed,
                        f"rmat scale={scale} draws={draws} +self-loops")
    raise KeyError(name)


def random_csr(n_dst, n_src, nnz_target, seed, allow_dup=False, sort_rows=True):
    """Small uniform random CSR for unit tests (numpy only; optional duplicates / unsorted rows)."""
    rng = np.random.Generator(np.random.Philox(seed))
    dst = rng.integers(0, n_dst, size=nnz_target)
    src = rng.integers(0, n_src, size=nnz_target)
    if not allow_dup:
        key = np.unique(dst.astype(np.int64) * n_src + src)
        dst, src = key // n_src, key % n_src
    order = np.lexsort((src, dst)) if sort_rows else np.argsort(dst, kind="stable")
    dst, src = dst[order], src[order]
    indptr = np.zeros(n_dst + 1, dtype=np.int64)
    np.add.at(indptr, dst + 1, 1)
    indptr = np.cumsum(indptr)
    return indptr, src.astype(np.int32)
