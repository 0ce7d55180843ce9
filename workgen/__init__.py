"""Seeded synthetic input generators shared by the CPU oracle and the GPU path.

Nothing in this package implements any step of the one-sided method itself:
it only draws op tables, fill patterns, key arrays and graphs.  Random numbers
come from numpy's Philox (a counter-based 64-bit generator) keyed by the seed;
the R-MAT edge list comes from the small C generator in ``rmat.c`` (its own
counter-based draw), built by ``workgen.build``.

Seeds follow one convention: ``BASE_SEED + k`` for configuration k = 1..5 and
``BASE_SEED + 50`` for BFS roots.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

BASE_SEED = 251115076

# 64-byte operation descriptor (window/offset addressing, sizes, an inline
# value) -- the record shape of the Proxy backend's queue entries (Sec. III-C).
OP_PUT, OP_GET, OP_IPUT, OP_IGET = 0, 1, 2, 3
OP_DESC = np.dtype([
    ("kind", "<u4"), ("pe_self", "<u4"), ("pe", "<u4"), ("elem_bytes", "<u4"),
    ("local_off", "<u8"), ("sym_off", "<u8"), ("count", "<u8"),
    ("local_stride", "<i8"), ("sym_stride", "<i8"),
    ("value", "<u8"),
])
assert OP_DESC.itemsize == 64


def rng_for(seed: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=int(seed)))


def random_words(seed: int, nwords: int) -> np.ndarray:
    """nwords uniform uint64 values (heap / source fill pattern)."""
    return rng_for(seed).integers(0, 2**64 - 1, size=nwords, dtype=np.uint64, endpoint=True)


# --------------------------------------------------------------------------
# config 1: random conflict-free put/get table
# --------------------------------------------------------------------------
def _overlaps(ranges, lo, hi):
    for (a, b) in ranges:
        if lo < b and a < hi:
            return True
    return False


def cfg1_op_table(seed: int = BASE_SEED + 1, npes: int = 4, heap_bytes: int = 1 << 20,
                  nops: int = 10000, batch: int = 100, min_log2: int = 3,
                  max_log2: int = 12, align: int = 8) -> np.ndarray:
    """Random put/get descriptors, conflict-free inside every batch.

    Within one batch no written range intersects any other range (read or
    written) of the batch, and no op reads what it writes, so every delivery
    order gives the same heap.  Rejected draws are redrawn.
    """
    rng = rng_for(seed)
    ops = np.zeros(nops, dtype=OP_DESC)
    i = 0
    while i < nops:
        nb = min(batch, nops - i)
        reads = [[] for _ in range(npes)]
        writes = [[] for _ in range(npes)]
        k = 0
        while k < nb:
            kind = int(rng.integers(0, 2))
            pe_self = int(rng.integers(0, npes))
            pe = int(rng.integers(0, npes))
            n = 1 << int(rng.integers(min_log2, max_log2 + 1))
            if n > heap_bytes:
                continue
            span = (heap_bytes - n) // align + 1
            loff = int(rng.integers(0, span)) * align
            soff = int(rng.integers(0, span)) * align
            if kind == OP_PUT:
                rpe, roff, wpe, woff = pe_self, loff, pe, soff
            else:
                rpe, roff, wpe, woff = pe, soff, pe_self, loff
            if rpe == wpe and roff < woff + n and woff < roff + n:
                continue
            if _overlaps(writes[wpe], woff, woff + n) or _overlaps(reads[wpe], woff, woff + n):
                continue
            if _overlaps(writes[rpe], roff, roff + n):
                continue
            reads[rpe].append((roff, roff + n))
            writes[wpe].append((woff, woff + n))
            d = ops[i + k]
            d["kind"], d["pe_self"], d["pe"], d["elem_bytes"] = kind, pe_self, pe, 1
            d["local_off"], d["sym_off"], d["count"] = loff, soff, n
            d["local_stride"], d["sym_stride"] = 1, 1
            k += 1
        i += nb
    return ops


# --------------------------------------------------------------------------
# config 3: atomic op arrays
# --------------------------------------------------------------------------
def zipf_indices(rng: np.random.Generator, n: int, T: int, s: float = 1.0) -> np.ndarray:
    """n indices in [0,T): rank r (1-based) has probability ~ r^-s, index r-1."""
    if T == 1:
        return np.zeros(n, dtype=np.uint32)
    w = 1.0 / np.arange(1, T + 1, dtype=np.float64) ** s
    cdf = np.cumsum(w)
    cdf /= cdf[-1]
    u = rng.random(n)
    idx = np.searchsorted(cdf, u, side="right")
    return np.minimum(idx, T - 1).astype(np.uint32)


def cfg3_amo_ops(seed: int = BASE_SEED + 3, n: int = 1 << 24, npes: int = 64,
                 T: int = 1024, dist: str = "uniform", addend: str = "one"):
    """(target_pe int32[n], index uint32[n], operand uint64[n]).

    addend = "one": operand 1; "rand16": uniform in [1, 2^16]; "tag": i + 1
    (the unique non-zero tag of op i, used by the compare-swap workloads).
    """
    rng = rng_for(seed + (0 if dist == "uniform" else 7) + 131 * T % 1000003)
    pe = rng.integers(0, npes, size=n, dtype=np.int32)
    if dist == "uniform":
        idx = rng.integers(0, T, size=n, dtype=np.uint32)
    elif dist == "zipf":
        idx = zipf_indices(rng, n, T, 1.0)
    else:
        raise ValueError(dist)
    if addend == "one":
        a = np.ones(n, dtype=np.uint64)
    elif addend == "rand16":
        a = rng.integers(1, 1 << 16, size=n, dtype=np.uint64, endpoint=True)
    elif addend == "tag":
        a = np.arange(1, n + 1, dtype=np.uint64)
    else:
        raise ValueError(addend)
    return pe, idx, a


# --------------------------------------------------------------------------
# config 4: hash keys and queries
# --------------------------------------------------------------------------
def cfg4_keys(seed: int = BASE_SEED + 4, n: int = 1 << 26) -> np.ndarray:
    """n uniform uint64 keys in [1, 2^64)."""
    return rng_for(seed).integers(1, 2**64 - 1, size=n, dtype=np.uint64, endpoint=True)


def cfg4_queries(keys: np.ndarray, seed: int = BASE_SEED + 4, n: int | None = None) -> np.ndarray:
    """n queries: half sampled (with replacement) from keys, half fresh, shuffled."""
    n = len(keys) if n is None else n
    rng = rng_for(seed + 1000)
    half = n // 2
    present = keys[rng.integers(0, len(keys), size=half)]
    fresh = rng.integers(1, 2**64 - 1, size=n - half, dtype=np.uint64, endpoint=True)
    q = np.concatenate([present, fresh])
    rng.shuffle(q)
    return q


# --------------------------------------------------------------------------
# config 5: R-MAT graph in CSR form, BFS roots
# --------------------------------------------------------------------------
# --------------------------------------------------------------------------
# MoE-shaped all-to-all traffic (small token batches, top-k routing)
# --------------------------------------------------------------------------
def moe_routing(seed: int = BASE_SEED + 60, npes: int = 8, num_experts: int = 288, max_tokens: int = 128,
                topk: int = 8, ntok=None, dist: str = "uniform", drop: float = 0.0) -> tuple[np.ndarray, np.ndarray]:
    """Routing tables of a decode-sized expert-parallel batch.

    Returns (topk_idx, ntok): topk_idx is int32 [npes, max_tokens, topk], the experts of
    each token (distinct within a token, -1 = unused entry; rows at or beyond a PE's ntok are
    all -1); ntok is int32 [npes].  ``dist`` is "uniform" or "zipf" (expert popularity
    proportional to 1/(rank+1)); ``drop`` is the probability that an entry is replaced by -1.
    """
    rng = rng_for(seed)
    if ntok is None:
        ntok = np.full(npes, max_tokens, dtype=np.int32)
    ntok = np.broadcast_to(np.asarray(ntok, dtype=np.int32), (npes,)).copy()
    assert ntok.min() >= 0 and ntok.max() <= max_tokens and topk <= num_experts
    if dist == "uniform":
        score = rng.random((npes, max_tokens, num_experts))
    elif dist == "zipf":
        w = 1.0 / (1.0 + rng.permutation(num_experts))
        score = rng.random((npes, max_tokens, num_experts)) ** (1.0 / w)      # weighted sampling without replacement
    else:
        raise ValueError(dist)
    idx = np.argsort(-score, axis=2)[:, :, :topk].astype(np.int32)
    if drop > 0:
        idx[rng.random(idx.shape) < drop] = -1
    for p in range(npes):
        idx[p, ntok[p]:] = -1
    return np.ascontiguousarray(idx), ntok


def moe_tokens(seed: int = BASE_SEED + 61, npes: int = 8, max_tokens: int = 128, hidden_bytes: int = 14336) -> np.ndarray:
    """Token payloads: uint8 [npes, max_tokens, hidden_bytes] of uniform random bytes."""
    words = rng_for(seed).integers(0, 2**32 - 1, size=(npes, max_tokens, hidden_bytes // 4), dtype=np.uint32, endpoint=True)
    return words.view(np.uint8).reshape(npes, max_tokens, hidden_bytes)


_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libworkgen.so")
_lib = None


def build(verbose: bool = False) -> str:
    """Compile rmat.c with gcc into libworkgen.so (host code only)."""
    cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-pthread",
           os.path.join(_HERE, "rmat.c"), "-o", _LIB_PATH]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return _LIB_PATH


def _load():
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            build()
        lib = ctypes.CDLL(_LIB_PATH)
        lib.wg_rmat_edges.restype = ctypes.c_int
        lib.wg_rmat_edges.argtypes = [ctypes.c_int, ctypes.c_uint64, ctypes.c_double,
                                      ctypes.c_double, ctypes.c_double, ctypes.c_uint64,
                                      ctypes.c_int, ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p]
        lib.wg_csr_build.restype = ctypes.c_int
        lib.wg_csr_build.argtypes = [ctypes.c_uint32, ctypes.c_uint64, ctypes.c_void_p,
                                     ctypes.c_void_p, ctypes.c_int, ctypes.c_void_p,
                                     ctypes.c_void_p, ctypes.POINTER(ctypes.c_uint64)]
        _lib = lib
    return _lib


def _nthreads() -> int:
    return max(1, min(16, os.cpu_count() or 1))


def rmat_edges(scale: int, edge_factor: int = 16, abc=(0.57, 0.19, 0.19),
               seed: int = BASE_SEED + 5, relabel: bool = True):
    """(src uint32[E], dst uint32[E]) with E = edge_factor * 2^scale."""
    lib = _load()
    ne = edge_factor << scale
    src = np.empty(ne, dtype=np.uint32)
    dst = np.empty(ne, dtype=np.uint32)
    rc = lib.wg_rmat_edges(scale, ne, abc[0], abc[1], abc[2], seed, _nthreads(),
                           int(relabel), src.ctypes.data, dst.ctypes.data)
    if rc != 0:
        raise RuntimeError(f"wg_rmat_edges failed: {rc}")
    return src, dst


def csr_from_edges(nverts: int, src: np.ndarray, dst: np.ndarray):
    """Undirected CSR (row_off uint64[n+1], nbr uint32[nnz]); self-loops dropped,
    duplicates kept, neighbour order = stable by edge position."""
    lib = _load()
    src = np.ascontiguousarray(src, dtype=np.uint32)
    dst = np.ascontiguousarray(dst, dtype=np.uint32)
    row = np.empty(nverts + 1, dtype=np.uint64)
    nnz = ctypes.c_uint64(0)
    rc = lib.wg_csr_build(nverts, len(src), src.ctypes.data, dst.ctypes.data, _nthreads(),
                          row.ctypes.data, None, ctypes.byref(nnz))
    if rc != 0:
        raise RuntimeError(f"wg_csr_build(count) failed: {rc}")
    nbr = np.empty(nnz.value, dtype=np.uint32)
    rc = lib.wg_csr_build(nverts, len(src), src.ctypes.data, dst.ctypes.data, _nthreads(),
                          row.ctypes.data, nbr.ctypes.data, ctypes.byref(nnz))
    if rc != 0:
        raise RuntimeError(f"wg_csr_build(fill) failed: {rc}")
    return row, nbr


def rmat_csr(scale: int, edge_factor: int = 16, abc=(0.57, 0.19, 0.19),
             seed: int = BASE_SEED + 5):
    src, dst = rmat_edges(scale, edge_factor, abc, seed)
    return csr_from_edges(1 << scale, src, dst)


def bfs_roots(row_off: np.ndarray, nroots: int = 64, seed: int = BASE_SEED + 50) -> np.ndarray:
    """nroots distinct vertices of degree >= 1."""
    rng = rng_for(seed)
    n = len(row_off) - 1
    deg = np.diff(row_off)
    if int((deg > 0).sum()) < nroots:
        raise ValueError("not enough non-isolated vertices")
    roots, seen = [], set()
    while len(roots) < nroots:
        v = int(rng.integers(0, n))
        if deg[v] > 0 and v not in seen:
            seen.add(v)
            roots.append(v)
    return np.array(roots, dtype=np.uint32)
