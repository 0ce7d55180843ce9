"""ctypes wrapper over the C oracle (``shmem_oracle.c``).

TEST INFRASTRUCTURE ONLY: imported by tests, the smoke check and the
benchmark's cpu_baseline leg.  It never imports the GPU package and the GPU
package never imports it.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libshmem_oracle.so")
_lib = None

EAGER, AT_QUIET, SHUFFLED = 0, 1, 2
OP_PUT, OP_GET, OP_IPUT, OP_IGET = 0, 1, 2, 3
AMO_FETCH_ADD, AMO_COMPARE_SWAP, AMO_FETCH_OR, AMO_MIN_CAS_LOOP = 0, 1, 2, 3
HASH_INSERTED, HASH_DUPLICATE, HASH_FULL = 0, 1, 2
BFS_NONE = 0xFFFFFFFF


class BfsStats(C.Structure):
    _fields_ = [("nlevels", C.c_uint32), ("reached", C.c_uint64),
                ("edges_traversed", C.c_uint64), ("frontier_size", C.c_uint64 * 64)]


def build(verbose: bool = False) -> str:
    """Compile the oracle with gcc (host code only)."""
    cmd = ["gcc", "-O2", "-std=c11", "-Wall", "-fPIC", "-shared",
           os.path.join(_HERE, "shmem_oracle.c"), "-o", _LIB_PATH]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return _LIB_PATH


def _load():
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        build()
    L = C.CDLL(_LIB_PATH)
    vp, i, u64, sz, i64 = C.c_void_p, C.c_int, C.c_uint64, C.c_size_t, C.c_int64
    pu64 = C.POINTER(C.c_uint64)
    sig = {
        "orc_init": (vp, [i, sz, i, u64]),
        "orc_finalize": (None, [vp]),
        "orc_n_pes": (i, [vp]),
        "orc_heap_bytes": (sz, [vp]),
        "orc_heap": (vp, [vp, i]),
        "orc_pending": (sz, [vp, i]),
        "orc_malloc": (i64, [vp, sz]),
        "orc_align": (i64, [vp, sz, sz]),
        "orc_free": (i, [vp, i64]),
        "orc_live_blocks": (sz, [vp]),
        "orc_put": (i, [vp, i, u64, u64, sz, i]),
        "orc_put_value": (i, [vp, i, u64, u64, sz, i]),
        "orc_get": (i, [vp, i, u64, u64, sz, i]),
        "orc_iput": (i, [vp, i, u64, u64, i64, i64, sz, sz, i]),
        "orc_iget": (i, [vp, i, u64, u64, i64, i64, sz, sz, i]),
        "orc_atomic_fetch_add": (i, [vp, i, u64, u64, i, pu64]),
        "orc_atomic_compare_swap": (i, [vp, i, u64, u64, u64, i, pu64]),
        "orc_atomic_fetch_or": (i, [vp, i, u64, u64, i, pu64]),
        "orc_signal_add": (i, [vp, i, u64, u64, i]),
        "orc_fence": (i, [vp, i]),
        "orc_quiet": (i, [vp, i]),
        "orc_barrier_all": (i, [vp]),
        "orc_team_sync": (i, [vp, i, i, i]),
        "orc_op_batch": (i, [vp, vp, sz, sz]),
        "orc_amo_batch": (i, [vp, i, u64, vp, vp, vp, vp, vp, sz]),
        "orc_hash_mix64": (u64, [u64]),
        "orc_hash_insert": (i, [vp, u64, sz, vp, sz, vp]),
        "orc_hash_lookup": (i, [vp, u64, sz, vp, sz, vp]),
        "orc_bfs": (i, [vp, C.c_uint32, vp, vp, C.c_uint32, vp, vp, C.POINTER(BfsStats)]),
    }
    for name, (res, args) in sig.items():
        fn = getattr(L, name)
        fn.restype, fn.argtypes = res, args
    _lib = L
    return L


def mix64(key: int) -> int:
    return int(_load().orc_hash_mix64(int(key) & (2**64 - 1)))


def _ptr(a):
    return None if a is None else a.ctypes.data


class World:
    """npes host-array PEs, each with a heap_bytes symmetric segment."""

    def __init__(self, npes: int, heap_bytes: int, mode: int = SHUFFLED, shuffle_seed: int = 1):
        self._L = _load()
        self._w = self._L.orc_init(npes, heap_bytes, mode, shuffle_seed)
        if not self._w:
            raise ValueError("orc_init rejected its arguments")
        self.npes, self.heap_bytes = npes, heap_bytes

    def close(self):
        if self._w:
            self._L.orc_finalize(self._w)
            self._w = None

    def __del__(self):
        self.close()

    def __enter__(self):
        return self

    def __exit__(self, *a):
        self.close()

    def heap(self, pe: int) -> np.ndarray:
        """uint8 view (no copy) of PE pe's segment."""
        p = self._L.orc_heap(self._w, pe)
        buf = (C.c_uint8 * self.heap_bytes).from_address(p)
        return np.frombuffer(buf, dtype=np.uint8)

    def heaps(self) -> np.ndarray:
        return np.stack([self.heap(p) for p in range(self.npes)])

    def pending(self, pe): return self._L.orc_pending(self._w, pe)
    def malloc(self, n): return self._L.orc_malloc(self._w, n)
    def align(self, a, n): return self._L.orc_align(self._w, a, n)
    def free(self, off): return self._L.orc_free(self._w, off)
    def live_blocks(self): return self._L.orc_live_blocks(self._w)

    def put(self, pe_self, dst_sym, src_local, nbytes, pe):
        return self._L.orc_put(self._w, pe_self, dst_sym, src_local, nbytes, pe)

    def put_value(self, pe_self, dst_sym, value, nbytes, pe):
        return self._L.orc_put_value(self._w, pe_self, dst_sym, value, nbytes, pe)

    def get(self, pe_self, dst_local, src_sym, nbytes, pe):
        return self._L.orc_get(self._w, pe_self, dst_local, src_sym, nbytes, pe)

    def iput(self, pe_self, dst_sym, src_local, dst_stride, src_stride, nelems, elem_bytes, pe):
        return self._L.orc_iput(self._w, pe_self, dst_sym, src_local, dst_stride, src_stride,
                                nelems, elem_bytes, pe)

    def iget(self, pe_self, dst_local, src_sym, dst_stride, src_stride, nelems, elem_bytes, pe):
        return self._L.orc_iget(self._w, pe_self, dst_local, src_sym, dst_stride, src_stride,
                                nelems, elem_bytes, pe)

    def _amo(self, fn, *args):
        old = C.c_uint64(0)
        rc = fn(self._w, *args, C.byref(old))
        if rc:
            raise RuntimeError(f"oracle AMO failed: {rc}")
        return old.value

    def atomic_fetch_add(self, pe_self, sym, value, pe):
        return self._amo(self._L.orc_atomic_fetch_add, pe_self, sym, value, pe)

    def atomic_compare_swap(self, pe_self, sym, cond, value, pe):
        return self._amo(self._L.orc_atomic_compare_swap, pe_self, sym, cond, value, pe)

    def atomic_fetch_or(self, pe_self, sym, value, pe):
        return self._amo(self._L.orc_atomic_fetch_or, pe_self, sym, value, pe)

    def signal_add(self, pe_self, sig_sym, value, pe):
        return self._L.orc_signal_add(self._w, pe_self, sig_sym, value, pe)

    def fence(self, pe_self): return self._L.orc_fence(self._w, pe_self)
    def quiet(self, pe_self=-1): return self._L.orc_quiet(self._w, pe_self)
    def barrier_all(self): return self._L.orc_barrier_all(self._w)
    def team_sync(self, start, stride, size): return self._L.orc_team_sync(self._w, start, stride, size)

    def op_batch(self, ops: np.ndarray, quiet_every: int) -> int:
        ops = np.ascontiguousarray(ops)
        assert ops.dtype.itemsize == 64
        return self._L.orc_op_batch(self._w, ops.ctypes.data, len(ops), quiet_every)

    def amo_batch(self, kind, ctr_sym, pe, idx, a, b=None):
        n = len(pe)
        pe = np.ascontiguousarray(pe, dtype=np.int32)
        idx = np.ascontiguousarray(idx, dtype=np.uint32)
        a = np.ascontiguousarray(a, dtype=np.uint64)
        b = None if b is None else np.ascontiguousarray(b, dtype=np.uint64)
        if kind == AMO_COMPARE_SWAP and b is None:
            raise ValueError("compare_swap needs b")
        old = np.empty(n, dtype=np.uint64)
        rc = self._L.orc_amo_batch(self._w, kind, ctr_sym, _ptr(pe), _ptr(idx), _ptr(a), _ptr(b),
                                   _ptr(old), n)
        if rc:
            raise RuntimeError(f"orc_amo_batch failed: {rc}")
        return old

    def hash_insert(self, table_sym, slots_per_pe, keys):
        keys = np.ascontiguousarray(keys, dtype=np.uint64)
        st = np.empty(len(keys), dtype=np.uint8)
        rc = self._L.orc_hash_insert(self._w, table_sym, slots_per_pe, _ptr(keys), len(keys), _ptr(st))
        if rc:
            raise RuntimeError(f"orc_hash_insert failed: {rc}")
        return st

    def hash_lookup(self, table_sym, slots_per_pe, keys):
        keys = np.ascontiguousarray(keys, dtype=np.uint64)
        f = np.empty(len(keys), dtype=np.uint8)
        rc = self._L.orc_hash_lookup(self._w, table_sym, slots_per_pe, _ptr(keys), len(keys), _ptr(f))
        if rc:
            raise RuntimeError(f"orc_hash_lookup failed: {rc}")
        return f

    def bfs(self, row_off, nbr, root):
        row_off = np.ascontiguousarray(row_off, dtype=np.uint64)
        nbr = np.ascontiguousarray(nbr, dtype=np.uint32)
        n = len(row_off) - 1
        level = np.empty(n, dtype=np.int32)
        parent = np.empty(n, dtype=np.uint32)
        st = BfsStats()
        rc = self._L.orc_bfs(self._w, n, _ptr(row_off), _ptr(nbr), int(root), _ptr(level),
                             _ptr(parent), C.byref(st))
        if rc:
            raise RuntimeError(f"orc_bfs failed: {rc}")
        stats = {"nlevels": st.nlevels, "reached": st.reached,
                 "edges_traversed": st.edges_traversed,
                 "frontier_size": [int(st.frontier_size[i]) for i in range(min(st.nlevels, 64))]}
        return level, parent, stats


def canonical_parents(row_off, nbr, level, root):
    """Canonical BFS tree for given levels: parent[v] = the smallest neighbour u of v with
    level[u] == level[v] - 1 (parent[root] = root, unreached vertices keep BFS_NONE).  The levels of
    a BFS are unique, so this tree is too -- unlike the first-claimer tree, it can be compared
    vertex by vertex."""
    row_off = np.asarray(row_off, dtype=np.int64)
    nbr = np.asarray(nbr, dtype=np.int64)
    level = np.asarray(level, dtype=np.int64)
    n = len(row_off) - 1
    src = np.repeat(np.arange(n, dtype=np.int64), np.diff(row_off))
    good = (level[src] > 0) & (level[nbr] == level[src] - 1)
    parent = np.full(n, BFS_NONE, dtype=np.int64)
    np.minimum.at(parent, src[good], nbr[good])
    parent[root] = root
    return parent.astype(np.uint32)


def transpose(w: "World", out_sym: int, in_sym: int, n: int, elem_bytes: int):
    """Distributed transpose of an n x n matrix by one-sided strided gets (a variant the method invites;
    the paper has no such operation, so this is the ordinary OpenSHMEM idiom): PE p holds rows
    [p*R, (p+1)*R) of A (R = n / npes, row-major at in_sym) and produces the same rows of B = A^T at
    out_sym.  Row i of B on PE p = column p*R + i of A: one iget per source PE q fetches
    A_q[0..R)[p*R + i] (source stride n) into B_p[i][q*R .. (q+1)*R) (unit stride)."""
    P = w.npes
    assert n % P == 0
    R = n // P
    for p in range(P):
        for i in range(R):
            for q in range(P):
                rc = w.iget(p, out_sym + (i * n + q * R) * elem_bytes, in_sym + (p * R + i) * elem_bytes,
                            1, n, R, elem_bytes, q)
                if rc:
                    raise RuntimeError(f"iget failed: {rc}")

