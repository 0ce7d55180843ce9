"""Thin ctypes binding over ``libmi_shmem.so`` (the C ABI of ``include/mi_shmem.h``).

Argument marshalling only: every step of the path runs in the library's HIP
kernels.  Device memory is passed as integer addresses (``tensor.data_ptr()``)
or as torch tensors, from which the address is taken.  There is no CPU
fallback: if the library is missing, importing this package raises.
"""
from __future__ import annotations

import ctypes as C
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmi_shmem.so")

OK = 0
ERR_NOT_INIT, ERR_ALREADY_INIT, ERR_INVALID_ARG, ERR_INVALID_PE = -1, -2, -3, -4
ERR_OUT_OF_RANGE, ERR_ALIGN, ERR_NOMEM, ERR_BAD_FREE, ERR_DEVICE, ERR_DEVICE_FAULT = -5, -6, -7, -8, -9, -10
OP_PUT, OP_GET, OP_IPUT, OP_IGET = 0, 1, 2, 3
AMO_FETCH_ADD, AMO_COMPARE_SWAP, AMO_FETCH_OR, AMO_MIN_CAS_LOOP = 0, 1, 2, 3
HASH_INSERTED, HASH_DUPLICATE, HASH_FULL = 0, 1, 2
BFS_NONE = 0xFFFFFFFF
BFS_TOP_DOWN, BFS_DIRECTION_OPTIMIZING, BFS_BOTTOM_UP = 0, 1, 2
BFS_CANONICAL_PARENTS = 0x100


class ShmemError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {strerror(status)} ({status})")


class BfsStats(C.Structure):
    _fields_ = [("nlevels", C.c_uint32), ("reached", C.c_uint64),
                ("edges_traversed", C.c_uint64), ("frontier_size", C.c_uint64 * 64)]


if not os.path.exists(LIB_PATH):
    raise ImportError(
        f"{LIB_PATH} is missing: build it first (python -c 'import __graft_entry__ as g; g.build()'). "
        "This package has no CPU fallback.")

# The library must share ONE HIP runtime with whoever allocates the device memory it is handed.  PyTorch's
# wheel ships its own copy of the runtime; if the library were loaded first it would bind to the system's copy
# and torch's pointers would mean nothing to it (shmem_init then fails with ERR_DEVICE).  So where torch is
# installed it is loaded first, whatever order the caller imports things in.
try:
    import torch as _torch  # noqa: F401
except ImportError:  # callers that bring device memory from elsewhere (plain HIP through ctypes, say)
    _torch = None

_L = C.CDLL(LIB_PATH)
_vp, _i, _u64, _sz, _pd = C.c_void_p, C.c_int, C.c_uint64, C.c_size_t, C.c_ssize_t
_SIG = {
    "shmem_strerror": (C.c_char_p, [_i]),
    "shmem_scratch_bytes": (_sz, [_i]),
    "shmem_init": (_i, [_i, _sz, _vp, _vp, _vp]),
    "shmem_finalize": (_i, []),
    "shmem_n_pes": (_i, []),
    "shmem_malloc": (_vp, [_sz]),
    "shmem_align": (_vp, [_sz, _sz]),
    "shmem_free": (_i, [_vp]),
    "shmem_ptr": (_vp, [_vp, _i]),
    "shmem_put": (_i, [_i, _vp, _vp, _sz, _i]),
    "shmem_get": (_i, [_i, _vp, _vp, _sz, _i]),
    "shmem_put_signal": (_i, [_i, _vp, _vp, _sz, _vp, _u64, _i]),
    "shmem_iput": (_i, [_i, _vp, _vp, _pd, _pd, _sz, _sz, _i]),
    "shmem_iget": (_i, [_i, _vp, _vp, _pd, _pd, _sz, _sz, _i]),
    "shmem_atomic_fetch_add": (_i, [_i, _vp, _u64, _i, _vp]),
    "shmem_atomic_compare_swap": (_i, [_i, _vp, _u64, _u64, _i, _vp]),
    "shmem_atomic_fetch_or": (_i, [_i, _vp, _u64, _i, _vp]),
    "shmem_fence": (_i, [_i]),
    "shmem_quiet": (_i, [_i]),
    "shmem_barrier_all": (_i, []),
    "shmem_stream_sync": (_i, [C.POINTER(C.c_uint64)]),
    "shmem_op_batch": (_i, [_vp, _sz, _sz, _i]),
    "shmem_op_batch_noalloc": (_i, [_i, _sz, _vp, _vp, _sz, _sz, _i, _vp, _vp]),
    "shmem_copy_sweep": (_i, [_i, _vp, _vp, _sz, _sz, _pd, _pd, _sz, _sz, _sz, _i, _i]),
    "shmem_copy_sweep_geometry": (_i, [_i, _vp, _vp, _sz, _sz, _sz, _sz, _i, _i, C.POINTER(C.c_int), C.POINTER(C.c_int)]),
    "shmem_amo_batch": (_i, [_i, _vp, _sz, _vp, _vp, _vp, _vp, _vp, _sz, _i, _i]),
    "shmem_hash_insert": (_i, [_vp, _sz, _vp, _sz, _vp, _i]),
    "shmem_hash_lookup": (_i, [_vp, _sz, _vp, _sz, _vp, _i]),
    "shmem_bfs_create": (_i, [C.c_uint32, _vp, _vp, _i, C.POINTER(_vp)]),
    "shmem_bfs_destroy": (_i, [_vp]),
    "shmem_bfs_configure": (_i, [_vp, _i, _i, _i]),
    "shmem_bfs": (_i, [_vp, C.c_uint32, _vp, _vp, C.POINTER(BfsStats)]),
    "shmem_bfs_level_times": (_i, [_vp, C.POINTER(C.c_uint32), C.POINTER(C.c_float), C.POINTER(C.c_uint8), C.c_uint32]),
    "shmem_gin_create": (_i, [_i, _i, C.POINTER(_vp)]),
    "shmem_gin_destroy": (_i, [_vp]),
    "shmem_gin_signal_sym": (_vp, [_vp, _i]),
    "shmem_gin_counter_sym": (_vp, [_vp, _i]),
    "shmem_device_context": (_i, [_vp]),
    "shmem_gin_device_state": (_i, [_vp, _vp]),
    "shmem_team_create": (_i, [_i, _i, _i, _vp]),
    "shmem_team_destroy": (_i, [_vp]),
    "shmem_team_device_state": (_i, [_vp, _vp]),
    "shmem_team_sync": (_i, [_vp, _i]),
    "shmem_team_epochs": (_i, [_vp, _vp, _i, _vp, _i, _vp]),
    "shmem_ring_exchange": (_i, [_vp, _vp, _sz, _vp, _i, _i, _i, _i]),
    "shmem_pingpong": (_i, [_vp, _sz, _vp, _i, _i]),
    "shmem_barrier_epochs": (_i, [_vp, _i, _i, _vp]),
    "shmem_fence_litmus": (_i, [_vp, _sz, _i, _i, _vp]),
    "shmem_moe_create": (_i, [_i, _i, _i, _sz, C.POINTER(_vp)]),
    "shmem_moe_destroy": (_i, [_vp]),
    "shmem_moe_dispatch": (_i, [_vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _i]),
    "shmem_moe_combine": (_i, [_vp, _vp, _vp, _vp, _vp, _vp, _vp, _i]),
    "shmem_proxy_create": (_i, [_sz, C.POINTER(_vp)]),
    "shmem_proxy_submit": (_i, [_vp, _vp, _sz, _i]),
    "shmem_proxy_quiet": (_i, [_vp, C.POINTER(C.c_uint64)]),
    "shmem_proxy_stats": (_i, [_vp, C.POINTER(C.c_uint64), C.POINTER(C.c_uint64), C.POINTER(C.c_uint64)]),
    "shmem_proxy_destroy": (_i, [_vp]),
    "shmem_transpose": (_i, [_vp, _vp, _sz, _sz, _i]),
}
for _name, (_res, _args) in _SIG.items():
    _fn = getattr(_L, _name)
    _fn.restype, _fn.argtypes = _res, _args

EXPORTS = tuple(_SIG)


def _addr(x):
    """Integer device address of a torch tensor / int / None."""
    if x is None:
        return None
    if hasattr(x, "data_ptr"):
        return x.data_ptr()
    return int(x)


def _check(status: int, where: str) -> int:
    if status != OK:
        raise ShmemError(status, where)
    return status


def strerror(status: int) -> str:
    return _L.shmem_strerror(status).decode()


def scratch_bytes(npes: int) -> int:
    return _L.shmem_scratch_bytes(npes)


def init(npes, heap_bytes_per_pe, dev_heap, dev_scratch, hip_stream=0):
    return _check(_L.shmem_init(npes, heap_bytes_per_pe, _addr(dev_heap), _addr(dev_scratch),
                                _addr(hip_stream) or None), "shmem_init")


def finalize():
    return _check(_L.shmem_finalize(), "shmem_finalize")


def n_pes() -> int:
    return _L.shmem_n_pes()


def malloc(nbytes: int):
    """Symmetric address (int) or None."""
    return _L.shmem_malloc(nbytes)


def align(alignment: int, nbytes: int):
    return _L.shmem_align(alignment, nbytes)


def free(sym):
    return _check(_L.shmem_free(sym), "shmem_free")


def ptr(sym, pe: int):
    return _L.shmem_ptr(sym, pe)


def put(pe_self, dst_sym, src_local, nbytes, pe):
    return _check(_L.shmem_put(pe_self, _addr(dst_sym), _addr(src_local), nbytes, pe), "shmem_put")


def put_signal(pe_self, dst_sym, src_local, nbytes, sig_sym, value, pe):
    return _check(_L.shmem_put_signal(pe_self, _addr(dst_sym), _addr(src_local), nbytes, _addr(sig_sym), value, pe),
                  "shmem_put_signal")


def get(pe_self, dst_local, src_sym, nbytes, pe):
    return _check(_L.shmem_get(pe_self, _addr(dst_local), _addr(src_sym), nbytes, pe), "shmem_get")


def iput(pe_self, dst_sym, src_local, dst_stride, src_stride, nelems, elem_bytes, pe):
    return _check(_L.shmem_iput(pe_self, _addr(dst_sym), _addr(src_local), dst_stride, src_stride,
                                nelems, elem_bytes, pe), "shmem_iput")


def iget(pe_self, dst_local, src_sym, dst_stride, src_stride, nelems, elem_bytes, pe):
    return _check(_L.shmem_iget(pe_self, _addr(dst_local), _addr(src_sym), dst_stride, src_stride,
                                nelems, elem_bytes, pe), "shmem_iget")


def atomic_fetch_add(pe_self, dst_sym, value, pe, dev_result=None):
    return _check(_L.shmem_atomic_fetch_add(pe_self, _addr(dst_sym), value, pe, _addr(dev_result)),
                  "shmem_atomic_fetch_add")


def atomic_compare_swap(pe_self, dst_sym, cond, value, pe, dev_result=None):
    return _check(_L.shmem_atomic_compare_swap(pe_self, _addr(dst_sym), cond, value, pe, _addr(dev_result)),
                  "shmem_atomic_compare_swap")


def atomic_fetch_or(pe_self, dst_sym, value, pe, dev_result=None):
    return _check(_L.shmem_atomic_fetch_or(pe_self, _addr(dst_sym), value, pe, _addr(dev_result)),
                  "shmem_atomic_fetch_or")


def fence(pe_self):
    return _check(_L.shmem_fence(pe_self), "shmem_fence")


def quiet(pe_self=-1):
    return _check(_L.shmem_quiet(pe_self), "shmem_quiet")


def barrier_all():
    return _check(_L.shmem_barrier_all(), "shmem_barrier_all")


def stream_sync():
    """Waits for the stream; raises ShmemError(ERR_DEVICE_FAULT) with the first bad op index."""
    bad = C.c_uint64(0)
    rc = _L.shmem_stream_sync(C.byref(bad))
    if rc == ERR_DEVICE_FAULT:
        e = ShmemError(rc, f"shmem_stream_sync (first rejected op {bad.value})")
        e.first_bad_index = bad.value
        raise e
    return _check(rc, "shmem_stream_sync")


def op_batch(dev_ops, n, quiet_every, wgs_per_pe):
    return _check(_L.shmem_op_batch(_addr(dev_ops), n, quiet_every, wgs_per_pe), "shmem_op_batch")


def op_batch_noalloc(npes, heap_bytes_per_pe, dev_heap, dev_ops, n, quiet_every, wgs_per_pe, dev_fault, hip_stream):
    return _check(_L.shmem_op_batch_noalloc(npes, heap_bytes_per_pe, _addr(dev_heap), _addr(dev_ops), n, quiet_every,
                                            wgs_per_pe, _addr(dev_fault), hip_stream), "shmem_op_batch_noalloc")


def copy_sweep(kind, remote_sym, local_sym, count, elem_bytes=1, remote_stride=1, local_stride=1,
               remote_slot_bytes=0, local_slot_bytes=0, nslots=1, ops_per_pe=1, wgs_per_pe=1):
    return _check(_L.shmem_copy_sweep(kind, _addr(remote_sym), _addr(local_sym), count, elem_bytes,
                                      remote_stride, local_stride, remote_slot_bytes, local_slot_bytes,
                                      nslots, ops_per_pe, wgs_per_pe), "shmem_copy_sweep")


def copy_sweep_geometry(kind, remote_sym, local_sym, count, remote_slot_bytes, local_slot_bytes, nslots, ops_per_pe,
                        wgs_per_pe):
    """(workgroups, threads per workgroup) of the launch copy_sweep makes for this cell."""
    wgs, thr = C.c_int(0), C.c_int(0)
    _check(_L.shmem_copy_sweep_geometry(kind, _addr(remote_sym), _addr(local_sym), count, remote_slot_bytes,
                                        local_slot_bytes, nslots, ops_per_pe, wgs_per_pe, C.byref(wgs), C.byref(thr)),
           "shmem_copy_sweep_geometry")
    return wgs.value, thr.value


def amo_batch(kind, ctr_sym, T, dev_pe, dev_idx, dev_a, dev_b, dev_old, n, wgs_per_pe, aggregate=0):
    return _check(_L.shmem_amo_batch(kind, _addr(ctr_sym), T, _addr(dev_pe), _addr(dev_idx), _addr(dev_a),
                                     _addr(dev_b), _addr(dev_old), n, wgs_per_pe, aggregate),
                  "shmem_amo_batch")


def hash_insert(table_sym, slots_per_pe, dev_keys, n, dev_status, wgs_per_pe):
    return _check(_L.shmem_hash_insert(_addr(table_sym), slots_per_pe, _addr(dev_keys), n,
                                       _addr(dev_status), wgs_per_pe), "shmem_hash_insert")


def hash_lookup(table_sym, slots_per_pe, dev_keys, n, dev_found, wgs_per_pe):
    return _check(_L.shmem_hash_lookup(_addr(table_sym), slots_per_pe, _addr(dev_keys), n,
                                       _addr(dev_found), wgs_per_pe), "shmem_hash_lookup")


def bfs_create(nverts, dev_row_off, dev_nbr, wgs_per_pe):
    g = _vp(0)
    _check(_L.shmem_bfs_create(nverts, _addr(dev_row_off), _addr(dev_nbr), wgs_per_pe, C.byref(g)),
           "shmem_bfs_create")
    return g


def bfs_configure(graph, mode, alpha=0, beta=0):
    return _check(_L.shmem_bfs_configure(graph, mode, alpha, beta), "shmem_bfs_configure")


def bfs_destroy(graph):
    return _check(_L.shmem_bfs_destroy(graph), "shmem_bfs_destroy")


def bfs(graph, root, dev_level=None, dev_parent=None):
    st = BfsStats()
    _check(_L.shmem_bfs(graph, int(root), _addr(dev_level), _addr(dev_parent), C.byref(st)), "shmem_bfs")
    return {"nlevels": st.nlevels, "reached": st.reached, "edges_traversed": st.edges_traversed,
            "frontier_size": [int(st.frontier_size[i]) for i in range(min(st.nlevels, 64))]}


def bfs_level_times(graph):
    """[(microseconds, ran bottom-up)] per level of the last search on this graph (the first 64 levels)."""
    n = C.c_uint32(0)
    us = (C.c_float * 64)()
    bu = (C.c_uint8 * 64)()
    _check(_L.shmem_bfs_level_times(graph, C.byref(n), us, bu, 64), "shmem_bfs_level_times")
    return [(float(us[i]), bool(bu[i])) for i in range(n.value)]


def gin_create(nsignals, ncounters):
    g = _vp(0)
    _check(_L.shmem_gin_create(nsignals, ncounters, C.byref(g)), "shmem_gin_create")
    return g


def gin_destroy(gin):
    return _check(_L.shmem_gin_destroy(gin), "shmem_gin_destroy")


def gin_signal_sym(gin, signal_id):
    return _L.shmem_gin_signal_sym(gin, signal_id)


def gin_counter_sym(gin, counter_id):
    return _L.shmem_gin_counter_sym(gin, counter_id)


class PeTeam(C.Structure):
    _fields_ = [("start", C.c_uint32), ("stride", C.c_uint32), ("size", C.c_uint32), ("pad", C.c_uint32), ("words_off", C.c_uint64)]


def team_create(start, stride, size):
    t = _vp(0)
    _check(_L.shmem_team_create(start, stride, size, C.byref(t)), "shmem_team_create")
    return t


def team_destroy(team):
    return _check(_L.shmem_team_destroy(team), "shmem_team_destroy")


def team_device_state(team):
    st = PeTeam()
    _check(_L.shmem_team_device_state(team, C.byref(st)), "shmem_team_device_state")
    return st


def team_sync(team, wgs_per_pe=1):
    return _check(_L.shmem_team_sync(team, wgs_per_pe), "shmem_team_sync")


def team_epochs(teams, rounds, slots_sym, wgs_per_pe=1, dev_errors=None):
    n = len(teams)
    arr = (C.c_void_p * max(n, 1))(*[t.value if hasattr(t, "value") else t for t in teams])
    rr = (C.c_int * max(n, 1))(*rounds)
    return _check(_L.shmem_team_epochs(arr, rr, n, _addr(slots_sym), wgs_per_pe, _addr(dev_errors)), "shmem_team_epochs")


class DeviceCtx(C.Structure):
    _fields_ = [("heap", C.c_void_p), ("seg", C.c_uint64), ("scratch", C.c_void_p), ("npes", C.c_int)]


class GinState(C.Structure):
    _fields_ = [("signals_off", C.c_uint64), ("counters_off", C.c_uint64), ("nsignals", C.c_uint32), ("ncounters", C.c_uint32)]


def device_context():
    ctx = DeviceCtx()
    _check(_L.shmem_device_context(C.byref(ctx)), "shmem_device_context")
    return ctx


def gin_device_state(gin):
    st = GinState()
    _check(_L.shmem_gin_device_state(gin, C.byref(st)), "shmem_gin_device_state")
    return st


def ring_exchange(recv_sym, send_sym, slot_bytes, gin, signal_id=0, counter_id=0, rounds=1, wgs_per_pe=1):
    return _check(_L.shmem_ring_exchange(_addr(recv_sym), _addr(send_sym), slot_bytes, gin, signal_id, counter_id,
                                         rounds, wgs_per_pe), "shmem_ring_exchange")


def pingpong(buf_sym, nbytes, gin, signal_id, iters):
    return _check(_L.shmem_pingpong(_addr(buf_sym), nbytes, gin, signal_id, iters), "shmem_pingpong")


def barrier_epochs(slots_sym, rounds, wgs_per_pe, dev_errors=None):
    return _check(_L.shmem_barrier_epochs(_addr(slots_sym), rounds, wgs_per_pe, _addr(dev_errors)),
                  "shmem_barrier_epochs")


def fence_litmus(buf_sym, nbytes, rounds, use_quiet=0, dev_errors=None):
    return _check(_L.shmem_fence_litmus(_addr(buf_sym), nbytes, rounds, use_quiet, _addr(dev_errors)),
                  "shmem_fence_litmus")


def moe_create(num_experts, max_tokens, topk, hidden_bytes):
    m = _vp(0)
    _check(_L.shmem_moe_create(num_experts, max_tokens, topk, hidden_bytes, C.byref(m)), "shmem_moe_create")
    return m


def moe_destroy(moe):
    return _check(_L.shmem_moe_destroy(moe), "shmem_moe_destroy")


def moe_dispatch(moe, dev_x, dev_topk, dev_ntok, dev_recv_x, dev_recv_info, dev_recv_range, dev_recv_count,
                 wgs_per_pe):
    return _check(_L.shmem_moe_dispatch(moe, _addr(dev_x), _addr(dev_topk), _addr(dev_ntok), _addr(dev_recv_x),
                                        _addr(dev_recv_info), _addr(dev_recv_range), _addr(dev_recv_count),
                                        wgs_per_pe), "shmem_moe_dispatch")


def moe_combine(moe, dev_expert_out, dev_recv_info, dev_recv_range, dev_topk, dev_ntok, dev_combined, wgs_per_pe):
    return _check(_L.shmem_moe_combine(moe, _addr(dev_expert_out), _addr(dev_recv_info), _addr(dev_recv_range),
                                       _addr(dev_topk), _addr(dev_ntok), _addr(dev_combined), wgs_per_pe),
                  "shmem_moe_combine")


def proxy_create(queue_entries):
    p = _vp(0)
    _check(_L.shmem_proxy_create(queue_entries, C.byref(p)), "shmem_proxy_create")
    return p


def proxy_submit(proxy, dev_ops, n, workgroups=4):
    return _check(_L.shmem_proxy_submit(proxy, _addr(dev_ops), n, workgroups), "shmem_proxy_submit")


def proxy_quiet(proxy):
    """Waits until the proxy has carried out everything submitted; raises ShmemError(ERR_DEVICE_FAULT)
    with the first rejected ticket if it skipped a descriptor."""
    bad = C.c_uint64(0)
    rc = _L.shmem_proxy_quiet(proxy, C.byref(bad))
    if rc == ERR_DEVICE_FAULT:
        e = ShmemError(rc, f"shmem_proxy_quiet (first rejected ticket {bad.value})")
        e.first_bad_index = bad.value
        raise e
    return _check(rc, "shmem_proxy_quiet")


def proxy_stats(proxy):
    a, b, c = C.c_uint64(0), C.c_uint64(0), C.c_uint64(0)
    _check(_L.shmem_proxy_stats(proxy, C.byref(a), C.byref(b), C.byref(c)), "shmem_proxy_stats")
    return {"submitted": a.value, "executed": b.value, "rejected": c.value}


def proxy_destroy(proxy):
    return _check(_L.shmem_proxy_destroy(proxy), "shmem_proxy_destroy")


def transpose(out_sym, in_sym, n, elem_bytes, wgs_per_pe):
    return _check(_L.shmem_transpose(_addr(out_sym), _addr(in_sym), n, elem_bytes, wgs_per_pe), "shmem_transpose")

