"""The executor entry point that allocates nothing (its barrier and fault words live in the library's code object)
against the ordinary one: same table, same heap afterwards, bit for bit; two calls in a row, the second smaller."""
import numpy as np
import pytest
import torch

import workgen

pytestmark = pytest.mark.gpu
sh = pytest.importorskip("paper_2511_15076_amd")
from gpu_util import heaps_of, shmem_world  # noqa: E402


def run_ordinary(npes, hb, init, ops, quiet_every, wgs):
    with shmem_world(npes, hb) as (heap, base):
        heap.copy_(torch.from_numpy(init.reshape(-1)))
        sh.op_batch(torch.from_numpy(ops.view(np.uint8).reshape(-1)).to("cuda:0"), len(ops), quiet_every, wgs)
        sh.stream_sync()
        return heaps_of(heap, npes)


def run_noalloc(npes, hb, init, ops, quiet_every, wgs):
    dev = torch.device("cuda:0")
    heap = torch.zeros(npes * hb, dtype=torch.uint8, device=dev)
    heap.copy_(torch.from_numpy(init.reshape(-1)))
    d_ops = torch.from_numpy(ops.view(np.uint8).reshape(-1)).to(dev)
    fault = torch.full((2,), 7, dtype=torch.int64, device=dev)
    sh.op_batch_noalloc(npes, hb, heap, d_ops, len(ops), quiet_every, wgs, fault, torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    return heaps_of(heap, npes), fault.cpu().numpy()


def test_noalloc_executor_matches_the_ordinary_one_twice():
    rng = np.random.default_rng(5)
    for npes, hb, nops, quiet_every, wgs, seed in ((4, 1 << 20, 10000, 100, 2, 251115077), (2, 1 << 18, 700, 50, 1, 99)):
        init = rng.integers(0, 256, size=(npes, hb), dtype=np.uint8)
        ops = workgen.cfg1_op_table(seed=seed, npes=npes, heap_bytes=hb, nops=nops)
        want = run_ordinary(npes, hb, init, ops, quiet_every, wgs)
        got, fault = run_noalloc(npes, hb, init, ops, quiet_every, wgs)
        assert np.array_equal(got, want)
        assert not np.array_equal(got, init)
        assert fault.tolist() == [0, 0]


def test_noalloc_executor_reports_a_bad_descriptor_and_rejects_what_it_cannot_hold():
    npes, hb = 2, 1 << 16
    ops = workgen.cfg1_op_table(seed=3, npes=npes, heap_bytes=hb, nops=64)
    ops = ops.copy()
    ops["pe"][10] = 9                                     # no such PE: skipped on the device, recorded
    init = np.zeros((npes, hb), dtype=np.uint8)
    got, fault = run_noalloc(npes, hb, init, ops, 0, 1)
    assert fault.tolist() == [1, 10]
    heap = torch.zeros(65 * 256, dtype=torch.uint8, device="cuda:0")
    with pytest.raises(sh.ShmemError) as e:
        sh.op_batch_noalloc(65, 256, heap, None, 0, 0, 1, None, torch.cuda.current_stream().cuda_stream)
    assert e.value.status == sh.ERR_OUT_OF_RANGE
