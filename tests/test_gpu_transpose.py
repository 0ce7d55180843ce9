"""GPU parity for the distributed transpose: the LDS-tiled kernel (contiguous one-sided gets of tile
rows) against the oracle's formulation as strided igets, whole heaps compared byte for byte."""
import numpy as np
import pytest
import torch

import oracle
import workgen

pytestmark = pytest.mark.gpu

sh = pytest.importorskip("paper_2511_15076_amd")
from gpu_util import heaps_of, shmem_world  # noqa: E402


@pytest.mark.parametrize("npes,n,eb,wgs", [
    (1, 5, 4, 1), (2, 64, 4, 2), (4, 128, 8, 3), (3, 195, 4, 2),       # ragged tiles: 65 rows per PE
    (8, 1000, 4, 5), (16, 1024, 8, 4), (5, 70, 8, 1),
    (4, 320, 4, 3), (2, 392, 4, 2),                                    # 16-byte path with ragged 128-row and 64-column tiles
    (8, 1000, 4, 128), (4, 1544, 4, 256), (16, 2048, 4, 64), (8, 1024, 8, 128),   # launches of 1024 workgroups and more: 128 x 128 tiles for 4-byte elements, ragged both ways
])
def test_transpose_matches_igets(npes, n, eb, wgs):
    R = n // npes
    blk = (R * n * eb + 255) // 256 * 256
    hb = 2 * blk + 512
    init = np.stack([workgen.random_words(500 + p + n, hb // 8).view(np.uint8) for p in range(npes)])
    w = oracle.World(npes, hb, oracle.SHUFFLED, 6)
    for p in range(npes):
        w.heap(p)[:] = init[p]
    in_off, out_off = 0, blk + 256
    oracle.transpose(w, out_off, in_off, n, eb)
    with shmem_world(npes, hb) as (heap, base):
        heap.copy_(torch.from_numpy(init.reshape(-1)))
        sh.transpose(base + out_off, base + in_off, n, eb, wgs)
        sh.stream_sync()
        got = heaps_of(heap, npes)
    assert np.array_equal(got, w.heaps())
    assert not np.array_equal(got, init)


def test_transpose_as_benchmarked_sampled():
    # 8 PEs, 16384 x 16384 uint32 (1 GiB): the assembled result against numpy's transpose
    npes, n, eb, wgs = 8, 16384, 4, 256
    R = n // npes
    blk = R * n * eb
    with shmem_world(npes, 2 * blk) as (heap, base):
        heap.view(torch.int64).random_()
        h = heap.view(npes, 2 * blk)
        A = torch.cat([h[p, :blk].view(torch.int32).view(R, n) for p in range(npes)])
        sh.transpose(base + blk, base, n, eb, wgs)
        sh.stream_sync()
        B = torch.cat([h[p, blk:].view(torch.int32).view(R, n) for p in range(npes)])
        assert torch.equal(B, A.t())                      # the definition, evaluated by a library routine
        An = A[:70, :].cpu().numpy()                      # and a corner element by element on the CPU
        assert np.array_equal(B[:, :70].cpu().numpy(), An.T)


def test_transpose_argument_checks():
    with shmem_world(4, 1 << 20) as (heap, base):
        for args, st in [((base + 65536, base, 6, 4, 1), sh.ERR_INVALID_ARG),       # n not a multiple of npes
                         ((base + 65536, base, 8, 2, 1), sh.ERR_INVALID_ARG),       # element size
                         ((base + 65536, base, 8, 4, 0), sh.ERR_INVALID_ARG),
                         ((base + 32, base, 8, 4, 1), sh.ERR_INVALID_ARG),          # overlapping blocks
                         ((base + 65536, base + 2, 8, 4, 1), sh.ERR_ALIGN),
                         ((base + 65536, base, 4096, 4, 1), sh.ERR_OUT_OF_RANGE)]:
            with pytest.raises(sh.ShmemError) as ei:
                sh.transpose(*args)
            assert ei.value.status == st, args
        sh.transpose(base + 65536, base, 0, 4, 1)                                    # nothing to do
