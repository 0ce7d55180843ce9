"""Helpers for the GPU parity tests: a torch-backed symmetric heap around the C ABI."""
import contextlib

import numpy as np
import torch

import paper_2511_15076_amd as sh


@contextlib.contextmanager
def shmem_world(npes, heap_bytes):
    """Initialises the library on a fresh zeroed heap; yields (heap tensor, base address)."""
    dev = torch.device("cuda:0")
    heap = torch.zeros(npes * heap_bytes, dtype=torch.uint8, device=dev)
    scratch = torch.zeros(sh.scratch_bytes(npes), dtype=torch.uint8, device=dev)
    sh.init(npes, heap_bytes, heap, scratch, torch.cuda.current_stream().cuda_stream)
    try:
        yield heap, heap.data_ptr()
    finally:
        sh.finalize()
        del heap, scratch


def to_dev(a: np.ndarray) -> torch.Tensor:
    a = np.ascontiguousarray(a)
    return torch.from_numpy(a.view(np.uint8).reshape(-1)).to("cuda:0")


def heaps_of(heap: torch.Tensor, npes: int) -> np.ndarray:
    torch.cuda.synchronize()
    return heap.cpu().numpy().reshape(npes, -1)


def dev_u8(n, fill=0):
    return torch.full((n,), fill, dtype=torch.uint8, device="cuda:0")


def as_np(t: torch.Tensor, dtype) -> np.ndarray:
    torch.cuda.synchronize()
    return t.cpu().numpy().view(dtype)
