// Device half of the proxy-style executor (Sec. III-C, "Proxy Backend"): GPU
// threads enqueue 64-byte operation descriptors into a ring in host memory
// with fire-and-forget stores; a host thread polls the ring and carries the
// operations out.  The ring is multi-producer without atomics: the descriptor
// with table index i of a submission takes ticket base + i, so the queue order
// is the table order whatever order the lanes run in.  A slot becomes valid
// when its flag reads ticket + 1 (written after the descriptor, behind a
// system-scope release) and reusable when the host's `head` has passed it.
#pragma once
#include "../../include/mi_shmem.h"
#include "../../include/mi_shmemx.hpp"

namespace shmemx {

struct ProxyQueue {            // by value to the kernel; all three arrays are pinned, GPU-mapped host memory
    shmem_op_desc *ring;       // `mask + 1` descriptors
    uint64_t *flags;           // flags[slot] == ticket + 1: descriptor `ticket` is complete in ring[slot]
    const uint64_t *head;      // descriptors the host thread has taken out so far
    uint64_t mask;             // entries - 1 (entries is a power of two)
};

__global__ __launch_bounds__(256) void k_proxy_submit(Ctx c, ProxyQueue q, const shmem_op_desc *ops, uint64_t n,
                                                      uint64_t base)
{
    const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
    uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    bool live = i < n;
    uint32_t spins = 0;
    // The lanes of a wave hold consecutive tickets, and with a ring shorter than a wave the higher lanes'
    // slots only become free after the host has taken out what the LOWER lanes of the same wave publish.
    // So no lane may wait inside a loop of its own: every pass of this wave-wide loop lets each lane look
    // at its slot once, and a lane publishes (descriptor, release, flag) in the pass in which it finds its
    // slot free, while the others go round again.
    while (ballot(live)) {
        if (live) {
            const uint64_t ticket = base + i, slot = ticket & q.mask;
            // flow control: the slot still holds descriptor ticket - entries until the host has taken it out
            if (ticket <= __hip_atomic_load(q.head, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM) + q.mask) {
                const u32x4 *s = (const u32x4 *)(ops + i);
                u32x4 *d = (u32x4 *)(q.ring + slot);
                const u32x4 a = s[0], b = s[1], e = s[2], f = s[3];
                d[0] = a; d[1] = b; d[2] = e; d[3] = f;                         // fire and forget: nothing is read back
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "");                   // system scope: the descriptor before its flag
                __hip_atomic_store(q.flags + slot, ticket + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
                i += stride;
                live = i < n;
                spins = 0;
            } else if (timed_out(c)) {
                live = false;
            } else {
                __builtin_amdgcn_s_sleep(8);
                if (++spins > SPIN_LIMIT) { report(c, DEV_ERR_BARRIER_TIMEOUT, i); live = false; }
            }
        }
    }
}

}  // namespace shmemx
