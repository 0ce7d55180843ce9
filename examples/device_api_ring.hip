// A kernel of the caller's own on the device API (include/mi_shmem_device.hpp): a ring exchange in the
// manner of Listing 2 of the paper, written outside the library.  PE r puts slice `peer` of its send
// buffer into slice r of the receive buffer of peer = (r + 1) mod n with a SignalAdd of the byte count,
// waits until its own signal shows that many bytes, works on what it received (adds 1 to every word:
// the data must be visible for that), and acknowledges to its predecessor with a putValue.  The host
// side uses the C ABI only.  Built by paper_2511_15076_amd/build.py; tests/test_gpu_c_client.py runs it.
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstdio>
#include <vector>

#include "mi_shmem.h"
#include "mi_shmem_device.hpp"

#define HIP_OK(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__); return 2; } } while (0)
#define SHMEM_OK_OR_FAIL(x) do { int s_ = (x); if (s_ != SHMEM_OK) { printf("%s -> %s (%d) at line %d\n", #x, shmem_strerror(s_), s_, __LINE__); return 3; } } while (0)
#define CHECK(c) do { if (!(c)) { printf("check failed at line %d: %s\n", __LINE__, #c); return 4; } } while (0)

__global__ __launch_bounds__(256) void my_ring(shmemx::Ctx c, shmemx::GinState gs, uint64_t send_off, uint64_t recv_off,
                                               uint64_t ack_off, uint64_t ds, uint32_t wgs_per_pe)
{
    const uint32_t pe = blockIdx.x / wgs_per_pe, wg = blockIdx.x % wgs_per_pe;
    const shmemx::Gin gin{c, gs, pe, wgs_per_pe};
    const uint32_t n = (uint32_t)c.npes, peer = (pe + 1) % n, pred = (pe + n - 1) % n;
    shmemx::GinActions act;
    act.signal_id = 0;
    act.signal_value = ds;                                   // SignalAdd{0, bytes}
    gin.put(peer, recv_off + (uint64_t)pe * ds, send_off + (uint64_t)peer * ds, ds, act);
    gin.wait_signal(0, ds);                                  // the predecessor's slice is in and visible
    uint32_t *slice = (uint32_t *)shmemx::ptr(c, recv_off + (uint64_t)pred * ds, pe);
    for (uint64_t i = (uint64_t)wg * blockDim.x + threadIdx.x; i < ds / 4; i += (uint64_t)wgs_per_pe * blockDim.x) slice[i] += 1;
    if (wg == 0 && threadIdx.x == 0) gin.put_value(pred, ack_off, ds / 4);   // "I have worked through so many words of yours"
    gin.barrier_sync();                                      // quiet + barrier over all PEs
}

int main()
{
    const int npes = 4, wgs_per_pe = 2;
    const size_t seg = 1 << 20, ds = 20000;                  // 5000 words per slice
    uint8_t *heap = nullptr, *scratch = nullptr;
    HIP_OK(hipMalloc((void **)&heap, npes * seg));
    HIP_OK(hipMalloc((void **)&scratch, shmem_scratch_bytes(npes)));
    HIP_OK(hipMemset(heap, 0, npes * seg));
    SHMEM_OK_OR_FAIL(shmem_init(npes, seg, heap, scratch, nullptr));
    uint8_t *send = (uint8_t *)shmem_malloc(npes * ds), *recv = (uint8_t *)shmem_malloc(npes * ds);
    uint64_t *ack = (uint64_t *)shmem_malloc(256);
    void *gin = nullptr;
    CHECK(send && recv && ack);
    SHMEM_OK_OR_FAIL(shmem_gin_create(1, 0, &gin));
    // send buffer of PE p: word i of slice q = p * 1000000 + q * 10000 + i
    std::vector<uint32_t> h(npes * ds / 4);
    for (int p = 0; p < npes; ++p) {
        for (int q = 0; q < npes; ++q)
            for (size_t i = 0; i < ds / 4; ++i) h[q * (ds / 4) + i] = (uint32_t)(p * 1000000 + q * 10000 + i);
        HIP_OK(hipMemcpy(shmem_ptr(send, p), h.data(), npes * ds, hipMemcpyHostToDevice));
    }
    shmem_device_ctx hc;
    shmem_gin_state hs;
    SHMEM_OK_OR_FAIL(shmem_device_context(&hc));
    SHMEM_OK_OR_FAIL(shmem_gin_device_state(gin, &hs));
    shmemx::Ctx c{(uint8_t *)hc.heap, hc.seg, hc.scratch, hc.npes};
    shmemx::GinState gs{hs.signals_off, hs.counters_off, hs.nsignals, hs.ncounters};
    hipLaunchKernelGGL(my_ring, dim3(npes * wgs_per_pe), dim3(256), 0, nullptr, c, gs, (uint64_t)(send - heap), (uint64_t)(recv - heap),
                       (uint64_t)((uint8_t *)ack - heap), (uint64_t)ds, (uint32_t)wgs_per_pe);
    HIP_OK(hipGetLastError());
    uint64_t first_bad = 0;
    SHMEM_OK_OR_FAIL(shmem_stream_sync(&first_bad));         // also: no wait timed out, nothing was rejected

    for (int p = 0; p < npes; ++p) {
        const int q = (p + npes - 1) % npes;                 // p received slice p of q's send buffer, into slot q
        HIP_OK(hipMemcpy(h.data(), shmem_ptr(recv, p), npes * ds, hipMemcpyDeviceToHost));
        for (int slot = 0; slot < npes; ++slot)
            for (size_t i = 0; i < ds / 4; ++i) {
                const uint32_t want = slot == q ? (uint32_t)(q * 1000000 + p * 10000 + i) + 1 : 0;
                CHECK(h[slot * (ds / 4) + i] == want);
            }
        uint64_t word = 0;
        HIP_OK(hipMemcpy(&word, shmem_ptr(ack, p), 8, hipMemcpyDeviceToHost));
        CHECK(word == ds / 4);                               // the successor's acknowledgement
        HIP_OK(hipMemcpy(&word, shmem_ptr(shmem_gin_signal_sym(gin, 0), p), 8, hipMemcpyDeviceToHost));
        CHECK(word == ds);                                   // SignalAdd of the byte count, not reset
    }
    SHMEM_OK_OR_FAIL(shmem_gin_destroy(gin));
    SHMEM_OK_OR_FAIL(shmem_finalize());
    HIP_OK(hipFree(scratch)); HIP_OK(hipFree(heap));
    printf("device_api_ring ok\n");
    return 0;
}
