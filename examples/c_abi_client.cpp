// A client of the C ABI without Python or PyTorch: device memory from hipMalloc, the library's entry
// points called directly, results read back with hipMemcpy and checked on the host.  Built by
// paper_2511_15076_amd/build.py into examples/c_abi_client; tests/test_gpu_c_client.py runs it.
// Exit status 0 and a last line "c_abi_client ok" mean every check passed.
#include <hip/hip_runtime_api.h>

#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "mi_shmem.h"

#define HIP_OK(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__); return 2; } } while (0)
#define SHMEM_OK_OR_FAIL(x) do { int s_ = (x); if (s_ != SHMEM_OK) { printf("%s -> %s (%d) at line %d\n", #x, shmem_strerror(s_), s_, __LINE__); return 3; } } while (0)
#define CHECK(c) do { if (!(c)) { printf("check failed at line %d: %s\n", __LINE__, #c); return 4; } } while (0)

int main()
{
    const int npes = 4;
    const size_t seg = 1 << 20;
    uint8_t *heap = nullptr, *scratch = nullptr;
    uint64_t *dev_old = nullptr;
    HIP_OK(hipMalloc((void **)&heap, npes * seg));
    HIP_OK(hipMalloc((void **)&scratch, shmem_scratch_bytes(npes)));
    HIP_OK(hipMalloc((void **)&dev_old, 64));
    // every PE's segment starts as bytes (pe + 1) * 16 + (offset mod 13)
    std::vector<uint8_t> init(npes * seg);
    for (int p = 0; p < npes; ++p)
        for (size_t i = 0; i < seg; ++i) init[p * seg + i] = (uint8_t)((p + 1) * 16 + i % 13);
    HIP_OK(hipMemcpy(heap, init.data(), init.size(), hipMemcpyHostToDevice));

    CHECK(shmem_n_pes() == 0);
    CHECK(shmem_malloc(256) == nullptr);                                  // not initialised yet
    SHMEM_OK_OR_FAIL(shmem_init(npes, seg, heap, scratch, nullptr));      // the default stream
    CHECK(shmem_n_pes() == npes);
    CHECK(shmem_init(npes, seg, heap, scratch, nullptr) == SHMEM_ERR_ALREADY_INIT);

    uint8_t *a = (uint8_t *)shmem_malloc(8192), *b = (uint8_t *)shmem_malloc(4096);
    uint64_t *ctr = (uint64_t *)shmem_malloc(256);
    CHECK(a == heap && b == heap + 8192 && (uint8_t *)ctr == heap + 12288);   // first fit from the start of the segment
    CHECK(shmem_ptr(b, 3) == (void *)(b + 3 * seg));

    // PE 0 puts 5000 bytes of its `a` into PE 2's `a` at +100; PE 3 gets 1000 bytes of PE 1's `b`
    SHMEM_OK_OR_FAIL(shmem_put(0, a + 100, shmem_ptr(a, 0), 5000, 2));
    SHMEM_OK_OR_FAIL(shmem_get(3, (uint8_t *)shmem_ptr(b, 3) + 7, b + 11, 1000, 1));
    // every third uint32 of PE 1's `a` goes to consecutive uint32 of PE 0's `b`
    SHMEM_OK_OR_FAIL(shmem_iput(1, b, shmem_ptr(a, 1), 1, 3, 500, 4, 0));
    SHMEM_OK_OR_FAIL(shmem_quiet(-1));
    // counters: zero them on every PE, then fetch-add, compare-swap, fetch-or on PE 2's
    for (int p = 0; p < npes; ++p) HIP_OK(hipMemsetAsync(shmem_ptr(ctr, p), 0, 256, nullptr));
    SHMEM_OK_OR_FAIL(shmem_atomic_fetch_add(0, ctr, 5, 2, dev_old + 0));
    SHMEM_OK_OR_FAIL(shmem_atomic_fetch_add(1, ctr, 7, 2, dev_old + 1));
    SHMEM_OK_OR_FAIL(shmem_atomic_compare_swap(3, ctr + 1, 0, 99, 2, dev_old + 2));
    SHMEM_OK_OR_FAIL(shmem_atomic_compare_swap(0, ctr + 1, 0, 42, 2, dev_old + 3));   // loses: sees 99
    SHMEM_OK_OR_FAIL(shmem_atomic_fetch_or(2, ctr + 2, 0xF0, 2, dev_old + 4));
    // put with a signal: 1000 bytes of PE 0's `a` into PE 1's `a` at +6000, then 9 is added to PE 1's fourth counter
    SHMEM_OK_OR_FAIL(shmem_put_signal(0, a + 6000, shmem_ptr(a, 0), 1000, ctr + 3, 9, 1));
    // a team of PEs 0 and 2 and one barrier of it (its 256 bytes of the heap are the library's own)
    shmem_team_t team = nullptr;
    shmem_pe_team team_state;
    SHMEM_OK_OR_FAIL(shmem_team_create(0, 2, 2, &team));
    SHMEM_OK_OR_FAIL(shmem_team_device_state(team, &team_state));
    CHECK(team_state.start == 0 && team_state.stride == 2 && team_state.size == 2 && team_state.words_off == 12544);
    SHMEM_OK_OR_FAIL(shmem_team_sync(team, 2));
    CHECK(shmem_team_create(1, 2, 3, &team) == SHMEM_ERR_INVALID_PE);     // 1, 3, 5: there is no PE 5
    SHMEM_OK_OR_FAIL(shmem_barrier_all());
    uint64_t first_bad = 0;
    SHMEM_OK_OR_FAIL(shmem_stream_sync(&first_bad));

    // host-visible errors enqueue nothing
    CHECK(shmem_put(0, a, shmem_ptr(a, 0), 16, npes) == SHMEM_ERR_INVALID_PE);
    CHECK(shmem_put(0, a + seg - 8, shmem_ptr(b, 0), 16, 1) == SHMEM_ERR_OUT_OF_RANGE);
    CHECK(shmem_iput(0, a + 2, shmem_ptr(b, 0), 1, 1, 4, 4, 1) == SHMEM_ERR_ALIGN);
    CHECK(shmem_free(a + 64) == SHMEM_ERR_BAD_FREE);

    std::vector<uint8_t> got(npes * seg);
    uint64_t old[5];
    HIP_OK(hipMemcpy(got.data(), heap, got.size(), hipMemcpyDeviceToHost));
    HIP_OK(hipMemcpy(old, dev_old, sizeof old, hipMemcpyDeviceToHost));
    // expected heap: the same operations on the host copy
    std::vector<uint8_t> want = init;
    memcpy(&want[2 * seg + 100], &init[0 * seg + 0], 5000);
    memcpy(&want[3 * seg + 8192 + 7], &init[1 * seg + 8192 + 11], 1000);
    for (int i = 0; i < 500; ++i) memcpy(&want[0 * seg + 8192 + 4 * i], &init[1 * seg + 12 * i], 4);
    for (int p = 0; p < npes; ++p) memset(&want[p * seg + 12288], 0, 256);
    uint64_t c0 = 12, c1 = 99, c2 = 0xF0;
    memcpy(&want[2 * seg + 12288], &c0, 8); memcpy(&want[2 * seg + 12296], &c1, 8); memcpy(&want[2 * seg + 12304], &c2, 8);
    memcpy(&want[1 * seg + 6000], &init[0 * seg + 0], 1000);
    uint64_t c3 = 9;
    memcpy(&want[1 * seg + 12288 + 24], &c3, 8);
    for (int p = 0; p < npes; ++p) {                                      // the team's words: not ours to predict
        memset(&want[p * seg + 12544], 0, 256);
        memset(&got[p * seg + 12544], 0, 256);
    }
    size_t bad = 0;
    for (size_t i = 0; i < want.size(); ++i) bad += want[i] != got[i];
    CHECK(bad == 0);
    CHECK(old[0] == 0 && old[1] == 5 && old[2] == 0 && old[3] == 99 && old[4] == 0);   // one stream: the calls ran in order

    SHMEM_OK_OR_FAIL(shmem_team_destroy(team));
    SHMEM_OK_OR_FAIL(shmem_free(b));
    SHMEM_OK_OR_FAIL(shmem_free(a));
    SHMEM_OK_OR_FAIL(shmem_free(ctr));
    CHECK(shmem_malloc(seg) == (void *)heap);                                // everything came back
    SHMEM_OK_OR_FAIL(shmem_finalize());
    CHECK(shmem_finalize() == SHMEM_ERR_NOT_INIT);
    HIP_OK(hipFree(dev_old)); HIP_OK(hipFree(scratch)); HIP_OK(hipFree(heap));
    printf("c_abi_client ok\n");
    return 0;
}
