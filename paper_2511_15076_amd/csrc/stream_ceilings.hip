// Plain-stream ceilings of the box: read-only, write-only and copy kernels with
// 16 bytes per lane over 2 GiB buffers, plus the runtime's own memcpy / memset.
// These are the sanity ceilings the put/get kernels are held against; this
// program is a measurement aid, not part of the library.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <vector>

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
#define CK(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__); exit(1); } } while (0)

__global__ __launch_bounds__(256) void k_read(const u32x4 *s, uint64_t nv, uint32_t *out)
{
    u32x4 acc = {0, 0, 0, 0};
    for (uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < nv; i += (uint64_t)gridDim.x * blockDim.x)
        acc ^= __builtin_nontemporal_load(s + i);
    if ((acc.x ^ acc.y ^ acc.z ^ acc.w) == 0x12345u) out[0] = 1;
}

__global__ __launch_bounds__(256) void k_write(u32x4 *d, uint64_t nv)
{
    const u32x4 v = {1, 2, 3, threadIdx.x};
    for (uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < nv; i += (uint64_t)gridDim.x * blockDim.x)
        __builtin_nontemporal_store(v, d + i);
}

template <int U>
__global__ __launch_bounds__(256) void k_copy(const u32x4 *s, u32x4 *d, uint64_t nv)
{
    const uint64_t tile = (uint64_t)blockDim.x * U;
    for (uint64_t t = blockIdx.x; t * tile < nv; t += gridDim.x) {
        u32x4 r[U];
#pragma unroll
        for (int j = 0; j < U; ++j) {
            const uint64_t i = t * tile + (uint64_t)j * blockDim.x + threadIdx.x;
            r[j] = i < nv ? __builtin_nontemporal_load(s + i) : u32x4{0, 0, 0, 0};
        }
#pragma unroll
        for (int j = 0; j < U; ++j) {
            const uint64_t i = t * tile + (uint64_t)j * blockDim.x + threadIdx.x;
            if (i < nv) __builtin_nontemporal_store(r[j], d + i);
        }
    }
}

template <typename F>
static float median_ms(F f, int reps = 9)
{
    hipEvent_t a, b;
    CK(hipEventCreate(&a)); CK(hipEventCreate(&b));
    f(); f();
    CK(hipDeviceSynchronize());
    std::vector<float> ms;
    for (int r = 0; r < reps; ++r) {
        CK(hipEventRecord(a)); f(); CK(hipEventRecord(b)); CK(hipEventSynchronize(b));
        float m; CK(hipEventElapsedTime(&m, a, b)); ms.push_back(m);
    }
    std::sort(ms.begin(), ms.end());
    CK(hipEventDestroy(a)); CK(hipEventDestroy(b));
    return ms[ms.size() / 2];
}

int main()
{
    const uint64_t bytes = 2ull << 30, nv = bytes / 16;
    uint8_t *buf; uint32_t *flag;
    CK(hipMalloc(&buf, 2 * bytes)); CK(hipMalloc(&flag, 4));
    CK(hipMemset(buf, 1, 2 * bytes));
    const u32x4 *s = (const u32x4 *)buf;
    u32x4 *d = (u32x4 *)(buf + bytes);
    printf("{");
    for (int g : {256, 1024, 2048, 4096}) {
        float ms = median_ms([&] { hipLaunchKernelGGL(k_read, dim3(g), dim3(256), 0, 0, s, nv, flag); });
        printf("\"read_grid%d_GBs\": %.0f, ", g, bytes / ms / 1e6);
        ms = median_ms([&] { hipLaunchKernelGGL(k_write, dim3(g), dim3(256), 0, 0, d, nv); });
        printf("\"write_grid%d_GBs\": %.0f, ", g, bytes / ms / 1e6);
        ms = median_ms([&] { hipLaunchKernelGGL(k_copy<4>, dim3(g), dim3(256), 0, 0, s, d, nv); });
        printf("\"copy_u4_grid%d_GBs\": %.0f, ", g, 2.0 * bytes / ms / 1e6);
        ms = median_ms([&] { hipLaunchKernelGGL(k_copy<1>, dim3(g), dim3(256), 0, 0, s, d, nv); });
        printf("\"copy_u1_grid%d_GBs\": %.0f, ", g, 2.0 * bytes / ms / 1e6);
    }
    float ms = median_ms([&] { CK(hipMemcpyAsync(d, s, bytes, hipMemcpyDeviceToDevice, 0)); });
    printf("\"hipMemcpyDtoD_GBs\": %.0f, ", 2.0 * bytes / ms / 1e6);
    ms = median_ms([&] { CK(hipMemsetAsync(d, 7, bytes, 0)); });
    printf("\"hipMemset_GBs\": %.0f, \"bytes_per_buffer\": %llu}\n", bytes / ms / 1e6, (unsigned long long)bytes);
    return 0;
}
