// Plain-stream ceilings of the box: read-only, write-only and copy kernels with
// 16 bytes per lane over 2 GiB buffers, plus the runtime's own memcpy / memset.
// These are the sanity ceilings the put/get kernels are held against.  Also the
// random-access ceilings the AMO, hash and BFS kernels are held against: random
// 8-byte reads over footprints from L2-resident to HBM-sized, returning 64-bit
// atomics to distinct lines (R_indep) and to one address (R_same).  Also the
// mixed read / write ceilings of a copy: wave-specialised workgroups (reader
// waves filling an LDS ring with global-load-to-LDS, writer waves draining it)
// over a sweep of reader waves, writer waves, stage size and ring depth, all
// unpaced, and the library's own streaming copy at a sweep of paces.  This
// program is a measurement aid, not part of the library.
#include <hip/hip_runtime.h>

#include "paper_2511_15076_amd/csrc/kernels_stream.hpp"   // the library's streaming copy, measured here at several paces

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

// Copy with a three-deep software pipeline per wave: each wave owns every (waves)-th 4 KiB task, keeps two
// tasks' loads in flight while it stores a third.  With one workgroup per CU this is the fastest plain copy
// found on the box.  The host sizes the copy so that every wave has a whole number of rounds of three.
__global__ __launch_bounds__(256) void k_copy_pipe(const uint8_t *__restrict__ src, uint8_t *__restrict__ dst, uint64_t tasks)
{
    constexpr int D = 3, VPL = 4;
    constexpr uint64_t TASK = 1024ull * VPL;
    const uint64_t waves = (uint64_t)gridDim.x * 4, my = (uint64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    const uint32_t lo = (threadIdx.x & 63) * 16;
    const uint64_t mine = tasks / waves;
    u32x4 v[D][VPL];
#pragma unroll
    for (int d = 0; d < D - 1; ++d)
#pragma unroll
        for (int j = 0; j < VPL; ++j) v[d][j] = __builtin_nontemporal_load((const u32x4 *)(src + (my + d * waves) * TASK + lo) + 64 * j);
    for (uint64_t r = 0; r < mine; r += D) {
#pragma unroll
        for (int d = 0; d < D; ++d) {
            const uint64_t ahead = r + d + D - 1;            // its loads go into the register set stored last
            if (ahead < mine) {
#pragma unroll
                for (int j = 0; j < VPL; ++j)
                    v[(d + D - 1) % D][j] = __builtin_nontemporal_load((const u32x4 *)(src + (my + ahead * waves) * TASK + lo) + 64 * j);
            }
#pragma unroll
            for (int j = 0; j < VPL; ++j) __builtin_nontemporal_store(v[d][j], (u32x4 *)(dst + (my + (r + d) * waves) * TASK + lo) + 64 * j);
        }
    }
}

// counter-based index stream (SplitMix64 finaliser of the global op number)
__device__ __forceinline__ uint64_t mix(uint64_t z)
{
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

// n random reads of one T (8 or 4 bytes) over `words` words of that size (a power of two), PER independent
// reads in flight per lane
template <int PER, typename T = uint64_t, bool NT = false>
__global__ __launch_bounds__(256) void k_randread(const T *a, uint64_t words, uint64_t n, uint32_t *out)
{
    T acc = 0;
    const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
    for (uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride * PER) {
        T v[PER];
#pragma unroll
        for (int k = 0; k < PER; ++k) {
            const T *p = a + (mix(i + k * stride) & (words - 1));
            v[k] = NT ? __builtin_nontemporal_load(p) : *p;
        }
#pragma unroll
        for (int k = 0; k < PER; ++k) acc ^= v[k];
    }
    if (acc == 0x12345u) out[0] = 1;
}

// n returning 64-bit fetch-adds (agent scope): word = 16 * (random line index) so that every op has its
// own 128-byte line when `lines` is large, or all ops hit word 0 when lines == 1
__global__ __launch_bounds__(256) void k_atomics(uint64_t *a, uint64_t lines, uint64_t n, uint32_t *out)
{
    uint64_t acc = 0;
    const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
    for (uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride)
        acc ^= __hip_atomic_fetch_add(a + 16 * (mix(i) & (lines - 1)), 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (acc == 0x12345u) out[0] = 1;
}

// ---------------------------------------------------------------------------
// Mixed ceiling: one workgroup per compute unit, `nr` reader waves that load `lps` KiB each per stage
// straight into an LDS ring of `S` stages, `nwr` writer waves that store a stage from the ring; one
// s_barrier per stage, nothing paced (every load goes out as soon as a ring slot is free).  Workgroup b
// takes stages b, b + grid, ...
struct MixedParams { const uint8_t *src; uint8_t *dst; uint32_t nr, nwr, lps, S, steps; };

__device__ __forceinline__ void wait_vm(uint32_t n)      // s_waitcnt vmcnt(n), n a run-time value
{
    switch (n) {
#define C1(n) case n: ST_WAIT_VM(n); break;
#define C8(b) C1(b) C1(b + 1) C1(b + 2) C1(b + 3) C1(b + 4) C1(b + 5) C1(b + 6) C1(b + 7)
        C8(0) C8(8) C8(16) C8(24) C8(32) C8(40) C8(48)
        C1(56) C1(57) C1(58) C1(59) C1(60) C1(61) C1(62)
    default: ST_WAIT_VM(63); break;
    }
}

__global__ __launch_bounds__(1024) void k_mixed(MixedParams p)
{
    extern __shared__ __attribute__((aligned(16))) uint8_t mixed_ring[];
    const uint32_t lane = threadIdx.x & 63;
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const uint32_t stage_bytes = p.nr * p.lps * 1024, T = p.steps, S = p.S;
    if (wave < p.nr) {
        const uint32_t my = wave * p.lps * 1024;
        auto issue = [&](uint32_t t) {
            const uint8_t *g = p.src + ((uint64_t)t * gridDim.x + blockIdx.x) * stage_bytes + my + lane * 16;
            uint8_t *l = mixed_ring + (t % S) * stage_bytes + my;
            for (uint32_t i = 0; i < p.lps; ++i)
                __builtin_amdgcn_global_load_lds((shmemx::glb_ptr_t)(g + i * 1024), (shmemx::lds_ptr_t)(l + i * 1024), 16, 0, 2);
        };
        const uint32_t pro = S - 1 < T ? S - 1 : T;
        for (uint32_t t = 0; t < pro; ++t) issue(t);
        for (uint32_t t = 0; t < T; ++t) {
            const uint32_t later = S - 2 < T - 1 - t ? S - 2 : T - 1 - t;
            wait_vm(later * p.lps);
            asm volatile("" ::: "memory");
            __builtin_amdgcn_s_barrier();
            asm volatile("" ::: "memory");
            if (t + S - 1 < T) issue(t + S - 1);
        }
    } else {
        const uint32_t w = wave - p.nr, per = stage_bytes / p.nwr, n = per / 1024;
        for (uint32_t t = 0; t < T; ++t) {
            asm volatile("" ::: "memory");
            __builtin_amdgcn_s_barrier();
            asm volatile("" ::: "memory");
            const u32x4 *l = (const u32x4 *)(mixed_ring + (t % S) * stage_bytes + w * per) + lane;
            u32x4 *g = (u32x4 *)(p.dst + ((uint64_t)t * gridDim.x + blockIdx.x) * stage_bytes + w * per) + lane;
            for (uint32_t j = 0; j < n; ++j) __builtin_nontemporal_store(l[j * 64], g + j * 64);
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
    CK(hipMalloc(&buf, 3 * bytes)); CK(hipMalloc(&flag, 4));     // the third buffer: room to displace the destination
    CK(hipMemset(buf, 1, 3 * bytes));
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
    // the pipelined copy, one workgroup per CU, and how its rate depends on WHERE the destination lies
    // relative to the source: destination = source + 2 GiB + one more address bit (the reads and the
    // writes of a moment then meet, or do not meet, in the same channels and banks)
    const uint64_t ptasks = bytes / 4096 / (256 * 4 * 3) * (256 * 4 * 3);
    printf("\"copy_pipelined_grid256_GBs_by_extra_delta_bit\": {");
    for (int bit = 11; bit <= 30; ++bit) {
        const uint64_t shift = bit == 11 ? 0 : 1ull << bit;
        float pms = median_ms([&] { hipLaunchKernelGGL(k_copy_pipe, dim3(256), dim3(256), 0, 0, buf, buf + bytes + shift, ptasks); });
        char key[16];
        if (bit == 11) snprintf(key, sizeof key, "none"); else snprintf(key, sizeof key, "%d", bit);
        printf("\"%s\": %.0f%s", key, 2.0 * ptasks * 4096 / pms / 1e6, bit == 30 ? "}, " : ", ");
    }
    // mixed read + write ceilings, unpaced: (reader waves, writer waves, KiB per reader per stage, ring stages)
    CK(hipFuncSetAttribute((const void *)k_mixed, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024));
    printf("\"copy_wave_specialised_unpaced_GBs\": {");
    {
        bool first = true;
        float best = 0;
        for (uint32_t nr : {2u, 4u, 8u, 12u})
            for (uint32_t nwr : {1u, 2u, 4u})
                for (uint32_t lps : {1u, 2u, 4u, 8u})
                    for (uint32_t S : {4u, 8u, 16u}) {
                        const uint32_t stage = nr * lps * 1024;
                        if (stage * S > 160 * 1024 || (nr * lps) % nwr || (S - 2) * lps > 63 || stage * (S - 1) < 16 * 1024) continue;
                        MixedParams mp{buf, buf + bytes, nr, nwr, lps, S, (uint32_t)(bytes / stage / 256)};
                        float mms = median_ms([&] { hipLaunchKernelGGL(k_mixed, dim3(256), dim3((nr + nwr) * 64), stage * S, 0, mp); }, 5);
                        const float gbs = 2.0 * mp.steps * 256.0 * stage / mms / 1e6;
                        best = std::max(best, gbs);
                        printf("%s\"r%u_w%u_stage%uKiB_ring%u\": %.0f", first ? "" : ", ", nr, nwr, stage >> 10, S, gbs);
                        first = false;
                    }
        printf(", \"best\": %.0f}, ", best);
    }
    // the library's streaming copy (4 reader waves, 2 writer waves, 4 KiB tasks, ring of 16) on one 2 GiB stream,
    // by pace: ns per task and workgroup with 256 workgroups (0 = unpaced); median and worst of 15 launches
    {
        int khz = 100000;
        (void)hipDeviceGetAttribute(&khz, hipDeviceAttributeWallClockRate, 0);
        printf("\"copy_streaming_one_stream_GBs_by_pace_ns\": {");
        bool first = true;
        for (double pace : {0.0, 290.0, 300.0, 308.0, 315.0, 322.0, 330.0, 340.0, 360.0}) {
            const uint32_t period = (uint32_t)(pace * khz / 1e6 * 256.0 + 0.5);
            const uint32_t chunks = (uint32_t)(bytes / shmemx::ST_CHUNK);
            std::vector<float> v;
            hipEvent_t a, b;
            CK(hipEventCreate(&a)); CK(hipEventCreate(&b));
            for (int r = 0; r < 17; ++r) {
                CK(hipEventRecord(a));
                hipLaunchKernelGGL(shmemx::k_copy_stream_lds, dim3(256), dim3(shmemx::ST_THREADS), 0, 0, buf + bytes, buf, chunks, period);
                CK(hipEventRecord(b)); CK(hipEventSynchronize(b));
                float m; CK(hipEventElapsedTime(&m, a, b));
                if (r >= 2) v.push_back(m);
            }
            std::sort(v.begin(), v.end());
            printf("%s\"%.0f\": {\"median\": %.0f, \"worst\": %.0f}", first ? "" : ", ", pace, 2.0 * bytes / v[v.size() / 2] / 1e6, 2.0 * bytes / v.back() / 1e6);
            first = false;
            CK(hipEventDestroy(a)); CK(hipEventDestroy(b));
        }
        printf("}, ");
    }
    float ms = median_ms([&] { CK(hipMemcpyAsync(d, s, bytes, hipMemcpyDeviceToDevice, 0)); });
    printf("\"hipMemcpyDtoD_GBs\": %.0f, ", 2.0 * bytes / ms / 1e6);
    ms = median_ms([&] { CK(hipMemsetAsync(d, 7, bytes, 0)); });
    printf("\"hipMemset_GBs\": %.0f, \"bytes_per_buffer\": %llu, ", bytes / ms / 1e6, (unsigned long long)bytes);
    // random 8-byte reads: 2 MiB (one die's L2 holds it), 16 MiB, 1 GiB and 2 GiB footprints
    const uint64_t nops = 1ull << 28;
    for (uint64_t fp : {2ull << 20, 16ull << 20, 1ull << 30, 2ull << 30}) {
        ms = median_ms([&] { hipLaunchKernelGGL((k_randread<4, uint64_t>), dim3(4096), dim3(256), 0, 0, (const uint64_t *)buf, fp / 8, nops, flag); }, 5);
        printf("\"randread8_%lluMiB_Gops\": %.1f, ", (unsigned long long)(fp >> 20), nops / ms / 1e6);
    }
    // the L2-resident footprint again: 4-byte reads, and 8 reads in flight per lane
    ms = median_ms([&] { hipLaunchKernelGGL((k_randread<4, uint32_t>), dim3(4096), dim3(256), 0, 0, (const uint32_t *)buf, (2ull << 20) / 4, nops, flag); }, 5);
    printf("\"randread4_2MiB_Gops\": %.1f, ", nops / ms / 1e6);
    ms = median_ms([&] { hipLaunchKernelGGL((k_randread<8, uint64_t>), dim3(4096), dim3(256), 0, 0, (const uint64_t *)buf, (2ull << 20) / 8, nops, flag); }, 5);
    printf("\"randread8_2MiB_8inflight_Gops\": %.1f, ", nops / ms / 1e6);
    // the HBM-sized footprint with non-temporal loads (does the L2 still fetch whole 128-byte lines?)
    ms = median_ms([&] { hipLaunchKernelGGL((k_randread<4, uint64_t, true>), dim3(4096), dim3(256), 0, 0, (const uint64_t *)buf, (1ull << 30) / 8, nops, flag); }, 5);
    printf("\"randread8_1024MiB_nontemporal_Gops\": %.1f, ", nops / ms / 1e6);
    // returning atomics: distinct 128-byte lines over 1 GiB, over 8 MiB (64 Ki lines), and one address
    const uint64_t natom = 1ull << 26;
    CK(hipMemset(buf, 0, bytes));
    ms = median_ms([&] { hipLaunchKernelGGL(k_atomics, dim3(4096), dim3(256), 0, 0, (uint64_t *)buf, (1ull << 30) / 128, natom, flag); }, 5);
    printf("\"atomic_indep_1GiB_Gops\": %.2f, ", natom / ms / 1e6);
    ms = median_ms([&] { hipLaunchKernelGGL(k_atomics, dim3(4096), dim3(256), 0, 0, (uint64_t *)buf, 1ull << 16, natom, flag); }, 5);
    printf("\"atomic_indep_8MiB_Gops\": %.2f, ", natom / ms / 1e6);
    const uint64_t nsame = 1ull << 22;
    ms = median_ms([&] { hipLaunchKernelGGL(k_atomics, dim3(1024), dim3(256), 0, 0, (uint64_t *)buf, 1ull, nsame, flag); }, 5);
    printf("\"atomic_same_address_Gops\": %.3f}\n", nsame / ms / 1e6);
    return 0;
}
