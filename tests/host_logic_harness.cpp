// CPU driver for the library's HIP-free host logic (csrc/host_logic.hpp): reads commands from stdin,
// prints one result per line.  Built and run by tests/test_host_logic_cpu.py.
//   I base seg            reset the allocator
//   A alignment nbytes    -> offset or -1
//   F offset              -> 1 released / 0 not a live block
//   N                     -> live blocks, free blocks
//   C npes seg pe_self pe sym_off nbytes                                     -> status of a put / get
//   S npes seg pe_self pe sym_off sym_stride local_addr local_stride nelems eb -> status of an iput / iget
//   M npes seg pe_self pe sym_off                                            -> status of an atomic
//   V npes seg kind pe_self pe elem_bytes local_off sym_off count local_stride sym_stride  -> 1 valid / 0
#include <cinttypes>
#include <cstdio>
#include <cstring>

#include "../paper_2511_15076_amd/csrc/host_logic.hpp"

int main()
{
    hostlogic::SymAllocator alloc;
    char cmd;
    while (scanf(" %c", &cmd) == 1) {
        if (cmd == 'I') {
            uint64_t base, seg;
            if (scanf("%" SCNu64 " %" SCNu64, &base, &seg) != 2) return 2;
            alloc.reset(base, seg);
            puts("0");
        } else if (cmd == 'A') {
            uint64_t al, n;
            if (scanf("%" SCNu64 " %" SCNu64, &al, &n) != 2) return 2;
            const uint64_t off = alloc.align(al, n);
            if (off == UINT64_MAX) puts("-1"); else printf("%" PRIu64 "\n", off);
        } else if (cmd == 'F') {
            uint64_t off;
            if (scanf("%" SCNu64, &off) != 1) return 2;
            puts(alloc.release(off) ? "1" : "0");
        } else if (cmd == 'N') {
            printf("%zu %zu\n", alloc.live_blocks(), alloc.free_blocks());
        } else if (cmd == 'C' || cmd == 'S' || cmd == 'M') {
            int npes, me, pe; uint64_t seg, off;
            if (scanf("%d %" SCNu64 " %d %d %" SCNu64, &npes, &seg, &me, &pe, &off) != 5) return 2;
            if (cmd == 'C') {
                uint64_t n;
                if (scanf("%" SCNu64, &n) != 1) return 2;
                printf("%d\n", hostlogic::check_contig(npes, seg, me, pe, off, n));
            } else if (cmd == 'S') {
                int64_t ss, ls; uint64_t la, n, eb;
                if (scanf("%" SCNd64 " %" SCNu64 " %" SCNd64 " %" SCNu64 " %" SCNu64, &ss, &la, &ls, &n, &eb) != 5) return 2;
                printf("%d\n", hostlogic::check_strided(npes, seg, me, pe, off, (ptrdiff_t)ss, la, (ptrdiff_t)ls, (size_t)n, (size_t)eb));
            } else {
                printf("%d\n", hostlogic::check_amo(npes, seg, me, pe, off));
            }
        } else if (cmd == 'V') {
            uint32_t npes; uint64_t seg;
            shmem_op_desc d;
            memset(&d, 0, sizeof d);
            if (scanf("%" SCNu32 " %" SCNu64 " %" SCNu32 " %" SCNu32 " %" SCNu32 " %" SCNu32 " %" SCNu64 " %" SCNu64 " %" SCNu64
                      " %" SCNd64 " %" SCNd64, &npes, &seg, &d.kind, &d.pe_self, &d.pe, &d.elem_bytes, &d.local_off, &d.sym_off,
                      &d.count, &d.local_stride, &d.sym_stride) != 11) return 2;
            puts(hostlogic::desc_valid(d, npes, seg) ? "1" : "0");
        } else {
            return 3;
        }
    }
    return 0;
}
