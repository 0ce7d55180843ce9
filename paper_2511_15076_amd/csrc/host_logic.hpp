// Host-side logic of the library that needs no device: the symmetric-heap allocator and the validation
// of 64-byte op descriptors.  Plain C++ (no HIP), so that the CPU tests can compile and drive exactly
// the code the library runs.
#pragma once
#include <algorithm>
#include <cstddef>
#include <cstdint>
#include <vector>

#include "../../include/mi_shmem.h"

namespace hostlogic {

constexpr uint64_t GRAN = 256;   // allocator granularity / minimum alignment

// First-fit allocator over one PE's segment [0, seg): offsets are the same on every PE (a symmetric
// allocation is one offset).  Free blocks are kept address-ordered and merged with their neighbours.
class SymAllocator {
public:
    struct Block { uint64_t off, len; };

    // base = device address of PE 0's segment: alignments are those of the resulting address
    void reset(uint64_t base, uint64_t seg)
    {
        base_ = base; seg_ = seg;
        free_.assign(1, Block{0, seg});
        live_.clear();
    }
    void clear() { free_.clear(); live_.clear(); seg_ = 0; }

    // offset of a new block of nbytes (rounded up to GRAN) aligned to `alignment` (a power of two; at
    // least GRAN is used), or UINT64_MAX
    uint64_t align(uint64_t alignment, uint64_t nbytes)
    {
        if (nbytes == 0 || alignment == 0 || (alignment & (alignment - 1))) return UINT64_MAX;
        if (alignment < GRAN) alignment = GRAN;
        if (seg_ % alignment || nbytes > seg_) return UINT64_MAX;   // the alignment must hold on every PE's copy
        const uint64_t need = (nbytes + GRAN - 1) / GRAN * GRAN;
        for (size_t i = 0; i < free_.size(); ++i) {
            const uint64_t b = free_[i].off, e = b + free_[i].len;
            const uint64_t a = (base_ + b + alignment - 1) / alignment * alignment - base_;
            if (a < b || a + need > e || a + need < a) continue;
            free_.erase(free_.begin() + (ptrdiff_t)i);
            if (a > b) insert_free(b, a - b);
            if (a + need < e) insert_free(a + need, e - (a + need));
            live_.push_back(Block{a, need});
            return a;
        }
        return UINT64_MAX;
    }

    // false when off is not the start of a live block
    bool release(uint64_t off)
    {
        for (size_t i = 0; i < live_.size(); ++i)
            if (live_[i].off == off) {
                const uint64_t len = live_[i].len;
                live_[i] = live_.back(); live_.pop_back();
                insert_free(off, len);
                return true;
            }
        return false;
    }

    size_t live_blocks() const { return live_.size(); }
    size_t free_blocks() const { return free_.size(); }

private:
    void insert_free(uint64_t off, uint64_t len)
    {
        auto it = std::lower_bound(free_.begin(), free_.end(), off, [](const Block &b, uint64_t o) { return b.off < o; });
        it = free_.insert(it, Block{off, len});
        auto nx = it + 1;
        if (nx != free_.end() && it->off + it->len == nx->off) { it->len += nx->len; it = free_.erase(nx) - 1; }
        if (it != free_.begin()) {
            auto pv = it - 1;
            if (pv->off + pv->len == it->off) { pv->len += it->len; free_.erase(it); }
        }
    }
    uint64_t base_ = 0, seg_ = 0;
    std::vector<Block> free_, live_;
};

// bytes spanned by nelems elements of eb bytes at a pitch of stride elements; false on overflow
inline bool strided_span(size_t nelems, ptrdiff_t stride, size_t eb, uint64_t *span)
{
    if (nelems == 0) { *span = 0; return true; }
    unsigned __int128 last = (unsigned __int128)(nelems - 1) * (unsigned __int128)(uint64_t)stride;
    unsigned __int128 bytes = last * eb + eb;
    if (bytes > (unsigned __int128)UINT64_MAX) return false;
    *span = (uint64_t)bytes;
    return true;
}

// Argument checks of the single-operation entry points, in the order in which their errors are reported
// (PE, element size, strides, alignment, range).  sym_off = symmetric address - heap address in unsigned
// arithmetic (an address below the heap becomes a huge offset and is out of range); local_addr is only
// looked at for its alignment.  A range may end exactly at the end of a segment, an empty one may start there.
inline bool pe_in(int pe, int npes) { return pe >= 0 && pe < npes; }
inline bool range_in(uint64_t seg, uint64_t off, uint64_t span) { return off <= seg && span <= seg - off; }

inline int check_contig(int npes, uint64_t seg, int pe_self, int pe, uint64_t sym_off, uint64_t nbytes)
{
    if (!pe_in(pe_self, npes) || !pe_in(pe, npes)) return SHMEM_ERR_INVALID_PE;
    return range_in(seg, sym_off, nbytes) ? SHMEM_OK : SHMEM_ERR_OUT_OF_RANGE;
}

inline int check_strided(int npes, uint64_t seg, int pe_self, int pe, uint64_t sym_off, ptrdiff_t sym_stride,
                         uint64_t local_addr, ptrdiff_t local_stride, size_t nelems, size_t eb)
{
    if (!pe_in(pe_self, npes) || !pe_in(pe, npes)) return SHMEM_ERR_INVALID_PE;
    if (eb != 1 && eb != 2 && eb != 4 && eb != 8) return SHMEM_ERR_INVALID_ARG;
    if (sym_stride < 1 || local_stride < 1) return SHMEM_ERR_INVALID_ARG;
    if (sym_off % eb || local_addr % eb) return SHMEM_ERR_ALIGN;
    uint64_t span;
    if (!strided_span(nelems, sym_stride, eb, &span)) return SHMEM_ERR_OUT_OF_RANGE;
    return range_in(seg, sym_off, span) ? SHMEM_OK : SHMEM_ERR_OUT_OF_RANGE;
}

inline int check_amo(int npes, uint64_t seg, int pe_self, int pe, uint64_t sym_off)
{
    if (!pe_in(pe_self, npes) || !pe_in(pe, npes)) return SHMEM_ERR_INVALID_PE;
    if (sym_off % 8) return SHMEM_ERR_ALIGN;
    return range_in(seg, sym_off, 8) ? SHMEM_OK : SHMEM_ERR_OUT_OF_RANGE;
}

// A descriptor as the host-side executor accepts it (the device-side executor applies the same rules):
// known kind, both PEs in range, both ranges inside a segment; strided ops: element size 1/2/4/8,
// strides >= 1, offsets aligned to the element.
inline bool desc_valid(const shmem_op_desc &d, uint32_t npes, uint64_t seg)
{
    if (d.pe >= npes || d.pe_self >= npes) return false;
    if (d.kind == SHMEM_OP_PUT || d.kind == SHMEM_OP_GET)
        return d.local_off <= seg && d.count <= seg - d.local_off && d.sym_off <= seg && d.count <= seg - d.sym_off;
    if (d.kind == SHMEM_OP_IPUT || d.kind == SHMEM_OP_IGET) {
        const uint32_t eb = d.elem_bytes;
        if (eb != 1 && eb != 2 && eb != 4 && eb != 8) return false;
        if (d.local_stride < 1 || d.sym_stride < 1 || d.local_off % eb || d.sym_off % eb) return false;
        if (d.count == 0) return d.local_off <= seg && d.sym_off <= seg;
        // (a stride only matters from the second element on; bounding the factors keeps the products in 128 bits)
        if (d.count > seg || (d.count > 1 && ((uint64_t)d.local_stride > seg || (uint64_t)d.sym_stride > seg))) return false;
        const unsigned __int128 ls = (unsigned __int128)(d.count - 1) * (uint64_t)d.local_stride * eb + eb;
        const unsigned __int128 ss = (unsigned __int128)(d.count - 1) * (uint64_t)d.sym_stride * eb + eb;
        return d.local_off <= seg && ls <= seg - d.local_off && d.sym_off <= seg && ss <= seg - d.sym_off;
    }
    return false;
}

}  // namespace hostlogic
