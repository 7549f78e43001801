// Host-side planning: region sub-allocator, tensor classification and static
// placement (paper sections 3.1, 3.2-3.4).  No GPU code in here.
#pragma once
#include <cstdint>
#include <map>
#include <string>
#include <vector>

#include "rdev.h"

namespace rdev {

// itemsize of an element type code, 0 if unknown
uint32_t dtype_size(uint32_t dtype);

// bytes = itemsize * prod(dims); RDEV_E_INVAL on unknown dtype / bad rank / negative dim,
// RDEV_E_OVERFLOW when the product does not fit 64 bits
rdev_status tensor_bytes(uint32_t dtype, uint32_t ndims, const int64_t *dims, uint64_t *out, std::string &err);

inline bool is_pow2(uint64_t x) { return x && !(x & (x - 1)); }
inline bool round_up_checked(uint64_t x, uint64_t a, uint64_t *out) {
    uint64_t t;
    if (__builtin_add_overflow(x, a - 1, &t)) return false;
    *out = t & ~(a - 1);
    return true;
}

// First fit from the lowest address; free blocks sorted by offset and merged on release.
class RegionAllocator {
public:
    explicit RegionAllocator(uint64_t bytes = 0);
    rdev_status alloc(uint64_t bytes, uint64_t align, uint64_t *offset_out, std::string &err);
    rdev_status release(uint64_t offset, uint64_t bytes, std::string &err);
    size_t live() const { return used_.size(); }
private:
    std::map<uint64_t, uint64_t> free_;   // offset -> bytes
    std::map<uint64_t, uint64_t> used_;   // offset -> bytes
};

struct ArenaLayout {
    uint64_t base = 0;          // offset of the plan's block in the arena
    uint64_t static_bytes = 0;  // regions + metadata slots
    uint64_t heap_offset = 0;   // absolute, once base is known
    uint64_t heap_bytes = 0;
    uint64_t heap_ptr = 0;      // bump pointer relative to heap_offset
    uint64_t total() const { return static_bytes + heap_bytes; }
};

// Classify + place relative to each arena's block start (base 0).
// kind/static bytes land in `out` (input order), per-arena sums in `arenas`.
rdev_status layout(const rdev_tensor_desc *t, uint32_t n, uint64_t align, uint64_t max_static_bytes,
                   uint64_t dyn_heap_bytes, std::vector<rdev_placement> &out,
                   std::map<uint32_t, ArenaLayout> &arenas, std::string &err);

}  // namespace rdev
