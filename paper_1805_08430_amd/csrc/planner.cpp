#include "planner.h"

#include <unordered_set>

namespace rdev {

uint32_t dtype_size(uint32_t dtype) {
    switch (dtype) {
        case RDEV_U8: case RDEV_I8: return 1;
        case RDEV_I16: case RDEV_F16: case RDEV_BF16: return 2;
        case RDEV_I32: case RDEV_F32: return 4;
        case RDEV_I64: case RDEV_F64: return 8;
        default: return 0;
    }
}

rdev_status tensor_bytes(uint32_t dtype, uint32_t ndims, const int64_t *dims, uint64_t *out, std::string &err) {
    uint64_t n = dtype_size(dtype);
    if (!n) { err = "unknown element type " + std::to_string(dtype); return RDEV_E_INVAL; }
    if (ndims > RDEV_MAX_DIMS) { err = "rank " + std::to_string(ndims) + " exceeds RDEV_MAX_DIMS"; return RDEV_E_INVAL; }
    bool zero = false, over = false;
    for (uint32_t i = 0; i < ndims; ++i) {
        if (dims[i] < 0) { err = "dim " + std::to_string(i) + " is not known"; return RDEV_E_INVAL; }
        if (dims[i] == 0) zero = true;
        if (__builtin_mul_overflow(n, (uint64_t)dims[i], &n)) over = true;
    }
    if (zero) { *out = 0; return RDEV_OK; }
    if (over) { err = "tensor bytes do not fit 64 bits"; return RDEV_E_OVERFLOW; }
    *out = n;
    return RDEV_OK;
}

RegionAllocator::RegionAllocator(uint64_t bytes) {
    if (bytes) free_[0] = bytes;
}

rdev_status RegionAllocator::alloc(uint64_t bytes, uint64_t align, uint64_t *offset_out, std::string &err) {
    if (!bytes) { err = "region bytes must be positive"; return RDEV_E_INVAL; }
    if (!is_pow2(align)) { err = "alignment must be a power of two"; return RDEV_E_ALIGN; }
    for (auto it = free_.begin(); it != free_.end(); ++it) {
        const uint64_t off = it->first, sz = it->second;
        uint64_t start, end;
        if (!round_up_checked(off, align, &start)) break;
        if (__builtin_add_overflow(start, bytes, &end)) continue;
        if (end > off + sz) continue;
        free_.erase(it);
        if (start > off) free_[off] = start - off;
        if (end < off + sz) free_[end] = off + sz - end;
        used_[start] = bytes;
        *offset_out = start;
        return RDEV_OK;
    }
    err = "no free block of " + std::to_string(bytes) + " bytes (align " + std::to_string(align) + ") in the arena";
    return RDEV_E_NOMEM;
}

rdev_status RegionAllocator::release(uint64_t offset, uint64_t bytes, std::string &err) {
    auto it = used_.find(offset);
    if (it == used_.end() || it->second != bytes) { err = "not an allocated region"; return RDEV_E_INVAL; }
    used_.erase(it);
    auto ins = free_.emplace(offset, bytes).first;
    auto next = std::next(ins);
    if (next != free_.end() && ins->first + ins->second == next->first) {
        ins->second += next->second;
        free_.erase(next);
    }
    if (ins != free_.begin()) {
        auto prev = std::prev(ins);
        if (prev->first + prev->second == ins->first) {
            prev->second += ins->second;
            free_.erase(ins);
        }
    }
    return RDEV_OK;
}

rdev_status layout(const rdev_tensor_desc *t, uint32_t n, uint64_t align, uint64_t max_static_bytes,
                   uint64_t dyn_heap_bytes, std::vector<rdev_placement> &out,
                   std::map<uint32_t, ArenaLayout> &arenas, std::string &err) {
    if (!is_pow2(align) || align < 16) { err = "plan alignment must be a power of two >= 16"; return RDEV_E_ALIGN; }
    out.clear();
    arenas.clear();
    std::unordered_set<uint32_t> seen;
    for (uint32_t i = 0; i < n; ++i) {
        const rdev_tensor_desc &d = t[i];
        if (!seen.insert(d.tensor_id).second) { err = "duplicate tensor id " + std::to_string(d.tensor_id); return RDEV_E_INVAL; }
        if (d.tensor_id == RDEV_ALL_TENSORS) { err = "tensor id 0xFFFFFFFF is reserved"; return RDEV_E_INVAL; }
        if (d.ndims > RDEV_MAX_DIMS) { err = "rank exceeds RDEV_MAX_DIMS"; return RDEV_E_INVAL; }
        if (!dtype_size(d.dtype)) { err = "unknown element type"; return RDEV_E_INVAL; }
        bool unknown = false;
        for (uint32_t k = 0; k < d.ndims; ++k) {
            if (d.dims[k] < -1) { err = "negative dim"; return RDEV_E_INVAL; }
            if (d.dims[k] == -1) unknown = true;
        }
        rdev_placement p{};
        p.tensor_id = d.tensor_id;
        p.dst_arena = d.dst_arena;
        uint64_t nb = 0;
        if (!unknown) {
            rdev_status st = tensor_bytes(d.dtype, d.ndims, d.dims, &nb, err);
            if (st != RDEV_OK) return st;
        }
        const bool is_static = !unknown && !(max_static_bytes && nb > max_static_bytes);
        ArenaLayout &al = arenas[d.dst_arena];
        const uint64_t ptr = al.static_bytes;
        uint64_t region;
        if (is_static) {
            uint64_t padded, with_flag;
            if (!round_up_checked(nb, 16, &padded) || __builtin_add_overflow(padded, (uint64_t)16, &with_flag) ||
                !round_up_checked(with_flag, align, &region)) { err = "region size overflows"; return RDEV_E_OVERFLOW; }
            p.kind = RDEV_STATIC;
            p.data_offset = ptr;
            p.bytes = nb;
            if (__builtin_add_overflow(ptr, padded, &p.flag_offset)) { err = "arena offset overflows"; return RDEV_E_OVERFLOW; }
        } else {
            region = (RDEV_META_BYTES + align - 1) & ~(align - 1);
            p.kind = RDEV_DYNAMIC;
            p.meta_offset = ptr;
            if (__builtin_add_overflow(ptr, (uint64_t)(RDEV_META_BYTES - 4), &p.flag_offset)) { err = "arena offset overflows"; return RDEV_E_OVERFLOW; }
        }
        p.region_bytes = region;
        if (__builtin_add_overflow(ptr, region, &al.static_bytes)) { err = "arena offset overflows"; return RDEV_E_OVERFLOW; }
        out.push_back(p);
    }
    uint64_t heap;
    if (!round_up_checked(dyn_heap_bytes, align, &heap)) { err = "heap size overflows"; return RDEV_E_OVERFLOW; }
    for (auto &kv : arenas) {
        kv.second.heap_offset = kv.second.static_bytes;
        kv.second.heap_bytes = heap;
        uint64_t tot;
        if (__builtin_add_overflow(kv.second.static_bytes, heap, &tot)) { err = "arena bytes overflow"; return RDEV_E_OVERFLOW; }
    }
    return RDEV_OK;
}

}  // namespace rdev
