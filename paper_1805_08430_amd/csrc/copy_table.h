// Host side of the batched copy: cutting tensors into the work items that
// copy_table_kernel walks, and the order of the table.  No GPU calls in here.
#pragma once
#include <algorithm>
#include <cstdint>
#include <vector>

#include "copy_kernel.h"

namespace rdev {

// A tensor that was cut into full-size items: a candidate for a range in the kernel arguments.
struct RangeCand {
    uint32_t first_item, n_items;
    const uint8_t *src;
    uint8_t *dst;
    uint64_t bytes;
};

// cut one tensor into work items (appended to `items` in order; small tensors are collected 16 to an item)
inline void cut_items(const uint8_t *src, uint8_t *dst, uint64_t bytes, uint32_t tensor, uint64_t chunk, uint32_t small,
                      std::vector<Item> &items, std::vector<Item> &subs, std::vector<Item> &pending_small,
                      std::vector<RangeCand> *cands = nullptr) {
    if (bytes <= small) {
        pending_small.push_back(Item{src, dst, (uint32_t)bytes, 0, 0, tensor});
        if (pending_small.size() == kWavesPerBlock) {
            items.push_back(Item{nullptr, nullptr, 0, (uint32_t)pending_small.size(), (uint32_t)subs.size(), tensor});
            subs.insert(subs.end(), pending_small.begin(), pending_small.end());
            pending_small.clear();
        }
        return;
    }
    const size_t first = items.size();
    for (uint64_t off = 0; off < bytes; off += chunk) {
        const uint64_t n = std::min<uint64_t>(chunk, bytes - off);
        items.push_back(Item{src + off, dst + off, (uint32_t)n, 0, 0, tensor});
    }
    if (cands && items.size() - first >= 2 && items.size() <= 0xFFFFFFFFull)
        cands->push_back(RangeCand{(uint32_t)first, (uint32_t)(items.size() - first), src, dst, bytes});
}

inline void flush_small(std::vector<Item> &items, std::vector<Item> &subs, std::vector<Item> &pending_small) {
    if (pending_small.empty()) return;
    items.push_back(Item{nullptr, nullptr, 0, (uint32_t)pending_small.size(), (uint32_t)subs.size(), 0});
    subs.insert(subs.end(), pending_small.begin(), pending_small.end());
    pending_small.clear();
}

// The launch description of one table of n_items items (device pointers are filled in by the caller): the XCD
// order, the number of workgroups, and the kMaxRanges candidates with the most items as ranges.  `base` is the index
// of the table's first item inside the vector the candidates were recorded against.
inline TableArgs make_table_args(size_t n_items, uint32_t chunk, std::vector<RangeCand> cands, size_t base,
                                 uint32_t *n_blocks_out) {
    TableArgs a{};
    a.n_items = (uint32_t)n_items;
    a.chunk = chunk;
    a.per_xcd = n_items < 2 * kXcds ? 0 : (uint32_t)((n_items + kXcds - 1) / kXcds);
    *n_blocks_out = a.per_xcd ? a.per_xcd * kXcds : (uint32_t)n_items;
    std::stable_sort(cands.begin(), cands.end(), [](const RangeCand &x, const RangeCand &y) { return x.n_items > y.n_items; });
    for (size_t k = 0; k < cands.size() && k < kMaxRanges; ++k) {
        a.first[k] = (uint32_t)(cands[k].first_item - base);
        a.count[k] = cands[k].n_items;
        a.src[k] = cands[k].src;
        a.dst[k] = cands[k].dst;
        a.bytes[k] = cands[k].bytes;
    }
    return a;
}

// The same XCD order for tables that are permuted on the host (the unpack tables of the copying modes).
template <typename T>
void xcd_order(std::vector<T> &items) {
    const size_t n = items.size();
    if (n < 2 * kXcds) return;
    const size_t per = (n + kXcds - 1) / kXcds;
    std::vector<T> out(per * kXcds, T{});
    for (size_t b = 0; b < out.size(); ++b) {
        const size_t c = (b % kXcds) * per + b / kXcds;
        if (c < n) out[b] = items[c];
    }
    items.swap(out);
}

}  // namespace rdev
