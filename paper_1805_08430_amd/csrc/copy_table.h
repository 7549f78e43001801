// Host side of the batched copy: cutting tensors into the work items that
// copy_table_kernel walks, and the order of the table.  No GPU calls in here.
#pragma once
#include <algorithm>
#include <cstdint>
#include <vector>

#include "copy_kernel.h"

namespace rdev {

// cut one tensor into work items
inline void cut_items(const uint8_t *src, uint8_t *dst, uint64_t bytes, uint32_t tensor, uint64_t chunk, uint32_t small,
               std::vector<Item> &items, std::vector<Item> &subs, std::vector<Item> &pending_small) {
    if (bytes <= small) {
        pending_small.push_back(Item{src, dst, (uint32_t)bytes, 0, 0, tensor});
        if (pending_small.size() == kWavesPerBlock) {
            items.push_back(Item{nullptr, nullptr, 0, (uint32_t)pending_small.size(), (uint32_t)subs.size(), tensor});
            subs.insert(subs.end(), pending_small.begin(), pending_small.end());
            pending_small.clear();
        }
        return;
    }
    for (uint64_t off = 0; off < bytes; off += chunk) {
        const uint64_t n = std::min<uint64_t>(chunk, bytes - off);
        items.push_back(Item{src + off, dst + off, (uint32_t)n, 0, 0, tensor});
    }
}

inline void flush_small(std::vector<Item> &items, std::vector<Item> &subs, std::vector<Item> &pending_small) {
    if (pending_small.empty()) return;
    items.push_back(Item{nullptr, nullptr, 0, (uint32_t)pending_small.size(), (uint32_t)subs.size(), 0});
    subs.insert(subs.end(), pending_small.begin(), pending_small.end());
    pending_small.clear();
}

// Workgroups are handed to the 8 XCDs round-robin (workgroup b runs on XCD
// b % 8), each XCD with its own L2.  Reorder the table so that every XCD walks
// one contiguous eighth of the work instead of every eighth item: measured a
// few percent faster for a streaming copy.  Padding entries do nothing.
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
