// Device code (gfx950) around the data mover of copy_kernel.h: flag publication, the
// dynamic path's metadata / receive kernels, the copying baselines, the sparse-id
// producer and the receiver-side consumer.  LDS appears only in the producer, the
// consumer's reduction and the device-side receive.  Completion flags are stored by a
// separate small kernel enqueued behind the copy on the same stream, so the kernel
// boundary is the release point: section 3.2 needs a flag that becomes visible only
// after the whole tensor; a NIC gets that from ascending-address writes, a GPU does not.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "copy_kernel.h"
#include "rdev.h"

namespace rdev {

struct FlagEnt {
    uint32_t *arena_flag;   // flag word inside the receiver arena
    uint32_t mirror_idx;    // index of its host-visible word
    uint32_t _pad;
};
static_assert(sizeof(FlagEnt) == 16, "FlagEnt is 16 bytes");

struct MetaBatch {
    uint32_t words[kMetaInlineMax][30];     // the first 120 bytes of each record
    uint8_t *slot[kMetaInlineMax];          // receiver slot in the arena
    uint32_t meta_idx[kMetaInlineMax];      // index of the host-visible copy of the record
    uint32_t flag_idx[kMetaInlineMax];      // index of the host-visible metadata flag
    const uint32_t *dim0_dev[kMetaInlineMax]; // when set: the leading dim is read from this device word at run time
    uint64_t row_bytes[kMetaInlineMax];     // bytes per unit of the leading dim (used with dim0_dev)
    uint64_t dim0_max[kMetaInlineMax];      // the caller's bound on the leading dim (used with dim0_dev)
    uint32_t n;
    uint32_t seq;
};

struct PostBatch {                           // after a pull: record the offset, raise payload-complete
    uint8_t *slot[kInlineMax];
    uint64_t dst_offset[kInlineMax];
    uint32_t meta_idx[kInlineMax];
    uint32_t flag_idx[kInlineMax];
    uint32_t n;
    uint32_t seq;
};

// s_waitcnt vmcnt(0): this wave's vector-memory stores (and loads) issued so far have completed.  The operand is the
// gfx9 encoding with the export and LDS/scalar counters left at "do not wait".
__device__ __forceinline__ void wait_stores_acked() { __builtin_amdgcn_s_waitcnt(0x0F70); }

// Stores that every compute die (and a later kernel on any of them) must see without a cache write-back: agent-scope
// relaxed atomic stores write through.  Used for the few words of records and flags; payloads go through copy_span.
__device__ __forceinline__ void store_through(uint32_t *p, uint32_t v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void store_through(uint64_t *p, uint64_t v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// The same towards pinned host memory.  A plain store there may sit in a device cache until the kernel ends and be
// overtaken by a flag stored with system scope; these leave the device in program order.
__device__ __forceinline__ void store_host(uint32_t *p, uint32_t v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
}
__device__ __forceinline__ void store_host(uint64_t *p, uint64_t v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
}

// flag <- value for a table of tensors (in-arena words), then ONE host-visible word for the whole table.
// The payload these flags announce was written by the kernel enqueued before this
// one on the same stream, so it is already visible when this kernel starts: the
// stores here need the right scope but no cache write-back of their own.
// The host is told with one word for the whole table (a delivery token):
// per-tensor host words would be thousands of separate writes across the host
// link for the many-small-tensor sets.  One workgroup walks the table, and the
// token is stored only after every in-arena word has been acknowledged: the
// agent-scope stores write through, each wave waits until its own outstanding
// stores have been acknowledged (wait_stores_acked: the wait alone, without the
// L2 write-back a release fence of agent or system scope would add), then the
// barrier, and one lane stores the token behind it.  A receiver that has seen the token may therefore clear
// the in-arena words from any other stream without meeting a late store.
constexpr uint32_t kFlagTableThreads = 1024;
__global__ __launch_bounds__(kFlagTableThreads) void flag_table_kernel(const FlagEnt *__restrict__ ents, uint32_t n,
                                                                        uint32_t value, uint32_t *batch_word,
                                                                        uint32_t token) {
    for (uint32_t i = threadIdx.x; i < n; i += 4 * kFlagTableThreads) {        // four table entries in flight per lane
        uint32_t *f[4];
#pragma unroll
        for (uint32_t k = 0; k < 4; ++k) f[k] = i + k * kFlagTableThreads < n ? ents[i + k * kFlagTableThreads].arena_flag : nullptr;
#pragma unroll
        for (uint32_t k = 0; k < 4; ++k)
            if (f[k]) __hip_atomic_store(f[k], value, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    if (!batch_word) return;
    wait_stores_acked();
    __syncthreads();
    if (threadIdx.x == 0) __hip_atomic_store(batch_word, token, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
}

constexpr uint32_t kFlagInlineMax = 32;
struct InlineFlags {
    uint32_t *arena_flag[kFlagInlineMax];
    uint32_t mirror_idx[kFlagInlineMax];
    uint32_t n;
    uint32_t value;
};

// the same for a few tensors named in the kernel arguments (no table to fetch first: one memory round trip less).
// With `mirror`: one host-visible word each, stored once the lane's in-arena store has been acknowledged.
// With `batch_word`: one token for all of them, stored by lane 0 once the wave's stores have been acknowledged.
__global__ __launch_bounds__(64) void flag_inline_kernel(InlineFlags f, uint32_t *mirror, uint32_t *batch_word,
                                                         uint32_t token) {
    const uint32_t i = threadIdx.x;
    if (i < f.n) __hip_atomic_store(f.arena_flag[i], f.value, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (!mirror && !batch_word) return;
    wait_stores_acked();                     // one wave: its own wait covers every lane's store
    if (mirror && i < f.n) __hip_atomic_store(mirror + f.mirror_idx[i], f.value, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
    if (batch_word && i == 0) __hip_atomic_store(batch_word, token, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
}

// Dynamic path, sender side: 120 bytes of metadata into the receiver's slot
// (and its host-visible copy), then the flag in the record's last word.
__global__ __launch_bounds__(64) void meta_write_kernel(MetaBatch b, uint32_t *mirror_flags, rdev_meta *mirror_meta) {
    const uint32_t k = blockIdx.x;
    const uint32_t t = threadIdx.x;
    uint32_t *slot = (uint32_t *)b.slot[k];
    uint32_t *host = (uint32_t *)(mirror_meta + b.meta_idx[k]);
    if (t < 30) {
        uint32_t w = b.words[k][t];
        if (b.dim0_dev[k] && (t == 2 || t == 3 || t == 6 || t == 7)) {
            // a size known only on the device: leading dim (words 6,7) and bytes (words 2,3) are filled in here;
            // a count beyond the caller's bound is cut to the bound
            uint64_t d0 = *b.dim0_dev[k];
            if (d0 > b.dim0_max[k]) d0 = b.dim0_max[k];
            const uint64_t v = (t < 4) ? d0 * b.row_bytes[k] : d0;
            w = (t & 1) ? (uint32_t)(v >> 32) : (uint32_t)v;
        }
        store_through(slot + t, w);
        store_host(host + t, w);
    }
    // the flag goes out once every word of the record has been acknowledged (one wave: its own wait is enough)
    wait_stores_acked();
    if (t == 0) {
        store_through(slot + 31, b.seq);
        store_host(mirror_flags + b.flag_idx[k], b.seq);
    }
}

// Dynamic path, receiver side, behind the pull: record where the payload went, raise payload-complete.
__global__ void post_pull_kernel(PostBatch b, uint32_t *mirror_flags, rdev_meta *mirror_meta) {
    const uint32_t i = threadIdx.x;
    if (i >= b.n) return;
    // the payload was written by the kernel before this one; within this kernel the offset must be out before the flag
    store_through((uint64_t *)(b.slot[i] + 88), b.dst_offset[i]);
    store_host((uint64_t *)&mirror_meta[b.meta_idx[i]].dst_offset, b.dst_offset[i]);
    wait_stores_acked();
    store_through((uint32_t *)(b.slot[i] + 120), b.seq);
    store_host(mirror_flags + b.flag_idx[i], b.seq);
}

// ---- dynamic path, receiver side, with the sizes taken on the device (section 3.3) ----
//
// The receiver's part of the protocol - see the metadata, clear its flag, allocate
// storage, pull the payload, raise payload-complete - without a host round trip:
// the kernels are enqueued behind the sender's metadata write and read the
// record from the slot themselves.  Allocation is the same bump allocator the
// host path runs (batch order, round_up(bytes, align) each), so the arena image
// is the same.  Every workgroup derives the batch's layout from the same memory
// with the same code; a batch that fails any check moves nothing.

constexpr uint32_t kRecvMax = 8;                 // tensors per launch
constexpr uint32_t kRecvMaxBlocks = 2048;           // with a size hint from the caller
constexpr uint32_t kRecvBlocksNoHint = 256;       // without: the workgroups stride over whatever the records say

struct ArenaEnt {                                // device table of the registered arenas
    uint8_t *base;
    uint64_t bytes;
};
struct HeapWord {                                // device-resident bump pointer of one arena's dynamic heap
    uint64_t ptr;                                // relative to the heap's start
    uint32_t epoch;                              // valid for this iteration number only (rdev_dyn_reset starts a new one)
    uint32_t _pad;
};
struct RecvEnt {
    uint8_t *slot;                               // the tensor's metadata slot
    uint8_t *arena_base;                         // base of the receiving arena
    uint64_t heap_offset;                        // start of its dynamic heap, bytes from the arena base
    uint64_t heap_bytes;
    uint64_t heap_ptr_host;                      // what the host path has handed out so far in this iteration
    uint32_t heap_word;                          // index of the arena's HeapWord
    uint32_t dst_arena;
    uint32_t meta_idx, flag_idx;                 // host-visible copies: record, flag pair (2*index)
};
constexpr uint32_t kArenaArgs = 16;              // arenas 0..15 travel in the kernel arguments (no dependent table load)
struct RecvBatch {
    RecvEnt e[kRecvMax];
    ArenaEnt arena[kArenaArgs];
    uint64_t align;
    uint32_t n, seq, epoch, chunk, n_arenas, call_id;
};
struct RecvLayout {                              // what every workgroup works out for itself
    const uint8_t *src[kRecvMax];
    uint8_t *dst[kRecvMax];
    uint64_t bytes[kRecvMax];
    uint64_t dst_offset[kRecvMax];               // bytes from the arena base
    uint64_t new_ptr[kRecvMax];                  // the arena's heap pointer after this entry
    uint64_t first_chunk[kRecvMax + 1];
    int32_t status;                              // RDEV_OK, RDEV_NOT_READY (a metadata flag is not set) or an RDEV_E_* code
    uint32_t bad;                                // entry the status refers to
};

// Lanes 0..n-1 fetch their record, lane 0 runs the allocator over the batch.  Call with all lanes of the workgroup.
__device__ __forceinline__ void recv_layout(const RecvBatch &b, const ArenaEnt *__restrict__ arenas,
                                            const HeapWord *__restrict__ heap, RecvLayout &L) {
    __shared__ uint64_t s_bytes[kRecvMax], s_src_off[kRecvMax], s_heap[kRecvMax];
    __shared__ uint32_t s_src_arena[kRecvMax], s_flag[kRecvMax];
    const uint32_t t = threadIdx.x;
    if (t < b.n) {
        const uint8_t *slot = b.e[t].slot;
        s_flag[t] = __hip_atomic_load((const uint32_t *)(slot + 124), __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_AGENT);
        s_bytes[t] = *(const uint64_t *)(slot + 8);
        s_src_off[t] = *(const uint64_t *)(slot + 16);
        s_src_arena[t] = *(const uint32_t *)(slot + 96);
        const HeapWord h = heap[b.e[t].heap_word];
        s_heap[t] = h.epoch == b.epoch ? h.ptr : b.e[t].heap_ptr_host;
    }
    __syncthreads();
    if (t == 0) {
        int32_t st = RDEV_OK;
        uint32_t bad = 0;
        uint64_t chunks = 0;
        for (uint32_t k = 0; k < b.n && st == RDEV_OK; ++k) {
            bad = k;
            uint64_t ptr = s_heap[k];
            for (uint32_t j = 0; j < k; ++j)
                if (b.e[j].heap_word == b.e[k].heap_word) ptr = L.new_ptr[j];      // same arena earlier in the batch
            const uint64_t nb = s_bytes[k], need = (nb + b.align - 1) & ~(b.align - 1);
            if (!s_flag[k]) { st = RDEV_NOT_READY; break; }
            if (s_src_arena[k] >= b.n_arenas) { st = RDEV_E_RANGE; break; }
            const ArenaEnt sa = s_src_arena[k] < kArenaArgs ? b.arena[s_src_arena[k]] : arenas[s_src_arena[k]];
            if (!sa.bytes) { st = RDEV_E_RANGE; break; }
            if (s_src_off[k] > sa.bytes || nb > sa.bytes - s_src_off[k]) { st = RDEV_E_RANGE; break; }
            if (need < nb || ptr > b.e[k].heap_bytes || need > b.e[k].heap_bytes - ptr) { st = RDEV_E_NOMEM; break; }
            const uint64_t dst_off = b.e[k].heap_offset + ptr;
            if (nb && s_src_arena[k] == b.e[k].dst_arena && s_src_off[k] < dst_off + nb && dst_off < s_src_off[k] + nb) {
                st = RDEV_E_OVERLAP;
                break;
            }
            L.src[k] = sa.base + s_src_off[k];
            L.dst[k] = b.e[k].arena_base + dst_off;
            L.bytes[k] = nb;
            L.dst_offset[k] = dst_off;
            L.new_ptr[k] = ptr + need;
            L.first_chunk[k] = chunks;
            chunks += (nb + b.chunk - 1) / b.chunk;
        }
        L.first_chunk[b.n] = chunks;
        if (st != RDEV_OK) L.first_chunk[b.n] = 0;
        L.status = st;
        L.bad = bad;
    }
    __syncthreads();
}

// The receive in one launch.  Every workgroup works the layout out, pulls its share of the chunks (striding over the
// chunks of all payloads of the batch), waits until its stores are acknowledged and then counts itself in; the
// workgroup that arrives last finds every payload byte in place and does what follows the pull: record the offsets,
// consume the metadata flags, move the heap words, raise payload-complete, and tell the host how the batch went
// (status[0] = code, [1] = entry it refers to, [2] = call id, stored last).  The count carries, in its upper half,
// how many workgroups found the batch in order: if a record changed under the kernel (a sender still writing - a
// misuse), some did and some did not, and nothing is published.  *arrivals is zero between launches: the last
// workgroup clears it, so launches on one plan must not overlap (they would race on the heap words as well).
__global__ __launch_bounds__(kBlockThreads) void recv_kernel(RecvBatch b, const ArenaEnt *__restrict__ arenas, HeapWord *heap,
                                                              uint32_t *arrivals, uint32_t *mirror_flags, rdev_meta *mirror_meta,
                                                              uint32_t *status) {
    __shared__ RecvLayout L;
    __shared__ uint32_t s_seen;
    recv_layout(b, arenas, heap, L);
    const uint32_t t = threadIdx.x;
    const bool ok = L.status == RDEV_OK;
    if (ok) {
        const uint64_t total = L.first_chunk[b.n];
        for (uint64_t c = blockIdx.x; c < total; c += gridDim.x) {
            uint32_t k = 0;
            while (c >= L.first_chunk[k + 1]) ++k;
            const uint64_t off = (c - L.first_chunk[k]) * b.chunk;
            const uint64_t rem = L.bytes[k] - off;
            copy_span(L.src[k] + off, L.dst[k] + off, rem < b.chunk ? (uint32_t)rem : b.chunk, t, kBlockThreads);
        }
    }
    wait_stores_acked();                                                 // every wave: its payload stores have landed
    __syncthreads();
    if (t == 0) s_seen = __hip_atomic_fetch_add(arrivals, ok ? 0x10001u : 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __syncthreads();
    const uint32_t seen = s_seen;
    if ((seen & 0xffffu) != gridDim.x - 1) return;                       // somebody else arrives later
    const uint32_t n_ok = (seen >> 16) + (ok ? 1u : 0u);
    const bool publish = ok && n_ok == gridDim.x;
    if (publish && t < b.n) {
        uint8_t *slot = b.e[t].slot;
        store_through((uint64_t *)(slot + 88), L.dst_offset[t]);
        store_host((uint64_t *)&mirror_meta[b.e[t].meta_idx].dst_offset, L.dst_offset[t]);
        store_through((uint32_t *)(slot + 124), 0u);                     // metadata consumed
        store_host(mirror_flags + b.e[t].flag_idx + 1, 0u);
        bool last = true;                                                // last entry of its arena stores the heap pointer
        for (uint32_t j = t + 1; j < b.n; ++j)
            if (b.e[j].heap_word == b.e[t].heap_word) last = false;
        if (last) {
            store_through(&heap[b.e[t].heap_word].ptr, L.new_ptr[t]);
            store_through(&heap[b.e[t].heap_word].epoch, b.epoch);
        }
        wait_stores_acked();                                             // offset and cleared flag first, then payload-complete
        store_through((uint32_t *)(slot + 120), b.seq);
        store_host(mirror_flags + b.e[t].flag_idx, b.seq);
    }
    if (t == 0) {
        store_through(arrivals, 0u);
        const bool mixed = n_ok != 0 && n_ok != gridDim.x;               // the records changed while the kernel ran
        store_host(status, (uint32_t)(mixed ? RDEV_NOT_READY : L.status));
        store_host(status + 1, L.bad);
        wait_stores_acked();
        store_host(status + 2, b.call_id);
    }
}

// ---- the copying alternatives the paper argues against (sections 2.2, 5.1) ----

constexpr uint32_t kMaxHeapSlots = 16;
struct HeapBases {
    uint8_t *base[kMaxHeapSlots];   // start of the fresh-allocation area of each destination arena for this call
};

// One unit of unpack work: a chunk of one message's payload.  Grouping as in Item.
struct UItem {
    const uint8_t *hdr;     // the message header (or, with kFragBit, a fragment header) in the receive buffer
    uint64_t dst_rel;       // where this piece starts inside this call's fresh-allocation area
    uint32_t chunk_index;
    uint32_t heap_slot;     // | kFragBit when hdr is a fragment header
    uint32_t n_sub;
    uint32_t sub_first;
};
constexpr uint32_t kFragBit = 0x80000000u;
static_assert(sizeof(UItem) == 32, "UItem is 32 bytes");

// pack, part 1: the 128-byte header of every message (seq patched in) and the zero padding behind the payload
__global__ void rpc_header_kernel(const rdev_meta *__restrict__ headers, uint8_t *const *__restrict__ msg_ptrs,
                                  uint32_t n, uint32_t seq, uint32_t pad_payload) {
    const uint32_t gid = blockIdx.x * blockDim.x + threadIdx.x;
    const uint32_t t = gid >> 5, w = gid & 31;
    if (t >= n) return;
    const uint32_t *hw = (const uint32_t *)(headers + t);
    uint8_t *msg = msg_ptrs[t];
    ((uint32_t *)msg)[w] = (w == 26) ? seq : hw[w];
    if (!pad_payload) return;                       // fragmented messages pad behind each fragment instead
    const uint64_t bytes = headers[t].bytes;
    const uint32_t pad = (16 - (uint32_t)(bytes & 15)) & 15;
    if (w < pad) msg[RDEV_META_BYTES + bytes + w] = 0;
}

// pack, fragmented messages: the 32-byte header of every fragment (seq patched in) and the padding behind its payload
__global__ void rpc_frag_header_kernel(const rdev_frag *__restrict__ frags, uint8_t *const *__restrict__ frag_ptrs,
                                       uint32_t n, uint32_t seq) {
    const uint32_t gid = blockIdx.x * blockDim.x + threadIdx.x;
    const uint32_t f = gid >> 3, w = gid & 7;
    if (f >= n) return;
    const uint32_t *hw = (const uint32_t *)(frags + f);
    uint8_t *p = frag_ptrs[f];
    ((uint32_t *)p)[w] = (w == 1) ? seq : hw[w];
    const uint32_t bytes = frags[f].bytes;
    const uint32_t pad = (16 - (bytes & 15)) & 15;
    for (uint32_t k = w; k < pad; k += 8) p[sizeof(rdev_frag) + bytes + k] = 0;
}

__device__ __forceinline__ void unpack_one(const UItem &it, const HeapBases &hb, uint32_t chunk, uint32_t tid,
                                           uint32_t nth) {
    if (!it.hdr) return;                                          // padding entry of the table
    const bool frag = it.heap_slot & kFragBit;
    // the length comes from the message itself: the tensor's header, or the fragment's
    const uint64_t bytes = frag ? ((const rdev_frag *)it.hdr)->bytes : ((const rdev_meta *)it.hdr)->bytes;
    const uint32_t head = frag ? (uint32_t)sizeof(rdev_frag) : (uint32_t)RDEV_META_BYTES;
    const uint64_t off = (uint64_t)it.chunk_index * chunk;
    if (off >= bytes) return;
    const uint64_t rem = bytes - off;
    const uint32_t n = rem < chunk ? (uint32_t)rem : chunk;
    copy_span(it.hdr + head + off, hb.base[it.heap_slot & ~kFragBit] + it.dst_rel + off, n, tid, nth);
}

// unpack: parse each header, copy the payload out into the fresh allocation
__global__ __launch_bounds__(kBlockThreads) void unpack_table_kernel(const UItem *__restrict__ items,
                                                                      const UItem *__restrict__ subs, HeapBases hb,
                                                                      uint32_t chunk) {
    const UItem it = items[blockIdx.x];
    if (it.n_sub == 0) {
        unpack_one(it, hb, chunk, threadIdx.x, kBlockThreads);
    } else {
        const uint32_t wave = threadIdx.x >> 6;
        if (wave < it.n_sub) unpack_one(subs[it.sub_first + wave], hb, chunk, threadIdx.x & 63, 64);
    }
}

// flags of delivered messages: the value is the seq found in each header; token last, as in flag_table_kernel
__global__ __launch_bounds__(kFlagTableThreads) void rpc_flag_kernel(const FlagEnt *__restrict__ ents,
                                                                      uint8_t *const *__restrict__ hdr_ptrs, uint32_t n,
                                                                      uint32_t *batch_word, uint32_t token) {
    for (uint32_t i = threadIdx.x; i < n; i += kFlagTableThreads) {
        const uint32_t seq = ((const rdev_meta *)hdr_ptrs[i])->seq;
        __hip_atomic_store(ents[i].arena_flag, seq, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    wait_stores_acked();
    __syncthreads();
    if (threadIdx.x == 0) __hip_atomic_store(batch_word, token, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
}

// ---- producer of the sparse case: distinct ids (ascending) and their rows ----

constexpr uint32_t kUniqueThreads = 1024;
constexpr uint32_t kUniqueMaxVocab = 262144;             // 32 KiB bitmap in LDS

// One workgroup: mark every id in an LDS bitmap, rank the set bits with a
// two-level prefix sum of population counts, write the ids out in ascending order.
__global__ __launch_bounds__(kUniqueThreads) void unique_ids_kernel(const int64_t *__restrict__ ids, uint32_t n_ids,
                                                                     uint32_t vocab, int64_t *__restrict__ out_ids,
                                                                     uint32_t *__restrict__ count_out) {
    __shared__ uint32_t bm[kUniqueMaxVocab / 32];
    __shared__ uint32_t part[kUniqueThreads];
    __shared__ uint32_t bad;
    const uint32_t t = threadIdx.x;
    const uint32_t words = (vocab + 31) / 32;
    for (uint32_t w = t; w < words; w += kUniqueThreads) bm[w] = 0;
    if (t == 0) bad = 0;
    __syncthreads();
    for (uint32_t i = t; i < n_ids; i += kUniqueThreads) {
        const int64_t id = ids[i];
        if (id >= 0 && id < (int64_t)vocab) atomicOr(&bm[(uint32_t)id >> 5], 1u << ((uint32_t)id & 31));
        else atomicAdd(&bad, 1u);
    }
    __syncthreads();
    const uint32_t seg = (words + kUniqueThreads - 1) / kUniqueThreads;      // contiguous words per lane
    const uint32_t w0 = t * seg, w1 = min(w0 + seg, words);
    uint32_t mine = 0;
    for (uint32_t w = w0; w < w1; ++w) mine += __popc(bm[w]);
    part[t] = mine;
    __syncthreads();
    for (uint32_t off = 1; off < kUniqueThreads; off <<= 1) {                // inclusive scan
        const uint32_t v = t >= off ? part[t - off] : 0;
        __syncthreads();
        part[t] += v;
        __syncthreads();
    }
    uint32_t rank = part[t] - mine;
    for (uint32_t w = w0; w < w1; ++w) {
        uint32_t bits = bm[w];
        while (bits) {
            const uint32_t b = __ffs(bits) - 1;
            out_ids[rank++] = (int64_t)w * 32 + b;
            bits &= bits - 1;
        }
    }
    if (t == kUniqueThreads - 1) {
        count_out[0] = part[t];
        count_out[1] = bad;
    }
}

// row r of the output <- table[out_ids[r]]; workgroups beyond the count leave at once
__global__ __launch_bounds__(256) void gather_rows_kernel(const int64_t *__restrict__ out_ids,
                                                           const uint32_t *__restrict__ count, const uint8_t *__restrict__ table,
                                                           uint32_t row_bytes, uint8_t *__restrict__ out_rows) {
    const uint32_t r = blockIdx.x;
    if (r >= count[0]) return;
    const v4u *s = (const v4u *)(table + (size_t)out_ids[r] * row_bytes);
    v4u *d = (v4u *)(out_rows + (size_t)r * row_bytes);
    for (uint32_t i = threadIdx.x; i < row_bytes / 16; i += 256) d[i] = __builtin_nontemporal_load(s + i);
}

// ---- receiver-side consumer (sections 4, 5.1) ----

// Launch shape: 1024-lane workgroups that stay and stride over the payload, two 16-byte loads in flight per lane,
// two workgroups per compute unit at most.  Read-only 553 MB this way runs at 80 % of HBM peak (82 % with one or with
// four loads in flight; two keep the kernel within 40 registers, see consume_accumulate); 256-lane workgroups reach
// 78 % with 512 of them and 68 % with 2048, and a fresh workgroup per 64 KiB (whose two atomics per workgroup then
// dominate) 32 %.  The arithmetic is free beside the loads (the same loop with one xor per word takes as long).
constexpr uint32_t kConsumeThreads = 1024;
constexpr uint32_t kConsumeInFlight = 2;
constexpr uint32_t kConsumeMaxBlocks = 64;         // when the kernel waits for the flag on the device
constexpr uint32_t kConsumeMaxBlocksNoWait = 512;  // when the host has seen the flag already

// order-preserving map of non-NaN floats to unsigned (and -0 < +0)
__device__ __forceinline__ uint32_t f2ord(uint32_t bits) { return bits ^ ((bits >> 31) ? 0xFFFFFFFFu : 0x80000000u); }
__device__ __forceinline__ uint32_t ord2f(uint32_t o) { return o ^ ((o >> 31) ? 0x80000000u : 0xFFFFFFFFu); }
constexpr uint32_t kOrdNegInf = 0x007FFFFFu;     // f2ord(bits of -inf = 0xFF800000)

__device__ __forceinline__ void consume_init_one(rdev_consume_result *out) {
    out->status = 1;
    out->seen_flag = 0;
    ((uint32_t *)&out->max)[0] = kOrdNegInf;         // holds the ordered key until the last workgroup converts it
    out->_arrivals = 0;
    out->word_sum = 0;
}

__global__ void consume_init_kernel(rdev_consume_result *out, uint32_t n) {
    const uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) consume_init_one(out + i);
}

// One workgroup's wait for a tensor's in-arena flag: at most max_spins loads by one lane (agent scope, relaxed: they
// go past the caches and cost no invalidation each), the answer shared with the others.  Once the flag is up the
// polling wave makes ONE acquire before the others are let go, so that none of the payload is served from lines an
// earlier iteration left in the caches: the vector cache belongs to the compute unit and the L2 to the die, so one
// wave's invalidation serves the whole workgroup (an acquire in each of the sixteen waves made the waiting consumer
// 40 % slower).  Returns the flag value seen, 0 = gave up.
__device__ __forceinline__ uint32_t consume_wait(const uint32_t *flag, uint32_t max_spins, uint32_t *s_seen) {
    __syncthreads();                                    // s_seen may still be read from an earlier wait
    if (threadIdx.x == 0) {
        uint32_t v = 0;
        for (uint32_t k = 0; k < max_spins; ++k) {
            v = __hip_atomic_load(flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (v) break;
            // Back off: hundreds of workgroups poll the same few words, and every poll goes to the one memory channel
            // that holds the word; polled hard, that channel starves the copy the pollers are waiting for.
            const uint32_t naps = k < 8 ? 1 : (k < 32 ? 2 : 4);          // about 3.4 us each
            for (uint32_t j = 0; j < naps; ++j) __builtin_amdgcn_s_sleep(127);
        }
        *s_seen = v;
        if (v) {
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
            wait_stores_acked();                        // the invalidation has been performed before anyone goes on
        }
    }
    __syncthreads();
    return *s_seen;
}

// A lane's running result over the 32-bit words it has looked at.
struct ConsumeAcc {
    uint32_t m = kOrdNegInf;        // ordered key of the largest non-NaN value so far
    uint64_t sum = 0;
    __device__ __forceinline__ void take(uint32_t w) {
        sum += w;
        // NaNs drop out by their keys: those of positive NaNs lie above the key of +inf and are replaced by 0, those of
        // negative NaNs lie below the key of -inf, which m starts from
        uint32_t o = f2ord(w);
        o = o > 0xFF800000u ? 0u : o;
        m = o > m ? o : m;
    }
};

// Lane-local part: the 16-byte vectors [v0, v1) of payload, taken by the kConsumeThreads lanes of the workgroup in
// rounds of `stride` vectors (lane l takes v0 + l, v0 + l + stride, ...), plus the up to three trailing words when
// `tail` is set.  v0, v1 and stride are the same for every lane.  kConsumeInFlight loads are in flight per lane (the
// loop is latency-bound otherwise); as long as a whole round lies inside the range the addresses are a uniform base
// plus a 32-bit lane offset, which keeps the kernel at the register count of the copy kernel - a waiting consumer
// whose waves need a different amount of registers than the copy's leaves holes in the register files that no copy
// workgroup fits into, and a copy that is running when such a consumer arrives all but stops until it leaves.
__device__ __forceinline__ void consume_accumulate(ConsumeAcc &acc, const uint8_t *payload, uint64_t bytes, uint64_t v0,
                                                   uint64_t v1, uint64_t stride, bool tail) {
    constexpr uint32_t K = kConsumeInFlight;
    const uint32_t lane_off = threadIdx.x * 16u;
    uint64_t iu = v0;
    for (; iu + (K - 1) * stride + kConsumeThreads <= v1; iu += K * stride) {
        const uint8_t *q = payload + iu * 16;                            // uniform
        v4u v[K];
#pragma unroll
        for (uint32_t k = 0; k < K; ++k) v[k] = __builtin_nontemporal_load((const v4u *)(q + k * stride * 16 + lane_off));
#pragma unroll
        for (uint32_t k = 0; k < K; ++k) {
            acc.take(v[k].x); acc.take(v[k].y); acc.take(v[k].z); acc.take(v[k].w);
            __builtin_amdgcn_sched_barrier(0);           // one vector at a time: interleaving all sixteen words costs 30 registers
        }
    }
    for (uint64_t i = iu + threadIdx.x; i < v1; i += stride) {
        const v4u v = __builtin_nontemporal_load((const v4u *)payload + i);
        acc.take(v.x); acc.take(v.y); acc.take(v.z); acc.take(v.w);
    }
    if (tail) {
        const uint32_t nt = (uint32_t)((bytes & 15) >> 2);
        if (threadIdx.x < nt) acc.take(((const uint32_t *)payload)[(bytes >> 4) * 4 + threadIdx.x]);
    }
}

// Workgroup part 1: fold the lanes' results; the workgroup's result is in thread 0 afterwards.  Call with all
// kConsumeThreads lanes.
__device__ __forceinline__ void consume_fold(const ConsumeAcc &acc, uint32_t *s_max, uint64_t *s_sum, uint32_t &m, uint64_t &sum) {
    m = acc.m;
    sum = acc.sum;
    for (int off = 32; off > 0; off >>= 1) {
        const uint32_t om = __shfl_down(m, off, 64);
        const uint64_t os = __shfl_down(sum, off, 64);
        m = om > m ? om : m;
        sum += os;
    }
    __syncthreads();                                     // s_max / s_sum may still be read from an earlier fold
    if ((threadIdx.x & 63) == 0) { s_max[threadIdx.x >> 6] = m; s_sum[threadIdx.x >> 6] = sum; }
    __syncthreads();
    if (threadIdx.x < 64) {                              // the first wave folds the waves' results, one per lane
        constexpr uint32_t kWaves = kConsumeThreads / 64;
        m = threadIdx.x < kWaves ? s_max[threadIdx.x] : 0u;
        sum = threadIdx.x < kWaves ? s_sum[threadIdx.x] : 0ull;
        for (int off = kWaves / 2; off > 0; off >>= 1) {
            const uint32_t om = __shfl_down(m, off, 64);
            const uint64_t os = __shfl_down(sum, off, 64);
            m = om > m ? om : m;
            sum += os;
        }
    }
}

// Workgroup part 2: merge a workgroup's result for a tensor into *out and count `done` arrivals in; whoever brings the
// count to `needed` publishes the result.  Called by all lanes of ONE wave; each lane with `active` set brings its own
// tensor, so several tensors cost the wave the same two memory round trips as one.
// Everything the workgroups exchange goes through agent-scope atomics, which are performed where all compute dies
// meet; so no cache write-back or invalidation is needed around the arrival count, only that the lane's two
// contributions have been performed before it counts itself in.
__device__ __forceinline__ void consume_merge(bool active, rdev_consume_result *out, uint32_t m, uint64_t sum, uint32_t seen,
                                              uint32_t done, uint32_t needed) {
    if (active) {
        __hip_atomic_fetch_max((uint32_t *)&out->max, m, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __hip_atomic_fetch_add((unsigned long long *)&out->word_sum, (unsigned long long)sum, __ATOMIC_RELAXED,
                               __HIP_MEMORY_SCOPE_AGENT);
    }
    __atomic_signal_fence(__ATOMIC_SEQ_CST);
    wait_stores_acked();
    __atomic_signal_fence(__ATOMIC_SEQ_CST);
    if (active) {
        const uint32_t prev = __hip_atomic_fetch_add(&out->_arrivals, done, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (prev + done == needed) {                     // last one: publish
            const uint32_t key = __hip_atomic_load((uint32_t *)&out->max, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            ((uint32_t *)&out->max)[0] = ord2f(key);
            out->seen_flag = seen;
            out->status = 0;
        }
    }
}

__global__ __launch_bounds__(kConsumeThreads) void consume_reduce_max_kernel(const uint32_t *flag, const uint8_t *payload,
                                                                             uint64_t bytes, uint32_t max_spins,
                                                                             rdev_consume_result *out) {
    __shared__ uint32_t s_seen;
    __shared__ uint32_t s_max[kConsumeThreads / 64];
    __shared__ uint64_t s_sum[kConsumeThreads / 64];
    uint32_t seen = 0;
    if (max_spins) {
        seen = consume_wait(flag, max_spins, &s_seen);
        if (!seen) return;                              // status stays 1: every workgroup leaves
    }
    ConsumeAcc acc;
    consume_accumulate(acc, payload, bytes, (uint64_t)blockIdx.x * kConsumeThreads, bytes >> 4,
                       (uint64_t)gridDim.x * kConsumeThreads, blockIdx.x == 0);
    uint32_t m;
    uint64_t sum;
    consume_fold(acc, s_max, s_sum, m, sum);
    if (threadIdx.x < 64) consume_merge(threadIdx.x == 0, out, m, sum, seen, 1, gridDim.x);
}

// The same for a list of tensors in one launch.  A tensor is cut into units of kConsumeUnitBytes; workgroup w takes
// units w, w + grid, ... of the whole list in order, so tensors early in the list are reduced first.  A workgroup
// keeps its lanes' results across the units of one tensor; when it moves on to another tensor it folds them and puts
// the tensor's result aside, and merges the results it has put aside - up to kConsumePending, one per lane - in one
// go (merging per unit would queue thousands of atomics on the three words of a large tensor's result, merging per
// tensor costs every workgroup two memory round trips for each tensor it touches).  With max_spins > 0 a workgroup
// first waits (bounded) for the in-arena flag of each tensor it meets, which lets one launch follow a delivery that
// is still in flight: tensors whose flag is up are reduced while later ones are still moving.  Units of a tensor whose
// wait ran out are skipped; its result keeps status 1.  Every workgroup ends.
constexpr uint32_t kConsumeBatchMax = 32;
constexpr uint32_t kConsumeUnitBytes = kConsumeThreads * kConsumeInFlight * 16;     // one round of loads
constexpr uint32_t kConsumeTableMaxBlocks = 256;     // when the kernel may have to wait (waiting workgroups hold wave slots)
constexpr uint32_t kConsumePending = 8;

struct ConsumeEnt {
    const uint32_t *flag;
    const uint8_t *payload;
    uint64_t bytes;
    uint32_t first_unit;        // units of the tensors before it in the list
    uint32_t n_units;           // >= 1 (an empty tensor still gets its result published)
};
struct ConsumeBatch {
    ConsumeEnt e[kConsumeBatchMax];
    uint32_t n, n_units, max_spins, _pad;
};
struct ConsumePend {            // a workgroup's results of finished tensors that are still to be merged
    rdev_consume_result *out[kConsumePending];
    uint64_t sum[kConsumePending];
    uint32_t m[kConsumePending], seen[kConsumePending], done[kConsumePending], needed[kConsumePending];
};

__global__ __launch_bounds__(kConsumeThreads) void consume_table_kernel(ConsumeBatch b, rdev_consume_result *out) {
    __shared__ uint32_t s_seen;
    __shared__ uint32_t s_max[kConsumeThreads / 64];
    __shared__ uint64_t s_sum[kConsumeThreads / 64];
    __shared__ ConsumePend pend;
    uint32_t k = 0, cur = 0xFFFFFFFFu, seen = 0, done = 0, n_pend = 0;
    ConsumeAcc acc;
    auto merge_pending = [&]() {
        __syncthreads();
        if (threadIdx.x < 64) {
            const uint32_t j = threadIdx.x < n_pend ? threadIdx.x : 0;
            consume_merge(threadIdx.x < n_pend, pend.out[j], pend.m[j], pend.sum[j], pend.seen[j], pend.done[j], pend.needed[j]);
        }
        n_pend = 0;
    };
    auto put_aside = [&]() {                                          // tensor `cur` is finished as far as this workgroup goes
        uint32_t m;
        uint64_t sum;
        consume_fold(acc, s_max, s_sum, m, sum);
        if (threadIdx.x == 0) {
            pend.out[n_pend] = out + cur;
            pend.m[n_pend] = m;
            pend.sum[n_pend] = sum;
            pend.seen[n_pend] = seen;
            pend.done[n_pend] = done;
            pend.needed[n_pend] = b.e[cur].n_units;
        }
        if (++n_pend == kConsumePending) merge_pending();
    };
    for (uint32_t u = blockIdx.x; u < b.n_units; u += gridDim.x) {
        while (u >= b.e[k].first_unit + b.e[k].n_units) ++k;          // units ascend, so does the tensor
        if (k != cur) {                                               // on to another tensor
            if (done) put_aside();
            acc = ConsumeAcc();
            done = 0;
            cur = k;
            seen = b.max_spins ? consume_wait(b.e[k].flag, b.max_spins, &s_seen) : 0;
        }
        if (b.max_spins && !seen) continue;
        const ConsumeEnt &e = b.e[k];
        const uint32_t j = u - e.first_unit;
        const uint64_t nvec = e.bytes >> 4, per = kConsumeUnitBytes / 16;
        const uint64_t v0 = (uint64_t)j * per, v1 = v0 + per < nvec ? v0 + per : nvec;
        consume_accumulate(acc, e.payload, e.bytes, v0, v1, kConsumeThreads, j + 1 == e.n_units);
        ++done;
    }
    if (done) put_aside();
    if (n_pend) merge_pending();
}

}  // namespace rdev
