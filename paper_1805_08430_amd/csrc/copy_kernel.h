// The data mover (gfx950): pure byte movement with 16-byte vector loads/stores,
// one vector per lane per step, no LDS and no matrix cores - the work is bound by
// HBM bandwidth, so what matters is coalesced streaming access, enough loads in
// flight per compute unit, and a workgroup order that lets each XCD stream one
// contiguous part of the batch.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace rdev {

constexpr uint32_t kBlockThreads = 1024;     // 16 wavefronts
constexpr uint32_t kWavesPerBlock = kBlockThreads / 64;
constexpr uint32_t kXcds = 8;                // workgroup b is dispatched to XCD b % 8
constexpr uint32_t kInlineMax = 8;           // explicit transfers per inline launch
constexpr uint32_t kMetaInlineMax = 4;       // metadata records per launch (kernel-argument space)

// One unit of copy work.  n_sub == 0: the whole block copies (src, dst, bytes).
// n_sub > 0: wavefront w < n_sub copies sub-item [sub_first + w] (small tensors).
struct Item {
    const uint8_t *src;
    uint8_t *dst;           // always 16-byte aligned
    uint32_t bytes;
    uint32_t n_sub;
    uint32_t sub_first;
    uint32_t tensor;        // index in plan order (diagnostics only)
};
static_assert(sizeof(Item) == 32, "Item is 32 bytes");

struct InlineEnt {
    const uint8_t *src;
    uint8_t *dst;
    uint64_t bytes;
    uint32_t first_block;   // first workgroup of this transfer; it owns 8 * per_xcd workgroups
    uint32_t per_xcd;       // ceil(chunks / 8)
};
struct InlineBatch {
    InlineEnt e[kInlineMax];
    uint32_t n;
    uint32_t chunk;
};

typedef uint32_t v4u __attribute__((ext_vector_type(4)));
typedef v4u v4u_a4 __attribute__((aligned(4)));   // a 16-byte vector at a 4-byte aligned address

// The store of the data mover: a 16-byte streaming store that also writes through (sc1), so that the line does not
// wait in the L2 for a later write-back.  The compiler's non-temporal store sets "nt" only; there is no builtin for
// the write-through bit on a 16-byte store, hence the one line of assembly.  Measured on the 553 MB copy: 163.7 us
// against 167.6 us with the plain non-temporal store (loads: non-temporal is best, further bits change nothing).
// The s_nop keeps a following write of the data registers clear of the store's operand read.
__device__ __forceinline__ void store_stream(v4u *p, v4u r) {
    asm volatile("global_store_dwordx4 %0, %1, off sc1 nt\n\ts_nop 1" ::"v"(p), "v"(r) : "memory");
}

__device__ __forceinline__ uint32_t funnel(uint32_t lo, uint32_t hi, uint32_t shift_bits) {
    return (uint32_t)((((uint64_t)hi << 32) | lo) >> shift_bits);
}

// Copy `bytes` from src to dst with `nth` cooperating lanes, lane id `tid`.
// dst is 16-byte aligned.  src may have any alignment:
//   src % 16 == 0 : 16-byte loads
//   src %  4 == 0 : 16-byte loads at 4-byte alignment
//   otherwise     : five aligned dwords per vector, shifted into place (four loaded,
//                   the fifth handed over by the neighbouring lane); the extra
//                   dword always shares a word with a valid source byte, so
//                   nothing outside the source's pages is touched.
// nth must be a multiple of 64 and the lanes of a wave must hold consecutive tid.
// Streaming (non-temporal) accesses: nothing is reused.
__device__ __forceinline__ void copy_span(const uint8_t *__restrict__ src, uint8_t *__restrict__ dst,
                                          uint32_t bytes, uint32_t tid, uint32_t nth) {
    const uint32_t nvec = bytes >> 4;
    const uintptr_t sa = (uintptr_t)src;
    v4u *d = (v4u *)dst;
    if ((sa & 15) == 0) {
        const v4u *s = (const v4u *)src;
        for (uint32_t i = tid; i < nvec; i += nth)
            store_stream(d + i, __builtin_nontemporal_load(s + i));
    } else if ((sa & 3) == 0) {
        const v4u_a4 *s = (const v4u_a4 *)src;
        for (uint32_t i = tid; i < nvec; i += nth)        // same instruction, streaming as well: measured equal to the aligned case
            store_stream(d + i, (v4u)__builtin_nontemporal_load(s + i));
    } else {
        // Byte-misaligned source: vector i needs the five aligned dwords that cover it.  Four come with one 16-byte
        // load; the fifth is the first dword of vector i + 1, which the next lane has just loaded, so it is passed
        // across the wave instead of being loaded again.  Only a lane whose neighbour holds no vector (the last lane
        // of the wave, or the last vector) fetches its fifth dword itself.  The wave walks the loop as a whole.
        const uint32_t m = (uint32_t)(sa & 3);
        const uint32_t sh = m * 8;
        const uint32_t *base = (const uint32_t *)(sa - m);
        const uint32_t lane = tid & 63;
        for (uint32_t i0 = tid - lane; i0 < nvec; i0 += nth) {          // i0: this wave's first vector, same for all its lanes
            const uint32_t i = i0 + lane;
            const bool on = i < nvec;
            const uint32_t *w = base + 4 * (size_t)i;
            const bool own5 = on && (lane == 63 || i + 1 >= nvec);
            v4u lo = {0, 0, 0, 0};
            uint32_t own = 0;
            if (on) lo = __builtin_nontemporal_load((const v4u_a4 *)w);
            if (own5) own = __builtin_nontemporal_load(w + 4);          // issued before anything waits for `lo`
            uint32_t w4 = __shfl_down(lo.x, 1, 64);
            if (own5) w4 = own;
            if (on) {
                v4u r;
                r.x = funnel(lo.x, lo.y, sh);
                r.y = funnel(lo.y, lo.z, sh);
                r.z = funnel(lo.z, lo.w, sh);
                r.w = funnel(lo.w, w4, sh);
                store_stream(d + i, r);
            }
        }
    }
    const uint32_t rem = bytes & 15;
    if (tid < rem) {
        const size_t o = (size_t)nvec * 16 + tid;
        dst[o] = src[o];
    }
}

// The batched transfer: block b takes items[b].  The entry is a load that no other workgroup has made, so it comes
// from HBM in front of the payload load; on the 553 MB copy that is worth about 2.5 us (165.5 us with the dependent
// load, 163.0 us with addresses computed from the workgroup number).  Describing the largest tensors as ranges that
// a workgroup searches instead - in the kernel arguments, or in one small device record shared by all workgroups -
// was measured too and is slower than the table (186 us and 178 us): three scalar loads in a row in front of every
// workgroup's first payload load cost more than the one load they save.
__global__ __launch_bounds__(kBlockThreads) void copy_table_kernel(const Item *__restrict__ items,
                                                                    const Item *__restrict__ subs) {
    const Item it = items[blockIdx.x];
    if (it.n_sub == 0) {
        copy_span(it.src, it.dst, it.bytes, threadIdx.x, kBlockThreads);
    } else {
        const uint32_t wave = threadIdx.x >> 6;
        if (wave < it.n_sub) {
            const Item s = subs[it.sub_first + wave];
            copy_span(s.src, s.dst, s.bytes, threadIdx.x & 63, 64);
        }
    }
}

// A few explicit transfers whose descriptors travel in the kernel arguments.
__global__ __launch_bounds__(kBlockThreads) void copy_inline_kernel(InlineBatch b) {
    uint32_t k = 0;
    for (uint32_t i = 1; i < b.n; ++i)
        if (blockIdx.x >= b.e[i].first_block) k = i;
    // same XCD-contiguous order as the table: workgroup j of a transfer takes chunk (j % 8) * per_xcd + j / 8
    const uint32_t j = blockIdx.x - b.e[k].first_block;
    const uint64_t off = ((uint64_t)(j % kXcds) * b.e[k].per_xcd + j / kXcds) * b.chunk;
    if (off >= b.e[k].bytes) return;
    const uint64_t rem = b.e[k].bytes - off;
    const uint32_t n = rem < b.chunk ? (uint32_t)rem : b.chunk;
    copy_span(b.e[k].src + off, b.e[k].dst + off, n, threadIdx.x, kBlockThreads);
}

}  // namespace rdev
