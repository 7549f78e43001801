// C-ABI entry points of the memory-region device (see include/rdev.h).
// Host logic + kernel launches; the kernels are in kernels.h, the planner in planner.cpp.
#include <hip/hip_ext.h>
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstring>
#include <memory>
#include <string>
#include <unordered_map>
#include <vector>

#include "copy_table.h"
#include "kernels.h"
#include "planner.h"
#include "rdev.h"

using rdev::ArenaLayout;
using rdev::FlagEnt;
using rdev::Item;
using rdev::cut_items;
using rdev::flush_small;
using rdev::xcd_order;

namespace {

thread_local std::string g_err = "";

rdev_status fail(rdev_status st, std::string msg) {
    g_err = std::move(msg);
    return st;
}

}  // namespace

namespace rdev {
rdev_status fail_msg(rdev_status st, const std::string &msg) { return fail(st, msg); }
}  // namespace rdev

namespace {

#define HIP_TRY(expr)                                                                      \
    do {                                                                                   \
        hipError_t e_ = (expr);                                                            \
        if (e_ != hipSuccess) return fail(RDEV_E_HIP, std::string(#expr) + ": " + hipGetErrorString(e_)); \
    } while (0)

#define RDEV_TRY(expr)                 \
    do {                               \
        rdev_status s_ = (expr);       \
        if (s_ != RDEV_OK) return s_;  \
    } while (0)

struct Arena {
    uint8_t *base = nullptr;
    uint64_t bytes = 0;
    uint32_t flags = 0;
    rdev::RegionAllocator alloc;
};

struct SrcLoc {
    bool bound = false;
    uint32_t arena = 0;
    uint64_t offset = 0;
};

constexpr uint32_t kMaxArenas = 4096;                // arena ids a device hands out (ids are not reused)
constexpr uint32_t kTokenRing = 1024;                // whole-plan deliveries that may be in flight behind a completed one
constexpr uint32_t kMaxBlocksPerLaunch = 1u << 21;   // x 1024 lanes stays below 2^32 work-items per launch
constexpr uint64_t kDefaultChunk = 16384;   // one 16-byte vector per lane of a 1024-lane block
constexpr uint32_t kDefaultSmall = 4096;    // up to this size a tensor is one wavefront's work

template <typename T>
struct DevBuf {                               // library-owned device table
    T *ptr = nullptr;
    size_t n = 0;
    ~DevBuf() { reset(); }
    void reset() {
        if (ptr) (void)hipFree(ptr);
        ptr = nullptr;
        n = 0;
    }
    hipError_t upload(const std::vector<T> &h) {
        reset();
        if (h.empty()) return hipSuccess;
        hipError_t e = hipMalloc((void **)&ptr, h.size() * sizeof(T));
        if (e != hipSuccess) { ptr = nullptr; return e; }
        n = h.size();
        return hipMemcpy(ptr, h.data(), h.size() * sizeof(T), hipMemcpyHostToDevice);
    }
};

}  // namespace

// Staging memory of rdev_write_batch_fixed_staging: part of the library's device image, so that entry
// point never allocates.  Every GPU the library runs on holds its own copy until the process ends.  In host
// code this name only stands for the symbol; the device address is looked up once per device in rdev_open.
static __device__ __align__(256) uint8_t scratch[RDEV_FIXED_STAGING_BYTES];

struct rdev_device_s {
    int hip_device = RDEV_HOST_ONLY;
    std::vector<Arena> arenas;
    int n_plans = 0;
    uint8_t *fixed_staging = nullptr;     // device address of `scratch` on hip_device
    rdev::ArenaEnt *d_arenas = nullptr;   // device copy of (base, bytes) per arena id, kMaxArenas entries (GPU devices)
    bool gpu() const { return hip_device >= 0; }
};

struct rdev_plan_s {
    rdev_device_t *dev = nullptr;
    rdev_plan_opts opts{};
    std::vector<rdev_tensor_desc> descs;
    std::vector<rdev_placement> pl;
    std::unordered_map<uint32_t, uint32_t> by_id;    // tensor_id -> index
    std::map<uint32_t, ArenaLayout> arenas;          // destination arena -> layout
    std::vector<rdev_region> blocks;                 // what was taken from the sub-allocators
    std::vector<SrcLoc> src;                         // bound sources, by index
    std::vector<int32_t> dyn_index;                  // index -> slot in the metadata mirror, -1 if static
    uint32_t n_dyn = 0;
    uint32_t n_static = 0;
    bool bound_all = false;

    // device tables for the "whole plan" transfer
    DevBuf<Item> d_items, d_subs;
    DevBuf<FlagEnt> d_flags;                         // static tensors, plan order
    std::vector<uint32_t *> h_flag_ptrs;             // the same in-arena flag addresses, host copy
    uint32_t n_blocks = 0;

    // host-visible words: flags[2*i] = completion / payload-complete, flags[2*i+1] = metadata flag
    uint32_t *h_flags = nullptr, *d_flags_view = nullptr;
    // whole-plan deliveries are announced to the host by one word: h_flags[2*n] holds the token of the
    // last one completed; a static tensor is ready when that token differs from the one it consumed
    // With flag_groups = G the static tensors (plan order) form G consecutive groups of about equal bytes;
    // group g has its own launch, its own slice of the flag table and its own token word h_batch[g].
    struct Group { uint32_t first_block = 0, n_blocks = 0, first_flag = 0, n_flags = 0; };
    std::vector<Group> groups;
    std::vector<uint32_t> group_of;                  // per index (static tensors)
    uint32_t *h_batch = nullptr, *d_batch_view = nullptr;
    uint32_t issued_token = 0;
    uint32_t seq_ring[kTokenRing] = {0};             // flag value (seq) of the delivery that carried each recent token
    std::vector<uint32_t> consumed_token;
    rdev_meta *h_meta = nullptr, *d_meta_view = nullptr;
    std::vector<rdev_meta> polled;                   // record seen by the last metadata poll
    std::vector<uint8_t> polled_valid;
    std::vector<uint32_t> tok_scratch;               // rdev_poll(RDEV_ALL_TENSORS): token observed per tensor
    std::vector<uint64_t> rpc_offset;                // per index: fresh allocation of the last RPC-mode delivery
    std::vector<uint8_t> rpc_valid;

    // receives that take their sizes on the device (rdev_read_batch_device)
    DevBuf<rdev::HeapWord> d_heap;                   // one bump pointer per destination arena, in map order
    DevBuf<uint32_t> d_recv_arrivals;                // workgroups of the running receive kernel that are done; 0 between launches
    std::map<uint32_t, uint32_t> heap_word_of;       // destination arena -> index in d_heap
    uint32_t heap_epoch = 1;                         // iteration number; rdev_dyn_reset starts the next one
    bool heap_on_device = false;                     // this iteration's allocations are known to the device only
    uint32_t *h_status = nullptr, *d_status_view = nullptr;   // pinned: code, entry, call id of the last device receive
    uint32_t recv_calls = 0;

    // the in-arena clear of a consume may travel on another stream than the deliveries (the receiver's own queue)
    hipStream_t delivery_stream = nullptr;
    hipStream_t clear_stream = nullptr;
    hipEvent_t ev_clear = nullptr;
    bool clear_pending = false;

    // optional timing of the batched copy kernel
    std::vector<hipEvent_t> ev_start, ev_stop;
    uint32_t ev_used = 0, ev_every = 1, ev_count = 0;

    // buffers and tables of the copying modes (built on first use)
    bool have_send = false, have_recv = false;
    rdev_region send_buf{}, recv_buf{};
    bool copy_tables = false;
    uint64_t msg_total = 0;                          // packed bytes of the whole plan
    uint64_t stage_end = 0;                          // end of the last staged tensor
    std::vector<uint32_t> heap_slot_arena;           // heap slot -> destination arena
    std::vector<uint64_t> heap_need;                 // per slot: fresh-allocation bytes of one whole-plan delivery
    std::vector<uint64_t> rpc_rel;                   // per index: offset inside the slot's area
    std::vector<uint32_t> rpc_slot;                  // per index
    DevBuf<Item> d_pack_items, d_pack_subs, d_stage_items, d_stage_subs, d_unstage_items, d_unstage_subs;
    DevBuf<rdev::UItem> d_unpack_send_items, d_unpack_send_subs, d_unpack_recv_items, d_unpack_recv_subs;
    DevBuf<rdev_meta> d_headers;
    DevBuf<uint8_t *> d_msg_send, d_msg_recv;
    DevBuf<rdev_frag> d_frags;                       // fragmented messages: one header per fragment
    DevBuf<uint8_t *> d_frag_send;
    uint32_t n_frags = 0;
    uint32_t n_pack_blocks = 0, n_stage_blocks = 0, n_unpack_blocks = 0;
};

struct rdev_tracer_s {
    rdev_device_t *dev = nullptr;
    uint8_t *pool_base = nullptr;
    uint64_t pool_bytes = 0;
    uint32_t arena_id = 0;
    rdev::RegionAllocator pool;
    uint32_t iteration = 0;                                             // 0 = none begun yet
    std::map<uint32_t, uint32_t> next_index;                            // node -> allocations so far this iteration
    std::map<uintptr_t, std::pair<uint32_t, uint32_t>> site_of;         // address -> (node, index), last writer wins
    std::vector<std::pair<uint32_t, uint32_t>> S;                       // insertion order
    std::map<std::pair<uint32_t, uint32_t>, bool> in_S;
    struct Buf { uint64_t offset, bytes; bool arena; };
    std::map<uintptr_t, Buf> live;                                      // buffers handed out, by address
    std::vector<rdev_region> staging;                                   // staging regions of this iteration
};

namespace {

rdev_status arena_of(rdev_device_t *dev, uint32_t id, Arena **out) {
    if (id >= dev->arenas.size() || !dev->arenas[id].bytes) return fail(RDEV_E_INVAL, "unknown arena " + std::to_string(id));
    *out = &dev->arenas[id];
    return RDEV_OK;
}

// which registered arena holds [p, p+bytes)?
rdev_status locate(rdev_device_t *dev, const void *p, uint64_t bytes, SrcLoc *out) {
    const uintptr_t a = (uintptr_t)p;
    for (uint32_t i = 0; i < dev->arenas.size(); ++i) {
        const Arena &ar = dev->arenas[i];
        const uintptr_t lo = (uintptr_t)ar.base;
        if (!ar.base || a < lo || a - lo > ar.bytes) continue;
        if (bytes > ar.bytes - (a - lo)) continue;
        out->bound = true;
        out->arena = i;
        out->offset = a - lo;
        return RDEV_OK;
    }
    return fail(RDEV_E_RANGE, "address range is not inside a registered arena");
}

bool ranges_overlap(uint32_t a0, uint64_t o0, uint32_t a1, uint64_t o1, uint64_t bytes) {
    return bytes && a0 == a1 && o0 < o1 + bytes && o1 < o0 + bytes;
}

rdev_status index_of(const rdev_plan_t *plan, uint32_t tensor_id, uint32_t *idx) {
    auto it = plan->by_id.find(tensor_id);
    if (it == plan->by_id.end()) return fail(RDEV_E_INVAL, "unknown tensor " + std::to_string(tensor_id));
    *idx = it->second;
    return RDEV_OK;
}

uint8_t *arena_ptr(rdev_plan_t *plan, uint32_t arena, uint64_t off) { return plan->dev->arenas[arena].base + off; }

// What a static tensor's completion shows to the host: its flag value, 0 = not ready.
// *tok_out (may be NULL) = the delivery token this answer was read from; a consume must record exactly
// that token, so that a delivery landing between the test and the consume is not swallowed.
// *stale_out (may be NULL) is set when the tensor is ready but so many whole-plan deliveries have been
// issued since the completed one that its ring slot was recycled: the flag value is then unknown.
uint32_t static_ready(const rdev_plan_t *plan, uint32_t i, uint32_t *tok_out = nullptr, bool *stale_out = nullptr) {
    const uint32_t tok = __atomic_load_n(plan->h_batch + plan->group_of[i], __ATOMIC_ACQUIRE);
    if (tok_out) *tok_out = tok;
    const uint32_t v = __atomic_load_n(&plan->h_flags[2 * i], __ATOMIC_ACQUIRE);
    if (v) return v;
    if (tok == plan->consumed_token[i]) return 0;
    if (plan->issued_token - tok >= kTokenRing) {
        if (stale_out) *stale_out = true;
        return 1;
    }
    return plan->seq_ring[tok % kTokenRing];
}

void static_consume(rdev_plan_t *plan, uint32_t i, uint32_t tok) {
    __atomic_store_n(&plan->h_flags[2 * i], 0u, __ATOMIC_RELEASE);
    plan->consumed_token[i] = tok;
}

uint32_t next_token(rdev_plan_t *plan, uint32_t seq) {
    if (++plan->issued_token == 0) ++plan->issued_token;      // 0 means "nothing delivered yet"
    plan->seq_ring[plan->issued_token % kTokenRing] = seq;
    return plan->issued_token;
}

rdev_status stale_error() {
    return fail(RDEV_E_STATE, "more than " + std::to_string(kTokenRing - 1) + " whole-plan deliveries were issued behind the "
                              "completed one: its flag value is no longer known (consume, or wait, more often)");
}

rdev_status launch_check(const char *what) {
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(RDEV_E_HIP, std::string(what) + ": " + hipGetErrorString(e));
    return RDEV_OK;
}

// A delivery on stream s is about to be enqueued.  If the receiver's last clear of this plan's flags travelled on
// another stream and may still be pending, s waits for it: a late clear must not wipe the flags of this delivery.
rdev_status before_delivery(rdev_plan_t *plan, hipStream_t s) {
    if (plan->clear_pending && plan->clear_stream != s) {
        // The clear is one tiny kernel that was enqueued on an otherwise idle stream: it is normally done by now, or
        // within microseconds.  Ask on the host for a short while first; a wait inside stream s is the fallback, as
        // a cross-stream dependency costs the delivery more than the clear itself takes.
        hipError_t q = hipErrorNotReady;
        for (int spin = 0; spin < 100 && q == hipErrorNotReady; ++spin) q = hipEventQuery(plan->ev_clear);
        if (q == hipErrorNotReady) {
            (void)hipGetLastError();
            HIP_TRY(hipStreamWaitEvent(s, plan->ev_clear, 0));
        } else if (q != hipSuccess) {
            return fail(RDEV_E_HIP, std::string("hipEventQuery: ") + hipGetErrorString(q));
        }
        (void)hipGetLastError();
    }
    plan->clear_pending = false;
    plan->delivery_stream = s;
    return RDEV_OK;
}

// A clear of in-arena flag words has just been enqueued on stream s.  The host-visible word that made the receiver
// consume is stored after the in-arena words it stands for, so the clear needs no wait of its own; the next
// delivery does (before_delivery) when s is not the stream it travels on.
rdev_status after_clear(rdev_plan_t *plan, hipStream_t s) {
    if (s == plan->delivery_stream) return RDEV_OK;
    HIP_TRY(hipEventRecord(plan->ev_clear, s));
    plan->clear_pending = true;
    plan->clear_stream = s;
    return RDEV_OK;
}

// one table of work items, in as many launches as the per-launch limit asks for (workgroups are independent)
rdev_status launch_copy_table(const Item *items, const Item *subs, uint32_t n_blocks, hipStream_t s, const char *what) {
    for (uint32_t first = 0; first < n_blocks; first += kMaxBlocksPerLaunch) {
        const uint32_t n = std::min(kMaxBlocksPerLaunch, n_blocks - first);
        hipLaunchKernelGGL(rdev::copy_table_kernel, dim3(n), dim3(rdev::kBlockThreads), 0, s, items + first, subs);
        RDEV_TRY(launch_check(what));
    }
    return RDEV_OK;
}

// flags of one group (in-arena words <- seq, the group's host word <- token)
rdev_status launch_group_flags(rdev_plan_t *plan, uint32_t g, uint32_t seq, uint32_t token, hipStream_t s) {
    const rdev_plan_s::Group &gr = plan->groups[g];
    if (!gr.n_flags) return RDEV_OK;
    if (gr.n_flags <= rdev::kFlagInlineMax) {        // few enough to travel in the kernel arguments
        rdev::InlineFlags f{};
        f.value = seq;
        f.n = gr.n_flags;
        for (uint32_t k = 0; k < gr.n_flags; ++k) f.arena_flag[k] = plan->h_flag_ptrs[gr.first_flag + k];
        hipLaunchKernelGGL(rdev::flag_inline_kernel, dim3(1), dim3(64), 0, s, f, (uint32_t *)nullptr,
                           plan->d_batch_view + g, token);
        return launch_check("flag_inline_kernel");
    }
    hipLaunchKernelGGL(rdev::flag_table_kernel, dim3(1), dim3(rdev::kFlagTableThreads), 0, s,
                       plan->d_flags.ptr + gr.first_flag, gr.n_flags, seq, plan->d_batch_view + g, token);
    return launch_check("flag_table_kernel");
}

rdev_status require_gpu(const rdev_device_t *dev) {
    if (!dev->gpu()) return fail(RDEV_E_HIP, "host-only device: no GPU to run a transfer on");
    return RDEV_OK;
}

struct ResolvedStatic {
    uint32_t idx;
    const uint8_t *src;
    uint8_t *dst;
    uint64_t bytes;
};

// validate one static transfer and resolve its addresses
rdev_status resolve_static(rdev_plan_t *plan, uint32_t idx, const void *src_override, ResolvedStatic *out) {
    const rdev_placement &p = plan->pl[idx];
    SrcLoc loc;
    if (src_override) {
        RDEV_TRY(locate(plan->dev, src_override, p.bytes, &loc));
    } else {
        loc = plan->src[idx];
        if (!loc.bound) return fail(RDEV_E_STATE, "tensor " + std::to_string(p.tensor_id) + " has no bound source");
    }
    if (ranges_overlap(loc.arena, loc.offset, p.dst_arena, p.data_offset, p.bytes))
        return fail(RDEV_E_OVERLAP, "source of tensor " + std::to_string(p.tensor_id) + " overlaps its destination");
    out->idx = idx;
    out->src = plan->dev->arenas[loc.arena].base + loc.offset;
    out->dst = arena_ptr(plan, p.dst_arena, p.data_offset);
    out->bytes = p.bytes;
    return RDEV_OK;
}

// enqueue copies for up to any number of resolved transfers, kInlineMax per launch
rdev_status launch_inline_copies(rdev_plan_t *plan, const std::vector<ResolvedStatic> &in, hipStream_t s) {
    const uint64_t chunk = plan->opts.chunk_bytes;
    // a transfer that alone exceeds the per-launch limit is cut into pieces that fit
    const uint64_t piece = (uint64_t)(kMaxBlocksPerLaunch - rdev::kXcds) * chunk;
    std::vector<ResolvedStatic> v;
    for (const ResolvedStatic &r : in) {
        for (uint64_t off = 0; off < r.bytes || (off == 0 && r.bytes == 0); off += piece) {
            v.push_back(ResolvedStatic{r.idx, r.src + off, r.dst + off, std::min(piece, r.bytes - off)});
            if (!r.bytes) break;
        }
    }
    size_t i = 0;
    while (i < v.size()) {
        rdev::InlineBatch b{};
        b.chunk = (uint32_t)chunk;
        uint64_t blocks = 0;
        while (i < v.size() && b.n < rdev::kInlineMax) {
            const uint64_t per = ((v[i].bytes + chunk - 1) / chunk + rdev::kXcds - 1) / rdev::kXcds;
            const uint64_t nb = per * rdev::kXcds;
            if (blocks + nb > kMaxBlocksPerLaunch && b.n) break;      // next launch
            if (nb) {
                b.e[b.n] = rdev::InlineEnt{v[i].src, v[i].dst, v[i].bytes, (uint32_t)blocks, (uint32_t)per};
                b.n++;
                blocks += nb;
            }
            ++i;
        }
        if (blocks) {
            hipLaunchKernelGGL(rdev::copy_inline_kernel, dim3((uint32_t)blocks), dim3(rdev::kBlockThreads), 0, s, b);
            RDEV_TRY(launch_check("copy_inline_kernel"));
        }
    }
    return RDEV_OK;
}

// flag words (in arena + host-visible) <- value, for a list of (arena pointer, mirror index)
rdev_status launch_inline_flags(rdev_plan_t *plan, const std::vector<std::pair<uint32_t *, uint32_t>> &v,
                                uint32_t value, bool with_mirror, hipStream_t s) {
    size_t i = 0;
    while (i < v.size()) {
        rdev::InlineFlags f{};
        f.value = value;
        while (i < v.size() && f.n < rdev::kFlagInlineMax) {
            f.arena_flag[f.n] = v[i].first;
            f.mirror_idx[f.n] = v[i].second;
            f.n++;
            ++i;
        }
        hipLaunchKernelGGL(rdev::flag_inline_kernel, dim3(1), dim3(64), 0, s, f,
                           with_mirror ? plan->d_flags_view : nullptr, (uint32_t *)nullptr, 0u);
        RDEV_TRY(launch_check("flag_inline_kernel"));
    }
    return RDEV_OK;
}

void free_plan_blocks(rdev_plan_t *plan) {
    std::string ignore;
    for (const rdev_region &r : plan->blocks) plan->dev->arenas[r.arena_id].alloc.release(r.offset, r.bytes, ignore);
    plan->blocks.clear();
}

void drop_events(rdev_plan_t *plan) {
    for (hipEvent_t e : plan->ev_start) (void)hipEventDestroy(e);
    for (hipEvent_t e : plan->ev_stop) (void)hipEventDestroy(e);
    plan->ev_start.clear();
    plan->ev_stop.clear();
    plan->ev_used = 0;
}

void destroy_plan(rdev_plan_t *plan) {
    free_plan_blocks(plan);
    drop_events(plan);
    if (plan->ev_clear) (void)hipEventDestroy(plan->ev_clear);
    if (plan->h_flags) (void)hipHostFree(plan->h_flags);
    if (plan->h_meta) (void)hipHostFree(plan->h_meta);
    plan->dev->n_plans--;
    delete plan;
}

}  // namespace

extern "C" {

const char *rdev_last_error(void) { return g_err.c_str(); }

void rdev_abi_sizes(uint32_t out[6]) {
    out[0] = sizeof(rdev_tensor_desc);
    out[1] = sizeof(rdev_placement);
    out[2] = sizeof(rdev_plan_opts);
    out[3] = sizeof(rdev_meta);
    out[4] = sizeof(rdev_xfer);
    out[5] = sizeof(rdev_region);
}

rdev_status rdev_open(rdev_device_t **out, int hip_device) {
    if (!out) return fail(RDEV_E_INVAL, "out is NULL");
    if (hip_device < RDEV_HOST_ONLY) return fail(RDEV_E_INVAL, "bad device index");
    if (hip_device >= 0) {
        int n = 0;
        HIP_TRY(hipGetDeviceCount(&n));
        if (hip_device >= n) return fail(RDEV_E_HIP, "no such HIP device");
        HIP_TRY(hipSetDevice(hip_device));
    }
    uint8_t *staging = nullptr;
    rdev::ArenaEnt *d_arenas = nullptr;
    if (hip_device >= 0) {
        HIP_TRY(hipGetSymbolAddress((void **)&staging, HIP_SYMBOL(scratch)));   // this device's copy
        HIP_TRY(hipMalloc((void **)&d_arenas, kMaxArenas * sizeof(rdev::ArenaEnt)));
        hipError_t e = hipMemset(d_arenas, 0, kMaxArenas * sizeof(rdev::ArenaEnt));
        if (e != hipSuccess) { (void)hipFree(d_arenas); return fail(RDEV_E_HIP, std::string("hipMemset: ") + hipGetErrorString(e)); }
    }
    rdev_device_t *d = new rdev_device_t();
    d->hip_device = hip_device;
    d->fixed_staging = staging;
    d->d_arenas = d_arenas;
    *out = d;
    return RDEV_OK;
}

rdev_status rdev_close(rdev_device_t *dev) {
    if (!dev) return fail(RDEV_E_INVAL, "dev is NULL");
    if (dev->n_plans) return fail(RDEV_E_BUSY, "plans are still alive on this device");
    if (dev->d_arenas) (void)hipFree(dev->d_arenas);
    delete dev;
    return RDEV_OK;
}

rdev_status rdev_register_arena(rdev_device_t *dev, void *base, uint64_t bytes, uint32_t arena_flags,
                                uint32_t *arena_id_out) {
    if (!dev || !arena_id_out) return fail(RDEV_E_INVAL, "NULL argument");
    if (arena_flags) return fail(RDEV_E_INVAL, "unknown arena flags");
    if (!bytes) return fail(RDEV_E_INVAL, "arena bytes must be positive");
    if (dev->gpu() && !base) return fail(RDEV_E_INVAL, "arena base is NULL");
    if ((uintptr_t)base & 255) return fail(RDEV_E_ALIGN, "arena base must be 256-byte aligned");
    if (base && (uintptr_t)base + bytes < (uintptr_t)base) return fail(RDEV_E_OVERFLOW, "arena wraps the address space");
    for (const Arena &a : dev->arenas) {
        if (!a.base || !base) continue;
        const uintptr_t lo = (uintptr_t)a.base, hi = lo + a.bytes, l2 = (uintptr_t)base, h2 = l2 + bytes;
        if (l2 < hi && lo < h2) return fail(RDEV_E_OVERLAP, "arena overlaps a registered arena");
    }
    if (dev->arenas.size() >= kMaxArenas) return fail(RDEV_E_NOMEM, "a device registers at most " + std::to_string(kMaxArenas) + " arenas over its lifetime");
    if (dev->gpu()) {      // the device-side copy used by receives that read the sender's address on the GPU
        const rdev::ArenaEnt ent{(uint8_t *)base, bytes};
        HIP_TRY(hipSetDevice(dev->hip_device));
        HIP_TRY(hipMemcpy(dev->d_arenas + dev->arenas.size(), &ent, sizeof(ent), hipMemcpyHostToDevice));
    }
    Arena a;
    a.base = (uint8_t *)base;
    a.bytes = bytes;
    a.flags = arena_flags;
    a.alloc = rdev::RegionAllocator(bytes);
    dev->arenas.push_back(std::move(a));
    *arena_id_out = (uint32_t)dev->arenas.size() - 1;
    return RDEV_OK;
}

rdev_status rdev_unregister_arena(rdev_device_t *dev, uint32_t arena_id) {
    if (!dev) return fail(RDEV_E_INVAL, "NULL argument");
    Arena *a;
    RDEV_TRY(arena_of(dev, arena_id, &a));
    if (a->alloc.live()) return fail(RDEV_E_BUSY, "regions are still allocated in arena " + std::to_string(arena_id));
    if (dev->gpu()) {
        const rdev::ArenaEnt none{nullptr, 0};
        HIP_TRY(hipSetDevice(dev->hip_device));
        HIP_TRY(hipMemcpy(dev->d_arenas + arena_id, &none, sizeof(none), hipMemcpyHostToDevice));
    }
    *a = Arena();
    return RDEV_OK;
}

rdev_status rdev_alloc_region(rdev_device_t *dev, uint32_t arena_id, uint64_t bytes, uint64_t align, rdev_region *out) {
    if (!dev || !out) return fail(RDEV_E_INVAL, "NULL argument");
    Arena *a;
    RDEV_TRY(arena_of(dev, arena_id, &a));
    uint64_t off;
    std::string err;
    rdev_status st = a->alloc.alloc(bytes, align, &off, err);
    if (st != RDEV_OK) return fail(st, err);
    out->arena_id = arena_id;
    out->_pad = 0;
    out->offset = off;
    out->bytes = bytes;
    return RDEV_OK;
}

rdev_status rdev_free_region(rdev_device_t *dev, const rdev_region *region) {
    if (!dev || !region) return fail(RDEV_E_INVAL, "NULL argument");
    Arena *a;
    RDEV_TRY(arena_of(dev, region->arena_id, &a));
    std::string err;
    rdev_status st = a->alloc.release(region->offset, region->bytes, err);
    if (st != RDEV_OK) return fail(st, err);
    return RDEV_OK;
}

rdev_status rdev_plan(rdev_device_t *dev, const rdev_tensor_desc *t, uint32_t n, const rdev_plan_opts *opts,
                      rdev_plan_t **plan_out) {
    if (!dev || !plan_out || (!t && n)) return fail(RDEV_E_INVAL, "NULL argument");
    rdev_plan_opts o{};
    if (opts) o = *opts;
    if (!o.align) o.align = RDEV_DEFAULT_ALIGN;
    if (!o.chunk_bytes) o.chunk_bytes = kDefaultChunk;
    if (!o.small_bytes) o.small_bytes = kDefaultSmall;
    if (o.chunk_bytes % 256 || o.chunk_bytes > (1u << 30)) return fail(RDEV_E_INVAL, "chunk_bytes must be a multiple of 256, at most 1 GiB");
    if (o.small_bytes > o.chunk_bytes) o.small_bytes = (uint32_t)o.chunk_bytes;
    if (o.flags & ~(uint32_t)RDEV_PLAN_CHECK_BUSY) return fail(RDEV_E_INVAL, "unknown plan flags");
    if (o.rpc_frag_bytes % 16 || o.rpc_frag_bytes > 0xFFFFFFF0ull) return fail(RDEV_E_INVAL, "rpc_frag_bytes must be a multiple of 16 below 4 GiB");

    if (!o.flag_groups) o.flag_groups = 1;
    if (o.flag_groups > 1024) return fail(RDEV_E_INVAL, "flag_groups must be at most 1024");

    std::unique_ptr<rdev_plan_t> plan(new rdev_plan_t());
    plan->dev = dev;
    plan->opts = o;
    std::string err;
    rdev_status st = rdev::layout(t, n, o.align, o.max_static_bytes, o.dyn_heap_bytes, plan->pl, plan->arenas, err);
    if (st != RDEV_OK) return fail(st, err);
    for (auto &kv : plan->arenas)
        if (kv.first >= dev->arenas.size() || !dev->arenas[kv.first].bytes)
            return fail(RDEV_E_INVAL, "unknown arena " + std::to_string(kv.first));

    // one block per destination arena from its sub-allocator (ascending arena id)
    for (auto &kv : plan->arenas) {
        ArenaLayout &al = kv.second;
        if (!al.total()) continue;
        uint64_t base;
        st = dev->arenas[kv.first].alloc.alloc(al.total(), o.align, &base, err);
        if (st != RDEV_OK) {
            free_plan_blocks(plan.get());
            return fail(st, "arena " + std::to_string(kv.first) + ": " + err);
        }
        plan->blocks.push_back(rdev_region{kv.first, 0, base, al.total()});
        al.base = base;
        al.heap_offset += base;
    }
    plan->descs.assign(t, t + n);
    plan->src.resize(n);
    plan->dyn_index.assign(n, -1);
    plan->rpc_offset.assign(n, 0);
    plan->rpc_valid.assign(n, 0);
    for (uint32_t i = 0; i < n; ++i) {
        rdev_placement &p = plan->pl[i];
        const uint64_t b = plan->arenas[p.dst_arena].base;
        if (p.kind == RDEV_STATIC) { p.data_offset += b; plan->n_static++; }
        else { p.meta_offset += b; plan->dyn_index[i] = (int32_t)plan->n_dyn++; }
        p.flag_offset += b;
        plan->by_id[p.tensor_id] = i;
    }
    plan->polled.resize(plan->n_dyn);
    plan->polled_valid.assign(plan->n_dyn, 0);
    {   // groups: cut the static tensors, in plan order, where the running byte count passes k/G of the total
        uint64_t total = 0, run = 0;
        for (uint32_t i = 0; i < n; ++i) if (plan->pl[i].kind == RDEV_STATIC) total += plan->pl[i].bytes;
        const uint32_t G = o.flag_groups;
        plan->groups.assign(G, rdev_plan_s::Group());
        plan->group_of.assign(n, 0);
        uint32_t g = 0, flag_i = 0;
        for (uint32_t i = 0; i < n; ++i) {
            if (plan->pl[i].kind != RDEV_STATIC) continue;
            while (g + 1 < G && total && run >= (__uint128_t)total * (g + 1) / G) ++g;
            plan->group_of[i] = g;
            if (!plan->groups[g].n_flags) plan->groups[g].first_flag = flag_i;
            plan->groups[g].n_flags++;
            run += plan->pl[i].bytes;
            ++flag_i;
        }
    }

    dev->n_plans++;              // from here on destroy_plan() undoes everything
    rdev_plan_t *raw = plan.release();
    if (dev->gpu()) {
        auto bail = [&](hipError_t e, const char *what) {
            destroy_plan(raw);
            return fail(RDEV_E_HIP, std::string(what) + ": " + hipGetErrorString(e));
        };
        hipError_t e = hipSetDevice(dev->hip_device);
        if (e != hipSuccess) return bail(e, "hipSetDevice");
        const size_t nflags = 2 * (size_t)n + o.flag_groups + 8;     // per-tensor pairs, group tokens, receive status
        e = hipHostMalloc((void **)&raw->h_flags, nflags * sizeof(uint32_t), hipHostMallocMapped | hipHostMallocCoherent);
        if (e != hipSuccess) { raw->h_flags = nullptr; return bail(e, "hipHostMalloc(flags)"); }
        std::memset(raw->h_flags, 0, nflags * sizeof(uint32_t));
        e = hipHostGetDevicePointer((void **)&raw->d_flags_view, raw->h_flags, 0);
        if (e != hipSuccess) return bail(e, "hipHostGetDevicePointer(flags)");
        raw->h_batch = raw->h_flags + 2 * (size_t)n;
        raw->d_batch_view = raw->d_flags_view + 2 * (size_t)n;
        raw->h_status = raw->h_batch + o.flag_groups;
        raw->d_status_view = raw->d_batch_view + o.flag_groups;
        e = hipEventCreateWithFlags(&raw->ev_clear, hipEventDisableTiming);
        if (e != hipSuccess) { raw->ev_clear = nullptr; return bail(e, "hipEventCreate"); }
        {
            uint32_t w = 0;
            for (auto &kv : raw->arenas) raw->heap_word_of[kv.first] = w++;
            e = raw->d_heap.upload(std::vector<rdev::HeapWord>(std::max<size_t>(w, 1), rdev::HeapWord{0, 0, 0}));
            if (e != hipSuccess) return bail(e, "upload(heap words)");
            e = raw->d_recv_arrivals.upload(std::vector<uint32_t>(1, 0u));
            if (e != hipSuccess) return bail(e, "upload(receive arrival count)");
        }
        raw->consumed_token.assign(n, 0);
        const size_t nmeta = std::max<size_t>(raw->n_dyn, 1);
        e = hipHostMalloc((void **)&raw->h_meta, nmeta * sizeof(rdev_meta), hipHostMallocMapped | hipHostMallocCoherent);
        if (e != hipSuccess) { raw->h_meta = nullptr; return bail(e, "hipHostMalloc(meta)"); }
        std::memset(raw->h_meta, 0, nmeta * sizeof(rdev_meta));
        e = hipHostGetDevicePointer((void **)&raw->d_meta_view, raw->h_meta, 0);
        if (e != hipSuccess) return bail(e, "hipHostGetDevicePointer(meta)");

        // flag table of the static tensors; clear every flag word and metadata slot
        std::vector<FlagEnt> fe;
        for (uint32_t i = 0; i < n; ++i) {
            const rdev_placement &p = raw->pl[i];
            if (p.kind == RDEV_STATIC) {
                fe.push_back(FlagEnt{(uint32_t *)arena_ptr(raw, p.dst_arena, p.flag_offset), 2 * i, 0});
            } else {
                e = hipMemset(arena_ptr(raw, p.dst_arena, p.meta_offset), 0, RDEV_META_BYTES);
                if (e != hipSuccess) return bail(e, "hipMemset(metadata slot)");
            }
        }
        for (const FlagEnt &f : fe) raw->h_flag_ptrs.push_back(f.arena_flag);
        e = raw->d_flags.upload(fe);
        if (e != hipSuccess) return bail(e, "upload(flag table)");
        if (!fe.empty()) {
            hipLaunchKernelGGL(rdev::flag_table_kernel, dim3(1), dim3(rdev::kFlagTableThreads), 0, 0,
                               raw->d_flags.ptr, (uint32_t)fe.size(), 0u, (uint32_t *)nullptr, 0u);
            e = hipGetLastError();
            if (e != hipSuccess) return bail(e, "flag_table_kernel");
        }
        e = hipDeviceSynchronize();
        if (e != hipSuccess) return bail(e, "hipDeviceSynchronize");
    }
    *plan_out = raw;
    return RDEV_OK;
}

rdev_status rdev_plan_count(const rdev_plan_t *plan, uint32_t *n_out) {
    if (!plan || !n_out) return fail(RDEV_E_INVAL, "NULL argument");
    *n_out = (uint32_t)plan->pl.size();
    return RDEV_OK;
}

rdev_status rdev_plan_get(const rdev_plan_t *plan, uint32_t i, rdev_placement *out) {
    if (!plan || !out) return fail(RDEV_E_INVAL, "NULL argument");
    if (i >= plan->pl.size()) return fail(RDEV_E_INVAL, "placement index out of range");
    *out = plan->pl[i];
    return RDEV_OK;
}

rdev_status rdev_plan_arena_info(const rdev_plan_t *plan, uint32_t arena_id, uint64_t *base, uint64_t *static_bytes,
                                 uint64_t *heap_offset, uint64_t *heap_bytes) {
    if (!plan) return fail(RDEV_E_INVAL, "NULL argument");
    auto it = plan->arenas.find(arena_id);
    if (it == plan->arenas.end()) return fail(RDEV_E_INVAL, "arena is not a destination of this plan");
    if (base) *base = it->second.base;
    if (static_bytes) *static_bytes = it->second.static_bytes;
    if (heap_offset) *heap_offset = it->second.heap_offset;
    if (heap_bytes) *heap_bytes = it->second.heap_bytes;
    return RDEV_OK;
}

rdev_status rdev_plan_bind_sources(rdev_plan_t *plan, const void *const *src_ptrs, uint32_t n) {
    if (!plan || (!src_ptrs && n)) return fail(RDEV_E_INVAL, "NULL argument");
    if (n != plan->pl.size()) return fail(RDEV_E_INVAL, "need one source pointer per planned tensor");
    std::vector<SrcLoc> locs(n);
    bool all = true;
    for (uint32_t i = 0; i < n; ++i) {
        const rdev_placement &p = plan->pl[i];
        if (p.kind != RDEV_STATIC) continue;
        if (!src_ptrs[i]) { all = false; continue; }
        if (plan->dev->gpu() || plan->dev->arenas.size()) {
            RDEV_TRY(locate(plan->dev, src_ptrs[i], p.bytes, &locs[i]));
        }
        if (ranges_overlap(locs[i].arena, locs[i].offset, p.dst_arena, p.data_offset, p.bytes))
            return fail(RDEV_E_OVERLAP, "source of tensor " + std::to_string(p.tensor_id) + " overlaps its destination");
    }
    // descriptor table (section 3.4: the sender keeps each destination address with the sending node)
    std::vector<Item> items, subs;
    for (uint32_t g = 0; g < plan->groups.size(); ++g) {
        std::vector<Item> gi, pending;
        for (uint32_t i = 0; i < n; ++i) {
            const rdev_placement &p = plan->pl[i];
            if (p.kind != RDEV_STATIC || !locs[i].bound || plan->group_of[i] != g) continue;
            const uint8_t *s = plan->dev->arenas[locs[i].arena].base + locs[i].offset;
            cut_items(s, arena_ptr(plan, p.dst_arena, p.data_offset), p.bytes, i, plan->opts.chunk_bytes,
                      plan->opts.small_bytes, gi, subs, pending);
        }
        flush_small(gi, subs, pending);
        xcd_order(gi);
        plan->groups[g].first_block = (uint32_t)items.size();
        plan->groups[g].n_blocks = (uint32_t)gi.size();
        items.insert(items.end(), gi.begin(), gi.end());
    }
    if (items.size() > 0xffffffffull) return fail(RDEV_E_INVAL, "too many work items; raise chunk_bytes");
    if (plan->dev->gpu()) {
        HIP_TRY(hipSetDevice(plan->dev->hip_device));
        HIP_TRY(hipDeviceSynchronize());          // nothing may still read the old tables
        HIP_TRY(plan->d_items.upload(items));
        HIP_TRY(plan->d_subs.upload(subs));
    }
    plan->n_blocks = (uint32_t)items.size();
    plan->src = std::move(locs);
    plan->bound_all = all;
    plan->copy_tables = false;
    return RDEV_OK;
}

namespace {

// Tables of the copying modes for a whole-plan batch: message layout (header ||
// payload || pad to 16, back to back), staging layout (align-spaced), and the
// per-arena layout of the fresh allocations an unpack makes.
rdev_status build_copy_tables(rdev_plan_t *plan) {
    rdev_device_t *dev = plan->dev;
    const uint32_t n = (uint32_t)plan->pl.size();
    const uint64_t chunk = plan->opts.chunk_bytes, A = plan->opts.align;
    const uint32_t small = plan->opts.small_bytes;
    if (!plan->have_send) return fail(RDEV_E_STATE, "copying modes need rdev_plan_bind_buffers");
    if (!plan->bound_all) return fail(RDEV_E_STATE, "not every static tensor has a bound source");
    if (plan->arenas.size() > rdev::kMaxHeapSlots) return fail(RDEV_E_INVAL, "copying modes support at most 16 destination arenas");
    std::map<uint32_t, uint32_t> slot_of;
    plan->heap_slot_arena.clear();
    for (auto &kv : plan->arenas) {
        slot_of[kv.first] = (uint32_t)plan->heap_slot_arena.size();
        plan->heap_slot_arena.push_back(kv.first);
    }
    plan->heap_need.assign(plan->heap_slot_arena.size(), 0);
    plan->rpc_rel.assign(n, 0);
    plan->rpc_slot.assign(n, 0);
    uint8_t *sb = dev->arenas[plan->send_buf.arena_id].base + plan->send_buf.offset;
    uint8_t *rb = plan->have_recv ? dev->arenas[plan->recv_buf.arena_id].base + plan->recv_buf.offset : nullptr;

    std::vector<Item> pack, pack_s, stage, stage_s, unstage, unstage_s, pend_a, pend_b, pend_c;
    std::vector<rdev::UItem> us, us_s, ur, ur_s, upend_s, upend_r;
    std::vector<rdev_meta> headers;
    std::vector<uint8_t *> msg_send, msg_recv, frag_send;
    std::vector<rdev_frag> frags;
    const uint64_t F = plan->opts.rpc_frag_bytes;
    uint64_t mptr = 0, sptr = 0;
    plan->stage_end = 0;
    auto push_unpack = [&](std::vector<rdev::UItem> &items, std::vector<rdev::UItem> &subs, std::vector<rdev::UItem> &pend,
                           const uint8_t *hdr, uint64_t rel, uint32_t slot, uint64_t bytes) {
        if (bytes <= small) {
            pend.push_back(rdev::UItem{hdr, rel, 0, slot, 0, 0});
            if (pend.size() == rdev::kWavesPerBlock) {
                items.push_back(rdev::UItem{nullptr, 0, 0, 0, (uint32_t)pend.size(), (uint32_t)subs.size()});
                subs.insert(subs.end(), pend.begin(), pend.end());
                pend.clear();
            }
            return;
        }
        for (uint64_t off = 0, c = 0; off < bytes; off += chunk, ++c)
            items.push_back(rdev::UItem{hdr, rel, (uint32_t)c, slot, 0, 0});
    };
    for (uint32_t i = 0; i < n; ++i) {
        const rdev_placement &p = plan->pl[i];
        if (p.kind != RDEV_STATIC) continue;
        const rdev_tensor_desc &d = plan->descs[i];
        const SrcLoc &loc = plan->src[i];
        const uint8_t *src = dev->arenas[loc.arena].base + loc.offset;
        // message
        rdev_meta h{};
        h.ndims = d.ndims;
        h.dtype = d.dtype;
        h.bytes = p.bytes;
        h.src_offset = loc.offset;
        for (uint32_t j = 0; j < d.ndims; ++j) h.dims[j] = d.dims[j];
        h.src_arena = loc.arena;
        h.tensor_id = p.tensor_id;
        headers.push_back(h);
        msg_send.push_back(sb + mptr);
        msg_recv.push_back(rb ? rb + mptr : nullptr);
        const uint32_t slot = slot_of[p.dst_arena];
        plan->rpc_slot[i] = slot;
        plan->rpc_rel[i] = plan->heap_need[slot];
        if (!F) {
            cut_items(src, sb + mptr + RDEV_META_BYTES, p.bytes, i, chunk, small, pack, pack_s, pend_a);
            push_unpack(us, us_s, upend_s, sb + mptr, plan->rpc_rel[i], slot, p.bytes);
            if (rb) push_unpack(ur, ur_s, upend_r, rb + mptr, plan->rpc_rel[i], slot, p.bytes);
            mptr += RDEV_META_BYTES + ((p.bytes + 15) & ~(uint64_t)15);
        } else {
            // header, then ceil(bytes / F) fragments, each: 32-byte fragment header || piece || pad to 16
            mptr += RDEV_META_BYTES;
            const uint64_t nfrag = (p.bytes + F - 1) / F;
            for (uint64_t k = 0; k < nfrag; ++k) {
                const uint64_t off = k * F, fb = std::min<uint64_t>(F, p.bytes - off);
                frags.push_back(rdev_frag{p.tensor_id, 0, (uint32_t)k, (uint32_t)nfrag, off, (uint32_t)fb, 0});
                frag_send.push_back(sb + mptr);
                cut_items(src + off, sb + mptr + sizeof(rdev_frag), fb, i, chunk, small, pack, pack_s, pend_a);
                push_unpack(us, us_s, upend_s, sb + mptr, plan->rpc_rel[i] + off, slot | rdev::kFragBit, fb);
                if (rb) push_unpack(ur, ur_s, upend_r, rb + mptr, plan->rpc_rel[i] + off, slot | rdev::kFragBit, fb);
                mptr += sizeof(rdev_frag) + ((fb + 15) & ~(uint64_t)15);
            }
        }
        plan->heap_need[slot] += (p.bytes + A - 1) & ~(A - 1);
        // staging
        plan->stage_end = std::max(plan->stage_end, sptr + p.bytes);
        cut_items(src, sb + sptr, p.bytes, i, chunk, small, stage, stage_s, pend_b);
        cut_items(sb + sptr, arena_ptr(plan, p.dst_arena, p.data_offset), p.bytes, i, chunk, small, unstage, unstage_s, pend_c);
        sptr += (p.bytes + A - 1) & ~(A - 1);
    }
    flush_small(pack, pack_s, pend_a);
    flush_small(stage, stage_s, pend_b);
    flush_small(unstage, unstage_s, pend_c);
    if (!upend_s.empty()) {
        us.push_back(rdev::UItem{nullptr, 0, 0, 0, (uint32_t)upend_s.size(), (uint32_t)us_s.size()});
        us_s.insert(us_s.end(), upend_s.begin(), upend_s.end());
    }
    if (!upend_r.empty()) {
        ur.push_back(rdev::UItem{nullptr, 0, 0, 0, (uint32_t)upend_r.size(), (uint32_t)ur_s.size()});
        ur_s.insert(ur_s.end(), upend_r.begin(), upend_r.end());
    }
    plan->msg_total = mptr;
    xcd_order(pack);
    xcd_order(stage);
    xcd_order(unstage);
    xcd_order(us);
    xcd_order(ur);
    HIP_TRY(hipSetDevice(dev->hip_device));
    HIP_TRY(hipDeviceSynchronize());
    HIP_TRY(plan->d_pack_items.upload(pack));
    HIP_TRY(plan->d_pack_subs.upload(pack_s));
    HIP_TRY(plan->d_stage_items.upload(stage));
    HIP_TRY(plan->d_stage_subs.upload(stage_s));
    HIP_TRY(plan->d_unstage_items.upload(unstage));
    HIP_TRY(plan->d_unstage_subs.upload(unstage_s));
    HIP_TRY(plan->d_unpack_send_items.upload(us));
    HIP_TRY(plan->d_unpack_send_subs.upload(us_s));
    HIP_TRY(plan->d_unpack_recv_items.upload(ur));
    HIP_TRY(plan->d_unpack_recv_subs.upload(ur_s));
    HIP_TRY(plan->d_headers.upload(headers));
    HIP_TRY(plan->d_msg_send.upload(msg_send));
    HIP_TRY(plan->d_msg_recv.upload(msg_recv));
    HIP_TRY(plan->d_frags.upload(frags));
    HIP_TRY(plan->d_frag_send.upload(frag_send));
    plan->n_frags = (uint32_t)frags.size();
    plan->n_pack_blocks = (uint32_t)pack.size();
    plan->n_stage_blocks = (uint32_t)stage.size();
    plan->n_unpack_blocks = (uint32_t)us.size();
    plan->copy_tables = true;
    return RDEV_OK;
}

rdev_status check_busy_all(rdev_plan_t *plan) {
    if (!(plan->opts.flags & RDEV_PLAN_CHECK_BUSY)) return RDEV_OK;
    for (uint32_t i = 0; i < plan->pl.size(); ++i)
        if (plan->pl[i].kind == RDEV_STATIC && static_ready(plan, i))
            return fail(RDEV_E_BUSY, "tensor " + std::to_string(plan->pl[i].tensor_id) + " has not been consumed");
    return RDEV_OK;
}

// whole-plan batch through one of the copying modes
rdev_status write_copy_mode(rdev_plan_t *plan, uint32_t mode, uint32_t seq, hipStream_t s) {
    if (!plan->copy_tables) RDEV_TRY(build_copy_tables(plan));
    RDEV_TRY(check_busy_all(plan));
    if (mode != RDEV_SENDERCOPY && plan->heap_on_device)
        return fail(RDEV_E_STATE, "this iteration's heap allocations were made on the device: call rdev_dyn_reset first");
    RDEV_TRY(before_delivery(plan, s));
    uint32_t token = 0;
    if (mode == RDEV_SENDERCOPY) {
        if (plan->stage_end > plan->send_buf.bytes) return fail(RDEV_E_NOMEM, "staging buffer too small");
        if (plan->n_static) token = next_token(plan, seq);
        std::fill(plan->rpc_valid.begin(), plan->rpc_valid.end(), 0);
        if (plan->n_stage_blocks) {
            RDEV_TRY(launch_copy_table(plan->d_stage_items.ptr, plan->d_stage_subs.ptr, plan->n_stage_blocks, s,
                                       "copy_table_kernel(stage)"));
            RDEV_TRY(launch_copy_table(plan->d_unstage_items.ptr, plan->d_unstage_subs.ptr, plan->n_stage_blocks, s,
                                       "copy_table_kernel(write)"));
        }
        if (plan->n_static) {
            for (uint32_t g = 0; g < plan->groups.size(); ++g) RDEV_TRY(launch_group_flags(plan, g, seq, token, s));
        }
        return RDEV_OK;
    }
    const bool wire = mode == RDEV_RPC3;
    if (plan->msg_total > plan->send_buf.bytes) return fail(RDEV_E_NOMEM, "message buffer too small");
    if (wire && (!plan->have_recv || plan->msg_total > plan->recv_buf.bytes)) return fail(RDEV_E_NOMEM, "receive buffer missing or too small");
    rdev::HeapBases hb{};
    for (size_t k = 0; k < plan->heap_slot_arena.size(); ++k) {
        const ArenaLayout &al = plan->arenas[plan->heap_slot_arena[k]];
        if (plan->heap_need[k] > al.heap_bytes - al.heap_ptr)
            return fail(RDEV_E_NOMEM, "dynamic heap of arena " + std::to_string(plan->heap_slot_arena[k]) + " exhausted");
    }
    for (size_t k = 0; k < plan->heap_slot_arena.size(); ++k) {
        ArenaLayout &al = plan->arenas[plan->heap_slot_arena[k]];
        hb.base[k] = arena_ptr(plan, plan->heap_slot_arena[k], al.heap_offset + al.heap_ptr);
    }
    if (plan->n_static) {
        token = next_token(plan, seq);
        // pack: headers, then payloads
        hipLaunchKernelGGL(rdev::rpc_header_kernel, dim3((plan->n_static * 32 + 255) / 256), dim3(256), 0, s,
                           plan->d_headers.ptr, plan->d_msg_send.ptr, plan->n_static, seq,
                           plan->opts.rpc_frag_bytes ? 0u : 1u);
        RDEV_TRY(launch_check("rpc_header_kernel"));
        if (plan->n_frags) {
            hipLaunchKernelGGL(rdev::rpc_frag_header_kernel, dim3((plan->n_frags * 8 + 255) / 256), dim3(256), 0, s,
                               plan->d_frags.ptr, plan->d_frag_send.ptr, plan->n_frags, seq);
            RDEV_TRY(launch_check("rpc_frag_header_kernel"));
        }
        if (plan->n_pack_blocks) {
            RDEV_TRY(launch_copy_table(plan->d_pack_items.ptr, plan->d_pack_subs.ptr, plan->n_pack_blocks, s,
                                       "copy_table_kernel(pack)"));
        }
        if (wire) {
            uint8_t *sb = plan->dev->arenas[plan->send_buf.arena_id].base + plan->send_buf.offset;
            uint8_t *rb = plan->dev->arenas[plan->recv_buf.arena_id].base + plan->recv_buf.offset;
            std::vector<ResolvedStatic> one{ResolvedStatic{0, sb, rb, plan->msg_total}};
            RDEV_TRY(launch_inline_copies(plan, one, s));
        }
        for (uint32_t first = 0; first < plan->n_unpack_blocks; first += kMaxBlocksPerLaunch) {
            const uint32_t nb = std::min(kMaxBlocksPerLaunch, plan->n_unpack_blocks - first);
            hipLaunchKernelGGL(rdev::unpack_table_kernel, dim3(nb), dim3(rdev::kBlockThreads), 0, s,
                               (wire ? plan->d_unpack_recv_items.ptr : plan->d_unpack_send_items.ptr) + first,
                               wire ? plan->d_unpack_recv_subs.ptr : plan->d_unpack_send_subs.ptr, hb,
                               (uint32_t)plan->opts.chunk_bytes);
            RDEV_TRY(launch_check("unpack_table_kernel"));
        }
        for (uint32_t g = 0; g < plan->groups.size(); ++g) {
            const rdev_plan_s::Group &gr = plan->groups[g];
            if (!gr.n_flags) continue;
            hipLaunchKernelGGL(rdev::rpc_flag_kernel, dim3(1), dim3(rdev::kFlagTableThreads), 0, s,
                               plan->d_flags.ptr + gr.first_flag,
                               (wire ? plan->d_msg_recv.ptr : plan->d_msg_send.ptr) + gr.first_flag, gr.n_flags,
                               plan->d_batch_view + g, token);
            RDEV_TRY(launch_check("rpc_flag_kernel"));
        }
    }
    // where each tensor went (for rdev_poll), and the heap pointers
    for (uint32_t i = 0; i < plan->pl.size(); ++i) {
        if (plan->pl[i].kind != RDEV_STATIC) continue;
        const ArenaLayout &al = plan->arenas[plan->pl[i].dst_arena];
        plan->rpc_offset[i] = al.heap_offset + al.heap_ptr + plan->rpc_rel[i];
        plan->rpc_valid[i] = 1;
    }
    for (size_t k = 0; k < plan->heap_slot_arena.size(); ++k)
        plan->arenas[plan->heap_slot_arena[k]].heap_ptr += plan->heap_need[k];
    return RDEV_OK;
}

}  // namespace

rdev_status rdev_plan_bind_buffers(rdev_plan_t *plan, const rdev_region *send_buf, const rdev_region *recv_buf) {
    if (!plan || !send_buf) return fail(RDEV_E_INVAL, "NULL argument");
    for (const rdev_region *r : {send_buf, recv_buf}) {
        if (!r) continue;
        Arena *a;
        RDEV_TRY(arena_of(plan->dev, r->arena_id, &a));
        if (r->offset % 256) return fail(RDEV_E_ALIGN, "buffer must be 256-byte aligned");
        if (r->offset > a->bytes || r->bytes > a->bytes - r->offset) return fail(RDEV_E_RANGE, "buffer outside its arena");
    }
    plan->send_buf = *send_buf;
    plan->copy_tables = false;
    plan->have_send = true;
    plan->have_recv = recv_buf != nullptr;
    if (recv_buf) plan->recv_buf = *recv_buf;
    return RDEV_OK;
}

rdev_status rdev_dyn_reset(rdev_plan_t *plan) {
    if (!plan) return fail(RDEV_E_INVAL, "NULL argument");
    for (auto &kv : plan->arenas) kv.second.heap_ptr = 0;
    plan->heap_epoch++;                 // the device-resident pointers of the last iteration no longer count
    plan->heap_on_device = false;
    return RDEV_OK;
}

rdev_status rdev_plan_free(rdev_plan_t *plan) {
    if (!plan) return fail(RDEV_E_INVAL, "NULL argument");
    if (plan->dev->gpu()) {
        HIP_TRY(hipSetDevice(plan->dev->hip_device));
        HIP_TRY(hipDeviceSynchronize());          // kernels may still read the tables
    }
    destroy_plan(plan);
    return RDEV_OK;
}

static rdev_status write_static_all(rdev_plan_t *plan, uint32_t seq, hipStream_t s) {
    if (!plan->bound_all) return fail(RDEV_E_STATE, "not every static tensor has a bound source");
    std::fill(plan->rpc_valid.begin(), plan->rpc_valid.end(), 0);
    RDEV_TRY(check_busy_all(plan));
    RDEV_TRY(before_delivery(plan, s));
    uint32_t token = 0;
    if (plan->n_static) token = next_token(plan, seq);
    for (uint32_t g = 0; g < plan->groups.size(); ++g) {
        const rdev_plan_s::Group &gr = plan->groups[g];
        if (gr.n_blocks) {
            // the timing bracket covers the launch of the first group (the only one unless flag_groups > 1)
            const bool timed = g == 0 && plan->ev_used < plan->ev_start.size() && (plan->ev_count++ % plan->ev_every) == 0;
            if (timed && gr.n_blocks <= kMaxBlocksPerLaunch) {
                // the launch carries its own start and stop events: they take the kernel's begin and end times,
                // with no marker packets of their own in the stream
                hipExtLaunchKernelGGL(rdev::copy_table_kernel, dim3(gr.n_blocks), dim3(rdev::kBlockThreads), 0, s,
                                      plan->ev_start[plan->ev_used], plan->ev_stop[plan->ev_used], 0,
                                      (const Item *)(plan->d_items.ptr + gr.first_block), (const Item *)plan->d_subs.ptr);
                RDEV_TRY(launch_check("copy_table_kernel"));
                plan->ev_used++;
            } else {
                if (timed) HIP_TRY(hipEventRecord(plan->ev_start[plan->ev_used], s));
                RDEV_TRY(launch_copy_table(plan->d_items.ptr + gr.first_block, plan->d_subs.ptr, gr.n_blocks, s,
                                           "copy_table_kernel"));
                if (timed) HIP_TRY(hipEventRecord(plan->ev_stop[plan->ev_used++], s));
            }
        }
        RDEV_TRY(launch_group_flags(plan, g, seq, token, s));
    }
    return RDEV_OK;
}

// comparison path: the runtime's own device-to-device copy, one call per tensor, then the flags
static rdev_status write_dma_mode(rdev_plan_t *plan, uint32_t seq, hipStream_t s) {
    if (!plan->bound_all) return fail(RDEV_E_STATE, "not every static tensor has a bound source");
    RDEV_TRY(check_busy_all(plan));
    RDEV_TRY(before_delivery(plan, s));
    std::fill(plan->rpc_valid.begin(), plan->rpc_valid.end(), 0);
    for (uint32_t i = 0; i < plan->pl.size(); ++i) {
        const rdev_placement &p = plan->pl[i];
        if (p.kind != RDEV_STATIC || !p.bytes) continue;
        const SrcLoc &loc = plan->src[i];
        HIP_TRY(hipMemcpyAsync(arena_ptr(plan, p.dst_arena, p.data_offset), plan->dev->arenas[loc.arena].base + loc.offset,
                               p.bytes, hipMemcpyDeviceToDevice, s));
    }
    if (plan->n_static) {
        const uint32_t token = next_token(plan, seq);
        for (uint32_t g = 0; g < plan->groups.size(); ++g) RDEV_TRY(launch_group_flags(plan, g, seq, token, s));
    }
    return RDEV_OK;
}

// static tensors listed explicitly (write or pull: on one GPU the same movement)
static rdev_status transfer_static_list(rdev_plan_t *plan, const std::vector<std::pair<uint32_t, const void *>> &list,
                                        uint32_t seq, hipStream_t s) {
    std::vector<ResolvedStatic> v(list.size());
    std::vector<std::pair<uint32_t *, uint32_t>> flags;
    for (size_t k = 0; k < list.size(); ++k) {
        RDEV_TRY(resolve_static(plan, list[k].first, list[k].second, &v[k]));
        const rdev_placement &p = plan->pl[list[k].first];
        if ((plan->opts.flags & RDEV_PLAN_CHECK_BUSY) && static_ready(plan, list[k].first))
            return fail(RDEV_E_BUSY, "tensor " + std::to_string(p.tensor_id) + " has not been consumed");
        flags.emplace_back((uint32_t *)arena_ptr(plan, p.dst_arena, p.flag_offset), 2 * list[k].first);
    }
    RDEV_TRY(before_delivery(plan, s));
    for (const auto &e : list) plan->rpc_valid[e.first] = 0;      // back in its static region
    RDEV_TRY(launch_inline_copies(plan, v, s));
    return launch_inline_flags(plan, flags, seq, true, s);
}

rdev_status rdev_write_batch(rdev_device_t *dev, rdev_plan_t *plan, const rdev_xfer *x, uint32_t n, uint32_t mode,
                             uint32_t seq, void *stream) {
    if (!dev || !plan || plan->dev != dev) return fail(RDEV_E_INVAL, "NULL argument or plan of another device");
    if ((x == nullptr) != (n == 0)) return fail(RDEV_E_INVAL, "x and n must both be empty or both be given");
    if (!seq) return fail(RDEV_E_INVAL, "seq must be >= 1");
    if (mode > RDEV_DMA) return fail(RDEV_E_INVAL, "unknown mode");
    RDEV_TRY(require_gpu(dev));
    hipStream_t s = (hipStream_t)stream;
    if (mode != RDEV_ZEROCOPY) {
        if (x) return fail(RDEV_E_INVAL, "modes other than RDEV_ZEROCOPY take the whole plan (x == NULL)");
        if (mode == RDEV_DMA) return write_dma_mode(plan, seq, s);
        return write_copy_mode(plan, mode, seq, s);
    }
    if (!x) return write_static_all(plan, seq, s);

    // validate the whole batch first
    std::vector<std::pair<uint32_t, const void *>> statics;
    struct Dyn { uint32_t idx; SrcLoc loc; uint64_t bytes; const rdev_xfer *x; };
    std::vector<Dyn> dyns;
    for (uint32_t k = 0; k < n; ++k) {
        uint32_t idx;
        RDEV_TRY(index_of(plan, x[k].tensor_id, &idx));
        const rdev_placement &p = plan->pl[idx];
        if (p.kind == RDEV_STATIC) {
            ResolvedStatic r;
            RDEV_TRY(resolve_static(plan, idx, x[k].src, &r));
            if ((plan->opts.flags & RDEV_PLAN_CHECK_BUSY) && static_ready(plan, idx))
                return fail(RDEV_E_BUSY, "tensor " + std::to_string(p.tensor_id) + " has not been consumed");
            statics.emplace_back(idx, x[k].src);
            continue;
        }
        const rdev_tensor_desc &d = plan->descs[idx];
        if (x[k].ndims != d.ndims) return fail(RDEV_E_INVAL, "run-time rank differs from the planned rank");
        if (x[k].dtype != d.dtype) return fail(RDEV_E_INVAL, "run-time element type differs from the planned one");
        for (uint32_t j = 0; j < d.ndims; ++j)
            if (d.dims[j] >= 0 && x[k].dims[j] != d.dims[j]) return fail(RDEV_E_INVAL, "a dim known at plan time changed");
        uint64_t nb;
        std::string err;
        rdev_status st = rdev::tensor_bytes(x[k].dtype, x[k].ndims, x[k].dims, &nb, err);
        if (st != RDEV_OK) return fail(st, err);
        if (!x[k].src) return fail(RDEV_E_INVAL, "a dynamic tensor needs a source address");
        if (x[k].dim0_dev && (!x[k].ndims || ((uintptr_t)x[k].dim0_dev & 3)))
            return fail(RDEV_E_INVAL, "dim0_dev needs a tensor of rank >= 1 and a 4-byte aligned device word");
        Dyn dy{idx, {}, nb, &x[k]};
        RDEV_TRY(locate(dev, x[k].src, nb, &dy.loc));
        if ((plan->opts.flags & RDEV_PLAN_CHECK_BUSY) && __atomic_load_n(&plan->h_flags[2 * idx + 1], __ATOMIC_ACQUIRE))
            return fail(RDEV_E_BUSY, "metadata of tensor " + std::to_string(p.tensor_id) + " has not been consumed");
        dyns.push_back(dy);
    }
    // enqueue in batch order: runs of static tensors, runs of dynamic ones
    // (order inside the stream equals batch order because each group is launched when met)
    size_t si = 0, di = 0;
    uint32_t k = 0;
    while (k < n) {
        uint32_t idx = plan->by_id[x[k].tensor_id];
        if (plan->pl[idx].kind == RDEV_STATIC) {
            std::vector<std::pair<uint32_t, const void *>> run;
            while (k < n && plan->pl[plan->by_id[x[k].tensor_id]].kind == RDEV_STATIC) { run.push_back(statics[si++]); ++k; }
            RDEV_TRY(transfer_static_list(plan, run, seq, s));
        } else {
            while (k < n && plan->pl[plan->by_id[x[k].tensor_id]].kind == RDEV_DYNAMIC) {
                rdev::MetaBatch mb{};
                mb.seq = seq;
                while (k < n && mb.n < rdev::kMetaInlineMax && plan->pl[plan->by_id[x[k].tensor_id]].kind == RDEV_DYNAMIC) {
                    const Dyn &dy = dyns[di++];
                    const rdev_placement &p = plan->pl[dy.idx];
                    rdev_meta rec{};
                    rec.ndims = dy.x->ndims;
                    rec.dtype = dy.x->dtype;
                    rec.bytes = dy.bytes;
                    rec.src_offset = dy.loc.offset;
                    for (uint32_t j = 0; j < dy.x->ndims; ++j) rec.dims[j] = dy.x->dims[j];
                    rec.src_arena = dy.loc.arena;
                    rec.tensor_id = p.tensor_id;
                    rec.seq = seq;
                    std::memcpy(mb.words[mb.n], &rec, 120);
                    mb.slot[mb.n] = arena_ptr(plan, p.dst_arena, p.meta_offset);
                    mb.meta_idx[mb.n] = (uint32_t)plan->dyn_index[dy.idx];
                    mb.flag_idx[mb.n] = 2 * dy.idx + 1;
                    if (dy.x->dim0_dev) {
                        mb.dim0_dev[mb.n] = dy.x->dim0_dev;
                        mb.dim0_max[mb.n] = (uint64_t)dy.x->dims[0];
                        mb.row_bytes[mb.n] = dy.x->dims[0] ? dy.bytes / (uint64_t)dy.x->dims[0] : 0;
                    }
                    mb.n++;
                    ++k;
                }
                RDEV_TRY(before_delivery(plan, s));
                hipLaunchKernelGGL(rdev::meta_write_kernel, dim3(mb.n), dim3(64), 0, s, mb, plan->d_flags_view,
                                   plan->d_meta_view);
                RDEV_TRY(launch_check("meta_write_kernel"));
            }
        }
    }
    return RDEV_OK;
}

rdev_status rdev_write_batch_fixed_staging(rdev_device_t *dev, rdev_plan_t *plan, const rdev_xfer *x, uint32_t n,
                                           uint32_t seq, void *stream) {
    if (!dev || !plan || plan->dev != dev) return fail(RDEV_E_INVAL, "NULL argument or plan of another device");
    if ((x == nullptr) != (n == 0)) return fail(RDEV_E_INVAL, "x and n must both be empty or both be given");
    if (!seq) return fail(RDEV_E_INVAL, "seq must be >= 1");
    RDEV_TRY(require_gpu(dev));
    hipStream_t s = (hipStream_t)stream;
    // the tensors, in order: the whole plan's static tensors, or the listed ones
    std::vector<std::pair<uint32_t, const void *>> list;
    if (!x) {
        for (uint32_t i = 0; i < plan->pl.size(); ++i)
            if (plan->pl[i].kind == RDEV_STATIC) list.emplace_back(i, nullptr);
    } else {
        for (uint32_t k = 0; k < n; ++k) {
            uint32_t idx;
            RDEV_TRY(index_of(plan, x[k].tensor_id, &idx));
            if (plan->pl[idx].kind != RDEV_STATIC) return fail(RDEV_E_INVAL, "the staged write takes static tensors");
            list.emplace_back(idx, x[k].src);
        }
    }
    // validate everything and lay the staging area out (align-spaced, in batch order) before anything is enqueued
    const uint64_t A = plan->opts.align;
    std::vector<ResolvedStatic> stage(list.size()), write(list.size());
    std::vector<std::pair<uint32_t *, uint32_t>> flags;
    uint64_t ptr = 0;
    for (size_t k = 0; k < list.size(); ++k) {
        ResolvedStatic r;
        RDEV_TRY(resolve_static(plan, list[k].first, list[k].second, &r));
        const rdev_placement &p = plan->pl[r.idx];
        if ((plan->opts.flags & RDEV_PLAN_CHECK_BUSY) && static_ready(plan, r.idx))
            return fail(RDEV_E_BUSY, "tensor " + std::to_string(p.tensor_id) + " has not been consumed");
        if (r.bytes > RDEV_FIXED_STAGING_BYTES || ptr > RDEV_FIXED_STAGING_BYTES - r.bytes)
            return fail(RDEV_E_NOMEM, "batch needs more than the " + std::to_string(RDEV_FIXED_STAGING_BYTES) +
                                          " bytes of fixed staging memory");
        stage[k] = ResolvedStatic{r.idx, r.src, dev->fixed_staging + ptr, r.bytes};
        write[k] = ResolvedStatic{r.idx, dev->fixed_staging + ptr, r.dst, r.bytes};
        flags.emplace_back((uint32_t *)arena_ptr(plan, p.dst_arena, p.flag_offset), 2 * r.idx);
        ptr += (r.bytes + A - 1) & ~(A - 1);
    }
    for (const auto &e : list) plan->rpc_valid[e.first] = 0;
    RDEV_TRY(before_delivery(plan, s));
    RDEV_TRY(launch_inline_copies(plan, stage, s));      // sender: tensor -> staging
    RDEV_TRY(launch_inline_copies(plan, write, s));      // staging -> receiver region (the kernel boundary orders the two)
    return launch_inline_flags(plan, flags, seq, true, s);
}

rdev_status rdev_read_batch(rdev_device_t *dev, rdev_plan_t *plan, const rdev_xfer *x, uint32_t n, uint32_t seq,
                            void *stream) {
    if (!dev || !plan || plan->dev != dev) return fail(RDEV_E_INVAL, "NULL argument or plan of another device");
    if ((x == nullptr) != (n == 0)) return fail(RDEV_E_INVAL, "x and n must both be empty or both be given");
    if (!seq) return fail(RDEV_E_INVAL, "seq must be >= 1");
    RDEV_TRY(require_gpu(dev));
    hipStream_t s = (hipStream_t)stream;
    if (!x) return write_static_all(plan, seq, s);

    // validate; heap space is claimed for the batch only if all of it fits
    std::map<uint32_t, uint64_t> heap_ptr;
    for (auto &kv : plan->arenas) heap_ptr[kv.first] = kv.second.heap_ptr;
    struct Pull { uint32_t idx; ResolvedStatic r; uint64_t dst_offset; };
    std::vector<Pull> pulls;
    std::vector<std::pair<uint32_t, const void *>> statics;
    for (uint32_t k = 0; k < n; ++k) {
        uint32_t idx;
        RDEV_TRY(index_of(plan, x[k].tensor_id, &idx));
        const rdev_placement &p = plan->pl[idx];
        if (p.kind == RDEV_STATIC) {
            ResolvedStatic r;
            RDEV_TRY(resolve_static(plan, idx, x[k].src, &r));
            if ((plan->opts.flags & RDEV_PLAN_CHECK_BUSY) && static_ready(plan, idx))
                return fail(RDEV_E_BUSY, "tensor " + std::to_string(p.tensor_id) + " has not been consumed");
            continue;
        }
        const int32_t di = plan->dyn_index[idx];
        if (plan->heap_on_device)
            return fail(RDEV_E_STATE, "this iteration's heap allocations were made on the device: call rdev_dyn_reset first");
        if (!plan->polled_valid[di]) return fail(RDEV_E_STATE, "metadata of tensor " + std::to_string(p.tensor_id) + " has not been polled");
        const rdev_meta &m = plan->polled[di];
        Arena *sa;
        RDEV_TRY(arena_of(dev, m.src_arena, &sa));
        if (m.src_offset > sa->bytes || m.bytes > sa->bytes - m.src_offset) return fail(RDEV_E_RANGE, "sender address outside its arena");
        const ArenaLayout &al = plan->arenas[p.dst_arena];
        uint64_t need;
        if (!rdev::round_up_checked(m.bytes, plan->opts.align, &need) || heap_ptr[p.dst_arena] + need < need ||
            heap_ptr[p.dst_arena] + need > al.heap_bytes)
            return fail(RDEV_E_NOMEM, "dynamic heap of arena " + std::to_string(p.dst_arena) + " exhausted");
        Pull pu;
        pu.idx = idx;
        pu.dst_offset = al.heap_offset + heap_ptr[p.dst_arena];
        heap_ptr[p.dst_arena] += need;
        if (ranges_overlap(m.src_arena, m.src_offset, p.dst_arena, pu.dst_offset, m.bytes))
            return fail(RDEV_E_OVERLAP, "sender tensor overlaps the receiver's fresh allocation");
        pu.r = ResolvedStatic{idx, sa->base + m.src_offset, arena_ptr(plan, p.dst_arena, pu.dst_offset), m.bytes};
        pulls.push_back(pu);
    }
    // commit
    for (auto &kv : plan->arenas) kv.second.heap_ptr = heap_ptr[kv.first];
    size_t pi = 0;
    uint32_t k = 0;
    while (k < n) {
        if (plan->pl[plan->by_id[x[k].tensor_id]].kind == RDEV_STATIC) {
            std::vector<std::pair<uint32_t, const void *>> run;
            while (k < n && plan->pl[plan->by_id[x[k].tensor_id]].kind == RDEV_STATIC) {
                run.emplace_back(plan->by_id[x[k].tensor_id], x[k].src);
                ++k;
            }
            RDEV_TRY(transfer_static_list(plan, run, seq, s));
            continue;
        }
        std::vector<ResolvedStatic> copies;
        rdev::PostBatch pb{};
        pb.seq = seq;
        while (k < n && pb.n < rdev::kInlineMax && plan->pl[plan->by_id[x[k].tensor_id]].kind == RDEV_DYNAMIC) {
            const Pull &pu = pulls[pi++];
            const rdev_placement &p = plan->pl[pu.idx];
            copies.push_back(pu.r);
            pb.slot[pb.n] = arena_ptr(plan, p.dst_arena, p.meta_offset);
            pb.dst_offset[pb.n] = pu.dst_offset;
            pb.meta_idx[pb.n] = (uint32_t)plan->dyn_index[pu.idx];
            pb.flag_idx[pb.n] = 2 * pu.idx;
            pb.n++;
            plan->polled_valid[plan->dyn_index[pu.idx]] = 0;
            ++k;
        }
        RDEV_TRY(launch_inline_copies(plan, copies, s));
        hipLaunchKernelGGL(rdev::post_pull_kernel, dim3(1), dim3(64), 0, s, pb, plan->d_flags_view, plan->d_meta_view);
        RDEV_TRY(launch_check("post_pull_kernel"));
    }
    return RDEV_OK;
}

rdev_status rdev_read_batch_device(rdev_device_t *dev, rdev_plan_t *plan, const rdev_xfer *x, uint32_t n, uint32_t seq,
                                   void *stream) {
    if (!dev || !plan || plan->dev != dev || !x || !n) return fail(RDEV_E_INVAL, "NULL argument, empty batch or plan of another device");
    if (!seq) return fail(RDEV_E_INVAL, "seq must be >= 1");
    RDEV_TRY(require_gpu(dev));
    hipStream_t s = (hipStream_t)stream;
    std::vector<uint32_t> idx(n);
    for (uint32_t k = 0; k < n; ++k) {
        RDEV_TRY(index_of(plan, x[k].tensor_id, &idx[k]));
        if (plan->pl[idx[k]].kind != RDEV_DYNAMIC) return fail(RDEV_E_INVAL, "the device-side receive takes dynamic tensors");
        for (uint32_t j = 0; j < k; ++j)
            if (idx[j] == idx[k]) return fail(RDEV_E_INVAL, "a tensor is listed twice");
    }
    if (n > rdev::kRecvMax) return fail(RDEV_E_INVAL, "the device-side receive takes at most 8 tensors per call");
    for (uint32_t first = 0; first < n; first += rdev::kRecvMax) {
        rdev::RecvBatch b{};
        b.n = std::min<uint32_t>(rdev::kRecvMax, n - first);
        b.seq = seq;
        b.epoch = plan->heap_epoch;
        b.chunk = (uint32_t)plan->opts.chunk_bytes;
        b.align = plan->opts.align;
        b.n_arenas = (uint32_t)dev->arenas.size();
        b.call_id = ++plan->recv_calls;
        for (uint32_t a = 0; a < rdev::kArenaArgs && a < dev->arenas.size(); ++a)
            b.arena[a] = rdev::ArenaEnt{dev->arenas[a].base, dev->arenas[a].bytes};
        uint64_t room = 0, hint = 0;
        bool hinted = true;
        for (uint32_t k = 0; k < b.n; ++k) {
            const uint32_t i = idx[first + k];
            const rdev_placement &p = plan->pl[i];
            const ArenaLayout &al = plan->arenas[p.dst_arena];
            rdev::RecvEnt &e = b.e[k];
            e.slot = arena_ptr(plan, p.dst_arena, p.meta_offset);
            e.arena_base = dev->arenas[p.dst_arena].base;
            e.heap_offset = al.heap_offset;
            e.heap_bytes = al.heap_bytes;
            e.heap_ptr_host = al.heap_ptr;
            e.heap_word = plan->heap_word_of[p.dst_arena];
            e.dst_arena = p.dst_arena;
            e.meta_idx = (uint32_t)plan->dyn_index[i];
            e.flag_idx = 2 * i;
            room += al.heap_bytes;
            plan->polled_valid[plan->dyn_index[i]] = 0;
            // optional size hint: dims given with the entry (an upper bound is fine) shape the launch, nothing else
            uint64_t hb = 0;
            std::string ignore;
            const rdev_xfer &xe = x[first + k];
            if (xe.ndims && rdev::tensor_bytes(xe.dtype, xe.ndims, xe.dims, &hb, ignore) == RDEV_OK) hint += hb;
            else hinted = false;
        }
        // The payload sizes are not known on the host.  The workgroups stride over the chunks the records call for, so
        // any grid is correct; a hinted batch gets one workgroup per chunk, an unhinted one a modest fixed number
        // (idle workgroups still cost a layout pass each and take wave slots from whatever else is running).
        const uint64_t want = (hinted ? hint : room) / plan->opts.chunk_bytes + b.n;
        const uint32_t grid = (uint32_t)std::min<uint64_t>(want, hinted ? rdev::kRecvMaxBlocks : rdev::kRecvBlocksNoHint);
        hipLaunchKernelGGL(rdev::recv_kernel, dim3(grid), dim3(rdev::kBlockThreads), 0, s, b, dev->d_arenas, plan->d_heap.ptr,
                           plan->d_recv_arrivals.ptr, plan->d_flags_view, plan->d_meta_view, plan->d_status_view);
        RDEV_TRY(launch_check("recv_kernel"));
        plan->heap_on_device = true;
    }
    return RDEV_OK;
}

rdev_status rdev_recv_status(rdev_plan_t *plan, int32_t *status_out, uint32_t *entry_out, uint32_t *calls_done_out,
                             uint32_t *calls_made_out) {
    if (!plan) return fail(RDEV_E_INVAL, "NULL argument");
    RDEV_TRY(require_gpu(plan->dev));
    const uint32_t done = __atomic_load_n(&plan->h_status[2], __ATOMIC_ACQUIRE);
    if (calls_done_out) *calls_done_out = done;
    if (status_out) *status_out = (int32_t)plan->h_status[0];
    if (entry_out) *entry_out = plan->h_status[1];
    if (calls_made_out) *calls_made_out = plan->recv_calls;
    return RDEV_OK;
}

rdev_status rdev_poll(rdev_device_t *dev, rdev_plan_t *plan, uint32_t tensor_id, uint32_t poll_flags, rdev_meta *meta_out,
                      void *stream) {
    if (!dev || !plan || plan->dev != dev) return fail(RDEV_E_INVAL, "NULL argument or plan of another device");
    if (poll_flags & ~(uint32_t)(RDEV_POLL_CONSUME | RDEV_POLL_META | RDEV_POLL_ARENA)) return fail(RDEV_E_INVAL, "unknown poll flags");
    RDEV_TRY(require_gpu(dev));
    hipStream_t s = (hipStream_t)stream;
    const bool consume = poll_flags & RDEV_POLL_CONSUME;

    if (tensor_id == RDEV_ALL_TENSORS) {
        if (poll_flags & (RDEV_POLL_META | RDEV_POLL_ARENA)) return fail(RDEV_E_INVAL, "RDEV_ALL_TENSORS polls host-visible static flags only");
        std::vector<uint32_t> &toks = plan->tok_scratch;
        toks.resize(plan->pl.size());
        bool stale = false;
        for (uint32_t i = 0; i < plan->pl.size(); ++i)
            if (plan->pl[i].kind == RDEV_STATIC && !static_ready(plan, i, &toks[i], &stale)) return RDEV_NOT_READY;
        if (stale) return stale_error();
        if (consume && plan->n_static) {
            for (uint32_t i = 0; i < plan->pl.size(); ++i)
                if (plan->pl[i].kind == RDEV_STATIC) static_consume(plan, i, toks[i]);
            if (plan->n_static <= rdev::kFlagInlineMax) {
                rdev::InlineFlags f{};
                f.n = plan->n_static;
                for (uint32_t k = 0; k < plan->n_static; ++k) f.arena_flag[k] = plan->h_flag_ptrs[k];
                hipLaunchKernelGGL(rdev::flag_inline_kernel, dim3(1), dim3(64), 0, s, f, (uint32_t *)nullptr,
                                   (uint32_t *)nullptr, 0u);
                RDEV_TRY(launch_check("flag_inline_kernel"));
            } else {
                hipLaunchKernelGGL(rdev::flag_table_kernel, dim3(1), dim3(rdev::kFlagTableThreads), 0, s,
                                   plan->d_flags.ptr, plan->n_static, 0u, (uint32_t *)nullptr, 0u);
                RDEV_TRY(launch_check("flag_table_kernel"));
            }
            RDEV_TRY(after_clear(plan, s));
        }
        return RDEV_OK;
    }

    uint32_t idx;
    RDEV_TRY(index_of(plan, tensor_id, &idx));
    const rdev_placement &p = plan->pl[idx];
    const bool dyn = p.kind == RDEV_DYNAMIC;
    if ((poll_flags & RDEV_POLL_META) && !dyn) return fail(RDEV_E_INVAL, "RDEV_POLL_META on a static tensor");
    const bool want_meta = dyn && (poll_flags & RDEV_POLL_META);
    const uint32_t widx = 2 * idx + (want_meta ? 1 : 0);
    uint32_t *arena_flag = (uint32_t *)arena_ptr(plan, p.dst_arena, dyn ? p.meta_offset + (want_meta ? 124 : 120) : p.flag_offset);

    uint32_t v, tok = 0;
    if (!dyn) tok = __atomic_load_n(plan->h_batch + plan->group_of[idx], __ATOMIC_ACQUIRE);
    if (poll_flags & RDEV_POLL_ARENA) {
        HIP_TRY(hipMemcpy(&v, arena_flag, sizeof(v), hipMemcpyDeviceToHost));
    } else {
        bool stale = false;
        v = dyn ? __atomic_load_n(&plan->h_flags[widx], __ATOMIC_ACQUIRE) : static_ready(plan, idx, &tok, &stale);
        if (stale) return stale_error();
    }
    if (!v) return RDEV_NOT_READY;

    if (dyn) {
        rdev_meta rec;
        if (poll_flags & RDEV_POLL_ARENA) {
            HIP_TRY(hipMemcpy(&rec, arena_ptr(plan, p.dst_arena, p.meta_offset), sizeof(rec), hipMemcpyDeviceToHost));
        } else {
            std::memcpy(&rec, &plan->h_meta[plan->dyn_index[idx]], sizeof(rec));
            rec.data_flag = __atomic_load_n(&plan->h_flags[2 * idx], __ATOMIC_ACQUIRE);
            rec.meta_flag = __atomic_load_n(&plan->h_flags[2 * idx + 1], __ATOMIC_ACQUIRE);
        }
        if (want_meta) {
            plan->polled[plan->dyn_index[idx]] = rec;
            plan->polled_valid[plan->dyn_index[idx]] = 1;
        }
        if (meta_out) *meta_out = rec;
    } else if (meta_out) {
        std::memset(meta_out, 0, sizeof(*meta_out));
        const rdev_tensor_desc &d = plan->descs[idx];
        meta_out->ndims = d.ndims;
        meta_out->dtype = d.dtype;
        meta_out->bytes = p.bytes;
        for (uint32_t j = 0; j < d.ndims; ++j) meta_out->dims[j] = d.dims[j];
        meta_out->tensor_id = p.tensor_id;
        meta_out->seq = v;
        meta_out->data_flag = v;
        meta_out->dst_offset = plan->rpc_valid[idx] ? plan->rpc_offset[idx] : p.data_offset;
    }
    if (consume) {
        if (dyn) __atomic_store_n(&plan->h_flags[widx], 0u, __ATOMIC_RELEASE);
        else static_consume(plan, idx, tok);
        std::vector<std::pair<uint32_t *, uint32_t>> f{{arena_flag, widx}};
        RDEV_TRY(launch_inline_flags(plan, f, 0u, false, s));
        RDEV_TRY(after_clear(plan, s));
    }
    return RDEV_OK;
}

rdev_status rdev_gather_unique_rows(rdev_device_t *dev, const int64_t *ids, uint32_t n_ids, uint32_t vocab,
                                    const void *table, uint32_t row_bytes, int64_t *out_ids, void *out_rows,
                                    uint32_t *count_out, void *stream) {
    if (!dev || (!ids && n_ids) || !table || !out_ids || !out_rows || !count_out) return fail(RDEV_E_INVAL, "NULL argument");
    RDEV_TRY(require_gpu(dev));
    if (!vocab || vocab > rdev::kUniqueMaxVocab) return fail(RDEV_E_INVAL, "vocab must be in 1 .. 262144");
    if (!row_bytes || row_bytes % 16) return fail(RDEV_E_INVAL, "row_bytes must be a positive multiple of 16");
    if (((uintptr_t)table | (uintptr_t)out_rows) & 15) return fail(RDEV_E_ALIGN, "table and out_rows must be 16-byte aligned");
    if (((uintptr_t)ids | (uintptr_t)out_ids) & 7 || ((uintptr_t)count_out & 3)) return fail(RDEV_E_ALIGN, "ids, out_ids, count_out must be naturally aligned");
    hipStream_t s = (hipStream_t)stream;
    hipLaunchKernelGGL(rdev::unique_ids_kernel, dim3(1), dim3(rdev::kUniqueThreads), 0, s, ids, n_ids, vocab, out_ids, count_out);
    RDEV_TRY(launch_check("unique_ids_kernel"));
    const uint32_t grid = std::min(n_ids, vocab);
    if (grid) {
        hipLaunchKernelGGL(rdev::gather_rows_kernel, dim3(grid), dim3(256), 0, s, out_ids, count_out, (const uint8_t *)table,
                           row_bytes, (uint8_t *)out_rows);
        RDEV_TRY(launch_check("gather_rows_kernel"));
    }
    return RDEV_OK;
}

// ---- receiver-side consumer (sections 4, 5.1) ----

static rdev_status consume_checked(rdev_plan_t *plan, uint32_t idx, uint32_t max_spins, rdev_consume_result *out,
                                   hipStream_t s) {
    const rdev_placement &p = plan->pl[idx];
    hipLaunchKernelGGL(rdev::consume_init_kernel, dim3(1), dim3(64), 0, s, out, 1u);
    RDEV_TRY(launch_check("consume_init_kernel"));
    const uint64_t per_block = rdev::kConsumeUnitBytes;                          // at least one full round of loads each
    const uint32_t cap = max_spins ? rdev::kConsumeMaxBlocks : rdev::kConsumeMaxBlocksNoWait;
    uint32_t grid = (uint32_t)std::min<uint64_t>(cap, (p.bytes + per_block - 1) / per_block);
    if (!grid) grid = 1;
    hipLaunchKernelGGL(rdev::consume_reduce_max_kernel, dim3(grid), dim3(rdev::kConsumeThreads), 0, s,
                       (const uint32_t *)arena_ptr(plan, p.dst_arena, p.flag_offset),
                       (const uint8_t *)arena_ptr(plan, p.dst_arena, p.data_offset), p.bytes, max_spins, out);
    return launch_check("consume_reduce_max_kernel");
}

static rdev_status consume_validate(rdev_plan_t *plan, uint32_t tensor_id, const rdev_consume_result *out, uint32_t *idx) {
    RDEV_TRY(index_of(plan, tensor_id, idx));
    const rdev_placement &p = plan->pl[*idx];
    if (p.kind != RDEV_STATIC) return fail(RDEV_E_INVAL, "the consumer takes static tensors");
    if (p.bytes % 4) return fail(RDEV_E_INVAL, "the consumer reduces 32-bit elements: bytes must be a multiple of 4");
    if (!out || ((uintptr_t)out & 7)) return fail(RDEV_E_ALIGN, "result pointer must be 8-byte aligned device memory");
    return RDEV_OK;
}

rdev_status rdev_consume_reduce_max(rdev_device_t *dev, rdev_plan_t *plan, uint32_t tensor_id, uint32_t max_spins,
                                    rdev_consume_result *out, void *stream) {
    if (!dev || !plan || plan->dev != dev) return fail(RDEV_E_INVAL, "NULL argument or plan of another device");
    RDEV_TRY(require_gpu(dev));
    uint32_t idx;
    RDEV_TRY(consume_validate(plan, tensor_id, out, &idx));
    return consume_checked(plan, idx, max_spins, out, (hipStream_t)stream);
}

// one launch (per 32 tensors) over a list of validated static tensors; out[k] belongs to idx[k]
static rdev_status consume_list(rdev_plan_t *plan, const uint32_t *idx, uint32_t n, uint32_t max_spins,
                                rdev_consume_result *out, hipStream_t s) {
    if (!n) return RDEV_OK;
    hipLaunchKernelGGL(rdev::consume_init_kernel, dim3((n + 255) / 256), dim3(256), 0, s, out, n);
    RDEV_TRY(launch_check("consume_init_kernel"));
    for (uint32_t first = 0; first < n; first += rdev::kConsumeBatchMax) {
        rdev::ConsumeBatch b{};
        b.n = std::min<uint32_t>(rdev::kConsumeBatchMax, n - first);
        b.max_spins = max_spins;
        uint64_t units = 0;
        for (uint32_t k = 0; k < b.n; ++k) {
            const rdev_placement &p = plan->pl[idx[first + k]];
            const uint64_t nvec = p.bytes >> 4, per = rdev::kConsumeUnitBytes / 16;
            const uint64_t nu = std::max<uint64_t>(1, (nvec + per - 1) / per);
            if (units + nu > 0xFFFFFFFFull) return fail(RDEV_E_INVAL, "tensor list too large for one consumer batch");
            b.e[k] = rdev::ConsumeEnt{(const uint32_t *)arena_ptr(plan, p.dst_arena, p.flag_offset),
                                      (const uint8_t *)arena_ptr(plan, p.dst_arena, p.data_offset), p.bytes, (uint32_t)units,
                                      (uint32_t)nu};
            units += nu;
        }
        b.n_units = (uint32_t)units;
        const uint32_t cap = max_spins ? rdev::kConsumeTableMaxBlocks : rdev::kConsumeMaxBlocksNoWait;
        hipLaunchKernelGGL(rdev::consume_table_kernel, dim3(std::min<uint32_t>(b.n_units, cap)), dim3(rdev::kConsumeThreads), 0, s,
                           b, out + first);
        RDEV_TRY(launch_check("consume_table_kernel"));
    }
    return RDEV_OK;
}

rdev_status rdev_consume_batch(rdev_device_t *dev, rdev_plan_t *plan, const uint32_t *tensor_ids, uint32_t n,
                               uint32_t max_spins, rdev_consume_result *out, void *stream) {
    if (!dev || !plan || plan->dev != dev || (!tensor_ids && n)) return fail(RDEV_E_INVAL, "NULL argument or plan of another device");
    RDEV_TRY(require_gpu(dev));
    std::vector<uint32_t> idx(n);
    for (uint32_t i = 0; i < n; ++i) RDEV_TRY(consume_validate(plan, tensor_ids[i], out + i, &idx[i]));
    return consume_list(plan, idx.data(), n, max_spins, out, (hipStream_t)stream);
}

rdev_status rdev_recv_polling_async(rdev_device_t *dev, rdev_plan_t *plan, const uint32_t *tensor_ids, uint32_t n,
                                    rdev_consume_result *out, void *flag_stream, void *consumer_stream,
                                    uint64_t max_polls, uint64_t *polls_out) {
    if (!dev || !plan || plan->dev != dev || (!tensor_ids && n)) return fail(RDEV_E_INVAL, "NULL argument or plan of another device");
    RDEV_TRY(require_gpu(dev));
    std::vector<uint32_t> idx(n);
    for (uint32_t i = 0; i < n; ++i) RDEV_TRY(consume_validate(plan, tensor_ids[i], out + i, &idx[i]));
    std::vector<uint32_t> queue(n);                 // positions 0..n-1 of the caller's list, in ready-queue order
    for (uint32_t i = 0; i < n; ++i) queue[i] = i;
    size_t head = 0;
    uint64_t polls = 0, failed = 0;
    rdev_status result = RDEV_OK;
    // Ops whose poll succeeded since the last failed poll turn asynchronous together: one clear launch and one
    // consumer launch for the run, instead of two launches per tensor.  Results must be contiguous per launch, so a
    // run is cut where the caller's positions stop being consecutive.
    std::vector<uint32_t> run;                      // positions, consecutive and ascending
    auto flush = [&]() -> rdev_status {
        if (run.empty()) return RDEV_OK;
        std::vector<std::pair<uint32_t *, uint32_t>> f;
        std::vector<uint32_t> ridx;
        for (uint32_t pos : run) {
            const rdev_placement &p = plan->pl[idx[pos]];
            f.emplace_back((uint32_t *)arena_ptr(plan, p.dst_arena, p.flag_offset), 2 * idx[pos]);
            ridx.push_back(idx[pos]);
        }
        RDEV_TRY(launch_inline_flags(plan, f, 0u, false, (hipStream_t)flag_stream));
        RDEV_TRY(after_clear(plan, (hipStream_t)flag_stream));
        RDEV_TRY(consume_list(plan, ridx.data(), (uint32_t)ridx.size(), 0, out + run.front(), (hipStream_t)consumer_stream));
        run.clear();
        return RDEV_OK;
    };
    while (head < queue.size()) {
        const uint32_t i = queue[head++];
        ++polls;
        uint32_t tok;
        bool stale = false;
        const uint32_t ready = static_ready(plan, idx[i], &tok, &stale);
        if (stale) return stale_error();
        if (!ready) {
            RDEV_TRY(flush());                      // what is ready starts before the host goes on waiting
            if (++failed >= max_polls) { result = RDEV_NOT_READY; break; }
            queue.push_back(i);                     // back to the tail of the ready queue
            if (head > 4096 && head * 2 > queue.size()) {   // keep the vector from growing without bound
                queue.erase(queue.begin(), queue.begin() + head);
                head = 0;
            }
            continue;
        }
        // success: consume the flag, the op turns asynchronous
        static_consume(plan, idx[i], tok);
        if (!run.empty() && (i != run.back() + 1 || run.size() == rdev::kConsumeBatchMax)) RDEV_TRY(flush());
        run.push_back(i);
    }
    RDEV_TRY(flush());
    if (polls_out) *polls_out = polls;
    return result;
}

// ---- allocation-site tracing (section 3.4) ----

static void tracer_release_all(rdev_tracer_t *tr) {
    std::string ignore;
    Arena &ar = tr->dev->arenas[tr->arena_id];
    for (auto &kv : tr->live) {
        if (kv.second.arena) ar.alloc.release(kv.second.offset, kv.second.bytes, ignore);
        else tr->pool.release(kv.second.offset, kv.second.bytes, ignore);
    }
    tr->live.clear();
    for (const rdev_region &r : tr->staging) ar.alloc.release(r.offset, r.bytes, ignore);
    tr->staging.clear();
}

rdev_status rdev_tracer_open(rdev_device_t *dev, void *pool_base, uint64_t pool_bytes, uint32_t arena_id,
                             rdev_tracer_t **out) {
    if (!dev || !out || !pool_base || !pool_bytes) return fail(RDEV_E_INVAL, "NULL argument");
    Arena *a;
    RDEV_TRY(arena_of(dev, arena_id, &a));
    if ((uintptr_t)pool_base & 255) return fail(RDEV_E_ALIGN, "pool base must be 256-byte aligned");
    SrcLoc loc;
    if (locate(dev, pool_base, pool_bytes, &loc) == RDEV_OK || locate(dev, pool_base, 1, &loc) == RDEV_OK)
        return fail(RDEV_E_OVERLAP, "the ordinary pool must not be registered memory");
    rdev_tracer_t *tr = new rdev_tracer_t();
    tr->dev = dev;
    tr->pool_base = (uint8_t *)pool_base;
    tr->pool_bytes = pool_bytes;
    tr->arena_id = arena_id;
    tr->pool = rdev::RegionAllocator(pool_bytes);
    *out = tr;
    return RDEV_OK;
}

rdev_status rdev_tracer_close(rdev_tracer_t *tr) {
    if (!tr) return fail(RDEV_E_INVAL, "NULL argument");
    tracer_release_all(tr);
    delete tr;
    return RDEV_OK;
}

rdev_status rdev_tracer_begin_iteration(rdev_tracer_t *tr) {
    if (!tr) return fail(RDEV_E_INVAL, "NULL argument");
    tracer_release_all(tr);
    tr->next_index.clear();
    tr->iteration++;
    return RDEV_OK;
}

rdev_status rdev_tracer_alloc(rdev_tracer_t *tr, uint32_t node_id, uint64_t bytes, void **ptr_out,
                              uint32_t *alloc_index_out, uint32_t *in_arena_out) {
    if (!tr || !ptr_out) return fail(RDEV_E_INVAL, "NULL argument");
    if (!tr->iteration) return fail(RDEV_E_STATE, "no iteration begun");
    if (!bytes) return fail(RDEV_E_INVAL, "bytes must be positive");
    const uint32_t idx = tr->next_index[node_id];
    const bool arena = tr->iteration > 1 && tr->in_S.count({node_id, idx});
    uint64_t off;
    std::string err;
    Arena &ar = tr->dev->arenas[tr->arena_id];
    rdev_status st = arena ? ar.alloc.alloc(bytes, 256, &off, err) : tr->pool.alloc(bytes, 256, &off, err);
    if (st != RDEV_OK) return fail(st, std::string(arena ? "registered arena: " : "ordinary pool: ") + err);
    tr->next_index[node_id] = idx + 1;
    uint8_t *p = (arena ? ar.base : tr->pool_base) + off;
    tr->live[(uintptr_t)p] = rdev_tracer_s::Buf{off, bytes, arena};
    if (tr->iteration == 1) tr->site_of[(uintptr_t)p] = {node_id, idx};      // last writer wins
    *ptr_out = p;
    if (alloc_index_out) *alloc_index_out = idx;
    if (in_arena_out) *in_arena_out = arena ? 1 : 0;
    return RDEV_OK;
}

rdev_status rdev_tracer_free(rdev_tracer_t *tr, void *ptr) {
    if (!tr) return fail(RDEV_E_INVAL, "NULL argument");
    auto it = tr->live.find((uintptr_t)ptr);
    if (it == tr->live.end()) return fail(RDEV_E_INVAL, "not a live buffer of this tracer");
    std::string err;
    if (it->second.arena) tr->dev->arenas[tr->arena_id].alloc.release(it->second.offset, it->second.bytes, err);
    else tr->pool.release(it->second.offset, it->second.bytes, err);
    tr->live.erase(it);
    return RDEV_OK;
}

rdev_status rdev_tracer_mark_sent(rdev_tracer_t *tr, const void *ptr, uint32_t *registered_out) {
    if (!tr || !ptr) return fail(RDEV_E_INVAL, "NULL argument");
    auto it = tr->live.find((uintptr_t)ptr);
    if (it == tr->live.end()) return fail(RDEV_E_INVAL, "not a live buffer of this tracer");
    if (tr->iteration == 1) {
        auto site = tr->site_of.find((uintptr_t)ptr);
        if (site != tr->site_of.end() && !tr->in_S.count(site->second)) {
            tr->in_S[site->second] = true;
            tr->S.push_back(site->second);
        }
    }
    if (registered_out) *registered_out = it->second.arena ? 1 : 0;
    return RDEV_OK;
}

rdev_status rdev_tracer_send(rdev_tracer_t *tr, rdev_plan_t *plan, uint32_t tensor_id, const void *ptr, uint32_t seq,
                             void *stream, uint32_t *copied_out) {
    if (!tr || !plan || plan->dev != tr->dev || !ptr) return fail(RDEV_E_INVAL, "NULL argument or plan of another device");
    if (!seq) return fail(RDEV_E_INVAL, "seq must be >= 1");
    RDEV_TRY(require_gpu(tr->dev));
    uint32_t idx;
    RDEV_TRY(index_of(plan, tensor_id, &idx));
    const rdev_placement &p = plan->pl[idx];
    if (p.kind != RDEV_STATIC) return fail(RDEV_E_INVAL, "not a static tensor");
    auto it = tr->live.find((uintptr_t)ptr);
    if (it == tr->live.end()) return fail(RDEV_E_INVAL, "not a live buffer of this tracer");
    if (it->second.bytes < p.bytes) return fail(RDEV_E_RANGE, "buffer is smaller than the tensor");
    hipStream_t s = (hipStream_t)stream;
    const void *src = ptr;
    uint32_t copied = 0;
    rdev_region stage{};
    if (!it->second.arena) {
        // not registered: stage through a fresh registered buffer
        if (p.bytes) {
            uint64_t off;
            std::string err;
            rdev_status st = tr->dev->arenas[tr->arena_id].alloc.alloc(p.bytes, 256, &off, err);
            if (st != RDEV_OK) return fail(st, "staging buffer: " + err);
            stage = rdev_region{tr->arena_id, 0, off, p.bytes};
            src = tr->dev->arenas[tr->arena_id].base + off;
        } else {
            src = tr->dev->arenas[tr->arena_id].base;
        }
        copied = 1;
    }
    // validate the write before anything is enqueued
    ResolvedStatic r;
    rdev_status st = resolve_static(plan, idx, src, &r);
    if (st == RDEV_OK && (plan->opts.flags & RDEV_PLAN_CHECK_BUSY) && static_ready(plan, idx))
        st = fail(RDEV_E_BUSY, "tensor " + std::to_string(tensor_id) + " has not been consumed");
    if (st != RDEV_OK) {
        std::string ignore;
        if (stage.bytes) tr->dev->arenas[tr->arena_id].alloc.release(stage.offset, stage.bytes, ignore);
        return st;
    }
    RDEV_TRY(rdev_tracer_mark_sent(tr, ptr, nullptr));
    if (copied && p.bytes) {
        tr->staging.push_back(stage);
        std::vector<ResolvedStatic> one{ResolvedStatic{idx, (const uint8_t *)ptr, (uint8_t *)const_cast<void *>(src), p.bytes}};
        RDEV_TRY(launch_inline_copies(plan, one, s));
    }
    std::vector<std::pair<uint32_t, const void *>> list{{idx, src}};
    RDEV_TRY(transfer_static_list(plan, list, seq, s));
    if (copied_out) *copied_out = copied;
    return RDEV_OK;
}

rdev_status rdev_tracer_set_size(const rdev_tracer_t *tr, uint32_t *n_out) {
    if (!tr || !n_out) return fail(RDEV_E_INVAL, "NULL argument");
    *n_out = (uint32_t)tr->S.size();
    return RDEV_OK;
}

rdev_status rdev_tracer_set_get(const rdev_tracer_t *tr, uint32_t i, uint32_t *node_id_out, uint32_t *alloc_index_out) {
    if (!tr || !node_id_out || !alloc_index_out) return fail(RDEV_E_INVAL, "NULL argument");
    if (i >= tr->S.size()) return fail(RDEV_E_INVAL, "index out of range");
    *node_id_out = tr->S[i].first;
    *alloc_index_out = tr->S[i].second;
    return RDEV_OK;
}

rdev_status rdev_device_info(rdev_device_t *dev, uint64_t out[4]) {
    if (!dev || !out) return fail(RDEV_E_INVAL, "NULL argument");
    RDEV_TRY(require_gpu(dev));
    hipDeviceProp_t p;
    HIP_TRY(hipGetDeviceProperties(&p, dev->hip_device));
    out[0] = (uint64_t)p.memoryClockRate;
    out[1] = (uint64_t)p.memoryBusWidth;
    out[2] = (uint64_t)p.multiProcessorCount;
    out[3] = (uint64_t)p.l2CacheSize;
    return RDEV_OK;
}

rdev_status rdev_plan_profile(rdev_plan_t *plan, uint32_t max_samples, uint32_t every) {
    if (!plan) return fail(RDEV_E_INVAL, "NULL argument");
    plan->ev_every = every ? every : 1;
    plan->ev_count = 0;
    RDEV_TRY(require_gpu(plan->dev));
    if (max_samples == plan->ev_start.size()) {      // same events again: re-arm only, no wait for the device
        plan->ev_used = 0;                           // (samples not read yet are dropped)
        return RDEV_OK;
    }
    HIP_TRY(hipSetDevice(plan->dev->hip_device));
    HIP_TRY(hipDeviceSynchronize());
    drop_events(plan);
    for (uint32_t i = 0; i < max_samples; ++i) {
        hipEvent_t a, b;
        HIP_TRY(hipEventCreate(&a));
        plan->ev_start.push_back(a);
        HIP_TRY(hipEventCreate(&b));
        plan->ev_stop.push_back(b);
    }
    return RDEV_OK;
}

rdev_status rdev_plan_profile_read(rdev_plan_t *plan, float *ms_out, uint32_t cap, uint32_t *n_out) {
    if (!plan || !n_out || (!ms_out && cap)) return fail(RDEV_E_INVAL, "NULL argument");
    RDEV_TRY(require_gpu(plan->dev));
    uint32_t n = std::min(cap, plan->ev_used);
    for (uint32_t i = 0; i < n; ++i) {
        HIP_TRY(hipEventSynchronize(plan->ev_stop[i]));
        HIP_TRY(hipEventElapsedTime(&ms_out[i], plan->ev_start[i], plan->ev_stop[i]));
    }
    *n_out = n;
    plan->ev_used = 0;
    return RDEV_OK;
}

}  // extern "C"
