/*
 * rdev.h - C ABI of the memory-region "device" for cross-partition tensor transfer.
 *
 * The paper (abstract, section 1, section 3.1) replaces RPC by a device-like
 * interface: a remote machine is a *device* on which memory regions can be
 * allocated, read and written, and a transfer is a memory copy between a local
 * and a remote region.  Here one GPU plays both ends: sender tensors and
 * receiver regions live in separate registered arenas of the same HBM, and the
 * copy engine is a HIP kernel instead of a NIC.
 *
 * Conventions
 *   - Every function returns rdev_status: RDEV_OK (0), RDEV_NOT_READY (1, only
 *     from rdev_poll, not an error) or a negative RDEV_E_* code.  Nothing is
 *     thrown across the boundary.  rdev_last_error() gives a human-readable
 *     string for the last failure on the calling thread.
 *   - "device pointer" = address in GPU memory; "host pointer" = ordinary
 *     process memory.  Each argument says which one it is.
 *   - Arenas and source tensors are owned by the caller and must outlive every
 *     plan that names them.  Plans, descriptor tables and the pinned host words
 *     that mirror flags are owned by the library.
 *   - All sizes and offsets are 64-bit.
 *   - Transfers are asynchronous: they are enqueued on the caller's HIP stream
 *     (a hipStream_t passed as void*, NULL = the null stream) and the call
 *     returns.  Completion is observed with rdev_poll (per-tensor flags) or by
 *     synchronising the stream.
 *   - No consumed-acknowledgement exists (section 4): the caller issues the
 *     next write of a tensor only after the receiver has consumed the previous
 *     one.  A plan created with RDEV_PLAN_CHECK_BUSY reports RDEV_E_BUSY instead
 *     of overwriting an unconsumed tensor.
 *   - Calls on one rdev_device / rdev_plan are not thread-safe against each
 *     other, except rdev_poll without RDEV_POLL_CONSUME, which only reads.
 */
#ifndef RDEV_H
#define RDEV_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define RDEV_MAX_DIMS       8
#define RDEV_META_BYTES     128
#define RDEV_DEFAULT_ALIGN  256
#define RDEV_ALL_TENSORS    0xFFFFFFFFu
#define RDEV_HOST_ONLY      (-1)

typedef int32_t rdev_status;
enum {
    RDEV_OK          = 0,
    RDEV_NOT_READY   = 1,
    RDEV_E_INVAL     = -1,  /* bad argument: null pointer, unknown id, rank > RDEV_MAX_DIMS, dim < -1, unknown dtype/mode */
    RDEV_E_NOMEM     = -2,  /* region, plan, heap or message buffer does not fit */
    RDEV_E_OVERLAP   = -3,  /* a source range overlaps its own destination range */
    RDEV_E_ALIGN     = -4,  /* alignment not a power of two (plans: also < 16) */
    RDEV_E_RANGE     = -5,  /* address not inside a registered arena */
    RDEV_E_OVERFLOW  = -6,  /* dims product or an offset does not fit 64 bits */
    RDEV_E_BUSY      = -7,  /* unconsumed flag (RDEV_PLAN_CHECK_BUSY), or arena still referenced */
    RDEV_E_HIP       = -8,  /* a HIP call failed, or a transfer was requested on a host-only device */
    RDEV_E_STATE     = -9   /* call out of protocol order (sources not bound, metadata not polled, ...) */
};

/* element type codes carried in the metadata record (section 3.3 lists the element type as one of its fields) */
enum {
    RDEV_U8 = 0, RDEV_I8 = 1, RDEV_I16 = 2, RDEV_I32 = 3, RDEV_I64 = 4,
    RDEV_F16 = 5, RDEV_BF16 = 6, RDEV_F32 = 7, RDEV_F64 = 8
};

enum { RDEV_STATIC = 0, RDEV_DYNAMIC = 1 };

/* transfer modes of rdev_write_batch */
enum {
    RDEV_ZEROCOPY   = 0,  /* section 3.2: one-sided write into the pre-allocated region */
    RDEV_RPC2       = 1,  /* section 2.2: pack header+payload into a message buffer, unpack into a fresh allocation */
    RDEV_RPC3       = 2,  /* section 5.1 (RPC over RDMA): as RPC2 plus a buffer-to-buffer copy in between */
    RDEV_SENDERCOPY = 3,  /* section 5.1 (analysis off): stage into a registered buffer, then zero-copy write */
    RDEV_DMA        = 4   /* comparison only: one hipMemcpyAsync (device to device) per tensor instead of the batched
                             kernel.  Despite the name no DMA engine is involved: inside one GPU the runtime serves
                             such a copy with a copy kernel of its own, so this measures per-tensor runtime calls */
};

enum { RDEV_POLL_CONSUME = 1, RDEV_POLL_META = 2, RDEV_POLL_ARENA = 4 };
enum { RDEV_PLAN_CHECK_BUSY = 1 };

typedef struct rdev_device_s rdev_device_t;
typedef struct rdev_plan_s   rdev_plan_t;

typedef struct {
    uint32_t arena_id;
    uint32_t _pad;
    uint64_t offset;    /* bytes from the arena base */
    uint64_t bytes;
} rdev_region;

/* A tensor that crosses the partition, as known before the computation starts.
 * dims[i] == -1: unknown until run time (the rank is always known, section 3.3). */
typedef struct {
    uint32_t tensor_id;             /* caller's id, unique within a plan */
    uint32_t dtype;                 /* RDEV_U8 ... RDEV_F64 */
    uint32_t ndims;                 /* 0 .. RDEV_MAX_DIMS; 0 = scalar */
    uint32_t dst_arena;             /* receiver arena id from rdev_register_arena */
    int64_t  dims[RDEV_MAX_DIMS];
} rdev_tensor_desc;

/* Where the planner put a tensor.  Offsets are bytes from the arena base.
 * static : payload at data_offset (bytes long), completion flag (uint32) at flag_offset.
 * dynamic: 128-byte metadata slot at meta_offset; flag_offset is its last word
 *          (the metadata flag); the word before it is the payload-complete flag. */
typedef struct {
    uint32_t tensor_id, kind, dst_arena, _pad;
    uint64_t data_offset, bytes, flag_offset, meta_offset, region_bytes;
} rdev_placement;

typedef struct {
    uint64_t align;             /* region alignment, power of two >= 16; 0 = RDEV_DEFAULT_ALIGN */
    uint64_t max_static_bytes;  /* known-size tensors larger than this are sent dynamically; 0 = no limit */
    uint64_t dyn_heap_bytes;    /* dynamic heap reserved after the regions of every destination arena */
    uint64_t chunk_bytes;       /* large tensors are cut into work items of this size; multiple of 256; 0 = default */
    uint32_t small_bytes;       /* tensors up to this size are copied by one wavefront; 0 = default */
    uint32_t flags;             /* RDEV_PLAN_* */
    uint64_t rpc_frag_bytes;    /* RPC modes only (section 2.2: a message larger than the receiver's buffer is split
                                   into fragments, each with header information for re-assembly): 0 = every payload
                                   in one piece; otherwise a multiple of 16, and every payload travels as
                                   ceil(bytes / rpc_frag_bytes) fragments, each behind a 32-byte rdev_frag header */
    uint32_t flag_groups;       /* whole-plan transfers run as this many launches over consecutive tensors of about
                                   equal bytes, each followed by the flags of its tensors, so that early tensors
                                   can be consumed while later ones are still moving (section 3.2: one flag per
                                   tensor); 0 or 1 = one launch, all flags at its end.  Each extra group costs one
                                   launch gap. */
    uint32_t _reserved;
} rdev_plan_opts;

/* Fragment header of the RPC modes (little endian, 32 bytes), followed by the
 * fragment's payload bytes and zero padding to a multiple of 16. */
typedef struct {
    uint32_t tensor_id;
    uint32_t seq;
    uint32_t frag_index;
    uint32_t frag_count;
    uint64_t offset;        /* of this fragment inside the tensor */
    uint32_t bytes;
    uint32_t reserved;
} rdev_frag;

/* The metadata record of the dynamic path, exactly as it lies in the
 * receiver's slot (section 3.3: number of dims, size of each dim, element
 * type, address of the sender-side tensor).  Little endian, 128 bytes.  The
 * sender address is (src_arena, src_offset): a one-sided read can only target
 * registered memory (section 3.4).  Also used as the message header of the RPC
 * modes. */
typedef struct {
    uint32_t ndims;                 /*   0 */
    uint32_t dtype;                 /*   4 */
    uint64_t bytes;                 /*   8 */
    uint64_t src_offset;            /*  16 */
    int64_t  dims[RDEV_MAX_DIMS];   /*  24, unused = 0 */
    uint64_t dst_offset;            /*  88, filled by the receiver when it allocates */
    uint32_t src_arena;             /*  96 */
    uint32_t tensor_id;             /* 100 */
    uint32_t seq;                   /* 104 */
    uint32_t reserved[3];           /* 108 */
    uint32_t data_flag;             /* 120, payload complete */
    uint32_t meta_flag;             /* 124, metadata complete: the flag at the tail of the record */
} rdev_meta;

/* One entry of an explicit batch. */
typedef struct {
    uint32_t    tensor_id;
    uint32_t    ndims;              /* dynamic tensors: run-time rank (must equal the planned rank) */
    const void *src;                /* device pointer inside a registered arena; NULL = the bound source (static only) */
    uint32_t    dtype;              /* dynamic tensors: run-time element type (must equal the planned one) */
    uint32_t    _pad;
    int64_t     dims[RDEV_MAX_DIMS];/* dynamic tensors: run-time dims, all >= 0 */
    const uint32_t *dim0_dev;       /* dynamic tensors, optional: device pointer to the leading dim, read by the
                                       metadata kernel when it runs (a size that only the GPU knows, e.g. the count
                                       rdev_gather_unique_rows produced on the same stream - no host round trip).
                                       dims[0] is then the caller's upper bound: the source range is validated with
                                       it and a larger count is cut to it.  NULL = dims[0] is the size. */
} rdev_xfer;

/* ---- device (section 3.1) ------------------------------------------------ */

/* Open the device on HIP device `hip_device`.  RDEV_HOST_ONLY gives a device
 * without a GPU on which arenas, regions and plans (layout only) work and every
 * transfer returns RDEV_E_HIP.  *out is owned by the library until rdev_close. */
rdev_status rdev_open(rdev_device_t **out, int hip_device);
/* Frees the device.  Plans must have been freed before (else RDEV_E_BUSY). */
rdev_status rdev_close(rdev_device_t *dev);
/* Last error text of the calling thread (never NULL; host pointer, valid until the next call). */
const char *rdev_last_error(void);
/* sizeof the ABI structs, for bindings to check: desc, placement, opts, meta, xfer, region. */
void rdev_abi_sizes(uint32_t out[6]);

/* Register caller-owned memory as an arena (section 3.4: one large buffer
 * registered once, sub-allocated afterwards).  base: device pointer, 256-byte
 * aligned (NULL is allowed on a host-only device).  arena_flags: 0.
 * Arena ids count up from 0 in registration order. */
rdev_status rdev_register_arena(rdev_device_t *dev, void *base, uint64_t bytes,
                                uint32_t arena_flags, uint32_t *arena_id_out);

/* Forget an arena.  RDEV_E_BUSY while regions or plan blocks are still allocated
 * in it; plans whose sources point into it must have been freed by the caller.
 * Its id is not reused. */
rdev_status rdev_unregister_arena(rdev_device_t *dev, uint32_t arena_id);

/* Allocate / free a region inside an arena (section 3.1).  First fit from the
 * lowest address; align must be a power of two; bytes > 0.  rdev_free_region
 * takes exactly a region returned by rdev_alloc_region. */
rdev_status rdev_alloc_region(rdev_device_t *dev, uint32_t arena_id, uint64_t bytes,
                              uint64_t align, rdev_region *out);
rdev_status rdev_free_region(rdev_device_t *dev, const rdev_region *region);

/* ---- static planner (sections 3.2 - 3.4) --------------------------------- */

/* Classify each tensor (static iff every dim is known and bytes <=
 * max_static_bytes), reserve one block per destination arena from that arena's
 * sub-allocator and place, in input order: for a static tensor a region
 * [payload | pad to 16 | flag word | pad to align]; for a dynamic tensor a
 * 128-byte metadata slot padded to align; then the arena's dynamic heap.
 * On a GPU device the flag words and metadata slots are cleared (synchronously).
 * t: host pointer to n descriptors.  opts: host pointer or NULL for defaults.
 * On failure nothing stays allocated. */
rdev_status rdev_plan(rdev_device_t *dev, const rdev_tensor_desc *t, uint32_t n,
                      const rdev_plan_opts *opts, rdev_plan_t **plan_out);
rdev_status rdev_plan_count(const rdev_plan_t *plan, uint32_t *n_out);
/* i-th placement in input order. */
rdev_status rdev_plan_get(const rdev_plan_t *plan, uint32_t i, rdev_placement *out);
/* Per destination arena: offset of the plan's block, bytes of regions+slots,
 * offset and size of the dynamic heap.  Any out pointer may be NULL. */
rdev_status rdev_plan_arena_info(const rdev_plan_t *plan, uint32_t arena_id, uint64_t *base,
                                 uint64_t *static_bytes, uint64_t *heap_offset, uint64_t *heap_bytes);
/* Hand-off (section 3.4: destination addresses become properties of the sender
 * nodes): bind the source of the i-th tensor to src_ptrs[i] (device pointers
 * inside registered arenas; NULL entries = not bound; entries of dynamic tensors
 * are ignored) and build + upload the descriptor table that rdev_write_batch
 * walks.  Source ranges must not overlap their destination. */
rdev_status rdev_plan_bind_sources(rdev_plan_t *plan, const void *const *src_ptrs, uint32_t n);
/* Buffers for the copying modes: send_buf is the message / staging buffer,
 * recv_buf the second buffer of RDEV_RPC3 (may be NULL otherwise).  Regions
 * from rdev_alloc_region, 256-byte aligned. */
rdev_status rdev_plan_bind_buffers(rdev_plan_t *plan, const rdev_region *send_buf, const rdev_region *recv_buf);
/* Start of an iteration on the receiver: every dynamic heap of the plan is empty again. */
rdev_status rdev_dyn_reset(rdev_plan_t *plan);
/* Frees the plan, its tables and its blocks in the arenas. */
rdev_status rdev_plan_free(rdev_plan_t *plan);

/* ---- transfer (sections 3.2, 3.3) ---------------------------------------- */

/* One-sided batched write, sender side.
 *   x == NULL, n == 0 : every static tensor of the plan from its bound source
 *                       (one kernel over the resident descriptor table).
 *   otherwise         : the n listed tensors, in order.  A static tensor's
 *                       payload is written to its region, then its flag = seq.
 *                       For a dynamic tensor the metadata record is written
 *                       into the receiver's slot, then the metadata flag = seq;
 *                       the payload stays where it is until the receiver pulls.
 * mode != RDEV_ZEROCOPY takes the whole plan (x == NULL); the copying modes
 * RDEV_RPC2 / RDEV_RPC3 / RDEV_SENDERCOPY need rdev_plan_bind_buffers.
 * seq >= 1 is the value stored into the flags.
 * The whole batch is validated before anything is enqueued.  Errors: RDEV_E_STATE
 * (source not bound, buffers not bound), RDEV_E_RANGE (source outside registered
 * memory), RDEV_E_OVERLAP, RDEV_E_BUSY (RDEV_PLAN_CHECK_BUSY), RDEV_E_NOMEM
 * (message buffer or heap of a copying mode), RDEV_E_INVAL, RDEV_E_HIP.
 * A whole-plan call (x == NULL) must not be recorded into a HIP graph: it hands
 * the flag kernel a fresh delivery token, which a replay would repeat.  Explicit
 * batches of static tensors launch kernels only and may be recorded and replayed
 * (consume the flags between replays, as between eager calls). */
rdev_status rdev_write_batch(rdev_device_t *dev, rdev_plan_t *plan, const rdev_xfer *x, uint32_t n,
                             uint32_t mode, uint32_t seq, void *stream);

/* For callers that cannot allocate device memory - code recorded under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc: the
 * RDEV_SENDERCOPY delivery (every tensor copied into a staging buffer, then
 * written from there into its region, then its flag = seq) with the staging
 * buffer in a fixed array of RDEV_FIXED_STAGING_BYTES inside the library's
 * device image, instead of the bound send buffer and the device tables that
 * rdev_write_batch(RDEV_SENDERCOPY) builds on first use.  Calls no hipMalloc /
 * hipFree; launches kernels only (descriptors travel in kernel arguments).
 *   x == NULL, n == 0 : every static tensor of the plan, in plan order, from its bound source.
 *   otherwise         : the n listed static tensors (x[i].src as in rdev_write_batch).
 * Tensor k is staged at the sum of round_up(bytes, align) of the tensors before
 * it; a batch whose staging layout exceeds RDEV_FIXED_STAGING_BYTES is rejected
 * with RDEV_E_NOMEM and nothing moves.  Completion is announced per tensor (host
 * word + in-arena flag), as for an explicit rdev_write_batch.
 * Every call on one GPU uses that GPU's one staging array, whatever device
 * handle or plan it is made with: calls on the same stream follow each other,
 * calls that overlap on different streams race on the staging bytes.  The array
 * keeps the last call's contents; nothing in it needs clearing.
 * Other errors as rdev_write_batch: RDEV_E_STATE, RDEV_E_RANGE, RDEV_E_OVERLAP, RDEV_E_BUSY, RDEV_E_INVAL, RDEV_E_HIP. */
#define RDEV_FIXED_STAGING_BYTES (16u << 20)
rdev_status rdev_write_batch_fixed_staging(rdev_device_t *dev, rdev_plan_t *plan, const rdev_xfer *x, uint32_t n,
                                           uint32_t seq, void *stream);

/* One-sided batched read, receiver side: local region <- remote tensor.
 * Dynamic tensor (section 3.3): its metadata must have been seen by
 * rdev_poll(..., RDEV_POLL_META); storage of round_up(bytes, align) is taken
 * from the arena's dynamic heap in batch order, the chosen offset is recorded
 * in the slot, the payload is copied from the sender's address, then the
 * payload-complete flag = seq.  x[i].src/dims are ignored for dynamic tensors.
 * Static tensor: pulled into its region exactly as rdev_write_batch would push it. */
rdev_status rdev_read_batch(rdev_device_t *dev, rdev_plan_t *plan, const rdev_xfer *x, uint32_t n,
                            uint32_t seq, void *stream);

/* The receiver's half of the dynamic protocol (section 3.3) without the host in
 * the loop: enqueued on `stream` behind the sender's metadata write (the same
 * stream, or one ordered after it), one kernel reads each listed tensor's record
 * from its slot, clears the metadata flag, takes round_up(bytes, align) from the
 * arena's dynamic heap in batch order, pulls the payload from the sender's
 * address, records the offset in the slot and raises the payload-complete flag =
 * seq.  The arena ends up byte for byte as after rdev_poll(RDEV_POLL_META |
 * RDEV_POLL_CONSUME) + rdev_read_batch; no host poll of the metadata is needed,
 * and rdev_poll(tensor) later reports the payload as usual.
 *   x, n : 1..8 dynamic tensors.  Only tensor_id matters; ndims/dtype/dims, when given, are a size hint (an
 *          upper bound is fine) that shapes the launch and nothing else.
 * The checks the host path makes are made on the device: metadata flag set,
 * sender range inside a registered arena, heap space, no overlap.  If any entry
 * fails, nothing of the batch moves and no flag changes; rdev_recv_status tells.
 * The heap pointers then live on the device until the next rdev_dyn_reset:
 * rdev_read_batch of dynamic tensors and the RPC modes return RDEV_E_STATE in
 * between (allocations made through them earlier in the iteration are honoured).
 * Calls on one plan must follow each other (one stream, or streams ordered by
 * events): they share the plan's heap words and its count of finished workgroups. */
rdev_status rdev_read_batch_device(rdev_device_t *dev, rdev_plan_t *plan, const rdev_xfer *x, uint32_t n,
                                   uint32_t seq, void *stream);
/* How the device-side receives of this plan went.  *calls_made_out = calls of
 * rdev_read_batch_device so far, *calls_done_out = how many of them the GPU has
 * finished; *status_out / *entry_out = outcome of the last finished one: RDEV_OK,
 * RDEV_NOT_READY (entry's metadata flag was not set), RDEV_E_RANGE,
 * RDEV_E_NOMEM (heap exhausted) or RDEV_E_OVERLAP, and the batch entry it
 * refers to.  Reads pinned host words; any out pointer may be NULL. */
rdev_status rdev_recv_status(rdev_plan_t *plan, int32_t *status_out, uint32_t *entry_out, uint32_t *calls_done_out,
                             uint32_t *calls_made_out);

/* Non-blocking completion test (section 3.2: the receiver polls the flag,
 * clears it, then lets dependants run).  Reads pinned host words that the flag
 * kernel stores with system scope - one word per listed tensor for explicit
 * batches, one delivery token for a whole-plan batch - so no GPU work is issued
 * for a test (section 3.5: poll on the CPU side).
 *   static tensor : ready when its flag != 0.
 *   dynamic tensor: RDEV_POLL_META tests the metadata flag (and remembers the
 *                   record for rdev_read_batch); otherwise the payload-complete flag.
 *   RDEV_ALL_TENSORS: ready when every static tensor of the plan is.
 * RDEV_POLL_CONSUME clears the flag on success: the host side at once, the
 * in-arena word by a small kernel enqueued on `stream`.  That may be the
 * delivery's stream or a stream of the receiver's own: the host-visible word is
 * stored after the in-arena words it announces, so the clear cannot overtake
 * them, and the next delivery of this plan waits for a clear that is still
 * pending on another stream (an event, checked on the host first).
 * RDEV_POLL_ARENA reads the in-arena word with a synchronous copy instead (slow; for checks).
 * meta_out (host pointer, may be NULL): dynamic tensors - the record as last
 * delivered; static tensors after an RPC-mode delivery - dst_offset of the fresh allocation. */
rdev_status rdev_poll(rdev_device_t *dev, rdev_plan_t *plan, uint32_t tensor_id,
                      uint32_t poll_flags, rdev_meta *meta_out, void *stream);

/* ---- sender-side producer of a run-time-sized tensor ----------------------- */

/* The sparse case that motivates the dynamic path (section 3.3: shapes that
 * depend on the mini-batch): from the token ids of a mini-batch, the ascending
 * list of distinct ids and the rows of `table` they select.  Both outputs have a
 * leading dim known only after the kernel ran; they are then sent with
 * rdev_write_batch as dynamic tensors.
 *   ids      device pointer, n_ids int64 values in [0, vocab)
 *   table    device pointer, vocab rows of row_bytes each; 16-byte aligned, row_bytes % 16 == 0
 *   out_ids  device pointer, room for min(n_ids, vocab) int64
 *   out_rows device pointer, room for min(n_ids, vocab) * row_bytes, 16-byte aligned
 *   count_out device pointer to two uint32: [0] = number of distinct ids, [1] = ids outside [0, vocab) (ignored)
 * vocab <= 262144 (the id set is a bitmap in LDS).  Enqueued on `stream`. */
rdev_status rdev_gather_unique_rows(rdev_device_t *dev, const int64_t *ids, uint32_t n_ids, uint32_t vocab,
                                    const void *table, uint32_t row_bytes, int64_t *out_ids, void *out_rows,
                                    uint32_t *count_out, void *stream);

/* ---- receiver-side consumer (sections 4 and 5.1) -------------------------- */

/* Result of the device-side consumer; lives in device memory. */
typedef struct {
    uint32_t status;        /* 0 = reduced; 1 = the flag was not seen within max_spins polls */
    uint32_t seen_flag;     /* flag value the kernel saw (0 when it did not wait) */
    float    max;           /* maximum of the fp32 elements; NaNs are skipped, -0 < +0, empty or all-NaN = -inf */
    uint32_t _arrivals;     /* internal */
    uint64_t word_sum;      /* sum of the payload's 32-bit words modulo 2^64 */
} rdev_consume_result;

/* The light consumer of the paper's send/receive micro-benchmark (reduce_max,
 * section 5.1) for one static tensor whose size is a multiple of 4 bytes.
 * With max_spins > 0 a small grid (64 workgroups of 1024 lanes at most: waiting workgroups
 * occupy compute units, the cost section 3.5 warns of) first waits until the tensor's
 * in-arena flag is non-zero - at most max_spins polls per workgroup, a few
 * microseconds apart (about 14 us once it has been waiting for a while) - and
 * then reduces the payload.  max_spins == 0: do not look at the
 * flag at all (the caller has polled it on the host).  out: device pointer, 8-byte
 * aligned; written by kernels on `stream`.  Never waits forever.  A waiting
 * consumer that is enqueued BEFORE the delivery only sees it arrive if the two
 * streams are served by different hardware queues (a process has few of them);
 * on a shared queue the delivery sits behind the waiter until its spins run out. */
rdev_status rdev_consume_reduce_max(rdev_device_t *dev, rdev_plan_t *plan, uint32_t tensor_id, uint32_t max_spins,
                                    rdev_consume_result *out, void *stream);

/* The same consumer for a list of static tensors in one launch per 32 tensors:
 * out[i] belongs to tensor_ids[i].  Tensors are cut into 32 KiB units that the
 * workgroups take in list order, so tensors early in the list are reduced first.
 * With max_spins == 0 nothing waits: enqueue it on the delivery's own stream right
 * behind rdev_write_batch (stream order stands in for the flags; the cheapest way
 * to consume a whole batch), or anywhere once the host has seen the flags.
 * With max_spins > 0 a workgroup first waits (at most max_spins polls, a few
 * microseconds apart) for the in-arena flag of each tensor it meets; enqueued on a second stream behind a delivery that
 * is still in flight, one launch then consumes each tensor as its flag comes up
 * (with flag_groups > 1 while later groups are still moving).  At most 256
 * workgroups of 1024 lanes wait at a time; they hold wave slots the copy could use
 * (section 3.5: a copy beside them runs about a third slower).  A tensor whose flag does not come up in time keeps status 1.  The flags
 * are not cleared: consume them with rdev_poll afterwards.  For the waiting to
 * make progress the delivery must be on another stream, mapped to another
 * hardware queue, or already enqueued. */
rdev_status rdev_consume_batch(rdev_device_t *dev, rdev_plan_t *plan, const uint32_t *tensor_ids, uint32_t n,
                               uint32_t max_spins, rdev_consume_result *out, void *stream);

/* Polling-async reception (section 4): the listed static tensors form a ready
 * queue; the head is polled on the host; if its flag is not set it goes back to
 * the tail, otherwise the flag is consumed and the op turns asynchronous: its
 * consumer runs on consumer_stream and writes out[i] for tensor_ids[i].  Ops that
 * succeed one after the other are launched together (one clear on flag_stream,
 * one consumer launch) when the next poll fails or the queue is empty.  Returns
 * RDEV_OK when the queue is empty,
 * RDEV_NOT_READY after max_polls failed polls in total.  *polls_out (may be NULL)
 * = polls made. */
rdev_status rdev_recv_polling_async(rdev_device_t *dev, rdev_plan_t *plan, const uint32_t *tensor_ids, uint32_t n,
                                    rdev_consume_result *out, void *flag_stream, void *consumer_stream,
                                    uint64_t max_polls, uint64_t *polls_out);

/* ---- sender-side allocation-site tracing (section 3.4) ------------------- */

/* A tensor can only be sent without a copy if its buffer was allocated in
 * registered memory, and the buffer of a sent tensor may have been allocated
 * several nodes upstream (in-place nodes pass buffers through).  The paper
 * instruments the runtime's allocator: during the first mini-batch every
 * allocation is recorded as address -> (node id, index of this allocation
 * within the node's execution), a later allocation at the same address
 * overwriting the earlier one; when a node sends a tensor its buffer address is
 * looked up and the allocation site found is added to a set S; from the second
 * mini-batch on, an allocation whose (node id, index) is in S is served from the
 * allocator of the registered arena, every other one from the ordinary allocator.
 *
 * The tracer owns two sub-allocators: one over `pool` (caller-owned device
 * memory that is NOT registered: the ordinary allocator) and the registered
 * arena `arena_id`'s own (rdev_alloc_region).  Buffers are 256-byte aligned. */
typedef struct rdev_tracer_s rdev_tracer_t;

rdev_status rdev_tracer_open(rdev_device_t *dev, void *pool_base /* device pointer */, uint64_t pool_bytes,
                             uint32_t arena_id, rdev_tracer_t **out);
/* Releases every buffer and staging region still held, then the tracer. */
rdev_status rdev_tracer_close(rdev_tracer_t *tr);
/* Start of a mini-batch: every buffer and staging region of the previous one is
 * released (the caller has waited for its transfers), per-node allocation
 * indices restart at 0.  The first iteration begun is the tracing iteration. */
rdev_status rdev_tracer_begin_iteration(rdev_tracer_t *tr);
/* The instrumented allocator.  *alloc_index_out = how many allocations node_id
 * made before this one in the current iteration; *in_arena_out = 1 when the
 * buffer came from the registered arena.  RDEV_E_NOMEM if the chosen allocator is full. */
rdev_status rdev_tracer_alloc(rdev_tracer_t *tr, uint32_t node_id, uint64_t bytes, void **ptr_out,
                              uint32_t *alloc_index_out, uint32_t *in_arena_out);
/* Give a buffer back before the iteration ends (its address may be handed out again). */
rdev_status rdev_tracer_free(rdev_tracer_t *tr, void *ptr);
/* The lookup of section 3.4 alone, nothing moves: the buffer at `ptr` is being
 * transferred; in the tracing iteration its allocation site is added to S.
 * *registered_out = 1 when the buffer lies in the registered arena.  (Works on a
 * host-only device.) */
rdev_status rdev_tracer_mark_sent(rdev_tracer_t *tr, const void *ptr, uint32_t *registered_out);
/* Send static tensor `tensor_id` of `plan` from the buffer at `ptr` (a pointer
 * returned by rdev_tracer_alloc).  In the tracing iteration the buffer's
 * allocation site is added to S.  If the buffer is in registered memory this is
 * a zero-copy rdev_write_batch of one tensor; otherwise a registered staging
 * region is allocated in the arena, the tensor copied into it and written from
 * there (section 5.1, analysis switched off).  *copied_out = 1 in the second case. */
rdev_status rdev_tracer_send(rdev_tracer_t *tr, rdev_plan_t *plan, uint32_t tensor_id, const void *ptr,
                             uint32_t seq, void *stream, uint32_t *copied_out);
/* The set S, in insertion order. */
rdev_status rdev_tracer_set_size(const rdev_tracer_t *tr, uint32_t *n_out);
rdev_status rdev_tracer_set_get(const rdev_tracer_t *tr, uint32_t i, uint32_t *node_id_out, uint32_t *alloc_index_out);

/* ---- graph analysis: static shape inference (section 3.4, first step) ----- */

/* A small dataflow graph: values (tensors on edges) are produced by inputs
 * (placeholders with user-annotated shapes, variables) and by nodes with one
 * output each; every node has a shape-inference function that gives the output
 * shape from the input shapes.  Unknown dims (-1) propagate.  After inference,
 * every value consumed in another partition than the one that produces it is a
 * transferred tensor, and rdev_graph_transfers emits the rdev_tensor_desc list
 * that rdev_plan classifies and places (static iff no dim is -1). */
typedef struct rdev_graph_s rdev_graph_t;

enum {
    RDEV_OP_UNARY     = 0,  /* 1 input; output = input shape.  attrs: none */
    RDEV_OP_BINARY    = 1,  /* 2 inputs, elementwise with broadcasting (trailing dims aligned, 1 stretches) */
    RDEV_OP_MATMUL    = 2,  /* [.., m, k] x [k, n] -> [.., m, n].  attrs: transpose_a, transpose_b (of the last two dims) */
    RDEV_OP_TRANSPOSE = 3,  /* attrs: the permutation */
    RDEV_OP_RESHAPE   = 4,  /* attrs: target dims, at most one -1 (inferred when the element count is known) */
    RDEV_OP_CONCAT    = 5,  /* >= 1 inputs.  attrs: axis */
    RDEV_OP_REDUCE    = 6,  /* attrs: keepdims, then the reduced axes */
    RDEV_OP_GATHER    = 7,  /* inputs: params [V, ...], ids [...] -> ids.shape + params.shape[1:] */
    RDEV_OP_UNIQUE    = 8,  /* any shape -> [-1]: the count depends on the data */
    RDEV_OP_CONV2D    = 9,  /* x [N,H,W,C], filter [kh,kw,C,O].  attrs: stride_h, stride_w, padding (0 valid, 1 same) */
    RDEV_OP_GRAD      = 10, /* inputs: anything..., last = the value differentiated against -> its shape and type */
    RDEV_OP_CAST      = 11  /* attrs: new element type */
};

rdev_status rdev_graph_open(rdev_graph_t **out);
rdev_status rdev_graph_close(rdev_graph_t *g);
/* A value that enters the graph in `partition` with an annotated shape (dims[i] == -1: unknown). */
rdev_status rdev_graph_input(rdev_graph_t *g, uint32_t dtype, uint32_t ndims, const int64_t *dims, uint32_t partition,
                             uint32_t *value_out);
/* A node placed in `partition`; inputs are value ids created earlier (so insertion order is a topological order). */
rdev_status rdev_graph_node(rdev_graph_t *g, uint32_t op, const uint32_t *inputs, uint32_t n_inputs,
                            const int64_t *attrs, uint32_t n_attrs, uint32_t partition, uint32_t *value_out);
/* Run every node's shape function.  RDEV_E_INVAL with the node named in rdev_last_error() when known dims contradict. */
rdev_status rdev_graph_infer(rdev_graph_t *g);
/* Inferred type and shape of a value (out->tensor_id = value id, out->dst_arena = its partition). */
rdev_status rdev_graph_value(const rdev_graph_t *g, uint32_t value, rdev_tensor_desc *out);
/* The tensors that cross partitions, ordered by (value id, consumer partition):
 * out[i].tensor_id = i, out[i].dst_arena = partition_to_arena[consumer partition].
 * values_out / dst_partitions_out (host arrays of cap entries, may be NULL) tell which value goes where.
 * *n_out = number of transfers (also when cap is too small: then RDEV_E_NOMEM). */
rdev_status rdev_graph_transfers(const rdev_graph_t *g, const uint32_t *partition_to_arena, uint32_t n_partitions,
                                 rdev_tensor_desc *out, uint32_t *values_out, uint32_t *dst_partitions_out,
                                 uint32_t cap, uint32_t *n_out);

/* ---- measurement -------------------------------------------------------- */

/* What the HIP runtime reports for the device: out[0] = memory clock (kHz),
 * out[1] = memory bus width (bits), out[2] = compute units, out[3] = L2 cache bytes. */
rdev_status rdev_device_info(rdev_device_t *dev, uint64_t out[4]);

/* Time the batched copy kernel of whole-plan transfers (x == NULL) with HIP
 * events on the transfer's own stream: the launch is given a start and a stop
 * event of its own, which take the kernel's begin and end times (the flag
 * kernel that follows is outside).  Every `every`-th launch is timed, up to
 * max_samples of them; max_samples == 0 switches timing off.  Changing
 * max_samples waits for the device and re-creates the events; calling again
 * with the same max_samples only re-arms: no wait, samples not read yet are
 * dropped, and the caller must have waited for launches that were being timed.
 * Section 5 reports means over runs of 100 iterations; this gives the per-launch
 * figure those means are made of. */
rdev_status rdev_plan_profile(rdev_plan_t *plan, uint32_t max_samples, uint32_t every);
/* Waits for the recorded events, writes the durations in milliseconds of the
 * launches timed since the last read (at most cap) to ms_out (host pointer),
 * their number to *n_out, and starts over. */
rdev_status rdev_plan_profile_read(rdev_plan_t *plan, float *ms_out, uint32_t cap, uint32_t *n_out);

#ifdef __cplusplus
}
#endif
#endif /* RDEV_H */
