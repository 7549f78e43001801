/* Host-only workout of the library for a sanitizer build (address + undefined
 * behaviour): planner, region sub-allocator, graph analyzer and the tracer's
 * bookkeeping, all through the C ABI on a device without a GPU.  Prints
 * "san host ok" and returns 0 when every check holds; the sanitizers abort
 * the process on a memory error or undefined behaviour in the library. */
#include <stdio.h>
#include <stdlib.h>
#include <string.h>
#include "rdev.h"

#define CHECK(cond) do { if (!(cond)) { printf("FAILED line %d: %s (%s)\n", __LINE__, #cond, rdev_last_error()); return 1; } } while (0)

static uint64_t rnd_state = 88172645463325252ull;
static uint32_t rnd(void) {            /* xorshift64 */
    rnd_state ^= rnd_state << 13; rnd_state ^= rnd_state >> 7; rnd_state ^= rnd_state << 17;
    return (uint32_t)(rnd_state >> 11);
}

int main(void) {
    rdev_device_t *dev = NULL;
    uint32_t arenas[4], i, n;
    CHECK(rdev_open(&dev, RDEV_HOST_ONLY) == RDEV_OK);
    for (i = 0; i < 4; ++i)
        CHECK(rdev_register_arena(dev, (void *)(0x700000000000ull + ((uint64_t)i << 40)), 1ull << 34, 0, &arenas[i]) == RDEV_OK);
    CHECK(rdev_register_arena(dev, (void *)0x700000000100ull, 4096, 0, &n) == RDEV_E_OVERLAP);
    CHECK(rdev_register_arena(dev, (void *)0x123, 4096, 0, &n) == RDEV_E_ALIGN);

    /* region allocator: random alloc / free, then everything returned leaves one free block */
    {
        rdev_region live[64];
        uint32_t nlive = 0, step;
        for (step = 0; step < 4000; ++step) {
            if (nlive < 64 && (rnd() & 3)) {
                uint64_t align = 1ull << (rnd() % 13);
                if (rdev_alloc_region(dev, arenas[0], 1 + rnd() % 100000, align, &live[nlive]) == RDEV_OK) {
                    CHECK(live[nlive].offset % align == 0);
                    ++nlive;
                }
            } else if (nlive) {
                uint32_t k = rnd() % nlive;
                CHECK(rdev_free_region(dev, &live[k]) == RDEV_OK);
                CHECK(rdev_free_region(dev, &live[k]) == RDEV_E_INVAL);     /* double free is refused */
                live[k] = live[--nlive];
            }
        }
        while (nlive) CHECK(rdev_free_region(dev, &live[--nlive]) == RDEV_OK);
        CHECK(rdev_alloc_region(dev, arenas[0], 1ull << 34, 256, &live[0]) == RDEV_OK && live[0].offset == 0);
        CHECK(rdev_alloc_region(dev, arenas[0], 1, 1, &live[1]) == RDEV_E_NOMEM);
        CHECK(rdev_free_region(dev, &live[0]) == RDEV_OK);
        CHECK(rdev_alloc_region(dev, arenas[0], 16, 3, &live[0]) == RDEV_E_ALIGN);
        CHECK(rdev_alloc_region(dev, 99, 16, 16, &live[0]) == RDEV_E_INVAL);
    }

    /* plans: many random tensors, every option; then the error paths */
    {
        uint32_t round;
        for (round = 0; round < 30; ++round) {
            enum { N = 300 };
            static rdev_tensor_desc t[N];
            rdev_plan_opts o;
            rdev_plan_t *plan = NULL;
            rdev_placement p;
            const void *src[N];
            uint32_t cnt;
            memset(t, 0, sizeof t);
            memset(&o, 0, sizeof o);
            for (i = 0; i < N; ++i) {
                uint32_t d;
                t[i].tensor_id = 1000 + i;
                t[i].dtype = rnd() % 9;
                t[i].ndims = rnd() % (RDEV_MAX_DIMS + 1);
                t[i].dst_arena = arenas[rnd() % 4];
                for (d = 0; d < t[i].ndims; ++d) t[i].dims[d] = (rnd() % 17 == 0) ? -1 : (int64_t)(rnd() % 9);
                src[i] = (const void *)(0x700000000000ull + ((uint64_t)3 << 40) + (1ull << 33) + 4096ull * i);
            }
            o.align = 16ull << (rnd() % 9);
            o.max_static_bytes = (round & 1) ? 1 + rnd() % 5000 : 0;
            o.dyn_heap_bytes = rnd() % 100000;
            o.chunk_bytes = 256ull * (1 + rnd() % 64);
            o.small_bytes = rnd() % 8192;
            o.flag_groups = rnd() % 7;
            o.rpc_frag_bytes = 16ull * (rnd() % 100);
            CHECK(rdev_plan(dev, t, N, &o, &plan) == RDEV_OK);
            CHECK(rdev_plan_count(plan, &cnt) == RDEV_OK && cnt == N);
            for (i = 0; i < N; ++i) {
                CHECK(rdev_plan_get(plan, i, &p) == RDEV_OK && p.tensor_id == 1000 + i);
                CHECK((p.kind == RDEV_STATIC ? p.data_offset : p.meta_offset) % o.align == 0);
            }
            CHECK(rdev_plan_get(plan, N, &p) == RDEV_E_INVAL);
            CHECK(rdev_plan_bind_sources(plan, src, N) == RDEV_OK);          /* builds the work-item table on the host */
            CHECK(rdev_plan_bind_sources(plan, src, N - 1) == RDEV_E_INVAL);
            CHECK(rdev_dyn_reset(plan) == RDEV_OK);
            CHECK(rdev_write_batch(dev, plan, NULL, 0, RDEV_ZEROCOPY, 1, NULL) == RDEV_E_HIP);
            CHECK(rdev_write_batch_fixed_staging(dev, plan, NULL, 0, 1, NULL) == RDEV_E_HIP);
            CHECK(rdev_read_batch_device(dev, plan, NULL, 0, 1, NULL) == RDEV_E_INVAL);
            CHECK(rdev_plan_free(plan) == RDEV_OK);
        }
        {
            rdev_tensor_desc t[2];
            rdev_plan_t *plan = NULL;
            rdev_plan_opts o;
            memset(t, 0, sizeof t);
            memset(&o, 0, sizeof o);
            t[0].tensor_id = 1; t[0].dtype = RDEV_F64; t[0].ndims = 3; t[0].dst_arena = arenas[1];
            t[0].dims[0] = 1ll << 31; t[0].dims[1] = 1ll << 31; t[0].dims[2] = 4;      /* 2^67 bytes */
            CHECK(rdev_plan(dev, t, 1, NULL, &plan) == RDEV_E_OVERFLOW);
            t[0].dims[0] = 1ll << 40; t[0].dims[1] = 1; t[0].dims[2] = 1;              /* 8 TiB does not fit a 16 GiB arena */
            CHECK(rdev_plan(dev, t, 1, NULL, &plan) == RDEV_E_NOMEM);
            t[0].dims[0] = 4; t[0].dims[1] = -2;
            CHECK(rdev_plan(dev, t, 1, NULL, &plan) == RDEV_E_INVAL);
            t[0].dims[1] = 2; t[0].ndims = RDEV_MAX_DIMS + 1;
            CHECK(rdev_plan(dev, t, 1, NULL, &plan) == RDEV_E_INVAL);
            t[0].ndims = 2; t[0].dtype = 77;
            CHECK(rdev_plan(dev, t, 1, NULL, &plan) == RDEV_E_INVAL);
            t[0].dtype = RDEV_U8; t[1] = t[0];
            CHECK(rdev_plan(dev, t, 2, NULL, &plan) == RDEV_E_INVAL);                  /* duplicate id */
            t[1].tensor_id = 2; t[1].dst_arena = 1234;
            CHECK(rdev_plan(dev, t, 2, NULL, &plan) == RDEV_E_INVAL);                  /* unknown arena */
            t[1].dst_arena = arenas[2];
            o.align = 48;
            CHECK(rdev_plan(dev, t, 2, &o, &plan) == RDEV_E_ALIGN);
            o.align = 8;
            CHECK(rdev_plan(dev, t, 2, &o, &plan) == RDEV_E_ALIGN);
            o.align = 0; o.chunk_bytes = 100;
            CHECK(rdev_plan(dev, t, 2, &o, &plan) == RDEV_E_INVAL);
            o.chunk_bytes = 0; o.flags = 0x80;
            CHECK(rdev_plan(dev, t, 2, &o, &plan) == RDEV_E_INVAL);
            CHECK(rdev_plan(dev, NULL, 0, NULL, &plan) == RDEV_OK);                    /* an empty plan is legal */
            CHECK(rdev_plan_free(plan) == RDEV_OK);
        }
    }

    /* graph analyzer: a chain of every op, unknown dims, contradictions */
    {
        rdev_graph_t *g = NULL;
        uint32_t x, w, v, u, ids, nt, p2a[2];
        int64_t d2[2], at[4];
        uint32_t in2[2];
        rdev_tensor_desc out[16];
        uint32_t vals[16], parts[16];
        rdev_tensor_desc val;
        p2a[0] = arenas[0]; p2a[1] = arenas[1];
        CHECK(rdev_graph_open(&g) == RDEV_OK);
        d2[0] = -1; d2[1] = 64;
        CHECK(rdev_graph_input(g, RDEV_F32, 2, d2, 0, &x) == RDEV_OK);
        d2[0] = 64; d2[1] = 32;
        CHECK(rdev_graph_input(g, RDEV_F32, 2, d2, 1, &w) == RDEV_OK);
        in2[0] = x; in2[1] = w; at[0] = 0; at[1] = 0;
        CHECK(rdev_graph_node(g, RDEV_OP_MATMUL, in2, 2, at, 2, 0, &v) == RDEV_OK);
        at[0] = 1; at[1] = 0;
        CHECK(rdev_graph_node(g, RDEV_OP_TRANSPOSE, &v, 1, at, 2, 0, &v) == RDEV_OK);
        at[0] = -1; at[1] = 8;
        CHECK(rdev_graph_node(g, RDEV_OP_RESHAPE, &v, 1, at, 2, 0, &v) == RDEV_OK);
        at[0] = 0; at[1] = 1;
        CHECK(rdev_graph_node(g, RDEV_OP_REDUCE, &v, 1, at, 2, 0, &v) == RDEV_OK);
        d2[0] = 7;
        CHECK(rdev_graph_input(g, RDEV_I64, 1, d2, 0, &ids) == RDEV_OK);
        CHECK(rdev_graph_node(g, RDEV_OP_UNIQUE, &ids, 1, NULL, 0, 0, &u) == RDEV_OK);
        in2[0] = w; in2[1] = u;
        CHECK(rdev_graph_node(g, RDEV_OP_GATHER, in2, 2, NULL, 0, 0, &v) == RDEV_OK);
        in2[0] = v; in2[1] = w;
        CHECK(rdev_graph_node(g, RDEV_OP_GRAD, in2, 2, NULL, 0, 0, &v) == RDEV_OK);
        in2[0] = w; in2[1] = v;
        CHECK(rdev_graph_node(g, RDEV_OP_BINARY, in2, 2, NULL, 0, 1, &v) == RDEV_OK);
        at[0] = RDEV_F16;
        CHECK(rdev_graph_node(g, RDEV_OP_CAST, &v, 1, at, 1, 1, &v) == RDEV_OK);
        CHECK(rdev_graph_value(g, v, &val) == RDEV_E_STATE);
        CHECK(rdev_graph_infer(g) == RDEV_OK);
        CHECK(rdev_graph_value(g, v, &val) == RDEV_OK && val.dtype == RDEV_F16 && val.ndims == 2 && val.dims[0] == 64 && val.dims[1] == 32);
        CHECK(rdev_graph_transfers(g, p2a, 2, NULL, NULL, NULL, 0, &nt) == RDEV_E_NOMEM || nt == 0);
        CHECK(nt >= 2 && nt <= 16);
        CHECK(rdev_graph_transfers(g, p2a, 2, out, vals, parts, 16, &nt) == RDEV_OK);
        CHECK(rdev_graph_transfers(g, p2a, 1, out, vals, parts, 16, &nt) == RDEV_E_INVAL);
        in2[0] = x; in2[1] = x; at[0] = 0; at[1] = 0;
        CHECK(rdev_graph_node(g, RDEV_OP_MATMUL, in2, 2, at, 2, 0, &v) == RDEV_OK);      /* [-1,64] x [-1,64]: 64 vs unknown is fine */
        d2[0] = 5; d2[1] = 6;
        CHECK(rdev_graph_input(g, RDEV_F32, 2, d2, 0, &x) == RDEV_OK);
        in2[0] = x; in2[1] = w;
        CHECK(rdev_graph_node(g, RDEV_OP_MATMUL, in2, 2, at, 2, 0, &v) == RDEV_OK);      /* 6 vs 64: contradiction */
        CHECK(rdev_graph_infer(g) == RDEV_E_INVAL);
        in2[0] = 1000;
        CHECK(rdev_graph_node(g, RDEV_OP_UNARY, in2, 1, NULL, 0, 0, &v) == RDEV_E_INVAL);
        CHECK(rdev_graph_close(g) == RDEV_OK);
    }

    /* tracer bookkeeping (no transfers on a host-only device) */
    {
        rdev_tracer_t *tr = NULL;
        void *p[8];
        uint32_t idx, in_arena, reg, ns, a, b, it;
        CHECK(rdev_tracer_open(dev, (void *)0x600000000000ull, 1u << 20, arenas[3], &tr) == RDEV_OK);
        CHECK(rdev_tracer_alloc(tr, 1, 100, &p[0], &idx, &in_arena) == RDEV_E_STATE);
        for (it = 0; it < 3; ++it) {
            CHECK(rdev_tracer_begin_iteration(tr) == RDEV_OK);
            for (i = 0; i < 8; ++i) {
                CHECK(rdev_tracer_alloc(tr, i % 3, 1000 + 10 * i, &p[i], &idx, &in_arena) == RDEV_OK);
                CHECK(idx == i / 3);
                CHECK(in_arena == (it > 0 && (i == 2 || i == 5)));
            }
            CHECK(rdev_tracer_mark_sent(tr, p[2], &reg) == RDEV_OK && reg == (it > 0));
            CHECK(rdev_tracer_mark_sent(tr, p[5], &reg) == RDEV_OK);
            CHECK(rdev_tracer_free(tr, p[0]) == RDEV_OK);
            CHECK(rdev_tracer_free(tr, p[0]) == RDEV_E_INVAL);
            CHECK(rdev_tracer_mark_sent(tr, p[0], &reg) == RDEV_E_INVAL);
        }
        CHECK(rdev_tracer_set_size(tr, &ns) == RDEV_OK && ns == 2);
        CHECK(rdev_tracer_set_get(tr, 0, &a, &b) == RDEV_OK && a == 2 && b == 0);
        CHECK(rdev_tracer_set_get(tr, 1, &a, &b) == RDEV_OK && a == 2 && b == 1);
        CHECK(rdev_tracer_set_get(tr, 2, &a, &b) == RDEV_E_INVAL);
        CHECK(rdev_tracer_close(tr) == RDEV_OK);
    }

    for (i = 0; i < 4; ++i) CHECK(rdev_unregister_arena(dev, arenas[i]) == RDEV_OK);
    CHECK(rdev_unregister_arena(dev, arenas[0]) == RDEV_E_INVAL);
    CHECK(rdev_close(dev) == RDEV_OK);
    printf("san host ok\n");
    return 0;
}
