/*
 * The library used from plain C, with nothing but the HIP runtime around it:
 * device memory from hipMalloc, pinned memory from hipHostMalloc, no Python.
 * One small batch goes pool -> transfer buffer -> second pool on the GPU and is
 * compared byte for byte with the CPU oracle (compiled into this program from
 * oracle/kvl_oracle.c).  Because every buffer here is an allocation of exactly
 * its own size, the entry points' buffer checks are exercised at their edges: a
 * pool one block short and a transfer buffer shorter than its stated capacity
 * must come back as KVL_ESPACE, pageable host memory as KVL_EINVAL, and none
 * of them may launch anything.  Then the other calls of the boundary: the
 * host-buffer load, the appended tail's way back, a layer out of Full Blocks in
 * pinned memory, and three layers streamed into two resident slots (staged and
 * zero-copy), each against the oracle.
 *
 * Prints one line per check and "c parity ok" at the end; exit status 0 only
 * if every check passed.
 *
 * With the argument "submission" it runs the submission-cost study instead
 * (Section 5.2 of the paper: handing a copy engine many small copies is bound by
 * the cost of submitting each): 2048 Layer Blocks of 72 KiB in random pool
 * order, host buffer -> pool, by one hipMemcpyAsync per block, by one
 * hipMemcpyBatchAsync for all of them (this program links the system's HIP
 * runtime, which has that call), by the staged path and by the zero-copy kernel;
 * every result is compared with the oracle's.
 */
#define _POSIX_C_SOURCE 199309L
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>
#include <time.h>

#include <hip/hip_runtime_api.h>

#include "kvl.h"

/* the oracle's entry points (oracle/kvl_oracle.c) */
int kvo_pack(uint32_t bs, uint32_t n_planes, const uint32_t *row_bytes, uint32_t n_req, const uint32_t *hit,
             const int32_t *const *tables, const uint8_t *const *pool_planes, uint8_t *xfer,
             uint32_t r_begin, uint32_t r_end);
int kvo_unpack(uint32_t bs, uint32_t n_planes, const uint32_t *row_bytes, uint32_t n_req, const uint32_t *hit,
               const int32_t *const *tables, const uint8_t *xfer, uint8_t *const *pool_planes,
               uint32_t r_begin, uint32_t r_end);
uint64_t kvo_payload_bytes(uint32_t n_req, const uint32_t *hit, uint32_t n_planes, const uint32_t *row_bytes);
int kvo_pack_range(uint32_t bs, uint32_t n_planes, const uint32_t *row_bytes, uint32_t n_req, const uint32_t *first,
                   const uint32_t *count, const int32_t *const *tables, const uint8_t *const *pool_planes,
                   uint8_t *xfer, uint32_t r_begin, uint32_t r_end);
int kvo_unpack_range(uint32_t bs, uint32_t n_planes, const uint32_t *row_bytes, uint32_t n_req, const uint32_t *first,
                     const uint32_t *count, const int32_t *const *tables, const uint8_t *xfer,
                     uint8_t *const *pool_planes, uint32_t r_begin, uint32_t r_end);
uint64_t kvo_fullblock_bytes(uint32_t bs, uint32_t n_layers, uint32_t n_planes, const uint32_t *row_bytes);
uint64_t kvo_fullblock_count(uint32_t bs, uint32_t n_req, const uint32_t *first, const uint32_t *count);
int kvo_fullblocks_to_pool(uint32_t bs, uint32_t n_layers, uint32_t n_planes, const uint32_t *row_bytes, uint32_t n_req,
                           const uint32_t *first, const uint32_t *count, const int32_t *const *tables, uint32_t layer,
                           const uint8_t *blocks, uint8_t *const *pool_planes);

#define HIP_OK(call)                                                                      \
    do {                                                                                  \
        hipError_t e_ = (call);                                                           \
        if (e_ != hipSuccess) {                                                           \
            fprintf(stderr, "%s:%d: %s: %s\n", __FILE__, __LINE__, #call, hipGetErrorString(e_)); \
            exit(2);                                                                      \
        }                                                                                 \
    } while (0)

static int failures = 0;

static void expect(int got, int want, const char *what) {
    printf("%-72s %s (%d)\n", what, got == want ? "ok" : "FAILED", got);
    fflush(stdout);
    if (got != want) ++failures;
}

/* splitmix64: the inputs are this program's own, seeded */
static uint64_t rng_state = 20260221u;
static uint64_t rnd(void) {
    uint64_t z = (rng_state += 0x9E3779B97F4A7C15ull);
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

enum { R = 5, BS = 16, P = 2, POOL_BLOCKS = 96 };

/* kvl_stream_layers' host_fill: the storage read of layer `layer` delivers its bytes here */
struct fill_ctx {
    uint8_t *const *layer_payload;
    int calls;
};
static int fill_layer(void *user, uint32_t layer, void *host_slot, uint64_t bytes) {
    struct fill_ctx *c = (struct fill_ctx *)user;
    memcpy(host_slot, c->layer_payload[layer], bytes);
    c->calls++;
    return 0;
}

static double now_ms(void) {
    struct timespec t;
    clock_gettime(CLOCK_MONOTONIC, &t);
    return t.tv_sec * 1e3 + t.tv_nsec * 1e-6;
}

static int submission_study(void) {
    enum { SR = 8, SBS = 64, BLOCKS_PER_REQ = 256, SPOOL = 2304 };
    const uint32_t row[1] = {1152};
    const size_t blk = (size_t)SBS * row[0];
    static int32_t tab[SR][BLOCKS_PER_REQ];
    static int32_t perm[SPOOL];
    const int32_t *tabs[SR];
    kvl_request_t req[SR];
    uint32_t hit[SR];
    for (int i = 0; i < SPOOL; ++i) perm[i] = i;
    for (int i = SPOOL - 1; i > 0; --i) {
        int j = (int)(rnd() % (uint64_t)(i + 1));
        int32_t t = perm[i]; perm[i] = perm[j]; perm[j] = t;
    }
    for (int r = 0; r < SR; ++r) {
        for (int b = 0; b < BLOCKS_PER_REQ; ++b) tab[r][b] = perm[r * BLOCKS_PER_REQ + b];
        tabs[r] = tab[r];
        hit[r] = BLOCKS_PER_REQ * SBS;
        req[r].hit_tokens = hit[r];
        req[r].append_tokens = 0;
        req[r].n_blocks = BLOCKS_PER_REQ;
        req[r].block_table = tab[r];
    }
    kvl_layout_t lay;
    memset(&lay, 0, sizeof lay);
    lay.n_layers = 1; lay.block_tokens = SBS; lay.n_planes = 1; lay.row_bytes[0] = row[0]; lay.pool_blocks = SPOOL;
    kvl_plan_t *s = NULL;
    expect(kvl_plan(&lay, req, SR, KVL_SCATTER | KVL_NO_MERGE, &s), KVL_OK, "kvl_plan (2048 blocks, unmerged)");
    if (failures) return 1;
    uint64_t payload = 0, n_units = 0;
    kvl_plan_payload_bytes(s, &payload);
    kvl_plan_n_units(s, &n_units);
    const size_t pool_bytes = (size_t)SPOOL * blk;
    uint8_t *want = malloc(pool_bytes), *got = malloc(pool_bytes);
    void *pinned = NULL, *d_pool = NULL, *d_stage = NULL;
    HIP_OK(hipHostMalloc(&pinned, payload, hipHostMallocDefault));
    for (uint64_t i = 0; i < payload; ++i) ((uint8_t *)pinned)[i] = (uint8_t)rnd();
    HIP_OK(hipMalloc(&d_pool, pool_bytes));
    const uint64_t chunk = 16u << 20, stage_bytes = 3 * chunk;
    HIP_OK(hipMalloc(&d_stage, stage_bytes));
    memset(want, 0xA5, pool_bytes);
    uint8_t *wantp[1] = {want};
    if (kvo_unpack(SBS, 1, row, SR, hit, tabs, pinned, wantp, 0, SR) != 0) return 2;
    hipStream_t cs, ks;
    HIP_OK(hipStreamCreateWithFlags(&cs, hipStreamNonBlocking));
    HIP_OK(hipStreamCreateWithFlags(&ks, hipStreamNonBlocking));
    void *planes[1] = {d_pool};
    printf("%llu descriptors of %zu bytes, payload %.1f MB\n", (unsigned long long)n_units, blk, payload / 1e6);
    for (int mode = 0; mode < 4; ++mode) {
        static const char *names[4] = {"one hipMemcpyAsync per block", "one hipMemcpyBatchAsync for all blocks",
                                       "staged: 16 MiB chunks, 3 slots, scatter kernels", "zero-copy scatter kernel"};
        double best_submit = 1e30, best_total = 1e30;
        int rc = KVL_OK;
        for (int rep = 0; rep < 4 && rc == KVL_OK; ++rep) {
            HIP_OK(hipMemset(d_pool, 0xA5, pool_bytes));
            HIP_OK(hipDeviceSynchronize());
            uint64_t copies = 0;
            const double t0 = now_ms();
            if (mode == 0) rc = kvl_h2d_blockwise_layer(s, pinned, planes, ks, &copies);
            else if (mode == 1) rc = kvl_h2d_blockwise_batched_layer(s, pinned, planes, ks, &copies);
            else if (mode == 2) rc = kvl_h2d_unpack_layer(s, pinned, d_stage, stage_bytes, chunk, planes, cs, ks);
            else rc = kvl_h2d_unpack_layer(s, pinned, NULL, 0, 0, planes, cs, ks);
            const double t1 = now_ms();
            HIP_OK(hipStreamSynchronize(ks));
            HIP_OK(hipStreamSynchronize(cs));
            const double t2 = now_ms();
            if (rep) {      /* the first round warms up */
                if (t1 - t0 < best_submit) best_submit = t1 - t0;
                if (t2 - t0 < best_total) best_total = t2 - t0;
            }
        }
        if (rc == KVL_ENOSYS) {
            printf("%-52s not available in this HIP runtime\n", names[mode]);
            continue;
        }
        expect(rc, KVL_OK, names[mode]);
        HIP_OK(hipMemcpy(got, d_pool, pool_bytes, hipMemcpyDeviceToHost));
        expect(memcmp(got, want, pool_bytes) == 0, 1, "  pool equals the oracle's");
        printf("  host time in the call %.3f ms (%.2f us per block), until done %.3f ms = %.2f GB/s\n", best_submit,
               best_submit * 1e3 / (double)n_units, best_total, payload / best_total / 1e6);
        fflush(stdout);
    }
    kvl_plan_destroy(s);
    kvl_release_cached_memory();
    HIP_OK(hipStreamDestroy(cs));
    HIP_OK(hipStreamDestroy(ks));
    HIP_OK(hipFree(d_stage));
    HIP_OK(hipFree(d_pool));
    HIP_OK(hipHostFree(pinned));
    free(want); free(got);
    if (failures) {
        printf("submission study: %d check(s) FAILED\n", failures);
        return 1;
    }
    printf("submission study ok\n");
    return 0;
}

int main(int argc, char **argv) {
    if (argc > 1 && strcmp(argv[1], "submission") == 0) return submission_study();
    const uint32_t rows[P] = {656, 256};
    const uint32_t hit[R] = {100, 16, 0, 333, 47}, app[R] = {9, 0, 20, 3, 1};
    int32_t src_tab[R][32], dst_tab[R][32];
    const int32_t *src_tabs[R], *dst_tabs[R];
    kvl_request_t src_req[R], dst_req[R];

    /* two independent seeded permutations of the pool's blocks, dealt out in order */
    int32_t perm_a[POOL_BLOCKS], perm_b[POOL_BLOCKS];
    for (int i = 0; i < POOL_BLOCKS; ++i) perm_a[i] = perm_b[i] = i;
    for (int i = POOL_BLOCKS - 1; i > 0; --i) {
        int j = (int)(rnd() % (uint64_t)(i + 1)), k = (int)(rnd() % (uint64_t)(i + 1));
        int32_t t = perm_a[i]; perm_a[i] = perm_a[j]; perm_a[j] = t;
        t = perm_b[i]; perm_b[i] = perm_b[k]; perm_b[k] = t;
    }
    uint32_t next = 0;
    for (int r = 0; r < R; ++r) {
        const uint32_t nb = (hit[r] + app[r] + BS - 1) / BS;
        for (uint32_t b = 0; b < nb; ++b, ++next) {
            src_tab[r][b] = perm_a[next];
            dst_tab[r][b] = perm_b[next];
        }
        src_tabs[r] = src_tab[r];
        dst_tabs[r] = dst_tab[r];
        src_req[r].hit_tokens = dst_req[r].hit_tokens = hit[r];
        src_req[r].append_tokens = dst_req[r].append_tokens = app[r];
        src_req[r].n_blocks = dst_req[r].n_blocks = nb;
        src_req[r].block_table = src_tab[r];
        dst_req[r].block_table = dst_tab[r];
    }
    if (next > POOL_BLOCKS) return 2;

    kvl_layout_t lay;
    memset(&lay, 0, sizeof lay);
    lay.n_layers = 1;
    lay.block_tokens = BS;
    lay.n_planes = P;
    lay.row_bytes[0] = rows[0];
    lay.row_bytes[1] = rows[1];
    lay.pool_blocks = POOL_BLOCKS;

    /* host copies: source pool of seeded bytes, destination pool of a sentinel */
    size_t plane_bytes[P];
    uint8_t *h_src[P], *h_dst[P], *h_dst_want[P];
    void *d_src[P], *d_dst[P];
    for (int p = 0; p < P; ++p) {
        plane_bytes[p] = (size_t)POOL_BLOCKS * BS * rows[p];
        h_src[p] = malloc(plane_bytes[p]);
        h_dst[p] = malloc(plane_bytes[p]);
        h_dst_want[p] = malloc(plane_bytes[p]);
        for (size_t i = 0; i < plane_bytes[p]; ++i) h_src[p][i] = (uint8_t)rnd();
        memset(h_dst_want[p], 0xA5, plane_bytes[p]);
        HIP_OK(hipMalloc(&d_src[p], plane_bytes[p]));
        HIP_OK(hipMalloc(&d_dst[p], plane_bytes[p]));
        HIP_OK(hipMemcpy(d_src[p], h_src[p], plane_bytes[p], hipMemcpyHostToDevice));
        HIP_OK(hipMemset(d_dst[p], 0xA5, plane_bytes[p]));
    }

    const uint64_t payload = kvo_payload_bytes(R, hit, P, rows);
    uint8_t *want_xfer = malloc(payload), *got_xfer = malloc(payload);
    if (kvo_pack(BS, P, rows, R, hit, src_tabs, (const uint8_t *const *)h_src, want_xfer, 0, R) != 0) return 2;
    if (kvo_unpack(BS, P, rows, R, hit, dst_tabs, want_xfer, h_dst_want, 0, R) != 0) return 2;

    kvl_plan_t *g = NULL, *s = NULL;
    expect(kvl_plan(&lay, src_req, R, KVL_GATHER, &g), KVL_OK, "kvl_plan (gather)");
    expect(kvl_plan(&lay, dst_req, R, KVL_SCATTER, &s), KVL_OK, "kvl_plan (scatter)");
    if (failures) return 1;
    uint64_t lib_payload = 0;
    kvl_plan_payload_bytes(g, &lib_payload);
    expect(lib_payload == payload, 1, "payload bytes equal the oracle's");

    void *d_xfer = NULL, *d_short = NULL, *pinned = NULL;
    HIP_OK(hipMalloc(&d_xfer, payload));
    HIP_OK(hipMalloc(&d_short, payload - 4096));
    HIP_OK(hipHostMalloc(&pinned, payload, hipHostMallocDefault));

    /* --- refusals first.  Each bad buffer is shown to kvl_check_buffer alone before an
     * entry point sees it, and the entry point is only called if that check refused it:
     * whatever happens, nothing here launches a kernel on memory that is not there. --- */
    expect(kvl_check_buffer(d_xfer, payload, 0), KVL_OK, "kvl_check_buffer: exact device allocation");
    expect(kvl_check_buffer(d_xfer, payload + 1, 0), KVL_ESPACE, "kvl_check_buffer: one byte past the allocation");
    expect(kvl_check_buffer((char *)d_xfer + payload - 16, 16, 0), KVL_OK, "kvl_check_buffer: last 16 bytes");
    expect(kvl_check_buffer(pinned, payload, 1), KVL_OK, "kvl_check_buffer: pinned host memory where allowed");
    expect(kvl_check_buffer(pinned, payload, 0), KVL_EINVAL, "kvl_check_buffer: pinned host memory where not");
    expect(kvl_check_buffer(pinned, payload + 1, 1), KVL_ESPACE, "kvl_check_buffer: one byte past a pinned allocation");
    expect(kvl_check_buffer((char *)pinned + 64, payload - 64, 1), KVL_OK, "kvl_check_buffer: inside a pinned allocation");

    void *short_pool[P] = {d_src[0], NULL};
    HIP_OK(hipMalloc(&short_pool[1], plane_bytes[1] - (size_t)BS * rows[1]));
    void *host_pool[P] = {h_dst[0], h_dst[1]};
    int refused;
    refused = kvl_check_buffer(short_pool[1], plane_bytes[1], 0);
    expect(refused, KVL_ESPACE, "kvl_check_buffer: pool plane one block short");
    if (refused != KVL_OK)
        expect(kvl_pack_layer(g, (const void *const *)short_pool, d_xfer, payload, NULL), KVL_ESPACE,
               "pack from a pool plane one block short");
    refused = kvl_check_buffer(d_short, payload, 1);
    expect(refused, KVL_ESPACE, "kvl_check_buffer: allocation shorter than the payload");
    if (refused != KVL_OK) {
        expect(kvl_pack_layer(g, (const void *const *)d_src, d_short, payload, NULL), KVL_ESPACE,
               "pack into an allocation shorter than the stated capacity");
        expect(kvl_unpack_layer(s, d_short, payload, d_dst, NULL), KVL_ESPACE,
               "unpack from an allocation shorter than the stated size");
    }
    refused = kvl_check_buffer((char *)d_xfer + 16, payload, 1);
    expect(refused, KVL_ESPACE, "kvl_check_buffer: span that starts 16 bytes into its allocation");
    if (refused != KVL_OK)
        expect(kvl_pack_layer(g, (const void *const *)d_src, (char *)d_xfer + 16, payload, NULL), KVL_ESPACE,
               "pack into a buffer that starts 16 bytes into its allocation");
    refused = kvl_check_buffer(got_xfer, payload, 1);
    expect(refused, KVL_EINVAL, "kvl_check_buffer: pageable host memory");
    if (refused != KVL_OK) {
        expect(kvl_pack_layer(g, (const void *const *)d_src, got_xfer, payload, NULL), KVL_EINVAL,
               "pack into pageable host memory");
        expect(kvl_unpack_layer(s, d_xfer, payload, host_pool, NULL), KVL_EINVAL,
               "unpack into a pool in pageable host memory");
    }

    /* --- the hop on the device --- */
    HIP_OK(hipMemset(d_xfer, 0, payload));
    expect(kvl_pack_layer(g, (const void *const *)d_src, d_xfer, payload, NULL), KVL_OK, "kvl_pack_layer");
    HIP_OK(hipDeviceSynchronize());
    HIP_OK(hipMemcpy(got_xfer, d_xfer, payload, hipMemcpyDeviceToHost));
    expect(memcmp(got_xfer, want_xfer, payload) == 0, 1, "transfer buffer equals the oracle's");
    expect(kvl_unpack_layer(s, d_xfer, payload, d_dst, NULL), KVL_OK, "kvl_unpack_layer");
    HIP_OK(hipDeviceSynchronize());
    for (int p = 0; p < P; ++p) {
        HIP_OK(hipMemcpy(h_dst[p], d_dst[p], plane_bytes[p], hipMemcpyDeviceToHost));
        expect(memcmp(h_dst[p], h_dst_want[p], plane_bytes[p]) == 0, 1,
               p == 0 ? "destination pool plane 0 equals the oracle's (sentinel elsewhere)"
                      : "destination pool plane 1 equals the oracle's (sentinel elsewhere)");
    }

    /* --- the same gather written straight into pinned host memory --- */
    memset(pinned, 0, payload);
    expect(kvl_pack_layer(g, (const void *const *)d_src, pinned, payload, NULL), KVL_OK,
           "kvl_pack_layer into pinned host memory");
    HIP_OK(hipDeviceSynchronize());
    expect(memcmp(pinned, want_xfer, payload) == 0, 1, "pinned transfer buffer equals the oracle's");

    /* --- host buffer -> staging -> pool --- */
    for (int p = 0; p < P; ++p) HIP_OK(hipMemset(d_dst[p], 0xA5, plane_bytes[p]));
    void *d_stage = NULL;
    const uint64_t chunk = 131072, stage_bytes = 3 * chunk;   /* no descriptor exceeds 128 KiB */
    HIP_OK(hipMalloc(&d_stage, stage_bytes));
    hipStream_t cs, ks;
    HIP_OK(hipStreamCreateWithFlags(&cs, hipStreamNonBlocking));
    HIP_OK(hipStreamCreateWithFlags(&ks, hipStreamNonBlocking));
    expect(kvl_h2d_unpack_layer(s, pinned, d_stage, stage_bytes, chunk, d_dst, cs, ks), KVL_OK,
           "kvl_h2d_unpack_layer (3 staging slots of 128 KiB)");
    HIP_OK(hipStreamSynchronize(ks));
    HIP_OK(hipStreamSynchronize(cs));
    for (int p = 0; p < P; ++p) {
        HIP_OK(hipMemcpy(h_dst[p], d_dst[p], plane_bytes[p], hipMemcpyDeviceToHost));
        expect(memcmp(h_dst[p], h_dst_want[p], plane_bytes[p]) == 0, 1, "pool plane after the host-buffer load");
    }
    refused = kvl_check_buffer(d_stage, 4 * chunk, 0);
    expect(refused, KVL_ESPACE, "kvl_check_buffer: staging area stated larger than its allocation");
    if (refused != KVL_OK)
        expect(kvl_h2d_unpack_layer(s, pinned, d_stage, 4 * chunk, chunk, d_dst, cs, ks), KVL_ESPACE,
               "host-buffer load with a staging area stated larger than its allocation");

    /* --- the appended tail goes back (Section 4.1: only the miss tokens' cache returns to the decode
     * engine, where it is merged with the hit tokens' cache): gather rows [hit, hit + app) from the
     * pool just loaded, scatter them into a copy of the source pool --- */
    {
        kvl_plan_t *ga = NULL, *sa = NULL;
        expect(kvl_plan(&lay, dst_req, R, KVL_GATHER | KVL_TOKENS_APPEND, &ga), KVL_OK, "kvl_plan (gather, appended tail)");
        expect(kvl_plan(&lay, src_req, R, KVL_SCATTER | KVL_TOKENS_APPEND, &sa), KVL_OK, "kvl_plan (scatter, appended tail)");
        const uint64_t tail_bytes = kvo_payload_bytes(R, app, P, rows);
        uint64_t lib_tail = 0;
        kvl_plan_payload_bytes(ga, &lib_tail);
        expect(lib_tail == tail_bytes, 1, "tail payload bytes equal the oracle's");
        uint8_t *want_tail = malloc(tail_bytes), *got_tail = malloc(tail_bytes);
        uint8_t *h_back_want[P], *h_back[P];
        void *d_back[P], *d_tail = NULL;
        HIP_OK(hipMalloc(&d_tail, tail_bytes));
        for (int p = 0; p < P; ++p) {
            h_back_want[p] = malloc(plane_bytes[p]);
            h_back[p] = malloc(plane_bytes[p]);
            memcpy(h_back_want[p], h_src[p], plane_bytes[p]);
            HIP_OK(hipMalloc(&d_back[p], plane_bytes[p]));
            HIP_OK(hipMemcpy(d_back[p], h_src[p], plane_bytes[p], hipMemcpyHostToDevice));
        }
        if (kvo_pack_range(BS, P, rows, R, hit, app, dst_tabs, (const uint8_t *const *)h_dst_want, want_tail, 0, R) != 0) return 2;
        if (kvo_unpack_range(BS, P, rows, R, hit, app, src_tabs, want_tail, h_back_want, 0, R) != 0) return 2;
        expect(kvl_pack_layer(ga, (const void *const *)d_dst, d_tail, tail_bytes, ks), KVL_OK, "kvl_pack_layer (appended tail)");
        expect(kvl_unpack_layer(sa, d_tail, tail_bytes, d_back, ks), KVL_OK, "kvl_unpack_layer (appended tail)");
        HIP_OK(hipStreamSynchronize(ks));
        HIP_OK(hipMemcpy(got_tail, d_tail, tail_bytes, hipMemcpyDeviceToHost));
        expect(memcmp(got_tail, want_tail, tail_bytes) == 0, 1, "tail transfer buffer equals the oracle's");
        for (int p = 0; p < P; ++p) {
            HIP_OK(hipMemcpy(h_back[p], d_back[p], plane_bytes[p], hipMemcpyDeviceToHost));
            expect(memcmp(h_back[p], h_back_want[p], plane_bytes[p]) == 0, 1, "pool plane after the tail was merged in");
            HIP_OK(hipFree(d_back[p]));
            free(h_back[p]); free(h_back_want[p]);
        }
        HIP_OK(hipFree(d_tail));
        free(want_tail); free(got_tail);
        kvl_plan_destroy(ga);
        kvl_plan_destroy(sa);
    }

    /* --- storage layout (Appendix A.5): layer 1 of 3-layer Full Blocks in pinned host memory -> pool --- */
    {
        enum { LFB = 3 };
        kvl_layout_t lay3 = lay;
        lay3.n_layers = LFB;
        kvl_plan_t *sf = NULL;
        expect(kvl_plan(&lay3, dst_req, R, KVL_SCATTER | KVL_NO_MERGE, &sf), KVL_OK, "kvl_plan (scatter, one descriptor per block)");
        uint64_t fb = 0, nfb = 0;
        expect(kvl_plan_fullblock_geometry(sf, &fb, &nfb), KVL_OK, "kvl_plan_fullblock_geometry");
        expect(fb == kvo_fullblock_bytes(BS, LFB, P, rows) && nfb == kvo_fullblock_count(BS, R, NULL, hit), 1,
               "Full-Block size and count equal the oracle's");
        void *blocks = NULL;
        HIP_OK(hipHostMalloc(&blocks, fb * nfb, hipHostMallocDefault));
        for (uint64_t i = 0; i < fb * nfb; ++i) ((uint8_t *)blocks)[i] = (uint8_t)rnd();
        uint8_t *h_fb_want[P];
        for (int p = 0; p < P; ++p) {
            h_fb_want[p] = malloc(plane_bytes[p]);
            memset(h_fb_want[p], 0xA5, plane_bytes[p]);
            HIP_OK(hipMemset(d_dst[p], 0xA5, plane_bytes[p]));
        }
        if (kvo_fullblocks_to_pool(BS, LFB, P, rows, R, NULL, hit, dst_tabs, 1, blocks, h_fb_want) != 0) return 2;
        expect(kvl_fullblocks_to_pool_layer(sf, blocks, fb * nfb, 1, d_dst, ks), KVL_OK, "kvl_fullblocks_to_pool_layer (pinned buffer)");
        HIP_OK(hipStreamSynchronize(ks));
        for (int p = 0; p < P; ++p) {
            HIP_OK(hipMemcpy(h_dst[p], d_dst[p], plane_bytes[p], hipMemcpyDeviceToHost));
            expect(memcmp(h_dst[p], h_fb_want[p], plane_bytes[p]) == 0, 1, "pool plane after the Full-Block load");
            free(h_fb_want[p]);
        }
        expect(kvl_fullblocks_to_pool_layer(sf, blocks, fb * nfb - 1, 1, d_dst, ks), KVL_ESPACE, "Full-Block buffer stated one byte short");
        expect(kvl_fullblocks_to_pool_layer(sf, blocks, fb * nfb, LFB, d_dst, ks), KVL_EINVAL, "Full-Block load of a layer that does not exist");
        kvl_plan_destroy(sf);
        HIP_OK(hipHostFree(blocks));
    }

    /* --- kvl_stream_layers: 3 layers through 2 host buffers into 2 resident slots, under 50 us of
     * compute each; what every layer's compute saw is kept and compared with the oracle's slot --- */
    {
        enum { LS = 3, S = 2, H = 2 };
        uint8_t *layer_payload[LS];
        for (int l = 0; l < LS; ++l) {
            layer_payload[l] = malloc(payload);
            for (uint64_t i = 0; i < payload; ++i) layer_payload[l][i] = (uint8_t)rnd();
        }
        void *host_slots[H], *slot_planes[S * P], *snap[LS * P];
        uint8_t *h_slot[S][P], *h_seen[LS][P];
        hipStream_t ms;
        HIP_OK(hipStreamCreateWithFlags(&ms, hipStreamNonBlocking));
        for (int h = 0; h < H; ++h) HIP_OK(hipHostMalloc(&host_slots[h], payload, hipHostMallocDefault));
        for (int sl = 0; sl < S; ++sl)
            for (int p = 0; p < P; ++p) HIP_OK(hipMalloc(&slot_planes[sl * P + p], plane_bytes[p]));
        for (int l = 0; l < LS; ++l)
            for (int p = 0; p < P; ++p) {
                HIP_OK(hipMalloc(&snap[l * P + p], plane_bytes[p]));
                h_seen[l][p] = malloc(plane_bytes[p]);
            }
        for (int form = 0; form < 2; ++form) {            /* staged, then zero-copy */
            for (int sl = 0; sl < S; ++sl)
                for (int p = 0; p < P; ++p) {
                    HIP_OK(hipMemset(slot_planes[sl * P + p], 0xA5, plane_bytes[p]));
                    if (form == 0) h_slot[sl][p] = malloc(plane_bytes[p]);
                    memset(h_slot[sl][p], 0xA5, plane_bytes[p]);
                }
            /* the oracle: layer l is unpacked into slot l mod S; that slot is what its compute sees */
            for (int l = 0; l < LS; ++l) {
                if (kvo_unpack(BS, P, rows, R, hit, dst_tabs, layer_payload[l], h_slot[l % S], 0, R) != 0) return 2;
                for (int p = 0; p < P; ++p) memcpy(h_seen[l][p], h_slot[l % S][p], plane_bytes[p]);
            }
            struct fill_ctx ctx = {layer_payload, 0};
            kvl_stream_cfg_t cfg;
            memset(&cfg, 0, sizeof cfg);
            cfg.n_layers = LS;
            cfg.n_host_slots = H;
            cfg.host_layers = host_slots;
            cfg.n_dev_slots = S;
            cfg.dev_slot_planes = slot_planes;
            cfg.dev_staging = form == 0 ? d_stage : NULL;
            cfg.staging_bytes = form == 0 ? stage_bytes : 0;
            cfg.chunk_bytes = form == 0 ? chunk : 0;
            cfg.compute_us = 50;
            cfg.snapshot_planes = snap;
            cfg.host_fill = fill_layer;
            cfg.host_fill_user = &ctx;
            cfg.copy_stream = cs;
            cfg.kernel_stream = ks;
            cfg.compute_stream = ms;
            kvl_stream_stats_t st;
            memset(&st, 0, sizeof st);
            expect(kvl_stream_layers(s, &cfg, &st), KVL_OK,
                   form == 0 ? "kvl_stream_layers (staged, 2 slots)" : "kvl_stream_layers (zero-copy, 2 slots)");
            expect(ctx.calls == LS, 1, "host_fill called once per layer");
            expect(st.total_ms >= LS * 0.05 && st.h2d_bytes == (double)payload * LS, 1, "stream statistics");
            for (int l = 0; l < LS; ++l)
                for (int p = 0; p < P; ++p) {
                    HIP_OK(hipMemcpy(h_dst[p], snap[l * P + p], plane_bytes[p], hipMemcpyDeviceToHost));
                    expect(memcmp(h_dst[p], h_seen[l][p], plane_bytes[p]) == 0, 1, "slot as the layer's compute saw it equals the oracle's");
                }
        }
        for (int l = 0; l < LS; ++l) {
            free(layer_payload[l]);
            for (int p = 0; p < P; ++p) { HIP_OK(hipFree(snap[l * P + p])); free(h_seen[l][p]); }
        }
        for (int sl = 0; sl < S; ++sl)
            for (int p = 0; p < P; ++p) { HIP_OK(hipFree(slot_planes[sl * P + p])); free(h_slot[sl][p]); }
        for (int h = 0; h < H; ++h) HIP_OK(hipHostFree(host_slots[h]));
        HIP_OK(hipStreamDestroy(ms));
    }

    /* --- a plan outlives a stream it was used on: kvl_plan_destroy follows the streams its kernels ran
     * on, and one that no longer exists must not trip it (it then waits for the device instead) --- */
    {
        kvl_plan_t *g2 = NULL;
        hipStream_t gone;
        expect(kvl_plan(&lay, src_req, R, KVL_GATHER, &g2), KVL_OK, "kvl_plan (for a stream that will be destroyed)");
        HIP_OK(hipStreamCreateWithFlags(&gone, hipStreamNonBlocking));
        HIP_OK(hipMemset(d_xfer, 0, payload));
        expect(kvl_pack_layer(g2, (const void *const *)d_src, d_xfer, payload, gone), KVL_OK, "kvl_pack_layer on that stream");
        HIP_OK(hipStreamSynchronize(gone));
        HIP_OK(hipStreamDestroy(gone));
        kvl_plan_destroy(g2);
        (void)hipGetLastError();
        HIP_OK(hipMemcpy(got_xfer, d_xfer, payload, hipMemcpyDeviceToHost));
        expect(memcmp(got_xfer, want_xfer, payload) == 0, 1, "plan destroyed after its stream: result intact, no error left behind");
        kvl_plan_t *g3 = NULL;                       /* and the library still works */
        expect(kvl_plan(&lay, src_req, R, KVL_GATHER, &g3), KVL_OK, "kvl_plan after that");
        expect(kvl_pack_layer(g3, (const void *const *)d_src, d_xfer, payload, ks), KVL_OK, "kvl_pack_layer after that");
        HIP_OK(hipStreamSynchronize(ks));
        kvl_plan_destroy(g3);
    }

    kvl_plan_destroy(g);
    kvl_plan_destroy(s);
    kvl_release_cached_memory();
    HIP_OK(hipStreamDestroy(cs));
    HIP_OK(hipStreamDestroy(ks));
    HIP_OK(hipFree(d_stage));
    HIP_OK(hipFree(short_pool[1]));
    HIP_OK(hipFree(d_xfer));
    HIP_OK(hipFree(d_short));
    HIP_OK(hipHostFree(pinned));
    for (int p = 0; p < P; ++p) {
        HIP_OK(hipFree(d_src[p]));
        HIP_OK(hipFree(d_dst[p]));
        free(h_src[p]); free(h_dst[p]); free(h_dst_want[p]);
    }
    free(want_xfer); free(got_xfer);
    if (failures) {
        printf("c parity: %d check(s) FAILED\n", failures);
        return 1;
    }
    printf("c parity ok\n");
    return 0;
}
