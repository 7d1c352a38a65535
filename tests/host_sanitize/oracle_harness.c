/* Drives the C oracle over random small batches with every buffer allocated at
 * its exact size, so that AddressSanitizer / UBSan see any stray access.
 * Built and run by tests/test_host_sanitizers.py (host only, no GPU). */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

uint64_t kvo_payload_bytes(uint32_t, const uint32_t *, uint32_t, const uint32_t *);
int kvo_check(uint32_t, uint64_t, uint32_t, const uint32_t *, const uint32_t *, const uint32_t *,
              const int32_t *const *, int);
int kvo_pack(uint32_t, uint32_t, const uint32_t *, uint32_t, const uint32_t *, const int32_t *const *,
             const uint8_t *const *, uint8_t *, uint32_t, uint32_t);
int kvo_unpack(uint32_t, uint32_t, const uint32_t *, uint32_t, const uint32_t *, const int32_t *const *,
               const uint8_t *, uint8_t *const *, uint32_t, uint32_t);
int kvo_pack_range(uint32_t, uint32_t, const uint32_t *, uint32_t, const uint32_t *, const uint32_t *,
                   const int32_t *const *, const uint8_t *const *, uint8_t *, uint32_t, uint32_t);
int kvo_unpack_range(uint32_t, uint32_t, const uint32_t *, uint32_t, const uint32_t *, const uint32_t *,
                     const int32_t *const *, const uint8_t *, uint8_t *const *, uint32_t, uint32_t);
uint64_t kvo_fullblock_bytes(uint32_t, uint32_t, uint32_t, const uint32_t *);
uint64_t kvo_fullblock_count(uint32_t, uint32_t, const uint32_t *, const uint32_t *);
int kvo_fullblocks_to_pool(uint32_t, uint32_t, uint32_t, const uint32_t *, uint32_t, const uint32_t *,
                           const uint32_t *, const int32_t *const *, uint32_t, const uint8_t *, uint8_t *const *);
int kvo_pool_to_fullblocks(uint32_t, uint32_t, uint32_t, const uint32_t *, uint32_t, const uint32_t *,
                           const uint32_t *, const int32_t *const *, uint32_t, const uint8_t *const *, uint8_t *);

static uint64_t rng_state = 88172645463325252ull;
static uint32_t rnd(uint32_t n) {
    rng_state ^= rng_state << 13; rng_state ^= rng_state >> 7; rng_state ^= rng_state << 17;
    return (uint32_t)((rng_state >> 11) % n);
}

int main(void) {
    const uint32_t row_choices[] = {5, 16, 48, 656};
    for (int it = 0; it < 200; ++it) {
        uint32_t bs = 1 + rnd(17), n_planes = 1 + rnd(3), n_req = rnd(6), L = 1 + rnd(3);
        uint32_t rows[3];
        for (uint32_t p = 0; p < n_planes; ++p) rows[p] = row_choices[rnd(4)];
        uint32_t *hit = malloc(sizeof(uint32_t) * (n_req ? n_req : 1));
        uint32_t *app = malloc(sizeof(uint32_t) * (n_req ? n_req : 1));
        uint32_t *len = malloc(sizeof(uint32_t) * (n_req ? n_req : 1));
        uint32_t *all = malloc(sizeof(uint32_t) * (n_req ? n_req : 1));
        int32_t **tabs = malloc(sizeof(int32_t *) * (n_req ? n_req : 1));
        uint64_t blocks = 0;
        for (uint32_t r = 0; r < n_req; ++r) {
            hit[r] = rnd(5 * bs + 1); app[r] = rnd(2 * bs + 1); all[r] = hit[r] + app[r];
            len[r] = (hit[r] + app[r] + bs - 1) / bs;
            blocks += len[r];
        }
        uint64_t pool_blocks = blocks + 1 + rnd(4);
        /* disjoint tables: a shuffled identity */
        int32_t *perm = malloc(sizeof(int32_t) * pool_blocks);
        for (uint64_t i = 0; i < pool_blocks; ++i) perm[i] = (int32_t)i;
        for (uint64_t i = pool_blocks - 1; i > 0; --i) { uint64_t j = rnd((uint32_t)i + 1); int32_t t = perm[i]; perm[i] = perm[j]; perm[j] = t; }
        uint64_t pos = 0;
        for (uint32_t r = 0; r < n_req; ++r) {
            tabs[r] = malloc(sizeof(int32_t) * (len[r] ? len[r] : 1));
            for (uint32_t b = 0; b < len[r]; ++b) tabs[r][b] = perm[pos++];
        }
        if (kvo_check(bs, pool_blocks, n_req, hit, app, len, (const int32_t *const *)tabs, 1) != 0) { printf("check failed\n"); return 1; }
        uint8_t *pool[3], *dst[3];
        for (uint32_t p = 0; p < n_planes; ++p) {
            size_t n = (size_t)pool_blocks * bs * rows[p];
            pool[p] = malloc(n); dst[p] = malloc(n);
            for (size_t i = 0; i < n; ++i) pool[p][i] = (uint8_t)rnd(256);
            memset(dst[p], 0xA5, n);
        }
        /* prefix */
        uint64_t nb = kvo_payload_bytes(n_req, hit, n_planes, rows);
        uint8_t *x = malloc(nb ? nb : 1);
        if (kvo_pack(bs, n_planes, rows, n_req, hit, (const int32_t *const *)tabs, (const uint8_t *const *)pool, x, 0, n_req)) return 2;
        if (kvo_unpack(bs, n_planes, rows, n_req, hit, (const int32_t *const *)tabs, x, dst, 0, n_req)) return 3;
        free(x);
        /* tail and whole prompt */
        nb = kvo_payload_bytes(n_req, app, n_planes, rows);
        x = malloc(nb ? nb : 1);
        if (kvo_pack_range(bs, n_planes, rows, n_req, hit, app, (const int32_t *const *)tabs, (const uint8_t *const *)pool, x, 0, n_req)) return 4;
        if (kvo_unpack_range(bs, n_planes, rows, n_req, hit, app, (const int32_t *const *)tabs, x, dst, 0, n_req)) return 5;
        free(x);
        /* after prefix + tail the destination equals the source on every row of the prompt */
        nb = kvo_payload_bytes(n_req, all, n_planes, rows);
        x = malloc(nb ? nb : 1);
        uint8_t *y = malloc(nb ? nb : 1);
        kvo_pack_range(bs, n_planes, rows, n_req, NULL, all, (const int32_t *const *)tabs, (const uint8_t *const *)pool, x, 0, n_req);
        kvo_pack_range(bs, n_planes, rows, n_req, NULL, all, (const int32_t *const *)tabs, (const uint8_t *const *)dst, y, 0, n_req);
        if (nb && memcmp(x, y, nb)) { printf("merge identity failed\n"); return 6; }
        free(x); free(y);
        /* storage layout, every layer, then back */
        uint64_t fb = kvo_fullblock_bytes(bs, L, n_planes, rows), nfb = kvo_fullblock_count(bs, n_req, NULL, all);
        uint8_t *buf = malloc(fb * nfb ? fb * nfb : 1);
        for (uint32_t l = 0; l < L; ++l)
            if (kvo_pool_to_fullblocks(bs, L, n_planes, rows, n_req, NULL, all, (const int32_t *const *)tabs, l, (const uint8_t *const *)pool, buf)) return 7;
        for (uint32_t l = 0; l < L; ++l)
            if (kvo_fullblocks_to_pool(bs, L, n_planes, rows, n_req, NULL, all, (const int32_t *const *)tabs, l, buf, dst)) return 8;
        free(buf);
        for (uint32_t p = 0; p < n_planes; ++p) { free(pool[p]); free(dst[p]); }
        for (uint32_t r = 0; r < n_req; ++r) free(tabs[r]);
        free(tabs); free(perm); free(hit); free(app); free(len); free(all);
    }
    printf("oracle harness ok\n");
    return 0;
}
