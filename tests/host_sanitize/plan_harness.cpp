// Drives kvl_plan's host logic (KVL_HOST_ONLY: no device is touched) over random
// batches, every token range and the error paths, under AddressSanitizer / UBSan.
// Built and run by tests/test_host_sanitizers.py.
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "kvl.h"
#include "kvl_internal.h"      // launch_groups: how a launch is kept below 2^32 lanes

static uint64_t rng_state = 0x9E3779B97F4A7C15ull;
static uint32_t rnd(uint32_t n) {
    rng_state ^= rng_state << 13; rng_state ^= rng_state >> 7; rng_state ^= rng_state << 17;
    return (uint32_t)((rng_state >> 11) % n);
}

#define REQUIRE(c) do { if (!(c)) { std::printf("plan harness: %s failed at line %d\n", #c, __LINE__); return 1; } } while (0)

int main() {
    const uint32_t row_choices[] = {5, 16, 48, 656, 1152};
    for (int it = 0; it < 300; ++it) {
        kvl_layout_t lay{};
        lay.n_layers = 1 + rnd(4);
        lay.block_tokens = 1 + rnd(64);
        lay.n_planes = 1 + rnd(KVL_MAX_PLANES);
        for (uint32_t p = 0; p < lay.n_planes; ++p) lay.row_bytes[p] = row_choices[rnd(5)];
        const uint32_t n_req = rnd(8);
        std::vector<kvl_request_t> req(n_req);
        std::vector<std::vector<int32_t>> tabs(n_req);
        uint64_t blocks = 0;
        for (uint32_t r = 0; r < n_req; ++r) {
            req[r].hit_tokens = rnd(6 * lay.block_tokens + 1);
            req[r].append_tokens = rnd(2 * lay.block_tokens + 1);
            req[r].n_blocks = (req[r].hit_tokens + req[r].append_tokens + lay.block_tokens - 1) / lay.block_tokens + rnd(2);
            blocks += req[r].n_blocks;
        }
        lay.pool_blocks = blocks + 1 + rnd(8);
        // tables: runs of consecutive ids (so that merging happens), disjoint across requests
        uint64_t next = 0;
        for (uint32_t r = 0; r < n_req; ++r) {
            tabs[r].resize(req[r].n_blocks);
            for (uint32_t b = 0; b < req[r].n_blocks; ++b) tabs[r][b] = (int32_t)next++;
            if (req[r].n_blocks > 2 && rnd(2)) std::swap(tabs[r][0], tabs[r][req[r].n_blocks - 1]);
            req[r].block_table = tabs[r].empty() ? nullptr : tabs[r].data();
        }
        const uint32_t ranges[] = {0u, KVL_TOKENS_APPEND, KVL_TOKENS_ALL};
        for (uint32_t range : ranges) {
            for (uint32_t extra : {0u, (uint32_t)KVL_NO_MERGE}) {
                kvl_tuning_t t{};
                t.unit_bytes = rnd(2) ? 0 : 64 + rnd(5000);
                kvl_plan_t *p = nullptr;
                int rc = kvl_plan_tuned(&lay, req.data(), n_req, KVL_GATHER | KVL_SCATTER | KVL_HOST_ONLY | range | extra, &t, &p);
                REQUIRE(rc == KVL_OK && p);
                uint64_t n = 0, T = 0, bytes = 0, fb = 0, nfb = 0;
                REQUIRE(kvl_plan_n_units(p, &n) == KVL_OK && kvl_plan_hit_tokens(p, &T) == KVL_OK);
                REQUIRE(kvl_plan_payload_bytes(p, &bytes) == KVL_OK && kvl_plan_fullblock_geometry(p, &fb, &nfb) == KVL_OK);
                std::vector<kvl_unit_t> u(n);
                REQUIRE(kvl_plan_get_units(p, u.data(), n, &n) == KVL_OK);
                uint64_t row = 0, sum = 0;
                for (const kvl_unit_t &d : u) {                 // descriptors tile the buffer, stay in the pool
                    REQUIRE(d.xfer_row == row && d.n_rows > 0);
                    REQUIRE((uint64_t)d.pool_row + d.n_rows <= lay.pool_blocks * lay.block_tokens);
                    REQUIRE(d.block_index < nfb);
                    if (extra) REQUIRE(d.pool_row % lay.block_tokens + d.n_rows <= lay.block_tokens);
                    row += d.n_rows;
                }
                REQUIRE(row == T);
                for (uint32_t q = 0; q < lay.n_planes; ++q) sum += T * lay.row_bytes[q];
                REQUIRE(sum == bytes);
                uint64_t nc = 0;
                const uint64_t chunk = 1 << 20;
                REQUIRE(kvl_plan_get_chunks(p, chunk, nullptr, 0, &nc) == KVL_OK);
                std::vector<kvl_chunk_t> ch(nc);
                REQUIRE(kvl_plan_get_chunks(p, chunk, ch.data(), nc, &nc) == KVL_OK);
                uint64_t covered = 0;
                for (const kvl_chunk_t &c : ch) { REQUIRE(c.host_offset == covered && c.bytes <= chunk); covered += c.bytes; }
                REQUIRE(covered == bytes);
                kvl_plan_destroy(p);
            }
        }
        // error paths leave nothing behind
        if (n_req) {
            kvl_plan_t *p = nullptr;
            std::vector<int32_t> bad = tabs[0];
            if (!bad.empty() && req[0].hit_tokens + req[0].append_tokens > 0) {
                bad[0] = (int32_t)lay.pool_blocks;
                kvl_request_t save = req[0];
                req[0].block_table = bad.data();
                REQUIRE(kvl_plan(&lay, req.data(), n_req, KVL_GATHER | KVL_HOST_ONLY, &p) == KVL_ERANGE && !p);
                req[0] = save;
                req[0].n_blocks = 0;
                REQUIRE(kvl_plan(&lay, req.data(), n_req, KVL_GATHER | KVL_HOST_ONLY, &p) == KVL_ERANGE && !p);
                req[0] = save;
            }
            if (n_req >= 2 && req[0].hit_tokens && req[1].hit_tokens) {
                std::vector<int32_t> dup = tabs[1];
                dup[0] = tabs[0][0];
                kvl_request_t save = req[1];
                req[1].block_table = dup.data();
                REQUIRE(kvl_plan(&lay, req.data(), n_req, KVL_SCATTER | KVL_HOST_ONLY, &p) == KVL_EALIAS && !p);
                REQUIRE(kvl_plan(&lay, req.data(), n_req, KVL_GATHER | KVL_HOST_ONLY, &p) == KVL_OK && p);
                kvl_plan_destroy(p);
                req[1] = save;
            }
        }
    }
    // launch geometry: one workgroup per tile while that fits, else (or on request) a capped grid that walks
    {
        bool walk = true;
        REQUIRE(kvl::launch_groups(1000, 256, 0, &walk) == 1000 && !walk);
        REQUIRE(kvl::launch_groups(1000, 256, 64, &walk) == 64 && walk);
        REQUIRE(kvl::launch_groups(64, 256, 64, &walk) == 64 && !walk);
        REQUIRE(kvl::launch_groups(10, 256, UINT32_MAX, &walk) == 10 && !walk);
        const uint64_t most256 = ((1ull << 32) - 1) / 256, most1024 = ((1ull << 32) - 1) / 1024;
        REQUIRE(kvl::launch_groups(most256, 256, 0, &walk) == most256 && !walk);            // 2^32 - 256 lanes: fits
        REQUIRE(kvl::launch_groups(most256 + 1, 256, 0, &walk) == most256 && walk);         // 2^32 lanes: must walk
        REQUIRE(kvl::launch_groups(1ull << 31, 1024, UINT32_MAX, &walk) == most1024 && walk);
        for (uint32_t threads : {64u, 128u, 256u, 512u, 1024u})
            for (uint64_t work : {1ull, 4194303ull, 16777216ull, 1ull << 26, (1ull << 31) - 1}) {
                const uint32_t g = kvl::launch_groups(work, threads, 0, &walk);
                REQUIRE((uint64_t)g * threads < (1ull << 32) && g >= 1 && (walk || g == work));
            }
    }
    std::printf("plan harness ok\n");
    return 0;
}
