/*
 * CPU oracle for the layer-wise KV-cache load path.  TEST INFRASTRUCTURE ONLY:
 * it exists so that tests, the smoke check and the benchmark's CPU-baseline leg
 * can say what the right bytes are.  The product library never calls it and
 * shares no code, header or table with it.
 *
 * What it computes is a definition, not an algorithm: the hit tokens' cache
 * rows of one layer are copied between a paged pool and a dense transfer
 * buffer.  The layout follows the paper's Appendix A.5: a Layer Block is a byte
 * tensor [1, tokens, bytes] holding one layer's cache for block_size tokens,
 * and a request's cached prefix ("hit" tokens, Section 4.1: only the hit
 * tokens' cache is loaded, the appended tokens' cache is computed) occupies
 * the first hit_r token rows of the blocks its block table names, in order.
 *
 *   pool_p   : plane p of the paged pool, bytes [pool_blocks][bs][row_p]
 *   tbl_r    : block table of request r (physical block ids)
 *   xfer     : transfer buffer, plane-major; inside a plane request-major,
 *              token-major, dense:
 *                 base_p  = sum_{q<p} T * row_q,  T = sum_r hit_r
 *                 off_r,p = base_p + sum_{s<r} hit_s * row_p
 *
 *   pack  : xfer[off_r,p + t*row_p + j] = pool_p[(tbl_r[t/bs]*bs + t%bs)*row_p + j]
 *   unpack: pool_p[(tbl_r[t/bs]*bs + t%bs)*row_p + j] = xfer[off_r,p + t*row_p + j]
 *           for r in requests, t in [0, hit_r), j in [0, row_p); every other
 *           byte of the pool keeps its value.
 *
 * Everything is single-threaded scalar loops with 64-bit offsets.  The
 * [r_begin, r_end) arguments restrict the loops to a range of requests (the
 * offsets are still those of the whole batch) so that a caller can time it
 * over several host threads without changing the arithmetic.
 *
 * Pins (tests/test_oracle_pins.py): round trip into a sentinel pool, byte
 * conservation, an independent per-byte brute force in Python on tiny pools
 * (exhaustive over permutations of up to 5 blocks), memcpy and numpy.take
 * special cases, permutation algebra across two tables, and a closed-form
 * self-describing fill; for token ranges (below) an independent brute force,
 * the reduction to the prefix case, and the merge identity "hit rows scattered,
 * then tail rows scattered = whole prompt scattered"; for the Full-Block storage
 * layout (bottom of this file) NumPy reshapes of its defining sentence, a
 * per-byte brute force and agreement with the Layer-Block path.  A last test plants
 * mistakes in copies of this file and demands that the pins notice each.  The
 * paper prints no worked example for this path.
 */
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define KVO_OK            0
#define KVO_E_ARG        -1   /* null pointer, zero block size, zero row */
#define KVO_E_TABLE      -2   /* table shorter than ceil((hit+app)/bs) */
#define KVO_E_BLOCK      -3   /* block id outside [0, pool_blocks) */
#define KVO_E_DUP        -4   /* block named twice in a scatter destination */

/* Total hit tokens of the batch. */
uint64_t kvo_total_hit_tokens(uint32_t n_req, const uint32_t *hit)
{
    uint64_t T = 0;
    for (uint32_t r = 0; r < n_req; ++r) T += hit[r];
    return T;
}

/* Bytes one layer's transfer buffer holds: sum over planes of T * row_p. */
uint64_t kvo_payload_bytes(uint32_t n_req, const uint32_t *hit,
                           uint32_t n_planes, const uint32_t *row_bytes)
{
    uint64_t T = kvo_total_hit_tokens(n_req, hit);
    uint64_t bytes = 0;
    for (uint32_t p = 0; p < n_planes; ++p) bytes += T * (uint64_t)row_bytes[p];
    return bytes;
}

/* Preconditions of the definition.  scatter != 0 also demands that no block
 * that receives hit rows is named twice, because then two sources would claim
 * the same destination bytes. */
int kvo_check(uint32_t bs, uint64_t pool_blocks, uint32_t n_req,
              const uint32_t *hit, const uint32_t *app,
              const uint32_t *table_len, const int32_t *const *tables,
              int scatter)
{
    if (!hit || !app || !table_len || !tables || bs == 0) return KVO_E_ARG;
    uint8_t *seen = NULL;
    if (scatter) {
        seen = (uint8_t *)calloc(pool_blocks ? pool_blocks : 1, 1);
        if (!seen) return KVO_E_ARG;
    }
    int rc = KVO_OK;
    for (uint32_t r = 0; r < n_req && rc == KVO_OK; ++r) {
        uint64_t tokens = (uint64_t)hit[r] + app[r];
        uint64_t need = (tokens + bs - 1) / bs;
        if (table_len[r] < need) { rc = KVO_E_TABLE; break; }
        if (need && !tables[r]) { rc = KVO_E_ARG; break; }
        uint64_t hit_blocks = ((uint64_t)hit[r] + bs - 1) / bs;
        for (uint64_t b = 0; b < need; ++b) {
            int64_t id = tables[r][b];
            if (id < 0 || (uint64_t)id >= pool_blocks) { rc = KVO_E_BLOCK; break; }
            if (scatter && b < hit_blocks) {
                if (seen[id]) { rc = KVO_E_DUP; break; }
                seen[id] = 1;
            }
        }
    }
    free(seen);
    return rc;
}

/*
 * Token ranges.  The prefix case above is first_r = 0, count_r = hit_r.  The
 * tail a prefill engine computes (the "miss" tokens of Section 4.1, sent on
 * after a layer's computation and merged with the hit tokens' cache on the
 * decode side) is first_r = hit_r, count_r = append_r; the whole prompt is
 * first_r = 0, count_r = hit_r + append_r.  The transfer buffer is laid out as
 * before with count_r in the place of hit_r, and token k of the range is token
 * t = first_r + k of the request:
 *
 *   pack  : xfer[off_r,p + k*row_p + j] = pool_p[(tbl_r[t/bs]*bs + t%bs)*row_p + j]
 *   unpack: the same assignment read right to left.
 *
 * first == NULL means all zeros.
 */
static uint64_t sum_u32(uint32_t n, const uint32_t *v)
{
    uint64_t s = 0;
    for (uint32_t i = 0; i < n; ++i) s += v[i];
    return s;
}

int kvo_pack_range(uint32_t bs, uint32_t n_planes, const uint32_t *row_bytes,
                   uint32_t n_req, const uint32_t *first, const uint32_t *count,
                   const int32_t *const *tables,
                   const uint8_t *const *pool_planes, uint8_t *xfer,
                   uint32_t r_begin, uint32_t r_end)
{
    if (!row_bytes || !count || !tables || !pool_planes || !xfer || bs == 0) return KVO_E_ARG;
    uint64_t T = sum_u32(n_req, count);
    uint64_t base = 0;
    for (uint32_t p = 0; p < n_planes; ++p) {
        uint64_t row = row_bytes[p];
        const uint8_t *pool = pool_planes[p];
        uint64_t off = base;
        for (uint32_t r = 0; r < n_req; ++r) {
            if (r >= r_begin && r < r_end) {
                for (uint64_t k = 0; k < count[r]; ++k) {
                    uint64_t t = (first ? first[r] : 0) + k;
                    uint64_t phys_row = (uint64_t)tables[r][t / bs] * bs + t % bs;
                    for (uint64_t j = 0; j < row; ++j)
                        xfer[off + k * row + j] = pool[phys_row * row + j];
                }
            }
            off += (uint64_t)count[r] * row;
        }
        base += T * row;
    }
    return KVO_OK;
}

int kvo_unpack_range(uint32_t bs, uint32_t n_planes, const uint32_t *row_bytes,
                     uint32_t n_req, const uint32_t *first, const uint32_t *count,
                     const int32_t *const *tables,
                     const uint8_t *xfer, uint8_t *const *pool_planes,
                     uint32_t r_begin, uint32_t r_end)
{
    if (!row_bytes || !count || !tables || !pool_planes || !xfer || bs == 0) return KVO_E_ARG;
    uint64_t T = sum_u32(n_req, count);
    uint64_t base = 0;
    for (uint32_t p = 0; p < n_planes; ++p) {
        uint64_t row = row_bytes[p];
        uint8_t *pool = pool_planes[p];
        uint64_t off = base;
        for (uint32_t r = 0; r < n_req; ++r) {
            if (r >= r_begin && r < r_end) {
                for (uint64_t k = 0; k < count[r]; ++k) {
                    uint64_t t = (first ? first[r] : 0) + k;
                    uint64_t phys_row = (uint64_t)tables[r][t / bs] * bs + t % bs;
                    for (uint64_t j = 0; j < row; ++j)
                        pool[phys_row * row + j] = xfer[off + k * row + j];
                }
            }
            off += (uint64_t)count[r] * row;
        }
        base += T * row;
    }
    return KVO_OK;
}

/* Destination blocks of a scatter over token ranges must be distinct
 * (0 or KVO_E_DUP); table length and block ids are checked by kvo_check. */
int kvo_check_range_scatter(uint32_t bs, uint64_t pool_blocks, uint32_t n_req,
                            const uint32_t *first, const uint32_t *count,
                            const int32_t *const *tables)
{
    if (!count || !tables || bs == 0) return KVO_E_ARG;
    uint8_t *seen = (uint8_t *)calloc(pool_blocks ? pool_blocks : 1, 1);
    if (!seen) return KVO_E_ARG;
    int rc = KVO_OK;
    for (uint32_t r = 0; r < n_req && rc == KVO_OK; ++r) {
        if (count[r] == 0) continue;
        uint64_t t0 = first ? first[r] : 0, t1 = t0 + count[r];
        for (uint64_t b = t0 / bs; b <= (t1 - 1) / bs; ++b) {
            int64_t id = tables[r][b];
            if (id < 0 || (uint64_t)id >= pool_blocks) { rc = KVO_E_BLOCK; break; }
            if (seen[id]) { rc = KVO_E_DUP; break; }
            seen[id] = 1;
        }
    }
    free(seen);
    return rc;
}

/* pack: paged pool -> dense transfer buffer, requests [r_begin, r_end). */
int kvo_pack(uint32_t bs, uint32_t n_planes, const uint32_t *row_bytes,
             uint32_t n_req, const uint32_t *hit, const int32_t *const *tables,
             const uint8_t *const *pool_planes, uint8_t *xfer,
             uint32_t r_begin, uint32_t r_end)
{
    if (!row_bytes || !hit || !tables || !pool_planes || !xfer || bs == 0) return KVO_E_ARG;
    uint64_t T = kvo_total_hit_tokens(n_req, hit);
    uint64_t base = 0;
    for (uint32_t p = 0; p < n_planes; ++p) {
        uint64_t row = row_bytes[p];
        const uint8_t *pool = pool_planes[p];
        uint64_t off = base;
        for (uint32_t r = 0; r < n_req; ++r) {
            if (r >= r_begin && r < r_end) {
                for (uint64_t t = 0; t < hit[r]; ++t) {
                    uint64_t phys_row = (uint64_t)tables[r][t / bs] * bs + t % bs;
                    for (uint64_t j = 0; j < row; ++j)
                        xfer[off + t * row + j] = pool[phys_row * row + j];
                }
            }
            off += (uint64_t)hit[r] * row;
        }
        base += T * row;
    }
    return KVO_OK;
}

/* unpack: dense transfer buffer -> paged pool, requests [r_begin, r_end). */
int kvo_unpack(uint32_t bs, uint32_t n_planes, const uint32_t *row_bytes,
               uint32_t n_req, const uint32_t *hit, const int32_t *const *tables,
               const uint8_t *xfer, uint8_t *const *pool_planes,
               uint32_t r_begin, uint32_t r_end)
{
    if (!row_bytes || !hit || !tables || !pool_planes || !xfer || bs == 0) return KVO_E_ARG;
    uint64_t T = kvo_total_hit_tokens(n_req, hit);
    uint64_t base = 0;
    for (uint32_t p = 0; p < n_planes; ++p) {
        uint64_t row = row_bytes[p];
        uint8_t *pool = pool_planes[p];
        uint64_t off = base;
        for (uint32_t r = 0; r < n_req; ++r) {
            if (r >= r_begin && r < r_end) {
                for (uint64_t t = 0; t < hit[r]; ++t) {
                    uint64_t phys_row = (uint64_t)tables[r][t / bs] * bs + t % bs;
                    for (uint64_t j = 0; j < row; ++j)
                        pool[phys_row * row + j] = xfer[off + t * row + j];
                }
            }
            off += (uint64_t)hit[r] * row;
        }
        base += T * row;
    }
    return KVO_OK;
}

/*
 * Storage layout.  Appendix A.5: a Full Block is a byte tensor
 * [layer, tokens, bytes], the concatenation of one block's Layer Blocks, and all
 * traffic with storage uses Full Blocks while the per-layer loads use Layer
 * Blocks (Section 4.1, "Different Block Layouts").  With several planes a Layer
 * Block is its planes' spans one after the other, so
 *
 *   LB = bs * sum_p row_p               bytes of one Layer Block
 *   FB = n_layers * LB                  bytes of one Full Block
 *   byte (l, p, w, j) of a Full Block   at  l*LB + bs*sum_{q<p} row_q + w*row_p + j
 *
 * The buffer holds the Full Blocks that the token ranges touch, request after
 * request, each request's blocks in table order: request r contributes blocks
 * first_r/bs .. (first_r+count_r-1)/bs (none if count_r = 0).  Loading layer l
 * from it into a paged pool moves, for every token t = first_r + k of a range,
 * its row from Full Block f = F_r + (t/bs - first_r/bs), row w = t % bs; storing
 * is the same assignment the other way.  Bytes of the buffer outside the ranges'
 * rows of layer l are not touched.
 */
uint64_t kvo_fullblock_bytes(uint32_t bs, uint32_t n_layers, uint32_t n_planes,
                             const uint32_t *row_bytes)
{
    uint64_t lb = 0;
    for (uint32_t p = 0; p < n_planes; ++p) lb += (uint64_t)bs * row_bytes[p];
    return lb * n_layers;
}

uint64_t kvo_fullblock_count(uint32_t bs, uint32_t n_req, const uint32_t *first,
                             const uint32_t *count)
{
    uint64_t n = 0;
    for (uint32_t r = 0; r < n_req; ++r) {
        if (count[r] == 0) continue;
        uint64_t t0 = first ? first[r] : 0, t1 = t0 + count[r];
        n += (t1 - 1) / bs - t0 / bs + 1;
    }
    return n;
}

static int fullblocks_move(int to_pool, uint32_t bs, uint32_t n_layers, uint32_t n_planes,
                           const uint32_t *row_bytes, uint32_t n_req,
                           const uint32_t *first, const uint32_t *count,
                           const int32_t *const *tables, uint32_t layer,
                           uint8_t *blocks, uint8_t *const *pool_planes)
{
    if (!row_bytes || !count || !tables || !blocks || !pool_planes || bs == 0) return KVO_E_ARG;
    if (layer >= n_layers) return KVO_E_ARG;
    uint64_t lb = 0;
    for (uint32_t p = 0; p < n_planes; ++p) lb += (uint64_t)bs * row_bytes[p];
    uint64_t fb = lb * n_layers;
    uint64_t plane_off = 0;
    for (uint32_t p = 0; p < n_planes; ++p) {
        uint64_t row = row_bytes[p];
        uint8_t *pool = pool_planes[p];
        uint64_t f_base = 0;                     /* Full Blocks of the requests before r */
        for (uint32_t r = 0; r < n_req; ++r) {
            if (count[r] == 0) continue;
            uint64_t t0 = first ? first[r] : 0;
            for (uint64_t k = 0; k < count[r]; ++k) {
                uint64_t t = t0 + k;
                uint64_t f = f_base + (t / bs - t0 / bs);
                uint64_t w = t % bs;
                uint64_t in_blocks = f * fb + (uint64_t)layer * lb + plane_off + w * row;
                uint64_t in_pool = ((uint64_t)tables[r][t / bs] * bs + w) * row;
                for (uint64_t j = 0; j < row; ++j) {
                    if (to_pool) pool[in_pool + j] = blocks[in_blocks + j];
                    else blocks[in_blocks + j] = pool[in_pool + j];
                }
            }
            f_base += (t0 + count[r] - 1) / bs - t0 / bs + 1;
        }
        plane_off += (uint64_t)bs * row;
    }
    return KVO_OK;
}

int kvo_fullblocks_to_pool(uint32_t bs, uint32_t n_layers, uint32_t n_planes,
                           const uint32_t *row_bytes, uint32_t n_req,
                           const uint32_t *first, const uint32_t *count,
                           const int32_t *const *tables, uint32_t layer,
                           const uint8_t *blocks, uint8_t *const *pool_planes)
{
    return fullblocks_move(1, bs, n_layers, n_planes, row_bytes, n_req, first, count, tables,
                           layer, (uint8_t *)blocks, pool_planes);
}

int kvo_pool_to_fullblocks(uint32_t bs, uint32_t n_layers, uint32_t n_planes,
                           const uint32_t *row_bytes, uint32_t n_req,
                           const uint32_t *first, const uint32_t *count,
                           const int32_t *const *tables, uint32_t layer,
                           const uint8_t *const *pool_planes, uint8_t *blocks)
{
    return fullblocks_move(0, bs, n_layers, n_planes, row_bytes, n_req, first, count, tables,
                           layer, blocks, (uint8_t *const *)pool_planes);
}
