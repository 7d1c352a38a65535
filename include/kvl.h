/*
 * kvl -- layer-wise KV-cache load for one MI355X (gfx950), C ABI.
 *
 * The paper's dual-path loading (Section 4.1) brings the cache of a request's
 * hit tokens -- the prefix of its context that is already cached -- into the
 * prefill engine's HBM one layer at a time, either from the prefill engine's
 * own host buffer or from a decode engine's buffer, while the layers before it
 * are being computed.  The unit of that traffic is the Layer Block of
 * Appendix A.5: a byte tensor [1, tokens, bytes] with one layer's cache of
 * block_size tokens.  This library is the GPU side of that load:
 *
 *   kvl_plan              host: turn block tables into copy descriptors (once
 *                         per batch; the same tables serve every layer, since a
 *                         Full Block is the concatenation of one block's Layer
 *                         Blocks, Appendix A.5)
 *   kvl_pack_layer        decode side: gather hit rows of one layer from a
 *                         paged pool into a dense transfer buffer
 *   kvl_unpack_layer      prefill side: scatter a transfer buffer into a paged
 *                         pool
 *   kvl_h2d_unpack_layer  the same with the transfer buffer in pinned host
 *                         memory (the prefill engine's host buffer)
 *   kvl_stream_layers     all layers: load of layer l+1 under compute of layer l
 *
 * Transfer-buffer layout (one layer), with T = sum of hit tokens of the batch
 * (for a plan over another token range, KVL_TOKENS_*: read "tokens of the range"
 * for "hit tokens" throughout):
 *   plane p starts at byte  sum_{q<p} T * row_bytes[q];
 *   inside plane p request r starts at  sum_{s<r} hit_s * row_bytes[p];
 *   token t of request r follows at t * row_bytes[p].  Dense, no padding.
 * Pool layout (one layer, one plane): bytes [pool_blocks][block_tokens][row_bytes[p]];
 *   token t of request r lives in block table[t / block_tokens], row
 *   t % block_tokens.  Only tokens t < hit_tokens are ever moved; the appended
 *   tokens' rows are never read or written.
 *
 * A gather plan and a scatter plan built from the same hit_tokens list give
 * the same transfer-buffer layout; that is what lets the buffer cross from one
 * engine to the other.
 *
 * Conventions.  Every function returns 0 (KVL_OK) or a negative KVL_E* code
 * and never throws.  "device" pointers are HIP device memory of the device
 * that was current when the plan was made; "host" pointers are ordinary host
 * memory unless "pinned" is said.  The caller owns every pool, buffer and
 * stream; the library owns only the plan (with its small device descriptor
 * array and a few events).  Stream arguments are hipStream_t passed as void*;
 * NULL means the default stream.  pack/unpack/h2d_unpack only enqueue work and
 * return; results are ready when the stream reaches that point.
 * A plan may be used by one thread at a time, and only while the device it was
 * made on is the current one (KVL_EINVAL otherwise).
 */
#ifndef KVL_H
#define KVL_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define KVL_MAX_PLANES 4

/* error codes */
#define KVL_OK       0
#define KVL_EINVAL  -1   /* null pointer, zero size, bad flag, plan of the wrong kind */
#define KVL_ERANGE  -2   /* block id outside the pool, table too short, size beyond 32-bit row index */
#define KVL_EALIAS  -3   /* scatter plan names one destination block twice */
#define KVL_ESPACE  -4   /* buffer, staging area or chunk too small */
#define KVL_EHIP    -5   /* a HIP call failed: see kvl_last_hip_error */
#define KVL_ENOMEM  -6   /* host allocation failed */
#define KVL_ENOSYS  -7   /* the HIP runtime in this process lacks a call the function is built on */

/* plan flags */
#define KVL_GATHER     1u  /* plan may be used with kvl_pack_layer */
#define KVL_SCATTER    2u  /* plan may be used with unpack / h2d_unpack / stream_layers;
                              destination blocks must be distinct */
#define KVL_HOST_ONLY  4u  /* make descriptors on the host only (no device is touched);
                              such a plan can be inspected but not executed */
#define KVL_NO_MERGE   8u  /* do not merge physically adjacent blocks into one run */
#define KVL_NO_POINTER_CHECKS 64u  /* skip kvl_check_buffer on every call made with this plan */
#define KVL_CALLER_SYNCS 128u      /* the caller promises that everything enqueued with the plan has finished
                                      by the time it destroys the plan: launches are then not followed by an
                                      event each (about 3 us per launch, which only shows on layers of a few
                                      MB), and kvl_plan_destroy hands the descriptor array on at once */
/* Which token rows of each request the plan moves.  Default: the hit prefix
 * [0, hit).  The other two serve the step after a layer's computation
 * (Section 4.1): the decode-engine read path sends on only the miss tokens'
 * cache, which is merged with the hit tokens' cache already there; the
 * prefill-engine read path sends on hit and miss tokens together. */
#define KVL_TOKENS_APPEND 16u  /* the appended tail [hit, hit + append) */
#define KVL_TOKENS_ALL    32u  /* the whole prompt [0, hit + append) */

typedef struct kvl_plan_s kvl_plan_t;   /* opaque, library-owned */

/* Geometry of one layer of a paged cache (Appendix A.5). */
typedef struct {
    uint32_t n_layers;                   /* layers of the model; used by kvl_stream_layers */
    uint32_t block_tokens;               /* block_size: tokens per block */
    uint32_t n_planes;                   /* 1 (e.g. MLA latent+rope) or 2 (separate K and V), <= KVL_MAX_PLANES */
    uint32_t row_bytes[KVL_MAX_PLANES];  /* cache bytes per token per layer, per plane */
    uint64_t pool_blocks;                /* blocks in the pool the tables index */
} kvl_layout_t;

/* One request of the batch: a hit prefix plus a short appended tail
 * (Section 2: each turn's prompt is the cached context plus appended tokens). */
typedef struct {
    uint32_t hit_tokens;         /* cached prefix length; these rows are moved */
    uint32_t append_tokens;      /* tail computed by prefill; never moved */
    uint32_t n_blocks;           /* entries in block_table, >= ceil((hit+append)/block_tokens) */
    const int32_t *block_table;  /* host pointer, borrowed for the duration of kvl_plan */
} kvl_request_t;

/* One copy descriptor: n_rows consecutive token rows, contiguous on both sides.
 * pool_row = block * block_tokens + row_in_block; xfer_row = index of the row
 * among the batch's hit tokens.  The same descriptors serve every plane. */
typedef struct {
    uint32_t pool_row;
    uint32_t xfer_row;
    uint32_t n_rows;
    uint32_t block_index;   /* block of the first row, counted over the blocks the plan touches, in request order */
} kvl_unit_t;

/* Optional tuning; a zero field means "library default". */
typedef struct {
    uint32_t unit_bytes;     /* upper limit for the bytes of one descriptor: runs are split evenly into pieces at or
                                below it; the plan picks one piece size for the whole batch (block_tokens * 2^j or
                                this limit) so that its descriptors are alike */
    uint32_t block_threads;  /* threads per workgroup: 64, 128, 256, 512 or 1024 */
    uint32_t variant;        /* 0: default; 1..512: an explicit kernel variant, see kvl_variant_name */
    uint32_t max_groups;     /* tiled and Full-Block kernels: at most this many workgroups per launch and
                                plane, each walking over several tiles.  0: one workgroup per tile, except
                                that a kernel whose far side is host memory is kept to 64 (enough to fill
                                the host link; the rest of the machine stays free for other kernels);
                                UINT32_MAX: never walk.  (A launch always stays below 2^32 lanes: beyond
                                that the workgroups walk, whatever this says.)  Flat kernels (token-granular
                                pools): at most this many workgroups per launch, the descriptors being
                                spread over as many launches as that takes; 0: as many as a launch holds */
} kvl_tuning_t;

/* Build a plan.  Validates the batch (KVL_ERANGE: a block id outside
 * [0, pool_blocks), a table shorter than the request needs, or more than 2^32-1
 * pool rows or moved tokens; KVL_EALIAS: with KVL_SCATTER, a block that receives
 * rows is named twice), lays out the transfer buffer, merges physically
 * adjacent blocks of a request into runs, splits runs into descriptors and,
 * unless KVL_HOST_ONLY, uploads them to the current device.
 * requests: host array of n_req entries (n_req may be 0).  *out receives the
 * plan; free it with kvl_plan_destroy.  tuning may be NULL. */
int kvl_plan(const kvl_layout_t *layout, const kvl_request_t *requests, uint32_t n_req,
             uint32_t flags, kvl_plan_t **out);
int kvl_plan_tuned(const kvl_layout_t *layout, const kvl_request_t *requests, uint32_t n_req,
                   uint32_t flags, const kvl_tuning_t *tuning, kvl_plan_t **out);
/* Frees the plan.  The call does not wait for the device: kernels enqueued with the
 * plan may still be running or queued.  Every launch made with a plan is followed by
 * an event on its stream (one event per stream, recorded again after each launch);
 * the plan's device descriptor array is retired with those events and goes back to a
 * small cache inside the library (at most 16 buffers / 256 MiB, from which later
 * plans are served without a device allocation) only when they have fired.  The
 * streams themselves are not touched here and may be gone already.  Only the plan's
 * own lanes, if a host-buffer call left work on them that is not finished, are
 * waited for.  A plan whose launches were captured into a HIP graph cannot be followed
 * that way: destroying it waits for the device, and the graph must not be replayed
 * afterwards.  A plan made with KVL_CALLER_SYNCS is not followed at all (see there).
 * kvl_release_cached_memory empties the cache and the library's pool of lanes; it
 * waits for the kernels of destroyed plans, and for nothing else. */
void kvl_plan_destroy(kvl_plan_t *plan);
void kvl_release_cached_memory(void);

/* Change launch tuning (block_threads if not 0, variant, max_groups) of an existing
 * plan; unit_bytes is fixed at plan time and ignored here. */
int kvl_plan_set_tuning(kvl_plan_t *plan, const kvl_tuning_t *tuning);

/* Plan inspection (host side, valid for any plan). */
int kvl_plan_payload_bytes(const kvl_plan_t *plan, uint64_t *bytes_per_layer); /* all planes */
int kvl_plan_hit_tokens(const kvl_plan_t *plan, uint64_t *tokens);             /* T: tokens the plan moves */
int kvl_plan_n_units(const kvl_plan_t *plan, uint64_t *n_units);
/* Copy up to capacity descriptors into out (host array); *n_units gets the total. */
int kvl_plan_get_units(const kvl_plan_t *plan, kvl_unit_t *out, uint64_t capacity, uint64_t *n_units);

/* One host-to-device chunk of the h2d path: descriptors [unit_begin, unit_end)
 * of plane `plane`, whose rows are the contiguous bytes
 * [host_offset, host_offset + bytes) of the transfer buffer. */
typedef struct {
    uint32_t plane;
    uint32_t unit_begin;
    uint32_t unit_end;
    uint32_t reserved;
    uint64_t host_offset;
    uint64_t bytes;
} kvl_chunk_t;
/* How kvl_h2d_unpack_layer would cut a layer into chunks of at most chunk_bytes
 * (KVL_ESPACE if one descriptor alone is larger).  Host side only. */
int kvl_plan_get_chunks(const kvl_plan_t *plan, uint64_t chunk_bytes,
                        kvl_chunk_t *out, uint64_t capacity, uint64_t *n_chunks);

/* Decode side (Section 4.1, decode-engine read path: the layer's hit cache
 * leaves the decode engine's buffer as Layer Blocks): gather.
 * pool_planes: host array of n_planes device pointers, layer l's plane bases.
 * xfer: device buffer of xfer_capacity >= payload bytes (else KVL_ESPACE); it may
 * also be pinned host memory mapped into the device's address space (the host
 * buffer of the engine the cache is sent on to): the kernel then writes it
 * across the host link itself.
 * Needs a KVL_GATHER plan.  Enqueues on stream. */
int kvl_pack_layer(const kvl_plan_t *plan, const void *const *pool_planes,
                   void *xfer, uint64_t xfer_capacity, void *stream);

/* Both sides on one device.  When the source pool and the destination pool live
 * in the same GPU's memory (engines sharing a device, or a cache being re-paged),
 * the transfer buffer between kvl_pack_layer and kvl_unpack_layer is pure
 * overhead: kvl_plan_pair joins a gather plan and a scatter plan over the same
 * token ranges (same block_tokens, planes and row sizes; KVL_EINVAL otherwise)
 * into one plan whose descriptors map source rows straight to destination rows,
 * and kvl_move_layer runs it: the result in the destination pool is exactly that
 * of pack followed by unpack, with half the memory traffic.  The two pools must
 * not overlap.  The paired plan is independent of the two it was made from. */
int kvl_plan_pair(const kvl_plan_t *gather, const kvl_plan_t *scatter, kvl_plan_t **out);
/* (A paired plan keeps its descriptors in the order of their destination rows, so that the
 * writes of a move run forward through the destination pool.) */
int kvl_move_layer(const kvl_plan_t *paired, const void *const *src_pool_planes,
                   void *const *dst_pool_planes, void *stream);

/* Prefill side (Section 4.1: before a layer's attention is computed its hit
 * cache is placed in the prefill engine's HBM): scatter.  Rows that hold no
 * hit token keep their bytes.  xfer_bytes must be >= payload bytes (KVL_ESPACE).
 * Needs a KVL_SCATTER plan.  Enqueues on stream. */
int kvl_unpack_layer(const kvl_plan_t *plan, const void *xfer, uint64_t xfer_bytes,
                     void *const *pool_planes, void *stream);

/* kvl_unpack_layer for callers that cannot allocate: code that must not call hipMalloc or
 * hipFree where it runs (tight serving loops, harnesses that forbid device allocation,
 * processes whose memory is fully handed out).  It takes the batch instead of a plan -- the
 * arguments of kvl_plan (flags: any of KVL_NO_MERGE, KVL_TOKENS_APPEND, KVL_TOKENS_ALL,
 * KVL_NO_POINTER_CHECKS; KVL_SCATTER is implied) followed by those of kvl_unpack_layer --
 * builds the descriptors on the host as kvl_plan does (same validation and error codes),
 * uploads them on `stream` into a fixed array in device memory that belongs to the library's
 * code object (KVL_NOALLOC_MAX_UNITS descriptors of 16 bytes = 8 MiB on every GPU the library
 * is loaded on, held until the process ends) and enqueues the same scatter kernels there.
 * The result in the pool is that of kvl_plan + kvl_unpack_layer.  It allocates no device or
 * pinned memory and creates no stream; its first call on a device creates two events.
 * KVL_ESPACE if the batch needs more than KVL_NOALLOC_MAX_UNITS descriptors (one per block of
 * a fragmented table) or xfer_bytes is below the payload.  Every call on a GPU uses that GPU's
 * one array: a call orders itself after the previous call's kernels (by an event, whatever
 * their streams) and calls are serialised by a lock inside the library, so calls from several
 * threads or streams are safe but do not overlap.  The descriptors are uploaded from host
 * memory, so the call cannot be captured into a HIP graph. */
#define KVL_NOALLOC_MAX_UNITS 524288u
int kvl_unpack_layer_noalloc(const kvl_layout_t *layout, const kvl_request_t *requests, uint32_t n_req,
                             uint32_t flags, const void *xfer, uint64_t xfer_bytes,
                             void *const *pool_planes, void *stream);

/* Prefill-engine read path, host buffer -> HBM for one layer (Section 4.1,
 * steps 3-4 of that path): the transfer buffer lies in PINNED host memory; it is
 * copied in chunks of at most chunk_bytes with hipMemcpyAsync into
 * k = min(8, floor(staging_bytes / chunk_bytes)) slots of dev_staging (device
 * memory, 16-byte aligned) and every landed chunk is scattered by a kernel.  Each
 * slot has a stream of the library's own on which its copies and scatters
 * alternate; the k of them run side by side, so the scatters hide under the
 * copies.  The call orders that work after everything already enqueued on
 * copy_stream and kernel_stream, and makes kernel_stream wait for its end: the
 * pool is complete when kernel_stream reaches the end of the enqueued work, and
 * a staging area may be reused by the next call at once.  KVL_ESPACE: staging
 * smaller than one chunk, or a chunk smaller than one descriptor.  Chunks of
 * 8 MiB or more keep the per-copy submission cost (Section 5.2) negligible.
 * chunk_bytes == 0 selects the zero-copy form: no staging, no copies; one scatter
 * kernel on kernel_stream reads the pinned buffer across the host link itself
 * (dev_staging, staging_bytes and copy_stream are then unused); it runs with few
 * workgroups (kvl_tuning_t::max_groups), enough to fill the link, so that it does
 * not take the compute units from other kernels.  Which to take: every
 * copy-then-kernel turn of a lane costs on the order of 100 us whatever the chunk's
 * size, so the staged form only draws level for layers of gigabytes on an otherwise
 * idle GPU; for small layers and beside heavy compute the zero-copy form is the
 * faster one.  The call only enqueues work and joins
 * its lanes by events, so it can be captured in a HIP graph (pass the capturing
 * stream for both stream arguments, after one eager call has made the lanes). */
int kvl_h2d_unpack_layer(const kvl_plan_t *plan, const void *pinned_host_xfer,
                         void *dev_staging, uint64_t staging_bytes, uint64_t chunk_bytes,
                         void *const *pool_planes, void *copy_stream, void *kernel_stream);

/* The way out of the prefill engine (Section 4.1: as a layer is computed its cache is
 * sent on to the decode engine's buffer in host memory): the staged form of
 * kvl_pack_layer with a pinned host destination.  The gather runs chunk by chunk
 * into the slots of dev_staging and every packed chunk is copied to its place in
 * pinned_host_xfer by the copy engine (hipMemcpyAsync), on the library's lanes; no
 * wavefront waits on the host link.  Ordered after everything enqueued on both
 * streams; the host buffer is complete when kernel_stream reaches the end of the
 * enqueued work.  Chunking, slots and errors as in kvl_h2d_unpack_layer
 * (chunk_bytes must not be 0); needs a KVL_GATHER plan. */
int kvl_d2h_pack_layer(const kvl_plan_t *plan, const void *const *pool_planes, void *dev_staging,
                       uint64_t staging_bytes, uint64_t chunk_bytes, void *pinned_host_xfer,
                       uint64_t host_capacity, void *kernel_stream, void *copy_stream);

/* Storage layout (Section 4.1 "Different Block Layouts", Appendix A.5).  All
 * traffic with storage uses Full Blocks, byte tensors [layer, tokens, bytes] that
 * are the concatenation of one block's Layer Blocks; with several planes a Layer
 * Block is its planes' spans one after the other:
 *   LB = block_tokens * sum_p row_bytes[p],  FB = n_layers * LB,
 *   byte (layer l, plane p, row w, j) of a Full Block at
 *       l*LB + block_tokens * sum_{q<p} row_bytes[q] + w*row_bytes[p] + j.
 * A Full-Block buffer holds the blocks the plan's token ranges touch, request
 * after request, each request's blocks in table order (kvl_unit_t::block_index
 * counts them).  The two calls below move ONE layer's rows between such a buffer
 * and a paged pool with a single kernel that does the layout conversion on the
 * fly; the buffer may be device memory or pinned host memory mapped into the
 * device (then the kernel crosses the host link itself and nothing is staged).
 * Both need a plan made with KVL_NO_MERGE (descriptors must not span blocks);
 * KVL_EINVAL otherwise or if layer >= n_layers; KVL_ESPACE if the buffer is
 * smaller than n_full_blocks * full_block_bytes. */
int kvl_plan_fullblock_geometry(const kvl_plan_t *plan, uint64_t *full_block_bytes, uint64_t *n_full_blocks);
/* storage read -> prefill pool, layer by layer (KVL_SCATTER plan) */
int kvl_fullblocks_to_pool_layer(const kvl_plan_t *plan, const void *full_blocks, uint64_t full_blocks_bytes,
                                 uint32_t layer, void *const *pool_planes, void *stream);
/* decode pool -> Full Blocks to persist (KVL_GATHER plan); bytes of the buffer that
 * belong to other layers or to rows outside the ranges are left as they are */
int kvl_pool_to_fullblocks_layer(const kvl_plan_t *plan, const void *const *pool_planes, uint32_t layer,
                                 void *full_blocks, uint64_t full_blocks_bytes, void *stream);
/* Staged form of kvl_fullblocks_to_pool_layer: layer `layer` of the blocks is
 * brought into the slots of dev_staging by the runtime's strided copies
 * (hipMemcpy2DAsync: per chunk of floor(chunk_bytes / LB) blocks, rows of LB bytes
 * at a pitch of FB) and converted into the pool from there by a kernel per chunk,
 * on the library's lanes and with the stream semantics of kvl_h2d_unpack_layer.
 * How the copies cross the link is the runtime's business (on the machine this was
 * written on it uses a copy kernel of its own for them).
 * KVL_ESPACE also if chunk_bytes < LB or staging_bytes < chunk_bytes. */
int kvl_h2d_fullblocks_layer(const kvl_plan_t *plan, const void *full_blocks, uint64_t full_blocks_bytes,
                             uint32_t layer, void *dev_staging, uint64_t staging_bytes, uint64_t chunk_bytes,
                             void *const *pool_planes, void *copy_stream, void *kernel_stream);

/* Staged form of kvl_pool_to_fullblocks_layer: a kernel per chunk of blocks lays
 * the rows out as Layer Blocks in a staging slot, and copies of the runtime
 * (hipMemcpy2DAsync, hipMemcpyAsync) write them into the buffer: runs of wholly covered
 * blocks with one strided copy each, the rows of a partly covered block (the ends
 * of a request's range) with one copy per plane.  As with the one-kernel form no
 * byte outside the plan's rows is written.  Streams, slots and errors as in
 * kvl_h2d_fullblocks_layer; needs a KVL_GATHER | KVL_NO_MERGE plan. */
int kvl_d2h_fullblocks_layer(const kvl_plan_t *plan, const void *const *pool_planes, uint32_t layer,
                             void *dev_staging, uint64_t staging_bytes, uint64_t chunk_bytes,
                             void *full_blocks, uint64_t full_blocks_bytes, void *kernel_stream,
                             void *copy_stream);

/* Confine the scatter kernels of the host-buffer path to some compute units.
 * The paper isolates cache traffic from the model's own traffic with network QoS
 * (Section 5.1); on the GPU the matching question is how many compute units the
 * load may occupy.  The staged chunks arrive at host-link rate, which a handful
 * of compute units can scatter, so the library's lanes can be created with a
 * compute-unit mask (hipExtStreamCreateWithCUMask: bit i of mask[] enables CU i;
 * n_words 32-bit words).  n_words == 0 removes the mask.  Existing lanes are
 * drained and re-created; a mask the runtime cannot honour (on MI355X: fewer than
 * one compute unit in each of the 8 XCDs, i.e. fewer than the first 8 bits) shows
 * up as KVL_EHIP from the next host-buffer call.  Every masked lane takes a
 * hardware queue of its own.  Streams the caller passes in are the caller's to mask. */
int kvl_plan_set_lane_cu_mask(kvl_plan_t *plan, const uint32_t *mask, uint32_t n_words);

/* The same result with one hipMemcpyAsync per descriptor and plane, straight from
 * the pinned host buffer into the paged pool: no staging, no kernel.  This is the
 * many-small-copies pattern whose per-copy submission cost Section 5.2 measures
 * (5-7 us per copy on its hardware); it exists to measure that cost here and is
 * not the fast path.  *n_copies (may be NULL) receives the number of copies
 * enqueued on stream. */
int kvl_h2d_blockwise_layer(const kvl_plan_t *plan, const void *pinned_host_xfer,
                            void *const *pool_planes, void *stream, uint64_t *n_copies);
/* The same copies handed to the runtime in one call (hipMemcpyBatchAsync, which newer
 * HIP runtimes have): what batching the submission buys on this platform, for the
 * same study.  KVL_ENOSYS if the runtime loaded in this process has no such call. */
int kvl_h2d_blockwise_batched_layer(const kvl_plan_t *plan, const void *pinned_host_xfer,
                                    void *const *pool_planes, void *stream, uint64_t *n_copies);

/* A 16-byte sample of what the compute of a layer sees. */
typedef struct {
    uint32_t plane;
    uint32_t reserved;
    uint64_t byte_offset;   /* into the slot's plane, multiple of 16 */
} kvl_probe_t;

/* Called on the calling thread before layer `layer`'s host buffer
 * (host_layers[layer % n_host_slots]) is read, once all earlier reads of that
 * slot have completed: the place where the storage read of that layer would
 * deliver its bytes.  Return non-zero to abort the run. */
typedef int (*kvl_host_fill_fn)(void *user, uint32_t layer, void *host_slot, uint64_t bytes);

/* The caller's own per-layer computation, in place of the synthetic kernel.  Called
 * on the calling thread, in layer order, once compute_stream has been made to wait
 * for layer `layer`'s load: enqueue the layer's work on compute_stream and return
 * (do not synchronise).  slot_planes are the n_planes device bases of the slot that
 * holds the layer.  Whatever the callback enqueues is what the next load into that
 * slot waits for.  Return non-zero to abort the run. */
typedef int (*kvl_compute_fn)(void *user, uint32_t layer, void *const *slot_planes, void *compute_stream);

typedef struct {
    uint32_t n_layers;                 /* 0: take layout.n_layers */
    uint32_t n_host_slots;             /* H >= 1 */
    void *const *host_layers;          /* [H] pinned host transfer buffers */
    uint32_t n_dev_slots;              /* S >= 1 resident destination layers */
    void *const *dev_slot_planes;      /* [S * n_planes] device plane bases, slot-major */
    void *dev_staging;                 /* as in kvl_h2d_unpack_layer; chunk_bytes == 0: zero-copy loads */
    uint64_t staging_bytes;
    uint64_t chunk_bytes;
    uint32_t compute_us;               /* duration of the synthetic per-layer compute kernel */
    uint32_t n_probes;                 /* optional samples taken by the compute kernel */
    const kvl_probe_t *probes;         /* host array [n_probes] */
    void *probe_out;                   /* device, n_layers * n_probes * 16 bytes */
    void *const *snapshot_planes;      /* optional [n_layers * n_planes] device buffers: a copy of the
                                          slot taken on the compute stream right after compute(l) */
    kvl_host_fill_fn host_fill;        /* optional */
    void *host_fill_user;
    void *copy_stream;                 /* three distinct non-default streams recommended */
    void *kernel_stream;
    void *compute_stream;
    /* Optional storage-layout source.  When full_blocks is not NULL the layers are
     * loaded from a buffer of the plan's Full Blocks (device memory, or pinned host
     * memory mapped into the device) as kvl_fullblocks_to_pool_layer does: layer l
     * by one converting kernel on kernel_stream (chunk_bytes == 0), or staged through
     * dev_staging as kvl_h2d_fullblocks_layer does (chunk_bytes != 0).  host_layers and
     * host_fill are then unused.  Needs a plan made with KVL_NO_MERGE. */
    const void *full_blocks;
    uint64_t full_blocks_bytes;
    /* Optional: the caller's computation instead of the synthetic kernel (compute_us
     * and the probes are then unused; snapshots are still taken after it). */
    kvl_compute_fn compute;
    void *compute_user;
    /* Optional outflow (Section 4.1: once a layer has been computed its cache, hit and
     * appended tokens alike, leaves for the decode engine's buffer while the next
     * layers are loaded and computed).  After the compute of layer l, out_plan (a
     * KVL_GATHER plan over the same pool geometry, typically KVL_TOKENS_ALL) gathers
     * slot l % S into out_host_layers[l % n_out_host_slots] (pinned host memory of
     * out_plan's payload size): staged through out_staging as kvl_d2h_pack_layer does
     * (out_chunk_bytes != 0) or by a kernel that writes the host buffer itself
     * (out_chunk_bytes == 0).  The load of layer l + S then waits for that gather
     * rather than for the compute alone.  host_drain, if given, is called on the
     * calling thread with (user, l, buffer, payload bytes of out_plan) once layer l
     * has arrived in its buffer and before the buffer is reused: the place where the
     * send to the decode engine would go. */
    const kvl_plan_t *out_plan;
    uint32_t n_out_host_slots;
    void *const *out_host_layers;
    void *out_staging;
    uint64_t out_staging_bytes;
    uint64_t out_chunk_bytes;
    kvl_host_fill_fn host_drain;
    void *host_drain_user;
} kvl_stream_cfg_t;

typedef struct {
    double total_ms;         /* first copy enqueued .. last compute (or outflow) finished (device clock) */
    double h2d_bytes;        /* bytes that crossed the host link */
    double link_gbps;        /* h2d_bytes / total_ms, GB/s */
    double exposed_ms;       /* total_ms minus the compute time (n_layers * compute_us, or the measured
                                sum of the caller's computations): load time not hidden */
    /* optional per-layer times in ms since the start, host arrays of n_layers or NULL */
    float *t_loaded;         /* layer's scatter finished */
    float *t_compute_begin;
    float *t_compute_end;
    float *t_out_done;       /* layer's outflow arrived in host memory (with out_plan) */
    double d2h_bytes;        /* bytes the outflow sent over the host link */
    double out_gbps;         /* d2h_bytes / total_ms */
} kvl_stream_stats_t;

/* Layer-wise load of all layers (Section 4.1: the load of a layer overlaps the
 * computation of the layers before it; layer-wise prefill keeps only a few
 * layers' cache resident).  For l = 0 .. n_layers-1: layer l is loaded from
 * host_layers[l % H] into destination slot l % S by the h2d path; the compute
 * of layer l (a kernel that spins compute_us on the compute stream, or what
 * cfg->compute enqueues there) starts after that load; the load of layer l + S starts scattering only after the
 * compute of layer l has finished.  Blocks until everything has finished and
 * fills *stats (may be NULL).  Needs a KVL_SCATTER plan. */
int kvl_stream_layers(const kvl_plan_t *plan, const kvl_stream_cfg_t *cfg, kvl_stream_stats_t *stats);

/* Measure the host link: time `reps` host-to-device hipMemcpyAsync of `bytes`
 * from pinned host memory on `stream`; *gbps gets the best rate in GB/s. */
int kvl_measure_h2d_peak(const void *pinned_host, void *dev, uint64_t bytes, uint32_t reps,
                         void *stream, double *gbps);

/* Plain device-to-device streaming copy with the same load/store code as the
 * pack kernel (bytes multiple of 16, pointers 16-byte aligned): the ceiling a
 * gather with perfect locality could reach, and the known-size kernel used to
 * calibrate HBM byte counters. */
int kvl_copy_linear(const void *src, void *dst, uint64_t bytes, void *stream);

/* Reference streams for measuring what the memory can do, beside the kernels of the load path
 * (the benchmark's ceilings): plain device memory, the load/store instructions and cache policies
 * of the default gather and scatter, no descriptors.
 *   block_bytes == 0: one linear stream of `bytes` bytes, src (+ skew_bytes) -> dst;
 *   block_bytes != 0: the access shape of a paged copy without its block tables: one side
 *     ("dense") is a linear stream, the other hops every block_bytes: block u of the dense
 *     side lives in block (u * odd constant) mod 2^hop_blocks_log2 of the hopping side, or in
 *     block block_table[u] if block_table (device, bytes / block_bytes entries, each below
 *     2^hop_blocks_log2 -- the caller's responsibility) is given: one scalar load per workgroup
 *     before the data can be addressed, as the descriptor fetch of the real kernels.
 *     hopping_side 0: the source hops (a gather; src holds 2^hop_blocks_log2 blocks, dst
 *     bytes + skew_bytes), 1: the destination hops (a scatter).  skew_bytes (multiple of 16, below
 *     128) shifts the dense side, so that the two sides sit differently in their 128-byte lines.
 * mode: copy, or only the reads, or only the writes of that copy.  Both pointers 128-byte
 * aligned; sizes are checked against the buffers (KVL_ESPACE).  What lands in dst is of no
 * use.  Enqueues on stream; the caller times it. */
#define KVL_CEILING_COPY  0u
#define KVL_CEILING_READ  1u
#define KVL_CEILING_WRITE 2u
typedef struct {
    uint32_t mode;
    uint32_t block_bytes;
    uint32_t hopping_side;
    uint32_t skew_bytes;
    uint32_t hop_blocks_log2;
} kvl_ceiling_t;
int kvl_ceiling_kernel(const kvl_ceiling_t *c, const void *src, uint64_t src_bytes, void *dst, uint64_t dst_bytes,
                       uint64_t bytes, const uint32_t *block_table, void *stream);

/* What every entry point asks of a buffer before a kernel may touch it: is
 * [ptr, ptr + bytes) memory this device can address?  Host memory passes only if
 * allow_host is non-zero and it is pinned and mapped (pageable host memory and
 * stray pointers give KVL_EINVAL); device and pinned allocations are checked
 * against their extent (KVL_ESPACE if the span runs past it).  A wrong pointer thus comes back as
 * an error code instead of a memory fault on the GPU.  Costs a few microseconds
 * per buffer; a plan made with KVL_NO_POINTER_CHECKS skips it. */
int kvl_check_buffer(const void *ptr, uint64_t bytes, int allow_host);

const char *kvl_strerror(int code);
/* hipError_t of the last KVL_EHIP on this thread, and its text. */
int kvl_last_hip_error(void);
const char *kvl_last_hip_error_string(void);
const char *kvl_variant_name(uint32_t variant);   /* thread-local text; NULL beyond the last variant */
const char *kvl_version(void);

#ifdef __cplusplus
}
#endif
#endif /* KVL_H */
