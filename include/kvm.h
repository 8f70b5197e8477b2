/*
 * kvm.h - C ABI of libkvm: paged-KV-cache migration for one MI355X (gfx950).
 *
 * The library implements the data path of Mell's adaptive request migration
 * (arXiv 2501.06709, Sec. "Adaptive Request Migration", step "Hybrid
 * Migration": the class of requests that is moved as KV cache rather than as
 * tokens).  A request's KV cache lives in a paged block pool (Sec. "Background
 * & Related Work": KV cache in non-contiguous paged memory); migrating it means
 * reading tokens [0,k) of every layer, K and V, through the source block table
 * and writing them into freshly allocated blocks of another pool under a new
 * block table.  Tokens [k,len) are the part the method would re-prefill from
 * token ids on the destination and are never touched here.
 *
 * Conventions for every entry point
 *   - "host" pointers are ordinary CPU memory, "device" pointers are HBM
 *     addresses valid on the current HIP device.  The caller owns every buffer.
 *   - `hip_stream` is a hipStream_t (NULL = the default stream).  Kernels are
 *     enqueued on it and the call returns without synchronising.  The library
 *     allocates no device memory.
 *   - Return value: KVM_OK (0) or a negative kvm_status.  All argument checks
 *     run on the host before the first launch, so KVM_EINVAL / KVM_ENOMEM mean
 *     that no device byte was written.  kvm_last_error() gives the detail.
 *   - Elements are 16-bit (fp16 or bf16) and are moved as raw bit patterns.
 */
#ifndef KVM_H
#define KVM_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  KVM_OK = 0,
  KVM_EINVAL = -1, /* bad argument: see kvm_last_error() */
  KVM_ENOMEM = -2, /* free list cannot supply the blocks; nothing was popped */
  KVM_EHIP = -3    /* a HIP call failed; kvm_last_error() holds its text */
} kvm_status;

typedef enum { KVM_F16 = 0, KVM_BF16 = 1 } kvm_dtype;

/*
 * Per-model KV layout (the method serves several models from one cluster, so a
 * layout travels with every pool).  An element (layer l, kv in {0:K,1:V},
 * physical block b, KV head h, slot s in [0,block_tokens), dim d) sits at
 *   base + 2 * (l*stride_layer + kv*stride_kv + b*stride_block
 *               + h*stride_head + s*stride_slot + d)          bytes.
 * Strides are in elements, the dim stride is 1.  The same block id addresses
 * the block in every (layer, kv) plane.  Required: head_dim*2 and every
 * stride*2 are multiples of 16 bytes; n_q_heads is a multiple of n_kv_heads;
 * stride_slot >= head_dim; (n_kv_heads-1)*stride_head + (block_tokens-1)*
 * stride_slot + head_dim < 2^31 (a block's own extent fits 32 bits of bytes).
 */
typedef struct {
  int32_t n_layers;
  int32_t n_kv_heads;
  int32_t n_q_heads;
  int32_t head_dim;
  int32_t block_tokens;
  int32_t dtype; /* kvm_dtype */
  int64_t stride_layer;
  int64_t stride_kv;
  int64_t stride_block;
  int64_t stride_head;
  int64_t stride_slot;
} kvm_layout;

/* One block pool: `base` is a device pointer, 16-byte aligned, caller-owned. */
typedef struct {
  void* base;
  int64_t n_blocks;
  kvm_layout layout;
} kvm_pool;

/*
 * A batch of requests of ONE model with their block tables in CSR form.
 * Request r owns table entries bt_offsets[r] .. bt_offsets[r+1]-1; entry j
 * holds the physical block of tokens [j*B, j*B+B), B = block_tokens.
 * k[r] is the split point of the method's migrate-versus-recompute choice:
 * tokens [0,k[r]) are moved (or, for kvm_paged_decode, attended over);
 * 0 <= k[r] <= B * (entries of r).  k[r] = 0 makes the request a no-op.
 */
typedef struct {
  int32_t n_req;
  const int32_t* bt_offsets;     /* host,   [n_req+1], bt_offsets[0] = 0 */
  const int32_t* bt_blocks_dev;  /* device, [bt_offsets[n_req]] */
  const int32_t* bt_blocks_host; /* host copy of bt_blocks_dev, or NULL.  When
                                    given, every id that will be dereferenced is
                                    range-checked, and on the writing side
                                    checked for duplicates.  NULL skips those
                                    checks: ids are then the caller's promise. */
  const int32_t* k;              /* host,   [n_req] */
  const int32_t* start;          /* host,   [n_req] or NULL (= all zero): first
                                    token to move.  With start[r] > 0 only tokens
                                    [start[r], k[r]) are moved; they keep their
                                    logical index, so entry j of the table still
                                    covers tokens [j*B, j*B+B).  This is the unit
                                    of a multi-round live migration, where an
                                    earlier round has already moved [0,start).
                                    0 <= start[r] <= k[r]. */
} kvm_batch;

/* ---- closed-form sizes (host, pure) -------------------------------------
 * Sec. "System Model": a request's KV size grows linearly with its tokens;
 * bytes per token = n_layers * 2 * n_kv_heads * head_dim * 2.  Return -1 on a
 * NULL or inconsistent layout. */
int64_t kvm_bytes_per_token(const kvm_layout* layout);
int64_t kvm_block_bytes(const kvm_layout* layout); /* block_tokens * bytes_per_token */
/* Sum over the batch of (k[r] - start[r]) * bytes_per_token: the size of the
 * staging buffer written by kvm_pack and read by kvm_unpack.  Exactly linear in
 * the number of tokens, no padding. */
int64_t kvm_staging_bytes(const kvm_layout* layout, const kvm_batch* batch);

/* Fill `out` with the canonical dense layout
 *   pool[layer][kv][block][head][slot][dim]
 * for a pool of n_blocks blocks.  Returns KVM_EINVAL on non-positive sizes,
 * n_q_heads not a multiple of n_kv_heads, or head_dim*2 not a multiple of 16. */
int kvm_layout_canonical(kvm_layout* out, int32_t n_layers, int32_t n_kv_heads,
                         int32_t n_q_heads, int32_t head_dim, int32_t block_tokens,
                         int32_t dtype, int64_t n_blocks);
/* Bytes a pool with this layout and n_blocks spans from `base` (largest byte
 * offset of any element + 1); -1 on a bad layout. */
int64_t kvm_pool_span_bytes(const kvm_layout* layout, int64_t n_blocks);

/* ---- the migration data path --------------------------------------------
 * Sec. "Adaptive Request Migration" (KV-cache class of "Hybrid Migration") and
 * Sec. "Motivation", Finding 4 (copying the KV of the legacy tokens relies on
 * the cache being append-only, so a prefix [0,k) is a valid unit of transfer).
 *
 * Staging ("wire") format, shared by kvm_pack and kvm_unpack: requests in
 * batch order, each as [layer][kv][head][token start[r] <= t < k[r]][dim], 16-bit
 * elements, no padding; request r starts at byte
 * (sum_{r'<r} (k[r'] - start[r'])) * bytes_per_token.
 *
 * Token ranges (Sec. "Background & Related Work": live migration copies the
 * cache of the legacy tokens while new tokens are still being decoded, which the
 * append-only cache allows): with batch.start set, each call moves only
 * [start[r], k[r]); moving [0,a) and later [a,b) leaves the destination exactly
 * as moving [0,b) at once.
 *
 * Limits: a single request may move at most 65535 blocks in one call (a range
 * [start,k) splits longer moves); batches of any size are split into launches
 * of 64 requests internally.
 */

/* Gather: staging[...] = src pool contents of tokens [0,k[r]) of each request.
 * staging_dev: device, 16-byte aligned, staging_bytes >= kvm_staging_bytes().
 * Reads the pool and the table only; writes exactly kvm_staging_bytes() bytes.
 * KVM_EINVAL: NULL pointer, bad layout, k out of range, block id outside
 * [0,n_blocks) (when host ids are given), staging too small, misaligned or
 * overlapping the pool's span. */
int kvm_pack(const kvm_pool* src, const kvm_batch* src_reqs, void* staging_dev,
             int64_t staging_bytes, void* hip_stream);

/* Scatter: inverse of kvm_pack into the blocks named by dst_reqs.  Slots
 * >= k[r] mod B of a request's last block, and all other blocks of the pool,
 * keep their bytes.  In addition to kvm_pack's checks: a block id that occurs
 * twice among the written entries of dst_reqs is KVM_EINVAL. */
int kvm_unpack(const void* staging_dev, int64_t staging_bytes, const kvm_pool* dst,
               const kvm_batch* dst_reqs, void* hip_stream);

/* Fused gather+scatter without staging: for every request r, layer, K and V,
 * head and token t < k[r], the element at logical position t of the source
 * request is copied to logical position t of the destination request.
 * The source pool is never written (Sec. "Adaptive Request Migration",
 * "Boundary Profiling": source memory stays allocated until the transfer is
 * complete; releasing it is the caller's later step).
 * KVM_EINVAL additionally when: n_req or any k[r] or start[r] differs between the
 * two batches; the layouts differ in anything but strides; src and dst are the
 * same allocation region and a written dst block id is also a read src id. */
int kvm_migrate(const kvm_pool* src, const kvm_batch* src_reqs, const kvm_pool* dst,
                const kvm_batch* dst_reqs, void* hip_stream);

/* ---- paged decode attention ----------------------------------------------
 * Sec. "Background & Related Work": the decoding phase reads the KV cache of
 * all previous tokens to produce the next one.  For request r, layer l, query
 * head hq (KV head g = hq / (n_q_heads / n_kv_heads)):
 *   s_t = scale * sum_d q[r][l][hq][d] * K_t[g][d],   t in [0,k[r])
 *   out[r][l][hq][:] = sum_t softmax(s)_t * V_t[g][:]
 * read through the block table.  q_dev: device, [n_req][n_layers][n_q_heads]
 * [head_dim] in the pool's dtype.  out_dev: same shape, float32 when
 * out_is_f32 != 0, else the pool's dtype (round to nearest even).  Accumulation
 * is fp32.  scale = 0 selects 1/sqrt(head_dim).  A request with k[r] = 0 leaves
 * its output rows untouched.
 * workspace_dev / workspace_bytes: device scratch for splitting long contexts
 * over several workgroups (size from kvm_decode_workspace_bytes; 16-byte
 * aligned).  NULL or too small a workspace is legal: the context is then not
 * split.  The result depends only on logical token positions, never on which
 * physical blocks hold them.  reqs->start must be NULL or all zero.
 * block_tokens 16 with head_dim 64 or 128 runs the tuned kernel; any other block
 * size and head_dim up to 512 runs a plain fallback kernel (head_dim > 512 is
 * KVM_EINVAL). */
int kvm_paged_decode(const kvm_pool* pool, const kvm_batch* reqs, const void* q_dev,
                     void* out_dev, int out_is_f32, float scale, void* workspace_dev,
                     int64_t workspace_bytes, void* hip_stream);
int64_t kvm_decode_workspace_bytes(const kvm_layout* layout, const kvm_batch* reqs);

/* kvm_paged_decode with an explicit row per request: request r reads its query
 * from row rows[r] of q_dev and writes row rows[r] of out_dev (rows: host,
 * [n_req]; NULL = the identity, i.e. kvm_paged_decode).  This is what lets the
 * requests that one time slot's migration orders moved into a pool (Sec. "Online KV
 * Cache Scheduling", request operation batching: a slot's moves are known together)
 * be decoded by ONE call although their queries sit in rows of a larger per-model
 * query buffer.  Rows beyond the buffers are the caller's responsibility.
 * KVM_EINVAL in addition to kvm_paged_decode's: a negative row, or two requests
 * with k > 0 that share a row. */
int kvm_paged_decode_rows(const kvm_pool* pool, const kvm_batch* reqs, const int32_t* rows,
                          const void* q_dev, void* out_dev, int out_is_f32, float scale,
                          void* workspace_dev, int64_t workspace_bytes, void* hip_stream);

/* kvm_paged_decode for callers that cannot allocate device memory or pass a
 * workspace along: code under HIP graph capture, tight serving loops, harnesses
 * that forbid hipMalloc.  Same arguments, checks, kernels and results as
 * kvm_paged_decode, but the context-split workspace is a fixed array of
 * KVM_STATIC_SCRATCH_BYTES that the library holds in device memory of every GPU
 * it runs on (until the process ends); the call allocates nothing on the device.
 * KVM_EINVAL (before any launch) when the batch's split workspace,
 * kvm_decode_workspace_bytes(), exceeds KVM_STATIC_SCRATCH_BYTES; with default
 * options no batch needs more than about 17 MiB.  KVM_EHIP when the array's
 * device address cannot be obtained.  All calls on one GPU share the array:
 * two calls may not overlap in time on one GPU (calls on one stream never do);
 * nothing in it has to survive between calls and nothing needs clearing. */
#define KVM_STATIC_SCRATCH_BYTES (32 << 20)
int kvm_paged_decode_static(const kvm_pool* pool, const kvm_batch* reqs, const void* q_dev,
                            void* out_dev, int out_is_f32, float scale, void* hip_stream);

/* ---- host free-list allocator (integers only) ----------------------------
 * Destination blocks for a migrated request come from the destination pool's
 * free list (capacity constraint of Sec. "System Model", Eq. 2).  Lowest free
 * id first; all-or-nothing. */
typedef struct kvm_freelist kvm_freelist;
/* occupied: host, n_blocks bytes, non-zero = block in use; NULL = all free.
 * Returns NULL on n_blocks <= 0 or n_blocks > 2^31-1. */
kvm_freelist* kvm_freelist_create(int64_t n_blocks, const uint8_t* occupied);
void kvm_freelist_destroy(kvm_freelist* fl);
int64_t kvm_freelist_available(const kvm_freelist* fl);
/* Pop the n lowest free ids into out_ids (host, ascending).  KVM_ENOMEM if
 * fewer than n are free: then nothing is popped and out_ids is untouched. */
int kvm_freelist_alloc(kvm_freelist* fl, int32_t n, int32_t* out_ids);
/* Return ids to the list.  KVM_EINVAL (and no change) if an id is out of
 * range, already free, or repeated in `ids`. */
int kvm_freelist_free(kvm_freelist* fl, int32_t n, const int32_t* ids);
/* Take exactly these ids off the list (rebuilding a list from existing block
 * tables).  KVM_EINVAL (and no change) if an id is out of range, not free, or
 * repeated in `ids`. */
int kvm_freelist_reserve(kvm_freelist* fl, int32_t n, const int32_t* ids);

/* ---- hybrid-migration divider (host, integers only) -----------------------
 * Sec. "Adaptive Request Migration", "Hybrid Migration" and "Global Consensus":
 * every request to be migrated is put into one of two classes, transferred as KV
 * cache (k = len for kvm_migrate) or transferred as tokens and re-prefilled on the
 * destination (k = 0), so that the KV bytes sent over each link stay within the
 * link's communication boundary and the tokens to prefill on each destination
 * instance stay within its computation boundary: a two-bin packing solved
 * greedily.  All pending moves of the whole system are given in one list, in an
 * order every instance agrees on; the function is deterministic, so every
 * instance that runs it reaches the same division.
 *
 * Moves are taken in list order.  KVM_FIRST_FIT tries the KV class first, then
 * the token class.  KVM_BEST_FIT picks, among the classes that still have room,
 * the one whose bin is left with the smaller free fraction of its boundary
 * (ties: KV).  A move that fits neither bin is KVM_CLASS_DEFER (left for a later
 * epoch).  A boundary of 0 closes the bin; moves with kv_bytes = 0 or tokens = 0
 * cost nothing in that bin.
 * KVM_EINVAL: NULL pointers, negative sizes or boundaries, link / dst out of
 * range, unknown policy. */
typedef struct {
  int32_t link;     /* index into comm_boundary: the link the KV bytes would cross */
  int32_t dst;      /* index into comp_boundary: the instance that would prefill */
  int64_t kv_bytes; /* size of the request's KV cache (len * bytes_per_token) */
  int64_t tokens;   /* tokens to prefill if sent as tokens */
} kvm_move;
typedef enum { KVM_CLASS_KV = 0, KVM_CLASS_TOKENS = 1, KVM_CLASS_DEFER = 2 } kvm_move_class;
typedef enum { KVM_FIRST_FIT = 0, KVM_BEST_FIT = 1 } kvm_divide_policy;
int kvm_divide_moves(const kvm_move* moves, int32_t n_moves, const int64_t* comm_boundary,
                     int32_t n_links, const int64_t* comp_boundary, int32_t n_instances,
                     int32_t policy, int32_t* out_class);

/* ---- order sequencing (host; launches through the entry points above) -------
 * Sec. "Adaptive Request Migration", "Boundary Profiling": the source memory of a
 * migrating request cannot be released until the transfer is complete; Sec. "Online
 * KV Cache Scheduling", request operation batching: the moves of a time slot are
 * known together.  An order moves tokens [0,k) of one request from `src` into
 * freshly allocated blocks of `dst` (two pools of one model).  Orders are staged and
 * then enqueued together by a flush:
 *   - one host-to-device copy carries the block tables of all staged orders;
 *   - the staged orders that share a (src, dst) pool pair become ONE kvm_migrate call
 *     and, where a decode was asked for, ONE kvm_paged_decode_rows call (float32
 *     output, default scale) over the destination;
 *   - one event is recorded behind the flush; the source blocks of its orders go back
 *     to their free lists once it has completed.  At most `depth` flushes are in flight
 *     before a call waits for the oldest, so the stream never drains between flushes.
 * An order whose source blocks are written by an order that is still staged (the same
 * request moved twice) is not grouped with it: staging it flushes first.
 *
 * The sequencer allocates no device memory: the caller hands it a pinned host buffer
 * and a device buffer of kvm_sequencer_table_ints() int32 each for the tables (both
 * must outlive it), and optionally a decode workspace.  A sequencer, and the free
 * lists it is given, belong to one host thread at a time; all its launches go to the
 * stream passed with each call (use one stream per sequencer). */
typedef struct kvm_sequencer kvm_sequencer;
int64_t kvm_sequencer_table_ints(int32_t max_blocks_per_request, int32_t max_staged, int32_t depth);
/* NULL (kvm_last_error() says why) on non-positive sizes, NULL table buffers or
 * table_ints below kvm_sequencer_table_ints(). */
kvm_sequencer* kvm_sequencer_create(int32_t max_blocks_per_request, int32_t max_staged, int32_t depth,
                                    int32_t* tables_host_pinned, int32_t* tables_dev, int64_t table_ints,
                                    void* decode_workspace_dev, int64_t decode_workspace_bytes);
/* Waits for everything in flight, releases its source blocks, hands the destination
 * blocks of orders that were never enqueued back, frees the host state. */
void kvm_sequencer_destroy(kvm_sequencer* seq);
/* Stage one order: pops ceil(k / block_tokens) blocks from dst_free into
 * dst_table_out (host, ascending) and notes the order for the next flush; a full
 * stage (max_staged orders) flushes first.  src_table: host, the request's
 * n_src_blocks block ids in src (copied).  q_dev != NULL asks for paged decode of the
 * request over the destination after its copy: query row `row` of q_dev, output row
 * `row` of out_dev (float32), both [rows][layers][query heads][head_dim]; orders
 * staged together that share q_dev / out_dev need distinct rows.
 * KVM_ENOMEM when dst_free cannot supply the blocks even after everything staged and
 * in flight has been enqueued, awaited and released; the order is then not staged and
 * dst_table_out is untouched.  KVM_EINVAL: NULL argument, k outside
 * [0, n_src_blocks * block_tokens], n_src_blocks above max_blocks_per_request, a
 * source id outside the pool.  An error of a flush that this call triggered is
 * returned as that flush's (see kvm_sequencer_flush); the order is then not staged. */
int kvm_sequencer_stage(kvm_sequencer* seq, const kvm_pool* src, kvm_freelist* src_free,
                        const kvm_pool* dst, kvm_freelist* dst_free, const int32_t* src_table,
                        int32_t n_src_blocks, int32_t k, const void* q_dev, void* out_dev, int32_t row,
                        int32_t* dst_table_out, void* hip_stream);
/* Enqueue everything staged on hip_stream (no-op when nothing is staged).  On an
 * error of one of its launches the groups already enqueued stay in flight (their
 * sources are released after the flush's event as usual), the destination blocks of
 * the groups not enqueued go back to their free lists at once and their sources stay
 * allocated; the error is returned. */
int kvm_sequencer_flush(kvm_sequencer* seq, void* hip_stream);
/* kvm_sequencer_flush, then wait for every flush in flight and release its sources. */
int kvm_sequencer_drain(kvm_sequencer* seq, void* hip_stream);
/* kvm_migrate + kvm_paged_decode_rows calls made so far (-1 on NULL). */
int64_t kvm_sequencer_launches(const kvm_sequencer* seq);
/* Measurement support: with timing enabled every kvm_migrate call is bracketed by a
 * pair of HIP events on the launch stream; kvm_sequencer_copy_stats waits for them and
 * returns their summed duration, the bytes read + written by those calls and their
 * number.  Enabling or disabling clears what was collected. */
int kvm_sequencer_timing(kvm_sequencer* seq, int enable);
int kvm_sequencer_copy_stats(kvm_sequencer* seq, double* ms_out, int64_t* bytes_out, int64_t* launches_out);

/* ---- diagnostics ---------------------------------------------------------- */
const char* kvm_strerror(int status);
/* Detail of the last failure on the calling thread ("" if none); the pointer
 * stays valid until the next failing call on this thread. */
const char* kvm_last_error(void);
/* Launch options; unknown name or out-of-range value gives KVM_EINVAL.  Every
 * option's default is automatic and is what the measurements in the repository
 * were taken with; the other settings exist to compare against.  Names:
 *  "reset"              every option back to its default (the value is ignored).
 *  "copy.nontemporal"   0/1 (default 1): streaming cache policy on loads and stores.
 *  "copy.order"         1: the (layer, K|V) plane is the outermost grid dimension;
 *                       0: consecutive workgroups walk the planes of one block;
 *                       -1 (default): 1 for layer-major pools (stride_kv >=
 *                       stride_block) and for kvm_pack, 0 for block-major pools.
 *  "copy.stage_linear"  bit 0: kvm_pack, bit 1: kvm_unpack assign work in staging
 *                       order (one 4 KiB piece of the staging buffer per workgroup)
 *                       instead of by pool block; -1 (default): kvm_pack does when
 *                       the batch's mean request moves 4096 tokens or more.
 *  "decode.mfma"        scores on the matrix cores (head_dim 128, 16-token blocks):
 *                       -1 (default) and 1: groups of four and of eight query
 *                       heads; 0 never.
 *  "decode.cap_waves"   -1 (default): the tuned decode kernels run at most two waves
 *                       per SIMD, with two tiles in flight, when the mean context per
 *                       workgroup is 12 blocks or more (the matrix-core kernel for
 *                       groups of four never does); 0 never, 1 always.
 *  "decode.spread"      log2 of the distance, in block-table entries, between the
 *                       four blocks the head_dim-128 decode kernels read in one step
 *                       (0..6; 0 = neighbouring entries); -1 (default): about 1 MiB of
 *                       pool memory when ids are consecutive.
 *  "decode.split_target" workgroups a decode launch should reach by splitting
 *                       contexts (default 2048).
 *  "decode.max_splits"  1..64 (default 16).
 *  "decode.force_splits" 0 = automatic, else exactly this many context splits.
 *
 * Thread safety of the library.  Options are process-wide and unsynchronised: set
 * them before other threads launch.  kvm_last_error() is per thread.  The size
 * helpers, kvm_layout_canonical, kvm_divide_moves and kvm_strerror are pure.
 * kvm_pack, kvm_unpack, kvm_migrate, kvm_paged_decode and kvm_paged_decode_rows keep
 * no state between calls and may run concurrently from several host threads and
 * on several streams; the device buffers they write must not overlap between
 * concurrent calls.  A kvm_freelist is not synchronised: one thread at a time per
 * list.  kvm_paged_decode_static is safe to call from several threads, but its
 * launches on one GPU must not overlap in time (they share the static array). */
int kvm_set_option(const char* name, int64_t value);

#ifdef __cplusplus
}
#endif
#endif /* KVM_H */
