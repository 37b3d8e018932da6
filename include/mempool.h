/*
 * mempool.h -- C ABI of libmempool: MI355X-native movement of paged KV-cache blocks.
 *
 * The calls follow the Elastic Memory Pool API of the MemServe paper (Table 1:
 * alloc_mem, free_mem, insert, match, swap_out / swap_in, transfer, transfer_with_insert;
 * Table 3 adds evict).  Two "inference instances" of the paper are two pool handles in one
 * process, so the paper's destination instance id becomes a destination pool handle.
 *
 * GEOMETRY (paper section 5.2, "Memory and Network Optimization")
 *   L = n_layers, H = n_kv_heads, D = head_dim, bs = block_size (tokens), e = elem_bytes.
 *   fragment   : the KV of bs tokens for ONE layer and ONE of {K,V}: F = bs*H*D*e bytes,
 *                contiguous.  This is the engine's "block"; bs tokens need 2*L of them.
 *   record     : the 2*L fragments of one run of bs tokens laid end to end, B = 2*L*F bytes.
 *                This is the paper's aggregated block.
 *   discrete layout   : [L][2][NB][F] bytes; fragment (l,kv,b) starts at byte
 *                ((l*2+kv)*NB + b)*F of `base`.  The engine's native layout (two blocks per
 *                layer); the default for an HBM pool.
 *   aggregated layout : [NB][L][2][F] bytes; block b is the contiguous record at byte b*B of
 *                `base` (the paper's block aggregation).  Always used by a pinned-host pool;
 *                an HBM pool may opt in with MP_LAYOUT_AGGREGATED.
 *   staging    : [n][L][2][F] bytes, record i (the i-th entry of a block table) at i*B.
 *   F must be a multiple of 16 bytes.  The copy never looks inside a fragment.
 *
 * MEMORY OWNERSHIP
 *   The caller owns `base` and `staging` (for an HBM pool: device memory, e.g. a torch tensor's
 *   data_ptr; for a host pool: pinned host memory) and keeps them alive and 16-byte aligned
 *   until mp_pool_destroy.  The library owns the handle, the host-side index / free list /
 *   reference counts, small device + pinned buffers for block tables, tokens and hashes, one
 *   side stream for host-tier copies, one for hashing host-resident tokens, and a few events.  Every pointer argument of every call
 *   below is a HOST pointer unless its comment says "device".
 *
 * BLOCK LIFE CYCLE (paper section 4.1: active vs historical KV cache)
 *   FREE --mp_alloc--> held (ref = 1) --mp_insert--> held + indexed --mp_free--> ref - 1;
 *   at ref 0 an indexed block is HISTORICAL (evictable), a non-indexed one returns to FREE.
 *   mp_evict turns HISTORICAL leaf blocks into FREE ones.  mp_match(MP_MATCH_PIN) adds one
 *   reference per returned block (dropped again with mp_free).
 *   The free list is a LIFO stack: a fresh pool hands out 0,1,2,...; freed / evicted ids are
 *   pushed in the order they are released.
 *
 * ERRORS
 *   Every call returns MP_OK (0) or a negative code.  Calls are all-or-nothing: when a code
 *   other than MP_OK, MP_EHIP or MP_EHOST comes back, no pool byte, index entry, reference count or
 *   free-list entry has changed.  After MP_EHIP a transfer has handed freshly allocated
 *   destination blocks back to the free list (evictions made to find them are not undone) and
 *   pool bytes may be partly written.  mp_last_error(pool) returns a text for the last failure.
 *   A pool is bound to the device that is current at its first device call; keep that device
 *   current for every later call on the pool.
 *
 * THREADS AND STREAMS
 *   One thread at a time per pool.  Device work of a transfer is enqueued on the SOURCE pool's
 *   stream (the sender executes the transmission, paper section 4.3); hashing for
 *   match/insert of device-resident tokens (MP_TOKENS_ON_DEVICE), and whenever the device probe
 *   is on, runs on the stream of the pool whose index is consulted; host-resident tokens are
 *   hashed on a stream of the library's own and the call returns when the hashes are there,
 *   whatever is still queued on the pool's stream.  Without MP_ASYNC a
 *   call returns after its device work has completed.  With MP_ASYNC a transfer returns once
 *   its work is enqueued: destination ids and the index are already final, the bytes are valid
 *   in the order of the executing stream (the source pool's; the HBM pool's when the source is
 *   a host pool).  Until that work has run the caller must not free, evict or overwrite the
 *   blocks involved, and work on other streams that reads the destination must wait for it.
 */
#ifndef MEMPOOL_H
#define MEMPOOL_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct mp_pool mp_pool_t; /* opaque, library-owned */

/* memory "type" of Table 1 */
#define MP_TIER_HBM 0u
#define MP_TIER_HOST_PINNED 1u

/* pool memory layout (paper section 5.2: original discrete blocks vs aggregated blocks) */
#define MP_LAYOUT_DEFAULT 0u    /* discrete for an HBM pool, aggregated for a host pool */
#define MP_LAYOUT_DISCRETE 1u   /* HBM pools only */
#define MP_LAYOUT_AGGREGATED 2u

/* return codes */
#define MP_OK 0
#define MP_EINVAL (-1)     /* null pointer, id out of range, id not held, duplicate dst id, ... */
#define MP_ESHAPE (-2)     /* src / dst geometry differs (asymmetric parallelism unsupported) */
#define MP_ENOMEM (-3)     /* destination cannot supply the requested number of blocks */
#define MP_ENOSTAGING (-4) /* staging buffer missing or smaller than what the call needs */
#define MP_EHIP (-5)       /* a HIP runtime call failed */
#define MP_ESTALE (-6)     /* transfer_with_insert: blocks [0,first_block) not in dst index */
#define MP_EHOST (-7)      /* host memory allocation failed / internal error (state undefined) */

/* flags (bitmask) */
#define MP_DST_GIVEN 0x01u        /* caller supplies dst_blocks; allocation step skipped      */
#define MP_EVICT_ON_DEMAND 0x02u  /* allocation may evict historical blocks to make room      */
#define MP_ASYNC 0x04u            /* enqueue only; results valid in stream order              */
#define MP_MATCH_PIN 0x08u        /* mp_match: take one reference on every returned block     */
#define MP_TOKENS_ON_DEVICE 0x10u /* `tokens` is a device pointer (same device as the pool)   */
#define MP_PER_FRAGMENT 0x40u     /* reference point only: one copy-engine call per discrete
                                     fragment (2*L per block), the one-call-per-block pattern
                                     the paper measures as "Original" (sections 5.2, 8.4)     */
#define MP_DIRECT 0x20u           /* one fused kernel, no staging round trip; with a pinned-host
                                     pool at one end the kernel accesses host memory itself  */

typedef struct {
  uint32_t n_layers, n_kv_heads, head_dim, block_size, elem_bytes;
  uint32_t n_blocks;     /* NB */
  uint32_t tier;         /* MP_TIER_HBM or MP_TIER_HOST_PINNED */
  uint32_t instance_id;  /* kept in every index node (paper section 4.2, second extension) */
  uint64_t hash_seed;    /* h_{-1} of the chained block hash */
  void *base;            /* caller-owned pool memory, 2*L*NB*F bytes, 16-byte aligned */
  void *staging;         /* caller-owned DEVICE buffer for records; may be NULL */
  uint64_t staging_bytes;
  void *stream;          /* hipStream_t; NULL = the default stream */
  uint32_t layout;       /* MP_LAYOUT_* */
  uint32_t reserved;     /* must be 0 */
} mp_pool_desc_t;

typedef struct {
  uint32_t n_blocks, n_free, n_held, n_indexed, n_historical;
  uint64_t clock; /* logical LRU clock: +1 per index-touching call */
} mp_pool_stats_t;

/* Create / destroy a pool handle.  Never allocates or frees base / staging. */
int mp_pool_create(const mp_pool_desc_t *desc, mp_pool_t **out);
int mp_pool_destroy(mp_pool_t *p);
int mp_pool_stats(mp_pool_t *p, mp_pool_stats_t *out);
const char *mp_last_error(mp_pool_t *p); /* never NULL; valid until the next call on p */
const char *mp_strerror(int code);

/* alloc_mem / free_mem (Table 1, memory block APIs).  mp_alloc pops n ids (ref = 1 each);
 * with MP_EVICT_ON_DEMAND it first evicts exactly the shortfall.  MP_ENOMEM if impossible.
 * mp_free drops one reference per listed id (an id may be listed as often as it is
 * referenced); MP_EINVAL if an id is out of range or not referenced that often. */
int mp_alloc(mp_pool_t *p, uint32_t n, int32_t *blocks_out, uint32_t flags);
int mp_free(mp_pool_t *p, const int32_t *blocks, uint32_t n);

/* insert (Table 1): map each FULL block i < floor(n_tokens/bs) of the prompt to blocks[i].
 * A prefix that is already indexed keeps its existing block (first writer wins; blocks[i]
 * stays the caller's).  Blocks that get adopted must be held by the caller and not indexed
 * elsewhere.  n_blocks >= floor(n_tokens/bs).  *n_new_out = number of nodes created. */
int mp_insert(mp_pool_t *p, const uint32_t *tokens, uint32_t n_tokens, const int32_t *blocks,
              uint32_t n_blocks, uint32_t flags, uint32_t *n_new_out);

/* match (Table 1): longest indexed block-aligned prefix of the prompt, at most cap blocks.
 * Writes the m block ids to blocks_out and m to *n_matched_out. */
int mp_match(mp_pool_t *p, const uint32_t *tokens, uint32_t n_tokens, int32_t *blocks_out,
             uint32_t cap, uint32_t *n_matched_out, uint32_t flags);

/* delete (Table 1): delete the prompt's cached data, if any.  Walking up from the deepest
 * indexed block of the prompt, every node that is an unreferenced leaf is removed and its
 * block freed (deepest first); the walk stops at the first node that other prompts share
 * (it has other children) or that is referenced.  *n_deleted_out = blocks freed. */
int mp_delete(mp_pool_t *p, const uint32_t *tokens, uint32_t n_tokens, uint32_t flags,
              uint32_t *n_deleted_out);

/* evict (Table 3): up to n_blocks times, free the least recently used unreferenced LEAF of the
 * index (ties: smallest block id).  *n_evicted_out may be smaller than n_blocks. */
int mp_evict(mp_pool_t *p, uint32_t n_blocks, uint32_t *n_evicted_out);

/* transfer (Table 1, section 4.3): allocate n blocks at dst (unless MP_DST_GIVEN), then copy
 * block src_blocks[i] of src into block dst_blocks[i] of dst for all i (all 2*L fragments).
 * HBM->HBM: gather into src's staging, scatter from it (or one fused kernel with MP_DIRECT).
 * HBM->host: gather, then asynchronous device-to-host copies of records on the side stream
 *           (with MP_DIRECT: one kernel that stores straight into the mapped host pool).
 * host->HBM: host-to-device copies into dst's staging, then scatter (MP_DIRECT: one kernel
 *           that loads straight from the mapped host pool).  host->host is not supported.
 * Transfers larger than the staging buffer are cut into staging-sized rounds.
 * src ids must be held or historical; given dst ids must be held and duplicate-free.
 * Inside ONE pool (src == dst) the source blocks are held while the destination blocks are
 * allocated, so MP_EVICT_ON_DEMAND never evicts what the call is about to copy.
 * The entries may be copied in any order (the library sorts the pair of tables by destination
 * id before the launch); dst_blocks comes back in the caller's order.
 * priv / priv_len: opaque user data handed to the receiver callback, never sent to the GPU. */
int mp_transfer(mp_pool_t *src, mp_pool_t *dst, const int32_t *src_blocks,
                int32_t *dst_blocks /* in with MP_DST_GIVEN, else out */, uint32_t n,
                uint32_t flags, const void *priv, uint64_t priv_len);

/* transfer for n_req requests at once: request r owns entries blk_off[r] .. blk_off[r+1] of both
 * tables.  The data plane never needs the request boundaries (one launch covers the whole
 * table), so this is mp_transfer over blk_off[n_req] entries after the offsets are checked. */
int mp_transfer_batch(mp_pool_t *src, mp_pool_t *dst, const int32_t *src_blocks,
                      int32_t *dst_blocks, const uint32_t *blk_off, uint32_t n_req,
                      uint32_t flags);

/* By-layer transfer (section 4.3 names layer-by-layer transmission as the use of an explicit
 * destination list; section 5.2 compares by-layer with by-request): copies only
 * layers [layer_begin, layer_end) of every listed block, so an engine can ship a layer as soon
 * as its prefill finished.  The destination ids are always given (allocate them once with
 * mp_alloc before the first layer; insert with mp_insert after the last).  Staging holds packed
 * records of 2*(layer_end-layer_begin) fragments.  With a host-tier pool at one end MP_DIRECT
 * is required (else MP_ESHAPE). */
int mp_transfer_layers(mp_pool_t *src, mp_pool_t *dst, const int32_t *src_blocks,
                       const int32_t *dst_blocks, uint32_t n, uint32_t layer_begin,
                       uint32_t layer_end, uint32_t flags);

/* transfer_with_insert (Table 1, section 4.3): transfer, then the receiver inserts the prompt.
 * Blocks [0,first_block) of the prompt must already be in dst's index (else MP_ESTALE);
 * src_blocks / dst_blocks describe prompt blocks first_block .. first_block+n-1, and
 * first_block + n >= floor(n_tokens/bs).  A trailing partial block is copied, not indexed. */
int mp_transfer_with_insert(mp_pool_t *src, mp_pool_t *dst, const uint32_t *tokens,
                            uint32_t n_tokens, uint32_t first_block, const int32_t *src_blocks,
                            int32_t *dst_blocks, uint32_t n, uint32_t flags, const void *priv,
                            uint64_t priv_len);

/* Batched forms: n_req prompts concatenated in `tokens`, prompt r = tokens[tok_off[r] ..
 * tok_off[r+1]).  One hash launch / one copy launch per round for the whole batch. */
int mp_match_batch(mp_pool_t *p, const uint32_t *tokens, const uint32_t *tok_off,
                   uint32_t n_req, int32_t *blocks_out,
                   const uint32_t *blk_off /* n_req+1: slot range of request r in blocks_out */,
                   uint32_t *n_matched_out /* n_req */, uint32_t flags);
int mp_transfer_with_insert_batch(mp_pool_t *src, mp_pool_t *dst, const uint32_t *tokens,
                                  const uint32_t *tok_off, uint32_t n_req,
                                  const uint32_t *first_block /* n_req */,
                                  const int32_t *src_blocks, int32_t *dst_blocks,
                                  const uint32_t *blk_off /* n_req+1 into both tables */,
                                  uint32_t flags);

/* swap_out (Table 1: moves a given number of blocks from HBM down to DRAM; section 4.2: index
 * nodes may point to HBM or DRAM).  `upper` and `lower` are two pools of one instance (same
 * geometry and hash_seed, else MP_ESHAPE / MP_EINVAL), normally an HBM pool and a pinned-host
 * pool.  Up to num_blocks times: take the block mp_evict(upper) would take next (least recently
 * used unreferenced leaf); make sure its whole prompt prefix is cached in `lower` -- the part
 * `lower` lacks is copied there and indexed exactly as by mp_transfer_with_insert(upper ->
 * lower, that prefix, MP_EVICT_ON_DEMAND) followed by mp_free of the new lower blocks, so they
 * are historical at once; ancestors that stay cached in `upper` are then cached in both; a
 * victim that lies on a prefix handled earlier in the same call needs nothing below --; then
 * drop the block from upper's index and free it.  Cached data is never lost: whatever
 * matched in `upper` before still matches in `upper` or `lower` afterwards, unless `lower`
 * itself had to evict.  Stops early, without error, when `upper` has no victim left or `lower`
 * cannot supply blocks; *n_swapped_out = blocks freed in `upper` (their ids are pushed on the
 * free list in that order).  The copies of all victims share launches and have completed on
 * return (MP_ASYNC is ignored); MP_DIRECT selects the fused / zero-copy kernel.  After MP_EHIP
 * the cached content of `lower` is undefined. */
int mp_swap_out(mp_pool_t *upper, mp_pool_t *lower, uint32_t num_blocks, uint32_t flags,
                uint32_t *n_swapped_out);

/* swap_in (Table 1: brings the blocks at the given addresses from DRAM up to HBM; section 8.3:
 * historical KV that sits in DRAM is swapped into HBM before prefill uses it).  lower_blocks: n ids that
 * are indexed in `lower` (what mp_match(lower) returned).  The call is one use of the lower
 * tier (one clock tick).  For every id, deepest prefix first (ties: list order): unless the id
 * lies on a prefix handled earlier in the same call, its path is touched in `lower` and the
 * part of the prefix that `upper` lacks is copied up and indexed as by
 * mp_transfer_with_insert(lower -> upper, that prefix, MP_EVICT_ON_DEMAND) followed by mp_free
 * of the new blocks; then upper_blocks_out[i] = the block of `upper` that caches the same prefix
 * block, with ONE reference taken for the caller (release with mp_free).  Listing a whole
 * matched path therefore costs one copy and one index operation.  `lower` keeps its copy.  On MP_ENOMEM
 * (upper cannot supply blocks) the references taken so far are dropped again; blocks already
 * brought up stay cached. */
int mp_swap_in(mp_pool_t *lower, mp_pool_t *upper, const int32_t *lower_blocks, uint32_t n,
               int32_t *upper_blocks_out, uint32_t flags);

/* For callers that cannot allocate device memory -- code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc: mp_transfer with an explicit destination list between
 * two HBM pools that allocates nothing.  Where mp_transfer keeps the two block tables in
 * library-allocated device buffers, this call keeps them in a fixed array inside the library's
 * device image (2 * MP_STATIC_MAX_BLOCKS ids = 512 KiB on every GPU the library runs on, held
 * until the process ends); the call makes no hipMalloc / hipFree / hipHostMalloc, creates no
 * stream or event, and grows no host container.
 *   src_blocks, dst_blocks: n host ids each; source ids held or historical, destination ids
 *   held and distinct (as for mp_transfer with MP_DST_GIVEN).  n <= MP_STATIC_MAX_BLOCKS, else
 *   MP_EINVAL ("more than MP_STATIC_MAX_BLOCKS ..." in mp_last_error).
 *   flags: MP_DIRECT (one fused kernel) and MP_ASYNC; without MP_DIRECT the records go through
 *   src's staging buffer in rounds, as in mp_transfer.  Both pools must be HBM pools (MP_ESHAPE).
 *   The work runs on src's stream; the tables are uploaded on that stream too, so calls on one
 *   stream may follow each other without waiting.  Pageable host tables are read before the
 *   call returns; tables in pinned host memory must stay unchanged until the work has run.
 *   Every call on a GPU shares that GPU's one array: calls that overlap in time on DIFFERENT
 *   streams of one GPU race on it -- the caller orders them.
 *   No receiver callback, no kernel timing (both would allocate). */
#define MP_STATIC_MAX_BLOCKS 65536u
int mp_transfer_static(mp_pool_t *src, mp_pool_t *dst, const int32_t *src_blocks,
                       const int32_t *dst_blocks, uint32_t n, uint32_t flags);

/* Chained block hashes of one prompt (section 4.2 index key; the hash itself is this
 * library's convention): out[i] for i < floor(n_tokens/bs), computed by the device kernel. */
int mp_block_hashes(mp_pool_t *p, const uint32_t *tokens, uint32_t n_tokens, uint64_t *out,
                    uint32_t flags);

/* The same for n_req prompts in one kernel launch: prompt r's hashes are written back to back,
 * floor(len_r/bs) each, in request order. */
int mp_block_hashes_batch(mp_pool_t *p, const uint32_t *tokens, const uint32_t *tok_off,
                          uint32_t n_req, uint64_t *out, uint32_t flags);

/* Host-only forms of insert / match for callers that already hold the prompt's chained
 * hashes (e.g. computed once by mp_block_hashes where the request entered the cluster and
 * forwarded with it): hashes[i] for i < floor(n_tokens/bs).  No device work. */
int mp_insert_hashed(mp_pool_t *p, const uint32_t *tokens, uint32_t n_tokens,
                     const uint64_t *hashes, const int32_t *blocks, uint32_t n_blocks,
                     uint32_t flags, uint32_t *n_new_out);
int mp_match_hashed(mp_pool_t *p, const uint32_t *tokens, uint32_t n_tokens,
                    const uint64_t *hashes, int32_t *blocks_out, uint32_t cap,
                    uint32_t *n_matched_out, uint32_t flags);
int mp_delete_hashed(mp_pool_t *p, const uint32_t *tokens, uint32_t n_tokens,
                     const uint64_t *hashes, uint32_t *n_deleted_out);

/* The two data-plane steps of a transfer on their own (section 5.2: the 2*L discrete fragments
 * of a block <-> one aggregated record), exposed for tests and measurement.  mp_gather copies
 * block tbl[i] of the pool into record i of the pool's staging buffer; mp_scatter copies record
 * i into block tbl[i] (ids distinct).  `tbl`: HOST array of n ids; n records must fit the
 * staging buffer (MP_ENOSTAGING).  The record order is the table order (nothing is sorted).
 * With MP_ASYNC the work is only enqueued on the pool's stream. */
int mp_gather(mp_pool_t *p, const int32_t *tbl, uint32_t n, uint32_t flags);
int mp_scatter(mp_pool_t *p, const int32_t *tbl, uint32_t n, uint32_t flags);

/* Receiver callback for `priv` (paper: request id, sampling parameters, ...). */
typedef void (*mp_recv_cb)(void *user, const void *priv, uint64_t priv_len,
                           const int32_t *dst_blocks, uint32_t n);
int mp_set_recv_callback(mp_pool_t *p, mp_recv_cb cb, void *user);

/* Kernel timing with HIP events on the launch stream.  kind: 0 gather, 1 scatter, 2 direct,
 * 3 block_hash.  mp_profile_read synchronises, returns total ms and launch count since the
 * last read, and clears them. */
int mp_profile_enable(mp_pool_t *p, int on);
int mp_profile_read(mp_pool_t *p, int kind, double *total_ms_out, uint64_t *launches_out,
                    uint64_t *bytes_out);

/* Kernel launch-shape knobs (for tuning sweeps; defaults are chosen per geometry, and the
 * value -1 restores the default).
 * key: "order" (0 record-major, 1 plane-major), "plane_tile" (>0: that many planes of an
 * entry are walked together, rounded down to a divisor of the plane count -- all planes is
 * order 0, one plane is order 1; 0 = what "order" says), "unroll" (1,2,4,8), "wg_per_cu" (0 = one
 * workgroup per tile group, >0 = persistent grid of that many workgroups per CU),
 * "nontemporal" (0/1), "waves_per_wg" (1 or 4), "xcd_contiguous" (0/1: each XCD walks one
 * contiguous eighth of the work instead of every eighth workgroup), "item_limit" (>0: cap on
 * wave-items per launch, so a table is cut into several launches; 0 = 2^31-1),
 * "device_probe" (1: keep a copy of the index -- hash table, parent links, node tokens -- in
 * HBM and let mp_match / mp_match_batch walk it in a kernel right behind the hash kernel; the
 * host then only stamps, pins and copies out the result.  Same answers as the host walk.) */
int mp_set_tunable(mp_pool_t *p, const char *key, int value);

/* Calibration yardstick: one contiguous device-to-device copy of `bytes` (multiple of 16;
 * dst, src: DEVICE pointers) with the same per-lane load/store shape as the table-driven
 * copy, timed with HIP events on `stream`; synchronous.  Its time gives the copy ceiling of
 * the GPU at hand; its hardware-counter readings scale those of the real kernels. */
int mp_plain_copy(void *dst, const void *src, uint64_t bytes, void *stream, double *ms_out);

/* Host-only self check of internal integer work: the multiply-shift division used for the
 * work-item decomposition, and the sort of table pairs (both of its code paths).  Returns
 * MP_OK or MP_EINVAL. */
int mp_selftest(void);

#ifdef __cplusplus
}
#endif
#endif /* MEMPOOL_H */
