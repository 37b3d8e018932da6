/*
 * mempool_oracle.h -- C interface of the CPU oracle for the KV-block transfer / match path.
 *
 * TEST INFRASTRUCTURE ONLY.  A plain, single-threaded, obviously-correct statement of what
 * the GPU library must compute; it shares no code with that library.  Only tests, the smoke
 * check and the benchmark's cpu_baseline leg may use it.
 *
 * What is pinned, and to what (see tests/test_oracle_*.py):
 *   orc_gather / orc_scatter / orc_transfer : closed forms (permutation of an identity table,
 *       round-trip identity, untouched-block invariant), fragment counts of section 5.2.
 *   orc_transfer_layers : numpy slicing closed form; layer ranges that tile [0,L) add up to
 *       orc_transfer.
 *   orc_fnv1a64   : published FNV-1a-64 test vectors.
 *   orc_fmix64 / orc_chain_step : published splitmix64 outputs for seed 0.
 *   orc_block_hashes : composition of the two above, worked vectors under tests/golden/.
 *   orc_match / orc_insert : brute-force longest common block-aligned prefix on tiny inputs.
 *   orc_evict, orc_delete, orc_alloc / orc_free : scripted scenarios derived by hand from the rule.
 *   orc_swap_out / orc_swap_in : a scripted scenario, and invariants that hold whatever the
 *       conventions are -- no cached prefix is lost from the union of the two tiers, bytes are
 *       carried unchanged, the upper tier frees exactly the blocks evict would have freed.
 *   PARITY UNPINNED against the paper: the paper fixes neither a hash function, nor the
 *   allocation order, nor an eviction policy; those three are conventions of this build
 *   and are pinned only to their own written definitions.
 */
#ifndef MEMPOOL_ORACLE_H
#define MEMPOOL_ORACLE_H
#include <stdint.h>
#ifdef __cplusplus
extern "C" {
#endif

typedef struct orc_pool orc_pool_t;

/* same numeric interface values as the library's public header (a shared format) */
#define ORC_OK 0
#define ORC_EINVAL (-1)
#define ORC_ESHAPE (-2)
#define ORC_ENOMEM (-3)
#define ORC_ESTALE (-6)
#define ORC_TIER_HBM 0u
#define ORC_TIER_HOST 1u
#define ORC_DST_GIVEN 0x01u
#define ORC_EVICT_ON_DEMAND 0x02u
#define ORC_MATCH_PIN 0x08u

/* hash pieces */
uint64_t orc_fnv1a64(const uint8_t *bytes, uint64_t n);
uint64_t orc_fmix64(uint64_t x);
uint64_t orc_chain_step(uint64_t h_prev, uint64_t digest);
uint64_t orc_block_digest(const uint32_t *block_tokens, uint32_t bs);
void orc_block_hashes(const uint32_t *tokens, uint32_t n_tokens, uint32_t bs, uint64_t seed,
                      uint64_t *out /* floor(n_tokens/bs) */);

/* pool over caller-owned bytes `base` (2*L*NB*F bytes) */
orc_pool_t *orc_pool_create(uint32_t L, uint32_t H, uint32_t D, uint32_t bs, uint32_t e,
                            uint32_t NB, uint32_t tier, uint32_t instance_id, uint64_t seed,
                            uint8_t *base, uint32_t layout /* 0 default, 1 discrete, 2 aggregated */);
void orc_pool_destroy(orc_pool_t *p);
uint64_t orc_fragment_bytes(const orc_pool_t *p);
uint64_t orc_record_bytes(const orc_pool_t *p);
uint64_t orc_fragment_offset(const orc_pool_t *p, uint32_t l, uint32_t kv, uint32_t b);
void orc_stats(const orc_pool_t *p, uint32_t *n_free, uint32_t *n_held, uint32_t *n_indexed,
               uint32_t *n_historical, uint64_t *clock);

int orc_alloc(orc_pool_t *p, uint32_t n, int32_t *out, uint32_t flags);
int orc_free(orc_pool_t *p, const int32_t *blocks, uint32_t n);
int orc_insert(orc_pool_t *p, const uint32_t *tokens, uint32_t n_tokens, const int32_t *blocks,
               uint32_t n_blocks, uint32_t *n_new);
int orc_match(orc_pool_t *p, const uint32_t *tokens, uint32_t n_tokens, int32_t *blocks_out,
              uint32_t cap, uint32_t *n_matched, uint32_t flags);
int orc_evict(orc_pool_t *p, uint32_t k, uint32_t *n_evicted);
int orc_delete(orc_pool_t *p, const uint32_t *tokens, uint32_t n_tokens, uint32_t *n_deleted);

/* copy by block table; staging is [n][L][2][F] */
int orc_gather(const orc_pool_t *p, const int32_t *tbl, uint32_t n, uint8_t *staging);
int orc_scatter(orc_pool_t *p, const int32_t *tbl, uint32_t n, const uint8_t *staging);

int orc_transfer(orc_pool_t *src, orc_pool_t *dst, const int32_t *src_blocks,
                 int32_t *dst_blocks, uint32_t n, uint32_t flags);
int orc_transfer_layers(orc_pool_t *src, orc_pool_t *dst, const int32_t *src_blocks,
                        const int32_t *dst_blocks, uint32_t n, uint32_t l0, uint32_t l1);
int orc_transfer_with_insert(orc_pool_t *src, orc_pool_t *dst, const uint32_t *tokens,
                             uint32_t n_tokens, uint32_t first_block,
                             const int32_t *src_blocks, int32_t *dst_blocks, uint32_t n,
                             uint32_t flags);
int orc_transfer_with_insert_batch(orc_pool_t *src, orc_pool_t *dst, const uint32_t *tokens,
                                   const uint32_t *tok_off, uint32_t n_req,
                                   const uint32_t *first_block, const int32_t *src_blocks,
                                   int32_t *dst_blocks, const uint32_t *blk_off,
                                   uint32_t flags);
/* the two tiers of one instance: move cached blocks down (by the eviction order) / up */
int orc_swap_out(orc_pool_t *upper, orc_pool_t *lower, uint32_t num_blocks, uint32_t *n_swapped);
int orc_swap_in(orc_pool_t *lower, orc_pool_t *upper, const int32_t *lower_blocks, uint32_t n,
                int32_t *upper_blocks);
#ifdef __cplusplus
}
#endif
#endif
