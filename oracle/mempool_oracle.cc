// mempool_oracle.cc -- CPU oracle for the KV-block transfer / match path.
//
// TEST INFRASTRUCTURE ONLY: a slow, single-threaded, by-the-definition implementation that
// the GPU library is compared against.  It shares no code with that library.
//
// Sources in the MemServe paper:
//   * Table 1 (MemPool API): alloc_mem, free_mem, insert, match, delete, swap_out, swap_in,
//     transfer, transfer_with_insert; Table 3 adds evict.
//   * Section 4.2 (Indexing): a token-keyed radix tree whose nodes have the engine's block
//     granularity, may reference HBM or DRAM, and carry an instance id.  Written here as a
//     trie with one node per block of bs tokens.
//   * Section 4.3 (Distributed Transfer): allocation -> transmission -> insertion; an
//     explicit destination list skips allocation.
//   * Section 5.2: bs tokens occupy 2*L discrete blocks ("fragments" here), one K and one V
//     per layer; aggregation lays the 2*L fragments end to end in one block ("record").
//
// Conventions of this build where the paper is silent (each also implemented, separately,
// by the GPU library): LIFO free list; first writer wins on a duplicate prefix; eviction of
// the least recently used unreferenced leaf, ties by smallest block id; the chained block
// hash h_i = fmix64((h_{i-1} + G) xor FNV1a64(bytes of block i)).
#include "mempool_oracle.h"

#include <algorithm>
#include <cstring>
#include <map>
#include <set>
#include <vector>

namespace {

struct Node {
  Node *parent = nullptr;
  std::vector<uint32_t> key;  // the bs tokens of this block (edge label from the parent)
  std::map<std::vector<uint32_t>, Node *> children;
  int32_t block = -1;
  uint32_t tier = 0, instance_id = 0;
  uint64_t last_use = 0;
};

}  // namespace

struct orc_pool {
  uint32_t L, H, D, bs, e, NB, tier, instance_id;
  bool aggregated;  // [NB][L][2][F] instead of [L][2][NB][F]
  uint64_t seed;
  uint64_t F, B;
  uint8_t *base;
  std::vector<int32_t> free_stack;  // back() is popped next
  std::vector<uint32_t> ref;        // references per block
  std::vector<Node *> node_of;      // index node that owns the block, or null
  Node root;
  uint64_t clock = 0;
};

namespace {

bool is_free(const orc_pool *p, int32_t b) { return p->ref[b] == 0 && p->node_of[b] == nullptr; }
bool in_range(const orc_pool *p, int32_t b) { return b >= 0 && (uint32_t)b < p->NB; }

bool same_geometry(const orc_pool *a, const orc_pool *b) {
  return a->L == b->L && a->H == b->H && a->D == b->D && a->bs == b->bs && a->e == b->e;
}

std::vector<uint32_t> block_key(const orc_pool *p, const uint32_t *tokens, uint32_t i) {
  return std::vector<uint32_t>(tokens + (uint64_t)i * p->bs, tokens + (uint64_t)(i + 1) * p->bs);
}

// Walk the trie along the first `nblk` blocks of `tokens`; returns the nodes found, stopping
// at the first block that is absent.
std::vector<Node *> walk(orc_pool *p, const uint32_t *tokens, uint32_t nblk) {
  std::vector<Node *> path;
  Node *cur = &p->root;
  for (uint32_t i = 0; i < nblk; ++i) {
    auto it = cur->children.find(block_key(p, tokens, i));
    if (it == cur->children.end()) break;
    cur = it->second;
    path.push_back(cur);
  }
  return path;
}

// A node can eventually be evicted iff neither it nor any descendant is referenced.
bool subtree_unreferenced(const orc_pool *p, const Node *n, uint32_t *count) {
  bool all = true;
  for (auto &kv : n->children)
    if (!subtree_unreferenced(p, kv.second, count)) all = false;
  if (n->block >= 0) {  // not the root
    if (p->ref[n->block] != 0) all = false;
    if (all) ++*count;
  }
  return all;
}

uint32_t evictable_total(const orc_pool *p) {
  uint32_t c = 0;
  subtree_unreferenced(p, &p->root, &c);
  return c;
}

// The eviction rule: least recently used unreferenced leaf, ties by smallest block id.
Node *next_victim(const orc_pool *p) {
  Node *victim = nullptr;
  for (uint32_t b = 0; b < p->NB; ++b) {
    Node *n = p->node_of[b];
    if (!n || p->ref[b] != 0 || !n->children.empty()) continue;
    if (!victim || n->last_use < victim->last_use) victim = n;  // ascending b => ties keep smaller id
  }
  return victim;
}

// One eviction step.
bool evict_one(orc_pool *p) {
  Node *victim = next_victim(p);
  if (!victim) return false;
  victim->parent->children.erase(victim->key);
  p->node_of[victim->block] = nullptr;
  p->free_stack.push_back(victim->block);
  delete victim;
  return true;
}

// Would `insert` accept blocks[m..nb) as new nodes?  (held by the caller, not indexed,
// pairwise distinct)
int check_adoptable(const orc_pool *p, const int32_t *blocks, uint32_t m, uint32_t nb) {
  std::set<int32_t> seen;
  for (uint32_t i = m; i < nb; ++i) {
    int32_t b = blocks[i];
    if (!in_range(p, b) || p->ref[b] == 0 || p->node_of[b] != nullptr) return ORC_EINVAL;
    if (!seen.insert(b).second) return ORC_EINVAL;
  }
  return ORC_OK;
}

void delete_subtree(Node *n) {
  for (auto &kv : n->children) {
    delete_subtree(kv.second);
    delete kv.second;
  }
}

int check_src_ids(const orc_pool *p, const int32_t *ids, uint32_t n) {
  for (uint32_t i = 0; i < n; ++i)
    if (!in_range(p, ids[i]) || is_free(p, ids[i])) return ORC_EINVAL;
  return ORC_OK;
}

int check_given_dst_ids(const orc_pool *p, const int32_t *ids, uint32_t n) {
  std::set<int32_t> seen;
  for (uint32_t i = 0; i < n; ++i) {
    if (!in_range(p, ids[i]) || p->ref[ids[i]] == 0) return ORC_EINVAL;
    if (!seen.insert(ids[i]).second) return ORC_EINVAL;
  }
  return ORC_OK;
}

// Allocation with optional eviction of exactly the shortfall; all-or-nothing.
int alloc_blocks(orc_pool *p, uint32_t n, int32_t *out, uint32_t flags) {
  uint32_t nfree = (uint32_t)p->free_stack.size();
  if (nfree < n) {
    if (!(flags & ORC_EVICT_ON_DEMAND)) return ORC_ENOMEM;
    if (nfree + evictable_total(p) < n) return ORC_ENOMEM;
    for (uint32_t k = nfree; k < n; ++k) evict_one(p);
  }
  for (uint32_t i = 0; i < n; ++i) {
    int32_t b = p->free_stack.back();
    p->free_stack.pop_back();
    p->ref[b] = 1;
    out[i] = b;
  }
  return ORC_OK;
}

// The insertion step proper (already validated): first writer wins.
uint32_t do_insert(orc_pool *p, const uint32_t *tokens, uint32_t nb, const int32_t *blocks) {
  ++p->clock;
  uint32_t created = 0;
  Node *cur = &p->root;
  for (uint32_t i = 0; i < nb; ++i) {
    std::vector<uint32_t> key = block_key(p, tokens, i);
    auto it = cur->children.find(key);
    Node *n;
    if (it != cur->children.end()) {
      n = it->second;
    } else {
      n = new Node;
      n->parent = cur;
      n->key = key;
      n->block = blocks[i];
      n->tier = p->tier;
      n->instance_id = p->instance_id;
      cur->children[key] = n;
      p->node_of[blocks[i]] = n;
      ++created;
    }
    n->last_use = p->clock;
    cur = n;
  }
  return created;
}

// A transfer inside ONE pool reads its source blocks after the allocation step (section 4.3:
// allocation, then transmission), so the sources are in use for the whole call: they carry a
// reference while the destination blocks are found, and on-demand eviction cannot take a
// historical source block away (and hand it back as a destination).  Between two pools the
// source pool is not touched by the allocation, and nothing needs holding.
void hold_sources(orc_pool *src, const orc_pool *dst, const int32_t *ids, uint32_t n, int delta) {
  if (src != dst) return;
  for (uint32_t i = 0; i < n; ++i) src->ref[ids[i]] += delta;
}

void copy_all(const orc_pool *src, orc_pool *dst, const int32_t *s, const int32_t *d, uint32_t n) {
  std::vector<uint8_t> staging((size_t)n * src->B);
  orc_gather(src, s, n, staging.data());
  orc_scatter(dst, d, n, staging.data());
}

}  // namespace

extern "C" {

// ---- chained block hash ------------------------------------------------------------------
// Step 1: byte-wise FNV-1a-64 (offset basis 0xcbf29ce484222325, prime 0x100000001b3).
uint64_t orc_fnv1a64(const uint8_t *bytes, uint64_t n) {
  uint64_t a = 0xcbf29ce484222325ull;
  for (uint64_t i = 0; i < n; ++i) {
    a ^= (uint64_t)bytes[i];
    a *= 0x100000001b3ull;
  }
  return a;
}

// The splitmix64 output function.
uint64_t orc_fmix64(uint64_t x) {
  x ^= x >> 30;
  x *= 0xbf58476d1ce4e5b9ull;
  x ^= x >> 27;
  x *= 0x94d049bb133111ebull;
  x ^= x >> 31;
  return x;
}

// Step 2: h_i = fmix64((h_{i-1} + G) xor d_i), G = 0x9e3779b97f4a7c15.
uint64_t orc_chain_step(uint64_t h_prev, uint64_t digest) {
  return orc_fmix64((h_prev + 0x9e3779b97f4a7c15ull) ^ digest);
}

// Digest of one block: FNV-1a-64 over its 4*bs bytes, each token least-significant byte first.
uint64_t orc_block_digest(const uint32_t *t, uint32_t bs) {
  std::vector<uint8_t> bytes;
  for (uint32_t j = 0; j < bs; ++j)
    for (int k = 0; k < 4; ++k) bytes.push_back((uint8_t)((t[j] >> (8 * k)) & 0xffu));
  return orc_fnv1a64(bytes.data(), bytes.size());
}

// Step 3: only full blocks are hashed.
void orc_block_hashes(const uint32_t *tokens, uint32_t n_tokens, uint32_t bs, uint64_t seed,
                      uint64_t *out) {
  uint64_t h = seed;
  for (uint32_t i = 0; i < n_tokens / bs; ++i) {
    h = orc_chain_step(h, orc_block_digest(tokens + (uint64_t)i * bs, bs));
    out[i] = h;
  }
}

// ---- pool -------------------------------------------------------------------------------
orc_pool_t *orc_pool_create(uint32_t L, uint32_t H, uint32_t D, uint32_t bs, uint32_t e,
                            uint32_t NB, uint32_t tier, uint32_t instance_id, uint64_t seed,
                            uint8_t *base, uint32_t layout) {
  if (!L || !H || !D || !bs || !e || !NB || !base || tier > 1 || layout > 2) return nullptr;
  if (tier == ORC_TIER_HOST && layout == 1) return nullptr;  // a host pool is always aggregated
  orc_pool *p = new orc_pool;
  p->L = L; p->H = H; p->D = D; p->bs = bs; p->e = e; p->NB = NB;
  p->tier = tier; p->instance_id = instance_id; p->seed = seed; p->base = base;
  p->aggregated = layout == 2 || (layout == 0 && tier == ORC_TIER_HOST);
  p->F = (uint64_t)bs * H * D * e;
  p->B = 2ull * L * p->F;
  p->ref.assign(NB, 0);
  p->node_of.assign(NB, nullptr);
  for (int64_t b = (int64_t)NB - 1; b >= 0; --b) p->free_stack.push_back((int32_t)b);  // pops 0,1,2,...
  return p;
}

void orc_pool_destroy(orc_pool_t *p) {
  if (!p) return;
  delete_subtree(&p->root);
  delete p;
}

uint64_t orc_fragment_bytes(const orc_pool_t *p) { return p->F; }
uint64_t orc_record_bytes(const orc_pool_t *p) { return p->B; }

// Where fragment (l, kv, b) starts.  Discrete layout [L][2][NB][F] (the engine's own, two
// blocks per layer; default for HBM) or aggregated layout [NB][L][2][F] (one record per block,
// section 5.2; always for a host pool, optional for HBM).
uint64_t orc_fragment_offset(const orc_pool_t *p, uint32_t l, uint32_t kv, uint32_t b) {
  if (!p->aggregated) return (((uint64_t)l * 2 + kv) * p->NB + b) * p->F;
  return (((uint64_t)b * p->L + l) * 2 + kv) * p->F;
}

void orc_stats(const orc_pool_t *p, uint32_t *n_free, uint32_t *n_held, uint32_t *n_indexed,
               uint32_t *n_historical, uint64_t *clock) {
  uint32_t held = 0, idx = 0, hist = 0;
  for (uint32_t b = 0; b < p->NB; ++b) {
    if (p->ref[b] > 0) ++held;
    if (p->node_of[b]) ++idx;
    if (p->node_of[b] && p->ref[b] == 0) ++hist;
  }
  *n_free = (uint32_t)p->free_stack.size();
  *n_held = held; *n_indexed = idx; *n_historical = hist; *clock = p->clock;
}

// alloc_mem (Table 1: hands out blocks of the pool's memory type as an address list); the table's
// caption allows on-demand allocation, here: eviction of the shortfall when the flag asks.
int orc_alloc(orc_pool_t *p, uint32_t n, int32_t *out, uint32_t flags) {
  if (!p || (!out && n)) return ORC_EINVAL;
  return alloc_blocks(p, n, out, flags);
}

// free_mem (Table 1).  A block that the index still maps stays resident as historical KV
// (section 4.1: active vs historical cache) until it is evicted or deleted.
int orc_free(orc_pool_t *p, const int32_t *blocks, uint32_t n) {
  if (!p || (!blocks && n)) return ORC_EINVAL;
  std::map<int32_t, uint32_t> times;
  for (uint32_t i = 0; i < n; ++i) {
    if (!in_range(p, blocks[i])) return ORC_EINVAL;
    if (++times[blocks[i]] > p->ref[blocks[i]]) return ORC_EINVAL;
  }
  for (uint32_t i = 0; i < n; ++i) {
    int32_t b = blocks[i];
    if (--p->ref[b] == 0 && p->node_of[b] == nullptr) p->free_stack.push_back(b);
  }
  return ORC_OK;
}

// insert (Table 1: records, in the local index, which blocks hold the KV of the prompt's tokens);
// granularity = the engine's block (section 4.2, last paragraph).
int orc_insert(orc_pool_t *p, const uint32_t *tokens, uint32_t n_tokens, const int32_t *blocks,
               uint32_t n_blocks, uint32_t *n_new) {
  if (!p || (!tokens && n_tokens) || !n_new) return ORC_EINVAL;
  uint32_t nb = n_tokens / p->bs;  // only full blocks are indexed
  if (n_blocks < nb || (!blocks && nb)) return ORC_EINVAL;
  uint32_t m = (uint32_t)walk(p, tokens, nb).size();
  int rc = check_adoptable(p, blocks, m, nb);
  if (rc != ORC_OK) return rc;
  *n_new = do_insert(p, tokens, nb, blocks);
  return ORC_OK;
}

// match (Table 1: returns the addresses of the prompt's cached KV, if there is any): the longest indexed
// block-aligned prefix.
int orc_match(orc_pool_t *p, const uint32_t *tokens, uint32_t n_tokens, int32_t *blocks_out,
              uint32_t cap, uint32_t *n_matched, uint32_t flags) {
  if (!p || (!tokens && n_tokens) || !n_matched || (!blocks_out && cap)) return ORC_EINVAL;
  uint32_t nb = n_tokens / p->bs;
  if (nb > cap) nb = cap;
  ++p->clock;
  std::vector<Node *> path = walk(p, tokens, nb);
  for (size_t i = 0; i < path.size(); ++i) {
    path[i]->last_use = p->clock;
    blocks_out[i] = path[i]->block;
    if (flags & ORC_MATCH_PIN) ++p->ref[path[i]->block];
  }
  *n_matched = (uint32_t)path.size();
  return ORC_OK;
}

// delete (Table 1: drops the prompt's cached KV, if there is any).  The paper says no more; reading:
// the prompt's own blocks go, shared or referenced ones stay -- from the deepest matched node
// upwards, remove nodes while they are unreferenced leaves.
int orc_delete(orc_pool_t *p, const uint32_t *tokens, uint32_t n_tokens, uint32_t *n_deleted) {
  if (!p || (!tokens && n_tokens) || !n_deleted) return ORC_EINVAL;
  std::vector<Node *> path = walk(p, tokens, n_tokens / p->bs);
  uint32_t done = 0;
  while (!path.empty()) {
    Node *n = path.back();
    if (!n->children.empty() || p->ref[n->block] != 0) break;
    path.pop_back();
    n->parent->children.erase(n->key);
    p->node_of[n->block] = nullptr;
    p->free_stack.push_back(n->block);
    delete n;
    ++done;
  }
  *n_deleted = done;
  return ORC_OK;
}

// evict (named among the index APIs in Table 3 only; the policy is this build's convention).
int orc_evict(orc_pool_t *p, uint32_t k, uint32_t *n_evicted) {
  if (!p || !n_evicted) return ORC_EINVAL;
  uint32_t done = 0;
  while (done < k && evict_one(p)) ++done;
  *n_evicted = done;
  return ORC_OK;
}

// ---- copy by block table (section 5.2: 2*L fragments <-> one aggregated record) ----------
int orc_gather(const orc_pool_t *p, const int32_t *tbl, uint32_t n, uint8_t *staging) {
  for (uint32_t i = 0; i < n; ++i)
    for (uint32_t l = 0; l < p->L; ++l)
      for (uint32_t kv = 0; kv < 2; ++kv)
        std::memcpy(staging + (((uint64_t)i * p->L + l) * 2 + kv) * p->F,
                    p->base + orc_fragment_offset(p, l, kv, (uint32_t)tbl[i]), p->F);
  return ORC_OK;
}

int orc_scatter(orc_pool_t *p, const int32_t *tbl, uint32_t n, const uint8_t *staging) {
  for (uint32_t i = 0; i < n; ++i)
    for (uint32_t l = 0; l < p->L; ++l)
      for (uint32_t kv = 0; kv < 2; ++kv)
        std::memcpy(p->base + orc_fragment_offset(p, l, kv, (uint32_t)tbl[i]),
                    staging + (((uint64_t)i * p->L + l) * 2 + kv) * p->F, p->F);
  return ORC_OK;
}

// ---- transfer (section 4.3: allocation, transmission, insertion) ------------------------
int orc_transfer(orc_pool_t *src, orc_pool_t *dst, const int32_t *src_blocks,
                 int32_t *dst_blocks, uint32_t n, uint32_t flags) {
  if (!src || !dst || ((!src_blocks || !dst_blocks) && n)) return ORC_EINVAL;
  if (!same_geometry(src, dst)) return ORC_ESHAPE;
  int rc = check_src_ids(src, src_blocks, n);
  if (rc != ORC_OK) return rc;
  if (flags & ORC_DST_GIVEN) {
    rc = check_given_dst_ids(dst, dst_blocks, n);
  } else {
    hold_sources(src, dst, src_blocks, n, +1);
    rc = alloc_blocks(dst, n, dst_blocks, flags);
    hold_sources(src, dst, src_blocks, n, -1);
  }
  if (rc != ORC_OK) return rc;
  copy_all(src, dst, src_blocks, dst_blocks, n);
  return ORC_OK;
}

// By-layer transfer (section 4.3, explicit destination list for layer-by-layer transmission;
// section 5.2, by-layer approach): only layers [l0, l1) of each listed block move.  All source
// fragments are read before any destination fragment is written.
int orc_transfer_layers(orc_pool_t *src, orc_pool_t *dst, const int32_t *src_blocks,
                        const int32_t *dst_blocks, uint32_t n, uint32_t l0, uint32_t l1) {
  if (!src || !dst || ((!src_blocks || !dst_blocks) && n)) return ORC_EINVAL;
  if (!same_geometry(src, dst)) return ORC_ESHAPE;
  if (l0 >= l1 || l1 > src->L) return ORC_EINVAL;
  int rc = check_src_ids(src, src_blocks, n);
  if (rc != ORC_OK) return rc;
  rc = check_given_dst_ids(dst, dst_blocks, n);
  if (rc != ORC_OK) return rc;
  std::vector<uint8_t> tmp((size_t)n * 2 * (l1 - l0) * src->F);
  size_t k = 0;
  for (uint32_t i = 0; i < n; ++i)
    for (uint32_t l = l0; l < l1; ++l)
      for (uint32_t kv = 0; kv < 2; ++kv, ++k)
        std::memcpy(&tmp[k * src->F],
                    src->base + orc_fragment_offset(src, l, kv, (uint32_t)src_blocks[i]), src->F);
  k = 0;
  for (uint32_t i = 0; i < n; ++i)
    for (uint32_t l = l0; l < l1; ++l)
      for (uint32_t kv = 0; kv < 2; ++kv, ++k)
        std::memcpy(dst->base + orc_fragment_offset(dst, l, kv, (uint32_t)dst_blocks[i]),
                    &tmp[k * src->F], src->F);
  return ORC_OK;
}

// transfer_with_insert (Table 1; section 4.3: after the data has arrived the receiver inserts
// the prompt into its own index, which saves a round trip).  Blocks [0, first_block) are the
// part of the prompt the receiver already holds (section 5.1: with a cache at the receiver only
// the new KV moves).
int orc_transfer_with_insert(orc_pool_t *src, orc_pool_t *dst, const uint32_t *tokens,
                             uint32_t n_tokens, uint32_t first_block,
                             const int32_t *src_blocks, int32_t *dst_blocks, uint32_t n,
                             uint32_t flags) {
  if (!src || !dst || (!tokens && n_tokens) || ((!src_blocks || !dst_blocks) && n))
    return ORC_EINVAL;
  if (!same_geometry(src, dst)) return ORC_ESHAPE;
  uint32_t nb = n_tokens / dst->bs;
  if (first_block > nb || (uint64_t)first_block + n < nb) return ORC_EINVAL;
  int rc = check_src_ids(src, src_blocks, n);
  if (rc != ORC_OK) return rc;
  if (flags & ORC_DST_GIVEN) {
    rc = check_given_dst_ids(dst, dst_blocks, n);
    if (rc != ORC_OK) return rc;
  }
  // the receiver must already index blocks [0, first_block)
  std::vector<Node *> path = walk(dst, tokens, nb);
  if (path.size() < first_block) return ORC_ESTALE;
  std::vector<int32_t> ids(std::max<uint32_t>(nb, first_block + n), -1);
  for (uint32_t i = 0; i < first_block; ++i) ids[i] = path[i]->block;
  if (flags & ORC_DST_GIVEN) {
    for (uint32_t i = 0; i < n; ++i) ids[first_block + i] = dst_blocks[i];
    rc = check_adoptable(dst, ids.data(), (uint32_t)path.size(), nb);
    if (rc != ORC_OK) return rc;
  }
  // keep the matched prefix safe from on-demand eviction while this call runs
  for (uint32_t i = 0; i < first_block; ++i) ++dst->ref[path[i]->block];
  if (!(flags & ORC_DST_GIVEN)) {
    hold_sources(src, dst, src_blocks, n, +1);
    rc = alloc_blocks(dst, n, dst_blocks, flags);
    hold_sources(src, dst, src_blocks, n, -1);
    if (rc != ORC_OK) {
      for (uint32_t i = 0; i < first_block; ++i) --dst->ref[path[i]->block];
      return rc;
    }
    for (uint32_t i = 0; i < n; ++i) ids[first_block + i] = dst_blocks[i];
  }
  copy_all(src, dst, src_blocks, dst_blocks, n);          // transmission
  do_insert(dst, tokens, nb, ids.data());                 // insertion, after all data is there
  for (uint32_t i = 0; i < first_block; ++i) --dst->ref[ids[i]];
  return ORC_OK;
}

// Batched form: validation and allocation for all requests up front (one eviction of the
// total shortfall), one copy, then one insert per request in order.
int orc_transfer_with_insert_batch(orc_pool_t *src, orc_pool_t *dst, const uint32_t *tokens,
                                   const uint32_t *tok_off, uint32_t n_req,
                                   const uint32_t *first_block, const int32_t *src_blocks,
                                   int32_t *dst_blocks, const uint32_t *blk_off,
                                   uint32_t flags) {
  if (!src || !dst || !tok_off || !blk_off || (!first_block && n_req)) return ORC_EINVAL;
  if (flags & ORC_DST_GIVEN) return ORC_EINVAL;
  if (!same_geometry(src, dst)) return ORC_ESHAPE;
  uint32_t total = blk_off[n_req];
  if ((!src_blocks || !dst_blocks) && total) return ORC_EINVAL;
  if (!tokens && tok_off[n_req]) return ORC_EINVAL;
  if (blk_off[0] != 0 || tok_off[0] != 0) return ORC_EINVAL;
  for (uint32_t r = 0; r < n_req; ++r) {
    if (tok_off[r + 1] < tok_off[r] || blk_off[r + 1] < blk_off[r]) return ORC_EINVAL;
    uint32_t nb = (tok_off[r + 1] - tok_off[r]) / dst->bs, n = blk_off[r + 1] - blk_off[r];
    if (first_block[r] > nb || (uint64_t)first_block[r] + n < nb) return ORC_EINVAL;
  }
  int rc = check_src_ids(src, src_blocks, total);
  if (rc != ORC_OK) return rc;
  std::vector<std::vector<Node *>> prefix(n_req);
  for (uint32_t r = 0; r < n_req; ++r) {
    prefix[r] = walk(dst, tokens + tok_off[r], first_block[r]);
    if (prefix[r].size() < first_block[r]) return ORC_ESTALE;
  }
  for (auto &pr : prefix) for (Node *nd : pr) ++dst->ref[nd->block];
  hold_sources(src, dst, src_blocks, total, +1);
  rc = alloc_blocks(dst, total, dst_blocks, flags);
  hold_sources(src, dst, src_blocks, total, -1);
  if (rc == ORC_OK) {
    copy_all(src, dst, src_blocks, dst_blocks, total);
    for (uint32_t r = 0; r < n_req; ++r) {
      uint32_t nb = (tok_off[r + 1] - tok_off[r]) / dst->bs, n = blk_off[r + 1] - blk_off[r];
      std::vector<int32_t> ids(std::max<uint32_t>(nb, first_block[r] + n), -1);
      for (uint32_t i = 0; i < first_block[r]; ++i) ids[i] = prefix[r][i]->block;
      for (uint32_t i = 0; i < n; ++i) ids[first_block[r] + i] = dst_blocks[blk_off[r] + i];
      do_insert(dst, tokens + tok_off[r], nb, ids.data());
    }
  }
  for (auto &pr : prefix) for (Node *nd : pr) --dst->ref[nd->block];
  return rc;
}

// ---- swap between the two tiers of one instance -------------------------------------------
// Table 1 names swap_out(num_blocks) and swap_in(addrList) and says no more; section 4.2 lets
// an index node point to HBM or DRAM.  Reading of this build: the two tiers are two pools with
// an index each; the lower tier's index stays closed under prefixes, so moving a block down
// means caching its whole prompt prefix below (copying what is missing), and the upper tier
// then forgets the block.  The prefix of a node is read off the trie: the edge labels from the
// root down to it.
namespace {
void prefix_of(const Node *n, std::vector<uint32_t> *tokens, std::vector<int32_t> *blocks) {
  std::vector<const Node *> chain;
  for (const Node *a = n; a->block >= 0; a = a->parent) chain.push_back(a);
  tokens->clear();
  blocks->clear();
  for (size_t i = chain.size(); i-- > 0;) {
    tokens->insert(tokens->end(), chain[i]->key.begin(), chain[i]->key.end());
    blocks->push_back(chain[i]->block);
  }
}

int check_tier_pair(const orc_pool *a, const orc_pool *b) {
  if (!a || !b || a == b) return ORC_EINVAL;
  if (!same_geometry(a, b)) return ORC_ESHAPE;
  if (a->tier == ORC_TIER_HOST && b->tier == ORC_TIER_HOST) return ORC_ESHAPE;
  if (a->seed != b->seed) return ORC_EINVAL;
  return ORC_OK;
}

// Cache the prefix (tokens, held in `from` under `blocks`) in `to`: transfer_with_insert of the
// part `to` lacks, new blocks released at once.  `known` remembers, for the rest of the call,
// which block of `to` caches each block of that prefix.
int cache_prefix(orc_pool *from, orc_pool *to, const std::vector<uint32_t> &tokens,
                 const std::vector<int32_t> &blocks, std::map<int32_t, int32_t> *known) {
  const uint32_t d = (uint32_t)blocks.size();
  const uint32_t m = (uint32_t)walk(to, tokens.data(), d).size();
  std::vector<int32_t> fresh(d - m + 1);
  int rc = orc_transfer_with_insert(from, to, tokens.data(), d * to->bs, m, blocks.data() + m,
                                    fresh.data(), d - m, ORC_EVICT_ON_DEMAND);
  if (rc != ORC_OK) return rc;
  rc = orc_free(to, fresh.data(), d - m);
  std::vector<Node *> there = walk(to, tokens.data(), d);
  for (uint32_t i = 0; i < d; ++i) (*known)[blocks[i]] = there[i]->block;
  return rc;
}
}  // namespace

// swap_out: the victims evict would take, in that order.  A victim whose prefix this call has
// not yet cached below is cached there first (one transfer_with_insert of the missing part);
// a victim lying on a prefix handled earlier in the same call needs nothing below.
int orc_swap_out(orc_pool_t *upper, orc_pool_t *lower, uint32_t num_blocks, uint32_t *n_swapped) {
  int rc = check_tier_pair(upper, lower);
  if (rc != ORC_OK) return rc;
  if (!n_swapped) return ORC_EINVAL;
  std::map<int32_t, int32_t> known;  // upper block -> lower block caching the same prefix block
  uint32_t done = 0;
  while (done < num_blocks) {
    Node *victim = next_victim(upper);
    if (!victim) break;
    if (!known.count(victim->block)) {
      std::vector<uint32_t> tokens;
      std::vector<int32_t> blocks;
      prefix_of(victim, &tokens, &blocks);
      rc = cache_prefix(upper, lower, tokens, blocks, &known);
      if (rc == ORC_ENOMEM) break;  // the lower tier is full of referenced data
      if (rc != ORC_OK) return rc;
    }
    evict_one(upper);  // nothing in `upper` changed meanwhile: removes `victim`
    ++done;
  }
  *n_swapped = done;
  return ORC_OK;
}

// swap_in: the call is one use of the lower tier (one clock tick).  Deepest prefix first; a
// listed block on a prefix handled earlier in the same call only gets its reference.
int orc_swap_in(orc_pool_t *lower, orc_pool_t *upper, const int32_t *lower_blocks, uint32_t n,
                int32_t *upper_blocks) {
  int rc = check_tier_pair(lower, upper);
  if (rc != ORC_OK) return rc;
  if ((!lower_blocks || !upper_blocks) && n) return ORC_EINVAL;
  std::vector<std::pair<uint32_t, uint32_t>> order;  // (depth, position)
  for (uint32_t i = 0; i < n; ++i) {
    if (!in_range(lower, lower_blocks[i]) || !lower->node_of[lower_blocks[i]]) return ORC_EINVAL;
    uint32_t depth = 0;
    for (const Node *a = lower->node_of[lower_blocks[i]]; a->block >= 0; a = a->parent) ++depth;
    order.push_back({depth, i});
  }
  if (n == 0) return ORC_OK;
  std::stable_sort(order.begin(), order.end(),
                   [](const std::pair<uint32_t, uint32_t> &a, const std::pair<uint32_t, uint32_t> &b) {
                     return a.first > b.first;
                   });
  ++lower->clock;
  std::map<int32_t, int32_t> known;  // lower block -> upper block caching the same prefix block
  std::vector<int32_t> taken;
  for (const auto &o : order) {
    const int32_t b = lower_blocks[o.second];
    if (!known.count(b)) {
      Node *node = lower->node_of[b];
      std::vector<uint32_t> tokens;
      std::vector<int32_t> blocks;
      prefix_of(node, &tokens, &blocks);
      for (Node *a = node; a->block >= 0; a = a->parent) a->last_use = lower->clock;
      rc = cache_prefix(lower, upper, tokens, blocks, &known);
      if (rc != ORC_OK) {
        orc_free(upper, taken.data(), (uint32_t)taken.size());
        return rc;
      }
    }
    const int32_t up = known[b];
    ++upper->ref[up];
    taken.push_back(up);
    upper_blocks[o.second] = up;
  }
  return ORC_OK;
}

}  // extern "C"
