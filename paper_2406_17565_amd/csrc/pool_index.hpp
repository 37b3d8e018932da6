// pool_index.hpp -- host control plane of one memory pool: block allocator, reference
// counts, and the prompt index keyed by chained block hashes.
//
// Paper: Table 1 (alloc_mem / free_mem / insert / match), Table 3 (evict), section 4.2
// (token-keyed radix tree at block granularity, nodes carry tier and instance id).
//
// Design (differs from the paper's Python radix tree on purpose): every indexed block has
// exactly one index node, so nodes live in flat arrays addressed by block id; the tree edges
// are "parent block id" fields; lookup goes through an open-addressing table from the
// 64-bit chained hash of a prefix to the block id.  A hit is accepted only if the parent
// link and the block's bs tokens match, so a hash collision degrades to a miss and answers
// are those of an exact token trie.  Evictable leaves sit in an ordered set keyed by
// (last_use, block id), so eviction is O(log n) per block.
#pragma once

#include <cstdint>
#include <cstring>
#include <set>
#include <utility>
#include <vector>

namespace mempool {

constexpr int32_t kNoBlock = -1;

class HashTable {  // hash -> block id, linear probing, backward-shift deletion
 public:
  void init(uint32_t n_blocks) {
    cap_ = 16;
    while (cap_ < 2ull * n_blocks) cap_ <<= 1;
    keys_.assign(cap_, 0);
    vals_.assign(cap_, kNoBlock);
  }
  int32_t find(uint64_t h) const {
    for (uint64_t s = slot(h);; s = (s + 1) & (cap_ - 1)) {
      if (vals_[s] == kNoBlock) return kNoBlock;
      if (keys_[s] == h) return vals_[s];
    }
  }
  void put(uint64_t h, int32_t b) {  // caller guarantees h is absent and the table is < 50 % full
    uint64_t s = slot(h);
    while (vals_[s] != kNoBlock) s = (s + 1) & (cap_ - 1);
    keys_[s] = h;
    vals_[s] = b;
    if (log_) log_->push_back((uint32_t)s);
  }
  void erase(uint64_t h) {
    uint64_t s = slot(h);
    while (vals_[s] != kNoBlock && keys_[s] != h) s = (s + 1) & (cap_ - 1);
    if (vals_[s] == kNoBlock) return;
    uint64_t hole = s;
    for (uint64_t j = (s + 1) & (cap_ - 1); vals_[j] != kNoBlock; j = (j + 1) & (cap_ - 1)) {
      uint64_t home = slot(keys_[j]);
      // can entry j move into the hole?  yes iff its home is not cyclically inside (hole, j]
      bool stays = (hole <= j) ? (home > hole && home <= j) : (home > hole || home <= j);
      if (!stays) {
        keys_[hole] = keys_[j];
        vals_[hole] = vals_[j];
        if (log_) log_->push_back((uint32_t)hole);
        hole = j;
      }
    }
    vals_[hole] = kNoBlock;
    if (log_) log_->push_back((uint32_t)hole);
  }

  // A device-side copy of the table is kept current by replaying the slots logged here.
  void set_log(std::vector<uint32_t> *log) { log_ = log; }
  uint64_t capacity() const { return cap_; }
  uint64_t key_at(uint64_t s) const { return keys_[s]; }
  int32_t val_at(uint64_t s) const { return vals_[s]; }
  const uint64_t *keys() const { return keys_.data(); }
  const int32_t *vals() const { return vals_.data(); }
  // home slot of a hash; the device probe uses the same function
  static uint64_t home(uint64_t h, uint64_t cap) { return (h ^ (h >> 32)) & (cap - 1); }

 private:
  uint64_t slot(uint64_t h) const { return home(h, cap_); }
  std::vector<uint32_t> *log_ = nullptr;
  uint64_t cap_ = 0;
  std::vector<uint64_t> keys_;
  std::vector<int32_t> vals_;
};

class PoolIndex {
 public:
  void init(uint32_t n_blocks, uint32_t block_size, uint32_t tier, uint32_t instance_id) {
    nb_ = n_blocks;
    bs_ = block_size;
    tier_ = tier;
    instance_ = instance_id;
    ref_.assign(nb_, 0);
    indexed_.assign(nb_, 0);
    parent_.assign(nb_, kNoBlock);
    n_children_.assign(nb_, 0);
    last_use_.assign(nb_, 0);
    hash_.assign(nb_, 0);
    node_tier_.assign(nb_, 0);
    node_instance_.assign(nb_, 0);
    in_lru_.assign(nb_, 0);
    mark_.assign(nb_, 0);
    lru_key_.assign(nb_, 0);
    lru_.clear();
    n_indexed_ = 0;
    clock_ = 0;
    tokens_.assign((size_t)nb_ * bs_, 0);
    table_.init(nb_);
    free_.clear();
    free_.reserve(nb_);
    for (int64_t b = (int64_t)nb_ - 1; b >= 0; --b) free_.push_back((int32_t)b);
  }

  // ---- queries -------------------------------------------------------------------------
  uint32_t n_blocks() const { return nb_; }
  uint32_t n_free() const { return (uint32_t)free_.size(); }
  uint32_t n_indexed() const { return n_indexed_; }
  uint64_t clock() const { return clock_; }
  bool in_range(int32_t b) const { return b >= 0 && (uint32_t)b < nb_; }
  bool is_free(int32_t b) const { return ref_[b] == 0 && !indexed_[b]; }
  uint32_t ref(int32_t b) const { return ref_[b]; }
  bool indexed(int32_t b) const { return indexed_[b] != 0; }
  uint32_t n_held() const {
    uint32_t c = 0;
    for (uint32_t b = 0; b < nb_; ++b) c += ref_[b] > 0;
    return c;
  }
  uint32_t n_historical() const {
    uint32_t c = 0;
    for (uint32_t b = 0; b < nb_; ++b) c += (indexed_[b] && ref_[b] == 0);
    return c;
  }

  // Number of index nodes that repeated leaf eviction could remove: nodes that are
  // unreferenced and have no referenced descendant.
  uint32_t evictable_total() const {
    std::vector<uint8_t> blocked(nb_, 0);
    uint32_t n_blocked = 0;
    for (uint32_t b = 0; b < nb_; ++b) {
      if (!indexed_[b] || ref_[b] == 0) continue;
      for (int32_t a = (int32_t)b; a != kNoBlock && !blocked[a]; a = parent_[a]) {
        blocked[a] = 1;
        ++n_blocked;
      }
    }
    return n_indexed_ - n_blocked;
  }

  // ---- allocator (LIFO) ----------------------------------------------------------------
  // Pops n ids; with `may_evict` first evicts exactly the shortfall.  false = cannot (no change).
  bool alloc(uint32_t n, int32_t *out, bool may_evict) {
    uint32_t nfree = n_free();
    if (nfree < n) {
      if (!may_evict) return false;
      // Every current unreferenced leaf can go, and an eviction removes at most one leaf from
      // that set (it may add the parent), so `shortfall` leaves at hand are enough; only
      // otherwise is the whole index counted.
      if (lru_.size() < n - nfree && nfree + evictable_total() < n) return false;
      evict(n - nfree);
    }
    for (uint32_t i = 0; i < n; ++i) {
      int32_t b = free_.back();
      free_.pop_back();
      ref_[b] = 1;
      out[i] = b;
    }
    return true;
  }

  // Drops one reference per listed id.  false = some id invalid (no change).
  bool release(const int32_t *blocks, uint32_t n) {
    uint32_t ok = 0;  // tentative decrements, undone below, validate multiplicities in O(n)
    for (; ok < n; ++ok) {
      if (!in_range(blocks[ok]) || ref_[blocks[ok]] == 0) break;
      --ref_[blocks[ok]];
    }
    for (uint32_t i = 0; i < ok; ++i) ++ref_[blocks[i]];
    if (ok < n) return false;
    for (uint32_t i = 0; i < n; ++i) {
      int32_t b = blocks[i];
      if (--ref_[b] == 0) {
        if (indexed_[b]) refresh_lru(b);
        else free_.push_back(b);
      }
    }
    return true;
  }

  void pin(int32_t b) {
    ++ref_[b];
    refresh_lru(b);
  }
  void unpin(int32_t b) {
    --ref_[b];
    refresh_lru(b);
  }

  // ---- index ---------------------------------------------------------------------------
  // Longest indexed prefix of the first nblk blocks.  hashes[i] = chained hash of blocks 0..i.
  uint32_t walk(const uint32_t *tokens, const uint64_t *hashes, uint32_t nblk,
                int32_t *blocks_out) const {
    int32_t parent = kNoBlock;
    uint32_t m = 0;
    for (; m < nblk; ++m) {
      int32_t b = table_.find(hashes[m]);
      if (b == kNoBlock || parent_[b] != parent ||
          std::memcmp(&tokens_[(size_t)b * bs_], tokens + (size_t)m * bs_, 4ull * bs_) != 0)
        break;
      if (blocks_out) blocks_out[m] = b;
      parent = b;
    }
    return m;
  }

  void tick() { ++clock_; }

  void touch(const int32_t *blocks, uint32_t n) {
    for (uint32_t i = 0; i < n; ++i) {
      last_use_[blocks[i]] = clock_;
      refresh_lru(blocks[i]);
    }
  }

  // Can blocks[m..nblk) become new nodes?  (held, not indexed, pairwise distinct)
  bool adoptable(const int32_t *blocks, uint32_t m, uint32_t nblk) {
    bool ok = true;
    uint32_t i = m;
    for (; i < nblk; ++i) {
      int32_t b = blocks[i];
      if (!in_range(b) || ref_[b] == 0 || indexed_[b] || mark_[b]) {
        ok = false;
        break;
      }
      mark_[b] = 1;
    }
    for (uint32_t j = m; j < i; ++j) mark_[blocks[j]] = 0;
    return ok;
  }

  // Are ids pairwise distinct, in range and referenced?  (explicit destination lists)
  bool held_and_distinct(const int32_t *blocks, uint32_t n) {
    bool ok = true;
    uint32_t i = 0;
    for (; i < n; ++i) {
      int32_t b = blocks[i];
      if (!in_range(b) || ref_[b] == 0 || mark_[b]) {
        ok = false;
        break;
      }
      mark_[b] = 1;
    }
    for (uint32_t j = 0; j < i; ++j) mark_[blocks[j]] = 0;
    return ok;
  }

  // Does any id of b[0..n) also occur in a[0..n)?  (ids already range-checked)
  bool lists_overlap(const int32_t *a, const int32_t *b, uint32_t n) {
    for (uint32_t i = 0; i < n; ++i) mark_[a[i]] = 1;
    bool hit = false;
    for (uint32_t i = 0; i < n && !hit; ++i) hit = mark_[b[i]] != 0;
    for (uint32_t i = 0; i < n; ++i) mark_[a[i]] = 0;
    return hit;
  }

  // Are ids in range and pairwise distinct?  (a scatter table; no reference needed)
  bool in_range_and_distinct(const int32_t *blocks, uint32_t n) {
    bool ok = true;
    uint32_t i = 0;
    for (; i < n; ++i) {
      int32_t b = blocks[i];
      if (!in_range(b) || mark_[b]) {
        ok = false;
        break;
      }
      mark_[b] = 1;
    }
    for (uint32_t j = 0; j < i; ++j) mark_[blocks[j]] = 0;
    return ok;
  }

  // insert proper: one clock tick, existing prefix touched, the rest adopted.  ids[i] is
  // ignored for blocks already present.  Returns the number of nodes created.
  uint32_t insert(const uint32_t *tokens, const uint64_t *hashes, uint32_t nblk,
                  const int32_t *ids) {
    tick();
    std::vector<int32_t> &path = scratch_path_;
    path.resize(nblk);
    uint32_t m = walk(tokens, hashes, nblk, path.data());
    touch(path.data(), m);
    int32_t parent = m ? path[m - 1] : kNoBlock;
    uint32_t created = 0;
    for (uint32_t i = m; i < nblk; ++i) {
      // A different prefix with the same 64-bit hash already sits in the table: this prompt's
      // remaining blocks stay un-indexed (a miss later, never wrong data).
      if (table_.find(hashes[i]) != kNoBlock) break;
      int32_t b = ids[i];
      indexed_[b] = 1;
      parent_[b] = parent;
      n_children_[b] = 0;
      hash_[b] = hashes[i];
      node_tier_[b] = tier_;
      node_instance_[b] = instance_;
      last_use_[b] = clock_;
      std::memcpy(&tokens_[(size_t)b * bs_], tokens + (size_t)i * bs_, 4ull * bs_);
      table_.put(hashes[i], b);
      if (mirror_log_) dirty_nodes_.push_back(b);
      ++n_indexed_;
      if (parent != kNoBlock) {
        ++n_children_[parent];
        refresh_lru(parent);
      }
      refresh_lru(b);
      parent = b;
      ++created;
    }
    return created;
  }

  // Least recently used unreferenced leaf first, ties by smallest block id.
  uint32_t evict(uint32_t k) {
    uint32_t done = 0;
    while (done < k && !lru_.empty()) {
      free_.push_back(unindex_victim());
      ++done;
    }
    return done;
  }

  // The block evict() would take next, or kNoBlock.
  int32_t next_victim() const { return lru_.empty() ? kNoBlock : lru_.begin()->second; }

  // Evicts next_victim() from the index but keeps the block out of the free list, held by one
  // reference: its bytes stay valid until the caller releases it (swap-out copies them first).
  int32_t evict_next_held() {
    const int32_t b = unindex_victim();
    ref_[b] = 1;
    return b;
  }

  // Block ids from the root of the tree down to indexed block b.
  void path_to(int32_t b, std::vector<int32_t> &out) const {
    out.clear();
    for (int32_t a = b; a != kNoBlock; a = parent_[a]) out.push_back(a);
    for (size_t i = 0, j = out.size(); i + 1 < j; ++i, --j) std::swap(out[i], out[j - 1]);
  }
  const uint32_t *tokens_of(int32_t b) const { return &tokens_[(size_t)b * bs_]; }
  uint64_t hash_of(int32_t b) const { return hash_[b]; }

  // delete: drop the prompt's own cached blocks -- from the deepest matched node upwards,
  // every node that is an unreferenced leaf; stops at the first node that is shared (has other
  // children) or referenced.  `path` = the matched blocks, root side first.
  uint32_t erase_path(const int32_t *path, uint32_t m) {
    uint32_t done = 0;
    for (uint32_t i = m; i-- > 0;) {
      const int32_t b = path[i];
      if (n_children_[b] != 0 || ref_[b] != 0) break;
      if (in_lru_[b]) {
        lru_.erase({lru_key_[b], b});
        in_lru_[b] = 0;
      }
      table_.erase(hash_[b]);
      indexed_[b] = 0;
      --n_indexed_;
      const int32_t par = parent_[b];
      parent_[b] = kNoBlock;
      if (par != kNoBlock) {
        --n_children_[par];
        refresh_lru(par);
      }
      free_.push_back(b);
      ++done;
    }
    return done;
  }

  // ---- change log for a device-resident copy of the index ------------------------------------
  void enable_mirror_log(bool on) {
    mirror_log_ = on;
    table_.set_log(on ? &dirty_slots_ : nullptr);
    dirty_slots_.clear();
    dirty_nodes_.clear();
  }
  const HashTable &table() const { return table_; }
  std::vector<uint32_t> &dirty_slots() { return dirty_slots_; }
  std::vector<int32_t> &dirty_nodes() { return dirty_nodes_; }
  const int32_t *parents() const { return parent_.data(); }
  const uint32_t *node_tokens() const { return tokens_.data(); }
  uint32_t block_size() const { return bs_; }

  uint32_t node_instance(int32_t b) const { return node_instance_[b]; }
  uint32_t node_tier(int32_t b) const { return node_tier_[b]; }

 private:
  // removes the least recently used unreferenced leaf from the index; the caller decides
  // where the block goes
  int32_t unindex_victim() {
    const int32_t b = lru_.begin()->second;
    lru_.erase(lru_.begin());
    in_lru_[b] = 0;
    table_.erase(hash_[b]);
    indexed_[b] = 0;
    --n_indexed_;
    const int32_t par = parent_[b];
    parent_[b] = kNoBlock;
    if (par != kNoBlock) {
      --n_children_[par];
      refresh_lru(par);
    }
    return b;
  }

  // keep `lru_` equal to { (last_use, b) : b indexed, unreferenced, childless }
  void refresh_lru(int32_t b) {
    if (in_lru_[b]) {
      lru_.erase({lru_key_[b], b});
      in_lru_[b] = 0;
    }
    if (indexed_[b] && ref_[b] == 0 && n_children_[b] == 0) {
      lru_key_[b] = last_use_[b];
      lru_.insert({last_use_[b], b});
      in_lru_[b] = 1;
    }
  }

  uint32_t nb_ = 0, bs_ = 0, tier_ = 0, instance_ = 0, n_indexed_ = 0;
  uint64_t clock_ = 0;
  std::vector<int32_t> free_;
  std::vector<uint32_t> ref_, n_children_, node_tier_, node_instance_;
  std::vector<uint8_t> indexed_, in_lru_, mark_;
  std::vector<int32_t> parent_;
  std::vector<uint64_t> last_use_, hash_, lru_key_;
  std::vector<uint32_t> tokens_;
  HashTable table_;
  std::set<std::pair<uint64_t, int32_t>> lru_;
  std::vector<int32_t> scratch_path_;
  bool mirror_log_ = false;
  std::vector<uint32_t> dirty_slots_;
  std::vector<int32_t> dirty_nodes_;
};

}  // namespace mempool
