// sanitize_driver.cc -- the CPU oracle and the library's host control plane (pool_index.hpp),
// side by side under AddressSanitizer + UndefinedBehaviorSanitizer.  Built and run by
// tests/test_sanitizers.py; no GPU, no Python in the loop.
//
// Part 1 drives one PoolIndex and one oracle pool through the same seeded random call
// sequence (alloc, free, insert, match with and without pin, evict, delete) and stops at the
// first answer that differs.  Part 2 pushes the oracle's data plane (gather / scatter /
// transfer, by-layer, transfer_with_insert with eviction, swap between two tiers) through
// random tables on exactly sized heap buffers, so any out-of-range memcpy trips the sanitizer.
#include <algorithm>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <random>
#include <vector>

#include "../oracle/mempool_oracle.h"
#include "../paper_2406_17565_amd/csrc/pool_index.hpp"

using mempool::PoolIndex;

namespace {

struct Rng {
  std::mt19937_64 g;
  explicit Rng(uint64_t s) : g(s) {}
  uint32_t below(uint32_t n) { return n ? (uint32_t)(g() % n) : 0; }
  bool coin() { return (g() & 1) != 0; }
};

#define REQUIRE(cond)                                                                  \
  do {                                                                                 \
    if (!(cond)) {                                                                     \
      std::printf("DIFFERS %s:%d  %s  (seed %llu, step %u)\n", __FILE__, __LINE__, #cond, \
                  (unsigned long long)seed, step);                                     \
      return false;                                                                    \
    }                                                                                  \
  } while (0)

bool same_counts(const PoolIndex &lib, const orc_pool_t *orc) {
  uint32_t nf, nh, ni, nhist;
  uint64_t clk;
  orc_stats(orc, &nf, &nh, &ni, &nhist, &clk);
  return lib.n_free() == nf && lib.n_held() == nh && lib.n_indexed() == ni &&
         lib.n_historical() == nhist && lib.clock() == clk;
}

// A prompt: a prefix of an earlier one (so prefixes are shared) plus a few fresh tokens from a
// tiny alphabet (so equal blocks turn up by chance as well).
std::vector<uint32_t> next_prompt(Rng &r, const std::vector<std::vector<uint32_t>> &seen, uint32_t bs) {
  std::vector<uint32_t> t;
  if (!seen.empty() && r.below(3)) {
    const std::vector<uint32_t> &b = seen[r.below((uint32_t)seen.size())];
    t.assign(b.begin(), b.begin() + r.below((uint32_t)b.size() + 1));
  }
  for (uint32_t k = r.below(4 * bs); k > 0; --k) t.push_back(r.below(3));
  return t;
}

bool control_plane_run(uint64_t seed) {
  Rng r(seed);
  unsigned step = 0;
  const uint32_t bs = 1 + r.below(5), nb_pool = 5 + r.below(60);
  std::vector<uint8_t> bytes(2ull * nb_pool * bs * 2);  // L=1, H=1, D=1, e=2
  orc_pool_t *orc = orc_pool_create(1, 1, 1, bs, 2, nb_pool, ORC_TIER_HBM, 7, seed, bytes.data(), 0);
  if (!orc) return false;
  PoolIndex lib;
  lib.init(nb_pool, bs, 0, 7);
  std::vector<int32_t> refs;  // one entry per reference the "caller" owns
  std::vector<std::vector<uint32_t>> seen;
  bool ok = [&]() {
    for (step = 0; step < 800; ++step) {
      const uint32_t op = r.below(8);
      if (op == 0) {  // alloc, sometimes with eviction on demand
        const uint32_t n = r.below(7);
        const bool ev = r.coin();
        std::vector<int32_t> a(n + 1, -7), b(n + 1, -7);
        const bool got = lib.alloc(n, a.data(), ev);
        const int rc = orc_alloc(orc, n, b.data(), ev ? ORC_EVICT_ON_DEMAND : 0);
        REQUIRE(got == (rc == ORC_OK));
        if (got) {
          REQUIRE(std::equal(a.begin(), a.begin() + n, b.begin()));
          refs.insert(refs.end(), a.begin(), a.begin() + n);
        }
      } else if (op == 1) {  // free a few references; now and then one id too many or out of range
        std::vector<int32_t> ids;
        for (uint32_t k = r.below(5); k > 0 && !refs.empty(); --k) {
          const uint32_t j = r.below((uint32_t)refs.size());
          ids.push_back(refs[j]);
          refs.erase(refs.begin() + j);
        }
        const uint32_t spoil = r.below(10);
        if (spoil == 0) ids.push_back((int32_t)(nb_pool + r.below(3)));
        if (spoil == 1) ids.push_back(-1);
        const bool got = lib.release(ids.data(), (uint32_t)ids.size());
        const int rc = orc_free(orc, ids.data(), (uint32_t)ids.size());
        REQUIRE(got == (rc == ORC_OK));
        if (!got) {
          ids.pop_back();
          refs.insert(refs.end(), ids.begin(), ids.end());
        }
      } else if (op <= 4) {  // insert (2), match (3), match + pin (4)
        std::vector<uint32_t> t = next_prompt(r, seen, bs);
        const uint32_t nblk = (uint32_t)t.size() / bs;
        std::vector<uint64_t> h(nblk + 1);
        orc_block_hashes(t.data(), (uint32_t)t.size(), bs, seed, h.data());
        if (op == 2) {
          std::vector<int32_t> a(nblk + 1), b(nblk + 1);
          const bool got = lib.alloc(nblk, a.data(), false);
          REQUIRE(got == (orc_alloc(orc, nblk, b.data(), 0) == ORC_OK));
          if (!got) continue;
          REQUIRE(std::equal(a.begin(), a.begin() + nblk, b.begin()));
          refs.insert(refs.end(), a.begin(), a.begin() + nblk);
          const uint32_t m = lib.walk(t.data(), h.data(), nblk, nullptr);
          REQUIRE(lib.adoptable(a.data(), m, nblk));
          uint32_t made_o = 0;
          const uint32_t made = lib.insert(t.data(), h.data(), nblk, a.data());
          REQUIRE(orc_insert(orc, t.data(), (uint32_t)t.size(), b.data(), nblk, &made_o) == ORC_OK);
          REQUIRE(made == made_o);
          seen.push_back(t);
        } else {
          const bool pin = op == 4;
          const uint32_t cap = r.coin() ? nblk : r.below(nblk + 1);
          std::vector<int32_t> a(cap + 1, -7), b(cap + 1, -7);
          uint32_t m_o = 0;
          lib.tick();
          const uint32_t m = lib.walk(t.data(), h.data(), std::min(nblk, cap), a.data());
          lib.touch(a.data(), m);
          if (pin)
            for (uint32_t i = 0; i < m; ++i) lib.pin(a[i]);
          REQUIRE(orc_match(orc, t.data(), (uint32_t)t.size(), b.data(), cap, &m_o,
                            pin ? ORC_MATCH_PIN : 0) == ORC_OK);
          REQUIRE(m == m_o && std::equal(a.begin(), a.begin() + m, b.begin()));
          if (pin) refs.insert(refs.end(), a.begin(), a.begin() + m);
        }
      } else if (op == 5) {  // evict
        const uint32_t k = r.below(6);
        uint32_t done_o = 0;
        const int32_t victim = lib.next_victim();
        const uint32_t done = lib.evict(k);
        REQUIRE(orc_evict(orc, k, &done_o) == ORC_OK && done == done_o);
        REQUIRE(k == 0 || (done > 0) == (victim != mempool::kNoBlock));
      } else if (op == 6 && !seen.empty()) {  // delete a prompt seen before (or a stretch of it)
        std::vector<uint32_t> t = seen[r.below((uint32_t)seen.size())];
        t.resize(r.below((uint32_t)t.size() + 1));
        const uint32_t nblk = (uint32_t)t.size() / bs;
        std::vector<uint64_t> h(nblk + 1);
        orc_block_hashes(t.data(), (uint32_t)t.size(), bs, seed, h.data());
        std::vector<int32_t> path(nblk + 1);
        const uint32_t m = lib.walk(t.data(), h.data(), nblk, path.data());
        uint32_t gone_o = 0;
        const uint32_t gone = lib.erase_path(path.data(), m);
        REQUIRE(orc_delete(orc, t.data(), (uint32_t)t.size(), &gone_o) == ORC_OK && gone == gone_o);
      } else {  // list checks used by transfers: they must leave the mark array clean
        std::vector<int32_t> a, b;
        for (uint32_t k = r.below(6); k > 0; --k) {
          a.push_back((int32_t)r.below(nb_pool));
          b.push_back((int32_t)r.below(nb_pool));
        }
        bool want = false;
        for (int32_t x : b) want = want || std::find(a.begin(), a.end(), x) != a.end();
        REQUIRE(lib.lists_overlap(a.data(), b.data(), (uint32_t)a.size()) == want);
        std::vector<int32_t> s = b;
        std::sort(s.begin(), s.end());
        const bool distinct = std::adjacent_find(s.begin(), s.end()) == s.end();
        REQUIRE(lib.in_range_and_distinct(b.data(), (uint32_t)b.size()) == distinct);
        bool held = distinct;
        for (int32_t x : b) held = held && lib.ref(x) > 0;
        REQUIRE(lib.held_and_distinct(b.data(), (uint32_t)b.size()) == held);
      }
      REQUIRE(same_counts(lib, orc));
    }
    return true;
  }();
  orc_pool_destroy(orc);
  return ok;
}

// The oracle's data plane on heap buffers of the exact size.
bool data_plane_run(uint64_t seed) {
  Rng r(seed);
  unsigned step = 0;
  const uint32_t L = 1 + r.below(3), H = 1 + r.below(2), D = 8, bs = 1 + r.below(4), e = 1 + r.below(2);
  const uint32_t nb_a = 6 + r.below(20), nb_b = 6 + r.below(20), nb_h = 4 + r.below(12);
  const uint64_t F = (uint64_t)bs * H * D * e, B = 2ull * L * F;
  std::vector<uint8_t> mem_a(B * nb_a), mem_b(B * nb_b), mem_h(B * nb_h);
  for (auto *m : {&mem_a, &mem_b, &mem_h})
    for (uint8_t &x : *m) x = (uint8_t)r.below(256);
  orc_pool_t *a = orc_pool_create(L, H, D, bs, e, nb_a, ORC_TIER_HBM, 0, seed, mem_a.data(), r.below(3));
  orc_pool_t *b = orc_pool_create(L, H, D, bs, e, nb_b, ORC_TIER_HBM, 1, seed, mem_b.data(), r.below(3));
  orc_pool_t *h = orc_pool_create(L, H, D, bs, e, nb_h, ORC_TIER_HOST, 1, seed, mem_h.data(), 0);
  if (!a || !b || !h) return false;
  bool ok = [&]() {
    REQUIRE(orc_fragment_bytes(a) == F && orc_record_bytes(a) == B);
    std::vector<int32_t> all(nb_a);
    REQUIRE(orc_alloc(a, nb_a, all.data(), 0) == ORC_OK);
    for (step = 0; step < 60; ++step) {
      const uint32_t n = r.below(nb_a + 1);
      std::vector<int32_t> tbl(n + 1), out(n + 1, -7);
      for (uint32_t i = 0; i < n; ++i) tbl[i] = (int32_t)r.below(nb_a);
      const uint32_t op = r.below(5);
      if (op == 0) {  // gather, then scatter the records back under a permutation
        std::vector<uint8_t> staging(B * n);
        REQUIRE(orc_gather(a, tbl.data(), n, staging.data()) == ORC_OK);
        std::vector<int32_t> perm(nb_a);
        for (uint32_t i = 0; i < nb_a; ++i) perm[i] = (int32_t)i;
        std::shuffle(perm.begin(), perm.end(), r.g);
        REQUIRE(orc_scatter(a, perm.data(), std::min(n, nb_a), staging.data()) == ORC_OK);
      } else if (op == 1) {  // transfer with allocation at b (evicting), then give the blocks back
        const int rc = orc_transfer(a, b, tbl.data(), out.data(), n, ORC_EVICT_ON_DEMAND);
        REQUIRE(rc == ORC_OK || rc == ORC_ENOMEM);
        if (rc == ORC_OK) REQUIRE(orc_free(b, out.data(), n) == ORC_OK);
      } else if (op == 2) {  // by-layer into given destinations
        const uint32_t k = std::min(n, nb_b);
        const int rc = orc_alloc(b, k, out.data(), ORC_EVICT_ON_DEMAND);
        if (rc != ORC_OK) continue;
        const uint32_t l0 = r.below(L), l1 = l0 + 1 + r.below(L - l0);
        REQUIRE(orc_transfer_layers(a, b, tbl.data(), out.data(), k, l0, l1) == ORC_OK);
        REQUIRE(orc_free(b, out.data(), k) == ORC_OK);
      } else if (op == 3) {  // transfer_with_insert of a fresh prompt, blocks become historical
        const uint32_t k = std::min(n, nb_b / 2);
        std::vector<uint32_t> t((size_t)k * bs + r.below(bs));
        for (uint32_t &x : t) x = r.below(4);
        const uint32_t cover = ((uint32_t)t.size() + bs - 1) / bs;
        std::vector<int32_t> d(cover + 1, -7), s(tbl.begin(), tbl.begin() + std::min(cover, n));
        s.resize(cover, 0);
        const int rc = orc_transfer_with_insert(a, b, t.data(), (uint32_t)t.size(), 0, s.data(), d.data(),
                                                cover, ORC_EVICT_ON_DEMAND);
        REQUIRE(rc == ORC_OK || rc == ORC_ENOMEM);
        if (rc == ORC_OK) REQUIRE(orc_free(b, d.data(), cover) == ORC_OK);
      } else {  // move part of b's cache down to the host tier and bring one block back up
        uint32_t moved = 0;
        REQUIRE(orc_swap_out(b, h, 1 + r.below(4), &moved) == ORC_OK);
        for (int32_t id = 0; id < (int32_t)nb_h; ++id) {
          int32_t up = -7;
          const int rc = orc_swap_in(h, b, &id, 1, &up);  // ORC_EINVAL when id is not indexed below
          if (rc == ORC_OK) {
            REQUIRE(up >= 0 && (uint32_t)up < nb_b);
            REQUIRE(orc_free(b, &up, 1) == ORC_OK);
            break;
          }
          REQUIRE(rc == ORC_EINVAL || rc == ORC_ENOMEM);
        }
      }
    }
    return true;
  }();
  orc_pool_destroy(a);
  orc_pool_destroy(b);
  orc_pool_destroy(h);
  return ok;
}

}  // namespace

int main(int argc, char **argv) {
  const unsigned n_seeds = argc > 1 ? (unsigned)std::atoi(argv[1]) : 40;
  for (uint64_t seed = 0; seed < n_seeds; ++seed) {
    if (!control_plane_run(seed)) return 1;
    if (!data_plane_run(1000 + seed)) return 1;
  }
  std::printf("sanitize ok: %u control-plane and %u data-plane sequences\n", n_seeds, n_seeds);
  return 0;
}
