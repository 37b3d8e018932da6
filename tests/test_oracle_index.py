"""Pins for the oracle's allocator, prompt index (insert / match / evict) and the transfer
workflow of the paper's section 4.3 (allocate -> transmit -> insert)."""
import numpy as np

from oracle import oracle as O
from paper_2406_17565_amd import workloads as W

GEOM = (2, 1, 8, 4, 2)  # L, H, D, bs, e  -> F = 64 bytes
BS = 4


def pool(NB=32, seed=0, **kw):
    rng = np.random.default_rng(seed)
    L, H, D, bs, e = GEOM
    return O.OraclePool(*GEOM, NB, data=W.kv_bytes(rng, 2 * L * NB * bs * H * D * e), **kw)


# ---- allocator: LIFO stack ---------------------------------------------------------------
def test_allocator_script():
    p = pool(8)
    rc, a = p.alloc(3)
    assert rc == 0 and a.tolist() == [0, 1, 2]
    assert p.free([2, 0]) == 0                    # pushed in the order given: 2 then 0
    rc, b = p.alloc(3)
    assert b.tolist() == [0, 2, 3]                # 0 popped first (last pushed), then 2, then fresh 3
    assert p.stats()["n_free"] == 4 and p.stats()["n_held"] == 4
    rc, _ = p.alloc(5)
    assert rc == O.ENOMEM and p.stats()["n_free"] == 4       # all-or-nothing
    assert p.free([1, 1]) == O.EINVAL             # listed more often than referenced
    assert p.free([7]) == O.EINVAL                # free block
    assert p.free([8]) == O.EINVAL and p.free([-1]) == O.EINVAL
    assert p.stats()["n_held"] == 4
    rc, c = p.alloc(0)
    assert rc == 0 and c.size == 0


# ---- match == brute-force longest common block-aligned prefix ---------------------------
def _lcp_blocks(a, b):
    m = 0
    while (m + 1) * BS <= min(len(a), len(b)) and np.array_equal(a[m * BS:(m + 1) * BS],
                                                                 b[m * BS:(m + 1) * BS]):
        m += 1
    return m


def test_match_is_brute_force_lcp():
    rng = np.random.default_rng(42)
    for trial in range(40):
        p = pool(128, seed=trial)
        stored, ids = [], []
        for _ in range(rng.integers(1, 9)):
            n = int(rng.integers(0, 8 * BS + 1))
            t = rng.integers(0, 2, n, dtype=np.uint32)          # binary vocabulary: many shared prefixes
            rc, blk = p.alloc(n // BS)
            assert rc == 0
            rc, n_new = p.insert(t, blk)
            assert rc == 0
            # first writer wins: blocks created only past the longest prefix already stored
            known = max([_lcp_blocks(t, s) for s in stored], default=0)
            assert n_new == n // BS - known
            stored.append(t)
            ids.append(blk)
        for _ in range(10):
            q = rng.integers(0, 2, int(rng.integers(0, 9 * BS)), dtype=np.uint32)
            rc, got = p.match(q)
            assert rc == 0
            lcps = [_lcp_blocks(q, s) for s in stored]
            assert len(got) == max(lcps)
            for i, b in enumerate(got):   # each matched block belongs to the EARLIEST prompt with that prefix
                first = next(k for k, s in enumerate(stored) if _lcp_blocks(q, s) > i)
                assert b == ids[first][i]
            rc, capped = p.match(q, cap=1)
            assert len(capped) == min(1, max(lcps))


def test_insert_validation_and_first_writer_wins():
    p = pool(16)
    t = np.arange(3 * BS + 2, dtype=np.uint32)     # 3 full blocks + partial
    rc, a = p.alloc(4)
    assert p.insert(t, a[:2])[0] == O.EINVAL       # fewer ids than full blocks
    assert p.insert(t, [a[0], a[1], 9])[0] == O.EINVAL      # block 9 is free, not held
    assert p.insert(t, [a[0], a[1], a[1]])[0] == O.EINVAL   # duplicate among adopted
    assert p.stats()["n_indexed"] == 0
    assert p.insert(t, a) == (0, 3)                # partial block never indexed
    rc, b = p.alloc(3)
    assert p.insert(t, b) == (0, 0)                # same prompt again: nothing adopted
    assert p.match(t)[1].tolist() == a[:3].tolist()
    assert p.free(b) == 0 and p.stats()["n_free"] == 16 - 4
    t2 = t.copy()
    t2[2 * BS] += 1                                # diverges in block 2
    rc, c = p.alloc(3)
    assert p.insert(t2, [c[0], c[1], a[2]])[0] == O.EINVAL  # a[2] is indexed elsewhere
    assert p.insert(t2, c) == (0, 1)
    assert p.match(t2)[1].tolist() == [a[0], a[1], c[2]]


# ---- evict: least recently used unreferenced leaf, ties by smallest block id ---------------
def test_evict_script():
    p = pool(16)
    A = np.arange(0, 3 * BS, dtype=np.uint32)                   # blocks a0 a1 a2
    Bq = np.concatenate([A[:BS], np.arange(100, 100 + 2 * BS, dtype=np.uint32)])  # a0 b1 b2
    _, a = p.alloc(3)
    p.insert(A, a)            # clock 1: nodes 0,1,2
    _, b = p.alloc(3)         # ids 3,4,5; b[0] not adopted
    p.insert(Bq, b)           # clock 2: touches node 0, creates 4,5
    assert p.evict(1) == (0, 0)                                  # everything still referenced
    p.free(a)
    p.free(b)                                                    # block 3 returns to the free list
    st = p.stats()
    assert st["n_historical"] == 5 and st["n_free"] == 16 - 5
    p.match(A[:2 * BS])       # clock 3: touches nodes 0,1
    # leaves: 2 (last_use 1), 5 (last_use 2) -> 2 first; then 5; then leaves 1 (3) and 4 (2) -> 4; then 1; then 0
    order = []
    for _ in range(5):
        free_before = p.stats()["n_free"]
        assert p.evict(1) == (0, 1)
        assert p.stats()["n_free"] == free_before + 1
        rc, got = p.alloc(1)  # LIFO: the block just evicted comes back first
        order.append(int(got[0]))
    assert order == [2, 5, 4, 1, 0]
    assert p.evict(3) == (0, 0)
    assert p.stats()["n_indexed"] == 0


def test_evict_ties_and_pins():
    p = pool(16)
    t = np.arange(4 * BS, dtype=np.uint32)
    _, a = p.alloc(4)
    p.insert(t, a)
    u = np.arange(500, 500 + BS, dtype=np.uint32)
    _, c = p.alloc(1)
    p.insert(u, c)
    p.free(a)
    p.free(c)
    rc, m = p.match(t[:2 * BS], flags=O.MATCH_PIN)   # pins blocks 0,1
    assert m.tolist() == [0, 1]
    assert p.evict(10) == (0, 3)                     # 3, 2 (chain unwinds) and 4; never 0 / 1
    st = p.stats()
    assert st["n_indexed"] == 2 and st["n_held"] == 2
    assert p.match(t)[1].tolist() == [0, 1]          # index stays prefix-closed
    p.free(m)
    assert p.evict(10) == (0, 2)
    # two sibling leaves: the one matched longer ago goes first, whatever its block id
    q = pool(16)
    _, ids = q.alloc(3)
    x, y = np.full(BS, 7, np.uint32), np.full(BS, 8, np.uint32)
    q.insert(y, [ids[2]])
    q.insert(x, [ids[0]])
    q.free(ids)
    q.match(y)
    q.match(x)       # x more recent than y
    assert q.evict(1) == (0, 1)
    assert q.match(x)[1].size == 1 and q.match(y)[1].size == 0


def test_insert_refreshes_the_existing_prefix():
    p = pool(16)
    A = np.arange(2 * BS, dtype=np.uint32)
    Bq = np.arange(300, 300 + BS, dtype=np.uint32)
    _, a = p.alloc(2)
    p.insert(A, a)                 # clock 1
    _, b = p.alloc(1)
    p.insert(Bq, b)                # clock 2
    _, a2 = p.alloc(2)
    assert p.insert(A, a2) == (0, 0)   # clock 3: nothing new, but the A path was used again
    p.free(a)
    p.free(b)
    p.free(a2)
    assert p.evict(1) == (0, 1)
    assert p.match(Bq)[1].size == 0 and p.match(A)[1].size == 2


def test_delete_script():
    p = pool(16)
    A = np.arange(0, 3 * BS, dtype=np.uint32)                                     # a0 a1 a2
    Bq = np.concatenate([A[:BS], np.arange(100, 100 + 2 * BS, dtype=np.uint32)])  # a0 b1 b2
    _, a = p.alloc(3)
    p.insert(A, a)
    _, b = p.alloc(3)
    p.insert(Bq, b)                     # adopts b[1], b[2]
    assert p.delete(A) == (0, 0)        # still referenced: nothing goes
    p.free(a)
    p.free(b)
    free0 = p.stats()["n_free"]
    assert p.delete(A) == (0, 2)        # a2, a1 go; a0 is shared with Bq and stays
    assert p.stats()["n_free"] == free0 + 2
    assert p.alloc(2)[1].tolist() == [int(a[1]), int(a[2])]      # freed deepest first -> a1 on top
    assert p.match(A)[1].tolist() == [int(a[0])] and p.match(Bq)[1].size == 3
    assert p.delete(np.arange(900, 900 + BS, dtype=np.uint32)) == (0, 0)   # unknown prompt
    assert p.delete(Bq[: 2 * BS]) == (0, 0)   # its deepest matched node b1 has a child
    rc, pin = p.match(Bq[: 2 * BS], flags=O.MATCH_PIN)
    assert p.delete(Bq) == (0, 1)       # b2 goes, b1 is pinned
    p.free(pin)
    assert p.delete(Bq) == (0, 2)       # b1 and, no longer shared, a0
    assert p.stats()["n_indexed"] == 0


def test_evict_on_demand_is_all_or_nothing():
    p = pool(6)
    t = np.arange(4 * BS, dtype=np.uint32)
    _, a = p.alloc(4)
    p.insert(t, a)
    p.free(a[2:])                                   # blocks 2,3 historical; 0,1 still held
    assert p.alloc(5)[0] == O.ENOMEM                # 2 free + 2 evictable < 5 even with eviction
    assert p.alloc(5, O.EVICT_ON_DEMAND)[0] == O.ENOMEM
    assert p.stats()["n_indexed"] == 4              # nothing was evicted by the failed call
    rc, got = p.alloc(3, O.EVICT_ON_DEMAND)         # shortfall 1: evicts leaf 3 only
    assert rc == 0 and got.tolist() == [3, 4, 5]
    assert p.stats()["n_indexed"] == 3


# ---- transfer workflow --------------------------------------------------------------------
def _two_pools():
    src, dst = pool(32, seed=1), pool(24, seed=2)
    src.alloc(32)
    return src, dst


def test_transfer_with_insert_equals_transfer_then_insert():
    rng = np.random.default_rng(3)
    t = rng.integers(0, 1000, 5 * BS + 3, dtype=np.uint32)
    tbl = W.random_table(rng, 32, 6)               # 5 full blocks + the partial one
    src1, dst1 = _two_pools()
    rc, d1 = O.transfer_with_insert(src1, dst1, t, 0, tbl)
    assert rc == 0
    src2, dst2 = _two_pools()
    rc, d2 = O.transfer(src2, dst2, tbl)
    assert rc == 0
    assert dst2.insert(t, d2) == (0, 5)
    assert d1.tolist() == d2.tolist() == [0, 1, 2, 3, 4, 5]
    assert np.array_equal(dst1.data, dst2.data)
    assert dst1.stats() == dst2.stats()
    assert dst1.match(t)[1].tolist() == dst2.match(t)[1].tolist() == [0, 1, 2, 3, 4]
    assert np.array_equal(dst1.gather(d1), src1.gather(tbl))


def test_incremental_transfer_and_errors():
    rng = np.random.default_rng(4)
    src, dst = _two_pools()
    t1 = rng.integers(0, 1000, 3 * BS, dtype=np.uint32)
    t2 = np.concatenate([t1, rng.integers(0, 1000, 2 * BS + 1, dtype=np.uint32)])
    rc, d1 = O.transfer_with_insert(src, dst, t1, 0, [10, 11, 12])
    assert rc == 0
    rc, m = dst.match(t2, flags=O.MATCH_PIN)
    assert m.tolist() == d1.tolist()
    snap, st = dst.data.copy(), dst.stats()
    # wrong prefix claim: block 3 of t2 is not at dst
    assert O.transfer_with_insert(src, dst, t2, 4, [20, 21])[0] == O.ESTALE
    # too few blocks for the full blocks of the prompt
    assert O.transfer_with_insert(src, dst, t2, 3, [20])[0] == O.EINVAL
    assert O.transfer_with_insert(src, dst, t2, 6, [])[0] == O.EINVAL
    # source id out of range / dst given with duplicates / not held
    assert O.transfer_with_insert(src, dst, t2, 3, [20, 32, 22])[0] == O.EINVAL
    assert O.transfer(src, dst, [1, 2], [5, 5], flags=O.DST_GIVEN)[0] == O.EINVAL
    assert O.transfer(src, dst, [1, 2], [5, 6], flags=O.DST_GIVEN)[0] == O.EINVAL
    other = O.OraclePool(3, 1, 8, 4, 2, 8)
    assert O.transfer(src, other, [1], None)[0] == O.ESHAPE
    assert np.array_equal(dst.data, snap) and dst.stats() == st
    # only the new suffix moves (PD-Caching with a cache at the receiver): 2 full + 1 partial
    rc, d2 = O.transfer_with_insert(src, dst, t2, 3, [20, 21, 22])
    assert rc == 0 and d2.tolist() == [3, 4, 5]
    assert dst.match(t2)[1].tolist() == [0, 1, 2, 3, 4]
    assert np.array_equal(dst.gather(d2), src.gather([20, 21, 22]))


def test_transfer_with_insert_protects_its_prefix_from_eviction():
    src, dst = pool(32, seed=1), pool(6, seed=2)
    src.alloc(32)
    t1 = np.arange(3 * BS, dtype=np.uint32)
    t2 = np.concatenate([t1, np.arange(900, 900 + 3 * BS, dtype=np.uint32)])
    other = np.arange(700, 700 + 2 * BS, dtype=np.uint32)
    rc, d1 = O.transfer_with_insert(src, dst, t1, 0, [1, 2, 3])
    rc, d0 = O.transfer_with_insert(src, dst, other, 0, [4, 5])
    dst.free(d1)
    dst.free(d0)                                   # everything historical, 1 block free
    dst.match(other)                               # `other` is now the most recent
    rc, d2 = O.transfer_with_insert(src, dst, t2, 3, [6, 7, 8], flags=O.EVICT_ON_DEMAND)
    assert rc == 0                                 # must evict `other` (2 blocks), not t1's prefix
    assert dst.match(t2)[1].size == 6 and dst.match(other)[1].size == 0
    assert dst.stats()["n_held"] == 3              # the temporary pins are gone


def test_in_pool_transfer_holds_its_sources_while_it_allocates():
    """A transfer inside one pool (section 4.3: allocation first, transmission second) reads its
    sources after the destination blocks were found, so on-demand eviction must not take a
    historical SOURCE block -- else the block would come back as its own destination and its
    index entry would be lost.  Derived by hand from the rules: LRU leaf eviction, LIFO free
    list, sources referenced for the duration of the allocation."""
    A = np.arange(100, 100 + BS, dtype=np.uint32)           # two one-block prompts, cached and
    Bq = np.arange(200, 200 + BS, dtype=np.uint32)          # unreferenced (historical)
    p = pool(4, seed=3)
    for t in (A, Bq):
        rc, ids = p.alloc(1)
        assert rc == 0 and p.insert(t, ids) == (0, 1) and p.free(ids) == 0
    rc, held = p.alloc(2)                                    # the pool is full: 0,1 historical, 2,3 held
    assert rc == 0 and held.tolist() == [2, 3]
    before = p.data.copy()
    # both historical blocks are sources: nothing may be evicted, the call fails and changes nothing
    rc, _ = O.transfer(p, p, [0, 1], flags=O.EVICT_ON_DEMAND)
    assert rc == O.ENOMEM
    assert np.array_equal(p.data, before) and p.stats()["n_historical"] == 2
    assert p.match(A)[1].tolist() == [0] and p.match(Bq)[1].tolist() == [1]
    # one source: the OTHER historical block is the victim although the source is the older one
    rc, d = O.transfer(p, p, [0], flags=O.EVICT_ON_DEMAND)
    assert rc == 0 and d.tolist() == [1]
    F = p.F
    view = p.data.reshape(2 * GEOM[0], 4, F)
    assert np.array_equal(view[:, 1], before.reshape(2 * GEOM[0], 4, F)[:, 0])   # block 0 copied into 1
    assert p.match(A)[1].tolist() == [0] and p.match(Bq)[1].size == 0           # A survived, Bq was evicted
    assert p.stats()["n_held"] == 3 and p.free(d) == 0
    # the same through transfer_with_insert inside one pool
    q = pool(4, seed=4)
    for t in (A, Bq):
        rc, ids = q.alloc(1)
        assert q.insert(t, ids) == (0, 1) and q.free(ids) == 0
    q.alloc(2)
    C = np.arange(300, 300 + BS, dtype=np.uint32)
    rc, d = O.transfer_with_insert(q, q, C, 0, [0], flags=O.EVICT_ON_DEMAND)
    assert rc == 0 and d.tolist() == [1] and q.match(A)[1].tolist() == [0] and q.match(C)[1].tolist() == [1]
    # between two pools nothing is held: the source pool's references are untouched
    r1, r2 = pool(4, seed=5), pool(4, seed=6)
    rc, ids = r1.alloc(1)
    assert r1.insert(A, ids) == (0, 1) and r1.free(ids) == 0
    rc, d = O.transfer(r1, r2, [0], flags=O.EVICT_ON_DEMAND)
    assert rc == 0 and r1.stats()["n_held"] == 0 and r1.stats()["n_historical"] == 1


def test_batch_form():
    rng = np.random.default_rng(6)
    src, dst = _two_pools()
    shared = rng.integers(0, 1000, 2 * BS, dtype=np.uint32)
    prompts = [np.concatenate([shared, rng.integers(0, 1000, n, dtype=np.uint32)]) for n in (5, 9, 0)]
    toks, tok_off = W.csr(prompts)
    nblk = [(len(p) + BS - 1) // BS for p in prompts]
    tables = [W.random_table(rng, 32, n) for n in nblk]
    s, blk_off = W.csr(tables, np.int32)
    rc, d = O.transfer_with_insert_batch(src, dst, toks, tok_off, [0, 0, 0], s, blk_off)
    assert rc == 0 and d.tolist() == list(range(sum(nblk)))
    assert np.array_equal(dst.gather(d), src.gather(s))
    # first request wins the shared prefix; the others' copies stay un-indexed but held
    for r, p_ in enumerate(prompts):
        got = dst.match(p_)[1].tolist()
        full = len(p_) // BS
        own = d[blk_off[r]:blk_off[r + 1]].tolist()
        assert got == d[:2].tolist() + own[2:full]
    assert dst.stats()["n_indexed"] == 2 + sum(len(p_) // BS - 2 for p_ in prompts)
    assert O.transfer_with_insert_batch(src, dst, toks, tok_off, [0, 0, 0], s, blk_off,
                                        flags=O.DST_GIVEN)[0] == O.EINVAL


def test_tiny_config_walkthrough():
    """Config 1: 8 requests of 128 tokens sharing a 64-token prefix; match, then
    transfer_with_insert of the unmatched suffix, then match again."""
    g = W.CONFIGS[1]
    rng = np.random.default_rng(1)
    src = O.OraclePool(g.L, g.H, g.D, g.bs, g.e, g.NB, data=W.kv_bytes(rng, g.pool_bytes()))
    dst = O.OraclePool(g.L, g.H, g.D, g.bs, g.e, g.NB)
    src.alloc(g.NB)
    moved = []
    for t in W.tiny_requests():
        tbl = W.random_table(rng, g.NB, 8)
        rc, m = dst.match(t, flags=O.MATCH_PIN)
        rc, d = O.transfer_with_insert(src, dst, t, len(m), tbl[len(m):])
        assert rc == 0
        moved.append(len(d))
        rc, again = dst.match(t)
        assert again.tolist() == m.tolist() + d.tolist()
        assert np.array_equal(dst.gather(d), src.gather(tbl[len(m):]))
    assert moved == [8, 4, 4, 4, 4, 4, 4, 4]          # 36 blocks, 576 KiB
    assert sum(moved) * g.B == 576 * 1024
    assert dst.stats()["n_free"] == g.NB - 36


# ---- invariants that hold whatever the order of calls ------------------------------------------
def test_invariants_under_random_calls():
    """Properties the rules imply for ANY call sequence: every block is in exactly one of the
    states free / held / historical; evict frees exactly what it reports and nothing that is
    referenced; a pinned match stays matched; a match is never longer than the longest
    block-aligned prefix shared with some inserted prompt, and two prompts get the same ids on
    the prefix they share."""
    for seed in range(8):
        rng = np.random.default_rng(900 + seed)
        NB = 24
        p = pool(NB, seed)
        inserted, pinned = [], []          # prompts ever inserted; (prompt, ids) pinned matches
        held = []                          # id arrays this test still has to free
        for step in range(200):
            op = int(rng.integers(0, 6))
            st0 = p.stats()
            if op == 0:                                                   # insert a new prompt
                if inserted and rng.integers(0, 2):
                    base = inserted[int(rng.integers(0, len(inserted)))]
                    t = np.concatenate([base[: BS * int(rng.integers(0, len(base) // BS + 1))],
                                        rng.integers(0, 9, int(rng.integers(1, 3 * BS)), dtype=np.uint32)])
                else:
                    t = rng.integers(0, 9, int(rng.integers(0, 5 * BS)), dtype=np.uint32)
                rc, ids = p.alloc(len(t) // BS, flags=O.EVICT_ON_DEMAND)
                if rc == 0:
                    rc2, n_new = p.insert(t, ids)
                    assert rc2 == 0 and n_new <= len(ids)
                    inserted.append(t)
                    held.append(ids)
                else:
                    assert rc == O.ENOMEM and p.stats() == st0            # all or nothing
            elif op == 1 and held:                                        # a request finishes
                ids = held.pop(int(rng.integers(0, len(held))))
                assert p.free(ids) == 0
            elif op == 2:                                                 # evict
                k = int(rng.integers(0, 6))
                rc, e = p.evict(k)
                st = p.stats()
                assert rc == 0 and e <= k
                assert st["n_free"] == st0["n_free"] + e and st["n_indexed"] == st0["n_indexed"] - e
                assert st["n_held"] == st0["n_held"]
            elif op == 3 and inserted:                                    # match with a pin
                t = inserted[int(rng.integers(0, len(inserted)))]
                rc, m = p.match(t, flags=O.MATCH_PIN)
                assert rc == 0
                pinned.append((t, m))
                held.append(m)
            elif op == 4 and inserted:                                    # plain match, bounds
                t = inserted[int(rng.integers(0, len(inserted)))]
                q = np.concatenate([t, rng.integers(0, 9, BS, dtype=np.uint32)])
                rc, m = p.match(q)
                lcp = 0
                for s in inserted:
                    c, lim = 0, min(len(s), len(q)) // BS
                    while c < lim and np.array_equal(s[c * BS:(c + 1) * BS], q[c * BS:(c + 1) * BS]):
                        c += 1
                    lcp = max(lcp, c)
                assert rc == 0 and len(m) <= lcp
                assert len(set(m.tolist())) == len(m)
            elif op == 5 and len(inserted) >= 2:                          # shared prefixes share ids
                a = inserted[int(rng.integers(0, len(inserted)))]
                b = inserted[int(rng.integers(0, len(inserted)))]
                ma, mb = p.match(a)[1], p.match(b)[1]
                c = 0
                while c < min(len(ma), len(mb)) and np.array_equal(a[c * BS:(c + 1) * BS], b[c * BS:(c + 1) * BS]):
                    assert ma[c] == mb[c]
                    c += 1
            st = p.stats()
            assert st["n_free"] + st["n_held"] + st["n_historical"] == NB
            assert st["n_historical"] <= st["n_indexed"]
            for t, m in pinned:                                           # pins survive everything
                if any(m is h for h in held):
                    got = p.match(t)[1]
                    assert got[: len(m)].tolist() == m.tolist()
        for ids in held:
            assert p.free(ids) == 0
        rc, e = p.evict(NB)
        st = p.stats()
        assert st["n_indexed"] == 0 and st["n_free"] == NB and st["n_held"] == 0
