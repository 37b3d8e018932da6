"""Host control plane of the library (allocator, hash-keyed index, eviction) against the
oracle's token trie, with no GPU: the chained hashes are supplied through the *_hashed entry
points.  Random operation sequences must give identical answers and identical pool statistics.
"""
import numpy as np
import pytest

from oracle import oracle as O
from paper_2406_17565_amd import mempool as M

BS = 4
GEOM = (2, 1, 8, BS, 2)


class Pair:
    """The same pool on both sides."""

    def __init__(self, NB, seed=0):
        self.NB = NB
        self.o = O.OraclePool(*GEOM, NB, seed=seed)
        self._buf = np.zeros(64, np.uint8)   # never dereferenced by the host-only calls
        base = (self._buf.ctypes.data + 15) // 16 * 16
        rc, self.g = M.mp_pool_create(*GEOM, NB, base, hash_seed=seed)
        assert rc == 0
        self.seed = seed

    def hashes(self, t):
        return O.block_hashes(t, BS, self.seed)

    def check_stats(self):
        rc, s = M.mp_pool_stats(self.g)
        assert rc == 0 and s == self.o.stats()

    def __del__(self):
        M.mp_pool_destroy(self.g)


def test_scripted_lifecycle():
    p = Pair(8)
    rc, a = M.mp_alloc(p.g, 3)
    assert (rc, a.tolist()) == (0, [0, 1, 2])
    assert M.mp_free(p.g, [2, 0]) == 0
    assert M.mp_alloc(p.g, 3)[1].tolist() == [0, 2, 3]
    assert M.mp_alloc(p.g, 5)[0] == M.MP_ENOMEM
    assert M.mp_free(p.g, [1, 1]) == M.MP_EINVAL
    assert M.mp_free(p.g, [7]) == M.MP_EINVAL and M.mp_free(p.g, [8]) == M.MP_EINVAL
    t = np.arange(2 * BS + 1, dtype=np.uint32)
    h = p.hashes(t)
    assert M.mp_insert_hashed(p.g, t, h, [0])[0] == M.MP_EINVAL
    assert M.mp_insert_hashed(p.g, t, h, [0, 5])[0] == M.MP_EINVAL      # 5 is free
    assert M.mp_insert_hashed(p.g, t, h, [0, 1]) == (0, 2)
    assert M.mp_match_hashed(p.g, t, h, 2)[1].tolist() == [0, 1]
    assert M.mp_match_hashed(p.g, t, h, 1)[1].tolist() == [0]
    # same hash, different tokens (a forged collision): must be a miss, never a wrong block
    t2 = t.copy()
    t2[0] += 1
    assert M.mp_match_hashed(p.g, t2, h, 2)[1].size == 0


@pytest.mark.parametrize("seed", range(6))
def test_random_sequences_match_the_oracle(seed):
    rng = np.random.default_rng(seed)
    NB = int(rng.integers(6, 40))
    p = Pair(NB, seed=seed)
    held = []          # ids we hold one reference on (same on both sides)
    prompts = []
    for step in range(400):
        op = rng.integers(0, 7)
        if op == 0:      # alloc
            n = int(rng.integers(0, 6))
            fl = M.MP_EVICT_ON_DEMAND if rng.integers(0, 2) else 0
            rc_g, a = M.mp_alloc(p.g, n, fl)
            rc_o, b = p.o.alloc(n, fl)
            assert rc_g == rc_o
            if rc_g == 0:
                assert a.tolist() == b.tolist()
                held += a.tolist()
        elif op == 1 and held:   # free a random subset (sometimes with an invalid id)
            k = int(rng.integers(1, min(len(held), 5) + 1))
            idx = rng.permutation(len(held))[:k]
            ids = [held[i] for i in idx]
            if rng.integers(0, 8) == 0:
                ids.append(int(rng.integers(NB, NB + 3)))
            rc_g, rc_o = M.mp_free(p.g, ids), p.o.free(ids)
            assert rc_g == rc_o
            if rc_g == 0:
                for i in sorted(idx.tolist(), reverse=True):
                    held.pop(i)
        elif op == 2:    # insert a prompt (often extending or repeating an earlier one)
            if prompts and rng.integers(0, 2):
                base = prompts[int(rng.integers(0, len(prompts)))]
                t = np.concatenate([base[: int(rng.integers(0, len(base) + 1))],
                                    rng.integers(0, 3, int(rng.integers(0, 3 * BS)), dtype=np.uint32)])
            else:
                t = rng.integers(0, 3, int(rng.integers(0, 5 * BS)), dtype=np.uint32)
            nb = len(t) // BS
            rc_g, a = M.mp_alloc(p.g, nb)
            rc_o, b = p.o.alloc(nb)
            assert rc_g == rc_o
            if rc_g != 0:
                continue
            assert a.tolist() == b.tolist()
            held += a.tolist()
            rg = M.mp_insert_hashed(p.g, t, p.hashes(t), a)
            ro = p.o.insert(t, a)
            assert rg == ro
            prompts.append(t)
        elif op == 3 and prompts:  # match, sometimes pinning
            base = prompts[int(rng.integers(0, len(prompts)))]
            t = np.concatenate([base, rng.integers(0, 3, int(rng.integers(0, BS + 2)), dtype=np.uint32)])
            cap = int(rng.integers(0, len(t) // BS + 2))
            fl = M.MP_MATCH_PIN if rng.integers(0, 3) == 0 else 0
            rc_g, a = M.mp_match_hashed(p.g, t, p.hashes(t), cap, fl)
            rc_o, b = p.o.match(t, cap, fl)
            assert rc_g == rc_o == 0 and a.tolist() == b.tolist()
            if fl:
                held += a.tolist()
        elif op == 4:    # evict
            k = int(rng.integers(0, 4))
            assert M.mp_evict(p.g, k) == p.o.evict(k)
        elif op == 5 and prompts:   # delete a stored prompt (or a prefix / extension of one)
            base = prompts[int(rng.integers(0, len(prompts)))]
            t = base[: int(rng.integers(0, len(base) + 1))] if rng.integers(0, 2) else base
            assert M.mp_delete_hashed(p.g, t, p.hashes(t)) == p.o.delete(t)
        p.check_stats()
    # drain: everything released and evicted leaves an empty pool on both sides
    assert M.mp_free(p.g, held) == p.o.free(held) == 0
    assert M.mp_evict(p.g, NB) == p.o.evict(NB)
    p.check_stats()
    assert M.mp_pool_stats(p.g)[1]["n_free"] == NB
    # and the free lists are in the same order
    assert M.mp_alloc(p.g, NB)[1].tolist() == p.o.alloc(NB)[1].tolist()


def test_swap_argument_checks_need_no_device():
    a, b = Pair(8), Pair(8)
    assert M.mp_swap_out(a.g, a.g, 1)[0] == M.MP_EINVAL                 # one pool is not two tiers
    assert M.mp_swap_out(a.g, None, 1)[0] == M.MP_EINVAL
    assert M.mp_swap_out(a.g, b.g, 4) == (0, 0)                         # nothing cached: nothing to move
    seeded = Pair(8, seed=5)
    assert M.mp_swap_out(a.g, seeded.g, 1)[0] == M.MP_EINVAL            # tiers of one instance share the seed
    buf = np.zeros(64, np.uint8)
    base = (buf.ctypes.data + 15) // 16 * 16
    rc, other = M.mp_pool_create(3, 1, 8, BS, 2, 8, base)
    assert rc == 0 and M.mp_swap_out(a.g, other, 1)[0] == M.MP_ESHAPE
    rc, h1 = M.mp_pool_create(*GEOM, 8, base, tier=M.MP_TIER_HOST_PINNED)
    rc, h2 = M.mp_pool_create(*GEOM, 8, base, tier=M.MP_TIER_HOST_PINNED)
    assert M.mp_swap_out(h1, h2, 1)[0] == M.MP_ESHAPE                   # host to host
    assert M.mp_swap_in(h1, a.g, [0])[0] == M.MP_EINVAL                 # block 0 of h1 is not indexed
    assert M.mp_swap_in(h1, a.g, [9])[0] == M.MP_EINVAL
    assert M.mp_swap_in(h1, a.g, [])[0] == 0
    for h in (other, h1, h2):
        M.mp_pool_destroy(h)
