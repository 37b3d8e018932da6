"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle -- bit-exact,
because the work is byte copies and integer hashes.  Sizes span several wave-items, several
staging rounds and ragged tails; the full-size configurations are in test_gpu_fullsize.py."""
import numpy as np
import pytest

from oracle import oracle as O
from paper_2406_17565_amd import workloads as W

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def gpu():
    if not torch.cuda.is_available():
        pytest.fail("no GPU visible: -m gpu tests need a real MI355X")
    from paper_2406_17565_amd import mempool as M
    from paper_2406_17565_amd.pool import TorchPool
    return M, TorchPool


GEOMS = {  # name: (L, H, D, bs, e)
    "tiny": (2, 2, 64, 16, 2),          # F = 4 KiB
    "f64": (3, 1, 8, 4, 2),             # F = 64 B: a fragment smaller than one wave-load
    "f480": (1, 5, 24, 2, 2),           # F = 480 B: multiple of 16, not of 64 -> ragged lanes
    "f32k": (4, 8, 128, 16, 2),         # F = 32 KiB (config 3's fragment), several chunks
    "f2560": (2, 5, 128, 2, 1),         # F = 1280 B with 1-byte elements
    "f20k": (3, 5, 128, 16, 1),         # F = 10 KiB: 2.5 wave-items at unroll 4
    "f16": (1, 1, 16, 1, 1),            # F = 16 B: one 16-byte vector per fragment, bs = 1
}


def make_pair(gpu, geom, NB, seed, staging_blocks, tier=0, hash_seed=0, layout=0):
    M, TorchPool = gpu
    L, H, D, bs, e = geom
    rng = np.random.default_rng(seed)
    data = W.kv_bytes(rng, 2 * L * NB * bs * H * D * e)
    o = O.OraclePool(*geom, NB, tier=tier, seed=hash_seed, data=data.copy(), layout=layout)
    g = TorchPool(*geom, NB, tier=tier, staging_blocks=staging_blocks, seed=hash_seed, layout=layout)
    g.load(data)
    return o, g


# ---- a1: chained block hash ------------------------------------------------------------------
@pytest.mark.parametrize("bs", [16, 32, 4, 1, 3, 40])
def test_block_hashes(gpu, bs):
    M, TorchPool = gpu
    geom = (1, 1, 8, bs, 2)
    rng = np.random.default_rng(bs)
    for seed in (0, 0x1234567890ABCDEF):
        p = TorchPool(*geom, 4, seed=seed)
        for n in [0, 1, bs - 1, bs, bs + 1, 3 * bs, 64 * bs, 65 * bs + 3, 1024 * bs, 1025 * bs + 1,
                  2500 * bs + 7]:
            t = rng.integers(0, 2**32, n, dtype=np.uint32)
            rc, h = M.mp_block_hashes(p.h, t, bs)
            assert rc == 0, M.mp_last_error(p.h)
            assert np.array_equal(h, O.block_hashes(t, bs, seed)), (bs, n)
            dt = torch.from_numpy(t.view(np.int32)).cuda()
            rc, h2 = M.mp_block_hashes(p.h, dt.data_ptr() if n else 0, bs, M.MP_TOKENS_ON_DEVICE,
                                       n_tokens=n)
            assert rc == 0 and np.array_equal(h2, h)
        p.close()


def test_block_hashes_batch(gpu):
    M, TorchPool = gpu
    bs = 16
    rng = np.random.default_rng(77)
    p = TorchPool(1, 1, 8, bs, 2, 4, seed=5)
    prompts = [rng.integers(0, 2**32, int(n), dtype=np.uint32)
               for n in (0, 5, 16, 700, 16 * 1030 + 9, 31, 4096)]
    toks, tok_off = W.csr(prompts)
    rc, h, hoff = M.mp_block_hashes_batch(p.h, toks, tok_off, bs)
    assert rc == 0
    for r, t in enumerate(prompts):
        assert np.array_equal(h[hoff[r]:hoff[r + 1]], O.block_hashes(t, bs, 5))
    p.close()


def test_block_hashes_of_many_prompts_in_a_row(gpu):
    """Thousands of prompts per launch, many of them empty or shorter than a block, then smaller
    batches on the same pool: every launch reports per prompt, and no report of an earlier launch
    may pass for a later one."""
    M, TorchPool = gpu
    bs = 8
    rng = np.random.default_rng(78)
    p = TorchPool(1, 1, 8, bs, 2, 4, seed=9)
    for n_req in (3000, 3000, 700, 1, 64, 2999):
        lens = rng.choice([0, 3, bs, 5 * bs + 1, 40 * bs, 130 * bs + 7], n_req, p=[.2, .1, .2, .3, .15, .05])
        prompts = [rng.integers(0, 2**32, int(n), dtype=np.uint32) for n in lens]
        toks, tok_off = W.csr(prompts)
        rc, h, hoff = M.mp_block_hashes_batch(p.h, toks, tok_off, bs)
        assert rc == 0, M.mp_last_error(p.h)
        want = np.concatenate([O.block_hashes(t, bs, 9) for t in prompts] + [np.zeros(0, np.uint64)])
        assert np.array_equal(h, want), n_req
    p.close()


def test_block_hashes_golden(gpu, golden_dir):
    M, TorchPool = gpu
    import os
    cases = {"arange48": np.arange(48), "zeros32": np.zeros(32), "arange64": np.arange(64),
             "arange16": np.arange(16)}
    for line in open(os.path.join(golden_dir, "block_hash_vectors.txt")):
        if line.startswith("#") or not line.strip():
            continue
        case, bs, seed, i, d, h = line.split()
        p = TorchPool(1, 1, 8, int(bs), 2, 4, seed=int(seed))
        rc, got = M.mp_block_hashes(p.h, cases[case].astype(np.uint32), int(bs))
        assert rc == 0 and int(got[int(i)]) == int(h, 16)
        p.close()


# ---- a5 / a6: gather and scatter ----------------------------------------------------------------
@pytest.mark.parametrize("name", list(GEOMS))
def test_gather_scatter_all_launch_shapes(gpu, name):
    M, TorchPool = gpu
    geom = GEOMS[name]
    NB, n = 61, 45
    o, g = make_pair(gpu, geom, NB, 1, staging_blocks=n)
    rng = np.random.default_rng(2)
    src_tbl = rng.integers(0, NB, n).astype(np.int32)      # duplicates allowed when reading
    dst_tbl = W.random_table(rng, NB, n)
    want_staging = o.gather(src_tbl)
    shapes = [(order, 0, u, wg, nt, w, xcd) for order in (0, 1) for u in (1, 2, 4, 8)
              for wg, nt, w, xcd in ((0, 1, 4, 0), (2, 0, 1, 1), (0, 1, 1, 1), (1, 1, 4, 1))]
    shapes += [(0, tile, 1, wg, 1, w, xcd) for tile in (2, 3, 4, 5, 64)    # 5 is rounded to a divisor
               for wg, w, xcd in ((0, 1, 1), (2, 4, 0))]
    for order, tile, u, wg, nt, w, xcd in shapes:
        for k, v in (("order", order), ("plane_tile", tile), ("unroll", u), ("wg_per_cu", wg),
                     ("nontemporal", nt), ("waves_per_wg", w), ("xcd_contiguous", xcd)):
            assert M.mp_set_tunable(g.h, k, v) == 0
        g.staging.zero_()
        assert M.mp_gather(g.h, src_tbl) == 0, M.mp_last_error(g.h)
        assert np.array_equal(g.staging_bytes(n), want_staging), (name, order, tile, u, wg, nt, w, xcd)
        # scatter the gathered records under a permuted table; oracle does the same
        o2 = O.OraclePool(*geom, NB, data=o.data.copy())
        o2.scatter(dst_tbl, want_staging)
        before = g.bytes()
        assert M.mp_scatter(g.h, dst_tbl) == 0
        assert np.array_equal(g.bytes(), o2.data), (name, order, tile, u, wg, nt, w, xcd)
        g.load(before)
    assert M.mp_gather(g.h, np.zeros(0, np.int32)) == 0
    assert M.mp_gather(g.h, [NB]) == M.MP_EINVAL
    assert M.mp_scatter(g.h, [1, 1]) == M.MP_EINVAL
    assert M.mp_gather(g.h, np.zeros(n + 1, np.int32)) == M.MP_ENOSTAGING
    g.close()


def test_tables_split_over_several_launches(gpu):
    """A table whose wave-item count exceeds the per-launch index range is cut into several
    launches; forced here with a tiny limit."""
    M, TorchPool = gpu
    geom = GEOMS["f20k"]
    NB, n = 50, 37
    o, g = make_pair(gpu, geom, NB, 11, staging_blocks=n)
    rng = np.random.default_rng(12)
    tbl = W.random_table(rng, NB, n)
    for limit, order in ((100, 0), (61, 1), (1, 0)):      # 60 items per entry at unroll 1
        assert M.mp_set_tunable(g.h, "item_limit", limit) == 0
        assert M.mp_set_tunable(g.h, "order", order) == 0
        g.staging.zero_()
        assert M.mp_gather(g.h, tbl) == 0
        assert np.array_equal(g.staging_bytes(n), o.gather(tbl)), limit
        o2 = O.OraclePool(*geom, NB, data=o.data.copy())
        dst_tbl = W.random_table(rng, NB, n)
        o2.scatter(dst_tbl, o.gather(tbl))
        before = g.bytes()
        assert M.mp_scatter(g.h, dst_tbl) == 0
        assert np.array_equal(g.bytes(), o2.data), limit
        g.load(before)
    g.close()


def test_special_bit_patterns_survive(gpu):
    M, TorchPool = gpu
    geom = GEOMS["tiny"]
    o, g = make_pair(gpu, geom, 8, 3, staging_blocks=8)
    o.data.reshape(geom[0], 2, 8, o.F)[:, :, 5, :] = W.special_half_patterns(o.F)
    g.load(o.data)
    tbl = np.array([5, 0, 5], np.int32)
    assert M.mp_gather(g.h, tbl) == 0
    assert np.array_equal(g.staging_bytes(3), o.gather(tbl))
    g.close()


# ---- the whole transfer workflow -----------------------------------------------------------------
def _same_state(o, g):
    assert np.array_equal(g.bytes(), o.data)
    assert g.stats() == o.stats()


@pytest.mark.parametrize("mode", ["staged", "rounds", "direct"])
def test_transfer_and_errors(gpu, mode):
    M, TorchPool = gpu
    geom = GEOMS["f480"]
    flags = M.MP_DIRECT if mode == "direct" else 0
    so, sg = make_pair(gpu, geom, 40, 4, staging_blocks=3 if mode == "rounds" else 40)
    do, dg = make_pair(gpu, geom, 30, 5, staging_blocks=0)
    assert M.mp_alloc(sg.h, 40)[0] == so.alloc(40)[0] == 0
    rng = np.random.default_rng(6)
    tbl = rng.integers(0, 40, 17).astype(np.int32)
    rc, d = M.mp_transfer(sg.h, dg.h, tbl, flags=flags)
    rco, d_o = O.transfer(so, do, tbl)
    assert rc == rco == 0 and d.tolist() == d_o.tolist()
    _same_state(do, dg)
    # explicit destination list (skips allocation)
    given = d[::-1].copy()
    rc, _ = M.mp_transfer(sg.h, dg.h, tbl, given, flags=flags | M.MP_DST_GIVEN)
    rco, _ = O.transfer(so, do, tbl, given, flags=O.DST_GIVEN)
    assert rc == rco == 0
    _same_state(do, dg)
    # errors leave everything untouched
    snap = dg.bytes()
    st = dg.stats()
    for args, kw, want in [
        (([40],), {}, M.MP_EINVAL),                                   # src id out of range
        (([1, 2], [d[0], d[0]]), {"flags": M.MP_DST_GIVEN}, M.MP_EINVAL),   # duplicate dst
        (([1, 2], [29, 28]), {"flags": M.MP_DST_GIVEN}, M.MP_EINVAL),       # dst not held
        ((np.arange(14),), {}, M.MP_ENOMEM),                          # 13 free at dst
    ]:
        kw = dict(kw)
        kw["flags"] = kw.get("flags", 0) | flags
        rc, _ = M.mp_transfer(sg.h, dg.h, *args, **kw)
        assert rc == want, (args, M.mp_last_error(sg.h))
    other = TorchPool(3, 5, 24, 2, 2, 8)
    assert M.mp_transfer(sg.h, other.h, [1])[0] == M.MP_ESHAPE
    assert np.array_equal(dg.bytes(), snap) and dg.stats() == st
    # batched form and the one-call-per-fragment reference point give the same bytes
    tb = rng.integers(0, 40, 5).astype(np.int32)
    rc, db = M.mp_transfer_batch(sg.h, dg.h, tb, [0, 2, 2, 5], flags=flags)
    rco, db_o = O.transfer(so, do, tb)
    assert rc == rco == 0 and db.tolist() == db_o.tolist()
    rc, _ = M.mp_transfer(sg.h, dg.h, tb[::-1].copy(), db, flags=M.MP_PER_FRAGMENT | M.MP_DST_GIVEN)
    rco, _ = O.transfer(so, do, tb[::-1].copy(), db_o, flags=O.DST_GIVEN)
    assert rc == rco == 0
    _same_state(do, dg)
    assert M.mp_transfer_batch(sg.h, dg.h, tb, [1, 5], flags=flags)[0] == M.MP_EINVAL
    # n = 0
    rc, d0 = M.mp_transfer(sg.h, dg.h, np.zeros(0, np.int32), flags=flags)
    assert rc == 0 and d0.size == 0
    for p in (sg, dg, other):
        p.close()


@pytest.mark.parametrize("direct", [0, 1])
def test_table_sizes_around_the_code_path_switches(gpu, direct):
    """The copy takes a different route depending on the table length: ids in the kernel
    arguments up to 192 entries, an uploaded table sorted by comparison up to 512 and by radix
    sort beyond.  Lengths on both sides of each switch, staged (several rounds included) and
    fused, every byte against the oracle."""
    M, TorchPool = gpu
    geom = GEOMS["f480"]
    fl = M.MP_DIRECT if direct else 0
    so, sg = make_pair(gpu, geom, 900, 31, staging_blocks=200)
    do, dg = make_pair(gpu, geom, 900, 32, staging_blocks=0)
    assert M.mp_alloc(sg.h, 900)[0] == so.alloc(900)[0] == 0
    rng = np.random.default_rng(33)
    for n in (1, 2, 191, 192, 193, 200, 201, 511, 512, 513, 700):
        tbl = rng.integers(0, 900, n).astype(np.int32)            # sources may repeat
        rc, d = M.mp_transfer(sg.h, dg.h, tbl, flags=fl | M.MP_ASYNC)
        rco, d_o = O.transfer(so, do, tbl)
        assert rc == rco == 0 and d.tolist() == d_o.tolist(), (n, M.mp_last_error(sg.h))
        given = rng.permutation(d).astype(np.int32)               # explicit, shuffled destinations
        rc, _ = M.mp_transfer(sg.h, dg.h, tbl, given, flags=fl | M.MP_DST_GIVEN)
        rco, _ = O.transfer(so, do, tbl, given, flags=O.DST_GIVEN)
        assert rc == rco == 0
        _same_state(do, dg)
        assert M.mp_free(dg.h, d) == do.free(d_o) == 0
    sg.close()
    dg.close()


def test_transfer_without_staging_is_refused(gpu):
    M, TorchPool = gpu
    geom = GEOMS["f64"]
    so, sg = make_pair(gpu, geom, 8, 1, staging_blocks=0)
    do, dg = make_pair(gpu, geom, 8, 2, staging_blocks=0)
    M.mp_alloc(sg.h, 8)
    assert M.mp_transfer(sg.h, dg.h, [1, 2])[0] == M.MP_ENOSTAGING
    assert dg.stats()["n_free"] == 8
    rc, d = M.mp_transfer(sg.h, dg.h, [1, 2], flags=M.MP_DIRECT)   # the fused path needs none
    assert rc == 0 and d.tolist() == [0, 1]
    sg.close()
    dg.close()


def test_transfer_inside_one_pool(gpu):
    M, TorchPool = gpu
    geom = GEOMS["f64"]
    o, g = make_pair(gpu, geom, 12, 7, staging_blocks=3)
    M.mp_alloc(g.h, 6)
    o.alloc(6)
    rc, _ = M.mp_transfer(g.h, g.h, [0, 1, 2], [1, 2, 0], flags=M.MP_DST_GIVEN)   # rotation, one round
    rco, _ = O.transfer(o, o, [0, 1, 2], [1, 2, 0], flags=O.DST_GIVEN)
    assert rc == rco == 0
    _same_state(o, g)
    # overlapping tables that need two rounds, or the fused kernel: refused
    assert M.mp_transfer(g.h, g.h, [0, 1, 2, 3], [1, 2, 3, 0], flags=M.MP_DST_GIVEN)[0] == M.MP_ENOSTAGING
    assert M.mp_transfer(g.h, g.h, [0, 1], [1, 0], flags=M.MP_DST_GIVEN | M.MP_DIRECT)[0] == M.MP_EINVAL
    # fresh destination ids cannot overlap: rounds and fused are fine
    for fl in (0, M.MP_DIRECT):
        rc, d = M.mp_transfer(g.h, g.h, [0, 1, 2, 3], flags=fl)
        rco, d_o = O.transfer(o, o, [0, 1, 2, 3])
        assert rc == rco == 0 and d.tolist() == d_o.tolist()
        M.mp_free(g.h, d)
        o.free(d_o)
        _same_state(o, g)
    g.close()


@pytest.mark.parametrize("direct", [0, 1])
def test_in_pool_transfer_never_evicts_its_sources(gpu, direct):
    """Inside one pool the sources are held while destination blocks are allocated: with
    on-demand eviction a historical source block is never the victim (it would come back as its
    own destination).  Same calls on the oracle, whole state compared."""
    M, TorchPool = gpu
    geom = GEOMS["f480"]
    bs = geom[3]
    fl = M.MP_EVICT_ON_DEMAND | (M.MP_DIRECT if direct else 0)
    o, g = make_pair(gpu, geom, 10, 21, staging_blocks=2)
    rng = np.random.default_rng(22)
    prompts = [rng.integers(0, 1000, bs * k, dtype=np.uint32) for k in (1, 1, 2, 3)]
    for t in prompts:                                   # 7 cached, unreferenced blocks
        rc, ids = M.mp_alloc(g.h, len(t) // bs)
        assert rc == 0 and ids.tolist() == o.alloc(len(t) // bs)[1].tolist()
        assert M.mp_insert(g.h, t, ids) == o.insert(t, ids) and M.mp_free(g.h, ids) == o.free(ids) == 0
    rc, held = M.mp_alloc(g.h, 3)                       # the pool is full
    assert rc == 0 and held.tolist() == o.alloc(3)[1].tolist()
    for src_tbl in ([0], [1, 0], [2, 3, 0], [4, 5, 6, 1], [0, 1, 2, 3, 4, 5, 6]):
        rc, d = M.mp_transfer(g.h, g.h, src_tbl, flags=fl)
        rco, d_o = O.transfer(o, o, src_tbl, flags=O.EVICT_ON_DEMAND)
        assert rc == rco, (src_tbl, M.mp_last_error(g.h))
        if rc == 0:
            assert d.tolist() == d_o.tolist() and not set(d.tolist()) & set(src_tbl)
            assert M.mp_free(g.h, d) == o.free(d_o) == 0
        _same_state(o, g)
    t = rng.integers(0, 1000, 2 * bs, dtype=np.uint32)
    rc, d = M.mp_transfer_with_insert(g.h, g.h, t, 0, [0, 2], flags=fl)
    rco, d_o = O.transfer_with_insert(o, o, t, 0, [0, 2], flags=O.EVICT_ON_DEMAND)
    assert rc == rco and d.tolist() == d_o.tolist()
    _same_state(o, g)
    for p in prompts + [t]:
        assert M.mp_match(g.h, p, 4)[1].tolist() == o.match(p)[1].tolist()
    g.close()


def test_tiny_config_walkthrough(gpu):
    """Config 1: match, transfer_with_insert of the unmatched suffix, match again."""
    M, TorchPool = gpu
    g_ = W.CONFIGS[1]
    geom = (g_.L, g_.H, g_.D, g_.bs, g_.e)
    so, sg = make_pair(gpu, geom, g_.NB, 1, staging_blocks=8)
    do = O.OraclePool(*geom, g_.NB)
    dg = TorchPool(*geom, g_.NB)
    dg.mem.zero_()
    M.mp_alloc(sg.h, g_.NB)
    so.alloc(g_.NB)
    rng = np.random.default_rng(1)
    moved = []
    for t in W.tiny_requests():
        tbl = W.random_table(rng, g_.NB, 8)
        rc, m = M.mp_match(dg.h, t, 8, M.MP_MATCH_PIN)
        rco, mo = do.match(t, flags=O.MATCH_PIN)
        assert rc == rco == 0 and m.tolist() == mo.tolist()
        rc, d = M.mp_transfer_with_insert(sg.h, dg.h, t, len(m), tbl[len(m):])
        rco, d_o = O.transfer_with_insert(so, do, t, len(mo), tbl[len(mo):])
        assert rc == rco == 0 and d.tolist() == d_o.tolist(), M.mp_last_error(sg.h)
        moved.append(len(d))
        assert M.mp_match(dg.h, t, 8)[1].tolist() == do.match(t)[1].tolist() == m.tolist() + d.tolist()
        _same_state(do, dg)
    assert moved == [8, 4, 4, 4, 4, 4, 4, 4]
    sg.close()
    dg.close()


@pytest.mark.parametrize("seed,probe", [(0, 0), (1, 0), (2, 0), (0, 1), (3, 1), (4, 1)])
def test_random_workflow_against_oracle(gpu, seed, probe):
    """Random interleaving of match / transfer_with_insert / free / evict on a small, tight
    destination pool: ids, index answers, statistics and every pool byte must agree."""
    M, TorchPool = gpu
    geom = GEOMS["f64"]
    bs = geom[3]
    rng = np.random.default_rng(100 + seed)
    so, sg = make_pair(gpu, geom, 64, seed, staging_blocks=5)
    do, dg = make_pair(gpu, geom, 24, seed + 50, staging_blocks=0, hash_seed=seed)
    assert M.mp_set_tunable(dg.h, "device_probe", probe) == 0    # index walk on the GPU or on the host
    M.mp_alloc(sg.h, 64)
    so.alloc(64)
    prompts, live = [], []
    for step in range(60):
        if prompts and rng.integers(0, 2):
            base = prompts[int(rng.integers(0, len(prompts)))]
            t = np.concatenate([base, rng.integers(0, 50, int(rng.integers(1, 3 * bs)), dtype=np.uint32)])
        else:
            t = rng.integers(0, 50, int(rng.integers(0, 6 * bs)), dtype=np.uint32)
        nblk = (len(t) + bs - 1) // bs
        rc, m = M.mp_match(dg.h, t, nblk, M.MP_MATCH_PIN)
        rco, mo = do.match(t, flags=O.MATCH_PIN)
        assert rc == rco == 0 and m.tolist() == mo.tolist()
        tbl = rng.integers(0, 64, nblk - len(m)).astype(np.int32)
        fl = M.MP_EVICT_ON_DEMAND if rng.integers(0, 3) else 0
        if rng.integers(0, 4) == 0:
            fl |= M.MP_DIRECT
        rc, d = M.mp_transfer_with_insert(sg.h, dg.h, t, len(m), tbl, flags=fl)
        rco, d_o = O.transfer_with_insert(so, do, t, len(mo), tbl, flags=fl & 0x3)
        assert rc == rco, (step, rc, rco, M.mp_last_error(sg.h))
        if rc == 0:
            assert d.tolist() == d_o.tolist()
            prompts.append(t)
            live.append(np.concatenate([m, d]))
        else:
            live.append(m)
        if len(live) > 3 or rc != 0:      # requests finish: their blocks become historical
            k = int(rng.integers(0, len(live)))
            ids = live.pop(k)
            assert M.mp_free(dg.h, ids) == do.free(ids) == 0
        if rng.integers(0, 5) == 0:
            k = int(rng.integers(0, 4))
            assert M.mp_evict(dg.h, k) == do.evict(k)
        if prompts and rng.integers(0, 6) == 0:
            t = prompts[int(rng.integers(0, len(prompts)))]
            assert M.mp_delete(dg.h, t) == do.delete(t)
        _same_state(do, dg)
    sg.close()
    dg.close()


def test_stale_prefix_and_given_destinations(gpu):
    M, TorchPool = gpu
    geom = GEOMS["f64"]
    bs = geom[3]
    so, sg = make_pair(gpu, geom, 32, 1, staging_blocks=8)
    do, dg = make_pair(gpu, geom, 16, 2, staging_blocks=0)
    M.mp_alloc(sg.h, 32)
    so.alloc(32)
    rng = np.random.default_rng(9)
    t1 = rng.integers(0, 1000, 3 * bs, dtype=np.uint32)
    t2 = np.concatenate([t1, rng.integers(0, 1000, 2 * bs + 1, dtype=np.uint32)])
    assert M.mp_transfer_with_insert(sg.h, dg.h, t1, 0, [10, 11, 12])[0] == 0
    O.transfer_with_insert(so, do, t1, 0, [10, 11, 12])
    snap, st = dg.bytes(), dg.stats()
    assert M.mp_transfer_with_insert(sg.h, dg.h, t2, 4, [20, 21])[0] == M.MP_ESTALE
    assert M.mp_transfer_with_insert(sg.h, dg.h, t2, 3, [20])[0] == M.MP_EINVAL
    assert M.mp_transfer_with_insert(sg.h, dg.h, t2, 6, [])[0] == M.MP_EINVAL
    assert np.array_equal(dg.bytes(), snap) and dg.stats() == st
    # explicit destinations: allocate first, then transfer_with_insert into them
    rc, mine = M.mp_alloc(dg.h, 3)
    rco, mine_o = do.alloc(3)
    rc, d = M.mp_transfer_with_insert(sg.h, dg.h, t2, 3, [20, 21, 22], mine, flags=M.MP_DST_GIVEN)
    rco, d_o = O.transfer_with_insert(so, do, t2, 3, [20, 21, 22], mine_o, flags=O.DST_GIVEN)
    assert rc == rco == 0 and d.tolist() == d_o.tolist() == mine.tolist()
    _same_state(do, dg)
    assert M.mp_match(dg.h, t2, 8)[1].tolist() == do.match(t2)[1].tolist()
    # a given destination that is already indexed cannot be adopted again
    t3 = rng.integers(0, 1000, bs, dtype=np.uint32)
    assert M.mp_transfer_with_insert(sg.h, dg.h, t3, 0, [5], [mine[0]], flags=M.MP_DST_GIVEN)[0] == M.MP_EINVAL
    assert O.transfer_with_insert(so, do, t3, 0, [5], [mine_o[0]], flags=O.DST_GIVEN)[0] == O.EINVAL
    _same_state(do, dg)
    sg.close()
    dg.close()


@pytest.mark.parametrize("probe", [0, 1])
def test_batched_forms(gpu, probe):
    M, TorchPool = gpu
    geom = GEOMS["tiny"]
    bs = geom[3]
    rng = np.random.default_rng(12)
    so, sg = make_pair(gpu, geom, 96, 3, staging_blocks=7)       # several staging rounds
    do, dg = make_pair(gpu, geom, 200, 4, staging_blocks=0)
    assert M.mp_set_tunable(dg.h, "device_probe", probe) == 0
    M.mp_alloc(sg.h, 96)
    so.alloc(96)
    shared = rng.integers(0, 32000, 3 * bs, dtype=np.uint32)
    for turn in range(3):
        prompts = [np.concatenate([shared, rng.integers(0, 32000, int(n), dtype=np.uint32)])
                   for n in rng.integers(0, 5 * bs, 6)] + [np.zeros(0, np.uint32)]
        toks, tok_off = W.csr(prompts)
        nblk = np.array([(len(p) + bs - 1) // bs for p in prompts], np.uint32)
        cap_off = np.concatenate([[0], np.cumsum(nblk)]).astype(np.uint32)
        rc, mb, m = M.mp_match_batch(dg.h, toks, tok_off, cap_off, M.MP_MATCH_PIN)
        assert rc == 0
        mo = [do.match(p, flags=O.MATCH_PIN)[1] for p in prompts]
        assert m.tolist() == [len(x) for x in mo]
        for r in range(len(prompts)):
            assert mb[cap_off[r]:cap_off[r] + m[r]].tolist() == mo[r].tolist()
        tables = [rng.integers(0, 96, int(nblk[r] - m[r])).astype(np.int32) for r in range(len(prompts))]
        s, blk_off = W.csr(tables, np.int32)
        rc, d = M.mp_transfer_with_insert_batch(sg.h, dg.h, toks, tok_off, m, s, blk_off)
        rco, d_o = O.transfer_with_insert_batch(so, do, toks, tok_off, m, s, blk_off)
        assert rc == rco == 0 and d.tolist() == d_o.tolist(), M.mp_last_error(sg.h)
        _same_state(do, dg)
        held = np.concatenate([mb[cap_off[r]:cap_off[r] + m[r]] for r in range(len(prompts))] + [d])
        assert M.mp_free(dg.h, held) == do.free(held) == 0
        _same_state(do, dg)
    assert M.mp_transfer_with_insert_batch(sg.h, dg.h, toks, tok_off, m, s, blk_off,
                                           flags=M.MP_DST_GIVEN)[0] == M.MP_EINVAL
    sg.close()
    dg.close()


def test_host_tier_both_directions(gpu):
    """HBM -> pinned host (swap-out / transfer to a DRAM tier) and back (swap-in)."""
    M, TorchPool = gpu
    geom = GEOMS["tiny"]
    so, sg = make_pair(gpu, geom, 48, 1, staging_blocks=6)       # 2 slots of 3 records
    ho, hg = make_pair(gpu, geom, 40, 2, staging_blocks=0, tier=1)
    bo, bg = make_pair(gpu, geom, 48, 3, staging_blocks=4)
    M.mp_alloc(sg.h, 48)
    so.alloc(48)
    rng = np.random.default_rng(5)
    # fragment the host pool's free list so records do not land in one run
    rc, a = M.mp_alloc(hg.h, 40)
    ho.alloc(40)
    perm = rng.permutation(40).astype(np.int32)
    assert M.mp_free(hg.h, perm[:30]) == ho.free(perm[:30]) == 0
    tbl = rng.integers(0, 48, 17).astype(np.int32)
    rc, d = M.mp_transfer(sg.h, hg.h, tbl)
    rco, d_o = O.transfer(so, ho, tbl)
    assert rc == rco == 0 and d.tolist() == d_o.tolist(), M.mp_last_error(sg.h)
    _same_state(ho, hg)
    rc, d2 = M.mp_transfer(hg.h, bg.h, d)
    rco, d2_o = O.transfer(ho, bo, d_o)
    assert rc == rco == 0 and d2.tolist() == d2_o.tolist(), M.mp_last_error(hg.h)
    _same_state(bo, bg)
    # the round trip through the host tier is the identity on the moved blocks
    assert M.mp_gather(bg.h, d2[:4]) == 0
    assert np.array_equal(bg.staging_bytes(4), so.gather(tbl[:4]))
    # transfer_with_insert into the host tier indexes DRAM-resident blocks
    t = rng.integers(0, 32000, 3 * geom[3] + 1, dtype=np.uint32)
    rc, d3 = M.mp_transfer_with_insert(sg.h, hg.h, t, 0, [3, 4, 5, 6])
    rco, d3_o = O.transfer_with_insert(so, ho, t, 0, [3, 4, 5, 6])
    assert rc == rco == 0 and d3.tolist() == d3_o.tolist()
    _same_state(ho, hg)
    assert M.mp_match(hg.h, t, 4)[1].tolist() == ho.match(t)[1].tolist()
    assert M.mp_transfer(hg.h, hg.h, [int(d3[0])])[0] == M.MP_ESHAPE   # host -> host unsupported
    # zero-copy variants: the fused kernel stores into / loads from the mapped host pool itself
    tbl2 = rng.integers(0, 48, 9).astype(np.int32)
    rc, d4 = M.mp_transfer(sg.h, hg.h, tbl2, flags=M.MP_DIRECT)
    rco, d4_o = O.transfer(so, ho, tbl2)
    assert rc == rco == 0 and d4.tolist() == d4_o.tolist(), M.mp_last_error(sg.h)
    _same_state(ho, hg)
    rc, d5 = M.mp_transfer(hg.h, bg.h, d4, flags=M.MP_DIRECT)
    rco, d5_o = O.transfer(ho, bo, d4_o)
    assert rc == rco == 0 and d5.tolist() == d5_o.tolist(), M.mp_last_error(hg.h)
    _same_state(bo, bg)
    for p in (sg, hg, bg):
        p.close()


def test_staging_is_ordered_between_main_and_side_stream(gpu):
    """Asynchronous multi-round transfers OUT of a pool keep its staging buffer busy on the
    main stream; host-tier transfers INTO the same pool, issued right behind them, fill that
    buffer on the side stream.  Nothing is synchronised in between, in either slot layout (two
    half-buffer slots, then one whole-buffer slot), so the result equals the oracle's sequential
    one only if the side stream waits for every earlier user of the buffer."""
    M, TorchPool = gpu
    geom = GEOMS["f32k"]                       # 256 KiB records
    bs = geom[3]
    xo, xg = make_pair(gpu, geom, 768, 11, staging_blocks=32)
    yo, yg = make_pair(gpu, geom, 1100, 12, staging_blocks=0)
    ho, hg = make_pair(gpu, geom, 256, 13, staging_blocks=0, tier=1)
    rng = np.random.default_rng(14)
    rc, held = M.mp_alloc(xg.h, 512)
    assert rc == 0 and held.tolist() == xo.alloc(512)[1].tolist()
    # the host tier caches 8 prompts of 16 blocks (historical), plus 96 held blocks
    prompts = [rng.integers(0, 32000, 16 * bs, dtype=np.uint32) for _ in range(8)]
    for t in prompts:
        rc, ids = M.mp_alloc(hg.h, 16)
        assert rc == 0 and ids.tolist() == ho.alloc(16)[1].tolist()
        assert M.mp_insert(hg.h, t, ids) == ho.insert(t, ids)
        assert M.mp_free(hg.h, ids) == ho.free(ids) == 0
    rc, h_held = M.mp_alloc(hg.h, 96)
    assert rc == 0 and h_held.tolist() == ho.alloc(96)[1].tolist()
    low_ids = np.concatenate([ho.match(t)[1] for t in prompts[:3]])
    for t in prompts[:3]:
        assert M.mp_match(hg.h, t, 16)[0] == 0
    fl = M.MP_ASYNC
    # 1. 16 staging rounds on the main stream, not waited for
    tbl1 = rng.permutation(held)[:512].astype(np.int32)
    rc, d1 = M.mp_transfer(xg.h, yg.h, tbl1, flags=fl)
    assert rc == 0 and d1.tolist() == O.transfer(xo, yo, tbl1)[1].tolist()
    # 2. host -> X through the same buffer, two slots of 16 records, copies on the side stream
    src2 = rng.permutation(h_held)[:80].astype(np.int32)
    rc, d2 = M.mp_transfer(hg.h, xg.h, src2, flags=fl)
    assert rc == 0 and d2.tolist() == O.transfer(ho, xo, src2)[1].tolist(), M.mp_last_error(hg.h)
    # 3. out of X again (main stream), then a host -> X transfer that fits ONE whole-buffer slot
    tbl3 = rng.permutation(held)[:500].astype(np.int32)
    rc, d3 = M.mp_transfer(xg.h, yg.h, tbl3, flags=fl)
    assert rc == 0 and d3.tolist() == O.transfer(xo, yo, tbl3)[1].tolist()
    src4 = rng.permutation(h_held)[:30].astype(np.int32)
    rc, d4 = M.mp_transfer(hg.h, xg.h, src4, flags=fl)
    assert rc == 0 and d4.tolist() == O.transfer(ho, xo, src4)[1].tolist()
    # 4. a gather and a scatter of the data-plane pieces, then swap_in through the same buffer
    assert M.mp_gather(xg.h, tbl1[:32], fl) == 0
    assert M.mp_scatter(xg.h, d2[:32], fl) == 0
    xo.scatter(d2[:32], xo.gather(tbl1[:32]))
    rc, up = M.mp_swap_in(hg.h, xg.h, low_ids)
    rco, up_o = O.swap_in(ho, xo, low_ids)
    assert rc == rco == 0 and up.tolist() == up_o.tolist(), M.mp_last_error(hg.h)
    # 5. X -> host right behind an asynchronous main-stream user, then host -> X once more
    rc, d5 = M.mp_transfer(xg.h, yg.h, tbl1[:64], flags=fl)
    assert rc == 0 and d5.tolist() == O.transfer(xo, yo, tbl1[:64])[1].tolist()
    rc, d6 = M.mp_transfer(xg.h, hg.h, tbl3[:24], flags=fl)
    assert rc == 0 and d6.tolist() == O.transfer(xo, ho, tbl3[:24])[1].tolist(), M.mp_last_error(xg.h)
    rc, d7 = M.mp_transfer(hg.h, xg.h, d6, flags=fl)
    assert rc == 0 and d7.tolist() == O.transfer(ho, xo, d6)[1].tolist()
    torch.cuda.synchronize()
    _same_state(xo, xg)
    _same_state(yo, yg)
    _same_state(ho, hg)
    for p in (xg, yg, hg):
        p.close()


def test_async_and_callback(gpu):
    M, TorchPool = gpu
    geom = GEOMS["f32k"]
    so, sg = make_pair(gpu, geom, 24, 1, staging_blocks=24)
    do, dg = make_pair(gpu, geom, 24, 2, staging_blocks=0)
    M.mp_alloc(sg.h, 24)
    so.alloc(24)
    seen = []

    def on_recv(user, priv, priv_len, blocks, n):
        import ctypes
        seen.append((ctypes.string_at(priv, priv_len) if priv else b"", [blocks[i] for i in range(n)]))

    cb = M.RECV_CB(on_recv)
    assert M.mp_set_recv_callback(dg.h, cb) == 0
    tbl = np.arange(23, -1, -1, dtype=np.int32)
    rc, d = M.mp_transfer(sg.h, dg.h, tbl, flags=M.MP_ASYNC, priv=b"req-42")
    rc2, d2 = M.mp_transfer(sg.h, dg.h, tbl[:4], d[:4], flags=M.MP_ASYNC | M.MP_DST_GIVEN)
    torch.cuda.synchronize()
    O.transfer(so, do, tbl)
    assert rc == rc2 == 0
    _same_state(do, dg)
    assert seen[0] == (b"req-42", d.tolist()) and seen[1][1] == d[:4].tolist()
    M.mp_set_recv_callback(dg.h, None)
    sg.close()
    dg.close()


def test_match_and_insert_while_copies_are_still_queued(gpu):
    """Prompts in host memory are hashed on a stream of the library's own and waited for through
    completion words, not through the pool's stream: with asynchronous copies still queued on
    both pools' streams, insert, match and the hashes return the oracle's results, and the
    queued copies land untouched."""
    M, TorchPool = gpu
    geom = GEOMS["f32k"]                                   # 256 KiB blocks
    NB = 768
    so, sg = make_pair(gpu, geom, NB, 11, staging_blocks=NB)
    do, dg = make_pair(gpu, geom, NB, 12, staging_blocks=0)
    M.mp_alloc(sg.h, NB)
    so.alloc(NB)
    rng = np.random.default_rng(5)
    tbl = W.random_table(rng, NB, 700)
    rc, d = M.mp_transfer(sg.h, dg.h, tbl, flags=M.MP_ASYNC)
    rco, d_o = O.transfer(so, do, tbl)
    assert rc == rco == 0 and d.tolist() == d_o.tolist()
    bs, at = geom[3], 0
    for k in range(6):                                     # more copies behind it, then the index calls
        fl = M.MP_ASYNC | M.MP_DST_GIVEN | (M.MP_DIRECT if k & 1 else 0)
        assert M.mp_transfer(sg.h, dg.h, tbl, d, flags=fl)[0] == 0
        t = rng.integers(0, 128256, (30 + 25 * k) * bs + k, dtype=np.uint32)
        nb = len(t) // bs
        ids = d[at:at + nb]
        at += nb
        rc, n_new = M.mp_insert(dg.h, t, ids)
        rco, n_o = do.insert(t, ids)
        assert rc == rco == 0 and n_new == n_o == nb, M.mp_last_error(dg.h)
        rc, m = M.mp_match(dg.h, t, nb + 4)
        rco, mo = do.match(t)
        assert rc == rco == 0 and m.tolist() == mo.tolist() == ids.tolist()
        rc, h = M.mp_block_hashes(dg.h, t[bs:], bs)
        assert rc == 0 and np.array_equal(h, O.block_hashes(t[bs:], bs, 0))
    torch.cuda.synchronize()
    _same_state(do, dg)
    sg.close()
    dg.close()


def test_profile_counters(gpu):
    M, TorchPool = gpu
    geom = GEOMS["f32k"]
    so, sg = make_pair(gpu, geom, 16, 1, staging_blocks=16)
    do, dg = make_pair(gpu, geom, 16, 2, staging_blocks=0)
    M.mp_alloc(sg.h, 16)
    assert M.mp_profile_enable(sg.h, True) == 0
    rc, d = M.mp_transfer(sg.h, dg.h, np.arange(16))
    assert rc == 0
    for kind in (M.PROF_GATHER, M.PROF_SCATTER):
        rc, ms, n, nbytes = M.mp_profile_read(sg.h, kind)
        assert rc == 0 and n == 1 and ms > 0 and nbytes == 2 * 16 * sg.B
    assert M.mp_profile_read(sg.h, M.PROF_GATHER)[2] == 0      # cleared by the read
    sg.close()
    dg.close()


@pytest.mark.parametrize("mode", ["staged", "rounds", "direct"])
def test_transfer_layers(gpu, mode):
    """By-layer transfer: explicit destinations, a layer range per call."""
    M, TorchPool = gpu
    geom = (5, 2, 64, 16, 2)                     # L = 5, F = 4 KiB
    flags = M.MP_DIRECT if mode == "direct" else 0
    so, sg = make_pair(gpu, geom, 40, 4, staging_blocks=2 if mode == "rounds" else 16)
    do, dg = make_pair(gpu, geom, 30, 5, staging_blocks=0)
    M.mp_alloc(sg.h, 40)
    so.alloc(40)
    rng = np.random.default_rng(6)
    tbl = rng.integers(0, 40, 13).astype(np.int32)
    rc, d = M.mp_alloc(dg.h, 13)
    rco, d_o = do.alloc(13)
    assert rc == rco == 0 and d.tolist() == d_o.tolist()
    for l0, l1 in ((0, 1), (1, 2), (2, 5)):       # the engine ships layers as they finish
        assert M.mp_transfer_layers(sg.h, dg.h, tbl, d, l0, l1, flags) == 0, M.mp_last_error(sg.h)
        assert O.transfer_layers(so, do, tbl, d_o, l0, l1) == 0
        _same_state(do, dg)
    # after the last layer the destination equals a whole-block transfer
    ref = O.OraclePool(*geom, 30, data=make_pair(gpu, geom, 30, 5, 0)[0].data)
    ref.alloc(13)
    assert O.transfer(so, ref, tbl, d_o, flags=O.DST_GIVEN)[0] == 0
    assert np.array_equal(dg.bytes(), ref.data)
    snap = dg.bytes()
    assert M.mp_transfer_layers(sg.h, dg.h, tbl, d, 2, 2, flags) == M.MP_EINVAL
    assert M.mp_transfer_layers(sg.h, dg.h, tbl, d, 3, 6, flags) == M.MP_EINVAL
    assert M.mp_transfer_layers(sg.h, dg.h, tbl[:2], [29, 28], 0, 1, flags) == M.MP_EINVAL   # not held
    assert M.mp_transfer_layers(sg.h, dg.h, tbl[:2], [d[0], d[0]], 0, 1, flags) == M.MP_EINVAL
    assert np.array_equal(dg.bytes(), snap)
    # host tier: only through the fused kernel
    ho, hg = make_pair(gpu, geom, 16, 8, staging_blocks=0, tier=1)
    rc, h = M.mp_alloc(hg.h, 13)
    ho.alloc(13)
    assert M.mp_transfer_layers(sg.h, hg.h, tbl, h, 1, 4, 0) == M.MP_ESHAPE
    assert M.mp_transfer_layers(sg.h, hg.h, tbl, h, 1, 4, M.MP_DIRECT) == 0
    assert O.transfer_layers(so, ho, tbl, h, 1, 4) == 0
    _same_state(ho, hg)
    for p in (sg, dg, hg):
        p.close()


@pytest.mark.parametrize("layouts", [(2, 2), (2, 0), (0, 2)])
def test_aggregated_hbm_pools(gpu, layouts):
    """HBM pools that opted into the aggregated layout, on either or both ends."""
    M, TorchPool = gpu
    geom = GEOMS["f480"]
    so, sg = make_pair(gpu, geom, 40, 4, staging_blocks=5, layout=layouts[0])
    do, dg = make_pair(gpu, geom, 30, 5, staging_blocks=0, layout=layouts[1])
    M.mp_alloc(sg.h, 40)
    so.alloc(40)
    rng = np.random.default_rng(8)
    for flags in (0, M.MP_DIRECT):
        tbl = rng.integers(0, 40, 11).astype(np.int32)
        rc, d = M.mp_transfer(sg.h, dg.h, tbl, flags=flags)
        rco, d_o = O.transfer(so, do, tbl)
        assert rc == rco == 0 and d.tolist() == d_o.tolist(), M.mp_last_error(sg.h)
        _same_state(do, dg)
    assert M.mp_gather(sg.h, tbl[:5]) == 0
    assert np.array_equal(sg.staging_bytes(5), so.gather(tbl[:5]))
    rc, ids = M.mp_alloc(dg.h, 3)
    do.alloc(3)
    assert M.mp_transfer_layers(sg.h, dg.h, tbl[:3], ids, 0, 1, 0) == 0
    assert O.transfer_layers(so, do, tbl[:3], ids, 0, 1) == 0
    _same_state(do, dg)
    sg.close()
    dg.close()
    assert M.mp_pool_create(*geom, 8, 4096, tier=M.MP_TIER_HOST_PINNED,
                            layout=M.MP_LAYOUT_DISCRETE)[0] == M.MP_EINVAL


@pytest.mark.parametrize("seed", range(6))
def test_mixed_features_random(gpu, seed):
    """Everything interleaved: HBM and host-tier destinations, discrete and aggregated pools,
    staged / fused / asynchronous transfers, swap-in, by-layer rewrites, delete, evict."""
    M, TorchPool = gpu
    geoms = [(3, 1, 8, 4, 2), (2, 2, 64, 16, 2), (1, 5, 24, 2, 2), (4, 3, 40, 8, 2)]
    rng = np.random.default_rng(1000 + seed)
    geom = geoms[seed % len(geoms)]
    bs = geom[3]
    lay_s, lay_d = int(rng.integers(0, 2)) * 2, int(rng.integers(0, 2)) * 2
    so, sg = make_pair(gpu, geom, 64, seed, staging_blocks=int(rng.integers(1, 9)), layout=lay_s)
    do, dg = make_pair(gpu, geom, int(rng.integers(16, 40)), seed + 50,
                       staging_blocks=int(rng.integers(1, 5)), hash_seed=seed, layout=lay_d)
    ho, hg = make_pair(gpu, geom, 24, seed + 70, staging_blocks=0, tier=1, hash_seed=seed)
    for p in (dg, hg):
        assert M.mp_set_tunable(p.h, "device_probe", seed % 2) == 0
    M.mp_alloc(sg.h, 64)
    so.alloc(64)
    prompts, live, hlive = [], [], []
    for step in range(60):
        if prompts and rng.integers(0, 2):
            base = prompts[int(rng.integers(0, len(prompts)))]
            t = np.concatenate([base, rng.integers(0, 50, int(rng.integers(1, 3 * bs)), dtype=np.uint32)])
        else:
            t = rng.integers(0, 50, int(rng.integers(0, 6 * bs)), dtype=np.uint32)
        nblk = (len(t) + bs - 1) // bs
        t_o, t_g, lv = (do, dg, live) if rng.integers(0, 4) else (ho, hg, hlive)
        rc, m = M.mp_match(t_g.h, t, nblk, M.MP_MATCH_PIN)
        rco, mo = t_o.match(t, flags=O.MATCH_PIN)
        assert rc == rco == 0 and m.tolist() == mo.tolist()
        tbl = rng.integers(0, 64, nblk - len(m)).astype(np.int32)
        fl = M.MP_EVICT_ON_DEMAND if rng.integers(0, 3) else 0
        fl |= M.MP_DIRECT if rng.integers(0, 3) == 0 else 0
        fl |= M.MP_ASYNC if rng.integers(0, 2) else 0
        rc, d = M.mp_transfer_with_insert(sg.h, t_g.h, t, len(m), tbl, flags=fl)
        rco, d_o = O.transfer_with_insert(so, t_o, t, len(mo), tbl, flags=fl & 0x3)
        assert rc == rco, (seed, step, rc, rco, M.mp_last_error(sg.h))
        torch.cuda.synchronize()
        if rc == 0:
            assert d.tolist() == d_o.tolist()
            prompts.append(t)
            lv.append(np.concatenate([m, d]))
        else:
            lv.append(m)
        if len(lv) > 3 or rc != 0:
            ids = lv.pop(int(rng.integers(0, len(lv))))
            assert M.mp_free(t_g.h, ids) == t_o.free(ids) == 0
        r = rng.integers(0, 8)
        if r == 0:
            k = int(rng.integers(0, 4))
            assert M.mp_evict(t_g.h, k) == t_o.evict(k)
        elif r == 1 and prompts:
            q = prompts[int(rng.integers(0, len(prompts)))]
            assert M.mp_delete(t_g.h, q) == t_o.delete(q)
        elif r == 2 and hlive:                      # swap a held host block set into the HBM pool
            ids = hlive[int(rng.integers(0, len(hlive)))]
            if len(ids):
                f2 = M.MP_EVICT_ON_DEMAND | (M.MP_DIRECT if rng.integers(0, 2) else 0)
                rc, d2 = M.mp_transfer(hg.h, dg.h, ids, flags=f2)
                rco, d2o = O.transfer(ho, do, ids, flags=O.EVICT_ON_DEMAND)
                assert rc == rco, (seed, step, rc, rco, M.mp_last_error(hg.h))
                if rc == 0:
                    assert d2.tolist() == d2o.tolist()
                    live.append(d2)
        elif r == 3 and live:                       # by-layer rewrite of a held destination set
            ids = np.unique(live[int(rng.integers(0, len(live)))])
            if len(ids):
                srcs = rng.integers(0, 64, len(ids)).astype(np.int32)
                l0 = int(rng.integers(0, geom[0]))
                l1 = int(rng.integers(l0 + 1, geom[0] + 1))
                f2 = M.MP_DIRECT if rng.integers(0, 2) else 0
                assert M.mp_transfer_layers(sg.h, dg.h, srcs, ids, l0, l1, f2) == 0
                assert O.transfer_layers(so, do, srcs, ids, l0, l1) == 0
        _same_state(do, dg)
        _same_state(ho, hg)
    for p in (sg, dg, hg):
        p.close()


def test_device_probe_switched_on_late_and_long_prompts(gpu):
    """The device copy of the index is seeded from a populated index, follows inserts, evictions
    and deletes, and handles prompts longer than one probe tile (1024 blocks)."""
    M, TorchPool = gpu
    geom = (1, 1, 8, 2, 2)                       # bs = 2: long chains from few tokens
    bs = 2
    NB = 6000
    o = O.OraclePool(*geom, NB)
    g = TorchPool(*geom, NB)
    rng = np.random.default_rng(31)
    long_a = rng.integers(0, 5, 2 * 2500, dtype=np.uint32)           # 2500 blocks
    long_b = np.concatenate([long_a[: 2 * 1500], rng.integers(0, 5, 2 * 700 + 1, dtype=np.uint32)])
    for t in (long_a, long_b):
        nb = len(t) // bs
        rc, ids = M.mp_alloc(g.h, nb)
        _, ids_o = o.alloc(nb)
        assert M.mp_insert(g.h, t, ids) == o.insert(t, ids_o)
        assert M.mp_free(g.h, ids) == o.free(ids_o) == 0
    assert M.mp_set_tunable(g.h, "device_probe", 1) == 0             # seeded from the live index
    for t in (long_a, long_b, long_a[: 2 * 1024], long_a[: 2 * 1025 + 1], long_b[:3], np.zeros(0, np.uint32)):
        nb = len(t) // bs
        assert M.mp_match(g.h, t, nb)[1].tolist() == o.match(t)[1].tolist()
        assert M.mp_match(g.h, t, max(nb - 3, 0))[1].tolist() == o.match(t, cap=max(nb - 3, 0))[1].tolist()
    assert M.mp_delete(g.h, long_b) == o.delete(long_b)
    assert M.mp_evict(g.h, 900) == o.evict(900)
    for t in (long_a, long_b):
        assert M.mp_match(g.h, t, len(t) // bs)[1].tolist() == o.match(t)[1].tolist()
    # a hash that is in the table but with other tokens (forged via the *_hashed entry) stays a miss
    t2 = long_a[: 2 * 4].copy()
    rc, h2 = M.mp_block_hashes(g.h, t2, bs)
    t2[0] ^= 1
    rc, ids = M.mp_alloc(g.h, 0)
    assert M.mp_match(g.h, t2, 4)[1].tolist() == o.match(t2)[1].tolist()
    assert g.stats() == o.stats()
    assert M.mp_set_tunable(g.h, "device_probe", 0) == 0
    assert M.mp_match(g.h, long_a, 2500)[1].tolist() == o.match(long_a)[1].tolist()
    g.close()


# ---- swap between the two tiers of one instance (Table 1: swap_out / swap_in) -------------------
@pytest.mark.parametrize("lower_tier,direct", [(1, 0), (1, 1), (0, 0)])
def test_swap_script(gpu, lower_tier, direct):
    """The hand-derived scenario the oracle is pinned to, step by step on the GPU."""
    M, TorchPool = gpu
    geom = GEOMS["tiny"]
    bs = geom[3]
    fl = M.MP_DIRECT if direct else 0
    uo, ug = make_pair(gpu, geom, 8, 1, staging_blocks=2)                 # two records: forces rounds
    lo, lg = make_pair(gpu, geom, 8, 2, staging_blocks=0 if lower_tier else 2, tier=lower_tier)
    A = np.arange(0, 3 * bs, dtype=np.uint32)
    Bq = np.concatenate([A[:bs], np.arange(100, 100 + bs, dtype=np.uint32)])
    for t, n in ((A, 3), (Bq, 2)):
        rc, ids = M.mp_alloc(ug.h, n)
        assert rc == 0 and ids.tolist() == uo.alloc(n)[1].tolist()
        assert M.mp_insert(ug.h, t, ids) == uo.insert(t, ids)
        assert M.mp_free(ug.h, ids) == uo.free(ids) == 0
    for k in (1, 2, 3):
        assert M.mp_swap_out(ug.h, lg.h, k, fl) == O.swap_out(uo, lo, k), M.mp_last_error(ug.h)
        _same_state(uo, ug)
        _same_state(lo, lg)
    for t in (A, Bq):
        assert M.mp_match(lg.h, t, 3)[1].tolist() == lo.match(t)[1].tolist()
        assert M.mp_match(ug.h, t, 3)[1].tolist() == uo.match(t)[1].tolist() == []
    low_ids = lo.match(A)[1]
    assert M.mp_match(lg.h, A, 3)[1].tolist() == low_ids.tolist() and len(low_ids) == 3
    rc, up = M.mp_swap_in(lg.h, ug.h, low_ids[[0, 2]], fl)                # shallow id first, deep one second
    rco, up_o = O.swap_in(lo, uo, low_ids[[0, 2]])
    assert rc == rco == 0 and up.tolist() == up_o.tolist(), M.mp_last_error(lg.h)
    _same_state(uo, ug)
    _same_state(lo, lg)
    assert M.mp_match(ug.h, A, 3)[1].tolist() == uo.match(A)[1].tolist() and len(uo.match(A)[1]) == 3
    assert M.mp_evict(ug.h, 8) == uo.evict(8) == (0, 0)                   # the deep block is referenced
    assert M.mp_free(ug.h, up) == uo.free(up) == 0
    assert M.mp_evict(ug.h, 8) == uo.evict(8) == (0, 3)
    ug.close()
    lg.close()


@pytest.mark.parametrize("seed,lower_tier,direct,probe", [(0, 1, 0, 0), (1, 1, 1, 0), (2, 0, 0, 0),
                                                         (3, 1, 0, 1), (4, 0, 1, 1), (5, 1, 0, 0)])
def test_swap_random_against_oracle(gpu, seed, lower_tier, direct, probe):
    """Random mix of insert / free / swap_out / swap_in / evict / match on a tight upper pool and
    a lower pool that sometimes has to evict too: ids, statistics and every byte of both pools."""
    M, TorchPool = gpu
    geom = GEOMS["f64"]
    bs = geom[3]
    fl = M.MP_DIRECT if direct else 0
    rng = np.random.default_rng(700 + seed)
    uo, ug = make_pair(gpu, geom, 20, seed, staging_blocks=3, hash_seed=seed)
    NB_low = 12 if seed % 2 else 28                     # the small one must evict on demand itself
    lo, lg = make_pair(gpu, geom, NB_low, seed + 30, staging_blocks=0 if lower_tier else 2,
                        tier=lower_tier, hash_seed=seed)
    assert M.mp_set_tunable(ug.h, "device_probe", probe) == 0
    prompts, held = [], []
    n_out = n_in = 0
    for step in range(160):
        op = int(rng.choice([0, 0, 0, 2, 2, 3, 3, 3, 4, 4, 4, 5, 6]))
        if op == 0:                                                        # a request finishes prefill
            if prompts and rng.integers(0, 2):
                base = prompts[int(rng.integers(0, len(prompts)))]
                t = np.concatenate([base[: bs * int(rng.integers(0, len(base) // bs + 1))],
                                    rng.integers(0, 6, int(rng.integers(1, 3 * bs)), dtype=np.uint32)])
            else:
                t = rng.integers(0, 6, int(rng.integers(0, 5 * bs)), dtype=np.uint32)
            nb = len(t) // bs
            rc, ids = M.mp_alloc(ug.h, nb)
            rco, ids_o = uo.alloc(nb)
            assert rc == rco
            if rc == 0:
                assert ids.tolist() == ids_o.tolist()
                assert M.mp_insert(ug.h, t, ids) == uo.insert(t, ids)
                prompts.append(t)
                held.append(ids)
        elif op == 2 and held:
            ids = held.pop(int(rng.integers(0, len(held))))
            assert M.mp_free(ug.h, ids) == uo.free(ids) == 0
        elif op == 3:
            k = int(rng.integers(0, 7))
            got = M.mp_swap_out(ug.h, lg.h, k, fl)
            assert got == O.swap_out(uo, lo, k), (step, M.mp_last_error(ug.h))
            n_out += got[1]
        elif op == 4 and prompts:
            t = prompts[int(rng.integers(0, len(prompts)))]
            rc, low_ids = M.mp_match(lg.h, t, len(t) // bs)
            assert low_ids.tolist() == lo.match(t)[1].tolist()
            if len(low_ids):
                pick = low_ids[rng.permutation(len(low_ids))[: int(rng.integers(1, len(low_ids) + 1))]]
                rc, up = M.mp_swap_in(lg.h, ug.h, pick, fl)
                rco, up_o = O.swap_in(lo, uo, pick)
                assert rc == rco, (step, rc, rco, M.mp_last_error(lg.h))
                if rc == 0:
                    assert up.tolist() == up_o.tolist()
                    held.append(up)
                    n_in += len(up)
        elif op == 5:
            k = int(rng.integers(0, 3))
            pg, po = (ug, uo) if rng.integers(0, 4) else (lg, lo)
            assert M.mp_evict(pg.h, k) == po.evict(k)
        elif op == 6 and prompts:
            t = prompts[int(rng.integers(0, len(prompts)))]
            for pg, po in ((ug, uo), (lg, lo)):
                assert M.mp_match(pg.h, t, len(t) // bs)[1].tolist() == po.match(t)[1].tolist()
        _same_state(uo, ug)
        _same_state(lo, lg)
    assert n_out >= 10 and n_in >= 3                   # the run did move blocks both ways
    ug.close()
    lg.close()


def test_table1_names_walkthrough(gpu):
    """Every call of the paper's Table 1 once, through the class that carries their names."""
    M, TorchPool = gpu
    from paper_2406_17565_amd.pool import MemPool, MemPoolError
    geom = GEOMS["tiny"]
    bs = geom[3]
    rng = np.random.default_rng(11)

    def pair(NB, seed, **kw):
        L, H, D, b, e = geom
        data = W.kv_bytes(np.random.default_rng(seed), 2 * L * NB * b * H * D * e)
        tier = kw.get("tier", 0)
        g = MemPool(*geom, NB, **kw)
        g.load(data)
        return O.OraclePool(*geom, NB, tier=tier, data=data.copy()), g

    po, p = pair(16, 1, staging_blocks=4)                  # "prefill" instance
    do, d = pair(12, 2, staging_blocks=4)                  # "decode" instance, HBM
    ho, h = pair(12, 3, tier=M.MP_TIER_HOST_PINNED)        # its DRAM tier
    t = rng.integers(0, 32000, 5 * bs + 3, dtype=np.uint32)
    src = p.alloc_mem(6)
    assert src.tolist() == po.alloc(6)[1].tolist()
    assert p.insert(t, src) == po.insert(t, src)[1] == 5
    got = p.transfer_with_insert(d, t, src, private=b"request 7")
    assert got.tolist() == O.transfer_with_insert(po, do, t, 0, src)[1].tolist()
    assert d.match(t).tolist() == do.match(t)[1].tolist() == got[:5].tolist()
    d.free_mem(got)
    do.free(got)
    assert d.swap_out(h, 3) == O.swap_out(do, ho, 3)[1] == 3
    low = h.match(t)
    assert low.tolist() == ho.match(t)[1].tolist() and len(low) == 5
    up = d.swap_in(h, low[-1:])
    assert up.tolist() == O.swap_in(ho, do, low[-1:])[1].tolist()
    d.free_mem(up)
    do.free(up)
    moved = p.transfer(d, src[:2])
    assert moved.tolist() == O.transfer(po, do, src[:2])[1].tolist()
    assert d.delete(t) == do.delete(t)[1]
    assert d.evict(2) == do.evict(2)[1]
    for o, g in ((po, p), (do, d), (ho, h)):
        _same_state(o, g)
    with pytest.raises(MemPoolError) as e:
        d.alloc_mem(13)
    assert e.value.code == M.MP_ENOMEM
    for g in (p, d, h):
        g.close()
