"""GPU parity at the full sizes of configurations 2-5, in the launch shape bench.py times
(batched, asynchronous calls on per-pool streams).

At these sizes a dense CPU copy of the pools does not fit a test, so the check is split:
  * control plane (block ids handed out, match results, pool statistics): the oracle runs the
    very same calls on pools of the same block size and block count but one-element-wide
    fragments -- allocation, index and eviction do not depend on the fragment size;
  * data plane: for a seeded sample of table entries the source blocks are fetched from the
    GPU, pushed through the oracle's own gather / scatter, and compared byte for byte with the
    destination blocks on the GPU;
  * every entry: a position-weighted 64-bit checksum of EVERY destination fragment named by the
    table (all entries, all planes), taken on the GPU, must equal the checksum of its source
    fragment -- so a defect that hits only entries outside the sample (a grid tail, an entry
    behind a staging-round boundary) cannot pass;
  * untouched blocks: the same checksums of every (plane, block) fragment of the destination
    pool, taken before and after, must be unchanged outside the destination table.
"""
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


def fill_random(pool):
    """Any bytes will do for a copy; int32 noise is the fastest fill torch has."""
    v = pool.mem.view(torch.int32)
    step = 1 << 28
    for off in range(0, v.numel(), step):
        v[off:off + step].random_()
    torch.cuda.synchronize()


_WEIGHTS = {}


def _weights(n_words, device):
    """One odd 64-bit multiplier per 8-byte word of a fragment, so that words that swap places
    inside a fragment change the checksum (a plain sum would not notice)."""
    key = (n_words, str(device))
    if key not in _WEIGHTS:
        j = torch.arange(n_words, dtype=torch.int64, device=device)
        _WEIGHTS[key] = (2 * j + 1) * -7046029254386353131          # 0x9E3779B97F4A7C15, wraps mod 2^64
    return _WEIGHTS[key]


def checksums(pool, ids=None):
    """[2L, n] checksums sum_j word_j * odd_j (mod 2^64) of the fragments of blocks `ids` (all
    blocks if None), computed where the pool lives, plane by plane to bound the temporaries."""
    L2, w = 2 * pool.geom[0], pool.F // 8
    dev = pool.mem.device
    idx = None if ids is None else torch.as_tensor(np.asarray(ids, dtype=np.int64), device=dev)
    n = pool.NB if idx is None else idx.numel()
    W = _weights(w, dev)
    out = torch.empty(L2, n, dtype=torch.int64, device=dev)
    words = pool.mem.view(torch.int64)
    for p in range(L2):
        if pool.aggregated:
            plane = words.view(pool.NB, L2, w)[:, p, :]
        else:
            plane = words.view(L2, pool.NB, w)[p]
        step = max(1, (1 << 27) // w)                                  # 1 GiB of words at a time
        for lo in range(0, n, step):
            rows = plane[lo:lo + step] if idx is None else plane[idx[lo:lo + step]]
            out[p, lo:lo + step] = (rows * W).sum(dim=1)
    return out


def check_all_entries(src, dst, src_tbl, dst_tbl, dst_sums=None):
    """Every fragment of every table entry arrived: checksum(dst fragment) == checksum(src fragment)."""
    torch.cuda.synchronize()
    if len(src_tbl) == 0:
        return
    want = checksums(src, src_tbl).cpu()
    if dst_sums is None:
        got = checksums(dst, dst_tbl).cpu()
    else:
        got = dst_sums[:, torch.as_tensor(np.asarray(dst_tbl, dtype=np.int64), device=dst_sums.device)].cpu()
    bad = (want != got).nonzero()
    assert bad.numel() == 0, f"{bad.shape[0]} fragments differ, first (plane, entry) = {bad[0].tolist()}"


def blocks_of(pool, ids):
    """[len(ids), 2L, F] bytes of the given blocks, on the host."""
    L2 = 2 * pool.geom[0]
    idx = torch.as_tensor(np.asarray(ids, dtype=np.int64), device=pool.mem.device)
    if not pool.aggregated:
        x = pool.mem.view(L2, pool.NB, pool.F)[:, idx, :].permute(1, 0, 2)
    else:
        x = pool.mem.view(pool.NB, L2, pool.F)[idx]
    return x.contiguous().cpu().numpy()


def check_sample(geom, src, dst, src_tbl, dst_tbl, rng, k=24):
    """Oracle-computed destination blocks for k sampled table entries == GPU destination blocks."""
    torch.cuda.synchronize()
    n = len(src_tbl)
    if n == 0:
        return
    pick = rng.choice(n, size=min(k, n), replace=False)
    L, H, D, bs, e = geom
    k = len(pick)
    src_blocks = blocks_of(src, src_tbl[pick])                       # [k, 2L, F]
    o_src = O.OraclePool(L, H, D, bs, e, k,
                         data=np.ascontiguousarray(src_blocks.transpose(1, 0, 2)).reshape(-1))
    o_dst = O.OraclePool(L, H, D, bs, e, k)
    o_src.alloc(k)
    perm = rng.permutation(k).astype(np.int32)
    o_dst.alloc(k)
    rc, _ = O.transfer(o_src, o_dst, np.arange(k), perm, flags=O.DST_GIVEN)
    assert rc == 0
    want = o_dst.data.reshape(2 * L, k, src.F).transpose(1, 0, 2)[perm]   # entry j -> block perm[j]
    got = blocks_of(dst, dst_tbl[pick])
    assert np.array_equal(got, want)


class Mirror:
    """Oracle pools with one-element fragments that replay the control plane."""

    def __init__(self, bs, NB_src, NB_dst):
        self.src = O.OraclePool(1, 1, 8, bs, 1, NB_src)
        self.dst = O.OraclePool(1, 1, 8, bs, 1, NB_dst)
        self.src.alloc(NB_src)


def make_pools(gpu, g, NB_src, NB_dst, staging_blocks, layouts=(0, 0)):
    M, TorchPool = gpu
    geom = (g.L, g.H, g.D, g.bs, g.e)
    s_src, s_dst = torch.cuda.Stream(), torch.cuda.Stream()
    src = TorchPool(*geom, NB_src, staging_blocks=staging_blocks, stream=s_src, layout=layouts[0])
    dst = TorchPool(*geom, NB_dst, stream=s_dst, layout=layouts[1])
    fill_random(src)
    fill_random(dst)
    assert M.mp_alloc(src.h, NB_src)[0] == 0
    return geom, src, dst


def release(*pools):
    for p in pools:
        p.free_memory()               # also checks the canary bands around pool and staging
    torch.cuda.empty_cache()


def test_config3_multiturn_sessions(gpu):
    """Llama-3-8B GQA shape, 16384-block pools, 64 sessions x 4 turns exactly as bench.py runs
    them: mp_match_batch (pin) then asynchronous mp_transfer_with_insert_batch per turn."""
    M, TorchPool = gpu
    g = W.CONFIGS[3]
    geom, src, dst = make_pools(gpu, g, g.NB, g.NB, staging_blocks=64 * 50)
    mir = Mirror(g.bs, g.NB, g.NB)
    rng = np.random.default_rng(33)
    sessions = W.multiturn_sessions(seed=3)
    flags = M.MP_EVICT_ON_DEMAND | M.MP_ASYNC
    held, held_o, moved = [], [], []
    for t in range(4):
        prompts = [sessions[s][t] for s in range(64)]
        toks, tok_off = W.csr(prompts)
        nblk = np.array([(len(p) + g.bs - 1) // g.bs for p in prompts], np.uint32)
        cap_off = np.concatenate([[0], np.cumsum(nblk)]).astype(np.uint32)
        rc, mb, m = M.mp_match_batch(dst.h, toks, tok_off, cap_off, M.MP_MATCH_PIN)
        assert rc == 0
        mo = [mir.dst.match(p, flags=O.MATCH_PIN)[1] for p in prompts]
        assert m.tolist() == [len(x) for x in mo]
        assert all(mb[cap_off[r]:cap_off[r] + m[r]].tolist() == mo[r].tolist() for r in range(64))
        blk_off = np.concatenate([[0], np.cumsum(nblk - m)]).astype(np.uint32)
        src_tbl = rng.permutation(g.NB)[: int(blk_off[-1])].astype(np.int32)
        before = checksums(dst)
        rc, d = M.mp_transfer_with_insert_batch(src.h, dst.h, toks, tok_off, m, src_tbl, blk_off, flags)
        assert rc == 0, M.mp_last_error(src.h)
        rco, d_o = O.transfer_with_insert_batch(mir.src, mir.dst, toks, tok_off, m, src_tbl, blk_off,
                                                flags=O.EVICT_ON_DEMAND)
        assert rco == 0 and d.tolist() == d_o.tolist()
        check_sample(geom, src, dst, src_tbl, d, rng)
        after = checksums(dst)
        check_all_entries(src, dst, src_tbl, d, dst_sums=after)
        untouched = torch.ones(g.NB, dtype=torch.bool, device="cuda")
        untouched[torch.as_tensor(d.astype(np.int64), device="cuda")] = False
        assert torch.equal(before[:, untouched], after[:, untouched])
        assert dst.stats() == mir.dst.stats()
        moved.append(len(d))
    # the volumes of the recipe: first turn moves whole prompts, later turns only the new suffix
    assert moved[0] == sum((len(sessions[s][0]) + 15) // 16 for s in range(64))
    assert all(moved[t] < sum((len(sessions[s][t]) + 15) // 16 for s in range(64)) for t in (1, 2, 3))
    release(src, dst)


@pytest.mark.parametrize("direct", [0, 1])
def test_config3_one_call_per_request(gpu, direct):
    """The per-request flavour bench.py also times, at the full pool size: mp_match (pin) and one
    asynchronous mp_transfer_with_insert per request -- 24-50 blocks each, so the block ids travel
    in the kernel arguments -- staged and fused, every entry and plane checked per request."""
    M, TorchPool = gpu
    g = W.CONFIGS[3]
    geom, src, dst = make_pools(gpu, g, g.NB, g.NB, staging_blocks=64)
    mir = Mirror(g.bs, g.NB, g.NB)
    rng = np.random.default_rng(34 + direct)
    sessions = W.multiturn_sessions(seed=3)
    flags = M.MP_EVICT_ON_DEMAND | M.MP_ASYNC | (M.MP_DIRECT if direct else 0)
    before = checksums(dst)
    touched = torch.zeros(g.NB, dtype=torch.bool, device="cuda")
    for t in range(2):
        perm = rng.permutation(g.NB).astype(np.int32)
        at = 0
        for s in range(0, 64, 3):                                   # 22 requests per turn
            p = sessions[s][t]
            nblk = (len(p) + g.bs - 1) // g.bs
            rc, m = M.mp_match(dst.h, p, nblk, M.MP_MATCH_PIN)
            rco, mo = mir.dst.match(p, flags=O.MATCH_PIN)
            assert rc == rco == 0 and m.tolist() == mo.tolist()
            n = nblk - len(m)
            assert 0 < n <= 192
            src_tbl = perm[at:at + n]
            at += n
            rc, d = M.mp_transfer_with_insert(src.h, dst.h, p, len(m), src_tbl, flags=flags)
            assert rc == 0, M.mp_last_error(src.h)
            rco, d_o = O.transfer_with_insert(mir.src, mir.dst, p, len(mo), src_tbl, flags=O.EVICT_ON_DEMAND)
            assert rco == 0 and d.tolist() == d_o.tolist()
            check_all_entries(src, dst, src_tbl, d)
            if s % 12 == 0:
                check_sample(geom, src, dst, src_tbl, d, rng, k=8)
            touched[torch.as_tensor(d.astype(np.int64), device="cuda")] = True
            assert dst.stats() == mir.dst.stats()
    after = checksums(dst)
    assert torch.equal(before[:, ~touched], after[:, ~touched])      # nothing else was written
    assert int(touched.sum()) > 800
    release(src, dst)


@pytest.mark.parametrize("direct", [0, 1])
def test_config3_layer_by_layer(gpu, direct):
    """mp_transfer_layers at the full pool size with a turn-sized table (the by-layer mode bench.py
    times): layer ranges of one, two and five layers into explicit destinations; the planes of
    the moved layers equal the source's for every entry, every other plane and block is unchanged."""
    M, TorchPool = gpu
    g = W.CONFIGS[3]
    geom, src, dst = make_pools(gpu, g, g.NB, g.NB, staging_blocks=64 * 50)
    rng = np.random.default_rng(36 + direct)
    n = 2300
    rc, d = M.mp_alloc(dst.h, n)
    assert rc == 0
    src_sums = checksums(src)
    flags = M.MP_ASYNC | (M.MP_DIRECT if direct else 0)
    for l0, l1 in ((0, 1), (13, 15), (27, 32), (31, 32)):
        src_tbl = rng.permutation(g.NB)[:n].astype(np.int32)
        before = checksums(dst)
        pick = rng.choice(n, size=6, replace=False)
        src_blocks, dst_before = blocks_of(src, src_tbl[pick]), blocks_of(dst, d[pick])
        assert M.mp_transfer_layers(src.h, dst.h, src_tbl, d, l0, l1, flags) == 0, M.mp_last_error(src.h)
        torch.cuda.synchronize()
        after = checksums(dst)
        # the sampled entries through the oracle's own by-layer transfer, byte for byte
        L, H, D, bs, e = geom
        as_pool = lambda blocks: np.ascontiguousarray(blocks.transpose(1, 0, 2)).reshape(-1)
        o_src = O.OraclePool(L, H, D, bs, e, 6, data=as_pool(src_blocks))
        o_dst = O.OraclePool(L, H, D, bs, e, 6, data=as_pool(dst_before))
        o_src.alloc(6)
        o_dst.alloc(6)
        assert O.transfer_layers(o_src, o_dst, np.arange(6), np.arange(6), l0, l1) == 0
        assert np.array_equal(blocks_of(dst, d[pick]), o_dst.data.reshape(2 * L, 6, src.F).transpose(1, 0, 2))
        si = torch.as_tensor(src_tbl.astype(np.int64), device="cuda")
        di = torch.as_tensor(d.astype(np.int64), device="cuda")
        want = before.clone()
        want[2 * l0:2 * l1, di] = src_sums[2 * l0:2 * l1][:, si]
        bad = (want != after).nonzero()
        assert bad.numel() == 0, f"{bad.shape[0]} fragments differ, first (plane, block) = {bad[0].tolist()}"
    release(src, dst)


@pytest.mark.parametrize("layouts,direct", [((2, 2), 0), ((2, 0), 1), ((0, 2), 0), ((2, 2), 1)])
def test_config3_aggregated_pools(gpu, layouts, direct):
    """HBM pools in the aggregated layout (one or both ends) at the full size of config 3: one
    turn-sized asynchronous transfer; every entry and plane, and everything outside the table."""
    M, TorchPool = gpu
    g = W.CONFIGS[3]
    geom, src, dst = make_pools(gpu, g, g.NB, g.NB, staging_blocks=2400, layouts=layouts)
    rng = np.random.default_rng(40 + direct)
    mir = Mirror(g.bs, g.NB, g.NB)
    for n in (2300, 1266):
        src_tbl = rng.permutation(g.NB)[:n].astype(np.int32)
        before = checksums(dst)
        rc, d = M.mp_transfer(src.h, dst.h, src_tbl, flags=M.MP_ASYNC | (M.MP_DIRECT if direct else 0))
        rco, d_o = O.transfer(mir.src, mir.dst, src_tbl)
        assert rc == rco == 0 and d.tolist() == d_o.tolist(), M.mp_last_error(src.h)
        check_sample(geom, src, dst, src_tbl, d, rng, k=8)
        after = checksums(dst)
        check_all_entries(src, dst, src_tbl, d, dst_sums=after)
        untouched = torch.ones(g.NB, dtype=torch.bool, device="cuda")
        untouched[torch.as_tensor(d.astype(np.int64), device="cuda")] = False
        assert torch.equal(before[:, untouched], after[:, untouched])
    release(src, dst)


def test_config2_lognormal_requests(gpu):
    """Llama-2-7B shape (128 KiB fragments), 8192-block pools (64 GiB each), 16 requests with
    log-normal lengths, fragmented tables; per-request calls and one batched call."""
    M, TorchPool = gpu
    g = W.CONFIGS[2]
    geom, src, dst = make_pools(gpu, g, g.NB, g.NB, staging_blocks=100)
    mir = Mirror(g.bs, g.NB, g.NB)
    rng = np.random.default_rng(22)
    # fragment the destination free list: allocate everything, release in random order
    ids = M.mp_alloc(dst.h, g.NB)[1]
    mir.dst.alloc(g.NB)
    order = rng.permutation(g.NB).astype(np.int32)
    assert M.mp_free(dst.h, ids[order]) == mir.dst.free(ids[order]) == 0
    lengths = W.lognormal_lengths()
    prompts = W.random_prompts(2, lengths, g.vocab)
    for r, p in enumerate(prompts[:6]):          # per-request calls (several staging rounds for long ones)
        nb = (len(p) + g.bs - 1) // g.bs
        tbl = rng.permutation(g.NB)[:nb].astype(np.int32)
        rc, d = M.mp_transfer_with_insert(src.h, dst.h, p, 0, tbl)
        rco, d_o = O.transfer_with_insert(mir.src, mir.dst, p, 0, tbl)
        assert rc == rco == 0 and d.tolist() == d_o.tolist()
        check_sample(geom, src, dst, tbl, d, rng, k=8)
        check_all_entries(src, dst, tbl, d)
        assert M.mp_match(dst.h, p, nb)[1].tolist() == mir.dst.match(p)[1].tolist() == d[: len(p) // g.bs].tolist()
    rest = prompts[6:]
    toks, tok_off = W.csr(rest)
    nblk = np.array([(len(p) + g.bs - 1) // g.bs for p in rest], np.uint32)
    blk_off = np.concatenate([[0], np.cumsum(nblk)]).astype(np.uint32)
    tbl = rng.permutation(g.NB)[: int(blk_off[-1])].astype(np.int32)
    before = checksums(dst)
    rc, d = M.mp_transfer_with_insert_batch(src.h, dst.h, toks, tok_off, np.zeros(len(rest), np.uint32),
                                            tbl, blk_off, M.MP_ASYNC)
    rco, d_o = O.transfer_with_insert_batch(mir.src, mir.dst, toks, tok_off, np.zeros(len(rest), np.uint32),
                                            tbl, blk_off)
    assert rc == rco == 0 and d.tolist() == d_o.tolist()
    check_sample(geom, src, dst, tbl, d, rng, k=16)
    after = checksums(dst)
    check_all_entries(src, dst, tbl, d, dst_sums=after)
    untouched = torch.ones(g.NB, dtype=torch.bool, device="cuda")
    untouched[torch.as_tensor(d.astype(np.int64), device="cuda")] = False
    assert torch.equal(before[:, untouched], after[:, untouched])
    assert dst.stats() == mir.dst.stats()
    release(src, dst)


def test_config4_long_context_with_eviction(gpu):
    """Llama-2-13B shape (320 KiB fragments, 25 MiB records), 32 requests of 16384 tokens, 90 %
    sharing an 8192-token prefix; the 4096-block destination overflows and evicts on demand."""
    M, TorchPool = gpu
    g = W.CONFIGS[4]
    NB_src, NB_dst = 1024, 4096
    geom, src, dst = make_pools(gpu, g, NB_src, NB_dst, staging_blocks=128)
    mir = Mirror(g.bs, NB_src, NB_dst)
    rng = np.random.default_rng(44)
    moved = []
    for r, p in enumerate(W.long_context_requests()):
        nb = len(p) // g.bs
        rc, m = M.mp_match(dst.h, p, nb, M.MP_MATCH_PIN)
        rco, mo = mir.dst.match(p, flags=O.MATCH_PIN)
        assert rc == rco == 0 and m.tolist() == mo.tolist()
        tbl = rng.permutation(NB_src)[: nb - len(m)].astype(np.int32)
        fl = M.MP_EVICT_ON_DEMAND | (M.MP_ASYNC if r % 2 else 0)
        before = checksums(dst) if r % 8 == 0 else None
        rc, d = M.mp_transfer_with_insert(src.h, dst.h, p, len(m), tbl, flags=fl)
        rco, d_o = O.transfer_with_insert(mir.src, mir.dst, p, len(mo), tbl, flags=O.EVICT_ON_DEMAND)
        assert rc == rco == 0 and d.tolist() == d_o.tolist(), M.mp_last_error(src.h)
        if r % 4 == 0:
            check_sample(geom, src, dst, tbl, d, rng, k=4)
        check_all_entries(src, dst, tbl, d)
        if before is not None:
            untouched = torch.ones(NB_dst, dtype=torch.bool, device="cuda")
            untouched[torch.as_tensor(d.astype(np.int64), device="cuda")] = False
            assert torch.equal(before[:, untouched], checksums(dst)[:, untouched])
        ids = np.concatenate([m, d])
        assert M.mp_free(dst.h, ids) == mir.dst.free(ids) == 0          # the request finishes
        assert dst.stats() == mir.dst.stats()
        moved.append(len(d))
    assert sorted(set(moved)) == [256, 512] and moved.count(256) == 28   # 29 sharers, the first moves 512
    assert dst.stats()["n_free"] < 512                                   # the pool did overflow
    release(src, dst)


def test_config5_tp_share_and_host_tier(gpu):
    """One GPU's share of a 70B model: 160 fragments of 4 KiB per block.  256 requests of 2048
    tokens in one batched call through a staging buffer eight times smaller than the batch, then
    a slice of it out to a pinned-host pool and back."""
    M, TorchPool = gpu
    g = W.CONFIGS[5]
    geom, src, dst = make_pools(gpu, g, g.NB, g.NB, staging_blocks=4096)
    mir = Mirror(g.bs, g.NB, g.NB)
    rng = np.random.default_rng(55)
    prompts = W.random_prompts(5, [2048] * 256, g.vocab)
    toks, tok_off = W.csr(prompts)
    blk_off = (np.arange(257) * 128).astype(np.uint32)
    tbl = rng.permutation(g.NB)[: 256 * 128].astype(np.int32)
    before = checksums(dst)
    first = np.zeros(256, np.uint32)
    rc, d = M.mp_transfer_with_insert_batch(src.h, dst.h, toks, tok_off, first, tbl, blk_off, M.MP_ASYNC)
    rco, d_o = O.transfer_with_insert_batch(mir.src, mir.dst, toks, tok_off, first, tbl, blk_off)
    assert rc == rco == 0 and d.tolist() == d_o.tolist(), M.mp_last_error(src.h)
    check_sample(geom, src, dst, tbl, d, rng, k=64)
    after = checksums(dst)
    check_all_entries(src, dst, tbl, d, dst_sums=after)
    untouched = torch.ones(g.NB, dtype=torch.bool, device="cuda")
    untouched[torch.as_tensor(d.astype(np.int64), device="cuda")] = False
    assert torch.equal(before[:, untouched], after[:, untouched])
    assert dst.stats() == mir.dst.stats()
    rc, mb, m = M.mp_match_batch(dst.h, toks, tok_off, blk_off)
    assert rc == 0 and m.tolist() == [128] * 256 and mb.tolist() == d.tolist()
    for p in prompts:
        mir.dst.match(p)

    # host tier: 2048 blocks (1.25 GiB) out to pinned memory and back in
    host = TorchPool(*geom, 2048, tier=M.MP_TIER_HOST_PINNED)
    o_host = O.OraclePool(1, 1, 8, g.bs, 1, 2048, tier=O.TIER_HOST)
    pick = rng.permutation(256 * 128)[:2048]
    rc, h_ids = M.mp_transfer(dst.h, host.h, d[pick])       # dst has no staging -> refused
    assert rc == M.MP_ENOSTAGING
    rc, h_ids = M.mp_transfer(src.h, host.h, tbl[pick])
    rco, h_o = O.transfer(mir.src, o_host, tbl[pick])
    assert rc == rco == 0 and h_ids.tolist() == h_o.tolist(), M.mp_last_error(src.h)
    check_sample(geom, src, host, tbl[pick], h_ids, rng, k=32)
    check_all_entries(src, host, tbl[pick], h_ids)
    back = TorchPool(*geom, 2048, staging_blocks=256)
    rc, b_ids = M.mp_transfer(host.h, back.h, h_ids)
    assert rc == 0, M.mp_last_error(host.h)
    check_sample(geom, host, back, h_ids, b_ids, rng, k=32)
    check_sample(geom, src, back, tbl[pick], b_ids, rng, k=32)   # round trip = identity
    check_all_entries(src, back, tbl[pick], b_ids)

    # swap: the receiver's cache moves its 1500 coldest blocks down to a host pool (zero-copy
    # kernel), then one prompt is brought back up
    assert M.mp_free(dst.h, d) == mir.dst.free(d) == 0
    low = TorchPool(*geom, 4096, tier=M.MP_TIER_HOST_PINNED)
    o_low = O.OraclePool(1, 1, 8, g.bs, 1, 4096, tier=O.TIER_HOST)
    assert M.mp_swap_out(dst.h, low.h, 1500, M.MP_DIRECT) == O.swap_out(mir.dst, o_low, 1500) == (0, 1500)
    assert dst.stats() == mir.dst.stats() and low.stats() == o_low.stats()
    hit = [r for r in range(256) if len(o_low.match(prompts[r])[1])]
    assert hit == [r for r in range(256) if len(M.mp_match(low.h, prompts[r], 128)[1])]
    assert len(hit) == 12                                        # 11 whole prompts and part of a 12th
    for r in (hit[0], hit[-1]):
        rc, low_ids = M.mp_match(low.h, prompts[r], 128)
        assert rc == 0 and low_ids.tolist() == o_low.match(prompts[r])[1].tolist() and len(low_ids) == 128
        sl = tbl[r * 128:(r + 1) * 128]
        check_sample(geom, src, low, sl, low_ids, rng, k=32)     # src -> dst -> host tier, bytes intact
        check_all_entries(src, low, sl, low_ids)
    r = hit[0]
    assert len(M.mp_match(dst.h, prompts[r], 128)[1]) == len(mir.dst.match(prompts[r])[1]) == 0
    low_ids = M.mp_match(low.h, prompts[r], 128)[1]
    assert low_ids.tolist() == o_low.match(prompts[r])[1].tolist()
    rc, up = M.mp_swap_in(low.h, dst.h, low_ids, M.MP_DIRECT)
    rco, up_o = O.swap_in(o_low, mir.dst, low_ids)
    assert rc == rco == 0 and up.tolist() == up_o.tolist(), M.mp_last_error(low.h)
    assert M.mp_match(dst.h, prompts[r], 128)[1].tolist() == up.tolist()
    mir.dst.match(prompts[r])
    check_sample(geom, src, dst, tbl[r * 128:(r + 1) * 128], up, rng, k=32)
    check_all_entries(src, dst, tbl[r * 128:(r + 1) * 128], up)
    assert M.mp_free(dst.h, up) == mir.dst.free(up) == 0
    assert dst.stats() == mir.dst.stats() and low.stats() == o_low.stats()
    release(src, dst, host, back, low)


@pytest.mark.parametrize("cfg,NB", [(2, 64), (3, 256), (4, 24), (5, 512)])
@pytest.mark.parametrize("direct", [0, 1])
def test_exact_geometry_dense_compare(gpu, cfg, NB, direct):
    """The exact L / F of each configuration with few enough blocks (0.3-0.6 GiB a pool) that the
    oracle holds dense copies: after batched asynchronous transfers in the default launch shape,
    staged or fused, every byte of the destination pool, every id and the statistics agree."""
    M, TorchPool = gpu
    g = W.CONFIGS[cfg]
    geom, src, dst = make_pools(gpu, g, NB, NB, staging_blocks=max(2, NB // 5))
    o_src = O.OraclePool(*geom, NB, data=src.bytes())
    o_dst = O.OraclePool(*geom, NB, data=dst.bytes())
    o_src.alloc(NB)
    rng = np.random.default_rng(1000 + cfg)
    flags = M.MP_EVICT_ON_DEMAND | M.MP_ASYNC | (M.MP_DIRECT if direct else 0)
    n_req = 6
    shared = rng.integers(0, g.vocab, 2 * g.bs, dtype=np.uint32)
    for rnd in range(3):                  # later rounds find the shared prefix and must evict
        lens = rng.integers(1, max(2, NB // 8) * g.bs, n_req)
        prompts = [np.concatenate([shared, rng.integers(0, g.vocab, int(n), dtype=np.uint32)])
                   for n in lens]
        toks, tok_off = W.csr(prompts)
        nblk = np.array([(len(p) + g.bs - 1) // g.bs for p in prompts], np.uint32)
        cap_off = np.concatenate([[0], np.cumsum(nblk)]).astype(np.uint32)
        rc, mb, m = M.mp_match_batch(dst.h, toks, tok_off, cap_off, M.MP_MATCH_PIN)
        mo = [o_dst.match(p, flags=O.MATCH_PIN)[1] for p in prompts]
        assert rc == 0 and m.tolist() == [len(x) for x in mo]
        blk_off = np.concatenate([[0], np.cumsum(nblk - m)]).astype(np.uint32)
        src_tbl = rng.integers(0, NB, int(blk_off[-1])).astype(np.int32)
        rc, d = M.mp_transfer_with_insert_batch(src.h, dst.h, toks, tok_off, m, src_tbl, blk_off, flags)
        rco, d_o = O.transfer_with_insert_batch(o_src, o_dst, toks, tok_off, m, src_tbl, blk_off,
                                                flags=O.EVICT_ON_DEMAND)
        assert rc == rco, (rnd, rc, rco, M.mp_last_error(src.h))
        ids = [mb[cap_off[r]:cap_off[r] + m[r]] for r in range(n_req)]
        if rc == 0:
            assert d.tolist() == d_o.tolist()
            ids.append(d)
        ids = np.concatenate(ids).astype(np.int32)
        assert M.mp_free(dst.h, ids) == o_dst.free(ids) == 0
        assert dst.stats() == o_dst.stats()
        assert np.array_equal(dst.bytes(), o_dst.data), (cfg, rnd)
    assert np.array_equal(src.bytes(), o_src.data)
    release(src, dst)
