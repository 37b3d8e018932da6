"""Pins for the oracle's copy-by-block-table: closed forms through numpy's own reshape /
transpose / take, round-trip identity, untouched-block invariant and the fragment counts
the paper states (section 5.2: bs tokens = 2*L discrete blocks = one aggregated block)."""
import numpy as np
import pytest

from oracle import oracle as O
from paper_2406_17565_amd import workloads as W

GEOMS = [  # (L, H, D, bs, e)
    (2, 2, 64, 16, 2),
    (3, 1, 8, 4, 2),     # F = 64 bytes, ragged everything
    (1, 5, 24, 2, 2),    # F = 480: a multiple of 16 but not of 256
]


def _pool(geom, NB, seed, tier=O.TIER_HBM):
    L, H, D, bs, e = geom
    rng = np.random.default_rng(seed)
    data = W.kv_bytes(rng, 2 * L * NB * bs * H * D * e, "fp16")
    return O.OraclePool(L, H, D, bs, e, NB, tier=tier, data=data)


@pytest.mark.parametrize("geom", GEOMS)
def test_sizes_follow_the_paper(geom):
    L, H, D, bs, e = geom
    p = _pool(geom, 8, 0)
    assert p.F == bs * H * D * e
    assert p.B == 2 * L * p.F                      # aggregated block = 2*L small blocks
    assert p.data.size == 8 * p.B
    # discrete layout: fragments of one block are NB*F apart, K before V, layer-major
    assert p.fragment_offset(0, 0, 3) == 3 * p.F
    assert p.fragment_offset(0, 1, 0) == 8 * p.F
    assert p.fragment_offset(1, 0, 0) == 2 * 8 * p.F
    h = _pool(geom, 8, 0, tier=O.TIER_HOST)
    assert h.fragment_offset(0, 0, 3) == 3 * p.B   # aggregated layout: block = one record
    assert h.fragment_offset(0, 1, 0) == p.F
    assert h.fragment_offset(1, 0, 0) == 2 * p.F
    a = O.OraclePool(L, H, D, bs, e, 8, layout=2)   # an HBM pool that opted into aggregation
    assert [a.fragment_offset(*x) for x in ((0, 0, 3), (0, 1, 0), (1, 0, 0))] == [3 * p.B, p.F, 2 * p.F]
    with pytest.raises(ValueError):
        O.OraclePool(L, H, D, bs, e, 8, tier=O.TIER_HOST, layout=1)


@pytest.mark.parametrize("geom", GEOMS)
def test_identity_table_is_a_permutation_of_axes(geom):
    L = geom[0]
    n = 6
    p = _pool(geom, n, 1)
    staging = p.gather(np.arange(n))
    want = p.data.reshape(L, 2, n, p.F).transpose(2, 0, 1, 3)
    assert np.array_equal(staging.reshape(n, L, 2, p.F), want)


@pytest.mark.parametrize("geom", GEOMS)
def test_gather_equals_numpy_take(geom):
    L = geom[0]
    NB = 37
    p = _pool(geom, NB, 2)
    rng = np.random.default_rng(3)
    tbl = rng.integers(0, NB, 50).astype(np.int32)          # duplicates allowed on the source side
    staging = p.gather(tbl)
    want = np.take(p.data.reshape(L, 2, NB, p.F), tbl, axis=2).transpose(2, 0, 1, 3)
    assert np.array_equal(staging.reshape(len(tbl), L, 2, p.F), want)
    assert p.gather(np.zeros(0, np.int32)).size == 0


@pytest.mark.parametrize("geom", GEOMS)
def test_scatter_then_gather_round_trip_and_untouched(geom):
    L = geom[0]
    NB = 29
    dst = _pool(geom, NB, 4)
    before = dst.data.copy()
    rng = np.random.default_rng(5)
    tbl = W.random_table(rng, NB, 11)
    staging = W.kv_bytes(rng, 11 * dst.B, "fp16")
    assert dst.scatter(tbl, staging) == 0
    assert np.array_equal(dst.gather(tbl), staging)           # gather(scatter(S,t),t) == S
    touched = np.zeros(NB, bool)
    touched[tbl] = True
    a = dst.data.reshape(L, 2, NB, dst.F)
    b = before.reshape(L, 2, NB, dst.F)
    assert np.array_equal(a[:, :, ~touched], b[:, :, ~touched])
    assert not np.array_equal(a[:, :, touched], b[:, :, touched])


def test_scatter_of_gather_into_zero_pool():
    geom = GEOMS[0]
    L = geom[0]
    NB = 16
    src = _pool(geom, NB, 6)
    zero = O.OraclePool(*geom, NB)
    rng = np.random.default_rng(7)
    tbl = W.random_table(rng, NB, 5)
    zero.scatter(tbl, src.gather(tbl))
    a = zero.data.reshape(L, 2, NB, src.F)
    b = src.data.reshape(L, 2, NB, src.F)
    mask = np.zeros(NB, bool)
    mask[tbl] = True
    assert np.array_equal(a[:, :, mask], b[:, :, mask])
    assert not a[:, :, ~mask].any()


def test_transfer_moves_bytes_exactly_including_nan_payloads():
    geom = GEOMS[0]
    L = geom[0]
    src = _pool(geom, 8, 8)
    F = src.F
    s4 = src.data.reshape(L, 2, 8, F)
    s4[:, :, 5, :] = W.special_half_patterns(F)           # NaN payloads, -0, inf, denormal
    dst = _pool(geom, 12, 9)
    before = dst.data.copy()
    rc, ids = src.alloc(8)
    assert rc == 0
    rc, d = O.transfer(src, dst, [5, 2, 5], None)
    assert rc == 0 and d.tolist() == [0, 1, 2]            # fresh pool hands out 0,1,2
    d4 = dst.data.reshape(L, 2, 12, F)
    for i, sb in enumerate([5, 2, 5]):
        assert np.array_equal(d4[:, :, d[i]], s4[:, :, sb])
    assert np.array_equal(d4[:, :, 3:], before.reshape(L, 2, 12, F)[:, :, 3:])


def test_host_tier_pool_holds_records():
    geom = GEOMS[1]
    src = _pool(geom, 10, 10)
    src.alloc(10)
    host = O.OraclePool(*geom, 6, tier=O.TIER_HOST)
    rc, d = O.transfer(src, host, [7, 1, 4], None)
    assert rc == 0
    rec = src.gather([7, 1, 4]).reshape(3, src.B)
    for i in range(3):
        assert np.array_equal(host.data.reshape(6, src.B)[d[i]], rec[i])
    # and back (swap-in direction)
    back = O.OraclePool(*geom, 10)
    rc, d2 = O.transfer(host, back, d, None)
    assert rc == 0
    assert np.array_equal(back.gather(d2), src.gather([7, 1, 4]))


def test_transfer_within_one_pool_reads_everything_before_writing():
    geom = GEOMS[1]
    p = _pool(geom, 6, 12)
    p.alloc(6)
    before = p.gather(np.arange(6))
    rc, _ = O.transfer(p, p, [0, 1, 2], [1, 2, 0], flags=O.DST_GIVEN)  # a rotation
    assert rc == 0
    after = p.gather(np.arange(6)).reshape(6, p.B)
    b = before.reshape(6, p.B)
    assert np.array_equal(after[1], b[0]) and np.array_equal(after[2], b[1])
    assert np.array_equal(after[0], b[2]) and np.array_equal(after[3:], b[3:])


def test_transfer_layers_is_a_slice_of_the_transfer():
    geom = (5, 2, 8, 4, 2)                       # L = 5
    L = geom[0]
    rng = np.random.default_rng(21)
    s_ids, d_ids = [7, 2, 7, 9], [3, 0, 5, 1]
    for l0, l1 in ((0, 1), (2, 5), (1, 3), (0, 5)):
        src, dst = _pool(geom, 12, 20), _pool(geom, 8, 21)
        src.alloc(12)
        dst.alloc(6)
        before = dst.data.copy().reshape(L, 2, 8, dst.F)
        assert O.transfer_layers(src, dst, s_ids, d_ids, l0, l1) == 0
        after = dst.data.reshape(L, 2, 8, dst.F)
        s4 = src.data.reshape(L, 2, 12, src.F)
        assert np.array_equal(after[l0:l1][:, :, d_ids], s4[l0:l1][:, :, s_ids])
        mask = np.ones((L, 2, 8), bool)
        mask[l0:l1, :, d_ids] = False
        assert np.array_equal(after[mask], before[mask])          # other layers / blocks untouched
    # ranges that tile [0, L) add up to the whole-block transfer
    src, a, b = _pool(geom, 12, 20), _pool(geom, 8, 21), _pool(geom, 8, 21)
    src.alloc(12)
    a.alloc(6)
    b.alloc(6)
    for l0, l1 in ((3, 5), (0, 2), (2, 3)):
        assert O.transfer_layers(src, a, s_ids, d_ids, l0, l1) == 0
    assert O.transfer(src, b, s_ids, d_ids, flags=O.DST_GIVEN)[0] == 0
    assert np.array_equal(a.data, b.data)
    # errors
    assert O.transfer_layers(src, a, s_ids, d_ids, 2, 2) == O.EINVAL
    assert O.transfer_layers(src, a, s_ids, d_ids, 4, 6) == O.EINVAL
    assert O.transfer_layers(src, a, s_ids, [3, 3, 5, 1], 0, 1) == O.EINVAL
    assert O.transfer_layers(src, a, s_ids, [3, 0, 5, 7], 0, 1) == O.EINVAL   # 7 not held
    assert np.array_equal(a.data, b.data)


def test_aggregated_hbm_pool_is_the_staging_layout():
    geom = GEOMS[0]
    src = _pool(geom, 10, 30)
    src.alloc(10)
    agg = O.OraclePool(*geom, 6, layout=2)
    rc, d = O.transfer(src, agg, [7, 1, 4], None)
    assert rc == 0
    # block d[i] of an aggregated pool IS record i of the gather
    assert np.array_equal(agg.data.reshape(6, src.B)[d], src.gather([7, 1, 4]).reshape(3, src.B))
    assert np.array_equal(agg.gather(d), src.gather([7, 1, 4]))
