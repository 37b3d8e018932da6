"""mp_transfer_static -- the entry point that allocates nothing (block tables in a fixed array of
the library's device image) -- against mp_transfer with an explicit destination list, which
keeps its tables in library-allocated buffers.  Same inputs, two destination pools, every byte
equal (the work is a byte copy: no tolerance), and both equal to the CPU oracle.  Two calls in a
row share the one array, the second with a smaller table; then the size limit."""
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


def _pool(gpu, geom, NB, seed, staging_blocks=0):
    M, TorchPool = gpu
    L, H, D, bs, e = geom
    data = W.kv_bytes(np.random.default_rng(seed), 2 * L * NB * bs * H * D * e)
    g = TorchPool(*geom, NB, staging_blocks=staging_blocks)
    g.load(data)
    return data, g


@pytest.mark.parametrize("direct", [0, 1])
def test_static_tables_match_allocated_tables(gpu, direct):
    M, TorchPool = gpu
    geom = (4, 8, 128, 16, 2)                 # 32 KiB fragments, 256 KiB records
    NB = 300
    fl = M.MP_DIRECT if direct else 0
    src_data, src = _pool(gpu, geom, NB, 1, staging_blocks=37)        # staged: several rounds, ragged tail
    dst_data, ref = _pool(gpu, geom, NB, 2)                          # written by mp_transfer
    _, new = _pool(gpu, geom, NB, 2)                                 # written by mp_transfer_static
    o_src = O.OraclePool(*geom, NB, data=src_data.copy())
    o_dst = O.OraclePool(*geom, NB, data=dst_data.copy())
    for p in (src, ref, new):
        assert M.mp_alloc(p.h, NB)[0] == 0
    o_src.alloc(NB)
    o_dst.alloc(NB)
    rng = np.random.default_rng(3)
    for n in (257, 41):                       # two calls in a row, the second with a smaller table
        s = rng.integers(0, NB, n).astype(np.int32)                  # sources may repeat
        d = rng.permutation(NB)[:n].astype(np.int32)
        rc, _ = M.mp_transfer(src.h, ref.h, s, d, flags=fl | M.MP_DST_GIVEN | M.MP_ASYNC)
        assert rc == 0, M.mp_last_error(src.h)
        assert M.mp_transfer_static(src.h, new.h, s, d, fl | M.MP_ASYNC) == 0, M.mp_last_error(src.h)
        assert O.transfer(o_src, o_dst, s, d, flags=O.DST_GIVEN)[0] == 0
        torch.cuda.synchronize()
        got, want = new.bytes(), ref.bytes()
        assert np.array_equal(got, want), (direct, n)
        assert np.array_equal(got, o_dst.data), (direct, n)
    # synchronous form, n = 1 and n = 0
    s, d = np.array([5], np.int32), np.array([7], np.int32)
    assert M.mp_transfer(src.h, ref.h, s, d, flags=fl | M.MP_DST_GIVEN)[0] == 0
    assert M.mp_transfer_static(src.h, new.h, s, d, fl) == 0
    assert np.array_equal(new.bytes(), ref.bytes())
    assert M.mp_transfer_static(src.h, new.h, np.zeros(0, np.int32), np.zeros(0, np.int32), fl) == 0
    # argument errors change nothing
    snap = new.bytes()
    assert M.mp_transfer_static(src.h, new.h, [NB], [1], fl) == M.MP_EINVAL          # source out of range
    assert M.mp_transfer_static(src.h, new.h, [1, 2], [3, 3], fl) == M.MP_EINVAL      # repeated destination
    assert M.mp_transfer_static(src.h, new.h, [1], [2], fl | M.MP_EVICT_ON_DEMAND) == M.MP_EINVAL
    assert np.array_equal(new.bytes(), snap)
    assert src.stats() == o_src.stats() and new.stats() == o_dst.stats()
    for p in (src, ref, new):
        p.close()


def test_static_table_limit(gpu):
    """The array holds MP_STATIC_MAX_BLOCKS ids per side: a table of exactly that size works, one
    entry more is refused with a clear message and moves nothing."""
    M, TorchPool = gpu
    geom = (1, 1, 16, 1, 1)                   # 16-byte fragments, 32-byte records
    NB = M.MP_STATIC_MAX_BLOCKS + 8
    src_data, src = _pool(gpu, geom, NB, 4)
    dst_data, ref = _pool(gpu, geom, NB, 5)
    _, new = _pool(gpu, geom, NB, 5)
    for p in (src, ref, new):
        assert M.mp_alloc(p.h, NB)[0] == 0
    rng = np.random.default_rng(6)
    n = M.MP_STATIC_MAX_BLOCKS
    s = rng.integers(0, NB, n + 1).astype(np.int32)
    d = rng.permutation(NB)[: n + 1].astype(np.int32)
    snap = new.bytes()
    assert M.mp_transfer_static(src.h, new.h, s, d, M.MP_DIRECT) == M.MP_EINVAL
    assert "MP_STATIC_MAX_BLOCKS" in M.mp_last_error(src.h)
    assert np.array_equal(new.bytes(), snap)
    assert M.mp_transfer(src.h, ref.h, s[:n], d[:n], flags=M.MP_DIRECT | M.MP_DST_GIVEN)[0] == 0
    assert M.mp_transfer_static(src.h, new.h, s[:n], d[:n], M.MP_DIRECT) == 0, M.mp_last_error(src.h)
    got = new.bytes()
    assert np.array_equal(got, ref.bytes())
    o_src = O.OraclePool(*geom, NB, data=src_data.copy())
    o_dst = O.OraclePool(*geom, NB, data=dst_data.copy())
    o_src.alloc(NB)
    o_dst.alloc(NB)
    assert O.transfer(o_src, o_dst, s[:n], d[:n], flags=O.DST_GIVEN)[0] == 0
    assert np.array_equal(got, o_dst.data)
    for p in (src, ref, new):
        p.close()
