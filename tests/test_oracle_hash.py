"""Pins for the oracle's chained block hash: published vectors of its two primitives, worked
examples from tests/golden, and structural invariants of a prefix chain."""
import os

import numpy as np

from oracle import oracle as O

G = 0x9E3779B97F4A7C15
M64 = (1 << 64) - 1


def _read(golden_dir, name):
    rows = []
    with open(os.path.join(golden_dir, name)) as f:
        for line in f:
            line = line.strip()
            if line and not line.startswith("#"):
                rows.append(line.split())
    return rows


def test_fnv1a64_published_vectors(golden_dir):
    n = 0
    for kind, arg, val in _read(golden_dir, "published_hash_vectors.txt"):
        if kind == "fnv1a64":
            assert O.fnv1a64(arg.strip('"').encode()) == int(val, 16)
            n += 1
    assert n == 3


def test_fmix_and_chain_step_are_splitmix64(golden_dir):
    # splitmix64 keeps a counter state s += G and outputs fmix64(s).  A chain step with digest 0
    # is exactly one splitmix64 step whose state is the previous chain value.
    n = 0
    for kind, k, val in _read(golden_dir, "published_hash_vectors.txt"):
        if kind == "splitmix64":
            k = int(k)
            assert O.fmix64(k * G & M64) == int(val, 16)
            assert O.chain_step((k - 1) * G & M64, 0) == int(val, 16)
            n += 1
    assert n == 4


def test_chain_step_xors_digest_after_adding_G():
    # fmix64 is a bijection with fmix64(0) == 0, so the pre-image of 0 pins the argument order:
    # (h_prev + G) xor d == 0  <=>  d == h_prev + G.
    for h in (0, 1, 0x1234567890ABCDEF, M64):
        assert O.chain_step(h, (h + G) & M64) == 0
        assert O.chain_step(h, h) != 0


def test_digest_is_fnv_over_little_endian_token_bytes():
    rng = np.random.default_rng(7)
    for bs in (1, 8, 16, 32):
        t = rng.integers(0, 2**32, bs, dtype=np.uint32)
        assert O.block_digest(t) == O.fnv1a64(t.astype("<u4").tobytes())
    # "foob"/"ar\0\0" style: a token whose LE bytes spell ascii
    t = np.frombuffer(b"foobarba", dtype="<u4")
    assert O.block_digest(t) == O.fnv1a64(b"foobarba")


def _case_tokens(case):
    return {"arange48": np.arange(48), "zeros32": np.zeros(32), "arange64": np.arange(64),
            "arange16": np.arange(16)}[case].astype(np.uint32)


def test_worked_examples(golden_dir):
    rows = _read(golden_dir, "block_hash_vectors.txt")
    assert len(rows) == 8
    for case, bs, seed, i, d, h in rows:
        bs, seed, i = int(bs), int(seed), int(i)
        t = _case_tokens(case)
        assert O.block_digest(t[i * bs:(i + 1) * bs]) == int(d, 16)
        assert int(O.block_hashes(t, bs, seed)[i]) == int(h, 16)


def test_only_full_blocks_are_hashed():
    t = np.arange(100, dtype=np.uint32)
    assert O.block_hashes(t, 16).size == 6
    assert O.block_hashes(t[:15], 16).size == 0
    assert np.array_equal(O.block_hashes(t, 16), O.block_hashes(t[:96], 16))


def test_prefix_chain_invariants():
    rng = np.random.default_rng(11)
    bs = 16
    a = rng.integers(0, 32000, 10 * bs, dtype=np.uint32)
    b = a.copy()
    j = 4
    b[j * bs + 3] ^= 1  # first differing block is j
    ha, hb = O.block_hashes(a, bs), O.block_hashes(b, bs)
    assert np.array_equal(ha[:j], hb[:j])
    assert np.all(ha[j:] != hb[j:])
    hs = O.block_hashes(a, bs, seed=99)
    assert np.all(hs != ha)
    # equal blocks at different positions: equal digests, different chain values
    z = np.zeros(4 * bs, dtype=np.uint32)
    hz = O.block_hashes(z, bs)
    assert len(set(hz.tolist())) == 4
    assert len({O.block_digest(z[i * bs:(i + 1) * bs]) for i in range(4)}) == 1
    # h_i depends only on tokens[0:(i+1)*bs]
    assert np.array_equal(O.block_hashes(a[:5 * bs], bs), ha[:5])


def test_chain_recurrence_from_primitives():
    # h_i rebuilt from the separately pinned primitives (fnv over LE bytes, chain_step)
    rng = np.random.default_rng(5)
    for bs in (16, 32):
        t = rng.integers(0, 128256, 7 * bs + 5, dtype=np.uint32)
        h, want = 0xABCDEF, []
        for i in range(7):
            h = O.chain_step(h, O.fnv1a64(t[i * bs:(i + 1) * bs].astype("<u4").tobytes()))
            want.append(h)
        assert O.block_hashes(t, bs, 0xABCDEF).tolist() == want
