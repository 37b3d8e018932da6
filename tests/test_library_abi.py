"""The C-ABI library loads and exports every symbol its public header declares (no GPU)."""
import ctypes
import os
import re

from paper_2406_17565_amd import build as B
from paper_2406_17565_amd import mempool as M

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "mempool.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = set(re.findall(r"\b(mp_[a-z_]+)\s*\(", text))
    names -= {"mp_recv_cb"}
    return names


def test_library_is_built():
    assert os.path.exists(B.LIB), "run __graft_entry__.build() first"


def test_every_declared_symbol_is_exported():
    names = _declared()
    assert {"mp_pool_create", "mp_insert", "mp_match", "mp_transfer", "mp_transfer_with_insert",
            "mp_evict"} <= names
    lib = ctypes.CDLL(B.LIB)
    for n in sorted(names):
        assert hasattr(lib, n), f"{n} declared in include/mempool.h but not exported"
    assert names == set(M.EXPORTS), names ^ set(M.EXPORTS)


def test_selftest_and_strerror():
    assert M.mp_selftest() == 0
    assert M.mp_strerror(0) == "ok"
    assert "staging" in M.mp_strerror(M.MP_ENOSTAGING)


def test_header_constants_match_binding():
    text = open(os.path.join(ROOT, "include", "mempool.h")).read()
    for name in ("MP_EINVAL", "MP_ESHAPE", "MP_ENOMEM", "MP_ENOSTAGING", "MP_EHIP", "MP_ESTALE",
                 "MP_EHOST"):
        m = re.search(rf"#define {name} \((-\d+)\)", text)
        assert int(m.group(1)) == getattr(M, name)
    for name in ("MP_DST_GIVEN", "MP_EVICT_ON_DEMAND", "MP_ASYNC", "MP_MATCH_PIN",
                 "MP_TOKENS_ON_DEVICE", "MP_DIRECT", "MP_PER_FRAGMENT"):
        m = re.search(rf"#define {name} (0x[0-9a-f]+)u", text)
        assert int(m.group(1), 16) == getattr(M, name)


def test_pool_create_rejects_bad_descriptors():
    import numpy as np
    buf = np.zeros(4096 + 16, np.uint8)
    base = (buf.ctypes.data + 15) // 16 * 16
    assert M.mp_pool_create(2, 1, 8, 4, 2, 8, base)[0] == 0
    assert M.mp_pool_create(0, 1, 8, 4, 2, 8, base)[0] == M.MP_EINVAL
    assert M.mp_pool_create(2, 1, 8, 4, 2, 8, None)[0] == M.MP_EINVAL
    assert M.mp_pool_create(2, 1, 8, 4, 2, 8, base + 4)[0] == M.MP_EINVAL     # misaligned
    assert M.mp_pool_create(2, 1, 3, 1, 2, 8, base)[0] == M.MP_EINVAL         # F = 6 bytes
    assert M.mp_pool_create(2, 1, 8, 4, 2, 8, base, tier=7)[0] == M.MP_EINVAL
