"""ctypes access to the CPU oracle (oracle/liboracle.so).

TEST INFRASTRUCTURE ONLY: imported by tests/, the smoke check and the benchmark's
cpu_baseline leg.  Nothing in the product package imports this module.
"""
import ctypes as C
import os

import numpy as np

from . import build as _build

OK, EINVAL, ESHAPE, ENOMEM, ESTALE = 0, -1, -2, -3, -6
TIER_HBM, TIER_HOST = 0, 1
DST_GIVEN, EVICT_ON_DEMAND, MATCH_PIN = 0x01, 0x02, 0x08

_lib = None


def lib():
    global _lib
    if _lib is None:
        path = _build.LIB
        if not os.path.exists(path):
            _build.build()
        L = C.CDLL(path)
        u8p, u32p, i32p, u64p = (C.POINTER(t) for t in (C.c_uint8, C.c_uint32, C.c_int32, C.c_uint64))
        vp = C.c_void_p
        L.orc_fnv1a64.restype = C.c_uint64
        L.orc_fnv1a64.argtypes = [vp, C.c_uint64]
        L.orc_fmix64.restype = C.c_uint64
        L.orc_fmix64.argtypes = [C.c_uint64]
        L.orc_chain_step.restype = C.c_uint64
        L.orc_chain_step.argtypes = [C.c_uint64, C.c_uint64]
        L.orc_block_digest.restype = C.c_uint64
        L.orc_block_digest.argtypes = [vp, C.c_uint32]
        L.orc_block_hashes.restype = None
        L.orc_block_hashes.argtypes = [vp, C.c_uint32, C.c_uint32, C.c_uint64, vp]
        L.orc_pool_create.restype = vp
        L.orc_pool_create.argtypes = [C.c_uint32] * 8 + [C.c_uint64, vp, C.c_uint32]
        L.orc_pool_destroy.restype = None
        L.orc_pool_destroy.argtypes = [vp]
        L.orc_fragment_bytes.restype = C.c_uint64
        L.orc_fragment_bytes.argtypes = [vp]
        L.orc_record_bytes.restype = C.c_uint64
        L.orc_record_bytes.argtypes = [vp]
        L.orc_fragment_offset.restype = C.c_uint64
        L.orc_fragment_offset.argtypes = [vp, C.c_uint32, C.c_uint32, C.c_uint32]
        L.orc_stats.restype = None
        L.orc_stats.argtypes = [vp, u32p, u32p, u32p, u32p, u64p]
        L.orc_alloc.argtypes = [vp, C.c_uint32, vp, C.c_uint32]
        L.orc_free.argtypes = [vp, vp, C.c_uint32]
        L.orc_insert.argtypes = [vp, vp, C.c_uint32, vp, C.c_uint32, u32p]
        L.orc_match.argtypes = [vp, vp, C.c_uint32, vp, C.c_uint32, u32p, C.c_uint32]
        L.orc_evict.argtypes = [vp, C.c_uint32, u32p]
        L.orc_delete.argtypes = [vp, vp, C.c_uint32, u32p]
        L.orc_gather.argtypes = [vp, vp, C.c_uint32, vp]
        L.orc_scatter.argtypes = [vp, vp, C.c_uint32, vp]
        L.orc_transfer.argtypes = [vp, vp, vp, vp, C.c_uint32, C.c_uint32]
        L.orc_transfer_layers.argtypes = [vp, vp, vp, vp, C.c_uint32, C.c_uint32, C.c_uint32]
        L.orc_transfer_with_insert.argtypes = [vp, vp, vp, C.c_uint32, C.c_uint32, vp, vp,
                                               C.c_uint32, C.c_uint32]
        L.orc_transfer_with_insert_batch.argtypes = [vp, vp, vp, vp, C.c_uint32, vp, vp, vp, vp,
                                                     C.c_uint32]
        L.orc_swap_out.argtypes = [vp, vp, C.c_uint32, u32p]
        L.orc_swap_in.argtypes = [vp, vp, vp, C.c_uint32, vp]
        _lib = L
    return _lib


def _u32(a):
    return np.ascontiguousarray(a, dtype=np.uint32)


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def _ptr(a):
    return a.ctypes.data_as(C.c_void_p) if a is not None and a.size else None


def fnv1a64(data: bytes) -> int:
    buf = np.frombuffer(data, dtype=np.uint8) if len(data) else np.zeros(0, np.uint8)
    return lib().orc_fnv1a64(_ptr(buf), len(data))


def fmix64(x: int) -> int:
    return lib().orc_fmix64(x)


def chain_step(h_prev: int, digest: int) -> int:
    return lib().orc_chain_step(h_prev, digest)


def block_digest(block_tokens) -> int:
    t = _u32(block_tokens)
    return lib().orc_block_digest(_ptr(t), t.size)


def block_hashes(tokens, bs: int, seed: int = 0) -> np.ndarray:
    t = _u32(tokens)
    out = np.zeros(t.size // bs, dtype=np.uint64)
    lib().orc_block_hashes(_ptr(t), t.size, bs, seed, _ptr(out))
    return out


class OraclePool:
    """A pool over a numpy byte array that the oracle reads and writes in place."""

    def __init__(self, L, H, D, bs, e, NB, tier=TIER_HBM, instance_id=0, seed=0, data=None,
                 layout=0):
        self.geom = (L, H, D, bs, e)
        self.NB, self.tier, self.bs = NB, tier, bs
        self.F = bs * H * D * e
        self.B = 2 * L * self.F
        nbytes = 2 * L * NB * self.F
        if data is None:
            data = np.zeros(nbytes, dtype=np.uint8)
        assert data.dtype == np.uint8 and data.size == nbytes and data.flags.c_contiguous
        self.data = data
        self.h = lib().orc_pool_create(L, H, D, bs, e, NB, tier, instance_id, seed, _ptr(data),
                                       layout)
        if not self.h:
            raise ValueError("orc_pool_create refused the geometry")

    def __del__(self):
        try:
            if getattr(self, "h", None):
                lib().orc_pool_destroy(self.h)
                self.h = None
        except Exception:      # interpreter shutdown: the module globals may be gone already
            pass

    def fragment_offset(self, l, kv, b):
        return lib().orc_fragment_offset(self.h, l, kv, b)

    def stats(self):
        v = [C.c_uint32() for _ in range(4)]
        clk = C.c_uint64()
        lib().orc_stats(self.h, *[C.byref(x) for x in v], C.byref(clk))
        return dict(n_blocks=self.NB, n_free=v[0].value, n_held=v[1].value, n_indexed=v[2].value,
                    n_historical=v[3].value, clock=clk.value)

    def alloc(self, n, flags=0):
        out = np.full(n, -1, dtype=np.int32)
        rc = lib().orc_alloc(self.h, n, _ptr(out), flags)
        return rc, out

    def free(self, blocks):
        b = _i32(blocks)
        return lib().orc_free(self.h, _ptr(b), b.size)

    def insert(self, tokens, blocks):
        t, b = _u32(tokens), _i32(blocks)
        n_new = C.c_uint32(0)
        rc = lib().orc_insert(self.h, _ptr(t), t.size, _ptr(b), b.size, C.byref(n_new))
        return rc, n_new.value

    def match(self, tokens, cap=None, flags=0):
        t = _u32(tokens)
        if cap is None:
            cap = t.size // self.bs
        out = np.full(max(cap, t.size // self.bs) + 1, -1, dtype=np.int32)  # room to expose an overrun
        m = C.c_uint32(0)
        rc = lib().orc_match(self.h, _ptr(t), t.size, _ptr(out), cap, C.byref(m), flags)
        return rc, out[: m.value].copy()

    def delete(self, tokens):
        t = _u32(tokens)
        n = C.c_uint32(0)
        rc = lib().orc_delete(self.h, _ptr(t), t.size, C.byref(n))
        return rc, n.value

    def evict(self, k):
        n = C.c_uint32(0)
        rc = lib().orc_evict(self.h, k, C.byref(n))
        return rc, n.value

    def gather(self, tbl):
        t = _i32(tbl)
        staging = np.zeros(t.size * self.B, dtype=np.uint8)
        lib().orc_gather(self.h, _ptr(t), t.size, _ptr(staging))
        return staging

    def scatter(self, tbl, staging):
        t = _i32(tbl)
        assert staging.dtype == np.uint8 and staging.size == t.size * self.B
        return lib().orc_scatter(self.h, _ptr(t), t.size, _ptr(np.ascontiguousarray(staging)))


def transfer(src: OraclePool, dst: OraclePool, src_blocks, dst_blocks=None, flags=0):
    s = _i32(src_blocks)
    d = _i32(dst_blocks) if dst_blocks is not None else np.full(s.size, -1, dtype=np.int32)
    d = d.copy()
    rc = lib().orc_transfer(src.h, dst.h, _ptr(s), _ptr(d), s.size, flags)
    return rc, d


def transfer_layers(src, dst, src_blocks, dst_blocks, l0, l1):
    s, d = _i32(src_blocks), _i32(dst_blocks)
    return lib().orc_transfer_layers(src.h, dst.h, _ptr(s), _ptr(d), s.size, l0, l1)


def transfer_with_insert(src, dst, tokens, first_block, src_blocks, dst_blocks=None, flags=0):
    t, s = _u32(tokens), _i32(src_blocks)
    d = _i32(dst_blocks).copy() if dst_blocks is not None else np.full(s.size, -1, dtype=np.int32)
    rc = lib().orc_transfer_with_insert(src.h, dst.h, _ptr(t), t.size, first_block, _ptr(s),
                                        _ptr(d), s.size, flags)
    return rc, d


def transfer_with_insert_batch(src, dst, tokens, tok_off, first_block, src_blocks, blk_off, flags=0):
    t, to, fb, s, bo = _u32(tokens), _u32(tok_off), _u32(first_block), _i32(src_blocks), _u32(blk_off)
    d = np.full(s.size, -1, dtype=np.int32)
    rc = lib().orc_transfer_with_insert_batch(src.h, dst.h, _ptr(t), to.ctypes.data_as(C.c_void_p),
                                              fb.size, _ptr(fb), _ptr(s), _ptr(d),
                                              bo.ctypes.data_as(C.c_void_p), flags)
    return rc, d


def swap_out(upper: OraclePool, lower: OraclePool, num_blocks):
    n = C.c_uint32(0)
    rc = lib().orc_swap_out(upper.h, lower.h, num_blocks, C.byref(n))
    return rc, n.value


def swap_in(lower: OraclePool, upper: OraclePool, lower_blocks):
    b = _i32(lower_blocks)
    out = np.full(b.size, -1, dtype=np.int32)
    rc = lib().orc_swap_in(lower.h, upper.h, _ptr(b), b.size, _ptr(out))
    return rc, out
