"""Thin ctypes binding of libmempool.so: same names as include/mempool.h, argument marshalling
only.  Every step of the path (gather, scatter, hashing) runs in the library's HIP kernels;
there is no Python or CPU fallback -- if the library is missing, importing callers fail.

Block tables, tokens and outputs are numpy arrays on the host; pool / staging memory is given
as raw addresses (torch tensors' data_ptr()).
"""
import ctypes as C
import os

import numpy as np

from . import build as _build

MP_TIER_HBM, MP_TIER_HOST_PINNED = 0, 1
MP_LAYOUT_DEFAULT, MP_LAYOUT_DISCRETE, MP_LAYOUT_AGGREGATED = 0, 1, 2
MP_OK, MP_EINVAL, MP_ESHAPE, MP_ENOMEM, MP_ENOSTAGING, MP_EHIP, MP_ESTALE = 0, -1, -2, -3, -4, -5, -6
MP_EHOST = -7
MP_DST_GIVEN, MP_EVICT_ON_DEMAND, MP_ASYNC = 0x01, 0x02, 0x04
MP_MATCH_PIN, MP_TOKENS_ON_DEVICE, MP_DIRECT = 0x08, 0x10, 0x20
MP_PER_FRAGMENT = 0x40
PROF_GATHER, PROF_SCATTER, PROF_DIRECT, PROF_HASH = 0, 1, 2, 3
MP_STATIC_MAX_BLOCKS = 65536

EXPORTS = [
    "mp_pool_create", "mp_pool_destroy", "mp_pool_stats", "mp_last_error", "mp_strerror",
    "mp_alloc", "mp_free", "mp_insert", "mp_match", "mp_evict", "mp_transfer",
    "mp_transfer_with_insert", "mp_match_batch", "mp_transfer_with_insert_batch",
    "mp_block_hashes", "mp_insert_hashed", "mp_match_hashed", "mp_gather", "mp_scatter",
    "mp_set_recv_callback", "mp_profile_enable", "mp_profile_read", "mp_set_tunable",
    "mp_selftest", "mp_plain_copy", "mp_transfer_layers",
    "mp_block_hashes_batch", "mp_delete", "mp_delete_hashed", "mp_transfer_batch",
    "mp_swap_out", "mp_swap_in", "mp_transfer_static",
]


class mp_pool_desc_t(C.Structure):
    _fields_ = [(n, C.c_uint32) for n in ("n_layers", "n_kv_heads", "head_dim", "block_size",
                                          "elem_bytes", "n_blocks", "tier", "instance_id")] + [
        ("hash_seed", C.c_uint64), ("base", C.c_void_p), ("staging", C.c_void_p),
        ("staging_bytes", C.c_uint64), ("stream", C.c_void_p), ("layout", C.c_uint32),
        ("reserved", C.c_uint32)]


class mp_pool_stats_t(C.Structure):
    _fields_ = [(n, C.c_uint32) for n in ("n_blocks", "n_free", "n_held", "n_indexed",
                                          "n_historical")] + [("clock", C.c_uint64)]


RECV_CB = C.CFUNCTYPE(None, C.c_void_p, C.c_void_p, C.c_uint64, C.POINTER(C.c_int32), C.c_uint32)

_lib = None


def lib():
    """Load libmempool.so (built in-tree by build.py).  No fallback: raises if absent."""
    global _lib
    if _lib is None:
        path = _build.LIB
        if not os.path.exists(path):
            raise RuntimeError(f"{path} is not built; run `python -c 'import __graft_entry__ as g; "
                               "g.build()'` (needs hipcc)")
        # torch first: its bundled HIP runtime must be the one this library binds to, so that
        # torch's streams and device pointers are valid inside the library.
        import torch  # noqa: F401
        L = C.CDLL(path)
        vp, u32, u64, i32 = C.c_void_p, C.c_uint32, C.c_uint64, C.c_int
        sig = {
            "mp_pool_create": [C.POINTER(mp_pool_desc_t), C.POINTER(vp)],
            "mp_pool_destroy": [vp],
            "mp_pool_stats": [vp, C.POINTER(mp_pool_stats_t)],
            "mp_alloc": [vp, u32, vp, u32],
            "mp_free": [vp, vp, u32],
            "mp_insert": [vp, vp, u32, vp, u32, u32, C.POINTER(u32)],
            "mp_match": [vp, vp, u32, vp, u32, C.POINTER(u32), u32],
            "mp_evict": [vp, u32, C.POINTER(u32)],
            "mp_delete": [vp, vp, u32, u32, C.POINTER(u32)],
            "mp_delete_hashed": [vp, vp, u32, vp, C.POINTER(u32)],
            "mp_transfer": [vp, vp, vp, vp, u32, u32, vp, u64],
            "mp_transfer_with_insert": [vp, vp, vp, u32, u32, vp, vp, u32, u32, vp, u64],
            "mp_transfer_layers": [vp, vp, vp, vp, u32, u32, u32, u32],
            "mp_transfer_batch": [vp, vp, vp, vp, vp, u32, u32],
            "mp_transfer_static": [vp, vp, vp, vp, u32, u32],
            "mp_match_batch": [vp, vp, vp, u32, vp, vp, vp, u32],
            "mp_transfer_with_insert_batch": [vp, vp, vp, vp, u32, vp, vp, vp, vp, u32],
            "mp_block_hashes": [vp, vp, u32, vp, u32],
            "mp_block_hashes_batch": [vp, vp, vp, u32, vp, u32],
            "mp_insert_hashed": [vp, vp, u32, vp, vp, u32, u32, C.POINTER(u32)],
            "mp_match_hashed": [vp, vp, u32, vp, vp, u32, C.POINTER(u32), u32],
            "mp_swap_out": [vp, vp, u32, u32, C.POINTER(u32)],
            "mp_swap_in": [vp, vp, vp, u32, vp, u32],
            "mp_gather": [vp, vp, u32, u32],
            "mp_scatter": [vp, vp, u32, u32],
            "mp_set_recv_callback": [vp, RECV_CB, vp],
            "mp_profile_enable": [vp, i32],
            "mp_profile_read": [vp, i32, C.POINTER(C.c_double), C.POINTER(u64), C.POINTER(u64)],
            "mp_set_tunable": [vp, C.c_char_p, i32],
            "mp_selftest": [],
            "mp_plain_copy": [vp, vp, u64, vp, C.POINTER(C.c_double)],
        }
        for name, args in sig.items():
            fn = getattr(L, name)
            fn.argtypes = args
            fn.restype = C.c_int
        L.mp_last_error.argtypes = [vp]
        L.mp_last_error.restype = C.c_char_p
        L.mp_strerror.argtypes = [C.c_int]
        L.mp_strerror.restype = C.c_char_p
        _lib = L
    return _lib


def _u32(a):
    return np.ascontiguousarray(a, dtype=np.uint32)


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def _ptr(a):
    """Host numpy array -> address (None for empty), int -> itself (device pointer)."""
    if a is None:
        return None
    if isinstance(a, int):
        return a
    return a.ctypes.data if a.size else None


# ---- same names as the C header ------------------------------------------------------------
def mp_pool_create(n_layers, n_kv_heads, head_dim, block_size, elem_bytes, n_blocks, base,
                   tier=MP_TIER_HBM, instance_id=0, hash_seed=0, staging=None, staging_bytes=0,
                   stream=None, layout=MP_LAYOUT_DEFAULT):
    d = mp_pool_desc_t(n_layers, n_kv_heads, head_dim, block_size, elem_bytes, n_blocks, tier,
                       instance_id, hash_seed, base, staging, staging_bytes, stream, layout, 0)
    h = C.c_void_p()
    rc = lib().mp_pool_create(C.byref(d), C.byref(h))
    return rc, (h.value if rc == MP_OK else None)


def mp_pool_destroy(p):
    return lib().mp_pool_destroy(p)


def mp_pool_stats(p):
    s = mp_pool_stats_t()
    rc = lib().mp_pool_stats(p, C.byref(s))
    return rc, {k: getattr(s, k) for k, _ in mp_pool_stats_t._fields_}


def mp_last_error(p):
    return lib().mp_last_error(p).decode()


def mp_strerror(code):
    return lib().mp_strerror(code).decode()


def mp_alloc(p, n, flags=0):
    out = np.full(n, -1, dtype=np.int32)
    rc = lib().mp_alloc(p, n, _ptr(out), flags)
    return rc, out


def mp_free(p, blocks):
    b = _i32(blocks)
    return lib().mp_free(p, _ptr(b), b.size)


def _tok(tokens, n_tokens):
    """tokens: host array, or (device_ptr:int with explicit n_tokens)."""
    if isinstance(tokens, int):
        return tokens, n_tokens, None
    t = _u32(tokens)
    return _ptr(t), t.size, t


def mp_insert(p, tokens, blocks, flags=0, n_tokens=None):
    tp, nt, keep = _tok(tokens, n_tokens)
    b = _i32(blocks)
    n_new = C.c_uint32(0)
    rc = lib().mp_insert(p, tp, nt, _ptr(b), b.size, flags, C.byref(n_new))
    return rc, n_new.value


def mp_match(p, tokens, cap, flags=0, n_tokens=None):
    tp, nt, keep = _tok(tokens, n_tokens)
    out = np.full(cap + 1, -1, dtype=np.int32)
    m = C.c_uint32(0)
    rc = lib().mp_match(p, tp, nt, _ptr(out), cap, C.byref(m), flags)
    return rc, out[: m.value].copy()


def mp_delete(p, tokens, flags=0, n_tokens=None):
    tp, nt, keep = _tok(tokens, n_tokens)
    n = C.c_uint32(0)
    rc = lib().mp_delete(p, tp, nt, flags, C.byref(n))
    return rc, n.value


def mp_delete_hashed(p, tokens, hashes):
    t = _u32(tokens)
    h = np.ascontiguousarray(hashes, dtype=np.uint64)
    n = C.c_uint32(0)
    rc = lib().mp_delete_hashed(p, _ptr(t), t.size, _ptr(h), C.byref(n))
    return rc, n.value


def mp_evict(p, n_blocks):
    n = C.c_uint32(0)
    rc = lib().mp_evict(p, n_blocks, C.byref(n))
    return rc, n.value


def mp_transfer(src, dst, src_blocks, dst_blocks=None, flags=0, priv=b""):
    s = _i32(src_blocks)
    d = _i32(dst_blocks).copy() if dst_blocks is not None else np.full(s.size, -1, dtype=np.int32)
    rc = lib().mp_transfer(src, dst, _ptr(s), _ptr(d), s.size, flags, priv or None, len(priv))
    return rc, d


def mp_transfer_batch(src, dst, src_blocks, blk_off, dst_blocks=None, flags=0):
    s, bo = _i32(src_blocks), _u32(blk_off)
    d = _i32(dst_blocks).copy() if dst_blocks is not None else np.full(s.size, -1, dtype=np.int32)
    rc = lib().mp_transfer_batch(src, dst, _ptr(s), _ptr(d), bo.ctypes.data, bo.size - 1, flags)
    return rc, d


def mp_transfer_layers(src, dst, src_blocks, dst_blocks, layer_begin, layer_end, flags=0):
    s, d = _i32(src_blocks), _i32(dst_blocks)
    assert s.size == d.size
    return lib().mp_transfer_layers(src, dst, _ptr(s), _ptr(d), s.size, layer_begin, layer_end, flags)


def mp_transfer_static(src, dst, src_blocks, dst_blocks, flags=0):
    s, d = _i32(src_blocks), _i32(dst_blocks)
    assert s.size == d.size
    return lib().mp_transfer_static(src, dst, _ptr(s), _ptr(d), s.size, flags)


def mp_transfer_with_insert(src, dst, tokens, first_block, src_blocks, dst_blocks=None, flags=0,
                            priv=b"", n_tokens=None):
    tp, nt, keep = _tok(tokens, n_tokens)
    s = _i32(src_blocks)
    d = _i32(dst_blocks).copy() if dst_blocks is not None else np.full(s.size, -1, dtype=np.int32)
    rc = lib().mp_transfer_with_insert(src, dst, tp, nt, first_block, _ptr(s), _ptr(d), s.size,
                                       flags, priv or None, len(priv))
    return rc, d


def mp_match_batch(p, tokens, tok_off, blk_off, flags=0):
    """blk_off[r]..blk_off[r+1] is request r's slot range (its cap) in the output."""
    to, bo = _u32(tok_off), _u32(blk_off)
    tp, nt, keep = _tok(tokens, int(to[-1]))
    n_req = to.size - 1
    out = np.full(int(bo[-1]) + 1, -1, dtype=np.int32)
    m = np.zeros(max(n_req, 1), dtype=np.uint32)
    rc = lib().mp_match_batch(p, tp, to.ctypes.data, n_req, out.ctypes.data, bo.ctypes.data,
                              m.ctypes.data, flags)
    return rc, out[:-1], m[:n_req]


def mp_transfer_with_insert_batch(src, dst, tokens, tok_off, first_block, src_blocks, blk_off,
                                  flags=0):
    to, bo, fb, s = _u32(tok_off), _u32(blk_off), _u32(first_block), _i32(src_blocks)
    tp, nt, keep = _tok(tokens, int(to[-1]))
    d = np.full(s.size, -1, dtype=np.int32)
    rc = lib().mp_transfer_with_insert_batch(src, dst, tp, to.ctypes.data, to.size - 1, _ptr(fb),
                                             _ptr(s), _ptr(d), bo.ctypes.data, flags)
    return rc, d


def mp_block_hashes(p, tokens, block_size, flags=0, n_tokens=None):
    tp, nt, keep = _tok(tokens, n_tokens)
    out = np.zeros(nt // block_size, dtype=np.uint64)
    rc = lib().mp_block_hashes(p, tp, nt, _ptr(out), flags)
    return rc, out


def mp_block_hashes_batch(p, tokens, tok_off, block_size, flags=0):
    """Returns (rc, hashes of all prompts back to back, hash offsets[n_req+1])."""
    to = _u32(tok_off)
    tp, nt, keep = _tok(tokens, int(to[-1]))
    nb = (to[1:] - to[:-1]) // block_size
    hoff = np.concatenate([[0], np.cumsum(nb)]).astype(np.uint32)
    out = np.zeros(int(hoff[-1]), dtype=np.uint64)
    rc = lib().mp_block_hashes_batch(p, tp, to.ctypes.data, to.size - 1, _ptr(out), flags)
    return rc, out, hoff


def mp_insert_hashed(p, tokens, hashes, blocks, flags=0):
    t, b = _u32(tokens), _i32(blocks)
    h = np.ascontiguousarray(hashes, dtype=np.uint64)
    n_new = C.c_uint32(0)
    rc = lib().mp_insert_hashed(p, _ptr(t), t.size, _ptr(h), _ptr(b), b.size, flags, C.byref(n_new))
    return rc, n_new.value


def mp_match_hashed(p, tokens, hashes, cap, flags=0):
    t = _u32(tokens)
    h = np.ascontiguousarray(hashes, dtype=np.uint64)
    out = np.full(cap + 1, -1, dtype=np.int32)
    m = C.c_uint32(0)
    rc = lib().mp_match_hashed(p, _ptr(t), t.size, _ptr(h), _ptr(out), cap, C.byref(m), flags)
    return rc, out[: m.value].copy()


def mp_swap_out(upper, lower, num_blocks, flags=0):
    n = C.c_uint32(0)
    rc = lib().mp_swap_out(upper, lower, num_blocks, flags, C.byref(n))
    return rc, n.value


def mp_swap_in(lower, upper, lower_blocks, flags=0):
    b = _i32(lower_blocks)
    out = np.full(b.size, -1, dtype=np.int32)
    rc = lib().mp_swap_in(lower, upper, _ptr(b), b.size, _ptr(out), flags)
    return rc, out


def mp_gather(p, tbl, flags=0):
    t = _i32(tbl)
    return lib().mp_gather(p, _ptr(t), t.size, flags)


def mp_scatter(p, tbl, flags=0):
    t = _i32(tbl)
    return lib().mp_scatter(p, _ptr(t), t.size, flags)


def mp_set_recv_callback(p, cb):
    """cb: a RECV_CB instance (keep a reference to it) or None."""
    return lib().mp_set_recv_callback(p, cb if cb is not None else RECV_CB(), None)


def mp_profile_enable(p, on=True):
    return lib().mp_profile_enable(p, int(on))


def mp_profile_read(p, kind):
    ms, n, b = C.c_double(0), C.c_uint64(0), C.c_uint64(0)
    rc = lib().mp_profile_read(p, kind, C.byref(ms), C.byref(n), C.byref(b))
    return rc, ms.value, n.value, b.value


def mp_set_tunable(p, key, value):
    return lib().mp_set_tunable(p, key.encode(), int(value))


def mp_selftest():
    return lib().mp_selftest()


def mp_plain_copy(dst_ptr, src_ptr, nbytes, stream=None):
    ms = C.c_double(0)
    rc = lib().mp_plain_copy(dst_ptr, src_ptr, nbytes, stream, C.byref(ms))
    return rc, ms.value
