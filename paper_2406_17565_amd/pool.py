"""Device-memory plumbing: a pool handle of libmempool over torch-allocated memory.

torch supplies the HBM tensors (pool and staging), the pinned host tensor of a host-tier pool
and the stream; everything that moves or hashes data is done by the library's kernels.
"""
import weakref

import numpy as np
import torch

from . import mempool as M


class TorchPool:
    # Canary bands: with GUARD_BYTES > 0 (a multiple of 256; the GPU tests switch it on) every
    # pool, staging and pinned-host buffer is allocated with that many extra bytes in front and
    # behind, filled with GUARD_VALUE; guards_intact() tells whether a copy strayed into them.
    GUARD_BYTES = 0
    GUARD_VALUE = 0xA5
    live = weakref.WeakSet()

    def _buffer(self, nbytes, device=None):
        g = self._guard
        if device is None:
            raw = torch.empty(nbytes + 2 * g, dtype=torch.uint8, pin_memory=True)
        else:
            raw = torch.empty(nbytes + 2 * g, dtype=torch.uint8, device=device)
        if g:
            raw[:g] = self.GUARD_VALUE
            raw[g + nbytes:] = self.GUARD_VALUE
        self._raw.append((raw, nbytes))
        return raw[g:g + nbytes]

    def guards_intact(self) -> bool:
        g = self._guard
        if not g:
            return True
        if any(raw.is_cuda for raw, _ in self._raw):
            torch.cuda.synchronize()
        return all(bool((raw[:g] == self.GUARD_VALUE).all()) and
                   bool((raw[g + n:] == self.GUARD_VALUE).all()) for raw, n in self._raw)

    def __init__(self, L, H, D, bs, e, NB, tier=M.MP_TIER_HBM, staging_blocks=0, seed=0,
                 instance_id=0, device="cuda:0", stream=None, layout=M.MP_LAYOUT_DEFAULT):
        self.geom = (L, H, D, bs, e)
        self.NB, self.tier, self.bs = NB, tier, bs
        self.aggregated = layout == M.MP_LAYOUT_AGGREGATED or (
            layout == M.MP_LAYOUT_DEFAULT and tier == M.MP_TIER_HOST_PINNED)
        self.F = bs * H * D * e
        self.B = 2 * L * self.F
        nbytes = 2 * L * NB * self.F
        self._guard, self._raw, self.h = self.GUARD_BYTES, [], None
        self.mem = self._buffer(nbytes, device if tier == M.MP_TIER_HBM else None)
        self.staging = None
        if staging_blocks:
            self.staging = self._buffer(staging_blocks * self.B, device)
        self.stream = stream if stream is not None else torch.cuda.current_stream(device)
        rc, self.h = M.mp_pool_create(
            L, H, D, bs, e, NB, self.mem.data_ptr(), tier=tier, instance_id=instance_id,
            hash_seed=seed,
            staging=self.staging.data_ptr() if self.staging is not None else None,
            staging_bytes=self.staging.numel() if self.staging is not None else 0,
            stream=self.stream.cuda_stream or None, layout=layout)
        if rc != M.MP_OK:
            raise ValueError(f"mp_pool_create: {M.mp_strerror(rc)}")
        TorchPool.live.add(self)

    def close(self):
        if self.h is not None:
            M.mp_pool_destroy(self.h)          # waits for the pool's streams
            self.h = None
            if not self.guards_intact():
                raise RuntimeError("a copy wrote outside the pool / staging memory (canary band changed)")

    def free_memory(self):
        """close(), then drop the tensors (the caller may empty torch's cache afterwards)."""
        self.close()
        self.mem = self.staging = None
        self._raw = []

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # harness helpers (not part of the path)
    def load(self, data: np.ndarray):
        self.mem.copy_(torch.from_numpy(data))
        if self.mem.is_cuda:
            torch.cuda.synchronize()

    def bytes(self) -> np.ndarray:
        if self.mem.is_cuda:
            torch.cuda.synchronize()
        return self.mem.cpu().numpy().copy()

    def staging_bytes(self, n_blocks) -> np.ndarray:
        torch.cuda.synchronize()
        return self.staging[: n_blocks * self.B].cpu().numpy().copy()

    def stats(self):
        return M.mp_pool_stats(self.h)[1]


class MemPoolError(RuntimeError):
    def __init__(self, code, text):
        super().__init__(f"{M.mp_strerror(code)} ({code}): {text}")
        self.code = code


class MemPool(TorchPool):
    """The calls of the paper's Table 1 under their own names, on one pool handle.  Argument
    marshalling only: every method is one call of the C ABI; a negative return code becomes a
    MemPoolError.  Block lists are numpy int32 arrays."""

    def _ok(self, rc, who=None):
        if rc != M.MP_OK:
            raise MemPoolError(rc, M.mp_last_error((who or self).h))

    def alloc_mem(self, n, evict_on_demand=False):
        rc, ids = M.mp_alloc(self.h, n, M.MP_EVICT_ON_DEMAND if evict_on_demand else 0)
        self._ok(rc)
        return ids

    def free_mem(self, blocks):
        self._ok(M.mp_free(self.h, blocks))

    def insert(self, tokens, blocks):
        rc, n_new = M.mp_insert(self.h, tokens, blocks)
        self._ok(rc)
        return n_new

    def match(self, tokens, pin=False):
        rc, ids = M.mp_match(self.h, tokens, len(tokens) // self.bs, M.MP_MATCH_PIN if pin else 0)
        self._ok(rc)
        return ids

    def delete(self, tokens):
        rc, n = M.mp_delete(self.h, tokens)
        self._ok(rc)
        return n

    def evict(self, n):
        rc, done = M.mp_evict(self.h, n)
        self._ok(rc)
        return done

    def swap_out(self, lower, num_blocks, flags=0):
        rc, n = M.mp_swap_out(self.h, lower.h, num_blocks, flags)
        self._ok(rc)
        return n

    def swap_in(self, lower, lower_blocks, flags=0):
        rc, ids = M.mp_swap_in(lower.h, self.h, lower_blocks, flags)
        self._ok(rc, lower)
        return ids

    def transfer(self, dst, src_blocks, dst_blocks=None, flags=0, private=b""):
        if dst_blocks is not None:
            flags |= M.MP_DST_GIVEN
        rc, ids = M.mp_transfer(self.h, dst.h, src_blocks, dst_blocks, flags, private)
        self._ok(rc)
        return ids

    def transfer_with_insert(self, dst, tokens, src_blocks, first_block=0, dst_blocks=None, flags=0,
                             private=b""):
        if dst_blocks is not None:
            flags |= M.MP_DST_GIVEN
        rc, ids = M.mp_transfer_with_insert(self.h, dst.h, tokens, first_block, src_blocks, dst_blocks,
                                            flags, private)
        self._ok(rc)
        return ids
