"""Device-memory plumbing: a pool handle of libmempool over torch-allocated memory.

torch supplies the HBM tensors (pool and staging), the pinned host tensor of a host-tier pool
and the stream; everything that moves or hashes data is done by the library's kernels.
"""
import numpy as np
import torch

from . import mempool as M


class TorchPool:
    def __init__(self, L, H, D, bs, e, NB, tier=M.MP_TIER_HBM, staging_blocks=0, seed=0,
                 instance_id=0, device="cuda:0", stream=None, layout=M.MP_LAYOUT_DEFAULT):
        self.geom = (L, H, D, bs, e)
        self.NB, self.tier, self.bs = NB, tier, bs
        self.aggregated = layout == M.MP_LAYOUT_AGGREGATED or (
            layout == M.MP_LAYOUT_DEFAULT and tier == M.MP_TIER_HOST_PINNED)
        self.F = bs * H * D * e
        self.B = 2 * L * self.F
        nbytes = 2 * L * NB * self.F
        if tier == M.MP_TIER_HBM:
            self.mem = torch.empty(nbytes, dtype=torch.uint8, device=device)
        else:
            self.mem = torch.empty(nbytes, dtype=torch.uint8, pin_memory=True)
        self.staging = None
        if staging_blocks:
            self.staging = torch.empty(staging_blocks * self.B, dtype=torch.uint8, device=device)
        self.stream = stream if stream is not None else torch.cuda.current_stream(device)
        rc, self.h = M.mp_pool_create(
            L, H, D, bs, e, NB, self.mem.data_ptr(), tier=tier, instance_id=instance_id,
            hash_seed=seed,
            staging=self.staging.data_ptr() if self.staging is not None else None,
            staging_bytes=self.staging.numel() if self.staging is not None else 0,
            stream=self.stream.cuda_stream or None, layout=layout)
        if rc != M.MP_OK:
            raise ValueError(f"mp_pool_create: {M.mp_strerror(rc)}")

    def close(self):
        if self.h is not None:
            M.mp_pool_destroy(self.h)
            self.h = None

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
