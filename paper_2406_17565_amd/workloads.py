"""Seeded synthetic inputs for the KV-block transfer / match path.

This module only draws shapes, token ids, block tables and KV bytes.  It contains none of the
method's arithmetic (no hashing, no copying by table, no index), so both the GPU library's
tests and the CPU oracle may be fed from it.

The five geometries and workloads mirror the serving scenarios of the MemServe paper's
evaluation (section 8.2: multi-turn chat sessions, long shared documents, a 2048-token
transfer test in the block-aggregation study of section 8.4); the datasets themselves are
not used -- every length and id below is synthetic.
"""
from dataclasses import dataclass

import numpy as np


@dataclass(frozen=True)
class Geometry:
    name: str
    L: int        # layers
    H: int        # kv heads (per GPU)
    D: int        # head dim
    bs: int       # tokens per block
    e: int        # bytes per element
    dtype: str    # "fp16" | "bf16"
    NB: int       # blocks per pool at full scale
    vocab: int

    @property
    def F(self):  # fragment bytes: one (layer, K|V, block)
        return self.bs * self.H * self.D * self.e

    @property
    def B(self):  # record bytes: the 2*L fragments of one block
        return 2 * self.L * self.F

    def pool_bytes(self, NB=None):
        return 2 * self.L * (self.NB if NB is None else NB) * self.F


CONFIGS = {
    1: Geometry("tiny", 2, 2, 64, 16, 2, "fp16", 256, 32000),
    2: Geometry("llama2-7b", 32, 32, 128, 16, 2, "fp16", 8192, 32000),
    3: Geometry("llama3-8b-gqa", 32, 8, 128, 16, 2, "bf16", 16384, 128256),
    4: Geometry("llama2-13b", 40, 40, 128, 32, 2, "fp16", 4096, 32000),
    5: Geometry("70b-tp-share", 80, 1, 128, 16, 2, "bf16", 40960, 128256),
}


def kv_bytes(rng: np.random.Generator, nbytes: int, dtype: str = "fp16") -> np.ndarray:
    """N(0,1) KV values of the given 16-bit type, returned as raw bytes."""
    n = nbytes // 2
    x = rng.standard_normal(n, dtype=np.float32)
    if dtype == "fp16":
        raw = x.astype(np.float16).view(np.uint16)
    else:  # bf16: upper half of the fp32 bit pattern
        raw = (x.view(np.uint32) >> 16).astype(np.uint16)
    out = raw.view(np.uint8)
    if nbytes % 2:
        out = np.concatenate([out, np.zeros(1, np.uint8)])
    return np.ascontiguousarray(out)


def special_half_patterns(nbytes: int) -> np.ndarray:
    """NaN payload, all-ones and negative-zero 16-bit patterns: must survive a byte copy."""
    pat = np.array([0x7E01, 0xFFFF, 0x8000, 0x0001, 0x7C00, 0xFC00], dtype=np.uint16)
    return np.ascontiguousarray(np.resize(pat, nbytes // 2).view(np.uint8))


def random_table(rng: np.random.Generator, NB: int, n: int) -> np.ndarray:
    """n distinct block ids in random order (a fragmented block table)."""
    return rng.permutation(NB)[:n].astype(np.int32)


def tiny_requests(seed: int = 1, n_req: int = 8, prefix_len: int = 64, own_len: int = 64,
                  vocab: int = 32000):
    """Config 1: n_req prompts sharing one prefix."""
    rng = np.random.default_rng(seed)
    prefix = rng.integers(0, vocab, prefix_len, dtype=np.uint32)
    return [np.concatenate([prefix, rng.integers(0, vocab, own_len, dtype=np.uint32)])
            for _ in range(n_req)]


def lognormal_lengths(seed: int = 2, n_req: int = 16, median: int = 1024, sigma: float = 0.8,
                      lo: int = 16, hi: int = 4096) -> np.ndarray:
    """Config 2: prompt lengths."""
    rng = np.random.default_rng(seed)
    x = np.rint(rng.lognormal(np.log(median), sigma, n_req))
    return np.clip(x, lo, hi).astype(np.int64)


def random_prompts(seed: int, lengths, vocab: int):
    rng = np.random.default_rng(seed)
    return [rng.integers(0, vocab, int(n), dtype=np.uint32) for n in lengths]


def multiturn_sessions(seed: int = 3, n_sessions: int = 64, n_turns: int = 4, reply: int = 256,
                       new_lo: int = 128, new_hi: int = 512, vocab: int = 128256):
    """Config 3: prompts[s][t]; prompt_t = prompt_{t-1} + reply tokens + new user tokens."""
    rng = np.random.default_rng(seed)
    new_len = rng.integers(new_lo, new_hi + 1, size=(n_sessions, n_turns))
    prompts = []
    for s in range(n_sessions):
        turns, cur = [], np.zeros(0, dtype=np.uint32)
        for t in range(n_turns):
            parts = [cur]
            if t > 0:
                parts.append(rng.integers(0, vocab, reply, dtype=np.uint32))
            parts.append(rng.integers(0, vocab, int(new_len[s, t]), dtype=np.uint32))
            cur = np.concatenate(parts)
            turns.append(cur)
        prompts.append(turns)
    return prompts


def long_context_requests(seed: int = 4, n_req: int = 32, length: int = 16384,
                          prefix_len: int = 8192, share: float = 0.9, vocab: int = 32000):
    """Config 4: long prompts, a fraction `share` of which start with one common prefix."""
    rng = np.random.default_rng(seed)
    prefix = rng.integers(0, vocab, prefix_len, dtype=np.uint32)
    n_share = int(round(share * n_req))
    sharers = set(rng.permutation(n_req)[:n_share].tolist())
    out = []
    for r in range(n_req):
        if r in sharers:
            out.append(np.concatenate([prefix, rng.integers(0, vocab, length - prefix_len,
                                                            dtype=np.uint32)]))
        else:
            out.append(rng.integers(0, vocab, length, dtype=np.uint32))
    return out


def csr(arrays, dtype=np.uint32):
    """Concatenate ragged arrays: (flat, offsets[len+1])."""
    off = np.zeros(len(arrays) + 1, dtype=np.uint32)
    for i, a in enumerate(arrays):
        off[i + 1] = off[i] + len(a)
    flat = np.concatenate(arrays).astype(dtype) if len(arrays) else np.zeros(0, dtype)
    return np.ascontiguousarray(flat), off
