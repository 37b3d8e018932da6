#!/usr/bin/env python3
"""Benchmark of the KV-block transfer / match hot path on one MI355X.

A "step" is one pass of the whole path over one batch: for the 64 sessions of a multi-turn
workload (Llama-3-8B GQA-shaped KV, config 3), mp_match_batch against the destination index,
then mp_transfer_with_insert_batch of every unmatched suffix (allocate, upload tables, gather,
scatter, insert).  Four consecutive steps are the four turns of one set of sessions; after the
fourth turn the sessions end (their blocks become historical) and a new set starts, so the
destination pool evicts on demand in steady state.

Prints ONE JSON line.
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0  # MI355X published HBM3E peak


def _turn(W, geom, prompts):
    toks, tok_off = W.csr(prompts)
    nblk = np.array([(len(p) + geom.bs - 1) // geom.bs for p in prompts], dtype=np.uint32)
    cap_off = np.concatenate([[0], np.cumsum(nblk)]).astype(np.uint32)
    return dict(toks=toks, tok_off=tok_off, nblk=nblk, cap_off=cap_off)


def build_epoch(W, geom, cfg, epoch, n_sessions=64, n_turns=4):
    """One epoch = the steps after which every request of the epoch has finished.  Token ids
    are fresh per epoch, so nothing matches across epochs.
      config 3: 4 steps, one per turn of 64 multi-turn sessions
      config 2: 1 step, 16 requests with log-normal lengths
      config 4: 32 steps, one 16384-token request each, 29 of them sharing an 8192-token prefix
      config 5: 1 step, 256 requests of 2048 tokens"""
    seed = cfg + 1000 * epoch
    if cfg == 3:
        sessions = W.multiturn_sessions(seed=seed, n_sessions=n_sessions, n_turns=n_turns,
                                        vocab=geom.vocab)
        return [_turn(W, geom, [sessions[s][t] for s in range(n_sessions)]) for t in range(n_turns)]
    if cfg == 2:
        return [_turn(W, geom, W.random_prompts(seed, W.lognormal_lengths(seed=seed), geom.vocab))]
    if cfg == 4:
        return [_turn(W, geom, [p]) for p in W.long_context_requests(seed=seed, vocab=geom.vocab)]
    if cfg == 5:
        return [_turn(W, geom, W.random_prompts(seed, [2048] * 256, geom.vocab))]
    raise ValueError("config must be 2, 3, 4 or 5")


def run_step_by_layer(M, src, dst, turn, perm, state, flags, n_layers, bs):
    """The by-layer flavour of a step: match, allocate once, ship one layer per call (as an
    engine would while prefill advances), then insert the prompts."""
    rc, mb, m = M.mp_match_batch(dst.h, turn["toks"], turn["tok_off"], turn["cap_off"],
                                 M.MP_MATCH_PIN)
    assert rc == 0, M.mp_last_error(dst.h)
    need = turn["nblk"] - m
    blk_off = np.concatenate([[0], np.cumsum(need)]).astype(np.int64)
    total = int(blk_off[-1])
    src_blocks = perm[:total]
    rc, d = M.mp_alloc(dst.h, total, M.MP_EVICT_ON_DEMAND)
    assert rc == 0, M.mp_last_error(dst.h)
    for l in range(n_layers):
        rc = M.mp_transfer_layers(src.h, dst.h, src_blocks, d, l, l + 1, flags)
        assert rc == 0, M.mp_last_error(src.h)
    rc, hashes, hoff = M.mp_block_hashes_batch(dst.h, turn["toks"], turn["tok_off"], bs)
    assert rc == 0
    held = [d]
    for r in range(len(m)):
        t = turn["toks"][turn["tok_off"][r]:turn["tok_off"][r + 1]]
        known = mb[turn["cap_off"][r]:turn["cap_off"][r] + m[r]]
        ids = np.concatenate([known, d[blk_off[r]:blk_off[r + 1]]])
        rc, _ = M.mp_insert_hashed(dst.h, t, hashes[hoff[r]:hoff[r + 1]], ids)
        assert rc == 0, M.mp_last_error(dst.h)
        held.append(known)
    state["held"].append(np.concatenate(held))
    return total


def run_step_per_request(M, src, dst, turn, perm, state, flags):
    """The unbatched flavour of a step: one mp_match and one mp_transfer_with_insert per request."""
    total = 0
    held = []
    for r in range(len(turn["nblk"])):
        t = turn["toks"][turn["tok_off"][r]:turn["tok_off"][r + 1]]
        nblk = int(turn["nblk"][r])
        rc, m = M.mp_match(dst.h, t, nblk, M.MP_MATCH_PIN)
        assert rc == 0, M.mp_last_error(dst.h)
        n = nblk - len(m)
        rc, d = M.mp_transfer_with_insert(src.h, dst.h, t, len(m), perm[total:total + n], flags=flags)
        assert rc == 0, M.mp_last_error(src.h)
        total += n
        held += [m, d]
    state["held"].append(np.concatenate(held))
    return total


def run_step(M, src, dst, turn, perm, state, flags):
    """One step.  Returns the number of blocks moved."""
    rc, mb, m = M.mp_match_batch(dst.h, turn["toks"], turn["tok_off"], turn["cap_off"],
                                 M.MP_MATCH_PIN)
    assert rc == 0, M.mp_last_error(dst.h)
    need = turn["nblk"] - m
    blk_off = np.concatenate([[0], np.cumsum(need)]).astype(np.uint32)
    total = int(blk_off[-1])
    # the sender's KV sits in random (fragmented) blocks of its pool
    src_blocks = perm[:total]
    rc, d = M.mp_transfer_with_insert_batch(src.h, dst.h, turn["toks"], turn["tok_off"], m,
                                            src_blocks, blk_off, flags)
    assert rc == 0, M.mp_last_error(src.h)
    pinned = [mb[turn["cap_off"][r]:turn["cap_off"][r] + m[r]] for r in range(len(m))]
    state["held"].append(np.concatenate(pinned + [d]))
    return total


def cpu_baseline(W, geom, n_sessions=64, n_turns=4, NB_src=4096, NB_dst=8704):
    """The CPU oracle, as it stands, on a bounded sample of the same workload: the four turns of
    the first two sets of sessions, same geometry, pools cut to what one set needs.  One thread,
    pinned to one core; the copy part (transfer_with_insert: allocation, memcpy by table, trie
    insert) and the hash + match part (chained block hashes of every prompt, trie walk) are timed
    separately."""
    from oracle import oracle as O
    pinned_to = None
    try:
        cores = sorted(os.sched_getaffinity(0))
        os.sched_setaffinity(0, {cores[-1]})
        pinned_to = cores[-1]
    except (AttributeError, OSError):
        cores = None
    rng = np.random.default_rng(3)
    chunk = rng.integers(0, 256, 64 << 20, dtype=np.uint8)
    src_data = np.tile(chunk, geom.pool_bytes(NB_src) // chunk.size)
    src = O.OraclePool(geom.L, geom.H, geom.D, geom.bs, geom.e, NB_src, data=src_data)
    src.alloc(NB_src)
    moved = hashed = 0
    t_copy = t_match = 0.0
    n_epochs = 2                    # about 10 s of single-thread work
    for epoch in range(n_epochs):
        dst = O.OraclePool(geom.L, geom.H, geom.D, geom.bs, geom.e, NB_dst)   # a fresh receiver
        for turn in build_epoch(W, geom, 3, epoch, n_sessions, n_turns):
            t0 = time.perf_counter()
            ms = []
            for r in range(n_sessions):
                t = turn["toks"][turn["tok_off"][r]:turn["tok_off"][r + 1]]
                O.block_hashes(t, geom.bs, 0)
                ms.append(len(dst.match(t, flags=O.MATCH_PIN)[1]))
            t_match += time.perf_counter() - t0
            need = turn["nblk"] - np.array(ms, dtype=np.uint32)
            blk_off = np.concatenate([[0], np.cumsum(need)]).astype(np.uint32)
            src_blocks = rng.permutation(NB_src)[: int(blk_off[-1])].astype(np.int32)
            t0 = time.perf_counter()
            rc, d = O.transfer_with_insert_batch(src, dst, turn["toks"], turn["tok_off"], ms, src_blocks,
                                                 blk_off, flags=O.EVICT_ON_DEMAND)
            t_copy += time.perf_counter() - t0
            assert rc == 0
            moved += int(blk_off[-1])
            hashed += int(sum(len(turn["toks"][turn["tok_off"][r]:turn["tok_off"][r + 1]]) // geom.bs
                              for r in range(n_sessions)))
        del dst
    if cores is not None:
        os.sched_setaffinity(0, set(cores))
    model = ""
    try:
        with open("/proc/cpuinfo") as f:
            model = next((ln.split(":", 1)[1].strip() for ln in f if ln.startswith("model name")), "")
    except OSError:
        pass
    t_total = t_copy + t_match
    return dict(value=moved * geom.B / t_total / 1e9, unit="GB/s", cores=1, kind="oracle",
                pinned_to_core=pinned_to, host_cpu=model, host_cores_visible=os.cpu_count(),
                sample=f"config 3, the {n_turns} turns of {n_epochs} sets of {n_sessions} sessions "
                       f"({moved} blocks = {moved * geom.B / 2**30:.2f} GiB payload, {hashed} blocks "
                       f"hashed+matched), pools reduced to {NB_src}/{NB_dst} blocks",
                seconds=round(t_total, 3), blocks_per_s=round(moved / t_total, 1),
                copy={"GBs": round(moved * geom.B / t_copy / 1e9, 2), "seconds": round(t_copy, 3),
                      "what": "transfer_with_insert: allocation, gather + scatter by memcpy, trie insert"},
                hash_match={"blocks_per_s": round(hashed / t_match, 1), "seconds": round(t_match, 4),
                            "what": "chained block hashes of every prompt + trie walk (match)"})


def per_request_c(mode, timed_sets=3):
    """Builds bench_per_request.c with gcc and runs it: the per-request flavour of the path from
    plain C, so the library's own time per request is seen without Python around it."""
    import shutil
    import subprocess
    import tempfile
    from paper_2406_17565_amd import build as B
    gcc = shutil.which("gcc")
    if gcc is None:
        return {"error": "gcc not found"}
    libdir, hip = os.path.dirname(B.LIB), "/opt/rocm/lib"
    with tempfile.TemporaryDirectory() as tmp:
        exe = os.path.join(tmp, "bench_per_request")
        cmd = [gcc, "-O2", "-std=c99", "-I", os.path.join(ROOT, "include"),
               os.path.join(ROOT, "bench_per_request.c"), "-o", exe, "-L", libdir, "-lmempool", "-L", hip,
               "-lamdhip64", f"-Wl,-rpath,{libdir}", f"-Wl,-rpath,{hip}"]
        try:
            subprocess.check_call(cmd)
            out = subprocess.run([exe, mode, str(timed_sets)], capture_output=True, text=True, timeout=300)
        except (subprocess.CalledProcessError, subprocess.TimeoutExpired, OSError) as e:
            return {"error": str(e)[:200]}
        if out.returncode != 0:
            return {"error": (out.stderr or out.stdout)[-300:]}
        res = json.loads(out.stdout.strip().splitlines()[-1])
        res.pop("what", None)
        return res


def hash_floor_us(turn, bs, clock_hz=2.4e9, pcie_bytes_per_s=64e9):
    """What the hash kernel cannot beat on one batch: the serial chain of the longest prompt (25
    dependent scalar instructions per step, and a lone wave issues one instruction every four
    cycles), and fetching the host-resident tokens over the host link."""
    nblk = (turn["tok_off"][1:] - turn["tok_off"][:-1]) // bs
    chain = float(nblk.max()) * 25 * 4 / clock_hz * 1e6
    fetch = 4.0 * float(turn["tok_off"][-1]) / pcie_bytes_per_s * 1e6
    return chain, fetch


def host_tier(args):
    """Config 5's variant: HBM pool -> pinned-host pool (gather kernel, then device-to-host
    copies of records on the side stream) and back (host-to-device, then scatter kernel).
    Bound by the host link, not by HBM; never used as the headline value."""
    import torch
    from paper_2406_17565_amd import mempool as M
    from paper_2406_17565_amd import workloads as W
    from paper_2406_17565_amd.pool import TorchPool
    g = W.CONFIGS[5]
    geom = (g.L, g.H, g.D, g.bs, g.e)
    n = 4096                                            # 2.5 GiB per transfer
    src = TorchPool(*geom, g.NB, staging_blocks=512)    # two slots of 160 MiB
    host = TorchPool(*geom, n, tier=M.MP_TIER_HOST_PINNED)
    src.mem.view(torch.int32).random_()
    torch.cuda.synchronize()
    assert M.mp_alloc(src.h, g.NB)[0] == 0
    rng = np.random.default_rng(5)
    res = {}
    for name, fl in (("copy_engine", 0), ("zero_copy_kernel", M.MP_DIRECT)):
        out_t, in_t = [], []
        for rep in range(args.steps or 5):
            tbl = rng.permutation(g.NB)[:n].astype(np.int32)
            t0 = time.perf_counter()
            rc, h = M.mp_transfer(src.h, host.h, tbl, flags=fl)
            out_t.append(time.perf_counter() - t0)
            assert rc == 0, M.mp_last_error(src.h)
            t0 = time.perf_counter()
            rc, _ = M.mp_transfer(host.h, src.h, h, tbl, flags=fl | M.MP_DST_GIVEN)   # swap back in place
            in_t.append(time.perf_counter() - t0)
            assert rc == 0, M.mp_last_error(host.h)
            assert M.mp_free(host.h, h) == 0
        res[name] = (min(out_t[1:]), min(in_t[1:]))
    # swap_out / swap_in (Table 1) between the two tiers of one instance: a cache of 32 prompts of
    # 2048 tokens moves down, coldest leaf first, and comes back prompt by prompt in one call
    up = TorchPool(*geom, n, staging_blocks=512)
    low = TorchPool(*geom, n, tier=M.MP_TIER_HOST_PINNED)
    up.mem.view(torch.int32).random_()
    torch.cuda.synchronize()
    prompts = W.random_prompts(55, [2048] * 32, g.vocab)
    swap = {}
    for name, fl in (("copy_engine", 0), ("zero_copy_kernel", M.MP_DIRECT)):
        for p in prompts:
            rc, ids = M.mp_alloc(up.h, 128)
            assert rc == 0 and M.mp_insert(up.h, p, ids)[0] == 0 and M.mp_free(up.h, ids) == 0
        t0 = time.perf_counter()
        rc, moved = M.mp_swap_out(up.h, low.h, n, fl)
        t_out = time.perf_counter() - t0
        assert rc == 0 and moved == n, M.mp_last_error(up.h)
        low_ids = np.concatenate([M.mp_match(low.h, p, 128)[1] for p in prompts])
        assert low_ids.size == n
        t0 = time.perf_counter()
        rc, up_ids = M.mp_swap_in(low.h, up.h, low_ids, fl)
        t_in = time.perf_counter() - t0
        assert rc == 0, M.mp_last_error(low.h)
        swap[name] = {"swap_out_GBs": round(n * g.B / t_out / 1e9, 2),
                      "swap_in_GBs": round(n * g.B / t_in / 1e9, 2),
                      "swap_out_us_per_block": round(t_out / n * 1e6, 2),
                      "swap_in_us_per_block": round(t_in / n * 1e6, 2)}
        assert M.mp_free(up.h, up_ids) == 0                   # empty both caches for the next flavour
        assert M.mp_evict(up.h, n) == (0, n) and M.mp_evict(low.h, n) == (0, n)
    up.close()
    low.close()
    # yardstick: one plain copy of the same bytes between a device tensor and pinned memory
    dev = src.staging[: min(src.staging.numel(), 1 << 30)]
    pin = host.mem[: dev.numel()]
    plain = {}
    for name, (a, b) in (("d2h", (pin, dev)), ("h2d", (dev, pin))):
        ts = []
        for _ in range(4):
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            a.copy_(b, non_blocking=True)
            torch.cuda.synchronize()
            ts.append(time.perf_counter() - t0)
        plain[name] = dev.numel() / min(ts[1:]) / 1e9
    payload = n * g.B
    peak = 64.0
    rate = {k: (payload / v[0] / 1e9, payload / v[1] / 1e9) for k, v in res.items()}
    best = max(rate["copy_engine"][0], rate["zero_copy_kernel"][0])
    print(json.dumps({
        "metric": "host-tier KV transfer GB/s (HBM <-> pinned host), 1 MI355X", "unit": "GB/s",
        "value": round(best, 2),
        "hbm_to_host": {k: round(v[0], 2) for k, v in rate.items()},
        "host_to_hbm": {k: round(v[1], 2) for k, v in rate.items()},
        "plain_pinned_copy": {k: round(v, 2) for k, v in plain.items()},
        "swap": swap,
        "n_gpus": 1, "dtype": "u8", "data": "synthetic",
        "config": {"workload": f"config 5 ({g.name}): {n} blocks ({payload / 2**30:.2f} GiB) per "
                               f"transfer; copy_engine = gather + hipMemcpyAsync through two 160 MiB "
                               f"staging slots, zero_copy_kernel = fused kernel on mapped host memory"},
        "roofline": {"bound": "pcie", "achieved": round(best, 2), "peak": peak, "unit": "GB/s",
                     "frac": round(best / peak, 4), "note": "PCIe Gen5 x16, one direction"}}))
    src.close()
    host.close()


def per_fragment_reference(args):
    """Reference point: the same small transfer as one copy-engine call per discrete fragment
    (the paper's one-network-call-per-block pattern, its "Original" layout) against one launch
    per direction (staged) and one fused launch."""
    import torch
    from paper_2406_17565_amd import mempool as M
    from paper_2406_17565_amd import workloads as W
    from paper_2406_17565_amd.pool import TorchPool
    out = {"metric": "per-fragment copy calls vs one launch, KV transfer GB/s", "unit": "GB/s",
           "n_gpus": 1, "dtype": "u8", "data": "synthetic", "rows": []}
    for cfg, n in ((3, 64), (5, 64)):
        g = W.CONFIGS[cfg]
        geom = (g.L, g.H, g.D, g.bs, g.e)
        NB = 2048
        src = TorchPool(*geom, NB, staging_blocks=n)
        dst = TorchPool(*geom, NB)
        src.mem.view(torch.int32).random_()
        torch.cuda.synchronize()
        M.mp_alloc(src.h, NB)
        rc, d = M.mp_alloc(dst.h, n)
        rng = np.random.default_rng(cfg)
        row = {"config": cfg, "blocks": n, "fragments": n * 2 * g.L, "fragment_bytes": g.F,
               "payload_MiB": round(n * g.B / 2**20, 1)}
        for name, fl in (("per_fragment_calls", M.MP_PER_FRAGMENT), ("staged_two_launches", 0),
                         ("fused_one_launch", M.MP_DIRECT)):
            ts = []
            for _ in range(6):
                tbl = rng.permutation(NB)[:n].astype(np.int32)
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                rc, _ = M.mp_transfer(src.h, dst.h, tbl, d, flags=fl | M.MP_DST_GIVEN)
                ts.append(time.perf_counter() - t0)
                assert rc == 0, M.mp_last_error(src.h)
            t = min(ts[1:])
            row[name] = {"GBs": round(n * g.B / t / 1e9, 2), "us": round(t * 1e6, 1),
                         "us_per_fragment": round(t * 1e6 / (n * 2 * g.L), 3)}
        out["rows"].append(row)
        src.close()
        dst.close()
        del src, dst
        torch.cuda.empty_cache()
    print(json.dumps(out))


def api_latency(args):
    """Latency of the control-plane calls, next to the paper's API study (section 8.4: about
    800 ns per block for the memory APIs, at most 0.7 ms to insert a 4K-token prompt of 256
    blocks, on the authors' Xeon host in Python)."""
    import torch
    from paper_2406_17565_amd import mempool as M
    from paper_2406_17565_amd import workloads as W
    from paper_2406_17565_amd.pool import TorchPool
    g = W.CONFIGS[3]
    p = TorchPool(1, 1, 8, g.bs, 2, g.NB)      # the control plane does not depend on fragment size
    rng = np.random.default_rng(0)

    def best(f, reps=30):
        ts = []
        for _ in range(reps):
            t0 = time.perf_counter()
            f()
            ts.append(time.perf_counter() - t0)
        return min(ts)

    out = {"metric": "MemPool API latency", "unit": "us", "n_gpus": 1, "data": "synthetic",
           "paper_context": {"alloc_free_ns_per_block": 800, "insert_256_blocks_ms": 0.7}}
    for n in (16, 256, 4096):
        def alloc_free():
            rc, ids = M.mp_alloc(p.h, n)
            M.mp_free(p.h, ids)
        out[f"alloc+free_{n}_blocks_ns_per_block"] = round(best(alloc_free) / n * 1e9, 1)
    prompt = rng.integers(0, g.vocab, 256 * g.bs, dtype=np.uint32)      # 4K tokens = 256 blocks
    rc, ids = M.mp_alloc(p.h, 256)
    rc, hashes = M.mp_block_hashes(p.h, prompt, g.bs)
    other = rng.integers(0, g.vocab, 256 * g.bs, dtype=np.uint32)
    flip = [0]

    def fresh():                 # the library remembers the last hashed batch: alternate two prompts
        flip[0] ^= 1
        return other if flip[0] else prompt
    out["block_hashes_256_blocks_us"] = round(best(lambda: M.mp_block_hashes(p.h, fresh(), g.bs)) * 1e6, 1)
    M.mp_profile_enable(p.h, True)
    for _ in range(10):
        M.mp_block_hashes(p.h, fresh(), g.bs)
    _, k_ms, k_n, _ = M.mp_profile_read(p.h, M.PROF_HASH)
    M.mp_profile_enable(p.h, False)
    out["block_hash_kernel_256_blocks_us"] = round(k_ms / max(k_n, 1) * 1e3, 1)
    for cached in (0, 128, 256):                 # cached ratio 0 %, 50 %, 100 %
        ts_i, ts_m = [], []
        for _ in range(20):
            # rebuild the state: nothing indexed, `ids` held, first `cached` blocks inserted
            M.mp_free(p.h, ids); M.mp_evict(p.h, 4096); rc, ids = M.mp_alloc(p.h, 256)
            if cached:
                M.mp_insert_hashed(p.h, prompt[: cached * g.bs], hashes[:cached], ids[:cached])
            t0 = time.perf_counter()
            rc, n_new = M.mp_insert_hashed(p.h, prompt, hashes, ids)
            ts_i.append(time.perf_counter() - t0)
            assert rc == 0 and n_new == 256 - cached
            t0 = time.perf_counter()
            rc, m = M.mp_match_hashed(p.h, prompt, hashes, 256)
            ts_m.append(time.perf_counter() - t0)
            assert len(m) == 256
        out[f"insert_hashed_256_blocks_cached{cached}_us"] = round(min(ts_i) * 1e6, 1)
        out[f"match_hashed_256_blocks_cached{cached}_us"] = round(min(ts_m) * 1e6, 1)
    out["match_256_blocks_end_to_end_us"] = round(best(lambda: M.mp_match(p.h, fresh(), 256)) * 1e6, 1)
    M.mp_free(p.h, ids); M.mp_evict(p.h, 4096); rc, ids = M.mp_alloc(p.h, 256)

    def ins():
        M.mp_block_hashes(p.h, other, g.bs)       # evict the remembered hashes of `prompt`
        t0 = time.perf_counter()
        M.mp_insert(p.h, prompt, ids)
        return time.perf_counter() - t0
    out["insert_256_blocks_end_to_end_us"] = round(min(ins() for _ in range(20)) * 1e6, 1)
    # Prefix check against prompt length (the paper's caching study, section 8.4, finds a
    # hash-per-block prefix check growing steeply with the prompt; here one chained pass and one
    # table walk: linear, a few ns per token).  Fully cached prompts, GPU hashing included.
    M.mp_free(p.h, ids); M.mp_evict(p.h, 4096)
    by_len = {}
    for nblk in (64, 256, 1024, 4096):
        t_a = rng.integers(0, g.vocab, nblk * g.bs, dtype=np.uint32)
        t_b = t_a.copy()
        t_b[-1] ^= 1                                  # same prefix but for the last block
        rc, held = M.mp_alloc(p.h, nblk)
        assert rc == 0 and M.mp_insert(p.h, t_a, held)[0] == 0
        alt = [0]

        def one():
            alt[0] ^= 1
            return M.mp_match(p.h, t_b if alt[0] else t_a, nblk)
        by_len[nblk * g.bs] = round(best(one, reps=20) * 1e6, 1)
        M.mp_free(p.h, held); M.mp_evict(p.h, 4096)
    out["match_fully_cached_us_by_prompt_tokens"] = by_len
    rc, ids = M.mp_alloc(p.h, 256)
    turns = build_epoch(W, g, 3, 0)[2:4]          # 64 prompts of about 1.5K / 2K tokens
    turn = turns[1]
    nb = int(((turn["tok_off"][1:] - turn["tok_off"][:-1]) // g.bs).sum())

    def mb():
        M.mp_match_batch(p.h, turns[0]["toks"], turns[0]["tok_off"], turns[0]["cap_off"])
        t0 = time.perf_counter()
        M.mp_match_batch(p.h, turn["toks"], turn["tok_off"], turn["cap_off"])
        return time.perf_counter() - t0
    t = min(mb() for _ in range(20))
    out["match_batch_64_prompts_us"] = round(t * 1e6, 1)
    out["match_batch_blocks_per_s"] = round(nb / t, 1)
    print(json.dumps(out))
    p.close()


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=None)
    ap.add_argument("--config", type=int, default=3)
    ap.add_argument("--direct", action="store_true", help="fused pool-to-pool kernel (no staging)")
    ap.add_argument("--sync", action="store_true", help="every call waits for its device work")
    ap.add_argument("--aggregated", action="store_true",
                    help="both pools in the aggregated layout (the paper's block aggregation)")
    ap.add_argument("--per-request", action="store_true",
                    help="one mp_match + mp_transfer_with_insert per request instead of batched calls")
    ap.add_argument("--by-layer", action="store_true",
                    help="ship one layer per call (mp_transfer_layers) instead of whole blocks")
    ap.add_argument("--host-tier", action="store_true", help="config 5 HBM <-> pinned-host variant")
    ap.add_argument("--api-latency", action="store_true", help="latency of the control-plane calls")
    ap.add_argument("--per-fragment", action="store_true",
                    help="reference point: one copy call per discrete fragment vs one launch")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-per-request", action="store_true", help="skip the per-request figures (C helper + binding)")
    ap.add_argument("--tune", default="", help="comma list key=value for mp_set_tunable")
    ap.add_argument("--guard-bytes", type=int, default=0,
                    help="allocate every pool / staging buffer between two canary bands of this many bytes "
                         "(a multiple of 256); also shifts the buffers against each other")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); "
              "run it with --gpus 1", file=sys.stderr)
        sys.exit(2)

    if args.host_tier:
        return host_tier(args)
    if args.api_latency:
        return api_latency(args)
    if args.per_fragment:
        return per_fragment_reference(args)
    if args.steps is None:
        args.steps = {2: 8, 3: 20, 4: 32, 5: 6}[args.config]
    if args.warmup is None:
        args.warmup = {2: 2, 3: 4, 4: 32, 5: 2}[args.config]

    import torch
    from paper_2406_17565_amd import mempool as M
    from paper_2406_17565_amd import workloads as W
    from paper_2406_17565_amd.pool import TorchPool

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    TorchPool.GUARD_BYTES = args.guard_bytes
    geom = W.CONFIGS[args.config]
    L, H, D, bs, e = geom.L, geom.H, geom.D, geom.bs, geom.e
    epoch0 = build_epoch(W, geom, args.config, 0)
    n_turns = len(epoch0)
    NB_src = 1024 if args.config == 4 else geom.NB   # config 4: the working set cannot be resident twice
    NB_dst = geom.NB

    # The two pools stand for two instances, so each gets its own stream: the sender's
    # transmission runs on the source stream, the receiver's hashing on the destination stream.
    # Staging: one whole step if that is below 8 GiB, else 4 GiB (the transfer runs in rounds).
    if args.config == 3:   # per turn only the reply + new tokens (and a partial block) move
        biggest = 64 * ((256 + 512 + bs - 1) // bs + 2)
    else:
        biggest = max(int(t["nblk"].sum()) for t in epoch0) + 64
    staging_blocks = biggest if biggest * geom.B <= (8 << 30) else (4 << 30) // geom.B
    s_src, s_dst = torch.cuda.Stream(), torch.cuda.Stream()
    layout = M.MP_LAYOUT_AGGREGATED if args.aggregated else M.MP_LAYOUT_DEFAULT
    src = TorchPool(L, H, D, bs, e, NB_src, staging_blocks=staging_blocks, stream=s_src, layout=layout)
    dst = TorchPool(L, H, D, bs, e, NB_dst, stream=s_dst, layout=layout)
    # KV fill: N(0,1) in the model dtype, plane by plane (harness work, not the path)
    torch.manual_seed(args.config)
    tdt = torch.bfloat16 if geom.dtype == "bf16" else torch.float16
    view = src.mem.view(tdt)
    step_elems = 1 << 28
    for off in range(0, view.numel(), step_elems):
        n = min(step_elems, view.numel() - off)
        view[off:off + n].normal_()
    dst.mem.zero_()
    torch.cuda.synchronize()
    assert M.mp_alloc(src.h, NB_src)[0] == 0       # the sender's engine owns all its blocks
    for kv in filter(None, args.tune.split(",")):
        k, v = kv.split("=")
        for p in (src, dst):
            assert M.mp_set_tunable(p.h, k, int(v)) == 0

    # MP_ASYNC: a call returns once its device work is enqueued, so the host side of step k+1
    # (match, allocation, table upload) overlaps the copy kernels of step k; the timed region
    # ends with a device synchronisation.
    flags = M.MP_EVICT_ON_DEMAND | (M.MP_DIRECT if args.direct else 0) | (0 if args.sync else M.MP_ASYNC)
    total_steps = args.warmup + args.steps
    n_epochs = (total_steps + n_turns - 1) // n_turns
    epochs = [epoch0] + [build_epoch(W, geom, args.config, ep) for ep in range(1, n_epochs)]
    rng = np.random.default_rng(args.config)
    perms = [rng.permutation(NB_src).astype(np.int32) for _ in range(total_steps)]
    state = dict(held=[])

    def do_step(i):
        ep, t = divmod(i, n_turns)
        if args.per_request:
            moved = run_step_per_request(M, src, dst, epochs[ep][t], perms[i], state, flags)
        elif args.by_layer:
            moved = run_step_by_layer(M, src, dst, epochs[ep][t], perms[i], state,
                                      flags & ~M.MP_EVICT_ON_DEMAND, L, bs)
        else:
            moved = run_step(M, src, dst, epochs[ep][t], perms[i], state, flags)
        hashed = int(((epochs[ep][t]["tok_off"][1:] - epochs[ep][t]["tok_off"][:-1]) // bs).sum())
        # requests finish: everything they held becomes historical (config 3: sessions live
        # through their four turns; the other configs' requests are single-shot)
        if t == n_turns - 1 or args.config != 3:
            for ids in state["held"]:
                assert M.mp_free(dst.h, ids) == 0
            state["held"].clear()
        return moved, hashed

    for i in range(args.warmup):
        do_step(i)
    torch.cuda.synchronize()
    # yardstick: a plain contiguous device-to-device copy (pool -> staging) on the same box
    cal_bytes = min(4 << 30, src.staging.numel() // 16 * 16)
    cal_ms = []
    for _ in range(4):
        rc, ms = M.mp_plain_copy(src.staging.data_ptr(), src.mem.data_ptr(), cal_bytes,
                                 src.stream.cuda_stream or None)
        assert rc == 0
        cal_ms.append(ms)
    copy_ceiling = 2 * cal_bytes / (min(cal_ms[1:]) * 1e-3) / 1e9
    M.mp_profile_enable(src.h, True)
    M.mp_profile_enable(dst.h, True)
    moved = hashed = 0
    # per-step device times: an event on the executing (source) stream behind every step; the
    # host may run ahead of the GPU, the gaps between events are what the GPU spent per step
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
    marks[0].record(src.stream)
    t0 = time.perf_counter()
    for k, i in enumerate(range(args.warmup, total_steps)):
        mv, hs = do_step(i)
        marks[k + 1].record(src.stream)
        moved += mv
        hashed += hs
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    step_ms = sorted(marks[k].elapsed_time(marks[k + 1]) for k in range(args.steps))
    _, h_ms, h_n, h_bytes = M.mp_profile_read(dst.h, M.PROF_HASH)      # hash launches of the timed steps

    # match on its own: the batches of the last two steps are fully indexed at the destination,
    # so every block is hashed (kernel) and probed (host).  Two batches alternate because the
    # library remembers the hashes of the last batch; no pinning, so state is unchanged.
    pair = []
    for i in (total_steps - 1, total_steps - 2):
        ep, t = divmod(i, n_turns)
        if args.config == 3 and ep != (total_steps - 1) // n_turns:
            continue                     # an earlier epoch's sessions may already be evicted
        pair.append(epochs[ep][t])
    if args.config != 3 or len(pair) < 2:
        pair = [epochs[(total_steps - 1) // n_turns][(total_steps - 1) % n_turns]]
    m_ts, m_blocks = [], 0
    for k in range(12):
        b = pair[k % len(pair)]
        nb_b = int(((b["tok_off"][1:] - b["tok_off"][:-1]) // bs).sum())
        if len(pair) == 1:               # defeat the hash cache with a one-token change
            b = dict(b, toks=b["toks"].copy())
            b["toks"][-1] ^= np.uint32(k + 1)
        t1 = time.perf_counter()
        rc, mb, m = M.mp_match_batch(dst.h, b["toks"], b["tok_off"], b["cap_off"])
        if k >= 2:
            m_ts.append(time.perf_counter() - t1)
            m_blocks += nb_b
        assert rc == 0
    match_only = m_blocks / sum(m_ts)
    last_blocks = m_blocks // len(m_ts)

    # the dominant kernel: the block-table copy (gather + scatter launches, or the fused one)
    k_ms = k_n = k_bytes = 0
    kinds = [M.PROF_DIRECT] if args.direct else [M.PROF_GATHER, M.PROF_SCATTER]
    per_kind = {}
    for kind in kinds:
        rc, ms, n, nbytes = M.mp_profile_read(src.h, kind)
        per_kind[kind] = (ms, n, nbytes)
        k_ms, k_n, k_bytes = k_ms + ms, k_n + n, k_bytes + nbytes
    _, sh_ms, sh_n, _ = M.mp_profile_read(dst.h, M.PROF_HASH)          # those of the stand-alone matches
    achieved = k_bytes / (k_ms * 1e-3) / 1e9 if k_ms else 0.0
    floors = [hash_floor_us(b, bs) for b in pair]
    chain_floor = sum(f[0] for f in floors) / len(floors)
    fetch_floor = sum(f[1] for f in floors) / len(floors)
    hash_us = sh_ms / sh_n * 1e3 if sh_n else None
    roofline_hash = {
        "bound": "latency",
        "kernel": "block_hash_kernel",
        "unit": "us per launch",
        "achieved": round(hash_us, 2) if hash_us else None,
        "peak": round(max(chain_floor, fetch_floor), 2),
        "frac": round(max(chain_floor, fetch_floor) / hash_us, 4) if hash_us else None,
        "chain_floor_us": round(chain_floor, 2),
        "token_fetch_floor_us": round(fetch_floor, 2),
        "launches": sh_n,
        "blocks_per_launch": last_blocks,
        "what": "stand-alone mp_match_batch of fully indexed batches; achieved = mean launch duration by HIP "
                "events on the destination stream (the events themselves add a few us to a launch this short); "
                "peak = the floor no schedule can beat: max(serial chain of the longest prompt at 25 dependent "
                "scalar instructions x 4 cycles per step at 2.4 GHz, host-resident tokens at 64 GB/s over the host link)",
    }

    # the same workload once more with the fused pool-to-pool kernel (half the HBM traffic), as a
    # second figure next to the headline; not part of the timed K steps above
    fused = None
    if args.config == 3 and not (args.direct or args.per_request or args.by_layer):
        for ids in state["held"]:
            assert M.mp_free(dst.h, ids) == 0
        state["held"].clear()
        n_extra = 2 * n_turns
        extra = [build_epoch(W, geom, args.config, n_epochs + k) for k in range(2)]
        f_flags = flags | M.MP_DIRECT
        f_moved, f_t0 = 0, None
        for j in range(n_extra):
            if j == n_turns:                   # first extra epoch = warm-up of the fused path
                torch.cuda.synchronize()
                M.mp_profile_read(src.h, M.PROF_DIRECT)
                f_t0 = time.perf_counter()
            mv = run_step(M, src, dst, extra[j // n_turns][j % n_turns],
                          rng.permutation(NB_src).astype(np.int32), state, f_flags)
            if j >= n_turns:
                f_moved += mv
            if j % n_turns == n_turns - 1:
                for ids in state["held"]:
                    assert M.mp_free(dst.h, ids) == 0
                state["held"].clear()
        torch.cuda.synchronize()
        f_dt = time.perf_counter() - f_t0
        _, f_ms, f_n, f_bytes = M.mp_profile_read(src.h, M.PROF_DIRECT)
        fused = {"value": round(f_moved * geom.B / f_dt / 1e9, 2), "unit": "GB/s",
                 "ms_per_step": round(f_dt / n_turns * 1e3, 4), "steps": n_turns,
                 "kernel_GBs": round(f_bytes / (f_ms * 1e-3) / 1e9, 1) if f_ms else None,
                 "path": "direct (fused pool->pool, MP_DIRECT)"}

    # HBM traffic per launch.  Counters cannot be read from inside this run: the figure is
    # DERIVED from the committed rocprofv3 FETCH_SIZE / WRITE_SIZE summary of this same command
    # (bytes fetched + written per algorithmic byte, per kernel kind) times this run's algorithmic
    # bytes -- and only if that summary was made with the kernel source as it is now; else null.
    traffic = traffic_src = None
    tpath = os.path.join(ROOT, "profiles", f"kv_block_copy_config{args.config}_hbm_traffic.json")
    if os.path.exists(tpath) and k_n:
        import profile_summary
        with open(tpath) as f:
            tj = json.load(f)
        ratios = tj.get("traffic_per_algorithmic_byte", {})
        names = {M.PROF_DIRECT: "fused", M.PROF_GATHER: "gather", M.PROF_SCATTER: "scatter"}
        if tj.get("kernel_source_sha") == profile_summary.kernel_sha() and all(names[k] in ratios for k in kinds):
            traffic = int(sum(ratios[names[k]] * per_kind[k][2] for k in kinds) / k_n)
            traffic_src = (f"derived: {os.path.relpath(tpath, ROOT)} (rocprofv3 counter ratio of this "
                           f"command, same kernel source) x this run's algorithmic bytes")
        else:
            traffic_src = "null: the committed counter summary was made with a different kernel source"

    payload = moved * geom.B
    out = {
        "metric": "KV transfer GB/s (gather+scatter) & % of HBM peak; match blocks/s, 1 MI355X",
        "value": round(payload / dt / 1e9, 2),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(dt / args.steps * 1e3, 4),
        "median_ms": round(step_ms[len(step_ms) // 2], 4),
        "min_ms": round(step_ms[0], 4),
        "max_ms": round(step_ms[-1], 4),
        "step_times": "device time between events recorded on the source stream behind every step "
                      "(steps differ in size: turn 1 of a session set moves about half of what turns 2-4 move)",
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "u8",
        "data": "synthetic",
        "config": {
            "workload": f"config {args.config} ({geom.name}): " + {
                3: "64 multi-turn sessions x 4 turns, one batched call per turn",
                2: "16 requests with log-normal lengths per step, one batched call",
                4: "one 16384-token request per step, 29 of 32 share an 8192-token prefix, "
                   "destination evicts on demand",
                5: "256 requests of 2048 tokens per step, one batched call"}[args.config]
                        + "; match, then transfer_with_insert of the unmatched suffix",
            "geometry": f"L={L} H={H} D={D} bs={bs} {geom.dtype}, F={geom.F} B={geom.B}, "
                        f"pools {NB_src}/{NB_dst} blocks ({geom.pool_bytes(NB_src) / 2**30:.0f}/"
                        f"{geom.pool_bytes(NB_dst) / 2**30:.0f} GiB), staging {staging_blocks} blocks",
            "path": "direct (fused pool->pool)" if args.direct else "staged (gather -> staging -> scatter)",
            "pool_layout": "aggregated [NB][L][2][F]" if args.aggregated else "discrete [L][2][NB][F]",
            "granularity": "by-layer (one mp_transfer_layers call per layer)" if args.by_layer
                           else "by-request (whole blocks)",
            "batching": "one call per request" if args.per_request else "one batched call per step",
            "calls": "synchronous" if args.sync else "MP_ASYNC (host work of the next step overlaps the copy kernels)",
            "blocks_moved": moved,
            "payload_GiB": round(payload / 2**30, 3),
        },
        "match_blocks_per_s": round(match_only, 1),
        "match": {"standalone_batched_blocks_per_s": round(match_only, 1),
                  "standalone_batch_us": round(sum(m_ts) / len(m_ts) * 1e6, 1),
                  "blocks_per_batch": last_blocks,
                  "inside_pipelined_steps_blocks_per_s": round(hashed / dt, 1)},
        "hash_kernel": {"launches": h_n, "avg_us": round(h_ms / h_n * 1e3, 2) if h_n else None,
                        "where": "inside the timed steps"},
        "roofline_hash": roofline_hash,
        "roofline": {
            "bound": "hbm",
            "achieved": round(achieved, 1),
            "peak": HBM_PEAK_GBS,
            "unit": "GB/s",
            "frac": round(achieved / HBM_PEAK_GBS, 4),
            "traffic": traffic,
            "traffic_source": traffic_src,
            "plain_copy_ceiling_GBs": round(copy_ceiling, 1),
            "plain_copy_bytes_each_way": cal_bytes,
            "frac_of_plain_copy": round(achieved / copy_ceiling, 4),
            "kernel": "kv_block_copy",
            "launches": k_n,
            "avg_launch_us": round(k_ms / k_n * 1e3, 2) if k_n else None,
            "alg_bytes_per_launch": int(k_bytes / k_n) if k_n else 0,
            "per_kind_GBs": {("direct" if k == M.PROF_DIRECT else "gather" if k == M.PROF_GATHER
                              else "scatter"): round(v[2] / (v[0] * 1e-3) / 1e9, 1) if v[0] else None
                             for k, v in per_kind.items()},
        },
    }
    if fused:
        out["fused"] = fused
    if args.config == 3 and not (args.direct or args.per_request or args.by_layer or args.no_per_request):
        # (A) one call per session, next to (B) the batched call per turn that `value` is: the same
        # workload with mp_match + mp_transfer_with_insert per request, from plain C (the library's
        # own time) and through this Python binding (ctypes + numpy on top)
        for ids in state["held"]:
            assert M.mp_free(dst.h, ids) == 0
        state["held"].clear()
        per_request = {"c_abi": {"staged": per_request_c("staged"), "direct": per_request_c("direct")},
                       "python_binding": {}}
        for j, (name, fl) in enumerate((("staged", flags), ("direct", flags | M.MP_DIRECT))):
            eps = [build_epoch(W, geom, 3, 100 + 2 * j + k) for k in range(2)]   # fresh prompts per flavour
            n_req = mv = 0
            for k, ep in enumerate(eps):                       # the first set of sessions warms up
                if k == 1:
                    torch.cuda.synchronize()
                    t1 = time.perf_counter()
                for turn in ep:
                    got = run_step_per_request(M, src, dst, turn, rng.permutation(NB_src).astype(np.int32),
                                               state, fl)
                    if k == 1:
                        mv += got
                        n_req += len(turn["nblk"])
                for ids in state["held"]:
                    assert M.mp_free(dst.h, ids) == 0
                state["held"].clear()
            torch.cuda.synchronize()
            t_pr = time.perf_counter() - t1
            per_request["python_binding"][name] = {"requests": n_req, "us_per_request": round(t_pr / n_req * 1e6, 2),
                                                   "GBs": round(mv * geom.B / t_pr / 1e9, 1)}
        per_request["what"] = ("config 3, one mp_match + one asynchronous mp_transfer_with_insert per request "
                               "(24-50 blocks = 48-100 MiB each); us_per_request = wall time / requests, "
                               "device synchronisation at the end included")
        out["per_request"] = per_request
    if not args.no_cpu_baseline and args.config == 3:
        out["cpu_baseline"] = cpu_baseline(W, geom)
    print(json.dumps(out))
    src.close()
    dst.close()


if __name__ == "__main__":
    main()
