// kv_copy.hpp -- host-side interface of the block-table copy kernel (gfx950).
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>

namespace mempool {

// One end of a block-table copy.  Fragment (plane p, entry i) starts at
//   base + p * plane_stride + id(i) * block_stride,   id(i) = tbl ? tbl[i] : i.
// An HBM pool ([L][2][NB][F], the discrete layout of the paper's section 5.2) has
// plane_stride = NB*F and block_stride = F; staging and the aggregated host layout
// ([n][L][2][F]) have plane_stride = F and block_stride = 2*L*F.
struct CopySide {
  void *base = nullptr;
  const int32_t *tbl = nullptr;  // DEVICE pointer, or null for the identity
  uint64_t plane_stride = 0;
  uint64_t block_stride = 0;
  bool ascending = false;        // the ids in tbl are known to ascend (the host sorted the table)
};

// Launch shape of the copy kernel.  -1 = choose from the geometry (see default_tune).
struct CopyTune {
  int order = -1;           // 0: walk records (entry-major), 1: walk planes (plane-major)
  int plane_tile = -1;      // >0: planes walked together per entry (rounded down to a divisor of
                            // the plane count); the two orders are its extremes: all planes / 1
  int unroll = -1;          // 16-byte loads in flight per lane: 1, 2, 4 or 8
  int wg_per_cu = -1;       // 0: one pass over the items; >0: persistent grid of that many WGs per CU
  int nontemporal = -1;     // stream past the caches
  int waves_per_wg = -1;    // 1 or 4 wavefronts per workgroup
  int xcd_contiguous = -1;  // 1: each XCD walks one contiguous eighth of the work items
  int item_limit = 0;       // >0: at most this many wave-items per launch (tests of the
                            // multi-launch split); 0 = the kernel's index range, 2^31-1
};

// Fills every field of `t` that is still -1.  Measured on MI355X (sweeps over all five
// geometries): one 16-byte load per lane and one-wave workgroups give the most bandwidth
// (many small independent waves beat deep unrolling).  Reads run at the same rate whatever
// the order of the fragments; WRITES are the sensitive side -- they reach copy speed only
// when the stores that are in flight together sweep ascending addresses of one plane.  So:
// when the destination is a discrete pool and its ids ascend (the host sorts the table pair by
// destination id), walk plane by plane with each XCD on a contiguous eighth of the items;
// otherwise walk records when one side is contiguous (staging, an aggregated pool) and planes
// when both sides are discrete pools; the per-XCD contiguous walk then helps for fragments of
// 64 KiB and more, and from 16 KiB when the destination is a discrete pool.  Waves per
// workgroup (1 to 16 tried) make no difference once the XCDs walk contiguous ranges; one it is.
CopyTune default_tune(CopyTune t, uint64_t frag_bytes, bool both_sides_discrete_pools,
                      bool dst_is_discrete_pool, bool dst_ids_ascend);

// Unsigned division by an invariant divisor for numerators below 2^31:
// x / d == (x * m) >> s.
struct FastDiv {
  uint32_t d = 1, m = 0x80000000u, s = 31;
};
FastDiv make_fastdiv(uint32_t d);
__host__ __device__ inline uint32_t fastdiv(uint32_t x, const FastDiv &f) {
  return (uint32_t)(((uint64_t)x * f.m) >> f.s);
}

// Copies n entries x n_planes fragments of frag_bytes (a multiple of 16) from src to dst.
// Enqueues on `stream`; returns the launch status.  n_cus sizes a persistent grid.
hipError_t launch_block_copy(const CopySide &src, const CopySide &dst, uint32_t n,
                             uint32_t n_planes, uint64_t frag_bytes, const CopyTune &tune,
                             int n_cus, hipStream_t stream);

// A transfer of one request has a few dozen table entries: its ids travel in the kernel
// arguments, so no table has to be copied to the device before the launch.
constexpr uint32_t kSmallTable = 192;
struct SmallTables {
  int32_t src[kSmallTable];
  int32_t dst[kSmallTable];
};
// Can launch_block_copy_small take this copy?  (n within the argument tables, default launch
// shape apart from the walk order)
bool small_copy_possible(uint32_t n, uint32_t n_planes, uint64_t frag_bytes, const CopyTune &tune);
// The same copy as launch_block_copy with the ids of the sides that have a table (src_tbl /
// dst_tbl) taken from `ids`; CopySide::tbl is ignored.
hipError_t launch_block_copy_small(const CopySide &src, const CopySide &dst, const SmallTables &ids,
                                   bool src_tbl, bool dst_tbl, uint32_t n, uint32_t n_planes,
                                   uint64_t frag_bytes, const CopyTune &tune, int n_cus,
                                   hipStream_t stream);

// Contiguous device-to-device copy of `bytes` (a multiple of 16): the calibration yardstick.
hipError_t launch_plain_copy(void *dst, const void *src, uint64_t bytes, hipStream_t stream);

// Chained block hashes for a batch of prompts (one workgroup per prompt).
//   tokens  : device, all prompts concatenated
//   tok_off : device, n_req+1 token offsets
//   blk_off : device, n_req+1 output offsets (prefix sums of floor(len/bs))
//   out     : device, blk_off[n_req] hashes
//   done    : null, or n_req words in host-visible memory: prompt r's word is set to done_mark
//             (system scope) once its hashes are written, for a host that polls
hipError_t launch_block_hash(const uint32_t *tokens, const uint32_t *tok_off,
                             const uint32_t *blk_off, uint32_t n_req, uint32_t bs, uint64_t seed,
                             uint64_t *out, hipStream_t stream, uint32_t *done = nullptr,
                             uint32_t done_mark = 0);

// Probe of the device-resident index copy for a batch of prompts, right behind the hash kernel.
//   hashes / hash_off : the chained hashes and their n_req+1 offsets (floor(len/bs) per prompt)
//   out_off           : n_req+1 slot offsets into ids_out (request r may use out_off[r+1]-out_off[r])
//   keys/vals/parent/node_tokens : the device copy (capacity a power of two)
//   ids_out[out_off[r] + i] = block of prompt r's block i for i < n_matched_out[r]
hipError_t launch_index_probe(const uint32_t *tokens, const uint32_t *tok_off,
                              const uint32_t *hash_off, const uint64_t *hashes,
                              const uint32_t *out_off, uint32_t n_req, uint32_t bs,
                              const uint64_t *keys, const int32_t *vals, const int32_t *parent,
                              const uint32_t *node_tokens, uint64_t capacity, int32_t *ids_out,
                              uint32_t *n_matched_out, hipStream_t stream);

// Replays the host index's change log onto the device copy.
hipError_t launch_index_apply(const uint32_t *slot_upd, uint32_t n_slots, const uint32_t *node_upd,
                              uint32_t n_nodes, uint32_t bs, uint64_t *keys, int32_t *vals,
                              int32_t *parent, uint32_t *node_tokens, hipStream_t stream);

}  // namespace mempool
