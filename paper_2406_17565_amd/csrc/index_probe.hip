// index_probe.hip -- device-resident copy of the prompt index and its probe kernel (gfx950).
//
// Paper section 4.2: match walks the token-keyed index at block granularity.  Here the walk
// can run on the GPU right behind the hash kernel: an open-addressing table (chained hash ->
// block id) plus each node's parent id and bs tokens live in HBM, kept current by replaying
// the host index's change log.  A hit is accepted under the same three checks as on the host
// (hash equal, parent link equal, tokens equal), so both probes give identical answers.
//
// Mapping: one workgroup per prompt; lane-per-block lookups and token compares run in
// parallel, the parent links are checked in a second pass over an LDS tile of candidates, and
// an LDS atomic-min finds the first block that fails.  Loops over the table are bounded by
// its capacity, so every wave terminates whatever the table holds.
#include "kv_copy.hpp"

namespace mempool {
namespace {

constexpr int kThreads = 256;
constexpr int kTile = 1024;

__device__ inline uint64_t home_slot(uint64_t h, uint64_t mask) { return (h ^ (h >> 32)) & mask; }

__global__ __launch_bounds__(kThreads) void index_probe_kernel(
    const uint32_t *__restrict__ tokens, const uint32_t *__restrict__ tok_off,
    const uint32_t *__restrict__ hash_off, const uint64_t *__restrict__ hashes,
    const uint32_t *__restrict__ out_off, uint32_t bs, const uint64_t *__restrict__ keys,
    const int32_t *__restrict__ vals, const int32_t *__restrict__ parent,
    const uint32_t *__restrict__ node_tokens, uint64_t mask, int32_t *__restrict__ ids_out,
    uint32_t *__restrict__ n_matched_out) {
  __shared__ int32_t cand[kTile];
  __shared__ uint32_t first_bad;
  __shared__ int32_t carry;
  const uint32_t r = blockIdx.x;
  const uint32_t t0 = tok_off[r], h0 = hash_off[r], o0 = out_off[r];
  const uint32_t nblk = min(hash_off[r + 1] - h0, out_off[r + 1] - o0);
  if (threadIdx.x == 0) {
    first_bad = nblk;
    carry = -1;
  }
  __syncthreads();
  for (uint32_t base = 0; base < nblk; base += kTile) {
    const uint32_t cnt = min((uint32_t)kTile, nblk - base);
    for (uint32_t j = threadIdx.x; j < cnt; j += kThreads) {
      const uint64_t h = hashes[h0 + base + j];
      uint64_t s = home_slot(h, mask);
      int32_t b = -1;
      for (uint64_t probes = 0; probes <= mask; ++probes) {  // bounded by the capacity
        const int32_t v = vals[s];
        if (v < 0) break;
        if (keys[s] == h) {
          b = v;
          break;
        }
        s = (s + 1) & mask;
      }
      if (b >= 0) {
        const uint32_t *a = tokens + t0 + (uint64_t)(base + j) * bs;
        const uint32_t *n = node_tokens + (uint64_t)b * bs;
        for (uint32_t k = 0; k < bs; ++k)
          if (a[k] != n[k]) {
            b = -1;
            break;
          }
      }
      cand[j] = b;
    }
    __syncthreads();
    for (uint32_t j = threadIdx.x; j < cnt; j += kThreads) {
      const int32_t b = cand[j];
      const int32_t prev = j ? cand[j - 1] : carry;
      if (b >= 0 && parent[b] == prev) ids_out[o0 + base + j] = b;
      else atomicMin(&first_bad, base + j);
    }
    __syncthreads();
    if (first_bad < base + cnt) break;  // uniform: read after the barrier
    if (threadIdx.x == 0) carry = cand[cnt - 1];
    __syncthreads();
  }
  if (threadIdx.x == 0) n_matched_out[r] = first_bad;
}

// Replays a change log: slot updates are (slot, val, key) records of 16 bytes, node updates
// are (block, parent, tokens[bs]) records of 2 + bs dwords.
__global__ __launch_bounds__(kThreads) void index_apply_kernel(
    const uint32_t *__restrict__ slot_upd, uint32_t n_slots, const uint32_t *__restrict__ node_upd,
    uint32_t n_nodes, uint32_t bs, uint64_t *__restrict__ keys, int32_t *__restrict__ vals,
    int32_t *__restrict__ parent, uint32_t *__restrict__ node_tokens) {
  const uint32_t i = blockIdx.x * kThreads + threadIdx.x;
  if (i < n_slots) {
    const uint32_t *u = slot_upd + 4ull * i;
    keys[u[0]] = ((uint64_t)u[3] << 32) | u[2];
    vals[u[0]] = (int32_t)u[1];
  }
  if (i < n_nodes) {
    const uint32_t *u = node_upd + (uint64_t)(2 + bs) * i;
    const uint32_t b = u[0];
    parent[b] = (int32_t)u[1];
    for (uint32_t k = 0; k < bs; ++k) node_tokens[(uint64_t)b * bs + k] = u[2 + k];
  }
}

}  // namespace

hipError_t launch_index_probe(const uint32_t *tokens, const uint32_t *tok_off,
                              const uint32_t *hash_off, const uint64_t *hashes,
                              const uint32_t *out_off, uint32_t n_req, uint32_t bs,
                              const uint64_t *keys, const int32_t *vals, const int32_t *parent,
                              const uint32_t *node_tokens, uint64_t capacity, int32_t *ids_out,
                              uint32_t *n_matched_out, hipStream_t stream) {
  if (n_req == 0) return hipSuccess;
  if (!tok_off || !hash_off || !out_off || !keys || !vals || !parent || !node_tokens || !ids_out ||
      !n_matched_out || capacity == 0 || (capacity & (capacity - 1)))
    return hipErrorInvalidValue;
  hipLaunchKernelGGL(index_probe_kernel, dim3(n_req), dim3(kThreads), 0, stream, tokens, tok_off,
                     hash_off, hashes, out_off, bs, keys, vals, parent, node_tokens, capacity - 1,
                     ids_out, n_matched_out);
  return hipGetLastError();
}

hipError_t launch_index_apply(const uint32_t *slot_upd, uint32_t n_slots, const uint32_t *node_upd,
                              uint32_t n_nodes, uint32_t bs, uint64_t *keys, int32_t *vals,
                              int32_t *parent, uint32_t *node_tokens, hipStream_t stream) {
  const uint32_t n = n_slots > n_nodes ? n_slots : n_nodes;
  if (n == 0) return hipSuccess;
  hipLaunchKernelGGL(index_apply_kernel, dim3((n + kThreads - 1) / kThreads), dim3(kThreads), 0,
                     stream, slot_upd, n_slots, node_upd, n_nodes, bs, keys, vals, parent,
                     node_tokens);
  return hipGetLastError();
}

}  // namespace mempool
