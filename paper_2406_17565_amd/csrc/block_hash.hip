// block_hash.hip -- chained 64-bit hashes of token blocks on gfx950.
//
// The paper's index (section 4.2) is keyed by prompt tokens at block granularity; this
// library keys it by a chained hash of each block-aligned prefix:
//   d_i = FNV-1a-64 over the 4*bs bytes of block i (each uint32 token low byte first)
//   h_i = fmix64((h_{i-1} + G) xor d_i),  h_{-1} = seed,  fmix64 = splitmix64's finalizer
// Only full blocks are hashed.
//
// Mapping to the machine: integer work bound by dependent 64-bit multiplies, not by memory
// (64 B of tokens per block).  One workgroup per prompt.  Stage 1 is parallel: one lane per
// block computes d_i into LDS.  Stage 2 is the serial chain, two multiplies per block; it is
// wave-uniform, so it is written on values fetched with readlane and runs on the scalar ALU.
// Stage 3 writes the tile of hashes back coalesced.
#include "kv_copy.hpp"

namespace mempool {
namespace {

constexpr uint64_t kFnvOffset = 0xcbf29ce484222325ull;
constexpr uint64_t kFnvPrime = 0x100000001b3ull;
constexpr uint64_t kGolden = 0x9e3779b97f4a7c15ull;
constexpr uint64_t kMix1 = 0xbf58476d1ce4e5b9ull;
constexpr uint64_t kMix2 = 0x94d049bb133111ebull;
constexpr int kThreads = 256;
constexpr int kTile = 1024;  // blocks chained per LDS tile (8 KiB)

__device__ inline uint64_t fmix64(uint64_t x) {
  x ^= x >> 30;
  x *= kMix1;
  x ^= x >> 27;
  x *= kMix2;
  x ^= x >> 31;
  return x;
}

__global__ __launch_bounds__(kThreads) void block_hash_kernel(
    const uint32_t *__restrict__ tokens, const uint32_t *__restrict__ tok_off,
    const uint32_t *__restrict__ blk_off, uint32_t bs, uint64_t seed,
    uint64_t *__restrict__ out) {
  __shared__ uint64_t tile[kTile];
  const uint32_t r = blockIdx.x;
  const uint32_t t0 = tok_off[r];
  const uint32_t nblk = (tok_off[r + 1] - t0) / bs;
  const uint32_t o0 = blk_off[r];
  uint64_t h = seed;  // carried by wave 0 across tiles
  for (uint32_t base = 0; base < nblk; base += kTile) {
    const uint32_t cnt = min((uint32_t)kTile, nblk - base);
    // stage 1: digests
    for (uint32_t j = threadIdx.x; j < cnt; j += kThreads) {
      const uint32_t *t = tokens + t0 + (uint64_t)(base + j) * bs;
      uint64_t a = kFnvOffset;
      for (uint32_t k = 0; k < bs; ++k) {
        const uint32_t w = t[k];
        a = (a ^ (w & 0xffu)) * kFnvPrime;
        a = (a ^ ((w >> 8) & 0xffu)) * kFnvPrime;
        a = (a ^ ((w >> 16) & 0xffu)) * kFnvPrime;
        a = (a ^ (w >> 24)) * kFnvPrime;
      }
      tile[j] = a;
    }
    __syncthreads();
    // stage 2: chain, on wave 0.  Each lane fetches one digest; step k reads lane k's digest
    // into scalar registers, so h lives in SGPRs and the multiplies issue on the scalar ALU.
    if (threadIdx.x < 64) {
      const uint32_t lane = threadIdx.x;
      // (the lane builtins return int: go through uint32_t so nothing gets sign-extended)
      h = ((uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((uint32_t)(h >> 32)) << 32) |
          (uint32_t)__builtin_amdgcn_readfirstlane((uint32_t)h);
      for (uint32_t jj = 0; jj < cnt; jj += 64) {
        const uint64_t dv = (jj + lane < cnt) ? tile[jj + lane] : 0;
        const uint32_t dlo = (uint32_t)dv, dhi = (uint32_t)(dv >> 32);
#pragma unroll
        for (int k = 0; k < 64; ++k) {
          if (jj + k < cnt) {  // wave-uniform
            const uint64_t d = ((uint64_t)(uint32_t)__builtin_amdgcn_readlane(dhi, k) << 32) |
                               (uint32_t)__builtin_amdgcn_readlane(dlo, k);
            h = fmix64((h + kGolden) ^ d);
            if (lane == 0) tile[jj + k] = h;  // the digest of step k is already in registers
          }
        }
      }
    }
    __syncthreads();
    // stage 3: write back
    for (uint32_t j = threadIdx.x; j < cnt; j += kThreads) out[o0 + base + j] = tile[j];
    __syncthreads();
  }
}

}  // namespace

hipError_t launch_block_hash(const uint32_t *tokens, const uint32_t *tok_off,
                             const uint32_t *blk_off, uint32_t n_req, uint32_t bs, uint64_t seed,
                             uint64_t *out, hipStream_t stream) {
  if (n_req == 0) return hipSuccess;
  if (!tok_off || !blk_off || bs == 0) return hipErrorInvalidValue;
  hipLaunchKernelGGL(block_hash_kernel, dim3(n_req), dim3(kThreads), 0, stream, tokens, tok_off,
                     blk_off, bs, seed, out);
  return hipGetLastError();
}

}  // namespace mempool
