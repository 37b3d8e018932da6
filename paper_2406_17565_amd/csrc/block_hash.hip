// block_hash.hip -- chained 64-bit hashes of token blocks on gfx950.
//
// The paper's index (section 4.2) is keyed by prompt tokens at block granularity; this
// library keys it by a chained hash of each block-aligned prefix:
//   d_i = FNV-1a-64 over the 4*bs bytes of block i (each uint32 token low byte first)
//   h_i = fmix64((h_{i-1} + G) xor d_i),  h_{-1} = seed,  fmix64 = splitmix64's finalizer
// Only full blocks are hashed.
//
// Mapping to the machine: integer work bound by dependent 64-bit multiplies, not by memory
// (64 B of tokens per block).  One workgroup per prompt.  The digests are parallel: one lane
// per block computes d_i into LDS (the producer wave, 64 blocks at a time).  The chain is
// serial, two multiplies per block; it is wave-uniform, so it is written on values fetched with
// readlane and runs on the scalar ALU of a second wave, which starts as soon as the first 64
// digests are there; each h_i is parked in lane i of a result register and stored 64 at a time.
#include "kv_copy.hpp"

namespace mempool {
namespace {

constexpr uint64_t kFnvOffset = 0xcbf29ce484222325ull;
constexpr uint64_t kFnvPrime = 0x100000001b3ull;
constexpr uint64_t kGolden = 0x9e3779b97f4a7c15ull;
constexpr uint64_t kMix1 = 0xbf58476d1ce4e5b9ull;
constexpr uint64_t kMix2 = 0x94d049bb133111ebull;
constexpr int kThreads = 128;  // one consumer wave, one producer wave
constexpr int kTile = 1024;  // blocks chained per LDS tile (8 KiB)
static_assert(kThreads == 128, "the kernel is written for exactly one consumer and one producer wave");

__device__ inline uint64_t fmix64(uint64_t x) {
  x ^= x >> 30;
  x *= kMix1;
  x ^= x >> 27;
  x *= kMix2;
  x ^= x >> 31;
  return x;
}

// FNV-1a-64 over the four bytes of one token, least significant byte first.
__device__ inline uint64_t fnv_token(uint64_t a, uint32_t w) {
  a = (a ^ (w & 0xffu)) * kFnvPrime;
  a = (a ^ ((w >> 8) & 0xffu)) * kFnvPrime;
  a = (a ^ ((w >> 16) & 0xffu)) * kFnvPrime;
  a = (a ^ (w >> 24)) * kFnvPrime;
  return a;
}

// One chain step for block K of the current group of 64: digest from lane K, result to lane K.
template <int K>
__device__ inline void chain_step(uint64_t &h, uint32_t dlo, uint32_t dhi, uint32_t &rlo,
                                  uint32_t &rhi) {
  const uint64_t d = ((uint64_t)(uint32_t)__builtin_amdgcn_readlane(dhi, K) << 32) |
                     (uint32_t)__builtin_amdgcn_readlane(dlo, K);
  h = fmix64((h + kGolden) ^ d);
  const uint32_t lo = (uint32_t)h, hi = (uint32_t)(h >> 32);
  asm volatile("v_writelane_b32 %0, %1, %2" : "+v"(rlo) : "s"(lo), "n"(K));
  asm volatile("v_writelane_b32 %0, %1, %2" : "+v"(rhi) : "s"(hi), "n"(K));
}

template <int K0>
__device__ inline void chain16(uint64_t &h, uint32_t dlo, uint32_t dhi, uint32_t &rlo,
                               uint32_t &rhi) {
  chain_step<K0 + 0>(h, dlo, dhi, rlo, rhi);
  chain_step<K0 + 1>(h, dlo, dhi, rlo, rhi);
  chain_step<K0 + 2>(h, dlo, dhi, rlo, rhi);
  chain_step<K0 + 3>(h, dlo, dhi, rlo, rhi);
  chain_step<K0 + 4>(h, dlo, dhi, rlo, rhi);
  chain_step<K0 + 5>(h, dlo, dhi, rlo, rhi);
  chain_step<K0 + 6>(h, dlo, dhi, rlo, rhi);
  chain_step<K0 + 7>(h, dlo, dhi, rlo, rhi);
  chain_step<K0 + 8>(h, dlo, dhi, rlo, rhi);
  chain_step<K0 + 9>(h, dlo, dhi, rlo, rhi);
  chain_step<K0 + 10>(h, dlo, dhi, rlo, rhi);
  chain_step<K0 + 11>(h, dlo, dhi, rlo, rhi);
  chain_step<K0 + 12>(h, dlo, dhi, rlo, rhi);
  chain_step<K0 + 13>(h, dlo, dhi, rlo, rhi);
  chain_step<K0 + 14>(h, dlo, dhi, rlo, rhi);
  chain_step<K0 + 15>(h, dlo, dhi, rlo, rhi);
}

// FNV-1a-64 digest of one block of bs tokens.  The tokens are fetched in groups of 16 / 4
// independent loads before they are consumed, so a block costs one or two memory round trips
// (the tokens may sit in pinned host memory) instead of one per token.
__device__ inline uint64_t block_digest(const uint32_t *__restrict__ t, uint32_t bs) {
  uint64_t a = kFnvOffset;
  uint32_t k = 0;
  for (; k + 16 <= bs; k += 16) {
    uint32_t w[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) w[i] = t[k + i];
#pragma unroll
    for (int i = 0; i < 16; ++i) a = fnv_token(a, w[i]);
  }
  for (; k + 4 <= bs; k += 4) {
    uint32_t w[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) w[i] = t[k + i];
#pragma unroll
    for (int i = 0; i < 4; ++i) a = fnv_token(a, w[i]);
  }
  for (; k < bs; ++k) a = fnv_token(a, t[k]);
  return a;
}

// One workgroup per prompt, two waves.  Wave 1 PRODUCES: group after group of 64 blocks, in
// order, it fetches the tokens, computes the digests into an LDS tile and raises the group's
// flag.  Wave 0 CONSUMES: it chains a group as soon as its flag is up.  Because every prompt of
// a batch asks for its first 64 blocks first, those tokens arrive first (over the host link,
// when they sit in pinned host memory), and the serial chain of the early groups runs while
// the later tokens are still on their way: a batch costs about max(token fetch, chain) plus
// one group, not their sum.  The producer never waits for anybody inside a tile, so the
// consumer's wait always ends; both waves meet at the barrier that closes the tile.
__global__ __launch_bounds__(kThreads) void block_hash_kernel(
    const uint32_t *__restrict__ tokens, const uint32_t *__restrict__ tok_off,
    const uint32_t *__restrict__ blk_off, uint32_t bs, uint64_t seed,
    uint64_t *__restrict__ out, uint32_t *__restrict__ done, uint32_t done_mark) {
  __shared__ uint64_t tile[kTile];
  __shared__ int ready[kTile / 64];  // ready[g] == e: the digests of group g of tile e are in LDS
  const uint32_t r = blockIdx.x;
  const uint32_t t0 = tok_off[r];
  const uint32_t nblk = (tok_off[r + 1] - t0) / bs;
  const uint32_t o0 = blk_off[r];
  const uint32_t lane = threadIdx.x & 63u;
  const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  if (threadIdx.x < kTile / 64) ready[threadIdx.x] = 0;
  __syncthreads();
  uint64_t h = seed;  // carried by wave 0 across tiles
  int epoch = 0;
  for (uint32_t base = 0; base < nblk; base += kTile) {
    ++epoch;
    const uint32_t cnt = min((uint32_t)kTile, nblk - base);
    const uint32_t groups = (cnt + 63u) / 64u;
    if (wave != 0) {
      for (uint32_t g = 0; g < groups; ++g) {
        const uint32_t j = 64u * g + lane;
        if (j < cnt) tile[j] = block_digest(tokens + t0 + (uint64_t)(base + j) * bs, bs);
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");  // the wave's LDS stores are done
        if (lane == 0)
          __hip_atomic_store(&ready[g], epoch, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
      }
    } else {
      // The chain.  Each lane fetches one digest; step k reads lane k's digest into scalar
      // registers, so h lives in SGPRs and the multiplies issue on the scalar ALU.  A lone wave
      // issues one instruction every four cycles, so the step is kept as short as possible: no
      // per-step bounds check (16 steps per check), and h_k is parked in lane k of a result
      // register with v_writelane, to be stored 64 at a time.
      // (the lane builtins return int: go through uint32_t so nothing gets sign-extended)
      h = ((uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((uint32_t)(h >> 32)) << 32) |
          (uint32_t)__builtin_amdgcn_readfirstlane((uint32_t)h);
      for (uint32_t g = 0; g < groups; ++g) {
        while (__hip_atomic_load(&ready[g], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP) != epoch)
          __builtin_amdgcn_s_sleep(1);
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
        const uint32_t jj = 64u * g;
        const uint64_t dv = (jj + lane < cnt) ? tile[jj + lane] : 0;
        const uint32_t dlo = (uint32_t)dv, dhi = (uint32_t)(dv >> 32);
        uint32_t rlo = 0, rhi = 0;
        // steps past cnt (at most 15, only in a prompt's last group) chain zeros into a copy
        // of h that is never used again
        chain16<0>(h, dlo, dhi, rlo, rhi);
        if (jj + 16 < cnt) chain16<16>(h, dlo, dhi, rlo, rhi);
        if (jj + 32 < cnt) chain16<32>(h, dlo, dhi, rlo, rhi);
        if (jj + 48 < cnt) chain16<48>(h, dlo, dhi, rlo, rhi);
        if (jj + lane < cnt) out[o0 + base + jj + lane] = ((uint64_t)rhi << 32) | rlo;
      }
    }
    __syncthreads();  // the tile and its flags are reused by the next round
  }
  // Completion mark of this prompt for a host that polls instead of synchronising the stream:
  // written after the prompt's hashes have left the wave (the fence waits for its stores and
  // pushes them out at system scope).
  if (done != nullptr && wave == 0) {
    __threadfence_system();
    if (lane == 0) __hip_atomic_store(done + r, done_mark, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_SYSTEM);
  }
}

}  // namespace

hipError_t launch_block_hash(const uint32_t *tokens, const uint32_t *tok_off,
                             const uint32_t *blk_off, uint32_t n_req, uint32_t bs, uint64_t seed,
                             uint64_t *out, hipStream_t stream, uint32_t *done, uint32_t done_mark) {
  if (n_req == 0) return hipSuccess;
  if (!tok_off || !blk_off || bs == 0) return hipErrorInvalidValue;
  hipLaunchKernelGGL(block_hash_kernel, dim3(n_req), dim3(kThreads), 0, stream, tokens, tok_off,
                     blk_off, bs, seed, out, done, done_mark);
  return hipGetLastError();
}

}  // namespace mempool
