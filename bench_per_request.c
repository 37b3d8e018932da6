/* bench_per_request.c -- the per-request flavour of the hot path, driven from plain C so that
 * the library's own time per request is seen without any Python / ctypes / numpy around it.
 *
 * Workload: configuration 3 (Llama-3-8B GQA shape: L=32, H=8, D=128, bs=16, 2-byte elements;
 * 32 KiB fragments, 2 MiB records), pools of 16384 blocks, 64 multi-turn sessions x 4 turns with
 * prompt_t = prompt_{t-1} + 256 reply tokens + U{128..512} new tokens.  For every request of a
 * turn: mp_match(dst, MP_MATCH_PIN), then mp_transfer_with_insert of the unmatched suffix
 * (MP_EVICT_ON_DEMAND | MP_ASYNC, or MP_DIRECT on top with `direct`).  After the fourth turn the
 * sessions end (everything they held becomes historical) and a new set starts, so the
 * destination evicts on demand in steady state.  One set of sessions warms up, the rest is
 * timed with clock_gettime around each call and around the whole timed part (which ends with a
 * device synchronisation).
 *
 * Built and run by bench.py (one JSON line on stdout); stand-alone:
 *   gcc -O2 -std=c99 -I include bench_per_request.c -o bench_per_request \
 *       -L paper_2406_17565_amd -lmempool -L /opt/rocm/lib -lamdhip64 \
 *       -Wl,-rpath,$PWD/paper_2406_17565_amd -Wl,-rpath,/opt/rocm/lib
 *   ./bench_per_request [staged|direct] [timed_sets]
 */
#define _POSIX_C_SOURCE 200809L
#include <stdio.h>
#include <stdlib.h>
#include <string.h>
#include <time.h>

#include "mempool.h"

/* the few HIP runtime calls needed, declared by hand to stay free of C++ headers */
extern int hipMalloc(void **p, size_t n);
extern int hipFree(void *p);
extern int hipMemset(void *p, int v, size_t n);
extern int hipDeviceSynchronize(void);
extern int hipStreamCreateWithFlags(void **s, unsigned flags);
extern int hipStreamDestroy(void *s);

#define CHECK(x) do { if (!(x)) { fprintf(stderr, "FAILED line %d: %s\n", __LINE__, #x); return 1; } } while (0)

enum { L = 32, H = 8, D = 128, BS = 16, E = 2, NB = 16384, SESSIONS = 64, TURNS = 4, REPLY = 256 };

static uint64_t rng_state = 0x9E3779B97F4A7C15ull;
static uint32_t rnd(void) { /* xorshift64* */
  rng_state ^= rng_state >> 12; rng_state ^= rng_state << 25; rng_state ^= rng_state >> 27;
  return (uint32_t)((rng_state * 0x2545F4914F6CDD1Dull) >> 32);
}
static double now_us(void) {
  struct timespec t;
  clock_gettime(CLOCK_MONOTONIC, &t);
  return t.tv_sec * 1e6 + t.tv_nsec * 1e-3;
}

int main(int argc, char **argv) {
  const int direct = argc > 1 && !strcmp(argv[1], "direct");
  const int timed_sets = argc > 2 ? atoi(argv[2]) : 3;
  const size_t F = (size_t)BS * H * D * E, B = 2 * L * F;
  const size_t pool_bytes = B * NB, staging_blocks = 64, max_tok = TURNS * (512 + REPLY);
  void *d_src, *d_dst, *d_stage, *s_src, *s_dst;
  mp_pool_t *src = NULL, *dst = NULL;
  mp_pool_desc_t ds, dd;
  int32_t *all = malloc(sizeof(int32_t) * NB), *perm = malloc(sizeof(int32_t) * NB);
  int32_t *held = malloc(sizeof(int32_t) * NB * 2), *matched = malloc(sizeof(int32_t) * 256),
          *dst_ids = malloc(sizeof(int32_t) * 256);
  uint32_t *tokens = malloc(sizeof(uint32_t) * SESSIONS * max_tok), len[SESSIONS];
  uint32_t flags = MP_EVICT_ON_DEMAND | MP_ASYNC | (direct ? MP_DIRECT : 0);
  double t_match = 0, t_xfer = 0, t_wall = 0, t0 = 0;
  unsigned long long blocks = 0, requests = 0, hashed = 0;
  int set, turn, s, i;
  CHECK(all && perm && held && matched && dst_ids && tokens);
  CHECK(hipMalloc(&d_src, pool_bytes) == 0 && hipMalloc(&d_dst, pool_bytes) == 0 &&
        hipMalloc(&d_stage, staging_blocks * B) == 0);
  CHECK(hipMemset(d_src, 0x5a, pool_bytes) == 0 && hipMemset(d_dst, 0, pool_bytes) == 0);
  CHECK(hipStreamCreateWithFlags(&s_src, 1) == 0 && hipStreamCreateWithFlags(&s_dst, 1) == 0);
  memset(&ds, 0, sizeof ds);
  ds.n_layers = L; ds.n_kv_heads = H; ds.head_dim = D; ds.block_size = BS; ds.elem_bytes = E;
  ds.n_blocks = NB; ds.tier = MP_TIER_HBM;
  dd = ds;
  ds.base = d_src; ds.staging = d_stage; ds.staging_bytes = staging_blocks * B; ds.stream = s_src;
  dd.base = d_dst; dd.stream = s_dst; dd.instance_id = 1;
  CHECK(mp_pool_create(&ds, &src) == MP_OK && mp_pool_create(&dd, &dst) == MP_OK);
  CHECK(mp_alloc(src, NB, all, 0) == MP_OK); /* the sender's engine owns all its blocks */
  for (i = 0; i < NB; ++i) perm[i] = i;
  CHECK(hipDeviceSynchronize() == 0);

  for (set = 0; set < 1 + timed_sets; ++set) {
    uint32_t n_held = 0;
    if (set == 1) { CHECK(hipDeviceSynchronize() == 0); t0 = now_us(); }
    memset(len, 0, sizeof len);
    for (turn = 0; turn < TURNS; ++turn) {
      uint32_t next = 0;
      for (i = NB - 1; i > 0; --i) { /* the sender's KV sits in random blocks: fresh permutation per turn */
        const uint32_t j = rnd() % (uint32_t)(i + 1);
        const int32_t t = perm[i]; perm[i] = perm[j]; perm[j] = t;
      }
      for (s = 0; s < SESSIONS; ++s) {
        uint32_t *tok = tokens + (size_t)s * max_tok, add = (turn ? REPLY : 0) + 128 + rnd() % 385, m = 0, k;
        uint32_t n_tok, nblk, n;
        double a, b, c;
        for (k = 0; k < add; ++k) tok[len[s] + k] = rnd() % 128256u;
        len[s] += add;
        n_tok = len[s];
        nblk = (n_tok + BS - 1) / BS;
        a = now_us();
        CHECK(mp_match(dst, tok, n_tok, matched, nblk, &m, MP_MATCH_PIN) == MP_OK);
        b = now_us();
        n = nblk - m;
        CHECK(next + n <= NB);
        CHECK(mp_transfer_with_insert(src, dst, tok, n_tok, m, perm + next, dst_ids, n, flags, NULL, 0) == MP_OK);
        c = now_us();
        next += n;
        memcpy(held + n_held, matched, sizeof(int32_t) * m); n_held += m;
        memcpy(held + n_held, dst_ids, sizeof(int32_t) * n); n_held += n;
        if (set >= 1) { t_match += b - a; t_xfer += c - b; blocks += n; ++requests; hashed += n_tok / BS; }
      }
    }
    CHECK(mp_free(dst, held, n_held) == MP_OK); /* the sessions end */
  }
  CHECK(hipDeviceSynchronize() == 0);
  t_wall = now_us() - t0;
  printf("{\"path\": \"%s\", \"requests\": %llu, \"blocks_moved\": %llu, \"payload_GiB\": %.3f, "
         "\"us_per_request\": %.2f, \"match_us\": %.2f, \"transfer_with_insert_us\": %.2f, "
         "\"GBs\": %.1f, \"match_blocks_per_s\": %.0f, \"what\": \"plain C over the C ABI: wall time of the "
         "timed part / requests (ends with a device synchronisation); match_us and transfer_with_insert_us "
         "are the mean host time inside each call (mp_match waits for its hashes, the transfer is MP_ASYNC)\"}\n",
         direct ? "direct" : "staged", requests, blocks, blocks * (double)B / (1u << 30), t_wall / requests,
         t_match / requests, t_xfer / requests, blocks * (double)B / (t_wall * 1e-6) / 1e9,
         hashed / (t_match * 1e-6));
  CHECK(mp_pool_destroy(src) == MP_OK && mp_pool_destroy(dst) == MP_OK);
  hipStreamDestroy(s_src); hipStreamDestroy(s_dst);
  hipFree(d_src); hipFree(d_dst); hipFree(d_stage);
  return 0;
}
