/* A plain-C user of the library: proves that include/mempool.h is valid C and that the
 * transfer path can be driven without Python or torch.  Built and run by
 * tests/test_c_abi.py (the GPU part only on a GPU machine).
 * usage: c_abi_smoke host   -> control-plane calls only (no GPU needed)
 *        c_abi_smoke gpu    -> a small transfer_with_insert on device 0, verified on the host */
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "mempool.h"

/* the few HIP runtime calls a C program needs, declared by hand to stay free of C++ headers */
extern int hipMalloc(void **p, size_t n);
extern int hipFree(void *p);
extern int hipMemcpy(void *d, const void *s, size_t n, int kind);
extern int hipHostMalloc(void **p, size_t n, unsigned flags);
extern int hipHostFree(void *p);
enum { H2D = 1, D2H = 2 };

#define CHECK(x) do { if (!(x)) { fprintf(stderr, "FAILED line %d: %s\n", __LINE__, #x); return 1; } } while (0)

static mp_pool_desc_t desc(void *base, void *staging, uint64_t staging_bytes, uint32_t nb) {
  mp_pool_desc_t d;
  memset(&d, 0, sizeof d);
  d.n_layers = 2; d.n_kv_heads = 1; d.head_dim = 8; d.block_size = 4; d.elem_bytes = 2;
  d.n_blocks = nb; d.tier = MP_TIER_HBM; d.base = base; d.staging = staging;
  d.staging_bytes = staging_bytes;
  return d;
}

int main(int argc, char **argv) {
  const uint32_t NB = 16, F = 4 * 1 * 8 * 2, B = 4 * F;
  CHECK(argc == 2);
  CHECK(mp_selftest() == MP_OK);
  if (!strcmp(argv[1], "host")) {
    static char fake[64];
    void *base = (void *)(((uintptr_t)fake + 15) & ~(uintptr_t)15);
    mp_pool_desc_t d = desc(base, NULL, 0, NB);
    mp_pool_t *p = NULL;
    int32_t ids[4];
    mp_pool_stats_t st;
    uint32_t n = 99;
    CHECK(mp_pool_create(&d, &p) == MP_OK);
    CHECK(mp_alloc(p, 4, ids, 0) == MP_OK && ids[0] == 0 && ids[3] == 3);
    CHECK(mp_free(p, ids + 1, 2) == MP_OK);
    CHECK(mp_pool_stats(p, &st) == MP_OK && st.n_free == NB - 2 && st.n_held == 2);
    CHECK(mp_alloc(p, NB, ids, 0) == MP_ENOMEM);
    CHECK(mp_evict(p, 3, &n) == MP_OK && n == 0);
    CHECK(strlen(mp_strerror(MP_ENOMEM)) > 0);
    CHECK(mp_pool_destroy(p) == MP_OK);
    printf("c_abi_smoke host ok\n");
    return 0;
  }
  {
    const size_t pool_bytes = (size_t)NB * B;
    unsigned char *h_src = malloc(pool_bytes), *h_dst = malloc(pool_bytes);
    void *d_src, *d_dst, *d_stage;
    mp_pool_t *src = NULL, *dst = NULL;
    uint32_t tokens[10], m = 0, i, pl, k;
    int32_t all[16], s_ids[3] = {9, 2, 14}, d_ids[3], got[2];
    mp_pool_desc_t ds, dd;
    for (i = 0; i < pool_bytes; ++i) h_src[i] = (unsigned char)(i * 131u + 7u);
    for (i = 0; i < 10; ++i) tokens[i] = 1000 + i;           /* 2 full blocks + 2 tokens */
    CHECK(hipMalloc(&d_src, pool_bytes) == 0 && hipMalloc(&d_dst, pool_bytes) == 0 &&
          hipMalloc(&d_stage, 3 * B) == 0);
    CHECK(hipMemcpy(d_src, h_src, pool_bytes, H2D) == 0);
    memset(h_dst, 0, pool_bytes);
    CHECK(hipMemcpy(d_dst, h_dst, pool_bytes, H2D) == 0);
    ds = desc(d_src, d_stage, 3 * B, NB);
    dd = desc(d_dst, NULL, 0, NB);
    CHECK(mp_pool_create(&ds, &src) == MP_OK && mp_pool_create(&dd, &dst) == MP_OK);
    CHECK(mp_alloc(src, NB, all, 0) == MP_OK);
    CHECK(mp_transfer_with_insert(src, dst, tokens, 10, 0, s_ids, d_ids, 3, 0, NULL, 0) == MP_OK);
    CHECK(d_ids[0] == 0 && d_ids[1] == 1 && d_ids[2] == 2);
    CHECK(mp_match(dst, tokens, 10, got, 2, &m, 0) == MP_OK && m == 2 && got[0] == 0 && got[1] == 1);
    CHECK(hipMemcpy(h_dst, d_dst, pool_bytes, D2H) == 0);
    for (k = 0; k < 3; ++k)                                   /* fragment (plane, block) at (plane*NB+block)*F */
      for (pl = 0; pl < 4; ++pl)
        CHECK(memcmp(h_dst + ((size_t)pl * NB + d_ids[k]) * F,
                     h_src + ((size_t)pl * NB + s_ids[k]) * F, F) == 0);
    {
      /* the receiver's two cached blocks move down to a pinned-host tier and one comes back */
      void *h_low = NULL;
      mp_pool_t *low = NULL;
      mp_pool_desc_t dl;
      uint32_t n_out = 0;
      int32_t one = 1, up = -1;
      const unsigned char *rec;
      CHECK(hipHostMalloc(&h_low, 4 * (size_t)B, 0) == 0);
      dl = desc(h_low, NULL, 0, 4);
      dl.tier = MP_TIER_HOST_PINNED;
      CHECK(mp_pool_create(&dl, &low) == MP_OK);
      CHECK(mp_free(dst, d_ids, 3) == MP_OK);
      CHECK(mp_swap_out(dst, low, 2, MP_DIRECT, &n_out) == MP_OK && n_out == 2);
      CHECK(mp_match(dst, tokens, 10, got, 2, &m, 0) == MP_OK && m == 0);
      CHECK(mp_match(low, tokens, 10, got, 2, &m, 0) == MP_OK && m == 2 && got[0] == 0 && got[1] == 1);
      for (k = 0; k < 2; ++k)                                 /* host block = one record [plane][F] */
        for (pl = 0; pl < 4; ++pl) {
          rec = (const unsigned char *)h_low + (size_t)k * B + (size_t)pl * F;
          CHECK(memcmp(rec, h_src + ((size_t)pl * NB + s_ids[k]) * F, F) == 0);
        }
      CHECK(mp_swap_in(low, dst, &one, 1, &up, MP_DIRECT) == MP_OK && up >= 0);
      CHECK(mp_match(dst, tokens, 10, got, 2, &m, 0) == MP_OK && m == 2 && got[1] == up);
      CHECK(mp_free(dst, &up, 1) == MP_OK);
      CHECK(mp_pool_destroy(low) == MP_OK);
      hipHostFree(h_low);
    }
    CHECK(mp_pool_destroy(src) == MP_OK && mp_pool_destroy(dst) == MP_OK);
    hipFree(d_src); hipFree(d_dst); hipFree(d_stage);
    printf("c_abi_smoke gpu ok\n");
  }
  return 0;
}
