// mempool_api.hip -- the C ABI of libmempool (see include/mempool.h for the contract).
//
// Paper: Table 1 (MemPool API), section 4.3 (transfer = allocation, transmission, insertion;
// an explicit destination list skips allocation; transfer_with_insert lets the receiver
// insert locally), section 4.2 (index), section 5.2 (discrete vs aggregated layout).
//
// This file holds host orchestration only: argument checks, the order of the three steps,
// table / token staging through pinned memory, stream and event plumbing.  All data movement
// and hashing is done by the kernels in kv_copy.hip and block_hash.hip (plus hipMemcpyAsync
// for the pinned-host tier).
#include "../../include/mempool.h"

#include <hip/hip_runtime.h>

#include <algorithm>
#include <atomic>
#include <chrono>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>
#include <string>
#include <vector>

#include "kv_copy.hpp"
#include "pool_index.hpp"

using namespace mempool;

// Block tables of mp_transfer_static: [src ids, MP_STATIC_MAX_BLOCKS][dst ids, MP_STATIC_MAX_BLOCKS]
// in the library's device image, 512 KiB per GPU, held until the process ends.  In host code
// this name is only a handle for hipGetSymbolAddress; kernels and copies get the per-device
// address kept in g_static_tables[].
static __device__ __align__(256) int32_t scratch[2 * MP_STATIC_MAX_BLOCKS];

namespace {

constexpr int kMaxDevices = 64;
int32_t *g_static_tables[kMaxDevices] = {};  // device address of `scratch`, per device
std::mutex g_static_mutex;

enum ProfKind { kProfGather = 0, kProfScatter = 1, kProfDirect = 2, kProfHash = 3, kProfKinds = 4 };

struct ProfRec {
  int kind;
  hipEvent_t start, stop;
  uint64_t bytes;
};

// A device buffer with a pinned host mirror, grown on demand.
struct MirrorBuf {
  void *dev = nullptr;
  void *host = nullptr;
  size_t cap = 0;
};

struct DeviceCtx {
  bool ready = false;
  int device = 0;
  int n_cus = 256;
  hipStream_t stream = nullptr;  // the caller's stream (from the pool descriptor)
  hipStream_t side = nullptr;    // library-owned, for pinned-host tier copies
  hipStream_t hash = nullptr;    // library-owned: hashing of host-resident tokens, which touches
                                 // no pool memory and so need not queue behind the pool's copies
  // Block tables go up through a small ring of pinned buffers so that asynchronous calls can
  // run ahead of the GPU; the last uploaded pair is remembered, because by-layer transfers
  // repeat one table pair for every layer.
  static constexpr int kTableSlots = 4;
  MirrorBuf tables[kTableSlots];  // each [src ids][dst ids]
  hipEvent_t tables_uploaded[kTableSlots] = {nullptr, nullptr, nullptr, nullptr};
  bool tables_pending[kTableSlots] = {false, false, false, false};
  int tables_next = 0;
  int tables_last = -1;           // slot holding `last_ids`, -1 = none
  uint32_t last_n = 0;
  bool last_has_src = false, last_has_dst = false;
  int last_sort_by = -1;
  std::vector<int32_t> last_ids;  // the caller's arrays of the last upload: [src n][dst n]
  MirrorBuf tokens;              // concatenated prompts
  MirrorBuf offsets;             // [tok_off][blk_off]
  MirrorBuf hashes;
  MirrorBuf hash_done;           // pinned: one completion word per prompt, polled by the host
  uint32_t hash_mark = 0;        // value the words take for the current launch (never 0)
  // the pinned buffers above still hold the last hashed batch: a transfer_with_insert that
  // follows a match of the same prompts reuses the hashes instead of launching again
  bool hash_cache_valid = false;
  uint32_t hash_cache_n_req = 0;
  // device-resident copy of the index (open-addressing table + per-node parent and tokens),
  // present once the "device_probe" tunable has been switched on
  bool mirror_on = false;
  uint64_t mirror_cap = 0;
  uint64_t *m_keys = nullptr;
  int32_t *m_vals = nullptr;
  int32_t *m_parent = nullptr;
  uint32_t *m_tokens = nullptr;
  MirrorBuf m_updates;  // pinned change records the apply kernel reads
  MirrorBuf m_out;      // pinned: [out offsets][matched counts][block ids]
  // Ordering of the staging buffer between the main stream and the side stream (host-tier
  // copies): `staging_idle` is recorded on the main stream when a host-tier transfer starts and
  // the side stream waits for it, so the copy engine never touches staging before every
  // earlier main-stream user (gather, scatter, HBM->HBM rounds) is done with it; inside the
  // call the two slots are handed back and forth with the per-slot events.
  hipEvent_t staging_idle = nullptr;
  hipEvent_t slot_filled[2] = {nullptr, nullptr};   // main -> side (or side -> main)
  hipEvent_t slot_drained[2] = {nullptr, nullptr};  // the other direction
  bool profiling = false;
  std::vector<ProfRec> prof;
  double prof_ms[kProfKinds] = {0, 0, 0, 0};
  uint64_t prof_launches[kProfKinds] = {0, 0, 0, 0};
  uint64_t prof_bytes[kProfKinds] = {0, 0, 0, 0};
};

}  // namespace

struct mp_pool {
  mp_pool_desc_t desc;
  uint64_t F = 0, B = 0;
  uint32_t P = 0;  // planes = 2*L
  PoolIndex idx;
  DeviceCtx dev;
  CopyTune tune;
  std::string err;
  mp_recv_cb cb = nullptr;
  void *cb_user = nullptr;
  std::vector<int32_t> scratch_ids;
  std::vector<uint64_t> sort_a, sort_b;  // table sorting
  std::vector<uint32_t> twi_hoff, twi_ids_off, twi_present, match_hoff;  // per-call scratch of
  std::vector<int32_t> twi_ids;                                          // transfer_with_insert / match
};

namespace {

int fail(mp_pool *p, int code, const char *msg) {
  if (p) p->err = msg;
  return code;
}

int fail_hip(mp_pool *p, hipError_t e, const char *where) {
  if (p) p->err = std::string(where) + ": " + hipGetErrorString(e);
  return MP_EHIP;
}

// No C++ exception may cross the C ABI: every entry point that can allocate host memory
// turns a failure into MP_EHOST.
#define MP_CATCH(pool)                                                        \
  catch (const std::bad_alloc &) {                                            \
    return fail(pool, MP_EHOST, "out of host memory");                        \
  }                                                                           \
  catch (...) {                                                               \
    return fail(pool, MP_EHOST, "unexpected internal error");                 \
  }

#define HIP_TRY(pool, expr)                                  \
  do {                                                       \
    hipError_t e_ = (expr);                                  \
    if (e_ != hipSuccess) return fail_hip(pool, e_, #expr);  \
  } while (0)

bool aggregated(const mp_pool *p) {
  return p->desc.layout == MP_LAYOUT_AGGREGATED ||
         (p->desc.layout == MP_LAYOUT_DEFAULT && p->desc.tier == MP_TIER_HOST_PINNED);
}

bool same_geometry(const mp_pool *a, const mp_pool *b) {
  return a->desc.n_layers == b->desc.n_layers && a->desc.n_kv_heads == b->desc.n_kv_heads &&
         a->desc.head_dim == b->desc.head_dim && a->desc.block_size == b->desc.block_size &&
         a->desc.elem_bytes == b->desc.elem_bytes;
}

// ---- device context ----------------------------------------------------------------------
void destroy_device_objects(DeviceCtx &d) {
  if (d.side) (void)hipStreamDestroy(d.side);
  if (d.hash) (void)hipStreamDestroy(d.hash);
  d.side = d.hash = nullptr;
  for (int s = 0; s < DeviceCtx::kTableSlots; ++s) {
    if (d.tables_uploaded[s]) (void)hipEventDestroy(d.tables_uploaded[s]);
    d.tables_uploaded[s] = nullptr;
  }
  if (d.staging_idle) (void)hipEventDestroy(d.staging_idle);
  d.staging_idle = nullptr;
  for (int s = 0; s < 2; ++s) {
    if (d.slot_filled[s]) (void)hipEventDestroy(d.slot_filled[s]);
    if (d.slot_drained[s]) (void)hipEventDestroy(d.slot_drained[s]);
    d.slot_filled[s] = d.slot_drained[s] = nullptr;
  }
}

int create_device_objects(mp_pool *p) {
  DeviceCtx &d = p->dev;
  HIP_TRY(p, hipGetDevice(&d.device));
  int cus = 0;
  HIP_TRY(p, hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, d.device));
  d.n_cus = cus > 0 ? cus : 256;
  d.stream = (hipStream_t)p->desc.stream;
  HIP_TRY(p, hipStreamCreateWithFlags(&d.side, hipStreamNonBlocking));
  HIP_TRY(p, hipStreamCreateWithFlags(&d.hash, hipStreamNonBlocking));
  for (int s = 0; s < DeviceCtx::kTableSlots; ++s)
    HIP_TRY(p, hipEventCreateWithFlags(&d.tables_uploaded[s], hipEventDisableTiming));
  HIP_TRY(p, hipEventCreateWithFlags(&d.staging_idle, hipEventDisableTiming));
  for (int s = 0; s < 2; ++s) {
    HIP_TRY(p, hipEventCreateWithFlags(&d.slot_filled[s], hipEventDisableTiming));
    HIP_TRY(p, hipEventCreateWithFlags(&d.slot_drained[s], hipEventDisableTiming));
  }
  return MP_OK;
}

// Streams and events are created at the first call that needs the device, so that the
// control-plane calls work without a GPU.
int ensure_device(mp_pool *p) {
  DeviceCtx &d = p->dev;
  if (d.ready) return MP_OK;
  const int rc = create_device_objects(p);
  if (rc != MP_OK) {
    destroy_device_objects(d);  // nothing half-made is kept
    return rc;
  }
  d.ready = true;
  return MP_OK;
}

int reserve(mp_pool *p, MirrorBuf &b, size_t bytes, bool need_dev = true) {
  if (bytes <= b.cap) return MP_OK;
  size_t cap = b.cap ? b.cap : 4096;
  while (cap < bytes) cap *= 2;
  // earlier work may still read the old buffers
  HIP_TRY(p, hipStreamSynchronize(p->dev.stream));
  if (b.dev) HIP_TRY(p, hipFree(b.dev));
  if (b.host) HIP_TRY(p, hipHostFree(b.host));
  b.dev = b.host = nullptr;
  b.cap = 0;
  if (need_dev) HIP_TRY(p, hipMalloc(&b.dev, cap));
  HIP_TRY(p, hipHostMalloc(&b.host, cap, hipHostMallocDefault));
  b.cap = cap;
  return MP_OK;
}

void release(MirrorBuf &b) {
  if (b.dev) (void)hipFree(b.dev);
  if (b.host) (void)hipHostFree(b.host);
  b = MirrorBuf();
}

// ---- profiling ---------------------------------------------------------------------------
struct ProfScope {
  mp_pool *p;
  ProfRec rec;
  bool on;
  ProfScope(mp_pool *pool, int kind, uint64_t bytes) : p(pool), on(pool->dev.profiling) {
    if (!on) return;
    rec.kind = kind;
    rec.bytes = bytes;
    if (hipEventCreate(&rec.start) != hipSuccess || hipEventCreate(&rec.stop) != hipSuccess) {
      on = false;
      return;
    }
    (void)hipEventRecord(rec.start, p->dev.stream);
  }
  ~ProfScope() {
    if (!on) return;
    (void)hipEventRecord(rec.stop, p->dev.stream);
    p->dev.prof.push_back(rec);
  }
};

void prof_drain(mp_pool *p) {
  DeviceCtx &d = p->dev;
  for (ProfRec &r : d.prof) {
    float ms = 0.f;
    if (hipEventSynchronize(r.stop) == hipSuccess &&
        hipEventElapsedTime(&ms, r.start, r.stop) == hipSuccess) {
      d.prof_ms[r.kind] += ms;
      d.prof_launches[r.kind] += 1;
      d.prof_bytes[r.kind] += r.bytes;
    }
    (void)hipEventDestroy(r.start);
    (void)hipEventDestroy(r.stop);
  }
  d.prof.clear();
}

// ---- hashing through the device kernel ------------------------------------------------------
// Computes the chained hashes of n_req prompts into p->dev.hashes.host; blk_off_out receives
// the n_req+1 offsets into that array.  Host tokens are copied into pinned memory; device
// tokens are also copied back, because index nodes keep (and compare) their tokens.
// On return *host_tokens points at a host copy of all tokens.
// The completion words of one hash launch, for a caller that wants to use the hashes of the
// first prompts while the later ones are still being computed.  Whoever holds one must not
// return to the library's caller before everything has arrived: the destructor sees to that.
struct HashWait {
  mp_pool *p = nullptr;
  const volatile uint32_t *words = nullptr;  // null: nothing (or nothing any more) to wait for
  uint32_t mark = 0, n_req = 0, next = 0;    // prompts [0, next) have reported
  hipStream_t hs = nullptr;
  std::chrono::steady_clock::time_point give_up;
  // Returns once the hashes of prompts 0..r are in host memory.  A launch that has not
  // reported by `give_up` is waited for with a stream synchronisation instead.
  int upto(uint32_t r) {
    if (!words) return MP_OK;
    for (uint32_t spin = 0; next <= r; ++spin) {
      while (next < n_req && words[next] == mark) ++next;
      if (next > r) break;
      if ((spin & 1023u) == 1023u && std::chrono::steady_clock::now() > give_up) {
        words = nullptr;
        const hipError_t e = hipStreamSynchronize(hs);
        if (e == hipSuccess) return MP_OK;
        p->dev.hash_cache_valid = false;  // what the pinned buffers hold is not to be reused
        return fail_hip(p, e, "hipStreamSynchronize(hash stream)");
      }
      __builtin_ia32_pause();
    }
    std::atomic_thread_fence(std::memory_order_acquire);
    if (next == n_req) words = nullptr;
    return MP_OK;
  }
  HashWait() = default;
  HashWait(const HashWait &) = delete;
  HashWait &operator=(const HashWait &) = delete;
  ~HashWait() {
    if (words && n_req) (void)upto(n_req - 1);
  }
};

int mirror_sync(mp_pool *p);
int launch_probe(mp_pool *p, const uint32_t *k_tok, uint32_t n_req, const uint32_t *probe_off);

// With probe_off (n_req+1 output slot offsets) the index probe kernel runs right behind the
// hash kernel, before the one synchronisation; its results land in p->dev.m_out.
int device_hashes(mp_pool *p, const uint32_t *tokens, const uint32_t *tok_off, uint32_t n_req,
                  bool on_device, std::vector<uint32_t> &blk_off_out,
                  const uint32_t **host_tokens, const uint64_t **host_hashes,
                  const uint32_t *probe_off = nullptr, HashWait *defer = nullptr) {
  int rc = ensure_device(p);
  if (rc != MP_OK) return rc;
  DeviceCtx &d = p->dev;
  const uint32_t bs = p->desc.block_size;
  const uint32_t total_tok = tok_off[n_req];
  blk_off_out.assign(n_req + 1, 0);
  for (uint32_t r = 0; r < n_req; ++r)
    blk_off_out[r + 1] = blk_off_out[r] + (tok_off[r + 1] - tok_off[r]) / bs;
  const uint32_t total_blk = blk_off_out[n_req];
  if (d.hash_cache_valid && !on_device && d.hash_cache_n_req == n_req && total_blk &&
      std::memcmp(d.offsets.host, tok_off, 4ull * (n_req + 1)) == 0 &&
      std::memcmp(d.tokens.host, tokens, 4ull * total_tok) == 0) {
    *host_tokens = tokens;
    *host_hashes = (const uint64_t *)d.hashes.host;
    if (probe_off) {  // the hashes are remembered, the index may have changed: probe again
      if ((rc = launch_probe(p, (const uint32_t *)d.tokens.host, n_req, probe_off)) != MP_OK) return rc;
      HIP_TRY(p, hipStreamSynchronize(d.stream));
    }
    return MP_OK;
  }
  d.hash_cache_valid = false;
  if ((rc = reserve(p, d.tokens, std::max<size_t>(4, 4ull * total_tok), false)) != MP_OK) return rc;
  if ((rc = reserve(p, d.offsets, 8ull * (n_req + 1), false)) != MP_OK) return rc;
  if ((rc = reserve(p, d.hashes, std::max<size_t>(8, 8ull * total_blk), false)) != MP_OK) return rc;
  *host_tokens = on_device ? (const uint32_t *)d.tokens.host : tokens;
  *host_hashes = (const uint64_t *)d.hashes.host;
  if (total_blk == 0) return MP_OK;

  // Offsets, host tokens and the hashes live in pinned host memory that the kernel addresses
  // directly (zero-copy): a match costs one kernel launch and one wait for its completion
  // words, no copy-engine commands.  The volumes are tiny (4 B per token in, 8 B per block out).
  uint32_t *h_off = (uint32_t *)d.offsets.host;
  std::memcpy(h_off, tok_off, 4ull * (n_req + 1));
  std::memcpy(h_off + n_req + 1, blk_off_out.data(), 4ull * (n_req + 1));
  const uint32_t *k_tok;
  if (on_device) {
    k_tok = tokens;
    HIP_TRY(p, hipMemcpyAsync(d.tokens.host, tokens, 4ull * total_tok, hipMemcpyDeviceToHost,
                              d.stream));
  } else {
    std::memcpy(d.tokens.host, tokens, 4ull * total_tok);
    k_tok = (const uint32_t *)d.tokens.host;
  }
  // Without a probe kernel behind it, the launch is not waited for with a stream
  // synchronisation: every prompt's workgroup sets a word in pinned memory when its hashes are
  // out, and the host polls those words (a few us less per call).  If they do not all turn up
  // within a generous time the stream is synchronised after all.  Host-resident tokens are
  // then hashed on a stream of the library's own: the kernel reads and writes pinned host
  // memory only, so it has no business waiting behind block copies that earlier asynchronous
  // calls left on the pool's stream.  The host never returns to the library's caller before the
  // kernel has delivered (or the stream is synchronised), so that stream is idle between calls.
  // With `defer` the waiting is left to the caller of this function, prompt by prompt.
  const bool poll = !probe_off && !d.profiling;
  uint32_t *done = nullptr;
  if (poll) {
    if ((rc = reserve(p, d.hash_done, 4ull * n_req, false)) != MP_OK) return rc;
    done = (uint32_t *)d.hash_done.host;
    if (++d.hash_mark == 0) d.hash_mark = 1;
    std::memset(done, 0, 4ull * n_req);  // the mark is never 0: no stale or uninitialised word passes
  }
  const hipStream_t hs = (poll && !on_device) ? d.hash : d.stream;
  {
    ProfScope ps(p, kProfHash, 4ull * bs * total_blk + 8ull * total_blk);
    HIP_TRY(p, launch_block_hash(k_tok, h_off, h_off + n_req + 1, n_req, bs, p->desc.hash_seed,
                                 (uint64_t *)d.hashes.host, hs, done, d.hash_mark));
  }
  if (probe_off && (rc = launch_probe(p, k_tok, n_req, probe_off)) != MP_OK) return rc;
  // (device-resident tokens were also copied back on this stream in front of the kernel: in
  // stream order that copy is complete once the kernel has run)
  if (!poll) {
    HIP_TRY(p, hipStreamSynchronize(hs));
    d.hash_cache_valid = !on_device;
    d.hash_cache_n_req = n_req;
    return MP_OK;
  }
  // the remembered batch is consulted by later calls only, and none starts before the wait is over
  d.hash_cache_valid = !on_device;
  d.hash_cache_n_req = n_req;
  HashWait here;
  HashWait &w = defer ? *defer : here;
  w.p = p;
  w.words = done;
  w.mark = d.hash_mark;
  w.n_req = n_req;
  w.next = 0;
  w.hs = hs;
  w.give_up = std::chrono::steady_clock::now() + std::chrono::milliseconds(20);
  return defer ? MP_OK : w.upto(n_req - 1);
}

// ---- device-resident index copy ----------------------------------------------------------------
void free_mirror_arrays(DeviceCtx &d) {
  if (d.m_keys) (void)hipFree(d.m_keys);
  if (d.m_vals) (void)hipFree(d.m_vals);
  if (d.m_parent) (void)hipFree(d.m_parent);
  if (d.m_tokens) (void)hipFree(d.m_tokens);
  d.m_keys = nullptr;
  d.m_vals = nullptr;
  d.m_parent = nullptr;
  d.m_tokens = nullptr;
}

int mirror_enable(mp_pool *p) {
  int rc = ensure_device(p);
  if (rc != MP_OK) return rc;
  DeviceCtx &d = p->dev;
  if (d.mirror_on) return MP_OK;
  const HashTable &t = p->idx.table();
  const uint32_t nb = p->desc.n_blocks, bs = p->desc.block_size;
  d.mirror_cap = t.capacity();
  if (d.mirror_cap > 0x80000000ull) return fail(p, MP_EINVAL, "pool too large for the device index copy");
  hipError_t e = hipMalloc((void **)&d.m_keys, 8ull * d.mirror_cap);
  if (e == hipSuccess) e = hipMalloc((void **)&d.m_vals, 4ull * d.mirror_cap);
  if (e == hipSuccess) e = hipMalloc((void **)&d.m_parent, 4ull * nb);
  if (e == hipSuccess) e = hipMalloc((void **)&d.m_tokens, 4ull * nb * bs);
  // first copy: everything, synchronously
  if (e == hipSuccess) e = hipMemcpy(d.m_keys, t.keys(), 8ull * d.mirror_cap, hipMemcpyHostToDevice);
  if (e == hipSuccess) e = hipMemcpy(d.m_vals, t.vals(), 4ull * d.mirror_cap, hipMemcpyHostToDevice);
  if (e == hipSuccess) e = hipMemcpy(d.m_parent, p->idx.parents(), 4ull * nb, hipMemcpyHostToDevice);
  if (e == hipSuccess)
    e = hipMemcpy(d.m_tokens, p->idx.node_tokens(), 4ull * nb * bs, hipMemcpyHostToDevice);
  if (e != hipSuccess) {
    free_mirror_arrays(d);
    return fail_hip(p, e, "device index copy");
  }
  p->idx.enable_mirror_log(true);
  d.mirror_on = true;
  return MP_OK;
}

void mirror_disable(mp_pool *p) {
  DeviceCtx &d = p->dev;
  if (!d.mirror_on) return;
  (void)hipStreamSynchronize(d.stream);
  p->idx.enable_mirror_log(false);
  free_mirror_arrays(d);
  d.mirror_on = false;
}

// Brings the device copy up to date: the changed slots and nodes are written, with their
// CURRENT host values, into pinned records that a small kernel scatters into HBM.
int mirror_sync(mp_pool *p) {
  DeviceCtx &d = p->dev;
  std::vector<uint32_t> &slots = p->idx.dirty_slots();
  std::vector<int32_t> &nodes = p->idx.dirty_nodes();
  if (slots.empty() && nodes.empty()) return MP_OK;
  const uint32_t bs = p->desc.block_size;
  const HashTable &t = p->idx.table();
  const size_t slot_dwords = 4ull * slots.size(), node_dwords = (size_t)(2 + bs) * nodes.size();
  int rc = reserve(p, d.m_updates, 4ull * (slot_dwords + node_dwords), false);
  if (rc != MP_OK) return rc;
  uint32_t *u = (uint32_t *)d.m_updates.host;
  for (size_t i = 0; i < slots.size(); ++i) {
    const uint64_t k = t.key_at(slots[i]);
    u[4 * i + 0] = slots[i];
    u[4 * i + 1] = (uint32_t)t.val_at(slots[i]);
    u[4 * i + 2] = (uint32_t)k;
    u[4 * i + 3] = (uint32_t)(k >> 32);
  }
  uint32_t *nu = u + slot_dwords;
  for (size_t i = 0; i < nodes.size(); ++i) {
    uint32_t *r = nu + (size_t)(2 + bs) * i;
    r[0] = (uint32_t)nodes[i];
    r[1] = (uint32_t)p->idx.parents()[nodes[i]];
    std::memcpy(r + 2, p->idx.node_tokens() + (size_t)nodes[i] * bs, 4ull * bs);
  }
  HIP_TRY(p, launch_index_apply(u, (uint32_t)slots.size(), nu, (uint32_t)nodes.size(), bs, d.m_keys,
                                d.m_vals, d.m_parent, d.m_tokens, d.stream));
  slots.clear();
  nodes.clear();
  return MP_OK;
}

// Enqueues change replay + probe.  m_out layout (pinned): [n_req+1 slot offsets][n_req matched
// counts][ids, probe_off[n_req] of them].
int launch_probe(mp_pool *p, const uint32_t *k_tok, uint32_t n_req, const uint32_t *probe_off) {
  DeviceCtx &d = p->dev;
  int rc = mirror_sync(p);
  if (rc != MP_OK) return rc;
  const size_t head = 2ull * n_req + 1;
  if ((rc = reserve(p, d.m_out, 4ull * (head + probe_off[n_req]) + 4, false)) != MP_OK) return rc;
  uint32_t *o = (uint32_t *)d.m_out.host;
  std::memcpy(o, probe_off, 4ull * (n_req + 1));
  const uint32_t *h_off = (const uint32_t *)d.offsets.host;
  HIP_TRY(p, launch_index_probe(k_tok, h_off, h_off + n_req + 1, (const uint64_t *)d.hashes.host, o,
                                n_req, p->desc.block_size, d.m_keys, d.m_vals, d.m_parent,
                                d.m_tokens, d.mirror_cap, (int32_t *)(o + head),
                                o + n_req + 1, d.stream));
  return MP_OK;
}

// ---- block-table upload -----------------------------------------------------------------------
// Orders the table pair by one side's ids (results do not depend on the order of the entries;
// destination ids are distinct).  Keys are (id << 32 | other id); small tables use std::sort,
// large ones an LSD radix sort over the id bits, so the cost stays a few ns per entry.
void sort_pairs(std::vector<uint64_t> &a, std::vector<uint64_t> &b, const int32_t *key_ids,
                const int32_t *other_ids, uint32_t n, uint32_t key_range, int32_t *key_out,
                int32_t *other_out) {
  a.resize(n);
  for (uint32_t i = 0; i < n; ++i)
    a[i] = ((uint64_t)(uint32_t)key_ids[i] << 32) | (uint32_t)other_ids[i];
  if (n <= 512) {
    std::sort(a.begin(), a.end());
  } else {
    b.resize(n);
    uint32_t bits = 1;
    while (bits < 32 && (1ull << bits) < key_range) ++bits;
    for (uint32_t shift = 32; shift < 32 + bits; shift += 11) {
      uint32_t count[2049] = {0};
      for (uint32_t i = 0; i < n; ++i) ++count[((a[i] >> shift) & 2047u) + 1];
      for (uint32_t d = 0; d < 2048; ++d) count[d + 1] += count[d];
      for (uint32_t i = 0; i < n; ++i) b[count[(a[i] >> shift) & 2047u]++] = a[i];
      a.swap(b);
    }
  }
  for (uint32_t i = 0; i < n; ++i) {
    key_out[i] = (int32_t)(uint32_t)(a[i] >> 32);
    other_out[i] = (int32_t)(uint32_t)a[i];
  }
}

// Puts [src ids][dst ids] on the device of `x` (either may be null); device pointers come back,
// and host pointers to the same arrays as they were uploaded.  sort_by: -1 keeps the caller's
// order (the staging order of mp_gather / mp_scatter is part of their contract); 0 / 1 sorts
// the pair by source / destination id first (both tables must be given).
int upload_tables(mp_pool *x, const int32_t *src_ids, const int32_t *dst_ids, uint32_t n,
                  const int32_t **d_src, const int32_t **d_dst, int sort_by = -1,
                  uint32_t key_range = 0, const int32_t **h_src = nullptr,
                  const int32_t **h_dst = nullptr) {
  DeviceCtx &d = x->dev;
  if (!src_ids || !dst_ids || n < 2) sort_by = -1;
  auto hand_out = [&](int slot) {
    const int32_t *h = (const int32_t *)d.tables[slot].host;
    *d_src = (const int32_t *)d.tables[slot].dev;
    *d_dst = (const int32_t *)d.tables[slot].dev + n;
    if (h_src) *h_src = h;
    if (h_dst) *h_dst = h + n;
  };
  // same pair as last time (every layer of a by-layer transfer): nothing to sort or send
  if (d.tables_last >= 0 && d.last_n == n && d.last_has_src == (src_ids != nullptr) &&
      d.last_has_dst == (dst_ids != nullptr) && d.last_sort_by == sort_by &&
      (!src_ids || std::memcmp(d.last_ids.data(), src_ids, 4ull * n) == 0) &&
      (!dst_ids || std::memcmp(d.last_ids.data() + n, dst_ids, 4ull * n) == 0)) {
    hand_out(d.tables_last);
    return MP_OK;
  }
  const int slot = d.tables_next;
  d.tables_next = (slot + 1) % DeviceCtx::kTableSlots;
  if (d.tables_last == slot) d.tables_last = -1;
  if (d.tables_pending[slot]) {  // an earlier asynchronous call may still be reading this pinned copy
    HIP_TRY(x, hipEventSynchronize(d.tables_uploaded[slot]));
    d.tables_pending[slot] = false;
  }
  int rc = reserve(x, d.tables[slot], std::max<size_t>(8, 8ull * n));
  if (rc != MP_OK) return rc;
  int32_t *h = (int32_t *)d.tables[slot].host;
  if (sort_by == 0) sort_pairs(x->sort_a, x->sort_b, src_ids, dst_ids, n, key_range, h, h + n);
  else if (sort_by == 1) sort_pairs(x->sort_a, x->sort_b, dst_ids, src_ids, n, key_range, h + n, h);
  else {
    if (src_ids) std::memcpy(h, src_ids, 4ull * n);
    if (dst_ids) std::memcpy(h + n, dst_ids, 4ull * n);
  }
  HIP_TRY(x, hipMemcpyAsync(d.tables[slot].dev, h, 8ull * n, hipMemcpyHostToDevice, d.stream));
  HIP_TRY(x, hipEventRecord(d.tables_uploaded[slot], d.stream));
  d.tables_pending[slot] = true;
  d.last_ids.resize(2ull * n);  // the caller's own arrays: what the next call is compared with
  if (src_ids) std::memcpy(d.last_ids.data(), src_ids, 4ull * n);
  if (dst_ids) std::memcpy(d.last_ids.data() + n, dst_ids, 4ull * n);
  d.last_n = n;
  d.last_has_src = src_ids != nullptr;
  d.last_has_dst = dst_ids != nullptr;
  d.last_sort_by = sort_by;
  d.tables_last = slot;
  hand_out(slot);
  return MP_OK;
}

// `l0` = first layer addressed (by-layer transfers start in the middle of a block's planes).
CopySide pool_side(const mp_pool *p, const int32_t *d_tbl, uint32_t l0 = 0, bool ascending = false) {
  CopySide s;
  s.tbl = d_tbl;
  s.ascending = ascending;
  if (!aggregated(p)) {  // discrete layout [L][2][NB][F]
    s.plane_stride = (uint64_t)p->desc.n_blocks * p->F;
    s.block_stride = p->F;
  } else {  // aggregated layout [NB][L][2][F]
    s.plane_stride = p->F;
    s.block_stride = p->B;
  }
  s.base = (uint8_t *)p->desc.base + 2ull * l0 * s.plane_stride;
  return s;
}

// Records of `planes` fragments each, packed back to back (planes = 2*L for whole blocks).
CopySide record_side(const mp_pool *p, void *base, uint32_t planes) {
  CopySide s;
  s.base = base;
  s.tbl = nullptr;
  s.plane_stride = p->F;
  s.block_stride = (uint64_t)planes * p->F;
  return s;
}

bool tables_overlap(mp_pool *p, const int32_t *a, const int32_t *b, uint32_t n) {
  return p->idx.lists_overlap(a, b, n);
}

// Which staging problems would the copy hit?  Checked before any state changes.
int check_copy_feasible(mp_pool *src, mp_pool *dst, uint32_t n, uint32_t flags,
                        uint32_t n_layers = 0 /* 0 = all */) {
  const bool s_hbm = src->desc.tier == MP_TIER_HBM, d_hbm = dst->desc.tier == MP_TIER_HBM;
  if (!s_hbm && !d_hbm) return fail(src, MP_ESHAPE, "host-to-host transfers are not supported");
  if (flags & (MP_DIRECT | MP_PER_FRAGMENT)) return MP_OK;  // no staging involved
  if (n_layers && (!s_hbm || !d_hbm))
    return fail(src, MP_ESHAPE, "a by-layer transfer with a host-tier pool needs MP_DIRECT");
  if (n == 0) return MP_OK;
  mp_pool *x = s_hbm ? src : dst;
  const uint64_t rec = n_layers ? 2ull * n_layers * x->F : x->B;
  if (!x->desc.staging || x->desc.staging_bytes < rec)
    return fail(src, MP_ENOSTAGING, "staging buffer missing or smaller than one record");
  return MP_OK;
}

// The transmission step.  All ids are already validated.  Enqueues on the executing pool's
// stream; the caller synchronises if it must.
// Layers [l0, l1) of every block are moved (l1 = 0 means all layers).
int run_copy(mp_pool *src, mp_pool *dst, const int32_t *src_ids, const int32_t *dst_ids,
             uint32_t n, uint32_t flags, uint32_t l0 = 0, uint32_t l1 = 0) {
  if (n == 0) return MP_OK;
  if (l1 == 0) l1 = src->desc.n_layers;
  const uint32_t planes = 2 * (l1 - l0);
  const bool s_hbm = src->desc.tier == MP_TIER_HBM, d_hbm = dst->desc.tier == MP_TIER_HBM;
  mp_pool *x = s_hbm ? src : dst;  // the pool whose device context executes
  int rc = ensure_device(x);
  if (rc != MP_OK) return rc;
  DeviceCtx &d = x->dev;
  const CopyTune tune = x->tune;
  const uint64_t B = (uint64_t)planes * x->F;  // bytes moved per table entry
  const int32_t *d_src = nullptr, *d_dst = nullptr;
  const bool direct = (flags & MP_DIRECT) != 0;
  bool dst_ascends = false;

  // A transfer of one request (a few dozen blocks) between HBM pools: the ids, sorted by
  // destination, travel in the kernel arguments -- no table upload, no event, one launch
  // (fused) or two (through one staging round).
  if (!(flags & MP_PER_FRAGMENT) && s_hbm && d_hbm && small_copy_possible(n, planes, x->F, tune) &&
      (direct || (uint64_t)n * B <= x->desc.staging_bytes)) {
    uint64_t keys[kSmallTable];
    for (uint32_t i = 0; i < n; ++i)
      keys[i] = ((uint64_t)(uint32_t)dst_ids[i] << 32) | (uint32_t)src_ids[i];
    std::sort(keys, keys + n);
    SmallTables ids;
    for (uint32_t i = 0; i < n; ++i) {
      ids.dst[i] = (int32_t)(uint32_t)(keys[i] >> 32);
      ids.src[i] = (int32_t)(uint32_t)keys[i];
    }
    const CopySide from = pool_side(src, nullptr, l0), to = pool_side(dst, nullptr, l0, true);
    if (direct) {
      ProfScope ps(x, kProfDirect, 2ull * n * B);
      HIP_TRY(x, launch_block_copy_small(from, to, ids, true, true, n, planes, x->F, tune, d.n_cus,
                                         d.stream));
      return MP_OK;
    }
    const CopySide records = record_side(x, x->desc.staging, planes);
    {
      ProfScope ps(x, kProfGather, 2ull * n * B);
      HIP_TRY(x, launch_block_copy_small(from, records, ids, true, false, n, planes, x->F, tune,
                                         d.n_cus, d.stream));
    }
    {
      ProfScope ps(x, kProfScatter, 2ull * n * B);
      HIP_TRY(x, launch_block_copy_small(records, to, ids, false, true, n, planes, x->F, tune,
                                         d.n_cus, d.stream));
    }
    return MP_OK;
  }

  if (!(flags & MP_PER_FRAGMENT)) {
    // The pair of tables is sorted before it goes up (the result does not depend on the order
    // of the entries): by destination id, so that the stores of a launch sweep each plane of
    // the destination pool upwards -- the write pattern HBM takes at copy speed --; or, when the
    // copy engine moves the records of a host pool, by that pool's ids, so that runs of
    // consecutive ids merge into single copies.
    const int sort_by = (!direct && !s_hbm) ? 0 : 1;
    const int32_t *h_src = src_ids, *h_dst = dst_ids;
    rc = upload_tables(x, src_ids, dst_ids, n, &d_src, &d_dst, sort_by,
                       sort_by ? dst->desc.n_blocks : src->desc.n_blocks, &h_src, &h_dst);
    if (rc != MP_OK) return rc;
    src_ids = h_src;  // from here on: the order the device tables (and staging) have
    dst_ids = h_dst;
    dst_ascends = sort_by == 1;
  }

  if (flags & MP_PER_FRAGMENT) {
    // Reference point, not a product path: one copy-engine call per discrete fragment, the way
    // a per-block network API moves a paged KV cache (paper sections 5.2 and 7).
    for (uint32_t i = 0; i < n; ++i)
      for (uint32_t pl = 0; pl < planes; ++pl) {
        const CopySide s = pool_side(src, nullptr, l0), t = pool_side(dst, nullptr, l0);
        const uint8_t *from = (const uint8_t *)s.base + pl * s.plane_stride +
                              (uint64_t)src_ids[i] * s.block_stride;
        uint8_t *to = (uint8_t *)t.base + pl * t.plane_stride + (uint64_t)dst_ids[i] * t.block_stride;
        HIP_TRY(x, hipMemcpyAsync(to, from, x->F, hipMemcpyDefault, d.stream));
      }
    return MP_OK;
  }

  if (direct) {
    // One fused kernel, fragment to fragment.  With a pinned-host pool at one end the kernel
    // reads or writes host memory through the host link itself (zero-copy): no staging write,
    // no copy-engine hop.
    ProfScope ps(x, kProfDirect, 2ull * n * B);
    HIP_TRY(x, launch_block_copy(pool_side(src, d_src, l0), pool_side(dst, d_dst, l0, dst_ascends), n,
                                 planes, x->F, tune, d.n_cus, d.stream));
    return MP_OK;
  }

  uint8_t *staging = (uint8_t *)x->desc.staging;
  if (s_hbm && d_hbm) {  // gather into records, scatter out of them, staging-sized rounds
    const uint32_t cap = (uint32_t)std::min<uint64_t>(x->desc.staging_bytes / B, 0xffffffffu);
    for (uint32_t first = 0; first < n; first += cap) {
      const uint32_t cnt = std::min(cap, n - first);
      {
        ProfScope ps(x, kProfGather, 2ull * cnt * B);
        HIP_TRY(x, launch_block_copy(pool_side(src, d_src + first, l0),
                                     record_side(x, staging, planes), cnt, planes, x->F, tune,
                                     d.n_cus, d.stream));
      }
      {
        ProfScope ps(x, kProfScatter, 2ull * cnt * B);
        HIP_TRY(x, launch_block_copy(record_side(x, staging, planes),
                                     pool_side(dst, d_dst + first, l0, dst_ascends), cnt, planes,
                                     x->F, tune, d.n_cus, d.stream));
      }
    }
    return MP_OK;
  }

  // One end is the pinned-host tier (aggregated layout: a block is one contiguous record).
  // Two staging slots let the kernel of round k+1 overlap the host-link copies of round k.
  //
  // Who may touch staging, and when.  Kernels read and write it on the main stream only; the
  // copy engine reads (HBM -> host) or writes (host -> HBM) it on the side stream only.  The
  // main stream is the single line of order between calls: a host-tier call starts by making
  // the side stream wait for everything enqueued on the main stream so far (earlier
  // asynchronous gathers, scatters and HBM -> HBM rounds may still be using any part of the
  // buffer, whatever slot layout they had), and it ends with the main stream ordered behind
  // every side-stream copy it issued.  In between, a slot goes back and forth with one event
  // per direction, and a slot is reused only after the event of its previous round.
  uint32_t n_slots = 2;
  uint64_t slot_bytes = (x->desc.staging_bytes / 2) / B * B;
  if (slot_bytes == 0 || (uint64_t)n * B <= x->desc.staging_bytes / B * B) {
    n_slots = 1;
    slot_bytes = x->desc.staging_bytes / B * B;
  }
  const uint32_t cap = (uint32_t)std::min<uint64_t>(slot_bytes / B, 0xffffffffu);
  uint8_t *host_base = (uint8_t *)(s_hbm ? dst : src)->desc.base;
  const int32_t *host_ids = s_hbm ? dst_ids : src_ids;
  HIP_TRY(x, hipEventRecord(d.staging_idle, d.stream));
  HIP_TRY(x, hipStreamWaitEvent(d.side, d.staging_idle, 0));
  bool slot_used[2] = {false, false};  // in this call: its `drained` event is pending
  uint32_t round = 0;
  for (uint32_t first = 0; first < n; first += cap, ++round) {
    const uint32_t cnt = std::min(cap, n - first);
    const uint32_t s = round % n_slots;
    uint8_t *slot = staging + (uint64_t)s * slot_bytes;
    if (s_hbm) {  // HBM -> host: gather on the main stream, then device-to-host on the side stream
      if (slot_used[s]) HIP_TRY(x, hipStreamWaitEvent(d.stream, d.slot_drained[s], 0));
      {
        ProfScope ps(x, kProfGather, 2ull * cnt * B);
        HIP_TRY(x, launch_block_copy(pool_side(src, d_src + first), record_side(x, slot, x->P), cnt,
                                     x->P, x->F, tune, d.n_cus, d.stream));
      }
      HIP_TRY(x, hipEventRecord(d.slot_filled[s], d.stream));
      HIP_TRY(x, hipStreamWaitEvent(d.side, d.slot_filled[s], 0));
    } else {  // host -> HBM: wait until the scatter that last read this slot is done
      if (slot_used[s]) HIP_TRY(x, hipStreamWaitEvent(d.side, d.slot_drained[s], 0));
    }
    for (uint32_t i = 0; i < cnt;) {  // one copy per run of consecutive host block ids
      uint32_t j = i + 1;
      while (j < cnt && host_ids[first + j] == host_ids[first + j - 1] + 1) ++j;
      uint8_t *h = host_base + (uint64_t)host_ids[first + i] * B;
      uint8_t *g = slot + (uint64_t)i * B;
      if (s_hbm)
        HIP_TRY(x, hipMemcpyAsync(h, g, (uint64_t)(j - i) * B, hipMemcpyDeviceToHost, d.side));
      else
        HIP_TRY(x, hipMemcpyAsync(g, h, (uint64_t)(j - i) * B, hipMemcpyHostToDevice, d.side));
      i = j;
    }
    if (s_hbm) {
      HIP_TRY(x, hipEventRecord(d.slot_drained[s], d.side));
    } else {
      HIP_TRY(x, hipEventRecord(d.slot_filled[s], d.side));
      HIP_TRY(x, hipStreamWaitEvent(d.stream, d.slot_filled[s], 0));
      {
        ProfScope ps(x, kProfScatter, 2ull * cnt * B);
        HIP_TRY(x, launch_block_copy(record_side(x, slot, x->P), pool_side(dst, d_dst + first), cnt,
                                     x->P, x->F, tune, d.n_cus, d.stream));
      }
      HIP_TRY(x, hipEventRecord(d.slot_drained[s], d.stream));
    }
    slot_used[s] = true;
  }
  if (s_hbm) {  // the main stream becomes the single point of completion
    for (uint32_t s = 0; s < n_slots; ++s)
      if (slot_used[s]) HIP_TRY(x, hipStreamWaitEvent(d.stream, d.slot_drained[s], 0));
  }
  return MP_OK;
}

int finish_copy(mp_pool *src, mp_pool *dst, uint32_t flags) {
  if (flags & MP_ASYNC) return MP_OK;
  mp_pool *x = src->desc.tier == MP_TIER_HBM ? src : dst;
  if (!x->dev.ready) return MP_OK;
  HIP_TRY(x, hipStreamSynchronize(x->dev.stream));
  return MP_OK;
}

// A transfer inside one pool with an explicit destination list may read and write the same
// blocks.  The staged path is defined as "gather everything, then scatter", which holds only
// if the whole table fits one staging round; the fused path cannot honour it at all.
// (Freshly allocated destination ids never overlap the sources: the sources are held while
// the destination blocks are allocated.)
int check_same_pool(mp_pool *src, mp_pool *dst, const int32_t *src_ids, const int32_t *dst_ids,
                    uint32_t n, uint32_t flags) {
  if (src != dst || !(flags & MP_DST_GIVEN) || n == 0) return MP_OK;
  if (!tables_overlap(src, src_ids, dst_ids, n)) return MP_OK;
  if (flags & MP_DIRECT)
    return fail(src, MP_EINVAL, "MP_DIRECT within one pool needs disjoint tables");
  if ((uint64_t)n * src->B > src->desc.staging_bytes)
    return fail(src, MP_ENOSTAGING, "overlapping in-pool transfer must fit the staging buffer");
  return MP_OK;
}

// The sources of a transfer inside one pool are read after the allocation step, so they are
// held (one reference each) while destination blocks are found: on-demand eviction then cannot
// take a historical source block and hand it back as its own destination.
void hold_sources(mp_pool *src, mp_pool *dst, const int32_t *ids, uint32_t n, bool hold) {
  if (src != dst) return;
  for (uint32_t i = 0; i < n; ++i) {
    if (hold) src->idx.pin(ids[i]);
    else src->idx.unpin(ids[i]);
  }
}

int check_src_ids(mp_pool *src, const int32_t *ids, uint32_t n) {
  for (uint32_t i = 0; i < n; ++i)
    if (!src->idx.in_range(ids[i]) || src->idx.is_free(ids[i]))
      return fail(src, MP_EINVAL, "source block id out of range or free");
  return MP_OK;
}

// host part of match on precomputed hashes
void match_walk(mp_pool *p, const uint32_t *tokens, const uint64_t *hashes, uint32_t nblk,
                int32_t *blocks_out, uint32_t *n_matched, uint32_t flags) {
  p->idx.tick();
  uint32_t m = p->idx.walk(tokens, hashes, nblk, blocks_out);
  p->idx.touch(blocks_out, m);
  if (flags & MP_MATCH_PIN)
    for (uint32_t i = 0; i < m; ++i) p->idx.pin(blocks_out[i]);
  *n_matched = m;
}

// Shared core of transfer_with_insert and its batched form.
int twi_core(mp_pool *src, mp_pool *dst, const uint32_t *tokens, const uint32_t *tok_off,
             uint32_t n_req, const uint32_t *first_block, const int32_t *src_blocks,
             int32_t *dst_blocks, const uint32_t *blk_off, uint32_t flags, const void *priv,
             uint64_t priv_len) {
  if (!src || !dst) return MP_EINVAL;
  if (!tok_off || !blk_off || (!first_block && n_req))
    return fail(src, MP_EINVAL, "null offset / first_block array");
  if (!same_geometry(src, dst)) return fail(src, MP_ESHAPE, "source and destination geometry differ");
  if (blk_off[0] != 0 || tok_off[0] != 0) return fail(src, MP_EINVAL, "offsets must start at 0");
  const uint32_t bs = dst->desc.block_size;
  for (uint32_t r = 0; r < n_req; ++r) {
    if (tok_off[r + 1] < tok_off[r] || blk_off[r + 1] < blk_off[r])
      return fail(src, MP_EINVAL, "offsets must be non-decreasing");
    const uint32_t nb = (tok_off[r + 1] - tok_off[r]) / bs, n = blk_off[r + 1] - blk_off[r];
    if (first_block[r] > nb || (uint64_t)first_block[r] + n < nb)
      return fail(src, MP_EINVAL, "first_block / table length inconsistent with the prompt");
  }
  const uint32_t total = blk_off[n_req];
  if ((!src_blocks || !dst_blocks) && total) return fail(src, MP_EINVAL, "null block table");
  if (!tokens && tok_off[n_req]) return fail(src, MP_EINVAL, "null tokens");
  int rc = check_src_ids(src, src_blocks, total);
  if (rc != MP_OK) return rc;
  if ((flags & MP_DST_GIVEN) && !dst->idx.held_and_distinct(dst_blocks, total))
    return fail(src, MP_EINVAL, "given destination ids must be held and distinct");
  if ((rc = check_copy_feasible(src, dst, total, flags)) != MP_OK) return rc;
  if ((rc = check_same_pool(src, dst, src_blocks, dst_blocks, total, flags)) != MP_OK) return rc;

  // the receiver hashes the prompts (device kernel)
  std::vector<uint32_t> &hoff = dst->twi_hoff;  // pool-owned scratch: no allocation per call
  const uint32_t *htok = nullptr;
  const uint64_t *hh = nullptr;
  rc = device_hashes(dst, tokens, tok_off, n_req, (flags & MP_TOKENS_ON_DEVICE) != 0, hoff, &htok,
                     &hh);
  if (rc != MP_OK) return rc;

  // blocks [0, first_block) must already be indexed at the receiver.  ids of request r:
  // ids[ids_off[r] ..), one per prompt block (and per table entry beyond the full blocks)
  std::vector<int32_t> &ids = dst->twi_ids;
  std::vector<uint32_t> &ids_off = dst->twi_ids_off, &present = dst->twi_present;
  ids_off.resize(n_req + 1);
  present.resize(n_req);
  ids_off[0] = 0;
  for (uint32_t r = 0; r < n_req; ++r) {
    const uint32_t nb = hoff[r + 1] - hoff[r], n = blk_off[r + 1] - blk_off[r];
    ids_off[r + 1] = ids_off[r] + std::max(nb, first_block[r] + n);
  }
  ids.assign(ids_off[n_req], kNoBlock);
  for (uint32_t r = 0; r < n_req; ++r) {
    present[r] = dst->idx.walk(htok + tok_off[r], hh + hoff[r], hoff[r + 1] - hoff[r],
                               ids.data() + ids_off[r]);
    if (present[r] < first_block[r])
      return fail(src, MP_ESTALE, "claimed prefix is not in the destination index");
  }
  if (flags & MP_DST_GIVEN) {
    if (n_req != 1) return fail(src, MP_EINVAL, "MP_DST_GIVEN is not supported in batched form");
    for (uint32_t i = 0; i < total; ++i) ids[first_block[0] + i] = dst_blocks[i];
    if (!dst->idx.adoptable(ids.data(), present[0], hoff[1]))
      return fail(src, MP_EINVAL, "a given destination block is already indexed");
  }
  // allocation step, with the matched prefixes protected from on-demand eviction
  for (uint32_t r = 0; r < n_req; ++r)
    for (uint32_t i = 0; i < first_block[r]; ++i) dst->idx.pin(ids[ids_off[r] + i]);
  auto unpin_all = [&]() {
    for (uint32_t r = 0; r < n_req; ++r)
      for (uint32_t i = 0; i < first_block[r]; ++i) dst->idx.unpin(ids[ids_off[r] + i]);
  };
  if (!(flags & MP_DST_GIVEN)) {
    hold_sources(src, dst, src_blocks, total, true);
    const bool got = dst->idx.alloc(total, dst_blocks, (flags & MP_EVICT_ON_DEMAND) != 0);
    hold_sources(src, dst, src_blocks, total, false);
    if (!got) {
      unpin_all();
      return fail(src, MP_ENOMEM, "destination pool cannot supply the blocks");
    }
    for (uint32_t r = 0; r < n_req; ++r)
      for (uint32_t i = 0; i < blk_off[r + 1] - blk_off[r]; ++i)
        ids[ids_off[r] + first_block[r] + i] = dst_blocks[blk_off[r] + i];
  }

  // transmission step
  rc = run_copy(src, dst, src_blocks, dst_blocks, total, flags);
  if (rc == MP_OK) rc = finish_copy(src, dst, flags);
  if (rc != MP_OK) {  // a HIP failure: hand the fresh destination blocks back
    unpin_all();
    if (!(flags & MP_DST_GIVEN)) (void)dst->idx.release(dst_blocks, total);
    return rc;
  }

  // insertion step: only after all data is in place (or ordered behind it on the stream)
  for (uint32_t r = 0; r < n_req; ++r)
    dst->idx.insert(htok + tok_off[r], hh + hoff[r], hoff[r + 1] - hoff[r], ids.data() + ids_off[r]);
  unpin_all();
  if (dst->cb) dst->cb(dst->cb_user, priv, priv_len, dst_blocks, total);
  return MP_OK;
}

// ---- swap between the two tiers of one instance ------------------------------------------------
// Both directions cache a prompt prefix that one pool holds in the other pool.  The index work
// is done call by call in the defined order; the copies are collected and share launches.
struct TierMove {
  TierMove(mp_pool *f, mp_pool *t, uint32_t fl)
      : from(f), to(t), flags(fl), known(f->desc.n_blocks, kNoBlock) {}
  mp_pool *from, *to;
  uint32_t flags;
  // for the rest of the call: block of `to` that caches the same prefix block as block b of
  // `from` (set for every block on a prefix that has been handled)
  std::vector<int32_t> known;
  std::vector<int32_t> src, dst;  // pending copies: block src[i] of `from` -> block dst[i] of `to`
  std::vector<uint32_t> tokens;
  std::vector<uint64_t> hashes;
  std::vector<int32_t> path, ids, fresh;
};

int tier_pair_ok(mp_pool *a, mp_pool *b) {
  if (!a || !b || a == b) return fail(a, MP_EINVAL, "swap needs two different pools");
  if (!same_geometry(a, b)) return fail(a, MP_ESHAPE, "the two tiers differ in geometry");
  if (a->desc.tier != MP_TIER_HBM && b->desc.tier != MP_TIER_HBM)
    return fail(a, MP_ESHAPE, "host-to-host transfers are not supported");
  if (a->desc.hash_seed != b->desc.hash_seed)
    return fail(a, MP_EINVAL, "the two tiers of one instance must share hash_seed");
  return MP_OK;
}

int flush_moves(TierMove &mv) {
  if (mv.src.empty()) return MP_OK;
  const int rc = run_copy(mv.from, mv.to, mv.src.data(), mv.dst.data(), (uint32_t)mv.src.size(),
                          mv.flags & MP_DIRECT);
  mv.src.clear();
  mv.dst.clear();
  return rc;
}

// Makes `to` cache the prefix that ends in block `leaf` of `from`: the index part of
// transfer_with_insert(from -> to, prefix, first_block = what `to` already has,
// MP_EVICT_ON_DEMAND) followed by a release of the new blocks; the copies are only queued.
// The chained hashes are the ones `from` keeps in its nodes (same seed, same prefix).
// *last_out = the block of `to` that caches the prefix's last block, referenced once if
// `keep_last`.  MP_ENOMEM changes nothing.
int cache_prefix(TierMove &mv, int32_t leaf, bool keep_last, int32_t *last_out) {
  PoolIndex &fi = mv.from->idx, &ti = mv.to->idx;
  const uint32_t bs = mv.to->desc.block_size;
  fi.path_to(leaf, mv.path);
  const uint32_t d = (uint32_t)mv.path.size();
  mv.tokens.resize((size_t)d * bs);
  mv.hashes.resize(d);
  for (uint32_t i = 0; i < d; ++i) {
    std::memcpy(&mv.tokens[(size_t)i * bs], fi.tokens_of(mv.path[i]), 4ull * bs);
    mv.hashes[i] = fi.hash_of(mv.path[i]);
  }
  mv.ids.assign(d, kNoBlock);
  const uint32_t m = ti.walk(mv.tokens.data(), mv.hashes.data(), d, mv.ids.data());
  const uint32_t need = d - m;
  mv.fresh.resize(need);
  if (need > ti.n_free()) {
    // eviction may hand out a block that a queued copy still targets: run the queue first
    const int rc = flush_moves(mv);
    if (rc != MP_OK) return rc;
  }
  for (uint32_t i = 0; i < m; ++i) ti.pin(mv.ids[i]);
  const bool ok = ti.alloc(need, mv.fresh.data(), true);
  for (uint32_t i = 0; i < m; ++i) ti.unpin(mv.ids[i]);
  if (!ok) return fail(mv.from, MP_ENOMEM, "the other tier cannot supply the blocks");
  for (uint32_t i = 0; i < need; ++i) mv.ids[m + i] = mv.fresh[i];
  ti.insert(mv.tokens.data(), mv.hashes.data(), d, mv.ids.data());
  if (keep_last && d) ti.pin(mv.ids[d - 1]);
  (void)ti.release(mv.fresh.data(), need);
  for (uint32_t i = 0; i < need; ++i)
    if (!ti.is_free(mv.fresh[i])) {  // (a 64-bit hash collision would leave a block un-indexed)
      mv.src.push_back(mv.path[m + i]);
      mv.dst.push_back(mv.fresh[i]);
    }
  for (uint32_t i = 0; i < d; ++i)
    if (ti.indexed(mv.ids[i]) || (keep_last && i + 1 == d)) mv.known[mv.path[i]] = mv.ids[i];
  if (last_out) *last_out = d ? mv.ids[d - 1] : kNoBlock;
  // start moving bytes while the host goes on planning: send the queue once it holds 64 MiB
  // (staged path: a whole staging buffer, so that each call still pipelines its rounds)
  const mp_pool *x = mv.from->desc.tier == MP_TIER_HBM ? mv.from : mv.to;
  const uint64_t enough =
      (mv.flags & MP_DIRECT) ? (64ull << 20) : std::max<uint64_t>(64ull << 20, x->desc.staging_bytes);
  if ((uint64_t)mv.src.size() * mv.to->B >= enough) return flush_moves(mv);
  return MP_OK;
}

}  // namespace

// =============================================================================================
extern "C" {

const char *mp_strerror(int code) {
  switch (code) {
    case MP_OK: return "ok";
    case MP_EINVAL: return "invalid argument";
    case MP_ESHAPE: return "geometry mismatch";
    case MP_ENOMEM: return "out of blocks";
    case MP_ENOSTAGING: return "staging buffer missing or too small";
    case MP_EHIP: return "HIP runtime error";
    case MP_ESTALE: return "claimed prefix not in destination index";
    case MP_EHOST: return "host memory allocation failed or internal error";
    default: return "unknown error";
  }
}

int mp_selftest(void) {
  const uint32_t ds[] = {1, 2, 3, 5, 7, 8, 20, 64, 80, 160, 255, 256, 257, 1000, 4097, 65535,
                         65536, 65537, 1u << 20, (1u << 20) + 1, 0x7fffffffu};
  const uint32_t xs[] = {0, 1, 2, 63, 64, 65, 4095, 4096, 1u << 16, (1u << 24) - 1, 1u << 24,
                         0x3fffffffu, 0x40000000u, 0x7ffffffeu, 0x7fffffffu};
  for (uint32_t d : ds) {
    const FastDiv f = make_fastdiv(d);
    for (uint32_t x : xs)
      for (uint32_t k = 0; k < 3; ++k) {
        const uint32_t v = x >= k ? x - k : x;
        if (fastdiv(v, f) != v / d) return MP_EINVAL;
      }
    for (uint64_t q = 0; q < 64; ++q) {  // around multiples of d
      const uint64_t base = q * d * 33554431ull % 0x80000000ull / d * d;
      for (int k = -1; k <= 1; ++k) {
        const int64_t v = (int64_t)base + k;
        if (v < 0 || v > 0x7fffffffll) continue;
        if (fastdiv((uint32_t)v, f) != (uint32_t)v / d) return MP_EINVAL;
      }
    }
  }
  // table sorting: both code paths (comparison sort, radix sort) against a reference, key
  // ranges around the digit boundaries, repeated keys
  try {
    std::vector<uint64_t> a, b;
    uint64_t seed = 88172645463325252ull;
    auto next = [&]() { seed ^= seed << 13; seed ^= seed >> 7; seed ^= seed << 17; return seed; };
    for (uint32_t range : {1u, 2u, 2047u, 2048u, 2049u, 40960u, (1u << 22) + 5u, 0x7fffffffu})
      for (uint32_t n : {0u, 1u, 2u, 511u, 512u, 513u, 5000u}) {
        std::vector<int32_t> key(n), other(n), ko(n), oo(n);
        for (uint32_t i = 0; i < n; ++i) {
          key[i] = (int32_t)(next() % range);
          other[i] = (int32_t)(next() % 0x7fffffffu);
        }
        sort_pairs(a, b, key.data(), other.data(), n, range, ko.data(), oo.data());
        std::vector<std::pair<int32_t, int32_t>> want(n), got(n);
        for (uint32_t i = 0; i < n; ++i) want[i] = {key[i], other[i]}, got[i] = {ko[i], oo[i]};
        for (uint32_t i = 1; i < n; ++i)
          if (ko[i] < ko[i - 1]) return MP_EINVAL;
        std::sort(want.begin(), want.end());
        std::sort(got.begin(), got.end());
        if (want != got) return MP_EINVAL;  // the same pairs, none lost or split
      }
  } catch (...) {
    return MP_EHOST;
  }
  return MP_OK;
}

int mp_pool_create(const mp_pool_desc_t *desc, mp_pool_t **out) {
  try {
    if (!desc || !out) return MP_EINVAL;
    *out = nullptr;
    if (!desc->n_layers || !desc->n_kv_heads || !desc->head_dim || !desc->block_size ||
        !desc->elem_bytes || !desc->n_blocks || !desc->base)
      return MP_EINVAL;
    if (desc->tier != MP_TIER_HBM && desc->tier != MP_TIER_HOST_PINNED) return MP_EINVAL;
    if (desc->layout > MP_LAYOUT_AGGREGATED || desc->reserved != 0) return MP_EINVAL;
    if (desc->tier == MP_TIER_HOST_PINNED && desc->layout == MP_LAYOUT_DISCRETE) return MP_EINVAL;
    if (desc->n_blocks > 0x7fffffffu || desc->n_layers > 0x7fffu) return MP_EINVAL;
    const uint64_t F = (uint64_t)desc->block_size * desc->n_kv_heads * desc->head_dim * desc->elem_bytes;
    if (F % 16 != 0 || F > (1ull << 34)) return MP_EINVAL;
    if (((uintptr_t)desc->base & 15u) || ((uintptr_t)desc->staging & 15u)) return MP_EINVAL;
    mp_pool *p = new mp_pool;
    p->desc = *desc;
    p->F = F;
    p->P = 2 * desc->n_layers;
    p->B = F * p->P;
    p->idx.init(desc->n_blocks, desc->block_size, desc->tier, desc->instance_id);
    *out = p;
    return MP_OK;
  }
  MP_CATCH(nullptr)
}

int mp_pool_destroy(mp_pool_t *p) {
  if (!p) return MP_EINVAL;
  DeviceCtx &d = p->dev;
  if (d.ready) {
    (void)hipStreamSynchronize(d.stream);
    (void)hipStreamSynchronize(d.side);
    (void)hipStreamSynchronize(d.hash);
    prof_drain(p);
    for (int s = 0; s < DeviceCtx::kTableSlots; ++s) release(d.tables[s]);
    release(d.tokens);
    release(d.offsets);
    release(d.hashes);
    release(d.hash_done);
    mirror_disable(p);
    release(d.m_updates);
    release(d.m_out);
    destroy_device_objects(d);
  }
  delete p;
  return MP_OK;
}

int mp_pool_stats(mp_pool_t *p, mp_pool_stats_t *out) {
  if (!p || !out) return MP_EINVAL;
  out->n_blocks = p->idx.n_blocks();
  out->n_free = p->idx.n_free();
  out->n_held = p->idx.n_held();
  out->n_indexed = p->idx.n_indexed();
  out->n_historical = p->idx.n_historical();
  out->clock = p->idx.clock();
  return MP_OK;
}

const char *mp_last_error(mp_pool_t *p) { return p ? p->err.c_str() : "null pool"; }

int mp_alloc(mp_pool_t *p, uint32_t n, int32_t *blocks_out, uint32_t flags) {
  try {
    if (!p) return MP_EINVAL;
    if (!blocks_out && n) return fail(p, MP_EINVAL, "null output array");
    if (!p->idx.alloc(n, blocks_out, (flags & MP_EVICT_ON_DEMAND) != 0))
      return fail(p, MP_ENOMEM, "not enough free (or evictable) blocks");
    return MP_OK;
  }
  MP_CATCH(p)
}

int mp_free(mp_pool_t *p, const int32_t *blocks, uint32_t n) {
  try {
    if (!p) return MP_EINVAL;
    if (!blocks && n) return fail(p, MP_EINVAL, "null block list");
    if (!p->idx.release(blocks, n)) return fail(p, MP_EINVAL, "id out of range or not referenced");
    return MP_OK;
  }
  MP_CATCH(p)
}

int mp_insert_hashed(mp_pool_t *p, const uint32_t *tokens, uint32_t n_tokens,
                     const uint64_t *hashes, const int32_t *blocks, uint32_t n_blocks,
                     uint32_t flags, uint32_t *n_new_out) {
  try {
    (void)flags;
    if (!p) return MP_EINVAL;
    if ((!tokens && n_tokens) || !n_new_out) return fail(p, MP_EINVAL, "null argument");
    const uint32_t nb = n_tokens / p->desc.block_size;
    if (n_blocks < nb || ((!blocks || !hashes) && nb))
      return fail(p, MP_EINVAL, "fewer block ids than full blocks");
    const uint32_t m = p->idx.walk(tokens, hashes, nb, nullptr);
    if (!p->idx.adoptable(blocks, m, nb))
      return fail(p, MP_EINVAL, "blocks to adopt must be held, un-indexed and distinct");
    *n_new_out = p->idx.insert(tokens, hashes, nb, blocks);
    return MP_OK;
  }
  MP_CATCH(p)
}

int mp_match_hashed(mp_pool_t *p, const uint32_t *tokens, uint32_t n_tokens,
                    const uint64_t *hashes, int32_t *blocks_out, uint32_t cap,
                    uint32_t *n_matched_out, uint32_t flags) {
  try {
    if (!p) return MP_EINVAL;
    if ((!tokens && n_tokens) || !n_matched_out || (!blocks_out && cap))
      return fail(p, MP_EINVAL, "null argument");
    uint32_t nb = std::min(n_tokens / p->desc.block_size, cap);
    if (!hashes && nb) return fail(p, MP_EINVAL, "null hashes");
    match_walk(p, tokens, hashes, nb, blocks_out, n_matched_out, flags);
    return MP_OK;
  }
  MP_CATCH(p)
}

int mp_block_hashes(mp_pool_t *p, const uint32_t *tokens, uint32_t n_tokens, uint64_t *out,
                    uint32_t flags) {
  try {
    if (!p) return MP_EINVAL;
    if ((!tokens && n_tokens) || (!out && n_tokens / p->desc.block_size))
      return fail(p, MP_EINVAL, "null argument");
    const uint32_t tok_off[2] = {0, n_tokens};
    std::vector<uint32_t> hoff;
    const uint32_t *htok;
    const uint64_t *hh;
    int rc = device_hashes(p, tokens, tok_off, 1, (flags & MP_TOKENS_ON_DEVICE) != 0, hoff, &htok, &hh);
    if (rc != MP_OK) return rc;
    std::memcpy(out, hh, 8ull * hoff[1]);
    return MP_OK;
  }
  MP_CATCH(p)
}

int mp_block_hashes_batch(mp_pool_t *p, const uint32_t *tokens, const uint32_t *tok_off,
                          uint32_t n_req, uint64_t *out, uint32_t flags) {
  try {
    if (!p) return MP_EINVAL;
    if (!tok_off) return fail(p, MP_EINVAL, "null argument");
    if (tok_off[0] != 0) return fail(p, MP_EINVAL, "offsets must start at 0");
    for (uint32_t r = 0; r < n_req; ++r)
      if (tok_off[r + 1] < tok_off[r]) return fail(p, MP_EINVAL, "offsets must be non-decreasing");
    if (!tokens && tok_off[n_req]) return fail(p, MP_EINVAL, "null tokens");
    std::vector<uint32_t> hoff;
    const uint32_t *htok;
    const uint64_t *hh;
    int rc = device_hashes(p, tokens, tok_off, n_req, (flags & MP_TOKENS_ON_DEVICE) != 0, hoff, &htok,
                           &hh);
    if (rc != MP_OK) return rc;
    if (hoff[n_req] && !out) return fail(p, MP_EINVAL, "null output array");
    std::memcpy(out, hh, 8ull * hoff[n_req]);
    return MP_OK;
  }
  MP_CATCH(p)
}

int mp_insert(mp_pool_t *p, const uint32_t *tokens, uint32_t n_tokens, const int32_t *blocks,
              uint32_t n_blocks, uint32_t flags, uint32_t *n_new_out) {
  try {
    if (!p) return MP_EINVAL;
    if ((!tokens && n_tokens) || !n_new_out) return fail(p, MP_EINVAL, "null argument");
    const uint32_t nb = n_tokens / p->desc.block_size;
    if (n_blocks < nb || (!blocks && nb)) return fail(p, MP_EINVAL, "fewer block ids than full blocks");
    const uint32_t tok_off[2] = {0, n_tokens};
    std::vector<uint32_t> hoff;
    const uint32_t *htok;
    const uint64_t *hh;
    int rc = device_hashes(p, tokens, tok_off, 1, (flags & MP_TOKENS_ON_DEVICE) != 0, hoff, &htok, &hh);
    if (rc != MP_OK) return rc;
    return mp_insert_hashed(p, htok, n_tokens, hh, blocks, n_blocks, flags, n_new_out);
  }
  MP_CATCH(p)
}

int mp_match_batch(mp_pool_t *p, const uint32_t *tokens, const uint32_t *tok_off, uint32_t n_req,
                   int32_t *blocks_out, const uint32_t *blk_off, uint32_t *n_matched_out,
                   uint32_t flags) {
  try {
    if (!p) return MP_EINVAL;
    if (!tok_off || !blk_off || (!n_matched_out && n_req)) return fail(p, MP_EINVAL, "null argument");
    if (tok_off[0] != 0) return fail(p, MP_EINVAL, "offsets must start at 0");
    for (uint32_t r = 0; r < n_req; ++r)
      if (tok_off[r + 1] < tok_off[r] || blk_off[r + 1] < blk_off[r])
        return fail(p, MP_EINVAL, "offsets must be non-decreasing");
    if (!tokens && tok_off[n_req]) return fail(p, MP_EINVAL, "null tokens");
    if (!blocks_out && blk_off[n_req] != blk_off[0]) return fail(p, MP_EINVAL, "null output array");
    std::vector<uint32_t> &hoff = p->match_hoff;
    const uint32_t *htok;
    const uint64_t *hh;
    if (p->dev.mirror_on && n_req) {
      // device probe: slot offsets relative to the first request's slot; the host only stamps,
      // pins and copies out what the kernel found
      std::vector<uint32_t> rel(n_req + 1);
      for (uint32_t r = 0; r <= n_req; ++r) rel[r] = blk_off[r] - blk_off[0];
      int rc = device_hashes(p, tokens, tok_off, n_req, (flags & MP_TOKENS_ON_DEVICE) != 0, hoff,
                             &htok, &hh, rel.data());
      if (rc != MP_OK) return rc;
      const uint32_t *o = (const uint32_t *)p->dev.m_out.host;
      const uint32_t *cnt = o + n_req + 1;
      const int32_t *ids = (const int32_t *)(o + 2ull * n_req + 1);
      for (uint32_t r = 0; r < n_req; ++r) {
        p->idx.tick();
        const bool any = hoff[r + 1] > hoff[r] && rel[r + 1] > rel[r];
        const uint32_t m = any ? cnt[r] : 0;
        int32_t *dst = blocks_out + blk_off[r];
        if (m) std::memcpy(dst, ids + rel[r], 4ull * m);
        p->idx.touch(dst, m);
        if (flags & MP_MATCH_PIN)
          for (uint32_t i = 0; i < m; ++i) p->idx.pin(dst[i]);
        n_matched_out[r] = m;
      }
      return MP_OK;
    }
    // the index walk of a prompt starts as soon as its hashes are there, while the kernel is
    // still busy with longer prompts
    HashWait arriving;
    int rc = device_hashes(p, tokens, tok_off, n_req, (flags & MP_TOKENS_ON_DEVICE) != 0, hoff, &htok,
                           &hh, nullptr, &arriving);
    if (rc != MP_OK) return rc;
    for (uint32_t r = 0; r < n_req; ++r) {
      if ((rc = arriving.upto(r)) != MP_OK) return rc;
      const uint32_t nb = std::min(hoff[r + 1] - hoff[r], blk_off[r + 1] - blk_off[r]);
      match_walk(p, htok + tok_off[r], hh + hoff[r], nb, blocks_out + blk_off[r], &n_matched_out[r],
                 flags);
    }
    return MP_OK;
  }
  MP_CATCH(p)
}

int mp_match(mp_pool_t *p, const uint32_t *tokens, uint32_t n_tokens, int32_t *blocks_out,
             uint32_t cap, uint32_t *n_matched_out, uint32_t flags) {
  try {
    if (!p) return MP_EINVAL;
    if (!n_matched_out) return fail(p, MP_EINVAL, "null argument");
    const uint32_t tok_off[2] = {0, n_tokens}, blk_off[2] = {0, cap};
    return mp_match_batch(p, tokens, tok_off, 1, blocks_out, blk_off, n_matched_out, flags);
  }
  MP_CATCH(p)
}

int mp_delete_hashed(mp_pool_t *p, const uint32_t *tokens, uint32_t n_tokens,
                     const uint64_t *hashes, uint32_t *n_deleted_out) {
  try {
    if (!p) return MP_EINVAL;
    if ((!tokens && n_tokens) || !n_deleted_out) return fail(p, MP_EINVAL, "null argument");
    const uint32_t nb = n_tokens / p->desc.block_size;
    if (!hashes && nb) return fail(p, MP_EINVAL, "null hashes");
    std::vector<int32_t> &path = p->scratch_ids;
    path.resize(nb);
    const uint32_t m = p->idx.walk(tokens, hashes, nb, path.data());
    *n_deleted_out = p->idx.erase_path(path.data(), m);
    return MP_OK;
  }
  MP_CATCH(p)
}

int mp_delete(mp_pool_t *p, const uint32_t *tokens, uint32_t n_tokens, uint32_t flags,
              uint32_t *n_deleted_out) {
  try {
    if (!p) return MP_EINVAL;
    if ((!tokens && n_tokens) || !n_deleted_out) return fail(p, MP_EINVAL, "null argument");
    const uint32_t tok_off[2] = {0, n_tokens};
    std::vector<uint32_t> hoff;
    const uint32_t *htok;
    const uint64_t *hh;
    int rc = device_hashes(p, tokens, tok_off, 1, (flags & MP_TOKENS_ON_DEVICE) != 0, hoff, &htok, &hh);
    if (rc != MP_OK) return rc;
    return mp_delete_hashed(p, htok, n_tokens, hh, n_deleted_out);
  }
  MP_CATCH(p)
}

int mp_evict(mp_pool_t *p, uint32_t n_blocks, uint32_t *n_evicted_out) {
  try {
    if (!p) return MP_EINVAL;
    if (!n_evicted_out) return fail(p, MP_EINVAL, "null argument");
    *n_evicted_out = p->idx.evict(n_blocks);
    return MP_OK;
  }
  MP_CATCH(p)
}

int mp_transfer(mp_pool_t *src, mp_pool_t *dst, const int32_t *src_blocks, int32_t *dst_blocks,
                uint32_t n, uint32_t flags, const void *priv, uint64_t priv_len) {
  try {
    if (!src || !dst) return MP_EINVAL;
    if ((!src_blocks || !dst_blocks) && n) return fail(src, MP_EINVAL, "null block table");
    if (!same_geometry(src, dst)) return fail(src, MP_ESHAPE, "source and destination geometry differ");
    int rc = check_src_ids(src, src_blocks, n);
    if (rc != MP_OK) return rc;
    if ((flags & MP_DST_GIVEN) && !dst->idx.held_and_distinct(dst_blocks, n))
      return fail(src, MP_EINVAL, "given destination ids must be held and distinct");
    if ((rc = check_copy_feasible(src, dst, n, flags)) != MP_OK) return rc;
    if ((rc = check_same_pool(src, dst, src_blocks, dst_blocks, n, flags)) != MP_OK) return rc;
    if (!(flags & MP_DST_GIVEN)) {
      hold_sources(src, dst, src_blocks, n, true);
      const bool got = dst->idx.alloc(n, dst_blocks, (flags & MP_EVICT_ON_DEMAND) != 0);
      hold_sources(src, dst, src_blocks, n, false);
      if (!got) return fail(src, MP_ENOMEM, "destination pool cannot supply the blocks");
    }
    rc = run_copy(src, dst, src_blocks, dst_blocks, n, flags);
    if (rc == MP_OK) rc = finish_copy(src, dst, flags);
    if (rc != MP_OK) {  // a HIP failure: hand the fresh destination blocks back
      if (!(flags & MP_DST_GIVEN)) (void)dst->idx.release(dst_blocks, n);
      return rc;
    }
    if (dst->cb) dst->cb(dst->cb_user, priv, priv_len, dst_blocks, n);
    return MP_OK;
  }
  MP_CATCH(src)
}

int mp_transfer_batch(mp_pool_t *src, mp_pool_t *dst, const int32_t *src_blocks,
                      int32_t *dst_blocks, const uint32_t *blk_off, uint32_t n_req,
                      uint32_t flags) {
  try {
    if (!src || !dst) return MP_EINVAL;
    if (!blk_off) return fail(src, MP_EINVAL, "null offsets");
    if (blk_off[0] != 0) return fail(src, MP_EINVAL, "offsets must start at 0");
    for (uint32_t r = 0; r < n_req; ++r)
      if (blk_off[r + 1] < blk_off[r]) return fail(src, MP_EINVAL, "offsets must be non-decreasing");
    return mp_transfer(src, dst, src_blocks, dst_blocks, blk_off[n_req], flags, nullptr, 0);
  }
  MP_CATCH(src)
}

int mp_transfer_layers(mp_pool_t *src, mp_pool_t *dst, const int32_t *src_blocks,
                       const int32_t *dst_blocks, uint32_t n, uint32_t layer_begin,
                       uint32_t layer_end, uint32_t flags) {
  try {
    if (!src || !dst) return MP_EINVAL;
    if ((!src_blocks || !dst_blocks) && n) return fail(src, MP_EINVAL, "null block table");
    if (!same_geometry(src, dst)) return fail(src, MP_ESHAPE, "source and destination geometry differ");
    if (layer_begin >= layer_end || layer_end > src->desc.n_layers)
      return fail(src, MP_EINVAL, "layer range must be non-empty and inside [0, n_layers]");
    int rc = check_src_ids(src, src_blocks, n);
    if (rc != MP_OK) return rc;
    if (!dst->idx.held_and_distinct(dst_blocks, n))
      return fail(src, MP_EINVAL, "destination ids must be held and distinct");
    if ((rc = check_copy_feasible(src, dst, n, flags, layer_end - layer_begin)) != MP_OK) return rc;
    if (src == dst && n && tables_overlap(src, src_blocks, dst_blocks, n)) {
      if (flags & MP_DIRECT)
        return fail(src, MP_EINVAL, "MP_DIRECT within one pool needs disjoint tables");
      if ((uint64_t)n * 2ull * (layer_end - layer_begin) * src->F > src->desc.staging_bytes)
        return fail(src, MP_ENOSTAGING, "overlapping in-pool transfer must fit the staging buffer");
    }
    rc = run_copy(src, dst, src_blocks, dst_blocks, n, flags, layer_begin, layer_end);
    if (rc == MP_OK) rc = finish_copy(src, dst, flags);
    return rc;
  }
  MP_CATCH(src)
}

int mp_transfer_with_insert(mp_pool_t *src, mp_pool_t *dst, const uint32_t *tokens,
                            uint32_t n_tokens, uint32_t first_block, const int32_t *src_blocks,
                            int32_t *dst_blocks, uint32_t n, uint32_t flags, const void *priv,
                            uint64_t priv_len) {
  try {
    const uint32_t tok_off[2] = {0, n_tokens}, blk_off[2] = {0, n};
    return twi_core(src, dst, tokens, tok_off, 1, &first_block, src_blocks, dst_blocks, blk_off,
                    flags, priv, priv_len);
  }
  MP_CATCH(src)
}

int mp_transfer_with_insert_batch(mp_pool_t *src, mp_pool_t *dst, const uint32_t *tokens,
                                  const uint32_t *tok_off, uint32_t n_req,
                                  const uint32_t *first_block, const int32_t *src_blocks,
                                  int32_t *dst_blocks, const uint32_t *blk_off, uint32_t flags) {
  try {
    if (src && (flags & MP_DST_GIVEN))
      return fail(src, MP_EINVAL, "MP_DST_GIVEN is not supported in batched form");
    return twi_core(src, dst, tokens, tok_off, n_req, first_block, src_blocks, dst_blocks, blk_off,
                    flags, nullptr, 0);
  }
  MP_CATCH(src)
}

int mp_swap_out(mp_pool_t *upper, mp_pool_t *lower, uint32_t num_blocks, uint32_t flags,
                uint32_t *n_swapped_out) {
  try {
    int rc = tier_pair_ok(upper, lower);
    if (rc != MP_OK) return rc;
    if (!n_swapped_out) return fail(upper, MP_EINVAL, "null argument");
    *n_swapped_out = 0;
    if (num_blocks == 0 || upper->idx.next_victim() == kNoBlock) return MP_OK;
    if ((rc = check_copy_feasible(upper, lower, 1, flags)) != MP_OK) return rc;
    TierMove mv(upper, lower, flags);
    std::vector<int32_t> freed;  // victims: out of the index, kept off the free list until copied
    while (freed.size() < num_blocks) {
      const int32_t victim = upper->idx.next_victim();
      if (victim == kNoBlock) break;
      if (mv.known[victim] == kNoBlock) {  // else: on a prefix this call has already cached below
        rc = cache_prefix(mv, victim, false, nullptr);
        if (rc == MP_ENOMEM) {  // the lower tier is full of referenced data: not an error
          rc = MP_OK;
          break;
        }
        if (rc != MP_OK) break;
      }
      freed.push_back(upper->idx.evict_next_held());
    }
    if (rc == MP_OK) rc = flush_moves(mv);
    if (rc == MP_OK) rc = finish_copy(upper, lower, 0);
    (void)upper->idx.release(freed.data(), (uint32_t)freed.size());
    *n_swapped_out = (uint32_t)freed.size();
    return rc;
  }
  MP_CATCH(upper)
}

int mp_swap_in(mp_pool_t *lower, mp_pool_t *upper, const int32_t *lower_blocks, uint32_t n,
               int32_t *upper_blocks_out, uint32_t flags) {
  try {
    int rc = tier_pair_ok(lower, upper);
    if (rc != MP_OK) return rc;
    if ((!lower_blocks || !upper_blocks_out) && n) return fail(lower, MP_EINVAL, "null block list");
    for (uint32_t i = 0; i < n; ++i)
      if (!lower->idx.in_range(lower_blocks[i]) || !lower->idx.indexed(lower_blocks[i]))
        return fail(lower, MP_EINVAL, "block id out of range or not in the lower tier's index");
    if (n == 0) return MP_OK;
    if ((rc = check_copy_feasible(lower, upper, 1, flags)) != MP_OK) return rc;
    TierMove mv(lower, upper, flags);
    // deepest prefix first, so that one copy brings up a whole chain and its ancestors only
    // need a reference
    std::vector<std::pair<uint32_t, uint32_t>> order(n);  // (depth, position)
    for (uint32_t i = 0; i < n; ++i) {
      lower->idx.path_to(lower_blocks[i], mv.path);
      order[i] = {(uint32_t)mv.path.size(), i};
    }
    std::stable_sort(order.begin(), order.end(),
                     [](const std::pair<uint32_t, uint32_t> &a, const std::pair<uint32_t, uint32_t> &b) {
                       return a.first > b.first;
                     });
    std::vector<int32_t> taken;
    lower->idx.tick();  // the call is one use of the lower tier
    for (const auto &o : order) {
      const int32_t b = lower_blocks[o.second];
      int32_t up = mv.known[b];
      if (up != kNoBlock) {  // on a prefix brought up earlier in this call: only the reference
        upper->idx.pin(up);
      } else {
        lower->idx.path_to(b, mv.path);
        lower->idx.touch(mv.path.data(), (uint32_t)mv.path.size());
        rc = cache_prefix(mv, b, true, &up);
        if (rc != MP_OK) break;
      }
      taken.push_back(up);
      upper_blocks_out[o.second] = up;
    }
    if (rc == MP_OK) rc = flush_moves(mv);
    else (void)flush_moves(mv);  // what was indexed so far must still receive its bytes
    const int rc2 = finish_copy(lower, upper, 0);
    if (rc == MP_OK) rc = rc2;
    if (rc != MP_OK) (void)upper->idx.release(taken.data(), (uint32_t)taken.size());
    return rc;
  }
  MP_CATCH(lower)
}

int mp_transfer_static(mp_pool_t *src, mp_pool_t *dst, const int32_t *src_blocks,
                       const int32_t *dst_blocks, uint32_t n, uint32_t flags) {
  // No allocation of any kind on this path: no hipMalloc / hipFree / hipHostMalloc, no stream or
  // event creation, no std::vector growth.
  if (!src || !dst) return MP_EINVAL;
  try {
    if ((!src_blocks || !dst_blocks) && n) return fail(src, MP_EINVAL, "null block table");
    if (flags & ~(MP_DST_GIVEN | MP_ASYNC | MP_DIRECT))
      return fail(src, MP_EINVAL, "mp_transfer_static takes MP_ASYNC and MP_DIRECT only");
    if (n > MP_STATIC_MAX_BLOCKS)
      return fail(src, MP_EINVAL, "more than MP_STATIC_MAX_BLOCKS (65536) table entries");
    if (!same_geometry(src, dst)) return fail(src, MP_ESHAPE, "source and destination geometry differ");
    if (src->desc.tier != MP_TIER_HBM || dst->desc.tier != MP_TIER_HBM)
      return fail(src, MP_ESHAPE, "mp_transfer_static moves blocks between HBM pools only");
    int rc = check_src_ids(src, src_blocks, n);
    if (rc != MP_OK) return rc;
    if (!dst->idx.held_and_distinct(dst_blocks, n))
      return fail(src, MP_EINVAL, "destination ids must be held and distinct");
    const bool direct = (flags & MP_DIRECT) != 0;
    if (!direct && n && (!src->desc.staging || src->desc.staging_bytes < src->B))
      return fail(src, MP_ENOSTAGING, "staging buffer missing or smaller than one record");
    if ((rc = check_same_pool(src, dst, src_blocks, dst_blocks, n, flags | MP_DST_GIVEN)) != MP_OK)
      return rc;
    if (n == 0) return MP_OK;

    int dev = 0;
    HIP_TRY(src, hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return fail(src, MP_EINVAL, "device ordinal out of range");
    int32_t *tables = nullptr;
    {
      std::lock_guard<std::mutex> lock(g_static_mutex);
      if (!g_static_tables[dev])  // once per device, with that device current
        HIP_TRY(src, hipGetSymbolAddress((void **)&g_static_tables[dev], HIP_SYMBOL(scratch)));
      tables = g_static_tables[dev];
    }
    if (!tables) return fail(src, MP_EHIP, "no device address for the static block tables");

    // Both tables go up on the executing stream, so they are ordered behind the kernels of an
    // earlier call on the same stream that still read the array.
    hipStream_t stream = (hipStream_t)src->desc.stream;
    int32_t *d_src = tables, *d_dst = tables + MP_STATIC_MAX_BLOCKS;
    HIP_TRY(src, hipMemcpyAsync(d_src, src_blocks, 4ull * n, hipMemcpyHostToDevice, stream));
    HIP_TRY(src, hipMemcpyAsync(d_dst, dst_blocks, 4ull * n, hipMemcpyHostToDevice, stream));
    const int n_cus = src->dev.n_cus;
    bool ascends = true;  // nothing is sorted here (no host buffer to sort into): take what the caller gives
    for (uint32_t i = 1; i < n && ascends; ++i) ascends = dst_blocks[i] > dst_blocks[i - 1];
    if (direct) {
      HIP_TRY(src, launch_block_copy(pool_side(src, d_src), pool_side(dst, d_dst, 0, ascends), n, src->P,
                                     src->F, src->tune, n_cus, stream));
    } else {
      const uint32_t cap = (uint32_t)std::min<uint64_t>(src->desc.staging_bytes / src->B, 0xffffffffu);
      for (uint32_t first = 0; first < n; first += cap) {
        const uint32_t cnt = std::min(cap, n - first);
        HIP_TRY(src, launch_block_copy(pool_side(src, d_src + first),
                                       record_side(src, src->desc.staging, src->P), cnt, src->P, src->F,
                                       src->tune, n_cus, stream));
        HIP_TRY(src, launch_block_copy(record_side(src, src->desc.staging, src->P),
                                       pool_side(dst, d_dst + first, 0, ascends), cnt, src->P, src->F,
                                       src->tune, n_cus, stream));
      }
    }
    if (!(flags & MP_ASYNC)) HIP_TRY(src, hipStreamSynchronize(stream));
    return MP_OK;
  }
  MP_CATCH(src)
}

int mp_gather(mp_pool_t *p, const int32_t *tbl, uint32_t n, uint32_t flags) {
  try {
    if (!p) return MP_EINVAL;
    if (!tbl && n) return fail(p, MP_EINVAL, "null table");
    if (p->desc.tier != MP_TIER_HBM) return fail(p, MP_EINVAL, "mp_gather needs an HBM pool");
    for (uint32_t i = 0; i < n; ++i)
      if (!p->idx.in_range(tbl[i])) return fail(p, MP_EINVAL, "block id out of range");
    if (n == 0) return MP_OK;
    if (!p->desc.staging || (uint64_t)n * p->B > p->desc.staging_bytes)
      return fail(p, MP_ENOSTAGING, "staging buffer too small for the table");
    int rc = ensure_device(p);
    if (rc != MP_OK) return rc;
    const int32_t *d_src, *d_dst;
    if ((rc = upload_tables(p, tbl, nullptr, n, &d_src, &d_dst)) != MP_OK) return rc;
    {
      ProfScope ps(p, kProfGather, 2ull * n * p->B);
      HIP_TRY(p, launch_block_copy(pool_side(p, d_src), record_side(p, p->desc.staging, p->P), n, p->P,
                                   p->F, p->tune, p->dev.n_cus, p->dev.stream));
    }
    if (!(flags & MP_ASYNC)) HIP_TRY(p, hipStreamSynchronize(p->dev.stream));
    return MP_OK;
  }
  MP_CATCH(p)
}

int mp_scatter(mp_pool_t *p, const int32_t *tbl, uint32_t n, uint32_t flags) {
  try {
    if (!p) return MP_EINVAL;
    if (!tbl && n) return fail(p, MP_EINVAL, "null table");
    if (p->desc.tier != MP_TIER_HBM) return fail(p, MP_EINVAL, "mp_scatter needs an HBM pool");
    if (!p->idx.in_range_and_distinct(tbl, n))
      return fail(p, MP_EINVAL, "block id out of range or repeated");
    if (n == 0) return MP_OK;
    if (!p->desc.staging || (uint64_t)n * p->B > p->desc.staging_bytes)
      return fail(p, MP_ENOSTAGING, "staging buffer too small for the table");
    int rc = ensure_device(p);
    if (rc != MP_OK) return rc;
    const int32_t *d_src, *d_dst;
    if ((rc = upload_tables(p, nullptr, tbl, n, &d_src, &d_dst)) != MP_OK) return rc;
    {
      ProfScope ps(p, kProfScatter, 2ull * n * p->B);
      HIP_TRY(p, launch_block_copy(record_side(p, p->desc.staging, p->P), pool_side(p, d_dst), n, p->P,
                                   p->F, p->tune, p->dev.n_cus, p->dev.stream));
    }
    if (!(flags & MP_ASYNC)) HIP_TRY(p, hipStreamSynchronize(p->dev.stream));
    return MP_OK;
  }
  MP_CATCH(p)
}

int mp_set_recv_callback(mp_pool_t *p, mp_recv_cb cb, void *user) {
  if (!p) return MP_EINVAL;
  p->cb = cb;
  p->cb_user = user;
  return MP_OK;
}

int mp_profile_enable(mp_pool_t *p, int on) {
  if (!p) return MP_EINVAL;
  p->dev.profiling = on != 0;
  return MP_OK;
}

int mp_profile_read(mp_pool_t *p, int kind, double *total_ms_out, uint64_t *launches_out,
                    uint64_t *bytes_out) {
  try {
    if (!p) return MP_EINVAL;
    if (kind < 0 || kind >= kProfKinds) return fail(p, MP_EINVAL, "unknown kernel kind");
    prof_drain(p);
    if (total_ms_out) *total_ms_out = p->dev.prof_ms[kind];
    if (launches_out) *launches_out = p->dev.prof_launches[kind];
    if (bytes_out) *bytes_out = p->dev.prof_bytes[kind];
    p->dev.prof_ms[kind] = 0;
    p->dev.prof_launches[kind] = 0;
    p->dev.prof_bytes[kind] = 0;
    return MP_OK;
  }
  MP_CATCH(p)
}

int mp_plain_copy(void *dst, const void *src, uint64_t bytes, void *stream, double *ms_out) {
  if (!dst || !src || (bytes & 15u)) return MP_EINVAL;
  hipStream_t s = (hipStream_t)stream;
  hipEvent_t a, b;
  if (hipEventCreate(&a) != hipSuccess) return MP_EHIP;
  if (hipEventCreate(&b) != hipSuccess) {
    (void)hipEventDestroy(a);
    return MP_EHIP;
  }
  int rc = MP_OK;
  float ms = 0.f;
  if (hipEventRecord(a, s) != hipSuccess || launch_plain_copy(dst, src, bytes, s) != hipSuccess ||
      hipEventRecord(b, s) != hipSuccess || hipEventSynchronize(b) != hipSuccess ||
      hipEventElapsedTime(&ms, a, b) != hipSuccess)
    rc = MP_EHIP;
  (void)hipEventDestroy(a);
  (void)hipEventDestroy(b);
  if (ms_out) *ms_out = ms;
  return rc;
}

int mp_set_tunable(mp_pool_t *p, const char *key, int value) {
  try {
    if (!p || !key) return MP_EINVAL;
    const std::string k(key);
    const bool dflt = value == -1;  // -1 restores the geometry-based default
    if (k == "order" && (dflt || value == 0 || value == 1)) p->tune.order = value;
    else if (k == "plane_tile" && value >= -1 && value <= 65535) p->tune.plane_tile = value;
    else if (k == "unroll" && (dflt || value == 1 || value == 2 || value == 4 || value == 8)) p->tune.unroll = value;
    else if (k == "wg_per_cu" && value >= -1 && value <= 64) p->tune.wg_per_cu = value;
    else if (k == "nontemporal" && (dflt || value == 0 || value == 1)) p->tune.nontemporal = value;
    else if (k == "waves_per_wg" && (dflt || value == 1 || value == 4)) p->tune.waves_per_wg = value;
    else if (k == "xcd_contiguous" && (dflt || value == 0 || value == 1)) p->tune.xcd_contiguous = value;
    else if (k == "item_limit" && value >= 0) p->tune.item_limit = value;
    else if (k == "device_probe" && (value == 0 || value == 1)) {
      if (value) return mirror_enable(p);
      mirror_disable(p);
    }
    else return fail(p, MP_EINVAL, "unknown tunable or value out of range");
    return MP_OK;
  }
  MP_CATCH(p)
}

}  // extern "C"
