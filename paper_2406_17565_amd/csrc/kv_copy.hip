// kv_copy.hip -- block-table-driven copy of paged KV fragments on gfx950 (CDNA4).
//
// What it computes (paper section 5.2): bs tokens of KV live in 2*L discrete fragments of
// F bytes, one per (layer, K|V) plane; a transfer moves, for every entry i of a block table,
// all 2*L fragments between a pool and a contiguous record (the paper's aggregated block).
// One launch covers every entry, layer and K/V plane of a request batch, instead of one
// network call per discrete block as in the paper's NCCL path (section 7).
//
// Mapping to the machine: the path is pure data movement, so no MFMA and no LDS.  The unit of
// work is a wave-item: one 64-lane wavefront moves U*1 KiB of one fragment with U 16-byte
// loads per lane in flight before the first store.  Block ids are wave-uniform, so table
// reads and all address arithmetic up to the lane offset run on the scalar unit; the item ->
// (entry, plane, chunk) split uses multiply-shift division by launch invariants.
#include "kv_copy.hpp"

#include <algorithm>

namespace mempool {

FastDiv make_fastdiv(uint32_t d) {
  FastDiv f;
  f.d = d;
  uint32_t l = 0;
  while ((1ull << l) < d) ++l;  // l = ceil(log2 d)
  f.s = 31 + l;
  f.m = (uint32_t)(((1ull << f.s) + d - 1) / d);  // ceil(2^(31+l) / d) < 2^32
  return f;
}

CopyTune default_tune(CopyTune t, uint64_t frag_bytes, bool both_sides_discrete_pools,
                      bool dst_is_discrete_pool, bool dst_ids_ascend) {
  const bool sweep = dst_is_discrete_pool && dst_ids_ascend;  // stores ascend inside each plane
  if (t.order < 0) t.order = (sweep || both_sides_discrete_pools) ? 1 : 0;
  if (t.plane_tile < 0) t.plane_tile = 0;  // 0: what `order` says
  if (t.unroll < 0) t.unroll = 1;
  if (t.wg_per_cu < 0) t.wg_per_cu = 0;
  if (t.nontemporal < 0) t.nontemporal = 1;
  if (t.waves_per_wg < 0) t.waves_per_wg = 1;
  if (t.xcd_contiguous < 0)
    t.xcd_contiguous = (sweep || frag_bytes >= (64u << 10) ||
                        (frag_bytes >= (16u << 10) && dst_is_discrete_pool)) ? 1 : 0;
  return t;
}

namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// Streaming 16-byte store.  Measured on MI355X over all five geometries (fused, gather and
// scatter launches alike): next to the streaming hint (nt), agent scope on the store (sc1) is
// worth another 1-2.5 % -- the compiler's non-temporal builtin sets nt only, so the store is
// written out.  The value operand comes from compiler-tracked loads, so the compiler still
// places the wait for them in front of this instruction.
__device__ inline void store_streaming(u32x4 v, u32x4 *p) {
  asm volatile("global_store_dwordx4 %0, %1, off sc1 nt" : : "v"(p), "v"(v) : "memory");
}

struct CopyArgs {
  const uint8_t *src_base;
  uint8_t *dst_base;
  uint64_t src_plane_stride, src_block_stride;
  uint64_t dst_plane_stride, dst_block_stride;
  uint32_t n_items;    // n * n_planes * chunks_per_frag  (< 2^31)
  uint32_t frag_vecs;  // F / 16
  uint32_t n_planes;
  uint32_t n_entries;
  uint32_t xcd_span;   // workgroups per XCD for the contiguous re-mapping, 0 = off
  // The walk: plane tiles outermost, then entries, then the planes of the tile, then the
  // chunks of a fragment.  A tile of all planes walks records (entry-major), a tile of one
  // plane walks planes (plane-major).
  FastDiv by_chunks;   // / chunks_per_frag
  FastDiv by_tile;     // / planes per tile (divides n_planes)
  FastDiv by_entries;  // / n_entries
};

// W = wavefronts per workgroup.  Workgroups are dealt round-robin to the 8 XCDs in launch
// order; with a.xcd_span > 0 the workgroup index is re-mapped so that each XCD walks one
// contiguous eighth of the item space instead of every eighth item.
// KIND says which sides have a table, so the id fetch is decided at compile time -- and a
// kernel trace tells the three uses apart by name.  IDS supplies the (wave-uniform) ids.
enum CopyKind { kGather = 0 /* table on src */, kScatter = 1 /* on dst */, kFused = 2 /* both */,
                kRecords = 3 /* neither */ };
template <int U, bool NT, int W, int KIND, class IDS>
__device__ __forceinline__ void copy_items(const CopyArgs &a, const IDS &ids) {
  const uint32_t lane = threadIdx.x & 63u;
  const uint32_t wave = W == 1 ? 0u : __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const uint32_t step = gridDim.x * W;
  uint32_t wg = blockIdx.x;
  if (a.xcd_span && wg < 8u * a.xcd_span) wg = (wg & 7u) * a.xcd_span + (wg >> 3);
  for (uint32_t item = wg * W + wave; item < a.n_items; item += step) {
    // wave-uniform decomposition: item = ((tile * n_entries + i) * tile_planes + p_in) * chunks + c
    const uint32_t q = fastdiv(item, a.by_chunks);
    const uint32_t c = item - q * a.by_chunks.d;
    const uint32_t q2 = fastdiv(q, a.by_tile);
    const uint32_t p_in = q - q2 * a.by_tile.d;
    const uint32_t tile = fastdiv(q2, a.by_entries);
    const uint32_t i = q2 - tile * a.by_entries.d;   // table entry
    const uint32_t p = tile * a.by_tile.d + p_in;    // plane = layer * 2 + (K|V)
    const bool s_tbl = KIND == kGather || KIND == kFused, d_tbl = KIND == kScatter || KIND == kFused;
    const uint32_t sid = __builtin_amdgcn_readfirstlane(s_tbl ? ids.src(i) : i);
    const uint32_t did = __builtin_amdgcn_readfirstlane(d_tbl ? ids.dst(i) : i);
    const u32x4 *s = reinterpret_cast<const u32x4 *>(a.src_base + p * a.src_plane_stride +
                                                     sid * a.src_block_stride);
    u32x4 *d = reinterpret_cast<u32x4 *>(a.dst_base + p * a.dst_plane_stride +
                                         did * a.dst_block_stride);
    const uint32_t v0 = c * (64u * U) + lane;
    u32x4 reg[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const uint32_t v = v0 + 64u * u;
      if (v < a.frag_vecs) reg[u] = NT ? __builtin_nontemporal_load(s + v) : s[v];
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const uint32_t v = v0 + 64u * u;
      if (v < a.frag_vecs) {
        if (NT) store_streaming(reg[u], d + v);
        else d[v] = reg[u];
      }
    }
  }
}

// Ids from tables in device memory.  The tables are separate restrict-qualified read-only
// kernel arguments so that the wave-uniform id loads can be issued as scalar loads.  (A table
// never aliases pool or staging memory.)
struct MemoryIds {
  const int32_t *__restrict__ s;
  const int32_t *__restrict__ d;
  __device__ uint32_t src(uint32_t i) const { return (uint32_t)s[i]; }
  __device__ uint32_t dst(uint32_t i) const { return (uint32_t)d[i]; }
};
template <int U, bool NT, int W, int KIND>
__global__ __launch_bounds__(64 * W) void kv_block_copy(const CopyArgs a,
                                                        const int32_t *__restrict__ src_tbl,
                                                        const int32_t *__restrict__ dst_tbl) {
  copy_items<U, NT, W, KIND>(a, MemoryIds{src_tbl, dst_tbl});
}

// Ids from tables that travel in the kernel arguments (a transfer of one request: a few dozen
// entries): nothing has to be copied to the device before the launch.  The ids are read with
// scalar loads from the kernel-argument segment.
struct ArgumentIds {
  const SmallTables &t;
  __device__ uint32_t src(uint32_t i) const { return (uint32_t)t.src[i]; }
  __device__ uint32_t dst(uint32_t i) const { return (uint32_t)t.dst[i]; }
};
template <int W, int KIND>
__global__ __launch_bounds__(64 * W) void kv_block_copy_args(const CopyArgs a, const SmallTables t) {
  copy_items<1, true, W, KIND>(a, ArgumentIds{t});
}

// Contiguous copy with the default per-lane shape of the table-driven kernel (one-wave
// workgroups, one streaming 16-byte load and store per lane): the yardstick for what a pure
// copy reaches on this GPU, and the kernel whose hardware-counter readings calibrate the
// traffic figures of the table-driven copy.
__global__ __launch_bounds__(64) void plain_copy_kernel(const u32x4 *__restrict__ src,
                                                        u32x4 *__restrict__ dst, uint64_t n_vecs) {
  const uint64_t v = (uint64_t)blockIdx.x * 64u + threadIdx.x;
  if (v < n_vecs) store_streaming(__builtin_nontemporal_load(src + v), dst + v);
}

template <int U, int W, int KIND>
hipError_t launch_nt(const CopyArgs &a, const int32_t *st, const int32_t *dt, bool nt, dim3 grid,
                     hipStream_t stream) {
  if (nt)
    hipLaunchKernelGGL((kv_block_copy<U, true, W, KIND>), grid, dim3(64 * W), 0, stream, a, st, dt);
  else
    hipLaunchKernelGGL((kv_block_copy<U, false, W, KIND>), grid, dim3(64 * W), 0, stream, a, st, dt);
  return hipGetLastError();
}

template <int U, int W>
hipError_t launch_kind(const CopyArgs &a, const int32_t *st, const int32_t *dt, bool nt, dim3 grid,
                       hipStream_t stream) {
  if (st && dt) return launch_nt<U, W, kFused>(a, st, dt, nt, grid, stream);
  if (st) return launch_nt<U, W, kGather>(a, st, dt, nt, grid, stream);
  if (dt) return launch_nt<U, W, kScatter>(a, st, dt, nt, grid, stream);
  return launch_nt<U, W, kRecords>(a, st, dt, nt, grid, stream);
}

template <int U>
hipError_t launch_waves(const CopyArgs &a, const int32_t *st, const int32_t *dt, int waves,
                        bool nt, dim3 grid, hipStream_t stream) {
  return waves == 1 ? launch_kind<U, 1>(a, st, dt, nt, grid, stream)
                    : launch_kind<U, 4>(a, st, dt, nt, grid, stream);
}

}  // namespace

hipError_t launch_plain_copy(void *dst, const void *src, uint64_t bytes, hipStream_t stream) {
  if (bytes == 0) return hipSuccess;
  if (!dst || !src || (bytes & 15u) || (bytes >> 4) > 0x7fffffffull * 64ull)
    return hipErrorInvalidValue;
  const uint64_t n_vecs = bytes >> 4;
  const uint64_t wgs = (n_vecs + 63u) / 64u;
  hipLaunchKernelGGL(plain_copy_kernel, dim3((uint32_t)wgs), dim3(64), 0, stream,
                     (const u32x4 *)src, (u32x4 *)dst, n_vecs);
  return hipGetLastError();
}

namespace {

// Launch geometry of one launch over entries [first, first + cnt).
struct Launch {
  CopyArgs a;
  uint32_t wgs = 0, W = 1;
  int U = 1;
  bool nt = true;
};

hipError_t check_sides(const CopySide &src, const CopySide &dst, uint32_t n_planes,
                       uint64_t frag_bytes) {
  if (!src.base || !dst.base || n_planes == 0 || frag_bytes == 0 || (frag_bytes & 15u) ||
      (frag_bytes >> 4) > 0x7fffffffull)
    return hipErrorInvalidValue;
  return hipSuccess;
}

CopyTune tune_for(const CopySide &src, const CopySide &dst, bool src_tbl, bool dst_tbl,
                  uint64_t frag_bytes, const CopyTune &tune_in) {
  // plane-major walking pays off only when both ends are discrete-layout pools
  const bool both_discrete = src_tbl && dst_tbl && src.plane_stride > src.block_stride &&
                             dst.plane_stride > dst.block_stride;
  const bool dst_discrete = dst_tbl && dst.plane_stride > dst.block_stride;
  return default_tune(tune_in, frag_bytes, both_discrete, dst_discrete, dst.ascending);
}

Launch prepare(const CopySide &src, const CopySide &dst, bool src_tbl, bool dst_tbl, uint32_t first,
               uint32_t cnt, uint32_t n_planes, uint64_t frag_bytes, const CopyTune &tune, int U,
               int n_cus) {
  Launch l;
  CopyArgs &a = l.a;
  const uint32_t frag_vecs = (uint32_t)(frag_bytes >> 4);
  const uint32_t chunks = (frag_vecs + 64u * U - 1) / (64u * U);
  // a table-less side addresses entry i directly, so shift its base instead of its table
  a.src_base = (const uint8_t *)src.base + (src_tbl ? 0 : (uint64_t)first * src.block_stride);
  a.dst_base = (uint8_t *)dst.base + (dst_tbl ? 0 : (uint64_t)first * dst.block_stride);
  a.src_plane_stride = src.plane_stride;
  a.src_block_stride = src.block_stride;
  a.dst_plane_stride = dst.plane_stride;
  a.dst_block_stride = dst.block_stride;
  a.n_items = (uint32_t)((uint64_t)n_planes * chunks * cnt);
  a.frag_vecs = frag_vecs;
  a.n_planes = n_planes;
  a.n_entries = cnt;
  a.by_chunks = make_fastdiv(chunks);
  uint32_t tile_planes = tune.plane_tile > 0 ? std::min<uint32_t>((uint32_t)tune.plane_tile, n_planes)
                                             : (tune.order == 0 ? n_planes : 1u);
  while (n_planes % tile_planes) --tile_planes;  // a divisor of the plane count
  a.by_tile = make_fastdiv(tile_planes);
  a.by_entries = make_fastdiv(cnt);
  l.W = tune.waves_per_wg == 1 ? 1u : 4u;
  l.wgs = (a.n_items + l.W - 1u) / l.W;
  if (tune.wg_per_cu > 0) {
    const uint64_t cap = (uint64_t)tune.wg_per_cu * (uint64_t)(n_cus > 0 ? n_cus : 256);
    if (l.wgs > cap) l.wgs = (uint32_t)cap;
  }
  a.xcd_span = tune.xcd_contiguous ? l.wgs / 8u : 0u;
  l.U = U;
  l.nt = tune.nontemporal != 0;
  return l;
}

template <int W>
hipError_t launch_args_kind(const Launch &l, const SmallTables &t, bool st, bool dt,
                            hipStream_t stream) {
  const dim3 grid(l.wgs), block(64 * W);
  if (st && dt) hipLaunchKernelGGL((kv_block_copy_args<W, kFused>), grid, block, 0, stream, l.a, t);
  else if (st) hipLaunchKernelGGL((kv_block_copy_args<W, kGather>), grid, block, 0, stream, l.a, t);
  else hipLaunchKernelGGL((kv_block_copy_args<W, kScatter>), grid, block, 0, stream, l.a, t);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_block_copy(const CopySide &src, const CopySide &dst, uint32_t n,
                             uint32_t n_planes, uint64_t frag_bytes, const CopyTune &tune_in,
                             int n_cus, hipStream_t stream) {
  if (n == 0) return hipSuccess;
  if (check_sides(src, dst, n_planes, frag_bytes) != hipSuccess) return hipErrorInvalidValue;
  const CopyTune tune =
      tune_for(src, dst, src.tbl != nullptr, dst.tbl != nullptr, frag_bytes, tune_in);
  int U = tune.unroll;
  if (U != 1 && U != 2 && U != 4 && U != 8) return hipErrorInvalidValue;
  const uint32_t frag_vecs = (uint32_t)(frag_bytes >> 4);
  while (U > 1 && 64u * (U / 2) >= frag_vecs) U /= 2;  // no wider than the fragment
  const uint32_t chunks = (frag_vecs + 64u * U - 1) / (64u * U);
  const uint64_t per_entry = (uint64_t)n_planes * chunks;
  if (per_entry > 0x7fffffffull) return hipErrorInvalidValue;

  // keep every item index below 2^31: split very large tables into several launches
  const uint64_t item_cap = tune.item_limit > 0 ? (uint64_t)tune.item_limit : 0x7fffffffull;
  const uint32_t max_entries = (uint32_t)std::max<uint64_t>(item_cap / per_entry, 1);

  for (uint32_t first = 0; first < n; first += max_entries) {
    const uint32_t cnt = (n - first < max_entries) ? n - first : max_entries;
    const Launch l = prepare(src, dst, src.tbl != nullptr, dst.tbl != nullptr, first, cnt, n_planes,
                             frag_bytes, tune, U, n_cus);
    const int32_t *st = src.tbl ? src.tbl + first : nullptr;
    const int32_t *dt = dst.tbl ? dst.tbl + first : nullptr;
    const dim3 grid(l.wgs);
    hipError_t e;
    switch (U) {
      case 1: e = launch_waves<1>(l.a, st, dt, (int)l.W, l.nt, grid, stream); break;
      case 2: e = launch_waves<2>(l.a, st, dt, (int)l.W, l.nt, grid, stream); break;
      case 4: e = launch_waves<4>(l.a, st, dt, (int)l.W, l.nt, grid, stream); break;
      default: e = launch_waves<8>(l.a, st, dt, (int)l.W, l.nt, grid, stream); break;
    }
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

bool small_copy_possible(uint32_t n, uint32_t n_planes, uint64_t frag_bytes, const CopyTune &tune) {
  const uint64_t chunks = ((frag_bytes >> 4) + 63u) / 64u;
  return n >= 1 && n <= kSmallTable && tune.unroll < 0 && tune.nontemporal < 0 &&
         tune.wg_per_cu < 0 && tune.item_limit == 0 &&
         (uint64_t)n * n_planes * chunks <= 0x7fffffffull;
}

hipError_t launch_block_copy_small(const CopySide &src, const CopySide &dst, const SmallTables &ids,
                                   bool src_tbl, bool dst_tbl, uint32_t n, uint32_t n_planes,
                                   uint64_t frag_bytes, const CopyTune &tune_in, int n_cus,
                                   hipStream_t stream) {
  if (!small_copy_possible(n, n_planes, frag_bytes, tune_in) || (!src_tbl && !dst_tbl) ||
      check_sides(src, dst, n_planes, frag_bytes) != hipSuccess)
    return hipErrorInvalidValue;
  const CopyTune tune = tune_for(src, dst, src_tbl, dst_tbl, frag_bytes, tune_in);
  const Launch l = prepare(src, dst, src_tbl, dst_tbl, 0, n, n_planes, frag_bytes, tune, 1, n_cus);
  return l.W == 1 ? launch_args_kind<1>(l, ids, src_tbl, dst_tbl, stream)
                  : launch_args_kind<4>(l, ids, src_tbl, dst_tbl, stream);
}

}  // namespace mempool
