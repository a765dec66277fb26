// Host side of libtutti: the C ABI declared in include/tutti.h.
//
// Each entry point checks its host arguments in O(1), fills a small argument struct and
// enqueues a constant number of kernels on the caller's stream.  No allocation, no
// synchronisation, no device-to-host copy, and no state that one call leaves for another (the
// only thing remembered is the device's compute-unit count).  The set-up calls tutti_place_* are
// the exception: they time the restore on candidate planes and return host values.
//
// The same file builds the measurement library libtutti_bench.so when TUTTI_BENCH_BUILD is defined:
// the same entry points, plus the launch-tuning knobs (per host thread), the baseline kernels and
// every launch shape the knobs can select, all declared in include/tutti_bench.h.  The product
// library holds the two launch shapes it uses and no knob.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <atomic>
#include <chrono>
#include <unordered_map>
#include <vector>

#include "tutti.h"
#ifdef TUTTI_BENCH_BUILD
#include "tutti_bench.h"
#endif
#include "tutti_kernels.hip.h"

// Bitmap of tutti_table_validate_static: one bit per pool block, kept by the library on every GPU it runs on.
// In host code this name is only a stand-in; the array's device address is looked up per device (scratch_bits()).
static __device__ __align__(256) uint32_t scratch[TUTTI_STATIC_VALIDATE_MAX_BLOCKS / 32u];

namespace {

using namespace tutti;

thread_local int t_last_hip = 0;

constexpr uint32_t kDefaultWgsPerCu = 8;     // whole-GPU launches: 8 x 256 threads = 32 wavefronts per CU
constexpr uint32_t kDefaultUnroll = 4;       // 4 x 16 B in flight per lane: 4 KiB slices
constexpr uint32_t kBudgetUnroll = 8;        // CU-budgeted launches keep more bytes in flight per wavefront
constexpr int kMaxDevices = 64;

// What an experiment may change about a launch; 0 = the library's own choice.
struct Tuning {
  uint32_t wgs_per_cu = 0;
  uint32_t unroll = 0;
  uint32_t nontemporal = 3;     // bit 0: loads, bit 1: stores
  uint32_t xcd_contiguous = 0;  // item numbering per XCD (see MoveArgs::xcd_contiguous)
  uint32_t hnd_mode = 0;        // head-major pools: 0 = choose, 1 = direct, 2 = through LDS when possible
};

#ifdef TUTTI_BENCH_BUILD
thread_local Tuning t_tuning;  // set by tutti_set_*: only the calls of the same host thread see it
inline Tuning tuning() { return t_tuning; }
#else
inline Tuning tuning() { return Tuning{}; }
#endif

std::atomic<int> g_cu_count[kMaxDevices];

int hip_fail(hipError_t e) {
  t_last_hip = static_cast<int>(e);
  return TUTTI_EHIP;
}

// Compute units of the current device (queried once per device).
int cu_count() {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return hip_fail(e);
  if (dev < 0 || dev >= kMaxDevices) return TUTTI_ERANGE;
  int n = g_cu_count[dev].load(std::memory_order_relaxed);
  if (n > 0) return n;
  e = hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev);
  if (e != hipSuccess) return hip_fail(e);
  if (n <= 0) return TUTTI_ERANGE;
  g_cu_count[dev].store(n, std::memory_order_relaxed);
  return n;
}

bool is_pow2(uint32_t x) { return x != 0 && (x & (x - 1)) == 0; }
bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Geometry checks shared by every entry point; *block_bytes = T*h*d*e.
int check_geometry(const tutti_pool *pool, const tutti_objcfg *cfg, uint32_t *block_bytes) {
  if (!pool || !cfg) return TUTTI_EINVAL;
  uint64_t b = pool->block_tokens;
  b *= pool->num_kv_heads;
  if (b > 0xffffffffull) return TUTTI_EINVAL;
  b *= pool->head_dim;
  if (b > 0xffffffffull) return TUTTI_EINVAL;
  b *= pool->elt_bytes;
  if (b == 0 || b > 0xffffffffull || b % 16 != 0) return TUTTI_EINVAL;
  if (pool->num_blocks == 0) return TUTTI_EINVAL;
  if (pool->block_stride < b || pool->block_stride % 16 != 0) return TUTTI_EINVAL;
  if (pool->pool_layout != TUTTI_LAYOUT_NHD && pool->pool_layout != TUTTI_LAYOUT_HND) return TUTTI_EINVAL;
  if (!is_pow2(cfg->align) || cfg->align < 16) return TUTTI_EINVAL;
  if (cfg->chunk_bytes == 0 || cfg->chunk_bytes % cfg->align != 0) return TUTTI_EINVAL;
  if (cfg->num_layers == 0 || cfg->num_layers > 65536u) return TUTTI_EINVAL;
  *block_bytes = static_cast<uint32_t>(b);
  return TUTTI_OK;
}

int check_planes(const tutti_pool *pool) {
  if (!pool->k_base || !pool->v_base || !aligned16(pool->k_base) || !aligned16(pool->v_base)) return TUTTI_EINVAL;
  if (pool->pool_layout == TUTTI_LAYOUT_HND) {
    // a head-major row (d*e bytes) must hold whole 16-byte units
    const uint64_t row = static_cast<uint64_t>(pool->head_dim) * pool->elt_bytes;
    if (row % 16 != 0) return TUTTI_EINVAL;
  }
  return TUTTI_OK;
}

// Workgroup shape of the entry builders.  Every workgroup first stages and checks all n_req extents, so with
// thousands of requests that preamble is what a launch of many small workgroups spends its instructions on (and
// its LDS: 24 bytes per request and workgroup limit a CU to three 256-thread workgroups at 2048 requests); the
// large shape has a quarter of the workgroups do it, with four times the wavefronts each.
struct EntryLaunch {
  uint32_t wg_threads;
  uint32_t grid;
};

EntryLaunch entry_launch(uint32_t n_req, uint64_t quarters, int cus, uint32_t small_wgs_per_cu) {
  EntryLaunch L;
  L.wg_threads = n_req > 512 ? kBudgetWgThreads : kWgThreads;
  uint64_t need = (quarters + L.wg_threads - 1) / L.wg_threads;
  if (need == 0) need = 1;
  const uint64_t per_cu = L.wg_threads == kWgThreads ? small_wgs_per_cu : 2;
  const uint64_t lim = static_cast<uint64_t>(cus) * per_cu;
  L.grid = static_cast<uint32_t>(need < lim ? need : lim);
  return L;
}

SqeArgs sqe_args(const uint32_t *d_file_id, tutti_sqe *d_sqe, uint32_t *d_status, uint64_t stage_addr,
                 uint32_t sqe_cap, uint32_t chunk_bytes, uint32_t layer, uint32_t opcode, uint32_t sgl_id) {
  SqeArgs q;
  q.file_id = d_file_id;
  q.sqe = d_sqe;
  q.status = d_status;
  q.stage_addr = stage_addr;
  q.sqe_cap = sqe_cap;
  q.chunk_bytes = chunk_bytes;
  q.layer = layer;
  q.opcode = opcode;
  q.sgl_id = sgl_id;
  return q;
}

DirectArgs direct_args(const uint32_t *d_block_table, uint64_t sgl_table_addr, uint32_t table_len,
                       uint32_t num_blocks, uint32_t block_bytes) {
  DirectArgs d;
  d.table = d_block_table;
  d.sgl_table_addr = sgl_table_addr;
  d.table_len = table_len;
  d.num_blocks = num_blocks;
  d.block_bytes = block_bytes;
  return d;
}

LayoutArgs layout_args(const uint32_t *d_n_blocks, tutti_extent *d_extents, uint64_t *d_totals, uint32_t block_bytes,
                       const tutti_objcfg *cfg, uint32_t n_req) {
  LayoutArgs a;
  a.n_blocks = d_n_blocks;
  a.extents = d_extents;
  a.totals = d_totals;
  a.geom = ScanGeom{block_bytes, cfg->align, cfg->chunk_bytes};
  a.n_req = n_req;
  return a;
}

struct Launch {
  uint32_t grid;
  uint32_t wg_threads;   // kWgThreads, or kBudgetWgThreads under a CU budget
  uint32_t unroll;
  uint32_t nontemporal;  // bit 0: loads, bit 1: stores
  bool hnd_lds;          // head-major pool moved through LDS; unroll then holds 16-byte units per thread per tile
  uint32_t tile_lds;     // bytes of LDS for the tile
};

constexpr uint32_t kHndTileCap = 16384;      // largest tile staged in LDS: 8 workgroups per CU keep their tiles resident
constexpr uint32_t kDynLdsCap = 65536;       // dynamic LDS a launch may ask for without opting in to more
uint32_t log2u(uint32_t x) {
  uint32_t n = 0;
  while ((1u << n) < x) ++n;
  return n;
}

// Launch shape.  Whole GPU (cu_budget = 0): persistent 256-thread workgroups, enough for every
// item to have its own wavefront, at most wgs_per_cu per CU.  Under a CU budget B: B workgroups of
// 1024 threads, i.e. one full-size workgroup per budgeted CU, so the launch occupies at most B
// compute units and a concurrent compute kernel keeps the others to itself.
int plan_launch(uint32_t cu_budget, uint64_t n_wave_items, Launch *out) {
  const int cus = cu_count();
  if (cus < 0) return cus;
  if (cu_budget > static_cast<uint32_t>(cus)) return TUTTI_ERANGE;
  const Tuning t = tuning();
  uint32_t u = t.unroll;
  out->nontemporal = t.nontemporal & 3u;
  if (cu_budget) {
    out->hnd_lds = false;
    out->tile_lds = 0;
    out->wg_threads = kBudgetWgThreads;
    out->unroll = u ? u : kBudgetUnroll;
    const uint64_t waves = kBudgetWgThreads / kWave;
    uint64_t need = (n_wave_items + waves - 1) / waves;
    if (need == 0) need = 1;
    out->grid = static_cast<uint32_t>(need < cu_budget ? need : cu_budget);
    return TUTTI_OK;
  }
  uint32_t per_cu = t.wgs_per_cu;
  if (per_cu == 0) per_cu = kDefaultWgsPerCu;
  const uint64_t cap = static_cast<uint64_t>(cus) * per_cu;
  const uint64_t waves = kWgThreads / kWave;
  uint64_t need = (n_wave_items + waves - 1) / waves;
  if (need == 0) need = 1;
  out->hnd_lds = false;
  out->tile_lds = 0;
  out->wg_threads = kWgThreads;
  out->unroll = u ? u : kDefaultUnroll;
  out->grid = static_cast<uint32_t>(need < cap ? need : cap);
  return TUTTI_OK;
}

// Workgroups of a whole-GPU launch that fills every place (what plan_launch caps its grid at).
uint32_t whole_gpu_wgs() {
  const int cus = cu_count();
  uint32_t per_cu = tuning().wgs_per_cu;
  if (per_cu == 0) per_cu = kDefaultWgsPerCu;
  return cus > 0 ? static_cast<uint32_t>(cus) * per_cu : 0u;
}

// Fills the kernel arguments and settles how a head-major pool is moved (L->hnd_lds, L->unroll,
// L->tile_lds).  L must already hold the workgroup size and default unroll from plan_launch.
int fill_move_args(const tutti_pool *pool, uint32_t block_bytes, const uint32_t *d_block_table, uint32_t table_len,
                   const void *d_stage, uint64_t stage_cap, uint32_t *d_status, uint32_t n_req, uint32_t align,
                   Launch *L, MoveArgs *m) {
  m->k_base = static_cast<unsigned char *>(pool->k_base);
  m->v_base = static_cast<unsigned char *>(pool->v_base);
  m->stage = static_cast<unsigned char *>(const_cast<void *>(d_stage));
  m->table = d_block_table;
  m->status = d_status;
  m->block_stride = pool->block_stride;
  m->stage_cap = stage_cap;
  m->num_blocks = pool->num_blocks;
  m->block_bytes = block_bytes;
  m->table_len = table_len;
  m->row_bytes = pool->head_dim * pool->elt_bytes;
  m->block_tokens = pool->block_tokens;
  m->num_kv_heads = pool->num_kv_heads;
  m->row_shift = m->head_shift = m->token_shift = m->tile_shift = m->lds_pitch = 0;
  m->direct = 0;
  m->layer = 0;
  m->file_stride = 0;
  m->ctx_cap = 0;
  m->visit = nullptr;

  L->hnd_lds = false;
  L->tile_lds = 0;
  const uint32_t mode = tuning().hnd_mode;
  if (pool->pool_layout == TUTTI_LAYOUT_HND && mode != 1) {
    // through LDS: T, h and the row size powers of two, one token of all heads within the tile cap,
    // the tile a whole number (1, 2, 4 or 8) of 16-byte units per thread, and LDS to hold it
    const uint32_t row = m->row_bytes, T = pool->block_tokens, h = pool->num_kv_heads;
    const uint64_t group = static_cast<uint64_t>(h) * row;
    if (is_pow2(row) && is_pow2(T) && is_pow2(h) && row >= 16 && group <= kHndTileCap) {
      uint32_t tile_tokens = static_cast<uint32_t>(kHndTileCap / group);
      if (tile_tokens > T) tile_tokens = T;
      const uint32_t tile_bytes = tile_tokens * static_cast<uint32_t>(group);
      const uint32_t per_thread = tile_bytes / (L->wg_threads * 16u);
      const uint32_t pitch = static_cast<uint32_t>(group) + row;
      const uint64_t lds = static_cast<uint64_t>(align16(req_lds_bytes(n_req))) + static_cast<uint64_t>(tile_tokens) * pitch;
      const bool fits = tile_bytes % (L->wg_threads * 16u) == 0 && per_thread >= 1 && per_thread <= 8 &&
                        is_pow2(per_thread) && lds <= kDynLdsCap;
      // worth it when a row is shorter than a 128-byte line (or when asked for)
      if (fits && (mode == 2 || row < 128)) {
        L->hnd_lds = true;
        L->unroll = per_thread;
        L->tile_lds = tile_tokens * pitch;
        m->row_shift = log2u(row);
        m->head_shift = log2u(h);
        m->token_shift = log2u(T);
        m->tile_shift = log2u(tile_tokens);
        m->lds_pitch = pitch;
        m->slices_per_block = T / tile_tokens;
      }
    }
  }
  if (!L->hnd_lds) {
    const uint32_t slice = kWave * 16u * L->unroll;
    m->slices_per_block = static_cast<uint32_t>((static_cast<uint64_t>(block_bytes) + slice - 1) / slice);
  }
  // the kernels number work items in 32 bits
  if (2ull * table_len * m->slices_per_block > 0xffffffffull) return TUTTI_ERANGE;
  m->items_bound = 2u * table_len * m->slices_per_block;
  m->xcd_contiguous = tuning().xcd_contiguous;
  // dense staging: no padding anywhere and no ragged slice, so the staging offset of an item is item * slice
  const uint32_t slice_bytes = kWave * 16u * L->unroll;
  m->dense = (!L->hnd_lds && block_bytes % align == 0 && block_bytes % slice_bytes == 0) ? 1u : 0u;
  return TUTTI_OK;
}

// Work items of a move, counted in wavefronts' worth for plan_launch (an LDS tile occupies a whole workgroup).
uint64_t move_wave_items(const Launch &L, const MoveArgs &m) {
  const uint64_t items = 2ull * m.table_len * m.slices_per_block;
  return L.hnd_lds ? items * (L.wg_threads / kWave) : items;
}

template <int DIR>
hipError_t launch_move_lds(const Launch &L, uint32_t lds, hipStream_t s, const MoveArgs &m, const tutti_extent *ext,
                           uint32_t n_req) {
#define TUTTI_LDS_CASE(PT)                                                                                        \
  case PT:                                                                                                        \
    if (L.wg_threads == kWgThreads)                                                                               \
      hipLaunchKernelGGL((k_move_lds<DIR, PT, kWgThreads>), dim3(L.grid), dim3(kWgThreads), lds, s, m, ext,        \
                         n_req);                                                                                  \
    else                                                                                                          \
      hipLaunchKernelGGL((k_move_lds<DIR, PT, kBudgetWgThreads>), dim3(L.grid), dim3(kBudgetWgThreads), lds, s,    \
                         m, ext, n_req);                                                                          \
    break;
  switch (L.unroll) {
    TUTTI_LDS_CASE(1)
    TUTTI_LDS_CASE(2)
    TUTTI_LDS_CASE(4)
    TUTTI_LDS_CASE(8)
    default:
      return hipErrorInvalidValue;
  }
#undef TUTTI_LDS_CASE
  return hipGetLastError();
}

// Who does what in a fused launch (see k_layer).  L.grid is what plan_launch gave the copy; `entry_quarters` is
// the number of 16-byte quarters of entries to write.  All copy workgroups start at workgroup 0; as many
// workgroups as there are single passes of entries (one quarter per lane) also write entries, and the grid only
// grows beyond the copy's when the entries need more workgroups than the copy does, never beyond what the chip
// holds at once (a CU-budgeted launch never grows: its workgroups take several passes instead).
Roles make_roles(const Launch &L, uint64_t entry_quarters, uint32_t *grid) {
  uint64_t need = (entry_quarters + L.wg_threads - 1) / L.wg_threads;
  if (need < 1) need = 1;
  uint64_t limit = L.grid;
  if (L.wg_threads == kWgThreads) {
    uint32_t per_cu = tuning().wgs_per_cu;
    if (per_cu == 0) per_cu = kDefaultWgsPerCu;
    const int cus = cu_count();
    const uint64_t cap = cus > 0 ? static_cast<uint64_t>(cus) * per_cu : L.grid;
    if (cap > limit) limit = cap;
  }
  Roles w;
  w.sqe_wgs = static_cast<uint32_t>(need < limit ? need : limit);
  w.copy_first = 0;
  w.copy_wgs = L.grid;
  *grid = w.sqe_wgs > L.grid ? w.sqe_wgs : L.grid;
  return w;
}

template <int DIR>
hipError_t launch_layer_lds(const Launch &L, uint64_t entry_quarters, uint32_t lds, hipStream_t s, const MoveArgs &m,
                            const SqeArgs &q, const LayoutArgs &a) {
  uint32_t n_wgs = 0;
  const Roles w = make_roles(L, entry_quarters, &n_wgs);
  const dim3 grid(n_wgs);
#define TUTTI_LDS_CASE(PT)                                                                                        \
  case PT:                                                                                                        \
    if (L.wg_threads == kWgThreads)                                                                               \
      hipLaunchKernelGGL((k_layer_lds<DIR, PT, kWgThreads>), grid, dim3(kWgThreads), lds, s, m, q, a, w);         \
    else                                                                                                          \
      hipLaunchKernelGGL((k_layer_lds<DIR, PT, kBudgetWgThreads>), grid, dim3(kBudgetWgThreads), lds, s, m, q, a, \
                         w);                                                                                      \
    break;
  switch (L.unroll) {
    TUTTI_LDS_CASE(1)
    TUTTI_LDS_CASE(2)
    TUTTI_LDS_CASE(4)
    TUTTI_LDS_CASE(8)
    default:
      return hipErrorInvalidValue;
  }
#undef TUTTI_LDS_CASE
  return hipGetLastError();
}

// The launch shape as template arguments: U = 16-byte accesses in flight per lane, NT = non-temporal mask,
// WG = workgroup size.  The product library holds the two shapes plan_launch chooses by itself (whole GPU and
// under a CU budget); the measurement build adds every shape the tuning knobs can ask for.
template <int U_, int NT_, int WG_>
struct Shape {
  static constexpr int U = U_, NT = NT_, WG = WG_;
};

template <typename F>
hipError_t with_shape(const Launch &L, F &&f) {
#define TUTTI_SHAPE(U, NT, WG) \
  if (L.unroll == U && L.nontemporal == NT && L.wg_threads == WG) return f(Shape<U, NT, WG>{});
  TUTTI_SHAPE(4, 3, kWgThreads)
  TUTTI_SHAPE(8, 3, kBudgetWgThreads)
#ifdef TUTTI_BENCH_BUILD
#define TUTTI_SHAPES_NT(U, WG) TUTTI_SHAPE(U, 0, WG) TUTTI_SHAPE(U, 1, WG) TUTTI_SHAPE(U, 2, WG) TUTTI_SHAPE(U, 3, WG)
  TUTTI_SHAPES_NT(1, kWgThreads)
  TUTTI_SHAPES_NT(2, kWgThreads)
  TUTTI_SHAPES_NT(4, kWgThreads)
  TUTTI_SHAPES_NT(8, kWgThreads)
  TUTTI_SHAPES_NT(1, kBudgetWgThreads)
  TUTTI_SHAPES_NT(2, kBudgetWgThreads)
  TUTTI_SHAPES_NT(4, kBudgetWgThreads)
  TUTTI_SHAPES_NT(8, kBudgetWgThreads)
#undef TUTTI_SHAPES_NT
#endif
#undef TUTTI_SHAPE
  return hipErrorInvalidValue;
}

template <int DIR, bool HND>
hipError_t launch_move(const Launch &L, uint32_t lds, hipStream_t s, const MoveArgs &m, const tutti_extent *ext,
                       uint32_t n_req) {
  return with_shape(L, [&](auto sh) {
    using S = decltype(sh);
    hipLaunchKernelGGL((k_move<DIR, HND, S::U, S::NT, S::WG>), dim3(L.grid), dim3(S::WG), lds, s, m, ext, n_req);
    return hipGetLastError();
  });
}

template <int DIR, bool HND>
hipError_t launch_layer(const Launch &L, uint64_t entry_quarters, uint32_t lds, hipStream_t s, const MoveArgs &m,
                        const SqeArgs &q, const LayoutArgs &a) {
  uint32_t n_wgs = 0;
  const Roles w = make_roles(L, entry_quarters, &n_wgs);
  return with_shape(L, [&](auto sh) {
    using S = decltype(sh);
    if constexpr (DIR == kUnpack) {
      if (m.visit) {  // the caller's visiting order
        hipLaunchKernelGGL((k_layer<DIR, HND, S::U, S::NT, S::WG, true>), dim3(n_wgs), dim3(S::WG), lds, s, m, q, a,
                           w);
        return hipGetLastError();
      }
    }
    hipLaunchKernelGGL((k_layer<DIR, HND, S::U, S::NT, S::WG>), dim3(n_wgs), dim3(S::WG), lds, s, m, q, a, w);
    return hipGetLastError();
  });
}

template <int DIR>
int move_entry(const tutti_pool *pool, const tutti_objcfg *cfg, const tutti_extent *d_extents, uint32_t n_req,
               const uint32_t *d_block_table, uint32_t table_len, const void *d_stage, uint64_t stage_cap,
               uint32_t cu_budget, uint32_t *d_status, void *stream) {
  uint32_t bb = 0;
  int rc = check_geometry(pool, cfg, &bb);
  if (rc) return rc;
  rc = check_planes(pool);
  if (rc) return rc;
  if (n_req > TUTTI_MAX_REQ) return TUTTI_ERANGE;
  if (n_req > 0 && !d_extents) return TUTTI_EINVAL;
  if (table_len > 0 && !d_block_table) return TUTTI_EINVAL;
  if (!d_stage && (stage_cap > 0 || table_len > 0)) return TUTTI_EINVAL;
  if (!aligned16(d_stage)) return TUTTI_EINVAL;
  if (n_req == 0) return TUTTI_OK;  // nothing to move (with an empty table the kernel still reports the requests it skips)
  Launch L;
  // the workgroup size and unroll decide the item size, so settle them before sizing the grid
  rc = plan_launch(cu_budget, 0, &L);
  if (rc) return rc;
  MoveArgs m;
  rc = fill_move_args(pool, bb, d_block_table, table_len, d_stage, stage_cap, d_status, n_req, cfg->align, &L, &m);
  if (rc) return rc;
  Launch G;
  rc = plan_launch(cu_budget, move_wave_items(L, m), &G);
  if (rc) return rc;
  L.grid = G.grid;
  hipStream_t s = static_cast<hipStream_t>(stream);
  hipError_t e;
  if (L.hnd_lds) {
    e = launch_move_lds<DIR>(L, align16(req_lds_bytes(n_req)) + L.tile_lds, s, m, d_extents, n_req);
  } else {
    const uint32_t lds = req_lds_bytes(n_req);
    e = (pool->pool_layout == TUTTI_LAYOUT_HND) ? launch_move<DIR, true>(L, lds, s, m, d_extents, n_req)
                                                 : launch_move<DIR, false>(L, lds, s, m, d_extents, n_req);
  }
  return e == hipSuccess ? TUTTI_OK : hip_fail(e);
}

}  // namespace

extern "C" {

int tutti_obj_layout(const tutti_pool *pool, const tutti_objcfg *cfg, const uint32_t *d_n_blocks, uint32_t n_req,
                     tutti_extent *d_extents, uint64_t *d_totals, void *stream) {
  uint32_t bb = 0;
  int rc = check_geometry(pool, cfg, &bb);
  if (rc) return rc;
  if (n_req > TUTTI_MAX_REQ) return TUTTI_ERANGE;
  if (!d_totals || (n_req > 0 && (!d_n_blocks || !d_extents))) return TUTTI_EINVAL;
  const LayoutArgs a = layout_args(d_n_blocks, d_extents, d_totals, bb, cfg, n_req);
  hipLaunchKernelGGL(k_layout, dim3(1), dim3(kWave), req_lds_bytes(n_req), static_cast<hipStream_t>(stream), a);
  hipError_t e = hipGetLastError();
  return e == hipSuccess ? TUTTI_OK : hip_fail(e);
}

int tutti_obj_pack(const tutti_pool *pool, const tutti_objcfg *cfg, const tutti_extent *d_extents, uint32_t n_req,
                   const uint32_t *d_block_table, uint32_t table_len, void *d_stage, uint64_t stage_cap,
                   uint32_t cu_budget, uint32_t *d_status, void *stream) {
  return move_entry<kPack>(pool, cfg, d_extents, n_req, d_block_table, table_len, d_stage, stage_cap, cu_budget,
                           d_status, stream);
}

int tutti_obj_unpack(const tutti_pool *pool, const tutti_objcfg *cfg, const tutti_extent *d_extents, uint32_t n_req,
                     const uint32_t *d_block_table, uint32_t table_len, const void *d_stage, uint64_t stage_cap,
                     uint32_t cu_budget, uint32_t *d_status, void *stream) {
  return move_entry<kUnpack>(pool, cfg, d_extents, n_req, d_block_table, table_len, d_stage, stage_cap, cu_budget,
                             d_status, stream);
}

int tutti_sqe_build(const tutti_pool *pool, const tutti_objcfg *cfg, const tutti_extent *d_extents, uint32_t n_req,
                    const uint32_t *d_file_id, uint32_t layer, uint32_t opcode, uint64_t stage_addr, uint32_t sgl_id,
                    tutti_sqe *d_sqe, uint32_t sqe_cap, uint32_t *d_status, void *stream) {
  uint32_t bb = 0;
  int rc = check_geometry(pool, cfg, &bb);
  if (rc) return rc;
  if (n_req > TUTTI_MAX_REQ) return TUTTI_ERANGE;
  if (n_req > 0 && (!d_extents || !d_file_id)) return TUTTI_EINVAL;
  if (sqe_cap > 0 && (!d_sqe || !aligned16(d_sqe))) return TUTTI_EINVAL;
  if (opcode != TUTTI_OP_READ && opcode != TUTTI_OP_WRITE) return TUTTI_EINVAL;
  if (layer >= cfg->num_layers) return TUTTI_EINVAL;
  if (stage_addr % cfg->align != 0) return TUTTI_EINVAL;
  if (n_req == 0) return TUTTI_OK;
  const int cus = cu_count();
  if (cus < 0) return cus;
  const SqeArgs q = sqe_args(d_file_id, d_sqe, d_status, stage_addr, sqe_cap, cfg->chunk_bytes, layer,
                             opcode, sgl_id);
  // one lane per 16-byte quarter of an entry; at most a few workgroups per CU
  const EntryLaunch E = entry_launch(n_req, 4ull * sqe_cap, cus, 4);
  const ScanGeom geom{bb, cfg->align, cfg->chunk_bytes};
  if (E.wg_threads == kWgThreads)
    hipLaunchKernelGGL(k_sqe<kWgThreads>, dim3(E.grid), dim3(kWgThreads), req_lds_bytes(n_req),
                       static_cast<hipStream_t>(stream), q, geom, d_extents, n_req);
  else
    hipLaunchKernelGGL(k_sqe<kBudgetWgThreads>, dim3(E.grid), dim3(kBudgetWgThreads), req_lds_bytes(n_req),
                       static_cast<hipStream_t>(stream), q, geom, d_extents, n_req);
  hipError_t e = hipGetLastError();
  return e == hipSuccess ? TUTTI_OK : hip_fail(e);
}

extern "C++" {
namespace {
// One layer in one launch: extents, entries (READ for a restore, WRITE for a save), then the copy.
template <int DIR>
int layer_entry(const tutti_pool *pool, const tutti_objcfg *cfg, const uint32_t *d_n_blocks, uint32_t n_req,
                const uint32_t *d_block_table, uint32_t table_len, const uint32_t *d_file_id, uint32_t layer,
                const void *d_stage, uint64_t stage_cap, uint64_t stage_addr, uint32_t sgl_id,
                tutti_extent *d_extents, uint64_t *d_totals, tutti_sqe *d_sqe, uint32_t sqe_cap, uint32_t cu_budget,
                uint32_t *d_status, void *stream, const uint32_t *d_visit = nullptr) {
  uint32_t bb = 0;
  int rc = check_geometry(pool, cfg, &bb);
  if (rc) return rc;
  rc = check_planes(pool);
  if (rc) return rc;
  if (n_req > TUTTI_MAX_REQ) return TUTTI_ERANGE;
  if (!d_totals || (n_req > 0 && (!d_n_blocks || !d_extents || !d_file_id))) return TUTTI_EINVAL;
  if (table_len > 0 && !d_block_table) return TUTTI_EINVAL;
  if (!d_stage && (stage_cap > 0 || table_len > 0)) return TUTTI_EINVAL;
  if (!aligned16(d_stage)) return TUTTI_EINVAL;
  if (sqe_cap > 0 && (!d_sqe || !aligned16(d_sqe))) return TUTTI_EINVAL;
  if (layer >= cfg->num_layers) return TUTTI_EINVAL;
  if (stage_addr % cfg->align != 0) return TUTTI_EINVAL;

  Launch L;
  rc = plan_launch(cu_budget, 0, &L);
  if (rc) return rc;
  MoveArgs m;
  rc = fill_move_args(pool, bb, d_block_table, table_len, d_stage, stage_cap, d_status, n_req, cfg->align, &L, &m);
  if (rc) return rc;
  if (!L.hnd_lds) m.visit = d_visit;  // the tiles of the through-LDS path keep staging order
  Launch G;
  rc = plan_launch(cu_budget, move_wave_items(L, m), &G);
  if (rc) return rc;
  L.grid = G.grid;
  // one lane per 16-byte quarter of an entry; no more entries than the capacity, nor than the table can give
  // (every request has at most obj/chunk + 1 chunks per object, and obj < blocks*block_bytes + align <= ... + chunk)
  uint64_t max_entries = 2ull * ((static_cast<uint64_t>(table_len) * bb) / cfg->chunk_bytes + 2ull * n_req);
  if (max_entries > sqe_cap) max_entries = sqe_cap;
  const uint64_t entry_quarters = 4ull * max_entries;

  const SqeArgs q = sqe_args(d_file_id, d_sqe, d_status, stage_addr, sqe_cap, cfg->chunk_bytes, layer,
                             (DIR == kUnpack) ? TUTTI_OP_READ : TUTTI_OP_WRITE, sgl_id);

  const LayoutArgs a = layout_args(d_n_blocks, d_extents, d_totals, bb, cfg, n_req);

  hipStream_t s = static_cast<hipStream_t>(stream);
  hipError_t e;
  if (L.hnd_lds) {
    e = launch_layer_lds<DIR>(L, entry_quarters, align16(req_lds_bytes(n_req)) + L.tile_lds, s, m, q, a);
  } else {
    const uint32_t lds = req_lds_bytes(n_req);
    e = (pool->pool_layout == TUTTI_LAYOUT_HND) ? launch_layer<DIR, true>(L, entry_quarters, lds, s, m, q, a)
                                                 : launch_layer<DIR, false>(L, entry_quarters, lds, s, m, q, a);
  }
  return e == hipSuccess ? TUTTI_OK : hip_fail(e);
}
}  // namespace
}  // extern "C++"

int tutti_layer_restore(const tutti_pool *pool, const tutti_objcfg *cfg, const uint32_t *d_n_blocks, uint32_t n_req,
                        const uint32_t *d_block_table, uint32_t table_len, const uint32_t *d_file_id,
                        uint32_t layer, const void *d_stage, uint64_t stage_cap, uint64_t stage_addr,
                        uint32_t sgl_id, tutti_extent *d_extents, uint64_t *d_totals, tutti_sqe *d_sqe,
                        uint32_t sqe_cap, uint32_t cu_budget, uint32_t *d_status, void *stream) {
  return layer_entry<kUnpack>(pool, cfg, d_n_blocks, n_req, d_block_table, table_len, d_file_id, layer, d_stage,
                              stage_cap, stage_addr, sgl_id, d_extents, d_totals, d_sqe, sqe_cap, cu_budget, d_status,
                              stream);
}

int tutti_layer_restore_ordered(const tutti_pool *pool, const tutti_objcfg *cfg, const uint32_t *d_n_blocks,
                                uint32_t n_req, const uint32_t *d_block_table, uint32_t table_len,
                                const uint32_t *d_file_id, uint32_t layer, const void *d_stage, uint64_t stage_cap,
                                uint64_t stage_addr, uint32_t sgl_id, tutti_extent *d_extents, uint64_t *d_totals,
                                tutti_sqe *d_sqe, uint32_t sqe_cap, uint32_t cu_budget, const uint32_t *d_visit,
                                uint32_t *d_status, void *stream) {
  return layer_entry<kUnpack>(pool, cfg, d_n_blocks, n_req, d_block_table, table_len, d_file_id, layer, d_stage,
                              stage_cap, stage_addr, sgl_id, d_extents, d_totals, d_sqe, sqe_cap, cu_budget, d_status,
                              stream, d_visit);
}

int tutti_layer_save(const tutti_pool *pool, const tutti_objcfg *cfg, const uint32_t *d_n_blocks, uint32_t n_req,
                     const uint32_t *d_block_table, uint32_t table_len, const uint32_t *d_file_id, uint32_t layer,
                     void *d_stage, uint64_t stage_cap, uint64_t stage_addr, uint32_t sgl_id, tutti_extent *d_extents,
                     uint64_t *d_totals, tutti_sqe *d_sqe, uint32_t sqe_cap, uint32_t cu_budget, uint32_t *d_status,
                     void *stream) {
  return layer_entry<kPack>(pool, cfg, d_n_blocks, n_req, d_block_table, table_len, d_file_id, layer, d_stage,
                            stage_cap, stage_addr, sgl_id, d_extents, d_totals, d_sqe, sqe_cap, cu_budget, d_status,
                            stream);
}

int tutti_sgl_table_build(const tutti_pool *pool, uint64_t k_addr, uint64_t v_addr, uint32_t sgl_id,
                          tutti_sgl *d_table, uint32_t cap, uint32_t *d_status, void *stream) {
  if (!pool) return TUTTI_EINVAL;
  uint64_t b = pool->block_tokens;
  b *= pool->num_kv_heads;
  if (b > 0xffffffffull) return TUTTI_EINVAL;
  b *= pool->head_dim;
  if (b > 0xffffffffull) return TUTTI_EINVAL;
  b *= pool->elt_bytes;
  if (b == 0 || b > 0xffffffffull || b % 16 != 0 || pool->num_blocks == 0) return TUTTI_EINVAL;
  if (pool->block_stride < b || pool->block_stride % 16 != 0) return TUTTI_EINVAL;
  if (cap > 0 && (!d_table || !aligned16(d_table))) return TUTTI_EINVAL;
  const int cus = cu_count();
  if (cus < 0) return cus;
  SglArgs a;
  a.table = d_table;
  a.status = d_status;
  a.k_addr = k_addr;
  a.v_addr = v_addr;
  a.block_stride = pool->block_stride;
  a.num_blocks = pool->num_blocks;
  a.block_bytes = static_cast<uint32_t>(b);
  a.sgl_id = sgl_id;
  a.cap = cap;
  uint64_t need = (2ull * pool->num_blocks + kWgThreads - 1) / kWgThreads;
  const uint64_t lim = static_cast<uint64_t>(cus) * 8;
  const uint32_t grid = static_cast<uint32_t>(need < lim ? need : lim);
  hipLaunchKernelGGL(k_sgl_table, dim3(grid), dim3(kWgThreads), 0, static_cast<hipStream_t>(stream), a);
  hipError_t e = hipGetLastError();
  return e == hipSuccess ? TUTTI_OK : hip_fail(e);
}

int tutti_sqe_build_direct(const tutti_pool *pool, const tutti_objcfg *cfg, const tutti_extent *d_extents,
                           uint32_t n_req, const uint32_t *d_block_table, uint32_t table_len,
                           const uint32_t *d_file_id, uint32_t layer, uint32_t opcode, uint64_t sgl_table_addr,
                           uint32_t sgl_id, tutti_sqe *d_sqe, uint32_t sqe_cap, uint32_t *d_status, void *stream) {
  uint32_t bb = 0;
  int rc = check_geometry(pool, cfg, &bb);
  if (rc) return rc;
  if (bb % cfg->align != 0) return TUTTI_EINVAL;
  if (n_req > TUTTI_MAX_REQ) return TUTTI_ERANGE;
  if (n_req > 0 && (!d_extents || !d_file_id)) return TUTTI_EINVAL;
  if (table_len > 0 && !d_block_table) return TUTTI_EINVAL;
  if (sqe_cap > 0 && (!d_sqe || !aligned16(d_sqe))) return TUTTI_EINVAL;
  if (opcode != TUTTI_OP_READ && opcode != TUTTI_OP_WRITE) return TUTTI_EINVAL;
  if (layer >= cfg->num_layers) return TUTTI_EINVAL;
  if (sgl_table_addr % 16 != 0) return TUTTI_EINVAL;
  if (n_req == 0) return TUTTI_OK;
  const int cus = cu_count();
  if (cus < 0) return cus;
  const SqeArgs q = sqe_args(d_file_id, d_sqe, d_status, 0, sqe_cap, bb, layer,
                             opcode, sgl_id);
  const DirectArgs d = direct_args(d_block_table, sgl_table_addr, table_len, pool->num_blocks, bb);
  const EntryLaunch E = entry_launch(n_req, 4ull * sqe_cap, cus, 8);
  const ScanGeom geom{bb, cfg->align, cfg->chunk_bytes};
  if (E.wg_threads == kWgThreads)
    hipLaunchKernelGGL(k_sqe_direct<kWgThreads>, dim3(E.grid), dim3(kWgThreads), req_lds_bytes(n_req),
                       static_cast<hipStream_t>(stream), q, d, geom, d_extents, n_req);
  else
    hipLaunchKernelGGL(k_sqe_direct<kBudgetWgThreads>, dim3(E.grid), dim3(kBudgetWgThreads), req_lds_bytes(n_req),
                       static_cast<hipStream_t>(stream), q, d, geom, d_extents, n_req);
  hipError_t e = hipGetLastError();
  return e == hipSuccess ? TUTTI_OK : hip_fail(e);
}

namespace {
int check_ring(const tutti_ring *ring, uint32_t first_slot, uint32_t n_slots) {
  if (!ring || !ring->d_sq || !ring->d_cq || ring->depth == 0) return TUTTI_EINVAL;
  if (!aligned16(ring->d_sq) || !aligned16(ring->d_cq)) return TUTTI_EINVAL;
  if (first_slot >= ring->depth || n_slots > ring->depth) return TUTTI_EINVAL;
  return TUTTI_OK;
}

// The IOCBs a chained launch completes are an earlier call's: none of them may be one this call fills or executes.
int check_done_range(const tutti_ring *ring, uint32_t first_slot, uint32_t n_slots, uint32_t done_first,
                     uint32_t done_n) {
  if (done_n == 0) return TUTTI_OK;
  const int rc = check_ring(ring, done_first, done_n);
  if (rc) return rc;
  const uint32_t ahead = (done_first + ring->depth - first_slot) % ring->depth;   // done_first seen from first_slot
  const uint32_t behind = (first_slot + ring->depth - done_first) % ring->depth;  // and the other way round
  if (n_slots > 0 && (ahead < n_slots || behind < done_n)) return TUTTI_EINVAL;
  return TUTTI_OK;
}
}  // namespace

int tutti_ring_init(const tutti_ring *ring, void *stream) {
  int rc = check_ring(ring, 0, 0);
  if (rc) return rc;
  const uint32_t n = ring->depth > 16 ? ring->depth : 16;
  hipLaunchKernelGGL(k_ring_init, dim3((n + kWgThreads - 1) / kWgThreads), dim3(kWgThreads), 0,
                     static_cast<hipStream_t>(stream), ring->d_sq, static_cast<tutti_cq_hdr *>(ring->d_cq), ring->depth);
  hipError_t e = hipGetLastError();
  return e == hipSuccess ? TUTTI_OK : hip_fail(e);
}

int tutti_iocb_fill_direct(const tutti_ring *ring, uint32_t first_slot, uint32_t n_slots, const tutti_pool *pool,
                           const tutti_objcfg *cfg, const tutti_extent *d_extents, uint32_t n_req,
                           const uint32_t *d_block_table, uint32_t table_len, const uint32_t *d_file_id,
                           uint32_t layer, uint32_t opcode, uint64_t sgl_table_addr, uint32_t sgl_id,
                           uint32_t *d_status, void *stream) {
  int rc = check_ring(ring, first_slot, n_slots);
  if (rc) return rc;
  uint32_t bb = 0;
  rc = check_geometry(pool, cfg, &bb);
  if (rc) return rc;
  if (bb % cfg->align != 0) return TUTTI_EINVAL;
  if (n_req > TUTTI_MAX_REQ) return TUTTI_ERANGE;
  if (n_req > 0 && (!d_extents || !d_file_id)) return TUTTI_EINVAL;
  if (table_len > 0 && !d_block_table) return TUTTI_EINVAL;
  if (opcode != TUTTI_OP_READ && opcode != TUTTI_OP_WRITE) return TUTTI_EINVAL;
  if (layer >= cfg->num_layers) return TUTTI_EINVAL;
  if (sgl_table_addr % 16 != 0) return TUTTI_EINVAL;
  const int cus = cu_count();
  if (cus < 0) return cus;
  RingArgs g{ring->d_sq, static_cast<tutti_cq_hdr *>(ring->d_cq), ring->depth, first_slot, n_slots};
  const SqeArgs q = sqe_args(d_file_id, nullptr, d_status, 0, 0, bb, layer,
                             opcode, sgl_id);
  const DirectArgs d = direct_args(d_block_table, sgl_table_addr, table_len, pool->num_blocks, bb);
  // (no IOCBs given: one workgroup still reports the dropped contexts)
  const EntryLaunch E = entry_launch(n_req, 4ull * n_slots * TUTTI_IOCB_SLOTS, cus, 8);
  const ScanGeom geom{bb, cfg->align, cfg->chunk_bytes};
  if (E.wg_threads == kWgThreads)
    hipLaunchKernelGGL(k_iocb_fill<kWgThreads>, dim3(E.grid), dim3(kWgThreads), req_lds_bytes(n_req),
                       static_cast<hipStream_t>(stream), g, q, d, geom, d_extents, n_req);
  else
    hipLaunchKernelGGL(k_iocb_fill<kBudgetWgThreads>, dim3(E.grid), dim3(kBudgetWgThreads), req_lds_bytes(n_req),
                       static_cast<hipStream_t>(stream), g, q, d, geom, d_extents, n_req);
  hipError_t e = hipGetLastError();
  return e == hipSuccess ? TUTTI_OK : hip_fail(e);
}

extern "C++" {
namespace {
// issue_io: the entry-driven I/O kernel, then the completion kernel (complete), or neither (a chained train: this
// launch completes the IOCBs [done_first, done_first + done_n) of an earlier one instead).
int issue_io_entry(const tutti_ring *ring, uint32_t first_slot, uint32_t n_slots, const tutti_sgl *d_sgl_table,
                   uint32_t n_desc, uint64_t sgl_table_addr, const tutti_filestore *store, uint32_t max_len,
                   uint32_t cu_budget, uint32_t *d_status, void *stream, bool complete, uint32_t done_first,
                   uint32_t done_n) {
  int rc = check_ring(ring, first_slot, n_slots);
  if (rc) return rc;
  rc = check_done_range(ring, first_slot, n_slots, done_first, done_n);
  if (rc) return rc;
  if (!store || !store->base || !aligned16(store->base) || store->file_stride % 16 != 0) return TUTTI_EINVAL;
  if (n_desc > 0 && (!d_sgl_table || !aligned16(d_sgl_table))) return TUTTI_EINVAL;
  if (max_len == 0 || max_len % 16 != 0 || sgl_table_addr % 16 != 0) return TUTTI_EINVAL;
  hipStream_t s = static_cast<hipStream_t>(stream);
  RingArgs gd{ring->d_sq, static_cast<tutti_cq_hdr *>(ring->d_cq), ring->depth, done_first, done_n};
  if (n_slots == 0) {
    if (done_n == 0) return TUTTI_OK;
    hipLaunchKernelGGL(k_complete, dim3(1), dim3(kWave), 0, s, gd);  // nothing to execute: only the completion
    const hipError_t e0 = hipGetLastError();
    return e0 == hipSuccess ? TUTTI_OK : hip_fail(e0);
  }
  Launch L;
  rc = plan_launch(cu_budget, 0, &L);
  if (rc) return rc;
  const uint32_t unroll = (L.unroll == 8) ? 8u : 4u;  // 8 KiB slices under a CU budget, 4 KiB otherwise
  const uint32_t slice = kWave * 16u * unroll;
  IoArgs a;
  a.sgl = d_sgl_table;
  a.store_base = static_cast<unsigned char *>(store->base);
  a.status = d_status;
  a.sgl_table_addr = sgl_table_addr;
  a.file_stride = store->file_stride;
  a.n_desc = n_desc;
  a.first_file_id = store->first_file_id;
  a.n_files = store->n_files;
  a.max_len = max_len;
  a.slices = static_cast<uint32_t>((static_cast<uint64_t>(max_len) + slice - 1) / slice);
  const uint64_t items = static_cast<uint64_t>(n_slots) * TUTTI_IOCB_SLOTS * a.slices;
  if (items > 0xffffffffull) return TUTTI_ERANGE;
  rc = plan_launch(cu_budget, items, &L);
  if (rc) return rc;
  // a chained launch: one more workgroup in front; a whole-GPU grid gives it one of its places
  const uint32_t lead = done_n > 0 ? 1u : 0u;
  if (lead && cu_budget == 0 && L.grid > 1 && L.grid == whole_gpu_wgs()) L.grid -= 1;
  RingArgs g{ring->d_sq, static_cast<tutti_cq_hdr *>(ring->d_cq), ring->depth, first_slot, n_slots};
  const dim3 grid(L.grid + lead);
  if (L.wg_threads == kWgThreads) {
    if (unroll == 8)
      hipLaunchKernelGGL((k_issue_io<8, kWgThreads>), grid, dim3(kWgThreads), 0, s, g, gd, a);
    else
      hipLaunchKernelGGL((k_issue_io<4, kWgThreads>), grid, dim3(kWgThreads), 0, s, g, gd, a);
  } else {
    if (unroll == 8)
      hipLaunchKernelGGL((k_issue_io<8, kBudgetWgThreads>), grid, dim3(kBudgetWgThreads), 0, s, g, gd, a);
    else
      hipLaunchKernelGGL((k_issue_io<4, kBudgetWgThreads>), grid, dim3(kBudgetWgThreads), 0, s, g, gd, a);
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return hip_fail(e);
  if (!complete) return TUTTI_OK;
  hipLaunchKernelGGL(k_complete, dim3(1), dim3(kWave), 0, s, g);
  e = hipGetLastError();
  return e == hipSuccess ? TUTTI_OK : hip_fail(e);
}
}  // namespace
}  // extern "C++"

int tutti_issue_io(const tutti_ring *ring, uint32_t first_slot, uint32_t n_slots, const tutti_sgl *d_sgl_table,
                   uint32_t n_desc, uint64_t sgl_table_addr, const tutti_filestore *store, uint32_t max_len,
                   uint32_t cu_budget, uint32_t *d_status, void *stream) {
  return issue_io_entry(ring, first_slot, n_slots, d_sgl_table, n_desc, sgl_table_addr, store, max_len, cu_budget,
                        d_status, stream, true, 0, 0);
}

int tutti_issue_io_chained(const tutti_ring *ring, uint32_t first_slot, uint32_t n_slots, uint32_t done_first_slot,
                           uint32_t done_n_slots, const tutti_sgl *d_sgl_table, uint32_t n_desc,
                           uint64_t sgl_table_addr, const tutti_filestore *store, uint32_t max_len, uint32_t cu_budget,
                           uint32_t *d_status, void *stream) {
  return issue_io_entry(ring, first_slot, n_slots, d_sgl_table, n_desc, sgl_table_addr, store, max_len, cu_budget,
                        d_status, stream, false, done_first_slot, done_n_slots);
}

extern "C++" {
namespace {
// retrieve_layer (DIR = kUnpack) / store_layer (DIR = kPack) through the rings: one launch that scans, records
// the contexts and moves the blocks, then the completion kernel.
template <int DIR>
int ring_layer_entry(const tutti_ring *ring, uint32_t first_slot, uint32_t n_slots, const tutti_pool *pool,
                     const tutti_objcfg *cfg, const uint32_t *d_n_blocks, uint32_t n_req,
                     const uint32_t *d_block_table, uint32_t table_len, const uint32_t *d_file_id, uint32_t layer,
                     uint64_t sgl_table_addr, uint32_t sgl_id, const tutti_filestore *store, tutti_extent *d_extents,
                     uint64_t *d_totals, uint32_t cu_budget, uint32_t *d_status, void *stream, bool complete = true,
                     uint32_t done_first = 0, uint32_t done_n = 0) {
  int rc = check_ring(ring, first_slot, n_slots);
  if (rc) return rc;
  rc = check_done_range(ring, first_slot, n_slots, done_first, done_n);
  if (rc) return rc;
  uint32_t bb = 0;
  rc = check_geometry(pool, cfg, &bb);
  if (rc) return rc;
  rc = check_planes(pool);
  if (rc) return rc;
  if (bb % cfg->align != 0) return TUTTI_EINVAL;
  if (n_req > TUTTI_MAX_REQ) return TUTTI_ERANGE;
  if (!d_totals || (n_req > 0 && (!d_n_blocks || !d_extents || !d_file_id))) return TUTTI_EINVAL;
  if (table_len > 0 && !d_block_table) return TUTTI_EINVAL;
  if (layer >= cfg->num_layers || sgl_table_addr % 16 != 0) return TUTTI_EINVAL;
  if (!store || !store->base || !aligned16(store->base) || store->file_stride % 16 != 0) return TUTTI_EINVAL;

  Launch L;
  rc = plan_launch(cu_budget, 0, &L);
  if (rc) return rc;
  tutti_pool raw = *pool;  // blocks travel as raw bytes: no head-major handling
  raw.pool_layout = TUTTI_LAYOUT_NHD;
  MoveArgs m;
  rc = fill_move_args(&raw, bb, d_block_table, table_len, store->base, 0, d_status, n_req, cfg->align, &L, &m);
  if (rc) return rc;
  m.dense = 0;
  m.direct = 1;
  m.layer = layer;
  m.file_stride = store->file_stride;
  m.ctx_cap = static_cast<uint64_t>(n_slots) * TUTTI_IOCB_SLOTS;
  if (m.ctx_cap * m.slices_per_block > 0xffffffffull) return TUTTI_ERANGE;  // work items are numbered in 32 bits
  Launch G;
  rc = plan_launch(cu_budget, move_wave_items(L, m), &G);
  if (rc) return rc;
  L.grid = G.grid;
  // a chained launch has one more workgroup in front (it completes the earlier call's IOCBs and leaves); a
  // whole-GPU grid gives it one of its places, so that every workgroup is still resident from the start
  const uint32_t lead = done_n > 0 ? 1u : 0u;
  if (lead && cu_budget == 0 && L.grid > 1 && L.grid == whole_gpu_wgs()) L.grid -= 1;
  // contexts to record: no more than the IOCBs hold, no more than two per table position
  uint64_t n_ctx = static_cast<uint64_t>(n_slots) * TUTTI_IOCB_SLOTS;
  if (n_ctx > 2ull * table_len) n_ctx = 2ull * table_len;

  const SqeArgs q = sqe_args(d_file_id, nullptr, d_status, 0, 0, bb, layer,
                             (DIR == kUnpack) ? TUTTI_OP_READ : TUTTI_OP_WRITE, sgl_id);
  const DirectArgs d = direct_args(d_block_table, sgl_table_addr, table_len, pool->num_blocks, bb);
  RingArgs g{ring->d_sq, static_cast<tutti_cq_hdr *>(ring->d_cq), ring->depth, first_slot, n_slots};
  RingArgs gd{ring->d_sq, static_cast<tutti_cq_hdr *>(ring->d_cq), ring->depth, done_first, done_n};
  FileArgs f{store->file_stride, store->first_file_id, store->n_files};
  const LayoutArgs a = layout_args(d_n_blocks, d_extents, d_totals, bb, cfg, n_req);

  hipStream_t s = static_cast<hipStream_t>(stream);
  uint32_t n_wgs = 0;
  const Roles w = make_roles(L, 4 * n_ctx, &n_wgs);
  const uint32_t lds = req_lds_bytes(n_req);
  Launch R = L;
  R.nontemporal = 3;  // the ring kernels have one cache policy
  hipError_t e = with_shape(R, [&](auto sh) {
    using S = decltype(sh);
    hipLaunchKernelGGL((k_layer_ring<DIR, S::U, S::WG>), dim3(n_wgs + lead), dim3(S::WG), lds, s, m, q, d, g, gd, f, a,
                       w);
    return hipGetLastError();
  });
  if (e != hipSuccess) return hip_fail(e);
  if (!complete) return TUTTI_OK;
  hipLaunchKernelGGL(k_complete, dim3(1), dim3(kWave), 0, s, g);
  e = hipGetLastError();
  return e == hipSuccess ? TUTTI_OK : hip_fail(e);
}
}  // namespace
}  // extern "C++"

int tutti_retrieve_layer_issue(const tutti_ring *ring, uint32_t first_slot, uint32_t n_slots, const tutti_pool *pool,
                               const tutti_objcfg *cfg, const uint32_t *d_n_blocks, uint32_t n_req,
                               const uint32_t *d_block_table, uint32_t table_len, const uint32_t *d_file_id,
                               uint32_t layer, uint64_t sgl_table_addr, uint32_t sgl_id, const tutti_filestore *store,
                               tutti_extent *d_extents, uint64_t *d_totals, uint32_t cu_budget, uint32_t *d_status,
                               void *stream) {
  return ring_layer_entry<kUnpack>(ring, first_slot, n_slots, pool, cfg, d_n_blocks, n_req, d_block_table, table_len,
                                   d_file_id, layer, sgl_table_addr, sgl_id, store, d_extents, d_totals, cu_budget,
                                   d_status, stream, false);
}

int tutti_store_layer_issue(const tutti_ring *ring, uint32_t first_slot, uint32_t n_slots, const tutti_pool *pool,
                            const tutti_objcfg *cfg, const uint32_t *d_n_blocks, uint32_t n_req,
                            const uint32_t *d_block_table, uint32_t table_len, const uint32_t *d_file_id,
                            uint32_t layer, uint64_t sgl_table_addr, uint32_t sgl_id, const tutti_filestore *store,
                            tutti_extent *d_extents, uint64_t *d_totals, uint32_t cu_budget, uint32_t *d_status,
                            void *stream) {
  return ring_layer_entry<kPack>(ring, first_slot, n_slots, pool, cfg, d_n_blocks, n_req, d_block_table, table_len,
                                 d_file_id, layer, sgl_table_addr, sgl_id, store, d_extents, d_totals, cu_budget,
                                 d_status, stream, false);
}

int tutti_retrieve_layer_chained(const tutti_ring *ring, uint32_t first_slot, uint32_t n_slots, uint32_t done_first_slot,
                                 uint32_t done_n_slots, const tutti_pool *pool, const tutti_objcfg *cfg,
                                 const uint32_t *d_n_blocks, uint32_t n_req, const uint32_t *d_block_table,
                                 uint32_t table_len, const uint32_t *d_file_id, uint32_t layer, uint64_t sgl_table_addr,
                                 uint32_t sgl_id, const tutti_filestore *store, tutti_extent *d_extents,
                                 uint64_t *d_totals, uint32_t cu_budget, uint32_t *d_status, void *stream) {
  return ring_layer_entry<kUnpack>(ring, first_slot, n_slots, pool, cfg, d_n_blocks, n_req, d_block_table, table_len,
                                   d_file_id, layer, sgl_table_addr, sgl_id, store, d_extents, d_totals, cu_budget,
                                   d_status, stream, false, done_first_slot, done_n_slots);
}

int tutti_store_layer_chained(const tutti_ring *ring, uint32_t first_slot, uint32_t n_slots, uint32_t done_first_slot,
                              uint32_t done_n_slots, const tutti_pool *pool, const tutti_objcfg *cfg,
                              const uint32_t *d_n_blocks, uint32_t n_req, const uint32_t *d_block_table,
                              uint32_t table_len, const uint32_t *d_file_id, uint32_t layer, uint64_t sgl_table_addr,
                              uint32_t sgl_id, const tutti_filestore *store, tutti_extent *d_extents,
                              uint64_t *d_totals, uint32_t cu_budget, uint32_t *d_status, void *stream) {
  return ring_layer_entry<kPack>(ring, first_slot, n_slots, pool, cfg, d_n_blocks, n_req, d_block_table, table_len,
                                 d_file_id, layer, sgl_table_addr, sgl_id, store, d_extents, d_totals, cu_budget,
                                 d_status, stream, false, done_first_slot, done_n_slots);
}

int tutti_complete_io(const tutti_ring *ring, uint32_t first_slot, uint32_t n_slots, void *stream) {
  const int rc = check_ring(ring, first_slot, n_slots);
  if (rc) return rc;
  if (n_slots == 0) return TUTTI_OK;
  RingArgs g{ring->d_sq, static_cast<tutti_cq_hdr *>(ring->d_cq), ring->depth, first_slot, n_slots};
  hipLaunchKernelGGL(k_complete, dim3(1), dim3(kWave), 0, static_cast<hipStream_t>(stream), g);
  const hipError_t e = hipGetLastError();
  return e == hipSuccess ? TUTTI_OK : hip_fail(e);
}

int tutti_retrieve_layer(const tutti_ring *ring, uint32_t first_slot, uint32_t n_slots, const tutti_pool *pool,
                         const tutti_objcfg *cfg, const uint32_t *d_n_blocks, uint32_t n_req,
                         const uint32_t *d_block_table, uint32_t table_len, const uint32_t *d_file_id, uint32_t layer,
                         uint64_t sgl_table_addr, uint32_t sgl_id, const tutti_filestore *store,
                         tutti_extent *d_extents, uint64_t *d_totals, uint32_t cu_budget, uint32_t *d_status,
                         void *stream) {
  return ring_layer_entry<kUnpack>(ring, first_slot, n_slots, pool, cfg, d_n_blocks, n_req, d_block_table, table_len,
                                   d_file_id, layer, sgl_table_addr, sgl_id, store, d_extents, d_totals, cu_budget,
                                   d_status, stream);
}

int tutti_store_layer(const tutti_ring *ring, uint32_t first_slot, uint32_t n_slots, const tutti_pool *pool,
                      const tutti_objcfg *cfg, const uint32_t *d_n_blocks, uint32_t n_req,
                      const uint32_t *d_block_table, uint32_t table_len, const uint32_t *d_file_id, uint32_t layer,
                      uint64_t sgl_table_addr, uint32_t sgl_id, const tutti_filestore *store, tutti_extent *d_extents,
                      uint64_t *d_totals, uint32_t cu_budget, uint32_t *d_status, void *stream) {
  return ring_layer_entry<kPack>(ring, first_slot, n_slots, pool, cfg, d_n_blocks, n_req, d_block_table, table_len,
                                 d_file_id, layer, sgl_table_addr, sgl_id, store, d_extents, d_totals, cu_budget,
                                 d_status, stream);
}

int tutti_wait_cqe(const tutti_ring *ring, uint32_t slot, uint32_t *d_flag, void *stream) {
  int rc = check_ring(ring, slot, 0);
  if (rc) return rc;
  if (!d_flag) return TUTTI_EINVAL;
  hipLaunchKernelGGL(k_cq_check, dim3(1), dim3(kWave), 0, static_cast<hipStream_t>(stream), ring->d_sq, ring->depth, slot,
                     1u, d_flag);
  hipError_t e = hipGetLastError();
  return e == hipSuccess ? TUTTI_OK : hip_fail(e);
}

int tutti_wait_cqe_range(const tutti_ring *ring, uint32_t first_slot, uint32_t n_slots, uint32_t *d_flags,
                         void *stream) {
  int rc = check_ring(ring, first_slot, n_slots);
  if (rc) return rc;
  if (n_slots > 0 && !d_flags) return TUTTI_EINVAL;
  if (n_slots == 0) return TUTTI_OK;
  const uint32_t grid = (n_slots + kWgThreads - 1) / kWgThreads;
  hipLaunchKernelGGL(k_cq_check, dim3(grid < 64u ? grid : 64u), dim3(kWgThreads), 0, static_cast<hipStream_t>(stream),
                     ring->d_sq, ring->depth, first_slot, n_slots, d_flags);
  hipError_t e = hipGetLastError();
  return e == hipSuccess ? TUTTI_OK : hip_fail(e);
}

int tutti_table_validate(uint32_t num_blocks, const uint32_t *d_block_table, uint32_t table_len, uint32_t *d_status,
                         void *stream) {
  if (num_blocks == 0 || !d_status || (table_len > 0 && !d_block_table)) return TUTTI_EINVAL;
  if (table_len == 0) return TUTTI_OK;
  const int cus = cu_count();
  if (cus < 0) return cus;
  const uint64_t tiles = (static_cast<uint64_t>(table_len) + kWgThreads - 1) / kWgThreads;
  const uint64_t lim = static_cast<uint64_t>(cus) * 8;
  const uint32_t grid = static_cast<uint32_t>(tiles < lim ? tiles : lim);
  hipLaunchKernelGGL(k_table_validate, dim3(grid), dim3(kWgThreads), 0, static_cast<hipStream_t>(stream), d_block_table,
                     table_len, num_blocks, d_status);
  hipError_t e = hipGetLastError();
  return e == hipSuccess ? TUTTI_OK : hip_fail(e);
}

extern "C++" {
namespace {
// The linear-time table check on `bits` (device memory for at least ceil(num_blocks / 32) words).
int validate_with_bitmap(uint32_t num_blocks, const uint32_t *d_block_table, uint32_t table_len, uint32_t *d_status,
                         uint32_t *bits, hipStream_t s) {
  const int cus = cu_count();
  if (cus < 0) return cus;
  const uint32_t n_words = (num_blocks + 31u) / 32u;
  const uint64_t lim = static_cast<uint64_t>(cus) * 8;
  uint64_t need = (static_cast<uint64_t>(n_words) + kWgThreads - 1) / kWgThreads;
  hipLaunchKernelGGL(k_bitmap_clear, dim3(static_cast<uint32_t>(need < lim ? need : lim)), dim3(kWgThreads), 0, s, bits,
                     n_words);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return hip_fail(e);
  need = (static_cast<uint64_t>(table_len) + kWgThreads - 1) / kWgThreads;
  hipLaunchKernelGGL(k_table_validate_bitmap, dim3(static_cast<uint32_t>(need < lim ? need : lim)), dim3(kWgThreads), 0, s,
                     d_block_table, table_len, num_blocks, bits, d_status);
  e = hipGetLastError();
  return e == hipSuccess ? TUTTI_OK : hip_fail(e);
}
}  // namespace
}  // extern "C++"

uint64_t tutti_table_validate_work_bytes(uint32_t num_blocks) {
  return ((static_cast<uint64_t>(num_blocks) + 31u) / 32u * 4u + 255u) & ~255ull;
}

int tutti_table_validate_ws(uint32_t num_blocks, const uint32_t *d_block_table, uint32_t table_len, uint32_t *d_status,
                            void *d_work, uint64_t work_bytes, void *stream) {
  if (num_blocks == 0 || !d_status || (table_len > 0 && !d_block_table)) return TUTTI_EINVAL;
  if (!d_work || !aligned16(d_work)) return TUTTI_EINVAL;
  if (work_bytes < tutti_table_validate_work_bytes(num_blocks)) return TUTTI_ERANGE;
  if (table_len == 0) return TUTTI_OK;
  return validate_with_bitmap(num_blocks, d_block_table, table_len, d_status, static_cast<uint32_t *>(d_work),
                              static_cast<hipStream_t>(stream));
}

extern "C++" {
namespace {
std::atomic<uint32_t *> g_scratch_ptr[kMaxDevices];

// Device address of `scratch` on the current device: looked up once per device, with that device current (every
// GPU holds its own copy of the array at its own address).
int scratch_bits(uint32_t **out) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return hip_fail(e);
  if (dev < 0 || dev >= kMaxDevices) return TUTTI_ERANGE;
  uint32_t *p = g_scratch_ptr[dev].load(std::memory_order_acquire);
  if (!p) {
    void *addr = nullptr;
    e = hipGetSymbolAddress(&addr, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return hip_fail(e);
    if (!addr) return TUTTI_EHIP;
    p = static_cast<uint32_t *>(addr);
    g_scratch_ptr[dev].store(p, std::memory_order_release);
  }
  *out = p;
  return TUTTI_OK;
}
}  // namespace
}  // extern "C++"

int tutti_table_validate_static(uint32_t num_blocks, const uint32_t *d_block_table, uint32_t table_len,
                                uint32_t *d_status, void *stream) {
  if (num_blocks == 0 || !d_status || (table_len > 0 && !d_block_table)) return TUTTI_EINVAL;
  if (num_blocks > TUTTI_STATIC_VALIDATE_MAX_BLOCKS) return TUTTI_ERANGE;  // the static bitmap has no bit for them
  if (table_len == 0) return TUTTI_OK;
  uint32_t *bits = nullptr;
  const int rc = scratch_bits(&bits);
  if (rc) return rc;
  return validate_with_bitmap(num_blocks, d_block_table, table_len, d_status, bits, static_cast<hipStream_t>(stream));
}

// ---- visiting order by ascending block id
// work memory: 64 words whose first holds what the check found, then the bitmap, then its prefix sums
uint64_t tutti_table_order_work_bytes(uint32_t num_blocks) {
  return 256u + 2u * tutti_table_validate_work_bytes(num_blocks);
}

int tutti_table_order(uint32_t num_blocks, const uint32_t *d_block_table, uint32_t table_len, uint32_t *d_visit,
                      void *d_work, uint64_t work_bytes, uint32_t *d_status, void *stream) {
  if (num_blocks == 0 || (table_len > 0 && (!d_block_table || !d_visit))) return TUTTI_EINVAL;
  if (!d_work || !aligned16(d_work)) return TUTTI_EINVAL;
  if (work_bytes < tutti_table_order_work_bytes(num_blocks)) return TUTTI_ERANGE;
  if (table_len == 0) return TUTTI_OK;
  const int cus = cu_count();
  if (cus < 0) return cus;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const uint32_t n_words = (num_blocks + 31u) / 32u;
  uint32_t *flags = static_cast<uint32_t *>(d_work);
  uint32_t *bits = flags + 64;
  uint32_t *prefix = bits + tutti_table_validate_work_bytes(num_blocks) / 4u;
  const uint64_t lim = static_cast<uint64_t>(cus) * 8;
  uint64_t need = (64ull + n_words + kWgThreads - 1) / kWgThreads;
  hipLaunchKernelGGL(k_bitmap_clear, dim3(static_cast<uint32_t>(need < lim ? need : lim)), dim3(kWgThreads), 0, s, flags,
                     64u + n_words);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return hip_fail(e);
  need = (static_cast<uint64_t>(table_len) + kWgThreads - 1) / kWgThreads;
  const uint32_t grid = static_cast<uint32_t>(need < lim ? need : lim);
  hipLaunchKernelGGL(k_table_validate_bitmap, dim3(grid), dim3(kWgThreads), 0, s, d_block_table, table_len, num_blocks,
                     bits, flags);
  e = hipGetLastError();
  if (e != hipSuccess) return hip_fail(e);
  hipLaunchKernelGGL(k_bitmap_prefix, dim3(1), dim3(kPrefixThreads), 0, s, bits, n_words, prefix);
  e = hipGetLastError();
  if (e != hipSuccess) return hip_fail(e);
  hipLaunchKernelGGL(k_table_rank, dim3(grid), dim3(kWgThreads), 0, s, d_block_table, table_len, bits, prefix, flags,
                     d_visit, d_status);
  e = hipGetLastError();
  return e == hipSuccess ? TUTTI_OK : hip_fail(e);
}

// ---- set-up: where a pool's planes sit in HBM (timing probe).  These calls block and return host values.

extern "C++" {
namespace {

// The probe: a restore of 2048 blocks of 32 KiB (128 MiB of payload), the shape the effect was measured with.
constexpr uint32_t kProbeBlocks = 2048, kProbeTokens = 16, kProbeHeads = 8, kProbeDim = 128, kProbeElt = 2;
constexpr uint32_t kProbeBlockBytes = kProbeTokens * kProbeHeads * kProbeDim * kProbeElt;
constexpr uint64_t kProbePayload = 2ull * kProbeBlocks * kProbeBlockBytes;
constexpr uint32_t kProbeChunk = 2u << 20;
constexpr uint32_t kProbeEntries = 2u * (kProbeBlocks * kProbeBlockBytes / kProbeChunk);
// d_work: a header (block count, file id, status, totals, one extent), the block table, the entries, the staging area
constexpr uint64_t kProbeOffStatus = 8, kProbeOffTotals = 16, kProbeOffExtent = 64, kProbeOffTable = 256;
constexpr uint64_t kProbeOffSqe = kProbeOffTable + 4ull * kProbeBlocks;
constexpr uint64_t kProbeOffStage = 65536;
static_assert(kProbeOffSqe + 64ull * kProbeEntries <= kProbeOffStage, "the probe's small buffers overlap its staging area");
static_assert(kProbePayload == TUTTI_PLACE_MIN_PLANE_BYTES, "a plane must hold the probe's blocks twice over");

uint64_t splitmix64(uint64_t *x) {
  uint64_t z = (*x += 0x9e3779b97f4a7c15ull);
  z = (z ^ (z >> 30)) * 0xbf58476d1ce4e5b9ull;
  z = (z ^ (z >> 27)) * 0x94d049bb133111ebull;
  return z ^ (z >> 31);
}

struct Events {
  std::vector<hipEvent_t> ev;
  ~Events() {
    for (hipEvent_t e : ev) (void)hipEventDestroy(e);
  }
  hipError_t make(size_t n) {
    ev.reserve(n);
    for (size_t i = 0; i < n; ++i) {
      hipEvent_t e;
      const hipError_t rc = hipEventCreate(&e);
      if (rc != hipSuccess) return rc;
      ev.push_back(e);
    }
    return hipSuccess;
  }
};

struct Probe {
  char *work = nullptr;
  uint64_t plane_bytes = 0;
  hipStream_t stream = nullptr;
  tutti_objcfg cfg{4096u, kProbeChunk, 1u};

  // Checks the arguments the two calls share and writes the header and the table: 2048 distinct block ids drawn
  // from the whole plane (the first 2048 places of a Fisher-Yates shuffle, kept sparse).
  int init(uint64_t plane_bytes_, void *d_work, uint64_t work_bytes, void *stream_) {
    if (!d_work || reinterpret_cast<uintptr_t>(d_work) % 256 != 0) return TUTTI_EINVAL;
    if (plane_bytes_ < TUTTI_PLACE_MIN_PLANE_BYTES || work_bytes < tutti_place_work_bytes()) return TUTTI_ERANGE;
    if (plane_bytes_ / kProbeBlockBytes > 0xffffffffull) return TUTTI_ERANGE;
    work = static_cast<char *>(d_work);
    plane_bytes = plane_bytes_;
    stream = static_cast<hipStream_t>(stream_);
    const uint32_t num_blocks = static_cast<uint32_t>(plane_bytes / kProbeBlockBytes);
    std::vector<uint32_t> head((kProbeOffTable + 4ull * kProbeBlocks) / 4, 0u);
    head[0] = kProbeBlocks;  // the one request's block count
    head[1] = 1u;            // its file id
    std::unordered_map<uint32_t, uint32_t> moved;  // places of the shuffle that no longer hold their own index
    uint64_t seed = 0x7475747469ull;
    for (uint32_t j = 0; j < kProbeBlocks; ++j) {
      const uint32_t k = j + static_cast<uint32_t>(splitmix64(&seed) % (num_blocks - j));
      const auto at_k = moved.find(k);
      const auto at_j = moved.find(j);
      const uint32_t vk = at_k == moved.end() ? k : at_k->second;
      const uint32_t vj = at_j == moved.end() ? j : at_j->second;
      moved[k] = vj;
      head[kProbeOffTable / 4 + j] = vk;
    }
    hipError_t e = hipMemcpyAsync(work, head.data(), head.size() * 4, hipMemcpyHostToDevice, stream);
    if (e != hipSuccess) return hip_fail(e);
    e = hipStreamSynchronize(stream);  // `head` goes out of scope
    return e == hipSuccess ? TUTTI_OK : hip_fail(e);
  }

  int restore(const void *k_plane, const void *v_plane) const {
    tutti_pool pool{};
    pool.k_base = const_cast<void *>(k_plane);
    pool.v_base = const_cast<void *>(v_plane);
    pool.block_stride = kProbeBlockBytes;
    pool.num_blocks = static_cast<uint32_t>(plane_bytes / kProbeBlockBytes);
    pool.block_tokens = kProbeTokens;
    pool.num_kv_heads = kProbeHeads;
    pool.head_dim = kProbeDim;
    pool.elt_bytes = kProbeElt;
    pool.pool_layout = TUTTI_LAYOUT_NHD;
    return tutti_layer_restore(&pool, &cfg, reinterpret_cast<const uint32_t *>(work), 1u,
                               reinterpret_cast<const uint32_t *>(work + kProbeOffTable), kProbeBlocks,
                               reinterpret_cast<const uint32_t *>(work + 4), 0u, work + kProbeOffStage, kProbePayload,
                               0ull, 1u, reinterpret_cast<tutti_extent *>(work + kProbeOffExtent),
                               reinterpret_cast<uint64_t *>(work + kProbeOffTotals),
                               reinterpret_cast<tutti_sqe *>(work + kProbeOffSqe), kProbeEntries, 0u,
                               reinterpret_cast<uint32_t *>(work + kProbeOffStatus), stream);
  }

  // us[i] <- median over `reps` passes of the restore on (ref, cands[i]), timed between events on the stream
  int pair_times(const void *ref, const void *const *cands, uint32_t n, uint32_t reps, float *us) const {
    Events evs;
    hipError_t e = evs.make(n + 1u);
    if (e != hipSuccess) return hip_fail(e);
    std::vector<float> t(static_cast<size_t>(reps) * n);
    for (uint32_t rep = 0; rep <= reps; ++rep) {  // the first pass warms up
      int rc = restore(ref, cands[n - 1]);        // so that the first timed launch does not start an idle queue
      if (rc) return rc;
      for (uint32_t i = 0; i < n; ++i) {
        e = hipEventRecord(evs.ev[i], stream);
        if (e != hipSuccess) return hip_fail(e);
        rc = restore(ref, cands[i]);
        if (rc) return rc;
      }
      e = hipEventRecord(evs.ev[n], stream);
      if (e != hipSuccess) return hip_fail(e);
      e = hipStreamSynchronize(stream);
      if (e != hipSuccess) return hip_fail(e);
      if (rep == 0) continue;
      for (uint32_t i = 0; i < n; ++i) {
        float ms = 0.f;
        e = hipEventElapsedTime(&ms, evs.ev[i], evs.ev[i + 1]);
        if (e != hipSuccess) return hip_fail(e);
        t[static_cast<size_t>(i) * reps + (rep - 1)] = ms * 1e3f;
      }
    }
    for (uint32_t i = 0; i < n; ++i) {
      float *row = t.data() + static_cast<size_t>(i) * reps;
      std::sort(row, row + reps);
      us[i] = (reps & 1u) ? row[reps / 2] : 0.5f * (row[reps / 2 - 1] + row[reps / 2]);
    }
    return TUTTI_OK;
  }

  // the status word the probe's launches ORed into: anything but 0 means the planes were not what the call was told
  int status_clean() const {
    uint32_t st = 0;
    const hipError_t e = hipMemcpy(&st, work + kProbeOffStatus, 4, hipMemcpyDeviceToHost);
    if (e != hipSuccess) return hip_fail(e);
    return st == 0 ? TUTTI_OK : TUTTI_EINVAL;
  }
};

constexpr int32_t kSetAside = -2;  // during classification: a reference that turned out to share its region with nothing

int check_plane_list(const void *const *planes, uint32_t n) {
  if (n == 0 || !planes) return TUTTI_EINVAL;
  if (n > 65536u) return TUTTI_ERANGE;
  for (uint32_t i = 0; i < n; ++i)
    if (!planes[i] || !aligned16(planes[i])) return TUTTI_EINVAL;
  return TUTTI_OK;
}

}  // namespace
}  // extern "C++"

uint64_t tutti_place_work_bytes(void) { return kProbeOffStage + kProbePayload; }

int tutti_place_pair_times(const void *ref, const void *const *cands, uint32_t n, uint64_t plane_bytes, void *d_work,
                           uint64_t work_bytes, uint32_t reps, float *us, void *stream) {
  int rc = check_plane_list(cands, n);
  if (rc) return rc;
  if (!ref || !aligned16(ref) || !us || reps == 0 || reps > 16) return TUTTI_EINVAL;
  Probe p;
  rc = p.init(plane_bytes, d_work, work_bytes, stream);
  if (rc) return rc;
  rc = p.pair_times(ref, cands, n, reps, us);
  return rc ? rc : p.status_clean();
}

int tutti_place_classify(const void *const *planes, uint32_t n, uint64_t plane_bytes, void *d_work,
                         uint64_t work_bytes, uint32_t max_regions, double min_gap_us, int32_t *classes,
                         tutti_place_round *rounds, uint32_t *n_rounds, void *stream) {
  if (n_rounds) *n_rounds = 0;
  int rc = check_plane_list(planes, n);
  if (rc) return rc;
  if (!classes || max_regions == 0 || max_regions > TUTTI_PLACE_MAX_REGIONS || !(min_gap_us >= 0.0)) return TUTTI_EINVAL;
  Probe p;
  rc = p.init(plane_bytes, d_work, work_bytes, stream);
  if (rc) return rc;
  for (uint32_t i = 0; i < n; ++i) classes[i] = -1;
  std::vector<uint32_t> todo;
  std::vector<const void *> cands;
  std::vector<float> us;
  uint32_t c = 0;
  for (uint32_t attempt = 0; c < max_regions && attempt < max_regions + 4u; ++attempt) {
    todo.clear();
    for (uint32_t i = 0; i < n; ++i)
      if (classes[i] == -1) todo.push_back(i);
    if (todo.empty()) break;
    const uint32_t r = todo[0];
    cands.assign(1, planes[r]);  // (r, r): both planes in one region by construction
    for (uint32_t i : todo) cands.push_back(planes[i]);
    us.assign(cands.size(), 0.f);
    rc = p.pair_times(planes[r], cands.data(), static_cast<uint32_t>(cands.size()), 3u, us.data());
    if (rc) return rc;
    const float slow = us[0];
    const float fast = *std::min_element(us.begin() + 1, us.end());
    uint32_t members = 0;
    if (slow - fast < min_gap_us) {  // nothing left lies in another region
      for (uint32_t i : todo) classes[i] = static_cast<int32_t>(c);
      members = static_cast<uint32_t>(todo.size());
    } else {
      const float mid = 0.5f * (slow + fast);
      for (size_t k = 0; k < todo.size(); ++k)
        if (us[k + 1] > mid || todo[k] == r) ++members;
      if (members == 1) {
        // nothing shares the reference's region although other planes are left: most likely a plane that
        // straddles two regions (every pair with it times in between).  It is set aside and gets no class.
        classes[r] = kSetAside;
        continue;
      }
      for (size_t k = 0; k < todo.size(); ++k)
        if (us[k + 1] > mid || todo[k] == r) classes[todo[k]] = static_cast<int32_t>(c);
    }
    if (rounds) rounds[c] = tutti_place_round{r, members, slow, fast};
    ++c;
    if (n_rounds) *n_rounds = c;
    if (members == todo.size()) break;
  }
  for (uint32_t i = 0; i < n; ++i)
    if (classes[i] == kSetAside) classes[i] = -1;
  return p.status_clean();
}

#ifdef TUTTI_BENCH_BUILD
// ---- measurement aids (include/tutti_bench.h): ceilings, floors and the tuning knobs

int tutti_copy_baseline(void *d_dst, const void *d_src, uint64_t bytes, uint32_t cu_budget, void *stream) {
  if (!d_dst || !d_src || !aligned16(d_dst) || !aligned16(d_src) || bytes % 16 != 0) return TUTTI_EINVAL;
  if (bytes == 0) return TUTTI_OK;
  Launch L;
  int rc = plan_launch(cu_budget, 0, &L);
  if (rc) return rc;
  const uint64_t slice = kWave * 16ull * L.unroll;
  rc = plan_launch(cu_budget, (bytes + slice - 1) / slice, &L);
  if (rc) return rc;
  hipStream_t s = static_cast<hipStream_t>(stream);
  unsigned char *dst = static_cast<unsigned char *>(d_dst);
  const unsigned char *src = static_cast<const unsigned char *>(d_src);
  const hipError_t e = with_shape(L, [&](auto sh) {
    using S = decltype(sh);
    hipLaunchKernelGGL((k_copy<S::U, S::NT, S::WG>), dim3(L.grid), dim3(S::WG), 0, s, dst, src, bytes);
    return hipGetLastError();
  });
  return e == hipSuccess ? TUTTI_OK : hip_fail(e);
}

int tutti_stream_baseline(void *d_buf, uint64_t bytes, uint32_t write, uint32_t *d_xor, uint32_t cu_budget,
                          void *stream) {
  if (!d_buf || !aligned16(d_buf) || bytes % 16 != 0) return TUTTI_EINVAL;
  if (!write && !d_xor) return TUTTI_EINVAL;
  if (bytes == 0) return TUTTI_OK;
  Launch L;
  int rc = plan_launch(cu_budget, 0, &L);
  if (rc) return rc;
  const uint32_t unroll = (L.unroll == 8) ? 8u : 4u;
  const uint64_t slice = kWave * 16ull * unroll;
  rc = plan_launch(cu_budget, (bytes + slice - 1) / slice, &L);
  if (rc) return rc;
  hipStream_t s = static_cast<hipStream_t>(stream);
  unsigned char *buf = static_cast<unsigned char *>(d_buf);
#define TUTTI_STREAM(W, U)                                                                                          \
  do {                                                                                                              \
    if (L.wg_threads == kWgThreads)                                                                                 \
      hipLaunchKernelGGL((k_stream<W, U, kWgThreads>), dim3(L.grid), dim3(kWgThreads), 0, s, buf, bytes, d_xor);   \
    else                                                                                                            \
      hipLaunchKernelGGL((k_stream<W, U, kBudgetWgThreads>), dim3(L.grid), dim3(kBudgetWgThreads), 0, s, buf, bytes, \
                         d_xor);                                                                                   \
  } while (0)
  if (write) {
    if (unroll == 8) TUTTI_STREAM(1, 8); else TUTTI_STREAM(1, 4);
  } else {
    if (unroll == 8) TUTTI_STREAM(0, 8); else TUTTI_STREAM(0, 4);
  }
#undef TUTTI_STREAM
  hipError_t e = hipGetLastError();
  return e == hipSuccess ? TUTTI_OK : hip_fail(e);
}

int tutti_scatter_baseline(void *d_scattered, uint64_t span_bytes, void *d_contig, uint64_t bytes,
                           const uint32_t *d_perm, uint32_t gran, uint32_t scatter_writes, uint32_t shape,
                           uint32_t cu_budget, void *stream) {
  if (!d_scattered || !d_contig || !d_perm || !aligned16(d_scattered) || !aligned16(d_contig)) return TUTTI_EINVAL;
  if (gran == 0 || gran % 4096 != 0 || bytes % gran != 0) return TUTTI_EINVAL;
  if (shape > TUTTI_SCATTER_SHAPE_MAX) return TUTTI_EINVAL;
  if (bytes == 0) return TUTTI_OK;
  const int cus = cu_count();
  if (cus < 0) return cus;
  hipStream_t s = static_cast<hipStream_t>(stream);
  unsigned char *sc = static_cast<unsigned char *>(d_scattered);
  unsigned char *ct = static_cast<unsigned char *>(d_contig);
  const uint32_t to = scatter_writes ? 1u : 0u;
  if (shape == TUTTI_SCATTER_WAVE_SLICE) {  // the product's shape: a wavefront per 4 KiB, 256-thread workgroups
    Launch L;
    int rc = plan_launch(cu_budget, bytes / 4096, &L);
    if (rc) return rc;
    if (L.wg_threads == kWgThreads)
      hipLaunchKernelGGL((k_scatter<4, kWgThreads>), dim3(L.grid), dim3(kWgThreads), 0, s, sc, span_bytes, ct, bytes,
                         d_perm, gran, to);
    else
      hipLaunchKernelGGL((k_scatter<4, kBudgetWgThreads>), dim3(L.grid), dim3(kBudgetWgThreads), 0, s, sc, span_bytes,
                         ct, bytes, d_perm, gran, to);
  } else {
    if (cu_budget != 0) return TUTTI_EINVAL;  // the other shapes are whole-GPU launches
    const uint64_t pieces = bytes / gran;
    const uint64_t cap = static_cast<uint64_t>(cus) * 8;
    switch (shape) {
      case TUTTI_SCATTER_WAVE_SLICE_1024: {
        const uint64_t need = (bytes / 4096 + 15) / 16;
        const uint64_t lim = static_cast<uint64_t>(cus) * 2;
        hipLaunchKernelGGL((k_scatter<4, kBudgetWgThreads>), dim3(static_cast<uint32_t>(need < lim ? need : lim)),
                           dim3(kBudgetWgThreads), 0, s, sc, span_bytes, ct, bytes, d_perm, gran, to);
        break;
      }
      case TUTTI_SCATTER_WAVE_PIECE: {
        const uint64_t need = (pieces + 3) / 4;
        hipLaunchKernelGGL((k_scatter_piece<false, 3>), dim3(static_cast<uint32_t>(need < cap ? need : cap)),
                           dim3(kWgThreads), 0, s, sc, span_bytes, ct, bytes, d_perm, gran, to);
        break;
      }
      case TUTTI_SCATTER_WG_PIECE:
        hipLaunchKernelGGL((k_scatter_piece<true, 3>), dim3(static_cast<uint32_t>(pieces < cap ? pieces : cap)),
                           dim3(kWgThreads), 0, s, sc, span_bytes, ct, bytes, d_perm, gran, to);
        break;
      case TUTTI_SCATTER_WG_PIECE_PLAIN:
        hipLaunchKernelGGL((k_scatter_piece<true, 0>), dim3(static_cast<uint32_t>(pieces < cap ? pieces : cap)),
                           dim3(kWgThreads), 0, s, sc, span_bytes, ct, bytes, d_perm, gran, to);
        break;
      case TUTTI_SCATTER_WG_PIECE_NT_LOADS:
        hipLaunchKernelGGL((k_scatter_piece<true, 1>), dim3(static_cast<uint32_t>(pieces < cap ? pieces : cap)),
                           dim3(kWgThreads), 0, s, sc, span_bytes, ct, bytes, d_perm, gran, to);
        break;
      case TUTTI_SCATTER_WG_PIECE_NT_STORES:
        hipLaunchKernelGGL((k_scatter_piece<true, 2>), dim3(static_cast<uint32_t>(pieces < cap ? pieces : cap)),
                           dim3(kWgThreads), 0, s, sc, span_bytes, ct, bytes, d_perm, gran, to);
        break;
      default:
        return TUTTI_EINVAL;
    }
  }
  hipError_t e = hipGetLastError();
  return e == hipSuccess ? TUTTI_OK : hip_fail(e);
}

int tutti_host_cost_of_restore(const tutti_pool *pool, const tutti_objcfg *cfg, const uint32_t *d_n_blocks,
                               uint32_t n_req, const uint32_t *d_block_table, uint32_t table_len,
                               const uint32_t *d_file_id, uint32_t layer, const void *d_stage, uint64_t stage_cap,
                               uint64_t stage_addr, uint32_t sgl_id, tutti_extent *d_extents, uint64_t *d_totals,
                               tutti_sqe *d_sqe, uint32_t sqe_cap, uint32_t cu_budget, uint32_t *d_status,
                               void *stream, uint32_t n_calls, double *host_ns_per_call) {
  if (n_calls == 0 || !host_ns_per_call) return TUTTI_EINVAL;
  const auto t0 = std::chrono::steady_clock::now();
  for (uint32_t i = 0; i < n_calls; ++i) {
    const int rc = tutti_layer_restore(pool, cfg, d_n_blocks, n_req, d_block_table, table_len, d_file_id, layer,
                                       d_stage, stage_cap, stage_addr, sgl_id, d_extents, d_totals, d_sqe, sqe_cap,
                                       cu_budget, d_status, stream);
    if (rc) return rc;
  }
  const auto t1 = std::chrono::steady_clock::now();
  *host_ns_per_call = std::chrono::duration<double, std::nano>(t1 - t0).count() / n_calls;
  return TUTTI_OK;
}

int tutti_set_tuning(uint32_t wgs_per_cu, uint32_t unroll) {
  if (unroll != 0 && unroll != 1 && unroll != 2 && unroll != 4 && unroll != 8) return TUTTI_EINVAL;
  if (wgs_per_cu > 1024) return TUTTI_ERANGE;
  t_tuning.wgs_per_cu = wgs_per_cu;
  t_tuning.unroll = unroll;
  return TUTTI_OK;
}

int tutti_set_hnd_mode(uint32_t mode) {
  if (mode > 2u) return TUTTI_EINVAL;
  t_tuning.hnd_mode = mode;
  return TUTTI_OK;
}

int tutti_set_xcd_mapping(uint32_t contiguous) {
  t_tuning.xcd_contiguous = contiguous ? 1u : 0u;
  return TUTTI_OK;
}

int tutti_set_nontemporal(uint32_t mask) {
  if (mask > 3u) return TUTTI_EINVAL;
  t_tuning.nontemporal = mask;
  return TUTTI_OK;
}
#endif  // TUTTI_BENCH_BUILD

int tutti_io_domain_create(uint32_t n_cus, void **stream) {
  if (!stream) return TUTTI_EINVAL;
  *stream = nullptr;
  const int cus = cu_count();
  if (cus < 0) return cus;
  if (n_cus == 0 || n_cus > static_cast<uint32_t>(cus)) return TUTTI_ERANGE;
  // one bit per compute unit, the first n_cus of them: the only kind of mask every runtime tried so far accepts
  constexpr uint32_t kWords = 32;  // room for 1024 compute units
  uint32_t mask[kWords] = {0};
  if (static_cast<uint32_t>(cus) > 32u * kWords) return TUTTI_ERANGE;
  for (uint32_t i = 0; i < n_cus; ++i) mask[i / 32] |= 1u << (i % 32);
  const uint32_t words = (static_cast<uint32_t>(cus) + 31u) / 32u;
  hipStream_t s = nullptr;
  const hipError_t e = hipExtStreamCreateWithCUMask(&s, words, mask);
  if (e != hipSuccess) return hip_fail(e);
  *stream = s;
  return TUTTI_OK;
}

int tutti_io_domain_destroy(void *stream) {
  if (!stream) return TUTTI_EINVAL;
  const hipError_t e = hipStreamDestroy(static_cast<hipStream_t>(stream));
  return e == hipSuccess ? TUTTI_OK : hip_fail(e);
}

const char *tutti_strerror(int code) {
  switch (code) {
    case TUTTI_OK:
      return "ok";
    case TUTTI_EINVAL:
      return "invalid argument (null pointer, zero dimension, bad alignment, layout, opcode or layer)";
    case TUTTI_ERANGE:
      return "out of range (too many requests, CU budget above the CU count, table too long, workspace too small, or "
             "more pool blocks than the static bitmap of tutti_table_validate_static covers)";
    case TUTTI_EHIP:
      return "a HIP call failed (see tutti_last_hip_error)";
    case TUTTI_EAGAIN:
      return "not now (too few free IOCBs, or no compute-unit budget fits the slack window)";
    default:
      return "unknown tutti error code";
  }
}

int tutti_last_hip_error(void) { return t_last_hip; }

int tutti_resident_wgs_per_cu(uint32_t which) {
  // the default (unroll 4, non-temporal, 256-thread) instantiation of each data-moving kernel, with the dynamic LDS
  // of a single-request launch (and a full 16 KiB tile + padding for the LDS-staged kernels)
  const uint32_t lds = req_lds_bytes(1);
  const uint32_t lds_tile = align16(lds) + kHndTileCap + kHndTileCap / 8;
  int n = 0;
  hipError_t e;
  switch (which) {
    case 0: e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, k_layer<kUnpack, false, 4, 3, kWgThreads>, kWgThreads, lds); break;
    case 1: e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, k_layer<kPack, false, 4, 3, kWgThreads>, kWgThreads, lds); break;
    case 2: e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, k_move<kUnpack, false, 4, 3, kWgThreads>, kWgThreads, lds); break;
    case 3: e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, k_move<kPack, false, 4, 3, kWgThreads>, kWgThreads, lds); break;
    case 4: e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, k_layer_ring<kUnpack, 4, kWgThreads>, kWgThreads, lds); break;
    case 5: e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, k_layer_ring<kPack, 4, kWgThreads>, kWgThreads, lds); break;
    case 6: e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, k_layer<kUnpack, true, 4, 3, kWgThreads>, kWgThreads, lds); break;
    case 7: e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, k_layer<kPack, true, 4, 3, kWgThreads>, kWgThreads, lds); break;
    case 8: e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, k_layer_lds<kUnpack, 4, kWgThreads>, kWgThreads, lds_tile); break;
    case 9: e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, k_layer_lds<kPack, 4, kWgThreads>, kWgThreads, lds_tile); break;
    case 10: e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, k_issue_io<4, kWgThreads>, kWgThreads, 0); break;
    default: return TUTTI_EINVAL;
  }
  return e == hipSuccess ? n : hip_fail(e);
}

int tutti_cu_count(void) { return cu_count(); }

uint32_t tutti_version(void) { return 0x00000100u; }

int tutti_abi_describe(uint32_t *out, uint32_t cap) {
  if (!out || cap < 52) return TUTTI_EINVAL;
  uint32_t i = 0;
  out[i++] = sizeof(tutti_extent);
  out[i++] = offsetof(tutti_extent, stage_off);
  out[i++] = offsetof(tutti_extent, obj_bytes);
  out[i++] = offsetof(tutti_extent, n_blocks);
  out[i++] = offsetof(tutti_extent, n_chunks);
  out[i++] = offsetof(tutti_extent, sqe_base);
  out[i++] = offsetof(tutti_extent, table_off);
  out[i++] = sizeof(tutti_sqe);
  out[i++] = offsetof(tutti_sqe, opcode);
  out[i++] = offsetof(tutti_sqe, kind);
  out[i++] = offsetof(tutti_sqe, layer);
  out[i++] = offsetof(tutti_sqe, file_id);
  out[i++] = offsetof(tutti_sqe, file_off);
  out[i++] = offsetof(tutti_sqe, addr);
  out[i++] = offsetof(tutti_sqe, len);
  out[i++] = offsetof(tutti_sqe, sgl_id);
  out[i++] = offsetof(tutti_sqe, user_data);
  out[i++] = offsetof(tutti_sqe, iocb_idx);
  out[i++] = offsetof(tutti_sqe, ioctx_slot);
  out[i++] = sizeof(tutti_pool);
  out[i++] = offsetof(tutti_pool, k_base);
  out[i++] = offsetof(tutti_pool, v_base);
  out[i++] = offsetof(tutti_pool, block_stride);
  out[i++] = offsetof(tutti_pool, num_blocks);
  out[i++] = offsetof(tutti_pool, block_tokens);
  out[i++] = offsetof(tutti_pool, num_kv_heads);
  out[i++] = offsetof(tutti_pool, head_dim);
  out[i++] = offsetof(tutti_pool, elt_bytes);
  out[i++] = offsetof(tutti_pool, pool_layout);
  out[i++] = sizeof(tutti_objcfg);
  out[i++] = offsetof(tutti_objcfg, align);
  out[i++] = offsetof(tutti_objcfg, chunk_bytes);
  out[i++] = offsetof(tutti_objcfg, num_layers);
  out[i++] = sizeof(tutti_sgl);
  out[i++] = offsetof(tutti_sgl, addr);
  out[i++] = offsetof(tutti_sgl, len);
  out[i++] = offsetof(tutti_sgl, id);
  out[i++] = sizeof(tutti_iocb_hdr);
  out[i++] = offsetof(tutti_iocb_hdr, iocb_idx);
  out[i++] = offsetof(tutti_iocb_hdr, num_ioctx);
  out[i++] = offsetof(tutti_iocb_hdr, state);
  out[i++] = offsetof(tutti_iocb_hdr, done);
  out[i++] = offsetof(tutti_iocb_hdr, layer);
  out[i++] = offsetof(tutti_iocb_hdr, opcode);
  out[i++] = sizeof(tutti_iocb);
  out[i++] = offsetof(tutti_iocb, ioctx);
  out[i++] = sizeof(tutti_cq_hdr);
  out[i++] = sizeof(tutti_filestore);
  out[i++] = offsetof(tutti_filestore, base);
  out[i++] = offsetof(tutti_filestore, file_stride);
  out[i++] = offsetof(tutti_filestore, first_file_id);
  out[i++] = offsetof(tutti_filestore, n_files);
  return static_cast<int>(i);
}

}  // extern "C"
