// Device code of libtutti for gfx950 (wave64).  Included once, by tutti_api.hip.
//
// Kernels
//   k_layout        one wavefront: extents of all requests by a wave-level prefix scan
//   k_sqe           submission entries from extents, four lanes per 64-byte entry
//   k_move          pack / unpack between paged blocks and objects, extents given
//   k_move_lds      the same for head-major pools with short rows: token tile transposed in LDS
//   k_layer         one layer's restore (or save) in one launch: scan + entries + unpack (or pack)
//   k_layer_lds     the same with the LDS-staged transpose
//   k_sgl_table     direct-to-block mode: the pool's mapping table, one 16-byte descriptor per block
//   k_sqe_direct    one entry per (hit block, K|V), naming the block's descriptor: no staging copy
//   k_ring_init, k_iocb_fill, k_issue_io, k_complete, k_cq_check
//                   SQ/CQ rings: IOCBs filled by the GPU, the entry-driven I/O kernel, completions
//   k_layer_ring    one layer through the rings in one launch: scan + IOCB fill + the blocks' I/O
//   k_copy, k_stream, k_scatter, k_scatter_piece   (measurement build only) plain copy, one-direction streams and
//                   copies with one side permuted at a given granularity: ceilings and floors for the above
//   k_table_validate  debugging aid: ids in range and no id twice, by all-pairs comparison (no workspace)
//   k_bitmap_clear, k_table_validate_bitmap   the same check in linear time with one bit per pool block
//
// Every workgroup first puts the per-request offsets into LDS (from the extents, or by redoing
// the scan), then walks work items with a persistent grid-stride loop, so the grid can be any
// size: the whole GPU, or a few compute units' worth when the caller sets a CU budget.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "tutti.h"

namespace tutti {

constexpr uint32_t kWave = 64;
constexpr uint32_t kWgThreads = 256;         // whole-GPU launches: 8 such workgroups per CU
constexpr uint32_t kBudgetWgThreads = 1024;  // CU-budgeted launches: one 16-wave workgroup per budgeted CU

// Wavefronts per SIMD the register allocator must leave room for: the whole-GPU grids are sized for eight
// 256-thread workgroups per CU being resident at once (a kernel that needs more than 64 VGPRs would hold only
// seven, and the persistent workgroups beyond that would run after the others: a tail).  Asked for where it
// costs no spills: 256-thread kernels with at most four 16-byte units in flight per lane.
constexpr int min_waves_per_simd(int wg_threads, int units) { return (wg_threads == 256 && units <= 4) ? 8 : 4; }

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// A wave-uniform 32-bit value moved to a scalar register.
__device__ __forceinline__ uint32_t rfl(uint32_t v) { return static_cast<uint32_t>(__builtin_amdgcn_readfirstlane(v)); }

// NT is a bit mask: bit 0 = non-temporal loads, bit 1 = non-temporal stores.
template <int NT>
__device__ __forceinline__ u32x4 ld16(const unsigned char *p) {
  if (NT & 1) return __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(p));
  return *reinterpret_cast<const u32x4 *>(p);
}
template <int NT>
__device__ __forceinline__ void st16(unsigned char *p, u32x4 v) {
  if (NT & 2)
    __builtin_nontemporal_store(v, reinterpret_cast<u32x4 *>(p));
  else
    *reinterpret_cast<u32x4 *>(p) = v;
}


// ------------------------------------------------------------------------------------------
// Per-request offsets in LDS.  Laid out in the dynamic LDS block as
//   u64 stage_off[R] | u64 obj_bytes[R] | u32 table_off[R+1] | u32 sqe_base[R+1]
// with the totals in the two sentinel slots.  24*R + 8 bytes.
// blk_off[r] is the number of blocks of the requests before r that the call moves: the copy loops number their
// work items by it.  When the library computed the extents itself it is the table offset (same array); a copy
// kernel that was handed extents keeps it in the sqe_base array, which it has no other use for.
// ------------------------------------------------------------------------------------------
struct ReqLds {
  uint64_t *stage_off;
  uint64_t *obj_bytes;
  uint32_t *table_off;
  uint32_t *sqe_base;
  uint32_t *blk_off;
};

__device__ __forceinline__ ReqLds carve_lds(unsigned char *smem, uint32_t n_req, bool caller_extents = false) {
  ReqLds l;
  l.stage_off = reinterpret_cast<uint64_t *>(smem);
  l.obj_bytes = l.stage_off + n_req;
  l.table_off = reinterpret_cast<uint32_t *>(l.obj_bytes + n_req);
  l.sqe_base = l.table_off + n_req + 1;
  l.blk_off = caller_extents ? l.sqe_base : l.table_off;
  return l;
}

__host__ __device__ constexpr uint32_t req_lds_bytes(uint32_t n_req) { return 24u * n_req + 8u; }

__device__ __forceinline__ uint64_t shfl_up_u64(uint64_t v, uint32_t delta) {
  uint32_t lo = __shfl_up(static_cast<uint32_t>(v), delta, kWave);
  uint32_t hi = __shfl_up(static_cast<uint32_t>(v >> 32), delta, kWave);
  return (static_cast<uint64_t>(hi) << 32) | lo;
}

__device__ __forceinline__ uint64_t shfl_u64(uint64_t v, uint32_t src) {
  uint32_t lo = __shfl(static_cast<uint32_t>(v), src, kWave);
  uint32_t hi = __shfl(static_cast<uint32_t>(v >> 32), src, kWave);
  return (static_cast<uint64_t>(hi) << 32) | lo;
}

// Inclusive prefix sums of three values at once over the first `active` lanes of the wavefront (the other lanes
// hold zeros and their results are not used).  One loop for the three sums keeps their cross-lane moves
// independent and back to back, and only ceil(log2(active)) steps are taken: a single request needs none.
__device__ __forceinline__ void wave_inclusive_scan3(uint64_t &a, uint64_t &b, uint64_t &c, uint32_t lane,
                                                     uint32_t active) {
  for (uint32_t d = 1; d < active; d <<= 1) {
    const uint64_t ta = shfl_up_u64(a, d), tb = shfl_up_u64(b, d), tc = shfl_up_u64(c, d);
    if (lane >= d) {
      a += ta;
      b += tb;
      c += tc;
    }
  }
}

// The file store of the direct-to-block mode: file f at base + (f - first_file_id)*file_stride.
struct FileArgs {
  uint64_t file_stride;
  uint32_t first_file_id;
  uint32_t n_files;
};

constexpr uint64_t kNoFile = ~0ull;

struct ScanGeom {
  uint32_t block_bytes;
  uint32_t align;       // power of two
  uint32_t chunk_bytes; // multiple of align
};

// Extents of all requests, computed by ONE wavefront (the caller passes lane = its lane id and
// makes sure only one wave of the workgroup runs this).  64 requests per pass, running totals
// carried between passes.  Results go to LDS and, when ext_out != nullptr, to global memory.
// In the staged mode (file_id == nullptr) the requests are taken in order while the running sum of
// their blocks stays within table_len: the request that pushes it beyond, and every later one, gets no
// work items (its LDS table offset is the cut, so it owns no blocks) and TUTTI_ST_BAD_EXTENT is reported
// by the workgroup that publishes.  The published extents are the plain sums either way.
__device__ __forceinline__ void wave_scan_extents(const ScanGeom g, const uint32_t *__restrict__ n_blocks, uint32_t n_req,
                                                  uint32_t lane, ReqLds l, tutti_extent *__restrict__ ext_out,
                                                  uint64_t *__restrict__ totals_out, uint32_t table_len,
                                                  uint32_t *__restrict__ status, bool with_chunks = true,
                                                  const uint32_t *__restrict__ file_id = nullptr,
                                                  const FileArgs files = FileArgs{0, 0, 0}) {
  uint64_t carry_stage = 0, carry_sqe = 0, carry_tab = 0;
  bool cut_found = false;   // wave-uniform: some request so far ran beyond the table
  uint32_t cut_total = 0;   // blocks of the requests in front of the first such request
  for (uint32_t base = 0; base < n_req; base += kWave) {
    const uint32_t r = base + lane;
    const uint32_t n = (r < n_req) ? n_blocks[r] : 0u;
    // direct-to-block mode: the per-request slot that holds the staging offset holds the start of the request's
    // file in the store instead (kNoFile if the store has no such file); the published extents are unaffected
    const uint32_t fid = (file_id && r < n_req) ? file_id[r] : 0u;
    const uint64_t raw = static_cast<uint64_t>(n) * g.block_bytes;
    const uint64_t obj = (raw + (g.align - 1)) & ~static_cast<uint64_t>(g.align - 1);
    // a workgroup that only moves blocks never reads the entry bases: it skips the 64-bit division
    const uint64_t chunks = with_chunks ? (obj + g.chunk_bytes - 1) / g.chunk_bytes : 0;
    const uint32_t active = n_req - base < kWave ? n_req - base : kWave;  // requests of this pass
    uint64_t inc_stage = 2 * obj, inc_sqe = 2 * chunks, inc_tab = n;
    wave_inclusive_scan3(inc_stage, inc_sqe, inc_tab, lane, active);
    const bool beyond = !file_id && r < n_req && carry_tab + inc_tab > table_len;
    const uint64_t beyond_mask = __ballot(beyond);
    if (!cut_found && beyond_mask != 0) {
      const uint32_t first = static_cast<uint32_t>(__ffsll(static_cast<long long>(beyond_mask))) - 1u;
      cut_total = static_cast<uint32_t>(carry_tab + shfl_u64(inc_tab - n, first));
      cut_found = true;
    }
    if (r < n_req) {
      const uint64_t stage_off = carry_stage + inc_stage - 2 * obj;
      const uint32_t sqe_base = static_cast<uint32_t>(carry_sqe + inc_sqe - 2 * chunks);
      const uint32_t table_off = static_cast<uint32_t>(carry_tab + inc_tab - n);
      const uint32_t rel = fid - files.first_file_id;
      const bool has_file = fid >= files.first_file_id && rel < files.n_files;
      l.stage_off[r] = !file_id ? stage_off : has_file ? static_cast<uint64_t>(rel) * files.file_stride : kNoFile;
      l.obj_bytes[r] = obj;
      l.table_off[r] = beyond ? cut_total : table_off;
      l.sqe_base[r] = sqe_base;
      if (ext_out) {
        tutti_extent e;
        e.stage_off = stage_off;
        e.obj_bytes = obj;
        e.n_blocks = n;
        e.n_chunks = static_cast<uint32_t>(chunks);
        e.sqe_base = sqe_base;
        e.table_off = table_off;
        ext_out[r] = e;
      }
    }
    carry_stage += shfl_u64(inc_stage, active - 1);  // the pass total sits in its last active lane
    carry_sqe += shfl_u64(inc_sqe, active - 1);
    carry_tab += shfl_u64(inc_tab, active - 1);
  }
  if (lane == 0) {
    l.table_off[n_req] = cut_found ? cut_total : static_cast<uint32_t>(carry_tab);
    l.sqe_base[n_req] = static_cast<uint32_t>(carry_sqe);
    if (totals_out) {
      totals_out[0] = carry_stage;
      totals_out[1] = carry_sqe;
    }
    if (cut_found && totals_out && status) atomicOr(status, TUTTI_ST_BAD_EXTENT);
  }
}

// Per-request offsets for the entry builders, from extents the caller already has (workgroup-wide, with
// barriers).  The entry builders number entries by sqe_base (or by twice table_off in the direct-to-block mode)
// and take a request's chunk and block counts from the differences of consecutive offsets, which is right for
// extents as tutti_obj_layout writes them for exactly these requests: offsets running from 0 without gaps, sizes
// that follow from n_blocks.  That is checked here, every request against its successor; the result is the same
// in every workgroup.  Returns false (after reporting TUTTI_ST_BAD_EXTENT once) if the extents are anything else:
// the caller then writes nothing.
template <int WG>
__device__ __forceinline__ bool lds_from_extents(const tutti_extent *__restrict__ ext, uint32_t n_req, ReqLds l,
                                                 const ScanGeom g, uint32_t *__restrict__ status) {
  // Called by workgroups of WG threads: thread t holds requests t, t + WG, ... (at most kPer of them).  The loop is
  // fully unrolled so that a thread's loads are all in flight together; a request's successor sits in the next
  // lane, and for the last lane of a wavefront in LDS once the barrier has been crossed.  Every workgroup of an
  // entry builder runs this over all requests, so its instruction count matters when there are thousands of
  // both: the host then launches few, large workgroups (entry_launch in the host code).
  constexpr uint32_t kPer = TUTTI_MAX_REQ / WG;
  const uint32_t lane = threadIdx.x & (kWave - 1);
  bool bad = false;
  uint32_t nx_sqe[kPer], nx_tab[kPer];
#pragma unroll
  for (uint32_t k = 0; k < kPer; ++k) {
    const uint32_t r = k * WG + threadIdx.x;
    tutti_extent e;
    e.stage_off = e.obj_bytes = 0;
    e.n_blocks = e.n_chunks = e.sqe_base = e.table_off = 0;
    if (r < n_req) e = ext[r];
    uint64_t next_sqe = 0, next_tab = 0;
    if (r < n_req) {
      l.stage_off[r] = e.stage_off;
      l.obj_bytes[r] = e.obj_bytes;
      l.table_off[r] = e.table_off;
      l.sqe_base[r] = e.sqe_base;
      const uint64_t raw = static_cast<uint64_t>(e.n_blocks) * g.block_bytes;
      const uint64_t obj = (raw + (g.align - 1)) & ~static_cast<uint64_t>(g.align - 1);
      // n_chunks == ceil(obj / chunk_bytes), without the 64-bit division: c*chunk >= obj > (c-1)*chunk
      const uint32_t c = e.n_chunks;
      const bool chunks_ok = obj == 0 ? c == 0
                                      : (c >= 1 && static_cast<uint64_t>(c) * g.chunk_bytes >= obj &&
                                         static_cast<uint64_t>(c - 1) * g.chunk_bytes < obj);
      bad = bad || e.obj_bytes != obj || !chunks_ok;
      // 64-bit sums: offsets that would wrap around 32 bits are not dense either
      next_sqe = static_cast<uint64_t>(e.sqe_base) + 2ull * e.n_chunks;
      next_tab = static_cast<uint64_t>(e.table_off) + e.n_blocks;
      bad = bad || next_sqe > 0xffffffffull || next_tab > 0xffffffffull;
      if (r == 0) bad = bad || e.sqe_base != 0 || e.table_off != 0;
      if (r + 1 == n_req) {
        l.table_off[n_req] = static_cast<uint32_t>(next_tab);
        l.sqe_base[n_req] = static_cast<uint32_t>(next_sqe);
      }
    }
    nx_sqe[k] = static_cast<uint32_t>(next_sqe);
    nx_tab[k] = static_cast<uint32_t>(next_tab);
    // the successor's offsets, from the next lane (every lane takes part in the exchange)
    const uint32_t f_sqe = static_cast<uint32_t>(__shfl_down(static_cast<int>(e.sqe_base), 1, kWave));
    const uint32_t f_tab = static_cast<uint32_t>(__shfl_down(static_cast<int>(e.table_off), 1, kWave));
    if (r + 1 < n_req && lane != kWave - 1) bad = bad || f_sqe != nx_sqe[k] || f_tab != nx_tab[k];
  }
  if (n_req == 0 && threadIdx.x == 0) {
    l.table_off[0] = 0;
    l.sqe_base[0] = 0;
  }
  __syncthreads();  // publishes the LDS writes above
  if (lane == kWave - 1) {
#pragma unroll
    for (uint32_t k = 0; k < kPer; ++k) {
      const uint32_t r = k * WG + threadIdx.x;
      if (r + 1 < n_req) bad = bad || l.sqe_base[r + 1] != nx_sqe[k] || l.table_off[r + 1] != nx_tab[k];
    }
  }
  const bool any_bad = __syncthreads_or(bad ? 1 : 0) != 0;
  if (any_bad && blockIdx.x == 0 && threadIdx.x == 0 && status) atomicOr(status, TUTTI_ST_BAD_EXTENT);
  return !any_bad;
}

__device__ __forceinline__ uint64_t wave_inclusive_scan(uint64_t a, uint32_t lane, uint32_t active) {
  for (uint32_t d = 1; d < active; d <<= 1) {
    const uint64_t t = shfl_up_u64(a, d);
    if (lane >= d) a += t;
  }
  return a;
}

// Per-request offsets for the copy kernels, from extents the caller hands in: every field is honoured as it
// stands (a gap between requests, any order in the staging buffer, a table range that does not start at 0), and
// what cannot be honoured is taken out here, once, so that the copy loop never sees it:
//   - requests are taken in order while the running sum of n_blocks stays within table_len; the request that
//     pushes it beyond and every later one get no work items (TUTTI_ST_BAD_EXTENT);
//   - a request whose stage_off or obj_bytes is not a multiple of 16 (TUTTI_ST_BAD_EXTENT), or whose two objects
//     do not fit in stage_cap (TUTTI_ST_STAGE_CAP), keeps its work items but gets a zero-sized object, so the
//     copy loop skips every block of it;
//   - blocks that would end beyond their object are skipped by the copy loop (TUTTI_ST_BAD_EXTENT).
// All threads stage the raw fields, then the first wavefront scans n_blocks (64 requests per pass) into
// blk_off[], the numbering of the work items.  Workgroup 0 reports.
__device__ __forceinline__ void lds_from_caller_extents(const tutti_extent *__restrict__ ext, uint32_t n_req, ReqLds l,
                                                        uint32_t table_len, uint32_t block_bytes, uint64_t stage_cap,
                                                        uint32_t *__restrict__ status) {
  for (uint32_t r = threadIdx.x; r < n_req; r += blockDim.x) {
    const tutti_extent e = ext[r];
    l.stage_off[r] = e.stage_off;
    l.obj_bytes[r] = e.obj_bytes;
    l.table_off[r] = e.table_off;
    l.blk_off[r] = e.n_blocks;  // replaced by its exclusive prefix sum below
  }
  __syncthreads();
  if (threadIdx.x < kWave) {
    const uint32_t lane = threadIdx.x;
    uint64_t carry = 0;
    bool cut_found = false;
    uint32_t cut_total = 0, flags = 0;
    for (uint32_t base = 0; base < n_req; base += kWave) {
      const uint32_t r = base + lane;
      const uint32_t active = n_req - base < kWave ? n_req - base : kWave;
      const uint32_t n = r < n_req ? l.blk_off[r] : 0u;
      const uint64_t incl = carry + wave_inclusive_scan(n, lane, active);
      const bool beyond = r < n_req && incl > table_len;
      const uint64_t beyond_mask = __ballot(beyond);
      if (!cut_found && beyond_mask != 0) {
        const uint32_t first = static_cast<uint32_t>(__ffsll(static_cast<long long>(beyond_mask))) - 1u;
        cut_total = static_cast<uint32_t>(shfl_u64(incl - n, first));
        cut_found = true;
      }
      if (r < n_req) {
        const uint64_t so = l.stage_off[r], ob = l.obj_bytes[r];
        bool dead = true;
        if (beyond)
          flags |= TUTTI_ST_BAD_EXTENT;
        else if (((so | ob) & 15u) != 0)
          flags |= TUTTI_ST_BAD_EXTENT;
        else if (so > stage_cap || ob > (stage_cap - so) / 2)
          flags |= TUTTI_ST_STAGE_CAP;
        else {
          dead = false;
          if (static_cast<uint64_t>(n) * block_bytes > ob) flags |= TUTTI_ST_BAD_EXTENT;
        }
        if (dead) {
          l.stage_off[r] = 0;
          l.obj_bytes[r] = 0;
        }
        l.blk_off[r] = beyond ? cut_total : static_cast<uint32_t>(incl - n);
      }
      carry = shfl_u64(incl, active - 1);
    }
    if (lane == 0) l.blk_off[n_req] = cut_found ? cut_total : static_cast<uint32_t>(carry);
    if (flags != 0 && blockIdx.x == 0 && status) atomicOr(status, flags);
  }
  __syncthreads();
}

// Largest r in [0, n) with a[r] <= key, for a non-decreasing a with a[0] <= key.  Empty
// requests share their offset with the next one, so the answer is never an empty request
// when key is below the total.
__device__ __forceinline__ uint32_t find_owner(const uint32_t *a, uint32_t n, uint32_t key) {
  uint32_t lo = 0, hi = n;
  while (hi - lo > 1) {
    const uint32_t mid = (lo + hi) >> 1;
    if (a[mid] <= key)
      lo = mid;
    else
      hi = mid;
  }
  return lo;
}

// ------------------------------------------------------------------------------------------
// Submission entries.  Four consecutive lanes write the four 16-byte quarters of one 64-byte
// entry, so a wavefront's store covers 16 whole entries = 1 KiB of consecutive bytes.
// ------------------------------------------------------------------------------------------
struct SqeArgs {
  const uint32_t *file_id;
  tutti_sqe *sqe;
  uint32_t *status;
  uint64_t stage_addr;
  uint32_t sqe_cap;
  uint32_t chunk_bytes;
  uint32_t layer;
  uint32_t opcode;
  uint32_t sgl_id;
};

// Quarter `part` (16 bytes) of entry i, which belongs to request r whose file id is fid.
__device__ __forceinline__ u32x4 sqe_quarter(const SqeArgs &a, const ReqLds &l, uint32_t r, uint32_t i, uint32_t part,
                                             uint32_t fid) {
  const uint32_t base = l.sqe_base[r];
  const uint32_t n_chunks = (l.sqe_base[r + 1] - base) >> 1;
  const uint32_t v = i - base;
  const uint32_t kind = v >= n_chunks ? 1u : 0u;
  const uint32_t c = v - kind * n_chunks;
  const uint64_t obj = l.obj_bytes[r];
  const uint64_t in_obj = static_cast<uint64_t>(c) * a.chunk_bytes;
  u32x4 w = {0u, 0u, 0u, 0u};
  if (part == 0) {
    const uint64_t file_off = (2ull * a.layer + kind) * obj + in_obj;
    w.x = (a.opcode & 0xffu) | (kind << 8) | (a.layer << 16);
    w.y = fid;
    w.z = static_cast<uint32_t>(file_off);
    w.w = static_cast<uint32_t>(file_off >> 32);
  } else if (part == 1) {
    const uint64_t addr = a.stage_addr + l.stage_off[r] + kind * obj + in_obj;
    const uint64_t left = obj - in_obj;
    w.x = static_cast<uint32_t>(addr);
    w.y = static_cast<uint32_t>(addr >> 32);
    w.z = left < a.chunk_bytes ? static_cast<uint32_t>(left) : a.chunk_bytes;
    w.w = a.sgl_id;
  } else if (part == 2) {
    w.x = i;
    w.y = r;
    w.z = i / TUTTI_IOCB_SLOTS;
    w.w = i % TUTTI_IOCB_SLOTS;
  }
  return w;
}

// The entries of a layer are written by the `n_wgs` workgroups starting at workgroup `first_wg`, one lane per
// quarter.  A workgroup that also moves blocks splits the job: sqe_head, right after the scan, finds the owner
// of the lane's first quarter and requests its file id (the only value that comes from global memory);
// emit_sqes, after the copy loop, assembles and stores, so the load's latency is spent under the copy.
struct SqeHead {
  uint64_t q;    // the lane's first quarter
  uint32_t r;    // its request
  uint32_t fid;  // file id of that request (quarter 0 only)
  bool live;     // the lane has a first quarter
};

__device__ __forceinline__ SqeHead sqe_head(const SqeArgs a, const ReqLds l, uint32_t n_req, uint32_t first_wg) {
  const uint32_t n_sqe = l.sqe_base[n_req];
  const uint32_t n_write = n_sqe < a.sqe_cap ? n_sqe : a.sqe_cap;
  SqeHead h;
  h.q = static_cast<uint64_t>(blockIdx.x - first_wg) * blockDim.x + threadIdx.x;
  h.live = h.q < 4ull * n_write;
  h.r = 0;
  h.fid = 0;
  if (h.live) {
    h.r = find_owner(l.sqe_base, n_req, static_cast<uint32_t>(h.q >> 2));
    if ((h.q & 3) == 0) h.fid = a.file_id[h.r];
  }
  return h;
}

__device__ __forceinline__ void emit_sqes(const SqeArgs a, const ReqLds l, uint32_t n_req, uint32_t first_wg,
                                          uint32_t n_wgs, const SqeHead h) {
  const uint32_t n_sqe = l.sqe_base[n_req];
  const uint32_t n_write = n_sqe < a.sqe_cap ? n_sqe : a.sqe_cap;
  const uint32_t wg = blockIdx.x - first_wg;
  if (n_sqe > a.sqe_cap && wg == 0 && threadIdx.x == 0 && a.status) atomicOr(a.status, TUTTI_ST_SQE_CAP);
  if (!h.live) return;
  const uint64_t n_quarters = 4ull * n_write;
  const uint64_t stride = static_cast<uint64_t>(n_wgs) * blockDim.x;
  u32x4 *out = reinterpret_cast<u32x4 *>(a.sqe);
  const uint32_t part = static_cast<uint32_t>(h.q & 3);  // the stride is a multiple of 4: the same quarter every pass
  out[h.q] = sqe_quarter(a, l, h.r, static_cast<uint32_t>(h.q >> 2), part, h.fid);
  for (uint64_t q = h.q + stride; q < n_quarters; q += stride) {
    const uint32_t i = static_cast<uint32_t>(q >> 2);
    const uint32_t r = find_owner(l.sqe_base, n_req, i);
    out[q] = sqe_quarter(a, l, r, i, part, part == 0 ? a.file_id[r] : 0u);
  }
}

// ------------------------------------------------------------------------------------------
// Direct-to-block mode.  The mapping table holds one 16-byte descriptor per pool block; an entry
// then names the descriptor of the block it transfers instead of a staging address.
// ------------------------------------------------------------------------------------------
struct SglArgs {
  tutti_sgl *table;
  uint32_t *status;
  uint64_t k_addr;
  uint64_t v_addr;
  uint64_t block_stride;
  uint32_t num_blocks;
  uint32_t block_bytes;
  uint32_t sgl_id;
  uint32_t cap;
};

__global__ __launch_bounds__(kWgThreads) void k_sgl_table(const SglArgs a) {
  const uint64_t n = 2ull * a.num_blocks;
  if (n > a.cap && blockIdx.x == 0 && threadIdx.x == 0 && a.status) atomicOr(a.status, TUTTI_ST_SQE_CAP);
  const uint64_t n_write = n < a.cap ? n : a.cap;
  const uint64_t stride = static_cast<uint64_t>(gridDim.x) * blockDim.x;
  u32x4 *out = reinterpret_cast<u32x4 *>(a.table);
  for (uint64_t i = static_cast<uint64_t>(blockIdx.x) * blockDim.x + threadIdx.x; i < n_write; i += stride) {
    const bool v_plane = i >= a.num_blocks;
    const uint64_t b = v_plane ? i - a.num_blocks : i;
    const uint64_t addr = (v_plane ? a.v_addr : a.k_addr) + b * a.block_stride;
    u32x4 w;
    w.x = static_cast<uint32_t>(addr);
    w.y = static_cast<uint32_t>(addr >> 32);
    w.z = a.block_bytes;
    w.w = a.sgl_id;
    out[i] = w;  // a wavefront stores 64 descriptors = 1 KiB of consecutive bytes
  }
}

struct DirectArgs {
  const uint32_t *table;
  uint64_t sgl_table_addr;
  uint32_t table_len;
  uint32_t num_blocks;
  uint32_t block_bytes;
};

// Direct-mode entry i in two steps, so that the loads of the next entry can be in flight while the current one
// is assembled.  Step one: where the entry sits in its request, and the two values that come from global
// memory (the block id; the file id for the lane that writes the first quarter).
struct DirectLoc {
  uint32_t r, kind, j;
  uint32_t id;   // block id, or num_blocks when the table has no such position
  uint32_t fid;  // file id of the request (quarter 0 only)
};

__device__ __forceinline__ DirectLoc direct_locate(const SqeArgs &a, const DirectArgs &d, const ReqLds &l, uint32_t r,
                                                   uint32_t i, uint32_t part) {
  DirectLoc c;
  const uint32_t toff = l.table_off[r];
  const uint32_t n = l.table_off[r + 1] - toff;
  const uint32_t v = i - 2u * toff;
  c.r = r;
  c.kind = v >= n ? 1u : 0u;
  c.j = v - c.kind * n;
  const uint32_t tab_idx = toff + c.j;
  c.id = d.num_blocks;
  if (tab_idx < d.table_len) c.id = d.table[tab_idx];  // the four lanes of an entry read the same word
  c.fid = part == 0 ? a.file_id[r] : 0u;
  return c;
}

// Step two: quarter `part` (16 bytes) of the entry.  *bad is set for an id out of range.
__device__ __forceinline__ u32x4 direct_entry_quarter(const SqeArgs &a, const DirectArgs &d, const ReqLds &l,
                                                      const DirectLoc &c, uint32_t i, uint32_t part, bool *bad) {
  const bool ok = c.id < d.num_blocks;
  *bad = !ok;
  u32x4 w = {0u, 0u, 0u, 0u};
  if (part == 0) {
    const uint64_t file_off = (2ull * a.layer + c.kind) * l.obj_bytes[c.r] + static_cast<uint64_t>(c.j) * d.block_bytes;
    w.x = (a.opcode & 0xffu) | (c.kind << 8) | (a.layer << 16);
    w.y = c.fid;
    w.z = static_cast<uint32_t>(file_off);
    w.w = static_cast<uint32_t>(file_off >> 32);
  } else if (part == 1) {
    const uint64_t addr = ok ? d.sgl_table_addr + 16ull * (static_cast<uint64_t>(c.kind) * d.num_blocks + c.id) : 0ull;
    w.x = static_cast<uint32_t>(addr);
    w.y = static_cast<uint32_t>(addr >> 32);
    w.z = ok ? d.block_bytes : 0u;
    w.w = a.sgl_id;
  } else if (part == 2) {
    w.x = i;
    w.y = c.r;
    w.z = i / TUTTI_IOCB_SLOTS;
    w.w = i % TUTTI_IOCB_SLOTS;
  }
  return w;
}

// The request that owns block-table position `key`, found from the owner of an earlier (smaller) position:
// the offsets are non-decreasing, so walking forward gives what find_owner gives.
__device__ __forceinline__ uint32_t advance_owner(const uint32_t *table_off, uint32_t n_req, uint32_t r, uint32_t key) {
  while (r + 1 < n_req && table_off[r + 1] <= key) ++r;
  return r;
}

// Four lanes per entry, as in emit_sqes: a wavefront's store covers 16 whole entries.  The `n_wgs` workgroups
// starting at `first_wg` each take one contiguous run of entries (a whole number of 4 KiB workgroup stores), so a
// thread's consecutive entries are 64 apart and their owner is found by walking on from the previous one: one
// binary search per thread instead of one per entry.  The loop is pipelined by one entry: the table and file-id
// loads of the next entry are issued before the current one is assembled and stored; the first entry's are issued
// by direct_head, which a workgroup that also moves blocks calls before its copy loop.  `dst(i)` gives the
// address of entry i.
struct DirectHead {
  uint64_t q, end;  // the lane's first quarter and the end of its workgroup's run
  DirectLoc loc;    // that quarter's entry, located, with its loads requested
  bool live;
};

__device__ __forceinline__ DirectHead direct_head(const SqeArgs a, const DirectArgs d, const ReqLds l, uint32_t n_req,
                                                  uint64_t n_write, uint32_t first_wg, uint32_t n_wgs) {
  const uint64_t n_quarters = 4ull * n_write;
  const uint64_t per_pass = blockDim.x;  // quarters one workgroup writes per pass: 4 KiB for 256 threads
  const uint64_t passes = (n_quarters + per_pass * n_wgs - 1) / (per_pass * n_wgs);
  const uint64_t begin = static_cast<uint64_t>(blockIdx.x - first_wg) * passes * per_pass;
  DirectHead h;
  h.end = begin + passes * per_pass;
  if (h.end > n_quarters) h.end = n_quarters;
  h.q = begin + threadIdx.x;
  h.live = h.q < h.end;
  if (h.live) {
    const uint32_t i = static_cast<uint32_t>(h.q >> 2);
    h.loc = direct_locate(a, d, l, find_owner(l.table_off, n_req, i >> 1), i, static_cast<uint32_t>(h.q & 3));
  }
  return h;
}

template <typename Dst>
__device__ __forceinline__ void emit_direct_entries(const SqeArgs a, const DirectArgs d, const ReqLds l, uint32_t n_req,
                                                    const DirectHead h, Dst dst) {
  if (!h.live) return;
  const uint64_t per_pass = blockDim.x;
  uint64_t q = h.q;
  uint32_t i = static_cast<uint32_t>(q >> 2);
  const uint32_t part = static_cast<uint32_t>(q & 3);  // per_pass is a multiple of 4: the same quarter every pass
  DirectLoc cur = h.loc;
  for (;;) {
    const uint64_t qn = q + per_pass;
    const bool more = qn < h.end;
    const uint32_t in = static_cast<uint32_t>(qn >> 2);
    DirectLoc nxt = cur;
    if (more) nxt = direct_locate(a, d, l, advance_owner(l.table_off, n_req, cur.r, in >> 1), in, part);
    bool bad = false;
    const u32x4 w = direct_entry_quarter(a, d, l, cur, i, part, &bad);
    if (bad && part == 0 && a.status) atomicOr(a.status, TUTTI_ST_BAD_BLOCK);
    reinterpret_cast<u32x4 *>(dst(i))[part] = w;
    if (!more) break;
    q = qn;
    i = in;
    cur = nxt;
  }
}

__device__ __forceinline__ void emit_direct_sqes(const SqeArgs a, const DirectArgs d, const ReqLds l, uint32_t n_req) {
  const uint64_t n_sqe = 2ull * l.table_off[n_req];
  const uint64_t n_write = n_sqe < a.sqe_cap ? n_sqe : a.sqe_cap;
  if (n_sqe > a.sqe_cap && blockIdx.x == 0 && threadIdx.x == 0 && a.status) atomicOr(a.status, TUTTI_ST_SQE_CAP);
  tutti_sqe *out = a.sqe;
  emit_direct_entries(a, d, l, n_req, direct_head(a, d, l, n_req, n_write, 0, gridDim.x),
                      [out](uint32_t i) { return out + i; });
}

// ------------------------------------------------------------------------------------------
// Rings.  An SQ slot is an IOCB: 64-byte header + 2048 contexts.
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(kWgThreads) void k_ring_init(tutti_iocb *sq, tutti_cq_hdr *cq, uint32_t depth) {
  const uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < depth) {
    u32x4 *h = reinterpret_cast<u32x4 *>(&sq[i].hdr);
    const u32x4 zero = {0u, 0u, 0u, 0u};
    const u32x4 first = {i, 0u, TUTTI_IOCB_FREE, 0u};
    h[0] = first;
    h[1] = zero;
    h[2] = zero;
    h[3] = zero;
    reinterpret_cast<uint32_t *>(cq + 1)[i] = 0xffffffffu;
  }
  if (i < 16) reinterpret_cast<uint32_t *>(cq)[i] = (i == 1) ? depth : 0u;
}

struct RingArgs {
  tutti_iocb *sq;
  tutti_cq_hdr *cq;
  uint32_t depth;
  uint32_t first_slot;
  uint32_t n_slots;
};

// Contexts of one layer dealt into IOCBs (see emit_direct_sqes for the entry itself), plus the headers, by the
// `n_wgs` workgroups starting at workgroup `first_wg`: iocb_head before a copy loop, emit_iocbs after it.
__device__ __forceinline__ uint64_t iocb_fill_count(const RingArgs &g, const ReqLds &l, uint32_t n_req) {
  const uint64_t n_ctx = 2ull * l.table_off[n_req];
  const uint64_t cap = static_cast<uint64_t>(g.n_slots) * TUTTI_IOCB_SLOTS;
  return n_ctx < cap ? n_ctx : cap;
}

__device__ __forceinline__ DirectHead iocb_head(const RingArgs g, const SqeArgs a, const DirectArgs d, const ReqLds l,
                                                uint32_t n_req, uint32_t first_wg, uint32_t n_wgs) {
  return direct_head(a, d, l, n_req, iocb_fill_count(g, l, n_req), first_wg, n_wgs);
}

__device__ __forceinline__ void emit_iocbs(const RingArgs g, const SqeArgs a, const DirectArgs d, const ReqLds l,
                                           uint32_t n_req, uint32_t first_wg, uint32_t n_wgs, const DirectHead h) {
  const uint64_t n_ctx = 2ull * l.table_off[n_req];
  const uint64_t cap = static_cast<uint64_t>(g.n_slots) * TUTTI_IOCB_SLOTS;
  const uint64_t n_fill = iocb_fill_count(g, l, n_req);
  const uint64_t tid = static_cast<uint64_t>(blockIdx.x - first_wg) * blockDim.x + threadIdx.x;
  if (n_ctx > cap && tid == 0 && a.status) atomicOr(a.status, TUTTI_ST_SQE_CAP);
  const uint64_t stride = static_cast<uint64_t>(n_wgs) * blockDim.x;
  for (uint64_t b = tid; b < g.n_slots; b += stride) {  // one thread per IOCB header
    const uint64_t lo = b * TUTTI_IOCB_SLOTS;
    uint64_t cnt = n_fill > lo ? n_fill - lo : 0;
    if (cnt > TUTTI_IOCB_SLOTS) cnt = TUTTI_IOCB_SLOTS;
    tutti_iocb_hdr *hd = &g.sq[(g.first_slot + b) % g.depth].hdr;
    hd->num_ioctx = static_cast<uint32_t>(cnt);
    hd->state = TUTTI_IOCB_FILLED;
    hd->done = 0;
    hd->layer = a.layer;
    hd->opcode = a.opcode;
  }
  const RingArgs ring = g;
  emit_direct_entries(a, d, l, n_req, h, [ring](uint32_t i) {
    return &ring.sq[(ring.first_slot + i / TUTTI_IOCB_SLOTS) % ring.depth].ioctx[i % TUTTI_IOCB_SLOTS];
  });
}

template <int WG>
__global__ __launch_bounds__(WG) void k_iocb_fill(const RingArgs g, const SqeArgs a, const DirectArgs d,
                                                           const ScanGeom geom, const tutti_extent *__restrict__ ext,
                                                           uint32_t n_req) {
  extern __shared__ __align__(16) unsigned char smem[];
  const ReqLds l = carve_lds(smem, n_req);
  if (!lds_from_extents<WG>(ext, n_req, l, geom, a.status)) return;
  emit_iocbs(g, a, d, l, n_req, 0, gridDim.x, iocb_head(g, a, d, l, n_req, 0, gridDim.x));
}

struct IoArgs {
  const tutti_sgl *sgl;
  unsigned char *store_base;
  uint32_t *status;
  uint64_t sgl_table_addr;
  uint64_t file_stride;
  uint32_t n_desc;
  uint32_t first_file_id;
  uint32_t n_files;
  uint32_t max_len;
  uint32_t slices;  // ceil(max_len / slice bytes)
};

// One slice of one context, resolved: where its bytes come from and go to.  Wave-uniform.
struct IoItem {
  const unsigned char *src;  // nullptr: nothing to move (empty slot, no-op or rejected context, slice beyond len)
  unsigned char *dst;
  uint32_t len;              // bytes of the context
  uint32_t in_ctx;           // first byte of the slice within the context
};

// Everything between the item number and the two addresses: IOCB header, context, SGL descriptor, validity.
// Three dependent loads (header and context together, then the descriptor), all of wave-uniform words.
template <int U>
__device__ __forceinline__ IoItem io_decode(const RingArgs &g, const IoArgs &a, uint32_t it, uint32_t per_iocb,
                                            uint32_t lane) {
  constexpr uint32_t kSlice = kWave * 16u * U;
  IoItem r;
  r.src = nullptr;
  r.dst = nullptr;
  r.len = 0;
  const uint32_t b = it / per_iocb;
  const uint32_t rem = it - b * per_iocb;
  const uint32_t k = rem / a.slices;
  const uint32_t s = rem - k * a.slices;
  r.in_ctx = s * kSlice;
  const tutti_iocb *io = &g.sq[(g.first_slot + b) % g.depth];
  const u32x4 hdr = *reinterpret_cast<const u32x4 *>(&io->hdr);  // iocb_idx, num_ioctx, state, done
  const u32x4 *e = reinterpret_cast<const u32x4 *>(&io->ioctx[k]);
  const u32x4 q0 = e[0], q1 = e[1];
  const uint32_t num = rfl(hdr.y), state = rfl(hdr.z);
  if (state != TUTTI_IOCB_FILLED || k >= num) return r;  // nothing submitted in this slot / position
  const uint32_t opcode = rfl(q0.x) & 0xffu;
  const uint32_t file_id = rfl(q0.y);
  const uint64_t file_off = (static_cast<uint64_t>(rfl(q0.w)) << 32) | rfl(q0.z);
  const uint64_t addr = (static_cast<uint64_t>(rfl(q1.y)) << 32) | rfl(q1.x);
  const uint32_t len = rfl(q1.z);
  if (len == 0) return r;  // a no-op context
  bool ok = (opcode == TUTTI_OP_READ || opcode == TUTTI_OP_WRITE) && addr >= a.sgl_table_addr &&
            ((addr - a.sgl_table_addr) & 15u) == 0 && len <= a.max_len && (len & 15u) == 0 && (file_off & 15u) == 0;
  const uint64_t di = ok ? (addr - a.sgl_table_addr) >> 4 : 0;
  ok = ok && di < a.n_desc;
  uint64_t blk_addr = 0;
  if (ok) {
    const u32x4 dsc = *reinterpret_cast<const u32x4 *>(&a.sgl[di]);
    blk_addr = (static_cast<uint64_t>(rfl(dsc.y)) << 32) | rfl(dsc.x);
    ok = len <= rfl(dsc.z) && (blk_addr & 15u) == 0;
  }
  ok = ok && file_id >= a.first_file_id && file_id - a.first_file_id < a.n_files &&
       file_off + len <= a.file_stride && file_off + len >= file_off;
  if (!ok) {
    if (lane == 0 && s == 0 && a.status) atomicOr(a.status, TUTTI_ST_BAD_BLOCK);
    return r;
  }
  if (r.in_ctx >= len) return r;  // the context is shorter than max_len: this slice holds none of it
  unsigned char *blk = reinterpret_cast<unsigned char *>(blk_addr);
  unsigned char *fil = a.store_base + static_cast<uint64_t>(file_id - a.first_file_id) * a.file_stride + file_off;
  const bool rd = opcode == TUTTI_OP_READ;
  r.src = rd ? fil : blk;
  r.dst = rd ? blk : fil;
  r.len = len;
  return r;
}

// The I/O kernel: one wavefront per slice of one context, no inter-wave communication.  Software-pipelined by
// one item: the loads of the current slice are issued, then the next item is resolved (its header, context and
// descriptor loads run under the data loads), then the current slice is stored.  Completion is published by
// k_complete, enqueued right behind it on the same stream: counting finished items with atomics on the IOCB
// header serialises on one address (measured: 1.5 ms per 4096-context layer instead of 55 us), and a kernel
// boundary already is the "all contexts done" event.
__device__ __forceinline__ void complete_iocbs(const RingArgs g, uint32_t lane);  // defined below

// `done`: IOCBs that an earlier launch on the same stream has executed; when done.n_slots is not 0 the grid has one
// workgroup more, in front, whose first wavefront completes them and leaves (see k_layer_ring).
template <int U, int WG>
__global__ __launch_bounds__(WG, min_waves_per_simd(WG, U)) void k_issue_io(const RingArgs g, const RingArgs done,
                                                                             const IoArgs a) {
  constexpr uint32_t kSlice = kWave * 16u * U;
  const uint32_t lane = threadIdx.x & (kWave - 1);
  const uint32_t wave_in_wg = rfl(threadIdx.x / kWave);
  const uint32_t lead = done.n_slots != 0 ? 1u : 0u;
  if (lead && blockIdx.x == 0) {
    if (threadIdx.x < kWave) complete_iocbs(done, threadIdx.x);
    return;
  }
  const uint32_t n_waves = (gridDim.x - lead) * (blockDim.x / kWave);
  const uint32_t per_iocb = TUTTI_IOCB_SLOTS * a.slices;
  const uint32_t n_items = g.n_slots * per_iocb;  // the host checked this fits 32 bits

  uint32_t it = (blockIdx.x - lead) * (blockDim.x / kWave) + wave_in_wg;
  if (it >= n_items) return;
  IoItem cur = io_decode<U>(g, a, it, per_iocb, lane);
  for (;;) {
    const uint32_t nit = it + n_waves;
    const bool more = nit < n_items;
    const bool whole = cur.src != nullptr && cur.in_ctx + kSlice <= cur.len;
    const uint32_t o0 = cur.in_ctx + lane * 16u;
    u32x4 buf[U];
    if (whole) {
#pragma unroll
      for (int u = 0; u < U; ++u) buf[u] = ld16<3>(cur.src + o0 + u * (kWave * 16u));
    }
    IoItem nxt = cur;
    if (more) nxt = io_decode<U>(g, a, nit, per_iocb, lane);
    if (whole) {
#pragma unroll
      for (int u = 0; u < U; ++u) st16<3>(cur.dst + o0 + u * (kWave * 16u), buf[u]);
    } else if (cur.src != nullptr) {  // ragged last slice of a context
      for (int u = 0; u < U; ++u) {
        const uint32_t o = o0 + u * (kWave * 16u);
        if (o < cur.len) st16<3>(cur.dst + o, ld16<3>(cur.src + o));
      }
    }
    if (!more) break;
    cur = nxt;
    it = nit;
  }
}

// Completion of the IOCBs an I/O kernel has executed: FILLED -> DONE, done = num_ioctx, index appended to the CQ
// in slot order.  Run by ONE wavefront (lane = its lane id) once every store of the I/O is visible to it: the
// k_complete kernel enqueued behind the I/O kernel (stream order).  Doing it inside the I/O kernel instead, by
// whichever workgroup finishes last (each workgroup releasing its stores at agent scope and counting itself in
// on a two-level tree of counters), was built and measured: 153 us per layer against 50 + 4: an agent-scope
// release writes back the XCD's whole L2, and 2048 workgroups each pay for one.  The CQ tail is only ever
// advanced here, so no read-modify-write atomics are needed within a stream.  The state and the tail are
// published with system-scope release stores, so a ring (or just its CQ) placed in pinned host memory can be
// polled by the CPU while the stream runs on: whoever sees the new tail also sees the entries before it.
__device__ __forceinline__ void complete_iocbs(const RingArgs g, uint32_t lane) {
  uint32_t *cq_entry = reinterpret_cast<uint32_t *>(g.cq + 1);
  uint32_t tail = g.cq->tail;  // every lane reads the same word
  // one lane per IOCB, 64 per pass (the host checked n_slots <= depth, so the slots are distinct): the header
  // loads of a pass are in flight together, and a ballot gives each executed IOCB its place in the queue
  for (uint32_t base = 0; base < g.n_slots; base += kWave) {
    const uint32_t b = base + lane;
    tutti_iocb_hdr *h = nullptr;
    uint32_t num = 0, idx = 0;
    bool live = false;
    if (b < g.n_slots) {
      h = &g.sq[(g.first_slot + b) % g.depth].hdr;
      live = h->state == TUTTI_IOCB_FILLED;
      num = h->num_ioctx;
      idx = h->iocb_idx;
    }
    const uint64_t mask = __ballot(live);
    const uint32_t before = static_cast<uint32_t>(__popcll(mask & ((1ull << lane) - 1ull)));
    if (live) {
      h->done = num;
      cq_entry[(tail + before) % g.depth] = idx;
      __hip_atomic_store(&h->state, TUTTI_IOCB_DONE, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_SYSTEM);
    }
    tail += static_cast<uint32_t>(__popcll(mask));
  }
  // every lane releases its own queue entries before lane 0 publishes the tail (the wavefront runs in step, so
  // lane 0's store is issued after the other lanes' fences)
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "");  // system scope
  __builtin_amdgcn_wave_barrier();
  if (lane == 0) __hip_atomic_store(&g.cq->tail, tail, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_SYSTEM);
}

__global__ __launch_bounds__(kWave) void k_complete(const RingArgs g) {
  if (blockIdx.x != 0) return;
  complete_iocbs(g, threadIdx.x);
}

// wait_cqe for n slots from `slot` on (wrapping at depth): flag[i] <- 1 if IOCB (slot + i) % depth is DONE, else 0.
__global__ __launch_bounds__(kWgThreads) void k_cq_check(const tutti_iocb *sq, uint32_t depth, uint32_t slot, uint32_t n,
                                                          uint32_t *flag) {
  for (uint32_t i = blockIdx.x * blockDim.x + threadIdx.x; i < n; i += gridDim.x * blockDim.x) {
    const uint32_t st =
        __hip_atomic_load(&sq[(slot + i) % depth].hdr.state, __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_AGENT);
    flag[i] = st == TUTTI_IOCB_DONE ? 1u : 0u;
  }
}

template <int WG>
__global__ __launch_bounds__(WG) void k_sqe_direct(const SqeArgs a, const DirectArgs d, const ScanGeom geom,
                                                            const tutti_extent *__restrict__ ext, uint32_t n_req) {
  extern __shared__ __align__(16) unsigned char smem[];
  const ReqLds l = carve_lds(smem, n_req);
  if (!lds_from_extents<WG>(ext, n_req, l, geom, a.status)) return;
  emit_direct_sqes(a, d, l, n_req);
}

// ------------------------------------------------------------------------------------------
// Pack / unpack.  A work item is one slice of one (block, K|V): kSliceUnits*1 KiB, moved by one
// wavefront with 16-byte accesses per lane (1 KiB per wavefront instruction, whole cache lines
// on both sides).  Items are numbered in staging-buffer order (request, K then V, block, slice),
// so neighbouring wavefronts stream neighbouring object bytes while the pool side jumps from
// block to block as the table says.
// ------------------------------------------------------------------------------------------
struct MoveArgs {
  unsigned char *k_base;
  unsigned char *v_base;
  unsigned char *stage;
  const uint32_t *table;
  uint32_t *status;
  uint64_t block_stride;
  uint64_t stage_cap;
  uint32_t num_blocks;
  uint32_t block_bytes;
  uint32_t table_len;
  uint32_t slices_per_block;
  // head-major pools only: a row is the d*e bytes of one (token, head)
  uint32_t row_bytes;
  uint32_t block_tokens;
  uint32_t num_kv_heads;
  // head-major pools moved through LDS (T, h and the row size are powers of two there):
  // a tile is 2^tile_shift tokens x all heads; slices_per_block then counts tiles
  uint32_t row_shift;    // log2(row_bytes)
  uint32_t head_shift;   // log2(num_kv_heads)
  uint32_t token_shift;  // log2(block_tokens)
  uint32_t tile_shift;   // log2(tokens per tile)
  uint32_t lds_pitch;    // bytes between consecutive tokens of the tile in LDS: h*row_bytes + row_bytes
  // dense staging: blocks are whole alignment units and whole slices, so item `it` of an unpack reads the
  // staging bytes [it*slice, (it+1)*slice) whatever the extents are; items_bound = 2 * table_len * slices
  uint32_t dense;
  uint32_t items_bound;
  // workgroup -> item mapping: 0 = workgroup b starts at item 4b (neighbouring workgroups, which the
  // dispatcher deals round-robin to the 8 XCDs, take neighbouring 16 KiB); 1 = each XCD takes one
  // contiguous eighth of the copy workgroups' items
  uint32_t xcd_contiguous;
  // direct-to-block mode (the rings' one-launch layer path): `stage` is the base of the file store, the
  // per-request staging offsets in LDS hold the start of each request's file in it (kNoFile if the store has no
  // such file), and the object side of (request, kind, block j) is the file offset of the context that
  // emit_iocbs records for it; only the first ctx_cap contexts were recorded and are executed
  uint32_t direct;
  uint32_t layer;
  uint64_t file_stride;
  uint64_t ctx_cap;
  // ordered restore: table positions in the order in which their blocks are to be visited (table_len entries);
  // unit u of the launch is (plane u / table_len, position visit[u % table_len]) instead of staging order
  const uint32_t *visit;
};


// The workgroup index used for item numbering (see MoveArgs::xcd_contiguous).
__device__ __forceinline__ uint32_t item_wg(const MoveArgs &a, uint32_t wg, uint32_t copy_wgs) {
  const uint32_t b = wg;  // index among the copy workgroups
  if (!a.xcd_contiguous || copy_wgs < 16u) return b;
  const uint32_t per = copy_wgs / 8u;            // workgroups per XCD (the remainder keeps its own index)
  if (b >= per * 8u) return b;
  return (b % 8u) * per + b / 8u;
}

constexpr int kPack = 0;   // pool -> object
constexpr int kUnpack = 1; // object -> pool

// Offset inside a head-major block [h][T][row] of the 16 bytes that sit at canonical
// (token-major, [T][h][row]) offset o.
__device__ __forceinline__ uint32_t hnd_offset(uint32_t o, uint32_t row_bytes, uint32_t T, uint32_t h) {
  const uint32_t row = o / row_bytes;
  const uint32_t w = o - row * row_bytes;
  const uint32_t t = row / h;
  const uint32_t i = row - t * h;
  return (i * T + t) * row_bytes + w;
}

// Wave-uniform description of one work item: where its slice sits on the object side and which
// block-table entry names the pool side.
struct Item {
  unsigned char *obj_ptr;  // start of the (request, kind) object; nullptr = skip the item
  unsigned char *obj_blk;  // where block j of it sits on the object side
  uint64_t obj_bytes;
  uint32_t tab_idx;        // index into the block table
  uint32_t n;              // blocks of the request
  uint32_t j;              // block within the request
  uint32_t s;              // slice within the block
  uint32_t kind;
};

// Wave-uniform words (block ids, visiting order) are fetched through the scalar (constant) path: one s_load per
// wavefront, counted apart from the vector loads and stores in flight, so waiting for it does not wait for them.
typedef const __attribute__((address_space(4))) uint32_t *const_u32_ptr;

// SEP: the extents came from the caller (lds_from_caller_extents): items are numbered by blk_off, the table is
// indexed by the request's own table_off, and requests that cannot be honoured already have a zero-sized object.
// ORD: the units are visited in the order a.visit lists (all K blocks, then all V blocks, each in that order);
// a listed position that is not a block of a request that takes part is passed over.
template <bool SEP, bool ORD = false>
__device__ __forceinline__ Item decode_item(const MoveArgs &a, const ReqLds &l, uint32_t n_req, uint32_t it,
                                            uint32_t lane) {
  Item d;
  const uint32_t S = a.slices_per_block;
  const uint32_t u = it / S;  // (block, kind) unit in staging order
  d.s = it - u * S;
  const uint32_t *off = SEP ? l.blk_off : l.table_off;
  uint32_t r, toff;
  if (ORD) {
    d.kind = u >= a.table_len ? 1u : 0u;
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Wold-style-cast"
    const_u32_ptr vis = (const_u32_ptr)a.visit;
#pragma clang diagnostic pop
    const uint32_t pos = vis[rfl(u - d.kind * a.table_len)];  // wave-uniform index: one scalar load
    if (pos >= l.table_off[n_req]) {  // beyond the blocks of the requests that take part
      d.obj_ptr = nullptr;
      d.obj_blk = nullptr;
      d.obj_bytes = 0;
      d.tab_idx = d.n = d.j = 0;
      return d;
    }
    r = find_owner(l.table_off, n_req, pos);
    toff = l.table_off[r];
    d.n = l.table_off[r + 1] - toff;
    d.j = pos - toff;
  } else {
    r = find_owner(off, n_req, u >> 1);
    toff = off[r];
    d.n = off[r + 1] - toff;
    const uint32_t v = u - 2u * toff;
    d.kind = v >= d.n ? 1u : 0u;
    d.j = v - d.kind * d.n;
  }
  d.obj_bytes = l.obj_bytes[r];
  d.tab_idx = (SEP ? l.table_off[r] : toff) + d.j;
  const uint64_t stage_off = l.stage_off[r];
  if (a.direct) {
    // same arithmetic as the context's file offset (direct_entry_quarter), then the I/O kernel's checks
    const uint64_t file_off = (2ull * a.layer + d.kind) * d.obj_bytes + static_cast<uint64_t>(d.j) * a.block_bytes;
    const uint64_t end = file_off + a.block_bytes;
    d.obj_ptr = a.stage;
    d.obj_blk = a.stage + stage_off + file_off;
    if (u >= a.ctx_cap) {
      d.obj_ptr = nullptr;  // beyond the IOCBs the caller gave: not recorded, not executed
    } else if (stage_off == kNoFile || end > a.file_stride || end < file_off) {
      if (lane == 0 && d.s == 0 && a.status) atomicOr(a.status, TUTTI_ST_BAD_BLOCK);
      d.obj_ptr = nullptr;
    }
    return d;
  }
  d.obj_ptr = a.stage + stage_off + d.kind * d.obj_bytes;
  d.obj_blk = d.obj_ptr + static_cast<uint64_t>(d.j) * a.block_bytes;
  if (!SEP && (stage_off > a.stage_cap || d.obj_bytes > (a.stage_cap - stage_off) / 2)) {
    // the request's objects do not fit: skip it, report once
    // (an ordered launch reports from its first workgroup instead: its list need not name the request's first block)
    if (!ORD && lane == 0 && d.j == 0 && d.s == 0 && d.kind == 0 && a.status) atomicOr(a.status, TUTTI_ST_STAGE_CAP);
    d.obj_ptr = nullptr;
  } else if ((static_cast<uint64_t>(d.j) + 1) * a.block_bytes > d.obj_bytes) {
    d.obj_ptr = nullptr;  // the block would end beyond its object (caller-made extents only)
  }
  return d;
}

// Block id of an item through the scalar (constant) path: the index is wave-uniform, so this is
// one s_load that overlaps the vector loads and stores of the item before it.
__device__ __forceinline__ uint32_t load_block_id(const MoveArgs &a, const Item &d) {
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Wold-style-cast"
  const_u32_ptr tab = (const_u32_ptr)a.table;
#pragma clang diagnostic pop
  const uint32_t idx = __builtin_amdgcn_readfirstlane(d.tab_idx);  // uniform by construction
  const bool ok = __builtin_amdgcn_readfirstlane(d.obj_ptr != nullptr && idx < a.table_len ? 1 : 0) != 0;
  return ok ? tab[idx] : a.num_blocks;
}

template <int DIR, bool HND, int U, int NT>
__device__ __forceinline__ void move_one(const MoveArgs &a, const Item &d, uint32_t id, uint32_t lane) {
  constexpr uint32_t kSlice = kWave * 16u * U;
  if (d.obj_ptr == nullptr) return;
  const uint32_t in_blk = d.s * kSlice;  // first byte of the slice inside the block
  if (id < a.num_blocks) {
    unsigned char *blk_ptr = (d.kind ? a.v_base : a.k_base) + static_cast<uint64_t>(id) * a.block_stride;
    unsigned char *obj_blk = d.obj_blk;
    const uint32_t o0 = in_blk + lane * 16u;  // this lane's first 16 bytes, canonical offset in the block
    if (in_blk + kSlice <= a.block_bytes) {
      // whole slice inside the block: U independent loads in flight, then U stores
      u32x4 buf[U];
#pragma unroll
      for (int k = 0; k < U; ++k) {
        const uint32_t o = o0 + k * (kWave * 16u);
        if (DIR == kPack)
          buf[k] = ld16<NT>(blk_ptr + (HND ? hnd_offset(o, a.row_bytes, a.block_tokens, a.num_kv_heads) : o));
        else
          buf[k] = ld16<NT>(obj_blk + o);
      }
#pragma unroll
      for (int k = 0; k < U; ++k) {
        const uint32_t o = o0 + k * (kWave * 16u);
        if (DIR == kPack)
          st16<NT>(obj_blk + o, buf[k]);
        else
          st16<NT>(blk_ptr + (HND ? hnd_offset(o, a.row_bytes, a.block_tokens, a.num_kv_heads) : o), buf[k]);
      }
    } else {
      // ragged last slice of a block: one guarded 16-byte move at a time
      for (int k = 0; k < U; ++k) {
        const uint32_t o = o0 + k * (kWave * 16u);
        if (o < a.block_bytes) {
          const uint32_t po = HND ? hnd_offset(o, a.row_bytes, a.block_tokens, a.num_kv_heads) : o;
          if (DIR == kPack)
            st16<NT>(obj_blk + o, ld16<NT>(blk_ptr + po));
          else
            st16<NT>(blk_ptr + po, ld16<NT>(obj_blk + o));
        }
      }
    }
  } else if (lane == 0 && d.s == 0 && a.status) {
    atomicOr(a.status, TUTTI_ST_BAD_BLOCK);
  }
  if (DIR == kPack && !a.direct && d.j + 1 == d.n && d.s + 1 == a.slices_per_block) {
    // zero the tail of the object up to its aligned size (fewer than `align` bytes)
    const uint64_t used = static_cast<uint64_t>(d.n) * a.block_bytes;
    const u32x4 zero = {0u, 0u, 0u, 0u};
    for (uint64_t o = used + lane * 16ull; o < d.obj_bytes; o += kWave * 16ull) st16<0>(d.obj_ptr + o, zero);
  }
}

// First item of a wavefront in an unpack from dense staging: its source bytes do not depend on the extents,
// so their loads can be in flight while the workgroup is still fetching or scanning the extents.
template <int U>
struct Preload {
  u32x4 buf[U];
  const unsigned char *src;  // where the slice was read from (wave-uniform)
  bool valid;
};

template <int U, int NT>
__device__ __forceinline__ Preload<U> preload_first(const MoveArgs &a, uint32_t wg, uint32_t copy_wgs) {
  constexpr uint32_t kSlice = kWave * 16u * U;
  const uint32_t lane = threadIdx.x & (kWave - 1);
  const uint32_t it = item_wg(a, wg, copy_wgs) * (blockDim.x / kWave) + rfl(threadIdx.x / kWave);
  Preload<U> p;
  p.valid = a.dense != 0 && it < a.items_bound && (static_cast<uint64_t>(it) + 1) * kSlice <= a.stage_cap;
  p.src = a.stage + static_cast<uint64_t>(it) * kSlice;
  if (p.valid) {
    const unsigned char *src = p.src + lane * 16u;
#pragma unroll
    for (int k = 0; k < U; ++k) p.buf[k] = ld16<NT>(src + k * (kWave * 16u));
  }
  return p;
}

// Stores of an unpack item whose slice was preloaded (whole slices only: dense staging).
template <bool HND, int U, int NT>
__device__ __forceinline__ void store_preloaded(const MoveArgs &a, const Item &d, uint32_t id, uint32_t lane,
                                                const Preload<U> &p) {
  constexpr uint32_t kSlice = kWave * 16u * U;
  if (d.obj_ptr == nullptr) return;
  if (id < a.num_blocks) {
    unsigned char *blk_ptr = (d.kind ? a.v_base : a.k_base) + static_cast<uint64_t>(id) * a.block_stride;
    const uint32_t o0 = d.s * kSlice + lane * 16u;
#pragma unroll
    for (int k = 0; k < U; ++k) {
      const uint32_t o = o0 + k * (kWave * 16u);
      st16<NT>(blk_ptr + (HND ? hnd_offset(o, a.row_bytes, a.block_tokens, a.num_kv_heads) : o), p.buf[k]);
    }
  } else if (lane == 0 && d.s == 0 && a.status) {
    atomicOr(a.status, TUTTI_ST_BAD_BLOCK);
  }
}

// The copy loop of the `copy_wgs` copy workgroups of the grid; `wg` is this workgroup's index among them (the
// grid may hold other workgroups with other work).
// Software-pipelined by one item: the next item is decoded and its block id requested before the
// current item's loads and stores are issued.
// Number of work items of a copy.  Staged mode: the scan (or the loader of caller-made extents) has already cut
// the requests at table_len blocks.  Direct-to-block mode: one unit per recorded context.  The host checked that
// the bound (2 * table_len, or the contexts the IOCBs hold) times the slices per block fits 32 bits.
template <bool SEP, bool ORD = false>
__device__ __forceinline__ uint32_t count_items(const MoveArgs &a, const ReqLds &l, uint32_t n_req) {
  if (ORD) return 2u * a.table_len * a.slices_per_block;  // every listed position, for K and for V
  if (a.direct) {
    const uint64_t units = 2ull * l.table_off[n_req];
    return static_cast<uint32_t>(units < a.ctx_cap ? units : a.ctx_cap) * a.slices_per_block;
  }
  return 2u * (SEP ? l.blk_off[n_req] : l.table_off[n_req]) * a.slices_per_block;
}

template <int DIR, bool HND, int U, int NT, bool SEP, bool ORD = false>
__device__ __forceinline__ void move_items(const MoveArgs a, const ReqLds l, uint32_t n_req, uint32_t wg,
                                           uint32_t copy_wgs, const Preload<U> &pre) {
  constexpr uint32_t kSlice = kWave * 16u * U;
  const uint32_t lane = threadIdx.x & (kWave - 1);
  const uint32_t wave_in_wg = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
  const uint32_t n_waves = copy_wgs * (blockDim.x / kWave);
  const uint32_t n_items = count_items<SEP, ORD>(a, l, n_req);

  uint32_t it = item_wg(a, wg, copy_wgs) * (blockDim.x / kWave) + wave_in_wg;
  if (it >= n_items) return;
  Item cur = decode_item<SEP, ORD>(a, l, n_req, it, lane);
  uint32_t id = load_block_id(a, cur);
  bool first = true;
  for (;;) {
    const uint32_t nit = it + n_waves;
    const bool more = nit < n_items;
    Item nxt = cur;
    uint32_t nid = a.num_blocks;
    if (more) {
      nxt = decode_item<SEP, ORD>(a, l, n_req, nit, lane);
      nid = load_block_id(a, nxt);
    }
    // the preloaded bytes were read where the item's slice sits when the extents are the library's own; extents
    // from the caller (and the files of the direct-to-block mode) may put it elsewhere: then the slice is loaded
    // from where they say
    const bool preloaded = DIR == kUnpack && first && pre.valid &&
                           ((!SEP && !ORD && !a.direct) ||
                            cur.obj_blk + static_cast<uint64_t>(cur.s) * kSlice == pre.src);
    if (preloaded)
      store_preloaded<HND, U, NT>(a, cur, id, lane, pre);
    else
      move_one<DIR, HND, U, NT>(a, cur, id, lane);
    first = false;
    if (!more) break;
    cur = nxt;
    id = nid;
    it = nit;
  }
}

// ------------------------------------------------------------------------------------------
// Head-major pools with short rows.  A block is stored [h][T][row]; the object wants [T][h][row].
// Moving 16 bytes per lane straight between the two orders touches the pool in row-sized pieces,
// which is fine while a row fills whole 128-byte lines and poor below that (partial-line writes).
// Here a workgroup stages one tile (2^tile_shift tokens x all heads) in LDS instead: the object
// side is read or written as one contiguous run, the pool side as h runs of tile_tokens*row bytes,
// and the transpose happens in LDS.  Tokens are padded by one row in LDS so that the lanes of a
// wavefront, which walk the rows of one head, fall on different banks.
// PT = 16-byte units per thread per tile (tile bytes = PT * 16 * workgroup size).
// ------------------------------------------------------------------------------------------
// Shifts and masks of the tile geometry.
struct TileGeom {
  uint32_t rs, gs, hr;               // log2 bytes of a row, of one token across all heads, of one head's run in the tile
  uint32_t g_mask, hr_mask, r_mask;
};

// The tile of an item on both sides: global loads of its PT 16-byte units per thread (object order for an
// unpack, pool order for a pack), and where they go afterwards.
template <int DIR, int PT, int WG>
struct TileMove {
  static __device__ __forceinline__ unsigned char *obj_tile(const MoveArgs &a, const TileGeom &g, const Item &d) {
    const uint32_t t0 = d.s << a.tile_shift;
    return d.obj_ptr + static_cast<uint64_t>(d.j) * a.block_bytes + (static_cast<uint64_t>(t0) << g.gs);
  }
  static __device__ __forceinline__ unsigned char *blk(const MoveArgs &a, const Item &d, uint32_t id) {
    return (d.kind ? a.v_base : a.k_base) + static_cast<uint64_t>(id) * a.block_stride;
  }
  // byte offset inside the block of pool-order position p of the tile that starts at token t0
  static __device__ __forceinline__ uint32_t pool_off(const MoveArgs &a, const TileGeom &g, uint32_t t0, uint32_t p) {
    const uint32_t i = p >> g.hr, t = (p & g.hr_mask) >> g.rs, w = p & g.r_mask;
    return (((i << a.token_shift) + t0 + t) << g.rs) + w;
  }
  // LDS offset of object-order position o, and of pool-order position p
  static __device__ __forceinline__ uint32_t lds_obj(const MoveArgs &a, const TileGeom &g, uint32_t o) {
    return (o >> g.gs) * a.lds_pitch + (o & g.g_mask);
  }
  static __device__ __forceinline__ uint32_t lds_pool(const MoveArgs &a, const TileGeom &g, uint32_t p) {
    const uint32_t i = p >> g.hr, t = (p & g.hr_mask) >> g.rs, w = p & g.r_mask;
    return t * a.lds_pitch + (i << g.rs) + w;
  }
  static __device__ __forceinline__ void load(const MoveArgs &a, const TileGeom &g, const Item &d, uint32_t id,
                                              uint32_t tid, u32x4 (&v)[PT]) {
    const uint32_t t0 = d.s << a.tile_shift;
    const unsigned char *src = DIR == kUnpack ? obj_tile(a, g, d) : blk(a, d, id);
#pragma unroll
    for (int k = 0; k < PT; ++k) {
      const uint32_t q = (k * WG + tid) * 16u;
      v[k] = ld16<1>(src + (DIR == kUnpack ? q : pool_off(a, g, t0, q)));
    }
  }
  static __device__ __forceinline__ void to_lds(const MoveArgs &a, const TileGeom &g, uint32_t tid, unsigned char *tile,
                                                const u32x4 (&v)[PT]) {
#pragma unroll
    for (int k = 0; k < PT; ++k) {
      const uint32_t q = (k * WG + tid) * 16u;
      *reinterpret_cast<u32x4 *>(tile + (DIR == kUnpack ? lds_obj(a, g, q) : lds_pool(a, g, q))) = v[k];
    }
  }
  static __device__ __forceinline__ void from_lds_and_store(const MoveArgs &a, const TileGeom &g, const Item &d,
                                                            uint32_t id, uint32_t tid, const unsigned char *tile) {
    const uint32_t t0 = d.s << a.tile_shift;
    unsigned char *dst = DIR == kUnpack ? blk(a, d, id) : obj_tile(a, g, d);
    u32x4 w[PT];
#pragma unroll
    for (int k = 0; k < PT; ++k) {
      const uint32_t q = (k * WG + tid) * 16u;
      w[k] = *reinterpret_cast<const u32x4 *>(tile + (DIR == kUnpack ? lds_pool(a, g, q) : lds_obj(a, g, q)));
    }
#pragma unroll
    for (int k = 0; k < PT; ++k) {
      const uint32_t q = (k * WG + tid) * 16u;
      st16<2>(dst + (DIR == kUnpack ? pool_off(a, g, t0, q) : q), w[k]);
    }
  }
};

// One tile per workgroup and iteration.  Not pipelined across tiles: holding the next tile's loads in
// registers cost the eighth resident workgroup per CU (more than 64 VGPRs) and bought 0.3 us; the eight
// workgroups of a CU cover each other's latency instead.
template <int DIR, int PT, int WG, bool SEP>
__device__ __forceinline__ void move_items_hnd_lds(const MoveArgs a, const ReqLds l, uint32_t n_req, uint32_t wg,
                                                   uint32_t copy_wgs, unsigned char *tile) {
  typedef TileMove<DIR, PT, WG> TM;
  const uint32_t tid = threadIdx.x;
  const uint32_t n_items = count_items<SEP>(a, l, n_req);
  TileGeom g;
  g.rs = a.row_shift;
  g.gs = a.row_shift + a.head_shift;
  g.hr = a.tile_shift + a.row_shift;
  g.g_mask = (1u << g.gs) - 1u;
  g.hr_mask = (1u << g.hr) - 1u;
  g.r_mask = (1u << g.rs) - 1u;

  for (uint32_t it = wg; it < n_items; it += copy_wgs) {
    const Item d = decode_item<SEP>(a, l, n_req, it, tid);  // workgroup-uniform; thread 0 reports
    const uint32_t id = load_block_id(a, d);
    if (d.obj_ptr != nullptr && id < a.num_blocks) {
      u32x4 v[PT];
      TM::load(a, g, d, id, tid, v);
      TM::to_lds(a, g, tid, tile, v);
      __syncthreads();
      TM::from_lds_and_store(a, g, d, id, tid, tile);
      __syncthreads();  // the tile is free again
    } else if (d.obj_ptr != nullptr && tid == 0 && d.s == 0 && a.status) {
      atomicOr(a.status, TUTTI_ST_BAD_BLOCK);
    }
    if (DIR == kPack && d.obj_ptr != nullptr && d.j + 1 == d.n && d.s + 1 == a.slices_per_block) {
      const uint64_t used = static_cast<uint64_t>(d.n) * a.block_bytes;
      const u32x4 zero = {0u, 0u, 0u, 0u};
      for (uint64_t o = used + tid * 16ull; o < d.obj_bytes; o += WG * 16ull) st16<0>(d.obj_ptr + o, zero);
    }
  }
}

__host__ __device__ constexpr uint32_t align16(uint32_t x) { return (x + 15u) & ~15u; }

struct LayoutArgs {
  const uint32_t *n_blocks;
  tutti_extent *extents;
  uint64_t *totals;
  ScanGeom geom;
  uint32_t n_req;
};

__global__ __launch_bounds__(kWave) void k_layout(const LayoutArgs a) {
  extern __shared__ __align__(16) unsigned char smem[];
  const ReqLds l = carve_lds(smem, a.n_req);
  wave_scan_extents(a.geom, a.n_blocks, a.n_req, threadIdx.x, l, a.extents, a.totals, 0xffffffffu, nullptr);
}

template <int WG>
__global__ __launch_bounds__(WG) void k_sqe(const SqeArgs a, const ScanGeom g,
                                                     const tutti_extent *__restrict__ ext, uint32_t n_req) {
  extern __shared__ __align__(16) unsigned char smem[];
  const ReqLds l = carve_lds(smem, n_req);
  if (!lds_from_extents<WG>(ext, n_req, l, g, a.status)) return;
  emit_sqes(a, l, n_req, 0, gridDim.x, sqe_head(a, l, n_req, 0));
}

template <int DIR, bool HND, int U, int NT, int WG>
__global__ __launch_bounds__(WG, min_waves_per_simd(WG, U)) void k_move(const MoveArgs a, const tutti_extent *__restrict__ ext,
                                                      uint32_t n_req) {
  extern __shared__ __align__(16) unsigned char smem[];
  const ReqLds l = carve_lds(smem, n_req, true);
  Preload<U> pre;
  pre.valid = false;
  if (DIR == kUnpack) pre = preload_first<U, NT>(a, blockIdx.x, gridDim.x);
  lds_from_caller_extents(ext, n_req, l, a.table_len, a.block_bytes, a.stage_cap, a.status);
  move_items<DIR, HND, U, NT, true>(a, l, n_req, blockIdx.x, gridDim.x, pre);
}

template <int DIR, int PT, int WG>
__global__ __launch_bounds__(WG, min_waves_per_simd(WG, PT)) void k_move_lds(const MoveArgs a, const tutti_extent *__restrict__ ext,
                                                  uint32_t n_req) {
  extern __shared__ __align__(16) unsigned char smem[];
  const ReqLds l = carve_lds(smem, n_req, true);
  lds_from_caller_extents(ext, n_req, l, a.table_len, a.block_bytes, a.stage_cap, a.status);
  move_items_hnd_lds<DIR, PT, WG, true>(a, l, n_req, blockIdx.x, gridDim.x, smem + align16(req_lds_bytes(n_req)));
}

// One layer's restore (DIR = kUnpack) or save (DIR = kPack) in one launch: every workgroup redoes the
// (tiny) scan into its own LDS with its first wavefront.  The workgroups [copy_first, copy_first + copy_wgs)
// move the blocks; the first `sqe_wgs` workgroups of the grid also (or only) write the entries, one quarter per
// lane, and workgroup 0 publishes extents and totals.  The copy workgroups are persistent and split the items
// evenly, so the kernel ends when its slowest workgroup does: a workgroup with extra work in front of or behind
// its share, or one that has to wait for a free slot because the grid is larger than what the chip holds at
// once, adds that work's latency to the whole kernel (measured: 2.4 us of 53 with the entry writers as extra
// workgroups behind a full grid).  So the entries ride along: an entry-writing workgroup finds its quarter's
// request and asks for the file id right after the scan, runs its share of the copy, and only then assembles
// and stores the entry; with enough entries every workgroup of the grid takes one pass of them.
struct Roles {
  uint32_t sqe_wgs;     // workgroups [0, sqe_wgs) write entries
  uint32_t copy_first;  // workgroups [copy_first, copy_first + copy_wgs) move blocks (the grid may be larger when
  uint32_t copy_wgs;    // there are more passes of entries than copy workgroups)
};

// ORD (restore only): the blocks are visited in the order m.visit lists instead of staging order; the first slices
// cannot be preloaded then (where they sit depends on the list).
template <int DIR, bool HND, int U, int NT, int WG, bool ORD = false>
__global__ __launch_bounds__(WG, min_waves_per_simd(WG, U)) void k_layer(const MoveArgs m, const SqeArgs q, const LayoutArgs a, const Roles w) {
  extern __shared__ __align__(16) unsigned char smem[];
  const ReqLds l = carve_lds(smem, a.n_req);
  const uint32_t wg = blockIdx.x - w.copy_first;  // wraps for the workgroups in front of the copy ones
  const bool copies = wg < w.copy_wgs;
  Preload<U> pre;
  pre.valid = false;
  if (DIR == kUnpack && !ORD && copies) pre = preload_first<U, NT>(m, wg, w.copy_wgs);  // in flight during the scan
  if (threadIdx.x < kWave) {
    const bool publish = blockIdx.x == 0;
    wave_scan_extents(a.geom, a.n_blocks, a.n_req, threadIdx.x, l, publish ? a.extents : nullptr,
                      publish ? a.totals : nullptr, m.table_len, m.status, blockIdx.x < w.sqe_wgs);
  }
  __syncthreads();
  SqeHead head;
  head.live = false;
  if (blockIdx.x < w.sqe_wgs) head = sqe_head(q, l, a.n_req, 0);
  if (ORD && wg == 0 && m.status) {
    // requests whose objects do not fit the staging buffer are skipped by every item: report them here, once
    for (uint32_t r = threadIdx.x; r < a.n_req; r += WG)
      if (l.table_off[r + 1] > l.table_off[r] &&
          (l.stage_off[r] > m.stage_cap || l.obj_bytes[r] > (m.stage_cap - l.stage_off[r]) / 2))
        atomicOr(m.status, TUTTI_ST_STAGE_CAP);
  }
  if (copies) move_items<DIR, HND, U, NT, false, ORD>(m, l, a.n_req, wg, w.copy_wgs, pre);
  if (blockIdx.x < w.sqe_wgs) emit_sqes(q, l, a.n_req, 0, w.sqe_wgs, head);
}

// First item of a wavefront in a retrieve of ONE request: its file bytes sit at
//   file start + 2*layer*obj_bytes + item*slice        (obj_bytes = n_blocks*block_bytes: blocks are whole
// alignment units in this mode), which takes two words from memory, the block count and the file id, and no scan.
// Every wavefront fetches them itself through the scalar path and has its loads in flight while the workgroup's
// first wavefront scans and the barrier is crossed; move_items checks the address against the decoded one.
template <int U>
__device__ __forceinline__ Preload<U> preload_first_direct(const MoveArgs &m, const uint32_t *n_blocks,
                                                           const uint32_t *file_id, const FileArgs f, uint32_t wg,
                                                           uint32_t copy_wgs) {
  constexpr uint32_t kSlice = kWave * 16u * U;
  const uint32_t lane = threadIdx.x & (kWave - 1);
  const uint32_t it = item_wg(m, wg, copy_wgs) * (blockDim.x / kWave) + rfl(threadIdx.x / kWave);
  Preload<U> p;
  p.valid = false;
  if (m.block_bytes % kSlice != 0) return p;
  const uint32_t n = rfl(n_blocks[0]), fid = rfl(file_id[0]);
  const uint32_t rel = fid - f.first_file_id;
  const uint64_t obj = static_cast<uint64_t>(n) * m.block_bytes;
  const uint64_t units = 2ull * (n < m.table_len ? n : m.table_len);
  const uint64_t lo = 2ull * m.layer * obj;  // file offset of the layer's K object
  // inside the table, inside the recorded contexts, inside the file (K and V objects of the layer: 2*obj bytes)
  if (fid < f.first_file_id || rel >= f.n_files || it >= units * m.slices_per_block ||
      it / m.slices_per_block >= m.ctx_cap || obj == 0 || lo / obj != 2ull * m.layer || lo + 2 * obj < lo ||
      lo + 2 * obj > f.file_stride)
    return p;
  p.valid = true;
  p.src = m.stage + static_cast<uint64_t>(rel) * f.file_stride + lo + static_cast<uint64_t>(it) * kSlice;
  const unsigned char *src = p.src + lane * 16u;
#pragma unroll
  for (int k = 0; k < U; ++k) p.buf[k] = ld16<3>(src + k * (kWave * 16u));
  return p;
}

// retrieve_layer / store_layer through the rings in one launch (direct-to-block mode): the scan puts the start
// of every request's file in the store where the staging offsets would be, then the first `sqe_wgs`
// workgroups record the layer's contexts in the IOCBs while the copy workgroups move the very same blocks,
// each item deriving its file offset and block from the extents and the table exactly as its context does.
// Blocks go to the file as they sit in the pool (a descriptor names raw bytes), so there is no head-major case.
// The completion of these IOCBs is a kernel boundary away: the host enqueues k_complete behind this kernel, or the
// next layer's launch carries it along (`done`: the IOCBs an earlier launch on the same stream has executed; when
// done.n_slots is not 0 the grid has one workgroup more, in front, whose first wavefront completes them and leaves,
// so a train of layers pays for no kernel boundary between a layer's data and the next layer's).
template <int DIR, int U, int WG>
__global__ __launch_bounds__(WG, min_waves_per_simd(WG, U)) void k_layer_ring(const MoveArgs m, const SqeArgs q, const DirectArgs d,
                                                    const RingArgs g, const RingArgs done, const FileArgs f,
                                                    const LayoutArgs a, const Roles w) {
  extern __shared__ __align__(16) unsigned char smem[];
  const uint32_t lead = done.n_slots != 0 ? 1u : 0u;
  if (lead && blockIdx.x == 0) {  // the whole workgroup takes this branch: no barrier is left waiting
    if (threadIdx.x < kWave) complete_iocbs(done, threadIdx.x);
    return;
  }
  const uint32_t bx = blockIdx.x - lead;
  const ReqLds l = carve_lds(smem, a.n_req);
  const bool copies = bx - w.copy_first < w.copy_wgs;
  Preload<U> pre;
  pre.valid = false;
  if (DIR == kUnpack && copies && a.n_req == 1)
    pre = preload_first_direct<U>(m, a.n_blocks, q.file_id, f, bx - w.copy_first, w.copy_wgs);
  if (threadIdx.x < kWave) {
    const bool publish = bx == 0;
    // chunk counts only matter for the published extents; the LDS copy gets file starts instead of staging offsets
    wave_scan_extents(a.geom, a.n_blocks, a.n_req, threadIdx.x, l, publish ? a.extents : nullptr,
                      publish ? a.totals : nullptr, 0xffffffffu, nullptr, publish, q.file_id, f);
  }
  __syncthreads();
  DirectHead head;
  head.live = false;
  if (bx < w.sqe_wgs) head = iocb_head(g, q, d, l, a.n_req, lead, w.sqe_wgs);
  if (copies) move_items<DIR, false, U, 3, false>(m, l, a.n_req, bx - w.copy_first, w.copy_wgs, pre);
  if (bx < w.sqe_wgs) emit_iocbs(g, q, d, l, a.n_req, lead, w.sqe_wgs, head);
}

template <int DIR, int PT, int WG>
__global__ __launch_bounds__(WG, min_waves_per_simd(WG, PT)) void k_layer_lds(const MoveArgs m, const SqeArgs q, const LayoutArgs a, const Roles w) {
  extern __shared__ __align__(16) unsigned char smem[];
  const ReqLds l = carve_lds(smem, a.n_req);
  if (threadIdx.x < kWave) {
    const bool publish = blockIdx.x == 0;
    wave_scan_extents(a.geom, a.n_blocks, a.n_req, threadIdx.x, l, publish ? a.extents : nullptr,
                      publish ? a.totals : nullptr, m.table_len, m.status, blockIdx.x < w.sqe_wgs);
  }
  __syncthreads();
  SqeHead head;
  head.live = false;
  if (blockIdx.x < w.sqe_wgs) head = sqe_head(q, l, a.n_req, 0);
  if (blockIdx.x - w.copy_first < w.copy_wgs)
    move_items_hnd_lds<DIR, PT, WG, false>(m, l, a.n_req, blockIdx.x - w.copy_first, w.copy_wgs,
                                    smem + align16(req_lds_bytes(a.n_req)));
  if (blockIdx.x < w.sqe_wgs) emit_sqes(q, l, a.n_req, 0, w.sqe_wgs, head);
}

// The preconditions of an unpack on its table, checked without any workspace: every id below num_blocks, no id
// twice.  All pairs: workgroup b takes the 256 table positions [256b, 256b + 256) as rows (one per thread), walks
// the column tiles from its own onwards through LDS and compares each row with the later positions of the tile,
// four ids per LDS read.  O(table_len^2) comparisons: a debugging aid (a 40,000-entry table takes microseconds, a
// million entries tens of milliseconds), not part of the per-layer path.
__global__ __launch_bounds__(kWgThreads) void k_table_validate(const uint32_t *__restrict__ table, uint32_t n,
                                                                uint32_t num_blocks, uint32_t *__restrict__ status) {
  __shared__ __align__(16) uint32_t tile[kWgThreads];
  const uint32_t n_tiles = (n + kWgThreads - 1) / kWgThreads;
  uint32_t found = 0;
  for (uint32_t b = blockIdx.x; b < n_tiles; b += gridDim.x) {
    const uint32_t i = b * kWgThreads + threadIdx.x;
    const uint32_t id = i < n ? table[i] : 0xffffffffu;
    const bool valid = id < num_blocks;
    if (i < n && !valid) found |= TUTTI_ST_BAD_BLOCK;
    for (uint32_t c = b; c < n_tiles; ++c) {
      const uint32_t j0 = c * kWgThreads;
      const uint32_t j = j0 + threadIdx.x;
      __syncthreads();  // the previous tile has been read by everyone
      tile[threadIdx.x] = j < n ? table[j] : 0xffffffffu;  // an id no valid row can equal
      __syncthreads();
      if (valid) {
        // positions after i only: in the row's own tile start behind it (rounded down to a group of four,
        // with the row's own and earlier positions masked out), in later tiles take everything
        const uint32_t first = c == b ? (threadIdx.x + 1) : 0;
        for (uint32_t k = first & ~3u; k < kWgThreads; k += 4) {
          const u32x4 t = *reinterpret_cast<const u32x4 *>(&tile[k]);
          const bool e0 = t.x == id && k + 0 >= first, e1 = t.y == id && k + 1 >= first;
          const bool e2 = t.z == id && k + 2 >= first, e3 = t.w == id && k + 3 >= first;
          if (e0 || e1 || e2 || e3) found |= TUTTI_ST_DUP_BLOCK;
        }
      }
    }
  }
  if (found && status) atomicOr(status, found);
}

// The same two preconditions in time linear in the table, with one bit per pool block in memory that the caller
// lends (or that the library keeps): a thread sets the bit of its id with an atomic OR and has found a duplicate
// when the bit was already set.  The bits a call uses are cleared by a kernel in front of it (a fill kernel, not
// a memset node, so that the pair can be captured in a graph).
__global__ __launch_bounds__(kWgThreads) void k_bitmap_clear(uint32_t *__restrict__ bits, uint32_t n_words) {
  for (uint32_t i = blockIdx.x * blockDim.x + threadIdx.x; i < n_words; i += gridDim.x * blockDim.x) bits[i] = 0u;
}

__global__ __launch_bounds__(kWgThreads) void k_table_validate_bitmap(const uint32_t *__restrict__ table, uint32_t n,
                                                                       uint32_t num_blocks, uint32_t *__restrict__ bits,
                                                                       uint32_t *__restrict__ status) {
  uint32_t found = 0;
  for (uint32_t i = blockIdx.x * blockDim.x + threadIdx.x; i < n; i += gridDim.x * blockDim.x) {
    const uint32_t id = table[i];
    if (id >= num_blocks) {
      found |= TUTTI_ST_BAD_BLOCK;
    } else {
      const uint32_t bit = 1u << (id & 31u);
      if (atomicOr(&bits[id >> 5], bit) & bit) found |= TUTTI_ST_DUP_BLOCK;
    }
  }
  // one atomic per wavefront that found something
  const uint32_t lane = threadIdx.x & (kWave - 1);
  uint32_t any = found;
#pragma unroll
  for (uint32_t d = kWave / 2; d >= 1; d >>= 1) any |= __shfl_xor(any, d, kWave);
  if (lane == 0 && any && status) atomicOr(status, any);
}

// The visiting order of a table by ascending block id, from the bitmap of its ids: the rank of an id is the number
// of set bits below it.  k_bitmap_prefix (ONE workgroup) turns the per-word bit counts into exclusive prefix sums;
// k_table_rank then places every table position at its id's rank.  If the check that set the bits found an id out
// of range or twice (flags != 0) the ranks are not a permutation and the identity order is written instead.
constexpr uint32_t kPrefixThreads = 1024;

__global__ __launch_bounds__(kPrefixThreads) void k_bitmap_prefix(const uint32_t *__restrict__ bits, uint32_t n_words,
                                                                   uint32_t *__restrict__ prefix) {
  __shared__ uint32_t part[kPrefixThreads];
  const uint32_t t = threadIdx.x;
  const uint32_t per = (n_words + kPrefixThreads - 1) / kPrefixThreads;  // consecutive words per thread
  const uint32_t lo = t * per < n_words ? t * per : n_words;
  const uint32_t hi = lo + per < n_words ? lo + per : n_words;
  uint32_t sum = 0;
  for (uint32_t i = lo; i < hi; ++i) sum += static_cast<uint32_t>(__popc(bits[i]));
  part[t] = sum;
  __syncthreads();
  for (uint32_t d = 1; d < kPrefixThreads; d <<= 1) {  // inclusive scan of the per-thread sums
    const uint32_t v = t >= d ? part[t - d] : 0u;
    __syncthreads();
    part[t] += v;
    __syncthreads();
  }
  uint32_t run = part[t] - sum;  // bits in front of this thread's words
  for (uint32_t i = lo; i < hi; ++i) {
    prefix[i] = run;
    run += static_cast<uint32_t>(__popc(bits[i]));
  }
}

__global__ __launch_bounds__(kWgThreads) void k_table_rank(const uint32_t *__restrict__ table, uint32_t n,
                                                            const uint32_t *__restrict__ bits,
                                                            const uint32_t *__restrict__ prefix,
                                                            const uint32_t *__restrict__ flags, uint32_t *__restrict__ visit,
                                                            uint32_t *__restrict__ status) {
  const uint32_t found = flags[0];  // what the check in front of this kernel found
  if (found && status && blockIdx.x == 0 && threadIdx.x == 0) atomicOr(status, found);
  for (uint32_t i = blockIdx.x * blockDim.x + threadIdx.x; i < n; i += gridDim.x * blockDim.x) {
    if (found) {
      visit[i] = i;
    } else {
      const uint32_t id = table[i];
      const uint32_t below = bits[id >> 5] & ((1u << (id & 31u)) - 1u);
      visit[prefix[id >> 5] + static_cast<uint32_t>(__popc(below))] = i;
    }
  }
}

#ifdef TUTTI_BENCH_BUILD
// ---- measurement kernels (libtutti_bench.so only)

// Plain contiguous copy with the access shape of move_items: the ceiling pack / unpack can reach.
template <int U, int NT, int WG>
__global__ __launch_bounds__(WG, min_waves_per_simd(WG, U)) void k_copy(unsigned char *__restrict__ dst,
                                                      const unsigned char *__restrict__ src, uint64_t bytes) {
  constexpr uint64_t kSlice = kWave * 16ull * U;
  const uint32_t lane = threadIdx.x & (kWave - 1);
  const uint64_t n_waves = static_cast<uint64_t>(gridDim.x) * (blockDim.x / kWave);
  const uint64_t n_items = (bytes + kSlice - 1) / kSlice;
  for (uint64_t it = static_cast<uint64_t>(blockIdx.x) * (blockDim.x / kWave) + threadIdx.x / kWave; it < n_items;
       it += n_waves) {
    const uint64_t o0 = it * kSlice + lane * 16ull;
    if ((it + 1) * kSlice <= bytes) {
      u32x4 buf[U];
#pragma unroll
      for (int k = 0; k < U; ++k) buf[k] = ld16<NT>(src + o0 + k * (kWave * 16ull));
#pragma unroll
      for (int k = 0; k < U; ++k) st16<NT>(dst + o0 + k * (kWave * 16ull), buf[k]);
    } else {
      for (int k = 0; k < U; ++k) {
        const uint64_t o = o0 + k * (kWave * 16ull);
        if (o < bytes) st16<NT>(dst + o, ld16<NT>(src + o));
      }
    }
  }
}

// One direction only, same access shape: READ xors every 16-byte unit into four words per wavefront, added to
// one of TUTTI_STREAM_SLOTS slots at the end, FILL writes unit i as {lo(i), hi(i), ~lo(i), tag}.  What a CU, or the chip, can read or
// write when it does nothing else.
constexpr uint32_t kFillTag = 0x54555454u;

template <int WRITE, int U, int WG>
__global__ __launch_bounds__(WG, min_waves_per_simd(WG, U)) void k_stream(unsigned char *__restrict__ buf, uint64_t bytes, uint32_t *__restrict__ xor4) {
  constexpr uint64_t kSlice = kWave * 16ull * U;
  const uint32_t lane = threadIdx.x & (kWave - 1);
  const uint64_t n_waves = static_cast<uint64_t>(gridDim.x) * (blockDim.x / kWave);
  const uint64_t n_items = (bytes + kSlice - 1) / kSlice;
  u32x4 acc = {0u, 0u, 0u, 0u};
  for (uint64_t it = static_cast<uint64_t>(blockIdx.x) * (blockDim.x / kWave) + threadIdx.x / kWave; it < n_items;
       it += n_waves) {
    const uint64_t o0 = it * kSlice + lane * 16ull;
    const bool whole = (it + 1) * kSlice <= bytes;
    if (WRITE) {
#pragma unroll
      for (int k = 0; k < U; ++k) {
        const uint64_t o = o0 + k * (kWave * 16ull);
        const uint64_t unit = o >> 4;
        const u32x4 v = {static_cast<uint32_t>(unit), static_cast<uint32_t>(unit >> 32), ~static_cast<uint32_t>(unit),
                         kFillTag};
        if (whole || o < bytes) st16<3>(buf + o, v);
      }
    } else if (whole) {
      u32x4 v[U];
#pragma unroll
      for (int k = 0; k < U; ++k) v[k] = ld16<3>(buf + o0 + k * (kWave * 16ull));
#pragma unroll
      for (int k = 0; k < U; ++k) acc ^= v[k];
    } else {
      for (int k = 0; k < U; ++k) {
        const uint64_t o = o0 + k * (kWave * 16ull);
        if (o < bytes) acc ^= ld16<3>(buf + o);
      }
    }
  }
  if (!WRITE) {
#pragma unroll
    for (uint32_t d = kWave / 2; d >= 1; d >>= 1) {
      acc.x ^= __shfl_xor(acc.x, d, kWave);
      acc.y ^= __shfl_xor(acc.y, d, kWave);
      acc.z ^= __shfl_xor(acc.z, d, kWave);
      acc.w ^= __shfl_xor(acc.w, d, kWave);
    }
    if (lane == 0) {
      // one slot per wavefront (modulo the slot count): atomics on one address from every wavefront of the chip
      // would take longer than the reads themselves
      const uint32_t w = blockIdx.x * (blockDim.x / kWave) + threadIdx.x / kWave;
      uint32_t *slot = xor4 + 4u * (w % TUTTI_STREAM_SLOTS);
      atomicXor(&slot[0], acc.x);
      atomicXor(&slot[1], acc.y);
      atomicXor(&slot[2], acc.z);
      atomicXor(&slot[3], acc.w);
    }
  }
}

// The copy with one side permuted at `gran` bytes: the memory system's own cost of the scatter.
template <int U, int WG>
__global__ __launch_bounds__(WG, min_waves_per_simd(WG, U)) void k_scatter(unsigned char *__restrict__ scattered, uint64_t span_bytes,
                                                 unsigned char *__restrict__ contig, uint64_t bytes,
                                                 const uint32_t *__restrict__ perm, uint32_t gran, uint32_t to_scattered) {
  constexpr uint32_t kSlice = kWave * 16u * U;  // gran is a multiple of 4096 and of kSlice (host-checked)
  const uint32_t lane = threadIdx.x & (kWave - 1);
  const uint32_t wave_in_wg = rfl(threadIdx.x / kWave);
  const uint64_t n_waves = static_cast<uint64_t>(gridDim.x) * (blockDim.x / kWave);
  const uint32_t per = gran / kSlice;
  const uint64_t n_items = bytes / kSlice;
  for (uint64_t it = static_cast<uint64_t>(blockIdx.x) * (blockDim.x / kWave) + wave_in_wg; it < n_items; it += n_waves) {
    const uint64_t piece = it / per;
    const uint32_t s = static_cast<uint32_t>(it - piece * per);
    const uint64_t so = static_cast<uint64_t>(rfl(perm[piece])) * gran;
    if (so + gran > span_bytes) continue;
    unsigned char *sp = scattered + so + s * kSlice + lane * 16u;
    unsigned char *cp = contig + it * kSlice + lane * 16u;
    const unsigned char *src = to_scattered ? cp : sp;
    unsigned char *dst = to_scattered ? sp : cp;
    u32x4 buf[U];
#pragma unroll
    for (int u = 0; u < U; ++u) buf[u] = ld16<3>(src + u * (kWave * 16u));
#pragma unroll
    for (int u = 0; u < U; ++u) st16<3>(dst + u * (kWave * 16u), buf[u]);
  }
}

// The same scattered copy with the work dealt differently: a whole piece per wavefront (PER_WG = false) or per
// workgroup (true), walked in 4 KiB steps, with any of the four cache policies.  Whether another way of dealing
// out the same bytes would suit the memory system better than the product's wavefront-per-4-KiB.
template <bool PER_WG, int NT>
__global__ __launch_bounds__(kWgThreads, 8) void k_scatter_piece(unsigned char *__restrict__ scattered, uint64_t span_bytes,
                                                                  unsigned char *__restrict__ contig, uint64_t bytes,
                                                                  const uint32_t *__restrict__ perm, uint32_t gran,
                                                                  uint32_t to_scattered) {
  constexpr uint32_t kStep = kWave * 16u * 4u;  // 4 KiB per wavefront and step; gran is a multiple of it
  const uint32_t lane = threadIdx.x & (kWave - 1);
  const uint32_t wave_in_wg = rfl(threadIdx.x / kWave);
  const uint32_t waves = blockDim.x / kWave;
  const uint64_t n_pieces = bytes / gran;
  const uint64_t first = PER_WG ? blockIdx.x : static_cast<uint64_t>(blockIdx.x) * waves + wave_in_wg;
  const uint64_t stride = PER_WG ? gridDim.x : static_cast<uint64_t>(gridDim.x) * waves;
  for (uint64_t piece = first; piece < n_pieces; piece += stride) {
    const uint64_t so = static_cast<uint64_t>(rfl(perm[piece])) * gran;
    if (so + gran > span_bytes) continue;
    for (uint32_t off = PER_WG ? wave_in_wg * kStep : 0u; off < gran; off += PER_WG ? waves * kStep : kStep) {
      unsigned char *sp = scattered + so + off + lane * 16u;
      unsigned char *cp = contig + piece * gran + off + lane * 16u;
      const unsigned char *src = to_scattered ? cp : sp;
      unsigned char *dst = to_scattered ? sp : cp;
      u32x4 buf[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) buf[u] = ld16<NT>(src + u * (kWave * 16u));
#pragma unroll
      for (int u = 0; u < 4; ++u) st16<NT>(dst + u * (kWave * 16u), buf[u]);
    }
  }
}

#endif  // TUTTI_BENCH_BUILD

}  // namespace tutti
