/*
 * tutti_oracle.c -- CPU oracle for the per-layer KV object path. TEST INFRASTRUCTURE ONLY.
 *
 * Plain C, one thread, one loop per index of the definition (the d contiguous elements of a
 * (token, head) row move as one memcpy); no blocking, no tiling, no vector code.
 * See tutti_oracle.h for what the paper fixes and what is a repository reading.
 * The only callers allowed are the tests, the smoke check and the benchmark's cpu_baseline leg.
 */
#include "tutti_oracle.h"

#include <pthread.h>
#include <stddef.h>
#include <stdlib.h>
#include <string.h>

/* ------------------------------------------------------------------ helpers */

static int is_pow2(uint32_t x) { return x != 0 && (x & (x - 1)) == 0; }

static uint64_t align_up(uint64_t x, uint64_t a) { return (x + a - 1) / a * a; }

/* Bytes of one block of one plane: T*h*d*e for a [Block, h, d] block (sec. 2.1). */
uint32_t orc_block_bytes(const orc_pool *pool) {
  if (!pool) return 0;
  uint64_t b = (uint64_t)pool->block_tokens;
  b *= pool->num_kv_heads;
  if (b > 0xffffffffull) return 0;
  b *= pool->head_dim;
  if (b > 0xffffffffull) return 0;
  b *= pool->elt_bytes;
  if (b > 0xffffffffull) return 0;
  return (uint32_t)b;
}

static int check_geometry(const orc_pool *pool, const orc_objcfg *cfg) {
  if (!pool || !cfg) return ORC_EINVAL;
  uint32_t bb = orc_block_bytes(pool);
  if (bb == 0 || bb % 16 != 0) return ORC_EINVAL;
  if (pool->num_blocks == 0) return ORC_EINVAL;
  if (pool->block_stride < bb || pool->block_stride % 16 != 0) return ORC_EINVAL;
  if (pool->pool_layout != ORC_LAYOUT_NHD && pool->pool_layout != ORC_LAYOUT_HND) return ORC_EINVAL;
  if (!is_pow2(cfg->align) || cfg->align < 16) return ORC_EINVAL;
  if (cfg->chunk_bytes == 0 || cfg->chunk_bytes % cfg->align != 0) return ORC_EINVAL;
  if (cfg->num_layers == 0 || cfg->num_layers > 65536u) return ORC_EINVAL;
  return ORC_OK;
}

int orc_abi_describe(uint32_t *out, uint32_t cap) {
  if (!out || cap < 52) return ORC_EINVAL;
  uint32_t i = 0;
  out[i++] = sizeof(orc_extent);
  out[i++] = offsetof(orc_extent, stage_off);
  out[i++] = offsetof(orc_extent, obj_bytes);
  out[i++] = offsetof(orc_extent, n_blocks);
  out[i++] = offsetof(orc_extent, n_chunks);
  out[i++] = offsetof(orc_extent, sqe_base);
  out[i++] = offsetof(orc_extent, table_off);
  out[i++] = sizeof(orc_sqe);
  out[i++] = offsetof(orc_sqe, opcode);
  out[i++] = offsetof(orc_sqe, kind);
  out[i++] = offsetof(orc_sqe, layer);
  out[i++] = offsetof(orc_sqe, file_id);
  out[i++] = offsetof(orc_sqe, file_off);
  out[i++] = offsetof(orc_sqe, addr);
  out[i++] = offsetof(orc_sqe, len);
  out[i++] = offsetof(orc_sqe, sgl_id);
  out[i++] = offsetof(orc_sqe, user_data);
  out[i++] = offsetof(orc_sqe, iocb_idx);
  out[i++] = offsetof(orc_sqe, ioctx_slot);
  out[i++] = sizeof(orc_pool);
  out[i++] = offsetof(orc_pool, k_base);
  out[i++] = offsetof(orc_pool, v_base);
  out[i++] = offsetof(orc_pool, block_stride);
  out[i++] = offsetof(orc_pool, num_blocks);
  out[i++] = offsetof(orc_pool, block_tokens);
  out[i++] = offsetof(orc_pool, num_kv_heads);
  out[i++] = offsetof(orc_pool, head_dim);
  out[i++] = offsetof(orc_pool, elt_bytes);
  out[i++] = offsetof(orc_pool, pool_layout);
  out[i++] = sizeof(orc_objcfg);
  out[i++] = offsetof(orc_objcfg, align);
  out[i++] = offsetof(orc_objcfg, chunk_bytes);
  out[i++] = offsetof(orc_objcfg, num_layers);
  out[i++] = sizeof(orc_sgl);
  out[i++] = offsetof(orc_sgl, addr);
  out[i++] = offsetof(orc_sgl, len);
  out[i++] = offsetof(orc_sgl, id);
  out[i++] = sizeof(orc_iocb_hdr);
  out[i++] = offsetof(orc_iocb_hdr, iocb_idx);
  out[i++] = offsetof(orc_iocb_hdr, num_ioctx);
  out[i++] = offsetof(orc_iocb_hdr, state);
  out[i++] = offsetof(orc_iocb_hdr, done);
  out[i++] = offsetof(orc_iocb_hdr, layer);
  out[i++] = offsetof(orc_iocb_hdr, opcode);
  out[i++] = sizeof(orc_iocb);
  out[i++] = offsetof(orc_iocb, ioctx);
  out[i++] = sizeof(orc_cq_hdr);
  out[i++] = sizeof(orc_filestore);
  out[i++] = offsetof(orc_filestore, base);
  out[i++] = offsetof(orc_filestore, file_stride);
  out[i++] = offsetof(orc_filestore, first_file_id);
  out[i++] = offsetof(orc_filestore, n_files);
  return (int)i;
}

/* Pool of pool_bytes, one descriptor per gran bytes (sec. 3.1, "P2P Memory Mapping Table"). */
uint64_t orc_desc_count(uint64_t pool_bytes, uint64_t gran) {
  if (gran == 0) return 0;
  return (pool_bytes + gran - 1) / gran;
}

/* ------------------------------------------------------------------ extents */

/*
 * Extents.  One K object and one V object per (request, layer) (sec. 3.1, "Scalable GPU File
 * Pool"); each holds the request's n hit blocks back to back and is padded to the alignment
 * unit; an I/O context has an offset and a length (sec. 3.2), so an object is cut into
 * chunks of at most C bytes.  Offsets are running sums over the requests in order.
 */
int orc_obj_layout(const orc_pool *pool, const orc_objcfg *cfg, const uint32_t *n_blocks, uint32_t n_req,
                   orc_extent *extents, uint64_t *totals) {
  int rc = check_geometry(pool, cfg);
  if (rc) return rc;
  if (n_req > 0 && (!n_blocks || !extents)) return ORC_EINVAL;
  if (!totals) return ORC_EINVAL;
  const uint64_t bb = orc_block_bytes(pool);
  const uint64_t A = cfg->align;
  const uint64_t C = cfg->chunk_bytes;

  uint64_t stage = 0; /* bytes used so far in the staging buffer */
  uint64_t n_sqe = 0; /* entries so far */
  uint64_t n_tab = 0; /* block-table entries so far */
  for (uint32_t r = 0; r < n_req; ++r) {
    uint64_t obj = align_up((uint64_t)n_blocks[r] * bb, A);
    uint64_t chunks = (obj + C - 1) / C;
    extents[r].stage_off = stage;
    extents[r].obj_bytes = obj;
    extents[r].n_blocks = n_blocks[r];
    extents[r].n_chunks = (uint32_t)chunks;
    extents[r].sqe_base = (uint32_t)n_sqe;
    extents[r].table_off = (uint32_t)n_tab;
    stage += 2 * obj;    /* K object, then V object */
    n_sqe += 2 * chunks; /* K chunks, then V chunks */
    n_tab += n_blocks[r];
  }
  totals[0] = stage;
  totals[1] = n_sqe;
  return ORC_OK;
}

/* ------------------------------------------------------------------ pack / unpack */

/*
 * Copy one block between its place in the pool and its place in the object.
 * The object is token-major: token t, head i, dim k of the block at ((t*h + i)*d + k)*e.
 * An NHD block [T][h][d] (the paper's [Block, h, d], sec. 2.1) is already in that order.
 * An HND block [h][T][d] holds the same element at ((i*T + t)*d + k)*e.
 * to_object != 0: pool -> object; else object -> pool.
 */
static void move_block(const orc_pool *pool, uint8_t *blk, uint8_t *obj, int to_object) {
  const uint64_t T = pool->block_tokens, h = pool->num_kv_heads, d = pool->head_dim, e = pool->elt_bytes;
  for (uint64_t t = 0; t < T; ++t) {
    for (uint64_t i = 0; i < h; ++i) {
      /* the d elements of (t, i) are contiguous in both orders: move them as one row */
      uint64_t in_obj = ((t * h + i) * d) * e;
      uint64_t in_blk = (pool->pool_layout == ORC_LAYOUT_NHD) ? in_obj : ((i * T + t) * d) * e;
      if (to_object)
        memcpy(obj + in_obj, blk + in_blk, d * e);
      else
        memcpy(blk + in_blk, obj + in_obj, d * e);
    }
  }
}

/*
 * Shared body of pack and unpack.  A request's table range is [table_off, table_off + n_blocks); the mt timing
 * helpers pass a sub-range [g_lo, g_hi) of table positions, the single-threaded oracle passes everything.
 *
 * The paper defines the objects (sec. 3.1) but not what a library does with extents that a caller wrote by hand,
 * so the rules for those are this repository's reading; each one skips and reports instead of touching memory
 * outside the buffers the caller named:
 *   - requests are taken in order while the running sum of n_blocks stays within table_len; the request that
 *     pushes it beyond, and every later one, is skipped (ORC_ST_BAD_EXTENT);
 *   - a request whose stage_off or obj_bytes is not a multiple of 16 is skipped (ORC_ST_BAD_EXTENT);
 *   - a request whose two objects do not fit in stage_cap is skipped (ORC_ST_STAGE_CAP);
 *   - a block that would end beyond its object is skipped (ORC_ST_BAD_EXTENT);
 *   - a block whose table position is >= table_len, or whose id is >= num_blocks, is skipped (ORC_ST_BAD_BLOCK).
 * Extents that orc_obj_layout made, with the table they describe, trip none of the first four.
 */
static void move_range(const orc_pool *pool, const orc_extent *extents, uint32_t n_req, const uint32_t *block_table,
                       uint32_t table_len, uint8_t *stage, uint64_t stage_cap, int to_object, uint64_t g_lo,
                       uint64_t g_hi, uint32_t *status) {
  const uint64_t bb = orc_block_bytes(pool);
  uint32_t st = 0;
  uint64_t used = 0; /* table entries claimed by the requests so far */
  for (uint32_t r = 0; r < n_req; ++r) {
    const orc_extent *x = &extents[r];
    used += x->n_blocks;
    if (used > table_len) { /* more blocks than the table holds: this request and all later ones */
      st |= ORC_ST_BAD_EXTENT;
      continue;
    }
    if (x->stage_off % 16 != 0 || x->obj_bytes % 16 != 0) {
      st |= ORC_ST_BAD_EXTENT;
      continue;
    }
    if (x->stage_off > stage_cap || x->obj_bytes > (stage_cap - x->stage_off) / 2) { /* K + V do not fit */
      st |= ORC_ST_STAGE_CAP;
      continue;
    }
    const uint64_t filled = (uint64_t)x->n_blocks * bb; /* bytes of the object that blocks occupy */
    if (filled > x->obj_bytes) st |= ORC_ST_BAD_EXTENT;  /* the blocks beyond the object are skipped below */
    for (uint32_t kind = 0; kind < 2; ++kind) {
      uint8_t *plane = (uint8_t *)(kind == 0 ? pool->k_base : pool->v_base);
      uint8_t *obj = stage + x->stage_off + kind * x->obj_bytes; /* V object follows K object */
      for (uint32_t j = 0; j < x->n_blocks; ++j) {
        uint64_t g = (uint64_t)x->table_off + j;
        if (g < g_lo || g >= g_hi) continue;
        if (((uint64_t)j + 1) * bb > x->obj_bytes) continue; /* would end beyond the object */
        if (g >= table_len) {
          st |= ORC_ST_BAD_BLOCK;
        } else {
          uint32_t id = block_table[g];
          if (id >= pool->num_blocks) {
            st |= ORC_ST_BAD_BLOCK;
          } else {
            move_block(pool, plane + (uint64_t)id * pool->block_stride, obj + (uint64_t)j * bb, to_object);
          }
        }
        if (to_object && j + 1 == x->n_blocks) /* pad the tail of the object with zeros */
          memset(obj + filled, 0, x->obj_bytes - filled);
      }
    }
  }
  if (status && st) __atomic_fetch_or(status, st, __ATOMIC_RELAXED);
}

static int check_move_args(const orc_pool *pool, const orc_objcfg *cfg, const orc_extent *extents, uint32_t n_req,
                           const uint32_t *block_table, uint32_t table_len, const void *stage) {
  int rc = check_geometry(pool, cfg);
  if (rc) return rc;
  if (!pool->k_base || !pool->v_base) return ORC_EINVAL;
  if (n_req > 0 && (!extents || !stage)) return ORC_EINVAL;
  if (table_len > 0 && !block_table) return ORC_EINVAL;
  return ORC_OK;
}

/* Save direction: every hit block of every request into its object (sec. 3.1; store_layer of sec. 3.4). */
int orc_obj_pack(const orc_pool *pool, const orc_objcfg *cfg, const orc_extent *extents, uint32_t n_req,
                 const uint32_t *block_table, uint32_t table_len, void *stage, uint64_t stage_cap, uint32_t *status) {
  int rc = check_move_args(pool, cfg, extents, n_req, block_table, table_len, stage);
  if (rc) return rc;
  move_range(pool, extents, n_req, block_table, table_len, (uint8_t *)stage, stage_cap, 1, 0, UINT64_MAX, status);
  return ORC_OK;
}

/* Restore direction: every object back into the request's blocks (retrieve_layer of sec. 3.4). */
int orc_obj_unpack(const orc_pool *pool, const orc_objcfg *cfg, const orc_extent *extents, uint32_t n_req,
                   const uint32_t *block_table, uint32_t table_len, const void *stage, uint64_t stage_cap,
                   uint32_t *status) {
  int rc = check_move_args(pool, cfg, extents, n_req, block_table, table_len, stage);
  if (rc) return rc;
  move_range(pool, extents, n_req, block_table, table_len, (uint8_t *)(uintptr_t)stage, stage_cap, 0, 0, UINT64_MAX,
             status);
  return ORC_OK;
}

/* ------------------------------------------------------------------ submission entries */

/*
 * The entry builders number entries by sqe_base (or by twice table_off in the direct-to-block mode), so the
 * extents they take are the ones orc_obj_layout writes for exactly these requests: sizes that follow from
 * n_blocks, offsets running from 0 without gaps and fitting 32 bits.  The paper is silent on other extents;
 * reading taken: an entry builder handed anything else writes nothing and reports ORC_ST_BAD_EXTENT.
 * stage_off is free (it is only added to the staging address).
 */
static int extents_are_dense(const orc_pool *pool, const orc_objcfg *cfg, const orc_extent *extents, uint32_t n_req) {
  const uint64_t bb = orc_block_bytes(pool);
  uint64_t want_sqe = 0, want_tab = 0; /* what orc_obj_layout would have written */
  for (uint32_t r = 0; r < n_req; ++r) {
    const orc_extent *x = &extents[r];
    uint64_t obj = align_up((uint64_t)x->n_blocks * bb, cfg->align);
    uint64_t chunks = (obj + cfg->chunk_bytes - 1) / cfg->chunk_bytes;
    if (x->obj_bytes != obj || x->n_chunks != chunks) return 0;
    if (x->sqe_base != want_sqe || x->table_off != want_tab) return 0;
    want_sqe += chunks + chunks;
    want_tab += x->n_blocks;
    if (want_sqe > 0xffffffffull || want_tab > 0xffffffffull) return 0;
  }
  return 1;
}

/*
 * Entries of one layer in the order: request ascending; K object then V object; chunk ascending.
 * Each carries the I/O-context fields (address, GPU-file offset, length: sec. 3.2), the SGL
 * identifier (sec. 3.1) and its place in the 2048-slot IOCBs (sec. 3.2).  A request's GPU file
 * holds its 2*L objects layer-major, K before V (sec. 3.1: 2*L objects per file; the order is
 * this repository's reading).
 */
int orc_sqe_build(const orc_pool *pool, const orc_objcfg *cfg, const orc_extent *extents, uint32_t n_req,
                  const uint32_t *file_id, uint32_t layer, uint32_t opcode, uint64_t stage_addr, uint32_t sgl_id,
                  orc_sqe *sqe, uint32_t sqe_cap, uint32_t *status) {
  int rc = check_geometry(pool, cfg);
  if (rc) return rc;
  if (n_req > 0 && (!extents || !file_id)) return ORC_EINVAL;
  if (sqe_cap > 0 && !sqe) return ORC_EINVAL;
  if (opcode != ORC_OP_READ && opcode != ORC_OP_WRITE) return ORC_EINVAL;
  if (layer >= cfg->num_layers) return ORC_EINVAL;
  if (stage_addr % cfg->align != 0) return ORC_EINVAL;
  if (!extents_are_dense(pool, cfg, extents, n_req)) {
    if (status) *status |= ORC_ST_BAD_EXTENT;
    return ORC_OK;
  }
  const uint64_t C = cfg->chunk_bytes;
  uint32_t st = 0;

  for (uint32_t r = 0; r < n_req; ++r) {
    const orc_extent *x = &extents[r];
    for (uint32_t kind = 0; kind < 2; ++kind) {
      for (uint32_t c = 0; c < x->n_chunks; ++c) {
        uint64_t i = (uint64_t)x->sqe_base + (uint64_t)kind * x->n_chunks + c;
        if (i >= sqe_cap) {
          st |= ORC_ST_SQE_CAP;
          continue;
        }
        uint64_t left = x->obj_bytes - (uint64_t)c * C;
        orc_sqe s;
        memset(&s, 0, sizeof s);
        s.opcode = (uint8_t)opcode;
        s.kind = (uint8_t)kind;
        s.layer = (uint16_t)layer;
        s.file_id = file_id[r];
        s.file_off = (2ull * layer + kind) * x->obj_bytes + (uint64_t)c * C;
        s.addr = stage_addr + x->stage_off + (uint64_t)kind * x->obj_bytes + (uint64_t)c * C;
        s.len = (uint32_t)(left < C ? left : C);
        s.sgl_id = sgl_id;
        s.user_data = ((uint64_t)r << 32) | (uint32_t)i;
        s.iocb_idx = (uint32_t)(i / ORC_IOCB_SLOTS);
        s.ioctx_slot = (uint32_t)(i % ORC_IOCB_SLOTS);
        sqe[i] = s;
      }
    }
  }
  if (status && st) *status |= st;
  return ORC_OK;
}

/* ------------------------------------------------------------------ direct-to-block mode */

/*
 * The P2P memory mapping table of sec. 3.1: one 16-byte descriptor (address, length, identifier)
 * per pool block, K plane first, then V plane.  The pool is fixed for the engine's lifetime, so
 * this is computed once.
 */
int orc_sgl_table_build(const orc_pool *pool, uint64_t k_addr, uint64_t v_addr, uint32_t sgl_id, orc_sgl *table,
                        uint32_t cap, uint32_t *status) {
  if (!pool) return ORC_EINVAL;
  const uint32_t bb = orc_block_bytes(pool);
  if (bb == 0 || bb % 16 != 0 || pool->num_blocks == 0) return ORC_EINVAL;
  if (pool->block_stride < bb || pool->block_stride % 16 != 0) return ORC_EINVAL;
  if (cap > 0 && !table) return ORC_EINVAL;
  uint32_t st = 0;
  for (uint32_t kind = 0; kind < 2; ++kind) {
    for (uint32_t b = 0; b < pool->num_blocks; ++b) {
      uint64_t i = (uint64_t)kind * pool->num_blocks + b;
      if (i >= cap) {
        st |= ORC_ST_SQE_CAP;
        continue;
      }
      table[i].addr = (kind == 0 ? k_addr : v_addr) + (uint64_t)b * pool->block_stride;
      table[i].len = bb;
      table[i].id = sgl_id;
    }
  }
  if (status && st) *status |= st;
  return ORC_OK;
}

/* One direct-mode context: block j of request r (extent x), plane `kind`, entry index i of the layer. */
static uint32_t make_direct_entry(const orc_pool *pool, const orc_extent *x, uint32_t r, uint32_t kind, uint32_t j,
                                  uint32_t id, uint32_t file_id, uint32_t layer, uint32_t opcode,
                                  uint64_t sgl_table_addr, uint32_t sgl_id, uint64_t i, orc_sqe *out) {
  const uint64_t bb = orc_block_bytes(pool);
  uint32_t st = 0;
  orc_sqe s;
  memset(&s, 0, sizeof s);
  s.opcode = (uint8_t)opcode;
  s.kind = (uint8_t)kind;
  s.layer = (uint16_t)layer;
  s.file_id = file_id;
  s.file_off = (2ull * layer + kind) * x->obj_bytes + (uint64_t)j * bb;
  if (id < pool->num_blocks) {
    s.addr = sgl_table_addr + 16ull * ((uint64_t)kind * pool->num_blocks + id);
    s.len = (uint32_t)bb;
  } else {
    st = ORC_ST_BAD_BLOCK; /* a no-op entry: nothing to transfer */
  }
  s.sgl_id = sgl_id;
  s.user_data = ((uint64_t)r << 32) | (uint32_t)i;
  s.iocb_idx = (uint32_t)(i / ORC_IOCB_SLOTS);
  s.ioctx_slot = (uint32_t)(i % ORC_IOCB_SLOTS);
  *out = s;
  return st;
}

/*
 * Entries of the paper's own data path: each hit block is one object (sec. 3.1, "representing each
 * memory block as one object") and one I/O context whose SGL address is the block's descriptor in
 * the mapping table (sec. 3.2).  The GPU-file layout is the one of the staged mode.
 */
int orc_sqe_build_direct(const orc_pool *pool, const orc_objcfg *cfg, const orc_extent *extents, uint32_t n_req,
                         const uint32_t *block_table, const uint32_t *file_id, uint32_t layer, uint32_t opcode,
                         uint64_t sgl_table_addr, uint32_t sgl_id, orc_sqe *sqe, uint32_t sqe_cap, uint32_t *status) {
  int rc = check_geometry(pool, cfg);
  if (rc) return rc;
  const uint64_t bb = orc_block_bytes(pool);
  if (bb % cfg->align != 0) return ORC_EINVAL;
  if (n_req > 0 && (!extents || !file_id)) return ORC_EINVAL;
  if (sqe_cap > 0 && !sqe) return ORC_EINVAL;
  if (opcode != ORC_OP_READ && opcode != ORC_OP_WRITE) return ORC_EINVAL;
  if (layer >= cfg->num_layers) return ORC_EINVAL;
  if (sgl_table_addr % 16 != 0) return ORC_EINVAL;
  if (!extents_are_dense(pool, cfg, extents, n_req)) {
    if (status) *status |= ORC_ST_BAD_EXTENT;
    return ORC_OK;
  }
  uint64_t n_tab = 0;
  for (uint32_t r = 0; r < n_req; ++r) n_tab += extents[r].n_blocks;
  if (n_tab > 0 && !block_table) return ORC_EINVAL;
  uint32_t st = 0;

  for (uint32_t r = 0; r < n_req; ++r) {
    const orc_extent *x = &extents[r];
    for (uint32_t kind = 0; kind < 2; ++kind) {
      for (uint32_t j = 0; j < x->n_blocks; ++j) {
        uint64_t i = 2ull * x->table_off + (uint64_t)kind * x->n_blocks + j;
        if (i >= sqe_cap) {
          st |= ORC_ST_SQE_CAP;
          continue;
        }
        uint32_t id = block_table[(uint64_t)x->table_off + j];
        orc_sqe s;
        st |= make_direct_entry(pool, x, r, kind, j, id, file_id[r], layer, opcode, sgl_table_addr, sgl_id, i, &s);
        sqe[i] = s;
      }
    }
  }
  if (status && st) *status |= st;
  return ORC_OK;
}

/* ------------------------------------------------------------------ rings */

/* init_queue(depth) of sec. 3.2: depth IOCBs, each with a unique index, and an empty CQ. */
int orc_ring_init(orc_iocb *sq, void *cq, uint32_t depth) {
  if (!sq || !cq || depth == 0) return ORC_EINVAL;
  for (uint32_t b = 0; b < depth; ++b) {
    memset(&sq[b].hdr, 0, sizeof sq[b].hdr);
    sq[b].hdr.iocb_idx = b;
    sq[b].hdr.state = ORC_IOCB_FREE;
  }
  orc_cq_hdr *c = (orc_cq_hdr *)cq;
  memset(c, 0, sizeof *c);
  c->depth = depth;
  uint32_t *entry = (uint32_t *)(c + 1);
  for (uint32_t b = 0; b < depth; ++b) entry[b] = 0xffffffffu;
  return ORC_OK;
}

/*
 * get_iocb + fill (sec. 3.2): the contexts of one layer, as orc_sqe_build_direct numbers them, laid into
 * consecutive IOCBs of 2048 contexts each; num_ioctx records how many of an IOCB's slots are valid.
 */
int orc_iocb_fill_direct(orc_iocb *sq, uint32_t depth, uint32_t first_slot, uint32_t n_slots, const orc_pool *pool,
                         const orc_objcfg *cfg, const orc_extent *extents, uint32_t n_req, const uint32_t *block_table,
                         const uint32_t *file_id, uint32_t layer, uint32_t opcode, uint64_t sgl_table_addr,
                         uint32_t sgl_id, uint32_t *status) {
  if (!sq || depth == 0 || n_slots > depth || first_slot >= depth) return ORC_EINVAL;
  int rc = check_geometry(pool, cfg);
  if (rc) return rc;
  if (orc_block_bytes(pool) % cfg->align != 0) return ORC_EINVAL;
  if (opcode != ORC_OP_READ && opcode != ORC_OP_WRITE) return ORC_EINVAL;
  if (layer >= cfg->num_layers || sgl_table_addr % 16 != 0) return ORC_EINVAL;
  if (n_req > 0 && (!extents || !file_id)) return ORC_EINVAL;
  if (!extents_are_dense(pool, cfg, extents, n_req)) {
    if (status) *status |= ORC_ST_BAD_EXTENT;
    return ORC_OK;
  }
  uint64_t n = 0;
  for (uint32_t r = 0; r < n_req; ++r) n += 2ull * extents[r].n_blocks;
  if (n > 0 && !block_table) return ORC_EINVAL;
  const uint64_t cap = (uint64_t)n_slots * ORC_IOCB_SLOTS;
  const uint64_t n_fill = n < cap ? n : cap;

  for (uint32_t b = 0; b < n_slots; ++b) {
    orc_iocb *io = &sq[(first_slot + b) % depth];
    uint64_t lo = (uint64_t)b * ORC_IOCB_SLOTS;
    uint64_t cnt = n_fill > lo ? n_fill - lo : 0;
    if (cnt > ORC_IOCB_SLOTS) cnt = ORC_IOCB_SLOTS;
    io->hdr.num_ioctx = (uint32_t)cnt;
    io->hdr.state = ORC_IOCB_FILLED;
    io->hdr.done = 0;
    io->hdr.layer = layer;
    io->hdr.opcode = opcode;
  }
  uint32_t st = 0;
  for (uint32_t r = 0; r < n_req; ++r) {
    const orc_extent *x = &extents[r];
    for (uint32_t kind = 0; kind < 2; ++kind) {
      for (uint32_t j = 0; j < x->n_blocks; ++j) {
        uint64_t i = 2ull * x->table_off + (uint64_t)kind * x->n_blocks + j;
        if (i >= cap) {
          st |= ORC_ST_SQE_CAP;
          continue;
        }
        orc_iocb *io = &sq[(first_slot + (uint32_t)(i / ORC_IOCB_SLOTS)) % depth];
        orc_sqe *s = &io->ioctx[i % ORC_IOCB_SLOTS];
        st |= make_direct_entry(pool, x, r, kind, j, block_table[(uint64_t)x->table_off + j], file_id[r], layer, opcode,
                                sgl_table_addr, sgl_id, i, s);
      }
    }
  }
  if (status && st) *status |= st;
  return ORC_OK;
}

/*
 * issue_io (sec. 3.2): every context becomes one transfer between the block its SGL descriptor describes and
 * the GPU file at its offset; when an IOCB's contexts are done its index goes to the CQ.
 * The paper does not say what happens to a context that cannot be executed (the application may have filled
 * it by hand).  Reading taken: such a context is skipped and ORC_ST_BAD_BLOCK reported, and the IOCB still
 * completes.  A context cannot be executed when: its opcode is neither READ nor WRITE; its SGL address is not
 * that of a descriptor of the table (below it, not a multiple of 16 from it, index >= n_desc); its length is
 * not a multiple of 16, exceeds max_len or the descriptor's length; the block address or the file offset is
 * not a multiple of 16; the file id is outside the store; or [file_off, file_off + len) is not inside the file.
 * Length 0 is a no-op, not an error.
 */
int orc_issue_io(orc_iocb *sq, void *cq, uint32_t depth, uint32_t first_slot, uint32_t n_slots,
                 const orc_sgl *sgl_table, uint32_t n_desc, uint64_t sgl_table_addr, const orc_filestore *store,
                 uint32_t max_len, uint32_t *status) {
  if (!sq || !cq || depth == 0 || n_slots > depth || first_slot >= depth) return ORC_EINVAL;
  if (!store || !store->base || (n_desc > 0 && !sgl_table)) return ORC_EINVAL;
  if (max_len == 0 || max_len % 16 != 0 || sgl_table_addr % 16 != 0) return ORC_EINVAL;
  orc_cq_hdr *c = (orc_cq_hdr *)cq;
  uint32_t *entry = (uint32_t *)(c + 1);
  uint32_t st = 0;
  for (uint32_t b = 0; b < n_slots; ++b) {
    orc_iocb *io = &sq[(first_slot + b) % depth];
    if (io->hdr.state != ORC_IOCB_FILLED) continue; /* nothing was submitted in this slot */
    for (uint32_t k = 0; k < io->hdr.num_ioctx && k < ORC_IOCB_SLOTS; ++k) {
      const orc_sqe *s = &io->ioctx[k];
      if (s->len == 0) continue; /* a no-op context */
      if (s->opcode != ORC_OP_READ && s->opcode != ORC_OP_WRITE) {
        st |= ORC_ST_BAD_BLOCK;
        continue;
      }
      if (s->addr < sgl_table_addr || (s->addr - sgl_table_addr) % 16 != 0) {
        st |= ORC_ST_BAD_BLOCK;
        continue;
      }
      uint64_t di = (s->addr - sgl_table_addr) / 16;
      if (di >= n_desc || s->len > sgl_table[di].len) {
        st |= ORC_ST_BAD_BLOCK;
        continue;
      }
      if (s->len > max_len || s->len % 16 != 0 || s->file_off % 16 != 0 || sgl_table[di].addr % 16 != 0) {
        st |= ORC_ST_BAD_BLOCK;
        continue;
      }
      if (s->file_id < store->first_file_id || s->file_id - store->first_file_id >= store->n_files ||
          s->file_off > store->file_stride || s->len > store->file_stride - s->file_off) {
        st |= ORC_ST_BAD_BLOCK;
        continue;
      }
      uint8_t *blk = (uint8_t *)(uintptr_t)sgl_table[di].addr;
      uint8_t *fil = (uint8_t *)store->base + (uint64_t)(s->file_id - store->first_file_id) * store->file_stride + s->file_off;
      if (s->opcode == ORC_OP_READ)
        memcpy(blk, fil, s->len);
      else
        memcpy(fil, blk, s->len);
    }
    io->hdr.state = ORC_IOCB_DONE;
    io->hdr.done = io->hdr.num_ioctx;
    entry[c->tail % depth] = io->hdr.iocb_idx;
    c->tail += 1;
  }
  if (status && st) *status |= st;
  return ORC_OK;
}

/* ------------------------------------------------------------------ fused restore */

/* One layer's restore as the library's single call does it: extents, READ entries, unpack. */
int orc_layer_restore(const orc_pool *pool, const orc_objcfg *cfg, const uint32_t *n_blocks, uint32_t n_req,
                      const uint32_t *block_table, uint32_t table_len, const uint32_t *file_id, uint32_t layer,
                      const void *stage,
                      uint64_t stage_cap, uint64_t stage_addr, uint32_t sgl_id, orc_extent *extents,
                      uint64_t *totals, orc_sqe *sqe, uint32_t sqe_cap, uint32_t *status) {
  int rc = check_geometry(pool, cfg);
  if (rc) return rc;
  if (layer >= cfg->num_layers || stage_addr % cfg->align != 0) return ORC_EINVAL;
  if (n_req > 0 && (!file_id || !stage)) return ORC_EINVAL;
  if (!pool->k_base || !pool->v_base) return ORC_EINVAL;
  if (sqe_cap > 0 && !sqe) return ORC_EINVAL;
  rc = orc_obj_layout(pool, cfg, n_blocks, n_req, extents, totals);
  if (rc) return rc;
  rc = orc_sqe_build(pool, cfg, extents, n_req, file_id, layer, ORC_OP_READ, stage_addr, sgl_id, sqe, sqe_cap, status);
  if (rc) return rc;
  return orc_obj_unpack(pool, cfg, extents, n_req, block_table, table_len, stage, stage_cap, status);
}

/* One layer's save as the library's single call does it: extents, WRITE entries, pack (store_layer of sec. 3.4). */
int orc_layer_save(const orc_pool *pool, const orc_objcfg *cfg, const uint32_t *n_blocks, uint32_t n_req,
                   const uint32_t *block_table, uint32_t table_len, const uint32_t *file_id, uint32_t layer, void *stage,
                   uint64_t stage_cap, uint64_t stage_addr, uint32_t sgl_id, orc_extent *extents, uint64_t *totals,
                   orc_sqe *sqe, uint32_t sqe_cap, uint32_t *status) {
  int rc = check_geometry(pool, cfg);
  if (rc) return rc;
  if (layer >= cfg->num_layers || stage_addr % cfg->align != 0) return ORC_EINVAL;
  if (n_req > 0 && (!file_id || !stage)) return ORC_EINVAL;
  if (!pool->k_base || !pool->v_base) return ORC_EINVAL;
  if (sqe_cap > 0 && !sqe) return ORC_EINVAL;
  rc = orc_obj_layout(pool, cfg, n_blocks, n_req, extents, totals);
  if (rc) return rc;
  rc = orc_sqe_build(pool, cfg, extents, n_req, file_id, layer, ORC_OP_WRITE, stage_addr, sgl_id, sqe, sqe_cap, status);
  if (rc) return rc;
  return orc_obj_pack(pool, cfg, extents, n_req, block_table, table_len, stage, stage_cap, status);
}

/* retrieve_layer(layer) / store_layer(layer) of sec. 3.4 through the rings, in direct-to-block mode, written as
 * the sequence of the steps above: extents, the mapping table of this very pool (descriptors name the planes'
 * own addresses), the layer's contexts into IOCBs, then the I/O itself with its completions. */
static int ring_layer(uint32_t opcode, orc_iocb *sq, void *cq, uint32_t depth, uint32_t first_slot, uint32_t n_slots,
                      const orc_pool *pool, const orc_objcfg *cfg, const uint32_t *n_blocks, uint32_t n_req,
                      const uint32_t *block_table, const uint32_t *file_id, uint32_t layer, uint64_t sgl_table_addr,
                      uint32_t sgl_id, const orc_filestore *store, orc_extent *extents, uint64_t *totals,
                      uint32_t *status) {
  int rc = check_geometry(pool, cfg);
  if (rc) return rc;
  if (!pool->k_base || !pool->v_base || !cq) return ORC_EINVAL;
  rc = orc_obj_layout(pool, cfg, n_blocks, n_req, extents, totals);
  if (rc) return rc;
  const uint32_t n_desc = 2u * pool->num_blocks;
  orc_sgl *table = (orc_sgl *)malloc((size_t)n_desc * sizeof(orc_sgl));
  if (!table) return ORC_EINVAL;
  rc = orc_sgl_table_build(pool, (uint64_t)(uintptr_t)pool->k_base, (uint64_t)(uintptr_t)pool->v_base, sgl_id, table,
                           n_desc, NULL);
  if (!rc)
    rc = orc_iocb_fill_direct(sq, depth, first_slot, n_slots, pool, cfg, extents, n_req, block_table, file_id, layer,
                              opcode, sgl_table_addr, sgl_id, status);
  if (!rc)
    rc = orc_issue_io(sq, cq, depth, first_slot, n_slots, table, n_desc, sgl_table_addr, store, orc_block_bytes(pool),
                      status);
  free(table);
  return rc;
}

int orc_retrieve_layer(orc_iocb *sq, void *cq, uint32_t depth, uint32_t first_slot, uint32_t n_slots,
                       const orc_pool *pool, const orc_objcfg *cfg, const uint32_t *n_blocks, uint32_t n_req,
                       const uint32_t *block_table, const uint32_t *file_id, uint32_t layer, uint64_t sgl_table_addr,
                       uint32_t sgl_id, const orc_filestore *store, orc_extent *extents, uint64_t *totals,
                       uint32_t *status) {
  return ring_layer(ORC_OP_READ, sq, cq, depth, first_slot, n_slots, pool, cfg, n_blocks, n_req, block_table, file_id,
                    layer, sgl_table_addr, sgl_id, store, extents, totals, status);
}

int orc_store_layer(orc_iocb *sq, void *cq, uint32_t depth, uint32_t first_slot, uint32_t n_slots,
                    const orc_pool *pool, const orc_objcfg *cfg, const uint32_t *n_blocks, uint32_t n_req,
                    const uint32_t *block_table, const uint32_t *file_id, uint32_t layer, uint64_t sgl_table_addr,
                    uint32_t sgl_id, const orc_filestore *store, orc_extent *extents, uint64_t *totals,
                    uint32_t *status) {
  return ring_layer(ORC_OP_WRITE, sq, cq, depth, first_slot, n_slots, pool, cfg, n_blocks, n_req, block_table, file_id,
                    layer, sgl_table_addr, sgl_id, store, extents, totals, status);
}

int orc_table_validate(uint32_t num_blocks, const uint32_t *block_table, uint32_t table_len, uint32_t *status) {
  if (num_blocks == 0 || !status || (table_len > 0 && !block_table)) return ORC_EINVAL;
  uint8_t *seen = (uint8_t *)calloc(num_blocks, 1);
  if (!seen) return ORC_EINVAL;
  uint32_t st = 0;
  for (uint32_t i = 0; i < table_len; ++i) {
    const uint32_t id = block_table[i];
    if (id >= num_blocks) {
      st |= ORC_ST_BAD_BLOCK;
    } else if (seen[id]) {
      st |= ORC_ST_DUP_BLOCK;
    } else {
      seen[id] = 1;
    }
  }
  free(seen);
  *status |= st;
  return ORC_OK;
}

/* ------------------------------------------------------------------ visiting order */

/*
 * The order in which a restore may visit the blocks of a table so that it walks the pool by ascending address:
 * visit[k] = the table position of the k-th smallest block id.  The paper keeps token order (sec. 3.1: an object
 * holds a request's blocks as they come); the visiting order is this repository's addition and changes no result,
 * only the order of the writes.  A table that a restore may not use anyway (an id out of range, or an id twice:
 * orc_table_validate) gets the identity order, and the status bits say why.
 */
int orc_table_order(uint32_t num_blocks, const uint32_t *block_table, uint32_t table_len, uint32_t *visit,
                    uint32_t *status) {
  if (num_blocks == 0 || (table_len > 0 && (!block_table || !visit))) return ORC_EINVAL;
  uint32_t st = 0;
  int rc = orc_table_validate(num_blocks, block_table, table_len, &st);
  if (rc) return rc;
  if (status) *status |= st;
  for (uint32_t k = 0; k < table_len; ++k) visit[k] = k;
  if (st) return ORC_OK;
  /* insertion sort of the positions by block id: plain, quadratic, obviously an ascending order */
  for (uint32_t k = 1; k < table_len; ++k) {
    uint32_t pos = visit[k];
    uint32_t m = k;
    while (m > 0 && block_table[visit[m - 1]] > block_table[pos]) {
      visit[m] = visit[m - 1];
      --m;
    }
    visit[m] = pos;
  }
  return ORC_OK;
}

/*
 * One layer's restore with the blocks visited in the order `visit` gives (table positions, table_len of them):
 * extents and READ entries as orc_layer_restore, then for every listed position, in list order, the K block and
 * the V block it names.  A position that lies beyond the blocks the requests claim (or beyond table_len) is
 * passed over; a position listed twice is restored twice; one not listed is not restored.  With a permutation of
 * the positions the result is orc_layer_restore's.
 */
int orc_layer_restore_ordered(const orc_pool *pool, const orc_objcfg *cfg, const uint32_t *n_blocks, uint32_t n_req,
                              const uint32_t *block_table, uint32_t table_len, const uint32_t *file_id, uint32_t layer,
                              const void *stage, uint64_t stage_cap, uint64_t stage_addr, uint32_t sgl_id,
                              orc_extent *extents, uint64_t *totals, orc_sqe *sqe, uint32_t sqe_cap,
                              const uint32_t *visit, uint32_t *status) {
  int rc = check_geometry(pool, cfg);
  if (rc) return rc;
  if (layer >= cfg->num_layers || stage_addr % cfg->align != 0) return ORC_EINVAL;
  if (n_req > 0 && (!file_id || !stage)) return ORC_EINVAL;
  if (!pool->k_base || !pool->v_base) return ORC_EINVAL;
  if (sqe_cap > 0 && !sqe) return ORC_EINVAL;
  if (table_len > 0 && (!visit || !block_table)) return ORC_EINVAL;
  rc = orc_obj_layout(pool, cfg, n_blocks, n_req, extents, totals);
  if (rc) return rc;
  rc = orc_sqe_build(pool, cfg, extents, n_req, file_id, layer, ORC_OP_READ, stage_addr, sgl_id, sqe, sqe_cap, status);
  if (rc) return rc;
  const uint64_t bb = orc_block_bytes(pool);
  uint32_t st = 0;
  /* the requests that take part: in order, while their blocks fit the table (as in orc_obj_unpack) */
  uint64_t live_blocks = 0;
  uint32_t live_req = 0;
  while (live_req < n_req && live_blocks + extents[live_req].n_blocks <= table_len) {
    live_blocks += extents[live_req].n_blocks;
    ++live_req;
  }
  if (live_req < n_req) st |= ORC_ST_BAD_EXTENT;
  for (uint32_t r = 0; r < live_req; ++r)
    if (extents[r].stage_off > stage_cap || extents[r].obj_bytes > (stage_cap - extents[r].stage_off) / 2)
      st |= ORC_ST_STAGE_CAP;
  for (uint32_t kind = 0; kind < 2; ++kind) {
    uint8_t *plane = (uint8_t *)(kind == 0 ? pool->k_base : pool->v_base);
    for (uint32_t k = 0; k < table_len; ++k) {
      const uint64_t pos = visit[k];
      if (pos >= live_blocks) continue; /* not a block of a request that takes part */
      uint32_t r = 0;
      while (pos >= (uint64_t)extents[r].table_off + extents[r].n_blocks) ++r; /* the request that owns it */
      const orc_extent *x = &extents[r];
      if (x->stage_off > stage_cap || x->obj_bytes > (stage_cap - x->stage_off) / 2) continue;
      const uint64_t j = pos - x->table_off;
      const uint32_t id = block_table[pos];
      if (id >= pool->num_blocks) {
        st |= ORC_ST_BAD_BLOCK;
        continue;
      }
      uint8_t *obj = (uint8_t *)(uintptr_t)stage + x->stage_off + kind * x->obj_bytes;
      move_block(pool, plane + (uint64_t)id * pool->block_stride, obj + j * bb, 0);
    }
  }
  if (status && st) *status |= st;
  return ORC_OK;
}

/* ------------------------------------------------------------------ threaded timing helpers */

typedef struct {
  const orc_pool *pool;
  const orc_extent *extents;
  uint32_t n_req;
  const uint32_t *block_table;
  uint32_t table_len;
  uint8_t *stage;
  uint64_t stage_cap;
  int to_object;
  uint64_t g_lo, g_hi;
} mt_job;

static void *mt_run(void *p) {
  mt_job *j = (mt_job *)p;
  move_range(j->pool, j->extents, j->n_req, j->block_table, j->table_len, j->stage, j->stage_cap, j->to_object, j->g_lo,
             j->g_hi, NULL);
  return NULL;
}

static int move_mt(const orc_pool *pool, const orc_objcfg *cfg, const orc_extent *extents, uint32_t n_req,
                   const uint32_t *block_table, uint32_t table_len, uint8_t *stage, uint64_t stage_cap, int to_object,
                   uint32_t n_threads) {
  int rc = check_move_args(pool, cfg, extents, n_req, block_table, table_len, stage);
  if (rc) return rc;
  if (n_threads == 0 || n_threads > 1024) return ORC_ERANGE;
  uint64_t n = table_len; /* table positions, split evenly over the threads */
  pthread_t tid[1024];
  mt_job job[1024];
  uint32_t started = 0;
  for (uint32_t t = 0; t < n_threads; ++t) {
    job[t].pool = pool;
    job[t].extents = extents;
    job[t].n_req = n_req;
    job[t].block_table = block_table;
    job[t].table_len = table_len;
    job[t].stage = stage;
    job[t].stage_cap = stage_cap;
    job[t].to_object = to_object;
    job[t].g_lo = n * t / n_threads;
    job[t].g_hi = n * (t + 1) / n_threads;
    if (pthread_create(&tid[t], NULL, mt_run, &job[t]) != 0) break;
    ++started;
  }
  for (uint32_t t = 0; t < started; ++t) pthread_join(tid[t], NULL);
  return started == n_threads ? ORC_OK : ORC_ERANGE;
}

int orc_obj_pack_mt(const orc_pool *pool, const orc_objcfg *cfg, const orc_extent *extents, uint32_t n_req,
                    const uint32_t *block_table, uint32_t table_len, void *stage, uint64_t stage_cap,
                    uint32_t n_threads) {
  return move_mt(pool, cfg, extents, n_req, block_table, table_len, (uint8_t *)stage, stage_cap, 1, n_threads);
}

int orc_obj_unpack_mt(const orc_pool *pool, const orc_objcfg *cfg, const orc_extent *extents, uint32_t n_req,
                      const uint32_t *block_table, uint32_t table_len, const void *stage, uint64_t stage_cap,
                      uint32_t n_threads) {
  return move_mt(pool, cfg, extents, n_req, block_table, table_len, (uint8_t *)(uintptr_t)stage, stage_cap, 0,
                 n_threads);
}
