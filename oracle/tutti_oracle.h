/*
 * tutti_oracle.h -- CPU oracle for the per-layer KV object path. TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, single-threaded, obviously-correct host implementation of what the GPU
 * library computes: object extents, pack (paged blocks -> contiguous per-layer objects),
 * unpack (objects -> paged blocks) and submission-entry construction.  It exists so that
 * the tests, the smoke check and the benchmark's cpu_baseline leg can compare the HIP path
 * against an independent definition.  Nothing on the product path may include, link or
 * call it, and it shares no source, header, table or helper with the HIP library: every
 * record below is re-declared here on purpose (a test checks that both sides agree on
 * sizeof/offsetof).
 *
 * What the paper fixes and what is this repository's reading of it:
 *   - a paged KV block has shape [Block, h, d] (sec. 2.1, "Paged KV Memory Management");
 *   - there is one key object and one value object per layer, and a GPU file holds 2*L
 *     objects (sec. 3.1, "Scalable GPU File Pool");
 *   - an I/O context carries an SGL address, a GPU-file offset and a length, and 2048 of
 *     them form one IOCB = one submission-queue entry (sec. 3.2, "Zero-Copy Ring Buffers");
 *   - an SGL descriptor is 16 bytes: address 8, length 4, identifier 4 (sec. 3.1, "P2P
 *     Memory Mapping Table").
 *   The paper gives no byte layout for any record, no alignment unit, no chunk size, no
 *   order of the 2*L objects in a file and no padding content.  Those are repository
 *   readings: 4 KiB alignment, caller-chosen chunk size, layer-major K-then-V object
 *   order, zero padding.  The record layouts, user_data packing and these readings are
 *   "parity unpinned" by the paper: they are pinned only by closed forms, invariants and
 *   brute force in the CPU tests.
 *
 * All pointers are HOST pointers.  Every function returns 0 on success and a negative
 * ORC_E* code on bad arguments; nothing is written on error.
 */
#ifndef TUTTI_ORACLE_H
#define TUTTI_ORACLE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define ORC_OK 0
#define ORC_EINVAL (-1)
#define ORC_ERANGE (-2)

#define ORC_LAYOUT_NHD 0u /* block stored [T][h][d]  (the paper's [Block, h, d]) */
#define ORC_LAYOUT_HND 1u /* block stored [h][T][d]  (head-major engines)        */

#define ORC_OP_READ 1u  /* object -> HBM, restore */
#define ORC_OP_WRITE 2u /* HBM -> object, save    */

#define ORC_IOCB_SLOTS 2048u /* I/O contexts per IOCB, sec. 3.2 */

/* Bits of the optional status word (ORed in, never cleared, by pack / unpack / restore). */
#define ORC_ST_BAD_BLOCK 1u  /* a block-table entry >= num_blocks: that block was skipped */
#define ORC_ST_STAGE_CAP 2u  /* a request's objects end beyond stage_cap: the request was skipped */
#define ORC_ST_SQE_CAP 4u    /* more entries than sqe_cap: the excess was not written */
#define ORC_ST_DUP_BLOCK 8u  /* orc_table_validate only: a block id appears more than once in the table */
#define ORC_ST_BAD_EXTENT 16u /* pack / unpack: an extent that cannot be honoured (see orc_obj_pack) */

/* One layer's paged pool: a K plane and a V plane of num_blocks blocks each. */
typedef struct {
  void *k_base;
  void *v_base;
  uint64_t block_stride; /* bytes between consecutive blocks of a plane, >= block_bytes */
  uint32_t num_blocks;
  uint32_t block_tokens; /* T */
  uint32_t num_kv_heads; /* h */
  uint32_t head_dim;     /* d */
  uint32_t elt_bytes;    /* e */
  uint32_t pool_layout;  /* ORC_LAYOUT_* */
} orc_pool;

typedef struct {
  uint32_t align;       /* object alignment unit A, power of two >= 16 */
  uint32_t chunk_bytes; /* C, multiple of A: one submission entry covers at most C bytes */
  uint32_t num_layers;  /* L */
} orc_objcfg;

/* Per-request extent, identical for every layer. */
typedef struct {
  uint64_t stage_off; /* byte offset of the request's K object in the layer's staging buffer */
  uint64_t obj_bytes; /* align_up(n_blocks*block_bytes, A); the V object follows the K object */
  uint32_t n_blocks;
  uint32_t n_chunks;  /* ceil(obj_bytes / C), per object */
  uint32_t sqe_base;  /* index of the request's first entry in the layer's entry array */
  uint32_t table_off; /* index of the request's first entry in the flattened block table */
} orc_extent;

/* Submission entry, 64 bytes, little-endian, naturally aligned. */
typedef struct {
  uint8_t opcode;
  uint8_t kind; /* 0 = K object, 1 = V object */
  uint16_t layer;
  uint32_t file_id;
  uint64_t file_off;
  uint64_t addr;
  uint32_t len;
  uint32_t sgl_id;
  uint64_t user_data; /* (request << 32) | entry index within the layer */
  uint32_t iocb_idx;
  uint32_t ioctx_slot;
  uint8_t rsvd[16];
} orc_sqe;

/* Size/offset table of the records above, for the cross-check against the library's header:
 * out[0..]: sizeof(extent), offsets of its 6 fields, sizeof(sqe), offsets of its 11 fields,
 * sizeof(pool), offsets of its 9 fields, sizeof(objcfg), offsets of its 3 fields, sizeof(sgl), offsets of
 * its 3 fields, sizeof(iocb_hdr), offsets of its 6 named fields, sizeof(iocb), offset of its contexts,
 * sizeof(cq_hdr), sizeof(filestore), offsets of its 4 fields (52 values). */
int orc_abi_describe(uint32_t *out, uint32_t cap);

/* T*h*d*e, or 0 if any factor is 0 or the product does not fit 32 bits. */
uint32_t orc_block_bytes(const orc_pool *pool);

/* Extents of n_req requests; totals[0] = staging bytes of one layer, totals[1] = entries of one layer. */
int orc_obj_layout(const orc_pool *pool, const orc_objcfg *cfg, const uint32_t *n_blocks, uint32_t n_req,
                   orc_extent *extents, uint64_t *totals);

/* Paged blocks -> objects.  stage receives, per request, the K object (at stage_off) then the V object
 * (obj_bytes later), each zero-padded from n_blocks*block_bytes to obj_bytes; block j of request r is the
 * one table entry table_off_r + j names.  The extents are honoured field by field, whoever wrote them
 * (gaps between requests, any order in the staging buffer, a table range that does not start at 0).
 * What cannot be honoured is skipped and reported in *status (may be NULL), in this order per request:
 *   running sum of n_blocks over the requests so far > table_len   request and all later ones skipped, BAD_EXTENT
 *   stage_off or obj_bytes not a multiple of 16                    request skipped, BAD_EXTENT
 *   stage_off + 2*obj_bytes > stage_cap                            request skipped, STAGE_CAP
 *   (j+1)*block_bytes > obj_bytes                                  block skipped, BAD_EXTENT
 *   table_off + j >= table_len, or the id there >= num_blocks      block skipped, BAD_BLOCK
 * A skipped block leaves its object bytes as they were. */
int orc_obj_pack(const orc_pool *pool, const orc_objcfg *cfg, const orc_extent *extents, uint32_t n_req,
                 const uint32_t *block_table, uint32_t table_len, void *stage, uint64_t stage_cap, uint32_t *status);

/* Objects -> paged blocks, same rules; padding is not read; blocks not named in the table are not touched. */
int orc_obj_unpack(const orc_pool *pool, const orc_objcfg *cfg, const orc_extent *extents, uint32_t n_req,
                   const uint32_t *block_table, uint32_t table_len, const void *stage, uint64_t stage_cap,
                   uint32_t *status);

/* One entry per chunk of every K and V object of one layer.  Entries with index >= sqe_cap are not written.
 * The entry builders (this one, orc_sqe_build_direct, orc_iocb_fill_direct) take extents exactly as orc_obj_layout
 * writes them for these n_req requests (sqe_base and table_off running from 0 without gaps, obj_bytes and n_chunks
 * following from n_blocks; stage_off is free); handed anything else they write nothing and set ORC_ST_BAD_EXTENT. */
int orc_sqe_build(const orc_pool *pool, const orc_objcfg *cfg, const orc_extent *extents, uint32_t n_req,
                  const uint32_t *file_id, uint32_t layer, uint32_t opcode, uint64_t stage_addr, uint32_t sgl_id,
                  orc_sqe *sqe, uint32_t sqe_cap, uint32_t *status);

/* layout, then READ entries, then unpack, for one layer. */
int orc_layer_restore(const orc_pool *pool, const orc_objcfg *cfg, const uint32_t *n_blocks, uint32_t n_req,
                      const uint32_t *block_table, uint32_t table_len, const uint32_t *file_id, uint32_t layer,
                      const void *stage, uint64_t stage_cap, uint64_t stage_addr, uint32_t sgl_id, orc_extent *extents,
                      uint64_t *totals, orc_sqe *sqe, uint32_t sqe_cap, uint32_t *status);

/* layout, then WRITE entries, then pack, for one layer (the save direction of the fused call). */
int orc_layer_save(const orc_pool *pool, const orc_objcfg *cfg, const uint32_t *n_blocks, uint32_t n_req,
                   const uint32_t *block_table, uint32_t table_len, const uint32_t *file_id, uint32_t layer,
                   void *stage, uint64_t stage_cap, uint64_t stage_addr, uint32_t sgl_id, orc_extent *extents, uint64_t *totals,
                   orc_sqe *sqe, uint32_t sqe_cap, uint32_t *status);

/* ---- direct-to-block mode: the paper's own data path, no staging copy (sec. 3.1, "P2P Memory
 * Mapping Table"; sec. 3.2: an I/O context records the SGL address, the GPU-file offset and the length).
 *
 * 16-byte SGL descriptor of one pool block: address 8, length 4, identifier 4. */
typedef struct {
  uint64_t addr;
  uint32_t len;
  uint32_t id;
} orc_sgl;

/* The mapping table of one layer's pool, computed once at start-up: descriptor b describes K block b,
 * descriptor num_blocks + b describes V block b: { base + b*block_stride, block_bytes, sgl_id }.
 * k_addr / v_addr are the addresses the descriptors should name for the two planes (arithmetic only).
 * Descriptors with index >= cap are not written (ORC_ST_SQE_CAP). */
int orc_sgl_table_build(const orc_pool *pool, uint64_t k_addr, uint64_t v_addr, uint32_t sgl_id, orc_sgl *table,
                        uint32_t cap, uint32_t *status);

/* One entry per (hit block, K|V) of one layer, in the order request ascending, K then V, block ascending:
 * index = 2*table_off_r + kind*n_r + j.  addr = sgl_table_addr + 16*(kind*num_blocks + id) (the block's
 * descriptor), len = block_bytes, file_off = (2*layer + kind)*obj_bytes_r + j*block_bytes, i.e. the same
 * GPU-file layout as the staged mode.  block_bytes must be a multiple of the alignment unit.  A block id
 * >= num_blocks yields an entry with addr = 0 and len = 0 and sets ORC_ST_BAD_BLOCK. */
int orc_sqe_build_direct(const orc_pool *pool, const orc_objcfg *cfg, const orc_extent *extents, uint32_t n_req,
                         const uint32_t *block_table, const uint32_t *file_id, uint32_t layer, uint32_t opcode,
                         uint64_t sgl_table_addr, uint32_t sgl_id, orc_sqe *sqe, uint32_t sqe_cap, uint32_t *status);

/* ---- submission / completion rings (sec. 3.2 "Zero-Copy Ring Buffers", "Async I/O Processing").
 * An SQ entry is an IOCB: a 64-byte header and 2048 I/O contexts (submission entries).  The CQ holds
 * the indices of completed IOCBs.  Repository readings: the header layout, the CQ layout (tail counter
 * + index array) and the file store that stands in for the SSD are not fixed by the paper. */
#define ORC_IOCB_FREE 0u
#define ORC_IOCB_FILLED 1u
#define ORC_IOCB_DONE 2u

typedef struct {
  uint32_t iocb_idx;  /* unique index = slot in the SQ */
  uint32_t num_ioctx; /* valid contexts */
  uint32_t state;     /* ORC_IOCB_* */
  uint32_t done;      /* contexts completed: 0 while FILLED, num_ioctx once DONE */
  uint32_t layer;
  uint32_t opcode;
  uint32_t rsvd[10];
} orc_iocb_hdr;

typedef struct {
  orc_iocb_hdr hdr;
  orc_sqe ioctx[ORC_IOCB_SLOTS];
} orc_iocb;

typedef struct {
  uint32_t tail; /* completions so far */
  uint32_t depth;
  uint32_t rsvd[14];
  /* followed by uint32_t entry[depth]: entry[t % depth] = index of the t-th completed IOCB */
} orc_cq_hdr;

/* The stand-in for the SSD: n_files GPU files of file_stride bytes, file f at base + (f - first_file_id)*file_stride. */
typedef struct {
  void *base;
  uint64_t file_stride;
  uint32_t first_file_id;
  uint32_t n_files;
} orc_filestore;

/* init_queue(depth): every IOCB free with its unique index, CQ empty. */
int orc_ring_init(orc_iocb *sq, void *cq, uint32_t depth);

/* get_iocb + fill for one layer in direct-to-block mode: context i of orc_sqe_build_direct goes to IOCB slot
 * (first_slot + i / 2048) % depth, position i % 2048.  All n_slots IOCBs become FILLED with their num_ioctx
 * (0 if unused), layer and opcode.  Contexts beyond n_slots*2048 are dropped (ORC_ST_SQE_CAP). */
int orc_iocb_fill_direct(orc_iocb *sq, uint32_t depth, uint32_t first_slot, uint32_t n_slots, const orc_pool *pool,
                         const orc_objcfg *cfg, const orc_extent *extents, uint32_t n_req, const uint32_t *block_table,
                         const uint32_t *file_id, uint32_t layer, uint32_t opcode, uint64_t sgl_table_addr,
                         uint32_t sgl_id, uint32_t *status);

/* issue_io: execute every context of the n_slots IOCBs starting at first_slot, in order: resolve the SGL
 * descriptor the context names (index (addr - sgl_table_addr)/16 into sgl_table, n_desc entries), then move
 * len bytes between that block and the request's GPU file at file_off (READ: file -> block, WRITE: block ->
 * file).  The descriptor's address is used as a host pointer here.  Each IOCB is then marked DONE and its
 * index appended to the CQ.  A context that cannot be executed is skipped (ORC_ST_BAD_BLOCK): opcode neither
 * READ nor WRITE; address not that of a descriptor of the table; length not a multiple of 16 or beyond max_len
 * or the descriptor's length; block address or file offset not a multiple of 16; file id outside the store;
 * [file_off, file_off + len) not inside the file.  Length 0 is a no-op.  max_len: multiple of 16, > 0. */
int orc_issue_io(orc_iocb *sq, void *cq, uint32_t depth, uint32_t first_slot, uint32_t n_slots,
                 const orc_sgl *sgl_table, uint32_t n_desc, uint64_t sgl_table_addr, const orc_filestore *store,
                 uint32_t max_len, uint32_t *status);

/* retrieve_layer(layer) / store_layer(layer) (sec. 3.4) through the rings in direct-to-block mode: extents of
 * the requests, the layer's contexts into n_slots IOCBs from first_slot, their execution against the file
 * store and the completions: orc_obj_layout, orc_iocb_fill_direct and orc_issue_io in that order, with the
 * mapping table of this very pool (orc_sgl_table_build at the planes' own addresses).  extents (n_req records)
 * and totals (2 values) are outputs. */
int orc_retrieve_layer(orc_iocb *sq, void *cq, uint32_t depth, uint32_t first_slot, uint32_t n_slots,
                       const orc_pool *pool, const orc_objcfg *cfg, const uint32_t *n_blocks, uint32_t n_req,
                       const uint32_t *block_table, const uint32_t *file_id, uint32_t layer, uint64_t sgl_table_addr,
                       uint32_t sgl_id, const orc_filestore *store, orc_extent *extents, uint64_t *totals,
                       uint32_t *status);
int orc_store_layer(orc_iocb *sq, void *cq, uint32_t depth, uint32_t first_slot, uint32_t n_slots,
                    const orc_pool *pool, const orc_objcfg *cfg, const uint32_t *n_blocks, uint32_t n_req,
                    const uint32_t *block_table, const uint32_t *file_id, uint32_t layer, uint64_t sgl_table_addr,
                    uint32_t sgl_id, const orc_filestore *store, orc_extent *extents, uint64_t *totals,
                    uint32_t *status);

/* The preconditions an unpack places on its table, checked: every id below num_blocks (else ORC_ST_BAD_BLOCK) and
 * no id twice (else ORC_ST_DUP_BLOCK: two writers to one block, whose result would depend on their order).  Out-of-
 * range ids are not counted as duplicates of each other.  *status receives the bits (ORed in). */
int orc_table_validate(uint32_t num_blocks, const uint32_t *block_table, uint32_t table_len, uint32_t *status);

/* visit[k] = table position of the k-th smallest block id (an ascending walk through the pool); the identity, with
 * the bits of orc_table_validate in *status, for a table with an id out of range or an id twice. */
int orc_table_order(uint32_t num_blocks, const uint32_t *block_table, uint32_t table_len, uint32_t *visit,
                    uint32_t *status);

/* orc_layer_restore with the blocks visited in the listed order of table positions (table_len entries).  A
 * position beyond the blocks of the requests that take part is passed over, one listed twice is restored twice,
 * one not listed is not restored; a permutation gives exactly orc_layer_restore's result. */
int orc_layer_restore_ordered(const orc_pool *pool, const orc_objcfg *cfg, const uint32_t *n_blocks, uint32_t n_req,
                              const uint32_t *block_table, uint32_t table_len, const uint32_t *file_id, uint32_t layer,
                              const void *stage, uint64_t stage_cap, uint64_t stage_addr, uint32_t sgl_id,
                              orc_extent *extents, uint64_t *totals, orc_sqe *sqe, uint32_t sqe_cap,
                              const uint32_t *visit, uint32_t *status);

/* Descriptor count for a pool of pool_bytes described at gran bytes per descriptor
 * (the arithmetic of sec. 3.1, "P2P Memory Mapping Table"). */
uint64_t orc_desc_count(uint64_t pool_bytes, uint64_t gran);

/* Timing helpers for the benchmark's cpu_baseline leg only: the same per-block copies as
 * orc_obj_pack / orc_obj_unpack, with the flattened block range split evenly over n_threads
 * POSIX threads.  Parity never uses these. */
int orc_obj_pack_mt(const orc_pool *pool, const orc_objcfg *cfg, const orc_extent *extents, uint32_t n_req,
                    const uint32_t *block_table, uint32_t table_len, void *stage, uint64_t stage_cap,
                    uint32_t n_threads);
int orc_obj_unpack_mt(const orc_pool *pool, const orc_objcfg *cfg, const orc_extent *extents, uint32_t n_req,
                      const uint32_t *block_table, uint32_t table_len, const void *stage, uint64_t stage_cap,
                      uint32_t n_threads);

#ifdef __cplusplus
}
#endif
#endif
