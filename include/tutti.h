/*
 * tutti.h -- C ABI of libtutti: the per-layer KV-object hot path on one MI355X (gfx950).
 *
 * The library moves one layer's KV cache between the paged blocks an inference engine keeps
 * scattered in HBM and contiguous, aligned per-layer KV objects (pack on save, unpack on
 * restore), and builds the submission entries that describe those objects' I/O, all on the
 * GPU, so the host does a constant amount of work per layer whatever the number of blocks
 * (the paper's O(layer) instead of O(layer x blocks): sec. 1 and sec. 3.1).
 *
 * Conventions for every entry point
 *   - Pointers named d_* are DEVICE pointers owned by the caller; tutti_pool / tutti_objcfg
 *     pointers are HOST pointers read during the call.  `stream` is a hipStream_t passed as
 *     void* (NULL = the null stream).
 *   - The library allocates no device memory and keeps no state between calls: what a call does
 *     depends on its arguments alone (the pool is fixed for the engine's lifetime and nothing on
 *     the I/O path may allocate: sec. 3.1 "P2P Memory Mapping Table", sec. 3.2 "Zero-Copy Ring
 *     Buffers").  The one exception is stated where it is declared: tutti_table_validate_static
 *     works in a fixed array inside the library.  Launch-tuning knobs and baseline kernels for
 *     measurements live in a separate library (tutti_bench.h), not here.
 *   - A call validates its host arguments in O(1), enqueues a constant number of kernels on
 *     `stream` and returns; it never synchronises and never copies to the host.  Results are
 *     valid once the caller has synchronised the stream.  (The set-up calls tutti_place_* are
 *     the exception, stated where they are declared: they time launches and block.)
 *   - Return value: 0 (TUTTI_OK) or a negative TUTTI_E* code; on error nothing was enqueued.
 *   - What only the device can know is reported through the optional status word d_status
 *     (TUTTI_ST_* bits, ORed in atomically, never cleared by the library) and never causes an
 *     out-of-bounds access: offending blocks / requests / entries are skipped.
 *   - Overlapping calls that write the same blocks or the same staging bytes race.
 */
#ifndef TUTTI_H
#define TUTTI_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define TUTTI_OK 0
#define TUTTI_EINVAL (-1) /* null pointer, zero dimension, bad alignment / layout / opcode / layer */
#define TUTTI_ERANGE (-2) /* n_req > TUTTI_MAX_REQ, cu_budget > number of CUs */
#define TUTTI_EHIP (-3)   /* a HIP call failed; see tutti_last_hip_error() */
#define TUTTI_EAGAIN (-4) /* host-side ring calls: not enough free IOCBs now / no budget fits the slack window */

#define TUTTI_LAYOUT_NHD 0u /* block stored [T][h][d]: the paper's [Block, h, d] (sec. 2.1) */
#define TUTTI_LAYOUT_HND 1u /* block stored [h][T][d]: head-major engines; objects stay token-major */

#define TUTTI_OP_READ 1u  /* object -> HBM (restore / retrieve_layer) */
#define TUTTI_OP_WRITE 2u /* HBM -> object (save / store_layer) */

#define TUTTI_IOCB_SLOTS 2048u /* I/O contexts per IOCB (sec. 3.2 "Zero-Copy Ring Buffers") */
#define TUTTI_MAX_REQ 2048u    /* requests per call */

#define TUTTI_ST_BAD_BLOCK 1u /* a block-table entry >= num_blocks, or beyond table_len: block skipped */
#define TUTTI_ST_STAGE_CAP 2u /* a request's objects end beyond stage_cap: request skipped */
#define TUTTI_ST_SQE_CAP 4u   /* more entries than sqe_cap: the excess was not written */
#define TUTTI_ST_DUP_BLOCK 8u /* tutti_table_validate* and tutti_table_order only: a block id appears twice in the table */
#define TUTTI_ST_BAD_EXTENT 16u /* an extent that cannot be honoured: see tutti_obj_pack and tutti_sqe_build */

/* One layer's paged pool (sec. 2.1 "Paged KV Memory Management"): a K plane and a V plane, each
 * num_blocks blocks of T*h*d*e bytes, block b at base + b*block_stride.  Planes stay owned by the
 * caller.  Requirements: bases and block_stride multiples of 16; T*h*d*e a multiple of 16.
 * The two planes may lie anywhere.  Measured on the MI355X: its 288 GB of HBM behave as three regions of 96 GB, and
 * a restore (32 KiB blocks scattered over the K plane, then over the V plane) runs at the speed of a contiguous
 * copy when the two planes lie in different regions, 15 % slower when they share one; tutti_place_classify and
 * tutti_place_pairs below find such pairs of buffers by timing when a pool is created. */
typedef struct tutti_pool {
  void *k_base;
  void *v_base;
  uint64_t block_stride;
  uint32_t num_blocks;
  uint32_t block_tokens; /* T */
  uint32_t num_kv_heads; /* h */
  uint32_t head_dim;     /* d */
  uint32_t elt_bytes;    /* e */
  uint32_t pool_layout;  /* TUTTI_LAYOUT_* */
} tutti_pool;

/* Object geometry: `align` is the alignment unit of every object and offset (power of two >= 16,
 * 4096 in every workload here), `chunk_bytes` the largest span one submission entry covers
 * (multiple of align), `num_layers` the L of the 2*L objects in a GPU file (sec. 3.1). */
typedef struct tutti_objcfg {
  uint32_t align;
  uint32_t chunk_bytes;
  uint32_t num_layers;
} tutti_objcfg;

/* Extent of one request's objects; the same for every layer.  32 bytes. */
typedef struct tutti_extent {
  uint64_t stage_off; /* offset of the K object in the layer's staging buffer; multiple of align */
  uint64_t obj_bytes; /* align_up(n_blocks * block_bytes, align); the V object follows the K object */
  uint32_t n_blocks;
  uint32_t n_chunks;  /* ceil(obj_bytes / chunk_bytes), per object */
  uint32_t sqe_base;  /* index of the request's first submission entry of a layer */
  uint32_t table_off; /* index of the request's first entry in the flattened block table */
} tutti_extent;

/* Submission entry: 64 bytes, little-endian.  It carries what the paper's I/O context records
 * (SGL address, GPU-file offset, length: sec. 3.2), the 16-byte SGL triple address / length /
 * identifier (sec. 3.1 "P2P Memory Mapping Table") and the entry's place in the 2048-slot IOCBs. */
typedef struct tutti_sqe {
  uint8_t opcode;      /* TUTTI_OP_* */
  uint8_t kind;        /* 0 = K object, 1 = V object */
  uint16_t layer;
  uint32_t file_id;    /* GPU file of the request (caller-supplied) */
  uint64_t file_off;   /* (2*layer + kind) * obj_bytes + chunk * chunk_bytes */
  uint64_t addr;       /* stage_addr + stage_off + kind * obj_bytes + chunk * chunk_bytes */
  uint32_t len;        /* min(chunk_bytes, rest of the object); multiple of align */
  uint32_t sgl_id;     /* caller-supplied registration identifier */
  uint64_t user_data;  /* (request << 32) | entry index within the layer */
  uint32_t iocb_idx;   /* entry index / 2048 */
  uint32_t ioctx_slot; /* entry index % 2048 */
  uint8_t rsvd[16];    /* zero */
} tutti_sqe;

/* ---- a1: extents.  Sec. 3.1 "Scalable GPU File Pool" (a K object and a V object per layer in a request's GPU
 * file), sec. 3.2 (offset and length of an I/O context).  For request r with n_r = d_n_blocks[r] hit blocks:
 * obj_bytes = align_up(n_r*block_bytes, align), n_chunks = ceil(obj_bytes/chunk_bytes); stage_off,
 * sqe_base and table_off are the exclusive prefix sums over r of 2*obj_bytes, 2*n_chunks and n_r.
 * Writes d_extents[0..n_req) and d_totals[0] = staging bytes of a layer, d_totals[1] = entries of a
 * layer.  n_req may be 0.  sqe_base / table_off are meaningful only while the totals fit 32 bits. */
int tutti_obj_layout(const tutti_pool *pool, const tutti_objcfg *cfg, const uint32_t *d_n_blocks, uint32_t n_req,
                     tutti_extent *d_extents, uint64_t *d_totals, void *stream);

/* ---- a2: pack (save; store_layer of sec. 3.4 "Integration with vLLM"; the objects of sec. 3.1).  For every
 * request r, kind in {K, V} and j < n_blocks_r, object bytes [j*block_bytes, (j+1)*block_bytes) <- pool block
 * d_block_table[table_off_r + j], in token-major order ((t*h + i)*d + k)*e whatever the pool layout; the tail
 * from n_blocks_r*block_bytes up to obj_bytes_r <- 0.  The K object of r starts at d_stage + stage_off_r, its V
 * object obj_bytes_r later.
 * Extents: the fields stage_off, obj_bytes, n_blocks and table_off of every record are honoured as they stand,
 * whoever wrote them (n_chunks and sqe_base are not used): tutti_obj_layout's output, a sub-range of it, records
 * with gaps between the requests or in any order in the staging buffer.  What cannot be honoured is skipped and
 * reported in *d_status, never dereferenced; per request, in this order:
 *   running sum of n_blocks over the requests so far > table_len   request and all later ones skipped, BAD_EXTENT
 *   stage_off or obj_bytes not a multiple of 16                    request skipped, BAD_EXTENT
 *   stage_off + 2*obj_bytes > stage_cap (no wrap-around)           request skipped, STAGE_CAP
 *   (j+1)*block_bytes > obj_bytes                                  block skipped, BAD_EXTENT
 *   table_off + j >= table_len, or the id there >= num_blocks      block skipped, BAD_BLOCK
 * Objects of different requests must not overlap (two writers race).
 * table_len = number of entries in d_block_table (entries beyond it are never read).
 * d_stage: 16-byte aligned, stage_cap bytes.  cu_budget: 0 = whole GPU, else the launch is limited
 * to about that many compute units' worth of workgroups (see tutti_layer_restore). */
int tutti_obj_pack(const tutti_pool *pool, const tutti_objcfg *cfg, const tutti_extent *d_extents, uint32_t n_req,
                   const uint32_t *d_block_table, uint32_t table_len, void *d_stage, uint64_t stage_cap,
                   uint32_t cu_budget, uint32_t *d_status, void *stream);

/* ---- a3: unpack (restore; retrieve_layer of sec. 3.4, the objects of sec. 3.1).  The inverse copy: pool block <-
 * object bytes, with the same extents contract and the same skip rules as tutti_obj_pack.  Padding is not read;
 * pool blocks not named in the table are not touched.  A block id must not appear twice in one call (two writers
 * of one block race). */
int tutti_obj_unpack(const tutti_pool *pool, const tutti_objcfg *cfg, const tutti_extent *d_extents, uint32_t n_req,
                     const uint32_t *d_block_table, uint32_t table_len, const void *d_stage, uint64_t stage_cap,
                     uint32_t cu_budget, uint32_t *d_status, void *stream);

/* ---- a4: submission entries (sec. 3.2: commands are generated on the GPU, one I/O context per
 * transfer, 2048 per IOCB).  One entry per chunk of every K and V object of `layer`, in the order
 * request ascending, K then V, chunk ascending; entry index = sqe_base_r + kind*n_chunks_r + chunk.
 * stage_addr is the address the entries should name for byte 0 of the staging buffer (multiple of
 * align); it is only arithmetic, never dereferenced.  Entries with index >= sqe_cap are dropped.
 * Extents: the entry builders (this call, tutti_sqe_build_direct, tutti_iocb_fill_direct) number entries by
 * sqe_base and table_off, so they take extents exactly as tutti_obj_layout writes them for these n_req requests:
 * sqe_base and table_off running from 0 without gaps, obj_bytes and n_chunks as defined under a1 (stage_off is
 * free: it is only added to stage_addr).  This is checked on the device; for any other extents the call writes
 * nothing at all and reports TUTTI_ST_BAD_EXTENT. */
int tutti_sqe_build(const tutti_pool *pool, const tutti_objcfg *cfg, const tutti_extent *d_extents, uint32_t n_req,
                    const uint32_t *d_file_id, uint32_t layer, uint32_t opcode, uint64_t stage_addr, uint32_t sgl_id,
                    tutti_sqe *d_sqe, uint32_t sqe_cap, uint32_t *d_status, void *stream);

/* ---- a5 + a6: one layer's restore in ONE launch (retrieve_layer of sec. 3.4; sec. 1 has the CPU launch I/O
 * kernels once per layer and no more): extents from d_n_blocks, READ entries for `layer`, then the
 * unpack of every hit block, as tutti_obj_layout + tutti_sqe_build(READ) + tutti_obj_unpack would (so requests
 * whose blocks run beyond table_len are skipped and reported as tutti_obj_unpack does).
 * Also writes d_extents[0..n_req) and d_totals[0..2).  d_stage must be device-accessible.
 * cu_budget stands in for the SM count of the paper's issue_io(IOCB_ids, SMs) (sec. 3.2): 0 = whole
 * GPU; B > 0 limits the grid to B compute units' worth of persistent workgroups so a concurrent
 * compute kernel keeps the rest; B > CU count is TUTTI_ERANGE. */
int tutti_layer_restore(const tutti_pool *pool, const tutti_objcfg *cfg, const uint32_t *d_n_blocks, uint32_t n_req,
                        const uint32_t *d_block_table, uint32_t table_len, const uint32_t *d_file_id,
                        uint32_t layer, const void *d_stage, uint64_t stage_cap, uint64_t stage_addr,
                        uint32_t sgl_id, tutti_extent *d_extents, uint64_t *d_totals, tutti_sqe *d_sqe,
                        uint32_t sqe_cap, uint32_t cu_budget, uint32_t *d_status, void *stream);

/* The same restore with the blocks visited in an order the caller names (sec. 3.4 fixes what a layer's restore
 * moves, not the order in which its blocks are written; on a pool whose hit blocks are dense in memory, visiting
 * them by ascending address keeps neighbouring wavefronts on neighbouring DRAM pages).  d_visit: table_len table
 * positions, device memory, as tutti_table_order writes them; the launch visits position d_visit[0], d_visit[1],
 * ... for the K plane, then the same for V.  A position that is not a block of a request that takes part
 * (>= the blocks of the requests within table_len) is passed over; a position listed twice is restored twice (same
 * bytes); a position not listed is not restored.  Everything else (entries, extents, totals, status bits, skip
 * rules) as tutti_layer_restore, whose results a permutation of 0..table_len-1 reproduces bit for bit.  d_visit ==
 * NULL is tutti_layer_restore itself.  A head-major pool that goes through LDS tiles keeps staging order (d_visit
 * is not read). */
int tutti_layer_restore_ordered(const tutti_pool *pool, const tutti_objcfg *cfg, const uint32_t *d_n_blocks,
                                uint32_t n_req, const uint32_t *d_block_table, uint32_t table_len,
                                const uint32_t *d_file_id, uint32_t layer, const void *d_stage, uint64_t stage_cap,
                                uint64_t stage_addr, uint32_t sgl_id, tutti_extent *d_extents, uint64_t *d_totals,
                                tutti_sqe *d_sqe, uint32_t sqe_cap, uint32_t cu_budget, const uint32_t *d_visit,
                                uint32_t *d_status, void *stream);

/* The visiting order of a block table by ascending block id (= ascending address in both planes), computed on the
 * device in time linear in table_len + num_blocks: d_visit[k] <- the table position that holds the k-th smallest
 * id.  A table with an id >= num_blocks or an id twice has no such order that a restore may use: the identity
 * (d_visit[k] = k) is written and TUTTI_ST_BAD_BLOCK / TUTTI_ST_DUP_BLOCK are ORed into *d_status (may be NULL),
 * as tutti_table_validate reports them.  d_work: device memory lent for the call, 16-byte aligned, work_bytes >=
 * tutti_table_order_work_bytes(num_blocks) (about num_blocks / 4 bytes; TUTTI_ERANGE if smaller), contents
 * garbage before and after; cleared by a kernel on `stream`, so the launches can be captured in a graph.  One
 * table serves every layer of a request batch: compute the order once, restore all layers with it. */
uint64_t tutti_table_order_work_bytes(uint32_t num_blocks);
int tutti_table_order(uint32_t num_blocks, const uint32_t *d_block_table, uint32_t table_len, uint32_t *d_visit,
                      void *d_work, uint64_t work_bytes, uint32_t *d_status, void *stream);

/* ---- one layer's save in ONE launch (store_layer of sec. 3.4): extents from d_n_blocks, WRITE entries for
 * `layer`, then the pack of every hit block with zero padding, as tutti_obj_layout + tutti_sqe_build(WRITE) +
 * tutti_obj_pack would.  Arguments as in tutti_layer_restore; d_stage is written. */
int tutti_layer_save(const tutti_pool *pool, const tutti_objcfg *cfg, const uint32_t *d_n_blocks, uint32_t n_req,
                     const uint32_t *d_block_table, uint32_t table_len, const uint32_t *d_file_id, uint32_t layer,
                     void *d_stage, uint64_t stage_cap, uint64_t stage_addr, uint32_t sgl_id, tutti_extent *d_extents,
                     uint64_t *d_totals, tutti_sqe *d_sqe, uint32_t sqe_cap, uint32_t cu_budget, uint32_t *d_status,
                     void *stream);

/* ---- direct-to-block mode: the paper's own data path, with no staging copy (sec. 3.1 "P2P Memory
 * Mapping Table"; the three fields of an I/O context: sec. 3.2 "Zero-Copy Ring Buffers").
 *
 * 16-byte SGL descriptor of one pool block: address 8, length 4, identifier 4 (sec. 3.1). */
typedef struct tutti_sgl {
  uint64_t addr;
  uint32_t len;
  uint32_t id;
} tutti_sgl;

/* The mapping table of one layer's pool, built once at start-up (the pool never moves: sec. 3.1):
 * d_table[b] describes K block b, d_table[num_blocks + b] describes V block b, each
 * { plane address + b*block_stride, block_bytes, sgl_id }.  k_addr / v_addr are the addresses the
 * descriptors should name for the planes (a bus address in a real deployment; arithmetic only here,
 * pool->k_base / v_base are not used).  Descriptors with index >= cap are dropped (TUTTI_ST_SQE_CAP). */
int tutti_sgl_table_build(const tutti_pool *pool, uint64_t k_addr, uint64_t v_addr, uint32_t sgl_id,
                          tutti_sgl *d_table, uint32_t cap, uint32_t *d_status, void *stream);

/* One entry per (hit block, K|V) of `layer`: index = 2*table_off_r + kind*n_r + j, in the order request
 * ascending, K then V, block ascending.  addr = sgl_table_addr + 16*(kind*num_blocks + block id), i.e. the
 * block's descriptor in the mapping table; len = block_bytes; file_off = (2*layer + kind)*obj_bytes_r +
 * j*block_bytes: the GPU-file layout of the staged mode, so either mode can read what the other wrote.
 * block_bytes must be a multiple of cfg->align (else TUTTI_EINVAL); sgl_table_addr a multiple of 16.
 * A block id >= num_blocks (or beyond table_len) gives a no-op entry (addr 0, len 0) and TUTTI_ST_BAD_BLOCK. */
int tutti_sqe_build_direct(const tutti_pool *pool, const tutti_objcfg *cfg, const tutti_extent *d_extents,
                           uint32_t n_req, const uint32_t *d_block_table, uint32_t table_len,
                           const uint32_t *d_file_id, uint32_t layer, uint32_t opcode, uint64_t sgl_table_addr,
                           uint32_t sgl_id, tutti_sqe *d_sqe, uint32_t sqe_cap, uint32_t *d_status, void *stream);

/* ---- submission / completion rings (sec. 3.2 "Zero-Copy Ring Buffers" and "Async I/O Processing").
 * An SQ entry is an IOCB: a 64-byte header followed by 2048 I/O contexts (tutti_sqe records); the CQ
 * collects the indices of completed IOCBs.  Rings live in caller-allocated device-accessible memory (the paper maps
 * them to the CPU so that it can fill them; here the GPU fills them itself, so no mapping is needed).  Device
 * memory is the normal choice; a CQ (or a whole ring) in pinned host memory also works, and the CPU can then poll
 * the CQ tail without synchronising the stream: completions are published with system-scope release stores.
 * The header layout, the CQ layout and the file store that stands in for the SSD are this repository's. */
#define TUTTI_IOCB_FREE 0u
#define TUTTI_IOCB_FILLED 1u
#define TUTTI_IOCB_DONE 2u

typedef struct tutti_iocb_hdr {
  uint32_t iocb_idx;  /* unique index = slot in the SQ (tutti_ring_init) */
  uint32_t num_ioctx; /* valid contexts (tutti_iocb_fill_direct) */
  uint32_t state;     /* TUTTI_IOCB_* */
  uint32_t done;      /* contexts completed: 0 while FILLED, num_ioctx once DONE */
  uint32_t layer;
  uint32_t opcode;
  uint32_t rsvd[10];
} tutti_iocb_hdr;

typedef struct tutti_iocb {
  tutti_iocb_hdr hdr;
  tutti_sqe ioctx[TUTTI_IOCB_SLOTS];
} tutti_iocb; /* 64 + 2048*64 = 131136 bytes */

typedef struct tutti_cq_hdr {
  uint32_t tail;  /* completions so far */
  uint32_t depth;
  uint32_t rsvd[14];
  /* followed by uint32_t entry[depth]: entry[t % depth] = index of the t-th completed IOCB */
} tutti_cq_hdr;

/* Host-side handle of a ring: d_sq = depth IOCBs, d_cq = tutti_cq_hdr + depth entries (64 + 4*depth bytes),
 * both 16-byte aligned device memory owned by the caller. */
typedef struct tutti_ring {
  tutti_iocb *d_sq;
  void *d_cq;
  uint32_t depth;
} tutti_ring;

/* The stand-in for the SSD: n_files GPU files of file_stride bytes in device(-accessible) memory,
 * file f at base + (f - first_file_id)*file_stride; base and file_stride multiples of 16. */
typedef struct tutti_filestore {
  void *base;
  uint64_t file_stride;
  uint32_t first_file_id;
  uint32_t n_files;
} tutti_filestore;

/* init_queue(depth): every IOCB FREE with its unique index, CQ empty (entries 0xffffffff). */
int tutti_ring_init(const tutti_ring *ring, void *stream);

/* get_iocb + fill, done by the GPU for one layer in direct-to-block mode: context i of
 * tutti_sqe_build_direct goes to IOCB slot (first_slot + i/2048) % depth, position i % 2048.  All n_slots
 * IOCBs become FILLED with num_ioctx (0 if unused), layer, opcode and done = 0.  The host picks first_slot
 * and n_slots (ceil(2*table_len/2048) always suffices); contexts beyond n_slots*2048 are dropped and
 * reported (TUTTI_ST_SQE_CAP).  Other arguments as in tutti_sqe_build_direct. */
int tutti_iocb_fill_direct(const tutti_ring *ring, uint32_t first_slot, uint32_t n_slots, const tutti_pool *pool,
                           const tutti_objcfg *cfg, const tutti_extent *d_extents, uint32_t n_req,
                           const uint32_t *d_block_table, uint32_t table_len, const uint32_t *d_file_id,
                           uint32_t layer, uint32_t opcode, uint64_t sgl_table_addr, uint32_t sgl_id,
                           uint32_t *d_status, void *stream);

/* issue_io(IOCB_ids, SMs): the I/O kernel.  Executes every context of the n_slots FILLED IOCBs starting
 * at first_slot: resolves the SGL descriptor the context names (index (addr - sgl_table_addr)/16 into
 * d_sgl_table of n_desc descriptors, whose addr fields must be device addresses here), then moves len
 * bytes between that block and the request's GPU file at file_off (READ: file -> block, WRITE: block ->
 * file), one wavefront per 4 or 8 KiB slice.  A one-wavefront completion kernel enqueued right behind the
 * I/O kernel then marks every executed IOCB DONE (done = num_ioctx) and appends its index to the CQ, in slot
 * order: the kernel boundary is the "all contexts finished" event (counting finished contexts with atomics on
 * the IOCB header was measured 28x slower).  max_len bounds the length of any context (the pool's block size).
 * The IOCBs may have been filled by the GPU (tutti_iocb_fill_direct) or by the application itself, as in the
 * paper's flow (sec. 3.2 "Async I/O Processing", step 2): an SQ in pinned host memory, contexts, num_ioctx,
 * layer, opcode and state = TUTTI_IOCB_FILLED written by the CPU; so a context may hold anything.  One that
 * cannot be executed is skipped (TUTTI_ST_BAD_BLOCK) and its IOCB still completes: opcode neither READ nor
 * WRITE; address not that of a descriptor of the table; length not a multiple of 16, or beyond max_len or the
 * descriptor's length; block address or file offset not a multiple of 16; file id outside the store;
 * [file_off, file_off + len) not inside the file.  Length 0 is a no-op.  cu_budget as in tutti_layer_restore.
 * Two tutti_issue_io calls on the same ring must be ordered by the stream (they share the CQ tail). */
int tutti_issue_io(const tutti_ring *ring, uint32_t first_slot, uint32_t n_slots, const tutti_sgl *d_sgl_table,
                   uint32_t n_desc, uint64_t sgl_table_addr, const tutti_filestore *store, uint32_t max_len,
                   uint32_t cu_budget, uint32_t *d_status, void *stream);

/* retrieve_layer(layer) / store_layer(layer) (sec. 3.4 "Integration with vLLM") through the rings, in
 * direct-to-block mode, as ONE data-moving launch plus the completion kernel: the result (extents, totals,
 * IOCBs, CQ, pool blocks or file store, status word) is that of tutti_obj_layout, tutti_iocb_fill_direct with
 * READ (retrieve) or WRITE (store) and tutti_issue_io run one after the other, with a mapping table that
 * tutti_sgl_table_build made for this pool at its own plane addresses and max_len = the block size.  The
 * kernel takes block addresses from `pool` itself, so no table is passed; sgl_table_addr and sgl_id only go
 * into the recorded contexts.  Blocks travel as raw bytes whatever pool->pool_layout says (as in
 * tutti_issue_io).  Arguments as in those three calls; d_extents (n_req records) and d_totals (2 values) are
 * outputs.  Same errors as tutti_iocb_fill_direct and tutti_issue_io. */
int tutti_retrieve_layer(const tutti_ring *ring, uint32_t first_slot, uint32_t n_slots, const tutti_pool *pool,
                         const tutti_objcfg *cfg, const uint32_t *d_n_blocks, uint32_t n_req,
                         const uint32_t *d_block_table, uint32_t table_len, const uint32_t *d_file_id, uint32_t layer,
                         uint64_t sgl_table_addr, uint32_t sgl_id, const tutti_filestore *store,
                         tutti_extent *d_extents, uint64_t *d_totals, uint32_t cu_budget, uint32_t *d_status,
                         void *stream);
int tutti_store_layer(const tutti_ring *ring, uint32_t first_slot, uint32_t n_slots, const tutti_pool *pool,
                      const tutti_objcfg *cfg, const uint32_t *d_n_blocks, uint32_t n_req,
                      const uint32_t *d_block_table, uint32_t table_len, const uint32_t *d_file_id, uint32_t layer,
                      uint64_t sgl_table_addr, uint32_t sgl_id, const tutti_filestore *store, tutti_extent *d_extents,
                      uint64_t *d_totals, uint32_t cu_budget, uint32_t *d_status, void *stream);

/* The two halves of tutti_retrieve_layer / tutti_store_layer, for callers that pipeline layers: the _issue calls
 * enqueue the data-moving launch only and leave the IOCBs FILLED; tutti_complete_io enqueues the completion kernel
 * alone: every FILLED IOCB of the n_slots slots from first_slot becomes DONE (done = num_ioctx) and its index is
 * appended to the CQ, in slot order (sec. 3.2 "Async I/O Processing", step 4).  tutti_complete_io must be ordered
 * after the launch that executed those IOCBs (same stream, or an event), and completions of one ring after each
 * other (they share the CQ tail); it does not check that the IOCBs were executed.  On one stream, _issue followed by
 * tutti_complete_io IS the one-call form.  With the completions on a second stream, each behind an event recorded
 * after its layer's _issue call, the next layer's data kernel does not wait for the completion kernel of the
 * layer before it (different IOCB slots, different blocks, different file ranges: nothing is shared but the CQ
 * tail, which only the completions touch), which takes the completion's launch boundary off the layer train. */
int tutti_retrieve_layer_issue(const tutti_ring *ring, uint32_t first_slot, uint32_t n_slots, const tutti_pool *pool,
                               const tutti_objcfg *cfg, const uint32_t *d_n_blocks, uint32_t n_req,
                               const uint32_t *d_block_table, uint32_t table_len, const uint32_t *d_file_id,
                               uint32_t layer, uint64_t sgl_table_addr, uint32_t sgl_id, const tutti_filestore *store,
                               tutti_extent *d_extents, uint64_t *d_totals, uint32_t cu_budget, uint32_t *d_status,
                               void *stream);
int tutti_store_layer_issue(const tutti_ring *ring, uint32_t first_slot, uint32_t n_slots, const tutti_pool *pool,
                            const tutti_objcfg *cfg, const uint32_t *d_n_blocks, uint32_t n_req,
                            const uint32_t *d_block_table, uint32_t table_len, const uint32_t *d_file_id,
                            uint32_t layer, uint64_t sgl_table_addr, uint32_t sgl_id, const tutti_filestore *store,
                            tutti_extent *d_extents, uint64_t *d_totals, uint32_t cu_budget, uint32_t *d_status,
                            void *stream);
int tutti_complete_io(const tutti_ring *ring, uint32_t first_slot, uint32_t n_slots, void *stream);

/* A train of layers on ONE stream without a completion kernel between them (sec. 3.4 "Integration with vLLM": the
 * layers of a request are retrieved one after the other): as the _issue calls, and the same launch also completes
 * the IOCBs [done_first_slot, done_first_slot + done_n_slots) that an EARLIER call on the same stream executed
 * (typically the layer before), exactly as tutti_complete_io would: one more workgroup, in front of the grid, does it
 * and leaves.  Stream order has made the earlier launch's stores visible before this launch starts, so the
 * completion is published as early as a completion kernel's would be, and the train pays for no kernel boundary
 * between a layer's data and the next layer's.  The last layer of a train is completed with tutti_complete_io.
 * done_n_slots = 0: nothing to complete (the first layer of a train).  The two slot ranges must not overlap
 * (TUTTI_EINVAL); a later completion of the same ring must still be ordered after this launch (they share the CQ
 * tail).  Under a cu_budget the launch has cu_budget + 1 workgroups for as long as the completing one lives (a few
 * microseconds). */
int tutti_retrieve_layer_chained(const tutti_ring *ring, uint32_t first_slot, uint32_t n_slots, uint32_t done_first_slot,
                                 uint32_t done_n_slots, const tutti_pool *pool, const tutti_objcfg *cfg,
                                 const uint32_t *d_n_blocks, uint32_t n_req, const uint32_t *d_block_table,
                                 uint32_t table_len, const uint32_t *d_file_id, uint32_t layer, uint64_t sgl_table_addr,
                                 uint32_t sgl_id, const tutti_filestore *store, tutti_extent *d_extents,
                                 uint64_t *d_totals, uint32_t cu_budget, uint32_t *d_status, void *stream);
int tutti_store_layer_chained(const tutti_ring *ring, uint32_t first_slot, uint32_t n_slots, uint32_t done_first_slot,
                              uint32_t done_n_slots, const tutti_pool *pool, const tutti_objcfg *cfg,
                              const uint32_t *d_n_blocks, uint32_t n_req, const uint32_t *d_block_table,
                              uint32_t table_len, const uint32_t *d_file_id, uint32_t layer, uint64_t sgl_table_addr,
                              uint32_t sgl_id, const tutti_filestore *store, tutti_extent *d_extents,
                              uint64_t *d_totals, uint32_t cu_budget, uint32_t *d_status, void *stream);

/* tutti_issue_io for a train of issues on ONE stream in the same way: the entry-driven I/O kernel alone, and the same
 * launch completes the IOCBs [done_first_slot, done_first_slot + done_n_slots) that an earlier call on the stream
 * executed; the last issue of a train is completed with tutti_complete_io.  n_slots = 0 with done_n_slots > 0 only
 * completes.  Other arguments, errors and status bits as tutti_issue_io; the slot ranges must not overlap. */
int tutti_issue_io_chained(const tutti_ring *ring, uint32_t first_slot, uint32_t n_slots, uint32_t done_first_slot,
                           uint32_t done_n_slots, const tutti_sgl *d_sgl_table, uint32_t n_desc,
                           uint64_t sgl_table_addr, const tutti_filestore *store, uint32_t max_len, uint32_t cu_budget,
                           uint32_t *d_status, void *stream);

/* wait_cqe(): a check, not a blocking wait.  *d_flag <- 1 if IOCB slot `slot` is DONE, else 0; enqueue
 * it on any stream and read the flag after synchronising that stream. */
int tutti_wait_cqe(const tutti_ring *ring, uint32_t slot, uint32_t *d_flag, void *stream);
/* The same check for the n_slots IOCBs from first_slot on (wrapping at depth) in one launch: d_flags[i] <- 1 if IOCB
 * (first_slot + i) % depth is DONE, else 0.  d_flags: n_slots words of device memory. */
int tutti_wait_cqe_range(const tutti_ring *ring, uint32_t first_slot, uint32_t n_slots, uint32_t *d_flags,
                         void *stream);

/* ---- I/O domain (sec. 3.2 "SM Partitioning For Accurate I/O": the I/O kernels get compute units of their own,
 * isolated in hardware from the compute kernels).  *stream <- a new stream whose kernels the hardware dispatches
 * only to the first n_cus compute units of the device (a compute-unit mask on the stream's queue); pass it as
 * `stream` to any call above with cu_budget = 0, and the call occupies those units and no others, whatever its
 * grid.  Unlike cu_budget, which only bounds how many workgroups exist, the mask binds placement.  Other streams
 * are not kept off those units.  TUTTI_ERANGE if n_cus is 0 or above the CU count, TUTTI_EHIP if the runtime
 * refuses the mask (tutti_last_hip_error() tells why).  The stream has default priority and belongs to the caller
 * until tutti_io_domain_destroy. */
int tutti_io_domain_create(uint32_t n_cus, void **stream);
int tutti_io_domain_destroy(void *stream);

/* ---- the application's side of the rings: get_iocb and the reaping of completions (sec. 3.2 "Async I/O
 * Processing", steps 2 and 4).  Host code only: no HIP call, no device access, O(1) per IOCB.  The state lives in
 * host memory the caller owns (one per ring, used from one thread at a time).  IOCBs are handed out in ring order,
 * so a run of n is always the n consecutive slots (modulo depth) that the fill / issue calls take as
 * (first_slot, n_slots); a slot is handed out again only after its completion has been reaped AND every older
 * slot has been given back (completions may arrive in any order, e.g. deferred writes behind later reads). */
typedef struct tutti_sq_state {
  uint32_t depth;
  uint32_t head;    /* the next slot to hand out */
  uint32_t held;    /* slots handed out and not yet given back: the `held` slots in front of head */
  uint32_t cq_seen; /* completions consumed from the CQ so far (modulo 2^32, as the CQ tail) */
  uint8_t *done;    /* depth flags (caller's memory): completed, waiting for an older slot to be given back */
} tutti_sq_state;

/* flags: depth bytes of host memory that stay valid as long as the state is used. */
int tutti_sq_state_init(tutti_sq_state *s, uint32_t depth, uint8_t *flags);
/* get_iocb(n): *first_slot <- the first of n consecutive free slots.  TUTTI_EAGAIN if fewer than n are free
 * (nothing changes), TUTTI_EINVAL for n = 0 or n > depth. */
int tutti_get_iocb(tutti_sq_state *s, uint32_t n, uint32_t *first_slot);
uint32_t tutti_sq_free_count(const tutti_sq_state *s);
/* Consumes the completions the CQ has gained since the last call.  cq_host: a host-readable view of the ring's
 * CQ (the CQ itself when it lives in pinned host memory: no synchronisation is needed, the tail is read with
 * acquire order; otherwise a host copy taken after synchronising).  sq_host: the SQ when it lives in
 * host-accessible memory, else NULL; each reaped IOCB's state becomes TUTTI_IOCB_FREE there.  *n_new (may be
 * NULL) <- completions consumed.  TUTTI_EINVAL, with nothing consumed, if the queue names a slot that is not
 * held, names one twice, or holds more completions than slots are held. */
int tutti_reap_cqe(tutti_sq_state *s, const void *cq_host, tutti_iocb *sq_host, uint32_t *n_new);
/* 1 if the IOCB last handed out in `slot` has completed (as far as the reaping has seen), else 0. */
int tutti_iocb_completed(const tutti_sq_state *s, uint32_t slot);
/* wait_cqe() from the host: reaps until `slot` has completed or max_polls further polls have not shown it.
 * Returns 1 (completed), 0 (not yet) or a negative TUTTI_E*.  A bounded wait: it never spins for ever. */
int tutti_wait_cqe_host(tutti_sq_state *s, const void *cq_host, tutti_iocb *sq_host, uint32_t slot,
                        uint32_t max_polls);

/* ---- slack table (sec. 3.3 "Offline Profiling of SM Slack Windows": besides the slack windows of the model,
 * the execution time of the read / write kernels under different IOCB counts and compute-unit budgets is
 * profiled offline, and the runtime picks a launch size by table lookup).  A row is one profiled launch; the
 * table is whatever the profiling run measured (bench.py writes one), in any order.  Pure lookups, no
 * interpolation: a launch is taken to cost what the next larger profiled launch at the same budget cost. */
typedef struct tutti_io_profile {
  uint32_t cu_budget; /* compute units given to the I/O kernel; 0 = whole GPU */
  uint32_t n_iocbs;   /* IOCBs (2048 contexts each) in the launch */
  float read_us;      /* measured duration of a retrieve of that size; <= 0 = not measured */
  float write_us;     /* the same for a store */
} tutti_io_profile;

/* How many IOCBs may be launched into a slack window of slack_us microseconds that leaves cu_budget compute
 * units free: the largest profiled count at that budget whose duration fits; *n_iocbs <- 0 if none does. */
int tutti_iocbs_for_slack(const tutti_io_profile *rows, uint32_t n_rows, uint32_t cu_budget, uint32_t opcode,
                          double slack_us, uint32_t *n_iocbs);
/* The smallest budget in [1, max_budget] at which n_iocbs IOCBs fit a window of slack_us microseconds.
 * TUTTI_EAGAIN (*cu_budget <- 0) if none does: the caller then defers a write, or launches a read on the whole
 * GPU at once because retrieval has become the bottleneck (sec. 3.3 "Decoupled Scheduling for Read and Write"). */
int tutti_budget_for_slack(const tutti_io_profile *rows, uint32_t n_rows, uint32_t n_iocbs, uint32_t opcode,
                           double slack_us, uint32_t max_budget, uint32_t *cu_budget);

/* ---- debugging aid: the preconditions that an unpack (tutti_obj_unpack, tutti_layer_restore, a READ through the
 * rings) places on its flattened block table, checked on the device: every id < num_blocks (else
 * TUTTI_ST_BAD_BLOCK; the data calls skip such blocks anyway) and no id twice (else TUTTI_ST_DUP_BLOCK: two
 * writers to one block, which the data calls neither detect nor order; out-of-range ids do not count as duplicates
 * of each other).  The bits are ORed into *d_status.  Needs no workspace and costs O(table_len^2) comparisons:
 * microseconds for the tables of one layer, tens of milliseconds for a million entries.  Not meant for the
 * per-layer path. */
int tutti_table_validate(uint32_t num_blocks, const uint32_t *d_block_table, uint32_t table_len, uint32_t *d_status,
                         void *stream);

/* The same check in time linear in table_len, for the tables of whole batches: one bit per pool block in device
 * memory that the caller lends for the call: d_work, 16-byte aligned, work_bytes >=
 * tutti_table_validate_work_bytes(num_blocks) (= num_blocks / 8, rounded up to 256; TUTTI_ERANGE if smaller).  Its
 * contents need not be initialised and are garbage afterwards; the call clears what it uses with a kernel on
 * `stream`, so the pair of launches can be captured in a graph.  Same status bits as tutti_table_validate. */
uint64_t tutti_table_validate_work_bytes(uint32_t num_blocks);
int tutti_table_validate_ws(uint32_t num_blocks, const uint32_t *d_block_table, uint32_t table_len, uint32_t *d_status,
                            void *d_work, uint64_t work_bytes, void *stream);

/* For callers that cannot allocate device memory or lend any: code under HIP-graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  tutti_table_validate_ws with the bitmap in an array the library itself keeps
 * on every GPU it runs on (TUTTI_STATIC_VALIDATE_MAX_BLOCKS bits = 512 KiB, held until the process ends); the call
 * allocates nothing.  num_blocks above TUTTI_STATIC_VALIDATE_MAX_BLOCKS is TUTTI_ERANGE (nothing is enqueued).
 * Every call on a GPU uses that GPU's one array and clears the bits it needs first: calls that overlap on one GPU
 * (two streams, two threads) race and must be ordered by the caller.  Same status bits as tutti_table_validate. */
#define TUTTI_STATIC_VALIDATE_MAX_BLOCKS (1u << 22)
int tutti_table_validate_static(uint32_t num_blocks, const uint32_t *d_block_table, uint32_t table_len,
                                uint32_t *d_status, void *stream);

/* ---- set-up: where a pool's planes sit in HBM.  The pool is allocated and registered once and stays fixed for
 * the engine's life (sec. 3.1 "Scalable GPU File Pool", "P2P Memory Mapping Table"), so its place in memory is
 * chosen once, before any layer is restored (sec. 3.4 "Integration with vLLM").  Measured on the MI355X: its 288 GB
 * of HBM behave as three regions of 96 GB; a restore runs at the speed of a contiguous copy when a layer's K plane
 * and V plane lie in different regions and about 15 % slower when they share one.  Nothing in an address tells the
 * region, so the calls below tell it by timing: the library's own restore (tutti_layer_restore, 2048 blocks of
 * 32 KiB picked by a fixed pseudo-random table) on the pool (plane a, plane b) is slow exactly when a and b share a
 * region.  Unlike the data calls these BLOCK: they synchronise `stream`, time with events and return host values;
 * they allocate no device memory (the caller lends d_work) and OVERWRITE blocks of the planes they are given with the
 * bytes of d_work, so they run before the pool is filled.
 *
 * planes: a HOST array of n device pointers, each the start of a buffer of plane_bytes bytes (16-byte aligned,
 * plane_bytes >= TUTTI_PLACE_MIN_PLANE_BYTES, else TUTTI_ERANGE).  d_work: device memory, 256-byte aligned,
 * work_bytes >= tutti_place_work_bytes() (else TUTTI_ERANGE); contents need not be initialised. */
#define TUTTI_PLACE_MIN_PLANE_BYTES (128ull << 20)
#define TUTTI_PLACE_MAX_REGIONS 8u
uint64_t tutti_place_work_bytes(void);
/* us[i] (HOST array of n floats) <- microseconds of the probe restore on the pool (ref, cands[i]): the median of
 * `reps` (1..16) timed passes after one warm-up pass; each figure includes the gap between two launches, the same
 * for all.  TUTTI_EINVAL if the device reported a status (it cannot with valid planes). */
int tutti_place_pair_times(const void *ref, const void *const *cands, uint32_t n, uint64_t plane_bytes, void *d_work,
                           uint64_t work_bytes, uint32_t reps, float *us, void *stream);
/* One round of the classification, for the caller's records. */
typedef struct tutti_place_round {
  uint32_t reference;   /* index of the round's reference plane */
  uint32_t members;     /* planes put into the reference's class */
  float same_region_us; /* the pool (reference, reference): one region by construction, the slow case */
  float fastest_us;     /* the fastest pool (reference, x) of the round */
} tutti_place_round;
/* classes[i] (HOST array of n) <- region class 0, 1, ... of planes[i], or -1 if max_regions rounds did not reach
 * it.  Round c takes the first unclassified plane r as reference and times (r, r) and (r, x) for every
 * unclassified x; x joins class c if its time is nearer the slow case (r, r) than the round's fastest pair.  A
 * round in which nothing beats the slow case by min_gap_us puts everything left into class c (a part with one
 * region ends there, with every plane in class 0).  A plane that straddles two regions times in between against
 * everything: as a reference it finds no partner and is set aside (class -1, and the round is not counted, at most
 * four times); as a candidate it joins the nearer side.  Planes much larger than the 2 GiB of the measurements are
 * better cut into several candidates.  max_regions in 1..TUTTI_PLACE_MAX_REGIONS.  rounds (HOST,
 * max_regions records, may be NULL) and *n_rounds (may be NULL) <- what each round measured. */
int tutti_place_classify(const void *const *planes, uint32_t n, uint64_t plane_bytes, void *d_work,
                         uint64_t work_bytes, uint32_t max_regions, double min_gap_us, int32_t *classes,
                         tutti_place_round *rounds, uint32_t *n_rounds, void *stream);
/* Host code only.  pairs[2p], pairs[2p+1] (p < n_pairs) <- indices (K plane, V plane) with different classes >= 0,
 * every plane used at most once; taken greedily from the two classes with the most planes left, lowest indices
 * first, which forms as many such pairs as any pairing can.  *n_mixed (may be NULL) <- how many pairs were formed
 * that way.  If fewer than n_pairs: TUTTI_EAGAIN when strict != 0 (pairs untouched beyond *n_mixed); otherwise
 * the rest is filled with pairs of the planes left over (same class or class -1), lowest indices first, and
 * TUTTI_ERANGE if even that does not give n_pairs. */
int tutti_place_pairs(const int32_t *classes, uint32_t n, uint32_t n_pairs, uint32_t strict, uint32_t *pairs,
                      uint32_t *n_mixed);

/* ---- housekeeping */
const char *tutti_strerror(int code);
int tutti_last_hip_error(void);     /* hipError_t of the last failed HIP call on this thread, 0 if none */
int tutti_cu_count(void);           /* compute units of the current device, or a negative TUTTI_E* */
/* How many 256-thread workgroups of a data-moving kernel one compute unit holds at once, as the runtime's
 * occupancy calculator sees it (default instantiation, single-request launch).  The whole-GPU grids are sized for
 * 8; fewer would leave part of a persistent grid waiting behind the rest.  which: 0 / 1 fused restore / save,
 * 2 / 3 unpack / pack alone, 4 / 5 retrieve / store through the rings, 6 / 7 fused restore / save of a head-major
 * pool, 8 / 9 the same through LDS (with a full tile), 10 the entry-driven I/O kernel.  Returns the count or a
 * negative TUTTI_E*. */
int tutti_resident_wgs_per_cu(uint32_t which);
uint32_t tutti_version(void);       /* 0x00MMmmpp */
/* sizeof / offsetof table of the records above (52 values: extent size + 6 offsets, sqe size + 11,
 * pool size + 9, objcfg size + 3, sgl size + 3, iocb_hdr size + 6, iocb size + offset of its contexts,
 * cq_hdr size, filestore size + 4); returns the count or TUTTI_EINVAL if cap is too small. */
int tutti_abi_describe(uint32_t *out, uint32_t cap);

#ifdef __cplusplus
}
#endif
#endif /* TUTTI_H */
