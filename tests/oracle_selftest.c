/* Sanitizer-built self test of the CPU oracle (test infrastructure for test infrastructure).
 *
 * Every buffer the oracle reads or writes is a heap allocation of exactly the size its contract states, so
 * AddressSanitizer turns any out-of-bounds access of the oracle into a failure, and UBSan does the same for
 * misaligned or overflowing arithmetic.  Inputs are seeded random shapes including the awkward ones: empty
 * requests, strided pools, head-major pools, block ids out of range, capacities that cut the output short.
 * Besides "no sanitizer report", the driver checks properties that hold whatever the shape: unpack(pack(x))
 * restores the named blocks and touches nothing else, the direct mode writes the file bytes the staged mode
 * packs, and the one-call ring functions equal their three-step sequence.
 *
 * Built and run by tests/test_oracle_sanitized.py; prints "ok <cases>" and exits 0 on success. */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "tutti_oracle.h"

static uint64_t rng_state = 0x243f6a8885a308d3ull;
static uint32_t rnd(void) {
  rng_state = rng_state * 6364136223846793005ull + 1442695040888963407ull;
  return (uint32_t)(rng_state >> 33);
}
static uint32_t rnd_in(uint32_t lo, uint32_t hi) { return lo + rnd() % (hi - lo + 1); }

#define CHECK(cond)                                                             \
  do {                                                                          \
    if (!(cond)) {                                                              \
      fprintf(stderr, "case %d: check failed at line %d: %s\n", case_no, __LINE__, #cond); \
      exit(2);                                                                  \
    }                                                                           \
  } while (0)

static void *xmalloc(size_t n) {
  void *p = malloc(n ? n : 1);
  if (!p) exit(3);
  return p;
}

static void fill_random(uint8_t *p, size_t n) {
  for (size_t i = 0; i < n; ++i) p[i] = (uint8_t)rnd();
}

static int case_no = 0;

static void one_case(void) {
  /* geometry: rows of whole 16-byte units so that both layouts are legal */
  const uint32_t T = rnd_in(1, 5), h = rnd_in(1, 3), e = (rnd() & 1) ? 2 : 1, d = 16 * rnd_in(1, 3) / e * 1;
  const uint32_t bb = T * h * d * e;
  const uint32_t N = rnd_in(4, 24);
  const uint64_t stride = bb + 16 * rnd_in(0, 2);
  const uint32_t layout = rnd() & 1;
  const uint32_t A = 16u << rnd_in(0, 4);
  const uint32_t C = A * rnd_in(1, 4);
  const uint32_t L = rnd_in(1, 3);
  const uint32_t layer = rnd() % L;
  const uint32_t n_req = rnd_in(0, 5);

  uint8_t *k = xmalloc(N * stride), *v = xmalloc(N * stride);
  fill_random(k, N * stride);
  fill_random(v, N * stride);
  orc_pool pool = {k, v, stride, N, T, h, d, e, layout};
  orc_objcfg cfg = {A, C, L};

  uint32_t *nb = xmalloc(sizeof(uint32_t) * n_req);
  uint32_t *fid = xmalloc(sizeof(uint32_t) * n_req);
  uint32_t total = 0;
  for (uint32_t r = 0; r < n_req; ++r) {
    nb[r] = rnd_in(0, 4);
    if (total + nb[r] > N) nb[r] = 0;
    total += nb[r];
    fid[r] = 500 + r;
  }
  /* a table of distinct ids: a random permutation prefix */
  uint32_t *perm = xmalloc(sizeof(uint32_t) * N);
  for (uint32_t i = 0; i < N; ++i) perm[i] = i;
  for (uint32_t i = N - 1; i > 0; --i) {
    uint32_t j = rnd() % (i + 1), t = perm[i];
    perm[i] = perm[j];
    perm[j] = t;
  }
  uint32_t *table = xmalloc(sizeof(uint32_t) * total);
  memcpy(table, perm, sizeof(uint32_t) * total);
  const int plant_bad = total > 0 && (rnd() % 4 == 0);
  const uint32_t bad_at = plant_bad ? rnd() % total : 0;
  if (plant_bad) table[bad_at] = N + rnd() % 3;

  orc_extent *ext = xmalloc(sizeof(orc_extent) * n_req);
  uint64_t tot[2] = {0, 0};
  CHECK(orc_obj_layout(&pool, &cfg, nb, n_req, ext, tot) == ORC_OK);
  uint64_t want_stage = 0, want_sqe = 0;
  for (uint32_t r = 0; r < n_req; ++r) {
    const uint64_t obj = ((uint64_t)nb[r] * bb + A - 1) / A * A;
    CHECK(ext[r].stage_off == want_stage && ext[r].obj_bytes == obj && ext[r].sqe_base == want_sqe);
    want_stage += 2 * obj;
    want_sqe += 2 * ((obj + C - 1) / C);
  }
  CHECK(tot[0] == want_stage && tot[1] == want_sqe);

  /* pack into an exact-size staging buffer, unpack into a zeroed pool */
  uint8_t *stage = xmalloc(tot[0]);
  memset(stage, 0xA5, tot[0]);
  uint32_t st = 0;
  CHECK(orc_obj_pack(&pool, &cfg, ext, n_req, table, total, stage, tot[0], &st) == ORC_OK);
  CHECK((st != 0) == (plant_bad != 0));
  uint8_t *k2 = xmalloc(N * stride), *v2 = xmalloc(N * stride);
  memset(k2, 0, N * stride);
  memset(v2, 0, N * stride);
  orc_pool pool2 = pool;
  pool2.k_base = k2;
  pool2.v_base = v2;
  st = 0;
  CHECK(orc_obj_unpack(&pool2, &cfg, ext, n_req, table, total, stage, tot[0], &st) == ORC_OK);
  uint8_t *named = xmalloc(N);
  memset(named, 0, N);
  for (uint32_t i = 0; i < total; ++i)
    if (table[i] < N) named[table[i]] = 1;
  for (uint32_t b = 0; b < N; ++b) {
    if (named[b]) {
      CHECK(memcmp(k2 + b * stride, k + b * stride, bb) == 0 && memcmp(v2 + b * stride, v + b * stride, bb) == 0);
    } else {
      for (uint32_t i = 0; i < bb; ++i) CHECK(k2[b * stride + i] == 0 && v2[b * stride + i] == 0);
    }
    for (uint64_t i = bb; i < stride; ++i) CHECK(k2[b * stride + i] == 0);
  }
  /* a staging capacity one byte short of the last non-empty request skips exactly that request */
  if (tot[0] > 0) {
    uint8_t *shorter = xmalloc(tot[0] - 1);
    memset(shorter, 0x5A, tot[0] - 1);
    st = 0;
    CHECK(orc_obj_pack(&pool, &cfg, ext, n_req, table, total, shorter, tot[0] - 1, &st) == ORC_OK);
    CHECK(st & ORC_ST_STAGE_CAP);
    free(shorter);
  }

  /* extents written by hand: a gap in front of every request, the requests in reverse order in the staging
   * buffer, and requests 1.. passed alone with the whole table; each packs into an exact-size buffer and
   * restores the named blocks of the requests it covers, nothing else */
  for (int variant = 0; variant < 3 && n_req > 0; ++variant) {
    const uint64_t gap = 16 * rnd_in(1, 8);
    orc_extent *hx = xmalloc(sizeof(orc_extent) * n_req);
    memcpy(hx, ext, sizeof(orc_extent) * n_req);
    uint64_t end = 0;
    if (variant == 0 || variant == 2) {
      for (uint32_t r = 0; r < n_req; ++r) {
        hx[r].stage_off = end + gap;
        end = hx[r].stage_off + 2 * hx[r].obj_bytes;
      }
    } else {
      for (uint32_t r = n_req; r-- > 0;) {
        hx[r].stage_off = end;
        end += 2 * hx[r].obj_bytes;
      }
    }
    const uint32_t first = variant == 2 ? 1 : 0;
    uint8_t *hs = xmalloc(end);
    memset(hs, 0x3C, end);
    st = 0;
    CHECK(orc_obj_pack(&pool, &cfg, hx + first, n_req - first, table, total, hs, end, &st) == ORC_OK);
    CHECK((st & ~ORC_ST_BAD_BLOCK) == 0);
    if (variant != 1)
      for (uint32_t r = 0; r < n_req; ++r) /* the gaps stay as they were */
        for (uint64_t i = hx[r].stage_off - gap; i < hx[r].stage_off; ++i) CHECK(hs[i] == 0x3C);
    uint8_t *k4 = xmalloc(N * stride), *v4 = xmalloc(N * stride);
    memset(k4, 0, N * stride);
    memset(v4, 0, N * stride);
    orc_pool pool4 = pool;
    pool4.k_base = k4;
    pool4.v_base = v4;
    st = 0;
    CHECK(orc_obj_unpack(&pool4, &cfg, hx + first, n_req - first, table, total, hs, end, &st) == ORC_OK);
    uint8_t *covered_blk = xmalloc(N);
    memset(covered_blk, 0, N);
    for (uint32_t r = first; r < n_req; ++r)
      for (uint32_t j = 0; j < hx[r].n_blocks; ++j)
        if (table[hx[r].table_off + j] < N) covered_blk[table[hx[r].table_off + j]] = 1;
    for (uint32_t b = 0; b < N; ++b) {
      if (covered_blk[b]) {
        CHECK(memcmp(k4 + b * stride, k + b * stride, bb) == 0 && memcmp(v4 + b * stride, v + b * stride, bb) == 0);
      } else {
        for (uint32_t i = 0; i < bb; ++i) CHECK(k4[b * stride + i] == 0 && v4[b * stride + i] == 0);
      }
    }
    free(k4);
    free(v4);
    /* a table one entry short: the request that crosses the limit and all later ones are skipped, in bounds */
    if (total > 0 && variant == 0) {
      uint32_t *shorter_tab = xmalloc(sizeof(uint32_t) * (total - 1));
      memcpy(shorter_tab, table, sizeof(uint32_t) * (total - 1));
      st = 0;
      CHECK(orc_obj_pack(&pool, &cfg, hx, n_req, shorter_tab, total - 1, hs, end, &st) == ORC_OK);
      CHECK(st & ORC_ST_BAD_EXTENT);
      free(shorter_tab);
    }
    /* an object one alignment unit too small for its blocks: the last block is skipped, in bounds */
    if (variant == 0 && nb[0] > 0 && ext[0].obj_bytes >= A && ext[0].obj_bytes - A < (uint64_t)nb[0] * bb) {
      orc_extent small = ext[0];
      small.obj_bytes -= A;
      uint8_t *ss = xmalloc(2 * small.obj_bytes);
      st = 0;
      CHECK(orc_obj_pack(&pool, &cfg, &small, 1, table, total, ss, 2 * small.obj_bytes, &st) == ORC_OK);
      CHECK(st & ORC_ST_BAD_EXTENT);
      free(ss);
    }
    free(covered_blk);
    free(hs);
    free(hx);
  }

  /* entries: exact-size array, and an array one entry short */
  orc_sqe *sqe = xmalloc(sizeof(orc_sqe) * tot[1]);
  st = 0;
  CHECK(orc_sqe_build(&pool, &cfg, ext, n_req, fid, layer, ORC_OP_READ, 4096 * 7, 9, sqe, (uint32_t)tot[1], &st) == ORC_OK);
  CHECK(st == 0);
  uint64_t covered = 0;
  for (uint64_t i = 0; i < tot[1]; ++i) {
    CHECK(sqe[i].len > 0 && sqe[i].len <= C && sqe[i].opcode == ORC_OP_READ && sqe[i].layer == layer);
    CHECK((uint32_t)sqe[i].user_data == i && sqe[i].iocb_idx == i / ORC_IOCB_SLOTS);
    covered += sqe[i].len;
  }
  CHECK(covered == tot[0]);
  if (tot[1] > 0) {
    orc_sqe *fewer = xmalloc(sizeof(orc_sqe) * (tot[1] - 1));
    st = 0;
    CHECK(orc_sqe_build(&pool, &cfg, ext, n_req, fid, layer, ORC_OP_WRITE, 0, 9, fewer, (uint32_t)tot[1] - 1, &st) == ORC_OK);
    CHECK(st == ORC_ST_SQE_CAP);
    free(fewer);
  }

  /* the fused calls equal their steps */
  {
    orc_extent *ext2 = xmalloc(sizeof(orc_extent) * n_req);
    uint64_t tot2[2];
    orc_sqe *sqe2 = xmalloc(sizeof(orc_sqe) * tot[1]);
    uint8_t *stage2 = xmalloc(tot[0]);
    memset(stage2, 0xA5, tot[0]);
    st = 0;
    CHECK(orc_layer_save(&pool, &cfg, nb, n_req, table, total, fid, layer, stage2, tot[0], 4096 * 7, 9, ext2, tot2, sqe2,
                         (uint32_t)tot[1], &st) == ORC_OK);
    CHECK(memcmp(stage2, stage, tot[0]) == 0 && memcmp(ext2, ext, sizeof(orc_extent) * n_req) == 0);
    for (uint64_t i = 0; i < tot[1]; ++i) CHECK(sqe2[i].opcode == ORC_OP_WRITE && sqe2[i].addr == sqe[i].addr);
    uint8_t *k3 = xmalloc(N * stride), *v3 = xmalloc(N * stride);
    memset(k3, 0, N * stride);
    memset(v3, 0, N * stride);
    orc_pool pool3 = pool;
    pool3.k_base = k3;
    pool3.v_base = v3;
    CHECK(orc_layer_restore(&pool3, &cfg, nb, n_req, table, total, fid, layer, stage, tot[0], 4096 * 7, 9, ext2, tot2, sqe2,
                            (uint32_t)tot[1], &st) == ORC_OK);
    CHECK(memcmp(k3, k2, N * stride) == 0 && memcmp(v3, v2, N * stride) == 0);
    CHECK(memcmp(sqe2, sqe, sizeof(orc_sqe) * tot[1]) == 0);
    /* the ordered restore with the order orc_table_order gives (the identity when the table has a bad id) equals
     * the plain one */
    {
      uint32_t *visit = xmalloc(sizeof(uint32_t) * total);
      uint32_t st_o = 0;
      CHECK(orc_table_order(N, table, total, visit, &st_o) == ORC_OK);
      CHECK((st_o != 0) == (plant_bad != 0));
      uint8_t *k5 = xmalloc(N * stride), *v5 = xmalloc(N * stride);
      memset(k5, 0, N * stride);
      memset(v5, 0, N * stride);
      orc_pool pool5 = pool;
      pool5.k_base = k5;
      pool5.v_base = v5;
      uint32_t st5 = 0;
      CHECK(orc_layer_restore_ordered(&pool5, &cfg, nb, n_req, table, total, fid, layer, stage, tot[0], 4096 * 7, 9, ext2,
                                      tot2, sqe2, (uint32_t)tot[1], visit, &st5) == ORC_OK);
      CHECK(memcmp(k5, k3, N * stride) == 0 && memcmp(v5, v3, N * stride) == 0);
      free(k5);
      free(v5);
      free(visit);
    }
    free(k3);
    free(v3);
    free(stage2);
    free(sqe2);
    free(ext2);
  }

  /* direct mode and rings need whole alignment units per block and move raw bytes */
  if (bb % A == 0) {
    const uint32_t n_ctx = 2 * total;
    orc_sgl *sgl = xmalloc(sizeof(orc_sgl) * 2 * N);
    st = 0;
    CHECK(orc_sgl_table_build(&pool, (uint64_t)(uintptr_t)k, (uint64_t)(uintptr_t)v, 3, sgl, 2 * N, &st) == ORC_OK);
    CHECK(st == 0 && sgl[N].addr == (uint64_t)(uintptr_t)v && sgl[N - 1].addr == (uint64_t)(uintptr_t)k + (N - 1) * stride);
    orc_sqe *dsqe = xmalloc(sizeof(orc_sqe) * n_ctx);
    st = 0;
    const uint64_t base = 0x600000000000ull;
    CHECK(orc_sqe_build_direct(&pool, &cfg, ext, n_req, table, fid, layer, ORC_OP_WRITE, base, 3, dsqe, n_ctx, &st) == ORC_OK);
    CHECK((st != 0) == (plant_bad != 0));

    uint64_t max_obj = 0;
    for (uint32_t r = 0; r < n_req; ++r)
      if (ext[r].obj_bytes > max_obj) max_obj = ext[r].obj_bytes;
    const uint64_t file_stride = 2ull * L * max_obj + 16;
    const uint32_t n_files = n_req ? n_req : 1;
    uint8_t *store_a = xmalloc(n_files * file_stride), *store_b = xmalloc(n_files * file_stride);
    memset(store_a, 0x11, n_files * file_stride);
    memset(store_b, 0x11, n_files * file_stride);
    orc_filestore fa = {store_a, file_stride, 500, n_files}, fb = {store_b, file_stride, 500, n_files};
    const uint32_t depth = 3, n_slots = (n_ctx + ORC_IOCB_SLOTS - 1) / ORC_IOCB_SLOTS;
    CHECK(n_slots <= depth);
    orc_iocb *sq_a = xmalloc(sizeof(orc_iocb) * depth), *sq_b = xmalloc(sizeof(orc_iocb) * depth);
    uint8_t *cq_a = xmalloc(sizeof(orc_cq_hdr) + 4 * depth), *cq_b = xmalloc(sizeof(orc_cq_hdr) + 4 * depth);
    memset(sq_a, 0, sizeof(orc_iocb) * depth);
    memset(sq_b, 0, sizeof(orc_iocb) * depth);
    CHECK(orc_ring_init(sq_a, cq_a, depth) == ORC_OK && orc_ring_init(sq_b, cq_b, depth) == ORC_OK);
    const uint32_t first = rnd() % depth;
    uint32_t st_a = 0, st_b = 0;
    /* three steps on A, one call on B */
    CHECK(orc_iocb_fill_direct(sq_a, depth, first, n_slots, &pool, &cfg, ext, n_req, table, fid, layer, ORC_OP_WRITE, base,
                               3, &st_a) == ORC_OK);
    CHECK(orc_issue_io(sq_a, cq_a, depth, first, n_slots, sgl, 2 * N, base, &fa, bb, &st_a) == ORC_OK);
    orc_extent *ext_b = xmalloc(sizeof(orc_extent) * n_req);
    uint64_t tot_b[2];
    CHECK(orc_store_layer(sq_b, cq_b, depth, first, n_slots, &pool, &cfg, nb, n_req, table, fid, layer, base, 3, &fb, ext_b,
                          tot_b, &st_b) == ORC_OK);
    CHECK(st_a == st_b && memcmp(store_a, store_b, n_files * file_stride) == 0);
    CHECK(memcmp(sq_a, sq_b, sizeof(orc_iocb) * depth) == 0 && memcmp(cq_a, cq_b, sizeof(orc_cq_hdr) + 4 * depth) == 0);
    CHECK(memcmp(ext_b, ext, sizeof(orc_extent) * n_req) == 0 && tot_b[0] == tot[0]);
    /* the file holds what the staged mode packs (token-major pools only: the direct mode moves raw blocks) */
    if (layout == ORC_LAYOUT_NHD && !plant_bad) {
      for (uint32_t r = 0; r < n_req; ++r)
        for (uint32_t kind = 0; kind < 2; ++kind)
          CHECK(memcmp(store_a + (uint64_t)r * file_stride + (2ull * layer + kind) * ext[r].obj_bytes,
                       stage + ext[r].stage_off + kind * ext[r].obj_bytes, (uint64_t)nb[r] * bb) == 0);
    }
    /* and a retrieve from that file into a zeroed pool brings the named blocks back */
    memset(k2, 0, N * stride);
    memset(v2, 0, N * stride);
    st_b = 0;
    CHECK(orc_retrieve_layer(sq_b, cq_b, depth, (first + 1) % depth, n_slots, &pool2, &cfg, nb, n_req, table, fid, layer,
                             base, 3, &fb, ext_b, tot_b, &st_b) == ORC_OK);
    for (uint32_t b = 0; b < N; ++b)
      if (named[b]) CHECK(memcmp(k2 + b * stride, k + b * stride, bb) == 0 && memcmp(v2 + b * stride, v + b * stride, bb) == 0);
    free(ext_b);
    free(cq_a);
    free(cq_b);
    free(sq_a);
    free(sq_b);
    free(store_a);
    free(store_b);
    free(dsqe);
    free(sgl);
  }

  free(sqe);
  free(named);
  free(k2);
  free(v2);
  free(stage);
  free(ext);
  free(table);
  free(perm);
  free(fid);
  free(nb);
  free(k);
  free(v);
}

int main(int argc, char **argv) {
  const int n = argc > 1 ? atoi(argv[1]) : 300;
  for (case_no = 0; case_no < n; ++case_no) one_case();
  printf("ok %d\n", n);
  return 0;
}
