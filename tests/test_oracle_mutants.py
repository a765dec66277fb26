"""CPU test of the pins themselves: each plausible mistake, planted in a copy of the oracle's
source and compiled with gcc, must be caught by at least one check of tests/oracle_checks.py.
The mistakes are planted in the oracle only, on the CPU; nothing here touches the HIP path."""
import os
import subprocess
import sys

import pytest

import oracle_checks as oc

SRC = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "oracle", "tutti_oracle.c")

MUTANTS = {
    "v_object_overlaps_k": ("stage += 2 * obj;", "stage += obj;"),
    "entries_counted_once": ("n_sqe += 2 * chunks;", "n_sqe += chunks;"),
    "align_down": ("return (x + a - 1) / a * a;", "return x / a * a;"),
    "chunks_floor": ("uint64_t chunks = (obj + C - 1) / C;", "uint64_t chunks = obj / C;"),
    "table_off_is_request": ("extents[r].table_off = (uint32_t)n_tab;", "extents[r].table_off = r;"),
    "k_v_planes_swapped": ("kind == 0 ? pool->k_base : pool->v_base", "kind == 1 ? pool->k_base : pool->v_base", 0),
    "ordered_k_v_planes_swapped": ("kind == 0 ? pool->k_base : pool->v_base",
                                   "kind == 1 ? pool->k_base : pool->v_base", 1),
    "v_object_at_k": ("uint8_t *obj = stage + x->stage_off + kind * x->obj_bytes;",
                      "uint8_t *obj = stage + x->stage_off;"),
    "hnd_ignored": ("? in_obj : ((i * T + t) * d) * e;", "? in_obj : ((t * h + i) * d) * e;"),
    "hnd_transposed_wrong": ("((i * T + t) * d) * e;", "((i * h + t) * d) * e;"),
    "stride_ignored": ("plane + (uint64_t)id * pool->block_stride", "plane + (uint64_t)id * bb", 0),
    "ordered_stride_ignored": ("plane + (uint64_t)id * pool->block_stride", "plane + (uint64_t)id * bb", 1),
    "object_uses_stride": ("obj + (uint64_t)j * bb, to_object", "obj + (uint64_t)j * pool->block_stride, to_object"),
    "padding_not_zeroed": ("memset(obj + filled, 0,", "if (0) memset(obj + filled, 0,"),
    "table_offset_dropped": ("uint32_t id = block_table[g];", "uint32_t id = block_table[j];"),
    "block_bound_off_by_one": ("if (id >= pool->num_blocks) {", "if (id > pool->num_blocks) {", 0),
    "ordered_block_bound_off_by_one": ("if (id >= pool->num_blocks) {", "if (id > pool->num_blocks) {", 1),
    "unpack_direction": ("(uint8_t *)(uintptr_t)stage, stage_cap, 0, 0, UINT64_MAX,",
                         "(uint8_t *)(uintptr_t)stage, stage_cap, 1, 0, UINT64_MAX,"),
    "file_off_layer_kind": ("s.file_off = (2ull * layer + kind)", "s.file_off = (2ull * kind + layer)", 0),
    "direct_file_off_layer_kind": ("s.file_off = (2ull * layer + kind)", "s.file_off = (2ull * kind + layer)", 1),
    "direct_file_id_of_first": ("make_direct_entry(pool, x, r, kind, j, id, file_id[r],",
                                "make_direct_entry(pool, x, r, kind, j, id, file_id[0],"),
    "direct_iocb_div_mod_swapped": ("s.iocb_idx = (uint32_t)(i / ORC_IOCB_SLOTS);",
                                    "s.iocb_idx = (uint32_t)(i % ORC_IOCB_SLOTS);", 1),
    "direct_user_data_swapped": ("s.user_data = ((uint64_t)r << 32) | (uint32_t)i;",
                                 "s.user_data = ((uint64_t)i << 32) | r;", 1),
    "direct_rsvd_dirty": ("memset(&s, 0, sizeof s);", "memset(&s, 0xff, sizeof s);", 1),
    "file_off_all_k_then_v": ("s.file_off = (2ull * layer + kind) * x->obj_bytes",
                              "s.file_off = ((uint64_t)kind * cfg->num_layers + layer) * x->obj_bytes", 0),
    "addr_without_kind": ("s.addr = stage_addr + x->stage_off + (uint64_t)kind * x->obj_bytes",
                          "s.addr = stage_addr + x->stage_off"),
    "len_always_chunk": ("s.len = (uint32_t)(left < C ? left : C);", "s.len = (uint32_t)C;"),
    "iocb_div_mod_swapped": ("s.iocb_idx = (uint32_t)(i / ORC_IOCB_SLOTS);", "s.iocb_idx = (uint32_t)(i % ORC_IOCB_SLOTS);", 0),
    "iocb_2000": ("s.ioctx_slot = (uint32_t)(i % ORC_IOCB_SLOTS);", "s.ioctx_slot = (uint32_t)(i % 2000);", 0),
    "user_data_swapped": ("s.user_data = ((uint64_t)r << 32) | (uint32_t)i;", "s.user_data = ((uint64_t)i << 32) | r;", 0),
    "entries_interleaved": ("(uint64_t)x->sqe_base + (uint64_t)kind * x->n_chunks + c;",
                            "(uint64_t)x->sqe_base + 2ull * c + kind;"),
    "file_id_of_first": ("s.file_id = file_id[r];", "s.file_id = file_id[0];", 0),
    "rsvd_dirty": ("memset(&s, 0, sizeof s);", "memset(&s, 0xff, sizeof s);", 0),
    "cap_check_inclusive": ("x->obj_bytes > (stage_cap - x->stage_off) / 2) {", "x->obj_bytes >= (stage_cap - x->stage_off) / 2) {"),
    "cap_check_overflows": ("if (x->stage_off > stage_cap || x->obj_bytes > (stage_cap - x->stage_off) / 2) {",
                            "if (x->stage_off + 2 * x->obj_bytes > stage_cap) {"),
    "table_sum_inclusive": ("if (used > table_len) {", "if (used >= table_len) {"),
    "table_sum_unchecked": ("if (used > table_len) {", "if (0) {"),
    "table_sum_skips_only_one": ("    used += x->n_blocks;\n    if (used > table_len) {",
                                 "    if (used + x->n_blocks > table_len) {\n      st |= ORC_ST_BAD_EXTENT;\n      continue;\n    }\n    used += x->n_blocks;\n    if (0) {"),
    "extent_alignment_unchecked": ("if (x->stage_off % 16 != 0 || x->obj_bytes % 16 != 0) {", "if (0) {"),
    "block_beyond_object_moved": ("if (((uint64_t)j + 1) * bb > x->obj_bytes) continue;", ""),
    "block_beyond_object_off_by_one": ("if (((uint64_t)j + 1) * bb > x->obj_bytes) continue;",
                                       "if (((uint64_t)j + 2) * bb > x->obj_bytes) continue;"),
    "table_position_unchecked": ("if (g >= table_len) {", "if (0) {"),
    "v_object_after_blocks": ("uint8_t *obj = stage + x->stage_off + kind * x->obj_bytes;",
                              "uint8_t *obj = stage + x->stage_off + kind * filled;"),
    "dense_check_skipped_sqe": ("if (!extents_are_dense(pool, cfg, extents, n_req)) {", "if (0) {", 0),
    "dense_check_skipped_direct": ("if (!extents_are_dense(pool, cfg, extents, n_req)) {", "if (0) {", 1),
    "dense_check_skipped_fill": ("if (!extents_are_dense(pool, cfg, extents, n_req)) {", "if (0) {", 2),
    "dense_ignores_sizes": ("if (x->obj_bytes != obj || x->n_chunks != chunks) return 0;", ""),
    "dense_ignores_offsets": ("if (x->sqe_base != want_sqe || x->table_off != want_tab) return 0;", ""),
    "dense_ignores_wrap": ("if (want_sqe > 0xffffffffull || want_tab > 0xffffffffull) return 0;", ""),
    "order_descending": ("while (m > 0 && block_table[visit[m - 1]] > block_table[pos]) {",
                         "while (m > 0 && block_table[visit[m - 1]] < block_table[pos]) {"),
    "order_by_position": ("while (m > 0 && block_table[visit[m - 1]] > block_table[pos]) {",
                          "while (m > 0 && visit[m - 1] > block_table[pos]) {"),
    "order_sorts_invalid_tables": ("  if (st) return ORC_OK;\n  /* insertion sort", "  /* insertion sort"),
    "ordered_uses_list_index": ("      const uint64_t pos = visit[k];", "      const uint64_t pos = k;"),
    "ordered_ignores_dead_requests": ("      if (pos >= live_blocks) continue;", "      if (pos >= table_len) continue;"),
    "ordered_object_offset_by_list": ("move_block(pool, plane + (uint64_t)id * pool->block_stride, obj + j * bb, 0);",
                                      "move_block(pool, plane + (uint64_t)id * pool->block_stride, obj + (uint64_t)k * bb, 0);"),
    "ordered_packs": ("move_block(pool, plane + (uint64_t)id * pool->block_stride, obj + j * bb, 0);",
                      "move_block(pool, plane + (uint64_t)id * pool->block_stride, obj + j * bb, 1);"),
    "table_off_ignored": ("uint64_t g = (uint64_t)x->table_off + j;", "uint64_t g = used - x->n_blocks + j;"),
    "sgl_v_plane_uses_k_address": ("table[i].addr = (kind == 0 ? k_addr : v_addr) + (uint64_t)b * pool->block_stride;",
                                   "table[i].addr = k_addr + (uint64_t)b * pool->block_stride;"),
    "sgl_ignores_stride": ("table[i].addr = (kind == 0 ? k_addr : v_addr) + (uint64_t)b * pool->block_stride;",
                           "table[i].addr = (kind == 0 ? k_addr : v_addr) + (uint64_t)b * bb;"),
    "sgl_len_is_stride": ("table[i].len = bb;", "table[i].len = (uint32_t)pool->block_stride;"),
    "direct_descriptor_of_k_only": ("s.addr = sgl_table_addr + 16ull * ((uint64_t)kind * pool->num_blocks + id);",
                                    "s.addr = sgl_table_addr + 16ull * id;"),
    "direct_addr_by_position": ("s.addr = sgl_table_addr + 16ull * ((uint64_t)kind * pool->num_blocks + id);",
                                "s.addr = sgl_table_addr + 16ull * ((uint64_t)kind * pool->num_blocks + j);"),
    "direct_file_off_by_id": ("s.file_off = (2ull * layer + kind) * x->obj_bytes + (uint64_t)j * bb;",
                              "s.file_off = (2ull * layer + kind) * x->obj_bytes + (uint64_t)id * bb;"),
    "fill_table_offset_dropped": ("block_table[(uint64_t)x->table_off + j], file_id[r], layer, opcode,",
                                  "block_table[j], file_id[r], layer, opcode,"),
    "direct_index_interleaved": ("uint64_t i = 2ull * x->table_off + (uint64_t)kind * x->n_blocks + j;",
                                 "uint64_t i = 2ull * x->table_off + 2ull * j + kind;", 0),
    "fill_index_interleaved": ("uint64_t i = 2ull * x->table_off + (uint64_t)kind * x->n_blocks + j;",
                               "uint64_t i = 2ull * x->table_off + 2ull * j + kind;", 1),
    "direct_table_offset_dropped": ("uint32_t id = block_table[(uint64_t)x->table_off + j];",
                                    "uint32_t id = block_table[j];"),
    "direct_bad_id_bound": ("if (id < pool->num_blocks) {\n    s.addr", "if (id <= pool->num_blocks) {\n    s.addr"),
    "ring_index_not_unique": ("sq[b].hdr.iocb_idx = b;", "sq[b].hdr.iocb_idx = 0;"),
    "ring_no_wraparound": ("orc_iocb *io = &sq[(first_slot + (uint32_t)(i / ORC_IOCB_SLOTS)) % depth];",
                           "orc_iocb *io = &sq[(first_slot + (uint32_t)(i / ORC_IOCB_SLOTS)) % (depth + 1)];"),
    "ring_num_ioctx_full": ("io->hdr.num_ioctx = (uint32_t)cnt;", "io->hdr.num_ioctx = ORC_IOCB_SLOTS;"),
    "ring_slot_position": ("orc_sqe *s = &io->ioctx[i % ORC_IOCB_SLOTS];", "orc_sqe *s = &io->ioctx[i % 2047];"),
    "io_direction_swapped": ("if (s->opcode == ORC_OP_READ)\n        memcpy(blk, fil, s->len);",
                             "if (s->opcode == ORC_OP_WRITE)\n        memcpy(blk, fil, s->len);"),
    "io_file_stride_ignored": ("(uint64_t)(s->file_id - store->first_file_id) * store->file_stride + s->file_off;",
                               "s->file_off;"),
    "io_descriptor_index": ("uint64_t di = (s->addr - sgl_table_addr) / 16;", "uint64_t di = (s->addr - sgl_table_addr) / 32;"),
    "io_cq_index": ("entry[c->tail % depth] = io->hdr.iocb_idx;", "entry[c->tail % depth] = b;"),
    "io_not_marked_done": ("io->hdr.state = ORC_IOCB_DONE;", "io->hdr.state = ORC_IOCB_FILLED;"),
    "io_file_bound": ("s->file_off > store->file_stride || s->len > store->file_stride - s->file_off) {",
                      "s->file_off > store->file_stride) {"),
    "io_file_bound_wraps": ("s->file_off > store->file_stride || s->len > store->file_stride - s->file_off) {",
                            "s->file_off + s->len > store->file_stride) {"),
    "io_opcode_unchecked": ("if (s->opcode != ORC_OP_READ && s->opcode != ORC_OP_WRITE) {", "if (0) {"),
    "io_max_len_unchecked": ("if (s->len > max_len || s->len % 16 != 0", "if (s->len % 16 != 0"),
    "io_len_alignment_unchecked": ("s->len % 16 != 0 || s->file_off % 16 != 0 ||", "s->file_off % 16 != 0 ||"),
    "io_offset_alignment_unchecked": ("s->len % 16 != 0 || s->file_off % 16 != 0 ||", "s->len % 16 != 0 ||"),
    "io_block_alignment_unchecked": (" || sgl_table[di].addr % 16 != 0) {", ") {"),
    "io_descriptor_length_unchecked": ("if (di >= n_desc || s->len > sgl_table[di].len) {", "if (di >= n_desc) {"),
    "io_address_between_descriptors": ("if (s->addr < sgl_table_addr || (s->addr - sgl_table_addr) % 16 != 0) {",
                                       "if (s->addr < sgl_table_addr) {"),
    "io_runs_beyond_num_ioctx": ("k < io->hdr.num_ioctx && k < ORC_IOCB_SLOTS; ++k) {", "k < ORC_IOCB_SLOTS; ++k) {"),
    "io_zero_length_is_error": ("if (s->len == 0) continue; /* a no-op context */",
                                "if (s->len == 0) { st |= ORC_ST_BAD_BLOCK; continue; }"),
    "save_builds_read": ("ORC_OP_WRITE, stage_addr, sgl_id, sqe, sqe_cap, status);",
                         "ORC_OP_READ, stage_addr, sgl_id, sqe, sqe_cap, status);"),
    "save_unpacks": ("  return orc_obj_pack(pool, cfg, extents, n_req, block_table, table_len, stage, stage_cap, status);\n}\n\n/* retrieve_layer",
                     "  return orc_obj_unpack(pool, cfg, extents, n_req, block_table, table_len, stage, stage_cap, status);\n}\n\n/* retrieve_layer"),
    "ring_layer_planes_swapped": ("(uint64_t)(uintptr_t)pool->k_base, (uint64_t)(uintptr_t)pool->v_base, sgl_id, table,",
                                  "(uint64_t)(uintptr_t)pool->v_base, (uint64_t)(uintptr_t)pool->k_base, sgl_id, table,"),
    "retrieve_layer_writes": ("return ring_layer(ORC_OP_READ, sq,", "return ring_layer(ORC_OP_WRITE, sq,"),
    "store_layer_reads": ("return ring_layer(ORC_OP_WRITE, sq,", "return ring_layer(ORC_OP_READ, sq,"),
    "ring_layer_half_table": ("const uint32_t n_desc = 2u * pool->num_blocks;", "const uint32_t n_desc = 1u * pool->num_blocks;"),
    "ring_layer_skips_issue": ("  if (!rc)\n    rc = orc_issue_io(sq, cq, depth, first_slot, n_slots, table, n_desc,",
                               "  if (rc)\n    rc = orc_issue_io(sq, cq, depth, first_slot, n_slots, table, n_desc,"),
    "validate_first_seen_counts": ("    } else if (seen[id]) {\n      st |= ORC_ST_DUP_BLOCK;\n    } else {\n      seen[id] = 1;",
                                   "    } else if (seen[id]++) {\n      st |= ORC_ST_DUP_BLOCK;\n    } else {\n      seen[id] = 0;"),
    "validate_bound_off_by_one": ("    if (id >= num_blocks) {\n      st |= ORC_ST_BAD_BLOCK;", "    if (id > num_blocks) {\n      st |= ORC_ST_BAD_BLOCK;"),
    "validate_bad_ids_as_duplicates": ("    if (id >= num_blocks) {\n      st |= ORC_ST_BAD_BLOCK;\n    } else if (seen[id]) {",
                                       "    if (id >= num_blocks) {\n      st |= ORC_ST_BAD_BLOCK | ORC_ST_DUP_BLOCK;\n    } else if (seen[id]) {"),
    "restore_builds_write": ("ORC_OP_READ, stage_addr, sgl_id, sqe, sqe_cap, status);",
                             "ORC_OP_WRITE, stage_addr, sgl_id, sqe, sqe_cap, status);", 0),
    "ordered_restore_builds_write": ("ORC_OP_READ, stage_addr, sgl_id, sqe, sqe_cap, status);",
                                     "ORC_OP_WRITE, stage_addr, sgl_id, sqe, sqe_cap, status);", 1),
}


RUNNER = """
import ctypes, sys
sys.path.insert(0, {root!r}); sys.path.insert(0, {tests!r})
from oracle import tutti_oracle as orc
import oracle_checks as oc
lib = ctypes.CDLL({so!r})
lib.orc_block_bytes.restype = ctypes.c_uint32
lib.orc_desc_count.restype = ctypes.c_uint64
lib.orc_desc_count.argtypes = [ctypes.c_uint64, ctypes.c_uint64]
orc._LIB = lib
for check in oc.ALL_CHECKS:
    try:
        check(orc)
    except (AssertionError, orc.OracleError, IndexError, ValueError):
        print("caught by", check.__name__)
        sys.exit(3)
sys.exit(0)
"""


@pytest.mark.parametrize("name", sorted(MUTANTS))
def test_mutant_is_caught(orc, tmp_path, name):
    old, new, *which = MUTANTS[name]
    which = which[0] if which else 0        # which occurrence of the site to change (default: the only one)
    text = open(SRC).read()
    assert text.count(old) == (1 if not MUTANTS[name][2:] else text.count(old)) and text.count(old) > which, \
        f"mutation site for {name} not found as expected in the oracle source"
    parts = text.split(old)
    mutated = old.join(parts[:which + 1]) + new + old.join(parts[which + 1:])
    src = tmp_path / "mutant.c"
    src.write_text(mutated)
    so = tmp_path / "libmutant.so"
    subprocess.run(["gcc", "-std=c11", "-O1", "-w", "-fPIC", "-shared", "-pthread", f"-I{os.path.dirname(SRC)}",
                    str(src), "-o", str(so)], check=True)
    # a separate process: a broken oracle may run out of bounds and take the interpreter with it
    tests = os.path.dirname(os.path.abspath(__file__))
    code = RUNNER.format(root=os.path.dirname(tests), tests=tests, so=str(so))
    r = subprocess.run([sys.executable, "-c", code], capture_output=True, text=True, timeout=300)
    assert r.returncode != 0, f"no pin notices the mistake '{name}'"
