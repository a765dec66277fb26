"""CPU tests of the boundary: the library loads, exports what include/tutti.h declares, agrees
with the oracle on every record layout, and rejects bad host arguments before touching HIP."""
import os
import re

import numpy as np
import pytest

from paper_2605_03375_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared(header_name):
    header = open(os.path.join(ROOT, "include", header_name)).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)          # comments mention calls of other headers
    return sorted(set(re.findall(r"\b(tutti_[a-z_0-9]+)\s*\(", header)))


def test_library_exports_every_declared_symbol():
    """libtutti.so exports exactly what include/tutti.h declares; libtutti_bench.so (the same sources with the
    measurement aids compiled in) exports that plus what include/tutti_bench.h declares."""
    import subprocess
    declared = _declared("tutti.h")
    bench_declared = _declared("tutti_bench.h")
    assert set(declared) == set(B.EXPORTS) and set(bench_declared) == set(B.BENCH_EXPORTS)
    for path, names in ((B.LIB_PATH, declared), (B.BENCH_LIB_PATH, declared + bench_declared)):
        out = subprocess.run(["nm", "-D", "--defined-only", path], capture_output=True, text=True, check=True).stdout
        exported = sorted(line.split()[-1] for line in out.splitlines() if " T tutti_" in line)
        assert exported == sorted(names), path
    L, LB = B.product_lib(), B.bench_lib()
    for name in declared:
        assert getattr(L, name) is not None and getattr(LB, name) is not None
    for name in bench_declared:
        assert getattr(LB, name) is not None and not hasattr(L, name)
    for name in ("tutti_obj_layout", "tutti_obj_pack", "tutti_obj_unpack", "tutti_sqe_build", "tutti_layer_restore",
                 "tutti_layer_save", "tutti_sgl_table_build", "tutti_sqe_build_direct", "tutti_ring_init", "tutti_iocb_fill_direct",
                 "tutti_issue_io", "tutti_wait_cqe"):
        assert name in declared and callable(getattr(B, name))
    assert B.tutti_version() >= 0x100


def test_record_layouts_agree_with_oracle(orc):
    lib_abi = B.tutti_abi_describe()
    assert lib_abi == orc.abi_describe()
    E, S = B.EXTENT_DTYPE, B.SQE_DTYPE
    assert [E.itemsize] + [E.fields[n][1] for n in E.names] == lib_abi[0:7]
    assert [S.itemsize] + [S.fields[n][1] for n in S.names[:-1]] == lib_abi[7:19]
    import ctypes
    assert ctypes.sizeof(B.tutti_pool) == lib_abi[19] and ctypes.sizeof(B.tutti_objcfg) == lib_abi[29]
    assert [getattr(B.tutti_pool, f).offset for f, _ in B.tutti_pool._fields_] == lib_abi[20:29]
    assert [getattr(B.tutti_objcfg, f).offset for f, _ in B.tutti_objcfg._fields_] == lib_abi[30:33]
    G = B.SGL_DTYPE
    assert [G.itemsize] + [G.fields[n][1] for n in G.names] == lib_abi[33:37]
    Hd, Io = B.IOCB_HDR_DTYPE, B.IOCB_DTYPE
    assert [Hd.itemsize] + [Hd.fields[n][1] for n in Hd.names] == lib_abi[37:44]
    assert [Io.itemsize, Io.fields["ioctx"][1]] == lib_abi[44:46] and B.CQ_HDR_BYTES == lib_abi[46]
    assert [ctypes.sizeof(B.tutti_filestore)] + [getattr(B.tutti_filestore, f).offset
                                                 for f, _ in B.tutti_filestore._fields_] == lib_abi[47:52]
    assert ctypes.sizeof(B.tutti_ring) == 24 and B.ring_bytes(3) == (3 * 131136, 64 + 12)
    for a, b in [(B.OP_READ, orc.OP_READ), (B.OP_WRITE, orc.OP_WRITE), (B.LAYOUT_HND, orc.LAYOUT_HND),
                 (B.IOCB_SLOTS, orc.IOCB_SLOTS), (B.ST_BAD_BLOCK, orc.ST_BAD_BLOCK),
                 (B.ST_STAGE_CAP, orc.ST_STAGE_CAP), (B.ST_SQE_CAP, orc.ST_SQE_CAP)]:
        assert a == b


def test_header_is_plain_c(tmp_path):
    """include/tutti.h compiles as strict C11 and as C++17 on its own, with the record sizes the ABI promises."""
    import subprocess
    src = """
#include "tutti.h"
_Static_assert(sizeof(tutti_extent) == 32, "extent");
_Static_assert(sizeof(tutti_sqe) == 64, "sqe");
_Static_assert(sizeof(tutti_sgl) == 16, "sgl");
_Static_assert(sizeof(tutti_iocb_hdr) == 64, "iocb header");
_Static_assert(sizeof(tutti_iocb) == 64 + 64 * TUTTI_IOCB_SLOTS, "iocb");
_Static_assert(sizeof(tutti_cq_hdr) == 64, "cq header");
int (*const p_restore)(const tutti_pool *, const tutti_objcfg *, const uint32_t *, uint32_t, const uint32_t *, uint32_t,
                       const uint32_t *, uint32_t, const void *, uint64_t, uint64_t, uint32_t, tutti_extent *,
                       uint64_t *, tutti_sqe *, uint32_t, uint32_t, uint32_t *, void *) = tutti_layer_restore;
int main(void) { (void)p_restore; return 0; }
"""
    inc = os.path.join(ROOT, "include")
    c = tmp_path / "abi.c"
    c.write_text(src)
    subprocess.run(["gcc", "-std=c11", "-pedantic", "-Wall", "-Wextra", "-Werror", "-fsyntax-only", f"-I{inc}", str(c)],
                   check=True)
    cpp = tmp_path / "abi.cc"
    cpp.write_text(src.replace("_Static_assert", "static_assert"))
    subprocess.run(["g++", "-std=c++17", "-pedantic", "-Wall", "-Wextra", "-Werror", "-fsyntax-only", f"-I{inc}",
                    str(cpp)], check=True)


def test_strerror():
    for code in (B.OK, B.EINVAL, B.ERANGE, B.EHIP, B.EAGAIN, -99):
        assert isinstance(B.tutti_strerror(code), str) and B.tutti_strerror(code)


GOOD = dict(num_blocks=8, block_tokens=16, num_kv_heads=2, head_dim=64, elt_bytes=2)
FAKE = 0x10000  # a non-null, 16-byte aligned stand-in for device pointers: never dereferenced on these paths


def _expect(code, fn, *a, **kw):
    with pytest.raises(B.TuttiError) as ei:
        fn(*a, **kw, stream=0)
    assert ei.value.code == code, ei.value


@pytest.mark.parametrize("bad", [dict(block_tokens=0), dict(num_blocks=0), dict(head_dim=3, elt_bytes=1,
                                 block_tokens=1, num_kv_heads=1), dict(block_stride=4000), dict(block_stride=4104),
                                 dict(pool_layout=2)])
def test_bad_pool_is_einval(bad):
    kw = dict(GOOD)
    kw.update(bad)
    p = B.make_pool(FAKE, FAKE, **kw)
    _expect(B.EINVAL, B.tutti_obj_layout, p, B.make_cfg(), FAKE, 1, FAKE, FAKE)
    _expect(B.EINVAL, B.tutti_obj_pack, p, B.make_cfg(), FAKE, 1, FAKE, 1, FAKE, 1 << 20)
    _expect(B.EINVAL, B.tutti_obj_unpack, p, B.make_cfg(), FAKE, 1, FAKE, 1, FAKE, 1 << 20)
    _expect(B.EINVAL, B.tutti_sqe_build, p, B.make_cfg(), FAKE, 1, FAKE, 0, B.OP_READ, 0, 0, FAKE, 4)
    _expect(B.EINVAL, B.tutti_layer_restore, p, B.make_cfg(), FAKE, 1, FAKE, 1, FAKE, 0, FAKE, 1 << 20, 0, 0, FAKE,
            FAKE, FAKE, 4)
    _expect(B.EINVAL, B.tutti_layer_save, p, B.make_cfg(), FAKE, 1, FAKE, 1, FAKE, 0, FAKE, 1 << 20, 0, 0, FAKE,
            FAKE, FAKE, 4)


@pytest.mark.parametrize("bad", [dict(align=4095), dict(align=8), dict(align=0), dict(chunk_bytes=0),
                                 dict(chunk_bytes=6144), dict(num_layers=0)])
def test_bad_cfg_is_einval(bad):
    kw = dict(align=4096, chunk_bytes=8192, num_layers=2)
    kw.update(bad)
    p = B.make_pool(FAKE, FAKE, **GOOD)
    _expect(B.EINVAL, B.tutti_obj_layout, p, B.make_cfg(**kw), FAKE, 1, FAKE, FAKE)
    _expect(B.EINVAL, B.tutti_sqe_build, p, B.make_cfg(**kw), FAKE, 1, FAKE, 0, B.OP_READ, 0, 0, FAKE, 4)


def test_null_and_misaligned_pointers_are_einval():
    cfg = B.make_cfg(num_layers=2)
    p = B.make_pool(FAKE, FAKE, **GOOD)
    _expect(B.EINVAL, B.tutti_obj_layout, p, cfg, 0, 1, FAKE, FAKE)
    _expect(B.EINVAL, B.tutti_obj_layout, p, cfg, FAKE, 1, 0, FAKE)
    _expect(B.EINVAL, B.tutti_obj_layout, p, cfg, FAKE, 1, FAKE, 0)
    _expect(B.EINVAL, B.tutti_obj_pack, p, cfg, 0, 1, FAKE, 1, FAKE, 4096)
    _expect(B.EINVAL, B.tutti_obj_pack, p, cfg, FAKE, 1, 0, 1, FAKE, 4096)
    _expect(B.EINVAL, B.tutti_obj_pack, p, cfg, FAKE, 1, FAKE, 1, 0, 4096)
    _expect(B.EINVAL, B.tutti_obj_unpack, p, cfg, FAKE, 1, FAKE, 1, FAKE + 8, 4096)      # staging not 16-aligned
    _expect(B.EINVAL, B.tutti_obj_pack, B.make_pool(0, FAKE, **GOOD), cfg, FAKE, 1, FAKE, 1, FAKE, 4096)
    _expect(B.EINVAL, B.tutti_obj_pack, B.make_pool(FAKE, FAKE + 4, **GOOD), cfg, FAKE, 1, FAKE, 1, FAKE, 4096)
    _expect(B.EINVAL, B.tutti_sqe_build, p, cfg, FAKE, 1, 0, 0, B.OP_READ, 0, 0, FAKE, 4)
    _expect(B.EINVAL, B.tutti_sqe_build, p, cfg, FAKE, 1, FAKE, 0, B.OP_READ, 0, 0, 0, 4)
    _expect(B.EINVAL, B.tutti_sqe_build, p, cfg, FAKE, 1, FAKE, 2, B.OP_READ, 0, 0, FAKE, 4)        # layer >= L
    _expect(B.EINVAL, B.tutti_sqe_build, p, cfg, FAKE, 1, FAKE, 0, 3, 0, 0, FAKE, 4)                # opcode
    _expect(B.EINVAL, B.tutti_sqe_build, p, cfg, FAKE, 1, FAKE, 0, B.OP_READ, 100, 0, FAKE, 4)      # stage_addr
    _expect(B.EINVAL, B.tutti_layer_restore, p, cfg, FAKE, 1, FAKE, 1, FAKE, 2, FAKE, 4096, 0, 0, FAKE, FAKE, FAKE, 4)
    _expect(B.EINVAL, B.tutti_layer_restore, p, cfg, FAKE, 1, FAKE, 1, FAKE, 0, FAKE, 4096, 0, 0, FAKE, 0, FAKE, 4)
    _expect(B.EINVAL, B.tutti_sqe_build_direct, p, cfg, FAKE, 1, FAKE, 1, FAKE, 0, B.OP_READ, 8, 0, FAKE, 4)  # table addr
    _expect(B.EINVAL, B.tutti_sqe_build_direct, p, cfg, FAKE, 1, FAKE, 1, FAKE, 5, B.OP_READ, 0, 0, FAKE, 4)  # layer
    _expect(B.EINVAL, B.tutti_sqe_build_direct, p, cfg, FAKE, 1, 0, 1, FAKE, 0, B.OP_READ, 0, 0, FAKE, 4)     # table
    odd = B.make_pool(FAKE, FAKE, num_blocks=8, block_tokens=16, num_kv_heads=5, head_dim=40, elt_bytes=2)
    _expect(B.EINVAL, B.tutti_sqe_build_direct, odd, cfg, FAKE, 1, FAKE, 1, FAKE, 0, B.OP_READ, 0, 0, FAKE, 4)
    _expect(B.EINVAL, B.tutti_sgl_table_build, p, 0, 0, 0, 0, 4)
    _expect(B.EINVAL, B.tutti_sgl_table_build, B.make_pool(FAKE, FAKE, **dict(GOOD, num_blocks=0)), 0, 0, 0, FAKE, 4)
    ring = B.make_ring(FAKE, FAKE, 4)
    fs = B.make_filestore(FAKE, 4096, 0, 1)
    _expect(B.EINVAL, B.tutti_ring_init, B.make_ring(0, FAKE, 4))
    _expect(B.EINVAL, B.tutti_ring_init, B.make_ring(FAKE, FAKE, 0))
    _expect(B.EINVAL, B.tutti_iocb_fill_direct, ring, 4, 1, p, cfg, FAKE, 1, FAKE, 1, FAKE, 0, B.OP_READ, 0, 0)  # slot
    _expect(B.EINVAL, B.tutti_iocb_fill_direct, ring, 0, 5, p, cfg, FAKE, 1, FAKE, 1, FAKE, 0, B.OP_READ, 0, 0)  # n_slots
    _expect(B.EINVAL, B.tutti_iocb_fill_direct, ring, 0, 1, p, cfg, FAKE, 1, FAKE, 1, FAKE, 0, 9, 0, 0)          # opcode
    _expect(B.EINVAL, B.tutti_issue_io, ring, 0, 1, FAKE, 4, 0, B.make_filestore(0, 4096, 0, 1), 4096)
    _expect(B.EINVAL, B.tutti_issue_io, ring, 0, 1, FAKE, 4, 0, B.make_filestore(FAKE, 4100, 0, 1), 4096)
    _expect(B.EINVAL, B.tutti_issue_io, ring, 0, 1, FAKE, 4, 0, fs, 0)
    _expect(B.EINVAL, B.tutti_issue_io, ring, 0, 1, 0, 4, 0, fs, 4096)
    for one_call in (B.tutti_retrieve_layer, B.tutti_store_layer):
        ok = (p, cfg, FAKE, 1, FAKE, 1, FAKE, 0, 0, 0, fs, FAKE, FAKE)
        _expect(B.EINVAL, one_call, B.make_ring(0, FAKE, 4), 0, 1, *ok)                                   # no SQ
        _expect(B.EINVAL, one_call, ring, 4, 1, *ok)                                                      # slot
        _expect(B.EINVAL, one_call, ring, 0, 5, *ok)                                                      # n_slots
        _expect(B.EINVAL, one_call, ring, 0, 1, odd, *ok[1:])                                             # block % align
        _expect(B.EINVAL, one_call, ring, 0, 1, B.make_pool(0, FAKE, **GOOD), *ok[1:])                    # no K plane
        _expect(B.EINVAL, one_call, ring, 0, 1, p, cfg, 0, 1, FAKE, 1, FAKE, 0, 0, 0, fs, FAKE, FAKE)     # n_blocks
        _expect(B.EINVAL, one_call, ring, 0, 1, p, cfg, FAKE, 1, 0, 1, FAKE, 0, 0, 0, fs, FAKE, FAKE)     # table
        _expect(B.EINVAL, one_call, ring, 0, 1, p, cfg, FAKE, 1, FAKE, 1, 0, 0, 0, 0, fs, FAKE, FAKE)     # file ids
        _expect(B.EINVAL, one_call, ring, 0, 1, p, cfg, FAKE, 1, FAKE, 1, FAKE, 2, 0, 0, fs, FAKE, FAKE)  # layer
        _expect(B.EINVAL, one_call, ring, 0, 1, p, cfg, FAKE, 1, FAKE, 1, FAKE, 0, 8, 0, fs, FAKE, FAKE)  # table addr
        _expect(B.EINVAL, one_call, ring, 0, 1, p, cfg, FAKE, 1, FAKE, 1, FAKE, 0, 0, 0,
                B.make_filestore(0, 4096, 0, 1), FAKE, FAKE)
        _expect(B.EINVAL, one_call, ring, 0, 1, p, cfg, FAKE, 1, FAKE, 1, FAKE, 0, 0, 0,
                B.make_filestore(FAKE, 4100, 0, 1), FAKE, FAKE)
        _expect(B.EINVAL, one_call, ring, 0, 1, p, cfg, FAKE, 1, FAKE, 1, FAKE, 0, 0, 0, fs, 0, FAKE)     # extents
        _expect(B.EINVAL, one_call, ring, 0, 1, p, cfg, FAKE, 1, FAKE, 1, FAKE, 0, 0, 0, fs, FAKE, 0)     # totals
        _expect(B.ERANGE, one_call, ring, 0, 1, p, cfg, FAKE, B.MAX_REQ + 1, FAKE, 1, FAKE, 0, 0, 0, fs, FAKE, FAKE)
    for chained in (B.tutti_retrieve_layer_chained, B.tutti_store_layer_chained):
        ok = (p, cfg, FAKE, 1, FAKE, 1, FAKE, 0, 0, 0, fs, FAKE, FAKE)
        _expect(B.EINVAL, chained, ring, 0, 1, 4, 1, *ok)              # the earlier call's first slot is not in the ring
        _expect(B.EINVAL, chained, ring, 0, 1, 1, 5, *ok)              # more of its slots than the ring has
        _expect(B.EINVAL, chained, ring, 0, 2, 1, 1, *ok)              # its slots are among the ones this call fills
        _expect(B.EINVAL, chained, ring, 3, 2, 0, 1, *ok)              # the same, with this call's slots wrapping
        _expect(B.EINVAL, chained, ring, 1, 1, 0, 2, *ok)              # this call's slot is among the earlier call's
        _expect(B.EINVAL, chained, ring, 4, 1, 0, 1, *ok)              # the ordinary checks still come first
        _expect(B.EINVAL, chained, ring, 0, 1, 2, 1, odd, *ok[1:])     # ... and after
    _expect(B.EINVAL, B.tutti_issue_io_chained, ring, 0, 2, 1, 1, FAKE, 4, 0, fs, 4096)   # overlapping slot ranges
    _expect(B.EINVAL, B.tutti_issue_io_chained, ring, 0, 1, 4, 1, FAKE, 4, 0, fs, 4096)   # earlier slots not in the ring
    _expect(B.EINVAL, B.tutti_issue_io_chained, ring, 0, 1, 2, 1, FAKE, 4, 0, fs, 0)      # the ordinary checks
    _expect(B.EINVAL, B.tutti_wait_cqe, ring, 4, FAKE)
    _expect(B.EINVAL, B.tutti_wait_cqe, ring, 0, 0)
    _expect(B.EINVAL, B.tutti_table_validate, 0, FAKE, 4, FAKE)
    _expect(B.EINVAL, B.tutti_table_validate, 8, 0, 4, FAKE)
    _expect(B.EINVAL, B.tutti_table_validate, 8, FAKE, 4, 0)
    _expect(B.EINVAL, B.tutti_table_validate_ws, 8, FAKE, 4, FAKE, 0, 256)
    _expect(B.EINVAL, B.tutti_table_validate_ws, 8, FAKE, 4, 0, FAKE, 256)
    _expect(B.ERANGE, B.tutti_table_validate_ws, 4096, FAKE, 4, FAKE, FAKE, 256)
    assert B.tutti_table_validate_work_bytes(1) == 256 and B.tutti_table_validate_work_bytes(65536) == 8192
    _expect(B.EINVAL, B.tutti_copy_baseline, FAKE, FAKE, 24)
    _expect(B.EINVAL, B.tutti_copy_baseline, 0, FAKE, 32)
    # head-major pools need rows of whole 16-byte units
    hp = B.make_pool(FAKE, FAKE, num_blocks=8, block_tokens=16, num_kv_heads=2, head_dim=4, elt_bytes=2,
                     pool_layout=B.LAYOUT_HND)
    _expect(B.EINVAL, B.tutti_obj_pack, hp, cfg, FAKE, 1, FAKE, 1, FAKE, 4096)


def test_too_many_requests_is_erange():
    p = B.make_pool(FAKE, FAKE, **GOOD)
    cfg = B.make_cfg()
    _expect(B.ERANGE, B.tutti_obj_layout, p, cfg, FAKE, B.MAX_REQ + 1, FAKE, FAKE)
    _expect(B.ERANGE, B.tutti_obj_pack, p, cfg, FAKE, B.MAX_REQ + 1, FAKE, 1, FAKE, 4096)
    _expect(B.ERANGE, B.tutti_sqe_build, p, cfg, FAKE, B.MAX_REQ + 1, FAKE, 0, B.OP_READ, 0, 0, FAKE, 4)


def test_tuning_arguments():
    with pytest.raises(B.TuttiError):
        B.tutti_set_tuning(0, 3)
    B.tutti_set_tuning(0, 0)


def test_empty_calls_do_not_need_a_gpu():
    """n_req = 0 is a no-op for pack / unpack / entries: nothing is enqueued."""
    p = B.make_pool(FAKE, FAKE, **GOOD)
    cfg = B.make_cfg()
    assert B.tutti_obj_pack(p, cfg, 0, 0, 0, 0, FAKE, 0, stream=0) == B.OK
    assert B.tutti_obj_unpack(p, cfg, 0, 0, 0, 0, FAKE, 0, stream=0) == B.OK
    assert B.tutti_sqe_build(p, cfg, 0, 0, 0, 0, B.OP_READ, 0, 0, 0, 0, stream=0) == B.OK
    assert B.tutti_copy_baseline(FAKE, FAKE, 0, stream=0) == B.OK


def test_table_order_arguments_are_checked_before_any_gpu_call():
    """The visiting-order call: sizes and pointers are checked on the host; an empty table enqueues nothing."""
    need = B.tutti_table_order_work_bytes(65536)
    assert need % 256 == 0 and need >= 2 * 65536 // 8 and need == 256 + 2 * B.tutti_table_validate_work_bytes(65536)
    assert B.tutti_table_order_work_bytes(1) == 256 + 2 * 256
    assert B.tutti_table_order(65536, 0, 0, 0, FAKE, need, stream=0) == B.OK
    for kw, code in ((dict(num_blocks=0), B.EINVAL), (dict(d_block_table=0), B.EINVAL), (dict(d_visit=0), B.EINVAL),
                     (dict(d_work=0), B.EINVAL), (dict(d_work=FAKE + 4), B.EINVAL), (dict(work_bytes=need - 1), B.ERANGE)):
        args = dict(num_blocks=65536, d_block_table=FAKE, table_len=8, d_visit=FAKE, d_work=FAKE, work_bytes=need)
        args.update(kw)
        with pytest.raises(B.TuttiError) as ei:
            B.tutti_table_order(**args, stream=0)
        assert ei.value.code == code, kw
    # the ordered restore checks what the plain one checks, before anything is enqueued
    p = B.make_pool(FAKE, FAKE, **GOOD)
    with pytest.raises(B.TuttiError) as ei:
        B.tutti_layer_restore_ordered(p, B.make_cfg(4096, 1 << 20, 4), FAKE, 1, FAKE, 8, FAKE, 9, FAKE, 1 << 20, 0, 0,
                                      FAKE, FAKE, FAKE, 4, FAKE, stream=0)      # layer 9 of 4
    assert ei.value.code == B.EINVAL


def test_workloads_are_seeded_and_shaped():
    from paper_2605_03375_amd import workloads as W
    a, b = W.batch64_zipf(), W.batch64_zipf()
    assert np.array_equal(a.block_table, b.block_table) and np.array_equal(a.n_blocks, b.n_blocks)
    assert a.n_req == 64 and len(set(a.block_table.tolist())) == a.block_table.size
    t = W.tiny()
    assert t.block_table.size == 32 and t.shape.num_blocks == 256
    w2 = W.llama8b_32k()
    assert w2.block_table.size == 2048 and w2.shape.num_blocks == 65536 and w2.shape.num_layers == 32
    w4 = W.llama70b_128k()
    assert w4.block_table.size == 8192 and w4.shape.num_blocks == 38146 and w4.shape.num_layers == 80
    assert len(set(w4.block_table.tolist())) == 8192 and int(w4.block_table.max()) < 38146
    v = W.host_values(1, 1000, "bf16")
    assert v.dtype == np.uint16 and np.array_equal(v, W.host_values(1, 1000, "bf16"))
