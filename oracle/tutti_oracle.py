"""ctypes wrapper of the CPU oracle (oracle/tutti_oracle.c).  TEST INFRASTRUCTURE ONLY.

Only tests, `__graft_entry__.smoke()` and `bench.py`'s cpu_baseline leg may import this.
It shares nothing with the HIP library or its binding: the records are declared here a
third time as numpy dtypes / ctypes structures, and a test checks all declarations agree.

Every array is a host numpy array.  K and V planes are uint8 arrays of
`num_blocks * block_stride` bytes (any dtype is viewed as bytes).
"""
import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB = None

LAYOUT_NHD, LAYOUT_HND = 0, 1
OP_READ, OP_WRITE = 1, 2
ST_BAD_BLOCK, ST_STAGE_CAP, ST_SQE_CAP, ST_DUP_BLOCK, ST_BAD_EXTENT = 1, 2, 4, 8, 16
IOCB_SLOTS = 2048

EXTENT_DTYPE = np.dtype([("stage_off", "<u8"), ("obj_bytes", "<u8"), ("n_blocks", "<u4"), ("n_chunks", "<u4"),
                         ("sqe_base", "<u4"), ("table_off", "<u4")], align=True)
SQE_DTYPE = np.dtype([("opcode", "u1"), ("kind", "u1"), ("layer", "<u2"), ("file_id", "<u4"), ("file_off", "<u8"),
                      ("addr", "<u8"), ("len", "<u4"), ("sgl_id", "<u4"), ("user_data", "<u8"), ("iocb_idx", "<u4"),
                      ("ioctx_slot", "<u4"), ("rsvd", "u1", (16,))], align=True)


SGL_DTYPE = np.dtype([("addr", "<u8"), ("len", "<u4"), ("id", "<u4")], align=True)


IOCB_FREE, IOCB_FILLED, IOCB_DONE = 0, 1, 2
IOCB_HDR_DTYPE = np.dtype([("iocb_idx", "<u4"), ("num_ioctx", "<u4"), ("state", "<u4"), ("done", "<u4"),
                           ("layer", "<u4"), ("opcode", "<u4"), ("rsvd", "<u4", (10,))], align=True)
IOCB_DTYPE = np.dtype([("hdr", IOCB_HDR_DTYPE), ("ioctx", SQE_DTYPE, (IOCB_SLOTS,))], align=True)
CQ_HDR_WORDS = 16  # tail, depth, 14 reserved; then depth entries


class OrcFileStore(C.Structure):
    _fields_ = [("base", C.c_void_p), ("file_stride", C.c_uint64), ("first_file_id", C.c_uint32),
                ("n_files", C.c_uint32)]


class OrcPool(C.Structure):
    _fields_ = [("k_base", C.c_void_p), ("v_base", C.c_void_p), ("block_stride", C.c_uint64),
                ("num_blocks", C.c_uint32), ("block_tokens", C.c_uint32), ("num_kv_heads", C.c_uint32),
                ("head_dim", C.c_uint32), ("elt_bytes", C.c_uint32), ("pool_layout", C.c_uint32)]


class OrcObjCfg(C.Structure):
    _fields_ = [("align", C.c_uint32), ("chunk_bytes", C.c_uint32), ("num_layers", C.c_uint32)]


class OracleError(RuntimeError):
    def __init__(self, fn, rc):
        super().__init__(f"{fn} returned {rc}")
        self.rc = rc


def lib():
    """Load the oracle library, building it with gcc first if it is not there."""
    global _LIB
    if _LIB is None:
        path = os.path.join(_HERE, "libtutti_oracle.so")
        if not os.path.exists(path):
            import importlib.util
            spec = importlib.util.spec_from_file_location("_oracle_build", os.path.join(_HERE, "build.py"))
            mod = importlib.util.module_from_spec(spec)
            spec.loader.exec_module(mod)
            mod.build_oracle()
        L = C.CDLL(path)
        L.orc_block_bytes.restype = C.c_uint32
        L.orc_desc_count.restype = C.c_uint64
        L.orc_desc_count.argtypes = [C.c_uint64, C.c_uint64]
        _LIB = L
    return _LIB


def _ptr(a):
    return C.c_void_p(a.ctypes.data if a is not None else 0)


def _bytes_view(a):
    a = np.ascontiguousarray(a)
    return a.view(np.uint8).reshape(-1)


def make_pool(k_plane, v_plane, *, num_blocks, block_tokens, num_kv_heads, head_dim, elt_bytes, block_stride=None,
              pool_layout=LAYOUT_NHD):
    """Describe one layer's pool.  k_plane / v_plane: writable contiguous host arrays (or None)."""
    bb = block_tokens * num_kv_heads * head_dim * elt_bytes
    p = OrcPool()
    p.k_base = k_plane.ctypes.data if k_plane is not None else 0
    p.v_base = v_plane.ctypes.data if v_plane is not None else 0
    p.block_stride = bb if block_stride is None else block_stride
    p.num_blocks, p.block_tokens, p.num_kv_heads = num_blocks, block_tokens, num_kv_heads
    p.head_dim, p.elt_bytes, p.pool_layout = head_dim, elt_bytes, pool_layout
    p._keep = (k_plane, v_plane)
    return p


def make_cfg(align=4096, chunk_bytes=2 << 20, num_layers=1):
    return OrcObjCfg(align, chunk_bytes, num_layers)


def abi_describe():
    out = np.zeros(64, np.uint32)
    n = lib().orc_abi_describe(_ptr(out), C.c_uint32(out.size))
    if n < 0:
        raise OracleError("orc_abi_describe", n)
    return out[:n].tolist()


def block_bytes(pool):
    return int(lib().orc_block_bytes(C.byref(pool)))


def desc_count(pool_bytes, gran):
    return int(lib().orc_desc_count(pool_bytes, gran))


def obj_layout(pool, cfg, n_blocks):
    n_blocks = np.ascontiguousarray(n_blocks, dtype=np.uint32)
    ext = np.zeros(n_blocks.size, EXTENT_DTYPE)
    totals = np.zeros(2, np.uint64)
    rc = lib().orc_obj_layout(C.byref(pool), C.byref(cfg), _ptr(n_blocks), C.c_uint32(n_blocks.size), _ptr(ext),
                              _ptr(totals))
    if rc:
        raise OracleError("orc_obj_layout", rc)
    return ext, totals


def obj_pack(pool, cfg, extents, block_table, stage, stage_cap=None, n_threads=0, table_len=None):
    """Pack into `stage` (uint8 host array, modified in place).  Returns the status word.
    table_len: how many entries of block_table may be read (default: all of them)."""
    block_table = np.ascontiguousarray(block_table, dtype=np.uint32)
    extents = np.ascontiguousarray(extents)
    cap = stage.nbytes if stage_cap is None else stage_cap
    tl = block_table.size if table_len is None else table_len
    assert tl <= block_table.size
    status = C.c_uint32(0)
    if n_threads:
        rc = lib().orc_obj_pack_mt(C.byref(pool), C.byref(cfg), _ptr(extents), C.c_uint32(extents.size),
                                   _ptr(block_table), C.c_uint32(tl), _ptr(stage), C.c_uint64(cap),
                                   C.c_uint32(n_threads))
    else:
        rc = lib().orc_obj_pack(C.byref(pool), C.byref(cfg), _ptr(extents), C.c_uint32(extents.size),
                                _ptr(block_table), C.c_uint32(tl), _ptr(stage), C.c_uint64(cap), C.byref(status))
    if rc:
        raise OracleError("orc_obj_pack", rc)
    return status.value


def obj_unpack(pool, cfg, extents, block_table, stage, stage_cap=None, n_threads=0, table_len=None):
    """Unpack `stage` into the planes the pool points at.  Returns the status word."""
    block_table = np.ascontiguousarray(block_table, dtype=np.uint32)
    extents = np.ascontiguousarray(extents)
    cap = stage.nbytes if stage_cap is None else stage_cap
    tl = block_table.size if table_len is None else table_len
    assert tl <= block_table.size
    status = C.c_uint32(0)
    if n_threads:
        rc = lib().orc_obj_unpack_mt(C.byref(pool), C.byref(cfg), _ptr(extents), C.c_uint32(extents.size),
                                     _ptr(block_table), C.c_uint32(tl), _ptr(stage), C.c_uint64(cap),
                                     C.c_uint32(n_threads))
    else:
        rc = lib().orc_obj_unpack(C.byref(pool), C.byref(cfg), _ptr(extents), C.c_uint32(extents.size),
                                  _ptr(block_table), C.c_uint32(tl), _ptr(stage), C.c_uint64(cap), C.byref(status))
    if rc:
        raise OracleError("orc_obj_unpack", rc)
    return status.value


def sqe_build(pool, cfg, extents, file_id, layer, opcode, stage_addr, sgl_id, sqe_cap=None):
    """Returns (sqe array of sqe_cap entries, status).  Default capacity: exactly what the extents need."""
    file_id = np.ascontiguousarray(file_id, dtype=np.uint32)
    need = int(2 * extents["n_chunks"].astype(np.uint64).sum())
    cap = need if sqe_cap is None else sqe_cap
    sqe = np.zeros(cap, SQE_DTYPE)
    status = C.c_uint32(0)
    rc = lib().orc_sqe_build(C.byref(pool), C.byref(cfg), _ptr(extents), C.c_uint32(extents.size), _ptr(file_id),
                             C.c_uint32(layer), C.c_uint32(opcode), C.c_uint64(stage_addr), C.c_uint32(sgl_id),
                             _ptr(sqe), C.c_uint32(cap), C.byref(status))
    if rc:
        raise OracleError("orc_sqe_build", rc)
    return sqe, status.value


def layer_restore(pool, cfg, n_blocks, block_table, file_id, layer, stage, stage_addr, sgl_id, sqe_cap,
                  stage_cap=None, table_len=None):
    """Returns (extents, totals, sqe, status); the planes the pool points at are modified in place."""
    n_blocks = np.ascontiguousarray(n_blocks, dtype=np.uint32)
    block_table = np.ascontiguousarray(block_table, dtype=np.uint32)
    file_id = np.ascontiguousarray(file_id, dtype=np.uint32)
    ext = np.zeros(n_blocks.size, EXTENT_DTYPE)
    totals = np.zeros(2, np.uint64)
    sqe = np.zeros(sqe_cap, SQE_DTYPE)
    cap = stage.nbytes if stage_cap is None else stage_cap
    status = C.c_uint32(0)
    tl = block_table.size if table_len is None else table_len
    assert tl <= block_table.size
    rc = lib().orc_layer_restore(C.byref(pool), C.byref(cfg), _ptr(n_blocks), C.c_uint32(n_blocks.size),
                                 _ptr(block_table), C.c_uint32(tl), _ptr(file_id), C.c_uint32(layer), _ptr(stage),
                                 C.c_uint64(cap),
                                 C.c_uint64(stage_addr), C.c_uint32(sgl_id), _ptr(ext), _ptr(totals), _ptr(sqe),
                                 C.c_uint32(sqe_cap), C.byref(status))
    if rc:
        raise OracleError("orc_layer_restore", rc)
    return ext, totals, sqe, status.value


def sgl_table_build(pool, k_addr, v_addr, sgl_id, cap=None):
    """Returns (descriptor array, status).  Default capacity: 2 * num_blocks."""
    n = 2 * pool.num_blocks if cap is None else cap
    table = np.zeros(n, SGL_DTYPE)
    status = C.c_uint32(0)
    rc = lib().orc_sgl_table_build(C.byref(pool), C.c_uint64(k_addr), C.c_uint64(v_addr), C.c_uint32(sgl_id),
                                   _ptr(table), C.c_uint32(n), C.byref(status))
    if rc:
        raise OracleError("orc_sgl_table_build", rc)
    return table, status.value


def sqe_build_direct(pool, cfg, extents, block_table, file_id, layer, opcode, sgl_table_addr, sgl_id, sqe_cap=None):
    """Returns (sqe array, status).  Default capacity: 2 * sum(n_blocks)."""
    block_table = np.ascontiguousarray(block_table, dtype=np.uint32)
    file_id = np.ascontiguousarray(file_id, dtype=np.uint32)
    need = int(2 * extents["n_blocks"].astype(np.uint64).sum())
    cap = need if sqe_cap is None else sqe_cap
    sqe = np.zeros(cap, SQE_DTYPE)
    status = C.c_uint32(0)
    rc = lib().orc_sqe_build_direct(C.byref(pool), C.byref(cfg), _ptr(extents), C.c_uint32(extents.size),
                                    _ptr(block_table), _ptr(file_id), C.c_uint32(layer), C.c_uint32(opcode),
                                    C.c_uint64(sgl_table_addr), C.c_uint32(sgl_id), _ptr(sqe), C.c_uint32(cap),
                                    C.byref(status))
    if rc:
        raise OracleError("orc_sqe_build_direct", rc)
    return sqe, status.value


def ring_alloc(depth):
    """Host memory for an SQ of `depth` IOCBs and its CQ (uint32 words: 16 header words + depth entries)."""
    return np.zeros(depth, IOCB_DTYPE), np.zeros(CQ_HDR_WORDS + depth, np.uint32)


def ring_init(sq, cq):
    rc = lib().orc_ring_init(_ptr(sq), _ptr(cq), C.c_uint32(sq.size))
    if rc:
        raise OracleError("orc_ring_init", rc)


def iocb_fill_direct(sq, first_slot, n_slots, pool, cfg, extents, block_table, file_id, layer, opcode,
                     sgl_table_addr, sgl_id):
    block_table = np.ascontiguousarray(block_table, dtype=np.uint32)
    file_id = np.ascontiguousarray(file_id, dtype=np.uint32)
    status = C.c_uint32(0)
    rc = lib().orc_iocb_fill_direct(_ptr(sq), C.c_uint32(sq.size), C.c_uint32(first_slot), C.c_uint32(n_slots),
                                    C.byref(pool), C.byref(cfg), _ptr(extents), C.c_uint32(extents.size),
                                    _ptr(block_table), _ptr(file_id), C.c_uint32(layer), C.c_uint32(opcode),
                                    C.c_uint64(sgl_table_addr), C.c_uint32(sgl_id), C.byref(status))
    if rc:
        raise OracleError("orc_iocb_fill_direct", rc)
    return status.value


def issue_io(sq, cq, first_slot, n_slots, sgl_table, sgl_table_addr, store, file_stride, first_file_id, n_files,
             max_len=None):
    """`store`: uint8 host array of n_files * file_stride bytes.  max_len: longest context allowed (default: the
    longest descriptor of the table).  Returns the status word."""
    fs = OrcFileStore(store.ctypes.data, file_stride, first_file_id, n_files)
    status = C.c_uint32(0)
    if max_len is None:
        max_len = int(sgl_table["len"].max()) if sgl_table.size else 16
    rc = lib().orc_issue_io(_ptr(sq), _ptr(cq), C.c_uint32(sq.size), C.c_uint32(first_slot), C.c_uint32(n_slots),
                            _ptr(sgl_table), C.c_uint32(sgl_table.size), C.c_uint64(sgl_table_addr), C.byref(fs),
                            C.c_uint32(max_len), C.byref(status))
    if rc:
        raise OracleError("orc_issue_io", rc)
    return status.value


def _ring_layer(fn, sq, cq, first_slot, n_slots, pool, cfg, n_blocks, block_table, file_id, layer, sgl_table_addr,
                sgl_id, store, file_stride, first_file_id, n_files):
    n_blocks = np.ascontiguousarray(n_blocks, dtype=np.uint32)
    block_table = np.ascontiguousarray(block_table, dtype=np.uint32)
    file_id = np.ascontiguousarray(file_id, dtype=np.uint32)
    ext = np.zeros(n_blocks.size, EXTENT_DTYPE)
    totals = np.zeros(2, np.uint64)
    fs = OrcFileStore(store.ctypes.data, file_stride, first_file_id, n_files)
    status = C.c_uint32(0)
    rc = getattr(lib(), fn)(_ptr(sq), _ptr(cq), C.c_uint32(sq.size), C.c_uint32(first_slot), C.c_uint32(n_slots),
                            C.byref(pool), C.byref(cfg), _ptr(n_blocks), C.c_uint32(n_blocks.size), _ptr(block_table),
                            _ptr(file_id), C.c_uint32(layer), C.c_uint64(sgl_table_addr), C.c_uint32(sgl_id),
                            C.byref(fs), _ptr(ext), _ptr(totals), C.byref(status))
    if rc:
        raise OracleError(fn, rc)
    return ext, totals, status.value


def retrieve_layer(sq, cq, first_slot, n_slots, pool, cfg, n_blocks, block_table, file_id, layer, sgl_table_addr,
                   sgl_id, store, file_stride, first_file_id, n_files):
    """File store -> pool blocks through the rings.  Returns (extents, totals, status); pool, sq, cq change in place."""
    return _ring_layer("orc_retrieve_layer", sq, cq, first_slot, n_slots, pool, cfg, n_blocks, block_table, file_id,
                       layer, sgl_table_addr, sgl_id, store, file_stride, first_file_id, n_files)


def store_layer(sq, cq, first_slot, n_slots, pool, cfg, n_blocks, block_table, file_id, layer, sgl_table_addr,
                sgl_id, store, file_stride, first_file_id, n_files):
    """Pool blocks -> file store through the rings.  Returns (extents, totals, status); store, sq, cq change in place."""
    return _ring_layer("orc_store_layer", sq, cq, first_slot, n_slots, pool, cfg, n_blocks, block_table, file_id,
                       layer, sgl_table_addr, sgl_id, store, file_stride, first_file_id, n_files)


def table_validate(num_blocks, block_table):
    """Status bits for a table: ST_BAD_BLOCK for ids out of range, ST_DUP_BLOCK for an id that appears twice."""
    block_table = np.ascontiguousarray(block_table, dtype=np.uint32)
    status = C.c_uint32(0)
    rc = lib().orc_table_validate(C.c_uint32(num_blocks), _ptr(block_table), C.c_uint32(block_table.size),
                                  C.byref(status))
    if rc:
        raise OracleError("orc_table_validate", rc)
    return status.value


def layer_save(pool, cfg, n_blocks, block_table, file_id, layer, stage, stage_addr, sgl_id, sqe_cap, stage_cap=None,
               table_len=None):
    """Returns (extents, totals, sqe, status); `stage` is written in place."""
    n_blocks = np.ascontiguousarray(n_blocks, dtype=np.uint32)
    block_table = np.ascontiguousarray(block_table, dtype=np.uint32)
    file_id = np.ascontiguousarray(file_id, dtype=np.uint32)
    ext = np.zeros(n_blocks.size, EXTENT_DTYPE)
    totals = np.zeros(2, np.uint64)
    sqe = np.zeros(sqe_cap, SQE_DTYPE)
    cap = stage.nbytes if stage_cap is None else stage_cap
    status = C.c_uint32(0)
    tl = block_table.size if table_len is None else table_len
    assert tl <= block_table.size
    rc = lib().orc_layer_save(C.byref(pool), C.byref(cfg), _ptr(n_blocks), C.c_uint32(n_blocks.size),
                              _ptr(block_table), C.c_uint32(tl), _ptr(file_id), C.c_uint32(layer), _ptr(stage),
                              C.c_uint64(cap),
                              C.c_uint64(stage_addr), C.c_uint32(sgl_id), _ptr(ext), _ptr(totals), _ptr(sqe),
                              C.c_uint32(sqe_cap), C.byref(status))
    if rc:
        raise OracleError("orc_layer_save", rc)
    return ext, totals, sqe, status.value


def table_order(num_blocks, block_table):
    """Returns (visit, status): table positions in ascending order of block id; identity + status bits for a table
    that table_validate objects to."""
    block_table = np.ascontiguousarray(block_table, dtype=np.uint32)
    visit = np.zeros(block_table.size, np.uint32)
    status = C.c_uint32(0)
    rc = lib().orc_table_order(C.c_uint32(num_blocks), _ptr(block_table), C.c_uint32(block_table.size), _ptr(visit),
                               C.byref(status))
    if rc:
        raise OracleError("orc_table_order", rc)
    return visit, status.value


def layer_restore_ordered(pool, cfg, n_blocks, block_table, file_id, layer, stage, stage_addr, sgl_id, sqe_cap, visit,
                          stage_cap=None, table_len=None):
    """layer_restore with the blocks visited in the order `visit` lists (table positions)."""
    n_blocks = np.ascontiguousarray(n_blocks, dtype=np.uint32)
    block_table = np.ascontiguousarray(block_table, dtype=np.uint32)
    file_id = np.ascontiguousarray(file_id, dtype=np.uint32)
    visit = np.ascontiguousarray(visit, dtype=np.uint32)
    ext = np.zeros(n_blocks.size, EXTENT_DTYPE)
    totals = np.zeros(2, np.uint64)
    sqe = np.zeros(sqe_cap, SQE_DTYPE)
    cap = stage.nbytes if stage_cap is None else stage_cap
    tl = block_table.size if table_len is None else table_len
    assert tl <= block_table.size and tl <= visit.size
    status = C.c_uint32(0)
    rc = lib().orc_layer_restore_ordered(C.byref(pool), C.byref(cfg), _ptr(n_blocks), C.c_uint32(n_blocks.size),
                                         _ptr(block_table), C.c_uint32(tl), _ptr(file_id), C.c_uint32(layer),
                                         _ptr(stage), C.c_uint64(cap), C.c_uint64(stage_addr), C.c_uint32(sgl_id),
                                         _ptr(ext), _ptr(totals), _ptr(sqe), C.c_uint32(sqe_cap), _ptr(visit),
                                         C.byref(status))
    if rc:
        raise OracleError("orc_layer_restore_ordered", rc)
    return ext, totals, sqe, status.value
