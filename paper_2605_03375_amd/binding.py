"""ctypes binding of libtutti (include/tutti.h): argument marshalling only.

Every function has the name and argument order of its C entry point; device pointers may be
given as torch tensors (their data_ptr() is taken) or as integers.  `stream=None` means
torch's current stream.  A non-zero return code raises TuttiError.  There is no fallback:
if the HIP library has not been built, `lib()` raises.

Two libraries are built from the same sources: libtutti.so, the product, and libtutti_bench.so, which
exports the same entry points plus the measurement aids of include/tutti_bench.h (baseline kernels, tuning
knobs, every launch shape).  The wrappers of the measurement aids always call the latter;
`use_bench_library(True)` also routes the ordinary entry points through it, so that an experiment can run the
product's kernels in another launch shape.  Nothing but bench.py and the tests of those aids does that.
"""
import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libtutti.so")
BENCH_LIB_PATH = os.path.join(_HERE, "libtutti_bench.so")
_LIB = None
_BENCH_LIB = None
_USE_BENCH = False

OK, EINVAL, ERANGE, EHIP, EAGAIN = 0, -1, -2, -3, -4
LAYOUT_NHD, LAYOUT_HND = 0, 1
OP_READ, OP_WRITE = 1, 2
STREAM_SLOTS = 4096
IOCB_SLOTS = 2048
MAX_REQ = 2048
ST_BAD_BLOCK, ST_STAGE_CAP, ST_SQE_CAP, ST_DUP_BLOCK, ST_BAD_EXTENT = 1, 2, 4, 8, 16

# Declarations of the C records for decoding results on the host.
EXTENT_DTYPE = np.dtype({"names": ["stage_off", "obj_bytes", "n_blocks", "n_chunks", "sqe_base", "table_off"],
                         "formats": ["<u8", "<u8", "<u4", "<u4", "<u4", "<u4"],
                         "offsets": [0, 8, 16, 20, 24, 28], "itemsize": 32})
SQE_DTYPE = np.dtype({"names": ["opcode", "kind", "layer", "file_id", "file_off", "addr", "len", "sgl_id",
                                "user_data", "iocb_idx", "ioctx_slot", "rsvd"],
                      "formats": ["u1", "u1", "<u2", "<u4", "<u8", "<u8", "<u4", "<u4", "<u8", "<u4", "<u4",
                                  ("u1", (16,))],
                      "offsets": [0, 1, 2, 4, 8, 16, 24, 28, 32, 40, 44, 48], "itemsize": 64})

SGL_DTYPE = np.dtype({"names": ["addr", "len", "id"], "formats": ["<u8", "<u4", "<u4"], "offsets": [0, 8, 12],
                      "itemsize": 16})

EXPORTS = ["tutti_obj_layout", "tutti_obj_pack", "tutti_obj_unpack", "tutti_sqe_build", "tutti_layer_restore",
           "tutti_layer_save", "tutti_sgl_table_build", "tutti_sqe_build_direct", "tutti_ring_init",
           "tutti_iocb_fill_direct", "tutti_issue_io", "tutti_wait_cqe", "tutti_retrieve_layer", "tutti_store_layer",
           "tutti_table_validate", "tutti_strerror", "tutti_last_hip_error", "tutti_cu_count",
           "tutti_resident_wgs_per_cu", "tutti_version", "tutti_abi_describe",
           "tutti_sq_state_init", "tutti_get_iocb", "tutti_sq_free_count", "tutti_reap_cqe", "tutti_iocb_completed",
           "tutti_wait_cqe_host", "tutti_iocbs_for_slack", "tutti_budget_for_slack", "tutti_io_domain_create",
           "tutti_io_domain_destroy", "tutti_table_validate_work_bytes", "tutti_table_validate_ws",
           "tutti_table_validate_static", "tutti_layer_restore_ordered", "tutti_table_order",
           "tutti_table_order_work_bytes", "tutti_retrieve_layer_issue", "tutti_store_layer_issue",
           "tutti_complete_io", "tutti_wait_cqe_range", "tutti_place_work_bytes", "tutti_place_pair_times",
           "tutti_place_classify", "tutti_place_pairs", "tutti_retrieve_layer_chained",
           "tutti_store_layer_chained", "tutti_issue_io_chained"]
BENCH_EXPORTS = ["tutti_copy_baseline", "tutti_stream_baseline", "tutti_scatter_baseline", "tutti_set_tuning",
                 "tutti_set_nontemporal", "tutti_set_hnd_mode", "tutti_set_xcd_mapping",
                 "tutti_host_cost_of_restore"]   # include/tutti_bench.h
SCATTER_SHAPES = {"wave_slice": 0, "wave_slice_1024": 1, "wave_piece": 2, "wg_piece": 3, "wg_piece_plain": 4,
                  "wg_piece_nt_loads": 5, "wg_piece_nt_stores": 6}


class tutti_pool(C.Structure):
    _fields_ = [("k_base", C.c_void_p), ("v_base", C.c_void_p), ("block_stride", C.c_uint64),
                ("num_blocks", C.c_uint32), ("block_tokens", C.c_uint32), ("num_kv_heads", C.c_uint32),
                ("head_dim", C.c_uint32), ("elt_bytes", C.c_uint32), ("pool_layout", C.c_uint32)]


class tutti_objcfg(C.Structure):
    _fields_ = [("align", C.c_uint32), ("chunk_bytes", C.c_uint32), ("num_layers", C.c_uint32)]


class tutti_ring(C.Structure):
    _fields_ = [("d_sq", C.c_void_p), ("d_cq", C.c_void_p), ("depth", C.c_uint32)]


class tutti_filestore(C.Structure):
    _fields_ = [("base", C.c_void_p), ("file_stride", C.c_uint64), ("first_file_id", C.c_uint32),
                ("n_files", C.c_uint32)]


class tutti_sq_state(C.Structure):
    _fields_ = [("depth", C.c_uint32), ("head", C.c_uint32), ("held", C.c_uint32), ("cq_seen", C.c_uint32),
                ("done", C.c_void_p)]


class tutti_place_round(C.Structure):
    _fields_ = [("reference", C.c_uint32), ("members", C.c_uint32), ("same_region_us", C.c_float),
                ("fastest_us", C.c_float)]


PLACE_MIN_PLANE_BYTES = 128 << 20
PLACE_MAX_REGIONS = 8


class tutti_io_profile(C.Structure):
    _fields_ = [("cu_budget", C.c_uint32), ("n_iocbs", C.c_uint32), ("read_us", C.c_float), ("write_us", C.c_float)]


IOCB_FREE, IOCB_FILLED, IOCB_DONE = 0, 1, 2
IOCB_HDR_DTYPE = np.dtype({"names": ["iocb_idx", "num_ioctx", "state", "done", "layer", "opcode"],
                           "formats": ["<u4"] * 6, "offsets": [0, 4, 8, 12, 16, 20], "itemsize": 64})
IOCB_DTYPE = np.dtype({"names": ["hdr", "ioctx"], "formats": [IOCB_HDR_DTYPE, (SQE_DTYPE, (IOCB_SLOTS,))],
                       "offsets": [0, 64], "itemsize": 64 + 64 * IOCB_SLOTS})
IOCB_BYTES = IOCB_DTYPE.itemsize
CQ_HDR_BYTES = 64


def ring_bytes(depth):
    """Bytes of device memory for an SQ and a CQ of `depth` IOCBs."""
    return depth * IOCB_BYTES, CQ_HDR_BYTES + 4 * depth


def make_ring(d_sq, d_cq, depth):
    r = tutti_ring(_p(d_sq), _p(d_cq), depth)
    r._keep = (d_sq, d_cq)
    return r


def make_filestore(base, file_stride, first_file_id, n_files):
    f = tutti_filestore(_p(base), file_stride, first_file_id, n_files)
    f._keep = base
    return f


class TuttiError(RuntimeError):
    def __init__(self, fn, code):
        self.fn, self.code = fn, code
        msg = lib().tutti_strerror(code).decode()
        hip = lib().tutti_last_hip_error() if code == EHIP else 0
        super().__init__(f"{fn}: {msg} (code {code}" + (f", hipError {hip})" if hip else ")"))


def _declare(L, bench):
    vp, u32, u64 = C.c_void_p, C.c_uint32, C.c_uint64
    pp, pc = C.POINTER(tutti_pool), C.POINTER(tutti_objcfg)
    L.tutti_obj_layout.argtypes = [pp, pc, vp, u32, vp, vp, vp]
    L.tutti_obj_pack.argtypes = [pp, pc, vp, u32, vp, u32, vp, u64, u32, vp, vp]
    L.tutti_obj_unpack.argtypes = [pp, pc, vp, u32, vp, u32, vp, u64, u32, vp, vp]
    L.tutti_sqe_build.argtypes = [pp, pc, vp, u32, vp, u32, u32, u64, u32, vp, u32, vp, vp]
    L.tutti_layer_restore.argtypes = [pp, pc, vp, u32, vp, u32, vp, u32, vp, u64, u64, u32, vp, vp, vp, u32, u32,
                                      vp, vp]
    L.tutti_layer_save.argtypes = L.tutti_layer_restore.argtypes
    L.tutti_layer_restore_ordered.argtypes = [pp, pc, vp, u32, vp, u32, vp, u32, vp, u64, u64, u32, vp, vp, vp, u32,
                                              u32, vp, vp, vp]
    L.tutti_table_order.argtypes = [u32, vp, u32, vp, vp, u64, vp, vp]
    L.tutti_table_order_work_bytes.argtypes = [u32]
    L.tutti_table_order_work_bytes.restype = u64
    L.tutti_table_validate.argtypes = [u32, vp, u32, vp, vp]
    L.tutti_table_validate_ws.argtypes = [u32, vp, u32, vp, vp, u64, vp]
    L.tutti_table_validate_static.argtypes = [u32, vp, u32, vp, vp]
    L.tutti_table_validate_work_bytes.argtypes = [u32]
    L.tutti_table_validate_work_bytes.restype = u64
    pr, pf = C.POINTER(tutti_ring), C.POINTER(tutti_filestore)
    L.tutti_ring_init.argtypes = [pr, vp]
    L.tutti_iocb_fill_direct.argtypes = [pr, u32, u32, pp, pc, vp, u32, vp, u32, vp, u32, u32, u64, u32, vp, vp]
    L.tutti_issue_io.argtypes = [pr, u32, u32, vp, u32, u64, pf, u32, u32, vp, vp]
    L.tutti_issue_io_chained.argtypes = [pr, u32, u32, u32, u32, vp, u32, u64, pf, u32, u32, vp, vp]
    L.tutti_wait_cqe.argtypes = [pr, u32, vp, vp]
    L.tutti_wait_cqe_range.argtypes = [pr, u32, u32, vp, vp]
    L.tutti_retrieve_layer.argtypes = [pr, u32, u32, pp, pc, vp, u32, vp, u32, vp, u32, u64, u32, pf, vp, vp, u32,
                                       vp, vp]
    L.tutti_store_layer.argtypes = L.tutti_retrieve_layer.argtypes
    L.tutti_retrieve_layer_issue.argtypes = L.tutti_retrieve_layer.argtypes
    L.tutti_store_layer_issue.argtypes = L.tutti_retrieve_layer.argtypes
    L.tutti_complete_io.argtypes = [pr, u32, u32, vp]
    L.tutti_retrieve_layer_chained.argtypes = [pr, u32, u32, u32, u32] + L.tutti_retrieve_layer.argtypes[3:]
    L.tutti_store_layer_chained.argtypes = L.tutti_retrieve_layer_chained.argtypes
    L.tutti_sgl_table_build.argtypes = [pp, u64, u64, u32, vp, u32, vp, vp]
    L.tutti_sqe_build_direct.argtypes = [pp, pc, vp, u32, vp, u32, vp, u32, u32, u64, u32, vp, u32, vp, vp]
    L.tutti_strerror.argtypes = [C.c_int]
    L.tutti_strerror.restype = C.c_char_p
    L.tutti_version.restype = u32
    L.tutti_abi_describe.argtypes = [vp, u32]
    L.tutti_resident_wgs_per_cu.argtypes = [u32]
    L.tutti_io_domain_create.argtypes = [u32, C.POINTER(vp)]
    L.tutti_io_domain_destroy.argtypes = [vp]
    ps, pio = C.POINTER(tutti_sq_state), C.POINTER(tutti_io_profile)
    L.tutti_sq_state_init.argtypes = [ps, u32, vp]
    L.tutti_get_iocb.argtypes = [ps, u32, C.POINTER(u32)]
    L.tutti_sq_free_count.argtypes = [ps]
    L.tutti_sq_free_count.restype = u32
    L.tutti_reap_cqe.argtypes = [ps, vp, vp, C.POINTER(u32)]
    L.tutti_iocb_completed.argtypes = [ps, u32]
    L.tutti_wait_cqe_host.argtypes = [ps, vp, vp, u32, u32]
    L.tutti_iocbs_for_slack.argtypes = [pio, u32, u32, u32, C.c_double, C.POINTER(u32)]
    L.tutti_budget_for_slack.argtypes = [pio, u32, u32, u32, C.c_double, u32, C.POINTER(u32)]
    L.tutti_place_work_bytes.argtypes = []
    L.tutti_place_work_bytes.restype = u64
    L.tutti_place_pair_times.argtypes = [vp, C.POINTER(vp), u32, u64, vp, u64, u32, C.POINTER(C.c_float), vp]
    L.tutti_place_classify.argtypes = [C.POINTER(vp), u32, u64, vp, u64, u32, C.c_double, C.POINTER(C.c_int32),
                                       C.POINTER(tutti_place_round), C.POINTER(u32), vp]
    L.tutti_place_pairs.argtypes = [C.POINTER(C.c_int32), u32, u32, u32, C.POINTER(u32), C.POINTER(u32)]
    for name in EXPORTS:
        if name not in ("tutti_strerror", "tutti_version", "tutti_sq_free_count", "tutti_table_validate_work_bytes",
                        "tutti_table_order_work_bytes", "tutti_place_work_bytes"):
            getattr(L, name).restype = C.c_int
    if bench:
        L.tutti_copy_baseline.argtypes = [vp, vp, u64, u32, vp]
        L.tutti_stream_baseline.argtypes = [vp, u64, u32, vp, u32, vp]
        L.tutti_scatter_baseline.argtypes = [vp, u64, vp, u64, vp, u32, u32, u32, u32, vp]
        L.tutti_set_tuning.argtypes = [u32, u32]
        L.tutti_set_nontemporal.argtypes = [u32]
        L.tutti_set_hnd_mode.argtypes = [u32]
        L.tutti_set_xcd_mapping.argtypes = [u32]
        L.tutti_host_cost_of_restore.argtypes = L.tutti_layer_restore.argtypes + [u32, C.POINTER(C.c_double)]
        for name in BENCH_EXPORTS:
            getattr(L, name).restype = C.c_int
    return L


def _load(path, bench):
    if not os.path.exists(path):
        raise RuntimeError(f"{path} is missing: build it with `python -m paper_2605_03375_amd.build` "
                           "(or __graft_entry__.build()); libtutti has no CPU fallback")
    # PyTorch ships its own HIP runtime (same soname as the system one).  Import it first so
    # that libtutti binds to the runtime that owns the process's device context and streams;
    # two HIP runtimes in one process do not share a device.
    import torch  # noqa: F401
    return _declare(C.CDLL(path), bench)


def product_lib():
    """libtutti.so.  Raises if it has not been built: there is no other path."""
    global _LIB
    if _LIB is None:
        _LIB = _load(LIB_PATH, False)
    return _LIB


def bench_lib():
    """libtutti_bench.so: the same entry points plus the measurement aids."""
    global _BENCH_LIB
    if _BENCH_LIB is None:
        _BENCH_LIB = _load(BENCH_LIB_PATH, True)
    return _BENCH_LIB


def use_bench_library(on=True):
    """Route the ordinary entry points through libtutti_bench.so (experiments with the tuning knobs) or back."""
    global _USE_BENCH
    _USE_BENCH = bool(on)


def lib():
    """The library the ordinary wrappers call: the product, unless use_bench_library(True) was called."""
    return bench_lib() if _USE_BENCH else product_lib()


def _p(x):
    """Device (or host) pointer of a tensor / array / int / None, as c_void_p."""
    if x is None:
        return C.c_void_p(0)
    if hasattr(x, "data_ptr"):
        return C.c_void_p(x.data_ptr())
    if isinstance(x, np.ndarray):
        return C.c_void_p(x.ctypes.data)
    return C.c_void_p(int(x))


def _stream(stream):
    if stream is None:
        import torch
        return C.c_void_p(torch.cuda.current_stream().cuda_stream)
    if hasattr(stream, "cuda_stream"):
        return C.c_void_p(stream.cuda_stream)
    return C.c_void_p(int(stream))


def _check(fn, rc):
    if rc != OK:
        raise TuttiError(fn, rc)
    return rc


def make_pool(k_base, v_base, *, num_blocks, block_tokens, num_kv_heads, head_dim, elt_bytes, block_stride=None,
              pool_layout=LAYOUT_NHD):
    p = tutti_pool()
    p.k_base, p.v_base = _p(k_base), _p(v_base)
    p.block_stride = (block_tokens * num_kv_heads * head_dim * elt_bytes) if block_stride is None else block_stride
    p.num_blocks, p.block_tokens, p.num_kv_heads = num_blocks, block_tokens, num_kv_heads
    p.head_dim, p.elt_bytes, p.pool_layout = head_dim, elt_bytes, pool_layout
    p._keep = (k_base, v_base)
    return p


def make_cfg(align=4096, chunk_bytes=2 << 20, num_layers=1):
    return tutti_objcfg(align, chunk_bytes, num_layers)


def tutti_obj_layout(pool, cfg, d_n_blocks, n_req, d_extents, d_totals, stream=None):
    return _check("tutti_obj_layout", lib().tutti_obj_layout(C.byref(pool), C.byref(cfg), _p(d_n_blocks), n_req,
                                                             _p(d_extents), _p(d_totals), _stream(stream)))


def tutti_obj_pack(pool, cfg, d_extents, n_req, d_block_table, table_len, d_stage, stage_cap, cu_budget=0,
                   d_status=None, stream=None):
    return _check("tutti_obj_pack", lib().tutti_obj_pack(C.byref(pool), C.byref(cfg), _p(d_extents), n_req,
                                                         _p(d_block_table), table_len, _p(d_stage), stage_cap,
                                                         cu_budget, _p(d_status), _stream(stream)))


def tutti_obj_unpack(pool, cfg, d_extents, n_req, d_block_table, table_len, d_stage, stage_cap, cu_budget=0,
                     d_status=None, stream=None):
    return _check("tutti_obj_unpack", lib().tutti_obj_unpack(C.byref(pool), C.byref(cfg), _p(d_extents), n_req,
                                                             _p(d_block_table), table_len, _p(d_stage), stage_cap,
                                                             cu_budget, _p(d_status), _stream(stream)))


def tutti_sqe_build(pool, cfg, d_extents, n_req, d_file_id, layer, opcode, stage_addr, sgl_id, d_sqe, sqe_cap,
                    d_status=None, stream=None):
    return _check("tutti_sqe_build", lib().tutti_sqe_build(C.byref(pool), C.byref(cfg), _p(d_extents), n_req,
                                                           _p(d_file_id), layer, opcode, stage_addr, sgl_id,
                                                           _p(d_sqe), sqe_cap, _p(d_status), _stream(stream)))


def tutti_layer_restore(pool, cfg, d_n_blocks, n_req, d_block_table, table_len, d_file_id, layer, d_stage,
                        stage_cap, stage_addr, sgl_id, d_extents, d_totals, d_sqe, sqe_cap, cu_budget=0,
                        d_status=None, stream=None):
    return _check("tutti_layer_restore",
                  lib().tutti_layer_restore(C.byref(pool), C.byref(cfg), _p(d_n_blocks), n_req, _p(d_block_table),
                                            table_len, _p(d_file_id), layer, _p(d_stage), stage_cap, stage_addr,
                                            sgl_id, _p(d_extents), _p(d_totals), _p(d_sqe), sqe_cap, cu_budget,
                                            _p(d_status), _stream(stream)))


def tutti_layer_restore_ordered(pool, cfg, d_n_blocks, n_req, d_block_table, table_len, d_file_id, layer, d_stage,
                                stage_cap, stage_addr, sgl_id, d_extents, d_totals, d_sqe, sqe_cap, d_visit,
                                cu_budget=0, d_status=None, stream=None):
    return _check("tutti_layer_restore_ordered",
                  lib().tutti_layer_restore_ordered(C.byref(pool), C.byref(cfg), _p(d_n_blocks), n_req,
                                                    _p(d_block_table), table_len, _p(d_file_id), layer, _p(d_stage),
                                                    stage_cap, stage_addr, sgl_id, _p(d_extents), _p(d_totals),
                                                    _p(d_sqe), sqe_cap, cu_budget, _p(d_visit), _p(d_status),
                                                    _stream(stream)))


def tutti_table_order_work_bytes(num_blocks):
    return int(lib().tutti_table_order_work_bytes(num_blocks))


def tutti_table_order(num_blocks, d_block_table, table_len, d_visit, d_work, work_bytes, d_status=None, stream=None):
    return _check("tutti_table_order", lib().tutti_table_order(num_blocks, _p(d_block_table), table_len, _p(d_visit),
                                                               _p(d_work), work_bytes, _p(d_status), _stream(stream)))


def tutti_sgl_table_build(pool, k_addr, v_addr, sgl_id, d_table, cap, d_status=None, stream=None):
    return _check("tutti_sgl_table_build", lib().tutti_sgl_table_build(C.byref(pool), k_addr, v_addr, sgl_id,
                                                                       _p(d_table), cap, _p(d_status),
                                                                       _stream(stream)))


def tutti_sqe_build_direct(pool, cfg, d_extents, n_req, d_block_table, table_len, d_file_id, layer, opcode,
                           sgl_table_addr, sgl_id, d_sqe, sqe_cap, d_status=None, stream=None):
    return _check("tutti_sqe_build_direct",
                  lib().tutti_sqe_build_direct(C.byref(pool), C.byref(cfg), _p(d_extents), n_req, _p(d_block_table),
                                               table_len, _p(d_file_id), layer, opcode, sgl_table_addr, sgl_id,
                                               _p(d_sqe), sqe_cap, _p(d_status), _stream(stream)))


def tutti_ring_init(ring, stream=None):
    return _check("tutti_ring_init", lib().tutti_ring_init(C.byref(ring), _stream(stream)))


def tutti_iocb_fill_direct(ring, first_slot, n_slots, pool, cfg, d_extents, n_req, d_block_table, table_len,
                           d_file_id, layer, opcode, sgl_table_addr, sgl_id, d_status=None, stream=None):
    return _check("tutti_iocb_fill_direct",
                  lib().tutti_iocb_fill_direct(C.byref(ring), first_slot, n_slots, C.byref(pool), C.byref(cfg),
                                               _p(d_extents), n_req, _p(d_block_table), table_len, _p(d_file_id),
                                               layer, opcode, sgl_table_addr, sgl_id, _p(d_status), _stream(stream)))


def tutti_issue_io(ring, first_slot, n_slots, d_sgl_table, n_desc, sgl_table_addr, store, max_len, cu_budget=0,
                   d_status=None, stream=None):
    return _check("tutti_issue_io",
                  lib().tutti_issue_io(C.byref(ring), first_slot, n_slots, _p(d_sgl_table), n_desc, sgl_table_addr,
                                       C.byref(store), max_len, cu_budget, _p(d_status), _stream(stream)))


def tutti_issue_io_chained(ring, first_slot, n_slots, done_first_slot, done_n_slots, d_sgl_table, n_desc,
                           sgl_table_addr, store, max_len, cu_budget=0, d_status=None, stream=None):
    return _check("tutti_issue_io_chained",
                  lib().tutti_issue_io_chained(C.byref(ring), first_slot, n_slots, done_first_slot, done_n_slots,
                                               _p(d_sgl_table), n_desc, sgl_table_addr, C.byref(store), max_len,
                                               cu_budget, _p(d_status), _stream(stream)))


def tutti_retrieve_layer(ring, first_slot, n_slots, pool, cfg, d_n_blocks, n_req, d_block_table, table_len, d_file_id,
                         layer, sgl_table_addr, sgl_id, store, d_extents, d_totals, cu_budget=0, d_status=None,
                         stream=None):
    return _check("tutti_retrieve_layer",
                  lib().tutti_retrieve_layer(C.byref(ring), first_slot, n_slots, C.byref(pool), C.byref(cfg),
                                             _p(d_n_blocks), n_req, _p(d_block_table), table_len, _p(d_file_id), layer,
                                             sgl_table_addr, sgl_id, C.byref(store), _p(d_extents), _p(d_totals),
                                             cu_budget, _p(d_status), _stream(stream)))


def _ring_layer_call(name):
    def call(ring, first_slot, n_slots, pool, cfg, d_n_blocks, n_req, d_block_table, table_len, d_file_id, layer,
             sgl_table_addr, sgl_id, store, d_extents, d_totals, cu_budget=0, d_status=None, stream=None):
        return _check(name, getattr(lib(), name)(C.byref(ring), first_slot, n_slots, C.byref(pool), C.byref(cfg),
                                                 _p(d_n_blocks), n_req, _p(d_block_table), table_len, _p(d_file_id),
                                                 layer, sgl_table_addr, sgl_id, C.byref(store), _p(d_extents),
                                                 _p(d_totals), cu_budget, _p(d_status), _stream(stream)))
    call.__name__ = name
    return call


def _ring_layer_chained_call(name):
    def call(ring, first_slot, n_slots, done_first_slot, done_n_slots, pool, cfg, d_n_blocks, n_req, d_block_table,
             table_len, d_file_id, layer, sgl_table_addr, sgl_id, store, d_extents, d_totals, cu_budget=0,
             d_status=None, stream=None):
        return _check(name, getattr(lib(), name)(C.byref(ring), first_slot, n_slots, done_first_slot, done_n_slots,
                                                 C.byref(pool), C.byref(cfg), _p(d_n_blocks), n_req,
                                                 _p(d_block_table), table_len, _p(d_file_id), layer, sgl_table_addr,
                                                 sgl_id, C.byref(store), _p(d_extents), _p(d_totals), cu_budget,
                                                 _p(d_status), _stream(stream)))
    call.__name__ = name
    return call


tutti_retrieve_layer_chained = _ring_layer_chained_call("tutti_retrieve_layer_chained")
tutti_store_layer_chained = _ring_layer_chained_call("tutti_store_layer_chained")
tutti_retrieve_layer_issue = _ring_layer_call("tutti_retrieve_layer_issue")
tutti_store_layer_issue = _ring_layer_call("tutti_store_layer_issue")


def tutti_complete_io(ring, first_slot, n_slots, stream=None):
    return _check("tutti_complete_io", lib().tutti_complete_io(C.byref(ring), first_slot, n_slots, _stream(stream)))


def tutti_store_layer(ring, first_slot, n_slots, pool, cfg, d_n_blocks, n_req, d_block_table, table_len, d_file_id,
                      layer, sgl_table_addr, sgl_id, store, d_extents, d_totals, cu_budget=0, d_status=None,
                      stream=None):
    return _check("tutti_store_layer",
                  lib().tutti_store_layer(C.byref(ring), first_slot, n_slots, C.byref(pool), C.byref(cfg),
                                          _p(d_n_blocks), n_req, _p(d_block_table), table_len, _p(d_file_id), layer,
                                          sgl_table_addr, sgl_id, C.byref(store), _p(d_extents), _p(d_totals),
                                          cu_budget, _p(d_status), _stream(stream)))


def tutti_wait_cqe(ring, slot, d_flag, stream=None):
    return _check("tutti_wait_cqe", lib().tutti_wait_cqe(C.byref(ring), slot, _p(d_flag), _stream(stream)))


def tutti_wait_cqe_range(ring, first_slot, n_slots, d_flags, stream=None):
    return _check("tutti_wait_cqe_range", lib().tutti_wait_cqe_range(C.byref(ring), first_slot, n_slots, _p(d_flags),
                                                                     _stream(stream)))


def tutti_layer_save(pool, cfg, d_n_blocks, n_req, d_block_table, table_len, d_file_id, layer, d_stage, stage_cap,
                     stage_addr, sgl_id, d_extents, d_totals, d_sqe, sqe_cap, cu_budget=0, d_status=None, stream=None):
    return _check("tutti_layer_save",
                  lib().tutti_layer_save(C.byref(pool), C.byref(cfg), _p(d_n_blocks), n_req, _p(d_block_table),
                                         table_len, _p(d_file_id), layer, _p(d_stage), stage_cap, stage_addr, sgl_id,
                                         _p(d_extents), _p(d_totals), _p(d_sqe), sqe_cap, cu_budget, _p(d_status),
                                         _stream(stream)))


def tutti_table_validate(num_blocks, d_block_table, table_len, d_status, stream=None):
    return _check("tutti_table_validate", lib().tutti_table_validate(num_blocks, _p(d_block_table), table_len,
                                                                     _p(d_status), _stream(stream)))


def tutti_table_validate_work_bytes(num_blocks):
    return int(lib().tutti_table_validate_work_bytes(num_blocks))


def tutti_table_validate_ws(num_blocks, d_block_table, table_len, d_status, d_work, work_bytes, stream=None):
    return _check("tutti_table_validate_ws", lib().tutti_table_validate_ws(num_blocks, _p(d_block_table), table_len,
                                                                           _p(d_status), _p(d_work), work_bytes,
                                                                           _stream(stream)))


STATIC_VALIDATE_MAX_BLOCKS = 1 << 22


def tutti_table_validate_static(num_blocks, d_block_table, table_len, d_status, stream=None):
    return _check("tutti_table_validate_static", lib().tutti_table_validate_static(num_blocks, _p(d_block_table),
                                                                                   table_len, _p(d_status),
                                                                                   _stream(stream)))


def tutti_stream_baseline(d_buf, nbytes, write, d_xor=None, cu_budget=0, stream=None):
    return _check("tutti_stream_baseline", bench_lib().tutti_stream_baseline(_p(d_buf), nbytes, 1 if write else 0, _p(d_xor),
                                                                       cu_budget, _stream(stream)))


def tutti_copy_baseline(d_dst, d_src, nbytes, cu_budget=0, stream=None):
    return _check("tutti_copy_baseline", bench_lib().tutti_copy_baseline(_p(d_dst), _p(d_src), nbytes, cu_budget,
                                                                   _stream(stream)))


def tutti_scatter_baseline(d_scattered, span_bytes, d_contig, nbytes, d_perm, gran, scatter_writes, shape=0,
                           cu_budget=0, stream=None):
    shape = SCATTER_SHAPES.get(shape, shape)
    return _check("tutti_scatter_baseline",
                  bench_lib().tutti_scatter_baseline(_p(d_scattered), span_bytes, _p(d_contig), nbytes, _p(d_perm), gran,
                                                     1 if scatter_writes else 0, shape, cu_budget, _stream(stream)))


def tutti_strerror(code):
    return lib().tutti_strerror(code).decode()


def tutti_last_hip_error():
    return lib().tutti_last_hip_error()


def tutti_resident_wgs_per_cu(which):
    n = lib().tutti_resident_wgs_per_cu(int(which))
    if n < 0:
        raise TuttiError("tutti_resident_wgs_per_cu", n)
    return n


def tutti_cu_count():
    n = lib().tutti_cu_count()
    if n < 0:
        raise TuttiError("tutti_cu_count", n)
    return n


def tutti_version():
    return lib().tutti_version()


def tutti_abi_describe():
    out = np.zeros(64, np.uint32)
    n = lib().tutti_abi_describe(_p(out), out.size)
    if n < 0:
        raise TuttiError("tutti_abi_describe", n)
    return out[:n].tolist()


def tutti_set_tuning(wgs_per_cu=0, unroll=0):
    return _check("tutti_set_tuning", bench_lib().tutti_set_tuning(wgs_per_cu, unroll))


def tutti_set_nontemporal(mask=3):
    return _check("tutti_set_nontemporal", bench_lib().tutti_set_nontemporal(int(mask)))


def tutti_set_hnd_mode(mode=0):
    return _check("tutti_set_hnd_mode", bench_lib().tutti_set_hnd_mode(int(mode)))


def tutti_set_xcd_mapping(contiguous=0):
    return _check("tutti_set_xcd_mapping", bench_lib().tutti_set_xcd_mapping(1 if contiguous else 0))


# ---- the application's side of the rings (host code only: none of these needs a GPU)

def make_sq_state(depth):
    """Host bookkeeping of one ring's SQ (tutti_sq_state_init).  The flag bytes live in a numpy array kept alive
    by the returned structure."""
    st = tutti_sq_state()
    flags = np.zeros(max(depth, 1), np.uint8)
    st._keep = flags
    _check("tutti_sq_state_init", lib().tutti_sq_state_init(C.byref(st), depth, _p(flags)))
    return st


def tutti_get_iocb(state, n):
    """First of n consecutive free slots; raises TuttiError(EAGAIN) when fewer than n are free."""
    first = C.c_uint32(0)
    _check("tutti_get_iocb", lib().tutti_get_iocb(C.byref(state), n, C.byref(first)))
    return first.value


def tutti_sq_free_count(state):
    return lib().tutti_sq_free_count(C.byref(state))


def tutti_reap_cqe(state, cq_host, sq_host=None):
    """Consumes new completions from a host-readable CQ; returns how many."""
    n = C.c_uint32(0)
    _check("tutti_reap_cqe", lib().tutti_reap_cqe(C.byref(state), _p(cq_host), _p(sq_host), C.byref(n)))
    return n.value


def tutti_iocb_completed(state, slot):
    rc = lib().tutti_iocb_completed(C.byref(state), slot)
    if rc < 0:
        raise TuttiError("tutti_iocb_completed", rc)
    return bool(rc)


def tutti_wait_cqe_host(state, cq_host, sq_host, slot, max_polls):
    rc = lib().tutti_wait_cqe_host(C.byref(state), _p(cq_host), _p(sq_host), slot, max_polls)
    if rc < 0:
        raise TuttiError("tutti_wait_cqe_host", rc)
    return bool(rc)


def make_io_profile(rows):
    """rows: iterable of (cu_budget, n_iocbs, read_us, write_us) -> ctypes array of tutti_io_profile."""
    rows = list(rows)
    arr = (tutti_io_profile * max(len(rows), 1))()
    for i, (b, n, r, w) in enumerate(rows):
        arr[i] = tutti_io_profile(int(b), int(n), float(r), float(w))
    return arr, len(rows)


def tutti_iocbs_for_slack(profile, n_rows, cu_budget, opcode, slack_us):
    out = C.c_uint32(0)
    _check("tutti_iocbs_for_slack", lib().tutti_iocbs_for_slack(profile, n_rows, cu_budget, opcode, slack_us,
                                                               C.byref(out)))
    return out.value


def tutti_budget_for_slack(profile, n_rows, n_iocbs, opcode, slack_us, max_budget):
    """Smallest budget that fits, or None when none does (EAGAIN)."""
    out = C.c_uint32(0)
    rc = lib().tutti_budget_for_slack(profile, n_rows, n_iocbs, opcode, slack_us, max_budget, C.byref(out))
    if rc == EAGAIN:
        return None
    _check("tutti_budget_for_slack", rc)
    return out.value


def tutti_io_domain_create(n_cus):
    """A stream confined to the first n_cus compute units, as an integer handle (hipStream_t)."""
    s = C.c_void_p(0)
    _check("tutti_io_domain_create", lib().tutti_io_domain_create(n_cus, C.byref(s)))
    return s.value


def tutti_io_domain_destroy(stream):
    return _check("tutti_io_domain_destroy", lib().tutti_io_domain_destroy(C.c_void_p(int(stream))))


def tutti_place_work_bytes():
    return lib().tutti_place_work_bytes()


def _plane_array(planes):
    return (C.c_void_p * len(planes))(*[_p(x) for x in planes])


def tutti_place_pair_times(ref, cands, plane_bytes, d_work, work_bytes, reps=3, stream=None):
    """Microseconds of the probe restore on the pool (ref, c) for every c in cands (a list of floats).  Blocks."""
    us = (C.c_float * len(cands))()
    _check("tutti_place_pair_times",
           lib().tutti_place_pair_times(_p(ref), _plane_array(cands), len(cands), plane_bytes, _p(d_work), work_bytes,
                                        reps, us, _stream(stream)))
    return list(us)


def tutti_place_classify(planes, plane_bytes, d_work, work_bytes, max_regions=3, min_gap_us=3.0, stream=None):
    """(classes, rounds): the region class of every plane and the tutti_place_round records.  Blocks."""
    n = len(planes)
    classes = (C.c_int32 * n)()
    rounds = (tutti_place_round * PLACE_MAX_REGIONS)()
    n_rounds = C.c_uint32(0)
    _check("tutti_place_classify",
           lib().tutti_place_classify(_plane_array(planes), n, plane_bytes, _p(d_work), work_bytes, max_regions,
                                      min_gap_us, classes, rounds, C.byref(n_rounds), _stream(stream)))
    return list(classes), [rounds[i] for i in range(n_rounds.value)]


def tutti_place_pairs(classes, n_pairs, strict=True):
    """(pairs, n_mixed): n_pairs (K plane, V plane) index pairs, the first n_mixed from different classes.  Host
    code only.  Raises TuttiError(EAGAIN) when strict and the classes do not allow n_pairs mixed pairs,
    TuttiError(ERANGE) when the planes do not make n_pairs pairs at all."""
    n = len(classes)
    cls = (C.c_int32 * n)(*classes)
    pairs = (C.c_uint32 * (2 * n_pairs))()
    n_mixed = C.c_uint32(0)
    _check("tutti_place_pairs", lib().tutti_place_pairs(cls, n, n_pairs, 1 if strict else 0, pairs, C.byref(n_mixed)))
    return [(pairs[2 * i], pairs[2 * i + 1]) for i in range(n_pairs)], n_mixed.value


def tutti_host_cost_of_restore(pool, cfg, d_n_blocks, n_req, d_block_table, table_len, d_file_id, layer, d_stage,
                               stage_cap, stage_addr, sgl_id, d_extents, d_totals, d_sqe, sqe_cap, n_calls,
                               cu_budget=0, d_status=None, stream=None):
    """Host nanoseconds per tutti_layer_restore call when the calls come from C (measurement library only)."""
    ns = C.c_double(0.0)
    _check("tutti_host_cost_of_restore",
           bench_lib().tutti_host_cost_of_restore(C.byref(pool), C.byref(cfg), _p(d_n_blocks), n_req,
                                                  _p(d_block_table), table_len, _p(d_file_id), layer, _p(d_stage),
                                                  stage_cap, stage_addr, sgl_id, _p(d_extents), _p(d_totals),
                                                  _p(d_sqe), sqe_cap, cu_budget, _p(d_status), _stream(stream),
                                                  n_calls, C.byref(ns)))
    return ns.value
