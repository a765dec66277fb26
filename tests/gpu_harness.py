"""Helpers for the GPU parity tests: one layer's inputs on host and device, both sides run on them.

The HIP path is always called through the C ABI (paper_2605_03375_amd.binding); the oracle through
oracle.tutti_oracle.  Nothing computed by one side is ever fed to the other: both start from the
same seeded inputs and only their outputs are compared, byte for byte.
"""
import numpy as np
import torch

from paper_2605_03375_amd import binding as B
from paper_2605_03375_amd import workloads as W

DEV = "cuda:0"


def to_dev(a):
    a = np.ascontiguousarray(a)
    if a.dtype == np.uint32:
        a = a.view(np.int32)
    return torch.from_numpy(a).to(DEV)


def as_u8(t):
    return t.contiguous().view(torch.uint8).reshape(-1)


class LayerCase:
    """One layer's pool, table and object geometry, resident on host (numpy) and device (torch)."""

    def __init__(self, *, T, h, d, e, N, n_blocks, table, file_id=None, align=4096, chunk=2 << 20, L=1, layout=0,
                 pad=0, fill="values", seed=1, dtype="bf16", name="case"):
        self.T, self.h, self.d, self.e, self.N = T, h, d, e, N
        self.bb = T * h * d * e
        self.stride = self.bb + pad
        self.align, self.chunk, self.L, self.layout, self.name = align, chunk, L, layout, name
        self.n_blocks = np.ascontiguousarray(n_blocks, np.uint32)
        self.table = np.ascontiguousarray(table, np.uint32)
        self.file_id = (np.arange(self.n_blocks.size, dtype=np.uint32) + 1000) if file_id is None else \
            np.ascontiguousarray(file_id, np.uint32)
        nbytes = N * self.stride
        if fill == "tags":
            self.k_dev = W.device_address_tags(nbytes, 0, DEV)
            self.v_dev = W.device_address_tags(nbytes, 1 << 30, DEV)
        else:
            self.k_dev = as_u8(W.device_values(seed, nbytes // 2, dtype, DEV))
            self.v_dev = as_u8(W.device_values(seed + 7, nbytes // 2, dtype, DEV))
        self.k_host = self.k_dev.cpu().numpy()
        self.v_host = self.v_dev.cpu().numpy()
        self.d_n_blocks = to_dev(self.n_blocks) if self.n_blocks.size else torch.zeros(1, dtype=torch.int32, device=DEV)
        self.d_table = to_dev(self.table) if self.table.size else torch.zeros(1, dtype=torch.int32, device=DEV)
        self.d_file_id = to_dev(self.file_id) if self.file_id.size else torch.zeros(1, dtype=torch.int32, device=DEV)

    @classmethod
    def from_workload(cls, w, **kw):
        s = w.shape
        return cls(T=s.block_tokens, h=s.num_kv_heads, d=s.head_dim, e=s.elt_bytes, N=s.num_blocks,
                   n_blocks=w.n_blocks, table=w.block_table, file_id=w.file_id, align=w.align, chunk=w.chunk_bytes,
                   L=s.num_layers, dtype=s.dtype, seed=w.seed, name=w.name, **kw)

    # ---- descriptors for each side
    def geom(self):
        return dict(num_blocks=self.N, block_tokens=self.T, num_kv_heads=self.h, head_dim=self.d, elt_bytes=self.e,
                    block_stride=self.stride, pool_layout=self.layout)

    def gpu_pool(self, k=None, v=None):
        return B.make_pool(self.k_dev if k is None else k, self.v_dev if v is None else v, **self.geom())

    def orc_pool(self, orc, k=None, v=None):
        return orc.make_pool(self.k_host if k is None else k, self.v_host if v is None else v, **self.geom())

    def gpu_cfg(self):
        return B.make_cfg(self.align, self.chunk, self.L)

    def orc_cfg(self, orc):
        return orc.make_cfg(self.align, self.chunk, self.L)

    @property
    def n_req(self):
        return int(self.n_blocks.size)


def new_status():
    return torch.zeros(1, dtype=torch.int32, device=DEV)


def gpu_layout(c):
    ext = torch.zeros(max(1, c.n_req) * 32, dtype=torch.uint8, device=DEV)
    tot = torch.zeros(2, dtype=torch.int64, device=DEV)
    B.tutti_obj_layout(c.gpu_pool(), c.gpu_cfg(), c.d_n_blocks, c.n_req, ext, tot)
    torch.cuda.synchronize()
    return ext, tot


def ext_np(ext, n_req):
    return ext.cpu().numpy()[: 32 * n_req].view(B.EXTENT_DTYPE)


def check_layout(orc, c):
    ext, tot = gpu_layout(c)
    o_ext, o_tot = orc.obj_layout(c.orc_pool(orc), c.orc_cfg(orc), c.n_blocks)
    assert ext.cpu().numpy()[: 32 * c.n_req].tobytes() == o_ext.tobytes(), f"{c.name}: extents differ"
    assert np.array_equal(tot.cpu().numpy().view(np.uint64), o_tot), f"{c.name}: totals differ"
    return ext, tot, o_ext, o_tot


def check_pack(orc, c, ext, o_ext, o_tot, cu_budget=0, stage_cap=None, table_len=None):
    nbytes = max(int(o_tot[0]), 16)
    fill = 0xA5
    stage = torch.full((nbytes,), fill, dtype=torch.uint8, device=DEV)
    st = new_status()
    B.tutti_obj_pack(c.gpu_pool(), c.gpu_cfg(), ext, c.n_req, c.d_table,
                     c.table.size if table_len is None else table_len, stage,
                     int(o_tot[0]) if stage_cap is None else stage_cap, cu_budget, st)
    torch.cuda.synchronize()
    o_stage = np.full(nbytes, fill, np.uint8)
    o_st = orc.obj_pack(c.orc_pool(orc), c.orc_cfg(orc), o_ext, c.table, o_stage,
                        stage_cap=int(o_tot[0]) if stage_cap is None else stage_cap)
    got = stage.cpu().numpy()
    assert np.array_equal(got, o_stage), f"{c.name}: packed objects differ at byte {first_diff(got, o_stage)}"
    assert int(st.item()) == o_st, f"{c.name}: pack status {int(st.item())} vs oracle {o_st}"
    return stage


def first_diff(a, b):
    idx = np.flatnonzero(a != b)
    return int(idx[0]) if idx.size else -1


def check_unpack(orc, c, ext, o_ext, o_tot, cu_budget=0, seed=99, stage_cap=None):
    nbytes = max(int(o_tot[0]), 16)
    g = torch.Generator(device=DEV)
    g.manual_seed(seed)
    stage = torch.randint(0, 256, (nbytes,), dtype=torch.uint8, device=DEV, generator=g)
    k2, v2 = c.k_dev.clone(), c.v_dev.clone()
    st = new_status()
    B.tutti_obj_unpack(c.gpu_pool(k2, v2), c.gpu_cfg(), ext, c.n_req, c.d_table, c.table.size, stage,
                       int(o_tot[0]) if stage_cap is None else stage_cap, cu_budget, st)
    torch.cuda.synchronize()
    ok, ov = c.k_host.copy(), c.v_host.copy()
    o_st = orc.obj_unpack(c.orc_pool(orc, ok, ov), c.orc_cfg(orc), o_ext, c.table, stage.cpu().numpy(),
                          stage_cap=int(o_tot[0]) if stage_cap is None else stage_cap)
    gk, gv = k2.cpu().numpy(), v2.cpu().numpy()
    assert np.array_equal(gk, ok), f"{c.name}: K plane differs at byte {first_diff(gk, ok)}"
    assert np.array_equal(gv, ov), f"{c.name}: V plane differs at byte {first_diff(gv, ov)}"
    assert int(st.item()) == o_st
    return stage


def check_moves_with_extents(orc, c, x, stage_bytes, table_len=None, stage_cap=None, cu_budget=0, seed=77, label=""):
    """tutti_obj_pack and tutti_obj_unpack with extents written by the test (numpy records, B.EXTENT_DTYPE),
    whole buffers and the status word against the oracle given the very same records."""
    x = np.ascontiguousarray(x, dtype=B.EXTENT_DTYPE)
    o_x = np.zeros(x.size, orc.EXTENT_DTYPE)
    for f in B.EXTENT_DTYPE.names:
        o_x[f] = x[f]
    n_req = int(x.size)
    d_x = torch.from_numpy(x.view(np.uint8).copy()).to(DEV) if n_req else torch.zeros(32, dtype=torch.uint8, device=DEV)
    tl = c.table.size if table_len is None else table_len
    cap = stage_bytes if stage_cap is None else stage_cap
    nbytes = max(stage_bytes, 16)
    # pack
    stage = torch.full((nbytes,), 0xA5, dtype=torch.uint8, device=DEV)
    st = new_status()
    B.tutti_obj_pack(c.gpu_pool(), c.gpu_cfg(), d_x, n_req, c.d_table, tl, stage, cap, cu_budget, st)
    torch.cuda.synchronize()
    o_stage = np.full(nbytes, 0xA5, np.uint8)
    o_st = orc.obj_pack(c.orc_pool(orc), c.orc_cfg(orc), o_x, c.table, o_stage, stage_cap=cap, table_len=tl)
    got = stage.cpu().numpy()
    assert np.array_equal(got, o_stage), f"{c.name} {label}: packed bytes differ at {first_diff(got, o_stage)}"
    assert int(st.item()) == o_st, f"{c.name} {label}: pack status {int(st.item())} vs oracle {o_st}"
    # unpack
    g = torch.Generator(device=DEV)
    g.manual_seed(seed)
    stage = torch.randint(0, 256, (nbytes,), dtype=torch.uint8, device=DEV, generator=g)
    k2, v2 = c.k_dev.clone(), c.v_dev.clone()
    st = new_status()
    B.tutti_obj_unpack(c.gpu_pool(k2, v2), c.gpu_cfg(), d_x, n_req, c.d_table, tl, stage, cap, cu_budget, st)
    torch.cuda.synchronize()
    ok, ov = c.k_host.copy(), c.v_host.copy()
    o_st = orc.obj_unpack(c.orc_pool(orc, ok, ov), c.orc_cfg(orc), o_x, c.table, stage.cpu().numpy(), stage_cap=cap,
                          table_len=tl)
    gk, gv = k2.cpu().numpy(), v2.cpu().numpy()
    assert np.array_equal(gk, ok), f"{c.name} {label}: K plane differs at byte {first_diff(gk, ok)}"
    assert np.array_equal(gv, ov), f"{c.name} {label}: V plane differs at byte {first_diff(gv, ov)}"
    assert int(st.item()) == o_st, f"{c.name} {label}: unpack status {int(st.item())} vs oracle {o_st}"
    return o_st


def check_sqe(orc, c, ext, o_ext, o_tot, layer=0, stage_addr=0x7F1200000000, sgl_id=42, sqe_cap=None):
    n = int(o_tot[1])
    cap = n if sqe_cap is None else sqe_cap
    for op in (B.OP_READ, B.OP_WRITE):
        sqe = torch.full((max(cap, 1) * 64,), 0x3C, dtype=torch.uint8, device=DEV)
        st = new_status()
        B.tutti_sqe_build(c.gpu_pool(), c.gpu_cfg(), ext, c.n_req, c.d_file_id, layer, op, stage_addr, sgl_id, sqe,
                          cap, st)
        torch.cuda.synchronize()
        o_sqe, o_st = orc.sqe_build(c.orc_pool(orc), c.orc_cfg(orc), o_ext, c.file_id, layer, op, stage_addr, sgl_id,
                                    sqe_cap=cap)
        n_written = min(n, cap)
        got = sqe.cpu().numpy()
        assert got[: 64 * n_written].tobytes() == o_sqe[:n_written].tobytes(), f"{c.name}: entries differ (op {op})"
        assert np.all(got[64 * n_written:] == 0x3C), "entries beyond the count must stay untouched"
        assert int(st.item()) == o_st


def check_layer_restore(orc, c, layer=0, cu_budget=0, stage_addr=0x7F1200000000, sgl_id=7, seed=5, sqe_cap=None,
                        stage_cap=None, table_len=None, visit=None):
    """visit: table positions in visiting order (numpy): both sides run their ordered restore on the same list."""
    tl = c.table.size if table_len is None else table_len
    o_ext0, o_tot0 = orc.obj_layout(c.orc_pool(orc), c.orc_cfg(orc), c.n_blocks)
    nbytes = max(int(o_tot0[0]), 16)
    n_sqe = int(o_tot0[1])
    cap = n_sqe if sqe_cap is None else sqe_cap
    scap = int(o_tot0[0]) if stage_cap is None else stage_cap
    g = torch.Generator(device=DEV)
    g.manual_seed(seed)
    stage = torch.randint(0, 256, (nbytes,), dtype=torch.uint8, device=DEV, generator=g)
    k2, v2 = c.k_dev.clone(), c.v_dev.clone()
    ext = torch.zeros(max(1, c.n_req) * 32, dtype=torch.uint8, device=DEV)
    tot = torch.zeros(2, dtype=torch.int64, device=DEV)
    sqe = torch.full((max(cap, 1) * 64,), 0x3C, dtype=torch.uint8, device=DEV)
    st = new_status()
    ok, ov = c.k_host.copy(), c.v_host.copy()
    if visit is None:
        B.tutti_layer_restore(c.gpu_pool(k2, v2), c.gpu_cfg(), c.d_n_blocks, c.n_req, c.d_table, tl, c.d_file_id,
                              layer, stage, scap, stage_addr, sgl_id, ext, tot, sqe, cap, cu_budget, st)
        torch.cuda.synchronize()
        o_ext, o_tot, o_sqe, o_st = orc.layer_restore(c.orc_pool(orc, ok, ov), c.orc_cfg(orc), c.n_blocks, c.table,
                                                      c.file_id, layer, stage.cpu().numpy(), stage_addr, sgl_id, cap,
                                                      stage_cap=scap, table_len=tl)
    else:
        visit = np.ascontiguousarray(visit, np.uint32)
        assert visit.size >= tl
        d_visit = to_dev(visit) if visit.size else torch.zeros(1, dtype=torch.int32, device=DEV)
        B.tutti_layer_restore_ordered(c.gpu_pool(k2, v2), c.gpu_cfg(), c.d_n_blocks, c.n_req, c.d_table, tl,
                                      c.d_file_id, layer, stage, scap, stage_addr, sgl_id, ext, tot, sqe, cap, d_visit,
                                      cu_budget, st)
        torch.cuda.synchronize()
        o_ext, o_tot, o_sqe, o_st = orc.layer_restore_ordered(c.orc_pool(orc, ok, ov), c.orc_cfg(orc), c.n_blocks,
                                                              c.table, c.file_id, layer, stage.cpu().numpy(),
                                                              stage_addr, sgl_id, cap, visit, stage_cap=scap,
                                                              table_len=tl)
    assert ext.cpu().numpy()[: 32 * c.n_req].tobytes() == o_ext.tobytes()
    assert np.array_equal(tot.cpu().numpy().view(np.uint64), o_tot)
    n_written = min(n_sqe, cap)
    got = sqe.cpu().numpy()
    assert got[: 64 * n_written].tobytes() == o_sqe[:n_written].tobytes(), f"{c.name}: restore entries differ"
    assert np.all(got[64 * n_written:] == 0x3C)
    gk, gv = k2.cpu().numpy(), v2.cpu().numpy()
    assert np.array_equal(gk, ok), f"{c.name}: restore K plane differs at byte {first_diff(gk, ok)}"
    assert np.array_equal(gv, ov), f"{c.name}: restore V plane differs at byte {first_diff(gv, ov)}"
    assert int(st.item()) == o_st


def check_layer_save(orc, c, layer=0, cu_budget=0, stage_addr=0x7F1200000000, sgl_id=8, sqe_cap=None, stage_cap=None,
                     table_len=None):
    tl = c.table.size if table_len is None else table_len
    o_ext0, o_tot0 = orc.obj_layout(c.orc_pool(orc), c.orc_cfg(orc), c.n_blocks)
    nbytes = max(int(o_tot0[0]), 16)
    n_sqe = int(o_tot0[1])
    cap = n_sqe if sqe_cap is None else sqe_cap
    scap = int(o_tot0[0]) if stage_cap is None else stage_cap
    stage = torch.full((nbytes,), 0x5A, dtype=torch.uint8, device=DEV)
    ext = torch.zeros(max(1, c.n_req) * 32, dtype=torch.uint8, device=DEV)
    tot = torch.zeros(2, dtype=torch.int64, device=DEV)
    sqe = torch.full((max(cap, 1) * 64,), 0x3C, dtype=torch.uint8, device=DEV)
    st = new_status()
    B.tutti_layer_save(c.gpu_pool(), c.gpu_cfg(), c.d_n_blocks, c.n_req, c.d_table, tl, c.d_file_id, layer,
                       stage, scap, stage_addr, sgl_id, ext, tot, sqe, cap, cu_budget, st)
    torch.cuda.synchronize()
    o_stage = np.full(nbytes, 0x5A, np.uint8)
    o_ext, o_tot, o_sqe, o_st = orc.layer_save(c.orc_pool(orc), c.orc_cfg(orc), c.n_blocks, c.table, c.file_id, layer,
                                               o_stage, stage_addr, sgl_id, cap, stage_cap=scap, table_len=tl)
    assert ext.cpu().numpy()[: 32 * c.n_req].tobytes() == o_ext.tobytes()
    assert np.array_equal(tot.cpu().numpy().view(np.uint64), o_tot)
    w = min(n_sqe, cap)
    got = sqe.cpu().numpy()
    assert got[: 64 * w].tobytes() == o_sqe[:w].tobytes() and np.all(got[64 * w:] == 0x3C)
    gs = stage.cpu().numpy()
    assert np.array_equal(gs, o_stage), f"{c.name}: saved objects differ at byte {first_diff(gs, o_stage)}"
    assert int(st.item()) == o_st


def check_everything(orc, c, cu_budget=0):
    """All five entry points on one case, each against the oracle."""
    ext, tot, o_ext, o_tot = check_layout(orc, c)
    check_pack(orc, c, ext, o_ext, o_tot, cu_budget)
    check_unpack(orc, c, ext, o_ext, o_tot, cu_budget)
    check_sqe(orc, c, ext, o_ext, o_tot, layer=c.L - 1)
    check_layer_restore(orc, c, layer=c.L - 1, cu_budget=cu_budget)
    check_layer_save(orc, c, layer=c.L - 1, cu_budget=cu_budget)


def check_direct_mode(orc, c, layer=0, sgl_id=17, sqe_cap=None, table_len=None):
    """Mapping table and per-block entries (no staging copy) against the oracle."""
    k_addr, v_addr = c.k_dev.data_ptr(), c.v_dev.data_ptr()
    n_desc = 2 * c.N
    sgl = torch.full((n_desc * 16 + 64,), 0x3C, dtype=torch.uint8, device=DEV)
    st = new_status()
    B.tutti_sgl_table_build(c.gpu_pool(), k_addr, v_addr, sgl_id, sgl, n_desc, st)
    torch.cuda.synchronize()
    o_sgl, o_st = orc.sgl_table_build(c.orc_pool(orc), k_addr, v_addr, sgl_id)
    got = sgl.cpu().numpy()
    assert got[: 16 * n_desc].tobytes() == o_sgl.tobytes(), f"{c.name}: mapping table differs"
    assert np.all(got[16 * n_desc:] == 0x3C) and int(st.item()) == o_st == 0
    ext, tot, o_ext, o_tot = check_layout(orc, c)
    n = 2 * int(c.n_blocks.sum())
    cap = n if sqe_cap is None else sqe_cap
    tl = c.table.size if table_len is None else table_len
    o_table = c.table.copy()
    o_table[tl:] = 0xFFFFFFFF          # entries beyond table_len count as out of range
    for op in (B.OP_READ, B.OP_WRITE):
        sqe = torch.full((max(cap, 1) * 64,), 0x3C, dtype=torch.uint8, device=DEV)
        st = new_status()
        B.tutti_sqe_build_direct(c.gpu_pool(), c.gpu_cfg(), ext, c.n_req, c.d_table, tl, c.d_file_id, layer, op,
                                 sgl.data_ptr(), sgl_id, sqe, cap, st)
        torch.cuda.synchronize()
        o_sqe, o_st = orc.sqe_build_direct(c.orc_pool(orc), c.orc_cfg(orc), o_ext, o_table, c.file_id, layer, op,
                                           sgl.data_ptr(), sgl_id, sqe_cap=cap)
        w = min(n, cap)
        got = sqe.cpu().numpy()
        assert got[: 64 * w].tobytes() == o_sqe[:w].tobytes(), f"{c.name}: direct entries differ (op {op})"
        assert np.all(got[64 * w:] == 0x3C) and int(st.item()) == o_st
    return sgl


def check_rings(orc, c, layer, opcode, depth, first_slot, n_slots, cu_budget=0, n_desc=None, first_file_id=1000,
                stride_cut=0, seed=3):
    """init_queue -> fill -> issue_io -> wait_cqe on device and in the oracle; same inputs, compare outputs."""
    assert c.bb % c.align == 0
    o_ext, o_tot = orc.obj_layout(c.orc_pool(orc), c.orc_cfg(orc), c.n_blocks)
    ext, tot = gpu_layout(c)
    file_stride = max(16, int(2 * c.L * (int(o_ext["obj_bytes"].max()) if c.n_req else 0)) - stride_cut)
    n_files = max(1, c.n_req)
    g = torch.Generator(device=DEV)
    g.manual_seed(seed)
    store = torch.randint(0, 256, (n_files * file_stride,), dtype=torch.uint8, device=DEV, generator=g)
    o_store = store.cpu().numpy().copy()
    k2, v2 = c.k_dev.clone(), c.v_dev.clone()
    ok, ov = c.k_host.copy(), c.v_host.copy()
    # mapping tables: device addresses on the device, host addresses for the oracle (it dereferences them)
    nd = 2 * c.N
    sgl = torch.zeros(nd * 16, dtype=torch.uint8, device=DEV)
    B.tutti_sgl_table_build(c.gpu_pool(k2, v2), k2.data_ptr(), v2.data_ptr(), 5, sgl, nd)
    o_sgl, _ = orc.sgl_table_build(c.orc_pool(orc, ok, ov), ok.ctypes.data, ov.ctypes.data, 5)
    table_addr = sgl.data_ptr()                       # the same arithmetic base on both sides
    sq_bytes, cq_bytes = B.ring_bytes(depth)
    sq = torch.zeros(sq_bytes, dtype=torch.uint8, device=DEV)
    cq = torch.zeros(cq_bytes, dtype=torch.uint8, device=DEV)
    ring = B.make_ring(sq, cq, depth)
    o_sq, o_cq = orc.ring_alloc(depth)
    st = new_status()
    B.tutti_ring_init(ring)
    orc.ring_init(o_sq, o_cq)
    torch.cuda.synchronize()
    assert sq.cpu().numpy().tobytes() == o_sq.tobytes() and cq.cpu().numpy().tobytes() == o_cq.tobytes()
    B.tutti_iocb_fill_direct(ring, first_slot, n_slots, c.gpu_pool(k2, v2), c.gpu_cfg(), ext, c.n_req, c.d_table,
                             c.table.size, c.d_file_id, layer, opcode, table_addr, 5, st)
    o_st = orc.iocb_fill_direct(o_sq, first_slot, n_slots, c.orc_pool(orc, ok, ov), c.orc_cfg(orc), o_ext, c.table,
                                c.file_id, layer, opcode, table_addr, 5)
    torch.cuda.synchronize()
    assert sq.cpu().numpy().tobytes() == o_sq.tobytes(), f"{c.name}: filled IOCBs differ"
    assert int(st.item()) == o_st
    fs = B.make_filestore(store, file_stride, first_file_id, n_files)
    ndv = nd if n_desc is None else n_desc
    st2 = new_status()
    B.tutti_issue_io(ring, first_slot, n_slots, sgl, ndv, table_addr, fs, c.bb, cu_budget, st2)
    o_st2 = orc.issue_io(o_sq, o_cq, first_slot, n_slots, o_sgl[:ndv], table_addr, o_store, file_stride, first_file_id,
                         n_files)
    flags = torch.full((depth,), 9, dtype=torch.int32, device=DEV)
    for slot in range(depth):
        B.tutti_wait_cqe(ring, slot, flags[slot:])
    torch.cuda.synchronize()
    assert int(st2.item()) == o_st2, f"{c.name}: issue_io status {int(st2.item())} vs oracle {o_st2}"
    gk, gv = k2.cpu().numpy(), v2.cpu().numpy()
    assert np.array_equal(gk, ok), f"{c.name}: K plane differs at byte {first_diff(gk, ok)}"
    assert np.array_equal(gv, ov), f"{c.name}: V plane differs at byte {first_diff(gv, ov)}"
    gs = store.cpu().numpy()
    assert np.array_equal(gs, o_store), f"{c.name}: file store differs at byte {first_diff(gs, o_store)}"
    assert sq.cpu().numpy().tobytes() == o_sq.tobytes(), f"{c.name}: IOCBs differ after issue_io"
    g_cq = cq.cpu().numpy().view(np.uint32)
    assert g_cq.tobytes() == o_cq.tobytes(), f"{c.name}: completion queue differs"
    n_done = int(o_cq[0])
    done_slots = {int(x) for x in o_cq[16:16 + min(n_done, depth)]}
    assert flags.cpu().tolist() == [1 if s in done_slots else 0 for s in range(depth)]
    return n_done


def check_ring_layer(orc, c, layer, write, depth, first_slot, n_slots, cu_budget=0, first_file_id=1000, n_files=None,
                     stride_cut=0, seed=5, prefill=False, side_completion=False):
    """retrieve_layer / store_layer through the rings in one call, device against oracle: same inputs, every
    output compared (extents, totals, status, planes, file store, IOCBs, completion queue, wait_cqe flags).
    prefill: the ring already holds completions of an earlier call (the CQ tail is not 0)."""
    assert c.bb % c.align == 0
    o_ext0, _ = orc.obj_layout(c.orc_pool(orc), c.orc_cfg(orc), c.n_blocks)
    file_stride = max(16, int(2 * c.L * (int(o_ext0["obj_bytes"].max()) if c.n_req else 0)) - stride_cut)
    n_files = max(1, c.n_req) if n_files is None else n_files
    g = torch.Generator(device=DEV)
    g.manual_seed(seed)
    store = torch.randint(0, 256, (n_files * file_stride,), dtype=torch.uint8, device=DEV, generator=g)
    o_store = store.cpu().numpy().copy()
    k2, v2 = c.k_dev.clone(), c.v_dev.clone()
    ok, ov = c.k_host.copy(), c.v_host.copy()
    table_addr = 0x7f00_0000_1000                    # only recorded in the contexts: the same value on both sides
    sq_bytes, cq_bytes = B.ring_bytes(depth)
    sq = torch.zeros(sq_bytes, dtype=torch.uint8, device=DEV)
    cq = torch.zeros(cq_bytes, dtype=torch.uint8, device=DEV)
    ring = B.make_ring(sq, cq, depth)
    o_sq, o_cq = orc.ring_alloc(depth)
    B.tutti_ring_init(ring)
    orc.ring_init(o_sq, o_cq)
    fs = B.make_filestore(store, file_stride, first_file_id, n_files)
    ext = torch.zeros(max(1, c.n_req) * 32, dtype=torch.uint8, device=DEV)
    tot = torch.zeros(2, dtype=torch.int64, device=DEV)
    fn = B.tutti_store_layer if write else B.tutti_retrieve_layer
    if side_completion:
        # the two halves: the data launch on the current stream, the completion on a second stream behind an event
        issue = B.tutti_store_layer_issue if write else B.tutti_retrieve_layer_issue
        side = torch.cuda.Stream()

        def fn(ring, fslot, ns, *rest):
            issue(ring, fslot, ns, *rest)
            ev = torch.cuda.Event()
            ev.record()
            side.wait_event(ev)
            B.tutti_complete_io(ring, fslot, ns, side)
    o_fn = orc.store_layer if write else orc.retrieve_layer
    calls = [(0, min(1, depth), (layer + 1) % c.L)] if prefill else []
    calls.append((first_slot, n_slots, layer))
    for (fslot, ns, lay) in calls:
        st = new_status()
        fn(ring, fslot, ns, c.gpu_pool(k2, v2), c.gpu_cfg(), c.d_n_blocks, c.n_req, c.d_table, c.table.size,
           c.d_file_id, lay, table_addr, 5, fs, ext, tot, cu_budget, st)
        o_ext, o_tot, o_st = o_fn(o_sq, o_cq, fslot, ns, c.orc_pool(orc, ok, ov), c.orc_cfg(orc), c.n_blocks, c.table,
                                  c.file_id, lay, table_addr, 5, o_store, file_stride, first_file_id, n_files)
        torch.cuda.synchronize()
        assert int(st.item()) == o_st, f"{c.name}: status {int(st.item())} vs oracle {o_st}"
    flags = torch.full((depth,), 9, dtype=torch.int32, device=DEV)
    for slot in range(depth):
        B.tutti_wait_cqe(ring, slot, flags[slot:])
    torch.cuda.synchronize()
    assert ext.cpu().numpy()[: 32 * c.n_req].tobytes() == o_ext.tobytes(), f"{c.name}: extents differ"
    assert np.array_equal(tot.cpu().numpy().view(np.uint64), o_tot), f"{c.name}: totals differ"
    gk, gv = k2.cpu().numpy(), v2.cpu().numpy()
    assert np.array_equal(gk, ok), f"{c.name}: K plane differs at byte {first_diff(gk, ok)}"
    assert np.array_equal(gv, ov), f"{c.name}: V plane differs at byte {first_diff(gv, ov)}"
    gs = store.cpu().numpy()
    assert np.array_equal(gs, o_store), f"{c.name}: file store differs at byte {first_diff(gs, o_store)}"
    assert sq.cpu().numpy().tobytes() == o_sq.tobytes(), f"{c.name}: IOCBs differ"
    assert cq.cpu().numpy().tobytes() == o_cq.tobytes(), f"{c.name}: completion queue differs"
    done = o_sq["hdr"]["state"] == orc.IOCB_DONE
    assert flags.cpu().tolist() == [1 if x else 0 for x in done]
    # the same answers from one launch over the whole ring, starting in the middle and wrapping around
    start = depth // 2
    many = torch.full((depth + 1,), 9, dtype=torch.int32, device=DEV)
    B.tutti_wait_cqe_range(ring, start, depth, many)
    torch.cuda.synchronize()
    assert many.cpu().tolist() == [1 if done[(start + i) % depth] else 0 for i in range(depth)] + [9]
    if write:
        assert np.array_equal(gk, c.k_host) and np.array_equal(gv, c.v_host)
    return o_st

def check_ring_layer_train(orc, c, layers, write, depth, n_slots, first_slot=0, cu_budget=0, first_file_id=1000,
                           seed=5):
    """A train of layers through the chained calls (each launch also completes the IOCBs of the call before it, the
    last layer is completed by tutti_complete_io), against the oracle's sequence of one-call retrieve_layer /
    store_layer: every output compared once the train is through.  Before the last completion the last call's IOCBs
    must not read as DONE and every earlier call's must.  Consecutive calls take consecutive slot ranges (modulo
    depth), so depth >= 2 * n_slots keeps a call's range apart from the one it completes."""
    assert c.bb % c.align == 0 and depth >= 2 * n_slots and n_slots > 0
    o_ext0, _ = orc.obj_layout(c.orc_pool(orc), c.orc_cfg(orc), c.n_blocks)
    file_stride = max(16, int(2 * c.L * (int(o_ext0["obj_bytes"].max()) if c.n_req else 0)))
    n_files = max(1, c.n_req)
    g = torch.Generator(device=DEV)
    g.manual_seed(seed)
    store = torch.randint(0, 256, (n_files * file_stride,), dtype=torch.uint8, device=DEV, generator=g)
    o_store = store.cpu().numpy().copy()
    k2, v2 = c.k_dev.clone(), c.v_dev.clone()
    ok, ov = c.k_host.copy(), c.v_host.copy()
    table_addr = 0x7f00_0000_1000
    sq_bytes, cq_bytes = B.ring_bytes(depth)
    sq = torch.zeros(sq_bytes, dtype=torch.uint8, device=DEV)
    cq = torch.zeros(cq_bytes, dtype=torch.uint8, device=DEV)
    ring = B.make_ring(sq, cq, depth)
    o_sq, o_cq = orc.ring_alloc(depth)
    B.tutti_ring_init(ring)
    orc.ring_init(o_sq, o_cq)
    fs = B.make_filestore(store, file_stride, first_file_id, n_files)
    ext = torch.zeros(max(1, c.n_req) * 32, dtype=torch.uint8, device=DEV)
    tot = torch.zeros(2, dtype=torch.int64, device=DEV)
    fn = B.tutti_store_layer_chained if write else B.tutti_retrieve_layer_chained
    o_fn = orc.store_layer if write else orc.retrieve_layer
    st = new_status()
    o_st_all = 0
    prev = (0, 0)
    slots = []
    for i, lay in enumerate(layers):
        fslot = (first_slot + i * n_slots) % depth
        fn(ring, fslot, n_slots, prev[0], prev[1], c.gpu_pool(k2, v2), c.gpu_cfg(), c.d_n_blocks, c.n_req, c.d_table,
           c.table.size, c.d_file_id, lay, table_addr, 5, fs, ext, tot, cu_budget, st)      # no synchronisation
        o_ext, o_tot, o_st = o_fn(o_sq, o_cq, fslot, n_slots, c.orc_pool(orc, ok, ov), c.orc_cfg(orc), c.n_blocks,
                                  c.table, c.file_id, lay, table_addr, 5, o_store, file_stride, first_file_id, n_files)
        o_st_all |= o_st
        prev = (fslot, n_slots)
        slots.append(fslot)
    # the train is through but for its last completion
    flags = torch.full((depth,), 9, dtype=torch.int32, device=DEV)
    B.tutti_wait_cqe_range(ring, 0, depth, flags)
    torch.cuda.synchronize()
    got = flags.cpu().tolist()
    last = {(prev[0] + k) % depth for k in range(n_slots)}
    done = o_sq["hdr"]["state"] == orc.IOCB_DONE
    assert got == [0 if s in last else (1 if done[s] else 0) for s in range(depth)], f"{c.name}: {got}"
    tail_before = int(cq[:8].cpu().numpy().view(np.uint32)[0])
    B.tutti_complete_io(ring, prev[0], prev[1])
    torch.cuda.synchronize()
    assert int(st.item()) == o_st_all, f"{c.name}: status {int(st.item())} vs oracle {o_st_all}"
    assert ext.cpu().numpy()[: 32 * c.n_req].tobytes() == o_ext.tobytes(), f"{c.name}: extents differ"
    assert np.array_equal(tot.cpu().numpy().view(np.uint64), o_tot), f"{c.name}: totals differ"
    gk, gv = k2.cpu().numpy(), v2.cpu().numpy()
    assert np.array_equal(gk, ok), f"{c.name}: K plane differs at byte {first_diff(gk, ok)}"
    assert np.array_equal(gv, ov), f"{c.name}: V plane differs at byte {first_diff(gv, ov)}"
    gs = store.cpu().numpy()
    assert np.array_equal(gs, o_store), f"{c.name}: file store differs at byte {first_diff(gs, o_store)}"
    assert sq.cpu().numpy().tobytes() == o_sq.tobytes(), f"{c.name}: IOCBs differ"
    assert cq.cpu().numpy().tobytes() == o_cq.tobytes(), f"{c.name}: completion queue differs"
    return o_st_all, tail_before

def check_rings_train(orc, c, steps, depth, n_slots, first_slot=0, cu_budget=0, first_file_id=1000, seed=3):
    """A train of fill + tutti_issue_io_chained calls (steps: (layer, opcode) pairs; each issue completes the IOCBs of
    the one before it, tutti_complete_io ends the train) against the oracle's fill + issue_io sequence: IOCBs, CQ,
    planes, file store and status compared once the train is through."""
    assert c.bb % c.align == 0 and depth >= 2 * n_slots and n_slots > 0
    o_ext, o_tot = orc.obj_layout(c.orc_pool(orc), c.orc_cfg(orc), c.n_blocks)
    ext, tot = gpu_layout(c)
    file_stride = max(16, int(2 * c.L * (int(o_ext["obj_bytes"].max()) if c.n_req else 0)))
    n_files = max(1, c.n_req)
    g = torch.Generator(device=DEV)
    g.manual_seed(seed)
    store = torch.randint(0, 256, (n_files * file_stride,), dtype=torch.uint8, device=DEV, generator=g)
    o_store = store.cpu().numpy().copy()
    k2, v2 = c.k_dev.clone(), c.v_dev.clone()
    ok, ov = c.k_host.copy(), c.v_host.copy()
    nd = 2 * c.N
    sgl = torch.zeros(nd * 16, dtype=torch.uint8, device=DEV)
    B.tutti_sgl_table_build(c.gpu_pool(k2, v2), k2.data_ptr(), v2.data_ptr(), 5, sgl, nd)
    o_sgl, _ = orc.sgl_table_build(c.orc_pool(orc, ok, ov), ok.ctypes.data, ov.ctypes.data, 5)
    table_addr = sgl.data_ptr()
    sq_bytes, cq_bytes = B.ring_bytes(depth)
    sq = torch.zeros(sq_bytes, dtype=torch.uint8, device=DEV)
    cq = torch.zeros(cq_bytes, dtype=torch.uint8, device=DEV)
    ring = B.make_ring(sq, cq, depth)
    o_sq, o_cq = orc.ring_alloc(depth)
    B.tutti_ring_init(ring)
    orc.ring_init(o_sq, o_cq)
    fs = B.make_filestore(store, file_stride, first_file_id, n_files)
    st = new_status()
    o_st_all = 0
    prev = (0, 0)
    for i, (layer, opcode) in enumerate(steps):
        fslot = (first_slot + i * n_slots) % depth
        B.tutti_iocb_fill_direct(ring, fslot, n_slots, c.gpu_pool(k2, v2), c.gpu_cfg(), ext, c.n_req, c.d_table,
                                 c.table.size, c.d_file_id, layer, opcode, table_addr, 5, st)
        B.tutti_issue_io_chained(ring, fslot, n_slots, prev[0], prev[1], sgl, nd, table_addr, fs, c.bb, cu_budget, st)
        o_st_all |= orc.iocb_fill_direct(o_sq, fslot, n_slots, c.orc_pool(orc, ok, ov), c.orc_cfg(orc), o_ext, c.table,
                                         c.file_id, layer, opcode, table_addr, 5)
        o_st_all |= orc.issue_io(o_sq, o_cq, fslot, n_slots, o_sgl, table_addr, o_store, file_stride, first_file_id,
                                 n_files)
        prev = (fslot, n_slots)
    flags = torch.full((depth,), 9, dtype=torch.int32, device=DEV)
    B.tutti_wait_cqe_range(ring, 0, depth, flags)
    torch.cuda.synchronize()
    last = {(prev[0] + k) % depth for k in range(n_slots)}
    done = o_sq["hdr"]["state"] == orc.IOCB_DONE
    assert flags.cpu().tolist() == [0 if s in last else (1 if done[s] else 0) for s in range(depth)]
    B.tutti_issue_io_chained(ring, 0, 0, prev[0], prev[1], sgl, nd, table_addr, fs, c.bb, cu_budget, st)   # only completes
    torch.cuda.synchronize()
    assert int(st.item()) == o_st_all, f"{c.name}: status {int(st.item())} vs oracle {o_st_all}"
    gk, gv = k2.cpu().numpy(), v2.cpu().numpy()
    assert np.array_equal(gk, ok), f"{c.name}: K plane differs at byte {first_diff(gk, ok)}"
    assert np.array_equal(gv, ov), f"{c.name}: V plane differs at byte {first_diff(gv, ov)}"
    gs = store.cpu().numpy()
    assert np.array_equal(gs, o_store), f"{c.name}: file store differs at byte {first_diff(gs, o_store)}"
    assert sq.cpu().numpy().tobytes() == o_sq.tobytes(), f"{c.name}: IOCBs differ"
    assert cq.cpu().numpy().tobytes() == o_cq.tobytes(), f"{c.name}: completion queue differs"
    return o_st_all
