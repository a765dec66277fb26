"""Pins for the CPU oracle: what the paper prints, closed forms, library routines, brute force.

Every check takes the oracle wrapper module `orc` and raises AssertionError on a mismatch, so
the same checks run against the real oracle (tests must pass) and against deliberately broken
copies of its source (tests/test_oracle_mutants.py: every check list must catch its mutants).
Nothing here retypes the oracle's own code path: expected values come from the paper's printed
numbers (tests/golden/paper_counts.txt), numpy library routines (cumsum, fancy indexing,
transpose), or a six-deep pure-Python loop written from the element-wise definition.
"""
import itertools
import os

import numpy as np

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "paper_counts.txt")


def golden():
    out = {}
    with open(GOLDEN) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            name, value, _ = [x.strip() for x in line.split("|", 2)]
            out[name] = int(value)
    return out


def _pool(orc, T, h, d, e, N, k=None, v=None, stride=None, layout=0):
    return orc.make_pool(k, v, num_blocks=N, block_tokens=T, num_kv_heads=h, head_dim=d, elt_bytes=e,
                         block_stride=stride, pool_layout=layout)


def _planes(rng, N, stride):
    k = rng.integers(0, 256, size=N * stride, dtype=np.uint8)
    v = rng.integers(0, 256, size=N * stride, dtype=np.uint8)
    return k, v


# ---------------------------------------------------------------------------- paper counts

def check_paper_counts(orc):
    g = golden()
    # 64 layers, 64-token blocks, 128K tokens, one entry per block (chunk = block): sec. 2.2
    T, h, d, e = 64, 8, 128, 2
    bb = T * h * d * e
    p = _pool(orc, T, h, d, e, 4096)
    cfg = orc.make_cfg(4096, bb, 64)
    n = 128 * 1024 // T
    ext, tot = orc.obj_layout(p, cfg, [n])
    assert int(tot[1]) * 64 == g["io_count_64layer_block64_128k"]
    assert int(tot[1]) == g["objects_per_file_factor"] * n
    # 256-token chunks, 128K tokens, K and V counted separately: sec. 2.2
    p = _pool(orc, 256, 8, 128, 2, 1024)
    cfg = orc.make_cfg(4096, 256 * 8 * 128 * 2, 32)
    ext, tot = orc.obj_layout(p, cfg, [128 * 1024 // 256])
    assert int(tot[1]) == g["chunk_accesses_256tok_128k"]
    # descriptor arithmetic: sec. 3.1
    assert orc.desc_count(60 * 1024 ** 3, 4096) == g["pool_pages_60GiB_4KiB"]
    nd = orc.desc_count(60 * 1024 ** 3, 64 * 1024)
    assert nd == g["descriptors_60GiB_64KiB"]
    assert nd * 4096 == g["prp_bytes"] and nd * g["sgl_descriptor_bytes"] == g["sgl_bytes"]
    assert orc.desc_count(65537, 65536) == 2 and orc.desc_count(65536, 65536) == 1
    assert orc.IOCB_SLOTS == g["iocb_slots"]


def check_closed_forms_8b(orc):
    """The 8B shape: 2048 blocks of 32 KiB, 2 MiB chunks -> 64 entries and 128 MiB per layer."""
    p = _pool(orc, 16, 8, 128, 2, 65536)
    assert orc.block_bytes(p) == 32768
    cfg = orc.make_cfg(4096, 2 << 20, 32)
    ext, tot = orc.obj_layout(p, cfg, [2048])
    assert int(tot[0]) == 134217728 and int(tot[1]) == 64
    assert int(ext["obj_bytes"][0]) == 67108864 and int(ext["n_chunks"][0]) == 32
    # Tiny: 32 blocks of 4 KiB -> one 128 KiB object per plane; 4 KiB chunks -> 32 entries per object
    p = _pool(orc, 16, 2, 64, 2, 256)
    assert orc.block_bytes(p) == 4096
    ext, tot = orc.obj_layout(p, orc.make_cfg(4096, 4096, 1), [32])
    assert int(tot[0]) == 262144 and int(tot[1]) == 64
    ext, tot = orc.obj_layout(p, orc.make_cfg(4096, 2 << 20, 1), [32])
    assert int(tot[1]) == 2


def check_abi(orc):
    g = golden()
    d = orc.abi_describe()
    assert len(d) == 52
    ext, sqe, pool, cfg, sgl = d[0:7], d[7:19], d[19:29], d[29:33], d[33:37]
    hdr, iocb, cqh, fst = d[37:44], d[44:46], d[46], d[47:52]
    assert hdr == [64, 0, 4, 8, 12, 16, 20] and iocb == [64 + g["iocb_slots"] * 64, 64] and cqh == 64
    assert fst == [24, 0, 8, 16, 20]
    Hd, Io = orc.IOCB_HDR_DTYPE, orc.IOCB_DTYPE
    assert Hd.itemsize == 64 and [Hd.fields[n][1] for n in Hd.names[:6]] == hdr[1:]
    assert Io.itemsize == iocb[0] and Io.fields["ioctx"][1] == 64 and orc.CQ_HDR_WORDS * 4 == cqh
    import ctypes as _c
    assert _c.sizeof(orc.OrcFileStore) == 24
    assert sgl == [g["sgl_descriptor_bytes"], 0, 8, 12]      # address 8 + length 4 + identifier 4: sec. 3.1
    G = orc.SGL_DTYPE
    assert [G.itemsize] + [G.fields[n][1] for n in G.names] == sgl
    assert ext == [32, 0, 8, 16, 20, 24, 28]
    assert sqe == [64, 0, 1, 2, 4, 8, 16, 24, 28, 32, 40, 44]
    assert pool == [48, 0, 8, 16, 24, 28, 32, 36, 40, 44]
    assert cfg == [12, 0, 4, 8]
    # the wrapper's numpy / ctypes declarations agree with the C ones
    E, S = orc.EXTENT_DTYPE, orc.SQE_DTYPE
    assert E.itemsize == 32 and [E.fields[n][1] for n in E.names] == ext[1:]
    assert S.itemsize == 64 and [S.fields[n][1] for n in S.names[:-1]] == sqe[1:]
    assert S.fields["rsvd"][1] == 48
    import ctypes
    assert ctypes.sizeof(orc.OrcPool) == 48 and ctypes.sizeof(orc.OrcObjCfg) == 12
    # the SGL triple (address 8, length 4, identifier 4) sits in 16 consecutive bytes: sec. 3.1
    assert S.fields["addr"][1] + 8 == S.fields["len"][1] and S.fields["len"][1] + 4 == S.fields["sgl_id"][1]
    assert S.fields["sgl_id"][1] + 4 - S.fields["addr"][1] == g["sgl_descriptor_bytes"]


# ---------------------------------------------------------------------------- extents

def check_layout_scan(orc, seed=11):
    """Offsets are exclusive prefix sums (numpy cumsum) and obey the alignment / packing invariants."""
    rng = np.random.default_rng(seed)
    for T, h, d, e, A, C in [(16, 8, 128, 2, 4096, 2 << 20), (16, 2, 64, 2, 4096, 4096), (16, 5, 40, 2, 4096, 8192),
                             (3, 1, 8, 2, 512, 512), (16, 8, 128, 2, 4096, 32768), (7, 3, 16, 1, 64, 192)]:
        bb = T * h * d * e
        for R in (1, 2, 7, 64, 65, 300):
            n = rng.integers(0, 50, size=R).astype(np.uint32)
            n[rng.integers(0, R)] = 0
            p = _pool(orc, T, h, d, e, 1 << 16)
            ext, tot = orc.obj_layout(p, orc.make_cfg(A, C, 4), n)
            obj = (n.astype(np.uint64) * bb + A - 1) // A * A
            chunks = (obj + C - 1) // C
            assert np.array_equal(ext["n_blocks"], n)
            assert np.array_equal(ext["obj_bytes"], obj)
            assert np.array_equal(ext["n_chunks"], chunks.astype(np.uint32))
            assert np.array_equal(ext["stage_off"], np.cumsum(2 * obj) - 2 * obj)
            assert np.array_equal(ext["sqe_base"], (np.cumsum(2 * chunks) - 2 * chunks).astype(np.uint32))
            assert np.array_equal(ext["table_off"], (np.cumsum(n.astype(np.uint64)) - n).astype(np.uint32))
            assert int(tot[0]) == int((2 * obj).sum()) and int(tot[1]) == int((2 * chunks).sum())
            assert np.all(ext["stage_off"] % A == 0) and np.all(ext["obj_bytes"] % A == 0)
            assert np.all(ext["obj_bytes"] >= n.astype(np.uint64) * bb)
            assert np.all(ext["obj_bytes"] < n.astype(np.uint64) * bb + A)
            # naive O(R^2) sums
            for r in range(0, R, max(1, R // 5)):
                assert int(ext["stage_off"][r]) == sum(2 * int(o) for o in obj[:r])
    # no requests at all
    ext, tot = orc.obj_layout(_pool(orc, 16, 8, 128, 2, 64), orc.make_cfg(), np.zeros(0, np.uint32))
    assert ext.size == 0 and int(tot[0]) == 0 and int(tot[1]) == 0


# ---------------------------------------------------------------------------- pack / unpack

def _ref_extents(n_blocks, bb, A):
    """Plain-Python extents for the reference formulations below: (stage_off, obj_bytes) per request."""
    out, off = [], 0
    for n in n_blocks:
        obj = -(-int(n) * bb // A) * A
        out.append((off, obj))
        off += 2 * obj
    return out, off


def ref_pack_elementwise(k, v, layout, T, h, d, e, stride, n_blocks, table, A):
    """The definition, element by element: six nested loops (request, kind, block, token, head, dim)."""
    bb = T * h * d * e
    ext, total = _ref_extents(n_blocks, bb, A)
    stage = np.zeros(total, np.uint8)
    pos = 0
    for r, n in enumerate(n_blocks):
        off, obj = ext[r]
        for kind in range(2):
            plane = (k, v)[kind]
            for j in range(int(n)):
                blk = int(table[pos + j]) * stride
                for t in range(T):
                    for i in range(h):
                        for x in range(d):
                            src = ((t * h + i) * d + x) * e if layout == 0 else ((i * T + t) * d + x) * e
                            dst = off + kind * obj + j * bb + ((t * h + i) * d + x) * e
                            stage[dst:dst + e] = plane[blk + src: blk + src + e]
        pos += int(n)
    return stage


def check_pack_bruteforce(orc):
    """Pools of <= 6 blocks: every ordered selection of blocks as the table, both layouts."""
    rng = np.random.default_rng(5)
    T, h, d, e, A = 3, 2, 4, 2, 64  # block_bytes 48: not a multiple of A, so every object has padding
    bb = T * h * d * e
    for N in (1, 3, 4):
        k, v = _planes(rng, N, bb)
        for layout in (0, 1):
            p = _pool(orc, T, h, d, e, N, k, v, layout=layout)
            cfg = orc.make_cfg(A, A, 2)
            for m in range(0, N + 1):
                for table in itertools.permutations(range(N), m):
                    ext, tot = orc.obj_layout(p, cfg, [m])
                    stage = np.full(int(tot[0]), 0xAB, np.uint8)
                    assert orc.obj_pack(p, cfg, ext, np.array(table, np.uint32), stage) == 0
                    want = ref_pack_elementwise(k, v, layout, T, h, d, e, bb, [m], table, A)
                    assert np.array_equal(stage, want), (N, layout, table)
    # two requests sharing one pool of 6 blocks, every split of a permutation
    N = 6
    k, v = _planes(rng, N, bb)
    for layout in (0, 1):
        p = _pool(orc, T, h, d, e, N, k, v, layout=layout)
        cfg = orc.make_cfg(A, 2 * A, 2)
        for perm in itertools.islice(itertools.permutations(range(N)), 0, 720, 7):
            for cut in range(0, N + 1):
                nb = [cut, N - cut]
                ext, tot = orc.obj_layout(p, cfg, nb)
                stage = np.full(int(tot[0]), 0xCD, np.uint8)
                orc.obj_pack(p, cfg, ext, np.array(perm, np.uint32), stage)
                want = ref_pack_elementwise(k, v, layout, T, h, d, e, bb, nb, perm, A)
                assert np.array_equal(stage, want), (layout, perm, cut)


def check_pack_vs_numpy(orc, seed=3):
    """NHD pack is a fancy-index gather; identity table is a memcpy; HND is a transpose; strided pools."""
    rng = np.random.default_rng(seed)
    for T, h, d, e, A, pad in [(16, 2, 64, 2, 4096, 0), (16, 8, 128, 2, 4096, 0), (16, 5, 40, 2, 4096, 0),
                               (16, 2, 64, 2, 4096, 256), (4, 3, 8, 2, 128, 16)]:
        bb = T * h * d * e
        stride = bb + pad
        N = 64
        k, v = _planes(rng, N, stride)
        k2, v2 = k.reshape(N, stride), v.reshape(N, stride)
        n = np.array([5, 0, 17, 1, 9], np.uint32)
        table = rng.permutation(N)[: int(n.sum())].astype(np.uint32)
        cfg = orc.make_cfg(A, 4 * A, 3)
        for layout in (0, 1):
            p = _pool(orc, T, h, d, e, N, k, v, stride=stride, layout=layout)
            ext, tot = orc.obj_layout(p, cfg, n)
            stage = np.full(int(tot[0]), 0xEE, np.uint8)
            assert orc.obj_pack(p, cfg, ext, table, stage) == 0
            pos = 0
            for r in range(n.size):
                ids = table[pos:pos + n[r]]
                for kind, plane in enumerate((k2, v2)):
                    blocks = plane[ids, :bb]                     # library gather
                    if layout == 1:                              # [h][T][d*e] -> [T][h][d*e]
                        blocks = blocks.reshape(-1, h, T, d * e).transpose(0, 2, 1, 3)
                    want = np.ascontiguousarray(blocks).reshape(-1)
                    o = int(ext["stage_off"][r]) + kind * int(ext["obj_bytes"][r])
                    got = stage[o:o + int(ext["obj_bytes"][r])]
                    assert np.array_equal(got[:want.size], want), (layout, r, kind)
                    assert not got[want.size:].any(), "padding must be zero"
                pos += int(n[r])
        # identity table on a dense NHD pool: the K object is the first n*bb bytes of the plane
        if pad == 0:
            p = _pool(orc, T, h, d, e, N, k, v)
            ext, tot = orc.obj_layout(p, cfg, [N])
            stage = np.zeros(int(tot[0]), np.uint8)
            orc.obj_pack(p, cfg, ext, np.arange(N, dtype=np.uint32), stage)
            assert stage[:N * bb].tobytes() == k.tobytes()
            o = int(ext["obj_bytes"][0])
            assert stage[o:o + N * bb].tobytes() == v.tobytes()


def check_address_tags(orc):
    """Each 32-bit word of the pool holds its own index: every misplaced word is visible."""
    T, h, d, e, A, N = 16, 2, 64, 2, 4096, 32
    bb = T * h * d * e
    words = bb // 4
    k = np.arange(N * words, dtype=np.uint32)
    v = np.arange(N * words, dtype=np.uint32) + (1 << 30)
    table = np.array([9, 3, 31, 0, 17], np.uint32)
    p = _pool(orc, T, h, d, e, N, k.view(np.uint8), v.view(np.uint8))
    cfg = orc.make_cfg(A, A, 1)
    ext, tot = orc.obj_layout(p, cfg, [table.size])
    stage = np.zeros(int(tot[0]), np.uint8)
    orc.obj_pack(p, cfg, ext, table, stage)
    sw = stage.view(np.uint32)
    for j, b in enumerate(table):
        assert np.array_equal(sw[j * words:(j + 1) * words], np.arange(b * words, (b + 1) * words, dtype=np.uint32))
        vo = int(ext["obj_bytes"][0]) // 4
        assert np.array_equal(sw[vo + j * words: vo + (j + 1) * words],
                              np.arange(b * words, (b + 1) * words, dtype=np.uint32) + (1 << 30))


def check_roundtrip_and_untouched(orc, seed=8):
    """unpack(pack(P)) = P on the named blocks; unpack writes nothing else; pack(unpack(S)) = S."""
    rng = np.random.default_rng(seed)
    for T, h, d, e, A, pad, layout in [(16, 2, 64, 2, 4096, 0, 0), (16, 2, 64, 2, 4096, 0, 1),
                                       (16, 5, 40, 2, 4096, 64, 0), (4, 3, 8, 2, 128, 16, 1)]:
        bb = T * h * d * e
        stride = bb + pad
        N = 48
        k, v = _planes(rng, N, stride)
        n = np.array([7, 0, 12, 3], np.uint32)
        table = rng.permutation(N)[: int(n.sum())].astype(np.uint32)
        cfg = orc.make_cfg(A, 2 * A, 2)
        p = _pool(orc, T, h, d, e, N, k, v, stride=stride, layout=layout)
        ext, tot = orc.obj_layout(p, cfg, n)
        stage = np.zeros(int(tot[0]), np.uint8)
        orc.obj_pack(p, cfg, ext, table, stage)
        # restore into a different, pre-filled pool
        k2, v2 = _planes(rng, N, stride)
        k2_before, v2_before = k2.copy(), v2.copy()
        p2 = _pool(orc, T, h, d, e, N, k2, v2, stride=stride, layout=layout)
        assert orc.obj_unpack(p2, cfg, ext, table, stage) == 0
        named = np.zeros(N, bool)
        named[table] = True
        for b in range(N):
            sl = slice(b * stride, b * stride + bb)
            gap = slice(b * stride + bb, (b + 1) * stride)
            if named[b]:
                assert np.array_equal(k2[sl], k[sl]) and np.array_equal(v2[sl], v[sl])
            else:
                assert np.array_equal(k2[sl], k2_before[sl]) and np.array_equal(v2[sl], v2_before[sl])
            assert np.array_equal(k2[gap], k2_before[gap]) and np.array_equal(v2[gap], v2_before[gap])
        # and back: pack of the restored pool reproduces the staging buffer, padding zero
        stage2 = np.full(int(tot[0]), 0x77, np.uint8)
        orc.obj_pack(p2, cfg, ext, table, stage2)
        assert np.array_equal(stage2, stage)
        # K and V are not swapped: the first object of request 0 holds K bytes
        if layout == 0:
            b0 = int(table[0])
            assert np.array_equal(stage[:bb], k[b0 * stride: b0 * stride + bb])


def check_skips_and_status(orc):
    rng = np.random.default_rng(21)
    T, h, d, e, A, N = 4, 2, 8, 2, 128, 16
    bb = T * h * d * e
    k, v = _planes(rng, N, bb)
    p = _pool(orc, T, h, d, e, N, k, v)
    cfg = orc.make_cfg(A, A, 1)
    n = np.array([3, 2], np.uint32)
    ext, tot = orc.obj_layout(p, cfg, n)
    table = np.array([1, 99, 4, 7, 8], np.uint32)  # 99 is out of range
    stage = np.full(int(tot[0]), 0x55, np.uint8)
    st = orc.obj_pack(p, cfg, ext, table, stage)
    assert st == orc.ST_BAD_BLOCK
    assert np.all(stage[bb:2 * bb] == 0x55), "a skipped block leaves its object bytes alone"
    assert np.array_equal(stage[:bb], k[bb:2 * bb]) and np.array_equal(stage[2 * bb:3 * bb], k[4 * bb:5 * bb])
    # the first id that is out of range is num_blocks itself (planes hold one spare block here)
    kx, vx = _planes(rng, N + 1, bb)
    px = _pool(orc, T, h, d, e, N, kx, vx)
    stage = np.full(int(tot[0]), 0x55, np.uint8)
    st = orc.obj_pack(px, cfg, ext, np.array([N - 1, N, 0, 1, 2], np.uint32), stage)
    assert st == orc.ST_BAD_BLOCK and np.all(stage[bb:2 * bb] == 0x55)
    assert np.array_equal(stage[:bb], kx[(N - 1) * bb:N * bb])
    # staging buffer too small for the second request: only the first is packed
    table = np.array([1, 2, 4, 7, 8], np.uint32)
    cap = int(ext["stage_off"][1]) + 8
    stage = np.full(int(tot[0]), 0x55, np.uint8)
    st = orc.obj_pack(p, cfg, ext, table, stage, stage_cap=cap)
    assert st == orc.ST_STAGE_CAP
    assert np.all(stage[int(ext["stage_off"][1]):] == 0x55)
    assert np.array_equal(stage[:bb], k[bb:2 * bb])
    k2, v2 = k.copy(), v.copy()
    p2 = _pool(orc, T, h, d, e, N, k2, v2)
    stage[:] = 0
    st = orc.obj_unpack(p2, cfg, ext, table, stage, stage_cap=cap)
    assert st == orc.ST_STAGE_CAP
    assert not k2[bb:3 * bb].any() and np.array_equal(k2[7 * bb:9 * bb], k[7 * bb:9 * bb])
    # entry capacity
    sqe, st = orc.sqe_build(p, cfg, ext, [5, 6], 0, orc.OP_READ, 0, 0, sqe_cap=3)
    assert st == orc.ST_SQE_CAP and sqe.size == 3 and np.all(sqe["opcode"] == orc.OP_READ)


def check_errors(orc):
    import pytest
    p = _pool(orc, 16, 2, 64, 2, 8)
    for bad in [dict(align=4095), dict(align=8), dict(chunk_bytes=4097), dict(chunk_bytes=0), dict(num_layers=0)]:
        kw = dict(align=4096, chunk_bytes=8192, num_layers=1)
        kw.update(bad)
        with pytest.raises(orc.OracleError):
            orc.obj_layout(p, orc.make_cfg(**kw), [1])
    for bad in [dict(T=0), dict(d=3, e=1, T=1, h=1), dict(N=0), dict(stride=4095), dict(layout=2)]:
        kw = dict(T=16, h=2, d=64, e=2, N=8, stride=None, layout=0)
        kw.update(bad)
        with pytest.raises(orc.OracleError):
            orc.obj_layout(_pool(orc, kw["T"], kw["h"], kw["d"], kw["e"], kw["N"], stride=kw["stride"],
                                 layout=kw["layout"]), orc.make_cfg(), [1])
    ext, _ = orc.obj_layout(p, orc.make_cfg(num_layers=2), [2])
    with pytest.raises(orc.OracleError):
        orc.sqe_build(p, orc.make_cfg(num_layers=2), ext, [1], 2, orc.OP_READ, 0, 0)      # layer >= L
    with pytest.raises(orc.OracleError):
        orc.sqe_build(p, orc.make_cfg(num_layers=2), ext, [1], 0, 3, 0, 0)               # bad opcode
    with pytest.raises(orc.OracleError):
        orc.sqe_build(p, orc.make_cfg(num_layers=2), ext, [1], 0, orc.OP_READ, 100, 0)   # misaligned address


# ---------------------------------------------------------------------------- submission entries

def check_sqe_fields(orc, seed=13):
    """Entry order, every field, and the tiling invariants, from a separate Python enumeration."""
    rng = np.random.default_rng(seed)
    for T, h, d, e, A, C, L in [(16, 8, 128, 2, 4096, 2 << 20, 32), (16, 2, 64, 2, 4096, 4096, 1),
                                (16, 5, 40, 2, 4096, 12288, 5), (16, 8, 128, 2, 4096, 32768, 80)]:
        bb = T * h * d * e
        p = _pool(orc, T, h, d, e, 1 << 16)
        cfg = orc.make_cfg(A, C, L)
        n = rng.integers(0, 300, size=9).astype(np.uint32)
        n[4] = 0
        fid = rng.integers(0, 1 << 32, size=n.size, dtype=np.uint64).astype(np.uint32)
        ext, tot = orc.obj_layout(p, cfg, n)
        base = 0x7F0000000000
        for layer, op in [(0, orc.OP_READ), (L - 1, orc.OP_WRITE)]:
            sqe, st = orc.sqe_build(p, cfg, ext, fid, layer, op, base, 77)
            assert st == 0 and sqe.size == int(tot[1])
            i = 0
            stage_off = 0
            for r in range(n.size):
                obj = -(-int(n[r]) * bb // A) * A
                for kind in range(2):
                    c = 0
                    covered = 0
                    while covered < obj:
                        s = sqe[i]
                        ln = min(C, obj - covered)
                        assert (s["opcode"], s["kind"], s["layer"], s["file_id"]) == (op, kind, layer, fid[r])
                        assert int(s["len"]) == ln and ln % A == 0
                        assert int(s["addr"]) == base + stage_off + kind * obj + covered
                        assert int(s["file_off"]) == (2 * layer + kind) * obj + covered
                        assert int(s["sgl_id"]) == 77
                        assert int(s["user_data"]) == (r << 32) | i
                        assert (int(s["iocb_idx"]), int(s["ioctx_slot"])) == divmod(i, 2048)
                        assert not s["rsvd"].any()
                        covered += ln
                        c += 1
                        i += 1
                    assert c == int(ext["n_chunks"][r])
                stage_off += 2 * obj
            assert i == sqe.size
            # the entries tile the staging range exactly, in order
            ends = sqe["addr"] + sqe["len"]
            assert sqe.size == 0 or (int(sqe["addr"][0]) == base and int(ends[-1]) == base + int(tot[0]))
            assert np.array_equal(sqe["addr"][1:], ends[:-1])
        # the last chunk of (layer L-1, V) ends the request's GPU file of 2*L objects: sec. 3.1
        sqe, _ = orc.sqe_build(p, cfg, ext, fid, L - 1, orc.OP_READ, base, 0)
        for r in range(n.size):
            if n[r] == 0:
                continue
            last = sqe[int(ext["sqe_base"][r]) + 2 * int(ext["n_chunks"][r]) - 1]
            assert int(last["kind"]) == 1
            assert int(last["file_off"]) + int(last["len"]) == 2 * L * int(ext["obj_bytes"][r])
    # more than one IOCB: 2048 slots each (sec. 3.2)
    p = _pool(orc, 16, 2, 64, 2, 1 << 16)
    cfg = orc.make_cfg(4096, 4096, 1)
    ext, tot = orc.obj_layout(p, cfg, [1500, 1000])
    sqe, _ = orc.sqe_build(p, cfg, ext, [1, 2], 0, orc.OP_READ, 0, 0)
    assert sqe.size == 5000 and int(sqe["iocb_idx"][-1]) == 2 and int(sqe["ioctx_slot"][2048]) == 0
    assert np.array_equal(sqe["iocb_idx"].astype(np.int64) * 2048 + sqe["ioctx_slot"], np.arange(5000))


def check_layer_restore(orc, seed=17):
    """The fused call equals layout + READ entries + unpack done one by one."""
    rng = np.random.default_rng(seed)
    T, h, d, e, A, N = 16, 2, 64, 2, 4096, 64
    bb = T * h * d * e
    for layout in (0, 1):
        n = np.array([4, 0, 9, 2], np.uint32)
        table = rng.permutation(N)[: int(n.sum())].astype(np.uint32)
        fid = np.array([10, 11, 12, 13], np.uint32)
        cfg = orc.make_cfg(A, 2 * A, 3)
        k, v = _planes(rng, N, bb)
        ka, va = k.copy(), v.copy()
        pa = _pool(orc, T, h, d, e, N, ka, va, layout=layout)
        ext, tot = orc.obj_layout(pa, cfg, n)
        stage = rng.integers(0, 256, size=int(tot[0]), dtype=np.uint8)
        sqe, _ = orc.sqe_build(pa, cfg, ext, fid, 1, orc.OP_READ, 8192, 5)
        orc.obj_unpack(pa, cfg, ext, table, stage)
        kb, vb = k.copy(), v.copy()
        pb = _pool(orc, T, h, d, e, N, kb, vb, layout=layout)
        ext2, tot2, sqe2, st = orc.layer_restore(pb, cfg, n, table, fid, 1, stage, 8192, 5, sqe.size)
        assert st == 0 and np.array_equal(tot, tot2)
        assert ext.tobytes() == ext2.tobytes() and sqe.tobytes() == sqe2.tobytes()
        assert np.array_equal(ka, kb) and np.array_equal(va, vb)
        assert not np.array_equal(ka, k)
        # the save direction: extents, WRITE entries and packed objects as the separate calls give them
        wsqe, _ = orc.sqe_build(pa, cfg, ext, fid, 2, orc.OP_WRITE, 4096, 6)
        s1 = np.full(int(tot[0]), 0x42, np.uint8)
        orc.obj_pack(pa, cfg, ext, table, s1)
        s2 = np.full(int(tot[0]), 0x42, np.uint8)
        ext3, tot3, wsqe3, st = orc.layer_save(pa, cfg, n, table, fid, 2, s2, 4096, 6, wsqe.size)
        assert st == 0 and np.array_equal(tot, tot3) and ext.tobytes() == ext3.tobytes()
        assert wsqe.tobytes() == wsqe3.tobytes() and np.all(wsqe3["opcode"] == orc.OP_WRITE)
        assert np.array_equal(s1, s2) and not np.all(s2 == 0x42)


def check_threaded(orc, seed=19):
    """The threaded timing helpers produce the single-threaded result."""
    rng = np.random.default_rng(seed)
    T, h, d, e, A, N = 16, 2, 64, 2, 4096, 128
    bb = T * h * d * e
    for layout in (0, 1):
        k, v = _planes(rng, N, bb)
        n = np.array([30, 0, 41, 5], np.uint32)
        table = rng.permutation(N)[: int(n.sum())].astype(np.uint32)
        cfg = orc.make_cfg(A, A, 1)
        p = _pool(orc, T, h, d, e, N, k, v, layout=layout)
        ext, tot = orc.obj_layout(p, cfg, n)
        s1 = np.zeros(int(tot[0]), np.uint8)
        orc.obj_pack(p, cfg, ext, table, s1)
        for nt in (1, 3, 8):
            s2 = np.full(int(tot[0]), 0x11, np.uint8)
            orc.obj_pack(p, cfg, ext, table, s2, n_threads=nt)
            assert np.array_equal(s1, s2)
            k2, v2 = np.zeros_like(k), np.zeros_like(v)
            k3, v3 = np.zeros_like(k), np.zeros_like(v)
            orc.obj_unpack(_pool(orc, T, h, d, e, N, k2, v2, layout=layout), cfg, ext, table, s1)
            orc.obj_unpack(_pool(orc, T, h, d, e, N, k3, v3, layout=layout), cfg, ext, table, s1, n_threads=nt)
            assert np.array_equal(k2, k3) and np.array_equal(v2, v3)


# ---------------------------------------------------------------------------- direct-to-block mode

def check_sgl_table(orc):
    """The mapping table: the paper's descriptor arithmetic, and descriptors that tile the planes."""
    g = golden()
    # 60 GiB of KV memory described at 64 KiB granularity (sec. 3.1): K and V planes of 491,520 blocks each
    p = _pool(orc, 16, 8, 256, 2, 491520)
    assert orc.block_bytes(p) == 65536
    assert 2 * p.num_blocks * 65536 == 60 * 1024 ** 3
    table, st = orc.sgl_table_build(p, 0x100000000000, 0x200000000000, 9)
    assert st == 0 and table.size == g["descriptors_60GiB_64KiB"] and table.nbytes == g["sgl_bytes"]
    for base, lo in ((0x100000000000, 0), (0x200000000000, p.num_blocks)):
        part = table[lo:lo + p.num_blocks]
        assert int(part["addr"][0]) == base and np.all(part["len"] == 65536) and np.all(part["id"] == 9)
        assert np.array_equal(part["addr"][1:], part["addr"][:-1] + part["len"][:-1])   # tiles the plane
        assert int(part["addr"][-1]) + 65536 == base + 30 * 1024 ** 3
    # strided pool: addresses step by the stride, lengths stay the block size
    p = _pool(orc, 16, 2, 64, 2, 10, stride=4096 + 512)
    table, st = orc.sgl_table_build(p, 1 << 20, 1 << 30, 3)
    assert np.array_equal(table["addr"][:10], (1 << 20) + np.arange(10, dtype=np.uint64) * 4608)
    assert np.array_equal(table["addr"][10:], (1 << 30) + np.arange(10, dtype=np.uint64) * 4608)
    assert np.all(table["len"] == 4096)
    table, st = orc.sgl_table_build(p, 1 << 20, 1 << 30, 3, cap=13)
    assert st == orc.ST_SQE_CAP and table.size == 13 and int(table["addr"][12]) == (1 << 30) + 2 * 4608


def check_direct_entries(orc, seed=23):
    """One entry per (hit block, K|V): the paper's count, every field from a separate enumeration, and
    agreement with the staged mode on everything but the address."""
    g = golden()
    # 64 layers, 64-token blocks, 128K tokens: 2 x 64 x 128K/64 objects in total (sec. 2.2)
    T, h, d, e = 64, 8, 128, 2
    bb = T * h * d * e
    n = 128 * 1024 // T
    p = _pool(orc, T, h, d, e, 4096)
    cfg = orc.make_cfg(4096, bb, 64)
    ext, tot = orc.obj_layout(p, cfg, [n])
    sqe, st = orc.sqe_build_direct(p, cfg, ext, np.arange(n), [5], 63, orc.OP_READ, 1 << 32, 0)
    assert st == 0 and sqe.size * 64 == g["io_count_64layer_block64_128k"]
    rng = np.random.default_rng(seed)
    for T, h, d, e, A, pad in [(16, 8, 128, 2, 4096, 0), (16, 2, 64, 2, 4096, 128), (4, 4, 16, 2, 256, 0)]:
        bb = T * h * d * e
        N, L = 500, 7
        p = _pool(orc, T, h, d, e, N, stride=bb + pad)
        cfg = orc.make_cfg(A, bb, L)
        nb = np.array([6, 0, 40, 1, 13], np.uint32)
        table = rng.permutation(N)[: int(nb.sum())].astype(np.uint32)
        fid = np.array([11, 12, 13, 14, 15], np.uint32)
        ext, tot = orc.obj_layout(p, cfg, nb)
        base = 0x7E0000000000
        k_addr, v_addr = 0x100000000, 0x900000000
        sgl, _ = orc.sgl_table_build(p, k_addr, v_addr, 21)
        for layer, op in ((0, orc.OP_WRITE), (L - 1, orc.OP_READ)):
            sqe, st = orc.sqe_build_direct(p, cfg, ext, table, fid, layer, op, base, 21)
            assert st == 0 and sqe.size == 2 * int(nb.sum())
            i, pos = 0, 0
            for r in range(nb.size):
                obj = int(nb[r]) * bb           # block size is a multiple of A here: no padding
                for kind in range(2):
                    for j in range(int(nb[r])):
                        s = sqe[i]
                        bid = int(table[pos + j])
                        assert (s["opcode"], s["kind"], s["layer"], s["file_id"]) == (op, kind, layer, fid[r])
                        assert int(s["len"]) == bb and int(s["sgl_id"]) == 21
                        assert int(s["file_off"]) == (2 * layer + kind) * obj + j * bb
                        assert int(s["addr"]) == base + 16 * (kind * N + bid)
                        # the descriptor the entry names describes exactly that block
                        dsc = sgl[(int(s["addr"]) - base) // 16]
                        assert int(dsc["addr"]) == (k_addr, v_addr)[kind] + bid * (bb + pad) and int(dsc["len"]) == bb
                        assert int(s["user_data"]) == (r << 32) | i
                        assert (int(s["iocb_idx"]), int(s["ioctx_slot"])) == divmod(i, 2048)
                        assert not s["rsvd"].any()
                        i += 1
                pos += int(nb[r])
            # same GPU-file layout as the staged mode with one chunk per block
            staged, _ = orc.sqe_build(p, cfg, ext, fid, layer, op, 0, 21)
            for f in ("opcode", "kind", "layer", "file_id", "file_off", "len", "sgl_id", "user_data", "iocb_idx",
                      "ioctx_slot"):
                assert np.array_equal(staged[f], sqe[f]), f
    # out-of-range ids become no-op entries; the capacity clamps
    p = _pool(orc, 16, 2, 64, 2, 8)
    cfg = orc.make_cfg(4096, 4096, 1)
    ext, _ = orc.obj_layout(p, cfg, [3])
    sqe, st = orc.sqe_build_direct(p, cfg, ext, [1, 8, 2], [1], 0, orc.OP_READ, 0, 0)
    assert st == orc.ST_BAD_BLOCK and int(sqe["len"][1]) == 0 and int(sqe["addr"][1]) == 0 and int(sqe["len"][4]) == 0
    assert int(sqe["len"][0]) == 4096 and int(sqe["addr"][5]) == 16 * (8 + 2)
    sqe, st = orc.sqe_build_direct(p, cfg, ext, [1, 3, 2], [1], 0, orc.OP_READ, 0, 0, sqe_cap=4)
    assert st == orc.ST_SQE_CAP and sqe.size == 4
    import pytest
    with pytest.raises(orc.OracleError):   # blocks must be whole alignment units in this mode
        orc.sqe_build_direct(_pool(orc, 16, 5, 40, 2, 8), orc.make_cfg(4096, 8192, 1), ext, [1, 3, 2], [1], 0,
                             orc.OP_READ, 0, 0)


# ---------------------------------------------------------------------------- rings

def check_ring_fill(orc, seed=29):
    """init_queue / get_iocb + fill: unique indices, 2048 contexts per IOCB, wrap-around, capacities."""
    g = golden()
    rng = np.random.default_rng(seed)
    depth = 8
    sq, cq = orc.ring_alloc(depth)
    sq["hdr"]["state"] = 7
    cq[:] = 5
    orc.ring_init(sq, cq)
    assert np.array_equal(sq["hdr"]["iocb_idx"], np.arange(depth)) and np.all(sq["hdr"]["state"] == orc.IOCB_FREE)
    assert np.all(sq["hdr"]["num_ioctx"] == 0) and int(cq[0]) == 0 and int(cq[1]) == depth
    T, h, d, e, N, L = 16, 2, 64, 2, 4000, 5
    p = _pool(orc, T, h, d, e, N)
    cfg = orc.make_cfg(4096, 4096, L)
    nb = np.array([1500, 0, 1000], np.uint32)           # 5000 contexts: 2048 + 2048 + 904
    table = rng.permutation(N)[: int(nb.sum())].astype(np.uint32)
    fid = np.array([40, 41, 42], np.uint32)
    ext, _ = orc.obj_layout(p, cfg, nb)
    want, _ = orc.sqe_build_direct(p, cfg, ext, table, fid, 3, orc.OP_READ, 1 << 36, 9)
    st = orc.iocb_fill_direct(sq, 6, 4, p, cfg, ext, table, fid, 3, orc.OP_READ, 1 << 36, 9)   # slots 6, 7, 0, 1
    assert st == 0
    slots = [6, 7, 0, 1]
    counts = [g["iocb_slots"], g["iocb_slots"], 5000 - 2 * g["iocb_slots"], 0]
    got = []
    for slot, cnt in zip(slots, counts):
        hd = sq["hdr"][slot]
        assert (int(hd["num_ioctx"]), int(hd["state"]), int(hd["layer"]), int(hd["opcode"]), int(hd["iocb_idx"])) == \
            (cnt, orc.IOCB_FILLED, 3, orc.OP_READ, slot)
        got.append(sq["ioctx"][slot][:cnt])
    assert np.concatenate(got).tobytes() == want.tobytes()   # the layer's contexts, dealt 2048 per IOCB
    for slot in (2, 3, 4, 5):
        assert int(sq["hdr"]["state"][slot]) == orc.IOCB_FREE
    # every context knows its own place: i = 2048 * iocb_idx + ioctx_slot (relative to the first IOCB)
    allc = np.concatenate(got)
    assert np.array_equal(allc["iocb_idx"].astype(np.int64) * 2048 + allc["ioctx_slot"], np.arange(5000))
    # too few IOCBs: exactly n_slots * 2048 contexts, reported
    orc.ring_init(sq, cq)
    st = orc.iocb_fill_direct(sq, 0, 2, p, cfg, ext, table, fid, 3, orc.OP_WRITE, 1 << 36, 9)
    assert st == orc.ST_SQE_CAP and int(sq["hdr"]["num_ioctx"][1]) == 2048 and int(sq["hdr"]["state"][2]) == orc.IOCB_FREE
    assert np.concatenate([sq["ioctx"][0], sq["ioctx"][1]])["file_off"].tobytes() == want["file_off"][:4096].tobytes()
    import pytest
    with pytest.raises(orc.OracleError):
        orc.iocb_fill_direct(sq, 0, depth + 1, p, cfg, ext, table, fid, 3, orc.OP_READ, 1 << 36, 9)
    with pytest.raises(orc.OracleError):
        orc.iocb_fill_direct(sq, depth, 1, p, cfg, ext, table, fid, 3, orc.OP_READ, 1 << 36, 9)


def check_issue_io(orc, seed=37):
    """issue_io: READ lands each file chunk in the block its descriptor names, WRITE the reverse; the CQ lists
    the completed IOCBs.  Expected bytes come from numpy fancy indexing on independently built files."""
    rng = np.random.default_rng(seed)
    T, h, d, e, N, L, A = 16, 2, 64, 2, 3000, 3, 4096
    bb = T * h * d * e
    for pad in (0, 512):
        stride = bb + pad
        k, v = _planes(rng, N, stride)
        k0, v0 = k.copy(), v.copy()
        p = _pool(orc, T, h, d, e, N, k, v, stride=stride)
        cfg = orc.make_cfg(A, bb, L)
        nb = np.array([1100, 3, 0, 200], np.uint32)       # 2606 contexts: two IOCBs
        table = rng.permutation(N)[: int(nb.sum())].astype(np.uint32)
        fid = np.array([70, 71, 72, 73], np.uint32)
        ext, _ = orc.obj_layout(p, cfg, nb)
        file_stride = int(2 * L * ext["obj_bytes"].max())
        store = rng.integers(0, 256, size=4 * file_stride, dtype=np.uint8)
        store0 = store.copy()
        sgl, _ = orc.sgl_table_build(p, k.ctypes.data, v.ctypes.data, 4)
        base = 0x5000_0000_0000
        depth = 4
        sq, cq = orc.ring_alloc(depth)
        orc.ring_init(sq, cq)
        layer = 1
        assert orc.iocb_fill_direct(sq, 3, 2, p, cfg, ext, table, fid, layer, orc.OP_READ, base, 4) == 0
        assert orc.issue_io(sq, cq, 3, 2, sgl, base, store, file_stride, 70, 4) == 0
        assert int(cq[0]) == 2 and list(cq[16:18]) == [3, 0] and np.all(sq["hdr"]["state"][[3, 0]] == orc.IOCB_DONE)
        assert np.array_equal(sq["hdr"]["done"][[3, 0]], sq["hdr"]["num_ioctx"][[3, 0]]) and int(sq["hdr"]["done"][1]) == 0
        k2, v2 = k.reshape(N, stride), v.reshape(N, stride)
        pos = 0
        named = np.zeros(N, bool)
        for r in range(nb.size):
            ids = table[pos:pos + nb[r]]
            named[ids] = True
            obj = int(ext["obj_bytes"][r])
            for kind, plane in enumerate((k2, v2)):
                lo = r * file_stride + (2 * layer + kind) * obj
                want = store0[lo:lo + int(nb[r]) * bb].reshape(-1, bb)
                assert np.array_equal(plane[ids, :bb], want), (pad, r, kind)        # library gather
            pos += int(nb[r])
        assert np.array_equal(k2[~named], k0.reshape(N, stride)[~named]) and np.array_equal(store, store0)
        assert np.array_equal(k2[:, bb:], k0.reshape(N, stride)[:, bb:])            # stride gaps untouched
        # WRITE: a fresh layer region of every file receives the blocks
        k[:] = k0
        v[:] = v0
        orc.ring_init(sq, cq)
        assert orc.iocb_fill_direct(sq, 0, 2, p, cfg, ext, table, fid, 2, orc.OP_WRITE, base, 4) == 0
        assert orc.issue_io(sq, cq, 0, 2, sgl, base, store, file_stride, 70, 4) == 0
        pos = 0
        touched = np.zeros(store.size, bool)
        for r in range(nb.size):
            ids = table[pos:pos + nb[r]]
            obj = int(ext["obj_bytes"][r])
            for kind, plane in enumerate((k2, v2)):
                lo = r * file_stride + (4 + kind) * obj
                assert np.array_equal(store[lo:lo + int(nb[r]) * bb], plane[ids, :bb].reshape(-1))
                touched[lo:lo + int(nb[r]) * bb] = True
            pos += int(nb[r])
        assert np.array_equal(store[~touched], store0[~touched])
    # contexts that point outside the table, the store or the file are skipped and reported
    orc.ring_init(sq, cq)
    orc.iocb_fill_direct(sq, 0, 2, p, cfg, ext, table, fid, 0, orc.OP_READ, base, 4)
    kb = k.copy()
    assert orc.issue_io(sq, cq, 0, 2, sgl[:N], base, store, file_stride, 70, 4) == orc.ST_BAD_BLOCK   # V descriptors cut off
    assert orc.issue_io(sq, cq, 0, 2, sgl, base, store, file_stride, 71, 4) == 0       # already DONE: nothing re-runs
    orc.ring_init(sq, cq)
    orc.iocb_fill_direct(sq, 0, 2, p, cfg, ext, table, fid, 0, orc.OP_READ, base, 4)
    k[:] = kb
    assert orc.issue_io(sq, cq, 0, 2, sgl, base, store, file_stride, 71, 4) == orc.ST_BAD_BLOCK       # file 70 unknown
    orc.ring_init(sq, cq)
    orc.iocb_fill_direct(sq, 0, 2, p, cfg, ext, table, fid, L - 1, orc.OP_READ, base, 4)   # last layer: ends at the file's end
    assert orc.issue_io(sq, cq, 0, 2, sgl, base, store, file_stride - 16, 70, 4) == orc.ST_BAD_BLOCK  # file too short
    assert orc.issue_io(sq, cq, 2, 2, sgl, base, store, file_stride, 70, 4) == 0 and int(cq[0]) == 2  # FREE slots: no-op


def check_issue_io_hand_filled(orc, seed=59):
    """The paper's own flow (sec. 3.2 "Async I/O Processing"): the application fills the contexts and num_ioctx
    itself.  Contexts written here with numpy, one per rule; expected bytes are numpy slices."""
    rng = np.random.default_rng(seed)
    N, bb = 12, 256
    k = rng.integers(0, 256, N * bb, dtype=np.uint8)
    k0 = k.copy()
    sgl = np.zeros(N, orc.SGL_DTYPE)
    sgl["addr"] = k.ctypes.data + bb * np.arange(N, dtype=np.uint64)
    sgl["len"] = bb
    sgl["len"][5] = 128                       # a short descriptor
    sgl["addr"][6] += 8                       # a misaligned block address
    sgl["len"][9] = 512                       # a descriptor longer than max_len below
    sgl["id"] = 3
    base = 0x4000_0000
    file_stride, n_files, first_file = 4096, 2, 40
    store = rng.integers(0, 256, n_files * file_stride, dtype=np.uint8)
    store0 = store.copy()

    def ctx(op, blk, fid, off, ln, addr=None):
        c = np.zeros((), orc.SQE_DTYPE)
        c["opcode"], c["file_id"], c["file_off"], c["len"] = op, fid, off, ln
        c["addr"] = base + 16 * blk if addr is None else addr
        return c

    good = [ctx(orc.OP_READ, 0, 40, 0, 256), ctx(orc.OP_READ, 1, 41, 4096 - 256, 256), ctx(orc.OP_WRITE, 2, 40, 512, 128),
            ctx(orc.OP_READ, 3, 41, 16, 16), ctx(orc.OP_READ, 5, 40, 1024, 128), ctx(orc.OP_READ, 4, 40, 2048, 0)]
    bad = [ctx(0, 7, 40, 0, 256), ctx(3, 7, 40, 0, 256),                  # opcode
           ctx(orc.OP_READ, 7, 40, 0, 256, addr=base - 16),              # below the table
           ctx(orc.OP_READ, 7, 40, 0, 256, addr=base + 16 * 7 + 8),      # between two descriptors
           ctx(orc.OP_READ, N, 40, 0, 256),                              # beyond the table
           ctx(orc.OP_READ, 5, 40, 0, 144),                              # longer than its descriptor
           ctx(orc.OP_READ, 9, 40, 0, 272),                              # within its descriptor, beyond max_len
           ctx(orc.OP_READ, 7, 40, 0, 24),                               # length not a multiple of 16
           ctx(orc.OP_READ, 7, 40, 8, 256),                              # file offset not a multiple of 16
           ctx(orc.OP_READ, 6, 40, 0, 256),                              # block address not a multiple of 16
           ctx(orc.OP_READ, 7, 39, 0, 256), ctx(orc.OP_READ, 7, 42, 0, 256),   # file outside the store
           ctx(orc.OP_READ, 7, 40, 4096 - 240, 256),                     # runs off the end of the file
           ctx(orc.OP_READ, 7, 40, (1 << 64) - 16, 256)]                 # offset + length wraps around
    depth = 3
    sq, cq = orc.ring_alloc(depth)
    orc.ring_init(sq, cq)
    # application side: IOCB 2 takes the good contexts and IOCB 0 the bad ones (wrap-around), num_ioctx updated
    for slot, items in ((2, good), (0, bad)):
        for i, c in enumerate(items):
            sq["ioctx"][slot][i] = c
        sq["hdr"]["num_ioctx"][slot] = len(items)
        sq["hdr"]["state"][slot] = orc.IOCB_FILLED
    sq["ioctx"][2][len(good)] = ctx(orc.OP_READ, 8, 40, 0, 256)   # beyond num_ioctx: must not run
    st = orc.issue_io(sq, cq, 2, 2, sgl[:N], base, store, file_stride, first_file, n_files, max_len=256)
    assert st == orc.ST_BAD_BLOCK
    want_k, want_store = k0.copy(), store0.copy()
    want_k[0:256] = store0[0:256]
    want_k[256:512] = store0[file_stride + 4096 - 256: file_stride + 4096]
    want_store[512:640] = k0[2 * bb: 2 * bb + 128]
    want_k[3 * bb: 3 * bb + 16] = store0[file_stride + 16: file_stride + 32]
    want_k[5 * bb: 5 * bb + 128] = store0[1024:1152]
    assert np.array_equal(k, want_k) and np.array_equal(store, want_store)
    assert int(cq[0]) == 2 and list(cq[16:18]) == [2, 0]
    assert list(sq["hdr"]["state"]) == [orc.IOCB_DONE, orc.IOCB_FREE, orc.IOCB_DONE]
    assert int(sq["hdr"]["done"][0]) == len(bad) and int(sq["hdr"]["done"][2]) == len(good)
    # each bad context alone trips the status word; each good one alone does not
    for items, want in ((bad, orc.ST_BAD_BLOCK), (good, 0)):
        for c in items:
            orc.ring_init(sq, cq)
            sq["ioctx"][1][0] = c
            sq["hdr"]["num_ioctx"][1] = 1
            sq["hdr"]["state"][1] = orc.IOCB_FILLED
            kb, sb = k.copy(), store.copy()
            st = orc.issue_io(sq, cq, 1, 1, sgl[:N], base, store, file_stride, first_file, n_files, max_len=256)
            assert st == want, c
            if want:
                assert np.array_equal(k, kb) and np.array_equal(store, sb), c


def check_ring_layer(orc, seed=41):
    """store_layer / retrieve_layer through the rings: the file regions hold what obj_pack stages for the same
    requests (either mode reads what the other wrote), a retrieve into a wiped pool brings the named blocks
    back (numpy fancy indexing as the reference), extents are those of obj_layout, completions are in slot order."""
    rng = np.random.default_rng(seed)
    T, h, d, e, N, L, A = 16, 2, 64, 2, 2600, 3, 4096
    bb = T * h * d * e
    stride = bb + 256
    k, v = _planes(rng, N, stride)
    k0, v0 = k.copy(), v.copy()
    p = _pool(orc, T, h, d, e, N, k, v, stride=stride)
    cfg = orc.make_cfg(A, bb, L)
    nb = np.array([7, 0, 1200, 31], np.uint32)             # 2476 contexts: two IOCBs
    table = rng.permutation(N)[: int(nb.sum())].astype(np.uint32)
    fid = np.array([9, 6, 7, 8], np.uint32)                # files are not in request order
    ext0, tot0 = orc.obj_layout(p, cfg, nb)
    file_stride = int(2 * L * ext0["obj_bytes"].max())
    store = rng.integers(0, 256, size=4 * file_stride, dtype=np.uint8)
    store0 = store.copy()
    base = 0x7000_0000_0000
    depth, layer = 3, 2
    sq, cq = orc.ring_alloc(depth)
    orc.ring_init(sq, cq)
    ext, tot, st = orc.store_layer(sq, cq, 2, 2, p, cfg, nb, table, fid, layer, base, 11, store, file_stride, 6, 4)
    assert st == 0 and ext.tobytes() == ext0.tobytes() and np.array_equal(tot, tot0)
    assert np.array_equal(k, k0) and np.array_equal(v, v0)                       # a store does not touch the pool
    assert int(cq[0]) == 2 and list(cq[16:18]) == [2, 0]
    assert list(sq["hdr"]["state"]) == [orc.IOCB_DONE, orc.IOCB_FREE, orc.IOCB_DONE]
    assert list(sq["hdr"]["num_ioctx"][[2, 0]]) == [2048, 2 * int(nb.sum()) - 2048]
    assert np.all(sq["hdr"]["opcode"][[2, 0]] == orc.OP_WRITE) and np.all(sq["hdr"]["layer"][[2, 0]] == layer)
    # the staged mode's objects for the same requests: K object then V object per request
    stage = np.zeros(int(tot0[0]), np.uint8)
    assert orc.obj_pack(p, cfg, ext0, table, stage) == 0
    touched = np.zeros(store.size, bool)
    k2, v2 = k.reshape(N, stride), v.reshape(N, stride)
    pos = 0
    for r in range(nb.size):
        obj = int(ext0["obj_bytes"][r])
        so = int(ext0["stage_off"][r])
        ids = table[pos:pos + nb[r]]
        for kind, plane in enumerate((k2, v2)):
            lo = (int(fid[r]) - 6) * file_stride + (2 * layer + kind) * obj
            assert np.array_equal(store[lo:lo + obj], stage[so + kind * obj: so + (kind + 1) * obj]), (r, kind)
            assert np.array_equal(store[lo:lo + obj], plane[ids, :bb].reshape(-1)), (r, kind)
            touched[lo:lo + obj] = True
        pos += int(nb[r])
    assert np.array_equal(store[~touched], store0[~touched])
    # retrieve into a wiped pool: named blocks come back, nothing else is written
    k[:] = 0
    v[:] = 0
    ext, tot, st = orc.retrieve_layer(sq, cq, 1, 2, p, cfg, nb, table, fid, layer, base, 11, store, file_stride, 6, 4)
    assert st == 0 and ext.tobytes() == ext0.tobytes() and np.array_equal(tot, tot0)
    named = np.zeros(N, bool)
    named[table] = True
    k0r, v0r = k0.reshape(N, stride), v0.reshape(N, stride)
    assert np.array_equal(k2[named, :bb], k0r[named, :bb]) and np.array_equal(v2[named, :bb], v0r[named, :bb])
    assert not k2[~named].any() and not v2[~named].any() and not k2[:, bb:].any() and not v2[:, bb:].any()
    assert int(cq[0]) == 4 and list(cq[16:19]) == [2, 0, 1]    # completions 2, 3 (slots 1, 2) land in entries 2, 0
    assert np.all(sq["hdr"]["opcode"][[1, 2]] == orc.OP_READ)
    # too few IOCBs: contexts beyond n_slots*2048 are neither recorded nor executed
    k[:] = 0
    v[:] = 0
    orc.ring_init(sq, cq)
    _, _, st = orc.retrieve_layer(sq, cq, 0, 1, p, cfg, nb, table, fid, layer, base, 11, store, file_stride, 6, 4)
    assert st == orc.ST_SQE_CAP and int(cq[0]) == 1
    first = np.zeros(N, bool)          # contexts 0..2047: request 0 whole, request 2's K and the head of its V
    n0, n2 = int(nb[0]), int(nb[2])
    k_ids = np.concatenate([table[:n0], table[n0:n0 + n2]])
    v_ids = np.concatenate([table[:n0], table[n0:n0 + (2048 - 2 * n0 - n2)]])
    first[k_ids] = True
    assert np.array_equal(k2[first, :bb], k0r[first, :bb]) and not k2[~first].any()
    vm = np.zeros(N, bool)
    vm[v_ids] = True
    assert np.array_equal(v2[vm, :bb], v0r[vm, :bb]) and not v2[~vm].any()
    # a block id out of range is a no-op context, reported; the others still move
    bad = table.copy()
    bad[5] = N
    k[:] = 0
    v[:] = 0
    orc.ring_init(sq, cq)
    _, _, st = orc.retrieve_layer(sq, cq, 0, 2, p, cfg, nb, bad, fid, layer, base, 11, store, file_stride, 6, 4)
    assert st == orc.ST_BAD_BLOCK
    good = np.zeros(N, bool)
    good[np.delete(table, 5)] = True
    assert np.array_equal(k2[good, :bb], k0r[good, :bb]) and not k2[~good].any()


def _expect_pack(stage, planes, stride, bb, ext, table, live_blocks):
    """Independent formulation of a pack for hand-made extents: numpy gathers, one per live (request, kind, block)."""
    k, v = planes
    for r, kind, j in live_blocks:
        so, ob, toff = int(ext["stage_off"][r]), int(ext["obj_bytes"][r]), int(ext["table_off"][r])
        b = int(table[toff + j])
        src = (k, v)[kind]
        stage[so + kind * ob + j * bb: so + kind * ob + (j + 1) * bb] = src[b * stride: b * stride + bb]


def check_caller_extents(orc, seed=47):
    """Extents written by hand are honoured field by field (a gap between requests, a sub-range of the
    requests, any order in the staging buffer), and what cannot be honoured is skipped and reported.
    Expected bytes come from numpy slices written here, never from orc_obj_layout."""
    rng = np.random.default_rng(seed)
    T, h, d, e, N = 4, 2, 8, 2, 32
    bb = T * h * d * e                    # 128
    A = 128
    stride = bb + 16
    k, v = _planes(rng, N, stride)
    p = _pool(orc, T, h, d, e, N, k, v, stride=stride)
    cfg = orc.make_cfg(A, A, 1)
    n = [3, 2, 4]
    table = rng.permutation(N)[:9].astype(np.uint32)

    def ext_of(rows):
        x = np.zeros(len(rows), orc.EXTENT_DTYPE)
        for i, (so, ob, nb, toff) in enumerate(rows):
            x[i] = (so, ob, nb, 1, 0, toff)
        return x

    def all_blocks(x):
        return [(r, kind, j) for r in range(x.size) for kind in (0, 1) for j in range(int(x["n_blocks"][r]))]

    def run_pack(x, tab=table, cap=None, table_len=None, size=8192, fill=0x6D):
        stage = np.full(size, fill, np.uint8)
        st = orc.obj_pack(p, cfg, x, tab, stage, stage_cap=cap, table_len=table_len)
        return stage, st

    # (a) a gap between the requests, and objects larger than their blocks (padding is zeroed up to obj_bytes)
    x = ext_of([(0, 3 * bb, 3, 0), (2048, 2 * bb + 256, 2, 3), (4096 + 512, 4 * bb, 4, 5)])
    got, st = run_pack(x)
    want = np.full(8192, 0x6D, np.uint8)
    _expect_pack(want, (k, v), stride, bb, x, table, all_blocks(x))
    for kind in (0, 1):
        o = 2048 + kind * (2 * bb + 256)
        want[o + 2 * bb: o + 2 * bb + 256] = 0
    assert st == 0 and np.array_equal(got, want), "gap between requests / padding of a hand-made object"
    # (b) requests 1.. of that layout passed alone, with the whole table: the table range starts at 3
    got, st = run_pack(x[1:])
    want = np.full(8192, 0x6D, np.uint8)
    _expect_pack(want, (k, v), stride, bb, x[1:], table, all_blocks(x[1:]))
    for kind in (0, 1):
        o = 2048 + kind * (2 * bb + 256)
        want[o + 2 * bb: o + 2 * bb + 256] = 0
    assert st == 0 and np.array_equal(got, want), "sub-range of the requests"
    # (c) the last request first in the staging buffer
    y = ext_of([(6 * bb + 8 * bb, 3 * bb, 3, 0), (8 * bb, 2 * bb, 2, 3), (0, 4 * bb, 4, 5)])
    got, st = run_pack(y)
    want = np.full(8192, 0x6D, np.uint8)
    _expect_pack(want, (k, v), stride, bb, y, table, all_blocks(y))
    assert st == 0 and np.array_equal(got, want), "requests in reverse order in the staging buffer"
    # ... and the same three shapes restore what they packed, into another pool, touching nothing else
    for z in (x, x[1:], y):
        stage = rng.integers(0, 256, 8192, dtype=np.uint8)
        k2, v2 = _planes(rng, N, stride)
        kb, vb = k2.copy(), v2.copy()
        p2 = _pool(orc, T, h, d, e, N, k2, v2, stride=stride)
        assert orc.obj_unpack(p2, cfg, z, table, stage) == 0
        for r, kind, j in all_blocks(z):
            so, ob, toff = int(z["stage_off"][r]), int(z["obj_bytes"][r]), int(z["table_off"][r])
            b = int(table[toff + j])
            dst = (kb, vb)[kind]
            dst[b * stride: b * stride + bb] = stage[so + kind * ob + j * bb: so + kind * ob + (j + 1) * bb]
        assert np.array_equal(k2, kb) and np.array_equal(v2, vb), "unpack of hand-made extents"

    # ---- what cannot be honoured
    base = ext_of([(0, 3 * bb, 3, 0), (6 * bb, 2 * bb, 2, 3), (10 * bb, 4 * bb, 4, 5)])
    # the table holds 8 entries but the requests claim 9: the request that crosses the limit is skipped whole
    got, st = run_pack(base, table_len=8)
    want = np.full(8192, 0x6D, np.uint8)
    _expect_pack(want, (k, v), stride, bb, base, table, all_blocks(base[:2]))
    assert st == orc.ST_BAD_EXTENT and np.array_equal(got, want), "running sum of n_blocks beyond table_len"
    # ... and so is every request after it, even one that would fit on its own
    z = ext_of([(0, 3 * bb, 3, 0), (6 * bb, 7 * bb, 7, 0), (20 * bb, bb, 1, 8)])
    got, st = run_pack(z)
    want = np.full(8192, 0x6D, np.uint8)
    _expect_pack(want, (k, v), stride, bb, z, table, all_blocks(z[:1]))
    assert st == orc.ST_BAD_EXTENT and np.array_equal(got, want), "requests after the one that overran the table"
    # an exact fit is fine
    z = ext_of([(0, 9 * bb, 9, 0)])
    got, st = run_pack(z)
    want = np.full(8192, 0x6D, np.uint8)
    _expect_pack(want, (k, v), stride, bb, z, table, all_blocks(z))
    assert st == 0 and np.array_equal(got, want)
    # offsets and sizes must be multiples of 16
    for rows in ([(8, 3 * bb, 3, 0)], [(0, 3 * bb + 8, 3, 0)]):
        got, st = run_pack(ext_of(rows))
        assert st == orc.ST_BAD_EXTENT and np.all(got == 0x6D), "misaligned extent must be skipped"
    got, st = run_pack(ext_of([(16, 3 * bb + 16, 3, 0)]))
    assert st == 0 and np.array_equal(got[16:16 + bb], k[int(table[0]) * stride: int(table[0]) * stride + bb])
    assert np.array_equal(got[16 + 3 * bb + 16: 16 + 4 * bb + 16], v[int(table[0]) * stride: int(table[0]) * stride + bb])
    # sizes that would wrap around 64 bits do not fit any capacity
    for rows in ([(0, 1 << 63, 3, 0)], [((1 << 64) - 16, 3 * bb, 3, 0)], [(4096, (1 << 63) - 2048, 3, 0)]):
        got, st = run_pack(ext_of(rows))
        assert st == orc.ST_STAGE_CAP and np.all(got == 0x6D), "overflowing extent must not fit"
    # an object too small for its blocks: the blocks that still fit are moved, no padding, V right behind K
    z = ext_of([(256, 2 * bb, 3, 0), (256 + 4 * bb + 1024, bb + 64, 2, 3)])
    got, st = run_pack(z)
    want = np.full(8192, 0x6D, np.uint8)
    _expect_pack(want, (k, v), stride, bb, z, table, [(0, 0, 0), (0, 0, 1), (0, 1, 0), (0, 1, 1), (1, 0, 0), (1, 1, 0)])
    assert st == orc.ST_BAD_EXTENT and np.array_equal(got, want), "blocks beyond their object"
    # a table range that runs off the end of the table: the positions beyond it are skipped
    z = ext_of([(0, 3 * bb, 3, 7)])
    longer = np.r_[table, np.uint32(1), np.uint32(2)]
    got, st = run_pack(z, tab=longer, table_len=9)
    want = np.full(8192, 0x6D, np.uint8)
    _expect_pack(want, (k, v), stride, bb, z, table, [(0, 0, 0), (0, 0, 1), (0, 1, 0), (0, 1, 1)])
    assert st == orc.ST_BAD_BLOCK and np.array_equal(got, want), "table position beyond table_len"
    # capacity: the request whose V object ends one byte beyond it is skipped, the others are not
    got, st = run_pack(base, cap=18 * bb - 1)
    want = np.full(8192, 0x6D, np.uint8)
    _expect_pack(want, (k, v), stride, bb, base, table, all_blocks(base[:2]))
    assert st == orc.ST_STAGE_CAP and np.array_equal(got, want)
    got, st = run_pack(base, cap=18 * bb)
    assert st == 0


def check_entry_builders_want_layout_extents(orc, seed=53):
    """The entry builders take extents as obj_layout writes them; anything else: nothing written, BAD_EXTENT."""
    rng = np.random.default_rng(seed)
    T, h, d, e, N, A = 4, 2, 8, 2, 32, 128
    bb = T * h * d * e
    k, v = _planes(rng, N, bb)
    p = _pool(orc, T, h, d, e, N, k, v)
    cfg = orc.make_cfg(A, 2 * A, 2)
    n = np.array([3, 2, 4], np.uint32)
    table = rng.permutation(N)[:9].astype(np.uint32)
    fid = np.array([7, 8, 9], np.uint32)
    ext, tot = orc.obj_layout(p, cfg, n)
    good, st = orc.sqe_build(p, cfg, ext, fid, 1, orc.OP_READ, 4096, 5)
    assert st == 0 and good.size == int(tot[1]) and np.all(good["len"] > 0)
    gd, st = orc.sqe_build_direct(p, cfg, ext, table, fid, 1, orc.OP_WRITE, 1 << 20, 5)
    assert st == 0 and np.all(gd["len"] == bb)

    def variants():
        for field, delta in (("sqe_base", 2), ("table_off", 1), ("obj_bytes", A), ("n_chunks", 1), ("n_blocks", 1)):
            for r in range(3):
                x = ext.copy()
                x[field][r] += delta
                yield f"{field}[{r}]", x, fid
        yield "requests 1.. alone", ext[1:].copy(), fid[1:]
        # one request whose entry count no longer fits 32 bits (2 * 2^31 chunks), everything else consistent
        big, _ = orc.obj_layout(p, cfg, [0xFFFFFFFF])
        assert int(big["n_chunks"][0]) == 1 << 31
        yield "entry count beyond 32 bits", big, fid[:1]

    for name, x, f in variants():
        sqe, st = orc.sqe_build(p, cfg, x, f, 1, orc.OP_READ, 4096, 5, sqe_cap=int(tot[1]))
        assert st == orc.ST_BAD_EXTENT and not sqe.view(np.uint8).any(), f"sqe_build with {name}"
        sqe, st = orc.sqe_build_direct(p, cfg, x, table, f, 1, orc.OP_WRITE, 1 << 20, 5, sqe_cap=18)
        assert st == orc.ST_BAD_EXTENT and not sqe.view(np.uint8).any(), f"sqe_build_direct with {name}"
        sq, cq = orc.ring_alloc(2)
        orc.ring_init(sq, cq)
        before = sq.copy()
        st = orc.iocb_fill_direct(sq, 0, 1, p, cfg, x, table, f, 1, orc.OP_WRITE, 1 << 20, 5)
        assert st == orc.ST_BAD_EXTENT and sq.tobytes() == before.tobytes(), f"iocb_fill_direct with {name}"
    # the staging offset is free: it only moves the addresses
    x = ext.copy()
    x["stage_off"] += 1 << 20
    sqe, st = orc.sqe_build(p, cfg, x, fid, 1, orc.OP_READ, 4096, 5)
    assert st == 0 and np.array_equal(sqe["addr"], good["addr"] + (1 << 20))
    assert np.array_equal(sqe["file_off"], good["file_off"])


def check_visit_order(orc, seed=67):
    """table_order against numpy.argsort; the ordered restore against the plain one for permutations, and against
    numpy slices for lists that are not permutations."""
    rng = np.random.default_rng(seed)
    for _ in range(40):
        N = int(rng.integers(1, 400))
        n = int(rng.integers(0, N + 1))
        t = rng.permutation(N)[:n].astype(np.uint32)
        visit, st = orc.table_order(N, t)
        assert st == 0 and np.array_equal(visit, np.argsort(t, kind="stable").astype(np.uint32))
        assert np.all(np.diff(t[visit].astype(np.int64)) > 0) if n > 1 else True
    t = np.array([5, 2, 9, 2, 7], np.uint32)
    visit, st = orc.table_order(10, t)
    assert st == orc.ST_DUP_BLOCK and np.array_equal(visit, np.arange(5))
    visit, st = orc.table_order(8, np.array([5, 2, 9, 7], np.uint32))
    assert st == orc.ST_BAD_BLOCK and np.array_equal(visit, np.arange(4))
    assert orc.table_order(4, [])[0].size == 0
    # restore: any permutation gives the plain restore's result, entries and extents included
    T, h, d, e, N, A = 4, 2, 8, 2, 64, 128
    bb = T * h * d * e
    for layout in (0, 1):
        n = np.array([5, 0, 9, 3], np.uint32)
        table = rng.permutation(N)[: int(n.sum())].astype(np.uint32)
        fid = np.array([3, 4, 5, 6], np.uint32)
        cfg = orc.make_cfg(A, 2 * A, 3)
        k0, v0 = _planes(rng, N, bb)
        p0 = _pool(orc, T, h, d, e, N, k0, v0, layout=layout)
        ext, tot = orc.obj_layout(p0, cfg, n)
        stage = rng.integers(0, 256, int(tot[0]), dtype=np.uint8)
        ka, va = k0.copy(), v0.copy()
        ea, ta, sa, st_a = orc.layer_restore(_pool(orc, T, h, d, e, N, ka, va, layout=layout), cfg, n, table, fid, 2,
                                             stage, 4096, 7, int(tot[1]))
        for visit in (orc.table_order(N, table)[0], rng.permutation(table.size), np.arange(table.size)[::-1]):
            kb, vb = k0.copy(), v0.copy()
            eb, tb, sb, st_b = orc.layer_restore_ordered(_pool(orc, T, h, d, e, N, kb, vb, layout=layout), cfg, n, table,
                                                         fid, 2, stage, 4096, 7, int(tot[1]), visit)
            assert st_a == st_b == 0 and np.array_equal(ka, kb) and np.array_equal(va, vb)
            assert ea.tobytes() == eb.tobytes() and sa.tobytes() == sb.tobytes() and np.array_equal(ta, tb)
    # a padded pool (the block stride is not the block size) with ids out of range, the first of them num_blocks
    # itself (the planes hold one spare block here): again what the plain restore gives, spare block untouched
    stride = bb + 48
    n = np.array([3, 4], np.uint32)
    table = np.array([9, N, 2, 63, 0, 0xFFFFFFFF, 17], np.uint32)
    cfg = orc.make_cfg(A, 2 * A, 2)
    k0, v0 = _planes(rng, N + 1, stride)
    ext, tot = orc.obj_layout(_pool(orc, T, h, d, e, N, k0, v0, stride=stride), cfg, n)
    stage = rng.integers(0, 256, int(tot[0]), dtype=np.uint8)
    ka, va = k0.copy(), v0.copy()
    ea, ta, sa, st_a = orc.layer_restore(_pool(orc, T, h, d, e, N, ka, va, stride=stride), cfg, n, table, [8, 9], 1,
                                         stage, 0, 0, int(tot[1]))
    kb, vb = k0.copy(), v0.copy()
    eb, tb, sb, st_b = orc.layer_restore_ordered(_pool(orc, T, h, d, e, N, kb, vb, stride=stride), cfg, n, table, [8, 9],
                                                 1, stage, 0, 0, int(tot[1]), np.array([6, 1, 0, 5, 4, 3, 2], np.uint32))
    assert st_a == st_b == orc.ST_BAD_BLOCK and np.array_equal(ka, kb) and np.array_equal(va, vb)
    assert np.array_equal(kb[N * stride:], k0[N * stride:]) and np.array_equal(vb[N * stride:], v0[N * stride:])
    assert not np.array_equal(kb, k0) and not np.array_equal(kb, vb)
    assert sa.tobytes() == sb.tobytes() and np.all(sb["opcode"] == orc.OP_READ)
    # a list that is not a permutation: listed positions are restored, the others are not (NHD: a block is one slice)
    n = np.array([4, 3], np.uint32)
    table = np.array([10, 3, 7, 20, 1, 30, 12], np.uint32)
    cfg = orc.make_cfg(A, A, 1)
    k0, v0 = _planes(rng, N, bb)
    p0 = _pool(orc, T, h, d, e, N, k0, v0)
    ext, tot = orc.obj_layout(p0, cfg, n)
    stage = rng.integers(0, 256, int(tot[0]), dtype=np.uint8)
    visit = np.array([5, 5, 0, 99, 6, 7, 2], np.uint32)       # 1, 3, 4 missing; 5 twice; 99 and 7 out of range
    kb, vb = k0.copy(), v0.copy()
    _, _, _, st = orc.layer_restore_ordered(_pool(orc, T, h, d, e, N, kb, vb), cfg, n, table, [1, 2], 0, stage, 0, 0,
                                            int(tot[1]), visit)
    want_k, want_v = k0.copy(), v0.copy()
    for pos in (5, 0, 6, 2):
        r = 0 if pos < 4 else 1
        j = pos - int(ext["table_off"][r])
        so, ob = int(ext["stage_off"][r]), int(ext["obj_bytes"][r])
        b = int(table[pos])
        want_k[b * bb:(b + 1) * bb] = stage[so + j * bb: so + (j + 1) * bb]
        want_v[b * bb:(b + 1) * bb] = stage[so + ob + j * bb: so + ob + (j + 1) * bb]
    assert st == 0 and np.array_equal(kb, want_k) and np.array_equal(vb, want_v)
    # the table one entry short: the second request does not take part, whatever the list says
    kb, vb = k0.copy(), v0.copy()
    _, _, _, st = orc.layer_restore_ordered(_pool(orc, T, h, d, e, N, kb, vb), cfg, n, table, [1, 2], 0, stage, 0, 0,
                                            int(tot[1]), np.arange(7, dtype=np.uint32), table_len=6)
    want_k, want_v = k0.copy(), v0.copy()
    for pos in range(4):
        b = int(table[pos])
        want_k[b * bb:(b + 1) * bb] = stage[pos * bb:(pos + 1) * bb]
        want_v[b * bb:(b + 1) * bb] = stage[int(ext["obj_bytes"][0]) + pos * bb: int(ext["obj_bytes"][0]) + (pos + 1) * bb]
    assert st == orc.ST_BAD_EXTENT and np.array_equal(kb, want_k) and np.array_equal(vb, want_v)


def check_table_validate(orc, seed=43):
    """Duplicates and out-of-range ids, against numpy.unique on independently built tables."""
    rng = np.random.default_rng(seed)
    assert orc.table_validate(10, []) == 0 and orc.table_validate(1, [0]) == 0
    assert orc.table_validate(1, [0, 0]) == orc.ST_DUP_BLOCK and orc.table_validate(1, [1]) == orc.ST_BAD_BLOCK
    assert orc.table_validate(4, [7, 7]) == orc.ST_BAD_BLOCK            # out of range twice is not a duplicate
    assert orc.table_validate(4, [3, 9, 3]) == (orc.ST_BAD_BLOCK | orc.ST_DUP_BLOCK)
    for _ in range(200):
        N = int(rng.integers(1, 300))
        n = int(rng.integers(0, 400))
        t = rng.integers(0, N + int(rng.integers(0, 3)), size=n).astype(np.uint32)
        ok = t[t < N]
        want = (orc.ST_BAD_BLOCK if (t >= N).any() else 0) | (orc.ST_DUP_BLOCK if np.unique(ok).size != ok.size else 0)
        assert orc.table_validate(N, t) == want, (N, t)
        assert orc.table_validate(N, rng.permutation(N)[: min(n, N)]) == 0    # a permutation prefix is always clean
    # first and last entry equal, ids at the ends of the range
    assert orc.table_validate(65536, np.r_[np.arange(65535, 0, -1), 65535].astype(np.uint32)) == orc.ST_DUP_BLOCK
    assert orc.table_validate(65536, np.arange(65536, dtype=np.uint32)) == 0


ALL_CHECKS = [check_paper_counts, check_closed_forms_8b, check_abi, check_layout_scan, check_pack_bruteforce,
              check_pack_vs_numpy, check_address_tags, check_roundtrip_and_untouched, check_skips_and_status,
              check_sqe_fields, check_layer_restore, check_threaded, check_sgl_table, check_direct_entries, check_ring_fill, check_issue_io, check_issue_io_hand_filled,
              check_ring_layer, check_table_validate, check_caller_extents,
              check_entry_builders_want_layout_extents, check_visit_order]
