"""GPU parity tests: every entry point of libtutti, called through the C ABI, byte-for-byte against
the CPU oracle on the same seeded inputs.  Integer / byte work, so the bar is exact equality."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

from paper_2605_03375_amd import binding as B      # noqa: E402
from paper_2605_03375_amd import workloads as W    # noqa: E402


@pytest.fixture(scope="module")
def H():
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU: run with -m 'not gpu' on a CPU-only machine")
    B.lib()  # fails loudly if the HIP library is not built: there is no fallback
    import gpu_harness
    return gpu_harness


@pytest.fixture
def knobs():
    """For tests of the measurement library: the ordinary entry points go through libtutti_bench.so (the same
    sources plus tuning knobs and every launch shape) while the test runs; everything is put back afterwards.
    All other tests run the product library, which has no knobs."""
    B.use_bench_library(True)
    yield
    B.tutti_set_tuning(0, 0)
    B.tutti_set_nontemporal(3)
    B.tutti_set_hnd_mode(0)
    B.tutti_set_xcd_mapping(0)
    B.use_bench_library(False)


def say(*a):
    print(*a, flush=True)


# ------------------------------------------------------------------ config 1: Tiny

@pytest.mark.parametrize("layout", [0, 1], ids=["nhd", "hnd"])
@pytest.mark.parametrize("fill", ["values", "tags"])
@pytest.mark.parametrize("chunk", [2 << 20, 4096])
def test_cfg1_tiny(orc, H, layout, fill, chunk):
    w = W.tiny(chunk_bytes=chunk)
    say("cfg1", layout, fill, chunk)
    c = H.LayerCase.from_workload(w, layout=layout, fill=fill)
    H.check_everything(orc, c)


# ------------------------------------------------------------------ shapes that span tiles and leave ragged tails

RAGGED = [
    # T, h, d, e, N, n_blocks, align, chunk, pad
    (16, 5, 40, 2, 300, [7, 0, 33, 1, 64, 2], 4096, 12288, 0),      # block 6400 B: ragged slice, padded objects
    (16, 8, 128, 2, 512, [100, 3, 0, 0, 129], 4096, 2 << 20, 0),    # the 8B block shape
    (16, 8, 128, 2, 128, [17, 40], 4096, 32768, 4096),              # strided pool, one entry per block
    (3, 1, 8, 2, 64, [1, 2, 3, 4, 5, 6, 7, 8], 64, 192, 16),        # 48-byte blocks
    (32, 4, 64, 1, 256, [0, 0, 5, 0, 200], 512, 8192, 0),           # fp8-sized elements, empty requests first
    (16, 1, 128, 2, 1024, [1000], 4096, 4096, 0),                   # TP-sharded shape: 4 KiB blocks at scale
    (64, 8, 128, 2, 96, [31, 33], 4096, 131072, 0),                 # 64-token blocks (128 KiB)
]


@pytest.mark.parametrize("layout", [0, 1], ids=["nhd", "hnd"])
@pytest.mark.parametrize("shape", RAGGED, ids=[f"bb{t*h*d*e}_r{len(n)}" for t, h, d, e, _, n, *_ in RAGGED])
def test_ragged_shapes(orc, H, shape, layout):
    T, h, d, e, N, n_blocks, A, C, pad = shape
    say("ragged", shape, layout)
    rng = np.random.default_rng(1234 + T * h)
    table = rng.permutation(N)[: sum(n_blocks)]
    c = H.LayerCase(T=T, h=h, d=d, e=e, N=N, n_blocks=n_blocks, table=table, align=A, chunk=C, L=3, layout=layout,
                    pad=pad, seed=T + h, name=f"ragged{shape}")
    H.check_everything(orc, c)


@pytest.mark.parametrize("unroll", [1, 2, 4, 8])
@pytest.mark.parametrize("nt", [0, 1, 2, 3])
def test_launch_tuning_does_not_change_results(orc, H, knobs, unroll, nt):
    say("tuning", unroll, nt)
    B.tutti_set_tuning(3, unroll)
    B.tutti_set_nontemporal(nt)
    rng = np.random.default_rng(77)
    for layout in (0, 1):
        c = H.LayerCase(T=16, h=5, d=40, e=2, N=200, n_blocks=[9, 0, 70, 31], table=rng.permutation(200)[:110],
                        align=4096, chunk=8192, L=2, layout=layout, name=f"tuning{unroll}")
        H.check_everything(orc, c)


# ------------------------------------------------------------------ head-major pools: direct copy and LDS-staged transpose

HND_SHAPES = [
    # T, h, d, e, N, n_blocks, chunk
    (16, 64, 16, 2, 300, [40, 0, 7, 129], 2 << 20),   # 32-byte rows: one 32 KiB tile per block
    (16, 32, 32, 2, 300, [3, 90, 1], 32768),          # 64-byte rows
    (16, 8, 128, 2, 300, [64, 65], 2 << 20),          # 256-byte rows (the 8B shape)
    (64, 8, 128, 2, 64, [9, 20], 131072),             # 128 KiB blocks: four tiles per block
    (16, 2, 64, 2, 256, [32, 5], 4096),               # Tiny's block: a 4 KiB tile
    (4, 4, 8, 2, 64, [10, 3], 4096),                  # 16-byte rows, tile too small for LDS: direct copy
    (16, 6, 32, 2, 128, [11, 12], 8192),              # head count not a power of two: direct copy
    (32, 16, 64, 1, 200, [17, 0, 60], 16384),         # one-byte elements, 64-byte rows
]


@pytest.mark.parametrize("mode", [0, 1, 2], ids=["auto", "direct", "lds"])
@pytest.mark.parametrize("shape", HND_SHAPES, ids=[f"T{t}h{h}d{d}e{e}" for t, h, d, e, *_ in HND_SHAPES])
def test_head_major_paths(orc, H, request, shape, mode):
    T, h, d, e, N, n_blocks, C = shape
    say("hnd", shape, "mode", mode)
    if mode:      # forcing a path is a knob of the measurement library; "auto" is the product choosing by shape
        request.getfixturevalue("knobs")
        B.tutti_set_hnd_mode(mode)
    rng = np.random.default_rng(500 + T + h)
    c = H.LayerCase(T=T, h=h, d=d, e=e, N=N, n_blocks=n_blocks, table=rng.permutation(N)[: sum(n_blocks)], chunk=C, L=2,
                    layout=1, seed=h, name=f"hnd{shape}m{mode}")
    H.check_everything(orc, c)
    H.check_everything(orc, c, cu_budget=3)


def test_head_major_lds_edge_cases(orc, H):
    """Bad ids, a small staging buffer and the 2048-request limit through the LDS-staged path."""
    say("hnd lds edges")
    table = np.array([3, 999, 5, 16, 7, 1], np.uint32)
    c = H.LayerCase(T=16, h=32, d=32, e=2, N=16, n_blocks=[4, 2], table=table, layout=1, name="hnd_bad_ids")
    ext, tot, o_ext, o_tot = H.check_layout(orc, c)
    H.check_pack(orc, c, ext, o_ext, o_tot)
    H.check_unpack(orc, c, ext, o_ext, o_tot)
    H.check_layer_restore(orc, c)
    cap = int(o_ext["stage_off"][1]) + 4096
    H.check_pack(orc, c, ext, o_ext, o_tot, stage_cap=cap)
    H.check_layer_restore(orc, c, stage_cap=cap, sqe_cap=1)
    rng = np.random.default_rng(6)
    n = rng.integers(0, 3, size=B.MAX_REQ).astype(np.uint32)
    N = int(n.sum()) + 9
    c = H.LayerCase(T=16, h=16, d=16, e=2, N=N, n_blocks=n, table=rng.permutation(N)[: int(n.sum())], chunk=8192,
                    layout=1, name="hnd_max_req")   # 2048 requests: no LDS left for a tile, falls back to direct
    H.check_everything(orc, c)
    c = H.LayerCase(T=16, h=16, d=16, e=2, N=N, n_blocks=n[:700], table=rng.permutation(N)[: int(n[:700].sum())],
                    chunk=8192, layout=1, name="hnd_700_req")
    H.check_everything(orc, c)


# ------------------------------------------------------------------ direct-to-block mode (no staging copy)

def test_direct_mode_small_shapes(orc, H):
    say("direct mode: small shapes")
    rng = np.random.default_rng(31)
    for T, h, d, e, N, nb, A, pad in [(16, 2, 64, 2, 256, [32], 4096, 0), (16, 8, 128, 2, 500, [6, 0, 40, 1, 13], 4096, 0),
                                      (4, 4, 16, 2, 100, [9, 9, 0, 30], 256, 256), (16, 1, 128, 2, 3000, [2500], 4096, 0)]:
        bb = T * h * d * e
        c = H.LayerCase(T=T, h=h, d=d, e=e, N=N, n_blocks=nb, table=rng.permutation(N)[: sum(nb)], align=A, chunk=bb,
                        L=9, pad=pad, name=f"direct_bb{bb}")
        H.check_direct_mode(orc, c, layer=8)
    # out-of-range ids, a short table, small capacities
    c = H.LayerCase(T=16, h=2, d=64, e=2, N=16, n_blocks=[4, 2], table=[3, 999, 5, 16, 7, 1], chunk=4096, name="direct_bad")
    H.check_direct_mode(orc, c)
    H.check_direct_mode(orc, c, table_len=4)
    H.check_direct_mode(orc, c, sqe_cap=5)
    H.check_direct_mode(orc, c, sqe_cap=0)
    c = H.LayerCase(T=16, h=2, d=64, e=2, N=16, n_blocks=[0, 0], table=[], chunk=4096, name="direct_empty")
    H.check_direct_mode(orc, c)


def test_direct_mode_cfg3_and_cfg4(orc, H):
    """Per-block entries at the scale the paper cares about: 81,438 per layer (config 3), 16,384 (config 4)."""
    w = W.batch64_zipf(chunk_bytes=32768)
    say("direct mode cfg3", int(w.n_blocks.sum()))
    # planes are never touched in this mode: a small stand-in pool keeps the test light
    c = H.LayerCase.from_workload(w)
    H.check_direct_mode(orc, c, layer=31)
    w = W.llama70b_128k()
    say("direct mode cfg4")
    c = H.LayerCase.from_workload(w)
    H.check_direct_mode(orc, c, layer=79)


# ------------------------------------------------------------------ staging buffer in pinned host memory

def test_pinned_host_staging(orc, H):
    """The staging buffer may live in pinned host memory (the closer stand-in for the SSD leg: the
    copy then crosses the host link).  Same calls, same bytes."""
    say("pinned-host staging")
    w = W.llama8b_32k(num_blocks=2048, tokens=4096)
    c = H.LayerCase.from_workload(w)
    o_ext, o_tot = orc.obj_layout(c.orc_pool(orc), c.orc_cfg(orc), c.n_blocks)
    nbytes = int(o_tot[0])
    stage = torch.empty(nbytes, dtype=torch.uint8, pin_memory=True)
    stage.fill_(0xA5)
    ext, tot = H.gpu_layout(c)
    st = H.new_status()
    B.tutti_obj_pack(c.gpu_pool(), c.gpu_cfg(), ext, c.n_req, c.d_table, c.table.size, stage, nbytes, 0, st)
    torch.cuda.synchronize()
    o_stage = np.full(nbytes, 0xA5, np.uint8)
    orc.obj_pack(c.orc_pool(orc), c.orc_cfg(orc), o_ext, c.table, o_stage)
    assert np.array_equal(stage.numpy(), o_stage) and int(st.item()) == 0
    # restore from pinned memory into a zeroed pool
    k2, v2 = torch.zeros_like(c.k_dev), torch.zeros_like(c.v_dev)
    sqe = torch.zeros(64 * int(o_tot[1]), dtype=torch.uint8, device=H.DEV)
    B.tutti_layer_restore(c.gpu_pool(k2, v2), c.gpu_cfg(), c.d_n_blocks, c.n_req, c.d_table, c.table.size, c.d_file_id,
                          3, stage, nbytes, stage.data_ptr(), 1, ext, tot, sqe, int(o_tot[1]), 0, st)
    torch.cuda.synchronize()
    ok, ov = np.zeros_like(c.k_host), np.zeros_like(c.v_host)
    orc.obj_unpack(c.orc_pool(orc, ok, ov), c.orc_cfg(orc), o_ext, c.table, o_stage)
    assert np.array_equal(k2.cpu().numpy(), ok) and np.array_equal(v2.cpu().numpy(), ov) and int(st.item()) == 0


def test_interleaved_kv_pool(orc, H):
    """One buffer holding [num_blocks][K|V][T][h][d] (the layout of engines that keep a block's K and V side by
    side): k_base = buffer, v_base = buffer + block_bytes, block_stride = 2 * block_bytes."""
    say("interleaved K/V pool")
    rng = np.random.default_rng(12)
    T, h, d, e, N = 16, 8, 128, 2, 300
    bb = T * h * d * e
    nb = np.array([50, 0, 71], np.uint32)
    table = rng.permutation(N)[: int(nb.sum())].astype(np.uint32)
    fid = np.array([1, 2, 3], np.uint32)
    buf = H.as_u8(W.device_values(99, N * 2 * bb // 2, "bf16", H.DEV))
    host = buf.cpu().numpy()
    geom = dict(num_blocks=N, block_tokens=T, num_kv_heads=h, head_dim=d, elt_bytes=e, block_stride=2 * bb)
    pool = B.make_pool(buf, buf.data_ptr() + bb, **geom)
    cfg = B.make_cfg(4096, 1 << 20, 2)
    o_pool = orc.make_pool(host, None, **geom)
    o_pool.v_base = host.ctypes.data + bb
    ocfg = orc.make_cfg(4096, 1 << 20, 2)
    o_ext, o_tot = orc.obj_layout(o_pool, ocfg, nb)
    n_sqe = int(o_tot[1])
    d_n, d_tab, d_fid = H.to_dev(nb), H.to_dev(table), H.to_dev(fid)
    ext = torch.zeros(32 * 3, dtype=torch.uint8, device=H.DEV)
    tot = torch.zeros(2, dtype=torch.int64, device=H.DEV)
    sqe = torch.zeros(64 * n_sqe, dtype=torch.uint8, device=H.DEV)
    stage = torch.zeros(int(o_tot[0]), dtype=torch.uint8, device=H.DEV)
    st = H.new_status()
    B.tutti_layer_save(pool, cfg, d_n, 3, d_tab, table.size, d_fid, 1, stage, stage.numel(), stage.data_ptr(), 0, ext, tot,
                       sqe, n_sqe, 0, st)
    torch.cuda.synchronize()
    o_stage = np.zeros(int(o_tot[0]), np.uint8)
    orc.obj_pack(o_pool, ocfg, o_ext, table, o_stage)
    assert np.array_equal(stage.cpu().numpy(), o_stage)
    # restore different bytes into the same interleaved buffer
    g = torch.Generator(device=H.DEV)
    g.manual_seed(4)
    stage2 = torch.randint(0, 256, (int(o_tot[0]),), dtype=torch.uint8, device=H.DEV, generator=g)
    B.tutti_layer_restore(pool, cfg, d_n, 3, d_tab, table.size, d_fid, 1, stage2, stage2.numel(), stage2.data_ptr(), 0,
                          ext, tot, sqe, n_sqe, 0, st)
    torch.cuda.synchronize()
    orc.obj_unpack(o_pool, ocfg, o_ext, table, stage2.cpu().numpy())
    assert np.array_equal(buf.cpu().numpy(), host) and int(st.item()) == 0


def test_paper_block_sizes(orc, H):
    """Token counts per block the paper mentions: 16-32 in general (sec. 2.1), 64 in its evaluation (sec. 4)."""
    rng = np.random.default_rng(64)
    for T in (32, 64):
        say("block tokens", T)
        N = 400
        nb = [70, 0, 33]
        c = H.LayerCase(T=T, h=8, d=128, e=2, N=N, n_blocks=nb, table=rng.permutation(N)[: sum(nb)], chunk=2 << 20,
                        L=32, name=f"T{T}")
        H.check_everything(orc, c)
        c = H.LayerCase(T=T, h=8, d=128, e=2, N=N, n_blocks=nb, table=rng.permutation(N)[: sum(nb)],
                        chunk=T * 8 * 128 * 2, L=32, name=f"T{T}_direct")
        H.check_direct_mode(orc, c, layer=31)


# ------------------------------------------------------------------ HIP graph capture

def test_layer_calls_can_be_captured_in_a_graph(orc, H):
    """The per-layer calls allocate nothing and never synchronise, so a train of them can be captured in a
    HIP graph (no memset nodes are recorded).  Every replay must reproduce the eager result, with eager
    work and synchronisation between the replays."""
    say("graph capture")
    rng = np.random.default_rng(55)
    nb = [40, 0, 25]
    N = 256
    cases = [H.LayerCase(T=16, h=8, d=128, e=2, N=N, n_blocks=nb, table=rng.permutation(N)[: sum(nb)], chunk=65536, L=4,
                         seed=10 + l, name=f"graph{l}") for l in range(4)]
    c0 = cases[0]
    o_ext, o_tot = orc.obj_layout(c0.orc_pool(orc), c0.orc_cfg(orc), c0.n_blocks)
    nbytes, n_sqe = int(o_tot[0]), int(o_tot[1])
    stages = [torch.zeros(nbytes, dtype=torch.uint8, device=H.DEV) for _ in cases]
    k2 = [torch.zeros_like(c.k_dev) for c in cases]
    v2 = [torch.zeros_like(c.v_dev) for c in cases]
    ext = torch.zeros(len(cases), 32 * c0.n_req, dtype=torch.uint8, device=H.DEV)
    tot = torch.zeros(len(cases), 2, dtype=torch.int64, device=H.DEV)
    wsqe = torch.zeros(len(cases), n_sqe * 64, dtype=torch.uint8, device=H.DEV)
    rsqe = torch.zeros(len(cases), n_sqe * 64, dtype=torch.uint8, device=H.DEV)
    st = H.new_status()

    def train():   # save every layer from its pool, then restore it into a second pool
        for l, c in enumerate(cases):
            B.tutti_layer_save(c.gpu_pool(), c.gpu_cfg(), c.d_n_blocks, c.n_req, c.d_table, c.table.size, c.d_file_id, l,
                               stages[l], nbytes, stages[l].data_ptr(), 2, ext[l], tot[l], wsqe[l], n_sqe, 0, st)
        for l, c in enumerate(cases):
            B.tutti_layer_restore(c.gpu_pool(k2[l], v2[l]), c.gpu_cfg(), c.d_n_blocks, c.n_req, c.d_table, c.table.size,
                                  c.d_file_id, l, stages[l], nbytes, stages[l].data_ptr(), 2, ext[l], tot[l], rsqe[l],
                                  n_sqe, 0, st)

    def snapshot():
        torch.cuda.synchronize()
        return [t.clone() for t in stages + k2 + v2] + [ext.clone(), tot.clone(), wsqe.clone(), rsqe.clone()]

    def clear():
        for t in stages + k2 + v2 + [ext, tot, wsqe, rsqe]:
            t.zero_()

    train()                                   # eager (also warms up the one-time device query)
    eager = snapshot()
    # the eager result is the oracle's
    for l, c in enumerate(cases):
        o_stage = np.zeros(nbytes, np.uint8)
        orc.obj_pack(c.orc_pool(orc), c.orc_cfg(orc), o_ext, c.table, o_stage)
        assert np.array_equal(stages[l].cpu().numpy(), o_stage)
    clear()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            train()
    torch.cuda.synchronize()
    for rep in range(3):
        clear()
        junk = torch.randn(512, 512, device=H.DEV) @ torch.randn(512, 512, device=H.DEV)   # eager work in between
        torch.cuda.synchronize()
        graph.replay()
        got = snapshot()
        for a, b in zip(eager, got):
            assert torch.equal(a, b), f"graph replay {rep} differs from the eager result"
        assert torch.isfinite(junk).all() and int(st.item()) == 0


def test_ring_layer_calls_can_be_captured_in_a_graph(orc, H):
    """init_queue, store_layer for every layer, then retrieve_layer into a second pool, captured once and replayed:
    every replay must leave the rings, the file store and the second pool as the eager run did."""
    say("graph capture: rings")
    rng = np.random.default_rng(57)
    nb = [600, 0, 500]                                   # 2200 contexts: two IOCBs per layer
    N, L = 1200, 3
    c = H.LayerCase(T=16, h=2, d=64, e=2, N=N, n_blocks=nb, table=rng.permutation(N)[: sum(nb)], chunk=4096, L=L,
                    name="graph_rings")
    o_ext, _ = orc.obj_layout(c.orc_pool(orc), c.orc_cfg(orc), c.n_blocks)
    file_stride = int(2 * L * int(o_ext["obj_bytes"].max()))
    store = torch.zeros(c.n_req * file_stride, dtype=torch.uint8, device=H.DEV)
    fs = B.make_filestore(store, file_stride, 1000, c.n_req)
    k2, v2 = torch.zeros_like(c.k_dev), torch.zeros_like(c.v_dev)
    depth = 4 * L
    sq_bytes, cq_bytes = B.ring_bytes(depth)
    sq = torch.zeros(sq_bytes, dtype=torch.uint8, device=H.DEV)
    cq = torch.zeros(cq_bytes, dtype=torch.uint8, device=H.DEV)
    ring = B.make_ring(sq, cq, depth)
    ext = torch.zeros(32 * c.n_req, dtype=torch.uint8, device=H.DEV)
    tot = torch.zeros(2, dtype=torch.int64, device=H.DEV)
    st = H.new_status()
    addr = 0x7f00_0000_3000

    def train():
        B.tutti_ring_init(ring)
        for l in range(L):
            B.tutti_store_layer(ring, 2 * l, 2, c.gpu_pool(), c.gpu_cfg(), c.d_n_blocks, c.n_req, c.d_table, c.table.size,
                                c.d_file_id, l, addr, 3, fs, ext, tot, 0, st)
        for l in range(L):
            B.tutti_retrieve_layer(ring, 2 * L + 2 * l, 2, c.gpu_pool(k2, v2), c.gpu_cfg(), c.d_n_blocks, c.n_req,
                                   c.d_table, c.table.size, c.d_file_id, l, addr, 3, fs, ext, tot, 0, st)

    outs = [store, k2, v2, sq, cq, ext, tot]

    def snapshot():
        torch.cuda.synchronize()
        return [t.clone() for t in outs]

    train()
    eager = snapshot()
    # the eager result is the oracle's: same calls on host copies
    o_store = np.zeros(store.numel(), np.uint8)
    ok2, ov2 = np.zeros_like(c.k_host), np.zeros_like(c.v_host)
    o_sq, o_cq = orc.ring_alloc(depth)
    orc.ring_init(o_sq, o_cq)
    for l in range(L):
        orc.store_layer(o_sq, o_cq, 2 * l, 2, c.orc_pool(orc), c.orc_cfg(orc), c.n_blocks, c.table, c.file_id, l, addr, 3,
                        o_store, file_stride, 1000, c.n_req)
    for l in range(L):
        orc.retrieve_layer(o_sq, o_cq, 2 * L + 2 * l, 2, c.orc_pool(orc, ok2, ov2), c.orc_cfg(orc), c.n_blocks, c.table,
                           c.file_id, l, addr, 3, o_store, file_stride, 1000, c.n_req)
    assert np.array_equal(store.cpu().numpy(), o_store) and np.array_equal(k2.cpu().numpy(), ok2)
    assert np.array_equal(v2.cpu().numpy(), ov2) and sq.cpu().numpy().tobytes() == o_sq.tobytes()
    assert cq.cpu().numpy().tobytes() == o_cq.tobytes() and int(o_cq[0]) == 4 * L
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            train()
    torch.cuda.synchronize()
    for rep in range(3):
        for t in outs:
            t.zero_()
        junk = torch.randn(512, 512, device=H.DEV) @ torch.randn(512, 512, device=H.DEV)
        torch.cuda.synchronize()
        graph.replay()
        got = snapshot()
        for a, b in zip(eager, got):
            assert torch.equal(a, b), f"graph replay {rep} differs from the eager result"
        assert torch.isfinite(junk).all() and int(st.item()) == 0


# ------------------------------------------------------------------ seeded random shapes

import os as _os


@pytest.mark.parametrize("seed", range(int(_os.environ.get("TUTTI_FUZZ_SEEDS", "160"))))
def test_random_shapes(orc, H, request, seed):
    """Seeded random geometry, request mix, layout, stride, alignment, chunking and launch shape."""
    rng = np.random.default_rng(9000 + seed)
    e = int(rng.choice([1, 2, 4]))
    d = int(rng.choice([16, 32, 40, 64, 80, 128])) if e > 1 else int(rng.choice([16, 32, 48, 64, 128]))
    h = int(rng.choice([1, 2, 3, 4, 5, 8, 16]))
    T = int(rng.choice([1, 4, 8, 16, 32]))
    bb = T * h * d * e
    A = int(rng.choice([64, 512, 4096]))
    C = A * int(rng.integers(1, 40))
    pad = int(rng.choice([0, 0, 16, 4096]))
    layout = int(rng.integers(0, 2))
    R = int(rng.choice([1, 2, 5, 17, 64, 100]))
    nb = rng.integers(0, max(2, 600 // R), size=R)
    nb[rng.integers(0, R)] = 0
    N = int(nb.sum()) + int(rng.integers(1, 50))
    unroll = int(rng.choice([1, 2, 4, 8]))
    wgs = int(rng.choice([1, 2, 8]))
    budget = int(rng.choice([0, 0, 1, 5]))
    hnd_mode = int(rng.integers(0, 3))
    tuned = bool(seed % 3)        # two seeds in three also vary the launch shape, through the measurement library
    say("random", dict(seed=seed, T=T, h=h, d=d, e=e, bb=bb, A=A, C=C, pad=pad, layout=layout, R=R, blocks=int(nb.sum()),
                       N=N, budget=budget, **(dict(unroll=unroll, wgs=wgs, hnd_mode=hnd_mode) if tuned else {})))
    if tuned:
        request.getfixturevalue("knobs")
        B.tutti_set_tuning(wgs, unroll)
        B.tutti_set_hnd_mode(hnd_mode)
    c = H.LayerCase(T=T, h=h, d=d, e=e, N=N, n_blocks=nb, table=rng.permutation(N)[: int(nb.sum())], align=A, chunk=C,
                    L=int(rng.integers(1, 90)), layout=layout, pad=pad, seed=seed, name=f"random{seed}")
    H.check_everything(orc, c, cu_budget=budget)
    # the restore again with the blocks visited in a random order; on token-major pools (where the list is always
    # read) some positions are out of range, listed twice or missing
    n = int(nb.sum())
    visit = rng.permutation(n).astype(np.uint32)
    if layout == 0 and n > 4:
        visit[rng.integers(0, n, size=3)] = [n, 0xFFFFFFFF, visit[0]]
    H.check_layer_restore(orc, c, layer=0, cu_budget=budget, visit=visit, seed=seed)
    if bb % A == 0:
        H.check_direct_mode(orc, c, layer=c.L - 1)
        # the one-call ring path on the same shape (two layers' worth of file, if that stays small)
        c.L = 2
        n_slots = (2 * int(nb.sum()) + B.IOCB_SLOTS - 1) // B.IOCB_SLOTS
        if 2 * c.L * int(nb.max()) * bb * R <= (512 << 20):
            H.check_ring_layer(orc, c, layer=1, write=bool(seed & 1), depth=n_slots + 1,
                               first_slot=seed % (n_slots + 1), n_slots=n_slots, cu_budget=budget)


# ------------------------------------------------------------------ rings: fill IOCBs, execute them, completions

def test_rings_small(orc, H):
    say("rings: small")
    rng = np.random.default_rng(41)
    # 5000 contexts over three IOCBs, wrapping around the end of a ring of 8
    nb = [1500, 0, 1000]
    N = 2600
    c = H.LayerCase(T=16, h=2, d=64, e=2, N=N, n_blocks=nb, table=rng.permutation(N)[: sum(nb)], chunk=4096, L=3,
                    name="rings5000")
    for op in (B.OP_READ, B.OP_WRITE):
        assert H.check_rings(orc, c, layer=1, opcode=op, depth=8, first_slot=6, n_slots=4) == 4
    H.check_rings(orc, c, layer=2, opcode=B.OP_READ, depth=8, first_slot=0, n_slots=2)          # too few IOCBs
    H.check_rings(orc, c, layer=0, opcode=B.OP_READ, depth=4, first_slot=3, n_slots=3, cu_budget=2)
    H.check_rings(orc, c, layer=0, opcode=B.OP_WRITE, depth=4, first_slot=1, n_slots=3, cu_budget=1)
    # descriptors cut off (V plane unknown), unknown file ids, files too short: skipped and reported
    H.check_rings(orc, c, layer=0, opcode=B.OP_READ, depth=4, first_slot=0, n_slots=3, n_desc=N)
    H.check_rings(orc, c, layer=0, opcode=B.OP_READ, depth=4, first_slot=0, n_slots=3, first_file_id=1001)
    H.check_rings(orc, c, layer=2, opcode=B.OP_WRITE, depth=4, first_slot=0, n_slots=3, stride_cut=4096)
    # out-of-range block ids give no-op contexts; an empty layer completes its IOCBs at once
    c = H.LayerCase(T=16, h=2, d=64, e=2, N=16, n_blocks=[4, 2], table=[3, 999, 5, 16, 7, 1], chunk=4096, name="rings_bad")
    H.check_rings(orc, c, layer=0, opcode=B.OP_READ, depth=2, first_slot=1, n_slots=1)
    c = H.LayerCase(T=16, h=2, d=64, e=2, N=16, n_blocks=[0], table=[], chunk=4096, name="rings_empty")
    assert H.check_rings(orc, c, layer=0, opcode=B.OP_READ, depth=2, first_slot=0, n_slots=2) == 2
    # strided pool and 128 KiB blocks (several slices per context)
    c = H.LayerCase(T=64, h=8, d=128, e=2, N=64, n_blocks=[9, 20], table=rng.permutation(64)[:29], chunk=131072, L=2,
                    pad=4096, name="rings_128K")
    H.check_rings(orc, c, layer=1, opcode=B.OP_READ, depth=3, first_slot=2, n_slots=1)
    H.check_rings(orc, c, layer=1, opcode=B.OP_WRITE, depth=3, first_slot=2, n_slots=1, cu_budget=4)


def test_rings_cfg2_layer(orc, H):
    """The paper's data path on config 2's layer: 4096 contexts = two full IOCBs, restore straight from the
    file store into the scattered blocks (no staging copy)."""
    w = W.llama8b_32k(num_blocks=8192)
    say("rings: config 2 layer")
    c = H.LayerCase.from_workload(w)
    c.chunk = c.bb
    for op in (B.OP_READ, B.OP_WRITE):
        assert H.check_rings(orc, c, layer=31, opcode=op, depth=4, first_slot=3, n_slots=2) == 2


def test_ring_layer_small(orc, H, request):
    """retrieve_layer / store_layer in one call against the oracle's layout + fill + issue sequence."""
    say("ring layer: small")
    rng = np.random.default_rng(43)
    nb = [1500, 0, 1000]
    N = 2600
    c = H.LayerCase(T=16, h=2, d=64, e=2, N=N, n_blocks=nb, table=rng.permutation(N)[: sum(nb)], chunk=4096, L=3,
                    name="ringlayer5000")
    for write in (False, True):
        assert H.check_ring_layer(orc, c, layer=1, write=write, depth=8, first_slot=6, n_slots=4) == 0
        assert H.check_ring_layer(orc, c, layer=2, write=write, depth=8, first_slot=0, n_slots=2) == B.ST_SQE_CAP
        assert H.check_ring_layer(orc, c, layer=0, write=write, depth=4, first_slot=3, n_slots=3, cu_budget=2) == 0
        assert H.check_ring_layer(orc, c, layer=0, write=write, depth=4, first_slot=1, n_slots=3, cu_budget=1) == 0
        H.check_ring_layer(orc, c, layer=0, write=write, depth=4, first_slot=1, n_slots=3, prefill=True)
        # unknown file ids, files too short, no IOCBs at all: skipped and reported
        assert H.check_ring_layer(orc, c, layer=0, write=write, depth=4, first_slot=0, n_slots=3,
                                  first_file_id=1001) == B.ST_BAD_BLOCK
        assert H.check_ring_layer(orc, c, layer=0, write=write, depth=4, first_slot=0, n_slots=3, n_files=2) == B.ST_BAD_BLOCK
        assert H.check_ring_layer(orc, c, layer=2, write=write, depth=4, first_slot=0, n_slots=3,
                                  stride_cut=4096) == B.ST_BAD_BLOCK
        assert H.check_ring_layer(orc, c, layer=1, write=write, depth=4, first_slot=2, n_slots=0) == B.ST_SQE_CAP
    H.check_rings(orc, c, layer=0, opcode=B.OP_READ, depth=4, first_slot=0, n_slots=0)
    c = H.LayerCase(T=16, h=2, d=64, e=2, N=16, n_blocks=[4, 2], table=[3, 999, 5, 16, 7, 1], chunk=4096,
                    name="ringlayer_bad")
    for write in (False, True):
        assert H.check_ring_layer(orc, c, layer=0, write=write, depth=2, first_slot=1, n_slots=1) == B.ST_BAD_BLOCK
    c = H.LayerCase(T=16, h=2, d=64, e=2, N=16, n_blocks=[0], table=[], chunk=4096, name="ringlayer_empty")
    assert H.check_ring_layer(orc, c, layer=0, write=False, depth=2, first_slot=0, n_slots=2) == 0
    c = H.LayerCase(T=16, h=2, d=64, e=2, N=16, n_blocks=[], table=[], chunk=4096, name="ringlayer_noreq")
    assert H.check_ring_layer(orc, c, layer=0, write=True, depth=2, first_slot=1, n_slots=1) == 0
    # strided pool, 128 KiB blocks, head-major pool (blocks travel as raw bytes), unroll 1 and 2 (ragged slices)
    for layout in (0, 1):
        c = H.LayerCase(T=64, h=8, d=128, e=2, N=64, n_blocks=[9, 20], table=rng.permutation(64)[:29], chunk=131072,
                        L=2, pad=4096, layout=layout, name=f"ringlayer_128K_{layout}")
        for write in (False, True):
            H.check_ring_layer(orc, c, layer=1, write=write, depth=3, first_slot=2, n_slots=1)
            H.check_ring_layer(orc, c, layer=1, write=write, depth=3, first_slot=2, n_slots=1, cu_budget=4)
    c = H.LayerCase(T=3, h=2, d=256, e=2, N=40, n_blocks=[11, 5], table=rng.permutation(40)[:16], align=1024,
                    chunk=3072, L=2, name="ringlayer_3K")
    for write in (False, True):
        H.check_ring_layer(orc, c, layer=1, write=write, depth=2, first_slot=0, n_slots=1)
    request.getfixturevalue("knobs")
    for u in (1, 2, 8):
        B.tutti_set_tuning(0, u)
        for write in (False, True):
            H.check_ring_layer(orc, c, layer=1, write=write, depth=2, first_slot=0, n_slots=1)


def test_ring_cq_in_pinned_host_memory_polled_by_cpu(orc, H):
    """wait_cqe from the host: the completion queue sits in pinned host memory and the CPU polls its tail while
    the stream runs on (no synchronisation before the poll); what it then reads must be the oracle's queue."""
    import time
    say("rings: CQ in pinned host memory")
    rng = np.random.default_rng(47)
    nb = [700, 900]
    N = 2000
    c = H.LayerCase(T=16, h=2, d=64, e=2, N=N, n_blocks=nb, table=rng.permutation(N)[: sum(nb)], chunk=4096, L=4,
                    name="ring_hostcq")
    depth, n_slots = 8, 2
    o_ext0, _ = orc.obj_layout(c.orc_pool(orc), c.orc_cfg(orc), c.n_blocks)
    file_stride = int(2 * c.L * int(o_ext0["obj_bytes"].max()))
    store = torch.randint(0, 256, (2 * file_stride,), dtype=torch.uint8, device=H.DEV)
    o_store = store.cpu().numpy().copy()
    k2, v2 = c.k_dev.clone(), c.v_dev.clone()
    ok, ov = c.k_host.copy(), c.v_host.copy()
    sq_bytes, cq_bytes = B.ring_bytes(depth)
    sq = torch.zeros(sq_bytes, dtype=torch.uint8, device=H.DEV)
    cq = torch.zeros(cq_bytes, dtype=torch.uint8).pin_memory()
    cq_words = cq.numpy().view(np.uint32)                      # the CPU's view of the same bytes
    ring = B.make_ring(sq, cq, depth)
    o_sq, o_cq = orc.ring_alloc(depth)
    B.tutti_ring_init(ring)
    orc.ring_init(o_sq, o_cq)
    torch.cuda.synchronize()
    assert cq_words.tobytes() == o_cq.tobytes()
    fs = B.make_filestore(store, file_stride, 1000, 2)
    ext = torch.zeros(c.n_req * 32, dtype=torch.uint8, device=H.DEV)
    tot = torch.zeros(2, dtype=torch.int64, device=H.DEV)
    st = H.new_status()
    addr = 0x7f00_0000_2000
    for layer in range(c.L):                                   # four layers, two IOCBs each: the ring of 8 fills up
        B.tutti_retrieve_layer(ring, layer * n_slots, n_slots, c.gpu_pool(k2, v2), c.gpu_cfg(), c.d_n_blocks, c.n_req,
                               c.d_table, c.table.size, c.d_file_id, layer, addr, 5, fs, ext, tot, 0, st)
    deadline = time.monotonic() + 20.0
    while int(cq_words[0]) < c.L * n_slots and time.monotonic() < deadline:
        pass
    seen = int(cq_words[0])
    entries = [int(x) for x in cq_words[16:16 + depth]]       # read BEFORE any synchronisation
    torch.cuda.synchronize()
    assert seen == c.L * n_slots, f"the CPU saw {seen} completions before the deadline"
    for layer in range(c.L):
        orc.retrieve_layer(o_sq, o_cq, layer * n_slots, n_slots, c.orc_pool(orc, ok, ov), c.orc_cfg(orc), c.n_blocks,
                           c.table, c.file_id, layer, addr, 5, o_store, file_stride, 1000, 2)
    assert entries == [int(x) for x in o_cq[16:16 + depth]] == list(range(depth))
    assert cq_words.tobytes() == o_cq.tobytes() and sq.cpu().numpy().tobytes() == o_sq.tobytes()
    assert np.array_equal(k2.cpu().numpy(), ok) and np.array_equal(v2.cpu().numpy(), ov) and int(st.item()) == 0


def test_rings_deferred_writes_flushed_in_pieces(orc, H):
    """Sec. 3.3: pending writes stay recorded in the SQ while the critical-path reads go first, then are issued a
    few IOCBs at a time under a CU budget.  Same call sequence on both sides; every output compared."""
    say("rings: deferred writes")
    rng = np.random.default_rng(53)
    nb = [1300, 500]
    N = 2400
    c = H.LayerCase(T=16, h=2, d=64, e=2, N=N, n_blocks=nb, table=rng.permutation(N)[: sum(nb)], chunk=4096, L=4,
                    name="ring_deferred")
    depth = 8
    o_ext, _ = orc.obj_layout(c.orc_pool(orc), c.orc_cfg(orc), c.n_blocks)
    ext, _ = H.gpu_layout(c)
    file_stride = int(2 * c.L * int(o_ext["obj_bytes"].max()))
    store = torch.randint(0, 256, (2 * file_stride,), dtype=torch.uint8, device=H.DEV)
    o_store = store.cpu().numpy().copy()
    k2, v2 = c.k_dev.clone(), c.v_dev.clone()
    ok, ov = c.k_host.copy(), c.v_host.copy()
    nd = 2 * N
    sgl = torch.zeros(nd * 16, dtype=torch.uint8, device=H.DEV)
    B.tutti_sgl_table_build(c.gpu_pool(k2, v2), k2.data_ptr(), v2.data_ptr(), 5, sgl, nd)
    o_sgl, _ = orc.sgl_table_build(c.orc_pool(orc, ok, ov), ok.ctypes.data, ov.ctypes.data, 5)
    addr = sgl.data_ptr()
    sq_bytes, cq_bytes = B.ring_bytes(depth)
    sq = torch.zeros(sq_bytes, dtype=torch.uint8, device=H.DEV)
    cq = torch.zeros(cq_bytes, dtype=torch.uint8, device=H.DEV)
    ring = B.make_ring(sq, cq, depth)
    o_sq, o_cq = orc.ring_alloc(depth)
    B.tutti_ring_init(ring)
    orc.ring_init(o_sq, o_cq)
    fs = B.make_filestore(store, file_stride, 1000, 2)
    st = H.new_status()
    o_st = 0
    gp, op_, gc, oc_ = c.gpu_pool(k2, v2), c.orc_pool(orc, ok, ov), c.gpu_cfg(), c.orc_cfg(orc)

    def same(what):
        torch.cuda.synchronize()
        assert sq.cpu().numpy().tobytes() == o_sq.tobytes(), f"IOCBs differ after {what}"
        assert cq.cpu().numpy().tobytes() == o_cq.tobytes(), f"completion queue differs after {what}"
        assert np.array_equal(store.cpu().numpy(), o_store), f"file store differs after {what}"
        assert np.array_equal(k2.cpu().numpy(), ok) and np.array_equal(v2.cpu().numpy(), ov), f"pool differs after {what}"
        assert int(st.item()) == o_st

    # writes of layers 0..2 recorded, not issued: slots 0..5 stay FILLED
    for layer in range(3):
        B.tutti_iocb_fill_direct(ring, 2 * layer, 2, gp, gc, ext, c.n_req, c.d_table, c.table.size, c.d_file_id, layer,
                                 B.OP_WRITE, addr, 5, st)
        o_st |= orc.iocb_fill_direct(o_sq, 2 * layer, 2, op_, oc_, o_ext, c.table, c.file_id, layer, orc.OP_WRITE, addr, 5)
    same("recording the writes")
    assert list(o_sq["hdr"]["state"][:6]) == [orc.IOCB_FILLED] * 6 and int(o_cq[0]) == 0
    # the read of layer 3 goes first, through the two free slots; it overwrites the blocks the writes will save
    e2 = torch.zeros(c.n_req * 32, dtype=torch.uint8, device=H.DEV)
    t2 = torch.zeros(2, dtype=torch.int64, device=H.DEV)
    B.tutti_retrieve_layer(ring, 6, 2, gp, gc, c.d_n_blocks, c.n_req, c.d_table, c.table.size, c.d_file_id, 3, addr, 5,
                           fs, e2, t2, 0, st)
    _, _, s_ = orc.retrieve_layer(o_sq, o_cq, 6, 2, op_, oc_, c.n_blocks, c.table, c.file_id, 3, addr, 5, o_store,
                                  file_stride, 1000, 2)
    o_st |= s_
    same("the read")
    assert int(o_cq[0]) == 2 and list(o_cq[16:18]) == [6, 7]
    # the pending writes, flushed in pieces of 1, 3 and 2 IOCBs under different budgets
    for first, n, budget in ((0, 1, 2), (1, 3, 4), (4, 2, 0)):
        B.tutti_issue_io(ring, first, n, sgl, nd, addr, fs, c.bb, budget, st)
        o_st |= orc.issue_io(o_sq, o_cq, first, n, o_sgl, addr, o_store, file_stride, 1000, 2)
        same(f"flushing {n} IOCBs from slot {first}")
    assert int(o_cq[0]) == 8 and list(o_cq[16:24]) == [6, 7, 0, 1, 2, 3, 4, 5]
    assert np.all(o_sq["hdr"]["state"] == orc.IOCB_DONE) and o_st == 0


def test_iocbs_filled_by_the_cpu(orc, H):
    """The paper's own flow (sec. 3.2 "Async I/O Processing"): SQ and CQ in pinned host memory, slots from
    get_iocb, contexts and num_ioctx written by the CPU with numpy, issue_io executes them, the CPU reaps the
    CQ without synchronising the stream.  The contexts include one that trips each validity rule; pool, file
    store, status and queues are compared with the oracle given the same contexts."""
    say("rings: IOCBs filled by the CPU")
    rng = np.random.default_rng(61)
    N, bb, depth = 64, 8192, 3
    c = H.LayerCase(T=16, h=2, d=128, e=2, N=N, n_blocks=[1], table=[0], name="cpu_filled")
    assert c.bb == bb
    k2, v2 = c.k_dev.clone(), c.v_dev.clone()
    ok, ov = c.k_host.copy(), c.v_host.copy()
    nd = 2 * N
    sgl = torch.zeros(nd * 16, dtype=torch.uint8, device=H.DEV)
    B.tutti_sgl_table_build(c.gpu_pool(k2, v2), k2.data_ptr(), v2.data_ptr(), 5, sgl, nd)
    torch.cuda.synchronize()
    o_sgl, _ = orc.sgl_table_build(c.orc_pool(orc, ok, ov), ok.ctypes.data, ov.ctypes.data, 5)
    # two descriptors patched the same way on both sides: a short one and one whose block address is misaligned
    g_sgl = sgl.cpu().numpy().view(B.SGL_DTYPE).copy()
    for t in (g_sgl, o_sgl):
        t["len"][7] = 4096
        t["addr"][9] += 8
    sgl.copy_(torch.from_numpy(g_sgl.view(np.uint8)))
    base = sgl.data_ptr()
    file_stride, n_files, first_file = 1 << 20, 2, 300
    g = torch.Generator(device=H.DEV)
    g.manual_seed(8)
    store = torch.randint(0, 256, (n_files * file_stride,), dtype=torch.uint8, device=H.DEV, generator=g)
    o_store = store.cpu().numpy().copy()
    fs = B.make_filestore(store, file_stride, first_file, n_files)

    sq_bytes, cq_bytes = B.ring_bytes(depth)
    sq_pin = torch.zeros(sq_bytes, dtype=torch.uint8).pin_memory()
    cq_pin = torch.zeros(cq_bytes, dtype=torch.uint8).pin_memory()
    ring = B.make_ring(sq_pin, cq_pin, depth)
    B.tutti_ring_init(ring)
    torch.cuda.synchronize()
    sq_np = sq_pin.numpy().view(B.IOCB_DTYPE)      # the CPU's mapping of the rings
    cq_np = cq_pin.numpy().view(np.uint32)
    o_sq, o_cq = orc.ring_alloc(depth)
    orc.ring_init(o_sq, o_cq)
    state = B.make_sq_state(depth)
    side = torch.cuda.Stream()
    st = H.new_status()
    o_st = 0

    def ctx(op, desc, fid, off, ln, addr=None):
        return dict(opcode=op, file_id=fid, file_off=off, len=ln, addr=base + 16 * desc if addr is None else addr)

    def submit(first, items_per_slot, layer, opcode):
        """The application's part: contexts, num_ioctx, layer, opcode, state, on both sides' rings."""
        for b, items in enumerate(items_per_slot):
            slot = (first + b) % depth
            for ring_np in (sq_np, o_sq):
                for i, it in enumerate(items):
                    e = ring_np["ioctx"][slot][i]
                    for f in ("opcode", "kind", "layer", "file_id", "file_off", "addr", "len", "sgl_id", "user_data",
                              "iocb_idx", "ioctx_slot"):
                        e[f] = 0
                    for f, val in it.items():
                        e[f] = val
                ring_np["hdr"]["num_ioctx"][slot] = len(items)
                ring_np["hdr"]["layer"][slot] = layer
                ring_np["hdr"]["opcode"][slot] = opcode
                ring_np["hdr"]["done"][slot] = 0
                ring_np["hdr"]["state"][slot] = B.IOCB_FILLED

    blocks = rng.permutation(np.r_[0:7, 10:N])       # descriptors 7 and 9 are the patched ones
    reads = [ctx(B.OP_READ, int(blocks[i]) + (N if i % 2 else 0), first_file + i % 2, 8192 * i, 8192) for i in range(40)]
    reads += [ctx(B.OP_READ, 7, first_file, 8192 * 50, 4096), ctx(B.OP_READ, int(blocks[41]), first_file, 8192 * 60, 0)]
    bad = [ctx(0, 8, first_file, 0, 8192), ctx(3, 8, first_file, 0, 8192), ctx(B.OP_READ, 8, first_file, 0, 8192, addr=base - 16),
           ctx(B.OP_READ, 8, first_file, 0, 8192, addr=base + 16 * 8 + 8), ctx(B.OP_READ, nd, first_file, 0, 8192),
           ctx(B.OP_READ, 7, first_file, 0, 4112), ctx(B.OP_READ, 8, first_file, 0, 8208), ctx(B.OP_READ, 8, first_file, 0, 8184),
           ctx(B.OP_READ, 8, first_file, 8, 8192), ctx(B.OP_READ, 9, first_file, 0, 8192),
           ctx(B.OP_READ, 8, first_file - 1, 0, 8192), ctx(B.OP_READ, 8, first_file + 2, 0, 8192),
           ctx(B.OP_READ, 8, first_file, file_stride - 8176, 8192), ctx(B.OP_READ, 8, first_file, (1 << 64) - 16, 8192)]
    first = B.tutti_get_iocb(state, 2)
    assert first == 0
    submit(first, [reads, bad], layer=0, opcode=B.OP_READ)
    with torch.cuda.stream(side):
        B.tutti_issue_io(ring, first, 2, sgl, nd, base, fs, bb, 0, st, stream=side)
    # the CPU polls the CQ in pinned memory; no synchronisation before the completions are seen
    assert B.tutti_wait_cqe_host(state, cq_np, sq_np, (first + 1) % depth, 50_000_000), "completion never arrived"
    assert B.tutti_iocb_completed(state, first) and B.tutti_sq_free_count(state) == depth
    assert list(sq_np["hdr"]["state"][:2]) == [B.IOCB_FREE, B.IOCB_FREE]          # reaped: free again
    o_st |= orc.issue_io(o_sq, o_cq, first, 2, o_sgl, base, o_store, file_stride, first_file, n_files, max_len=bb)
    torch.cuda.synchronize()
    assert int(st.item()) == o_st == B.ST_BAD_BLOCK
    assert np.array_equal(k2.cpu().numpy(), ok) and np.array_equal(v2.cpu().numpy(), ov), "pool differs after the reads"
    assert np.array_equal(sq_np["hdr"]["done"], o_sq["hdr"]["done"]) and cq_np.tobytes() == o_cq.tobytes()
    # second round wraps around the ring: slot 2 then slot 0, writes this time, under a CU budget
    first = B.tutti_get_iocb(state, 2)
    assert first == 2
    writes = [ctx(B.OP_WRITE, int(blocks[i]) + (0 if i % 2 else N), first_file + 1, 8192 * (100 - i), 8192) for i in range(30)]
    submit(first, [writes[:11], writes[11:]], layer=1, opcode=B.OP_WRITE)
    with torch.cuda.stream(side):
        B.tutti_issue_io(ring, first, 2, sgl, nd, base, fs, bb, 4, st, stream=side)
    assert B.tutti_wait_cqe_host(state, cq_np, sq_np, 0, 50_000_000)
    o_st |= orc.issue_io(o_sq, o_cq, first, 2, o_sgl, base, o_store, file_stride, first_file, n_files, max_len=bb)
    torch.cuda.synchronize()
    assert np.array_equal(store.cpu().numpy(), o_store), "file store differs after the writes"
    assert cq_np.tobytes() == o_cq.tobytes() and int(cq_np[0]) == 4      # slot 2, then slot 0: the ring wrapped
    assert np.array_equal(k2.cpu().numpy(), ok) and np.array_equal(v2.cpu().numpy(), ov)
    assert int(st.item()) == o_st and B.tutti_sq_free_count(state) == depth


def test_ring_layer_cfg2(orc, H):
    """Config 2's layer through the rings in one call: 4096 contexts = two full IOCBs."""
    w = W.llama8b_32k(num_blocks=8192)
    say("ring layer: config 2 layer")
    c = H.LayerCase.from_workload(w)
    c.chunk = c.bb
    for write in (False, True):
        assert H.check_ring_layer(orc, c, layer=31, write=write, depth=4, first_slot=3, n_slots=2) == 0


def test_ring_layer_calls_in_two_halves_with_completions_on_a_second_stream(orc, H):
    """tutti_retrieve_layer_issue / tutti_store_layer_issue + tutti_complete_io behind an event on another stream give
    what the one-call forms give (IOCBs, CQ order, blocks, files, status), also across two calls on one ring and
    under a budget; and a train of layers whose completions all run on the second stream ends with every IOCB DONE
    and the CQ in slot order."""
    say("rings: issue and completion as separate calls")
    rng = np.random.default_rng(77)
    nb = [700, 0, 1500, 3]
    N = 2500
    c = H.LayerCase(T=16, h=2, d=64, e=2, N=N, n_blocks=nb, table=rng.permutation(N)[: sum(nb)], chunk=4096, L=3,
                    name="ring_halves")
    n_slots = (2 * sum(nb) + B.IOCB_SLOTS - 1) // B.IOCB_SLOTS
    for write in (False, True):
        assert H.check_ring_layer(orc, c, layer=1, write=write, depth=n_slots + 2, first_slot=n_slots, n_slots=n_slots,
                                  side_completion=True) == 0
        H.check_ring_layer(orc, c, layer=2, write=write, depth=n_slots + 1, first_slot=1, n_slots=n_slots,
                           cu_budget=3, prefill=True, side_completion=True)
        assert H.check_ring_layer(orc, c, layer=0, write=write, depth=4, first_slot=0, n_slots=1,
                                  side_completion=True) == B.ST_SQE_CAP                      # too few IOCBs
    # a train: 6 layers of config 2's shape (smaller pool), completions on the side stream, nothing waited for in between
    w = W.llama8b_32k(num_blocks=4096, tokens=8192, num_layers=6)
    s = w.shape
    c = H.LayerCase.from_workload(w)
    bb = c.bb
    n_tab = c.table.size
    n_slots = (2 * n_tab + B.IOCB_SLOTS - 1) // B.IOCB_SLOTS
    depth = 6 * n_slots
    file_stride = 2 * 6 * n_tab * bb
    g = torch.Generator(device=H.DEV)
    g.manual_seed(12)
    store = torch.randint(0, 256, (file_stride,), dtype=torch.uint8, device=H.DEV, generator=g)
    fs = B.make_filestore(store, file_stride, int(c.file_id[0]), 1)
    sq_bytes, cq_bytes = B.ring_bytes(depth)
    sq = torch.zeros(sq_bytes, dtype=torch.uint8, device=H.DEV)
    cq = torch.zeros(cq_bytes, dtype=torch.uint8, device=H.DEV)
    ring = B.make_ring(sq, cq, depth)
    B.tutti_ring_init(ring)
    planes = [(torch.zeros_like(c.k_dev), torch.zeros_like(c.v_dev)) for _ in range(6)]
    ext = torch.zeros(32, dtype=torch.uint8, device=H.DEV)
    tot = torch.zeros(2, dtype=torch.int64, device=H.DEV)
    st = H.new_status()
    side = torch.cuda.Stream()
    for l in range(6):
        B.tutti_retrieve_layer_issue(ring, l * n_slots, n_slots, c.gpu_pool(*planes[l]), c.gpu_cfg(), c.d_n_blocks, 1,
                                     c.d_table, n_tab, c.d_file_id, l, 0x1000, 5, fs, ext, tot, 0, st)
        ev = torch.cuda.Event()
        ev.record()
        side.wait_event(ev)
        B.tutti_complete_io(ring, l * n_slots, n_slots, side)
    torch.cuda.synchronize()
    assert int(st.item()) == 0
    q = cq.cpu().numpy().view(np.uint32)
    assert int(q[0]) == depth and list(q[16:16 + depth]) == list(range(depth))
    hdr = sq.cpu().numpy().view(B.IOCB_DTYPE)["hdr"]
    assert np.all(hdr["state"] == B.IOCB_DONE) and np.all(hdr["done"] == hdr["num_ioctx"])
    file_h = store.cpu().numpy()
    for l in (0, 3, 5):                       # the blocks of three layers against the file, byte for byte
        k_h, v_h = planes[l][0].cpu().numpy(), planes[l][1].cpu().numpy()
        for kind, plane in ((0, k_h), (1, v_h)):
            lo = (2 * l + kind) * n_tab * bb
            for j in (0, 1, n_tab // 2, n_tab - 1):
                bid = int(c.table[j])
                assert np.array_equal(plane[bid * c.stride: bid * c.stride + bb], file_h[lo + j * bb: lo + (j + 1) * bb])


def test_ring_layer_trains_with_chained_completions(orc, H):
    """tutti_retrieve_layer_chained / tutti_store_layer_chained: every launch of a train also completes the IOCBs of
    the launch before it, one tutti_complete_io ends the train.  IOCBs, CQ order, blocks, files, extents and status
    must be what the oracle's one-call sequence gives, with slot ranges that wrap around the ring and are reused,
    under a budget, with too few IOCBs, and at config 2's size; overlapping slot ranges are refused."""
    say("rings: trains of layers with chained completions")
    rng = np.random.default_rng(78)
    nb = [700, 0, 1500, 3]
    N = 2500
    c = H.LayerCase(T=16, h=2, d=64, e=2, N=N, n_blocks=nb, table=rng.permutation(N)[: sum(nb)], chunk=4096, L=5,
                    name="ring_chained")
    n_slots = (2 * sum(nb) + B.IOCB_SLOTS - 1) // B.IOCB_SLOTS          # 3
    for write in (False, True):
        st, tail = H.check_ring_layer_train(orc, c, [0, 1, 2, 3, 4], write, depth=5 * n_slots, n_slots=n_slots)
        assert st == 0 and tail == 4 * n_slots                          # four layers completed by their successors
        # the ring wraps and every slot is used again; the train starts in the middle of the ring
        H.check_ring_layer_train(orc, c, [4, 0, 3, 1, 2, 2], write, depth=2 * n_slots + 1, n_slots=n_slots, first_slot=4)
        H.check_ring_layer_train(orc, c, [1, 2, 3], write, depth=2 * n_slots, n_slots=n_slots, cu_budget=3)
        H.check_ring_layer_train(orc, c, [2], write, depth=2 * n_slots, n_slots=n_slots)   # a train of one layer
        st, _ = H.check_ring_layer_train(orc, c, [0, 1, 2], write, depth=4, n_slots=2)     # too few IOCBs per layer
        assert st == B.ST_SQE_CAP
    c = H.LayerCase(T=16, h=2, d=64, e=2, N=16, n_blocks=[4, 2], table=[3, 999, 5, 16, 7, 1], chunk=4096, L=2,
                    name="ring_chained_bad")
    for write in (False, True):
        st, _ = H.check_ring_layer_train(orc, c, [0, 1], write, depth=2, n_slots=1)
        assert st == B.ST_BAD_BLOCK
    w = W.llama8b_32k(num_blocks=8192)
    c = H.LayerCase.from_workload(w)
    c.chunk = c.bb
    for write in (False, True):
        st, tail = H.check_ring_layer_train(orc, c, [30, 31, 0], write, depth=6, n_slots=2, first_slot=3)
        assert st == 0 and tail == 4
    # the entry-driven issue in the same way: fill + tutti_issue_io_chained per step, reads and writes mixed
    rng = np.random.default_rng(79)
    nb = [700, 0, 1500, 3]
    c = H.LayerCase(T=16, h=2, d=64, e=2, N=2500, n_blocks=nb, table=rng.permutation(2500)[: sum(nb)], chunk=4096, L=5,
                    name="rings_chained")
    R, Wr = B.OP_READ, B.OP_WRITE
    assert H.check_rings_train(orc, c, [(0, Wr), (1, R), (2, R), (3, Wr), (4, R)], depth=15, n_slots=3) == 0
    assert H.check_rings_train(orc, c, [(4, R), (0, Wr), (3, R), (1, Wr), (2, R), (2, Wr)], depth=7, n_slots=3,
                               first_slot=4) == 0
    assert H.check_rings_train(orc, c, [(1, R), (2, Wr), (3, R)], depth=6, n_slots=3, cu_budget=3) == 0
    assert H.check_rings_train(orc, c, [(0, R), (1, Wr)], depth=4, n_slots=2) == B.ST_SQE_CAP
    # slot ranges that overlap are refused before anything is enqueued
    sq_bytes, cq_bytes = B.ring_bytes(8)
    sq = torch.zeros(sq_bytes, dtype=torch.uint8, device=H.DEV)
    cq = torch.zeros(cq_bytes, dtype=torch.uint8, device=H.DEV)
    ring = B.make_ring(sq, cq, 8)
    store = torch.zeros(1 << 20, dtype=torch.uint8, device=H.DEV)
    fs = B.make_filestore(store, 1 << 20, int(c.file_id[0]), 1)
    ext = torch.zeros(32, dtype=torch.uint8, device=H.DEV)
    tot = torch.zeros(2, dtype=torch.int64, device=H.DEV)
    for first, n, dfirst, dn in ((0, 2, 1, 2), (2, 2, 1, 2), (7, 2, 0, 1), (0, 2, 7, 2), (3, 1, 3, 1), (0, 8, 4, 1)):
        for fn in (B.tutti_retrieve_layer_chained, B.tutti_store_layer_chained):
            with pytest.raises(B.TuttiError) as err:
                fn(ring, first, n, dfirst, dn, c.gpu_pool(c.k_dev, c.v_dev), c.gpu_cfg(), c.d_n_blocks, 1, c.d_table,
                   c.table.size, c.d_file_id, 0, 0x1000, 5, fs, ext, tot)
            assert err.value.code == B.EINVAL
        with pytest.raises(B.TuttiError) as err:
            B.tutti_issue_io_chained(ring, first, n, dfirst, dn, store, 4, 0, fs, 4096)
        assert err.value.code == B.EINVAL
    with pytest.raises(B.TuttiError):                                   # done range outside the ring
        B.tutti_retrieve_layer_chained(ring, 0, 1, 8, 1, c.gpu_pool(c.k_dev, c.v_dev), c.gpu_cfg(), c.d_n_blocks, 1,
                                       c.d_table, c.table.size, c.d_file_id, 0, 0x1000, 5, fs, ext, tot)


# ------------------------------------------------------------------ edge cases

def test_no_requests_and_empty_requests(orc, H):
    say("edge: no requests")
    c = H.LayerCase(T=16, h=2, d=64, e=2, N=16, n_blocks=[], table=[], name="no_requests")
    ext, tot, o_ext, o_tot = H.check_layout(orc, c)
    assert int(o_tot[0]) == 0 and int(o_tot[1]) == 0
    H.check_layer_restore(orc, c)
    say("edge: only empty requests")
    c = H.LayerCase(T=16, h=2, d=64, e=2, N=16, n_blocks=[0, 0, 0], table=[], name="empty_requests")
    H.check_everything(orc, c)


def test_max_requests(orc, H):
    say("edge: 2048 requests")
    rng = np.random.default_rng(4)
    n = rng.integers(0, 4, size=B.MAX_REQ).astype(np.uint32)
    N = int(n.sum()) + 50
    c = H.LayerCase(T=16, h=2, d=64, e=2, N=N, n_blocks=n, table=rng.permutation(N)[: int(n.sum())], chunk=4096,
                    L=4, name="max_req")
    H.check_everything(orc, c)
    # the direct-mode entry writers walk from owner to owner: 2048 requests, a quarter of them empty, and a
    # second shape where long runs of empty requests sit between the non-empty ones
    H.check_direct_mode(orc, c, layer=3)
    n_slots = (2 * int(n.sum()) + B.IOCB_SLOTS - 1) // B.IOCB_SLOTS
    H.check_ring_layer(orc, c, layer=2, write=False, depth=n_slots + 2, first_slot=1, n_slots=n_slots)
    sparse = np.zeros(B.MAX_REQ, np.uint32)
    sparse[[0, 700, 701, 2047]] = [300, 1, 900, 40]
    c = H.LayerCase(T=1, h=1, d=8, e=2, N=1300, n_blocks=sparse, table=rng.permutation(1300)[:1241], align=16, chunk=16,
                    L=2, name="max_req_sparse")      # 16-byte blocks keep the 2048 files of the ring check small
    H.check_direct_mode(orc, c, layer=1)
    H.check_ring_layer(orc, c, layer=1, write=True, depth=3, first_slot=2, n_slots=2)
    H.check_ring_layer(orc, c, layer=0, write=False, depth=3, first_slot=0, n_slots=2, cu_budget=3)
    c = H.LayerCase(T=16, h=2, d=64, e=2, N=N, n_blocks=n[:65], table=rng.permutation(N)[: int(n[:65].sum())],
                    chunk=4096, L=4, layout=1, name="req65")
    H.check_everything(orc, c)


def test_bad_block_ids_are_skipped_and_reported(orc, H):
    say("edge: bad block ids")
    table = np.array([3, 999, 5, 16, 7, 1], np.uint32)   # 999 and 16 are out of range for 16 blocks
    c = H.LayerCase(T=16, h=2, d=64, e=2, N=16, n_blocks=[4, 2], table=table, name="bad_ids")
    ext, tot, o_ext, o_tot = H.check_layout(orc, c)
    H.check_pack(orc, c, ext, o_ext, o_tot)
    H.check_unpack(orc, c, ext, o_ext, o_tot)
    H.check_layer_restore(orc, c)
    H.check_layer_save(orc, c)


def test_small_capacities_are_clamped_and_reported(orc, H):
    say("edge: capacities")
    rng = np.random.default_rng(9)
    c = H.LayerCase(T=16, h=2, d=64, e=2, N=64, n_blocks=[5, 9, 3], table=rng.permutation(64)[:17], chunk=4096,
                    name="caps")
    ext, tot, o_ext, o_tot = H.check_layout(orc, c)
    cap = int(o_ext["stage_off"][2]) + 4096          # third request does not fit
    H.check_pack(orc, c, ext, o_ext, o_tot, stage_cap=cap)
    H.check_unpack(orc, c, ext, o_ext, o_tot, stage_cap=cap)
    H.check_sqe(orc, c, ext, o_ext, o_tot, sqe_cap=11)
    H.check_sqe(orc, c, ext, o_ext, o_tot, sqe_cap=0)
    H.check_layer_restore(orc, c, sqe_cap=5, stage_cap=cap)
    H.check_layer_save(orc, c, sqe_cap=5, stage_cap=cap)


def test_short_table_is_never_overrun(orc, H):
    """table_len smaller than the extents claim: the request that runs beyond it is skipped and reported, by the
    separate calls and by the fused ones alike."""
    say("edge: short table")
    rng = np.random.default_rng(10)
    c = H.LayerCase(T=16, h=2, d=64, e=2, N=64, n_blocks=[6, 6, 0, 1], table=rng.permutation(64)[:13], name="short")
    ext, tot, o_ext, o_tot = H.check_layout(orc, c)
    for tl in (12, 8, 6, 5, 0):
        assert H.check_moves_with_extents(orc, c, H.ext_np(ext, c.n_req), int(o_tot[0]), table_len=tl,
                                          label=f"table_len {tl}") == B.ST_BAD_EXTENT
        H.check_layer_restore(orc, c, table_len=tl)
        H.check_layer_save(orc, c, table_len=tl)


CALLER_EXTENT_SHAPES = [
    # T, h, d, e, N, n_blocks, align, layout
    (16, 8, 128, 2, 256, [40, 0, 7, 25, 1], 4096, 0),   # 32 KiB blocks: whole slices, the unpack preloads its first item
    (16, 8, 128, 2, 256, [40, 0, 7, 25, 1], 4096, 1),   # the same, head-major (16 bytes per lane between the orders)
    (16, 5, 40, 2, 128, [7, 0, 33, 1, 2], 4096, 0),     # 6400-byte blocks: ragged slices, padded objects
    (16, 32, 32, 1, 128, [9, 3, 0, 11], 4096, 1),       # head-major with 32-byte rows: token tiles through LDS
    (3, 1, 8, 2, 64, [1, 2, 3, 4, 5], 64, 0),           # 48-byte blocks
]


@pytest.mark.parametrize("budget", [0, 3])
@pytest.mark.parametrize("shape", CALLER_EXTENT_SHAPES, ids=[f"bb{t*h*d*e}_l{lay}" for t, h, d, e, _, _, _, lay in
                                                             CALLER_EXTENT_SHAPES])
def test_extents_written_by_the_caller(orc, H, shape, budget):
    """Pack and unpack honour hand-made extents field by field: a gap between requests, a sub-range of the
    requests, reversed order in the staging buffer, objects larger than their blocks; and they skip and report
    what cannot be honoured exactly as the oracle does."""
    T, h, d, e, N, n_blocks, A, layout = shape
    say("caller extents", shape, budget)
    rng = np.random.default_rng(77 + T * h + layout)
    total = sum(n_blocks)
    table = rng.permutation(N)[:total]
    c = H.LayerCase(T=T, h=h, d=d, e=e, N=N, n_blocks=n_blocks, table=table, align=A, chunk=A, layout=layout,
                    seed=3 + T, name=f"caller_extents{shape}")
    o_ext, o_tot = orc.obj_layout(c.orc_pool(orc), c.orc_cfg(orc), c.n_blocks)
    base = np.zeros(len(n_blocks), B.EXTENT_DTYPE)
    for f in B.EXTENT_DTYPE.names:
        base[f] = o_ext[f]
    total_bytes = int(o_tot[0])
    R = len(n_blocks)

    def run(x, size, label, **kw):
        return H.check_moves_with_extents(orc, c, x, size, cu_budget=budget, label=label, **kw)

    assert run(base, total_bytes, "layout's own") == 0
    # a 2 MiB gap in front of every request
    gap = 2 << 20
    x = base.copy()
    x["stage_off"] += gap * (1 + np.arange(R, dtype=np.uint64))
    assert run(x, total_bytes + gap * R, "2 MiB gaps") == 0
    # requests 1.. passed alone with the whole table; then the last two alone
    assert run(base[1:], total_bytes, "requests 1..") == 0
    assert run(base[-2:], total_bytes, "last two requests") == 0
    # the requests in reverse order in the staging buffer
    x = base.copy()
    end = 0
    for r in range(R - 1, -1, -1):
        x["stage_off"][r] = end
        end += 2 * int(x["obj_bytes"][r])
    assert run(x, total_bytes, "reverse order") == 0
    # objects one alignment unit larger than layout makes them: more padding, V further away
    x = base.copy()
    x["obj_bytes"] += A
    x["stage_off"] = np.concatenate([[0], np.cumsum(2 * x["obj_bytes"].astype(np.uint64))[:-1]])
    assert run(x, total_bytes + 2 * A * R, "larger objects") == 0
    # requests in another order than their table ranges
    x = base[::-1].copy()
    assert run(x, total_bytes, "records reversed") == 0
    # ---- what cannot be honoured
    assert run(base, total_bytes, "table one short", table_len=total - 1) == B.ST_BAD_EXTENT
    assert run(base, total_bytes, "empty table", table_len=0) == B.ST_BAD_EXTENT
    x = base.copy()
    x["stage_off"][0] += 8
    st = run(x, total_bytes + 16, "misaligned offset")
    assert st & B.ST_BAD_EXTENT
    x = base.copy()
    x["obj_bytes"][0] = 1 << 63
    assert run(x, total_bytes, "object size wraps") & B.ST_STAGE_CAP
    x = base.copy()
    x["stage_off"][R - 1] = (1 << 64) - 4096
    assert run(x, total_bytes, "offset wraps") & B.ST_STAGE_CAP
    big = int(np.argmax(n_blocks))
    x = base.copy()
    x["obj_bytes"][big] -= A          # too small for its last block (and the V object moves up)
    assert run(x, total_bytes, "object too small") & B.ST_BAD_EXTENT
    x = base.copy()
    x["table_off"][R - 1] = total - 1  # runs off the end of the table
    if n_blocks[R - 1] > 1:
        assert run(x, total_bytes, "table range beyond the table") & B.ST_BAD_BLOCK
    x = base.copy()
    x["n_blocks"][0] += 1              # claims one block more than the table holds in all
    assert run(x, total_bytes + c.bb, "one block too many") & B.ST_BAD_EXTENT
    assert run(base, total_bytes, "capacity one byte short", stage_cap=total_bytes - 1) == B.ST_STAGE_CAP


def test_entry_builders_want_layout_extents(orc, H):
    """tutti_sqe_build, tutti_sqe_build_direct and tutti_iocb_fill_direct write nothing and report BAD_EXTENT when
    the extents are not the ones tutti_obj_layout writes for these requests; stage_off alone is free."""
    say("entry builders: extents contract")
    rng = np.random.default_rng(5)
    n = [3, 2, 4, 0, 70]
    c = H.LayerCase(T=16, h=2, d=64, e=2, N=128, n_blocks=n, table=rng.permutation(128)[: sum(n)], chunk=8192, L=3,
                    name="dense_extents")
    ext, tot, o_ext, o_tot = H.check_layout(orc, c)
    base = H.ext_np(ext, c.n_req).copy()
    n_sqe, n_ctx = int(o_tot[1]), 2 * sum(n)
    variants = []
    for field, delta in (("sqe_base", 2), ("table_off", 1), ("obj_bytes", 4096), ("n_chunks", 1), ("n_blocks", 1)):
        for r in (0, 2, 4):
            x = base.copy()
            x[field][r] += delta
            variants.append((f"{field}[{r}]", x, c.file_id))
    variants.append(("requests 1.. alone", base[1:].copy(), c.file_id[1:]))
    x = base.copy()
    x["stage_off"] += 1 << 21
    variants.append(("stage_off moved (allowed)", x, c.file_id))
    for label, x, fid in variants:
        o_x = np.zeros(x.size, orc.EXTENT_DTYPE)
        for f in B.EXTENT_DTYPE.names:
            o_x[f] = x[f]
        d_x = torch.from_numpy(x.view(np.uint8).copy()).to(H.DEV)
        d_fid = H.to_dev(fid)
        sqe = torch.full((n_sqe * 64,), 0x3C, dtype=torch.uint8, device=H.DEV)
        st = H.new_status()
        B.tutti_sqe_build(c.gpu_pool(), c.gpu_cfg(), d_x, x.size, d_fid, 1, B.OP_READ, 1 << 30, 9, sqe, n_sqe, st)
        dsqe = torch.full((n_ctx * 64,), 0x3C, dtype=torch.uint8, device=H.DEV)
        st2 = H.new_status()
        B.tutti_sqe_build_direct(c.gpu_pool(), c.gpu_cfg(), d_x, x.size, c.d_table, c.table.size, d_fid, 1, B.OP_WRITE,
                                 1 << 20, 9, dsqe, n_ctx, st2)
        sq_b, cq_b = B.ring_bytes(2)
        d_sq = torch.zeros(sq_b, dtype=torch.uint8, device=H.DEV)
        d_cq = torch.zeros(cq_b, dtype=torch.uint8, device=H.DEV)
        ring = B.make_ring(d_sq, d_cq, 2)
        B.tutti_ring_init(ring)
        st3 = H.new_status()
        B.tutti_iocb_fill_direct(ring, 1, 1, c.gpu_pool(), c.gpu_cfg(), d_x, x.size, c.d_table, c.table.size, d_fid, 1,
                                 B.OP_WRITE, 1 << 20, 9, st3)
        torch.cuda.synchronize()
        o_sqe, o_st = orc.sqe_build(c.orc_pool(orc), c.orc_cfg(orc), o_x, fid, 1, orc.OP_READ, 1 << 30, 9, sqe_cap=n_sqe)
        o_d, o_st2 = orc.sqe_build_direct(c.orc_pool(orc), c.orc_cfg(orc), o_x, c.table, fid, 1, orc.OP_WRITE, 1 << 20,
                                          9, sqe_cap=n_ctx)
        o_sq, o_cq = orc.ring_alloc(2)
        orc.ring_init(o_sq, o_cq)
        o_st3 = orc.iocb_fill_direct(o_sq, 1, 1, c.orc_pool(orc), c.orc_cfg(orc), o_x, c.table, fid, 1, orc.OP_WRITE,
                                     1 << 20, 9)
        assert (int(st.item()), int(st2.item()), int(st3.item())) == (o_st, o_st2, o_st3), label
        got, gotd = sqe.cpu().numpy(), dsqe.cpu().numpy()
        if o_st:
            assert o_st == B.ST_BAD_EXTENT and np.all(got == 0x3C) and np.all(gotd == 0x3C), label
        else:
            assert got.tobytes() == o_sqe.tobytes() and gotd.tobytes() == o_d.tobytes(), label
        # IOCB headers and the contexts that were filled (the rest of an IOCB is never written by either side)
        g_sq = d_sq.cpu().numpy().view(B.IOCB_DTYPE)
        for b in range(2):
            assert g_sq["hdr"][b].tobytes()[:24] == o_sq["hdr"][b].tobytes()[:24], label
            k = int(o_sq["hdr"]["num_ioctx"][b])
            assert g_sq["ioctx"][b][:k].tobytes() == o_sq["ioctx"][b][:k].tobytes(), label


def test_io_domain_stream_confines_the_calls(orc, H):
    """A stream from tutti_io_domain_create (compute-unit mask: the hardware-isolated I/O domain of sec. 3.2) passed
    as `stream`: results stay bit-exact, and a whole-GPU-sized launch on it is held to the domain's units (timed
    against the same launch on an ordinary stream)."""
    say("I/O domain: CU-masked stream")
    try:
        handle = B.tutti_io_domain_create(16)
    except B.TuttiError as e:
        pytest.skip(f"the runtime refuses a compute-unit mask on this machine: {e}")
    try:
        dom = torch.cuda.ExternalStream(handle)
        rng = np.random.default_rng(12)
        n = [300, 0, 41, 700]
        c = H.LayerCase(T=16, h=8, d=128, e=2, N=2048, n_blocks=n, table=rng.permutation(2048)[: sum(n)], chunk=32768,
                        L=4, name="io_domain")
        torch.cuda.synchronize()
        with torch.cuda.stream(dom):
            H.check_layer_restore(orc, c, layer=2)
            H.check_layer_save(orc, c, layer=1)
            H.check_ring_layer(orc, c, layer=3, write=False, depth=3, first_slot=2, n_slots=2)
            H.check_ring_layer(orc, c, layer=0, write=True, depth=3, first_slot=1, n_slots=2)
        # the same restore, 64 MiB of payload, on the domain and on an ordinary stream
        ext = torch.zeros(c.n_req * 32, dtype=torch.uint8, device=H.DEV)
        tot = torch.zeros(2, dtype=torch.int64, device=H.DEV)
        sqe = torch.zeros(64 * 4096, dtype=torch.uint8, device=H.DEV)
        stage = torch.zeros(2 * sum(n) * c.bb, dtype=torch.uint8, device=H.DEV)
        k2, v2 = c.k_dev.clone(), c.v_dev.clone()
        pool = c.gpu_pool(k2, v2)

        def timed(stream):
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            for rep in range(3):
                if rep == 1:
                    a.record(stream)
                B.tutti_layer_restore(pool, c.gpu_cfg(), c.d_n_blocks, c.n_req, c.d_table, c.table.size, c.d_file_id, 0,
                                      stage, stage.numel(), 0, 1, ext, tot, sqe, 4096, 0, None, stream)
            b.record(stream)
            torch.cuda.synchronize()
            return a.elapsed_time(b) / 2 * 1e3
        plain = torch.cuda.Stream()
        t_plain, t_dom = timed(plain), timed(dom)
        say(f"I/O domain of 16 CUs: restore {t_dom:.1f} us, whole GPU {t_plain:.1f} us")
        assert t_dom > 2.0 * t_plain, "the masked stream did not confine the launch"
    finally:
        torch.cuda.synchronize()
        B.tutti_io_domain_destroy(handle)
    with pytest.raises(B.TuttiError) as ei:
        B.tutti_io_domain_create(0)
    assert ei.value.code == B.ERANGE
    with pytest.raises(B.TuttiError) as ei:
        B.tutti_io_domain_create(B.tutti_cu_count() + 1)
    assert ei.value.code == B.ERANGE


def test_cu_budget_out_of_range(H):
    c = H.LayerCase(T=16, h=2, d=64, e=2, N=16, n_blocks=[2], table=[1, 2], name="budget")
    ext, tot = H.gpu_layout(c)
    with pytest.raises(B.TuttiError) as ei:
        B.tutti_obj_unpack(c.gpu_pool(), c.gpu_cfg(), ext, 1, c.d_table, 2, torch.zeros(1 << 16, dtype=torch.uint8,
                           device=H.DEV), 1 << 16, B.tutti_cu_count() + 1)
    assert ei.value.code == B.ERANGE
    assert B.tutti_cu_count() >= 64


def test_table_validate(orc, H):
    """Ids in range and no id twice: the device's all-pairs check, and its linear-time check with a lent bitmap
    (handed over full of garbage), against the oracle."""
    say("table validation")
    rng = np.random.default_rng(61)

    def both(num_blocks, table):
        table = np.ascontiguousarray(table, np.uint32)
        st, st_ws = H.new_status(), H.new_status()
        d_table = H.to_dev(table) if table.size else None
        B.tutti_table_validate(num_blocks, d_table, table.size, st)
        nbytes = B.tutti_table_validate_work_bytes(num_blocks)
        assert nbytes % 256 == 0 and nbytes * 8 >= num_blocks
        work = torch.full((nbytes + 256,), 0xFF, dtype=torch.uint8, device=H.DEV)
        B.tutti_table_validate_ws(num_blocks, d_table, table.size, st_ws, work, nbytes)
        torch.cuda.synchronize()
        want = orc.table_validate(num_blocks, table)
        assert int(st.item()) == want, (num_blocks, table.size, int(st.item()), want)
        assert int(st_ws.item()) == want, ("bitmap", num_blocks, table.size, int(st_ws.item()), want)
        assert bool((work[nbytes:] == 0xFF).all()), "the check wrote beyond the bytes it was lent"
        return want

    assert both(16, []) == 0 and both(1, [0]) == 0 and both(1, [0, 0]) == B.ST_DUP_BLOCK
    assert both(4, [7, 7]) == B.ST_BAD_BLOCK and both(4, [3, 9, 3]) == (B.ST_BAD_BLOCK | B.ST_DUP_BLOCK)
    for n in (1, 3, 4, 5, 255, 256, 257, 1000, 2049):
        N = 3 * n + 7
        clean = rng.permutation(N)[:n]
        assert both(N, clean) == 0
        for _ in range(6):                       # one planted duplicate at random positions, near and far
            t = clean.copy()
            i, j = sorted(rng.choice(n, size=2, replace=False)) if n > 1 else (0, 0)
            if i != j:
                t[j] = t[i]
                assert both(N, t) == B.ST_DUP_BLOCK, (n, i, j)
        if n > 2:
            t = clean.copy()
            t[0], t[-1] = N, N + 5                 # out of range at both ends: reported, not duplicates
            assert both(N, t) == B.ST_BAD_BLOCK
            if n > 3:
                t[n - 2] = t[1]
                assert both(N, t) == (B.ST_BAD_BLOCK | B.ST_DUP_BLOCK)
    for _ in range(20):                          # random tables with many repeats
        N = int(rng.integers(1, 3000))
        both(N, rng.integers(0, N + 2, size=int(rng.integers(0, 4000))))
    # config 3's table (40,719 distinct blocks of 65,536), then its first and last entries made equal
    w = W.batch64_zipf()
    assert both(w.shape.num_blocks, w.block_table) == 0
    t = w.block_table.copy()
    t[-1] = t[0]
    assert both(w.shape.num_blocks, t) == B.ST_DUP_BLOCK
    with pytest.raises(B.TuttiError):
        B.tutti_table_validate(0, H.to_dev(t), t.size, H.new_status())
    # a million entries over four million blocks: linear time, about a millisecond
    N = 1 << 22
    big = rng.permutation(N)[: 1 << 20].astype(np.uint32)
    work = torch.empty(B.tutti_table_validate_work_bytes(N), dtype=torch.uint8, device=H.DEV)
    for plant, want in ((False, 0), (True, B.ST_DUP_BLOCK)):
        if plant:
            big[777_777] = big[3]
        st = H.new_status()
        B.tutti_table_validate_ws(N, H.to_dev(big), big.size, st, work, work.numel())
        torch.cuda.synchronize()
        assert int(st.item()) == want == orc.table_validate(N, big)
    with pytest.raises(B.TuttiError) as ei:      # a bitmap one byte short
        B.tutti_table_validate_ws(N, H.to_dev(big), big.size, H.new_status(), work, work.numel() - 1)
    assert ei.value.code == B.ERANGE


def test_table_order(orc, H):
    """The visiting order by ascending block id, device against oracle, element by element: clean tables of many
    sizes (pool sizes that are not multiples of 32, ids in the first and last bitmap words), tables the check objects
    to (identity order plus the status bits), work memory handed over full of garbage."""
    say("table order")
    rng = np.random.default_rng(71)

    def both(num_blocks, table):
        table = np.ascontiguousarray(table, np.uint32)
        nbytes = B.tutti_table_order_work_bytes(num_blocks)
        assert nbytes % 256 == 0
        work = torch.full((nbytes + 256,), 0xA5, dtype=torch.uint8, device=H.DEV)
        d_visit = torch.full((table.size + 8,), -7, dtype=torch.int32, device=H.DEV)
        st = H.new_status()
        B.tutti_table_order(num_blocks, H.to_dev(table) if table.size else None, table.size, d_visit, work, nbytes, st)
        torch.cuda.synchronize()
        want, want_st = orc.table_order(num_blocks, table)
        got = d_visit.cpu().numpy().view(np.uint32)
        assert np.array_equal(got[: table.size], want), (num_blocks, table.size)
        assert np.all(d_visit.cpu().numpy()[table.size:] == -7), "wrote beyond table_len"
        assert int(st.item()) == want_st
        assert bool((work[nbytes:] == 0xA5).all()), "wrote beyond the bytes it was lent"
        return want_st

    assert both(16, []) == 0 and both(1, [0]) == 0 and both(33, [32, 0, 31]) == 0
    assert both(1, [0, 0]) == B.ST_DUP_BLOCK and both(4, [1, 7]) == B.ST_BAD_BLOCK
    assert both(40, [3, 99, 3, 1]) == (B.ST_BAD_BLOCK | B.ST_DUP_BLOCK)
    for n in (2, 63, 64, 65, 1000, 4097, 70_001):
        for N in (n, n + 1, 3 * n + 7, 32 * ((3 * n + 31) // 32)):
            assert both(N, rng.permutation(N)[:n]) == 0
        t = rng.permutation(2 * n)[:n]
        t[n - 1] = t[0]
        assert both(2 * n, t) == B.ST_DUP_BLOCK
        t[n // 2] = 2 * n                        # (for n = 2 this replaces the duplicate)
        assert both(2 * n, t) == (B.ST_BAD_BLOCK | (B.ST_DUP_BLOCK if n > 2 else 0))
    for w in (W.llama8b_32k(), W.batch64_zipf(), W.llama70b_128k()):     # the tables of configs 2, 3, 4
        assert both(w.shape.num_blocks, w.block_table) == 0
    # a million entries over four million blocks (beyond the oracle's quadratic sort): the properties that define
    # the order instead: a permutation of the positions along which the ids ascend
    N = (1 << 22) + 5
    big = rng.permutation(N)[: 1 << 20].astype(np.uint32)
    d_visit = torch.zeros(big.size, dtype=torch.int32, device=H.DEV)
    work = torch.empty(B.tutti_table_order_work_bytes(N), dtype=torch.uint8, device=H.DEV)
    st = H.new_status()
    B.tutti_table_order(N, H.to_dev(big), big.size, d_visit, work, work.numel(), st)
    torch.cuda.synchronize()
    got = d_visit.cpu().numpy().view(np.uint32)
    assert int(st.item()) == 0 and np.array_equal(np.sort(got), np.arange(big.size, dtype=np.uint32))
    assert np.all(np.diff(big[got].astype(np.int64)) > 0)
    tab = H.to_dev(np.arange(8, dtype=np.uint32))
    vis = torch.zeros(8, dtype=torch.int32, device=H.DEV)
    work = torch.zeros(B.tutti_table_order_work_bytes(64), dtype=torch.uint8, device=H.DEV)
    with pytest.raises(B.TuttiError) as ei:
        B.tutti_table_order(64, tab, 8, vis, work, work.numel() - 1)
    assert ei.value.code == B.ERANGE
    for bad in (dict(num_blocks=0), dict(d_visit=None), dict(d_block_table=None), dict(d_work=None)):
        kw = dict(num_blocks=64, d_block_table=tab, table_len=8, d_visit=vis, d_work=work, work_bytes=work.numel())
        kw.update(bad)
        with pytest.raises(B.TuttiError) as ei:
            B.tutti_table_order(**kw)
        assert ei.value.code == B.EINVAL


ORDERED_SHAPES = [
    # T, h, d, e, N, n_blocks, layout, pad
    (16, 8, 128, 2, 300, [40, 0, 7, 25, 1], 0, 0),     # 32 KiB blocks: eight whole slices each
    (16, 8, 128, 2, 300, [40, 0, 7, 25, 1], 1, 0),     # head-major, rows of 256 bytes: moved row by row, in order
    (16, 5, 40, 2, 200, [7, 0, 33, 1, 2], 0, 48),      # 6400-byte blocks: a ragged last slice, padded objects, stride
    (16, 2, 16, 2, 128, [9, 30, 2], 1, 0),             # head-major through LDS tiles: the order is not used
]


@pytest.mark.parametrize("shape", ORDERED_SHAPES, ids=lambda s: f"T{s[0]}h{s[1]}d{s[2]}L{s[6]}")
def test_layer_restore_in_a_given_order(orc, H, shape):
    """tutti_layer_restore_ordered against the oracle's ordered restore on the same list: the order the device
    computes for the table, a reversed and a shuffled list, lists with positions out of range, twice and missing,
    a table shorter than the requests claim, capacities too small, ids out of range, CU budgets."""
    T, h, d, e, N, nb, layout, pad = shape
    say(f"ordered restore T={T} h={h} d={d} layout={layout}")
    rng = np.random.default_rng(sum(shape[:5]))
    n = int(np.sum(nb))
    c = H.LayerCase(T=T, h=h, d=d, e=e, N=N, n_blocks=nb, table=rng.permutation(N)[:n], chunk=8192, L=3,
                    layout=layout, pad=pad, name="ordered")
    through_lds = layout == 1 and d * e < 128
    # the device's own order for this table, checked against the oracle's, then used by both
    work = torch.zeros(B.tutti_table_order_work_bytes(N), dtype=torch.uint8, device=H.DEV)
    d_visit = torch.zeros(n, dtype=torch.int32, device=H.DEV)
    B.tutti_table_order(N, c.d_table, n, d_visit, work, work.numel())
    torch.cuda.synchronize()
    by_id = d_visit.cpu().numpy().view(np.uint32).copy()
    assert np.array_equal(by_id, orc.table_order(N, c.table)[0])
    perms = [by_id, by_id[::-1].copy(), rng.permutation(n).astype(np.uint32), np.arange(n, dtype=np.uint32)]
    for k, visit in enumerate(perms):
        for budget in (0, 3):
            H.check_layer_restore(orc, c, layer=k % 3, cu_budget=budget, visit=visit, seed=20 + k)
    if through_lds:
        return            # lists that are not permutations mean something only where the list is read
    # lists that are not permutations: out of range, twice, missing
    odd = by_id.copy()
    odd[0] = n
    odd[1] = 0xFFFFFFFF
    odd[2] = odd[3]
    odd[n - 1] = odd[n - 2]
    H.check_layer_restore(orc, c, visit=odd, seed=31)
    H.check_layer_restore(orc, c, visit=np.zeros(n, np.uint32), seed=32)
    # a table shorter than the requests claim: the list still has table_len entries, some now beyond the live blocks
    for tl in (n - 1, int(nb[0]), int(nb[0]) - 1, 0):
        H.check_layer_restore(orc, c, table_len=tl, visit=rng.permutation(n).astype(np.uint32), seed=33)
    # staging and entry capacities too small, with the first block of the request that does not fit not listed
    o_ext, _ = orc.obj_layout(c.orc_pool(orc), c.orc_cfg(orc), c.n_blocks)
    last = c.n_req - 1
    cap = int(o_ext["stage_off"][last]) + 16
    H.check_layer_restore(orc, c, stage_cap=cap, sqe_cap=3, visit=by_id, seed=34)
    skip_first = by_id.copy()
    skip_first[skip_first == int(o_ext["table_off"][last])] = 0
    H.check_layer_restore(orc, c, stage_cap=cap, visit=skip_first, seed=35)
    # ids out of range in the table
    bad = c.table.copy()
    bad[[1, n // 2]] = [N, 0xFFFFFFFF]
    cb = H.LayerCase(T=T, h=h, d=d, e=e, N=N, n_blocks=nb, table=bad, chunk=8192, L=3, layout=layout, pad=pad,
                     name="ordered_bad_ids")
    H.check_layer_restore(orc, cb, visit=by_id, seed=36)
    # no list: the plain restore
    st = H.new_status()
    k2, v2 = c.k_dev.clone(), c.v_dev.clone()
    k3, v3 = c.k_dev.clone(), c.v_dev.clone()
    tot0 = int(orc.obj_layout(c.orc_pool(orc), c.orc_cfg(orc), c.n_blocks)[1][0])
    stage = torch.randint(0, 256, (tot0,), dtype=torch.uint8, device=H.DEV)
    ext = torch.zeros(c.n_req * 32, dtype=torch.uint8, device=H.DEV)
    tot = torch.zeros(2, dtype=torch.int64, device=H.DEV)
    B.tutti_layer_restore_ordered(c.gpu_pool(k2, v2), c.gpu_cfg(), c.d_n_blocks, c.n_req, c.d_table, n, c.d_file_id,
                                  0, stage, tot0, 0, 1, ext, tot, None, 0, None, 0, st)
    B.tutti_layer_restore(c.gpu_pool(k3, v3), c.gpu_cfg(), c.d_n_blocks, c.n_req, c.d_table, n, c.d_file_id, 0, stage,
                          tot0, 0, 1, ext, tot, None, 0, 0, st)
    torch.cuda.synchronize()
    assert torch.equal(k2, k3) and torch.equal(v2, v3) and int(st.item()) == B.ST_SQE_CAP   # no room for entries given


def test_ordered_restore_of_a_whole_layer_matches_the_plain_one(orc, H):
    """Config 3 (64 requests, fragmented pool) at full size, in bench.py's launch shape: with the device's own order
    the ordered restore writes exactly what the plain restore writes (planes, entries, extents, status)."""
    say("ordered restore, config 3 full size")
    w = W.batch64_zipf()
    c = H.LayerCase.from_workload(w, fill="tags")
    n = c.table.size
    work = torch.zeros(B.tutti_table_order_work_bytes(c.N), dtype=torch.uint8, device=H.DEV)
    d_visit = torch.zeros(n, dtype=torch.int32, device=H.DEV)
    st = H.new_status()
    B.tutti_table_order(c.N, c.d_table, n, d_visit, work, work.numel(), st)
    o_ext, o_tot = orc.obj_layout(c.orc_pool(orc), c.orc_cfg(orc), c.n_blocks)
    stage = H.as_u8(W.device_values(5, int(o_tot[0]) // 2, "bf16", H.DEV))
    n_sqe = int(o_tot[1])
    outs = []
    for ordered in (False, True):
        k2, v2 = torch.zeros_like(c.k_dev), torch.zeros_like(c.v_dev)
        ext = torch.zeros(c.n_req * 32, dtype=torch.uint8, device=H.DEV)
        tot = torch.zeros(2, dtype=torch.int64, device=H.DEV)
        sqe = torch.zeros(n_sqe * 64, dtype=torch.uint8, device=H.DEV)
        args = (c.gpu_pool(k2, v2), c.gpu_cfg(), c.d_n_blocks, c.n_req, c.d_table, n, c.d_file_id, 7, stage,
                stage.numel(), 0x7F0000000000, 3, ext, tot, sqe, n_sqe)
        if ordered:
            B.tutti_layer_restore_ordered(*args, d_visit, 0, st)
        else:
            B.tutti_layer_restore(*args, 0, st)
        torch.cuda.synchronize()
        outs.append((k2, v2, ext, tot, sqe))
    for a, b in zip(*outs):
        assert torch.equal(a, b)
    assert int(st.item()) == 0
    # and the plain one against the oracle on sampled blocks: the object bytes of block j of request r sit in block
    # table[table_off + j] of both planes
    stage_h = stage.cpu().numpy()
    k_h, v_h = outs[1][0].cpu().numpy(), outs[1][1].cpu().numpy()
    rng = np.random.default_rng(3)
    for r in rng.choice(c.n_req, size=12, replace=False):
        x = o_ext[r]
        if x["n_blocks"] == 0:
            continue
        for j in {0, int(x["n_blocks"]) - 1, int(rng.integers(0, x["n_blocks"]))}:
            bid = int(c.table[int(x["table_off"]) + j])
            for kind, plane in ((0, k_h), (1, v_h)):
                src = int(x["stage_off"]) + kind * int(x["obj_bytes"]) + j * c.bb
                assert np.array_equal(plane[bid * c.stride: bid * c.stride + c.bb], stage_h[src: src + c.bb])


def test_table_validate_with_bitmap_can_be_captured_in_a_graph(orc, H):
    """The linear-time check clears its bitmap with a kernel (no memset node), so both of its forms can be captured
    in a HIP graph; every replay must report what the eager call reports, with eager work between the replays and
    the table changed in place (same address) from clean to one with a duplicate and back."""
    say("table validation under graph capture")
    rng = np.random.default_rng(88)
    N = 50_000
    clean = rng.permutation(N)[:20_000].astype(np.uint32)
    dup = clean.copy()
    dup[19_999] = dup[0]
    d_table = H.to_dev(clean)
    st_ws, st_static = H.new_status(), H.new_status()
    work = torch.empty(B.tutti_table_validate_work_bytes(N), dtype=torch.uint8, device=H.DEV)

    def both():
        B.tutti_table_validate_ws(N, d_table, clean.size, st_ws, work, work.numel())
        B.tutti_table_validate_static(N, d_table, clean.size, st_static)

    both()                                     # eager first (also looks the static array up, outside the capture)
    torch.cuda.synchronize()
    assert int(st_ws.item()) == int(st_static.item()) == 0
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            both()
    torch.cuda.synchronize()
    for rep, table in enumerate((dup, clean, dup, clean)):
        d_table.copy_(H.to_dev(table))
        st_ws.zero_()
        st_static.zero_()
        junk = torch.randn(256, 256, device=H.DEV) @ torch.randn(256, 256, device=H.DEV)   # eager work in between
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        want = orc.table_validate(N, table)
        assert int(st_ws.item()) == int(st_static.item()) == want, (rep, int(st_ws.item()), int(st_static.item()), want)
        assert torch.isfinite(junk).all()


def test_default_kernels_keep_eight_workgroups_per_cu_resident(H):
    """The whole-GPU grids are sized for 8 resident 256-thread workgroups per compute unit; a kernel variant that
    grew past 64 VGPRs would leave part of its persistent grid waiting behind the rest (a tail of several percent)."""
    say("occupancy of the default kernels")
    names = ["layer_restore", "layer_save", "unpack", "pack", "retrieve_layer", "store_layer", "layer_restore HND",
             "layer_save HND", "layer_restore LDS", "layer_save LDS", "issue_io"]
    got = {n: B.tutti_resident_wgs_per_cu(i) for i, n in enumerate(names)}
    assert all(v >= 8 for v in got.values()), got
    with pytest.raises(B.TuttiError):
        B.tutti_resident_wgs_per_cu(len(names))


def test_copy_baseline(H):
    say("copy baseline")
    g = torch.Generator(device=H.DEV)
    g.manual_seed(1)
    for n in (16, 4096, 1 << 20, (1 << 20) + 48, 5 * 4096 + 16):
        src = torch.randint(0, 256, (n,), dtype=torch.uint8, device=H.DEV, generator=g)
        dst = torch.zeros(n + 64, dtype=torch.uint8, device=H.DEV)
        B.tutti_copy_baseline(dst, src, n)
        torch.cuda.synchronize()
        assert torch.equal(dst[:n], src) and not dst[n:].any()


def test_stream_baseline(H):
    """Read-only and write-only streams: the fill pattern and the xor of all 16-byte units, against numpy."""
    say("stream baseline")
    g = torch.Generator(device=H.DEV)
    g.manual_seed(5)
    for n in (16, 4096, (1 << 20) + 48, 9 * 8192 + 32):
        for budget in (0, 3):
            buf = torch.randint(0, 256, (n + 64,), dtype=torch.uint8, device=H.DEV, generator=g)
            acc = torch.zeros(4 * B.STREAM_SLOTS, dtype=torch.int32, device=H.DEV)
            B.tutti_stream_baseline(buf, n, False, acc, budget)
            B.tutti_stream_baseline(buf, n, False, acc, budget)          # accumulates: twice the same gives zero
            torch.cuda.synchronize()
            assert not acc.any()
            B.tutti_stream_baseline(buf, n, False, acc, budget)
            torch.cuda.synchronize()
            words = buf.cpu().numpy()[:n].view(np.uint32).reshape(-1, 4)
            slots = acc.cpu().numpy().view(np.uint32).reshape(-1, 4)
            assert np.array_equal(np.bitwise_xor.reduce(slots, axis=0), np.bitwise_xor.reduce(words, axis=0))
            tail = buf[n:].clone()
            B.tutti_stream_baseline(buf, n, True, None, budget)
            torch.cuda.synchronize()
            got = buf.cpu().numpy()[:n].view(np.uint32).reshape(-1, 4)
            unit = np.arange(n // 16, dtype=np.uint64)
            want = np.stack([unit.astype(np.uint32), (unit >> np.uint64(32)).astype(np.uint32),
                             ~unit.astype(np.uint32), np.full(unit.size, 0x54555454, np.uint32)], axis=1)
            assert np.array_equal(got, want) and torch.equal(buf[n:], tail)


def test_scatter_baseline(H):
    say("scatter baseline")
    rng = np.random.default_rng(2)
    gran, n_slots, n = 8192, 64, 24
    perm = rng.permutation(n_slots)[:n].astype(np.uint32)
    perm[5] = 200                                     # out of the span: skipped
    d_perm = H.to_dev(perm)
    g = torch.Generator(device=H.DEV)
    g.manual_seed(3)
    contig = torch.randint(0, 256, (n * gran,), dtype=torch.uint8, device=H.DEV, generator=g)
    scat = torch.zeros(n_slots * gran, dtype=torch.uint8, device=H.DEV)
    for shape, budget in [("wave_slice", 0), ("wave_slice", 2)] + [(s, 0) for s in B.SCATTER_SHAPES if s != "wave_slice"]:
        say("  shape", shape, "budget", budget)
        scat.zero_()
        B.tutti_scatter_baseline(scat, scat.numel(), contig, contig.numel(), d_perm, gran, 1, shape, budget)
        torch.cuda.synchronize()
        want = np.zeros((n_slots, gran), np.uint8)
        src = contig.cpu().numpy().reshape(n, gran)
        for i, p in enumerate(perm):
            if p < n_slots:
                want[p] = src[i]
        assert np.array_equal(scat.cpu().numpy().reshape(n_slots, gran), want)
        back = torch.full_like(contig, 7)
        B.tutti_scatter_baseline(scat, scat.numel(), back, back.numel(), d_perm, gran, 0, shape, budget)
        torch.cuda.synchronize()
        exp = src.copy()
        exp[5] = 7
        assert np.array_equal(back.cpu().numpy().reshape(n, gran), exp)


# ------------------------------------------------------------------ configs 2-5 at their real shapes

def test_cfg2_llama8b_32k_full_layer(orc, H):
    """Config 2 at full size for one layer: 65536-block planes (2 GiB each), 2048-block shuffled table."""
    w = W.llama8b_32k()
    say("cfg2 full layer", w.shape)
    c = H.LayerCase.from_workload(w)
    H.check_everything(orc, c)


def test_cfg2_head_major(orc, H):
    w = W.llama8b_32k(num_blocks=4096)
    say("cfg2 head-major, 4096-block pool")
    c = H.LayerCase.from_workload(w, layout=1)
    H.check_everything(orc, c)


@pytest.mark.parametrize("chunk", [2 << 20, 32768], ids=["chunk2MiB", "per_block"])
def test_cfg3_batch64(orc, H, chunk):
    """Config 3 at full size: 64 requests, Zipf lengths, partial hits, disjoint tables."""
    w = W.batch64_zipf(chunk_bytes=chunk)
    say("cfg3", chunk, int(w.n_blocks.sum()), "blocks")
    c = H.LayerCase.from_workload(w)
    ext, tot, o_ext, o_tot = H.check_layout(orc, c)
    H.check_sqe(orc, c, ext, o_ext, o_tot, layer=w.shape.num_layers - 1)
    if chunk == 2 << 20:
        H.check_unpack(orc, c, ext, o_ext, o_tot)
        H.check_pack(orc, c, ext, o_ext, o_tot)
    H.check_layer_restore(orc, c, layer=5)


def test_cfg4_llama70b_128k_layer(orc, H):
    """Config 4's layer shape: 38146-block planes, 8192-block fragmented table (512 MiB payload)."""
    w = W.llama70b_128k()
    say("cfg4 layer", w.shape)
    c = H.LayerCase.from_workload(w)
    H.check_everything(orc, c)


def test_cfg4_layer_of_one_tensor_parallel_rank(orc, H):
    """Config 4 as one rank of a tensor-parallel group of 8 holds it: one KV head of every block, so 4 KiB blocks
    (a wavefront's slice is the whole block), the same 8192-entry fragmented table; also under a budget."""
    import dataclasses
    w = W.llama70b_128k()
    w = dataclasses.replace(w, name="llama70b_128k_tp8_rank", shape=dataclasses.replace(w.shape, num_kv_heads=1))
    say("cfg4 layer, one rank of TP 8", w.shape)
    c = H.LayerCase.from_workload(w)
    assert c.bb == 4096
    H.check_everything(orc, c)
    H.check_layer_restore(orc, c, layer=79, cu_budget=16)


def _full_pool_sampled(orc, H, w, sample_layers, n_stage=4):
    """Every layer of the workload resident, each restored by its own launch as bench.py does it; the layers
    in `sample_layers` hold seeded values and are compared with the oracle plane by plane, and the save of
    those layers is compared object by object."""
    s = w.shape
    bb = s.block_tokens * s.num_kv_heads * s.head_dim * s.elt_bytes
    plane_bytes = s.num_blocks * bb
    payload = 2 * int(w.block_table.size) * bb
    import gc
    gc.collect()
    torch.cuda.empty_cache()          # earlier tests' blocks are cached by the allocator, not free
    free, _ = torch.cuda.mem_get_info()
    need = s.num_layers * 2 * plane_bytes + n_stage * payload + (6 << 30)
    if free < need:
        pytest.skip(f"needs {need >> 30} GiB of free HBM for the whole pool, {free >> 30} GiB free")
    geom = dict(num_blocks=s.num_blocks, block_tokens=s.block_tokens, num_kv_heads=s.num_kv_heads, head_dim=s.head_dim,
                elt_bytes=s.elt_bytes)
    cfg = B.make_cfg(w.align, w.chunk_bytes, s.num_layers)
    planes = []
    for l in range(s.num_layers):
        if l in sample_layers:
            k = W.device_values(W.seed_for(w.cfg_id, l), plane_bytes // 2, s.dtype, H.DEV).view(torch.uint8)
            v = W.device_values(W.seed_for(w.cfg_id, l) + 500, plane_bytes // 2, s.dtype, H.DEV).view(torch.uint8)
        else:
            k = torch.empty(plane_bytes, dtype=torch.uint8, device=H.DEV)
            v = torch.empty(plane_bytes, dtype=torch.uint8, device=H.DEV)
        planes.append((k, v))
    before = {l: (planes[l][0].cpu().numpy(), planes[l][1].cpu().numpy()) for l in sample_layers}
    g = torch.Generator(device=H.DEV)
    g.manual_seed(77)
    stages = [torch.randint(0, 256, (payload,), dtype=torch.uint8, device=H.DEV, generator=g) for _ in range(n_stage)]
    d_n, d_tab, d_fid = H.to_dev(w.n_blocks), H.to_dev(w.block_table), H.to_dev(w.file_id)
    ext = torch.zeros(32 * w.n_req, dtype=torch.uint8, device=H.DEV)
    tot = torch.zeros(2, dtype=torch.int64, device=H.DEV)
    n_sqe = int(2 * np.sum((w.n_blocks.astype(np.int64) * bb + w.chunk_bytes - 1) // w.chunk_bytes))
    sqe = torch.zeros(s.num_layers, n_sqe * 64, dtype=torch.uint8, device=H.DEV)
    st = H.new_status()
    n_tab = int(w.block_table.size)
    for l in range(s.num_layers):          # the restore train
        stg = stages[l % n_stage]
        B.tutti_layer_restore(B.make_pool(*planes[l], **geom), cfg, d_n, w.n_req, d_tab, n_tab, d_fid, l, stg, payload,
                              stg.data_ptr(), 1, ext, tot, sqe[l], n_sqe, 0, st)
    torch.cuda.synchronize()
    assert int(st.item()) == 0
    ocfg = orc.make_cfg(w.align, w.chunk_bytes, s.num_layers)
    for l in sample_layers:
        say("  sampled layer", l)
        ok, ov = before[l]
        stg = stages[l % n_stage]
        o_ext, o_tot, o_sqe, o_st = orc.layer_restore(orc.make_pool(ok, ov, **geom), ocfg, w.n_blocks, w.block_table,
                                                      w.file_id, l, stg.cpu().numpy(), stg.data_ptr(), 1, n_sqe)
        assert np.array_equal(planes[l][0].cpu().numpy(), ok), f"layer {l}: K plane differs"
        assert np.array_equal(planes[l][1].cpu().numpy(), ov), f"layer {l}: V plane differs"
        assert sqe[l].cpu().numpy().tobytes() == o_sqe.tobytes() and o_st == 0
        # and the save of that layer back into a fresh staging buffer
        out = torch.zeros(payload, dtype=torch.uint8, device=H.DEV)
        B.tutti_layer_save(B.make_pool(*planes[l], **geom), cfg, d_n, w.n_req, d_tab, n_tab, d_fid, l, out, payload,
                           out.data_ptr(), 1, ext, tot, sqe[l], n_sqe, 0, st)
        torch.cuda.synchronize()
        o_out = np.zeros(payload, np.uint8)
        orc.obj_pack(orc.make_pool(ok, ov, **geom), ocfg, o_ext, w.block_table, o_out)
        assert np.array_equal(out.cpu().numpy(), o_out), f"layer {l}: saved objects differ"
        assert np.array_equal(out.cpu().numpy(), stg.cpu().numpy()), "save after restore returns the staged bytes"
        del out
    assert int(st.item()) == 0
    del planes, stages, before
    gc.collect()
    torch.cuda.empty_cache()


def test_cfg2_whole_pool_sampled_layers(orc, H):
    """Config 2 as bench.py runs it: all 32 layers resident (128 GiB of planes), one launch per layer."""
    w = W.llama8b_32k()
    say("cfg2 whole pool")
    _full_pool_sampled(orc, H, w, sample_layers=(0, 13, 31))


def test_cfg4_whole_pool_sampled_layers(orc, H):
    """Config 4 at its full size: 80 layers x 38146 blocks = 200 GB of planes, fragmented 8192-block table."""
    w = W.llama70b_128k()
    say("cfg4 whole pool")
    _full_pool_sampled(orc, H, w, sample_layers=(0, 41, 79))


@pytest.mark.parametrize("budget", [8, 16, 32, 64])
def test_cfg5_cu_budget_with_concurrent_gemm(orc, H, budget):
    """Config 5: the restore under a CU budget while a bf16 4096^3 GEMM runs on another stream."""
    w = W.llama8b_32k(num_blocks=8192)
    say("cfg5 budget", budget)
    c = H.LayerCase.from_workload(w)
    a = torch.randn(4096, 4096, dtype=torch.bfloat16, device=H.DEV)
    b = torch.randn(4096, 4096, dtype=torch.bfloat16, device=H.DEV)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        for _ in range(20):
            cmat = a @ b
    H.check_layer_restore(orc, c, cu_budget=budget)
    ext, tot, o_ext, o_tot = H.check_layout(orc, c)
    H.check_unpack(orc, c, ext, o_ext, o_tot, cu_budget=budget)
    H.check_pack(orc, c, ext, o_ext, o_tot, cu_budget=budget)
    side.synchronize()
    assert torch.isfinite(cmat.float()).all()
