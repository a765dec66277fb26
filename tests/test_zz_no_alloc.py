"""GPU test of the entry point that allocates nothing: tutti_table_validate_static (the bitmap lives in a static
device array of the library) against tutti_table_validate_ws (the bitmap is lent by the caller), the entry point
it is a variant of.  Two calls in a row, the second on a smaller input: the array keeps the first call's bits,
and the second call must not see them."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

from paper_2605_03375_amd import binding as B      # noqa: E402

DEV = "cuda:0"


def _dev(a):
    return torch.from_numpy(np.ascontiguousarray(a, np.uint32).view(np.int32)).to(DEV)


def _both(num_blocks, table):
    """Status words of the static-array call and of the lent-workspace call on the same table."""
    d_table = _dev(table)
    st_static = torch.zeros(1, dtype=torch.int32, device=DEV)
    st_ws = torch.zeros(1, dtype=torch.int32, device=DEV)
    work = torch.empty(B.tutti_table_validate_work_bytes(num_blocks), dtype=torch.uint8, device=DEV)
    B.tutti_table_validate_static(num_blocks, d_table, table.size, st_static)
    B.tutti_table_validate_ws(num_blocks, d_table, table.size, st_ws, work, work.numel())
    torch.cuda.synchronize()
    return int(st_static.item()), int(st_ws.item())


def test_static_array_variant_matches_the_workspace_variant():
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU")
    B.lib()
    print("no-alloc entry point: tutti_table_validate_static", flush=True)
    rng = np.random.default_rng(2605)
    # first call: 300,000 distinct ids out of a million, one duplicate planted -> DUP
    N1 = 1_000_000
    t1 = rng.permutation(N1)[:300_000].astype(np.uint32)
    t1[123_456] = t1[7]
    a, b = _both(N1, t1)
    assert a == b == B.ST_DUP_BLOCK
    # second call, smaller: ids the first call has left set in the array; a clean table must come out clean
    N2 = 70_000
    t2 = np.unique(t1[t1 < N2])[:20_000].astype(np.uint32)
    assert t2.size > 1000
    a, b = _both(N2, t2)
    assert a == b == 0
    # ... and with an id out of range and a duplicate
    t3 = t2.copy()
    t3[5], t3[-1] = N2 + 3, t3[0]
    a, b = _both(N2, t3)
    assert a == b == (B.ST_BAD_BLOCK | B.ST_DUP_BLOCK)
    # third call larger again, clean
    a, b = _both(N1, rng.permutation(N1)[:500_000].astype(np.uint32))
    assert a == b == 0
    # sizes beyond the static array are refused before anything is enqueued
    st = torch.zeros(1, dtype=torch.int32, device=DEV)
    with pytest.raises(B.TuttiError) as ei:
        B.tutti_table_validate_static(B.STATIC_VALIDATE_MAX_BLOCKS + 1, _dev(t2), t2.size, st)
    assert ei.value.code == B.ERANGE and "static" in str(ei.value)
    # the largest size it covers
    big = rng.permutation(B.STATIC_VALIDATE_MAX_BLOCKS)[:100_000].astype(np.uint32)
    a, b = _both(B.STATIC_VALIDATE_MAX_BLOCKS, big)
    assert a == b == 0
    # the static calls take no device memory: free memory as the driver reports it does not move
    d_t2 = _dev(t2)
    st.zero_()
    torch.cuda.synchronize()
    before = torch.cuda.mem_get_info()[0]
    for _ in range(5):
        B.tutti_table_validate_static(N2, d_t2, t2.size, st)
    torch.cuda.synchronize()
    assert torch.cuda.mem_get_info()[0] == before and int(st.item()) == 0
