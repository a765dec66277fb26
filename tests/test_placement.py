"""The pool-placement helper: the pairing logic on the CPU, the timing probe on the GPU."""
import numpy as np
import pytest

from paper_2605_03375_amd import placement as P


def test_choose_pairs_only_pairs_different_regions():
    rng = np.random.default_rng(3)
    for _ in range(200):
        n = int(rng.integers(0, 40))
        classes = [int(c) for c in rng.integers(-1, 3, size=n)]
        counts = [classes.count(c) for c in range(3)]
        most = min(sum(counts) // 2, sum(counts) - max(counts)) if counts else 0      # what any pairing can reach
        pairs = P.choose_pairs(classes, most)
        used = [i for p in pairs for i in p]
        assert len(pairs) == most and len(set(used)) == len(used)
        assert all(classes[i] >= 0 and classes[j] >= 0 and classes[i] != classes[j] for i, j in pairs)
        with pytest.raises(ValueError):
            P.choose_pairs(classes, most + 1)
    # a fresh process: the first 47 planes of 2 GiB in one region, the next 48 in another, one in the third
    classes = [0] * 47 + [1] * 48 + [2]
    pairs = P.choose_pairs(classes, 32)
    assert len(pairs) == 32 and all(classes[i] != classes[j] for i, j in pairs)
    assert P.choose_pairs([], 0) == []
    # best effort: as many pairs from two regions as there can be, then whatever is left, and never a buffer twice
    classes = [0, 0, 0, 0, 1, -1, -1, 0]
    pairs = P.choose_pairs(classes, 4, strict=False)
    assert pairs[0] == (0, 4) and len(pairs) == 4 and sorted(i for p in pairs for i in p) == list(range(8))
    with pytest.raises(ValueError):
        P.choose_pairs(classes, 5, strict=False)


def test_pairing_is_as_good_as_any_on_small_cases():
    """Brute force over every way to pair up to 7 planes: none forms more pairs from different regions."""
    import itertools

    def best(classes, idx):
        if len(idx) < 2:
            return 0
        first, rest = idx[0], idx[1:]
        out = best(classes, rest)                                      # `first` stays single
        for k, other in enumerate(rest):
            if classes[first] != classes[other]:
                out = max(out, 1 + best(classes, rest[:k] + rest[k + 1:]))
        return out

    for n in range(0, 8):
        for classes in itertools.product((-1, 0, 1, 2), repeat=n):
            idx = [i for i, c in enumerate(classes) if c >= 0]
            most = best(classes, idx)
            pairs, n_mixed = P.B.tutti_place_pairs(list(classes), most, strict=True)
            assert n_mixed == most and all(classes[i] != classes[j] and min(classes[i], classes[j]) >= 0
                                           for i, j in pairs)
            assert len({i for p in pairs for i in p}) == 2 * most


def test_place_arguments_are_checked_before_any_gpu_call():
    B = P.B
    L = B.lib()
    import ctypes as C
    cls = (C.c_int32 * 2)(0, 9)
    out = (C.c_uint32 * 2)()
    assert L.tutti_place_pairs(cls, 2, 1, 1, out, None) == B.EINVAL          # class beyond TUTTI_PLACE_MAX_REGIONS
    assert L.tutti_place_pairs(None, 2, 1, 1, out, None) == B.EINVAL
    assert L.tutti_place_pairs((C.c_int32 * 2)(0, 1), 2, 1, 1, None, None) == B.EINVAL
    assert L.tutti_place_work_bytes() == (128 << 20) + 65536
    planes = (C.c_void_p * 2)(0x1000, 0x2000)
    us = (C.c_float * 2)()
    cl = (C.c_int32 * 2)()
    big, work = 1 << 30, L.tutti_place_work_bytes()
    # every one of these returns before the probe touches the device
    assert L.tutti_place_pair_times(0x1000, planes, 0, big, 0x10000, work, 3, us, None) == B.EINVAL      # no candidates
    assert L.tutti_place_pair_times(None, planes, 2, big, 0x10000, work, 3, us, None) == B.EINVAL
    assert L.tutti_place_pair_times(0x1000, planes, 2, big, 0x10000, work, 0, us, None) == B.EINVAL      # reps
    assert L.tutti_place_pair_times(0x1000, planes, 2, big, 0x10000, work, 17, us, None) == B.EINVAL
    assert L.tutti_place_pair_times(0x1000, planes, 2, big, 0x10000, work, 3, None, None) == B.EINVAL
    assert L.tutti_place_pair_times(0x1000, planes, 2, big, None, work, 3, us, None) == B.EINVAL
    assert L.tutti_place_pair_times(0x1000, planes, 2, big, 0x10010, work, 3, us, None) == B.EINVAL      # work alignment
    assert L.tutti_place_pair_times(0x1000, planes, 2, big, 0x10000, work - 1, 3, us, None) == B.ERANGE
    assert L.tutti_place_pair_times(0x1000, planes, 2, (128 << 20) - 16, 0x10000, work, 3, us, None) == B.ERANGE
    assert L.tutti_place_pair_times(0x1008, planes, 2, big, 0x10000, work, 3, us, None) == B.EINVAL      # plane alignment
    assert L.tutti_place_classify(planes, 2, big, 0x10000, work, 0, 3.0, cl, None, None, None) == B.EINVAL
    assert L.tutti_place_classify(planes, 2, big, 0x10000, work, 9, 3.0, cl, None, None, None) == B.EINVAL
    assert L.tutti_place_classify(planes, 2, big, 0x10000, work, 3, -1.0, cl, None, None, None) == B.EINVAL
    assert L.tutti_place_classify(planes, 2, big, 0x10000, work, 3, 3.0, None, None, None, None) == B.EINVAL
    assert L.tutti_place_classify(planes, 2, big, 0x10000, work - 1, 3, 3.0, cl, None, None, None) == B.ERANGE
    assert L.tutti_place_classify(None, 2, big, 0x10000, work, 3, 3.0, cl, None, None, None) == B.EINVAL


def test_same_region_pairs():
    classes = [0, 0, 1, 1, 1, 2, -1, 0, 0]
    pairs = P.same_region_pairs(classes, 10)
    assert pairs == [(0, 1), (7, 8), (2, 3)]
    assert P.same_region_pairs(classes, 1) == [(0, 1)]
    assert P.same_region_pairs([0, 1, 2], 3) == []


@pytest.mark.gpu
def test_classification_by_timing_agrees_with_direct_pair_timings():
    """100 GiB of 2 GiB candidates reach into a second HBM region whatever order the driver hands memory out in.
    The classes found must be consistent with direct timings of pairs that were not used to find them: a pair from
    one class is slower than a pair from two classes.  Skipped (not failed) if only one region is found."""
    import torch
    dev = "cuda:0"
    import gc
    gc.collect()
    torch.cuda.empty_cache()          # earlier tests' blocks are cached by the allocator, not free
    free, _ = torch.cuda.mem_get_info()
    n = int(min(50, (free - (8 << 30)) // (2 << 30)))
    if n < 8:
        pytest.skip("not enough free HBM for the candidates")
    cands = [torch.empty(2 << 30, dtype=torch.uint8, device=dev) for _ in range(n)]
    classes, report = P.classify_planes(cands, dev)
    print("regions in allocation order:", "".join("ABC?"[c] for c in classes), report)
    assert len(classes) == n and set(classes) <= {-1, 0, 1, 2} and classes[0] == 0
    if len({c for c in classes if c >= 0}) < 2:
        pytest.skip("all candidates lie in one region on this box")
    mixed = P.choose_pairs(classes, 3)
    same = P.same_region_pairs(classes, 3)
    t_mixed = [P.pair_times(cands[i], [cands[j]], dev)[0] for i, j in mixed]
    t_same = [P.pair_times(cands[i], [cands[j]], dev)[0] for i, j in same]
    print("pairs from two regions:", t_mixed, "pairs within a region:", t_same)
    # medians: one launch disturbed by something else on the box must not decide the test
    assert float(np.median(t_mixed)) + 2.0 < float(np.median(t_same)), (t_mixed, t_same)
