"""Where a pool's planes sit in HBM: a set-up step, run once when the pool is created (the pool is registered once
and fixed for the engine's life: sec. 3.1 "Scalable GPU File Pool").

Measured on the MI355X: its 288 GB of HBM3E behave as three regions of 96 GB (in a fresh process the first 94 GiB
the driver hands out are one region, the next 96 GiB the second, the rest the third; later processes get them in a
shuffled order, still in pieces of 2 GiB or more).  A restore scatters 32 KiB blocks over a layer's K plane and
then over its V plane.  When the two planes lie in DIFFERENT regions the restore of the Llama-3-8B shape runs at
the speed of a contiguous copy (44 us per 128 MiB layer); when they lie in the same region it takes 51-52 us,
whatever the staging buffer's place and whatever the block table.  Nothing in an address tells the region, so the
planes are classified by timing: the real restore call on the pool (reference plane, candidate plane) is slow
exactly when both are in one region.  `classify_planes` does that for a list of candidate buffers, `choose_pairs`
then gives every layer a K plane and a V plane from different regions.

The timing, the classification and the pairing are the library's (tutti_place_classify, tutti_place_pair_times,
tutti_place_pairs of the C ABI); this module lends them their work memory and turns lists of tensors into pointer
arrays.  `classify_planes` OVERWRITES blocks of the candidates: run it before the pool is filled.
"""
from . import binding as B


def _work(torch, device):
    return torch.empty(B.tutti_place_work_bytes(), dtype=torch.uint8, device=device)


def _plane_bytes(planes):
    sizes = {int(p.numel()) * int(p.element_size()) for p in planes}
    if len(sizes) != 1:
        raise ValueError("candidate planes must have one size")
    return sizes.pop()


def pair_times(ref, cands, device="cuda:0", reps=3):
    """Microseconds of the probe restore on the pool (ref, c) for every candidate c (median of `reps`)."""
    import torch
    work = _work(torch, device)
    return B.tutti_place_pair_times(ref, cands, _plane_bytes([ref] + list(cands)), work, work.numel(), reps)


def classify_planes(planes, device="cuda:0", max_regions=3, min_gap_us=3.0):
    """Region class (0, 1, 2; -1 = could not be told) of every buffer in `planes` (torch tensors of one size on
    `device`, at least 128 MiB each).  Returns (classes, report); `report` holds what every round measured: its
    reference, the time of the pool (reference, reference) (one region by construction: the slow case), the
    fastest pool of the round, and how many planes joined the reference's class.  OVERWRITES blocks of the buffers."""
    import torch
    if not planes:
        return [], {"rounds": []}
    work = _work(torch, device)
    classes, rounds = B.tutti_place_classify(planes, _plane_bytes(planes), work, work.numel(), max_regions, min_gap_us)
    return classes, {"rounds": [{"reference": r.reference, "same_region_us": round(r.same_region_us, 1),
                                "fastest_us": round(r.fastest_us, 1), "members": r.members} for r in rounds]}


def choose_pairs(classes, n_pairs, strict=True):
    """n_pairs pairs (i, j) of buffer indices with classes[i] != classes[j], every buffer used at most once, buffers
    of class -1 never; taken greedily from the two classes with the most buffers left, lowest indices first (which
    forms as many such pairs as any pairing can).  If the classes do not allow n_pairs of them: ValueError when
    strict, else the list is filled up with pairs of what is left (same region, or unclassified), lowest indices
    first; ValueError if even that does not give n_pairs."""
    try:
        pairs, _ = B.tutti_place_pairs(classes, n_pairs, strict)
    except B.TuttiError as err:
        if err.code == B.EAGAIN:
            raise ValueError(f"fewer than {n_pairs} pairs with planes in different regions can be formed") from err
        if err.code == B.ERANGE:
            raise ValueError(f"{len(classes)} buffers do not make {n_pairs} pairs") from err
        raise
    return pairs


def same_region_pairs(classes, n_pairs):
    """Up to n_pairs pairs (i, j) with classes[i] == classes[j] >= 0 (the layout to compare against)."""
    left = {}
    for i, c in enumerate(classes):
        if c >= 0:
            left.setdefault(c, []).append(i)
    pairs = []
    for c in sorted(left):
        idx = left[c]
        while len(idx) >= 2 and len(pairs) < n_pairs:
            pairs.append((idx.pop(0), idx.pop(0)))
    return pairs
