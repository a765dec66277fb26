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

This module only measures and chooses; the data path is the library's (`binding`), called through the same C ABI
as everywhere else.  `classify_planes` OVERWRITES blocks of the candidates: run it before the pool is filled.
"""
import numpy as np

from . import binding as B

# the probe: a restore of 2048 blocks of 32 KiB (128 MiB of payload), the shape the effect was measured with
_PROBE_BLOCK_TOKENS, _PROBE_HEADS, _PROBE_DIM, _PROBE_ELT = 16, 8, 128, 2
_PROBE_BLOCK_BYTES = _PROBE_BLOCK_TOKENS * _PROBE_HEADS * _PROBE_DIM * _PROBE_ELT
_PROBE_BLOCKS = 2048


class _Probe:
    """The buffers of the probe restore, allocated once per classification."""

    def __init__(self, torch, plane_bytes, device, seed=20260503):
        self.torch = torch
        self.num_blocks = plane_bytes // _PROBE_BLOCK_BYTES
        if self.num_blocks < 2 * _PROBE_BLOCKS:
            raise ValueError("planes of at least 128 MiB are needed to tell the regions apart by timing")
        rng = np.random.default_rng(seed)
        table = rng.permutation(self.num_blocks)[:_PROBE_BLOCKS].astype(np.uint32)
        self.payload = 2 * _PROBE_BLOCKS * _PROBE_BLOCK_BYTES
        self.d_tab = torch.from_numpy(table.view(np.int32)).to(device)
        self.d_n = torch.tensor([_PROBE_BLOCKS], dtype=torch.int32, device=device)
        self.d_fid = torch.tensor([1], dtype=torch.int32, device=device)
        self.stage = torch.zeros(self.payload, dtype=torch.uint8, device=device)
        self.ext = torch.zeros(32, dtype=torch.uint8, device=device)
        self.tot = torch.zeros(2, dtype=torch.int64, device=device)
        self.status = torch.zeros(1, dtype=torch.int32, device=device)
        self.n_sqe = 2 * ((_PROBE_BLOCKS * _PROBE_BLOCK_BYTES + (2 << 20) - 1) // (2 << 20))
        self.sqe = torch.zeros(self.n_sqe * 64, dtype=torch.uint8, device=device)
        self.cfg = B.make_cfg(4096, 2 << 20, 1)
        self.geom = dict(num_blocks=self.num_blocks, block_tokens=_PROBE_BLOCK_TOKENS, num_kv_heads=_PROBE_HEADS,
                         head_dim=_PROBE_DIM, elt_bytes=_PROBE_ELT)

    def pair_times(self, ref, cands, reps=3):
        """Microseconds of the probe restore on the pool (ref, c) for every candidate c (median of `reps`; each figure
        includes the gap between two launches, the same for all)."""
        torch = self.torch
        pools = [B.make_pool(ref, c, **self.geom) for c in cands]
        n = len(pools)
        acc = np.zeros((reps, n))

        def launch(p):
            B.tutti_layer_restore(p, self.cfg, self.d_n, 1, self.d_tab, _PROBE_BLOCKS, self.d_fid, 0, self.stage,
                                  self.payload, self.stage.data_ptr(), 1, self.ext, self.tot, self.sqe, self.n_sqe, 0,
                                  self.status)

        for rep in range(reps + 1):                    # the first pass warms up
            ev = [torch.cuda.Event(enable_timing=True) for _ in range(n + 1)]
            launch(pools[-1])                          # so that the first timed launch does not start an idle queue
            for i, p in enumerate(pools):
                ev[i].record()
                launch(p)
            ev[n].record()
            torch.cuda.synchronize()
            if rep:
                acc[rep - 1] = [ev[i].elapsed_time(ev[i + 1]) * 1e3 for i in range(n)]
        return np.median(acc, axis=0)


def classify_planes(planes, device="cuda:0", max_regions=3, min_gap_us=3.0):
    """Region class (0, 1, 2; -1 = could not be told) of every buffer in `planes` (uint8 torch tensors of one size on
    `device`, at least 128 MiB each).  Returns (classes, report); `report` holds the measured times of every round.

    Round c takes the first unclassified buffer as reference r, measures the pool (r, r) (both planes in one region by
    construction: the slow case) and the pools (r, x) for every unclassified x; x joins r's class if its time is nearer
    the slow case than the fastest pair of the round.  A round in which nothing is faster than the slow case by
    `min_gap_us` puts everything left into r's class.  OVERWRITES blocks of the buffers."""
    import torch
    if not planes:
        return [], {"rounds": []}
    sizes = {int(p.numel()) for p in planes}
    if len(sizes) != 1:
        raise ValueError("candidate planes must have one size")
    probe = _Probe(torch, sizes.pop(), device)
    classes = [-1] * len(planes)
    report = {"rounds": []}
    for c in range(max_regions):
        todo = [i for i, k in enumerate(classes) if k < 0]
        if not todo:
            break
        r = todo[0]
        t = probe.pair_times(planes[r], [planes[r]] + [planes[i] for i in todo])
        slow, rest = float(t[0]), t[1:]
        fast = float(rest.min())
        if slow - fast < min_gap_us:                    # nothing left lies in another region
            for i in todo:
                classes[i] = c
            report["rounds"].append({"reference": r, "same_region_us": round(slow, 1), "fastest_us": round(fast, 1),
                                     "members": len(todo)})
            break
        mid = 0.5 * (slow + fast)
        members = 0
        for i, x in zip(todo, rest):
            if x > mid or i == r:
                classes[i] = c
                members += 1
        report["rounds"].append({"reference": r, "same_region_us": round(slow, 1), "fastest_us": round(fast, 1),
                                 "members": members})
    if int(probe.status.item()) != 0:
        raise RuntimeError("the probe restore reported a device status")
    return classes, report


def choose_pairs(classes, n_pairs, strict=True):
    """n_pairs pairs (i, j) of buffer indices with classes[i] != classes[j], every buffer used at most once, buffers
    of class -1 never; taken greedily from the two classes with the most buffers left, lowest indices first (which
    forms as many such pairs as any pairing can).  If the classes do not allow n_pairs of them: ValueError when
    strict, else the list is filled up with pairs of what is left (same region, or unclassified), lowest indices
    first; ValueError if even that does not give n_pairs."""
    left = {}
    for i, c in enumerate(classes):
        if c >= 0:
            left.setdefault(c, []).append(i)
    pairs = []
    while len(pairs) < n_pairs:
        live = sorted((c for c in left if left[c]), key=lambda c: (-len(left[c]), c))
        if len(live) < 2:
            break
        a, b = live[0], live[1]
        pairs.append((left[a].pop(0), left[b].pop(0)))
    if len(pairs) < n_pairs:
        if strict:
            raise ValueError(f"only {len(pairs)} of {n_pairs} pairs with planes in different regions can be formed")
        used = {i for p in pairs for i in p}
        rest = [i for i in range(len(classes)) if i not in used]
        while len(pairs) < n_pairs and len(rest) >= 2:
            pairs.append((rest.pop(0), rest.pop(0)))
        if len(pairs) < n_pairs:
            raise ValueError(f"{len(classes)} buffers do not make {n_pairs} pairs")
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
