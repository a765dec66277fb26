"""Seeded synthetic inputs for the per-layer KV object path.

This module serves both the HIP path and the CPU oracle and therefore holds none of the
method's arithmetic: it only draws shapes, per-request block counts, block tables, file
ids and pool contents.  Everything is synthetic; the request-length mixes stand in for the
long-context suites the paper serves (sec. 4 "Workloads": inputs of 3K-200K tokens; fixed
32K / 64K / 128K prefixes in the ablations) without reproducing any item of them.

numpy only at import time; torch is imported inside the device fill helpers.
"""
from dataclasses import dataclass, field, replace

import numpy as np

BASE_SEED = 20260503


def seed_for(cfg_id: int, layer: int = 0) -> int:
    return BASE_SEED + 1000 * cfg_id + layer


@dataclass(frozen=True)
class KVShape:
    """Shape of one layer's paged pool.  dtype is a name only ("fp16" / "bf16")."""
    num_layers: int
    dtype: str
    elt_bytes: int
    block_tokens: int
    num_kv_heads: int
    head_dim: int
    num_blocks: int


@dataclass
class Workload:
    name: str
    cfg_id: int
    shape: KVShape
    n_blocks: np.ndarray      # uint32 [R]   hit blocks per request
    block_table: np.ndarray   # uint32 [sum n_blocks]  flattened, request after request
    file_id: np.ndarray       # uint32 [R]
    align: int = 4096
    chunk_bytes: int = 2 << 20
    seed: int = 0
    notes: dict = field(default_factory=dict)

    @property
    def n_req(self) -> int:
        return int(self.n_blocks.size)


def _zipf_ranks(rng, n, s=1.1, k_max=64):
    ranks = np.arange(1, k_max + 1, dtype=np.float64)
    p = ranks ** (-s)
    p /= p.sum()
    return rng.choice(np.arange(1, k_max + 1), size=n, p=p)


def tiny(chunk_bytes: int = 2 << 20) -> Workload:
    """Config 1: 1 layer, fp16, block 16, 2 heads x 64, 256 blocks, one 512-token prefix."""
    seed = seed_for(1)
    rng = np.random.default_rng(seed)
    shape = KVShape(1, "fp16", 2, 16, 2, 64, 256)
    table = rng.permutation(shape.num_blocks)[:32].astype(np.uint32)
    return Workload("tiny", 1, shape, np.array([32], np.uint32), table, np.array([1000], np.uint32),
                    chunk_bytes=chunk_bytes, seed=seed)


def llama8b_32k(num_blocks: int = 65536, tokens: int = 32768, num_layers: int = 32) -> Workload:
    """Config 2: 32 layers, bf16, block 16, 8 heads x 128, one 32K-token prefix, shuffled table."""
    seed = seed_for(2)
    rng = np.random.default_rng(seed)
    shape = KVShape(num_layers, "bf16", 2, 16, 8, 128, num_blocks)
    n = tokens // shape.block_tokens
    table = rng.permutation(num_blocks)[:n].astype(np.uint32)
    return Workload("llama8b_32k", 2, shape, np.array([n], np.uint32), table, np.array([1000], np.uint32),
                    chunk_bytes=2 << 20, seed=seed)


def batch64_zipf(n_req: int = 64, num_blocks: int = 65536, chunk_bytes: int = 2 << 20, len_unit: int = 1024,
                 num_layers: int = 32) -> Workload:
    """Config 3: 64 requests, lengths len_unit*Zipf(1.1) over ranks 1..64, hit fraction U[0.3,1.0).

    Reading of "Zipf over [1K, 64K] tokens": the rank is the length in Ki-tokens.  Only whole hit
    blocks count.  All requests' blocks are drawn without replacement from one permutation, so the
    tables are disjoint; the pool grows in steps of 65536 blocks if the hits do not fit.
    """
    seed = seed_for(3)
    rng = np.random.default_rng(seed)
    ranks = _zipf_ranks(rng, n_req)
    lens = len_unit * ranks
    frac = rng.uniform(0.3, 1.0, size=n_req)
    block_tokens = 16
    n_blocks = np.floor(lens * frac / block_tokens).astype(np.uint32)
    total = int(n_blocks.sum())
    nb = num_blocks
    while nb < total:
        nb += 65536
    shape = KVShape(num_layers, "bf16", 2, block_tokens, 8, 128, nb)
    table = rng.permutation(nb)[:total].astype(np.uint32)
    file_id = (1000 + np.arange(n_req)).astype(np.uint32)
    return Workload("batch64_zipf", 3, shape, n_blocks, table, file_id, chunk_bytes=chunk_bytes, seed=seed,
                    notes={"lens": lens, "frac": frac})


def fragmented_table(rng, num_blocks: int, want: int, rounds: int = 20000) -> np.ndarray:
    """Block ids handed out by a LIFO free list after `rounds` of allocate / free churn.

    The list starts as 0..num_blocks-1 (top of stack = last element).  Each round either allocates
    a sequence of 64*Zipf(1.1) blocks or frees a uniformly chosen live sequence, pushing its blocks
    back in sequence order; allocation is forced to a free when the list cannot satisfy it.  Then
    live sequences are freed in random order until `want` blocks are free, and `want` are popped.
    The result mixes short contiguous runs with far jumps.
    """
    free = list(range(num_blocks))
    live = []
    for _ in range(rounds):
        do_alloc = rng.random() < 0.5
        need = 64 * int(_zipf_ranks(rng, 1)[0])
        if do_alloc and need <= len(free):
            seq = [free.pop() for _ in range(need)]
            live.append(seq)
        elif live:
            seq = live.pop(int(rng.integers(len(live))))
            free.extend(seq)
    order = rng.permutation(len(live))
    for idx in order:
        if len(free) >= want:
            break
        free.extend(live[idx])
    if len(free) < want:
        raise ValueError("pool too small for the requested prefix")
    return np.array([free.pop() for _ in range(want)], dtype=np.uint32)


def llama70b_128k(num_blocks: int = 38146, tokens: int = 131072, num_layers: int = 80) -> Workload:
    """Config 4: 80 layers, bf16, same block shape, 128K-token prefix, fragmented free-list table.

    38146 blocks = floor(200e9 B / (80 layers * 2 planes * 32 KiB)): a pool of 200 GB of HBM.
    """
    seed = seed_for(4)
    rng = np.random.default_rng(seed)
    shape = KVShape(num_layers, "bf16", 2, 16, 8, 128, num_blocks)
    n = tokens // shape.block_tokens
    table = fragmented_table(rng, num_blocks, n)
    return Workload("llama70b_128k", 4, shape, np.array([n], np.uint32), table, np.array([1000], np.uint32),
                    chunk_bytes=2 << 20, seed=seed)


def corun() -> Workload:
    """Config 5: config 2's layer restore, launched under a CU budget beside a GEMM."""
    w = llama8b_32k()
    return replace(w, name="corun_8b_32k", cfg_id=5)


def scaled(w: Workload, num_layers: int) -> Workload:
    """Same workload with fewer layers resident (pool memory shortfall); tables unchanged."""
    return replace(w, shape=replace(w.shape, num_layers=num_layers))


# ---------------------------------------------------------------------------- pool contents

def host_values(seed: int, n_elts: int, dtype: str) -> np.ndarray:
    """n_elts seeded uniform[-1,1) values as raw 16-bit patterns (uint16) of fp16 or bf16."""
    rng = np.random.default_rng(seed)
    x = rng.uniform(-1.0, 1.0, size=n_elts).astype(np.float32)
    if dtype == "fp16":
        return x.astype(np.float16).view(np.uint16)
    if dtype == "bf16":
        return (x.view(np.uint32) >> 16).astype(np.uint16)
    raise ValueError(dtype)


def host_address_tags(n_bytes: int, base_word: int = 0) -> np.ndarray:
    """n_bytes (multiple of 4) of address tags: 32-bit word w holds base_word + w, as uint8."""
    return (np.arange(n_bytes // 4, dtype=np.uint64) + base_word).astype(np.uint32).view(np.uint8)


def device_values(seed: int, n_elts: int, dtype: str, device="cuda", out=None):
    """Seeded uniform[-1,1) fp16 / bf16 values drawn on the device (a torch tensor).  `out`: a tensor of n_elts
    elements of that dtype to fill in place (a buffer whose place in memory was chosen beforehand)."""
    import torch
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    td = {"fp16": torch.float16, "bf16": torch.bfloat16}[dtype]
    if out is None:
        out = torch.empty(n_elts, dtype=td, device=device)
    assert out.dtype == td and out.numel() == n_elts
    step = 1 << 28
    for lo in range(0, n_elts, step):
        out[lo:lo + step].uniform_(-1.0, 1.0, generator=g)
    return out


def device_address_tags(n_bytes: int, base_word: int = 0, device="cuda"):
    """Address tags as on the host, generated on the device (uint8 tensor of n_bytes)."""
    import torch
    w = torch.arange(base_word, base_word + n_bytes // 4, dtype=torch.int64, device=device) & 0xFFFFFFFF
    w = torch.where(w >= (1 << 31), w - (1 << 32), w)
    return w.to(torch.int32).view(torch.uint8)
