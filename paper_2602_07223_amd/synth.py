"""Seeded synthetic inputs shaped like the paper's long-context decoding workloads.

This module only *draws inputs*: tensors, page tables, lengths.  It holds none of the
method's arithmetic (no attention, no scores, no selection) so that both the CPU oracle
tests and the HIP path can be fed from it without sharing any computation.

Everything is host-side NumPy.  bf16 tensors are returned as ``uint16`` bit patterns
(round-to-nearest-even from float32).

Workloads stand in for the datasets the paper evaluates on (Sec. 5.1-5.3): only the
shapes carry over -- a Qwen3-8B-like attention shape (32 query / 8 KV heads, head_dim 128,
i.e. 4 KB of K+V per token, App. D), contexts of 4K-128K, small batches at long context,
a KV budget of a few percent of the context, gamma of 4-6.

Draw order inside one ``make_layer`` call (fixed; changing it changes every tensor):
  1. seq_lens                      (ragged configs only)
  2. physical page permutation     (shuffled configs only)
  3. K pool, V pool (physical order; jumped streams of the same seed, see normal_pool_bf16)
  4. verify-query normals
  5. per (sequence, KV head) directions u [, v_old, v_new]
  6. hitter run starts / positions per sequence [, drift positions]
  7. draft-query noise
"""
from __future__ import annotations

import dataclasses
from typing import Dict, List, Optional

import numpy as np

PAGE = 16
BF16_NAN = np.uint16(0x7FC0)


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """float32 -> bf16 bit pattern, round to nearest even (finite inputs)."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    out = np.empty(x.shape, dtype=np.uint16)
    flat_in, flat_out = x.reshape(-1).view(np.uint32), out.reshape(-1)
    step = 1 << 20                                    # cache-sized pieces, few temporaries
    for i in range(0, flat_in.size, step):
        u = flat_in[i:i + step]
        r = u >> np.uint32(16)
        r &= np.uint32(1)
        r += np.uint32(0x7FFF)
        r += u
        r >>= np.uint32(16)
        flat_out[i:i + step] = r
    return out


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """bf16 bit pattern -> float32 (exact)."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


@dataclasses.dataclass(frozen=True)
class WorkloadSpec:
    """Shape and planting recipe of one synthetic workload."""
    name: str
    config_id: int              # index used in the seed (1..5 for the baseline configs)
    batch: int
    num_q_heads: int
    num_kv_heads: int
    gamma: int                  # verify rows G = gamma + 1; draft steps = G
    budget_tokens: int
    seq_len: int = 0            # fixed context (0 when ragged)
    seq_len_lo: int = 0         # ragged: integer-uniform in [lo, hi]
    seq_len_hi: int = 0
    head_dim: int = 128
    layers: int = 1
    shuffle_pages: bool = False
    spare_pages: int = 0        # extra NaN-poisoned pages in the pool
    poison_slack: bool = False  # NaN in the unused slots of partial last pages
    hitters: int = -1           # planted heavy hitters per sequence (-1: seq_len // 256)
    hitter_run: int = 16        # 1 = isolated positions, else contiguous runs of this length
    drift: float = 0.0          # fraction of hitters re-drawn between verify and draft queries
    sink_tokens: int = 4
    sink_gain: float = 4.0
    hitter_gain: float = 3.0
    draft_noise: float = 0.1
    max_blocks: int = 0         # row stride of the block table (0: tight)
    tensor_scale: float = 0.0   # std of Q/K/V elements (0: 1/sqrt(head_dim))

    @property
    def num_queries(self) -> int:
        return self.gamma + 1

    @property
    def group(self) -> int:
        return self.num_q_heads // self.num_kv_heads


# The five baseline configurations.
CONFIGS: Dict[str, WorkloadSpec] = {
    "ctx4k": WorkloadSpec("ctx4k", 1, batch=1, num_q_heads=32, num_kv_heads=8, gamma=4,
                          budget_tokens=256, seq_len=4096, hitters=16, hitter_run=1),
    "ctx32k": WorkloadSpec("ctx32k", 2, batch=1, num_q_heads=32, num_kv_heads=8, gamma=4,
                           budget_tokens=2048, seq_len=32768, hitters=128, hitter_run=16),
    "ctx128k_drift": WorkloadSpec("ctx128k_drift", 3, batch=1, num_q_heads=32, num_kv_heads=8, gamma=6,
                                  budget_tokens=4096, seq_len=131072, drift=0.1),
    "ragged16": WorkloadSpec("ragged16", 4, batch=16, num_q_heads=64, num_kv_heads=8, gamma=4,
                             budget_tokens=2048, seq_len_lo=8192, seq_len_hi=65536,
                             shuffle_pages=True, spare_pages=64, poison_slack=True, max_blocks=4096),
    "stack32": WorkloadSpec("stack32", 5, batch=4, num_q_heads=32, num_kv_heads=8, gamma=4,
                            budget_tokens=4096, seq_len=65536, layers=32),
}


# Beyond the five: the second attention shape the paper evaluates (App. D: 2 KB of K+V per token; a
# gpt-oss-20b-like layer with 64 query / 8 KV heads of dimension 64), at the context of "ctx32k".
EXTRA_CONFIGS: Dict[str, WorkloadSpec] = {
    "hd64_ctx32k": WorkloadSpec("hd64_ctx32k", 6, batch=1, num_q_heads=64, num_kv_heads=8, gamma=4,
                                budget_tokens=2048, seq_len=32768, hitters=128, hitter_run=16, head_dim=64),
    # "ctx32k" at the batch size the paper runs its long-context workloads with (Sec. 2.2, Sec. 5: batch 4)
    "ctx32k_batch4": WorkloadSpec("ctx32k_batch4", 7, batch=4, num_q_heads=32, num_kv_heads=8, gamma=4,
                                  budget_tokens=2048, seq_len=32768, hitters=128, hitter_run=16),
}


def scaled(spec: WorkloadSpec, **changes) -> WorkloadSpec:
    """A copy of ``spec`` with some fields replaced (reduced-size parity cases)."""
    return dataclasses.replace(spec, **changes)


@dataclasses.dataclass
class LayerInputs:
    spec: WorkloadSpec
    layer: int
    seed: int
    q_verify: np.ndarray      # uint16 [B, G, H_q, D]
    q_draft: np.ndarray       # uint16 [G, B, H_q, D]  (one [B, H_q, D] slab per draft step)
    k_cache: np.ndarray       # uint16 [num_pages, 16, H_kv, D]
    v_cache: np.ndarray       # uint16 [num_pages, 16, H_kv, D]
    block_table: np.ndarray   # int32  [B, max_blocks], -1 beyond a sequence's pages
    seq_lens: np.ndarray      # int32  [B]
    softmax_scale: float
    sinks: List[np.ndarray]           # per sequence: planted sink positions
    hitters: List[np.ndarray]         # per sequence: hitter positions the verify queries align with
    draft_hitters: List[np.ndarray]   # per sequence: positions the draft queries align with
    k_new: Optional[np.ndarray] = None    # uint16 [steps, B, 1, H_kv, D]: the K row each draft step appends (with_growth)
    v_new: Optional[np.ndarray] = None

    @property
    def num_pages(self) -> int:
        return int(self.k_cache.shape[0])

    @property
    def max_blocks(self) -> int:
        return int(self.block_table.shape[1])


def with_growth(L: "LayerInputs", steps: int) -> "LayerInputs":
    """A copy of ``L`` prepared for a live drafting phase of ``steps`` appended tokens per sequence: the pool gets
    the extra pages the new positions need (NaN-filled until written), the block table is widened where necessary
    and names them, and k_new / v_new hold the rows each step appends -- N(0, std^2) like the rest of the cache,
    drawn from stream 2 of the layer's seed.  Inputs only: nothing of the method is computed here."""
    B = L.block_table.shape[0]
    Hkv, D = L.k_cache.shape[2], L.k_cache.shape[3]
    nblk = (L.seq_lens.astype(np.int64) + PAGE - 1) // PAGE
    need = (L.seq_lens.astype(np.int64) + steps + PAGE - 1) // PAGE
    extra = (need - nblk).astype(np.int64)
    mb = max(L.max_blocks, int(need.max()))
    table = np.full((B, mb), -1, dtype=np.int32)
    table[:, :L.max_blocks] = L.block_table
    first_new = L.num_pages
    nxt = first_new
    for b in range(B):
        for j in range(int(extra[b])):
            table[b, nblk[b] + j] = nxt
            nxt += 1
    pad = np.full((nxt - first_new, PAGE, Hkv, D), BF16_NAN, dtype=np.uint16)
    std = L.spec.tensor_scale if L.spec.tensor_scale > 0 else 1.0 / np.sqrt(D)
    k_new = normal_pool_bf16(L.seed, 2, (steps * B, 1, Hkv, D), std).reshape(steps, B, 1, Hkv, D)
    v_new = normal_pool_bf16(L.seed, 3, (steps * B, 1, Hkv, D), std).reshape(steps, B, 1, Hkv, D)
    return dataclasses.replace(L, k_cache=np.concatenate([L.k_cache, pad]), v_cache=np.concatenate([L.v_cache, pad]),
                               block_table=table, k_new=k_new, v_new=v_new)


_POOL_CHUNK_PAGES = 1024


def normal_pool_bf16(seed: int, stream: int, shape, std: float, workers: int = 8) -> np.ndarray:
    """bf16 bits of N(0, std^2) samples of `shape`, drawn in pieces of 1024 leading-axis entries.
    Piece c of stream s uses PCG64(seed).jumped(1 + 65536*s + c), so the result does not depend on
    the number of worker threads."""
    from concurrent.futures import ThreadPoolExecutor
    out = np.empty(shape, dtype=np.uint16)
    n0 = shape[0]
    pieces = [(c, lo, min(lo + _POOL_CHUNK_PAGES, n0)) for c, lo in enumerate(range(0, n0, _POOL_CHUNK_PAGES))]

    def work(item):
        c, lo, hi = item
        g = np.random.Generator(np.random.PCG64(seed).jumped(1 + 65536 * stream + c))
        x = g.standard_normal((hi - lo,) + tuple(shape[1:]), dtype=np.float32)
        x *= np.float32(std)
        out[lo:hi] = f32_to_bf16_bits(x)

    with ThreadPoolExecutor(max_workers=max(1, workers)) as ex:
        list(ex.map(work, pieces))
    return out


def _unit_rows(rng: np.random.Generator, shape) -> np.ndarray:
    x = rng.standard_normal(shape, dtype=np.float32)
    x /= np.linalg.norm(x, axis=-1, keepdims=True)
    return x


def _orthogonalise(v: np.ndarray, basis: List[np.ndarray]) -> np.ndarray:
    """Make rows of v orthogonal to the (row-wise orthonormal) rows of each basis array, unit length."""
    v = v.astype(np.float64)
    for u in basis:
        u = u.astype(np.float64)
        v = v - np.sum(v * u, axis=-1, keepdims=True) * u
    v /= np.linalg.norm(v, axis=-1, keepdims=True)
    return v.astype(np.float32)


def _run_starts(rng: np.random.Generator, lo: int, hi: int, runs: int, run: int) -> np.ndarray:
    """``runs`` non-overlapping runs of length ``run`` inside [lo, hi); starts not page-aligned if run>1."""
    starts: List[int] = []
    taken = np.zeros(hi, dtype=bool)
    guard = 0
    while len(starts) < runs:
        guard += 1
        if guard > 100000:
            raise RuntimeError("cannot place hitter runs")
        s = int(rng.integers(lo, hi - run + 1))
        if run > 1 and s % PAGE == 0:
            continue
        if taken[s:s + run].any():
            continue
        taken[s:s + run] = True
        starts.append(s)
    return np.asarray(sorted(starts), dtype=np.int64)


def make_layer(spec: WorkloadSpec, layer: int = 0) -> LayerInputs:
    """Draw one layer's inputs for ``spec``.  Seed = 7223000 + 100*config_id + layer."""
    seed = 7223000 + 100 * spec.config_id + layer
    rng = np.random.Generator(np.random.PCG64(seed))
    B, Hq, Hkv, D, G = spec.batch, spec.num_q_heads, spec.num_kv_heads, spec.head_dim, spec.num_queries
    g = spec.group
    std = spec.tensor_scale if spec.tensor_scale > 0 else 1.0 / np.sqrt(D)

    # 1. lengths
    if spec.seq_len > 0:
        seq_lens = np.full(B, spec.seq_len, dtype=np.int32)
    else:
        seq_lens = rng.integers(spec.seq_len_lo, spec.seq_len_hi + 1, size=B).astype(np.int32)
    nblk = (seq_lens.astype(np.int64) + PAGE - 1) // PAGE
    used_pages = int(nblk.sum())
    num_pages = used_pages + spec.spare_pages
    max_blocks = spec.max_blocks if spec.max_blocks > 0 else int(nblk.max())
    if max_blocks < int(nblk.max()):
        raise ValueError("max_blocks too small")

    # 2. page permutation
    if spec.shuffle_pages:
        perm = rng.permutation(num_pages).astype(np.int32)
    else:
        perm = np.arange(num_pages, dtype=np.int32)
    block_table = np.full((B, max_blocks), -1, dtype=np.int32)
    off = 0
    for b in range(B):
        block_table[b, :nblk[b]] = perm[off:off + nblk[b]]
        off += int(nblk[b])
    spare_ids = perm[off:]

    # 3. pools (bf16 bits; drawn from jumped streams of the same seed, in parallel)
    k_bits = normal_pool_bf16(seed, 0, (num_pages, PAGE, Hkv, D), std)
    v_bits = normal_pool_bf16(seed, 1, (num_pages, PAGE, Hkv, D), std)

    # 4. verify queries
    qv = rng.standard_normal((B, G, Hq, D), dtype=np.float32) * np.float32(std)

    # 5. directions
    u = _unit_rows(rng, (B, Hkv, D))
    if spec.drift > 0:
        v_old = _orthogonalise(_unit_rows(rng, (B, Hkv, D)), [u])
        v_new = _orthogonalise(_unit_rows(rng, (B, Hkv, D)), [u, v_old])
    else:
        v_old = v_new = None

    # 6. planted keys
    key_gain = np.float32(np.sqrt(D))     # a planted key a*sqrt(D)*u meets q = 1.0*u at scaled logit a
    sinks: List[np.ndarray] = []
    hit_v: List[np.ndarray] = []
    hit_d: List[np.ndarray] = []

    def plant(b: int, pos: np.ndarray, direction: np.ndarray, gain: float) -> None:
        if pos.size == 0:
            return
        pages = block_table[b, pos // PAGE]
        slots = pos % PAGE
        # direction: [Hkv, D]; the planted component is added to the (already rounded) base key
        base = bf16_bits_to_f32(k_bits[pages, slots])
        k_bits[pages, slots] = f32_to_bf16_bits(base + np.float32(gain) * key_gain * direction[None, :, :])

    for b in range(B):
        n = int(seq_lens[b])
        sink_pos = np.arange(min(spec.sink_tokens, max(n - G, 0)), dtype=np.int64)
        plant(b, sink_pos, u[b], spec.sink_gain)
        sinks.append(sink_pos)
        n_hit = spec.hitters if spec.hitters >= 0 else n // 256
        run = max(1, spec.hitter_run)
        lo, hi = spec.sink_tokens, n - G
        if n_hit > 0 and hi - lo >= 2 * n_hit + run:
            runs = max(1, n_hit // run)
            starts = _run_starts(rng, lo, hi, runs, run)
            pos = (starts[:, None] + np.arange(run)[None, :]).reshape(-1)
        else:
            pos = np.zeros(0, dtype=np.int64)
        if spec.drift > 0 and pos.size:
            n_drift = max(1, int(round(spec.drift * pos.size)))
            pick = rng.permutation(pos.size)[:n_drift]
            mask = np.zeros(pos.size, dtype=bool)
            mask[pick] = True
            plant(b, pos[~mask], u[b], spec.hitter_gain)
            plant(b, pos[mask], v_old[b], spec.hitter_gain)
            free = np.setdiff1d(np.arange(lo, hi, dtype=np.int64), pos, assume_unique=False)
            new_pos = np.sort(free[rng.permutation(free.size)[:n_drift]])
            plant(b, new_pos, v_new[b], spec.hitter_gain)
            hit_v.append(np.sort(pos))
            hit_d.append(np.sort(np.concatenate([pos[~mask], new_pos])))
        else:
            plant(b, pos, u[b], spec.hitter_gain)
            hit_v.append(np.sort(pos))
            hit_d.append(np.sort(pos))

    # queries carry the direction(s): head h of KV group h // g
    u_q = np.repeat(u, g, axis=1)                       # [B, Hq, D]
    q_base = qv.copy()
    qv += u_q[:, None, :, :]
    if spec.drift > 0:
        qv += np.repeat(v_old, g, axis=1)[:, None, :, :]

    # 7. draft queries = verify-query base + noise (+ the directions the draft phase aligns with)
    noise = rng.standard_normal((G, B, Hq, D), dtype=np.float32) * np.float32(spec.draft_noise * std)
    qd = np.transpose(q_base, (1, 0, 2, 3)) + noise + u_q[None, :, :, :]
    if spec.drift > 0:
        qd += np.repeat(v_new, g, axis=1)[None, :, :, :]

    # poison: spare pages and (optionally) the unused slots of partial last pages
    if spare_ids.size:
        k_bits[spare_ids] = BF16_NAN
        v_bits[spare_ids] = BF16_NAN
    if spec.poison_slack:
        for b in range(B):
            n = int(seq_lens[b])
            r = n % PAGE
            if r:
                last = block_table[b, nblk[b] - 1]
                k_bits[last, r:] = BF16_NAN
                v_bits[last, r:] = BF16_NAN

    return LayerInputs(
        spec=spec, layer=layer, seed=seed,
        q_verify=f32_to_bf16_bits(qv), q_draft=f32_to_bf16_bits(np.ascontiguousarray(qd)),
        k_cache=k_bits, v_cache=v_bits, block_table=block_table, seq_lens=seq_lens,
        softmax_scale=float(1.0 / np.sqrt(D)), sinks=sinks, hitters=hit_v, draft_hitters=hit_d,
    )


def make_random_case(seed: int, batch: int, num_q_heads: int, num_kv_heads: int, num_queries: int,
                     seq_lens, head_dim: int = 128, logit_std: float = 1.0, value_std: float = 1.0,
                     outliers: int = 0, outlier_logit: float = 30.0, shuffle: bool = True,
                     spare_pages: int = 3, poison: bool = True, max_blocks: int = 0) -> LayerInputs:
    """A "sharp" stress case: unit-scale tensors whose scaled logits have std ``logit_std``,
    optional keys with scaled logits near +-``outlier_logit``, shuffled pages, NaN poison in
    unreferenced pages and in the unused slots of partial last pages."""
    rng = np.random.Generator(np.random.PCG64(seed))
    B, Hq, Hkv, D, G = batch, num_q_heads, num_kv_heads, head_dim, num_queries
    seq_lens = np.asarray(seq_lens, dtype=np.int32).reshape(B)
    nblk = (seq_lens.astype(np.int64) + PAGE - 1) // PAGE
    num_pages = int(nblk.sum()) + spare_pages
    mb = max_blocks if max_blocks > 0 else max(1, int(nblk.max()))
    perm = rng.permutation(num_pages).astype(np.int32) if shuffle else np.arange(num_pages, dtype=np.int32)
    block_table = np.full((B, mb), -1, dtype=np.int32)
    off = 0
    for b in range(B):
        block_table[b, :nblk[b]] = perm[off:off + nblk[b]]
        off += int(nblk[b])
    spare_ids = perm[off:]
    # q ~ N(0,1), k ~ N(0, logit_std^2): scaled logit q.k/sqrt(D) has std logit_std
    k_pool = rng.standard_normal((num_pages, PAGE, Hkv, D), dtype=np.float32) * np.float32(logit_std)
    v_pool = rng.standard_normal((num_pages, PAGE, Hkv, D), dtype=np.float32) * np.float32(value_std)
    qv = rng.standard_normal((B, G, Hq, D), dtype=np.float32)
    hit: List[np.ndarray] = []
    if outliers > 0:
        u = _unit_rows(rng, (B, Hkv, D))
        qv += np.float32(np.sqrt(D)) * 0.25 * np.repeat(u, Hq // Hkv, axis=1)[:, None]
        for b in range(B):
            n = int(seq_lens[b])
            cnt = min(outliers, n)
            pos = np.sort(rng.permutation(n)[:cnt]).astype(np.int64)
            sign = np.where(rng.random(cnt) < 0.5, -1.0, 1.0).astype(np.float32)
            pages = block_table[b, pos // PAGE]
            # q.u = 0.25*sqrt(D); key = s*4*outlier*u -> scaled logit = s*outlier
            k_pool[pages, pos % PAGE] += (sign[:, None, None] * np.float32(4.0 * outlier_logit)) * u[b][None]
            hit.append(pos)
    else:
        hit = [np.zeros(0, dtype=np.int64) for _ in range(B)]
    noise = rng.standard_normal((G, B, Hq, D), dtype=np.float32) * np.float32(0.1)
    qd = np.transpose(qv, (1, 0, 2, 3)) + noise
    k_bits = f32_to_bf16_bits(k_pool)
    v_bits = f32_to_bf16_bits(v_pool)
    if poison:
        if spare_ids.size:
            k_bits[spare_ids] = BF16_NAN
            v_bits[spare_ids] = BF16_NAN
        for b in range(B):
            r = int(seq_lens[b]) % PAGE
            if r and nblk[b] > 0:
                last = block_table[b, nblk[b] - 1]
                k_bits[last, r:] = BF16_NAN
                v_bits[last, r:] = BF16_NAN
    spec = WorkloadSpec(f"random{seed}", 0, batch=B, num_q_heads=Hq, num_kv_heads=Hkv, gamma=G - 1,
                        budget_tokens=0, head_dim=D, max_blocks=mb)
    return LayerInputs(spec=spec, layer=0, seed=seed, q_verify=f32_to_bf16_bits(qv),
                       q_draft=f32_to_bf16_bits(np.ascontiguousarray(qd)), k_cache=k_bits, v_cache=v_bits,
                       block_table=block_table, seq_lens=seq_lens, softmax_scale=float(1.0 / np.sqrt(D)),
                       sinks=[np.zeros(0, dtype=np.int64)] * B, hitters=hit, draft_hitters=hit)
