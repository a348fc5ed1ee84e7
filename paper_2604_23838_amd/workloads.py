"""Seeded synthetic decode-attention workloads (input generation only).

This module builds the inputs of one rollout decode step: a batch of active
decoding requests with ragged, long-tailed sequence lengths and a paged KV
cache whose pages are scattered over a physical pool.  It holds none of the
attention arithmetic: it only draws lengths, a page permutation and N(0,1)
tensors rounded to bf16, so that the CPU oracle and the HIP library can be fed
the very same bits.

Why these shapes (paper, Motivation, "Varied Decoding Lengths"; Experimental
Setup): rollout batches are GRPO groups (global batch 64 x group 4 = 256
requests), response lengths are heavily skewed so that a few long sequences
dominate, multi-turn samples add 1..8 turns of context, and late in a step
only a handful of stragglers remain active.  The datasets and weights the
paper measures on are not used; lengths and tensors are synthetic stand-ins.

Layouts produced (all numpy, C-contiguous):
  q           uint16 [B, Hq, D]            bf16 bit patterns
  k_pages     uint16 [NP, Hkv, 16, D]      bf16 bit patterns
  v_pages     uint16 [NP, Hkv, 16, D]
  block_table int32  [B, MAXP]             physical page of logical page j; -1 where unused
  seq_lens    int32  [B]                   tokens per request, current token included
"""
from __future__ import annotations

import dataclasses
import math
from concurrent.futures import ThreadPoolExecutor

import numpy as np

PAGE = 16
BF16_NAN = np.uint16(0x7FC0)
SLACK_PAGES = 64  # pool pages no request owns; poisoned like every unused slot


@dataclasses.dataclass(frozen=True)
class Shape:
    name: str
    batch: int
    num_q_heads: int
    num_kv_heads: int
    head_dim: int
    layers: int  # layers of the model family the shape imitates (for derived per-model-step figures)


SHAPES = {
    1: Shape("tiny", 4, 8, 2, 64, 1),
    2: Shape("qwen3-8b-like-rollout", 256, 32, 8, 128, 36),
    3: Shape("straggler-phase", 8, 32, 8, 128, 36),
    4: Shape("qwen3-32b-like-agentic", 128, 64, 8, 128, 64),
    5: Shape("qwen2.5-0.5b-like-wide", 1024, 14, 2, 64, 24),
}


@dataclasses.dataclass
class Workload:
    cfg: int
    seed: int
    shape: Shape
    q: np.ndarray
    k_pages: np.ndarray
    v_pages: np.ndarray
    block_table: np.ndarray
    seq_lens: np.ndarray

    @property
    def total_tokens(self) -> int:
        return int(self.seq_lens.astype(np.int64).sum())

    @property
    def kv_bytes(self) -> int:
        """Bytes of K and V the step has to read: T x 2 x Hkv x D x 2."""
        s = self.shape
        return self.total_tokens * 2 * s.num_kv_heads * s.head_dim * 2

    @property
    def num_pages(self) -> int:
        return int(self.k_pages.shape[0])

    @property
    def max_pages_per_seq(self) -> int:
        return int(self.block_table.shape[1])


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even fp32 -> bf16, returned as uint16 bit patterns (finite inputs)."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32).copy()
    u += np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return (u >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f64(b: np.ndarray) -> np.ndarray:
    """Exact widening of bf16 bit patterns to float64."""
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)


def draw_seq_lens(cfg: int, rng: np.random.Generator) -> np.ndarray:
    """Sequence lengths of config `cfg` (first draw taken from `rng`)."""
    if cfg == 1:
        return np.array([17, 100, 250, 1000], dtype=np.int32)
    if cfg == 2:
        resp = np.floor(rng.lognormal(math.log(2048.0), 1.0, size=256))
        return (512 + np.minimum(resp, 16384)).astype(np.int32)
    if cfg == 3:
        return rng.integers(16384, 32768, size=8, endpoint=True).astype(np.int32)
    if cfg == 4:
        turns = rng.integers(1, 8, size=128, endpoint=True)
        lens = np.empty(128, dtype=np.int64)
        for i, t in enumerate(turns):
            lens[i] = int(np.floor(rng.lognormal(math.log(1024.0), 0.8, size=int(t))).sum())
        return np.clip(lens, 1, 32768).astype(np.int32)
    if cfg == 5:
        resp = np.floor(rng.lognormal(math.log(1024.0), 1.2, size=1024))
        return np.clip(resp, 1, 8192).astype(np.int32)
    raise ValueError(f"unknown config {cfg}")


def _normal_bf16_into(dst: np.ndarray, key: tuple, threads: int) -> None:
    """Fill flat uint16 `dst` with bf16(N(0,1)) drawn from counter-keyed child streams."""
    n = dst.size
    chunk = 1 << 22
    nchunks = (n + chunk - 1) // chunk

    def work(c: int) -> None:
        lo, hi = c * chunk, min(n, (c + 1) * chunk)
        g = np.random.default_rng([*key, c])
        dst[lo:hi] = f32_to_bf16_bits(g.standard_normal(hi - lo, dtype=np.float32))

    if nchunks <= 1 or threads <= 1:
        for c in range(nchunks):
            work(c)
    else:
        with ThreadPoolExecutor(max_workers=threads) as ex:
            list(ex.map(work, range(nchunks)))


def build(shape: Shape, seq_lens, seed: int = 0, *, cfg: int = 0, poison: bool = True,
          permute_pages: bool = True, threads: int = 8, rng: np.random.Generator | None = None) -> Workload:
    """Build a workload of arbitrary shape and lengths.

    Pages of all requests are dealt from a random permutation of the pool
    (NP = sum ceil(L/16) + SLACK_PAGES).  With `poison`, every slot no request
    reads (tail of a last page, slack pages) holds a bf16 NaN and unused block
    table entries are -1, so that any dependence on them shows up.
    """
    if rng is None:
        rng = np.random.default_rng(seed)
    seq_lens = np.asarray(seq_lens, dtype=np.int32)
    B, Hq, Hkv, D = len(seq_lens), shape.num_q_heads, shape.num_kv_heads, shape.head_dim
    npages = (seq_lens.astype(np.int64) + PAGE - 1) // PAGE
    used = int(npages.sum())
    NP = used + SLACK_PAGES
    maxp = max(1, int(npages.max()) if B else 1)
    perm = rng.permutation(NP) if permute_pages else np.arange(NP)
    block_table = np.full((B, maxp), -1, dtype=np.int32)
    off = 0
    for b in range(B):
        n = int(npages[b])
        block_table[b, :n] = perm[off:off + n]
        off += n

    q = f32_to_bf16_bits(rng.standard_normal((B, Hq, D), dtype=np.float32))
    k_pages = np.empty((NP, Hkv, PAGE, D), dtype=np.uint16)
    v_pages = np.empty((NP, Hkv, PAGE, D), dtype=np.uint16)
    _normal_bf16_into(k_pages.reshape(-1), (seed, cfg, 1), threads)
    _normal_bf16_into(v_pages.reshape(-1), (seed, cfg, 2), threads)

    if poison:
        k_pages[perm[used:]] = BF16_NAN
        v_pages[perm[used:]] = BF16_NAN
        for b in range(B):
            L = int(seq_lens[b])
            r = L % PAGE
            if L > 0 and r:
                last = int(block_table[b, (L - 1) // PAGE])
                k_pages[last, :, r:, :] = BF16_NAN
                v_pages[last, :, r:, :] = BF16_NAN
    return Workload(cfg, seed, dataclasses.replace(shape, batch=B), q, k_pages, v_pages, block_table, seq_lens)


def gen_config(cfg: int, seed: int = 0, *, threads: int = 8, poison: bool = True) -> Workload:
    """One of the five benchmark configurations.  Draw order: lengths, page permutation, q; K and V
    come from child streams keyed by (seed, cfg, tensor, chunk)."""
    rng = np.random.default_rng(seed)
    lens = draw_seq_lens(cfg, rng)
    return build(SHAPES[cfg], lens, seed, cfg=cfg, poison=poison, threads=threads, rng=rng)


def subset_requests(w: Workload, rows) -> Workload:
    """A workload holding only requests `rows` of `w`, with their pages compacted into a small pool.

    Used to time or check the CPU oracle on a bounded sample of a big workload
    without copying the whole pool.  The values every kept request reads are
    unchanged, so its outputs are those of the full workload.
    """
    rows = np.asarray(rows, dtype=np.int64)
    lens = w.seq_lens[rows]
    npages = (lens.astype(np.int64) + PAGE - 1) // PAGE
    maxp = max(1, int(npages.max()) if len(rows) else 1)
    bt = np.full((len(rows), maxp), -1, dtype=np.int32)
    ids = []
    off = 0
    for i, b in enumerate(rows):
        n = int(npages[i])
        ids.append(w.block_table[b, :n])
        bt[i, :n] = np.arange(off, off + n)
        off += n
    ids = np.concatenate(ids) if ids else np.zeros(0, dtype=np.int32)
    return Workload(w.cfg, w.seed, dataclasses.replace(w.shape, batch=len(rows)),
                    np.ascontiguousarray(w.q[rows]), np.ascontiguousarray(w.k_pages[ids]),
                    np.ascontiguousarray(w.v_pages[ids]), bt, np.ascontiguousarray(lens))
