"""Reference statement of the work partition (integer work).  TEST INFRASTRUCTURE ONLY.

The GPU library cuts one decode step's work into equal shares: the units
(request b, kv head, page), ordered request-major, then kv head, then page, form a
line of U = sum_b ceil(L_b / 16) * Hkv units; with `slots` waves and a minimum share
of `min_span` units, span = max(min_span, ceil(U / slots)), wave w < ceil(U / span)
owns units [w*span, min((w+1)*span, U)).  This is the intra-GPU counterpart of the
long-tail problem the paper describes for rollout (Motivation, "Varied Decoding
Lengths"): a few long sequences are spread over many waves, many short ones share a
wave.  Written as plain Python loops, independent of the HIP code.
"""
from __future__ import annotations

PAGE = 16


def pages(L: int, max_pages: int) -> int:
    n = (L + PAGE - 1) // PAGE if L > 0 else 0
    return min(n, max_pages)


def schedule(units: int, slots: int, min_span: int = 16):
    """(span, active_waves) for a work line of `units` page-units."""
    span = max(min_span, -(-units // slots))
    return span, -(-units // span)


def partition(seq_lens, num_kv_heads: int, slots: int, max_pages: int, min_span: int = 16):
    """Returns (header, wave_start, cum_pages) as the library reports them:
    header = [units, span, active_waves, slots];
    wave_start[w] = [request, kv head, page, 0] for w < active_waves."""
    n = [pages(int(L), max_pages) for L in seq_lens]
    cum = [0]
    for x in n:
        cum.append(cum[-1] + x)
    units = cum[-1] * num_kv_heads
    span = max(min_span, -(-units // slots))
    active = -(-units // span)
    # enumerate the line explicitly and read off where each wave starts
    starts = []
    line = ((b, kv, pg) for b in range(len(n)) for kv in range(num_kv_heads) for pg in range(n[b]))
    for u, (b, kv, pg) in enumerate(line):
        if u % span == 0:
            starts.append([b, kv, pg, 0])
    assert len(starts) == active
    return [units, span, active, slots], starts, cum


def segments(seq_lens, num_kv_heads: int, slots: int, max_pages: int, min_span: int = 16):
    """Every (wave, request, kv head, first page, end page) piece of the partition, by walking the line."""
    n = [pages(int(L), max_pages) for L in seq_lens]
    units = sum(n) * num_kv_heads
    span = max(min_span, -(-units // slots))
    out, u = [], 0
    for b in range(len(n)):
        for kv in range(num_kv_heads):
            pg = 0
            while pg < n[b]:
                w = u // span
                take = min(n[b] - pg, (w + 1) * span - u)
                out.append((w, b, kv, pg, pg + take))
                pg += take
                u += take
    return out
