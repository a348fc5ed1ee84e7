"""Host model of the work partition (integer work).  TEST INFRASTRUCTURE ONLY.

What fixes the partition is validity (every unit owned once, equal shares), which the GPU tests check on the
library's own tables without this module; the model below states one valid rule in plain loops and the CPU
suite checks that it has that property.

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


def partition(seq_lens, num_kv_heads: int, slots: int, max_pages: int, group_waves: int = 1, min_span: int = 16):
    """Returns (header, wave_start, cum_pages) as the library reports them:
    header = [units, span, active_groups, slots, group_waves];
    wave_start[w] = [request, kv head, page, 0] for the waves of the active groups.
    Waves work in groups of `group_waves`; member i of a group serves kv heads i, i + group_waves, ...;
    the line is made of group-units (request, kv-head group, page) and a group owns one span of it."""
    n = [pages(int(L), max_pages) for L in seq_lens]
    cum = [0]
    for x in n:
        cum.append(cum[-1] + x)
    hg = num_kv_heads // group_waves
    units = cum[-1] * hg
    span, active = schedule(units, slots // group_waves, min_span)
    # enumerate the line explicitly and read off where each group starts
    starts = []
    line = ((b, kvg, pg) for b in range(len(n)) for kvg in range(hg) for pg in range(n[b]))
    for u, (b, kvg, pg) in enumerate(line):
        if u % span == 0:
            for i in range(group_waves):
                starts.append([b, kvg * group_waves + i, pg, 0])
    assert len(starts) == active * group_waves
    return [units, span, active, slots, group_waves], starts, cum


def segments(seq_lens, num_kv_heads: int, slots: int, max_pages: int, group_waves: int = 1, min_span: int = 16):
    """Every (wave, request, kv head, first page, end page) piece of the partition, by walking the line."""
    n = [pages(int(L), max_pages) for L in seq_lens]
    hg = num_kv_heads // group_waves
    units = sum(n) * hg
    span, _ = schedule(units, slots // group_waves, min_span)
    out, u = [], 0
    for b in range(len(n)):
        for kvg in range(hg):
            pg = 0
            while pg < n[b]:
                g = u // span
                take = min(n[b] - pg, (g + 1) * span - u)
                for i in range(group_waves):
                    out.append((g * group_waves + i, b, kvg * group_waves + i, pg, pg + take))
                pg += take
                u += take
    return out
