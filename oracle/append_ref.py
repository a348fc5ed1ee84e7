"""Reference statement of the KV append (byte work).  TEST INFRASTRUCTURE ONLY.

One decode step first writes the new token's K and V rows into the paged cache and then attends over
the grown sequence (System Design, "Sub-Stage Graph Abstraction": each forward step processes the
active decoding requests; the KV cache holds their history).  Plain Python loops over requests and
heads, independent of the HIP code; operates on copies of the numpy arrays it is given.
"""
from __future__ import annotations

import numpy as np

PAGE = 16


def append_kv(k_new, v_new, k_pages, v_pages, block_table, seq_lens, active=None):
    """Returns (k_pages', v_pages', seq_lens') after appending row b of k_new / v_new ([B, Hkv, D] bf16 bit
    patterns) to every active request: slot L % 16 of page block_table[b][L // 16], then L -> L + 1.
    `active` None means every request with L > 0.  A request whose next slot lies beyond the block table or
    whose page id is outside the pool is left unchanged."""
    k_pages, v_pages, seq_lens = k_pages.copy(), v_pages.copy(), np.array(seq_lens, dtype=np.int32).copy()
    B, Hkv, D = k_new.shape
    NP, maxp = k_pages.shape[0], block_table.shape[1]
    for b in range(B):
        L = int(seq_lens[b])
        on = (L > 0) if active is None else bool(active[b])
        if not on or L < 0 or L // PAGE >= maxp:
            continue
        page = int(block_table[b, L // PAGE])
        if not 0 <= page < NP:
            continue
        for kv in range(Hkv):
            k_pages[page, kv, L % PAGE, :] = k_new[b, kv, :]
            v_pages[page, kv, L % PAGE, :] = v_new[b, kv, :]
        seq_lens[b] = L + 1
    return k_pages, v_pages, seq_lens
