"""Shared test helpers: packing hand-made K/V into a paged pool (no attention arithmetic)."""
import numpy as np

from paper_2604_23838_amd import workloads as W

PAGE = W.PAGE


def pack_paged(q, ks, vs, *, seed=0, slack=3, permute=True, poison=True):
    """q float [B,Hq,D]; ks, vs lists of float arrays [L_b,Hkv,D].  Values must be bf16-exact or are
    rounded to bf16.  Returns (q_bits, k_pages, v_pages, block_table, seq_lens) in library layouts."""
    q = np.asarray(q, dtype=np.float32)
    B, Hq, D = q.shape
    Hkv = ks[0].shape[1] if len(ks) else 1
    lens = np.array([k.shape[0] for k in ks], dtype=np.int32)
    npg = (lens + PAGE - 1) // PAGE
    NP = int(npg.sum()) + slack
    rng = np.random.default_rng(seed)
    perm = rng.permutation(NP) if permute else np.arange(NP)
    fill = W.BF16_NAN if poison else np.uint16(0)
    kp = np.full((NP, Hkv, PAGE, D), fill, dtype=np.uint16)
    vp = np.full((NP, Hkv, PAGE, D), fill, dtype=np.uint16)
    bt = np.full((B, max(1, int(npg.max()) if B else 1)), -1, dtype=np.int32)
    off = 0
    for b in range(B):
        kb = W.f32_to_bf16_bits(np.asarray(ks[b], dtype=np.float32))
        vb = W.f32_to_bf16_bits(np.asarray(vs[b], dtype=np.float32))
        for j in range(int(npg[b])):
            pg = int(perm[off])
            off += 1
            bt[b, j] = pg
            n = min(PAGE, int(lens[b]) - j * PAGE)
            kp[pg, :, :n, :] = kb[j * PAGE:j * PAGE + n].transpose(1, 0, 2)
            vp[pg, :, :n, :] = vb[j * PAGE:j * PAGE + n].transpose(1, 0, 2)
    return W.f32_to_bf16_bits(q), kp, vp, bt, lens


def gather_contiguous(w, b):
    """Float64 K, V [L, Hkv, D] of request b gathered through the block table (index work only)."""
    L = int(w.seq_lens[b])
    n = (L + PAGE - 1) // PAGE
    ids = w.block_table[b, :n]
    Hkv, D = w.k_pages.shape[1], w.k_pages.shape[3]
    k = W.bf16_bits_to_f64(w.k_pages[ids]).transpose(0, 2, 1, 3).reshape(n * PAGE, Hkv, D)[:L]
    v = W.bf16_bits_to_f64(w.v_pages[ids]).transpose(0, 2, 1, 3).reshape(n * PAGE, Hkv, D)[:L]
    return k, v


def error_report(got, ref, floor=1e-3):
    """max-abs and floored max-rel (|g-o| / max(|o|, floor)) between two float arrays."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    diff = np.abs(got - ref)
    return float(diff.max(initial=0.0)), float((diff / np.maximum(np.abs(ref), floor)).max(initial=0.0))


def prefill_inputs(w, q_lens, seed=0):
    """Packed queries for the last q_lens[b] tokens of every request of workload w."""
    rng = np.random.default_rng(seed)
    q_lens = np.asarray(q_lens, dtype=np.int32)
    offs = np.concatenate([[0], np.cumsum(q_lens)]).astype(np.int32)
    s = w.shape
    q = W.f32_to_bf16_bits(rng.standard_normal((int(offs[-1]) + 3, s.num_q_heads, s.head_dim), dtype=np.float32))
    return q, q_lens, offs
