"""Pins for the CPU oracle: closed forms, invariants, a library routine and a brute force.

The paper prints no numeric example of attention (it delegates rollout to an inference
engine), so there is no value of the paper's to store; what fixes the oracle is the
mathematics of softmax attention.  Each test below is chosen so that a plausible slip
(dropped scale, wrong head mapping, wrong page/slot index, mask off by one, transposed
operand, un-normalised weights) breaks at least one of them.
"""
import math

import numpy as np
import pytest

from paper_2604_23838_amd import workloads as W
from helpers import pack_paged, gather_contiguous

EXACT = 1e-12


def _ints(rng, shape, lo=-3, hi=3):
    return rng.integers(lo, hi, size=shape, endpoint=True).astype(np.float32)


def test_single_key_returns_v_exactly(jo):
    rng = np.random.default_rng(1)
    q = rng.standard_normal((3, 8, 64), dtype=np.float32)
    ks = [rng.standard_normal((1, 2, 64), dtype=np.float32) for _ in range(3)]
    vs = [rng.standard_normal((1, 2, 64), dtype=np.float32) for _ in range(3)]
    args = pack_paged(q, ks, vs)
    out = jo.decode_attention(*args)
    for b in range(3):
        vb = W.bf16_bits_to_f64(W.f32_to_bf16_bits(vs[b]))[0]
        for h in range(8):
            assert np.array_equal(out[b, h].astype(np.float64), vb[h // 4])


@pytest.mark.parametrize("L", [2, 16, 17, 31, 32, 33, 100])
def test_identical_keys_give_mean_of_v(jo, L):
    rng = np.random.default_rng(L)
    q = rng.standard_normal((1, 4, 64), dtype=np.float32)
    k1 = rng.standard_normal((1, 2, 64), dtype=np.float32)
    ks = [np.repeat(k1, L, axis=0)]
    vs = [_ints(rng, (L, 2, 64), -8, 8)]
    out, o64 = jo.decode_attention(*pack_paged(q, ks, vs), want64=True)
    mean = vs[0].astype(np.float64).mean(axis=0)
    for h in range(4):
        assert np.abs(o64[0, h] - mean[h // 2]).max() < EXACT


@pytest.mark.parametrize("L", [17, 31, 32, 33])
def test_zero_query_is_uniform_over_exactly_L_tokens(jo, L):
    # pins the masking of the last page: a mean over L-1 or L+1 slots differs by O(1/L)
    rng = np.random.default_rng(100 + L)
    q = np.zeros((1, 2, 128), dtype=np.float32)
    ks = [rng.standard_normal((L, 1, 128), dtype=np.float32)]
    vs = [_ints(rng, (L, 1, 128), -8, 8)]
    _, o64 = jo.decode_attention(*pack_paged(q, ks, vs), want64=True)
    assert np.abs(o64[0, 0] - vs[0].astype(np.float64).mean(axis=0)[0]).max() < EXACT


def test_page_permutation_invariance_bitwise(jo):
    rng = np.random.default_rng(3)
    lens = [17, 100, 250, 40]
    q = rng.standard_normal((4, 8, 64), dtype=np.float32)
    ks = [rng.standard_normal((L, 2, 64), dtype=np.float32) for L in lens]
    vs = [rng.standard_normal((L, 2, 64), dtype=np.float32) for L in lens]
    a = jo.decode_attention(*pack_paged(q, ks, vs, seed=0, permute=False))
    b = jo.decode_attention(*pack_paged(q, ks, vs, seed=1, permute=True))
    c = jo.decode_attention(*pack_paged(q, ks, vs, seed=2, permute=True, slack=11))
    assert np.array_equal(a.view(np.uint32), b.view(np.uint32))
    assert np.array_equal(a.view(np.uint32), c.view(np.uint32))


def test_weights_sum_to_one_and_reproduce_output(jo):
    w = W.gen_config(1, 0)
    args = (w.q, w.k_pages, w.v_pages, w.block_table, w.seq_lens)
    _, o64 = jo.decode_attention(*args, want64=True)
    for b in range(4):
        k, v = gather_contiguous(w, b)
        for h in (0, 3, 4, 7):
            wt = jo.softmax_weights(*args, b, h)
            assert wt.shape == (int(w.seq_lens[b]),)
            assert (wt > 0).all() and abs(wt.sum() - 1.0) < EXACT
            assert np.abs(wt @ v[:, h // 4, :] - o64[b, h]).max() < EXACT


def test_convex_hull_and_constant_v(jo):
    w = W.gen_config(1, 0)
    out = jo.decode_attention(w.q, w.k_pages, w.v_pages, w.block_table, w.seq_lens).astype(np.float64)
    for b in range(4):
        _, v = gather_contiguous(w, b)
        for h in range(8):
            assert (out[b, h] <= v[:, h // 4].max(axis=0) + 1e-7).all()
            assert (out[b, h] >= v[:, h // 4].min(axis=0) - 1e-7).all()
    rng = np.random.default_rng(5)
    q = rng.standard_normal((1, 4, 64), dtype=np.float32)
    ks = [rng.standard_normal((77, 2, 64), dtype=np.float32)]
    vs = [np.full((77, 2, 64), 1.5, dtype=np.float32)]
    vs[0][:, 1] = -0.25
    _, o64 = jo.decode_attention(*pack_paged(q, ks, vs), want64=True)
    assert np.abs(o64[0, :2] - 1.5).max() < EXACT and np.abs(o64[0, 2:] + 0.25).max() < EXACT


@pytest.mark.parametrize("D", [64, 128])
def test_two_keys_logistic_weight_and_default_scale(jo, D):
    # integer-valued bf16 q, k: the scores are exact, so w_0 = 1 / (1 + exp(-(s0 - s1))) with s = <q,k>/sqrt(D)
    rng = np.random.default_rng(D)
    q = _ints(rng, (1, 2, D))
    ks = [_ints(rng, (2, 1, D))]
    vs = [_ints(rng, (2, 1, D), -8, 8)]
    args = pack_paged(q, ks, vs)
    _, o64 = jo.decode_attention(*args, want64=True)
    for h in range(2):
        s = (q[0, h].astype(np.float64) * ks[0][:, 0].astype(np.float64)).sum(axis=1) / math.sqrt(D)
        w0 = 1.0 / (1.0 + math.exp(-(s[0] - s[1])))
        expect = w0 * vs[0][0, 0].astype(np.float64) + (1 - w0) * vs[0][1, 0].astype(np.float64)
        assert np.abs(o64[0, h] - expect).max() < EXACT
        wt = jo.softmax_weights(*args, 0, h)
        assert abs(wt[0] - w0) < EXACT
    # explicit scale overrides the default
    _, o_half = jo.decode_attention(*args, scale=0.5, want64=True)
    s = 0.5 * (q[0, 0].astype(np.float64) * ks[0][:, 0].astype(np.float64)).sum(axis=1)
    w0 = 1.0 / (1.0 + math.exp(-(s[0] - s[1])))
    expect = w0 * vs[0][0, 0].astype(np.float64) + (1 - w0) * vs[0][1, 0].astype(np.float64)
    assert np.abs(o_half[0, 0] - expect).max() < EXACT


def test_shift_invariance_of_keys(jo):
    rng = np.random.default_rng(6)
    L, D = 50, 64
    q = _ints(rng, (1, 4, D))
    k = _ints(rng, (L, 2, D))
    c = _ints(rng, (1, 2, D))
    v = rng.standard_normal((L, 2, D), dtype=np.float32)
    _, a = jo.decode_attention(*pack_paged(q, [k], [v]), want64=True)
    _, b = jo.decode_attention(*pack_paged(q, [k + c], [v]), want64=True)
    assert np.abs(a - b).max() < EXACT


def test_dominant_key_no_overflow(jo):
    D, L = 128, 40
    q = np.full((1, 1, D), 100.0, dtype=np.float32)
    k = np.zeros((L, 1, D), dtype=np.float32)
    k[7] = 100.0
    v = np.random.default_rng(7).standard_normal((L, 1, D), dtype=np.float32)
    out, o64 = jo.decode_attention(*pack_paged(q, [k], [v]), want64=True)
    assert np.isfinite(o64).all()
    assert np.array_equal(out[0, 0].astype(np.float64), W.bf16_bits_to_f64(W.f32_to_bf16_bits(v[7, 0])))


def test_gqa_structure(jo):
    rng = np.random.default_rng(8)
    L, D, Hq, Hkv = 60, 64, 14, 2     # G = 7, not a power of two
    G = Hq // Hkv
    q = rng.standard_normal((1, Hq, D), dtype=np.float32)
    q[0, 1] = q[0, 5]                  # same group (kv 0): equal queries -> equal outputs
    q[0, 8] = q[0, 1]                  # other group (kv 1): same query, different K/V -> different output
    k = rng.standard_normal((L, Hkv, D), dtype=np.float32)
    v = rng.standard_normal((L, Hkv, D), dtype=np.float32)
    _, a = jo.decode_attention(*pack_paged(q, [k], [v]), want64=True)
    assert np.array_equal(a[0, 1], a[0, 5]) and not np.allclose(a[0, 1], a[0, 8])
    # permuting the query heads inside a group permutes the output rows
    perm = np.arange(Hq)
    perm[:G] = perm[:G][::-1]
    _, b = jo.decode_attention(*pack_paged(q[:, perm], [k], [v]), want64=True)
    assert np.array_equal(b[0], a[0, perm])
    # changing kv head 1 leaves the heads of kv head 0 untouched and changes the others
    k2, v2 = k.copy(), v.copy()
    k2[:, 1] += 1.0
    v2[:, 1] -= 1.0
    _, c = jo.decode_attention(*pack_paged(q, [k2], [v2]), want64=True)
    assert np.array_equal(c[0, :G], a[0, :G]) and not np.allclose(c[0, G:], a[0, G:])


def test_split_and_merge_equals_whole(jo):
    w = W.gen_config(1, 0)
    args = (w.q, w.k_pages, w.v_pages, w.block_table, w.seq_lens)
    _, o64 = jo.decode_attention(*args, want64=True)
    rng = np.random.default_rng(9)
    for b, h in [(0, 0), (1, 5), (2, 2), (3, 7)]:
        L = int(w.seq_lens[b])
        toks = rng.permutation(L)
        cuts = np.sort(rng.integers(0, L, size=4, endpoint=True))
        pieces = np.split(toks, cuts)          # some pieces may be empty
        st = [jo.partial_state(*args, b, h, p) for p in pieces]
        merged = jo.merge_states([s[0] for s in st], [s[1] for s in st], np.stack([s[2] for s in st]))
        assert np.abs(merged - o64[b, h]).max() < EXACT
        # one piece holding everything: acc / l is the row itself
        m, l, acc = jo.partial_state(*args, b, h, np.arange(L))
        assert np.abs(acc / l - o64[b, h]).max() < EXACT
    # all-empty merge is the zero row
    assert np.array_equal(jo.merge_states([-np.inf], [0.0], np.zeros((1, 64))), np.zeros(64))


def test_matches_torch_sdpa_float64(jo):
    import torch
    w = W.gen_config(1, 0)
    _, o64 = jo.decode_attention(w.q, w.k_pages, w.v_pages, w.block_table, w.seq_lens, want64=True)
    qf = W.bf16_bits_to_f64(w.q)
    G = w.shape.num_q_heads // w.shape.num_kv_heads
    for b in range(4):
        k, v = gather_contiguous(w, b)
        kt = torch.from_numpy(k).permute(1, 0, 2).repeat_interleave(G, dim=0)   # [Hq, L, D]
        vt = torch.from_numpy(v).permute(1, 0, 2).repeat_interleave(G, dim=0)
        qt = torch.from_numpy(qf[b]).unsqueeze(1)                                # [Hq, 1, D]
        ref = torch.nn.functional.scaled_dot_product_attention(qt, kt, vt).squeeze(1).numpy()
        assert np.abs(ref - o64[b]).max() < EXACT


def test_matches_numpy_brute_force(jo):
    # separately written: explicit loops over requests, heads and tokens, no shared code with the C file
    w = W.gen_config(1, 0)
    _, o64 = jo.decode_attention(w.q, w.k_pages, w.v_pages, w.block_table, w.seq_lens, want64=True)
    s = w.shape
    G = s.num_q_heads // s.num_kv_heads
    for b in range(s.batch):
        L = int(w.seq_lens[b])
        for h in range(s.num_q_heads):
            qv = W.bf16_bits_to_f64(w.q[b, h])
            sc = np.empty(L)
            vals = np.empty((L, s.head_dim))
            for j in range(L):
                pg, slot = int(w.block_table[b, j // 16]), j % 16
                sc[j] = (qv * W.bf16_bits_to_f64(w.k_pages[pg, h // G, slot])).sum() / math.sqrt(s.head_dim)
                vals[j] = W.bf16_bits_to_f64(w.v_pages[pg, h // G, slot])
            e = np.exp(sc - sc.max())
            assert np.abs((e / e.sum()) @ vals - o64[b, h]).max() < EXACT


def test_poisoned_slots_never_influence(jo):
    a = W.gen_config(1, 0, poison=True)
    b = W.gen_config(1, 0, poison=False)
    assert np.isnan(W.bf16_bits_to_f64(a.k_pages)).any() and not np.isnan(W.bf16_bits_to_f64(b.k_pages)).any()
    oa = jo.decode_attention(a.q, a.k_pages, a.v_pages, a.block_table, a.seq_lens)
    ob = jo.decode_attention(b.q, b.k_pages, b.v_pages, b.block_table, b.seq_lens)
    assert np.isfinite(oa).all() and np.array_equal(oa.view(np.uint32), ob.view(np.uint32))


def test_empty_request_gives_zero_row_and_rows_subset(jo):
    rng = np.random.default_rng(11)
    q = rng.standard_normal((3, 4, 64), dtype=np.float32)
    lens = [5, 0, 33]
    ks = [rng.standard_normal((L, 2, 64), dtype=np.float32) for L in lens]
    vs = [rng.standard_normal((L, 2, 64), dtype=np.float32) for L in lens]
    args = pack_paged(q, ks, vs)
    out = jo.decode_attention(*args)
    assert np.array_equal(out[1], np.zeros((4, 64), dtype=np.float32)) and np.isfinite(out).all()
    rows = [(2, 3), (0, 0), (1, 2)]
    sub = jo.decode_attention(*args, rows=rows)
    for i, (b, h) in enumerate(rows):
        assert np.array_equal(sub[i], out[b, h])
    one = jo.decode_attention(*args, threads=1)
    assert np.array_equal(one, out)


def test_frozen_outputs_of_tiny_config(jo):
    # regression guard: values written by tests/golden/make_expected.py (oracle only)
    import os
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "cfg1_seed0_expected.txt")
    w = W.gen_config(1, 0)
    out = jo.decode_attention(w.q, w.k_pages, w.v_pages, w.block_table, w.seq_lens)
    n = 0
    for line in open(path):
        if line.startswith("#"):
            continue
        parts = line.split()
        b, h = int(parts[0]), int(parts[1])
        bits = np.array([int(x, 16) for x in parts[2:12]], dtype=np.uint32)
        got = np.concatenate([out[b, h, :8], out[b, h, -2:]]).view(np.uint32)
        assert np.array_equal(got, bits), (b, h)
        assert abs(float(out[b, h].astype(np.float64).sum()) - float(parts[12])) < 1e-12
        n += 1
    assert n == 32
