"""Pins for the oracle's causal prefill attention (CPU only)."""
import numpy as np
import pytest

from paper_2604_23838_amd import workloads as W
from helpers import gather_contiguous, pack_paged, prefill_inputs


def test_single_new_token_is_decode_attention(jo):
    w = W.gen_config(1, 0)
    q, ql, offs = prefill_inputs(w, [1, 1, 1, 1])
    out = jo.prefill_attention(q, w.k_pages, w.v_pages, w.block_table, w.seq_lens, ql, offs)
    dec = jo.decode_attention(q[:4], w.k_pages, w.v_pages, w.block_table, w.seq_lens)
    assert np.array_equal(out[:4].view(np.uint32), dec.view(np.uint32))
    assert np.array_equal(out[4:], np.zeros_like(out[4:]))      # rows no request owns stay zero


def test_matches_torch_sdpa_with_causal_mask_float64(jo):
    import torch
    w = W.gen_config(1, 1)
    ql = [17, 100, 33, 250]                      # request 1: full prefill; the others: a chunk after a context
    q, ql, offs = prefill_inputs(w, ql)
    _, o64 = jo.prefill_attention(q, w.k_pages, w.v_pages, w.block_table, w.seq_lens, ql, offs, want64=True)
    G = w.shape.num_q_heads // w.shape.num_kv_heads
    qf = W.bf16_bits_to_f64(q)
    for b in range(4):
        k, v = gather_contiguous(w, b)
        L, n = int(w.seq_lens[b]), int(ql[b])
        kt = torch.from_numpy(k).permute(1, 0, 2).repeat_interleave(G, dim=0)      # [Hq, L, D]
        vt = torch.from_numpy(v).permute(1, 0, 2).repeat_interleave(G, dim=0)
        qt = torch.from_numpy(qf[offs[b]:offs[b] + n]).permute(1, 0, 2)           # [Hq, n, D]
        pos = torch.arange(L - n, L).unsqueeze(1)                                   # absolute position of each query
        mask = torch.arange(L).unsqueeze(0) <= pos                                  # [n, L], True = attend
        ref = torch.nn.functional.scaled_dot_product_attention(qt, kt, vt, attn_mask=mask).permute(1, 0, 2).numpy()
        assert np.abs(ref - o64[offs[b]:offs[b] + n]).max() < 1e-12


def test_first_token_of_a_full_prefill_returns_v0_and_future_tokens_do_not_matter(jo):
    rng = np.random.default_rng(4)
    L = 70
    q = rng.standard_normal((L, 4, 64), dtype=np.float32)
    k = rng.standard_normal((L, 2, 64), dtype=np.float32)
    v = rng.standard_normal((L, 2, 64), dtype=np.float32)
    _, kp, vp, bt, lens = pack_paged(q[:1], [k], [v])
    qb = W.f32_to_bf16_bits(q)
    out = jo.prefill_attention(qb, kp, vp, bt, lens, [L], [0])
    v0 = W.bf16_bits_to_f64(W.f32_to_bf16_bits(v[0]))
    for h in range(4):
        assert np.array_equal(out[0, h].astype(np.float64), v0[h // 2])
    # causality: rewriting every key and value after position p leaves the outputs up to p untouched
    p = 40
    k2, v2 = k.copy(), v.copy()
    k2[p + 1:] = rng.standard_normal((L - p - 1, 2, 64), dtype=np.float32)
    v2[p + 1:] = 7.0
    _, kp2, vp2, bt2, _ = pack_paged(q[:1], [k2], [v2])
    out2 = jo.prefill_attention(qb, kp2, vp2, bt2, lens, [L], [0])
    assert np.array_equal(out[:p + 1].view(np.uint32), out2[:p + 1].view(np.uint32))
    assert not np.allclose(out[p + 1:], out2[p + 1:])


def test_chunked_prefill_equals_one_shot(jo):
    # the tokens of a request prefilled in two chunks (context 0 + 45, then 45 + 55) give the rows of one full pass
    w = W.build(W.SHAPES[1], [100], seed=9, cfg=120)
    rng = np.random.default_rng(1)
    q = W.f32_to_bf16_bits(rng.standard_normal((100, 8, 64), dtype=np.float32))
    full = jo.prefill_attention(q, w.k_pages, w.v_pages, w.block_table, [100], [100], [0])
    first = jo.prefill_attention(q[:45], w.k_pages, w.v_pages, w.block_table, [45], [45], [0])
    second = jo.prefill_attention(q[45:], w.k_pages, w.v_pages, w.block_table, [100], [55], [0])
    assert np.array_equal(full[:45].view(np.uint32), first.view(np.uint32))
    assert np.array_equal(full[45:].view(np.uint32), second.view(np.uint32))


def test_malformed_arguments_are_rejected(jo):
    w = W.gen_config(1, 0)
    q, ql, offs = prefill_inputs(w, [1, 1, 1, 1])
    with pytest.raises(ValueError):
        jo.prefill_attention(q, w.k_pages, w.v_pages, w.block_table, w.seq_lens, [18, 1, 1, 1], [0, 18, 19, 20])  # n > L
    with pytest.raises(ValueError):
        jo.prefill_attention(q, w.k_pages, w.v_pages, w.block_table, w.seq_lens, [2, 2, 0, 0], [0, 1, 4, 4])       # overlap
